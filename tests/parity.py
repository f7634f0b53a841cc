"""Helpers of the GPU parity tests: run the HIP path through the C ABI, compare with the CPU oracle.

Tolerances (stated by the build's target): kept / assignment indices bit-exact except where a score
lies within 1e-3 relative of the k-th threshold or the chosen slot's cosine lies within 1e-3 relative
of the oracle's maximum; merged features within 2e-2 max-abs in bf16 (1e-4 in fp32); attention within
2e-2 max-abs in bf16 (1e-4 in fp32).  Importance scores themselves must agree to 1e-3 relative (the
threshold tolerance); float32 accumulation of exact bf16 products keeps them near 1e-5.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

import oracle
from paper_2511_12280_amd import binding as B

TOL_Y = {"bf16": 2e-2, "f32": 1e-4}
TOL_O = {"bf16": 2e-2, "f32": 1e-4}
TOL_S_REL = 1e-3
EXCUSE_REL = 1e-3


class GpuStep:
    """Device buffers + launches of one batch through the four entry points."""

    def __init__(self, samples: Sequence[dict], keeps: Sequence[int], dtype: str, mode: int = B.D3TOM_MERGE_MEAN):
        self.samples, self.keeps, self.dtype, self.mode = samples, list(keeps), dtype, mode
        s0 = samples[0]
        self.H, self.dh = s0["q"].shape[1], s0["q"].shape[2]
        self.d = s0["x"].shape[1]
        self.lay = B.Layout([s["N"] for s in samples], [s["vis_start"] for s in samples], [s["V"] for s in samples],
                            [s["dec_idx"] for s in samples], self.keeps)
        cat = lambda key: np.concatenate([s[key] for s in samples], axis=0)
        self.q = B.to_device(cat("q"), dtype)
        self.k = B.to_device(cat("k"), dtype)
        self.x = B.to_device(cat("x"), dtype)
        lay = self.lay
        tdt = torch.float32 if dtype == "f32" else torch.bfloat16
        self.scores = torch.zeros(lay.sum_V, dtype=torch.float32, device="cuda")
        self.kept_idx = torch.full((lay.sum_keep,), -7, dtype=torch.int32, device="cuda")
        self.slot_of = torch.full((lay.sum_V,), -7, dtype=torch.int32, device="cuda")
        self.y = torch.zeros((lay.sum_Nm, self.d), dtype=tdt, device="cuda")
        self.assign = torch.full((lay.sum_V,), -7, dtype=torch.int32, device="cuda")
        self.counts = torch.full((lay.sum_keep,), -7, dtype=torch.int32, device="cuda")
        self.src_pos = torch.full((lay.sum_Nm,), -7, dtype=torch.int32, device="cuda")
        self.ws_imp = B.workspace(B.d3tom_workspace_bytes(B.D3TOM_OP_IMPORTANCE, lay.B, lay.max_N, lay.max_V, self.H, self.dh, lay.max_D))
        self.ws_merge = B.workspace(B.d3tom_workspace_bytes(B.D3TOM_OP_MERGE, lay.B, lay.max_N, lay.max_V, self.H, self.dh, lay.max_D))
        self.scale = 1.0 / np.sqrt(self.dh)

    def importance(self):
        B.d3tom_importance(self.q, self.k, self.lay, self.scale, self.scores, self.ws_imp)
        torch.cuda.synchronize()
        return self.split(B.to_host(self.scores), self.lay.V)

    def select_topk(self, scores: Optional[List[np.ndarray]] = None):
        if scores is not None:
            self.scores.copy_(torch.from_numpy(np.concatenate(scores).astype(np.float32)))
        B.d3tom_select_topk(self.scores, self.lay, self.kept_idx, self.slot_of)
        torch.cuda.synchronize()
        return self.split(B.to_host(self.kept_idx), self.lay.keep), self.split(B.to_host(self.slot_of), self.lay.V)

    def merge(self, kept: Optional[List[np.ndarray]] = None, sim_rows: Optional[np.ndarray] = None):
        """`sim_rows` [sum N, d_sim]: separate features for the cosine (the payload stays `x`)."""
        if kept is not None:
            self.kept_idx.copy_(torch.from_numpy(np.concatenate(kept).astype(np.int32)))
        sim = B.to_device(sim_rows, self.dtype) if sim_rows is not None else None
        B.d3tom_merge(self.x, sim, self.lay, self.kept_idx, self.mode, self.y, self.assign, self.counts, self.src_pos,
                      self.ws_merge)
        torch.cuda.synchronize()
        lay = self.lay
        return dict(y=self.split(B.to_host(self.y), lay.Nm), assign=self.split(B.to_host(self.assign), lay.V),
                    counts=self.split(B.to_host(self.counts), lay.keep), src_pos=self.split(B.to_host(self.src_pos), lay.Nm))

    def merge_layer(self, ratios: Sequence[float], sim_rows: Optional[np.ndarray] = None):
        """The merge layer in one call (d3tom_merge_layer) at tight host bounds on the kept counts, into buffers of
        its own: (scores, kept, outputs of the merge) in the shape the separate calls return them."""
        lay = self.lay
        sim = B.to_device(sim_rows, self.dtype) if sim_rows is not None else None
        nb = lay.B
        i32 = lambda n: torch.full((n,), -7, dtype=torch.int32, device="cuda")
        scores = torch.zeros(lay.sum_V, dtype=torch.float32, device="cuda")
        keep_k, kept_off, out_off, kept_idx = i32(nb), i32(nb + 1), i32(nb + 1), i32(nb * lay.max_V)
        y = torch.zeros((lay.sum_N, self.d), dtype=self.y.dtype, device="cuda")
        assign, counts, src_pos = i32(lay.sum_V), i32(nb * lay.max_V), i32(lay.sum_N)
        ws = B.workspace(B.d3tom_merge_layer_workspace_bytes(nb, lay.max_N, lay.max_V, self.H, self.dh, lay.max_D))
        B.d3tom_merge_layer(self.q, self.k, self.x, sim, lay, self.scale, torch.tensor(list(ratios), dtype=torch.float64, device="cuda"),
                            min(lay.keep), max(lay.keep), self.mode, scores, keep_k, kept_off, kept_idx, out_off, y, assign,
                            counts, src_pos, ws)
        torch.cuda.synchronize()
        assert keep_k.cpu().tolist() == lay.keep
        return (self.split(B.to_host(scores), lay.V), self.split(B.to_host(kept_idx[:lay.sum_keep]), lay.keep),
                dict(y=self.split(B.to_host(y[:lay.sum_Nm]), lay.Nm), assign=self.split(B.to_host(assign), lay.V),
                     counts=self.split(B.to_host(counts[:lay.sum_keep]), lay.keep),
                     src_pos=self.split(B.to_host(src_pos[:lay.sum_Nm]), lay.Nm)))

    def merge_kv(self, v_cache_rows: np.ndarray, kept: Optional[List[np.ndarray]] = None):
        """KV-cache variant: the samples' `x` rows play the key cache, `v_cache_rows` [sum N, d] the value cache."""
        if kept is not None:
            self.kept_idx.copy_(torch.from_numpy(np.concatenate(kept).astype(np.int32)))
        vc = B.to_device(v_cache_rows, self.dtype)
        v_out = torch.zeros_like(self.y)
        B.d3tom_merge_kv(self.x, vc, self.lay, self.kept_idx, self.mode, self.y, v_out, self.assign, self.counts,
                         self.src_pos, self.ws_merge)
        torch.cuda.synchronize()
        lay = self.lay
        return dict(y=self.split(B.to_host(self.y), lay.Nm), v=self.split(B.to_host(v_out), lay.Nm),
                    assign=self.split(B.to_host(self.assign), lay.V), counts=self.split(B.to_host(self.counts), lay.keep),
                    src_pos=self.split(B.to_host(self.src_pos), lay.Nm))

    @staticmethod
    def split(a: np.ndarray, sizes: Sequence[int]) -> List[np.ndarray]:
        out, o = [], 0
        for n in sizes:
            out.append(a[o:o + n]); o += n
        return out


def gpu_attend(qkv_list: Sequence[tuple], dtype: str, scale: Optional[float] = None) -> List[np.ndarray]:
    """Variable-length batch of (q, k, v) numpy triples through d3tom_attend."""
    lens = [t[0].shape[0] for t in qkv_list]
    H, dh = qkv_list[0][0].shape[1:]
    q = B.to_device(np.concatenate([t[0] for t in qkv_list]), dtype)
    k = B.to_device(np.concatenate([t[1] for t in qkv_list]), dtype)
    v = B.to_device(np.concatenate([t[2] for t in qkv_list]), dtype)
    o = torch.zeros_like(q)
    cu = torch.from_numpy(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)).cuda()
    B.d3tom_attend(q, k, v, cu, max(lens), (1.0 / np.sqrt(dh)) if scale is None else scale, o)
    torch.cuda.synchronize()
    return GpuStep.split(B.to_host(o), lens)


def gpu_attend_weighted(qkv_list: Sequence[tuple], counts: Sequence[np.ndarray], vis_starts: Sequence[int], dtype: str,
                        scale: Optional[float] = None) -> List[np.ndarray]:
    """Variable-length batch through d3tom_attend_weighted: sample b's key rows vis_starts[b] .. + len(counts[b])
    carry the member counts counts[b], every other row weighs 1."""
    lens = [t[0].shape[0] for t in qkv_list]
    H, dh = qkv_list[0][0].shape[1:]
    q = B.to_device(np.concatenate([t[0] for t in qkv_list]), dtype)
    k = B.to_device(np.concatenate([t[1] for t in qkv_list]), dtype)
    v = B.to_device(np.concatenate([t[2] for t in qkv_list]), dtype)
    o = torch.zeros_like(q)
    i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()
    cu = i32(np.concatenate([[0], np.cumsum(lens)]))
    kept_off = i32(np.concatenate([[0], np.cumsum([len(c) for c in counts])]))
    B.d3tom_attend_weighted(q, k, v, cu, max(lens), (1.0 / np.sqrt(dh)) if scale is None else scale,
                            i32(np.concatenate(counts)), kept_off, i32(vis_starts), o)
    torch.cuda.synchronize()
    return GpuStep.split(B.to_host(o), lens)


def key_weights(n: int, vis_start: int, counts: np.ndarray) -> np.ndarray:
    """Per-key weights of a merged sequence of n rows: the member counts on the merged rows, 1 elsewhere."""
    w = np.ones(n, dtype=np.float64)
    w[vis_start:vis_start + len(counts)] = counts
    return w


# ---- comparisons ------------------------------------------------------------------------------------
def check_scores(S_gpu: np.ndarray, S_ref: np.ndarray):
    rel = np.abs(S_gpu.astype(np.float64) - S_ref) / np.maximum(np.abs(S_ref), 1e-300)
    assert rel.max() <= TOL_S_REL, f"importance relative error {rel.max():.3e}"
    return float(rel.max())


def check_kept(kept_gpu: np.ndarray, slot_gpu: np.ndarray, S_ref: np.ndarray, k: int):
    """Kept set vs the oracle's; differences only among scores within 1e-3 relative of the threshold."""
    kept_ref, slot_ref = oracle.select_topk(S_ref, k)
    assert len(kept_gpu) == k and np.all(np.diff(kept_gpu) > 0), "kept list must be ascending and of size k"
    V = len(S_ref)
    exp_slot = np.full(V, -1, np.int32); exp_slot[kept_gpu] = np.arange(k)
    np.testing.assert_array_equal(slot_gpu, exp_slot)
    diff = np.setxor1d(kept_gpu, kept_ref)
    if len(diff):
        thr = np.sort(S_ref)[::-1][k - 1]
        bad = [int(j) for j in diff if abs(S_ref[j] - thr) > EXCUSE_REL * abs(thr)]
        assert not bad, f"kept-set mismatch away from the threshold at {bad[:8]}"
    return len(diff) // 2


def check_assign(assign_gpu: np.ndarray, x: np.ndarray, vis_start: int, V: int, kept: np.ndarray,
                 only: Optional[np.ndarray] = None):
    """Assignment vs the oracle's; a different slot is excused iff its oracle cosine is within 1e-3
    relative of the oracle's maximum."""
    a_ref, bc = oracle.assign(x, vis_start, V, kept, return_cos=True, only=only)
    np.testing.assert_array_equal(assign_gpu[kept], np.arange(len(kept)))
    rows = np.arange(V) if only is None else np.asarray(only)
    assert np.all((assign_gpu >= 0) & (assign_gpu < len(kept)))
    excused = 0
    for m in rows:
        if a_ref[m] != assign_gpu[m]:
            c = oracle.cosine(x, vis_start + int(m), vis_start + int(kept[assign_gpu[m]]))
            assert c >= bc[m] - EXCUSE_REL * abs(bc[m]), f"token {m}: slot {assign_gpu[m]} (cos {c}) vs oracle {a_ref[m]} (cos {bc[m]})"
            excused += 1
    return excused


def check_merge(out: dict, x: np.ndarray, vis_start: int, V: int, kept: np.ndarray, dtype: str, mode: str = "mean"):
    """Merged rows / counts / positions vs the oracle run on the GPU's own assignment."""
    y_ref, counts_ref, src_ref = oracle.merge(x, vis_start, V, kept, out["assign"], mode)
    np.testing.assert_array_equal(out["counts"], counts_ref)
    np.testing.assert_array_equal(out["src_pos"], src_ref)
    y = out["y"].astype(np.float64)
    assert y.shape == y_ref.shape
    # One rounding to the storage type is half an ulp: 2^-9 |y| in bf16.  For O(1) values (MEAN mode,
    # |y| < 8) that is inside the 2e-2 bound; SUM rows grow with the member count, so the bound scales
    # with the magnitude there: max(2e-2, 2^-8 |y|) in bf16, max(1e-4, 2^-22 |y|) in fp32.
    rel = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -22
    excess = np.abs(y - y_ref) - np.maximum(TOL_Y[dtype], rel * np.abs(y_ref))
    err = np.abs(y - y_ref).max()
    assert excess.max() <= 0, f"merged features max abs error {err:.3e}"
    # rows that absorbed nothing, and all non-visual rows, are bit-exact copies
    k = len(kept)
    exact = np.ones(y.shape[0], bool)
    exact[vis_start:vis_start + k] = counts_ref == 1
    np.testing.assert_array_equal(y[exact], y_ref[exact])
    return float(err)


def check_attend(o_gpu: np.ndarray, q, k, v, dtype: str, rows=None, scale=None, key_weight=None):
    ref = oracle.attend(q, k, v, scale=scale, rows=rows, key_weight=key_weight)
    sel = slice(None) if rows is None else np.asarray(rows)
    err = np.abs(o_gpu.astype(np.float64)[sel] - ref[sel]).max()
    assert err <= TOL_O[dtype], f"attention max abs error {err:.3e}"
    return float(err)


def check_full_sample(step: GpuStep, b: int, S_gpu, kept_gpu, slot_gpu, mout, assign_rows=None, mode="mean"):
    """Chained check of sample b: every GPU stage against the oracle stage fed with the GPU's own
    (excused) upstream indices, so that a legitimate tie choice does not cascade."""
    s = step.samples[b]
    k = step.keeps[b]
    S_ref = oracle.importance(s["q"], s["k"], s["dec_idx"], s["vis_start"], s["V"])
    rel = check_scores(S_gpu[b], S_ref)
    nk = check_kept(kept_gpu[b], slot_gpu[b], S_ref, k)
    out = {key: mout[key][b] for key in mout}
    na = check_assign(out["assign"], s["x"], s["vis_start"], s["V"], kept_gpu[b], only=assign_rows)
    err = check_merge(out, s["x"], s["vis_start"], s["V"], kept_gpu[b], step.dtype, mode)
    return dict(score_rel=rel, kept_excused=nk, assign_excused=na, y_err=err)
