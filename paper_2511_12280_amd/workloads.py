"""Seeded synthetic workloads for the D3ToM merge layer and the attention after it.

This module only *draws inputs*: hidden states with the redundancy structure the
paper reports for visual tokens (many near-duplicates, a few tokens that attract
the decider tokens' attention), random projection weights, and the per-step
decider / mask layout of the response region.  It contains none of the method's
arithmetic (no importance map, no selection, no similarity, no merging, no
attention); both the HIP path and the CPU oracle consume what it produces, and
it imports neither of them.

Shapes follow the paper's cost-model constants (Appendix B, "Shared Notation":
hidden 4096, 32 layers, 64 prompt / 64 output tokens, about 10^3 visual tokens,
T = 32 steps) and the keep ratios of Table 2 (10 % .. 50 %).  The structure
(visual redundancy, sparse step-dependent saliency) follows Section 1 and the
saliency figures of the supplementary material.  These inputs stand in for the
LLaVA-Bench / LaViDa-LLaDA-8B setting the paper measures on.

Everything is generated on the host with numpy's PCG64 (`default_rng`), in
float32, and then rounded to the workload's storage type (float32 or bfloat16,
round-to-nearest-even), so that every consumer sees bit-identical values.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np


# ----------------------------------------------------------------------------
# storage-type helpers (pure bit manipulation)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit pattern (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bfloat16 bit pattern (uint16) -> float32 (exact)."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round a float32 array to `dtype` ("f32" or "bf16"); result is float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "f32":
        return a
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(a)).reshape(a.shape)
    raise ValueError(f"unknown dtype {dtype!r}")


# ----------------------------------------------------------------------------
# workload descriptions
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    """One benchmark configuration (token counts per sample)."""
    name: str
    dtype: str            # "f32" | "bf16": storage type of x, q, k, v
    B: int                # samples per batch
    d: int                # hidden size
    H: int                # attention heads
    dh: int               # head dimension (H * dh == d)
    P: int                # prompt tokens (before the visual block)
    V: int                # visual tokens
    O: int                # response slots (after the visual block)
    crops: int            # visual block = `crops` equal parts, each with own centres
    centres: int          # Gaussian cluster centres per crop
    seed: int
    salient: float        # >= 1: number of salient tokens; < 1: fraction of V
    noise: float = 0.3    # std of the per-token noise around its centre
    boost: float = 3.0    # key boost along the mean decider-query direction
    steps: int = 1        # denoising steps in the sweep
    note: str = ""

    @property
    def N(self) -> int:
        return self.P + self.V + self.O

    @property
    def n_salient(self) -> int:
        return int(self.salient) if self.salient >= 1 else int(round(self.salient * self.V))


WORKLOADS: Dict[str, Workload] = {
    # tiny single layer, fp32
    "tiny_f32": Workload("tiny_f32", "f32", 1, 256, 4, 64, 32, 144, 32, 1, 16, 0, 8,
                         note="16 deciders + 16 mask, keep 0.25"),
    # LLaDA-V-like single step
    "llada_v_1024": Workload("llada_v_1024", "bf16", 1, 4096, 32, 128, 64, 1024, 64, 1, 128, 1, 0.05,
                             note="32 deciders + 32 mask, keep 0.10"),
    # multi-crop LaViDa-like step sweep
    "lavida_3645_sweep": Workload("lavida_3645_sweep", "bf16", 1, 4096, 32, 128, 64, 3645, 64, 5, 256, 2, 0.05,
                                  steps=32, note="deciders 2..64, keep 0.10..0.50"),
    # batched serving shape
    "serving_b16": Workload("serving_b16", "bf16", 16, 4096, 32, 128, 128, 2304, 256, 1, 192, 3, 0.05,
                            note="per-sample deciders U[8,256], keep U[0.1,0.5]"),
}


def sweep_schedule(wl: Workload) -> List[dict]:
    """Per-step (decider count, keep ratio) of a workload's denoising sweep."""
    if wl.name == "lavida_3645_sweep":
        T = wl.steps
        return [dict(step=s, D=2 * (s + 1), keep_ratio=0.10 + 0.40 * s / (T - 1)) for s in range(T)]
    if wl.name == "llada_v_1024":
        return [dict(step=0, D=32, keep_ratio=0.10)]
    if wl.name == "tiny_f32":
        return [dict(step=0, D=16, keep_ratio=0.25)]
    raise ValueError(f"{wl.name} has no single-sample sweep")


def serving_draws(wl: Workload) -> List[dict]:
    """Per-sample (seed, decider count, keep ratio) of the batched serving workload."""
    rng = np.random.default_rng([wl.seed, 77])
    Ds = rng.integers(8, 257, size=wl.B)
    keeps = rng.uniform(0.1, 0.5, size=wl.B)
    return [dict(sample=b, seed=wl.seed * 1000 + b, D=int(Ds[b]), keep_ratio=float(keeps[b]))
            for b in range(wl.B)]


# ----------------------------------------------------------------------------
# generators
# ----------------------------------------------------------------------------
class Projections:
    """Random-init W_Q, W_K, W_V ~ N(0, 1/sqrt(d)) of one workload (shared by all samples)."""

    def __init__(self, wl: Workload):
        rng = np.random.default_rng([wl.seed, 11])
        std = 1.0 / math.sqrt(wl.d)
        self.wl = wl
        self.wq = rng.standard_normal((wl.d, wl.d), dtype=np.float32) * np.float32(std)
        self.wk = rng.standard_normal((wl.d, wl.d), dtype=np.float32) * np.float32(std)
        self.wv = rng.standard_normal((wl.d, wl.d), dtype=np.float32) * np.float32(std)

    def qkv(self, hidden: np.ndarray):
        """Project rows [n, d] (already in storage precision) to q, k, v [n, H, dh], rounded."""
        wl = self.wl
        h = np.ascontiguousarray(hidden, dtype=np.float32)
        out = []
        for w in (self.wq, self.wk, self.wv):
            out.append(round_to(h @ w, wl.dtype).reshape(h.shape[0], wl.H, wl.dh))
        return tuple(out)


class SampleGen:
    """All step-independent draws of one sample; `step(D)` lays out one denoising step."""

    def __init__(self, wl: Workload, proj: Optional[Projections] = None, seed: Optional[int] = None):
        self.wl = wl
        self.proj = proj if proj is not None else Projections(wl)
        seed = wl.seed if seed is None else seed
        rng = np.random.default_rng([seed, 23])
        d = wl.d
        # visual block: per crop, tokens = centre[picked] + noise
        per_crop = [wl.V // wl.crops + (1 if c < wl.V % wl.crops else 0) for c in range(wl.crops)]
        parts = []
        self.centre_of = []
        for c, n in enumerate(per_crop):
            cen = rng.standard_normal((wl.centres, d), dtype=np.float32)
            pick = rng.integers(0, wl.centres, size=n)
            parts.append(cen[pick] + np.float32(wl.noise) * rng.standard_normal((n, d), dtype=np.float32))
            self.centre_of.append(pick + c * wl.centres)
        self.centre_of = np.concatenate(self.centre_of).astype(np.int32)
        self.h_vis = round_to(np.concatenate(parts, axis=0), wl.dtype)
        self.h_prompt = round_to(rng.standard_normal((wl.P, d), dtype=np.float32), wl.dtype)
        self.h_decoded = round_to(rng.standard_normal((wl.O, d), dtype=np.float32), wl.dtype)
        self.h_mask = round_to(rng.standard_normal((1, d), dtype=np.float32), wl.dtype)
        self.salient_idx = np.sort(rng.choice(wl.V, size=wl.n_salient, replace=False)).astype(np.int32)
        # step-independent projections (float32, unrounded until the step is assembled)
        self._q_pv = np.concatenate([self.h_prompt, self.h_vis]) @ self.proj.wq
        self._k_pv = np.concatenate([self.h_prompt, self.h_vis]) @ self.proj.wk
        self._qkv_pv = None

    def step(self, D: int) -> dict:
        """One denoising step: response = D decoded (decider) tokens followed by O-D mask slots."""
        wl = self.wl
        if not (0 <= D <= wl.O):
            raise ValueError("decider count out of range")
        P, V, O, H, dh = wl.P, wl.V, wl.O, wl.H, wl.dh
        h_resp = np.concatenate([self.h_decoded[:D], np.repeat(self.h_mask, O - D, axis=0)], axis=0)
        x = np.concatenate([self.h_prompt, self.h_vis, h_resp], axis=0)
        q = np.concatenate([self._q_pv, h_resp @ self.proj.wq], axis=0).reshape(wl.N, H, dh).copy()
        k = np.concatenate([self._k_pv, h_resp @ self.proj.wk], axis=0).reshape(wl.N, H, dh).copy()
        dec_idx = np.arange(P + V, P + V + D, dtype=np.int32)
        if D > 0 and len(self.salient_idx) > 0:
            # boost the salient tokens' keys along the mean decider-query direction of each head
            u = q[dec_idx].mean(axis=0)                                   # [H, dh]
            u = u / np.maximum(np.linalg.norm(u, axis=1, keepdims=True), 1e-20)
            rows = P + self.salient_idx
            a = np.einsum("jhc,hc->jh", k[rows], u)                       # component along u
            k[rows] += ((wl.boost * np.abs(a) - a)[:, :, None] * u[None, :, :]).astype(np.float32)
        return dict(x=round_to(x, wl.dtype), q=round_to(q, wl.dtype), k=round_to(k, wl.dtype),
                    dec_idx=dec_idx, vis_start=P, V=V, N=wl.N, D=D,
                    salient_idx=self.salient_idx, centre_of=self.centre_of)

    def attention_inputs(self, n_tokens: int, D: int = 0):
        """q, k, v [n_tokens, H, dh] of a shortened sequence of the given length.

        Rows are prompt | the first n_tokens-P-O visual hidden states | response, projected
        with the workload's weights.  Used where the attention is measured or checked on its
        own; chained checks project the merged rows instead (see `Projections.qkv`).
        """
        wl = self.wl
        nv = n_tokens - wl.P - wl.O
        if nv < 0 or nv > wl.V:
            raise ValueError("n_tokens out of range")
        if self._qkv_pv is None:      # projections of prompt | all visual rows, computed once
            self._qkv_pv = self.proj.qkv(np.concatenate([self.h_prompt, self.h_vis], axis=0))
        h_resp = np.concatenate([self.h_decoded[:D], np.repeat(self.h_mask, wl.O - D, axis=0)], axis=0)
        resp = self.proj.qkv(h_resp)
        return tuple(np.concatenate([pv[:wl.P + nv], r], axis=0) for pv, r in zip(self._qkv_pv, resp))


def random_case(seed: int, N: int, d: int, H: int, P: int, V: int, D: int, dtype: str = "f32",
                centres: int = 8, noise: float = 0.3) -> dict:
    """Small unstructured case for parity/edge tests: arbitrary sizes, deciders anywhere outside
    the visual block (unsorted), clustered visual rows."""
    assert d % H == 0 and P + V <= N
    rng = np.random.default_rng([seed, 5])
    dh = d // H
    x = rng.standard_normal((N, d), dtype=np.float32)
    if V > 0:
        cen = rng.standard_normal((max(1, centres), d), dtype=np.float32)
        pick = rng.integers(0, max(1, centres), size=V)
        x[P:P + V] = cen[pick] + np.float32(noise) * rng.standard_normal((V, d), dtype=np.float32)
    q = rng.standard_normal((N, H, dh), dtype=np.float32)
    k = rng.standard_normal((N, H, dh), dtype=np.float32)
    outside = np.concatenate([np.arange(0, P), np.arange(P + V, N)])
    D = min(D, len(outside))
    dec_idx = rng.permutation(outside)[:D].astype(np.int32)
    return dict(x=round_to(x, dtype), q=round_to(q, dtype), k=round_to(k, dtype), dec_idx=dec_idx,
                vis_start=P, V=V, N=N, D=D)


def random_qkv(seed: int, n: int, H: int, dh: int, dtype: str = "f32", spread: float = 1.0):
    """Unstructured q, k, v [n, H, dh] ~ N(0, spread) for attention tests."""
    rng = np.random.default_rng([seed, 9])
    return tuple(round_to(np.float32(spread) * rng.standard_normal((n, H, dh), dtype=np.float32), dtype)
                 for _ in range(3))


def mask_trajectory(seed: int, n_prefix: int, n_response: int, steps: int, mask_id: int = 126336, vocab: int = 32000):
    """Token-id states of one sample over a denoising run: `steps + 1` int32 arrays of length
    n_prefix + n_response.  The prefix (visual + prompt positions) always holds ordinary ids; the response
    starts fully masked and a random subset of the still-masked positions is revealed at every step (all
    of them by the last one).  Which positions are revealed when is the only thing drawn here."""
    rng = np.random.default_rng(seed)
    ids = rng.integers(0, vocab, size=n_prefix + n_response).astype(np.int32)
    order = rng.permutation(n_response)
    cuts = np.sort(rng.choice(np.arange(1, n_response), size=min(steps - 1, n_response - 1), replace=False)) \
        if n_response > 1 and steps > 1 else np.array([], dtype=np.int64)
    bounds = np.concatenate([[0], cuts, [n_response]]).astype(np.int64)
    state = ids.copy()
    state[n_prefix:] = mask_id
    states = [state.copy()]
    for a, b in zip(bounds[:-1], bounds[1:]):
        pos = n_prefix + order[a:b]
        state[pos] = ids[pos]
        states.append(state.copy())
    return states



def stack_case(seed: int, L: int, d: int, H: int, F: int, P: int, V: int, O: int, D: int, std: float = 0.02,
               gain_jitter: float = 0.0, centres: int = 16, noise: float = 0.3) -> dict:
    """Inputs of one denoising step through a stack of L blocks, all rounded to bf16: random-init weights
    ~ N(0, std) stored as [out, in] rows, RMSNorm gains 1 (+ N(0, gain_jitter) so that a test can see them),
    hidden states of prompt | clustered visual tokens | response, of which D response positions hold decoded
    tokens (the deciders, ascending) and the others all share the one [MASK] embedding."""
    rng = np.random.default_rng([seed, 11])
    N = P + V + O

    def w(rows, cols):
        return round_to((std * rng.standard_normal((rows, cols))).astype(np.float32), "bf16")

    def g():
        return round_to((1.0 + gain_jitter * rng.standard_normal(d)).astype(np.float32), "bf16")

    blocks = [dict(attn_norm=g(), wq=w(d, d), wk=w(d, d), wv=w(d, d), wo=w(d, d), ffn_norm=g(),
                   w_gate=w(F, d), w_up=w(F, d), w_down=w(d, F)) for _ in range(L)]
    x = rng.standard_normal((N, d)).astype(np.float32)
    if V > 0:
        cen = rng.standard_normal((max(1, centres), d)).astype(np.float32)
        pick = rng.integers(0, max(1, centres), size=V)
        x[P:P + V] = cen[pick] + np.float32(noise) * rng.standard_normal((V, d)).astype(np.float32)
    D = min(D, O)
    dec_idx = np.sort(P + V + rng.permutation(O)[:D]).astype(np.int32)
    mask_vec = rng.standard_normal(d).astype(np.float32)
    is_mask = np.ones(N, dtype=bool)
    is_mask[:P + V] = False
    is_mask[dec_idx] = False
    x[is_mask] = mask_vec
    return dict(x=round_to(x, "bf16"), blocks=blocks, dec_idx=dec_idx, vis_start=P, V=V, N=N, D=D, H=H, d=d, F=F, L=L)


# ----------------------------------------------------------------------------
# full denoising-step stack (32 Llama-style blocks around the merge layer)
# ----------------------------------------------------------------------------
STACK_3645 = dict(name="denoise_stack_3645", L=32, d=4096, H=32, F=11008, P=64, V=3645, O=64, keep_ratio=0.10,
                  merge_layer=3, T=64, seed=4, std=0.02, eps=1e-5, theta=10000.0, centres=256, crops=5, noise=0.3,
                  mask_id=126336, table_rows=1024)


def stack_device_inputs(cfg: dict, device: str = "cuda") -> dict:
    """Inputs of the full-size stack, drawn on the device (6.5e9 weights are too many for the host
    generator): random-init N(0, std) projection weights, unit RMSNorm gains, hidden rows of prompt |
    clustered visual tokens (per crop: `centres` cluster centres + N(0, noise)) | response, an embedding
    table for revealed response tokens and the one [MASK] embedding.  bf16 throughout."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(cfg["seed"])
    d, F, L = cfg["d"], cfg["F"], cfg["L"]
    P, V, O = cfg["P"], cfg["V"], cfg["O"]

    def rnd(*shape, std=1.0):
        return (torch.randn(*shape, generator=g, device=device) * std).to(torch.bfloat16)

    ones = lambda: torch.ones(d, dtype=torch.bfloat16, device=device)
    blocks = [dict(attn_norm=ones(), w_qkv=rnd(3 * d, d, std=cfg["std"]), w_o=rnd(d, d, std=cfg["std"]), ffn_norm=ones(),
                   w_gate_up=rnd(2 * F, d, std=cfg["std"]), w_down=rnd(d, F, std=cfg["std"])) for _ in range(L)]
    x = rnd(P + V + O, d)
    per = V // cfg["crops"]
    for c in range(cfg["crops"]):
        lo = P + c * per
        hi = P + V if c == cfg["crops"] - 1 else lo + per
        cen = rnd(cfg["centres"], d).float()
        pick = torch.randint(0, cfg["centres"], (hi - lo,), generator=g, device=device)
        x[lo:hi] = (cen[pick] + cfg["noise"] * torch.randn(hi - lo, d, generator=g, device=device)).to(torch.bfloat16)
    return dict(blocks=blocks, x=x, table=rnd(cfg["table_rows"], d), mask_vec=rnd(d))
