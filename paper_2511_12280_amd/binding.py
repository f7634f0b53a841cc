"""ctypes binding of libd3tom.so (include/d3tom.h): argument marshalling only.

Every function here has the name of the C entry point it calls and does no arithmetic of the
method: it turns torch tensors into device pointers, passes sizes through and raises on a non-zero
status.  PyTorch supplies device memory and the current HIP stream, nothing else.  There is no
fallback: if the shared library is missing, importing this module fails.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libd3tom.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2511_12280_amd.build` "
                      "(hipcc, --offload-arch=gfx950); there is no CPU fallback")
_lib = ctypes.CDLL(LIB_PATH)

D3TOM_OK, D3TOM_ERR_INVALID_ARG, D3TOM_ERR_NO_DECIDERS, D3TOM_ERR_WORKSPACE_TOO_SMALL, \
    D3TOM_ERR_UNSUPPORTED, D3TOM_ERR_DEVICE = range(6)
D3TOM_F32, D3TOM_BF16 = 0, 1
D3TOM_MERGE_MEAN, D3TOM_MERGE_SUM = 0, 1
D3TOM_OP_IMPORTANCE, D3TOM_OP_SELECT_TOPK, D3TOM_OP_MERGE, D3TOM_OP_ATTEND = range(4)
D3TOM_MAX_VISUAL, D3TOM_MAX_DECIDERS = 16384, 256
D3TOM_IMPORTANCE_STATIC_BYTES = 16 << 20
D3TOM_LINEAR_PLAIN, D3TOM_LINEAR_RESIDUAL, D3TOM_LINEAR_SWIGLU = range(3)

EXPORTS = ["d3tom_keep_count", "d3tom_schedule", "d3tom_model_flops", "d3tom_workspace_bytes",
           "d3tom_status_string", "d3tom_importance", "d3tom_importance_static", "d3tom_select_topk", "d3tom_merge", "d3tom_merge_kv", "d3tom_merge_layer_workspace_bytes", "d3tom_merge_layer", "d3tom_attend", "d3tom_attend_weighted", "d3tom_update_deciders",
           "d3tom_rmsnorm", "d3tom_rope", "d3tom_linear", "d3tom_linear_tile", "d3tom_stack_workspace_bytes", "d3tom_stack_step", "d3tom_stack_batch_workspace_bytes", "d3tom_stack_step_batch",
           "d3tom_profile_enable", "d3tom_profile_kernel_count", "d3tom_profile_kernel_name", "d3tom_profile_collect"]

_vp, _i, _f, _d, _sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_double, ctypes.c_size_t
_lib.d3tom_keep_count.restype = _i
_lib.d3tom_keep_count.argtypes = [_i, _d]
_lib.d3tom_schedule.restype = _d
_lib.d3tom_schedule.argtypes = [_i, _i, _d, _d]
_lib.d3tom_model_flops.restype = _d
_lib.d3tom_model_flops.argtypes = [_d, _i, _i, _i, _i, _i, _i, _i, _i]
_lib.d3tom_workspace_bytes.restype = _sz
_lib.d3tom_workspace_bytes.argtypes = [_i] * 7
_lib.d3tom_status_string.restype = ctypes.c_char_p
_lib.d3tom_status_string.argtypes = [_i]
_lib.d3tom_importance.restype = _i
_lib.d3tom_importance.argtypes = [_vp, _vp, _i, _i, _vp, _i, _i, _f, _vp, _vp, _i, _i, _vp, _vp, _vp, _i, _i,
                                  _vp, _vp, _sz, _vp]
_lib.d3tom_importance_static.restype = _i
_lib.d3tom_importance_static.argtypes = [_vp, _vp, _i, _i, _vp, _i, _i, _f, _vp, _vp, _i, _i, _vp, _vp, _vp, _i, _i, _vp, _vp]
_lib.d3tom_select_topk.restype = _i
_lib.d3tom_select_topk.argtypes = [_vp, _i, _vp, _vp, _vp, _i, _vp, _vp, _vp, _sz, _vp]
_lib.d3tom_merge.restype = _i
_lib.d3tom_merge.argtypes = [_vp, _vp, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i,
                             _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.d3tom_merge_kv.restype = _i
_lib.d3tom_merge_kv.argtypes = [_vp, _vp, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i,
                                _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.d3tom_merge_layer_workspace_bytes.restype = _sz
_lib.d3tom_merge_layer_workspace_bytes.argtypes = [_i] * 6
_lib.d3tom_merge_layer.restype = _i
_lib.d3tom_merge_layer.argtypes = [_vp, _vp, _vp, _vp, _i, _i, _i, _i, _vp, _i, _i, _f, _vp, _vp, _i, _i, _vp, _vp, _vp,
                                   _vp, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.d3tom_update_deciders.restype = _i
_lib.d3tom_update_deciders.argtypes = [_vp, _vp, _i, _i, _vp, _i, _vp, _vp, _vp, _vp]
_lib.d3tom_attend.restype = _i
_lib.d3tom_attend.argtypes = [_vp, _vp, _vp, _i, _i, _vp, _i, _i, _i, _f, _vp, _vp, _sz, _vp]
_lib.d3tom_attend_weighted.restype = _i
_lib.d3tom_attend_weighted.argtypes = [_vp, _vp, _vp, _i, _i, _vp, _i, _i, _i, _f, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.d3tom_rmsnorm.restype = _i
_lib.d3tom_rmsnorm.argtypes = [_vp, _vp, _i, _i, _f, _vp, _vp]
_lib.d3tom_rope.restype = _i
_lib.d3tom_rope.argtypes = [_vp, _vp, _vp, _i, _i, _i, _f, _vp]
_lib.d3tom_linear.restype = _i
_lib.d3tom_linear.argtypes = [_vp, _vp, _i, _i, _i, _i, _vp, _vp, _i, _vp]
_lib.d3tom_linear_tile.restype = _i
_lib.d3tom_linear_tile.argtypes = [_vp, _vp, _i, _i, _i, _i, _vp, _vp, _i, _i, _vp]


class BlockWeights(ctypes.Structure):
    """d3tom_block_weights: device pointers of one block's parameters."""
    _fields_ = [(n, _vp) for n in ("attn_norm", "w_qkv", "w_o", "ffn_norm", "w_gate_up", "w_down")]


_lib.d3tom_stack_workspace_bytes.restype = _sz
_lib.d3tom_stack_workspace_bytes.argtypes = [_i] * 6
_lib.d3tom_stack_step.restype = _i
_lib.d3tom_stack_step.argtypes = [_vp, _i, _i, _i, _i, _i, ctypes.POINTER(BlockWeights), _i, _vp, _i, _i, _i, _i, _i,
                                  _f, _f, _vp, _vp, _vp, _vp, _vp, ctypes.POINTER(_i), _vp, _sz, _vp]

_i32p = ctypes.POINTER(ctypes.c_int32)
_lib.d3tom_stack_batch_workspace_bytes.restype = _sz
_lib.d3tom_stack_batch_workspace_bytes.argtypes = [_i] * 9
_lib.d3tom_stack_step_batch.restype = _i
_lib.d3tom_stack_step_batch.argtypes = [_vp, _i, _i32p, _i, _i, _i, _i, ctypes.POINTER(BlockWeights), _i, _vp, _i32p, _i32p, _i32p,
                                        _i32p, _i, _f, _f, _vp, _vp, _vp, _vp, _vp, ctypes.POINTER(_i), _vp, _sz, _vp]

_lib.d3tom_profile_enable.restype = _i
_lib.d3tom_profile_enable.argtypes = [_i]
_lib.d3tom_profile_kernel_count.restype = _i
_lib.d3tom_profile_kernel_name.restype = ctypes.c_char_p
_lib.d3tom_profile_kernel_name.argtypes = [_i]
_lib.d3tom_profile_collect.restype = _i
_lib.d3tom_profile_collect.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_longlong), _i]


class D3tomError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {d3tom_status_string(status)} (status {status})")


def _check(status: int, where: str):
    if status != D3TOM_OK:
        raise D3tomError(status, where)


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("device entry points take contiguous tensors on the GPU")
    return ctypes.c_void_p(t.data_ptr())


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return D3TOM_F32
    if t.dtype == torch.bfloat16:
        return D3TOM_BF16
    raise ValueError(f"unsupported element type {t.dtype}")


def _stream(stream) -> ctypes.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


# ---- host-only helpers ------------------------------------------------------------------------
def d3tom_keep_count(V: int, keep_ratio: float) -> int:
    return int(_lib.d3tom_keep_count(int(V), float(keep_ratio)))


def d3tom_schedule(step: int, T: int, r_first: float, r_last: float) -> float:
    return float(_lib.d3tom_schedule(int(step), int(T), float(r_first), float(r_last)))


def d3tom_model_flops(alpha: float, l_star: int, L: int, T: int, V: int, P: int, O: int, d: int, m: int) -> float:
    return float(_lib.d3tom_model_flops(float(alpha), l_star, L, T, V, P, O, d, m))


def d3tom_workspace_bytes(op: int, B: int, max_N: int, max_V: int, H: int, dh: int, max_D: int) -> int:
    return int(_lib.d3tom_workspace_bytes(op, B, max_N, max_V, H, dh, max_D))


def d3tom_status_string(status: int) -> str:
    return _lib.d3tom_status_string(int(status)).decode()


def d3tom_profile_enable(on: bool) -> None:
    _check(_lib.d3tom_profile_enable(1 if on else 0), "d3tom_profile_enable")


def d3tom_profile_kernel_count() -> int:
    return int(_lib.d3tom_profile_kernel_count())


def d3tom_profile_kernel_name(kernel: int) -> str:
    return _lib.d3tom_profile_kernel_name(int(kernel)).decode()


def d3tom_profile_collect() -> dict:
    """{kernel name: (total ms, launches)} since the last collect."""
    n = d3tom_profile_kernel_count()
    ms = (ctypes.c_double * n)()
    calls = (ctypes.c_longlong * n)()
    _check(_lib.d3tom_profile_collect(ms, calls, n), "d3tom_profile_collect")
    return {d3tom_profile_kernel_name(i): (float(ms[i]), int(calls[i])) for i in range(n)}


# ---- batch metadata (device int32 arrays + the host-known maxima the launches need) -------------
class Layout:
    """Per-sample token counts of one batch, resident on the device.

    N[b] tokens, visual block [vis_start[b], vis_start[b]+V[b]), decider positions dec[b] (relative
    to the sample), kept count keep[b].  Pure bookkeeping: offsets are prefix sums.
    """

    def __init__(self, N: Sequence[int], vis_start: Sequence[int], V: Sequence[int],
                 dec: Sequence[Sequence[int]], keep: Sequence[int], device="cuda"):
        B = len(N)
        assert len(vis_start) == B and len(V) == B and len(dec) == B and len(keep) == B
        self.B = B
        self.N, self.V, self.keep = [int(a) for a in N], [int(a) for a in V], [int(a) for a in keep]
        self.vis_start_h = [int(a) for a in vis_start]
        self.D = [len(a) for a in dec]
        self.Nm = [n - (v - k) for n, v, k in zip(self.N, self.V, self.keep)]
        self.max_N, self.max_V, self.max_keep = max(self.N), max(self.V), max(self.keep)
        self.min_D, self.max_D, self.max_Nm = min(self.D), max(self.D), max(self.Nm)
        self.max_pruned = max(v - k for v, k in zip(self.V, self.keep))
        self.sum_N, self.sum_V, self.sum_keep, self.sum_Nm = sum(self.N), sum(self.V), sum(self.keep), sum(self.Nm)

        def pre(a):
            return np.concatenate([[0], np.cumsum(a)]).astype(np.int32)

        def dev(a):
            return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(device)
        self.seq_off = dev(pre(self.N))
        self.vis_start = dev(self.vis_start_h)
        self.vis_count = dev(self.V)
        self.vis_off = dev(pre(self.V))             # also the offsets into `scores` / `assign`
        self.dec_off = dev(pre(self.D))
        flat = np.concatenate([np.asarray(a, dtype=np.int32) for a in dec]) if sum(self.D) else np.zeros(1, np.int32)
        self.dec_idx = dev(flat)
        self.keep_k = dev(self.keep)
        self.kept_off = dev(pre(self.keep))
        self.out_off = dev(pre(self.Nm))
        self.device = device


def workspace(nbytes: int, device="cuda") -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


# ---- device entry points ---------------------------------------------------------------------------
def d3tom_importance(q: torch.Tensor, k: torch.Tensor, lay: Layout, scale: float,
                     scores: torch.Tensor, ws: torch.Tensor, stream=None) -> torch.Tensor:
    """q, k [sum N, H, dh]; scores float32 [sum V] (written)."""
    H, dh = q.shape[-2], q.shape[-1]
    _check(_lib.d3tom_importance(_ptr(q), _ptr(k), _dt(q), lay.B, _ptr(lay.seq_off), H, dh, float(scale),
                                 _ptr(lay.dec_idx), _ptr(lay.dec_off), lay.min_D, lay.max_D,
                                 _ptr(lay.vis_start), _ptr(lay.vis_count), _ptr(lay.vis_off), lay.max_N, lay.max_V,
                                 _ptr(scores), _ptr(ws), ws.numel(), _stream(stream)), "d3tom_importance")
    return scores


def d3tom_importance_static(q: torch.Tensor, k: torch.Tensor, lay: Layout, scale: float,
                            scores: torch.Tensor, stream=None) -> torch.Tensor:
    """d3tom_importance without a workspace argument (the library's own static scratch array)."""
    H, dh = q.shape[-2], q.shape[-1]
    _check(_lib.d3tom_importance_static(_ptr(q), _ptr(k), _dt(q), lay.B, _ptr(lay.seq_off), H, dh, float(scale),
                                        _ptr(lay.dec_idx), _ptr(lay.dec_off), lay.min_D, lay.max_D,
                                        _ptr(lay.vis_start), _ptr(lay.vis_count), _ptr(lay.vis_off), lay.max_N, lay.max_V,
                                        _ptr(scores), _stream(stream)), "d3tom_importance_static")
    return scores


def d3tom_select_topk(scores: torch.Tensor, lay: Layout, kept_idx: torch.Tensor, slot_of: torch.Tensor,
                      ws: Optional[torch.Tensor] = None, stream=None):
    """scores float32 [sum V]; kept_idx int32 [sum keep], slot_of int32 [sum V] (written)."""
    _check(_lib.d3tom_select_topk(_ptr(scores), lay.B, _ptr(lay.vis_off), _ptr(lay.keep_k), _ptr(lay.kept_off),
                                  lay.max_V, _ptr(kept_idx), _ptr(slot_of), _ptr(ws), ws.numel() if ws is not None else 0,
                                  _stream(stream)), "d3tom_select_topk")
    return kept_idx, slot_of


def d3tom_merge(x: torch.Tensor, sim: Optional[torch.Tensor], lay: Layout, kept_idx: torch.Tensor, mode: int,
                y: torch.Tensor, assign: Optional[torch.Tensor], counts: Optional[torch.Tensor],
                src_pos: Optional[torch.Tensor], ws: torch.Tensor, stream=None):
    """x [sum N, d]; y [sum N_m, d] (written); assign int32 [sum V], counts int32 [sum keep],
    src_pos int32 [sum N_m] optional outputs."""
    d = x.shape[-1]
    d_sim = sim.shape[-1] if sim is not None else d
    _check(_lib.d3tom_merge(_ptr(x), _ptr(sim), d, d_sim, _dt(x), lay.B, _ptr(lay.seq_off), _ptr(lay.vis_start),
                            _ptr(lay.vis_count), _ptr(lay.vis_off), _ptr(kept_idx), _ptr(lay.kept_off),
                            lay.max_N, lay.max_V, lay.max_keep, lay.max_pruned, lay.max_Nm, int(mode), _ptr(lay.out_off), _ptr(y),
                            _ptr(assign), _ptr(counts), _ptr(src_pos), _ptr(ws), ws.numel(), _stream(stream)),
           "d3tom_merge")
    return y


def d3tom_merge_kv(k_cache: torch.Tensor, v_cache: torch.Tensor, lay: Layout, kept_idx: torch.Tensor, mode: int,
                   k_out: torch.Tensor, v_out: torch.Tensor, assign: Optional[torch.Tensor],
                   counts: Optional[torch.Tensor], src_pos: Optional[torch.Tensor], ws: torch.Tensor, stream=None):
    """k_cache, v_cache [sum N, d]; k_out, v_out [sum N_m, d] (written); index outputs as in d3tom_merge."""
    d = k_cache.shape[-1]
    _check(_lib.d3tom_merge_kv(_ptr(k_cache), _ptr(v_cache), d, _dt(k_cache), lay.B, _ptr(lay.seq_off),
                               _ptr(lay.vis_start), _ptr(lay.vis_count), _ptr(lay.vis_off), _ptr(kept_idx),
                               _ptr(lay.kept_off), lay.max_N, lay.max_V, lay.max_keep, lay.max_pruned, lay.max_Nm,
                               int(mode), _ptr(lay.out_off), _ptr(k_out), _ptr(v_out), _ptr(assign), _ptr(counts),
                               _ptr(src_pos), _ptr(ws), ws.numel(), _stream(stream)),
           "d3tom_merge_kv")
    return k_out, v_out


def d3tom_merge_layer_workspace_bytes(B: int, max_N: int, max_V: int, H: int, dh: int, max_D: int) -> int:
    return int(_lib.d3tom_merge_layer_workspace_bytes(B, max_N, max_V, H, dh, max_D))


def d3tom_merge_layer(q: torch.Tensor, k: torch.Tensor, x: torch.Tensor, sim: Optional[torch.Tensor], lay: Layout, scale: float,
                      keep_ratio: torch.Tensor, min_keep: int, max_keep: int, mode: int, scores: torch.Tensor,
                      keep_k: torch.Tensor, kept_off: torch.Tensor, kept_idx: torch.Tensor, out_off: torch.Tensor,
                      y: torch.Tensor, assign: Optional[torch.Tensor], counts: Optional[torch.Tensor],
                      src_pos: Optional[torch.Tensor], ws: torch.Tensor, stream=None):
    """The three merge-layer calls in one, kept counts from keep_ratio (float64 [B] on the device).  Only the sizes
    and decider lists of `lay` are used; its keep counts are not."""
    H, dh = q.shape[-2], q.shape[-1]
    d = x.shape[-1]
    d_sim = sim.shape[-1] if sim is not None else d
    assert keep_ratio.dtype == torch.float64 and keep_ratio.numel() == lay.B
    _check(_lib.d3tom_merge_layer(_ptr(q), _ptr(k), _ptr(x), _ptr(sim), d, d_sim, _dt(x), lay.B, _ptr(lay.seq_off), H, dh,
                                  float(scale), _ptr(lay.dec_idx), _ptr(lay.dec_off), lay.min_D, lay.max_D,
                                  _ptr(lay.vis_start), _ptr(lay.vis_count), _ptr(lay.vis_off), _ptr(keep_ratio),
                                  lay.max_N, lay.max_V, int(min_keep), int(max_keep), int(mode), _ptr(scores), _ptr(keep_k),
                                  _ptr(kept_off), _ptr(kept_idx), _ptr(out_off), _ptr(y), _ptr(assign), _ptr(counts),
                                  _ptr(src_pos), _ptr(ws), ws.numel(), _stream(stream)), "d3tom_merge_layer")
    return y


def d3tom_attend(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, cu_seqlens: torch.Tensor, max_seqlen: int,
                 scale: float, o: torch.Tensor, ws: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """q, k, v, o [sum n, H, dh]; cu_seqlens int32 [B+1] on the device."""
    H, dh = q.shape[-2], q.shape[-1]
    B = cu_seqlens.numel() - 1
    _check(_lib.d3tom_attend(_ptr(q), _ptr(k), _ptr(v), _dt(q), B, _ptr(cu_seqlens), int(max_seqlen), H, dh,
                             float(scale), _ptr(o), _ptr(ws), ws.numel() if ws is not None else 0, _stream(stream)),
           "d3tom_attend")
    return o


def d3tom_attend_weighted(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, cu_seqlens: torch.Tensor, max_seqlen: int,
                          scale: float, counts: torch.Tensor, kept_off: torch.Tensor, vis_start: torch.Tensor,
                          o: torch.Tensor, stream=None) -> torch.Tensor:
    """d3tom_attend with the merge's member counts as key weights (counts int32 [sum keep], kept_off int32 [B+1],
    vis_start int32 [B], all on the device)."""
    H, dh = q.shape[-2], q.shape[-1]
    B = cu_seqlens.numel() - 1
    _check(_lib.d3tom_attend_weighted(_ptr(q), _ptr(k), _ptr(v), _dt(q), B, _ptr(cu_seqlens), int(max_seqlen), H, dh,
                                      float(scale), _ptr(counts), _ptr(kept_off), _ptr(vis_start), _ptr(o), None, 0,
                                      _stream(stream)), "d3tom_attend_weighted")
    return o


def d3tom_update_deciders(prev_ids: torch.Tensor, cur_ids: torch.Tensor, mask_id: int, seq_off: torch.Tensor, max_D: int,
                          dec_idx: torch.Tensor, dec_off: torch.Tensor, dec_count: Optional[torch.Tensor] = None,
                          stream=None):
    """prev_ids, cur_ids int32 [sum N]; dec_idx int32 [B * max_D], dec_off int32 [B + 1], dec_count int32 [B] (written)."""
    Bn = seq_off.numel() - 1
    assert dec_idx.numel() >= Bn * max_D and dec_off.numel() >= Bn + 1
    _check(_lib.d3tom_update_deciders(_ptr(prev_ids), _ptr(cur_ids), int(mask_id), Bn, _ptr(seq_off), int(max_D),
                                      _ptr(dec_idx), _ptr(dec_off), _ptr(dec_count), _stream(stream)),
           "d3tom_update_deciders")
    return dec_idx, dec_off


# ---- tensor <-> numpy helpers for the storage types (bit moves only) ---------------------------------
def d3tom_rmsnorm(x: torch.Tensor, gain: torch.Tensor, eps: float, y: torch.Tensor, stream=None) -> None:
    rows, d = x.shape
    _check(_lib.d3tom_rmsnorm(_ptr(x), _ptr(gain), rows, d, eps, _ptr(y), _stream(stream)), "d3tom_rmsnorm")


def d3tom_rope(q: torch.Tensor, k: torch.Tensor, pos: torch.Tensor, theta: float, stream=None) -> None:
    rows, H, dh = q.shape
    assert k.shape == q.shape and pos.dtype == torch.int32 and pos.numel() >= rows
    _check(_lib.d3tom_rope(_ptr(q), _ptr(k), _ptr(pos), rows, H, dh, theta, _stream(stream)), "d3tom_rope")


def _linear_sizes(a, w, epilogue, out, residual):
    rows, K = a.shape
    n_w_rows, K2 = w.shape
    assert K2 == K and a.dtype == torch.bfloat16 and w.dtype == torch.bfloat16 and out.dtype == torch.bfloat16
    n_out = n_w_rows // 2 if epilogue == D3TOM_LINEAR_SWIGLU else n_w_rows
    assert out.numel() >= rows * n_out and (residual is None or residual.numel() >= rows * n_out)
    return rows, n_w_rows, K


def d3tom_linear(a: torch.Tensor, w: torch.Tensor, epilogue: int, out: torch.Tensor,
                 residual: Optional[torch.Tensor] = None, out_chunk: int = 0, stream=None) -> None:
    rows, n_w_rows, K = _linear_sizes(a, w, epilogue, out, residual)
    _check(_lib.d3tom_linear(_ptr(a), _ptr(w), rows, n_w_rows, K, epilogue, _ptr(residual), _ptr(out), out_chunk,
                             _stream(stream)), "d3tom_linear")


def d3tom_linear_tile(a: torch.Tensor, w: torch.Tensor, epilogue: int, out: torch.Tensor, tile: int,
                      residual: Optional[torch.Tensor] = None, out_chunk: int = 0, stream=None) -> None:
    rows, n_w_rows, K = _linear_sizes(a, w, epilogue, out, residual)
    _check(_lib.d3tom_linear_tile(_ptr(a), _ptr(w), rows, n_w_rows, K, epilogue, _ptr(residual), _ptr(out), out_chunk,
                                  tile, _stream(stream)), "d3tom_linear_tile")


def block_weights(blocks: Sequence[dict]):
    """Host array of d3tom_block_weights from dicts of device tensors (keys = field names).  The caller keeps
    the tensors alive."""
    arr = (BlockWeights * len(blocks))()
    for i, b in enumerate(blocks):
        for name, _ in BlockWeights._fields_:
            setattr(arr[i], name, b[name].data_ptr())
    return arr


def d3tom_stack_workspace_bytes(N: int, d: int, H: int, F: int, V: int, max_D: int) -> int:
    return int(_lib.d3tom_stack_workspace_bytes(N, d, H, F, V, max_D))


def d3tom_stack_step(x: torch.Tensor, H: int, F: int, blocks, L: int, merge_layer: int, dec_idx: Optional[torch.Tensor],
                     D: int, vis_start: int, V: int, keep_k: int, mode: int, eps: float, theta: float, y: torch.Tensor,
                     ws: torch.Tensor, src_pos: Optional[torch.Tensor] = None, scores: Optional[torch.Tensor] = None,
                     kept_idx: Optional[torch.Tensor] = None, assign: Optional[torch.Tensor] = None, stream=None) -> int:
    """Returns the number of output rows."""
    N, d = x.shape
    assert x.dtype == torch.bfloat16 and y.dtype == torch.bfloat16 and y.numel() >= N * d
    assert src_pos is None or (src_pos.dtype == torch.int32 and src_pos.numel() >= N)
    assert scores is None or (scores.dtype == torch.float32 and scores.numel() >= V)
    assert kept_idx is None or (kept_idx.dtype == torch.int32 and kept_idx.numel() >= keep_k)
    assert assign is None or (assign.dtype == torch.int32 and assign.numel() >= V)
    n_out = ctypes.c_int(0)
    _check(_lib.d3tom_stack_step(_ptr(x), N, d, H, F, L, blocks, merge_layer, _ptr(dec_idx), D, vis_start, V, keep_k,
                                 mode, eps, theta, _ptr(y), _ptr(src_pos), _ptr(scores), _ptr(kept_idx), _ptr(assign),
                                 ctypes.byref(n_out), _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)),
           "d3tom_stack_step")
    return n_out.value


def d3tom_stack_batch_workspace_bytes(B: int, sum_N: int, max_N: int, d: int, H: int, F: int, sum_V: int, max_V: int,
                                      max_D: int) -> int:
    return int(_lib.d3tom_stack_batch_workspace_bytes(B, sum_N, max_N, d, H, F, sum_V, max_V, max_D))


def d3tom_stack_step_batch(x: torch.Tensor, N: Sequence[int], H: int, F: int, blocks, L: int, merge_layer: int,
                           dec_idx: Optional[torch.Tensor], D: Sequence[int], vis_start: Sequence[int], V: Sequence[int],
                           keep_k: Sequence[int], mode: int, eps: float, theta: float, y: torch.Tensor, ws: torch.Tensor,
                           src_pos: Optional[torch.Tensor] = None, scores: Optional[torch.Tensor] = None,
                           kept_idx: Optional[torch.Tensor] = None, assign: Optional[torch.Tensor] = None, stream=None) -> List[int]:
    """Returns the number of output rows of every sample.  Per-sample sizes are host lists."""
    Bn = len(N)
    assert x.shape[0] == sum(N) and len(D) == Bn and len(vis_start) == Bn and len(V) == Bn and len(keep_k) == Bn
    d = x.shape[1]
    arr = lambda a: (ctypes.c_int32 * Bn)(*[int(v) for v in a])
    n_out = (ctypes.c_int * Bn)()
    _check(_lib.d3tom_stack_step_batch(_ptr(x), Bn, arr(N), d, H, F, L, blocks, merge_layer, _ptr(dec_idx), arr(D), arr(vis_start),
                                       arr(V), arr(keep_k), mode, eps, theta, _ptr(y), _ptr(src_pos), _ptr(scores), _ptr(kept_idx),
                                       _ptr(assign), n_out, _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)),
           "d3tom_stack_step_batch")
    return [int(v) for v in n_out]


def to_device(a: np.ndarray, dtype: str, device="cuda") -> torch.Tensor:
    """float32 numpy array whose values are representable in `dtype` -> device tensor of that type."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "f32":
        return torch.from_numpy(a).to(device)
    if dtype == "bf16":
        bits = (a.view(np.uint32) >> np.uint32(16)).astype(np.uint16)       # exact: low 16 bits are zero
        return torch.from_numpy(bits.view(np.int16)).to(device).view(torch.bfloat16).reshape(a.shape)
    raise ValueError(dtype)


def to_host(t: torch.Tensor) -> np.ndarray:
    """device tensor (float32 / bfloat16 / int32) -> numpy (bfloat16 widened exactly to float32)."""
    if t.dtype == torch.bfloat16:
        return t.float().cpu().numpy()
    return t.cpu().numpy()
