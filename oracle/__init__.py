"""Python face of the CPU oracle (oracle/d3tom_oracle.c, fp64).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The HIP library and its binding never import it,
and it never imports them.

`build()` compiles the C file with gcc (-O2, OpenMP); `lib()` loads it, building
first if the shared object is missing.  The functions below marshal numpy
arrays; all arithmetic happens in the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "d3tom_oracle.c")
_SO = os.path.join(_HERE, "libd3tom_oracle.so")
_lib = None

_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)
_i32p = ctypes.POINTER(ctypes.c_int32)


def build(force: bool = True) -> str:
    """Compile the oracle.  Returns the path of the shared object."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        L = ctypes.CDLL(_SO)
        L.oracle_threads.restype = ctypes.c_int
        L.oracle_keep_count.restype = ctypes.c_int
        L.oracle_keep_count.argtypes = [ctypes.c_int, ctypes.c_double]
        L.oracle_deciders.restype = ctypes.c_int
        L.oracle_deciders.argtypes = [_i32p, _i32p, ctypes.c_int, ctypes.c_int, _i32p, ctypes.c_int]
        L.oracle_schedule.restype = ctypes.c_double
        L.oracle_schedule.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_double, ctypes.c_double]
        L.oracle_importance.argtypes = [_f32p, _f32p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                        _i32p, ctypes.c_int, ctypes.c_int, ctypes.c_int, _f64p, _f64p]
        L.oracle_select_topk.argtypes = [_f64p, ctypes.c_int, ctypes.c_int, _i32p, _i32p]
        L.oracle_assign.argtypes = [_f32p, ctypes.c_int, ctypes.c_int, ctypes.c_int, _i32p, ctypes.c_int,
                                    _i32p, _f64p, _i32p]
        L.oracle_cosine.restype = ctypes.c_double
        L.oracle_cosine.argtypes = [_f32p, ctypes.c_int, ctypes.c_int, ctypes.c_int]
        L.oracle_merge.argtypes = [_f32p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, _i32p,
                                   ctypes.c_int, _i32p, ctypes.c_int, _f64p, _i32p, _i32p]
        L.oracle_attend.argtypes = [_f32p, _f32p, _f32p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                    ctypes.c_double, _f64p, _f64p, _i32p, ctypes.c_int]
        for name, n in (("oracle_flops_layer", 3), ("oracle_flops_attn", 2), ("oracle_flops_ffn", 3),
                        ("oracle_flops_merge", 3)):
            f = getattr(L, name)
            f.restype = ctypes.c_double
            f.argtypes = [ctypes.c_double] * n
        L.oracle_flops_step.restype = ctypes.c_double
        L.oracle_flops_step.argtypes = [ctypes.c_double, ctypes.c_int, ctypes.c_int] + [ctypes.c_double] * 5
        L.oracle_flops_total.restype = ctypes.c_double
        L.oracle_flops_total.argtypes = [ctypes.c_double, ctypes.c_int, ctypes.c_int, ctypes.c_int] + \
                                        [ctypes.c_double] * 5
        _lib = L
    return _lib


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a, t):
    return a.ctypes.data_as(t)


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"oracle {what}: invalid arguments (code {rc})")


def threads() -> int:
    return int(lib().oracle_threads())


def keep_count(V: int, keep_ratio: float) -> int:
    return int(lib().oracle_keep_count(int(V), float(keep_ratio)))


def schedule(step: int, T: int, r_first: float, r_last: float) -> float:
    return float(lib().oracle_schedule(int(step), int(T), float(r_first), float(r_last)))


def deciders(prev_ids, cur_ids, mask_id: int) -> np.ndarray:
    """Ascending positions that hold a token now and held [MASK] one iteration earlier."""
    p = _i32(prev_ids); c = _i32(cur_ids)
    assert p.shape == c.shape and p.ndim == 1
    out = np.zeros(max(len(p), 1), dtype=np.int32)
    n = lib().oracle_deciders(_p(p, _i32p), _p(c, _i32p), len(p), int(mask_id), _p(out, _i32p), len(out))
    return out[:n].copy()


def importance(q, k, dec_idx, vis_start: int, V: int, scale: Optional[float] = None,
               return_all: bool = False):
    """S[V] (float64); with return_all also the score of every key position, [N]."""
    q = _f32(q); k = _f32(k); dec = _i32(dec_idx)
    N, H, dh = q.shape
    assert k.shape == q.shape
    scale = 1.0 / np.sqrt(dh) if scale is None else scale
    S = np.zeros(V, dtype=np.float64)
    S_all = np.zeros(N, dtype=np.float64)
    _check(lib().oracle_importance(_p(q, _f32p), _p(k, _f32p), N, H, dh, float(scale), _p(dec, _i32p), len(dec),
                                   int(vis_start), int(V), _p(S, _f64p), _p(S_all, _f64p)), "importance")
    return (S, S_all) if return_all else S


def select_topk(S, keep_k: int) -> Tuple[np.ndarray, np.ndarray]:
    """(kept_idx ascending [keep_k], slot_of [V]) for scores S (any float type, widened exactly)."""
    S = np.ascontiguousarray(S, dtype=np.float64)
    V = S.shape[0]
    kept = np.zeros(keep_k, dtype=np.int32)
    slot = np.zeros(V, dtype=np.int32)
    _check(lib().oracle_select_topk(_p(S, _f64p), V, int(keep_k), _p(kept, _i32p), _p(slot, _i32p)), "select_topk")
    return kept, slot


def assign(f, vis_start: int, V: int, kept_idx, return_cos: bool = False, only=None):
    """assign[V]: slot of every visual token (cosine argmax for pruned ones).

    `only`: optional list of visual indices; pruned tokens outside it are skipped (assign = -1)."""
    f = _f32(f); kept = _i32(kept_idx)
    d = f.shape[1]
    a = np.zeros(V, dtype=np.int32)
    bc = np.zeros(V, dtype=np.float64)
    mask = None
    if only is not None:
        mask = np.zeros(V, dtype=np.int32)
        mask[np.asarray(only, dtype=np.int64)] = 1
    _check(lib().oracle_assign(_p(f, _f32p), d, int(vis_start), int(V), _p(kept, _i32p), len(kept),
                               _p(a, _i32p), _p(bc, _f64p), _p(mask, _i32p) if mask is not None else None), "assign")
    return (a, bc) if return_cos else a


def cosine(f, row_a: int, row_b: int) -> float:
    f = _f32(f)
    return float(lib().oracle_cosine(_p(f, _f32p), f.shape[1], int(row_a), int(row_b)))


def merge(x, vis_start: int, V: int, kept_idx, assign_, mode: str = "mean"):
    """(y [N_m, d] float64, counts [k], src_pos [N_m])."""
    x = _f32(x); kept = _i32(kept_idx); a = _i32(assign_)
    N, d = x.shape
    k = len(kept)
    N_m = N - (V - k)
    y = np.zeros((N_m, d), dtype=np.float64)
    counts = np.zeros(k, dtype=np.int32)
    src = np.zeros(N_m, dtype=np.int32)
    _check(lib().oracle_merge(_p(x, _f32p), N, d, int(vis_start), int(V), _p(kept, _i32p), k, _p(a, _i32p),
                              {"mean": 0, "sum": 1}[mode], _p(y, _f64p), _p(counts, _i32p), _p(src, _i32p)),
           "merge")
    return y, counts, src


def attend(q, k, v, scale: Optional[float] = None, rows=None, key_weight=None) -> np.ndarray:
    """out [n, H, dh] float64, no mask.  `rows`: optional query rows to evaluate (others stay 0);
    `key_weight` [n]: optional positive per-key weights (softmax of logit + log weight)."""
    q = _f32(q); k = _f32(k); v = _f32(v)
    n, H, dh = q.shape
    assert k.shape == q.shape and v.shape == q.shape
    scale = 1.0 / np.sqrt(dh) if scale is None else scale
    out = np.zeros((n, H, dh), dtype=np.float64)
    r = _i32(rows) if rows is not None else None
    w = np.ascontiguousarray(key_weight, dtype=np.float64) if key_weight is not None else None
    assert w is None or w.shape == (n,)
    _check(lib().oracle_attend(_p(q, _f32p), _p(k, _f32p), _p(v, _f32p), n, H, dh, float(scale),
                               _p(w, _f64p) if w is not None else None, _p(out, _f64p),
                               _p(r, _i32p) if r is not None else None, len(r) if r is not None else 0), "attend")
    return out


def merge_layer(q, k, x, dec_idx, vis_start: int, V: int, keep_k: int, mode: str = "mean",
                sim=None, scale: Optional[float] = None) -> dict:
    """The four merge stages in the order of Algorithm 1 (importance, top-k, assignment, aggregation)."""
    S = importance(q, k, dec_idx, vis_start, V, scale)
    kept, slot_of = select_topk(S, keep_k)
    a, bc = assign(x if sim is None else sim, vis_start, V, kept, return_cos=True)
    y, counts, src = merge(x, vis_start, V, kept, a, mode)
    return dict(S=S, kept_idx=kept, slot_of=slot_of, assign=a, best_cos=bc, y=y, counts=counts, src_pos=src)


def merge_kv(k_cache, v_cache, vis_start: int, V: int, kept_idx, mode: str = "mean") -> dict:
    """KV-cache variant (Section 4.4): routing pi(m) from the cosine of the cached key rows, then the
    same aggregation applied to the key cache and to the value cache, merged positions dropped."""
    a, bc = assign(k_cache, vis_start, V, kept_idx, return_cos=True)
    yk, counts, src = merge(k_cache, vis_start, V, kept_idx, a, mode)
    yv, counts_v, src_v = merge(v_cache, vis_start, V, kept_idx, a, mode)
    assert np.array_equal(counts, counts_v) and np.array_equal(src, src_v)
    return dict(assign=a, best_cos=bc, k=yk, v=yv, counts=counts, src_pos=src)


# cost model (Section 4.3 / Appendix B)
def flops_layer(n, d, m): return float(lib().oracle_flops_layer(n, d, m))
def flops_merge(alpha, V, d): return float(lib().oracle_flops_merge(alpha, V, d))
def flops_step(alpha, l_star, L, V, P, O, d, m): return float(lib().oracle_flops_step(alpha, l_star, L, V, P, O, d, m))
def flops_total(alpha, l_star, L, T, V, P, O, d, m):
    return float(lib().oracle_flops_total(alpha, l_star, L, T, V, P, O, d, m))
