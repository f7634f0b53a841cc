"""fp64 oracle of one denoising step through a stack of Llama-style blocks with the merge layer inside
(Algorithm 1, the loop over layers; Section 3.2 for where the merge sits).

TEST INFRASTRUCTURE ONLY, like the rest of this package: tests, the smoke check and the benchmark's CPU
leg may import it; the HIP library and its binding never do.

Each function is the textbook definition written with numpy in float64.  The merge layer itself
(importance, top-k, assignment, aggregation) is the C oracle of this package; nothing here is shared
with the HIP path.

Storage type.  The workload is a bf16 model: every tensor that a layer hands to the next one is stored
in bf16.  `store="bf16"` rounds (to nearest, ties to even) at exactly those hand-over points and nowhere
else; `store=None` keeps float64 throughout (then the inputs of the C merge oracle, which reads
float32, are the only values that get rounded, to float32).  The hand-over points are:
  normalised rows, q / k / v, rotated q / k, attention output, post-attention hidden state,
  merged rows, SwiGLU activation, block output.
A sum with the residual stream is formed before the rounding (one rounding per stored tensor).

Pins: tests/test_stack_oracle_pins.py.
"""
from __future__ import annotations

from typing import Callable, List, Optional, Sequence

import numpy as np

from . import assign as _assign
from . import importance as _importance
from . import merge as _merge
from . import select_topk as _select_topk


def round_bf16(a) -> np.ndarray:
    """Nearest bf16 value (8 significant bits, ties to even) of every float64 entry, returned as float64.

    Written on the mantissa/exponent split so that it rounds once, straight from float64.  Values in
    the subnormal range of bf16 are not special-cased (the workloads stay far away from 1e-38)."""
    a = np.asarray(a, dtype=np.float64)
    m, e = np.frexp(a)                       # a = m * 2**e, 0.5 <= |m| < 1
    return np.ldexp(np.rint(m * 256.0), e - 8)   # rint: ties to even


def _store_fn(store) -> Callable[[np.ndarray], np.ndarray]:
    """The function applied to every tensor at a hand-over point: identity in float64 (None), rounding to
    bf16 ("bf16"), or a caller's own function of one array."""
    if store is None:
        return lambda a: np.asarray(a, dtype=np.float64)
    if store == "bf16":
        return round_bf16
    if callable(store):
        return store
    raise ValueError("store must be None, 'bf16' or a function")


def rmsnorm(x, gain, eps: float) -> np.ndarray:
    """Row-wise x / sqrt(mean(x^2) + eps) * gain."""
    x = np.asarray(x, dtype=np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(gain, dtype=np.float64)


def rope(x, pos, theta: float) -> np.ndarray:
    """Rotary position embedding on x [n, H, dh]: channel c < dh/2 is paired with channel c + dh/2 and the
    pair is rotated by the angle pos * theta**(-2c/dh)."""
    x = np.asarray(x, dtype=np.float64)
    n, H, dh = x.shape
    half = dh // 2
    c = np.arange(half, dtype=np.float64)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * theta ** (-2.0 * c / dh)[None, :]      # [n, half]
    co, si = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * co - b * si, b * co + a * si], axis=-1)


def linear(a, w) -> np.ndarray:
    """a [m, K] times the transpose of w [n, K] (weights stored as rows of output features)."""
    return np.asarray(a, dtype=np.float64) @ np.asarray(w, dtype=np.float64).T


def swiglu(gate, up) -> np.ndarray:
    gate = np.asarray(gate, dtype=np.float64)
    return gate / (1.0 + np.exp(-gate)) * np.asarray(up, dtype=np.float64)


def attention(q, k, v, scale: Optional[float] = None) -> np.ndarray:
    """softmax(q k^T * scale) v per head, no mask; q, k, v [n, H, dh]."""
    q = np.asarray(q, dtype=np.float64); k = np.asarray(k, dtype=np.float64); v = np.asarray(v, dtype=np.float64)
    n, H, dh = q.shape
    scale = 1.0 / np.sqrt(dh) if scale is None else scale
    out = np.empty_like(q)
    for h in range(H):
        logit = q[:, h, :] @ k[:, h, :].T * scale
        logit -= logit.max(axis=1, keepdims=True)
        p = np.exp(logit)
        p /= p.sum(axis=1, keepdims=True)
        out[:, h, :] = p @ v[:, h, :]
    return out


class Block:
    """Weights of one block: RMSNorm gains [d], projections as [out, in] matrices."""

    def __init__(self, attn_norm, wq, wk, wv, wo, ffn_norm, w_gate, w_up, w_down):
        self.attn_norm, self.wq, self.wk, self.wv, self.wo = attn_norm, wq, wk, wv, wo
        self.ffn_norm, self.w_gate, self.w_up, self.w_down = ffn_norm, w_gate, w_up, w_down


def attention_part(h, blk: Block, H: int, pos, eps: float, theta: float, rt) -> tuple:
    """First half of a block on hidden states h [n, d] whose tokens sit at positions pos [n]:
        a = rmsnorm(h);  q, k, v = a Wq^T, a Wk^T, a Wv^T;  q, k rotated at pos;
        h~ = h + attention(q, k, v) Wo^T
    rt is applied to every tensor where it is handed on.  Returns (h~, rotated q, rotated k)."""
    n, d = h.shape
    dh = d // H
    a = rt(rmsnorm(h, blk.attn_norm, eps))
    q = rt(linear(a, blk.wq)).reshape(n, H, dh)
    k = rt(linear(a, blk.wk)).reshape(n, H, dh)
    v = rt(linear(a, blk.wv)).reshape(n, H, dh)
    q = rt(rope(q, pos, theta)); k = rt(rope(k, pos, theta))
    o = rt(attention(q, k, v)).reshape(n, d)
    return rt(h + linear(o, blk.wo)), q, k


def ffn_part(ht, blk: Block, eps: float, rt) -> np.ndarray:
    """Second half of a block: h = h~ + (silu(f Wg^T) * (f Wu^T)) Wd^T with f = rmsnorm(h~)."""
    f = rt(rmsnorm(ht, blk.ffn_norm, eps))
    act = rt(swiglu(linear(f, blk.w_gate), linear(f, blk.w_up)))
    return rt(ht + linear(act, blk.w_down))


def stack_step(x, blocks: Sequence[Block], H: int, dec_idx, vis_start: int, V: int, keep_k: int,
               merge_layer: int, eps: float = 1e-5, theta: float = 10000.0, store="bf16", mode: str = "mean") -> dict:
    """One denoising step: hidden states x [N, d] through all blocks.

    Per block l = 1 .. L (pre-norm residual blocks):
        h~, q, k = attention_part(h)                           (post-attention hidden state)
        if l == merge_layer and there are deciders:            (Algorithm 1)
            S from this block's q, k (the attention it just used);  keep the keep_k best visual tokens;
            pruned tokens go to their most cosine-similar kept token in h~;  h~ <- merged rows,
            positions of the dropped tokens are removed (kept tokens keep their original positions)
        h = ffn_part(h~)
    Positions are the indices 0 .. N-1 of the input sequence.  No final norm, no decoding head.
    Returns y [N_out, d], src_pos [N_out] and the merge layer's intermediate results."""
    rt = _store_fn(store)
    h = np.asarray(x, dtype=np.float64)
    N, d = h.shape
    pos = np.arange(N, dtype=np.int64)
    dec = np.asarray(dec_idx, dtype=np.int32) if dec_idx is not None else np.zeros(0, dtype=np.int32)
    info = dict(merged=False)
    for l, blk in enumerate(blocks, start=1):
        ht, q, k = attention_part(h, blk, H, pos, eps, theta, rt)
        if l == merge_layer and len(dec) > 0:
            S = _importance(q, k, dec, vis_start, V)
            kept, slot_of = _select_topk(S, keep_k)
            asg, best_cos = _assign(ht, vis_start, V, kept, return_cos=True)
            y, counts, src = _merge(ht, vis_start, V, kept, asg, mode)
            pre_merge = ht
            # rows with a single member are the kept token itself: already stored values, rounding is a no-op
            ht = rt(y)
            pos = pos[src]
            info = dict(merged=True, S=S, kept_idx=kept, slot_of=slot_of, assign=asg, best_cos=best_cos, counts=counts,
                        pre_merge=pre_merge)
        h = ffn_part(ht, blk, eps, rt)
    info.update(y=h, src_pos=pos.astype(np.int32))
    return info
