"""Test-side composition of the stack oracle's pieces for chained GPU comparisons.

oracle/stack.py is the definition alone (Algorithm 1 with the oracle's own top-k and argmax).  A whole-step
comparison needs two things that are not part of the method and therefore live here:
  * the GPU's (already checked) kept list and assignment in place of the oracle's own choices, so that an
    excused near-tie does not cascade through the blocks that follow;
  * a storage function that perturbs every value by a few float32 ulps before it is rounded, which
    measures how far stored bf16 results move under the difference any float32 implementation has to
    float64 (the rounding floor the whole-step tolerance is sized from).
The blocks themselves are OS.attention_part / OS.ffn_part and the C oracle's stages, called in the
order OS.stack_step calls them.
"""
from __future__ import annotations

import numpy as np

import oracle
from oracle import stack as OS


def jittered_bf16(jitter: float, seed: int = 0):
    """Rounding to bf16 of values first multiplied by (1 + jitter * N(0,1))."""
    rng = np.random.default_rng(seed)
    return lambda a: OS.round_bf16(np.asarray(a, dtype=np.float64) * (1.0 + jitter * rng.standard_normal(np.shape(a))))


def stack_step_given(x, blocks, H, dec_idx, vis_start, V, keep_k, merge_layer, kept=None, assign=None,
                     eps=1e-5, theta=10000.0, store="bf16", mode="mean") -> dict:
    """OS.stack_step with the merge driven by the given kept list / assignment (None = the oracle's own).
    Returns what OS.stack_step returns plus the oracle's own choices (own_kept_idx, own_assign)."""
    rt = OS._store_fn(store)
    h = np.asarray(x, dtype=np.float64)
    pos = np.arange(h.shape[0], dtype=np.int64)
    dec = np.asarray(dec_idx, dtype=np.int32) if dec_idx is not None else np.zeros(0, dtype=np.int32)
    info = dict(merged=False)
    for l, blk in enumerate(blocks, start=1):
        ht, q, k = OS.attention_part(h, blk, H, pos, eps, theta, rt)
        if l == merge_layer and len(dec) > 0:
            S = oracle.importance(q, k, dec, vis_start, V)
            own_kept, _ = oracle.select_topk(S, keep_k)
            use_kept = own_kept if kept is None else np.asarray(kept, dtype=np.int32)
            own_assign, best_cos = oracle.assign(ht, vis_start, V, use_kept, return_cos=True)
            use_assign = own_assign if assign is None else np.asarray(assign, dtype=np.int32)
            y, counts, src = oracle.merge(ht, vis_start, V, use_kept, use_assign, mode)
            info = dict(merged=True, S=S, kept_idx=use_kept, own_kept_idx=own_kept, assign=use_assign,
                        own_assign=own_assign, best_cos=best_cos, counts=counts, pre_merge=ht)
            ht = rt(y)
            pos = pos[src]
        h = OS.ffn_part(ht, blk, eps, rt)
    info.update(y=h, src_pos=pos.astype(np.int32))
    return info
