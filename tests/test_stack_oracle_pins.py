"""Pins for the stack oracle (oracle/stack.py): each building block against a library routine, a closed
form or an invariant that does not go through the oracle's own formula, and the whole step against a
model assembled from torch's CPU routines in float64.

The paper prints no numeric example of a block; what fixes the result is the definition of the
standard operations (RMSNorm, rotary embedding, SwiGLU, softmax attention) and Algorithm 1's placement
of the merge between a block's attention and its feed-forward part.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from oracle import stack as OS
from paper_2511_12280_amd import workloads as W
from stack_chain import jittered_bf16, stack_step_given


def _rng(seed):
    return np.random.default_rng(seed)


# ---- storage rounding ------------------------------------------------------------------------
def test_round_bf16_hand_values():
    # 8 significant bits: spacing 2^-7 in [1, 2)
    u = 2.0 ** -7
    cases = {1.0: 1.0, 1.0 + u / 2: 1.0,               # tie -> even mantissa (1.0)
             1.0 + 3 * u / 2: 1.0 + 2 * u,             # tie -> even mantissa (1 + 2u)
             1.0 + 0.51 * u: 1.0 + u, 1.0 + 0.49 * u: 1.0,
             -3.0 - 2 * u * 0.75: -3.0 - 2 * u,        # spacing 2^-6 in [2, 4)
             0.0: 0.0, 2.0 - u / 4: 2.0}               # carries into the next binade
    for x, want in cases.items():
        assert OS.round_bf16(np.array([x]))[0] == want, x


def test_round_bf16_matches_torch_cast():
    x = (_rng(0).standard_normal(20000) * np.exp(_rng(1).uniform(-20, 20, 20000))).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(OS.round_bf16(x.astype(np.float64)), want)


def test_round_bf16_rounds_once_from_float64():
    # just above a bf16 tie: going through float32 first would land on the tie and round down to even
    x = 1.0 + 2.0 ** -8 + 2.0 ** -40
    assert np.float32(x) == np.float32(1.0 + 2.0 ** -8)
    assert OS.round_bf16(np.array([x]))[0] == 1.0 + 2.0 ** -7


# ---- RMSNorm ---------------------------------------------------------------------------------
def test_rmsnorm_matches_torch():
    x = _rng(2).standard_normal((7, 48)); g = _rng(3).standard_normal(48)
    want = F.rms_norm(torch.from_numpy(x), (48,), torch.from_numpy(g), eps=1e-5).numpy()
    np.testing.assert_allclose(OS.rmsnorm(x, g, 1e-5), want, rtol=1e-13, atol=1e-15)


def test_rmsnorm_invariants():
    x = _rng(4).standard_normal((5, 64)) * 7.0
    y = OS.rmsnorm(x, np.ones(64), 0.0)
    np.testing.assert_allclose(np.sqrt((y * y).mean(axis=1)), 1.0, rtol=1e-13)      # unit rms
    np.testing.assert_allclose(OS.rmsnorm(3.5 * x, np.ones(64), 0.0), y, rtol=1e-13)  # scale invariance
    # eps enters under the root, next to the mean square
    one = OS.rmsnorm(np.full((1, 4), 2.0), np.ones(4), 5.0)
    np.testing.assert_allclose(one, 2.0 / 3.0, rtol=1e-15)


# ---- rotary embedding ------------------------------------------------------------------------
def _rope_complex(x, pos, theta):
    """Same rotation written as a complex multiplication with torch.polar."""
    n, H, dh = x.shape
    half = dh // 2
    xc = torch.complex(torch.from_numpy(x[..., :half].copy()), torch.from_numpy(x[..., half:].copy()))
    freq = torch.tensor(theta, dtype=torch.float64) ** (-torch.arange(0, dh, 2, dtype=torch.float64) / dh)
    ang = torch.from_numpy(np.asarray(pos, dtype=np.float64))[:, None] * freq[None, :]
    rot = torch.polar(torch.ones_like(ang), ang)[:, None, :]
    out = xc * rot
    return torch.cat([out.real, out.imag], dim=-1).numpy()


def test_rope_matches_complex_rotation():
    x = _rng(5).standard_normal((9, 3, 16)); pos = np.array([0, 1, 2, 5, 40, 41, 1000, 3772, 7])
    np.testing.assert_allclose(OS.rope(x, pos, 10000.0), _rope_complex(x, pos, 10000.0), rtol=1e-12, atol=1e-13)


def test_rope_hand_value_and_identity():
    # one head, two channels: a plain rotation of the pair by `pos` radians (theta^0 = 1)
    x = np.array([[[1.0, 0.0]], [[0.0, 2.0]]])
    y = OS.rope(x, np.array([0.5, np.pi / 2]), 10000.0)
    np.testing.assert_allclose(y[0, 0], [np.cos(0.5), np.sin(0.5)], atol=1e-15)
    np.testing.assert_allclose(y[1, 0], [-2.0, 0.0], atol=1e-15)
    z = _rng(6).standard_normal((4, 2, 8))
    np.testing.assert_array_equal(OS.rope(z, np.zeros(4), 500000.0), z)                 # position 0: identity


def test_rope_scores_depend_on_relative_position_only():
    q = _rng(7).standard_normal((1, 2, 32)); k = _rng(8).standard_normal((1, 2, 32))
    def score(m, n):
        return (OS.rope(q, np.array([m]), 10000.0) * OS.rope(k, np.array([n]), 10000.0)).sum(axis=-1)
    np.testing.assert_allclose(score(3, 10), score(103, 110), rtol=1e-11)
    np.testing.assert_allclose(score(50, 20), score(30, 0), rtol=1e-11)
    # the slowest channel pair turns by theta^(-(dh-2)/dh) per position
    x = np.zeros((1, 1, 32)); x[0, 0, 15] = 1.0
    y = OS.rope(x, np.array([1]), 10000.0)
    np.testing.assert_allclose(y[0, 0, 15], np.cos(10000.0 ** (-30.0 / 32.0)), rtol=1e-14)
    np.testing.assert_allclose(y[0, 0, 31], np.sin(10000.0 ** (-30.0 / 32.0)), rtol=1e-12)


# ---- SwiGLU, linear, attention ---------------------------------------------------------------
def test_swiglu_matches_torch_silu():
    g = _rng(9).standard_normal(1000) * 4; u = _rng(10).standard_normal(1000)
    want = (F.silu(torch.from_numpy(g)) * torch.from_numpy(u)).numpy()
    np.testing.assert_allclose(OS.swiglu(g, u), want, rtol=1e-13, atol=1e-300)


def test_linear_is_rows_of_w():
    a = _rng(11).standard_normal((3, 5)); w = _rng(12).standard_normal((4, 5))
    want = np.array([[sum(a[i, c] * w[j, c] for c in range(5)) for j in range(4)] for i in range(3)])
    np.testing.assert_allclose(OS.linear(a, w), want, rtol=1e-14)
    np.testing.assert_allclose(OS.linear(a, w), F.linear(torch.from_numpy(a), torch.from_numpy(w)).numpy(), rtol=1e-14)


def test_attention_matches_torch_sdpa_and_c_oracle():
    q, k, v = (_rng(s).standard_normal((23, 3, 8)) for s in (13, 14, 15))
    tq, tk, tv = (torch.from_numpy(t).permute(1, 0, 2) for t in (q, k, v))
    want = F.scaled_dot_product_attention(tq, tk, tv).permute(1, 0, 2).numpy()
    got = OS.attention(q, k, v)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-14)
    q32, k32, v32 = (t.astype(np.float32) for t in (q, k, v))
    np.testing.assert_allclose(OS.attention(q32, k32, v32), oracle.attend(q32, k32, v32), rtol=1e-12, atol=1e-14)


# ---- the whole step --------------------------------------------------------------------------
def _blocks(case):
    return [OS.Block(**b) for b in case["blocks"]]


def _torch_stack(case, eps, theta, upto=None, start=None):
    """Unmerged stack from torch's float64 CPU routines (rms_norm, linear, SDPA, silu) and the complex
    form of the rotation."""
    H, d = case["H"], case["d"]
    dh = d // H
    h = torch.from_numpy(case["x"].astype(np.float64)) if start is None else start
    n = h.shape[0]
    pos = np.arange(n)
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    for b in case["blocks"][:upto]:
        a = F.rms_norm(h, (d,), t(b["attn_norm"]), eps=eps)
        q = F.linear(a, t(b["wq"])).reshape(n, H, dh).numpy()
        k = F.linear(a, t(b["wk"])).reshape(n, H, dh).numpy()
        v = F.linear(a, t(b["wv"])).reshape(n, H, dh)
        q = torch.from_numpy(_rope_complex(q, pos, theta)); k = torch.from_numpy(_rope_complex(k, pos, theta))
        o = F.scaled_dot_product_attention(q.permute(1, 0, 2), k.permute(1, 0, 2), v.permute(1, 0, 2))
        h = h + F.linear(o.permute(1, 0, 2).reshape(n, d), t(b["wo"]))
        f = F.rms_norm(h, (d,), t(b["ffn_norm"]), eps=eps)
        h = h + F.linear(F.silu(F.linear(f, t(b["w_gate"]))) * F.linear(f, t(b["w_up"])), t(b["w_down"]))
    return h.numpy()


def test_stack_without_deciders_is_the_plain_model():
    c = W.stack_case(1, L=3, d=64, H=2, F=96, P=3, V=20, O=6, D=3, std=0.15, gain_jitter=0.2)
    out = OS.stack_step(c["x"], _blocks(c), c["H"], None, c["vis_start"], c["V"], 5, merge_layer=2,
                        eps=1e-5, theta=10000.0, store=None)
    assert not out["merged"] and out["y"].shape == (c["N"], c["d"])
    np.testing.assert_array_equal(out["src_pos"], np.arange(c["N"]))
    np.testing.assert_allclose(out["y"], _torch_stack(c, 1e-5, 10000.0), rtol=1e-10, atol=1e-12)


def test_stack_keeping_every_token_changes_nothing():
    c = W.stack_case(2, L=3, d=64, H=2, F=96, P=3, V=20, O=6, D=3, std=0.15, gain_jitter=0.2)
    out = OS.stack_step(c["x"], _blocks(c), c["H"], c["dec_idx"], c["vis_start"], c["V"], c["V"], merge_layer=2,
                        store=None)
    assert out["merged"] and out["y"].shape[0] == c["N"]
    # the merge oracle reads float32, so the identity holds to float32 rounding of one hidden state
    np.testing.assert_allclose(out["y"], _torch_stack(c, 1e-5, 10000.0), rtol=2e-6, atol=2e-6)


def test_stack_merge_sits_between_attention_and_ffn_of_its_block():
    """Rebuild the merged step from the pieces: torch model up to the merge block's attention, the C merge
    oracle on that hidden state, then the remaining layers on the short sequence with the original positions."""
    c = W.stack_case(3, L=3, d=64, H=2, F=96, P=4, V=24, O=6, D=4, std=0.15, gain_jitter=0.2)
    eps, theta, l_star, keep_k = 1e-5, 10000.0, 2, 7
    H, d = c["H"], c["d"]; dh = d // H
    out = OS.stack_step(c["x"], _blocks(c), H, c["dec_idx"], c["vis_start"], c["V"], keep_k, merge_layer=l_star,
                        eps=eps, theta=theta, store=None)
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    h = t(_torch_stack(c, eps, theta, upto=l_star - 1))
    n = h.shape[0]
    b = c["blocks"][l_star - 1]
    a = F.rms_norm(h, (d,), t(b["attn_norm"]), eps=eps)
    q = _rope_complex(F.linear(a, t(b["wq"])).reshape(n, H, dh).numpy(), np.arange(n), theta)
    k = _rope_complex(F.linear(a, t(b["wk"])).reshape(n, H, dh).numpy(), np.arange(n), theta)
    v = F.linear(a, t(b["wv"])).reshape(n, H, dh)
    o = F.scaled_dot_product_attention(t(q).permute(1, 0, 2), t(k).permute(1, 0, 2), v.permute(1, 0, 2))
    ht = (h + F.linear(o.permute(1, 0, 2).reshape(n, d), t(b["wo"]))).numpy()
    m = oracle.merge_layer(q, k, ht, c["dec_idx"], c["vis_start"], c["V"], keep_k)
    np.testing.assert_array_equal(out["kept_idx"], m["kept_idx"])
    np.testing.assert_array_equal(out["src_pos"], m["src_pos"])
    assert out["y"].shape[0] == c["N"] - (c["V"] - keep_k)
    # FFN of the merge block and the last block, short sequence, rotary angles from the original positions
    hm = t(m["y"]); pos = m["src_pos"]; nm = hm.shape[0]
    f = F.rms_norm(hm, (d,), t(b["ffn_norm"]), eps=eps)
    hm = hm + F.linear(F.silu(F.linear(f, t(b["w_gate"]))) * F.linear(f, t(b["w_up"])), t(b["w_down"]))
    for b in c["blocks"][l_star:]:
        a = F.rms_norm(hm, (d,), t(b["attn_norm"]), eps=eps)
        q = t(_rope_complex(F.linear(a, t(b["wq"])).reshape(nm, H, dh).numpy(), pos, theta))
        k = t(_rope_complex(F.linear(a, t(b["wk"])).reshape(nm, H, dh).numpy(), pos, theta))
        v = F.linear(a, t(b["wv"])).reshape(nm, H, dh)
        o = F.scaled_dot_product_attention(q.permute(1, 0, 2), k.permute(1, 0, 2), v.permute(1, 0, 2))
        hm = hm + F.linear(o.permute(1, 0, 2).reshape(nm, d), t(b["wo"]))
        f = F.rms_norm(hm, (d,), t(b["ffn_norm"]), eps=eps)
        hm = hm + F.linear(F.silu(F.linear(f, t(b["w_gate"]))) * F.linear(f, t(b["w_up"])), t(b["w_down"]))
    np.testing.assert_allclose(out["y"], hm.numpy(), rtol=5e-6, atol=5e-6)


def test_stack_bf16_storage_stays_close_to_exact_arithmetic():
    c = W.stack_case(4, L=4, d=64, H=2, F=128, P=4, V=24, O=6, D=4, std=0.15, gain_jitter=0.1)
    kw = dict(merge_layer=2, eps=1e-5, theta=10000.0)
    exact = OS.stack_step(c["x"], _blocks(c), c["H"], c["dec_idx"], c["vis_start"], c["V"], 8, store=None, **kw)
    b16 = stack_step_given(c["x"], _blocks(c), c["H"], c["dec_idx"], c["vis_start"], c["V"], 8, store="bf16",
                           kept=exact["kept_idx"], assign=exact["assign"], **kw)
    # every stored value is a bf16 number
    np.testing.assert_array_equal(OS.round_bf16(b16["y"]), b16["y"])
    err = np.sqrt(np.mean((b16["y"] - exact["y"]) ** 2)) / np.sqrt(np.mean(exact["y"] ** 2))
    # ~10 roundings per block, each 2^-9/sqrt(3) relative rms, adding in quadrature: ~7e-3 for 4 blocks
    assert 1e-4 < err < 3e-2, err


def test_chain_wrapper_is_the_oracle_step_when_nothing_is_given_and_follows_what_is_given():
    # the test-side composition (tests/stack_chain.py) calls the same pieces in the same order: with no kept
    # list / assignment handed in it must reproduce OS.stack_step bit for bit; handed a different kept list it
    # must use it and still report the oracle's own choice
    c = W.stack_case(5, L=2, d=64, H=2, F=64, P=2, V=16, O=4, D=2, std=0.15)
    base = OS.stack_step(c["x"], _blocks(c), c["H"], c["dec_idx"], c["vis_start"], c["V"], 4, merge_layer=1)
    same = stack_step_given(c["x"], _blocks(c), c["H"], c["dec_idx"], c["vis_start"], c["V"], 4, 1)
    for key in ("y", "src_pos", "S", "kept_idx", "assign", "counts"):
        np.testing.assert_array_equal(same[key], base[key])
    other = np.sort(np.setdiff1d(np.arange(c["V"]), base["kept_idx"])[:4]).astype(np.int32)
    alt = stack_step_given(c["x"], _blocks(c), c["H"], c["dec_idx"], c["vis_start"], c["V"], 4, 1, kept=other)
    np.testing.assert_array_equal(alt["own_kept_idx"], base["kept_idx"])
    np.testing.assert_array_equal(alt["kept_idx"], other)
    assert not np.array_equal(alt["src_pos"], base["src_pos"])
    # a jittered storage function moves stored values by whole bf16 steps only
    jit = stack_step_given(c["x"], _blocks(c), c["H"], c["dec_idx"], c["vis_start"], c["V"], 4, 1,
                           kept=base["kept_idx"], assign=base["assign"], store=jittered_bf16(3e-7, 1))
    np.testing.assert_array_equal(OS.round_bf16(jit["y"]), jit["y"])
    assert 0 < np.abs(jit["y"] - base["y"]).max() < 0.1 * np.abs(base["y"]).max()
