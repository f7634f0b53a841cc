"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_12280_amd import workloads as W

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from paper_2511_12280_amd import binding as B
    from parity import (GpuStep, check_assign, check_attend, check_full_sample, check_kept, check_merge,
                        check_scores, gpu_attend, gpu_attend_weighted, key_weights)


def _chain(samples, keeps, dtype, mode="mean", assign_rows=None, check=None):
    step = GpuStep(samples, keeps, dtype, B.D3TOM_MERGE_MEAN if mode == "mean" else B.D3TOM_MERGE_SUM)
    S = step.importance()
    kept, slot = step.select_topk()
    mout = step.merge()
    stats = []
    for b in (range(len(samples)) if check is None else check):
        stats.append(check_full_sample(step, b, S, kept, slot, mout, assign_rows=assign_rows, mode=mode))
    return step, S, kept, mout, stats


# ---- the tiny fp32 layer: whole chain including the attention on the merged rows -------------------
def test_tiny_f32_chain_with_attention():
    wl = W.WORKLOADS["tiny_f32"]
    g = W.SampleGen(wl)
    s = g.step(16)
    k = oracle.keep_count(wl.V, 0.25)
    assert k == 36 and B.d3tom_keep_count(wl.V, 0.25) == 36
    step, S, kept, mout, stats = _chain([s], [k], "f32")
    assert stats[0]["kept_excused"] == 0 and stats[0]["assign_excused"] == 0
    y = mout["y"][0]
    assert y.shape == (100, 256)
    q2, k2, v2 = g.proj.qkv(y)                       # projection of the merged rows (host, not on the path)
    o = gpu_attend([(q2, k2, v2)], "f32")[0]
    check_attend(o, q2, k2, v2, "f32")


# ---- bf16 cases spanning several tiles with ragged tails ----------------------------------------------
@pytest.mark.parametrize("P,V,O,H,dh,D,keep,mode", [
    (37, 700, 40, 8, 128, 20, 0.23, "mean"),
    (5, 333, 9, 4, 64, 3, 0.50, "mean"),
    (0, 130, 17, 2, 128, 17, 0.10, "sum"),
    (3, 1000, 70, 4, 128, 70, 0.77, "mean"),
])
def test_bf16_cases(P, V, O, H, dh, D, keep, mode):
    c = W.random_case(100 + V, P + V + O, H * dh, H, P, V, D, dtype="bf16", centres=max(4, V // 6))
    k = oracle.keep_count(V, keep)
    _chain([c], [k], "bf16", mode=mode)


def test_f32_generic_case_and_odd_head_size():
    c = W.random_case(7, 150, 4 * 36, 4, 10, 120, 6, dtype="f32", centres=9)      # dh = 36
    _chain([c], [oracle.keep_count(120, 0.3)], "f32")
    c = W.random_case(8, 90, 2 * 40, 2, 4, 80, 5, dtype="bf16", centres=9)        # bf16 with dh = 40: generic kernels
    _chain([c], [oracle.keep_count(80, 0.25)], "bf16")


# ---- tile-edge shapes: counts that sit exactly on, one below and one above the kernels' tile sizes --------
@pytest.mark.parametrize("P,V,O,D,k", [
    (0, 512, 16, 16, 128),       # keys = one 512-key chunk + deciders, kept = one 128-slot column tile, pruned = 6 x 64
    (1, 513, 33, 33, 129),       # one past every boundary
    (0, 511, 256, 256, 127),     # the largest decider set, one below the boundaries
    (3, 257, 17, 17, 256),       # a single pruned token
    (5, 640, 48, 47, 64),        # 9 row tiles x 1 half-filled column tile (split along the contraction)
])
def test_tile_edge_shapes(P, V, O, D, k):
    c = W.random_case(1000 + V + k, P + V + O, 2 * 128, 2, P, V, D, dtype="bf16", centres=max(4, V // 9))
    step, S, kept, mout, stats = _chain([c], [k], "bf16")
    assert mout["y"][0].shape[0] == P + k + O
    n_m = P + k + O
    qkv = W.random_qkv(2000 + n_m, n_m, 2, 128, "bf16")
    check_attend(gpu_attend([qkv], "bf16")[0], *qkv, "bf16")


# ---- ragged batch ----------------------------------------------------------------------------------
def test_ragged_batch_bf16():
    shapes = [(20, 300, 30, 9, 0.2), (64, 513, 64, 33, 0.5), (1, 128, 5, 1, 0.1), (7, 129, 300, 100, 0.33), (0, 64, 2, 2, 1.0)]
    samples, keeps = [], []
    for i, (P, V, O, D, keep) in enumerate(shapes):
        samples.append(W.random_case(200 + i, P + V + O, 4 * 128, 4, P, V, D, dtype="bf16", centres=max(3, V // 5)))
        keeps.append(oracle.keep_count(V, keep))
    step, S, kept, mout, stats = _chain(samples, keeps, "bf16")
    # keep ratio 1: identity
    np.testing.assert_array_equal(mout["y"][4], samples[4]["x"])
    np.testing.assert_array_equal(kept[4], np.arange(64))


# ---- top-k in isolation: exact, ties, extremes ---------------------------------------------------------
def _topk_only(scores_list, ks):
    V = [len(s) for s in scores_list]
    lay = B.Layout(V, [0] * len(V), V, [[0]] * len(V), ks)
    sc = torch.from_numpy(np.concatenate(scores_list).astype(np.float32)).cuda()
    kept = torch.zeros(sum(ks), dtype=torch.int32, device="cuda")
    slot = torch.zeros(sum(V), dtype=torch.int32, device="cuda")
    B.d3tom_select_topk(sc, lay, kept, slot)
    torch.cuda.synchronize()
    return GpuStep.split(kept.cpu().numpy(), ks), GpuStep.split(slot.cpu().numpy(), V)


def test_topk_exact_including_ties_and_extremes():
    rng = np.random.default_rng(0)
    cases = [
        (rng.standard_normal(1).astype(np.float32), 1),
        (rng.standard_normal(1000).astype(np.float32), 1),
        (rng.standard_normal(1000).astype(np.float32), 1000),
        (rng.random(3645).astype(np.float32), 365),
        (np.round(rng.random(5000) * 8).astype(np.float32) / 8, 1234),          # heavy ties
        (np.zeros(777, np.float32), 100),                                      # all equal: lowest indices
        (np.concatenate([-rng.random(500), rng.random(500)]).astype(np.float32), 600),   # negative scores
        (rng.random(B.D3TOM_MAX_VISUAL).astype(np.float32) * 1e-6, 4000),      # largest supported |V|
        (np.float32(1.0) + rng.integers(0, 3, 4097).astype(np.float32) * np.float32(2 ** -23), 2048),  # 1-ulp apart
    ]
    kept, slot = _topk_only([c[0] for c in cases], [c[1] for c in cases])
    for (s, k), kg, sg in zip(cases, kept, slot):
        kr, sr = oracle.select_topk(s, k)
        np.testing.assert_array_equal(kg, kr)
        np.testing.assert_array_equal(sg, sr)


# ---- workspace -------------------------------------------------------------------------------------------
@pytest.mark.parametrize("P,V,O,D,k,d", [(8, 700, 16, 9, 150, 512),      # normal cosine path (several tiles)
                                          (4, 300, 8, 5, 40, 4096)])      # few tiles, long rows: split along k
def test_workspace_contents_do_not_matter(P, V, O, D, k, d):
    """The workspace carries no state: whatever bytes it holds on entry (zeros, all-ones = NaN / -1), the
    outputs are bit-identical."""
    c = W.random_case(11, P + V + O, d, d // 128, P, V, D, dtype="bf16", centres=30)
    runs = []
    for fill in (0, 255):
        step = GpuStep([c], [k], "bf16")
        step.ws_imp.fill_(fill); step.ws_merge.fill_(fill)
        S = step.importance()
        step.ws_imp.fill_(fill)
        kept, slot = step.select_topk()
        mout = step.merge()
        runs.append((S[0], kept[0], mout["y"][0], mout["assign"][0], mout["counts"][0], mout["src_pos"][0]))
    for a, b in zip(*runs):
        np.testing.assert_array_equal(a, b)


# ---- attention in isolation ---------------------------------------------------------------------------
@pytest.mark.parametrize("H,dh,dtype", [(4, 128, "bf16"), (3, 64, "bf16"), (2, 64, "f32"), (2, 40, "bf16")])
def test_attend_varlen(H, dh, dtype):
    lens = [1, 63, 64, 65, 200, 231, 493] if dh in (64, 128) and dtype == "bf16" else [1, 65, 300]
    qkv = [W.random_qkv(300 + n, n, H, dh, dtype) for n in lens]
    outs = gpu_attend(qkv, dtype)
    for (q, k, v), o in zip(qkv, outs):
        check_attend(o, q, k, v, dtype)


@pytest.mark.parametrize("longest", [512, 513])
@pytest.mark.parametrize("H,dh", [(5, 128), (3, 64)])
def test_attend_both_sides_of_the_short_sample_limit(H, dh, longest):
    """Up to 512 keys per sample the keys are split across the waves of a workgroup; one key more and the
    tiled kernel takes the whole batch, short samples included."""
    lens = [1, 31, 32, 33, 97, 129, longest]
    qkv = [W.random_qkv(700 + n, n, H, dh, "bf16") for n in lens]
    outs = gpu_attend(qkv, "bf16")
    for (q, k, v), o in zip(qkv, outs):
        check_attend(o, q, k, v, "bf16")


def test_attend_special_cases_bf16():
    q, k, v = W.random_qkv(5, 150, 2, 128, "bf16", spread=2.0)
    v1 = np.broadcast_to(v[:1], v.shape).copy()
    o = gpu_attend([(q, k, v1)], "bf16")[0]
    np.testing.assert_allclose(o, v1, atol=1e-2)            # identical value rows come back (rows sum to one)
    perm = np.random.default_rng(1).permutation(150)
    o1 = gpu_attend([(q, k, v)], "bf16")[0]
    o2 = gpu_attend([(q, k[perm], v[perm])], "bf16")[0]
    np.testing.assert_allclose(o1, o2, atol=2e-2)           # no mask: key order is irrelevant


# ---- size-weighted attention (member counts of the merge as key weights) -------------------------------
@pytest.mark.parametrize("H,dh,dtype,lens", [
    (4, 128, "bf16", [700, 65, 1300]),          # tiled kernel, ragged
    (3, 64, "bf16", [300, 1, 512, 33]),         # short-sample kernel
    (2, 64, "f32", [90, 17]),                   # generic kernel, float32
    (2, 40, "bf16", [70]),                      # generic kernel, odd head size
])
def test_attend_weighted_varlen(H, dh, dtype, lens):
    rng = np.random.default_rng(len(lens) * 100 + dh)
    qkv = [W.random_qkv(900 + n, n, H, dh, dtype) for n in lens]
    vis, counts = [], []
    for n in lens:
        vs = int(rng.integers(0, max(1, n // 3)))
        kn = int(rng.integers(0, n - vs + 1))          # merged rows: anything from none to the rest of the sample
        vis.append(vs)
        counts.append(rng.integers(1, 40, size=kn).astype(np.int32))
    outs = gpu_attend_weighted(qkv, counts, vis, dtype)
    plain = gpu_attend(qkv, dtype)
    for (q, k, v), o, o1, vs, c, n in zip(qkv, outs, plain, vis, counts, lens):
        check_attend(o, q, k, v, dtype, key_weight=key_weights(n, vs, c))
        if len(c) and c.max() > 1 and n > 1:
            assert np.abs(o - o1).max() > 1e-3          # the weights do change the result
    # all counts 1: the plain attention, bit for bit (same kernel arithmetic up to the added zero)
    ones = [np.ones(len(c), np.int32) for c in counts]
    for o, o1 in zip(gpu_attend_weighted(qkv, ones, vis, dtype), plain):
        np.testing.assert_allclose(o, o1, atol=TOL_SAME[dtype])


TOL_SAME = {"bf16": 2.0 ** -7, "f32": 1e-5}


def test_merge_counts_feed_weighted_attention():
    """The counts d3tom_merge writes are what d3tom_attend_weighted reads: merge a sample, project the merged rows
    (host, not on the path), attend with the counts as key weights, compare with the oracle given the same weights."""
    wl = W.WORKLOADS["tiny_f32"]
    g = W.SampleGen(wl)
    s = g.step(16)
    k = oracle.keep_count(wl.V, 0.25)
    step, S, kept, mout, stats = _chain([s], [k], "f32")
    q2, k2, v2 = g.proj.qkv(mout["y"][0])
    n_m = q2.shape[0]
    cu = torch.tensor([0, n_m], dtype=torch.int32, device="cuda")
    o = torch.zeros((n_m,) + q2.shape[1:], dtype=torch.float32, device="cuda")
    B.d3tom_attend_weighted(B.to_device(q2, "f32"), B.to_device(k2, "f32"), B.to_device(v2, "f32"), cu, n_m,
                            1.0 / np.sqrt(q2.shape[2]), step.counts, step.lay.kept_off, step.lay.vis_start, o)
    torch.cuda.synchronize()
    assert mout["counts"][0].sum() == wl.V
    check_attend(B.to_host(o), q2, k2, v2, "f32", key_weight=key_weights(n_m, s["vis_start"], mout["counts"][0]))


# ---- the merge layer in one call, kept counts computed on the device --------------------------------------
@pytest.mark.parametrize("tight", [True, False])
def test_merge_layer_one_call_with_device_side_keep_counts(tight):
    """d3tom_merge_layer against the three separate calls on a ragged batch: the kept counts it computes on the
    device from the ratios are those of d3tom_keep_count (and of the oracle), and with tight bounds on them every
    output is bit-identical to the separate calls; with the loosest bounds (1 .. |V|) the launches are shaped
    differently, so the outputs are checked against the oracle instead."""
    shapes = [(20, 300, 30, 9, 0.2), (64, 513, 64, 33, 0.5), (1, 128, 5, 1, 0.1), (7, 129, 300, 20, 1.0 / 3.0), (0, 64, 2, 2, 1.0),
              (3, 700, 9, 4, 0.25)]
    samples, ratios = [], []
    for i, (P, V, O, D, keep) in enumerate(shapes):
        samples.append(W.random_case(300 + i, P + V + O, 4 * 128, 4, P, V, D, dtype="bf16", centres=max(3, V // 5)))
        ratios.append(keep)
    keeps = [oracle.keep_count(s["V"], r) for s, r in zip(samples, ratios)]
    assert keeps == [B.d3tom_keep_count(s["V"], r) for s, r in zip(samples, ratios)]
    ref = GpuStep(samples, keeps, "bf16")
    S = ref.importance(); kept, slot = ref.select_topk(); mout = ref.merge()
    lay = ref.lay
    nb = lay.B
    dev_i32 = lambda n: torch.full((n,), -7, dtype=torch.int32, device="cuda")
    scores = torch.zeros(lay.sum_V, dtype=torch.float32, device="cuda")
    keep_k, kept_off, out_off = dev_i32(nb), dev_i32(nb + 1), dev_i32(nb + 1)
    kept_idx = dev_i32(nb * lay.max_V)
    y = torch.zeros((lay.sum_N, ref.d), dtype=torch.bfloat16, device="cuda")
    assign, counts, src_pos = dev_i32(lay.sum_V), dev_i32(nb * lay.max_V), dev_i32(lay.sum_N)
    ws = B.workspace(B.d3tom_merge_layer_workspace_bytes(nb, lay.max_N, lay.max_V, ref.H, ref.dh, lay.max_D))
    ws.fill_(255)
    lo, hi = (min(keeps), max(keeps)) if tight else (1, lay.max_V)
    B.d3tom_merge_layer(ref.q, ref.k, ref.x, None, lay, ref.scale, torch.tensor(ratios, dtype=torch.float64, device="cuda"),
                        lo, hi, B.D3TOM_MERGE_MEAN, scores, keep_k, kept_off, kept_idx, out_off, y, assign, counts, src_pos, ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(keep_k.cpu().numpy(), keeps)
    np.testing.assert_array_equal(kept_off.cpu().numpy(), np.concatenate([[0], np.cumsum(keeps)]))
    np.testing.assert_array_equal(out_off.cpu().numpy(), np.concatenate([[0], np.cumsum(lay.Nm)]))
    np.testing.assert_array_equal(scores.cpu().numpy(), np.concatenate(S))
    np.testing.assert_array_equal(kept_idx[:lay.sum_keep].cpu().numpy(), np.concatenate(kept))
    got = dict(y=GpuStep.split(B.to_host(y[:lay.sum_Nm]), lay.Nm), assign=GpuStep.split(assign.cpu().numpy(), lay.V),
               counts=GpuStep.split(counts[:lay.sum_keep].cpu().numpy(), lay.keep),
               src_pos=GpuStep.split(src_pos[:lay.sum_Nm].cpu().numpy(), lay.Nm))
    for b in range(nb):
        if tight:
            for key in got:
                np.testing.assert_array_equal(got[key][b], mout[key][b])
        else:
            check_full_sample(ref, b, S, kept, slot, got)


@pytest.mark.parametrize("dtype,d,H,shapes", [
    ("f32", 96, 2, [(5, 90, 7, 3, 0.3), (0, 33, 4, 2, 0.5), (9, 200, 1, 6, 0.12)]),       # float32: the generic kernels
    ("bf16", 4096, 32, [(8, 260, 6, 3, 0.15)]),                                           # one short sample: cosine GEMM cut along the contraction
    ("bf16", 200, 5, [(3, 150, 5, 4, 0.4), (6, 61, 2, 1, 0.7)]),                          # bf16 rows of 400 bytes, head size 40: generic kernels
])
def test_merge_layer_one_call_on_every_kernel_path(dtype, d, H, shapes):
    """The one-call merge layer prepares the merge inside its selection launch (row norms by token, pruned list,
    token table); every cosine kernel reads that form.  Each path against the separate calls, bit for bit, and
    the separate calls against the oracle."""
    samples, ratios = [], []
    for i, (P, V, O, D, keep) in enumerate(shapes):
        samples.append(W.random_case(500 + i, P + V + O, d, H, P, V, D, dtype=dtype, centres=max(3, V // 6)))
        ratios.append(keep)
    keeps = [oracle.keep_count(s["V"], r) for s, r in zip(samples, ratios)]
    ref = GpuStep(samples, keeps, dtype)
    S = ref.importance(); kept, slot = ref.select_topk(); mout = ref.merge()
    for b in range(len(samples)):
        check_full_sample(ref, b, S, kept, slot, mout)
    S1, kept1, m1 = ref.merge_layer(ratios)
    for b in range(len(samples)):
        np.testing.assert_array_equal(S1[b], S[b])
        np.testing.assert_array_equal(kept1[b], kept[b])
        for key in m1:
            np.testing.assert_array_equal(m1[key][b], mout[key][b])


@pytest.mark.parametrize("d_sim", [128, 72])          # MFMA cosine path (a multiple of 64) and the generic one
def test_merge_layer_one_call_with_separate_similarity_features(d_sim):
    """`sim` != x in the one-call merge layer: the selection launch takes its row norms from `sim` (other row length
    than the payload), the payload rows come from x.  Against d3tom_merge with the same `sim`, bit for bit, and that
    against the oracle's assignment on the `sim` rows."""
    shapes = [(4, 210, 6, 3, 0.2), (0, 77, 3, 2, 0.6)]
    samples, ratios = [], []
    for i, (P, V, O, D, keep) in enumerate(shapes):
        samples.append(W.random_case(600 + i, P + V + O, 256, 4, P, V, D, dtype="bf16", centres=9))
        ratios.append(keep)
    keeps = [oracle.keep_count(s["V"], r) for s, r in zip(samples, ratios)]
    rng = np.random.default_rng(601)
    sim_rows = W.round_to(rng.standard_normal((sum(s["N"] for s in samples), d_sim)).astype(np.float32), "bf16")
    ref = GpuStep(samples, keeps, "bf16")
    S = ref.importance(); kept, slot = ref.select_topk(); mout = ref.merge(sim_rows=sim_rows)
    off = 0
    for b, s in enumerate(samples):
        check_assign(mout["assign"][b], sim_rows[off:off + s["N"]], s["vis_start"], s["V"], kept[b])
        off += s["N"]
    S1, kept1, m1 = ref.merge_layer(ratios, sim_rows=sim_rows)
    for b in range(len(samples)):
        np.testing.assert_array_equal(S1[b], S[b])
        np.testing.assert_array_equal(kept1[b], kept[b])
        for key in m1:
            np.testing.assert_array_equal(m1[key][b], mout[key][b])


# ---- degenerate inputs the oracle defines ------------------------------------------------------------------
@pytest.mark.parametrize("dtype,d,H", [("bf16", 512, 4), ("bf16", 4096, 32), ("f32", 96, 2)])
def test_zero_rows_in_the_similarity_features(dtype, d, H):
    """A zero row has cosine 0 with everything: a zero PRUNED row ties on all slots and goes to slot 0; a zero KEPT
    row scores 0 against every pruned row, so it wins exactly the pruned rows whose other cosines are all negative.
    MFMA path (bf16, d a multiple of 64, tiled and split along the contraction) and generic path (float32)."""
    P, V, O = 6, 330, 10
    c = W.random_case(71, P + V + O, d, H, P, V, 4, dtype=dtype, centres=3, noise=1.0)
    x = c["x"].copy()
    rng = np.random.default_rng(72)
    kept = np.sort(rng.choice(V, size=9, replace=False)).astype(np.int32)
    pruned = np.setdiff1d(np.arange(V), kept)
    zero_pruned, zero_kept = pruned[[3, 100, 250]], kept[[0, 5]]
    x[P + zero_pruned] = 0.0
    x[P + zero_kept] = 0.0
    # make a few pruned rows point away from every non-zero kept row, so that the zero kept rows get members
    x[P + pruned[[7, 8]]] = -x[P + kept[2]]
    c["x"] = x
    step = GpuStep([c], [len(kept)], dtype)
    out = step.merge([kept])
    a = out["assign"][0]
    ref, bc = oracle.assign(x, P, V, kept, return_cos=True)
    assert np.all(a[zero_pruned] == 0) and np.all(ref[zero_pruned] == 0) and np.all(bc[zero_pruned] == 0.0)
    check_assign(a, x, P, V, kept)
    check_merge({key: out[key][0] for key in out}, x, P, V, kept, dtype)
    assert np.isfinite(out["y"][0]).all()


def test_deciders_anywhere_with_a_repeat_on_the_mfma_path():
    """Decider positions inside and in front of the visual block, one of them listed twice (its row counts twice):
    the score is defined for any list of rows."""
    P, V, O, H, dh = 40, 600, 30, 4, 128
    c = W.random_case(73, P + V + O, H * dh, H, P, V, 3, dtype="bf16", centres=50)
    c["dec_idx"] = np.array([5, P + 10, P + V - 1, P + 10, P + V + 7, 0, 39], dtype=np.int32)
    c["D"] = len(c["dec_idx"])
    k = oracle.keep_count(V, 0.2)
    step = GpuStep([c], [k], "bf16")
    S = step.importance()
    S_ref = oracle.importance(c["q"], c["k"], c["dec_idx"], P, V)
    check_scores(S[0], S_ref)
    kept, slot = step.select_topk()
    check_kept(kept[0], slot[0], S_ref, k)
    # and a long list (above the size whose logits are kept) with the same properties
    c["dec_idx"] = np.concatenate([np.arange(P + 100, P + 140), np.arange(0, 8), [P + 100, P + 100]]).astype(np.int32)
    c["D"] = len(c["dec_idx"])
    step = GpuStep([c], [k], "bf16")
    check_scores(step.importance()[0], oracle.importance(c["q"], c["k"], c["dec_idx"], P, V))


def test_one_token_merged_away_at_full_width():
    """keep_k = V - 1 at d = 4096: a single pruned row against V - 1 kept rows on the MFMA path."""
    P, V, O, H, dh = 4, 300, 6, 32, 128
    c = W.random_case(74, P + V + O, H * dh, H, P, V, 2, dtype="bf16", centres=20)
    step, S, kept, mout, stats = _chain([c], [V - 1], "bf16")
    assert mout["counts"][0].sum() == V and mout["counts"][0].max() == 2 and mout["y"][0].shape[0] == P + V - 1 + O


# ---- full-size workloads ---------------------------------------------------------------------------------
def test_llada_v_1024_full_chain():
    wl = W.WORKLOADS["llada_v_1024"]
    g = W.SampleGen(wl)
    s = g.step(32)
    k = oracle.keep_count(wl.V, 0.10)
    assert k == 103
    step, S, kept, mout, stats = _chain([s], [k], "bf16")
    assert mout["y"][0].shape[0] == 231
    q2, k2, v2 = g.proj.qkv(mout["y"][0])
    o = gpu_attend([(q2, k2, v2)], "bf16")[0]
    check_attend(o, q2, k2, v2, "bf16")
    # also the 263-token length quoted for this workload
    qkv = g.attention_inputs(263, 32)
    check_attend(gpu_attend([qkv], "bf16")[0], *qkv, "bf16")


@pytest.mark.parametrize("s_idx", [0, 5, 6, 16, 31])        # 5 | 6: the cosine tile height changes between them
def test_lavida_3645_sweep_steps_sampled(s_idx):
    wl = W.WORKLOADS["lavida_3645_sweep"]
    g = W.SampleGen(wl)
    sch = W.sweep_schedule(wl)[s_idx]
    s = g.step(sch["D"])
    k = oracle.keep_count(wl.V, sch["keep_ratio"])
    rng = np.random.default_rng(s_idx)
    step = GpuStep([s], [k], "bf16")
    S = step.importance(); kept, slot = step.select_topk(); mout = step.merge()
    pruned = np.setdiff1d(np.arange(wl.V), kept[0])
    rows = rng.choice(pruned, size=192, replace=False)
    st = check_full_sample(step, 0, S, kept, slot, mout, assign_rows=rows)
    n_m = wl.N - (wl.V - k)
    assert mout["y"][0].shape[0] == n_m
    # the benchmark's step calls the merge layer in one piece, with the keep ratio on the device: same kernels,
    # same launch shapes, so every output is that of the separate calls bit for bit
    S1, kept1, m1 = step.merge_layer([sch["keep_ratio"]])
    np.testing.assert_array_equal(S1[0], S[0])
    np.testing.assert_array_equal(kept1[0], kept[0])
    for key in m1:
        np.testing.assert_array_equal(m1[key][0], mout[key][0])
    qkv = g.attention_inputs(n_m, sch["D"])
    o = gpu_attend([qkv], "bf16")[0]
    check_attend(o, *qkv, "bf16", rows=rng.choice(n_m, size=48, replace=False))


def test_serving_shape_ragged_subset():
    wl = W.WORKLOADS["serving_b16"]
    proj = W.Projections(wl)
    draws = W.serving_draws(wl)[:3]
    samples = [W.SampleGen(wl, proj, seed=dr["seed"]).step(dr["D"]) for dr in draws]
    keeps = [oracle.keep_count(wl.V, dr["keep_ratio"]) for dr in draws]
    rng = np.random.default_rng(3)
    step = GpuStep(samples, keeps, "bf16")
    S = step.importance(); kept, slot = step.select_topk(); mout = step.merge()
    for b in range(len(samples)):
        pruned = np.setdiff1d(np.arange(wl.V), kept[b])
        check_full_sample(step, b, S, kept, slot, mout, assign_rows=rng.choice(pruned, size=96, replace=False))


def test_serving_shape_full_batch_of_16():
    """The whole ragged serving batch in one launch set (the configuration the kernels' batch mapping and
    the XCD-aware grids see in production): every sample's index outputs are checked for consistency, four
    samples (first, last, fewest kept, most deciders) are checked against the oracle stage by stage, and
    the attention over the 16 merged lengths is checked on sampled query rows."""
    wl = W.WORKLOADS["serving_b16"]
    proj = W.Projections(wl)
    draws = W.serving_draws(wl)
    gens = [W.SampleGen(wl, proj, seed=dr["seed"]) for dr in draws]
    samples = [g.step(dr["D"]) for g, dr in zip(gens, draws)]
    keeps = [oracle.keep_count(wl.V, dr["keep_ratio"]) for dr in draws]
    rng = np.random.default_rng(5)
    step = GpuStep(samples, keeps, "bf16")
    S = step.importance(); kept, slot = step.select_topk(); mout = step.merge()
    for b in range(wl.B):
        assert len(kept[b]) == keeps[b] and (np.diff(kept[b]) > 0).all()
        np.testing.assert_array_equal(np.where(slot[b] >= 0)[0], kept[b])
        assert mout["counts"][b].sum() == wl.V and mout["counts"][b].min() >= 1
        np.testing.assert_array_equal(mout["assign"][b][kept[b]], np.arange(keeps[b]))
        np.testing.assert_array_equal(np.bincount(mout["assign"][b], minlength=keeps[b]), mout["counts"][b])
        assert mout["y"][b].shape == (wl.N - (wl.V - keeps[b]), wl.d)
    detail = sorted({0, wl.B - 1, int(np.argmin(keeps)), int(np.argmax([dr["D"] for dr in draws]))})
    for b in detail:
        pruned = np.setdiff1d(np.arange(wl.V), kept[b])
        check_full_sample(step, b, S, kept, slot, mout, assign_rows=rng.choice(pruned, size=64, replace=False))
    qkv = [g.attention_inputs(wl.N - (wl.V - k), dr["D"]) for g, dr, k in zip(gens, draws, keeps)]
    outs = gpu_attend(qkv, "bf16")
    for b in detail[:3]:
        rows = rng.choice(qkv[b][0].shape[0], size=24, replace=False)
        check_attend(outs[b], *qkv[b], "bf16", rows=rows)


# ---- edge cases, determinism, error paths ---------------------------------------------------------------
def test_edge_counts():
    # k = 1 (everything merges into one token), D = 1, visual block at the very end
    c = W.random_case(31, 80, 2 * 128, 2, 10, 70, 1, dtype="bf16", centres=3)
    step, S, kept, mout, stats = _chain([c], [1], "bf16")
    assert mout["counts"][0][0] == 70 and mout["y"][0].shape[0] == 11
    # identical visual rows: every pruned token ties on all slots -> lowest slot takes all
    c2 = W.random_case(32, 60, 128, 1, 5, 50, 2, dtype="bf16", centres=1, noise=0.0)
    step, S, kept, mout, stats = _chain([c2], [5], "bf16")
    np.testing.assert_array_equal(mout["counts"][0], [46, 1, 1, 1, 1])
    # one slot with far more members than one staging pass of the scatter kernel holds (several windows,
    # windows that straddle the parts of the table scanned by different waves), in both merge modes
    c3 = W.random_case(33, 1530, 2 * 128, 2, 12, 1500, 4, dtype="bf16", centres=7)
    for mode in ("mean", "sum"):
        step, S, kept, mout, stats = _chain([c3], [1], "bf16", mode=mode)
        assert mout["counts"][0][0] == 1500 and mout["y"][0].shape[0] == 31
    c4 = W.random_case(34, 1210, 128, 1, 5, 1200, 2, dtype="bf16", centres=1, noise=0.0)
    step, S, kept, mout, stats = _chain([c4], [5], "bf16")
    np.testing.assert_array_equal(mout["counts"][0], [1196, 1, 1, 1, 1])


# ---- cosine taken on separate features (Section 4.4 compares keys while other rows are merged) --------
@pytest.mark.parametrize("dtype,d_sim", [("bf16", 256), ("bf16", 4 * 128 + 8), ("f32", 96)])
def test_merge_with_separate_similarity_features(dtype, d_sim):
    # d_sim = 256: MFMA path (split along the contraction, short sequence); 520: not a multiple of 64 -> generic path
    shapes = [(12, 500, 20, 0.3), (0, 260, 5, 0.6)]
    samples, keeps, sims = [], [], []
    for i, (P, V, O, keep) in enumerate(shapes):
        c = W.random_case(800 + i, P + V + O, 4 * 128, 4, P, V, 4, dtype=dtype, centres=max(4, V // 7))
        f = W.random_case(900 + i, P + V + O, d_sim, 1, P, V, 4, dtype=dtype, centres=max(4, V // 9))["x"]
        samples.append(c); keeps.append(oracle.keep_count(V, keep)); sims.append(f)
    rng = np.random.default_rng(9)
    kept = [np.sort(rng.choice(s["V"], size=k, replace=False)).astype(np.int32) for s, k in zip(samples, keeps)]
    out = GpuStep(samples, keeps, dtype).merge(kept, sim_rows=np.concatenate(sims))
    for b, s in enumerate(samples):
        check_assign(out["assign"][b], sims[b], s["vis_start"], s["V"], kept[b])          # routing follows `sim`
        check_merge({key: out[key][b] for key in out}, s["x"], s["vis_start"], s["V"], kept[b], dtype)   # payload is `x`


# ---- KV-cache variant (Section 4.4): one routing from the key cache, both caches aggregated ------------
@pytest.mark.parametrize("mode", ["mean", "sum"])
def test_merge_kv_ragged_batch(mode):
    shapes = [(64, 900, 0, 0.2), (20, 411, 0, 0.5), (0, 1300, 0, 0.1)]          # (prompt, visual, response, keep)
    samples, keeps, vrows = [], [], []
    for i, (P, V, O, keep) in enumerate(shapes):
        c = W.random_case(500 + i, P + V + O, 4 * 128, 4, P, V, 3, dtype="bf16", centres=max(4, V // 8))
        samples.append(c); keeps.append(oracle.keep_count(V, keep))
        vrows.append(W.round_to(np.random.default_rng(600 + i).standard_normal(c["x"].shape).astype(np.float32), "bf16"))
    step = GpuStep(samples, keeps, "bf16", B.D3TOM_MERGE_MEAN if mode == "mean" else B.D3TOM_MERGE_SUM)
    rng = np.random.default_rng(7)
    kept = [np.sort(rng.choice(s["V"], size=k, replace=False)).astype(np.int32) for s, k in zip(samples, keeps)]
    out = step.merge_kv(np.concatenate(vrows), kept)
    for b, s in enumerate(samples):
        check_assign(out["assign"][b], s["x"], s["vis_start"], s["V"], kept[b])
        # both caches against the oracle's aggregation run on the GPU's own routing
        check_merge({"y": out["y"][b], "assign": out["assign"][b], "counts": out["counts"][b], "src_pos": out["src_pos"][b]},
                    s["x"], s["vis_start"], s["V"], kept[b], "bf16", mode)
        check_merge({"y": out["v"][b], "assign": out["assign"][b], "counts": out["counts"][b], "src_pos": out["src_pos"][b]},
                    vrows[b], s["vis_start"], s["V"], kept[b], "bf16", mode)
    # the key half equals what d3tom_merge gives for the same rows and kept set (same kernels, same routing)
    ref = GpuStep(samples, keeps, "bf16", step.mode).merge(kept)
    for b in range(len(samples)):
        np.testing.assert_array_equal(ref["y"][b], out["y"][b])
        np.testing.assert_array_equal(ref["assign"][b], out["assign"][b])


# ---- decider bookkeeping on the device (Section 3.2) ----------------------------------------------------
def test_update_deciders_batch_and_chain_into_importance():
    M = 126336
    specs = [(300, 64, 9), (1152 - 64, 64, 5), (0, 1500, 4), (2688 - 256, 256, 2), (10, 1, 1)]     # (prefix, response, steps)
    trajs = [W.mask_trajectory(70 + i, p, r, t, mask_id=M) for i, (p, r, t) in enumerate(specs)]
    lens = [p + r for p, r, _ in specs]
    seq_off = torch.from_numpy(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)).cuda()
    nb = len(specs)
    for max_D, pick in ((256, 1), (16, 1), (256, 0)):       # pick: which transition of each trajectory (0 = the first)
        prev = np.concatenate([t[min(pick, len(t) - 2)] for t in trajs])
        cur = np.concatenate([t[min(pick, len(t) - 2) + 1] for t in trajs])
        dec_idx = torch.full((nb * max_D,), -7, dtype=torch.int32, device="cuda")
        dec_off = torch.full((nb + 1,), -7, dtype=torch.int32, device="cuda")
        dec_cnt = torch.full((nb,), -7, dtype=torch.int32, device="cuda")
        B.d3tom_update_deciders(torch.from_numpy(prev).cuda(), torch.from_numpy(cur).cuda(), M, seq_off, max_D,
                                dec_idx, dec_off, dec_cnt)
        torch.cuda.synchronize()
        off, cnt, idx = dec_off.cpu().numpy(), dec_cnt.cpu().numpy(), dec_idx.cpu().numpy()
        o = 0
        for b in range(nb):
            a0 = sum(lens[:b])
            ref = oracle.deciders(prev[a0:a0 + lens[b]], cur[a0:a0 + lens[b]], M)
            assert cnt[b] == len(ref) and off[b] == o
            np.testing.assert_array_equal(idx[o:o + min(len(ref), max_D)], ref[:max_D])
            o += min(len(ref), max_D)
        assert off[nb] == o
    # the device-built list feeds d3tom_importance directly and gives the scores of the host-built one
    c = W.random_case(90, 700, 4 * 128, 4, 30, 600, 12, dtype="bf16", centres=40)
    c["dec_idx"] = np.sort(c["dec_idx"])
    step = GpuStep([c], [60], "bf16")
    S_ref = step.importance()[0].copy()
    prev = np.full(700, 7, np.int32); cur = prev.copy()
    prev[c["dec_idx"]] = M
    so = torch.tensor([0, 700], dtype=torch.int32, device="cuda")
    step.lay.dec_idx.zero_()
    B.d3tom_update_deciders(torch.from_numpy(prev).cuda(), torch.from_numpy(cur).cuda(), M, so, 12,
                            step.lay.dec_idx, step.lay.dec_off, None)
    np.testing.assert_array_equal(step.importance()[0], S_ref)


def test_bitwise_determinism():
    c = W.random_case(41, 900, 4 * 128, 4, 30, 800, 12, dtype="bf16", centres=60)
    k = oracle.keep_count(800, 0.2)
    outs = []
    for _ in range(2):
        step = GpuStep([c], [k], "bf16")
        S = step.importance(); kept, slot = step.select_topk(); m = step.merge()
        outs.append((S[0].copy(), kept[0].copy(), m["y"][0].copy(), m["assign"][0].copy()))
    for a, b in zip(outs[0], outs[1]):
        np.testing.assert_array_equal(a, b)
    qkv = W.random_qkv(42, 333, 4, 128, "bf16")
    np.testing.assert_array_equal(gpu_attend([qkv], "bf16")[0], gpu_attend([qkv], "bf16")[0])


def test_error_statuses():
    c = W.random_case(51, 40, 128, 1, 4, 30, 2, dtype="bf16")
    step = GpuStep([c], [5], "bf16")
    lay0 = B.Layout([40], [4], [30], [[]], [5])                                # empty decider set
    with pytest.raises(B.D3tomError) as e:
        B.d3tom_importance(step.q, step.k, lay0, 0.1, step.scores, step.ws_imp)
    assert e.value.status == B.D3TOM_ERR_NO_DECIDERS
    with pytest.raises(B.D3tomError) as e:
        B.d3tom_importance(step.q, step.k, step.lay, 0.1, step.scores, B.workspace(256))
    assert e.value.status == B.D3TOM_ERR_WORKSPACE_TOO_SMALL
    with pytest.raises(B.D3tomError) as e:
        B.d3tom_merge(step.x, None, step.lay, step.kept_idx, 7, step.y, None, None, None, step.ws_merge)
    assert e.value.status == B.D3TOM_ERR_INVALID_ARG
    q = torch.zeros((8, 1, 300), dtype=torch.float32, device="cuda")           # head size above the limit
    cu = torch.tensor([0, 8], dtype=torch.int32, device="cuda")
    with pytest.raises(B.D3tomError) as e:
        B.d3tom_attend(q, q, q, cu, 8, 1.0, torch.zeros_like(q))
    assert e.value.status == B.D3TOM_ERR_UNSUPPORTED
    q2 = torch.zeros((8, 1, 64), dtype=torch.bfloat16, device="cuda")
    for bad_scale in (0.0, -0.125, float("inf"), float("nan")):                # the logit scale must be finite and > 0
        with pytest.raises(B.D3tomError) as e:
            B.d3tom_attend(q2, q2, q2, cu, 8, bad_scale, torch.zeros_like(q2))
        assert e.value.status == B.D3TOM_ERR_INVALID_ARG
        with pytest.raises(B.D3tomError) as e:
            B.d3tom_importance(step.q, step.k, step.lay, bad_scale, step.scores, step.ws_imp)
        assert e.value.status == B.D3TOM_ERR_INVALID_ARG
    torch.cuda.synchronize()
