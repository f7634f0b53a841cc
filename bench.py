#!/usr/bin/env python3
"""Benchmark of the D3ToM hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input already resident in HBM:
d3tom_importance -> d3tom_select_topk -> d3tom_merge -> d3tom_attend (the attention runs on
pre-generated q/k/v of the merged length; the projection between merge and attention is not on the path).

Prints ONE JSON line: denoise steps/s of the workload the metric is quoted on (the 3645-visual-token
LaViDa-like sweep; the 1024-token LLaDA-V-like step and the batched serving shape are reported beside it
under "also"), the roofline figure of the dominant kernel (HIP-event timings taken live, algorithmic bytes /
flops from the shapes), and the CPU oracle timed on the host cores on a bounded sample of the same workload.

Which steps are timed.  The sweep has 32 steps of growing cost (deciders 2..64, keep ratio 0.10..0.50).  The K
timed steps always cover it evenly: whole sweeps in order while K allows, and a remainder (or a K below 32)
spread evenly over the sweep, so that the mean step time estimates the mean over the whole sweep whatever K
is.  The indices are reported under "timed_steps".
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np
import torch

PEAK_HBM_GBS = 8000.0          # MI355X HBM3E, published
PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published


def build_steps(wl_name: str):
    """Generate every step of the workload on the host and upload it.  Returns (workload, list of step dicts)."""
    from paper_2511_12280_amd import binding as B
    from paper_2511_12280_amd import workloads as W
    wl = W.WORKLOADS[wl_name]
    steps = []
    if wl.B == 1:
        g = W.SampleGen(wl)
        for sch in W.sweep_schedule(wl):
            s = g.step(sch["D"])
            k = B.d3tom_keep_count(wl.V, sch["keep_ratio"])
            n_m = wl.N - (wl.V - k)
            steps.append(dict(samples=[s], keeps=[k], attn=[g.attention_inputs(n_m, sch["D"])], sch=sch))
    else:
        proj = W.Projections(wl)
        samples, keeps, attn = [], [], []
        for dr in W.serving_draws(wl):
            g = W.SampleGen(wl, proj, seed=dr["seed"])
            samples.append(g.step(dr["D"]))
            k = B.d3tom_keep_count(wl.V, dr["keep_ratio"])
            keeps.append(k)
            attn.append(g.attention_inputs(wl.N - (wl.V - k), dr["D"]))
        steps.append(dict(samples=samples, keeps=keeps, attn=attn, sch=dict(step=0)))
    dev = []
    for st in steps:
        sm = st["samples"]
        lay = B.Layout([s["N"] for s in sm], [s["vis_start"] for s in sm], [s["V"] for s in sm],
                       [s["dec_idx"] for s in sm], st["keeps"])
        cat = lambda key: np.concatenate([s[key] for s in sm], axis=0)
        d = dict(lay=lay, q=B.to_device(cat("q"), wl.dtype), k=B.to_device(cat("k"), wl.dtype),
                 x=B.to_device(cat("x"), wl.dtype),
                 qa=B.to_device(np.concatenate([a[0] for a in st["attn"]]), wl.dtype),
                 ka=B.to_device(np.concatenate([a[1] for a in st["attn"]]), wl.dtype),
                 va=B.to_device(np.concatenate([a[2] for a in st["attn"]]), wl.dtype),
                 cu=torch.from_numpy(np.concatenate([[0], np.cumsum(lay.Nm)]).astype(np.int32)).cuda(),
                 host=st)
        dev.append(d)
    return wl, dev


class Runner:
    """Shared output buffers + workspaces, and the launches of one step: the merge layer in one call
    (d3tom_merge_layer, kept counts computed on the device from the keep ratios) followed by the attention;
    with one_call=False the four separate entry points instead."""

    def __init__(self, wl, dev, one_call=True):
        from paper_2511_12280_amd import binding as B
        self.B, self.wl, self.dev, self.one_call = B, wl, dev, one_call
        mx = lambda f: max(f(d["lay"]) for d in dev)
        tdt = torch.float32 if wl.dtype == "f32" else torch.bfloat16
        i32 = lambda m: torch.zeros(m, dtype=torch.int32, device="cuda")
        nb, mN, mV, mD = mx(lambda l: l.B), mx(lambda l: l.max_N), mx(lambda l: l.max_V), mx(lambda l: l.max_D)
        self.scores = torch.zeros(mx(lambda l: l.sum_V), dtype=torch.float32, device="cuda")
        self.kept = i32(nb * mV)
        self.slot = i32(mx(lambda l: l.sum_V))
        self.y = torch.zeros((mx(lambda l: l.sum_N), wl.d), dtype=tdt, device="cuda")
        self.counts = i32(nb * mV)
        self.src = i32(mx(lambda l: l.sum_N))
        self.o = torch.zeros((mx(lambda l: l.sum_Nm), wl.H, wl.dh), dtype=tdt, device="cuda")
        self.ws_imp = B.workspace(B.d3tom_workspace_bytes(B.D3TOM_OP_IMPORTANCE, nb, mN, mV, wl.H, wl.dh, mD))
        self.ws_merge = B.workspace(B.d3tom_workspace_bytes(B.D3TOM_OP_MERGE, nb, mN, mV, wl.H, wl.dh, mD))
        self.scale = 1.0 / float(np.sqrt(wl.dh))
        # the one-call path: keep ratios on the device, the kept counts and offsets are outputs
        self.keep_k, self.kept_off, self.out_off = i32(nb), i32(nb + 1), i32(nb + 1)
        self.ws_layer = B.workspace(B.d3tom_merge_layer_workspace_bytes(nb, mN, mV, wl.H, wl.dh, mD))
        self.ratios = []
        for d in dev:
            h = d["host"]
            r = [h["sch"]["keep_ratio"]] if wl.B == 1 else [k / s["V"] for k, s in zip(h["keeps"], h["samples"])]
            self.ratios.append(torch.tensor(r, dtype=torch.float64, device="cuda"))

    def step(self, i: int):
        B, d = self.B, self.dev[i]
        lay = d["lay"]
        if self.one_call:
            # tight host bounds on the kept counts: the launch shapes are those of the separate calls
            B.d3tom_merge_layer(d["q"], d["k"], d["x"], None, lay, self.scale, self.ratios[i], min(lay.keep), max(lay.keep),
                                B.D3TOM_MERGE_MEAN, self.scores, self.keep_k, self.kept_off, self.kept, self.out_off,
                                self.y, None, self.counts, self.src, self.ws_layer)
        else:
            B.d3tom_importance(d["q"], d["k"], lay, self.scale, self.scores, self.ws_imp)
            B.d3tom_select_topk(self.scores, lay, self.kept, self.slot)
            B.d3tom_merge(d["x"], None, lay, self.kept, B.D3TOM_MERGE_MEAN, self.y, None, self.counts, self.src, self.ws_merge)
        B.d3tom_attend(d["qa"], d["ka"], d["va"], d["cu"], lay.max_Nm, self.scale, self.o)


def algorithmic(wl, lay):
    """Per-kernel algorithmic bytes and flops of ONE launch for this batch layout (what the method must
    move / compute: K once per sweep, the visual rows once, input + output rows once, 4 n^2 d for attention)."""
    eb = 4 if wl.dtype == "f32" else 2
    d = wl.d
    out = {k: [0.0, 0.0] for k in ("imp_stats", "imp_scores", "imp_finish", "topk_select", "merge_norms",
                                   "cos_argmax", "merge_assign", "merge_scatter", "attend")}
    for N, V, k, D, Nm in zip(lay.N, lay.V, lay.keep, lay.D, lay.Nm):
        M = V - k
        out["imp_stats"][0] += (N + D) * d * eb;            out["imp_stats"][1] += 2.0 * D * N * d
        out["imp_scores"][0] += (V + D) * d * eb + 4 * V;   out["imp_scores"][1] += 2.0 * D * V * d
        out["imp_finish"][0] += 4 * V * (wl.H + 1)
        out["topk_select"][0] += 4 * V + 4 * k + 4 * V
        out["merge_norms"][0] += k * d * eb + 4 * k
        out["cos_argmax"][0] += V * d * eb;                 out["cos_argmax"][1] += 2.0 * M * k * d
        out["merge_assign"][0] += 8 * M * max(1, -(-k // 128)) + 8 * V
        out["merge_scatter"][0] += (N + Nm) * d * eb + 4 * V
        out["attend"][0] += 4 * Nm * d * eb;                out["attend"][1] += 4.0 * Nm * Nm * d
    return out


def step_order(n: int, K: int):
    """Indices of the K timed steps of an n-step workload: whole passes in order, the remainder spread evenly."""
    full, rest = divmod(K, n)
    order = list(range(n)) * full
    order += [min(n - 1, int((i + 0.5) * n / rest)) for i in range(rest)]
    return order


def run_workload(wl_name: str, steps: int, warmup: int, cpu_baseline: bool, one_call: bool = True):
    from paper_2511_12280_amd import binding as B
    t0 = time.time()
    wl, dev = build_steps(wl_name)
    gen_s = time.time() - t0
    r = Runner(wl, dev, one_call)
    n = len(dev)
    order = step_order(n, steps)
    # untimed: every step once (first-use set-up, inputs touched), repeated until the device has been busy for a
    # quarter of a second: after the host-side input generation its clocks take that long to come up, and a short
    # timed region (K = 20 steps is 2.7 ms) would otherwise be measured on the ramp
    t_ramp = time.perf_counter()
    while True:
        for i in range(n):
            r.step(i)
        torch.cuda.synchronize()
        if time.perf_counter() - t_ramp > 0.25:
            break
    for i in step_order(n, warmup):
        r.step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in order:
        r.step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    # the same K steps again with HIP events around every kernel launch
    B.d3tom_profile_enable(True)
    for i in order:
        r.step(i)
    torch.cuda.synchronize()
    prof = B.d3tom_profile_collect()
    B.d3tom_profile_enable(False)
    alg = {k: [0.0, 0.0] for k in prof}
    for i in order:
        a = algorithmic(wl, dev[i]["lay"])
        for k in alg:
            by, fl = a.get(k, (0.0, 0.0))
            alg[k][0] += by; alg[k][1] += fl
    kernels = {}
    for k, (ms, calls) in prof.items():
        if calls == 0:
            continue
        by, fl = alg[k]
        t = ms * 1e-3
        hbm_t, mfma_t = by / (PEAK_HBM_GBS * 1e9), fl / (PEAK_BF16_TFLOPS * 1e12)
        bound = "mfma" if mfma_t > hbm_t else "hbm"
        ach = (fl / t / 1e12) if bound == "mfma" else (by / t / 1e9)
        peak = PEAK_BF16_TFLOPS if bound == "mfma" else PEAK_HBM_GBS
        kernels[k] = dict(avg_us=round(ms * 1e3 / calls, 3), launches=calls, bound=bound, achieved=round(ach, 2),
                          peak=peak, unit="TFLOP/s" if bound == "mfma" else "GB/s", frac=round(ach / peak, 4),
                          share=0.0)
    tot_ms = sum(ms for ms, c in prof.values())
    for k in kernels:
        kernels[k]["share"] = round(prof[k][0] / tot_ms, 4)
    dom = max(kernels, key=lambda k: prof[k][0])
    # The event brackets add about 2 us per launch, so the bracketed times sum to more than the step takes
    # un-bracketed.  The split of the step into merge layer and attention uses the bracketed SHARES applied to
    # the un-bracketed step time: the two figures add up to ms_per_step.
    us_per_step = elapsed * 1e6 / steps
    attend_share = prof["attend"][0] / tot_ms
    res = dict(workload=wl_name, steps_per_s=steps / elapsed, ms_per_step=elapsed * 1e3 / steps,
               merge_layer_us=round(us_per_step * (1.0 - attend_share), 2), attend_us=round(us_per_step * attend_share, 2),
               kernels=kernels, dominant=dom, gen_s=round(gen_s, 1), timed_steps=order)
    if cpu_baseline:
        res["cpu_baseline"] = oracle_baseline(wl, dev)
    return wl, res


def run_separate_calls(wl_name: str, steps: int, warmup: int):
    """The same steps through the four separate entry points (importance, selection, merge, attention) with the
    kept counts on the host: what a caller pays who needs a host decision between the stages."""
    wl, dev = build_steps(wl_name)
    r = Runner(wl, dev, one_call=False)
    n = len(dev)
    t_ramp = time.perf_counter()
    while True:                                  # as in run_workload: untimed passes until the clocks are up
        for i in range(n):
            r.step(i)
        torch.cuda.synchronize()
        if time.perf_counter() - t_ramp > 0.25:
            break
    for i in step_order(n, warmup):
        r.step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in step_order(n, steps):
        r.step(i)
    torch.cuda.synchronize()
    el = time.perf_counter() - t0
    return dict(steps_per_s=round(steps / el, 2), ms_per_step=round(el * 1e3 / steps, 4))


def run_kv_cache(wl_name: str, steps: int, warmup: int):
    """d3tom_merge_kv (Section 4.4) on a cache of the workload's prompt + visual rows: key cache = the
    synthetic hidden rows (they carry the cluster structure the routing sees), value cache = N(0,1) rows,
    kept sets drawn at the sweep's keep ratios.  One launch set per step; merge-only time."""
    from paper_2511_12280_amd import binding as B
    from paper_2511_12280_amd import workloads as W
    wl = W.WORKLOADS[wl_name]
    g = W.SampleGen(wl)
    s = g.step(32)
    n = wl.P + wl.V
    rng = np.random.default_rng(11)
    kc = B.to_device(s["x"][:n], wl.dtype)
    vc = B.to_device(W.round_to(rng.standard_normal((n, wl.d)).astype(np.float32), wl.dtype), wl.dtype)
    lays, kepts = [], []
    for sch in W.sweep_schedule(wl):
        k = B.d3tom_keep_count(wl.V, sch["keep_ratio"])
        lays.append(B.Layout([n], [wl.P], [wl.V], [[0]], [k]))
        kepts.append(torch.from_numpy(np.sort(rng.choice(wl.V, size=k, replace=False)).astype(np.int32)).cuda())
    mx = max(l.sum_Nm for l in lays)
    tdt = torch.float32 if wl.dtype == "f32" else torch.bfloat16
    ko = torch.zeros((mx, wl.d), dtype=tdt, device="cuda"); vo = torch.zeros_like(ko)
    counts = torch.zeros(wl.V, dtype=torch.int32, device="cuda")
    ws = B.workspace(B.d3tom_workspace_bytes(B.D3TOM_OP_MERGE, 1, n, wl.V, wl.H, wl.dh, 1))
    def step(j):
        B.d3tom_merge_kv(kc, vc, lays[j], kepts[j], B.D3TOM_MERGE_MEAN, ko, vo, None, counts, None, ws)
    order = step_order(len(lays), steps)
    for i in list(range(len(lays))) + step_order(len(lays), warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in order:
        step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    B.d3tom_profile_enable(True)
    for i in order:
        step(i)
    torch.cuda.synchronize()
    prof = B.d3tom_profile_collect()
    B.d3tom_profile_enable(False)
    return dict(merge_kv_us=round(elapsed * 1e6 / steps, 2), cache_rows=n,
                kernels={k: round(ms * 1e3 / c, 3) for k, (ms, c) in prof.items() if c})


def time_attention(wl_name: str, n_tokens: int, steps: int, warmup: int) -> float:
    """d3tom_attend alone on sequences of n_tokens of the workload's shape (several input sets, so K / V come
    from HBM as in the step); microseconds per call."""
    from paper_2511_12280_amd import binding as B
    from paper_2511_12280_amd import workloads as W
    wl = W.WORKLOADS[wl_name]
    g = W.SampleGen(wl)
    sets = [tuple(B.to_device(a, wl.dtype) for a in g.attention_inputs(n_tokens, 32)) for _ in range(8)]
    tdt = torch.float32 if wl.dtype == "f32" else torch.bfloat16
    o = torch.zeros((n_tokens, wl.H, wl.dh), dtype=tdt, device="cuda")
    cu = torch.tensor([0, n_tokens], dtype=torch.int32, device="cuda")
    scale = 1.0 / float(np.sqrt(wl.dh))
    def step(i):
        q, k, v = sets[i % len(sets)]
        B.d3tom_attend(q, k, v, cu, n_tokens, scale, o)
    # calls of ~10 us: a long warm-up, or the clocks are still ramping after the host-side input generation
    warmup, steps = max(warmup, 1000), max(steps, 500)
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e6 / steps


def run_cosine_cold_warm(reps: int = 6):
    """The cosine kernel of d3tom_merge alone at 3645 visual rows of 4096 bf16, over kept counts, in three memory
    states: the same tensor as the previous call (rows in the memory-side cache), a different tensor every call
    (rows cold in HBM, as in the sweep), and a different tensor read front to back just before the call.
    Microseconds per launch from the library's HIP-event brackets; prints a table (the evidence behind the
    row-streaming workgroups of the one-call merge layer)."""
    from paper_2511_12280_amd import binding as B
    V, d, NX = 3645, 4096, 12
    rng = np.random.default_rng(5)
    gen = torch.Generator(device="cuda"); gen.manual_seed(5)
    xs = [torch.randn((V, d), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16) for _ in range(NX)]
    y = torch.empty((V, d), dtype=torch.bfloat16, device="cuda")
    counts = torch.empty(V, dtype=torch.int32, device="cuda")
    src = torch.empty(V, dtype=torch.int32, device="cuda")
    ws = B.workspace(B.d3tom_workspace_bytes(B.D3TOM_OP_MERGE, 1, V, V, 32, 128, 64))
    rows = []
    for k in (365, 512, 647, 694, 741, 768, 788, 882, 1023, 1030, 1280, 1500, 1822):
        lay = B.Layout([V], [0], [V], [[0]], [k])
        kept = torch.from_numpy(np.sort(rng.choice(V, k, replace=False)).astype(np.int32)).cuda()
        res = {}
        for state in ("same_tensor", "cold", "read_before"):
            def call(i):
                x = xs[0] if state == "same_tensor" else xs[i % NX]
                if state == "read_before":
                    x.view(torch.int32).sum()
                B.d3tom_merge(x, None, lay, kept, B.D3TOM_MERGE_MEAN, y, None, counts, src, ws)
            for i in range(3):
                call(i)
            torch.cuda.synchronize()
            B.d3tom_profile_enable(True)
            for i in range(reps):
                call(3 + i)
            torch.cuda.synchronize()
            prof = B.d3tom_profile_collect()
            B.d3tom_profile_enable(False)
            res[state] = prof["cos_argmax"][0] * 1e3 / prof["cos_argmax"][1]
        rows.append((k, res))
    print("cosine kernel of d3tom_merge, 3645 visual rows x 4096 bf16, microseconds per launch (HIP events around the launch)")
    print(f"{'kept':>6s} {'pruned':>7s} {'same tensor':>12s} {'cold':>8s} {'read before':>12s}")
    for k, r in rows:
        print(f"{k:6d} {V - k:7d} {r['same_tensor']:12.1f} {r['cold']:8.1f} {r['read_before']:12.1f}")


def run_stack(traj_repeats: int = 1):
    """Whole denoising trajectory through the 32-block stack (the full-stack configuration): T steps, each
    = decider update on the device, embedding of the current response tokens (one row gather, plumbing),
    d3tom_stack_step.  Step 0 has no deciders and runs unmerged; every later step merges inside block l*.
    Which response positions are revealed when comes from the synthetic scheduler (no decoding head)."""
    from paper_2511_12280_amd import binding as B
    from paper_2511_12280_amd import workloads as W
    cfg = W.STACK_3645
    L, d, H, F, P, V, O, T = (cfg[k] for k in ("L", "d", "H", "F", "P", "V", "O", "T"))
    N = P + V + O
    keep_k = B.d3tom_keep_count(V, cfg["keep_ratio"])
    inp = W.stack_device_inputs(cfg)
    arr = B.block_weights(inp["blocks"])
    states = torch.from_numpy(np.stack(W.mask_trajectory(cfg["seed"], P + V, O, T, cfg["mask_id"]))).cuda()   # [T+1, N]
    seq_off = torch.tensor([0, N], dtype=torch.int32, device="cuda")
    dec_idx = torch.zeros(B.D3TOM_MAX_DECIDERS, dtype=torch.int32, device="cuda")
    dec_off = torch.zeros(2, dtype=torch.int32, device="cuda")
    dec_count = torch.zeros(1, dtype=torch.int32, device="cuda")
    ws = B.workspace(B.d3tom_stack_workspace_bytes(N, d, H, F, V, B.D3TOM_MAX_DECIDERS))
    x = inp["x"].clone()
    y = torch.zeros(N, d, dtype=torch.bfloat16, device="cuda")
    # embedding rows of the response positions: one table with the [MASK] row appended, and per state the row
    # index of every response position (the scheduler's output in the form the gather takes)
    table = torch.cat([inp["table"], inp["mask_vec"][None, :]], dim=0)
    resp_ids = states[:, P + V:].long()
    emb_idx = torch.where(resp_ids == cfg["mask_id"], torch.full_like(resp_ids, cfg["table_rows"]), resp_ids % cfg["table_rows"])
    x_resp = x[P + V:]                                     # view of the response rows of x

    def step(s: int) -> int:
        cur = states[s]
        D = 0
        if s > 0:
            B.d3tom_update_deciders(states[s - 1], cur, cfg["mask_id"], seq_off, B.D3TOM_MAX_DECIDERS, dec_idx, dec_off, dec_count)
            D = min(int(dec_count.item()), B.D3TOM_MAX_DECIDERS)       # 4 bytes back to the host: the launch sizes need it
        torch.index_select(table, 0, emb_idx[s], out=x_resp)
        return B.d3tom_stack_step(x, H, F, arr, L, cfg["merge_layer"], dec_idx, D, P, V, keep_k, B.D3TOM_MERGE_MEAN,
                                  cfg["eps"], cfg["theta"], y, ws)

    step(0); step(1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(traj_repeats):
        for s in range(T):
            n_out = step(s)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    def timed(s, reps):
        torch.cuda.synchronize(); t = time.perf_counter()
        for _ in range(reps):
            step(s)
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3 / reps
    first_ms, merged_ms = timed(0, 3), timed(T // 2, 8)
    B.d3tom_profile_enable(True)
    step(T // 2)
    torch.cuda.synchronize()
    prof = B.d3tom_profile_collect()
    B.d3tom_profile_enable(False)
    # algorithmic flops of the projections of one merged step: 4 n d^2 + 3 n d F per block part at its length
    Nm = N - (V - keep_k)
    l_star = cfg["merge_layer"]
    attn_proj = lambda n: 2.0 * n * d * 4 * d
    ffn_proj = lambda n: 2.0 * n * d * 3 * F
    lin_flops = l_star * attn_proj(N) + (l_star - 1) * ffn_proj(N) + (L - l_star) * attn_proj(Nm) + (L - l_star + 1) * ffn_proj(Nm)
    lin_ms = prof["linear"][0]
    tf = lin_flops / (lin_ms * 1e-3) / 1e12
    # the paper's cost model (Section 4.3) for the same step: its l* counts the full layers before the split one
    alpha = 1.0 - keep_k / V
    mf = lambda a, T_: B.d3tom_model_flops(a, l_star - 1, L, T_, V, P, O, d, F)
    model_full, model_merged = mf(0.0, 1), mf(alpha, 2) - mf(alpha, 1)
    return {
        "workload": f"{cfg['name']}: {L} blocks, hidden {d}, {H}x{d // H} heads, SwiGLU {F}, {V} visual + {P} prompt + {O} response "
                    f"tokens, merge inside block {l_star} at keep ratio {cfg['keep_ratio']} ({N} -> {Nm} tokens), T={T}",
        "steps_per_s": round(traj_repeats * T / elapsed, 2), "ms_per_step": round(elapsed * 1e3 / (traj_repeats * T), 3),
        "first_step_unmerged_ms": round(first_ms, 3), "merged_step_ms": round(merged_ms, 3),
        "speedup_of_a_merged_step": round(first_ms / merged_ms, 2),
        "cost_model_flops_ratio_unmerged_over_merged": round(model_full / model_merged, 2), "out_rows": int(n_out),
        "roofline": {"kernel": "linear", "bound": "mfma", "achieved": round(tf, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(tf / PEAK_BF16_TFLOPS, 4), "calls_per_step": prof["linear"][1],
                     "total_us_per_step": round(lin_ms * 1e3, 1)},
        "kernels_us_per_step": {k: round(ms * 1e3, 1) for k, (ms, c) in prof.items() if c},
    }


def oracle_baseline(wl, dev):
    """The fp64 oracle, as it stands, on the host cores: whole steps of the workload (all five stages),
    taken in bit-reversed order (0, 16, 8, 24, ...) so that whatever number of steps fits into about 12 s of CPU
    time is spread evenly over the sweep; every sampled step counts once, like every step of the sweep does in
    the GPU figure, so the sample mean estimates the same sweep mean."""
    import oracle
    order = sorted(range(len(dev)), key=lambda i: (bin(i)[::-1], i))     # spread over the sweep, step 0 first
    done, spent, n_steps = [], 0.0, 0.0
    for i in order:
        st = dev[i]["host"]
        t0 = time.perf_counter()
        s, k, (qa, ka, va) = st["samples"][0], st["keeps"][0], st["attn"][0]
        oracle.merge_layer(s["q"], s["k"], s["x"], s["dec_idx"], s["vis_start"], s["V"], k)
        oracle.attend(qa, ka, va)
        t = time.perf_counter() - t0
        spent += t
        n_steps += 1.0 / len(st["samples"])       # batched workload: one sample is 1/B of a step
        done.append(i)
        if spent >= 12.0:
            break
    return dict(value=round(n_steps / spent, 4), unit="steps/s", cores=oracle.threads(), kind="oracle",
                sample=f"{len(done)} of {len(dev)} steps of the workload, spread evenly over it (indices {sorted(done)}), "
                       f"each weighted once, first sample of each, all five stages, {spent:.1f} s of oracle time")


TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "lavida_3645_sweep_hbm_traffic.txt")
KERNEL_OF_SYMBOL = (("imp_stats", "imp_stats"), ("imp_scores", "imp_scores"), ("imp_finish", "imp_finish"), ("topk_select", "topk_select"),
                    ("merge_norms", "merge_norms"), ("cos_argmax", "cos_argmax"), ("cos_reduce", "cos_reduce"),
                    ("merge_scatter", "merge_scatter"), ("attend", "attend"))


def measured_traffic(wl_name: str):
    """HBM bytes per launch (fetch + write) of every kernel from the rocprofv3 --pmc summary kept under profiles/
    (counters cannot be read from inside this process): {kernel: bytes}, launch-weighted over a kernel's template
    variants, plus a note saying where the figures come from.  None when there is no summary for the workload."""
    import re
    if wl_name != "lavida_3645_sweep" or not os.path.exists(TRAFFIC_PROFILE):
        return None, "no rocprofv3 counter summary for this workload under profiles/"
    acc = {}
    for line in open(TRAFFIC_PROFILE):
        m = re.match(r"^(\S.*?)\s+(\d+)\s+([0-9.]+)\s+([0-9.]+)\s*$", line)
        if not m:
            continue
        sym, launches, fetch, write = m.group(1), int(m.group(2)), float(m.group(3)), float(m.group(4))
        for prefix, name in KERNEL_OF_SYMBOL:
            if sym.startswith(prefix):
                b, n = acc.get(name, (0.0, 0))
                acc[name] = (b + (fetch + write) * 1e6 * launches, n + launches)
    out = {k: b / n for k, (b, n) in acc.items() if n}
    note = "from profiles/lavida_3645_sweep_hbm_traffic.txt (two rocprofv3 --pmc runs over whole sweeps), not measured in this run"
    # the summary names the kernel sources it was measured on (a digest); say whether they are the current ones
    from paper_2511_12280_amd.build import source_digest
    m = re.search(r"kernel sources digest: ([0-9a-f]+)", open(TRAFFIC_PROFILE).read())
    if m is None:
        note += "; the summary does not say which sources it was measured on"
    elif m.group(1) != source_digest():
        note += "; the kernel sources have changed since the summary was taken"
    else:
        note += ", on the current kernel sources"
    return out, note


# The paper's own measurement at the sweep's first keep ratio, as context (another machine, a whole model on a
# benchmark this build does not have): Table 2, D3ToM keeping 10 % of the visual tokens.
PAPER_CONTEXT = {"source": "Table 2, D3ToM, 10 % of the visual tokens kept, LaViDa-LLaDA-8B on LLaVA-Bench, T = 32",
                 "hardware": "NVIDIA A6000", "wall_clock_vs_unmerged": 0.426, "theoretical_flops_vs_unmerged": 0.302,
                 "wall_clock_s": 492.70, "unmerged_wall_clock_s": 1156.65}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=128)
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--workload", default="lavida_3645_sweep")
    ap.add_argument("--also", default="llada_v_1024,serving_b16", help="workloads reported beside the first ('' = none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stack", action="store_true", help="skip the full 32-block stack trajectory")
    ap.add_argument("--stack-only", action="store_true",
                    help="run only the 32-block stack trajectory and print its record (for profiling that part alone)")
    ap.add_argument("--cosine-cold-warm", action="store_true",
                    help="time the cosine kernel alone with its rows cached / cold / read just before, print a table and exit")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy, the known-size reference for HBM counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the path is a single-GPU kernel chain (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    if args.calibrate_copy:
        a = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b
    if args.cosine_cold_warm:
        run_cosine_cold_warm()
        return
    if args.stack_only:
        print(json.dumps(run_stack()))
        return
    wl, res = run_workload(args.workload, args.steps, args.warmup, not args.no_cpu_baseline)
    dom = res["kernels"][res["dominant"]]
    traffic, traffic_note = measured_traffic(wl.name)
    line = {
        "metric": "denoise steps/sec of the hot path (merge layer + bidirectional attention over the merged sequence)",
        "value": round(res["steps_per_s"], 2), "unit": "steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(res["ms_per_step"], 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.V} visual + {wl.P} prompt + {wl.O} response tokens, hidden {wl.d}, "
                               f"{wl.H}x{wl.dh} heads, batch {wl.B}, {wl.note}", "timed": "inputs resident in HBM",
                   "calls_per_step": "d3tom_merge_layer (keep ratios on the device) + d3tom_attend",
                   "timed_steps": res["timed_steps"]},
        "merge_layer_us": res["merge_layer_us"], "attend_us": res["attend_us"],
        "roofline": {"kernel": res["dominant"], "bound": dom["bound"], "achieved": dom["achieved"], "peak": dom["peak"],
                     "unit": dom["unit"], "frac": dom["frac"],
                     "traffic": (traffic or {}).get(res["dominant"]), "traffic_source": traffic_note, "avg_us": dom["avg_us"]},
        "kernels": res["kernels"],
        "paper_context": PAPER_CONTEXT,
    }
    if traffic:
        line["traffic_per_launch"] = {k: round(v) for k, v in traffic.items()}
    if "cpu_baseline" in res:
        line["cpu_baseline"] = res["cpu_baseline"]
    also = [a for a in args.also.split(",") if a]
    if also:
        line["also"] = {}
    for name in also:
        _, r2 = run_workload(name, args.steps, args.warmup, False)
        d2 = r2["kernels"][r2["dominant"]]
        line["also"][name] = {"steps_per_s": round(r2["steps_per_s"], 2), "ms_per_step": round(r2["ms_per_step"], 4),
                              "merge_layer_us": r2["merge_layer_us"], "attend_us": r2["attend_us"],
                              "roofline": {"kernel": r2["dominant"], "bound": d2["bound"], "achieved": d2["achieved"],
                                           "peak": d2["peak"], "unit": d2["unit"], "frac": d2["frac"]},
                              "kernels": r2["kernels"]}
        if name == "llada_v_1024":
            # the workload text quotes 263 tokens after the merge, its own counts give 231 (timed above): both lengths
            line["also"][name]["attend_alone_us"] = {str(n): round(time_attention(name, n, args.steps, args.warmup), 2)
                                                     for n in (231, 263)}
    if also:
        line["also"]["kv_cache_of_" + args.workload] = run_kv_cache(args.workload, args.steps, args.warmup)
        line["also"]["separate_calls_" + args.workload] = run_separate_calls(args.workload, args.steps, args.warmup)
        if not args.no_stack:
            line["also"]["denoise_stack_3645"] = run_stack()
    print(json.dumps(line))


if __name__ == "__main__":
    main()
