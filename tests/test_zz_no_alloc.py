"""d3tom_importance_static (the entry point that allocates nothing: its scratch memory is a static device
array inside the library) against d3tom_importance on the same inputs, through the C ABI."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2511_12280_amd import workloads as W

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from paper_2511_12280_amd import binding as B


def _both(case):
    lay = B.Layout([case["N"]], [case["vis_start"]], [case["V"]], [case["dec_idx"]], [1])
    q, k = B.to_device(case["q"], "bf16"), B.to_device(case["k"], "bf16")
    H, dh = q.shape[1], q.shape[2]
    scale = 1.0 / np.sqrt(dh)
    ref = torch.full((case["V"],), -1.0, dtype=torch.float32, device="cuda")
    out = torch.full((case["V"],), -2.0, dtype=torch.float32, device="cuda")
    ws = B.workspace(B.d3tom_workspace_bytes(B.D3TOM_OP_IMPORTANCE, 1, lay.max_N, lay.max_V, H, dh, lay.max_D))
    B.d3tom_importance(q, k, lay, scale, ref, ws)
    torch.cuda.synchronize()
    # torch's caching allocator counts every allocation request it serves: none may come from this call
    before = torch.cuda.memory_stats().get("allocation.all.allocated", 0)
    B.d3tom_importance_static(q, k, lay, scale, out)
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats().get("allocation.all.allocated", 0) == before
    return ref.cpu().numpy(), out.cpu().numpy()


def test_static_scratch_entry_point_matches_the_workspace_one_twice_in_a_row():
    # two calls in a row on the same GPU, the second with a smaller input: the static array still holds
    # the first call's partial results, and none of them may leak into the second call's scores
    big = W.random_case(61, 1500, 4 * 128, 4, 40, 1400, 37, dtype="bf16", centres=50)
    small = W.random_case(62, 300, 4 * 128, 4, 9, 260, 5, dtype="bf16", centres=20)
    for case in (big, small):
        ref, out = _both(case)
        assert np.isfinite(ref).all() and ref.min() >= 0.0
        np.testing.assert_array_equal(out, ref)          # same kernels, same order of operations: bit-identical


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    # a batch whose workspace is larger than the static array is refused on the host, nothing is enqueued
    Bn, N, V, H, dh, D = 64, 4096, 4000, 32, 128, 256
    need = B.d3tom_workspace_bytes(B.D3TOM_OP_IMPORTANCE, Bn, N, V, H, dh, D)
    assert need > B.D3TOM_IMPORTANCE_STATIC_BYTES
    lay = B.Layout([N] * Bn, [0] * Bn, [V] * Bn, [list(range(D))] * Bn, [1] * Bn)
    q = torch.zeros((8, H, dh), dtype=torch.bfloat16, device="cuda")       # never read: the call fails on the host
    scores = torch.zeros(Bn * V, dtype=torch.float32, device="cuda")
    with pytest.raises(B.D3tomError) as e:
        B.d3tom_importance_static(q, q, lay, 0.1, scores)
    assert e.value.status == B.D3TOM_ERR_UNSUPPORTED
    torch.cuda.synchronize()
