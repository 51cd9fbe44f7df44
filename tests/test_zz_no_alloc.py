"""sb_op_head_static (the entry point for callers that cannot allocate: its scratch area is a
static device array of the library) against sb_op_head, through the C ABI: same kernels, so
arg max and confidence must be bit-identical; two calls in a row, the second with a smaller
input, so that what the first call left in the shared array is seen not to matter."""
import numpy as np
import pytest

import sb_inputs as si

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sb():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2604_12247_amd as sb
    return sb


def _case(sb, torch, N, K, M, kernel, seed, T):
    g = np.random.default_rng(seed)
    Wf = (g.standard_normal((N, K)) * 0.05).astype(np.float32)
    x = torch.from_numpy(g.standard_normal((M, K)).astype(np.float32)).cuda()
    if kernel == sb.PROJ_VALU:
        W = torch.from_numpy(Wf).cuda()
    else:
        W = torch.from_numpy(si.round_to_bf16(Wf).view(np.int16)).cuda()
        if kernel == sb.PROJ_MFMA_PACKED:
            W = sb.op_repack(W)
    return W, x, T


@pytest.mark.parametrize("kernel_name", ["VALU", "MFMA", "MFMA_PACKED"])
def test_static_scratch_head_matches_the_workspace_one(sb, kernel_name):
    import torch
    kernel = getattr(sb, "PROJ_" + kernel_name)
    # second call smaller in every dimension (rows, outputs, inner size)
    cases = [_case(sb, torch, 32000, 4096, 8, kernel, 5, 1.7), _case(sb, torch, 4112, 1024, 3, kernel, 6, 0.8)]
    am = torch.full((8,), -7, dtype=torch.int32, device="cuda")
    cf = torch.full((8,), -7.0, dtype=torch.float32, device="cuda")
    # (a first call, not measured: the runtime loads the library's code objects at a first launch)
    sb.op_head_static(cases[0][0], cases[0][1], cases[0][2], kernel, am, cf)
    for W, x, T in cases:
        M = x.shape[0]
        am.fill_(-7); cf.fill_(-7.0)
        torch.cuda.synchronize()
        # no allocation during the call: torch's count of allocations made stays (memory in use may
        # drop meanwhile, when Python collects earlier tests' tensors) and the device's free memory,
        # which a hipMalloc by the library would lower, does not go down
        n_alloc = torch.cuda.memory_stats()["allocation.all.allocated"]
        free_before = torch.cuda.mem_get_info()[0]
        sb.op_head_static(W, x, T, kernel, am, cf)
        assert torch.cuda.memory_stats()["allocation.all.allocated"] == n_alloc
        assert torch.cuda.mem_get_info()[0] >= free_before
        ref_am, ref_cf, _ = sb.op_head(W, x, T, kernel)
        torch.cuda.synchronize()
        assert am[:M].tolist() == ref_am.tolist()
        assert cf[:M].cpu().numpy().tobytes() == ref_cf.cpu().numpy().tobytes()     # same kernels: same bits
        assert am[M:].tolist() == [-7] * (8 - M) and cf[M:].tolist() == [-7.0] * (8 - M)


def test_static_scratch_head_rejects_sizes_beyond_its_area(sb):
    import torch
    x = torch.zeros((1, 16384), dtype=torch.float32, device="cuda")
    W = torch.zeros((16, 16384), dtype=torch.float32, device="cuda")
    am = torch.zeros(8, dtype=torch.int32, device="cuda")
    cf = torch.zeros(8, dtype=torch.float32, device="cuda")
    with pytest.raises(sb.SbError) as e:
        sb.op_head_static(W, x, 1.0, sb.PROJ_VALU, am, cf)        # K beyond the limit
    assert e.value.code == sb.ECAPACITY
    W2 = torch.zeros((131072 + 16, 8), dtype=torch.float32, device="cuda")
    with pytest.raises(sb.SbError) as e:
        sb.op_head_static(W2, x[:, :8].contiguous(), 1.0, sb.PROJ_VALU, am, cf)   # N beyond the limit
    assert e.value.code == sb.ECAPACITY
