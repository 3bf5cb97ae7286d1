"""The entry point for callers that cannot allocate (is_gemm_w4a8_intscale_prepacked_noalloc) against the workspace
form of the same GEMM: same kernels, so outputs and accumulators must agree to the bit.  Two calls in a row share the
library's fixed scratch, the second with a smaller input."""
import numpy as np
import pytest
import torch

import paper_2405_14597_amd as P

pytestmark = pytest.mark.gpu
G = 128


def make_case(M, N, K, seed, dev):
    g = torch.Generator(device="cpu").manual_seed(seed)
    q = torch.randint(0, 256, (N, K // 2), dtype=torch.uint8, generator=g).to(dev)
    si = torch.randint(1, 1025, (N, K // G), dtype=torch.int32, generator=g).to(dev)
    c = (torch.rand((N,), generator=g) * 1e-3 + 1e-4).to(dev)
    xq = torch.randint(-127, 128, (M, K), dtype=torch.int8, generator=g).to(dev)
    sa = (torch.rand((M,), generator=g) * 0.05 + 0.01).to(dev)
    return xq, sa, P.is_prepack_w4(q, si, G), c


def run_both(M, N, K, seed, dev):
    xq, sa, pk, c = make_case(M, N, K, seed, dev)
    ref_out, ref_acc = P.is_gemm_w4a8_intscale_prepacked(xq, sa, pk, c, 10, want_acc=True)
    out = torch.full((M, N), float("nan"), dtype=torch.float16, device=dev)
    acc = torch.full((M, N), -1, dtype=torch.int32, device=dev)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    P.is_gemm_w4a8_intscale_prepacked_noalloc(xq, sa, pk, c, 10, out, acc)
    assert torch.cuda.memory_allocated() == before       # nothing came from torch's allocator either
    torch.cuda.synchronize()
    assert np.array_equal(acc.cpu().numpy(), ref_acc.cpu().numpy()), (M, N, K)
    assert np.array_equal(out.cpu().numpy().view(np.uint16), ref_out.cpu().numpy().view(np.uint16)), (M, N, K)


def test_noalloc_matches_workspace_form_on_two_calls_in_a_row():
    dev = torch.device("cuda:0")
    # K split across workgroups: partial sums and arrival counters live in the scratch
    big, small = (32, 2048, 28672), (5, 528, 8192)
    assert P.is_gemm_prepacked_workspace_bytes(*big, G) > 0 and P.is_gemm_prepacked_workspace_bytes(*small, G) > 0
    assert P.is_gemm_prepacked_workspace_bytes(*small, G) < P.is_gemm_prepacked_workspace_bytes(*big, G)
    print("noalloc decode", big, small, flush=True)
    run_both(*big, 11, dev)
    run_both(*small, 12, dev)
    run_both(*big, 13, dev)
    # tiled route: the prepared activations live in the scratch
    tbig, tsmall = (400, 520, 8192), (130, 264, 1024)
    assert P.is_gemm_prepacked_workspace_bytes(*tbig, G) <= P.IS_NOALLOC_SCRATCH_BYTES
    print("noalloc tiled", tbig, tsmall, flush=True)
    run_both(*tbig, 21, dev)
    run_both(*tsmall, 22, dev)
    # a shape without workspace, and the decode shape again after the tiled calls wrote over the counters' place
    run_both(3, 4096, 4096, 31, dev)
    run_both(*small, 32, dev)


def test_noalloc_rejects_sizes_beyond_the_scratch():
    dev = torch.device("cuda:0")
    M, N, K = 2048, 256, 28672
    assert P.is_gemm_prepacked_workspace_bytes(M, N, K, G) > P.IS_NOALLOC_SCRATCH_BYTES
    xq, sa, pk, c = make_case(M, N, K, 41, dev)
    out = torch.zeros((M, N), dtype=torch.float16, device=dev)
    with pytest.raises(P.IntScaleError) as err:
        P.is_gemm_w4a8_intscale_prepacked_noalloc(xq, sa, pk, c, 10, out)
    assert "IS_ERR_WORKSPACE" in str(err.value)
    assert float(out.abs().sum()) == 0.0     # nothing ran
