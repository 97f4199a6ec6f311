"""GPU: fp6_linear_static (the entry point that allocates nothing) against fp6_linear.

The two share planner and kernels and the kernels are deterministic, so the results must agree bit for
bit (which is inside the 2e-3 bar that fp6_linear itself is held to against the oracle).  Calls come in
pairs, the second with a smaller input, so that the second call finds the library's scratch as the first
one left it.  Collected last (file name): a failure here must not hide the other GPU tests."""
import ctypes

import pytest
import torch

import paper_2312_08583_amd as P
from paper_2312_08583_amd import binding as B
from paper_2312_08583_amd import inputs

from gpu_util import assert_y_close, oracle_reference

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _layer(N, K, seed):
    W = inputs.weight(N, K, seed=seed, sigma=0.02, outlier_frac=0.001, device=DEV)
    return (W,) + tuple(P.fp6_quantize_pack(W))


def _static_through_the_c_abi(X, hi, lo, sc, N, K):
    """Calls the exported symbol directly: raw device pointers, Y allocated here beforehand."""
    M = X.shape[0]
    Y = torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV)
    rc = B.lib().fp6_linear_static(X.data_ptr(), M, hi.data_ptr(), lo.data_ptr(), sc.data_ptr(), N, K, Y.data_ptr(),
                                   torch.cuda.current_stream().cuda_stream)
    assert rc == 0, B.fp6_status_string(rc)
    return Y


# (first call, second smaller call): plans with a counter meeting, a pairwise meeting, and no meeting at all
PAIRS = [
    ((512, 1024, 4096), (200, 512, 2048)),      # tiled kernel, K split, arrival counters + partial sums
    ((8, 1024, 4096), (2, 512, 4096)),          # streaming kernel, K split
    ((16, 2048, 2048), (1, 1024, 8192)),
    ((64, 1024, 2048), (1, 4096, 256)),         # the second call needs no scratch at all
]


@pytest.mark.parametrize("first,second", PAIRS)
def test_two_calls_in_a_row_match_fp6_linear(first, second):
    for (M, N, K) in (first, second):
        W, hi, lo, sc = _layer(N, K, seed=40 + N + K)
        X = inputs.activation(M, K, seed=41 + M, device=DEV)
        plan = P.fp6_linear_plan(M, N, K)
        Ys = _static_through_the_c_abi(X, hi, lo, sc, N, K)
        Yw = P.fp6_linear(X, hi, lo, sc, N, K)              # fresh zeroed workspace from the binding
        torch.cuda.synchronize()
        assert torch.equal(Ys.view(torch.int16), Yw.view(torch.int16)), (M, N, K, P.plan_text(plan))
        _, _, Yref = oracle_reference(W, X)
        assert_y_close(Ys, Yref, "static scratch %s" % P.plan_text(plan))


def test_the_pairs_above_do_use_the_scratch():
    used = [P.fp6_linear_plan(*shape)["workspace_bytes"] > 0 for pair in PAIRS for shape in pair]
    assert sum(used) >= 6, used


def test_a_shape_beyond_the_scratch_is_refused_and_nothing_is_written():
    a = torch.zeros(64, dtype=torch.uint8, device=DEV)      # never dereferenced: the call fails on the host
    Y = torch.zeros(16, dtype=torch.float16, device=DEV)
    refused = 0
    for (M, N, K) in [(512, 8192, 22016), (4096, 1024, 32768), (8192, 512, 16384), (8192, 1024, 65536)]:
        need = P.fp6_linear_workspace_bytes(M, N, K)
        if need <= P.FP6_STATIC_SCRATCH_BYTES:
            continue
        rc = B.lib().fp6_linear_static(a.data_ptr(), M, a.data_ptr(), a.data_ptr(), a.data_ptr(), N, K, Y.data_ptr(), None)
        assert rc == B.FP6_ERR_SCRATCH, (M, N, K, need)
        assert "scratch" in B.fp6_status_string(rc)
        refused += 1
    torch.cuda.synchronize()
    assert not Y.any()
    assert refused >= 1, "no candidate shape needs more than the built-in scratch"
