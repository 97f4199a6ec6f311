"""GPU: fp6_linear_group (several independent layers in one call) against the oracle, layer by layer.

For M <= 16 and a common K the group is one launch planned over the layers' channel blocks taken together,
so the cases are chosen for the plans they produce (full-tile and half-tile workgroups; no K-split, two
slices meeting pairwise, more slices meeting at a counter); groups with different K, or more than 16
rows, run as a sequence of launches and must give exactly what separate calls give."""
import numpy as np
import pytest
import torch

import paper_2312_08583_amd as P
from oracle import fp6_oracle as O
from paper_2312_08583_amd import binding as B
from paper_2312_08583_amd import inputs

from gpu_util import assert_y_close, from_np16, oracle_reference, to_np16

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _layers(M, shapes, seed, same_x=True):
    out = []
    for i, (N, K) in enumerate(shapes):
        W = inputs.weight(N, K, seed=seed + 10 * i, sigma=0.02, outlier_frac=0.001, device=DEV)
        X = inputs.activation(M, K, seed=seed + (0 if same_x else i) + 5, device=DEV)
        out.append((W, X) + tuple(P.fp6_quantize_pack(W)))
    return out


CASES = [
    # (M, [(N, K), ...])
    (1, [(512, 1024), (128, 1024), (128, 1024)]),
    (3, [(8192, 512), (1024, 512), (1024, 512)]),         # many blocks: no split
    (16, [(256, 4096), (64, 4096)]),                      # few blocks, long K: split
    (4, [(1024, 8192), (1024, 8192)]),
    (1, [(11008, 4096), (11008, 4096)]),                # 344 blocks: two slices, pairwise
    (2, [(4096, 2048), (512, 2048), (512, 2048), (64, 2048)]),
    (1, [(22016, 512), (22016, 512)]),
    (5, [(64, 64), (64, 64)]),
]


@pytest.mark.parametrize("M,shapes", CASES)
def test_group_matches_oracle_layer_by_layer(M, shapes):
    ls = _layers(M, shapes, seed=1000 + M)
    n_total, K = sum(N for N, _ in shapes), shapes[0][1]
    plan = P.fp6_linear_plan(M, n_total, K)
    layers = [(X, hi, lo, sc, N, K_) for (W, X, hi, lo, sc), (N, K_) in zip(ls, shapes)]
    need = P.fp6_linear_group_workspace_bytes(M, shapes)
    assert need == plan["workspace_bytes"]
    ws = P.new_workspace(max(need, 16), DEV)
    outs = [torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV) for N, _ in shapes]
    for _ in range(2):                                     # the second call reuses the workspace as the first left it
        ys = P.fp6_linear_group(layers, outs=outs, workspace=ws)
    torch.cuda.synchronize()
    for (W, X, *_), Y in zip(ls, ys):
        _, _, Yref = oracle_reference(W, X)
        assert_y_close(Y, Yref, "group %s" % P.plan_text(plan))
    if need:
        assert not ws[:min(need, B.FP6_WORKSPACE_ZERO_BYTES)].any(), "counters and slots are not left zero"


def test_the_cases_cover_the_plans_of_a_group():
    kinds = set()
    for M, shapes in CASES:
        p = P.fp6_linear_plan(M, sum(N for N, _ in shapes), shapes[0][1])
        kinds.add((p["half_tiles"], p["meeting"]))
    assert {h for h, _ in kinds} == {0, 1}, kinds
    assert {m for _, m in kinds} == {0, 1, 2}, kinds


def test_group_one_hot_rows_return_dequantized_weights_bit_exact():
    """X = unit vectors: every layer of the group must return its own W_hat columns exactly."""
    M, K, shapes = 8, 512, [(256, 512), (64, 512), (128, 512)]
    ls = _layers(M, shapes, seed=77)
    ks = [3, 64, 100, 255, 256, 300, 448, 511]
    X = torch.zeros((M, K), dtype=torch.float16, device=DEV)
    for m, k in enumerate(ks):
        X[m, k] = 1.0
    layers = [(X, hi, lo, sc, N, K) for (W, _, hi, lo, sc), (N, _) in zip(ls, shapes)]
    ys = P.fp6_linear_group(layers)
    torch.cuda.synchronize()
    for (W, _, hi, lo, sc), (N, _), Y in zip(ls, shapes, ys):
        # the expected values come from the oracle; a sum that starts at +0 cannot return -0, so zeros compare without sign
        codes_o, scales_o = O.quantize(to_np16(W))
        want = O.dequantize(codes_o, scales_o)[:, ks].T
        got = to_np16(Y)
        want = np.where((want & 0x7FFF) == 0, 0, want).astype(np.uint16)
        got = np.where((got & 0x7FFF) == 0, 0, got).astype(np.uint16)
        assert np.array_equal(got, want)


@pytest.mark.parametrize("M,shapes", [(2, [(256, 512), (128, 1024)]), (40, [(256, 512), (128, 512)]),
                                      (300, [(512, 1024), (64, 1024)]), (7, [(320, 768)])])
def test_groups_that_cannot_share_a_launch_equal_separate_calls(M, shapes):
    ls = _layers(M, shapes, seed=31, same_x=False)
    layers = [(X, hi, lo, sc, N, K) for (W, X, hi, lo, sc), (N, K) in zip(ls, shapes)]
    ys = P.fp6_linear_group(layers)
    for (W, X, hi, lo, sc), (N, K), Y in zip(ls, shapes, ys):
        Y1 = P.fp6_linear(X, hi, lo, sc, N, K)
        torch.cuda.synchronize()
        assert torch.equal(Y.view(torch.int16), Y1.view(torch.int16))
        _, _, Yref = oracle_reference(W, X)
        assert_y_close(Y, Yref, "sequential group")


def test_group_argument_errors():
    M, shapes = 2, [(128, 256), (64, 256)]
    ls = _layers(M, shapes, seed=3)
    layers = [(X, hi, lo, sc, N, K) for (W, X, hi, lo, sc), (N, K) in zip(ls, shapes)]
    with pytest.raises(P.Fp6Error):
        P.fp6_linear_group([])
    with pytest.raises(P.Fp6Error):
        P.fp6_linear_group(layers * 3)                       # more than FP6_GROUP_MAX
    with pytest.raises(P.Fp6Error):
        P.fp6_linear_group(layers, outs=[torch.empty((M, 64), dtype=torch.float16, device=DEV), None])
    bad = list(layers)
    bad[1] = (layers[1][0][:1].contiguous(),) + layers[1][1:]  # a layer with another M
    with pytest.raises(P.Fp6Error):
        P.fp6_linear_group(bad)
    L = B.lib()
    assert L.fp6_linear_group(1, None, 1, None, 0, None) == -1
    arr = (B.LinearProblem * 1)(B.LinearProblem(16, 16, 16, 16, 64, 100, 16))
    assert L.fp6_linear_group(1, arr, 1, None, 0, None) == -2
    assert L.fp6_linear_group(1, arr, 0, None, 0, None) == -2
