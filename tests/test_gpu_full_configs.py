"""GPU parity at the full sizes of the five benchmark configurations, in the launch configuration that
bench.py times (plain fp6_linear, automatic plan).  Configs 2-3 are checked on the full
matrix; configs 4-5 and the paper's kernel-table shapes on sampled output channels (rows
of W are quantized independently, so the oracle can do any subset of them one by one):
scales and codes bit-exact on the sample, Y within 2e-3 on the sample for all M rows.  The grouped
launches of the config-5 layer (fp6_linear_group over q+k+v and gate+up) are checked the same way."""
import numpy as np
import pytest
import torch

import paper_2312_08583_amd as P
from oracle import fp6_oracle as O
from paper_2312_08583_amd import inputs

from gpu_util import assert_y_close, to_np16

pytestmark = pytest.mark.gpu
DEV = "cuda"
_packed = {}
_oracle = {}


def _get(workload, si, layer=0):
    key = (workload, si, layer)
    if key not in _packed:
        _packed.clear()                      # keep one weight resident at a time
        W = inputs.workload_weight(workload, si, layer=layer, device=DEV)
        hi, lo, sc = P.fp6_quantize_pack(W)
        _packed[key] = (W, hi, lo, sc)
        _oracle.clear()
    return _packed[key]


def _check(workload, si, M, layer=0, sample=None):
    _, N, K = inputs.WORKLOADS[workload]["shapes"][si]
    W, hi, lo, sc = _get(workload, si, layer)
    X = inputs.activation(M, K, seed=inputs.workload_seed(workload, 5000 + 16 * layer + si) + M, device=DEV)
    Y = P.fp6_linear(X, hi, lo, sc, N, K)
    torch.cuda.synchronize()
    if sample is None:
        rows = np.arange(N)
    else:
        rng = np.random.default_rng(N * 31 + K + layer)
        rows = np.sort(rng.choice(N, size=sample, replace=False))
        rows[0], rows[-1] = 0, N - 1                      # first and last channel always
    ridx = torch.from_numpy(rows).to(DEV)
    okey = (workload, si, layer, sample)
    if okey not in _oracle:
        _oracle[okey] = O.quantize(to_np16(W[ridx]))
    codes_o, scales_o = _oracle[okey]
    assert np.array_equal(to_np16(sc[ridx]), scales_o)
    codes_g = P.fp6_unpack_codes(hi, lo, N, K)[ridx].cpu().numpy()
    assert np.array_equal(codes_g, codes_o)
    Yref = O.linear(to_np16(X), codes_o, scales_o)
    assert_y_close(Y[:, ridx], Yref, (workload, si, M))


@pytest.mark.parametrize("M", [1, 4, 16])
@pytest.mark.parametrize("si", [0, 1, 2])
def test_cfg2_llama7b_full_matrix(si, M):
    _check("cfg2_llama7b", si, M)


@pytest.mark.parametrize("M", [1, 8, 32, 128])
@pytest.mark.parametrize("si", [0, 1, 2])
def test_cfg3_llama13b_full_matrix(si, M):
    _check("cfg3_llama13b", si, M)


@pytest.mark.parametrize("M", [1, 16, 64, 256, 512])
@pytest.mark.parametrize("si", [0, 1])
def test_cfg4_llama70b_mlp_sampled(si, M):
    _check("cfg4_llama70b_mlp", si, M, sample=384)


@pytest.mark.parametrize("M", [1, 512])
@pytest.mark.parametrize("si", range(7))
@pytest.mark.parametrize("layer", [0, 47])
def test_cfg5_34b_stack_sampled(layer, si, M):
    _check("cfg5_34b_stack", si, M, layer=layer, sample=256)


@pytest.mark.parametrize("si", range(6))
def test_paper_kernel_table_shapes_batch8_sampled(si):
    _check("paper_table_b1", si, 8, sample=256)


# ---- fine-grained scales and FP5 at full sizes (sampled channels; every row is quantized on its own)

def _check_variant(kind, workload, si, M, block=128, sample=192):
    _, N, K = inputs.WORKLOADS[workload]["shapes"][si]
    W = inputs.workload_weight(workload, si, layer=0, device=DEV)
    X = inputs.activation(M, K, seed=inputs.workload_seed(workload, 7000 + si) + M, device=DEV)
    rng = np.random.default_rng(N * 17 + K)
    rows = np.sort(rng.choice(N, size=sample, replace=False))
    rows[0], rows[-1] = 0, N - 1
    ridx = torch.from_numpy(rows).to(DEV)
    Wr = to_np16(W[ridx])
    if kind == "fgq":
        hi, lo, sc = P.fp6_quantize_pack_fgq(W, block)
        Y = P.fp6_linear_fgq(X, hi, lo, sc, N, K, block)
        codes_o, scales_o = O.quantize_fgq(Wr, block)
        assert np.array_equal(to_np16(sc[:, ridx]), scales_o.T)
        assert np.array_equal(P.fp6_unpack_codes(hi, lo, N, K)[ridx].cpu().numpy(), codes_o)
        Yref = O.linear_fgq(to_np16(X), codes_o, scales_o, block)
    else:
        hi, lo, sc = P.fp5_quantize_pack(W)
        Y = P.fp5_linear(X, hi, lo, sc, N, K)
        codes_o, scales_o = O.quantize5(Wr)
        assert np.array_equal(to_np16(sc[ridx]), scales_o)
        assert np.array_equal(P.fp5_unpack_codes(hi, lo, N, K)[ridx].cpu().numpy(), codes_o)
        Yref = O.linear5(to_np16(X), codes_o, scales_o)
    torch.cuda.synchronize()
    assert_y_close(Y[:, ridx], Yref, (kind, workload, si, M))


@pytest.mark.parametrize("kind", ["fgq", "fp5"])
@pytest.mark.parametrize("si", range(6))
def test_paper_kernel_table_shapes_fgq_and_fp5_sampled(si, kind):
    _check_variant(kind, "paper_table_b1", si, 8)


@pytest.mark.parametrize("kind", ["fgq", "fp5"])
@pytest.mark.parametrize("M", [1, 512])
@pytest.mark.parametrize("si", [1, 4, 6])        # k (1024x8192), gate (22016x8192), down (8192x22016)
def test_cfg5_shapes_fgq_and_fp5_sampled(si, M, kind):
    _check_variant(kind, "cfg5_34b_stack", si, M, block=256)


# ---- the grouped launches of the config-5 layer (q+k+v, gate+up), as the benchmark's grouped leg issues them

@pytest.mark.parametrize("M", [1, 8, 512])
@pytest.mark.parametrize("group", [(0, 1, 2), (4, 5)])
def test_cfg5_grouped_launches_sampled(group, M, sample=128):
    workload = "cfg5_34b_stack"
    shapes = [inputs.WORKLOADS[workload]["shapes"][si][1:] for si in group]
    K = shapes[0][1]
    X = inputs.activation(M, K, seed=inputs.workload_seed(workload, 9000 + group[0]) + M, device=DEV)
    _packed.clear()
    layers, weights = [], []
    for si, (N, _) in zip(group, shapes):
        W = inputs.workload_weight(workload, si, layer=1, device=DEV)
        hi, lo, sc = P.fp6_quantize_pack(W)
        weights.append(W)
        layers.append((X, hi, lo, sc, N, K))
    ys = P.fp6_linear_group(layers)
    torch.cuda.synchronize()
    for si, (N, _), W, (_, hi, lo, sc, _, _), Y in zip(group, shapes, weights, layers, ys):
        rng = np.random.default_rng(N * 13 + si)
        rows = np.sort(rng.choice(N, size=sample, replace=False))
        rows[0], rows[-1] = 0, N - 1
        ridx = torch.from_numpy(rows).to(DEV)
        codes_o, scales_o = O.quantize(to_np16(W[ridx]))
        assert np.array_equal(P.fp6_unpack_codes(hi, lo, N, K)[ridx].cpu().numpy(), codes_o)
        Yref = O.linear(to_np16(X), codes_o, scales_o)
        assert_y_close(Y[:, ridx], Yref, (workload, "group", si, M))
