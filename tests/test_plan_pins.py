"""The launch plans of the benchmark configurations, pinned (CPU only: the planner is host code).

Parity tests prove that whatever plan ran gave the right numbers; they cannot see a planner that silently
stops choosing the streaming kernel, drops a K-split or turns half tiles off.  This table is the planner's
choice for every (shape, M) of the five benchmark configurations and of the paper's kernel table (Appendix B
shapes at batch 8), as reviewed against the sweep of forced plans that `bench.py` runs (`plan_check`: the
automatic plan is within 2 percent of the best forced plan on every row it covers, and ahead of it on the rows
whose best plan the sweep does not contain).  A deliberate change of the planner changes this table in the
same commit, with the measurement that justifies it."""
import pytest

import paper_2312_08583_amd as P
from paper_2312_08583_amd import inputs

PLANS = [
    ("cfg1_single", 1024, 1024, 1, "decode half rows16 split1 wg32"),
    ("cfg2_llama7b", 4096, 4096, 1, "decode half rows16 split2 pairwise wg256"),
    ("cfg2_llama7b", 4096, 4096, 4, "decode half rows16 split2 pairwise wg256"),
    ("cfg2_llama7b", 4096, 4096, 16, "decode rows16 split4 counter wg256"),
    ("cfg2_llama7b", 11008, 4096, 1, "decode rows16 split1 wg172"),
    ("cfg2_llama7b", 11008, 4096, 4, "decode rows16 split1 wg172"),
    ("cfg2_llama7b", 11008, 4096, 16, "decode rows16 split1 wg172"),
    ("cfg2_llama7b", 4096, 11008, 1, "decode half rows16 split2 pairwise wg256"),
    ("cfg2_llama7b", 4096, 11008, 4, "decode half rows16 split2 pairwise wg256"),
    ("cfg2_llama7b", 4096, 11008, 16, "decode rows16 split4 counter wg256"),
    ("cfg3_llama13b", 5120, 5120, 1, "decode half rows16 split1 wg160"),
    ("cfg3_llama13b", 5120, 5120, 8, "decode rows16 split5 counter wg400"),
    ("cfg3_llama13b", 5120, 5120, 32, "decode rows32 split2 counter wg160"),
    ("cfg3_llama13b", 5120, 5120, 128, "gemm 64x256 split5 counter wg208"),
    ("cfg3_llama13b", 13824, 5120, 1, "decode rows16 split1 wg216"),
    ("cfg3_llama13b", 13824, 5120, 8, "decode rows16 split1 wg216"),
    ("cfg3_llama13b", 13824, 5120, 32, "decode rows32 split1 wg216"),
    ("cfg3_llama13b", 13824, 5120, 128, "gemm 64x256 split2 counter wg224"),
    ("cfg3_llama13b", 5120, 13824, 1, "decode rows16 split3 counter wg240"),
    ("cfg3_llama13b", 5120, 13824, 8, "decode rows16 split3 counter wg240"),
    ("cfg3_llama13b", 5120, 13824, 32, "decode rows32 split3 counter wg240"),
    ("cfg3_llama13b", 5120, 13824, 128, "gemm 64x256 split6 counter wg240"),
    ("cfg4_llama70b_mlp", 28672, 8192, 1, "decode rows16 split1 wg448"),
    ("cfg4_llama70b_mlp", 28672, 8192, 16, "decode rows16 split1 wg448"),
    ("cfg4_llama70b_mlp", 28672, 8192, 64, "gemm 64x256 split2 counter wg224"),
    ("cfg4_llama70b_mlp", 28672, 8192, 256, "gemm 128x256 k2 split1 wg224"),
    ("cfg4_llama70b_mlp", 28672, 8192, 512, "gemm 128x512 split1 wg224"),
    ("cfg4_llama70b_mlp", 8192, 28672, 1, "decode half rows16 split1 wg256"),
    ("cfg4_llama70b_mlp", 8192, 28672, 16, "decode rows16 split2 pairwise wg256"),
    ("cfg4_llama70b_mlp", 8192, 28672, 64, "gemm 64x256 split7 counter wg224"),
    ("cfg4_llama70b_mlp", 8192, 28672, 256, "gemm 128x256 k2 split4 counter wg256"),
    ("cfg4_llama70b_mlp", 8192, 28672, 512, "gemm 128x256 k2 split2 counter wg256"),
    ("cfg5_34b_stack", 8192, 8192, 1, "decode half rows16 split1 wg256"),
    ("cfg5_34b_stack", 8192, 8192, 512, "gemm 128x256 k2 split2 counter wg256"),
    ("cfg5_34b_stack", 1024, 8192, 1, "decode half rows16 split8 counter wg256"),
    ("cfg5_34b_stack", 1024, 8192, 512, "gemm 32x256 split4 counter wg256"),
    ("cfg5_34b_stack", 22016, 8192, 1, "decode rows16 split2 pairwise wg688"),
    ("cfg5_34b_stack", 22016, 8192, 512, "gemm 128x512 split1 wg192"),
    ("cfg5_34b_stack", 8192, 22016, 1, "decode half rows16 split1 wg256"),
    ("cfg5_34b_stack", 8192, 22016, 512, "gemm 128x256 k2 split2 counter wg256"),
    ("paper_table_b1", 5504, 2048, 8, "decode rows16 split2 pairwise wg172"),
    ("paper_table_b1", 2048, 5504, 8, "decode rows16 split2 pairwise wg64"),
    ("paper_table_b1", 13824, 5120, 8, "decode rows16 split1 wg216"),
    ("paper_table_b1", 5120, 13824, 8, "decode rows16 split3 counter wg240"),
    ("paper_table_b1", 22016, 8192, 8, "decode rows16 split2 pairwise wg688"),
    ("paper_table_b1", 8192, 22016, 8, "decode rows16 split2 pairwise wg256"),
]

# groups of layers launched together (fp6_linear_group): the plan is that of the summed N
GROUP_PLANS = [
    (1, [(8192, 8192), (1024, 8192), (1024, 8192)], "decode rows16 split1 wg160"),
    (1, [(22016, 8192), (22016, 8192)], "decode rows16 split1 wg688"),
    (16, [(8192, 8192), (1024, 8192), (1024, 8192)], "decode rows16 split1 wg160"),
]


def test_every_configured_shape_is_pinned():
    want = {(wl, N, K, M) for wl, c in inputs.WORKLOADS.items() for (_, N, K) in c["shapes"] for M in c["Ms"]}
    assert want == {(wl, N, K, M) for (wl, N, K, M, _) in PLANS}


@pytest.mark.parametrize("wl,N,K,M,plan", PLANS)
def test_plan_of_configured_shape(wl, N, K, M, plan):
    assert P.plan_text(P.fp6_linear_plan(M, N, K)) == plan


@pytest.mark.parametrize("M,shapes,plan", GROUP_PLANS)
def test_plan_of_grouped_layers(M, shapes, plan):
    n_total, K = sum(N for N, _ in shapes), shapes[0][1]
    assert P.plan_text(P.fp6_linear_plan(M, n_total, K)) == plan
    assert P.fp6_linear_group_workspace_bytes(M, shapes) == P.fp6_linear_plan(M, n_total, K)["workspace_bytes"]
