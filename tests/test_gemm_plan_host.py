"""The work decomposition of the persistent contraction kernel, replayed on the host (no GPU): for the
layer shapes of every workload and for a seeded sweep of shapes and workgroup counts, every tile and every
slab of K must be covered exactly once, pieces must be even and contiguous, and the pieces of a cut tile must
sit in the slots the second kernel reads."""
import numpy as np
import pytest

from paper_2209_02341_amd import binding as E
from paper_2209_02341_amd import workloads as wl


def layer_shapes(w, T):
    H, A, F = w.hidden, w.attn_width, w.ffn
    return [(T, 3 * A, H), (T, H, A), (T, F, H), (T, H, F)]


@pytest.mark.parametrize("name", ["gpt13b_bf16", "gpt175b_tp8_shard_bf16", "heavy_pad_bf16"])
def test_layer_shapes_are_covered_exactly_once(name):
    w = wl.WORKLOADS[name]
    T = int(wl.sample_lengths(w).sum())
    cut = 0
    for M in (T, w.batch * w.max_len):
        for (m, n, k) in layer_shapes(w, M):
            for scratch in (False, True):
                st, pieces = E.energon_linear_plan_selfcheck(m, n, k, 32, scratch)
                assert st == 0, (name, m, n, k, scratch, st)
                assert pieces == 1 or scratch
                cut += pieces > 1
    assert cut > 0, "no shape of this workload is cut any more"


def test_the_planned_cuts_of_the_benchmark_workloads():
    # (shape, pieces per cut tile) as measured and documented: a change of the cost model must be a decision
    for shape, want in (((8428, 20480, 5120), 3), ((8428, 5120, 20480), 3), ((8428, 15360, 5120), 1), ((8428, 5120, 5120), 1),
                        ((3184, 6144, 12288), 4), ((3184, 12288, 6144), 2), ((3184, 4608, 12288), 1)):
        st, pieces = E.energon_linear_plan_selfcheck(*shape, 32, True)
        assert (st, pieces) == (0, want), (shape, st, pieces)


def test_random_shapes_and_workgroup_counts():
    rng = np.random.default_rng(2209)
    checked = cut = 0
    for _ in range(400):
        M = int(rng.integers(256, 40000))
        N = 8 * int(rng.integers(32, 5000))
        K = 128 * int(rng.integers(1, 200))
        wgs = int(rng.choice([1, 3, 7, 16, 30, 32, 38, 64]))
        for scratch in (False, True):
            st, pieces = E.energon_linear_plan_selfcheck(M, N, K, wgs, scratch)
            assert st in (0, -1), (M, N, K, wgs, scratch, st)
            if st == 0:
                checked += 1
                cut += pieces > 1
    assert checked > 300 and cut > 20, (checked, cut)


def test_shapes_the_kernel_does_not_take():
    assert E.energon_linear_plan_selfcheck(577, 1024, 1024)[0] == -1      # too few tiles
    assert E.energon_linear_plan_selfcheck(8428, 5120, 5184)[0] == -1     # odd number of slabs
    assert E.energon_linear_plan_selfcheck(8428, 5120, 5100)[0] == -1
