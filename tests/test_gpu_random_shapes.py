"""Seeded random layer shapes through the fused forward (Bi-GCN and Bi-GraphSAGE), layer by layer
against the CPU oracle.  The widths are drawn from the values on either side of every boundary of
the product-row formats (rows of 8 / 16 / 32 / 64 lanes; scale in the tail, in the last bytes,
in the top bits, separate; 7-bit forms with one-byte and fp16 alternates; fp16 and fp32 rows), a
few input rows equal a weight column (products of +-K), and every fifth case has more than 32768
nodes, where the bit-GEMM runs its kernels for large row counts."""
import numpy as np
import pytest

from helpers import compare_forward_layerwise, compare_forward_teacher_forced
from test_gpu_forward import gpu_prefix_runner
from test_gpu_sage import sage_prefix_runner, small_sage_workload
from workloads import chung_lu_csr
from workloads.build import Workload
from workloads.configs import WorkloadConfig

pytestmark = pytest.mark.gpu

WIDTHS = [1, 2, 3, 5, 7, 8, 9, 15, 16, 17, 31, 32, 33, 39, 40, 41, 47, 55, 56, 60, 61, 63, 64, 65, 79, 80, 81,
          100, 127, 128, 129, 200, 255, 256, 257, 300, 511, 512]
INPUTS = [1, 2, 31, 63, 64, 65, 100, 127, 128, 129, 191, 192, 193, 255, 256, 257, 320, 511, 512, 513, 640,
          1023, 1024, 1025, 2048, 2049]
CASES_PER_SEED = 10


@pytest.fixture(scope="module")
def B():
    import torch
    from paper_2210_13149_amd import binding
    assert torch.cuda.is_available()
    binding.lib()
    return binding


@pytest.mark.parametrize("seed", range(16))
def test_forward_random_shapes(B, seed):
    rng = np.random.default_rng(7000 + seed)
    for it in range(CASES_PER_SEED):
        depth = int(rng.integers(2, 4))
        dims = (int(rng.choice(INPUTS)),) + tuple(int(rng.choice(WIDTHS)) for _ in range(depth))
        n = 33000 + int(rng.integers(0, 200)) if it % 5 == 4 else int(rng.integers(200, 3000))
        n_edges = n * int(rng.integers(1, 6))
        bn = [None] * depth if it % 4 < 2 else ["calibrate"] * depth
        label = f"seed {seed} case {it}: dims {dims}, {n} nodes, {n_edges} edges"
        if it % 2 == 0:
            rp, ci = chung_lu_csr(n, n_edges, 2.5, 2.0, seed=1000 * seed + it)
            ws = [rng.uniform(-1, 1, size=(dims[i], dims[i + 1])).astype(np.float32) for i in range(depth)]
            x = rng.standard_normal((n, dims[0])).astype(np.float32)
            for k in range(0, min(40, n)):
                x[k] = ws[0][:, k % dims[1]] * (1 if k % 2 == 0 else -1)
            cfg = WorkloadConfig("random", "none", n, n_edges, 2.0, dims, "normal", 1.0, "first", 0)
            work = Workload(cfg, rp, ci, x, ws)
            teacher = compare_forward_teacher_forced(work, bn, gpu_prefix_runner(B, work), own_sum_bound=True)
            assert all(t['rows_compared'] == work.n for t in teacher)
            stats = compare_forward_layerwise(work, bn, gpu_prefix_runner(B, work), cancellation_aware=True)
        else:
            work = small_sage_workload(n, n_edges, dims, seed=1000 * seed + it)
            for k in range(0, min(40, n)):
                work.x[k] = work.weights[0][k % 2][:, k % dims[1]] * (1 if k % 4 < 2 else -1)
            teacher = compare_forward_teacher_forced(work, bn, sage_prefix_runner(B, work), own_sum_bound=True)
            assert all(t['rows_compared'] == work.n for t in teacher)
            stats = compare_forward_layerwise(work, bn, sage_prefix_runner(B, work), cancellation_aware=True)
        assert stats[0]["rows_compared"] == n, label
