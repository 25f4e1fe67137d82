"""GPU parity of the column-slice plan (the wave-column layout walked by persistent workgroups,
one per 64 partitions) against the CPU oracle: every output, element by element, bit-exact."""
import numpy as np
import pytest

from workloads import make_workload
from test_gpu_parity import _check, gpu  # noqa: F401

pytestmark = pytest.mark.gpu

SLICE = 5


def test_large_sparse_full_column_slice(gpu, oracle):
    _check(gpu, oracle, make_workload("large_sparse"), plans=(SLICE,), out_layouts=(0,))


def test_comm_heavy_full_column_slice(gpu, oracle):
    # rows of 1,000 edges are split over the workgroup's wavefronts
    _check(gpu, oracle, make_workload("comm_heavy"), plans=(SLICE,), out_layouts=(0,))


def test_small_workloads_and_layouts(gpu, oracle):
    _check(gpu, oracle, make_workload("tiny"), plans=(SLICE,), ticks=(4, 8), layouts=(0, 1))
    _check(gpu, oracle, make_workload("mlp", P=200), plans=(SLICE,))
    _check(gpu, oracle, make_workload("inception", P=70), plans=(SLICE,), out_layouts=(0,))


@pytest.mark.parametrize("P", [1, 63, 65, 130])
def test_ragged_slices(gpu, oracle, P):
    w = make_workload("comm_heavy", P=P, levels=5, width=600, hub_degree=300)
    _check(gpu, oracle, w, plans=(SLICE,), layouts=(0, 1), what=f"ragged P={P}")


def test_cost_models_without_multiply_shift_tables_are_refused(gpu):
    from gpu_util import run_gpu
    w = make_workload("tiny")
    k = 70                                             # more devices than the tables in LDS hold
    a = np.zeros((4, w.n), dtype=np.uint8)
    with pytest.raises(gpu.CpError) as e:
        run_gpu(w, SLICE, speeds=np.ones(k, dtype=np.int64), bandwidth=np.ones((k, k), dtype=np.int64),
                assignments=a)
    assert e.value.code == -12
