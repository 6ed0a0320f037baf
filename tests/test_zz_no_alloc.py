"""The allocation-free column-sum entry point against the entry point it is a variant of (GPU only).

bk_colsum_acc_static keeps its partial rows in a device array inside the library; it runs the same two
kernels as bk_colsum_acc, so the results must be bitwise equal.  Two calls in a row share the array, the
second with a smaller input: stale partial rows of the first call must not leak into the second."""
import numpy as np
import pytest
import torch

from paper_2204_12013_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def B():
    from paper_2204_12013_amd import binding
    return binding


def _input(rng, T, N, dtype):
    a = synth.round_to_storage(rng.standard_normal((T, N)).astype(np.float32), dtype)
    return a


@pytest.mark.parametrize("dtype", [0, 1])
def test_static_scratch_column_sum_equals_the_caller_scratch_one(B, dtype):
    rng = np.random.default_rng(11 + dtype)
    torch.cuda.synchronize()
    for T, N in ((4096, 3072), (515, 200)):          # the second call is smaller: fewer and shorter partial rows
        a_host = _input(rng, T, N, dtype)
        A = B.to_device(a_host, dtype, DEV)
        out0 = rng.standard_normal(N).astype(np.float32)
        want = torch.from_numpy(out0.copy()).to(DEV)
        got = torch.from_numpy(out0.copy()).to(DEV)
        B.bk_colsum_acc(A, want)
        B.bk_colsum_acc_static(A, got)
        torch.cuda.synchronize()
        assert torch.equal(got, want), (T, N)
        # and both are the column sums (fp64 on the host), added to what was there
        ref = a_host.astype(np.float64).sum(0)
        err = np.linalg.norm(got.cpu().numpy().astype(np.float64) - out0 - ref) / np.linalg.norm(ref)
        assert err <= 1e-4, err


def test_static_scratch_rejects_what_does_not_fit(B):
    cap = int(B.lib.bk_colsum_static_max_floats())
    assert cap == 512 * 1024
    N = cap + 2                                         # one partial row is already longer than the array
    A = torch.zeros(1, N, dtype=torch.bfloat16, device=DEV)
    out = torch.zeros(N, dtype=torch.float32, device=DEV)
    with pytest.raises(B.BambooError) as e:
        B.bk_colsum_acc_static(A, out)
    assert e.value.status == B.E_ARG
    assert float(out.abs().max()) == 0.0               # nothing was launched
