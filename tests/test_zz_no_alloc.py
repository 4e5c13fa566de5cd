"""The entry point that allocates nothing (split-K partial sums in the library's own static device array) against
mmm_matmul, through the C ABI: same plan, same kernels, so C must be identical bit for bit; twice in a row, the second
time on a smaller problem, so that what the first call left in the array is there when the second runs."""
import numpy as np
import pytest
import torch

import mmm_synth as synth
import oracle
import paper_2402_14118_amd as mm
from hip_harness import HipRun, assert_close

pytestmark = pytest.mark.gpu


def _both(w, accumulate=False):
    run = HipRun(w)
    run.build()
    run.matmul()
    if accumulate:
        run.matmul(accumulate=True)
    torch.cuda.synchronize()
    want = run.C.cpu().numpy().copy()
    run.Cbuf.fill_(float("nan"))
    run.eng.matmul_static_scratch(run.X, run.Y, run.C)
    if accumulate:
        run.eng.matmul_static_scratch(run.X, run.Y, run.C, accumulate=True)
    torch.cuda.synchronize()
    return run, want, run.C.cpu().numpy()


def test_static_scratch_matches_matmul_twice_in_a_row():
    mm.mmm_set_option("matmul_variant", -1)
    mm.mmm_set_option("split_k", 0)
    mm.mmm_set_option("matmul_path", mm.MMM_PATH_MATRIX)      # the kernel that splits K and needs the scratch
    # decode-like shapes: few tiles of C and a long K, so the plan splits K and the partial sums are used
    w1 = synth.random_masked(32, 8192, 512, 16, 0.1, 0.2, 901, dist="normal")
    run, want, got = _both(w1)
    assert run.eng.plan()[1] > 1
    np.testing.assert_array_equal(got, want)
    _, _, C_ref, mag = oracle.run_workload(w1)
    assert_close(got, C_ref, mag, w1.dtype, "static scratch, first call")
    w2 = synth.random_masked(20, 4100, 208, 8, 0.3, 0.3, 902, dist="smallint")      # smaller, ragged
    run, want, got = _both(w2, accumulate=True)
    assert run.eng.plan()[1] > 1
    np.testing.assert_array_equal(got, want)
    _, _, C_ref, _ = oracle.run_workload(w2)
    np.testing.assert_array_equal(got, 2 * C_ref)


def test_static_scratch_without_a_split_and_beyond_its_size():
    mm.mmm_set_option("matmul_path", mm.MMM_PATH_MATRIX)
    w = synth.random_masked(150, 300, 400, 16, 0.3, 0.3, 903, dist="smallint")       # plan does not split K: no scratch
    run, want, got = _both(w)
    assert run.eng.plan()[1] == 1
    np.testing.assert_array_equal(got, want)
    # 8 splits of a 512 x 4096 C are 64 MiB of partial sums: more than the 16 MiB array holds
    w = synth.random_masked(512, 2048, 4096, 16, 0.05, 0.05, 904, dist="smallint")
    run = HipRun(w)
    run.build()
    run.eng.set_plan(-1, 8)
    assert run.eng.plan()[1] == 8
    with pytest.raises(mm.MmmError) as e:
        run.eng.matmul_static_scratch(run.X, run.Y, run.C)
    assert e.value.status == mm.binding.MMM_ERR_WORKSPACE and "static scratch holds" in str(e.value)
    torch.cuda.synchronize()
    assert torch.isnan(run.Cbuf).all()          # nothing was launched
    run.matmul()                                 # the workspace variant still serves it
    torch.cuda.synchronize()
    _, _, C_ref, _ = oracle.run_workload(w)
    np.testing.assert_array_equal(run.C.cpu().numpy(), C_ref)


@pytest.fixture(autouse=True)
def _reset_path():
    yield
    mm.mmm_set_option("matmul_path", -1)
