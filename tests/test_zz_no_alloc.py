"""The entry point that allocates nothing: pvq_correct_static against pvq_correct, through the C library.

Two calls in a row on one GPU, the second with a smaller input, so that the second runs over what the
first left in the library's static work buffers; results must equal pvq_correct's bit for bit (both run
the same kernels in the same order), and pvq_correct's results are the oracle's (tests/test_gpu_correct.py;
one of the cases is checked against the oracle here too)."""
import ctypes as C
import gc

import numpy as np
import pytest

import paper_2410_16926_amd as pvq
import synth_inputs as si
from oracle import pvq_oracle as oracle
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def inputs(rows, cols, seed):
    W0 = np.asarray(si.gaussian_weights(rows, cols, 0.02, seed=seed, rotate=False, bf16=False), dtype=np.float32)
    _, U = si.calibration_hessian(cols, 2 * cols, seed + 1)
    return W0, U


def correct_static_raw(ctx, Wd, Ud):
    """Straight through ctypes: pointers, sizes, the current stream."""
    rows, cols = Wd.shape
    rc = pvq.lib().pvq_correct_static(ctx.handle, C.c_void_p(Wd.data_ptr()), rows, cols, Wd.stride(0),
                                      C.c_void_p(Ud.data_ptr()), Ud.stride(0),
                                      C.c_void_p(torch.cuda.current_stream().cuda_stream))
    return rc


@pytest.mark.parametrize("D,K", [(8, 16), (16, 33)])
def test_two_calls_in_a_row_the_second_smaller(D, K):
    ctx = pvq.pvq_ctx_create(D, K)
    first = True
    for rows, cols, seed in [(700, 384, si.BASE_SEED + 700 + D), (130, 192, si.BASE_SEED + 710 + D)]:
        W0, U = inputs(rows, cols, seed)
        Ud = gu.to_dev_f32(U)
        want = pvq.pvq_correct(ctx, gu.to_dev_f32(W0), Ud).cpu().numpy()
        Wd = gu.to_dev_f32(W0)
        gc.collect()                                            # tensors of earlier tests that are garbage go now, not in between
        before = torch.cuda.memory_allocated()
        assert correct_static_raw(ctx, Wd, Ud) == 0
        assert torch.cuda.memory_allocated() == before          # torch's allocator was not asked either
        got = Wd.cpu().numpy()
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), (rows, cols)
        if first:
            ref, _ = oracle.correct(W0, U, D, K, nthreads=8)
            assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))
            first = False
    ctx.close()


def test_limits_and_errors():
    ctx = pvq.pvq_ctx_create(8, 16)
    limit = pvq.pvq_correct_static_max_rows()
    assert limit == 8192
    cols = 64
    _, U = inputs(1, cols, si.BASE_SEED + 720)
    Ud = gu.to_dev_f32(U)
    # one row too many: refused before anything is launched, the matrix stays as it was
    Wd = torch.ones((limit + 1, cols), dtype=torch.float32, device="cuda")
    assert correct_static_raw(ctx, Wd, Ud) == -2
    assert torch.all(Wd == 1.0)
    # exactly the limit runs, and equals pvq_correct on the same rows
    W0 = np.asarray(si.gaussian_weights(limit, cols, 0.02, seed=si.BASE_SEED + 721, rotate=False, bf16=False), dtype=np.float32)
    want = pvq.pvq_correct(ctx, gu.to_dev_f32(W0), Ud).cpu().numpy()
    Wd = gu.to_dev_f32(W0)
    assert correct_static_raw(ctx, Wd, Ud) == 0
    assert np.array_equal(Wd.cpu().numpy().view(np.uint32), want.view(np.uint32))
    # the checks of pvq_correct
    assert pvq.lib().pvq_correct_static(ctx.handle, None, 4, cols, cols, C.c_void_p(Ud.data_ptr()), cols, None) == -1
    Wd = torch.ones((4, 72), dtype=torch.float32, device="cuda")
    assert correct_static_raw(ctx, Wd[:, :40], Ud) == -2                  # cols not a multiple of 64
    assert correct_static_raw(ctx, torch.ones((0, cols), dtype=torch.float32, device="cuda"), Ud) == 0
    ctx.close()


def test_with_the_python_wrapper_and_the_least_squares_amplitude():
    ctx = pvq.pvq_ctx_create(8, 16)
    ctx.set_amplitude("ls")
    W0, U = inputs(257, 256, si.BASE_SEED + 730)
    Ud = gu.to_dev_f32(U)
    want = pvq.pvq_correct(ctx, gu.to_dev_f32(W0), Ud).cpu().numpy()
    got = pvq.pvq_correct_static(ctx, gu.to_dev_f32(W0), Ud).cpu().numpy()
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    ctx.close()
