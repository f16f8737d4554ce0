"""GPU parity of the error correction (Sec. 3.3 Step 6): the corrected weight matrix must equal the
oracle's bit for bit (every later rounding is decided from these values), and so must its code."""
import numpy as np
import pytest

import paper_2410_16926_amd as pvq
import synth_inputs as si
from oracle import pvq_oracle as oracle
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def run_correct(D, K, rows, cols, seed, amplitude="l2", scale_bits=0, ld_extra=0):
    W0 = np.asarray(si.gaussian_weights(rows, cols, 0.02, seed=seed, rotate=False, bf16=False), dtype=np.float32)
    _, U = si.calibration_hessian(cols, 2 * cols, seed + 1)
    ctx, oe, oc = gu.make_ctx(D, K, scale_bits, cols // D)
    if amplitude == "ls":
        ctx.set_amplitude("ls")
    Wd = torch.zeros((rows, cols + ld_extra), dtype=torch.float32, device="cuda")
    Wd[:, :cols] = gu.to_dev_f32(W0)
    Ud = torch.zeros((cols, cols + ld_extra), dtype=torch.float32, device="cuda")
    Ud[:, :cols] = gu.to_dev_f32(U)
    Wv, Uv = Wd[:, :cols], Ud[:, :cols]
    pvq.pvq_correct(ctx, Wv, Uv)
    torch.cuda.synchronize()
    got = Wv.cpu().numpy()
    ref, _ = oracle.correct(W0, U, D, K, amplitude=amplitude, nthreads=8)
    bad = np.argwhere(got.view(np.uint32) != ref.view(np.uint32))
    assert bad.size == 0, f"{bad.shape[0]} corrected weights differ, first at {bad[0]}: {got[tuple(bad[0])]} vs {ref[tuple(bad[0])]}"
    if ld_extra:
        assert torch.all(Wd[:, cols:] == 0)
    # and the code of the corrected matrix is the oracle's code of its corrected matrix
    packed = pvq.pvq_encode(ctx, Wv.contiguous(), want_pulses=True)
    enc = oracle.encode(ref, D, K, scale_bits, oe, nthreads=8, amplitude=amplitude)
    gu.assert_encode_equal(packed, enc)
    ctx.close()
    return W0, ref


@pytest.mark.parametrize("D,K,rows,cols,amplitude", [
    (8, 16, 200, 256, "l2"), (8, 16, 70, 512, "ls"), (8, 16, 1, 64, "l2"), (8, 16, 129, 192, "l2"),
    (16, 33, 130, 256, "l2"), (16, 33, 65, 128, "ls"), (32, 60, 64, 128, "l2"), (32, 60, 131, 320, "ls"),
    (8, 5, 300, 128, "l2")])
def test_corrected_weights_equal_the_oracles(D, K, rows, cols, amplitude):
    run_correct(D, K, rows, cols, seed=si.BASE_SEED + 500 + rows + cols, amplitude=amplitude)


def test_corrected_weights_with_amplitude_codes_and_leading_dimensions():
    # amplitude codes (Sec. 3.3 Step 5) are formed when the corrected matrix is encoded; W and U as views
    run_correct(8, 16, 96, 1024, seed=si.BASE_SEED + 541, scale_bits=2, ld_extra=12)


def test_a_wider_matrix():
    # 24 blocks of 64 columns, row tiles with a ragged end: the order of the updates across blocks
    run_correct(8, 16, 700, 1536, seed=si.BASE_SEED + 542)


@pytest.mark.parametrize("D,K,rows,cols", [(8, 16, 1100, 448), (16, 33, 300, 640), (32, 60, 150, 384), (8, 16, 2100, 320)])
def test_wide_updates_beside_the_next_panel(D, K, rows, cols):
    # from the third panel on a launch holds panel workgroups and update tiles of the panel before (several row
    # tiles and column tiles, ragged ends), and the panels' t values alternate between two buffers; an odd number
    # of 64-column blocks ends in a half panel; the call is repeated on the same context
    W0, ref = run_correct(D, K, rows, cols, seed=si.BASE_SEED + 543 + rows)
    ctx = pvq.pvq_ctx_create(D, K)
    _, U = si.calibration_hessian(cols, 2 * cols, si.BASE_SEED + 543 + rows + 1)
    Ud = gu.to_dev_f32(U)
    for _ in range(2):
        Wd = gu.to_dev_f32(W0)
        pvq.pvq_correct(ctx, Wd, Ud)
        # work queued behind the call on the caller's stream sees the finished matrix
        got = (Wd + 0.0).cpu().numpy()
        assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))
    ctx.close()


@pytest.mark.parametrize("D,K,rows,cols,amplitude", [(8, 16, 700, 1536, "l2"), (8, 16, 130, 448, "ls"), (16, 33, 300, 640, "l2"),
                                                     (32, 60, 150, 384, "ls"), (8, 5, 65, 320, "l2")])
def test_narrow_update_inside_the_panel_workgroups(D, K, rows, cols, amplitude):
    # a launch with many update tiles lets its panel workgroups apply the panel before's update to their own
    # columns instead of a launch of its own; the threshold is lowered so that these small matrices take that path
    # in every launch that has update tiles at all (the last two panels of a matrix keep the separate launch)
    old = pvq.pvq_correct_set_front_tiles(1)
    try:
        run_correct(D, K, rows, cols, seed=si.BASE_SEED + 580 + rows + cols, amplitude=amplitude)
    finally:
        assert pvq.pvq_correct_set_front_tiles(old) == 1


@pytest.mark.parametrize("rows,cols", [(200, 256), (1100, 640)])
def test_the_call_can_be_captured_in_a_graph_and_replayed(rows, cols):
    # kernels only, all on the capturing stream; every replay must reproduce the eager result for the weights
    # then in the buffer
    D, K = 8, 16
    ctx = pvq.pvq_ctx_create(D, K)
    _, U = si.calibration_hessian(cols, 2 * cols, si.BASE_SEED + 561)
    Ud = gu.to_dev_f32(U)
    W = torch.empty((rows, cols), dtype=torch.float32, device="cuda")
    work = torch.empty((rows * 1024,), dtype=torch.uint8, device="cuda")

    def fill(seed):
        W.copy_(gu.to_dev_f32(si.gaussian_weights(rows, cols, 0.02, seed=si.BASE_SEED + seed, rotate=False, bf16=False)))

    fill(1)
    pvq.pvq_correct(ctx, W, Ud, work=work)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    fill(1)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            pvq.pvq_correct(ctx, W, Ud, work=work)
    torch.cuda.synchronize()
    for seed in (2, 3, 4):
        fill(seed)
        pvq.pvq_correct(ctx, W, Ud, work=work)
        torch.cuda.synchronize()
        want = W.clone()
        fill(seed)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(want, W)
    ctx.close()


def test_random_configurations():
    # seeded sweep: group size, pulse count, shape, amplitude kind, weight scale (bf16-valued weights in
    # every third case: exact ties are likelier) and damping drawn at random
    rng = np.random.default_rng(si.BASE_SEED + 570)
    for case in range(16):
        D = int(rng.choice([8, 16, 32]))
        K = int(rng.integers(1, {8: 22, 16: 40, 32: 70}[D]))
        rows = int(rng.integers(1, 400)); cols = 64 * int(rng.integers(1, 8))
        amp = str(rng.choice(["l2", "ls"]))
        sigma = float(rng.choice([1e-3, 0.02, 1.0, 50.0]))
        W0 = np.asarray(si.gaussian_weights(rows, cols, sigma, seed=3000 + case, rotate=False, bf16=False), dtype=np.float32)
        if case % 3 == 0:
            W0 = si.bf16_bits_to_f32(si.f32_to_bf16_bits(W0))
        _, U = si.calibration_hessian(cols, 2 * cols, 4000 + case, damp=float(rng.choice([0.01, 0.1])))
        ctx = pvq.pvq_ctx_create(D, K)
        if amp == "ls":
            ctx.set_amplitude("ls")
        Wd = gu.to_dev_f32(W0)
        pvq.pvq_correct(ctx, Wd, gu.to_dev_f32(U))
        ref, _ = oracle.correct(W0, U, D, K, amplitude=amp, nthreads=8)
        assert np.array_equal(Wd.cpu().numpy().view(np.uint32), ref.view(np.uint32)), (case, D, K, rows, cols, amp, sigma)
        ctx.close()


def test_corrected_code_has_the_lower_proxy_loss():
    # the point of the step (Sec. 2.1, Sec. 3.3 Step 6), end to end through the library: rotate-free synthetic
    # weights, correct, encode, decode; Tr((W - W_hat) H (W - W_hat)^T) against the plain code of the same matrix
    D, K, rows, cols = 8, 16, 48, 512
    W0 = np.asarray(si.gaussian_weights(rows, cols, 0.02, seed=93, rotate=False, bf16=False), dtype=np.float32)
    H, U = si.calibration_hessian(cols, 2 * cols, 94)
    ctx, _, _ = gu.make_ctx(D, K, 2, cols // D)

    def loss(What):
        d = W0.astype(np.float64) - What.astype(np.float64)
        return np.einsum("ri,ij,rj->", d, H, d)

    plain = pvq.pvq_decode(ctx, pvq.pvq_encode(ctx, gu.to_dev_f32(W0)), torch.float32).cpu().numpy()
    Wd = gu.to_dev_f32(W0)
    pvq.pvq_correct(ctx, Wd, gu.to_dev_f32(U))
    corrected = pvq.pvq_decode(ctx, pvq.pvq_encode(ctx, Wd), torch.float32).cpu().numpy()
    assert loss(corrected) < 0.7 * loss(plain)
    ctx.close()


@pytest.mark.parametrize("D,K", [(8, 16), (16, 33)])
def test_rounding_and_repair_ties_in_the_first_group(D, K):
    # every row starts with an adversarial group (half-integers after projection, repeated magnitudes, zeros,
    # one-hot, wide dynamic range): its point decides what the later columns receive
    rows, cols = 4096, 128
    W0 = np.asarray(si.gaussian_weights(rows, cols, 0.02, seed=97, rotate=False, bf16=False), dtype=np.float32)
    W0[:, :D] = si.adversarial_groups(rows, D, seed=98).reshape(rows, D)
    _, U = si.calibration_hessian(cols, 2 * cols, 99)
    ctx = pvq.pvq_ctx_create(D, K)
    Wd = gu.to_dev_f32(W0)
    pvq.pvq_correct(ctx, Wd, gu.to_dev_f32(U))
    ref, _ = oracle.correct(W0, U, D, K, nthreads=8)
    got = Wd.cpu().numpy()
    finite = np.isfinite(ref).all(axis=1)
    assert finite.sum() > rows * 0.9
    bad = np.argwhere(got[finite].view(np.uint32) != ref[finite].view(np.uint32))
    assert bad.size == 0, f"{bad.shape[0]} differ, first {bad[0]}"
    ctx.close()


def test_rows_that_are_not_finite_do_not_disturb_the_others():
    # rows are independent: rows of zeros, with infinities or not-a-numbers give unspecified values in those
    # rows only (and no fault); every other row still equals the oracle's
    D, K, rows, cols = 8, 16, 70, 256
    W0 = np.asarray(si.gaussian_weights(rows, cols, 0.02, seed=95, rotate=False, bf16=False), dtype=np.float32)
    W0[3] = 0.0
    W0[10, 17] = np.inf
    W0[20, 100] = np.nan
    W0[33, :8] = 3.0e38
    W0[47, 64:72] = 1.0e-44
    _, U = si.calibration_hessian(cols, 2 * cols, 96)
    ctx = pvq.pvq_ctx_create(D, K)
    Wd = gu.to_dev_f32(W0)
    pvq.pvq_correct(ctx, Wd, gu.to_dev_f32(U))
    torch.cuda.synchronize()
    got = Wd.cpu().numpy()
    ref, _ = oracle.correct(W0, U, D, K)
    clean = np.array([r for r in range(rows) if r not in (10, 20, 33)])
    assert np.array_equal(got[clean].view(np.uint32), ref[clean].view(np.uint32))
    assert np.all(got[3] == 0.0)
    ctx.close()


def test_entries_below_the_diagonal_are_not_used():
    D, K, rows, cols = 8, 16, 90, 192
    W0 = np.asarray(si.gaussian_weights(rows, cols, 0.02, seed=91, rotate=False, bf16=False), dtype=np.float32)
    _, U = si.calibration_hessian(cols, 2 * cols, 92)
    ref, _ = oracle.correct(W0, U, D, K)
    ctx = pvq.pvq_ctx_create(D, K)
    Wd = gu.to_dev_f32(W0)
    Ud = gu.to_dev_f32(U + np.tril(np.full((cols, cols), np.nan, dtype=np.float32), -1))
    pvq.pvq_correct(ctx, Wd, Ud)
    assert np.array_equal(Wd.cpu().numpy().view(np.uint32), ref.view(np.uint32))
    ctx.close()


def test_uncorrelated_inputs_leave_the_weights_alone():
    D, K, rows, cols = 8, 16, 50, 256
    W0 = np.asarray(si.gaussian_weights(rows, cols, 0.02, seed=77, rotate=False, bf16=False), dtype=np.float32)
    ctx = pvq.pvq_ctx_create(D, K)
    Wd = gu.to_dev_f32(W0)
    Ud = torch.diag(torch.linspace(0.5, 2.0, cols, device="cuda"))
    pvq.pvq_correct(ctx, Wd, Ud)
    assert np.array_equal(Wd.cpu().numpy().view(np.uint32), W0.view(np.uint32))
    ctx.close()


def test_argument_errors():
    ctx = pvq.pvq_ctx_create(8, 16)
    W = torch.zeros((4, 96), dtype=torch.float32, device="cuda")
    U = torch.eye(96, device="cuda")
    with pytest.raises(pvq.PvqError) as e:          # columns not in whole blocks of 64
        pvq.pvq_correct(ctx, W, U)
    assert e.value.status == -2
    W = torch.zeros((4, 128), dtype=torch.float32, device="cuda")
    U = torch.eye(128, device="cuda")
    with pytest.raises(pvq.PvqError) as e:          # work buffer too small
        pvq.pvq_correct(ctx, W, U, work=torch.empty((512,), dtype=torch.uint8, device="cuda"))
    assert e.value.status == -1
    pvq.pvq_correct(ctx, W[:0], U)                  # no rows: nothing to do
    ctx.close()
    wide = pvq.pvq_ctx_create(128, 187)
    with pytest.raises(pvq.PvqError) as e:
        pvq.pvq_correct(wide, W, U)
    assert e.value.status == -2
    wide.close()
