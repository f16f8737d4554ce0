"""GPU parity: the library (through its C ABI) against the CPU oracle on the same seeded inputs.
Integer results (pulse vectors, packed indices, amplitude codes) and the encoder's float32 values
must be identical; decoded weights within 1e-6 relative (float32) / 1 ulp (16-bit outputs); the
fused product within 1e-3 relative."""
import numpy as np
import pytest

import paper_2410_16926_amd as pvq
import synth_inputs as si
from oracle import pvq_oracle as oracle
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def run_case(W32, D, K, scale_bits, src_bits=None, batches=(1, 4), out_dtypes=("f32", "f16", "bf16"), seed=1,
             amplitude="l2"):
    rows, cols = W32.shape
    G = cols // D
    ctx, oe, oc = gu.make_ctx(D, K, scale_bits, G)
    if amplitude == "ls":
        ctx.set_amplitude("ls")
    Wd = gu.to_dev_bf16(src_bits) if src_bits is not None else gu.to_dev_f32(W32)
    packed = pvq.pvq_encode(ctx, Wd, want_pulses=True)
    torch.cuda.synchronize()
    enc = oracle.encode(W32, D, K, scale_bits, oe, nthreads=8, amplitude=amplitude)
    gu.assert_encode_equal(packed, enc)

    ref, _, _ = oracle.decode(enc, oc, nthreads=8)
    for setting in gu.decoder_settings(D):          # groups of 8: both decoders, whatever the matrix's size
        with gu.decoder_setting(setting):
            if "f32" in out_dtypes:
                got = pvq.pvq_decode(ctx, packed, torch.float32).cpu().numpy()
                gu.assert_decode_close(got, ref)
            if "f16" in out_dtypes:
                got = pvq.pvq_decode(ctx, packed, torch.float16).cpu().numpy()
                assert gu.ulp_f16(oracle.to_f16(ref).view(np.uint16), got.view(np.uint16)) <= 1
            if "bf16" in out_dtypes:
                got = gu.bf16_tensor_bits(pvq.pvq_decode(ctx, packed, torch.bfloat16))
                assert gu.ulp_f16(oracle.to_bf16_bits(ref), got) <= 1
    for B in batches:
        xf, xb = si.activations(B, cols, seed=seed + B)
        y = pvq.pvq_decode_gemv(ctx, packed, gu.to_dev_bf16(xb)).cpu().numpy()
        want = xf.astype(np.float64) @ ref.T
        gu.assert_gemv_close(y, want, gu.product_scale(xf, ref))
    ctx.close()
    return packed, enc


def test_config0_512x512_fp32_amplitudes():
    # 512x512 float32, N(0, 0.02^2), rotated; D=8, 24-bit indices (K=16), float32 amplitudes
    W = si.gaussian_weights(512, 512, 0.02, seed=si.BASE_SEED + 0)
    K = pvq.pvq_max_k(8, 24)
    assert K == 16
    run_case(W, 8, K, 0, batches=(1, 3, 16))


@pytest.mark.parametrize("bits", [8, 2, 4, 1])
def test_amplitude_codes_bf16_source(bits):
    # the Llama-3-8B up-projection family (bf16 source, N(0, 0.015^2), 4096 inputs), a row slice
    wf, wb = si.gaussian_weights(192, 4096, 0.015, seed=si.BASE_SEED + 1, bf16=True)
    run_case(wf, 8, 16, bits, src_bits=wb, batches=(1, 4, 16) if bits in (2, 8) else (1, 4))


@pytest.mark.parametrize("D,budget", [(16, 52), (32, 104), (16, 64), (8, 40), (16, 30), (32, 32)])
def test_wide_indices(D, budget):
    # multi-word indices: 52-bit (2 words) and 104-bit (4 words), plus widths that do not fill
    # their words and single-word indices at D=16/32
    K = pvq.pvq_max_k(D, budget)
    wf, wb = si.gaussian_weights(96, 2048, 0.015, seed=si.BASE_SEED + 2 + D, bf16=True)
    run_case(wf, D, K, 0, src_bits=wb, batches=(1, 2))


@pytest.mark.parametrize("K,bits", [(5, 0), (9, 2), (13, 8), (17, 2), (17, 0)])
def test_d8_other_pulse_counts(K, bits):
    # D = 8 with index widths other than 24 bits (13, 18, 22 and 25): the table-driven kernels with
    # indices that straddle words at varying offsets
    wf, wb = si.gaussian_weights(160, 2048, 0.015, seed=si.BASE_SEED + 60 + K, bf16=True)
    run_case(wf, 8, K, bits, src_bits=wb, batches=(1, 2, 5))


@pytest.mark.parametrize("rows,cols,K,bits", [(8192 + 21, 2048, 16, 2), (8192, 4096, 16, 0), (8200, 2048, 16, 8),
                                              (8192 + 5, 2048, 13, 2), (8192 + 16, 6144, 16, 2)])
def test_single_vector_on_tall_matrices(rows, cols, K, bits):
    # from 8192 rows on (32 per wave of a 256-unit GPU) and rows of whole slices of 256 groups, one vector goes
    # to the kernel in which every wave owns whole rows: a last workgroup with fewer rows, one to three
    # slices, fused gain table / amplitude table / float32 amplitudes, indices that are not 24 bits wide
    wf, wb = si.gaussian_weights(rows, cols, 0.015, seed=si.BASE_SEED + 80 + rows + cols + K, bf16=True)
    run_case(wf, 8, K, bits, src_bits=wb, batches=(1, 2), out_dtypes=())


@pytest.mark.parametrize("D,budget,bits,bf16", [(8, 24, 0, True), (8, 24, 2, True), (8, 24, 8, False),
                                                (16, 52, 0, False), (16, 52, 4, True), (32, 104, 0, True)])
def test_least_squares_amplitudes(D, budget, bits, bf16):
    # Sec. 3.3 Step 4 amplitudes (and their codes) instead of group norms; D = 16 with 4-bit codes is
    # the paper's 3.25 bits/weight setting
    K = pvq.pvq_max_k(D, budget)
    if bf16:
        wf, wb = si.gaussian_weights(128, 2048, 0.015, seed=si.BASE_SEED + 70 + D + bits, bf16=True)
        run_case(wf, D, K, bits, src_bits=wb, batches=(1, 4), amplitude="ls")
    else:
        W = si.gaussian_weights(128, 2048, 0.02, seed=si.BASE_SEED + 70 + D + bits)
        run_case(W, D, K, bits, batches=(1,), amplitude="ls")


def test_least_squares_amplitudes_adversarial():
    # ties, zeros (amplitude 0), one-hot groups, wide dynamic range
    n = 1 << 14
    W = si.adversarial_groups(n, 8, seed=91).reshape(n * 8 // 2048, 2048)
    run_case(W, 8, 16, 0, batches=(1,), out_dtypes=("f32",), amplitude="ls")
    run_case(W, 8, 16, 2, batches=(1,), out_dtypes=("f32",), amplitude="ls")


@pytest.mark.parametrize("D,budget,bits", [(16, 52, 4), (32, 104, 8)])
def test_wide_indices_with_codes(D, budget, bits):
    K = pvq.pvq_max_k(D, budget)
    W = si.gaussian_weights(64, 1024, 0.02, seed=si.BASE_SEED + 20 + D)
    run_case(W, D, K, bits, batches=(1,))


@pytest.mark.parametrize("rows,cols,D", [(1, 8, 8), (3, 8 * 37, 8), (5, 8 * 257, 8), (7, 16 * 33, 16),
                                         (2, 32 * 9, 32), (257, 8 * 3, 8), (4, 8 * 3584, 8)])
def test_ragged_shapes(rows, cols, D):
    # partial tiles, a single group, odd group counts (odd leftovers in the row sum), long rows
    K = pvq.pvq_max_k(D, 3 * D)
    W = si.gaussian_weights(rows, cols, 0.02, seed=si.BASE_SEED + rows + cols, rotate=False)
    run_case(W, D, K, 0, batches=(1,), out_dtypes=("f32",))
    if cols // D >= 2:
        run_case(W, D, K, 2, batches=(1,), out_dtypes=("f32",))


@pytest.mark.parametrize("rows,cols,bits", [(1, 8 * 4, 0), (5, 8 * 296, 2), (37, 8 * 1000, 8), (3, 8 * 3584, 2),
                                            (130, 8 * 64, 0)])
def test_many_vectors_on_ragged_shapes(rows, cols, bits):
    # the 16-vector pass (one group column per lane) with partial slices, few rows, rows that do not
    # fill a batch; and a batch size that the narrower passes share (4 + 2 + 1)
    wf, wb = si.gaussian_weights(rows, cols, 0.015, seed=si.BASE_SEED + 80 + rows, rotate=False, bf16=True)
    run_case(wf, 8, 16, bits, src_bits=wb, batches=(16, 11, 8, 7), out_dtypes=("bf16",))


@pytest.mark.parametrize("rows,cols,bits", [(1, 8 * 256, 0), (37, 8 * 256, 2), (130, 8 * 768, 8), (19, 8 * 1024, 2),
                                            (300, 8 * 512, 1), (16, 8 * 1024, 4), (33, 8 * 1024, 0),
                                            (120, 8 * 320, 2), (49, 8 * 448, 0), (97, 8 * 832, 2)])
def test_many_vectors_on_the_matrix_cores(rows, cols, bits):
    # 3..16 vectors with rows of 4, 5, 7, 8, 12, 13, 16 slabs of 64 groups: the pass whose dot products
    # run as 4x4x4 matrix instructions, one to four per half group; row counts that leave partial tiles of 16 rows and rounds of
    # four, two and one tile, every amplitude format
    wf, wb = si.gaussian_weights(rows, cols, 0.015, seed=si.BASE_SEED + 90 + rows, rotate=False, bf16=True)
    run_case(wf, 8, 16, bits, src_bits=wb, batches=(16, 5, 9, 13, 3), out_dtypes=())


@pytest.mark.parametrize("rows,cols,bits", [(21, 8 * 1088, 2), (40, 8 * 1792, 2), (17, 8 * 3584, 0), (3, 8 * 2048, 8),
                                            (70, 8 * 1984, 1)])
def test_many_vectors_on_the_matrix_cores_long_rows(rows, cols, bits):
    # rows of more than 16 slabs (17, 28, 56, 32, 31): the sixteen waves of a row tile take several slabs
    # each, some one more than others
    wf, wb = si.gaussian_weights(rows, cols, 0.015, seed=si.BASE_SEED + 95 + rows, rotate=False, bf16=True)
    run_case(wf, 8, 16, bits, src_bits=wb, batches=(16, 5, 3), out_dtypes=())


@pytest.mark.parametrize("rows,cols,bits,batch", [(4111, 8 * 320, 2, 5), (9001, 8 * 512, 0, 16), (20481, 8 * 256, 8, 3)])
def test_many_vectors_with_several_row_tiles_per_workgroup(rows, cols, bits, batch):
    # more than 256 tiles of 16 rows: workgroups own two to six tiles (the last one partial) and take them in
    # rounds of four, two and one
    wf, wb = si.gaussian_weights(rows, cols, 0.015, seed=si.BASE_SEED + 96 + rows, rotate=False, bf16=True)
    run_case(wf, 8, 16, bits, src_bits=wb, batches=(batch,), out_dtypes=())


@pytest.mark.parametrize("D,K", [(8, 16), (16, 33), (32, 60), (8, 1), (8, 127)])
def test_adversarial_groups(D, K):
    # rounding ties, repair ties, zeros, one-hot, wide dynamic range; 64k groups
    n = 1 << 16
    W = si.adversarial_groups(n, D, seed=77 + D + K).reshape(n * D // 2048, 2048)
    run_case(W, D, K, 0, batches=(1,), out_dtypes=("f32",))


def run_long_groups(X32, D, K, src_bits=None, amplitude="l2", want_pulses=False):
    """Groups of 64 / 128 values (the on-the-fly activation setting): indices and float32 amplitudes
    identical to the oracle's, decoded values within 1e-6 relative / 1 ulp; the fused product does
    not exist for them."""
    rows, cols = X32.shape
    ctx = pvq.pvq_ctx_create(D, K)
    assert ctx.index_bits == oracle.index_bits(D, K)
    if amplitude == "ls":
        ctx.set_amplitude("ls")
    Xd = gu.to_dev_bf16(src_bits) if src_bits is not None else gu.to_dev_f32(X32)
    packed = pvq.pvq_encode(ctx, Xd, want_pulses=want_pulses)
    torch.cuda.synchronize()
    enc = oracle.encode(X32, D, K, 0, None, nthreads=8, amplitude=amplitude)
    gu.assert_encode_equal(packed, enc, check_pulses=want_pulses)
    ref, _, _ = oracle.decode(enc, None, nthreads=8)
    gu.assert_decode_close(pvq.pvq_decode(ctx, packed, torch.float32).cpu().numpy(), ref)
    got = pvq.pvq_decode(ctx, packed, torch.float16).cpu().numpy()
    assert gu.ulp_f16(oracle.to_f16(ref).view(np.uint16), got.view(np.uint16)) <= 1
    got = gu.bf16_tensor_bits(pvq.pvq_decode(ctx, packed, torch.bfloat16))
    assert gu.ulp_f16(oracle.to_bf16_bits(ref), got) <= 1
    with pytest.raises(pvq.PvqError) as e:
        pvq.pvq_decode_gemv(ctx, packed, torch.zeros((1, cols), dtype=torch.bfloat16, device="cuda"))
    assert e.value.status == -2
    ctx.close()


@pytest.mark.parametrize("D,bits_per_value,tokens,hidden", [(128, 3, 48, 2048), (128, 2, 33, 1024), (128, 4, 9, 1024),
                                                            (64, 3, 40, 1024), (64, 2, 17, 64 * 13), (128, 3, 1, 128)])
def test_long_groups_bf16_activations(D, bits_per_value, tokens, hidden):
    # D = 128 at 3 bits per value is K = 187 with 384-bit indices (12 words); 2 and 4 bits give 8- and
    # 16-word integers; D = 64 likewise with 6, 4 words.  Index widths that are no multiple of 32 pack
    # several groups into a tile of whole words (ragged last tile at 13 groups per row)
    K = pvq.pvq_max_k(D, bits_per_value * D - (2 if bits_per_value == 4 else 0))
    xf, xb = si.activation_matrix(tokens, hidden, seed=si.BASE_SEED + D + bits_per_value,
                                  rotate=(hidden & (hidden - 1)) == 0)
    run_long_groups(xf, D, K, src_bits=xb)


@pytest.mark.parametrize("D,K,tokens,hidden,bf16", [(128, 187, 300, 8192, True), (128, 84, 260, 8192, False),
                                                    (64, 40, 1300, 64 * 13, True), (64, 96, 520, 2048, False),
                                                    (128, 1, 130, 128 * 130, True)])
def test_long_groups_large_batches(D, K, tokens, hidden, bf16):
    # from 16384 groups on the encoder works with 16 lanes per group, four groups per wave: 12-, 8- and
    # 4-word integers, 13 groups per row (a last tile with one of four groups), widths of 123 bits
    if bf16:
        xf, xb = si.activation_matrix(tokens, hidden, seed=si.BASE_SEED + D + K, rotate=False)
        run_long_groups(xf, D, K, src_bits=xb)
        run_long_groups(xf, D, K, src_bits=xb, amplitude="ls")
    else:
        X = si.activation_matrix(tokens, hidden, seed=si.BASE_SEED + D + K, rotate=False, bf16=False)
        run_long_groups(X, D, K, want_pulses=K <= 127)


@pytest.mark.parametrize("D,K", [(128, 187), (64, 40), (64, 127), (128, 1), (64, 2), (128, 382)])
def test_long_groups_float32_and_odd_widths(D, K):
    # float32 source without rotation (outlier channels stay: a few huge coordinates per group), index
    # widths of 123 bits (64, 40) and others that straddle words, int8 pulse plane where K allows it
    X = si.activation_matrix(21, D * 7, seed=si.BASE_SEED + D + K, rotate=False, bf16=False)
    run_long_groups(X, D, K, want_pulses=K <= 127)
    run_long_groups(X, D, K, amplitude="ls")


@pytest.mark.parametrize("D,K", [(128, 187), (64, 40)])
def test_long_groups_adversarial(D, K):
    # rounding ties, repair ties, zeros (index 0, amplitude 0), one-hot groups, wide dynamic range
    # 2048 groups (a wave per group) and 32768 groups (16 lanes per group)
    for n in (1 << 11, 1 << 15):
        X = si.adversarial_groups(n, D, seed=55 + D).reshape(n * D // 1024, 1024)
        run_long_groups(X, D, K)
        run_long_groups(X, D, K, amplitude="ls")


@pytest.mark.parametrize("tokens,hidden,block,bits_per_value,bf16", [(5, 8192, 8192, 3, True), (3, 16384, 8192, 3, False),
                                                                     (9, 4096, 4096, 3, True), (4, 12288, 4096, 2, False),
                                                                     (7, 2048, 512, 3, True), (6, 6144, 2048, 3, True),
                                                                     (2, 3072, 1024, 2, False), (300, 8192, 8192, 3, True)])
def test_rotation_and_encoding_in_one_kernel(tokens, hidden, block, bits_per_value, bf16):
    # pvq_rotate_encode must give exactly what the oracle's rotation (float32) followed by the oracle's
    # encoder gives: the rotated values stay in registers in the same float32 bits
    D = 128
    K = pvq.pvq_max_k(D, bits_per_value * D)
    rng = np.random.default_rng(tokens + hidden + block)
    sg = rng.integers(0, 2, size=hidden).astype(np.uint8)
    if bf16:
        xf, xb = si.activation_matrix(tokens, hidden, seed=si.BASE_SEED + block, rotate=False)
        Xd = gu.to_dev_bf16(xb)
    else:
        xf = si.activation_matrix(tokens, hidden, seed=si.BASE_SEED + block, rotate=False, bf16=False)
        Xd = gu.to_dev_f32(xf)
    rotated = oracle.hadamard_rows(xf, block, sg)
    for amplitude in ("l2", "ls"):
        ctx = pvq.pvq_ctx_create(D, K)
        ctx.set_amplitude({"l2": "norm", "ls": "ls"}[amplitude])
        packed = pvq.pvq_rotate_encode(ctx, Xd, block, torch.from_numpy(sg).cuda())
        torch.cuda.synchronize()
        enc = oracle.encode(rotated, D, K, 0, None, nthreads=8, amplitude=amplitude)
        gu.assert_encode_equal(packed, enc, check_pulses=False)
        # and the two separate calls agree with it as well
        two = pvq.pvq_encode(ctx, pvq.pvq_hadamard(Xd, block, torch.from_numpy(sg).cuda(), out_dtype=torch.float32))
        assert torch.equal(two.index, packed.index) and torch.equal(two.scale, packed.scale)
        ctx.close()
    # without signs
    ctx = pvq.pvq_ctx_create(D, K)
    packed = pvq.pvq_rotate_encode(ctx, Xd, block)
    enc = oracle.encode(oracle.hadamard_rows(xf, block), D, K, 0, None, nthreads=8)
    gu.assert_encode_equal(packed, enc, check_pulses=False)
    ctx.close()


@pytest.mark.parametrize("rows,cols,block,bits,bf16", [(5, 8192, 8192, 2, True), (3, 8192, 4096, 0, False),
                                                       (9, 4096, 4096, 8, True), (4, 2048, 512, 2, True),
                                                       (7, 2048, 64, 0, True), (3, 16384, 8192, 2, False),
                                                       (130, 8192, 1024, 2, True), (2, 6144, 2048, 4, True),
                                                       (1, 32768, 8, 1, False), (70, 8192, 8192, 0, True),
                                                       (40, 8192, 1024, 0, False)])
def test_rotation_and_encoding_in_one_kernel_for_groups_of_8(rows, cols, block, bits, bf16):
    # the weight path (Sec. 3.3 Steps 1, 3-5): rotate the rows, encode groups of 8 to 24-bit indices with float32
    # amplitudes or amplitude codes; indices, amplitudes / codes and row normalisers must be those of the oracle's
    # rotation (float32) followed by the oracle's encoder, and those of the two separate calls
    D, K = 8, 16
    rng = np.random.default_rng(rows + cols + block)
    sg = rng.integers(0, 2, size=cols).astype(np.uint8)
    if bf16:
        wf, wb = si.gaussian_weights(rows, cols, 0.02, seed=si.BASE_SEED + 300 + block, rotate=False, bf16=True)
        Xd = gu.to_dev_bf16(wb)
    else:
        wf = si.gaussian_weights(rows, cols, 0.02, seed=si.BASE_SEED + 300 + block, rotate=False)
        Xd = gu.to_dev_f32(wf)
    rotated = oracle.hadamard_rows(wf, block, sg)
    sgd = torch.from_numpy(sg).cuda()
    for amplitude in ("l2", "ls"):
        ctx, oe, oc = gu.make_ctx(D, K, bits, cols // D)
        ctx.set_amplitude({"l2": "norm", "ls": "ls"}[amplitude])
        packed = pvq.pvq_rotate_encode(ctx, Xd, block, sgd)
        torch.cuda.synchronize()
        enc = oracle.encode(rotated, D, K, bits, oe, nthreads=8, amplitude=amplitude)
        gu.assert_encode_equal(packed, enc, check_pulses=False)
        two = pvq.pvq_encode(ctx, pvq.pvq_hadamard(Xd, block, sgd, out_dtype=torch.float32))
        assert torch.equal(two.index, packed.index) and torch.equal(two.scale, packed.scale)
        if bits:
            assert torch.equal(two.rownorm, packed.rownorm)
        ctx.close()
    ctx, oe, oc = gu.make_ctx(D, K, bits, cols // D)           # without signs
    packed = pvq.pvq_rotate_encode(ctx, Xd, block)
    gu.assert_encode_equal(packed, oracle.encode(oracle.hadamard_rows(wf, block), D, K, bits, oe, nthreads=8), check_pulses=False)
    ctx.close()


def test_rotation_and_encoding_for_groups_of_8_limits():
    X = torch.zeros((2, 1024), dtype=torch.float32, device="cuda")
    ctx = pvq.pvq_ctx_create(8, 16)
    for block in (4, 96, 2048):                               # too small, no power of two, not dividing
        with pytest.raises(pvq.PvqError) as e:
            pvq.pvq_rotate_encode(ctx, X, block)
        assert e.value.status == -2
    with pytest.raises(pvq.PvqError) as e:
        pvq.pvq_rotate_encode(ctx, X, 1024)                   # 128 groups: not a whole chunk of 256
    assert e.value.status == -2
    ctx.close()
    ctx = pvq.pvq_ctx_create(8, 13)                           # 22-bit indices: no fused kernel
    with pytest.raises(pvq.PvqError) as e:
        pvq.pvq_rotate_encode(ctx, torch.zeros((2, 2048), dtype=torch.float32, device="cuda"), 512)
    assert e.value.status == -2
    ctx.close()
    e2, c2 = pvq.pvq_beta_tables(8, 256, 2)
    ctx = pvq.pvq_ctx_create(8, 16, 2, e2, c2)                # amplitude codes need the row normaliser's plane
    Xz = torch.zeros((2, 2048), dtype=torch.float32, device="cuda")
    p = pvq.alloc_packed(ctx, 2, 2048, Xz.device)
    import ctypes as C
    rc = pvq.lib().pvq_rotate_encode(ctx.handle, C.c_void_p(Xz.data_ptr()), 0, 2, 2048, 2048, 512, None,
                                     C.c_void_p(p.index.data_ptr()), C.c_void_p(p.scale.data_ptr()), None, None)
    assert rc == -1
    ctx.close()


def test_rotation_and_encoding_argument_errors():
    X = torch.zeros((2, 1024), dtype=torch.float32, device="cuda")
    ctx8 = pvq.pvq_ctx_create(8, 16)
    with pytest.raises(pvq.PvqError) as e:
        pvq.pvq_rotate_encode(ctx8, X, 1024)                 # groups of 8: 128 groups are not a whole chunk
    assert e.value.status == -2
    ctx8.close()
    ctx = pvq.pvq_ctx_create(128, 187)
    for block in (64, 96, 2048, 16384):                      # too small, no power of two, not dividing, too large
        with pytest.raises(pvq.PvqError) as e:
            pvq.pvq_rotate_encode(ctx, X, block)
        assert e.value.status == -2
    ctx.close()
    ctx = pvq.pvq_ctx_create(128, 186)                       # 383-bit indices: 16 groups do not fill whole words
    with pytest.raises(pvq.PvqError) as e:
        pvq.pvq_rotate_encode(ctx, X, 1024)
    assert e.value.status == -2
    ctx.close()


def test_long_groups_argument_errors():
    with pytest.raises(pvq.PvqError) as e:
        pvq.pvq_ctx_create(128, 400)              # N(128,400) needs more than 512 bits
    assert e.value.status == -2
    e2, c2 = pvq.pvq_beta_tables(128, 64, 2)
    with pytest.raises(pvq.PvqError) as e:
        pvq.pvq_ctx_create(128, 187, 2, e2, c2)   # amplitude codes are for small groups only
    assert e.value.status == -2
    ctx = pvq.pvq_ctx_create(128, 187)
    X = torch.zeros((2, 256), dtype=torch.float32, device="cuda")
    with pytest.raises(pvq.PvqError) as e:
        pvq.pvq_encode(ctx, X, want_pulses=True)  # no int8 pulse plane above K = 127
    assert e.value.status == -2
    out = pvq.pvq_encode(ctx, X)                  # all-zero groups: index 0, amplitude 0
    assert int(out.index.abs().sum()) == 0 and float(out.scale.abs().sum()) == 0.0
    assert float(pvq.pvq_decode(ctx, out, torch.float32).abs().sum()) == 0.0
    ctx.close()


def _random_configurations():
    rng = np.random.default_rng(si.BASE_SEED + 4242)
    out = []
    for i in range(36):
        D = int(rng.choice([8, 8, 8, 16, 32]))
        budget = int(rng.integers(D + 2, min(4 * D, 127) + 1))       # index bits per group
        bits = int(rng.choice([0, 0, 1, 2, 4, 8]))
        rows = int(rng.integers(1, 48))
        G = int(rng.integers(1, 70)) * int(rng.choice([1, 1, 4, 8]))
        if bits and G < 2:
            G = 2
        out.append((i, D, budget, bits, rows, G, bool(rng.integers(0, 2)), str(rng.choice(["l2", "ls"]))))
    return out


@pytest.mark.parametrize("i,D,budget,bits,rows,G,bf16,amplitude", _random_configurations())
def test_random_configurations(i, D, budget, bits, rows, G, bf16, amplitude):
    # seeded draws over group size, pulse count (through the index width), amplitude format, shape,
    # source type and amplitude kind: whichever kernel family the dispatch picks must match the oracle
    K = pvq.pvq_max_k(D, budget)
    cols = G * D
    if bf16:
        wf, wb = si.gaussian_weights(rows, cols, 0.02, seed=si.BASE_SEED + 5000 + i, rotate=False, bf16=True)
        run_case(wf, D, K, bits, src_bits=wb, batches=(1, 3, 6), out_dtypes=("f32", "bf16"), amplitude=amplitude)
    else:
        W = si.gaussian_weights(rows, cols, 0.02, seed=si.BASE_SEED + 5000 + i, rotate=False)
        run_case(W, D, K, bits, batches=(2, 16), out_dtypes=("f32", "f16"), amplitude=amplitude)


def test_calls_can_be_captured_in_a_graph_and_replayed():
    # encode, decode, the fused product (single-vector and matrix-core passes), the rotation and the size
    # table enqueue kernels only (no memset, no allocation), so a caller may capture them; every replay
    # must reproduce the eager results for the inputs then in the buffers
    D, K, bits, rows, cols = 8, 16, 2, 64, 2048
    ctx, _, _ = gu.make_ctx(D, K, bits, cols // D)
    W = torch.empty((rows, cols), dtype=torch.bfloat16, device="cuda")
    x = torch.empty((16, cols), dtype=torch.bfloat16, device="cuda")
    packed = pvq.alloc_packed(ctx, rows, cols, W.device)
    What = torch.empty((rows, cols), dtype=torch.float32, device="cuda")
    y1 = torch.empty((1, rows), dtype=torch.float32, device="cuda")
    y16 = torch.empty((16, rows), dtype=torch.float32, device="cuda")
    R = torch.empty((rows, cols), dtype=torch.bfloat16, device="cuda")

    def fill(seed):
        _, wb = si.gaussian_weights(rows, cols, 0.02, seed=si.BASE_SEED + seed, rotate=False, bf16=True)
        _, xb = si.activations(16, cols, seed=si.BASE_SEED + seed)
        W.copy_(gu.to_dev_bf16(wb)); x.copy_(gu.to_dev_bf16(xb))

    def run():
        pvq.pvq_encode(ctx, W, out=packed)
        pvq.pvq_decode(ctx, packed, out=What)
        pvq.pvq_decode_gemv(ctx, packed, x[:1], out=y1)
        pvq.pvq_decode_gemv(ctx, packed, x, out=y16)
        pvq.pvq_hadamard(W, 2048, out=R)

    fill(1)
    run()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            run()
    torch.cuda.synchronize()
    for seed in (2, 3, 4):
        fill(seed)
        run()
        torch.cuda.synchronize()
        want = [t.clone() for t in (packed.index, packed.scale, packed.rownorm, What, y1, y16, R)]
        for t in (packed.index, packed.scale, packed.rownorm, What, y1, y16, R):
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(want, (packed.index, packed.scale, packed.rownorm, What, y1, y16, R)):
            assert torch.equal(a, b)
    ctx.close()


def test_leading_dimensions_and_views():
    D, K = 8, 16
    rows, cols, ld = 33, 512, 640
    wf, wb = si.gaussian_weights(rows, ld, 0.02, seed=si.BASE_SEED + 50, bf16=True)
    ctx = pvq.pvq_ctx_create(D, K)
    big = gu.to_dev_bf16(wb)
    view = big[:, :cols]
    packed = pvq.pvq_encode(ctx, view, want_pulses=True)
    enc = oracle.encode(np.ascontiguousarray(wf[:, :cols]), D, K)
    gu.assert_encode_equal(packed, enc)
    ref, _, _ = oracle.decode(enc)
    for setting in gu.decoder_settings(D):
        with gu.decoder_setting(setting):
            out_big = torch.full((rows, ld), 7.0, dtype=torch.float32, device="cuda")
            pvq.pvq_decode(ctx, packed, out=out_big[:, :cols])
            gu.assert_decode_close(out_big[:, :cols].cpu().numpy(), ref)
            assert torch.all(out_big[:, cols:] == 7.0)          # nothing written past cols
    xf, xb = si.activations(2, ld, seed=5)
    xv = gu.to_dev_bf16(xb)[:, :cols]
    y_big = torch.full((2, rows + 5), -3.0, dtype=torch.float32, device="cuda")
    pvq.pvq_decode_gemv(ctx, packed, xv, out=y_big[:, :rows])
    gu.assert_gemv_close(y_big[:, :rows].cpu().numpy(), xf[:, :cols].astype(np.float64) @ ref.T,
                         gu.product_scale(xf[:, :cols], ref))
    assert torch.all(y_big[:, rows:] == -3.0)
    ctx.close()


def test_leading_dimensions_in_the_many_vector_pass():
    # rows of 256 groups with 24-bit indices go to the matrix-core pass for 3..16 vectors: activations
    # and results as views with larger leading dimensions, results beyond the rows untouched
    D, K, rows, cols, ld = 8, 16, 21, 2048, 2048 + 64
    wf, wb = si.gaussian_weights(rows, cols, 0.02, seed=si.BASE_SEED + 51, bf16=True)
    ctx = pvq.pvq_ctx_create(D, K)
    packed = pvq.pvq_encode(ctx, gu.to_dev_bf16(wb))
    ref, _, _ = oracle.decode(oracle.encode(wf, D, K))
    for batch in (5, 16):
        xf, xb = si.activations(batch, ld, seed=7 + batch)
        xv = gu.to_dev_bf16(xb)[:, :cols]
        y_big = torch.full((batch, rows + 11), -3.0, dtype=torch.float32, device="cuda")
        pvq.pvq_decode_gemv(ctx, packed, xv, out=y_big[:, :rows])
        gu.assert_gemv_close(y_big[:, :rows].cpu().numpy(), xf[:, :cols].astype(np.float64) @ ref.T,
                             gu.product_scale(xf[:, :cols], ref))
        assert torch.all(y_big[:, rows:] == -3.0)
    ctx.close()


def test_empty_inputs_and_argument_errors():
    ctx = pvq.pvq_ctx_create(8, 16)
    L = pvq.lib()
    h = ctx.handle
    # rows == 0 / cols == 0: nothing to do, success, no pointer is touched
    assert L.pvq_encode(h, None, 0, 0, 512, 512, None, None, None, None, None) == 0
    assert L.pvq_decode(h, None, None, None, 0, 512, None, 0, 512, None) == 0
    assert L.pvq_decode_gemv(h, None, None, None, 0, 512, None, 1, 512, None, 0, None) == 0
    y = torch.full((2, 16), 5.0, device="cuda")
    assert L.pvq_decode_gemv(h, None, None, None, 16, 0, None, 2, 0, y.data_ptr(), 16, None) == 0
    torch.cuda.synchronize()
    assert torch.all(y == 0)                            # empty sum
    W = torch.zeros((4, 512), dtype=torch.float32, device="cuda")
    p = pvq.alloc_packed(ctx, 4, 512, W.device)
    args = [h, W.data_ptr(), 0, 4, 512, 512, p.index.data_ptr(), p.scale.data_ptr(), None, None, None]
    bad = list(args); bad[4] = 516                      # cols not a multiple of D
    assert L.pvq_encode(*bad) == -2
    bad = list(args); bad[5] = 256                      # ld < cols
    assert L.pvq_encode(*bad) == -1
    bad = list(args); bad[1] = W.data_ptr() + 4         # misaligned
    assert L.pvq_encode(*bad) == -3
    bad = list(args); bad[2] = 1                        # float16 source is not supported
    assert L.pvq_encode(*bad) == -1
    bad = list(args); bad[6] = None
    assert L.pvq_encode(*bad) == -1
    x = torch.zeros((17, 512), dtype=torch.bfloat16, device="cuda")
    yy = torch.zeros((17, 4), device="cuda")
    assert L.pvq_decode_gemv(h, p.index.data_ptr(), p.scale.data_ptr(), None, 4, 512, x.data_ptr(), 17,
                             512, yy.data_ptr(), 4, None) == -2
    for D, K in [(7, 5), (8, 0), (8, 128), (32, 127)]:
        with pytest.raises(pvq.PvqError):
            pvq.pvq_ctx_create(D, K)
    with pytest.raises(pvq.PvqError):
        pvq.pvq_ctx_create(8, 16, 3, np.zeros(7), np.zeros(8))
    ctx.close()
    # amplitude codes and a row whose amplitudes do not fit a workgroup's LDS: refused as unsupported, not as a
    # failed launch
    for K, groups, want in ((5, 16384, -2), (16, 16384, -2), (5, 8192, 0)):
        cols = 8 * groups
        ctx, oe, oc = gu.make_ctx(8, K, 2, groups)
        Wl = torch.ones((1, cols), dtype=torch.float32, device="cuda")
        pl = pvq.alloc_packed(ctx, 1, cols, Wl.device)
        rc = L.pvq_encode(ctx.handle, Wl.data_ptr(), 0, 1, cols, cols, pl.index.data_ptr(), pl.scale.data_ptr(),
                          pl.rownorm.data_ptr(), None, None)
        torch.cuda.synchronize()
        assert rc == want, (K, groups, rc)
        ctx.close()


def test_zero_matrix_and_nonfinite_inputs_are_safe():
    D, K = 8, 16
    ctx = pvq.pvq_ctx_create(D, K)
    W = torch.zeros((8, 256), dtype=torch.float32, device="cuda")
    packed = pvq.pvq_encode(ctx, W, want_pulses=True)
    assert torch.all(packed.index == 0) and torch.all(packed.scale == 0)
    for setting in gu.decoder_settings(D):
        with gu.decoder_setting(setting):
            assert torch.all(pvq.pvq_decode(ctx, packed, torch.float32) == 0)
    W[0, 3] = float("nan"); W[1, 9] = float("inf"); W[2, :] = float("-inf"); W[3, 0] = 3e38; W[3, 1] = 3e38
    packed = pvq.pvq_encode(ctx, W, want_pulses=True)
    torch.cuda.synchronize()
    p = packed.pulses.cpu().numpy().astype(np.int64).reshape(8, 32, 8)
    assert np.all(np.abs(p).sum(axis=2) == K)           # every stored point is on the pyramid
    idx = np.array(oracle.unpack_fields(gu.words(packed.index), 32, 24))
    assert idx.max() < pvq.pvq_count(D, K)[0]
    ctx.close()


def test_corrupt_indices_do_not_fault():
    # stored fields at or above N(D,K): unspecified values, but every kernel family stays inside its tables
    # (D = 8: the index is clamped; generic kernels: the walk is bounded by the pulses left; long groups:
    # such a group decodes to zeros, like the oracle's)
    D, K = 8, 16
    ctx = pvq.pvq_ctx_create(D, K)
    idx = torch.full((16, 768), -1, dtype=torch.int32, device="cuda")     # every field = 2^24-1 >= N
    p = pvq.Packed(16, 8192, idx, torch.ones((16, 1024), device="cuda"), torch.ones(16, device="cuda"))
    for setting in gu.decoder_settings(D):
        with gu.decoder_setting(setting):
            out = pvq.pvq_decode(ctx, p, torch.float32)
            torch.cuda.synchronize()
            assert out.shape == (16, 8192) and bool(torch.isfinite(out).all())
    x = torch.ones((16, 8192), dtype=torch.bfloat16, device="cuda")
    for b in (1, 4, 16):                     # the single-vector, four-vector and matrix-core passes
        y = pvq.pvq_decode_gemv(ctx, p, x[:b])
        assert bool(torch.isfinite(y).all())
    torch.cuda.synchronize()
    assert out.shape == (16, 8192) and bool(torch.isfinite(out).all())
    ctx.close()

    ctx = pvq.pvq_ctx_create(16, 33)         # 52-bit fields, all ones
    idx = torch.full((8, 104), -1, dtype=torch.int32, device="cuda")
    p = pvq.Packed(8, 1024, idx, torch.ones((8, 64), device="cuda"), torch.ones(8, device="cuda"))
    out = pvq.pvq_decode(ctx, p, torch.float32)
    y = pvq.pvq_decode_gemv(ctx, p, x[:2, :1024].contiguous())
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all()) and bool(torch.isfinite(y).all())
    ctx.close()

    ctx = pvq.pvq_ctx_create(128, 187)       # 384-bit fields, all ones: not codewords, decoded as zeros
    idx = torch.full((4, 24), -1, dtype=torch.int32, device="cuda")
    p = pvq.Packed(4, 256, idx, torch.ones((4, 2), device="cuda"), torch.ones(4, device="cuda"))
    out = pvq.pvq_decode(ctx, p, torch.float32)
    torch.cuda.synchronize()
    assert float(out.abs().sum()) == 0.0
    ctx.close()


@pytest.mark.parametrize("D,K,words", [(8, 16, 1), (16, 33, 2), (32, 60, 4), (128, 187, 12), (64, 127, 16),
                                       (5, 0, 1), (0, 7, 1), (200, 1023, 16)])
def test_size_table_on_the_gpu(D, K, words):
    # App. C.2: every entry must equal the oracle's table, word for word
    table, flag = pvq.pvq_size_table_device(D, K, words)
    got = table.cpu().numpy().view(np.uint32)
    want = oracle.size_table(D, K) if (D, K, words) != (200, 1023, 16) else None
    if want is None:
        # far beyond 512 bits: only the flag and the rows that still fit are checked
        assert int(flag.cpu()[0]) == 1
        want = oracle.size_table(6, 1023)
        D = 6
    else:
        assert int(flag.cpu()[0]) == 0
    for d in range(D + 1):
        for k in range(0, K + 1, max(1, K // 37)):
            assert oracle.words_to_int(got[d, k]) == want[d][k], (d, k)


def test_size_table_overflow_flag():
    # N(16,33) needs 52 bits: one word is not enough, two are
    _, flag1 = pvq.pvq_size_table_device(16, 33, 1)
    t2, flag2 = pvq.pvq_size_table_device(16, 33, 2)
    assert int(flag1.cpu()[0]) == 1 and int(flag2.cpu()[0]) == 0
    assert oracle.words_to_int(t2.cpu().numpy().view(np.uint32)[16, 33]) == oracle.size_table(16, 33)[16][33]


@pytest.mark.parametrize("rows,cols,block", [(3, 8, 8), (5, 64, 16), (4, 8 * 37 * 8, 64), (7, 512, 512), (6, 3584, 512),
                                             (9, 2048, 2048), (5, 4096, 4096), (3, 8192, 8192), (2, 28672, 4096),
                                             (130, 1024, 128), (4, 3072, 1024), (2, 16384, 8192)])
def test_hadamard_rotation(rows, cols, block):
    # Sec. 3.3 Step 1: float32 butterflies in a fixed order, so float32 results are the oracle's bit for
    # bit and bf16 results are its values rounded once; the inverse undoes the rotation
    rng = np.random.default_rng(rows * 131 + cols)
    X = (rng.standard_normal((rows, cols)) * 0.02).astype(np.float32)
    sg = rng.integers(0, 2, size=cols).astype(np.uint8)
    want = oracle.hadamard_rows(X, block, sg)
    Xd, sd = gu.to_dev_f32(X), torch.from_numpy(sg).cuda()
    got = pvq.pvq_hadamard(Xd, block, sd)
    assert np.array_equal(got.cpu().numpy().view(np.uint32), want.view(np.uint32))
    got_bf = pvq.pvq_hadamard(Xd, block, sd, out_dtype=torch.bfloat16)
    assert np.array_equal(gu.bf16_tensor_bits(got_bf), oracle.to_bf16_bits(want.astype(np.float64)))
    # bf16 source, no signs
    xb = si.f32_to_bf16_bits(X)
    xf = si.bf16_bits_to_f32(xb)
    got2 = pvq.pvq_hadamard(gu.to_dev_bf16(xb), block, None, out_dtype=torch.float32)
    assert np.array_equal(got2.cpu().numpy().view(np.uint32), oracle.hadamard_rows(xf, block).view(np.uint32))
    # inverse, in place
    back = pvq.pvq_hadamard(got, block, sd, inverse=True, out=got)
    want_back = oracle.hadamard_rows(want, block, sg, signs_after=True)
    assert np.array_equal(back.cpu().numpy().view(np.uint32), want_back.view(np.uint32))
    assert np.allclose(back.cpu().numpy(), X, rtol=0, atol=4e-6 * np.abs(X).max() * np.log2(block))


def test_hadamard_argument_errors():
    X = torch.zeros((4, 96), dtype=torch.float32, device="cuda")
    for block in (4, 64, 48, 16384):       # too small, not dividing 96, not a power of two, too large
        with pytest.raises(pvq.PvqError):
            pvq.pvq_hadamard(X, block)
    with pytest.raises(pvq.PvqError):
        pvq.pvq_hadamard(X.to(torch.float16), 32)
    assert pvq.pvq_hadamard(torch.zeros((0, 96), dtype=torch.float32, device="cuda"), 32).shape == (0, 96)


def test_the_plan_of_passes_names_the_kernels_that_run():
    # host logic of the dispatch, asked through the diagnostics entry point (nothing is launched)
    e, c = pvq.pvq_beta_tables(8, 1024, 2)
    ctx = pvq.pvq_ctx_create(8, 16, 2, e, c)
    assert pvq.pvq_decode_gemv_plan(ctx, 28672, 8192, 1) == [("valu_fp32_rows", 1)]
    assert pvq.pvq_decode_gemv_plan(ctx, 28672, 8192, 4) == [("mfma_bf16", 4)]
    assert pvq.pvq_decode_gemv_plan(ctx, 28672, 8192, 16) == [("mfma_bf16", 16)]
    assert pvq.pvq_decode_gemv_plan(ctx, 28672, 8192, 2) == [("valu_fp32", 2)]
    assert pvq.pvq_decode_gemv_plan(ctx, 1024, 8192, 1) == [("valu_fp32", 1)]          # too few rows per wave
    assert pvq.pvq_decode_gemv_plan(ctx, 96, 8 * 36, 7) == [("valu_fp32", 4), ("valu_fp32", 2), ("valu_fp32", 1)]
    assert pvq.pvq_decode_gemv_plan(ctx, 96, 8 * 37, 7) == [("valu_fp32_generic", 7)]   # lanes take whole quads of groups
    assert sum(n for _, n in pvq.pvq_decode_gemv_plan(ctx, 512, 2048, 16)) == 16
    ctx.close()
    ctx = pvq.pvq_ctx_create(16, 33)
    assert pvq.pvq_decode_gemv_plan(ctx, 512, 2048, 5) == [("valu_fp32_generic", 5)]
    ctx.close()
