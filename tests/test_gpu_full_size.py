"""GPU parity at the full sizes of the measured workloads, in the launch configurations bench.py
times: whole-matrix bit-exact comparison of the encoder's outputs, whole-matrix 1-ulp comparison
of decoded bf16 weights, and the fused product against a float64 matmul of the oracle's weights.
The oracle runs on the host cores (16 threads); matrices are generated on the GPU from a seed."""
import numpy as np
import pytest

import paper_2410_16926_amd as pvq
import synth_inputs as si
from oracle import pvq_oracle as oracle
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")
THREADS = 16


def device_matrix(rows, cols, seed):
    W = si.gaussian_weights_device(rows, cols, 0.015, seed, torch.device("cuda:0"))
    return W, W.to(torch.float32).cpu().numpy()          # bf16 tensor, the same values as float32


def encode_decode_case(rows, cols, D, budget, scale_bits, seed, batches=()):
    K = pvq.pvq_max_k(D, budget)
    G = cols // D
    ctx, oe, oc = gu.make_ctx(D, K, scale_bits, G)
    W, wf = device_matrix(rows, cols, seed)
    packed = pvq.pvq_encode(ctx, W, want_pulses=True)
    torch.cuda.synchronize()
    enc = oracle.encode(wf, D, K, scale_bits, oe, want_pulses=True, nthreads=THREADS)
    gu.assert_encode_equal(packed, enc)
    del wf
    ref, _, _ = oracle.decode(enc, oc, nthreads=THREADS)
    got = gu.bf16_tensor_bits(pvq.pvq_decode(ctx, packed, torch.bfloat16))
    want = oracle.to_bf16_bits(ref)
    assert gu.ulp_f16(want, got) <= 1
    assert np.mean(want != got) < 1e-3                    # one-ulp cases are double-rounding cases: rare
    del got, want
    for B in batches:
        xf, xb = si.activations(B, cols, seed=seed + B)
        y = pvq.pvq_decode_gemv(ctx, packed, gu.to_dev_bf16(xb)).cpu().numpy()
        gu.assert_gemv_close(y, xf.astype(np.float64) @ ref.T, gu.product_scale(xf, ref))
    ctx.close()


def test_llama3_8b_up_projection_8bit_amplitudes():
    # 14336 x 4096 bf16, D=8, 24-bit indices, 8-bit Beta amplitude codes
    encode_decode_case(14336, 4096, 8, 24, 8, si.BASE_SEED + 1001)


@pytest.mark.parametrize("D,budget", [(16, 52), (32, 104)])
def test_llama3_8b_up_projection_wide_indices(D, budget):
    # the same matrix family with 52-bit (2 words) and 104-bit (4 words) indices, float32 amplitudes
    encode_decode_case(14336, 4096, D, budget, 0, si.BASE_SEED + 1002 + D)


@pytest.mark.parametrize("name", ["k", "q", "down"])
def test_llama3_70b_layer_shapes_2bit_amplitudes(name):
    # 3.25 bits/weight: D=8, 24-bit index + 2-bit amplitude code; k/v, q/o and down shapes; the fused product
    # with 1, 3 and 16 vectors (the matrix-core pass with one and two row tiles per workgroup, and with rows
    # of 56 slabs for the down projection)
    rows, cols = si.LLAMA3_70B_SHAPES[name]
    encode_decode_case(rows, cols, 8, 24, 2, si.BASE_SEED + 1100 + rows % 97, batches=(1, 3, 16))


def test_llama3_70b_gate_projection_with_fused_product():
    # the benchmark's matrix shape (28672 x 8192) end to end, and the fused product at batch 1, 4, 16
    rows, cols = si.LLAMA3_70B_SHAPES["gate"]
    encode_decode_case(rows, cols, 8, 24, 2, si.BASE_SEED + 1200, batches=(1, 4, 16))


def test_prefill_batch_of_activations_long_groups():
    # the on-the-fly activation setting at the size bench.py --extras times: 4096 tokens x 8192, D=128,
    # K=187 (384-bit indices), float32 amplitudes; whole index plane and amplitudes identical to the
    # oracle's, decoded bf16 values within 1 ulp
    tokens, hidden, D = 4096, 8192, 128
    K = pvq.pvq_max_k(D, 3 * D)
    ctx = pvq.pvq_ctx_create(D, K)
    xf, xb = si.activation_matrix(tokens, hidden, seed=si.BASE_SEED + 1300)
    packed = pvq.pvq_encode(ctx, gu.to_dev_bf16(xb))
    torch.cuda.synchronize()
    enc = oracle.encode(xf, D, K, 0, None, nthreads=THREADS)
    gu.assert_encode_equal(packed, enc, check_pulses=False)
    ref, _, _ = oracle.decode(enc, None, nthreads=THREADS)
    got = gu.bf16_tensor_bits(pvq.pvq_decode(ctx, packed, torch.bfloat16))
    assert gu.ulp_f16(oracle.to_bf16_bits(ref), got) <= 1
    ctx.close()


def test_error_correction_of_a_square_projection():
    # Sec. 3.3 Step 6 on 8192 x 8192 (the attention projections' shape), in the configuration that the
    # benchmark's extras time: 64 panels, each launch with 128 panel workgroups in front of up to 3968 update
    # tiles.  Rows are independent, so the oracle corrects a sample of rows (first and last rows of panel
    # workgroups and of update tiles, and rows in between) and those must match bit for bit.  The factor is a seeded well-conditioned upper triangular matrix (any such matrix is the
    # factor of some inverse Hessian); the arithmetic, not the statistics, is what is compared here.
    rows = cols = 8192
    D, K = 8, 16
    rng = np.random.default_rng(si.BASE_SEED + 900)
    U = np.triu(rng.standard_normal((cols, cols), dtype=np.float32) * np.float32(0.3 / cols ** 0.5))
    U[np.diag_indices(cols)] += np.float32(1.0)
    W0 = device_matrix(rows, cols, si.BASE_SEED + 901)[0].to(torch.float32)
    ctx = pvq.pvq_ctx_create(D, K)
    Wd = W0.clone()
    pvq.pvq_correct(ctx, Wd, gu.to_dev_f32(U))
    torch.cuda.synchronize()
    sample = np.array([0, 1, 63, 64, 127, 128, 2047, 2048, 4095, 4096, 5000, 6143, 6144, 8190, 8191])
    got = Wd[torch.from_numpy(sample).cuda()].cpu().numpy()
    ref, _ = oracle.correct(W0[torch.from_numpy(sample).cuda()].cpu().numpy(), U, D, K, nthreads=8)
    bad = np.argwhere(got.view(np.uint32) != ref.view(np.uint32))
    assert bad.size == 0, f"{bad.shape[0]} corrected weights differ, first at row {sample[bad[0][0]]}, column {bad[0][1]}"
    assert not np.array_equal(got, W0[torch.from_numpy(sample).cuda()].cpu().numpy())
    ctx.close()
