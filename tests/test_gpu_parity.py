"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Integer results (codes, row sums, INT32 accumulators) bit-exact; bf16 outputs within
2e-2 of max|ref|; code flip rate vs the oracle's own rotation <= 1e-4 (see parity_util)."""
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2506_15689_amd import binding as B
from paper_2506_15689_amd import synth_inputs as si

import parity_util as pu

pytestmark = pytest.mark.gpu


def announce(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


def run_case(lay, **kw):
    rows = kw.pop("rows", None)
    blas = kw.pop("use_blas_gemm", False)
    case = pu.make_case(lay, **kw)
    announce(f"M={case.M} K={case.K} N={case.N} rot={case.rot_size} clip=({case.clip_lo},{case.clip_hi})")
    d = pu.to_device(case)
    g = pu.run_gpu(case, d)
    stats = pu.check_parity(case, g, rows=rows, use_blas_gemm=blas)
    pu.check_fp6_path(case, g)
    pu.check_decode_layout(case, g)
    announce(f"ok {stats}")
    return stats


# ---------------------------------------------------------------- small and mid-size, element by element

def test_c1_full():
    run_case(si.make_layer(si.CONFIGS["C1"]))


@pytest.mark.parametrize("M,K,N", [(200, 2048, 328), (130, 512, 136), (161, 256, 40), (129, 4096, 96), (200, 512, 1152), (260, 1024, 1100),
                                   (201, 8192, 72), (300, 8192, 40), (600, 4096, 72)])
def test_ragged_multi_tile(M, K, N):
    """(The K = 4096 / 8192 cases also cover the rotate+quant kernels on both sides of their token-count switches:
    several waves per token up to 512 / 256 tokens, one wave per token beyond, each with the fp6 copy.)"""
    run_case(si.make_tiny(M, K, N, seed=M))


@pytest.mark.parametrize("M,K,N", [(129, 128, 8), (140, 384, 264), (290, 640, 130)])
def test_short_k_on_the_fp6_path(M, K, N):
    """One, three and five K-steps of the fp6 GEMM's stage ring (its prologue fills two stages), M just above
    the weight-streaming threshold, N below one MFMA tile."""
    run_case(si.make_tiny(M, K, N, seed=K + M), rot_size=128)


@pytest.mark.parametrize("M,K,N", [(150, 32768, 40), (20, 32768, 24), (140, 28 * 1024, 40), (133, 16384, 72)])
def test_largest_supported_k(M, K, N):
    """K = 32768 is the longest token the library accepts (the generic rotation holds it in 128 KB of LDS, the fp6
    accumulator is exact up to there); 28 * 1024 is the longest Kronecker size below it, and 16384 the first size whose
    token needs more than the default 64 KB of LDS."""
    run_case(si.make_tiny(M, K, N, seed=K // 1024 + M))


@pytest.mark.parametrize("K,rot", [(1024, 128), (512, 64), (256, 32), (64, 2)])
def test_blockwise_rotation(K, rot):
    run_case(si.make_tiny(48, K, 64, seed=K + rot), rot_size=rot)


@pytest.mark.parametrize("M,K,N,rot", [(300, 4096, 11008, 4096), (260, 11008, 4096, 256), (3, 11008, 4096, 256),
                                       (40, 4096, 11008, 4096)])
def test_layer_shapes_of_the_model_the_paper_times(M, K, N, rot):
    """Sec. 5.2 measures the prefill of a 7B LLaMA-2: hidden size 4096, MLP width 11008.  gate/up (K = 4096,
    N = 11008: 43 tiles of 256 columns) with the full-width rotation; down (K = 11008 = 43 * 256, which has no
    power-of-two or 28 * 2^t Hadamard of its own size) with the rotation applied blockwise on 256 channels, on the
    tiled path, on the weight-streaming path (40 tokens) and for a few decode tokens."""
    run_case(si.make_tiny(M, K, N, seed=K // 64 + M, act="swiglu" if K == 11008 else "gauss"), rot_size=rot,
             use_blas_gemm=True)


@pytest.mark.parametrize("M,K,N,rot", [(70, 256, 40, 128), (70, 256, 40, 256), (131, 512, 72, 512), (90, 768, 40, 256),
                                       (90, 768, 40, 128), (150, 1280, 136, 256), (40, 2048, 64, 512), (33, 5632, 40, 512),
                                       (140, 13824, 40, 512), (20, 16384, 24, 256), (20, 16384, 24, 128),
                                       (20, 16640, 24, 256)])
@pytest.mark.parametrize("scaled", [False, True])
def test_blockwise_rotation_fast_kernel(M, K, N, rot, scaled):
    """Blocks of 128, 256 or 512 channels with per-token ranges (the register-resident blockwise kernel): a token of
    half a 512-channel piece, of one piece, of whole pieces plus a half, every piece count per wave up to the largest
    K it takes (16384), and one size beyond it (the generic kernel); with and without s^a."""
    lay = si.make_tiny(M, K, N, seed=K // 128 + rot + M, act="swiglu" if K % 1024 else "gauss")
    sa = np.random.default_rng(K + rot).uniform(0.8, 1.25, K).astype(np.float32) if scaled else None
    run_case(lay, rot_size=rot, use_blas_gemm=True, act_scale=sa, clip_lo=0.95 if scaled else None,
             clip_hi=0.85 if scaled else None)


@pytest.mark.parametrize("K", [28 * 64, 28 * 16, 2 * 28 * 32])
def test_kronecker_rotation_with_h28(K):
    rot = K if K != 2 * 28 * 32 else 28 * 32
    run_case(si.make_tiny(70, K, 100, seed=K, act="swiglu", clip=0.85), rot_size=rot)


@pytest.mark.parametrize("M,scale", [(5, False), (2, True), (131, False), (11, True), (1030, True)])
def test_rotation_28x512_fast_kernel(M, scale):
    """K = 14336 = 28 * 512 takes the specialised kernel: two waves per token, two tokens per workgroup
    (four when s^a is staged next to b^c); ragged M leaves waves idle, M = 1030 needs a second round."""
    sa = None
    if scale:
        sa = np.random.default_rng(3).uniform(0.8, 1.25, 14336).astype(np.float32)
    run_case(si.make_tiny(M, 14336, 72, seed=M, act="swiglu", clip=0.85, n_outlier=32, outlier_scale=30.0),
             act_scale=sa)


@pytest.mark.parametrize("K,M", [(4096, 9), (8192, 6)])
def test_pow2_fast_kernel_with_scale(K, M):
    sa = np.random.default_rng(K).uniform(0.8, 1.25, K).astype(np.float32)
    run_case(si.make_tiny(M, K, 40, seed=K + M), act_scale=sa, clip_lo=0.9, clip_hi=1.0)


def test_asymmetric_scale_and_unequal_clips_and_layer_bias():
    cfg = si.LayerConfig("as", 0, 96, 1024, 160, 4, 20.0, 0.9, 0.02)
    lay = si.make_layer(cfg, seed=77, with_layer_bias=True)
    rng = np.random.default_rng(5)
    sa = rng.uniform(0.7, 1.5, 1024).astype(np.float32)
    run_case(lay, act_scale=sa, clip_lo=0.95, clip_hi=0.8)


def test_no_bias_no_out_bias():
    run_case(si.make_tiny(40, 512, 72, seed=9), use_bias=False, use_out_bias=False)


@pytest.mark.parametrize("name", ["C3_M1", "C3_M4", "C3_M16"])
def test_decode_shapes_full(name):
    run_case(si.make_layer(si.CONFIGS[name]), use_blas_gemm=True)


@pytest.mark.parametrize("M,K,N", [(1, 1024, 24), (3, 512, 16), (16, 256, 100), (5, 96, 33)])
def test_decode_ragged(M, K, N):
    run_case(si.make_tiny(M, K, N, seed=3 * M + N), rot_size=K if K != 96 else 32)


@pytest.mark.parametrize("M,K,N,scaled,biased", [(1, 8192, 24, False, False), (4, 8192, 100, True, True), (3, 8192, 48, False, True), (16, 8192, 48, False, False),
                                                 (3, 4096, 40, True, True), (4, 4096, 4096, False, True), (2, 4096, 17, True, False),
                                                 (5, 4096, 4096, False, True), (1, 4096, 4096, False, False), (1, 4096, 40, True, False),
                                                 (2, 4096, 264, False, True), (2, 4096, 4096, True, True), (1, 8192, 100, True, False)])
def test_decode_one_launch(M, K, N, scaled, biased):
    """Calls of at most 4 tokens with rot_size = K in {4096, 8192}, N <= 4096 and the streaming weight layout run
    the whole layer in one kernel (basq_linear_fused); run_case checks its output against the two-call path bit
    for bit, and that path against the oracle.  With and without s^a and the bias, ragged N; the cases above 4
    tokens take the two-kernel path on the same shapes.  One or two tokens of K = 4096 run two waves per token, one token
    of K = 8192 four (they exchange one or two butterfly stages, the range and the row sum through LDS); the
    two-kernel path splits tokens the same way up to a few hundred tokens."""
    lay = si.make_tiny(M, K, N, seed=M + K + N)
    sa = np.random.default_rng(M + N).uniform(0.7, 1.5, K).astype(np.float32) if scaled else None
    run_case(lay, act_scale=sa, use_bias=biased, use_out_bias=biased, use_blas_gemm=True)


@pytest.mark.parametrize("M,K,N", [(17, 4096, 96), (32, 512, 40), (33, 256, 100), (64, 1024, 1024), (65, 128, 24), (100, 640, 328),
                                   (128, 2048, 136), (40, 128, 16392), (128, 256, 16400), (50, 8192, 64)])
def test_batched_decode(M, K, N):
    """17 to 128 tokens stay on the weight-streaming kernel: two, four or eight token tiles against the same
    weight registers; one or (from 1024 blocks of 16 output channels) two weight tiles per workgroup; ragged
    token tiles, ragged and odd block counts, K from one chunk per row to 64."""
    run_case(si.make_tiny(M, K, N, seed=M * 7 + N), rot_size=K if (K & (K - 1)) == 0 else 128, use_blas_gemm=True)


@pytest.mark.parametrize("M,N", [(16, 16392), (9, 16400), (8, 16392)])
def test_decode_many_output_channels(M, N):
    """More than 1024 blocks of 16 output channels: with more than 8 tokens a workgroup takes two blocks
    (an odd number of blocks and a ragged last block here); with 8 tokens it takes one."""
    run_case(si.make_tiny(M, 128, N, seed=M + N), use_blas_gemm=True)


# ---------------------------------------------------------------- edge cases

def test_zero_tokens_is_a_no_op():
    dev = "cuda"
    K, N = 256, 64
    X = torch.empty((0, K), dtype=torch.bfloat16, device=dev)
    Aq, meta = B.alloc_activation_buffers(0, K, dev)
    B.basq_rotate_quant(X, K, None, None, 0.9, 0.9, Aq, meta)
    Wq, ws, wz, wsum = B.alloc_weight_buffers(N, K, dev)
    Y = torch.empty((0, N), dtype=torch.bfloat16, device=dev)
    B.basq_w4a4_gemm(Aq, meta, Wq, ws, wz, wsum, None, Y)
    torch.cuda.synchronize()


def test_degenerate_tokens_match_oracle():
    """Constant token, token with a NaN, token with +inf, all-zero token: same codes and records
    as the oracle's quantiser given the GPU's rotation output."""
    dev = "cuda"
    K = 512
    lay = si.make_tiny(8, K, 16, seed=21)
    X = lay.X.clone().float()
    X[1, :] = 0.0
    X[2, :] = 0.0
    X[2, 0] = 1.0                       # rotates to a constant token (every entry +1/sqrt(K))
    X[3, 7] = float("nan")
    X[4, 9] = float("inf")
    X = X.to(torch.bfloat16)
    Aq, meta = B.alloc_activation_buffers(8, K, dev)
    rot = torch.empty((8, K), dtype=torch.float32, device=dev)
    B.basq_rotate_quant(X.to(dev), K, None, None, 1.0, 1.0, Aq, meta, rot)
    torch.cuda.synchronize()
    r = rot.cpu().numpy()
    assert np.all(r[1] == 0) and np.allclose(r[2], 1 / np.sqrt(K))
    tq = oracle.quantize_tokens(r, None, None, 1.0, 1.0)
    codes = oracle.unpack_codes(Aq.cpu().numpy())
    mh = meta.cpu().numpy()
    np.testing.assert_array_equal(codes, tq.codes)
    np.testing.assert_array_equal(mh[:, 0].copy().view(np.uint32), tq.scale[:, 0].view(np.uint32))
    np.testing.assert_array_equal(mh[:, 1].copy().view(np.uint32), tq.lo[:, 0].view(np.uint32))
    np.testing.assert_array_equal(mh[:, 2], tq.rowsum[:, 0])
    assert mh[1, 0].view(np.float32) == 1.0 and (codes[1] == 0).all()


@pytest.mark.parametrize("K", [512, 4096, 8192, 14336])
def test_ties_round_to_even_in_both_code_forms(K):
    """Values exactly half-way between two codes: an all-zero input rotates to zero, so v = -b^c, and with the range
    [0, 15] and clip ratios of 1 the quantiser's step is exactly 1 and t = v.  Every k + 1/2 must become the even
    neighbour in the packed INT4 codes (integer conversion) and in the fp6 copy, which the K = 4096 / 8192 kernel
    makes with a floating-point conversion of its own (K = 512 and 14336: the other kernels, for comparison)."""
    dev = "cuda"
    M = 5
    v = (np.arange(K) % 15).astype(np.float32) + 0.5
    v[0], v[1] = 0.0, 15.0
    v[2::7] = (np.arange(len(v[2::7])) % 16).astype(np.float32)        # some exact codes in between
    X = torch.zeros((M, K), dtype=torch.bfloat16, device=dev)
    X[3, 5] = float("nan")                   # rotates to NaN everywhere: every code is 0, in both forms
    X[4, 9] = float("inf")                   # rotates to +-inf: codes 15 and 0, the same in both forms
    bias = torch.from_numpy(-v).to(dev)
    Aq, meta = B.alloc_activation_buffers(M, K, dev)
    A6 = B.alloc_fp6_buffer(M, K, dev).zero_()
    A6b = torch.zeros_like(A6)
    B.basq_rotate_quant(X, K, bias, None, 1.0, 1.0, Aq, meta, Aq6=A6)
    B.basq_pack_fp6(Aq, A6b)
    torch.cuda.synchronize()
    tq = oracle.quantize_tokens(np.zeros((M, K), dtype=np.float32), bias.cpu().numpy(), None, 1.0, 1.0)
    expect = np.rint(v).astype(tq.codes.dtype)                           # numpy rounds half to even
    np.testing.assert_array_equal(tq.codes, np.broadcast_to(expect, (M, K)))
    codes = oracle.unpack_codes(Aq.cpu().numpy())
    np.testing.assert_array_equal(codes[:3], tq.codes[:3])
    assert (codes[3] == 0).all() and set(np.unique(codes[4])) <= {0, 15}
    mh = meta.cpu().numpy()
    assert (mh[:3, 0].copy().view(np.float32) == 1.0).all() and (mh[:3, 1].copy().view(np.float32) == 0.0).all()
    assert torch.equal(A6, A6b), "the fp6 copy written by the quantiser differs from the packed codes"


@pytest.mark.parametrize("K", [4096, 8192])
def test_many_tokens_take_the_staged_fp6_tails(K):
    """From 32768 tokens on, the K = 4096 / 8192 kernel writes the 8-byte tail pieces of the fp6 copy through an LDS
    stage shared by the eight tokens of a workgroup.  Same bits as the plain path: codes and records of the first and
    last thousand tokens equal those of separate short calls, sampled tokens equal the oracle's quantiser on the GPU's rotation, and the fp6 copy
    equals the packed codes everywhere; 13 tokens past a multiple of 8 leave a ragged, odd last round, and rows past M
    in the last block stay untouched."""
    dev = "cuda"
    M = 32768 + 13
    gen = torch.Generator(device=dev).manual_seed(K)
    X = (torch.randn((M, K), generator=gen, device=dev) * 1.5).to(torch.bfloat16)
    X[:, 7] *= 20.0                                                        # an outlier channel
    bias = torch.randn(K, generator=gen, device=dev) * 0.1
    Aq, meta = B.alloc_activation_buffers(M, K, dev)
    A6 = B.alloc_fp6_buffer(M, K, dev).zero_()
    A6b = torch.zeros_like(A6)
    B.basq_rotate_quant(X, K, bias, None, 0.9, 0.95, Aq, meta, Aq6=A6)
    B.basq_pack_fp6(Aq, A6b)
    torch.cuda.synchronize()
    assert torch.equal(A6, A6b), "the staged fp6 copy differs from the packed codes"
    for lo, hi in ((0, 1000), (M - 1000, M)):
        Aq_s, meta_s = B.alloc_activation_buffers(hi - lo, K, dev)
        B.basq_rotate_quant(X[lo:hi], K, bias, None, 0.9, 0.95, Aq_s, meta_s)
        torch.cuda.synchronize()
        assert torch.equal(Aq[lo:hi], Aq_s) and torch.equal(meta[lo:hi], meta_s)
    assert int(meta[:, 2].min()) >= 0 and int(meta[:, 2].max()) <= 15 * K
    # and straight against the oracle: 64 sampled tokens plus the first and last rounds, on the GPU's own rotation
    rng = np.random.default_rng(K)
    rows = np.unique(np.concatenate([rng.choice(M, 64, replace=False), np.arange(8), np.arange(M - 13, M)]))
    pu.check_rows_against_oracle(X, rows, K, bias, None, 0.9, 0.95, Aq, meta, what="staged fp6 tails")


def test_strided_input_and_output():
    dev = "cuda"
    lay = si.make_tiny(50, 256, 48, seed=31)
    case = pu.make_case(lay)
    d = pu.to_device(case)
    Xbig = torch.zeros((50, 256 + 64), dtype=torch.bfloat16, device=dev)
    Xbig[:, :256] = d.X
    Ybig = torch.zeros((50, 48 + 16), dtype=torch.bfloat16, device=dev)
    Aq, meta = B.alloc_activation_buffers(50, 256, dev)
    Aq2, meta2 = B.alloc_activation_buffers(50, 256, dev)
    Y = torch.empty((50, 48), dtype=torch.bfloat16, device=dev)
    B.basq_rotate_quant(Xbig[:, :256], 256, d.bias, None, 0.9, 0.9, Aq, meta)
    B.basq_rotate_quant(d.X, 256, d.bias, None, 0.9, 0.9, Aq2, meta2)
    B.basq_w4a4_gemm(Aq, meta, d.Wq, d.w_scale, d.w_zero, d.w_sum, d.out_bias, Ybig[:, :48])
    B.basq_w4a4_gemm(Aq2, meta2, d.Wq, d.w_scale, d.w_zero, d.w_sum, d.out_bias, Y)
    torch.cuda.synchronize()
    assert torch.equal(Aq, Aq2) and torch.equal(meta[:, :3], meta2[:, :3])
    assert torch.equal(Ybig[:, :48], Y)
    assert (Ybig[:, 48:] == 0).all()


def test_output_width_not_a_multiple_of_eight():
    """N = 100 written into rows of 104 (16-byte aligned rows, ragged last piece) and into rows of 100
    (unaligned rows): both must equal the reference path that also dumps the accumulators."""
    dev = "cuda"
    lay = si.make_tiny(70, 512, 100, seed=51)
    case = pu.make_case(lay)
    d = pu.to_device(case)
    g = pu.run_gpu(case, d)
    pu.check_parity(case, g)
    Aq, meta = B.alloc_activation_buffers(70, 512, dev)
    B.basq_rotate_quant(d.X, 512, d.bias, None, case.clip_lo, case.clip_hi, Aq, meta)
    Ywide = torch.zeros((70, 104), dtype=torch.bfloat16, device=dev)
    Ytight = torch.zeros((70, 100), dtype=torch.bfloat16, device=dev)
    B.basq_w4a4_gemm(Aq, meta, d.Wq, d.w_scale, d.w_zero, d.w_sum, d.out_bias, Ywide[:, :100])
    B.basq_w4a4_gemm(Aq, meta, d.Wq, d.w_scale, d.w_zero, d.w_sum, d.out_bias, Ytight)
    torch.cuda.synchronize()
    ref = si.bits_to_bf16(g.y_bits).to(dev)
    assert torch.equal(Ywide[:, :100], ref) and torch.equal(Ytight, ref)
    assert (Ywide[:, 100:] == 0).all()


def test_same_input_twice_gives_identical_bits():
    lay = si.make_tiny(300, 1024, 200, seed=41)
    case = pu.make_case(lay)
    d = pu.to_device(case)
    g1 = pu.run_gpu(case, d)
    g2 = pu.run_gpu(case, d)
    np.testing.assert_array_equal(g1.codes, g2.codes)
    np.testing.assert_array_equal(g1.acc, g2.acc)
    np.testing.assert_array_equal(g1.y_bits, g2.y_bits)
    np.testing.assert_array_equal(g1.rot.view(np.uint32), g2.rot.view(np.uint32))


# ---------------------------------------------------------------- offline helpers

@pytest.mark.parametrize("N,K", [(64, 512), (100, 1792)])
def test_weight_quantiser_and_fused_bias(N, K):
    dev = "cuda"
    lay = si.make_tiny(16, K, N, seed=N)
    w = oracle.bf16_to_f32(si.bf16_bits(lay.W_rot))
    wq = oracle.quantize_weights(w)
    Wq, ws, wz, wsum = B.alloc_weight_buffers(N, K, dev)
    B.basq_quantize_weights(lay.W_rot.to(dev), Wq, ws, wz, wsum)
    rng = np.random.default_rng(N)
    bc = rng.standard_normal(K).astype(np.float32)
    lb = rng.standard_normal(N).astype(np.float32)
    ob = torch.empty(N, dtype=torch.float32, device=dev)
    B.basq_fused_bias(Wq, ws, wz, torch.from_numpy(bc).to(dev), torch.from_numpy(lb).to(dev), ob)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(oracle.unpack_codes(Wq.cpu().numpy()), wq.codes)
    np.testing.assert_array_equal(si.bf16_bits(ws.cpu()), wq.scale_bits)
    np.testing.assert_array_equal(si.bf16_bits(wz.cpu()), wq.zero_bits)
    np.testing.assert_array_equal(wsum.cpu().numpy().view(np.uint32), wq.wsum.view(np.uint32))
    np.testing.assert_allclose(ob.cpu().numpy(), oracle.fused_bias(wq, bc, lb), rtol=1e-6, atol=1e-6)


@pytest.mark.parametrize("N,K,rot", [(40, 1024, 1024), (33, 1792, 1792), (24, 512, 128), (19, 8192, 8192)])
def test_offline_weight_rotation(N, K, rot):
    """W' = W R in bf16: the oracle's fp64 rotation rounded once to bf16.  The kernel rounds its fp32 rotation,
    so a value that sits within an fp32 rounding error of a bf16 tie may land on the neighbouring bf16 number:
    at most 1e-3 of the values, each by one unit in the last place.  And the reason the rotation may be folded
    into the weights at all (Eq. 14): (X R)(W R)^T = X W^T, here to bf16 accuracy."""
    dev = "cuda"
    lay = si.make_tiny(32, K, N, seed=N + rot)
    W = lay.W_rot                                                   # any bf16 matrix serves as the unrotated weights
    w = oracle.bf16_to_f32(si.bf16_bits(W))
    ref_bits = oracle.f64_to_bf16(oracle.rotate_f64(w, rot))
    out = torch.full((N, K), float("nan"), dtype=torch.bfloat16, device=dev)
    ws = torch.empty(N * K, dtype=torch.float32, device=dev)
    B.basq_rotate_weights(W.to(dev), rot, out, ws)
    torch.cuda.synchronize()
    got_bits = si.bf16_bits(out.cpu())
    diff = got_bits.astype(np.int32) - ref_bits.astype(np.int32)
    assert (np.abs(diff) <= 1).all(), "a rotated weight is more than one bf16 step from the oracle's"
    assert (diff != 0).mean() <= 1e-3, f"{(diff != 0).mean()} of the rotated weights differ"
    x = oracle.bf16_to_f32(si.bf16_bits(lay.X)).astype(np.float64)
    lhs = oracle.rotate_f64(x, rot) @ oracle.bf16_to_f32(got_bits).astype(np.float64).T
    rhs = x @ w.astype(np.float64).T
    assert np.abs(lhs - rhs).max() <= 2.0 ** -7 * np.abs(rhs).max()


@pytest.mark.parametrize("K,rot", [(1024, 1024), (1792, 1792)])
def test_bias_calibration(K, rot):
    dev = "cuda"
    lay = si.make_tiny(256, K, 8, seed=K)
    x = oracle.bf16_to_f32(si.bf16_bits(lay.X))
    ref = oracle.channel_bias(x, rot)
    out = torch.empty(K, dtype=torch.float32, device=dev)
    ws = torch.empty(256 * K, dtype=torch.float32, device=dev)
    B.basq_calibrate_bias(lay.X.to(dev), rot, None, out, ws)
    torch.cuda.synchronize()
    np.testing.assert_allclose(out.cpu().numpy(), ref, rtol=1e-5, atol=2e-6)


# ---------------------------------------------------------------- group-wise ranges (per-head quantisation)

def run_group_case(M, K, rot, group, *, seed=0, scale=False, bias=True, clip_lo=0.9, clip_hi=0.95, strided=False):
    """basq_rotate_quant with group_size < K against the oracle's group-wise quantiser: codes, group records
    and row sums bit-exact on the GPU's own rotation output; flips against the oracle's rotation rare and +-1."""
    announce(f"group case M={M} K={K} rot={rot} group={group} scale={scale} bias={bias}")
    lay = si.make_tiny(M, K, 8, seed=seed, n_outlier=8, outlier_scale=20.0)
    x = oracle.bf16_to_f32(si.bf16_bits(lay.X))
    rng = np.random.default_rng(seed + 1)
    b = oracle.channel_bias(oracle.bf16_to_f32(si.bf16_bits(lay.X_calib)), rot) if bias else None
    sa = rng.uniform(0.8, 1.25, K).astype(np.float32) if scale else None
    if b is not None and sa is not None:
        b = (b.astype(np.float64) * sa).astype(np.float32)
    dev = "cuda"
    X = lay.X.to(dev)
    if strided:
        wide = torch.zeros((M, K + 64), dtype=torch.bfloat16, device=dev)
        wide[:, :K] = X
        X = wide[:, :K]
    G = K // group
    Aq = torch.zeros((M, K // 2), dtype=torch.uint8, device=dev)
    meta = torch.zeros((M * G, 4), dtype=torch.int32, device=dev)
    rot_out = torch.empty((M, K), dtype=torch.float32, device=dev)
    tb = None if b is None else torch.from_numpy(b).to(dev)
    ts = None if sa is None else torch.from_numpy(sa).to(dev)
    B.basq_rotate_quant(X, rot, tb, ts, clip_lo, clip_hi, Aq, meta, rot_out, group_size=group)
    Aq2 = torch.zeros_like(Aq)
    meta2 = torch.zeros_like(meta)
    B.basq_rotate_quant(X, rot, tb, ts, clip_lo, clip_hi, Aq2, meta2, None, group_size=group)   # no debug output: the fast variant
    torch.cuda.synchronize()
    assert torch.equal(Aq, Aq2) and torch.equal(meta, meta2)
    r_gpu = rot_out.cpu().numpy()
    ref = oracle.quantize_tokens(r_gpu, b, sa, clip_lo, clip_hi, group_size=group)
    codes = oracle.unpack_codes(Aq.cpu().numpy())
    mh = meta.cpu().numpy().reshape(M, G, 4)
    np.testing.assert_array_equal(codes, ref.codes, err_msg="codes (GPU rotation fed to the oracle)")
    np.testing.assert_array_equal(mh[:, :, 0].copy().view(np.uint32), ref.scale.view(np.uint32), err_msg="group scales")
    np.testing.assert_array_equal(mh[:, :, 1].copy().view(np.uint32), ref.lo.view(np.uint32), err_msg="group lower bounds")
    np.testing.assert_array_equal(mh[:, :, 2], ref.rowsum, err_msg="group code sums")
    r_ref = oracle.rotate(x, rot)
    assert np.abs(r_gpu - r_ref).max() <= 2e-5 * max(1.0, float(np.abs(r_ref).max()))
    full = oracle.quantize_tokens(r_ref, b, sa, clip_lo, clip_hi, group_size=group)
    d = codes.astype(np.int32) - full.codes.astype(np.int32)
    assert (d != 0).mean() <= 1e-4 and (np.abs(d[d != 0]) == 1).all()


@pytest.mark.parametrize("M,K", [(70, 4096), (33, 1024), (5, 512), (600, 2048)])
def test_per_head_kernel(M, K):
    """rot_size = group_size = 128: the wave-local kernel (one 512-channel item per wavefront)."""
    run_group_case(M, K, 128, 128, seed=K + M)


@pytest.mark.parametrize("M,K,scale,bias", [(9, 4096, False, True), (70, 8192, False, True), (6, 4096, True, True), (5, 8192, True, False)])
def test_full_rotation_with_groups_of_128(M, K, scale, bias):
    """rot_size = K in {4096, 8192} with group_size = 128: the one-wave-per-token kernel with one range per four
    neighbouring lanes."""
    run_group_case(M, K, K, 128, seed=K + M, scale=scale, bias=bias)


def test_per_head_kernel_variants():
    run_group_case(40, 4096, 128, 128, seed=1, scale=True)
    run_group_case(40, 1024, 128, 128, seed=2, bias=False, clip_lo=1.0, clip_hi=1.0)
    run_group_case(19, 2048, 128, 128, seed=3, strided=True)


@pytest.mark.parametrize("K,rot,group", [(1024, 64, 64), (1024, 128, 256), (768, 32, 96), (1024, 1024, 128), (28 * 64, 28 * 64, 64)])
def test_groupwise_ranges_generic_kernel(K, rot, group):
    """Other group sizes, groups that differ from the rotation block, and a 28 * 2^t rotation."""
    run_group_case(37, K, rot, group, seed=K + group)


# ---------------------------------------------------------------- group-wise ranges through the GEMM

def run_grouped_layer(M, K, N, rot, *, seed=0, scale=False, odd_ldy=False):
    """rotate+quant with group_size = 128, then basq_w4a4_gemm_grouped (int8 path, then fp6 path: same bits), against
    oracle.linear_grouped:
    (i) codes and group records bit-exact on the GPU's rotation; group column sums bit-exact;
    (ii) outputs: element by element within one bf16 step (2^-8 relative) plus 1e-5 of max|ref| of the oracle's
    output on the same codes (the kernel sums the groups in fp32, the oracle in fp64), and within 2e-2 of
    max|ref| of the oracle's output from X with its own rotation."""
    announce(f"grouped layer M={M} K={K} N={N} rot={rot} scale={scale}")
    dev = "cuda"
    G = 128
    lay = si.make_tiny(M, K, N, seed=seed, n_outlier=8, outlier_scale=20.0)
    x = oracle.bf16_to_f32(si.bf16_bits(lay.X))
    w = oracle.bf16_to_f32(si.bf16_bits(lay.W_rot))
    wq = oracle.quantize_weights(w)
    b = oracle.channel_bias(oracle.bf16_to_f32(si.bf16_bits(lay.X_calib)), rot)
    sa = np.random.default_rng(seed + 5).uniform(0.8, 1.25, K).astype(np.float32) if scale else None
    if sa is not None:
        b = (b.astype(np.float64) * sa).astype(np.float32)
    c = oracle.fused_bias(wq, b, None)
    ng = K // G
    X = lay.X.to(dev)
    Aq = torch.zeros((M, K // 2), dtype=torch.uint8, device=dev)
    meta = torch.zeros((M * ng, 4), dtype=torch.int32, device=dev)
    rot_out = torch.empty((M, K), dtype=torch.float32, device=dev)
    tb = torch.from_numpy(b).to(dev)
    ts = None if sa is None else torch.from_numpy(sa).to(dev)
    Wq = torch.from_numpy(oracle.pack_codes(wq.codes)).to(dev)
    w_scale = si.bits_to_bf16(wq.scale_bits).to(dev)
    w_zero = si.bits_to_bf16(wq.zero_bits).to(dev)
    out_bias = torch.from_numpy(c).to(dev)
    gsum = torch.full((ng, N), -1, dtype=torch.int32, device=dev)
    ldy = N + 3 if odd_ldy else N
    Ybuf = torch.full((M, ldy), float("nan"), dtype=torch.bfloat16, device=dev)
    Y = Ybuf[:, :N]
    A6 = B.alloc_fp6_buffer(M, K, dev).zero_()
    A6b = torch.zeros_like(A6)
    W6 = B.alloc_fp6_buffer(N, K, dev).zero_()
    B.basq_rotate_quant(X, rot, tb, ts, 0.9, 0.95, Aq, meta, rot_out, group_size=G, Aq6=A6)
    B.basq_group_colsums(Wq, G, gsum)
    B.basq_w4a4_gemm_grouped(Aq, meta, G, Wq, w_scale, w_zero, gsum, out_bias, Y)
    # the same product on the fp6 matrix-core path: bit-identical outputs
    B.basq_pack_fp6(Aq, A6b)
    B.basq_pack_fp6(Wq, W6)
    Y6buf = torch.full((M, ldy), float("nan"), dtype=torch.bfloat16, device=dev)
    B.basq_w4a4_gemm_grouped(Aq, meta, G, Wq, w_scale, w_zero, gsum, out_bias, Y6buf[:, :N], Aq6=A6, Wq6=W6)
    torch.cuda.synchronize()
    assert torch.equal(A6, A6b), "fp6 copy written with group-wise ranges differs from the packed codes"
    assert torch.equal(Y6buf[:, :N].view(torch.int16), Y.view(torch.int16)), "fp6 and int8 group-wise GEMMs differ"
    if odd_ldy:
        assert torch.isnan(Y6buf[:, N:]).all(), "fp6 path wrote past the row"
    np.testing.assert_array_equal(gsum.cpu().numpy(), oracle.group_colsums(wq, G), err_msg="group column sums")
    ref_i = oracle.linear_grouped(x, rot, b, sa, 0.9, 0.95, G, wq, c, r=rot_out.cpu().numpy())
    np.testing.assert_array_equal(oracle.unpack_codes(Aq.cpu().numpy()), ref_i.tq.codes, err_msg="codes")
    mh = meta.cpu().numpy().reshape(M, ng, 4)
    np.testing.assert_array_equal(mh[:, :, 0].copy().view(np.uint32), ref_i.tq.scale.view(np.uint32))
    np.testing.assert_array_equal(mh[:, :, 1].copy().view(np.uint32), ref_i.tq.lo.view(np.uint32))
    np.testing.assert_array_equal(mh[:, :, 2], ref_i.tq.rowsum)
    y = oracle.bf16_to_f32(si.bf16_bits(Y.cpu())).astype(np.float64)
    assert np.isfinite(y).all()
    top = float(np.abs(ref_i.y).max())
    assert (np.abs(y - ref_i.y) <= 2.0 ** -8 * np.abs(ref_i.y) + 1e-5 * top).all(), \
        f"worst {np.abs(y - ref_i.y).max() / top} of max|ref| on identical codes"
    if odd_ldy:
        assert torch.isnan(Ybuf[:, N:]).all(), "wrote past the row"
    ref = oracle.linear_grouped(x, rot, b, sa, 0.9, 0.95, G, wq, c)
    err = float(np.abs(y - ref.y).max() / np.abs(ref.y).max())
    assert err <= pu.Y_TOL, f"output error {err}"
    announce(f"ok y_err {err:.2e}")


@pytest.mark.parametrize("M,K,N,rot", [(128, 128, 128, 128), (130, 256, 136, 128), (70, 1024, 200, 1024), (257, 512, 100, 128),
                                       (5, 384, 17, 128), (300, 4096, 264, 4096), (200, 8192, 136, 8192), (140, 8192, 72, 128)])
def test_grouped_gemm(M, K, N, rot):
    """Group-wise activation ranges through the GEMM: one, two, several, 32 and 64 groups; ragged tiles in both
    directions; output widths that are no multiple of 8; per-head rotation (128) and full rotation."""
    run_grouped_layer(M, K, N, rot, seed=M + N)


def test_grouped_gemm_with_scale_and_unaligned_rows():
    run_grouped_layer(140, 768, 72, 128, seed=9, scale=True, odd_ldy=True)


# ---------------------------------------------------------------- HIP graph capture

@pytest.mark.parametrize("M,K,N,stream_layout", [(1, 4096, 4096, True), (16, 4096, 256, True), (40, 1024, 200, False), (200, 512, 136, False)])
def test_calls_can_be_captured_in_a_graph(M, K, N, stream_layout):
    """Hot calls allocate nothing, never synchronise and launch only kernels, so a serving loop may record them in a
    HIP graph: four layer calls are captured once and replayed three times, with eager work and synchronisations in
    between and fresh inputs before every replay; every replay must reproduce the eager call's bits."""
    dev = torch.device("cuda")
    lay = si.make_tiny(M, K, N, seed=M + N)
    case = pu.make_case(lay)
    d = pu.to_device(case)
    Wq, layout = d.Wq, B.BASQ_W_CANONICAL
    if stream_layout:
        Wq = torch.empty(B.basq_decode_bytes(N, K), dtype=torch.uint8, device=dev)
        B.basq_pack_decode(d.Wq, Wq)
        layout = B.BASQ_W_DECODE16
    W6 = None
    if M > B.STREAM_MAX_TOKENS:
        W6 = B.alloc_fp6_buffer(N, K, dev)
        B.basq_pack_fp6(d.Wq, W6)
    ws = torch.empty(max(B.basq_workspace_bytes(M, K, N), 256), dtype=torch.uint8, device=dev)
    X = [d.X.clone() for _ in range(4)]
    Y = [torch.empty((M, N), dtype=torch.bfloat16, device=dev) for _ in range(4)]

    def layer(i, stream=None):
        B.basq_linear_fused(X[i], case.rot_size, d.bias, d.act_scale, case.clip_lo, case.clip_hi, Wq, d.w_scale, d.w_zero,
                            d.w_sum, d.out_bias, Y[i], ws, Wq6=W6, w_layout=layout, N=N, stream=stream)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for i in range(4):
            layer(i)
    torch.cuda.synchronize()
    gen = torch.Generator(device="cpu").manual_seed(7)
    for rep in range(3):
        for i in range(4):                               # new tokens in the captured buffers
            X[i].copy_((torch.randn((M, K), generator=gen) * (1.0 + rep)).to(torch.bfloat16))
            Y[i].fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [y.clone() for y in Y]
        for i in range(4):                               # the same calls, eagerly
            Y[i].fill_(float("nan"))
            layer(i)
        torch.cuda.synchronize()
        for i in range(4):
            assert not torch.isnan(got[i].float()).any()
            assert torch.equal(got[i], Y[i]), f"replay {rep}, call {i}"
