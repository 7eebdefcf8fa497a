"""GPU parity on the edges of the fast rotate+quant kernels, through the C ABI against the CPU oracle.

Degenerate tokens (Eq. 4 has no answer for a token whose range is empty or not finite; the reading taken is
s = 1, NaN -> code 0, min/max ignore NaN) on every specialised kernel and on both sides of each of their
token-count switches, always as: the GPU's fp32 rotation of the checked rows (`rot_out`) -> oracle.quantize_tokens
-> codes and the BITS of scale, lower bound and row sum must equal what the kernel under test wrote for those rows.
The kernel under test runs WITHOUT `rot_out` (that is what selects the fast variants), with and without the fp6 copy.
Then: the many-token path, the one-launch decode kernel, and the group-wise layer at full benchmark size."""
import sys

import numpy as np
import pytest
import torch

import oracle
import layout_ref
from paper_2506_15689_amd import binding as B
from paper_2506_15689_amd import synth_inputs as si

import parity_util as pu

pytestmark = pytest.mark.gpu

DEV = "cuda"
N_SPECIAL = 10


def announce(msg):
    print(f"[edge] {msg}", flush=True)
    sys.stdout.flush()


def plant_degenerate_rows(X: torch.Tensor, first: int) -> None:
    """Overwrites rows first .. first + N_SPECIAL - 1 of X (bf16 [M, K]) with the degenerate tokens."""
    K = X.shape[1]
    X[first:first + N_SPECIAL] = 0.0                      # +0: all-zero token (constant when there is no bias)
    X[first + 1, 0] = 1.0                                 # rotates to the constant 1/sqrt(n) in its first block
    X[first + 2, K // 3] = float("nan")                   # NaN in every channel of that block after the rotation
    X[first + 3, 5] = float("inf")                        # +-inf everywhere in the block
    X[first + 4, K - 1] = float("-inf")
    X[first + 5, 3] = float("inf")                        # two infinities of one block: inf - inf = NaN in half of
    X[first + 5, 64] = float("inf")                       # the outputs, +-inf in the rest
    X[first + 6, :] = 3.0e38                              # finite inputs whose sums overflow
    X[first + 7, 0] = 2.0 ** -126                         # rotates into the subnormal range
    X[first + 8, :] = -1.5                                # one non-zero output per rotation block, the rest exact zeros
    X[first + 9, :] = float("nan")                        # nothing finite at all


def gpu_inputs(M, K, seed, *, with_bias, with_scale):
    gen = torch.Generator(device=DEV).manual_seed(seed)
    X = (torch.randn((M, K), generator=gen, device=DEV) * 1.5).to(torch.bfloat16)
    X[:, 7] *= 20.0                                       # an outlier channel (Sec. 3.1)
    bias = (torch.randn(K, generator=gen, device=DEV) * 0.3) if with_bias else None
    sa = (torch.rand(K, generator=gen, device=DEV) * 0.45 + 0.8) if with_scale else None
    return X, bias, sa


def rows_to_check(M, specials, rng, n_random=64):
    rows = set()
    for f in specials:
        rows |= set(range(f, f + N_SPECIAL))
    rows |= {0, M - 1}
    rows |= set(int(v) for v in rng.choice(M, size=min(n_random, M), replace=False))
    return np.array(sorted(rows))


def check_fp6_copy(Aq, A6, K, row_blocks):
    """The fp6 copy against the repacking kernel everywhere (whole 32-row blocks; the bytes of rows past M in the
    last block are undefined) and against the layout reference on the given 32-row blocks."""
    M = Aq.shape[0]
    A6b = torch.zeros_like(A6)
    B.basq_pack_fp6(Aq, A6b)
    torch.cuda.synchronize()
    RB = (M + 31) // 32
    full = M // 32
    v, vb = A6.view(K // 128, RB, 3072), A6b.view(K // 128, RB, 3072)
    assert torch.equal(v[:, :full], vb[:, :full]), "fp6 copy written by the quantiser differs from the repacked codes"
    for rb in row_blocks:
        if rb < 0 or rb >= full:
            continue
        codes = oracle.unpack_codes(Aq[32 * rb:32 * rb + 32].cpu().numpy())
        ref6 = layout_ref.pack_fp6(codes).reshape(K // 128, 3072)
        np.testing.assert_array_equal(v[:, rb].cpu().numpy(), ref6, err_msg=f"fp6 copy, row block {rb}")


# K = 4096: several waves per token up to 512 tokens, one wave per token in four-wave workgroups up to 2047,
# eight-wave workgroups up to 32767, and from 32768 tokens on with the fp6 copy the staged tails.
# K = 8192: split up to 256, four waves to 2047, eight waves to 4096, four waves beyond, staged tails from 32768;
# with s^a (staged in LDS beside b^c) eight waves from 1025 tokens on.
# K = 14336: two waves per token; four-wave workgroups, eight when both b^c and s^a are staged; 1024 tokens per round.
SWITCH_CASES = [
    (4096, 12), (4096, 512), (4096, 513), (4096, 2047), (4096, 2048), (4096, 2061), (4096, 32768 + 13),
    (8192, 11), (8192, 256), (8192, 257), (8192, 1024), (8192, 1025), (8192, 2047), (8192, 2048), (8192, 4096), (8192, 4097), (8192, 12301), (8192, 32768 + 13),
    (14336, 11), (14336, 131), (14336, 1030), (14336, 2048 + 5),
]


@pytest.mark.parametrize("K,M", SWITCH_CASES)
@pytest.mark.parametrize("with_bias,with_scale", [(False, False), (True, False), (True, True)])
def test_degenerate_tokens_on_the_fast_kernels(K, M, with_bias, with_scale):
    if M > 20000 and with_scale:
        pytest.skip("the many-token variants do not depend on s^a; covered with and without the bias")
    announce(f"degenerate tokens K={K} M={M} bias={with_bias} scale={with_scale}")
    X, bias, sa = gpu_inputs(M, K, seed=K + M, with_bias=with_bias, with_scale=with_scale)
    specials = sorted({0, M - N_SPECIAL} | ({M // 2 - 3} if M >= 4 * N_SPECIAL else set()))
    for f in reversed(specials):                          # the set at row 0 is planted last and stays whole
        plant_degenerate_rows(X, f)
    rng = np.random.default_rng(K + M)
    rows = rows_to_check(M, specials, rng)
    clip_lo, clip_hi = 0.9, 0.95
    # without the fp6 copy
    Aq, meta = B.alloc_activation_buffers(M, K, DEV)
    Aq.fill_(0xEE); meta.fill_(-7)
    B.basq_rotate_quant(X, K, bias, sa, clip_lo, clip_hi, Aq, meta)
    ref = pu.check_rows_against_oracle(X, rows, K, bias, sa, clip_lo, clip_hi, Aq, meta, what="no fp6 copy")
    # what the reading of a degenerate token promises, on the oracle's own output (rows of the first planted set)
    pos = {int(r): i for i, r in enumerate(rows)}
    f0 = specials[0]
    if not with_bias and not with_scale:
        i = pos[f0]                                       # the all-zero token is constant: s := 1, every code 0
        assert ref.scale[i, 0] == 1.0 and ref.lo[i, 0] == 0.0 and not ref.codes[i].any()
        i = pos[f0 + 1]                                   # a constant c > 0 with unequal clips: range [0.9 c, 0.95 c]
        assert ref.scale[i, 0] > 0 and set(np.unique(ref.codes[i])) == {15}
    i = pos[f0 + 9]
    assert ref.scale[i, 0] == 1.0 and not ref.codes[i].any(), "an all-NaN token has no finite range: s = 1, codes 0"
    i = pos[f0 + 2]
    assert not ref.codes[i].any(), "NaN -> code 0"
    # with the fp6 copy: same codes and records, and the copy holds the same codes
    Aq2, meta2 = B.alloc_activation_buffers(M, K, DEV)
    A6 = B.alloc_fp6_buffer(M, K, DEV).zero_()
    B.basq_rotate_quant(X, K, bias, sa, clip_lo, clip_hi, Aq2, meta2, Aq6=A6)
    torch.cuda.synchronize()
    pu.check_rows_against_oracle(X, rows, K, bias, sa, clip_lo, clip_hi, Aq2, meta2, what="with the fp6 copy")
    assert torch.equal(Aq2, Aq) and torch.equal(meta2[:, :3], meta[:, :3]), "codes or records change with the fp6 copy"
    check_fp6_copy(Aq2, A6, K, sorted({f // 32 for f in specials} | {(M - 1) // 32 - 1}))
    # the fp6 form alone (what the one-call layer asks for on the fp6 matrix path): same records, same fp6 bytes
    meta3 = torch.full_like(meta2, -7)
    A6c = B.alloc_fp6_buffer(M, K, DEV).zero_()
    B.basq_rotate_quant(X, K, bias, sa, clip_lo, clip_hi, None, meta3, Aq6=A6c)
    torch.cuda.synchronize()
    full = M // 32
    assert torch.equal(meta3[:, :3], meta2[:, :3]), "records change when the 4-bit codes are left out"
    assert torch.equal(A6c.view(K // 128, -1, 3072)[:, :full], A6.view(K // 128, -1, 3072)[:, :full]), \
        "fp6 form changes when the 4-bit codes are left out"
    # properties on all rows
    rs = meta[:, 2].to(torch.int64)
    assert torch.equal(rs, (Aq & 0x0F).to(torch.int64).sum(dim=1) + (Aq >> 4).to(torch.int64).sum(dim=1))


@pytest.mark.parametrize("K,M,rot,group", [(4096, 70, 128, 128), (2048, 600, 128, 128), (8192, 37, 128, 128),
                                           (4096, 12, 4096, 128), (8192, 70, 8192, 128), (1024, 33, 64, 64)])
@pytest.mark.parametrize("with_bias", [False, True])
def test_degenerate_tokens_with_groupwise_ranges(K, M, rot, group, with_bias):
    """Per-head kernel (rot = group = 128), the one-wave-per-token kernel with a range per four lanes
    (rot = K, group = 128) and the generic kernel: a degenerate GROUP next to ordinary ones in the same token."""
    announce(f"degenerate groups K={K} M={M} rot={rot} group={group} bias={with_bias}")
    X, bias, sa = gpu_inputs(M, K, seed=K + M + group, with_bias=with_bias, with_scale=False)
    specials = [0, M - N_SPECIAL]
    for f in reversed(specials):
        plant_degenerate_rows(X, f)
    # ordinary tokens with one dead head: all-zero, NaN and inf confined to one rotation block (rot = 128 only)
    if rot == 128 and M > 30:
        X[12, 256:384] = 0.0
        X[13, 128 + 5] = float("nan")
        X[14, 384 + 9] = float("inf")
    rows = np.arange(M) if M <= 80 else np.union1d(rows_to_check(M, specials, np.random.default_rng(M), n_random=48), [12, 13, 14])
    ng = K // group
    Aq = torch.full((M, K // 2), 0xEE, dtype=torch.uint8, device=DEV)
    meta = torch.full((M * ng, 4), -7, dtype=torch.int32, device=DEV)
    B.basq_rotate_quant(X, rot, bias, sa, 0.9, 0.95, Aq, meta, group_size=group)
    torch.cuda.synchronize()
    pu.check_rows_against_oracle(X, rows, rot, bias, sa, 0.9, 0.95, Aq, meta, group=group, what="group-wise")


@pytest.mark.parametrize("K,M,rot", [(11008, 300, 256), (1280, 70, 128), (2048, 41, 512), (768, 33, 256), (16384, 25, 512)])
@pytest.mark.parametrize("with_bias,with_scale", [(False, False), (True, False), (True, True)])
def test_degenerate_tokens_on_the_blockwise_kernel(K, M, rot, with_bias, with_scale):
    """Blockwise rotations of 128, 256 and 512 channels with per-token ranges (the register-resident blockwise
    kernel; K = 11008 and 768 end in a half piece of 256 channels): the degenerate tokens at both ends of the batch,
    and ordinary tokens with one dead rotation block (zero, NaN, inf confined to it)."""
    announce(f"degenerate tokens, blockwise K={K} M={M} rot={rot} bias={with_bias} scale={with_scale}")
    X, bias, sa = gpu_inputs(M, K, seed=K + M + rot, with_bias=with_bias, with_scale=with_scale)
    specials = [0, M - N_SPECIAL]
    for f in reversed(specials):
        plant_degenerate_rows(X, f)
    X[12, rot:2 * rot] = 0.0
    X[13, rot + 5] = float("nan")
    X[14, K - rot + 9] = float("inf")
    rows = np.arange(M) if M <= 80 else np.union1d(rows_to_check(M, specials, np.random.default_rng(M), n_random=48), [12, 13, 14])
    Aq, meta = B.alloc_activation_buffers(M, K, DEV)
    Aq.fill_(0xEE); meta.fill_(-7)
    A6 = B.alloc_fp6_buffer(M, K, DEV)
    B.basq_rotate_quant(X, rot, bias, sa, 0.9, 0.95, Aq, meta, Aq6=A6)
    torch.cuda.synchronize()
    pu.check_rows_against_oracle(X, rows, rot, bias, sa, 0.9, 0.95, Aq, meta, what="blockwise")
    check_fp6_copy(Aq, A6, K, row_blocks=[0, (M // 32) - 1])


@pytest.mark.parametrize("K", [4096, 8192])
@pytest.mark.parametrize("M", [1, 2, 4])
@pytest.mark.parametrize("with_bias", [False, True])
def test_degenerate_tokens_through_the_one_launch_decode_kernel(K, M, with_bias):
    """basq_linear_fused with at most four tokens on the streaming layout is one kernel that rotates, quantises and
    multiplies; its codes never reach memory, so the output is what is compared: with oracle.linear on the GPU's
    rotation of the same tokens (a separate call), NaN-aware -- where the reference is finite the usual tolerance,
    elsewhere the same kind of non-finite value -- and bit for bit with the two-call path."""
    N = 264
    lay = si.make_tiny(max(M, 16), K, N, seed=K + M)
    case = pu.make_case(lay, use_bias=with_bias, use_out_bias=with_bias)
    d = pu.to_device(case)
    kinds = {1: [[9], [0], [3], [6]], 2: [[0, 2], [3, 7]], 4: [[0, 1, 2, 3], [5, 6, 8, 9]]}[M]
    Wd = torch.empty(B.basq_decode_bytes(N, K), dtype=torch.uint8, device=DEV)
    B.basq_pack_decode(d.Wq, Wd)
    for kind in kinds + [None]:
        announce(f"one-launch decode K={K} M={M} bias={with_bias} degenerate kinds={kind}")
        X = d.X[:M].clone()
        if kind is not None:
            scratch = torch.zeros((N_SPECIAL, K), dtype=torch.bfloat16, device=DEV)
            plant_degenerate_rows(scratch, 0)
            for i, k in enumerate(kind):
                X[i] = scratch[k]
        Y1 = torch.full((M, N), 7.0, dtype=torch.bfloat16, device=DEV)
        ws = torch.empty(max(B.basq_workspace_bytes(M, K, N), 256), dtype=torch.uint8, device=DEV)
        B.basq_linear_fused(X, K, d.bias, None, case.clip_lo, case.clip_hi, Wd, d.w_scale, d.w_zero, d.w_sum,
                            d.out_bias, Y1, ws, w_layout=B.BASQ_W_DECODE16, N=N)
        # the two-call path on the same tokens, with the rotation dumped for the oracle
        Aq, meta = B.alloc_activation_buffers(M, K, DEV)
        r = torch.empty((M, K), dtype=torch.float32, device=DEV)
        Y2 = torch.full((M, N), 7.0, dtype=torch.bfloat16, device=DEV)
        B.basq_rotate_quant(X, K, d.bias, None, case.clip_lo, case.clip_hi, Aq, meta, r)
        B.basq_w4a4_gemm(Aq, meta, Wd, d.w_scale, d.w_zero, d.w_sum, d.out_bias, Y2, w_layout=B.BASQ_W_DECODE16, N=N)
        torch.cuda.synchronize()
        y1, y2 = si.bf16_bits(Y1.cpu()), si.bf16_bits(Y2.cpu())
        np.testing.assert_array_equal(y1, y2, err_msg="one launch vs two calls")
        x = oracle.bf16_to_f32(si.bf16_bits(X.cpu()))
        with np.errstate(all="ignore"):
            ref = oracle.linear(x, K, case.bias, None, case.clip_lo, case.clip_hi, case.wq, case.c, r=r.cpu().numpy())
        np.testing.assert_array_equal(oracle.unpack_codes(Aq.cpu().numpy()), ref.tq.codes)
        y = oracle.bf16_to_f32(y1).astype(np.float64)
        # bf16's largest finite value: beyond it the reference itself rounds to infinity
        fin = np.isfinite(ref.y) & (np.abs(ref.y) < 3.0e38)
        assert np.isfinite(y[fin]).all(), "a finite reference output came out non-finite"
        for m in range(M):                                # row by row: a degenerate token's outputs can be huge
            if fin[m].any():
                top = float(np.abs(ref.y[m][fin[m]]).max())
                assert np.abs(y[m][fin[m]] - ref.y[m][fin[m]]).max() <= pu.Y_TOL * max(top, 1e-30), f"token {m}"
        nan_ref = np.isnan(ref.y)
        assert np.isnan(y[nan_ref]).all(), "NaN in the reference, a number on the GPU"
        inf_ref = np.isinf(ref.y)
        assert (y[inf_ref] == ref.y[inf_ref]).all(), "infinite reference output: the GPU's differs"


@pytest.mark.parametrize("K", [8192, 4096])
def test_grouped_layer_at_benchmark_size(K):
    """The group-wise layer (activation ranges per 128 channels) at the size and in the launch configuration the
    benchmark times with --group-size 128 -- C5 (K = 8192: 64 groups) and C2 (K = 4096) -- checked on sampled token
    rows x output channels that include the first and last tiles: codes and group records bit-exact on the GPU's
    rotation, outputs within one bf16 step of oracle.linear_grouped on the same codes, within 2e-2 of max|ref| from
    X; the fp6 path (benchmarked) and the int8 path bit-identical on ALL elements."""
    name = "C5" if K == 8192 else "C2"
    cfg = si.CONFIGS[name]
    G = 128
    lay = si.make_layer(cfg)
    M, N = cfg.M, cfg.N
    ng = K // G
    announce(f"grouped layer at full size: {name} M={M} K={K} N={N}")
    rng = np.random.default_rng(cfg.index + 100)
    edge = 34
    rows = np.array(sorted(set(range(edge)) | set(range(M - edge, M)) | set(int(v) for v in rng.choice(M, 40, replace=False))))
    cols = np.array(sorted(set(range(edge)) | set(range(N - edge, N)) | set(int(v) for v in rng.choice(N, 400, replace=False))))
    xc = oracle.bf16_to_f32(si.bf16_bits(lay.X_calib))
    bc = oracle.channel_bias(xc, cfg.rot_size)
    w_s = oracle.bf16_to_f32(si.bf16_bits(lay.W_rot[torch.from_numpy(cols)]))
    wq_s = oracle.quantize_weights(w_s)
    c_s = oracle.fused_bias(wq_s, bc, None)

    W = lay.W_rot.to(DEV)
    Wq, w_scale, w_zero, w_sum = B.alloc_weight_buffers(N, K, DEV)
    B.basq_quantize_weights(W, Wq, w_scale, w_zero, w_sum)
    del W
    bias = torch.from_numpy(bc).to(DEV)
    out_bias = torch.empty(N, dtype=torch.float32, device=DEV)
    B.basq_fused_bias(Wq, w_scale, w_zero, bias, None, out_bias)
    gsum = torch.empty((ng, N), dtype=torch.int32, device=DEV)
    B.basq_group_colsums(Wq, G, gsum)
    W6 = B.alloc_fp6_buffer(N, K, DEV)
    B.basq_pack_fp6(Wq, W6)
    X = lay.X.to(DEV)
    Aq = torch.empty((M, K // 2), dtype=torch.uint8, device=DEV)
    meta = torch.empty((M * ng, 4), dtype=torch.int32, device=DEV)
    A6 = B.alloc_fp6_buffer(M, K, DEV)
    B.basq_rotate_quant(X, cfg.rot_size, bias, None, cfg.clip, cfg.clip, Aq, meta, group_size=G, Aq6=A6)
    Y6 = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
    B.basq_w4a4_gemm_grouped(Aq, meta, G, Wq, w_scale, w_zero, gsum, out_bias, Y6, Aq6=A6, Wq6=W6)
    Y8 = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
    B.basq_w4a4_gemm_grouped(Aq, meta, G, Wq, w_scale, w_zero, gsum, out_bias, Y8)
    torch.cuda.synchronize()
    assert torch.equal(Y6.view(torch.int16), Y8.view(torch.int16)), "fp6 and int8 group-wise GEMMs differ"
    assert not torch.isnan(Y6).any()

    t_rows, t_cols = torch.from_numpy(rows).to(DEV), torch.from_numpy(cols).to(DEV)
    np.testing.assert_array_equal(oracle.unpack_codes(Wq[t_cols].cpu().numpy()), wq_s.codes)
    np.testing.assert_array_equal(gsum[:, t_cols].cpu().numpy(), oracle.group_colsums(wq_s, G), err_msg="group column sums")
    ref_q = pu.check_rows_against_oracle(X, rows, cfg.rot_size, bias, None, cfg.clip, cfg.clip, Aq, meta, group=G,
                                      what="group-wise ranges at full size")
    x_s = oracle.bf16_to_f32(si.bf16_bits(lay.X[torch.from_numpy(rows)]))
    # the oracle's layer on the codes just verified: its quantiser is deterministic, so feed it the same rotation
    Xs = X[t_rows].contiguous()
    r = torch.empty((len(rows), K), dtype=torch.float32, device=DEV)
    B.basq_rotate_quant(Xs, cfg.rot_size, bias, None, cfg.clip, cfg.clip,
                        torch.empty((len(rows), K // 2), dtype=torch.uint8, device=DEV),
                        torch.empty((len(rows) * ng, 4), dtype=torch.int32, device=DEV), r, group_size=G)
    torch.cuda.synchronize()
    ref_i = oracle.linear_grouped(x_s, cfg.rot_size, bc, None, cfg.clip, cfg.clip, G, wq_s, c_s, r=r.cpu().numpy())
    np.testing.assert_array_equal(ref_i.tq.codes, ref_q.codes)
    y = oracle.bf16_to_f32(si.bf16_bits(Y6[t_rows][:, t_cols].cpu())).astype(np.float64)
    top = float(np.abs(ref_i.y).max())
    worst = float((np.abs(y - ref_i.y) - 2.0 ** -8 * np.abs(ref_i.y)).max() / top)
    assert worst <= 1e-5, f"worst excess over one bf16 step: {worst} of max|ref| on identical codes"
    ref = oracle.linear_grouped(x_s, cfg.rot_size, bc, None, cfg.clip, cfg.clip, G, wq_s, c_s)
    err = float(np.abs(y - ref.y).max() / np.abs(ref.y).max())
    assert err <= pu.Y_TOL, f"output error {err}"
    d = ref_q.codes.astype(np.int32) - ref.tq.codes.astype(np.int32)
    assert (d != 0).mean() <= pu.FLIP_TOL and (np.abs(d[d != 0]) == 1).all()
    announce(f"ok rows={len(rows)} cols={len(cols)} y_err={err:.2e} flips={(d != 0).mean():.2e}")


def test_worst_case_accumulator_on_both_matrix_paths():
    """The fp6 path is exact because S = sum (q_a/8)(q_w/8) fits the fp32 accumulator: at the longest row it takes,
    K = 32768, with every code 15 on both sides the INT32 accumulator of Sec. 5.2's INT4 GEMM must be 225 K on the
    fp6 path and on the int8 path; a few columns of smaller codes check that nothing saturates on the way."""
    K, M, N = 32768, 200, 72
    codes_a = torch.full((M, K // 2), 0xFF, dtype=torch.uint8, device=DEV)
    codes_w = torch.full((N, K // 2), 0xFF, dtype=torch.uint8, device=DEV)
    codes_w[5] = 0x11                                      # every code 1: ACC = 15 K
    codes_w[6] = 0xF0                                      # alternating 0, 15: ACC = 225 K / 2
    meta = torch.zeros((M, 4), dtype=torch.int32, device=DEV)
    meta[:, 0] = torch.tensor(1.0).view(torch.int32)       # scale 1, lower bound 0
    meta[:, 2] = 15 * K
    w_scale = torch.ones(N, dtype=torch.bfloat16, device=DEV)
    w_zero = torch.zeros(N, dtype=torch.bfloat16, device=DEV)
    w_sum = torch.zeros(N, dtype=torch.float32, device=DEV)
    A6, W6 = B.alloc_fp6_buffer(M, K, DEV), B.alloc_fp6_buffer(N, K, DEV)
    B.basq_pack_fp6(codes_a, A6)
    B.basq_pack_fp6(codes_w, W6)
    want = np.full((M, N), 225 * K, dtype=np.int64)
    want[:, 5] = 15 * K
    want[:, 6] = 225 * K // 2
    for name, kw in (("int8", {}), ("fp6", dict(Aq6=A6, Wq6=W6))):
        announce(f"worst-case accumulator, {name} path")
        acc = torch.full((M, N), -1, dtype=torch.int32, device=DEV)
        Y = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
        B.basq_w4a4_gemm(codes_a, meta, codes_w, w_scale, w_zero, w_sum, None, Y, acc, **kw)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(acc.cpu().numpy().astype(np.int64), want, err_msg=f"{name} path")
    # and the oracle's triple loop agrees on a few rows
    ref = oracle.int_gemm(oracle.unpack_codes(codes_a[:2].cpu().numpy()), oracle.unpack_codes(codes_w.cpu().numpy()))
    np.testing.assert_array_equal(ref, want[:2])


@pytest.mark.parametrize("N,K,with_bias,with_layer_bias", [(72, 512, True, True), (100, 1792, True, False),
                                                           (40, 4096, False, True), (33, 256, False, False)])
def test_prepare_weights_against_the_oracle(N, K, with_bias, with_layer_bias):
    """basq_prepare_weights: w_sum bit-exact against the oracle's weight quantiser, the fused bias of Eq. 14 against
    oracle.fused_bias (both accumulate in fp64; summation order differs), the prepacked weights equal to the layout
    reference; and the same numbers as the single-purpose helpers."""
    lay = si.make_tiny(8, K, N, seed=N + K)
    w = oracle.bf16_to_f32(si.bf16_bits(lay.W_rot))
    wq = oracle.quantize_weights(w)
    rng = np.random.default_rng(N)
    bc = rng.standard_normal(K).astype(np.float32) if with_bias else None
    lb = rng.standard_normal(N).astype(np.float32) if with_layer_bias else None
    Wq = torch.from_numpy(oracle.pack_codes(wq.codes)).to(DEV)
    w_scale, w_zero = si.bits_to_bf16(wq.scale_bits).to(DEV), si.bits_to_bf16(wq.zero_bits).to(DEV)
    tb = None if bc is None else torch.from_numpy(bc).to(DEV)
    tl = None if lb is None else torch.from_numpy(lb).to(DEV)
    w_sum = torch.full((N,), float("nan"), dtype=torch.float32, device=DEV)
    out_bias = torch.full((N,), float("nan"), dtype=torch.float32, device=DEV)
    W6 = B.alloc_fp6_buffer(N, K, DEV).zero_() if K % 128 == 0 else None
    B.basq_prepare_weights(Wq, w_scale, w_zero, tb, tl, w_sum, out_bias, W6)
    ob2 = torch.empty_like(out_bias)
    B.basq_fused_bias(Wq, w_scale, w_zero, tb, tl, ob2)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(w_sum.cpu().numpy().view(np.uint32), wq.wsum.view(np.uint32), err_msg="w_sum bits")
    ref = oracle.fused_bias(wq, bc, lb)
    np.testing.assert_allclose(out_bias.cpu().numpy(), ref, rtol=1e-6, atol=1e-6)
    assert torch.equal(out_bias, ob2), "basq_prepare_weights and basq_fused_bias disagree"
    if W6 is not None:
        full = (N // 32) * 32                              # bytes of rows past N in the last block are undefined
        got = W6.cpu().numpy().reshape(K // 128, -1, 3072)
        want = layout_ref.pack_fp6(wq.codes).reshape(K // 128, -1, 3072)
        np.testing.assert_array_equal(got[:, :full // 32], want[:, :full // 32], err_msg="prepacked weights")


@pytest.mark.parametrize("M", [524288 + 45, 1048576 + 19])
def test_packed_operands_of_two_to_four_gib_and_beyond(M):
    """The matrix-path kernels address their packed operands with 32-bit unsigned byte offsets, so an operand may be
    up to 4 GiB.  524288 + 45 tokens of K = 8192 (four times the largest batch of Sec. 5.2's prefill table, 131072
    tokens) make the 4-bit activations 2.0 GiB and their fp6 form 3.0 GiB: the rows behind byte 2^31 of either form
    must come out as the oracle computes them -- codes and records bit-exact, accumulators bit-exact on both matrix
    paths, outputs within one bf16 step on identical codes -- and the two paths must agree on every element.
    1048576 + 19 tokens put both forms beyond 4 GiB: the quantiser and the repacking kernel index with 64 bits, and
    the product falls back to the kernel that does too (with or without the fp6 operands); same checks, around byte
    2^32 as well."""
    K, N = 8192, 192
    announce(f"packed operands of {M * (K // 2) / 2 ** 30:.2f} GiB (4-bit) and {M * K * 0.75 / 2 ** 30:.2f} GiB (fp6): M={M} K={K} N={N}")
    gen = torch.Generator(device=DEV).manual_seed(2031)
    X = torch.empty((M, K), dtype=torch.bfloat16, device=DEV)
    for i in range(0, M, 65536):
        n = min(65536, M - i)
        X[i:i + n] = (torch.randn((n, K), generator=gen, device=DEV) * 1.5).to(torch.bfloat16)
    X[:, 7] *= 20.0
    bias = torch.randn(K, generator=gen, device=DEV) * 0.3
    W = (torch.randn((N, K), generator=gen, device=DEV) * 0.02).to(torch.bfloat16)
    Wq, w_scale, w_zero, w_sum = B.alloc_weight_buffers(N, K, DEV)
    B.basq_quantize_weights(W, Wq, w_scale, w_zero, w_sum)
    out_bias = torch.empty(N, dtype=torch.float32, device=DEV)
    B.basq_fused_bias(Wq, w_scale, w_zero, bias, None, out_bias)
    W6 = B.alloc_fp6_buffer(N, K, DEV)
    B.basq_pack_fp6(Wq, W6)

    Aq, meta = B.alloc_activation_buffers(M, K, DEV)
    A6 = B.alloc_fp6_buffer(M, K, DEV)
    assert Aq.numel() > 2 ** 31 and A6.numel() > 2 ** 31 and (Aq.numel() < 2 ** 32) == (M < 1048576)
    clip = 0.9
    B.basq_rotate_quant(X, K, bias, None, clip, clip, Aq, meta, Aq6=A6)
    torch.cuda.synchronize()
    # rows around byte 2^31 of the 4-bit form (row 524288), the first and last rows, and a random sample; the fp6
    # form is laid out chunk by chunk of 128 channels, so every row has codes on both sides of its byte 2^31
    rng = np.random.default_rng(2031)
    cross4 = 2 ** 31 // (K // 2)
    chunk6 = 2 ** 31 // (3072 * ((M + 31) // 32))                 # the 128-channel chunk of the fp6 form that straddles 2^31
    rows = set(range(8)) | set(range(cross4 - 40, min(M, cross4 + 45))) | set(range(M - 45, M))
    if M > 2 * cross4:
        rows |= set(range(2 * cross4 - 40, min(M, 2 * cross4 + 45)))      # byte 2^32
    rows |= set(int(v) for v in rng.choice(M, 64, replace=False))
    rows = np.array(sorted(rows))
    announce(f"  4-bit form crosses 2^31 at row {cross4}; fp6 form inside chunk {chunk6} of {K // 128} "
             f"(every row has codes behind it); {len(rows)} rows sampled")
    ref_q = pu.check_rows_against_oracle(X, rows, K, bias, None, clip, clip, Aq, meta, what="operands beyond 2 GiB")
    check_fp6_copy(Aq, A6, K, row_blocks=[0, cross4 // 32 - 1, cross4 // 32, M // 32 - 1])
    torch.cuda.empty_cache()

    acc8 = torch.full((M, N), -1, dtype=torch.int32, device=DEV)
    Y8 = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
    B.basq_w4a4_gemm(Aq, meta, Wq, w_scale, w_zero, w_sum, out_bias, Y8, acc8)
    acc6 = torch.full((M, N), -1, dtype=torch.int32, device=DEV)
    Y6 = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
    B.basq_w4a4_gemm(Aq, meta, Wq, w_scale, w_zero, w_sum, out_bias, Y6, acc6, Aq6=A6, Wq6=W6)
    torch.cuda.synchronize()
    assert torch.equal(acc6, acc8), "accumulators of the fp6 and int8 paths differ"
    assert torch.equal(Y6.view(torch.int16), Y8.view(torch.int16)), "outputs of the fp6 and int8 paths differ"
    assert not torch.isnan(Y6).any()

    wq_ref = oracle.quantize_weights(oracle.bf16_to_f32(si.bf16_bits(W.cpu())))
    np.testing.assert_array_equal(oracle.unpack_codes(Wq.cpu().numpy()), wq_ref.codes)
    c_ref = oracle.fused_bias(wq_ref, bias.cpu().numpy(), None)
    t_rows = torch.from_numpy(rows).to(DEV)
    acc_ref = oracle.int_gemm_blas(ref_q.codes, wq_ref.codes)
    np.testing.assert_array_equal(acc6[t_rows].cpu().numpy(), acc_ref, err_msg="accumulators behind 2^31")
    y_ref = oracle.dequant(acc_ref, ref_q, wq_ref, c_ref)
    y = oracle.bf16_to_f32(si.bf16_bits(Y6[t_rows].cpu())).astype(np.float64)
    top = float(np.abs(y_ref).max())
    worst = float((np.abs(y - y_ref) - 2.0 ** -8 * np.abs(y_ref)).max() / top)
    assert worst <= 1e-5, f"worst excess over one bf16 step: {worst} of max|ref| on identical codes"
    announce(f"ok worst excess {worst:.2e}")
