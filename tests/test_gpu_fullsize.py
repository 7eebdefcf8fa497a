"""GPU parity at the full benchmark shapes, in the launch configuration bench.py times: the whole
problem runs on the GPU (weights quantised, bias calibrated and fused bias built by the library),
and the oracle recomputes a sample of token rows x output channels one by one from the same
seeded inputs.  Sampled rows and channels always include the first and last tile of each axis."""
import sys

import numpy as np
import pytest
import torch

import oracle
import layout_ref
from paper_2506_15689_amd import binding as B
from paper_2506_15689_amd import synth_inputs as si

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[fullsize] {msg}", flush=True)
    sys.stdout.flush()


def sample_axis(n, count, rng, edge=40):
    idx = set(range(min(edge, n))) | set(range(max(0, n - edge), n))
    idx |= set(int(v) for v in rng.choice(n, size=min(count, n), replace=False))
    return np.array(sorted(idx))


def run_fullsize(name, n_rows, n_cols, M=None):
    dev = torch.device("cuda")
    cfg = si.CONFIGS[name]
    lay = si.make_layer(cfg, M=M)
    M = lay.X.shape[0]
    K, N = cfg.K, cfg.N
    say(f"{name}: M={M} K={K} N={N} rot={cfg.rot_size}")
    rng = np.random.default_rng(cfg.index)
    rows = sample_axis(M, n_rows, rng)
    cols = sample_axis(N, n_cols, rng)

    # ---- oracle side: bias from the calibration tokens, weights of the sampled channels
    xc = oracle.bf16_to_f32(si.bf16_bits(lay.X_calib))
    bc = oracle.channel_bias(xc, cfg.rot_size)
    w_s = oracle.bf16_to_f32(si.bf16_bits(lay.W_rot[torch.from_numpy(cols)]))
    wq_s = oracle.quantize_weights(w_s)
    c_s = oracle.fused_bias(wq_s, bc, None)

    # ---- GPU side: everything, full size
    W = lay.W_rot.to(dev)
    Wq, w_scale, w_zero, w_sum = B.alloc_weight_buffers(N, K, dev)
    B.basq_quantize_weights(W, Wq, w_scale, w_zero, w_sum)
    del W
    Xc = lay.X_calib.to(dev)
    bias_gpu = torch.empty(K, dtype=torch.float32, device=dev)
    ws = torch.empty(Xc.shape[0] * K, dtype=torch.float32, device=dev)
    B.basq_calibrate_bias(Xc, cfg.rot_size, None, bias_gpu, ws)
    torch.cuda.synchronize()
    del ws
    # the library's calibration agrees with the oracle's; the run itself uses the oracle's bits so
    # that the integer comparisons below are exact
    np.testing.assert_allclose(bias_gpu.cpu().numpy(), bc, rtol=1e-4, atol=1e-5 * float(np.abs(bc).max()))
    bias = torch.from_numpy(bc).to(dev)
    out_bias = torch.empty(N, dtype=torch.float32, device=dev)
    B.basq_fused_bias(Wq, w_scale, w_zero, bias, None, out_bias)

    X = lay.X.to(dev)
    Aq, meta = B.alloc_activation_buffers(M, K, dev)
    rot = torch.empty((M, K), dtype=torch.float32, device=dev)
    Y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
    acc = torch.empty((M, N), dtype=torch.int32, device=dev)
    B.basq_rotate_quant(X, cfg.rot_size, bias, None, cfg.clip, cfg.clip, Aq, meta, rot)
    B.basq_w4a4_gemm(Aq, meta, Wq, w_scale, w_zero, w_sum, out_bias, Y, acc)
    # the bench configuration: one fused call, no debug outputs
    Yf = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
    wsf = torch.empty(B.basq_workspace_bytes(M, K, N), dtype=torch.uint8, device=dev)
    B.basq_linear_fused(X, cfg.rot_size, bias, None, cfg.clip, cfg.clip, Wq, w_scale, w_zero, w_sum, out_bias, Yf, wsf)
    torch.cuda.synchronize()
    assert torch.equal(Y, Yf), "fused call differs from the two-call path"

    # ---- the fp6 matrix-core path (what bench.py times for prefill shapes): same bits everywhere
    if M > B.STREAM_MAX_TOKENS:
        Wq6 = B.alloc_fp6_buffer(N, K, dev)
        B.basq_pack_fp6(Wq, Wq6)
        Aq6 = B.alloc_fp6_buffer(M, K, dev)
        Aq2, meta2 = B.alloc_activation_buffers(M, K, dev)
        B.basq_rotate_quant(X, cfg.rot_size, bias, None, cfg.clip, cfg.clip, Aq2, meta2, None, Aq6=Aq6)
        acc6 = torch.empty((M, N), dtype=torch.int32, device=dev)
        Y6 = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
        B.basq_w4a4_gemm(Aq2, meta2, Wq, w_scale, w_zero, w_sum, out_bias, Y6, acc6, Aq6=Aq6, Wq6=Wq6)
        Y6f = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
        B.basq_linear_fused(X, cfg.rot_size, bias, None, cfg.clip, cfg.clip, Wq, w_scale, w_zero, w_sum, out_bias, Y6f, wsf,
                            Wq6=Wq6)
        torch.cuda.synchronize()
        assert torch.equal(Aq2, Aq) and torch.equal(meta2, meta)
        assert torch.equal(acc6, acc), "INT32 accumulators of the fp6 path differ from the int8 path"
        assert torch.equal(Y6, Y) and torch.equal(Y6f, Y), "outputs of the fp6 path differ from the int8 path"
        # both repacked operands against the oracle's encoder, on three 32-row blocks each
        for name6, buf, packed in (("activations", Aq6, Aq), ("weights", Wq6, Wq)):
            R = packed.shape[0]
            RB = (R + 31) // 32
            got = buf.view(K // 128, RB, 3072)
            for rb in sorted({0, RB // 2, R // 32 - 1}):
                codes_rb = oracle.unpack_codes(packed[32 * rb:32 * rb + 32].cpu().numpy())
                ref6 = layout_ref.pack_fp6(codes_rb).reshape(K // 128, 3072)
                np.testing.assert_array_equal(got[:, rb].cpu().numpy(), ref6, err_msg=f"fp6 form of the {name6}, block {rb}")
        del Wq6, Aq6, Aq2, meta2, acc6, Y6, Y6f

    # ---- decode-sized calls (the first 16 and the first 100 tokens) on the whole weight matrix in the streaming
    # layout: the bits of the canonical-layout call, which in turn equal the rows of the full product checked below
    for m16 in ((16, 100) if K % 128 == 0 else ()):
        Wd = torch.empty(B.basq_decode_bytes(N, K), dtype=torch.uint8, device=dev)
        B.basq_pack_decode(Wq, Wd)
        m16 = min(M, m16)
        accc = torch.empty((m16, N), dtype=torch.int32, device=dev)
        accd = torch.empty((m16, N), dtype=torch.int32, device=dev)
        Yc = torch.empty((m16, N), dtype=torch.bfloat16, device=dev)
        Yd = torch.empty((m16, N), dtype=torch.bfloat16, device=dev)
        B.basq_w4a4_gemm(Aq[:m16], meta[:m16], Wq, w_scale, w_zero, w_sum, out_bias, Yc, accc)
        B.basq_w4a4_gemm(Aq[:m16], meta[:m16], Wd, w_scale, w_zero, w_sum, out_bias, Yd, accd,
                         w_layout=B.BASQ_W_DECODE16, N=N)
        torch.cuda.synchronize()
        assert torch.equal(accc, acc[:m16]), "decode path differs from the prefill path on the same tokens"
        assert torch.equal(accd, accc) and torch.equal(Yd, Yc), "streaming layout differs from canonical"
        KB, NB = K // 2, (N + 15) // 16
        for nb in sorted({0, NB // 2, NB - 1}):
            refd = layout_ref.pack_decode16(Wq[16 * nb:16 * nb + 16].cpu().numpy())
            np.testing.assert_array_equal(Wd[nb * 16 * KB:(nb + 1) * 16 * KB].cpu().numpy(), refd,
                                          err_msg=f"streaming layout, block {nb}")
        del Wd, accc, accd, Yc, Yd

    t_rows = torch.from_numpy(rows).to(dev)
    t_cols = torch.from_numpy(cols).to(dev)
    # weights of the sampled channels: bit-exact
    np.testing.assert_array_equal(oracle.unpack_codes(Wq[t_cols].cpu().numpy()), wq_s.codes)
    np.testing.assert_array_equal(si.bf16_bits(w_scale[t_cols].cpu()), wq_s.scale_bits)
    np.testing.assert_array_equal(si.bf16_bits(w_zero[t_cols].cpu()), wq_s.zero_bits)
    np.testing.assert_array_equal(w_sum[t_cols].cpu().numpy().view(np.uint32), wq_s.wsum.view(np.uint32))
    np.testing.assert_allclose(out_bias[t_cols].cpu().numpy(), c_s, rtol=1e-5, atol=1e-6)

    # ---- level (i): oracle on the GPU's rotation output, sampled rows
    x_s = oracle.bf16_to_f32(si.bf16_bits(lay.X[torch.from_numpy(rows)]))
    r_gpu = rot[t_rows].cpu().numpy()
    ref_i = oracle.linear(x_s, cfg.rot_size, bc, None, cfg.clip, cfg.clip, wq_s, c_s, r=r_gpu, use_blas_gemm=True)
    codes = oracle.unpack_codes(Aq[t_rows].cpu().numpy())
    mh = meta[t_rows].cpu().numpy()
    np.testing.assert_array_equal(codes, ref_i.tq.codes)
    np.testing.assert_array_equal(mh[:, 0].copy().view(np.uint32), ref_i.tq.scale[:, 0].view(np.uint32))
    np.testing.assert_array_equal(mh[:, 1].copy().view(np.uint32), ref_i.tq.lo[:, 0].view(np.uint32))
    np.testing.assert_array_equal(mh[:, 2], ref_i.tq.rowsum[:, 0])
    acc_s = acc[t_rows][:, t_cols].cpu().numpy()
    np.testing.assert_array_equal(acc_s, ref_i.acc)

    # ---- levels (ii), (iii): oracle from X
    ref = oracle.linear(x_s, cfg.rot_size, bc, None, cfg.clip, cfg.clip, wq_s, c_s, use_blas_gemm=True)
    d = codes.astype(np.int32) - ref.tq.codes.astype(np.int32)
    flips = d != 0
    assert flips.mean() <= 1e-4, f"flip rate {flips.mean()}"
    assert (np.abs(d[flips]) == 1).all()
    y = oracle.bf16_to_f32(si.bf16_bits(Y[t_rows][:, t_cols].cpu())).astype(np.float64)
    err = np.abs(y - ref.y).max() / np.abs(ref.y).max()
    assert err <= 2e-2, f"output error {err}"

    # ---- properties that hold on ALL rows: code range, row sums, accumulator bounds
    rs = meta[:, 2].to(torch.int64)
    lo_nib = (Aq & 0x0F).to(torch.int64).sum(dim=1)
    hi_nib = (Aq >> 4).to(torch.int64).sum(dim=1)
    assert torch.equal(rs, lo_nib + hi_nib), "row sums inconsistent with the packed codes"
    assert int(acc.min()) >= 0 and int(acc.max()) <= 225 * K
    say(f"{name}: ok  rows={len(rows)} cols={len(cols)} flip_rate={flips.mean():.2e} y_err={err:.2e}")


def test_c2_fullsize():
    run_fullsize("C2", n_rows=256, n_cols=1024)


def test_c4_fullsize_kronecker():
    run_fullsize("C4", n_rows=96, n_cols=512)


def test_c5_fullsize():
    run_fullsize("C5", n_rows=96, n_cols=768)
