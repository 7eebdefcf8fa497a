"""Shared plumbing of the GPU parity tests: builds one case (oracle-side numpy arrays and the
device tensors made from the SAME bits), runs the HIP path through the binding, and compares
at the three levels the acceptance criteria name:

  (i)   the GPU's fp32 rotation output is fed to the oracle's quantiser and integer GEMM:
        codes, token records and INT32 accumulators must match bit for bit;
  (ii)  the oracle's whole path from X: bf16 outputs within 2e-2 of max|ref|;
  (iii) codes from the oracle's own (fp64) rotation vs the GPU's: at most 1e-4 of them differ,
        each by one code (fp32 summation order in the rotation is the only source).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

import oracle
import layout_ref
from paper_2506_15689_amd import binding as B
from paper_2506_15689_amd import synth_inputs as si

Y_TOL = 2e-2
FLIP_TOL = 1e-4


@dataclass
class Case:
    M: int
    K: int
    N: int
    rot_size: int
    clip_lo: float
    clip_hi: float
    x: np.ndarray                 # fp32 [M, K] (exact bf16 values)
    bias: Optional[np.ndarray]    # fp32 [K]
    act_scale: Optional[np.ndarray]
    wq: oracle.WeightQuant
    c: Optional[np.ndarray]       # fp32 [N]
    X_t: torch.Tensor             # bf16 CPU tensor


def make_case(lay: si.LayerInputs, *, rot_size: Optional[int] = None, clip_lo: Optional[float] = None,
              clip_hi: Optional[float] = None, act_scale: Optional[np.ndarray] = None, use_bias: bool = True,
              use_out_bias: bool = True) -> Case:
    cfg = lay.cfg
    M, K = lay.X.shape
    N = lay.W_rot.shape[0]
    n = cfg.rot_size if rot_size is None else rot_size
    x = oracle.bf16_to_f32(si.bf16_bits(lay.X))
    w = oracle.bf16_to_f32(si.bf16_bits(lay.W_rot))
    bias = None
    if use_bias:
        xc = oracle.bf16_to_f32(si.bf16_bits(lay.X_calib))
        bias = oracle.channel_bias(xc, n)
        if act_scale is not None:
            bias = (bias.astype(np.float64) * act_scale.astype(np.float64)).astype(np.float32)
    wq = oracle.quantize_weights(w)
    c = None
    if use_out_bias:
        lb = None if lay.layer_bias is None else lay.layer_bias.numpy()
        c = oracle.fused_bias(wq, bias, lb)
    return Case(M, K, N, n, cfg.clip if clip_lo is None else clip_lo, cfg.clip if clip_hi is None else clip_hi,
                x, bias, act_scale, wq, c, lay.X)


@dataclass
class DeviceCase:
    X: torch.Tensor
    bias: Optional[torch.Tensor]
    act_scale: Optional[torch.Tensor]
    Wq: torch.Tensor
    w_scale: torch.Tensor
    w_zero: torch.Tensor
    w_sum: torch.Tensor
    out_bias: Optional[torch.Tensor]


def to_device(case: Case, dev="cuda") -> DeviceCase:
    f = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    return DeviceCase(case.X_t.to(dev), f(case.bias), f(case.act_scale), f(oracle.pack_codes(case.wq.codes)),
                      si.bits_to_bf16(case.wq.scale_bits).to(dev), si.bits_to_bf16(case.wq.zero_bits).to(dev),
                      f(case.wq.wsum), f(case.c))


@dataclass
class GpuResult:
    rot: np.ndarray        # fp32 [M, K]
    codes: np.ndarray      # uint8 [M, K]
    scale: np.ndarray      # fp32 [M]
    lo: np.ndarray         # fp32 [M]
    rowsum: np.ndarray     # int32 [M]
    acc: np.ndarray        # int32 [M, N]
    y_bits: np.ndarray     # uint16 [M, N]
    y_fused_bits: np.ndarray
    # the same layer on the fp6 matrix-core path (None when K % 128 != 0)
    a6: Optional[np.ndarray] = None          # fp6 operand form of the activation codes, as written by rotate_quant
    w6: Optional[np.ndarray] = None          # ... of the weight codes, as written by pack_fp6
    acc6: Optional[np.ndarray] = None
    y6_bits: Optional[np.ndarray] = None
    y6_fused_bits: Optional[np.ndarray] = None
    # the same layer with the weights in the weight-streaming layout (None when K % 128 != 0)
    wd: Optional[np.ndarray] = None          # the layout as written by pack_decode
    accd: Optional[np.ndarray] = None        # decode-sized M only: the int32 accumulators of that path
    yd_bits: Optional[np.ndarray] = None
    yd_fused_bits: Optional[np.ndarray] = None


def run_gpu(case: Case, d: DeviceCase) -> GpuResult:
    dev = d.X.device
    M, K, N = case.M, case.K, case.N
    Aq, meta = B.alloc_activation_buffers(M, K, dev)
    rot = torch.empty((M, K), dtype=torch.float32, device=dev)
    Y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=dev)
    Yf = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=dev)
    acc = torch.full((M, N), -1, dtype=torch.int32, device=dev)
    ws = torch.empty(max(B.basq_workspace_bytes(M, K, N), 256), dtype=torch.uint8, device=dev)
    B.basq_rotate_quant(d.X, case.rot_size, d.bias, d.act_scale, case.clip_lo, case.clip_hi, Aq, meta, rot)
    B.basq_w4a4_gemm(Aq, meta, d.Wq, d.w_scale, d.w_zero, d.w_sum, d.out_bias, Y, acc)
    B.basq_linear_fused(d.X, case.rot_size, d.bias, d.act_scale, case.clip_lo, case.clip_hi, d.Wq, d.w_scale,
                        d.w_zero, d.w_sum, d.out_bias, Yf, ws)
    torch.cuda.synchronize()
    meta_h = meta.cpu().numpy()
    res = GpuResult(rot.cpu().numpy(), oracle.unpack_codes(Aq.cpu().numpy()),
                    meta_h[:, 0].copy().view(np.float32), meta_h[:, 1].copy().view(np.float32),
                    meta_h[:, 2].copy(), acc.cpu().numpy(), si.bf16_bits(Y.cpu()), si.bf16_bits(Yf.cpu()))
    if K % 128 == 0 and M > 0:
        # second pass with the fp6 operands: activations straight from rotate_quant, weights repacked
        Aq2, meta2 = B.alloc_activation_buffers(M, K, dev)
        A6 = B.alloc_fp6_buffer(M, K, dev).zero_()
        W6 = B.alloc_fp6_buffer(N, K, dev).zero_()
        Y6 = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=dev)
        Y6f = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=dev)
        acc6 = torch.full((M, N), -1, dtype=torch.int32, device=dev)
        B.basq_pack_fp6(d.Wq, W6)
        B.basq_rotate_quant(d.X, case.rot_size, d.bias, d.act_scale, case.clip_lo, case.clip_hi, Aq2, meta2, None, Aq6=A6)
        B.basq_w4a4_gemm(Aq2, meta2, d.Wq, d.w_scale, d.w_zero, d.w_sum, d.out_bias, Y6, acc6, Aq6=A6, Wq6=W6)
        B.basq_linear_fused(d.X, case.rot_size, d.bias, d.act_scale, case.clip_lo, case.clip_hi, d.Wq, d.w_scale,
                            d.w_zero, d.w_sum, d.out_bias, Y6f, ws, Wq6=W6)
        torch.cuda.synchronize()
        assert torch.equal(Aq2, Aq) and torch.equal(meta2, meta), "rotate_quant with and without the fp6 output"
        res.a6, res.w6 = A6.cpu().numpy(), W6.cpu().numpy()
        res.acc6, res.y6_bits, res.y6_fused_bits = acc6.cpu().numpy(), si.bf16_bits(Y6.cpu()), si.bf16_bits(Y6f.cpu())
        # third pass: weights in the streaming layout (read by the weight-streaming kernel; larger M runs on the fp6
        # operands and must not touch Wq at all)
        Wd = torch.empty(B.basq_decode_bytes(N, K), dtype=torch.uint8, device=dev).fill_(0xEE)
        B.basq_pack_decode(d.Wq, Wd)
        Yd = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=dev)
        Ydf = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=dev)
        accd = torch.full((M, N), -1, dtype=torch.int32, device=dev)
        fp6 = dict(Aq6=A6, Wq6=W6) if M > B.STREAM_MAX_TOKENS else {}
        B.basq_w4a4_gemm(Aq, meta, Wd, d.w_scale, d.w_zero, d.w_sum, d.out_bias, Yd, accd,
                         w_layout=B.BASQ_W_DECODE16, N=N, **fp6)
        B.basq_linear_fused(d.X, case.rot_size, d.bias, d.act_scale, case.clip_lo, case.clip_hi, Wd, d.w_scale,
                            d.w_zero, d.w_sum, d.out_bias, Ydf, ws, w_layout=B.BASQ_W_DECODE16, N=N,
                            Wq6=W6 if M > B.STREAM_MAX_TOKENS else None)
        torch.cuda.synchronize()
        res.wd, res.accd = Wd.cpu().numpy(), accd.cpu().numpy()
        res.yd_bits, res.yd_fused_bits = si.bf16_bits(Yd.cpu()), si.bf16_bits(Ydf.cpu())
    return res


def check_fp6_path(case: Case, g: GpuResult, *, row_blocks: Optional[np.ndarray] = None) -> None:
    """The fp6 matrix-core path must give the bits of the int8 path (which check_parity ties to the
    oracle), and both repacked operands must be the oracle's encoding of the same codes.
    ``row_blocks``: compare only these 32-row blocks of the operands (full-size cases)."""
    if g.a6 is None:
        return
    np.testing.assert_array_equal(g.acc6, g.acc, err_msg="INT32 accumulators, fp6 path vs int8 path")
    np.testing.assert_array_equal(g.y6_bits, g.y_bits, err_msg="outputs, fp6 path vs int8 path")
    np.testing.assert_array_equal(g.y6_fused_bits, g.y_bits, err_msg="basq_linear_fused on the fp6 path")
    for name, buf, codes in (("activations", g.a6, g.codes), ("weights", g.w6, case.wq.codes)):
        R, K = codes.shape
        RB = (R + 31) // 32
        if row_blocks is not None:
            blocks = np.asarray([b for b in row_blocks if b < RB])
        elif R * K <= (1 << 20):
            blocks = np.arange(RB)
        else:                                       # the encoder here is a Python loop: first, middle and last block
            blocks = np.unique([0, RB // 2, RB - 1])
        got = buf.reshape(K // 128, RB, 3072)
        for rb in blocks:
            rows = codes[32 * rb:32 * rb + 32]
            ref = layout_ref.pack_fp6(np.ascontiguousarray(rows)).reshape(K // 128, 1, 3072)[:, 0]
            n = rows.shape[0]
            if n == 32:
                np.testing.assert_array_equal(got[:, rb], ref, err_msg=f"fp6 form of the {name}, row block {rb}")
            else:                                   # ragged last block: only the bytes of real rows are defined
                mask = layout_ref.pack_fp6(np.full((n, K), 15, dtype=np.uint8)).reshape(K // 128, 3072) != 0
                mask |= layout_ref.pack_fp6(np.full((n, K), 1, dtype=np.uint8)).reshape(K // 128, 3072) != 0
                np.testing.assert_array_equal(got[:, rb][mask], ref[mask], err_msg=f"fp6 form of the {name}, last block")


def check_decode_layout(case: Case, g: GpuResult) -> None:
    """Weights in the streaming layout: the buffer is the oracle's permutation of the canonical bytes, and
    the layer gives the bits of the canonical-layout run (which check_parity ties to the oracle)."""
    if g.wd is None:
        return
    N, K = case.wq.codes.shape
    KB = K // 2
    NB = (N + 15) // 16
    blocks = np.arange(NB) if N * K <= (1 << 22) else np.unique([0, NB // 2, NB - 1])
    canon = oracle.pack_codes(case.wq.codes)
    for nb in blocks:                               # the layout is independent per 16-row block
        ref = layout_ref.pack_decode16(np.ascontiguousarray(canon[16 * nb:16 * nb + 16]))
        np.testing.assert_array_equal(g.wd[nb * 16 * KB:(nb + 1) * 16 * KB], ref, err_msg=f"streaming layout, block {nb}")
    np.testing.assert_array_equal(g.accd, g.acc, err_msg="INT32 accumulators, streaming layout vs canonical")
    np.testing.assert_array_equal(g.yd_bits, g.y_bits, err_msg="outputs, streaming layout vs canonical")
    np.testing.assert_array_equal(g.yd_fused_bits, g.y_bits, err_msg="basq_linear_fused, streaming layout")


def check_parity(case: Case, g: GpuResult, *, rows: Optional[np.ndarray] = None, use_blas_gemm: bool = False,
                 y_tol: float = Y_TOL, flip_tol: float = FLIP_TOL) -> dict:
    """Compare the GPU result with the oracle.  ``rows``: check only these token rows (full-size
    cases where the oracle would take too long on everything); the GPU still ran all rows."""
    sel = np.arange(case.M) if rows is None else np.asarray(rows)
    x = case.x[sel]
    # level (i): oracle on the GPU's rotation output
    ref_i = oracle.linear(x, case.rot_size, case.bias, case.act_scale, case.clip_lo, case.clip_hi, case.wq,
                          case.c, r=g.rot[sel], use_blas_gemm=use_blas_gemm)
    np.testing.assert_array_equal(g.codes[sel], ref_i.tq.codes, err_msg="activation codes (level i)")
    np.testing.assert_array_equal(g.scale[sel].view(np.uint32), ref_i.tq.scale[:, 0].view(np.uint32), err_msg="scale bits")
    np.testing.assert_array_equal(g.lo[sel].view(np.uint32), ref_i.tq.lo[:, 0].view(np.uint32), err_msg="lo bits")
    np.testing.assert_array_equal(g.rowsum[sel], ref_i.tq.rowsum[:, 0], err_msg="row sums")
    np.testing.assert_array_equal(g.acc[sel], ref_i.acc, err_msg="INT32 accumulators (level i)")
    # the one-call entry point runs the same kernels: identical bits
    np.testing.assert_array_equal(g.y_fused_bits, g.y_bits, err_msg="basq_linear_fused vs two calls")

    # levels (ii) and (iii): oracle from X with its own rotation
    ref = oracle.linear(x, case.rot_size, case.bias, case.act_scale, case.clip_lo, case.clip_hi, case.wq, case.c,
                        use_blas_gemm=use_blas_gemm)
    rot_err = float(np.abs(g.rot[sel].astype(np.float64) - ref.r.astype(np.float64)).max())
    rot_scale = float(np.abs(ref.r).max())
    assert rot_err <= 2e-5 * max(rot_scale, 1.0), f"rotation error {rot_err} (max |r| {rot_scale})"
    d = g.codes[sel].astype(np.int32) - ref.tq.codes.astype(np.int32)
    flips = d != 0
    flip_rate = float(flips.mean()) if flips.size else 0.0
    assert flip_rate <= flip_tol, f"code flip rate {flip_rate}"
    assert (np.abs(d[flips]) == 1).all(), "a code differs by more than one step"
    y = oracle.bf16_to_f32(g.y_bits[sel]).astype(np.float64)
    denom = float(np.abs(ref.y).max()) if ref.y.size else 1.0
    y_err = float(np.abs(y - ref.y).max() / denom) if ref.y.size else 0.0
    assert y_err <= y_tol, f"output error {y_err} of max|ref|"
    # and against the level-(i) reference the output differs only by fp32 epilogue rounding + bf16
    y_i = float(np.abs(y - ref_i.y).max() / denom) if ref.y.size else 0.0
    assert y_i <= 2 ** -7, f"epilogue error {y_i} of max|ref| on identical accumulators"
    return {"flip_rate": flip_rate, "y_err": y_err, "y_err_same_acc": y_i, "rot_err": rot_err}


def check_rows_against_oracle(X, rows, rot, bias, sa, clip_lo, clip_hi, Aq, meta, *, group=0, what=""):
    """The rows `rows` of a finished basq_rotate_quant call (codes Aq, records meta) against the oracle's quantiser
    on the GPU's own rotation of those rows."""
    M, K = X.shape
    G = K if group in (0, K) else group
    ng = K // G
    t_rows = torch.from_numpy(rows).to(X.device)
    Xs = X[t_rows].contiguous()
    r = torch.empty((len(rows), K), dtype=torch.float32, device=X.device)
    Aq_s = torch.empty((len(rows), K // 2), dtype=torch.uint8, device=X.device)
    meta_s = torch.empty((len(rows) * ng, 4), dtype=torch.int32, device=X.device)
    B.basq_rotate_quant(Xs, rot, bias, sa, clip_lo, clip_hi, Aq_s, meta_s, r, group_size=group)
    torch.cuda.synchronize()
    ref = oracle.quantize_tokens(r.cpu().numpy(), None if bias is None else bias.cpu().numpy(),
                                 None if sa is None else sa.cpu().numpy(), clip_lo, clip_hi, group_size=group)
    codes = oracle.unpack_codes(Aq[t_rows].cpu().numpy())
    mh = meta.view(M, ng, 4)[t_rows].cpu().numpy()
    bad = np.flatnonzero((codes != ref.codes).any(axis=1))
    assert bad.size == 0, f"{what}: codes differ from the oracle in rows {rows[bad][:8]}"
    for name, col, want in (("scale", 0, ref.scale.view(np.uint32)), ("lower bound", 1, ref.lo.view(np.uint32)),
                            ("row sum", 2, ref.rowsum.view(np.uint32))):
        got = mh[:, :, col].copy().view(np.uint32)
        bad = np.flatnonzero((got != want).any(axis=1))
        assert bad.size == 0, (f"{what}: {name} bits differ from the oracle in rows {rows[bad][:8]}: "
                               f"{got[bad[0]][:4]} vs {want[bad[0]][:4]}")
    return ref
