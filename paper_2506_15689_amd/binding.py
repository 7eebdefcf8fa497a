"""Thin ctypes binding of libbasq.so: same names as the C ABI (include/basq.h), torch tensors in,
argument marshalling only.  Every step of the layer runs in the HIP kernels; there is no CPU
fallback -- if the library is missing or a call fails, an exception is raised."""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libbasq.so")

BASQ_OK = 0
BASQ_EINVAL = -1
BASQ_EUNSUPPORTED = -2
BASQ_EWORKSPACE = -3
BASQ_EHIP = -4
BASQ_W_CANONICAL = 0
BASQ_W_DECODE16 = 1
STREAM_MAX_TOKENS = 128      # calls of at most this many tokens take the weight-streaming kernel (K % 128 == 0)

EXPORTS = ["basq_version", "basq_last_error", "basq_rotate_quant", "basq_w4a4_gemm", "basq_workspace_bytes",
           "basq_w4a4_gemm_grouped", "basq_group_colsums", "basq_fp6_bytes", "basq_pack_fp6", "basq_decode_bytes", "basq_pack_decode", "basq_linear_fused", "basq_linear_fused_static", "basq_rotate_weights", "basq_quantize_weights", "basq_fused_bias", "basq_prepare_weights", "basq_calibrate_bias",
           "basq_hadamard28", "basq_diag_stream", "basq_diag_read", "basq_diag_mfma_i8", "basq_diag_mfma_f6"]


class BasqError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"libbasq error {code}: {text}")
        self.code = code


_lib: Optional[ctypes.CDLL] = None


def load() -> ctypes.CDLL:
    """Load libbasq.so (built in-tree by paper_2506_15689_amd.build.build_lib)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2506_15689_amd.build` "
                          "(or __graft_entry__.build()); there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    c = ctypes
    vp, i64, i32, f32 = c.c_void_p, c.c_int64, c.c_int32, c.c_float
    lib.basq_version.restype = c.c_int
    lib.basq_version.argtypes = []
    lib.basq_last_error.restype = c.c_char_p
    lib.basq_last_error.argtypes = []
    lib.basq_rotate_quant.restype = c.c_int
    lib.basq_rotate_quant.argtypes = [vp, i64, i32, i64, i32, vp, vp, f32, f32, i32, i32, vp, vp, vp, vp, vp]
    lib.basq_w4a4_gemm.restype = c.c_int
    lib.basq_w4a4_gemm.argtypes = [vp, vp, i64, i32, vp, i32, i32, vp, vp, vp, vp, vp, i64, vp, vp, vp, vp]
    lib.basq_w4a4_gemm_grouped.restype = c.c_int
    lib.basq_w4a4_gemm_grouped.argtypes = [vp, vp, i64, i32, i32, vp, i32, vp, vp, vp, vp, vp, i64, vp, vp, vp]
    lib.basq_group_colsums.restype = c.c_int
    lib.basq_group_colsums.argtypes = [vp, i32, i32, i32, vp, vp]
    lib.basq_fp6_bytes.restype = c.c_size_t
    lib.basq_fp6_bytes.argtypes = [i64, i32]
    lib.basq_pack_fp6.restype = c.c_int
    lib.basq_pack_fp6.argtypes = [vp, i64, i32, vp, vp]
    lib.basq_decode_bytes.restype = c.c_size_t
    lib.basq_decode_bytes.argtypes = [i32, i32]
    lib.basq_pack_decode.restype = c.c_int
    lib.basq_pack_decode.argtypes = [vp, i32, i32, vp, vp]
    lib.basq_workspace_bytes.restype = c.c_size_t
    lib.basq_workspace_bytes.argtypes = [i64, i32, i32]
    lib.basq_linear_fused.restype = c.c_int
    lib.basq_linear_fused.argtypes = [vp, i64, i32, i64, i32, vp, vp, f32, f32, i32, i32,
                                      vp, i32, i32, vp, vp, vp, vp, vp, i64, vp, vp, c.c_size_t, vp]
    lib.basq_linear_fused_static.restype = c.c_int
    lib.basq_linear_fused_static.argtypes = [vp, i64, i32, i64, i32, vp, vp, f32, f32, i32, i32,
                                             vp, i32, i32, vp, vp, vp, vp, vp, i64, vp, vp]
    lib.basq_rotate_weights.restype = c.c_int
    lib.basq_rotate_weights.argtypes = [vp, i32, i32, i64, i32, vp, vp, c.c_size_t, vp]
    lib.basq_quantize_weights.restype = c.c_int
    lib.basq_quantize_weights.argtypes = [vp, i32, i32, i64, vp, vp, vp, vp, vp]
    lib.basq_fused_bias.restype = c.c_int
    lib.basq_fused_bias.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, vp]
    lib.basq_prepare_weights.restype = c.c_int
    lib.basq_prepare_weights.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.basq_calibrate_bias.restype = c.c_int
    lib.basq_calibrate_bias.argtypes = [vp, i64, i32, i64, i32, vp, vp, vp, c.c_size_t, vp]
    lib.basq_hadamard28.restype = c.c_int
    lib.basq_hadamard28.argtypes = [vp]
    lib.basq_diag_stream.restype = c.c_int
    lib.basq_diag_stream.argtypes = [vp, vp, vp, i64, i32, vp]
    lib.basq_diag_read.restype = c.c_int
    lib.basq_diag_read.argtypes = [vp, i64, vp, i32, vp]
    lib.basq_diag_mfma_i8.restype = c.c_int
    lib.basq_diag_mfma_i8.argtypes = [vp, i32, i32, vp]
    lib.basq_diag_mfma_f6.restype = c.c_int
    lib.basq_diag_mfma_f6.argtypes = [vp, i32, i32, vp]
    _lib = lib
    return lib


def _p(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream: Optional[torch.cuda.Stream]):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _check(rc: int) -> None:
    if rc != BASQ_OK:
        raise BasqError(rc, load().basq_last_error().decode("utf-8", "replace"))


def _need(t: Optional[torch.Tensor], nbytes: int, name: str) -> None:
    """Raw pointers carry no size: refuse a tensor smaller than what the kernels will touch."""
    if t is not None and t.numel() * t.element_size() < nbytes:
        raise ValueError(f"{name} holds {t.numel() * t.element_size()} bytes, the call needs {nbytes}")


def basq_version() -> int:
    return int(load().basq_version())


def basq_last_error() -> str:
    return load().basq_last_error().decode("utf-8", "replace")


def basq_hadamard28() -> torch.Tensor:
    out = torch.empty(28 * 28, dtype=torch.int8)
    _check(load().basq_hadamard28(ctypes.c_void_p(out.data_ptr())))
    return out.view(28, 28)


def basq_workspace_bytes(M: int, K: int, N: int) -> int:
    return int(load().basq_workspace_bytes(M, K, N))


def basq_rotate_quant(X: torch.Tensor, rot_size: int, bias: Optional[torch.Tensor], act_scale: Optional[torch.Tensor],
                      clip_lo: float, clip_hi: float, Aq: torch.Tensor, meta: torch.Tensor,
                      rot_out: Optional[torch.Tensor] = None, *, Aq6: Optional[torch.Tensor] = None, bits: int = 4,
                      group_size: int = 0, stream: Optional[torch.cuda.Stream] = None) -> None:
    """X bf16 [M, K] (row stride X.stride(0)); Aq uint8 [M, K/2]; meta int32 [M * K/group_size, 4] (16-byte records,
    one per token when group_size is 0 or K); Aq6 uint8 [basq_fp6_bytes(M, K)] = whole blocks of 32 rows (optional
    fp6 operand form of the codes, see alloc_fp6_buffer); rot_out fp32 [M, K]."""
    M, K = X.shape
    groups = 1 if group_size in (0, K) or group_size <= 0 else K // group_size
    _need(Aq, M * (K // 2), "Aq")
    _need(meta, 16 * M * groups, "meta")
    _need(rot_out, 4 * M * K, "rot_out")
    _need(Aq6, basq_fp6_bytes(M, K), "Aq6")
    _check(load().basq_rotate_quant(_p(X), M, K, X.stride(0) if M > 0 else K, rot_size, _p(bias), _p(act_scale),
                                    clip_lo, clip_hi, bits, group_size, _p(Aq), _p(meta), _p(rot_out), _p(Aq6),
                                    _stream(stream)))


def basq_w4a4_gemm(Aq: torch.Tensor, meta: torch.Tensor, Wq: torch.Tensor, w_scale: torch.Tensor,
                   w_zero: torch.Tensor, w_sum: torch.Tensor, out_bias: Optional[torch.Tensor], Y: torch.Tensor,
                   acc_out: Optional[torch.Tensor] = None, *, Aq6: Optional[torch.Tensor] = None,
                   Wq6: Optional[torch.Tensor] = None,
                   w_layout: int = BASQ_W_CANONICAL, N: Optional[int] = None,
                   stream: Optional[torch.cuda.Stream] = None) -> None:
    """N defaults to Wq.shape[0]; give it when Wq is a flat buffer in the streaming layout.  Aq6 / Wq6: uint8
    [basq_fp6_bytes(M, K)] / [basq_fp6_bytes(N, K)]."""
    M, KB = Aq.shape
    N = Wq.shape[0] if N is None else N
    _need(meta, 16 * M, "meta")
    _need(Wq, basq_decode_bytes(N, KB * 2) if w_layout == BASQ_W_DECODE16 else N * KB, "Wq")
    _need(Aq6, basq_fp6_bytes(M, KB * 2), "Aq6")
    _need(Wq6, basq_fp6_bytes(N, KB * 2), "Wq6")
    _need(acc_out, 4 * M * N, "acc_out")
    _check(load().basq_w4a4_gemm(_p(Aq), _p(meta), M, KB * 2, _p(Wq), N, w_layout, _p(w_scale), _p(w_zero),
                                 _p(w_sum), _p(out_bias), _p(Y), Y.stride(0) if M > 0 else N, _p(acc_out),
                                 _p(Aq6), _p(Wq6), _stream(stream)))


def basq_w4a4_gemm_grouped(Aq: torch.Tensor, meta: torch.Tensor, group_size: int, Wq: torch.Tensor, w_scale: torch.Tensor,
                           w_zero: torch.Tensor, w_gsum: torch.Tensor, out_bias: Optional[torch.Tensor], Y: torch.Tensor,
                           *, Aq6: Optional[torch.Tensor] = None, Wq6: Optional[torch.Tensor] = None,
                           stream: Optional[torch.cuda.Stream] = None) -> None:
    """Aq uint8 [M, K/2]; meta int32 [M*K/group_size, 4]; w_gsum int32 [K/group_size, N]; Aq6/Wq6: the fp6 operand
    forms (both or neither)."""
    M, KB = Aq.shape
    N = Wq.shape[0]
    if group_size > 0:
        _need(meta, 16 * M * (KB * 2 // group_size), "meta")
        _need(w_gsum, 4 * N * (KB * 2 // group_size), "w_gsum")
    _need(Aq6, basq_fp6_bytes(M, KB * 2), "Aq6")
    _need(Wq6, basq_fp6_bytes(N, KB * 2), "Wq6")
    _check(load().basq_w4a4_gemm_grouped(_p(Aq), _p(meta), M, KB * 2, group_size, _p(Wq), N, _p(w_scale), _p(w_zero),
                                         _p(w_gsum), _p(out_bias), _p(Y), Y.stride(0) if M > 0 else N,
                                         _p(Aq6), _p(Wq6), _stream(stream)))


def basq_group_colsums(Wq: torch.Tensor, group_size: int, w_gsum: torch.Tensor, *,
                       stream: Optional[torch.cuda.Stream] = None) -> None:
    N, KB = Wq.shape
    _check(load().basq_group_colsums(_p(Wq), N, KB * 2, group_size, _p(w_gsum), _stream(stream)))


def basq_fp6_bytes(rows: int, K: int) -> int:
    return int(load().basq_fp6_bytes(rows, K))


def basq_pack_fp6(codes: torch.Tensor, out6: torch.Tensor, *, stream: Optional[torch.cuda.Stream] = None) -> None:
    """codes uint8 [rows, K/2] -> out6 uint8 [basq_fp6_bytes(rows, K)] (fp6 operand form)."""
    rows, KB = codes.shape
    _check(load().basq_pack_fp6(_p(codes), rows, KB * 2, _p(out6), _stream(stream)))


def basq_decode_bytes(N: int, K: int) -> int:
    return int(load().basq_decode_bytes(N, K))


def basq_pack_decode(Wq: torch.Tensor, out: torch.Tensor, *, stream: Optional[torch.cuda.Stream] = None) -> None:
    """Wq uint8 [N, K/2] canonical -> out uint8 [basq_decode_bytes(N, K)] (weight-streaming layout)."""
    N, KB = Wq.shape
    _check(load().basq_pack_decode(_p(Wq), N, KB * 2, _p(out), _stream(stream)))


def basq_linear_fused(X: torch.Tensor, rot_size: int, bias: Optional[torch.Tensor],
                      act_scale: Optional[torch.Tensor], clip_lo: float, clip_hi: float, Wq: torch.Tensor,
                      w_scale: torch.Tensor, w_zero: torch.Tensor, w_sum: torch.Tensor,
                      out_bias: Optional[torch.Tensor], Y: torch.Tensor, workspace: torch.Tensor, *,
                      Wq6: Optional[torch.Tensor] = None,
                      bits: int = 4, group_size: int = 0, w_layout: int = BASQ_W_CANONICAL,
                      N: Optional[int] = None, stream: Optional[torch.cuda.Stream] = None) -> None:
    M, K = X.shape
    N = Wq.shape[0] if N is None else N
    _need(Wq6, basq_fp6_bytes(N, K), "Wq6")
    _check(load().basq_linear_fused(_p(X), M, K, X.stride(0) if M > 0 else K, rot_size, _p(bias), _p(act_scale),
                                    clip_lo, clip_hi, bits, group_size, _p(Wq), N, w_layout, _p(w_scale),
                                    _p(w_zero), _p(w_sum), _p(out_bias), _p(Y), Y.stride(0) if M > 0 else N,
                                    _p(Wq6), _p(workspace),
                                    workspace.numel() * workspace.element_size(), _stream(stream)))


STATIC_WORKSPACE_BYTES = 8 << 20      # BASQ_STATIC_WORKSPACE_BYTES of include/basq.h


def basq_linear_fused_static(X: torch.Tensor, rot_size: int, bias: Optional[torch.Tensor],
                             act_scale: Optional[torch.Tensor], clip_lo: float, clip_hi: float, Wq: torch.Tensor,
                             w_scale: torch.Tensor, w_zero: torch.Tensor, w_sum: torch.Tensor,
                             out_bias: Optional[torch.Tensor], Y: torch.Tensor, *,
                             Wq6: Optional[torch.Tensor] = None,
                             bits: int = 4, group_size: int = 0, w_layout: int = BASQ_W_CANONICAL,
                             N: Optional[int] = None, stream: Optional[torch.cuda.Stream] = None) -> None:
    """basq_linear_fused on the library's own workspace (no workspace argument, nothing allocated)."""
    M, K = X.shape
    N = Wq.shape[0] if N is None else N
    _need(Wq6, basq_fp6_bytes(N, K), "Wq6")
    _check(load().basq_linear_fused_static(_p(X), M, K, X.stride(0) if M > 0 else K, rot_size, _p(bias),
                                           _p(act_scale), clip_lo, clip_hi, bits, group_size, _p(Wq), N, w_layout,
                                           _p(w_scale), _p(w_zero), _p(w_sum), _p(out_bias), _p(Y),
                                           Y.stride(0) if M > 0 else N, _p(Wq6), _stream(stream)))


def basq_rotate_weights(W: torch.Tensor, rot_size: int, W_rot: torch.Tensor, workspace: torch.Tensor, *,
                        stream: Optional[torch.cuda.Stream] = None) -> None:
    """W bf16 [N, K] -> W_rot bf16 [N, K] = W . (H_n/sqrt(n)) blockwise; workspace >= N*K*4 bytes."""
    N, K = W.shape
    _check(load().basq_rotate_weights(_p(W), N, K, W.stride(0), rot_size, _p(W_rot), _p(workspace),
                                      workspace.numel() * workspace.element_size(), _stream(stream)))


def basq_quantize_weights(W_rot: torch.Tensor, Wq: torch.Tensor, w_scale: torch.Tensor, w_zero: torch.Tensor,
                          w_sum: torch.Tensor, *, stream: Optional[torch.cuda.Stream] = None) -> None:
    N, K = W_rot.shape
    _check(load().basq_quantize_weights(_p(W_rot), N, K, W_rot.stride(0), _p(Wq), _p(w_scale), _p(w_zero),
                                        _p(w_sum), _stream(stream)))


def basq_fused_bias(Wq: torch.Tensor, w_scale: torch.Tensor, w_zero: torch.Tensor, bias: Optional[torch.Tensor],
                    layer_bias: Optional[torch.Tensor], out_bias: torch.Tensor, *,
                    stream: Optional[torch.cuda.Stream] = None) -> None:
    N, KB = Wq.shape
    _check(load().basq_fused_bias(_p(Wq), N, KB * 2, _p(w_scale), _p(w_zero), _p(bias), _p(layer_bias),
                                  _p(out_bias), _stream(stream)))


def basq_prepare_weights(Wq: torch.Tensor, w_scale: torch.Tensor, w_zero: torch.Tensor, bias: Optional[torch.Tensor],
                         layer_bias: Optional[torch.Tensor], w_sum: torch.Tensor, out_bias: torch.Tensor,
                         Wq_prepacked: Optional[torch.Tensor] = None, *,
                         stream: Optional[torch.cuda.Stream] = None) -> None:
    """Wq uint8 [N, K/2] -> w_sum fp32 [N], out_bias fp32 [N], and (optional) the fp6 operand form of the weights."""
    N, KB = Wq.shape
    _need(w_sum, 4 * N, "w_sum")
    _need(out_bias, 4 * N, "out_bias")
    _need(Wq_prepacked, basq_fp6_bytes(N, KB * 2), "Wq_prepacked")
    _check(load().basq_prepare_weights(_p(Wq), N, KB * 2, _p(w_scale), _p(w_zero), _p(bias), _p(layer_bias),
                                       _p(w_sum), _p(out_bias), _p(Wq_prepacked), _stream(stream)))


def basq_calibrate_bias(X: torch.Tensor, rot_size: int, act_scale: Optional[torch.Tensor], bias_out: torch.Tensor,
                        workspace: torch.Tensor, *, stream: Optional[torch.cuda.Stream] = None) -> None:
    M, K = X.shape
    _check(load().basq_calibrate_bias(_p(X), M, K, X.stride(0), rot_size, _p(act_scale), _p(bias_out),
                                      _p(workspace), workspace.numel() * workspace.element_size(),
                                      _stream(stream)))


def basq_diag_stream(src: torch.Tensor, dst: torch.Tensor, meta: torch.Tensor, tokens: int, K: int, *,
                     stream: Optional[torch.cuda.Stream] = None) -> None:
    _check(load().basq_diag_stream(_p(src), _p(dst), _p(meta), tokens, K, _stream(stream)))


def basq_diag_read(src: torch.Tensor, out: torch.Tensor, blocks: int, *, stream: Optional[torch.cuda.Stream] = None) -> None:
    """src: any tensor of a multiple of 32768 bytes; out int32/uint32 [blocks*256]."""
    _check(load().basq_diag_read(_p(src), src.numel() * src.element_size(), _p(out), blocks, _stream(stream)))


def basq_diag_mfma_i8(out: torch.Tensor, blocks: int, iters: int, *, stream: Optional[torch.cuda.Stream] = None) -> None:
    _check(load().basq_diag_mfma_i8(_p(out), blocks, iters, _stream(stream)))


def basq_diag_mfma_f6(out: torch.Tensor, blocks: int, iters: int, *, stream: Optional[torch.cuda.Stream] = None) -> None:
    _check(load().basq_diag_mfma_f6(_p(out), blocks, iters, _stream(stream)))


# ---- allocation helpers (device memory only; no arithmetic) ----------------------------------

def alloc_activation_buffers(M: int, K: int, device="cuda") -> Tuple[torch.Tensor, torch.Tensor]:
    """(Aq uint8 [M, K/2], meta int32 [M, 4]) for basq_rotate_quant / basq_w4a4_gemm."""
    return (torch.empty((M, K // 2), dtype=torch.uint8, device=device),
            torch.empty((M, 4), dtype=torch.int32, device=device))


def alloc_fp6_buffer(rows: int, K: int, device="cuda") -> torch.Tensor:
    """out6 uint8 [basq_fp6_bytes(rows, K)] for basq_pack_fp6 / the Aq6 output of basq_rotate_quant."""
    return torch.empty(basq_fp6_bytes(rows, K), dtype=torch.uint8, device=device)


def alloc_weight_buffers(N: int, K: int, device="cuda"):
    """(Wq uint8 [N, K/2], w_scale bf16 [N], w_zero bf16 [N], w_sum fp32 [N])."""
    return (torch.empty((N, K // 2), dtype=torch.uint8, device=device),
            torch.empty(N, dtype=torch.bfloat16, device=device),
            torch.empty(N, dtype=torch.bfloat16, device=device),
            torch.empty(N, dtype=torch.float32, device=device))
