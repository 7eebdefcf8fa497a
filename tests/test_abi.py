"""The C-ABI library without a GPU: it loads, exports every symbol the header declares, and turns
bad arguments into error codes before anything would be launched."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_2506_15689_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2506_15689_amd import build
        build.build_lib(verbose=False)
    return B.load()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "basq.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(basq_[a-z0-9_]+)\s*\(", header))
    assert {"basq_rotate_quant", "basq_w4a4_gemm", "basq_linear_fused"} <= declared
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in basq.h but not exported"
    assert declared == set(B.EXPORTS)


def test_version_and_error_text(lib):
    assert B.basq_version() >= 100
    rc = lib.basq_rotate_quant(None, 4, 100, 100, 64, None, None, 0.9, 0.9, 4, 0, None, None, None, None, None)
    assert rc == B.BASQ_EINVAL and "multiple of 32" in B.basq_last_error()


FAKE = ctypes.c_void_p(0x1000)      # aligned, never dereferenced: validation fails first


@pytest.mark.parametrize("kw,code", [
    (dict(M=-1), B.BASQ_EINVAL),
    (dict(K=0), B.BASQ_EINVAL),
    (dict(K=48), B.BASQ_EINVAL),
    (dict(ldx=1016), B.BASQ_EINVAL),
    (dict(ldx=1028), B.BASQ_EINVAL),
    (dict(rot=1000), B.BASQ_EUNSUPPORTED),
    (dict(rot=28), B.BASQ_EUNSUPPORTED),
    (dict(rot=768), B.BASQ_EUNSUPPORTED),
    (dict(K=1024, rot=512 * 3), B.BASQ_EUNSUPPORTED),
    (dict(K=1024 + 512, ldx=2048, rot=1024), B.BASQ_EINVAL),
    (dict(bits=8), B.BASQ_EUNSUPPORTED),
    (dict(bits=3), B.BASQ_EUNSUPPORTED),
    (dict(group=100), B.BASQ_EINVAL),                                 # not a multiple of 32
    (dict(group=96), B.BASQ_EINVAL),                                  # does not divide K
    (dict(K=1056, ldx=1056, rot=32, group=96, Aq6=FAKE), B.BASQ_EINVAL),   # fp6 form with groups: still K % 128 == 0
    (dict(clip_lo=0.0), B.BASQ_EINVAL),
    (dict(clip_hi=1.5), B.BASQ_EINVAL),
    (dict(clip_lo=float("nan")), B.BASQ_EINVAL),
    (dict(X=None), B.BASQ_EINVAL),
    (dict(X=ctypes.c_void_p(0x1008)), B.BASQ_EINVAL),
    (dict(Aq=None), B.BASQ_EINVAL),
    (dict(Aq=None, Aq6=FAKE), B.BASQ_EUNSUPPORTED),                   # the fp6 form alone: only where the quantiser writes it itself
    (dict(Aq=None, Aq6=FAKE, K=4096, ldx=4096, rot=4096, group=128), B.BASQ_EUNSUPPORTED),
    (dict(meta=None), B.BASQ_EINVAL),
    (dict(K=65536, ldx=65536, rot=65536), B.BASQ_EUNSUPPORTED),
    (dict(K=1056, ldx=1056, rot=32, Aq6=FAKE), B.BASQ_EINVAL),        # fp6 form needs K % 128 == 0
    (dict(Aq6=ctypes.c_void_p(0x1008)), B.BASQ_EINVAL),
    (dict(bias=ctypes.c_void_p(0x1004)), B.BASQ_EINVAL),              # b^c and s^a are read four channels at a time
    (dict(sa=ctypes.c_void_p(0x1008)), B.BASQ_EINVAL),
])
def test_rotate_quant_rejects_bad_arguments(lib, kw, code):
    a = dict(X=FAKE, M=4, K=1024, ldx=1024, rot=1024, bias=None, sa=None, clip_lo=0.9, clip_hi=0.9, bits=4,
             group=0, Aq=FAKE, meta=FAKE, rot_out=None, Aq6=None)
    a.update(kw)
    rc = lib.basq_rotate_quant(a["X"], a["M"], a["K"], a["ldx"], a["rot"], a["bias"], a["sa"], a["clip_lo"],
                               a["clip_hi"], a["bits"], a["group"], a["Aq"], a["meta"], a["rot_out"], a["Aq6"], None)
    assert rc == code, B.basq_last_error()
    assert B.basq_last_error() != ""


@pytest.mark.parametrize("kw,code", [
    (dict(M=-2), B.BASQ_EINVAL),
    (dict(K=100), B.BASQ_EINVAL),
    (dict(N=0), B.BASQ_EINVAL),
    (dict(layout=7), B.BASQ_EUNSUPPORTED),
    (dict(ldy=100), B.BASQ_EINVAL),
    (dict(Wq=None), B.BASQ_EINVAL),
    (dict(w_scale=None), B.BASQ_EINVAL),
    (dict(w_zero=None), B.BASQ_EINVAL),
    (dict(w_sum=None), B.BASQ_EINVAL),
    (dict(Aq=None), B.BASQ_EINVAL),
    (dict(Y=None), B.BASQ_EINVAL),
    (dict(Aq=ctypes.c_void_p(0x1004)), B.BASQ_EINVAL),
    (dict(Y=ctypes.c_void_p(0x1001)), B.BASQ_EINVAL),
    (dict(Aq6=FAKE), B.BASQ_EINVAL),                                  # fp6 operands: both or neither
    (dict(Wq6=FAKE), B.BASQ_EINVAL),
    (dict(K=1056, Aq6=FAKE, Wq6=FAKE), B.BASQ_EINVAL),
    (dict(Aq6=FAKE, Wq6=ctypes.c_void_p(0x1004)), B.BASQ_EINVAL),
])
def test_gemm_rejects_bad_arguments(lib, kw, code):
    a = dict(Aq=FAKE, meta=FAKE, M=8, K=1024, Wq=FAKE, N=256, layout=0, w_scale=FAKE, w_zero=FAKE, w_sum=FAKE,
             out_bias=None, Y=FAKE, ldy=256, acc=None, Aq6=None, Wq6=None)
    a.update(kw)
    rc = lib.basq_w4a4_gemm(a["Aq"], a["meta"], a["M"], a["K"], a["Wq"], a["N"], a["layout"], a["w_scale"],
                            a["w_zero"], a["w_sum"], a["out_bias"], a["Y"], a["ldy"], a["acc"], a["Aq6"], a["Wq6"],
                            None)
    assert rc == code, B.basq_last_error()


def test_fused_call_checks_workspace(lib):
    need = B.basq_workspace_bytes(64, 1024, 256)
    assert need >= 64 * 512 + 64 * 16 and need % 256 == 0
    assert need >= 64 * 512 + 64 * 16 + B.basq_fp6_bytes(64, 1024)
    args = [FAKE, 64, 1024, 1024, 1024, None, None, 0.9, 0.9, 4, 0, FAKE, 256, 0, FAKE, FAKE, FAKE, None, FAKE, 256,
            None]
    assert lib.basq_linear_fused(*args, ctypes.c_void_p(0x2000), need - 1, None) == B.BASQ_EWORKSPACE
    assert "workspace too small" in B.basq_last_error()
    assert lib.basq_linear_fused(*args, None, need, None) == B.BASQ_EINVAL
    assert lib.basq_linear_fused(*args, ctypes.c_void_p(0x2010), need, None) == B.BASQ_EINVAL
    odd = list(args)
    odd[2] = odd[3] = 1056; odd[4] = 32                                     # fp6 weights need K % 128 == 0
    odd[-1] = FAKE
    assert lib.basq_linear_fused(*odd, ctypes.c_void_p(0x2000), 1 << 20, None) == B.BASQ_EINVAL


def test_static_workspace_call_rejects_what_does_not_fit(lib):
    """basq_linear_fused_static: shapes whose codes and records exceed the library's own workspace fail on the
    host, before the workspace is even looked up (so this runs without a GPU)."""
    args = lambda M, K: [FAKE, M, K, K, K, None, None, 0.9, 0.9, 4, 0, FAKE, 256, 0, FAKE, FAKE, FAKE, None, FAKE, 256,
                         None, None]
    assert B.basq_workspace_bytes(4096, 8192, 256) > B.STATIC_WORKSPACE_BYTES
    assert lib.basq_linear_fused_static(*args(4096, 8192)) == B.BASQ_EWORKSPACE
    assert "workspace" in B.basq_last_error()
    assert lib.basq_linear_fused_static(*args(-1, 1024)) == B.BASQ_EINVAL
    assert lib.basq_linear_fused_static(*args(8, 1000)) == B.BASQ_EINVAL
    header = open(os.path.join(ROOT, "include", "basq.h")).read()
    m = re.search(r"#define\s+BASQ_STATIC_WORKSPACE_BYTES\s+\((\d+)u\s*<<\s*(\d+)\)", header)
    assert m and int(m.group(1)) << int(m.group(2)) == B.STATIC_WORKSPACE_BYTES


def test_fp6_form_sizes_and_argument_checks(lib):
    assert B.basq_fp6_bytes(64, 1024) == 64 * 768
    assert B.basq_fp6_bytes(33, 256) == 64 * 192                      # whole 32-row blocks
    assert B.basq_fp6_bytes(5, 100) == 0 and B.basq_fp6_bytes(-1, 128) == 0
    assert lib.basq_pack_fp6(FAKE, 8, 100, FAKE, None) == B.BASQ_EINVAL
    assert lib.basq_pack_fp6(None, 8, 128, FAKE, None) == B.BASQ_EINVAL
    assert lib.basq_pack_fp6(FAKE, 8, 128, ctypes.c_void_p(0x1008), None) == B.BASQ_EINVAL
    assert lib.basq_pack_fp6(None, 0, 128, None, None) == 0


def test_decode_layout_sizes_and_argument_checks(lib):
    assert B.basq_decode_bytes(4096, 4096) == 4096 * 2048
    assert B.basq_decode_bytes(17, 256) == 32 * 128                        # whole 16-row blocks
    assert B.basq_decode_bytes(16, 96) == 0 and B.basq_decode_bytes(0, 128) == 0
    assert lib.basq_pack_decode(FAKE, 8, 96, FAKE, None) == B.BASQ_EINVAL
    assert lib.basq_pack_decode(None, 8, 128, FAKE, None) == B.BASQ_EINVAL
    assert lib.basq_pack_decode(FAKE, 0, 128, FAKE, None) == B.BASQ_EINVAL
    assert lib.basq_pack_decode(FAKE, 8, 128, ctypes.c_void_p(0x1008), None) == B.BASQ_EINVAL
    # the streaming layout: K % 128, and more than 128 tokens only with the fp6 operands
    gemm = lambda M, K, layout, a6=None, w6=None: lib.basq_w4a4_gemm(
        FAKE, FAKE, M, K, FAKE, 32, layout, FAKE, FAKE, FAKE, None, FAKE, 32, None, a6, w6, None)
    assert gemm(4, 96, B.BASQ_W_DECODE16) == B.BASQ_EINVAL
    assert gemm(129, 256, B.BASQ_W_DECODE16) == B.BASQ_EUNSUPPORTED
    assert "fp6" in B.basq_last_error()
    assert gemm(4, 256, 2) == B.BASQ_EUNSUPPORTED
    ws = ctypes.c_void_p(0x100000)
    assert lib.basq_linear_fused(FAKE, 129, 256, 256, 256, None, None, 0.9, 0.9, 4, 0, FAKE, 32, B.BASQ_W_DECODE16,
                                 FAKE, FAKE, FAKE, None, FAKE, 32, None, ws, 1 << 30, None) == B.BASQ_EUNSUPPORTED


def test_grouped_gemm_argument_checks(lib):
    call = lambda M, K, G, gs=FAKE, a6=None, w6=None: lib.basq_w4a4_gemm_grouped(
        FAKE, FAKE, M, K, G, FAKE, 32, FAKE, FAKE, gs, None, FAKE, 32, a6, w6, None)
    assert call(4, 256, 64) == B.BASQ_EUNSUPPORTED                     # only groups of 128
    assert call(4, 192, 128) == B.BASQ_EINVAL                          # K % 128
    assert call(4, 256, 128, None) == B.BASQ_EINVAL
    assert call(0, 256, 128) == 0                                      # no tokens: nothing launched
    assert call(4, 256, 128, FAKE, FAKE, None) == B.BASQ_EINVAL        # fp6 operands: both or neither
    assert call(4, 256, 128, FAKE, None, FAKE) == B.BASQ_EINVAL
    assert call(4, 256, 128, FAKE, FAKE, ctypes.c_void_p(0x1008)) == B.BASQ_EINVAL
    assert call(0, 256, 128, FAKE, FAKE, FAKE) == 0
    assert lib.basq_group_colsums(FAKE, 8, 192, 128, FAKE, None) == B.BASQ_EINVAL
    assert lib.basq_group_colsums(FAKE, 8, 256, 32, FAKE, None) == B.BASQ_EUNSUPPORTED
    assert lib.basq_group_colsums(None, 8, 256, 128, FAKE, None) == B.BASQ_EINVAL


def test_zero_tokens_is_valid_without_a_launch(lib):
    assert lib.basq_rotate_quant(None, 0, 1024, 1024, 1024, None, None, 0.9, 0.9, 4, 0, None, None, None, None, None) == 0
    assert lib.basq_w4a4_gemm(None, None, 0, 1024, FAKE, 16, 0, FAKE, FAKE, FAKE, None, None, 16, None, None, None, None) == 0


def test_offline_helpers_reject_bad_arguments(lib):
    assert lib.basq_rotate_weights(None, 8, 64, 64, 64, FAKE, FAKE, 1 << 20, None) == B.BASQ_EINVAL
    assert lib.basq_rotate_weights(FAKE, 8, 64, 64, 48, FAKE, FAKE, 1 << 20, None) != 0       # 48 is no Hadamard size
    assert lib.basq_rotate_weights(FAKE, 8, 64, 64, 64, FAKE, FAKE, 8 * 64 * 4 - 1, None) == B.BASQ_EWORKSPACE
    assert lib.basq_rotate_weights(FAKE, 0, 64, 64, 64, FAKE, FAKE, 1 << 20, None) == B.BASQ_EINVAL
    assert lib.basq_quantize_weights(None, 8, 64, 64, FAKE, FAKE, FAKE, FAKE, None) == B.BASQ_EINVAL
    assert lib.basq_quantize_weights(FAKE, 8, 64, 32, FAKE, FAKE, FAKE, FAKE, None) == B.BASQ_EINVAL
    assert lib.basq_fused_bias(FAKE, 0, 64, FAKE, FAKE, None, None, FAKE, None) == B.BASQ_EINVAL
    prep = lambda **kw: lib.basq_prepare_weights(*[{**dict(Wq=FAKE, N=8, K=128, ws=FAKE, wz=FAKE, b=None, lb=None, wsum=FAKE,
                                                           ob=FAKE, pre=None), **kw}[k]
                                                   for k in ("Wq", "N", "K", "ws", "wz", "b", "lb", "wsum", "ob", "pre")], None)
    assert prep(N=0) == B.BASQ_EINVAL and prep(K=48) == B.BASQ_EINVAL
    assert prep(Wq=None) == B.BASQ_EINVAL and prep(wsum=None) == B.BASQ_EINVAL and prep(ob=None) == B.BASQ_EINVAL
    assert prep(Wq=ctypes.c_void_p(0x1004)) == B.BASQ_EINVAL
    assert prep(K=96, pre=FAKE) == B.BASQ_EINVAL                       # the fp6 operand form needs K % 128 == 0
    assert prep(pre=ctypes.c_void_p(0x1008)) == B.BASQ_EINVAL
    assert lib.basq_calibrate_bias(FAKE, 16, 1024, 1024, 1024, None, FAKE, FAKE, 16 * 1024 * 4 - 1, None) == B.BASQ_EWORKSPACE
    assert lib.basq_calibrate_bias(FAKE, 0, 1024, 1024, 1024, None, FAKE, FAKE, 1 << 20, None) == B.BASQ_EINVAL
    assert lib.basq_hadamard28(None) == B.BASQ_EINVAL


def test_hadamard28_table_matches_oracle(lib):
    """The rotation for 28 * 2^t channels needs the same sign table on both sides; the library
    builds its own from the Paley construction."""
    np.testing.assert_array_equal(B.basq_hadamard28().numpy(), oracle.hadamard_paley28())
