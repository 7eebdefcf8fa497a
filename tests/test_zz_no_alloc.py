"""basq_linear_fused_static: the one-call layer on the library's own workspace, for callers that cannot allocate.
Called through the C ABI, twice in a row (the second call smaller, so the workspace still holds the first call's
codes), and compared bit for bit with basq_linear_fused on a caller workspace -- which test_gpu_parity.py ties to the
CPU oracle -- and, on the small first case, with the oracle itself."""
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


def _both(case, d, *, fp6, decode_layout=False):
    """(Y from basq_linear_fused_static, Y from basq_linear_fused) as bf16 bit arrays."""
    dev = d.X.device
    M, K, N = case.M, case.K, case.N
    kw = {}
    Wq = d.Wq
    if fp6:
        W6 = B.alloc_fp6_buffer(N, K, dev).zero_()
        B.basq_pack_fp6(d.Wq, W6)
        kw["Wq6"] = W6
    if decode_layout:
        Wq = torch.empty(B.basq_decode_bytes(N, K), dtype=torch.uint8, device=dev)
        B.basq_pack_decode(d.Wq, Wq)
        kw.update(w_layout=B.BASQ_W_DECODE16, N=N)
    Ys = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=dev)
    Yw = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=dev)
    ws = torch.empty(max(B.basq_workspace_bytes(M, K, N), 256), dtype=torch.uint8, device=dev)
    B.basq_linear_fused_static(d.X, case.rot_size, d.bias, d.act_scale, case.clip_lo, case.clip_hi, Wq, d.w_scale,
                               d.w_zero, d.w_sum, d.out_bias, Ys, **kw)
    B.basq_linear_fused(d.X, case.rot_size, d.bias, d.act_scale, case.clip_lo, case.clip_hi, Wq, d.w_scale,
                        d.w_zero, d.w_sum, d.out_bias, Yw, ws, **kw)
    torch.cuda.synchronize()
    return si.bf16_bits(Ys.cpu()), si.bf16_bits(Yw.cpu())


@pytest.mark.parametrize("shapes,fp6", [
    # (M, K, N) of the first and of the second, smaller call
    (((300, 4096, 264), (141, 4096, 264)), True),        # tiled fp6 GEMM both times, ragged row blocks
    (((200, 1024, 136), (37, 512, 72)), False),          # int8 GEMM, then the weight-streaming kernel on another K
    (((700, 8192, 72), (3, 8192, 72)), True),            # near the limit at K = 8192, then a decode-sized call
])
def test_static_workspace_matches_caller_workspace(shapes, fp6):
    for i, (M, K, N) in enumerate(shapes):
        announce(f"basq_linear_fused_static call {i}: M={M} K={K} N={N} fp6={fp6}")
        case = pu.make_case(si.make_tiny(M, K, N, seed=11 * M + i))
        d = pu.to_device(case)
        ys, yw = _both(case, d, fp6=fp6)
        assert not np.isnan(oracle.bf16_to_f32(ys)).any(), "an output element was not written"
        np.testing.assert_array_equal(ys, yw, err_msg=f"static vs caller workspace, call {i}")
        if M * K * N <= 200 * 1024 * 136:                # the small case also straight against the oracle
            ref = oracle.linear(case.x, case.rot_size, case.bias, case.act_scale, case.clip_lo, case.clip_hi,
                                case.wq, case.c)
            y = oracle.bf16_to_f32(ys).astype(np.float64)
            err = float(np.abs(y - ref.y).max() / np.abs(ref.y).max())
            assert err <= pu.Y_TOL, f"output error {err} of max|ref|"


def test_static_workspace_decode_one_launch_then_smaller():
    """Four tokens, then one, on the streaming layout: the one-launch kernel (its codes live in LDS, the workspace is
    only checked) after a call that did use the workspace."""
    big = pu.make_case(si.make_tiny(500, 4096, 256, seed=5))
    db = pu.to_device(big)
    ys, yw = _both(big, db, fp6=True)
    np.testing.assert_array_equal(ys, yw)
    for M in (4, 1):
        announce(f"basq_linear_fused_static decode M={M}")
        case = pu.make_case(si.make_tiny(M, 4096, 256, seed=40 + M))
        d = pu.to_device(case)
        ys, yw = _both(case, d, fp6=False, decode_layout=True)
        np.testing.assert_array_equal(ys, yw, err_msg=f"decode, M={M}")


def test_static_workspace_rejects_what_does_not_fit():
    """Beyond BASQ_STATIC_WORKSPACE_BYTES the call fails on the host and launches nothing."""
    M, K, N = 4096, 8192, 64
    assert B.basq_workspace_bytes(M, K, N) > B.STATIC_WORKSPACE_BYTES
    dev = torch.device("cuda")
    X = torch.zeros((M, K), dtype=torch.bfloat16, device=dev)
    Wq, w_scale, w_zero, w_sum = B.alloc_weight_buffers(N, K, dev)
    Y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=dev)
    with pytest.raises(B.BasqError) as e:
        B.basq_linear_fused_static(X, K, None, None, 0.9, 0.9, Wq, w_scale, w_zero, w_sum, None, Y)
    assert e.value.code == B.BASQ_EWORKSPACE and "workspace" in str(e.value)
    torch.cuda.synchronize()
    assert torch.isnan(Y).all(), "a rejected call wrote output"
    # the largest M that fits at this K is accepted
    M_fit = 800
    assert B.basq_workspace_bytes(M_fit, K, N) <= B.STATIC_WORKSPACE_BYTES < B.basq_workspace_bytes(M_fit + 32, K, N)
    B.basq_linear_fused_static(X[:M_fit], K, None, None, 0.9, 0.9, Wq.zero_(), w_scale.fill_(1.0), w_zero.zero_(),
                               w_sum.zero_(), None, Y[:M_fit])
    torch.cuda.synchronize()
    assert not torch.isnan(Y[:M_fit]).any()
