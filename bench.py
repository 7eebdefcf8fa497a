#!/usr/bin/env python3
"""Benchmark of the W4A4 rotated linear layer on one MI355X.

A step is one pass of the whole hot path -- online rotation + bias + per-token INT4 quantisation,
then the INT4 x INT4 GEMM with fused de-quantisation -- over one batch of synthetic activations
that already sit in HBM.  Prints ONE JSON line:

  value        whole-layer throughput, 2*M*N*K integer operations per second of step time (TOPS)
  roofline     the dominant kernel (the GEMM, bound by the matrix cores; for decode shapes HBM bound)
  roofline_rotate_quant   the rotate+bias+quant kernel against HBM bandwidth, priced on the method's own bytes
               (2.5 per channel + 16 per token); the bytes of the design's fp6 copy are reported beside it, and under
               "alu" the same launch against the vector pipes' issue rate (instructions from the counter summaries)
  other_workloads   the remaining workloads of the definition (C2, C4 prefill; C3 decode with 1, 4, 16 tokens),
               measured in the same process after the headline one
  cpu_baseline the CPU oracle timed on a bounded sample of the same workload, on all host threads and on one

Kernel durations come from HIP events recorded on the launch stream around back-to-back launches of
each kernel inside the timed region (mean over all launches; minimum and median over batches of ten).
Buffers rotate through several distinct sets so repeated steps do not find their inputs in the 256 MB
last-level cache.  `traffic` is read from profiles/traffic.json, which the profile summariser
(python -m paper_2506_15689_amd.profile_summary) writes from rocprofv3 counter runs of this same script.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
INT8_PEAK_TOPS = 5000.0      # MI355X dense int8 MFMA, published
FP6_PEAK_TOPS = 10100.0      # MI355X dense fp6 / fp4 MFMA, published
# 256 compute units x 4 SIMDs at 2.4 GHz, one 64-lane vector instruction per four cycles per SIMD (16 lanes wide;
# the published 157.3 TFLOP/s fp32 figure counts packed two-element fused multiply-adds, which this build does not use)
VALU_ISSUE_PEAK_G = 256 * 4 * 2.4 / 4
TRAFFIC_JSON = os.path.join(ROOT, "profiles", "traffic.json")
OTHER_WORKLOADS = ("C2", "C4", "C3_M1", "C3_M4", "C3_M16")


def parse_args(argv=None):
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=50)
    p.add_argument("--warmup", type=int, default=20)
    p.add_argument("--config", default="C5",
                   help="workload name from synth_inputs.CONFIGS (default C5: the M=4096 prefill GEMM the targets are quoted on)")
    p.add_argument("--sets", type=int, default=0, help="distinct buffer sets to rotate through (0 = auto)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--no-ceilings", action="store_true", help="skip the measured-ceiling diagnostics")
    p.add_argument("--no-other-workloads", action="store_true",
                   help="skip the other workloads of the definition (they run after the default C5 measurement only)")
    p.add_argument("--M", type=int, default=0, help="override the token count (sweeps)")
    p.add_argument("--calibrate-copy", action="store_true",
                   help="also run a plain 256 MiB device copy three times (scales the HBM byte counters of a profiler run)")
    p.add_argument("--no-bias", action="store_true", help="run the kernels without the channel bias (experiments)")
    p.add_argument("--matrix-path", default="fp6", choices=["fp6", "int8"],
                   help="prefill GEMM on the f8f6f4 matrix-core path (codes repacked as exact fp6 values; default) "
                        "or on the int8 path; decode-sized M always streams the INT4 weights")
    p.add_argument("--weight-layout", default="stream", choices=["stream", "canonical"],
                   help="decode shapes (M <= 128): weights in the weight-streaming layout (default) or canonical")
    p.add_argument("--graph", action="store_true",
                   help="record the K timed steps in one HIP graph and time its replay (decode shapes: removes the host's "
                        "launch cost of a few microseconds per call from the measurement)")
    p.add_argument("--rot-size", type=int, default=0, help="with --only rotate_quant: rotation block instead of the workload's")
    p.add_argument("--group-size", type=int, default=0,
                   help="with --only rotate_quant: channels per range (0 = per token); 128 with --rot-size 128 is the "
                        "per-head quantiser of q, k and the KV cache")
    p.add_argument("--only", default="", choices=["", "rotate_quant"],
                   help="time only the rotate+quant kernel (large-M sweeps; value is then its GB/s)")
    p.add_argument("--no-fp6-copy", action="store_true",
                   help="with --only rotate_quant: do not write the fp6 copy of the codes (the method's own bytes only)")
    return p.parse_args(argv)


def algorithmic_bytes_rotate_quant(M, K, fp6=False, group=0, codes4=True):
    # per token: 2K bytes of bf16 in, K/2 bytes of codes + 16 bytes per record out (one per token, or one per
    # group), and 3K/4 bytes more when the codes are also written in the fp6 operand form (codes4 = False: the
    # 4-bit form is not written at all, as in the one-call layer on the fp6 path)
    records = 1 if group in (0, K) else K // group
    return M * (2 * K + (K // 2 if codes4 else 0) + 16 * records + (3 * K // 4 if fp6 else 0))


def algorithmic_bytes_gemm(M, K, N, fp6=False):
    # codes of both operands (4 bits each, or 6 in the fp6 operand form), token records, per-channel
    # vectors, bf16 output
    per_code = 3 * K // 4 if fp6 else K // 2
    return M * (per_code + 16) + N * per_code + N * (2 + 2 + 4 + 4) + 2 * M * N


def load_traffic():
    """profiles/traffic.json: {"entries": {"<workload>/<kernel>": {"bytes_per_launch": ..., ...}}, ...} or {}."""
    try:
        with open(TRAFFIC_JSON) as f:
            return json.load(f)
    except (OSError, ValueError):
        return {}


def traffic_of(table, workload, kernel, field="bytes_per_launch"):
    """HBM-side bytes per launch of `kernel` (name prefix) on `workload` from the tracked counter summary (or another
    field of its entry), or None."""
    for key, ent in table.get("entries", {}).items():
        w, _, k = key.partition("/")
        if w == workload and k.startswith(kernel):
            return ent.get(field)
    return None


# ---- CPU oracle leg (runs in a child process so that its thread count can be set; never touches the GPU) -----------

def cpu_baseline_child(config, sample_tokens):
    import numpy as np
    import oracle
    from paper_2506_15689_amd import synth_inputs as si
    cfg = si.CONFIGS[config]
    lay = si.make_layer(cfg)
    sample_tokens = min(sample_tokens, lay.X.shape[0])
    x = oracle.bf16_to_f32(si.bf16_bits(lay.X[:sample_tokens]))
    w = oracle.bf16_to_f32(si.bf16_bits(lay.W_rot))
    xc = oracle.bf16_to_f32(si.bf16_bits(lay.X_calib))
    bc = oracle.channel_bias(xc, cfg.rot_size)            # offline parts are not timed
    wq = oracle.quantize_weights(w)
    c = oracle.fused_bias(wq, bc, None)
    oracle.hadamard_matrix(cfg.rot_size)                  # the dense matrix is a constant: built once
    t0 = time.perf_counter()
    res = oracle.linear(x, cfg.rot_size, bc, None, cfg.clip, cfg.clip, wq, c)
    dt = time.perf_counter() - t0
    ops = 2.0 * sample_tokens * cfg.N * cfg.K
    print(json.dumps({"value": ops / dt / 1e12, "unit": "TOPS", "cores": oracle.num_threads(), "kind": "oracle",
                      "sample": f"first {sample_tokens} of {lay.X.shape[0]} tokens x all N={cfg.N}, K={cfg.K}: "
                                f"{dt:.2f} s for rotation (fp64 dense) + quantiser + int32 triple-loop GEMM + dequant",
                      "seconds": dt, "checksum": float(np.abs(res.y).sum())}))


def cpu_baseline(config, sample_tokens, threads=None):
    """The oracle as it stands on the first `sample_tokens` tokens x all N, in a child process (threads: OpenMP and
    BLAS thread count of the child; None = whatever the box gives it)."""
    env = dict(os.environ)
    if threads is not None:
        for var in ("OMP_NUM_THREADS", "OPENBLAS_NUM_THREADS", "MKL_NUM_THREADS"):
            env[var] = str(threads)
    code = f"import sys; sys.path.insert(0, {ROOT!r}); import bench; bench.cpu_baseline_child({config!r}, {int(sample_tokens)})"
    p = subprocess.run([sys.executable, "-c", code], env=env, cwd=ROOT, stdout=subprocess.PIPE, stderr=subprocess.PIPE,
                       text=True, timeout=600)
    lines = [l for l in p.stdout.splitlines() if l.startswith("{")]
    if p.returncode != 0 or not lines:
        return {"error": (p.stderr or p.stdout)[-400:]}
    return json.loads(lines[-1])


# ---- one workload -----------------------------------------------------------------------------------------------

def run_workload(args, config, steps, warmup, *, with_ceilings, traffic_table, M_override=0, also_graph=False):
    """Prepares `config` through the library, times `steps` steps of the whole path and each kernel on its own.
    Returns (fields of the JSON line for this workload, cfg, M)."""
    import torch
    from paper_2506_15689_amd import binding as B
    from paper_2506_15689_amd import synth_inputs as si

    dev = torch.device("cuda:0")
    cfg = si.CONFIGS[config]
    grouped = args.group_size == 128 and args.only != "rotate_quant"     # group-wise ranges through the GEMM
    rot_size = args.rot_size if args.rot_size > 0 else cfg.rot_size
    group = args.group_size
    M = M_override if M_override > 0 else cfg.M
    K, N = cfg.K, cfg.N
    lay = si.make_layer(cfg, M=M)

    # ---- offline preparation, all through the library -------------------------------------
    W = lay.W_rot.to(dev)
    Wq, w_scale, w_zero, w_sum = B.alloc_weight_buffers(N, K, dev)
    B.basq_quantize_weights(W, Wq, w_scale, w_zero, w_sum)
    Xc = lay.X_calib[:4096].to(dev)           # the bias is calibrated on at most 4096 tokens
    bias = torch.empty(K, dtype=torch.float32, device=dev)
    cal_ws = torch.empty(Xc.shape[0] * K, dtype=torch.float32, device=dev)
    B.basq_calibrate_bias(Xc, rot_size, None, bias, cal_ws)
    out_bias = torch.empty(N, dtype=torch.float32, device=dev)
    rq_only = args.only == "rotate_quant"
    use_fp6 = args.matrix_path == "fp6" and K % 128 == 0 and M > B.STREAM_MAX_TOKENS and group in (0, K)
    g_fp6 = grouped and args.matrix_path == "fp6" and M > 0          # group-wise GEMM on the fp6 matrix-core path
    want6 = (use_fp6 or g_fp6) and not (rq_only and args.no_fp6_copy)
    Wq6 = B.alloc_fp6_buffer(N, K, dev) if (use_fp6 or g_fp6) else None
    # fused bias, weight sums and the fp6 form of the weights in the one offline call of the boundary
    B.basq_prepare_weights(Wq, w_scale, w_zero, bias, None, w_sum, out_bias, Wq6)
    w_gsum = None
    if grouped:
        w_gsum = torch.empty((K // 128, N), dtype=torch.int32, device=dev)
        B.basq_group_colsums(Wq, 128, w_gsum)
    # decode shapes stream the weights once per call: the streaming layout (offline repack), and as many
    # distinct copies as it takes to keep them out of the 256 MB last-level cache between calls
    decode = M <= B.STREAM_MAX_TOKENS and K % 128 == 0 and not grouped
    w_layout, wsets = B.BASQ_W_CANONICAL, [Wq]
    if decode:
        if args.weight_layout == "stream":
            Wd = torch.empty(B.basq_decode_bytes(N, K), dtype=torch.uint8, device=dev)
            B.basq_pack_decode(Wq, Wd)
            w_layout, wsets = B.BASQ_W_DECODE16, [Wd]
        n_w = max(2, min(64, -(-(640 << 20) // wsets[0].numel())))
        wsets = wsets + [wsets[0].clone() for _ in range(n_w - 1)]
    torch.cuda.synchronize()
    del W, cal_ws, Xc
    if args.no_bias:
        bias = None

    # ---- rotating buffer sets (cold-cache discipline) -------------------------------------
    per_set = M * K * 2 + M * (K // 2) + M * 16 + (0 if rq_only else M * N * 2) + (M * K * 3 // 4 if want6 else 0)
    nsets = args.sets if args.sets > 0 else max(2, min(32, -(-(640 << 20) // per_set)))
    X0 = lay.X.to(dev)
    sets = []
    for i in range(nsets):
        Xi = X0 if i == 0 else torch.roll(X0, shifts=i, dims=0).contiguous()
        Aq, meta = B.alloc_activation_buffers(M, K, dev)
        if group not in (0, K):
            meta = torch.empty((M * (K // group), 4), dtype=torch.int32, device=dev)
        Y = None if rq_only else torch.empty((M, N), dtype=torch.bfloat16, device=dev)
        Aq6 = B.alloc_fp6_buffer(M, K, dev) if want6 else None
        sets.append((Xi, Aq, meta, Y, Aq6))
    workspace = torch.empty(max(256, B.basq_workspace_bytes(M, K, N)), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()

    stream = torch.cuda.current_stream()
    one_launch = (w_layout == B.BASQ_W_DECODE16 and M <= 4 and N <= 4096 and K in (4096, 8192) and rot_size == K)

    # what the one-call layer launches on the fp6 path: the quantiser writes the fp6 form of the codes and leaves
    # the 4-bit form out (nothing reads it); timed on its own in that same configuration
    fp6_only = use_fp6 and want6 and rot_size == K and K in (4096, 8192, 14336) and group in (0, K)

    def rotate_quant(i, codes4=not fp6_only):
        Xi, Aq, meta, _, Aq6 = sets[i % nsets]
        B.basq_rotate_quant(Xi, rot_size, bias, None, cfg.clip, cfg.clip, Aq if codes4 else None, meta, None, Aq6=Aq6,
                            group_size=group, stream=stream)

    def gemm(i):
        _, Aq, meta, Y, Aq6 = sets[i % nsets]
        if grouped:
            B.basq_w4a4_gemm_grouped(Aq, meta, 128, Wq, w_scale, w_zero, w_gsum, out_bias, Y,
                                     Aq6=Aq6 if g_fp6 else None, Wq6=Wq6 if g_fp6 else None, stream=stream)
            return
        B.basq_w4a4_gemm(Aq, meta, wsets[i % len(wsets)], w_scale, w_zero, w_sum, out_bias, Y, None, Aq6=Aq6, Wq6=Wq6,
                         w_layout=w_layout, N=N, stream=stream)

    def gemm_int8(i):
        _, Aq, meta, Y, _ = sets[i % nsets]
        B.basq_w4a4_gemm(Aq, meta, Wq, w_scale, w_zero, w_sum, out_bias, Y, None, stream=stream)

    def step(i):
        """One pass of the whole hot path: the single fused entry point."""
        Xi, _, _, Y, _ = sets[i % nsets]
        if grouped:                               # no one-call entry point for groups: the two calls
            rotate_quant(i)
            gemm(i)
            return
        B.basq_linear_fused(Xi, cfg.rot_size, bias, None, cfg.clip, cfg.clip, wsets[i % len(wsets)], w_scale, w_zero,
                            w_sum, out_bias, Y, workspace, Wq6=Wq6, w_layout=w_layout, N=N, stream=stream)

    def timed(fn, count, batch=10):
        """`count` back-to-back calls on the launch stream.  Events bracket the whole run (-> mean) and sit between
        batches of `batch` calls (-> minimum and median of the batch means).  Times in ms per call."""
        nb = max(1, count // batch)
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(nb + 1)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        marks[0].record(stream)
        done, calls = 0, []
        for b in range(nb):
            upto = count if b == nb - 1 else (b + 1) * batch
            for i in range(done, upto):
                fn(i)
            marks[b + 1].record(stream)
            calls.append(upto - done)
            done = upto
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / count
        per_batch = [marks[b].elapsed_time(marks[b + 1]) / calls[b] for b in range(nb)]
        return {"mean": marks[0].elapsed_time(marks[nb]) / count, "min": min(per_batch),
                "median": statistics.median(per_batch), "wall": wall_ms, "launches": count}

    whole = rotate_quant if rq_only else step
    for i in range(nsets):                      # every set holds valid codes (both forms) before anything is timed
        rotate_quant(i, True)
    # the GPU comes out of the host-side preparation at idle clocks: a fixed stretch of untimed steps (about 20 ms)
    # brings it to the state a serving loop runs in, whatever --warmup says; then the W warm-up steps proper
    precondition = 0 if steps < 10 else max(0, min(400, int(0.02 / max(1e-6, 2.0 * M * N * K / 3.5e15 + 6e-6))))
    for i in range(precondition):
        whole(i)
    for i in range(warmup):
        whole(i)
        rotate_quant(i)
        if not rq_only:
            gemm(i)
    torch.cuda.synchronize()

    # the timed region: K steps of the whole path, then launches of each kernel on its own so that each kernel's
    # average duration is known (events around every single launch would add several microseconds of their own
    # to kernels this short)
    t_step = timed(whole, steps)
    ms_step = t_step["mean"]
    graph_note = None
    if args.graph or also_graph:
        # the same K steps, recorded once on a capture stream and replayed: the device-side time of the step
        cap = torch.cuda.Stream()
        cap.wait_stream(stream)
        g = torch.cuda.CUDAGraph()
        eager_stream = stream
        with torch.cuda.graph(g, stream=cap):
            stream = torch.cuda.current_stream()
            for i in range(steps):
                whole(i)
        stream = eager_stream
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        g.replay()
        e1.record(stream)
        torch.cuda.synchronize()
        if args.graph:
            graph_note = {"eager_ms_per_step": ms_step}
            ms_step = e0.elapsed_time(e1) / steps
        else:                                             # reported beside the eager step, which stays the step
            graph_note = {"graph_ms_per_step": e0.elapsed_time(e1) / steps}
    launches = max(steps, 50) if steps >= 10 else steps
    t_rq = timed(rotate_quant, launches)
    t_gemm = None if rq_only else timed(gemm, launches)
    t_gemm8 = timed(gemm_int8, launches) if use_fp6 and not rq_only else None
    rq_ms = t_rq["mean"]
    gemm_ms = float("nan") if rq_only else t_gemm["mean"]
    ops = 0.0 if rq_only else 2.0 * M * N * K
    value = ops / (ms_step * 1e-3) / 1e12

    modified = bool(M_override > 0 or args.no_bias or args.rot_size or args.group_size or
                    (args.matrix_path == "int8" and M > B.STREAM_MAX_TOKENS) or args.no_fp6_copy)
    table = {} if modified else traffic_table     # the stored counters belong to the unmodified configurations
    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- measured ceilings of this machine (diagnostic kernels of the library; a few milliseconds) ------
    ceilings = {}
    if with_ceilings:
        ct = max(M, 32768)                                  # enough tokens to reach the streaming asymptote
        ck = (K + 2047) // 2048 * 2048                      # the streaming kernel moves whole 2048-channel pieces
        csrc = torch.empty(ct * 2 * ck, dtype=torch.uint8, device=dev).fill_(1)
        cdst = torch.empty(ct * (ck // 2), dtype=torch.uint8, device=dev)
        cmeta = torch.empty(ct * 16, dtype=torch.uint8, device=dev)

        def stream_once(i):
            B.basq_diag_stream(csrc, cdst, cmeta, ct, ck, stream=stream)
        for i in range(3):
            stream_once(i)
        ms = timed(stream_once, 10)["mean"]
        ceilings["hbm_stream_GBps"] = ct * (2 * ck + ck // 2 + 16) / (ms * 1e-3) / 1e9
        del csrc, cdst, cmeta
        cout = torch.empty(512 * 256, dtype=torch.int32, device=dev)
        iters = 2000

        def mfma_once(i):
            B.basq_diag_mfma_i8(cout, 512, iters, stream=stream)
        mfma_once(0)
        ms = timed(mfma_once, 3)["mean"]
        ceilings["int8_mfma_TOPS"] = 512 * 4 * 8 * iters * 65536.0 / (ms * 1e-3) / 1e12
        del cout
        fout = torch.empty(512 * 256, dtype=torch.float32, device=dev)

        def mfma6_once(i):
            B.basq_diag_mfma_f6(fout, 512, iters, stream=stream)
        mfma6_once(0)
        ms = timed(mfma6_once, 3)["mean"]
        ceilings["fp6_mfma_TOPS"] = 512 * 4 * 8 * iters * 131072.0 / (ms * 1e-3) / 1e12
        del fout
    if decode and not rq_only:
        # read-only streaming over the same weight copies, launched the same way as the decode kernel: what a
        # kernel that only reads these bytes achieves at this size (a launch of a few microseconds is latency)
        views = [w.view(-1)[: w.numel() // 32768 * 32768] for w in wsets]
        rout = torch.empty(1024 * 256, dtype=torch.int32, device=dev)

        def read_once(i):
            B.basq_diag_read(views[i % len(views)], rout, 1024, stream=stream)
        if views[0].numel() > 0:
            for i in range(3):
                read_once(i)
            t_read = timed(read_once, launches)
            ceilings["hbm_read_GBps"] = views[0].numel() / (t_read["mean"] * 1e-3) / 1e9
            ceilings["hbm_read_us"] = t_read["mean"] * 1e3
        del rout

    def spread(t):
        return {"avg_kernel_ms": t["mean"], "min_kernel_ms": t["min"], "median_kernel_ms": t["median"], "launches": t["launches"]}

    # rotate+quant: priced on the method's own bytes (bf16 in, 4-bit codes and one record out); what this design
    # moves on top (the fp6 copy of the codes that its GEMM reads) is reported, not credited
    rq_bytes = algorithmic_bytes_rotate_quant(M, K, False, group)
    rq_design = algorithmic_bytes_rotate_quant(M, K, want6, group, codes4=not fp6_only)
    gemm_bytes = algorithmic_bytes_gemm(M, K, N, use_fp6)
    rq_gbs = rq_bytes / (rq_ms * 1e-3) / 1e9
    rq_kernel = ("rotate_quant_k28_kernel" if (K == 14336 and rot_size == K and group in (0, K)) else
                 "rotate_quant_pow2" if (K in (4096, 8192) and rot_size == K and group in (0, K, 128)) else
                 "rotate_quant_head_kernel" if (rot_size == 128 and group == 128 and K % 512 == 0) else
                 "rotate_quant_block_kernel" if (rot_size in (128, 256, 512) and group in (0, K) and K % 256 == 0 and
                                                 K % rot_size == 0 and K <= 16384) else "rotate_quant_generic_kernel")
    rq_traffic = traffic_of(table, config, rq_kernel)
    roof_rq = {"kernel": rq_kernel, "bound": "hbm", "achieved": rq_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
               "frac": rq_gbs / HBM_PEAK_GBS, "traffic": rq_traffic, "algorithmic_bytes": rq_bytes,
               "writes_4bit_codes": not fp6_only, "design_bytes": rq_design, "achieved_on_design_bytes": rq_design / (rq_ms * 1e-3) / 1e9,
               "traffic_over_algorithmic": (rq_traffic / rq_bytes) if rq_traffic else None, **spread(t_rq)}
    # The same kernel against the vector pipes' issue rate, which is what bounds it (one wave instruction per four
    # cycles per SIMD: packed fp32 is not used): vector instructions per launch from the tracked counter summary.
    rq_valu = traffic_of(table, config, rq_kernel, "valu_insts_per_launch")
    if rq_valu:
        ach = rq_valu / (rq_ms * 1e-3) / 1e9
        roof_rq["alu"] = {"bound": "alu", "achieved": ach, "peak": VALU_ISSUE_PEAK_G, "unit": "G wave-instructions/s",
                          "frac": ach / VALU_ISSUE_PEAK_G, "valu_insts_per_launch": rq_valu,
                          "valu_insts_per_token": rq_valu / max(M, 1)}
    if rq_only:
        roof = None
    elif decode:
        ach = gemm_bytes / (gemm_ms * 1e-3) / 1e9
        roof = {"kernel": "gemv_w4a4_kernel", "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": ach / HBM_PEAK_GBS, "traffic": traffic_of(table, config, "gemv_w4a4_kernel"),
                "algorithmic_bytes": gemm_bytes, **spread(t_gemm)}
        # the whole step as one HBM-bound pass: activations in, weights once, outputs out
        step_bytes = gemm_bytes - M * (K // 2 + 16) + 2 * M * K
        roof["step_algorithmic_bytes"] = step_bytes
        roof["step_GBps"] = step_bytes / (ms_step * 1e-3) / 1e9
        roof["step_frac"] = roof["step_GBps"] / HBM_PEAK_GBS
    else:
        ach = ops / (gemm_ms * 1e-3) / 1e12
        peak = FP6_PEAK_TOPS if (use_fp6 or g_fp6) else INT8_PEAK_TOPS
        kname = ("gemm_w4a4_fp6_kernel" if use_fp6 else
                 (("gemm_w4a4_grouped_fp6_kernel" if g_fp6 else "gemm_w4a4_grouped_kernel") if grouped else "gemm_w4a4_direct_kernel"))
        roof = {"kernel": kname, "bound": "mfma", "achieved": ach, "peak": peak, "unit": "TOP/s", "frac": ach / peak,
                "traffic": traffic_of(table, config, kname), "algorithmic_ops": ops, "algorithmic_bytes": gemm_bytes,
                **spread(t_gemm)}
        if roof["traffic"]:
            roof["traffic_over_algorithmic"] = roof["traffic"] / gemm_bytes
        if use_fp6:
            # the same product on the int8 matrix-core path (bit-identical output): the pipe the workload
            # definition prices the GEMM against
            ach8 = ops / (t_gemm8["mean"] * 1e-3) / 1e12
            roof["frac_of_int8_peak"] = ach / INT8_PEAK_TOPS
            roof["int8_path"] = {"kernel": "gemm_w4a4_direct_kernel", "achieved": ach8, "peak": INT8_PEAK_TOPS,
                                 "frac": ach8 / INT8_PEAK_TOPS, "traffic": traffic_of(table, config, "gemm_w4a4_direct_kernel"),
                                 **spread(t_gemm8)}

    if "hbm_stream_GBps" in ceilings:
        roof_rq["measured_ceiling"] = ceilings["hbm_stream_GBps"]
        roof_rq["frac_of_measured_ceiling"] = rq_gbs / ceilings["hbm_stream_GBps"]
    if roof is not None and roof["bound"] == "mfma" and "fp6_mfma_TOPS" in ceilings:
        ckey = "fp6_mfma_TOPS" if (use_fp6 or g_fp6) else "int8_mfma_TOPS"
        roof["measured_ceiling"] = ceilings[ckey]
        roof["frac_of_measured_ceiling"] = roof["achieved"] / ceilings[ckey]
        if use_fp6:
            roof["int8_path"]["measured_ceiling"] = ceilings["int8_mfma_TOPS"]
    elif roof is not None and "hbm_read_GBps" in ceilings:
        roof["measured_ceiling"] = ceilings["hbm_read_GBps"]
        roof["measured_ceiling_kind"] = ("read-only kernel over the same weight buffers, same launch path: "
                                         f"{ceilings['hbm_read_us']:.2f} us per launch (a launch this small is latency, not bandwidth)")
        roof["frac_of_measured_ceiling"] = roof["achieved"] / ceilings["hbm_read_GBps"]

    out = {
        "value": rq_gbs if rq_only else value, "unit": "GB/s" if rq_only else "TOPS",
        "ms_per_step": ms_step, "min_ms_per_step": t_step["min"], "median_ms_per_step": t_step["median"],
        "dtype": ("int4 codes as exact fp6 (e2m3) operands -> f32 accumulator == int32 (f8f6f4 MFMA)" if (use_fp6 or g_fp6) and not rq_only
                  else "int4 x int4 -> int32 (int8 MFMA)") + "; rotation and quantiser in f32; bf16 in/out",
        "config": {"workload": f"{cfg.name}: {cfg.description}", "M": M, "K": K, "N": N, "rot_size": rot_size, "group_size": group if group else K,
                   "clip": cfg.clip, "buffer_sets": nsets, "weight_copies": len(wsets),
                   "weight_layout": "streaming (16-row blocks)" if w_layout == B.BASQ_W_DECODE16 else "canonical",
                   "launch": "HIP graph replay of the K steps" if args.graph else "eager",
                   "precondition_steps": precondition,
                   "step_launches": 1 if one_launch else 2,
                   "matrix_path": "fp6" if (use_fp6 or g_fp6) else ("int4 weight streaming" if decode else "int8")},
        "rotate_quant_GBps": rq_gbs,
        "roofline": roof_rq if rq_only else roof,
        "roofline_rotate_quant": roof_rq,
    }
    if graph_note:
        out["graph"] = graph_note
    del sets, workspace, wsets, Wq, Wq6, X0
    torch.cuda.empty_cache()
    return out, cfg, M


def compact(full):
    """The few numbers of a secondary workload that go into the headline line."""
    r, q = full["roofline"], full["roofline_rotate_quant"]
    c = {"M": full["config"]["M"], "K": full["config"]["K"], "N": full["config"]["N"], "matrix_path": full["config"]["matrix_path"],
         "step_launches": full["config"]["step_launches"], "ms_per_step": full["ms_per_step"],
         "min_ms_per_step": full["min_ms_per_step"], "median_ms_per_step": full["median_ms_per_step"], "TOPS": full["value"],
         "dominant": {k: r.get(k) for k in ("kernel", "bound", "achieved", "peak", "unit", "frac", "traffic", "avg_kernel_ms",
                                            "min_kernel_ms", "median_kernel_ms", "frac_of_int8_peak", "measured_ceiling",
                                            "frac_of_measured_ceiling", "step_GBps", "step_frac") if r.get(k) is not None},
         "rotate_quant": {k: q.get(k) for k in ("kernel", "achieved", "frac", "algorithmic_bytes", "design_bytes", "traffic",
                                                "avg_kernel_ms", "min_kernel_ms", "median_kernel_ms") if q.get(k) is not None}}
    if "int8_path" in r:
        c["dominant"]["int8_path_frac_of_int8_peak"] = r["int8_path"]["frac"]
    if full.get("graph", {}).get("graph_ms_per_step") is not None:
        c["graph_ms_per_step"] = full["graph"]["graph_ms_per_step"]
    if "alu" in q:
        c["rotate_quant"]["valu_issue_frac"] = q["alu"]["frac"]
        c["rotate_quant"]["valu_insts_per_token"] = q["alu"]["valu_insts_per_token"]
    return c


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(the layer shards over tokens or output channels without communication)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2506_15689_amd import binding as B
    from paper_2506_15689_amd import synth_inputs as si

    if args.config not in si.CONFIGS:
        print(f"bench.py: unknown workload {args.config!r}; known: {', '.join(sorted(si.CONFIGS))}", file=sys.stderr)
        sys.exit(2)
    grouped = args.group_size == 128 and args.only != "rotate_quant"
    if (args.rot_size or args.group_size) and args.only != "rotate_quant" and not grouped:
        print("bench.py: --rot-size and --group-size go with --only rotate_quant (the GEMM takes per-token ranges, "
              "or groups of 128)", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    B.load()
    torch.cuda.set_device(torch.device("cuda:0"))
    table = load_traffic()

    main_fields, cfg, M = run_workload(args, args.config, args.steps, args.warmup, with_ceilings=not args.no_ceilings,
                                       traffic_table=table, M_override=args.M)
    out = {"metric": "W4A4 rotated-linear TOPS + fused rotate/quant GB/s, % of roofline, 1 MI355X",
           "value": main_fields.pop("value"), "unit": main_fields.pop("unit"), "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": main_fields.pop("ms_per_step"), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": main_fields.pop("dtype"), "data": "synthetic"}
    out.update(main_fields)
    if table.get("source"):
        out["traffic_source"] = table["source"]

    plain = (args.config == "C5" and not args.only and not args.M and not args.group_size and not args.rot_size and
             not args.no_bias and not args.graph and args.matrix_path == "fp6" and args.weight_layout == "stream")
    if plain and not args.no_other_workloads:
        others = {}
        for name in OTHER_WORKLOADS:
            # decode-sized steps last a few microseconds, about what one call costs the host: their device-side time
            # (the same steps replayed from a HIP graph) is reported beside the eager one
            full, _, _ = run_workload(args, name, max(10, min(args.steps, 50)), max(5, min(args.warmup, 10)),
                                      with_ceilings=False, traffic_table=table, also_graph=name.startswith("C3"))
            others[name] = compact(full)
        out["other_workloads"] = others

    if not args.no_cpu_baseline and not args.only and not grouped:
        # about 1.5e12 integer operations keep the oracle busy for 10-30 s on the machine's host threads; one thread
        # gets a twelfth of the sample
        sample = max(1, min(M, int(round(1.5e12 / (2.0 * cfg.N * cfg.K)))))
        base = cpu_baseline(args.config, sample)
        if "error" not in base:
            one = cpu_baseline(args.config, max(1, sample // 12), threads=1)
            base["single_thread"] = one
        out["cpu_baseline"] = base
    print(json.dumps(out))


if __name__ == "__main__":
    main()
