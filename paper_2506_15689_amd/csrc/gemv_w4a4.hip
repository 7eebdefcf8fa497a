// Decode-shaped W4A4 product (M <= 16 tokens): one pass over the packed weights, bound by HBM
// bandwidth.  Same arithmetic as the prefill GEMM (ACC in INT32, fused de-quantisation).
//
// A workgroup owns 16 output channels; its waves split K.  Each lane issues all of its 16-byte
// weight loads before it consumes any, so the whole weight matrix is in flight at once.  The
// 16 x 16 x 64 int8 MFMA takes the 16 weight rows as one operand and the (zero padded) tokens as
// the other; nibbles are split into low/high words exactly as in the prefill kernel.
//
// Weight layouts.  The MFMA operand puts 16 different rows on the 16 lanes of a quarter wave, so on
// canonical [N, K/2] weights every load instruction touches 16 rows x 64 bytes and each 128-byte line
// is fetched in eight 16-byte pieces.  The streaming layout (BASQ_W_DECODE16) stores the 1 KB a wave
// load needs contiguously, in lane order: 4 KB contiguous per workgroup step.
#include "basq_internal.h"

namespace basq {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

#ifndef GV_WAVES_CFG
#define GV_WAVES_CFG 4
#endif
constexpr int GV_WAVES = GV_WAVES_CFG;
constexpr int GV_THREADS = GV_WAVES * 64;
static_assert(GV_THREADS >= 256, "the epilogue maps one thread to each of the 16 x 16 outputs");
constexpr int GV_ROWS = 16;        // output channels per workgroup

// GV_MAX_STEPS: 64-byte k-chunks per lane held in registers at once (all of their loads are in flight together).
// TILES: 16-row tiles per workgroup; the tiles share the activation operand, so with 16 tokens (where the
// activations a workgroup reads from L2 are as many bytes as the weights of one tile) two tiles halve that traffic.
template <bool STREAM_LAYOUT, int GV_MAX_STEPS, int TILES>
__global__ __launch_bounds__(GV_THREADS) void gemv_w4a4_kernel(GemmArgs a) {
    __shared__ int part[GV_WAVES][TILES * GV_ROWS * 16];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n0 = blockIdx.x * (GV_ROWS * TILES);
    const int KB = a.K / 2;
    const int nchunks = KB / 64;               // 64-byte chunks per row (K % 128 == 0 checked by the caller)
    const int row = lane & 15, sub = lane >> 4;

    const bool t_ok = row < a.M;               // the same lane index selects the token on the other operand
    // chunk c of this lane: canonical = 16 bytes of row n at 64c + 16sub; streaming = piece `lane` of the
    // 16-row block's c-th KB (rows past N are stored as zeros there; a whole block past N does not exist)
    const uint8_t* wrow[TILES];
    bool w_ok[TILES];
#pragma unroll
    for (int t = 0; t < TILES; ++t) {
        const int nt0 = n0 + GV_ROWS * t, n = nt0 + row;
        w_ok[t] = STREAM_LAYOUT ? nt0 < a.N : n < a.N;
        wrow[t] = STREAM_LAYOUT ? a.Wq + (int64_t)(w_ok[t] ? nt0 : 0) * KB + lane * 16
                                : a.Wq + (int64_t)(w_ok[t] ? n : 0) * KB + sub * 16;
    }
    constexpr int WSTEP = STREAM_LAYOUT ? 1024 : 64;
    const uint8_t* arow = a.Aq + (int64_t)(t_ok ? row : 0) * KB + sub * 16;

    // epilogue constants of the outputs this thread will finish (16 consecutive channels of one token per
    // 16 threads, one such output per tile): requested now so that their latency overlaps the weight stream
    const int orow = tid & 15, otok = tid >> 4;
    basq_tokmeta mt = {0.f, 0.f, 0, 0};
    if (otok < a.M && otok < 16) mt = a.meta[otok];
    float sw[TILES], zp[TILES], ws[TILES], cb[TILES];
    bool out_ok[TILES];
#pragma unroll
    for (int t = 0; t < TILES; ++t) {
        const int on = n0 + GV_ROWS * t + orow;
        out_ok[t] = otok < a.M && on < a.N && otok < 16;
        sw[t] = zp[t] = ws[t] = cb[t] = 0.f;
        if (out_ok[t]) {
            sw[t] = bf16_to_f32(a.w_scale[on]);
            zp[t] = bf16_to_f32(a.w_zero[on]);
            ws[t] = a.w_sum[on];
            cb[t] = a.out_bias ? a.out_bias[on] : 0.0f;
        }
    }

    v4i acc[TILES], acc2[TILES];               // two chains per tile: low and high nibbles
#pragma unroll
    for (int t = 0; t < TILES; ++t) acc[t] = acc2[t] = v4i{0, 0, 0, 0};
    for (int c0 = wave; c0 < nchunks; c0 += GV_WAVES * GV_MAX_STEPS) {
        v4i w[TILES][GV_MAX_STEPS], x[GV_MAX_STEPS];
#pragma unroll
        for (int i = 0; i < GV_MAX_STEPS; ++i) {
            const int c = c0 + i * GV_WAVES;
            const bool ok = c < nchunks;
            // the weights are read once per call: streaming (non-temporal) loads
#pragma unroll
            for (int t = 0; t < TILES; ++t)
                w[t][i] = (ok && w_ok[t]) ? __builtin_nontemporal_load(reinterpret_cast<const v4i*>(wrow[t] + c * WSTEP))
                                          : v4i{0, 0, 0, 0};
            x[i] = (ok && t_ok) ? *reinterpret_cast<const v4i*>(arow + c * 64) : v4i{0, 0, 0, 0};
        }
#pragma unroll
        for (int i = 0; i < GV_MAX_STEPS; ++i) {
            const v4i xlo = x[i] & 0x0F0F0F0F, xhi = (x[i] >> 4) & 0x0F0F0F0F;
#pragma unroll
            for (int t = 0; t < TILES; ++t) {
                const v4i wlo = w[t][i] & 0x0F0F0F0F, whi = (w[t][i] >> 4) & 0x0F0F0F0F;
                acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wlo, xlo, acc[t], 0, 0, 0);
                acc2[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(whi, xhi, acc2[t], 0, 0, 0);
            }
        }
    }
    // accumulator register r of lane l: weight row 4*(l/16) + r, token l%16
#pragma unroll
    for (int t = 0; t < TILES; ++t) {
        acc[t] += acc2[t];
#pragma unroll
        for (int r = 0; r < 4; ++r) part[wave][t * 256 + (4 * sub + r) * 16 + row] = acc[t][r];
    }
    __syncthreads();

    if (GV_THREADS > 256 && tid >= 256) return;
#pragma unroll
    for (int t = 0; t < TILES; ++t) {
        int av = 0;
#pragma unroll
        for (int w = 0; w < GV_WAVES; ++w) av += part[w][t * 256 + orow * 16 + otok];
        if (out_ok[t]) {
            const int on = n0 + GV_ROWS * t + orow;
            const float tt = (float)av - zp[t] * (float)mt.rowsum;
            const float y = fmaf(mt.scale * sw[t], tt, fmaf(mt.lo, ws[t], cb[t]));
            a.Y[(int64_t)otok * a.ldy + on] = f32_to_bf16(y);
            if (a.acc_out) a.acc_out[(int64_t)otok * a.N + on] = av;
        }
    }
}

// canonical [N, K/2] -> streaming layout: one thread per 16-byte piece of the output
__global__ __launch_bounds__(256) void pack_decode16_kernel(const uint8_t* __restrict__ Wq, int N, int KB,
                                                            uint8_t* __restrict__ out, int64_t pieces) {
    const int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (p >= pieces) return;
    const int nchunks = KB / 64;
    const int ln = (int)(p & 63);
    const int64_t kb = p >> 6;                       // (block, chunk)
    const int c = (int)(kb % nchunks);
    const int64_t n = (kb / nchunks) * 16 + (ln & 15);
    uint4 v = make_uint4(0, 0, 0, 0);
    if (n < N) v = *reinterpret_cast<const uint4*>(Wq + n * KB + 64 * c + 16 * (ln >> 4));
    *reinterpret_cast<uint4*>(out + p * 16) = v;
}

}  // namespace

int launch_pack_decode16(const uint8_t* Wq, int32_t N, int32_t K, uint8_t* out, hipStream_t s) {
    const int KB = K / 2;
    const int64_t pieces = (int64_t)((N + 15) / 16) * (KB / 64) * 64;
    const int64_t blocks = (pieces + 255) / 256;
    if (blocks > 0x7FFFFFFFll) return fail(BASQ_EINVAL, "pack_decode: matrix too large");
    hipLaunchKernelGGL(pack_decode16_kernel, dim3((unsigned)blocks), dim3(256), 0, s, Wq, N, KB, out, pieces);
    return check_hip(hipGetLastError(), "pack_decode launch");
}

template <bool SL>
static void launch_gemv_layout(const GemmArgs& a, hipStream_t s) {
    const int blocks16 = (a.N + GV_ROWS - 1) / GV_ROWS;
    // long rows: twice the loads in flight per lane (measured: K = 8192 gains 6 %, K = 4096 loses 5 %)
    const bool deep = a.K / 128 > 32 * GV_WAVES / 4;
    // two tiles per workgroup once the activations weigh in (more than 8 tokens) and the chip stays filled
    const bool two = a.M > 8 && blocks16 >= 4 * 256;
    if (two)
        hipLaunchKernelGGL((gemv_w4a4_kernel<SL, 8, 2>), dim3((unsigned)((blocks16 + 1) / 2)), dim3(GV_THREADS), 0, s, a);
    else if (deep)
        hipLaunchKernelGGL((gemv_w4a4_kernel<SL, 16, 1>), dim3((unsigned)blocks16), dim3(GV_THREADS), 0, s, a);
    else
        hipLaunchKernelGGL((gemv_w4a4_kernel<SL, 8, 1>), dim3((unsigned)blocks16), dim3(GV_THREADS), 0, s, a);
}

int launch_gemv_decode(const GemmArgs& a, hipStream_t s) {
    if (a.M == 0) return BASQ_OK;
    if (a.w_layout == BASQ_W_DECODE16) launch_gemv_layout<true>(a, s);
    else launch_gemv_layout<false>(a, s);
    return check_hip(hipGetLastError(), "w4a4_gemv launch");
}

}  // namespace basq
