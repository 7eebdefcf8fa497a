// Decode-shaped W4A4 product (M <= 16 tokens): one pass over the packed weights, bound by HBM
// bandwidth.  Same arithmetic as the prefill GEMM (ACC in INT32, fused de-quantisation).
//
// A workgroup owns 16 output channels; its waves split K.  Each lane issues all of its 16-byte
// weight loads before it consumes any, so the whole weight matrix is in flight at once.  The
// 16 x 16 x 64 int8 MFMA takes the 16 weight rows as one operand and the (zero padded) tokens as
// the other; nibbles are split into low/high words exactly as in the prefill kernel.
#include "basq_internal.h"

namespace basq {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

#ifndef GV_WAVES_CFG
#define GV_WAVES_CFG 4
#endif
#ifndef GV_STEPS_CFG
#define GV_STEPS_CFG 8
#endif
constexpr int GV_WAVES = GV_WAVES_CFG;
constexpr int GV_THREADS = GV_WAVES * 64;
static_assert(GV_THREADS >= 256, "the epilogue maps one thread to each of the 16 x 16 outputs");
constexpr int GV_ROWS = 16;        // output channels per workgroup
constexpr int GV_MAX_STEPS = GV_STEPS_CFG;    // 64-byte k-chunks per wave held in registers at once

__global__ __launch_bounds__(GV_THREADS) void gemv_w4a4_kernel(GemmArgs a) {
    __shared__ int part[GV_WAVES][GV_ROWS * 16];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n0 = blockIdx.x * GV_ROWS;
    const int KB = a.K / 2;
    const int nchunks = KB / 64;               // 64-byte chunks per row (K % 128 == 0 checked by the caller)
    const int row = lane & 15, sub = lane >> 4;

    const int n = n0 + row;
    const bool n_ok = n < a.N;
    const bool t_ok = row < a.M;               // the same lane index selects the token on the other operand
    const uint8_t* wrow = a.Wq + (int64_t)(n_ok ? n : 0) * KB + sub * 16;
    const uint8_t* arow = a.Aq + (int64_t)(t_ok ? row : 0) * KB + sub * 16;

    // epilogue constants of the output this thread will finish (16 consecutive channels of one token per
    // 16 threads): requested now so that their latency overlaps the weight stream
    const int orow = tid & 15, otok = tid >> 4;
    const int on = n0 + orow;
    const bool out_ok = otok < a.M && on < a.N && otok < 16;
    basq_tokmeta mt = {0.f, 0.f, 0, 0};
    float sw = 0.f, zp = 0.f, ws = 0.f, cb = 0.f;
    if (out_ok) {
        mt = a.meta[otok];
        sw = bf16_to_f32(a.w_scale[on]);
        zp = bf16_to_f32(a.w_zero[on]);
        ws = a.w_sum[on];
        cb = a.out_bias ? a.out_bias[on] : 0.0f;
    }

    v4i acc = {0, 0, 0, 0};
    for (int c0 = wave; c0 < nchunks; c0 += GV_WAVES * GV_MAX_STEPS) {
        v4i w[GV_MAX_STEPS], x[GV_MAX_STEPS];
#pragma unroll
        for (int i = 0; i < GV_MAX_STEPS; ++i) {
            const int c = c0 + i * GV_WAVES;
            const bool ok = c < nchunks;
            w[i] = (ok && n_ok) ? *reinterpret_cast<const v4i*>(wrow + c * 64) : v4i{0, 0, 0, 0};
            x[i] = (ok && t_ok) ? *reinterpret_cast<const v4i*>(arow + c * 64) : v4i{0, 0, 0, 0};
        }
#pragma unroll
        for (int i = 0; i < GV_MAX_STEPS; ++i) {
            const v4i wlo = w[i] & 0x0F0F0F0F, whi = (w[i] >> 4) & 0x0F0F0F0F;
            const v4i xlo = x[i] & 0x0F0F0F0F, xhi = (x[i] >> 4) & 0x0F0F0F0F;
            acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(wlo, xlo, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(whi, xhi, acc, 0, 0, 0);
        }
    }
    // accumulator register r of lane l: weight row 4*(l/16) + r, token l%16
#pragma unroll
    for (int r = 0; r < 4; ++r) part[wave][(4 * sub + r) * 16 + row] = acc[r];
    __syncthreads();

    if (GV_THREADS > 256 && tid >= 256) return;
    int av = 0;
#pragma unroll
    for (int w = 0; w < GV_WAVES; ++w) av += part[w][orow * 16 + otok];
    if (out_ok) {
        const float t = (float)av - zp * (float)mt.rowsum;
        const float y = fmaf(mt.scale * sw, t, fmaf(mt.lo, ws, cb));
        a.Y[(int64_t)otok * a.ldy + on] = f32_to_bf16(y);
        if (a.acc_out) a.acc_out[(int64_t)otok * a.N + on] = av;
    }
}

}  // namespace

int launch_gemv_decode(const GemmArgs& a, hipStream_t s) {
    if (a.M == 0) return BASQ_OK;
    const unsigned blocks = (unsigned)((a.N + GV_ROWS - 1) / GV_ROWS);
    hipLaunchKernelGGL(gemv_w4a4_kernel, dim3(blocks), dim3(GV_THREADS), 0, s, a);
    return check_hip(hipGetLastError(), "w4a4_gemv launch");
}

}  // namespace basq
