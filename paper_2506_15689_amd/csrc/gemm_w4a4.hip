// INT4 x INT4 -> INT32 GEMM on the CDNA4 int8 matrix cores with the de-quantisation fused into
// the epilogue (paper Sec. 5.2: 4-bit matrix multiplication; Fig. 6: de-quantisation fused with
// the bias; Eq. 14: fused bias).
//
//   ACC[m,n] = sum_k q_a[m,k] q_w[n,k]
//   Y[m,n]   = bf16( s_m sw_n (ACC - zp_n rowsum_m) + lo_m wsum_n + c_n )
//
// Both operands stay packed (two codes per byte) in HBM and in LDS; a wave unpacks its fragments
// in registers with   lo = x & 0x0F0F0F0F,  hi = (x >> 4) & 0x0F0F0F0F.   The low-nibble and the
// high-nibble words feed two separate MFMAs; A and B use the same split, so each MFMA contracts
// over the same set of k on both sides and the sum over all MFMAs is the full dot product.
#include "basq_internal.h"

namespace basq {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BK_BYTES = 64;                  // packed bytes of K per row per main-loop step (128 codes)
constexpr int LDS_ROW = BK_BYTES + 16;        // padded row stride in LDS

template <int BM, int BN, int WAVES_M, int WAVES_N>
__global__ __launch_bounds__(WAVES_M * WAVES_N * 64) void gemm_w4a4_kernel(GemmArgs a) {
    constexpr int THREADS = WAVES_M * WAVES_N * 64;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;     // wave tile
    constexpr int TM = WM / 32, TN = WN / 32;               // 32x32 MFMA tiles per wave
    constexpr int A_CHUNKS = BM * (BK_BYTES / 16);          // 16-byte chunks per stage
    constexpr int B_CHUNKS = BN * (BK_BYTES / 16);
    constexpr int A_PER_T = (A_CHUNKS + THREADS - 1) / THREADS;
    constexpr int B_PER_T = (B_CHUNKS + THREADS - 1) / THREADS;
    static_assert(A_CHUNKS % THREADS == 0 && B_CHUNKS % THREADS == 0, "tile/threads mismatch");

    __shared__ __attribute__((aligned(16))) uint8_t lds_a[BM * LDS_ROW];
    __shared__ __attribute__((aligned(16))) uint8_t lds_b[BN * LDS_ROW];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int64_t m0 = (int64_t)blockIdx.y * BM;
    const int n0 = blockIdx.x * BN;
    const int KB = a.K / 2;                                  // packed bytes per row
    const int ksteps = (KB + BK_BYTES - 1) / BK_BYTES;

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    uint4 ra[A_PER_T], rb[B_PER_T];
    auto load_global = [&](int ks) {
#pragma unroll
        for (int i = 0; i < A_PER_T; ++i) {
            const int id = tid + i * THREADS;
            const int row = id >> 2, c = id & 3;
            const int kbyte = ks * BK_BYTES + c * 16;
            const int64_t m = m0 + row;
            ra[i] = (m < a.M && kbyte < KB) ? *reinterpret_cast<const uint4*>(a.Aq + m * KB + kbyte)
                                            : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < B_PER_T; ++i) {
            const int id = tid + i * THREADS;
            const int row = id >> 2, c = id & 3;
            const int kbyte = ks * BK_BYTES + c * 16;
            const int n = n0 + row;
            rb[i] = (n < a.N && kbyte < KB) ? *reinterpret_cast<const uint4*>(a.Wq + (int64_t)n * KB + kbyte)
                                            : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_lds = [&]() {
#pragma unroll
        for (int i = 0; i < A_PER_T; ++i) {
            const int id = tid + i * THREADS;
            *reinterpret_cast<uint4*>(lds_a + (id >> 2) * LDS_ROW + (id & 3) * 16) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < B_PER_T; ++i) {
            const int id = tid + i * THREADS;
            *reinterpret_cast<uint4*>(lds_b + (id >> 2) * LDS_ROW + (id & 3) * 16) = rb[i];
        }
    };

    load_global(0);
    for (int ks = 0; ks < ksteps; ++ks) {
        __syncthreads();                 // previous step's fragment reads are done
        store_lds();
        __syncthreads();
        if (ks + 1 < ksteps) load_global(ks + 1);

        const int frow = lane & 31, fhalf = lane >> 5;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int coff = (fhalf + 2 * h) * 16;
            v4i alo[TM], ahi[TM], blo[TN], bhi[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const v4i x = *reinterpret_cast<const v4i*>(lds_a + (wm * WM + i * 32 + frow) * LDS_ROW + coff);
                alo[i] = x & 0x0F0F0F0F;
                ahi[i] = (x >> 4) & 0x0F0F0F0F;
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const v4i x = *reinterpret_cast<const v4i*>(lds_b + (wn * WN + j * 32 + frow) * LDS_ROW + coff);
                blo[j] = x & 0x0F0F0F0F;
                bhi[j] = (x >> 4) & 0x0F0F0F0F;
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(alo[i], blo[j], acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ahi[i], bhi[j], acc[i][j], 0, 0, 0);
                }
        }
    }

    // epilogue: accumulator register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32
    const int col_in_tile = lane & 31, rgrp = lane >> 5;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = n0 + wn * WN + j * 32 + col_in_tile;
        const bool n_ok = n < a.N;
        const float sw = n_ok ? bf16_to_f32(a.w_scale[n]) : 0.0f;
        const float zp = n_ok ? bf16_to_f32(a.w_zero[n]) : 0.0f;
        const float ws = n_ok ? a.w_sum[n] : 0.0f;
        const float cb = (n_ok && a.out_bias) ? a.out_bias[n] : 0.0f;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t m = m0 + wm * WM + i * 32 + 8 * (r >> 2) + 4 * rgrp + (r & 3);
                if (m < a.M && n_ok) {
                    const basq_tokmeta mt = a.meta[m];
                    const int av = acc[i][j][r];
                    const float t = (float)av - zp * (float)mt.rowsum;
                    const float y = fmaf(mt.scale * sw, t, fmaf(mt.lo, ws, cb));
                    a.Y[m * a.ldy + n] = f32_to_bf16(y);
                    if (a.acc_out) a.acc_out[m * (int64_t)a.N + n] = av;
                }
            }
        }
    }
}

}  // namespace

int launch_gemm_prefill(const GemmArgs& a, hipStream_t s) {
    if (a.M == 0) return BASQ_OK;
    constexpr int BM = 128, BN = 128;
    const int64_t gy = (a.M + BM - 1) / BM;
    const int64_t gx = ((int64_t)a.N + BN - 1) / BN;
    if (gy > 65535) return fail(BASQ_EINVAL, "w4a4_gemm: M too large for one launch (%lld)", (long long)a.M);
    hipLaunchKernelGGL((gemm_w4a4_kernel<BM, BN, 2, 2>), dim3((unsigned)gx, (unsigned)gy), dim3(256), 0, s, a);
    return check_hip(hipGetLastError(), "w4a4_gemm launch");
}

}  // namespace basq
