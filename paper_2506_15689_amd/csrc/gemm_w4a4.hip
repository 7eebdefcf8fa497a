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
//
// Tiling: a workgroup of 4 waves owns a BM x BN tile of Y, each wave a (BM/WAVES_M) x (BN/WAVES_N)
// sub-tile made of 32 x 32 MFMA tiles; K advances 256 codes (128 packed bytes per row) per step
// through a double-buffered LDS stage.  Workgroup ids are remapped so that the workgroups running
// on one XCD (ids congruent mod 8) cover a compact patch of tiles and share their operands in
// that XCD's L2.
#include "basq_internal.h"

namespace basq {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BK_BYTES = 128;                 // packed bytes of K per row per main-loop step (256 codes): one full cache line
constexpr int LDS_ROW = BK_BYTES + 16;        // padded row stride: 16-byte reads of 8 consecutive rows hit distinct banks
constexpr int CHUNKS = BK_BYTES / 16;         // 16-byte chunks per row per step
constexpr int NUM_XCD = 8;

template <int BM, int BN, int WAVES_M, int WAVES_N, bool KTAIL>
__global__ __launch_bounds__(WAVES_M * WAVES_N * 64) void gemm_w4a4_kernel(GemmArgs a, int tiles_m, int tiles_n) {
    constexpr int THREADS = WAVES_M * WAVES_N * 64;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;     // wave tile
    constexpr int TM = WM / 32, TN = WN / 32;               // 32x32 MFMA tiles per wave
    constexpr int A_CHUNKS = BM * CHUNKS;                   // 16-byte chunks per stage
    constexpr int B_CHUNKS = BN * CHUNKS;
    static_assert(A_CHUNKS % THREADS == 0 && B_CHUNKS % THREADS == 0, "tile/threads mismatch");
    constexpr int A_PER_T = A_CHUNKS / THREADS;
    constexpr int B_PER_T = B_CHUNKS / THREADS;
    constexpr int STAGE_BYTES = (BM + BN) * LDS_ROW;

    __shared__ __attribute__((aligned(16))) uint8_t lds[2 * STAGE_BYTES];

    // ---- tile assignment: consecutive ids on one XCD walk a band of GROUP_M tile rows column by column
    int tile_m, tile_n;
    {
        const int total = tiles_m * tiles_n;
        const int pid = blockIdx.x;
        int t = pid;
        const int per_xcd = total / NUM_XCD;
        if (pid < per_xcd * NUM_XCD) t = (pid % NUM_XCD) * per_xcd + pid / NUM_XCD;   // the tail keeps its id
        constexpr int GROUP_M = 4;
        const int band = t / (GROUP_M * tiles_n);
        const int first_m = band * GROUP_M;
        const int rows = (tiles_m - first_m) < GROUP_M ? (tiles_m - first_m) : GROUP_M;
        const int in_band = t - band * GROUP_M * tiles_n;
        tile_m = first_m + in_band % rows;
        tile_n = in_band / rows;
    }

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int64_t m0 = (int64_t)tile_m * BM;
    const int n0 = tile_n * BN;
    const int KB = a.K / 2;                                  // packed bytes per row
    const int ksteps = (KB + BK_BYTES - 1) / BK_BYTES;

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // global -> register staging.  Thread t moves 16-byte chunk t % CHUNKS of rows t/CHUNKS + i*THREADS/CHUNKS.  Rows
    // past the end of the matrix are clamped to the last row (their results are never stored); a K
    // tail (K % 128 != 0, KTAIL kernels only) is filled with zeros.
    constexpr int ROWS_PER_PASS = THREADS / CHUNKS;
    const int lrow = tid / CHUNKS, lchunk = tid % CHUNKS;
    uint4 ra[A_PER_T], rb[B_PER_T];
    auto load_global = [&](int ks) {
        const int kbyte = ks * BK_BYTES + lchunk * 16;
        const bool kok = !KTAIL || kbyte < KB;
#pragma unroll
        for (int i = 0; i < A_PER_T; ++i) {
            int64_t m = m0 + lrow + i * ROWS_PER_PASS;
            m = m < a.M ? m : a.M - 1;
            ra[i] = kok ? *reinterpret_cast<const uint4*>(a.Aq + m * KB + kbyte) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < B_PER_T; ++i) {
            int n = n0 + lrow + i * ROWS_PER_PASS;
            n = n < a.N ? n : a.N - 1;
            rb[i] = kok ? *reinterpret_cast<const uint4*>(a.Wq + (int64_t)n * KB + kbyte) : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_lds = [&](int buf) {
        uint8_t* la = lds + buf * STAGE_BYTES + lrow * LDS_ROW + lchunk * 16;
        uint8_t* lb = la + BM * LDS_ROW;
#pragma unroll
        for (int i = 0; i < A_PER_T; ++i) *reinterpret_cast<uint4*>(la + i * ROWS_PER_PASS * LDS_ROW) = ra[i];
#pragma unroll
        for (int i = 0; i < B_PER_T; ++i) *reinterpret_cast<uint4*>(lb + i * ROWS_PER_PASS * LDS_ROW) = rb[i];
    };

    const int frow = lane & 31, fhalf = lane >> 5;
    const int a_off = (wm * WM + frow) * LDS_ROW + fhalf * 16;
    const int b_off = BM * LDS_ROW + (wn * WN + frow) * LDS_ROW + fhalf * 16;

    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int ks = 0; ks < ksteps; ++ks) {
        const int buf = ks & 1;
        if (ks + 1 < ksteps) load_global(ks + 1);            // in flight while this step computes

        const uint8_t* st = lds + buf * STAGE_BYTES;
#pragma unroll
        for (int h = 0; h < CHUNKS / 2; ++h) {
            v4i alo[TM], ahi[TM];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const v4i x = *reinterpret_cast<const v4i*>(st + a_off + i * 32 * LDS_ROW + h * 32);
                alo[i] = x & 0x0F0F0F0F;
                ahi[i] = (x >> 4) & 0x0F0F0F0F;
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const v4i x = *reinterpret_cast<const v4i*>(st + b_off + j * 32 * LDS_ROW + h * 32);
                const v4i blo = x & 0x0F0F0F0F;
                const v4i bhi = (x >> 4) & 0x0F0F0F0F;
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(alo[i], blo, acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ahi[i], bhi, acc[i][j], 0, 0, 0);
                }
            }
        }
        if (ks + 1 < ksteps) store_lds(buf ^ 1);             // the other buffer was last read one step ago
        __syncthreads();
    }

    // ---- epilogue --------------------------------------------------------------------------------
    // The per-row (token) and per-column (channel) constants of this tile go through LDS, which the
    // main loop no longer needs: row -> (s_m, lo_m, rowsum_m), column -> (sw_n, zp_n, wsum_n, c_n).
    float4* lrow_par = reinterpret_cast<float4*>(lds);
    float4* lcol_par = lrow_par + BM;
    for (int i = tid; i < BM; i += THREADS) {
        int64_t m = m0 + i;
        m = m < a.M ? m : a.M - 1;
        const basq_tokmeta mt = a.meta[m];
        lrow_par[i] = make_float4(mt.scale, mt.lo, (float)mt.rowsum, 0.0f);
    }
    for (int i = tid; i < BN; i += THREADS) {
        int n = n0 + i;
        n = n < a.N ? n : a.N - 1;
        lcol_par[i] = make_float4(bf16_to_f32(a.w_scale[n]), bf16_to_f32(a.w_zero[n]), a.w_sum[n],
                                  a.out_bias ? a.out_bias[n] : 0.0f);
    }
    __syncthreads();

    // accumulator register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32 of its 32x32 tile
    const int col_in_tile = lane & 31, rgrp = lane >> 5;
    float4 cp[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) cp[j] = lcol_par[wn * WN + j * 32 + col_in_tile];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = wm * WM + i * 32 + 8 * (r >> 2) + 4 * rgrp + (r & 3);
            const int64_t m = m0 + row;
            if (m >= a.M) continue;
            const float4 rp = lrow_par[row];
            uint16_t* yrow = a.Y + m * a.ldy;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int n = n0 + wn * WN + j * 32 + col_in_tile;
                if (n < a.N) {
                    const int av = acc[i][j][r];
                    const float t = (float)av - cp[j].y * rp.z;
                    const float y = fmaf(rp.x * cp[j].x, t, fmaf(rp.y, cp[j].z, cp[j].w));
                    yrow[n] = f32_to_bf16(y);
                    if (a.acc_out) a.acc_out[m * (int64_t)a.N + n] = av;
                }
            }
        }
    }
}

template <int BM, int BN, int WAVES_M, int WAVES_N>
int launch_tile(const GemmArgs& a, hipStream_t s) {
    const int64_t tm = (a.M + BM - 1) / BM;
    const int64_t tn = ((int64_t)a.N + BN - 1) / BN;
    if (tm * tn > 0x7FFFFFFFll) return fail(BASQ_EINVAL, "w4a4_gemm: problem too large for one launch");
    if (a.K % (2 * BK_BYTES) == 0)
        hipLaunchKernelGGL((gemm_w4a4_kernel<BM, BN, WAVES_M, WAVES_N, false>), dim3((unsigned)(tm * tn)),
                           dim3(WAVES_M * WAVES_N * 64), 0, s, a, (int)tm, (int)tn);
    else
        hipLaunchKernelGGL((gemm_w4a4_kernel<BM, BN, WAVES_M, WAVES_N, true>), dim3((unsigned)(tm * tn)),
                           dim3(WAVES_M * WAVES_N * 64), 0, s, a, (int)tm, (int)tn);
    return check_hip(hipGetLastError(), "w4a4_gemm launch");
}

}  // namespace

int launch_gemm_prefill(const GemmArgs& a, hipStream_t s) {
    if (a.M == 0) return BASQ_OK;
#ifndef GEMM_NO_DIRECT
    if (gemm_direct_applicable(a)) return launch_gemm_direct(a, s);
#endif
#ifdef GEMM_FORCE_TILE
    return launch_tile<GEMM_FORCE_TILE>(a, s);
#else
    // pick the largest tile that still gives every CU work (256 CUs)
    const int64_t t256 = ((a.M + 255) / 256) * (((int64_t)a.N + 255) / 256);
    const int64_t t256x128 = ((a.M + 255) / 256) * (((int64_t)a.N + 127) / 128);
    if (t256 >= 512) return launch_tile<256, 256, 2, 2>(a, s);
    if (t256x128 >= 512) return launch_tile<256, 128, 2, 2>(a, s);
    return launch_tile<128, 128, 2, 2>(a, s);
#endif
}

}  // namespace basq
