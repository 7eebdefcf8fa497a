// INT4 x INT4 GEMM for activations quantised in groups of 128 channels (every group of a token has its own
// step s_mg and lower bound z_mg; Eq. 4 applied per group -- the "group / per-token granularity" argument of the
// workload; the paper itself quantises per token, Sec. 5).  With x_hat = s_mg q_a + z_mg and W_hat = sw_n (q_w - zp_n):
//
//     Y[m,n] = sw_n * ( sum_g ( s_mg ACC_g[m,n] + z_mg colsum_g[n] ) - zp_n * R_m ) + c_n
//     ACC_g  = sum over the 128 channels of group g of q_a q_w            (INT32, exact)
//     R_m    = sum_g ( s_mg rowsum_mg + 128 z_mg )
//
// One LDS stage holds exactly one group (64 packed bytes per row), so a group's integer accumulator closes with
// the stage: it is scaled into an fp32 accumulator (convert, two multiply-adds per element) and starts again
// from zero.  On this chip fp32 vector multiply-adds do not run alongside MFMAs (a probe: 16 of them per
// int8 MFMA halve the MFMA rate, 16 integer instructions cost nothing), so a group costs its MFMA time
// plus its scaling time, and wave tiles are 64 x 64 (an integer and an fp32 accumulator set must fit the
// registers).  Running the two waves of a SIMD in opposite phases, or interleaving the scaling of group g-1 with
// the MFMAs of group g, was measured and is no faster for that reason.  This is the path for callers without the
// fp6 operand forms; with them gemm_w4a4_grouped_fp6.hip computes the same bits in three quarters of the time.
// Operands and the per-group constants (128 token records, 128 column sums) arrive by direct-to-LDS loads.
#include "basq_internal.h"

namespace basq {

namespace {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

#define GG_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

constexpr int GG_BM = 128, GG_BN = 128;
constexpr int GG_WAVES_M = 2, GG_WAVES_N = 2, GG_WAVES = 4, GG_THREADS = 256;
constexpr int GG_WM = 64, GG_WN = 64, GG_TM = 2, GG_TN = 2;
constexpr int GG_BKB = 64;                                    // packed bytes of K per row per stage = one group
constexpr int GG_NCH = 4;                                     // 16-byte chunks per row per stage
constexpr int GG_STAGES = 3;                                  // operand ring
constexpr int GG_OP_BYTES = (GG_BM + GG_BN) * GG_BKB;         // 16 KB per stage
constexpr int GG_LOADS = (GG_BM + GG_BN) * GG_NCH / GG_THREADS;   // operand loads per thread per stage
constexpr int GG_PSLOTS = 4;                                  // ring of per-group constants; one slot more than the
                                                              // operand ring because they are read after the MFMAs
constexpr int GG_PSLOT_BYTES = 3072;                          // 128 records of 16 B, then 128 column sums of 4 B
constexpr int GG_NUM_XCD = 8;

// Wait until at most N of this wave's direct-to-LDS loads are outstanding and its own LDS reads have returned,
// then join the workgroup barrier (one asm block: the compiler's own barrier would wait for every load).
template <int N>
__device__ __forceinline__ void gg_wait_loads_and_barrier() {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

__global__ __launch_bounds__(GG_THREADS, 2) void gemm_w4a4_grouped_kernel(GemmArgs a, const int32_t* w_gsum, int tiles_m, int tiles_n) {
#if defined(__HIP_DEVICE_COMPILE__)   // the body uses device-only buffer-resource types; the host pass only needs the stub
    __shared__ __attribute__((aligned(1024))) uint8_t lds[GG_STAGES * GG_OP_BYTES + GG_PSLOTS * GG_PSLOT_BYTES];
    uint8_t* const pring = lds + GG_STAGES * GG_OP_BYTES;

    // ---- tile assignment (ids congruent mod 8 run on one XCD and walk a compact band)
    int tile_m, tile_n;
    {
        const int total = tiles_m * tiles_n;
        const int pid = blockIdx.x;
        int t = pid;
        const int per_xcd = total / GG_NUM_XCD;
        if (pid < per_xcd * GG_NUM_XCD) t = (pid % GG_NUM_XCD) * per_xcd + pid / GG_NUM_XCD;
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
    const int wm = wave / GG_WAVES_N, wn = wave % GG_WAVES_N;
    const int64_t m0 = (int64_t)tile_m * GG_BM;
    const int n0 = tile_n * GG_BN;
    const int KB = a.K / 2;
    const int ngroups = KB / GG_BKB;

    // ---- direct loads.  Operand load i of wave w fills LDS chunks [(i*4 + w)*64, +64) of a stage; the lane picks
    // the global chunk whose swizzled position is its LDS slot.  One more load per wave brings the group's
    // constants: waves 0, 1 the token records of rows 64w + lane, waves 2, 3 the column sums of columns
    // 64(w-2) + lane.  Rows and columns past the matrix are clamped to the last one.
    constexpr int A_LOADS = GG_BM * GG_NCH / (64 * GG_WAVES);
    const int swave = __builtin_amdgcn_readfirstlane(wave);
    const __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(a.Aq), 0, (int)(a.M * KB), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(a.Wq), 0, (int)((int64_t)a.N * KB), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_m = __builtin_amdgcn_make_buffer_rsrc(const_cast<basq_tokmeta*>(a.meta), 0, (int)(a.M * ngroups * 16), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_c = __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t*>(w_gsum), 0, (int)((int64_t)ngroups * a.N * 4), 0x00020000);
    int voff[GG_LOADS];
#pragma unroll
    for (int i = 0; i < GG_LOADS; ++i) {
        const int L = (i * GG_WAVES + wave) * 64 + lane;
        const int row = L / GG_NCH, cpos = L % GG_NCH;
        const int c = cpos ^ ((row >> 2) & 3);                  // 16 consecutive rows hit 16 distinct 16-byte bank groups
        if (i < A_LOADS) {
            int64_t m = m0 + row;
            m = m < a.M ? m : a.M - 1;
            voff[i] = (int)(m * KB + c * 16);
        } else {
            int n = n0 + row - GG_BM;
            n = n < a.N ? n : a.N - 1;
            voff[i] = (int)((int64_t)n * KB + c * 16);
        }
    }
    int pvoff;
    if (swave < 2) {
        int64_t m = m0 + 64 * swave + lane;
        m = m < a.M ? m : a.M - 1;
        pvoff = (int)(m * ngroups * 16);
    } else {
        int n = n0 + 64 * (swave - 2) + lane;
        n = n < a.N ? n : a.N - 1;
        pvoff = n * 4;
    }
    auto issue_loads = [&](int g) {
        uint8_t* stage = lds + (g % GG_STAGES) * GG_OP_BYTES + swave * 1024;
        const int koff = g * GG_BKB;
#pragma unroll
        for (int i = 0; i < GG_LOADS; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(i < A_LOADS ? rsrc_a : rsrc_w, GG_LDS_PTR(stage + i * GG_WAVES * 1024), 16,
                                                     voff[i], koff, 0, 0);
        uint8_t* slot = pring + (g % GG_PSLOTS) * GG_PSLOT_BYTES;
        if (swave < 2)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_m, GG_LDS_PTR(slot + swave * 1024), 16, pvoff, g * 16, 0, 0);
        else
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_c, GG_LDS_PTR(slot + 2048 + (swave - 2) * 256), 4, pvoff, g * a.N * 4, 0, 0);
    };
    constexpr int VM_PER_STAGE = GG_LOADS + 1;

    // ---- fragment addressing: lane (frow, fhalf) reads chunk fhalf + 2h of its row, swizzled
    const int frow = lane & 31, fhalf = lane >> 5;
    const int fswz = (frow >> 2) & 3;
    int foff[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) foff[h] = (((fhalf + 2 * h) ^ fswz) << 4);
    const int a_row = (wm * GG_WM + frow) * GG_BKB;
    const int b_row = (GG_BM + wn * GG_WN + frow) * GG_BKB;
    const int col_in_tile = lane & 31, rgrp = lane >> 5;

    float facc[GG_TM][GG_TN][16];
#pragma unroll
    for (int i = 0; i < GG_TM; ++i)
#pragma unroll
        for (int j = 0; j < GG_TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) facc[i][j][r] = 0.0f;

    // ---- prologue: fill two stages
    issue_loads(0);
    if (ngroups > 1) { issue_loads(1); gg_wait_loads_and_barrier<VM_PER_STAGE>(); } else { gg_wait_loads_and_barrier<0>(); }

    for (int g = 0; g < ngroups; ++g) {
        const uint8_t* st = lds + (g % GG_STAGES) * GG_OP_BYTES;
        // the operand stage refilled now was read during step g-1 and every wave has passed that step's barrier;
        // the constants slot refilled now was read at the end of step g-2, before its reader reached step g-1's barrier
        if (g + 2 < ngroups) issue_loads(g + 2);
        v4i pa[2][GG_TM], pb[2][GG_TN];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
#pragma unroll
            for (int i = 0; i < GG_TM; ++i) pa[h][i] = *reinterpret_cast<const v4i*>(st + a_row + i * 32 * GG_BKB + foff[h]);
#pragma unroll
            for (int j = 0; j < GG_TN; ++j) pb[h][j] = *reinterpret_cast<const v4i*>(st + b_row + j * 32 * GG_BKB + foff[h]);
        }
        // the group's integer accumulators start from zero
        v16i acc[GG_TM][GG_TN];
        const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            v4i alo[GG_TM], ahi[GG_TM];
#pragma unroll
            for (int i = 0; i < GG_TM; ++i) { alo[i] = pa[h][i] & 0x0F0F0F0F; ahi[i] = (pa[h][i] >> 4) & 0x0F0F0F0F; }
#pragma unroll
            for (int j = 0; j < GG_TN; ++j) {
                const v4i blo = pb[h][j] & 0x0F0F0F0F, bhi = (pb[h][j] >> 4) & 0x0F0F0F0F;
#pragma unroll
                for (int i = 0; i < GG_TM; ++i) {
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(alo[i], blo, h == 0 ? zero : acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ahi[i], bhi, acc[i][j], 0, 0, 0);
                }
            }
        }
        // every read of this operand stage has been issued and consumed: pass the barrier that also makes the
        // next stage (and its constants) visible
        if (g + 1 < ngroups) {
            if (g + 2 < ngroups) gg_wait_loads_and_barrier<VM_PER_STAGE>(); else gg_wait_loads_and_barrier<0>();
        }
        // ---- close the group: F += s_mg * ACC_g + z_mg * colsum_g
        const uint8_t* slot = pring + (g % GG_PSLOTS) * GG_PSLOT_BYTES;
        float cs[GG_TN];
#pragma unroll
        for (int j = 0; j < GG_TN; ++j)
            cs[j] = (float)*reinterpret_cast<const int*>(slot + 2048 + (wn * GG_WN + j * 32 + col_in_tile) * 4);
#pragma unroll
        for (int i = 0; i < GG_TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int rloc = 8 * (r >> 2) + 4 * rgrp + (r & 3);
                // read as integers: the compiler puts a wait for every outstanding direct-to-LDS load in front of a
                // float-typed LDS read, which would drain the ring in every step
                const v2i szb = *reinterpret_cast<const v2i*>(slot + (wm * GG_WM + i * 32 + rloc) * 16);   // scale, lo
                const float sc = __int_as_float(szb[0]), lo = __int_as_float(szb[1]);
#pragma unroll
                for (int j = 0; j < GG_TN; ++j)
                    facc[i][j][r] = fmaf(sc, (float)acc[i][j][r], fmaf(lo, cs[j], facc[i][j][r]));
            }
    }
    __syncthreads();

    // ---- epilogue: R_m per row (a thread walks its token's records), column constants, then bf16 stores
    // through a wave-private LDS patch so that rows leave as 16-byte pieces
    float2* lrow = reinterpret_cast<float2*>(lds);                 // R_m
    float4* lcol = reinterpret_cast<float4*>(lds + GG_BM * 8);     // sw, sw*zp, c
    if (tid < GG_BM) {
        int64_t m = m0 + tid;
        m = m < a.M ? m : a.M - 1;
        const basq_tokmeta* rec = a.meta + m * ngroups;
        float R = 0.0f;
        for (int g = 0; g < ngroups; ++g) {
            const basq_tokmeta mt = rec[g];
            R += fmaf(mt.scale, (float)mt.rowsum, 128.0f * mt.lo);
        }
        lrow[tid] = make_float2(R, 0.0f);
    } else {
        int n = n0 + tid - GG_BM;
        n = n < a.N ? n : a.N - 1;
        const float sw = bf16_to_f32(a.w_scale[n]), zp = bf16_to_f32(a.w_zero[n]);
        lcol[tid - GG_BM] = make_float4(sw, sw * zp, a.out_bias ? a.out_bias[n] : 0.0f, 0.0f);
    }
    __syncthreads();

    float4 cp[GG_TN];
#pragma unroll
    for (int j = 0; j < GG_TN; ++j) cp[j] = lcol[wn * GG_WN + j * 32 + col_in_tile];
    const bool vec_ok = (a.ldy & 7) == 0 && (reinterpret_cast<uintptr_t>(a.Y) & 15) == 0;
    constexpr int PITCH = GG_WN * 2 + 16;                       // bytes
    constexpr int CH_PER_ROW = GG_WN / 8;                       // 16-byte pieces per row
    constexpr int PIECES = 32 * CH_PER_ROW / 64;                // per lane per 32-row block
    uint8_t* patch = lds + 4096 + wave * (32 * PITCH);
    static_assert(4096 + GG_WAVES * 32 * PITCH <= GG_STAGES * GG_OP_BYTES, "epilogue staging does not fit");
#pragma unroll
    for (int i = 0; i < GG_TM; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int rloc = 8 * (r >> 2) + 4 * rgrp + (r & 3);
            const float R = lrow[wm * GG_WM + i * 32 + rloc].x;
#pragma unroll
            for (int j = 0; j < GG_TN; ++j) {
                const float y = fmaf(cp[j].x, facc[i][j][r], fmaf(-cp[j].y, R, cp[j].z));
                if (vec_ok) {
                    *reinterpret_cast<uint16_t*>(patch + rloc * PITCH + (j * 32 + col_in_tile) * 2) = f32_to_bf16(y);
                } else {
                    const int64_t m = m0 + wm * GG_WM + i * 32 + rloc;
                    const int n = n0 + wn * GG_WN + j * 32 + col_in_tile;
                    if (m < a.M && n < a.N) a.Y[m * a.ldy + n] = f32_to_bf16(y);
                }
            }
        }
        if (!vec_ok) continue;
        // one wave's LDS operations complete in order: the reads below see the writes above
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int q = 0; q < PIECES; ++q) {
            const int id = q * 64 + lane;
            const int rloc = id / CH_PER_ROW, ch = id % CH_PER_ROW;
            const uint4 v = *reinterpret_cast<const uint4*>(patch + rloc * PITCH + ch * 16);
            const int64_t m = m0 + wm * GG_WM + i * 32 + rloc;
            const int n = n0 + wn * GG_WN + ch * 8;
            if (m < a.M) {
                uint16_t* dst = a.Y + m * a.ldy + n;
                if (n + 8 <= a.N) {
                    *reinterpret_cast<uint4*>(dst) = v;
                } else {
                    const uint16_t e[8] = {(uint16_t)v.x, (uint16_t)(v.x >> 16), (uint16_t)v.y, (uint16_t)(v.y >> 16),
                                           (uint16_t)v.z, (uint16_t)(v.z >> 16), (uint16_t)v.w, (uint16_t)(v.w >> 16)};
#pragma unroll
                    for (int u = 0; u < 8; ++u) if (n + u < a.N) dst[u] = e[u];
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
#endif  // __HIP_DEVICE_COMPILE__
}

// colsum[g][n] = sum of the codes of row n in group g: one thread per (g, n), 64 packed bytes each
__global__ __launch_bounds__(256) void group_colsums_kernel(const uint8_t* __restrict__ Wq, int N, int KB, int32_t* __restrict__ out) {
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int ngroups = KB / 64;
    if (id >= (int64_t)ngroups * N) return;
    const int g = (int)(id / N), n = (int)(id % N);
    const uint4* p = reinterpret_cast<const uint4*>(Wq + (int64_t)n * KB + g * 64);
    int sum = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint4 v = p[i];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            sum = __builtin_amdgcn_udot4(w[j] & 0x0F0F0F0Fu, 0x01010101u, sum, false);
            sum = __builtin_amdgcn_udot4((w[j] >> 4) & 0x0F0F0F0Fu, 0x01010101u, sum, false);
        }
    }
    out[id] = sum;
}

}  // namespace

bool gemm_grouped_applicable(const GemmArgs& a) {
    const int64_t ngroups = a.K / 128;
    // buffer addressing: every table must be smaller than 4 GiB
    return a.K % 128 == 0 && a.M >= 1 && a.M * (a.K / 2) < 0xFFFFFFFFll && (int64_t)a.N * (a.K / 2) < 0xFFFFFFFFll &&
           a.M * ngroups * 16 < 0xFFFFFFFFll && ngroups * a.N * 4 < 0x7FFFFFFFll;
}

int launch_gemm_grouped(const GemmArgs& a, const int32_t* w_gsum, hipStream_t s) {
    if (a.M == 0) return BASQ_OK;
    const int64_t tm = (a.M + GG_BM - 1) / GG_BM;
    const int64_t tn = ((int64_t)a.N + GG_BN - 1) / GG_BN;
    if (tm * tn > 0x7FFFFFFFll) return fail(BASQ_EINVAL, "w4a4_gemm_grouped: problem too large for one launch");
    hipLaunchKernelGGL(gemm_w4a4_grouped_kernel, dim3((unsigned)(tm * tn)), dim3(GG_THREADS), 0, s, a, w_gsum, (int)tm, (int)tn);
    return check_hip(hipGetLastError(), "w4a4_gemm_grouped launch");
}

int launch_group_colsums(const uint8_t* Wq, int32_t N, int32_t K, int32_t* out, hipStream_t s) {
    const int64_t total = (int64_t)(K / 128) * N;
    const int64_t blocks = (total + 255) / 256;
    if (blocks > 0x7FFFFFFFll) return fail(BASQ_EINVAL, "group_colsums: matrix too large");
    hipLaunchKernelGGL(group_colsums_kernel, dim3((unsigned)blocks), dim3(256), 0, s, Wq, N, K / 2, out);
    return check_hip(hipGetLastError(), "group_colsums launch");
}

}  // namespace basq
