// Prefill INT4 x INT4 -> INT32 GEMM, main kernel: operands go HBM/L2 -> LDS with direct-to-LDS
// loads (no register staging), a ring of LDS stages, XOR-swizzled rows instead of padding, wave
// tiles of 128 x 64 so that LDS traffic per MFMA stays low, and the de-quantisation fused into
// the epilogue (paper Sec. 5.2; Fig. 6; Eq. 14).  Same arithmetic and nibble split as
// gemm_w4a4.hip, which remains the fallback for K % 128 != 0.
#include "basq_internal.h"
#include <type_traits>

namespace basq {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int NUM_XCD = 8;

#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define GLB_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

// Wait until at most N of this wave's vector-memory operations (the direct-to-LDS loads) are still
// outstanding, then join the workgroup barrier.  Written as one asm block: the compiler's own
// barrier would first wait for ALL outstanding loads, which would serialise the LDS ring.
template <int N>
__device__ __forceinline__ void wait_loads_and_barrier() {
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}

// BKB: packed bytes of K per row per stage (64 -> 128 codes).  STAGES: LDS ring depth.
template <int BM, int BN, int WAVES_M, int WAVES_N, int BKB, int STAGES, int MINOCC>
__global__ __launch_bounds__(WAVES_M * WAVES_N * 64, MINOCC) void gemm_w4a4_direct_kernel(GemmArgs a, int tiles_m, int tiles_n) {
#if defined(__HIP_DEVICE_COMPILE__)   // the body uses device-only buffer-resource types; the host pass only needs the stub
    constexpr int WAVES = WAVES_M * WAVES_N;
    constexpr int THREADS = WAVES * 64;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int NCH = BKB / 16;                             // 16-byte chunks per row per stage
    constexpr int ROWS = BM + BN;
    constexpr int STAGE_BYTES = ROWS * BKB;
    constexpr int LOADS = ROWS * NCH / THREADS;               // direct loads per thread per stage
    static_assert((ROWS * NCH) % THREADS == 0, "stage does not divide over the threads");
    static_assert(BKB == 64 || BKB == 128, "BKB");
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile");

    __shared__ __attribute__((aligned(1024))) uint8_t lds[STAGES * STAGE_BYTES];

    // ---- tile assignment (XCD-aware: ids congruent mod 8 run on one XCD and walk a compact band)
    int tile_m, tile_n;
    {
        const int total = tiles_m * tiles_n;
        const int pid = blockIdx.x;
        int t = pid;
        const int per_xcd = total / NUM_XCD;
        if (pid < per_xcd * NUM_XCD) t = (pid % NUM_XCD) * per_xcd + pid / NUM_XCD;
#ifndef GD_GROUP_M
#define GD_GROUP_M 4
#endif
        constexpr int GROUP_M = GD_GROUP_M;
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
    const int KB = a.K / 2;
    const int ksteps = KB / BKB;                              // K % (2*BKB) == 0 is checked by the launcher

    // ---- direct loads: load i of wave w fills LDS chunks [(i*WAVES + w)*64, +64) of a stage; the lane
    // picks the global chunk whose swizzled position is its LDS slot.  Buffer loads: the per-lane byte
    // offset is fixed for the whole kernel, the K advance is a scalar offset, the LDS address sits in M0 --
    // no vector instruction is spent on addressing.  Rows past the matrix are clamped to the last row.
    constexpr int A_LOADS = BM * NCH / (64 * WAVES);          // loads 0 .. A_LOADS-1 fetch activations, the rest weights
    static_assert((BM * NCH) % (64 * WAVES) == 0, "A rows must fill whole wave loads");
    const int swave = __builtin_amdgcn_readfirstlane(wave);
    const __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(a.Aq), 0, (int)(a.M * KB), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(a.Wq), 0, (int)((int64_t)a.N * KB), 0x00020000);
    int voff[LOADS];
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
        const int L = (i * WAVES + wave) * 64 + lane;
        const int row = L / NCH, cpos = L % NCH;
        const int swz = (BKB == 128) ? ((row >> 1) & 7) : ((row >> 2) & 3);   // 16 consecutive rows hit 16 distinct 16-byte bank groups
        const int c = cpos ^ swz;
        if (i < A_LOADS) {
            int64_t m = m0 + row;
            m = m < a.M ? m : a.M - 1;
            voff[i] = (int)(m * KB + c * 16);
        } else {
            int n = n0 + row - BM;
            n = n < a.N ? n : a.N - 1;
            voff[i] = (int)((int64_t)n * KB + c * 16);
        }
    }
    auto issue_loads = [&](int ks) {
        uint8_t* stage = lds + (ks % STAGES) * STAGE_BYTES + swave * 1024;
        const int koff = ks * BKB;
#pragma unroll
        for (int i = 0; i < LOADS; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(i < A_LOADS ? rsrc_a : rsrc_w, LDS_PTR(stage + i * WAVES * 1024), 16,
                                                     voff[i], koff, 0, 0);
    };

    // ---- fragment addressing: lane (frow, fhalf) reads chunk fhalf + 2h of its row, swizzled
    const int frow = lane & 31, fhalf = lane >> 5;
    const int fswz = (BKB == 128) ? ((frow >> 1) & 7) : ((frow >> 2) & 3);
    int foff[NCH / 2];
#pragma unroll
    for (int h = 0; h < NCH / 2; ++h) foff[h] = (((fhalf + 2 * h) ^ fswz) << 4);
    const int a_row = (wm * WM + frow) * BKB;
    const int b_row = (BM + wn * WN + frow) * BKB;

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // ---- prologue: fill STAGES-1 stages
#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s)
        if (s < ksteps) issue_loads(s);
    if (STAGES >= 3 && ksteps > 1) wait_loads_and_barrier<LOADS>(); else wait_loads_and_barrier<0>();

    // Packed fragments are read from LDS one h ahead of the MFMAs that use them, into two register
    // sets used alternately.  The scheduling barriers keep the reads ahead of the MFMA block, so the
    // LDS latency hides behind sixteen or more MFMAs.
    v4i pa[2][TM], pb[2][TN];
    auto read_frags = [&](const uint8_t* st, int h, int set) {
#pragma unroll
        for (int i = 0; i < TM; ++i) pa[set][i] = *reinterpret_cast<const v4i*>(st + a_row + i * 32 * BKB + foff[h]);
#pragma unroll
        for (int j = 0; j < TN; ++j) pb[set][j] = *reinterpret_cast<const v4i*>(st + b_row + j * 32 * BKB + foff[h]);
    };
    auto compute = [&](int set) {
        v4i alo[TM], ahi[TM];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            alo[i] = pa[set][i] & 0x0F0F0F0F;
            ahi[i] = (pa[set][i] >> 4) & 0x0F0F0F0F;
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const v4i blo = pb[set][j] & 0x0F0F0F0F;
            const v4i bhi = (pb[set][j] >> 4) & 0x0F0F0F0F;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(alo[i], blo, acc[i][j], 0, 0, 0);
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ahi[i], bhi, acc[i][j], 0, 0, 0);
            }
        }
    };
    static_assert((NCH / 2) % 2 == 0, "the two fragment register sets alternate per h");
    read_frags(lds, 0, 0);

    // One K-step; the last one is peeled off the loop so that "is there a next stage to read" is known at compile
    // time: otherwise two paths meet in front of the last block of MFMAs, one without the next stage's reads in
    // flight, and the compiler waits there for every outstanding LDS read instead of only the operands in use.
    auto k_step = [&](int ks, auto has_next) {
        const uint8_t* st = lds + (ks % STAGES) * STAGE_BYTES;
        // the stage refilled now was read during step ks-1; every wave has passed that step's barrier
        if (ks + STAGES - 1 < ksteps) issue_loads(ks + STAGES - 1);
#pragma unroll
        for (int h = 0; h < NCH / 2; ++h) {
            if (h + 1 < NCH / 2) {
                read_frags(st, h + 1, (h + 1) & 1);
            } else {
                // last h of the step: every read of this stage has been issued and consumed; pass the
                // barrier (next stage complete and visible), then start the next step's first reads
                if (STAGES >= 3 && ks + STAGES - 1 < ksteps) wait_loads_and_barrier<LOADS>(); else wait_loads_and_barrier<0>();
                if (decltype(has_next)::value) read_frags(lds + ((ks + 1) % STAGES) * STAGE_BYTES, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            compute(h & 1);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    int ks = 0;
    for (; ks + 1 < ksteps; ++ks) k_step(ks, std::true_type{});
    k_step(ks, std::false_type{});
    __syncthreads();

    // ---- epilogue: row and column constants through LDS (free now), then one bf16 per lane per store
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

    const int col_in_tile = lane & 31, rgrp = lane >> 5;
    float4 cp[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) cp[j] = lcol_par[wn * WN + j * 32 + col_in_tile];

    // Vector path: each wave turns one 32-row block of its tile at a time into bf16 in a private LDS
    // patch (row pitch padded against bank conflicts) and writes it out as 16-byte pieces, whole rows of
    // the wave tile contiguous.  Needs 16-byte aligned rows of Y; the debug accumulator dump and
    // unaligned outputs take the scalar path below.
    const bool vec_ok = a.acc_out == nullptr && (a.ldy & 7) == 0 && (reinterpret_cast<uintptr_t>(a.Y) & 15) == 0;
    if (vec_ok) {
        constexpr int PITCH = WN * 2 + 16;                      // bytes
        constexpr int CH_PER_ROW = WN / 8;                      // 16-byte pieces per row
        constexpr int PIECES = 32 * CH_PER_ROW / 64;            // per lane per 32-row block
        uint8_t* patch = lds + (BM + BN) * 16 + wave * (32 * PITCH);
        static_assert((BM + BN) * 16 + WAVES * 32 * PITCH <= STAGES * STAGE_BYTES, "epilogue staging does not fit");
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int rloc = 8 * (r >> 2) + 4 * rgrp + (r & 3);
                const float4 rp = lrow_par[wm * WM + i * 32 + rloc];
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const float t = (float)acc[i][j][r] - cp[j].y * rp.z;
                    const float y = fmaf(rp.x * cp[j].x, t, fmaf(rp.y, cp[j].z, cp[j].w));
                    *reinterpret_cast<uint16_t*>(patch + rloc * PITCH + (j * 32 + col_in_tile) * 2) = f32_to_bf16(y);
                }
            }
            // one wave's LDS operations complete in order: the reads below see the writes above
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int q = 0; q < PIECES; ++q) {
                const int id = q * 64 + lane;
                const int rloc = id / CH_PER_ROW, ch = id % CH_PER_ROW;
                const uint4 v = *reinterpret_cast<const uint4*>(patch + rloc * PITCH + ch * 16);
                const int64_t m = m0 + wm * WM + i * 32 + rloc;
                const int n = n0 + wn * WN + ch * 8;
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
        return;
    }
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
#endif  // __HIP_DEVICE_COMPILE__
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int BKB, int STAGES, int MINOCC>
int launch_direct(const GemmArgs& a, hipStream_t s) {
    const int64_t tm = (a.M + BM - 1) / BM;
    const int64_t tn = ((int64_t)a.N + BN - 1) / BN;
    if (tm * tn > 0x7FFFFFFFll) return fail(BASQ_EINVAL, "w4a4_gemm: problem too large for one launch");
    hipLaunchKernelGGL((gemm_w4a4_direct_kernel<BM, BN, WAVES_M, WAVES_N, BKB, STAGES, MINOCC>), dim3((unsigned)(tm * tn)),
                       dim3(WAVES_M * WAVES_N * 64), 0, s, a, (int)tm, (int)tn);
    return check_hip(hipGetLastError(), "w4a4_gemm (direct) launch");
}

}  // namespace

bool gemm_direct_applicable(const GemmArgs& a) {
    // buffer addressing: both packed operands must be smaller than 4 GiB
    return a.K % 256 == 0 && a.M >= 1 && a.M * (a.K / 2) < 0xFFFFFFFFll && (int64_t)a.N * (a.K / 2) < 0xFFFFFFFFll;
}

namespace {
// share of the launched tile slots that hold a real tile when `tiles` tiles run `slots` at a time
double round_efficiency(int64_t tiles, int64_t slots) {
    const int64_t rounds = (tiles + slots - 1) / slots;
    return (double)tiles / (double)(rounds * slots);
}
}  // namespace

int launch_gemm_direct(const GemmArgs& a, hipStream_t s) {
#ifdef GEMM_DIRECT_CFG
    return launch_direct<GEMM_DIRECT_CFG>(a, s);
#else
    // Three tilings; larger tiles reuse operands better (less L2 traffic per MFMA) but quantise
    // worse on small problems.  256 CUs; the 4-wave tilings run two workgroups per CU.
    auto tiles = [&](int bm, int bn) { return ((a.M + bm - 1) / bm) * (((int64_t)a.N + bn - 1) / bn); };
    const double s_big = 1.00 * round_efficiency(tiles(256, 256), 256);
    const double s_mid = 0.95 * round_efficiency(tiles(256, 128), 512);
    const double s_small = 0.85 * round_efficiency(tiles(128, 128), 512);
    if (s_big >= s_mid && s_big >= s_small) return launch_direct<256, 256, 2, 4, 128, 2, 2>(a, s);
    if (s_mid >= s_small) return launch_direct<256, 128, 2, 2, 64, 3, 2>(a, s);
    return launch_direct<128, 128, 2, 2, 64, 3, 2>(a, s);
#endif
}

}  // namespace basq
