// The group-wise INT4 x INT4 GEMM of gemm_w4a4_grouped.hip on the f8f6f4 matrix-core path (Eq. 4 applied per group
// of 128 channels; the product itself as in Sec. 5.2):
//
//     Y[m,n] = sw_n * ( sum_g ( s_mg ACC_g[m,n] + z_mg colsum_g[n] ) - zp_n * R_m ) + c_n
//
// Operands in the fp6 operand form (fp6_pack.hip: code q stored as the e2m3 number q/8), so a group's accumulator is
// S_g = ACC_g / 64 in fp32, exactly, and needs no conversion before it is scaled.  One LDS stage of the ring is one
// chunk of 128 codes = one group: the MFMAs of a group start from a zero accumulator operand, and the group is
// closed into the fp32 sum F' = F / 64 = sum_g ( s_mg S_g + z_mg colsum_g / 64 ) with two multiply-adds per element
// (every term is the exact 1/64 of the int8 kernel's, so F' * 64 has that kernel's bits).  The scaling does not run
// alongside MFMAs on this chip, but here it is two instructions per element against three on the int8 path, and
// the MFMAs take half the time.
// 128 x 128 tiles, four waves of 64 x 64, two workgroups per compute unit; ring of three operand stages and three
// slots of per-group constants (128 token records, 128 column sums), all filled by direct-to-LDS loads.
#include "basq_internal.h"
#include <type_traits>

namespace basq {

namespace {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

#define G6G_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

constexpr int G6G_BM = 128, G6G_BN = 128;
constexpr int G6G_WAVES_N = 2, G6G_WAVES = 4, G6G_THREADS = 256;
constexpr int G6G_WM = 64, G6G_WN = 64, G6G_TM = 2, G6G_TN = 2;
constexpr int G6G_CHUNK = 96;                                  // bytes of one row per stage: 128 codes
constexpr int G6G_BLOCK = 32 * G6G_CHUNK;                      // a 32-row block of a stage
constexpr int G6G_STAGES = 3;
constexpr int G6G_STAGE_BYTES = (G6G_BM + G6G_BN) * G6G_CHUNK;  // 24 KB
constexpr int G6G_PIECES = G6G_STAGE_BYTES / 1024;             // 1 KB pieces of a stage, one wave-load each
constexpr int G6G_LOADS = G6G_PIECES / G6G_WAVES;              // operand loads per wave per stage
constexpr int G6G_A_LOADS = (G6G_BM * G6G_CHUNK / 1024) / G6G_WAVES;   // ... of which the first ones are activations
constexpr int G6G_PSLOTS = 3;                                  // ring of per-group constants
constexpr int G6G_PSLOT_BYTES = 2560;                          // 128 records of 16 B, then 128 column sums of 4 B
constexpr int G6G_NUM_XCD = 8;
static_assert(G6G_PIECES % G6G_WAVES == 0 && (G6G_BM * G6G_CHUNK / 1024) % G6G_WAVES == 0, "whole rounds of loads");
static_assert(2 * (G6G_STAGES * G6G_STAGE_BYTES + G6G_PSLOTS * G6G_PSLOT_BYTES) <= 160 * 1024, "two workgroups per compute unit");

// Wait until at most N of this wave's direct-to-LDS loads are outstanding and its own LDS reads have returned,
// then join the workgroup barrier (one asm block: the compiler's own barrier would wait for every load).
template <int N>
__device__ __forceinline__ void g6g_wait_loads_and_barrier() {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

__global__ __launch_bounds__(G6G_THREADS, 2) void gemm_w4a4_grouped_fp6_kernel(GemmArgs a, const int32_t* w_gsum, int tiles_m, int tiles_n) {
#if defined(__HIP_DEVICE_COMPILE__)   // the body uses device-only buffer-resource types; the host pass only needs the stub
    __shared__ __attribute__((aligned(1024))) uint8_t lds[G6G_STAGES * G6G_STAGE_BYTES + G6G_PSLOTS * G6G_PSLOT_BYTES];
    uint8_t* const pring = lds + G6G_STAGES * G6G_STAGE_BYTES;

    // ---- tile assignment (ids congruent mod 8 run on one XCD and walk a compact band)
    int tile_m, tile_n;
    {
        const int total = tiles_m * tiles_n;
        const int pid = blockIdx.x;
        int t = pid;
        const int per_xcd = total / G6G_NUM_XCD;
        if (pid < per_xcd * G6G_NUM_XCD) t = (pid % G6G_NUM_XCD) * per_xcd + pid / G6G_NUM_XCD;
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
    const int wm = wave / G6G_WAVES_N, wn = wave % G6G_WAVES_N;
    const int swave = __builtin_amdgcn_readfirstlane(wave);
    const int64_t m0 = (int64_t)tile_m * G6G_BM;
    const int n0 = tile_n * G6G_BN;
    const int ngroups = a.K / 128;
    const int rb_a = (int)((a.M + 31) >> 5), rb_w = (a.N + 31) >> 5;   // 32-row blocks per chunk of K
    const unsigned a_step = (unsigned)rb_a * G6G_BLOCK, w_step = (unsigned)rb_w * G6G_BLOCK;   // bytes from one chunk to the next
    const __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(a.Aq6), 0, (int)(a_step * (unsigned)ngroups), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(a.Wq6), 0, (int)(w_step * (unsigned)ngroups), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_m = __builtin_amdgcn_make_buffer_rsrc(const_cast<basq_tokmeta*>(a.meta), 0, (int)(a.M * ngroups * 16), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_c = __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t*>(w_gsum), 0, (int)((int64_t)ngroups * a.N * 4), 0x00020000);

    // ---- direct loads.  Operand load i of wave w copies the 1 KB piece i*4 + w of the stage (three pieces make one
    // 32-row block; which block is uniform over the wave and goes into the scalar offset; blocks past the matrix are
    // clamped to its last block).  One more load per wave brings a group's constants: waves 0, 1 the token records
    // of rows 64w + lane, waves 2, 3 the column sums of columns 64(w-2) + lane (clamped likewise).
    const int lane_off = lane * 16;
    int soff[G6G_LOADS];
#pragma unroll
    for (int i = 0; i < G6G_LOADS; ++i) {
        const int piece = i * G6G_WAVES + swave;
        int blk = piece / 3;
        const int part = piece % 3;
        if (i < G6G_A_LOADS) {
            blk += tile_m * (G6G_BM / 32);
            blk = blk < rb_a ? blk : rb_a - 1;
        } else {
            blk += tile_n * (G6G_BN / 32) - G6G_BM / 32;
            blk = blk < rb_w ? blk : rb_w - 1;
        }
        soff[i] = blk * G6G_BLOCK + part * 1024;
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
    auto issue_operands = [&](int g) {
        uint8_t* stage = lds + (g % G6G_STAGES) * G6G_STAGE_BYTES + swave * 1024;
        const unsigned koff_a = (unsigned)g * a_step, koff_w = (unsigned)g * w_step;   // unsigned 32-bit byte offsets
#pragma unroll
        for (int i = 0; i < G6G_LOADS; ++i) {
            if (i < G6G_A_LOADS)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a, G6G_LDS_PTR(stage + i * G6G_WAVES * 1024), 16, lane_off, (int)(koff_a + (unsigned)soff[i]), 0, 0);
            else
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_w, G6G_LDS_PTR(stage + i * G6G_WAVES * 1024), 16, lane_off, (int)(koff_w + (unsigned)soff[i]), 0, 0);
        }
    };
    auto issue_constants = [&](int g) {
        uint8_t* slot = pring + (g % G6G_PSLOTS) * G6G_PSLOT_BYTES;
        if (swave < 2)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_m, G6G_LDS_PTR(slot + swave * 1024), 16, pvoff, g * 16, 0, 0);
        else
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_c, G6G_LDS_PTR(slot + 2048 + (swave - 2) * 256), 4, pvoff, g * a.N * 4, 0, 0);
    };

    // ---- fragment addressing: lane (frow, fhalf) feeds k = 64*kb + 32*fhalf .. +31 of its row, i.e. group
    // f = 2*kb + fhalf of the row's block: 16 bytes among the pieces, 8 bytes among the tails
    const int frow = lane & 31, fhalf = lane >> 5;
    int moff[2], toff[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
        moff[kb] = 64 * frow + 16 * ((2 * kb + fhalf) ^ ((frow >> 2) & 3));
        toff[kb] = 2048 + 256 * (2 * kb + fhalf) + 8 * frow;
    }
    const int a_row = (wm * G6G_WM / 32) * G6G_BLOCK;
    const int b_row = (G6G_BM / 32 + wn * G6G_WN / 32) * G6G_BLOCK;
    // byte offsets of the 8-byte tail reads, one opaque register each: reads whose addresses share a visible base
    // get merged into paired reads, whose result could not land in two operand tuples without register copies
    int ta[2][G6G_TM], tb[2][G6G_TN];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int i = 0; i < G6G_TM; ++i) { ta[kb][i] = a_row + i * G6G_BLOCK + toff[kb]; asm volatile("" : "+v"(ta[kb][i])); }
#pragma unroll
        for (int j = 0; j < G6G_TN; ++j) { tb[kb][j] = b_row + j * G6G_BLOCK + toff[kb]; asm volatile("" : "+v"(tb[kb][j])); }
    }
    const int col_in_tile = lane & 31, rgrp = lane >> 5;

    float facc[G6G_TM][G6G_TN][16];                  // F / 64
#pragma unroll
    for (int i = 0; i < G6G_TM; ++i)
#pragma unroll
        for (int j = 0; j < G6G_TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) facc[i][j][r] = 0.0f;
    v16f acc[G6G_TM][G6G_TN];
    // operand registers: six consecutive VGPRs per fragment (the builtin takes eight; the fp6 form reads six)
    v8i pa[2][G6G_TM], pb[2][G6G_TN];
#pragma unroll
    for (int set = 0; set < 2; ++set) {
#pragma unroll
        for (int i = 0; i < G6G_TM; ++i) pa[set][i] = v8i{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int j = 0; j < G6G_TN; ++j) pb[set][j] = v8i{0, 0, 0, 0, 0, 0, 0, 0};
    }
    auto read_one = [&](v8i& dst, const uint8_t* main_ptr, const uint8_t* tail_ptr) {
        const v4i m = *reinterpret_cast<const v4i*>(main_ptr);
        const v2i t = *reinterpret_cast<const v2i*>(tail_ptr);
        dst[0] = m[0]; dst[1] = m[1]; dst[2] = m[2]; dst[3] = m[3]; dst[4] = t[0]; dst[5] = t[1];
    };
    // fragment number t of the read order B0, A0, B1, A1: the order in which the MFMAs (token block outer, channel
    // block inner) first need them
    auto read_nth = [&](int t, const uint8_t* st, int kb, int set) {
        if (t == 0) read_one(pb[set][0], st + b_row + moff[kb], st + tb[kb][0]);
        else if (t == 1) read_one(pa[set][0], st + a_row + moff[kb], st + ta[kb][0]);
        else if (t == 2) read_one(pb[set][1], st + b_row + G6G_BLOCK + moff[kb], st + tb[kb][1]);
        else read_one(pa[set][1], st + a_row + G6G_BLOCK + moff[kb], st + ta[kb][1]);
    };
    auto read_frags = [&](const uint8_t* st, int kb, int set) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            read_nth(t, st, kb, set);
            __builtin_amdgcn_sched_barrier(0);            // keep the order of the main loop (its waits count reads)
        }
    };
    const v16f zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    // Half a group: the four MFMAs of one k-block with the fragment reads of the next k-block issued between them
    // (all reads first and all MFMAs after makes every wave of the compute unit queue at the LDS together while
    // the matrix cores idle, as in the per-token fp6 kernel).
    auto half = [&](int use_set, bool from_zero, const uint8_t* rd_stage, int rd_kb, int rd_set, bool do_reads) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            if (do_reads) read_nth(t, rd_stage, rd_kb, rd_set);
            const int i = t >> 1, j = t & 1;
            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(pb[use_set][j], pa[use_set][i], from_zero ? zero : acc[i][j], 2, 2, 0, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // The weights are the first MFMA operand: accumulator register r of lane l belongs to token l % 32 of the row
    // block and to output channel 8*(r/4) + 4*(l/32) + r%4 of the column block.  A lane then needs one token record
    // per row block and group, and the 32 column sums come as eight 16-byte reads that are the same address for
    // half a wave.  The column sums are kept in LDS as floats, already divided by 64: waves 0 and 1 convert the slot
    // of group g+1 in place after the barrier of step g (64 values each); its readers come after the next barrier.
    auto convert_colsums_load = [&](int g) -> int {
        return *reinterpret_cast<const int*>(pring + (g % G6G_PSLOTS) * G6G_PSLOT_BYTES + 2048 + (swave * 64 + lane) * 4);
    };
    auto convert_colsums_store = [&](int g, int v) {
        *reinterpret_cast<int*>(pring + (g % G6G_PSLOTS) * G6G_PSLOT_BYTES + 2048 + (swave * 64 + lane) * 4) =
            __float_as_int(0.015625f * (float)v);
    };

    // ---- prologue: operands and constants of the first two groups.  A wave's loads complete in the order it issued
    // them, so "at most n outstanding" below always names the newest n.
    issue_operands(0);
    issue_constants(0);
    if (ngroups > 1) {
        issue_operands(1);
        issue_constants(1);
        g6g_wait_loads_and_barrier<G6G_LOADS + 1>();
    } else {
        g6g_wait_loads_and_barrier<0>();
    }
    if (swave < 2) convert_colsums_store(0, convert_colsums_load(0));
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");      // LDS only: the second stage stays in flight
    read_frags(lds, 0, 0);

    // One group.  The last one is peeled off the loop so that the compiler's LDS waits count only the operands in
    // use (as in the per-token fp6 kernel).
    auto k_step = [&](int g, auto has_next) {
        const uint8_t* st = lds + (g % G6G_STAGES) * G6G_STAGE_BYTES;
        // the operand stage refilled now was read during step g-1; every wave has passed that step's barrier
        const bool ahead = g + 2 < ngroups;
        if (ahead) issue_operands(g + 2);
        __builtin_amdgcn_sched_barrier(0);
        half(0, true, st, 1, 1, true);
        // every read of this stage has been issued; pass the barrier behind which the next stage and the next
        // group's constants are complete and visible: only the operand loads just issued may stay in flight
        int raw_cs = 0;
        if (decltype(has_next)::value) {
            if (ahead) g6g_wait_loads_and_barrier<G6G_LOADS>(); else g6g_wait_loads_and_barrier<0>();
            // the constants slot refilled now was read at the end of step g-1, which every wave has left
            if (ahead) issue_constants(g + 2);
            if (swave < 2) raw_cs = convert_colsums_load(g + 1);
        } else {
            // the last group's column sums were converted during the step before: make that visible
            g6g_wait_loads_and_barrier<0>();
        }
        // this group's constants, requested ahead of the MFMAs that hide their latency.  Read as integers: the
        // compiler puts a wait for every outstanding direct-to-LDS load in front of a float-typed LDS read, which
        // would drain the ring in every step.
        const uint8_t* slot = pring + (g % G6G_PSLOTS) * G6G_PSLOT_BYTES;
        v2i szb[G6G_TM];
        v4i csb[G6G_TN][4];
#pragma unroll
        for (int i = 0; i < G6G_TM; ++i)
            szb[i] = *reinterpret_cast<const v2i*>(slot + (wm * G6G_WM + i * 32 + col_in_tile) * 16);   // scale, lo
#pragma unroll
        for (int j = 0; j < G6G_TN; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                csb[j][q] = *reinterpret_cast<const v4i*>(slot + 2048 + (wn * G6G_WN + j * 32 + 8 * q + 4 * rgrp) * 4);
        __builtin_amdgcn_sched_barrier(0);
        half(1, false, lds + ((g + 1) % G6G_STAGES) * G6G_STAGE_BYTES, 0, 0, decltype(has_next)::value);
        if (decltype(has_next)::value) {
            if (swave < 2) convert_colsums_store(g + 1, raw_cs);
        }
        // ---- close the group: F' += s_mg * S_g + z_mg * (colsum_g / 64)
#pragma unroll
        for (int i = 0; i < G6G_TM; ++i) {
            const float sc = __int_as_float(szb[i][0]), lo = __int_as_float(szb[i][1]);
#pragma unroll
            for (int j = 0; j < G6G_TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    facc[i][j][r] = fmaf(sc, acc[i][j][r], fmaf(lo, __int_as_float(csb[j][r >> 2][r & 3]), facc[i][j][r]));
        }
    };
    int g = 0;
    for (; g + 1 < ngroups; ++g) k_step(g, std::true_type{});
    k_step(g, std::false_type{});
    __syncthreads();

    // ---- epilogue: R_m per row (a thread walks its token's records), column constants, then bf16 stores
    // through a wave-private LDS patch so that rows leave as 16-byte pieces
    float2* lrow = reinterpret_cast<float2*>(lds);                 // R_m
    float4* lcol = reinterpret_cast<float4*>(lds + G6G_BM * 8);    // sw, sw*zp, c
    if (tid < G6G_BM) {
        int64_t m = m0 + tid;
        m = m < a.M ? m : a.M - 1;
        const basq_tokmeta* rec = a.meta + m * ngroups;
        float R = 0.0f;
        for (int gg = 0; gg < ngroups; ++gg) {
            const basq_tokmeta mt = rec[gg];
            R += fmaf(mt.scale, (float)mt.rowsum, 128.0f * mt.lo);
        }
        lrow[tid] = make_float2(R, 0.0f);
    } else {
        int n = n0 + tid - G6G_BM;
        n = n < a.N ? n : a.N - 1;
        const float sw = bf16_to_f32(a.w_scale[n]), zp = bf16_to_f32(a.w_zero[n]);
        lcol[tid - G6G_BM] = make_float4(sw, sw * zp, a.out_bias ? a.out_bias[n] : 0.0f, 0.0f);
    }
    __syncthreads();

    const bool vec_ok = (a.ldy & 7) == 0 && (reinterpret_cast<uintptr_t>(a.Y) & 15) == 0;
    constexpr int PITCH = G6G_WN * 2 + 16;                       // bytes
    constexpr int CH_PER_ROW = G6G_WN / 8;                       // 16-byte pieces per row
    constexpr int OUT_PIECES = 32 * CH_PER_ROW / 64;             // per lane per 32-row block
    uint8_t* patch = lds + 4096 + wave * (32 * PITCH);
    static_assert(4096 + G6G_WAVES * 32 * PITCH <= G6G_STAGES * G6G_STAGE_BYTES, "epilogue staging does not fit");
#pragma unroll
    for (int i = 0; i < G6G_TM; ++i) {
        const float R = lrow[wm * G6G_WM + i * 32 + col_in_tile].x;
#pragma unroll
        for (int j = 0; j < G6G_TN; ++j) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int cloc = j * 32 + 8 * (r >> 2) + 4 * rgrp + (r & 3);
                const float4 cp = lcol[wn * G6G_WN + cloc];
                const float y = fmaf(cp.x, 64.0f * facc[i][j][r], fmaf(-cp.y, R, cp.z));
                if (vec_ok) {
                    *reinterpret_cast<uint16_t*>(patch + col_in_tile * PITCH + cloc * 2) = f32_to_bf16(y);
                } else {
                    const int64_t m = m0 + wm * G6G_WM + i * 32 + col_in_tile;
                    const int n = n0 + wn * G6G_WN + cloc;
                    if (m < a.M && n < a.N) a.Y[m * a.ldy + n] = f32_to_bf16(y);
                }
            }
        }
        if (!vec_ok) continue;
        // one wave's LDS operations complete in order: the reads below see the writes above
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int q = 0; q < OUT_PIECES; ++q) {
            const int id = q * 64 + lane;
            const int rloc = id / CH_PER_ROW, ch = id % CH_PER_ROW;
            const uint4 v = *reinterpret_cast<const uint4*>(patch + rloc * PITCH + ch * 16);
            const int64_t m = m0 + wm * G6G_WM + i * 32 + rloc;
            const int n = n0 + wn * G6G_WN + ch * 8;
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

}  // namespace

bool gemm_grouped_fp6_applicable(const GemmArgs& a) {
    const int64_t ngroups = a.K / 128;
    // buffer addressing: every table must be smaller than 4 GiB
    return a.Aq6 && a.Wq6 && a.K % 128 == 0 && a.M >= 1 && (int64_t)basq_fp6_bytes(a.M, a.K) < 0xFFFFFFFFll &&
           (int64_t)basq_fp6_bytes(a.N, a.K) < 0xFFFFFFFFll && a.M * ngroups * 16 < 0xFFFFFFFFll &&
           ngroups * a.N * 4 < 0x7FFFFFFFll;
}

int launch_gemm_grouped_fp6(const GemmArgs& a, const int32_t* w_gsum, hipStream_t s) {
    if (a.M == 0) return BASQ_OK;
    const int64_t tm = (a.M + G6G_BM - 1) / G6G_BM;
    const int64_t tn = ((int64_t)a.N + G6G_BN - 1) / G6G_BN;
    if (tm * tn > 0x7FFFFFFFll) return fail(BASQ_EINVAL, "w4a4_gemm_grouped: problem too large for one launch");
    hipLaunchKernelGGL(gemm_w4a4_grouped_fp6_kernel, dim3((unsigned)(tm * tn)), dim3(G6G_THREADS), 0, s, a, w_gsum, (int)tm, (int)tn);
    return check_hip(hipGetLastError(), "w4a4_gemm_grouped (fp6) launch");
}

}  // namespace basq
