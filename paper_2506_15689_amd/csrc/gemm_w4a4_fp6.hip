// Prefill INT4 x INT4 -> INT32 GEMM on the f8f6f4 matrix-core path (paper Sec. 5.2; Fig. 6; Eq. 14).
//
// Both operands arrive in the fp6 operand form of fp6_pack.hip: code q stored as the e2m3 number q/8.
// v_mfma_f32_32x32x64_f8f6f4 with two fp6 operands runs at twice the int8 rate and its fp32 accumulator
// holds S = sum_k (qa/8)(qb/8) exactly (multiples of 1/64, S < 2^17 for K <= 32768).  The integer
// accumulator of the INT4 product is ACC = 64*S; the epilogue de-quantises exactly as the int8 kernels do.
//
// Structure as in gemm_w4a4_direct.hip: direct-to-LDS buffer loads into a ring of stages, fragments
// read one step ahead into two register sets, XCD-aware tile order.  A stage holds 128 codes per row.
// The operands are stored as 3 KB blocks of 32 rows x 128 codes that already are the LDS image (see
// fp6_pack.hip): a stage is filled by contiguous 1 KB copies of whole cache lines, and both the 16-byte
// and the 8-byte fragment reads are free of bank conflicts.  No unpacking: LDS -> registers -> MFMA.
#include "basq_internal.h"
#include <type_traits>

namespace basq {

namespace {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int NUM_XCD = 8;
constexpr int CHUNK = 96;              // bytes of one row per stage: 128 codes
constexpr int BLOCK = 32 * CHUNK;      // one 32-row block of a stage: 2 KB of 16-byte pieces, 1 KB of 8-byte tails

#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

// Wait until at most N of this wave's direct-to-LDS loads are outstanding and its own LDS reads have
// returned, then join the workgroup barrier (one asm block: the compiler's own barrier would wait for
// every outstanding load and serialise the ring).
template <int N>
__device__ __forceinline__ void wait_loads_and_barrier() {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

#ifndef G6_GROUP_M
#define G6_GROUP_M 4
#endif

template <int BM, int BN, int WAVES_M, int WAVES_N, int STAGES, int MINOCC>
__global__ __launch_bounds__(WAVES_M * WAVES_N * 64, MINOCC) void gemm_w4a4_fp6_kernel(GemmArgs a, int tiles_m, int tiles_n) {
#if defined(__HIP_DEVICE_COMPILE__)   // the body uses device-only buffer-resource types; the host pass only needs the stub
    constexpr int WAVES = WAVES_M * WAVES_N;
    constexpr int THREADS = WAVES * 64;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int ROWS = BM + BN;
    constexpr int STAGE_BYTES = ROWS * CHUNK;
    constexpr int PIECES = STAGE_BYTES / 1024;                // 1 KB pieces of a stage, one wave-load each
    constexpr int LOADS = (PIECES + WAVES - 1) / WAVES;       // direct loads per thread per stage (the last one may be idle)
    constexpr int MIN_LOADS = PIECES / WAVES;                 // ... that every wave really issues: what the partial waits count
    constexpr int A_PIECES = BM * CHUNK / 1024;               // pieces 0 .. A_PIECES-1 of a stage are activations
    static_assert(STAGE_BYTES % 1024 == 0, "a stage is a whole number of 1 KB pieces");
    static_assert(BM % 32 == 0 && BN % 32 == 0, "tiles are made of 32-row blocks");
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile");
    static_assert(STAGES == 2 || STAGES == 3, "the wait counts below assume at most one stage in flight beyond the next");
    static_assert((BM + BN) * 16 <= STAGE_BYTES, "the epilogue constants live in the last stage");

    __shared__ __attribute__((aligned(1024))) uint8_t lds[STAGES * STAGE_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int swave = __builtin_amdgcn_readfirstlane(wave);
    const int ksteps = a.K / 128;
    const int rb_a = (int)((a.M + 31) >> 5), rb_w = (a.N + 31) >> 5;   // 32-row blocks per chunk of K
    const unsigned a_step = (unsigned)rb_a * BLOCK, w_step = (unsigned)rb_w * BLOCK;   // bytes from one chunk of K to the next
    const __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(a.Aq6), 0, (int)(a_step * (unsigned)ksteps), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(a.Wq6), 0, (int)(w_step * (unsigned)ksteps), 0x00020000);

    // ---- tile order (XCD-aware: workgroups congruent mod 8 run on one XCD; the tiles a workgroup takes,
    // blockIdx.x + i * gridDim.x, stay congruent when the grid is a multiple of 8 and walk a compact band)
    const int total = tiles_m * tiles_n;
    auto tile_of = [&](int pid, int& tile_m, int& tile_n) {
        int t = pid;
        const int per_xcd = total / NUM_XCD;
        if (pid < per_xcd * NUM_XCD) t = (pid % NUM_XCD) * per_xcd + pid / NUM_XCD;
        constexpr int GROUP_M = G6_GROUP_M;
        const int band = t / (GROUP_M * tiles_n);
        const int first_m = band * GROUP_M;
        const int rows = (tiles_m - first_m) < GROUP_M ? (tiles_m - first_m) : GROUP_M;
        const int in_band = t - band * GROUP_M * tiles_n;
        tile_m = first_m + in_band % rows;
        tile_n = in_band / rows;
    };

    // ---- direct loads: load i of wave w copies the 1 KB piece number i*WAVES + w of the stage; three
    // pieces make one 32-row block.  Which block a piece comes from is uniform over the wave, so it goes
    // into the scalar offset of the load; the only per-lane part is 16 * lane.  Blocks past the matrix
    // are clamped to its last block.
    const int lane_off = lane * 16;
    int soff[LOADS];                                           // scalar: block and part of each of this wave's pieces
    auto set_tile = [&](int tile_m, int tile_n) {
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            const int piece = i * WAVES + swave;
            int blk = piece / 3;
            const int part = piece % 3;
            if (piece < A_PIECES) {
                blk += tile_m * (BM / 32);
                blk = blk < rb_a ? blk : rb_a - 1;
            } else {
                blk += tile_n * (BN / 32) - BM / 32;
                blk = blk < rb_w ? blk : rb_w - 1;
            }
            soff[i] = blk * BLOCK + part * 1024;
        }
    };
    auto issue_loads = [&](int ks) {
        uint8_t* stage = lds + (ks % STAGES) * STAGE_BYTES + swave * 1024;
        const unsigned koff_a = (unsigned)ks * a_step, koff_w = (unsigned)ks * w_step;   // unsigned 32-bit byte offsets
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            // whether piece i * WAVES + wave exists is known at compile time for all but a last partial round, and
            // which operand it belongs to whenever the activation pieces fill whole rounds: no branch per load then
            // (the wave-dependent tests are uniform over the wave)
            if ((i + 1) * WAVES > PIECES && i * WAVES + swave >= PIECES) continue;
            if (A_PIECES % WAVES == 0 ? i < A_PIECES / WAVES : i * WAVES + swave < A_PIECES)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a, LDS_PTR(stage + i * WAVES * 1024), 16, lane_off, (int)(koff_a + (unsigned)soff[i]), 0, 0);
            else
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_w, LDS_PTR(stage + i * WAVES * 1024), 16, lane_off, (int)(koff_w + (unsigned)soff[i]), 0, 0);
        }
    };
    auto issue_prologue = [&]() {
#pragma unroll
        for (int s = 0; s < STAGES - 1; ++s)
            if (s < ksteps) issue_loads(s);
    };

    // ---- fragment addressing: lane (frow, fhalf) feeds k = 64*kb + 32*fhalf .. +31 of its row, i.e.
    // group f = 2*kb + fhalf of the row's block: 16 bytes among the pieces, 8 bytes among the tails
    const int frow = lane & 31, fhalf = lane >> 5;
    int moff[2], toff[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
        moff[kb] = 64 * frow + 16 * ((2 * kb + fhalf) ^ ((frow >> 2) & 3));
        toff[kb] = 2048 + 256 * (2 * kb + fhalf) + 8 * frow;
    }
    const int a_row = (wm * WM / 32) * BLOCK;
    const int b_row = (BM / 32 + wn * WN / 32) * BLOCK;
    // Byte offsets of the 8-byte tail reads, one opaque register each: reads whose addresses share a
    // visible base get merged into paired reads, whose result could not land in two operand tuples
    // without register copies.
    int ta[2][TM], tb[2][TN];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int i = 0; i < TM; ++i) { ta[kb][i] = a_row + i * BLOCK + toff[kb]; asm volatile("" : "+v"(ta[kb][i])); }
#pragma unroll
        for (int j = 0; j < TN; ++j) { tb[kb][j] = b_row + j * BLOCK + toff[kb]; asm volatile("" : "+v"(tb[kb][j])); }
    }

    // epilogue constants: in the last stage of the ring, which the next tile's first loads do not touch
    float4* lrow_par = reinterpret_cast<float4*>(lds + (STAGES - 1) * STAGE_BYTES);
    float4* lcol_par = lrow_par + BM;

    // ---- persistent loop over this workgroup's tiles
    int pid = blockIdx.x;
    int tile_m, tile_n;
    tile_of(pid, tile_m, tile_n);
    set_tile(tile_m, tile_n);
    issue_prologue();
    bool first = true;
    while (true) {
        const int64_t m0 = (int64_t)tile_m * BM;
        const int n0 = tile_n * BN;
        v16f acc[TM][TN];
        // Operand registers: six consecutive VGPRs per fragment (the builtin takes eight; the fp6 form of
        // the instruction reads the first six).  The two LDS reads of a fragment land in them directly.
        v8i pa[2][TM], pb[2][TN];
    #pragma unroll
        for (int set = 0; set < 2; ++set) {
    #pragma unroll
            for (int i = 0; i < TM; ++i) pa[set][i] = v8i{0, 0, 0, 0, 0, 0, 0, 0};
    #pragma unroll
            for (int j = 0; j < TN; ++j) pb[set][j] = v8i{0, 0, 0, 0, 0, 0, 0, 0};
        }
        auto read_one = [&](v8i& dst, const uint8_t* main_ptr, const uint8_t* tail_ptr) {
            const v4i m = *reinterpret_cast<const v4i*>(main_ptr);
            const v2i t = *reinterpret_cast<const v2i*>(tail_ptr);
            dst[0] = m[0]; dst[1] = m[1]; dst[2] = m[2]; dst[3] = m[3]; dst[4] = t[0]; dst[5] = t[1];
        };
        // fragment number t of the read order B0, A0, B1, .., B(TN-1), A1, .., A(TM-1): the order in which the MFMAs
        // (row block outer, column block inner) first need them
        auto read_nth = [&](int t, const uint8_t* st, int kb, int set) {
            if (t == 0) read_one(pb[set][0], st + b_row + moff[kb], st + tb[kb][0]);
            else if (t == 1) read_one(pa[set][0], st + a_row + moff[kb], st + ta[kb][0]);
            else if (t < TN + 1) read_one(pb[set][t - 1], st + b_row + (t - 1) * BLOCK + moff[kb], st + tb[kb][t - 1]);
            else read_one(pa[set][t - TN], st + a_row + (t - TN) * BLOCK + moff[kb], st + ta[kb][t - TN]);
        };
        auto read_frags = [&](const uint8_t* st, int kb, int set) {
    #pragma unroll
            for (int t = 0; t < TM + TN; ++t) {
                read_nth(t, st, kb, set);
                __builtin_amdgcn_sched_barrier(0);        // keep the order of the main loop (its waits count reads)
            }
        };


#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

        // Stage 0 must have landed: on the first tile the loads of stage 1 may stay in flight; on later
        // tiles both stages were waited for before the previous epilogue's stores went out.  The barrier
        // also ends every wave's use of the epilogue constants before step 0 refills the last stage.
        if (first) {
            if (STAGES >= 3 && ksteps > 1) wait_loads_and_barrier<MIN_LOADS*(STAGES - 2)>(); else wait_loads_and_barrier<0>();
        } else if (STAGES >= 3) {
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        } else {
            wait_loads_and_barrier<0>();
        }
        first = false;
        read_frags(lds, 0, 0);

        // Half a K-step: the TM*TN MFMAs of one k-block, with the fragment reads of the NEXT k-block issued between
        // them, one fragment (two LDS reads) in front of each of the first TM+TN MFMAs, in the order in which the
        // next half will need them (B0, A0, B1 .. , A1 ..).  Issuing all reads first and all MFMAs after made every
        // wave of the compute unit queue at the LDS at the same time while the matrix cores idled, and then run
        // its MFMAs while the LDS idled; interleaved, the two pipes work at the same time.
        auto half = [&](int use_set, const uint8_t* rd_stage, int rd_kb, int rd_set, bool do_reads) {
    #pragma unroll
            for (int t = 0; t < TM * TN; ++t) {
                if (do_reads && t < TM + TN) read_nth(t, rd_stage, rd_kb, rd_set);
                const int i = t / TN, j = t % TN;
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(pa[use_set][i], pb[use_set][j], acc[i][j], 2, 2, 0, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        // One K-step.  The last one is peeled off the loop: with the "is there a next stage to read" test inside the
        // loop, two paths meet in front of the second block of MFMAs, one of them without the reads of the next
        // stage in flight, and the compiler then waits for every outstanding LDS read there -- including the ones
        // just issued -- instead of only for the operands the MFMAs use (a bubble of an LDS latency per step).
        auto k_step = [&](int ks, auto has_next) {
            const uint8_t* st = lds + (ks % STAGES) * STAGE_BYTES;
            // the stage refilled now was read during step ks-1; every wave has passed that step's barrier
            if (ks + STAGES - 1 < ksteps) issue_loads(ks + STAGES - 1);
            __builtin_amdgcn_sched_barrier(0);
            // kb = 0, reading kb = 1 of this stage ahead
            half(0, st, 1, 1, true);
            // every read of this stage has been issued; pass the barrier (next stage complete and visible: all but
            // the newest STAGES-2 loads have landed), then kb = 1, reading the next stage's kb = 0 ahead
            if (STAGES >= 3 && ks + STAGES - 1 < ksteps) wait_loads_and_barrier<MIN_LOADS*(STAGES - 2)>(); else wait_loads_and_barrier<0>();
            half(1, lds + ((ks + 1) % STAGES) * STAGE_BYTES, 0, 0, decltype(has_next)::value);
        };
        int ks = 0;
        for (; ks + 1 < ksteps; ++ks) k_step(ks, std::true_type{});
        k_step(ks, std::false_type{});
        // every wave has passed the last step's barrier, after which nothing reads the ring: request the
        // next tile's first stages now, so that their latency hides behind this tile's epilogue
        const int next_pid = pid + gridDim.x;
        const bool more = next_pid < total;
        int next_m = 0, next_n = 0;
        if (more) {
            tile_of(next_pid, next_m, next_n);
            set_tile(next_m, next_n);
            if (STAGES >= 3) issue_prologue();            // with two stages the constants would be overwritten
        }

        // ---- epilogue: row and column constants through LDS
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

        // (re)derived per tile from an opaque copy of the lane index: everything computed from it below
        // would otherwise be hoisted out of the tile loop and held in registers across the main loop
        int elane = lane;
        asm volatile("" : "+v"(elane));
        const int col_in_tile = elane & 31, rgrp = elane >> 5;
        float4 cp[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) cp[j] = lcol_par[wn * WN + j * 32 + col_in_tile];

        // Pair path: two adjacent rows per step.  A lane turns its two values (same column, rows A and A+1)
        // into one packed bf16 pair, trades it with the neighbouring column's lane (DPP), and a byte permute
        // leaves even lanes with (row A; columns c, c+1) and odd lanes with (row A+1; columns c-1, c): every
        // lane stores one dword, every half-wave 64-byte runs of two rows.
        const bool pair_ok = a.acc_out == nullptr && (a.ldy & 1) == 0 && (a.N & 1) == 0 && (reinterpret_cast<uintptr_t>(a.Y) & 3) == 0;
        if (pair_ok) {
            typedef float f2 __attribute__((ext_vector_type(2)));
            typedef __bf16 b2 __attribute__((ext_vector_type(2)));
            const int odd = elane & 1;
            const unsigned sel = odd ? 0x03020706u : 0x05040100u;
            // first every output dword into registers (they take the accumulators' place) ...
            unsigned outv[TM][8][TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const int rowA = 8 * (q >> 1) + 4 * rgrp + 2 * (q & 1);        // register 2q; register 2q+1 is the next row
                    const float4 rpA = lrow_par[wm * WM + i * 32 + rowA];
                    const float4 rpB = lrow_par[wm * WM + i * 32 + rowA + 1];
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        const float tA = fmaf(64.0f, acc[i][j][2 * q], -(cp[j].y * rpA.z));      // 64*S is the integer accumulator, exactly
                        const float tB = fmaf(64.0f, acc[i][j][2 * q + 1], -(cp[j].y * rpB.z));
                        const float yA = fmaf(rpA.x * cp[j].x, tA, fmaf(rpA.y, cp[j].z, cp[j].w));
                        const float yB = fmaf(rpB.x * cp[j].x, tB, fmaf(rpB.y, cp[j].z, cp[j].w));
                        const unsigned mine = __builtin_bit_cast(unsigned, __builtin_convertvector((f2){yA, yB}, b2));   // hardware round-to-nearest-even
                        const unsigned other = (unsigned)__builtin_amdgcn_update_dpp(0, (int)mine, 0xB1, 0xF, 0xF, false);   // lane ^ 1
                        outv[i][q][j] = __builtin_amdgcn_perm(other, mine, sel);
                    }
                }
            }
            // ... then wait for the next tile's first stages (requested before this epilogue, so mostly
            // landed), and only then send the stores: a wait placed after them would have to wait for
            // the stores too, the counter being one and the same
            if (more && STAGES >= 3) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
            for (int i = 0; i < TM; ++i) {
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const int rowA = 8 * (q >> 1) + 4 * rgrp + 2 * (q & 1);
                    const int64_t m = m0 + wm * WM + i * 32 + rowA + odd;
                    uint16_t* yrow = a.Y + m * a.ldy + n0 + wn * WN + (col_in_tile & ~1);
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        const int n = n0 + wn * WN + j * 32 + (col_in_tile & ~1);
                        if (m < a.M && n < a.N) *reinterpret_cast<uint32_t*>(yrow + j * 32) = outv[i][q][j];
                    }
                }
            }
        } else {
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
                            const int av = __float2int_rn(64.0f * acc[i][j][r]);
                            const float t = (float)av - cp[j].y * rp.z;
                            const float y = fmaf(rp.x * cp[j].x, t, fmaf(rp.y, cp[j].z, cp[j].w));
                            yrow[n] = f32_to_bf16(y);
                            if (a.acc_out) a.acc_out[m * (int64_t)a.N + n] = av;
                        }
                    }
                }
            }
        }
        if (!more) break;
        if (!pair_ok && STAGES >= 3) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // slow path: loads and stores alike
        pid = next_pid; tile_m = next_m; tile_n = next_n;
        if (STAGES < 3) issue_prologue();                 // two stages: only now is the ring free of the constants
    }
#endif  // __HIP_DEVICE_COMPILE__
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int STAGES, int MINOCC>
int launch_fp6(const GemmArgs& a, hipStream_t s) {
    const int64_t tm = (a.M + BM - 1) / BM;
    const int64_t tn = ((int64_t)a.N + BN - 1) / BN;
    if (tm * tn > 0x7FFFFFFFll) return fail(BASQ_EINVAL, "w4a4_gemm: problem too large for one launch");
    // persistent workgroups: as many as the chip's 256 compute units hold at once (MINOCC waves per
    // SIMD), each walking the tiles blockIdx.x, blockIdx.x + gridDim.x, ...
    const int64_t resident = 256 * (MINOCC * 4 / (WAVES_M * WAVES_N));
    static_assert(MINOCC * 4 % (WAVES_M * WAVES_N) == 0 && MINOCC * 4 >= WAVES_M * WAVES_N, "whole workgroups per compute unit");
    const int64_t grid = tm * tn < resident ? tm * tn : resident;
    hipLaunchKernelGGL((gemm_w4a4_fp6_kernel<BM, BN, WAVES_M, WAVES_N, STAGES, MINOCC>), dim3((unsigned)grid),
                       dim3(WAVES_M * WAVES_N * 64), 0, s, a, (int)tm, (int)tn);
    return check_hip(hipGetLastError(), "w4a4_gemm (fp6) launch");
}

double round_efficiency6(int64_t tiles, int64_t slots) {
    const int64_t rounds = (tiles + slots - 1) / slots;
    return (double)tiles / (double)(rounds * slots);
}

}  // namespace

bool gemm_fp6_applicable(const GemmArgs& a) {
    // buffer addressing: both operands must be smaller than 4 GiB.  K <= 32768: the fp32 accumulator holds the sum of
    // K products of (q_a/8)(q_w/8) -- multiples of 1/64 up to 225 K / 64 -- exactly only while 225 K < 2^24; longer
    // rows take the int8 path, whose INT32 accumulator has no such limit.
    return a.Aq6 && a.Wq6 && a.K % 128 == 0 && a.K <= 32768 && a.M >= 1 &&
           (int64_t)basq_fp6_bytes(a.M, a.K) < 0xFFFFFFFFll && (int64_t)basq_fp6_bytes(a.N, a.K) < 0xFFFFFFFFll;
}

int launch_gemm_fp6(const GemmArgs& a, hipStream_t s) {
#ifdef GEMM_FP6_CFG
    return launch_fp6<GEMM_FP6_CFG>(a, s);
#else
    auto tiles = [&](int bm, int bn) { return ((a.M + bm - 1) / bm) * (((int64_t)a.N + bn - 1) / bn); };
    // Three tilings, chosen by how evenly their tiles fill the 256 compute units, weighted by the per-tile rate
    // measured against the square 256 tile (256 x 192: wave tiles of 64 x 96, 0.90; 128 x 128: 0.85)
    const double s_big = 1.00 * round_efficiency6(tiles(256, 256), 256);
    const double s_mid = 0.90 * round_efficiency6(tiles(256, 192), 256);
    const double s_small = 0.85 * round_efficiency6(tiles(128, 128), 512);
    if (s_big >= s_mid && s_big >= s_small) return launch_fp6<256, 256, 2, 4, 3, 2>(a, s);
    if (s_mid >= s_small) return launch_fp6<256, 192, 4, 2, 3, 2>(a, s);
    return launch_fp6<128, 128, 2, 2, 3, 2>(a, s);
#endif
}

}  // namespace basq
