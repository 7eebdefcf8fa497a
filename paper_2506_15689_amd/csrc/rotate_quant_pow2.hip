// Fast rotate + bias + quantise kernel for rot_size == K in {4096, 8192}: one wavefront per token,
// the token never leaves registers except for one wave-private LDS transpose (the per-token routine and
// its layout notes are in rotate_pow2_token.h; paper Sec. 3.1 rotation, Eq. 14 bias, Eq. 4 quantiser).
#include "rotate_pow2_token.h"

namespace basq {

namespace {

// Waves per SIMD the kernel is compiled for: three (168 registers) for the plain K = 4096 four-wave variant, two (256)
// for everything else -- K = 8192, and the variants that keep more per lane (group ranges, the fp32 rotation output)
// and would spill at 168.
constexpr int p2_waves_per_simd(int nc, int waves, bool rot_out, bool grouped) {
    return (nc == 8 && waves == 4 && !rot_out && !grouped) ? 3 : 2;
}

// NC: 16-byte loads per lane per token (K = 512 * NC).  FOLD_NORM: 1/sqrt(K) is a power of two and
// sits in the MFMA matrix; otherwise one fp32 multiply by `norm` follows the butterflies.
// GROUPED: one range and one record per 128 channels (group_size = 128) instead of per token.
// WAVES: wavefronts (= tokens in flight) per workgroup, 4 or 8.  Eight halve the number of workgroups that each
// stage the channel bias, which shows at a few thousand tokens; K = 4096 then runs two waves per SIMD instead of
// three, which costs 3 % at very large M.
// STAGE_TAILS (WAVES = 8, with the fp6 copy): the 8-byte tail pieces of the fp6 form are collected in LDS and
// leave as the 64 contiguous bytes that the workgroup's eight consecutive tokens own in every tail row.  An 8-byte
// store is one request to the L2 however it is aligned, and with them a token makes 385 write requests instead
// of 65; staged it is 161 (measured: 65536 tokens of K = 4096 in 170 us against 222 us).  The two barriers per
// round cost more than that saves below about 32768 tokens.
template <int NC, bool FOLD_NORM, bool HAS_BIAS, bool HAS_SCALE, bool ROT_OUT, bool GROUPED, int WAVES, bool STAGE_TAILS>
__global__ __launch_bounds__(WAVES * 64, p2_waves_per_simd(NC, WAVES, ROT_OUT, GROUPED)) void rotate_quant_pow2_kernel(RotateQuantArgs a, float norm) {
    constexpr int K = 512 * NC;
    constexpr int THREADS = WAVES * 64;
    constexpr bool PREFETCH = (NC == 8);
    static_assert(WAVES == 4 || WAVES == 8, "workgroups of four or eight wavefronts");
    static_assert(!STAGE_TAILS || (WAVES == 8 && !GROUPED), "the staged tails are those of eight consecutive tokens");
    // the channel bias and the channel scale (shared by the workgroup's waves; first, so that their reads are the
    // array's base plus a constant an LDS instruction can carry: offsets up to 64 KB), then the per-wave transpose
    // buffers, then the tail stage
    constexpr int BIAS_WORDS = HAS_BIAS ? K : 0;
    constexpr int SCALE_WORDS = HAS_SCALE ? K : 0;
    constexpr int VEC_WORDS = BIAS_WORDS + SCALE_WORDS;
    constexpr int TS_BYTES = STAGE_TAILS ? (K / 32) * WAVES * 8 : 0;      // per 32-channel group: 8 bytes per token
    __shared__ __attribute__((aligned(16))) float lds[VEC_WORDS + WAVES * P2_LDS_WORDS + TS_BYTES / 4];
    uint8_t* const tstage = reinterpret_cast<uint8_t*>(lds + VEC_WORDS + WAVES * P2_LDS_WORDS);

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float* wl = lds + VEC_WORDS + wave * P2_LDS_WORDS;
    const float4* lbias = reinterpret_cast<const float4*>(lds);
    const float4* lscale = reinterpret_cast<const float4*>(lds + BIAS_WORDS);
    v8bf bop[2];
    p2_make_bop<NC, FOLD_NORM>(lane, bop);
    const P2Lane pl = p2_lane(lane);

    // Workgroups g, g+8, g+16, ... run on one XCD.  Renumbering them so that an XCD owns a contiguous
    // range makes 32 consecutive tokens (one block of the fp6 output) meet in one L2, where their 8- and
    // 16-byte pieces merge into whole lines before they are written back.
    int vblock = blockIdx.x;
    if (a.Aq6 && (gridDim.x & 63) == 0) vblock = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    const int wave_id = vblock * WAVES + wave;
    const int wave_stride = gridDim.x * WAVES;
    const int64_t rb6 = (a.M + 31) >> 5;                       // 32-row blocks per chunk of the fp6 output

    uint4 raw[NC];
    auto load_token = [&](int64_t m) {
        const uint16_t* x = a.X + m * a.ldx + 8 * pl.chunk;
#pragma unroll
        for (int c = 0; c < NC; ++c) raw[c] = nt_load16(x + 512 * c);
    };

    // K = 4096: the first token is requested before the bias is staged, so that the two latencies overlap
    // (K = 8192 has no registers to carry a token across the loop edge: even a first token requested here keeps its
    // 64 registers live around the loop and the kernel spills)
    int64_t m = wave_id;
    if (PREFETCH && m < a.M) load_token(m);
    if (HAS_BIAS) p2_stage_bias<K>(lds, a.bias, threadIdx.x, THREADS);
    if (HAS_SCALE) p2_stage_bias<K>(lds + BIAS_WORDS, a.act_scale, threadIdx.x, THREADS);
    if (HAS_BIAS || HAS_SCALE) __syncthreads();

    // One round per iteration: the workgroup's waves take WAVES consecutive tokens (a whole number of rounds for
    // every wave, since the staged variant meets at barriers).
    for (int64_t mbase = (int64_t)vblock * WAVES; mbase < a.M; mbase += wave_stride, m += wave_stride) {
      if (m < a.M) {
        if (!PREFETCH) load_token(m);
        const int64_t mnext = m + wave_stride;
        const P2Meta tm = p2_token<NC, FOLD_NORM, HAS_BIAS, HAS_SCALE, ROT_OUT, GROUPED>(
            raw, bop, wl, lbias, lscale, ROT_OUT ? a.rot_out + m * (int64_t)K : nullptr, norm, a.clip_lo, a.clip_hi,
            lane, pl.wbase, pl.rbase,
            // prefetch the next token of this wave while the rest is computed (K = 4096: registers allow it)
            [&]() { if (PREFETCH && mnext < a.M) load_token(mnext); },
            [&](int hf, int b, const uint32_t (&words)[4], const v16f& te, const v16f& to) {
                // the 4-bit form is optional when the fp6 form is written (the one-call layer on the fp6 path reads only that)
                if (a.Aq) nt_store16(a.Aq + m * (int64_t)(K / 2) + 2048 * hf + 1024 * b + 16 * lane,
                                     make_uint4(words[0], words[1], words[2], words[3]));
                if (a.Aq6) {
                    // The same 32 codes as e2m3 numbers q/8, straight from the clamped values t in [0, 15]: the
                    // packed conversion divides by its scale operand, rounds to nearest-even -- on the e2m3 grid
                    // below 2 that is t/8 -> rint(t)/8, ties to the even code as in the integer conversion -- and
                    // interleaves its two sources (even and odd channels).
                    const v6i f6 = __builtin_amdgcn_cvt_scalef32_2xpk16_fp6_f32(te, to, 8.0f);
                    // group 128*hf + 64*b + lane of the token: chunk (group / 4), position (group % 4)
                    const int g = 128 * hf + 64 * b + lane, f = g & 3, r = (int)(m & 31);
                    uint8_t* blk = a.Aq6 + ((int64_t)(g >> 2) * rb6 + (m >> 5)) * 3072;
                    *reinterpret_cast<uint4*>(blk + 64 * r + 16 * (f ^ ((r >> 2) & 3))) =
                        make_uint4((uint32_t)f6[0], (uint32_t)f6[1], (uint32_t)f6[2], (uint32_t)f6[3]);
                    if (STAGE_TAILS)     // slot of this wave's token in the group's 64 bytes, swizzled against bank conflicts
                        *reinterpret_cast<uint2*>(tstage + g * (WAVES * 8) + 8 * (wave ^ ((g >> 1) & 7))) =
                            make_uint2((uint32_t)f6[4], (uint32_t)f6[5]);
                    else
                        *reinterpret_cast<uint2*>(blk + 2048 + 256 * f + 8 * r) = make_uint2((uint32_t)f6[4], (uint32_t)f6[5]);
                }
            },
            [&](int hf, int b, float gs, float glo, int gsum) {
                if ((lane & 3) == 0) {
                    basq_tokmeta mt;
                    mt.scale = gs; mt.lo = glo; mt.rowsum = gsum; mt.reserved = 0;
                    a.meta[m * (K / 128) + 32 * hf + 16 * b + (lane >> 2)] = mt;
                }
            });
        if (!GROUPED && lane == 0) {
            basq_tokmeta mt;
            mt.scale = tm.scale; mt.lo = tm.lo; mt.rowsum = tm.rowsum; mt.reserved = 0;
            a.meta[m] = mt;
        }
      }
      if (STAGE_TAILS && a.Aq6) {
        // the tails of tokens mbase .. mbase + 7 (one 32-row block: mbase is a multiple of 8): 16 bytes per thread,
        // four neighbouring threads write the 64 bytes of one group
        __syncthreads();
        constexpr int PIECES = TS_BYTES / 16;
        for (int p = threadIdx.x; p < PIECES; p += THREADS) {
            const int g = p / (WAVES / 2), q = p % (WAVES / 2);          // tokens mbase + 2q, + 2q + 1 of group g
            const int64_t mt = mbase + 2 * q;
            if (mt < a.M) {
                const int sw = (g >> 1) & 7;
                const uint2 v0 = *reinterpret_cast<const uint2*>(tstage + g * (WAVES * 8) + 8 * ((2 * q) ^ sw));
                const uint2 v1 = *reinterpret_cast<const uint2*>(tstage + g * (WAVES * 8) + 8 * ((2 * q + 1) ^ sw));
                uint8_t* dst = a.Aq6 + ((int64_t)(g >> 2) * rb6 + (mbase >> 5)) * 3072 + 2048 + 256 * (g & 3) + 8 * (int)(mt & 31);
                if (mt + 1 < a.M) *reinterpret_cast<uint4*>(dst) = make_uint4(v0.x, v0.y, v1.x, v1.y);
                else *reinterpret_cast<uint2*>(dst) = v0;
            }
        }
        __syncthreads();                 // the next round's tails go to the same stage
      }
    }
}

// Few tokens: NWAY = NC / 4 waves per token (p2_token_split; two for K = 4096, four for K = 8192), 4 / NWAY tokens per
// workgroup, one round.  A call this small is all latency -- one wave needs about 2.8 us (5.6 us) for a token -- and
// the split divides the chain.
template <int NC, bool HAS_BIAS, bool HAS_SCALE>
__global__ __launch_bounds__(256) void rotate_quant_pow2_split_kernel(RotateQuantArgs a, float norm) {
    constexpr int K = 512 * NC, NWAY = NC / 4, TOKENS = 4 / NWAY;
    __shared__ __attribute__((aligned(16))) float tr[4 * P2_LDS_WORDS];
    __shared__ __attribute__((aligned(16))) float lbias_s[HAS_BIAS ? K : 4];
    __shared__ __attribute__((aligned(16))) float lscale_s[HAS_SCALE ? K : 4];
    __shared__ __attribute__((aligned(16))) float4 xch[4 * 512];
    __shared__ float lred[8];
    __shared__ int lsum[TOKENS];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tl = wave / NWAY, part = wave % NWAY;
    const int64_t m = (int64_t)blockIdx.x * TOKENS + tl;
    const bool active = m < a.M;
    if (tid < TOKENS) lsum[tid] = 0;
    v8bf bop[2];
    p2_make_bop<NC, NC == 8>(lane, bop);
    const P2Lane pl = p2_lane(lane);
    uint4 raw4[4] = {};
    if (active) {
        const uint16_t* x = a.X + m * a.ldx + 8 * pl.chunk + 2048 * part;
#pragma unroll
        for (int j = 0; j < 4; ++j) raw4[j] = nt_load16(x + 512 * j);
    }
    if (HAS_BIAS) p2_stage_bias<K>(lbias_s, a.bias, tid, 256);          // complete behind the routine's first barrier
    if (HAS_SCALE) p2_stage_bias<K>(lscale_s, a.act_scale, tid, 256);
    const P2Meta tm = p2_token_split<NWAY, NC == 8, HAS_BIAS, HAS_SCALE>(
        active, part, raw4, bop, tr + wave * P2_LDS_WORDS, xch + tl * (NWAY * 512), lred + tl * (NWAY * 2),
        reinterpret_cast<const float4*>(lbias_s), reinterpret_cast<const float4*>(lscale_s), norm, a.clip_lo, a.clip_hi, lane,
        pl.wbase, pl.rbase, [&](const uint32_t (&words)[4], const v16f& te, const v16f& to) {
            if (a.Aq) nt_store16(a.Aq + m * (int64_t)(K / 2) + 1024 * part + 16 * lane, make_uint4(words[0], words[1], words[2], words[3]));
            if (a.Aq6) {      // the fp6 copy, as in the one-wave kernel: group 64*part + lane of the token
                const v6i f6 = __builtin_amdgcn_cvt_scalef32_2xpk16_fp6_f32(te, to, 8.0f);
                const int g = 64 * part + lane, f = g & 3, r = (int)(m & 31);
                uint8_t* blk = a.Aq6 + ((int64_t)(g >> 2) * ((a.M + 31) >> 5) + (m >> 5)) * 3072;
                *reinterpret_cast<uint4*>(blk + 64 * r + 16 * (f ^ ((r >> 2) & 3))) =
                    make_uint4((uint32_t)f6[0], (uint32_t)f6[1], (uint32_t)f6[2], (uint32_t)f6[3]);
                *reinterpret_cast<uint2*>(blk + 2048 + 256 * f + 8 * r) = make_uint2((uint32_t)f6[4], (uint32_t)f6[5]);
            }
        });
    if (active && part != 0 && lane == 0) atomicAdd(&lsum[tl], tm.rowsum);    // LDS integer adds: order-free
    __syncthreads();
    if (active && part == 0 && lane == 0) {
        basq_tokmeta mt;
        mt.scale = tm.scale; mt.lo = tm.lo; mt.rowsum = tm.rowsum + lsum[tl]; mt.reserved = 0;
        a.meta[m] = mt;
    }
}

#ifndef P2_SPLIT_MAX_TOKENS_4096
#define P2_SPLIT_MAX_TOKENS_4096 512      // measured: 4.6-5.6 us against 5.4-6.3 us up to here, slower from 1024 on
#endif
#ifndef P2_SPLIT_MAX_TOKENS_8192
#define P2_SPLIT_MAX_TOKENS_8192 256
#endif

template <int NC, bool FOLD, bool HB, bool HS, bool RO, bool GR, int WAVES, bool STAGE>
int launch_one(const RotateQuantArgs& a, hipStream_t s, float norm) {
    const int64_t want = (a.M + WAVES - 1) / WAVES;
    // workgroups the chip holds at once: by registers (the launch bounds) and by the 160 KB of LDS per compute unit
    constexpr int K = 512 * NC;
    constexpr int LDS_BYTES = 4 * (WAVES * P2_LDS_WORDS + (HB ? K : 0) + (HS ? K : 0)) + (STAGE ? (K / 32) * WAVES * 8 : 0);
    constexpr int BY_REGS = p2_waves_per_simd(NC, WAVES, RO, GR) * 4 / WAVES, BY_LDS = 163840 / LDS_BYTES;
    static_assert(BY_LDS >= 1, "the kernel's LDS must fit a compute unit");
    const int64_t resident = 256 * (BY_REGS < BY_LDS ? BY_REGS : BY_LDS);
    const unsigned blocks = (unsigned)(want < resident ? want : resident);        // waves loop over tokens
    hipLaunchKernelGGL((rotate_quant_pow2_kernel<NC, FOLD, HB, HS, RO, GR, WAVES, STAGE>), dim3(blocks), dim3(WAVES * 64), 0, s, a, norm);
    return check_hip(hipGetLastError(), "rotate_quant (pow2) launch");
}

template <int NC, bool FOLD, bool HB, bool HS>
int launch_flags(const RotateQuantArgs& a, hipStream_t s, float norm) {
    const bool grouped = a.group != a.K;
    if (a.rot_out && grouped) return launch_one<NC, FOLD, HB, HS, true, true, 4, false>(a, s, norm);
    if (grouped) return launch_one<NC, FOLD, HB, HS, false, true, 4, false>(a, s, norm);
    if (a.rot_out) return launch_one<NC, FOLD, HB, HS, true, false, 4, false>(a, s, norm);
    if (a.M <= (NC == 8 ? P2_SPLIT_MAX_TOKENS_4096 : P2_SPLIT_MAX_TOKENS_8192)) {
        constexpr int TOKENS = 16 / NC;                                   // per workgroup of four waves
        hipLaunchKernelGGL((rotate_quant_pow2_split_kernel<NC, HB, HS>), dim3((unsigned)((a.M + TOKENS - 1) / TOKENS)),
                           dim3(256), 0, s, a, norm);
        return check_hip(hipGetLastError(), "rotate_quant (pow2, split) launch");
    }
    // measured: the tail stage pays from about 32768 tokens on.  Without it, eight waves per workgroup help from 2048
    // tokens (fewer workgroups stage the bias; below that, four-wave workgroups spread the tokens over more compute
    // units, one wave per SIMD, which is worth 1-2 us) up to 32768 tokens for K = 4096 (10 % at 2048 .. 16384) and up
    // to 4096 for K = 8192 (4-10 %), and are neutral or slightly worse beyond.
    if (a.Aq6 && a.M >= 32768) return launch_one<NC, FOLD, HB, HS, false, false, 8, true>(a, s, norm);
    if (a.M >= 2048 && ((NC == 8 && a.M < 32768) || (NC == 16 && a.M <= 4096))) return launch_one<NC, FOLD, HB, HS, false, false, 8, false>(a, s, norm);
    // K = 8192 with s^a staged next to b^c: a four-wave workgroup's 96 KB leave room for one per compute unit, one
    // wave per SIMD; eight waves share the two vectors
    if (NC == 16 && HS && a.M > 1024) return launch_one<NC, FOLD, HB, HS, false, false, 8, false>(a, s, norm);
    return launch_one<NC, FOLD, HB, HS, false, false, 4, false>(a, s, norm);
}

template <int NC, bool FOLD>
int launch_nc(const RotateQuantArgs& a, hipStream_t s, float norm) {
    const bool hb = a.bias != nullptr, hs = a.act_scale != nullptr;
    if (hb && hs) return launch_flags<NC, FOLD, true, true>(a, s, norm);
    if (hb) return launch_flags<NC, FOLD, true, false>(a, s, norm);
    if (hs) return launch_flags<NC, FOLD, false, true>(a, s, norm);
    return launch_flags<NC, FOLD, false, false>(a, s, norm);
}

}  // namespace

bool rotate_quant_pow2_applicable(const RotateQuantArgs& a) {
    // per-token ranges, or groups of 128 channels (four neighbouring lanes; no fp6 copy: the GEMM that takes it is per token)
    // (the 4-bit codes may be left out when the fp6 form is written)
    return (a.group == a.K || (a.group == 128 && a.Aq6 == nullptr)) && !a.has28 && a.rot_size == a.K &&
           (a.K == 4096 || a.K == 8192) && (a.Aq != nullptr || a.Aq6 != nullptr) && a.meta != nullptr;
}

int launch_rotate_quant_pow2(const RotateQuantArgs& a, hipStream_t s) {
    const float norm = (float)(1.0 / sqrt((double)a.K));
    if (a.K == 4096) return launch_nc<8, true>(a, s, norm);
    return launch_nc<16, false>(a, s, norm);
}

}  // namespace basq
