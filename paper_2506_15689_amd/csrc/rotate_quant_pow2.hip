// Fast rotate + bias + quantise kernel for rot_size == K in {4096, 8192}: one wavefront per token,
// the token never leaves registers except for one wave-private LDS transpose (the per-token routine and
// its layout notes are in rotate_pow2_token.h; paper Sec. 3.1 rotation, Eq. 14 bias, Eq. 4 quantiser).
#include "rotate_pow2_token.h"

namespace basq {

namespace {

#ifndef P2_WAVES_CFG
#define P2_WAVES_CFG 4
#endif
constexpr int P2_WAVES = P2_WAVES_CFG;      // wavefronts per workgroup
constexpr int P2_THREADS = P2_WAVES * 64;
#ifndef P2_OCC_4096
#define P2_OCC_4096 3
#endif
#ifndef P2_PREFETCH
#define P2_PREFETCH 1
#endif

// NC: 16-byte loads per lane per token (K = 512 * NC).  FOLD_NORM: 1/sqrt(K) is a power of two and
// sits in the MFMA matrix; otherwise one fp32 multiply by `norm` follows the butterflies.
// GROUPED: one range and one record per 128 channels (group_size = 128) instead of per token.
template <int NC, bool FOLD_NORM, bool HAS_BIAS, bool HAS_SCALE, bool ROT_OUT, bool GROUPED>
__global__ __launch_bounds__(P2_THREADS, (NC == 8 ? P2_OCC_4096 : 2)) void rotate_quant_pow2_kernel(RotateQuantArgs a, float norm) {
    constexpr int K = 512 * NC;
    constexpr bool PREFETCH = (NC == 8) && P2_PREFETCH;
    // per-wave transpose buffers, then the channel bias (shared by the workgroup's waves)
    constexpr int BIAS_WORDS = HAS_BIAS ? K : 0;
    __shared__ __attribute__((aligned(16))) float lds[P2_WAVES * P2_LDS_WORDS + BIAS_WORDS];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float* wl = lds + wave * P2_LDS_WORDS;
    const float4* lbias = reinterpret_cast<const float4*>(lds + P2_WAVES * P2_LDS_WORDS);
    v8bf bop[2];
    p2_make_bop<NC, FOLD_NORM>(lane, bop);
    const P2Lane pl = p2_lane(lane);

    // Workgroups g, g+8, g+16, ... run on one XCD.  Renumbering them so that an XCD owns a contiguous
    // range makes 32 consecutive tokens (one block of the fp6 output) meet in one L2, where their 8- and
    // 16-byte pieces merge into whole lines before they are written back.
    int vblock = blockIdx.x;
    if (a.Aq6 && (gridDim.x & 63) == 0) vblock = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    const int wave_id = vblock * P2_WAVES + wave;
    const int wave_stride = gridDim.x * P2_WAVES;
    const int64_t rb6 = (a.M + 31) >> 5;                       // 32-row blocks per chunk of the fp6 output

    uint4 raw[NC];
    auto load_token = [&](int64_t m) {
        const uint16_t* x = a.X + m * a.ldx + 8 * pl.chunk;
#pragma unroll
        for (int c = 0; c < NC; ++c) raw[c] = nt_load16(x + 512 * c);
    };

    // K = 4096: the first token is requested before the bias is staged, so that the two latencies overlap
    // (K = 8192 has no registers to carry a token across the loop edge)
    int64_t m = wave_id;
    if (PREFETCH && m < a.M) load_token(m);
    if (HAS_BIAS) {
        p2_stage_bias<K>(lds + P2_WAVES * P2_LDS_WORDS, a.bias, threadIdx.x, P2_THREADS);
        __syncthreads();
    }

    for (; m < a.M; m += wave_stride) {
        if (!PREFETCH) load_token(m);
        const int64_t mnext = m + wave_stride;
        const P2Meta tm = p2_token<NC, FOLD_NORM, HAS_BIAS, HAS_SCALE, ROT_OUT, GROUPED>(
            raw, bop, wl, lbias, a.act_scale, ROT_OUT ? a.rot_out + m * (int64_t)K : nullptr, norm, a.clip_lo, a.clip_hi,
            lane, pl.wbase, pl.rbase,
            // prefetch the next token of this wave while the rest is computed (K = 4096: registers allow it)
            [&]() { if (PREFETCH && mnext < a.M) load_token(mnext); },
            [&](int hf, int b, const uint32_t (&words)[4], const v16f& te, const v16f& to) {
                uint8_t* dst = a.Aq + m * (int64_t)(K / 2) + 2048 * hf + 1024 * b + 16 * lane;
                nt_store16(dst, make_uint4(words[0], words[1], words[2], words[3]));
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
}

template <int NC, bool FOLD, bool HB, bool HS>
int launch_flags(const RotateQuantArgs& a, hipStream_t s, unsigned blocks, float norm) {
    const bool grouped = a.group != a.K;
    if (a.rot_out && grouped)
        hipLaunchKernelGGL((rotate_quant_pow2_kernel<NC, FOLD, HB, HS, true, true>), dim3(blocks), dim3(P2_THREADS), 0, s, a, norm);
    else if (grouped)
        hipLaunchKernelGGL((rotate_quant_pow2_kernel<NC, FOLD, HB, HS, false, true>), dim3(blocks), dim3(P2_THREADS), 0, s, a, norm);
    else if (a.rot_out)
        hipLaunchKernelGGL((rotate_quant_pow2_kernel<NC, FOLD, HB, HS, true, false>), dim3(blocks), dim3(P2_THREADS), 0, s, a, norm);
    else
        hipLaunchKernelGGL((rotate_quant_pow2_kernel<NC, FOLD, HB, HS, false, false>), dim3(blocks), dim3(P2_THREADS), 0, s, a, norm);
    return check_hip(hipGetLastError(), "rotate_quant (pow2) launch");
}

template <int NC, bool FOLD>
int launch_nc(const RotateQuantArgs& a, hipStream_t s, unsigned blocks, float norm) {
    const bool hb = a.bias != nullptr, hs = a.act_scale != nullptr;
    if (hb && hs) return launch_flags<NC, FOLD, true, true>(a, s, blocks, norm);
    if (hb) return launch_flags<NC, FOLD, true, false>(a, s, blocks, norm);
    if (hs) return launch_flags<NC, FOLD, false, true>(a, s, blocks, norm);
    return launch_flags<NC, FOLD, false, false>(a, s, blocks, norm);
}

}  // namespace

bool rotate_quant_pow2_applicable(const RotateQuantArgs& a) {
    // per-token ranges, or groups of 128 channels (four neighbouring lanes; no fp6 copy: the GEMM that takes it is per token)
    return (a.group == a.K || (a.group == 128 && a.Aq6 == nullptr)) && !a.has28 && a.rot_size == a.K &&
           (a.K == 4096 || a.K == 8192) && a.Aq != nullptr && a.meta != nullptr;
}

int launch_rotate_quant_pow2(const RotateQuantArgs& a, hipStream_t s) {
    const int64_t want = (a.M + P2_WAVES - 1) / P2_WAVES;
    const int64_t resident = 256 * (a.K == 4096 ? P2_OCC_4096 : 2) * 4 / P2_WAVES;  // workgroups the chip holds at once
    const unsigned blocks = (unsigned)(want < resident ? want : resident);   // waves loop over tokens
    const float norm = (float)(1.0 / sqrt((double)a.K));
    if (a.K == 4096) return launch_nc<8, true>(a, s, blocks, norm);
    return launch_nc<16, false>(a, s, blocks, norm);
}

}  // namespace basq
