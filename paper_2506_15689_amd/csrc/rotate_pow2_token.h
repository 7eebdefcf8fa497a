// One token through rotate + bias + quantise for rot_size == K in {4096, 8192}, by one wavefront, in
// registers except for one wave-private LDS transpose.  Shared by the rotate+quant kernel (which writes the
// codes to memory) and by the one-launch decode kernel (which keeps them in LDS for the weight stream).
// (Paper Sec. 5.2 applies the online Hadamard as matrix products on the matrix cores instead of a
// pure butterfly recursion; here the first five stages are one bf16 MFMA -- exact, since the inputs
// are bf16 and the matrix entries are +-2^-6 or +-1 -- and the remaining stages are fp32
// butterflies in registers.  Quantiser: Eq. 4 with the per-token range of Sec. 5.)
//
// Channel index e (12 bits for K = 4096; bit 12 for K = 8192 rides along in registers).
//   load      lane l reads 8 consecutive bf16 (16 B); 8 (16) loads of 1 KB each per token.
//             e = 512*c + 8*chunk(l) + t,  chunk bits (e3..e8) <- lane bits (2,3,0,1,4,5)
//   MFMA      D = A.B, A = the 16 x 32 slice of the token (row = l%16, k = 8*(l/16) + t), B = H_32
//             over the index bits (e0,e1,e2,e7,e8), columns permuted so that output bit e0 lands
//             in the half index h and (e1,e2,e7,e8) in output lane bits 0..3.
//             After it a lane holds d[c][h][r]: e0 = h, (e5,e6) = r, (e9..) = c,
//             lane bits (0,1,2,3,4,5) = (e1,e2,e7,e8,e3,e4).
//   stages    e5, e6, e9, e10, e11 (, e12) in registers.
//   transpose through LDS (8 KB per wave, reused per 2048 channels, 8-byte accesses, no bank conflicts) to the layout
//             lane bits (0..5) = (e5..e10), registers = (e0..e4, e11 (, e12)).
//   stages    e3, e4 in registers.
//   now a lane owns 32 consecutive channels (x2 or x4): bias, min/max, quantise, pack.
#ifndef BASQ_ROTATE_POW2_TOKEN_H
#define BASQ_ROTATE_POW2_TOKEN_H

#include "basq_internal.h"

namespace basq {
namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef int v6i __attribute__((ext_vector_type(6)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef short v8s __attribute__((ext_vector_type(8)));

constexpr int P2_LDS_WORDS = 2048;          // transpose buffer per wave, in floats

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
template <int CTRL>
__device__ __forceinline__ int dpp_i(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, false);
}
constexpr int DPP_QUAD_XOR1 = 0xB1;         // quad_perm [1,0,3,2]
constexpr int DPP_QUAD_XOR2 = 0x4E;         // quad_perm [2,3,0,1]
constexpr int DPP_ROW_HALF_MIRROR = 0x141;
constexpr int DPP_ROW_MIRROR = 0x140;

__device__ __forceinline__ float wave_min_f(float v) {
    v = fminf(v, dpp_f<DPP_QUAD_XOR1>(v));
    v = fminf(v, dpp_f<DPP_QUAD_XOR2>(v));
    v = fminf(v, dpp_f<DPP_ROW_HALF_MIRROR>(v));
    v = fminf(v, dpp_f<DPP_ROW_MIRROR>(v));
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
    return fminf(fminf(r0, r1), fminf(r2, r3));
}
__device__ __forceinline__ float wave_max_f(float v) {
    v = fmaxf(v, dpp_f<DPP_QUAD_XOR1>(v));
    v = fmaxf(v, dpp_f<DPP_QUAD_XOR2>(v));
    v = fmaxf(v, dpp_f<DPP_ROW_HALF_MIRROR>(v));
    v = fmaxf(v, dpp_f<DPP_ROW_MIRROR>(v));
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
    return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}
__device__ __forceinline__ int wave_sum_i(int v) {
    v += dpp_i<DPP_QUAD_XOR1>(v);
    v += dpp_i<DPP_QUAD_XOR2>(v);
    v += dpp_i<DPP_ROW_HALF_MIRROR>(v);
    v += dpp_i<DPP_ROW_MIRROR>(v);
    return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) +
           __builtin_amdgcn_readlane(v, 32) + __builtin_amdgcn_readlane(v, 48);
}

#define BFLY(x, y) do { const float _a = (x), _b = (y); (x) = _a + _b; (y) = _a - _b; } while (0)

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every global load the wave has
// in flight, which here may be a caller's prefetch (the weight stream of the one-launch decode kernel) that nothing
// on the other side of the barrier reads.
__device__ __forceinline__ void p2_lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Per-lane constants of the routine.
struct P2Lane {
    int chunk;      // global load: 16-byte chunk of the lane inside each 1 KB; bits (e3,e4,e5,e6,e7,e8) <- lane bits (2,3,0,1,4,5)
    int wbase;      // LDS write base (words), lane bits (0..5) = (e1,e2,e7,e8,e3,e4); address map at the transpose
    int rbase;      // LDS read base, lane bits (0..5) = (e5..e10)
};
__device__ __forceinline__ P2Lane p2_lane(int lane) {
    P2Lane c;
    c.chunk = ((lane >> 2) & 3) | ((lane & 3) << 2) | (lane & 0x30);
    c.wbase = ((lane & 15) << 1) | (((lane >> 4) & 3) << 7);
    c.rbase = ((lane & 15) << 1) | ((lane & 3) << 5) | (((lane >> 4) & 3) << 9);
    return c;
}

// B operand of the MFMA: column j' = lane%16 of half h, k = 8*(lane/16) + t; input index bits (t0,t1,t2,g0,g1),
// output index bits (h, j'0, j'1, j'2, j'3): sign = parity(popcount(kin & jout)).  FOLD_NORM: 1/sqrt(K) is a
// power of two and sits in the matrix.
template <int NC, bool FOLD_NORM>
__device__ __forceinline__ void p2_make_bop(int lane, v8bf (&bop)[2]) {
    const int jp = lane & 15, g = lane >> 4;
    const uint16_t mag = FOLD_NORM ? (uint16_t)(((127 - (NC == 8 ? 6 : 0)) << 7)) : (uint16_t)0x3F80;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        v8s tmp;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int kin = t | (g << 3), jout = h | (jp << 1);
            tmp[t] = (short)(mag | ((__builtin_popcount(kin & jout) & 1) ? 0x8000 : 0));
        }
        bop[h] = __builtin_bit_cast(v8bf, tmp);
    }
}

// A per-channel vector (the channel bias b^c, the scale s^a) staged in LDS so that lane l's i-th 16-byte piece sits at
// float4 index (piece group)*64 + l: conflict-free reads.  Called by all `nthreads` threads of the workgroup; the
// caller synchronises afterwards.
template <int K>
__device__ __forceinline__ void p2_stage_bias(float* lds_bias, const float* bias, int tid, int nthreads) {
    float4* dst = reinterpret_cast<float4*>(lds_bias);
    for (int f = tid; f < K / 4; f += nthreads) {
        const int e = 4 * f;                          // channels e .. e+3 belong to lane (e%2048)/32, piece (e%32)/4
        dst[((e >> 11) * 8 + ((e & 31) >> 2)) * 64 + ((e & 2047) >> 5)] = *reinterpret_cast<const float4*>(bias + e);
    }
}

struct P2Meta { float scale, lo; int rowsum; };

// raw: the token as loaded with P2Lane::chunk (raw[c] = 16 bytes at channel 512*c + 8*chunk).  wl: this wave's
// P2_LDS_WORDS floats.  lbias, lscale: b^c and s^a as staged by p2_stage_bias (s^a read from memory here would be
// a load per 16 bytes behind whatever the caller has in flight -- its prefetched next token, a weight stream --
// and loads complete in issue order).  rot_row: where the fp32 rotation of this token goes (ROT_OUT).
// after_mfma(): called once raw[] is dead.  sink(hf, b, words, te, to): the 32 codes of channels
// 4096*hf + 2048*b + 32*lane .. +31 -- words: packed two per byte (16 bytes); te[i] / to[i]: the clamped but not
// yet rounded value fma(v, inv, nlo) in [0, 15] of channel 2i / 2i + 1, whose rounding to nearest-even is the code
// (for callers that want the codes in another number format: a conversion that rounds the same way gives them).
// NC: 16-byte loads per lane per token (K = 512 * NC).  Without FOLD_NORM one fp32 multiply by `norm` follows
// the butterflies.
// GROUPED: one range per 128 consecutive channels instead of one per token (four neighbouring lanes own a group);
// gsink(hf, b, scale, lo, rowsum) then receives the record of group 32*hf + 16*b + lane/4 (the same values on
// the four lanes of the group) and the returned record is unused.
template <int NC, bool FOLD_NORM, bool HAS_BIAS, bool HAS_SCALE, bool ROT_OUT, bool GROUPED, class AfterMfma, class Sink,
          class GroupSink>
__device__ __forceinline__ P2Meta p2_token(uint4 (&raw)[NC], const v8bf (&bop)[2], float* wl, const float4* lbias,
                                           const float4* lscale, float* rot_row, float norm, float clip_lo,
                                           float clip_hi, int lane, int wbase, int rbase, AfterMfma&& after_mfma,
                                           Sink&& sink, GroupSink&& gsink) {
    constexpr int NH = NC / 8;                  // number of 4096-channel halves (bit 12)
    static_assert(NC == 8 || NC == 16, "K must be 4096 or 8192");
    // ---- first five stages on the matrix core ---------------------------------------------
    float d[NC][2][4];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const v8bf aop = __builtin_bit_cast(v8bf, raw[c]);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            v4f acc = {0.f, 0.f, 0.f, 0.f};
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aop, bop[h], acc, 0, 0, 0);
#pragma unroll
            for (int r = 0; r < 4; ++r) d[c][h][r] = acc[r];
        }
    }
    after_mfma();                  // raw[] is dead from here on: the caller may request its next token

    // ---- stages e5, e6 (r bits) and e9.. (c bits) --------------------------------------------
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            BFLY(d[c][h][0], d[c][h][1]);
            BFLY(d[c][h][2], d[c][h][3]);
            BFLY(d[c][h][0], d[c][h][2]);
            BFLY(d[c][h][1], d[c][h][3]);
        }
#pragma unroll
    for (int s = 1; s < NC; s <<= 1)
#pragma unroll
        for (int c = 0; c < NC; ++c)
            if ((c & s) == 0)
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int r = 0; r < 4; ++r) BFLY(d[c][h][r], d[c + s][h][r]);

    // ---- transpose through LDS, 2048 channels (one value of e11, e12) at a time ---------------------
    // word address bits: [0] = e0, [2:1] = (e1^e5, e2^e6), [4:3] = (e7,e8), [6:5] = (e5,e6),
    //                    [8:7] = (e3,e4), [10:9] = (e9,e10)
    // p[half][e11][idx], idx = e0..e4
    float p[NH][2][32];
#pragma unroll
    for (int hf = 0; hf < NH; ++hf)
#pragma unroll
        for (int c2 = 0; c2 < 2; ++c2) {
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int c01 = 0; c01 < 4; ++c01) {
                    const int r0 = r & 1, r1 = r >> 1;
                    const int addr = (wbase ^ ((r0 << 1) | (r1 << 2))) | (r0 << 5) | (r1 << 6) | (c01 << 9);
                    const int c = 8 * hf + 4 * c2 + c01;
                    *reinterpret_cast<float2*>(wl + addr) = make_float2(d[c][0][r], d[c][1][r]);
                }
            // LDS serves one wave's instructions in issue order: the reads below see these writes,
            // and the next round's writes do not overtake these reads
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const int e1 = q & 1, e2 = (q >> 1) & 1, e3 = (q >> 2) & 1, e4 = q >> 3;
                const int addr = (rbase ^ ((e1 << 1) | (e2 << 2))) | (e3 << 7) | (e4 << 8);
                const float2 v = *reinterpret_cast<const float2*>(wl + addr);
                const int idx = (e1 << 1) | (e2 << 2) | (e3 << 3) | (e4 << 4);
                p[hf][c2][idx] = v.x;
                p[hf][c2][idx | 1] = v.y;
            }
            __builtin_amdgcn_wave_barrier();
        }

    // ---- stages e3, e4 ----------------------------------------------------------------------
#pragma unroll
    for (int hf = 0; hf < NH; ++hf)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
#pragma unroll
            for (int i = 0; i < 32; ++i) if ((i & 8) == 0) BFLY(p[hf][b][i], p[hf][b][i | 8]);
#pragma unroll
            for (int i = 0; i < 32; ++i) if ((i & 16) == 0) BFLY(p[hf][b][i], p[hf][b][i | 16]);
        }
    // ---- normalise, bias, min/max; quantise, pack, store ------------------------------------------
    // this lane owns channels e = 4096*hf + 2048*b + 32*lane + i.  Per-token ranges take two passes over the blocks
    // (the range needs every value); with GROUPED a block is four lanes' own 128-channel group and is finished in
    // one go, which keeps fewer values live.
    float mn = INFINITY, mx = -INFINITY;
    auto prepare_block = [&](int hf, int b) {         // v = s^a r - b^c in place; widens (mn, mx)
        const int e0 = 4096 * hf + 2048 * b + 32 * lane;
#pragma unroll
        for (int i4 = 0; i4 < 8; ++i4) {
            float4 bb = make_float4(0.f, 0.f, 0.f, 0.f), ss = make_float4(1.f, 1.f, 1.f, 1.f);
            if (HAS_BIAS) bb = lbias[((2 * hf + b) * 8 + i4) * 64 + lane];
            if (HAS_SCALE) ss = lscale[((2 * hf + b) * 8 + i4) * 64 + lane];
            const float bv[4] = {bb.x, bb.y, bb.z, bb.w};
            const float sv[4] = {ss.x, ss.y, ss.z, ss.w};
            float rr[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float r = p[hf][b][4 * i4 + j];
                if (!FOLD_NORM) r = r * norm;
                rr[j] = r;
                const float v = HAS_SCALE ? fmaf(r, sv[j], -bv[j]) : r - bv[j];
                p[hf][b][4 * i4 + j] = v;
                mn = fminf(mn, v);
                mx = fmaxf(mx, v);
            }
            if (ROT_OUT)
                *reinterpret_cast<float4*>(rot_row + e0 + 4 * i4) =
                    make_float4(rr[0], rr[1], rr[2], rr[3]);
        }
    };

    // per-token constants, or (GROUPED) those of group (hf, b, lane/4)
    float lo, s, inv, nlo;
    auto range_constants = [&](float vmin, float vmax) {
        lo = clip_lo * vmin;
        const float hi = clip_hi * vmax;
        s = __fdiv_rn(hi - lo, 15.0f);
        if (!(s > 0.0f && s < INFINITY)) s = 1.0f;
        inv = __fdiv_rn(1.0f, s);
        nlo = -(lo * inv);
    };
    int sum = 0;
    auto quantise_block = [&](int hf, int b) {          // codes of the block with the current constants; adds to sum
        uint32_t words[4];
        v16f te, to;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            uint32_t ev = 0, od = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float t0 = __builtin_amdgcn_fmed3f(fmaf(p[hf][b][8 * w + 2 * j], inv, nlo), 0.0f, 15.0f);
                const float t1 = __builtin_amdgcn_fmed3f(fmaf(p[hf][b][8 * w + 2 * j + 1], inv, nlo), 0.0f, 15.0f);
                ev = __builtin_amdgcn_cvt_pk_u8_f32(t0, j, ev);     // round-half-to-even, NaN -> 0
                od = __builtin_amdgcn_cvt_pk_u8_f32(t1, j, od);
                te[4 * w + j] = t0;
                to[4 * w + j] = t1;
            }
            sum = __builtin_amdgcn_udot4(ev, 0x01010101u, sum, false);
            sum = __builtin_amdgcn_udot4(od, 0x01010101u, sum, false);
            words[w] = ev | (od << 4);
        }
        sink(hf, b, words, te, to);
    };

#pragma unroll
    for (int hf = 0; hf < NH; ++hf)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            if (GROUPED) { mn = INFINITY; mx = -INFINITY; }
            prepare_block(hf, b);
            if (GROUPED) {
                mn = fminf(mn, dpp_f<DPP_QUAD_XOR1>(mn)); mn = fminf(mn, dpp_f<DPP_QUAD_XOR2>(mn));
                mx = fmaxf(mx, dpp_f<DPP_QUAD_XOR1>(mx)); mx = fmaxf(mx, dpp_f<DPP_QUAD_XOR2>(mx));
                range_constants(mn, mx);
                sum = 0;
                quantise_block(hf, b);
                sum += dpp_i<DPP_QUAD_XOR1>(sum);
                sum += dpp_i<DPP_QUAD_XOR2>(sum);
                gsink(hf, b, s, lo, sum);
            }
        }
    if (!GROUPED) {
        mn = wave_min_f(mn);
        mx = wave_max_f(mx);
        range_constants(mn, mx);
#pragma unroll
        for (int hf = 0; hf < NH; ++hf)
#pragma unroll
            for (int b = 0; b < 2; ++b) quantise_block(hf, b);
    }
    if (!GROUPED) sum = wave_sum_i(sum);
    P2Meta out;
    out.scale = s; out.lo = lo; out.rowsum = sum;
    return out;
}


// NWAY wavefronts per token: two for K = 4096, four for K = 8192 (for calls with so few tokens that one wave's
// latency is the whole cost).  Wave `part` (0 .. NWAY-1) takes chunks 4*part .. 4*part+3 through the MFMA and the
// register stages.  The last one or two chunk stages (e11; e11 and e12) pair chunk c of one wave with chunk c of
// another, so the waves exchange their 32 values per lane through LDS and each keeps its own output of the
// butterflies; after that a wave owns one 2048-channel block (hf = part / 2, b = part % 2) for the transpose, the
// remaining stages and the quantiser, and only the token's range is combined across the waves.  Every value is
// produced by the same operations in the same order as in p2_token: same bits.
//   raw         this wave's four chunks: raw[j] = 16 bytes at channel 512*(4*part + j) + 8*chunk
//   xch         NWAY * 512 float4 in LDS shared by the token's waves;  red: NWAY * 2 floats likewise
//   sink(words, te, to) the 32 codes of channels 2048*part + 32*lane .. +31, packed two per byte, and the clamped
//               values before rounding (even / odd channels) as in p2_token
// Meets the workgroup's other waves at two barriers (LDS traffic only): every wave calls it, `active` or not.  Returns the token's scale and
// lower bound and the row sum of THIS wave's block; the caller adds the blocks.
template <int NWAY, bool FOLD_NORM, bool HAS_BIAS, bool HAS_SCALE, class Sink>
__device__ __forceinline__ P2Meta p2_token_split(bool active, int part, const uint4 (&raw)[4], const v8bf (&bop)[2], float* wl,
                                                 float4* xch, float* red, const float4* lbias, const float4* lscale,
                                                 float norm, float clip_lo, float clip_hi, int lane, int wbase, int rbase,
                                                 Sink&& sink) {
    static_assert(NWAY == 2 || NWAY == 4, "two waves for K = 4096, four for K = 8192");
    float d[4][2][4];
    if (active) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const v8bf aop = __builtin_bit_cast(v8bf, raw[j]);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                v4f acc = {0.f, 0.f, 0.f, 0.f};
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aop, bop[h], acc, 0, 0, 0);
#pragma unroll
                for (int r = 0; r < 4; ++r) d[j][h][r] = acc[r];
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                BFLY(d[j][h][0], d[j][h][1]);
                BFLY(d[j][h][2], d[j][h][3]);
                BFLY(d[j][h][0], d[j][h][2]);
                BFLY(d[j][h][1], d[j][h][3]);
            }
#pragma unroll
        for (int sft = 1; sft < 4; sft <<= 1)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if ((j & sft) == 0)
#pragma unroll
                    for (int h = 0; h < 2; ++h)
#pragma unroll
                        for (int r = 0; r < 4; ++r) BFLY(d[j][h][r], d[j + sft][h][r]);
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int h = 0; h < 2; ++h)
                xch[(part * 8 + 2 * j + h) * 64 + lane] = make_float4(d[j][h][0], d[j][h][1], d[j][h][2], d[j][h][3]);
    }
    p2_lds_barrier();
    float p[32];
    float mn = INFINITY, mx = -INFINITY;
    if (active) {
        // stage e11 pairs wave w with w ^ 1 (lower index: sum, upper: difference); stage e12 then pairs w with w ^ 2
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const float4 o1 = xch[((part ^ 1) * 8 + 2 * j + h) * 64 + lane];
                const float ov1[4] = {o1.x, o1.y, o1.z, o1.w};
                if (NWAY == 2) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) d[j][h][r] = (part & 1) == 0 ? d[j][h][r] + ov1[r] : ov1[r] - d[j][h][r];
                } else {
                    const float4 o2 = xch[((part ^ 2) * 8 + 2 * j + h) * 64 + lane];
                    const float4 o3 = xch[((part ^ 3) * 8 + 2 * j + h) * 64 + lane];
                    const float ov2[4] = {o2.x, o2.y, o2.z, o2.w};
                    const float ov3[4] = {o3.x, o3.y, o3.z, o3.w};
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        // e11 in this wave's pair and in the pair it meets at e12 (same position within the pair)
                        const float mine = (part & 1) == 0 ? d[j][h][r] + ov1[r] : ov1[r] - d[j][h][r];
                        const float theirs = (part & 1) == 0 ? ov2[r] + ov3[r] : ov3[r] - ov2[r];
                        d[j][h][r] = (part & 2) == 0 ? mine + theirs : theirs - mine;
                    }
                }
            }
        // transpose of this wave's 2048 channels, as in p2_token
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int c01 = 0; c01 < 4; ++c01) {
                const int r0 = r & 1, r1 = r >> 1;
                const int addr = (wbase ^ ((r0 << 1) | (r1 << 2))) | (r0 << 5) | (r1 << 6) | (c01 << 9);
                *reinterpret_cast<float2*>(wl + addr) = make_float2(d[c01][0][r], d[c01][1][r]);
            }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int qq = 0; qq < 16; ++qq) {
            const int e1 = qq & 1, e2 = (qq >> 1) & 1, e3 = (qq >> 2) & 1, e4 = qq >> 3;
            const int addr = (rbase ^ ((e1 << 1) | (e2 << 2))) | (e3 << 7) | (e4 << 8);
            const float2 v = *reinterpret_cast<const float2*>(wl + addr);
            const int idx = (e1 << 1) | (e2 << 2) | (e3 << 3) | (e4 << 4);
            p[idx] = v.x;
            p[idx | 1] = v.y;
        }
#pragma unroll
        for (int i = 0; i < 32; ++i) if ((i & 8) == 0) BFLY(p[i], p[i | 8]);
#pragma unroll
        for (int i = 0; i < 32; ++i) if ((i & 16) == 0) BFLY(p[i], p[i | 16]);
        const int e0 = 2048 * part + 32 * lane;
#pragma unroll
        for (int i4 = 0; i4 < 8; ++i4) {
            float4 bb = make_float4(0.f, 0.f, 0.f, 0.f), ss = make_float4(1.f, 1.f, 1.f, 1.f);
            if (HAS_BIAS) bb = lbias[(part * 8 + i4) * 64 + lane];
            if (HAS_SCALE) ss = lscale[(part * 8 + i4) * 64 + lane];
            const float bv[4] = {bb.x, bb.y, bb.z, bb.w};
            const float sv[4] = {ss.x, ss.y, ss.z, ss.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float r = p[4 * i4 + j];
                if (!FOLD_NORM) r = r * norm;
                const float v = HAS_SCALE ? fmaf(r, sv[j], -bv[j]) : r - bv[j];
                p[4 * i4 + j] = v;
                mn = fminf(mn, v);
                mx = fmaxf(mx, v);
            }
        }
        mn = wave_min_f(mn);
        mx = wave_max_f(mx);
        if (lane == 0) { red[2 * part] = mn; red[2 * part + 1] = mx; }
    }
    p2_lds_barrier();
    P2Meta out;
    out.scale = 1.0f; out.lo = 0.0f; out.rowsum = 0;
    if (active) {
#pragma unroll
        for (int o = 1; o < NWAY; ++o) {
            mn = fminf(mn, red[2 * (part ^ o)]);
            mx = fmaxf(mx, red[2 * (part ^ o) + 1]);
        }
        const float lo = clip_lo * mn;
        const float hi = clip_hi * mx;
        float s = __fdiv_rn(hi - lo, 15.0f);
        if (!(s > 0.0f && s < INFINITY)) s = 1.0f;
        const float inv = __fdiv_rn(1.0f, s);
        const float nlo = -(lo * inv);
        int sum = 0;
        uint32_t words[4];
        v16f te, to;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            uint32_t ev = 0, od = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float t0 = __builtin_amdgcn_fmed3f(fmaf(p[8 * w + 2 * j], inv, nlo), 0.0f, 15.0f);
                const float t1 = __builtin_amdgcn_fmed3f(fmaf(p[8 * w + 2 * j + 1], inv, nlo), 0.0f, 15.0f);
                ev = __builtin_amdgcn_cvt_pk_u8_f32(t0, j, ev);     // round-half-to-even, NaN -> 0
                od = __builtin_amdgcn_cvt_pk_u8_f32(t1, j, od);
                te[4 * w + j] = t0;
                to[4 * w + j] = t1;
            }
            sum = __builtin_amdgcn_udot4(ev, 0x01010101u, sum, false);
            sum = __builtin_amdgcn_udot4(od, 0x01010101u, sum, false);
            words[w] = ev | (od << 4);
        }
        sink(words, te, to);
        out.scale = s; out.lo = lo; out.rowsum = wave_sum_i(sum);
    }
    return out;
}

}  // namespace
}  // namespace basq

#endif
