// Fast rotate + bias + quantise kernel for rot_size == K == 14336 = 28 * 512: the rotation is
// H_28 (x) H_512 (Paley type-I H_28; paper Sec. 5.2 splits a large non-power-of-two rotation in one
// Cooley-Tukey step).  Channel k = i*512 + j, i the H_28 index.
//
// Two wavefronts share a token; wave half h owns output rows i' in [16h, 16h+16) (rows >= 28 idle).
//   1. H_28 along i on the matrix core, exact: lane (g = l/16, m = l%16) loads rows i = 8g+t, t = 0..7,
//      columns j = 128*jb + 8m .. +8 (16 B each), transposes the 8x8 bf16 block in registers
//      (v_perm), and feeds it as A (row = column group m, k = i) to one bf16 MFMA per column
//      offset jj against the +-1 matrix H_28 (k = i, n = i').  After it a lane holds, for its
//      i' = 16h + l%16, the columns j = 128*jb + 32*(l/16) + 8*r + jj.
//   2. H_512 along j in fp32: seven butterfly stages over register bits (jj, r, jb) and two over
//      lane bits 4 and 5, done by swapping register halves with v_permlane16_swap / v_permlane32_swap
//      so that both operands of a butterfly sit in one lane.
//   3. Every lane now owns 128 consecutive channels: normalise, bias (from LDS), min/max, the two
//      waves of the token combine their ranges through LDS, quantise, pack, store.
#include "basq_internal.h"

namespace basq {

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef int v6i __attribute__((ext_vector_type(6)));

constexpr int K28 = 14336;
// Workgroups of four waves (two tokens), two per compute unit, while one 64 KB vector (b^c or s^a) is
// staged in LDS; with both vectors staged, eight waves (four tokens) and one workgroup per unit.

struct H28Cols {
    uint32_t col[28];   // bit i of col[j] set  <=>  H28[i][j] == -1
};

template <int CTRL>
__device__ __forceinline__ float dppf(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
template <int CTRL>
__device__ __forceinline__ int dppi(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, false);
}

#define BFLY28(x, y) do { const float _a = (x), _b = (y); (x) = _a + _b; (y) = _a - _b; } while (0)

// butterfly across lane bit 5 (SWAP32) or lane bit 4 for the register pair (x, y): afterwards x holds
// the sums and y the differences; the lane bit now tells which of the two former registers it was
template <bool SWAP32>
__device__ __forceinline__ void cross_lane_bfly(float& x, float& y) {
    unsigned a = __float_as_uint(x), b = __float_as_uint(y);
    if (SWAP32) {
        auto r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
        a = r[0]; b = r[1];
    } else {
        auto r = __builtin_amdgcn_permlane16_swap(a, b, false, false);
        a = r[0]; b = r[1];
    }
    const float fa = __uint_as_float(a), fb = __uint_as_float(b);
    x = fa + fb;
    y = fa - fb;
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() would also wait for the global
// loads of the next token and for the code stores, which nothing on the other side of the barrier reads.
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <int K28_WAVES, bool HAS_BIAS, bool HAS_SCALE, bool ROT_OUT>
__global__ __launch_bounds__(K28_WAVES * 64, 8 / K28_WAVES) void rotate_quant_k28_kernel(RotateQuantArgs a, float norm, H28Cols hc) {
#if defined(__HIP_DEVICE_COMPILE__)   // the body uses device-only buffer-resource types; the host pass only needs the stub
    // bias (and s^a) laid out so that for a piece index q the 64 lanes of a wave half read consecutive float4s
    constexpr int K28_THREADS = K28_WAVES * 64;
    constexpr int VEC_WORDS = 2 * 32 * 64 * 4;
    constexpr int BIAS_WORDS = HAS_BIAS ? VEC_WORDS : 0;
    constexpr int SCALE_WORDS = HAS_SCALE ? VEC_WORDS : 0;
    __shared__ __attribute__((aligned(16))) float lds[BIAS_WORDS + SCALE_WORDS + 64];
    float* red = lds + BIAS_WORDS + SCALE_WORDS;   // [parity][token in block][half][mn, mx, sum, -]

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int half = wave & 1, tok_in_blk = wave >> 1;
    const int g = lane >> 4, m16 = lane & 15;
    const int ip = 16 * half + m16;                // output row i'
    const bool row_valid = ip < 28;

    if (HAS_BIAS || HAS_SCALE) {
        float4* dst = reinterpret_cast<float4*>(lds);
        for (int f = threadIdx.x; f < 2 * 32 * 64; f += K28_THREADS) {
            const int ln = f & 63, q = (f >> 6) & 31, hh = f >> 11;
            const int row = 16 * hh + (ln & 15);
            const int ch = row * 512 + 128 * (ln >> 4) + 4 * q;
            if (HAS_BIAS)
                dst[f] = row < 28 ? *reinterpret_cast<const float4*>(a.bias + ch) : make_float4(0.f, 0.f, 0.f, 0.f);
            if (HAS_SCALE)
                dst[BIAS_WORDS / 4 + f] = row < 28 ? *reinterpret_cast<const float4*>(a.act_scale + ch) : make_float4(1.f, 1.f, 1.f, 1.f);
        }
    }
    __syncthreads();
    const float4* lbias = reinterpret_cast<const float4*>(lds) + half * 32 * 64;
    const float4* lscale = reinterpret_cast<const float4*>(lds + BIAS_WORDS) + half * 32 * 64;

    // B operand: H_28[k = 8g + t][n = ip], zero outside 28 x 28
    v8bf bop;
    {
        typedef short v8s __attribute__((ext_vector_type(8)));
        v8s tmp;
        const uint32_t mask = row_valid ? hc.col[ip] : 0u;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int i = 8 * g + t;
            short v = 0;
            if (row_valid && i < 28) v = (short)(((mask >> i) & 1u) ? 0xBF80 : 0x3F80);
            tmp[t] = v;
        }
        bop = __builtin_bit_cast(v8bf, tmp);
    }

    // 16-byte loads of column block jb of a token: rows 8g .. 8g+7.  Buffer loads on a descriptor that ends with
    // the token: rows >= 28 lie past its end and read as zero without a branch -- with a branch per row the paths
    // that meet afterwards carry different numbers of loads in flight and every wait becomes a wait for all of them,
    // the prefetched block of the next token included.  `tok` is uniform over the wave.
    auto load_block = [&](v4u (&R)[8], int64_t tok, int jb) {
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(a.X + tok * a.ldx), 0, K28 * 2, 0x00020000);
        const int voff = 8192 * g + 16 * m16 + 256 * jb;                 // bytes; row i = 8g + t starts at 1024 i
#pragma unroll
        for (int t = 0; t < 8; ++t)
            R[t] = __builtin_bit_cast(v4u, __builtin_amdgcn_raw_buffer_load_b128(rs, voff + 1024 * t, 0, 2 /* non-temporal */));
    };

    // Workgroups g, g+8, ... share an XCD; renumbered so that an XCD owns a contiguous range, 32
    // consecutive tokens (one block of the fp6 output) meet in one L2 and their pieces merge there.
    int vblock = blockIdx.x;
    if ((gridDim.x & 127) == 0) vblock = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    const int64_t rb6 = (a.M + 31) >> 5;                    // 32-row blocks per chunk of the fp6 output
    const int tokens_per_round = gridDim.x * (K28_WAVES / 2);
    const int64_t m_first = (int64_t)vblock * (K28_WAVES / 2);
    v4u R[4][8];
    {
        const int64_t m = m_first + tok_in_blk;
        load_block(R[0], m < a.M ? m : a.M - 1, 0);
    }
    // The row sums of the two halves meet one token late, at the next token's barrier, so that a token
    // costs one barrier: red is double buffered by token parity.
    int parity = 0;
    int64_t prev_m = -1;
    float prev_s = 0.f, prev_lo = 0.f;
    for (int64_t m0 = m_first; m0 < a.M; m0 += tokens_per_round, parity ^= 1) {
        const int64_t m = m0 + tok_in_blk;
        const bool tok_valid = m < a.M;
        const int64_t mm = tok_valid ? m : a.M - 1;      // keep every wave on the same barrier schedule

        // ---- H_28 on the matrix core.  Block 0 was requested one token ago; blocks 1..3 are requested
        // together now, while the accumulators that will replace them are not live yet.
        float d[4][8][4];                                  // [jb][jj][r]
#pragma unroll
        for (int jb = 1; jb < 4; ++jb) load_block(R[jb], mm, jb);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int jb = 0; jb < 4; ++jb) {
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) {
                v4u A;
                const int w = jj >> 1;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    // bytes of (hi, lo) = (R[2u+1][w], R[2u][w]); even jj takes the low halves, odd jj the high halves
                    A[u] = (jj & 1) ? __builtin_amdgcn_perm(R[jb][2 * u + 1][w], R[jb][2 * u][w], 0x07060302u)
                                    : __builtin_amdgcn_perm(R[jb][2 * u + 1][w], R[jb][2 * u][w], 0x05040100u);
                }
                v4f acc = {0.f, 0.f, 0.f, 0.f};
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, A), bop, acc, 0, 0, 0);
#pragma unroll
                for (int r = 0; r < 4; ++r) d[jb][jj][r] = acc[r];
            }
        }
        // first block of this wave's next token: its latency hides behind the butterflies below
        {
            const int64_t mn_tok = m + tokens_per_round;
            load_block(R[0], mn_tok < a.M ? mn_tok : a.M - 1, 0);
            __builtin_amdgcn_sched_barrier(0);
        }

        // ---- H_512: register stages jj (j0..2), r (j3..4), jb (j7..8) ------------------------------------
#pragma unroll
        for (int jb = 0; jb < 4; ++jb) {
#pragma unroll
            for (int s = 1; s < 8; s <<= 1)
#pragma unroll
                for (int jj = 0; jj < 8; ++jj)
                    if ((jj & s) == 0)
#pragma unroll
                        for (int r = 0; r < 4; ++r) BFLY28(d[jb][jj][r], d[jb][jj + s][r]);
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) {
                BFLY28(d[jb][jj][0], d[jb][jj][1]);
                BFLY28(d[jb][jj][2], d[jb][jj][3]);
                BFLY28(d[jb][jj][0], d[jb][jj][2]);
                BFLY28(d[jb][jj][1], d[jb][jj][3]);
            }
        }
#pragma unroll
        for (int jj = 0; jj < 8; ++jj)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                BFLY28(d[0][jj][r], d[1][jj][r]);
                BFLY28(d[2][jj][r], d[3][jj][r]);
                BFLY28(d[0][jj][r], d[2][jj][r]);
                BFLY28(d[1][jj][r], d[3][jj][r]);
            }
        // ---- lane stages: j5 (lane bit 4) pairs jb bit 0, j6 (lane bit 5) pairs jb bit 1.  Afterwards
        // register index jb means (j5, j6) and lane bits (4, 5) mean (j7, j8).
#pragma unroll
        for (int jj = 0; jj < 8; ++jj)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                cross_lane_bfly<false>(d[0][jj][r], d[1][jj][r]);
                cross_lane_bfly<false>(d[2][jj][r], d[3][jj][r]);
                cross_lane_bfly<true>(d[0][jj][r], d[2][jj][r]);
                cross_lane_bfly<true>(d[1][jj][r], d[3][jj][r]);
            }

        // ---- this lane owns channels ip*512 + 128*g + c, c = 32*jb + 8*r + jj ---------------------------
        const int ch0 = ip * 512 + 128 * g;
        float mn = INFINITY, mx = -INFINITY;
#pragma unroll
        for (int jb = 0; jb < 4; ++jb)
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int q2 = 0; q2 < 2; ++q2) {
                    const int c = 32 * jb + 8 * r + 4 * q2;
                    float4 bb = make_float4(0.f, 0.f, 0.f, 0.f), ss = make_float4(1.f, 1.f, 1.f, 1.f);
                    if (HAS_BIAS) bb = lbias[(c >> 2) * 64 + lane];
                    if (HAS_SCALE) ss = lscale[(c >> 2) * 64 + lane];
                    const float bv[4] = {bb.x, bb.y, bb.z, bb.w};
                    const float sv[4] = {ss.x, ss.y, ss.z, ss.w};
                    float rr[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float rv = d[jb][4 * q2 + e][r] * norm;
                        rr[e] = rv;
                        const float v = HAS_SCALE ? fmaf(rv, sv[e], -bv[e]) : rv - bv[e];
                        d[jb][4 * q2 + e][r] = v;
                        mn = fminf(mn, v);
                        mx = fmaxf(mx, v);
                    }
                    if (ROT_OUT && row_valid && tok_valid)
                        *reinterpret_cast<float4*>(a.rot_out + m * (int64_t)K28 + ch0 + c) = make_float4(rr[0], rr[1], rr[2], rr[3]);
                }
        if (!row_valid) { mn = INFINITY; mx = -INFINITY; }
        // wave reduction, then the two halves of the token through LDS
        mn = fminf(mn, dppf<0xB1>(mn)); mx = fmaxf(mx, dppf<0xB1>(mx));
        mn = fminf(mn, dppf<0x4E>(mn)); mx = fmaxf(mx, dppf<0x4E>(mx));
        mn = fminf(mn, dppf<0x141>(mn)); mx = fmaxf(mx, dppf<0x141>(mx));
        mn = fminf(mn, dppf<0x140>(mn)); mx = fmaxf(mx, dppf<0x140>(mx));
        {
            float lo4[4], hi4[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                lo4[q] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(mn), 16 * q));
                hi4[q] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(mx), 16 * q));
            }
            mn = fminf(fminf(lo4[0], lo4[1]), fminf(lo4[2], lo4[3]));
            mx = fmaxf(fmaxf(hi4[0], hi4[1]), fmaxf(hi4[2], hi4[3]));
        }
        float* myred = red + (parity * (K28_WAVES / 2) + tok_in_blk) * 8;
        float* otherred = red + ((parity ^ 1) * (K28_WAVES / 2) + tok_in_blk) * 8;
        if (lane == 0) { myred[half * 4 + 0] = mn; myred[half * 4 + 1] = mx; }
        lds_barrier();
        mn = fminf(myred[0], myred[4]);
        mx = fmaxf(myred[1], myred[5]);
        if (half == 0 && lane == 0 && prev_m >= 0) {       // finish the previous token
            basq_tokmeta mt;
            mt.scale = prev_s; mt.lo = prev_lo;
            mt.rowsum = reinterpret_cast<int*>(otherred)[2] + reinterpret_cast<int*>(otherred)[6];
            mt.reserved = 0;
            a.meta[prev_m] = mt;
        }

        const float lo = a.clip_lo * mn;
        const float hi = a.clip_hi * mx;
        float s = __fdiv_rn(hi - lo, 15.0f);
        if (!(s > 0.0f && s < INFINITY)) s = 1.0f;
        const float inv = __fdiv_rn(1.0f, s);
        const float nlo = -(lo * inv);

        int sum = 0;
        uint32_t words[4][4];                              // [jb][r]: 16 bytes of codes per jb
#pragma unroll
        for (int jb = 0; jb < 4; ++jb) {
            v16f qe, qo;                                   // the clamped values before rounding: low / high nibbles
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                uint32_t ev = 0, od = 0;
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    const float t0 = __builtin_amdgcn_fmed3f(fmaf(d[jb][2 * p][r], inv, nlo), 0.0f, 15.0f);
                    const float t1 = __builtin_amdgcn_fmed3f(fmaf(d[jb][2 * p + 1][r], inv, nlo), 0.0f, 15.0f);
                    ev = __builtin_amdgcn_cvt_pk_u8_f32(t0, p, ev);
                    od = __builtin_amdgcn_cvt_pk_u8_f32(t1, p, od);
                    qe[4 * r + p] = t0;
                    qo[4 * r + p] = t1;
                }
                if (row_valid) {
                    sum = __builtin_amdgcn_udot4(ev, 0x01010101u, sum, false);
                    sum = __builtin_amdgcn_udot4(od, 0x01010101u, sum, false);
                }
                words[jb][r] = ev | (od << 4);
            }
            if (a.Aq6 && row_valid && tok_valid) {
                // The 32 codes of group jb once more, as e2m3 numbers q/8, straight from the clamped values: the
                // packed conversion divides by its scale operand, rounds to nearest-even (on the e2m3 grid below 2
                // that is t/8 -> rint(t)/8, ties as in the integer conversion) and interleaves its two sources.
                // A lane's 128 channels are one 128-code chunk of the fp6 layout: chunk 4*i' + g, group jb.
                const v6i f6 = __builtin_amdgcn_cvt_scalef32_2xpk16_fp6_f32(qe, qo, 8.0f);
                const int rr = (int)(m & 31);
                uint8_t* blk = a.Aq6 + ((int64_t)(4 * ip + g) * rb6 + (m >> 5)) * 3072;
                *reinterpret_cast<uint4*>(blk + 64 * rr + 16 * (jb ^ ((rr >> 2) & 3))) =
                    make_uint4((uint32_t)f6[0], (uint32_t)f6[1], (uint32_t)f6[2], (uint32_t)f6[3]);
                *reinterpret_cast<uint2*>(blk + 2048 + 256 * jb + 8 * rr) = make_uint2((uint32_t)f6[4], (uint32_t)f6[5]);
            }
        }
        // A lane holds 64 consecutive output bytes as four 16-byte pieces.  Transposing the pieces over
        // (jb, g) lets every store instruction write whole 64-byte segments (piece jb of lane g goes to
        // register g of lane jb), instead of four partial writes per segment.
        // (The 4-bit form is optional when the fp6 form is written.)
        if (a.Aq) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                auto s0 = __builtin_amdgcn_permlane16_swap(words[0][r], words[1][r], false, false);
                auto s1 = __builtin_amdgcn_permlane16_swap(words[2][r], words[3][r], false, false);
                auto t0 = __builtin_amdgcn_permlane32_swap(s0[0], s1[0], false, false);
                auto t1 = __builtin_amdgcn_permlane32_swap(s0[1], s1[1], false, false);
                words[0][r] = t0[0]; words[2][r] = t0[1];
                words[1][r] = t1[0]; words[3][r] = t1[1];
            }
            if (row_valid && tok_valid) {
                uint8_t* orow = a.Aq + m * (int64_t)(K28 / 2) + ip * 256 + 16 * g;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    nt_store16(orow + 64 * j, make_uint4(words[j][0], words[j][1], words[j][2], words[j][3]));
            }
        }
        sum += dppi<0xB1>(sum);
        sum += dppi<0x4E>(sum);
        sum += dppi<0x141>(sum);
        sum += dppi<0x140>(sum);
        sum = __builtin_amdgcn_readlane(sum, 0) + __builtin_amdgcn_readlane(sum, 16) +
              __builtin_amdgcn_readlane(sum, 32) + __builtin_amdgcn_readlane(sum, 48);
        if (lane == 0) reinterpret_cast<int*>(myred)[half * 4 + 2] = sum;
        prev_m = tok_valid ? m : -1;
        prev_s = s; prev_lo = lo;
    }
    lds_barrier();
    if (half == 0 && lane == 0 && prev_m >= 0) {
        const int* lastred = reinterpret_cast<const int*>(red + ((parity ^ 1) * (K28_WAVES / 2) + tok_in_blk) * 8);
        basq_tokmeta mt;
        mt.scale = prev_s; mt.lo = prev_lo;
        mt.rowsum = lastred[2] + lastred[6];
        mt.reserved = 0;
        a.meta[prev_m] = mt;
    }
#endif  // __HIP_DEVICE_COMPILE__
}

template <bool HB, bool HS>
int launch_k28_flags(const RotateQuantArgs& a, hipStream_t s, float norm, const H28Cols& hc) {
    constexpr int WAVES = (HB && HS) ? 8 : 4;
    constexpr int TOKENS = WAVES / 2;
    constexpr int MAX_BLOCKS = 256 * (8 / WAVES);
    const int64_t want = (a.M + TOKENS - 1) / TOKENS;
    const unsigned blocks = (unsigned)(want < MAX_BLOCKS ? want : MAX_BLOCKS);
    if (a.rot_out)
        hipLaunchKernelGGL((rotate_quant_k28_kernel<WAVES, HB, HS, true>), dim3(blocks), dim3(WAVES * 64), 0, s, a, norm, hc);
    else
        hipLaunchKernelGGL((rotate_quant_k28_kernel<WAVES, HB, HS, false>), dim3(blocks), dim3(WAVES * 64), 0, s, a, norm, hc);
    return check_hip(hipGetLastError(), "rotate_quant (28x512) launch");
}

}  // namespace

bool rotate_quant_k28_applicable(const RotateQuantArgs& a) {
    return a.group == a.K && a.has28 && a.rot_size == K28 && a.K == K28 && (a.Aq != nullptr || a.Aq6 != nullptr) &&
           a.meta != nullptr;
}

int launch_rotate_quant_k28(const RotateQuantArgs& a, hipStream_t s) {
    H28Cols hc{};
    const int8_t* h = hadamard28_host();
    for (int j = 0; j < 28; ++j) {
        uint32_t mk = 0;
        for (int i = 0; i < 28; ++i) if (h[i * 28 + j] < 0) mk |= 1u << i;
        hc.col[j] = mk;
    }
    const float norm = (float)(1.0 / sqrt((double)K28));
    const bool hb = a.bias != nullptr, hs = a.act_scale != nullptr;
    if (hb && hs) return launch_k28_flags<true, true>(a, s, norm, hc);
    if (hb) return launch_k28_flags<true, false>(a, s, norm, hc);
    if (hs) return launch_k28_flags<false, true>(a, s, norm, hc);
    return launch_k28_flags<false, false>(a, s, norm, hc);
}

}  // namespace basq
