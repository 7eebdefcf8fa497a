// Fast rotate + bias + quantise kernel for BLOCKWISE rotations: rot_size n in {128, 256, 512} applied to every
// block of n channels of a longer token (K a multiple of n and of 256, K <= 16384), per-token ranges.  This is the
// shape of a layer whose width has no Hadamard matrix of its own size in this library -- e.g. the 11008 = 43 * 256
// wide MLP of the 7B LLaMA-2 that the paper's Sec. 5.2 times -- rotated in blocks instead (paper Sec. 3.1 rotation,
// Eq. 14 bias, Eq. 15 scale, Eq. 4 quantiser with the per-token range of Sec. 5).
//
// One workgroup of four wavefronts per token; a wave takes the 512-channel pieces w, w+4, ... of the token and
// keeps them in registers (8 values per lane per piece) across the two passes that a per-token range needs.
// No LDS except for the workgroup's range and row sum.
//
// Inside a piece, channel e (9 bits):
//   load      lane l reads 8 consecutive bf16 (16 B) at chunk(l): e = 8*chunk + t, chunk bits (e3..e8) <- lane bits
//             (2,3,0,1,4,5), as in the K = 4096/8192 kernel (P2Lane).
//   MFMA      the stages over (e0,e1,e2,e7,e8) -- only (e0,e1,e2,e7) for n = 256, (e0,e1,e2) for n = 128 -- as one
//             16x16x32 bf16 MFMA pair against a +-1 (n = 256: +-2^-4, the exact normalisation) block-diagonal
//             operand: exact.  Afterwards e0 = h, (e5,e6) = r, lane bits (0..5) = (e1,e2,e7,e8,e3,e4).
//   stages    e5, e6 on the accumulator registers; e3, e4 across lane bits 4 and 5 by swapping register halves
//             (v_permlane16_swap / v_permlane32_swap) so that both operands of a butterfly sit in one lane.
//             Afterwards: e0 = h, (e3,e4) = r, lane bits (0..5) = (e1,e2,e7,e8,e5,e6).
//   codes     a lane's four bytes (two codes each) are 4 bytes apart and the four lanes of a quad fill the gaps:
//             a 4 x 4 byte transpose inside the quad (DPP + v_perm) gives every lane one aligned dword of the
//             16-byte segment, and a store instruction writes 256 contiguous bytes of the row.
#include "rotate_pow2_token.h"

namespace basq {

namespace {

constexpr int RB_WAVES = 4;
constexpr int RB_THREADS = RB_WAVES * 64;
constexpr int RB_PMAX = 8;                          // pieces per wave: K <= 4 * 8 * 512

// butterfly across lane bit 5 (SWAP32) or lane bit 4 for the register pair (x, y): afterwards x holds the sums and y
// the differences, and the lane bit tells which of the two former registers a lane's pair came from
template <bool SWAP32>
__device__ __forceinline__ void rb_cross_lane_bfly(float& x, float& y) {
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

// B operand of the MFMA: k = 8*(lane/16) + t carries input bits (e0,e1,e2,e7,e8), column lane%16 of half h carries
// output bits (h; e1,e2,e7,e8).  H over the low LOG2N-4 of those five bits, identity over the rest.
template <int LOG2N>
__device__ __forceinline__ void rb_make_bop(int lane, v8bf (&bop)[2]) {
    constexpr int MASK = (1 << (LOG2N - 4)) - 1;       // 7 -> 0b00111, 8 -> 0b01111, 9 -> 0b11111
    const int jp = lane & 15, g = lane >> 4;
    const uint16_t mag = LOG2N == 8 ? (uint16_t)((127 - 4) << 7) : (uint16_t)0x3F80;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        v8s tmp;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int kin = t | (g << 3), jout = h | (jp << 1);
            const bool same_block = ((kin ^ jout) & ~MASK & 31) == 0;
            const short v = (short)(mag | ((__builtin_popcount(kin & jout & MASK) & 1) ? 0x8000 : 0));
            tmp[t] = same_block ? v : (short)0;
        }
        bop[h] = __builtin_bit_cast(v8bf, tmp);
    }
}

template <int CTRL>
__device__ __forceinline__ uint32_t rb_dpp_u(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, false);
}

template <int LOG2N, bool HAS_BIAS, bool HAS_SCALE, bool ROT_OUT>
__global__ __launch_bounds__(RB_THREADS) void rotate_quant_block_kernel(RotateQuantArgs a, float norm) {
    constexpr bool FOLD_NORM = LOG2N == 8;           // 1/sqrt(256) = 2^-4 sits in the MFMA operand
    __shared__ float red_mn[RB_WAVES], red_mx[RB_WAVES];
    __shared__ int red_sum[RB_WAVES];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t m = blockIdx.x;
    const int K = a.K;
    const int np = (K + 511) >> 9;                    // pieces of the token (the last one may be half: K % 512 = 256)
    const P2Lane pl = p2_lane(lane);
    v8bf bop[2];
    rb_make_bop<LOG2N>(lane, bop);

    // where this lane's values of a piece end up: e = eout + h + 8*r0 + 16*r1
    const int eout = 2 * (lane & 1) + 4 * ((lane >> 1) & 1) + 128 * ((lane >> 2) & 1) + 256 * ((lane >> 3) & 1) +
                     32 * ((lane >> 4) & 1) + 64 * ((lane >> 5) & 1);

    // ---- all of this wave's pieces are requested at once ------------------------------------------------------
    const uint16_t* x = a.X + m * a.ldx;
    uint4 raw[RB_PMAX];
#pragma unroll
    for (int p = 0; p < RB_PMAX; ++p) {
        const int ein = 512 * (wave + RB_WAVES * p) + 8 * pl.chunk;
        raw[p] = ein < K ? nt_load16(x + ein) : make_uint4(0, 0, 0, 0);
    }

    // ---- pass 1: rotate, bias, range ---------------------------------------------------------------------------
    float v[RB_PMAX][2][4];
    float mn = INFINITY, mx = -INFINITY;
#pragma unroll
    for (int p = 0; p < RB_PMAX; ++p) {
        const int c = wave + RB_WAVES * p;
        if (c < np) {                                  // uniform over the wave
            float d[2][4];
            const v8bf aop = __builtin_bit_cast(v8bf, raw[p]);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                v4f acc = {0.f, 0.f, 0.f, 0.f};
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aop, bop[h], acc, 0, 0, 0);
#pragma unroll
                for (int r = 0; r < 4; ++r) d[h][r] = acc[r];
            }
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                BFLY(d[h][0], d[h][1]);                // e5
                BFLY(d[h][2], d[h][3]);
                BFLY(d[h][0], d[h][2]);                // e6
                BFLY(d[h][1], d[h][3]);
                rb_cross_lane_bfly<false>(d[h][0], d[h][1]);   // e3 <-> lane bit 4; register bit r0 now means e3
                rb_cross_lane_bfly<false>(d[h][2], d[h][3]);
                rb_cross_lane_bfly<true>(d[h][0], d[h][2]);    // e4 <-> lane bit 5; register bit r1 now means e4
                rb_cross_lane_bfly<true>(d[h][1], d[h][3]);
            }
            const int e0 = 512 * c + eout;
            const bool ok = e0 < K;                    // a half piece: the lanes of its missing 256 channels
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int e = e0 + 8 * r;              // channels e (h = 0) and e + 1 (h = 1)
                float2 bb = make_float2(0.f, 0.f), ss = make_float2(1.f, 1.f);
                if (HAS_BIAS && ok) bb = *reinterpret_cast<const float2*>(a.bias + e);
                if (HAS_SCALE && ok) ss = *reinterpret_cast<const float2*>(a.act_scale + e);
                float r0 = d[0][r], r1 = d[1][r];
                if (!FOLD_NORM) { r0 = r0 * norm; r1 = r1 * norm; }
                if (ROT_OUT && ok) *reinterpret_cast<float2*>(a.rot_out + m * (int64_t)K + e) = make_float2(r0, r1);
                const float v0 = HAS_SCALE ? fmaf(r0, ss.x, -bb.x) : r0 - bb.x;
                const float v1 = HAS_SCALE ? fmaf(r1, ss.y, -bb.y) : r1 - bb.y;
                v[p][0][r] = v0;
                v[p][1][r] = v1;
                if (ok) {
                    mn = fminf(mn, fminf(v0, v1));
                    mx = fmaxf(mx, fmaxf(v0, v1));
                }
            }
        }
    }
    mn = wave_min_f(mn);
    mx = wave_max_f(mx);
    if (lane == 0) { red_mn[wave] = mn; red_mx[wave] = mx; }
    __syncthreads();
    mn = fminf(fminf(red_mn[0], red_mn[1]), fminf(red_mn[2], red_mn[3]));
    mx = fmaxf(fmaxf(red_mx[0], red_mx[1]), fmaxf(red_mx[2], red_mx[3]));

    const float lo = a.clip_lo * mn;
    const float hi = a.clip_hi * mx;
    float s = __fdiv_rn(hi - lo, 15.0f);
    if (!(s > 0.0f && s < INFINITY)) s = 1.0f;
    const float inv = __fdiv_rn(1.0f, s);
    const float nlo = -(lo * inv);

    // ---- pass 2: quantise, pack, store -------------------------------------------------------------------------
    int sum = 0;
    const int q4 = lane & 3;                                             // position in the quad
    const uint32_t sel = (uint32_t)q4 | ((uint32_t)(4 + q4) << 8);       // v_perm: byte q4 of each of two dwords
    const int seg = ((lane >> 4) & 1) + 2 * ((lane >> 5) & 1) + 4 * ((lane >> 2) & 1) + 8 * ((lane >> 3) & 1);
    uint8_t* orow = a.Aq + m * (int64_t)(K / 2) + 16 * seg + 4 * q4;
#pragma unroll
    for (int p = 0; p < RB_PMAX; ++p) {
        const int c = wave + RB_WAVES * p;
        if (c < np) {
            const bool ok = 512 * c + eout < K;
            uint32_t ev = 0, od = 0;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float t0 = __builtin_amdgcn_fmed3f(fmaf(v[p][0][r], inv, nlo), 0.0f, 15.0f);
                const float t1 = __builtin_amdgcn_fmed3f(fmaf(v[p][1][r], inv, nlo), 0.0f, 15.0f);
                ev = __builtin_amdgcn_cvt_pk_u8_f32(t0, r, ev);          // round-half-to-even, NaN -> 0
                od = __builtin_amdgcn_cvt_pk_u8_f32(t1, r, od);
            }
            if (ok) {
                sum = __builtin_amdgcn_udot4(ev, 0x01010101u, sum, false);
                sum = __builtin_amdgcn_udot4(od, 0x01010101u, sum, false);
            }
            // byte r of `w`: the row's byte at 256*c + 16*seg + q4 + 4*r.  Quad transpose: lane q4 ends with the bytes
            // q4 of its quad's four words, i.e. the aligned dword at ... + 4*q4.
            const uint32_t w = ev | (od << 4);
            const uint32_t w0 = rb_dpp_u<0x00>(w), w1 = rb_dpp_u<0x55>(w), w2 = rb_dpp_u<0xAA>(w), w3 = rb_dpp_u<0xFF>(w);
            const uint32_t lo2 = __builtin_amdgcn_perm(w1, w0, sel);     // bytes (w0[q4], w1[q4], -, -)
            const uint32_t hi2 = __builtin_amdgcn_perm(w3, w2, sel);
            const uint32_t word = __builtin_amdgcn_perm(hi2, lo2, 0x05040100u);
            if (ok) *reinterpret_cast<uint32_t*>(orow + 256 * c) = word;
        }
    }
    sum = wave_sum_i(sum);
    if (lane == 0) red_sum[wave] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        basq_tokmeta mt;
        mt.scale = s; mt.lo = lo; mt.rowsum = red_sum[0] + red_sum[1] + red_sum[2] + red_sum[3]; mt.reserved = 0;
        a.meta[m] = mt;
    }
}

template <int LOG2N>
int launch_rb(const RotateQuantArgs& a, hipStream_t s, float norm) {
    const bool hb = a.bias != nullptr, hs = a.act_scale != nullptr, ro = a.rot_out != nullptr;
    const dim3 grid((unsigned)a.M), block(RB_THREADS);
#define RB_LAUNCH(HB, HS, RO) hipLaunchKernelGGL((rotate_quant_block_kernel<LOG2N, HB, HS, RO>), grid, block, 0, s, a, norm)
    if (hb && hs) { if (ro) RB_LAUNCH(true, true, true); else RB_LAUNCH(true, true, false); }
    else if (hb) { if (ro) RB_LAUNCH(true, false, true); else RB_LAUNCH(true, false, false); }
    else if (hs) { if (ro) RB_LAUNCH(false, true, true); else RB_LAUNCH(false, true, false); }
    else { if (ro) RB_LAUNCH(false, false, true); else RB_LAUNCH(false, false, false); }
#undef RB_LAUNCH
    return check_hip(hipGetLastError(), "rotate_quant (blockwise) launch");
}

}  // namespace

bool rotate_quant_block_applicable(const RotateQuantArgs& a) {
    // per-token ranges; n = 512 needs whole 512-channel pieces, 128 and 256 also take a last piece of 256 channels
    return a.group == a.K && !a.has28 && (a.rot_size == 128 || a.rot_size == 256 || a.rot_size == 512) &&
           a.K % 256 == 0 && a.K % a.rot_size == 0 && a.K <= RB_WAVES * RB_PMAX * 512 && a.Aq != nullptr &&
           a.meta != nullptr && a.M <= 0x7FFFFFFFll;
}

int launch_rotate_quant_block(const RotateQuantArgs& a, hipStream_t s) {
    const float norm = (float)(1.0 / sqrt((double)a.rot_size));
    if (a.rot_size == 128) return launch_rb<7>(a, s, norm);
    if (a.rot_size == 256) return launch_rb<8>(a, s, norm);
    return launch_rb<9>(a, s, norm);
}

}  // namespace basq
