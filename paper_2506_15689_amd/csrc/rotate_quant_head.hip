// Per-head rotate + bias + quantise: rot_size == group == 128 (the online Hadamard on q and k, R_qk, and
// the per-head asymmetric INT4 of the KV cache: paper Sec. 4 "online rotations", Sec. 5 "Deployment
// Details" and Sec. 5.2).  Every 128-channel head is rotated by H_128 / sqrt(128) and gets its own range
// and token record, so a 512-channel piece of a token (four heads) is an independent work item: one
// wavefront per item, nothing but registers in between.
//
// Channel bits of an item: e0..e6 inside the head, e7,e8 the head.
//   load   lane l reads 8 consecutive bf16 (e0..e2); its 16-byte unit is (e3,e4) <- lane bits (4,5),
//          (e5,e6) <- lane bits (0,1), (e7,e8) <- lane bits (2,3): a wave load is 1 KB, fully coalesced.
//   MFMA   A = 16 rows (lane%16 = e5..e8) x 32 (k = 8*(lane/16) + t = e0..e4), B = H_32 with its columns
//          permuted so that output bit e0 is the half index h and (e1..e4) the output lane%16.  Exact: bf16
//          inputs, +-1 entries.  Afterwards lane (col = e1..e4, lane/16 = e7,e8) holds d[h][r], r = (e5,e6).
//   stages e5, e6 on the four r registers.  The head of a value is lane/16: its 16 lanes are one DPP row.
//   bias (LDS copy), range over 8 registers and the row, quantise; the four bytes of a lane (one per r)
//   are transposed inside each quad so that a lane stores one dword and a wave 256 contiguous bytes.
#include "basq_internal.h"

namespace basq {

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef short v8s __attribute__((ext_vector_type(8)));

constexpr int RH_WAVES = 4;
constexpr int RH_THREADS = RH_WAVES * 64;

template <int CTRL>
__device__ __forceinline__ float rh_dppf(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
template <int CTRL>
__device__ __forceinline__ int rh_dppi(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, false);
}
// reductions over one DPP row (16 lanes); every lane of the row ends with the result
__device__ __forceinline__ float row_min(float v) {
    v = fminf(v, rh_dppf<0xB1>(v)); v = fminf(v, rh_dppf<0x4E>(v));
    v = fminf(v, rh_dppf<0x141>(v)); v = fminf(v, rh_dppf<0x140>(v));
    return v;
}
__device__ __forceinline__ float row_max(float v) {
    v = fmaxf(v, rh_dppf<0xB1>(v)); v = fmaxf(v, rh_dppf<0x4E>(v));
    v = fmaxf(v, rh_dppf<0x141>(v)); v = fmaxf(v, rh_dppf<0x140>(v));
    return v;
}
__device__ __forceinline__ int row_sum(int v) {
    v += rh_dppi<0xB1>(v); v += rh_dppi<0x4E>(v);
    v += rh_dppi<0x141>(v); v += rh_dppi<0x140>(v);
    return v;
}

#define RH_BFLY(x, y) do { const float _a = (x), _b = (y); (x) = _a + _b; (y) = _a - _b; } while (0)

template <bool HAS_BIAS, bool HAS_SCALE, bool ROT_OUT>
__global__ __launch_bounds__(RH_THREADS) void rotate_quant_head_kernel(RotateQuantArgs a, float norm) {
    // bias and s^a laid out so that lane l of piece (c, r) reads the float2 at ((c*4 + r)*64 + l)
    extern __shared__ __attribute__((aligned(16))) float rh_lds[];
    const int K = a.K;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 15, g = lane >> 4;
    float2* lbias = reinterpret_cast<float2*>(rh_lds);
    float2* lscale = reinterpret_cast<float2*>(rh_lds + (HAS_BIAS ? K : 0));
    if (HAS_BIAS || HAS_SCALE) {
        for (int f = threadIdx.x; f < K / 2; f += RH_THREADS) {
            // float2 number f of the staged copy: lane f%64, r = (f/64)%4, c = f/256
            const int ln = f & 63, r = (f >> 6) & 3, c = f >> 8;
            const int e = 512 * c + 128 * (ln >> 4) + 32 * r + 2 * (ln & 15);
            if (HAS_BIAS) lbias[f] = *reinterpret_cast<const float2*>(a.bias + e);
            if (HAS_SCALE) lscale[f] = *reinterpret_cast<const float2*>(a.act_scale + e);
        }
        __syncthreads();
    }

    // B operand: column j' = lane%16 of half h, k = 8*(lane/16) + t; input bits (t0,t1,t2,g0,g1) = e0..e4,
    // output bits (h, j'0..j'3) = e0..e4: sign = parity(popcount(kin & jout))
    v8bf bop[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        v8s tmp;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int kin = t | (g << 3), jout = h | (col << 1);
            tmp[t] = (short)(0x3F80 | ((__builtin_popcount(kin & jout) & 1) ? 0x8000 : 0));
        }
        bop[h] = __builtin_bit_cast(v8bf, tmp);
    }
    const int unit = g | ((lane & 3) << 2) | (((lane >> 2) & 3) << 4);       // 16-byte unit of the lane inside an item
    // byte transpose inside a quad: lane i of the quad collects byte i of the four lanes
    const int qi = lane & 3;
    const unsigned sel01 = 0x0C0C0000u | (unsigned)qi | ((unsigned)(4 + qi) << 8);
    const unsigned sel23 = 0x00000C0Cu | ((unsigned)qi << 16) | ((unsigned)(4 + qi) << 24);

    const int cpt = K / 512;                                   // items per token
    const int hpt = K / 128;                                   // heads (token records) per token
    // Item = (token m, piece c), uniform over the wave: kept in scalar registers and advanced without a
    // division (stride = sq tokens + sr pieces).
    const int swave = __builtin_amdgcn_readfirstlane(wave);
    const int64_t first = (int64_t)blockIdx.x * RH_WAVES + swave;
    const int64_t stride = (int64_t)gridDim.x * RH_WAVES;
    const int64_t sq = stride / cpt;
    const int sr = (int)(stride - sq * cpt);
    int64_t m = first / cpt;
    int c = (int)(first - m * cpt);
    for (; m < a.M; m += sq, c += sr) {
        if (c >= cpt) { c -= cpt; ++m; if (m >= a.M) break; }
        const uint4 raw = nt_load16(a.X + m * a.ldx + 512 * c + 8 * unit);
        const v8bf aop = __builtin_bit_cast(v8bf, raw);
        float d[2][4];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            v4f acc = {0.f, 0.f, 0.f, 0.f};
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aop, bop[h], acc, 0, 0, 0);
#pragma unroll
            for (int r = 0; r < 4; ++r) d[h][r] = acc[r];
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            RH_BFLY(d[h][0], d[h][1]);
            RH_BFLY(d[h][2], d[h][3]);
            RH_BFLY(d[h][0], d[h][2]);
            RH_BFLY(d[h][1], d[h][3]);
        }
        // this lane's values: channels 512c + 128g + 32r + 2col + h
        float mn = INFINITY, mx = -INFINITY;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            float2 bb = make_float2(0.f, 0.f), ss = make_float2(1.f, 1.f);
            if (HAS_BIAS) bb = lbias[(c * 4 + r) * 64 + lane];
            if (HAS_SCALE) ss = lscale[(c * 4 + r) * 64 + lane];
            const float r0 = d[0][r] * norm, r1 = d[1][r] * norm;
            if (ROT_OUT)
                *reinterpret_cast<float2*>(a.rot_out + m * (int64_t)K + 512 * c + 128 * g + 32 * r + 2 * col) = make_float2(r0, r1);
            const float v0 = HAS_SCALE ? fmaf(r0, ss.x, -bb.x) : r0 - bb.x;
            const float v1 = HAS_SCALE ? fmaf(r1, ss.y, -bb.y) : r1 - bb.y;
            d[0][r] = v0; d[1][r] = v1;
            mn = fminf(mn, fminf(v0, v1));
            mx = fmaxf(mx, fmaxf(v0, v1));
        }
        mn = row_min(mn);
        mx = row_max(mx);
        const float lo = a.clip_lo * mn;
        const float hi = a.clip_hi * mx;
        float s = __fdiv_rn(hi - lo, 15.0f);
        if (!(s > 0.0f && s < INFINITY)) s = 1.0f;
        const float inv = __fdiv_rn(1.0f, s);
        const float nlo = -(lo * inv);

        uint32_t ev = 0, od = 0;                                // byte r: the code of channel 2col (+1) of 32-block r
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float t0 = __builtin_amdgcn_fmed3f(fmaf(d[0][r], inv, nlo), 0.0f, 15.0f);
            const float t1 = __builtin_amdgcn_fmed3f(fmaf(d[1][r], inv, nlo), 0.0f, 15.0f);
            ev = __builtin_amdgcn_cvt_pk_u8_f32(t0, r, ev);     // round-half-to-even, NaN -> 0
            od = __builtin_amdgcn_cvt_pk_u8_f32(t1, r, od);
        }
        int sum = __builtin_amdgcn_udot4(ev, 0x01010101u, 0, false);
        sum = __builtin_amdgcn_udot4(od, 0x01010101u, sum, false);
        sum = row_sum(sum);
        const uint32_t mine = ev | (od << 4);                   // byte r = the packed byte at 256c + 64g + 16r + col
        const uint32_t x0 = (uint32_t)rh_dppi<0x00>((int)mine), x1 = (uint32_t)rh_dppi<0x55>((int)mine);
        const uint32_t x2 = (uint32_t)rh_dppi<0xAA>((int)mine), x3 = (uint32_t)rh_dppi<0xFF>((int)mine);
        const uint32_t word = __builtin_amdgcn_perm(x1, x0, sel01) | __builtin_amdgcn_perm(x3, x2, sel23);
        // lane (quad q = col/4, i = col%4) now holds bytes 256c + 64g + 16i + 4q .. +3
        *reinterpret_cast<uint32_t*>(a.Aq + m * (int64_t)(K / 2) + 256 * c + 64 * g + 16 * qi + 4 * (col >> 2)) = word;
        if (col == 0) {
            basq_tokmeta mt;
            mt.scale = s; mt.lo = lo; mt.rowsum = sum; mt.reserved = 0;
            a.meta[m * hpt + 4 * c + g] = mt;
        }
    }
}

template <bool HB, bool HS>
int launch_head_flags(const RotateQuantArgs& a, hipStream_t s, unsigned blocks, size_t lds, float norm) {
    if (a.rot_out)
        hipLaunchKernelGGL((rotate_quant_head_kernel<HB, HS, true>), dim3(blocks), dim3(RH_THREADS), lds, s, a, norm);
    else
        hipLaunchKernelGGL((rotate_quant_head_kernel<HB, HS, false>), dim3(blocks), dim3(RH_THREADS), lds, s, a, norm);
    return check_hip(hipGetLastError(), "rotate_quant (per head) launch");
}

}  // namespace

bool rotate_quant_head_applicable(const RotateQuantArgs& a) {
    // the staged bias and s^a must fit the default 64 KB of dynamic LDS
    const size_t lds = (size_t)a.K * sizeof(float) * ((a.bias ? 1 : 0) + (a.act_scale ? 1 : 0));
    return !a.has28 && a.rot_size == 128 && a.group == 128 && a.K % 512 == 0 && a.Aq != nullptr && a.meta != nullptr &&
           a.Aq6 == nullptr && lds <= 64 * 1024;
}

int launch_rotate_quant_head(const RotateQuantArgs& a, hipStream_t s) {
    const int64_t items = a.M * (int64_t)(a.K / 512);
    const int64_t want = (items + RH_WAVES - 1) / RH_WAVES;
    const int64_t cap = 256 * 8;                                // eight workgroups per compute unit
    const unsigned blocks = (unsigned)(want < cap ? want : cap);
    const size_t lds = (size_t)a.K * sizeof(float) * ((a.bias ? 1 : 0) + (a.act_scale ? 1 : 0));
    const float norm = (float)(1.0 / sqrt(128.0));
    const bool hb = a.bias != nullptr, hs = a.act_scale != nullptr;
    if (hb && hs) return launch_head_flags<true, true>(a, s, blocks, lds, norm);
    if (hb) return launch_head_flags<true, false>(a, s, blocks, lds, norm);
    if (hs) return launch_head_flags<false, true>(a, s, blocks, lds, norm);
    return launch_head_flags<false, false>(a, s, blocks, lds, norm);
}

}  // namespace basq
