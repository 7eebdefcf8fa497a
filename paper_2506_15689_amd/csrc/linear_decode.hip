// The whole layer in ONE launch for the smallest decode calls (M <= 4 tokens, rot_size == K in {4096, 8192}, at
// most one workgroup per compute unit: N <= 4096).  At this size the two-kernel path is bound by launch and
// dependency latency (each kernel lasts about 5 us for about 1 us of memory traffic), so every workgroup
// rotates and quantises the few tokens itself -- the same per-token routine as the rotate+quant kernel, hence
// the same bits -- while its slice of the weights is already on its way from memory.  One wavefront takes
// about 2.8 us per token when it is alone on its SIMD (about 900 dependent vector instructions), so the kernel
// pays only while each wave has at most one token: measured 7.8 us against 9.8 us per step at M = 1, and
// 19.6 us against 11.4 us at M = 16, which therefore stays on the two-kernel path.
// (Paper Sec. 5.2 measures the layer's speed; the arithmetic is Eq. 14 / Eq. 4 as in the two kernels.)
//
//   phase 0   every lane requests all of its 16-byte weight pieces (streaming layout) and its epilogue constants
//   phase 1   wave w rotates and quantises tokens w, w+4, ...; codes and token records go to LDS
//             (one or two tokens of K = 4096, one of K = 8192: several waves per token, see "split mode" below)
//   phase 2   16 x 16 x 64 int8 MFMA on the weights (registers) and the codes (LDS), cross-wave reduction,
//             de-quantisation, bf16 store -- as in the weight-streaming kernel
#include "rotate_pow2_token.h"

namespace basq {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int LD_WAVES = 4;
constexpr int LD_THREADS = LD_WAVES * 64;
constexpr int LD_ROWS = 16;                 // output channels per workgroup
constexpr int LD_MAX_TOKENS = 4;            // one token per wave

template <int NC, bool FOLD_NORM, bool HAS_BIAS, bool HAS_SCALE>
__global__ __launch_bounds__(LD_THREADS, 1) void linear_decode_kernel(RotateQuantArgs q, GemmArgs g, float norm) {
    constexpr int K = 512 * NC, KB = K / 2;
    constexpr int NCHUNKS = KB / 64;                    // 64-byte chunks per row
    constexpr int STEPS = NCHUNKS / LD_WAVES;           // chunks per wave: all of them in registers at once
    constexpr int XQ_STRIDE = KB + 16;                  // bytes per token in LDS: the tokens of a quarter wave read
                                                        // 16-byte pieces that fall on different bank groups
    __shared__ __attribute__((aligned(16))) float tr[LD_WAVES * P2_LDS_WORDS];
    __shared__ __attribute__((aligned(16))) float lbias_s[HAS_BIAS ? K : 4];
    __shared__ __attribute__((aligned(16))) uint8_t xq[LD_MAX_TOKENS * XQ_STRIDE];
    __shared__ basq_tokmeta lmeta[LD_MAX_TOKENS];
    __shared__ int lsum_hi[LD_MAX_TOKENS];               // split mode: the row sums of a token's blocks other than the first
    __shared__ int part[LD_WAVES][LD_ROWS * 16];
    // split mode (K = 4096: at most two tokens, two waves each; K = 8192: one token on all four waves), see below
    constexpr int NWAY = NC / 4;                         // waves per token in split mode
    __shared__ __attribute__((aligned(16))) float4 xch[LD_WAVES * 8 * 64];
    __shared__ float lred[LD_WAVES * 2];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int M = (int)g.M;
    const int n0 = blockIdx.x * LD_ROWS;

    // ---- phase 0: the weight stream ---------------------------------------------------------------
    const uint8_t* wblk = g.Wq + (int64_t)n0 * KB + lane * 16;        // piece `lane` of each of the block's KBs
    v4i w[STEPS];
#pragma unroll
    for (int i = 0; i < STEPS; ++i)
        w[i] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(wblk + (wave + i * LD_WAVES) * 1024));
    const int orow = tid & 15, otok = tid >> 4;
    const int on = n0 + orow;
    const bool out_ok = otok < M && on < g.N;
    float sw = 0.f, zp = 0.f, ws = 0.f, cb = 0.f;
    if (out_ok) {
        sw = bf16_to_f32(g.w_scale[on]);
        zp = bf16_to_f32(g.w_zero[on]);
        ws = g.w_sum[on];
        cb = g.out_bias ? g.out_bias[on] : 0.0f;
    }

    // ---- phase 1: rotate + quantise the tokens into LDS ---------------------------------------------------
    v8bf bop[2];
    p2_make_bop<NC, FOLD_NORM>(lane, bop);
    const P2Lane pl = p2_lane(lane);
    uint4 raw[NC];
    auto load_token = [&](int t) {
        const uint16_t* x = q.X + t * q.ldx + 8 * pl.chunk;
#pragma unroll
        for (int c = 0; c < NC; ++c) raw[c] = nt_load16(x + 512 * c);
    };
    // Split mode: with so few tokens that every token can have NWAY waves, they share it (p2_token_split: same bits).
    const bool split_mode = M * NWAY <= LD_WAVES;                       // uniform over the grid
    if (split_mode) {
        if (tid < LD_MAX_TOKENS) lsum_hi[tid] = 0;
        const int t = wave / NWAY, half = wave % NWAY;                  // token, and this wave's 2048-channel block of it
        const bool active = t < M;
        uint4 raw4[4] = {};
        if (active) {
            const uint16_t* x = q.X + t * q.ldx + 8 * pl.chunk + 2048 * half;
#pragma unroll
            for (int j = 0; j < 4; ++j) raw4[j] = nt_load16(x + 512 * j);
        }
        if (HAS_BIAS) p2_stage_bias<K>(lbias_s, q.bias, tid, LD_THREADS);   // complete behind the routine's first barrier
        const P2Meta tm = p2_token_split<NWAY, FOLD_NORM, HAS_BIAS, HAS_SCALE>(
            active, half, raw4, bop, tr + wave * P2_LDS_WORDS, xch + t * (NWAY * 512), lred + t * (NWAY * 2),
            reinterpret_cast<const float4*>(lbias_s), q.act_scale, norm, q.clip_lo, q.clip_hi, lane,
            pl.wbase, pl.rbase, [&](const uint32_t (&words)[4], const v16f&, const v16f&) {
                *reinterpret_cast<uint4*>(xq + t * XQ_STRIDE + 1024 * half + 16 * lane) =
                    make_uint4(words[0], words[1], words[2], words[3]);
            });
        if (active && lane == 0) {
            if (half == 0) {
                basq_tokmeta mt;
                mt.scale = tm.scale; mt.lo = tm.lo; mt.rowsum = tm.rowsum; mt.reserved = 0;
                lmeta[t] = mt;
            } else {
                atomicAdd(&lsum_hi[t], tm.rowsum);       // LDS integer adds: any order gives the same sum
            }
        }
    } else {
    if (tid < LD_MAX_TOKENS) lsum_hi[tid] = 0;
    if (wave < M) load_token(wave);
    if (HAS_BIAS) p2_stage_bias<K>(lbias_s, q.bias, tid, LD_THREADS);
    __syncthreads();
    for (int t = wave; t < M; t += LD_WAVES) {
        if (t != wave) load_token(t);
        const P2Meta tm = p2_token<NC, FOLD_NORM, HAS_BIAS, HAS_SCALE, false, false>(
            raw, bop, tr + wave * P2_LDS_WORDS, reinterpret_cast<const float4*>(lbias_s), q.act_scale, nullptr, norm,
            q.clip_lo, q.clip_hi, lane, pl.wbase, pl.rbase, []() {},
            [&](int hf, int b, const uint32_t (&words)[4], const v16f&, const v16f&) {
                *reinterpret_cast<uint4*>(xq + t * XQ_STRIDE + 2048 * hf + 1024 * b + 16 * lane) =
                    make_uint4(words[0], words[1], words[2], words[3]);
            },
            [](int, int, float, float, int) {});
        if (lane == 0) {
            basq_tokmeta mt;
            mt.scale = tm.scale; mt.lo = tm.lo; mt.rowsum = tm.rowsum; mt.reserved = 0;
            lmeta[t] = mt;
        }
    }
    }
    __syncthreads();

    // ---- phase 2: product, reduction, de-quantisation ------------------------------------------------------
    const int row = lane & 15, sub = lane >> 4;          // operand lane: weight row / token `row`, k-block `sub`
    const bool t_ok = row < M;
    const uint8_t* xrow = xq + (t_ok ? row : 0) * XQ_STRIDE + sub * 16;
    v4i acc = {0, 0, 0, 0}, acc2 = {0, 0, 0, 0};       // two chains: low and high nibbles
#pragma unroll
    for (int i = 0; i < STEPS; ++i) {
        const int c = wave + i * LD_WAVES;
        v4i x = {0, 0, 0, 0};
        if (t_ok) x = *reinterpret_cast<const v4i*>(xrow + c * 64);
        const v4i wlo = w[i] & 0x0F0F0F0F, whi = (w[i] >> 4) & 0x0F0F0F0F;
        const v4i xlo = x & 0x0F0F0F0F, xhi = (x >> 4) & 0x0F0F0F0F;
        acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(wlo, xlo, acc, 0, 0, 0);
        acc2 = __builtin_amdgcn_mfma_i32_16x16x64_i8(whi, xhi, acc2, 0, 0, 0);
    }
    acc += acc2;
    // accumulator register r of lane l: weight row 4*(l/16) + r, token l%16
#pragma unroll
    for (int r = 0; r < 4; ++r) part[wave][(4 * sub + r) * 16 + row] = acc[r];
    __syncthreads();
    int av = 0;
#pragma unroll
    for (int wv = 0; wv < LD_WAVES; ++wv) av += part[wv][orow * 16 + otok];
    if (out_ok) {
        const basq_tokmeta mt = lmeta[otok];
        const float t = (float)av - zp * (float)(mt.rowsum + lsum_hi[otok]);
        const float y = fmaf(mt.scale * sw, t, fmaf(mt.lo, ws, cb));
        g.Y[(int64_t)otok * g.ldy + on] = f32_to_bf16(y);
    }
}

template <int NC, bool FOLD>
int launch_ld(const RotateQuantArgs& q, const GemmArgs& g, hipStream_t s, unsigned blocks, float norm) {
    const bool hb = q.bias != nullptr, hs = q.act_scale != nullptr;
    if (hb && hs) hipLaunchKernelGGL((linear_decode_kernel<NC, FOLD, true, true>), dim3(blocks), dim3(LD_THREADS), 0, s, q, g, norm);
    else if (hb) hipLaunchKernelGGL((linear_decode_kernel<NC, FOLD, true, false>), dim3(blocks), dim3(LD_THREADS), 0, s, q, g, norm);
    else if (hs) hipLaunchKernelGGL((linear_decode_kernel<NC, FOLD, false, true>), dim3(blocks), dim3(LD_THREADS), 0, s, q, g, norm);
    else hipLaunchKernelGGL((linear_decode_kernel<NC, FOLD, false, false>), dim3(blocks), dim3(LD_THREADS), 0, s, q, g, norm);
    return check_hip(hipGetLastError(), "linear_decode launch");
}

}  // namespace

bool linear_decode_applicable(const RotateQuantArgs& q, const GemmArgs& g) {
    // one workgroup per compute unit at most: beyond that the repeated rotation costs more than the launch it saves
    return g.M >= 1 && g.M <= LD_MAX_TOKENS && g.N <= 256 * LD_ROWS && g.w_layout == BASQ_W_DECODE16 &&
           !q.has28 && q.rot_size == q.K && q.group == q.K && (q.K == 4096 || q.K == 8192) &&
           q.rot_out == nullptr && g.acc_out == nullptr;
}

int launch_linear_decode(const RotateQuantArgs& q, const GemmArgs& g, hipStream_t s) {
    const unsigned blocks = (unsigned)((g.N + LD_ROWS - 1) / LD_ROWS);
    const float norm = (float)(1.0 / sqrt((double)q.K));
    if (q.K == 4096) return launch_ld<8, true>(q, g, s, blocks, norm);
    return launch_ld<16, false>(q, g, s, blocks, norm);
}

}  // namespace basq
