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
    __shared__ __attribute__((aligned(16))) float lscale_s[HAS_SCALE ? K : 4];
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

    // ---- phase 0: requests, in the order their data is needed ----------------------------------------------
    // Vector-memory loads of a wave complete in issue order, so whatever is requested behind the weight stream
    // cannot be used before all of the wave's weights have arrived (3.8 us into the kernel).  The token and the
    // channel bias are therefore requested first: the rotation then runs while the weights stream in.
    v8bf bop[2];
    p2_make_bop<NC, FOLD_NORM>(lane, bop);
    const P2Lane pl = p2_lane(lane);
    const bool split_mode = M * NWAY <= LD_WAVES;                       // uniform over the grid
    uint4 raw[NC];
    uint4 raw4[4] = {};
    auto load_token = [&](int t) {
        const uint16_t* x = q.X + t * q.ldx + 8 * pl.chunk;
#pragma unroll
        for (int c = 0; c < NC; ++c) raw[c] = nt_load16(x + 512 * c);
    };
    if (split_mode) {
        const int t = wave / NWAY, half = wave % NWAY;
        if (t < M) {
            const uint16_t* x = q.X + t * q.ldx + 8 * pl.chunk + 2048 * half;
#pragma unroll
            for (int j = 0; j < 4; ++j) raw4[j] = nt_load16(x + 512 * j);
        }
    } else if (wave < M) {
        load_token(wave);
    }
    // b^c and s^a: K / 4 / 256 = 4 or 8 float4 pieces per thread each, held in named registers until they are staged
    // below (an array here ends up in LDS scratch, whose store would wait for the data at once)
    constexpr int VEC_PIECES = K / 4 / LD_THREADS;
    constexpr int BIAS_PIECES = HAS_BIAS ? VEC_PIECES : 0, SCALE_PIECES = HAS_SCALE ? VEC_PIECES : 0;
    static_assert(VEC_PIECES <= 8, "eight pieces of a channel vector per thread at most");
    float4 bp0 = {}, bp1 = {}, bp2 = {}, bp3 = {}, bp4 = {}, bp5 = {}, bp6 = {}, bp7 = {};
    float4 sp0 = {}, sp1 = {}, sp2 = {}, sp3 = {}, sp4 = {}, sp5 = {}, sp6 = {}, sp7 = {};
#define LD_VEC_LOAD(i) do { \
        if (BIAS_PIECES > i) bp##i = *reinterpret_cast<const float4*>(q.bias + 4 * (tid + i * LD_THREADS)); \
        if (SCALE_PIECES > i) sp##i = *reinterpret_cast<const float4*>(q.act_scale + 4 * (tid + i * LD_THREADS)); } while (0)
    LD_VEC_LOAD(0); LD_VEC_LOAD(1); LD_VEC_LOAD(2); LD_VEC_LOAD(3);
    LD_VEC_LOAD(4); LD_VEC_LOAD(5); LD_VEC_LOAD(6); LD_VEC_LOAD(7);
#undef LD_VEC_LOAD
    __builtin_amdgcn_sched_barrier(0);                   // keep the issue order: the compiler would move the weights up
    const uint8_t* wblk = g.Wq + (int64_t)n0 * KB + lane * 16;        // piece `lane` of each of the block's KBs
    v4i w[STEPS];
#pragma unroll
    for (int i = 0; i < STEPS; ++i)
        w[i] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(wblk + (wave + i * LD_WAVES) * 1024));
    const int orow = tid & 15, otok = tid >> 4;
    const int on = n0 + orow;
    const bool out_ok = otok < M && on < g.N;
    // the epilogue's constants: requested without a branch (clamped row) and converted only where they are used -- a
    // conversion here would wait for them, and with them for the weights requested before them
    const int on_c = on < g.N ? on : g.N - 1;
    const uint16_t sw_bits = g.w_scale[on_c], zp_bits = g.w_zero[on_c];
    const float ws = g.w_sum[on_c];
    float cb = 0.0f;
    if (g.out_bias) cb = g.out_bias[on_c];
    __builtin_amdgcn_sched_barrier(0);
    {                                                     // the staged layout of p2_stage_bias
        float4* dstb = reinterpret_cast<float4*>(lbias_s);
        float4* dsts = reinterpret_cast<float4*>(lscale_s);
#define LD_VEC_STAGE(i) do { \
        const int e = 4 * (tid + i * LD_THREADS), at = ((e >> 11) * 8 + ((e & 31) >> 2)) * 64 + ((e & 2047) >> 5); \
        if (BIAS_PIECES > i) dstb[at] = bp##i; \
        if (SCALE_PIECES > i) dsts[at] = sp##i; } while (0)
        LD_VEC_STAGE(0); LD_VEC_STAGE(1); LD_VEC_STAGE(2); LD_VEC_STAGE(3);
        LD_VEC_STAGE(4); LD_VEC_STAGE(5); LD_VEC_STAGE(6); LD_VEC_STAGE(7);
#undef LD_VEC_STAGE
    }

    // ---- phase 1: rotate + quantise the tokens into LDS ---------------------------------------------------
    // Split mode: with so few tokens that every token can have NWAY waves, they share it (p2_token_split: same bits).
    if (split_mode) {
        if (tid < LD_MAX_TOKENS) lsum_hi[tid] = 0;
        const int t = wave / NWAY, half = wave % NWAY;                  // token, and this wave's 2048-channel block of it
        const bool active = t < M;
        // (the staged bias is complete behind the routine's first barrier)
        const P2Meta tm = p2_token_split<NWAY, FOLD_NORM, HAS_BIAS, HAS_SCALE>(
            active, half, raw4, bop, tr + wave * P2_LDS_WORDS, xch + t * (NWAY * 512), lred + t * (NWAY * 2),
            reinterpret_cast<const float4*>(lbias_s), reinterpret_cast<const float4*>(lscale_s), norm, q.clip_lo, q.clip_hi, lane,
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
    p2_lds_barrier();                                    // the staged bias
    static_assert(LD_MAX_TOKENS <= LD_WAVES, "one token per wave at most: it was requested in phase 0");
    if (wave < M) {
        const int t = wave;
        const P2Meta tm = p2_token<NC, FOLD_NORM, HAS_BIAS, HAS_SCALE, false, false>(
            raw, bop, tr + wave * P2_LDS_WORDS, reinterpret_cast<const float4*>(lbias_s),
            reinterpret_cast<const float4*>(lscale_s), nullptr, norm,
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
    p2_lds_barrier();                                    // (not __syncthreads(): the weights may still be on their way)

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
    p2_lds_barrier();
    int av = 0;
#pragma unroll
    for (int wv = 0; wv < LD_WAVES; ++wv) av += part[wv][orow * 16 + otok];
    if (out_ok) {
        const basq_tokmeta mt = lmeta[otok];
        const float sw = bf16_to_f32(sw_bits), zp = bf16_to_f32(zp_bits);
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
