// Weight-streaming W4A4 product for few tokens (M <= 128: decode, batched decode, speculative decoding): one
// pass over the packed 4-bit weights, bound by HBM bandwidth up to about 64 tokens.  Same arithmetic as the
// prefill GEMM (ACC in INT32, fused de-quantisation).
//
// A workgroup owns 16 or 32 output channels; its waves split K.  Each lane issues a batch of 16-byte weight
// loads before it consumes any, so the whole weight matrix is in flight at once.  The 16 x 16 x 64 int8 MFMA
// takes 16 weight rows as one operand and 16 (zero padded) tokens as the other; more tokens are more token
// tiles against the same weight registers.  Nibbles are split into low/high words exactly as in the prefill
// kernel.
//
// Weight layouts.  The MFMA operand puts 16 different rows on the 16 lanes of a quarter wave, so on
// canonical [N, K/2] weights every load instruction touches 16 rows x 64 bytes and each 128-byte line
// is fetched in eight 16-byte pieces.  The streaming layout (BASQ_W_DECODE16) stores the 1 KB a wave
// load needs contiguously, in lane order: 4 KB contiguous per workgroup step.
#include "basq_internal.h"

namespace basq {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int GV_WAVES = 4;
constexpr int GV_THREADS = GV_WAVES * 64;           // the epilogue maps one thread to each of a tile's 16 x 16 outputs
constexpr int GV_ROWS = 16;                         // output channels per tile

// STEPS: 64-byte k-chunks per lane held in registers at once (all of their loads are in flight together).
// TILES: 16-row weight tiles per workgroup; they share the activation operand, which at 16 tokens is as many
//        L2 bytes per workgroup as one tile's weights.
// TT:    16-token tiles (M <= 16 * TT); they share the weight registers.
template <bool STREAM_LAYOUT, int STEPS, int TILES, int TT>
__global__ __launch_bounds__(GV_THREADS) void gemv_w4a4_kernel(GemmArgs a) {
    constexpr int NT = TILES * TT;                  // accumulator tiles per wave
    constexpr bool TWO_CHAINS = NT <= 2;            // few tiles: low and high nibbles on separate MFMA chains
    __shared__ int part[NT * 256];                  // cross-wave sums (integer adds: any order gives the same bits)

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n0 = blockIdx.x * (GV_ROWS * TILES);
    const int KB = a.K / 2;
    const int nchunks = KB / 64;               // 64-byte chunks per row (K % 128 == 0 checked by the caller)
    const int row = lane & 15, sub = lane >> 4;
    const int M = (int)a.M;

#pragma unroll
    for (int i = 0; i < NT; ++i) part[i * 256 + tid] = 0;

    // chunk c of this lane: canonical = 16 bytes of row n at 64c + 16sub; streaming = piece `lane` of the
    // 16-row block's c-th KB (rows past N are stored as zeros there; a whole block past N does not exist)
    const uint8_t* wrow[TILES];
    bool w_ok[TILES];
#pragma unroll
    for (int t = 0; t < TILES; ++t) {
        const int nt0 = n0 + GV_ROWS * t, n = nt0 + row;
        w_ok[t] = STREAM_LAYOUT ? nt0 < a.N : n < a.N;
        wrow[t] = STREAM_LAYOUT ? a.Wq + (int64_t)(w_ok[t] ? nt0 : 0) * KB + lane * 16
                                : a.Wq + (int64_t)(w_ok[t] ? n : 0) * KB + sub * 16;
    }
    constexpr int WSTEP = STREAM_LAYOUT ? 1024 : 64;
    // the same lane index selects the token of tile tt on the other operand
    const uint8_t* arow[TT];
    bool t_ok[TT];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        t_ok[tt] = 16 * tt + row < M;
        arow[tt] = a.Aq + (int64_t)(t_ok[tt] ? 16 * tt + row : 0) * KB + sub * 16;
    }

    // Epilogue constants and token records of the outputs this thread will finish (16 consecutive channels of one
    // token per 16 threads, one such output per tile), requested now so that their latency overlaps the weight
    // stream: without a branch (clamped indices) and as raw bits -- a conversion here would wait for them before
    // the first weight load is issued, and a record fetched in the epilogue is a memory latency at the very end.
    const int orow = tid & 15, otok = tid >> 4;
    uint16_t sw_bits[TILES], zp_bits[TILES];
    float ws[TILES], cb[TILES];
#pragma unroll
    for (int t = 0; t < TILES; ++t) {
        const int on = n0 + GV_ROWS * t + orow;
        const int on_c = on < a.N ? on : a.N - 1;
        sw_bits[t] = a.w_scale[on_c];
        zp_bits[t] = a.w_zero[on_c];
        ws[t] = a.w_sum[on_c];
        cb[t] = 0.0f;
        if (a.out_bias) cb[t] = a.out_bias[on_c];
    }
    basq_tokmeta mts[TT];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        const int tok = 16 * tt + otok;
        mts[tt] = a.meta[tok < M ? tok : M - 1];
    }

    v4i acc[NT], acc2[TWO_CHAINS ? NT : 1];
#pragma unroll
    for (int i = 0; i < NT; ++i) acc[i] = v4i{0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < (TWO_CHAINS ? NT : 1); ++i) acc2[i] = v4i{0, 0, 0, 0};
    for (int c0 = wave; c0 < nchunks; c0 += GV_WAVES * STEPS) {
        v4i w[TILES][STEPS], x[TT][STEPS];
#pragma unroll
        for (int i = 0; i < STEPS; ++i) {
            const int c = c0 + i * GV_WAVES;
            const bool ok = c < nchunks;
            // the weights are read once per call: streaming (non-temporal) loads
#pragma unroll
            for (int t = 0; t < TILES; ++t)
                w[t][i] = (ok && w_ok[t]) ? __builtin_nontemporal_load(reinterpret_cast<const v4i*>(wrow[t] + c * WSTEP))
                                          : v4i{0, 0, 0, 0};
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
                x[tt][i] = (ok && t_ok[tt]) ? *reinterpret_cast<const v4i*>(arow[tt] + c * 64) : v4i{0, 0, 0, 0};
        }
#pragma unroll
        for (int i = 0; i < STEPS; ++i) {
            v4i wlo[TILES], whi[TILES];
#pragma unroll
            for (int t = 0; t < TILES; ++t) { wlo[t] = w[t][i] & 0x0F0F0F0F; whi[t] = (w[t][i] >> 4) & 0x0F0F0F0F; }
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                const v4i xlo = x[tt][i] & 0x0F0F0F0F, xhi = (x[tt][i] >> 4) & 0x0F0F0F0F;
#pragma unroll
                for (int t = 0; t < TILES; ++t) {
                    const int at = t * TT + tt;
                    acc[at] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wlo[t], xlo, acc[at], 0, 0, 0);
                    if (TWO_CHAINS) acc2[at] = __builtin_amdgcn_mfma_i32_16x16x64_i8(whi[t], xhi, acc2[at], 0, 0, 0);
                    else acc[at] = __builtin_amdgcn_mfma_i32_16x16x64_i8(whi[t], xhi, acc[at], 0, 0, 0);
                }
            }
        }
    }
    // accumulator register r of lane l: weight row 4*(l/16) + r, token l%16
    __syncthreads();                                // every wave has zeroed its share of `part`
#pragma unroll
    for (int at = 0; at < NT; ++at) {
        if (TWO_CHAINS) acc[at] += acc2[at];
#pragma unroll
        for (int r = 0; r < 4; ++r) atomicAdd(&part[at * 256 + (4 * sub + r) * 16 + row], acc[at][r]);
    }
    __syncthreads();

#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        const int tok = 16 * tt + otok;
        if (tok >= M) continue;
        const basq_tokmeta mt = mts[tt];
#pragma unroll
        for (int t = 0; t < TILES; ++t) {
            const int on = n0 + GV_ROWS * t + orow;
            if (on >= a.N) continue;
            const int av = part[(t * TT + tt) * 256 + orow * 16 + otok];
            const float sw = bf16_to_f32(sw_bits[t]), zp = bf16_to_f32(zp_bits[t]);
            const float tv = (float)av - zp * (float)mt.rowsum;
            const float y = fmaf(mt.scale * sw, tv, fmaf(mt.lo, ws[t], cb[t]));
            a.Y[(int64_t)tok * a.ldy + on] = f32_to_bf16(y);
            if (a.acc_out) a.acc_out[(int64_t)tok * a.N + on] = av;
        }
    }
}

// canonical [N, K/2] -> streaming layout: one thread per 16-byte piece of the output
__global__ __launch_bounds__(256) void pack_decode16_kernel(const uint8_t* __restrict__ Wq, int N, int KB,
                                                            uint8_t* __restrict__ out, int64_t pieces) {
    const int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (p >= pieces) return;
    const int nchunks = KB / 64;
    const int ln = (int)(p & 63);
    const int64_t kb = p >> 6;                       // (block, chunk)
    const int c = (int)(kb % nchunks);
    const int64_t n = (kb / nchunks) * 16 + (ln & 15);
    uint4 v = make_uint4(0, 0, 0, 0);
    if (n < N) v = *reinterpret_cast<const uint4*>(Wq + n * KB + 64 * c + 16 * (ln >> 4));
    *reinterpret_cast<uint4*>(out + p * 16) = v;
}

}  // namespace

int launch_pack_decode16(const uint8_t* Wq, int32_t N, int32_t K, uint8_t* out, hipStream_t s) {
    const int KB = K / 2;
    const int64_t pieces = (int64_t)((N + 15) / 16) * (KB / 64) * 64;
    const int64_t blocks = (pieces + 255) / 256;
    if (blocks > 0x7FFFFFFFll) return fail(BASQ_EINVAL, "pack_decode: matrix too large");
    hipLaunchKernelGGL(pack_decode16_kernel, dim3((unsigned)blocks), dim3(256), 0, s, Wq, N, KB, out, pieces);
    return check_hip(hipGetLastError(), "pack_decode launch");
}

template <bool SL, int STEPS, int TILES, int TT>
static void launch_gemv_cfg(const GemmArgs& a, hipStream_t s, int blocks16) {
    hipLaunchKernelGGL((gemv_w4a4_kernel<SL, STEPS, TILES, TT>), dim3((unsigned)((blocks16 + TILES - 1) / TILES)),
                       dim3(GV_THREADS), 0, s, a);
}

template <bool SL, int STEPS, int TT>
static void launch_gemv_tiles(const GemmArgs& a, hipStream_t s, int blocks16) {
    // More weight tiles per workgroup = fewer passes over the activations, which is what bounds the kernel from
    // 32 tokens on -- as long as the workgroups still fill the chip (measured on N = 4096, 12288, 28672)
    if (blocks16 >= 1536) launch_gemv_cfg<SL, STEPS, 4, TT>(a, s, blocks16);
    else if (blocks16 >= 256) launch_gemv_cfg<SL, STEPS, 2, TT>(a, s, blocks16);
    else launch_gemv_cfg<SL, STEPS, 1, TT>(a, s, blocks16);
}

template <bool SL>
static void launch_gemv_layout(const GemmArgs& a, hipStream_t s) {
    const int blocks16 = (a.N + GV_ROWS - 1) / GV_ROWS;
    if (a.M <= 16) {
        // long rows: twice the loads in flight per lane (measured: K = 8192 gains 6 %, K = 4096 loses 5 %)
        const bool deep = a.K / 128 > 32;
        // two tiles per workgroup once the activations weigh in (more than 8 tokens) and the chip stays filled
        if (a.M > 8 && blocks16 >= 4 * 256) launch_gemv_cfg<SL, 8, 2, 1>(a, s, blocks16);
        // 65 .. 112 chunks per row (K = 14336): all of a lane's loads in one batch instead of one and a ragged one
        // (measured 8.0 us against 8.8 us on N = 4096)
        else if (a.K / 128 > 64 && a.K / 128 <= 112) launch_gemv_cfg<SL, 28, 1, 1>(a, s, blocks16);
        else if (deep) launch_gemv_cfg<SL, 16, 1, 1>(a, s, blocks16);
        else launch_gemv_cfg<SL, 8, 1, 1>(a, s, blocks16);
    } else if (a.M <= 32) {
        launch_gemv_tiles<SL, 2, 2>(a, s, blocks16);
    } else if (a.M <= 64) {
        launch_gemv_tiles<SL, 2, 4>(a, s, blocks16);
    } else {
        launch_gemv_tiles<SL, 1, 8>(a, s, blocks16);
    }
}

int launch_gemv_decode(const GemmArgs& a, hipStream_t s) {
    if (a.M == 0) return BASQ_OK;
    if (a.M > GEMV_MAX_TOKENS) return fail(BASQ_EINVAL, "weight-streaming kernel: more than %d tokens", GEMV_MAX_TOKENS);
    if (a.w_layout == BASQ_W_DECODE16) launch_gemv_layout<true>(a, s);
    else launch_gemv_layout<false>(a, s);
    return check_hip(hipGetLastError(), "w4a4_gemv launch");
}

}  // namespace basq
