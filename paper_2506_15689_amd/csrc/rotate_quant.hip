// Online rotation + bias + per-token INT4 quantisation (paper Sec. 3.1 rotation, Eq. 14 bias,
// Eq. 15 asymmetric scale, Eq. 4 quantiser; the "fused quant kernel" of Fig. 6).
//
// Generic kernel: one workgroup per token, the token staged in LDS as fp32.  The Sylvester factor
// is applied as in-register radix-16 butterfly passes over LDS, the optional H_28 factor as 28
// signed sums per column.  All fp32 operations of the quantiser are written out one by one and
// this file is compiled with -ffp-contract=off, so the only fused multiply-adds are the fmaf calls.
#include "basq_internal.h"

namespace basq {

namespace {

constexpr int RQ_THREADS = 256;

struct H28Masks {
    uint32_t col[28];   // bit i of col[j] set  <=>  H28[i][j] == -1
};

__device__ __forceinline__ float wave_min(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fminf(v, __shfl_xor(v, off, 64));
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}
__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// In-register Walsh-Hadamard butterflies on R = 2^NB values.
template <int NB>
__device__ __forceinline__ void butterflies(float (&v)[1 << NB]) {
#pragma unroll
    for (int s = 0; s < NB; ++s) {
        const int h = 1 << s;
#pragma unroll
        for (int i = 0; i < (1 << NB); ++i) {
            if ((i & h) == 0) {
                float a = v[i], b = v[i + h];
                v[i] = a + b;
                v[i + h] = a - b;
            }
        }
    }
}

// One radix-2^NB pass over address bits [b0, b0+NB) of the K floats in sm.
template <int NB>
__device__ __forceinline__ void lds_pass(float* sm, int K, int b0, int tid) {
    constexpr int R = 1 << NB;
    const int stride = 1 << b0;
    for (int g = tid; g < K / R; g += RQ_THREADS) {
        const int low = g & (stride - 1);
        const int base = ((g >> b0) << (b0 + NB)) | low;
        float v[R];
#pragma unroll
        for (int j = 0; j < R; ++j) v[j] = sm[base + j * stride];
        butterflies<NB>(v);
#pragma unroll
        for (int j = 0; j < R; ++j) sm[base + j * stride] = v[j];
    }
}

__global__ __launch_bounds__(RQ_THREADS) void rotate_quant_generic_kernel(RotateQuantArgs a, float norm,
                                                                          int log2p, H28Masks h28) {
    extern __shared__ float sm[];            // K floats, then 3 * (RQ_THREADS/64) reduction slots
    const int K = a.K;
    const int tid = threadIdx.x;
    const int64_t m = blockIdx.x;
    float* red = sm + K;

    // a1: load 8 bf16 (16 bytes) per thread per step, widen to fp32
    const uint16_t* x = a.X + m * a.ldx;
    for (int c = tid; c < K / 8; c += RQ_THREADS) {
        const uint4 raw = *reinterpret_cast<const uint4*>(x + 8 * c);
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            sm[8 * c + 2 * j] = __uint_as_float(w[j] << 16);
            sm[8 * c + 2 * j + 1] = __uint_as_float(w[j] & 0xFFFF0000u);
        }
    }
    __syncthreads();

    // a2: Sylvester factor on address bits [0, log2p) (blocks of 2^log2p are contiguous)
    int b0 = 0;
    while (log2p - b0 >= 4) { lds_pass<4>(sm, K, b0, tid); __syncthreads(); b0 += 4; }
    switch (log2p - b0) {
        case 3: lds_pass<3>(sm, K, b0, tid); __syncthreads(); break;
        case 2: lds_pass<2>(sm, K, b0, tid); __syncthreads(); break;
        case 1: lds_pass<1>(sm, K, b0, tid); __syncthreads(); break;
        default: break;
    }

    // a2 (n = 28 * 2^t): H_28 factor along the stride-2^t axis, u[i', j] = sum_i in[i, j] * H28[i][i']
    if (a.has28) {
        const int P = 1 << log2p;
        const int n = 28 * P;
        for (int col = tid; col < K / 28; col += RQ_THREADS) {
            const int blk = col / P, j = col - blk * P;
            float* p = sm + blk * n + j;
            float in[28];
#pragma unroll
            for (int i = 0; i < 28; ++i) in[i] = p[i * P];
#pragma unroll 4
            for (int o = 0; o < 28; ++o) {
                const uint32_t mask = h28.col[o];
                float acc = 0.0f;
#pragma unroll
                for (int i = 0; i < 28; ++i) acc += ((mask >> i) & 1u) ? -in[i] : in[i];
                p[o * P] = acc;
            }
        }
        __syncthreads();
    }

    // a3 + a4: normalise, scale/bias, running min/max; v is written back to LDS
    float mn = INFINITY, mx = -INFINITY;
    float* rot_row = a.rot_out ? a.rot_out + m * (int64_t)K : nullptr;
    for (int c = tid; c < K / 8; c += RQ_THREADS) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int k = 8 * c + j;
            const float r = sm[k] * norm;
            if (rot_row) rot_row[k] = r;
            const float b = a.bias ? a.bias[k] : 0.0f;
            const float v = a.act_scale ? fmaf(r, a.act_scale[k], -b) : r - b;
            sm[k] = v;
            mn = fminf(mn, v);
            mx = fmaxf(mx, v);
        }
    }
    if (a.Aq == nullptr) return;             // rotation-only mode (bias calibration)

    if (a.group < K) {
        // Group-wise ranges (per-head quantisation of q/k and of the KV cache, paper Sec. 5 "Deployment
        // Details"): one thread per group walks its channels in LDS.  Plain fallback; the per-head shape
        // rot_size = group = 128 has its own kernel.
        __syncthreads();
        const int G = a.group, ngroups = K / G;
        for (int g = tid; g < ngroups; g += RQ_THREADS) {
            const float* v = sm + g * G;
            float gmn = INFINITY, gmx = -INFINITY;
            for (int k = 0; k < G; ++k) { gmn = fminf(gmn, v[k]); gmx = fmaxf(gmx, v[k]); }
            const float lo = a.clip_lo * gmn;
            const float hi = a.clip_hi * gmx;
            float s = __fdiv_rn(hi - lo, 15.0f);
            if (!(s > 0.0f && s < INFINITY)) s = 1.0f;
            const float inv = __fdiv_rn(1.0f, s);
            const float nlo = -(lo * inv);
            int sum = 0;
            uint32_t* arow = reinterpret_cast<uint32_t*>(a.Aq + m * (int64_t)(K / 2) + g * (G / 2));
            for (int c = 0; c < G / 8; ++c) {
                uint32_t packed = 0;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    float t = fmaf(v[8 * c + j], inv, nlo);
                    t = fminf(fmaxf(t, 0.0f), 15.0f);
                    const int q = (int)rintf(t);
                    sum += q;
                    packed |= (uint32_t)q << (4 * j);
                }
                arow[c] = packed;
            }
            basq_tokmeta mt;
            mt.scale = s; mt.lo = lo; mt.rowsum = sum; mt.reserved = 0;
            a.meta[m * ngroups + g] = mt;
        }
        return;
    }

    mn = wave_min(mn);
    mx = wave_max(mx);
    const int wave = tid >> 6, lane = tid & 63;
    constexpr int NW = RQ_THREADS / 64;
    if (lane == 0) { red[wave] = mn; red[NW + wave] = mx; }
    __syncthreads();
    mn = red[0]; mx = red[NW];
#pragma unroll
    for (int w = 1; w < NW; ++w) { mn = fminf(mn, red[w]); mx = fmaxf(mx, red[NW + w]); }

    // per-token constants (every thread computes the same values)
    const float lo = a.clip_lo * mn;
    const float hi = a.clip_hi * mx;
    float s = __fdiv_rn(hi - lo, 15.0f);
    if (!(s > 0.0f && s < INFINITY)) s = 1.0f;
    const float inv = __fdiv_rn(1.0f, s);
    const float nlo = -(lo * inv);

    // a5: quantise, pack two codes per byte (low nibble = even k), row sum
    int sum = 0;
    uint32_t* arow = reinterpret_cast<uint32_t*>(a.Aq + m * (int64_t)(K / 2));
    for (int c = tid; c < K / 8; c += RQ_THREADS) {
        uint32_t packed = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            float t = fmaf(sm[8 * c + j], inv, nlo);
            t = fminf(fmaxf(t, 0.0f), 15.0f);
            const int q = (int)rintf(t);
            sum += q;
            packed |= (uint32_t)q << (4 * j);
        }
        arow[c] = packed;
    }
    sum = wave_sum(sum);
    int* redi = reinterpret_cast<int*>(red + 2 * NW);
    if (lane == 0) redi[wave] = sum;
    __syncthreads();
    if (tid == 0) {
        int tot = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) tot += redi[w];
        basq_tokmeta mt;
        mt.scale = s; mt.lo = lo; mt.rowsum = tot; mt.reserved = 0;
        a.meta[m] = mt;
    }
}

}  // namespace

namespace {
int launch_rotate_quant_generic(const RotateQuantArgs& a, hipStream_t s);
}

int launch_rotate_quant(const RotateQuantArgs& a, hipStream_t s) {
    if (a.M == 0) return BASQ_OK;
    if (a.Aq6 && a.group != a.K) {
        // group-wise ranges: the codes are the same kind of data, the fp6 copy is made from them afterwards
        RotateQuantArgs b = a;
        b.Aq6 = nullptr;
        const int rc = launch_rotate_quant(b, s);
        if (rc != BASQ_OK || !a.Aq) return rc;
        return launch_pack_fp6(a.Aq, a.M, a.K, a.Aq6, s);
    }
    // the two specialised kernels write the fp6 copy of the codes themselves
    if (rotate_quant_pow2_applicable(a)) return launch_rotate_quant_pow2(a, s);
    if (rotate_quant_k28_applicable(a)) return launch_rotate_quant_k28(a, s);
    if (rotate_quant_head_applicable(a)) return launch_rotate_quant_head(a, s);
    // the blockwise kernel and the generic one write the 4-bit codes only; the fp6 copy is made from them
    const int rc = rotate_quant_block_applicable(a) ? launch_rotate_quant_block(a, s) : launch_rotate_quant_generic(a, s);
    if (rc != BASQ_OK || !a.Aq6 || !a.Aq) return rc;
    return launch_pack_fp6(a.Aq, a.M, a.K, a.Aq6, s);
}

namespace {
int launch_rotate_quant_generic(const RotateQuantArgs& a, hipStream_t s) {
    int log2p = 0;
    while ((1 << log2p) < a.pow2) ++log2p;
    H28Masks masks{};
    if (a.has28) {
        const int8_t* h = hadamard28_host();
        for (int j = 0; j < 28; ++j) {
            uint32_t mk = 0;
            for (int i = 0; i < 28; ++i) if (h[i * 28 + j] < 0) mk |= 1u << i;
            masks.col[j] = mk;
        }
    }
    const float norm = (float)(1.0 / sqrt((double)a.rot_size));
    const size_t lds = (size_t)a.K * sizeof(float) + 3 * (RQ_THREADS / 64) * sizeof(float);
    static thread_local size_t lds_allowed = 64 * 1024;
    if (lds > lds_allowed) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(rotate_quant_generic_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return check_hip(e, "hipFuncSetAttribute(rotate_quant)");
        lds_allowed = 160 * 1024;
    }
    if (a.M > 0x7FFFFFFFll) return fail(BASQ_EINVAL, "rotate_quant: M too large");
    hipLaunchKernelGGL(rotate_quant_generic_kernel, dim3((unsigned)a.M), dim3(RQ_THREADS), lds, s, a, norm, log2p, masks);
    return check_hip(hipGetLastError(), "rotate_quant launch");
}

}  // namespace

}  // namespace basq
