// Offline helpers: per-output-channel asymmetric INT4 weight quantisation (paper Sec. 5,
// "Deployment Details": weights are quantised per channel), the fused bias W_hat b^c + b of
// Eq. 14, the column mean that calibrates the channel bias b^c (Sec. 3.2), and the fp32 -> bf16 pass that
// finishes the offline weight rotation W' = W R (Sec. 4: the rotation is folded into the weights).  Not on the timed
// path; written for clarity, one workgroup per row / one thread per column.
#include "basq_internal.h"

namespace basq {

namespace {

constexpr int WQ_THREADS = 256;

template <typename T, typename Op>
__device__ __forceinline__ T block_reduce(T v, T* scratch, Op op) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = op(v, __shfl_xor(v, off, 64));
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    __syncthreads();
    if (lane == 0) scratch[wave] = v;
    __syncthreads();
    T r = scratch[0];
    for (int w = 1; w < WQ_THREADS / 64; ++w) r = op(r, scratch[w]);
    return r;
}

__global__ __launch_bounds__(WQ_THREADS) void quantize_weights_kernel(const uint16_t* W, int N, int K, int64_t ldw,
                                                                      uint8_t* Wq, uint16_t* w_scale, uint16_t* w_zero,
                                                                      float* w_sum) {
    __shared__ float sf[WQ_THREADS / 64];
    __shared__ int si[WQ_THREADS / 64];
    const int n = blockIdx.x, tid = threadIdx.x;
    const uint16_t* w = W + (int64_t)n * ldw;

    float mn = INFINITY, mx = -INFINITY;
    for (int k = tid; k < K; k += WQ_THREADS) {
        const float v = bf16_to_f32(w[k]);
        mn = fminf(mn, v);
        mx = fmaxf(mx, v);
    }
    mn = block_reduce(mn, sf, [](float x, float y) { return fminf(x, y); });
    mx = block_reduce(mx, sf, [](float x, float y) { return fmaxf(x, y); });

    float sw32 = __fdiv_rn(mx - mn, 15.0f);
    if (!(sw32 > 0.0f && sw32 < INFINITY)) sw32 = 1.0f;
    const uint16_t sw_bits = f32_to_bf16(sw32);
    const float sw = bf16_to_f32(sw_bits);
    const float zp = fminf(fmaxf(rintf(__fdiv_rn(-mn, sw)), 0.0f), 15.0f);

    int colsum = 0;
    uint8_t* out = Wq + (int64_t)n * (K / 2);
    for (int j = tid; j < K / 2; j += WQ_THREADS) {
        const float v0 = bf16_to_f32(w[2 * j]), v1 = bf16_to_f32(w[2 * j + 1]);
        const int q0 = (int)fminf(fmaxf(rintf(__fdiv_rn(v0, sw)) + zp, 0.0f), 15.0f);
        const int q1 = (int)fminf(fmaxf(rintf(__fdiv_rn(v1, sw)) + zp, 0.0f), 15.0f);
        out[j] = (uint8_t)(q0 | (q1 << 4));
        colsum += q0 + q1;
    }
    colsum = block_reduce(colsum, si, [](int x, int y) { return x + y; });
    if (tid == 0) {
        w_scale[n] = sw_bits;
        w_zero[n] = f32_to_bf16(zp);
        w_sum[n] = (float)((double)sw * ((double)colsum - (double)K * (double)zp));
    }
}

// out_bias[n] = sum_k W_hat[n,k] b^c[k] + layer_bias[n] (the fused bias of Eq. 14), and, when w_sum is given,
// w_sum[n] = sw_n (sum_k q_w[n,k] - K zp_n) = sum_k W_hat[n,k] (the factor of the activations' lower bound in the
// de-quantisation), both from the packed codes of row n.
__global__ __launch_bounds__(WQ_THREADS) void fused_bias_kernel(const uint8_t* Wq, int N, int K, const uint16_t* w_scale,
                                                                const uint16_t* w_zero, const float* bias,
                                                                const float* layer_bias, float* out_bias, float* w_sum) {
    __shared__ double sd[WQ_THREADS / 64];
    __shared__ int si[WQ_THREADS / 64];
    const int n = blockIdx.x, tid = threadIdx.x;
    const double sw = (double)bf16_to_f32(w_scale[n]);
    const double zp = (double)bf16_to_f32(w_zero[n]);
    const uint8_t* row = Wq + (int64_t)n * (K / 2);
    double acc = 0.0;
    if (bias) {
        for (int j = tid; j < K / 2; j += WQ_THREADS) {
            const int b = row[j];
            acc += sw * ((double)(b & 15) - zp) * (double)bias[2 * j];
            acc += sw * ((double)(b >> 4) - zp) * (double)bias[2 * j + 1];
        }
    }
    acc = block_reduce(acc, sd, [](double x, double y) { return x + y; });
    if (out_bias && tid == 0) out_bias[n] = (float)(acc + (layer_bias ? (double)layer_bias[n] : 0.0));
    if (w_sum) {
        int colsum = 0;
        for (int j = tid; j < K / 2; j += WQ_THREADS) {
            const int b = row[j];
            colsum += (b & 15) + (b >> 4);
        }
        colsum = block_reduce(colsum, si, [](int x, int y) { return x + y; });
        if (tid == 0) w_sum[n] = (float)(sw * ((double)colsum - (double)K * zp));
    }
}

__global__ __launch_bounds__(WQ_THREADS) void column_mean_kernel(const float* r, int64_t M, int K, const float* act_scale,
                                                                 float* out) {
    const int k = blockIdx.x * WQ_THREADS + threadIdx.x;
    if (k >= K) return;
    double acc = 0.0;
    for (int64_t m = 0; m < M; ++m) acc += (double)r[m * K + k];
    double mean = acc / (double)M;
    if (act_scale) mean *= (double)act_scale[k];
    out[k] = (float)mean;
}

}  // namespace

int launch_quantize_weights(const uint16_t* W, int32_t N, int32_t K, int64_t ldw, uint8_t* Wq, uint16_t* w_scale,
                            uint16_t* w_zero, float* w_sum, hipStream_t s) {
    hipLaunchKernelGGL(quantize_weights_kernel, dim3((unsigned)N), dim3(WQ_THREADS), 0, s, W, N, K, ldw, Wq, w_scale,
                       w_zero, w_sum);
    return check_hip(hipGetLastError(), "quantize_weights launch");
}

int launch_fused_bias(const uint8_t* Wq, int32_t N, int32_t K, const uint16_t* w_scale, const uint16_t* w_zero,
                      const float* bias, const float* layer_bias, float* out_bias, float* w_sum, hipStream_t s) {
    hipLaunchKernelGGL(fused_bias_kernel, dim3((unsigned)N), dim3(WQ_THREADS), 0, s, Wq, N, K, w_scale, w_zero, bias,
                       layer_bias, out_bias, w_sum);
    return check_hip(hipGetLastError(), "fused_bias launch");
}

int launch_column_mean(const float* r, int64_t M, int32_t K, const float* act_scale, float* out, hipStream_t s) {
    const unsigned blocks = (unsigned)((K + WQ_THREADS - 1) / WQ_THREADS);
    hipLaunchKernelGGL(column_mean_kernel, dim3(blocks), dim3(WQ_THREADS), 0, s, r, M, K, act_scale, out);
    return check_hip(hipGetLastError(), "column_mean launch");
}

namespace {
__global__ __launch_bounds__(256) void f32_to_bf16_kernel(const float* __restrict__ in, uint16_t* __restrict__ out, int64_t n4) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n4) return;
    const float4 v = reinterpret_cast<const float4*>(in)[i];
    uint2 o;
    o.x = (uint32_t)f32_to_bf16(v.x) | ((uint32_t)f32_to_bf16(v.y) << 16);
    o.y = (uint32_t)f32_to_bf16(v.z) | ((uint32_t)f32_to_bf16(v.w) << 16);
    reinterpret_cast<uint2*>(out)[i] = o;
}
}  // namespace

int launch_f32_to_bf16(const float* in, uint16_t* out, int64_t count, hipStream_t s) {
    const int64_t n4 = count / 4;                       // count is a multiple of 32 (K % 32 == 0)
    const int64_t blocks = (n4 + 255) / 256;
    if (blocks > 0x7FFFFFFFll) return fail(BASQ_EINVAL, "rotate_weights: matrix too large");
    if (blocks > 0) hipLaunchKernelGGL(f32_to_bf16_kernel, dim3((unsigned)blocks), dim3(256), 0, s, in, out, n4);
    return check_hip(hipGetLastError(), "f32_to_bf16 launch");
}

}  // namespace basq
