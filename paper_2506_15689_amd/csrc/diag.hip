// Diagnostic kernels that measure what this machine sustains, so that the benchmark can report
// each hot kernel against a measured ceiling next to the published peak:
//   basq_diag_stream   a pure streaming kernel with the rotate+quant kernel's access pattern
//                      (one wave per token, 2K bytes in, K/2 + 16 bytes out, non-temporal)
//   basq_diag_read     a read-only streaming kernel with the decode kernel's access pattern (a workgroup
//                      requests 32 KB, eight 16-byte non-temporal loads per lane, before it consumes any)
//   basq_diag_mfma_i8  a register-resident v_mfma_i32_32x32x32_i8 loop, 4-bit valued operands
//   basq_diag_mfma_f6  the same with v_mfma_f32_32x32x64_f8f6f4 on fp6 (e2m3) operands that encode 4-bit codes
// Neither computes anything of the method.
#include "basq_internal.h"

namespace basq {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void diag_stream_kernel(const uint8_t* src, uint8_t* dst, uint8_t* meta, int64_t tokens, int K) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t wid = (int64_t)blockIdx.x * 4 + wave, stride = (int64_t)gridDim.x * 4;
    const int nload = K / 512;        // 16-byte loads per lane per token
    const int nstore = K / 2048;      // 16-byte stores per lane per token
    uint4 acc = make_uint4(0, 0, 0, 0);
    for (int64_t m = wid; m < tokens; m += stride) {
        const uint8_t* x = src + m * (int64_t)(2 * K) + lane * 16;
        for (int c = 0; c < nload; ++c) {
            const uint4 r = nt_load16(x + c * 1024);
            acc.x ^= r.x; acc.y += r.y; acc.z ^= r.z; acc.w += r.w;
        }
        uint8_t* y = dst + m * (int64_t)(K / 2) + lane * 16;
        for (int c = 0; c < nstore; ++c) nt_store16(y + c * 1024, acc);
        if (lane == 0) *reinterpret_cast<uint4*>(meta + m * 16) = acc;
    }
}

__global__ __launch_bounds__(256) void diag_read_kernel(const uint8_t* src, int64_t spans, uint32_t* out) {
    uint4 acc = make_uint4(0, 0, 0, 0);
    for (int64_t sp = blockIdx.x; sp < spans; sp += gridDim.x) {
        const uint8_t* p = src + sp * 32768 + threadIdx.x * 16;
        uint4 r[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) r[i] = nt_load16(p + i * 4096);
#pragma unroll
        for (int i = 0; i < 8; ++i) { acc.x ^= r[i].x; acc.y += r[i].y; acc.z ^= r[i].z; acc.w += r[i].w; }
    }
    out[blockIdx.x * 256 + threadIdx.x] = acc.x ^ acc.y ^ acc.z ^ acc.w;
}

__global__ __launch_bounds__(256) void diag_mfma_kernel(int* out, int iters) {
    v16i acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0;
    const int l = threadIdx.x;
    v4i a[2], b[2];
    a[0] = v4i{(l * 0x01030507) & 0x0F0F0F0F, (l * 0x0B0D1113) & 0x0F0F0F0F, 0x01020304, 0x0A0B0C0D};
    a[1] = v4i{(l * 0x11070503) & 0x0F0F0F0F, 0x0F0E0D0C, (l * 0x05030107) & 0x0F0F0F0F, 0x03020100};
    b[0] = v4i{0x08070605, (l * 0x07050301) & 0x0F0F0F0F, 0x0C0B0A09, (l * 0x0D0B0705) & 0x0F0F0F0F};
    b[1] = v4i{(l * 0x03050709) & 0x0F0F0F0F, 0x04030201, 0x0E0D0C0B, (l * 0x09070503) & 0x0F0F0F0F};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i & 1], b[(i >> 1) & 1], acc[i], 0, 0, 0);
            acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[(i + 1) & 1], b[i & 1], acc[i], 0, 0, 0);
        }
    }
    int s = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

// six-bit fields of a dword pattern forced into the range of the codes' encodings (0..15: the e2m3 values
// q/8); field boundaries do not matter for a throughput loop, only realistic bits
__device__ __forceinline__ int fp6_bits(int x) { return x & 0x3CF3CF3C; }

__global__ __launch_bounds__(256) void diag_mfma_f6_kernel(float* out, int iters) {
    v16f acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;
    const int l = threadIdx.x;
    v8i a[2], b[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int d = 0; d < 8; ++d) {
            a[t][d] = d < 6 ? fp6_bits((l + 3 * t + 1) * (0x01030507 + 0x00020406 * d)) : 0;
            b[t][d] = d < 6 ? fp6_bits((l + 5 * t + 2) * (0x0B0D1113 + 0x00040208 * d)) : 0;
        }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[i & 1], b[(i >> 1) & 1], acc[i], 2, 2, 0, 0, 0, 0);
            acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[(i + 1) & 1], b[i & 1], acc[i], 2, 2, 0, 0, 0, 0);
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace
}  // namespace basq

using namespace basq;

extern "C" {

int basq_diag_stream(const void* src, void* dst, void* meta, int64_t tokens, int32_t K, void* stream) {
    if (!src || !dst || !meta) return fail(BASQ_EINVAL, "diag_stream: a pointer is null");
    if (tokens < 1 || K < 2048 || K % 2048 != 0) return fail(BASQ_EINVAL, "diag_stream: K must be a multiple of 2048, tokens >= 1");
    const int64_t want = (tokens + 3) / 4;
    const unsigned blocks = (unsigned)(want < 1024 ? want : 1024);
    hipLaunchKernelGGL(diag_stream_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint8_t*>(src), static_cast<uint8_t*>(dst), static_cast<uint8_t*>(meta), tokens, K);
    return check_hip(hipGetLastError(), "diag_stream launch");
}

int basq_diag_read(const void* src, int64_t bytes, uint32_t* out, int32_t blocks, void* stream) {
    if (!src || !out) return fail(BASQ_EINVAL, "diag_read: a pointer is null");
    if (bytes < 32768 || bytes % 32768 != 0 || blocks < 1 || blocks > 65536)
        return fail(BASQ_EINVAL, "diag_read: bytes must be a positive multiple of 32768, blocks in 1..65536");
    hipLaunchKernelGGL(diag_read_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint8_t*>(src), bytes / 32768, out);
    return check_hip(hipGetLastError(), "diag_read launch");
}

int basq_diag_mfma_i8(int32_t* out, int32_t blocks, int32_t iters, void* stream) {
    if (!out || blocks < 1 || iters < 1) return fail(BASQ_EINVAL, "diag_mfma_i8: bad argument");
    hipLaunchKernelGGL(diag_mfma_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream), out, iters);
    return check_hip(hipGetLastError(), "diag_mfma_i8 launch");
}

int basq_diag_mfma_f6(float* out, int32_t blocks, int32_t iters, void* stream) {
    if (!out || blocks < 1 || iters < 1) return fail(BASQ_EINVAL, "diag_mfma_f6: bad argument");
    hipLaunchKernelGGL(diag_mfma_f6_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream), out, iters);
    return check_hip(hipGetLastError(), "diag_mfma_f6 launch");
}

}  // extern "C"
