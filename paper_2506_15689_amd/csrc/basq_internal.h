// Internal declarations shared by the HIP translation units of libbasq (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/basq.h"

namespace basq {

// ---- error reporting (api.hip) ---------------------------------------------------------------
int fail(int code, const char* fmt, ...);
int check_hip(hipError_t e, const char* what);

// ---- launchers; every argument already validated by the C-ABI layer --------------------------
struct RotateQuantArgs {
    const uint16_t* X;        // bf16 bits
    int64_t M;
    int32_t K;
    int64_t ldx;
    int32_t rot_size;         // n
    int32_t pow2;             // Sylvester factor of n (n itself, or n/28)
    int32_t has28;            // 1 if n = 28 * pow2
    const float* bias;
    const float* act_scale;
    float clip_lo, clip_hi;
    int32_t group;            // channels that share one range and one token record (K: the whole token)
    uint8_t* Aq;              // may be null in rot-only mode
    basq_tokmeta* meta;       // [M, K/group]; may be null in rot-only mode
    float* rot_out;           // optional
    uint8_t* Aq6;             // optional: the codes once more in the fp6 operand form (fp6_pack.hip)
};
int launch_rotate_quant(const RotateQuantArgs& a, hipStream_t s);
// register-resident kernel for rot_size == K in {4096, 8192} (rotate_quant_pow2.hip)
bool rotate_quant_pow2_applicable(const RotateQuantArgs& a);
int launch_rotate_quant_pow2(const RotateQuantArgs& a, hipStream_t s);
// wave-local kernel for per-head work: rot_size == group == 128, K % 512 == 0 (rotate_quant_head.hip)
bool rotate_quant_head_applicable(const RotateQuantArgs& a);
int launch_rotate_quant_head(const RotateQuantArgs& a, hipStream_t s);
// blockwise rotations of 128, 256 or 512 channels with per-token ranges, K <= 16384 (rotate_quant_block.hip)
bool rotate_quant_block_applicable(const RotateQuantArgs& a);
int launch_rotate_quant_block(const RotateQuantArgs& a, hipStream_t s);
// kernel for rot_size == K == 14336 = 28 * 512 (rotate_quant_k28.hip)
bool rotate_quant_k28_applicable(const RotateQuantArgs& a);
int launch_rotate_quant_k28(const RotateQuantArgs& a, hipStream_t s);

struct GemmArgs {
    const uint8_t* Aq;
    const basq_tokmeta* meta;
    int64_t M;
    int32_t K;
    const uint8_t* Wq;
    int32_t N;
    const uint16_t* w_scale;  // bf16 bits
    const uint16_t* w_zero;
    const float* w_sum;
    const float* out_bias;
    uint16_t* Y;
    int64_t ldy;
    int32_t* acc_out;
    // fp6 operand form of both matrices; both or neither (gemm_w4a4_fp6.hip)
    const uint8_t* Aq6;
    const uint8_t* Wq6;
    int32_t w_layout;         // layout of Wq: BASQ_W_CANONICAL, or BASQ_W_DECODE16 (read by the weight-streaming kernel only)
};
int launch_gemm_prefill(const GemmArgs& a, hipStream_t s);
// direct-to-LDS kernel for K % 256 == 0 (gemm_w4a4_direct.hip)
bool gemm_direct_applicable(const GemmArgs& a);
int launch_gemm_direct(const GemmArgs& a, hipStream_t s);
// activations quantised in groups of 128 channels (gemm_w4a4_grouped.hip); a.meta is [M, K/128]
bool gemm_grouped_applicable(const GemmArgs& a);
int launch_gemm_grouped(const GemmArgs& a, const int32_t* w_gsum, hipStream_t s);
int launch_group_colsums(const uint8_t* Wq, int32_t N, int32_t K, int32_t* out, hipStream_t s);
// the same product on the f8f6f4 matrix-core path: a.Aq6 / a.Wq6 in the fp6 operand form (gemm_w4a4_grouped_fp6.hip)
bool gemm_grouped_fp6_applicable(const GemmArgs& a);
int launch_gemm_grouped_fp6(const GemmArgs& a, const int32_t* w_gsum, hipStream_t s);
constexpr int GEMV_MAX_TOKENS = 128;                          // above it the tiled GEMMs take over
int launch_gemv_decode(const GemmArgs& a, hipStream_t s);   // M <= GEMV_MAX_TOKENS, K % 128 == 0
// one launch for the whole layer at decode size (linear_decode.hip)
bool linear_decode_applicable(const RotateQuantArgs& q, const GemmArgs& g);
int launch_linear_decode(const RotateQuantArgs& q, const GemmArgs& g, hipStream_t s);
int launch_pack_decode16(const uint8_t* Wq, int32_t N, int32_t K, uint8_t* out, hipStream_t s);
// f8f6f4 MFMA kernel on the fp6 operand form, K % 128 == 0 (gemm_w4a4_fp6.hip)
bool gemm_fp6_applicable(const GemmArgs& a);
int launch_gemm_fp6(const GemmArgs& a, hipStream_t s);
// INT4 codes [rows, K/2] -> fp6 operand form (fp6_pack.hip)
int launch_pack_fp6(const uint8_t* codes, int64_t rows, int32_t K, uint8_t* out6, hipStream_t s);

int launch_quantize_weights(const uint16_t* W, int32_t N, int32_t K, int64_t ldw, uint8_t* Wq,
                            uint16_t* w_scale, uint16_t* w_zero, float* w_sum, hipStream_t s);
// out_bias and w_sum may each be null (not computed)
int launch_fused_bias(const uint8_t* Wq, int32_t N, int32_t K, const uint16_t* w_scale, const uint16_t* w_zero,
                      const float* bias, const float* layer_bias, float* out_bias, float* w_sum, hipStream_t s);
int launch_f32_to_bf16(const float* in, uint16_t* out, int64_t count, hipStream_t s);
int launch_column_mean(const float* r, int64_t M, int32_t K, const float* act_scale, float* out, hipStream_t s);

// 28 x 28 Paley type-I matrix, row-major, built on the host at first use (hadamard28.hip).
const int8_t* hadamard28_host();

// ---- small device helpers --------------------------------------------------------------------
// 16-byte loads and stores with the non-temporal hint: streamed data (activations in, codes out) should
// not displace what the caches are better used for; on this part it also raises the sustained
// HBM rate of a mixed read/write stream by about a tenth.
typedef unsigned basq_v4u __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 nt_load16(const void* p) {
    const basq_v4u v = __builtin_nontemporal_load(reinterpret_cast<const basq_v4u*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void nt_store16(void* p, uint4 x) {
    const basq_v4u v = {x.x, x.y, x.z, x.w};
    __builtin_nontemporal_store(v, reinterpret_cast<basq_v4u*>(p));
}

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// fp32 -> bf16 bits, round-half-to-even, NaN kept quiet.
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

}  // namespace basq
