// C-ABI layer of libbasq: argument validation, error text, dispatch.  No arithmetic here.
#include "basq_internal.h"

#include <stdarg.h>
#include <stdio.h>

#include <mutex>

namespace basq {

namespace {
thread_local char g_err[512] = "";
}

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int check_hip(hipError_t e, const char* what) {
    if (e == hipSuccess) return BASQ_OK;
    return fail(BASQ_EHIP, "%s: %s", what, hipGetErrorString(e));
}

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool is_pow2(int64_t v) { return v > 0 && (v & (v - 1)) == 0; }

// n = 2^t (t >= 1) or 28 * 2^t (t >= 1); fills the Sylvester factor and the H_28 flag.
bool split_rot_size(int32_t n, int32_t* pow2, int32_t* has28) {
    if (n < 2) return false;
    if (is_pow2(n)) { *pow2 = n; *has28 = 0; return true; }
    if (n % 28 == 0 && is_pow2(n / 28) && n / 28 >= 2) { *pow2 = n / 28; *has28 = 1; return true; }
    return false;
}

int validate_rotate(const void* X, int64_t M, int32_t K, int64_t ldx, int32_t rot_size, int32_t bits,
                    int32_t group_size, float clip_lo, float clip_hi, int32_t* pow2, int32_t* has28,
                    const float* bias = nullptr, const float* act_scale = nullptr) {
    if (M < 0) return fail(BASQ_EINVAL, "M must be >= 0 (got %lld)", (long long)M);
    if (K <= 0 || K % 32 != 0) return fail(BASQ_EINVAL, "K must be a positive multiple of 32 (got %d)", K);
    if (K > 32768) return fail(BASQ_EUNSUPPORTED, "K up to 32768 is supported (got %d)", K);
    if (ldx < K || ldx % 8 != 0) return fail(BASQ_EINVAL, "ldx must be >= K and a multiple of 8 (got %lld)", (long long)ldx);
    if (!split_rot_size(rot_size, pow2, has28))
        return fail(BASQ_EUNSUPPORTED, "rot_size must be 2^t or 28*2^t with t >= 1 (got %d)", rot_size);
    if (K % rot_size != 0) return fail(BASQ_EINVAL, "K (%d) must be a multiple of rot_size (%d)", K, rot_size);
    if (bits != 4) return fail(BASQ_EUNSUPPORTED, "only bits == 4 is implemented (got %d)", bits);
    if (group_size != 0 && (group_size < 32 || group_size % 32 != 0 || K % group_size != 0))
        return fail(BASQ_EINVAL, "group_size must be 0 or a multiple of 32 that divides K (got %d)", group_size);
    if (!(clip_lo > 0.0f) || !(clip_hi > 0.0f) || !(clip_lo <= 1.0f) || !(clip_hi <= 1.0f))
        return fail(BASQ_EINVAL, "clip ratios must be in (0, 1] (got %g, %g)", (double)clip_lo, (double)clip_hi);
    if (M > 0 && X == nullptr) return fail(BASQ_EINVAL, "X is null");
    if (!aligned16(X)) return fail(BASQ_EINVAL, "X must be 16-byte aligned");
    // the kernels read b^c and s^a four channels at a time
    if (!aligned16(bias) || !aligned16(act_scale)) return fail(BASQ_EINVAL, "bias and act_scale must be 16-byte aligned");
    return BASQ_OK;
}

int validate_gemm(const uint8_t* Aq, const basq_tokmeta* meta, int64_t M, int32_t K, const uint8_t* Wq, int32_t N,
                  int32_t w_layout, const void* w_scale, const void* w_zero, const float* w_sum, const void* Y,
                  int64_t ldy) {
    if (M < 0) return fail(BASQ_EINVAL, "M must be >= 0 (got %lld)", (long long)M);
    if (K <= 0 || K % 32 != 0) return fail(BASQ_EINVAL, "K must be a positive multiple of 32 (got %d)", K);
    if (N <= 0) return fail(BASQ_EINVAL, "N must be >= 1 (got %d)", N);
    if (w_layout != BASQ_W_CANONICAL && w_layout != BASQ_W_DECODE16)
        return fail(BASQ_EUNSUPPORTED, "unknown w_layout %d", w_layout);
    if (w_layout == BASQ_W_DECODE16 && K % 128 != 0)
        return fail(BASQ_EINVAL, "the streaming weight layout needs K %% 128 == 0 (got %d)", K);
    if (ldy < N) return fail(BASQ_EINVAL, "ldy must be >= N (got %lld)", (long long)ldy);
    if (!Wq || !w_scale || !w_zero || !w_sum) return fail(BASQ_EINVAL, "a weight-side pointer is null");
    if (M > 0 && (!Aq || !meta || !Y)) return fail(BASQ_EINVAL, "an activation-side pointer is null");
    if (!aligned16(Aq) || !aligned16(Wq) || !aligned16(meta))
        return fail(BASQ_EINVAL, "Aq, meta and Wq must be 16-byte aligned");
    if ((reinterpret_cast<uintptr_t>(Y) & 1u) != 0) return fail(BASQ_EINVAL, "Y must be 2-byte aligned");
    if ((int64_t)K * 225 > 0x7FFFFFFFll) return fail(BASQ_EUNSUPPORTED, "K too large for INT32 accumulation");
    return BASQ_OK;
}

int run_gemm(const GemmArgs& g, hipStream_t s) {
    if (g.M <= GEMV_MAX_TOKENS && g.K % 128 == 0) return launch_gemv_decode(g, s);
    if (gemm_fp6_applicable(g)) return launch_gemm_fp6(g, s);
    if (g.w_layout != BASQ_W_CANONICAL)
        return fail(BASQ_EUNSUPPORTED, "more than 128 tokens with the streaming weight layout need the fp6 operands "
                                        "(the int8 kernels read canonical weights)");
    return launch_gemm_prefill(g, s);
}

// the fp6 operand form is all-or-nothing on the GEMM side
int validate_fp6(const uint8_t* Aq6, const uint8_t* Wq6, bool need_a, int32_t K) {
    const int given = (Wq6 != nullptr) + (need_a ? (Aq6 != nullptr) : 0);
    const int all = need_a ? 2 : 1;
    if (given != 0 && given != all)
        return fail(BASQ_EINVAL, "the fp6 operands (activations and weights) must be given together or not at all");
    if (given && K % 128 != 0) return fail(BASQ_EINVAL, "the fp6 operand form needs K %% 128 == 0 (got %d)", K);
    if (!aligned16(Aq6) || !aligned16(Wq6)) return fail(BASQ_EINVAL, "fp6 operands must be 16-byte aligned");
    return BASQ_OK;
}

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// The kernels that write the fp6 form of the codes themselves can leave the 4-bit form out.
bool fp6_only_applicable(const RotateQuantArgs& a) {
    RotateQuantArgs b = a;
    b.Aq = nullptr;
    return b.Aq6 != nullptr && b.group == b.K && (rotate_quant_pow2_applicable(b) || rotate_quant_k28_applicable(b));
}

// the one-call layer on a workspace of the caller's or of the library's own (both entry points end here)
int linear_fused_impl(const void* X, int64_t M, int32_t K, int64_t ldx, int32_t rot_size, const float* bias,
                      const float* act_scale, float clip_lo, float clip_hi, int32_t bits, int32_t group_size,
                      const uint8_t* Wq, int32_t N, int32_t w_layout, const void* w_scale, const void* w_zero,
                      const float* w_sum, const float* out_bias, void* Y, int64_t ldy,
                      const uint8_t* Wq6, void* workspace,
                      size_t workspace_bytes, void* stream) {
    RotateQuantArgs a{};
    int rc = validate_rotate(X, M, K, ldx, rot_size, bits, group_size, clip_lo, clip_hi, &a.pow2, &a.has28, bias, act_scale);
    if (rc != BASQ_OK) return rc;
    if (group_size != 0 && group_size != K)
        return fail(BASQ_EUNSUPPORTED, "the GEMM takes per-token ranges only: group_size must be 0 or K (got %d)", group_size);
    rc = validate_fp6(nullptr, Wq6, false, K);
    if (rc != BASQ_OK) return rc;
    if (M == 0) {
        return validate_gemm(nullptr, nullptr, 0, K, Wq, N, w_layout, w_scale, w_zero, w_sum, Y, ldy);
    }
    if (!workspace) return fail(BASQ_EINVAL, "workspace is null");
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return fail(BASQ_EINVAL, "workspace must be 256-byte aligned");
    const size_t need = basq_workspace_bytes(M, K, N);
    if (workspace_bytes < need)
        return fail(BASQ_EWORKSPACE, "workspace too small: %zu bytes given, %zu needed", workspace_bytes, need);
    uint8_t* Aq = static_cast<uint8_t*>(workspace);
    basq_tokmeta* meta = reinterpret_cast<basq_tokmeta*>(Aq + align_up((size_t)M * (size_t)(K / 2), 256));
    rc = validate_gemm(Aq, meta, M, K, Wq, N, w_layout, w_scale, w_zero, w_sum, Y, ldy);
    if (rc != BASQ_OK) return rc;

    a.X = static_cast<const uint16_t*>(X);
    a.M = M; a.K = K; a.ldx = ldx; a.rot_size = rot_size;
    a.bias = bias; a.act_scale = act_scale; a.clip_lo = clip_lo; a.clip_hi = clip_hi;
    // the fp6 copy of the codes is only worth making when the matrix-core path will take it
    uint8_t* Aq6 = nullptr;
    if (Wq6 && M > GEMV_MAX_TOKENS)
        Aq6 = reinterpret_cast<uint8_t*>(meta) + align_up((size_t)M * sizeof(basq_tokmeta), 256);
    a.group = K;
    a.Aq = Aq; a.meta = meta; a.rot_out = nullptr; a.Aq6 = Aq6;
    hipStream_t s = static_cast<hipStream_t>(stream);
    GemmArgs g{Aq, meta, M, K, Wq, N, static_cast<const uint16_t*>(w_scale), static_cast<const uint16_t*>(w_zero),
               w_sum, out_bias, static_cast<uint16_t*>(Y), ldy, nullptr, Aq6, Aq6 ? Wq6 : nullptr, w_layout};
    // when the product runs on the fp6 matrix path nothing reads the 4-bit codes: where the quantiser writes the
    // fp6 form itself it leaves them out
    if (Aq6 && gemm_fp6_applicable(g) && fp6_only_applicable(a)) a.Aq = nullptr;
    if (w_layout != BASQ_W_CANONICAL && M > GEMV_MAX_TOKENS && !gemm_fp6_applicable(g))      // before anything is launched
        return fail(BASQ_EUNSUPPORTED, "more than 128 tokens with the streaming weight layout need the fp6 operands "
                                        "(the int8 kernels read canonical weights)");
    if (linear_decode_applicable(a, g)) return launch_linear_decode(a, g, s);      // a few tokens: one launch
    rc = launch_rotate_quant(a, s);
    if (rc != BASQ_OK) return rc;
    return run_gemm(g, s);
}


// ---- the library's own workspace, for callers that cannot allocate one -------------------------------------
// One copy per GPU, created when the code object is loaded there and held until the process ends.  In host code
// the array's name is only a handle for hipGetSymbolAddress; kernels get the address that call returns.
static __device__ __attribute__((used)) __align__(256) unsigned char scratch[BASQ_STATIC_WORKSPACE_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[MAX_DEVICES] = {};

// The current device's copy of `scratch`; looked up once per device, with that device current.
int static_workspace(unsigned char** out) {
    int dev = -1;
    int rc = check_hip(hipGetDevice(&dev), "hipGetDevice");
    if (rc != BASQ_OK) return rc;
    if (dev < 0 || dev >= MAX_DEVICES) return fail(BASQ_EUNSUPPORTED, "device ordinal %d is beyond the %d this table holds", dev, MAX_DEVICES);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        rc = check_hip(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)");
        if (rc != BASQ_OK) return rc;
        if (p == nullptr || (reinterpret_cast<uintptr_t>(p) & 255u) != 0)
            return fail(BASQ_EHIP, "the library's workspace came back null or misaligned (%p)", p);
        g_scratch_ptr[dev] = static_cast<unsigned char*>(p);
    }
    *out = g_scratch_ptr[dev];
    return BASQ_OK;
}

}  // namespace
}  // namespace basq

using namespace basq;

extern "C" {

int basq_version(void) { return 100; }

const char* basq_last_error(void) { return g_err; }

int basq_rotate_quant(const void* X, int64_t M, int32_t K, int64_t ldx, int32_t rot_size, const float* bias,
                      const float* act_scale, float clip_lo, float clip_hi, int32_t bits, int32_t group_size,
                      uint8_t* Aq, basq_tokmeta* meta, float* rot_out, uint8_t* Aq6, void* stream) {
    RotateQuantArgs a{};
    int rc = validate_rotate(X, M, K, ldx, rot_size, bits, group_size, clip_lo, clip_hi, &a.pow2, &a.has28, bias, act_scale);
    if (rc != BASQ_OK) return rc;
    if (M > 0 && (!(Aq || Aq6) || !meta)) return fail(BASQ_EINVAL, "Aq or meta is null");
    if (!aligned16(Aq) || !aligned16(meta) || !aligned16(rot_out) || !aligned16(Aq6))
        return fail(BASQ_EINVAL, "Aq, meta, rot_out and Aq6 must be 16-byte aligned");
    if (Aq6 && K % 128 != 0) return fail(BASQ_EINVAL, "the fp6 operand form needs K %% 128 == 0 (got %d)", K);
    a.X = static_cast<const uint16_t*>(X);
    a.M = M; a.K = K; a.ldx = ldx; a.rot_size = rot_size;
    a.bias = bias; a.act_scale = act_scale; a.clip_lo = clip_lo; a.clip_hi = clip_hi;
    a.group = group_size == 0 ? K : group_size;
    a.Aq = Aq; a.meta = meta; a.rot_out = rot_out; a.Aq6 = Aq6;
    if (M > 0 && !Aq && !fp6_only_applicable(a))
        return fail(BASQ_EUNSUPPORTED, "Aq may be NULL only where the quantiser writes the fp6 form itself: per-token ranges "
                                        "with rot_size == K in {4096, 8192, 14336}");
    return launch_rotate_quant(a, static_cast<hipStream_t>(stream));
}

int basq_w4a4_gemm(const uint8_t* Aq, const basq_tokmeta* meta, int64_t M, int32_t K, const uint8_t* Wq, int32_t N,
                   int32_t w_layout, const void* w_scale, const void* w_zero, const float* w_sum,
                   const float* out_bias, void* Y, int64_t ldy, int32_t* acc_out,
                   const uint8_t* Aq6, const uint8_t* Wq6, void* stream) {
    int rc = validate_gemm(Aq, meta, M, K, Wq, N, w_layout, w_scale, w_zero, w_sum, Y, ldy);
    if (rc != BASQ_OK) return rc;
    rc = validate_fp6(Aq6, Wq6, true, K);
    if (rc != BASQ_OK) return rc;
    GemmArgs g{Aq, meta, M, K, Wq, N, static_cast<const uint16_t*>(w_scale), static_cast<const uint16_t*>(w_zero),
               w_sum, out_bias, static_cast<uint16_t*>(Y), ldy, acc_out, Aq6, Wq6, w_layout};
    return run_gemm(g, static_cast<hipStream_t>(stream));
}

int basq_w4a4_gemm_grouped(const uint8_t* Aq, const basq_tokmeta* meta, int64_t M, int32_t K, int32_t group_size,
                           const uint8_t* Wq, int32_t N, const void* w_scale, const void* w_zero,
                           const int32_t* w_gsum, const float* out_bias, void* Y, int64_t ldy,
                           const uint8_t* Aq6, const uint8_t* Wq6, void* stream) {
    const float dummy = 0.0f;   // validate_gemm wants the per-token weight sums, which this formula does not use
    int rc = validate_gemm(Aq, meta, M, K, Wq, N, BASQ_W_CANONICAL, w_scale, w_zero, &dummy, Y, ldy);
    if (rc != BASQ_OK) return rc;
    if (group_size != 128) return fail(BASQ_EUNSUPPORTED, "group-wise GEMM: group_size must be 128 (got %d)", group_size);
    if (K % 128 != 0) return fail(BASQ_EINVAL, "group-wise GEMM: K must be a multiple of 128 (got %d)", K);
    if (!w_gsum) return fail(BASQ_EINVAL, "w_gsum is null");
    if ((reinterpret_cast<uintptr_t>(w_gsum) & 3u) != 0) return fail(BASQ_EINVAL, "w_gsum must be 4-byte aligned");
    rc = validate_fp6(Aq6, Wq6, true, K);
    if (rc != BASQ_OK) return rc;
    GemmArgs g{Aq, meta, M, K, Wq, N, static_cast<const uint16_t*>(w_scale), static_cast<const uint16_t*>(w_zero),
               nullptr, out_bias, static_cast<uint16_t*>(Y), ldy, nullptr, Aq6, Wq6, BASQ_W_CANONICAL};
    if (M > 0 && gemm_grouped_fp6_applicable(g)) return launch_gemm_grouped_fp6(g, w_gsum, static_cast<hipStream_t>(stream));
    if (M > 0 && !gemm_grouped_applicable(g)) return fail(BASQ_EUNSUPPORTED, "group-wise GEMM: an operand exceeds 4 GiB");
    return launch_gemm_grouped(g, w_gsum, static_cast<hipStream_t>(stream));
}

int basq_group_colsums(const uint8_t* Wq, int32_t N, int32_t K, int32_t group_size, int32_t* w_gsum, void* stream) {
    if (N <= 0) return fail(BASQ_EINVAL, "N must be >= 1 (got %d)", N);
    if (K <= 0 || K % 128 != 0) return fail(BASQ_EINVAL, "K must be a positive multiple of 128 (got %d)", K);
    if (group_size != 128) return fail(BASQ_EUNSUPPORTED, "group_size must be 128 (got %d)", group_size);
    if (!Wq || !w_gsum) return fail(BASQ_EINVAL, "a pointer is null");
    if (!aligned16(Wq)) return fail(BASQ_EINVAL, "Wq must be 16-byte aligned");
    return launch_group_colsums(Wq, N, K, w_gsum, static_cast<hipStream_t>(stream));
}

size_t basq_workspace_bytes(int64_t M, int32_t K, int32_t N) {
    (void)N;
    if (M < 0 || K <= 0) return 0;
    return align_up((size_t)M * (size_t)(K / 2), 256) + align_up((size_t)M * sizeof(basq_tokmeta), 256) +
           align_up(basq_fp6_bytes(M, K), 256);
}

size_t basq_fp6_bytes(int64_t rows, int32_t K) {
    if (rows < 0 || K <= 0 || K % 128 != 0) return 0;
    return (size_t)((rows + 31) / 32 * 32) * (size_t)(K / 4 * 3);      // whole 32-row blocks
}

int basq_pack_fp6(const uint8_t* codes, int64_t rows, int32_t K, uint8_t* out6, void* stream) {
    if (rows < 0) return fail(BASQ_EINVAL, "rows must be >= 0 (got %lld)", (long long)rows);
    if (K <= 0 || K % 128 != 0) return fail(BASQ_EINVAL, "the fp6 operand form needs K to be a positive multiple of 128 (got %d)", K);
    if (rows > 0 && (!codes || !out6)) return fail(BASQ_EINVAL, "codes or out6 is null");
    if (!aligned16(codes) || !aligned16(out6)) return fail(BASQ_EINVAL, "codes and out6 must be 16-byte aligned");
    return launch_pack_fp6(codes, rows, K, out6, static_cast<hipStream_t>(stream));
}

size_t basq_decode_bytes(int32_t N, int32_t K) {
    if (N <= 0 || K <= 0 || K % 128 != 0) return 0;
    return (size_t)((N + 15) / 16 * 16) * (size_t)(K / 2);
}

int basq_pack_decode(const uint8_t* Wq, int32_t N, int32_t K, uint8_t* out, void* stream) {
    if (N <= 0) return fail(BASQ_EINVAL, "N must be >= 1 (got %d)", N);
    if (K <= 0 || K % 128 != 0) return fail(BASQ_EINVAL, "the streaming weight layout needs K to be a positive multiple of 128 (got %d)", K);
    if (!Wq || !out) return fail(BASQ_EINVAL, "Wq or out is null");
    if (!aligned16(Wq) || !aligned16(out)) return fail(BASQ_EINVAL, "Wq and out must be 16-byte aligned");
    return launch_pack_decode16(Wq, N, K, out, static_cast<hipStream_t>(stream));
}

int basq_linear_fused(const void* X, int64_t M, int32_t K, int64_t ldx, int32_t rot_size, const float* bias,
                      const float* act_scale, float clip_lo, float clip_hi, int32_t bits, int32_t group_size,
                      const uint8_t* Wq, int32_t N, int32_t w_layout, const void* w_scale, const void* w_zero,
                      const float* w_sum, const float* out_bias, void* Y, int64_t ldy,
                      const uint8_t* Wq6, void* workspace,
                      size_t workspace_bytes, void* stream) {
    return linear_fused_impl(X, M, K, ldx, rot_size, bias, act_scale, clip_lo, clip_hi, bits, group_size, Wq, N, w_layout,
                             w_scale, w_zero, w_sum, out_bias, Y, ldy, Wq6, workspace, workspace_bytes, stream);
}

int basq_linear_fused_static(const void* X, int64_t M, int32_t K, int64_t ldx, int32_t rot_size, const float* bias,
                             const float* act_scale, float clip_lo, float clip_hi, int32_t bits, int32_t group_size,
                             const uint8_t* Wq, int32_t N, int32_t w_layout, const void* w_scale, const void* w_zero,
                             const float* w_sum, const float* out_bias, void* Y, int64_t ldy,
                             const uint8_t* Wq6, void* stream) {
    if (M < 0) return fail(BASQ_EINVAL, "M must be >= 0 (got %lld)", (long long)M);
    if (K <= 0 || K % 32 != 0) return fail(BASQ_EINVAL, "K must be a positive multiple of 32 (got %d)", K);
    const size_t need = basq_workspace_bytes(M, K, N);
    if (need > (size_t)BASQ_STATIC_WORKSPACE_BYTES)
        return fail(BASQ_EWORKSPACE, "M = %lld tokens of K = %d need %zu bytes of workspace; the library's own holds %zu "
                                     "(use basq_linear_fused with a workspace of the caller's)",
                    (long long)M, K, need, (size_t)BASQ_STATIC_WORKSPACE_BYTES);
    unsigned char* ws = nullptr;
    const int rc = static_workspace(&ws);
    if (rc != BASQ_OK) return rc;
    // every byte of the codes and records the product reads is written by the quantiser of the same call first,
    // so nothing of the previous call's contents has to be cleared
    return linear_fused_impl(X, M, K, ldx, rot_size, bias, act_scale, clip_lo, clip_hi, bits, group_size, Wq, N, w_layout,
                             w_scale, w_zero, w_sum, out_bias, Y, ldy, Wq6, ws, (size_t)BASQ_STATIC_WORKSPACE_BYTES, stream);
}

int basq_quantize_weights(const void* W_rot, int32_t N, int32_t K, int64_t ldw, uint8_t* Wq, void* w_scale,
                          void* w_zero, float* w_sum, void* stream) {
    if (N <= 0) return fail(BASQ_EINVAL, "N must be >= 1 (got %d)", N);
    if (K <= 0 || K % 32 != 0) return fail(BASQ_EINVAL, "K must be a positive multiple of 32 (got %d)", K);
    if (ldw < K) return fail(BASQ_EINVAL, "ldw must be >= K");
    if (!W_rot || !Wq || !w_scale || !w_zero || !w_sum) return fail(BASQ_EINVAL, "a pointer is null");
    return launch_quantize_weights(static_cast<const uint16_t*>(W_rot), N, K, ldw, Wq, static_cast<uint16_t*>(w_scale),
                                   static_cast<uint16_t*>(w_zero), w_sum, static_cast<hipStream_t>(stream));
}

int basq_fused_bias(const uint8_t* Wq, int32_t N, int32_t K, const void* w_scale, const void* w_zero,
                    const float* bias, const float* layer_bias, float* out_bias, void* stream) {
    if (N <= 0) return fail(BASQ_EINVAL, "N must be >= 1 (got %d)", N);
    if (K <= 0 || K % 32 != 0) return fail(BASQ_EINVAL, "K must be a positive multiple of 32 (got %d)", K);
    if (!Wq || !w_scale || !w_zero || !out_bias) return fail(BASQ_EINVAL, "a pointer is null");
    return launch_fused_bias(Wq, N, K, static_cast<const uint16_t*>(w_scale), static_cast<const uint16_t*>(w_zero),
                             bias, layer_bias, out_bias, nullptr, static_cast<hipStream_t>(stream));
}

int basq_prepare_weights(const uint8_t* Wq_canonical, int32_t N, int32_t K, const void* w_scale, const void* w_zero,
                         const float* bias, const float* layer_bias, float* w_sum, float* out_bias,
                         uint8_t* Wq_prepacked, void* stream) {
    if (N <= 0) return fail(BASQ_EINVAL, "N must be >= 1 (got %d)", N);
    if (K <= 0 || K % 32 != 0) return fail(BASQ_EINVAL, "K must be a positive multiple of 32 (got %d)", K);
    if (!Wq_canonical || !w_scale || !w_zero || !w_sum || !out_bias) return fail(BASQ_EINVAL, "a pointer is null");
    if (!aligned16(Wq_canonical) || !aligned16(Wq_prepacked))
        return fail(BASQ_EINVAL, "Wq_canonical and Wq_prepacked must be 16-byte aligned");
    if (Wq_prepacked && K % 128 != 0)
        return fail(BASQ_EINVAL, "the fp6 operand form needs K to be a multiple of 128 (got %d)", K);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int rc = launch_fused_bias(Wq_canonical, N, K, static_cast<const uint16_t*>(w_scale),
                                     static_cast<const uint16_t*>(w_zero), bias, layer_bias, out_bias, w_sum, s);
    if (rc != BASQ_OK || !Wq_prepacked) return rc;
    return launch_pack_fp6(Wq_canonical, N, K, Wq_prepacked, s);
}

int basq_calibrate_bias(const void* X, int64_t M, int32_t K, int64_t ldx, int32_t rot_size, const float* act_scale,
                        float* bias_out, void* workspace, size_t workspace_bytes, void* stream) {
    RotateQuantArgs a{};
    int rc = validate_rotate(X, M, K, ldx, rot_size, 4, 0, 1.0f, 1.0f, &a.pow2, &a.has28, nullptr, act_scale);
    if (rc != BASQ_OK) return rc;
    if (M < 1) return fail(BASQ_EINVAL, "calibration needs at least one token");
    if (!bias_out || !workspace) return fail(BASQ_EINVAL, "a pointer is null");
    if (!aligned16(workspace)) return fail(BASQ_EINVAL, "workspace must be 16-byte aligned");
    const size_t need = (size_t)M * (size_t)K * sizeof(float);
    if (workspace_bytes < need)
        return fail(BASQ_EWORKSPACE, "workspace too small: %zu bytes given, %zu needed", workspace_bytes, need);
    a.X = static_cast<const uint16_t*>(X);
    a.M = M; a.K = K; a.ldx = ldx; a.rot_size = rot_size;
    a.clip_lo = a.clip_hi = 1.0f;
    a.group = K;
    a.rot_out = static_cast<float*>(workspace);      // rotation-only mode: Aq/meta stay null
    hipStream_t s = static_cast<hipStream_t>(stream);
    rc = launch_rotate_quant(a, s);
    if (rc != BASQ_OK) return rc;
    return launch_column_mean(a.rot_out, M, K, act_scale, bias_out, s);
}

int basq_rotate_weights(const void* W, int32_t N, int32_t K, int64_t ldw, int32_t rot_size, void* W_rot,
                        void* workspace, size_t workspace_bytes, void* stream) {
    RotateQuantArgs a{};
    int rc = validate_rotate(W, N, K, ldw, rot_size, 4, 0, 1.0f, 1.0f, &a.pow2, &a.has28);
    if (rc != BASQ_OK) return rc;
    if (N < 1) return fail(BASQ_EINVAL, "N must be >= 1 (got %d)", N);
    if (!W_rot || !workspace) return fail(BASQ_EINVAL, "a pointer is null");
    if (!aligned16(workspace) || !aligned16(W_rot)) return fail(BASQ_EINVAL, "W_rot and workspace must be 16-byte aligned");
    const size_t need = (size_t)N * (size_t)K * sizeof(float);
    if (workspace_bytes < need)
        return fail(BASQ_EWORKSPACE, "workspace too small: %zu bytes given, %zu needed", workspace_bytes, need);
    a.X = static_cast<const uint16_t*>(W);
    a.M = N; a.K = K; a.ldx = ldw; a.rot_size = rot_size;
    a.clip_lo = a.clip_hi = 1.0f;
    a.group = K;
    a.rot_out = static_cast<float*>(workspace);      // rotation-only mode: Aq/meta stay null
    hipStream_t s = static_cast<hipStream_t>(stream);
    rc = launch_rotate_quant(a, s);
    if (rc != BASQ_OK) return rc;
    return launch_f32_to_bf16(a.rot_out, static_cast<uint16_t*>(W_rot), (int64_t)N * K, s);
}

int basq_hadamard28(int8_t* out_host) {
    if (!out_host) return fail(BASQ_EINVAL, "out_host is null");
    const int8_t* h = hadamard28_host();
    for (int i = 0; i < 28 * 28; ++i) out_host[i] = h[i];
    return BASQ_OK;
}

}  // extern "C"
