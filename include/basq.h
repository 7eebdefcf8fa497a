/*
 * basq.h -- C ABI of the MI355X (gfx950) W4A4 rotated linear layer of BASE-Q.
 *
 * The layer (paper Sec. 4, Eq. 14 and Eq. 15; row-vector form, R orthogonal, W' = W R given):
 *
 *     Y = Q_a( s^a (X R) - b^c ) . Q_w(W')^T + c ,      c = W_hat b^c + b   ("fused bias")
 *
 *   R      normalised Hadamard rotation applied online to each block of rot_size channels
 *          (Sec. 3.1: entries +-n^(-1/2); Sec. 4 "online rotations"), n = 2^t or 28 * 2^t
 *   Q_a    per-token asymmetric uniform quantiser with lower bound z and step s (Eq. 4; "per-token
 *          asymmetric dynamic quantization", Sec. 5), range [clip_lo*min, clip_hi*max]
 *   Q_w    per-output-channel asymmetric INT4 weights: W_hat[n,k] = sw[n] * (q_w[n,k] - zp[n])
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer owned by the caller unless its comment says "host".
 *     The library never frees caller memory; hot calls allocate nothing and never synchronise.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work of a call
 *     is enqueued on it in order.
 *   - bf16 tensors are passed as void* (16-bit storage, round-to-nearest-even on output).
 *   - Return value: BASQ_OK or a negative error code.  Arguments are validated on the host before
 *     anything is launched; a failing call launches nothing.  basq_last_error() gives the text of
 *     the calling thread's last error.
 *   - Packed INT4 ("canonical") layout: byte j of a row holds code k = 2j in its low nibble and
 *     code k = 2j+1 in its high nibble.
 *   - Alignment: X, Aq, meta, Wq, bias (b^c) and act_scale (s^a) base pointers 16-byte aligned (BASQ_EINVAL
 *     otherwise); K % 32 == 0; ldx % 8 == 0.  Y needs only its natural 2-byte alignment and any ldy >= N.
 */
#ifndef BASQ_H
#define BASQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BASQ_OK            0
#define BASQ_EINVAL       (-1)  /* null pointer, bad shape, stride or alignment */
#define BASQ_EUNSUPPORTED (-2)  /* valid request the library does not implement (bits != 4, ...) */
#define BASQ_EWORKSPACE   (-3)  /* workspace too small */
#define BASQ_EHIP         (-4)  /* a HIP call or launch failed */

#define BASQ_W_CANONICAL 0      /* Wq is [N, K/2] in the canonical packed layout */
#define BASQ_W_DECODE16  1      /* Wq is in the weight-streaming layout written by basq_pack_decode */

/* Per-token quantisation record written by basq_rotate_quant and read by basq_w4a4_gemm.
 * x_hat[m,k] = scale * q[m,k] + lo   (Eq. 4 with z = lo);  rowsum = sum_k q[m,k]. */
typedef struct {
    float   scale;
    float   lo;
    int32_t rowsum;
    int32_t reserved;
} basq_tokmeta;

/* Library version (major*10000 + minor*100 + patch). */
int basq_version(void);

/* Text of the calling thread's most recent error ("" if none).  Host pointer, valid until the
 * thread's next failing call. */
const char* basq_last_error(void);

/*
 * Online rotation + bias + per-token quantisation (Sec. 3.1 rotation; Eq. 14 bias; Eq. 15 scale;
 * Eq. 4 quantiser; Fig. 6 "fused quant kernel").  For each token m:
 *
 *     r      = X[m,:] . (H_n / sqrt(n))     blockwise over K/rot_size blocks, fp32
 *     v_k    = r_k - bias_k                 (act_scale == NULL)
 *     v_k    = fma(r_k, act_scale_k, -bias_k)
 *     lo     = clip_lo * min_k v_k ;  hi = clip_hi * max_k v_k
 *     s      = (hi - lo) / 15  (1 if not a positive finite number) ;  inv = 1/s ;  nlo = -(lo*inv)
 *     q_k    = rint(min(max(fma(v_k, inv, nlo), 0), 15))        round-half-to-even, NaN -> 0
 *
 *   X          bf16 [M, ldx], row m at X + m*ldx, ldx >= K
 *   rot_size   n; K % n == 0; n = 2^t (t >= 1) or 28 * 2^t (t >= 1).  For n = 28 * 2^t the matrix is
 *              H_28 (x) H_(2^t) with the Paley type-I H_28 over GF(27) (see basq_hadamard28) and
 *              channel index k = i * 2^t + j, i the H_28 index.
 *   bias       fp32 [K] b^c in the rotated basis, or NULL (= 0)
 *   act_scale  fp32 [K] s^a, or NULL (= 1)
 *   bits       must be 4 (else BASQ_EUNSUPPORTED)
 *   group_size 0 or K: one range and one record per token (what basq_w4a4_gemm consumes).  Otherwise a
 *              multiple of 32 that divides K: every run of group_size consecutive channels gets its own
 *              range, steps 4-6 above and the record apply per group (per-head quantisation of q, k and
 *              the KV cache with rot_size = group_size = head_dim; Sec. 5 "Deployment Details").  Such
 *              codes are not an input of basq_w4a4_gemm; with group_size = 128 they are the input of
 *              basq_w4a4_gemm_grouped.
 *   Aq         out, uint8 [M, K/2] canonical packed codes.  May be NULL when Aq6 is given, with per-token ranges and
 *              rot_size == K in {4096, 8192, 14336} (the quantiser writes the fp6 form itself and then leaves the
 *              4-bit form out; elsewhere BASQ_EUNSUPPORTED)
 *   meta       out, [M, K/group_size] records, token-major (group_size 0 counts as K)
 *   rot_out    out, optional debug dump of r, fp32 [M, K]; NULL to skip
 *   Aq6        out, optional (NULL to skip): the same codes in the fp6 operand form described at
 *              basq_pack_fp6 (basq_fp6_bytes(M, K) bytes), 16-byte aligned; needs K % 128 == 0.  With per-token
 *              ranges and rot_size == K in {4096, 8192, 14336} the quantiser writes it itself; otherwise (other
 *              sizes, group-wise ranges) a packing pass follows on the same stream.
 * M == 0 is valid and does nothing.
 */
int basq_rotate_quant(const void* X, int64_t M, int32_t K, int64_t ldx, int32_t rot_size,
                      const float* bias, const float* act_scale,
                      float clip_lo, float clip_hi, int32_t bits, int32_t group_size,
                      uint8_t* Aq, basq_tokmeta* meta, float* rot_out, uint8_t* Aq6, void* stream);

/*
 * INT4 x INT4 GEMM with INT32 accumulation and fused de-quantisation (Sec. 5.2; Fig. 6
 * "de-quantisation" with the bias folded in; Eq. 14 fused bias):
 *
 *     ACC[m,n] = sum_k q_a[m,k] * q_w[n,k]
 *     Y[m,n]   = bf16( s_m * sw_n * (ACC[m,n] - zp_n * rowsum_m) + lo_m * w_sum_n + out_bias_n )
 *
 *   Aq, meta   as written by basq_rotate_quant, [M, K/2] and [M]
 *   Wq         uint8 [N, K/2] with w_layout = BASQ_W_CANONICAL, or the weight-streaming layout of
 *              basq_pack_decode with w_layout = BASQ_W_DECODE16.  The latter is read by the M <= 128 path
 *              only: with M > 128 it needs the fp6 operands (which replace Wq), else BASQ_EUNSUPPORTED.
 *   w_scale    bf16 [N] sw;  w_zero  bf16 [N] zp in code units (any real value)
 *   w_sum      fp32 [N] = sw_n * (sum_k q_w[n,k] - K * zp_n) = sum_k W_hat[n,k]
 *   out_bias   fp32 [N] c, or NULL (= 0)
 *   Y          out, bf16 [M, ldy], ldy >= N
 *   acc_out    out, optional debug dump of ACC, int32 [M, N]; NULL to skip
 *   Aq6, Wq6   optional, both or neither: the two code matrices in the fp6 operand form
 *              (basq_pack_fp6; Aq6 also straight from basq_rotate_quant).  With them, and M > 128, the
 *              product runs on the f8f6f4 matrix-core path at twice the int8 rate; ACC and Y are
 *              bit-identical to the int8 path.  Needs K % 128 == 0.
 * Any M >= 0, N >= 1; M <= 128 (decode, batched decode) takes a weight-streaming path, same results.
 */
int basq_w4a4_gemm(const uint8_t* Aq, const basq_tokmeta* meta, int64_t M, int32_t K,
                   const uint8_t* Wq, int32_t N, int32_t w_layout,
                   const void* w_scale, const void* w_zero, const float* w_sum, const float* out_bias,
                   void* Y, int64_t ldy, int32_t* acc_out,
                   const uint8_t* Aq6, const uint8_t* Wq6, void* stream);

/*
 * The same product for activations quantised in groups of 128 channels (basq_rotate_quant with group_size = 128:
 * every group g of token m has its own step s_mg, lower bound z_mg and code sum rowsum_mg; Eq. 4 per group):
 *
 *     ACC_g[m,n] = sum over the channels k of group g of q_a[m,k] * q_w[n,k]
 *     Y[m,n]     = bf16( sw_n * ( sum_g ( s_mg ACC_g[m,n] + z_mg w_gsum[g,n] )
 *                                 - zp_n * sum_g ( s_mg rowsum_mg + 128 z_mg ) ) + out_bias_n )
 *
 * which is sum_k x_hat[m,k] W_hat[n,k] + out_bias_n.  The integer products are exact; the sums over groups are
 * fp32 multiply-adds in group order.
 *   Aq, meta   as written by basq_rotate_quant with group_size = 128: [M, K/2] and [M, K/128] records
 *   group_size must be 128 (else BASQ_EUNSUPPORTED); K % 128 == 0
 *   Wq         uint8 [N, K/2] canonical;  w_scale, w_zero bf16 [N];  out_bias fp32 [N] or NULL
 *   w_gsum     int32 [K/128, N], group-major: w_gsum[g*N + n] = sum of the codes of row n in group g
 *              (basq_group_colsums)
 *   Y          out, bf16 [M, ldy]
 *   Aq6, Wq6   optional, both or neither: the same codes in the fp6 operand form (basq_rotate_quant's Aq6 output or
 *              basq_pack_fp6; basq_fp6_bytes each).  With them the product runs on the f8f6f4 matrix cores, about
 *              1.5 times as fast, with bit-identical Y.
 */
int basq_w4a4_gemm_grouped(const uint8_t* Aq, const basq_tokmeta* meta, int64_t M, int32_t K, int32_t group_size,
                           const uint8_t* Wq, int32_t N, const void* w_scale, const void* w_zero,
                           const int32_t* w_gsum, const float* out_bias, void* Y, int64_t ldy,
                           const uint8_t* Aq6, const uint8_t* Wq6, void* stream);

/* Offline: the per-group sums of the weight codes, w_gsum int32 [K/128, N] (see basq_w4a4_gemm_grouped). */
int basq_group_colsums(const uint8_t* Wq, int32_t N, int32_t K, int32_t group_size, int32_t* w_gsum, void* stream);

/*
 * The fp6 operand form of an INT4 code matrix (device-side repacking; offline for weights).
 * The matrix cores of this GPU multiply 6-bit floating-point operands (e2m3: sign, 2 exponent bits,
 * 3 mantissa bits) at twice their int8 rate.  Code q in 0..15 is stored as the e2m3 number q/8, which
 * is exact; S = sum_k (qa/8)(qb/8) is exact in the fp32 accumulator for K <= 32768 (longer rows run on the
 * int8 path whatever operands are given), and the INT32 accumulator of the INT4 GEMM (Sec. 5.2) is 64*S.
 * (The e2m3 bit pattern of q/8 is q itself.)
 *
 *   codes      device uint8 [rows, K/2], two codes per byte, low nibble first (as Aq and Wq)
 *   out6       out, device uint8, basq_fp6_bytes(rows, K) bytes, 16-byte aligned.  Blocks of 3072
 *              bytes, one per (chunk c of 128 codes along K, block rb of 32 rows), chunk-major: block
 *              (c, rb) at (c*ceil(rows/32) + rb)*3072.  Row r of the block, group f = 0..3 (codes
 *              128c + 32f .. +31) is a 24-byte little-endian string of 6-bit fields; its first 16 bytes
 *              sit at 64r + 16*(f ^ ((r>>2)&3)), its last 8 bytes at 2048 + 256f + 8r.  (The block is
 *              the image the GEMM keeps in LDS.)  Rows past the matrix in the last block stay unwritten.
 * K % 128 == 0.  basq_fp6_bytes returns ceil(rows/32)*32 * 3K/4 (0 for an unsupported K).
 */
size_t basq_fp6_bytes(int64_t rows, int32_t K);
int basq_pack_fp6(const uint8_t* codes, int64_t rows, int32_t K, uint8_t* out6, void* stream);

/*
 * The weight-streaming layout for decode-sized calls (M <= 128; such a call is one pass over the weights and
 * bound by memory bandwidth, the decode case of Sec. 5.2's speed measurement).  The matrix-core operand of
 * that path puts 16 different rows on the 16 lanes of a quarter wavefront, so canonical weights are read in
 * 16-byte pieces of 16 rows at a time; here the kilobyte one wavefront load consumes is contiguous instead.
 *
 *   Wq         device uint8 [N, K/2] canonical
 *   out        out, device uint8, basq_decode_bytes(N, K) = ceil(N/16)*16 * K/2 bytes, 16-byte aligned.
 *              Block nb (rows 16nb .. 16nb+15) at nb*16*K/2; inside it chunk c (bytes 64c .. 64c+63 of each
 *              row) is the KB at c*1024; inside that, the 16-byte piece at (16*s + r)*16, s = 0..3,
 *              r = 0..15, holds bytes 64c + 16s .. +15 of row 16nb + r.  Rows past N are zeros.
 * K % 128 == 0.  basq_decode_bytes returns 0 for an unsupported shape.
 */
size_t basq_decode_bytes(int32_t N, int32_t K);
int basq_pack_decode(const uint8_t* Wq, int32_t N, int32_t K, uint8_t* out, void* stream);

/* Bytes of workspace basq_linear_fused needs for this shape (activation codes, token records, and
 * the fp6 copy of the codes). */
size_t basq_workspace_bytes(int64_t M, int32_t K, int32_t N);

/*
 * The whole layer in one call: basq_rotate_quant then basq_w4a4_gemm on `stream`, the codes and
 * token records living in `workspace` (256-byte aligned, >= basq_workspace_bytes(M, K, N), else
 * BASQ_EWORKSPACE).  Arguments as in the two calls above; with Wq6, M > 128 takes the fp6 matrix-core path.
 * group_size must be 0 or K here (BASQ_EUNSUPPORTED otherwise: groups go through basq_rotate_quant and
 * basq_w4a4_gemm_grouped).  With at most 4 tokens, rot_size == K in {4096, 8192}, N <= 4096 and
 * w_layout = BASQ_W_DECODE16 the whole layer is one kernel launch (same results bit for bit).  Nothing in this
 * call allocates or synchronises, so it may be recorded in a HIP graph.
 */
int basq_linear_fused(const void* X, int64_t M, int32_t K, int64_t ldx, int32_t rot_size,
                      const float* bias, const float* act_scale,
                      float clip_lo, float clip_hi, int32_t bits, int32_t group_size,
                      const uint8_t* Wq, int32_t N, int32_t w_layout,
                      const void* w_scale, const void* w_zero, const float* w_sum, const float* out_bias,
                      void* Y, int64_t ldy, const uint8_t* Wq6,
                      void* workspace, size_t workspace_bytes, void* stream);

/*
 * basq_linear_fused for callers that cannot allocate a workspace or keep one alive: code recorded under HIP graph
 * capture, tight serving loops, harnesses in which hipMalloc is forbidden.  Same arguments, same kernels and
 * bit-identical results; the codes and token records live in a workspace of BASQ_STATIC_WORKSPACE_BYTES that is
 * part of the library's code object (every GPU the library runs on holds its own copy until the process ends).
 *   - basq_workspace_bytes(M, K, N) > BASQ_STATIC_WORKSPACE_BYTES returns BASQ_EWORKSPACE and launches nothing
 *     (8 MiB hold e.g. 192 tokens of K = 32768, 800 of K = 8192, 1632 of K = 4096).
 *   - The call allocates nothing, frees nothing and does not synchronise.  Its first call on a device looks the
 *     workspace's address up (hipGetSymbolAddress, which may load the code object): make that call outside stream
 *     capture.
 *   - All calls on one GPU share that GPU's workspace, which keeps the previous call's contents (the quantiser
 *     writes every byte the product reads, so nothing needs clearing).  Calls that overlap on one GPU - different
 *     streams, or threads - race on it; calls on one stream, or otherwise ordered, do not.
 */
#define BASQ_STATIC_WORKSPACE_BYTES (8u << 20)
int basq_linear_fused_static(const void* X, int64_t M, int32_t K, int64_t ldx, int32_t rot_size,
                             const float* bias, const float* act_scale,
                             float clip_lo, float clip_hi, int32_t bits, int32_t group_size,
                             const uint8_t* Wq, int32_t N, int32_t w_layout,
                             const void* w_scale, const void* w_zero, const float* w_sum, const float* out_bias,
                             void* Y, int64_t ldy, const uint8_t* Wq6, void* stream);

/* ---- offline helpers (not on the timed path) --------------------------------------------- */

/*
 * Offline weight rotation W' = W R (Sec. 4: the rotation of the activations is undone by folding R into the
 * weights; Eq. 14 writes the layer as (W R)(R^-1 x)): every row of W is rotated blockwise by H_n/sqrt(n) exactly
 * as basq_rotate_quant rotates a token (fp32), then rounded to bf16.
 *   W          bf16 [N, ldw], ldw >= K, ldw % 8 == 0, 16-byte aligned;  rot_size as in basq_rotate_quant
 *   W_rot      out, bf16 [N, K], 16-byte aligned
 *   workspace  >= N*K*4 bytes (the fp32 rotation), 16-byte aligned, else BASQ_EWORKSPACE
 */
int basq_rotate_weights(const void* W, int32_t N, int32_t K, int64_t ldw, int32_t rot_size, void* W_rot,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * Round-to-nearest per-output-channel asymmetric INT4 quantisation of rotated-basis weights
 * (weights are quantised per channel, Sec. 5 "Deployment Details"; asymmetric with a bf16
 * zero-point per the workload definition).  Per row n, every operation one fp32 operation:
 *     lo, hi = min_k W', max_k W' ;  sw = bf16((hi - lo)/15)  (1 if not positive finite)
 *     zp = clamp(rint(-lo/sw), 0, 15) ;  q = clamp(rint(W'/sw) + zp, 0, 15)
 *     w_sum = fp32( double(sw) * (sum_k q - K*zp) )
 *   W_rot bf16 [N, ldw];  outputs Wq [N, K/2] canonical, w_scale bf16 [N], w_zero bf16 [N], w_sum fp32 [N].
 */
int basq_quantize_weights(const void* W_rot, int32_t N, int32_t K, int64_t ldw,
                          uint8_t* Wq, void* w_scale, void* w_zero, float* w_sum, void* stream);

/*
 * Fused bias of Eq. 14 from the dequantised weights:  out_bias[n] = sum_k W_hat[n,k] * bias[k]
 * + layer_bias[n], accumulated in fp64, stored fp32.  bias (b^c, fp32 [K]) and layer_bias
 * (fp32 [N]) may each be NULL (= 0).
 */
int basq_fused_bias(const uint8_t* Wq, int32_t N, int32_t K, const void* w_scale, const void* w_zero,
                    const float* bias, const float* layer_bias, float* out_bias, void* stream);

/*
 * Everything the hot calls need from already quantised weights, in one offline call (Eq. 14: the "fused bias"
 * W_hat b^c + b that undoes the channel bias after the product; and the weight sums that carry the activations'
 * lower bound through the product: with x_hat = s_m q_a + z_m and W_hat = sw_n (q_w - zp_n),
 * sum_k x_hat W_hat = s_m sw_n (ACC - zp_n rowsum_m) + z_m w_sum_n):
 *     w_sum[n]    = fp32( double(sw_n) * (sum_k q_w[n,k] - K * zp_n) )
 *     out_bias[n] = fp32( sum_k W_hat[n,k] * bias[k] + layer_bias[n] ),  accumulated in fp64
 *   Wq_canonical  uint8 [N, K/2], 16-byte aligned;  w_scale, w_zero bf16 [N]
 *   bias          fp32 [K] b^c in the rotated basis, or NULL (= 0);  layer_bias fp32 [N], or NULL (= 0)
 *   w_sum, out_bias   out, fp32 [N] each (the w_sum and out_bias arguments of the hot calls)
 *   Wq_prepacked  out, optional (NULL to skip): the weights in the fp6 operand form, basq_fp6_bytes(N, K) bytes,
 *                 16-byte aligned, K % 128 == 0 -- the Wq6 argument of the hot calls (see basq_pack_fp6)
 * Same results as basq_fused_bias and basq_pack_fp6, and the w_sum of basq_quantize_weights.
 */
int basq_prepare_weights(const uint8_t* Wq_canonical, int32_t N, int32_t K, const void* w_scale, const void* w_zero,
                         const float* bias, const float* layer_bias, float* w_sum, float* out_bias,
                         uint8_t* Wq_prepacked, void* stream);

/*
 * Channel bias calibration (Sec. 3.2: the bias cancels the per-channel means after rotation):
 *     bias_out[k] = mean_m ( s^a_k * r[m,k] ),  r the rotated calibration tokens; fp64 mean, fp32 out.
 * workspace: >= M*K*4 bytes (holds r), else BASQ_EWORKSPACE.
 */
int basq_calibrate_bias(const void* X, int64_t M, int32_t K, int64_t ldx, int32_t rot_size,
                        const float* act_scale, float* bias_out,
                        void* workspace, size_t workspace_bytes, void* stream);

/* The 28 x 28 matrix of +-1 used for rot_size = 28 * 2^t, row-major into a HOST buffer of 784
 * int8 (Paley type-I construction over GF(27) = GF(3)[t]/(t^3 + 2t + 1)). */
int basq_hadamard28(int8_t* out_host);

/* ---- diagnostics: what this machine sustains (used by the benchmark's measured ceilings) ---------- */

/*
 * Pure streaming kernel with the access pattern of basq_rotate_quant (the paper's fused quant kernel,
 * Fig. 6, is bandwidth bound): one wavefront per token reads 2K bytes from src + m*2K and writes K/2
 * bytes to dst + m*K/2 and 16 bytes to meta + m*16.  K a multiple of 2048.  Moves tokens*(2.5K+16) bytes.
 */
int basq_diag_stream(const void* src, void* dst, void* meta, int64_t tokens, int32_t K, void* stream);

/*
 * Read-only streaming kernel with the access pattern of the decode-sized product (M <= 128: one pass over the
 * weights, bound by memory bandwidth): `blocks` workgroups walk `bytes` (a multiple of 32768) of src in 32 KB
 * spans, every lane requesting eight 16-byte pieces before it consumes any; out receives blocks*256 uint32
 * checksums.
 */
int basq_diag_read(const void* src, int64_t bytes, uint32_t* out, int32_t blocks, void* stream);

/*
 * Register-resident int8 MFMA loop (Sec. 5.2: the prefill GEMM is compute bound): `blocks` workgroups of
 * 4 waves, each wave issues 8*iters v_mfma_i32_32x32x32_i8 on 4-bit valued operands; out receives
 * blocks*256 int32 checksums.  Executes blocks*4*8*iters*65536 integer operations.
 */
int basq_diag_mfma_i8(int32_t* out, int32_t blocks, int32_t iters, void* stream);

/*
 * The same loop on the f8f6f4 matrix-core path the prefill GEMM uses by default: each wave issues
 * 8*iters v_mfma_f32_32x32x64_f8f6f4 with fp6 (e2m3) operands in the value range of the 4-bit codes;
 * out receives blocks*256 fp32 checksums.  Executes blocks*4*8*iters*131072 operations.
 */
int basq_diag_mfma_f6(float* out, int32_t blocks, int32_t iters, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BASQ_H */
