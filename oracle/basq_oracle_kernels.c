/*
 * CPU oracle for the W4A4 rotated linear layer -- the two steps that need either a fixed fp32
 * operation order or plain integer loops.  TEST INFRASTRUCTURE ONLY: this file is the checker the
 * GPU library is compared against; the product never calls it and it shares no code with the GPU
 * sources.  Compile with:  gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC
 * (-ffp-contract=off: every written operation is one IEEE-754 binary32 operation; the only fused
 * multiply-adds are the explicit fmaf calls.)
 *
 * Follows: uniform asymmetric quantiser with lower bound z and step s (paper Sec. 3.1, Eq. 4);
 * channel bias subtracted after the rotation (Sec. 4, Eq. 14); optional per-channel asymmetric
 * scale applied to the rotated activation (Sec. 4, Eq. 15); per-token dynamic range with clip
 * ratios ("Deployment Details", Sec. 5); INT4 x INT4 -> INT32 matrix product (Sec. 5.2).
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>

/*
 * Quantise rotated activations r[M,K] (fp32) group by group (group = G consecutive channels,
 * G == K is the per-token case the paper uses).
 *
 *   v_k   = r_k - b_k                         (no asymmetric scale; b absent => v_k = r_k)
 *   v_k   = fma(r_k, sa_k, -b_k)              (asymmetric scale sa given, Eq. 15)
 *   mn, mx = min_k v_k, max_k v_k             (NaN operands ignored, as fminf/fmaxf do)
 *   lo    = clip_lo * mn ;  hi = clip_hi * mx
 *   s     = (hi - lo) / L ,  L = 2^bits - 1 ;  s = 1 if s is not a positive finite number
 *   inv   = 1 / s ;  nlo = -(lo * inv)
 *   t_k   = fma(v_k, inv, nlo)                = (v_k - lo)/s of Eq. 4 with z = lo
 *   q_k   = rint(min(max(t_k, 0), L))         round-half-to-even; NaN -> 0
 *   rowsum = sum_k q_k
 *
 * Outputs: codes[M,K] one code per byte, scale[M,K/G], lo_out[M,K/G], rowsum[M,K/G].
 * Returns 0, or -1 on a bad argument.
 */
int orc_quantize_tokens(const float *r, int64_t M, int64_t K, int64_t G,
                        const float *bias, const float *act_scale,
                        float clip_lo, float clip_hi, int bits,
                        uint8_t *codes, float *scale, float *lo_out, int32_t *rowsum)
{
    if (!r || !codes || !scale || !lo_out || !rowsum) return -1;
    if (bits < 1 || bits > 8 || G <= 0 || K % G != 0) return -1;
    const float L = (float)((1 << bits) - 1);
    const int64_t ngroups = K / G;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t g = 0; g < ngroups; ++g) {
            const float *rr = r + m * K + g * G;
            const float *bb = bias ? bias + g * G : NULL;
            const float *ss = act_scale ? act_scale + g * G : NULL;
            uint8_t *qq = codes + m * K + g * G;
            float mn = INFINITY, mx = -INFINITY;
            for (int64_t k = 0; k < G; ++k) {
                float b = bb ? bb[k] : 0.0f;
                float v = ss ? fmaf(rr[k], ss[k], -b) : rr[k] - b;
                mn = fminf(mn, v);
                mx = fmaxf(mx, v);
            }
            float lo = clip_lo * mn;
            float hi = clip_hi * mx;
            float s = (hi - lo) / L;
            if (!(s > 0.0f && s < INFINITY)) s = 1.0f;
            float inv = 1.0f / s;
            float nlo = -(lo * inv);
            int32_t sum = 0;
            for (int64_t k = 0; k < G; ++k) {
                float b = bb ? bb[k] : 0.0f;
                float v = ss ? fmaf(rr[k], ss[k], -b) : rr[k] - b;
                float t = fmaf(v, inv, nlo);
                t = fminf(fmaxf(t, 0.0f), L);
                int32_t q = (int32_t)rintf(t);
                qq[k] = (uint8_t)q;
                sum += q;
            }
            scale[m * ngroups + g] = s;
            lo_out[m * ngroups + g] = lo;
            rowsum[m * ngroups + g] = sum;
        }
    }
    return 0;
}

/*
 * Integer matrix product of unsigned codes, both operands K-major:
 *   acc[m,n] = sum_k qa[m,k] * qw[n,k]          (int32; |acc| <= 255*255*K must fit)
 */
int orc_int_gemm(const uint8_t *qa, const uint8_t *qw, int64_t M, int64_t N, int64_t K, int32_t *acc)
{
    if (!qa || !qw || !acc) return -1;
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            const uint8_t *a = qa + m * K;
            const uint8_t *w = qw + n * K;
            int32_t s = 0;
            for (int64_t k = 0; k < K; ++k) s += (int32_t)a[k] * (int32_t)w[k];
            acc[m * N + n] = s;
        }
    }
    return 0;
}

/* Number of OpenMP threads the loops above use (reported next to timings). */
#ifdef _OPENMP
#include <omp.h>
int orc_num_threads(void) { return omp_get_max_threads(); }
#else
int orc_num_threads(void) { return 1; }
#endif
