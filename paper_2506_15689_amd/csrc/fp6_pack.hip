// INT4 codes -> the 6-bit floating-point operand form of the matrix core.
//
// A code q in 0..15 is stored as the e2m3 number q/8 (sign, 2 exponent bits, 3 mantissa bits).  Its bit
// pattern is q itself: below 8 the number is subnormal with mantissa q, from 8 on the exponent field is 1
// and the mantissa q - 8.  The f8f6f4 MFMA, twice as fast as the int8 one, then accumulates
// S = sum_k (qa/8)(qb/8) exactly in fp32 (multiples of 1/64 below 2^17 for K <= 32768), and the INT32
// accumulator of the paper's INT4 GEMM (Sec. 5.2) is 64*S.  (q/2 and q/4 are exact as well; q/8 keeps the
// two upper bits of every field zero, which the matrix cores reward with a few percent more throughput.)
//
// Layout: blocks of 3072 bytes, one per (chunk of 128 codes along K, block of 32 rows), chunk-major:
// block (c, rb) sits at ((c * ceil(rows/32)) + rb) * 3072.  It is the image the GEMM wants in LDS, so a
// stage of its ring is filled by plain contiguous copies and read without bank conflicts:
//   bytes [0, 2048)     row r (0..31), group f (codes 128c + 32f .. +31): the first 16 bytes of the
//                       group's 24-byte little-endian string of 6-bit fields, at 64r + 16*(f ^ ((r>>2)&3))
//   bytes [2048, 3072)  the last 8 bytes of that string, at 2048 + 256f + 8r
// Rows past the matrix inside the last block are never written; the GEMM discards what it computes from them.
#include "basq_internal.h"

namespace basq {

namespace {

// One workgroup per (block of 32 rows, pair of 128-code chunks): 256 threads convert one 32-code group each into the
// two blocks' LDS images, which then leave as contiguous 16-byte pieces (an 8-byte store is a request of its own to
// the L2 however it is aligned; written straight from the converting lanes, the tail pieces made four fifths of all
// write requests).  Rows past the matrix inside the last block are not written.
__global__ __launch_bounds__(256) void pack_fp6_kernel(const uint8_t* __restrict__ codes, int64_t rows, int32_t K,
                                                        uint8_t* __restrict__ out6) {
    __shared__ __attribute__((aligned(16))) uint8_t img[2][3072];
    const int tid = threadIdx.x;
    const int64_t rb = blockIdx.x, rb6 = (rows + 31) >> 5;
    const int nchunks = K / 128;
    const int cl = tid >> 7, r = (tid >> 2) & 31, f = tid & 3;
    const int c = 2 * (int)blockIdx.y + cl;
    const int64_t row = rb * 32 + r;
    if (c < nchunks && row < rows) {
        const uint4 in = *reinterpret_cast<const uint4*>(codes + row * (int64_t)(K / 2) + c * 64 + f * 16);
        const uint32_t w[4] = {in.x, in.y, in.z, in.w};
        uint32_t o[6] = {0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int e = 0; e < 32; ++e) {
            const uint32_t q = (w[e >> 3] >> (4 * (e & 7))) & 0xFu;      // the e2m3 pattern of q/8 is q itself
            const int bit = 6 * e;
            o[bit >> 5] |= q << (bit & 31);
            if ((bit & 31) > 26) o[(bit >> 5) + 1] |= q >> (32 - (bit & 31));
        }
        *reinterpret_cast<uint4*>(img[cl] + 64 * r + 16 * (f ^ ((r >> 2) & 3))) = make_uint4(o[0], o[1], o[2], o[3]);
        *reinterpret_cast<uint2*>(img[cl] + 2048 + 256 * f + 8 * r) = make_uint2(o[4], o[5]);
    }
    __syncthreads();
    const int64_t left = rows - rb * 32;
    const int valid = left < 32 ? (int)left : 32;                        // rows of this block inside the matrix
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int p = tid + 256 * k;                                     // 16-byte piece of the two images
        if (p >= 2 * 192) break;
        const int pc = p / 192, q = p % 192;
        const int cc = 2 * (int)blockIdx.y + pc;
        if (cc >= nchunks) continue;
        // pieces 0..127: row q/4 of the 16-byte parts; 128..191: rows 2t, 2t+1 (t = q%16) of the 8-byte tails
        const int first = q < 128 ? q >> 2 : 2 * (q & 15);
        if (first >= valid) continue;
        uint8_t* dst = out6 + ((int64_t)cc * rb6 + rb) * 3072 + q * 16;
        const uint4 v = *reinterpret_cast<const uint4*>(img[pc] + q * 16);
        if (q < 128 || first + 1 < valid) *reinterpret_cast<uint4*>(dst) = v;
        else *reinterpret_cast<uint2*>(dst) = make_uint2(v.x, v.y);
    }
}

}  // namespace

int launch_pack_fp6(const uint8_t* codes, int64_t rows, int32_t K, uint8_t* out6, hipStream_t s) {
    if (rows == 0) return BASQ_OK;
    const int64_t blocks = (rows + 31) / 32;
    if (blocks > 0x7FFFFFFFll) return fail(BASQ_EINVAL, "pack_fp6: too many rows for one launch");
    const unsigned pairs = (unsigned)((K / 128 + 1) / 2);
    if (pairs > 65535u) return fail(BASQ_EINVAL, "pack_fp6: K too large for one launch");
    hipLaunchKernelGGL(pack_fp6_kernel, dim3((unsigned)blocks, pairs), dim3(256), 0, s, codes, rows, K, out6);
    return check_hip(hipGetLastError(), "pack_fp6 launch");
}

}  // namespace basq
