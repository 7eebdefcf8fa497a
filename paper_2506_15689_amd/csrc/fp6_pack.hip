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

__global__ __launch_bounds__(256) void pack_fp6_kernel(const uint8_t* __restrict__ codes, int64_t rows, int32_t K,
                                                        uint8_t* __restrict__ out6) {
    // one wave per row: lane l converts groups l, l + 64, ...
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const uint8_t* src = codes + row * (int64_t)(K / 2);
    const int r = (int)(row & 31);
    uint8_t* dst = out6 + (row >> 5) * 3072;                       // this row's block of chunk 0
    const int64_t chunk_pitch = ((rows + 31) >> 5) * 3072;
    const int swz = (r >> 2) & 3;
    for (int g = lane; g < K / 32; g += 64) {
        const uint4 in = *reinterpret_cast<const uint4*>(src + g * 16);
        const uint32_t w[4] = {in.x, in.y, in.z, in.w};
        uint32_t o[6] = {0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int e = 0; e < 32; ++e) {
            const uint32_t q = (w[e >> 3] >> (4 * (e & 7))) & 0xFu;
            const uint32_t c = q;                                 // the e2m3 pattern of q/8
            const int bit = 6 * e;
            o[bit >> 5] |= c << (bit & 31);
            if ((bit & 31) > 26) o[(bit >> 5) + 1] |= c >> (32 - (bit & 31));
        }
        uint8_t* blk = dst + (g >> 2) * chunk_pitch;
        const int f = g & 3;
        *reinterpret_cast<uint4*>(blk + 64 * r + 16 * (f ^ swz)) = make_uint4(o[0], o[1], o[2], o[3]);
        *reinterpret_cast<uint2*>(blk + 2048 + 256 * f + 8 * r) = make_uint2(o[4], o[5]);
    }
}

}  // namespace

int launch_pack_fp6(const uint8_t* codes, int64_t rows, int32_t K, uint8_t* out6, hipStream_t s) {
    if (rows == 0) return BASQ_OK;
    const int64_t blocks = (rows + 3) / 4;
    if (blocks > 0x7FFFFFFFll) return fail(BASQ_EINVAL, "pack_fp6: too many rows for one launch");
    hipLaunchKernelGGL(pack_fp6_kernel, dim3((unsigned)blocks), dim3(256), 0, s, codes, rows, K, out6);
    return check_hip(hipGetLastError(), "pack_fp6 launch");
}

}  // namespace basq
