// Group-wise quantize-and-pack, Sec. 2.2 Eq. (2), for gfx950: the asymmetric form, the symmetric
// variant stated after Eq. (3), and quantize-dequantize to fp16 at 2..8 bits (Sec. 5.1).
//
// One 16-lane segment of a wavefront owns one group of 128 consecutive k of
// one row: every lane loads 8 halves (one 128-bit load, fully coalesced: a
// wavefront reads 1 KiB = 4 groups), the segment reduces min/max with DPP
// row shifts, every lane then derives the same s and z and writes its 8 codes
// with one 16-bit (2-bit codes), 32-bit (4-bit codes) or 64-bit (8-bit codes) store (3-bit
// codes: four lanes put a block of three words together).
//
// The arithmetic is pinned so that codes, scales and zeros are bit-exact
// against a binary32 evaluation with one rounding per operation: IEEE
// division, no fused multiply-add, round-half-to-even.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fq_internal.h"

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));

// min/max over the 16 lanes of a DPP row (lanes 16j .. 16j+15), result in all 16.
__device__ __forceinline__ float seg16_min(float v)
{
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1)
        v = fminf(v, __shfl_xor(v, off, 64));
    return v;
}
__device__ __forceinline__ float seg16_max(float v)
{
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1)
        v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

// Scale, zero point and code limits of a group from its range (every lane of the segment
// computes the same).  Asymmetric: the range always contains 0.  Symmetric: max |w| on the last of
// 2^(bits-1) - 1 levels either side; codes are stored offset by 2^(bits-1), which is also the
// stored zero point, so that Eq. (3) applies unchanged.
struct GroupParams {
    float s, z, qlo, qhi;
};
template <bool SYM>
__device__ __forceinline__ GroupParams group_params(float lo, float hi, int bits)
{
#pragma clang fp contract(off)
    GroupParams p;
    if (SYM) {
        const float amax = fmaxf(-lo, hi);
        const float lim = (float)((1 << (bits - 1)) - 1);
        p.s = amax == 0.0f ? 1.0f : __fdiv_rn(__fadd_rn(amax, amax), (float)((1 << bits) - 2));
        p.z = 0.0f;
        p.qlo = -lim;
        p.qhi = lim;
    } else {
        const float qmax = (float)((1 << bits) - 1);
        if (hi == lo) { // all-zero group
            p.s = 1.0f;
            p.z = 0.0f;
        } else {
            p.s = __fdiv_rn(__fsub_rn(hi, lo), qmax);
            p.z = fminf(fmaxf(rintf(__fdiv_rn(-lo, p.s)), 0.0f), qmax);
        }
        p.qlo = 0.0f;
        p.qhi = qmax;
    }
    return p;
}

template <int BITS, bool SYM>
__global__ __launch_bounds__(256) void quantize_kernel(const half8 *__restrict__ w,
                                                       long long n_groups, // N * K / 128
                                                       uint8_t *__restrict__ codes,
                                                       float *__restrict__ scales,
                                                       uint8_t *__restrict__ zeros)
{
#pragma clang fp contract(off)
    const long long seg = ((long long)blockIdx.x * 256 + threadIdx.x) >> 4; // group index
    const int sub = threadIdx.x & 15;
    // Whole 16-lane segments are in or out together, so the shuffles below never
    // read an inactive lane of their own segment.
    if (seg >= n_groups)
        return;
    const half8 v = w[seg * 16 + sub];
    float f[8];
    float lo = 0.0f, hi = 0.0f; // the range always contains 0
#pragma unroll
    for (int i = 0; i < 8; i++) {
        f[i] = (float)v[i];
        lo = fminf(lo, f[i]);
        hi = fmaxf(hi, f[i]);
    }
    lo = seg16_min(lo);
    hi = seg16_max(hi);

    const GroupParams p = group_params<SYM>(lo, hi, BITS);
    const float s = p.s;
    const float z = SYM ? (float)(1 << (BITS - 1)) : p.z; // what is stored
    uint32_t q[8];
#pragma unroll
    for (int i = 0; i < 8; i++) {
        float t = rintf(__fadd_rn(__fdiv_rn(f[i], s), p.z));
        t = fminf(fmaxf(t, p.qlo), p.qhi);
        q[i] = (uint32_t)(int)(SYM ? t + z : t);
    }
    if (BITS == 2) {
        uint32_t word = 0;
#pragma unroll
        for (int i = 0; i < 8; i++)
            word |= q[i] << (2 * i); // byte j = code(4j) | code(4j+1) << 2 | code(4j+2) << 4 | code(4j+3) << 6
        reinterpret_cast<uint16_t *>(codes)[seg * 16 + sub] = (uint16_t)word;
    } else if (BITS == 3) {
        // A block of 12 bytes = three words holds 32 codes: word j the codes 10 j .. 10 j + 9 whole
        // (code 10 j + 5 h + p in bits 16 h + 3 p .. + 2), the words' bits 15 and 31 the three bits
        // of codes 30 and 31.  The four lanes of a block place their eight codes each, the words
        // are OR-ed across the four, and lane t < 3 stores word t.
        const int t = sub & 3;
        uint32_t c[3] = {0u, 0u, 0u};
#pragma unroll
        for (int e = 0; e < 8; e++) {
            const int i = 8 * t + e;
            if (i < 30) {
                const int j = i / 10, r = i - 10 * j;
                const uint32_t v = q[e] << (r >= 5 ? 16 + 3 * (r - 5) : 3 * r);
#pragma unroll
                for (int jj = 0; jj < 3; jj++)
                    c[jj] |= j == jj ? v : 0u;
            } else {
                const int sh = 15 + 16 * (i - 30);
#pragma unroll
                for (int jj = 0; jj < 3; jj++)
                    c[jj] |= ((q[e] >> jj) & 1u) << sh;
            }
        }
#pragma unroll
        for (int jj = 0; jj < 3; jj++) {
            c[jj] |= (uint32_t)__shfl_xor((int)c[jj], 1, 64);
            c[jj] |= (uint32_t)__shfl_xor((int)c[jj], 2, 64);
        }
        if (t < 3)
            reinterpret_cast<uint32_t *>(codes)[(seg * 4 + (sub >> 2)) * 3 + t] = t == 0 ? c[0] : t == 1 ? c[1] : c[2];
    } else if (BITS == 4) {
        uint32_t word = 0;
#pragma unroll
        for (int i = 0; i < 8; i++)
            word |= q[i] << (4 * i); // code k in nibble k: byte j = code(2j) | code(2j+1) << 4
        reinterpret_cast<uint32_t *>(codes)[seg * 16 + sub] = word;
    } else {
        uint2 word;
        word.x = q[0] | (q[1] << 8) | (q[2] << 16) | (q[3] << 24);
        word.y = q[4] | (q[5] << 8) | (q[6] << 16) | (q[7] << 24);
        reinterpret_cast<uint2 *>(codes)[seg * 16 + sub] = word;
    }
    if (sub == 0) {
        scales[seg] = s;
        zeros[seg] = (uint8_t)z;
    }
}

// Eq. (2) then Eq. (3), rounded to fp16: w_hat = half(s * (q - z)).
template <bool SYM>
// (w_hat may be w itself: no __restrict__; a lane reads its eight weights before it writes them)
__global__ __launch_bounds__(256) void fake_quantize_kernel(const half8 *w, long long n_groups, int bits,
                                                            half8 *w_hat)
{
#pragma clang fp contract(off)
    const long long seg = ((long long)blockIdx.x * 256 + threadIdx.x) >> 4;
    const int sub = threadIdx.x & 15;
    if (seg >= n_groups)
        return;
    const half8 v = w[seg * 16 + sub];
    float f[8];
    float lo = 0.0f, hi = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; i++) {
        f[i] = (float)v[i];
        lo = fminf(lo, f[i]);
        hi = fmaxf(hi, f[i]);
    }
    lo = seg16_min(lo);
    hi = seg16_max(hi);
    const GroupParams p = group_params<SYM>(lo, hi, bits);
    half8 out;
#pragma unroll
    for (int i = 0; i < 8; i++) {
        float t = rintf(__fadd_rn(__fdiv_rn(f[i], p.s), p.z));
        t = fminf(fmaxf(t, p.qlo), p.qhi);
        const float code = (float)(int)t; // the stored code is an integer: -0 becomes 0
        float d = __fmul_rn(__fsub_rn(code, p.z), p.s);
        // two roundings, binary32 then binary16, as Eq. (3) in binary32 followed by a store to
        // fp16: kept apart from the conversion, which the compiler otherwise fuses with the
        // product into one mixed-precision instruction with a single rounding
        asm volatile("" : "+v"(d));
        out[i] = (_Float16)d;
    }
    w_hat[seg * 16 + sub] = out;
}

// One scale and zero point per weight row (group = K) at 8 bits: the granularity at which the INT8 copy
// meets 8-bit activations on the integer matrix cores without a fold per group (Sec. 4.1, 4.3).  Eq. (2)
// as above with Xmin / Xmax taken over the whole row.  One workgroup per row, two passes over it (the
// second finds it in cache).
template <bool SYM>
__global__ __launch_bounds__(256) void quantize_row8_kernel(const half8 *__restrict__ w, int K,
                                                            uint8_t *__restrict__ codes, float *__restrict__ scales,
                                                            uint8_t *__restrict__ zeros)
{
#pragma clang fp contract(off)
    __shared__ float s_lo[4], s_hi[4];
    const int t = threadIdx.x, nvec = K >> 3;
    const half8 *row = w + (size_t)blockIdx.x * nvec;
    float lo = 0.0f, hi = 0.0f; // the range always contains 0
    for (int i = t; i < nvec; i += 256) {
        const half8 v = row[i];
#pragma unroll
        for (int j = 0; j < 8; j++) {
            lo = fminf(lo, (float)v[j]);
            hi = fmaxf(hi, (float)v[j]);
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        lo = fminf(lo, __shfl_xor(lo, off, 64));
        hi = fmaxf(hi, __shfl_xor(hi, off, 64));
    }
    if ((t & 63) == 0) {
        s_lo[t >> 6] = lo;
        s_hi[t >> 6] = hi;
    }
    __syncthreads();
    lo = fminf(fminf(s_lo[0], s_lo[1]), fminf(s_lo[2], s_lo[3]));
    hi = fmaxf(fmaxf(s_hi[0], s_hi[1]), fmaxf(s_hi[2], s_hi[3]));
    const GroupParams p = group_params<SYM>(lo, hi, 8);
    const float z = SYM ? 128.0f : p.z; // what is stored
    for (int i = t; i < nvec; i += 256) {
        const half8 v = row[i];
        uint32_t q[8];
#pragma unroll
        for (int j = 0; j < 8; j++) {
            float c = rintf(__fadd_rn(__fdiv_rn((float)v[j], p.s), p.z));
            c = fminf(fmaxf(c, p.qlo), p.qhi);
            q[j] = (uint32_t)(int)(SYM ? c + z : c);
        }
        uint2 word;
        word.x = q[0] | (q[1] << 8) | (q[2] << 16) | (q[3] << 24);
        word.y = q[4] | (q[5] << 8) | (q[6] << 16) | (q[7] << 24);
        reinterpret_cast<uint2 *>(codes + (size_t)blockIdx.x * K)[i] = word;
    }
    if (t == 0) {
        scales[blockIdx.x] = p.s;
        zeros[blockIdx.x] = (uint8_t)(int)z;
    }
}

} // namespace

hipError_t fq_launch_quantize(const void *w, long long n_groups, int bits, bool symmetric, void *codes,
                              void *scales, void *zeros, hipStream_t stream)
{
    const long long threads = n_groups * 16;
    const unsigned blocks = (unsigned)((threads + 255) / 256);
    if (blocks == 0)
        return hipSuccess;
    const half8 *wp = (const half8 *)w;
    uint8_t *cp = (uint8_t *)codes, *zp = (uint8_t *)zeros;
    float *sp = (float *)scales;
    if (bits == 2 && !symmetric)
        quantize_kernel<2, false><<<blocks, 256, 0, stream>>>(wp, n_groups, cp, sp, zp);
    else if (bits == 2)
        quantize_kernel<2, true><<<blocks, 256, 0, stream>>>(wp, n_groups, cp, sp, zp);
    else if (bits == 3 && !symmetric)
        quantize_kernel<3, false><<<blocks, 256, 0, stream>>>(wp, n_groups, cp, sp, zp);
    else if (bits == 3)
        quantize_kernel<3, true><<<blocks, 256, 0, stream>>>(wp, n_groups, cp, sp, zp);
    else if (bits == 4 && !symmetric)
        quantize_kernel<4, false><<<blocks, 256, 0, stream>>>(wp, n_groups, cp, sp, zp);
    else if (bits == 4)
        quantize_kernel<4, true><<<blocks, 256, 0, stream>>>(wp, n_groups, cp, sp, zp);
    else if (!symmetric)
        quantize_kernel<8, false><<<blocks, 256, 0, stream>>>(wp, n_groups, cp, sp, zp);
    else
        quantize_kernel<8, true><<<blocks, 256, 0, stream>>>(wp, n_groups, cp, sp, zp);
    return hipGetLastError();
}

hipError_t fq_launch_fake_quantize(const void *w, long long n_groups, int bits, bool symmetric, void *w_hat,
                                   hipStream_t stream)
{
    const long long threads = n_groups * 16;
    const unsigned blocks = (unsigned)((threads + 255) / 256);
    if (blocks == 0)
        return hipSuccess;
    if (symmetric)
        fake_quantize_kernel<true><<<blocks, 256, 0, stream>>>((const half8 *)w, n_groups, bits, (half8 *)w_hat);
    else
        fake_quantize_kernel<false><<<blocks, 256, 0, stream>>>((const half8 *)w, n_groups, bits, (half8 *)w_hat);
    return hipGetLastError();
}

hipError_t fq_launch_quantize_row8(const void *w, int N, int K, bool symmetric, void *codes, void *scales, void *zeros,
                                   hipStream_t stream)
{
    if (N <= 0)
        return hipSuccess;
    if (symmetric)
        quantize_row8_kernel<true><<<N, 256, 0, stream>>>((const half8 *)w, K, (uint8_t *)codes, (float *)scales, (uint8_t *)zeros);
    else
        quantize_row8_kernel<false><<<N, 256, 0, stream>>>((const half8 *)w, K, (uint8_t *)codes, (float *)scales, (uint8_t *)zeros);
    return hipGetLastError();
}
