// Group-wise asymmetric quantize-and-pack, Sec. 2.2 Eq. (2), for gfx950.
//
// One 16-lane segment of a wavefront owns one group of 128 consecutive k of
// one row: every lane loads 8 halves (one 128-bit load, fully coalesced: a
// wavefront reads 1 KiB = 4 groups), the segment reduces min/max with DPP
// row shifts, every lane then derives the same s and z and writes its 8 codes
// with one 32-bit (4-bit codes) or 64-bit (8-bit codes) store.
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

template <int BITS>
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

    const float qmax = (float)((1 << BITS) - 1);
    float s, z;
    if (hi == lo) { // all-zero group
        s = 1.0f;
        z = 0.0f;
    } else {
        s = __fdiv_rn(__fsub_rn(hi, lo), qmax);
        z = rintf(__fdiv_rn(-lo, s));
        z = fminf(fmaxf(z, 0.0f), qmax);
    }
    uint32_t q[8];
#pragma unroll
    for (int i = 0; i < 8; i++) {
        float t = rintf(__fadd_rn(__fdiv_rn(f[i], s), z));
        t = fminf(fmaxf(t, 0.0f), qmax);
        q[i] = (uint32_t)t;
    }
    if (BITS == 4) {
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

} // namespace

hipError_t fq_launch_quantize(const void *w, long long n_groups, int bits, void *codes,
                              void *scales, void *zeros, hipStream_t stream)
{
    const long long threads = n_groups * 16;
    const unsigned blocks = (unsigned)((threads + 255) / 256);
    if (blocks == 0)
        return hipSuccess;
    if (bits == 4)
        quantize_kernel<4><<<blocks, 256, 0, stream>>>((const half8 *)w, n_groups, (uint8_t *)codes,
                                                      (float *)scales, (uint8_t *)zeros);
    else
        quantize_kernel<8><<<blocks, 256, 0, stream>>>((const half8 *)w, n_groups, (uint8_t *)codes,
                                                      (float *)scales, (uint8_t *)zeros);
    return hipGetLastError();
}
