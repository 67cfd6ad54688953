// Prefill-shaped weight-only quantized linear: y[M][N] = x[M][K] . dequant(W[N][K])^T for
// M in the hundreds or thousands, where the weight stream is amortised over many tokens
// and the contraction is compute bound (Sec. 4.1) -- a dense GEMM on the matrix cores with
// the dequantization of Sec. 2.2 Eq. (3) fused into the operand path.
//
// Tiling.  A workgroup (4 wavefronts) owns a 128 (tokens) x 256 (weight rows) tile of y and
// walks K in steps of 64.  The wavefronts split the weight rows: each owns 64 rows x all
// 128 tokens = 4 x 2 tiles of v_mfma_f32_32x32x16_f16 (A = x: 32 tokens x 16 k, B =
// weights: 16 k x 32 rows; 128 binary32 accumulator registers).
//   - x goes through LDS: the 128 x 64 slab of a step is written once (double buffered,
//     one barrier per step) and every wavefront reads its A operands from it as 128-bit
//     vectors, 4 reads per 8 MFMAs.
//   - the weights never touch LDS: lane (n = lane % 32, c = lane / 32) loads 16 bytes of row
//     n straight from global memory in the MFMA's own operand layout, two steps ahead, and
//     dequantizes them in registers.  No other wavefront needs the same rows, so nothing
//     is unpacked twice.
//
// Dequantization.  Codes become the exact integers q - z as halves (same bit tricks as the
// decode kernels) and are multiplied by the group's scale rounded to half (one
// v_pk_mul_f16 per register): the MFMA operand is half((q - z) * half(s)).  The decode
// kernels keep the scale in binary32 outside the group sum; here that would need a second
// set of 128 accumulator registers per wavefront and a 384-instruction fold per group, so
// the prefill path rounds twice at 2^-11 relative instead.  The error stays well inside the
// 2e-3 bound (about 5e-4 of the output magnitude in the worst one-group case).
//
// Workgroups that share a weight slab (the M tiles of one N tile) get consecutive logical
// ids, and logical ids are dealt to the 8 XCDs in contiguous runs, so that a slab is
// fetched into one L2 and reused there.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fq_internal.h"

namespace {

#define FQ_GLOBAL __attribute__((address_space(1)))

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int THREADS = 256;
constexpr int BM = 128, BN = 256, BK = 64;
constexpr int WN = BN / 4;  // weight rows per wavefront (2 MFMA tiles)
constexpr int LDK = BK + 8; // halves per LDS row: 144 bytes, keeps 128-bit reads conflict-free
constexpr int XLD = BM * (BK / 8) / THREADS; // 16-byte pieces of the x slab per thread (4)

__device__ __forceinline__ uint4 load16(const void *p)
{
    const u32x4 v = *(const FQ_GLOBAL u32x4 *)p;
    return make_uint4(v.x, v.y, v.z, v.w);
}

// (a + b) * s, each operation rounded to half; a + b is the exact integer q - z
__device__ __forceinline__ uint32_t deq(uint32_t a, uint32_t b, half2_t s)
{
    return __builtin_bit_cast(uint32_t, (__builtin_bit_cast(half2_t, a) + __builtin_bit_cast(half2_t, b)) * s);
}

__device__ __forceinline__ float16_t mfma32(uint4 a, const uint32_t (&b)[4], float16_t c)
{
    const u32x4 av = {a.x, a.y, a.z, a.w};
    const u32x4 bv = {b[0], b[1], b[2], b[3]};
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, av),
                                                  __builtin_bit_cast(half8_t, bv), c, 0, 0, 0);
}

// Packed weights of one K step for one lane: per n-tile, 16-byte loads covering 64 k.
//   4-bit: 1 load (32 codes: k = 32 c ..), 8-bit: 2 loads (16 codes each: k = 32 h + 16 c ..),
//   fp16: 4 loads (8 halves each: k = 16 i + 8 c ..)
template <int BITS>
struct WRegs {
    static constexpr int NL = BITS == 4 ? 1 : (BITS == 8 ? 2 : 4);
    uint4 w[2][NL];
    float s[2];
    uint32_t z[2];
};

template <int BITS>
__device__ __forceinline__ void load_w(const FqLinearDesc &d, const uint8_t *codes, const float *scales,
                                       const uint8_t *zeros, int n_wave0, int k0, WRegs<BITS> &R)
{
    const int lane = threadIdx.x & 63, n = lane & 31, c = lane >> 5;
    const uint32_t K = (uint32_t)d.K;
#pragma unroll
    for (int j = 0; j < 2; j++) {
        const size_t row = (size_t)min(n_wave0 + j * 32 + n, d.N - 1);
        if (BITS == 4) {
            R.w[j][0] = load16(codes + row * (K >> 1) + ((k0 + 32 * c) >> 1));
        } else if (BITS == 8) {
#pragma unroll
            for (int h = 0; h < 2; h++)
                R.w[j][h] = load16(codes + row * K + k0 + 32 * h + 16 * c);
        } else {
#pragma unroll
            for (int i = 0; i < 4; i++)
                R.w[j][i] = load16(codes + (row * K + k0 + 16 * i + 8 * c) * 2);
        }
        if (BITS != 16) {
            R.s[j] = ((const FQ_GLOBAL float *)scales)[row * (K >> 7) + (k0 >> 7)];
            R.z[j] = ((const FQ_GLOBAL uint8_t *)zeros)[row * (K >> 7) + (k0 >> 7)];
        }
    }
}

// The B operand (8 halves) of k16-step i for n-tile j.  Which 8 k a lane supplies:
//   4-bit: k0 + 32 c + 8 i + (0 4 1 5 2 6 3 7)   8-bit: k0 + 32 (i/2) + 16 c + 8 (i%2) + 0..7
//   fp16:  k0 + 16 i + 8 c + 0..7
template <int BITS>
__device__ __forceinline__ void b_operand(const WRegs<BITS> &R, int j, int i, uint32_t (&b)[4])
{
    if (BITS == 4) {
        const uint32_t z = R.z[j];
        const uint32_t nz_lo = (z | (z << 16)) | 0xE400E400u;        // -(1024 + z) twice
        const uint32_t nz_hi = ((z << 4) | (z << 20)) | 0xD400D400u; // -(  64 + z) twice
        const half2_t sh = {(_Float16)R.s[j], (_Float16)R.s[j]};
        const uint32_t ww[4] = {R.w[j][0].x, R.w[j][0].y, R.w[j][0].z, R.w[j][0].w};
        const uint32_t v = ww[i], v8 = v >> 8;
        b[0] = deq((v & 0x000F000Fu) | 0x64006400u, nz_lo, sh);  // (q0 - z, q4 - z) * s
        b[1] = deq((v & 0x00F000F0u) | 0x54005400u, nz_hi, sh);  // (q1 - z, q5 - z) * s
        b[2] = deq((v8 & 0x000F000Fu) | 0x64006400u, nz_lo, sh); // (q2 - z, q6 - z) * s
        b[3] = deq((v8 & 0x00F000F0u) | 0x54005400u, nz_hi, sh); // (q3 - z, q7 - z) * s
    } else if (BITS == 8) {
        const uint32_t z = R.z[j];
        const uint32_t nz = (z | (z << 16)) | 0xE400E400u;
        const half2_t sh = {(_Float16)R.s[j], (_Float16)R.s[j]};
        const uint4 q = R.w[j][i >> 1];
        const uint32_t lo = (i & 1) ? q.z : q.x, hi = (i & 1) ? q.w : q.y;
        b[0] = deq(__builtin_amdgcn_perm(0x64646464u, lo, 0x04010400u), nz, sh);
        b[1] = deq(__builtin_amdgcn_perm(0x64646464u, lo, 0x04030402u), nz, sh);
        b[2] = deq(__builtin_amdgcn_perm(0x64646464u, hi, 0x04010400u), nz, sh);
        b[3] = deq(__builtin_amdgcn_perm(0x64646464u, hi, 0x04030402u), nz, sh);
    } else {
        b[0] = R.w[j][i].x;
        b[1] = R.w[j][i].y;
        b[2] = R.w[j][i].z;
        b[3] = R.w[j][i].w;
    }
}

// 16-byte block of x (8 halves, block index inside the 64-k step) that pairs with b_operand.
template <int BITS>
__device__ __forceinline__ int a_block(int i, int c)
{
    if (BITS == 4)
        return 4 * c + i;
    if (BITS == 8)
        return 4 * (i >> 1) + 2 * c + (i & 1);
    return 2 * i + c;
}

struct XRegs {
    uint4 x[XLD];
};

__device__ __forceinline__ void load_x(const FqLinearDesc &d, int M, int m0, int k0, XRegs &R)
{
#pragma unroll
    for (int i = 0; i < XLD; i++) {
        const int idx = i * THREADS + threadIdx.x, row = idx >> 3, piece = idx & 7;
        const int m = min(m0 + row, M - 1);
        R.x[i] = load16(d.x + (size_t)m * d.K + k0 + piece * 8);
    }
}

// 4-bit: the unpacking yields each block of 8 codes in the order (0 4 1 5 2 6 3 7); x is
// written in the same order so that the MFMA sums matching pairs.
template <int BITS>
__device__ __forceinline__ void store_x(const XRegs &R, uint16_t *xs)
{
#pragma unroll
    for (int i = 0; i < XLD; i++) {
        const int idx = i * THREADS + threadIdx.x, row = idx >> 3, piece = idx & 7;
        uint4 v = R.x[i];
        if (BITS == 4) {
            uint4 p;
            p.x = __builtin_amdgcn_perm(v.z, v.x, 0x05040100u); // (x0, x4)
            p.y = __builtin_amdgcn_perm(v.z, v.x, 0x07060302u); // (x1, x5)
            p.z = __builtin_amdgcn_perm(v.w, v.y, 0x05040100u); // (x2, x6)
            p.w = __builtin_amdgcn_perm(v.w, v.y, 0x07060302u); // (x3, x7)
            v = p;
        }
        *reinterpret_cast<uint4 *>(xs + row * LDK + piece * 8) = v;
    }
}

template <int BITS>
__global__ __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void prefill_kernel(const FqLinearDesc d, int M, int m_tiles,
                                                          int n_tiles, int per_xcd)
{
    __shared__ __attribute__((aligned(16))) uint16_t xs[2][BM * LDK];

    // hardware deals consecutive workgroup ids round-robin to the 8 XCDs: give each XCD a
    // contiguous run of logical tiles
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= m_tiles * n_tiles)
        return;
    const int m0 = (logical % m_tiles) * BM, n0 = (logical / m_tiles) * BN;

    const uint8_t *codes = BITS == 4 ? d.codes4 : BITS == 8 ? d.codes8 : (const uint8_t *)d.w16;
    const float *scales = BITS == 4 ? d.scales4 : d.scales8;
    const uint8_t *zeros = BITS == 4 ? d.zeros4 : d.zeros8;

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int l32 = lane & 31, c = lane >> 5;
    const int n_wave0 = n0 + wave * WN;

    float16_t acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
            for (int v = 0; v < 16; v++)
                acc[i][j][v] = 0.f;

    const int nsteps = d.K / BK;
    XRegs X;
    WRegs<BITS> W0, W1;
    load_x(d, M, m0, 0, X);
    load_w<BITS>(d, codes, scales, zeros, n_wave0, 0, W0);
    store_x<BITS>(X, xs[0]);
    load_x(d, M, m0, min(1, nsteps - 1) * BK, X);
    load_w<BITS>(d, codes, scales, zeros, n_wave0, min(1, nsteps - 1) * BK, W1);
    __syncthreads();

    // One step: MFMAs of step s from xs[s & 1] and Wcur; meanwhile x of step s+1 goes from
    // registers to the other LDS buffer, and the loads of step s+2 (x and weights) are issued.
    auto step = [&](int s, WRegs<BITS> &Wcur) {
        const uint16_t *xc = xs[s & 1];
        store_x<BITS>(X, xs[(s + 1) & 1]); // last read in step s-1: a barrier has passed since
        load_x(d, M, m0, min(s + 2, nsteps - 1) * BK, X);
#pragma unroll
        for (int i = 0; i < 4; i++) {
            uint4 a[4];
#pragma unroll
            for (int mt = 0; mt < 4; mt++)
                a[mt] = *reinterpret_cast<const uint4 *>(xc + (mt * 32 + l32) * LDK + a_block<BITS>(i, c) * 8);
#pragma unroll
            for (int j = 0; j < 2; j++) {
                uint32_t b[4];
                b_operand<BITS>(Wcur, j, i, b);
#pragma unroll
                for (int mt = 0; mt < 4; mt++)
                    acc[mt][j] = mfma32(a[mt], b, acc[mt][j]);
            }
        }
        // Wcur is free: refill it for step s+2 (always issued: keeps the waits counted)
        load_w<BITS>(d, codes, scales, zeros, n_wave0, min(s + 2, nsteps - 1) * BK, Wcur);
        __syncthreads(); // xs[(s+1)&1] complete, xs[s&1] no longer read
    };
    // K is a multiple of 128, so the number of steps is even: two steps per trip, straight
    // line, each with its own register set for the weights
    for (int s = 0; s < nsteps; s += 2) {
        step(s, W0);
        step(s + 1, W1);
    }
    // D layout of the 32x32 MFMA: lane holds column l32, rows 8 * (v / 4) + 4 * (lane / 32) + v % 4.
#pragma unroll
    for (int mt = 0; mt < 4; mt++)
#pragma unroll
        for (int j = 0; j < 2; j++) {
            const int n = n_wave0 + j * 32 + l32;
#pragma unroll
            for (int v = 0; v < 16; v++) {
                const int m = m0 + mt * 32 + 8 * (v >> 2) + 4 * c + (v & 3);
                if (m < M && n < d.N)
                    ((FQ_GLOBAL uint16_t *)d.y)[(size_t)m * d.N + n] =
                        __builtin_bit_cast(uint16_t, (_Float16)acc[mt][j][v]);
            }
        }
}

} // namespace

hipError_t fq_launch_prefill(const FqLinearDesc &d, int bits, int M, hipStream_t stream)
{
    const int m_tiles = (M + BM - 1) / BM, n_tiles = (d.N + BN - 1) / BN;
    const long long total = (long long)m_tiles * n_tiles;
    if (total > 0x3fffffffLL)
        return hipErrorInvalidValue;
    const int per_xcd = (int)((total + 7) / 8);
    const unsigned grid = (unsigned)per_xcd * 8;
    if (bits == 4)
        prefill_kernel<4><<<grid, THREADS, 0, stream>>>(d, M, m_tiles, n_tiles, per_xcd);
    else if (bits == 8)
        prefill_kernel<8><<<grid, THREADS, 0, stream>>>(d, M, m_tiles, n_tiles, per_xcd);
    else
        prefill_kernel<16><<<grid, THREADS, 0, stream>>>(d, M, m_tiles, n_tiles, per_xcd);
    return hipGetLastError();
}
