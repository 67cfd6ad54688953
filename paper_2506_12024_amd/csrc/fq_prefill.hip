// Prefill-shaped weight-only quantized linear: y[M][N] = x[M][K] . dequant(W[N][K])^T for
// M in the hundreds or thousands, where the weight stream is amortised over many tokens
// and the contraction is compute bound (Sec. 4.1) -- a dense GEMM on the matrix cores with
// the dequantization of Sec. 2.2 Eq. (3) fused into the operand path.
//
// Tiling.  A workgroup (4 wavefronts, 2 x 2) owns a 128 (tokens) x 128 (weight rows) tile
// of y and walks K in steps of 64; each wavefront owns 64 x 64 = 2 x 2 MFMA tiles of
// v_mfma_f32_32x32x16_f16 (A = x: 32 tokens x 16 k, B = weights: 16 k x 32 rows, binary32
// accumulators).  Per step the workgroup brings in a 128 x 64 slab of x (halves) and the
// matching 128 x 64 slab of packed weights; the weights are unpacked in registers to the
// exact integers q - z as halves (same bit tricks as the decode kernels) and both slabs are
// written to LDS, from where the MFMA operands are read as 128-bit vectors.  The global
// loads of step i+1 are issued before the MFMAs of step i (register prefetch).
//
// Scale.  The products of one quantization group (two steps) are summed in a zeroed
// accumulator; at the end of the group every lane, which owns one weight row per MFMA
// tile, folds it into the running output as out += s[n][g] * acc.  This is Eq. (3) with the
// scale factored out of the group, in binary32, exactly as the decode kernels do.
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
constexpr int BM = 128, BN = 128, BK = 64;
constexpr int LDK = BK + 8; // halves per LDS row: 144 bytes, keeps 128-bit reads conflict-free

__device__ __forceinline__ uint4 load16(const void *p)
{
    const u32x4 v = *(const FQ_GLOBAL u32x4 *)p;
    return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ uint32_t pk_add(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2_t, a) + __builtin_bit_cast(half2_t, b));
}

__device__ __forceinline__ float16_t mfma32(uint4 a, uint4 b, float16_t c)
{
    const u32x4 av = {a.x, a.y, a.z, a.w};
    const u32x4 bv = {b.x, b.y, b.z, b.w};
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, av),
                                                  __builtin_bit_cast(half8_t, bv), c, 0, 0, 0);
}

// Per-thread share of one K step.
//   x slab: 128 rows x 64 halves = 1024 pieces of 16 bytes, 4 per thread
//   w slab: 4-bit 128 x 32 bytes = 256 pieces (1 per thread); 8-bit 512 (2); fp16 1024 (4)
template <int BITS>
struct Regs {
    uint4 x[4];
    uint4 w[BITS == 4 ? 1 : (BITS == 8 ? 2 : 4)];
    uint32_t z;
};

template <int BITS>
__device__ __forceinline__ void load_step(const FqLinearDesc &d, const uint8_t *codes,
                                          const uint8_t *zeros, int M, int m0, int n0, int k0,
                                          Regs<BITS> &R)
{
    const int t = threadIdx.x;
    const int K = d.K;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const int idx = i * THREADS + t, row = idx >> 3, piece = idx & 7;
        const int m = min(m0 + row, M - 1);
        R.x[i] = load16(d.x + (size_t)m * K + k0 + piece * 8);
    }
    if (BITS == 4) {
        const int row = t >> 1, piece = t & 1; // 32 codes = 16 bytes each
        const int n = min(n0 + row, d.N - 1);
        R.w[0] = load16(codes + (size_t)n * (K >> 1) + (k0 >> 1) + piece * 16);
        R.z = ((const FQ_GLOBAL uint8_t *)zeros)[(size_t)n * (K >> 7) + (k0 >> 7)];
    } else if (BITS == 8) {
        const int row = t >> 1, half = t & 1; // two pieces of 16 codes each
        const int n = min(n0 + row, d.N - 1);
#pragma unroll
        for (int i = 0; i < 2; i++)
            R.w[i] = load16(codes + (size_t)n * K + k0 + half * 32 + i * 16);
        R.z = ((const FQ_GLOBAL uint8_t *)zeros)[(size_t)n * (K >> 7) + (k0 >> 7)];
    } else {
        const int row = t >> 1, half = t & 1; // four pieces of 8 halves each
        const int n = min(n0 + row, d.N - 1);
#pragma unroll
        for (int i = 0; i < 4; i++)
            R.w[i] = load16(codes + ((size_t)n * K + k0 + half * 32 + i * 8) * 2);
    }
}

// Write the step's slabs to LDS.  4-bit: the unpacking yields each block of 8 codes in the
// order (0 4 1 5 2 6 3 7); x is written in the same order so the MFMA sums matching pairs.
template <int BITS>
__device__ __forceinline__ void store_step(const Regs<BITS> &R, uint16_t *xs, uint16_t *ws)
{
    const int t = threadIdx.x;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const int idx = i * THREADS + t, row = idx >> 3, piece = idx & 7;
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
    if (BITS == 4) {
        const int row = t >> 1, piece = t & 1;
        const uint32_t z = R.z;
        const uint32_t nz_lo = (z | (z << 16)) | 0xE400E400u;        // -(1024 + z) twice
        const uint32_t nz_hi = ((z << 4) | (z << 20)) | 0xD400D400u; // -(  64 + z) twice
        const uint32_t ww[4] = {R.w[0].x, R.w[0].y, R.w[0].z, R.w[0].w};
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const uint32_t v = ww[i], v8 = v >> 8;
            uint4 o;
            o.x = pk_add((v & 0x000F000Fu) | 0x64006400u, nz_lo);  // (q0 - z, q4 - z)
            o.y = pk_add((v & 0x00F000F0u) | 0x54005400u, nz_hi);  // (q1 - z, q5 - z)
            o.z = pk_add((v8 & 0x000F000Fu) | 0x64006400u, nz_lo); // (q2 - z, q6 - z)
            o.w = pk_add((v8 & 0x00F000F0u) | 0x54005400u, nz_hi); // (q3 - z, q7 - z)
            *reinterpret_cast<uint4 *>(ws + row * LDK + piece * 32 + i * 8) = o;
        }
    } else if (BITS == 8) {
        const int row = t >> 1, half = t & 1;
        const uint32_t z = R.z;
        const uint32_t nz = (z | (z << 16)) | 0xE400E400u;
#pragma unroll
        for (int i = 0; i < 2; i++) {
            const uint32_t ww[4] = {R.w[i].x, R.w[i].y, R.w[i].z, R.w[i].w};
#pragma unroll
            for (int h = 0; h < 2; h++) {
                uint4 o;
                o.x = pk_add(__builtin_amdgcn_perm(0x64646464u, ww[2 * h], 0x04010400u), nz);
                o.y = pk_add(__builtin_amdgcn_perm(0x64646464u, ww[2 * h], 0x04030402u), nz);
                o.z = pk_add(__builtin_amdgcn_perm(0x64646464u, ww[2 * h + 1], 0x04010400u), nz);
                o.w = pk_add(__builtin_amdgcn_perm(0x64646464u, ww[2 * h + 1], 0x04030402u), nz);
                *reinterpret_cast<uint4 *>(ws + row * LDK + half * 32 + i * 16 + h * 8) = o;
            }
        }
    } else {
        const int row = t >> 1, half = t & 1;
#pragma unroll
        for (int i = 0; i < 4; i++)
            *reinterpret_cast<uint4 *>(ws + row * LDK + half * 32 + i * 8) = R.w[i];
    }
}

template <int BITS>
__global__ __launch_bounds__(THREADS) void prefill_kernel(const FqLinearDesc d, int M, int m_tiles,
                                                          int n_tiles, int per_xcd)
{
    __shared__ __attribute__((aligned(16))) uint16_t xs[BM * LDK];
    __shared__ __attribute__((aligned(16))) uint16_t ws[BN * LDK];

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
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64; // wavefront's corner inside the tile
    const int l32 = lane & 31, khalf = lane >> 5;

    float16_t acc[2][2], out[2][2];
#pragma unroll
    for (int a = 0; a < 2; a++)
#pragma unroll
        for (int b = 0; b < 2; b++)
#pragma unroll
            for (int v = 0; v < 16; v++) {
                acc[a][b][v] = 0.f;
                out[a][b][v] = 0.f;
            }

    const int nsteps = d.K / BK; // K is a multiple of 128: an even number of steps
    Regs<BITS> R;
    load_step<BITS>(d, codes, zeros, M, m0, n0, 0, R);
    for (int s = 0; s < nsteps; s++) {
        __syncthreads(); // everyone is done reading the previous slabs
        store_step<BITS>(R, xs, ws);
        __syncthreads();
        // prefetch the next step (the last iteration re-reads its own: keeps the waits counted)
        load_step<BITS>(d, codes, zeros, M, m0, n0, min(s + 1, nsteps - 1) * BK, R);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 16) {
            uint4 a[2], b[2];
#pragma unroll
            for (int i = 0; i < 2; i++) {
                a[i] = *reinterpret_cast<const uint4 *>(xs + (wm + i * 32 + l32) * LDK + kk + khalf * 8);
                b[i] = *reinterpret_cast<const uint4 *>(ws + (wn + i * 32 + l32) * LDK + kk + khalf * 8);
            }
#pragma unroll
            for (int i = 0; i < 2; i++)
#pragma unroll
                for (int j = 0; j < 2; j++)
                    acc[i][j] = mfma32(a[i], b[j], acc[i][j]);
        }
        if (BITS != 16 && (s & 1)) { // a group of 128 k is complete
            const int g = (s * BK) >> 7;
#pragma unroll
            for (int j = 0; j < 2; j++) {
                const int n = min(n0 + wn + j * 32 + l32, d.N - 1);
                const float sc = ((const FQ_GLOBAL float *)scales)[(size_t)n * (d.K >> 7) + g];
#pragma unroll
                for (int i = 0; i < 2; i++) {
                    out[i][j] += sc * acc[i][j];
#pragma unroll
                    for (int v = 0; v < 16; v++)
                        acc[i][j][v] = 0.f;
                }
            }
        }
    }
    // D layout of the 32x32 MFMA: lane holds column l32, rows 8 * (v / 4) + 4 * (lane / 32) + v % 4.
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
        for (int j = 0; j < 2; j++) {
            const int n = n0 + wn + j * 32 + l32;
#pragma unroll
            for (int v = 0; v < 16; v++) {
                const int m = m0 + wm + i * 32 + 8 * (v >> 2) + 4 * khalf + (v & 3);
                const float val = BITS == 16 ? acc[i][j][v] : out[i][j][v];
                if (m < M && n < d.N)
                    ((FQ_GLOBAL uint16_t *)d.y)[(size_t)m * d.N + n] =
                        __builtin_bit_cast(uint16_t, (_Float16)val);
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
