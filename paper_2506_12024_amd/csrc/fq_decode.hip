// Decode-phase weight-only quantized linear for gfx950: y = x . dequant(W)^T
// with dequant = Sec. 2.2 Eq. (3), one row of x (this file: M = 1, a GEMV).
// The decode phase is bound by streaming the weights (Sec. 4.1), so the kernel
// is built around the HBM stream: it reads the packed copy of the bit-width
// chosen for this call exactly once with coalesced 128-bit loads and keeps
// everything else (x, per-slice sums of x) in LDS.
//
// Work list.  A launch serves one linear (descriptor passed by value) or a
// table of independent linears (plan).  Rows are cut into tiles of 16
// (4 wavefronts x 4 rows); tiles of all entries are numbered consecutively and
// workgroup b takes tiles b, b + gridDim, ...  The bit-width of an entry is a
// run-time value (host argument or device array): all three inner loops live
// in the one kernel and the choice is a wavefront-uniform branch, so switching
// precision per token costs a pointer select and nothing else.
//
// Inner loop, 4-bit.  A lane owns 32 consecutive codes (16 bytes) of a row:
// slice j of the row covers k = 2048 j + 32 lane .. +31, all inside one
// quantization group.  Codes are turned into halves without any int->float
// conversion: (w & 0x000F000F) | 0x64006400 is the half pair (1024 + q0,
// 1024 + q4), (w & 0x00F000F0) | 0x54005400 is (64 + q1, 64 + q5); the upper two
// bytes follow after one shift.  Each pair goes through one v_dot2_f32_f16
// against the matching pair of x (x is staged in LDS already permuted), in
// binary32.  The offsets and the zero point are removed once per slice:
//   sum_k x_k (q_k - z) = acc - (1024 sum_even x + 64 sum_odd x) - z sum x
// where the two sums of x over the slice come precomputed from LDS, then the
// slice is scaled by s[n][g] and added to the row's accumulator.
// 8-bit: v_perm_b32 places each byte under the exponent 0x64 (1024 + q), the
// rest is the same.  16-bit: the halves are used as they are.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fq_internal.h"

namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

constexpr int WG_THREADS = 256;
constexpr int WAVES = WG_THREADS / 64;
constexpr int ROWS_PER_WAVE = 4;
constexpr int TILE_ROWS = WAVES * ROWS_PER_WAVE;

__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c)
{
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, a), __builtin_bit_cast(half2_t, b), c,
                                  false);
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1)
        v += __shfl_xor(v, off, 64);
    return v;
}

// ---- x staging -------------------------------------------------------------
// LDS holds x in 16-byte blocks of 8 halves (block b = k / 8), placed so that
// the blocks one lane needs for one slice are read by consecutive lanes from
// consecutive addresses (no bank conflicts), and, for 4-bit, permuted inside
// the block to the pair order the unpacking produces.  Blocks past K are zero.
// After the blocks come the per-slice sums of x.
//
//   bits  codes/lane/slice  blocks/lane  block position
//    4        32               4         ((b >> 8) * 4 + (b & 3)) * 64 + ((b >> 2) & 63)
//    8        16               2         ((b >> 7) * 2 + (b & 1)) * 64 + ((b >> 1) & 63)
//   16         8               1         b
template <int BITS>
__device__ __forceinline__ int block_pos(int b)
{
    if (BITS == 4)
        return ((b >> 8) * 4 + (b & 3)) * 64 + ((b >> 2) & 63);
    if (BITS == 8)
        return ((b >> 7) * 2 + (b & 1)) * 64 + ((b >> 1) & 63);
    return b;
}

__device__ __forceinline__ int padded_k(int K, int bits)
{
    const int span = bits == 4 ? 2048 : (bits == 8 ? 1024 : 512); // k per wavefront slice
    return (K + span - 1) / span * span;
}

template <int BITS>
__device__ __forceinline__ void stage_x(const uint16_t *__restrict__ x, int K, uint4 *lds)
{
    const int Kp = padded_k(K, BITS);
    const int nblk = Kp >> 3;
    float *sums = reinterpret_cast<float *>(lds + nblk); // [slices][2] for 4-bit, [slices] for 8-bit
    for (int b = threadIdx.x; b < nblk; b += WG_THREADS) {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (b * 8 < K)
            v = reinterpret_cast<const uint4 *>(x)[b];
        if (BITS == 16) {
            lds[b] = v;
            continue;
        }
        // binary32 sums of the even- and odd-indexed halves of the block
        float even = 0.f, odd = 0.f;
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const half2_t h = __builtin_bit_cast(half2_t, w[i]);
            even += (float)h[0];
            odd += (float)h[1];
        }
        if (BITS == 4) {
            // [x0 x1 | x2 x3 | x4 x5 | x6 x7] -> [x0 x4 | x1 x5 | x2 x6 | x3 x7]
            uint4 p;
            p.x = __builtin_amdgcn_perm(v.z, v.x, 0x05040100u); // (x0, x4)
            p.y = __builtin_amdgcn_perm(v.z, v.x, 0x07060302u); // (x1, x5)
            p.z = __builtin_amdgcn_perm(v.w, v.y, 0x05040100u); // (x2, x6)
            p.w = __builtin_amdgcn_perm(v.w, v.y, 0x07060302u); // (x3, x7)
            lds[block_pos<4>(b)] = p;
            // slice = 4 blocks = 4 consecutive threads (b & 3 == threadIdx & 3)
            even += __shfl_xor(even, 1, 64);
            odd += __shfl_xor(odd, 1, 64);
            even += __shfl_xor(even, 2, 64);
            odd += __shfl_xor(odd, 2, 64);
            if ((b & 3) == 0) {
                sums[(b >> 2) * 2 + 0] = 1024.0f * even + 64.0f * odd;
                sums[(b >> 2) * 2 + 1] = even + odd;
            }
        } else {
            lds[block_pos<8>(b)] = v;
            float s = even + odd;
            s += __shfl_xor(s, 1, 64);
            if ((b & 1) == 0)
                sums[b >> 1] = s;
        }
    }
}

// ---- per-wavefront row block: 4 rows x full K ---------------------------------

struct RowOut {
    float acc[ROWS_PER_WAVE];
};

__device__ __forceinline__ void rows_w4(const FqLinearDesc &d, int row0, const uint4 *lds,
                                        RowOut &out)
{
    const int lane = threadIdx.x & 63;
    const int K = d.K, G = K >> 7;
    const int nslice = (K + 2047) >> 11;
    const float2 *sums = reinterpret_cast<const float2 *>(lds + (padded_k(K, 4) >> 3));
    size_t rowoff[ROWS_PER_WAVE];
#pragma unroll
    for (int r = 0; r < ROWS_PER_WAVE; r++)
        rowoff[r] = (size_t)min(row0 + r, d.N - 1);
    // The two exponent patterns live in VGPRs (hidden from constant folding) so that
    // mask-and-merge is one v_and_or_b32 with the mask on the scalar bus.
    uint32_t magic_lo = 0x64006400u, magic_hi = 0x54005400u;
    asm volatile("" : "+v"(magic_lo), "+v"(magic_hi));
    for (int j = 0; j < nslice; j++) {
        const int k0 = j * 2048 + lane * 32;
        const int k0c = min(k0, K - 32); // lanes past K read a valid address; their x is zero
        uint4 w[ROWS_PER_WAVE];
        float s[ROWS_PER_WAVE];
        uint32_t z[ROWS_PER_WAVE];
#pragma unroll
        for (int r = 0; r < ROWS_PER_WAVE; r++) {
            w[r] = *reinterpret_cast<const uint4 *>(d.codes4 + rowoff[r] * (size_t)(K >> 1) + (k0c >> 1));
            s[r] = d.scales4[rowoff[r] * G + (k0c >> 7)];
            z[r] = d.zeros4[rowoff[r] * G + (k0c >> 7)];
        }
        uint4 xb[4];
#pragma unroll
        for (int i = 0; i < 4; i++)
            xb[i] = lds[(j * 4 + i) * 64 + lane];
        const float2 cs = sums[j * 64 + lane]; // (1024 sum_even + 64 sum_odd, sum)
#pragma unroll
        for (int r = 0; r < ROWS_PER_WAVE; r++) {
            const uint32_t ww[4] = {w[r].x, w[r].y, w[r].z, w[r].w};
            float a = 0.0f;
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const uint32_t v = ww[i], v8 = v >> 8;
                const uint32_t t0 = (v & 0x000F000Fu) | magic_lo;  // (1024+q0, 1024+q4)
                const uint32_t t1 = (v & 0x00F000F0u) | magic_hi;  // (  64+q1,   64+q5)
                const uint32_t t2 = (v8 & 0x000F000Fu) | magic_lo; // (1024+q2, 1024+q6)
                const uint32_t t3 = (v8 & 0x00F000F0u) | magic_hi; // (  64+q3,   64+q7)
                a = dot2(t0, xb[i].x, a);
                a = dot2(t1, xb[i].y, a);
                a = dot2(t2, xb[i].z, a);
                a = dot2(t3, xb[i].w, a);
            }
            const float part = a - cs.x - (float)z[r] * cs.y;
            out.acc[r] += s[r] * part;
        }
    }
}

__device__ __forceinline__ void rows_w8(const FqLinearDesc &d, int row0, const uint4 *lds,
                                        RowOut &out)
{
    const int lane = threadIdx.x & 63;
    const int K = d.K, G = K >> 7;
    const int nslice = (K + 1023) >> 10;
    const float *sums = reinterpret_cast<const float *>(lds + (padded_k(K, 8) >> 3));
    size_t rowoff[ROWS_PER_WAVE];
#pragma unroll
    for (int r = 0; r < ROWS_PER_WAVE; r++)
        rowoff[r] = (size_t)min(row0 + r, d.N - 1);
    for (int j = 0; j < nslice; j++) {
        const int k0 = j * 1024 + lane * 16;
        const int k0c = min(k0, K - 16);
        uint4 w[ROWS_PER_WAVE];
        float s[ROWS_PER_WAVE];
        uint32_t z[ROWS_PER_WAVE];
#pragma unroll
        for (int r = 0; r < ROWS_PER_WAVE; r++) {
            w[r] = *reinterpret_cast<const uint4 *>(d.codes8 + rowoff[r] * (size_t)K + k0c);
            s[r] = d.scales8[rowoff[r] * G + (k0c >> 7)];
            z[r] = d.zeros8[rowoff[r] * G + (k0c >> 7)];
        }
        const uint4 x0 = lds[(j * 2 + 0) * 64 + lane], x1 = lds[(j * 2 + 1) * 64 + lane];
        const uint32_t xx[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
        const float sx = sums[j * 64 + lane];
#pragma unroll
        for (int r = 0; r < ROWS_PER_WAVE; r++) {
            const uint32_t ww[4] = {w[r].x, w[r].y, w[r].z, w[r].w};
            float a = 0.0f;
#pragma unroll
            for (int i = 0; i < 4; i++) {
                // bytes b0..b3 -> halves 0x64b0, 0x64b1 | 0x64b2, 0x64b3 (1024 + code)
                const uint32_t lo = __builtin_amdgcn_perm(0x64646464u, ww[i], 0x04010400u);
                const uint32_t hi = __builtin_amdgcn_perm(0x64646464u, ww[i], 0x04030402u);
                a = dot2(lo, xx[2 * i], a);
                a = dot2(hi, xx[2 * i + 1], a);
            }
            const float part = a - (1024.0f + (float)z[r]) * sx;
            out.acc[r] += s[r] * part;
        }
    }
}

__device__ __forceinline__ void rows_w16(const FqLinearDesc &d, int row0, const uint4 *lds,
                                         RowOut &out)
{
    const int lane = threadIdx.x & 63;
    const int K = d.K;
    const int nslice = (K + 511) >> 9;
    size_t rowoff[ROWS_PER_WAVE];
#pragma unroll
    for (int r = 0; r < ROWS_PER_WAVE; r++)
        rowoff[r] = (size_t)min(row0 + r, d.N - 1);
    for (int j = 0; j < nslice; j++) {
        const int k0 = j * 512 + lane * 8;
        const int k0c = min(k0, K - 8);
        uint4 w[ROWS_PER_WAVE];
#pragma unroll
        for (int r = 0; r < ROWS_PER_WAVE; r++)
            w[r] = *reinterpret_cast<const uint4 *>(d.w16 + rowoff[r] * (size_t)K + k0c);
        const uint4 xv = lds[j * 64 + lane];
#pragma unroll
        for (int r = 0; r < ROWS_PER_WAVE; r++) {
            float a = out.acc[r];
            a = dot2(w[r].x, xv.x, a);
            a = dot2(w[r].y, xv.y, a);
            a = dot2(w[r].z, xv.z, a);
            a = dot2(w[r].w, xv.w, a);
            out.acc[r] = a;
        }
    }
}

__device__ __forceinline__ uint16_t to_half_bits(float f)
{
    return __builtin_bit_cast(uint16_t, (_Float16)f);
}

template <bool SINGLE>
__global__ __launch_bounds__(WG_THREADS) void decode_m1_kernel(const FqLinearDesc single,
                                                               int bits_host,
                                                               const FqLinearDesc *__restrict__ table,
                                                               const int32_t *__restrict__ bits_dev,
                                                               int count, int total_tiles)
{
    extern __shared__ uint4 lds[];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    int cur = -1; // entry whose x is staged
    int e = 0;
    for (int tile = blockIdx.x; tile < total_tiles; tile += gridDim.x) {
        FqLinearDesc d;
        int bits;
        if (SINGLE) {
            d = single;
            bits = bits_host;
        } else {
            // tiles are visited in increasing order: advance the entry cursor
            while (e + 1 < count && tile >= table[e + 1].tile_begin)
                e++;
            d = table[e];
            bits = bits_dev[e];
        }
        const bool ok = (bits == 4 && d.codes4) || (bits == 8 && d.codes8) || (bits == 16 && d.w16);
        if (!ok)
            continue; // uniform: a skipped entry leaves its y untouched
        if (cur != e) {
            __syncthreads(); // every wavefront is done reading the previous x
            if (bits == 4)
                stage_x<4>(d.x, d.K, lds);
            else if (bits == 8)
                stage_x<8>(d.x, d.K, lds);
            else
                stage_x<16>(d.x, d.K, lds);
            __syncthreads();
            cur = e;
        }
        const int row0 = (tile - d.tile_begin) * TILE_ROWS + wave * ROWS_PER_WAVE;
        if (row0 >= d.N)
            continue; // no barrier is skipped by this: the next staging syncs all wavefronts
        RowOut out;
#pragma unroll
        for (int r = 0; r < ROWS_PER_WAVE; r++)
            out.acc[r] = 0.0f;
        if (bits == 4)
            rows_w4(d, row0, lds, out);
        else if (bits == 8)
            rows_w8(d, row0, lds, out);
        else
            rows_w16(d, row0, lds, out);
#pragma unroll
        for (int r = 0; r < ROWS_PER_WAVE; r++) {
            const float v = wave_sum(out.acc[r]);
            if (lane == r && row0 + r < d.N)
                d.y[row0 + r] = to_half_bits(v);
        }
    }
}

} // namespace

int fq_decode_rows_per_tile(int M)
{
    (void)M;
    return TILE_ROWS;
}

static size_t lds_bytes_for(int max_K)
{
    // worst case over the three bit-widths: 4-bit pads K to 2048 and adds 8 bytes per 32 k
    const size_t kp = ((size_t)max_K + 2047) / 2048 * 2048;
    return kp * 2 + kp / 32 * 8 + 64;
}

hipError_t fq_launch_decode(const FqLinearDesc *single, int bits_host,
                            const FqLinearDesc *descs_dev, const int32_t *bits_dev, int count,
                            int total_tiles, int max_K, int M, hipStream_t stream)
{
    (void)M;
    if (total_tiles <= 0)
        return hipSuccess;
    const size_t lds = lds_bytes_for(max_K);
    // Persistent-style grid: enough workgroups to fill 256 CUs several times over,
    // never more than there are tiles.
    const int grid = total_tiles < 2048 ? total_tiles : 2048;
    if (single) {
        decode_m1_kernel<true><<<grid, WG_THREADS, lds, stream>>>(*single, bits_host, nullptr,
                                                                  nullptr, 1, total_tiles);
    } else {
        FqLinearDesc none = {};
        decode_m1_kernel<false><<<grid, WG_THREADS, lds, stream>>>(none, 0, descs_dev, bits_dev,
                                                                   count, total_tiles);
    }
    return hipGetLastError();
}
