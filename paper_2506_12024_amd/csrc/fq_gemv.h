// Device code shared by the batch-1 decode kernels (one launch per plan, and the stage-ordered
// persistent kernel): how a row of x is laid out in LDS for each bit-width, what one lane loads for
// one item of work, and the arithmetic of an item -- Sec. 2.2 Eq. (3) applied on the fly inside the
// dot product of Sec. 4.1's weight-only linear.  Both kernels give a row to one wavefront with the same lane ->
// k mapping and the same order of slices, so their results agree bit for bit.
#ifndef FQ_GEMV_H
#define FQ_GEMV_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

#define FQ_GLOBAL __attribute__((address_space(1)))

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// 128-bit load through an explicitly global pointer (global_load_dwordx4, vmcnt only).
__device__ __forceinline__ uint4 load16_global(const void *p)
{
    const u32x4 v = *(const FQ_GLOBAL u32x4 *)p;
    return make_uint4(v.x, v.y, v.z, v.w);
}

constexpr int ROWS_PER_WAVE = 4;

template <class T>
__device__ __forceinline__ const FQ_GLOBAL T *as_global(const void *p)
{
    return (const FQ_GLOBAL T *)p;
}

__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c)
{
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, a), __builtin_bit_cast(half2_t, b), c,
                                  false);
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_take(float v)
{
    // lanes whose row is masked out, or whose source lane does not exist, read 0
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL,
                                                                  ROW_MASK, 0xF, false));
}

// Sum over the 64 lanes with DPP modifiers only (no LDS crossbar): xor 1, xor 2 inside
// quads, mirror inside 8 and 16, then row broadcasts.  The total lands in lane 63.
__device__ __forceinline__ float wave_sum_lane63(float v)
{
    v += dpp_take<0xB1, 0xF>(v);  // quad_perm [1,0,3,2]
    v += dpp_take<0x4E, 0xF>(v);  // quad_perm [2,3,0,1]
    v += dpp_take<0x141, 0xF>(v); // row_half_mirror
    v += dpp_take<0x140, 0xF>(v); // row_mirror: every lane of a row holds the row's sum
    v += dpp_take<0x142, 0xA>(v); // row_bcast15 into rows 1 and 3
    v += dpp_take<0x143, 0xC>(v); // row_bcast31 into rows 2 and 3
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
//    2        64               8         ((b >> 9) * 8 + (b & 7)) * 64 + ((b >> 3) & 63), pairs of blocks interleaved
//    3        32               4         as for 4 bits (the lane's 32 x regrouped into the pairs its three code words meet)
//    4        32               4         ((b >> 8) * 4 + (b & 3)) * 64 + ((b >> 2) & 63)
//    8        16               2         ((b >> 7) * 2 + (b & 1)) * 64 + ((b >> 1) & 63)
//   16         8               1         b
template <int BITS>
__device__ __forceinline__ int block_pos(int b)
{
    if (BITS == 2)
        return ((b >> 9) * 8 + (b & 7)) * 64 + ((b >> 3) & 63);
    if (BITS == 4 || BITS == 3)
        return ((b >> 8) * 4 + (b & 3)) * 64 + ((b >> 2) & 63);
    if (BITS == 8)
        return ((b >> 7) * 2 + (b & 1)) * 64 + ((b >> 1) & 63);
    return b;
}

// k covered by one wavefront slice: 64 lanes x 16 bytes of codes
__device__ __forceinline__ int slice_span(int bits) { return bits == 2 ? 4096 : bits == 4 || bits == 3 ? 2048 : (bits == 8 ? 1024 : 512); }

__device__ __forceinline__ int padded_k(int K, int bits)
{
    const int span = slice_span(bits);
    return (K + span - 1) / span * span;
}

// 2 bits.  A 32-bit word of codes holds 16 consecutive k: code i in bits 2 i .. 2 i + 1.  The
// unpacking pairs code i of the low half-word with code 8 + i of the high one, so the two x blocks
// of those 16 k, A = x[0..7] and B = x[8..15], are stored interleaved: (A0 B0 A1 B1 A2 B2 A3 B3),
// (A4 B4 .. A7 B7).  A code keeps its bit position, which fixes its offset: 1024 / 256 / 64 / 16
// for i % 4 = 0 / 1 / 2 / 3.  A thread stages one such pair of blocks; the four threads of a lane's
// slice (64 k) add up its two sums.
// Places the pair of blocks pb (k = 16 pb .. 16 pb + 15; va, vb = its two blocks as loaded, zeros
// past K) and, from the first of every four consecutive lanes, the two sums of their slice.
// Consecutive lanes must hold consecutive pb, all lanes of a quad active.
__device__ __forceinline__ void place_pair2(int pb, uint4 va, uint4 vb, uint4 *lds, float2 *sums)
{
    float p[4] = {0.f, 0.f, 0.f, 0.f}; // sums of the x whose code sits at position i % 4
    const uint32_t w[8] = {va.x, va.y, va.z, va.w, vb.x, vb.y, vb.z, vb.w};
#pragma unroll
    for (int i = 0; i < 8; i++) {
        const half2_t h = __builtin_bit_cast(half2_t, w[i]); // halves 2 i, 2 i + 1 of their block
        p[(2 * i) & 3] += (float)h[0];
        p[(2 * i + 1) & 3] += (float)h[1];
    }
    uint4 o0, o1;
    o0.x = __builtin_amdgcn_perm(vb.x, va.x, 0x05040100u); // (A0, B0)
    o0.y = __builtin_amdgcn_perm(vb.x, va.x, 0x07060302u); // (A1, B1)
    o0.z = __builtin_amdgcn_perm(vb.y, va.y, 0x05040100u); // (A2, B2)
    o0.w = __builtin_amdgcn_perm(vb.y, va.y, 0x07060302u); // (A3, B3)
    o1.x = __builtin_amdgcn_perm(vb.z, va.z, 0x05040100u); // (A4, B4)
    o1.y = __builtin_amdgcn_perm(vb.z, va.z, 0x07060302u);
    o1.z = __builtin_amdgcn_perm(vb.w, va.w, 0x05040100u);
    o1.w = __builtin_amdgcn_perm(vb.w, va.w, 0x07060302u); // (A7, B7)
    lds[block_pos<2>(2 * pb)] = o0;
    lds[block_pos<2>(2 * pb + 1)] = o1;
    float c = 1024.0f * p[0] + 256.0f * p[1] + 64.0f * p[2] + 16.0f * p[3];
    float t = (p[0] + p[1]) + (p[2] + p[3]);
    // slice = 4 pairs = 4 consecutive threads
    c += dpp_take<0xB1, 0xF>(c);
    t += dpp_take<0xB1, 0xF>(t);
    c += dpp_take<0x4E, 0xF>(c);
    t += dpp_take<0x4E, 0xF>(t);
    if ((pb & 3) == 0)
        sums[pb >> 2] = make_float2(c, t);
}

// 3 bits.  A lane's 12 bytes = three words hold 32 codes: word j the codes 10 j + 5 h + p (h = 0,
// 1: the word's halves; p = 0 .. 4: bits 3 p .. 3 p + 2 of the half), the words' bits 15 and 31 the
// codes 30 and 31, bit j of each in word j.  The unpacking pairs the two halves of a word, so the
// lane's 32 x are stored as 16 pairs in the order it meets them: pair 5 j + p = (x[10 j + p],
// x[10 j + 5 + p]), pair 15 = (x[30], x[31]).  A whole code keeps its place in its half, which
// fixes its offset: 1024 / 128 / 16 for p = 0 / 1 / 2 and again, after a shift by 9 bits, 1024 /
// 128 for p = 3 / 4; a bit of the last two codes is read at bit 6 after that shift, under 16 / 32
// / 64 in words 0 / 1 / 2, where it is worth 1 / 2 / 4: offset 112 in all.
__device__ __forceinline__ constexpr float offset3(int i)
{
    return i >= 30 ? 112.0f : (i % 5 == 0 || i % 5 == 3) ? 1024.0f : (i % 5 == 1 || i % 5 == 4) ? 128.0f : 16.0f;
}

// Places the x of lane slice ls (k = 32 ls .. 32 ls + 31; v = its four blocks as loaded, zeros
// past K) and the slice's two sums: sum offset(k) x_k and sum x_k.
__device__ __forceinline__ void place_slice3(int ls, const uint4 (&v)[4], uint4 *lds, float2 *sums)
{
    const uint32_t w[16] = {v[0].x, v[0].y, v[0].z, v[0].w, v[1].x, v[1].y, v[1].z, v[1].w,
                            v[2].x, v[2].y, v[2].z, v[2].w, v[3].x, v[3].y, v[3].z, v[3].w};
    float c = 0.f, t = 0.f;
#pragma unroll
    for (int d = 0; d < 16; d++) {
        const half2_t h = __builtin_bit_cast(half2_t, w[d]); // x[2 d], x[2 d + 1]
        c += offset3(2 * d) * (float)h[0] + offset3(2 * d + 1) * (float)h[1];
        t += (float)h[0] + (float)h[1];
    }
    uint32_t o[16];
#pragma unroll
    for (int u = 0; u < 16; u++) {
        const int a = u < 15 ? 10 * (u / 5) + u % 5 : 30, b = u < 15 ? a + 5 : 31; // the pair (x[a], x[b])
        const uint32_t sel = ((b & 1) ? 0x07060000u : 0x05040000u) | ((a & 1) ? 0x0302u : 0x0100u);
        o[u] = __builtin_amdgcn_perm(w[b >> 1], w[a >> 1], sel);
    }
#pragma unroll
    for (int i = 0; i < 4; i++)
        lds[((ls >> 6) * 4 + i) * 64 + (ls & 63)] = make_uint4(o[4 * i], o[4 * i + 1], o[4 * i + 2], o[4 * i + 3]);
    sums[ls] = make_float2(c, t);
}

// Places block b (k = 8 b .. 8 b + 7; v as loaded, zeros past K) for 4, 8 or 16 bits and the sums
// of its slice.  Consecutive lanes must hold consecutive b, all lanes of a quad active.
template <int BITS>
__device__ __forceinline__ void place_block(int b, uint4 v, uint4 *lds, float *sums)
{
    if (BITS == 16) {
        lds[b] = v;
        return;
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
        even += dpp_take<0xB1, 0xF>(even);
        odd += dpp_take<0xB1, 0xF>(odd);
        even += dpp_take<0x4E, 0xF>(even);
        odd += dpp_take<0x4E, 0xF>(odd);
        if ((b & 3) == 0) {
            sums[(b >> 2) * 2 + 0] = 1024.0f * even + 64.0f * odd;
            sums[(b >> 2) * 2 + 1] = even + odd;
        }
    } else {
        lds[block_pos<8>(b)] = v;
        float s = even + odd;
        s += dpp_take<0xB1, 0xF>(s);
        if ((b & 1) == 0)
            sums[b >> 1] = s;
    }
}

// Stages a row of x with THREADS threads (threadIdx.x % THREADS = the thread's place among them).
template <int BITS, int THREADS>
__device__ __forceinline__ void stage_x(const uint16_t *x, int K, uint4 *lds)
{
    const int Kp = padded_k(K, BITS);
    if (BITS == 3) {
        const int nls = Kp >> 5; // lane slices of 32 k: a thread stages a whole one
        float2 *sums = reinterpret_cast<float2 *>(lds + (Kp >> 3)); // per lane slice: (sum off(k) x, sum x)
        for (int ls = threadIdx.x % THREADS; ls < nls; ls += THREADS) {
            uint4 v[4];
#pragma unroll
            for (int i = 0; i < 4; i++) // K is a multiple of 128: all four blocks or none
                v[i] = ls * 32 < K ? load16_global(x + (size_t)ls * 32 + 8 * i) : make_uint4(0, 0, 0, 0);
            place_slice3(ls, v, lds, sums);
        }
        return;
    }
    if (BITS == 2) {
        const int npair = Kp >> 4; // a multiple of 256: every thread makes the same number of trips
        float2 *sums = reinterpret_cast<float2 *>(lds + (Kp >> 3)); // per lane slice: (sum off(k) x, sum x)
        for (int pb = threadIdx.x % THREADS; pb < npair; pb += THREADS) {
            uint4 va = make_uint4(0, 0, 0, 0), vb = make_uint4(0, 0, 0, 0);
            if (pb * 16 < K) { // K is a multiple of 128: both blocks or neither
                va = load16_global(x + (size_t)pb * 16);
                vb = load16_global(x + (size_t)pb * 16 + 8);
            }
            place_pair2(pb, va, vb, lds, sums);
        }
        return;
    }
    const int nblk = Kp >> 3;
    float *sums = reinterpret_cast<float *>(lds + nblk); // [slices][2] for 4-bit, [slices] for 8-bit
    for (int b = threadIdx.x % THREADS; b < nblk; b += THREADS) {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (b * 8 < K)
            v = load16_global(x + (size_t)b * 8);
        place_block<BITS>(b, v, lds, sums);
    }
}

// ---- items --------------------------------------------------------------------

// What one lane holds for one item: 4 rows x (16 bytes of codes, scale, zero).
struct Loaded {
    uint4 w[ROWS_PER_WAVE];
    float s[ROWS_PER_WAVE];
    uint8_t z[ROWS_PER_WAVE]; // kept as bytes: converted where used, so that nothing touches a register while its load is in flight
};

// The copy of one entry selected by the call's bit-width (wavefront-uniform).
struct Sel {
    const uint8_t *codes; // fp16 weights for 16
    const float *scales;
    const uint8_t *zeros;
    int N, K;
};

// 128-bit streaming load: the weights are read once, keep them out of the caches' way.
__device__ __forceinline__ uint4 load16_stream(const void *p)
{
    const u32x4 v = __builtin_nontemporal_load((const FQ_GLOBAL u32x4 *)p);
    return make_uint4(v.x, v.y, v.z, v.w);
}

// The same from an address that is only 4-byte aligned (one instruction all the same).
__device__ __forceinline__ uint4 load16_stream_a4(const void *p)
{
    typedef u32x4 u32x4_a4 __attribute__((aligned(4)));
    const u32x4 v = __builtin_nontemporal_load((const FQ_GLOBAL u32x4_a4 *)p);
    return make_uint4(v.x, v.y, v.z, v.w);
}

// 96-bit streaming load (a 3-bit block: 4-byte aligned); .w is left 0.
__device__ __forceinline__ uint4 load12_stream(const void *p)
{
    typedef uint32_t u32x3 __attribute__((ext_vector_type(3)));
    typedef u32x3 u32x3_a4 __attribute__((aligned(4)));
    const u32x3 v = __builtin_nontemporal_load((const FQ_GLOBAL u32x3_a4 *)p);
    return make_uint4(v.x, v.y, v.z, 0u);
}

// Issue the global loads of item (rows row0..row0+3, slice j).  Rows past N and lanes
// past K are clamped to valid addresses (their results are discarded: the row is not
// stored, the lane's x is zero).
template <int BITS>
__device__ __forceinline__ void issue(const Sel &d, int row0, int j, Loaded &L)
{
    const int lane = threadIdx.x & 63;
    const uint32_t K = (uint32_t)d.K, G = K >> 7;
    constexpr int CODES = BITS == 3 ? 32 : 128 / BITS; // per lane per slice: 16 bytes (3 bits: a block of 12)
    const uint32_t k0 = min((uint32_t)(j * 64 + lane) * CODES, K - CODES);
    const uint32_t row_bytes = BITS == 2 ? (K >> 2) : BITS == 3 ? (K >> 3) * 3 : BITS == 4 ? (K >> 1) : (BITS == 8 ? K : 2 * K);
    const uint32_t byte0 = BITS == 2 ? (k0 >> 2) : BITS == 3 ? (k0 >> 5) * 12 : BITS == 4 ? (k0 >> 1) : (BITS == 8 ? k0 : 2 * k0);
    const uint32_t g = k0 >> 7;
#pragma unroll
    for (int r = 0; r < ROWS_PER_WAVE; r++) {
        // row0 is wavefront-uniform: the row bases are scalar, each lane adds a 32-bit offset
        const uint32_t row = (uint32_t)min(row0 + r, d.N - 1);
        const uint8_t *rowp = d.codes + (size_t)row * row_bytes;
        L.w[r] = BITS == 3 ? load12_stream(rowp + byte0) : load16_stream(rowp + byte0);
        if (BITS != 16) {
            const float *srow = d.scales + (size_t)row * G;
            const uint8_t *zrow = d.zeros + (size_t)row * G;
            L.s[r] = as_global<float>(srow)[g];
            L.z[r] = as_global<uint8_t>(zrow)[g];
        }
    }
}

template <int BITS>
__device__ __forceinline__ void compute(int K, int j, const Loaded &L, const uint4 *lds,
                                        float (&acc)[ROWS_PER_WAVE])
{
    const int lane = threadIdx.x & 63;
    if (BITS == 2) {
        const float2 *sums = reinterpret_cast<const float2 *>(lds + (padded_k(K, 2) >> 3));
        // exponent patterns under which a 2-bit field at bits 0, 2, 4, 6 of a half reads as
        // 1024 + q, 256 + q, 64 + q, 16 + q (kept in VGPRs as for 4 bits)
        uint32_t m0 = 0x64006400u, m1 = 0x5C005C00u, m2 = 0x54005400u, m3 = 0x4C004C00u;
        asm volatile("" : "+v"(m0), "+v"(m1), "+v"(m2), "+v"(m3));
        const float2 cs = sums[j * 64 + lane]; // (sum off(k) x, sum x) over the lane's 64 k
        float a[ROWS_PER_WAVE] = {0.f, 0.f, 0.f, 0.f};
        // two rounds of two code words each: the x blocks of a round are all that is held at once
#pragma unroll
        for (int h = 0; h < 2; h++) {
            uint4 xb[4];
#pragma unroll
            for (int i = 0; i < 4; i++)
                xb[i] = lds[(j * 8 + 4 * h + i) * 64 + lane];
#pragma unroll
            for (int r = 0; r < ROWS_PER_WAVE; r++) {
                const uint32_t ww[2] = {h ? L.w[r].z : L.w[r].x, h ? L.w[r].w : L.w[r].y};
#pragma unroll
                for (int i = 0; i < 2; i++) {
                    const uint32_t v = ww[i], v8 = v >> 8;
                    a[r] = dot2((v & 0x00030003u) | m0, xb[2 * i].x, a[r]);      // codes 0, 8
                    a[r] = dot2((v & 0x000C000Cu) | m1, xb[2 * i].y, a[r]);      // codes 1, 9
                    a[r] = dot2((v & 0x00300030u) | m2, xb[2 * i].z, a[r]);      // codes 2, 10
                    a[r] = dot2((v & 0x00C000C0u) | m3, xb[2 * i].w, a[r]);      // codes 3, 11
                    a[r] = dot2((v8 & 0x00030003u) | m0, xb[2 * i + 1].x, a[r]); // codes 4, 12
                    a[r] = dot2((v8 & 0x000C000Cu) | m1, xb[2 * i + 1].y, a[r]);
                    a[r] = dot2((v8 & 0x00300030u) | m2, xb[2 * i + 1].z, a[r]);
                    a[r] = dot2((v8 & 0x00C000C0u) | m3, xb[2 * i + 1].w, a[r]); // codes 7, 15
                }
            }
        }
#pragma unroll
        for (int r = 0; r < ROWS_PER_WAVE; r++)
            acc[r] += L.s[r] * (a[r] - cs.x - (float)L.z[r] * cs.y);
    } else if (BITS == 3) {
        const float2 *sums = reinterpret_cast<const float2 *>(lds + (padded_k(K, 3) >> 3));
        // exponent patterns under which a field of a half reads as offset + code: 1024 for a field
        // at bit 0, 128 at bit 3, 16 at bit 6; a single bit at bit 6 reads as 32 + 2 b under the
        // pattern of 32 and as 64 + 4 b under that of 64 (kept in VGPRs as for 4 bits)
        uint32_t m0 = 0x64006400u, m1 = 0x58005800u, m2 = 0x4C004C00u, m3 = 0x50005000u, m4 = 0x54005400u;
        asm volatile("" : "+v"(m0), "+v"(m1), "+v"(m2), "+v"(m3), "+v"(m4));
        uint4 xb[4];
#pragma unroll
        for (int i = 0; i < 4; i++)
            xb[i] = lds[(j * 4 + i) * 64 + lane];
        const uint32_t xx[16] = {xb[0].x, xb[0].y, xb[0].z, xb[0].w, xb[1].x, xb[1].y, xb[1].z, xb[1].w,
                                 xb[2].x, xb[2].y, xb[2].z, xb[2].w, xb[3].x, xb[3].y, xb[3].z, xb[3].w};
        const float2 cs = sums[j * 64 + lane]; // (sum offset(k) x, sum x) over the lane's 32 k
#pragma unroll
        for (int r = 0; r < ROWS_PER_WAVE; r++) {
            const uint32_t ww[3] = {L.w[r].x, L.w[r].y, L.w[r].z};
            float a = 0.0f;
#pragma unroll
            for (int i = 0; i < 3; i++) {
                const uint32_t v = ww[i], v9 = v >> 9;
                a = dot2((v & 0x00070007u) | m0, xx[5 * i + 0], a);  // codes 10 i + 0, 10 i + 5
                a = dot2((v & 0x00380038u) | m1, xx[5 * i + 1], a);  // codes 10 i + 1, 10 i + 6
                a = dot2((v & 0x01C001C0u) | m2, xx[5 * i + 2], a);  // codes 10 i + 2, 10 i + 7
                a = dot2((v9 & 0x00070007u) | m0, xx[5 * i + 3], a); // codes 10 i + 3, 10 i + 8
                a = dot2((v9 & 0x00380038u) | m1, xx[5 * i + 4], a); // codes 10 i + 4, 10 i + 9
                a = dot2((v9 & 0x00400040u) | (i == 0 ? m2 : i == 1 ? m3 : m4), xx[15], a); // bit i of codes 30, 31
            }
            const float part = a - cs.x - (float)L.z[r] * cs.y;
            acc[r] += L.s[r] * part;
        }
    } else if (BITS == 4) {
        const float2 *sums = reinterpret_cast<const float2 *>(lds + (padded_k(K, 4) >> 3));
        // The two exponent patterns live in VGPRs (hidden from constant folding) so that
        // mask-and-merge is one v_and_or_b32 with the mask on the scalar bus.
        uint32_t magic_lo = 0x64006400u, magic_hi = 0x54005400u;
        asm volatile("" : "+v"(magic_lo), "+v"(magic_hi));
        uint4 xb[4];
#pragma unroll
        for (int i = 0; i < 4; i++)
            xb[i] = lds[(j * 4 + i) * 64 + lane];
        const float2 cs = sums[j * 64 + lane]; // (1024 sum_even x + 64 sum_odd x, sum x)
#pragma unroll
        for (int r = 0; r < ROWS_PER_WAVE; r++) {
            const uint32_t ww[4] = {L.w[r].x, L.w[r].y, L.w[r].z, L.w[r].w};
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
            const float part = a - cs.x - (float)L.z[r] * cs.y;
            acc[r] += L.s[r] * part;
        }
    } else if (BITS == 8) {
        const float *sums = reinterpret_cast<const float *>(lds + (padded_k(K, 8) >> 3));
        const uint4 x0 = lds[(j * 2 + 0) * 64 + lane], x1 = lds[(j * 2 + 1) * 64 + lane];
        const uint32_t xx[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
        const float sx = sums[j * 64 + lane];
#pragma unroll
        for (int r = 0; r < ROWS_PER_WAVE; r++) {
            const uint32_t ww[4] = {L.w[r].x, L.w[r].y, L.w[r].z, L.w[r].w};
            float a = 0.0f;
#pragma unroll
            for (int i = 0; i < 4; i++) {
                // bytes b0..b3 -> halves 0x64b0, 0x64b1 | 0x64b2, 0x64b3 (1024 + code)
                const uint32_t lo = __builtin_amdgcn_perm(0x64646464u, ww[i], 0x04010400u);
                const uint32_t hi = __builtin_amdgcn_perm(0x64646464u, ww[i], 0x04030402u);
                a = dot2(lo, xx[2 * i], a);
                a = dot2(hi, xx[2 * i + 1], a);
            }
            const float part = a - (1024.0f + (float)L.z[r]) * sx;
            acc[r] += L.s[r] * part;
        }
    } else {
        const uint4 xv = lds[j * 64 + lane];
#pragma unroll
        for (int r = 0; r < ROWS_PER_WAVE; r++) {
            float a = acc[r];
            a = dot2(L.w[r].x, xv.x, a);
            a = dot2(L.w[r].y, xv.y, a);
            a = dot2(L.w[r].z, xv.z, a);
            a = dot2(L.w[r].w, xv.w, a);
            acc[r] = a;
        }
    }
}

__device__ __forceinline__ uint16_t to_half_bits(float f)
{
    return __builtin_bit_cast(uint16_t, (_Float16)f);
}

} // namespace

#endif
