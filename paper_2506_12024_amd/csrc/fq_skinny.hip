// Decode-phase weight-only quantized linear for small batches (2 <= M <= 32):
// y[M][N] = x[M][K] . dequant(W[N][K])^T, dequant = Sec. 2.2 Eq. (3).  Still bound by
// the weight stream (Sec. 4.1), but M multiply-adds per weight no longer fit the
// vector ALUs, so the contraction runs on the matrix cores:
// v_mfma_f32_16x16x32_f16 with A = x (16 batch rows x 32 k) and B = 16 weight rows x
// 32 k, accumulating in binary32.
//
// Streaming side (same as the batch-1 kernel): a wavefront owns RT row tiles of 16
// weight rows; lane (n = lane % 16, c = lane / 16) reads 16 bytes of row n per load
// at byte offset 64 * load + 16 * c -- 32 four-bit codes, 16 eight-bit codes or 8
// halves -- with 128-bit loads, double buffered.  One load of a
// wavefront covers 16 rows x 128 / 64 / 32 k, i.e. 4 / 2 / 1 MFMAs.  Loads are issued
// in pairs (64 * (2 i) and 64 * (2 i + 1)): a load touches only 64 bytes of each row,
// and the two halves of a 128-byte line must be requested back to back or HBM
// delivers the line twice.
//
// Dequantization.  Codes become halves by bit tricks ((w & 0x000F000F) | 0x64006400 is
// the pair (1024 + q0, 1024 + q4); nibbles in bits 4..7 use exponent 0x54 = 64 + q;
// bytes go under 0x64 with v_perm_b32), then one v_pk_add_f16 per register subtracts
// (offset + z): the MFMA operand is the exact integer q - z.  The products are summed
// per quantization group in a zeroed accumulator and folded into the output as
// out += s[n][g] * acc, which is Eq. (3) with the scale factored out of the group.
//
// x is staged through LDS in chunks of 1024 k (512 for more than 16 batch rows) as 16-byte
// blocks of 8 halves, [k block][batch row], for the 4-bit path permuted inside the block to
// the order the unpacking produces (x0 x4 x1 x5 x2 x6 x3 x7).  The scales and zeros of a
// chunk's groups are fetched once per chunk (each lane two groups of its row) and parked in
// a wavefront-private LDS area: fetching them per group would touch 16 cache lines per
// instruction and, with the weights streaming through the same caches, miss every time.
// Both x and the metadata of chunk c + 1 are prefetched into registers while chunk c is
// computed.
//
// Launches with few rows (a single linear of a few thousand rows) use a second kernel further
// down, in which the four wavefronts of a workgroup share one row tile and split K.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fq_internal.h"

namespace {

#define FQ_GLOBAL __attribute__((address_space(1)))

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int WG_THREADS = 256;
constexpr int WAVES = WG_THREADS / 64;
constexpr int KU = 2; // consecutive 64-byte loads per row issued together (one 128-byte line)

// k per LDS chunk of x: 1024 for up to 16 batch rows, 512 for up to 32 (32 KiB either way), staged
// by the whole workgroup.  SK (K split, below): 256 k, staged by one wavefront for itself.
template <int MT, bool SK = false>
struct Chunk {
    static constexpr int KC = SK ? 256 : 1024 / MT;
    static constexpr int STAGERS = SK ? 64 : WG_THREADS; // threads that stage one chunk
    static constexpr int GROUPS = KC / 128;              // quantization groups per chunk
    static constexpr int GPL = GROUPS >= 4 ? GROUPS / 4 : 1; // groups whose scale/zero one lane fetches
    static constexpr int XPER = 16 * MT * (KC / 8) / STAGERS; // 16-byte x blocks per thread
    static __device__ __forceinline__ int tid() { return SK ? (int)(threadIdx.x & 63) : (int)threadIdx.x; }
};

__device__ __forceinline__ uint4 load16_weights(const void *p)
{
    // plain (cached) load: a wavefront load touches half of each 128-byte line, the partner
    // load that follows finds the line on its way
    const u32x4 v = *(const FQ_GLOBAL u32x4 *)p;
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint4 load16_global(const void *p)
{
    const u32x4 v = *(const FQ_GLOBAL u32x4 *)p;
    return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ uint32_t pk_add(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2_t, a) + __builtin_bit_cast(half2_t, b));
}

struct Sel {
    const uint8_t *codes;
    const float *scales;
    const uint8_t *zeros;
    int N, K;
};

template <int RT>
struct Loaded { // one step of weights: RT row tiles x KU loads
    uint4 w[RT][KU];
};

template <int MT, int RT, class C = Chunk<MT>>
struct Staged { // what a lane prefetches for the next chunk
    uint4 x[C::XPER];
    float s[RT][C::GPL];
    uint32_t z[RT][C::GPL];
};

// Issue step `st`: loads 2 st and 2 st + 1 of every row tile.
template <int BITS, int RT>
__device__ __forceinline__ void issue(const Sel &d, int wave_row0, int st, int nload, Loaded<RT> &L)
{
    const int lane = threadIdx.x & 63, n = lane & 15, c = lane >> 4;
    const uint32_t K = (uint32_t)d.K;
    const uint32_t row_bytes = BITS == 2 ? (K >> 2) : BITS == 3 ? (K >> 3) * 3 : BITS == 4 ? (K >> 1) : (BITS == 8 ? K : 2 * K);
#pragma unroll
    for (int rt = 0; rt < RT; rt++) {
        const uint32_t row = (uint32_t)min(wave_row0 + rt * 16 + n, d.N - 1);
#pragma unroll
        for (int ku = 0; ku < KU; ku++) {
            // an odd number of loads (4-bit, K / 128 odd): the missing one re-reads the last
            const uint32_t li = (uint32_t)min(st * KU + ku, nload - 1);
            if (BITS == 2) {
                // 64 bytes of a row are two quantization groups: the lane takes 8 bytes (32 codes) of
                // either, so that the four lanes of a row supply whole groups to the MFMAs.  A row
                // may end after the first group (K / 128 odd): the second piece then re-reads the
                // first (its x is zero).
                const uint8_t *p = d.codes + (size_t)row * row_bytes + li * 64 + c * 8;
                const uint32_t second = li * 64 + 32 < row_bytes ? 32u : 0u;
                typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                const u32x2 a = *(const FQ_GLOBAL u32x2 *)p, b = *(const FQ_GLOBAL u32x2 *)(p + second);
                L.w[rt][ku] = make_uint4(a.x, a.y, b.x, b.y);
            } else if (BITS == 3) {
                // a load is one quantization group: the four lanes of a row take its four blocks of
                // 12 bytes (32 codes each), 48 consecutive bytes of the row
                typedef uint32_t u32x3 __attribute__((ext_vector_type(3)));
                typedef u32x3 u32x3_a4 __attribute__((aligned(4)));
                const u32x3 a = *(const FQ_GLOBAL u32x3_a4 *)(d.codes + (size_t)row * row_bytes + (li * 4 + c) * 12);
                L.w[rt][ku] = make_uint4(a.x, a.y, a.z, 0u);
            } else {
                L.w[rt][ku] = load16_weights(d.codes + (size_t)row * row_bytes + li * 64 + c * 16);
            }
        }
    }
}

// Which 16-byte block of a chunk of x (batch row m, k block kb) a thread stages as its block `it`:
// consecutive threads take consecutive k of one row; at 3 bits consecutive runs of four blocks
// (32 k, one block of codes), a thread's blocks 4 u .. 4 u + 3 being one run.
template <int BITS, class C>
__device__ __forceinline__ void x_block(int it, int &m, int &kb)
{
    constexpr int BLK = C::KC / 8;
    if (BITS == 3) {
        static_assert(C::XPER % 4 == 0, "a thread stages whole runs of four blocks");
        const int idx = (it >> 2) * C::STAGERS + C::tid();
        m = idx / (BLK / 4);
        kb = (idx % (BLK / 4)) * 4 + (it & 3);
    } else {
        const int idx = it * C::STAGERS + C::tid();
        m = idx / BLK;
        kb = idx % BLK;
    }
}

// Prefetch chunk `ch` of x (this thread's blocks) and the scales / zeros of the chunk's groups
// for this wavefront's rows: lane (n, c) fetches groups c * GPL .. of row n, so the 16 rows'
// lines are touched once per chunk instead of once per group.
template <int BITS, int MT, int RT, class C = Chunk<MT>>
__device__ __forceinline__ void prefetch_chunk(const Sel &d, const uint16_t *x, int M, int wave_row0,
                                               int ch, Staged<MT, RT, C> &S)
{
    const int kc = ch * C::KC;
#pragma unroll
    for (int it = 0; it < C::XPER; it++) {
        int m, kb;
        x_block<BITS, C>(it, m, kb);
        // rows past M and k past K are clamped: those blocks only feed outputs that are
        // never stored (rows) or are never read (k)
        const int mc = min(m, M - 1), k = min(kc + kb * 8, d.K - 8);
        S.x[it] = load16_global(x + (size_t)mc * d.K + k);
        if (BITS == 2 && kc + kb * 8 >= d.K) // 2 bits: the second group of a last load may lie past K
            S.x[it] = make_uint4(0, 0, 0, 0);
    }
    if (BITS != 16) {
        const int lane = threadIdx.x & 63, n = lane & 15, c = lane >> 4;
        const int G = d.K >> 7;
#pragma unroll
        for (int rt = 0; rt < RT; rt++) {
            const size_t row = (size_t)min(wave_row0 + rt * 16 + n, d.N - 1);
#pragma unroll
            for (int j = 0; j < C::GPL; j++) {
                // (fewer than four groups in a chunk: the lanes past them fetch the last one again)
                const int g = min(ch * C::GROUPS + min(c * C::GPL + j, C::GROUPS - 1), G - 1);
                S.s[rt][j] = ((const FQ_GLOBAL float *)d.scales)[row * G + g];
                S.z[rt][j] = ((const FQ_GLOBAL uint8_t *)d.zeros)[row * G + g];
            }
        }
    }
}

// Write a prefetched chunk to LDS: x blocks [k block][16 * MT rows] (4-bit: permuted to the
// unpack order), scales and zeros into the wavefront's own area as [row tile][group][row].
template <int BITS, int MT, int RT, class C = Chunk<MT>>
__device__ __forceinline__ void commit_chunk(const Staged<MT, RT, C> &S, uint4 *lds_x, float *ms, uint8_t *mz)
{
    constexpr int ROWS = 16 * MT;
    if (BITS == 3) {
        // The 32 k of a lane's block of codes reach the MFMAs as 16 pairs in the order the unpacking
        // meets them (pair 5 j + p = (x[10 j + p], x[10 j + 5 + p]), pair 15 = (x[30], x[31])), four
        // pairs to an operand: a thread holds all four blocks of such a run and regroups them.
#pragma unroll
        for (int u4 = 0; u4 < C::XPER / 4; u4++) {
            int m, kb;
            x_block<BITS, C>(4 * u4, m, kb);
            uint32_t w[16];
#pragma unroll
            for (int q = 0; q < 4; q++) {
                w[4 * q + 0] = S.x[4 * u4 + q].x;
                w[4 * q + 1] = S.x[4 * u4 + q].y;
                w[4 * q + 2] = S.x[4 * u4 + q].z;
                w[4 * q + 3] = S.x[4 * u4 + q].w;
            }
#pragma unroll
            for (int q = 0; q < 4; q++) {
                uint32_t o[4];
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    const int u = 4 * q + i;
                    const int a = u < 15 ? 10 * (u / 5) + u % 5 : 30, b = u < 15 ? a + 5 : 31; // the pair (x[a], x[b])
                    const uint32_t sel = ((b & 1) ? 0x07060000u : 0x05040000u) | ((a & 1) ? 0x0302u : 0x0100u);
                    o[i] = __builtin_amdgcn_perm(w[b >> 1], w[a >> 1], sel);
                }
                lds_x[(kb + q) * ROWS + m] = make_uint4(o[0], o[1], o[2], o[3]);
                asm volatile("" ::: "memory"); // one block at a time: the regrouped words are not all held at once
            }
        }
    }
#pragma unroll
    for (int it = 0; it < (BITS == 3 ? 0 : C::XPER); it++) {
        int m, kb;
        x_block<BITS, C>(it, m, kb);
        uint4 p = S.x[it];
        if (BITS == 2) {
            // Blocks kb (A = x0..7) and kb + 1 (B = x8..15) of 16 consecutive k, held by
            // neighbouring lanes, are stored interleaved -- (A0 B0 A1 B1 A2 B2 A3 B3) at kb,
            // (A4 B4 .. A7 B7) at kb + 1 -- the order in which a word of 16 two-bit codes unpacks.
            const bool odd = kb & 1;
            const uint32_t give0 = odd ? S.x[it].x : S.x[it].z, give1 = odd ? S.x[it].y : S.x[it].w;
            const uint32_t got0 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)give0, 0xB1, 0xF, 0xF, false);
            const uint32_t got1 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)give1, 0xB1, 0xF, 0xF, false);
            const uint32_t a0 = odd ? got0 : S.x[it].x, a1 = odd ? got1 : S.x[it].y; // words of A
            const uint32_t b0 = odd ? S.x[it].z : got0, b1 = odd ? S.x[it].w : got1; // words of B
            p.x = __builtin_amdgcn_perm(b0, a0, 0x05040100u);
            p.y = __builtin_amdgcn_perm(b0, a0, 0x07060302u);
            p.z = __builtin_amdgcn_perm(b1, a1, 0x05040100u);
            p.w = __builtin_amdgcn_perm(b1, a1, 0x07060302u);
        }
        if (BITS == 4) {
            p.x = __builtin_amdgcn_perm(S.x[it].z, S.x[it].x, 0x05040100u); // (x0, x4)
            p.y = __builtin_amdgcn_perm(S.x[it].z, S.x[it].x, 0x07060302u); // (x1, x5)
            p.z = __builtin_amdgcn_perm(S.x[it].w, S.x[it].y, 0x05040100u); // (x2, x6)
            p.w = __builtin_amdgcn_perm(S.x[it].w, S.x[it].y, 0x07060302u); // (x3, x7)
        }
        lds_x[kb * ROWS + m] = p;
    }
    if (BITS != 16) {
        const int lane = threadIdx.x & 63, n = lane & 15, c = lane >> 4;
#pragma unroll
        for (int rt = 0; rt < RT; rt++)
#pragma unroll
            for (int j = 0; j < C::GPL; j++) {
                const int gl = c * C::GPL + j; // group inside the chunk
                if (gl < C::GROUPS) {
                    ms[(rt * C::GROUPS + gl) * 16 + n] = S.s[rt][j];
                    mz[(rt * C::GROUPS + gl) * 16 + n] = (uint8_t)S.z[rt][j];
                }
            }
    }
}

__device__ __forceinline__ float4_t mfma(uint4 a, const uint32_t (&b)[4], float4_t c)
{
    const u32x4 av = {a.x, a.y, a.z, a.w};
    const u32x4 bv = {b[0], b[1], b[2], b[3]};
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, av),
                                                  __builtin_bit_cast(half8_t, bv), c, 0, 0, 0);
}

// 2 bits: one load's worth of work.  The lane holds 32 codes of each of the load's two groups
// (words 0, 1 and words 2, 3); a word of 16 codes unpacks into two MFMA operands, (q0 q8 q1 q9 q2
// q10 q3 q11) and (q4 q12 .. q7 q15): a 2-bit field at bits 0 / 2 / 4 / 6 of a half reads as 1024 + q
// / 256 + q / 64 + q / 16 + q under the exponents 0x64 / 0x5C / 0x54 / 0x4C, and one v_pk_add_f16 per
// register removes offset and zero point.  x is staged in the matching interleaved order.
template <int MT, int RT, int ku>
__device__ __forceinline__ void compute2(int st, const Loaded<RT> &L, const uint4 *lds_x, const float *ms,
                                         const uint8_t *mz, float4_t (&acc)[RT][MT], float4_t (&out)[RT][MT])
{
    typedef Chunk<MT> C;
    constexpr int ROWS = 16 * MT;
    constexpr int KPL = 256, LPC = C::KC / KPL;
    const int li = st * KU + ku;
    const int lane = threadIdx.x & 63, m = lane & 15, c = lane >> 4;
    const int lc = li % LPC; // load inside the chunk
    uint32_t m0 = 0x64006400u, m1 = 0x5C005C00u, m2 = 0x54005400u, m3 = 0x4C004C00u;
    asm volatile("" : "+v"(m0), "+v"(m1), "+v"(m2), "+v"(m3));
#pragma unroll
    for (int g2 = 0; g2 < 2; g2++) { // the load's two groups
        const int gl = lc * 2 + g2;  // group inside the chunk
        const int kk = gl * 128 + c * 32; // lane's first k of it inside the chunk
        float s[RT];
        uint32_t nz[RT][4];
#pragma unroll
        for (int rt = 0; rt < RT; rt++) {
            s[rt] = ms[(rt * C::GROUPS + gl) * 16 + m];
            const uint32_t z = mz[(rt * C::GROUPS + gl) * 16 + m]; // 0 .. 3
            const uint32_t zz = z | (z << 16);
            nz[rt][0] = zz | 0xE400E400u;        // -(1024 + z) twice
            nz[rt][1] = (zz << 2) | 0xDC00DC00u; // -( 256 + z)
            nz[rt][2] = (zz << 4) | 0xD400D400u; // -(  64 + z)
            nz[rt][3] = (zz << 6) | 0xCC00CC00u; // -(  16 + z)
        }
#pragma unroll
        for (int i = 0; i < 2; i++)     // word of the group
#pragma unroll
            for (int h = 0; h < 2; h++) { // codes 0..3 + 8..11, or 4..7 + 12..15 of the word
                uint4 a[MT];
#pragma unroll
                for (int mt = 0; mt < MT; mt++)
                    a[mt] = lds_x[((kk >> 3) + 2 * i + h) * ROWS + mt * 16 + m];
#pragma unroll
                for (int rt = 0; rt < RT; rt++) {
                    const uint32_t ww[4] = {L.w[rt][ku].x, L.w[rt][ku].y, L.w[rt][ku].z, L.w[rt][ku].w};
                    const uint32_t v = h ? (ww[2 * g2 + i] >> 8) : ww[2 * g2 + i];
                    uint32_t b[4];
                    b[0] = pk_add((v & 0x00030003u) | m0, nz[rt][0]);
                    b[1] = pk_add((v & 0x000C000Cu) | m1, nz[rt][1]);
                    b[2] = pk_add((v & 0x00300030u) | m2, nz[rt][2]);
                    b[3] = pk_add((v & 0x00C000C0u) | m3, nz[rt][3]);
#pragma unroll
                    for (int mt = 0; mt < MT; mt++)
                        acc[rt][mt] = mfma(a[mt], b, acc[rt][mt]);
                }
            }
#pragma unroll
        for (int rt = 0; rt < RT; rt++)
#pragma unroll
            for (int mt = 0; mt < MT; mt++) {
                out[rt][mt] += s[rt] * acc[rt][mt];
                acc[rt][mt] = float4_t{0.f, 0.f, 0.f, 0.f};
            }
    }
}

// One load's worth of work: dequantize, multiply with the staged x, fold finished groups.
template <int BITS, int MT, int RT, int ku, class C = Chunk<MT>>
__device__ __forceinline__ void compute(int st, const Loaded<RT> &L, const uint4 *lds_x, const float *ms,
                                        const uint8_t *mz, float4_t (&acc)[RT][MT],
                                        float4_t (&out)[RT][MT])
{
    constexpr int ROWS = 16 * MT;
    constexpr int KPL = BITS == 4 || BITS == 3 ? 128 : (BITS == 8 ? 64 : 32); // k per load
    constexpr int NM = KPL / 32;                                 // MFMAs per load
    constexpr int LPC = C::KC / KPL;                             // loads per chunk
    const int li = st * KU + ku;
    const int lane = threadIdx.x & 63, m = lane & 15, c = lane >> 4;
    const int lc = li % LPC;                      // load inside the chunk
    const int kk = lc * KPL + c * (KPL / 4);      // lane's first k inside the chunk
    const int gl = (lc * KPL) >> 7;               // group inside the chunk
    uint32_t magic_lo = 0x64006400u, magic_hi = 0x54005400u;
    asm volatile("" : "+v"(magic_lo), "+v"(magic_hi));

    float s[RT];
    uint32_t z[RT];
    if (BITS != 16) {
#pragma unroll
        for (int rt = 0; rt < RT; rt++) {
            s[rt] = ms[(rt * C::GROUPS + gl) * 16 + m];
            z[rt] = mz[(rt * C::GROUPS + gl) * 16 + m];
        }
    }
#pragma unroll
    for (int i = 0; i < NM; i++) {
        uint4 a[MT];
#pragma unroll
        for (int mt = 0; mt < MT; mt++)
            a[mt] = lds_x[((kk >> 3) + i) * ROWS + mt * 16 + m];
#pragma unroll
        for (int rt = 0; rt < RT; rt++) {
            const uint32_t ww[4] = {L.w[rt][ku].x, L.w[rt][ku].y, L.w[rt][ku].z, L.w[rt][ku].w};
            uint32_t b[4];
            if (BITS == 3) {
                // Word j of the block holds the codes 10 j + 5 h + p (h: the word's halves, p = 0 .. 4:
                // bits 3 p .. 3 p + 2 of the half); a field at bit 0 / 3 / 6 of a half reads as 1024 + q /
                // 128 + q / 16 + q under the exponents 0x64 / 0x58 / 0x4C, the fields p = 3, 4 after a
                // shift by 9 bits.  Bit 15 of the halves of word j is bit j of the codes 30 and 31:
                // after that shift it sits at bit 6, worth 1 / 2 / 4 under the exponents of 16 / 32 /
                // 64, and the three add up to 112 + q exactly.  Pair 5 j + p is the operand's k, four
                // pairs to an MFMA (x is staged in that order).
                const uint32_t zz = z[rt] | (z[rt] << 16);
                const uint32_t nz0 = zz | 0xE400E400u, nz1 = (zz << 3) | 0xD800D800u, nz2 = (zz << 6) | 0xCC00CC00u;
                const uint32_t M0 = 0x00070007u, M1 = 0x00380038u, M2 = 0x01C001C0u;
                const uint32_t e0 = 0x64006400u, e1 = 0x58005800u, e2 = 0x4C004C00u;
                auto pair = [&](int j, int p) -> uint32_t {
                    const uint32_t v = p < 3 ? ww[j] : ww[j] >> 9;
                    const int f = p < 3 ? p : p - 3;
                    return f == 0   ? pk_add((v & M0) | e0, nz0)
                           : f == 1 ? pk_add((v & M1) | e1, nz1)
                                    : pk_add((v & M2) | e2, nz2);
                };
                if (i == 0) {
                    b[0] = pair(0, 0);
                    b[1] = pair(0, 1);
                    b[2] = pair(0, 2);
                    b[3] = pair(0, 3);
                } else if (i == 1) {
                    b[0] = pair(0, 4);
                    b[1] = pair(1, 0);
                    b[2] = pair(1, 1);
                    b[3] = pair(1, 2);
                } else if (i == 2) {
                    b[0] = pair(1, 3);
                    b[1] = pair(1, 4);
                    b[2] = pair(2, 0);
                    b[3] = pair(2, 1);
                } else {
                    b[0] = pair(2, 2);
                    b[1] = pair(2, 3);
                    b[2] = pair(2, 4);
                    const uint32_t t0 = ((ww[0] >> 9) & 0x00400040u) | 0x4C004C00u; // 16 + bit 0
                    const uint32_t t1 = ((ww[1] >> 9) & 0x00400040u) | 0x50005000u; // 32 + 2 bit 1
                    const uint32_t t2 = ((ww[2] >> 9) & 0x00400040u) | 0x54005400u; // 64 + 4 bit 2
                    b[3] = pk_add(pk_add(pk_add(t0, t1), t2), (zz << 4) | 0xD700D700u); // - (112 + z)
                }
            } else if (BITS == 4) {
                const uint32_t nz_lo = (z[rt] | (z[rt] << 16)) | 0xE400E400u;        // -(1024 + z) twice
                const uint32_t nz_hi = ((z[rt] << 4) | (z[rt] << 20)) | 0xD400D400u; // -(  64 + z) twice
                const uint32_t v = ww[i], v8 = v >> 8;
                b[0] = pk_add((v & 0x000F000Fu) | magic_lo, nz_lo);  // (q0 - z, q4 - z)
                b[1] = pk_add((v & 0x00F000F0u) | magic_hi, nz_hi);  // (q1 - z, q5 - z)
                b[2] = pk_add((v8 & 0x000F000Fu) | magic_lo, nz_lo); // (q2 - z, q6 - z)
                b[3] = pk_add((v8 & 0x00F000F0u) | magic_hi, nz_hi); // (q3 - z, q7 - z)
            } else if (BITS == 8) {
                const uint32_t nz = (z[rt] | (z[rt] << 16)) | 0xE400E400u;
#pragma unroll
                for (int h = 0; h < 2; h++) {
                    const uint32_t v = ww[2 * i + h];
                    b[2 * h + 0] = pk_add(__builtin_amdgcn_perm(0x64646464u, v, 0x04010400u), nz);
                    b[2 * h + 1] = pk_add(__builtin_amdgcn_perm(0x64646464u, v, 0x04030402u), nz);
                }
            } else {
#pragma unroll
                for (int q = 0; q < 4; q++)
                    b[q] = ww[q];
            }
#pragma unroll
            for (int mt = 0; mt < MT; mt++)
                acc[rt][mt] = mfma(a[mt], b, acc[rt][mt]);
        }
    }
    // group complete: 3- and 4-bit after every load, 8-bit after every second load
    constexpr bool group_end = BITS == 4 || BITS == 3 || (BITS == 8 && ku == 1);
    if (group_end) {
#pragma unroll
        for (int rt = 0; rt < RT; rt++)
#pragma unroll
            for (int mt = 0; mt < MT; mt++) {
                out[rt][mt] += s[rt] * acc[rt][mt];
                acc[rt][mt] = float4_t{0.f, 0.f, 0.f, 0.f};
            }
    }
}

template <int BITS, int MT, int RT>
__device__ __forceinline__ void run_tile(const Sel &d, const uint16_t *x, uint16_t *y, int M,
                                         int wave_row0, uint4 *lds_x, float *ms, uint8_t *mz)
{
    typedef Chunk<MT> C;
    constexpr int KPL = BITS == 2 ? 256 : BITS == 4 || BITS == 3 ? 128 : (BITS == 8 ? 64 : 32);
    constexpr int SPC = C::KC / KPL / KU; // steps per chunk
    const int nload = (d.K + KPL - 1) / KPL; // 2 bits: a last load may hold one group only
    const int nstep = (nload + KU - 1) / KU;
    const int nchunk = (d.K + C::KC - 1) / C::KC;
    const int lane = threadIdx.x & 63, n = lane & 15, c = lane >> 4;
    float4_t acc[RT][MT], out[RT][MT];
#pragma unroll
    for (int rt = 0; rt < RT; rt++)
#pragma unroll
        for (int mt = 0; mt < MT; mt++) {
            acc[rt][mt] = float4_t{0.f, 0.f, 0.f, 0.f};
            out[rt][mt] = float4_t{0.f, 0.f, 0.f, 0.f};
        }
    Loaded<RT> A, B;
    Staged<MT, RT> S;
    issue<BITS, RT>(d, wave_row0, 0, nload, A);
    prefetch_chunk<BITS, MT, RT>(d, x, M, wave_row0, 0, S);
    auto step = [&](int st, Loaded<RT> &Lcur, Loaded<RT> &Lnext) {
        // Always issued (the last step re-reads its own item) so that the wait for Lcur can
        // be a counted vmcnt with Lnext's loads still in flight.
        issue<BITS, RT>(d, wave_row0, min(st + 1, nstep - 1), nload, Lnext);
        if (st % SPC == 0) {
            const int ch = st / SPC;
            __syncthreads(); // all wavefronts are done with the previous chunk of x
            commit_chunk<BITS, MT, RT>(S, lds_x, ms, mz);
            __syncthreads();
            // next chunk's x and metadata travel while this chunk is computed
            prefetch_chunk<BITS, MT, RT>(d, x, M, wave_row0, min(ch + 1, nchunk - 1), S);
        }
        if (BITS == 2) {
            compute2<MT, RT, 0>(st, Lcur, lds_x, ms, mz, acc, out);
            if (st * KU + 1 < nload)
                compute2<MT, RT, 1>(st, Lcur, lds_x, ms, mz, acc, out);
        } else {
            compute<BITS, MT, RT, 0>(st, Lcur, lds_x, ms, mz, acc, out);
            if (st * KU + 1 < nload)
                compute<BITS, MT, RT, 1>(st, Lcur, lds_x, ms, mz, acc, out);
        }
    };
    for (int st = 0; st < nstep; st += 2) {
        step(st, A, B);
        if (st + 1 < nstep)
            step(st + 1, B, A);
    }
    // D layout of the 16x16 MFMA: lane holds column n = lane % 16, rows 4 * (lane / 16) + r.
#pragma unroll
    for (int rt = 0; rt < RT; rt++) {
        const int row = wave_row0 + rt * 16 + n;
#pragma unroll
        for (int mt = 0; mt < MT; mt++) {
            const float4_t v = BITS == 16 ? acc[rt][mt] : out[rt][mt];
#pragma unroll
            for (int r = 0; r < 4; r++) {
                const int m = mt * 16 + c * 4 + r;
                if (m < M && row < d.N)
                    ((FQ_GLOBAL uint16_t *)y)[(size_t)m * d.N + row] =
                        __builtin_bit_cast(uint16_t, (_Float16)v[r]);
            }
        }
    }
}

// ---- K split: launches with few rows ------------------------------------------------------
// A single linear has only N / 64 tiles of the kind above, far too few wavefronts to keep HBM busy
// (4096 rows: 64 workgroups).  Here a workgroup owns one row tile of 16 rows and its four
// wavefronts split K between them: wavefront w takes the chunks of 256 k with index w, w + 4, ...,
// stages its own x and metadata in its own part of LDS (ordered by the wavefront's own instruction
// stream: no workgroup barrier), and the four partial results meet in LDS at the end.  4, 8 and 16
// bits (a 2-bit step is 512 k: those launches use the tiles above).
template <int BITS, int MT>
__device__ __forceinline__ void run_tile_sk(const Sel &d, const uint16_t *x, uint16_t *y, int M, int row0,
                                            int wave, uint4 *lds_x, float *ms, uint8_t *mz, float4_t *red)
{
    typedef Chunk<MT, true> C;
    constexpr int RT = 1;
    constexpr int KPL = BITS == 4 || BITS == 3 ? 128 : (BITS == 8 ? 64 : 32);
    constexpr int SPC = C::KC / KPL / KU; // steps per chunk: 1 / 2 / 4
    const int nload = d.K / KPL;
    const int nstep = (nload + KU - 1) / KU;
    const int nchunk = (d.K + C::KC - 1) / C::KC;
    const int lane = threadIdx.x & 63, n = lane & 15, c = lane >> 4;
    float4_t acc[RT][MT], out[RT][MT];
#pragma unroll
    for (int mt = 0; mt < MT; mt++) {
        acc[0][mt] = float4_t{0.f, 0.f, 0.f, 0.f};
        out[0][mt] = float4_t{0.f, 0.f, 0.f, 0.f};
    }
    Loaded<RT> A, B;
    Staged<MT, RT, C> S;
    int ch = wave, j = 0; // the wavefront's current chunk and step inside it
    if (ch < nchunk) {
        issue<BITS, RT>(d, row0, ch * SPC, nload, A);
        prefetch_chunk<BITS, MT, RT, C>(d, x, M, row0, ch, S);
    }
    // One step; returns false after the wavefront's last one.
    auto step = [&](Loaded<RT> &Lcur, Loaded<RT> &Lnext) -> bool {
        const int st = ch * SPC + j;
        int nch = ch, nj = j + 1;
        if (nj == SPC || ch * SPC + nj >= nstep) {
            nch = ch + WAVES;
            nj = 0;
        }
        const bool more = nch < nchunk;
        // Always issued (after the last step it re-reads its own item) so that the wait for Lcur
        // can be a counted vmcnt with Lnext's loads still in flight.
        issue<BITS, RT>(d, row0, more ? nch * SPC + nj : st, nload, Lnext);
        if (j == 0) {
            // the wavefront's LDS accesses execute in order: its reads of the previous chunk are
            // done before these writes, and the reads below see them
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            commit_chunk<BITS, MT, RT, C>(S, lds_x, ms, mz);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            prefetch_chunk<BITS, MT, RT, C>(d, x, M, row0, min(ch + WAVES, nchunk - 1), S);
        }
        compute<BITS, MT, RT, 0, C>(st, Lcur, lds_x, ms, mz, acc, out);
        if (st * KU + 1 < nload)
            compute<BITS, MT, RT, 1, C>(st, Lcur, lds_x, ms, mz, acc, out);
        ch = nch;
        j = nj;
        return more;
    };
    if (ch < nchunk) {
        for (;;) {
            if (!step(A, B))
                break;
            if (!step(B, A))
                break;
        }
    }
    // the four partial results: wavefronts 1..3 park theirs, wavefront 0 adds them up and stores
#pragma unroll
    for (int mt = 0; mt < MT; mt++) {
        const float4_t v = BITS == 16 ? acc[0][mt] : out[0][mt];
        if (wave > 0)
            red[((wave - 1) * MT + mt) * 64 + lane] = v;
    }
    __syncthreads();
    if (wave == 0) {
        // D layout of the 16x16 MFMA: lane holds column n = lane % 16, rows 4 * (lane / 16) + r.
        const int row = row0 + n;
#pragma unroll
        for (int mt = 0; mt < MT; mt++) {
            float4_t v = BITS == 16 ? acc[0][mt] : out[0][mt];
#pragma unroll
            for (int w = 0; w < WAVES - 1; w++)
                v += red[(w * MT + mt) * 64 + lane];
#pragma unroll
            for (int r = 0; r < 4; r++) {
                const int m = mt * 16 + c * 4 + r;
                if (m < M && row < d.N)
                    ((FQ_GLOBAL uint16_t *)y)[(size_t)m * d.N + row] = __builtin_bit_cast(uint16_t, (_Float16)v[r]);
            }
        }
    }
    __syncthreads(); // `red` is free again
}

// W3: with the 3-bit path (its unpacking and the regrouping of x cost registers: a launch that cannot
// meet a 3-bit entry runs the instance without)
template <bool SINGLE, int MT, bool W3>
__global__ __launch_bounds__(WG_THREADS) void decode_skinny_sk_kernel(const FqLinearDesc single, int bits_host,
                                                                      const FqLinearDesc *__restrict__ table,
                                                                      const int32_t *__restrict__ bits_dev,
                                                                      int count, int total_tiles, int M, int *flags)
{
    typedef Chunk<MT, true> C;
    __shared__ uint4 lds_x[WAVES][(C::KC / 8) * 16 * MT];
    __shared__ float lds_s[WAVES][C::GROUPS * 16];
    __shared__ uint8_t lds_z[WAVES][C::GROUPS * 16];
    __shared__ float4_t red[(WAVES - 1) * MT * 64];
    const int wave = threadIdx.x >> 6;
    int e = 0;
    for (int tile = blockIdx.x; tile < total_tiles; tile += gridDim.x) {
        const FqLinearDesc *dp;
        int bits;
        if (SINGLE) {
            dp = &single;
            bits = bits_host;
        } else {
            while (e + 1 < count && tile >= table[e + 1].tile_begin)
                e++;
            dp = &table[e];
            bits = bits_dev[e];
        }
        Sel d;
        d.N = dp->N;
        d.K = dp->K;
        d.codes = bits == 3    ? (W3 ? dp->codes3 : nullptr)
                  : bits == 4  ? dp->codes4
                  : bits == 8  ? dp->codes8
                  : bits == 16 ? (const uint8_t *)dp->w16
                               : nullptr;
        d.scales = bits == 3 ? dp->scales3 : bits == 4 ? dp->scales4 : dp->scales8;
        d.zeros = bits == 3 ? dp->zeros3 : bits == 4 ? dp->zeros4 : dp->zeros8;
        if (!d.codes) { // uniform over the workgroup
            if (flags && threadIdx.x == 0)
                *flags = 1; // no such width here, or no copy of it: nobody runs this entry
            continue;
        }
        const int row0 = (tile - dp->tile_begin) * 16;
        if (W3 && bits == 3)
            run_tile_sk<3, MT>(d, dp->x, dp->y, M, row0, wave, lds_x[wave], lds_s[wave], lds_z[wave], red);
        else if (bits == 4)
            run_tile_sk<4, MT>(d, dp->x, dp->y, M, row0, wave, lds_x[wave], lds_s[wave], lds_z[wave], red);
        else if (bits == 8)
            run_tile_sk<8, MT>(d, dp->x, dp->y, M, row0, wave, lds_x[wave], lds_s[wave], lds_z[wave], red);
        else
            run_tile_sk<16, MT>(d, dp->x, dp->y, M, row0, wave, lds_x[wave], lds_s[wave], lds_z[wave], red);
    }
}

template <bool SINGLE, int MT, int RT, bool W3>
__global__ __launch_bounds__(WG_THREADS) void decode_skinny_kernel(const FqLinearDesc single,
                                                                   int bits_host,
                                                                   const FqLinearDesc *__restrict__ table,
                                                                   const int32_t *__restrict__ bits_dev,
                                                                   int count, int total_tiles, int M, int *flags)
{
    __shared__ uint4 lds_x[(Chunk<MT>::KC / 8) * 16 * MT];
    __shared__ float lds_s[WAVES][RT * Chunk<MT>::GROUPS * 16];
    __shared__ uint8_t lds_z[WAVES][RT * Chunk<MT>::GROUPS * 16];
    constexpr int TILE_ROWS = WAVES * RT * 16;
    const int wave = threadIdx.x >> 6;
    int e = 0;
    for (int tile = blockIdx.x; tile < total_tiles; tile += gridDim.x) {
        const FqLinearDesc *dp;
        int bits, t; // t: the tile inside its entry
        if (SINGLE) {
            dp = &single;
            bits = bits_host;
            t = tile;
        } else {
            while (e + 1 < count && tile >= table[e + 1].tile_begin)
                e++;
            dp = &table[e];
            bits = bits_dev[e];
            t = tile - dp->tile_begin;
        }
        Sel d;
        d.N = dp->N;
        d.K = dp->K;
        d.codes = bits == 2    ? dp->codes2
                  : bits == 3  ? (W3 ? dp->codes3 : nullptr)
                  : bits == 4  ? dp->codes4
                  : bits == 8  ? dp->codes8
                  : bits == 16 ? (const uint8_t *)dp->w16
                               : nullptr;
        d.scales = bits == 2 ? dp->scales2 : bits == 3 ? dp->scales3 : bits == 4 ? dp->scales4 : dp->scales8;
        d.zeros = bits == 2 ? dp->zeros2 : bits == 3 ? dp->zeros3 : bits == 4 ? dp->zeros4 : dp->zeros8;
        if (!d.codes) { // uniform over the workgroup
            if (flags && threadIdx.x == 0)
                *flags = 1; // no such width here, or no copy of it: nobody runs this entry
            continue;
        }
        // All wavefronts of the workgroup run the tile (rows past N are clamped on load and
        // masked on store) so that every one of them reaches the staging barriers.
        const int wave_row0 = t * TILE_ROWS + wave * RT * 16;
        if (bits == 2)
            run_tile<2, MT, RT>(d, dp->x, dp->y, M, wave_row0, lds_x, lds_s[wave], lds_z[wave]);
        else if (W3 && bits == 3)
            run_tile<3, MT, RT>(d, dp->x, dp->y, M, wave_row0, lds_x, lds_s[wave], lds_z[wave]);
        else if (bits == 4)
            run_tile<4, MT, RT>(d, dp->x, dp->y, M, wave_row0, lds_x, lds_s[wave], lds_z[wave]);
        else if (bits == 8)
            run_tile<8, MT, RT>(d, dp->x, dp->y, M, wave_row0, lds_x, lds_s[wave], lds_z[wave]);
        else
            run_tile<16, MT, RT>(d, dp->x, dp->y, M, wave_row0, lds_x, lds_s[wave], lds_z[wave]);
    }
}

template <int MT, int RT, bool W3>
hipError_t launch(const FqLinearDesc *single, int bits_host, const FqLinearDesc *descs_dev,
                  const int32_t *bits_dev, int count, int total_tiles, int M, int cus,
                  hipStream_t stream, int *flags = nullptr)
{
    const int cap = cus * fq_workgroups_per_cu((const void *)decode_skinny_kernel<false, MT, RT, W3>, WG_THREADS, 0, 2);
    const int grid = total_tiles < cap ? total_tiles : cap;
    if (single) {
        decode_skinny_kernel<true, MT, RT, W3><<<grid, WG_THREADS, 0, stream>>>(*single, bits_host, nullptr,
                                                                               nullptr, 1, total_tiles, M, nullptr);
    } else {
        FqLinearDesc none = {};
        decode_skinny_kernel<false, MT, RT, W3><<<grid, WG_THREADS, 0, stream>>>(none, 0, descs_dev, bits_dev,
                                                                                count, total_tiles, M, flags);
    }
    return hipGetLastError();
}

template <int MT, bool W3>
hipError_t launch_sk(const FqLinearDesc *single, int bits_host, const FqLinearDesc *descs_dev,
                     const int32_t *bits_dev, int count, int total_tiles, int M, int cus, hipStream_t stream,
                     int *flags = nullptr)
{
    const int cap = cus * fq_workgroups_per_cu((const void *)decode_skinny_sk_kernel<false, MT, W3>, WG_THREADS, 0, 2);
    const int grid = total_tiles < cap ? total_tiles : cap;
    if (single) {
        decode_skinny_sk_kernel<true, MT, W3><<<grid, WG_THREADS, 0, stream>>>(*single, bits_host, nullptr, nullptr, 1,
                                                                            total_tiles, M, nullptr);
    } else {
        FqLinearDesc none = {};
        decode_skinny_sk_kernel<false, MT, W3><<<grid, WG_THREADS, 0, stream>>>(none, 0, descs_dev, bits_dev, count,
                                                                             total_tiles, M, flags);
    }
    return hipGetLastError();
}

template <bool W3>
hipError_t launch_any(const FqLinearDesc *single, int bits_host, const FqLinearDesc *descs_dev,
                      const int32_t *bits_dev, int count, int total_tiles, int tile_rows, int M, int cus,
                      hipStream_t stream, int *fl)
{
    const int rt = tile_rows / 64;
    if (tile_rows == 16)
        return M <= 16 ? launch_sk<1, W3>(single, bits_host, descs_dev, bits_dev, count, total_tiles, M, cus, stream, fl)
                       : launch_sk<2, W3>(single, bits_host, descs_dev, bits_dev, count, total_tiles, M, cus, stream, fl);
    if (M <= 16) {
        if (rt == 4)
            return launch<1, 4, W3>(single, bits_host, descs_dev, bits_dev, count, total_tiles, M, cus, stream, fl);
        if (rt == 2)
            return launch<1, 2, W3>(single, bits_host, descs_dev, bits_dev, count, total_tiles, M, cus, stream, fl);
        return launch<1, 1, W3>(single, bits_host, descs_dev, bits_dev, count, total_tiles, M, cus, stream, fl);
    }
    if (rt == 4)
        return launch<2, 4, W3>(single, bits_host, descs_dev, bits_dev, count, total_tiles, M, cus, stream, fl);
    if (rt == 2)
        return launch<2, 2, W3>(single, bits_host, descs_dev, bits_dev, count, total_tiles, M, cus, stream, fl);
    return launch<2, 1, W3>(single, bits_host, descs_dev, bits_dev, count, total_tiles, M, cus, stream, fl);
}

int device_cus() { return fq_device_cus(); }

} // namespace

// Rows per workgroup tile: 64 * RT with RT in {1, 2, 4} row tiles per wavefront, the largest that
// still gives every CU a few tiles; 16 (the K-split kernel) where even 64-row tiles would leave
// CUs without work.
int fq_skinny_tile_rows(long long total_rows, int M)
{
    (void)M;
    const long long want = 4LL * device_cus();
    int rt = 4;
    while (rt > 1 && total_rows / (64 * rt) < want)
        rt >>= 1;
    // (measured at M = 16: 4096 rows 16 -> 8 us with the K split, 11008 rows 16.7 -> 17.3 us)
    if (rt == 1 && total_rows / 64 < device_cus() / 2)
        return 16;
    return 64 * rt;
}

hipError_t fq_launch_skinny(const FqLinearDesc *single, int bits_host,
                            const FqLinearDesc *descs_dev, const int32_t *bits_dev, int count,
                            int total_tiles, int tile_rows, int M, bool with3, int *queue, void *order,
                            hipStream_t stream)
{
    if (total_tiles <= 0)
        return hipSuccess;
    const int cus = device_cus();
    int *fl = !single && queue ? queue + FQ_Q_FLAGS : nullptr;
    if (!single && tile_rows == 256)
        return fq_launch_skinny_stream(descs_dev, bits_dev, count, total_tiles, M, cus, queue, order, stream);
    return with3 ? launch_any<true>(single, bits_host, descs_dev, bits_dev, count, total_tiles, tile_rows, M, cus, stream, fl)
                 : launch_any<false>(single, bits_host, descs_dev, bits_dev, count, total_tiles, tile_rows, M, cus, stream, fl);
}
