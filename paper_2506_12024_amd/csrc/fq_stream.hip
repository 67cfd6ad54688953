// Decode-phase weight-only quantized linear for small batches (2 <= M <= 32), streaming
// kernel for launches with many 256-row tiles: y[M][N] = x[M][K] . dequant(W[N][K])^T,
// dequant = Sec. 2.2 Eq. (3).  The phase is bound by the weight stream (Sec. 4.1); the
// contraction runs on v_mfma_f32_16x16x32_f16 (A = x: 16 batch rows x 32 k, B = 16 weight
// rows x 32 k, binary32 accumulation; two batch tiles above 16 rows).  Launches with few or
// narrow tiles and single calls stay with the register-fed small-batch kernel.
//
// Work split.  A workgroup owns a tile of 256 weight rows and has twelve wavefronts: eight
// consumers (two per SIMD, so that one computes while the other waits), 32 rows = 2 MFMA row
// tiles each, and four loaders.
//
// Weight stream.  A stage is one 128-byte line of each of the consumer's 32 rows (512 / 256 /
// 128 / 64 k at 2 / 4 / 8 / 16 bits); a load instruction covers 8 rows x 128 bytes, whole lines only
// (halves of a line requested apart are fetched from HBM twice more often than not), marked
// non-temporal (read once).  Stages go from global memory straight into a wavefront-private
// LDS ring of two slots with direct-to-LDS loads (global_load_lds_dwordx4): no register
// staging, and the only synchronisation the stream needs is a counted s_waitcnt vmcnt(n) of
// the wavefront on its own loads.  A step waits for its stage, copies it to registers together
// with the x blocks and the scales / zero points it needs, and at once requests the stage two
// steps ahead into the slot it has just emptied: two stages per consumer, 64 KiB per CU, are
// in flight while the step computes (three measured the same: the memory system is the limit,
// not the depth).  These LDS reads are inline assembly: the compiler cannot tell a read of a
// run-time slot from the slots being filled and would wait for every outstanding load first.
// At the end of a tile the slots that the tile has no stage left for take the first stages of
// the workgroup's next tile (whatever its bit-width), so the ring does not run dry across the
// tile boundary.
//
// Loaders.  x and the metadata are what the stream cannot carry: a scale or zero-point fetch
// per stage touches one cache line per row (64 tiny requests per instruction, more than the
// weights themselves need), and the 4-bit path wants x permuted.  Four more wavefronts fetch
// them with ordinary loads -- their own vmcnt, nobody else waits -- in chunks of 512 k, the
// loaders taking the chunks in turn (a load returns behind everything the compute unit has
// requested before it, 64 KiB of weights included, so that a loader turns a chunk round in 4 to
// 5 us; at 4 bits the consumers use one up in 3), each requesting its next chunk as soon as
// it has written one, and its first chunk of the next tile after its last of this one: x as 16-byte
// blocks of 8 halves, one request of 1 KiB per batch row and chunk, stored [k block][batch
// row] with the rows of k block kb XOR-ed by kb % 8 + 8 (kb / 32) -- conflict free for the
// writer, whose lanes are k blocks (a 128-bit LDS write goes eight lanes at a time), and for the
// readers, whose lanes are batch rows (measured: a 128-bit read runs at full rate only if lanes
// 0 .. 7 and 8 .. 15 of every group of 16 lanes use different halves of the 256 bytes and the
// same ones in all four groups, i.e. whatever the k block) -- zero past K, for the
// 4-bit path permuted inside the block to the order the unpacking produces (x0 x4 x1 x5 x2 x6
// x3 x7); scales and zero points for a pair of chunks at a time (8 units: 32 + 8 contiguous
// bytes per row), stored [consumer][row][row tile][unit].  Chunks are handed over through
// counters in LDS, not through barriers (a barrier per chunk, two stages at 4 bits, makes every
// consumer wait for the slowest of the eight and for the loaders each time); the workgroup
// meets at one barrier per tile.
//
// Dequantization.  Codes become halves by bit tricks ((w & 0x000F000F) | 0x64006400 is the
// pair (1024 + q0, 1024 + q4); nibbles in bits 4..7 use exponent 0x54 = 64 + q; bytes go
// under 0x64 with v_perm_b32).  Offsets and zero point come off the operand by one packed fp16
// add per register, -(offset + z) in both halves: the difference is the small integer q - z,
// exact in binary16, so the accumulator holds sum x (q - z) over the stage, which is folded as
// out += s * acc -- Eq. (3) with the scale factored out of the group.  (At 8 bits with one batch
// tile, where the stream is memory-bound and registers are short, the offsets stay in the
// operand and a second MFMA per operand multiplies the same x block by the constant
// -(offset + z) instead; every product is exact in binary32.)  The vector ALUs carry 9
// instructions per 8 four-bit weights.
// At 2 bits a stage is four units; an MFMA's 32 k are 8 bytes of a line, 2 from each group of 16
// lanes, so a lane reads its 8 bytes of every unit (not 16 contiguous ones, which would put two
// units into one MFMA's sum); a byte holds four consecutive codes, which one v_perm_b32 copies to
// both halves of a word and two and-or instructions turn into the pairs (1024 + q0, 256 + q1) and
// (64 + q2, 16 + q3) -- x stays in its natural order -- and the constant that is added carries the
// four offsets by position.  A stage's x is 16 KiB, read from LDS unit by unit.
//
// LDS layout of a weight stage: per row tile 16 lines of 128 bytes, the eight 16-byte slots of
// line n XOR-ed by (n >> 1) & 7 -- a 128-bit read of the 16 rows at one piece is conflict
// free; the permutation is applied on the global side of the load.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fq_internal.h"

namespace {

#define FQ_GLOBAL __attribute__((address_space(1)))
#define FQ_LDS __attribute__((address_space(3)))

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int CONSUMERS = 8;
constexpr int LOADERS = 4;                    // 2 or 4 (a workgroup of twelve wavefronts: three to a SIMD)
constexpr int THREADS = (CONSUMERS + LOADERS) * 64;
constexpr int RT = 2;                         // MFMA row tiles (16 rows) per consumer
constexpr int TILE_ROWS = CONSUMERS * RT * 16;
constexpr int NS = 2;                         // ring slots per consumer (3 measured the same)
constexpr int STAGE_BYTES = RT * 16 * 128;    // 4 KiB of weights per stage
constexpr int SOPS = STAGE_BYTES / 1024;      // direct-to-LDS loads per lane and stage
constexpr int KC = 512;                       // k per chunk of x: one 16-byte block per loader lane and batch row
constexpr int UC = KC / 128;                  // units (quantization groups) per chunk
constexpr int UP = 2 * UC;                    // units per metadata fetch: a pair of chunks
// MT below: batch tiles of 16 rows (1 for M <= 16, 2 for M <= 32); an x buffer is 16 * MT * KC halves
// x buffers: a consumer may be this many chunks minus one ahead of the slowest one (three is
// what the metadata's two buffers of a pair of chunks allow; two batch tiles: LDS holds two)
__host__ __device__ constexpr int nxb(int mt) { return mt == 1 ? 3 : 2; }

// Workgroup barrier without the fence of __syncthreads() (which would wait for every
// outstanding load, i.e. drain the rings); the waits that matter are issued explicitly.
__device__ __forceinline__ void barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

__device__ __forceinline__ uint32_t pk_add_h(uint32_t a, uint32_t b)
{
    typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2_t, a) + __builtin_bit_cast(half2_t, b));
}

__device__ __forceinline__ float4_t mfma(const u32x4 a, const u32x4 b, float4_t c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, a), __builtin_bit_cast(half8_t, b), c,
                                                  0, 0, 0);
}

__device__ __forceinline__ uint32_t lds_addr(const void *p)
{
    return (uint32_t)(uintptr_t)(const FQ_LDS void *)p;
}

struct Sel {
    const uint8_t *codes;
    const float *scales;
    const uint8_t *zeros;
    const uint16_t *x;
    uint16_t *y;
    int N, K;
};

// The workgroup's LDS.  Metadata buffers come in pairs (parity of the pair of chunks).
struct Lds {
    uint8_t *ring;    // [CONSUMERS][NS][STAGE_BYTES]
    uint8_t *x;       // nxb(MT) buffers of [KC / 8][16 * MT] blocks of 16 bytes; k block kb holds batch row m at place m ^ (kb % 8 + 8 (kb / 32))
    float *ms[2];     // [CONSUMERS][16 rows][RT][UP] scales of a pair of chunks
    uint8_t *mz[2];   // same order, zero points
    int *flag;        // hand-over counters: [li] chunks written by loader li, [4] tiles drawn, [8 + w] chunks finished by consumer w
    int *mail;        // two tile records of 16 words, used in turn
};

// What a consumer has requested of its next tile while it finished the current one: the first
// `pf` stages, stage s in ring slot (slot0 + s) % NS.
struct Ahead {
    int pf, slot0;
};

typedef int int2_t __attribute__((ext_vector_type(2)));

// Hand-over of the x and metadata chunks between the loaders and the consumers without a
// workgroup barrier (a barrier per chunk, every two stages at 4 bits, makes each consumer wait
// for the slowest of the eight twice per 512 k).  Counters in LDS that only grow, chunks numbered
// through the tiles of the launch: loader li stores 1 + the number of the last chunk it has
// written, consumer w stores 1 + the number of the last chunk it has finished reading.  A
// wavefront's LDS operations are carried out in the order it issues them, and each side has
// waited for its own before it writes its counter.  The consumers' side is inline assembly for
// the same reason as take().
__device__ __forceinline__ void post(uint32_t addr, int value)
{
    if ((threadIdx.x & 63) == 0)
        asm volatile("ds_write_b32 %0, %1" ::"v"(addr), "v"(value) : "memory");
}

// Until the loaders of chunk number need - 1 have written it (one batch tile: the loader of the
// chunk's parity, whose counter is at `addr`; two: both, counters at addr and addr + 4).
template <int MT>
__device__ __forceinline__ void await_chunk(uint32_t addr, int need)
{
    for (;;) {
        int v;
        if (MT == 1) {
            asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(addr) : "memory");
        } else {
            int2_t v2;
            asm volatile("ds_read_b64 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v2) : "v"(addr) : "memory");
            v = min(v2.x, v2.y);
        }
        if (__builtin_amdgcn_readfirstlane(v) >= need)
            break;
        __builtin_amdgcn_s_sleep(1);
    }
}

// What a step holds in registers: the stage's weights (pieces c and c + 4 of the lane's line in
// each row tile), the scales and zero points of the lane's row in each row tile for the stage's
// units, and x blocks the lane supplies to the stage's MFMAs: 8 / 4 / 2 per batch tile at 4 / 8 /
// 16 bits; with two batch tiles the 4-bit stage takes its 16 in two rounds, one per unit.
struct Stage {
    u32x4 w[RT][2];
    float s[RT][2]; // [row tile][unit of the stage] (8 bits: one unit)
    uint32_t z;     // byte 2 * rt + unit
    u32x4 a[8];
    // 2 bits (a stage is four units): the lane's 8 bytes of each unit, 32 k, and the units' metadata
    u32x2 w2[RT][4];
    float4_t s4[RT];
    uint32_t z4[RT]; // byte = unit
};

typedef float float2_t __attribute__((ext_vector_type(2)));

// Wait until at most ALLOW of the wavefront's loads are outstanding (the stage of this step is
// older than those), then copy the slot, the metadata and the stage's x blocks to registers.
// `wa`, `wb`: LDS byte addresses of the lane's two pieces in row tile 0 of the slot; `sa`, `za`:
// of the lane's scales and zero points for row tile 0 (row tile 1: UP entries further); `xa`:
// of the lane's x blocks.  All of it is inline assembly on purpose: the compiler cannot tell
// these reads from the slots being filled and would wait for every outstanding load first.
// Which x blocks land in st.a: 4 bits, MT = 1: [unit][i]; 4 bits, MT = 2: [batch tile][i] of
// unit 0 (unit 1 follows with more_x); 8 bits: [batch tile][half][i]; 16 bits: [batch tile][half].
template <int BITS, int MT, int ALLOW>
__device__ __forceinline__ void take(uint32_t wa, uint32_t wb, uint32_t sa, uint32_t za, const uint32_t (&xa)[4],
                                     Stage &st)
{
    if constexpr (BITS == 4) {
        float2_t s0, s1;
        uint32_t z0, z1;
        asm volatile("s_waitcnt vmcnt(%24)\n\t"
                     "ds_read_b128 %0, %16\n\t"
                     "ds_read_b128 %1, %17\n\t"
                     "ds_read_b128 %2, %16 offset:2048\n\t"
                     "ds_read_b128 %3, %17 offset:2048\n\t"
                     "ds_read_b64 %4, %18\n\t"
                     "ds_read_b64 %5, %18 offset:32\n\t"
                     "ds_read_u16 %6, %19\n\t"
                     "ds_read_u16 %7, %19 offset:8\n\t"
                     "ds_read_b128 %8, %20\n\t"
                     "ds_read_b128 %9, %21\n\t"
                     "ds_read_b128 %10, %22\n\t"
                     "ds_read_b128 %11, %23\n\t"
                     "ds_read_b128 %12, %20 offset:%25\n\t"
                     "ds_read_b128 %13, %21 offset:%25\n\t"
                     "ds_read_b128 %14, %22 offset:%25\n\t"
                     "ds_read_b128 %15, %23 offset:%25\n\t"
                     "s_waitcnt lgkmcnt(0)"
                     : "=&v"(st.w[0][0]), "=&v"(st.w[0][1]), "=&v"(st.w[1][0]), "=&v"(st.w[1][1]), "=&v"(s0), "=&v"(s1),
                       "=&v"(z0), "=&v"(z1), "=&v"(st.a[0]), "=&v"(st.a[1]), "=&v"(st.a[2]), "=&v"(st.a[3]),
                       "=&v"(st.a[4]), "=&v"(st.a[5]), "=&v"(st.a[6]), "=&v"(st.a[7])
                     : "v"(wa), "v"(wb), "v"(sa), "v"(za), "v"(xa[0]), "v"(xa[1]), "v"(xa[2]), "v"(xa[3]), "n"(ALLOW),
                       "n"(MT == 1 ? 4096 : 256) // the second unit, or the second batch tile of the first unit
                     : "memory");
        st.s[0][0] = s0.x, st.s[0][1] = s0.y, st.s[1][0] = s1.x, st.s[1][1] = s1.y;
        st.z = z0 | (z1 << 16);
    } else if constexpr (BITS == 8) {
        uint32_t z0, z1;
        if constexpr (MT == 1) {
            asm volatile("s_waitcnt vmcnt(%20)\n\t"
                         "ds_read_b128 %0, %12\n\t"
                         "ds_read_b128 %1, %13\n\t"
                         "ds_read_b128 %2, %12 offset:2048\n\t"
                         "ds_read_b128 %3, %13 offset:2048\n\t"
                         "ds_read_b32 %4, %14\n\t"
                         "ds_read_b32 %5, %14 offset:32\n\t"
                         "ds_read_u8 %6, %15\n\t"
                         "ds_read_u8 %7, %15 offset:8\n\t"
                         "ds_read_b128 %8, %16\n\t"
                         "ds_read_b128 %9, %17\n\t"
                         "ds_read_b128 %10, %18\n\t"
                         "ds_read_b128 %11, %19\n\t"
                         "s_waitcnt lgkmcnt(0)"
                         : "=&v"(st.w[0][0]), "=&v"(st.w[0][1]), "=&v"(st.w[1][0]), "=&v"(st.w[1][1]),
                           "=&v"(st.s[0][0]), "=&v"(st.s[1][0]), "=&v"(z0), "=&v"(z1), "=&v"(st.a[0]), "=&v"(st.a[1]),
                           "=&v"(st.a[2]), "=&v"(st.a[3])
                         : "v"(wa), "v"(wb), "v"(sa), "v"(za), "v"(xa[0]), "v"(xa[1]), "v"(xa[2]), "v"(xa[3]),
                           "n"(ALLOW)
                         : "memory");
        } else {
            asm volatile("s_waitcnt vmcnt(%24)\n\t"
                         "ds_read_b128 %0, %16\n\t"
                         "ds_read_b128 %1, %17\n\t"
                         "ds_read_b128 %2, %16 offset:2048\n\t"
                         "ds_read_b128 %3, %17 offset:2048\n\t"
                         "ds_read_b32 %4, %18\n\t"
                         "ds_read_b32 %5, %18 offset:32\n\t"
                         "ds_read_u8 %6, %19\n\t"
                         "ds_read_u8 %7, %19 offset:8\n\t"
                         "ds_read_b128 %8, %20\n\t"
                         "ds_read_b128 %9, %21\n\t"
                         "ds_read_b128 %10, %22\n\t"
                         "ds_read_b128 %11, %23\n\t"
                         "ds_read_b128 %12, %20 offset:256\n\t"
                         "ds_read_b128 %13, %21 offset:256\n\t"
                         "ds_read_b128 %14, %22 offset:256\n\t"
                         "ds_read_b128 %15, %23 offset:256\n\t"
                         "s_waitcnt lgkmcnt(0)"
                         : "=&v"(st.w[0][0]), "=&v"(st.w[0][1]), "=&v"(st.w[1][0]), "=&v"(st.w[1][1]),
                           "=&v"(st.s[0][0]), "=&v"(st.s[1][0]), "=&v"(z0), "=&v"(z1), "=&v"(st.a[0]), "=&v"(st.a[1]),
                           "=&v"(st.a[2]), "=&v"(st.a[3]), "=&v"(st.a[4]), "=&v"(st.a[5]), "=&v"(st.a[6]),
                           "=&v"(st.a[7])
                         : "v"(wa), "v"(wb), "v"(sa), "v"(za), "v"(xa[0]), "v"(xa[1]), "v"(xa[2]), "v"(xa[3]),
                           "n"(ALLOW)
                         : "memory");
        }
        st.z = z0 | (z1 << 16);
    } else {
        if constexpr (MT == 1) {
            asm volatile("s_waitcnt vmcnt(%10)\n\t"
                         "ds_read_b128 %0, %6\n\t"
                         "ds_read_b128 %1, %7\n\t"
                         "ds_read_b128 %2, %6 offset:2048\n\t"
                         "ds_read_b128 %3, %7 offset:2048\n\t"
                         "ds_read_b128 %4, %8\n\t"
                         "ds_read_b128 %5, %9\n\t"
                         "s_waitcnt lgkmcnt(0)"
                         : "=&v"(st.w[0][0]), "=&v"(st.w[0][1]), "=&v"(st.w[1][0]), "=&v"(st.w[1][1]), "=&v"(st.a[0]),
                           "=&v"(st.a[1])
                         : "v"(wa), "v"(wb), "v"(xa[0]), "v"(xa[1]), "n"(ALLOW)
                         : "memory");
        } else {
            asm volatile("s_waitcnt vmcnt(%12)\n\t"
                         "ds_read_b128 %0, %8\n\t"
                         "ds_read_b128 %1, %9\n\t"
                         "ds_read_b128 %2, %8 offset:2048\n\t"
                         "ds_read_b128 %3, %9 offset:2048\n\t"
                         "ds_read_b128 %4, %10\n\t"
                         "ds_read_b128 %5, %11\n\t"
                         "ds_read_b128 %6, %10 offset:256\n\t"
                         "ds_read_b128 %7, %11 offset:256\n\t"
                         "s_waitcnt lgkmcnt(0)"
                         : "=&v"(st.w[0][0]), "=&v"(st.w[0][1]), "=&v"(st.w[1][0]), "=&v"(st.w[1][1]), "=&v"(st.a[0]),
                           "=&v"(st.a[1]), "=&v"(st.a[2]), "=&v"(st.a[3])
                         : "v"(wa), "v"(wb), "v"(xa[0]), "v"(xa[1]), "n"(ALLOW)
                         : "memory");
        }
    }
}

// The x blocks of the second unit of a 4-bit stage with two batch tiles: [batch tile][i].
__device__ __forceinline__ void more_x(uint32_t xa0, uint32_t xa1, uint32_t xa2, uint32_t xa3, Stage &st)
{
    asm volatile("ds_read_b128 %0, %8 offset:8192\n\t"
                 "ds_read_b128 %1, %9 offset:8192\n\t"
                 "ds_read_b128 %2, %10 offset:8192\n\t"
                 "ds_read_b128 %3, %11 offset:8192\n\t"
                 "ds_read_b128 %4, %8 offset:8448\n\t"
                 "ds_read_b128 %5, %9 offset:8448\n\t"
                 "ds_read_b128 %6, %10 offset:8448\n\t"
                 "ds_read_b128 %7, %11 offset:8448\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(st.a[0]), "=&v"(st.a[1]), "=&v"(st.a[2]), "=&v"(st.a[3]), "=&v"(st.a[4]), "=&v"(st.a[5]),
                   "=&v"(st.a[6]), "=&v"(st.a[7])
                 : "v"(xa0), "v"(xa1), "v"(xa2), "v"(xa3)
                 : "memory");
}

// A 2-bit stage: the lane's 8 bytes of each of the four units of both row tiles (`wq`: their LDS
// addresses in row tile 0), scales and zero points of the four units, the x blocks of the first
// unit (and first batch tile).  Same waits as take().
template <int ALLOW>
__device__ __forceinline__ void take2(const uint32_t (&wq)[4], uint32_t sa, uint32_t za, const uint32_t (&xa)[4],
                                      Stage &st)
{
    asm volatile("s_waitcnt vmcnt(%26)\n\t"
                 "ds_read_b64 %0, %16\n\t"
                 "ds_read_b64 %1, %17\n\t"
                 "ds_read_b64 %2, %18\n\t"
                 "ds_read_b64 %3, %19\n\t"
                 "ds_read_b64 %4, %16 offset:2048\n\t"
                 "ds_read_b64 %5, %17 offset:2048\n\t"
                 "ds_read_b64 %6, %18 offset:2048\n\t"
                 "ds_read_b64 %7, %19 offset:2048\n\t"
                 "ds_read_b128 %8, %20\n\t"
                 "ds_read_b128 %9, %20 offset:32\n\t"
                 "ds_read_b32 %10, %21\n\t"
                 "ds_read_b32 %11, %21 offset:8\n\t"
                 "ds_read_b128 %12, %22\n\t"
                 "ds_read_b128 %13, %23\n\t"
                 "ds_read_b128 %14, %24\n\t"
                 "ds_read_b128 %15, %25\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(st.w2[0][0]), "=&v"(st.w2[0][1]), "=&v"(st.w2[0][2]), "=&v"(st.w2[0][3]), "=&v"(st.w2[1][0]),
                   "=&v"(st.w2[1][1]), "=&v"(st.w2[1][2]), "=&v"(st.w2[1][3]), "=&v"(st.s4[0]), "=&v"(st.s4[1]),
                   "=&v"(st.z4[0]), "=&v"(st.z4[1]), "=&v"(st.a[0]), "=&v"(st.a[1]), "=&v"(st.a[2]), "=&v"(st.a[3])
                 : "v"(wq[0]), "v"(wq[1]), "v"(wq[2]), "v"(wq[3]), "v"(sa), "v"(za), "v"(xa[0]), "v"(xa[1]), "v"(xa[2]),
                   "v"(xa[3]), "n"(ALLOW)
                 : "memory");
}

// Four x blocks, OFF bytes past the addresses given, into st.a[D0 ..].
template <int OFF, int D0>
__device__ __forceinline__ void read_x4(const uint32_t (&xa)[4], Stage &st)
{
    asm volatile("ds_read_b128 %0, %4 offset:%8\n\t"
                 "ds_read_b128 %1, %5 offset:%8\n\t"
                 "ds_read_b128 %2, %6 offset:%8\n\t"
                 "ds_read_b128 %3, %7 offset:%8\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(st.a[D0]), "=&v"(st.a[D0 + 1]), "=&v"(st.a[D0 + 2]), "=&v"(st.a[D0 + 3])
                 : "v"(xa[0]), "v"(xa[1]), "v"(xa[2]), "v"(xa[3]), "n"(OFF)
                 : "memory");
}

template <int BITS>
struct Cfg {
    static constexpr int KPS = 128 * 8 / BITS; // k per stage: 512 / 256 / 128 / 64 at 2 / 4 / 8 / 16 bits
    static constexpr int SPC = KC / KPS;       // steps per chunk: 1 / 2 / 4 / 8
};

// ------------------------------------------------------------------ consumer wavefronts
template <int BITS, int MT>
struct Consumer {
    typedef Cfg<BITS> C;
    const Sel &d;
    const Lds &L;
    const int M, wave, lane, n, c, row0;
    const int row_bytes;  // a multiple of 64 (2 bits: of 32)
    const int nchunks;
    int T;                // steps: 128-byte lines of a row (the last may be half a line at 4 bits)
    uint8_t *ring;        // this wavefront's NS slots
    const uint8_t *gbase; // first byte of the wavefront's first row (wave-uniform)
    // per-lane constants of the weight loads: load i of a stage covers rows 8 i .. 8 i + 7, lane
    // -> row lane / 8 of those, LDS slot lane % 8, i.e. piece slot ^ ((row % 16) >> 1) of the line
    uint32_t ld_off[SOPS]; // byte offset of the lane's row from the first row, plus its piece
    uint32_t ld_hi;        // 64 if the lane's piece in even loads lies in the upper half of the line (odd: the other)
    uint32_t ld_piece;     // the lane's piece in even loads (odd ones: that ^ 4)
    uint32_t wa0, wb0;     // LDS addresses for take(): the lane's pieces c and c + 4 in slot 0
    uint32_t wq0;          // 2 bits: of the lane's 8 bytes of the stage's first unit (unit u: wq0 ^ 32 u)
    uint32_t ml;           // wave * 16 + n: the lane's place in the metadata of a pair of chunks
    // byte offsets of the lane's x blocks inside a stage's blocks (block kb of the chunk holds
    // batch row n at place n ^ (kb % 8 + 8 (kb / 32))).  4 bits: blocks 4 c + i of either unit; 8 bits: blocks 8 h + 2 c + i;
    // 16 bits: blocks 4 h + c of an even stage, 8 + 4 h + c of an odd one
    uint32_t xq[4];
    float4_t acc[RT][MT], out[RT][MT];
    const int base;        // number of the tile's first chunk in the launch's count
    const int tileno;      // number of the tile among the workgroup's
    // the next tile, looked up when the ring has room for it: 0 not yet, 1 to be requested, 2 not
    // to be (none, passed over, or rows of no more than NS lines)
    int nx_state;
    const uint8_t *ncodes;
    int nN, nrow_bytes, nrow0;
    Ahead ahead;

    __device__ __forceinline__ Consumer(const Sel &d_, const Lds &L_, int M_, int tile_row0, int wave_, int base_,
                                        int tileno_)
        : d(d_), L(L_), M(M_), wave(wave_), lane(threadIdx.x & 63), n(lane & 15), c(lane >> 4),
          row0(tile_row0 + wave_ * RT * 16), row_bytes(d_.K * BITS / 8), nchunks((d_.K + KC - 1) / KC), base(base_), tileno(tileno_), nx_state(0),
          ncodes(nullptr), nN(0), nrow_bytes(0), nrow0(0)
    {
        ahead.pf = 0, ahead.slot0 = 0;
        T = (row_bytes + 127) / 128;
        ring = L.ring + wave * NS * STAGE_BYTES;
        // the wavefront's rows span at most 32 * row_bytes < 4 GiB: 32-bit lane offsets from a uniform base
        const int first_row = min(row0, d.N - 1);
        gbase = d.codes + (size_t)first_row * (size_t)row_bytes;
        const int r = lane >> 3, slot = lane & 7;
#pragma unroll
        for (int i = 0; i < SOPS; i++) {
            const int rl = 8 * i + r; // row inside the wavefront's 32
            const int piece = slot ^ (((rl & 15) >> 1) & 7);
            const int row = min(row0 + rl, d.N - 1);
            ld_off[i] = (uint32_t)(row - first_row) * (uint32_t)row_bytes + (uint32_t)piece * 16;
        }
        ld_hi = ((slot ^ (r >> 1)) & 4) * 16; // bit 2 of the piece flips with the parity of i
        ld_piece = (uint32_t)(slot ^ (r >> 1));
        wa0 = lds_addr(ring) + n * 128 + ((c ^ ((n >> 1) & 7)) * 16);
        wb0 = wa0 ^ 64; // piece c + 4
        // a unit is 32 bytes of a line, an MFMA takes 8 of them: 2 from each group of 16 lanes
        wq0 = lds_addr(ring) + n * 128 + (((c >> 1) ^ ((n >> 1) & 7)) * 16) + (c & 1) * 8;
        ml = wave * 16 + n;
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int kb = BITS == 4 || BITS == 2 ? 4 * c + i : BITS == 8 ? 8 * (i >> 1) + 2 * c + (i & 1) : 4 * i + c;
            xq[i] = (uint32_t)(kb * (256 * MT) + ((n ^ (kb & 7)) * 16));
        }
#pragma unroll
        for (int rt = 0; rt < RT; rt++)
#pragma unroll
            for (int mt = 0; mt < MT; mt++) {
                acc[rt][mt] = float4_t{0.f, 0.f, 0.f, 0.f};
                out[rt][mt] = float4_t{0.f, 0.f, 0.f, 0.f};
            }
    }

    // Request step q (line q of every row) into ring slot `slot`.  A 4-bit row may end with
    // half a line: the lanes of the missing half re-read the present one (their x is zero).
    __device__ __forceinline__ void fetch(int q, int slot)
    {
        const uint8_t *base = gbase + (size_t)q * 128;
        uint8_t *dst = ring + slot * STAGE_BYTES;
        const bool half_line = BITS == 4 && q * 128 + 64 >= row_bytes;
        uint32_t back_even = half_line ? ld_hi : 0u, back_odd = half_line ? 64u - ld_hi : 0u;
        if (BITS == 2 && q * 128 + 128 > row_bytes) {
            // a 2-bit row may end with 2, 4 or 6 of a line's 8 pieces: piece p -> p % pieces
            const uint32_t np = (uint32_t)(row_bytes - q * 128) >> 4;
            const uint32_t pe = ld_piece, po = ld_piece ^ 4u;
            back_even = ((pe >= np) + (pe >= 2 * np) + (pe >= 3 * np)) * np * 16;
            back_odd = ((po >= np) + (po >= 2 * np) + (po >= 3 * np)) * np * 16;
        }
#pragma unroll
        for (int i = 0; i < SOPS; i++) {
            uint32_t off = ld_off[i];
            if (BITS == 4 || BITS == 2)
                off -= (i & 1) ? back_odd : back_even; // 4 bits: pieces 4..7 -> 0..3
            __builtin_amdgcn_global_load_lds((const FQ_GLOBAL void *)(base + off), (FQ_LDS void *)(dst + i * 1024), 16,
                                             0, 2 /* nt: the weights are read once */);
        }
    }

    // The ring slot `slot` has just been emptied and the tile has no stage left to put there:
    // request the next tile's (same rows of the tile, lines from the start), so that the ring
    // does not run dry across the tile boundary.  The next tile's record is in LDS once loader 1
    // has counted its draw in flag[4]; if that has not happened yet, nothing is requested.
    __device__ __forceinline__ void request_ahead(int slot)
    {
        if (nx_state == 0) {
            int drawn;
            asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(drawn) : "v"(lds_addr(L.flag) + 16u) : "memory");
            if (__builtin_amdgcn_readfirstlane(drawn) < tileno + 2)
                return;
            u32x4 a, b; // words 0 .. 7 of the record: e, t, bits, N, K, codes
            asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %2 offset:16\n\ts_waitcnt lgkmcnt(0)"
                         : "=&v"(a), "=&v"(b)
                         : "v"(lds_addr(L.mail) + 64u * ((tileno + 1) & 1))
                         : "memory");
            const int e = __builtin_amdgcn_readfirstlane((int)a.x), t = __builtin_amdgcn_readfirstlane((int)a.y),
                      bits = __builtin_amdgcn_readfirstlane((int)a.z), K = __builtin_amdgcn_readfirstlane((int)b.x);
            nN = __builtin_amdgcn_readfirstlane((int)a.w);
            ncodes = (const uint8_t *)(uintptr_t)((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)b.y) |
                                                  ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)b.z) << 32));
            nrow_bytes = K * bits / 8;
            nrow0 = t * TILE_ROWS + wave * RT * 16;
            // (a row of more than NS lines: none of the first NS is a last, possibly half, line)
            nx_state = e >= 0 && bits != 0 && nrow_bytes > NS * 128 ? 1 : 2;
        }
        if (nx_state != 1 || ahead.pf >= NS)
            return;
        if (ahead.pf == 0)
            ahead.slot0 = slot;
        const int first_row = min(nrow0, nN - 1);
        const uint8_t *src = ncodes + (size_t)first_row * (size_t)nrow_bytes + (size_t)ahead.pf * 128;
        uint8_t *dst = ring + slot * STAGE_BYTES;
        const int r = lane >> 3, sl = lane & 7;
#pragma unroll
        for (int i = 0; i < SOPS; i++) { // as in the constructor and fetch(), for the next tile
            const int rl = 8 * i + r;
            const int piece = sl ^ (((rl & 15) >> 1) & 7);
            const int row = min(nrow0 + rl, nN - 1);
            const uint32_t off = (uint32_t)(row - first_row) * (uint32_t)nrow_bytes + (uint32_t)piece * 16;
            __builtin_amdgcn_global_load_lds((const FQ_GLOBAL void *)(src + off), (FQ_LDS void *)(dst + i * 1024), 16, 0,
                                             2);
        }
        ahead.pf++;
    }

    // One unit (128 k) of a 4-bit stage: half h of the line, x blocks a[mt * AM + i].
    template <int AM, int H>
    __device__ __forceinline__ void unit4(const Stage &st, const u32x4 *a)
    {
        constexpr int h = H;
        // Offsets and zero point come off the operand itself, a packed fp16 add per register (exact:
        // (offset + q) - (offset + z) is a small integer): a second MFMA per operand on the constant
        // -(offset + z) instead was 3 % slower with one batch tile and 11 % with two.
        uint32_t magic_lo = 0x64006400u, magic_hi = 0x54005400u;
        asm volatile("" : "+v"(magic_lo), "+v"(magic_hi));
        const uint32_t z4 = (st.z << 4) & 0xF0F0F0F0u;
        u32x4 nz[RT];
#pragma unroll
        for (int rt = 0; rt < RT; rt++) {
            const uint32_t by = (uint32_t)(2 * rt + h), sel = 0x04000400u | by | (by << 16);
            const uint32_t lo = __builtin_amdgcn_perm(0xE4E4E4E4u, st.z, sel); // -(1024 + z) twice
            const uint32_t hi = __builtin_amdgcn_perm(0xD4D4D4D4u, z4, sel);   // -(  64 + z) twice
            nz[rt] = u32x4{lo, hi, lo, hi};
        }
#pragma unroll
        for (int i = 0; i < 4; i++) {
#pragma unroll
            for (int rt = 0; rt < RT; rt++) {
                const uint32_t w = st.w[rt][h][i], w8 = w >> 8;
                u32x4 b;
                b.x = (w & 0x000F000Fu) | magic_lo;  // (1024 + q0, 1024 + q4)
                b.y = (w & 0x00F000F0u) | magic_hi;  // (  64 + q1,   64 + q5)
                b.z = (w8 & 0x000F000Fu) | magic_lo; // (1024 + q2, 1024 + q6)
                b.w = (w8 & 0x00F000F0u) | magic_hi; // (  64 + q3,   64 + q7)
                b.x = pk_add_h(b.x, nz[rt].x);
                b.y = pk_add_h(b.y, nz[rt].y);
                b.z = pk_add_h(b.z, nz[rt].z);
                b.w = pk_add_h(b.w, nz[rt].w);
#pragma unroll
                for (int mt = 0; mt < MT; mt++)
                    acc[rt][mt] = mfma(a[mt * AM + i], b, acc[rt][mt]);
            }
        }
#pragma unroll
        for (int rt = 0; rt < RT; rt++)
#pragma unroll
            for (int mt = 0; mt < MT; mt++) {
                out[rt][mt] += st.s[rt][h] * acc[rt][mt];
                acc[rt][mt] = float4_t{0.f, 0.f, 0.f, 0.f};
            }
    }

    // One unit (128 k) of a 2-bit stage: the lane's 8 bytes st.w2[rt][U], x blocks st.a[mt * 4 + j].
    // A byte holds four consecutive codes: copied to both halves of a word, (t & 0x000C0003) |
    // 0x5C006400 is the pair (1024 + q0, 256 + q1) and (t & 0x00C00030) | 0x4C005400 the pair
    // (64 + q2, 16 + q3); a packed add of -(offset + z) per register leaves q - z.
    template <int U>
    __device__ __forceinline__ void unit2(const Stage &st)
    {
        uint32_t m01 = 0x5C006400u, m23 = 0x4C005400u;
        asm volatile("" : "+v"(m01), "+v"(m23));
        u32x4 nz[RT];
#pragma unroll
        for (int rt = 0; rt < RT; rt++) {
            const uint32_t zb = (st.z4[rt] >> (8 * U)) & 0xFFu, t = zb | (zb << 18);
            const uint32_t lo = 0xDC00E400u | t;        // -(1024 + z), -(256 + z)
            const uint32_t hi = 0xCC00D400u | (t << 4); // -(  64 + z), -( 16 + z)
            nz[rt] = u32x4{lo, hi, lo, hi};
        }
#pragma unroll
        for (int j = 0; j < 4; j++) {
#pragma unroll
            for (int rt = 0; rt < RT; rt++) {
                const u32x2 w = st.w2[rt][U];
                const uint32_t lo = w.x, hi = w.y; // (element by element from a copy)
                const uint32_t ia = 2 * j, ib = 2 * j + 1; // the two bytes of this MFMA's 8 codes
                const uint32_t ta = __builtin_amdgcn_perm(hi, lo, 0x0c000c00u | ia | (ia << 16));
                const uint32_t tb = __builtin_amdgcn_perm(hi, lo, 0x0c000c00u | ib | (ib << 16));
                u32x4 b;
                b.x = (ta & 0x000C0003u) | m01;
                b.y = (ta & 0x00C00030u) | m23;
                b.z = (tb & 0x000C0003u) | m01;
                b.w = (tb & 0x00C00030u) | m23;
                b.x = pk_add_h(b.x, nz[rt].x); // exact, as at 4 bits
                b.y = pk_add_h(b.y, nz[rt].y);
                b.z = pk_add_h(b.z, nz[rt].x);
                b.w = pk_add_h(b.w, nz[rt].y);
#pragma unroll
                for (int mt = 0; mt < MT; mt++) // (the unit's sum starts from the instruction's constant 0)
                    acc[rt][mt] = mfma(st.a[mt * 4 + j], b, j == 0 ? float4_t{0.f, 0.f, 0.f, 0.f} : acc[rt][mt]);
            }
        }
#pragma unroll
        for (int rt = 0; rt < RT; rt++) {
            const float4_t s4 = st.s4[rt];
            const float sc = U == 0 ? s4.x : U == 1 ? s4.y : U == 2 ? s4.z : s4.w;
#pragma unroll
            for (int mt = 0; mt < MT; mt++)
                out[rt][mt] += sc * acc[rt][mt];
        }
    }

    // The four units of a 2-bit stage; take2() has brought the first unit's x blocks of the first
    // batch tile, the others are read here.  `xa`: as given to take2(); the blocks of units 2 and
    // 3 sit 128 bytes the other way inside their rows of 16 (k block / 32 changes).
    __device__ __forceinline__ void compute2(Stage &st, uint32_t (&xa)[4])
    {
        if (MT == 2)
            read_x4<256, 4>(xa, st);
        unit2<0>(st);
        read_x4<4096 * MT, 0>(xa, st);
        if (MT == 2)
            read_x4<4096 * MT + 256, 4>(xa, st);
        unit2<1>(st);
        uint32_t(&xb)[4] = xa; // (in place: the addresses of units 0 and 1 are not needed again)
#pragma unroll
        for (int i = 0; i < 4; i++)
            xb[i] ^= 128u;
        read_x4<2 * 4096 * MT, 0>(xb, st);
        if (MT == 2)
            read_x4<2 * 4096 * MT + 256, 4>(xb, st);
        unit2<2>(st);
        read_x4<3 * 4096 * MT, 0>(xb, st);
        if (MT == 2)
            read_x4<3 * 4096 * MT + 256, 4>(xb, st);
        unit2<3>(st);
    }

    // The stage in `st` (for 4 bits and two batch tiles: its second unit is fetched here, xa as
    // given to take()).
    __device__ __forceinline__ void compute(Stage &st, uint32_t xa0, uint32_t xa1, uint32_t xa2, uint32_t xa3)
    {
        if (BITS == 4) {
            if (MT == 1) {
                unit4<0, 0>(st, st.a);
                unit4<0, 1>(st, st.a + 4);
            } else {
                unit4<4, 0>(st, st.a);
                more_x(xa0, xa1, xa2, xa3, st);
                unit4<4, 1>(st, st.a);
            }
        } else if (BITS == 8) {
            u32x4 nz[RT];
#pragma unroll
            for (int rt = 0; rt < RT; rt++) {
                const uint32_t by = (uint32_t)(2 * rt), sel = 0x04000400u | by | (by << 16);
                const uint32_t v = __builtin_amdgcn_perm(0xE4E4E4E4u, st.z, sel); // -(1024 + z) twice
                nz[rt] = u32x4{v, v, v, v};
            }
#pragma unroll
            for (int h = 0; h < 2; h++)
#pragma unroll
                for (int i = 0; i < 2; i++) {
#pragma unroll
                    for (int rt = 0; rt < RT; rt++) {
                        const uint32_t v0 = st.w[rt][h][2 * i], v1 = st.w[rt][h][2 * i + 1];
                        u32x4 b;
                        b.x = __builtin_amdgcn_perm(0x64646464u, v0, 0x04010400u);
                        b.y = __builtin_amdgcn_perm(0x64646464u, v0, 0x04030402u);
                        b.z = __builtin_amdgcn_perm(0x64646464u, v1, 0x04010400u);
                        b.w = __builtin_amdgcn_perm(0x64646464u, v1, 0x04030402u);
                        if (MT == 2) { // two batch tiles: q - z in the operand (as at 4 bits)
                            b.x = pk_add_h(b.x, nz[rt].x);
                            b.y = pk_add_h(b.y, nz[rt].x);
                            b.z = pk_add_h(b.z, nz[rt].x);
                            b.w = pk_add_h(b.w, nz[rt].x);
                        }
#pragma unroll
                        for (int mt = 0; mt < MT; mt++)
                            acc[rt][mt] = mfma(st.a[mt * 4 + 2 * h + i], b, acc[rt][mt]);
                    }
                    if (MT != 2) {
#pragma unroll
                        for (int rt = 0; rt < RT; rt++)
#pragma unroll
                            for (int mt = 0; mt < MT; mt++)
                                acc[rt][mt] = mfma(st.a[mt * 4 + 2 * h + i], nz[rt], acc[rt][mt]);
                    }
                }
#pragma unroll
            for (int rt = 0; rt < RT; rt++)
#pragma unroll
                for (int mt = 0; mt < MT; mt++) {
                    out[rt][mt] += st.s[rt][0] * acc[rt][mt];
                    acc[rt][mt] = float4_t{0.f, 0.f, 0.f, 0.f};
                }
        } else {
#pragma unroll
            for (int h = 0; h < 2; h++)
#pragma unroll
                for (int rt = 0; rt < RT; rt++)
#pragma unroll
                    for (int mt = 0; mt < MT; mt++)
                        acc[rt][mt] = mfma(st.a[mt * 2 + h], st.w[rt][h], acc[rt][mt]);
        }
    }

    // Chunk ch, whose x is in buffer xb.
    __device__ __forceinline__ void chunk(int ch, int xb, int &fq, int &slot)
    {
        // the loaders have written chunk ch
        await_chunk<MT>(lds_addr(L.flag) + (MT == 1 ? 4u * (ch % LOADERS) : 8u * (ch % (LOADERS / 2))), base + ch + 1);
        // metadata: buffer of the pair of chunks, the chunk's half of it, the lane's row
        const uint32_t mo = ml * (RT * UP) + (ch & 1) * UC;
        const uint32_t sbase = lds_addr((ch & 2) ? L.ms[1] : L.ms[0]) + mo * 4,
                       zbase = lds_addr((ch & 2) ? L.mz[1] : L.mz[0]) + mo;
        uint32_t xbase = lds_addr(L.x) + (uint32_t)xb * (16 * MT * KC * 2);
        asm volatile("" : "+s"(xbase)); // opaque: or every stage's x addresses are hoisted out of the tile and spill
#pragma unroll
        for (int j = 0; j < C::SPC; j++) {
            const int q = ch * C::SPC + j;
            if (q >= T)
                break;
            // where the stage sits inside the chunk: its first unit, its x blocks
            const int unit = j * C::KPS / 128;
            const uint32_t wa = wa0 + slot * STAGE_BYTES, wb = wb0 + slot * STAGE_BYTES, sa = sbase + unit * 4,
                           za = zbase + unit;
            uint32_t xa[4];
            if (BITS == 2) {
#pragma unroll
                for (int i = 0; i < 4; i++)
                    xa[i] = xbase + xq[i]; // the stage is the chunk
            } else if (BITS == 4) {
#pragma unroll
                for (int i = 0; i < 4; i++)
                    xa[i] = xbase + j * (8192 * MT) + (xq[i] ^ (j ? 128u : 0u));
            } else if (BITS == 8) {
#pragma unroll
                for (int i = 0; i < 4; i++)
                    xa[i] = xbase + j * (4096 * MT) + (xq[i] ^ ((j >> 1) ? 128u : 0u));
            } else {
                xa[0] = xbase + (j >> 1) * (4096 * MT) + (xq[2 * (j & 1)] ^ ((j >> 2) ? 128u : 0u));
                xa[1] = xbase + (j >> 1) * (4096 * MT) + (xq[2 * (j & 1) + 1] ^ ((j >> 2) ? 128u : 0u));
                xa[2] = xa[3] = 0;
            }
            Stage st;
            const int pend = __builtin_amdgcn_readfirstlane(fq + ahead.pf - 1 - q); // younger stages in flight
            if constexpr (BITS == 2) {
                const uint32_t w0 = wq0 + slot * STAGE_BYTES;
                const uint32_t wq[4] = {w0, w0 ^ 32u, w0 ^ 64u, w0 ^ 96u};
                if (NS > 2 && pend >= 2)
                    take2<2 * SOPS>(wq, sa, za, xa, st);
                else if (pend == 1)
                    take2<SOPS>(wq, sa, za, xa, st);
                else
                    take2<0>(wq, sa, za, xa, st);
            } else {
                if (NS > 2 && pend >= 2)
                    take<BITS, MT, 2 * SOPS>(wa, wb, sa, za, xa, st);
                else if (pend == 1)
                    take<BITS, MT, SOPS>(wa, wb, sa, za, xa, st);
                else
                    take<BITS, MT, 0>(wa, wb, sa, za, xa, st);
            }
            if (fq < T) { // the stage NS steps ahead, into the slot just emptied
                fetch(fq, slot);
                fq++;
            } else {
                request_ahead(slot);
            }
            __builtin_amdgcn_sched_barrier(0); // keep the requests here: the scheduler sinks them otherwise
            if constexpr (BITS == 2)
                compute2(st, xa);
            else
                compute(st, xa[0], xa[1], xa[2], xa[3]);
            slot = slot == NS - 1 ? 0 : slot + 1;
        }
        post(lds_addr(L.flag) + 4u * (8 + wave), base + ch + 1); // every read of the chunk's buffers has returned
    }

    // `in`: what the tile before this one has requested of this one.
    __device__ __forceinline__ Ahead run(const Ahead in)
    {
        int fq = in.pf, slot = in.pf ? in.slot0 : 0;
        for (int s = in.pf; s < NS; s++)
            if (fq < T) {
                fetch(fq, slot + s >= NS ? slot + s - NS : slot + s);
                fq++;
            }
        __builtin_amdgcn_sched_barrier(0);
        for (int ch = 0, xb = 0; ch < nchunks; ch++) {
            chunk(ch, xb, fq, slot);
            xb = xb == nxb(MT) - 1 ? 0 : xb + 1;
        }
        // D layout of the 16x16 MFMA: lane holds column n = lane % 16, rows 4 * (lane / 16) + r.
#pragma unroll
        for (int rt = 0; rt < RT; rt++) {
            const int row = row0 + rt * 16 + n;
#pragma unroll
            for (int mt = 0; mt < MT; mt++) {
                const float4_t v = BITS == 16 ? acc[rt][mt] : out[rt][mt];
#pragma unroll
                for (int r = 0; r < 4; r++) {
                    const int m = mt * 16 + c * 4 + r;
                    if (m < M && row < d.N)
                        ((FQ_GLOBAL uint16_t *)d.y)[(size_t)m * d.N + row] =
                            __builtin_bit_cast(uint16_t, (_Float16)v[r]);
                }
            }
        }
        __builtin_amdgcn_s_waitcnt(0xc07f); // lgkmcnt(0); the requests for the next tile stay in flight
        barrier(); // the loaders may refill the buffers for the next tile
        return ahead;
    }
};

// ------------------------------------------------------------------ loader wavefront
// (One code path for the three bit-widths, and one place each where a chunk is requested and
// where it is written: instantiated per width or per place, the register allocator sees several
// sets of staging registers live across the tile loop.)

// The tile a loader writes chunks of, or requests them for.
struct LoaderTile {
    Sel d;
    int tile_row0, G, nchunks, bits; // nchunks = 0: nothing to load (no tile, or one that is passed over)
};

template <int MT>
struct Loader {
    const Lds &L;
    const int M, lane;
    const int li; // which loader: 0 .. LOADERS - 1
    // With one batch tile the loaders take the chunks in turn; with two, loader li takes batch
    // tile li % 2 of every chunk (two loaders) or of every other chunk, those of parity li / 2.
    const int bt; // the batch tile of this loader
    // the chunk's block `lane` of 16 batch rows (with two batch tiles: loader li takes tile li):
    // one 1 KiB request per row
    u32x4 xr[16];
    // metadata of a pair of chunks (UP units): scales as 16 bytes = 4 units per lane, two lanes to
    // a row, 32 rows to an instruction; zero points as 8 bytes per lane, one lane to a row
    float4_t sr[TILE_ROWS / 32];
    uint32_t zr[TILE_ROWS / 64][2];

    __device__ __forceinline__ Loader(const Lds &L_, int M_, int li_)
        : L(L_), M(M_), lane(threadIdx.x & 63), li(li_), bt(MT == 2 ? li_ & 1 : 0)
    {
    }

    __device__ __forceinline__ void load_x(const LoaderTile &T, int ch)
    {
        const int k = ch * KC + lane * 8;

#pragma unroll
        for (int m = 0; m < 16; m++) {
            // batch rows past M feed outputs that are never stored; k past K meets re-read weights
            // (the missing half of a last line): x is zero there
            const int mm = min(16 * bt + m, M - 1);
            xr[m] = k < T.d.K ? *(const FQ_GLOBAL u32x4 *)(T.d.x + (size_t)mm * T.d.K + k) : u32x4{0u, 0u, 0u, 0u};
        }
    }

    __device__ __forceinline__ void store_x(int bits, int b)
    {
        u32x4 *xb = reinterpret_cast<u32x4 *>(L.x + b * (16 * MT * KC * 2));
#pragma unroll
        for (int m = 0; m < 16; m++) {
            u32x4 p = xr[m];
            if (bits == 4) { // (x0 .. x7) -> (x0 x4 x1 x5 x2 x6 x3 x7), the unpack order
                p.x = __builtin_amdgcn_perm(xr[m].z, xr[m].x, 0x05040100u);
                p.y = __builtin_amdgcn_perm(xr[m].z, xr[m].x, 0x07060302u);
                p.z = __builtin_amdgcn_perm(xr[m].w, xr[m].y, 0x05040100u);
                p.w = __builtin_amdgcn_perm(xr[m].w, xr[m].y, 0x07060302u);
            }
            // conflict free for the writer and for the readers
            xb[lane * (16 * MT) + 16 * bt + (m ^ ((lane & 7) | ((lane >> 2) & 8)))] = p;
        }
    }

    // Metadata of the pair of chunks cp: units UP * cp ...  Past G (a last, partial pair) the
    // unit index is clamped, and then every unit is fetched on its own.  Addresses are a uniform
    // base plus a 32-bit lane offset, recomputed per call (kept opaque: hoisted out of the tile
    // they would cost a register each).
    __device__ __forceinline__ void load_meta(const LoaderTile &T, int cp)
    {
        typedef float f32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));
        typedef uint32_t u32_a1 __attribute__((aligned(1)));
        const int G = T.G;
        const int u0 = cp * UP;
        const bool whole = u0 + UP <= G;
        int last = __builtin_amdgcn_readfirstlane(T.d.N - 1 - T.tile_row0); // rows of the tile past N repeat row N - 1
        asm volatile("" : "+s"(last));
        const float *sbase = T.d.scales + (size_t)T.tile_row0 * (size_t)G;
        const uint8_t *zbase = T.d.zeros + (size_t)T.tile_row0 * (size_t)G;
#pragma unroll
        for (int i = 0; i < TILE_ROWS / 32; i++) {
            const uint32_t row = (uint32_t)min(32 * i + (lane >> 1), last);
            const int u = u0 + 4 * (lane & 1);
            if (whole) {
                sr[i] = *(const FQ_GLOBAL f32x4_a4 *)(sbase + (row * (uint32_t)G + (uint32_t)u));
            } else {
#pragma unroll
                for (int g = 0; g < 4; g++)
                    sr[i][g] = ((const FQ_GLOBAL float *)sbase)[row * (uint32_t)G + (uint32_t)min(u + g, G - 1)];
            }
        }
#pragma unroll
        for (int j = 0; j < TILE_ROWS / 64; j++) {
            const uint32_t row = (uint32_t)min(64 * j + lane, last);
            if (whole) {
                zr[j][0] = *(const FQ_GLOBAL u32_a1 *)(zbase + (row * (uint32_t)G + (uint32_t)u0));
                zr[j][1] = *(const FQ_GLOBAL u32_a1 *)(zbase + (row * (uint32_t)G + (uint32_t)u0 + 4u));
            } else {
                zr[j][0] = zr[j][1] = 0;
#pragma unroll
                for (int g = 0; g < UP; g++)
                    zr[j][g >> 2] |= (uint32_t)((const FQ_GLOBAL uint8_t *)zbase)[row * (uint32_t)G + (uint32_t)min(u0 + g, G - 1)]
                                     << (8 * (g & 3));
            }
        }
    }

    // [consumer][row % 16][row tile][unit]
    __device__ __forceinline__ void store_meta(int b)
    {
        float *ms = b ? L.ms[1] : L.ms[0];
        uint8_t *mz = b ? L.mz[1] : L.mz[0];
#pragma unroll
        for (int i = 0; i < TILE_ROWS / 32; i++) {
            // row 32 i + lane / 2 of the tile: consumer i, row tile lane / 32, row (lane / 2) % 16
            const int idx = ((i * 16 + ((lane >> 1) & 15)) * RT + (lane >> 5)) * UP + 4 * (lane & 1);
            *reinterpret_cast<float4_t *>(ms + idx) = sr[i];
        }
#pragma unroll
        for (int j = 0; j < TILE_ROWS / 64; j++) {
            // row 64 j + lane: consumer 2 j + lane / 32, row tile (lane / 16) % 2, row lane % 16
            const int idx = (((2 * j + (lane >> 5)) * 16 + (lane & 15)) * RT + ((lane >> 4) & 1)) * UP;
            *reinterpret_cast<uint2 *>(mz + idx) = make_uint2(zr[j][0], zr[j][1]);
        }
    }

    __device__ __forceinline__ void load(const LoaderTile &T, int ch)
    {
        load_x(T, ch);
        if (T.bits != 16 && (li & 1) == 0 && (ch & 1) == 0) // (with one batch tile: loaders 0 and 2 own the even chunks)
            load_meta(T, ch >> 1);
    }
    __device__ __forceinline__ void store(int bits, int ch)
    {
        store_x(bits, ch % nxb(MT));
        if (bits != 16 && (li & 1) == 0 && (ch & 1) == 0)
            store_meta((ch >> 1) & 1);
    }

    // Until every consumer has finished the chunk numbered need - 1.
    __device__ __forceinline__ void await_consumers(int need)
    {
        const volatile FQ_LDS int *done = (const volatile FQ_LDS int *)(L.flag + 8);
        for (;;) {
            const int v = lane < CONSUMERS ? done[lane] : 0x7fffffff;
            if (!__ballot(v < need))
                break;
            __builtin_amdgcn_s_sleep(1);
        }
    }

    // Chunk c of the tile whose chunks start at number `base`, from the registers into LDS.  It
    // goes into the x buffer that chunk c - nxb(MT) was read from (the metadata of a pair of
    // chunks into the buffer of the pair before the last): written once every consumer has
    // finished that one.
    __device__ __forceinline__ void write(int bits, int base, int c)
    {
        if (c >= nxb(MT))
            await_consumers(base + c - nxb(MT) + 1);
        store(bits, c);
        __builtin_amdgcn_s_waitcnt(0xc07f); // lgkmcnt(0): the chunk is in LDS
        if (lane == 0)
            ((volatile FQ_LDS int *)L.flag)[li] = base + c + 1;
        __builtin_amdgcn_sched_barrier(0); // the registers are reused: no load before the last write
    }
};

// A tile as the workgroup's wavefronts find it in LDS: entry, tile of 256 rows, the selected
// bit-width (0: pass the tile over -- no such width in this kernel, or no copy of it attached)
// and the operands that go with it.  Sixteen words.
struct Tile {
    int e, t, bits;
    Sel d;
};

__device__ __forceinline__ void write_tile(int *mail, int e, int t, int bits, const Sel &d)
{
    volatile FQ_LDS int *m = (volatile FQ_LDS int *)mail;
    const uint64_t p[5] = {(uint64_t)(uintptr_t)d.codes, (uint64_t)(uintptr_t)d.scales, (uint64_t)(uintptr_t)d.zeros,
                           (uint64_t)(uintptr_t)d.x, (uint64_t)(uintptr_t)d.y};
    m[0] = e, m[1] = t, m[2] = bits, m[3] = d.N, m[4] = d.K;
#pragma unroll
    for (int i = 0; i < 5; i++) {
        m[5 + 2 * i] = (int)(uint32_t)p[i];
        m[6 + 2 * i] = (int)(uint32_t)(p[i] >> 32);
    }
}

__device__ __forceinline__ Tile read_tile(const int *mail)
{
    const volatile FQ_LDS int *m = (const volatile FQ_LDS int *)mail;
    int w[15];
#pragma unroll
    for (int i = 0; i < 15; i++)
        w[i] = __builtin_amdgcn_readfirstlane(m[i]);
    auto ptr = [&](int i) { return (uintptr_t)((uint64_t)(uint32_t)w[5 + 2 * i] | ((uint64_t)(uint32_t)w[6 + 2 * i] << 32)); };
    Tile T;
    T.e = w[0], T.t = w[1], T.bits = w[2];
    T.d.N = w[3], T.d.K = w[4];
    T.d.codes = (const uint8_t *)ptr(0);
    T.d.scales = (const float *)ptr(1);
    T.d.zeros = (const uint8_t *)ptr(2);
    T.d.x = (const uint16_t *)ptr(3);
    T.d.y = (uint16_t *)ptr(4);
    return T;
}

// The tiles of one workgroup: the roles walk the same tiles in separate loops so that neither
// carries the other's registers.  All wavefronts run every tile (rows past N are clamped on load
// and masked on store) so that every one of them takes part in the hand-over of every chunk and
// reaches the barrier at the end.
//
// Workgroups are dealt to the 8 XCDs in turn.  Tiles are handed out so that an XCD takes runs of
// XCD_RUN consecutive tiles: the x of a linear is then fetched into a few L2s rather than into all
// eight, while a linear's weight rows are still spread over several XCDs (measured on the mixed 7B
// step at batch 16: 1.362 / 1.347 / 1.348 / 1.349 / 1.351 ms for runs of 1 / 4 / 8 / 16 / 32; 8 is
// also the best for each single width).  Within an XCD the workgroups draw their tiles from a
// queue (`queue[xcd]`, a cursor in device memory): tiles take very different times (a fp16 tile
// four times as long as a 4-bit one) and a fixed deal leaves the workgroups with the long ones
// running alone at the end.  The queue runs over the tiles of the entries this kernel serves at
// this launch's bit-widths, in table order, as listed by plan_order_kernel just before the launch
// (entries at a width that is not attached cost nothing).  Loader 1 draws the next tile while the current one runs, at a point where it would
// otherwise wait for the consumers (the round trip of the atomic is not hidden anywhere on the
// way into a tile), looks up its entry and the operands of the entry's selected width, and leaves
// them in LDS (`mail`, two records used in turn): everybody reads a tile's record after the
// barrier that ends the tile before it -- LDS, not two dependent reads of device memory, stands
// between that barrier and the tile's first requests -- and the other record is written during
// the tile.  The loaders read it before that barrier (the others once loader 1 has counted the
// draw in flag[4]) and request their first chunk of the next tile, and so do the consumers, if
// the draw has been counted by then, for the first stages of their next tile.  The last workgroup to finish
// puts the cursors back to zero for the next launch.
template <int MT, int ROLE> // ROLE: 0 = consumer, 1 = loader
__device__ __forceinline__ void run_tiles(const FqLinearDesc *table, const int32_t *bits_dev, int M, const Lds &L,
                                          int wave, int *queue, const int2 *order, int *mail)
{
    constexpr int XCD_RUN = 8;
    const int li = wave - CONSUMERS; // a loader's number
    const bool draws = ROLE == 1 && li == 1;
    const int grid = gridDim.x;
    const int xcd = blockIdx.x & 7;
    const int listed_tiles = queue[FQ_Q_TILES], entries = queue[FQ_Q_ENTRIES];
    int drawn = 0;
    auto draw = [&](int lane, int *rec) { // whole wavefront; rec: the record to fill
        int q = 0;
        if (lane == 0)
            q = __hip_atomic_fetch_add(&queue[xcd], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        q = __builtin_amdgcn_readfirstlane(q);
        // the XCD's q-th tile: tile q % XCD_RUN of its run number q / XCD_RUN
        const int v = ((q / XCD_RUN) * 8 + xcd) * XCD_RUN + q % XCD_RUN;
        int e = -1, t = 0;
        if (v < listed_tiles) {
            for (int first = 0; first < entries; first += 64) { // the entry whose tiles [first, next first) hold v
                const int r = first + lane;
                const int2 o = r < entries ? order[r] : make_int2(0x7fffffff, 0);
                const int next = r + 1 < entries ? order[r + 1].x : listed_tiles;
                const uint64_t hit = __ballot(r < entries && o.x <= v && v < next);
                if (hit) {
                    const int src = __builtin_ctzll(hit);
                    e = __shfl(o.y, src, 64);
                    t = v - __shfl(o.x, src, 64);
                    break;
                }
            }
        }
        e = __builtin_amdgcn_readfirstlane(e);
        t = __builtin_amdgcn_readfirstlane(t);
        Sel d;
        d.codes = nullptr, d.scales = nullptr, d.zeros = nullptr, d.x = nullptr, d.y = nullptr, d.N = 0, d.K = 0;
        int bits = 0;
        if (e >= 0) {
            const FqLinearDesc *dp = &table[e];
            bits = bits_dev[e];
            d.N = dp->N;
            d.K = dp->K;
            d.codes = bits == 4   ? dp->codes4
                      : bits == 8 ? dp->codes8
                      : bits == 2 ? dp->codes2
                      : bits == 16 ? (const uint8_t *)dp->w16
                                   : nullptr;
            d.scales = bits == 4 ? dp->scales4 : bits == 2 ? dp->scales2 : dp->scales8;
            d.zeros = bits == 4 ? dp->zeros4 : bits == 2 ? dp->zeros2 : dp->zeros8;
            d.x = dp->x;
            d.y = dp->y;
            if (!d.codes)
                bits = 0;
        }
        drawn++;
        if (lane == 0) {
            write_tile(rec, e, t, bits, d);
            ((volatile FQ_LDS int *)L.flag)[4] = drawn; // after the record: a wavefront's LDS writes keep their order
        }
        __builtin_amdgcn_s_waitcnt(0xc07f); // lgkmcnt(0): written before this wavefront's next barrier
    };
    if (draws)
        draw(threadIdx.x & 63, mail);
    __syncthreads();
    int base = 0; // chunks of the tiles run so far
    if (ROLE == 0) {
        Tile cur = read_tile(mail);
        Ahead ahead;
        ahead.pf = 0, ahead.slot0 = 0;
        for (int par = 0, tileno = 0; cur.e >= 0; par ^= 1, tileno++) {
            if (cur.bits == 0) {
                __syncthreads(); // a tile that is passed over
            } else {
                const int tile_row0 = cur.t * TILE_ROWS;
                if (cur.bits == 4)
                    ahead = Consumer<4, MT>(cur.d, L, M, tile_row0, wave, base, tileno).run(ahead);
                else if (cur.bits == 8)
                    ahead = Consumer<8, MT>(cur.d, L, M, tile_row0, wave, base, tileno).run(ahead);
                else if (cur.bits == 2)
                    ahead = Consumer<2, MT>(cur.d, L, M, tile_row0, wave, base, tileno).run(ahead);
                else
                    ahead = Consumer<16, MT>(cur.d, L, M, tile_row0, wave, base, tileno).run(ahead);
                base += (cur.d.K + KC - 1) / KC;
            }
            cur = read_tile(mail + 16 * (par ^ 1));
        }
    } else {
        // One batch tile: loader li owns the chunks li, li + LOADERS, ... (the owner of an even
        // chunk with it the metadata, whose pairs start at even chunks) and requests its next
        // chunk as soon as it has written one.  Two batch tiles: loader li owns batch tile li % 2
        // of the chunks li / 2, li / 2 + LOADERS / 2, ...  After its last chunk of a tile a loader
        // requests its first chunk of the next tile (a request made at the start of a tile would
        // return behind the 64 KiB of weights that the consumers ask for at the same moment, and
        // they would wait for it), from the same place in the code: the walk starts with a tile
        // of no chunks before the first one, and a tile that is passed over is one of no chunks.
        // Loader 1 draws the tile after the current one once it has written its first chunk and
        // requested its second -- where it has time to spare -- or, in a tile where its first
        // turn is the last, before the request.
        constexpr int STEP = MT == 1 ? LOADERS : LOADERS / 2; // distance between the chunks of one loader
        const int c0 = MT == 1 ? li : li >> 1;
        auto as_loader_tile = [&](const Tile &T) {
            LoaderTile A;
            A.d = T.d;
            A.tile_row0 = T.t * TILE_ROWS;
            A.G = T.d.K >> 7;
            A.bits = T.bits;
            A.nchunks = T.e >= 0 && T.bits ? (T.d.K + KC - 1) / KC : 0;
            return A;
        };
        Loader<MT> ld(L, M, li);
        LoaderTile A; // the current tile; at first: none
        A.d.codes = nullptr, A.d.scales = nullptr, A.d.zeros = nullptr, A.d.x = nullptr, A.d.y = nullptr;
        A.d.N = 0, A.d.K = 0, A.tile_row0 = 0, A.G = 0, A.nchunks = 0, A.bits = 0;
        bool real = false;
        // record of the tile after A: tile number i of the workgroup is in record i % 2
        for (int par = 1, tileno = -1;; par ^= 1, tileno++) {
            int *rec = mail + 16 * (par ^ 1);
            Tile T; // the tile after A, read on A's last turn
            T.e = -1, T.t = 0, T.bits = 0, T.d = A.d;
            LoaderTile B = A;
            for (int c = c0;; c += STEP) {
                const bool last = c + STEP >= A.nchunks;
                if (c < A.nchunks)
                    ld.write(A.bits, base, c);
                if (last) { // what comes after A
                    if (draws && real && c == c0)
                        draw(threadIdx.x & 63, rec);
                    if (!draws) // until loader 1 has drawn it
                        while (__builtin_amdgcn_readfirstlane(((volatile FQ_LDS int *)L.flag)[4]) < tileno + 2)
                            __builtin_amdgcn_s_sleep(1);
                    T = read_tile(rec);
                    B = as_loader_tile(T);
                }
                // (field by field: a choice between the two objects would keep both in memory)
                LoaderTile from;
                from.d.codes = nullptr, from.d.y = nullptr;
                from.d.x = last ? B.d.x : A.d.x;
                from.d.scales = last ? B.d.scales : A.d.scales;
                from.d.zeros = last ? B.d.zeros : A.d.zeros;
                from.d.N = last ? B.d.N : A.d.N;
                from.d.K = last ? B.d.K : A.d.K;
                from.tile_row0 = last ? B.tile_row0 : A.tile_row0;
                from.G = last ? B.G : A.G;
                from.nchunks = last ? B.nchunks : A.nchunks;
                from.bits = last ? B.bits : A.bits;
                const int ch = last ? c0 : c + STEP;
                if (ch < from.nchunks)
                    ld.load(from, ch);
                if (draws && real && c == c0 && !last)
                    draw(threadIdx.x & 63, rec);
                if (last)
                    break;
            }
            if (real) {
                __builtin_amdgcn_s_waitcnt(0xc07f);
                barrier(); // the consumers have stored the tile and read its last chunk (or pass it over)
                base += A.nchunks;
            }
            if (T.e < 0)
                break;
            A = B;
            real = true;
        }
    }
    if (draws && (threadIdx.x & 63) == 0) {
        const int done = __hip_atomic_fetch_add(&queue[FQ_Q_DONE], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (done == grid - 1) { // every workgroup has drawn its last tile
            for (int i = 0; i <= FQ_Q_DONE; i++)
                __hip_atomic_store(&queue[i], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// Inclusive scan over the 256 threads of plan_order_kernel; `total` returns the sum.
__device__ __forceinline__ int scan256(int v, int *tmp, int &total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(v, off, 64);
        if (lane >= off)
            v += o;
    }
    __syncthreads(); // tmp may still be read from a previous call
    if (lane == 63)
        tmp[wave] = v;
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < 4; w++) {
        all += tmp[w];
        if (w < wave)
            before += tmp[w];
    }
    total = all;
    return v + before;
}

// What a batched plan launch runs under this launch's bit-widths, in table order: the entries at
// 2, 4, 8 or 16 bits whose copy is attached, in 256-row tiles.  order[r] = (first tile of the r-th
// such entry, entry); queue[FQ_Q_TILES] = their tiles, queue[FQ_Q_ENTRIES] = their number.  An
// entry at another width (3 bits) or without that copy is left out and flagged.  One workgroup.
__global__ __launch_bounds__(256) void plan_order_kernel(const FqLinearDesc *__restrict__ table,
                                                         const int32_t *__restrict__ bits_dev, int count, int *queue,
                                                         int2 *order)
{
    __shared__ int tmp[4];
    int first_tile = 0, first_rank = 0;
    for (int base = 0; base < count; base += 256) {
        const int e = base + threadIdx.x;
        int tiles = 0;
        bool listed = false;
        if (e < count) {
            const FqLinearDesc &d = table[e];
            const int bits = bits_dev[e];
            if ((bits == 16 && d.w16) || (bits == 8 && d.codes8) || (bits == 4 && d.codes4) || (bits == 2 && d.codes2)) {
                listed = true;
                tiles = (d.N + TILE_ROWS - 1) / TILE_ROWS;
            } else {
                queue[FQ_Q_FLAGS] = 1; // no such width here, or no copy of it: nobody runs this entry
            }
        }
        int sum_t, sum_e;
        const int incl_t = scan256(tiles, tmp, sum_t);
        const int incl_e = scan256(listed ? 1 : 0, tmp, sum_e);
        if (listed)
            order[first_rank + incl_e - 1] = make_int2(first_tile + incl_t - tiles, e);
        first_tile += sum_t;
        first_rank += sum_e;
    }
    if (threadIdx.x == 0) {
        queue[FQ_Q_TILES] = first_tile;
        queue[FQ_Q_ENTRIES] = first_rank;
    }
}

template <int MT>
__global__ __launch_bounds__(THREADS) void decode_stream_kernel(const FqLinearDesc *__restrict__ table,
                                                                const int32_t *__restrict__ bits_dev, int count,
                                                                int total_tiles, int M, int *queue,
                                                                const int2 *__restrict__ order)
{
    __shared__ __attribute__((aligned(16))) int mail[32];
    __shared__ __attribute__((aligned(8))) int flag[16];
    __shared__ __attribute__((aligned(1024))) uint8_t ring[CONSUMERS * NS * STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) uint8_t xbuf[nxb(MT) * 16 * MT * KC * 2];
    __shared__ __attribute__((aligned(256))) float ms0[UP * TILE_ROWS], ms1[UP * TILE_ROWS];
    __shared__ __attribute__((aligned(256))) uint8_t mz0[UP * TILE_ROWS], mz1[UP * TILE_ROWS];
    Lds L;
    L.ring = ring;
    L.x = xbuf;
    L.ms[0] = ms0, L.ms[1] = ms1;
    L.mz[0] = mz0, L.mz[1] = mz1;
    L.flag = flag;
    L.mail = mail;
    if (threadIdx.x < 16)
        flag[threadIdx.x] = 0; // before the barrier that run_tiles starts with
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (wave >= CONSUMERS)
        run_tiles<MT, 1>(table, bits_dev, M, L, wave, queue, order, mail);
    else
        run_tiles<MT, 0>(table, bits_dev, M, L, wave, queue, order, mail);
}

} // namespace

// A plan launch (device table of `count` linears, device-side bit-widths) for 2 <= M <= 32 and
// tiles of 256 rows.  `queue`: 16 ints in device memory that belong to the plan, zeroed once (the
// kernel leaves the cursors zeroed), and `order`: `count` pairs of ints of the plan's.  The
// queue hands out runs of 8 tiles to the 8 XCDs in turn: the grid (one workgroup per compute unit)
// must be a multiple of 64, which the plan's layout sees to (other devices get smaller tiles and
// the register-fed kernel).

hipError_t fq_launch_skinny_stream(const FqLinearDesc *descs_dev, const int32_t *bits_dev, int count, int total_tiles,
                                   int M, int cus, int *queue, void *order, hipStream_t stream)
{
    // one workgroup per CU (LDS): persistent over the tiles
    const int grid = total_tiles < cus ? total_tiles : cus;
    if (!queue || !order || grid % 64 != 0)
        return hipErrorInvalidValue;
    // what this launch runs, under its bit-widths
    plan_order_kernel<<<1, 256, 0, stream>>>(descs_dev, bits_dev, count, queue, (int2 *)order);
    if (M <= 16)
        decode_stream_kernel<1><<<grid, THREADS, 0, stream>>>(descs_dev, bits_dev, count, total_tiles, M, queue,
                                                              (const int2 *)order);
    else
        decode_stream_kernel<2><<<grid, THREADS, 0, stream>>>(descs_dev, bits_dev, count, total_tiles, M, queue,
                                                              (const int2 *)order);
    return hipGetLastError();
}
