// Decode-phase weight-only quantized linear for small batches (2 <= M <= 32), streaming
// kernel for launches with many 256-row tiles: y[M][N] = x[M][K] . dequant(W[N][K])^T,
// dequant = Sec. 2.2 Eq. (3).  The phase is bound by the weight stream (Sec. 4.1); the
// contraction runs on v_mfma_f32_16x16x32_f16 (A = x: 16 batch rows x 32 k, B = 16 weight
// rows x 32 k, binary32 accumulation; two batch tiles above 16 rows).  Launches with few or
// narrow tiles and single calls stay with the register-fed small-batch kernel.
//
// Work split.  A workgroup owns a tile of 256 weight rows at a time and has twelve wavefronts,
// three per SIMD: eight consumers (two per SIMD, so that one computes while the other waits),
// 32 rows = 2 MFMA row tiles each, and four loaders.  A workgroup's tiles (blockIdx.x,
// + gridDim.x, ...) and the 512-k chunks of each form one list that every wavefront walks on
// its own; one barrier per chunk is where they meet, and there is none between tiles.
//
// Weight stream.  A stage is one 128-byte line of each of the consumer's 32 rows (256 / 128 /
// 64 k at 4 / 8 / 16 bits); a load instruction covers 8 rows x 128 bytes, whole lines only
// (halves of a line requested apart are fetched from HBM twice more often than not), marked
// non-temporal (read once).  Stages go from global memory straight into a wavefront-private
// LDS ring of two slots with direct-to-LDS loads (global_load_lds_dwordx4): no register
// staging, and the only synchronisation the stream needs is a counted s_waitcnt vmcnt(n) of
// the wavefront on its own operations.  A step waits for its stage, copies it to registers
// together with the x blocks and the scales / zero points it needs, and at once requests the
// stage two steps ahead into the slot it has just emptied: two stages per consumer, 64 KiB per
// CU, are in flight while the step computes (three measured the same: the memory system is the
// limit, not the depth).  When a tile's stages have all been requested the requests go on with
// the first stages of the workgroup's next tile, so that it starts with its ring full (the
// counted waits of its first steps do not allow for the stores of the tile before: those have
// to be through as well).  The LDS reads are inline assembly: the compiler cannot tell a read of
// a run-time slot from the slots being filled and would wait for every outstanding load first.
//
// Loaders.  x and the metadata are what the stream cannot carry: a scale or zero-point fetch
// per stage touches one cache line per row (64 tiny requests per instruction, more than the
// weights themselves need), and the 4-bit path wants x permuted.  Four more wavefronts fetch
// them with ordinary loads -- their own vmcnt, nobody else waits.  Two fetch x in chunks of
// 512 k, each every other chunk, requested two chunk periods before they are due: 16-byte
// blocks of 8 halves, one request of 1 KiB per batch row and chunk, stored [k block][batch
// row] with the rows of k block kb XOR-ed by kb % 8 + 8 (kb / 32) -- conflict free for the
// writer, whose lanes are k blocks (a 128-bit LDS write goes eight lanes at a time), and for the
// readers, whose lanes are batch rows (measured: a 128-bit read runs at full rate only if lanes
// 0 .. 7 and 8 .. 15 of every group of 16 lanes use different halves of the 256 bytes and the
// same ones in all four groups, i.e. whatever the k block) -- zero past K, for the
// 4-bit path permuted inside the block to the order the unpacking produces (x0 x4 x1 x5 x2 x6
// x3 x7).  Two fetch scales and zero points, half the tile's rows each, 32 units (4096 k) of a
// row at a time -- a whole line of scales where rows start on one -- keep them in registers
// and write them to LDS a pair of chunks (8 units) at a time, stored [consumer][row][row
// tile][unit].  The loaders run ahead through the list: the first chunks of a tile are in LDS
// before the consumers have finished the one before.
//
// Dequantization.  Codes become halves by bit tricks ((w & 0x000F000F) | 0x64006400 is the
// pair (1024 + q0, 1024 + q4); nibbles in bits 4..7 use exponent 0x54 = 64 + q; bytes go
// under 0x64 with v_perm_b32).  The offsets and the zero point are not subtracted per weight:
// a second MFMA per operand multiplies the same x block by the constant -(offset + z), so
// that the accumulator holds sum x (q - z) over the stage (every product is exact in
// binary32), which is folded as out += s * acc -- Eq. (3) with the scale factored out of the
// group.  The vector ALUs are left with the unpacking (5 instructions per 8 four-bit weights).
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

constexpr int CONSUMERS = 8;
constexpr int LOADERS = 4;                     // two for x, two for the scales and zero points
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

// Workgroup barrier without the fence of __syncthreads() (which would wait for every
// outstanding load, i.e. drain the rings); the waits that matter are issued explicitly.
__device__ __forceinline__ void barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
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

// The workgroup's LDS.  x and metadata buffers come in pairs (chunk parity).
struct Lds {
    uint8_t *ring;    // [CONSUMERS][NS][STAGE_BYTES]
    uint8_t *x[2];    // [KC / 8][16 * MT] blocks of 16 bytes; k block kb holds batch row m at place m ^ (kb % 8 + 8 (kb / 32))
    float *ms[2];     // [CONSUMERS][16 rows][RT][UP] scales of a pair of chunks
    uint8_t *mz[2];   // same order, zero points
};

// What a step holds in registers: the stage's weights (pieces c and c + 4 of the lane's line in
// each row tile), the scales and zero points of the lane's row in each row tile for the stage's
// units, and x blocks the lane supplies to the stage's MFMAs: 8 / 4 / 2 per batch tile at 4 / 8 /
// 16 bits; with two batch tiles the 4-bit stage takes its 16 in two rounds, one per unit.
struct Stage {
    u32x4 w[RT][2];
    float s[RT][2]; // [row tile][unit of the stage] (8 bits: one unit)
    uint32_t z;     // byte 2 * rt + unit
    u32x4 a[8];
};

typedef float float2_t __attribute__((ext_vector_type(2)));

// Wait until at most n of the wavefront's vector memory operations are outstanding (n is rounded
// down to a value that has an instruction here).  n counts the loads of the stages requested
// after the one waited for; loads complete in order among themselves.  The stores of a tile's
// outputs, which may sit between the stages in flight, are never allowed for: whatever their
// order of completion relative to the loads, the stage waited for has then arrived.
__device__ __forceinline__ void wait_vm(int n)
{
    n = __builtin_amdgcn_readfirstlane(n);
    if (NS > 2 && n >= 2 * SOPS)
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * SOPS) : "memory");
    else if (n >= SOPS)
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(SOPS) : "memory");
    else
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// Copy a ring slot, the metadata and the stage's x blocks to registers (after wait_vm for the
// slot's stage).  `wa`, `wb`: LDS byte addresses of the lane's two pieces in row tile 0 of the
// slot; `sa`, `za`: of the lane's scales and zero points for row tile 0 (row tile 1: UP entries
// further); `xa`: of the lane's x blocks.  All of it is inline assembly on purpose: the compiler
// cannot tell these reads from the slots being filled and would wait for every outstanding load
// first.
// Which x blocks land in st.a: 4 bits, MT = 1: [unit][i]; 4 bits, MT = 2: [batch tile][i] of
// unit 0 (unit 1 follows with more_x); 8 bits: [batch tile][half][i]; 16 bits: [batch tile][half].
template <int BITS, int MT>
__device__ __forceinline__ void take(uint32_t wa, uint32_t wb, uint32_t sa, uint32_t za, const uint32_t (&xa)[4],
                                     Stage &st)
{
    if constexpr (BITS == 4) {
        float2_t s0, s1;
        uint32_t z0, z1;
        asm volatile("ds_read_b128 %0, %16\n\t"
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
                     "ds_read_b128 %12, %20 offset:%24\n\t"
                     "ds_read_b128 %13, %21 offset:%24\n\t"
                     "ds_read_b128 %14, %22 offset:%24\n\t"
                     "ds_read_b128 %15, %23 offset:%24\n\t"
                     "s_waitcnt lgkmcnt(0)"
                     : "=&v"(st.w[0][0]), "=&v"(st.w[0][1]), "=&v"(st.w[1][0]), "=&v"(st.w[1][1]), "=&v"(s0), "=&v"(s1),
                       "=&v"(z0), "=&v"(z1), "=&v"(st.a[0]), "=&v"(st.a[1]), "=&v"(st.a[2]), "=&v"(st.a[3]),
                       "=&v"(st.a[4]), "=&v"(st.a[5]), "=&v"(st.a[6]), "=&v"(st.a[7])
                     : "v"(wa), "v"(wb), "v"(sa), "v"(za), "v"(xa[0]), "v"(xa[1]), "v"(xa[2]), "v"(xa[3]),
                       "n"(MT == 1 ? 4096 : 256) // the second unit, or the second batch tile of the first unit
                     : "memory");
        st.s[0][0] = s0.x, st.s[0][1] = s0.y, st.s[1][0] = s1.x, st.s[1][1] = s1.y;
        st.z = z0 | (z1 << 16);
    } else if constexpr (BITS == 8) {
        uint32_t z0, z1;
        if constexpr (MT == 1) {
            asm volatile("ds_read_b128 %0, %12\n\t"
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
                         : "v"(wa), "v"(wb), "v"(sa), "v"(za), "v"(xa[0]), "v"(xa[1]), "v"(xa[2]), "v"(xa[3])
                         : "memory");
        } else {
            asm volatile("ds_read_b128 %0, %16\n\t"
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
                         : "v"(wa), "v"(wb), "v"(sa), "v"(za), "v"(xa[0]), "v"(xa[1]), "v"(xa[2]), "v"(xa[3])
                         : "memory");
        }
        st.z = z0 | (z1 << 16);
    } else {
        if constexpr (MT == 1) {
            asm volatile("ds_read_b128 %0, %6\n\t"
                         "ds_read_b128 %1, %7\n\t"
                         "ds_read_b128 %2, %6 offset:2048\n\t"
                         "ds_read_b128 %3, %7 offset:2048\n\t"
                         "ds_read_b128 %4, %8\n\t"
                         "ds_read_b128 %5, %9\n\t"
                         "s_waitcnt lgkmcnt(0)"
                         : "=&v"(st.w[0][0]), "=&v"(st.w[0][1]), "=&v"(st.w[1][0]), "=&v"(st.w[1][1]), "=&v"(st.a[0]),
                           "=&v"(st.a[1])
                         : "v"(wa), "v"(wb), "v"(xa[0]), "v"(xa[1])
                         : "memory");
        } else {
            asm volatile("ds_read_b128 %0, %8\n\t"
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
                         : "v"(wa), "v"(wb), "v"(xa[0]), "v"(xa[1])
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

template <int BITS>
struct Cfg {
    static constexpr int KPS = 128 * 8 / BITS; // k per stage: 256 / 128 / 64
    static constexpr int SPC = KC / KPS;       // steps per chunk: 2 / 4 / 8
};

// ------------------------------------------------------------------ the workgroup's work list
// The tiles of a workgroup (blockIdx.x, + gridDim.x, ...; entries whose selected width is not
// attached are passed over) and the chunks of each, numbered through: every wavefront of the
// workgroup walks the same list on its own, at its own distance ahead, and meets the others at
// one barrier per chunk.  All of it is wave-uniform.
struct Walk {
    const FqLinearDesc *table;
    const int32_t *bits_dev;
    int count, total_tiles;
    int tile, e; // tile >= total_tiles: the list has ended
    Sel d;
    int bits, tile_row0, nchunks;
    int ch; // chunk inside the tile
    int g;  // chunks before it in the list: its parity names the x buffer
    int p;  // pairs of chunks before its pair (pairs do not span tiles): parity of the metadata buffer

    __device__ __forceinline__ bool valid() const { return tile < total_tiles; }

    __device__ __forceinline__ void seek()
    {
        const int grid = gridDim.x;
        for (; tile < total_tiles; tile += grid) {
            while (e + 1 < count && tile >= table[e + 1].tile_begin)
                e++;
            const FqLinearDesc *dp = &table[e];
            bits = bits_dev[e];
            d.codes = bits == 4 ? dp->codes4 : bits == 8 ? dp->codes8 : bits == 16 ? (const uint8_t *)dp->w16 : nullptr;
            if (!d.codes)
                continue;
            d.scales = bits == 4 ? dp->scales4 : dp->scales8;
            d.zeros = bits == 4 ? dp->zeros4 : dp->zeros8;
            d.x = dp->x;
            d.y = dp->y;
            d.N = dp->N;
            d.K = dp->K;
            tile_row0 = (tile - dp->tile_begin) * TILE_ROWS;
            nchunks = (d.K + KC - 1) / KC;
            return;
        }
    }

    __device__ __forceinline__ void start(const FqLinearDesc *table_, const int32_t *bits_dev_, int count_,
                                          int total_tiles_)
    {
        table = table_, bits_dev = bits_dev_, count = count_, total_tiles = total_tiles_;
        tile = blockIdx.x, e = 0, ch = 0, g = 0, p = 0;
        bits = 0, tile_row0 = 0, nchunks = 0;
        d = Sel{nullptr, nullptr, nullptr, nullptr, nullptr, 1, 0};
        seek();
    }

    __device__ __forceinline__ void next_tile()
    {
        tile += gridDim.x;
        ch = 0;
        seek();
    }

    __device__ __forceinline__ void next_chunk()
    {
        g++;
        if (ch + 1 >= nchunks) {
            p++;
            next_tile();
        } else {
            ch++;
            p += (ch & 1) == 0;
        }
    }

    // From the first chunk of a tile to the first chunk of the next one.
    __device__ __forceinline__ void skip_tile()
    {
        g += nchunks;
        p += (nchunks + 1) >> 1;
        next_tile();
    }
};

// ------------------------------------------------------------------ consumer wavefronts
// Where a consumer's 32 rows of a tile lie in the code array (wave-uniform).
struct Rows {
    const uint8_t *gbase; // first byte of the first row
    uint32_t row_bytes;   // a multiple of 64
    int T;                // steps: 128-byte lines of a row (the last may be half a line at 4 bits); 0: no tile
    int lastrel;          // rows past N repeat row N - 1: the last row's distance from the first
    bool four;            // 4-bit codes

    __device__ __forceinline__ void set(const Walk &w, int wave)
    {
        row_bytes = (uint32_t)(w.d.K * w.bits) >> 3;
        T = (int)((row_bytes + 127) >> 7);
        // the wavefront's rows span at most 32 * row_bytes < 4 GiB: 32-bit lane offsets from a uniform base
        const int first = min(w.tile_row0 + wave * RT * 16, w.d.N - 1);
        gbase = w.d.codes + (size_t)first * (size_t)row_bytes;
        lastrel = w.d.N - 1 - first;
        four = w.bits == 4;
    }
    __device__ __forceinline__ void none()
    {
        gbase = nullptr, row_bytes = 0, T = 0, lastrel = 0, four = false;
    }
};

// A consumer's weight stream: the ring and the requests, which run on from a tile into the first
// stages of the next one, so that a new tile starts with its ring full.
struct Stream {
    uint8_t *ring;    // this wavefront's NS slots
    int rslot, wslot; // slot of the oldest stage in flight; slot of the next request
    int infl;         // stages in flight
    Rows cur, nxt;    // the tile being computed, the one after it
    int fq, nfq;      // stages requested so far of either
    // per-lane constants of the weight loads: load i of a stage covers rows 8 i .. 8 i + 7 of the
    // wavefront's 32, lane -> row lane / 8 of those, LDS slot lane % 8, i.e. piece
    // slot ^ ((row % 16) >> 1) of the line
    uint32_t r;    // lane / 8
    uint32_t pc16; // 16 * piece in even loads; odd loads: the piece 4 further, 16 * piece ^ 64

    __device__ __forceinline__ Stream(const Lds &L, int wave)
    {
        const uint32_t lane = threadIdx.x & 63;
        ring = L.ring + wave * NS * STAGE_BYTES;
        rslot = wslot = infl = fq = nfq = 0;
        r = lane >> 3;
        pc16 = ((lane & 7) ^ (r >> 1)) * 16;
        cur.none(), nxt.none();
    }

    // Request stages, of the current tile and then of the next, while a slot is free (one per
    // step in the steady state).  A 4-bit row may end with half a line: the lanes of the missing
    // half re-read the present one (their x is zero).
    __device__ __forceinline__ void request()
    {
#pragma nounroll
        while (infl < NS) {
            const bool c = fq < cur.T;
            if (!c && nfq >= nxt.T)
                break;
            const int q = c ? fq : nfq;
            const uint32_t row_bytes = c ? cur.row_bytes : nxt.row_bytes;
            const int lastrel = c ? cur.lastrel : nxt.lastrel;
            const bool four = c ? cur.four : nxt.four;
            const uint8_t *base = (c ? cur.gbase : nxt.gbase) + (size_t)q * 128;
            uint8_t *dst = ring + wslot * STAGE_BYTES;
            const uint32_t keep = four && (uint32_t)q * 128 + 64 >= row_bytes ? ~64u : ~0u; // pieces 4..7 -> 0..3
#pragma unroll
            for (int i = 0; i < SOPS; i++) {
                const uint32_t rel = (uint32_t)min((int)(8 * i + r), lastrel);
                const uint32_t off = rel * row_bytes + ((pc16 ^ (64u * (i & 1))) & keep);
                __builtin_amdgcn_global_load_lds((const FQ_GLOBAL void *)(base + off), (FQ_LDS void *)(dst + i * 1024),
                                                 16, 0, 2 /* nt: the weights are read once */);
            }
            fq += c, nfq += !c;
            wslot = wslot == NS - 1 ? 0 : wslot + 1;
            infl++;
        }
    }

    // Loads younger than those of the oldest stage in flight.
    __device__ __forceinline__ int younger() const { return (infl - 1) * SOPS; }

    // The oldest stage has been copied out of its slot.
    __device__ __forceinline__ void taken()
    {
        rslot = rslot == NS - 1 ? 0 : rslot + 1;
        infl--;
    }

    // The current tile is done and its outputs have been stored: go on to the next.
    __device__ __forceinline__ void advance()
    {
        cur = nxt;
        fq = nfq;
        nfq = 0;
        nxt.none();
    }
};

template <int BITS, int MT>
struct Consumer {
    typedef Cfg<BITS> C;
    Stream &S;
    const Lds &L;
    const int lane, n, c;
    uint32_t wa0, wb0; // LDS addresses for take(): the lane's pieces c and c + 4 in slot 0
    uint32_t ml;       // wave * 16 + n: the lane's place in the metadata of a pair of chunks
    // byte offsets of the lane's x blocks inside a stage's blocks (block kb of the chunk holds
    // batch row n at place n ^ (kb % 8 + 8 (kb / 32))).  4 bits: blocks 4 c + i of either unit; 8 bits: blocks 8 h + 2 c + i;
    // 16 bits: blocks 4 h + c of an even stage, 8 + 4 h + c of an odd one
    uint32_t xq[4];
    float4_t acc[RT][MT], out[RT][MT];

    __device__ __forceinline__ Consumer(Stream &S_, const Lds &L_, int wave)
        : S(S_), L(L_), lane(threadIdx.x & 63), n(lane & 15), c(lane >> 4)
    {
        wa0 = lds_addr(S.ring) + n * 128 + ((c ^ ((n >> 1) & 7)) * 16);
        wb0 = wa0 ^ 64; // piece c + 4
        ml = wave * 16 + n;
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int kb = BITS == 4 ? 4 * c + i : BITS == 8 ? 8 * (i >> 1) + 2 * c + (i & 1) : 4 * i + c;
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

    // One unit (128 k) of a 4-bit stage: half h of the line, x blocks a[mt * AM + i].
    template <int AM, int H>
    __device__ __forceinline__ void unit4(const Stage &st, const u32x4 *a)
    {
        constexpr int h = H;
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
#pragma unroll
                for (int mt = 0; mt < MT; mt++)
                    acc[rt][mt] = mfma(a[mt * AM + i], b, acc[rt][mt]);
            }
#pragma unroll
            for (int rt = 0; rt < RT; rt++)
#pragma unroll
                for (int mt = 0; mt < MT; mt++)
                    acc[rt][mt] = mfma(a[mt * AM + i], nz[rt], acc[rt][mt]);
        }
#pragma unroll
        for (int rt = 0; rt < RT; rt++)
#pragma unroll
            for (int mt = 0; mt < MT; mt++) {
                out[rt][mt] += st.s[rt][h] * acc[rt][mt];
                acc[rt][mt] = float4_t{0.f, 0.f, 0.f, 0.f};
            }
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
#pragma unroll
                        for (int mt = 0; mt < MT; mt++)
                            acc[rt][mt] = mfma(st.a[mt * 4 + 2 * h + i], b, acc[rt][mt]);
                    }
#pragma unroll
                    for (int rt = 0; rt < RT; rt++)
#pragma unroll
                        for (int mt = 0; mt < MT; mt++)
                            acc[rt][mt] = mfma(st.a[mt * 4 + 2 * h + i], nz[rt], acc[rt][mt]);
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

    // Chunk ch of the tile, whose x is in buffer xb and whose metadata is in buffer mb.
    __device__ __forceinline__ void chunk(int ch, int xb, int mb)
    {
        barrier(); // the loaders have written the chunk; everybody is done with the one before
        // metadata: buffer of the pair of chunks, the chunk's half of it, the lane's row
        const uint32_t mo = ml * (RT * UP) + (ch & 1) * UC;
        const uint32_t sbase = lds_addr(mb ? L.ms[1] : L.ms[0]) + mo * 4, zbase = lds_addr(mb ? L.mz[1] : L.mz[0]) + mo;
        uint32_t xbase = lds_addr(xb ? L.x[1] : L.x[0]);
        asm volatile("" : "+s"(xbase)); // opaque: or every stage's x addresses are hoisted out of the tile and spill
#pragma unroll
        for (int j = 0; j < C::SPC; j++) {
            const int q = ch * C::SPC + j;
            if (q >= S.cur.T)
                break;
            // where the stage sits inside the chunk: its first unit, its x blocks
            const int unit = j * C::KPS / 128;
            const uint32_t wa = wa0 + S.rslot * STAGE_BYTES, wb = wb0 + S.rslot * STAGE_BYTES, sa = sbase + unit * 4,
                           za = zbase + unit;
            uint32_t xa[4];
            // (k blocks 32 .. 63 of the chunk keep their batch rows in the other half of the places)
            if (BITS == 4) {
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
            wait_vm(S.younger());
            take<BITS, MT>(wa, wb, sa, za, xa, st);
            S.taken();
            S.request(); // into the slot just emptied: the stage NS steps ahead
            __builtin_amdgcn_sched_barrier(0); // keep the requests here: the scheduler sinks them otherwise
            compute(st, xa[0], xa[1], xa[2], xa[3]);
        }
    }

    // The tile at w (its first chunk).  The outputs leave through buffer stores: lanes with
    // nothing to store (batch rows past M, rows past N) point past the end of the buffer, where
    // the hardware drops the write -- no branches around the stores.
    __device__ __forceinline__ void run(const Walk &w, int M, int wave)
    {
        for (int ch = 0; ch < w.nchunks; ch++)
            chunk(ch, (w.g + ch) & 1, (w.p + (ch >> 1)) & 1);
        // D layout of the 16x16 MFMA: lane holds column n = lane % 16, rows 4 * (lane / 16) + r.
        const int N = w.d.N;
        const int row0 = w.tile_row0 + wave * RT * 16;
        const __amdgpu_buffer_rsrc_t yb =
            __builtin_amdgcn_make_buffer_rsrc((void *)w.d.y, 0, M * N * 2, 0x00020000 /* raw, 32-bit format */);
#pragma unroll
        for (int rt = 0; rt < RT; rt++) {
            const int row = row0 + rt * 16 + n;
#pragma unroll
            for (int mt = 0; mt < MT; mt++) {
                const float4_t v = BITS == 16 ? acc[rt][mt] : out[rt][mt];
#pragma unroll
                for (int r = 0; r < 4; r++) {
                    const int m = mt * 16 + c * 4 + r;
                    const int off = (m < M && row < N) ? (m * N + row) * 2 : (int)0x80000000u;
                    __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(short, (_Float16)v[r]), yb, off, 0, 0);
                }
            }
        }
        asm volatile("" ::: "memory");
    }
};

template <int MT>
__device__ __forceinline__ void consume(Walk w, const Lds &L, int M, int wave)
{
    Stream S(L, wave);
    S.cur.set(w, wave);
    bool first = true;
    while (w.valid()) {
        {
            Walk t = w; // look ahead: the tile after this one
            t.skip_tile();
            if (t.valid())
                S.nxt.set(t, wave);
        }
        if (first) {
            S.request();
            __builtin_amdgcn_sched_barrier(0);
            first = false;
        }
        if (w.bits == 4)
            Consumer<4, MT>(S, L, wave).run(w, M, wave);
        else if (w.bits == 8)
            Consumer<8, MT>(S, L, wave).run(w, M, wave);
        else
            Consumer<16, MT>(S, L, wave).run(w, M, wave);
        S.advance();
        w.skip_tile();
    }
}

// ------------------------------------------------------------------ loader wavefronts
// (One code path for the three bit-widths: instantiated per width, the register allocator sees
// three sets of staging registers live across the loop.)
template <int MT, int LI>
struct Loader {
    const Lds &L;
    const int M, lane;
    // a chunk's block `lane` of 16 batch rows (with two batch tiles: loader LI takes tile LI):
    // one 1 KiB request per row
    u32x4 xr[16];
    // what the registers hold: chunk h_g of the list (-1: nothing), of an entry of h_bits bits,
    // for x buffer h_xb
    int h_g, h_bits, h_xb;

    __device__ __forceinline__ Loader(const Lds &L_, int M_) : L(L_), M(M_), lane(threadIdx.x & 63), h_g(-1) {}

    __device__ __forceinline__ void load_x(const Sel &d, int ch)
    {
        const int k = ch * KC + lane * 8;

#pragma unroll
        for (int m = 0; m < 16; m++) {
            // batch rows past M feed outputs that are never stored; k past K meets re-read weights
            // (the missing half of a last line): x is zero there
            const int mm = min((MT == 2 ? 16 * LI : 0) + m, M - 1);
            xr[m] = k < d.K ? *(const FQ_GLOBAL u32x4 *)(d.x + (size_t)mm * d.K + k) : u32x4{0u, 0u, 0u, 0u};
        }
    }

    __device__ __forceinline__ void store_x()
    {
        u32x4 *xb = reinterpret_cast<u32x4 *>(h_xb ? L.x[1] : L.x[0]);
#pragma unroll
        for (int m = 0; m < 16; m++) {
            u32x4 p = xr[m];
            if (h_bits == 4) { // (x0 .. x7) -> (x0 x4 x1 x5 x2 x6 x3 x7), the unpack order
                p.x = __builtin_amdgcn_perm(xr[m].z, xr[m].x, 0x05040100u);
                p.y = __builtin_amdgcn_perm(xr[m].z, xr[m].x, 0x07060302u);
                p.z = __builtin_amdgcn_perm(xr[m].w, xr[m].y, 0x05040100u);
                p.w = __builtin_amdgcn_perm(xr[m].w, xr[m].y, 0x07060302u);
            }
            // conflict free for the writer and for the readers
            xb[lane * (16 * MT) + (MT == 2 ? 16 * LI : 0) + (m ^ ((lane & 7) | ((lane >> 2) & 8)))] = p;
        }
    }

    // Request the chunk at w.
    __device__ __forceinline__ void load(const Walk &w)
    {
        load_x(w.d, w.ch);
        h_g = w.g, h_bits = w.bits, h_xb = w.g & 1;
    }

    // w: this loader's next chunk.  Write what the registers hold, then request the loader's
    // next chunk (the registers are reused: no load before the last write).
    __device__ __forceinline__ void hand_over(Walk &w)
    {
        constexpr int STEP = MT == 1 ? 2 : 1; // distance between the chunks of one loader
        store_x();
        __builtin_amdgcn_sched_barrier(0);
        h_g = -1;
#pragma unroll
        for (int s = 0; s < STEP; s++)
            if (w.valid())
                w.next_chunk();
        if (w.valid())
            load(w);
    }

    // One batch tile: loader LI owns the chunks of parity LI in the list.  Chunk g + 1 is written
    // while the consumers work on chunk g, and the owner then requests chunk g + 3 at once.  Two
    // batch tiles: each loader owns one of them in every chunk and requests chunk g + 2 after
    // writing chunk g + 1.  The list runs through the tiles: the first chunks of a tile are
    // requested and written while the consumers are still in the one before.
    __device__ __forceinline__ void run(Walk w)
    {
        Walk b = w; // the chunk of the next barrier
        if (MT == 1 && LI == 1 && w.valid())
            w.next_chunk();
        if (w.valid())
            load(w);
        if (h_g == 0)
            hand_over(w);
        while (b.valid()) {
            __builtin_amdgcn_s_waitcnt(0xc07f); // lgkmcnt(0): this wavefront's LDS writes are done
            barrier();
            if (h_g == b.g + 1)
                hand_over(w);
            b.next_chunk();
        }
    }
};

// ------------------------------------------------------------------ metadata loader wavefronts
// Scales and zero points of rows 128 ML .. 128 ML + 127 of a tile.  They are fetched a block of
// 32 units (4096 k, eight chunks) at a time: 128 bytes of scales and 32 of zero points per row,
// i.e. whole lines of the scale array where a row starts on one -- fetched in smaller pieces, the
// pieces of a line arrive chunk periods apart and the line comes from HBM more than once.  The
// block stays in registers and is handed to the consumers a pair of chunks (UP units) at a time,
// in LDS as [consumer][row % 16][row tile][unit].  The next block (of this tile or the next) is
// requested when the last pair of the block has been written: two chunk periods before it is due.
template <int ML>
struct MetaLoader {
    static constexpr int BU = 32;        // units per block
    static constexpr int ROWS = TILE_ROWS / 2;
    const Lds &L;
    const int lane;
    float4_t sr[ROWS / 8]; // load i: rows 8 i + lane / 8, units 4 (lane % 8) .. + 3 of the block
    u32x4 zr[ROWS / 32];   // load j: rows 32 j + lane / 2, units 16 (lane % 2) .. + 15 of the block
    int h_tile, h_blk;     // the block in the registers (h_tile < 0: none)

    __device__ __forceinline__ MetaLoader(const Lds &L_) : L(L_), lane(threadIdx.x & 63), h_tile(-1), h_blk(0) {}

    // The block of the chunk at w.  Units past G (a last, partial block) repeat unit G - 1 (they
    // meet x = 0, so they must be finite), and rows past N repeat row N - 1.
    __device__ __forceinline__ void load(const Walk &w)
    {
        typedef float f32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));
        typedef uint32_t u32x4_a1 __attribute__((ext_vector_type(4), aligned(1)));
        const Sel &d = w.d;
        const int G = d.K >> 7;
        h_tile = w.tile, h_blk = w.ch / (BU / UC);
        const int ub = h_blk * BU;
        const int row_base = w.tile_row0 + ROWS * ML;
        int last = d.N - 1;
        asm volatile("" : "+s"(last));
        const FQ_GLOBAL float *sc = (const FQ_GLOBAL float *)d.scales;
        const FQ_GLOBAL uint8_t *zp = (const FQ_GLOBAL uint8_t *)d.zeros;
        {
            const int u = ub + 4 * (lane & 7);
            const bool inside = u + 4 <= G;
#pragma unroll
            for (int i = 0; i < ROWS / 8; i++) {
                const uint32_t row = (uint32_t)min(row_base + 8 * i + (lane >> 3), last);
                if (inside) {
                    sr[i] = *(const FQ_GLOBAL f32x4_a4 *)(sc + (row * (uint32_t)G + (uint32_t)u));
                } else {
#pragma unroll
                    for (int g = 0; g < 4; g++)
                        sr[i][g] = sc[row * (uint32_t)G + (uint32_t)min(u + g, G - 1)];
                }
            }
        }
        {
            const int u = ub + 16 * (lane & 1);
            const bool inside = u + 16 <= G;
#pragma unroll
            for (int j = 0; j < ROWS / 32; j++) {
                const uint32_t row = (uint32_t)min(row_base + 32 * j + (lane >> 1), last);
                if (inside) {
                    zr[j] = *(const FQ_GLOBAL u32x4_a1 *)(zp + (row * (uint32_t)G + (uint32_t)u));
                } else {
                    uint32_t v[4] = {0u, 0u, 0u, 0u};
#pragma unroll
                    for (int g = 0; g < 16; g++)
                        v[g >> 2] |= (uint32_t)zp[row * (uint32_t)G + (uint32_t)min(u + g, G - 1)] << (8 * (g & 3));
                    zr[j] = u32x4{v[0], v[1], v[2], v[3]};
                }
            }
        }
    }

    // Write the pair of chunks that starts at w (w.ch even), which lies in the block held.
    __device__ __forceinline__ void store(const Walk &w)
    {
        float *ms = (w.p & 1) ? L.ms[1] : L.ms[0];
        uint8_t *mz = (w.p & 1) ? L.mz[1] : L.mz[0];
        const int cp = (w.ch / 2) % (BU / UP); // the pair inside the block: units 8 cp .. 8 cp + 7
        if (((lane & 7) >> 1) == cp) {
#pragma unroll
            for (int i = 0; i < ROWS / 8; i++) {
                const int rl = ROWS * ML + 8 * i + (lane >> 3); // row of the tile: consumer rl / 32, row tile (rl / 16) % 2
                const int idx = (((rl >> 5) * 16 + (rl & 15)) * RT + ((rl >> 4) & 1)) * UP + 4 * (lane & 1);
                *reinterpret_cast<float4_t *>(ms + idx) = sr[i];
            }
        }
        if ((lane & 1) == (cp >> 1)) {
#pragma unroll
            for (int j = 0; j < ROWS / 32; j++) {
                const int rl = ROWS * ML + 32 * j + (lane >> 1);
                const int idx = (((rl >> 5) * 16 + (rl & 15)) * RT + ((rl >> 4) & 1)) * UP;
                const uint32_t a = (cp & 1) ? zr[j].z : zr[j].x, b = (cp & 1) ? zr[j].w : zr[j].y;
                *reinterpret_cast<uint2 *>(mz + idx) = make_uint2(a, b);
            }
        }
    }

    // w: the first chunk of the next pair to write.  Write it, go on to the next pair, and
    // request its block if that is another one (the registers are reused: no load before the
    // last write).
    __device__ __forceinline__ void hand_over(Walk &w)
    {
        if (w.bits != 16)
            store(w);
        __builtin_amdgcn_sched_barrier(0);
        w.next_chunk();
        if (w.valid() && (w.ch & 1))
            w.next_chunk();
        if (w.valid() && w.bits != 16 && (w.tile != h_tile || w.ch / (BU / UC) != h_blk))
            load(w);
    }

    __device__ __forceinline__ void run(Walk w)
    {
        Walk b = w; // the chunk of the next barrier
        if (w.valid()) {
            if (w.bits != 16)
                load(w);
            hand_over(w); // the first pair is due at the first barrier
        }
        while (b.valid()) {
            __builtin_amdgcn_s_waitcnt(0xc07f); // lgkmcnt(0): this wavefront's LDS writes are done
            barrier();
            if (w.valid() && w.g == b.g + 1)
                hand_over(w);
            b.next_chunk();
        }
    }
};

template <int MT>
__global__ __launch_bounds__(THREADS) void decode_stream_kernel(const FqLinearDesc *__restrict__ table,
                                                                const int32_t *__restrict__ bits_dev, int count,
                                                                int total_tiles, int M)
{
    __shared__ __attribute__((aligned(1024))) uint8_t ring[CONSUMERS * NS * STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) uint8_t x0[16 * MT * KC * 2], x1[16 * MT * KC * 2];
    __shared__ __attribute__((aligned(256))) float ms0[UP * TILE_ROWS], ms1[UP * TILE_ROWS];
    __shared__ __attribute__((aligned(256))) uint8_t mz0[UP * TILE_ROWS], mz1[UP * TILE_ROWS];
    Lds L;
    L.ring = ring;
    L.x[0] = x0, L.x[1] = x1;
    L.ms[0] = ms0, L.ms[1] = ms1;
    L.mz[0] = mz0, L.mz[1] = mz1;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    Walk w;
    w.start(table, bits_dev, count, total_tiles);
    if (wave < CONSUMERS)
        consume<MT>(w, L, M, wave);
    else if (wave == CONSUMERS)
        Loader<MT, 0>(L, M).run(w);
    else if (wave == CONSUMERS + 1)
        Loader<MT, 1>(L, M).run(w);
    else if (wave == CONSUMERS + 2)
        MetaLoader<0>(L).run(w);
    else
        MetaLoader<1>(L).run(w);
}

} // namespace

// A plan launch (device table of `count` linears, device-side bit-widths) for 2 <= M <= 32 and
// tiles of 256 rows (M * N < 2^30 for every entry: the outputs are stored through 32-bit offsets).
hipError_t fq_launch_skinny_stream(const FqLinearDesc *descs_dev, const int32_t *bits_dev, int count, int total_tiles,
                                   int M, int cus, hipStream_t stream)
{
    // one workgroup per CU (LDS): persistent over the tiles
    const int grid = total_tiles < cus ? total_tiles : cus;
    if (M <= 16)
        decode_stream_kernel<1><<<grid, THREADS, 0, stream>>>(descs_dev, bits_dev, count, total_tiles, M);
    else
        decode_stream_kernel<2><<<grid, THREADS, 0, stream>>>(descs_dev, bits_dev, count, total_tiles, M);
    return hipGetLastError();
}
