// Prefill-shaped weight-only quantized linear: y[M][N] = x[M][K] . dequant(W[N][K])^T for
// M in the hundreds or thousands, where the weight stream is amortised over many tokens
// and the contraction is compute bound (Sec. 4.1) -- a dense GEMM on the matrix cores with
// the dequantization of Sec. 2.2 Eq. (3) fused into the operand path.
//
// Tiling.  A workgroup (8 wavefronts, two per SIMD) owns a 256 (tokens) x 256 (weight rows)
// tile of y and walks K in steps of 64.  A wavefront owns 128 tokens x 64 rows = 4 x 2 tiles
// of v_mfma_f32_32x32x16_f16 (A = x: 32 tokens x 16 k, B = weights: 16 k x 32 rows; 128
// binary32 accumulator registers).  The large shared tile keeps the bytes fetched per MFMA
// low enough that one step of compute covers the latency of the next stage's fetch.
//
// Operand path.  Both slabs of a step -- x: 128 rows x 128 bytes, packed weights: 256 rows x
// 32 / 64 / 128 bytes for 4-bit / 8-bit / fp16 -- go from global memory straight into LDS
// (global_load_lds_dwordx4: no staging registers, a wavefront fetches whole rows), three
// stages deep (two for fp16 weights), one wait and one barrier per step.  Rows are stored 128 bytes apart (two 64-byte
// or four 32-byte weight rows share such a line) with the 16-byte slots of a line XOR-ed by
// (line >> 1) & 7, so that a 128-bit operand read of 16 consecutive rows touches every bank
// once; the permutation is applied on the global side of the load, where each lane is free to
// fetch any piece.  The packed weights are unpacked after the LDS read, in registers: the
// LDS traffic of the weight operand is that of the packed codes.
//
// Dequantization.  Codes become the exact integers q - z as halves (bit tricks: a byte under
// exponent 0x64 is 1024 + q, a nibble in bits 4..7 under 0x54 is 64 + q, a 2-bit field at bits
// 0 / 2 / 4 / 6 under 0x64 / 0x5C / 0x54 / 0x4C is 1024 / 256 / 64 / 16 + q; one v_pk_add_f16
// removes the offset and z) and are multiplied by the group's scale rounded to half (one
// v_pk_mul_f16 per register): the MFMA operand is half((q - z) * half(s)).  The decode
// kernels keep the scale in binary32 outside the group sum; here that would need a second
// set of 128 accumulator registers per wavefront and a 256-instruction fold per group, so
// the prefill path rounds twice at 2^-11 relative instead.  The error stays well inside the
// 2e-3 bound (about 5e-4 of the output magnitude in the worst one-group case).  So that this
// holds whatever the magnitude of the weights, the half carries s * 2^e with a power of two per
// weight row that is taken out of the row's sums at the end.
//
// Workgroups that share a weight slab (the M tiles of one N tile) get consecutive logical
// ids, and logical ids are dealt to the 8 XCDs in contiguous runs, so that a slab is
// fetched into one L2 and reused there.  The tiles an XCD has left for a last round that would
// fill at most half of its CUs run as half tiles (128 tokens) in a second launch.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "fq_internal.h"

namespace {

#define FQ_GLOBAL __attribute__((address_space(1)))
#define FQ_LDS __attribute__((address_space(3)))

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int THREADS = 512;
constexpr int WAVES = THREADS / 64;
constexpr int BM_FULL = 256, BN = 256, BK = 64;
constexpr int WN = 64;             // weight rows per wavefront (2 MFMA tiles)
constexpr int XRB = BK * 2;        // bytes of an x row per step (128)

// Byte offset of 16-byte chunk `ch` of row `r` in a slab whose rows are RB bytes long:
// 128 / RB rows share a 128-byte line, slots XOR-ed by (line >> 1) & 7.
template <int RB>
__device__ __forceinline__ int slab_offset(int r, int ch)
{
    constexpr int RPL = 128 / RB, CPR = RB / 16;
    const int line = r / RPL;
    return line * 128 + ((((r % RPL) * CPR + ch) ^ ((line >> 1) & 7)) << 4);
}

// Which chunks a thread fetches of a slab (ROWS rows of RB bytes).  Load i of wavefront w
// fills LDS chunks (i * WAVES + w) * 64 .. + 63, i.e. lines (i * WAVES + w) * 8 .. + 7; the
// lane owns slot (lane & 7) of line l0 + 8 * WAVES * i, and the piece stored there is the
// same for every i (8 * WAVES is a multiple of 16).
struct DmaLane {
    int r0;      // row of load 0
    int rstep;   // rows between consecutive loads
    int byte0;   // byte offset of the piece inside the row
};

template <int RB>
__device__ __forceinline__ DmaLane dma_lane()
{
    constexpr int RPL = 128 / RB, CPR = RB / 16;
    // a slab of 16-byte rows (2-bit weights) is 4 KiB, half a load of the workgroup: wavefronts
    // 4 .. 7 fetch the same pieces as 0 .. 3 (same bytes to the same place), so that every
    // wavefront issues the same number of loads per step -- the waits count them
    const int wave = RB == 16 ? (threadIdx.x >> 6) & 3 : threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int line = wave * 8 + (lane >> 3);
    const int slot = (lane & 7) ^ ((line >> 1) & 7);
    DmaLane L;
    L.r0 = line * RPL + slot / CPR;
    L.rstep = 8 * WAVES * RPL;
    L.byte0 = (slot % CPR) * 16;
    return L;
}

// Fetch one step of one operand straight into LDS.  `tile` points at (first row of the
// tile, first byte of the step) and is the same for the whole workgroup; rows past
// `last_row` (relative to the tile) are clamped to it; `pitch` = bytes between rows in
// global memory.
// Loads of a thread per step and slab.
template <int ROWS, int RB>
constexpr int dma_loads()
{
    return ROWS * RB / 16 / THREADS > 0 ? ROWS * RB / 16 / THREADS : 1;
}

// PART = -1: all the loads of the slab; PART = p (0 .. 3): quarter p of them (those with index i,
// i * 4 / LOADS = p), so that a step can issue its loads in four portions.
template <int ROWS, int RB, int PART = -1>
__device__ __forceinline__ void dma_slab(const uint8_t *tile, const DmaLane &L, int last_row, uint32_t pitch,
                                         uint8_t *slab)
{
    const int wave = RB == 16 ? (threadIdx.x >> 6) & 3 : threadIdx.x >> 6;
    constexpr int LOADS = dma_loads<ROWS, RB>();
#pragma unroll
    for (int i = 0; i < LOADS; i++) {
        if (PART >= 0 && (LOADS >= 4 ? i * 4 / LOADS : (LOADS == 2 ? 2 * i : 0)) != PART)
            continue;
        const uint32_t off = (uint32_t)min(L.r0 + i * L.rstep, last_row) * pitch + L.byte0;
        __builtin_amdgcn_global_load_lds((const FQ_GLOBAL void *)(tile + off),
                                         (FQ_LDS void *)(slab + (i * WAVES + wave) * 1024), 16, 0, 0);
    }
}

// (a + b) * s, each operation rounded to half; a + b is the exact integer q - z
__device__ __forceinline__ uint32_t deq(uint32_t a, uint32_t b, half2_t s)
{
    return __builtin_bit_cast(uint32_t, (__builtin_bit_cast(half2_t, a) + __builtin_bit_cast(half2_t, b)) * s);
}

__device__ __forceinline__ float as_float_global(const float *p) { return *(const FQ_GLOBAL float *)p; }

__device__ __forceinline__ float16_t mfma32(const u32x4 a, const uint32_t (&b)[4], float16_t c)
{
    const u32x4 bv = {b[0], b[1], b[2], b[3]};
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, a),
                                                  __builtin_bit_cast(half8_t, bv), c, 0, 0, 0);
}

// Which 8 k of the 64-k step lane (row, c) supplies in k16-step i, as the index of the
// 16-byte chunk of 8 halves in an x row:
//   4-bit: a lane reads one 16-byte chunk of codes (32 codes, k = 32 c ..), word i of it holds
//          k = 32 c + 8 i ..;   2-bit: the same k from 8 bytes of codes, half-word i;
//          8-bit and fp16: k = 16 i + 8 c ..
template <int BITS>
__device__ __forceinline__ int x_chunk(int i, int c)
{
    return BITS == 4 || BITS == 2 ? 4 * c + i : 2 * i + c;
}

// Scale and zero point of a lane's two weight rows for one quantization group.
struct Meta {
    float s[2];
    uint32_t z[2];
};

// HALF: the workgroup takes half a tile, 128 tokens x 256 weight rows (a wavefront 64 tokens x 64
// rows): the tiles left over after the last full round of workgroups are cut in two, so that they
// keep twice as many CUs busy for half as long.  `skip`: first tile of this launch inside an XCD's
// run of `per_xcd` tiles.
template <int BITS, bool HALF>
__global__ __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void prefill_kernel(
    const FqLinearDesc d, int M, int m_tiles, int n_tiles, int per_xcd, int skip)
{
    constexpr int BM = HALF ? BM_FULL / 2 : BM_FULL; // tokens per workgroup
    constexpr int WM = BM / 2;                       // tokens per wavefront
    constexpr int MTL = WM / 32;                     // MFMA tiles of a wavefront along the tokens (4 or 2)
    constexpr int XSLAB = BM * XRB;                  // 32 or 16 KiB
    constexpr int WRB = BK * BITS / 8;  // bytes of a packed weight row per step
    constexpr int WSLAB = BN * WRB;
    // Separate arrays, selected at compile time: the compiler can then tell that the operand
    // reads of a step do not touch the slabs its direct-to-LDS loads are filling, and does not
    // wait for those loads before the first read.
    constexpr int NST = BITS == 16 ? 2 : 3; // stages in flight (fp16 weights: 64 KiB per stage)
    // A step issues its fetch in four portions, one behind each quarter of its MFMAs, instead of all of
    // it ahead of them: the wavefronts of a workgroup leave the step's barrier together, and eight
    // wavefronts issuing five or six loads each at that moment keep the matrix pipes waiting
    // (2048 x 8192 x 28672 and its transpose, TFLOP/s: 2 bits 1105 -> 1143 and 1123 -> 1204, 4 bits 1040 ->
    // 1072 and 1084 -> 1131, 8 bits 1039 -> 1066 and 1086 -> 1116).  Not with two stages (fp16 weights: 1105 ->
    // 967): there a step waits for its own requests, and the late ones have less time to land.
    constexpr bool SPREAD = NST == 3;
    __shared__ __attribute__((aligned(1024))) uint8_t xs0[XSLAB], xs1[XSLAB], xs2[NST == 3 ? XSLAB : 1024];
    __shared__ __attribute__((aligned(1024))) uint8_t ws0[WSLAB], ws1[WSLAB], ws2[NST == 3 ? WSLAB : 1024];
    __shared__ __attribute__((aligned(1024))) float smeta[BN * 4]; // [row][4 groups] (one group per request: the first BN words)
    __shared__ __attribute__((aligned(1024))) uint32_t zmeta[BN];  // [row]: four groups' bytes, or one zero-extended

    // hardware deals consecutive workgroup ids round-robin to the 8 XCDs: give each XCD a
    // contiguous run of logical tiles
    const int in_run = skip + (HALF ? (int)(blockIdx.x >> 4) : (int)(blockIdx.x >> 3));
    const int logical = (blockIdx.x & 7) * per_xcd + in_run;
    if (in_run >= per_xcd || logical >= m_tiles * n_tiles)
        return;
    const int m0 = (logical % m_tiles) * BM_FULL + (HALF ? (int)((blockIdx.x >> 3) & 1) * BM : 0);
    const int n0 = (logical / m_tiles) * BN;
    if (m0 >= M)
        return; // the second half of a last, partly filled tile

    const uint8_t *codes = BITS == 2 ? d.codes2 : BITS == 4 ? d.codes4 : BITS == 8 ? d.codes8 : (const uint8_t *)d.w16;
    const float *scales = BITS == 2 ? d.scales2 : BITS == 4 ? d.scales4 : d.scales8;
    const uint8_t *zeros = BITS == 2 ? d.zeros2 : BITS == 4 ? d.zeros4 : d.zeros8;

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int l32 = lane & 31, c = lane >> 5;
    const int wm = (wave & 1) * WM, wn = (wave >> 1) * WN;

    float16_t acc[MTL][2];
#pragma unroll
    for (int i = 0; i < MTL; i++)
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
            for (int v = 0; v < 16; v++)
                acc[i][j][v] = 0.f;

    // Per-lane LDS offsets of the operand reads (tiles start at multiples of 32 rows, which
    // leaves the slot permutation of a lane unchanged from tile to tile).
    int aofs[4];
#pragma unroll
    for (int i = 0; i < 4; i++)
        aofs[i] = slab_offset<XRB>(l32, x_chunk<BITS>(i, c));
    // Weights: 8-bit and fp16 rows are 64 / 128 bytes, the second n-tile (32 rows on) sits a
    // whole number of 16-line blocks further and keeps the permutation: one offset per
    // k16-step.  4-bit rows are 32 bytes (one read per n-tile and step): 32 rows are 8 lines,
    // which changes the permutation, so each n-tile has its own offset.
    constexpr int WRB_ = BK * BITS / 8;
    int bofs[4];
#pragma unroll
    for (int i = 0; i < 4; i++)
        bofs[i] = BITS == 2 ? slab_offset<WRB_>(wn + (i & 1) * 32 + l32, 0) + 8 * c
                : BITS == 4 ? slab_offset<WRB_>(wn + (i & 1) * 32 + l32, c)
                : BITS == 8 ? slab_offset<WRB_>(wn + l32, i) + 8 * c
                            : slab_offset<WRB_>(wn + l32, 2 * i + c);
    constexpr int BJ = 32 * WRB_; // bytes from n-tile 0 to n-tile 1 (8-bit, fp16)

    const uint32_t K = (uint32_t)d.K, G = K >> 7;
    const int nsteps = d.K / BK;
    const DmaLane xl = dma_lane<XRB>(), wl = dma_lane<WRB>();
    const int x_last = M - 1 - m0, w_last = d.N - 1 - n0;
    const uint32_t w_pitch = K * BITS / 8;
    const uint8_t *x_tile = (const uint8_t *)d.x + (size_t)m0 * K * 2;
    const uint8_t *w_tile = codes + (size_t)n0 * w_pitch;
    const float *scales_tile = BITS == 16 ? nullptr : scales + (size_t)n0 * G;
    const uint8_t *zeros_tile = BITS == 16 ? nullptr : zeros + (size_t)n0 * G;
    // Scales and zero points of one quantization group for the tile's 256 weight rows also
    // come in through direct-to-LDS loads (a dword resp. a byte per lane; either lands in the
    // lane's dword slot, the byte zero-extended): wavefronts 0-3 fetch 64 scales each,
    // wavefronts 4-7 64 zero points each, so every wavefront issues the same number of loads
    // per step -- the waits below count them.  An ordinary load would do, but the compiler
    // assumes it may overtake pending direct-to-LDS loads and waits for all of them before its
    // first use, which would drain the fetch pipeline every other step.
    // A request of a lane's scale touches a cache line of its own, 512 lines per group and
    // workgroup against 384 for the operand slabs of a step (3 to 5 % of the kernel's time).  Where
    // a row's scales of four consecutive groups are 16 bytes that a 16-byte request may fetch --
    // K / 128 a multiple of 4 and the arrays aligned -- a request brings four groups (their zero
    // points are one 4-byte request), during the second step of every fourth group.
    const bool meta4 = BITS != 16 && (G & 3u) == 0 && ((uintptr_t)scales & 15u) == 0 && ((uintptr_t)zeros & 3u) == 0;
    auto fetch_meta = [&](int g) {
        if (BITS != 16) {
            const uint32_t row = (uint32_t)min((wave & 3) * 64 + lane, w_last) * G;
            if (meta4) {
                if ((g & 3) != 0)
                    return; // (requested with the first group of its four)
                if (wave < 4)
                    __builtin_amdgcn_global_load_lds((const FQ_GLOBAL void *)(scales_tile + g + row),
                                                     (FQ_LDS void *)(smeta + (wave & 3) * 256), 16, 0, 0);
                else
                    __builtin_amdgcn_global_load_lds((const FQ_GLOBAL void *)(zeros_tile + g + row),
                                                     (FQ_LDS void *)(zmeta + (wave & 3) * 64), 4, 0, 0);
                return;
            }
            if (wave < 4)
                __builtin_amdgcn_global_load_lds((const FQ_GLOBAL void *)(scales_tile + g + row),
                                                 (FQ_LDS void *)(smeta + (wave & 3) * 64), 4, 0, 0);
            else
                __builtin_amdgcn_global_load_lds((const FQ_GLOBAL void *)(zeros_tile + g + row),
                                                 (FQ_LDS void *)(zmeta + (wave & 3) * 64), 1, 0, 0);
        }
    };

    Meta cur;
    // The operand carries the group's scale as a half: a scale below 2^-14 would lose bits there and
    // one below 2^-25 the whole group.  Every weight row therefore gets a power of two, taken from
    // two of its scales (the first group's and the middle one's), that brings them to about 2^-4 --
    // halves then hold scales 2^10 times smaller and 2^12 times larger than those exactly as well --
    // and the row's sums are multiplied by its inverse at the end.
    int ex[2] = {0, 0};
    if (BITS != 16) {
#pragma unroll
        for (int j = 0; j < 2; j++) {
            const float *srow = scales_tile + (size_t)min(wn + j * 32 + l32, w_last) * G;
            const float m = fmaxf(as_float_global(srow), as_float_global(srow + (G >> 1)));
            ex[j] = -3 - __builtin_amdgcn_frexp_expf(m);
        }
    }
    // VMEM operations a thread issues per step: these may still be in flight at the end of the
    // step when a later stage is being filled (three stages)
    constexpr int DMA_OPS = BM * XRB / 16 / THREADS + (BN * WRB / 16 / THREADS > 0 ? BN * WRB / 16 / THREADS : 1);
    // s_waitcnt vmcnt(n) lgkmcnt(0) (expcnt untouched)
    auto wait_vm = [](auto n) {
        constexpr int N = decltype(n)::value;
        __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | ((N >> 4) << 14));
    };
    // Workgroup barrier without the memory fence of __syncthreads(): the fence would wait for
    // every outstanding load, including the stage that is meant to stay in flight.  The waits
    // that matter are issued explicitly before it; the empty asm statements keep the compiler
    // from moving LDS accesses across.
    auto barrier = [] {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    auto stage_x = [&](auto st) -> uint8_t * {
        constexpr int ST = decltype(st)::value;
        return ST == 0 ? xs0 : ST == 1 ? xs1 : xs2;
    };
    auto stage_w = [&](auto st) -> uint8_t * {
        constexpr int ST = decltype(st)::value;
        return ST == 0 ? ws0 : ST == 1 ? ws1 : ws2;
    };
    auto fetch = [&](int sf, auto st) { // step sf (clamped: always issued) into stage st
        const int sn = min(sf, nsteps - 1);
        dma_slab<BM, XRB>(x_tile + sn * XRB, xl, x_last, K * 2, stage_x(st));
        dma_slab<BN, WRB>(w_tile + sn * WRB, wl, w_last, w_pitch, stage_w(st));
    };
    // the same in four portions (x: a load each; weights: one, two or four loads dealt over them)
    auto fetch_part = [&](int sf, auto st, auto part) {
        constexpr int P = decltype(part)::value;
        const int sn = min(sf, nsteps - 1);
        dma_slab<BM, XRB, P>(x_tile + sn * XRB, xl, x_last, K * 2, stage_x(st));
        dma_slab<BN, WRB, P>(w_tile + sn * WRB, wl, w_last, w_pitch, stage_w(st));
    };
    fetch(0, std::integral_constant<int, 0>());
    if (NST == 3)
        fetch(1, std::integral_constant<int, 1>());
    fetch_meta(0);
    __builtin_amdgcn_s_waitcnt(0);
    barrier();

    // One step: the slabs of step s + NST - 1 are requested first and land in the stage that
    // was read during step s - 1, while the MFMAs of step s run on stage ST = s % NST.  A
    // quantization group is two steps; its scales and zero points are fetched during the
    // previous group's second (ODD) step and read into registers in its own first step.
    auto step = [&](int s, auto st, auto odd) {
        constexpr int ST = decltype(st)::value;
        constexpr bool ODD = decltype(odd)::value;
        if (!ODD && BITS != 16) {
            // first step of a group: its scales and zero points landed during the previous step
            // (nothing is writing smeta / zmeta now: the next request goes out a step later)
#pragma unroll
            for (int j = 0; j < 2; j++) {
                const int row = wn + j * 32 + l32, g4 = (s >> 1) & 3;
                cur.s[j] = __builtin_ldexpf(meta4 ? smeta[row * 4 + g4] : smeta[row], ex[j]);
                cur.z[j] = meta4 ? (zmeta[row] >> (8 * g4)) & 255u : zmeta[row];
            }
        }
        if (ODD && (!meta4 || (s >> 1) + 1 < (int)G)) // (four groups at a time: nothing to request past the last)
            fetch_meta(min((s >> 1) + 1, (int)G - 1)); // the oldest request of this step
        if (!SPREAD)
            fetch(s + NST - 1, std::integral_constant<int, (ST + NST - 1) % NST>());
        // keep the requests here, ahead of the step's MFMAs: left to itself the scheduler sinks
        // them to the end of the step, right in front of the wait
        __builtin_amdgcn_sched_barrier(0);
        const uint8_t *xc = stage_x(st), *wc = stage_w(st);
        // opaque per step: otherwise the sums of every stage's base and every offset are kept
        // in registers across the whole loop
#pragma unroll
        for (int i = 0; i < 4; i++)
            asm volatile("" : "+v"(aofs[i]), "+v"(bofs[i]));

        // constants of the group for the two n-tiles
        half2_t sh[2];
        uint32_t nz[2], nz2[2];
#pragma unroll
        for (int j = 0; j < 2; j++) {
            if (BITS != 16) {
                sh[j] = half2_t{(_Float16)cur.s[j], (_Float16)cur.s[j]};
                const uint32_t z = cur.z[j];
                nz[j] = BITS == 8 ? ((z | (z << 16)) | 0xE400E400u)               // -(1024 + z) twice
                      : BITS == 4 ? ((z | 0xE400u) | (((z << 4) | 0xD400u) << 16)) // -(1024 + z), -(64 + z)
                                  : ((z | 0xE400u) | (((z << 2) | 0xDC00u) << 16)); // -(1024 + z), -(256 + z)
                nz2[j] = ((z << 4) | 0xD400u) | (((z << 6) | 0xCC00u) << 16);     // 2 bits: -(64 + z), -(16 + z)
            }
        }
        u32x4 w4[2]; // 4-bit: the lane's 32 codes of the step, per n-tile
        if (BITS == 4) {
#pragma unroll
            for (int j = 0; j < 2; j++)
                w4[j] = *reinterpret_cast<const u32x4 *>(wc + bofs[j]);
        }
        u32x2 w2[2]; // 2-bit: the same 32 codes in 8 bytes
        if (BITS == 2) {
#pragma unroll
            for (int j = 0; j < 2; j++)
                w2[j] = *reinterpret_cast<const u32x2 *>(wc + bofs[j]);
        }
#pragma unroll
        for (int i = 0; i < 4; i++) {
            u32x4 a[MTL];
#pragma unroll
            for (int mt = 0; mt < MTL; mt++)
                a[mt] = *reinterpret_cast<const u32x4 *>(xc + (wm + mt * 32) * XRB + aofs[i]);
#pragma unroll
            for (int j = 0; j < 2; j++) {
                uint32_t b[4];
                if (BITS == 2) {
                    // half-word i: fields q0 .. q7 of k = 32 c + 8 i .., byte t holds q(4t) .. q(4t+3).
                    // The byte is copied under both halves; fields 0 and 1 (or 2 and 3) of it stay
                    // where they are, one per half, each under the exponent that makes it offset + q
                    const uint32_t v = i < 2 ? w2[j].x : w2[j].y;
                    const uint32_t lo = __builtin_amdgcn_perm(0u, v, (i & 1) ? 0x0c020c02u : 0x0c000c00u);
                    const uint32_t hi = __builtin_amdgcn_perm(0u, v, (i & 1) ? 0x0c030c03u : 0x0c010c01u);
                    b[0] = deq((lo & 0x000C0003u) | 0x5C006400u, nz[j], sh[j]);  // q0, q1
                    b[1] = deq((lo & 0x00C00030u) | 0x4C005400u, nz2[j], sh[j]); // q2, q3
                    b[2] = deq((hi & 0x000C0003u) | 0x5C006400u, nz[j], sh[j]);  // q4, q5
                    b[3] = deq((hi & 0x00C00030u) | 0x4C005400u, nz2[j], sh[j]); // q6, q7
                } else if (BITS == 4) {
                    // word i: nibbles q0 .. q7 of k = 32 c + 8 i ..; byte t holds (q(2t+1) q(2t)).
                    // The byte is copied under both halves, the low nibble kept in the low half
                    // (exponent 0x64: 1024 + q) and the high nibble in the high half (0x54: 64 + q)
                    const uint32_t v = w4[j][i];
                    b[0] = deq((__builtin_amdgcn_perm(0u, v, 0x0c000c00u) & 0x00F0000Fu) | 0x54006400u, nz[j], sh[j]);
                    b[1] = deq((__builtin_amdgcn_perm(0u, v, 0x0c010c01u) & 0x00F0000Fu) | 0x54006400u, nz[j], sh[j]);
                    b[2] = deq((__builtin_amdgcn_perm(0u, v, 0x0c020c02u) & 0x00F0000Fu) | 0x54006400u, nz[j], sh[j]);
                    b[3] = deq((__builtin_amdgcn_perm(0u, v, 0x0c030c03u) & 0x00F0000Fu) | 0x54006400u, nz[j], sh[j]);
                } else if (BITS == 8) {
                    const u32x2 q = *reinterpret_cast<const u32x2 *>(wc + j * BJ + bofs[i]); // k = 16 i + 8 c ..
                    b[0] = deq(__builtin_amdgcn_perm(0x64646464u, q.x, 0x04010400u), nz[j], sh[j]);
                    b[1] = deq(__builtin_amdgcn_perm(0x64646464u, q.x, 0x04030402u), nz[j], sh[j]);
                    b[2] = deq(__builtin_amdgcn_perm(0x64646464u, q.y, 0x04010400u), nz[j], sh[j]);
                    b[3] = deq(__builtin_amdgcn_perm(0x64646464u, q.y, 0x04030402u), nz[j], sh[j]);
                } else {
                    const u32x4 q = *reinterpret_cast<const u32x4 *>(wc + j * BJ + bofs[i]);
                    b[0] = q.x;
                    b[1] = q.y;
                    b[2] = q.z;
                    b[3] = q.w;
                }
#pragma unroll
                for (int mt = 0; mt < MTL; mt++)
                    acc[mt][j] = mfma32(a[mt], b, acc[mt][j]);
            }
            if (SPREAD) {
                // a quarter of the step's requests behind every quarter of its MFMAs; vector memory
                // instructions stay on their side of the line, everything else may cross it
                if (i == 0)
                    fetch_part(s + NST - 1, std::integral_constant<int, (ST + NST - 1) % NST>(), std::integral_constant<int, 0>());
                if (i == 1)
                    fetch_part(s + NST - 1, std::integral_constant<int, (ST + NST - 1) % NST>(), std::integral_constant<int, 1>());
                if (i == 2)
                    fetch_part(s + NST - 1, std::integral_constant<int, (ST + NST - 1) % NST>(), std::integral_constant<int, 2>());
                if (i == 3)
                    fetch_part(s + NST - 1, std::integral_constant<int, (ST + NST - 1) % NST>(), std::integral_constant<int, 3>());
                __builtin_amdgcn_sched_barrier(0x38F);
            }
        }
        // Stage s + 1 must have landed (it was requested one step earlier when there are three
        // stages, so this step's own requests -- the last DMA_OPS operations issued -- may stay
        // in flight), and this wavefront's LDS reads of stage ST must be done before anyone
        // refills it.
        if (NST == 3)
            wait_vm(std::integral_constant<int, DMA_OPS>());
        else
            wait_vm(std::integral_constant<int, 0>());
        barrier();
    };
    // K is a multiple of 128, so the number of steps is even.  Stages and group halves repeat
    // with period 6 (three stages) or 2 (two stages).
    int s = 0;
    if (NST == 3) {
        for (; s + 6 <= nsteps; s += 6) {
            step(s, std::integral_constant<int, 0>(), std::false_type());
            step(s + 1, std::integral_constant<int, 1>(), std::true_type());
            step(s + 2, std::integral_constant<int, 2>(), std::false_type());
            step(s + 3, std::integral_constant<int, 0>(), std::true_type());
            step(s + 4, std::integral_constant<int, 1>(), std::false_type());
            step(s + 5, std::integral_constant<int, 2>(), std::true_type());
        }
        if (s + 2 <= nsteps) {
            step(s, std::integral_constant<int, 0>(), std::false_type());
            step(s + 1, std::integral_constant<int, 1>(), std::true_type());
            s += 2;
        }
        if (s + 2 <= nsteps) {
            step(s, std::integral_constant<int, 2>(), std::false_type());
            step(s + 1, std::integral_constant<int, 0>(), std::true_type());
            s += 2;
        }
    } else {
        for (; s < nsteps; s += 2) {
            step(s, std::integral_constant<int, 0>(), std::false_type());
            step(s + 1, std::integral_constant<int, 1>(), std::true_type());
        }
    }
    __builtin_amdgcn_s_waitcnt(0); // nothing of this kernel's is in flight past this point
    // D layout of the 32x32 MFMA: lane holds column l32, rows 8 * (v / 4) + 4 * (lane / 32) + v % 4.
#pragma unroll
    for (int mt = 0; mt < MTL; mt++)
#pragma unroll
        for (int j = 0; j < 2; j++) {
            const int n = n0 + wn + j * 32 + l32;
#pragma unroll
            for (int v = 0; v < 16; v++) {
                const int m = m0 + wm + mt * 32 + 8 * (v >> 2) + 4 * c + (v & 3);
                if (m < M && n < d.N)
                    ((FQ_GLOBAL uint16_t *)d.y)[(size_t)m * d.N + n] =
                        __builtin_bit_cast(uint16_t, (_Float16)(BITS == 16 ? acc[mt][j][v] : __builtin_ldexpf(acc[mt][j][v], -ex[j])));
            }
        }
}

} // namespace

template <bool HALF>
static hipError_t launch_prefill(const FqLinearDesc &d, int bits, int M, int m_tiles, int n_tiles, int per_xcd,
                                 int skip, int per_launch, hipStream_t stream)
{
    if (per_launch <= 0)
        return hipSuccess;
    const unsigned grid = (unsigned)per_launch * (HALF ? 16u : 8u);
    if (bits == 2)
        prefill_kernel<2, HALF><<<grid, THREADS, 0, stream>>>(d, M, m_tiles, n_tiles, per_xcd, skip);
    else if (bits == 4)
        prefill_kernel<4, HALF><<<grid, THREADS, 0, stream>>>(d, M, m_tiles, n_tiles, per_xcd, skip);
    else if (bits == 8)
        prefill_kernel<8, HALF><<<grid, THREADS, 0, stream>>>(d, M, m_tiles, n_tiles, per_xcd, skip);
    else
        prefill_kernel<16, HALF><<<grid, THREADS, 0, stream>>>(d, M, m_tiles, n_tiles, per_xcd, skip);
    return hipGetLastError();
}

hipError_t fq_launch_prefill(const FqLinearDesc &d, int bits, int M, hipStream_t stream)
{
    const int m_tiles = (M + BM_FULL - 1) / BM_FULL, n_tiles = (d.N + BN - 1) / BN;
    const long long total = (long long)m_tiles * n_tiles;
    if (total > 0x3fffffffLL)
        return hipErrorInvalidValue;
    const int per_xcd = (int)((total + 7) / 8);
    // One workgroup per CU at a time: an XCD works through its run of tiles in rounds of its CU
    // count.  What is left for the last round, if it would fill at most half the CUs, runs as half
    // tiles in a second launch (2048 x 28672: 112 tiles per XCD = 3 rounds of 32 + 16 tiles, which
    // then take half a round instead of a whole one).
    const int cus = fq_device_cus();
    const int per_round = cus / 8 > 0 ? cus / 8 : 1;
    const int rest = per_xcd % per_round;
    const int tail = rest > 0 && 2 * rest <= per_round ? rest : 0;
    hipError_t e = launch_prefill<false>(d, bits, M, m_tiles, n_tiles, per_xcd, 0, per_xcd - tail, stream);
    if (e != hipSuccess)
        return e;
    return launch_prefill<true>(d, bits, M, m_tiles, n_tiles, per_xcd, per_xcd - tail, tail, stream);
}
