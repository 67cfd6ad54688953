// A decode step in the order a decoder must issue it, in ONE launch (batch 1).
//
// A token's linears are not independent: the output projection needs the attention's result, the
// down projection needs gate and up (Alg. 1's decode loop walks them in order).  Issued as one
// launch per dependent group, a 7B-shaped step is 128 launches of 2 to 14 microseconds of weight
// streaming each (Sec. 4.1: the decode phase is bound by loading the weights), and the gaps, ramps
// and tails between them cost more than the streaming.  This kernel keeps one persistent grid
// resident for the whole step: the plan's entries carry a stage number, stages run in order, and
// between two stages stands a grid-wide barrier instead of a kernel boundary.  What makes that pay
// is that the weights never depend on x: a wavefront keeps several items of weights in flight in
// registers at all times, across the barrier too, so the weight stream of stage s + 1 is already
// landing while stage s is being finished and the barrier is being crossed.
//
// Roles.  A workgroup (one per compute unit) has CW compute wavefronts and one service wavefront.
//   compute   walks its items -- (4 rows, one slice of K), as in the one-launch kernel -- through
//             all stages with two cursors: the issue cursor runs P items ahead of the compute
//             cursor and only touches weights, scales and zero points; the compute cursor needs
//             the stage's x in LDS and therefore stops at every stage boundary.  Finished rows go
//             to LDS, not to memory: a compute wavefront never stores, and between two stage
//             boundaries it never waits for more than the item it is about to use.
//   service   per stage: writes the workgroup's finished rows to y with write-through stores,
//             waits for them, announces the workgroup's arrival and waits until every workgroup
//             has arrived.
// After that all wavefronts stage the next stage's x into LDS together (one 16-byte block or a few
// per thread, read at agent scope so that no cache of this XCD can answer with an older use of the
// buffer).
//
// Shares.  In a stage every workgroup serves exactly one entry: the workgroups are dealt to the
// stage's entries in proportion to their cost (rows x K x bit-width, from the device-side
// bit-width array), and an entry's 4-row chunks are dealt evenly to its workgroups.  So a stage
// needs one x per workgroup, staged once, right after the barrier.
//
// Barrier.  128 arrival counters, each on a cache line of its own, count up through the launch:
// after its rows of stage s are acknowledged workgroup b adds one to counter b % 128 (adds to one
// counter are served one after the other where the counter lives, 80 ns each: with a single counter
// the last of 256 arrivals is 20 us late, with two workgroups per counter it does not show; an
// arrival word per workgroup, stored or added, made the polls four times as large and the stage
// slower), and a poll reads all the counters, two per lane, against what they must have reached
// after stage s.  One more word is the abort flag.  The wait is bounded: a service
// wavefront that has polled `wait_limit` times raises the abort flag and, if it is the first, adds
// one to a sticky count; every waiter sees the flag at its next poll and every workgroup leaves the
// kernel.  The last workgroup out (one more counter) puts the counters and the flag back to zero,
// so that the next launch, and a replayed HIP graph, find them clean.  All workgroups must be
// resident together (the host launches at most as many as fit).
//
// What a stage costs (7B-shaped stack, bits from {4, 8}, time stamps of every workgroup, 12.4 us
// per stage in all): the compute wavefronts' part 6.1 us; the workgroup's rows summed, stored and
// acknowledged 1.5; the wait for the other workgroups 3.8 (of which 1.0 is the median spread of the
// arrivals, 2.0 the way of the last arrival to the pollers); x 0.8.  In the compute part a wavefront
// hardly ever waits for an item's data (35 ns per item); it spends 1.1 us per item computing and 0.7
// requesting the next -- and with the arithmetic taken out, 0.2 and 1.8: the requests are accepted
// at the rate memory serves them, so the compute part is the stage's bytes at memory speed, and it
// does not overlap with the 6 us of the boundary, during which nothing is requested.
//
// Arithmetic: the item code of the one-launch kernel (fq_gemv.h).  A row whose slices are shared
// by two wavefronts is the sum, in wavefront order, of their partial sums: deterministic, the same
// whether the stage runs alone or after others, but not the one-launch kernel's order of additions.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

#include "../../include/flexq.h"
#include "fq_internal.h"
#include "fq_gemv.h"

namespace {

constexpr int CW = 8;                  // compute wavefronts per workgroup
constexpr int THREADS = (CW + 1) * 64; // + the service wavefront: up to three wavefronts per SIMD, 168 registers each
constexpr int P = 3;                   // items in flight per compute wavefront (register sets), 8 loads each.
                                       // Measured on the 7B-shaped step (ms, bits from {4,8} / all 4 / all 8):
                                       // CW 7, P 7: 1.86 / 1.57 / 2.05;  CW 8, P 4: 1.77 / 1.50 / 1.97;
                                       // CW 7, P 5: 1.84 / 1.54 / 2.03;  CW 11, P 3: 1.79 / 1.52 / 2.05;
                                       // and with the 128-counter barrier: CW 8, P 4 / 3 / 2: 1.485 / 1.476 / 1.476
                                       // (P 5 spills: 2.11), CW 9, P 3: 1.52, CW 10, P 3: 1.54, CW 6, P 5: 1.58,
                                       // CW 11 and 12, P 2: 1.54 and 1.56 -- the depth hardly matters, more
                                       // wavefronts cost
constexpr int XU = 3;                  // 16-byte blocks of x a thread fetches before it places them

// What a workgroup does in one stage.  64 bytes, kept in LDS for every stage of the plan.
struct Share {
    const uint8_t *codes; // the copy selected by the entry's bit-width (fp16 weights for 16)
    const float *scales;
    const uint8_t *zeros;
    const uint16_t *x;
    uint16_t *y;
    int N, K;
    int c0, c1; // this workgroup's 4-row chunks of the entry
    int bits;   // 0: nothing to do in this stage
    int pad;
};
static_assert(sizeof(Share) == 64, "Share is read from LDS as four 16-byte pieces");
static_assert(CW <= 15, "one word of the flags line per compute wavefront");

// Relative cost of one row of one quantization group at each width (the one-launch kernel's table).
__device__ __forceinline__ long long group_cost(const FqLinearDesc &d, int bits)
{
    if (bits == 2)
        return d.codes2 ? 64 * 230 * 730 / 1000 : 0;
    if (bits == 3)
        return d.codes3 ? 64 * 230 * 950 / 1000 : 0;
    if (bits == 4)
        return d.codes4 ? 64 * 230 : 0;
    if (bits == 8)
        return d.codes8 ? 128 * 200 : 0;
    if (bits == 16)
        return d.w16 ? 256 * 200 : 0;
    return 0;
}

__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

template <class T>
__device__ __forceinline__ T *uni_ptr(T *p)
{
    const uint64_t v = (uint64_t)p;
    const uint32_t lo = (uint32_t)uni((int)(uint32_t)v), hi = (uint32_t)uni((int)(uint32_t)(v >> 32));
    return (T *)(((uint64_t)hi << 32) | lo);
}

// f(0), f(1), ... with the index a compile-time constant.
template <class F, int... I>
__device__ __forceinline__ void for_each_index(F &f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}

// Workgroup barrier that leaves vector memory loads in flight: LDS traffic of this wavefront done,
// then s_barrier (no fence: __syncthreads() would wait for vmcnt(0)).
__device__ __forceinline__ void wg_barrier()
{
    __builtin_amdgcn_s_waitcnt(0xc07f); // lgkmcnt(0)
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// What one lane holds for one item in flight: 16 bytes of codes of each of the 4 rows, and its part
// of the item's scales and zero points, which are fetched TRANSPOSED: a slice touches GS = 32 / 16 /
// 8 groups of a row (2 / 4 / 8 bits), so (4 rows x GS groups) fit one or two loads of the wavefront
// -- lane l fetches row l / GS, group l % GS -- instead of one load per row and lane.  Eight load
// instructions and 20 registers per item; the lanes pick their rows' values out of the other lanes
// (ds_bpermute) when the item is computed.
struct Item {
    uint4 w[ROWS_PER_WAVE];
    float s[2];
    uint8_t z[2]; // kept as bytes: widened where used, so that nothing touches a register while its load is in flight
};

// One walker over a compute wavefront's items: stage by stage; inside a stage the workgroup's
// items -- its chunks in order, inside a chunk the slices in order -- are cut into CW equal runs,
// one per compute wavefront, so a chunk's slices may be shared by neighbouring wavefronts (a stage
// often gives a workgroup fewer chunks than it has wavefronts).  Uniform over the wavefront.  What
// an item's addresses need is kept per stage and per chunk, so that an item costs a handful of
// instructions: the wavefronts issue a few hundred instructions per 4 KiB of weights, and at five
// items per wavefront and stage that, not memory, is what a stage's compute part is made of.
struct Cursor {
    // per stage
    const uint8_t *codes;
    const float *scales;
    const uint8_t *zeros;
    int N, K, bits;
    int s;              // stage
    int item, end;      // this wavefront's items [item, end) still to do in stage s, counted from the share's first
    int nslice;
    int first;          // chunk (relative to the share's first) this wavefront's run begins in
    int wg_c0;          // the share's first chunk
    int csh, rsh, gsh;  // log2(codes per lane and slice); bytes = (2 k) >> rsh; log2(groups per slice)
    uint32_t row_bytes, G, kmax;
    // per chunk
    int chunk, j;       // chunk (absolute) and slice of `item`
    const uint8_t *crow; // codes of the chunk's first row
    const float *srow;
    const uint8_t *zrow;
    int last;           // rows of the chunk that exist, minus one (3 but for the matrix's last chunk)
};

__device__ __forceinline__ void set_chunk(Cursor &c)
{
    const int row0 = c.chunk * ROWS_PER_WAVE;
    c.last = min(ROWS_PER_WAVE - 1, c.N - 1 - row0);
    c.crow = c.codes + (size_t)row0 * c.row_bytes;
    c.srow = c.scales + (size_t)row0 * c.G;
    c.zrow = c.zeros + (size_t)row0 * c.G;
}

// A stage's constants for an entry of `bits` bits with rows of K inputs.
__device__ __forceinline__ void set_width(Cursor &c, int bits, int K)
{
    c.bits = bits;
    c.K = K;
    c.csh = bits == 2 ? 6 : bits == 4 || bits == 3 ? 5 : bits == 8 ? 4 : 3;
    c.rsh = bits == 2 ? 3 : bits == 4 ? 2 : bits == 8 ? 1 : 0; // (3 bits: unused)
    c.gsh = c.csh - 1; // 32 / 16 / 8 groups per slice (fp16: unused)
    c.row_bytes = bits == 3 ? ((uint32_t)K >> 3) * 3u : (2u * (uint32_t)K) >> c.rsh;
    c.G = (uint32_t)K >> 7;
    c.kmax = (uint32_t)K - (1u << c.csh);
}

__device__ __forceinline__ void enter_stage(Cursor &c, const Share *shares, int s, int wave)
{
    const Share *sh = &shares[s];
    c.s = s;
    const int bits = uni(sh->bits);
    c.codes = uni_ptr(sh->codes);
    c.scales = uni_ptr(sh->scales);
    c.zeros = uni_ptr(sh->zeros);
    c.N = uni(sh->N);
    set_width(c, bits, uni(sh->K));
    const int c0 = uni(sh->c0), c1 = uni(sh->c1);
    c.nslice = bits ? (c.K + slice_span(bits) - 1) / slice_span(bits) : 1;
    const int n = bits ? (c1 - c0) * c.nslice : 0;
    c.wg_c0 = c0;
    c.item = n * wave / CW; // (at most 1024 chunks x 64 slices x CW: no overflow)
    c.end = n * (wave + 1) / CW;
    c.first = c.item / c.nslice;
    c.chunk = c0 + c.first;
    c.j = c.item - c.first * c.nslice;
    if (c.item < c.end)
        set_chunk(c);
}

// The cursor's item is done (or requested): on to the next one of the run.
__device__ __forceinline__ void advance(Cursor &c)
{
    c.item++;
    if (++c.j == c.nslice) {
        c.j = 0;
        c.chunk++;
        if (c.item < c.end)
            set_chunk(c);
    }
}

// The loads of the cursor's item: the same eight load instructions whatever the bit-width (a
// run-time value), so that the count of loads in flight is the same on every path.  For 16 bits
// scales and zeros alias the weights (loaded, never used).
__device__ __forceinline__ void issue_item(const Cursor &c, Item &L)
{
    const int lane = threadIdx.x & 63;
    const uint32_t k0 = min((uint32_t)(c.j * 64 + lane) << c.csh, c.kmax);
    // 3 bits: the lane's block of 12 bytes comes with 4 bytes of a neighbour, the next block's
    // first for an even block, the previous block's last for an odd one (a row holds an even
    // number of blocks, so the 16 bytes never leave the row)
    const uint32_t blk = k0 >> 5;
    const uint32_t byte0 = c.bits == 3 ? blk * 12u - ((blk & 1u) << 2) : (2 * k0) >> c.rsh;
#pragma unroll
    for (int r = 0; r < ROWS_PER_WAVE; r++) // a row past the matrix's last repeats the last (discarded)
        L.w[r] = load16_stream_a4(c.crow + (byte0 + (uint32_t)min(r, c.last) * c.row_bytes)); // (3 bits: 8-byte aligned)
    // scales and zero points: lane l -> (row l >> gsh, group l & (GS - 1)) of the slice; at 2 bits the
    // second pair of loads takes rows 2 and 3, at the other widths it repeats the first
    const uint32_t g = min(((uint32_t)c.j << c.gsh) + (uint32_t)(lane & ((1 << c.gsh) - 1)), c.G - 1);
    const int rr = (lane >> c.gsh) & 3;
#pragma unroll
    for (int h = 0; h < 2; h++) {
        const uint32_t idx = (uint32_t)min(c.bits == 2 ? rr + 2 * h : rr, c.last) * c.G + g;
        L.s[h] = as_global<float>(c.srow)[idx];
        L.z[h] = as_global<uint8_t>(c.zrow)[idx];
    }
    // the loads stay here: the compiler would otherwise sink some of them towards their first use,
    // steps later, where their latency is no longer hidden
    asm volatile("" ::: "memory");
}

// The item as the shared arithmetic takes it: every lane gets the scale and zero point of its own
// group for each of the four rows from the lane that fetched them.
__device__ __forceinline__ void expand(const Item &I, const Cursor &c, Loaded &L)
{
    const int lane = threadIdx.x & 63;
    const uint32_t k0 = min((uint32_t)(c.j * 64 + lane) << c.csh, c.kmax);
    const int gi = (int)(k0 >> 7) - (c.j << c.gsh); // my group's place among the slice's groups
    const bool two = c.bits == 2;
    const bool odd3 = c.bits == 3 && ((k0 >> 5) & 1u); // a 3-bit block that sits in the last 12 of its 16 bytes
#pragma unroll
    for (int r = 0; r < ROWS_PER_WAVE; r++) {
        L.w[r] = I.w[r];
        if (odd3)
            L.w[r] = make_uint4(I.w[r].y, I.w[r].z, I.w[r].w, 0u);
        const int src = (((two ? r & 1 : r) << c.gsh) + gi) << 2;
        const bool h = two && r >= 2;
        L.s[r] = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(src, __builtin_bit_cast(int, h ? I.s[1] : I.s[0])));
        L.z[r] = (uint8_t)__builtin_amdgcn_ds_bpermute(src, (int)(h ? I.z[1] : I.z[0]));
    }
}

// 16 bytes of x, read at agent scope (two 64-bit relaxed atomic loads: they are served where the
// other XCDs' write-through stores have arrived, whatever this XCD's caches still hold of an
// earlier use of the buffer).
__device__ __forceinline__ uint4 load16_coherent(const uint16_t *p)
{
    const FQ_GLOBAL uint64_t *q = (const FQ_GLOBAL uint64_t *)p;
    const uint64_t lo = __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const uint64_t hi = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return make_uint4((uint32_t)lo, (uint32_t)(lo >> 32), (uint32_t)hi, (uint32_t)(hi >> 32));
}

// x of one entry into LDS in the layout of its bit-width, by all THREADS threads of the workgroup:
// XU blocks per thread are requested before the first is placed, so a row of up to 12288 inputs
// costs one memory round trip and three blocks' worth of placing per thread.
template <int BITS>
__device__ __forceinline__ void stage_x_all(const uint16_t *x, int K, uint4 *lds)
{
    const int tid = threadIdx.x;
    const int Kp = padded_k(K, BITS);
    if (BITS == 3) {
        const int nls = Kp >> 5; // lane slices of 32 k, one per thread and trip
        float2 *sums = reinterpret_cast<float2 *>(lds + (Kp >> 3));
        for (int ls = tid; ls < nls; ls += THREADS) {
            uint4 v[4];
#pragma unroll
            for (int i = 0; i < 4; i++)
                v[i] = ls * 32 < K ? load16_coherent(x + (size_t)ls * 32 + 8 * i) : make_uint4(0, 0, 0, 0);
            place_slice3(ls, v, lds, sums);
        }
        return;
    }
    if (BITS == 2) {
        const int npair = Kp >> 4; // a multiple of 256
        float2 *sums = reinterpret_cast<float2 *>(lds + (Kp >> 3));
        for (int base = 0; base < npair; base += THREADS * XU) {
            uint4 va[XU], vb[XU];
#pragma unroll
            for (int u = 0; u < XU; u++) {
                const int pb = base + u * THREADS + tid;
                va[u] = make_uint4(0, 0, 0, 0);
                vb[u] = make_uint4(0, 0, 0, 0);
                if (pb < npair && pb * 16 < K) {
                    va[u] = load16_coherent(x + (size_t)pb * 16);
                    vb[u] = load16_coherent(x + (size_t)pb * 16 + 8);
                }
            }
#pragma unroll
            for (int u = 0; u < XU; u++) {
                const int pb = base + u * THREADS + tid;
                if (((base + u * THREADS + tid) & ~63) < npair) // uniform over the wavefront: npair is a multiple of 64
                    place_pair2(pb, va[u], vb[u], lds, sums);
            }
        }
        return;
    }
    const int nblk = Kp >> 3; // a multiple of 64
    float *sums = reinterpret_cast<float *>(lds + nblk);
    for (int base = 0; base < nblk; base += THREADS * XU) {
        uint4 v[XU];
#pragma unroll
        for (int u = 0; u < XU; u++) {
            const int b = base + u * THREADS + tid;
            v[u] = make_uint4(0, 0, 0, 0);
            if (b < nblk && b * 8 < K)
                v[u] = load16_coherent(x + (size_t)b * 8);
        }
#pragma unroll
        for (int u = 0; u < XU; u++) {
            const int b = base + u * THREADS + tid;
            if ((b & ~63) < nblk) // uniform over the wavefront
                place_block<BITS>(b, v[u], lds, sums);
        }
    }
}

__device__ __forceinline__ void stage_share_x(const Share *sh, uint4 *xbuf)
{
    const int bits = uni(sh->bits);
    if (bits == 0 || uni(sh->c1) <= uni(sh->c0))
        return;
    const uint16_t *x = uni_ptr(sh->x);
    const int K = uni(sh->K);
    if (bits == 2)
        stage_x_all<2>(x, K, xbuf);
    else if (bits == 3)
        stage_x_all<3>(x, K, xbuf);
    else if (bits == 4)
        stage_x_all<4>(x, K, xbuf);
    else if (bits == 8)
        stage_x_all<8>(x, K, xbuf);
    else
        stage_x_all<16>(x, K, xbuf);
}

// Rows finished in this stage, LDS -> y.  A row's value is the sum, in wavefront order, of the
// partial sums of the wavefronts that shared its chunk (mostly one).  The stores write through to
// memory (visible to the other XCDs' caches once acknowledged).
__device__ __forceinline__ void store_share_y(const Share *sh, const float *part, int PK, const int *firsts)
{
    const int lane = threadIdx.x & 63;
    const int bits = uni(sh->bits), c0 = uni(sh->c0), c1 = uni(sh->c1), N = uni(sh->N), K = uni(sh->K);
    if (bits == 0 || c1 <= c0)
        return;
    uint16_t *y = uni_ptr(sh->y);
    const int nslice = (K + slice_span(bits) - 1) / slice_span(bits);
    const int n = (c1 - c0) * nslice; // items of the share (at most 1024 chunks x 64 slices)
    const int row0 = c0 * ROWS_PER_WAVE, rows = min(c1 * ROWS_PER_WAVE, N) - row0;
    for (int i = lane; i < rows; i += 64) {
        const int c = i / ROWS_PER_WAVE, r = i % ROWS_PER_WAVE; // chunk relative to the share's first
        float v = 0.0f;
#pragma unroll
        for (int w = 0; w < CW; w++) {
            const int i0 = n * w / CW, i1 = n * (w + 1) / CW; // wavefront w's run of items
            if (i1 > i0 && i0 < (c + 1) * nslice && i1 > c * nslice)
                v += part[(w * PK + (c - firsts[w])) * ROWS_PER_WAVE + r]; // firsts[w] = i0 / nslice, left by wavefront w
        }
        const uint32_t h = to_half_bits(v);
        uint16_t *p = y + row0 + i;
        asm volatile("global_store_short %0, %1, off sc0 sc1" ::"v"(p), "v"(h) : "memory");
    }
}

// Layout of the plan's sync words (ints): the abort flag, the sticky count of launches that gave
// up, flags (bit 0: an entry's bit-width is not attached to its layer, its y was left untouched;
// bit 1: a share too large for the results buffer), on the next line the count of finished
// workgroups, and from SY_COUNTERS on the NC arrival counters, CSTRIDE ints apart.
constexpr int NC = 128;     // arrival counters (workgroup b adds to counter b % NC)
constexpr int CSTRIDE = 32; // ints between two counters: a line each
constexpr int CPL = (NC + 63) / 64;  // counters a polling lane watches
static_assert(NC >= 1 && CPL <= 4, "a lane polls up to four counters");
constexpr int SY_ABORT = 0, SY_GAVE_UP = 1, SY_FLAGS = 2, SY_DONE = 32, SY_COUNTERS = 64;
static_assert((SY_COUNTERS + NC * CSTRIDE) * 4 <= FQ_STAGED_SYNC_BYTES, "the sync words fit the plan's workspace");

struct Polled {
    int c[CPL];
    int flag;
};

// Waits until every workgroup has arrived at the end of stage s.  False: the launch is aborted.
// Lane l watches counter l (and l + 64), lane 0 the abort flag besides.  A poll is a round trip to
// memory of a microsecond or more, so two are kept in flight: the arrival of the last workgroup is
// seen about one round trip after it happened, not up to two.  (A poll is 129 requests of the
// workgroup, and the polls of 256 workgroups compete with the arrivals they wait for: 7B-shaped
// step with 8 / 6 / 4 / 3 / 2 polls in flight: 1.58 / 1.56 / 1.51 / 1.50 / 1.50 ms.)
__device__ __forceinline__ bool wait_stage(int *sync, int s, int G, long long wait_limit)
{
    const int lane = threadIdx.x & 63;
    int mine[CPL];
#pragma unroll
    for (int i = 0; i < CPL; i++)
        mine[i] = lane + 64 * i < NC ? (s + 1) * ((G - (lane + 64 * i) + NC - 1) / NC) : 0; // workgroups b with b % NC = lane + 64 i
    auto poll = [&]() -> Polled {
        Polled p;
#pragma unroll
        for (int i = 0; i < CPL; i++)
            p.c[i] = lane + 64 * i < NC ? __hip_atomic_load(&sync[SY_COUNTERS + CSTRIDE * (lane + 64 * i)], __ATOMIC_RELAXED,
                                                            __HIP_MEMORY_SCOPE_AGENT)
                                        : 0;
        p.flag = 0;
        if (lane == 0)
            p.flag = __hip_atomic_load(&sync[SY_ABORT], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return p;
    };
    constexpr int Q = 2;
    Polled v[Q];
#pragma unroll
    for (int q = 0; q + 1 < Q; q++) {
        v[q] = poll();
        __builtin_amdgcn_s_sleep(1);
    }
    for (long long it = 0;; it += Q) {
#pragma unroll
        for (int q = 0; q < Q; q++) {
            v[(q + Q - 1) % Q] = poll();
            const Polled got = v[q]; // the oldest of the polls in flight
            if (__builtin_amdgcn_readfirstlane(got.flag))
                return false;
            bool ok = true;
#pragma unroll
            for (int i = 0; i < CPL; i++)
                ok = ok && got.c[i] >= mine[i];
            if (__builtin_amdgcn_ballot_w64(ok) == ~0ull)
                return true;
            __builtin_amdgcn_s_sleep(1);
        }
        if (it >= wait_limit) {
            // the first to give up in this launch raises the flag and counts the launch
            if (lane == 0 &&
                __hip_atomic_exchange(&sync[SY_ABORT], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0)
                __hip_atomic_fetch_add(&sync[SY_GAVE_UP], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return false;
        }
    }
}


__global__ __launch_bounds__(THREADS) void decode_staged_kernel(const FqLinearDesc *__restrict__ table,
                                                                const int32_t *__restrict__ bits_dev,
                                                                const int32_t *__restrict__ stage_begin,
                                                                int n_stages, int *sync, long long wait_limit,
                                                                int res_chunks)
{
    extern __shared__ uint4 lds[];
    const int PK = res_chunks / CW + 2; // chunks one wavefront can have a hand in per stage
    Share *shares = reinterpret_cast<Share *>(lds);                  // [n_stages]
    float *part = reinterpret_cast<float *>(lds + 4 * n_stages);     // [CW][PK][4] partial rows
    int *flags = reinterpret_cast<int *>(lds + 4 * n_stages + CW * PK); // [0]: abort; [1 + w]: first chunk of wavefront w's run
    uint4 *xbuf = lds + 4 * n_stages + CW * PK + 4;
    const int wave = uni(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int G = gridDim.x, b = blockIdx.x;

    // ---- every workgroup's share of every stage -------------------------------------------
    bool too_large = false, unattached = false;
    for (int s = threadIdx.x; s < n_stages; s += THREADS) {
        const int e0 = stage_begin[s], e1 = stage_begin[s + 1];
        long long C = 0;
        for (int e = e0; e < e1; e++) {
            const long long gc = group_cost(table[e], bits_dev[e]);
            unattached = unattached || gc == 0;
            C += gc * (table[e].K >> 7) * ((table[e].N + 3) >> 2);
        }
        Share sh = {};
        if (C > 0) {
            const long long avail = G - (e1 - e0);
            long long prefix = 0;
            for (int e = e0; e < e1; e++) {
                const FqLinearDesc d = table[e];
                const int bits = bits_dev[e];
                const int chunks = (d.N + 3) >> 2;
                const long long cost = group_cost(d, bits) * (d.K >> 7) * chunks;
                const int g_lo = (e - e0) + (int)(avail * prefix / C);
                prefix += cost;
                const int g_hi = (e - e0 + 1) + (int)(avail * prefix / C);
                if (b >= g_lo && b < g_hi && cost > 0) {
                    const long long idx = b - g_lo, n = g_hi - g_lo;
                    sh.codes = bits == 2   ? d.codes2
                               : bits == 3 ? d.codes3
                               : bits == 4 ? d.codes4
                               : bits == 8 ? d.codes8
                                           : (const uint8_t *)d.w16;
                    sh.scales = bits == 2   ? d.scales2
                                : bits == 3 ? d.scales3
                                : bits == 4 ? d.scales4
                                : bits == 8 ? d.scales8
                                            : (const float *)d.w16;
                    sh.zeros = bits == 2   ? d.zeros2
                               : bits == 3 ? d.zeros3
                               : bits == 4 ? d.zeros4
                               : bits == 8 ? d.zeros8
                                           : (const uint8_t *)d.w16;
                    sh.x = d.x;
                    sh.y = d.y;
                    sh.N = d.N;
                    sh.K = d.K;
                    sh.c0 = (int)(chunks * idx / n);
                    sh.c1 = (int)(chunks * (idx + 1) / n);
                    sh.bits = bits;
                    if (sh.c1 - sh.c0 > res_chunks) { // more rows than the results buffer holds: refuse
                        too_large = true;
                        sh.bits = 0;
                    }
                }
            }
        }
        shares[s] = sh;
    }
    if (threadIdx.x == 0)
        flags[0] = 0;
    if (unattached && b == 0)
        __hip_atomic_fetch_or(&sync[SY_FLAGS], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (too_large)
        __hip_atomic_fetch_or(&sync[SY_FLAGS], 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();

    // x of stage 0: by everyone, before anything else is requested
    stage_share_x(&shares[0], xbuf);

    if (wave == CW) {
        // ---- service wavefront ------------------------------------------------------------
        wg_barrier(); // x of stage 0 is in LDS
        for (int s = 0; s < n_stages; s++) {
            wg_barrier(); // the compute wavefronts' rows of stage s are in LDS
            store_share_y(&shares[s], part, PK, flags + 1);
            if (s + 1 == n_stages)
                break;
            __builtin_amdgcn_s_waitcnt(0x0f70); // vmcnt(0): the stores are acknowledged
            if (lane == 0)
                __hip_atomic_fetch_add(&sync[SY_COUNTERS + CSTRIDE * (b % NC)], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const bool aborted = !wait_stage(sync, s, G, wait_limit);
            if (aborted && lane == 0)
                flags[0] = 1;
            wg_barrier(); // every workgroup has arrived (or the abort flag is up)
            if (aborted)
                break;
            stage_share_x(&shares[s + 1], xbuf); // with the compute wavefronts
            __builtin_amdgcn_s_waitcnt(0xc07f);
            wg_barrier(); // x of stage s + 1 is in LDS
        }
        // last workgroup out puts the counters back
        if (lane == 0) {
            const int done = __hip_atomic_fetch_add(&sync[SY_DONE], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (done == G - 1) {
                for (int l = 0; l < NC; l++)
                    __hip_atomic_store(&sync[SY_COUNTERS + CSTRIDE * l], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(&sync[SY_ABORT], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(&sync[SY_DONE], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        return;
    }

    // ---- compute wavefronts ---------------------------------------------------------------
    Cursor ic, cc;
    enter_stage(ic, shares, 0, wave);
    enter_stage(cc, shares, 0, wave);
    if (lane == 0)
        flags[1 + wave] = cc.first;
    bool more = true; // the issue cursor still has items
    Item L[P];
    // Next item of the issue cursor into dst.  Past its last item the cursor is parked on the head of
    // the table (cached, the result discarded): the same eight load instructions -- the compiler
    // counts the loads in flight per path, and only with the same count on every path does it let
    // a set's loads stay in flight until the set is used.
    auto park = [&]() __attribute__((always_inline)) {
        more = false;
        ic.codes = (const uint8_t *)table;
        ic.scales = (const float *)table;
        ic.zeros = (const uint8_t *)table;
        ic.N = 1;
        set_width(ic, 16, 128);
        ic.chunk = 0;
        ic.j = 0;
        set_chunk(ic);
    };
    auto issue_next = [&](Item &dst) __attribute__((always_inline)) {
        while (more && ic.item >= ic.end) {
            if (ic.s + 1 >= n_stages)
                park();
            else
                enter_stage(ic, shares, ic.s + 1, wave);
        }
        issue_item(ic, dst);
        if (more)
            advance(ic);
    };
#pragma unroll
    for (int p = 0; p < P; p++)
        issue_next(L[p]);
    wg_barrier(); // x of stage 0 is in LDS
    float acc[ROWS_PER_WAVE] = {0.f, 0.f, 0.f, 0.f};
    // The loop is left at its bottom only.  The compiler counts the loads in flight per path, and it
    // routes every exit of a loop through the loop's latch: with a way out from the middle, each
    // step would have to wait as if its set had been requested last.  So a wavefront that is done
    // in step p idles through the rest of the round (requesting loads that are discarded).
    bool finished = false;
    // One step of the round on set p (a compile-time index: the sets must stay in registers).
    auto step = [&](auto pc) __attribute__((always_inline)) {
        constexpr int p = decltype(pc)::value;
        // bring the compute cursor to its next item, crossing stage boundaries on the way
        while (!finished && cc.item >= cc.end) {
            wg_barrier(); // this wavefront's rows of stage cc.s are in LDS
            if (cc.s + 1 >= n_stages) {
                finished = true;
            } else {
                wg_barrier(); // every workgroup has arrived (or the abort flag is up)
                if (uni(flags[0])) {
                    finished = true;
                } else {
                    // x of the next stage, with the service wavefront.  This waits for every load of
                    // this wavefront (returns are in order); they were all requested before the
                    // barrier was entered, microseconds ago.
                    stage_share_x(&shares[cc.s + 1], xbuf);
                    wg_barrier(); // x of the next stage is in LDS
                    enter_stage(cc, shares, cc.s + 1, wave);
                    if (lane == 0)
                        flags[1 + wave] = cc.first;
                }
            }
        }
        if (!finished) {
            Loaded T;
            expand(L[p], cc, T);
            if (cc.bits == 2)
                compute<2>(cc.K, cc.j, T, xbuf, acc);
            else if (cc.bits == 3)
                compute<3>(cc.K, cc.j, T, xbuf, acc);
            else if (cc.bits == 4)
                compute<4>(cc.K, cc.j, T, xbuf, acc);
            else if (cc.bits == 8)
                compute<8>(cc.K, cc.j, T, xbuf, acc);
            else
                compute<16>(cc.K, cc.j, T, xbuf, acc);
            if (cc.j + 1 == cc.nslice || cc.item + 1 == cc.end) {
                // this wavefront's part of the chunk's four rows: reduce over the lanes, lane 63
                // leaves the sums in LDS
                float v[ROWS_PER_WAVE];
#pragma unroll
                for (int r = 0; r < ROWS_PER_WAVE; r++) {
                    v[r] = wave_sum_lane63(acc[r]);
                    acc[r] = 0.0f;
                }
                if (lane == 63)
                    *reinterpret_cast<float4 *>(part + ((size_t)wave * PK + (cc.chunk - cc.wg_c0 - cc.first)) * ROWS_PER_WAVE) =
                        make_float4(v[0], v[1], v[2], v[3]);
            }
            advance(cc);
        }
        issue_next(L[p]);
    };
    do {
        for_each_index(step, std::make_integer_sequence<int, P>{});
    } while (!finished);
}

} // namespace


size_t fq_staged_lds_bytes(int n_stages, int max_K, int res_chunks)
{
    const size_t kp4 = ((size_t)max_K + 2047) / 2048 * 2048, kp2 = ((size_t)max_K + 4095) / 4096 * 4096;
    const size_t b4 = kp4 * 2 + kp4 / 32 * 8, b2 = kp2 * 2 + kp2 / 64 * 8;
    return (size_t)n_stages * sizeof(Share) + (size_t)CW * (res_chunks / CW + 2) * 16 + 64 + (b4 > b2 ? b4 : b2) + 64;
}

// Workgroups of the staged kernel: one per compute unit, and never more than fit at once (they
// wait for each other).  0: the kernel does not fit with this much LDS.
int fq_staged_grid(size_t lds_bytes)
{
    if (lds_bytes > 48 * 1024 &&
        fq_raise_dynamic_lds((const void *)decode_staged_kernel, 160 * 1024) != hipSuccess)
        return 0;
    const int per_cu = fq_workgroups_per_cu((const void *)decode_staged_kernel, THREADS, lds_bytes, 0);
    return per_cu < 1 ? 0 : fq_device_cus();
}

hipError_t fq_launch_decode_staged(const FqLinearDesc *table_dev, const int32_t *bits_dev,
                                   const int32_t *stage_begin_dev, int n_stages, int max_K, int res_chunks,
                                   int *sync_dev, long long wait_limit, hipStream_t stream)
{
    const size_t lds = fq_staged_lds_bytes(n_stages, max_K, res_chunks);
    const int grid = fq_staged_grid(lds);
    if (grid < 1)
        return hipErrorInvalidConfiguration;
    decode_staged_kernel<<<grid, THREADS, lds, stream>>>(table_dev, bits_dev, stage_begin_dev, n_stages, sync_dev,
                                                         wait_limit, res_chunks);
    return hipGetLastError();
}
