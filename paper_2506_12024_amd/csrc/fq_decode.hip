// Decode-phase weight-only quantized linear for gfx950: y = x . dequant(W)^T
// with dequant = Sec. 2.2 Eq. (3), one row of x (this file: M = 1, a GEMV).
// The decode phase is bound by streaming the weights (Sec. 4.1), so the kernel
// is built around the HBM stream: it reads the packed copy of the bit-width
// chosen for this call exactly once with coalesced 128-bit loads and keeps
// everything else (x, per-slice sums of x) in LDS.
//
// Work list.  A launch serves one linear (descriptor passed by value) or a
// table of independent linears (plan).  Rows are cut into tiles of `tile_rows`
// (a multiple of 16: 4 wavefronts x chunks of 4 rows; small for a single linear
// so that every CU gets work, large for a plan so that staging x is amortised);
// a single linear's tiles are dealt round-robin (workgroup b takes tiles b,
// b + gridDim, ...), a plan's rows are cut by cost (see "work partition" below).
// The bit-width of an entry (2, 3, 4, 8 or 16) is a run-time value (host argument
// or device array): all inner loops live in the one kernel and the choice is a
// wavefront-uniform branch, so switching precision per token costs a pointer
// select and nothing else.
//
// Streaming.  Inside a tile a wavefront walks items = (chunk of 4 rows, slice);
// an item is four non-temporal 128-bit loads per lane plus the scale and zero
// of each row's group.  The loads of item i+1 are issued before item i is
// computed (two register sets, loop unrolled by two so no set is ever copied),
// and the first item of a tile is issued before x is staged, so eight loads per
// lane are in flight almost all the time.
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
// 2-bit and 3-bit: fields of a half that lie inside its mantissa read as offset +
// code under the exponent that fits their place (the shared header has the layouts);
// both are bound by the vector ALUs rather than by the stream, which is why a plan
// launch lets more workgroups per compute unit take part when its bit-widths are low.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/flexq.h"
#include "fq_internal.h"
#include "fq_gemv.h"

namespace {

constexpr int WG_THREADS = 256;
constexpr int WAVES = WG_THREADS / 64;
constexpr int TILE_ROWS_MIN = WAVES * ROWS_PER_WAVE;

// One tile for one wavefront: rows [row_begin, row_end) in chunks of 4, all slices.
// `need_stage`: x of this entry is not in LDS yet (uniform over the workgroup).
template <int BITS>
__device__ __forceinline__ void run_tile(const Sel &d, const uint16_t *x, uint16_t *y, int row_begin,
                                         int row_end, bool need_stage, uint4 *lds)
{
    const int lane = threadIdx.x & 63;
    const int nslice = (d.K + slice_span(BITS) - 1) / slice_span(BITS);
    const int nchunk = row_end > row_begin ? (row_end - row_begin + ROWS_PER_WAVE - 1) / ROWS_PER_WAVE : 0;
    const int nitem = nchunk * nslice;
    Loaded A, B;
    // weights do not depend on x: get the first item moving before the staging barrier
    if (nitem > 0)
        issue<BITS>(d, row_begin, 0, A);
    if (need_stage) {
        __syncthreads(); // every wavefront is done reading the previous x
        stage_x<BITS, WG_THREADS>(x, d.K, lds);
        __syncthreads();
    }
    float acc[ROWS_PER_WAVE] = {0.f, 0.f, 0.f, 0.f};
    int c = 0, j = 0; // chunk and slice of the item being computed
    auto finish = [&](int chunk) {
        const int row0 = row_begin + chunk * ROWS_PER_WAVE;
#pragma unroll
        for (int r = 0; r < ROWS_PER_WAVE; r++) {
            const float v = wave_sum_lane63(acc[r]);
            if (lane == 63 && row0 + r < row_end)
                ((FQ_GLOBAL uint16_t *)y)[row0 + r] = to_half_bits(v);
            acc[r] = 0.0f;
        }
    };
    // One step: issue item i+1 into Lnext, compute item i from Lcur.
    auto step = [&](int i, Loaded &Lcur, Loaded &Lnext) {
        int cn = c, jn = j + 1;
        if (jn == nslice) {
            jn = 0;
            cn = c + 1;
        }
        // Always issued (past the last item it re-reads the last chunk) so that the wait
        // for Lcur can be a counted vmcnt with Lnext's loads still in flight.
        const bool more = i + 1 < nitem;
        issue<BITS>(d, row_begin + (more ? cn : c) * ROWS_PER_WAVE, more ? jn : j, Lnext);
        compute<BITS>(d.K, j, Lcur, lds, acc);
        if (jn == 0)
            finish(c);
        c = cn;
        j = jn;
    };
    for (int i = 0; i < nitem; i += 2) {
        step(i, A, B);
        if (i + 1 < nitem)
            step(i + 1, B, A);
    }
}

// ---- work partition of a plan ---------------------------------------------------
// The entries of a plan cost very different amounts (rows x K x bit-width, and the
// bit-widths are only known on the device), so a static deal of equal row tiles would
// leave the workgroups with the expensive tiles streaming alone at the end.  Instead
// every workgroup computes, from the table and the bit-width array, the same prefix sum
// of costs and takes the slice [b C / G, (b + 1) C / G) of the total cost C: a
// contiguous run of 16-row units, possibly spanning a few entries.  No atomics, no
// tail, and x is staged once per entry a workgroup touches.

struct Cut {
    int e;       // entry the boundary falls in (count = past the end)
    int unit;    // 16-row unit inside that entry
};

// Relative time of one quantization group (128 k) of one row at each width, a byte of 8-bit codes
// costing 200.  8 and 16 bits stream at the shared HBM rate: cost ~ bytes.  The unpacking of 4 and
// 2 bits makes a workgroup's own rate the limit, so their bytes are charged more: measured on the
// 7B stack, the mixed {4, 8} step takes 0.811 / 0.792 / 0.776 / 0.765 / 0.761 / 0.762 / 0.769 ms
// with a 4-bit byte charged 200 / 210 / 220 / 225 / 230 / 235 / 240, and a 2-bit group charged
// 0.64 / 0.68 / 0.72 / 0.76 / 0.80 of a 4-bit one gives 0.470 / 0.462 / 0.459 / 0.455 / 0.461 ms
// for bits from {2, 4} and 0.633 / 0.628 / 0.629 / 0.632 / 0.634 ms for {2, 4, 8}.
constexpr int W4_COST = 230;     // per byte
constexpr int W2_PER_MILLE = 730; // of the cost of a 4-bit group
constexpr int W3_PER_MILLE = 950; // a 3-bit group: three quarters of the bytes, a third more unpacking (0.511 ms against 0.539 ms for the 7B stack all at 3 or all at 4 bits)
__device__ __forceinline__ long long entry_unit_cost(const FqLinearDesc &d, int bits)
{
    const long long groups = d.K >> 7;
    if (bits == 2)
        return d.codes2 ? groups * (64 * W4_COST * W2_PER_MILLE / 1000) : 0;
    if (bits == 3)
        return d.codes3 ? groups * (64 * W4_COST * W3_PER_MILLE / 1000) : 0;
    if (bits == 4)
        return d.codes4 ? groups * (64 * W4_COST) : 0;
    if (bits == 8)
        return d.codes8 ? groups * (128 * 200) : 0;
    if (bits == 16)
        return d.w16 ? groups * (256 * 200) : 0;
    return 0;
}

// Inclusive scan over the 256 threads of the workgroup; `total` returns the sum.
__device__ __forceinline__ long long block_scan(long long v, long long *tmp, long long &total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const long long o = __shfl_up(v, off, 64);
        if (lane >= off)
            v += o;
    }
    __syncthreads(); // tmp may still be read from a previous call
    if (lane == 63)
        tmp[wave] = v;
    __syncthreads();
    long long before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < WAVES; w++) {
        const long long t = tmp[w];
        all += t;
        if (w < wave)
            before += t;
    }
    total = all;
    return v + before;
}

// Boundaries of this workgroup's slice.  Every thread returns the same values.
__device__ __forceinline__ void partition(const FqLinearDesc *table, const int32_t *bits_dev, int count,
                                          Cut &lo, Cut &hi, int *flags, int cus)
{
    __shared__ long long tmp[WAVES];
    __shared__ Cut cuts[2];
    // pass 1: total cost, and how much of it is at 2 or 3 bits
    long long C = 0, C_low = 0;
    for (int base = 0; base < count; base += WG_THREADS) {
        const int e = base + threadIdx.x;
        long long c = 0, c_low = 0;
        if (e < count) {
            const int bits = bits_dev[e];
            c = entry_unit_cost(table[e], bits) * ((table[e].N + 15) >> 4);
            c_low = bits == 2 || bits == 3 ? c : 0;
            if (c == 0 && flags && blockIdx.x == 0) // no such width, or no copy of it: nobody runs this entry
                *flags = 1;
        }
        long long chunk;
        block_scan(c, tmp, chunk);
        C += chunk;
        block_scan(c_low, tmp, chunk);
        C_low += chunk;
    }
    // Workgroups per compute unit that take part.  8- and 16-bit entries stream fastest with two
    // (fewer concurrent streams, better DRAM page locality: measured on the mixed 7B step 0.867 /
    // 0.763 / 0.788 / 0.795 ms with 1 / 2 / 3 / 4), but 2 and 3 bits are bound by the vector ALUs and
    // want more wavefronts: all at 2 bits 0.378 / 0.359 / 0.352 ms with 2 / 3 / 4, all at 3 bits
    // 0.502 / 0.474 / 0.472, bits from {2, 4} 0.465 / 0.453 / 0.458, from {3, 4} 0.529 / 0.515 /
    // 0.523, all at 4 bits 0.538 / 0.549 / 0.554.  The launch brings four per compute unit (as far
    // as they fit); those that this launch's bit-widths do not call for leave here.
    const int per_cu = C_low * 10 >= C * 9 ? 4 : C_low * 10 >= C * 3 ? 3 : 2;
    const long long G = min((long long)gridDim.x, (long long)per_cu * cus), b = blockIdx.x;
    if (b >= G) {
        lo = hi = Cut{count, 0};
        return;
    }
    const long long t_lo = b * C / G, t_hi = (b + 1) * C / G;
    if (threadIdx.x == 0) {
        cuts[0] = Cut{count, 0};
        cuts[1] = Cut{count, 0};
    }
    // pass 2: the entries whose cost interval [P_excl, P_incl) contains the two targets
    long long carry = 0;
    for (int base = 0; base < count; base += WG_THREADS) {
        const int e = base + threadIdx.x;
        long long unit = 0, c = 0;
        if (e < count) {
            unit = entry_unit_cost(table[e], bits_dev[e]);
            c = unit * ((table[e].N + 15) >> 4);
        }
        long long chunk;
        const long long incl = block_scan(c, tmp, chunk) + carry; // barriers inside order the cuts[] init
        const long long excl = incl - c;
        if (c > 0) {
            if (t_lo >= excl && t_lo < incl)
                cuts[0] = Cut{e, (int)((t_lo - excl) / unit)};
            if (t_hi >= excl && t_hi < incl)
                cuts[1] = Cut{e, (int)((t_hi - excl) / unit)};
        }
        carry += chunk;
    }
    __syncthreads();
    lo = cuts[0];
    hi = cuts[1]; // t_hi == C for the last workgroup: no interval contains it, stays {count, 0}
    if (C == 0)
        lo = Cut{count, 0};
}

template <bool SINGLE>
__global__ __launch_bounds__(WG_THREADS) void decode_m1_kernel(const FqLinearDesc single,
                                                               int bits_host,
                                                               const FqLinearDesc *__restrict__ table,
                                                               const int32_t *__restrict__ bits_dev,
                                                               int count, int total_tiles,
                                                               int tile_rows, int *flags, int cus)
{
    extern __shared__ uint4 lds[];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6); // scalar: keeps row math on the SALU
    if (SINGLE) {
        // one linear: equal row tiles dealt round-robin
        const int wave_rows = tile_rows / WAVES; // multiple of 4
        bool first = true;
        for (int tile = blockIdx.x; tile < total_tiles; tile += gridDim.x) {
            const int row_begin = min(tile * tile_rows + wave * wave_rows, single.N);
            const int row_end = min(row_begin + wave_rows, single.N);
            if (bits_host == 2) {
                const Sel d = {single.codes2, single.scales2, single.zeros2, single.N, single.K};
                run_tile<2>(d, single.x, single.y, row_begin, row_end, first, lds);
            } else if (bits_host == 3) {
                const Sel d = {single.codes3, single.scales3, single.zeros3, single.N, single.K};
                run_tile<3>(d, single.x, single.y, row_begin, row_end, first, lds);
            } else if (bits_host == 4) {
                const Sel d = {single.codes4, single.scales4, single.zeros4, single.N, single.K};
                run_tile<4>(d, single.x, single.y, row_begin, row_end, first, lds);
            } else if (bits_host == 8) {
                const Sel d = {single.codes8, single.scales8, single.zeros8, single.N, single.K};
                run_tile<8>(d, single.x, single.y, row_begin, row_end, first, lds);
            } else {
                const Sel d = {(const uint8_t *)single.w16, nullptr, nullptr, single.N, single.K};
                run_tile<16>(d, single.x, single.y, row_begin, row_end, first, lds);
            }
            first = false;
        }
        return;
    }
    Cut lo, hi;
    partition(table, bits_dev, count, lo, hi, flags, cus);
    for (int e = lo.e; e < count && e <= hi.e; e++) {
        const FqLinearDesc *dp = &table[e];
        const int bits = bits_dev[e];
        const int units = (dp->N + 15) >> 4;
        const int u0 = e == lo.e ? lo.unit : 0;
        const int u1 = e == hi.e ? hi.unit : units;
        if (u1 <= u0 || entry_unit_cost(*dp, bits) == 0)
            continue; // uniform over the workgroup: nothing of this entry falls in the slice
        // rows [16 u0, 16 u1) split over the 4 wavefronts in multiples of 4 rows
        const int r0 = u0 * 16, r1 = min(u1 * 16, dp->N);
        const int per_wave = ((r1 - r0 + WAVES * ROWS_PER_WAVE - 1) / (WAVES * ROWS_PER_WAVE)) * ROWS_PER_WAVE;
        const int row_begin = min(r0 + wave * per_wave, r1);
        const int row_end = min(row_begin + per_wave, r1);
        // the switch of precision: a pointer select on resident copies (each width names its own
        // copy inside its own branch: nothing is selected ahead of the branch)
        if (bits == 2) {
            const Sel d = {dp->codes2, dp->scales2, dp->zeros2, dp->N, dp->K};
            run_tile<2>(d, dp->x, dp->y, row_begin, row_end, true, lds);
        } else if (bits == 3) {
            const Sel d = {dp->codes3, dp->scales3, dp->zeros3, dp->N, dp->K};
            run_tile<3>(d, dp->x, dp->y, row_begin, row_end, true, lds);
        } else if (bits == 4) {
            const Sel d = {dp->codes4, dp->scales4, dp->zeros4, dp->N, dp->K};
            run_tile<4>(d, dp->x, dp->y, row_begin, row_end, true, lds);
        } else if (bits == 8) {
            const Sel d = {dp->codes8, dp->scales8, dp->zeros8, dp->N, dp->K};
            run_tile<8>(d, dp->x, dp->y, row_begin, row_end, true, lds);
        } else {
            const Sel d = {(const uint8_t *)dp->w16, nullptr, nullptr, dp->N, dp->K};
            run_tile<16>(d, dp->x, dp->y, row_begin, row_end, true, lds);
        }
    }
}

} // namespace

static size_t lds_bytes_for(int max_K)
{
    // worst case over the bit-widths: 4-bit pads K to 2048 and adds 8 bytes per 32 k, 2-bit pads
    // to 4096 and adds 8 bytes per 64 k
    const size_t kp4 = ((size_t)max_K + 2047) / 2048 * 2048, kp2 = ((size_t)max_K + 4095) / 4096 * 4096;
    const size_t b4 = kp4 * 2 + kp4 / 32 * 8, b2 = kp2 * 2 + kp2 / 64 * 8;
    return (b4 > b2 ? b4 : b2) + 64;
}

// Workgroups that can be resident at once on the current device: a persistent grid must
// not exceed it, or late workgroups would start a full pass late.
static int resident_workgroups(size_t lds)
{
    return fq_device_cus() * fq_workgroups_per_cu((const void *)decode_m1_kernel<false>, WG_THREADS, lds, 2);
}

int fq_decode_tile_rows(long long total_rows, int max_K, int M)
{
    (void)M;
    // Largest tile (fewest x stagings) that still leaves every resident workgroup
    // several tiles, so that the static round-robin stays balanced.
    const long long cap = resident_workgroups(lds_bytes_for(max_K));
    int rows = 128;
    while (rows > TILE_ROWS_MIN && total_rows / rows < 8 * cap)
        rows >>= 1;
    return rows;
}

hipError_t fq_launch_decode(const FqLinearDesc *single, int bits_host,
                            const FqLinearDesc *descs_dev, const int32_t *bits_dev, int count,
                            int total_tiles, int tile_rows, int max_K, int M, int *flags, hipStream_t stream)
{
    (void)M;
    if (total_tiles <= 0)
        return hipSuccess;
    const size_t lds = lds_bytes_for(max_K);
    if (lds > 48 * 1024) { // above the default limit of dynamic LDS: raised once per device
        const size_t most = lds_bytes_for(FQ_MAX_DECODE_K);
        hipError_t e = fq_raise_dynamic_lds((const void *)decode_m1_kernel<true>, most);
        if (e == hipSuccess)
            e = fq_raise_dynamic_lds((const void *)decode_m1_kernel<false>, most);
        if (e != hipSuccess)
            return e;
    }
    const int cap = resident_workgroups(lds);
    // A plan cuts its total cost into one equal slice per workgroup that takes part: two to four
    // per compute unit, which the kernel decides from the launch's bit-widths (a third register
    // set, i.e. twelve loads per lane in flight, made the mixed 7B step slower: 0.780 ms).
    const int cus = fq_device_cus();
    const int plan_grid = cap < 4 * cus ? cap : 4 * cus;
    const int grid = single ? (total_tiles < cap ? total_tiles : cap) : plan_grid;
    if (single) {
        decode_m1_kernel<true><<<grid, WG_THREADS, lds, stream>>>(*single, bits_host, nullptr,
                                                                  nullptr, 1, total_tiles, tile_rows, nullptr, cus);
    } else {
        FqLinearDesc none = {};
        decode_m1_kernel<false><<<grid, WG_THREADS, lds, stream>>>(none, 0, descs_dev, bits_dev,
                                                                   count, total_tiles, tile_rows, flags, cus);
    }
    return hipGetLastError();
}

