// W8A8 prefill (Sec. 4.1, 4.3, 4.5): during the prefill the resident INT8 weights meet 8-bit
// activations on the integer matrix cores.
//
// Activations.  The paper does not say how they are quantized; the reading taken is the
// symmetric form stated after Sec. 2.2 Eq. (3), per token: z = 0, Xmax = -Xmin = max |x|,
// 2^8 - 2 levels, so s_x = (2 max|x|) / 254 and q = round(x / s_x) in [-127, 127], binary32,
// one rounding per operation, IEEE division, round-half-to-even (an all-zero row: s_x = 1).
// quantize_act_kernel: one workgroup per token, two passes over the row (the second one
// finds it in L2).  It also writes the sum of the codes of every quantization group,
// xsum[g][m]: the GEMM needs it for the weights' zero points.
//
// Contraction.  With the weight codes q in [0, 255], zero points z, scales s (Eq. (2)):
//   y[m][n] = s_x[m] * sum_g s[n][g] * ( sum_{k in g} xq[m][k] (q[n][k] - 128)
//                                        - (z[n][g] - 128) * xsum[g][m] )
// -- q - 128 is a signed byte (one XOR of the stored code), which q - z is not.  The inner
// sum runs on v_mfma_i32_32x32x32_i8 (A = 32 tokens x 32 k, B = 32 k x 32 weight rows), four
// of them per group of 128; it is exact and is folded into a binary32 accumulator as
// out += s * (float)sum -- two vector instructions per output and group, which is what
// bounds the kernel.  The zero-point term, sum_g (s (128 - z))[n][g] * xsum[g][m], is a
// second, thin contraction over the groups: it runs on v_mfma_f32_32x32x2_f32 (two groups
// per instruction) into the same accumulators rather than costing a third vector
// instruction per output and group.
//
// Tiling.  A workgroup of 8 wavefronts (two per SIMD) owns 192 tokens x 256 weight rows, a
// wavefront 96 tokens x 64 rows = 3 x 2 MFMA tiles; the 96 binary32 accumulators are
// updated by vector instructions, so they sit in architectural registers (4 x 2 tiles would
// need 128 and no longer fit beside the operands without spilling).  A second instance with
// 128 tokens (2 x 2 tiles per wavefront) serves the launches whose tile count fits the chip
// better that way.  One step = one
// quantization group: both operand slabs of a step (192 and 256 rows x 128 bytes) are fetched
// straight into LDS by global_load_lds_dwordx4 -- no staging registers, nothing for the
// register allocator to juggle -- double buffered, one wait and one barrier per step.
// int8 doubles the MFMA rate and halves the bytes per operand element against the fp16
// kernel, so the tile has to be this large to keep the L2 traffic per MFMA down.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "fq_internal.h"

namespace {

#define FQ_GLOBAL __attribute__((address_space(1)))

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------------ activation quantizer

constexpr int QA_THREADS = 256;

__device__ __forceinline__ float wave_max_f(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1)
        v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

__global__ __launch_bounds__(QA_THREADS) void quantize_act_kernel(const half8 *__restrict__ x, int M, int K,
                                                                  int8_t *__restrict__ xq,
                                                                  float *__restrict__ sx,
                                                                  int32_t *__restrict__ xsum)
{
#pragma clang fp contract(off)
    __shared__ float s_max[QA_THREADS / 64];
    const int m = blockIdx.x, t = threadIdx.x;
    const int nvec = K >> 3; // 8 halves per vector; K is a multiple of 128, so nvec of 16
    const half8 *row = x + (size_t)m * nvec;

    float amax = 0.0f;
    for (int i = t; i < nvec; i += QA_THREADS) {
        const half8 v = row[i];
#pragma unroll
        for (int j = 0; j < 8; j++)
            amax = fmaxf(amax, fabsf((float)v[j]));
    }
    amax = wave_max_f(amax);
    if ((t & 63) == 0)
        s_max[t >> 6] = amax;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < QA_THREADS / 64; w++)
        amax = fmaxf(amax, s_max[w]);

    const float s = amax > 0.0f ? __fdiv_rn(__fadd_rn(amax, amax), 254.0f) : 1.0f;
    if (t == 0)
        sx[m] = s;

    // nvec is a multiple of 16 and QA_THREADS too: the 16 lanes of a segment enter and leave
    // the loop together, and they hold one quantization group (16 x 8 = 128 k)
    for (int i = t; i < nvec; i += QA_THREADS) {
        const half8 v = row[i];
        int q[8], sum = 0;
#pragma unroll
        for (int j = 0; j < 8; j++) {
            float r = rintf(__fdiv_rn((float)v[j], s));
            r = fminf(fmaxf(r, -127.0f), 127.0f);
            q[j] = (int)r;
            sum += q[j];
        }
        uint2 word;
        word.x = (q[0] & 255) | ((q[1] & 255) << 8) | ((q[2] & 255) << 16) | ((uint32_t)(q[3] & 255) << 24);
        word.y = (q[4] & 255) | ((q[5] & 255) << 8) | ((q[6] & 255) << 16) | ((uint32_t)(q[7] & 255) << 24);
        reinterpret_cast<uint2 *>(xq + (size_t)m * K)[i] = word;
#pragma unroll
        for (int off = 8; off >= 1; off >>= 1)
            sum += __shfl_xor(sum, off, 64);
        if ((t & 15) == 0)
            xsum[(size_t)(i >> 4) * M + m] = sum;
    }
}

// ------------------------------------------------------------------ int8 GEMM

constexpr int THREADS = 512;
constexpr int WAVES = THREADS / 64;
constexpr int MT_MAX = 3;        // MFMA tiles along the tokens, per wavefront (96 tokens; the kernel also
                                 // exists with 2: the launcher takes the one with fewer, cheaper rounds)
constexpr int BN = 256;
constexpr int BKB = 128;         // k (= bytes of a row) per step: one quantization group
constexpr int WN = 64;           // weight rows per wavefront (2 MFMA tiles)
constexpr int WSLAB = BN * BKB;  // bytes of the weight slab

struct W8A8Args {
    const uint8_t *codes;
    const float *scales;
    const uint8_t *zeros;
    const int8_t *xq;
    const float *sx;
    const int32_t *xsum;
    uint16_t *y;
    int M, N, K;
};

// Slab layout in LDS: row r (128 bytes) holds its eight 16-byte pieces at slot
// p ^ ((r >> 1) & 7).  A 128-bit operand read of 16 consecutive rows at one piece then
// touches every bank once, and no padding is needed (the direct-to-LDS loads write 64
// consecutive 16-byte chunks per instruction, lane l at chunk l: the permutation is applied
// on the global side, where each lane is free to fetch any piece).
__device__ __forceinline__ int slab_offset(int r, int p)
{
    return r * BKB + ((p ^ ((r >> 1) & 7)) << 4);
}

// Which 16-byte chunks a thread fetches of an operand slab (256 rows x 128 bytes of a
// [rows][K] byte matrix): load i of wavefront w covers chunks (i * 8 + w) * 64 .. + 63, i.e.
// rows (i * 8 + w) * 8 .. + 7; the lane takes slot (lane & 7) of row r0 + 64 i, which holds
// piece p = slot ^ ((r >> 1) & 7) -- the same p for every i.
struct DmaLane {
    int r0;  // row of load 0
    int p16; // byte offset of the piece inside the row
};

__device__ __forceinline__ DmaLane dma_lane()
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    DmaLane L;
    L.r0 = wave * 8 + (lane >> 3);
    L.p16 = ((lane & 7) ^ ((L.r0 >> 1) & 7)) << 4;
    return L;
}

// Fetch one step of one operand straight into LDS: `tile` points at (first row of the tile,
// first k of the step) and is the same for the whole workgroup; rows past `last_row` (relative
// to the tile) are clamped to it.  Every thread issues ROWS / 64 loads of 16 bytes.
template <int ROWS>
__device__ __forceinline__ void dma_slab(const uint8_t *tile, const DmaLane &L, int last_row, int K,
                                         uint8_t *slab)
{
    const int wave = threadIdx.x >> 6;
#pragma unroll
    for (int i = 0; i < ROWS * 8 / THREADS; i++) {
        // 32-bit offset from a scalar base: the load then takes the scalar-base form instead of
        // needing a 64-bit address pair per chunk
        const uint32_t off = (uint32_t)min(L.r0 + i * (WAVES * 8), last_row) * (uint32_t)K + L.p16;
        __builtin_amdgcn_global_load_lds((const FQ_GLOBAL void *)(tile + off),
                                         (__attribute__((address_space(3))) void *)(slab + (i * WAVES + wave) * 1024),
                                         16, 0, 0);
    }
}

// Scales and zero points reach the wavefronts through LDS, eight groups (steps) at a time: a lane
// needs those of its two weight rows for every step, and fetched per step and lane that is four
// loads of 64 different cache lines each per wavefront -- four times the requests of the operand
// slabs themselves (measured: a fifth of the kernel's time).  Block b (groups 8 b .. 8 b + 7) of
// the tile's 256 rows is 2 x 2048 words; it is requested with direct-to-LDS loads (a dword resp. a
// byte per lane, either landing in the lane's word, the byte zero-extended) during the first step
// of block b - 1, 64 instructions dealt over the eight wavefronts: instruction q fetches, for
// rows (q & 3) * 64 + lane, group (q >> 2) & 7 of the block, scales for q < 32 and zero points
// from there on.
constexpr int MB = 8; // groups per block of metadata

__device__ __forceinline__ void dma_meta(const float *scales_tile, const uint8_t *zeros_tile, uint32_t G, int w_last,
                                         int block, float *sm, uint32_t *zm)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
    for (int j = 0; j < 8; j++) {
        const int q = wave * 8 + j;
        const int rb = q & 3, gi = (q >> 2) & 7;
        const uint32_t g = min((uint32_t)(block * MB + gi), G - 1); // (past the last group: fetched again, never read)
        const uint32_t idx = (uint32_t)min(rb * 64 + lane, w_last) * G + g;
        if (q < 32)
            __builtin_amdgcn_global_load_lds((const FQ_GLOBAL void *)(scales_tile + idx),
                                             (__attribute__((address_space(3))) void *)(sm + gi * BN + rb * 64), 4, 0, 0);
        else
            __builtin_amdgcn_global_load_lds((const FQ_GLOBAL void *)(zeros_tile + idx),
                                             (__attribute__((address_space(3))) void *)(zm + gi * BN + rb * 64), 1, 0, 0);
    }
}

template <int V>
struct IntC {
    static constexpr int value = V;
};

template <int MT>
__global__ __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void w8a8_kernel(
    const W8A8Args d, int m_tiles, int n_tiles, int per_xcd)
{
    static_assert(MT >= 2 && MT <= MT_MAX, "two or three token tiles per wavefront");
    constexpr int BM = 2 * MT * 32;  // tokens per workgroup
    constexpr int XSLAB = BM * BKB;  // bytes of the x slab of a step (BM rows x 128 bytes)
    // Four separate arrays, selected at compile time: the compiler can then tell that the
    // operand reads of a step do not touch the slabs its direct-to-LDS loads are filling, and
    // does not wait for those loads before the first read.
    __shared__ __attribute__((aligned(1024))) uint8_t xs0[XSLAB], xs1[XSLAB], ws0[WSLAB], ws1[WSLAB];
    __shared__ float xsm[2][BM];
    __shared__ __attribute__((aligned(1024))) float sm[2][MB * BN];   // scales of two blocks of groups: [group][row]
    __shared__ __attribute__((aligned(1024))) uint32_t zm[2][MB * BN]; // zero points, same order

    // consecutive workgroup ids go round-robin to the 8 XCDs: give each XCD a contiguous run
    // of logical tiles (the M tiles of one N tile are neighbours and share the weight slab)
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= m_tiles * n_tiles)
        return;
    const int m0 = (logical % m_tiles) * BM, n0 = (logical / m_tiles) * BN;

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int l32 = lane & 31, c = lane >> 5;
    const int wm = (wave & 1) * (MT * 32); // first token of this wavefront inside the tile
    const int wn = (wave >> 1) * WN;   // first weight row
    const int n_wave0 = n0 + wn;

    v16f out[MT][2];
#pragma unroll
    for (int mt = 0; mt < MT; mt++)
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
            for (int v = 0; v < 16; v++)
                out[mt][j][v] = 0.f;

    // Operand reads: lane (l32, c) reads piece 2 i + c of row l32 of an MFMA tile; the slot of
    // a piece depends on the row only through (l32 >> 1) & 7, so four byte offsets serve every
    // tile of both operands (tiles start at multiples of 32 rows).
    int lofs[4];
#pragma unroll
    for (int i = 0; i < 4; i++)
        lofs[i] = slab_offset(l32, 2 * i + c);

    const int nsteps = d.K / BKB;
    const DmaLane dl = dma_lane();
    const int x_last = d.M - 1 - m0, w_last = d.N - 1 - n0;
    const uint8_t *x_tile = (const uint8_t *)d.xq + (size_t)m0 * d.K;
    const uint8_t *w_tile = d.codes + (size_t)n0 * d.K;
    const uint32_t G = (uint32_t)d.K >> 7;
    const uint32_t tok = (uint32_t)min((int)min(threadIdx.x, (unsigned)BM - 1), d.M - 1 - m0); // the thread's token (group sums)
    const float *scales_tile = d.scales + (size_t)n0 * G;
    const uint8_t *zeros_tile = d.zeros + (size_t)n0 * G;
    const int32_t *xsum_tile = d.xsum + m0;
    dma_slab<BM>(x_tile, dl, x_last, d.K, xs0);
    dma_slab<BN>(w_tile, dl, w_last, d.K, ws0);
    dma_meta(scales_tile, zeros_tile, G, w_last, 0, sm[0], zm[0]);
    int sum_next = ((const FQ_GLOBAL int32_t *)xsum_tile)[tok];
    if (threadIdx.x < BM)
        xsm[0][threadIdx.x] = (float)sum_next; // |sum| <= 128 * 127: exact
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    // Zero-point term of a pair of steps (groups g, g + 1), one v_mfma_f32_32x32x2_f32 per
    // tile: A = the tokens' group sums (lane: token l32, k = c), B = s * (128 - z) of the
    // lane's weight row (k = c), accumulated straight into `out`.  Lanes with c = 0 use the
    // first step's values, carried in az_first / bz_first (the first step's LDS copy of the
    // group sums is being overwritten with the next step's by the time the second step runs).
    float az_first[MT], bz_first[2] = {0.f, 0.f};
#pragma unroll
    for (int mt = 0; mt < MT; mt++)
        az_first[mt] = 0.f;

    // One step (one group): the slabs of step s+1 are requested first and land in the other
    // buffer while the MFMAs of step s run; one wait and one barrier per step.
    // PHASE 0: first step of a pair; PHASE 1: second step (adds the pair's zero-point term);
    // PHASE 2: a last unpaired step (adds its own).
    auto step = [&](int s, auto phase) {
        constexpr int PHASE = decltype(phase)::value;
        constexpr bool ODD = PHASE == 1; // steps alternate between the two buffer sets (s & 1)
        // scale and zero point of the lane's two weight rows for this step: read ahead of the step's
        // requests (the compiler cannot tell these words from the ones the direct-to-LDS loads below
        // write and would wait for every outstanding load first)
        float cur_s[2];
        uint32_t cur_z[2];
#pragma unroll
        for (int j = 0; j < 2; j++) {
            cur_s[j] = sm[(s >> 3) & 1][(s & (MB - 1)) * BN + wn + j * 32 + l32];
            cur_z[j] = zm[(s >> 3) & 1][(s & (MB - 1)) * BN + wn + j * 32 + l32];
        }
        const int sn = min(s + 1, nsteps - 1); // always issued: the last step refetches itself
        dma_slab<BM>(x_tile + sn * BKB, dl, x_last, d.K, ODD ? xs0 : xs1); // last read in step s-1: a barrier has passed
        dma_slab<BN>(w_tile + sn * BKB, dl, w_last, d.K, ODD ? ws0 : ws1);
        if ((s & (MB - 1)) == 0) // the next block of scales and zero points; its buffer was last read a block ago
            dma_meta(scales_tile, zeros_tile, G, w_last, (s >> 3) + 1, sm[((s >> 3) + 1) & 1], zm[((s >> 3) + 1) & 1]);
        sum_next = ((const FQ_GLOBAL int32_t *)(xsum_tile + (size_t)sn * (size_t)d.M))[tok];
        const uint8_t *xc = (ODD ? xs1 : xs0) + wm * BKB, *wc = (ODD ? ws1 : ws0) + wn * BKB;

        // all eight reads are requested before the first is waited for (left alone the scheduler waits
        // for each in turn, eight LDS round trips at the head of the step)
        v4i b[2][4];
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
            for (int i = 0; i < 4; i++)
                b[j][i] = *reinterpret_cast<const v4i *>(wc + j * 32 * BKB + lofs[i]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
            for (int i = 0; i < 4; i++) // stored code q -> signed byte q - 128
                b[j][i] = b[j][i] ^ (int)0x80808080;
        float az[MT], bz[2];
#pragma unroll
        for (int j = 0; j < 2; j++)
            bz[j] = cur_s[j] * (float)(128 - (int)cur_z[j]);
        // group sums of this step for the wavefront's tokens: only xsm[s & 1] is read during
        // step s (the other buffer receives step s + 1's values at the end of the step)
        const float *sc = xsm[s & 1] + wm;
#pragma unroll
        for (int mt = 0; mt < MT; mt++)
            az[mt] = sc[mt * 32 + l32];
        if (PHASE == 0) {
#pragma unroll
            for (int mt = 0; mt < MT; mt++)
                az_first[mt] = az[mt];
            bz_first[0] = bz[0];
            bz_first[1] = bz[1];
        } else if (PHASE == 1) { // k = 1 lanes: this step; k = 0 lanes: the first step of the pair
#pragma unroll
            for (int mt = 0; mt < MT; mt++)
                az[mt] = c ? az[mt] : az_first[mt];
            bz[0] = c ? bz[0] : bz_first[0];
            bz[1] = c ? bz[1] : bz_first[1];
        } else { // a last unpaired step: nothing on k = 1
#pragma unroll
            for (int mt = 0; mt < MT; mt++)
                az[mt] = c ? 0.f : az[mt];
        }

        // Tiles t = 2 mt + j.  A wavefront issues in order, and each MFMA of a tile's chain
        // depends on the one before: a chain followed by its fold would leave the vector pipe
        // idle during the chain and the matrix pipe idle during the fold.  So the chain of tile
        // t+1 is interleaved with the fold of tile t, one MFMA (32 cycles in the matrix pipe) per
        // eight vector instructions (32 cycles of issue).
        v4i a[4];
        v16i acc[2];
        auto read_a = [&](int mt) {
#pragma unroll
            for (int i = 0; i < 4; i++)
                a[i] = *reinterpret_cast<const v4i *>(xc + mt * 32 * BKB + lofs[i]);
        };
        auto chain = [&](int j) {
            v16i r = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int i = 0; i < 4; i++)
                r = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j][i], r, 0, 0, 0);
            return r;
        };
        read_a(0);
        acc[0] = chain(0);
#pragma unroll
        for (int t = 0; t < 2 * MT; t++) {
            const int mt = t >> 1, j = t & 1;
            if (t + 1 < 2 * MT)
                acc[(t + 1) & 1] = chain((t + 1) & 1);
#pragma unroll
            for (int v = 0; v < 16; v++)
                out[mt][j][v] += cur_s[j] * (float)acc[t & 1][v];
            if (t + 1 < 2 * MT) {
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0); // one MFMA
                    __builtin_amdgcn_sched_group_barrier(0x002, 8, 0); // eight vector instructions
                }
            }
            if (j == 0 && mt + 1 < MT)
                read_a(mt + 1); // both chains of mt are issued: fetch the next tokens' operands
            if (PHASE != 0)
                out[mt][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(az[mt], bz[j], out[mt][j], 0, 0, 0);
            // Pin the order across tiles: tile t is folded before the chain of tile t+2 (which
            // reads a[0]) is issued.  Left alone the compiler issues all eight chains first and
            // needs 96 more registers for their results.
            asm volatile("" : "+v"(out[mt][j]), "+v"(a[0]));
        }
        if (threadIdx.x < BM)
            xsm[(s + 1) & 1][threadIdx.x] = (float)sum_next;
        __builtin_amdgcn_s_waitcnt(0); // this wavefront's direct-to-LDS loads have landed
        __syncthreads();               // everyone's have; buffers of step s are free
    };
    int s = 0;
    for (; s + 1 < nsteps; s += 2) {
        step(s, IntC<0>());
        step(s + 1, IntC<1>());
    }
    if (s < nsteps)
        step(s, IntC<2>());

    // D layout of the 32x32 MFMA: lane holds column l32 (weight row), rows (tokens)
    // 8 * (v / 4) + 4 * (lane / 32) + v % 4.
#pragma unroll
    for (int mt = 0; mt < MT; mt++) {
#pragma unroll
        for (int v = 0; v < 16; v++) {
            const int m = m0 + wm + mt * 32 + 8 * (v >> 2) + 4 * c + (v & 3);
            if (m < d.M) {
                const float sxm = d.sx[m];
#pragma unroll
                for (int j = 0; j < 2; j++) {
                    const int n = n_wave0 + j * 32 + l32;
                    if (n < d.N)
                        ((FQ_GLOBAL uint16_t *)d.y)[(size_t)m * d.N + n] =
                            __builtin_bit_cast(uint16_t, (_Float16)(sxm * out[mt][j][v]));
                }
            }
        }
    }
}

// ---- one scale per weight row ------------------------------------------------------------------
// With a scale and a zero point per weight ROW (group = K) nothing has to be folded per group:
//   y[m][n] = s_x[m] * s[n] * ( sum_k xq[m][k] (q[n][k] - 128)  -  (z[n] - 128) * sum_k xq[m][k] ),
// the first sum exact in int32 over the whole of K (|.| <= K * 127 * 128 < 2^31 for K <= 65536), the
// second from the activations' group sums.  Same tiles, slabs and fetch as above; the six MFMA tiles of a
// wavefront are six independent int32 chains that run through all the steps, so that consecutive MFMAs
// never wait for each other, and the vector ALUs are left with the XOR of the weight bytes.
// RMT MFMA tiles along the tokens per wavefront: 4 (256 tokens per workgroup) -- the int32 accumulators
// are touched by MFMAs only, so 128 of them fit beside the operands.
// HALF: the workgroup takes half a tile, 128 tokens x 256 rows (RMT = 2): the tiles left over for a last
// round that would fill at most half of the compute units run this way, in a second launch (`skip`: the
// tiles of an XCD's run that the first launch has taken).
constexpr int RBM_FULL = 256;
template <bool HALF>
__global__ __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void w8a8_row_kernel(
    const W8A8Args d, int m_tiles, int n_tiles, int per_xcd, int skip)
{
    constexpr int RMT = HALF ? 2 : 4;
    constexpr int RBM = 2 * RMT * 32;
    constexpr int RXSLAB = RBM * BKB;
    static_assert(RBM == (HALF ? RBM_FULL / 2 : RBM_FULL), "two half tiles to a tile");
    __shared__ __attribute__((aligned(1024))) uint8_t xs0[RXSLAB], xs1[RXSLAB], ws0[WSLAB], ws1[WSLAB];
    __shared__ int xtot[RBM];

    const int in_run = skip + (HALF ? (int)(blockIdx.x >> 4) : (int)(blockIdx.x >> 3));
    const int logical = (blockIdx.x & 7) * per_xcd + in_run;
    if (in_run >= per_xcd || logical >= m_tiles * n_tiles)
        return;
    const int m0 = (logical % m_tiles) * RBM_FULL + (HALF ? (int)((blockIdx.x >> 3) & 1) * RBM : 0);
    const int n0 = (logical / m_tiles) * BN;
    if (m0 >= d.M)
        return; // the second half of a last, partly filled tile

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int l32 = lane & 31, c = lane >> 5;
    const int wm = (wave & 1) * (RMT * 32);
    const int wn = (wave >> 1) * WN;
    const int n_wave0 = n0 + wn;

    v16i acc[RMT][2];
#pragma unroll
    for (int mt = 0; mt < RMT; mt++)
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
            for (int v = 0; v < 16; v++)
                acc[mt][j][v] = 0;

    int lofs[4];
#pragma unroll
    for (int i = 0; i < 4; i++)
        lofs[i] = slab_offset(l32, 2 * i + c);

    const int nsteps = d.K / BKB;
    const DmaLane dl = dma_lane();
    const int x_last = d.M - 1 - m0, w_last = d.N - 1 - n0;
    const uint8_t *x_tile = (const uint8_t *)d.xq + (size_t)m0 * d.K;
    const uint8_t *w_tile = d.codes + (size_t)n0 * d.K;
    dma_slab<RBM>(x_tile, dl, x_last, d.K, xs0);
    dma_slab<BN>(w_tile, dl, w_last, d.K, ws0);
    // the tokens' sums over the whole row: the sum of their group sums
    if (threadIdx.x < RBM) {
        const int tok = min((int)threadIdx.x, d.M - 1 - m0);
        int t = 0;
        for (int g = 0; g < nsteps; g++)
            t += ((const FQ_GLOBAL int32_t *)(d.xsum + m0 + (size_t)g * (size_t)d.M))[tok];
        xtot[threadIdx.x] = t;
    }
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    auto step = [&](int s, auto odd) {
        constexpr bool ODD = decltype(odd)::value;
        const int sn = min(s + 1, nsteps - 1); // always issued: the last step refetches itself
        dma_slab<RBM>(x_tile + sn * BKB, dl, x_last, d.K, ODD ? xs0 : xs1); // last read in step s-1: a barrier has passed
        dma_slab<BN>(w_tile + sn * BKB, dl, w_last, d.K, ODD ? ws0 : ws1);
        // The requests stay here, ahead of the step's arithmetic: left to itself the scheduler sinks them to
        // the end of the step, just before the wait for them (1.49 instead of 1.74 POP/s).
        __builtin_amdgcn_sched_barrier(0);
        const uint8_t *xc = (ODD ? xs1 : xs0) + wm * BKB, *wc = (ODD ? ws1 : ws0) + wn * BKB;
        v4i b[2][4];
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
            for (int i = 0; i < 4; i++) { // stored code q -> signed byte q - 128
                const v4i raw = *reinterpret_cast<const v4i *>(wc + j * 32 * BKB + lofs[i]);
                b[j][i] = raw ^ (int)0x80808080;
            }
        v4i a[RMT][4];
#pragma unroll
        for (int mt = 0; mt < RMT; mt++)
#pragma unroll
            for (int i = 0; i < 4; i++)
                a[mt][i] = *reinterpret_cast<const v4i *>(xc + mt * 32 * BKB + lofs[i]);
        // six MFMAs in a row that do not depend on each other, four times
#pragma unroll
        for (int i = 0; i < 4; i++)
#pragma unroll
            for (int mt = 0; mt < RMT; mt++)
#pragma unroll
                for (int j = 0; j < 2; j++)
                    acc[mt][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[mt][i], b[j][i], acc[mt][j], 0, 0, 0);
        __builtin_amdgcn_s_waitcnt(0); // this wavefront's direct-to-LDS loads have landed
        __syncthreads();               // everyone's have; buffers of step s are free
    };
    int s = 0;
    for (; s + 1 < nsteps; s += 2) {
        step(s, std::false_type());
        step(s + 1, std::true_type());
    }
    if (s < nsteps)
        step(s, std::false_type());

    // D layout of the 32x32 MFMA: lane holds column l32 (weight row), rows (tokens)
    // 8 * (v / 4) + 4 * (lane / 32) + v % 4.
    float sn_[2];
    int zn[2];
#pragma unroll
    for (int j = 0; j < 2; j++) {
        const int n = min(n_wave0 + j * 32 + l32, d.N - 1);
        sn_[j] = d.scales[n];
        zn[j] = (int)d.zeros[n] - 128;
    }
#pragma unroll
    for (int mt = 0; mt < RMT; mt++) {
#pragma unroll
        for (int v = 0; v < 16; v++) {
            const int tl = wm + mt * 32 + 8 * (v >> 2) + 4 * c + (v & 3);
            const int m = m0 + tl;
            if (m < d.M) {
                const float sxm = d.sx[m];
                const int xt = xtot[tl];
#pragma unroll
                for (int j = 0; j < 2; j++) {
                    const int n = n_wave0 + j * 32 + l32;
                    if (n < d.N)
                        ((FQ_GLOBAL uint16_t *)d.y)[(size_t)m * d.N + n] = __builtin_bit_cast(
                            uint16_t, (_Float16)(sxm * (sn_[j] * (float)(acc[mt][j][v] - zn[j] * xt))));
                }
            }
        }
    }
}

} // namespace

hipError_t fq_launch_quantize_act(const void *x, int M, int K, void *xq, float *sx, int32_t *xsum,
                                  hipStream_t stream)
{
    if (M == 0)
        return hipSuccess;
    quantize_act_kernel<<<M, QA_THREADS, 0, stream>>>((const half8 *)x, M, K, (int8_t *)xq, sx, xsum);
    return hipGetLastError();
}

hipError_t fq_launch_w8a8(const FqLinearDesc &l, const void *xq, const float *sx, const int32_t *xsum,
                          int M, bool per_row, hipStream_t stream)
{
    if (M == 0)
        return hipSuccess;
    W8A8Args d;
    d.codes = l.codes8;
    d.scales = l.scales8;
    d.zeros = l.zeros8;
    d.xq = (const int8_t *)xq;
    d.sx = sx;
    d.xsum = xsum;
    d.y = l.y;
    d.M = M;
    d.N = l.N;
    d.K = l.K;
    const int cus = fq_device_cus();
    const int n_tiles = (l.N + BN - 1) / BN;
    // Groups of 128: 192 or 128 tokens per workgroup.  The larger tile unpacks a weight operand for three
    // MFMAs instead of two (2048 x 28672, five rounds of the one against seven of the other: 1142 against
    // 1077 TOP/s), so the smaller one is taken only where its rounds (one workgroup per compute unit at a
    // time) cost at least an eighth less in all -- 2048 x 8192: 352 tiles of 192 are two rounds, 512
    // tiles of 128 two rounds of two thirds the work (982 -> 1133 TOP/s).
    int mt = MT_MAX;
    if (!per_row) {
        const long long t3 = (long long)((M + 191) / 192) * n_tiles, t2 = (long long)((M + 127) / 128) * n_tiles;
        const long long c = cus > 0 ? cus : 1;
        if (((t2 + c - 1) / c) * 2 * 8 < ((t3 + c - 1) / c) * 3 * 7)
            mt = 2;
    }
    const int bm = per_row ? RBM_FULL : 2 * mt * 32;
    const int m_tiles = (M + bm - 1) / bm;
    const long long total = (long long)m_tiles * n_tiles;
    if (total > 0x3fffffffLL)
        return hipErrorInvalidValue;
    const int per_xcd = (int)((total + 7) / 8);
    if (!per_row) {
        if (mt == 2)
            w8a8_kernel<2><<<(unsigned)per_xcd * 8, THREADS, 0, stream>>>(d, m_tiles, n_tiles, per_xcd);
        else
            w8a8_kernel<3><<<(unsigned)per_xcd * 8, THREADS, 0, stream>>>(d, m_tiles, n_tiles, per_xcd);
        return hipGetLastError();
    }
    // One workgroup per compute unit at a time: an XCD works through its run of tiles in rounds of its
    // compute units.  What is left for the last round, if it would fill at most half of them, runs as
    // half tiles in a second launch (2048 x 28672: 112 tiles per XCD = 3 rounds of 32 + 16 tiles, which
    // then take half a round instead of a whole one).
    const int per_round = cus / 8 > 0 ? cus / 8 : 1;
    const int rest = per_xcd % per_round;
    const int tail = rest > 0 && 2 * rest <= per_round ? rest : 0;
    if (per_xcd - tail > 0) {
        w8a8_row_kernel<false><<<(unsigned)(per_xcd - tail) * 8, THREADS, 0, stream>>>(d, m_tiles, n_tiles, per_xcd, 0);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess)
            return e;
    }
    if (tail > 0)
        w8a8_row_kernel<true><<<(unsigned)tail * 16, THREADS, 0, stream>>>(d, m_tiles, n_tiles, per_xcd, per_xcd - tail);
    return hipGetLastError();
}
