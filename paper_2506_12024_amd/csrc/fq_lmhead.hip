// Output layer fused with what Alg. 1 takes from its logits in every decode step: the next
// token (argmax) and the entropy behind PPLE (Sec. 4.2 Eq. 5, softmax as in Sec. 2.3).
// logits[m][v] = sum_k x[m][k] * W[v][k] for the fp16 output-layer weight W[V][K] and 1 <= M <= 4
// rows of x, accumulated in binary32; the logits never have to travel through HBM (they are
// written only if the caller asks for them).  HBM bound: the weight is read once, 2 bytes per
// entry.
//
// A wavefront takes four vocabulary rows at a time; lane l reads 16 bytes (8 halves) of each at
// k = 512 j + 8 l, j = 0 .. K / 512 - 1 -- one non-temporal 128-bit load per row and j, a
// wavefront load is 1 KiB contiguous -- with the loads of step j + 1 in flight while step j is
// multiplied (v_dot2_f32_f16) against the matching x blocks, which sit in LDS for the whole
// kernel ([j][m][lane], conflict free).  The four sums are reduced across the wavefront and
// handed to lanes 0 .. 3, each of which keeps an online softmax state per row of x: running
// maximum and its index, S = sum exp(a - max), U = sum (a - max) exp(a - max).  States meet per
// wavefront, per workgroup (LDS) and per call: every workgroup leaves its partial in a static
// device array and a second, one-workgroup launch combines them, H = ln S - U / S.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "fq_internal.h"

namespace {

#define FQ_GLOBAL __attribute__((address_space(1)))

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int THREADS = 256;
constexpr int WAVES = THREADS / 64;
constexpr int RPW = 4;                 // vocabulary rows per wavefront and iteration
constexpr int ROWS_PER_WG = WAVES * RPW;
constexpr int MAX_M = 4;
constexpr int MAX_WGS = 1024; // also the size of the combining workgroup: one partial per thread

// Partials [workgroup][row of x]: (max, S, U), index of the max; one bank per stream (the two
// launches of a call follow one another on their stream; calls on different streams use different
// banks).
__device__ float g_part[FQ_BANKS][MAX_WGS][MAX_M][3];
__device__ int g_part_idx[FQ_BANKS][MAX_WGS][MAX_M];

__device__ __forceinline__ float dot8(const u32x4 w, const u32x4 x, float acc)
{
    // whole-vector casts: a bit cast of a single element of an ext_vector loses the other elements
    const half8_t wh = __builtin_bit_cast(half8_t, w), xh = __builtin_bit_cast(half8_t, x);
    acc = __builtin_amdgcn_fdot2(__builtin_shufflevector(wh, wh, 0, 1), __builtin_shufflevector(xh, xh, 0, 1), acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_shufflevector(wh, wh, 2, 3), __builtin_shufflevector(xh, xh, 2, 3), acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_shufflevector(wh, wh, 4, 5), __builtin_shufflevector(xh, xh, 4, 5), acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_shufflevector(wh, wh, 6, 7), __builtin_shufflevector(xh, xh, 6, 7), acc, false);
    return acc;
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1)
        v += __shfl_xor(v, off, 64);
    return v;
}

// Online softmax state of one row of x.
struct State {
    float mx, S, U;
    int idx;
    __device__ __forceinline__ void init()
    {
        mx = -INFINITY;
        S = 0.f;
        U = 0.f;
        idx = 0x7fffffff;
    }
    __device__ __forceinline__ void add(float a, int v)
    {
        if (a > mx) { // a new maximum: rebase what was summed so far (first element: S = U = 0)
            const float d = mx - a, f = mx == -INFINITY ? 0.f : __expf(d);
            U = mx == -INFINITY ? 0.f : f * (U + d * S);
            S = f * S + 1.f;
            mx = a;
            idx = v;
        } else {
            const float d = a - mx, e = __expf(d);
            S += e;
            U += d * e;
        }
    }
    // Another state's elements join this one's; (larger maximum, then smaller index) decides the
    // maximum.  An empty state has S = 0.
    __device__ __forceinline__ void merge(float omx, float oS, float oU, int oidx)
    {
        if (oS <= 0.f)
            return;
        if (S <= 0.f) {
            mx = omx, S = oS, U = oU, idx = oidx;
            return;
        }
        if (omx > mx || (omx == mx && oidx < idx)) {
            const float d = mx - omx, f = __expf(d);
            U = f * (U + d * S) + oU;
            S = f * S + oS;
            mx = omx;
            idx = oidx;
        } else {
            const float d = omx - mx, f = __expf(d);
            S += f * oS;
            U += f * (oU + d * oS);
        }
    }
    // Butterfly over the lanes whose index differs in the bits of `mask`.
    __device__ __forceinline__ void merge_lanes(int mask)
    {
        for (int off = 1; off <= mask; off <<= 1) {
            if (!(mask & off))
                continue;
            const float omx = __shfl_xor(mx, off, 64), oS = __shfl_xor(S, off, 64), oU = __shfl_xor(U, off, 64);
            const int oidx = __shfl_xor(idx, off, 64);
            merge(omx, oS, oU, oidx);
        }
    }
};

template <int M>
__global__ __launch_bounds__(THREADS) void lm_head_entropy_kernel(const uint16_t *__restrict__ x,
                                                                  const uint16_t *__restrict__ w, int V, int K,
                                                                  int bank, float *__restrict__ logits)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[]; // x: [K / 512][M][64] blocks of 16 bytes
    __shared__ float s_part[WAVES][M][3];
    __shared__ int s_idx[WAVES][M];
    u32x4 *xs = reinterpret_cast<u32x4 *>(lds_raw);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int J = K >> 9;

    for (int i = threadIdx.x; i < J * M * 64; i += THREADS) {
        const int l = i & 63, m = (i >> 6) % M, j = (i >> 6) / M;
        xs[i] = *(const FQ_GLOBAL u32x4 *)(x + (size_t)m * K + (size_t)j * 512 + l * 8);
    }
    __syncthreads();

    State st[M];
#pragma unroll
    for (int m = 0; m < M; m++)
        st[m].init();

    const int nblocks = (V + ROWS_PER_WG - 1) / ROWS_PER_WG;
    for (int rb = blockIdx.x; rb < nblocks; rb += gridDim.x) {
        const int row0 = rb * ROWS_PER_WG + wave * RPW;
        const FQ_GLOBAL u32x4 *wp[RPW];
#pragma unroll
        for (int r = 0; r < RPW; r++) // rows past V repeat row V - 1 and are dropped below
            wp[r] = (const FQ_GLOBAL u32x4 *)(w + (size_t)min(row0 + r, V - 1) * K) + lane;
        float acc[RPW][M];
#pragma unroll
        for (int r = 0; r < RPW; r++)
#pragma unroll
            for (int m = 0; m < M; m++)
                acc[r][m] = 0.f;
        u32x4 cur[RPW], nxt[RPW];
#pragma unroll
        for (int r = 0; r < RPW; r++)
            cur[r] = __builtin_nontemporal_load(wp[r]);
        for (int j = 0; j < J; j++) {
            const int jn = min(j + 1, J - 1); // the last step re-reads itself: the wait stays counted
#pragma unroll
            for (int r = 0; r < RPW; r++)
                nxt[r] = __builtin_nontemporal_load(wp[r] + jn * 64);
#pragma unroll
            for (int m = 0; m < M; m++) {
                const u32x4 xv = xs[(j * M + m) * 64 + lane];
#pragma unroll
                for (int r = 0; r < RPW; r++)
                    acc[r][m] = dot8(cur[r], xv, acc[r][m]);
            }
#pragma unroll
            for (int r = 0; r < RPW; r++)
                cur[r] = nxt[r];
        }
#pragma unroll
        for (int m = 0; m < M; m++) {
            float mine = 0.f;
#pragma unroll
            for (int r = 0; r < RPW; r++) {
                const float s = wave_sum(acc[r][m]);
                if (lane == r)
                    mine = s;
            }
            const int v = row0 + lane;
            if (lane < RPW && v < V) {
                st[m].add(mine, v);
                if (logits)
                    logits[(size_t)m * V + v] = mine;
            }
        }
    }

    // lanes 0 .. RPW - 1 of every wavefront -> lane 0 -> LDS -> the first wavefront -> the
    // workgroup's partial in the static array; binary32 throughout (v_exp_f32 for the rescaling)
#pragma unroll
    for (int m = 0; m < M; m++) {
        if (lane >= RPW)
            st[m].init();
        st[m].merge_lanes(RPW - 1);
        if (lane == 0) {
            s_part[wave][m][0] = st[m].mx;
            s_part[wave][m][1] = st[m].S;
            s_part[wave][m][2] = st[m].U;
            s_idx[wave][m] = st[m].idx;
        }
    }
    __syncthreads();
    if (wave != 0)
        return;
    State wg[M];
#pragma unroll
    for (int m = 0; m < M; m++) {
        wg[m].init();
        if (lane < WAVES) {
            wg[m].mx = s_part[lane][m][0];
            wg[m].S = s_part[lane][m][1];
            wg[m].U = s_part[lane][m][2];
            wg[m].idx = s_idx[lane][m];
        }
        wg[m].merge_lanes(WAVES - 1);
        if (lane == 0) {
            g_part[bank][blockIdx.x][m][0] = wg[m].mx;
            g_part[bank][blockIdx.x][m][1] = wg[m].S;
            g_part[bank][blockIdx.x][m][2] = wg[m].U;
            g_part_idx[bank][blockIdx.x][m] = wg[m].idx;
        }
    }
}

// Second launch (one workgroup): merges the workgroups' partials.  A separate launch because the
// alternative, a ticket that lets the last workgroup do it, needs every workgroup to make its
// partial visible to the other XCDs first, and that fence writes back an L2 per workgroup
// (measured: 50 us for 1024 workgroups, more than the whole weight stream).
template <int M>
__global__ __launch_bounds__(MAX_WGS) void lm_head_combine_kernel(int parts, int bank, float *__restrict__ H,
                                                                  int32_t *__restrict__ argmax)
{
    // one partial per thread (all loads in flight at once), wavefront butterflies, LDS, once more
    __shared__ float s_part[MAX_WGS / 64][M][3];
    __shared__ int s_idx[MAX_WGS / 64][M];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    State st[M];
#pragma unroll
    for (int m = 0; m < M; m++) {
        st[m].init();
        if (t < parts) {
            st[m].mx = g_part[bank][t][m][0];
            st[m].S = g_part[bank][t][m][1];
            st[m].U = g_part[bank][t][m][2];
            st[m].idx = g_part_idx[bank][t][m];
        }
    }
#pragma unroll
    for (int m = 0; m < M; m++) {
        st[m].merge_lanes(63);
        if (lane == 0) {
            s_part[wave][m][0] = st[m].mx;
            s_part[wave][m][1] = st[m].S;
            s_part[wave][m][2] = st[m].U;
            s_idx[wave][m] = st[m].idx;
        }
    }
    __syncthreads();
    if (wave != 0)
        return;
#pragma unroll
    for (int m = 0; m < M; m++) {
        State all;
        all.init();
        if (lane < MAX_WGS / 64) {
            all.mx = s_part[lane][m][0];
            all.S = s_part[lane][m][1];
            all.U = s_part[lane][m][2];
            all.idx = s_idx[lane][m];
        }
        all.merge_lanes(MAX_WGS / 64 - 1);
        if (lane == 0) {
            H[m] = (float)(log((double)all.S) - (double)all.U / (double)all.S);
            if (argmax)
                argmax[m] = all.idx;
        }
    }
}

int device_cus() { return fq_device_cus(); }

template <int M>
hipError_t launch(const uint16_t *x, const uint16_t *w, int V, int K, float *logits, float *H, int32_t *argmax,
                  hipStream_t stream)
{
    const size_t lds = (size_t)M * K * 2;
    if (lds > 48 * 1024) {
        hipError_t e = fq_raise_dynamic_lds((const void *)lm_head_entropy_kernel<M>, 64 * 1024);
        if (e != hipSuccess)
            return e;
    }
    const int nblocks = (V + ROWS_PER_WG - 1) / ROWS_PER_WG;
    int grid = 2 * device_cus();
    if (grid > MAX_WGS)
        grid = MAX_WGS;
    if (grid > nblocks)
        grid = nblocks;
    const int bank = fq_stream_bank(stream);
    if (bank < 0) // more streams than banks of partial results have used this call on this device
        return hipErrorOutOfMemory;
    lm_head_entropy_kernel<M><<<grid, THREADS, lds, stream>>>(x, w, V, K, bank, logits);
    lm_head_combine_kernel<M><<<1, MAX_WGS, 0, stream>>>(grid, bank, H, argmax);
    return hipGetLastError();
}

} // namespace

hipError_t fq_launch_lm_head_entropy(const void *x, const void *w, int M, int V, int K, float *logits, float *H,
                                     int32_t *argmax, hipStream_t stream)
{
    const uint16_t *xp = (const uint16_t *)x, *wp = (const uint16_t *)w;
    switch (M) {
    case 1:
        return launch<1>(xp, wp, V, K, logits, H, argmax, stream);
    case 2:
        return launch<2>(xp, wp, V, K, logits, H, argmax, stream);
    case 3:
        return launch<3>(xp, wp, V, K, logits, H, argmax, stream);
    default:
        return launch<4>(xp, wp, V, K, logits, H, argmax, stream);
    }
}
