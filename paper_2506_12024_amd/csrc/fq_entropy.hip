// Entropy of softmax(a) and KL(softmax(a) || softmax(b)) per row, one pass.
// Softmax: Sec. 2.3; the entropy is the exponent's argument of the perplexity
// entropy, Sec. 4.2 Eq. (5); the KL divergence is the layer-ranking signal of
// Sec. 3.1 / 4.3, taken between two next-token distributions.
//
// One workgroup per row -- or, for a handful of rows (the decode step has one), up to 32
// workgroups per row whose partials meet in a small static device array and are combined
// by whichever workgroup arrives last (one launch either way; a single CU would need
// ~8 us for the 64000 exponentials of one 32000-entry pair).
// Every lane keeps an online (running-max) partial
//   m  = max a_i            S  = sum e^(a_i - m)
//   U  = sum e^(a_i - m) (a_i - m)          D = sum e^(a_i - m) (a_i - b_i)
//   mb = max b_i            Sb = sum e^(b_i - mb)
// over the 128-bit vectors it streams (coalesced, four in flight), in binary32.
// Partials are then rescaled to the row maximum and summed across the
// workgroup in double, and one lane finishes in double:
//   H  = ln S - U / S
//   KL = D / S + (mb - m) + ln(Sb / S)
// so the difference of the two log-sum-exps, which is where binary32 would lose
// the small KL of two nearly equal distributions, never passes through binary32.
#include <hip/hip_runtime.h>
#include <float.h>
#include <math.h>
#include <stdint.h>

#include "fq_internal.h"

namespace {

// e^x as one v_exp_f32 of x * log2(e).  The product's rounding moves a term by at most
// |x| * 2^-24 relative; terms that carry weight have |x| < 20 or so, which leaves the sums three
// orders of magnitude inside the 1e-4 the results are held to, and the library routine's
// range handling costs more instructions per element than HBM delivers them.
#define EXPF(x) __expf(x)

typedef float f32x4 __attribute__((ext_vector_type(4)));
// Streaming load: each logit is read once, so it should not displace anything in the caches.
__device__ __forceinline__ float4 ld4_nt(const float4 *p)
{
    const f32x4 v = __builtin_nontemporal_load((const __attribute__((address_space(1))) f32x4 *)p);
    return make_float4(v.x, v.y, v.z, v.w);
}
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
// Vector i of a row: four consecutive logits widened to binary32 (binary16 widens exactly).
__device__ __forceinline__ float4 load4(const float *row, int i)
{
    return ld4_nt(reinterpret_cast<const float4 *>(row) + i);
}
__device__ __forceinline__ float4 load4(const _Float16 *row, int i)
{
    const half4_t v = __builtin_nontemporal_load((const __attribute__((address_space(1))) half4_t *)row + i);
    return make_float4((float)v.x, (float)v.y, (float)v.z, (float)v.w);
}

struct Partial {
    float m, S, U, D, mb, Sb;
};

__device__ __forceinline__ void part_init(Partial &p)
{
    p.m = -FLT_MAX;
    p.mb = -FLT_MAX;
    p.S = p.U = p.D = p.Sb = 0.0f;
}

__device__ __forceinline__ void raise_max_a(Partial &p, float cm)
{
    if (cm > p.m) {
        if (p.S > 0.0f) {
            const float d = p.m - cm;
            const float c = EXPF(d);
            p.U = c * (p.U + d * p.S);
            p.S *= c;
            p.D *= c;
        }
        p.m = cm;
    }
}

__device__ __forceinline__ void raise_max_b(Partial &p, float cm)
{
    if (cm > p.mb) {
        if (p.Sb > 0.0f)
            p.Sb *= EXPF(p.mb - cm);
        p.mb = cm;
    }
}

template <bool HAS_B>
__device__ __forceinline__ void add_one(Partial &p, float a, float b)
{
    const float t = a - p.m;
    const float e = EXPF(t);
    const bool live = e > 0.0f; // e = 0 (a = -inf or far below the maximum) adds nothing
    p.S += e;
    p.U += live ? e * t : 0.0f;
    if (HAS_B) {
        p.D += live ? e * (a - b) : 0.0f;
        p.Sb += EXPF(b - p.mb);
    }
}

template <bool HAS_B>
__device__ __forceinline__ void add_vec(Partial &p, const float4 a, const float4 b)
{
    raise_max_a(p, fmaxf(fmaxf(a.x, a.y), fmaxf(a.z, a.w)));
    if (HAS_B)
        raise_max_b(p, fmaxf(fmaxf(b.x, b.y), fmaxf(b.z, b.w)));
    add_one<HAS_B>(p, a.x, b.x);
    add_one<HAS_B>(p, a.y, b.y);
    add_one<HAS_B>(p, a.z, b.z);
    add_one<HAS_B>(p, a.w, b.w);
}

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1)
        v += __shfl_xor(v, off, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1)
        v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

// Scratch of the split mode: partials [row][split][S, U, D, Sb, m, mb] and arrival tickets, one
// bank per stream (calls on one stream follow one another; calls on different streams use different
// banks).  Tickets are zero at load and the combining workgroup resets its row's ticket, so every
// launch finds them zero.
constexpr int MAX_SPLIT_ROWS = 64, MAX_SPLITS = 32;
__device__ double g_part[FQ_BANKS][MAX_SPLIT_ROWS][MAX_SPLITS][6];
__device__ unsigned int g_ticket[FQ_BANKS][MAX_SPLIT_ROWS];

template <int THREADS, bool HAS_B, bool VEC, typename T>
__global__ __launch_bounds__(THREADS) void entropy_kl_kernel(const T *__restrict__ a,
                                                             const T *__restrict__ b, int V,
                                                             int splits, int bank, float *__restrict__ H,
                                                             float *__restrict__ KL)
{
    constexpr int WAVES = THREADS / 64;
    __shared__ float s_max[2][WAVES];
    __shared__ double s_sum[4][WAVES];
    __shared__ unsigned int s_last;

    const int r = blockIdx.x / splits, sidx = blockIdx.x % splits;
    const int t = threadIdx.x;
    const T *ar = a + (size_t)r * V;
    const T *br = HAS_B ? b + (size_t)r * V : ar;

    Partial p;
    part_init(p);
    const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
    if (VEC) { // V % 4 == 0 and rows aligned to four entries
        const int nvec = V >> 2;
        const int per = (nvec + splits - 1) / splits;
        const int end = min(nvec, (sidx + 1) * per);
        int i = sidx * per + t;
        for (; i + 3 * THREADS < end; i += 4 * THREADS) {
            const float4 a0 = load4(ar, i), a1 = load4(ar, i + THREADS), a2 = load4(ar, i + 2 * THREADS),
                         a3 = load4(ar, i + 3 * THREADS);
            float4 b0 = zero4, b1 = zero4, b2 = zero4, b3 = zero4;
            if (HAS_B) {
                b0 = load4(br, i);
                b1 = load4(br, i + THREADS);
                b2 = load4(br, i + 2 * THREADS);
                b3 = load4(br, i + 3 * THREADS);
            }
            add_vec<HAS_B>(p, a0, b0);
            add_vec<HAS_B>(p, a1, b1);
            add_vec<HAS_B>(p, a2, b2);
            add_vec<HAS_B>(p, a3, b3);
        }
        for (; i < end; i += THREADS)
            add_vec<HAS_B>(p, load4(ar, i), HAS_B ? load4(br, i) : zero4);
    } else {
        const int per = (V + splits - 1) / splits;
        const int end = min(V, (sidx + 1) * per);
        for (int i = sidx * per + t; i < end; i += THREADS) {
            const float av = (float)ar[i];
            const float bv = HAS_B ? (float)br[i] : 0.0f;
            raise_max_a(p, av);
            if (HAS_B)
                raise_max_b(p, bv);
            add_one<HAS_B>(p, av, bv);
        }
    }

    // Maxima over the workgroup.
    const int wave = t >> 6, lane = t & 63;
    float gm = wave_max(p.m), gmb = wave_max(p.mb);
    if (lane == 0) {
        s_max[0][wave] = gm;
        s_max[1][wave] = gmb;
    }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < WAVES; w++) {
        gm = fmaxf(gm, s_max[0][w]);
        gmb = fmaxf(gmb, s_max[1][w]);
    }
    // Rescale this lane's partial to the maxima, then sum in double.
    double S = 0.0, U = 0.0, D = 0.0, Sb = 0.0;
    if (p.S > 0.0f) {
        const float d = p.m - gm;
        const double c = (double)expf(d);
        S = c * (double)p.S;
        U = c * ((double)p.U + (double)d * (double)p.S);
        D = c * (double)p.D;
    }
    if (HAS_B && p.Sb > 0.0f)
        Sb = (double)expf(p.mb - gmb) * (double)p.Sb;
    S = wave_sum(S);
    U = wave_sum(U);
    if (HAS_B) {
        D = wave_sum(D);
        Sb = wave_sum(Sb);
    }
    if (lane == 0) {
        s_sum[0][wave] = S;
        s_sum[1][wave] = U;
        s_sum[2][wave] = D;
        s_sum[3][wave] = Sb;
    }
    __syncthreads();
    S = U = D = Sb = 0.0;
#pragma unroll
    for (int w = 0; w < WAVES; w++) {
        S += s_sum[0][w];
        U += s_sum[1][w];
        D += s_sum[2][w];
        Sb += s_sum[3][w];
    }
    if (splits > 1) {
        // publish this workgroup's partial, then see whether it is the last to arrive
        if (t == 0) {
            double *slot = g_part[bank][r][sidx];
            slot[0] = S;
            slot[1] = U;
            slot[2] = D;
            slot[3] = Sb;
            slot[4] = (double)gm;
            slot[5] = (double)gmb;
            __threadfence();
            s_last = atomicAdd(&g_ticket[bank][r], 1u) == (unsigned)splits - 1 ? 1u : 0u;
        }
        __syncthreads();
        if (!s_last || wave != 0)
            return;
        __threadfence();
        // first wavefront of the last workgroup: lane i takes partial i
        double pm = -INFINITY, pmb = -INFINITY;
        S = U = D = Sb = 0.0;
        if (lane < splits) {
            const double *slot = g_part[bank][r][lane];
            S = __hip_atomic_load(&slot[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            U = __hip_atomic_load(&slot[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            D = __hip_atomic_load(&slot[2], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            Sb = __hip_atomic_load(&slot[3], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            pm = __hip_atomic_load(&slot[4], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            pmb = __hip_atomic_load(&slot[5], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        gm = wave_max((float)pm);
        gmb = wave_max((float)pmb);
        if (S > 0.0) {
            const float d = (float)pm - gm;
            const double c = (double)expf(d);
            U = c * (U + (double)d * S);
            S *= c;
            D *= c;
        }
        if (Sb > 0.0)
            Sb *= (double)expf((float)pmb - gmb);
        S = wave_sum(S);
        U = wave_sum(U);
        D = wave_sum(D);
        Sb = wave_sum(Sb);
        if (lane == 0)
            g_ticket[bank][r] = 0u; // ready for the next launch
    }
    if (t == 0) {
        H[r] = (float)(log(S) - U / S);
        if (HAS_B)
            KL[r] = (float)(D / S + ((double)gmb - (double)gm) + log(Sb / S));
    }
}

template <int THREADS, typename T>
hipError_t launch(const T *a, const T *b, int R, int V, int splits, int bank, float *H, float *KL,
                  hipStream_t stream)
{
    const uintptr_t mask = 4 * sizeof(T) - 1;
    const bool vec = (V % 4 == 0) && (((uintptr_t)a & mask) == 0) && (!b || ((uintptr_t)b & mask) == 0);
    const dim3 grid((unsigned)R * (unsigned)splits), block(THREADS);
    if (b) {
        if (vec)
            entropy_kl_kernel<THREADS, true, true, T><<<grid, block, 0, stream>>>(a, b, V, splits, bank, H, KL);
        else
            entropy_kl_kernel<THREADS, true, false, T><<<grid, block, 0, stream>>>(a, b, V, splits, bank, H, KL);
    } else {
        if (vec)
            entropy_kl_kernel<THREADS, false, true, T><<<grid, block, 0, stream>>>(a, b, V, splits, bank, H, KL);
        else
            entropy_kl_kernel<THREADS, false, false, T><<<grid, block, 0, stream>>>(a, b, V, splits, bank, H, KL);
    }
    return hipGetLastError();
}

template <typename T>
hipError_t dispatch(const T *a, const T *b, int R, int V, float *H, float *KL, hipStream_t stream)
{
    if (R == 0)
        return hipSuccess;
    // A few rows: split every row over several workgroups (>= 1024 entries each).
    // (if more streams than there are scratch banks have come by: whole rows, as below)
    const int bank = R <= MAX_SPLIT_ROWS && V >= 2048 ? fq_stream_bank(stream) : -1;
    if (bank >= 0) {
        int splits = V / 1024;
        if (splits > MAX_SPLITS)
            splits = MAX_SPLITS;
        return launch<256, T>(a, b, R, V, splits, bank, H, KL, stream);
    }
    // Otherwise one workgroup per row: large ones while there are too few rows to fill the
    // machine, 256 threads (several rows per CU) beyond that.
    if (R < 512)
        return launch<1024, T>(a, b, R, V, 1, 0, H, KL, stream);
    return launch<256, T>(a, b, R, V, 1, 0, H, KL, stream);
}

} // namespace

hipError_t fq_launch_entropy_kl(const float *a, const float *b, int R, int V, float *H, float *KL,
                                hipStream_t stream)
{
    return dispatch<float>(a, b, R, V, H, KL, stream);
}

hipError_t fq_launch_entropy_kl_f16(const uint16_t *a, const uint16_t *b, int R, int V, float *H,
                                    float *KL, hipStream_t stream)
{
    return dispatch<_Float16>(reinterpret_cast<const _Float16 *>(a), reinterpret_cast<const _Float16 *>(b),
                              R, V, H, KL, stream);
}
