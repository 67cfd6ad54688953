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
// of them per group of 128; it is exact, the zero-point term is added in integers, and the
// group result is folded into a binary32 accumulator as out += s * (float)t.
//
// Tiling.  A workgroup of 4 wavefronts owns 128 tokens x 256 weight rows, a wavefront
// 128 tokens x 64 rows = 4 x 2 MFMA tiles.  The binary32 accumulators are updated by vector
// instructions, so they must sit in the 256 architectural registers (the other half of the
// file only feeds MFMAs and loads): 128 of them is what leaves room for the rest.  x goes
// through LDS (128 x 128 bytes per step, double buffered, one barrier per step); a lane
// loads its weight rows straight from global memory in the MFMA operand layout (16
// consecutive k of row n), two steps ahead, so no weight byte is loaded twice inside a
// workgroup.  One step = one quantization group.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fq_internal.h"

namespace {

#define FQ_GLOBAL __attribute__((address_space(1)))

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
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

constexpr int THREADS = 256;
constexpr int BM = 128, BN = 256;
constexpr int BKB = 128;         // k (= bytes of a row) per step: one quantization group
constexpr int MT = BM / 32;      // MFMA tiles along the tokens, per wavefront (4)
constexpr int WN = BN / 4;       // weight rows per wavefront (2 MFMA tiles)
constexpr int LDB = BKB + 16;    // bytes per LDS row of x: 144, keeps the 128-bit reads conflict-free
constexpr int XLD = BM * (BKB / 16) / THREADS; // 16-byte pieces of the x slab per thread (4)

__device__ __forceinline__ uint4 load16(const void *p)
{
    const u32x4 v = *(const FQ_GLOBAL u32x4 *)p;
    return make_uint4(v.x, v.y, v.z, v.w);
}

// One step of weights for one lane: per n-tile, four 16-byte loads (k = 32 i + 16 c ..),
// the group's scale and 128 - z.
struct WRegs {
    uint4 w[2][4];
    float s[2];
    int nzc[2];
};

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

__device__ __forceinline__ void load_w(const W8A8Args &d, int n_wave0, int g, WRegs &R)
{
    const int lane = threadIdx.x & 63, n = lane & 31, c = lane >> 5;
    const uint32_t K = (uint32_t)d.K, G = K >> 7;
#pragma unroll
    for (int j = 0; j < 2; j++) {
        const size_t row = (size_t)min(n_wave0 + j * 32 + n, d.N - 1);
#pragma unroll
        for (int i = 0; i < 4; i++)
            R.w[j][i] = load16(d.codes + row * K + g * BKB + 32 * i + 16 * c);
        R.s[j] = ((const FQ_GLOBAL float *)d.scales)[row * G + g];
        R.nzc[j] = 128 - (int)((const FQ_GLOBAL uint8_t *)d.zeros)[row * G + g];
    }
}

struct XRegs {
    uint4 x[XLD];
    int sum;
};

__device__ __forceinline__ void load_x(const W8A8Args &d, int m0, int g, XRegs &R)
{
#pragma unroll
    for (int i = 0; i < XLD; i++) {
        const int idx = i * THREADS + threadIdx.x, row = idx >> 3, piece = idx & 7;
        const int m = min(m0 + row, d.M - 1);
        R.x[i] = load16(d.xq + (size_t)m * d.K + g * BKB + piece * 16);
    }
    // the first BM threads also fetch one token's group sum each
    R.sum = ((const FQ_GLOBAL int32_t *)d.xsum)[(size_t)g * d.M + min(m0 + (int)(threadIdx.x & (BM - 1)), d.M - 1)];
}

__device__ __forceinline__ void store_x(const XRegs &R, uint8_t *xs, int32_t *xsm)
{
#pragma unroll
    for (int i = 0; i < XLD; i++) {
        const int idx = i * THREADS + threadIdx.x, row = idx >> 3, piece = idx & 7;
        *reinterpret_cast<uint4 *>(xs + row * LDB + piece * 16) = R.x[i];
    }
    if (threadIdx.x < BM)
        xsm[threadIdx.x] = R.sum;
}

__global__ __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(1, 1))) void w8a8_kernel(
    const W8A8Args d, int m_tiles, int n_tiles, int per_xcd)
{
    __shared__ __attribute__((aligned(16))) uint8_t xs[2][BM * LDB];
    __shared__ __attribute__((aligned(16))) int32_t xsm[2][BM];

    // consecutive workgroup ids go round-robin to the 8 XCDs: give each XCD a contiguous run
    // of logical tiles (the M tiles of one N tile are neighbours and share the weight slab)
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= m_tiles * n_tiles)
        return;
    const int m0 = (logical % m_tiles) * BM, n0 = (logical / m_tiles) * BN;

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int l32 = lane & 31, c = lane >> 5;
    const int n_wave0 = n0 + wave * WN;

    float out[MT][2][16];
#pragma unroll
    for (int mt = 0; mt < MT; mt++)
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
            for (int v = 0; v < 16; v++)
                out[mt][j][v] = 0.f;

    const int nsteps = d.K / BKB;
    XRegs X;
    WRegs W0, W1;
    load_x(d, m0, 0, X);
    load_w(d, n_wave0, 0, W0);
    store_x(X, xs[0], xsm[0]);
    load_x(d, m0, min(1, nsteps - 1), X);
    load_w(d, n_wave0, min(1, nsteps - 1), W1);
    __syncthreads();

    // One step (one group): MFMAs of step s from xs[s & 1] and Wcur; meanwhile x of step s+1
    // goes from registers to the other LDS buffer and the loads of step s+2 are issued.
    auto step = [&](int s, WRegs &Wcur) {
        const uint8_t *xc = xs[s & 1];
        const int32_t *sc = xsm[s & 1];
        store_x(X, xs[(s + 1) & 1], xsm[(s + 1) & 1]); // last read in step s-1: a barrier has passed
        load_x(d, m0, min(s + 2, nsteps - 1), X);
        v4i b[2][4];
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
            for (int i = 0; i < 4; i++) { // stored code q -> signed byte q - 128
                b[j][i].x = (int)(Wcur.w[j][i].x ^ 0x80808080u);
                b[j][i].y = (int)(Wcur.w[j][i].y ^ 0x80808080u);
                b[j][i].z = (int)(Wcur.w[j][i].z ^ 0x80808080u);
                b[j][i].w = (int)(Wcur.w[j][i].w ^ 0x80808080u);
            }
#pragma unroll
        for (int mt = 0; mt < MT; mt++) {
            v4i a[4];
#pragma unroll
            for (int i = 0; i < 4; i++)
                a[i] = *reinterpret_cast<const v4i *>(xc + (mt * 32 + l32) * LDB + 32 * i + 16 * c);
            // group sums of the 16 tokens this lane holds results for (D layout below)
            v4i xsv[4];
#pragma unroll
            for (int q = 0; q < 4; q++)
                xsv[q] = *reinterpret_cast<const v4i *>(sc + mt * 32 + 8 * q + 4 * c);
#pragma unroll
            for (int j = 0; j < 2; j++) {
                v16i acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                for (int i = 0; i < 4; i++)
                    acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j][i], acc, 0, 0, 0);
#pragma unroll
                for (int v = 0; v < 16; v++) {
                    // sum x (q - z) = sum x (q - 128) + (128 - z) sum x, all in 24 bits
                    const int t = acc[v] + __mul24(Wcur.nzc[j], xsv[v >> 2][v & 3]);
                    out[mt][j][v] += Wcur.s[j] * (float)t;
                }
            }
        }
        load_w(d, n_wave0, min(s + 2, nsteps - 1), Wcur); // always issued: keeps the waits counted
        __syncthreads(); // xs[(s+1)&1] complete, xs[s&1] no longer read
    };
    int s = 0;
    for (; s + 1 < nsteps; s += 2) {
        step(s, W0);
        step(s + 1, W1);
    }
    if (s < nsteps)
        step(s, W0);

    // D layout of the 32x32 MFMA: lane holds column l32 (weight row), rows (tokens)
    // 8 * (v / 4) + 4 * (lane / 32) + v % 4.
#pragma unroll
    for (int mt = 0; mt < MT; mt++) {
#pragma unroll
        for (int v = 0; v < 16; v++) {
            const int m = m0 + mt * 32 + 8 * (v >> 2) + 4 * c + (v & 3);
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
                          int M, hipStream_t stream)
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
    const int m_tiles = (M + BM - 1) / BM, n_tiles = (l.N + BN - 1) / BN;
    const long long total = (long long)m_tiles * n_tiles;
    if (total > 0x3fffffffLL)
        return hipErrorInvalidValue;
    const int per_xcd = (int)((total + 7) / 8);
    w8a8_kernel<<<(unsigned)per_xcd * 8, THREADS, 0, stream>>>(d, m_tiles, n_tiles, per_xcd);
    return hipGetLastError();
}
