// fq_linears_static: a list of decode-phase linears run by one launch, for callers that cannot
// allocate -- code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
// It is fq_plan_create + fq_plan_run without the caller's workspace and without a plan object: the
// descriptor table, the tile queue and the per-launch entry lists that a plan keeps in its
// workspace live in a static device array of this library, and the table reaches it through the
// arguments of a small kernel (no copy from host memory, no synchronisation).
#include <hip/hip_runtime.h>

#include <mutex>

#include "../../include/flexq.h"
#include "fq_internal.h"

namespace {

constexpr size_t TABLE_BYTES = ((size_t)FQ_STATIC_MAX_ENTRIES * sizeof(FqLinearDesc) + 255) / 256 * 256;
constexpr size_t QUEUE_BYTES = 256;
constexpr size_t ORDER_BYTES = ((size_t)FQ_STATIC_MAX_ENTRIES * 8 + 255) / 256 * 256;
constexpr size_t SCRATCH_BYTES = TABLE_BYTES + QUEUE_BYTES + ORDER_BYTES;

} // namespace

// The workspace of every fq_linears_static call on a device (each device holds its own copy, at
// its own address, until the process ends).  In host code this name is only a handle for
// hipGetSymbolAddress: kernels and copies are given the address that call returns.
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

namespace {

constexpr int BATCH = 24; // descriptors per fill launch: 3264 bytes of kernel arguments

struct DescBatch {
    FqLinearDesc d[BATCH];
};

// Writes descriptors [first, first + n) of the table from the kernel arguments; the launch that
// carries the first batch also clears the queue words (the kernels that use them expect zeros and
// leave zeros, but a call cut short by an error on the device may not have).
__global__ __launch_bounds__(256) void table_fill_kernel(const DescBatch batch, int n, int first,
                                                         FqLinearDesc *table, int *queue)
{
    constexpr int WORDS = sizeof(FqLinearDesc) / 4;
    uint32_t *dst = reinterpret_cast<uint32_t *>(table + first);
    for (int i = 0; i < n; i++) { // i is uniform: the descriptor comes off the argument segment by scalar loads
        const FqLinearDesc d = batch.d[i];
        const uint32_t *src = reinterpret_cast<const uint32_t *>(&d);
        if (threadIdx.x < WORDS) {
            uint32_t w = 0;
#pragma unroll
            for (int j = 0; j < WORDS; j++)
                if ((int)threadIdx.x == j)
                    w = src[j];
            dst[i * WORDS + threadIdx.x] = w;
        }
    }
    if (first == 0 && threadIdx.x < (int)(QUEUE_BYTES / 4))
        queue[threadIdx.x] = 0;
}

constexpr int MAX_DEVICES = 64;
std::mutex g_lock;
unsigned char *g_scratch[MAX_DEVICES]; // device address of `scratch` on each device, null = not asked yet

// Address of the current device's copy of `scratch`.
hipError_t scratch_address(unsigned char **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return e;
    if (dev < 0 || dev >= MAX_DEVICES)
        return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> hold(g_lock);
    if (!g_scratch[dev]) {
        unsigned char *ptr = nullptr;
        e = hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess)
            return e;
        if (!ptr)
            return hipErrorInvalidSymbol;
        g_scratch[dev] = ptr;
    }
    *out = g_scratch[dev];
    return hipSuccess;
}

} // namespace

extern "C" int fq_linears_static(int count, const fq_layer *const *layers, const void *const *xs, void *const *ys,
                                 int M, const int32_t *bits_dev, void *stream)
{
    if (count > FQ_STATIC_MAX_ENTRIES)
        return fq_fail(FQ_ERR_SHAPE, "fq_linears_static: count=%d exceeds FQ_STATIC_MAX_ENTRIES=%d", count,
                       FQ_STATIC_MAX_ENTRIES);
    if (!bits_dev)
        return fq_fail(FQ_ERR_NULL, "fq_linears_static: bits_dev is NULL");
    if (reinterpret_cast<uintptr_t>(bits_dev) & 3u)
        return fq_fail(FQ_ERR_ALIGN, "fq_linears_static: bits_dev must be 4-byte aligned");
    static thread_local FqLinearDesc table[FQ_STATIC_MAX_ENTRIES]; // host side, no allocation per call
    FqPlanGeom geom;
    if (int rc = fq_plan_layout("fq_linears_static", count, layers, xs, ys, M, table, &geom))
        return rc;
    unsigned char *ptr = nullptr;
    hipError_t e = scratch_address(&ptr);
    if (e != hipSuccess)
        return fq_fail(FQ_ERR_HIP, "fq_linears_static: address of the static workspace: %s", hipGetErrorString(e));
    FqLinearDesc *table_dev = reinterpret_cast<FqLinearDesc *>(ptr);
    int *queue_dev = reinterpret_cast<int *>(ptr + TABLE_BYTES);
    void *order_dev = ptr + TABLE_BYTES + QUEUE_BYTES;
    for (int first = 0; first < count; first += BATCH) {
        DescBatch batch = {};
        const int n = count - first < BATCH ? count - first : BATCH;
        for (int i = 0; i < n; i++)
            batch.d[i] = table[first + i];
        table_fill_kernel<<<1, 256, 0, (hipStream_t)stream>>>(batch, n, first, table_dev, queue_dev);
        e = hipGetLastError();
        if (e != hipSuccess)
            return fq_fail(FQ_ERR_HIP, "fq_linears_static: table launch: %s", hipGetErrorString(e));
    }
    e = fq_plan_launch(geom, table_dev, queue_dev, order_dev, bits_dev, (hipStream_t)stream);
    if (e != hipSuccess)
        return fq_fail(FQ_ERR_HIP, "fq_linears_static launch: %s", hipGetErrorString(e));
    return FQ_OK;
}
