// fq_stream_read: a plain read-only pass over a buffer with the access pattern of the decode
// kernels (non-temporal 128-bit loads, a wavefront reading 1 KiB at a time, eight loads per lane in
// flight, two workgroups per compute unit), so that a benchmark can quote what the weight stream of
// Sec. 4.1 achieves against what this machine gives to a kernel that does nothing but read.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/flexq.h"
#include "fq_internal.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int THREADS = 256, UNROLL = 8;

__global__ __launch_bounds__(THREADS) void stream_read_kernel(const u32x4 *__restrict__ src, size_t n16,
                                                              uint32_t *__restrict__ sink)
{
    const size_t stride = (size_t)gridDim.x * THREADS;
    size_t i = (size_t)blockIdx.x * THREADS + threadIdx.x;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (; i + (UNROLL - 1) * stride < n16; i += UNROLL * stride) {
        u32x4 v[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; u++)
            v[u] = __builtin_nontemporal_load(&src[i + u * stride]);
#pragma unroll
        for (int u = 0; u < UNROLL; u++)
            acc ^= v[u];
    }
    for (; i < n16; i += stride)
        acc ^= __builtin_nontemporal_load(&src[i]);
    // the loads must not be optimised away; the store hardly ever happens
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u)
        sink[0] = 1u;
}

} // namespace

extern "C" int fq_stream_read(const void *src, size_t bytes, uint32_t *sink, void *stream)
{
    if (!src || !sink)
        return fq_fail(FQ_ERR_NULL, "fq_stream_read: NULL argument");
    if ((reinterpret_cast<uintptr_t>(src) & 15u) || (reinterpret_cast<uintptr_t>(sink) & 3u))
        return fq_fail(FQ_ERR_ALIGN, "fq_stream_read: src needs 16-byte, sink 4-byte alignment");
    if (bytes < 16)
        return FQ_OK;
    stream_read_kernel<<<2 * fq_device_cus(), THREADS, 0, (hipStream_t)stream>>>((const u32x4 *)src, bytes / 16, sink);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fq_fail(FQ_ERR_HIP, "fq_stream_read launch: %s", hipGetErrorString(e));
    return FQ_OK;
}
