// Per-device facts the launch code needs on every call -- the number of compute units, how many
// workgroups of a kernel fit on one, whether a kernel's dynamic LDS limit has been raised -- asked
// of the HIP runtime once per device and kept in fixed-size tables (no allocation), under a mutex
// so that several host threads, each with its own current device, may launch at once; and which
// bank of the library's static scratch arrays a stream uses.
#include <hip/hip_runtime.h>

#include <mutex>

#include "fq_internal.h"

namespace {

constexpr int MAX_DEVICES = 64;
constexpr int MAX_KERNEL_FACTS = 128; // per device: (kernel, threads, LDS bytes) -> workgroups per CU

struct KernelFact {
    const void *func;
    int threads;
    size_t lds;
    int per_cu;
};

struct DeviceFacts {
    int cus;       // 0 = not asked yet
    int n_facts;
    KernelFact facts[MAX_KERNEL_FACTS];
    int n_raised;
    const void *raised[MAX_KERNEL_FACTS]; // kernels whose dynamic LDS limit was raised
    size_t raised_to[MAX_KERNEL_FACTS];
    int n_banks;
    hipStream_t bank_stream[FQ_BANKS]; // the stream that bank i of the static scratch arrays belongs to
};

std::mutex g_lock;
DeviceFacts g_dev[MAX_DEVICES];

// The current device's table, or null (device index out of the table's range: ask every time).
DeviceFacts *current()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES)
        return nullptr;
    return &g_dev[dev];
}

int ask_cus()
{
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        return 256;
    return cus;
}

} // namespace

int fq_device_cus()
{
    std::lock_guard<std::mutex> hold(g_lock);
    DeviceFacts *d = current();
    if (!d)
        return ask_cus();
    if (d->cus == 0)
        d->cus = ask_cus();
    return d->cus;
}

int fq_workgroups_per_cu(const void *func, int threads, size_t lds, int fallback)
{
    std::lock_guard<std::mutex> hold(g_lock);
    DeviceFacts *d = current();
    if (d)
        for (int i = 0; i < d->n_facts; i++)
            if (d->facts[i].func == func && d->facts[i].threads == threads && d->facts[i].lds == lds)
                return d->facts[i].per_cu;
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, func, threads, lds) != hipSuccess || per_cu < 1)
        per_cu = fallback;
    if (d && d->n_facts < MAX_KERNEL_FACTS)
        d->facts[d->n_facts++] = KernelFact{func, threads, lds, per_cu};
    return per_cu;
}

int fq_stream_bank(hipStream_t stream)
{
    std::lock_guard<std::mutex> hold(g_lock);
    DeviceFacts *d = current();
    if (!d)
        return -1;
    for (int i = 0; i < d->n_banks; i++)
        if (d->bank_stream[i] == stream)
            return i;
    if (d->n_banks == FQ_BANKS)
        return -1;
    d->bank_stream[d->n_banks] = stream;
    return d->n_banks++;
}

hipError_t fq_raise_dynamic_lds(const void *func, size_t bytes)
{
    std::lock_guard<std::mutex> hold(g_lock);
    DeviceFacts *d = current();
    if (d)
        for (int i = 0; i < d->n_raised; i++)
            if (d->raised[i] == func && d->raised_to[i] >= bytes)
                return hipSuccess;
    const hipError_t e = hipFuncSetAttribute(func, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess)
        return e;
    if (d) {
        for (int i = 0; i < d->n_raised; i++)
            if (d->raised[i] == func) {
                d->raised_to[i] = bytes;
                return hipSuccess;
            }
        if (d->n_raised < MAX_KERNEL_FACTS) {
            d->raised[d->n_raised] = func;
            d->raised_to[d->n_raised++] = bytes;
        }
    }
    return hipSuccess;
}
