// Prefill-shaped dequant-GEMM (placeholder until the MFMA kernel lands).
#include <hip/hip_runtime.h>
#include "fq_internal.h"

hipError_t fq_launch_prefill(const FqLinearDesc &d, int bits, int M, hipStream_t stream)
{
    (void)d; (void)bits; (void)M; (void)stream;
    return hipErrorNotSupported;
}
