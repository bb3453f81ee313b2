/* GPU half of the synthetic model-data generator (see gen_core.h): fills device
 * buffers in place so that 100 GB of model data need not cross PCIe.  A fixture
 * for tests and the benchmark; not part of the optimizer library. */
#include <hip/hip_runtime.h>
#define SYNTH_HD static __device__ __host__ inline
#include "gen_core.h"

__global__ void __launch_bounds__(256) synth_fill_kernel(void *out, uint64_t count, synth_spec spec)
{
    uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride)
        synth_store(&spec, out, spec.first_index + i);
}

extern "C" int synth_gpu_fill(void *dev_out, uint64_t count, const synth_spec *spec, void *stream)
{
    if (count == 0) return 0;
    uint64_t blocks = (count + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(synth_fill_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       dev_out, count, *spec);
    return (int)hipGetLastError();
}
