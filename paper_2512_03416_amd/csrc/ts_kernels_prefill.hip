// Step a3: launcher of the prefill-tile kernel.
#include "ts_prefill_tile.h"

namespace ts {

// (held to 192 vector registers per lane like the resident form: the attribute counts in units of two)
template <typename KT>
__global__ __launch_bounds__(kPfThreads) __attribute__((amdgpu_num_vgpr(96))) void prefill_kernel(AttnArgs a)
{
    __shared__ PfLds lds;
    const int32_t TS_CONSTANT* slot = as_constant((const int32_t*)(a.pfmap + blockIdx.x));
    const int item_idx = slot[0], g = slot[1];
    if (item_idx < 0) return;                               // padding of the die-aware launch order
    prefill_tile<KT>(a, item_idx, g, lds, threadIdx.x);
}

int launch_prefill(const AttnArgs& a, void* stream)
{
    if (a.n_pf <= 0) return (int)hipSuccess;
    if (a.geo.D != 128 || a.geo.q_dtype != TS_BF16) return (int)hipErrorInvalidValue;
    dim3 grid((unsigned)a.n_pfmap), block(kPfThreads);
    hipStream_t st = (hipStream_t)stream;
    if (a.geo.kv_dtype == TS_BF16) hipLaunchKernelGGL((prefill_kernel<uint16_t>), grid, block, 0, st, a);
    else if (a.geo.kv_dtype == TS_FP8_E4M3) hipLaunchKernelGGL((prefill_kernel<uint8_t>), grid, block, 0, st, a);
    else return (int)hipErrorInvalidValue;
    return (int)hipGetLastError();
}

}  // namespace ts
