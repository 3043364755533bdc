// Step a5: the persistent mixed kernel.
//
// A Convertible Decoder's iteration holds HBM-bound decode rows and MFMA-bound prefill tiles at
// once (paper Sec. 3.4: the decoder's spare compute absorbs the prefill burst).  Launching the
// two kinds one after the other leaves the matrix cores idle during the decode scan and HBM idle
// during the prefill tiles.  Here a fixed grid of workgroups (as many as fit on the GPU) stays
// resident and pulls work from queues until they are empty, so both kinds are in flight on every
// CU for the whole launch:
//   - one queue per accelerator die (workgroup i runs on die i % n_xcd and starts on that die's
//     queue): a prefill stream stays on one die, whose L2 then holds its K/V pages once;
//   - the host interleaved the two kinds in each queue by their share of their own kind's cost,
//     decode first on ties, so both kinds drain at the same pace and finish together;
//   - a workgroup whose queue is empty helps on the next die's queue; it leaves when every queue
//     has been seen empty (queue heads only grow, so every workgroup ends);
//   - the last workgroup to leave puts the queue heads back to zero for the next launch.
// The work itself is the same code as the stand-alone kernels (decode_item, prefill_tile).
#include "ts_decode_item.h"
#include "ts_prefill_tile.h"

namespace ts {

union MixedLds {
    DecMerge<kPfWaves> mg;
    PfLds lds;
};

// The queue loop of a resident workgroup.  WITH_DECODE: the queues hold both kinds (one persistent kernel);
// without it they hold prefill tiles only and LDS is the tile ring alone.
// KT: element type the decode items read (the cache's); PKT: element type the prefill tiles read (the cache's,
// or bf16 when the pages of an e4m3 cache were widened before the launch).
template <typename KT, typename PKT, bool WIDE, int NBUF, bool WITH_DECODE, typename LDS>
__device__ __forceinline__ void drain_queues(const AttnArgs& a, LDS& sh)
{
    int& s_idx = *reinterpret_cast<int*>(&sh);             // LDS is idle between two items
    const int tid = threadIdx.x;
    const int n_xcd = a.n_xcd;
    const int32_t TS_CONSTANT* q_off = as_constant(a.q_off);
    int x = blockIdx.x % n_xcd;
    for (int n_empty = 0; n_empty < n_xcd;) {
        if (tid == 0) s_idx = __hip_atomic_fetch_add(a.q_ctr + x, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        const int idx = __builtin_amdgcn_readfirstlane(s_idx);
        __syncthreads();                                       // s_idx may be overwritten from here on
        const int begin = q_off[x], end = q_off[x + 1];
        if (idx >= end - begin) {                              // this queue is (now and for ever) empty
            ++n_empty;
            x = (x + 1) % n_xcd;
            continue;
        }
        const int32_t TS_CONSTANT* q = as_constant((const int32_t*)(a.queue + begin + idx));
        const int kind = q[0], item = q[1], g = q[2];
        int t = tid;
        asm volatile("" : "+v"(t));                            // (see prefill_tile)
        if constexpr (WITH_DECODE) {
            if (kind == 0) decode_item<KT, NBUF, kPfWaves>(a, load_dec_item(a.dec + item), g, sh.mg);
            else prefill_tile<PKT, WIDE, 128>(a, item, g, sh.lds, t);
        } else {
            prefill_tile<PKT, WIDE, 128>(a, item, g, sh, t);
        }
        __syncthreads();                                       // LDS is reused by the next item
    }
    // last workgroup out resets the counters
    if (tid == 0) {
        __threadfence();
        const int done = __hip_atomic_fetch_add(a.q_ctr + n_xcd, 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        if (done == (int)gridDim.x - 1) {
            for (int i = 0; i <= n_xcd; ++i)
                __hip_atomic_store(a.q_ctr + i, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

template <typename KT, typename PKT, bool WIDE, int NBUF>
__global__ __launch_bounds__(kPfThreads) void mixed_kernel(AttnArgs a)
{
    __shared__ MixedLds sh;
    drain_queues<KT, PKT, WIDE, NBUF, true>(a, sh);
}

// Co-resident form: one of these workgroups per CU stays for the whole launch and works through the prefill
// tiles; it is held to 192 vector registers per lane (two waves per SIMD: 384 of 512) and uses 128 of the
// 160 KB of LDS, so that every CU keeps room for one 4-wave decode workgroup of 128 registers per lane and
// 25 KB -- the decode grid that the host launches next to it on a second stream.  The HBM-bound scan then
// runs in the shadow of the MFMA-bound tiles on the same CU instead of taking turns with them.
// (The register attribute counts in units of two on this architecture: 96 means 192.)
template <typename KT, bool WIDE>
__global__ __launch_bounds__(kPfThreads) __attribute__((amdgpu_num_vgpr(96))) void prefill_resident_kernel(AttnArgs a)
{
    __shared__ PfLds lds;
    drain_queues<KT, KT, WIDE, 2, false>(a, lds);
}

template <typename KT>
static int resident_mixed_t()
{
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, mixed_kernel<KT, KT, false, 2>, kPfThreads, 0) != hipSuccess)
        return 0;
    return cus * (per_cu > 0 ? per_cu : 1);
}

int mixed_resident_workgroups(int kv_dtype)
{
    return kv_dtype == TS_FP8_E4M3 ? resident_mixed_t<uint8_t>() : resident_mixed_t<uint16_t>();
}

template <typename KT, typename PKT, bool WIDE>
static int launch_mixed_t(const AttnArgs& a, hipStream_t st)
{
    const int n = a.mixed_wgs;                                 // resident workgroups on the context's GPU
    if (n <= 0) return (int)hipErrorInvalidValue;
    const int grid = n < a.n_queue ? n : a.n_queue;
    hipLaunchKernelGGL((mixed_kernel<KT, PKT, WIDE, 2>), dim3((unsigned)grid), dim3(kPfThreads), 0, st, a);
    return (int)hipGetLastError();
}

int launch_prefill_resident(const AttnArgs& a, void* stream)
{
    if (a.n_queue <= 0) return (int)hipSuccess;
    if (a.geo.D != 128 || a.geo.q_dtype != TS_BF16 || a.n_xcd <= 0 || a.n_xcd > 64 || a.n_cu <= 0) return (int)hipErrorInvalidValue;
    const int want = a.pf_wgs > 0 && a.pf_wgs < a.n_cu ? a.pf_wgs : a.n_cu;   // (128 KB of LDS: at most one per CU)
    const int grid = want < a.n_queue ? want : a.n_queue;
    hipStream_t st = (hipStream_t)stream;
    const dim3 g3((unsigned)grid), b3(kPfThreads);
    if (a.geo.kv_dtype == TS_BF16) hipLaunchKernelGGL((prefill_resident_kernel<uint16_t, false>), g3, b3, 0, st, a);
    else if (a.geo.kv_dtype == TS_FP8_E4M3 && a.wide_base) hipLaunchKernelGGL((prefill_resident_kernel<uint16_t, true>), g3, b3, 0, st, a);
    else if (a.geo.kv_dtype == TS_FP8_E4M3) hipLaunchKernelGGL((prefill_resident_kernel<uint8_t, false>), g3, b3, 0, st, a);
    else return (int)hipErrorInvalidValue;
    return (int)hipGetLastError();
}

int launch_mixed(const AttnArgs& a, void* stream)
{
    if (a.n_queue <= 0) return (int)hipSuccess;
    if (a.geo.D != 128 || a.geo.q_dtype != TS_BF16 || a.n_xcd <= 0 || a.n_xcd > 64) return (int)hipErrorInvalidValue;
    hipStream_t st = (hipStream_t)stream;
    if (a.geo.kv_dtype == TS_BF16) return launch_mixed_t<uint16_t, uint16_t, false>(a, st);
    if (a.geo.kv_dtype == TS_FP8_E4M3 && a.wide_base) return launch_mixed_t<uint8_t, uint16_t, true>(a, st);
    if (a.geo.kv_dtype == TS_FP8_E4M3) return launch_mixed_t<uint8_t, uint8_t, false>(a, st);
    return (int)hipErrorInvalidValue;
}

}  // namespace ts
