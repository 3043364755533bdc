// Step a2 (+a4): launchers of the decode kernel and of the merge of split rows.
#include "ts_decode_item.h"

namespace ts {

// KV heads vary fastest over the grid: the Hkv workgroups of one item start together and read the
// Hkv adjacent tiles of each page (one contiguous run of the cache) at about the same time.
template <typename KT, int NBUF, int D>
__global__ __launch_bounds__(64 * kDecWaves) void decode_kernel(AttnArgs a)
{
    __shared__ DecMerge<kDecWaves, D> mg;
    decode_item<KT, NBUF, kDecWaves, D>(a, load_dec_item(a.dec + blockIdx.x / a.geo.Hkv), blockIdx.x % a.geo.Hkv, mg);
}

// The default form, two KV tiles in flight per wave, held to 128 vector registers per lane (the attribute
// counts in units of two here): one such workgroup then fits on a CU next to a resident prefill workgroup
// (see prefill_resident_kernel), and four fit on a CU of their own.  A single workgroup of four waves per CU
// already keeps enough loads in flight for the bf16 scan to run at its full rate.
template <typename KT, int D>
__global__ __launch_bounds__(64 * kDecWaves) __attribute__((amdgpu_num_vgpr(64))) void decode_kernel_lean(AttnArgs a)
{
    __shared__ DecMerge<kDecWaves, D> mg;
    decode_item<KT, 2, kDecWaves, D>(a, load_dec_item(a.dec + blockIdx.x / a.geo.Hkv), blockIdx.x % a.geo.Hkv, mg);
}

// The same with the merge of split rows by their last item compiled in (option "decode_merge_in_kernel").
template <typename KT, int D>
__global__ __launch_bounds__(64 * kDecWaves) void decode_kernel_merging(AttnArgs a)
{
    __shared__ DecMerge<kDecWaves, D> mg;
    decode_item<KT, 2, kDecWaves, D, true>(a, load_dec_item(a.dec + blockIdx.x / a.geo.Hkv), blockIdx.x % a.geo.Hkv, mg);
}

// Small decode-only batches are bound by their launches and by the chain of dependent reads at the start of an
// item.  Their fused form has one launch less and one link less: the items append the rows' new tokens themselves
// (decode_item<..., FUSED>: no append launch) and arrive as kernel arguments (no upload of the work lists and
// no read of a list from memory before the first page id can be asked for).
template <typename KT, int D>
__global__ __launch_bounds__(64 * kDecWaves) void decode_kernel_fused(AttnArgs a, SmallLists s)
{
    __shared__ DecMerge<kDecWaves, D> mg;
    decode_item<KT, 2, kDecWaves, D, false, true>(a, s.dec[blockIdx.x / a.geo.Hkv], blockIdx.x % a.geo.Hkv, mg);
}

// Merge of a row's splits, in split order:  M = max m_i, out = sum o_i 2^(m_i-M) / sum l_i 2^(m_i-M).
// The partials of up to eight splits are requested together and then added one after the other: the
// sums keep their order, and a row of ten splits waits for four loads instead of thirty.
__device__ __forceinline__ void combine_row(const AttnArgs& a, const CmbItem it)
{
    constexpr int kBatch = 8;
    const int h = blockIdx.y, d = threadIdx.x;
    const int Hq = a.geo.Hq, D = a.geo.D;
    const float* ml = a.part_ml + ((int64_t)it.part_begin * Hq + h) * 2;      // split k: ml[k * Hq * 2 + {0, 1}]
    const float* po = a.part_o + ((int64_t)it.part_begin * Hq + h) * D + d;    // split k: po[k * Hq * D]
    const int64_t ml_step = (int64_t)Hq * 2, po_step = (int64_t)Hq * D;
    float M = -INFINITY;
    for (int k0 = 0; k0 < it.n_split; k0 += kBatch) {
        float m[kBatch];
#pragma unroll
        for (int j = 0; j < kBatch; ++j) m[j] = k0 + j < it.n_split ? ml[(k0 + j) * ml_step] : -INFINITY;
#pragma unroll
        for (int j = 0; j < kBatch; ++j) M = fmaxf(M, m[j]);
    }
    float o = 0.0f, L = 0.0f;
    for (int k0 = 0; k0 < it.n_split; k0 += kBatch) {
        float m[kBatch], l[kBatch], v[kBatch];
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const bool in = k0 + j < it.n_split;
            m[j] = in ? ml[(k0 + j) * ml_step] : 0.0f;
            l[j] = in ? ml[(k0 + j) * ml_step + 1] : 0.0f;
            v[j] = in ? po[(k0 + j) * po_step] : 0.0f;
        }
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            if (k0 + j < it.n_split) {
                const float w = __builtin_amdgcn_exp2f(m[j] - M);
                L += l[j] * w;
                o += v[j] * w;
            }
        }
    }
    const float vscale = (a.geo.kv_dtype == TS_FP8_E4M3) ? a.v_scale[h / a.geo.G] : 1.0f;
    ((uint16_t*)a.out)[((int64_t)it.row * Hq + h) * D + d] = (uint16_t)float_to_bf16_bits(o * vscale / L);
}

__global__ __launch_bounds__(128) void combine_kernel(AttnArgs a)
{
    combine_row(a, a.cmb[blockIdx.x]);
}

__global__ __launch_bounds__(128) void combine_kernel_small(AttnArgs a, SmallLists s)
{
    combine_row(a, s.cmb[blockIdx.x]);
}

template <typename KT, int D>
static int launch_decode_t(const AttnArgs& a, hipStream_t st)
{
    dim3 grid((unsigned)a.n_dec * (unsigned)a.geo.Hkv), block(64 * kDecWaves);
    if (a.cmb_ctr) {
        hipLaunchKernelGGL((decode_kernel_merging<KT, D>), grid, block, 0, st, a);
        return (int)hipGetLastError();
    }
    switch (a.dec_nbuf) {
    case 3: hipLaunchKernelGGL((decode_kernel<KT, 3, D>), grid, block, 0, st, a); break;
    case 4: hipLaunchKernelGGL((decode_kernel<KT, 4, D>), grid, block, 0, st, a); break;
    default: hipLaunchKernelGGL((decode_kernel_lean<KT, D>), grid, block, 0, st, a); break;
    }
    return (int)hipGetLastError();
}

template <typename KT, int D>
static int resident_t(int nbuf)
{
    int per_cu = 0;
    hipError_t e;
    switch (nbuf) {
    case 3: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_kernel<KT, 3, D>, 64 * kDecWaves, 0); break;
    case 4: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_kernel<KT, 4, D>, 64 * kDecWaves, 0); break;
    default: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_kernel_lean<KT, D>, 64 * kDecWaves, 0); break;
    }
    return e == hipSuccess ? per_cu : 0;
}

int decode_resident_workgroups(int kv_dtype, int nbuf, int head_dim)
{
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        return 0;
    int per_cu;
    if (head_dim == 64) per_cu = kv_dtype == TS_FP8_E4M3 ? resident_t<uint8_t, 64>(nbuf) : resident_t<uint16_t, 64>(nbuf);
    else per_cu = kv_dtype == TS_FP8_E4M3 ? resident_t<uint8_t, 128>(nbuf) : resident_t<uint16_t, 128>(nbuf);
    return cus * per_cu;
}

int launch_decode(const AttnArgs& a, void* stream)
{
    if (a.n_dec <= 0) return (int)hipSuccess;
    if ((a.geo.D != 128 && a.geo.D != 64) || a.geo.q_dtype != TS_BF16) return (int)hipErrorInvalidValue;
    hipStream_t st = (hipStream_t)stream;
    if (a.geo.kv_dtype == TS_BF16) return a.geo.D == 64 ? launch_decode_t<uint16_t, 64>(a, st) : launch_decode_t<uint16_t, 128>(a, st);
    if (a.geo.kv_dtype == TS_FP8_E4M3) return a.geo.D == 64 ? launch_decode_t<uint8_t, 64>(a, st) : launch_decode_t<uint8_t, 128>(a, st);
    return (int)hipErrorInvalidValue;
}

template <typename KT, int D>
static int launch_fused_t(const AttnArgs& a, const SmallLists& s, hipStream_t st)
{
    dim3 grid((unsigned)s.n_dec * (unsigned)a.geo.Hkv), block(64 * kDecWaves);
    hipLaunchKernelGGL((decode_kernel_fused<KT, D>), grid, block, 0, st, a, s);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || s.n_cmb <= 0) return (int)e;
    dim3 cgrid((unsigned)s.n_cmb, (unsigned)a.geo.Hq), cblock((unsigned)a.geo.D);
    hipLaunchKernelGGL(combine_kernel_small, cgrid, cblock, 0, st, a, s);
    return (int)hipGetLastError();
}

int launch_decode_fused(const AttnArgs& a, const SmallLists& s, void* stream)
{
    if (s.n_dec <= 0) return (int)hipSuccess;
    if (s.n_dec > kSmallDec || s.n_cmb > kSmallCmb || !a.k_new || !a.v_new || a.cmb_ctr) return (int)hipErrorInvalidValue;
    if ((a.geo.D != 128 && a.geo.D != 64) || a.geo.q_dtype != TS_BF16) return (int)hipErrorInvalidValue;
    hipStream_t st = (hipStream_t)stream;
    if (a.geo.kv_dtype == TS_BF16) return a.geo.D == 64 ? launch_fused_t<uint16_t, 64>(a, s, st) : launch_fused_t<uint16_t, 128>(a, s, st);
    if (a.geo.kv_dtype == TS_FP8_E4M3) return a.geo.D == 64 ? launch_fused_t<uint8_t, 64>(a, s, st) : launch_fused_t<uint8_t, 128>(a, s, st);
    return (int)hipErrorInvalidValue;
}

int launch_combine(const AttnArgs& a, void* stream)
{
    if (a.n_cmb <= 0) return (int)hipSuccess;
    dim3 grid((unsigned)a.n_cmb, (unsigned)a.geo.Hq), block((unsigned)a.geo.D);
    hipLaunchKernelGGL(combine_kernel, grid, block, 0, (hipStream_t)stream, a);
    return (int)hipGetLastError();
}

}  // namespace ts
