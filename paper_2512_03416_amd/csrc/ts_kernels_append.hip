// Step a1: write the iteration's new K/V rows into the paged cache.
//
// Prefill builds cache entries for all input tokens, a decode iteration adds the entry of the
// last token (paper Sec. 2.1); in a Convertible Decoder both kinds of rows arrive in one batch
// (Sec. 3.4).  One workgroup per new token: it finds the token's sequence, position, page and
// slot, then scatters the token's Hkv x D values of K (as 16-byte dim-chunks) and of V
// (token-fastest tile) into place, converting to the cache element type on the way.
#include "ts_device.h"

namespace ts {

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const void* p, int64_t i) { return ((const float*)p)[i]; }
};
template <> struct Elem<uint16_t> {
    static __device__ __forceinline__ float load(const void* p, int64_t i)
    { return bf16_bits_to_float(((const uint16_t*)p)[i]); }
};

// SRC: element type of k_new/v_new (float or uint16_t holding bf16 bits).
// DST: cache element type (float, uint16_t bf16 bits, uint8_t e4m3).
template <typename SRC, typename DST>
__global__ __launch_bounds__(256) void append_kernel(AppendArgs a)
{
    const int row = blockIdx.x;
    const int Hkv = a.geo.Hkv, D = a.geo.D;
    // sequence of this row: last s with q_off[s] <= row  (empty sequences share the offset of the
    // next one and are skipped by taking the last match)
    int lo = 0, hi = a.num_seqs;                   // invariant: q_off[lo] <= row < q_off[hi]
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (a.seqs[mid].q_off <= row) lo = mid; else hi = mid;
    }
    const SeqMeta m = a.seqs[lo];
    const int pos = m.prefix + (row - m.q_off);
    const int64_t page = a.block_table[(int64_t)lo * a.geo.max_pages + (pos >> 4)];
    const int slot = pos & 15;
    constexpr int X = 16 / (int)sizeof(DST);       // elements per 16-byte dim-chunk
    const int n_elems = Hkv * D;
    const SRC* ks = (const SRC*)a.k_new + (int64_t)row * n_elems;
    const SRC* vs = (const SRC*)a.v_new + (int64_t)row * n_elems;
    DST* kc = (DST*)a.k_cache;
    DST* vc = (DST*)a.v_cache;
    for (int e = threadIdx.x; e < n_elems; e += blockDim.x) {
        const int g = e / D, dim = e - g * D;
        const int64_t tile = tile_elem_base(page, Hkv, g, D);
        const int64_t kidx = tile + (dim / X) * (kPage * X) + slot * X + (dim % X);
        const int64_t vidx = tile + dim * kPage + slot;
        if constexpr (sizeof(DST) == 1) {
            const float kf = Elem<SRC>::load(ks, e) / a.k_scale[g];
            const float vf = Elem<SRC>::load(vs, e) / a.v_scale[g];
            kc[kidx] = (uint8_t)float_to_e4m3_bits(kf);
            vc[vidx] = (uint8_t)float_to_e4m3_bits(vf);
        } else {
            kc[kidx] = (DST)ks[e];                 // same element type: plain copy of the bits
            vc[vidx] = (DST)vs[e];
        }
    }
}

int launch_append(const AppendArgs& a, void* stream)
{
    if (a.total_tokens <= 0) return (int)hipSuccess;
    dim3 grid((unsigned)a.total_tokens), block(256);
    hipStream_t st = (hipStream_t)stream;
    if (a.geo.q_dtype == TS_F32 && a.geo.kv_dtype == TS_F32)
        hipLaunchKernelGGL((append_kernel<float, float>), grid, block, 0, st, a);
    else if (a.geo.q_dtype == TS_BF16 && a.geo.kv_dtype == TS_BF16)
        hipLaunchKernelGGL((append_kernel<uint16_t, uint16_t>), grid, block, 0, st, a);
    else if (a.geo.q_dtype == TS_BF16 && a.geo.kv_dtype == TS_FP8_E4M3)
        hipLaunchKernelGGL((append_kernel<uint16_t, uint8_t>), grid, block, 0, st, a);
    else
        return (int)hipErrorInvalidValue;
    return (int)hipGetLastError();
}

}  // namespace ts
