// Step a3: launcher of the prefill-tile kernel.
#include "ts_prefill_tile.h"

namespace ts {

// (held to 192 vector registers per lane like the resident form: the attribute counts in units of two)
template <typename KT, bool WIDE, int D>
__global__ __launch_bounds__(kPfThreads) __attribute__((amdgpu_num_vgpr(96))) void prefill_kernel(AttnArgs a)
{
    __shared__ PfLdsT<D> lds;
    const int32_t TS_CONSTANT* slot = as_constant((const int32_t*)(a.pfmap + blockIdx.x));
    const int item_idx = slot[0], g = slot[1];
    if (item_idx < 0) return;                               // padding of the die-aware launch order
    prefill_tile<KT, WIDE, D>(a, item_idx, g, lds, threadIdx.x);
}

// fp8 caches: bf16 copies of the pages the prefill tiles will read, one workgroup per (page, KV head).  The
// copies keep the tile order of a bf16 cache -- K as 16-byte chunks of 8 dims [D/8][16 slots][8], V
// token-fastest [D][16 slots] -- so the tile kernel copies them into LDS exactly like bf16 cache pages.  Every
// e4m3 value is a bf16 value: the conversion is exact, and pages are copied whole (slots past the end of the
// sequence hold whatever the cache holds; the tile kernel masks them as it does for a bf16 cache).
template <int D>
__global__ __launch_bounds__(256) void widen_kernel(AttnArgs a, uint16_t* __restrict__ wk, uint16_t* __restrict__ wv)
{
    const int Hkv = a.geo.Hkv;
    constexpr int TB = 16 * D;                                 // bytes of an e4m3 tile = elements of a tile
    const int item = blockIdx.x / Hkv, g = blockIdx.x % Hkv;
    const int32_t TS_CONSTANT* w = as_constant((const int32_t*)(a.wide + item));
    const int seq = w[0], pidx = w[1];
    const int64_t page = as_constant(a.block_table)[(int64_t)seq * a.geo.max_pages + pidx];
    const uint8_t* ks = (const uint8_t*)a.k_cache + (page * Hkv + g) * TB;
    const uint8_t* vs = (const uint8_t*)a.v_cache + (page * Hkv + g) * TB;
    uint16_t* kd = wk + ((int64_t)item * Hkv + g) * TB;
    uint16_t* vd = wv + ((int64_t)item * Hkv + g) * TB;
    const int t = threadIdx.x;
    if (t >= TB / 8) return;
    // thread t takes 8 consecutive bytes of each tile.  K: bytes of chunk (c16 = t / 32, slot = (t / 2) % 16),
    // dims 16 c16 + 8 (t % 2) .. + 7 -> bf16 chunk (2 c16 + t % 2, slot).  V: elements 8 t .. 8 t + 7 keep their place.
    const uint2 kb = *(const uint2*)(ks + t * 8);
    const uint2 vb = *(const uint2*)(vs + t * 8);
    const int c16 = t >> 5, slot = (t >> 1) & 15, half = t & 1;
    const uint2 k0 = fp8x4_bf16x4(kb.x), k1 = fp8x4_bf16x4(kb.y);
    const uint2 v0 = fp8x4_bf16x4(vb.x), v1 = fp8x4_bf16x4(vb.y);
    *(uint4*)(kd + ((2 * c16 + half) * 16 + slot) * 8) = make_uint4(k0.x, k0.y, k1.x, k1.y);
    *(uint4*)(vd + t * 8) = make_uint4(v0.x, v0.y, v1.x, v1.y);
}

// Merge of the parts of a tile that was cut along the keys, in part order:
//   M = max m_i,  out = sum o_i 2^(m_i - M) / sum l_i 2^(m_i - M)  (times the V scale of an fp8 cache).
// One workgroup per (cut tile, KV head, 32 rows); D / 4 lanes hold the dims of a row.  The
// partial rows of up to eight parts are requested together, then added one after the other (the sums keep
// their order).
constexpr int kPfCmbRows = 32;
template <int D>
__global__ __launch_bounds__(256) void prefill_combine_kernel(AttnArgs a)
{
    constexpr int kBatch = 8, kGroups = kPfPartRows / kPfCmbRows;
    constexpr int kLanes = D / 4, kSub = 256 / kLanes;           // lanes per row (4 dims each), rows per step
    const int Hkv = a.geo.Hkv, G = a.geo.G, Hq = a.geo.Hq;
    const int grp = blockIdx.x % kGroups, g = (blockIdx.x / kGroups) % Hkv, ci = blockIdx.x / (kGroups * Hkv);
    const int32_t TS_CONSTANT* c = as_constant((const int32_t*)(a.pfcmb + ci));
    const int item = c[0], part0 = c[1], n_part = c[2];
    const int32_t TS_CONSTANT* it = as_constant((const int32_t*)(a.pf + item));
    const int row0 = it[1], tok_begin = it[4], tok_count = it[5];
    const float vscale = a.geo.kv_dtype == TS_FP8_E4M3 ? a.v_scale[g] : 1.0f;
    const int lane = threadIdx.x % kLanes, sub = threadIdx.x / kLanes;
    const int64_t part_step = (int64_t)Hkv * kPfPartRows;          // rows between two parts of one (tile, head)
#pragma unroll
    for (int step = 0; step < kPfCmbRows / kSub; ++step) {
        const int rho = grp * kPfCmbRows + step * kSub + sub;
        const int t = rho / G, hd = rho - t * G;
        if (t >= tok_count) continue;
        const int64_t slot0 = ((int64_t)part0 * Hkv + g) * kPfPartRows + rho;
        float M = -INFINITY;
        for (int k = 0; k < n_part; ++k) M = fmaxf(M, a.pf_part_ml[(slot0 + k * part_step) * 2]);
        f32x4 o = {0.f, 0.f, 0.f, 0.f};
        float L = 0.f;
        for (int k0 = 0; k0 < n_part; k0 += kBatch) {
            float2 ml[kBatch];
            f32x4 v[kBatch];
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                const int64_t slot = slot0 + min(k0 + j, n_part - 1) * part_step;
                ml[j] = *(const float2*)(a.pf_part_ml + slot * 2);
                v[j] = *(const f32x4*)(a.pf_part_o + slot * D + 4 * lane);
            }
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                if (k0 + j < n_part) {
                    const float w = __builtin_amdgcn_exp2f(ml[j].x - M);
                    L += ml[j].y * w;
                    o += v[j] * w;
                }
            }
        }
        const float inv = vscale / L;
        uint2 w;
        w.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{o[0] * inv, o[1] * inv}, bf16x2));
        w.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{o[2] * inv, o[3] * inv}, bf16x2));
        *(uint2*)((uint16_t*)a.out + ((int64_t)(row0 + tok_begin + t) * Hq + g * G + hd) * D + 4 * lane) = w;
    }
}

int launch_prefill_combine(const AttnArgs& a, void* stream)
{
    if (a.n_pfcmb <= 0) return (int)hipSuccess;
    if ((a.geo.D != 128 && a.geo.D != 64) || !a.pf_part_o || !a.pf_part_ml) return (int)hipErrorInvalidValue;
    const unsigned grid = (unsigned)a.n_pfcmb * (unsigned)a.geo.Hkv * (unsigned)(kPfPartRows / kPfCmbRows);
    if (a.geo.D == 64) hipLaunchKernelGGL(prefill_combine_kernel<64>, dim3(grid), dim3(256), 0, (hipStream_t)stream, a);
    else hipLaunchKernelGGL(prefill_combine_kernel<128>, dim3(grid), dim3(256), 0, (hipStream_t)stream, a);
    return (int)hipGetLastError();
}

int launch_widen(const AttnArgs& a, void* wide_k, void* wide_v, void* stream)
{
    if (a.n_wide <= 0) return (int)hipSuccess;
    if ((a.geo.D != 128 && a.geo.D != 64) || a.geo.kv_dtype != TS_FP8_E4M3 || !wide_k || !wide_v) return (int)hipErrorInvalidValue;
    const dim3 grid((unsigned)a.n_wide * (unsigned)a.geo.Hkv);
    if (a.geo.D == 64) hipLaunchKernelGGL(widen_kernel<64>, grid, dim3(256), 0, (hipStream_t)stream, a, (uint16_t*)wide_k, (uint16_t*)wide_v);
    else hipLaunchKernelGGL(widen_kernel<128>, grid, dim3(256), 0, (hipStream_t)stream, a, (uint16_t*)wide_k, (uint16_t*)wide_v);
    return (int)hipGetLastError();
}

int launch_prefill(const AttnArgs& a, void* stream)
{
    if (a.n_pf <= 0) return (int)hipSuccess;
    if ((a.geo.D != 128 && a.geo.D != 64) || a.geo.q_dtype != TS_BF16) return (int)hipErrorInvalidValue;
    dim3 grid((unsigned)a.n_pfmap), block(kPfThreads);
    hipStream_t st = (hipStream_t)stream;
    // (an fp8 cache whose pages were widened beforehand is read through the bf16 form; head dim 64 has no other)
    if (a.geo.D == 64) {
        if (a.geo.kv_dtype == TS_BF16) hipLaunchKernelGGL((prefill_kernel<uint16_t, false, 64>), grid, block, 0, st, a);
        else if (a.geo.kv_dtype == TS_FP8_E4M3 && a.wide_base) hipLaunchKernelGGL((prefill_kernel<uint16_t, true, 64>), grid, block, 0, st, a);
        else return (int)hipErrorInvalidValue;
    }
    else if (a.geo.kv_dtype == TS_BF16) hipLaunchKernelGGL((prefill_kernel<uint16_t, false, 128>), grid, block, 0, st, a);
    else if (a.geo.kv_dtype == TS_FP8_E4M3 && a.wide_base) hipLaunchKernelGGL((prefill_kernel<uint16_t, true, 128>), grid, block, 0, st, a);
    else if (a.geo.kv_dtype == TS_FP8_E4M3) hipLaunchKernelGGL((prefill_kernel<uint8_t, false, 128>), grid, block, 0, st, a);
    else return (int)hipErrorInvalidValue;
    return (int)hipGetLastError();
}

}  // namespace ts
