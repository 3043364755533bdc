// Step a2 (+a4): split-K decode attention over the paged cache, and the merge of the splits.
//
// A decode row reads its whole cached context once and does ~2*G flops per cache element, so
// the scan is bound by HBM bandwidth (the paper's "memory-intensive decode" whose spare compute
// lets a decoder absorb prefill work, Sec. 1, Sec. 3.4).  The kernel is therefore built around
// the loads:
//   - one wavefront owns one item = (decode row, KV head, range of <= 128 pages); no LDS, no
//     barriers, so many independent waves per CU keep loads in flight;
//   - every (page, KV head) tile is one contiguous 4 KB (bf16) / 2 KB (fp8) block; each load
//     instruction of the wave reads a contiguous 1 KB (K) or 512 B / 256 B (V) run of it, already
//     in matrix-operand order, straight into registers;
//   - NBUF tiles are in flight per wave (register ring, unconditional prefetch so the hardware
//     load counter is statically known);
//   - the G query heads of the KV head's group ride along as columns of the same MFMA
//     (S^T = K Q^T, 16 tokens x 16 columns), so each K/V byte is loaded once for the group;
//   - the accumulator layout of S^T is the B-operand layout of the next MFMA (O^T += V^T P^T),
//     so the softmax weights never leave registers; the only cross-lane traffic is a 2-step
//     reduction of the running maximum when it grows, and of the sum at the end.
// Online softmax keeps a reference maximum per head in log2 units; it is raised only when a page
// exceeds it by more than kRaise (any reference gives the same quotient, the bound only guards
// the fp32 range), which removes the accumulator rescale from almost every page.
#include "ts_device.h"

namespace ts {

constexpr float kRaise = 16.0f;   // log2 units: weights stay below 2^16 relative to the reference

template <typename KT> struct KVTile;
template <> struct KVTile<uint16_t> { uint4 k[4]; uint2 v[8]; };
template <> struct KVTile<uint8_t>  { uint4 k[2]; uint32_t v[8]; };

__device__ __forceinline__ void load_tile(KVTile<uint16_t>& t, const char* kc, const char* vc,
                                          int64_t tile, int lane)
{
    const char* kt = kc + tile * 4096 + lane * 16;
    const char* vt = vc + tile * 4096 + (lane & 15) * 32 + (lane >> 4) * 8;
#pragma unroll
    for (int b = 0; b < 4; ++b) t.k[b] = *(const uint4*)(kt + b * 1024);
#pragma unroll
    for (int b = 0; b < 8; ++b) t.v[b] = *(const uint2*)(vt + b * 512);
}

__device__ __forceinline__ void load_tile(KVTile<uint8_t>& t, const char* kc, const char* vc,
                                          int64_t tile, int lane)
{
    const char* kt = kc + tile * 2048 + lane * 16;
    const char* vt = vc + tile * 2048 + (lane & 15) * 16 + (lane >> 4) * 4;
#pragma unroll
    for (int b = 0; b < 2; ++b) t.k[b] = *(const uint4*)(kt + b * 1024);
#pragma unroll
    for (int b = 0; b < 8; ++b) t.v[b] = *(const uint32_t*)(vt + b * 256);
}

// four e4m3 bytes -> four bf16 (exact: every e4m3 value is a bf16 value)
__device__ __forceinline__ uint2 fp8x4_to_bf16x4(uint32_t w)
{
    const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, false);
    const f32x2 hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, true);
    uint2 r;
    r.x = __builtin_amdgcn_perm(__float_as_uint(lo.y), __float_as_uint(lo.x), 0x07060302u);
    r.y = __builtin_amdgcn_perm(__float_as_uint(hi.y), __float_as_uint(hi.x), 0x07060302u);
    return r;
}

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ s16x4 as_s16x4(uint2 v) { return __builtin_bit_cast(s16x4, v); }

// S^T (16 tokens x 16 columns) = K tile x Q^T for one page
__device__ __forceinline__ f32x4 qk_tile(const KVTile<uint16_t>& t, const bf16x8* qb)
{
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int b = 0; b < 4; ++b)
        s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(t.k[b]), qb[b], s, 0, 0, 0);
    return s;
}
__device__ __forceinline__ f32x4 qk_tile(const KVTile<uint8_t>& t, const bf16x8* qb)
{
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const uint2 a0 = fp8x4_to_bf16x4(t.k[j].x), a1 = fp8x4_to_bf16x4(t.k[j].y);
        const uint2 a2 = fp8x4_to_bf16x4(t.k[j].z), a3 = fp8x4_to_bf16x4(t.k[j].w);
        s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(make_uint4(a0.x, a0.y, a1.x, a1.y)),
                                                    qb[2 * j], s, 0, 0, 0);
        s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(make_uint4(a2.x, a2.y, a3.x, a3.y)),
                                                    qb[2 * j + 1], s, 0, 0, 0);
    }
    return s;
}

__device__ __forceinline__ uint2 v_operand(const KVTile<uint16_t>& t, int b) { return t.v[b]; }
__device__ __forceinline__ uint2 v_operand(const KVTile<uint8_t>& t, int b) { return fp8x4_to_bf16x4(t.v[b]); }

// dims held by k-block b of the Q operand for lane group r (must mirror the K tile order)
template <typename KT> __device__ __forceinline__ int q_dim0(int b, int r)
{
    if constexpr (sizeof(KT) == 2) return 8 * (4 * b + r);
    else return 16 * (4 * (b >> 1) + r) + 8 * (b & 1);
}

template <typename KT, int NBUF>
__global__ __launch_bounds__(64) void decode_kernel(AttnArgs a)
{
    constexpr int D = 128, KB = 4, DB = 8;
    const DecItem it = a.dec[blockIdx.x];
    const int g = blockIdx.y;
    const int lane = threadIdx.x, r = lane >> 4, n = lane & 15;
    const int Hq = a.geo.Hq, Hkv = a.geo.Hkv, G = a.geo.G;

    // Q^T operand: column n is query head g*G + n; columns >= G repeat the group's last head
    // (their results are finite and never stored)
    bf16x8 qb[KB];
    {
        const uint16_t* qrow = (const uint16_t*)a.q + ((int64_t)it.row * Hq + g * G + min(n, G - 1)) * D;
#pragma unroll
        for (int b = 0; b < KB; ++b) qb[b] = as_bf16x8(*(const uint4*)(qrow + q_dim0<KT>(b, r)));
    }
    const float kscale = (sizeof(KT) == 1) ? a.k_scale[g] : 1.0f;
    const float c = a.sm_scale * kscale * kLog2e;

    // page ids of this item: lane j holds the id of the item's page j (and j + 64)
    const int np = it.page_end - it.page_begin;
    const int32_t* bt = a.block_table + (int64_t)it.seq * a.geo.max_pages + it.page_begin;
    const int ids0 = bt[min(lane, np - 1)];
    const int ids1 = bt[min(lane + 64, np - 1)];
    auto tile_of = [&](int pi) -> int64_t {
        pi = min(pi, np - 1);
        const int id = (pi < 64) ? __builtin_amdgcn_readlane(ids0, pi) : __builtin_amdgcn_readlane(ids1, pi - 64);
        return (int64_t)id * Hkv + g;
    };

    const char* kc = (const char*)a.k_cache;
    const char* vc = (const char*)a.v_cache;
    KVTile<KT> buf[NBUF];
#pragma unroll
    for (int j = 0; j < NBUF; ++j) load_tile(buf[j], kc, vc, tile_of(j), lane);

    f32x4 acc[DB];
#pragma unroll
    for (int b = 0; b < DB; ++b) acc[b] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_ref = -INFINITY, l = 0.0f;

    for (int base = 0; base < np; base += NBUF) {
#pragma unroll
        for (int j = 0; j < NBUF; ++j) {
            const int pi = base + j;
            if (pi < np) {                                        // wave-uniform
                const KVTile<KT>& t = buf[j];
                f32x4 s = qk_tile(t, qb);
                float t0 = s[0] * c, t1 = s[1] * c, t2 = s[2] * c, t3 = s[3] * c;
                const int tok0 = (it.page_begin + pi) * kPage + 4 * r;
                const int nvalid = it.n_keys - tok0;              // tokens tok0 .. tok0+3 valid if < nvalid
                const bool tail = (it.page_begin + pi + 1) * kPage > it.n_keys;   // wave-uniform
                if (tail) {
                    t0 = nvalid > 0 ? t0 : -INFINITY; t1 = nvalid > 1 ? t1 : -INFINITY;
                    t2 = nvalid > 2 ? t2 : -INFINITY; t3 = nvalid > 3 ? t3 : -INFINITY;
                }
                const float lmax = fmaxf(fmaxf(t0, t1), fmaxf(t2, t3));
                if (__any(lmax > m_ref + kRaise)) {               // raise the reference (rare)
                    float full = fmaxf(lmax, __shfl_xor(lmax, 16, 64));
                    full = fmaxf(full, __shfl_xor(full, 32, 64));
                    const float m_new = fmaxf(m_ref, full);
                    const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);     // exp2(-inf) = 0 on the first page
#pragma unroll
                    for (int b = 0; b < DB; ++b) acc[b] *= alpha;
                    l *= alpha;
                    m_ref = m_new;
                }
                const float p0 = __builtin_amdgcn_exp2f(t0 - m_ref), p1 = __builtin_amdgcn_exp2f(t1 - m_ref);
                const float p2 = __builtin_amdgcn_exp2f(t2 - m_ref), p3 = __builtin_amdgcn_exp2f(t3 - m_ref);
                l += (p0 + p1) + (p2 + p3);
                const bf16x2 pa = __builtin_convertvector(f32x2{p0, p1}, bf16x2);
                const bf16x2 pb = __builtin_convertvector(f32x2{p2, p3}, bf16x2);
                uint2 pw;
                pw.x = __builtin_bit_cast(uint32_t, pa);
                pw.y = __builtin_bit_cast(uint32_t, pb);
                const s16x4 pv = as_s16x4(pw);
                uint64_t keep = ~0ull;                            // zero V of slots past n_keys (poison)
                if (tail) keep = nvalid >= 4 ? ~0ull : (nvalid <= 0 ? 0ull : ((1ull << (16 * nvalid)) - 1ull));
#pragma unroll
                for (int b = 0; b < DB; ++b) {
                    uint2 vv = v_operand(t, b);
                    if (tail) { vv.x &= (uint32_t)keep; vv.y &= (uint32_t)(keep >> 32); }
                    acc[b] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(as_s16x4(vv), pv, acc[b], 0, 0, 0);
                }
            }
            load_tile(buf[j], kc, vc, tile_of(pi + NBUF), lane);  // refill (clamped to the last page)
        }
    }

    float l_tot = l + __shfl_xor(l, 16, 64);
    l_tot += __shfl_xor(l_tot, 32, 64);
    if (n < G) {
        const int h = g * G + n;
        if (it.part < 0) {
            const float vscale = (sizeof(KT) == 1) ? a.v_scale[g] : 1.0f;
            const float inv = vscale / l_tot;
            uint16_t* o = (uint16_t*)a.out + ((int64_t)it.row * Hq + h) * D + 4 * r;
#pragma unroll
            for (int b = 0; b < DB; ++b) {
                const bf16x2 x = __builtin_convertvector(f32x2{acc[b][0] * inv, acc[b][1] * inv}, bf16x2);
                const bf16x2 y = __builtin_convertvector(f32x2{acc[b][2] * inv, acc[b][3] * inv}, bf16x2);
                uint2 w;
                w.x = __builtin_bit_cast(uint32_t, x);
                w.y = __builtin_bit_cast(uint32_t, y);
                *(uint2*)(o + 16 * b) = w;
            }
        } else {
            float* o = a.part_o + ((int64_t)it.part * Hq + h) * D + 4 * r;
#pragma unroll
            for (int b = 0; b < DB; ++b) *(f32x4*)(o + 16 * b) = acc[b];
            if (r == 0) {
                float* ml = a.part_ml + ((int64_t)it.part * Hq + h) * 2;
                ml[0] = m_ref;
                ml[1] = l_tot;
            }
        }
    }
}

// Merge of a row's splits, in split order:  M = max m_i, out = sum o_i 2^(m_i-M) / sum l_i 2^(m_i-M).
__global__ __launch_bounds__(128) void combine_kernel(AttnArgs a)
{
    const CmbItem it = a.cmb[blockIdx.x];
    const int h = blockIdx.y, d = threadIdx.x;
    const int Hq = a.geo.Hq, D = a.geo.D;
    float M = -INFINITY;
    for (int k = 0; k < it.n_split; ++k)
        M = fmaxf(M, a.part_ml[((int64_t)(it.part_begin + k) * Hq + h) * 2]);
    float o = 0.0f, L = 0.0f;
    for (int k = 0; k < it.n_split; ++k) {
        const int64_t p = (int64_t)(it.part_begin + k) * Hq + h;
        const float w = __builtin_amdgcn_exp2f(a.part_ml[p * 2] - M);
        L += a.part_ml[p * 2 + 1] * w;
        o += a.part_o[p * D + d] * w;
    }
    const float vscale = (a.geo.kv_dtype == TS_FP8_E4M3) ? a.v_scale[h / a.geo.G] : 1.0f;
    ((uint16_t*)a.out)[((int64_t)it.row * Hq + h) * D + d] = (uint16_t)float_to_bf16_bits(o * vscale / L);
}

static int g_decode_nbuf = 3;
void set_decode_nbuf(int n) { g_decode_nbuf = n; }

template <typename KT>
static int launch_decode_t(const AttnArgs& a, hipStream_t st)
{
    dim3 grid((unsigned)a.n_dec, (unsigned)a.geo.Hkv), block(64);
    switch (g_decode_nbuf) {
    case 2: hipLaunchKernelGGL((decode_kernel<KT, 2>), grid, block, 0, st, a); break;
    case 4: hipLaunchKernelGGL((decode_kernel<KT, 4>), grid, block, 0, st, a); break;
    default: hipLaunchKernelGGL((decode_kernel<KT, 3>), grid, block, 0, st, a); break;
    }
    return (int)hipGetLastError();
}

int launch_decode(const AttnArgs& a, void* stream)
{
    if (a.n_dec <= 0) return (int)hipSuccess;
    if (a.geo.D != 128 || a.geo.q_dtype != TS_BF16) return (int)hipErrorInvalidValue;
    hipStream_t st = (hipStream_t)stream;
    if (a.geo.kv_dtype == TS_BF16) return launch_decode_t<uint16_t>(a, st);
    if (a.geo.kv_dtype == TS_FP8_E4M3) return launch_decode_t<uint8_t>(a, st);
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
