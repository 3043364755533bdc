// Step a2: decode attention over the paged cache, as a device function shared by the decode
// kernel and the persistent mixed kernel.
//
// A decode row reads its whole cached context once and does ~2*G flops per cache element, so
// the scan is bound by HBM bandwidth (the paper's "memory-intensive decode" whose spare compute
// lets a decoder absorb prefill work, Sec. 1, Sec. 3.4).  The kernel is therefore built around
// the loads:
//   - one workgroup of 4 wavefronts owns one item = (decode row, KV head, page range), the waves
//     taking every 4th page; they share nothing until the end of the item, so many independent
//     waves per CU keep loads in flight;
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
#pragma once
#include <type_traits>

#include "ts_device.h"

namespace ts {

constexpr float kRaise = 16.0f;   // log2 units: weights stay below 2^16 relative to the reference

// One (page, KV head) tile in registers, D = head dim (64 or 128): K as 1 KB runs, V as 16-dim blocks.
template <typename KT, int D> struct KVTile;
template <int D> struct KVTile<uint16_t, D> { uint4 k[D / 32]; uint2 v[D / 16]; };
template <int D> struct KVTile<uint8_t, D>  { uint4 k[D / 64]; uint32_t v[D / 16]; };

// Tiles are read with the non-temporal hint: the scan touches every byte once, and keeping it out
// of the L2's replacement traffic raised the rate from 5.9 to 6.45 TB/s (bf16; fp8: 5.9 to 6.3).
template <int D>
__device__ __forceinline__ void load_tile(KVTile<uint16_t, D>& t, const char* kc, const char* vc,
                                          int64_t tile, int lane)
{
    const char* kt = kc + tile * (32 * D) + lane * 16;
    const char* vt = vc + tile * (32 * D) + (lane & 15) * 32 + (lane >> 4) * 8;
#pragma unroll
    for (int b = 0; b < D / 32; ++b) t.k[b] = load_nt4(kt + b * 1024);
#pragma unroll
    for (int b = 0; b < D / 16; ++b) t.v[b] = load_nt2(vt + b * 512);
}

template <int D>
__device__ __forceinline__ void load_tile(KVTile<uint8_t, D>& t, const char* kc, const char* vc,
                                          int64_t tile, int lane)
{
    const char* kt = kc + tile * (16 * D) + lane * 16;
    const char* vt = vc + tile * (16 * D) + (lane & 15) * 16 + (lane >> 4) * 4;
#pragma unroll
    for (int b = 0; b < D / 64; ++b) t.k[b] = load_nt4(kt + b * 1024);
#pragma unroll
    for (int b = 0; b < D / 16; ++b) t.v[b] = __builtin_nontemporal_load((const uint32_t*)(vt + b * 256));
}

// four e4m3 bytes -> four bf16 (exact: every e4m3 value is a bf16 value): one packed conversion per pair
__device__ __forceinline__ uint2 fp8x4_to_bf16x4(uint32_t w)
{
    uint2 r;
    r.x = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, false));
    r.y = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, true));
    return r;
}

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ s16x4 as_s16x4(uint2 v) { return __builtin_bit_cast(s16x4, v); }

// S^T (16 tokens x 16 columns) = K tile x Q^T for one page
template <int D>
__device__ __forceinline__ f32x4 qk_tile(const KVTile<uint16_t, D>& t, const bf16x8* qb)
{
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int b = 0; b < D / 32; ++b)
        s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(t.k[b]), qb[b], s, 0, 0, 0);
    return s;
}
template <int D>
__device__ __forceinline__ f32x4 qk_tile(const KVTile<uint8_t, D>& t, const bf16x8* qb)
{
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < D / 64; ++j) {
        const uint2 a0 = fp8x4_to_bf16x4(t.k[j].x), a1 = fp8x4_to_bf16x4(t.k[j].y);
        const uint2 a2 = fp8x4_to_bf16x4(t.k[j].z), a3 = fp8x4_to_bf16x4(t.k[j].w);
        s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(make_uint4(a0.x, a0.y, a1.x, a1.y)),
                                                    qb[2 * j], s, 0, 0, 0);
        s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(make_uint4(a2.x, a2.y, a3.x, a3.y)),
                                                    qb[2 * j + 1], s, 0, 0, 0);
    }
    return s;
}

template <int D> __device__ __forceinline__ uint2 v_operand(const KVTile<uint16_t, D>& t, int b) { return t.v[b]; }
template <int D> __device__ __forceinline__ uint2 v_operand(const KVTile<uint8_t, D>& t, int b) { return fp8x4_to_bf16x4(t.v[b]); }

// dims held by k-block b of the Q operand for lane group r (must mirror the K tile order)
template <typename KT> __device__ __forceinline__ int q_dim0(int b, int r)
{
    if constexpr (sizeof(KT) == 2) return 8 * (4 * b + r);
    else return 16 * (4 * (b >> 1) + r) + 8 * (b & 1);
}

// One workgroup of kDecWaves waves per item = (decode row, KV head, page range).  Wave w streams the
// pages begin+w, begin+w+kDecWaves, ... so the waves read neighbouring tiles at the same time; at
// the end their (max, sum, O) states meet in LDS and wave 0 merges them in wave order.  A row that
// fits one item is finished here (no partial ever goes to HBM: stores into the middle of a saturated
// read stream were measured to cost ~10x their byte share); only rows longer than one workgroup's
// fair share are cut into several items whose partials go through combine_kernel.
constexpr int kDecWaves = 4;               // stand-alone decode kernel; the mixed kernel uses 8

template <int WAVES, int D = 128>
struct DecMerge {                          // LDS image of the non-leading waves' state
    float o[WAVES - 1][D / 16][64][4];     // acc[b] of every lane
    float m[WAVES - 1][16];
    float l[WAVES - 1][16];
};

// An item of the device work list, through the scalar cache.
__device__ __forceinline__ DecItem load_dec_item(const DecItem* p)
{
    const int32_t TS_CONSTANT* w = as_constant((const int32_t*)p);
    return DecItem{w[0], w[1], w[2], w[3], w[4], w[5], w[6], w[7]};
}

// One decode item for KV head g, executed by a workgroup of WAVES waves.  All waves must call
// it; it contains one workgroup barrier, and the caller must place another barrier before mg is
// reused.
// MERGE: the code for merging a split row by its last item is compiled in (it is used when a.cmb_ctr is set).
// FUSED: the row's new token comes from a.k_new / a.v_new and is written into the cache here (see AttnArgs).
template <typename KT, int NBUF, int WAVES, int D = 128, bool MERGE = false, bool FUSED = false>
__device__ __forceinline__ void decode_item(const AttnArgs& a, const DecItem it, int g, DecMerge<WAVES, D>& mg)
{
    constexpr int KB = D / 32, DB = D / 16;    // 32-dim steps of K Q^T, 16-dim blocks of O^T
    const int it_row = it.row, it_seq = it.seq, it_keys = it.n_keys, it_pb = it.page_begin, it_pe = it.page_end, it_part = it.part;
    const int it_cmb = MERGE ? it.cmb : -1, it_part_first = MERGE ? it.part_first : -1;
    // (readfirstlane tells the compiler the wave index is uniform, which keeps everything derived
    // from it -- the page-id loads above all -- on the scalar unit)
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63, r = lane >> 4, n = lane & 15;
    const int Hq = a.geo.Hq, Hkv = a.geo.Hkv, G = a.geo.G;

    // this wave's pages: it_pb + wave + WAVES * k, k = 0 .. np-1
    const int np = max(0, (it_pe - it_pb - wave + WAVES - 1) / WAVES);
    const int32_t TS_CONSTANT* bt = as_constant(a.block_table) + (int64_t)it_seq * a.geo.max_pages + it_pb + wave;

    f32x4 acc[DB];
#pragma unroll
    for (int b = 0; b < DB; ++b) acc[b] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_ref = -INFINITY, l = 0.0f;

    // Fused form, e4m3 cache: the conversion of the row's new token (a division and an encoding per element) is
    // shared out over the whole workgroup, one or two elements per thread, instead of being done by the sixteen
    // lanes that need the bytes; every thread writes its V byte into the cache, the codes meet in LDS, and D/16
    // threads write the K chunks.  Only the item that holds the row's last page does this (all its waves do:
    // the condition is the same for the whole workgroup).
    [[maybe_unused]] __shared__ __align__(16) uint8_t new_tok[FUSED && sizeof(KT) == 1 ? 2 * D : 16];
    if constexpr (FUSED && sizeof(KT) == 1) {
        if (it_pe * kPage >= it_keys) {
            const int slot = (it_keys - 1) & (kPage - 1);
            const int64_t tile = (int64_t)as_constant(a.block_table)[(int64_t)it_seq * a.geo.max_pages + ((it_keys - 1) >> 4)] * Hkv + g;
            uint8_t* kc_w = (uint8_t*)const_cast<void*>(a.k_cache) + tile * (16 * D);
            uint8_t* vc_w = (uint8_t*)const_cast<void*>(a.v_cache) + tile * (16 * D);
            const uint16_t* kn = (const uint16_t*)a.k_new + ((int64_t)it_row * Hkv + g) * D;
            const uint16_t* vn = (const uint16_t*)a.v_new + ((int64_t)it_row * Hkv + g) * D;
            const float ks = a.k_scale[g], vs = a.v_scale[g];
            for (int e = threadIdx.x; e < 2 * D; e += 64 * WAVES) {
                const bool is_v = e >= D;
                const int dim = is_v ? e - D : e;
                const uint32_t code = float_to_e4m3_bits(bf16_bits_to_float(is_v ? vn[dim] : kn[dim]) / (is_v ? vs : ks));
                new_tok[e] = (uint8_t)code;
                if (is_v) __builtin_nontemporal_store((uint8_t)code, vc_w + dim * 16 + slot);
            }
            __syncthreads();
            if ((int)threadIdx.x < D / 16)
                store_nt(kc_w + (threadIdx.x * 16 + slot) * 16, *(const uint4*)(new_tok + 16 * threadIdx.x));
        }
    }

    if (np > 0) {                                                 // wave-uniform
        // Q^T operand: column n is query head g*G + n; columns >= G repeat the group's last head
        // (their results are finite and never stored)
        bf16x8 qb[KB];
        {
            const uint16_t* qrow = (const uint16_t*)a.q + ((int64_t)it_row * Hq + g * G + min(n, G - 1)) * D;
#pragma unroll
            for (int b = 0; b < KB; ++b) qb[b] = as_bf16x8(*(const uint4*)(qrow + q_dim0<KT>(b, r)));
        }
        const float kscale = (sizeof(KT) == 1) ? a.k_scale[g] : 1.0f;
        const float c = a.sm_scale * kscale * kLog2e;
        const char* kc = (const char*)a.k_cache;
        const char* vc = (const char*)a.v_cache;

        // page ids come through the scalar cache, one fetch ahead of their use
        int next_k = 0;
        int next_id = bt[0];
        auto fetch = [&](KVTile<KT, D>& t) {
            load_tile(t, kc, vc, (int64_t)next_id * Hkv + g, lane);
            next_k = min(next_k + 1, np - 1);                     // past the end: stay on the last page
            next_id = bt[WAVES * next_k];
        };
        KVTile<KT, D> buf[NBUF];
#pragma unroll
        for (int j = 0; j < NBUF; ++j) fetch(buf[j]);

        // (the wave's last page is partly filled only if it is the row's last page)
        const int page_last = it_pb + wave + WAVES * (np - 1);
        // (fused form: the row's last page always goes through the masked step, which patches in the new token)
        const bool has_tail = FUSED ? (page_last + 1) * kPage >= it_keys : (page_last + 1) * kPage > it_keys;   // wave-uniform
        const int np_main = np - (has_tail ? 1 : 0);
        // Fused form: the new token's K and V in cache form (converted exactly as the append kernels convert
        // them), asked for now so that the reads are under way during the scan.  K: the lanes of the token's slot
        // hold its dims in tile order; V: the lanes of the slot's group of four hold one element per dim block.
        constexpr int KR = sizeof(KT) == 2 ? D / 32 : D / 64;
        [[maybe_unused]] const int new_slot = (it_keys - 1) & (kPage - 1);
        [[maybe_unused]] uint4 new_k[KR];
        [[maybe_unused]] uint32_t new_v[DB];
        if constexpr (FUSED) {
            if (has_tail) {
                const uint16_t* kn = (const uint16_t*)a.k_new + ((int64_t)it_row * Hkv + g) * D;
                const uint16_t* vn = (const uint16_t*)a.v_new + ((int64_t)it_row * Hkv + g) * D;
                if constexpr (sizeof(KT) == 2) {
#pragma unroll
                    for (int b = 0; b < KR; ++b) new_k[b] = *(const uint4*)(kn + 8 * (4 * b + r));
#pragma unroll
                    for (int b = 0; b < DB; ++b) new_v[b] = vn[16 * b + n];
                } else {
                    // (converted by the whole workgroup above)
#pragma unroll
                    for (int j = 0; j < KR; ++j) new_k[j] = *(const uint4*)(new_tok + 16 * (4 * j + r));
#pragma unroll
                    for (int b = 0; b < DB; ++b) new_v[b] = new_tok[D + 16 * b + n];
                }
            }
        }

        // One page: S^T, online softmax against the reference maximum, O^T += V^T P^T.  MASKED is the row's last,
        // partly filled page: scores and V of the slots past n_keys are masked (the slots hold whatever was there
        // before).  It runs once per row, after the loop, so that the loop carries no mask arithmetic.
        auto page_step = [&](const KVTile<KT, D>& t_in, const int page, auto masked) {
            constexpr bool MASKED = decltype(masked)::value;
            KVTile<KT, D> t = t_in;
            if constexpr (MASKED && FUSED) {
                // The row's last page: slot (n_keys - 1) % 16 belongs to the token this pass appends.  Its K and V
                // (asked for before the scan, already in cache form) replace what the cache held in that slot and,
                // with a bf16 cache, go from here into the cache (an e4m3 cache got them from the workgroup above).
                const int64_t tile = (int64_t)bt[WAVES * (np - 1)] * Hkv + g;
                char* kc_w = (char*)const_cast<void*>(a.k_cache) + tile * (16 * D * (int)sizeof(KT));
                char* vc_w = (char*)const_cast<void*>(a.v_cache) + tile * (16 * D * (int)sizeof(KT));
                if (n == new_slot) {
#pragma unroll
                    for (int b = 0; b < KR; ++b) {
                        t.k[b] = new_k[b];
                        if constexpr (sizeof(KT) == 2) store_nt(kc_w + lane * 16 + b * 1024, new_k[b]);
                    }
                }
                if (r == (new_slot >> 2)) {
#pragma unroll
                    for (int b = 0; b < DB; ++b) {
                        if constexpr (sizeof(KT) == 2) {
                            const int sh = 16 * (new_slot & 1);
                            uint32_t& w = (new_slot & 2) ? t.v[b].y : t.v[b].x;
                            w = (w & ~(0xffffu << sh)) | (new_v[b] << sh);
                            __builtin_nontemporal_store((uint16_t)new_v[b], (uint16_t*)(vc_w + (16 * b + n) * 32 + new_slot * 2));
                        } else {
                            const int sh = 8 * (new_slot & 3);
                            t.v[b] = (t.v[b] & ~(0xffu << sh)) | (new_v[b] << sh);
                        }
                    }
                }
            }
            f32x4 s = qk_tile(t, qb);
            float t0 = s[0] * c, t1 = s[1] * c, t2 = s[2] * c, t3 = s[3] * c;
            const int nvalid = it_keys - (page * kPage + 4 * r);   // tokens tok0 .. tok0+3 valid if < nvalid
            if constexpr (MASKED) {
                t0 = nvalid > 0 ? t0 : -INFINITY; t1 = nvalid > 1 ? t1 : -INFINITY;
                t2 = nvalid > 2 ? t2 : -INFINITY; t3 = nvalid > 3 ? t3 : -INFINITY;
            }
            const float lmax = fmaxf(fmaxf(t0, t1), fmaxf(t2, t3));
            if (__any(lmax > m_ref + kRaise)) {           // raise the reference (rare)
                float full = fmaxf(lmax, __shfl_xor(lmax, 16, 64));
                full = fmaxf(full, __shfl_xor(full, 32, 64));
                const float m_new = fmaxf(m_ref, full);
                const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);   // 0 on the first page
#pragma unroll
                for (int b = 0; b < DB; ++b) acc[b] *= alpha;
                l *= alpha;
                m_ref = m_new;
            }
            const float p0 = __builtin_amdgcn_exp2f(t0 - m_ref), p1 = __builtin_amdgcn_exp2f(t1 - m_ref);
            const float p2 = __builtin_amdgcn_exp2f(t2 - m_ref), p3 = __builtin_amdgcn_exp2f(t3 - m_ref);
            l += (p0 + p1) + (p2 + p3);
            uint2 pw;
            pw.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{p0, p1}, bf16x2));
            pw.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{p2, p3}, bf16x2));
            const s16x4 pv = as_s16x4(pw);
            uint64_t keep = ~0ull;
            if constexpr (MASKED) keep = nvalid >= 4 ? ~0ull : (nvalid <= 0 ? 0ull : ((1ull << (16 * nvalid)) - 1ull));
#pragma unroll
            for (int b = 0; b < DB; ++b) {
                uint2 vv = v_operand(t, b);
                if constexpr (MASKED) { vv.x &= (uint32_t)keep; vv.y &= (uint32_t)(keep >> 32); }
                acc[b] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(as_s16x4(vv), pv, acc[b], 0, 0, 0);
            }
        };
        for (int base = 0; base < np_main; base += NBUF) {
#pragma unroll
            for (int j = 0; j < NBUF; ++j) {
                const int k = base + j;
                if (k < np_main) page_step(buf[j], it_pb + wave + WAVES * k, std::false_type{});   // wave-uniform
                fetch(buf[j]);                                    // refill (clamped to the wave's last page)
            }
        }
        if (has_tail) {
            // fetch number f reads page min(f, np - 1) into slot f % NBUF and at least np + NBUF - 1 fetches were
            // made: slot (np - 1) % NBUF holds the last page
            const int jt = (np - 1) % NBUF;
#pragma unroll
            for (int j = 0; j < NBUF; ++j)
                if (j == jt) page_step(buf[j], page_last, std::true_type{});
        }
    }

    float l_tot = l + __shfl_xor(l, 16, 64);
    l_tot += __shfl_xor(l_tot, 32, 64);

    // ---- merge the waves' states (wave order, so the result is reproducible) ----------------------
    if (wave > 0) {
#pragma unroll
        for (int b = 0; b < DB; ++b) *(f32x4*)mg.o[wave - 1][b][lane] = acc[b];
        if (r == 0) { mg.m[wave - 1][n] = m_ref; mg.l[wave - 1][n] = l_tot; }
    }
    __syncthreads();
    if (wave != 0) return;                                        // (leaves this function only)
    float M = m_ref;
#pragma unroll
    for (int w = 0; w < WAVES - 1; ++w) M = fmaxf(M, mg.m[w][n]);
    // wave 0 always holds the item's first page, so M is finite
    {
        const float w0 = __builtin_amdgcn_exp2f(m_ref - M);
#pragma unroll
        for (int b = 0; b < DB; ++b) acc[b] *= w0;
        l_tot *= w0;
    }
#pragma unroll
    for (int w = 0; w < WAVES - 1; ++w) {
        const float ww = __builtin_amdgcn_exp2f(mg.m[w][n] - M);  // exp2(-inf) = 0 for a wave without pages
        l_tot += mg.l[w][n] * ww;
#pragma unroll
        for (int b = 0; b < DB; ++b) acc[b] += *(const f32x4*)mg.o[w][b][lane] * ww;
    }

    if (n < G) {
        const int h = g * G + n;
        if (it_part < 0) {
            const float vscale = (sizeof(KT) == 1) ? a.v_scale[g] : 1.0f;
            const float inv = vscale / l_tot;
            uint16_t* o = (uint16_t*)a.out + ((int64_t)it_row * Hq + h) * D + 4 * r;
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
            float* o = a.part_o + ((int64_t)it_part * Hq + h) * D + 4 * r;
#pragma unroll
            for (int b = 0; b < DB; ++b) *(f32x4*)(o + 16 * b) = acc[b];
            if (r == 0) {
                float* ml = a.part_ml + ((int64_t)it_part * Hq + h) * 2;
                ml[0] = M;
                ml[1] = l_tot;
            }
        }
    }
    if constexpr (!MERGE) return;
    if (it_part < 0 || a.cmb_ctr == nullptr) return;

    // ---- a split row: the last of its items to get here merges the partials (no launch for the merge) ----
    // Release: this item's partials are visible device-wide before its arrival is counted; acquire: the item
    // that counts the last arrival sees every other item's partials.  The merge reads all partials back from
    // memory, its own included, in split order: the result does not depend on which item came last.
    const int32_t TS_CONSTANT* cm = as_constant((const int32_t*)(a.cmb + it_cmb));
    const int n_split = cm[2];
    __threadfence();
    int last = 0;
    if (lane == 0) {
        int32_t* ctr = a.cmb_ctr + (int64_t)it_cmb * Hkv + g;
        const int seen = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        last = seen == n_split - 1;
        if (last) __hip_atomic_store(ctr, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next launch
    }
    last = __builtin_amdgcn_readfirstlane(last);
    if (!last) return;
    __threadfence();
    if (n < G) {
        constexpr int kBatch = 4;
        const int h = g * G + n;
        const float* pml = a.part_ml + ((int64_t)it_part_first * Hq + h) * 2;     // split k: pml[k * Hq * 2 + {0, 1}]
        const float* po = a.part_o + ((int64_t)it_part_first * Hq + h) * D + 4 * r;   // split k: po[k * Hq * D + 16 b]
        const int64_t ml_step = (int64_t)Hq * 2, po_step = (int64_t)Hq * D;
        float Mx = -INFINITY;
        for (int k = 0; k < n_split; ++k) Mx = fmaxf(Mx, pml[k * ml_step]);
        f32x4 sum[DB];
#pragma unroll
        for (int b = 0; b < DB; ++b) sum[b] = f32x4{0.f, 0.f, 0.f, 0.f};
        float L = 0.0f;
        for (int k0 = 0; k0 < n_split; k0 += kBatch) {
            float w[kBatch];
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                const int k = min(k0 + j, n_split - 1);
                w[j] = k0 + j < n_split ? __builtin_amdgcn_exp2f(pml[k * ml_step] - Mx) : 0.0f;
                L += k0 + j < n_split ? pml[k * ml_step + 1] * w[j] : 0.0f;
            }
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                const int k = min(k0 + j, n_split - 1);
#pragma unroll
                for (int b = 0; b < DB; ++b) sum[b] += *(const f32x4*)(po + k * po_step + 16 * b) * w[j];
            }
        }
        const float vscale = (sizeof(KT) == 1) ? a.v_scale[g] : 1.0f;
        const float inv = vscale / L;
        uint16_t* o = (uint16_t*)a.out + ((int64_t)it_row * Hq + h) * D + 4 * r;
#pragma unroll
        for (int b = 0; b < DB; ++b) {
            const bf16x2 x = __builtin_convertvector(f32x2{sum[b][0] * inv, sum[b][1] * inv}, bf16x2);
            const bf16x2 y = __builtin_convertvector(f32x2{sum[b][2] * inv, sum[b][3] * inv}, bf16x2);
            uint2 wv;
            wv.x = __builtin_bit_cast(uint32_t, x);
            wv.y = __builtin_bit_cast(uint32_t, y);
            *(uint2*)(o + 16 * b) = wv;
        }
    }
}

}  // namespace ts
