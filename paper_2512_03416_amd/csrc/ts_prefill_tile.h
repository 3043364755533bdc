// Step a3 (device function shared by the prefill kernel and the persistent mixed kernel):
// causal attention of absorbed prefill chunks over the paged cache, on the matrix cores.
//
// A Convertible Decoder executes burst prefill requests as chunks next to its decode batch
// (paper Sec. 3.4, Sec. 4.4); a chunk row at position p attends to its cached prefix and to the
// chunk rows up to itself.  This part of the pass is a dense contraction (QK^T and PV), so it
// is tiled for MFMA:
//   - one workgroup (4 waves) owns a tile of 128 query rows = (128/G tokens) x (G query heads of
//     one KV head), so each K/V byte staged into LDS serves the whole head group;
//   - KV is consumed in stages of 64 tokens (4 pages).  Cache tiles are already in matrix-operand
//     order: K tiles are copied to LDS verbatim, V tiles are interleaved pairwise so that every
//     operand fetch is one conflict-free 16-byte LDS read at a lane-linear address;
//   - S^T = K Q^T (tokens x rows) so that the accumulator layout of S^T is the B-operand layout
//     of O^T += V^T P^T: the weights go from the first product to the second without leaving
//     registers, and softmax statistics are per lane (row) with a 2-step cross-lane reduction;
//   - the next stage's tiles are fetched from global memory into registers while the current
//     stage is multiplied.
// fp8 caches are widened to bf16 while being staged, so the multiply loop is the same.
#pragma once
#include "ts_device.h"

namespace ts {

constexpr float kRaisePf = 16.0f;
constexpr int kStageTok = 64;

__device__ __forceinline__ bf16x8 u4_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ uint2 fp8x4_bf16x4(uint32_t w)
{
    const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, false);
    const f32x2 hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, true);
    uint2 r;
    r.x = __builtin_amdgcn_perm(__float_as_uint(lo.y), __float_as_uint(lo.x), 0x07060302u);
    r.y = __builtin_amdgcn_perm(__float_as_uint(hi.y), __float_as_uint(hi.x), 0x07060302u);
    return r;
}

__device__ __forceinline__ float fmax3(float a, float b, float c) { return __builtin_fmaxf(__builtin_fmaxf(a, b), c); }

// keep the first n (0..8) 16-bit elements of a 16-byte vector (plain register arithmetic: local
// arrays here end up in scratch memory and serialise the prefetch)
__device__ __forceinline__ uint32_t mask16(int left) { return left >= 2 ? 0xffffffffu : (left == 1 ? 0xffffu : 0u); }
__device__ __forceinline__ uint4 keep_first16(uint4 v, int n)
{
    return make_uint4(v.x & mask16(n), v.y & mask16(n - 2), v.z & mask16(n - 4), v.w & mask16(n - 6));
}
// keep the first n (0..16) bytes of a 16-byte vector
__device__ __forceinline__ uint32_t mask8(int left)
{
    return left >= 4 ? 0xffffffffu : (left <= 0 ? 0u : ((1u << (8 * left)) - 1u));
}
__device__ __forceinline__ uint4 keep_first8(uint4 v, int n)
{
    return make_uint4(v.x & mask8(n), v.y & mask8(n - 4), v.z & mask8(n - 8), v.w & mask8(n - 12));
}

template <typename KT> struct Stage;                       // one thread's share of a 64-token stage
// (named members, no arrays: an array member that is ever indexed by a loop variable which the
// optimiser fails to fold sends the whole object to scratch memory)
template <> struct Stage<uint16_t> { uint4 k0, k1, k2, k3, v0, v1, v2, v3; };
template <> struct Stage<uint8_t>  { uint4 k0, k1, v0, v1; };

// LDS image of a stage (bf16 in both cases):
//   K: 4 pages x [16 dim-chunks][16 tokens][8]          = 4 x 4096 bytes
//   V: [2 page pairs][8 dim blocks][4 r][16 m][2 pages][4 tokens] = 16384 bytes
struct __align__(16) StageLds { unsigned char k[4 * 4096]; unsigned char v[16384]; };

__device__ __forceinline__ int v_lds_offset(int page_in_stage, int dim, int r)
{
    const int pp = page_in_stage >> 1, ab = page_in_stage & 1, blk = dim >> 4, m = dim & 15;
    return ((((pp * 8 + blk) * 4 + r) * 16 + m) * 2 + ab) * 8;
}

// ---- bf16 cache: each thread copies 16 bytes of every page's K tile and V tile ------------------
__device__ __forceinline__ void fetch_page_bf16(uint4& k, uint4& v, const AttnArgs& a,
                                                const int32_t TS_CONSTANT* bt, int page_idx, int last_page,
                                                int g, int tid)
{
    const int64_t tile = (int64_t)bt[min(page_idx, last_page)] * a.geo.Hkv + g;
    k = *(const uint4*)((const char*)a.k_cache + tile * 4096 + tid * 16);
    v = *(const uint4*)((const char*)a.v_cache + tile * 4096 + tid * 16);
}
__device__ __forceinline__ void stage_fetch(Stage<uint16_t>& st, const AttnArgs& a,
                                            const int32_t TS_CONSTANT* bt, int kv0, int last_page, int g, int tid)
{
    const int p0 = kv0 / kPage;
    fetch_page_bf16(st.k0, st.v0, a, bt, p0 + 0, last_page, g, tid);
    fetch_page_bf16(st.k1, st.v1, a, bt, p0 + 1, last_page, g, tid);
    fetch_page_bf16(st.k2, st.v2, a, bt, p0 + 2, last_page, g, tid);
    fetch_page_bf16(st.k3, st.v3, a, bt, p0 + 3, last_page, g, tid);
}
__device__ __forceinline__ void store_page_bf16(uint4 k, uint4 v, StageLds& lds, int i, int kv0, int ctx_len, int tid)
{
    *(uint4*)(lds.k + i * 4096 + tid * 16) = k;
    // V chunk: dim = tid/2, tokens 8*hf .. 8*hf+7 of page i
    const int dim = tid >> 1, hf = tid & 1;
    const int nvalid = ctx_len - (kv0 + i * kPage + 8 * hf);              // poison past ctx_len -> 0
    if (nvalid < 8) v = keep_first16(v, max(nvalid, 0));
    *(uint2*)(lds.v + v_lds_offset(i, dim, 2 * hf)) = make_uint2(v.x, v.y);
    *(uint2*)(lds.v + v_lds_offset(i, dim, 2 * hf + 1)) = make_uint2(v.z, v.w);
}
__device__ __forceinline__ void stage_store(const Stage<uint16_t>& st, StageLds& lds, int kv0, int ctx_len, int tid)
{
    store_page_bf16(st.k0, st.v0, lds, 0, kv0, ctx_len, tid);
    store_page_bf16(st.k1, st.v1, lds, 1, kv0, ctx_len, tid);
    store_page_bf16(st.k2, st.v2, lds, 2, kv0, ctx_len, tid);
    store_page_bf16(st.k3, st.v3, lds, 3, kv0, ctx_len, tid);
}

// ---- fp8 cache: 4 pages x 2048 bytes = 512 chunks of 16 bytes, two per thread, widened to bf16 ----
__device__ __forceinline__ void fetch_chunk_fp8(uint4& k, uint4& v, const AttnArgs& a,
                                                const int32_t TS_CONSTANT* bt, int kv0, int ci, int last_page, int g)
{
    const int pg = __builtin_amdgcn_readfirstlane(ci >> 7);       // uniform within a wave
    const int64_t tile = (int64_t)bt[min(kv0 / kPage + pg, last_page)] * a.geo.Hkv + g;
    k = *(const uint4*)((const char*)a.k_cache + tile * 2048 + (ci & 127) * 16);
    v = *(const uint4*)((const char*)a.v_cache + tile * 2048 + (ci & 127) * 16);
}
__device__ __forceinline__ void stage_fetch(Stage<uint8_t>& st, const AttnArgs& a,
                                            const int32_t TS_CONSTANT* bt, int kv0, int last_page, int g, int tid)
{
    fetch_chunk_fp8(st.k0, st.v0, a, bt, kv0, tid, last_page, g);
    fetch_chunk_fp8(st.k1, st.v1, a, bt, kv0, 256 + tid, last_page, g);
}
__device__ __forceinline__ void store_chunk_fp8(uint4 k, uint4 v, StageLds& lds, int ci, int kv0, int ctx_len)
{
    const int pg = ci >> 7, c = ci & 127;
    // K chunk: 16 dims (chunk c/16) of token c%16 -> two bf16 chunks of 8 dims
    const int c16 = c >> 4, tok = c & 15;
    const uint2 a0 = fp8x4_bf16x4(k.x), a1 = fp8x4_bf16x4(k.y), a2 = fp8x4_bf16x4(k.z), a3 = fp8x4_bf16x4(k.w);
    *(uint4*)(lds.k + pg * 4096 + ((2 * c16) * 16 + tok) * 16) = make_uint4(a0.x, a0.y, a1.x, a1.y);
    *(uint4*)(lds.k + pg * 4096 + ((2 * c16 + 1) * 16 + tok) * 16) = make_uint4(a2.x, a2.y, a3.x, a3.y);
    // V chunk: dim c, 16 tokens of page pg
    const int nvalid = ctx_len - (kv0 + pg * kPage);
    if (nvalid < 16) v = keep_first8(v, max(nvalid, 0));
    *(uint2*)(lds.v + v_lds_offset(pg, c, 0)) = fp8x4_bf16x4(v.x);
    *(uint2*)(lds.v + v_lds_offset(pg, c, 1)) = fp8x4_bf16x4(v.y);
    *(uint2*)(lds.v + v_lds_offset(pg, c, 2)) = fp8x4_bf16x4(v.z);
    *(uint2*)(lds.v + v_lds_offset(pg, c, 3)) = fp8x4_bf16x4(v.w);
}
__device__ __forceinline__ void stage_store(const Stage<uint8_t>& st, StageLds& lds, int kv0, int ctx_len, int tid)
{
    store_chunk_fp8(st.k0, st.v0, lds, tid, kv0, ctx_len);
    store_chunk_fp8(st.k1, st.v1, lds, 256 + tid, kv0, ctx_len);
}

// One causal tile for KV head g, executed by a workgroup of 256 threads.  All threads must call
// it; every stage ends with a workgroup barrier, so the two stage buffers lds2[0..1] may be reused
// right after it returns.
template <typename KT>
__device__ __forceinline__ void prefill_tile(const AttnArgs& a, int item_idx, int g, StageLds* lds2)
{
    constexpr int D = 128, KB = 4, DB = 8, NT = 2;
    const PfItem it = a.pf[item_idx];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane >> 4, n = lane & 15;
    const int Hq = a.geo.Hq, G = a.geo.G;

    // rows of this lane: rho = 32*wave + 16*nt + n  ->  (token rho / G, head rho % G)
    int tok[NT], hd[NT];
    bool row_ok[NT];
    bf16x8 qb[NT][KB];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int rho = 32 * wave + 16 * nt + n;
        const int t = rho / G;
        row_ok[nt] = t < it.tok_count;
        tok[nt] = min(t, it.tok_count - 1);                 // padding rows repeat the last token
        hd[nt] = rho - t * G;
        const uint16_t* qrow = (const uint16_t*)a.q +
            ((int64_t)(it.row0 + it.tok_begin + tok[nt]) * Hq + g * G + hd[nt]) * D + 8 * r;
#pragma unroll
        for (int b = 0; b < KB; ++b) qb[nt][b] = u4_bf16x8(*(const uint4*)(qrow + 32 * b));
    }
    const float kscale = (sizeof(KT) == 1) ? a.k_scale[g] : 1.0f;
    const float c = a.sm_scale * kscale * kLog2e;
    int qpos[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) qpos[nt] = it.prefix + it.tok_begin + tok[nt];
    const int wave_min_q = it.prefix + it.tok_begin + min((32 * wave) / G, it.tok_count - 1);
    const int wave_max_q = it.prefix + it.tok_begin + min((32 * wave + 31) / G, it.tok_count - 1);
    const int kv_hi = it.prefix + it.tok_begin + it.tok_count;     // keys [0, kv_hi) matter to this tile
    const int last_page = (it.ctx_len - 1) / kPage;
    const int32_t TS_CONSTANT* bt = as_constant(a.block_table) + (int64_t)it.seq * a.geo.max_pages;

    f32x4 acc[DB][NT];
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[b][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    // running sums of the weights come out of the matrix cores too: an all-ones A operand makes
    // every row of the product the column sum of P^T, i.e. the softmax denominator of the lane's row
    f32x4 accl[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) accl[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    const bf16x8 ones = u4_bf16x8(make_uint4(0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u));
    float m_ref[NT] = {-INFINITY, -INFINITY};

    // Two LDS stage buffers: while stage i is multiplied out of one, stage i+1 (fetched into
    // registers during stage i-1 and i) is written into the other, so a stage costs one barrier.
    Stage<KT> st;
    stage_fetch(st, a, bt, 0, last_page, g, tid);
    stage_store(st, lds2[0], 0, it.ctx_len, tid);
    if (kStageTok < kv_hi) stage_fetch(st, a, bt, kStageTok, last_page, g, tid);
    __syncthreads();
    int buf = 0;
    for (int kv0 = 0; kv0 < kv_hi; kv0 += kStageTok, buf ^= 1) {
        const StageLds& lds = lds2[buf];
        if (kv0 <= wave_max_q) {                            // wave-uniform: some row sees this stage
            // ---- S^T = K Q^T (raw scores; the softmax scale is folded into the exponent) ----
            f32x4 s[4][NT];
#pragma unroll
            for (int tt = 0; tt < 4; ++tt) {
                bf16x8 ak[KB];
#pragma unroll
                for (int b = 0; b < KB; ++b)
                    ak[b] = u4_bf16x8(*(const uint4*)(lds.k + tt * 4096 + b * 1024 + lane * 16));
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    f32x4 x = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int b = 0; b < KB; ++b)
                        x = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ak[b], qb[nt][b], x, 0, 0, 0);
                    s[tt][nt] = x;
                }
            }
            // ---- causal mask (only stages that reach the diagonal) ------------------------
            if (kv0 + kStageTok - 1 > wave_min_q) {
#pragma unroll
                for (int tt = 0; tt < 4; ++tt)
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (kv0 + tt * 16 + 4 * r + i > qpos[nt]) s[tt][nt][i] = -INFINITY;
            }
            // ---- online softmax, reference maximum (in scaled log2 units) raised lazily -----
            float lmax[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                float x = __builtin_fmaxf(s[0][nt][0], s[0][nt][1]);
                x = fmax3(x, s[0][nt][2], s[0][nt][3]);
#pragma unroll
                for (int tt = 1; tt < 4; ++tt) {
                    x = fmax3(x, s[tt][nt][0], s[tt][nt][1]);
                    x = fmax3(x, s[tt][nt][2], s[tt][nt][3]);
                }
                lmax[nt] = x * c;                          // c > 0: the maximum commutes with the scale
            }
            if (__any(lmax[0] > m_ref[0] + kRaisePf || lmax[1] > m_ref[1] + kRaisePf)) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    float full = fmaxf(lmax[nt], __shfl_xor(lmax[nt], 16, 64));
                    full = fmaxf(full, __shfl_xor(full, 32, 64));
                    const float m_new = fmaxf(m_ref[nt], full);
                    const float alpha = __builtin_amdgcn_exp2f(m_ref[nt] - m_new);
#pragma unroll
                    for (int b = 0; b < DB; ++b) acc[b][nt] *= alpha;
                    accl[nt] *= alpha;
                    m_ref[nt] = m_new;
                }
            }
            bf16x8 pop[2][NT];                             // P^T operands: [page pair][row tile]
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const float nm = -m_ref[nt];
#pragma unroll
                for (int pp = 0; pp < 2; ++pp) {
                    uint32_t w[4];
#pragma unroll
                    for (int ab = 0; ab < 2; ++ab) {
                        const f32x4 x = s[2 * pp + ab][nt];
                        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(x[0], c, nm));
                        const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(x[1], c, nm));
                        const float p2 = __builtin_amdgcn_exp2f(__builtin_fmaf(x[2], c, nm));
                        const float p3 = __builtin_amdgcn_exp2f(__builtin_fmaf(x[3], c, nm));
                        w[2 * ab] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{p0, p1}, bf16x2));
                        w[2 * ab + 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{p2, p3}, bf16x2));
                    }
                    pop[pp][nt] = u4_bf16x8(make_uint4(w[0], w[1], w[2], w[3]));
                }
            }
            // ---- O^T += V^T P^T (and the row sums) -----------------------------------------------
#pragma unroll
            for (int pp = 0; pp < 2; ++pp)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    accl[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pop[pp][nt], accl[nt], 0, 0, 0);
#pragma unroll
            for (int pp = 0; pp < 2; ++pp)
#pragma unroll
                for (int b = 0; b < DB; ++b) {
                    const bf16x8 av = u4_bf16x8(*(const uint4*)(lds.v + (pp * 8 + b) * 1024 + lane * 16));
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        acc[b][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, pop[pp][nt], acc[b][nt], 0, 0, 0);
                }
        }
        if (kv0 + kStageTok < kv_hi) {
            // the other buffer was last read during the previous stage, which every wave left
            // through the barrier below
            stage_store(st, lds2[buf ^ 1], kv0 + kStageTok, it.ctx_len, tid);
            if (kv0 + 2 * kStageTok < kv_hi) stage_fetch(st, a, bt, kv0 + 2 * kStageTok, last_page, g, tid);
        }
        __syncthreads();
    }

    const float vscale = (sizeof(KT) == 1) ? a.v_scale[g] : 1.0f;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const float lt = accl[nt][0];
        if (!row_ok[nt]) continue;
        const float inv = vscale / lt;
        uint16_t* o = (uint16_t*)a.out +
            ((int64_t)(it.row0 + it.tok_begin + tok[nt]) * Hq + g * G + hd[nt]) * D + 4 * r;
#pragma unroll
        for (int b = 0; b < DB; ++b) {
            const f32x4 x = acc[b][nt] * inv;
            uint2 w;
            w.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{x[0], x[1]}, bf16x2));
            w.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{x[2], x[3]}, bf16x2));
            *(uint2*)(o + 16 * b) = w;
        }
    }
}

}  // namespace ts
