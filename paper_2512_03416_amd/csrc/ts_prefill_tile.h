// Step a3 (device function shared by the prefill kernel and the persistent mixed kernel):
// causal attention of absorbed prefill chunks over the paged cache, on the matrix cores.
//
// A Convertible Decoder executes burst prefill requests as chunks next to its decode batch
// (paper Sec. 3.4, Sec. 4.4); a chunk row at position p attends to its cached prefix and to the
// chunk rows up to itself.  This part of the pass is a dense contraction (QK^T and PV), so it
// is tiled for MFMA:
//   - one workgroup (8 waves) owns a tile of 256 query rows = (256/G tokens) x (G query heads of
//     one KV head), so each K/V byte staged into LDS serves the whole head group;
//   - KV is consumed in stages of 64 tokens (4 pages).  Cache tiles are already in matrix-operand
//     order: K tiles are copied to LDS verbatim, V tiles are interleaved pairwise so that every
//     operand fetch is one conflict-free 16-byte LDS read at a lane-linear address;
//   - S^T = K Q^T (tokens x rows) so that the accumulator layout of S^T is the B-operand layout
//     of O^T += V^T P^T: the weights go from the first product to the second without leaving
//     registers, and softmax statistics are per lane (row) with a 2-step cross-lane reduction;
//   - the tiles of the next two stages are on their way from global memory into registers while
//     the current stage is multiplied.
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

constexpr int kPfWaves = 8;                                // 512 threads, 256 query rows per tile
constexpr int kPfThreads = 64 * kPfWaves;

template <typename KT> struct Stage;                       // one thread's share of a 64-token stage
// (named members, no arrays: an array member that is ever indexed by a loop variable which the
// optimiser fails to fold sends the whole object to scratch memory)
template <> struct Stage<uint16_t> { uint4 k0, k1, v0, v1; };
template <> struct Stage<uint8_t>  { uint4 k0, v0; };

// LDS image of a stage (bf16 in both cases):
//   K: 4 pages x [16 dim-chunks][16 tokens][8]          = 4 x 4096 bytes
//   V: [2 page pairs][8 dim blocks][4 r][16 m][2 pages][4 tokens] = 16384 bytes
// K is double-buffered, V triple-buffered.
struct __align__(16) PfLds {
    unsigned char k[2][4 * 4096];          // stage i lives in k[i & 1]
    unsigned char v[3][16384];             // stage i lives in v[i % 3] (kept one stage longer, see prefill_tile)
};

__device__ __forceinline__ int v_lds_offset(int page_in_stage, int dim, int r)
{
    const int pp = page_in_stage >> 1, ab = page_in_stage & 1, blk = dim >> 4, m = dim & 15;
    return ((((pp * 8 + blk) * 4 + r) * 16 + m) * 2 + ab) * 8;
}

// ---- bf16 cache: a stage is 4 pages x (4 KB K + 4 KB V) = 2 x 1024 chunks of 16 bytes; thread tid
// copies chunks tid and tid + 512 of K and of V (pages tid/256 and tid/256 + 2) -------------------
__device__ __forceinline__ void fetch_chunk_bf16(uint4& k, uint4& v, const AttnArgs& a,
                                                 const int32_t TS_CONSTANT* bt, int kv0, int ci, int last_page, int g)
{
    const int pg = __builtin_amdgcn_readfirstlane(ci >> 8);       // uniform within a wave
    const int64_t tile = (int64_t)bt[min(kv0 / kPage + pg, last_page)] * a.geo.Hkv + g;
    k = *(const uint4*)((const char*)a.k_cache + tile * 4096 + (ci & 255) * 16);
    v = *(const uint4*)((const char*)a.v_cache + tile * 4096 + (ci & 255) * 16);
}
__device__ __forceinline__ void stage_fetch(Stage<uint16_t>& st, const AttnArgs& a,
                                            const int32_t TS_CONSTANT* bt, int kv0, int last_page, int g, int tid)
{
    fetch_chunk_bf16(st.k0, st.v0, a, bt, kv0, tid, last_page, g);
    fetch_chunk_bf16(st.k1, st.v1, a, bt, kv0, tid + kPfThreads, last_page, g);
}
__device__ __forceinline__ void store_chunk_bf16(uint4 k, uint4 v, unsigned char* lk, unsigned char* lv, int ci, int kv0,
                                                 int ctx_len)
{
    const int pg = ci >> 8, c = ci & 255;
    *(uint4*)(lk + pg * 4096 + c * 16) = k;
    // V chunk: dim = c/2, tokens 8*hf .. 8*hf+7 of page pg
    const int dim = c >> 1, hf = c & 1;
    const int nvalid = ctx_len - (kv0 + pg * kPage + 8 * hf);             // poison past ctx_len -> 0
    if (nvalid < 8) v = keep_first16(v, max(nvalid, 0));
    *(uint2*)(lv + v_lds_offset(pg, dim, 2 * hf)) = make_uint2(v.x, v.y);
    *(uint2*)(lv + v_lds_offset(pg, dim, 2 * hf + 1)) = make_uint2(v.z, v.w);
}
__device__ __forceinline__ void stage_store(const Stage<uint16_t>& st, unsigned char* lk, unsigned char* lv, int kv0,
                                            int ctx_len, int tid)
{
    store_chunk_bf16(st.k0, st.v0, lk, lv, tid, kv0, ctx_len);
    store_chunk_bf16(st.k1, st.v1, lk, lv, tid + kPfThreads, kv0, ctx_len);
}

// ---- fp8 cache: 4 pages x 2048 bytes = 512 chunks of 16 bytes of K and of V, one each per thread,
// widened to bf16 on the way into LDS -------------------------------------------------------------
__device__ __forceinline__ void stage_fetch(Stage<uint8_t>& st, const AttnArgs& a,
                                            const int32_t TS_CONSTANT* bt, int kv0, int last_page, int g, int tid)
{
    const int pg = __builtin_amdgcn_readfirstlane(tid >> 7);      // uniform within a wave
    const int64_t tile = (int64_t)bt[min(kv0 / kPage + pg, last_page)] * a.geo.Hkv + g;
    st.k0 = *(const uint4*)((const char*)a.k_cache + tile * 2048 + (tid & 127) * 16);
    st.v0 = *(const uint4*)((const char*)a.v_cache + tile * 2048 + (tid & 127) * 16);
}
__device__ __forceinline__ void stage_store(const Stage<uint8_t>& st, unsigned char* lk, unsigned char* lv, int kv0,
                                            int ctx_len, int tid)
{
    const int pg = tid >> 7, c = tid & 127;
    // K chunk: 16 dims (chunk c/16) of token c%16 -> two bf16 chunks of 8 dims
    const int c16 = c >> 4, tok = c & 15;
    const uint4 k = st.k0;
    uint4 v = st.v0;
    const uint2 a0 = fp8x4_bf16x4(k.x), a1 = fp8x4_bf16x4(k.y), a2 = fp8x4_bf16x4(k.z), a3 = fp8x4_bf16x4(k.w);
    *(uint4*)(lk + pg * 4096 + ((2 * c16) * 16 + tok) * 16) = make_uint4(a0.x, a0.y, a1.x, a1.y);
    *(uint4*)(lk + pg * 4096 + ((2 * c16 + 1) * 16 + tok) * 16) = make_uint4(a2.x, a2.y, a3.x, a3.y);
    // V chunk: dim c, 16 tokens of page pg
    const int nvalid = ctx_len - (kv0 + pg * kPage);
    if (nvalid < 16) v = keep_first8(v, max(nvalid, 0));
    *(uint2*)(lv + v_lds_offset(pg, c, 0)) = fp8x4_bf16x4(v.x);
    *(uint2*)(lv + v_lds_offset(pg, c, 1)) = fp8x4_bf16x4(v.y);
    *(uint2*)(lv + v_lds_offset(pg, c, 2)) = fp8x4_bf16x4(v.z);
    *(uint2*)(lv + v_lds_offset(pg, c, 3)) = fp8x4_bf16x4(v.w);
}

// One causal tile for KV head g, executed by a workgroup of kPfThreads threads.  All threads must call
// it; it ends with a workgroup barrier, so lds may be reused right after it returns.
//
// The two waves that share a SIMD (wave w and w + 4) run half a stage apart: waves 0-3 do
// QK^T(i), softmax(i), PV(i) inside stage i's barrier interval, waves 4-7 do PV(i-1), QK^T(i),
// softmax(i).  The matrix-core phases of one wave then fall on the vector-ALU phase of the other;
// in lockstep the two phases of a stage simply add up (measured).  The lagging group needs V of
// the previous stage, hence the third V buffer.
template <typename KT>
__device__ __forceinline__ void prefill_tile(const AttnArgs& a, int item_idx, int g, PfLds& lds)
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

    // Pipeline: 256-row tiles (half the passes over K/V of 128-row tiles); two stages are always in
    // flight in registers (stA, stB) while a third is multiplied out of LDS; one barrier per stage.
    bf16x8 pop[2][NT];                                     // P^T operands: [page pair][row tile]

    // ---- QK^T and softmax of one stage: leaves the weights of the stage in pop ---------------------
    auto scores = [&](const unsigned char* lk, int kv0) {
        // S^T = K Q^T (raw scores; the softmax scale is folded into the exponent)
        f32x4 s[4][NT];
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
            bf16x8 ak[KB];
#pragma unroll
            for (int b = 0; b < KB; ++b)
                ak[b] = u4_bf16x8(*(const uint4*)(lk + tt * 4096 + b * 1024 + lane * 16));
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                f32x4 x = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int b = 0; b < KB; ++b)
                    x = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ak[b], qb[nt][b], x, 0, 0, 0);
                s[tt][nt] = x;
            }
        }
        // causal mask (only stages that reach the diagonal)
        if (kv0 + kStageTok - 1 > wave_min_q) {
#pragma unroll
            for (int tt = 0; tt < 4; ++tt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (kv0 + tt * 16 + 4 * r + i > qpos[nt]) s[tt][nt][i] = -INFINITY;
        }
        // online softmax, reference maximum (in scaled log2 units) raised lazily
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
            lmax[nt] = x * c;                              // c > 0: the maximum commutes with the scale
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
    };
    // ---- O^T += V^T P^T (and the row sums) of the stage whose weights are in pop --------------------
    auto weighted_values = [&](const unsigned char* lv) {
#pragma unroll
        for (int pp = 0; pp < 2; ++pp)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                accl[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pop[pp][nt], accl[nt], 0, 0, 0);
#pragma unroll
        for (int pp = 0; pp < 2; ++pp)
#pragma unroll
            for (int b = 0; b < DB; ++b) {
                const bf16x8 av = u4_bf16x8(*(const uint4*)(lv + (pp * 8 + b) * 1024 + lane * 16));
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    acc[b][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, pop[pp][nt], acc[b][nt], 0, 0, 0);
            }
    };

    const int n_stage = (kv_hi + kStageTok - 1) / kStageTok;
    const bool lagging = a.pf_skew != 0 && (a.pf_skew == 1 ? wave >= kPfWaves / 2 : (wave & 1) != 0);   // wave-uniform
    int pending = -1;                                      // lagging waves: stage whose PV is still to do
    // one stage: compute, then move stage i+1 from registers (st) into LDS and refill st with stage i+3
    auto step = [&](int i, Stage<KT>& st) {
        const int kv0 = i * kStageTok;
        const bool active = kv0 <= wave_max_q;             // wave-uniform: some row of the wave sees this stage
        if (lagging) {
            if (pending >= 0) weighted_values(lds.v[pending % 3]);
            pending = -1;
            if (active) { scores(lds.k[i & 1], kv0); pending = i; }
        } else if (active) {
            scores(lds.k[i & 1], kv0);
            weighted_values(lds.v[i % 3]);
        }
        if (i + 1 < n_stage) {
            // k[(i+1)&1] was last read in stage i-1, v[(i+1)%3] in stage i-1 by the lagging waves (PV of
            // stage i-2); every wave has left those stages through a barrier
            stage_store(st, lds.k[(i + 1) & 1], lds.v[(i + 1) % 3], kv0 + kStageTok, it.ctx_len, tid);
            if (i + 3 < n_stage) stage_fetch(st, a, bt, kv0 + 3 * kStageTok, last_page, g, tid);
        }
        __syncthreads();
    };
    Stage<KT> stA, stB;
    stage_fetch(stA, a, bt, 0, last_page, g, tid);
    if (n_stage > 1) stage_fetch(stB, a, bt, kStageTok, last_page, g, tid);
    stage_store(stA, lds.k[0], lds.v[0], 0, it.ctx_len, tid);
    if (n_stage > 2) stage_fetch(stA, a, bt, 2 * kStageTok, last_page, g, tid);
    __syncthreads();
    for (int i = 0; i < n_stage; i += 2) {
        step(i, stB);
        if (i + 1 < n_stage) step(i + 1, stA);
    }
    if (pending >= 0) weighted_values(lds.v[pending % 3]);
    __syncthreads();                                       // lds may be reused by the caller

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
