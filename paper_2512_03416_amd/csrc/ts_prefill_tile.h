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
constexpr int kPfRing = 4;                                 // stages resident in LDS

// LDS image of a stage (bf16 in both cases), both in the order of the cache tiles:
//   K: 4 pages x [16 dim-chunks][16 tokens][8]  = 4 x 4096 bytes
//   V: 4 pages x [8 dim blocks][2 token halves][16 dims][8 tokens] = 4 x 4096 bytes: the 16-byte
//      pieces (dim, 8 tokens) of the cache tile [128 dims][16 tokens], reordered so that the 16
//      dims of an MFMA operand lie side by side (conflict-free 8-byte operand reads)
// Stage i lives in slot i % kPfRing of both rings.
struct __align__(16) PfLds {
    unsigned char k[kPfRing][4 * 4096];
    unsigned char v[kPfRing][4 * 4096];
};

// byte offset inside a page's V image of the piece (dim, token half)
__device__ __forceinline__ int v_piece_offset(int dim, int half) { return (((dim >> 4) * 2 + half) * 16 + (dim & 15)) * 16; }

__device__ __forceinline__ uint32_t lds_address(const void* p)
{
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)p;
}

// ---- bf16 cache: the memory system copies a stage straight into LDS -------------------------------
// One instruction moves 64 x 16 bytes: lane l's chunk lands at lds_addr + 16 l (the instruction offset
// advances both the global and the LDS address).  A wave moves 2 KB of K and 2 KB of V per stage:
// half of page `wave / 2`.  The copies are counted by vmcnt like any load; nothing here tells the
// compiler that LDS changes, so the caller waits (pf_wait_copies) and publishes with a barrier.
__device__ __forceinline__ void copy_2k_to_lds(uint32_t lds_addr, const void* base, uint32_t lane_off)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
                 "global_load_lds_dwordx4 %1, %2\n\t"
                 "global_load_lds_dwordx4 %1, %2 offset:1024\n"
                 :: "s"(lds_addr), "v"(lane_off), "s"(base) : "memory");
}
__device__ __forceinline__ void stage_copy_bf16(const AttnArgs& a, const int32_t TS_CONSTANT* bt, int stage,
                                                int last_page, int g, int wave, int lane, PfLds& lds)
{
    const int page = min(stage * 4 + (wave >> 1), last_page);          // wave-uniform
    const int64_t off = ((int64_t)bt[page] * a.geo.Hkv + g) * 4096 + (wave & 1) * 2048;
    const int slot = stage % kPfRing;
    copy_2k_to_lds(lds_address(lds.k[slot]) + wave * 2048, (const char*)a.k_cache + off, lane * 16);
    // V: LDS piece p = 64 k + lane of this wave's 2 KB takes cache piece (dim 32 k + 16 (lane / 32) + lane % 16,
    // half (lane / 16) % 2); the second instruction (k = 1) is 1 KB further in both
    const int v_src = ((16 * (lane >> 5) + (lane & 15)) * 2 + ((lane >> 4) & 1)) * 16;
    copy_2k_to_lds(lds_address(lds.v[slot]) + wave * 2048, (const char*)a.v_cache + off, v_src);
}
constexpr int kCopiesPerStage = 4;                         // vmcnt units one stage_copy_bf16 adds per wave
template <int N> __device__ __forceinline__ void pf_wait_copies()
{
    static_assert(N >= 0 && N < 16, "vmcnt immediate");
    __builtin_amdgcn_s_waitcnt(0x0f70 | N);                // vmcnt(N); expcnt and lgkmcnt untouched
}
// V rows of tokens at or beyond ctx_len hold whatever the cache page held (possibly NaN patterns):
// their weights are zero, but 0 x NaN is not, so they are cleared in LDS once the stage has landed.
__device__ __forceinline__ void clear_v_tail(unsigned char* lv, int stage, int ctx_len, int tid)
{
    const int pg = tid >> 7, dim = tid & 127;
    const int nvalid = ctx_len - (stage * kStageTok + pg * kPage);     // valid tokens of this page
    if (nvalid >= kPage) return;
    uint4* lo = (uint4*)(lv + pg * 4096 + v_piece_offset(dim, 0));
    uint4* hi = (uint4*)(lv + pg * 4096 + v_piece_offset(dim, 1));
    *lo = keep_first16(*lo, max(nvalid, 0));
    *hi = keep_first16(*hi, max(nvalid - 8, 0));
}

// ---- fp8 cache: 4 pages x 2048 bytes = 512 chunks of 16 bytes of K and of V, one each per thread,
// widened to bf16 on the way into LDS -------------------------------------------------------------
struct StageFp8 { uint4 k0, v0; };                          // (named members: arrays end up in scratch memory)
__device__ __forceinline__ void stage_fetch(StageFp8& st, const AttnArgs& a, const int32_t TS_CONSTANT* bt, int kv0,
                                            int last_page, int g, int tid)
{
    const int pg = __builtin_amdgcn_readfirstlane(tid >> 7);      // uniform within a wave
    const int64_t tile = (int64_t)bt[min(kv0 / kPage + pg, last_page)] * a.geo.Hkv + g;
    st.k0 = *(const uint4*)((const char*)a.k_cache + tile * 2048 + (tid & 127) * 16);
    st.v0 = *(const uint4*)((const char*)a.v_cache + tile * 2048 + (tid & 127) * 16);
}
__device__ __forceinline__ void stage_store(const StageFp8& st, unsigned char* lk, unsigned char* lv, int kv0,
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
    // V chunk: dim c, 16 tokens of page pg -> two pieces of 8 tokens
    const int nvalid = ctx_len - (kv0 + pg * kPage);
    if (nvalid < 16) v = keep_first8(v, max(nvalid, 0));             // poison past ctx_len -> 0
    const uint2 b0 = fp8x4_bf16x4(v.x), b1 = fp8x4_bf16x4(v.y), b2 = fp8x4_bf16x4(v.z), b3 = fp8x4_bf16x4(v.w);
    *(uint4*)(lv + pg * 4096 + v_piece_offset(c, 0)) = make_uint4(b0.x, b0.y, b1.x, b1.y);
    *(uint4*)(lv + pg * 4096 + v_piece_offset(c, 1)) = make_uint4(b2.x, b2.y, b3.x, b3.y);
}

// One causal tile for KV head g, executed by a workgroup of kPfThreads threads.  All threads must call
// it; it ends with a workgroup barrier, so lds may be reused right after it returns.
//
// A wave works through its keys in half-stages of 32 tokens and keeps two of them in flight: while
// the matrix cores multiply K Q^T of half-stage h+1, the vector ALU turns the scores of half-stage
// h into weights (one fused multiply-add, one exp2 and half a pack per MFMA slot); while they
// multiply V^T P^T of half-stage h, it reduces the row maxima of h+1.  The instruction order of
// that steady state is written out slot by slot and pinned with scheduling barriers: an MFMA
// occupies its pipe for 16 cycles but the issue port for 4, and left to itself the compiler puts
// the two phases one after the other, where their times add up.
template <typename KT>
__device__ __forceinline__ void prefill_tile(const AttnArgs& a, int item_idx, int g, PfLds& lds)
{
    constexpr int D = 128, KB = 4, DB = 8, NT = 2, kHalf = 32;
    const PfItem it = a.pf[item_idx];
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, r = lane >> 4,
              n = lane & 15;
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
    // half-stages [0, hend) hold keys that some row of this wave sees; [0, hfull) need no causal mask
    const int hend = wave_max_q / kHalf + 1;
    const int hfull = (wave_min_q + 1) / kHalf;

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

    // lane's operand addresses of half-stage h inside the LDS rings.  K operand of dim block b of the
    // first / second 16 tokens: 16 bytes at kptr + b * 1024 (+ 4096).  V operand of dim block b: tokens
    // 4r..4r+3 of both pages of the half-stage, 8 bytes each at vptr + b * 512 (+ 4096): half of the
    // piece (dim 16 b + n, token half r / 2).
    auto kptr = [&](int h) { return lds.k[(h >> 1) % kPfRing] + (h & 1) * 8192 + lane * 16; };
    auto vptr = [&](int h) { return lds.v[(h >> 1) % kPfRing] + (h & 1) * 8192 + v_piece_offset(n, r >> 1) + (r & 1) * 8; };
    auto lds16 = [](const unsigned char* p) { return u4_bf16x8(*(const uint4*)p); };
    auto ldsv = [](const unsigned char* p) {
        const uint2 x = *(const uint2*)p, y = *(const uint2*)(p + 4096);
        return u4_bf16x8(make_uint4(x.x, x.y, y.x, y.y));
    };
    auto mfma = [](bf16x8 x, bf16x8 y, f32x4 z) { return __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, y, z, 0, 0, 0); };
    auto pack2 = [](float x, float y) {
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{x, y}, bf16x2));
    };

    // ---- plain building blocks (first and last half-stages of a wave) -------------------------------
    // S^T = K Q^T of one half-stage (raw scores; the softmax scale is folded into the exponent)
    auto qk_plain = [&](const unsigned char* lk, f32x4 (&s)[2][NT]) {
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
            bf16x8 ak[KB];
#pragma unroll
            for (int b = 0; b < KB; ++b) ak[b] = lds16(lk + tt * 4096 + b * 1024);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                f32x4 x = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int b = 0; b < KB; ++b) x = mfma(ak[b], qb[nt][b], x);
                s[tt][nt] = x;
            }
        }
    };
    auto causal_mask = [&](f32x4 (&s)[2][NT], int k0) {
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (k0 + tt * 16 + 4 * r + i > qpos[nt]) s[tt][nt][i] = -INFINITY;
    };
    // raise the reference maximum (scaled log2 units) when a row's scores outgrow it by kRaisePf
    auto raise = [&](float lmax0, float lmax1) {
        const float lm[NT] = {lmax0, lmax1};
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            float full = fmaxf(lm[nt], __shfl_xor(lm[nt], 16, 64));
            full = fmaxf(full, __shfl_xor(full, 32, 64));
            const float m_new = fmaxf(m_ref[nt], full);
            const float alpha = __builtin_amdgcn_exp2f(m_ref[nt] - m_new);
#pragma unroll
            for (int b = 0; b < DB; ++b) acc[b][nt] *= alpha;
            accl[nt] *= alpha;
            m_ref[nt] = m_new;
        }
    };
    auto raise_if_needed = [&](float lmax0, float lmax1) {
        if (__any(lmax0 > m_ref[0] + kRaisePf || lmax1 > m_ref[1] + kRaisePf)) raise(lmax0, lmax1);
    };
    auto lane_max = [&](const f32x4 (&s)[2][NT], int nt) {
        float x = fmax3(s[0][nt][0], s[0][nt][1], s[0][nt][2]);
        x = fmax3(x, s[0][nt][3], s[1][nt][0]);
        x = fmax3(x, s[1][nt][1], s[1][nt][2]);
        return __builtin_fmaxf(x, s[1][nt][3]) * c;         // c > 0: the maximum commutes with the scale
    };
    auto weights_plain = [&](const f32x4 (&s)[2][NT], bf16x8 (&pop)[NT]) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const float nm = -m_ref[nt];
            uint32_t w[4];
#pragma unroll
            for (int ab = 0; ab < 2; ++ab) {
                const f32x4 x = s[ab][nt];
                const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(x[0], c, nm));
                const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(x[1], c, nm));
                const float p2 = __builtin_amdgcn_exp2f(__builtin_fmaf(x[2], c, nm));
                const float p3 = __builtin_amdgcn_exp2f(__builtin_fmaf(x[3], c, nm));
                w[2 * ab] = pack2(p0, p1);
                w[2 * ab + 1] = pack2(p2, p3);
            }
            pop[nt] = u4_bf16x8(make_uint4(w[0], w[1], w[2], w[3]));
        }
    };
    // O^T += V^T P^T (and the row sums) of one half-stage
    auto pv_plain = [&](const unsigned char* lv, const bf16x8 (&pop)[NT]) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) accl[nt] = mfma(ones, pop[nt], accl[nt]);
#pragma unroll
        for (int b = 0; b < DB; ++b) {
            const bf16x8 av = ldsv(lv + b * 512);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) acc[b][nt] = mfma(av, pop[nt], acc[b][nt]);
        }
    };

    // ---- steady state: half-stage h with h+1 unmasked --------------------------------------------------
    // in: scores of h (maximum already accounted for in m_ref), kpre: K operands of the first 16 tokens
    // of h+1.  out: scores of h+1; kpre: the same for h+2.
    auto fast_half = [&](int h, const f32x4 (&in)[2][NT], f32x4 (&out)[2][NT], bf16x8 (&kpre)[KB]) {
        const unsigned char* lk = kptr(h + 1);
        const unsigned char* lv = vptr(h);
        const unsigned char* lkn = kptr(h + 2);
        const float nm[NT] = {-m_ref[0], -m_ref[1]};
        bf16x8 k1[KB], av[DB], pop[NT];
        uint32_t w[NT][4];
        float p_even = 0.f;
        __builtin_amdgcn_sched_barrier(0);
        // 16 slots: MFMA j of K Q^T(h+1)  |  weight j of half-stage h
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int tt = j >> 3, b = (j >> 1) & 3, nt = j & 1;
            const f32x4 cin = b == 0 ? f32x4{0.f, 0.f, 0.f, 0.f} : out[tt][nt];
            out[tt][nt] = mfma(tt == 0 ? kpre[b] : k1[b], qb[nt][b], cin);
            if (j < 4) k1[j] = lds16(lk + 4096 + j * 1024);              // second 16 tokens of h+1
            if (j >= 8 && j < 12) av[j - 8] = ldsv(lv + (j - 8) * 512);
            const int ent = j >> 3, ab = (j >> 2) & 1, i = j & 3;
            const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(in[ab][ent][i], c, nm[ent]));
            if (i & 1) w[ent][2 * ab + (i >> 1)] = pack2(p_even, p); else p_even = p;
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) pop[nt] = u4_bf16x8(make_uint4(w[nt][0], w[nt][1], w[nt][2], w[nt][3]));
        // 18 slots: row sums and V^T P^T(h)  |  lane maxima of h+1, operand reads
        float lmax[NT] = {0.f, 0.f};
        unsigned long long vote = 0;                       // taken early: the branch at the end finds it in a scalar register
#pragma unroll
        for (int j = 0; j < 18; ++j) {
            if (j < 2) accl[j] = mfma(ones, pop[j], accl[j]);
            else acc[(j - 2) >> 1][j & 1] = mfma(av[(j - 2) >> 1], pop[j & 1], acc[(j - 2) >> 1][j & 1]);
            if (j < 4) av[4 + j] = ldsv(lv + (4 + j) * 512);
            if (j >= 8 && j < 12) kpre[j - 8] = lds16(lkn + (j - 8) * 1024);   // first 16 tokens of h+2
            if (j == 6) lmax[0] = lane_max(out, 0);
            if (j == 7) lmax[1] = lane_max(out, 1);
            if (j == 9) vote = __builtin_amdgcn_ballot_w64(lmax[0] > m_ref[0] + kRaisePf || lmax[1] > m_ref[1] + kRaisePf);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (vote != 0) raise(lmax[0], lmax[1]);
    };
    // ---- any other half-stage -----------------------------------------------------------------------------
    auto slow_half = [&](int h, const f32x4 (&in)[2][NT], f32x4 (&out)[2][NT]) {
        const bool next = h + 1 < hend;                    // wave-uniform
        if (next) {
            qk_plain(kptr(h + 1), out);
            if (h + 1 >= hfull) causal_mask(out, (h + 1) * kHalf);
        }
        bf16x8 pop[NT];
        weights_plain(in, pop);
        pv_plain(vptr(h), pop);
        if (next) raise_if_needed(lane_max(out, 0), lane_max(out, 1));
    };
    f32x4 sA[2][NT], sB[2][NT];
    bf16x8 kpre[KB];

    const int n_stage = (kv_hi + kStageTok - 1) / kStageTok;
    // Body i multiplies stages i and i+1 (the scores run one half-stage ahead); the barrier that ends
    // it publishes stage i+2.  bf16: the copy of stage i+3 is started at the top of body i, over stage
    // i-1 whose last reader finished before the barrier that ended body i-1, and is awaited at the end
    // of body i+1.  fp8: stage i+2 goes from registers into LDS at the top of body i, stage i+3 is
    // fetched into the registers.
    constexpr bool kCopy = sizeof(KT) == 2;
    // bf16: the stage that holds tokens >= ctx_len (if this tile reads it) needs its V tail cleared
    const int clear_stage = (kCopy && it.ctx_len % kStageTok != 0 && it.ctx_len / kStageTok < n_stage)
                                ? it.ctx_len / kStageTok : -1;
    StageFp8 st;
    auto top = [&](int i) {
        if constexpr (kCopy) {
            if (i + 3 < n_stage) stage_copy_bf16(a, bt, i + 3, last_page, g, wave, lane, lds);
        } else {
            if (i + 2 < n_stage) {
                stage_store(st, lds.k[(i + 2) % kPfRing], lds.v[(i + 2) % kPfRing], (i + 2) * kStageTok, it.ctx_len, tid);
                if (i + 3 < n_stage) stage_fetch(st, a, bt, (i + 3) * kStageTok, last_page, g, tid);
            }
        }
    };
    auto bottom = [&](int i) {
        if constexpr (kCopy) {
            // the copies of stage i+2 must have landed; those of stage i+3 (if any) may still fly
            if (i + 3 < n_stage) pf_wait_copies<kCopiesPerStage>(); else pf_wait_copies<0>();
        }
        __syncthreads();
        if (i + 2 == clear_stage) {                        // tile-uniform, at most once per tile
            clear_v_tail(lds.v[clear_stage % kPfRing], clear_stage, it.ctx_len, tid);
            __syncthreads();
        }
    };
    if constexpr (kCopy) {
        stage_copy_bf16(a, bt, 0, last_page, g, wave, lane, lds);
        if (n_stage > 1) stage_copy_bf16(a, bt, 1, last_page, g, wave, lane, lds);
        if (n_stage > 2) { stage_copy_bf16(a, bt, 2, last_page, g, wave, lane, lds); pf_wait_copies<kCopiesPerStage>(); }
        else pf_wait_copies<0>();
    } else {
        StageFp8 st1;
        stage_fetch(st, a, bt, 0, last_page, g, tid);
        if (n_stage > 1) stage_fetch(st1, a, bt, kStageTok, last_page, g, tid);
        stage_store(st, lds.k[0], lds.v[0], 0, it.ctx_len, tid);
        if (n_stage > 2) stage_fetch(st, a, bt, 2 * kStageTok, last_page, g, tid);
        if (n_stage > 1) stage_store(st1, lds.k[1], lds.v[1], kStageTok, it.ctx_len, tid);
    }
    __syncthreads();
    if (clear_stage == 0 || clear_stage == 1) {
        clear_v_tail(lds.v[clear_stage], clear_stage, it.ctx_len, tid);
        __syncthreads();
    }
    // scores of half-stage 0 (every wave has at least one half-stage: key 0 is visible to every row)
    qk_plain(kptr(0), sA);
    if (hfull == 0) causal_mask(sA, 0);
    raise_if_needed(lane_max(sA, 0), lane_max(sA, 1));
#pragma unroll
    for (int b = 0; b < KB; ++b) kpre[b] = lds16(kptr(1) + b * 1024);

    // Bodies in which every wave of the tile is in its steady state: half-stages up to 2i+2 lie
    // below the first query position of the tile (wave 0 has the smallest).
    const int hfull_tile = (it.prefix + it.tok_begin + 1) / kHalf;
    const int n_fast = max(0, (hfull_tile - 1) / 2);
    int i = 0;
    for (; i < n_fast; ++i) {
        top(i);
        fast_half(2 * i, sA, sB, kpre);
        fast_half(2 * i + 1, sB, sA, kpre);
        bottom(i);
    }
    // the last bodies: waves run out of visible keys one after the other
    for (; i < n_stage; ++i) {
        top(i);
        if (2 * i < hend) slow_half(2 * i, sA, sB);
        if (2 * i + 1 < hend) slow_half(2 * i + 1, sB, sA);
        bottom(i);
    }
    // (the last body ended with a barrier: lds may be reused by the caller)

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
            w.x = pack2(x[0], x[1]);
            w.y = pack2(x[2], x[3]);
            *(uint2*)(o + 16 * b) = w;
        }
    }
}

}  // namespace ts
