// Step a3 (device function shared by the prefill kernel and the persistent mixed kernel):
// causal attention of absorbed prefill chunks over the paged cache, on the matrix cores.
//
// A Convertible Decoder executes burst prefill requests as chunks next to its decode batch
// (paper Sec. 3.4, Sec. 4.4); a chunk row at position p attends to its cached prefix and to the
// chunk rows up to itself.  This part of the pass is a dense contraction (QK^T and PV), so it
// is tiled for MFMA:
//   - one workgroup (8 waves) owns a tile of 256 query rows = (256/G tokens) x (G query heads of
//     one KV head), so each K/V byte staged into LDS serves the whole head group; a wave owns 32
//     rows, one per lane pair (lane n and lane n + 32);
//   - KV is consumed in stages of 64 tokens (4 pages) that sit in a ring of four LDS slots; a
//     wave works through a stage in two half-stages of 32 tokens (2 pages);
//   - both products use the 32x32x16 MFMA: it occupies the matrix pipe for 32 cycles but the
//     vector issue port for 8, so 24 of every 32 cycles are free for the softmax arithmetic (the
//     16x16x32 form leaves 8 of 16, which is less than one exponential per MFMA needs);
//   - S^T = K Q^T (tokens x rows).  The 16-byte pieces of the K tiles are placed in LDS such that
//     row rho of S^T is the token for which the accumulator registers of a lane come out as
//     "8 consecutive tokens of the first page, then the same 8 of the second page": packed to
//     bf16 they are the B operands of O^T += V^T P^T as they stand, and the matching A operand is
//     one natural 16-byte piece (dim, 8 tokens) of the V tile;
//   - three half-stages are in flight per wave: while the matrix cores multiply K Q^T of
//     half-stage h+2 and V^T P^T of half-stage h, the vector ALU turns the scores of h+1 into
//     weights.  The instruction order of that steady state is written out slot by slot and pinned
//     with scheduling barriers (left to itself the compiler puts the phases one after the other);
//   - bf16 caches: the memory system copies the tiles straight into LDS (no registers, no vector
//     instructions); fp8 caches are widened to bf16 by the threads while being staged, so the
//     multiply loop is the same;
//   - the finished rows are normalised, packed to bf16 and passed through LDS once more, so that they
//     reach memory as whole 256-byte rows.
#pragma once
#include <type_traits>
#include "ts_device.h"

namespace ts {

constexpr float kRaisePf = 16.0f;
constexpr float kBigSum = 16.0f * 65536.0f;               // 16 weights of 2^kRaisePf
constexpr int kStageTok = 64;

__device__ __forceinline__ bf16x8 u4_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ uint2 fp8x4_bf16x4(uint32_t w)
{
    uint2 r;
    r.x = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, false));
    r.y = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, true));
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
// MFMA slots between the LDS read of an operand and its use (2..4).  Every slot of lookahead keeps four more
// registers per lane busy.  Three slots (measured: as fast as four) let the bf16 forms fit the 192 registers of
// the co-resident launch without spilling -- a spilled value is reloaded with a vector load, and the wait for
// it also waits for the stage copies in flight, which cost the co-resident launch 10 % --; the fp8 form, which
// also holds a prefetched stage in registers, takes two.
#ifndef TS_PF_LOOKAHEAD
#define TS_PF_LOOKAHEAD 3
#endif
#ifndef TS_PF_LOOKAHEAD_FP8
#define TS_PF_LOOKAHEAD_FP8 2
#endif
template <typename KT, bool WIDE> constexpr int kPfLookahead = sizeof(KT) == 1 ? TS_PF_LOOKAHEAD_FP8 : TS_PF_LOOKAHEAD;

// LDS image of a stage (bf16 in both cases): per page the 256 16-byte pieces of the cache tile,
// reordered.
//   K page: piece (dim chunk c, token slot s) at [c][swap23(s)]: the slot index with its bits 2 and
//           3 exchanged.  Row rho of the A operand of S^T = K Q^T reads [c][rho % 16] of page
//           rho / 16, so row rho is token 16 (rho / 16) + swap23(rho % 16) of the half-stage, and
//           the 16 accumulator registers of lane (n, h) are tokens 8h..8h+7 of the first page
//           followed by tokens 8h..8h+7 of the second.
//   V page: piece (dim d, token half t) at [d / 32][t][d % 32]: the A operand (32 dims x 16
//           tokens) of dim block b is 1 KB at lane * 16.
// Stage i lives in slot i % kPfRing of both rings.
// D = head dim (128 or 64): a page takes 32 D bytes in either ring.
template <int D>
struct __align__(16) PfLdsT {
    unsigned char k[kPfRing][4 * 32 * D];
    unsigned char v[kPfRing][4 * 32 * D];
};
using PfLds = PfLdsT<128>;
__device__ __forceinline__ int swap23(int s) { return (s & 3) | ((s & 4) << 1) | ((s & 8) >> 1); }
__device__ __forceinline__ int k_piece_offset(int chunk, int slot) { return (chunk * 16 + swap23(slot)) * 16; }
__device__ __forceinline__ int v_piece_offset(int dim, int half) { return (((dim >> 5) * 2 + half) * 32 + (dim & 31)) * 16; }

__device__ __forceinline__ uint32_t lds_address(const void* p)
{
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)p;
}

// ---- bf16 cache: the memory system copies a stage straight into LDS -------------------------------
// One instruction moves 64 x 16 bytes: lane l's piece lands at lds_addr + 16 l (the instruction offset
// advances both the global and the LDS address).  A wave moves 2 KB of K and 2 KB of V per stage:
// half of page `wave / 2` of the stage.  The copies are counted by vmcnt like any load; nothing here tells the
// compiler that LDS changes, so the caller waits (pf_wait_copies) and publishes with a barrier.
__device__ __forceinline__ void copy_2k_to_lds(uint32_t lds_addr, const void* base, uint32_t lane_off)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
                 "global_load_lds_dwordx4 %1, %2\n\t"
                 "global_load_lds_dwordx4 %1, %2 offset:1024\n"
                 :: "s"(lds_addr), "v"(lane_off), "s"(base) : "memory", "m0");
}
template <int OFF>
__device__ __forceinline__ void copy_1k_to_lds(uint32_t lds_addr, const void* base, uint32_t lane_off)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
                 "global_load_lds_dwordx4 %1, %2 offset:%3\n"
                 :: "s"(lds_addr), "v"(lane_off), "s"(base), "n"(OFF) : "memory", "m0");
}
__device__ __forceinline__ int copy_k_lane_offset(int lane) { return (lane >> 4) * 256 + swap23(lane & 15) * 16; }
__device__ __forceinline__ int copy_v_lane_offset(int lane) { return (lane & 31) * 32 + (lane >> 5) * 16; }
template <int D>
__device__ __forceinline__ void stage_copy_bf16(const char* kbase, const char* vbase, int Hkv, int stage, int page_id, int g,
                                                int wave, int lane, PfLdsT<D>& lds)
{
    constexpr int PB = 32 * D;                             // bytes of a page: a wave copies half a page of K and of V
    const int64_t off = ((int64_t)page_id * Hkv + g) * PB + (wave & 1) * (PB / 2);   // (page_id: of page 4 stage + wave / 2)
    const int slot = stage % kPfRing;
    // K: LDS piece [c0 + lane / 16][lane % 16] takes cache piece (c0 + lane / 16, swap23(lane % 16))
    // V: LDS piece [b0][lane / 32][lane % 32] takes cache piece (dim 32 b0 + lane % 32, half lane / 32)
    if constexpr (D == 128) {
        copy_2k_to_lds(lds_address(lds.k[slot]) + wave * (PB / 2), kbase + off, copy_k_lane_offset(lane));
        copy_2k_to_lds(lds_address(lds.v[slot]) + wave * (PB / 2), vbase + off, copy_v_lane_offset(lane));
    } else {
        copy_1k_to_lds<0>(lds_address(lds.k[slot]) + wave * (PB / 2), kbase + off, copy_k_lane_offset(lane));
        copy_1k_to_lds<0>(lds_address(lds.v[slot]) + wave * (PB / 2), vbase + off, copy_v_lane_offset(lane));
    }
}
template <int D> constexpr int kCopiesPerStage = D / 32;   // vmcnt units one stage_copy_bf16 adds per wave (1 KB each)
template <int N> __device__ __forceinline__ void pf_wait_copies()
{
    static_assert(N >= 0 && N < 16, "vmcnt immediate");
    __builtin_amdgcn_s_waitcnt(0x0f70 | N);                // vmcnt(N); expcnt and lgkmcnt untouched
}
// V rows of tokens at or beyond ctx_len hold whatever the cache page held (possibly NaN patterns):
// their weights are zero, but 0 x NaN is not, so they are cleared in LDS once the stage has landed.
template <int D>
__device__ __forceinline__ void clear_v_tail(unsigned char* lv, int stage, int ctx_len, int tid)
{
    if (tid >= 4 * D) return;                              // one thread per (page of the stage, dim)
    const int pg = tid / D, dim = tid % D;
    const int nvalid = ctx_len - (stage * kStageTok + pg * kPage);     // valid tokens of this page
    if (nvalid >= kPage) return;
    uint4* lo = (uint4*)(lv + pg * (32 * D) + v_piece_offset(dim, 0));
    uint4* hi = (uint4*)(lv + pg * (32 * D) + v_piece_offset(dim, 1));
    *lo = keep_first16(*lo, max(nvalid, 0));
    *hi = keep_first16(*hi, max(nvalid - 8, 0));
}

// ---- fp8 cache: 4 pages x 2048 bytes = 512 chunks of 16 bytes of K and of V, one each per thread,
// widened to bf16 on the way into LDS -------------------------------------------------------------
struct StageFp8 { uint4 k0, v0; };                          // (named members: arrays end up in scratch memory)
__device__ __forceinline__ void stage_fetch(StageFp8& st, const AttnArgs& a, int page_id, int g, int tid)
{
    const int64_t tile = (int64_t)page_id * a.geo.Hkv + g;        // (page_id: of page 4 stage + wave / 2)
    st.k0 = *(const uint4*)((const char*)a.k_cache + tile * 2048 + (tid & 127) * 16);
    st.v0 = *(const uint4*)((const char*)a.v_cache + tile * 2048 + (tid & 127) * 16);
}
__device__ __forceinline__ void stage_store(const StageFp8& st, unsigned char* lk, unsigned char* lv, int kv0,
                                            int ctx_len, int tid)
{
    const int pg = tid >> 7, c = tid & 127;
    // K chunk: 16 dims (chunk c/16) of token c%16 -> two bf16 pieces of 8 dims
    const int c16 = c >> 4, tok = c & 15;
    const uint4 k = st.k0;
    uint4 v = st.v0;
    const uint2 a0 = fp8x4_bf16x4(k.x), a1 = fp8x4_bf16x4(k.y), a2 = fp8x4_bf16x4(k.z), a3 = fp8x4_bf16x4(k.w);
    *(uint4*)(lk + pg * 4096 + k_piece_offset(2 * c16, tok)) = make_uint4(a0.x, a0.y, a1.x, a1.y);
    *(uint4*)(lk + pg * 4096 + k_piece_offset(2 * c16 + 1, tok)) = make_uint4(a2.x, a2.y, a3.x, a3.y);
    // V chunk: dim c, 16 tokens of page pg -> two pieces of 8 tokens
    const int nvalid = ctx_len - (kv0 + pg * kPage);
    if (nvalid < 16) v = keep_first8(v, max(nvalid, 0));             // poison past ctx_len -> 0
    const uint2 b0 = fp8x4_bf16x4(v.x), b1 = fp8x4_bf16x4(v.y), b2 = fp8x4_bf16x4(v.z), b3 = fp8x4_bf16x4(v.w);
    *(uint4*)(lv + pg * 4096 + v_piece_offset(c, 0)) = make_uint4(b0.x, b0.y, b1.x, b1.y);
    *(uint4*)(lv + pg * 4096 + v_piece_offset(c, 1)) = make_uint4(b2.x, b2.y, b3.x, b3.y);
}

// Order of the MFMAs of a steady-state iteration.  Values 0 .. NV-1 = V^T P^T step u (page u / DB, dim block
// u % DB; NV = 2 DB), NV .. NV+KS-1 = K Q^T step u - NV.  warm: the K operands of the first slots were read
// during the previous iteration; cold: the K stage has only just been published, so V^T P^T steps come first.
template <int D>
__device__ __forceinline__ constexpr int pf_slot_op(bool warm, int j)
{
    if constexpr (D == 128) {
        constexpr int kWarm[16] = {0, 8, 1, 9, 2, 10, 3, 11, 4, 12, 5, 13, 6, 14, 7, 15};
        constexpr int kCold[16] = {0, 1, 2, 8, 3, 9, 4, 10, 5, 11, 6, 12, 7, 13, 14, 15};
        return warm ? kWarm[j] : kCold[j];
    } else {
        constexpr int kWarm[8] = {0, 4, 1, 5, 2, 6, 3, 7};
        constexpr int kCold[8] = {0, 1, 2, 4, 3, 5, 6, 7};
        return warm ? kWarm[j] : kCold[j];
    }
}

// One causal tile for KV head g, executed by a workgroup of kPfThreads threads.  All threads must call
// it; it ends with a workgroup barrier, so lds may be reused right after it returns.
// tid: the thread's index in the workgroup (a caller that runs tiles in a loop passes an opaque copy, so
// that the many lane offsets derived from it are worked out per tile instead of being kept in registers
// across the loop).
// WIDE: KT is bf16 and the pages are the widened copies of an e4m3 cache.
// D: head dim, 128 or 64 (64: bf16 pages only -- a bf16 cache or widened copies).
template <typename KT, bool WIDE, int D = 128>
__device__ __forceinline__ void prefill_tile(const AttnArgs& a, int item_idx, int g, PfLdsT<D>& lds, int tid)
{
    constexpr int KS = D / 16, DB = D / 32, kHalf = 32;    // KS: 16-dim steps of K Q^T, DB: 32-dim blocks of O^T
    constexpr int PB = 32 * D;                             // bytes of a (bf16) page in LDS and in a bf16 cache
    constexpr int NV = 2 * DB, NSLOT = NV + KS;            // MFMAs of an iteration: V^T P^T steps, then both products
    constexpr int WPS = 16 / NSLOT;                        // weights formed per MFMA slot (1 or 2)
    static_assert(D == 128 || (D == 64 && sizeof(KT) == 2), "head dim 64 reads bf16 pages");
    static_assert(NSLOT * WPS == 16, "16 weights per lane and half-stage");
    // (through the constant address space: the tile's description is wave-uniform and belongs in scalar registers)
    const int32_t TS_CONSTANT* itp = as_constant((const int32_t*)(a.pf + item_idx));
    const PfItem it{itp[0], itp[1], itp[2], itp[3], itp[4], itp[5], itp[6], itp[7], itp[8], itp[9], 0, 0};
    // A tile cut along the keys works on the keys [kv_begin, kv_end) only.  Everything below is written in
    // positions relative to kv_begin (a multiple of 64: stage 0 of this item is stage kv_begin / 64 of the
    // sequence); every row of the tile sees key kv_begin, and only the last part reaches the diagonal.
    const int kv0 = it.kv_begin;
    const int ctx_rel = it.ctx_len - kv0;                  // keys of the sequence from kv_begin on
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, h = lane >> 5,
              n = lane & 31;
    const int Hq = a.geo.Hq, G = a.geo.G;

    // row of this lane pair: rho = 32*wave + n  ->  (token rho / G, head rho % G)
    const int rho = 32 * wave + n;
    const int t_raw = rho / G;
    const int tok = min(t_raw, it.tok_count - 1);          // padding rows repeat the last token
    const int hd = rho - t_raw * G;
    bf16x8 qb[KS];                                          // Q^T operands: dims 16 s + 8 h .. + 7 of the row
    {
        const uint16_t* qrow = (const uint16_t*)a.q +
            ((int64_t)(it.row0 + it.tok_begin + tok) * Hq + g * G + hd) * D + 8 * h;
#pragma unroll
        for (int s = 0; s < KS; ++s) qb[s] = u4_bf16x8(*(const uint4*)(qrow + 16 * s));
    }
    // KT is the element type the tile reads: e4m3 straight from the cache, or bf16 -- the cache itself, or the
    // copy of an e4m3 cache that was widened before the launch (then the scales still apply and the pages of
    // the sequence are numbered consecutively from wide_base[seq] instead of going through the block table)
    static_assert(!WIDE || sizeof(KT) == 2, "widened pages are bf16");
    constexpr bool fp8_cache = sizeof(KT) == 1 || WIDE;
    constexpr bool widened = WIDE;
    // (the scale of the exponent is wave-uniform: kept in a scalar register, it costs no vector register)
    const float kscale = fp8_cache ? as_constant(a.k_scale)[g] : 1.0f;
    const float c = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(a.sm_scale * kscale * kLog2e)));
    const int qpos = it.prefix + it.tok_begin + tok - kv0;
    const int wave_min_q = it.prefix + it.tok_begin + min((32 * wave) / G, it.tok_count - 1) - kv0;
    const int kv_hi = min(it.prefix + it.tok_begin + it.tok_count, it.kv_end) - kv0;   // keys [0, kv_hi) matter to this item
    const int last_page = (it.ctx_len - 1) / kPage;
    const int32_t TS_CONSTANT* bt = as_constant(a.block_table) + (int64_t)it.seq * a.geo.max_pages;
    const int wbase = widened ? as_constant(a.wide_base)[it.seq] : 0;
    const char* const kbase = (const char*)(widened ? a.wide_k : a.k_cache);
    const char* const vbase = (const char*)(widened ? a.wide_v : a.v_cache);
    // Half-stages [0, hend) hold keys that some row of the tile sees; every wave works through all of
    // them (a wave whose rows all come earlier multiplies one or two fully masked half-stages: that
    // keeps the eight waves in the same loop).  Half-stages [0, hfull) need no causal mask in this wave.
    const int hend = (kv_hi - 1) / kHalf + 1;
    const int hfull = (wave_min_q + 1) / kHalf;

    // O^T: register v of acc[b] is dim 32 b + 8 (v / 4) + 4 h + v % 4 of the lane's row
    f32x16 acc[DB];
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[b][v] = 0.f;
    float l_part = 0.f;                                    // this lane's half of the row's weight sum
    float m_ref = -INFINITY;                               // reference maximum of the row (scaled log2 units)

    // lane's operand addresses of half-stage hs inside the LDS rings.  K operand of dim step s:
    // 16 bytes at kptr + 512 s.  V operand of page t, dim block b: 16 bytes at vptr + PB t + 1024 b.
    auto kptr = [&](int hs) {
        return lds.k[(hs >> 1) % kPfRing] + (hs & 1) * (2 * PB) + (n >> 4) * PB + h * 256 + (n & 15) * 16;
    };
    auto vptr = [&](int hs) { return lds.v[(hs >> 1) % kPfRing] + (hs & 1) * (2 * PB) + lane * 16; };
    auto lds16 = [](const unsigned char* p) { return u4_bf16x8(*(const uint4*)p); };
    auto mfma = [](bf16x8 x, bf16x8 y, f32x16 z) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, z, 0, 0, 0); };
    auto pack2 = [](float x, float y) {
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{x, y}, bf16x2));
    };
    // register v of a score accumulator is token 16 (v / 8) + 8 h + v % 8 of the half-stage

    // ---- plain building blocks (first and last half-stages of a wave) -------------------------------
    // S^T = K Q^T of one half-stage (raw scores; the softmax scale is folded into the exponent)
    auto qk_plain = [&](const unsigned char* lk, f32x16& s) {
#pragma unroll
        for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) s = mfma(lds16(lk + ks * 512), qb[ks], s);
    };
    auto causal_mask = [&](f32x16& s, int k0) {
#pragma unroll
        for (int v = 0; v < 16; ++v)
            if (k0 + 16 * (v >> 3) + 8 * h + (v & 7) > qpos) s[v] = -INFINITY;
    };
    auto lane_max = [&](const f32x16& s) {
        float x = fmax3(s[0], s[1], s[2]);
        x = fmax3(x, s[3], s[4]);
        x = fmax3(x, s[5], s[6]);
        x = fmax3(x, s[7], s[8]);
        x = fmax3(x, s[9], s[10]);
        x = fmax3(x, s[11], s[12]);
        x = fmax3(x, s[13], s[14]);
        return __builtin_fmaxf(x, s[15]) * c;              // c > 0: the maximum commutes with the scale
    };
    // New reference maximum of the row; returns the factor that rescales everything accumulated so
    // far.  The weight sum is rescaled here, the caller rescales acc.
    auto raise = [&](float lmax) {
        const float full = pair32_max(lmax);                 // the row's other half sits in lane ^ 32
        const float m_new = fmaxf(m_ref, full);
        const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);
        l_part *= alpha;
        m_ref = m_new;
        return alpha;
    };
    auto rescale = [&](float alpha) {
#pragma unroll
        for (int b = 0; b < DB; ++b) acc[b] *= alpha;
    };
    // weights of one half-stage: P^T operands of its two pages, and their sum
    auto weights_plain = [&](const f32x16& s, bf16x8 (&pop)[2]) {
        const float nm = -m_ref;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            uint32_t w[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[8 * t + 2 * i], c, nm));
                const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[8 * t + 2 * i + 1], c, nm));
                l_part += p0 + p1;
                w[i] = pack2(p0, p1);
            }
            pop[t] = u4_bf16x8(make_uint4(w[0], w[1], w[2], w[3]));
        }
    };
    // O^T += V^T P^T of one half-stage
    auto pv_plain = [&](const unsigned char* lv, const bf16x8 (&pop)[2]) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int b = 0; b < DB; ++b) acc[b] = mfma(lds16(lv + t * PB + b * 1024), pop[t], acc[b]);
    };

    // ---- steady state: one iteration = V^T P^T of half-stage hs and K Q^T of hs+2 on the matrix
    // cores, weights of hs+1 on the vector ALU.  s1: scores of hs+1 (in), s2: scores of hs+2 (out),
    // pop0: weights of hs (in), pop1: weights of hs+1 (out).  16 slots of one MFMA each; a slot also
    // carries one weight (fused multiply-add, exp2, add to the sum, running maximum; every other slot
    // a pack) and the LDS read of the operand needed four slots later.  The operands of the first
    // slots arrive in vpre / kpre, read during the previous iteration; those of the next iteration
    // are read during the last slots.  K operands cannot be read ahead across the barrier that
    // publishes their stage: the first iteration of a body (KIN false) reads them at its top and
    // starts with three V^T P^T slots.
    //
    // bf16 caches: the four copy instructions with which a wave brings in its part of the next stage are
    // issued from four slots of the first iteration of a body (DMA true).  Issued together at the top of
    // the body, right after the barrier, the 32 copies of the workgroup fill the queue of the memory
    // pipeline and every wave waits until its own have been accepted (measured: 0.11-0.17 us per body).
    uint32_t cp_lds_k = 0, cp_lds_v = 0;                   // set by top(): where the copy goes ...
    const char* cp_k = nullptr;                            // ... and what it reads (wave-uniform)
    const char* cp_v = nullptr;
    const int cp_k_src = copy_k_lane_offset(lane), cp_v_src = copy_v_lane_offset(lane);
    auto copy_quarter = [&](int q) {                       // q < kCopiesPerStage<D>: one 1 KB copy each
        if constexpr (D == 128) {
            if (q == 0) copy_1k_to_lds<0>(cp_lds_k, cp_k, cp_k_src);
            if (q == 1) copy_1k_to_lds<1024>(cp_lds_k, cp_k, cp_k_src);
            if (q == 2) copy_1k_to_lds<0>(cp_lds_v, cp_v, cp_v_src);
            if (q == 3) copy_1k_to_lds<1024>(cp_lds_v, cp_v, cp_v_src);
        } else {
            if (q == 0) copy_1k_to_lds<0>(cp_lds_k, cp_k, cp_k_src);
            if (q == 1) copy_1k_to_lds<0>(cp_lds_v, cp_v, cp_v_src);
        }
    };
    bf16x8 vpre[3], kpre[2];
    auto fast_iter = [&](auto kin_tag, auto kout_tag, auto dma_tag, int hs, bool masked, const f32x16& s1, f32x16& s2,
                         const bf16x8 (&pop0)[2], bf16x8 (&pop1)[2]) {
        constexpr bool KIN = decltype(kin_tag)::value, KOUT = decltype(kout_tag)::value, DMA = decltype(dma_tag)::value;
        const unsigned char* lk = kptr(hs + 2);
        const unsigned char* lv = vptr(hs);
        const unsigned char* lvn = vptr(hs + 1);
        const unsigned char* lkn = kptr(hs + 3);
        auto v_at = [&](const unsigned char* base, int u) { return lds16(base + (u / DB) * PB + (u % DB) * 1024); };
        // The weights of hs+1 are formed against the current reference maximum without looking at the
        // scores first; their sum shows afterwards whether one of them was above 2^kRaisePf, i.e. that
        // the maximum has to be raised (a sum above 16 x 2^kRaisePf needs such a weight; larger weights
        // that stay below it are harmless: the bound only keeps the sums far from overflow), and only
        // then are the weights of this half-stage formed again (the scores are still there).
        const float nm = -m_ref;
        const float l_before = l_part;
        bf16x8 kop[KS], vop[NV];
        uint32_t w[8];
        constexpr int LA = kPfLookahead<KT, WIDE>;
        __builtin_amdgcn_sched_barrier(0);
        // operands of the first LA slots: read during the previous iteration (V always, K only where the
        // stage was already published: KIN), else here
#pragma unroll
        for (int p = 0; p < LA; ++p) {
            const int op = pf_slot_op<D>(KIN, p);
            if (op < NV) vop[op] = vpre[op];
            else if constexpr (KIN) kop[op - NV] = kpre[op - NV];
            else kop[op - NV] = lds16(lk + (op - NV) * 512);
        }
        // The weight arithmetic is spread over the slots such that no instruction uses a result of its
        // own step: step i scales score i+1, takes the exponential of score i, adds weight i-1 to the
        // row sum and (even i) packs the weights i-2 and i-1; a slot carries WPS steps (one with 16 MFMAs per
        // iteration, two with 8).  Only instructions that measurably run in the shadow of an MFMA for free are
        // used here (fma, exp, add, pack; the bf16 dot-product instruction, which would sum two packed weights
        // at once, is not one of them: it delays the MFMAs of the SIMD).
        float t_next = __builtin_fmaf(s1[0], c, nm);
        float p_a = 0.f, p_b = 0.f;                        // the two most recent weights
        auto weight_step = [&](int i) {
            if (i >= 1) {
                l_part += (i & 1) ? p_a : p_b;             // weight i-1
                asm volatile("" : "+v"(l_part));           // (keeps the instruction in this slot)
                if (!(i & 1)) {
                    w[(i - 2) >> 1] = pack2(p_a, p_b);
                    asm volatile("" : "+v"(w[(i - 2) >> 1]));
                }
            }
            const float t_cur = t_next;
            if (i + 1 < 16) t_next = __builtin_fmaf(s1[i + 1], c, nm);
            const float p = __builtin_amdgcn_exp2f(t_cur);
            if (i & 1) p_b = p; else p_a = p;
        };
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < NSLOT; ++j) {
            const int op = pf_slot_op<D>(KIN, j);
            if (op < NV) {
                acc[op % DB] = mfma(vop[op], pop0[op / DB], acc[op % DB]);
            } else {
                if (op == NV) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) s2[v] = 0.f;
                }
                s2 = mfma(kop[op - NV], qb[op - NV], s2);
            }
            // read the operand of the MFMA LA slots on; the last LA slots read the first operands of the next
            // iteration (its K operands only if their stage is already published: KOUT)
            if (j + LA < NSLOT) {
                const int nx = pf_slot_op<D>(KIN, j + LA);
                if (nx < NV) vop[nx] = v_at(lv, nx);
                else kop[nx - NV] = lds16(lk + (nx - NV) * 512);
            } else {
                const int nx = pf_slot_op<D>(KOUT, j + LA - NSLOT);
                if (nx < NV) vpre[nx] = v_at(lvn, nx);
                else if constexpr (KOUT) kpre[nx - NV] = lds16(lkn + (nx - NV) * 512);
            }
#pragma unroll
            for (int k = 0; k < WPS; ++k) weight_step(j * WPS + k);
            if constexpr (DMA) {
                if ((j & 3) == 3 && (j >> 2) < kCopiesPerStage<D>) copy_quarter(j >> 2);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        l_part += p_b;
        w[7] = pack2(p_a, p_b);
        pop1[0] = u4_bf16x8(make_uint4(w[0], w[1], w[2], w[3]));
        pop1[1] = u4_bf16x8(make_uint4(w[4], w[5], w[6], w[7]));
        if (__any(!(l_part - l_before <= kBigSum))) {      // rare; also catches infinities and NaN
            l_part = l_before;
            const float alpha = raise(lane_max(s1));
            weights_plain(s1, pop1);
            rescale(alpha);                                // everything up to half-stage hs was relative to the old maximum
        }
        if (masked) causal_mask(s2, (hs + 2) * kHalf);     // wave-uniform
    };
    // ---- any other iteration --------------------------------------------------------------------------
    auto slow_iter = [&](int hs, const f32x16& s1, f32x16& s2, const bf16x8 (&pop0)[2], bf16x8 (&pop1)[2]) {
        pv_plain(vptr(hs), pop0);
        if (hs + 1 < hend) {                               // wave-uniform
            const float lmax = lane_max(s1);
            if (__any(lmax > m_ref + kRaisePf)) rescale(raise(lmax));
            weights_plain(s1, pop1);
        }
        if (hs + 2 < hend) {
            qk_plain(kptr(hs + 2), s2);
            if (hs + 2 >= hfull) causal_mask(s2, (hs + 2) * kHalf);
        }
    };

    const int n_stage = (kv_hi + kStageTok - 1) / kStageTok;
    // Body i runs iterations 2i and 2i+1: it reads V of stage i and K of stage i+1.  The barrier that
    // ends it publishes stage i+2.  bf16: the copy of stage i+3 is started at the top of body i, over
    // stage i-1 whose last reader finished before the barrier that ended body i-1, and is awaited at
    // the end of body i+1.  fp8: stage i+2 goes from registers into LDS at the top of body i, stage
    // i+3 is fetched into the registers.
    constexpr bool kCopy = sizeof(KT) == 2;
    // bf16: the stage that holds tokens >= ctx_len (if this tile reads it) needs its V tail cleared
    const int clear_stage = (kCopy && ctx_rel % kStageTok != 0 && ctx_rel / kStageTok < n_stage)
                                ? ctx_rel / kStageTok : -1;
    StageFp8 st;
    // Page of a stage this wave stages (a tile that ends inside the last page of the sequence repeats that
    // page).  The id comes through the scalar cache.  Read where it is used, the latency of that
    // dependent load would hold up every wave of the workgroup right after the barrier, when no wave
    // has anything else to issue; so the id that top(i+1) needs is requested between the two iterations
    // of body i, where the wait for it falls into a phase in which the other wave of the SIMD has work.
    auto page_id = [&](int stage) {
        const int j = min((kv0 >> 4) + stage * 4 + (wave >> 1), last_page);
        return widened ? wbase + j : bt[j];
    };
    int32_t pid_next;                                      // page id top(i) needs: that of stage i + 3
    // top(i), bf16: a steady body always copies "stage i+3" into the ring slot of stage i-1, whose last
    // reader finished before the barrier that ended body i-1; beyond the last stage that is the last
    // page again (nobody reads it).  The bodies of the draining loop copy nothing.
    auto top = [&](int i) {
        if constexpr (kCopy) {
            const int64_t off = ((int64_t)pid_next * a.geo.Hkv + g) * PB + (wave & 1) * (PB / 2);
            cp_lds_k = lds_address(lds.k[(i + 3) % kPfRing]) + wave * (PB / 2);
            cp_lds_v = lds_address(lds.v[(i + 3) % kPfRing]) + wave * (PB / 2);
            cp_k = kbase + off;
            cp_v = vbase + off;
        } else {
            if (i + 2 < n_stage) {
                // (the thread index goes through an opaque copy: the LDS and cache offsets derived from it are
                // then worked out here, once per body, instead of occupying six registers for the whole tile)
                int t = tid;
                asm volatile("" : "+v"(t));
                stage_store(st, lds.k[(i + 2) % kPfRing], lds.v[(i + 2) % kPfRing], (i + 2) * kStageTok, ctx_rel, t);
                if (i + 3 < n_stage) stage_fetch(st, a, pid_next, g, t);
            }
        }
    };
    auto request_page_id = [&](int i) {                    // between the two iterations of body i
        __builtin_amdgcn_sched_barrier(0);
        pid_next = page_id(i + 4);
        __builtin_amdgcn_sched_barrier(0);
    };
    auto bottom = [&](int i, auto steady_tag) {
        if constexpr (kCopy) {
            // the copies of stage i+2 must have landed; those this body issued (steady bodies) may still fly
            if constexpr (decltype(steady_tag)::value) pf_wait_copies<kCopiesPerStage<D>>(); else pf_wait_copies<0>();
        }
        __syncthreads();
        if constexpr (kCopy) {
            if (i + 2 == clear_stage) {                    // tile-uniform, at most once per tile
                clear_v_tail<D>(lds.v[clear_stage % kPfRing], clear_stage, ctx_rel, opaque(tid));
                __syncthreads();
            }
        }
    };
    if constexpr (kCopy) {
        const int32_t p0 = page_id(0), p1 = page_id(1), p2 = page_id(2);
        pid_next = page_id(3);
        stage_copy_bf16(kbase, vbase, a.geo.Hkv, 0, p0, g, wave, lane, lds);
        if (n_stage > 1) stage_copy_bf16(kbase, vbase, a.geo.Hkv, 1, p1, g, wave, lane, lds);
        if (n_stage > 2) { stage_copy_bf16(kbase, vbase, a.geo.Hkv, 2, p2, g, wave, lane, lds); pf_wait_copies<kCopiesPerStage<D>>(); }
        else pf_wait_copies<0>();
    } else {
        const int32_t p0 = page_id(0), p1 = page_id(1), p2 = page_id(2);
        pid_next = page_id(3);
        StageFp8 st1;
        stage_fetch(st, a, p0, g, tid);
        if (n_stage > 1) stage_fetch(st1, a, p1, g, tid);
        stage_store(st, lds.k[0], lds.v[0], 0, ctx_rel, tid);
        if (n_stage > 2) stage_fetch(st, a, p2, g, tid);
        if (n_stage > 1) stage_store(st1, lds.k[1], lds.v[1], kStageTok, ctx_rel, tid);
    }
    __syncthreads();
    if constexpr (kCopy) {
        if (clear_stage == 0 || clear_stage == 1) {
            clear_v_tail<D>(lds.v[clear_stage], clear_stage, ctx_rel, opaque(tid));
            __syncthreads();
        }
    }

    // Fill the pipeline: weights of half-stage 0 and scores of half-stage 1 (every wave has at least
    // one half-stage: key 0 is visible to every row).
    f32x16 sA, sB;
    bf16x8 popA[2], popB[2];
    qk_plain(kptr(0), sB);
    if (hfull == 0) causal_mask(sB, 0);
    raise(lane_max(sB));                                   // acc is still zero: nothing to rescale
    weights_plain(sB, popA);
    if (hend > 1) {
        qk_plain(kptr(1), sA);
        if (hfull <= 1) causal_mask(sA, kHalf);
    }

    // Bodies whose iterations all have a half-stage hs+2 to multiply run the steady state: first those
    // that lie below the first query position of the tile (no wave needs a mask), then those that
    // reach into the diagonal; the last one or two bodies drain the pipeline.
    const int hfull_tile = (it.prefix + it.tok_begin + 1 - kv0) / kHalf;
    const int n_steady = max(0, (hend - 2) / 2);           // 2i+3 < hend
    // (a part of a cut tile that ends below the diagonal has no masked body at all)
    const int n_plain = min(n_steady, max(0, (hfull_tile - 2) / 2));      // 2i+3 < hfull_tile
    int i = 0;
    constexpr std::true_type yes{};
    constexpr std::false_type no{};
    constexpr std::bool_constant<kCopy> dma{};
    {                                                      // V operands of the first slots of the first iteration
#pragma unroll
        for (int p = 0; p < kPfLookahead<KT, WIDE>; ++p) {
            const int op = pf_slot_op<D>(false, p);
            if (op < NV) vpre[op] = lds16(vptr(0) + (op / DB) * PB + (op % DB) * 1024);
        }
    }
    for (; i < n_plain; ++i) {
        top(i);
        fast_iter(no, yes, dma, 2 * i, false, sA, sB, popA, popB);
        request_page_id(i);
        fast_iter(yes, no, no, 2 * i + 1, false, sB, sA, popB, popA);
        bottom(i, yes);
    }
    for (; i < n_steady; ++i) {
        top(i);
        fast_iter(no, yes, dma, 2 * i, 2 * i + 2 >= hfull, sA, sB, popA, popB);
        request_page_id(i);
        fast_iter(yes, no, no, 2 * i + 1, 2 * i + 3 >= hfull, sB, sA, popB, popA);
        bottom(i, yes);
    }
    for (; i < n_stage; ++i) {
        if constexpr (!kCopy) top(i);
        if (2 * i < hend) slow_iter(2 * i, sA, sB, popA, popB);
        if (2 * i + 1 < hend) slow_iter(2 * i + 1, sB, sA, popB, popA);
        bottom(i, no);
    }
    // The last body ended with a barrier and no copy is in flight: LDS is free.  The rows leave through it:
    // a lane holds 4-dim pieces of its row (8 bytes each), written directly they would reach memory
    // as 16 stores of 32 scattered 16-byte runs per wave; staged in LDS (row stride 272 bytes), 16 lanes
    // store one whole 256-byte row as 16-byte pieces and an instruction covers 4 rows.
    // (Lane indices are derived afresh from an opaque copy of the thread index: nothing of this stage then
    // occupies a register during the loops above.)
    if (it.part >= 0) {
        // One part of a tile cut along the keys: the unnormalised rows and their (reference maximum, weight sum)
        // go to the partial-result buffers as they are; prefill_combine_kernel merges the parts.
        const int tid_o = opaque(tid), wave_o = __builtin_amdgcn_readfirstlane(tid_o >> 6), lane_o = tid_o & 63,
                  h_o = lane_o >> 5, n_o = lane_o & 31;
        const int64_t slot = ((int64_t)it.part * a.geo.Hkv + g) * kPfPartRows + 32 * wave_o + n_o;
        float* po = a.pf_part_o + slot * D + 4 * h_o;
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                *(f32x4*)(po + 32 * b + 8 * j) = f32x4{acc[b][4 * j], acc[b][4 * j + 1], acc[b][4 * j + 2], acc[b][4 * j + 3]};
        const float l_row = pair32_sum(l_part);
        if (h_o == 0) *(float2*)(a.pf_part_ml + slot * 2) = make_float2(m_ref, l_row);
        __syncthreads();                                   // LDS may be reused by the caller
        return;
    }
    constexpr int kOutStride = 2 * D + 16;                 // bytes of a staged row (16 bytes of padding against bank conflicts)
    constexpr int kLanesPerRow = D / 8, kRowsPerStep = 64 / kLanesPerRow;
    const int tid_o = opaque(tid), wave_o = __builtin_amdgcn_readfirstlane(tid_o >> 6), lane_o = tid_o & 63,
              h_o = lane_o >> 5, n_o = lane_o & 31;
    unsigned char* ob = (unsigned char*)&lds + wave_o * (32 * kOutStride);
    const float vscale = fp8_cache ? as_constant(a.v_scale)[g] : 1.0f;
    const float l_row = pair32_sum(l_part);
    const float inv = vscale / l_row;
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint2 w;
            w.x = pack2(acc[b][4 * j] * inv, acc[b][4 * j + 1] * inv);
            w.y = pack2(acc[b][4 * j + 2] * inv, acc[b][4 * j + 3] * inv);
            *(uint2*)(ob + n_o * kOutStride + 64 * b + 16 * j + 8 * h_o) = w;
        }
    __builtin_amdgcn_wave_barrier();                       // (the rows are read back by other lanes of this wave)
    const float inv_g = 1.0f / (float)opaque_uniform(G);
#pragma unroll
    for (int i = 0; i < 32 / kRowsPerStep; ++i) {
        const int r = kRowsPerStep * i + lane_o / kLanesPerRow;    // row of the wave, D / 8 lanes per row
        const int piece = lane_o % kLanesPerRow;
        const int rho_r = 32 * wave_o + r;
        const int t_r = (int)(((float)rho_r + 0.5f) * inv_g);      // rho_r / G (exact for rho_r < 256, G <= 16)
        const int hd_r = rho_r - t_r * G;
        const uint4 v = *(const uint4*)(ob + r * kOutStride + piece * 16);
        if (t_r < it.tok_count) {
            uint16_t* o = (uint16_t*)a.out + ((int64_t)(it.row0 + it.tok_begin + t_r) * Hq + g * G + hd_r) * D;
            *(uint4*)(o + piece * 8) = v;
        }
    }
    __syncthreads();                                       // LDS may be reused by the caller
}

}  // namespace ts
