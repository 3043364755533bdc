// Step a1: write the iteration's new K/V rows into the paged cache.
//
// Prefill builds cache entries for all input tokens, a decode iteration adds the entry of the
// last token (paper Sec. 2.1); in a Convertible Decoder both kinds of rows arrive in one batch
// (Sec. 3.4).  Two kernels:
//   - append_token_kernel: one workgroup per new token of a short sequence (decode rows): looks up the
//     token's page and slot and scatters its Hkv x D values of K (16-byte dim-chunks) and V
//     (token-fastest tile) into place.  The copy of the call's work lists from the pinned staging
//     buffer to device memory can ride along as extra workgroups of the same launch (a launch costs
//     more than either job: a decode step then has one kernel less in front of the scan);
//   - append_tile_kernel: one workgroup per (cache page, KV head) of a chunk: loads the page's up
//     to 16 new rows with full 256-byte reads, turns them into the K tile and -- through LDS --
//     into the token-fastest V tile, and writes whole 16-byte vectors.  (Scattering a chunk token
//     by token wrote 5.5x the new bytes: every 2-byte V element dirtied its own cache sector.)
// Both convert to the cache element type with the same functions, so the bytes are identical.
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
__global__ __launch_bounds__(256) void append_token_kernel(AppendArgs a)
{
    if ((int)blockIdx.x >= a.n_apr) {                  // work-list upload riding along
        const int64_t stride = (int64_t)a.up_blocks * blockDim.x;
        for (int64_t i = (int64_t)(blockIdx.x - a.n_apr) * blockDim.x + threadIdx.x; i < a.up_n16; i += stride)
            ((uint4*)a.up_dst)[i] = ((const uint4*)a.up_src)[i];
        return;
    }
    const AppRow r = a.apr[blockIdx.x];
    const int row = r.row, pos = r.pos;
    const int Hkv = a.geo.Hkv, D = a.geo.D;
    constexpr int X = 16 / (int)sizeof(DST);       // elements per 16-byte dim-chunk
    const int n_elems = Hkv * D;
    const SRC* ks = (const SRC*)a.k_new + (int64_t)row * n_elems;
    const SRC* vs = (const SRC*)a.v_new + (int64_t)row * n_elems;
    DST* kc = (DST*)a.k_cache;
    DST* vc = (DST*)a.v_cache;
    // (the values are requested before the page id is needed: the two loads wait together)
    const int32_t* page_ptr = a.block_table + (int64_t)r.seq * a.geo.max_pages + (pos >> 4);
    const int slot = pos & 15;
    for (int e0 = 0; e0 < n_elems; e0 += 4 * 256) {
        SRC kv[4], vv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = e0 + i * 256 + threadIdx.x;
            kv[i] = e < n_elems ? ks[e] : SRC(0);
            vv[i] = e < n_elems ? vs[e] : SRC(0);
        }
        const int64_t page = *page_ptr;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = e0 + i * 256 + threadIdx.x;
            if (e >= n_elems) continue;
            const int g = e / D, dim = e - g * D;
            const int64_t tile = tile_elem_base(page, Hkv, g, D);
            const int64_t kidx = tile + (dim / X) * (kPage * X) + slot * X + (dim % X);
            const int64_t vidx = tile + dim * kPage + slot;
            if constexpr (sizeof(DST) == 1) {
                const float kf = Elem<SRC>::load(&kv[i], 0) / a.k_scale[g];
                const float vf = Elem<SRC>::load(&vv[i], 0) / a.v_scale[g];
                __builtin_nontemporal_store((uint8_t)float_to_e4m3_bits(kf), &kc[kidx]);
                __builtin_nontemporal_store((uint8_t)float_to_e4m3_bits(vf), &vc[vidx]);
            } else {
                __builtin_nontemporal_store((DST)kv[i], &kc[kidx]);   // same element type: plain copy of the bits
                __builtin_nontemporal_store((DST)vv[i], &vc[vidx]);
            }
        }
    }
}

// Sixteen fp32 values -> sixteen e4m3 bytes (four words, value i in byte i % 4 of word i / 4), the same bytes as
// float_to_e4m3_bits gives.  The hardware conversion (two values per instruction, nearest-even, denormals and
// -0 as the definition wants) answers a value beyond the format's range, and any NaN, with the byte 0xFF; for
// every one of the 2^32 inputs it agrees with float_to_e4m3_bits once the value has been clamped to +-448,
// except on NaNs (compared exhaustively on the GPU).  So: clamp, convert, and take the integer encoder when
// any lane of the wave holds a NaN (rare; the branch is wave-uniform).
__device__ __forceinline__ void encode_e4m3x16(const float (&x)[16], uint32_t (&w)[4])
{
    bool nan = false;
#pragma unroll
    for (int i = 0; i < 16; ++i) nan |= x[i] != x[i];
    if (__any(nan)) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            w[j] = float_to_e4m3_bits(x[4 * j]) | (float_to_e4m3_bits(x[4 * j + 1]) << 8) |
                   (float_to_e4m3_bits(x[4 * j + 2]) << 16) | (float_to_e4m3_bits(x[4 * j + 3]) << 24);
        return;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float a = __builtin_amdgcn_fmed3f(x[4 * j], -448.0f, 448.0f), b = __builtin_amdgcn_fmed3f(x[4 * j + 1], -448.0f, 448.0f);
        const float c = __builtin_amdgcn_fmed3f(x[4 * j + 2], -448.0f, 448.0f), d = __builtin_amdgcn_fmed3f(x[4 * j + 3], -448.0f, 448.0f);
        int v = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false);
        v = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, v, true);
        w[j] = (uint32_t)v;
    }
}

// bf16 source rows, head dim D = 64 or 128; DST = uint16_t (bf16 cache) or uint8_t (e4m3 cache).
// Thread (t = tid / (D/8), c = tid % (D/8)) loads the 16 bytes (dims 8c .. 8c+7) of slot t's K and V row
// (head dim 64: the first 128 threads).
template <typename DST, int D>
__global__ __launch_bounds__(256) void append_tile_kernel(AppendArgs a)
{
    constexpr int CPR = D / 8;                         // 16-byte pieces per source row
    constexpr int kRowPad = D + 8;                     // LDS row stride in elements: avoids bank conflicts
    __shared__ __align__(16) uint16_t ks[16 * kRowPad];
    __shared__ __align__(16) uint16_t vs[16 * kRowPad];
    const int Hkv = a.geo.Hkv;
    if ((int)blockIdx.x >= a.n_apt * Hkv) {            // work-list upload riding along
        const int64_t stride = (int64_t)a.up_blocks * blockDim.x;
        for (int64_t i = (int64_t)(blockIdx.x - a.n_apt * Hkv) * blockDim.x + threadIdx.x; i < a.up_n16; i += stride)
            ((uint4*)a.up_dst)[i] = ((const uint4*)a.up_src)[i];
        return;
    }
    const int g = blockIdx.x % Hkv;
    const AppTile it = a.apt[blockIdx.x / Hkv];
    const int tid = threadIdx.x, t = tid / CPR, c = tid % CPR;
    const bool loader = tid < kPage * CPR;
    const int64_t page = a.block_table[(int64_t)it.seq * a.geo.max_pages + it.page_idx];
    const bool mine = loader && t >= it.slot_lo && t < it.slot_hi;
    uint4 kv = make_uint4(0, 0, 0, 0), vv = kv;
    if (mine) {
        const int64_t src = ((int64_t)(it.row_slot0 + t) * Hkv + g) * D + 8 * c;
        kv = *(const uint4*)((const uint16_t*)a.k_new + src);
        vv = *(const uint4*)((const uint16_t*)a.v_new + src);
    }
    if (loader) {
        *(uint4*)(vs + t * kRowPad + 8 * c) = vv;
        if constexpr (sizeof(DST) == 1) *(uint4*)(ks + t * kRowPad + 8 * c) = kv;
    }
    __syncthreads();
    const bool full = it.slot_lo == 0 && it.slot_hi == kPage;

    if constexpr (sizeof(DST) == 2) {
        uint16_t* kt = (uint16_t*)a.k_cache + tile_elem_base(page, Hkv, g, D);
        uint16_t* vt = (uint16_t*)a.v_cache + tile_elem_base(page, Hkv, g, D);
        // K tile [D/8 chunks][16 slots][8]: this thread's own 16 bytes
        if (mine) store_nt(kt + (c * 16 + t) * 8, kv);
        // V tile [D dims][16 slots]: thread (dim = tid / 2, half = tid % 2) gathers 8 slots of one dim
        const int dim = tid >> 1, hf = tid & 1;
        if (dim < D) {
            uint16_t e[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) e[i] = vs[(8 * hf + i) * kRowPad + dim];
            uint16_t* dst = vt + dim * kPage + 8 * hf;
            if (full) {
                store_nt(dst, make_uint4(e[0] | ((uint32_t)e[1] << 16), e[2] | ((uint32_t)e[3] << 16),
                                         e[4] | ((uint32_t)e[5] << 16), e[6] | ((uint32_t)e[7] << 16)));
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if (8 * hf + i >= it.slot_lo && 8 * hf + i < it.slot_hi) __builtin_nontemporal_store(e[i], &dst[i]);
            }
        }
    } else {
        uint8_t* kt = (uint8_t*)a.k_cache + tile_elem_base(page, Hkv, g, D);
        uint8_t* vt = (uint8_t*)a.v_cache + tile_elem_base(page, Hkv, g, D);
        const float kscale = a.k_scale[g], vscale = a.v_scale[g];
        if (tid < D) {
            // K tile [D/16 chunks of 16 dims][16 slots][16]: thread (chunk = tid / 16, slot = tid % 16)
            const int c16 = tid >> 4, slot = tid & 15;
            if (slot >= it.slot_lo && slot < it.slot_hi) {
                float x[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) x[i] = bf16_bits_to_float(ks[slot * kRowPad + 16 * c16 + i]) / kscale;
                uint32_t w[4];
                encode_e4m3x16(x, w);
                store_nt(kt + (c16 * 16 + slot) * 16, make_uint4(w[0], w[1], w[2], w[3]));
            }
        } else if (tid < 2 * D) {
            // V tile [D dims][16 slots]: thread dim = tid - D gathers the 16 slots of one dim
            const int dim = tid - D;
            float x[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) x[i] = bf16_bits_to_float(vs[i * kRowPad + dim]) / vscale;
            uint32_t w[4];
            encode_e4m3x16(x, w);
            uint8_t* dst = vt + dim * kPage;
            if (full) {
                store_nt(dst, make_uint4(w[0], w[1], w[2], w[3]));
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    if (i >= it.slot_lo && i < it.slot_hi)
                        __builtin_nontemporal_store((uint8_t)(w[i >> 2] >> (8 * (i & 3))), &dst[i]);
            }
        }
    }
}

int launch_append(const AppendArgs& args, void* stream)
{
    if (args.total_tokens <= 0) return (int)hipSuccess;
    hipStream_t st = (hipStream_t)stream;
    dim3 block(256);
    AppendArgs a = args;
    // the upload (if any) rides in the first launch, which then reads its own list from the staging buffer
    if (a.up_blocks > 0) {
        if (a.n_apr > 0) a.apr = a.apr_host; else a.apt = a.apt_host;
    }
    if (a.n_apr > 0) {
        dim3 grid((unsigned)(a.n_apr + a.up_blocks));
        if (a.geo.q_dtype == TS_F32 && a.geo.kv_dtype == TS_F32)
            hipLaunchKernelGGL((append_token_kernel<float, float>), grid, block, 0, st, a);
        else if (a.geo.q_dtype == TS_BF16 && a.geo.kv_dtype == TS_BF16)
            hipLaunchKernelGGL((append_token_kernel<uint16_t, uint16_t>), grid, block, 0, st, a);
        else if (a.geo.q_dtype == TS_BF16 && a.geo.kv_dtype == TS_FP8_E4M3)
            hipLaunchKernelGGL((append_token_kernel<uint16_t, uint8_t>), grid, block, 0, st, a);
        else
            return (int)hipErrorInvalidValue;
        a.up_blocks = 0;                               // done; the page-wise kernel finds its list on the device
        a.apt = args.apt;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || a.n_apt == 0) return (int)e;
    if (a.geo.q_dtype != TS_BF16 || (a.geo.D != 128 && a.geo.D != 64)) return (int)hipErrorInvalidValue;
    if (a.geo.kv_dtype != TS_BF16 && a.geo.kv_dtype != TS_FP8_E4M3) return (int)hipErrorInvalidValue;
    dim3 tgrid((unsigned)a.n_apt * (unsigned)a.geo.Hkv + (unsigned)a.up_blocks);
    const bool bf = a.geo.kv_dtype == TS_BF16;
    if (a.geo.D == 128) {
        if (bf) hipLaunchKernelGGL((append_tile_kernel<uint16_t, 128>), tgrid, block, 0, st, a);
        else hipLaunchKernelGGL((append_tile_kernel<uint8_t, 128>), tgrid, block, 0, st, a);
    } else {
        if (bf) hipLaunchKernelGGL((append_tile_kernel<uint16_t, 64>), tgrid, block, 0, st, a);
        else hipLaunchKernelGGL((append_tile_kernel<uint8_t, 64>), tgrid, block, 0, st, a);
    }
    return (int)hipGetLastError();
}

}  // namespace ts
