// Internal declarations shared by the host API, the planner and the kernel launchers.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "tokenscale.h"

namespace ts {

constexpr int kPage = TS_PAGE_SIZE;

// ---- work items (host planner -> device work list) ------------------------------------------

struct SeqMeta {          // one per sequence, plus a sentinel with q_off = T
    int32_t q_off;        // row index of the sequence's first new token
    int32_t q_len;
    int32_t ctx_len;
    int32_t prefix;       // ctx_len - q_len
};

struct DecItem {          // one split of one decode row; launched once per KV head
    int32_t row;          // query row in q / out
    int32_t seq;
    int32_t n_keys;       // keys the row sees
    int32_t page_begin;   // [page_begin, page_end) of the sequence's page list
    int32_t page_end;
    int32_t part;         // partial slot, or -1 when the row has a single split
    int32_t cmb;          // split rows: index of the row in the combine list (its arrival counters), else -1
    int32_t part_first;   // split rows: partial slot of the row's first split (the splits' slots are consecutive)
};

struct CmbItem {          // a decode row whose splits must be merged
    int32_t row;
    int32_t part_begin;
    int32_t n_split;
    int32_t pad;
};

struct PfItem {           // a causal tile of a prefill chunk; launched once per KV head
    int32_t seq;
    int32_t row0;         // row of the chunk's first token
    int32_t q_len;
    int32_t prefix;
    int32_t tok_begin;    // tile covers chunk tokens [tok_begin, tok_begin + tok_count)
    int32_t tok_count;
    int32_t ctx_len;
    int32_t part;         // -1: the item covers all keys of the tile and writes the output rows; else it covers the
                          // keys [kv_begin, kv_end) only and writes partial result number `part`
    int32_t kv_begin;     // multiple of 64, at most the tile's first query position: every row sees key kv_begin
    int32_t kv_end;       // multiple of 64, or INT32_MAX for "up to the tile's last key"
    int32_t pad0, pad1;
};

struct PfCmb {            // a tile whose key range was cut: its partial results part_begin .. part_begin + n_part - 1
    int32_t item;         // index of the tile's first part in the prefill list (for the rows it covers)
    int32_t part_begin;
    int32_t n_part;
    int32_t pad;
};
constexpr int kPfPartRows = 256;   // rows of one prefill partial result (a whole tile)

struct PfSlot {           // workgroup -> (prefill tile, KV head); item < 0 = nothing to do
    int32_t item;
    int32_t head_kv;
};

struct QItem {            // entry of a per-die work queue of the persistent mixed kernel
    int32_t kind;         // 0 = decode item, 1 = prefill tile
    int32_t item;
    int32_t head_kv;
    int32_t pad;
};

struct AppTile {          // one cache page of a chunk's new tokens; launched once per KV head
    int32_t seq;
    int32_t page_idx;     // index into the sequence's page list
    int32_t slot_lo;      // new tokens occupy slots [slot_lo, slot_hi) of the page
    int32_t slot_hi;
    int32_t row_slot0;    // row (in k_new / v_new) that slot 0 of the page would hold
    int32_t pad0, pad1, pad2;
};
constexpr int kAppendTileMin = 8;   // sequences with at least this many new tokens are appended page-wise
struct AppRow {           // one new token that is appended on its own
    int32_t row;
    int32_t seq;
    int32_t pos;          // its position in the sequence (prefix + index among the new tokens)
    int32_t pad;
};

struct WideItem {         // one page of a prefill chunk's sequence that is widened from e4m3 to bf16 before the tiles run
    int32_t seq;
    int32_t page_idx;     // index into the sequence's page list; the widened copy is page number = index in this list
};

struct RowItem {          // one query row for the generic kernel
    int32_t row;
    int32_t seq;
    int32_t n_keys;
    int32_t pad;
};

struct Plan {
    std::vector<SeqMeta> seqs;       // S + 1
    std::vector<DecItem> dec;
    std::vector<CmbItem> cmb;
    std::vector<PfItem> pf;
    std::vector<PfCmb> pfcmb;        // tiles cut along the keys: what to merge
    std::vector<PfSlot> pfmap;       // launch order of the prefill workgroups (XCD-aware)
    std::vector<AppTile> apt;        // page-wise append work of the chunks
    std::vector<AppRow> apr;         // token-wise append work: short sequences, and everything the page-wise kernel does not cover
    std::vector<QItem> queue;        // mixed batches: per-die queues, concatenated
    std::vector<int32_t> q_off;      // xcds + 1 offsets into queue
    std::vector<RowItem> rows;
    std::vector<WideItem> wide;      // fp8 caches: pages to widen, in the order of their widened copies
    std::vector<int32_t> wide_base;  // per sequence: number of its first widened page, -1 = not widened
    ts_plan_info info{};
};

struct PlanOptions {
    int32_t split_pages = 0;    // 0 = auto
    int32_t wg_slots = 768;     // decode workgroups resident at once (256 CUs x 3)
    int32_t n_cu = 256;         // compute units of the GPU
    int32_t xcds = 8;           // accelerator dies; workgroup i is dispatched to die i % xcds
    int32_t mixed_mode = TS_MIXED_CORESIDENT;   // how a batch with decode rows and prefill chunks is launched
    bool generic_only = false;  // every row through the generic kernel
    bool prefill_generic = false;
    int32_t tile_tokens = 0;    // query tokens per prefill tile
    int32_t pf_split_min_keys = 512;    // shortest key range of a cut prefill tile (multiple of 64; 0 = never cut)
    int32_t pf_resident_wgs = 0; // co-resident launch: resident prefill workgroups (0 = from the batch's two costs)
    int64_t widen_pages = 16384; // fp8 caches: most pages of prefill sequences that are widened to bf16 per pass (0 = never)
};

// Which kernels serve a descriptor: the full matrix-core set (head dim 128: tile kernels, resident launches of
// mixed batches and their scratch), the matrix-core decode items (head dim 64 or 128), the matrix-core tiles
// (head dim 64 or 128).  Everything else goes through the generic row kernel.
bool desc_uses_mfma(const ts_attn_desc& d);
bool desc_uses_mfma_decode(const ts_attn_desc& d);
bool desc_uses_mfma_tiles(const ts_attn_desc& d);      // (head dim 64: bf16 pages only, one launch per class)
int32_t prefill_tile_tokens(const ts_attn_desc& d);

// Validates lengths; returns TS_OK or an error and fills err.
int validate_batch(const ts_attn_desc& d, const int32_t* q_lens, const int32_t* ctx_lens,
                   int num_seqs, std::string* err);

// Builds the work lists (validate_batch must have passed).
void build_plan(const ts_attn_desc& d, const int32_t* q_lens, const int32_t* ctx_lens, int num_seqs,
                const PlanOptions& opt, Plan* plan);

// ---- device-side parameter blocks -------------------------------------------------------------

struct Geometry {
    int32_t Hq, Hkv, G, D;
    int32_t max_pages;         // block_table row stride
    int32_t q_dtype, kv_dtype;
};

struct AppendArgs {
    Geometry geo;
    const void* k_new; const void* v_new;
    void* k_cache; void* v_cache;
    const float* k_scale; const float* v_scale;
    const int32_t* block_table;
    const SeqMeta* seqs; int32_t num_seqs; int32_t total_tokens;
    const AppTile* apt; int32_t n_apt;
    const AppRow* apr; int32_t n_apr;
    // Work-list upload riding along in the first append launch (up_blocks > 0): extra workgroups copy
    // up_n16 16-byte pieces from the pinned staging buffer to device memory, and that launch reads its
    // own list from the staging buffer (apr_host / apt_host: the device copy does not exist before the
    // launch has finished).
    const void* up_src; void* up_dst; int64_t up_n16; int32_t up_blocks;
    const AppRow* apr_host; const AppTile* apt_host;
};

struct AttnArgs {
    Geometry geo;
    const void* q;
    const void* k_cache; const void* v_cache;
    const float* k_scale; const float* v_scale;
    const int32_t* block_table;
    float sm_scale;
    void* out;
    // work lists
    const DecItem* dec; int32_t n_dec;
    const CmbItem* cmb; int32_t n_cmb;
    const PfItem* pf;   int32_t n_pf;
    const PfSlot* pfmap; int32_t n_pfmap;
    const QItem* queue; const int32_t* q_off; int32_t n_queue; int32_t n_xcd;
    int32_t* q_ctr;            // n_xcd queue heads + 1 finished-workgroup count, zero between launches
    const RowItem* rows; int32_t n_rows;
    // fp8 caches: bf16 copies of the prefill sequences' pages (tiles [page][kv head], bf16 operand order), made
    // once per pass; wide_base[seq] = number of the sequence's first widened page.  NULL = the tiles read the
    // fp8 cache and widen it themselves.
    const void* wide_k; const void* wide_v; const int32_t* wide_base;
    const WideItem* wide; int32_t n_wide;
    int32_t dec_nbuf;          // KV tiles in flight per decode wave (2..4)
    int32_t mixed_wgs;         // workgroups of the persistent kernel that are resident on the GPU at once
    int32_t n_cu;              // compute units of the GPU
    int32_t pf_wgs;            // co-resident launch: resident workgroups for the prefill tiles (at most one per CU)
    // prefill tiles cut along the keys: partial results o [part][kv head][256 rows][D] fp32 (unnormalised),
    // ml [part][kv head][256 rows][2] = (reference maximum in log2 units, weight sum)
    const PfCmb* pfcmb; int32_t n_pfcmb;
    float* pf_part_o; float* pf_part_ml;
    // Arrival counters of the split decode rows, one per (combine row, KV head), zero between launches: the
    // workgroup that finds n_split - 1 in it is the last of the row and merges the partials itself.  NULL = the
    // items only write their partials and combine_kernel merges them.
    int32_t* cmb_ctr;
    // split-K partials: o [slot][Hq][D] fp32 (unnormalised), ml [slot][Hq][2] = (max, sum) in log2 units
    float* part_o; float* part_ml;
    // Small decode-only batches, fused form (k_new != NULL): the wave that reads a row's last page takes the row's
    // new token from k_new / v_new [T, Hkv, D] instead of the cache and writes its cache entry itself, so the pass
    // has no append launch.
    const void* k_new; const void* v_new;
};

// Work lists short enough to travel as kernel arguments (fused form of small decode-only batches).
constexpr int kSmallDec = 64, kSmallCmb = 32;
struct SmallLists {
    int32_t n_dec, n_cmb, pad0, pad1;
    DecItem dec[kSmallDec];
    CmbItem cmb[kSmallCmb];
};

// Launchers (defined in the .hip files).  All return a hipError_t cast to int.
int launch_append(const AppendArgs& a, void* stream);
int launch_rows(const AttnArgs& a, void* stream);
int launch_decode(const AttnArgs& a, void* stream);
int launch_combine(const AttnArgs& a, void* stream);
int launch_decode_fused(const AttnArgs& a, const SmallLists& lists, void* stream);   // decode items + merge of split rows
// Resident workgroups of the decode / persistent kernel on the current device (0 if unknown).  The
// caller keeps the answers per context: two contexts may sit on different GPUs.
int decode_resident_workgroups(int kv_dtype, int nbuf, int head_dim);
int mixed_resident_workgroups(int kv_dtype);
int launch_widen(const AttnArgs& a, void* wide_k, void* wide_v, void* stream);
int launch_prefill(const AttnArgs& a, void* stream);
int launch_mixed(const AttnArgs& a, void* stream);
int launch_prefill_resident(const AttnArgs& a, void* stream);
int launch_prefill_combine(const AttnArgs& a, void* stream);

}  // namespace ts
