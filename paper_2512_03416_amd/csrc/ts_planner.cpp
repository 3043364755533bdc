// Host work planner (step a0): turns the per-sequence lengths of one iteration's batch into the
// device work lists.  Pure host code, no GPU calls.
//
// The batch is the one a Convertible Decoder forms each iteration: its decode batch plus the
// prefill chunk(s) it absorbed, bounded by the profiled chunk size (paper Sec. 4.4).  Decode rows
// are cut into split-K items over the sequence's page list so that an HBM-bound scan is spread
// over all CUs; prefill chunks are cut into causal query tiles.  Items are ordered longest first
// so that the hardware dispatcher, which hands out workgroups in order, balances the tail.
#include <algorithm>
#include <climits>
#include <cmath>
#include <cstdio>
#include <cstring>

#include "ts_internal.h"

namespace ts {

bool desc_uses_mfma(const ts_attn_desc& d)
{
    return d.q_dtype == TS_BF16 && d.head_dim == 128 &&
           (d.kv_dtype == TS_BF16 || d.kv_dtype == TS_FP8_E4M3);
}

bool desc_uses_mfma_decode(const ts_attn_desc& d)
{
    return d.q_dtype == TS_BF16 && (d.head_dim == 128 || d.head_dim == 64) &&
           (d.kv_dtype == TS_BF16 || d.kv_dtype == TS_FP8_E4M3);
}

bool desc_uses_mfma_tiles(const ts_attn_desc& d)
{
    return desc_uses_mfma_decode(d);
}

int32_t prefill_tile_tokens(const ts_attn_desc& d)
{
    int G = d.num_q_heads / d.num_kv_heads;
    return 256 / G;     // 256 query rows (token, head-in-group) per tile
}

static int check_desc_impl(const ts_attn_desc* d, std::string* err)
{
    auto fail = [&](int code, const char* msg) { if (err) *err = msg; return code; };
    if (!d) return fail(TS_ERR_INVALID_ARG, "descriptor is NULL");
    if (d->page_size != kPage) return fail(TS_ERR_INVALID_ARG, "page_size must be 16");
    if (d->num_q_heads <= 0 || d->num_kv_heads <= 0 || d->num_q_heads % d->num_kv_heads)
        return fail(TS_ERR_INVALID_ARG, "num_q_heads must be a positive multiple of num_kv_heads");
    if (d->num_pages <= 0 || d->max_pages_per_seq <= 0)
        return fail(TS_ERR_INVALID_ARG, "num_pages and max_pages_per_seq must be positive");
    if (d->num_pages * (int64_t)d->num_kv_heads >= (int64_t)1 << 31)
        return fail(TS_ERR_INVALID_ARG, "num_pages * num_kv_heads must stay below 2^31");
    if (d->head_dim != 64 && d->head_dim != 128)
        return fail(TS_ERR_UNSUPPORTED, "head_dim must be 64 or 128");
    if (d->num_q_heads / d->num_kv_heads > 16)
        return fail(TS_ERR_UNSUPPORTED, "more than 16 query heads per KV head");
    bool ok = (d->q_dtype == TS_F32 && d->kv_dtype == TS_F32) ||
              (d->q_dtype == TS_BF16 && d->kv_dtype == TS_BF16) ||
              (d->q_dtype == TS_BF16 && d->kv_dtype == TS_FP8_E4M3);
    if (!ok) {
        bool known = d->q_dtype >= TS_F32 && d->q_dtype <= TS_FP8_E4M3 && d->kv_dtype >= TS_F32 &&
                     d->kv_dtype <= TS_FP8_E4M3;
        return fail(known ? TS_ERR_UNSUPPORTED : TS_ERR_INVALID_ARG,
                    "dtype pair must be (f32,f32), (bf16,bf16) or (bf16,fp8_e4m3)");
    }
    return TS_OK;
}

int validate_batch(const ts_attn_desc& d, const int32_t* q_lens, const int32_t* ctx_lens,
                   int num_seqs, std::string* err)
{
    char buf[160];
    if (num_seqs < 0) { *err = "num_seqs is negative"; return TS_ERR_INVALID_ARG; }
    if (num_seqs > 0 && (!q_lens || !ctx_lens)) {
        *err = "q_lens / ctx_lens is NULL";
        return TS_ERR_INVALID_ARG;
    }
    int64_t total = 0;
    for (int s = 0; s < num_seqs; ++s) {
        if (q_lens[s] < 0 || ctx_lens[s] < q_lens[s]) {
            snprintf(buf, sizeof buf, "sequence %d: q_len %d, ctx_len %d (need 0 <= q_len <= ctx_len)",
                     s, q_lens[s], ctx_lens[s]);
            *err = buf;
            return TS_ERR_INVALID_ARG;
        }
        if ((int64_t)ctx_lens[s] > (int64_t)kPage * d.max_pages_per_seq) {
            snprintf(buf, sizeof buf, "sequence %d: ctx_len %d exceeds 16 * max_pages_per_seq (%d)", s,
                     ctx_lens[s], d.max_pages_per_seq);
            *err = buf;
            return TS_ERR_INVALID_ARG;
        }
        total += q_lens[s];
    }
    if (total >= ((int64_t)1 << 31) / std::max(1, d.num_q_heads * d.head_dim / 64)) {
        *err = "batch has too many query tokens";
        return TS_ERR_INVALID_ARG;
    }
    return TS_OK;
}

// Pages per decode item.  A row that fits one item is finished by its workgroup without any
// partial result in HBM, so rows are cut only (a) when they exceed one workgroup slot's fair share
// of the batch (they would otherwise finish last), or (b) when the batch has fewer (row, KV head)
// pairs than the GPU has CUs: then the pages are dealt out so that there is about one workgroup per
// CU.  Pieces have at least 32 pages.  (Measured on 2-64 rows of 1500-6000 tokens: more and shorter
// items than that only add start-up, merge and combine work; 8 rows of 1500 tokens take 22 us per
// pass in pieces of 32 pages against 26 us in pieces of 8, next to a 256-token chunk 50 against 64 us;
// for 16-48 rows every choice between 32 and 128 pages lies within 10 % of the best.)
// In a mixed batch launched with resident workgroups (co-resident launch or one persistent kernel: a CU that
// holds a resident workgroup has room for one decode workgroup, a third of the stand-alone slots), (b) does not
// apply and the fair share in (a) is that of the slots actually there: measured on the burst configuration,
// 706 -> 692 us and no combine launch.
// Rates the two kinds of work reach on their own (decode scan: bytes per microsecond; prefill tiles: flop per
// microsecond, all CUs).
constexpr double kDecBytePerUs = 6.2e6;
constexpr double kPfFlopPerUs = 1.25e9;
// Co-resident launch: share of the CUs that get a resident prefill workgroup, from the ratio r of the two times:
// kPfShare0 + kPfShare1 * r, at most all of them.  Measured on one chunk of 128 ... 16 256 tokens over a prefix of 0
// or 4096 next to 128 decode rows of 1024-8192 tokens, and on the two burst configurations: too few workgroups
// make the tiles the critical path (the time rises steeply), a few too many cost 3-8 %; r = 0.3: best at 80-128 of
// 256, r = 0.8: 160-192, r = 1.0: 224, r >= 1.3: all.
constexpr double kPfShare0 = 0.25;
constexpr double kPfShare1 = 0.6;
// A mixed batch is launched class by class when either class is estimated below this many microseconds: running
// side by side hides about 40 % of the shorter class, and the fork and join of the co-resident launch cost
// 10-15 us.  Measured: 128 decode rows (395 us) next to a chunk of 128 / 896 tokens without prefix (estimates
// 0.1 / 5 us): 0.410 / 0.425 ms class by class against 0.423 / 0.432 ms; next to 384 tokens over a prefix of 4096
// (22 us): 0.450 against 0.429 ms; 16 decode rows of 2500 tokens (26 us) next to 256 tokens over 4096 (14 us):
// 85 against 89 us; 8 rows of 1500 tokens (8 us) next to 1024 tokens over 2048 (34 us): 85 against 100 us.
constexpr double kCoresidentMinUs = 20.0;

static int32_t auto_split_pages(int64_t decode_tiles, int64_t decode_pages, int64_t n_rows, int Hkv,
                                int32_t wg_slots, int32_t n_cu, bool filled_by_prefill, int32_t pf_wgs)
{
    // (next to a resident prefill workgroup a CU has room for one decode workgroup; the CUs without one hold
    // their usual share of the stand-alone slots)
    int64_t slots = std::max<int32_t>(1, filled_by_prefill ? n_cu : wg_slots);
    if (filled_by_prefill && pf_wgs > 0 && pf_wgs < n_cu)
        slots = pf_wgs + (int64_t)(n_cu - pf_wgs) * std::max(1, wg_slots / n_cu);
    int64_t L = std::max<int64_t>(32, (decode_tiles + slots - 1) / slots);
    if (!filled_by_prefill && n_rows * Hkv < n_cu && decode_pages > 0) {
        const int64_t want_items = (n_cu + Hkv - 1) / Hkv;             // per KV head
        L = std::min<int64_t>(L, std::max<int64_t>(32, (decode_pages + want_items - 1) / want_items));
    }
    return (int32_t)std::min<int64_t>(L, 1 << 20);
}

// Launch order of the prefill workgroups.  Workgroups are dispatched to the accelerator dies
// round-robin (workgroup i runs on die i % xcds) and every die has its own L2.  All tiles of one
// (chunk, KV head) stream read the same K/V pages, so a stream is pinned to one die and its tiles
// are launched next to each other: they walk the stream's pages almost in step, and the pages are
// fetched from HBM about once instead of once per tile.  Streams are spread over the dies by
// decreasing work (greedy), longest tiles of a stream first.
static int64_t pf_keys(const PfItem& t)
{
    return std::min(t.prefix + t.tok_begin + t.tok_count, t.kv_end) - t.kv_begin;
}

static void map_prefill_to_xcds(Plan& p, int Hkv, int xcds, int mixed_mode)
{
    p.pfmap.clear();
    p.queue.clear();
    p.q_off.clear();
    if (p.pf.empty()) return;
    struct Stream { int32_t seq; int32_t g; int64_t work; std::vector<int32_t> items; };
    std::vector<Stream> streams;
    {
        std::vector<int32_t> order(p.pf.size());
        for (size_t i = 0; i < order.size(); ++i) order[i] = (int32_t)i;
        std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return p.pf[a].seq < p.pf[b].seq; });
        size_t i = 0;
        while (i < order.size()) {
            size_t j = i;
            int64_t work = 0;
            std::vector<int32_t> items;
            while (j < order.size() && p.pf[order[j]].seq == p.pf[order[i]].seq) {
                const PfItem& it = p.pf[order[j]];
                work += std::min(it.prefix + it.tok_begin + it.tok_count, it.kv_end) - it.kv_begin;
                items.push_back(order[j]);       // p.pf is sorted longest first, the stable sort keeps that
                ++j;
            }
            for (int g = 0; g < Hkv; ++g) streams.push_back(Stream{p.pf[order[i]].seq, g, work, items});
            i = j;
        }
    }
    std::stable_sort(streams.begin(), streams.end(), [](const Stream& a, const Stream& b) { return a.work > b.work; });
    std::vector<std::vector<PfSlot>> per(xcds);
    std::vector<int64_t> load(xcds, 0);
    for (const Stream& st : streams) {
        int best = 0;
        for (int x = 1; x < xcds; ++x) if (load[x] < load[best]) best = x;
        load[best] += st.work;
        for (int32_t it : st.items) per[best].push_back(PfSlot{it, st.g});
    }
    size_t longest = 0;
    for (auto& v : per) longest = std::max(longest, v.size());
    p.pfmap.assign(longest * xcds, PfSlot{-1, 0});
    for (int x = 0; x < xcds; ++x)
        for (size_t k = 0; k < per[x].size(); ++k) p.pfmap[k * xcds + x] = per[x][k];
    if (mixed_mode == TS_MIXED_SEPARATE || p.dec.empty()) return;
    if (mixed_mode == TS_MIXED_CORESIDENT) {
        // The tiles alone, die by die in the launch order above, for the resident prefill workgroups; the
        // decode items run as a grid of their own next to them.
        p.q_off.assign(xcds + 1, 0);
        for (int x = 0; x < xcds; ++x) {
            for (const PfSlot& t : per[x]) p.queue.push_back(QItem{1, t.item, t.head_kv, 0});
            p.q_off[x + 1] = (int32_t)p.queue.size();
        }
        return;
    }

    // Mixed batch: one queue per die for the persistent kernel.  Decode items (HBM-bound) and
    // prefill tiles (MFMA-bound) are interleaved by their share of their own kind's total cost, so
    // that both kinds are in flight on every CU from the first to the last item and finish together.
    std::vector<std::vector<PfSlot>> dper(xcds);
    {
        int64_t j = 0;
        for (size_t i = 0; i < p.dec.size(); ++i)
            for (int g = 0; g < Hkv; ++g, ++j) dper[j % xcds].push_back(PfSlot{(int32_t)i, g});
    }
    p.q_off.assign(xcds + 1, 0);
    for (int x = 0; x < xcds; ++x) {
        double dtot = 0, ptot = 0;
        for (const PfSlot& d : dper[x]) dtot += p.dec[d.item].page_end - p.dec[d.item].page_begin;
        for (const PfSlot& t : per[x]) ptot += pf_keys(p.pf[t.item]);
        size_t di = 0, ti = 0;
        double dacc = 0, pacc = 0;
        while (di < dper[x].size() || ti < per[x].size()) {
            const double dkey = di < dper[x].size() ? dacc / std::max(1.0, dtot) : 2.0;
            const double pkey = ti < per[x].size() ? pacc / std::max(1.0, ptot) : 2.0;
            if (dkey <= pkey) {                            // decode first on ties (Sec. 4.5.2)
                const PfSlot& d = dper[x][di++];
                dacc += p.dec[d.item].page_end - p.dec[d.item].page_begin;
                p.queue.push_back(QItem{0, d.item, d.head_kv, 0});
            } else {
                const PfSlot& t = per[x][ti++];
                pacc += pf_keys(p.pf[t.item]);
                p.queue.push_back(QItem{1, t.item, t.head_kv, 0});
            }
        }
        p.q_off[x + 1] = (int32_t)p.queue.size();
    }
}

void build_plan(const ts_attn_desc& d, const int32_t* q_lens, const int32_t* ctx_lens, int num_seqs,
                const PlanOptions& opt, Plan* plan)
{
    Plan& p = *plan;
    p = Plan();
    const bool mfma = desc_uses_mfma(d) && !opt.generic_only;
    const bool mfma_dec = desc_uses_mfma_decode(d) && !opt.generic_only;
    // fp8 caches: can the pages of the chunks' sequences be widened to bf16 for this pass (see below)?
    int64_t chunk_pages = 0;
    for (int s = 0; s < num_seqs; ++s)
        if (q_lens[s] > 1) chunk_pages += (ctx_lens[s] + kPage - 1) / kPage;
    const bool widen = d.kv_dtype == TS_FP8_E4M3 && chunk_pages > 0 && opt.widen_pages > 0 && chunk_pages <= opt.widen_pages;
    // Chunk rows run as matrix-core tiles; with head dim 64 the tiles read bf16 pages only (a bf16 cache, or the
    // widened copies of an e4m3 cache), otherwise the rows go to the generic kernel.
    const bool mfma_tiles = desc_uses_mfma_tiles(d) && !opt.generic_only && !opt.prefill_generic &&
                            (d.head_dim == 128 || d.kv_dtype == TS_BF16 || widen);
    const int Hkv = d.num_kv_heads;
    p.seqs.resize((size_t)num_seqs + 1);
    int32_t off = 0;
    int64_t decode_tiles = 0, decode_pages = 0;
    for (int s = 0; s < num_seqs; ++s) {
        p.seqs[s] = SeqMeta{off, q_lens[s], ctx_lens[s], ctx_lens[s] - q_lens[s]};
        off += q_lens[s];
        p.info.ctx_pages += (ctx_lens[s] + kPage - 1) / kPage;
        if (q_lens[s] == 1) {
            p.info.decode_tokens += 1;
            decode_pages += (ctx_lens[s] + kPage - 1) / kPage;
            decode_tiles += (int64_t)((ctx_lens[s] + kPage - 1) / kPage) * Hkv;
        } else {
            p.info.prefill_tokens += q_lens[s];
        }
    }
    p.seqs[num_seqs] = SeqMeta{off, 0, 0, 0};
    p.info.total_tokens = off;

    // append work: chunks page by page where the page-wise kernel applies, the rest token by token
    const bool page_wise = d.q_dtype == TS_BF16 && d.kv_dtype != TS_F32 && (d.head_dim == 128 || d.head_dim == 64);
    for (int s = 0; s < num_seqs; ++s) {
        const SeqMeta& m = p.seqs[s];
        if (!page_wise || m.q_len < kAppendTileMin) {
            for (int32_t i = 0; i < m.q_len; ++i) p.apr.push_back(AppRow{m.q_off + i, s, m.prefix + i, 0});
            continue;
        }
        for (int32_t pg = m.prefix / kPage; pg <= (m.ctx_len - 1) / kPage; ++pg) {
            const int32_t lo = std::max(m.prefix, pg * kPage) - pg * kPage;
            const int32_t hi = std::min(m.ctx_len, (pg + 1) * kPage) - pg * kPage;
            p.apt.push_back(AppTile{s, pg, lo, hi, m.q_off + pg * kPage - m.prefix, 0, 0, 0});
        }
    }

    const int32_t TT = opt.tile_tokens > 0 ? opt.tile_tokens : prefill_tile_tokens(d);
    int64_t tile_heads = 0;                                // prefill workgroups of the batch
    if (mfma_tiles)
        for (int s = 0; s < num_seqs; ++s)
            if (p.seqs[s].q_len > 1) tile_heads += (int64_t)((p.seqs[s].q_len + TT - 1) / TT) * Hkv;
    // How a batch with both kinds of rows is launched.  Co-resident by default; class by class when either class
    // is too short for the overlap to pay for the fork and join (kCoresidentMinUs).
    int mixed_mode = opt.mixed_mode;
    double t_pf = 0, t_dec = 0;                            // microseconds each kind would take alone
    if (mixed_mode == TS_MIXED_CORESIDENT) {
        double flop = 0;
        for (int s = 0; s < num_seqs; ++s) {
            const SeqMeta& m = p.seqs[s];
            if (m.q_len > 1) flop += 4.0 * d.num_q_heads * d.head_dim * ((double)m.q_len * m.prefix + 0.5 * m.q_len * (m.q_len + 1.0));
        }
        t_pf = flop / kPfFlopPerUs;
        t_dec = (double)decode_tiles * 2.0 * kPage * d.head_dim * (d.kv_dtype == TS_FP8_E4M3 ? 1 : 2) / kDecBytePerUs;
        // (a stated number of resident workgroups asks for this launch form whatever the batch)
        if (opt.pf_resident_wgs <= 0 && std::min(t_pf, t_dec) < kCoresidentMinUs) mixed_mode = TS_MIXED_SEPARATE;
    }
    if (!mfma || p.info.decode_tokens == 0 || tile_heads == 0) mixed_mode = TS_MIXED_SEPARATE;
    if (!mfma_dec) { decode_tiles = 0; decode_pages = 0; }
    p.info.mixed_mode = mixed_mode;
    // Co-resident launch: how many CUs get a resident prefill workgroup.  Such a CU has room for one decode
    // workgroup instead of three, so a batch whose decode scan outlasts its tiles (one restricted chunk next to a
    // large decode batch, Sec. 4.4) keeps part of the CUs for decode rows alone: the tiles get a share of the CUs
    // that grows with the ratio of the two times (estimated from the batch's flops and bytes at the rates the
    // kernels reach alone), in multiples of the number of dies.
    int32_t pf_wgs = 0;
    if (mixed_mode == TS_MIXED_CORESIDENT) {
        const int32_t x = std::max(1, opt.xcds);
        const int32_t all = std::max(1, opt.n_cu);
        if (opt.pf_resident_wgs > 0) {
            pf_wgs = std::min(all, opt.pf_resident_wgs);
        } else {
            const double share = t_dec > 0 ? kPfShare0 + kPfShare1 * t_pf / t_dec : 1.0;
            pf_wgs = share >= 1.0 ? all : (int32_t)std::ceil(share * all);
        }
        pf_wgs = std::min(all, std::max(x, (pf_wgs + x - 1) / x * x));
    }
    const bool filled_by_prefill = mixed_mode != TS_MIXED_SEPARATE && (tile_heads >= opt.n_cu || pf_wgs > 0);
    const int32_t L = opt.split_pages > 0
                          ? opt.split_pages
                          : auto_split_pages(decode_tiles, decode_pages, p.info.decode_tokens, Hkv, opt.wg_slots,
                                             std::max(1, opt.n_cu), filled_by_prefill, pf_wgs);
    p.info.split_pages = L;
    p.info.tile_tokens = TT;

    int32_t part = 0, pf_part = 0;
    // parts per prefill tile that would give every CU a workgroup (1 = the tiles fill the GPU as they are)
    const int64_t pf_parts_wanted = tile_heads > 0 ? std::min<int64_t>(16, (pf_wgs > 0 ? pf_wgs : opt.n_cu) / tile_heads) : 1;
    for (int s = 0; s < num_seqs; ++s) {
        const SeqMeta& m = p.seqs[s];
        if (m.q_len == 0) continue;
        const bool as_decode = mfma_dec && m.q_len == 1;
        const bool as_tiles = mfma_tiles && m.q_len > 1;
        if (as_decode) {
            int32_t n_pages = (m.ctx_len + kPage - 1) / kPage;
            int32_t n_split = (n_pages + L - 1) / L;
            int32_t per = (n_pages + n_split - 1) / n_split;
            n_split = (n_pages + per - 1) / per;
            const int32_t cmb_idx = n_split > 1 ? (int32_t)p.cmb.size() : -1;
            if (n_split > 1) p.cmb.push_back(CmbItem{m.q_off, part, n_split, 0});
            for (int32_t k = 0; k < n_split; ++k) {
                int32_t b = k * per, e = std::min(n_pages, b + per);
                p.dec.push_back(DecItem{m.q_off, s, m.ctx_len, b, e, n_split > 1 ? part + k : -1, cmb_idx, n_split > 1 ? part : -1});
            }
            if (n_split > 1) part += n_split;
        } else if (as_tiles) {
            for (int32_t t0 = 0; t0 < m.q_len; t0 += TT) {
                const int32_t cnt = std::min(TT, m.q_len - t0);
                // Cut along the keys when the batch's tiles cannot occupy the GPU (a short chunk over a long
                // prefix -- the one-task-at-a-time shape of Sec. 4.4 -- walks thousands of keys in a handful of
                // workgroups otherwise).  Cuts lie at multiples of 64 keys at or below the tile's first query
                // position, so that every row sees the first key of every part; parts are of equal length.
                const int32_t below = (m.prefix + t0) / 64;                       // whole stages every row sees fully
                int32_t n_part = 1;
                if (pf_parts_wanted > 1 && opt.pf_split_min_keys > 0)
                    n_part = (int32_t)std::max<int64_t>(1, std::min<int64_t>(pf_parts_wanted, (int64_t)below * 64 / opt.pf_split_min_keys));
                if (n_part == 1) {
                    p.pf.push_back(PfItem{s, m.q_off, m.q_len, m.prefix, t0, cnt, m.ctx_len, -1, 0, INT32_MAX, 0, 0});
                    continue;
                }
                const int32_t total = (m.prefix + t0 + cnt + 63) / 64;            // stages of the whole tile
                const int32_t per = (total + n_part - 1) / n_part;
                int32_t begin = 0, made = 0;
                const int32_t first = pf_part;
                for (int32_t cut = per; cut <= below && cut < total; cut += per, ++made) {
                    p.pf.push_back(PfItem{s, m.q_off, m.q_len, m.prefix, t0, cnt, m.ctx_len, pf_part++, begin * 64, cut * 64, 0, 0});
                    begin = cut;
                }
                if (made == 0) {                                                   // no admissible cut after all
                    p.pf.push_back(PfItem{s, m.q_off, m.q_len, m.prefix, t0, cnt, m.ctx_len, -1, 0, INT32_MAX, 0, 0});
                    continue;
                }
                p.pf.push_back(PfItem{s, m.q_off, m.q_len, m.prefix, t0, cnt, m.ctx_len, pf_part++, begin * 64, INT32_MAX, 0, 0});
                ++made;
                p.pfcmb.push_back(PfCmb{(int32_t)p.pf.size() - made, first, made, 0});
            }
        } else {
            for (int32_t i = 0; i < m.q_len; ++i)
                p.rows.push_back(RowItem{m.q_off + i, s, m.prefix + i + 1, 0});
        }
    }
    // fp8 caches: the pages of the chunks' sequences are widened to bf16 once per pass (every tile of a chunk
    // reads the whole prefix: widening inside the tiles repeats the conversion once per tile and costs the tile
    // kernel 8 % of its time), provided they fit the scratch the option allows
    if (widen && !p.pf.empty()) {
        p.wide_base.assign((size_t)num_seqs, -1);
        for (int s = 0; s < num_seqs; ++s) {
            if (p.seqs[s].q_len <= 1) continue;
            p.wide_base[s] = (int32_t)p.wide.size();
            const int32_t n_pages = (p.seqs[s].ctx_len + kPage - 1) / kPage;
            for (int32_t j = 0; j < n_pages; ++j) p.wide.push_back(WideItem{s, j});
        }
    }
    p.info.widened_pages = (int64_t)p.wide.size();
    // longest first (stable, so equal lengths keep batch order and runs stay reproducible)
    std::stable_sort(p.dec.begin(), p.dec.end(), [](const DecItem& a, const DecItem& b) {
        return (a.page_end - a.page_begin) > (b.page_end - b.page_begin);
    });
    {
        // (the merge list refers to the tiles by position: sort a permutation and carry the references along)
        auto keys_of = [](const PfItem& t) {
            return std::min(t.prefix + t.tok_begin + t.tok_count, t.kv_end) - t.kv_begin;
        };
        std::vector<int32_t> order(p.pf.size()), where(p.pf.size());
        for (size_t i = 0; i < order.size(); ++i) order[i] = (int32_t)i;
        std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return keys_of(p.pf[a]) > keys_of(p.pf[b]); });
        std::vector<PfItem> sorted(p.pf.size());
        for (size_t i = 0; i < order.size(); ++i) { sorted[i] = p.pf[order[i]]; where[order[i]] = (int32_t)i; }
        p.pf.swap(sorted);
        for (PfCmb& cm : p.pfcmb) cm.item = where[cm.item];
    }
    map_prefill_to_xcds(p, Hkv, std::max(1, opt.xcds), mixed_mode);
    std::stable_sort(p.rows.begin(), p.rows.end(),
                     [](const RowItem& a, const RowItem& b) { return a.n_keys > b.n_keys; });
    p.info.n_decode_items = (int32_t)p.dec.size();
    p.info.n_combine_rows = (int32_t)p.cmb.size();
    p.info.n_prefill_tiles = (int32_t)p.pf.size();
    p.info.n_generic_rows = (int32_t)p.rows.size();
    p.info.partial_slots = part;
    p.info.prefill_parts = pf_part;
    p.info.prefill_workgroups = (int32_t)std::min<int64_t>(pf_wgs, (int64_t)p.queue.size());
}

}  // namespace ts

// ---- host-only C entry points -------------------------------------------------------------------

extern "C" int ts_check_desc(const ts_attn_desc* desc)
{
    return ts::check_desc_impl(desc, nullptr);
}

namespace ts { int check_desc_msg(const ts_attn_desc* d, std::string* err) { return check_desc_impl(d, err); } }

extern "C" int64_t ts_cache_bytes(const ts_attn_desc* d)
{
    if (ts::check_desc_impl(d, nullptr) != TS_OK) return 0;
    int64_t es = d->kv_dtype == TS_F32 ? 4 : (d->kv_dtype == TS_BF16 ? 2 : 1);
    return d->num_pages * d->num_kv_heads * ts::kPage * d->head_dim * es;
}

extern "C" int ts_plan_describe(const ts_attn_desc* desc, const int32_t* q_lens, const int32_t* ctx_lens,
                                int num_seqs, int32_t split_pages, ts_plan_info* out)
{
    std::string err;
    int rc = ts::check_desc_impl(desc, &err);
    if (rc != TS_OK) return rc;
    if (!out || split_pages < 0) return TS_ERR_INVALID_ARG;
    rc = ts::validate_batch(*desc, q_lens, ctx_lens, num_seqs, &err);
    if (rc != TS_OK) return rc;
    ts::Plan plan;
    ts::PlanOptions opt;
    opt.split_pages = split_pages;
    ts::build_plan(*desc, q_lens, ctx_lens, num_seqs, opt, &plan);
    *out = plan.info;
    return TS_OK;
}

extern "C" int64_t ts_plan_export(const ts_attn_desc* desc, const int32_t* q_lens, const int32_t* ctx_lens,
                                  int num_seqs, int32_t split_pages, int32_t wg_slots, int32_t mixed_mode, int which,
                                  int32_t* out, int64_t capacity)
{
    std::string err;
    int rc = ts::check_desc_impl(desc, &err);
    if (rc != TS_OK) return rc;
    if (split_pages < 0 || wg_slots < 0 || capacity < 0 || (capacity > 0 && !out)) return TS_ERR_INVALID_ARG;
    if (mixed_mode < -1 || mixed_mode > TS_MIXED_CORESIDENT) return TS_ERR_INVALID_ARG;
    rc = ts::validate_batch(*desc, q_lens, ctx_lens, num_seqs, &err);
    if (rc != TS_OK) return rc;
    ts::Plan plan;
    ts::PlanOptions opt;
    opt.split_pages = split_pages;
    if (wg_slots > 0) opt.wg_slots = wg_slots;
    if (mixed_mode >= 0) opt.mixed_mode = mixed_mode;
    ts::build_plan(*desc, q_lens, ctx_lens, num_seqs, opt, &plan);
    const void* src = nullptr;
    int64_t n = 0, words = 0;
    switch (which) {
    case TS_LIST_DECODE:  src = plan.dec.data();   n = (int64_t)plan.dec.size();   words = sizeof(ts::DecItem) / 4; break;
    case TS_LIST_COMBINE: src = plan.cmb.data();   n = (int64_t)plan.cmb.size();   words = sizeof(ts::CmbItem) / 4; break;
    case TS_LIST_PREFILL: src = plan.pf.data();    n = (int64_t)plan.pf.size();    words = sizeof(ts::PfItem) / 4; break;
    case TS_LIST_PFMAP:   src = plan.pfmap.data(); n = (int64_t)plan.pfmap.size(); words = sizeof(ts::PfSlot) / 4; break;
    case TS_LIST_ROWS:    src = plan.rows.data();  n = (int64_t)plan.rows.size();  words = sizeof(ts::RowItem) / 4; break;
    case TS_LIST_QUEUE:   src = plan.queue.data(); n = (int64_t)plan.queue.size(); words = sizeof(ts::QItem) / 4; break;
    case TS_LIST_QOFF:    src = plan.q_off.data(); n = (int64_t)plan.q_off.size(); words = 1; break;
    case TS_LIST_APPEND:  src = plan.apt.data();   n = (int64_t)plan.apt.size();   words = sizeof(ts::AppTile) / 4; break;
    case TS_LIST_APPEND_ROWS: src = plan.apr.data(); n = (int64_t)plan.apr.size(); words = sizeof(ts::AppRow) / 4; break;
    case TS_LIST_PFCOMBINE: src = plan.pfcmb.data(); n = (int64_t)plan.pfcmb.size(); words = sizeof(ts::PfCmb) / 4; break;
    case TS_LIST_WIDEN:   src = plan.wide.data();  n = (int64_t)plan.wide.size();  words = sizeof(ts::WideItem) / 4; break;
    default: return TS_ERR_INVALID_ARG;
    }
    const int64_t fit = words ? std::min<int64_t>(n, capacity / words) : 0;
    if (fit > 0) memcpy(out, src, (size_t)(fit * words) * 4);
    return n;
}
