// C-ABI boundary: argument checks, scratch, work-list upload, kernel launches, velocity counters.
//
// Every GPU step of the pass runs in the kernels of this library; this file only validates,
// plans (ts_planner.cpp), copies the small work lists to the device and launches.
#include <hip/hip_runtime.h>

#include <chrono>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "ts_internal.h"

namespace ts {
int check_desc_msg(const ts_attn_desc* d, std::string* err);
}

using namespace ts;

namespace {

thread_local std::string g_create_error;

// Scratch of the allocation-free entry point: device memory that exists from the moment the library is
// loaded on a GPU until the process ends, one copy per GPU.  Layout (bytes):
//   [0, 4 KiB)       queue heads of the persistent kernel, result words of the page-id check (first 1 KiB),
//                    arrival counters of split decode rows (768 words)
//   [4 KiB, 1 MiB)   device copy of the work lists
//   [1 MiB, 8 MiB)   split-K partial results
// In host code the array's name is only a handle: the address a kernel can use is asked for once per
// device (static_scratch_of) and kept.
constexpr size_t kStaticBytes = 8u << 20;
constexpr size_t kStaticCtrBytes = 4096;
constexpr int kStaticCmbCtrs = 768;                        // words [256, 1024) of the counter area
constexpr size_t kStaticWorkOff = kStaticCtrBytes, kStaticWorkBytes = (1u << 20) - kStaticCtrBytes;
constexpr size_t kStaticPartOff = 1u << 20, kStaticPartBytes = kStaticBytes - kStaticPartOff;
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
unsigned char* g_scratch_ptr[kMaxDevices] = {};

// Device address of this GPU's copy of `scratch`.  `device` must be the calling thread's current device.
hipError_t static_scratch_of(int device, unsigned char** out)
{
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[device]) {
        void* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = (unsigned char*)ptr;
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

constexpr int kRing = 4;

struct HostSlot {
    void* ptr = nullptr;             // pinned host memory ...
    void* dev_ptr = nullptr;         // ... and the address the GPU reads it at
    size_t cap = 0;
    hipEvent_t ev = nullptr;
    bool pending = false;
};

}  // namespace

struct ts_ctx {
    ts_attn_desc desc{};
    int device = 0;
    std::string err;
    PlanOptions opt;
    Plan plan;
    // device scratch
    char* d_work = nullptr;  size_t work_cap = 0;
    float* d_part_o = nullptr; float* d_part_ml = nullptr; int64_t part_cap = 0;
    int32_t* d_cmb_ctr = nullptr;    // arrival counters of split decode rows (part_cap x Hkv, zero between launches)
    int32_t* d_q_ctr = nullptr;      // queue heads of the persistent kernel (zero between launches)
    float* d_pf_part_o = nullptr; float* d_pf_part_ml = nullptr; int64_t pf_part_cap = 0;   // partial results of cut prefill tiles
    char* d_wide_k = nullptr; char* d_wide_v = nullptr; int64_t wide_cap = 0;   // fp8 caches: widened pages (capacity in pages)
    unsigned char* d_static = nullptr;  // this GPU's copy of the static scratch array
    bool static_call = false;        // the call in progress must not allocate (uses d_static)
    // pinned staging ring for the work lists
    HostSlot ring[kRing];
    int ring_pos = 0;
    // token velocity (Sec. 3.2)
    std::mutex mu;
    uint64_t prefill_tokens = 0, decode_tokens = 0, passes = 0;
    bool window_open = false;
    std::chrono::steady_clock::time_point t0;
    // One event per call, recorded behind its last kernel (the staging slot's): it frees the slot, it is
    // what a call on another stream waits for (the work-list buffer, the partials and the queue heads
    // are reused by every call), and it ends the last pass for the velocity counters.  (Every event
    // record keeps the GPU idle for about 5 us, so a call records exactly one.)
    HostSlot* cur_slot = nullptr;      // slot of the call in progress
    hipEvent_t last_event = nullptr;   // event of the most recent call
    hipStream_t last_stream = nullptr;
    bool have_work = false;
    // Co-resident launch of a mixed batch: the decode grid runs on this internal stream (default priority),
    // forked from the caller's stream behind the append and joined to it again with these two events.
    hipStream_t side = nullptr;
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    // Does the side stream run next to the caller's stream?  A process has few hardware queues and the runtime
    // decides which streams share one; two streams on one queue run in turn and the co-resident launch gains
    // nothing.  The first co-resident call therefore sends a probe ahead: a one-thread kernel on the caller's
    // stream that waits (bounded: kProbeTicks of the 100 MHz clock) for a flag which a kernel on the side stream
    // sets, and writes into pinned host memory whether it saw it.  A later call reads the answer (no wait) and,
    // if the two ran in turn, takes a new side stream and probes again, kProbeTries times at most.
    int side_state = 0;                // 0 = not probed, 1 = probe in flight, 2 = settled
    int side_tries = 0;
    int side_overlap = 0;              // answer of the last finished probe: 0 = none yet, 1 = side by side, 2 = in turn
    int32_t* h_probe = nullptr;        // pinned: one answer word per try
    int32_t* h_probe_dev = nullptr;    // the same words as the GPU addresses them
    std::vector<hipStream_t> parked;   // side streams that ran in turn with the caller's stream
    // Split decode rows are merged by a launch of their own (default) or by whichever item of a row finishes
    // last.  The second form saves a launch but needs a device-scope release in every item and an acquire in the
    // last one; on this GPU the release writes the L2 back, and 8 rows of 1500 tokens took 30 us per pass
    // instead of 20, a 256-token chunk next to 16 decode rows 154 us instead of 106.
    bool merge_in_kernel = false;
    // Small decode-only batches are bound by their launches: when the work lists are short enough to travel as
    // kernel arguments, the decode items append the rows' new tokens themselves (no append launch, no upload).
    // 8 rows of 1500 tokens: 19.4 -> 15.1 us per pass (e4m3 cache: 19.7 -> 14.4), 16 rows: 29.1 -> 25.8
    // (25.9 -> 20.4).  (In a large batch the stores in the middle of the scan cost more than the launch they
    // save -- 256 rows: 425 -> 444-450 us -- and the lists would not fit anyway.)
    bool fused_append = true;
    bool validate_pages = false;       // debug: check the page ids of a batch before anything is launched
    // launch shapes of this context's GPU, asked once per context (and again when the prefetch depth changes)
    int dec_nbuf = 2;                  // KV tiles in flight per decode wave
    int dec_slots = 0;                 // resident decode workgroups for dec_nbuf, 0 = not asked yet
    int mixed_wgs = 0;                 // resident workgroups of the persistent kernel, 0 = not asked yet
    // optional per-kernel timing
    int timing = 0;                    // 0 = off, N = time the launches of every N-th pass
    uint64_t timing_pass = 0;
    bool timing_now = false;
    struct Timed { int which; hipEvent_t a, b; };
    std::vector<Timed> timed;          // recorded, not yet read
    std::vector<hipEvent_t> ev_pool;   // spare events
    int64_t n_alloc = 0;               // device / pinned allocations made so far
    uint64_t k_launches[TS_K_COUNT] = {};
    double k_ms[TS_K_COUNT] = {};
};

namespace {

int fail(ts_ctx* c, int code, const std::string& msg)
{
    if (c) c->err = msg;
    return code;
}

int hip_fail(ts_ctx* c, hipError_t e, const char* what)
{
    return fail(c, TS_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

#define TS_HIP(c, call)                                              \
    do {                                                             \
        hipError_t e_ = (call);                                      \
        if (e_ != hipSuccess) return hip_fail((c), e_, #call);       \
    } while (0)

struct DeviceGuard {
    int prev = -1; bool switched = false;
    explicit DeviceGuard(int dev)
    {
        if (hipGetDevice(&prev) == hipSuccess && prev != dev) switched = hipSetDevice(dev) == hipSuccess;
    }
    ~DeviceGuard() { if (switched) (void)hipSetDevice(prev); }
};

size_t align16(size_t n) { return (n + 15) & ~(size_t)15; }

int ensure_work(ts_ctx* c, size_t bytes)
{
    if (c->static_call) {
        if (bytes <= kStaticWorkBytes) return TS_OK;
        return fail(c, TS_ERR_UNSUPPORTED, "batch too large for the allocation-free entry point: its work lists need " +
                                               std::to_string(bytes) + " bytes, the static scratch holds " +
                                               std::to_string(kStaticWorkBytes));
    }
    if (bytes <= c->work_cap) return TS_OK;
    size_t cap = std::max<size_t>(bytes * 2, 1 << 16);
    TS_HIP(c, hipDeviceSynchronize());
    if (c->d_work) TS_HIP(c, hipFree(c->d_work));
    c->d_work = nullptr; c->work_cap = 0;
    hipError_t e = hipMalloc((void**)&c->d_work, cap);
    if (e != hipSuccess) return fail(c, TS_ERR_NOMEM, "work-list scratch allocation failed");
    c->work_cap = cap;
    c->n_alloc += 1;
    return TS_OK;
}

int64_t static_partial_slots(const ts_ctx* c)
{
    const size_t per = (size_t)c->desc.num_q_heads * ((size_t)c->desc.head_dim + 2) * sizeof(float);
    return (int64_t)((kStaticPartBytes - 256) / per);
}

// Where the call in progress keeps its device-side scratch.
char* work_base(const ts_ctx* c) { return c->static_call ? (char*)c->d_static + kStaticWorkOff : c->d_work; }
int32_t* q_ctr_of(const ts_ctx* c) { return c->static_call ? (int32_t*)c->d_static : c->d_q_ctr; }
// Arrival counters for n split rows, or NULL when the static scratch has too few (the merge then runs as a launch).
int32_t* cmb_ctr_of(const ts_ctx* c, size_t n_rows)
{
    if (!c->static_call) return c->d_cmb_ctr;
    return n_rows * (size_t)c->desc.num_kv_heads <= (size_t)kStaticCmbCtrs ? (int32_t*)c->d_static + 256 : nullptr;
}
float* part_o_of(const ts_ctx* c) { return c->static_call ? (float*)(c->d_static + kStaticPartOff) : c->d_part_o; }
float* part_ml_of(const ts_ctx* c)
{
    if (!c->static_call) return c->d_part_ml;
    const size_t o_bytes = (size_t)static_partial_slots(c) * c->desc.num_q_heads * c->desc.head_dim * sizeof(float);
    return (float*)(c->d_static + kStaticPartOff + ((o_bytes + 255) & ~(size_t)255));
}

int ensure_partials(ts_ctx* c, int64_t slots)
{
    if (c->static_call) {
        if (slots <= static_partial_slots(c)) return TS_OK;
        return fail(c, TS_ERR_UNSUPPORTED, "batch too large for the allocation-free entry point: " + std::to_string(slots) +
                                               " split-K partial results, the static scratch holds " +
                                               std::to_string(static_partial_slots(c)));
    }
    if (slots <= c->part_cap) return TS_OK;
    int64_t cap = std::max<int64_t>(slots * 2, 1024);
    TS_HIP(c, hipDeviceSynchronize());
    if (c->d_part_o) TS_HIP(c, hipFree(c->d_part_o));
    if (c->d_part_ml) TS_HIP(c, hipFree(c->d_part_ml));
    if (c->d_cmb_ctr) TS_HIP(c, hipFree(c->d_cmb_ctr));
    c->d_part_o = c->d_part_ml = nullptr; c->d_cmb_ctr = nullptr; c->part_cap = 0;
    const size_t Hq = (size_t)c->desc.num_q_heads, D = (size_t)c->desc.head_dim;
    const size_t ctr_bytes = (size_t)cap * c->desc.num_kv_heads * sizeof(int32_t);
    if (hipMalloc((void**)&c->d_part_o, (size_t)cap * Hq * D * sizeof(float)) != hipSuccess ||
        hipMalloc((void**)&c->d_part_ml, (size_t)cap * Hq * 2 * sizeof(float)) != hipSuccess ||
        hipMalloc((void**)&c->d_cmb_ctr, ctr_bytes) != hipSuccess || hipMemset(c->d_cmb_ctr, 0, ctr_bytes) != hipSuccess)
        return fail(c, TS_ERR_NOMEM, "split-K partial scratch allocation failed");
    c->part_cap = cap;
    c->n_alloc += 3;
    return TS_OK;
}

// Partial results of prefill tiles cut along the keys: `parts` results of 256 rows for every KV head.
int ensure_pf_parts(ts_ctx* c, int64_t parts)
{
    if (parts <= c->pf_part_cap) return TS_OK;
    const size_t rows = (size_t)c->desc.num_kv_heads * kPfPartRows;
    const int64_t cap = std::max<int64_t>(parts * 2, 64);
    TS_HIP(c, hipDeviceSynchronize());
    if (c->d_pf_part_o) TS_HIP(c, hipFree(c->d_pf_part_o));
    if (c->d_pf_part_ml) TS_HIP(c, hipFree(c->d_pf_part_ml));
    c->d_pf_part_o = c->d_pf_part_ml = nullptr; c->pf_part_cap = 0;
    if (hipMalloc((void**)&c->d_pf_part_o, (size_t)cap * rows * c->desc.head_dim * sizeof(float)) != hipSuccess ||
        hipMalloc((void**)&c->d_pf_part_ml, (size_t)cap * rows * 2 * sizeof(float)) != hipSuccess)
        return fail(c, TS_ERR_NOMEM, "scratch for the partial results of cut prefill tiles could not be allocated");
    c->pf_part_cap = cap;
    c->n_alloc += 2;
    return TS_OK;
}

// fp8 caches: scratch for the bf16 copies of `pages` pages (K and V).
int ensure_wide(ts_ctx* c, int64_t pages)
{
    if (pages <= c->wide_cap) return TS_OK;
    const size_t page_bytes = (size_t)c->desc.num_kv_heads * kPage * c->desc.head_dim * 2;
    TS_HIP(c, hipDeviceSynchronize());
    if (c->d_wide_k) TS_HIP(c, hipFree(c->d_wide_k));
    if (c->d_wide_v) TS_HIP(c, hipFree(c->d_wide_v));
    c->d_wide_k = c->d_wide_v = nullptr; c->wide_cap = 0;
    const int64_t cap = std::min<int64_t>(std::max<int64_t>(pages + pages / 2, 256), std::max<int64_t>(pages, c->opt.widen_pages));
    if (hipMalloc((void**)&c->d_wide_k, (size_t)cap * page_bytes) != hipSuccess ||
        hipMalloc((void**)&c->d_wide_v, (size_t)cap * page_bytes) != hipSuccess)
        return fail(c, TS_ERR_NOMEM, "scratch for the widened fp8 pages could not be allocated");
    c->wide_cap = cap;
    c->n_alloc += 2;
    return TS_OK;
}

// Next pinned staging slot with at least `bytes`, free of any copy still in flight.
int acquire_slot(ts_ctx* c, size_t bytes, HostSlot** out, bool exact = false)
{
    HostSlot& s = c->ring[c->ring_pos];
    c->ring_pos = (c->ring_pos + 1) % kRing;
    if (s.pending) { TS_HIP(c, hipEventSynchronize(s.ev)); s.pending = false; }
    // (no system-scope fence: the event only orders GPU work against GPU work and against the host
    // overwriting a buffer the GPU has read)
    if (c->static_call && (!s.ev || bytes > s.cap))         // (cannot happen: ts_create sized the ring for kStaticWorkBytes)
        return fail(c, TS_ERR_UNSUPPORTED, "staging ring too small for the allocation-free entry point");
    if (!s.ev) TS_HIP(c, hipEventCreateWithFlags(&s.ev, hipEventDisableTiming | hipEventDisableSystemFence));
    if (bytes > s.cap) {
        if (s.ptr) TS_HIP(c, hipHostFree(s.ptr));
        s.ptr = s.dev_ptr = nullptr; s.cap = 0;
        size_t cap = exact ? bytes : std::max<size_t>(bytes * 2, 1 << 16);
        // (coherent: the GPU reads it uncached over PCIe, so a slot that is filled again is never seen stale)
        if (hipHostMalloc(&s.ptr, cap, hipHostMallocCoherent) != hipSuccess)
            return fail(c, TS_ERR_NOMEM, "pinned staging allocation failed");
        if (hipHostGetDevicePointer(&s.dev_ptr, s.ptr, 0) != hipSuccess) {
            (void)hipHostFree(s.ptr);
            s.ptr = s.dev_ptr = nullptr;
            return fail(c, TS_ERR_HIP, "pinned staging memory is not visible to the GPU");
        }
        s.cap = cap;
        c->n_alloc += 1;
    }
    *out = &s;
    return TS_OK;
}

// Brings the work lists from the pinned staging buffer into device memory.  A kernel instead of a copy
// command: between two kernels of a stream the GPU loses no time, around a copy command it idled
// 10 + 5 us per call (a twentieth of a decode step).
// zero / n_zero: words put back to zero by the same launch (the queue heads inside the static scratch, which
// any earlier call on this GPU may have left in any state).
__global__ __launch_bounds__(256) void upload_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t n16,
                                                     int32_t* zero, int n_zero)
{
    if (blockIdx.x == 0)
        for (int i = threadIdx.x; i < n_zero; i += blockDim.x) zero[i] = 0;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// Debug check of the device-side page table: every page a sequence of the batch uses must lie in
// [0, num_pages).  result[0] counts the offenders, result[1..2] = (sequence, page index) of one of them.
__global__ __launch_bounds__(256) void check_pages_kernel(const SeqMeta* __restrict__ seqs, const int32_t* __restrict__ bt,
                                                          int max_pages, int64_t num_pages, int32_t* result)
{
    const int s = blockIdx.x;
    const int used = (seqs[s].ctx_len + kPage - 1) / kPage;
    for (int p = threadIdx.x; p < used; p += blockDim.x) {
        const int32_t id = bt[(int64_t)s * max_pages + p];
        if (id < 0 || id >= num_pages) {
            if (atomicAdd(&result[0], 1) == 0) { result[1] = s; result[2] = p; }
        }
    }
}

struct WorkLayout {
    size_t seqs, dec, cmb, pf, pfcmb, pfmap, rows, queue, q_off, apt, apr, wide, wide_base, total;
};

WorkLayout layout_of(const Plan& p)
{
    WorkLayout w{};
    size_t o = 0;
    w.seqs = o; o = align16(o + p.seqs.size() * sizeof(SeqMeta));
    w.dec = o;  o = align16(o + p.dec.size() * sizeof(DecItem));
    w.cmb = o;  o = align16(o + p.cmb.size() * sizeof(CmbItem));
    w.pf = o;   o = align16(o + p.pf.size() * sizeof(PfItem));
    w.pfcmb = o; o = align16(o + p.pfcmb.size() * sizeof(PfCmb));
    w.pfmap = o; o = align16(o + p.pfmap.size() * sizeof(PfSlot));
    w.rows = o; o = align16(o + p.rows.size() * sizeof(RowItem));
    w.queue = o; o = align16(o + p.queue.size() * sizeof(QItem));
    w.q_off = o; o = align16(o + p.q_off.size() * sizeof(int32_t));
    w.apt = o; o = align16(o + p.apt.size() * sizeof(AppTile));
    w.apr = o; o = align16(o + p.apr.size() * sizeof(AppRow));
    w.wide = o; o = align16(o + p.wide.size() * sizeof(WideItem));
    w.wide_base = o; o = align16(o + p.wide_base.size() * sizeof(int32_t));
    w.total = o;
    return w;
}

struct UploadJob { const uint4* src = nullptr; uint4* dst = nullptr; int64_t n16 = 0; int blocks = 0; const char* host_lists = nullptr; };

// Fills a staging slot with the work lists.  With `defer` the copy to the device is left to the caller
// (it rides along in the append launch, see AppendArgs), else it is launched here.
int upload_plan(ts_ctx* c, hipStream_t st, const WorkLayout& w, UploadJob* defer = nullptr)
{
    int rc = ensure_work(c, w.total);
    if (rc != TS_OK) return rc;
    if (c->have_work && st != c->last_stream) TS_HIP(c, hipStreamWaitEvent(st, c->last_event, 0));
    HostSlot* slot = nullptr;
    rc = acquire_slot(c, w.total, &slot);
    if (rc != TS_OK) return rc;
    const Plan& p = c->plan;
    char* h = (char*)slot->ptr;
    memcpy(h + w.seqs, p.seqs.data(), p.seqs.size() * sizeof(SeqMeta));
    if (!p.dec.empty()) memcpy(h + w.dec, p.dec.data(), p.dec.size() * sizeof(DecItem));
    if (!p.cmb.empty()) memcpy(h + w.cmb, p.cmb.data(), p.cmb.size() * sizeof(CmbItem));
    if (!p.pf.empty()) memcpy(h + w.pf, p.pf.data(), p.pf.size() * sizeof(PfItem));
    if (!p.pfcmb.empty()) memcpy(h + w.pfcmb, p.pfcmb.data(), p.pfcmb.size() * sizeof(PfCmb));
    if (!p.pfmap.empty()) memcpy(h + w.pfmap, p.pfmap.data(), p.pfmap.size() * sizeof(PfSlot));
    if (!p.rows.empty()) memcpy(h + w.rows, p.rows.data(), p.rows.size() * sizeof(RowItem));
    if (!p.queue.empty()) memcpy(h + w.queue, p.queue.data(), p.queue.size() * sizeof(QItem));
    if (!p.q_off.empty()) memcpy(h + w.q_off, p.q_off.data(), p.q_off.size() * sizeof(int32_t));
    if (!p.apt.empty()) memcpy(h + w.apt, p.apt.data(), p.apt.size() * sizeof(AppTile));
    if (!p.apr.empty()) memcpy(h + w.apr, p.apr.data(), p.apr.size() * sizeof(AppRow));
    if (!p.wide.empty()) memcpy(h + w.wide, p.wide.data(), p.wide.size() * sizeof(WideItem));
    if (!p.wide_base.empty()) memcpy(h + w.wide_base, p.wide_base.data(), p.wide_base.size() * sizeof(int32_t));
    const int64_t n16 = (int64_t)(w.total / 16);           // (every list starts at a multiple of 16)
    const int blocks = (int)std::min<int64_t>(256, (n16 + 255) / 256);
    c->cur_slot = slot;                                    // its event is recorded by mark_work_done
    if (defer) {
        *defer = UploadJob{(const uint4*)slot->dev_ptr, (uint4*)work_base(c), n16, blocks, (const char*)slot->dev_ptr};
        return TS_OK;
    }
    if (n16 > 0) {
        hipLaunchKernelGGL(upload_kernel, dim3(blocks), dim3(256), 0, st, (const uint4*)slot->dev_ptr, (uint4*)work_base(c),
                           n16, c->static_call ? q_ctr_of(c) : nullptr, c->static_call ? (int)(kStaticCtrBytes / 4) : 0);
        TS_HIP(c, hipGetLastError());
    }
    return TS_OK;
}

// Debug option "validate_block_table": runs the check on the call's stream and waits for it, so that a
// bad page id is reported before any kernel of the pass has touched the caches.
int check_pages(ts_ctx* c, hipStream_t st, const WorkLayout& w, const int32_t* block_table, int num_seqs)
{
    if (!c->validate_pages || num_seqs <= 0) return TS_OK;
    int32_t* res = q_ctr_of(c) + 120;                      // (the queue heads use the first 65 words)
    TS_HIP(c, hipMemsetAsync(res, 0, 4 * sizeof(int32_t), st));
    hipLaunchKernelGGL(check_pages_kernel, dim3((unsigned)num_seqs), dim3(256), 0, st, (const SeqMeta*)(work_base(c) + w.seqs),
                       block_table, c->desc.max_pages_per_seq, (int64_t)c->desc.num_pages, res);
    TS_HIP(c, hipGetLastError());
    int32_t host[4] = {0, 0, 0, 0};
    TS_HIP(c, hipMemcpyAsync(host, res, sizeof host, hipMemcpyDeviceToHost, st));
    TS_HIP(c, hipStreamSynchronize(st));
    if (host[0] != 0)
        return fail(c, TS_ERR_INVALID_ARG, "block_table: " + std::to_string(host[0]) + " page id(s) outside [0, num_pages), e.g. sequence " +
                                               std::to_string(host[1]) + ", page " + std::to_string(host[2]));
    return TS_OK;
}

hipEvent_t take_event(ts_ctx* c)
{
    if (!c->ev_pool.empty()) { hipEvent_t e = c->ev_pool.back(); c->ev_pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    // (timing only: no cache write-back around the kernel being timed)
    if (hipEventCreateWithFlags(&e, hipEventDisableSystemFence) != hipSuccess) return nullptr;
    return e;
}

// Runs one launcher, bracketed by events on the launch stream when timing is on.
template <typename F>
int timed_launch(ts_ctx* c, int which, bool has_work, hipStream_t st, F&& launch)
{
    if (!c->timing_now || !has_work || c->timed.size() >= 65536) return launch();
    hipEvent_t ea = take_event(c), eb = take_event(c);
    if (!ea || !eb) return launch();
    (void)hipEventRecord(ea, st);
    int e = launch();
    (void)hipEventRecord(eb, st);
    c->timed.push_back({which, ea, eb});
    return e;
}

int drain_timed(ts_ctx* c)
{
    for (auto& t : c->timed) {
        TS_HIP(c, hipEventSynchronize(t.b));
        float ms = 0.f;
        TS_HIP(c, hipEventElapsedTime(&ms, t.a, t.b));
        c->k_ms[t.which] += ms;
        c->k_launches[t.which] += 1;
        c->ev_pool.push_back(t.a);
        c->ev_pool.push_back(t.b);
    }
    c->timed.clear();
    return TS_OK;
}

constexpr int kProbeTries = 4;
constexpr long long kProbeTicks = 6000;                   // 60 us of the 100 MHz clock
constexpr int kProbeFlagWord = 96;                         // words 96 .. 96 + kProbeTries - 1 of the counter block

// Waits until *flag is set or the time is up (every path ends: the loop is bounded in iterations as well).
__global__ void probe_wait_kernel(const int32_t* flag, int32_t* answer)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    const long long t0 = wall_clock64();
    int seen = 0;
    for (int i = 0; i < (1 << 16); ++i) {
        seen = __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (seen || wall_clock64() - t0 > kProbeTicks) break;
        __builtin_amdgcn_s_sleep(16);
    }
    __hip_atomic_store(answer, seen ? 1 : 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

__global__ void probe_set_kernel(int32_t* flag)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) __hip_atomic_store(flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Reads a finished probe's answer and sends the next probe if one is due.  Never waits and never fails the call:
// whatever goes wrong here leaves the side stream as it is.
void probe_side_stream(ts_ctx* c, hipStream_t st)
{
    if (c->side_state == 2 || c->static_call || !c->h_probe) return;
    if (c->side_state == 1) {
        const int32_t ans = __atomic_load_n(&c->h_probe[c->side_tries], __ATOMIC_RELAXED);
        if (ans == 0) return;                              // not there yet
        c->side_overlap = ans;
        c->side_tries += 1;
        if (ans == 1 || c->side_tries >= kProbeTries) { c->side_state = 2; return; }
        // in turn: another stream.  The old one is kept until the context goes (a stream made right after one was
        // released was seen to take the released one's queue again).
        hipStream_t fresh = nullptr;
        if (hipStreamCreateWithFlags(&fresh, hipStreamNonBlocking) != hipSuccess) { (void)hipGetLastError(); c->side_state = 2; return; }
        c->parked.push_back(c->side);
        c->side = fresh;
        c->side_state = 0;
    }
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone) { (void)hipGetLastError(); return; }
    int32_t* flag = c->d_q_ctr + kProbeFlagWord + c->side_tries;
    hipLaunchKernelGGL(probe_wait_kernel, dim3(1), dim3(64), 0, st, (const int32_t*)flag, c->h_probe_dev + c->side_tries);
    hipLaunchKernelGGL(probe_set_kernel, dim3(1), dim3(64), 0, c->side, flag);
    if (hipGetLastError() != hipSuccess) { c->side_state = 2; return; }
    c->side_state = 1;
}

// Marks the end of a call's device work on its stream: the call's one event.  Runs on every path that
// follows a successful upload_plan, error paths included (the upload kernel may still be reading the slot).
int mark_work_done(ts_ctx* c, hipStream_t st)
{
    HostSlot* slot = c->cur_slot;
    c->cur_slot = nullptr;
    if (!slot) return TS_OK;
    slot->pending = true;
    c->last_stream = st;
    c->have_work = true;
    c->last_event = slot->ev;
    TS_HIP(c, hipEventRecord(slot->ev, st));
    return TS_OK;
}

struct WorkDoneGuard {                                     // records the event when a call leaves early
    ts_ctx* c; hipStream_t st;
    ~WorkDoneGuard() { if (c->cur_slot) (void)mark_work_done(c, st); }
};

Geometry geometry_of(const ts_attn_desc& d)
{
    Geometry g{};
    g.Hq = d.num_q_heads; g.Hkv = d.num_kv_heads; g.G = d.num_q_heads / d.num_kv_heads;
    g.D = d.head_dim; g.max_pages = d.max_pages_per_seq; g.q_dtype = d.q_dtype; g.kv_dtype = d.kv_dtype;
    return g;
}

int check_common(ts_ctx* c, const void* k_cache, const void* v_cache, const float* k_scale,
                 const float* v_scale, const int32_t* block_table, const int32_t* q_lens,
                 const int32_t* ctx_lens, int num_seqs)
{
    if (!k_cache || !v_cache) return fail(c, TS_ERR_INVALID_ARG, "k_cache / v_cache is NULL");
    if (c->desc.kv_dtype == TS_FP8_E4M3 && (!k_scale || !v_scale))
        return fail(c, TS_ERR_INVALID_ARG, "fp8 cache needs k_scale and v_scale");
    if (num_seqs > 0 && !block_table) return fail(c, TS_ERR_INVALID_ARG, "block_table is NULL");
    std::string err;
    int rc = validate_batch(c->desc, q_lens, ctx_lens, num_seqs, &err);
    if (rc != TS_OK) return fail(c, rc, err);
    return TS_OK;
}

}  // namespace

// ---------------------------------------------------------------------------------------------------

extern "C" const char* ts_last_error(const ts_ctx* ctx)
{
    return ctx ? ctx->err.c_str() : g_create_error.c_str();
}

extern "C" int ts_create(const ts_attn_desc* desc, int device, ts_ctx** out)
{
    g_create_error.clear();
    if (!out) { g_create_error = "out is NULL"; return TS_ERR_INVALID_ARG; }
    *out = nullptr;
    int rc = check_desc_msg(desc, &g_create_error);
    if (rc != TS_OK) return rc;
    int n_dev = 0;
    hipError_t e = hipGetDeviceCount(&n_dev);
    if (e != hipSuccess || n_dev <= 0) {
        g_create_error = std::string("no HIP device available: ") + hipGetErrorString(e);
        return TS_ERR_HIP;
    }
    if (device < 0 || device >= n_dev) { g_create_error = "device index out of range"; return TS_ERR_INVALID_ARG; }
    struct Restore {                                       // the caller's current device comes back on return
        int prev = -1;
        ~Restore() { if (prev >= 0) (void)hipSetDevice(prev); }
    } restore;
    if (hipGetDevice(&restore.prev) != hipSuccess || restore.prev == device) restore.prev = -1;
    e = hipSetDevice(device);
    if (e != hipSuccess) { g_create_error = std::string("hipSetDevice: ") + hipGetErrorString(e); return TS_ERR_HIP; }
    ts_ctx* c = new (std::nothrow) ts_ctx();
    if (!c) { g_create_error = "out of host memory"; return TS_ERR_NOMEM; }
    c->desc = *desc;
    c->device = device;
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) == hipSuccess && cus > 0) c->opt.n_cu = cus;
    rc = ensure_work(c, 1 << 16);
    if (rc == TS_OK) rc = ensure_partials(c, 1024);
    if (rc == TS_OK) {
        if (hipMalloc((void**)&c->d_q_ctr, 128 * sizeof(int32_t)) != hipSuccess ||
            hipMemset(c->d_q_ctr, 0, 128 * sizeof(int32_t)) != hipSuccess) {
            c->err = "queue counter allocation failed";
            rc = TS_ERR_NOMEM;
        }
    }
    if (rc == TS_OK && desc_uses_mfma_decode(c->desc))     // launch shapes of this GPU, asked here so that no later call has to
        c->dec_slots = decode_resident_workgroups(c->desc.kv_dtype, c->dec_nbuf, c->desc.head_dim);
    if (rc == TS_OK && desc_uses_mfma(c->desc)) {
        c->mixed_wgs = mixed_resident_workgroups(c->desc.kv_dtype);
        if (c->mixed_wgs <= 0) rc = fail(c, TS_ERR_HIP, "occupancy query of the persistent kernel failed");
    }
    if (rc == TS_OK && desc_uses_mfma(c->desc)) {
        if (hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking) != hipSuccess ||
            hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming | hipEventDisableSystemFence) != hipSuccess ||
            hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming | hipEventDisableSystemFence) != hipSuccess)
            rc = fail(c, TS_ERR_HIP, "side stream / event creation failed");
        if (rc == TS_OK) {
            void* dev = nullptr;
            if (hipHostMalloc((void**)&c->h_probe, 64, hipHostMallocCoherent) == hipSuccess &&
                hipHostGetDevicePointer(&dev, c->h_probe, 0) == hipSuccess) {
                memset(c->h_probe, 0, 64);
                c->h_probe_dev = (int32_t*)dev;
            } else {
                (void)hipGetLastError();
                if (c->h_probe) (void)hipHostFree(c->h_probe);
                c->h_probe = nullptr;                      // (no probe then: the side stream stays as created)
            }
        }
    }
    if (rc == TS_OK) {
        // the allocation-free entry point: this GPU's static scratch, and a staging ring that holds the
        // largest work lists that scratch takes
        const hipError_t se = static_scratch_of(device, &c->d_static);
        if (se != hipSuccess) rc = hip_fail(c, se, "hipGetSymbolAddress(scratch)");
        for (int i = 0; rc == TS_OK && i < kRing; ++i) {
            HostSlot* s = nullptr;
            rc = acquire_slot(c, kStaticWorkBytes, &s, true);
        }
    }
    if (rc != TS_OK) { g_create_error = c->err; ts_destroy(c); return rc; }
    *out = c;
    return TS_OK;
}

extern "C" int ts_destroy(ts_ctx* c)
{
    if (!c) return TS_ERR_INVALID_ARG;
    DeviceGuard guard(c->device);
    (void)hipDeviceSynchronize();
    if (c->d_work) (void)hipFree(c->d_work);
    if (c->d_part_o) (void)hipFree(c->d_part_o);
    if (c->d_part_ml) (void)hipFree(c->d_part_ml);
    if (c->d_cmb_ctr) (void)hipFree(c->d_cmb_ctr);
    if (c->d_q_ctr) (void)hipFree(c->d_q_ctr);
    if (c->d_pf_part_o) (void)hipFree(c->d_pf_part_o);
    if (c->d_pf_part_ml) (void)hipFree(c->d_pf_part_ml);
    if (c->d_wide_k) (void)hipFree(c->d_wide_k);
    if (c->d_wide_v) (void)hipFree(c->d_wide_v);
    if (c->side) (void)hipStreamDestroy(c->side);
    for (hipStream_t s : c->parked) (void)hipStreamDestroy(s);
    if (c->h_probe) (void)hipHostFree(c->h_probe);
    if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
    if (c->ev_join) (void)hipEventDestroy(c->ev_join);
    for (HostSlot& s : c->ring) {
        if (s.ptr) (void)hipHostFree(s.ptr);
        if (s.ev) (void)hipEventDestroy(s.ev);
    }
    for (auto& t : c->timed) { (void)hipEventDestroy(t.a); (void)hipEventDestroy(t.b); }
    for (hipEvent_t e : c->ev_pool) (void)hipEventDestroy(e);
    delete c;
    return TS_OK;
}

extern "C" int ts_reserve(ts_ctx* c, int64_t max_tokens, int64_t max_seqs, int64_t max_ctx_pages)
{
    if (!c) return TS_ERR_INVALID_ARG;
    if (max_tokens < 0 || max_seqs < 0 || max_ctx_pages < 0)
        return fail(c, TS_ERR_INVALID_ARG, "negative size");
    DeviceGuard guard(c->device);
    // Upper bounds of every work list for such a batch under the options in force now: a sequence of n
    // pages gives at most n / L + 1 decode items (L = the decode_split_pages option, or the planner's own
    // minimum of 32 pages), a chunk of q tokens at most q / tile + 1 tiles and q / 16 + 2 append pages; the
    // die-aware launch order pads every die's list to the longest one.
    const size_t T = (size_t)max_tokens, S = (size_t)max_seqs, P = (size_t)max_ctx_pages;
    const size_t Hkv = (size_t)c->desc.num_kv_heads, xcds = (size_t)std::max(1, c->opt.xcds);
    const size_t L = c->opt.split_pages > 0 ? (size_t)c->opt.split_pages : 32;
    const size_t TT = (size_t)std::max<int32_t>(1, c->opt.tile_tokens > 0 ? c->opt.tile_tokens : prefill_tile_tokens(c->desc));
    const size_t items = P / L + S;
    const size_t tiles = T / TT + S + (size_t)c->opt.n_cu;      // (cutting tiles along the keys adds at most one item per CU)
    const size_t bytes = (S + 1) * sizeof(SeqMeta) + items * (sizeof(DecItem) + sizeof(CmbItem)) + tiles * (sizeof(PfItem) + sizeof(PfCmb)) +
                         tiles * Hkv * xcds * sizeof(PfSlot) + T * sizeof(RowItem) +
                         (items + tiles) * Hkv * sizeof(QItem) + (xcds + 1) * sizeof(int32_t) +
                         (T / kPage + 2 * S) * sizeof(AppTile) + T * sizeof(AppRow) +
                         (size_t)std::min<int64_t>((int64_t)P, c->opt.widen_pages) * sizeof(WideItem) + S * sizeof(int32_t) + 16 * 16;
    int rc = ensure_work(c, bytes);
    if (rc != TS_OK) return rc;
    if (desc_uses_mfma_tiles(c->desc) && c->opt.pf_split_min_keys > 0) {
        rc = ensure_pf_parts(c, (int64_t)c->opt.n_cu);
        if (rc != TS_OK) return rc;
    }
    if (c->desc.kv_dtype == TS_FP8_E4M3 && desc_uses_mfma_tiles(c->desc) && c->opt.widen_pages > 0) {
        rc = ensure_wide(c, std::min<int64_t>((int64_t)P, c->opt.widen_pages));
        if (rc != TS_OK) return rc;
    }
    for (int i = 0; i < kRing; ++i) {
        HostSlot* s = nullptr;
        rc = acquire_slot(c, bytes, &s);
        if (rc != TS_OK) return rc;
    }
    return ensure_partials(c, (int64_t)items);
}

extern "C" int ts_set_option(ts_ctx* c, const char* name, int64_t value)
{
    if (!c || !name) return TS_ERR_INVALID_ARG;
    if (!strcmp(name, "decode_split_pages")) {
        if (value < 0 || value > (1 << 20)) return fail(c, TS_ERR_INVALID_ARG, "decode_split_pages out of range");
        c->opt.split_pages = (int32_t)value;
        return TS_OK;
    }
    if (!strcmp(name, "prefill_path")) {
        if (value != 0 && value != 1) return fail(c, TS_ERR_INVALID_ARG, "prefill_path must be 0 or 1");
        c->opt.prefill_generic = value == 1;
        return TS_OK;
    }
    if (!strcmp(name, "decode_prefetch_tiles")) {
        if (value < 2 || value > 4) return fail(c, TS_ERR_INVALID_ARG, "decode_prefetch_tiles must be 2..4");
        if (c->dec_nbuf != (int)value) {
            DeviceGuard guard(c->device);
            c->dec_nbuf = (int)value;
            if (desc_uses_mfma_decode(c->desc))
                c->dec_slots = decode_resident_workgroups(c->desc.kv_dtype, c->dec_nbuf, c->desc.head_dim);
        }
        return TS_OK;
    }
    if (!strcmp(name, "mixed_mode")) {
        if (value < TS_MIXED_SEPARATE || value > TS_MIXED_CORESIDENT) return fail(c, TS_ERR_INVALID_ARG, "mixed_mode must be 0, 1 or 2");
        c->opt.mixed_mode = (int32_t)value;
        return TS_OK;
    }
    if (!strcmp(name, "decode_merge_in_kernel")) {
        c->merge_in_kernel = value != 0;
        return TS_OK;
    }
    if (!strcmp(name, "decode_fused_append")) {
        if (value != 0 && value != 1) return fail(c, TS_ERR_INVALID_ARG, "decode_fused_append must be 0 or 1");
        c->fused_append = value == 1;
        return TS_OK;
    }
    if (!strcmp(name, "prefill_split_min_keys")) {
        if (value < 0 || value > (1 << 24) || value % 64) return fail(c, TS_ERR_INVALID_ARG, "prefill_split_min_keys must be a multiple of 64");
        c->opt.pf_split_min_keys = (int32_t)value;
        return TS_OK;
    }
    if (!strcmp(name, "prefill_resident_workgroups")) {
        if (value < 0 || value > 65536) return fail(c, TS_ERR_INVALID_ARG, "prefill_resident_workgroups out of range");
        c->opt.pf_resident_wgs = (int32_t)value;
        return TS_OK;
    }
    if (!strcmp(name, "prefill_widen_pages")) {
        if (value < 0 || value > ((int64_t)1 << 24)) return fail(c, TS_ERR_INVALID_ARG, "prefill_widen_pages out of range");
        c->opt.widen_pages = value;
        return TS_OK;
    }
    if (!strcmp(name, "xcd_count")) {
        if (value < 1 || value > 64) return fail(c, TS_ERR_INVALID_ARG, "xcd_count must be 1..64");
        c->opt.xcds = (int32_t)value;
        return TS_OK;
    }
    if (!strcmp(name, "validate_block_table")) {
        c->validate_pages = value != 0;
        return TS_OK;
    }
    if (!strcmp(name, "kernel_timing")) {
        if (value < 0 || value > 1024) return fail(c, TS_ERR_INVALID_ARG, "kernel_timing must be 0..1024");
        c->timing = (int)value;
        c->timing_pass = 0;
        return TS_OK;
    }
    return fail(c, TS_ERR_INVALID_ARG, std::string("unknown option: ") + name);
}

extern "C" int ts_get_option(const ts_ctx* c, const char* name, int64_t* value)
{
    if (!c || !name || !value) return TS_ERR_INVALID_ARG;
    if (!strcmp(name, "decode_split_pages")) *value = c->opt.split_pages;
    else if (!strcmp(name, "prefill_path")) *value = c->opt.prefill_generic ? 1 : 0;
    else if (!strcmp(name, "decode_prefetch_tiles")) *value = c->dec_nbuf;
    else if (!strcmp(name, "mixed_mode")) *value = c->opt.mixed_mode;
    else if (!strcmp(name, "xcd_count")) *value = c->opt.xcds;
    else if (!strcmp(name, "prefill_widen_pages")) *value = c->opt.widen_pages;
    else if (!strcmp(name, "prefill_resident_workgroups")) *value = c->opt.pf_resident_wgs;
    else if (!strcmp(name, "side_stream_overlap")) *value = c->side_overlap;
    else if (!strcmp(name, "side_stream_probes")) *value = c->side_tries;
    else if (!strcmp(name, "prefill_split_min_keys")) *value = c->opt.pf_split_min_keys;
    else if (!strcmp(name, "decode_merge_in_kernel")) *value = c->merge_in_kernel ? 1 : 0;
    else if (!strcmp(name, "decode_fused_append")) *value = c->fused_append ? 1 : 0;
    else if (!strcmp(name, "validate_block_table")) *value = c->validate_pages ? 1 : 0;
    else if (!strcmp(name, "kernel_timing")) *value = c->timing;
    else if (!strcmp(name, "scratch_allocations")) *value = c->n_alloc;
    else return TS_ERR_INVALID_ARG;                         // (const context: the error text is left alone)
    return TS_OK;
}

extern "C" int ts_kv_append(ts_ctx* c, void* stream, const void* k_new, const void* v_new, void* k_cache,
                            void* v_cache, const float* k_scale, const float* v_scale,
                            const int32_t* block_table, const int32_t* q_lens, const int32_t* ctx_lens,
                            int num_seqs)
{
    if (!c) return TS_ERR_INVALID_ARG;
    c->err.clear();
    int rc = check_common(c, k_cache, v_cache, k_scale, v_scale, block_table, q_lens, ctx_lens, num_seqs);
    if (rc != TS_OK) return rc;
    DeviceGuard guard(c->device);
    c->timing_now = c->timing > 0 && (c->timing_pass++ % (uint64_t)c->timing) == 0;
    PlanOptions opt = c->opt;
    build_plan(c->desc, q_lens, ctx_lens, num_seqs, opt, &c->plan);
    if (c->plan.info.total_tokens == 0) return TS_OK;
    if (!k_new || !v_new) return fail(c, TS_ERR_INVALID_ARG, "k_new / v_new is NULL");
    // only the sequence table is needed on the device
    c->plan.dec.clear(); c->plan.cmb.clear(); c->plan.pf.clear(); c->plan.rows.clear(); c->plan.pfmap.clear();
    c->plan.queue.clear(); c->plan.q_off.clear();
    const WorkLayout w = layout_of(c->plan);
    hipStream_t st = (hipStream_t)stream;
    // no page check: the upload rides along in the first append launch
    const bool ride = !c->validate_pages;
    UploadJob job;
    rc = upload_plan(c, st, w, ride ? &job : nullptr);
    if (rc != TS_OK) return rc;
    WorkDoneGuard guard_done{c, st};
    rc = check_pages(c, st, w, block_table, num_seqs);
    if (rc != TS_OK) return rc;
    AppendArgs a{};
    a.geo = geometry_of(c->desc);
    a.k_new = k_new; a.v_new = v_new; a.k_cache = k_cache; a.v_cache = v_cache;
    a.k_scale = k_scale; a.v_scale = v_scale; a.block_table = block_table;
    a.seqs = (const SeqMeta*)(c->d_work + w.seqs);
    a.num_seqs = num_seqs; a.total_tokens = (int32_t)c->plan.info.total_tokens;
    a.apt = (const AppTile*)(c->d_work + w.apt); a.n_apt = (int32_t)c->plan.apt.size();
    a.apr = (const AppRow*)(c->d_work + w.apr); a.n_apr = (int32_t)c->plan.apr.size();
    if (ride) {
        a.apr_host = (const AppRow*)(job.host_lists + w.apr);
        a.apt_host = (const AppTile*)(job.host_lists + w.apt);
        a.up_src = job.src; a.up_dst = job.dst; a.up_n16 = job.n16; a.up_blocks = job.blocks;
    }
    hipError_t e = (hipError_t)timed_launch(c, TS_K_APPEND, true, st, [&] { return launch_append(a, stream); });
    if (e != hipSuccess) return hip_fail(c, e, "append launch");
    return mark_work_done(c, st);
}

namespace {

// The pass behind both entry points.  With c->static_call set, all device scratch lies inside the static
// array and nothing on this path allocates (no growth, no new events, no per-kernel timing).
int mixed_pass(ts_ctx* c, void* stream, const void* q, const void* k_new, const void* v_new, void* k_cache, void* v_cache,
               const float* k_scale, const float* v_scale, const int32_t* block_table, const int32_t* q_lens,
               const int32_t* ctx_lens, int num_seqs, float sm_scale, void* out)
{
    c->err.clear();
    int rc = check_common(c, k_cache, v_cache, k_scale, v_scale, block_table, q_lens, ctx_lens, num_seqs);
    if (rc != TS_OK) return rc;
    if ((k_new == nullptr) != (v_new == nullptr))
        return fail(c, TS_ERR_INVALID_ARG, "k_new and v_new must both be given or both be NULL");
    if (!(sm_scale == sm_scale)) return fail(c, TS_ERR_INVALID_ARG, "sm_scale is NaN");
    if (c->static_call && c->validate_pages)
        return fail(c, TS_ERR_UNSUPPORTED, "the validate_block_table option waits for the GPU and copies to the host: "
                                           "not available in the allocation-free entry point");
    DeviceGuard guard(c->device);
    c->timing_now = !c->static_call && c->timing > 0 && (c->timing_pass++ % (uint64_t)c->timing) == 0;
    if (c->dec_slots > 0) c->opt.wg_slots = c->dec_slots;
    {
        PlanOptions opt = c->opt;
        if (c->static_call) {                              // (no scratch for widened pages or for partial results of cut tiles)
            opt.widen_pages = 0;
            opt.pf_split_min_keys = 0;
        }
        build_plan(c->desc, q_lens, ctx_lens, num_seqs, opt, &c->plan);
    }
    const Plan& p = c->plan;
    if (p.info.total_tokens == 0) return TS_OK;
    if (!q || !out) return fail(c, TS_ERR_INVALID_ARG, "q / out is NULL");
    rc = ensure_partials(c, p.info.partial_slots);
    if (rc != TS_OK) return rc;
    if (!p.wide.empty()) {
        rc = ensure_wide(c, (int64_t)p.wide.size());
        if (rc != TS_OK) return rc;
    }
    if (p.info.prefill_parts > 0) {
        rc = ensure_pf_parts(c, p.info.prefill_parts);
        if (rc != TS_OK) return rc;
    }
    const WorkLayout w = layout_of(p);
    hipStream_t st = (hipStream_t)stream;
    // new tokens to append and no page check: the upload rides along in the first append launch (not in the
    // allocation-free call, whose upload launch also puts the shared queue heads back to zero)
    const bool ride = k_new && !c->validate_pages && !c->static_call;
    // decode-only batch of matrix-core items whose lists fit into the kernel arguments: the items append the new tokens
    const bool fuse = k_new && !c->validate_pages && c->fused_append && desc_uses_mfma_decode(c->desc) && !p.dec.empty() && p.pf.empty() &&
                p.rows.empty() && p.apt.empty() && p.info.prefill_tokens == 0 && c->dec_nbuf == 2 && !c->merge_in_kernel &&
                p.dec.size() <= (size_t)kSmallDec && p.cmb.size() <= (size_t)kSmallCmb;
    UploadJob job;
    rc = upload_plan(c, st, w, ride || fuse ? &job : nullptr);   // (fused form: nothing to upload)
    if (rc != TS_OK) return rc;
    WorkDoneGuard guard_done{c, st};
    rc = check_pages(c, st, w, block_table, num_seqs);
    if (rc != TS_OK) return rc;

    const Geometry geo = geometry_of(c->desc);
    const char* wb = work_base(c);
    if (k_new && !fuse) {
        AppendArgs ap{};
        ap.geo = geo;
        ap.k_new = k_new; ap.v_new = v_new; ap.k_cache = k_cache; ap.v_cache = v_cache;
        ap.k_scale = k_scale; ap.v_scale = v_scale; ap.block_table = block_table;
        ap.seqs = (const SeqMeta*)(wb + w.seqs);
        ap.num_seqs = num_seqs; ap.total_tokens = (int32_t)p.info.total_tokens;
        ap.apt = (const AppTile*)(wb + w.apt); ap.n_apt = (int32_t)p.apt.size();
        ap.apr = (const AppRow*)(wb + w.apr); ap.n_apr = (int32_t)p.apr.size();
        if (ride) {
            ap.apr_host = (const AppRow*)(job.host_lists + w.apr);
            ap.apt_host = (const AppTile*)(job.host_lists + w.apt);
            ap.up_src = job.src; ap.up_dst = job.dst; ap.up_n16 = job.n16; ap.up_blocks = job.blocks;
        }
        hipError_t e = (hipError_t)timed_launch(c, TS_K_APPEND, true, st, [&] { return launch_append(ap, stream); });
        if (e != hipSuccess) return hip_fail(c, e, "append launch");
    }
    AttnArgs a{};
    a.geo = geo;
    a.q = q; a.k_cache = k_cache; a.v_cache = v_cache; a.k_scale = k_scale; a.v_scale = v_scale;
    a.block_table = block_table;
    a.sm_scale = sm_scale > 0.0f ? sm_scale : 1.0f / sqrtf((float)c->desc.head_dim);
    a.out = out;
    a.dec = (const DecItem*)(wb + w.dec);   a.n_dec = (int32_t)p.dec.size();
    a.cmb = (const CmbItem*)(wb + w.cmb);   a.n_cmb = (int32_t)p.cmb.size();
    a.pf = (const PfItem*)(wb + w.pf);      a.n_pf = (int32_t)p.pf.size();
    a.pfcmb = (const PfCmb*)(wb + w.pfcmb); a.n_pfcmb = (int32_t)p.pfcmb.size();
    a.pf_part_o = c->d_pf_part_o; a.pf_part_ml = c->d_pf_part_ml;
    a.pfmap = (const PfSlot*)(wb + w.pfmap); a.n_pfmap = (int32_t)p.pfmap.size();
    a.rows = (const RowItem*)(wb + w.rows); a.n_rows = (int32_t)p.rows.size();
    a.queue = (const QItem*)(wb + w.queue); a.q_off = (const int32_t*)(wb + w.q_off);
    a.n_queue = (int32_t)p.queue.size(); a.n_xcd = p.q_off.empty() ? 0 : (int32_t)p.q_off.size() - 1;
    a.q_ctr = q_ctr_of(c);
    // (the merging form of the decode kernel exists for a prefetch depth of two tiles and outside the one-kernel launch)
    a.cmb_ctr = c->merge_in_kernel && c->dec_nbuf == 2 && p.info.mixed_mode != TS_MIXED_ONE_KERNEL ? cmb_ctr_of(c, p.cmb.size()) : nullptr;
    a.dec_nbuf = c->dec_nbuf; a.mixed_wgs = c->mixed_wgs; a.n_cu = c->opt.n_cu; a.pf_wgs = p.info.prefill_workgroups;
    a.part_o = part_o_of(c); a.part_ml = part_ml_of(c);
    if (!p.wide.empty()) {
        a.wide = (const WideItem*)(wb + w.wide); a.n_wide = (int32_t)p.wide.size();
        a.wide_base = (const int32_t*)(wb + w.wide_base);
        a.wide_k = c->d_wide_k; a.wide_v = c->d_wide_v;
    }

    if (fuse) { a.k_new = k_new; a.v_new = v_new; }

    hipError_t e;
    // fp8 cache: bf16 copies of the pages the prefill tiles read (behind the append: the chunk's own tokens are among them)
    e = (hipError_t)timed_launch(c, TS_K_PREFILL, false, st, [&] { return launch_widen(a, c->d_wide_k, c->d_wide_v, stream); });
    if (e != hipSuccess) return hip_fail(c, e, "widen launch");
    // decode first: the serving loop's TPOT depends on these rows (Sec. 4.5.2)
    if (a.n_queue > 0 && p.info.mixed_mode == TS_MIXED_CORESIDENT) {
        // mixed batch, co-resident: the prefill tiles go to resident workgroups on this stream, the decode items
        // (and the merge of split rows) to a grid of their own on the side stream, which starts behind everything
        // this stream holds so far (the append) and which this stream waits for again before the call's end
        // is marked.  The prefill launch comes first so that its workgroups take their places on the CUs.
        // Timed as one unit (TS_K_MIXED): events between the two launches would serialise them.
        probe_side_stream(c, st);
        e = (hipError_t)timed_launch(c, TS_K_MIXED, true, st, [&] {
            hipError_t r = hipEventRecord(c->ev_fork, st);
            if (r == hipSuccess) r = (hipError_t)launch_prefill_resident(a, stream);
            if (r == hipSuccess) r = hipStreamWaitEvent(c->side, c->ev_fork, 0);
            if (r == hipSuccess) r = (hipError_t)launch_decode(a, (void*)c->side);
            if (r == hipSuccess && !a.cmb_ctr) r = (hipError_t)launch_combine(a, (void*)c->side);
            // (the join is made even after a failed launch: the side stream must not run on unordered)
            const hipError_t j1 = hipEventRecord(c->ev_join, c->side);
            const hipError_t j2 = j1 == hipSuccess ? hipStreamWaitEvent(st, c->ev_join, 0) : j1;
            return (int)(r != hipSuccess ? r : j2);
        });
        if (e != hipSuccess) return hip_fail(c, e, "co-resident launch");
    } else if (a.n_queue > 0) {
        // mixed batch, by option: decode items and prefill tiles share the workgroups of one persistent launch
        e = (hipError_t)timed_launch(c, TS_K_MIXED, true, st, [&] { return launch_mixed(a, stream); });
        if (e != hipSuccess) return hip_fail(c, e, "mixed launch");
        e = (hipError_t)timed_launch(c, TS_K_COMBINE, a.n_cmb > 0 && !a.cmb_ctr, st, [&] { return a.cmb_ctr ? 0 : launch_combine(a, stream); });
        if (e != hipSuccess) return hip_fail(c, e, "combine launch");
    } else if (fuse) {
        // small decode-only batch: the lists travel as kernel arguments, the items append the new tokens
        // (nothing was uploaded: the staging slot only lends the call its event)
        SmallLists sl{};
        sl.n_dec = (int32_t)p.dec.size(); sl.n_cmb = (int32_t)p.cmb.size();
        std::copy(p.dec.begin(), p.dec.end(), sl.dec);
        std::copy(p.cmb.begin(), p.cmb.end(), sl.cmb);
        e = (hipError_t)timed_launch(c, TS_K_DECODE, true, st, [&] { return launch_decode_fused(a, sl, stream); });
        if (e != hipSuccess) return hip_fail(c, e, "fused decode launch");
    } else {
        e = (hipError_t)timed_launch(c, TS_K_DECODE, a.n_dec > 0, st, [&] { return launch_decode(a, stream); });
        if (e != hipSuccess) return hip_fail(c, e, "decode launch");
        e = (hipError_t)timed_launch(c, TS_K_COMBINE, a.n_cmb > 0 && !a.cmb_ctr, st, [&] { return a.cmb_ctr ? 0 : launch_combine(a, stream); });
        if (e != hipSuccess) return hip_fail(c, e, "combine launch");
        e = (hipError_t)timed_launch(c, TS_K_PREFILL, a.n_pf > 0, st, [&] { return launch_prefill(a, stream); });
        if (e != hipSuccess) return hip_fail(c, e, "prefill launch");
    }
    e = (hipError_t)timed_launch(c, TS_K_COMBINE, a.n_pfcmb > 0, st, [&] { return launch_prefill_combine(a, stream); });
    if (e != hipSuccess) return hip_fail(c, e, "prefill combine launch");
    e = (hipError_t)timed_launch(c, TS_K_ROWS, a.n_rows > 0, st, [&] { return launch_rows(a, stream); });
    if (e != hipSuccess) return hip_fail(c, e, "rows launch");

    rc = mark_work_done(c, st);
    if (rc != TS_OK) return rc;
    {
        std::lock_guard<std::mutex> lk(c->mu);
        if (!c->window_open) { c->window_open = true; c->t0 = std::chrono::steady_clock::now(); }
        c->prefill_tokens += (uint64_t)p.info.prefill_tokens;
        c->decode_tokens += (uint64_t)p.info.decode_tokens;
        c->passes += 1;
    }
    return TS_OK;
}

}  // namespace

extern "C" int ts_mixed_paged_attention(ts_ctx* c, void* stream, const void* q, const void* k_new,
                                        const void* v_new, void* k_cache, void* v_cache,
                                        const float* k_scale, const float* v_scale,
                                        const int32_t* block_table, const int32_t* q_lens,
                                        const int32_t* ctx_lens, int num_seqs, float sm_scale, void* out)
{
    if (!c) return TS_ERR_INVALID_ARG;
    c->static_call = false;
    return mixed_pass(c, stream, q, k_new, v_new, k_cache, v_cache, k_scale, v_scale, block_table, q_lens, ctx_lens,
                      num_seqs, sm_scale, out);
}

extern "C" int ts_mixed_paged_attention_noalloc(ts_ctx* c, void* stream, const void* q, const void* k_new,
                                                const void* v_new, void* k_cache, void* v_cache,
                                                const float* k_scale, const float* v_scale,
                                                const int32_t* block_table, const int32_t* q_lens,
                                                const int32_t* ctx_lens, int num_seqs, float sm_scale, void* out)
{
    if (!c) return TS_ERR_INVALID_ARG;
    c->static_call = true;
    const int rc = mixed_pass(c, stream, q, k_new, v_new, k_cache, v_cache, k_scale, v_scale, block_table, q_lens,
                              ctx_lens, num_seqs, sm_scale, out);
    c->static_call = false;
    return rc;
}

extern "C" int ts_token_velocity(ts_ctx* c, ts_velocity* out, int flags)
{
    if (!c || !out) return TS_ERR_INVALID_ARG;
    if (flags & ~(TS_VELOCITY_RESET | TS_VELOCITY_SYNC)) return fail(c, TS_ERR_INVALID_ARG, "unknown flag");
    if ((flags & TS_VELOCITY_SYNC) && c->have_work) {
        DeviceGuard guard(c->device);
        TS_HIP(c, hipEventSynchronize(c->last_event));     // the most recent call's end (a pass or an append)
    }
    std::lock_guard<std::mutex> lk(c->mu);
    ts_velocity v{};
    v.prefill_tokens = c->prefill_tokens;
    v.decode_tokens = c->decode_tokens;
    v.passes = c->passes;
    if (c->window_open) {
        v.window_s = std::chrono::duration<double>(std::chrono::steady_clock::now() - c->t0).count();
        if (v.window_s > 0) {
            v.prefill_tok_per_s = (double)v.prefill_tokens / v.window_s;
            v.decode_tok_per_s = (double)v.decode_tokens / v.window_s;
        }
    }
    *out = v;
    if (flags & TS_VELOCITY_RESET) {
        c->prefill_tokens = c->decode_tokens = c->passes = 0;
        c->window_open = false;
    }
    return TS_OK;
}

extern "C" int ts_kernel_times(ts_ctx* c, ts_kernel_stats* out, int reset)
{
    if (!c || !out) return TS_ERR_INVALID_ARG;
    DeviceGuard guard(c->device);
    int rc = drain_timed(c);
    if (rc != TS_OK) return rc;
    for (int k = 0; k < TS_K_COUNT; ++k) {
        out->launches[k] = c->k_launches[k];
        out->mean_ms[k] = c->k_launches[k] ? c->k_ms[k] / (double)c->k_launches[k] : 0.0;
        if (reset) { c->k_launches[k] = 0; c->k_ms[k] = 0.0; }
    }
    return TS_OK;
}
