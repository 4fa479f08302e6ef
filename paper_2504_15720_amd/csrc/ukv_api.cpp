// C-ABI entry points that enqueue device work: append, decode attention, gather.
// Host side only marshals: it plans, writes the plan into a pinned, device-mapped staging slot,
// and launches the kernels on the caller's stream (a small copy kernel moves the decode plan
// into the workspace; the append and gather kernels read their few records in place).
#include <algorithm>
#include <cstring>
#include <new>
#include <string>
#include <utility>
#include <vector>

#include "ukv_internal.h"

using namespace ukv;

namespace {

int hip_fail(hipError_t e, const char *what) {
    set_error(std::string(what) + ": " + hipGetErrorString(e));
    return UKV_EHIP;
}
#define HIP_TRY(expr, what)                                                                                        \
    do {                                                                                                           \
        hipError_t e_ = (expr);                                                                                    \
        if (e_ != hipSuccess)                                                                                      \
            return hip_fail(e_, what);                                                                             \
    } while (0)

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// Pinned staging ring: a slot is reused only after the copy that read it has completed.
int stage_acquire(ukv_pool *p, size_t bytes, ukv_pool::Stage **out) {
    ukv_pool::Stage &st = p->stage[p->next_stage];
    p->next_stage = (p->next_stage + 1) % ukv_pool::kStages;
    if (!st.ev)
        HIP_TRY(hipEventCreateWithFlags(&st.ev, hipEventDisableTiming), "hipEventCreate");
    if (st.pending) {
        HIP_TRY(hipEventSynchronize(st.ev), "hipEventSynchronize(staging)");
        st.pending = false;
    }
    if (st.cap < bytes) {
        if (st.host)
            HIP_TRY(hipHostFree(st.host), "hipHostFree");
        st.host = nullptr;
        st.cap = 0;
        const size_t cap = std::max<size_t>(align_up(bytes * 2, 4096), 64 * 1024);
        HIP_TRY(hipHostMalloc(&st.host, cap, hipHostMallocMapped), "hipHostMalloc");
        HIP_TRY(hipHostGetDevicePointer(&st.mapped, st.host, 0), "hipHostGetDevicePointer");
        st.cap = cap;
    }
    *out = &st;
    return UKV_OK;
}

// The slot may be rewritten once everything enqueued so far (its readers included) has run.
int stage_release_after(ukv_pool::Stage *st, hipStream_t s) {
    HIP_TRY(hipEventRecord(st->ev, s), "hipEventRecord(staging)");
    st->pending = true;
    return UKV_OK;
}

// Once a kernel that reads a staging slot has been enqueued, the slot must not be rewritten before that kernel has
// run, whatever way the call ends: leaving the scope with `launched` set records the slot's event (if even that
// fails, the stream is drained).  The normal path calls done(), which reports errors.
struct StageUse {
    ukv_pool::Stage *st;
    hipStream_t s;
    bool launched = false;
    int done() {
        launched = false;
        return stage_release_after(st, s);
    }
    ~StageUse() {
        if (!launched)
            return;
        if (hipEventRecord(st->ev, s) == hipSuccess)
            st->pending = true;
        else
            (void)hipStreamSynchronize(s);
    }
};

// Profiling: the kernel's own start/stop timestamps, attached to its dispatch (no extra
// barriers on the stream).  get() hands out a pair when profiling is on, else nulls.
static constexpr size_t kMaxPendingTimings = 8192; // launches timed but not yet read by ukv_profile_read

struct ProfPair {
    ukv_pool *p;
    int which;
    ukv_pool::EvPair ev{nullptr, nullptr, 0};
    int get() {
        if (!p->tun.profile)
            return UKV_OK;
        if (p->prof_seq[which]++ % (uint64_t)p->tun.profile != 0) // one launch in `profile` of each kind is timed
            return UKV_OK;
        if (p->ev_used.size() >= kMaxPendingTimings) { // nobody reads the profile: drop the oldest timings
            p->ev_free.insert(p->ev_free.end(), p->ev_used.begin(), p->ev_used.end());
            p->ev_used.clear();
        }
        if (p->ev_free.empty()) { // create a batch at once, so the timed loop rarely creates events
            for (int k = 0; k < 64; ++k) {
                ukv_pool::EvPair e{nullptr, nullptr, 0};
                HIP_TRY(hipEventCreate(&e.a), "hipEventCreate");
                HIP_TRY(hipEventCreate(&e.b), "hipEventCreate");
                p->ev_free.push_back(e);
            }
        }
        ev = p->ev_free.back();
        p->ev_free.pop_back();
        ev.which = which;
        return UKV_OK;
    }
    void done() { // the launch went out: the pair now waits for ukv_profile_read
        if (ev.a)
            p->ev_used.push_back(ev);
        ev.a = ev.b = nullptr;
    }
    ~ProfPair() { // the launch failed: the pair was never recorded and can be handed out again
        if (ev.a)
            p->ev_free.push_back(ev);
    }
};

// Opt-in check of the page tables (UKV_PARAM_VALIDATE).  report_bad_tables: at the start of every compute call,
// turns what an earlier call's check found into UKV_EINVAL.  validate_tables: enqueues the check of entries
// [0, ceil((ctx_len + adjust) T / P)) of every request (after the call's patches, before its kernels) and hands back
// the device address of the flag that makes those kernels leave at once; null while the check is off.
int report_bad_tables(ukv_pool *p, hipStream_t s) {
    if (!p->tun.validate || !p->val_host)
        return UKV_OK;
    volatile ValReport *r = p->val_host;
    if (!r->bad)
        return UKV_OK;
    HIP_TRY(hipMemsetAsync(p->val_flag, 0, sizeof(uint32_t), s), "hipMemsetAsync(check flag)");
    set_error("an earlier checked call found page id " + std::to_string((long long)r->page) + " in page_table[" +
              std::to_string((unsigned long long)r->entry) + "] (request " + std::to_string(r->req) +
              " of that call); the pool has " + std::to_string((unsigned long long)p->n_pages) +
              " pages.  The kernels of that call did nothing.");
    r->bad = 0;
    ++p->tun_epoch; // launches that left early did not advance their plan's span queue: kept plans are remade
    return UKV_EINVAL;
}

int validate_tables(ukv_pool *p, uint32_t n, const uint32_t *service_id, const uint32_t *ctx_len,
                    const uint64_t *table_off, const int32_t *page_table, int adjust, hipStream_t s,
                    const uint32_t **bad_out) {
    *bad_out = nullptr;
    if (!p->tun.validate || n == 0)
        return UKV_OK;
    if (!p->val_host) {
        void *h = nullptr, *d = nullptr;
        HIP_TRY(hipHostMalloc(&h, sizeof(ValReport), hipHostMallocMapped), "hipHostMalloc");
        std::memset(h, 0, sizeof(ValReport));
        HIP_TRY(hipHostGetDevicePointer(&d, h, 0), "hipHostGetDevicePointer");
        p->val_host = (ValReport *)h;
        p->val_dev = (ValReport *)d;
        void *f = nullptr;
        HIP_TRY(hipMalloc(&f, 256), "hipMalloc(check flag)");
        p->val_flag = (uint32_t *)f;
        HIP_TRY(hipMemsetAsync(f, 0, 256, s), "hipMemsetAsync(check flag)");
    }
    ukv_pool::Stage *st = nullptr;
    int rc = stage_acquire(p, align_up((size_t)n * sizeof(ValRec)), &st);
    if (rc != UKV_OK)
        return rc;
    ValRec *recs = (ValRec *)st->host;
    for (uint32_t i = 0; i < n; ++i) {
        const int64_t c = (int64_t)ctx_len[i] + adjust;
        recs[i] = ValRec{table_off[i], c > 0 ? ukv_pages_for_tokens(p, service_id[i], (uint64_t)c) : 0, i, 0};
    }
    HIP_TRY(launch_validate(page_table, (const ValRec *)st->mapped, n, p->n_pages, p->val_dev, p->val_flag, s),
            "launch page-table check");
    if ((rc = stage_release_after(st, s)) != UKV_OK)
        return rc;
    *bad_out = p->val_flag;
    return UKV_OK;
}

struct BlobLayout {
    size_t recs, spans, reduce, counters, queue, total;
};

BlobLayout blob_layout(size_t n_seqs, size_t n_items, size_t n_spans, size_t n_reduce) {
    BlobLayout b{};
    size_t o = 0;
    b.recs = o;
    o = align_up(o + n_items * sizeof(ItemRec));
    b.spans = o;
    o = align_up(o + (n_spans + 1) * sizeof(uint32_t));
    b.reduce = o;
    o = align_up(o + n_reduce * sizeof(ReduceRec));
    b.counters = o;
    o = align_up(o + n_seqs * sizeof(uint32_t));
    b.queue = o; // span queue counter; zero like the counters
    o = align_up(o + sizeof(uint32_t));
    b.total = o;
    return b;
}

size_t max_slices(const ukv_pool *p) {
    size_t m = 1;
    for (uint32_t s = 0; s < p->n_services; ++s)
        m = std::max<size_t>(m, p->classes.c[s].n_kv / p->classes.c[s].hs);
    return m;
}

size_t blob_capacity(const ukv_pool *p, uint32_t n_requests) {
    const size_t n_seqs = (size_t)n_requests * max_slices(p);
    const size_t n_spans = (size_t)(2 * p->tun.max_spans + 2);
    return blob_layout(n_seqs, n_seqs + n_spans, n_spans, n_seqs).total;
}

} // namespace

extern "C" {

size_t ukv_decode_workspace_bytes(const ukv_pool_t *p, uint32_t n_requests) {
    if (!p)
        return 0;
    return blob_capacity(p, n_requests) + align_up(max_partial_floats(p, n_requests) * sizeof(float));
}

int ukv_plan_decode(const ukv_pool_t *p, const ukv_batch_t *b, ukv_plan_info_t *info, uint32_t *items_out,
                    uint32_t n_items_cap) {
    if (!p || !b || !info) {
        set_error("null argument");
        return UKV_EINVAL;
    }
    Plan plan;
    int rc = build_plan(p, b, plan);
    if (rc != UKV_OK)
        return rc;
    info->n_seqs = (uint32_t)plan.seqs.size();
    info->n_items = (uint32_t)plan.items.size();
    info->n_spans = (uint32_t)plan.span_first.size() - 1;
    info->n_reduce = (uint32_t)plan.reduce.size();
    info->partial_floats = plan.partial_floats;
    info->plan_bytes = blob_layout(plan.seqs.size(), plan.items.size(), info->n_spans, plan.reduce.size()).total;
    info->kv_bytes = plan.kv_bytes;
    if (items_out) {
        const uint32_t n = std::min<uint32_t>(n_items_cap, info->n_items);
        for (uint32_t it = 0; it < n; ++it) {
            const Item &x = plan.items[it];
            const SeqRec &s = plan.seqs[x.seq];
            uint32_t *row = items_out + (size_t)it * 6;
            row[0] = plan.seq_req[x.seq];
            row[1] = s.head0;
            row[2] = p->classes.c[s.cls].hs;
            row[3] = x.t0;
            row[4] = x.t1;
            row[5] = plan.item_span[it];
        }
    }
    return UKV_OK;
}

} // extern "C"

// A plan kept in the caller's workspace across steps (ukv_plan_*): the launch parameters of the resident plan, the
// host's copy of the batch arrays (lengths advance with every step) and the step's new page ids as they go into the
// kernel arguments.
struct ukv_plan {
    ukv_pool *pool = nullptr;
    uint32_t n = 0;
    std::vector<uint32_t> service_id, ctx_len;
    std::vector<uint64_t> table_off, q_off, out_off, new_off, patch_entry;
    ukv_plan_io_t io{};
    void *workspace = nullptr;
    size_t ws_bytes = 0;
    bool resident = false; // the workspace holds a plan
    uint32_t delta = 0;    // tokens every request has grown since that plan was made
    uint64_t tun_epoch = 0;
    DecodeArgs args{};
    uint32_t n_spans = 0;
    uint32_t grid = 0;     // workgroups of a launch of the resident plan
    uint32_t queue_at = 0; // value of the span queue's counter after the launches enqueued so far (mod 2^32)
    size_t reduce_off = 0;
    uint32_t n_reduce = 0, n_reduce_many = 0, max_reduce_heads = 0, max_reduce_units = 0;
    StepPages sp{};
};

extern "C" {

// Attention alone, or (with_append) the whole step: the new page-table entries ride with the plan
// upload and the new tokens are stored by the decode workgroups that attend to them.  keep: where to note the
// launch parameters, for later launches of the same plan.
static int decode_impl(ukv_pool_t *p, const ukv_batch_t *b, void *workspace, size_t ws_bytes, void *stream,
                       bool with_append, ukv_plan *keep = nullptr) {
    Trace trace(keep ? "ukv_plan_step(replan)" : with_append ? "ukv_decode_step" : "ukv_decode_attention");
    if (!p || !b) {
        set_error("null pool or batch");
        return UKV_EINVAL;
    }
    const uint32_t n_patches = with_append ? b->n_patches : 0;
    if (b->n_requests == 0 && n_patches == 0)
        return UKV_OK;
    if (!b->page_table || (b->n_requests && (!b->q || !b->out))) {
        set_error("page_table, q and out must be non-null device pointers");
        return UKV_EINVAL;
    }
    if (with_append) {
        if (b->n_requests && (!b->new_k || !b->new_v || !b->new_off)) {
            set_error("a decode step needs new_k, new_v and new_off");
            return UKV_EINVAL;
        }
        if (n_patches && (!b->patch_entry || !b->patch_page)) {
            set_error("patch arrays missing");
            return UKV_EINVAL;
        }
        for (uint32_t i = 0; i < n_patches; ++i)
            if (b->patch_page[i] < 0 || (uint64_t)b->patch_page[i] >= p->n_pages) {
                set_error("patch page id out of range");
                return UKV_EINVAL;
            }
        for (uint32_t i = 0; i < b->n_requests; ++i)
            if (b->new_off[i] & 7) {
                set_error("new_off must be a multiple of 8 elements");
                return UKV_EINVAL;
            }
    }
    if (!workspace || ((uintptr_t)workspace & 255)) {
        set_error("workspace must be non-null and 256-byte aligned");
        return UKV_EINVAL;
    }
    hipStream_t s = (hipStream_t)stream;
    int rc = report_bad_tables(p, s);
    if (rc != UKV_OK)
        return rc;
    if (p->tun.slots_auto) { // once per pool (and after a block-size change): what the device keeps resident
        const int r = decode_resident_workgroups((uint32_t)p->tun.block_threads);
        if (r > 0)
            p->tun.slots = r;
        p->tun.slots_auto = false;
    }
    Plan &plan = p->plan_scratch; // storage reused from call to call
    rc = build_plan(p, b, plan);
    if (rc != UKV_OK)
        return rc;
    if (with_append)
        for (size_t k = 0; k < plan.seqs.size(); ++k)
            plan.seqs[k].new_off = b->new_off[plan.seq_req[k]];
    const uint32_t n_spans = (uint32_t)plan.span_first.size() - 1;
    const BlobLayout L = blob_layout(plan.seqs.size(), plan.items.size(), n_spans, plan.reduce.size());
    const size_t part_off = align_up(L.total);
    if (part_off + plan.partial_floats * sizeof(float) > ws_bytes) {
        set_error("workspace too small for this batch");
        return UKV_ENOSPC;
    }
    // the patch arrays are only read by the upload kernel, from the staging slot itself
    const size_t off_pe = align_up(L.total);
    const size_t off_pp = align_up(off_pe + (size_t)n_patches * sizeof(uint64_t));
    const size_t stage_bytes = align_up(off_pp + (size_t)n_patches * sizeof(int32_t));
    ukv_pool::Stage *st = nullptr;
    rc = stage_acquire(p, stage_bytes, &st);
    if (rc != UKV_OK)
        return rc;
    unsigned char *h = (unsigned char *)st->host;
    ItemRec *recs = (ItemRec *)(h + L.recs);
    for (size_t it = 0; it < plan.items.size(); ++it) {
        recs[it].it = plan.items[it];
        recs[it].s = plan.seqs[plan.items[it].seq];
        recs[it].c = p->classes.c[recs[it].s.cls];
    }
    std::memcpy(h + L.spans, plan.span_first.data(), plan.span_first.size() * sizeof(uint32_t));
    if (!plan.reduce.empty())
        std::memcpy(h + L.reduce, plan.reduce.data(), plan.reduce.size() * sizeof(ReduceRec));
    std::memset(h + L.counters, 0, L.total - L.counters);
    if (n_patches) {
        std::memcpy(h + off_pe, b->patch_entry, (size_t)n_patches * sizeof(uint64_t));
        std::memcpy(h + off_pp, b->patch_page, (size_t)n_patches * sizeof(int32_t));
    }
    const unsigned char *hm = (const unsigned char *)st->mapped;
    HIP_TRY(launch_stage_copy(workspace, st->mapped, L.total, b->page_table, (const uint64_t *)(hm + off_pe),
                              (const int32_t *)(hm + off_pp), n_patches, s),
            "launch plan upload");
    if ((rc = stage_release_after(st, s)) != UKV_OK)
        return rc;

    unsigned char *w = (unsigned char *)workspace;
    DecodeArgs a{};
    a.pool_base = p->base;
    a.log2_page = p->log2_page;
    a.page_table = b->page_table;
    a.q = b->q;
    a.out = (float *)b->out;
    a.recs = (const ItemRec *)(w + L.recs);
    a.span_first = (const uint32_t *)(w + L.spans);
    a.partials = (float *)(w + part_off);
    const bool fused = p->tun.fused_merge != 0;
    a.counters = fused ? (uint32_t *)(w + L.counters) : nullptr;
    a.merge_acq_rel = p->tun.merge_acq_rel ? 1u : 0u;
    a.new_k = with_append ? (const uint16_t *)b->new_k : nullptr;
    a.new_v = with_append ? (const uint16_t *)b->new_v : nullptr;
    a.delta = 0;
    if ((rc = validate_tables(p, b->n_requests, b->service_id, b->ctx_len, b->table_off, b->page_table, 0, s,
                              &a.bad)) != UKV_OK)
        return rc;
    a.queue = (uint32_t *)(w + L.queue);
    a.queue_base = 0; // the upload has just zeroed the counter
    a.n_spans = n_spans;
    a.n_spans_dev = nullptr;
    const uint32_t grid = decode_grid(n_spans, (uint32_t)p->tun.block_threads, p->kinds,
                                      p->tun.grid_is_first_round ? (uint32_t)p->tun.slots : 0);
    trace.add("requests", b->n_requests);
    trace.add("kv_bytes", plan.kv_bytes);
    trace.add("sequences", plan.seqs.size());
    trace.add("items", plan.items.size());
    trace.add("spans", n_spans);
    trace.add("workgroups", grid);
    trace.add("partial_floats", plan.partial_floats);
    trace.add("merged_by_second_launch", plan.reduce.size());
    if (keep) {
        keep->args = a;
        keep->grid = grid;
        keep->queue_at = n_spans; // where this launch leaves the counter
        keep->n_spans = n_spans;
        keep->reduce_off = L.reduce;
        keep->n_reduce = (uint32_t)plan.reduce.size();
        keep->n_reduce_many = plan.n_reduce_many;
        keep->max_reduce_heads = plan.max_reduce_heads;
        keep->max_reduce_units = plan.max_reduce_units;
    }

    if (n_spans) {
        ProfPair pp{p, 0};
        if ((rc = pp.get()) != UKV_OK)
            return rc;
        HIP_TRY(launch_decode(a, nullptr, grid, (uint32_t)p->tun.block_threads, p->kinds, s, pp.ev.a, pp.ev.b),
                "launch decode kernel");
        pp.done();
    }
    if (!plan.reduce.empty()) { // every cut sequence (two-launch mode), or only those with very many parts
        ProfPair pp{p, 1};
        if ((rc = pp.get()) != UKV_OK)
            return rc;
        HIP_TRY(launch_reduce((const ReduceRec *)(w + L.reduce), (uint32_t)plan.reduce.size(), plan.n_reduce_many,
                              plan.max_reduce_heads, plan.max_reduce_units, a.partials, a.out, s, pp.ev.a, pp.ev.b),
                "launch reduce kernel");
        pp.done();
    }
    return UKV_OK;
}

int ukv_decode_attention(ukv_pool_t *p, const ukv_batch_t *b, void *workspace, size_t ws_bytes, void *stream) {
    return decode_impl(p, b, workspace, ws_bytes, stream, false);
}

int ukv_decode_step(ukv_pool_t *p, const ukv_batch_t *b, void *workspace, size_t ws_bytes, void *stream) {
    return decode_impl(p, b, workspace, ws_bytes, stream, true);
}

int ukv_plan_create(ukv_pool_t *p, const ukv_batch_t *b, void *workspace, size_t ws_bytes, ukv_plan_t **out) {
    if (!p || !b || !out) {
        set_error("null argument");
        return UKV_EINVAL;
    }
    *out = nullptr;
    const uint32_t n = b->n_requests;
    if (n && (!b->service_id || !b->ctx_len || !b->table_off || !b->q_off || !b->out_off || !b->new_off)) {
        set_error("batch host arrays must be non-null");
        return UKV_EINVAL;
    }
    if (!b->page_table || (n && (!b->q || !b->out || !b->new_k || !b->new_v))) {
        set_error("page_table, q, out, new_k and new_v must be non-null device pointers");
        return UKV_EINVAL;
    }
    if (!workspace || ((uintptr_t)workspace & 255) || ws_bytes < ukv_decode_workspace_bytes(p, n)) {
        set_error("workspace must be 256-byte aligned and hold ukv_decode_workspace_bytes(pool, n_requests)");
        return workspace && !((uintptr_t)workspace & 255) ? UKV_ENOSPC : UKV_EINVAL;
    }
    for (uint32_t i = 0; i < n; ++i) {
        if (b->service_id[i] >= p->n_services) {
            set_error("service_id out of range");
            return UKV_EINVAL;
        }
        if ((b->q_off[i] & 7) || (b->out_off[i] & 3) || (b->new_off[i] & 7)) {
            set_error("q_off and new_off must be multiples of 8 elements, out_off of 4");
            return UKV_EINVAL;
        }
        if (ukv_pages_for_tokens(p, b->service_id[i], b->ctx_len[i]) > p->n_pages) {
            set_error("ctx_len exceeds what the pool can hold");
            return UKV_EINVAL;
        }
    }
    ukv_plan *pl = new (std::nothrow) ukv_plan();
    if (!pl) {
        set_error("host allocation failed");
        return UKV_ENOMEM;
    }
    pl->pool = p;
    pl->n = n;
    pl->service_id.assign(b->service_id, b->service_id + n);
    pl->ctx_len.assign(b->ctx_len, b->ctx_len + n);
    pl->table_off.assign(b->table_off, b->table_off + n);
    pl->q_off.assign(b->q_off, b->q_off + n);
    pl->out_off.assign(b->out_off, b->out_off + n);
    pl->new_off.assign(b->new_off, b->new_off + n);
    pl->io = ukv_plan_io_t{b->page_table, b->q, b->out, b->new_k, b->new_v};
    pl->workspace = workspace;
    pl->ws_bytes = ws_bytes;
    *out = pl;
    return UKV_OK;
}

int ukv_plan_destroy(ukv_plan_t *pl) {
    delete pl;
    return UKV_OK;
}

int ukv_plan_lengths(const ukv_plan_t *pl, uint32_t *ctx_len_out, uint32_t n) {
    if (!pl || (n && !ctx_len_out) || n != pl->n) {
        set_error("bad plan, output or count");
        return UKV_EINVAL;
    }
    std::memcpy(ctx_len_out, pl->ctx_len.data(), (size_t)n * sizeof(uint32_t));
    return UKV_OK;
}

int ukv_plan_step(ukv_plan_t *pl, const ukv_plan_io_t *io_in, int advance, const int32_t *new_pages,
                  uint32_t n_new_pages, void *stream) {
    if (!pl || (n_new_pages && !new_pages)) {
        set_error("null plan or page array");
        return UKV_EINVAL;
    }
    ukv_pool *p = pl->pool;
    const uint32_t n = pl->n;
    if (n == 0)
        return UKV_OK;
    const ukv_plan_io_t io = io_in ? *io_in : pl->io;
    if (!io.page_table || !io.q || !io.out || !io.new_k || !io.new_v) {
        set_error("page_table, q, out, new_k and new_v must be non-null device pointers");
        return UKV_EINVAL;
    }
    const uint32_t grow = advance ? 1u : 0u;
    // the table entries this step adds: request i gains entries [ceil((c-1) T / P), ceil(c T / P)), c its new length
    const bool in_args = n <= kStepMaxReq;
    uint64_t total = 0;
    for (uint32_t i = 0; i < n; ++i) {
        const uint64_t c = (uint64_t)pl->ctx_len[i] + grow;
        const uint32_t cls = pl->service_id[i];
        const uint64_t hi = ukv_pages_for_tokens(p, cls, c);
        if (c > 0xffffffffull || hi > p->n_pages || (c && hi == 0)) {
            set_error("a request outgrows the pool");
            return UKV_EINVAL;
        }
        if (in_args)
            pl->sp.first[i] = (uint16_t)std::min<uint64_t>(total, 0xffff);
        total += c ? hi - ukv_pages_for_tokens(p, cls, c - 1) : 0;
    }
    if (total != n_new_pages) {
        set_error("n_new_pages must be the number of table entries the step adds (" + std::to_string(total) + ")");
        return UKV_EINVAL;
    }
    for (uint32_t k = 0; k < n_new_pages; ++k)
        if (new_pages[k] < 0 || (uint64_t)new_pages[k] >= p->n_pages) {
            set_error("new page id out of range");
            return UKV_EINVAL;
        }
    const bool fast = pl->resident && in_args && total <= kStepMaxPages && pl->tun_epoch == p->tun_epoch &&
                      (uint64_t)pl->delta + grow <= (uint64_t)p->tun.replan_every;
    hipStream_t s = (hipStream_t)stream;
    if (!fast) {
        // Plan for the lengths as they are now and upload (the route of ukv_decode_step); the plan stays behind.
        pl->patch_entry.clear();
        for (uint32_t i = 0; i < n; ++i) {
            const uint64_t c = (uint64_t)pl->ctx_len[i] + grow;
            if (c == 0)
                continue;
            const uint64_t lo = ukv_pages_for_tokens(p, pl->service_id[i], c - 1),
                           hi = ukv_pages_for_tokens(p, pl->service_id[i], c);
            for (uint64_t e = lo; e < hi; ++e)
                pl->patch_entry.push_back(pl->table_off[i] + e);
        }
        for (uint32_t i = 0; i < n; ++i)
            pl->ctx_len[i] += grow;
        ukv_batch_t b{};
        b.n_requests = n;
        b.service_id = pl->service_id.data();
        b.ctx_len = pl->ctx_len.data();
        b.table_off = pl->table_off.data();
        b.page_table = io.page_table;
        b.q = io.q;
        b.q_off = pl->q_off.data();
        b.out = io.out;
        b.out_off = pl->out_off.data();
        b.new_k = io.new_k;
        b.new_v = io.new_v;
        b.new_off = pl->new_off.data();
        b.n_patches = n_new_pages;
        b.patch_entry = pl->patch_entry.data();
        b.patch_page = new_pages;
        pl->resident = false;
        const int rc = decode_impl(p, &b, pl->workspace, pl->ws_bytes, stream, true, pl);
        if (rc != UKV_OK) {
            for (uint32_t i = 0; i < n; ++i)
                pl->ctx_len[i] -= grow;
            return rc;
        }
        pl->resident = true;
        pl->delta = 0;
        pl->tun_epoch = p->tun_epoch;
        return UKV_OK;
    }
    // The resident plan serves: one launch, the new page ids in its arguments.
    Trace trace("ukv_plan_step");
    trace.add("requests", n);
    trace.add("new_pages", n_new_pages);
    trace.add("grown_since_plan", pl->delta + grow);
    trace.add("spans", pl->n_spans);
    trace.add("workgroups", pl->grid);
    int rc = report_bad_tables(p, s);
    if (rc != UKV_OK)
        return rc;
    pl->sp.n_req = n;
    pl->sp.first[n] = (uint16_t)total;
    if (n_new_pages)
        std::memcpy(pl->sp.page, new_pages, (size_t)n_new_pages * sizeof(int32_t));
    DecodeArgs a = pl->args;
    a.page_table = io.page_table;
    a.q = io.q;
    a.out = (float *)io.out;
    a.new_k = (const uint16_t *)io.new_k;
    a.new_v = (const uint16_t *)io.new_v;
    a.delta = pl->delta + grow;
    a.queue_base = pl->queue_at;
    // (the entries this step adds are not in the table yet: they were checked on the host above)
    if ((rc = validate_tables(p, n, pl->service_id.data(), pl->ctx_len.data(), pl->table_off.data(), io.page_table,
                              (int)grow - 1, s, &a.bad)) != UKV_OK)
        return rc;
    if (pl->n_spans) {
        ProfPair pp{p, 0};
        if ((rc = pp.get()) != UKV_OK)
            return rc;
        HIP_TRY(launch_decode(a, &pl->sp, pl->grid, (uint32_t)p->tun.block_threads, p->kinds, s, pp.ev.a, pp.ev.b),
                "launch decode kernel");
        pp.done();
        pl->queue_at += pl->n_spans;
    }
    for (uint32_t i = 0; i < n; ++i)
        pl->ctx_len[i] += grow;
    pl->delta += grow;
    if (pl->n_reduce) {
        ProfPair pp{p, 1};
        if ((rc = pp.get()) != UKV_OK)
            return rc;
        HIP_TRY(launch_reduce((const ReduceRec *)((unsigned char *)pl->workspace + pl->reduce_off), pl->n_reduce,
                              pl->n_reduce_many, pl->max_reduce_heads, pl->max_reduce_units, a.partials, a.out, s,
                              pp.ev.a, pp.ev.b),
                "launch reduce kernel");
        pp.done();
    }
    return UKV_OK;
}

int ukv_append(ukv_pool_t *p, const ukv_batch_t *b, void *stream) {
    Trace trace("ukv_append");
    if (b) {
        trace.add("requests", b->n_requests);
        trace.add("patches", b->n_patches);
    }
    if (!p || !b) {
        set_error("null pool or batch");
        return UKV_EINVAL;
    }
    const uint32_t n = b->n_requests;
    if (n == 0 && b->n_patches == 0)
        return UKV_OK;
    if (!b->page_table || (n && (!b->new_k || !b->new_v || !b->service_id || !b->ctx_len || !b->table_off ||
                                 !b->new_off))) {
        set_error("append needs page_table, new_k, new_v and the host arrays");
        return UKV_EINVAL;
    }
    if (b->n_patches && (!b->patch_entry || !b->patch_page)) {
        set_error("patch arrays missing");
        return UKV_EINVAL;
    }
    for (uint32_t i = 0; i < b->n_patches; ++i)
        if (b->patch_page[i] < 0 || (uint64_t)b->patch_page[i] >= p->n_pages) {
            set_error("patch page id out of range");
            return UKV_EINVAL;
        }
    for (uint32_t i = 0; i < n; ++i) {
        if (b->service_id[i] >= p->n_services) {
            set_error("service_id out of range");
            return UKV_EINVAL;
        }
        if (b->new_off[i] & 7) {
            set_error("new_off must be a multiple of 8 elements");
            return UKV_EINVAL;
        }
        if (ukv_pages_for_tokens(p, b->service_id[i], b->ctx_len[i]) > p->n_pages) {
            set_error("ctx_len exceeds what the pool can hold");
            return UKV_EINVAL;
        }
    }
    hipStream_t s = (hipStream_t)stream;
    int rc = report_bad_tables(p, s);
    if (rc != UKV_OK)
        return rc;
    size_t o = 0;
    const size_t off_cls = o;
    o = align_up(o + sizeof(ClassTable));
    const size_t off_recs = o;
    o = align_up(o + (size_t)n * sizeof(AppendRec));
    const size_t off_pe = o;
    o = align_up(o + (size_t)b->n_patches * sizeof(uint64_t));
    const size_t off_pp = o;
    o = align_up(o + (size_t)b->n_patches * sizeof(int32_t));
    const size_t total = o;
    ukv_pool::Stage *st = nullptr;
    if ((rc = stage_acquire(p, total, &st)) != UKV_OK)
        return rc;
    unsigned char *h = (unsigned char *)st->host;
    std::memcpy(h + off_cls, &p->classes, sizeof(ClassTable));
    // Entries patched by this call are handed to the append workgroups directly, so that patching
    // and appending can share one launch; a token touching more than four pages takes two launches.
    std::vector<std::pair<uint64_t, int32_t>> &patched = p->patch_scratch; // (entry, page) by entry; storage reused
    patched.clear();
    for (uint32_t i = 0; i < b->n_patches; ++i)
        patched.emplace_back(b->patch_entry[i], b->patch_page[i]);
    std::stable_sort(patched.begin(), patched.end(),
                     [](const std::pair<uint64_t, int32_t> &x, const std::pair<uint64_t, int32_t> &y) { return x.first < y.first; });
    bool one_launch = !p->tun.validate; // a checked call writes its patches first, so that the check sees them
    AppendRec *recs = (AppendRec *)(h + off_recs);
    for (uint32_t i = 0; i < n; ++i) {
        recs[i] = AppendRec{b->table_off[i], b->new_off[i], b->ctx_len[i], b->service_id[i], {-1, -1, -1, -1}};
        if (b->ctx_len[i] == 0 || patched.empty())
            continue;
        const uint64_t T = p->classes.c[b->service_id[i]].token_bytes;
        const uint64_t first = ((uint64_t)(b->ctx_len[i] - 1) * T) >> p->log2_page;
        const uint64_t last = ((uint64_t)b->ctx_len[i] * T - 1) >> p->log2_page;
        if (last - first >= 4)
            one_launch = false;
        for (uint64_t k = 0; k <= last - first && k < 4; ++k) {
            const uint64_t e = b->table_off[i] + first + k;
            // the last patch of an entry wins, as it would if the patches were applied in order
            auto it = std::upper_bound(patched.begin(), patched.end(), e,
                                       [](uint64_t v, const std::pair<uint64_t, int32_t> &x) { return v < x.first; });
            if (it != patched.begin() && (it - 1)->first == e)
                recs[i].page[k] = (it - 1)->second;
        }
    }
    if (b->n_patches) {
        std::memcpy(h + off_pe, b->patch_entry, (size_t)b->n_patches * sizeof(uint64_t));
        std::memcpy(h + off_pp, b->patch_page, (size_t)b->n_patches * sizeof(int32_t));
    }
    // the records are small: the kernels read them straight from the pinned, device-mapped slot
    unsigned char *d = (unsigned char *)st->mapped;
    uint32_t patches_in_append = b->n_patches;
    StageUse use{st, s};
    if (!one_launch) {
        HIP_TRY(launch_patch(b->page_table, (const uint64_t *)(d + off_pe), (const int32_t *)(d + off_pp),
                             b->n_patches, s),
                "launch patch kernel");
        use.launched = true;
        patches_in_append = 0;
    }
    const uint32_t *bad = nullptr;
    if ((rc = validate_tables(p, n, b->service_id, b->ctx_len, b->table_off, b->page_table, 0, s, &bad)) != UKV_OK)
        return rc;
    ProfPair pp{p, 2};
    if ((rc = pp.get()) != UKV_OK)
        return rc;
    HIP_TRY(launch_append(p->base, p->log2_page, b->page_table, (const AppendRec *)(d + off_recs), n,
                          (const ClassRec *)(d + off_cls), b->new_k, b->new_v, (const uint64_t *)(d + off_pe),
                          (const int32_t *)(d + off_pp), patches_in_append, bad, s, pp.ev.a, pp.ev.b),
            "launch append kernel");
    pp.done();
    use.launched = true;
    return use.done();
}

// n_last: null = whole requests; else only the n_last[i] last tokens of request i, which is then all
// that the contiguous arrays hold.
static int copy_tokens(bool to_pool, ukv_pool_t *p, const ukv_batch_t *b, const uint32_t *n_last, void *k_io,
                       void *v_io, const uint64_t *kv_off, void *stream) {
    Trace trace(!to_pool ? "ukv_gather" : n_last ? "ukv_scatter_tokens" : "ukv_scatter");
    if (b)
        trace.add("requests", b->n_requests);
    if (!p || !b || !k_io || !v_io || !kv_off || !b->page_table) {
        set_error("null argument");
        return UKV_EINVAL;
    }
    const uint32_t n = b->n_requests;
    if (n == 0)
        return UKV_OK;
    if (!b->service_id || !b->ctx_len || !b->table_off) {
        set_error("batch host arrays must be non-null");
        return UKV_EINVAL;
    }
    for (uint32_t i = 0; i < n; ++i) {
        if (b->service_id[i] >= p->n_services || (kv_off[i] & 7)) {
            set_error("service_id out of range or kv_off not a multiple of 8");
            return UKV_EINVAL;
        }
        if (ukv_pages_for_tokens(p, b->service_id[i], b->ctx_len[i]) > p->n_pages) {
            set_error("ctx_len exceeds what the pool can hold");
            return UKV_EINVAL;
        }
        if (n_last && n_last[i] > b->ctx_len[i]) {
            set_error("n_new exceeds ctx_len");
            return UKV_EINVAL;
        }
    }
    hipStream_t s = (hipStream_t)stream;
    int rc = report_bad_tables(p, s);
    if (rc != UKV_OK)
        return rc;
    // one record (= one workgroup) per chunk of about 1 MiB of a request's stream
    std::vector<GatherRec> &chunks = p->chunk_scratch; // storage reused from call to call
    chunks.clear();
    for (uint32_t i = 0; i < n; ++i) {
        const uint32_t T = p->classes.c[b->service_id[i]].token_bytes;
        const uint32_t step = std::max<uint32_t>(1, (1u << 20) / T);
        const uint32_t first = n_last ? b->ctx_len[i] - n_last[i] : 0;
        for (uint32_t t0 = first; t0 < b->ctx_len[i]; t0 += step)
            chunks.push_back(GatherRec{b->table_off[i], kv_off[i], t0, std::min(b->ctx_len[i], t0 + step),
                                       b->service_id[i], first});
    }
    if (chunks.empty())
        return UKV_OK;
    const size_t off_recs = align_up(sizeof(ClassTable));
    const size_t total = align_up(off_recs + chunks.size() * sizeof(GatherRec));
    const uint32_t *bad = nullptr;
    if ((rc = validate_tables(p, n, b->service_id, b->ctx_len, b->table_off, b->page_table, 0, s, &bad)) != UKV_OK)
        return rc;
    ukv_pool::Stage *st = nullptr;
    if ((rc = stage_acquire(p, total, &st)) != UKV_OK)
        return rc;
    trace.add("chunks", chunks.size());
    unsigned char *h = (unsigned char *)st->host;
    std::memcpy(h, &p->classes, sizeof(ClassTable));
    std::memcpy(h + off_recs, chunks.data(), chunks.size() * sizeof(GatherRec));
    unsigned char *d = (unsigned char *)st->mapped;
    HIP_TRY(launch_copy_tokens(to_pool, p->base, p->log2_page, b->page_table, (const GatherRec *)(d + off_recs),
                               (uint32_t)chunks.size(), (const ClassRec *)d, k_io, v_io, bad, s),
            "launch token copy kernel");
    return stage_release_after(st, s);
}

int ukv_gather(ukv_pool_t *p, const ukv_batch_t *b, void *k_out, void *v_out, const uint64_t *kv_off,
               void *stream) {
    return copy_tokens(false, p, b, nullptr, k_out, v_out, kv_off, stream);
}

int ukv_scatter(ukv_pool_t *p, const ukv_batch_t *b, const void *k_in, const void *v_in, const uint64_t *kv_off,
                void *stream) {
    return copy_tokens(true, p, b, nullptr, const_cast<void *>(k_in), const_cast<void *>(v_in), kv_off, stream);
}

int ukv_scatter_tokens(ukv_pool_t *p, const ukv_batch_t *b, const uint32_t *n_new, const void *k_in, const void *v_in,
                       const uint64_t *kv_off, void *stream) {
    if (!n_new) {
        set_error("n_new must be non-null");
        return UKV_EINVAL;
    }
    return copy_tokens(true, p, b, n_new, const_cast<void *>(k_in), const_cast<void *>(v_in), kv_off, stream);
}

// Prefill work list: one record per (request, kv head, tile of query rows), heaviest first.  Each XCD
// has its own L2 and consecutive workgroups go to consecutive XCDs, so the tiles of one (request, kv
// head) -- which read the same K/V -- are placed at launch positions of one residue modulo 8.
static constexpr uint32_t kXcds = 8;

static size_t prefill_rec_bound(const ukv_pool *p, uint32_t n_requests, uint64_t total_q_rows) {
    uint64_t max_kv = 1, max_g = 1;
    for (uint32_t s = 0; s < p->n_services; ++s) {
        max_kv = std::max<uint64_t>(max_kv, p->classes.c[s].n_kv);
        max_g = std::max<uint64_t>(max_g, prefill_group_columns(p->classes.c[s].g));
    }
    const uint64_t min_rows = std::max<uint64_t>(1, kPrefillCols / max_g);
    const uint64_t tiles = max_kv * (total_q_rows / min_rows + n_requests);
    return (size_t)(kXcds * (tiles + 1)); // the interleave pads every XCD's queue to the longest one
}

size_t ukv_prefill_workspace_bytes(const ukv_pool_t *p, uint32_t n_requests, uint64_t total_q_rows) {
    if (!p)
        return 0;
    return align_up(prefill_rec_bound(p, n_requests, total_q_rows) * sizeof(PrefillRec));
}

// One-part weights: the copy pass takes a request's tokens in chunks of about kV16ChunkBytes of V (all kv heads).
static constexpr uint64_t kV16ChunkBytes = 64 * 1024; // small enough that a few prompts already give every SIMD several waves
// One-part weights pay where a quarter of the kernel's time (its gain) exceeds one more launch with its gap (about
// 12 us) plus moving the fp16 copy (4 bytes per V element at about 4 TB/s): in flop of attention, at the kernel's rate,
static constexpr uint64_t kOnePartFlopFixed = 35000000000ull, kOnePartFlopPerByte = 1500;
static uint32_t v16_chunk_tokens(const ClassRec &c) {
    const uint64_t per_token = (uint64_t)c.n_kv * 2 * c.d;
    return (uint32_t)std::min<uint64_t>(4096, std::max<uint64_t>(8, kV16ChunkBytes / per_token));
}

size_t ukv_prefill_workspace_bytes_one_part(const ukv_pool_t *p, uint32_t n_requests, uint64_t total_q_rows,
                                            uint64_t total_ctx_tokens) {
    if (!p)
        return 0;
    uint64_t max_row = 1, min_chunk = 4096;
    for (uint32_t s = 0; s < p->n_services; ++s) {
        const ClassRec &c = p->classes.c[s];
        max_row = std::max<uint64_t>(max_row, (uint64_t)c.n_kv * 2 * c.d);
        min_chunk = std::min<uint64_t>(min_chunk, v16_chunk_tokens(c));
    }
    const uint64_t n_chunks = total_ctx_tokens / min_chunk + n_requests;
    // ... and room for the walks of few, long tiles to be cut into stretches: their records, merge list and partials
    const size_t split = align_up((size_t)kPrefillMaxParts * kXcds * sizeof(PrefillRec)) +
                         align_up((size_t)kPrefillMaxParts * sizeof(PrefillMergeRec)) +
                         align_up((size_t)kPrefillMaxParts * kPrefillPartFloats * sizeof(float));
    return ukv_prefill_workspace_bytes(p, n_requests, total_q_rows) + align_up((size_t)(n_chunks * sizeof(V16Rec))) +
           (size_t)(total_ctx_tokens * max_row) + 256 * (size_t)n_requests + split;
}

int ukv_prefill_attention(ukv_pool_t *p, const ukv_batch_t *b, const uint32_t *q_len, void *workspace,
                          size_t ws_bytes, void *stream) {
    Trace trace("ukv_prefill_attention");
    if (b)
        trace.add("requests", b->n_requests);
    if (!p || !b) {
        set_error("null pool or batch");
        return UKV_EINVAL;
    }
    const uint32_t n = b->n_requests;
    if (n == 0)
        return UKV_OK;
    if (!q_len || !b->service_id || !b->ctx_len || !b->table_off || !b->q_off || !b->out_off) {
        set_error("batch host arrays and q_len must be non-null");
        return UKV_EINVAL;
    }
    if (!b->page_table || !b->q || !b->out) {
        set_error("page_table, q and out must be non-null device pointers");
        return UKV_EINVAL;
    }
    if (!workspace || ((uintptr_t)workspace & 255)) {
        set_error("workspace must be non-null and 256-byte aligned");
        return UKV_EINVAL;
    }
    hipStream_t s = (hipStream_t)stream;
    int rc = report_bad_tables(p, s);
    if (rc != UKV_OK)
        return rc;
    struct Group {
        uint64_t cost;
        uint32_t req, kvh;
    };
    std::vector<Group> groups;
    uint64_t total_rows = 0;
    std::vector<uint64_t> v16_base(n, 0); // one-part weights: where request i's fp16 V rows start, relative to the copy's start
    uint64_t v16_bytes = 0, n_chunks = 0, flops = 0;
    for (uint32_t i = 0; i < n; ++i) {
        if (b->service_id[i] >= p->n_services) {
            set_error("service_id out of range");
            return UKV_EINVAL;
        }
        const ClassRec &c = p->classes.c[b->service_id[i]];
        if (q_len[i] > b->ctx_len[i]) {
            set_error("q_len exceeds ctx_len");
            return UKV_EINVAL;
        }
        if ((b->q_off[i] & 7) || (b->out_off[i] & 3)) {
            set_error("q_off must be a multiple of 8 elements and out_off of 4");
            return UKV_EINVAL;
        }
        if (ukv_pages_for_tokens(p, b->service_id[i], b->ctx_len[i]) > p->n_pages) {
            set_error("ctx_len exceeds what the pool can hold");
            return UKV_EINVAL;
        }
        if (q_len[i] == 0)
            continue;
        if ((c.d != 128 && c.d != 64) || c.g > 16) {
            set_error("prefill attention supports head_dim 128 or 64 with groups of up to 16 query heads");
            return UKV_EINVAL;
        }
        if (c.token_bytes >= (1u << 24)) { // the kernel's row offsets are products of 24-bit factors
            set_error("prefill attention supports token rows below 16 MiB");
            return UKV_EINVAL;
        }
        total_rows += q_len[i];
        // causal: row r looks at ctx_len - q_len + r + 1 tokens
        const uint64_t first = (uint64_t)b->ctx_len[i] - q_len[i] + 1, last = b->ctx_len[i];
        const uint64_t cost = (first + last) * q_len[i] / 2 * c.g;
        for (uint32_t h = 0; h < c.n_kv; ++h)
            groups.push_back(Group{cost, i, h});
        v16_base[i] = v16_bytes;
        v16_bytes += align_up((size_t)((uint64_t)b->ctx_len[i] * c.n_kv * 2 * c.d));
        n_chunks += ((uint64_t)b->ctx_len[i] + v16_chunk_tokens(c) - 1) / v16_chunk_tokens(c);
        flops += 4 * (uint64_t)c.d * c.n_kv * cost;
    }
    if (groups.empty())
        return UKV_OK;
    std::stable_sort(groups.begin(), groups.end(), [](const Group &x, const Group &y) { return x.cost > y.cost; });
    // One record list (= one launch) per head_dim.  Within a list: heaviest group first onto the least
    // loaded of the XCD queues, then the queues interleaved (padded with fillers to the longest).
    const uint32_t n_queues = p->tun.prefill_xcd ? kXcds : 1;
    static const uint32_t kDims[2] = {128, 64};
    // Few workgroups that each walk a long context (a chunk of one long prompt) leave most of the device idle and take
    // as long as the walk: where the longest walk is more than 5/4 of what an even spread over the resident
    // workgroups would give, the tiles' walks are cut into stretches of about that even share (at least 1024 tokens),
    // each a workgroup of its own that leaves a partial result, merged by a second launch.
    uint64_t total_walk = 0, longest_walk = 0; // in tokens, summed over every (request, kv head, tile of rows)
    for (const Group &g : groups) {
        const uint32_t i = g.req;
        const ClassRec &c = p->classes.c[b->service_id[i]];
        const uint32_t rows = kPrefillCols / prefill_group_columns(c.g);
        for (uint32_t r0 = 0; r0 < q_len[i]; r0 += rows) {
            const uint64_t walk = (uint64_t)b->ctx_len[i] - q_len[i] + std::min<uint32_t>(r0 + rows, q_len[i]);
            total_walk += walk;
            longest_walk = std::max(longest_walk, walk);
        }
    }
    static const int cus = decode_resident_workgroups(256); // asked once: the query costs as much as a small launch
    const uint64_t places = 2ull * (cus > 0 ? (uint64_t)cus : 256); // two workgroups of this kernel per compute unit
    uint32_t stretch = 0; // 0: every tile is walked by one workgroup
    if (4 * longest_walk > 5 * (total_walk / places) && longest_walk >= 2 * kPrefillMinStretch)
        stretch = (uint32_t)std::max<uint64_t>(kPrefillMinStretch, (total_walk / (2 * places) + 31) / 32 * 32);
    std::vector<PrefillRec> list[2];
    std::vector<PrefillMergeRec> merges;
    uint32_t n_parts = 0;
    size_t part_floats_total = 0;
    auto build_lists = [&](uint32_t stretch_tokens) {
    merges.clear();
    n_parts = 0;
    part_floats_total = 0;
    for (int di = 0; di < 2; ++di) {
        std::vector<std::vector<PrefillRec>> queue(n_queues);
        std::vector<uint64_t> load(n_queues, 0);
        for (const Group &g : groups) {
            const uint32_t i = g.req;
            const ClassRec &c = p->classes.c[b->service_id[i]];
            if (c.d != kDims[di])
                continue;
            const uint32_t k = (uint32_t)(std::min_element(load.begin(), load.end()) - load.begin());
            load[k] += g.cost;
            const uint32_t gl = prefill_group_columns(c.g);
            const uint32_t rows = kPrefillCols / gl;
            const uint32_t n_tiles = (q_len[i] + rows - 1) / rows;
            for (uint32_t t = n_tiles; t-- > 0;) { // the last rows look at the most tokens: they go first
                PrefillRec r{};
                r.table_off = b->table_off[i];
                r.q_off = b->q_off[i];
                r.out_off = b->out_off[i];
                r.ctx_len = b->ctx_len[i];
                r.q_len = q_len[i];
                r.kvh = g.kvh;
                r.v16_off = v16_base[i] + (uint64_t)g.kvh * b->ctx_len[i] * 2 * c.d; // made absolute below
                r.r0 = t * rows;
                r.g = c.g | (gl << 16);
                r.n_q = c.n_q;
                r.token_bytes = c.token_bytes;
                r.scale_log2e = c.scale_log2e;
                const uint32_t walk = b->ctx_len[i] - q_len[i] + std::min<uint32_t>(r.r0 + rows, q_len[i]);
                const uint32_t n_seg = stretch_tokens && walk > stretch_tokens + stretch_tokens / 2
                                           ? (walk + stretch_tokens - 1) / stretch_tokens : 1;
                if (n_seg == 1) {
                    r.t0 = 0;
                    r.t1 = walk;
                    r.part = kPrefillDirect;
                    queue[k].push_back(r);
                    continue;
                }
                const uint32_t seg = ((walk + n_seg - 1) / n_seg + 31) / 32 * 32; // stretches start at multiples of 32
                PrefillMergeRec m{};
                m.out_off = r.out_off;
                m.part0 = n_parts;
                m.q_len = r.q_len;
                m.r0 = r.r0;
                m.g = r.g;
                m.n_q = r.n_q;
                m.kvh = r.kvh;
                m.d = c.d;
                for (uint32_t t0 = 0; t0 < walk; t0 += seg) {
                    r.t0 = t0;
                    r.t1 = std::min(t0 + seg, walk);
                    r.part = n_parts++;
                    ++m.n_parts;
                    queue[k].push_back(r);
                }
                merges.push_back(m);
            }
        }
        size_t longest = 0;
        for (auto &qv : queue)
            longest = std::max(longest, qv.size());
        list[di].assign(longest * n_queues, PrefillRec{}); // q_len == 0: filler
        for (uint32_t k = 0; k < n_queues; ++k)
            for (size_t e = 0; e < queue[k].size(); ++e)
                list[di][e * n_queues + k] = queue[k][e];
    }
    part_floats_total = (size_t)n_parts * kPrefillPartFloats;
    };
    build_lists(stretch);
    auto fixed_bytes = [&]() { // records, merge list and partials: what the call needs whichever form the weights take
        return align_up((list[0].size() + list[1].size()) * sizeof(PrefillRec)) +
               align_up(merges.size() * sizeof(PrefillMergeRec)) + align_up(part_floats_total * sizeof(float));
    };
    if (stretch && (fixed_bytes() > ws_bytes || n_parts > kPrefillMaxParts)) {
        stretch = 0; // no room for the partial results: one workgroup per tile, as the smaller workspace size promises
        build_lists(0);
    }
    const size_t n_recs = list[0].size() + list[1].size();
    const size_t rec_bytes = align_up(n_recs * sizeof(PrefillRec)); // the records carry what they need of their class
    const size_t merge_bytes = align_up(merges.size() * sizeof(PrefillMergeRec));
    const size_t partial_bytes = align_up(part_floats_total * sizeof(float));
    if (rec_bytes > ws_bytes) {
        set_error("workspace too small for this batch");
        return UKV_ENOSPC;
    }
    // Form of the weights: one fp16 part needs the fp16 copy of V in the workspace, behind the records and the copy
    // pass's own work list.
    const size_t chunk_bytes = align_up((size_t)(n_chunks * sizeof(V16Rec)));
    const size_t one_part_total = rec_bytes + merge_bytes + chunk_bytes + (size_t)v16_bytes + partial_bytes;
    uint32_t parts = 2;
    if (p->tun.prefill_weights == 1) {
        if (one_part_total > ws_bytes) {
            set_error("workspace too small for one-part weights (see ukv_prefill_workspace_bytes_one_part)");
            return UKV_ENOSPC;
        }
        parts = 1;
    } else if (p->tun.prefill_weights == 0 && one_part_total <= ws_bytes && flops >= kOnePartFlopFixed + kOnePartFlopPerByte * v16_bytes) {
        parts = 1;
    }
    p->tun.prefill_form_used = parts;
    p->tun.prefill_partials_used = n_parts;
    trace.add("query_rows", total_rows);
    trace.add("workgroups", n_recs);
    trace.add("weight_parts", parts);
    trace.add("partial_results", n_parts);
    trace.add("flops", flops);
    const size_t total = rec_bytes + merge_bytes + (parts == 1 ? chunk_bytes : 0); // what is uploaded
    const size_t v16_start = total;
    const size_t partial_start = v16_start + (parts == 1 ? (size_t)v16_bytes : 0);
    ukv_pool::Stage *st = nullptr;
    if ((rc = stage_acquire(p, total, &st)) != UKV_OK)
        return rc;
    unsigned char *h = (unsigned char *)st->host;
    PrefillRec *recs = (PrefillRec *)h;
    if (!list[0].empty())
        std::memcpy(recs, list[0].data(), list[0].size() * sizeof(PrefillRec));
    if (!list[1].empty())
        std::memcpy(recs + list[0].size(), list[1].data(), list[1].size() * sizeof(PrefillRec));
    if (!merges.empty())
        std::memcpy(h + rec_bytes, merges.data(), merges.size() * sizeof(PrefillMergeRec));
    if (parts == 1) {
        for (size_t e = 0; e < n_recs; ++e)
            recs[e].v16_off += v16_start;
        V16Rec *ch = (V16Rec *)(h + rec_bytes + merge_bytes);
        size_t k = 0;
        for (uint32_t i = 0; i < n; ++i) {
            if (q_len[i] == 0)
                continue;
            const ClassRec &c = p->classes.c[b->service_id[i]];
            const uint32_t step = v16_chunk_tokens(c);
            for (uint64_t t0 = 0; t0 < b->ctx_len[i]; t0 += step) {
                V16Rec r{};
                r.table_off = b->table_off[i];
                r.v16_off = v16_start + v16_base[i];
                r.t0 = (uint32_t)t0;
                r.t1 = (uint32_t)std::min<uint64_t>(t0 + step, b->ctx_len[i]);
                r.ctx_len = b->ctx_len[i];
                r.token_bytes = c.token_bytes;
                r.n_kv = c.n_kv;
                r.d = c.d;
                ch[k++] = r;
            }
        }
    }
    HIP_TRY(launch_stage_copy(workspace, st->mapped, total, nullptr, nullptr, nullptr, 0, s), "launch plan upload");
    if ((rc = stage_release_after(st, s)) != UKV_OK)
        return rc;
    unsigned char *w = (unsigned char *)workspace;
    PrefillArgs a{};
    a.pool_base = p->base;
    a.log2_page = p->log2_page;
    a.page_table = b->page_table;
    a.q = (const uint16_t *)b->q;
    a.out = (float *)b->out;
    a.v16 = w;
    a.partials = (float *)(w + partial_start);
    if ((rc = validate_tables(p, n, b->service_id, b->ctx_len, b->table_off, b->page_table, 0, s, &a.bad)) != UKV_OK)
        return rc;
    if (parts == 1)
        HIP_TRY(launch_v16(p->base, p->log2_page, b->page_table, (const V16Rec *)(w + rec_bytes + merge_bytes),
                           (uint32_t)n_chunks, w, a.bad, s),
                "launch fp16 copy of V");
    size_t first = 0;
    for (int di = 0; di < 2; ++di) {
        if (list[di].empty())
            continue;
        a.recs = (const PrefillRec *)w + first;
        ProfPair pp{p, 3};
        if ((rc = pp.get()) != UKV_OK)
            return rc;
        HIP_TRY(launch_prefill(a, (uint32_t)list[di].size(), kDims[di], parts, s, pp.ev.a, pp.ev.b),
                "launch prefill kernel");
        pp.done();
        first += list[di].size();
    }
    HIP_TRY(launch_prefill_merge((const PrefillMergeRec *)(w + rec_bytes), (uint32_t)merges.size(), a.partials, a.out, a.bad,
                                 s),
            "launch merge of the prefill partials");
    (void)total_rows;
    return UKV_OK;
}

int ukv_profile_read(ukv_pool_t *p, ukv_profile_t *out) {
    if (!p || !out) {
        set_error("null argument");
        return UKV_EINVAL;
    }
    std::memset(out, 0, sizeof *out);
    for (auto &e : p->ev_used) {
        HIP_TRY(hipEventSynchronize(e.b), "hipEventSynchronize(profile)");
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, e.a, e.b), "hipEventElapsedTime");
        if (e.which == 0) {
            out->n_decode++;
            out->decode_ms += ms;
        } else if (e.which == 1) {
            out->n_reduce++;
            out->reduce_ms += ms;
        } else if (e.which == 2) {
            out->n_append++;
            out->append_ms += ms;
        } else {
            out->n_prefill++;
            out->prefill_ms += ms;
        }
        p->ev_free.push_back(e);
    }
    p->ev_used.clear();
    return UKV_OK;
}

} // extern "C"
