// Unified block manager: pool validation, per-service derived constants, LIFO free list.
// (Section 4.4 "Unified KV Cache" and the unified block manager of section 5.)  Host only.
#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>

#include "ukv_internal.h"

namespace ukv {

static thread_local std::string g_last_error;

static thread_local uint64_t g_errors = 0; // set_error calls of this thread (a traced call compares before and after)

void set_error(const std::string &msg) {
    g_last_error = msg;
    ++g_errors;
}

static uint64_t now_ns() {
    return (uint64_t)std::chrono::duration_cast<std::chrono::nanoseconds>(
               std::chrono::steady_clock::now().time_since_epoch())
        .count();
}
static bool trace_enabled() {
    static const bool on = [] {
        const char *e = std::getenv("UKV_TRACE");
        return e != nullptr && e[0] != '\0' && e[0] != '0';
    }();
    return on;
}
Trace::Trace(const char *call) : call_(call), on_(trace_enabled()), t0_ns_(0), errors_at_start_(g_errors) {
    kv_[0] = '\0';
    if (on_)
        t0_ns_ = now_ns();
}
void Trace::add(const char *key, uint64_t value) {
    if (!on_ || len_ >= sizeof(kv_) - 1)
        return;
    const int w = std::snprintf(kv_ + len_, sizeof(kv_) - len_, " %s=%llu", key, (unsigned long long)value);
    if (w > 0)
        len_ = std::min(sizeof(kv_) - 1, len_ + (size_t)w);
}
Trace::~Trace() {
    if (!on_)
        return;
    static const uint64_t first_ns = t0_ns_; // the first traced call of the process
    const uint64_t t1 = now_ns();
    std::fprintf(stderr, "ukv_trace call=%s t_us=%.1f host_us=%.1f status=%s%s\n", call_, (t0_ns_ - first_ns) * 1e-3,
                 (t1 - t0_ns_) * 1e-3, g_errors == errors_at_start_ ? "ok" : "error", kv_);
}

static int fail(int code, const std::string &msg) {
    set_error(msg);
    return code;
}

// Choose how a workgroup of `block_threads` lanes covers a service's token rows.
// A row (one kv head of one token) is read by head_dim/8 lanes, 16 bytes each, so a workgroup
// has NG = block_threads / (head_dim/8) row groups: hs kv heads times ti tokens per iteration.
// Among the divisors of n_kv_heads that keep (nearly) all groups busy, take the slice closest
// to 4 KiB of contiguous stream per token: wide enough for full-line streaming reads, narrow
// enough that a request splits into several independent sequences whose partial results are
// small and are merged by different workgroups.
static void choose_slicing(uint32_t n_kv, uint32_t d, uint32_t block_threads, int64_t forced, uint32_t *hs_out,
                           uint32_t *ti_out) {
    const uint32_t ng = block_threads / (d / 8);
    if (forced > 0 && forced <= (int64_t)ng && n_kv % (uint32_t)forced == 0) {
        *hs_out = (uint32_t)forced;
        *ti_out = ng / (uint32_t)forced;
        return;
    }
    const double want = 4096.0 / (4.0 * d); // heads per 4 KiB
    uint32_t best_hs = 1;
    double best_util = -1.0, best_dist = 0.0;
    for (uint32_t hs = 1; hs <= n_kv && hs <= ng; ++hs) {
        if (n_kv % hs)
            continue;
        double util = (double)(hs * (ng / hs)) / ng;
        if (util > 0.9)
            util = 1.0;
        const double dist = std::fabs(std::log((double)hs / want));
        if (util > best_util + 1e-9 || (std::fabs(util - best_util) < 1e-9 && dist < best_dist - 1e-9) ||
            (std::fabs(util - best_util) < 1e-9 && std::fabs(dist - best_dist) < 1e-9 && hs > best_hs)) {
            best_util = util;
            best_dist = dist;
            best_hs = hs;
        }
    }
    *hs_out = best_hs;
    *ti_out = ng / best_hs;
}

int derive_classes(ukv_pool *p) {
    p->kinds = 0;
    for (uint32_t s = 0; s < p->n_services; ++s) {
        const ukv_service_t &sv = p->services[s];
        ClassRec &c = p->classes.c[s];
        c.n_q = sv.n_q_heads;
        c.n_kv = sv.n_kv_heads;
        c.d = sv.head_dim;
        c.g = sv.n_q_heads / sv.n_kv_heads;
        c.row_bytes = 4 * sv.head_dim;
        c.token_bytes = c.row_bytes * sv.n_kv_heads;
        const double scale = sv.scale != 0.0f ? (double)sv.scale : 1.0 / std::sqrt((double)sv.head_dim);
        c.scale_log2e = (float)(scale * 1.4426950408889634);
        if (c.d == 128 && c.g >= 1 && c.g <= 16) // the matrix-core path pads a group to the 16 columns of a product
            c.kind = c.g == 1 ? kD128G1 : kD128GQA;
        else if (c.d == 64 && c.g >= 1 && c.g <= 16)
            c.kind = c.g == 1 ? kD64G1 : c.g == 2 ? kD64G2 : kD64GQA;
        else
            return fail(UKV_EINVAL, "unsupported shape: head_dim 128 or 64 with groups of 1 to 16 query heads");
        p->kinds |= 1u << c.kind;
        if (kind_is_gqa(c.kind)) {
            // matrix-core path: one wave per kv head of the slice, all waves on the same tokens
            const uint32_t waves = (uint32_t)p->tun.block_threads / 64;
            uint32_t hs = 1;
            for (uint32_t h = 1; h <= c.n_kv && h <= waves; ++h)
                if (c.n_kv % h == 0)
                    hs = h;
            c.hs = hs;
            c.ti = 1;
            continue;
        }
        choose_slicing(c.n_kv, c.d, (uint32_t)p->tun.block_threads, p->tun.heads_per_slice, &c.hs, &c.ti);
    }
    return UKV_OK;
}

} // namespace ukv

using namespace ukv;

extern "C" {

int ukv_pool_create(const ukv_pool_desc_t *desc, ukv_pool_t **out) {
    if (!desc || !out)
        return fail(UKV_EINVAL, "null argument");
    *out = nullptr;
    const uint32_t P = desc->page_bytes;
    // Upper bound: the kernels address a page-table window (at most 2048 pages) with 32-bit offsets.
    if (P < 1024 || P > (1u << 20) || (P & (P - 1)) != 0)
        return fail(UKV_EINVAL, "page_bytes must be a power of two in [1 KiB, 1 MiB]");
    if (!desc->base || ((uintptr_t)desc->base % P) != 0)
        return fail(UKV_EINVAL, "pool base must be non-null and page_bytes-aligned");
    if (desc->bytes / P == 0 || desc->bytes / P > 0x7fffffffull)
        return fail(UKV_EINVAL, "pool must hold between 1 and 2^31-1 pages");
    if (desc->n_services == 0 || desc->n_services > UKV_MAX_SERVICES || !desc->services)
        return fail(UKV_EINVAL, "n_services must be in [1, UKV_MAX_SERVICES]");
    for (uint32_t s = 0; s < desc->n_services; ++s) {
        const ukv_service_t &sv = desc->services[s];
        if (sv.n_kv_heads == 0 || sv.n_q_heads == 0 || sv.n_q_heads % sv.n_kv_heads != 0)
            return fail(UKV_EINVAL, "n_q_heads must be a positive multiple of n_kv_heads");
        if (sv.head_dim == 0 || P % (4 * sv.head_dim) != 0)
            return fail(UKV_EINVAL, "page_bytes must be a multiple of 4*head_dim (head-rows may not straddle pages)");
        if (!(sv.scale >= 0.0f) || !std::isfinite(sv.scale))
            return fail(UKV_EINVAL, "scale must be finite and >= 0");
    }
    ukv_pool *p = new (std::nothrow) ukv_pool();
    if (!p)
        return fail(UKV_ENOMEM, "host allocation failed");
    p->base = (unsigned char *)desc->base;
    p->page_bytes = P;
    p->log2_page = (uint32_t)__builtin_ctz(P);
    p->n_pages = desc->bytes / P;
    p->n_services = desc->n_services;
    std::memcpy(p->services, desc->services, sizeof(ukv_service_t) * desc->n_services);
    std::memset(&p->classes, 0, sizeof p->classes);
    int rc = derive_classes(p);
    if (rc == UKV_OK) {
        // A pool whose services all run on the matrix-core path does better with four waves (four
        // kv heads) per workgroup: smaller partials.  Its partials
        // are G times larger than those of the other kinds, and merging them in a second launch was
        // measured faster than inside the decode launch (2 % of the step on the GQA workload).  Two such
        // workgroups fit a compute unit, but one streams as fast as two, and a second one only uses up the later
        // rounds' small spans at the start of the launch: one workgroup per first-round span, and a larger
        // first round (94 % of the work: with single-kind batches the later rounds have less to even out).
        bool all_gqa = true;
        for (uint32_t s = 0; s < p->n_services; ++s)
            all_gqa = all_gqa && p->classes.c[s].kind == kD128GQA; // (the measured default: pools of the workloads' GQA shape)
        if (all_gqa) {
            p->tun.block_threads = 256;
            p->tun.fused_merge = 0;
            p->tun.grid_is_first_round = true;
            p->tun.taper = 94;
            rc = derive_classes(p);
        }
    }
    if (rc != UKV_OK) {
        delete p;
        return rc;
    }
    p->free_stack.resize(p->n_pages);
    for (uint64_t i = 0; i < p->n_pages; ++i)
        p->free_stack[i] = (int32_t)(p->n_pages - 1 - i); // top of stack (back) is page 0
    p->is_free.assign(p->n_pages, 1);
    *out = p;
    return UKV_OK;
}

int ukv_pool_destroy(ukv_pool_t *p) {
    if (!p)
        return UKV_OK;
    int rc = UKV_OK;
    for (auto &st : p->stage) {
        if (st.pending && st.ev)
            (void)hipEventSynchronize(st.ev);
        if (st.ev && hipEventDestroy(st.ev) != hipSuccess)
            rc = UKV_EHIP;
        if (st.host && hipHostFree(st.host) != hipSuccess)
            rc = UKV_EHIP;
    }
    if (p->val_host && hipHostFree(p->val_host) != hipSuccess)
        rc = UKV_EHIP;
    if (p->val_flag && hipFree(p->val_flag) != hipSuccess)
        rc = UKV_EHIP;
    for (auto *v : {&p->ev_used, &p->ev_free})
        for (auto &e : *v) {
            (void)hipEventDestroy(e.a);
            (void)hipEventDestroy(e.b);
        }
    delete p;
    return rc;
}

int ukv_pool_info(const ukv_pool_t *p, uint32_t service, ukv_service_info_t *out) {
    if (!p || !out || service >= p->n_services)
        return fail(UKV_EINVAL, "bad pool, service or output");
    const ClassRec &c = p->classes.c[service];
    out->n_q_heads = c.n_q;
    out->n_kv_heads = c.n_kv;
    out->head_dim = c.d;
    out->group = c.g;
    out->head_row_bytes = c.row_bytes;
    out->token_bytes = c.token_bytes;
    out->scale = p->services[service].scale != 0.0f ? p->services[service].scale
                                                    : (float)(1.0 / std::sqrt((double)c.d));
    out->heads_per_slice = c.hs;
    out->n_slices = c.n_kv / c.hs;
    out->token_lanes = c.ti;
    out->n_pages = p->n_pages;
    out->free_pages = p->free_stack.size();
    return UKV_OK;
}

uint64_t ukv_pages_for_tokens(const ukv_pool_t *p, uint32_t service, uint64_t n_tokens) {
    if (!p || service >= p->n_services)
        return 0;
    const uint64_t T = p->classes.c[service].token_bytes;
    if (n_tokens > (UINT64_MAX - p->page_bytes) / T)
        return 0;
    return (n_tokens * T + p->page_bytes - 1) >> p->log2_page;
}

int ukv_pages_alloc(ukv_pool_t *p, uint32_t n, int32_t *out_ids) {
    if (!p || (n && !out_ids))
        return fail(UKV_EINVAL, "null argument");
    if (n > p->free_stack.size())
        return fail(UKV_ENOMEM, "free list exhausted");
    for (uint32_t i = 0; i < n; ++i) {
        const int32_t id = p->free_stack.back();
        p->free_stack.pop_back();
        p->is_free[id] = 0;
        out_ids[i] = id;
    }
    return UKV_OK;
}

int ukv_pages_free(ukv_pool_t *p, uint32_t n, const int32_t *ids) {
    if (!p || (n && !ids))
        return fail(UKV_EINVAL, "null argument");
    for (uint32_t i = 0; i < n; ++i) {
        const int64_t id = ids[i];
        bool bad = id < 0 || (uint64_t)id >= p->n_pages || p->is_free[id];
        if (!bad) {
            p->is_free[id] = 2; // provisional: also catches a duplicate inside this call
        }
        if (bad) {
            for (uint32_t j = 0; j < i; ++j)
                p->is_free[ids[j]] = 0;
            return fail(UKV_EINVAL, "page id out of range or already free");
        }
    }
    for (uint32_t i = 0; i < n; ++i) {
        p->is_free[ids[i]] = 1;
        p->free_stack.push_back(ids[i]);
    }
    return UKV_OK;
}

int ukv_set_param(ukv_pool_t *p, int key, int64_t value) {
    if (!p)
        return fail(UKV_EINVAL, "null pool");
    if (key != UKV_PARAM_PROFILE && key != UKV_PARAM_VALIDATE && key != UKV_PARAM_PREFILL_WEIGHTS)
        ++p->tun_epoch; // kept plans are remade
    switch (key) {
    case UKV_PARAM_MERGE_ACQ_REL:
        p->tun.merge_acq_rel = value ? 1 : 0;
        return UKV_OK;
    case UKV_PARAM_VALIDATE:
        p->tun.validate = value ? 1 : 0;
        return UKV_OK;
    case UKV_PARAM_PREFILL_WEIGHTS:
        if (value < 0 || value > 2)
            return fail(UKV_EINVAL, "prefill_weights must be 0, 1 or 2");
        p->tun.prefill_weights = value;
        return UKV_OK;
    case UKV_PARAM_REPLAN_EVERY:
        if (value < 0 || value > (1 << 20))
            return fail(UKV_EINVAL, "replan_every out of range");
        p->tun.replan_every = value;
        return UKV_OK;
    case UKV_PARAM_MAX_SPANS:
        if (value < 1 || value > (1 << 20))
            return fail(UKV_EINVAL, "max_spans out of range");
        p->tun.max_spans = value;
        return UKV_OK;
    case UKV_PARAM_MIN_SPAN_BYTES:
        if (value < 1)
            return fail(UKV_EINVAL, "min_span_bytes must be positive");
        p->tun.min_span_bytes = value;
        p->tun.min_span_auto = false;
        return UKV_OK;
    case UKV_PARAM_BLOCK_THREADS:
        if (value != 256 && value != 512)
            return fail(UKV_EINVAL, "block_threads must be 256 or 512");
        p->tun.block_threads = value;
        p->tun.slots_auto = true;
        return derive_classes(p);
    case UKV_PARAM_HEADS_PER_SLICE:
        if (value < 0)
            return fail(UKV_EINVAL, "heads_per_slice must be >= 0");
        p->tun.heads_per_slice = value;
        return derive_classes(p);
    case UKV_PARAM_PROFILE:
        if (value < 0 || value > 1024)
            return fail(UKV_EINVAL, "profile must be 0 (off) or a stride in [1, 1024]");
        p->tun.profile = value;
        return UKV_OK;
    case UKV_PARAM_FUSED_MERGE:
        p->tun.fused_merge = value ? 1 : 0;
        return UKV_OK;
    case UKV_PARAM_SLOTS:
        if (value < 0 || value > (1 << 20))
            return fail(UKV_EINVAL, "slots out of range");
        p->tun.slots_auto = value == 0;
        if (value > 0)
            p->tun.slots = value;
        return UKV_OK;
    case UKV_PARAM_GQA_COST_PCT:
        if (value < 50 || value > 400)
            return fail(UKV_EINVAL, "gqa_cost_pct must lie in 50..400");
        p->tun.gqa_cost_pct = value;
        return UKV_OK;
    case UKV_PARAM_PREFILL_XCD:
        p->tun.prefill_xcd = value ? 1 : 0;
        return UKV_OK;
    case UKV_PARAM_TAPER:
        if (value < 0 || value > 95 || (value > 1 && value < 5))
            return fail(UKV_EINVAL, "taper must be 0, 1 or a percentage in 5..95");
        p->tun.taper = value;
        return UKV_OK;
    default:
        return fail(UKV_EINVAL, "unknown parameter");
    }
}

int ukv_get_param(const ukv_pool_t *p, int key, int64_t *value) {
    if (!p || !value)
        return fail(UKV_EINVAL, "null argument");
    switch (key) {
    case UKV_PARAM_MAX_SPANS: *value = p->tun.max_spans; return UKV_OK;
    case UKV_PARAM_MIN_SPAN_BYTES: *value = p->tun.min_span_bytes; return UKV_OK;
    case UKV_PARAM_BLOCK_THREADS: *value = p->tun.block_threads; return UKV_OK;
    case UKV_PARAM_HEADS_PER_SLICE: *value = p->tun.heads_per_slice; return UKV_OK;
    case UKV_PARAM_PROFILE: *value = p->tun.profile; return UKV_OK;
    case UKV_PARAM_FUSED_MERGE: *value = p->tun.fused_merge; return UKV_OK;
    case UKV_PARAM_SLOTS: *value = p->tun.slots; return UKV_OK;
    case UKV_PARAM_TAPER: *value = p->tun.taper; return UKV_OK;
    case UKV_PARAM_GQA_COST_PCT: *value = p->tun.gqa_cost_pct; return UKV_OK;
    case UKV_PARAM_PREFILL_XCD: *value = p->tun.prefill_xcd; return UKV_OK;
    case UKV_PARAM_REPLAN_EVERY: *value = p->tun.replan_every; return UKV_OK;
    case UKV_PARAM_MERGE_ACQ_REL: *value = p->tun.merge_acq_rel; return UKV_OK;
    case UKV_PARAM_VALIDATE: *value = p->tun.validate; return UKV_OK;
    case UKV_PARAM_PREFILL_WEIGHTS: *value = p->tun.prefill_weights; return UKV_OK;
    case UKV_PARAM_PREFILL_FORM_USED: *value = p->tun.prefill_form_used; return UKV_OK;
    case UKV_PARAM_PREFILL_PARTIALS_USED: *value = p->tun.prefill_partials_used; return UKV_OK;
    default: return fail(UKV_EINVAL, "unknown parameter");
    }
}

const char *ukv_strerror(int code) {
    switch (code) {
    case UKV_OK: return "ok";
    case UKV_EINVAL: return "invalid argument";
    case UKV_ENOMEM: return "out of pages or host memory";
    case UKV_ENOSPC: return "workspace too small";
    case UKV_EHIP: return "HIP runtime error";
    default: return "unknown error";
    }
}

const char *ukv_last_error(void) { return g_last_error.c_str(); }

} // extern "C"
