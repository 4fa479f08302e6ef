// Sanitizer driver for the host side of libukv (pool, planner, scheduler, argument checks and the staging of every
// compute call), linked against fake_hip_and_launchers.cpp.  Seeded pseudo-random scenarios; exits 0 when every call
// behaved as expected.  AddressSanitizer / UBSan report anything the host code reads or writes out of bounds.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "ukv.h"
#include "ukv_sched.h"

extern "C" void fake_device_set(uint64_t n_pages, uint32_t log2_page);
extern "C" void fake_device_counts(uint64_t *entries, uint64_t *items, uint64_t *appended);

static uint64_t g_state = 0x9E3779B97F4A7C15ull;
static uint64_t rnd() {
    g_state ^= g_state << 13;
    g_state ^= g_state >> 7;
    g_state ^= g_state << 17;
    return g_state;
}
static uint32_t rnd_below(uint32_t n) { return n ? (uint32_t)(rnd() % n) : 0; }

#define EXPECT(cond)                                                                                               \
    do {                                                                                                           \
        if (!(cond)) {                                                                                             \
            std::fprintf(stderr, "%s:%d: expectation failed: %s (last error: %s)\n", __FILE__, __LINE__, #cond,      \
                         ukv_last_error());                                                                        \
            std::exit(1);                                                                                          \
        }                                                                                                          \
    } while (0)

static const ukv_service_t kShapes[] = {{8, 8, 64, 0.f},   {12, 12, 64, 0.f}, {32, 32, 128, 0.f}, {40, 40, 128, 0.f},
                                        {32, 8, 128, 0.f}, {64, 8, 128, 0.f}, {16, 8, 128, 0.f},  {8, 4, 64, 0.125f}};

struct Scenario {
    ukv_pool_t *pool = nullptr;
    std::vector<ukv_service_t> services;
    uint32_t page_bytes = 0;
    uint64_t n_pages = 0;
    std::vector<uint32_t> sid, ctx;
    std::vector<uint64_t> table_off, cap, q_off, out_off, new_off;
    std::vector<int32_t> table; // "device" page table
    std::vector<uint64_t> T;
    void *base = nullptr, *dummy = nullptr, *ws = nullptr;
    size_t ws_bytes = 0;

    uint64_t pages_for(uint32_t i, uint64_t n) const { return (n * T[i] + page_bytes - 1) / page_bytes; }

    void make(uint32_t n_req, uint32_t max_ctx, uint32_t reserve) {
        const uint32_t n_sv = 1 + rnd_below(4);
        for (uint32_t s = 0; s < n_sv; ++s)
            services.push_back(kShapes[rnd_below(8)]);
        static const uint32_t kPages[] = {1024, 4096, 16384, 65536};
        page_bytes = kPages[rnd_below(4)];
        sid.resize(n_req), ctx.resize(n_req), table_off.resize(n_req), cap.resize(n_req), q_off.resize(n_req),
            out_off.resize(n_req), new_off.resize(n_req), T.resize(n_req);
        uint64_t entries = 0, rows = 0, need = 0;
        for (uint32_t i = 0; i < n_req; ++i) {
            sid[i] = rnd_below(n_sv);
            const ukv_service_t &sv = services[sid[i]];
            T[i] = 4ull * sv.head_dim * sv.n_kv_heads;
            ctx[i] = rnd_below(4) == 0 ? rnd_below(3) : rnd_below(max_ctx + 1);
            cap[i] = pages_for(i, (uint64_t)ctx[i] + reserve) + 1;
            table_off[i] = entries;
            entries += cap[i];
            q_off[i] = out_off[i] = new_off[i] = rows;
            rows += (uint64_t)sv.n_q_heads * sv.head_dim;
            need += cap[i];
        }
        n_pages = need + 7;
        base = std::aligned_alloc(page_bytes, page_bytes); // only its address is used
        dummy = std::malloc(64);
        ukv_pool_desc_t d{base, n_pages * page_bytes, page_bytes, n_sv, services.data()};
        EXPECT(ukv_pool_create(&d, &pool) == UKV_OK);
        uint32_t lg = 0;
        while ((1u << lg) < page_bytes)
            ++lg;
        fake_device_set(n_pages, lg);
        table.assign(entries, -1);
        for (uint32_t i = 0; i < n_req; ++i) {
            const uint64_t np = pages_for(i, ctx[i]);
            EXPECT(ukv_pages_for_tokens(pool, sid[i], ctx[i]) == np);
            if (np)
                EXPECT(ukv_pages_alloc(pool, (uint32_t)np, table.data() + table_off[i]) == UKV_OK);
        }
        resize_ws();
    }
    void resize_ws() {
        std::free(ws);
        ws_bytes = ukv_decode_workspace_bytes(pool, (uint32_t)sid.size());
        ws = std::aligned_alloc(256, (ws_bytes + 255) / 256 * 256);
    }
    ukv_batch_t batch() {
        ukv_batch_t b{};
        b.n_requests = (uint32_t)sid.size();
        b.service_id = sid.data();
        b.ctx_len = ctx.data();
        b.table_off = table_off.data();
        b.page_table = table.data();
        b.q = dummy, b.out = dummy, b.new_k = dummy, b.new_v = dummy;
        b.q_off = q_off.data(), b.out_off = out_off.data(), b.new_off = new_off.data();
        return b;
    }
    // grow every request by one token; the new entries' page ids in request order
    void grow(std::vector<uint64_t> &entry, std::vector<int32_t> &page) {
        entry.clear(), page.clear();
        for (uint32_t i = 0; i < sid.size(); ++i) {
            const uint64_t lo = pages_for(i, ctx[i]), hi = pages_for(i, (uint64_t)ctx[i] + 1);
            EXPECT(hi <= cap[i]);
            ++ctx[i];
            for (uint64_t e = lo; e < hi; ++e) {
                int32_t id = -1;
                EXPECT(ukv_pages_alloc(pool, 1, &id) == UKV_OK);
                entry.push_back(table_off[i] + e);
                page.push_back(id);
            }
        }
    }
    void destroy() {
        EXPECT(ukv_pool_destroy(pool) == UKV_OK);
        std::free(base), std::free(dummy), std::free(ws);
    }
};

static void run_scenario(uint32_t round) {
    Scenario sc;
    const uint32_t n_req = 1 + rnd_below(round % 7 == 0 ? 900 : 60);
    const uint32_t max_ctx = round % 5 == 0 ? 3000 : 300;
    sc.make(n_req, n_req > 200 ? 40 : max_ctx, 40);
    if (rnd_below(2))
        EXPECT(ukv_set_param(sc.pool, UKV_PARAM_BLOCK_THREADS, rnd_below(2) ? 256 : 512) == UKV_OK);
    if (rnd_below(2))
        EXPECT(ukv_set_param(sc.pool, UKV_PARAM_MIN_SPAN_BYTES, 1024 << rnd_below(10)) == UKV_OK);
    if (rnd_below(3) == 0)
        EXPECT(ukv_set_param(sc.pool, UKV_PARAM_MAX_SPANS, 1 + rnd_below(40)) == UKV_OK);
    if (rnd_below(3) == 0)
        EXPECT(ukv_set_param(sc.pool, UKV_PARAM_FUSED_MERGE, rnd_below(2)) == UKV_OK);
    if (rnd_below(4) == 0)
        EXPECT(ukv_set_param(sc.pool, UKV_PARAM_TAPER, rnd_below(2) ? 0 : 5 + rnd_below(90)) == UKV_OK);
    if (rnd_below(4) == 0)
        EXPECT(ukv_set_param(sc.pool, UKV_PARAM_PROFILE, 1 + rnd_below(3)) == UKV_OK);
    EXPECT(ukv_set_param(sc.pool, UKV_PARAM_REPLAN_EVERY, rnd_below(12)) == UKV_OK);
    EXPECT(ukv_set_param(sc.pool, UKV_PARAM_VALIDATE, rnd_below(2)) == UKV_OK);
    sc.resize_ws();

    ukv_batch_t b = sc.batch();
    ukv_plan_info_t info{};
    EXPECT(ukv_plan_decode(sc.pool, &b, &info, nullptr, 0) == UKV_OK);
    std::vector<uint32_t> items((size_t)info.n_items * 6 + 6);
    EXPECT(ukv_plan_decode(sc.pool, &b, &info, items.data(), info.n_items) == UKV_OK);
    EXPECT(ukv_decode_attention(sc.pool, &b, sc.ws, sc.ws_bytes, nullptr) == UKV_OK);
    EXPECT(ukv_decode_attention(sc.pool, &b, sc.ws, sc.ws_bytes / 2 > 256 ? 256 : 0, nullptr) != UKV_OK);

    std::vector<uint64_t> entry, kv_off(n_req);
    std::vector<int32_t> page;
    std::vector<uint32_t> q_len(n_req), n_new(n_req);
    for (int step = 0; step < 3; ++step) { // separate and fused steps, with the step's patches
        sc.grow(entry, page);
        b = sc.batch();
        b.n_patches = (uint32_t)entry.size();
        b.patch_entry = entry.data();
        b.patch_page = page.data();
        if (step == 1) {
            EXPECT(ukv_append(sc.pool, &b, nullptr) == UKV_OK);
            b.n_patches = 0;
            EXPECT(ukv_decode_attention(sc.pool, &b, sc.ws, sc.ws_bytes, nullptr) == UKV_OK);
        } else {
            EXPECT(ukv_decode_step(sc.pool, &b, sc.ws, sc.ws_bytes, nullptr) == UKV_OK);
        }
    }
    // bulk copies and prefill on the same batch
    uint64_t o = 0, rows = 0;
    for (uint32_t i = 0; i < n_req; ++i) {
        kv_off[i] = o;
        o += ((uint64_t)sc.ctx[i] * sc.T[i] / 4 + 7) / 8 * 8;
        q_len[i] = rnd_below(sc.ctx[i] + 1);
        n_new[i] = rnd_below(sc.ctx[i] + 1);
        rows += q_len[i];
    }
    b = sc.batch();
    EXPECT(ukv_gather(sc.pool, &b, sc.dummy, sc.dummy, kv_off.data(), nullptr) == UKV_OK);
    EXPECT(ukv_scatter(sc.pool, &b, sc.dummy, sc.dummy, kv_off.data(), nullptr) == UKV_OK);
    EXPECT(ukv_scatter_tokens(sc.pool, &b, n_new.data(), sc.dummy, sc.dummy, kv_off.data(), nullptr) == UKV_OK);
    const size_t pws = ukv_prefill_workspace_bytes(sc.pool, n_req, rows);
    void *pw = std::aligned_alloc(256, (pws + 255) / 256 * 256 + 256);
    EXPECT(ukv_prefill_attention(sc.pool, &b, q_len.data(), pw, pws, nullptr) == UKV_OK);
    // one-part weights: the fp16 copy of V lives in the workspace too
    EXPECT(ukv_set_param(sc.pool, UKV_PARAM_PREFILL_WEIGHTS, 1) == UKV_OK);
    {   // the two-part workspace is a bound, so a tiny batch's copy may fit it: either answer, nothing out of bounds
        const int r1 = ukv_prefill_attention(sc.pool, &b, q_len.data(), pw, pws, nullptr);
        EXPECT(r1 == UKV_OK || r1 == UKV_ENOSPC);
    }
    std::free(pw);
    uint64_t ctx_tokens = 0;
    for (uint32_t i = 0; i < n_req; ++i)
        ctx_tokens += q_len[i] ? sc.ctx[i] : 0;
    const size_t pws1 = ukv_prefill_workspace_bytes_one_part(sc.pool, n_req, rows, ctx_tokens);
    EXPECT(pws1 >= pws);
    pw = std::aligned_alloc(256, (pws1 + 255) / 256 * 256);
    EXPECT(ukv_prefill_attention(sc.pool, &b, q_len.data(), pw, pws1, nullptr) == UKV_OK);
    EXPECT(ukv_set_param(sc.pool, UKV_PARAM_PREFILL_WEIGHTS, 0) == UKV_OK);
    EXPECT(ukv_prefill_attention(sc.pool, &b, q_len.data(), pw, pws1, nullptr) == UKV_OK);
    EXPECT(ukv_set_param(sc.pool, UKV_PARAM_PREFILL_WEIGHTS, 3) == UKV_EINVAL);
    std::free(pw);

    // a plan kept across steps
    ukv_plan_t *plan = nullptr;
    EXPECT(ukv_plan_create(sc.pool, &b, sc.ws, sc.ws_bytes, &plan) == UKV_OK);
    std::vector<uint32_t> lens(n_req);
    for (int step = 0; step < 14; ++step) {
        sc.grow(entry, page);
        if (step == 5) { // a wrong count changes nothing
            page.push_back(0);
            EXPECT(ukv_plan_step(plan, nullptr, 1, page.data(), (uint32_t)page.size(), nullptr) == UKV_EINVAL);
            page.pop_back();
        }
        EXPECT(ukv_plan_step(plan, nullptr, 1, page.data(), (uint32_t)page.size(), nullptr) == UKV_OK);
        EXPECT(ukv_plan_lengths(plan, lens.data(), n_req) == UKV_OK);
        EXPECT(std::memcmp(lens.data(), sc.ctx.data(), n_req * sizeof(uint32_t)) == 0);
        if (step == 8)
            EXPECT(ukv_set_param(sc.pool, UKV_PARAM_MIN_SPAN_BYTES, 64 * 1024) == UKV_OK); // the plan is remade
    }
    EXPECT(ukv_plan_destroy(plan) == UKV_OK);
    ukv_profile_t prof{};
    EXPECT(ukv_profile_read(sc.pool, &prof) == UKV_OK);

    // pages go back; double frees and foreign ids are refused and change nothing
    for (uint32_t i = 0; i < n_req; ++i) {
        const uint64_t np = sc.pages_for(i, sc.ctx[i]);
        if (!np)
            continue;
        int32_t *ids = sc.table.data() + sc.table_off[i];
        EXPECT(ukv_pages_free(sc.pool, (uint32_t)np, ids) == UKV_OK);
        EXPECT(ukv_pages_free(sc.pool, 1, ids) == UKV_EINVAL);
    }
    int32_t bad = (int32_t)sc.n_pages;
    EXPECT(ukv_pages_free(sc.pool, 1, &bad) == UKV_EINVAL);
    ukv_service_info_t si{};
    EXPECT(ukv_pool_info(sc.pool, 0, &si) == UKV_OK && si.free_pages == sc.n_pages);
    sc.destroy();
}

static void bad_arguments() {
    ukv_pool_t *pool = nullptr;
    void *base = std::aligned_alloc(16384, 16384);
    ukv_service_t sv{32, 32, 128, 0.f};
    ukv_pool_desc_t d{base, 64 * 16384, 16384, 1, &sv};
    ukv_pool_desc_t bad = d;
    bad.page_bytes = 3000;
    EXPECT(ukv_pool_create(&bad, &pool) == UKV_EINVAL);
    bad = d, bad.base = (char *)base + 8;
    EXPECT(ukv_pool_create(&bad, &pool) == UKV_EINVAL);
    ukv_service_t odd{7, 3, 128, 0.f};
    bad = d, bad.services = &odd;
    EXPECT(ukv_pool_create(&bad, &pool) == UKV_EINVAL);
    ukv_service_t g17{68, 4, 128, 0.f}; // more query heads per kv head than a product has columns
    bad = d, bad.services = &g17;
    EXPECT(ukv_pool_create(&bad, &pool) == UKV_EINVAL);
    ukv_service_t g17d64{34, 2, 64, 0.f}; // the same at head_dim 64
    bad = d, bad.services = &g17d64;
    EXPECT(ukv_pool_create(&bad, &pool) == UKV_EINVAL);
    EXPECT(ukv_pool_create(&d, &pool) == UKV_OK);
    fake_device_set(64, 14);
    uint32_t sid = 0, ctx = 5;
    uint64_t zero = 0, odd_off = 3;
    int32_t table[8] = {0, 1, 2, 3, 4, 5, 6, 7};
    char dummy[64];
    ukv_batch_t b{};
    b.n_requests = 1, b.service_id = &sid, b.ctx_len = &ctx, b.table_off = &zero, b.page_table = table;
    b.q = dummy, b.out = dummy, b.q_off = &zero, b.out_off = &zero, b.new_k = dummy, b.new_v = dummy, b.new_off = &zero;
    const size_t wsb = ukv_decode_workspace_bytes(pool, 1);
    void *ws = std::aligned_alloc(256, (wsb + 255) / 256 * 256);
    EXPECT(ukv_decode_attention(nullptr, &b, ws, wsb, nullptr) == UKV_EINVAL);
    EXPECT(ukv_decode_attention(pool, &b, (char *)ws + 8, wsb, nullptr) == UKV_EINVAL);
    EXPECT(ukv_decode_attention(pool, &b, ws, 128, nullptr) == UKV_ENOSPC);
    b.q_off = &odd_off;
    EXPECT(ukv_decode_attention(pool, &b, ws, wsb, nullptr) == UKV_EINVAL);
    b.q_off = &zero;
    uint32_t bad_sid = 3, huge = 1000;
    b.service_id = &bad_sid;
    EXPECT(ukv_decode_attention(pool, &b, ws, wsb, nullptr) == UKV_EINVAL);
    EXPECT(ukv_append(pool, &b, nullptr) == UKV_EINVAL);
    b.service_id = &sid, b.ctx_len = &huge;
    EXPECT(ukv_decode_attention(pool, &b, ws, wsb, nullptr) == UKV_EINVAL);
    EXPECT(ukv_gather(pool, &b, dummy, dummy, &zero, nullptr) == UKV_EINVAL);
    b.ctx_len = &ctx;
    uint64_t pe = 2;
    int32_t pp = 64;
    b.n_patches = 1, b.patch_entry = &pe, b.patch_page = &pp;
    EXPECT(ukv_decode_step(pool, &b, ws, wsb, nullptr) == UKV_EINVAL);
    EXPECT(ukv_append(pool, &b, nullptr) == UKV_EINVAL);
    b.n_patches = 0;
    // the opt-in check: a table entry outside the pool stops the call's kernels and the next call says so
    EXPECT(ukv_set_param(pool, UKV_PARAM_VALIDATE, 1) == UKV_OK);
    EXPECT(ukv_decode_attention(pool, &b, ws, wsb, nullptr) == UKV_OK);
    table[1] = 64;
    EXPECT(ukv_decode_attention(pool, &b, ws, wsb, nullptr) == UKV_OK); // enqueued; its kernels leave at once
    EXPECT(ukv_gather(pool, &b, dummy, dummy, &zero, nullptr) == UKV_EINVAL);
    EXPECT(std::strstr(ukv_last_error(), "page id 64") != nullptr);
    table[1] = -3;
    EXPECT(ukv_append(pool, &b, nullptr) == UKV_OK);
    EXPECT(ukv_decode_attention(pool, &b, ws, wsb, nullptr) == UKV_EINVAL);
    table[1] = 1;
    EXPECT(ukv_decode_attention(pool, &b, ws, wsb, nullptr) == UKV_OK);
    EXPECT(ukv_decode_attention(pool, &b, ws, wsb, nullptr) == UKV_OK);
    EXPECT(ukv_set_param(pool, UKV_PARAM_VALIDATE, 0) == UKV_OK);
    uint32_t q_len = 9;
    EXPECT(ukv_prefill_attention(pool, &b, &q_len, ws, wsb, nullptr) == UKV_EINVAL);
    EXPECT(ukv_scatter_tokens(pool, &b, &q_len, dummy, dummy, &zero, nullptr) == UKV_EINVAL);
    ukv_plan_t *plan = nullptr;
    EXPECT(ukv_plan_create(pool, &b, ws, 64, &plan) == UKV_ENOSPC && plan == nullptr);
    EXPECT(ukv_set_param(pool, 99, 1) == UKV_EINVAL);
    EXPECT(ukv_set_param(pool, UKV_PARAM_BLOCK_THREADS, 300) == UKV_EINVAL);
    int64_t v = 0;
    EXPECT(ukv_get_param(pool, UKV_PARAM_TAPER, &v) == UKV_OK);
    EXPECT(std::strlen(ukv_strerror(UKV_ENOSPC)) > 0);
    std::free(ws);
    EXPECT(ukv_pool_destroy(pool) == UKV_OK);
    std::free(base);
}

// Chunks of long prompts: few tiles of query rows, each with a long walk, which the call cuts into stretches with
// partial results and a merge list (both forms of the weights, and a workspace without room for the partials).
static void long_context_chunks() {
    void *base = std::aligned_alloc(16384, 16384); // never dereferenced: the launchers are stand-ins
    ukv_service_t sv[2] = {{8, 8, 64, 0.f}, {28, 4, 128, 0.f}};
    const uint32_t n_pages = 4096;
    ukv_pool_desc_t d{base, (uint64_t)n_pages * 16384, 16384, 2, sv};
    ukv_pool_t *pool = nullptr;
    EXPECT(ukv_pool_create(&d, &pool) == UKV_OK);
    fake_device_set(n_pages, 14);
    const uint32_t n = 3;
    uint32_t sid[n] = {0, 1, 0}, ctx[n] = {6000, 9001, 70}, q_len[n] = {10, 300, 70};
    std::vector<int32_t> table(n_pages);
    for (uint32_t i = 0; i < n_pages; ++i)
        table[i] = (int32_t)(n_pages - 1 - i);
    uint64_t table_off[n] = {0, 1000, 3500}, q_off[n] = {0, 8192, 1 << 22}, out_off[n] = {0, 8192, 1 << 22};
    ukv_batch_t b{};
    b.n_requests = n;
    b.service_id = sid;
    b.ctx_len = ctx;
    b.table_off = table_off;
    b.page_table = table.data();
    b.q = base;
    b.q_off = q_off;
    b.out = base;
    b.out_off = out_off;
    const uint64_t rows = 10 + 300 + 70, toks = 6000 + 9001 + 70;
    const size_t small = ukv_prefill_workspace_bytes(pool, n, rows);
    const size_t full = ukv_prefill_workspace_bytes_one_part(pool, n, rows, toks);
    void *ws = std::aligned_alloc(256, (full + 255) / 256 * 256);
    int64_t form = 0;
    for (int64_t w = 0; w <= 2; ++w) {
        EXPECT(ukv_set_param(pool, UKV_PARAM_PREFILL_WEIGHTS, w) == UKV_OK);
        EXPECT(ukv_prefill_attention(pool, &b, q_len, ws, full, nullptr) == UKV_OK);
        EXPECT(ukv_get_param(pool, UKV_PARAM_PREFILL_FORM_USED, &form) == UKV_OK && (w == 0 || form == w));
        EXPECT(ukv_get_param(pool, UKV_PARAM_PREFILL_PARTIALS_USED, &form) == UKV_OK && form > 8);
    }
    EXPECT(ukv_prefill_attention(pool, &b, q_len, ws, small, nullptr) == UKV_OK); // no room: one workgroup per tile
    EXPECT(ukv_get_param(pool, UKV_PARAM_PREFILL_PARTIALS_USED, &form) == UKV_OK && form == 0);
    std::free(ws);
    EXPECT(ukv_pool_destroy(pool) == UKV_OK);
    std::free(base);
}

static void scheduler_trace(uint32_t round) {
    void *base = std::aligned_alloc(16384, 16384);
    ukv_service_t sv[3] = {{32, 32, 128, 0.f}, {40, 40, 128, 0.f}, {32, 8, 128, 0.f}};
    ukv_pool_desc_t d{base, 4096ull * 16384, 16384, 3, sv};
    ukv_pool_t *pool = nullptr;
    EXPECT(ukv_pool_create(&d, &pool) == UKV_OK);
    ukv_sched_service_t prof[3] = {{1e-3, 2e-4, 4e-3}, {3e-3, 1e-3, 6e-3}, {2e-3, 0.0, 1e30}};
    ukv_sched_t *s = nullptr;
    const uint32_t max_batch = 1 + rnd_below(8);
    EXPECT(ukv_sched_create(pool, prof, 3, max_batch, &s) == UKV_OK);
    ukv_sched_t *refused = nullptr;
    EXPECT(ukv_sched_create(pool, prof, 2, max_batch, &refused) == UKV_EINVAL && refused == nullptr);
    struct Req {
        uint32_t left;
    };
    std::vector<Req> reqs;
    double now = 0.0;
    uint64_t next_id = 0, free_pages = 600 + rnd_below(3000);
    std::vector<uint64_t> ids(max_batch + 2);
    std::vector<uint8_t> fin(max_batch + 2);
    for (int it = 0; it < 400 + (int)(round % 3) * 300; ++it) {
        if (reqs.size() < 40 && rnd_below(3) == 0) {
            EXPECT(ukv_sched_add_request(s, next_id, rnd_below(3), 1 + rnd_below(700), now) == UKV_OK);
            EXPECT(ukv_sched_add_request(s, next_id, 0, 5, now) == UKV_EINVAL); // id in use
            reqs.push_back(Req{2 + rnd_below(30)});
            ++next_id;
        }
        uint32_t n = 0, svc = 0, queue = 0;
        EXPECT(ukv_sched_next_batch(s, now, free_pages, ids.data(), max_batch, &n, &svc, &queue) == UKV_OK);
        EXPECT(n <= max_batch);
        const double elapsed = 1e-5 * (1 + rnd_below(50));
        now += elapsed;
        for (uint32_t k = 0; k < n; ++k) {
            uint64_t pages = 0;
            EXPECT(ukv_sched_pages_needed(s, ids[k], &pages) == UKV_OK);
            ukv_sched_request_t info{};
            EXPECT(ukv_sched_request_info(s, ids[k], &info) == UKV_OK && info.service == svc && info.queue == queue);
            fin[k] = queue == UKV_SCHED_DECODING && --reqs[ids[k]].left == 0;
        }
        if (n)
            EXPECT(ukv_sched_complete(s, ids.data(), fin.data(), n, elapsed, now) == UKV_OK);
        free_pages = 200 + rnd_below(3000);
    }
    uint64_t none = 0;
    EXPECT(ukv_sched_pages_needed(s, next_id + 5, &none) == UKV_EINVAL);
    EXPECT(ukv_sched_destroy(s) == UKV_OK);
    EXPECT(ukv_pool_destroy(pool) == UKV_OK);
    std::free(base);
}

int main(int argc, char **argv) {
    const int rounds = argc > 1 ? std::atoi(argv[1]) : 40;
    bad_arguments();
    long_context_chunks();
    for (int r = 0; r < rounds; ++r)
        run_scenario((uint32_t)r);
    for (int r = 0; r < 6; ++r)
        scheduler_trace((uint32_t)r);
    uint64_t entries = 0, items = 0, appended = 0;
    fake_device_counts(&entries, &items, &appended);
    std::printf("host driver ok: %d scenarios, %llu work items walked, %llu table entries checked, %llu fused appends\n",
                rounds, (unsigned long long)items, (unsigned long long)entries, (unsigned long long)appended);
    return 0;
}
