// Host-only stand-ins for the HIP runtime calls and the kernel launchers that libukv's host code uses, for the
// sanitizer build (tests/test_sanitize.py): "device" memory is ordinary host memory, a launch runs a plain C++ walk
// over what the kernel would read and write, so that AddressSanitizer / UBSan see every byte the host code prepared
// (plan blobs, staging slots, record lists, page-table patches) being consumed within the bounds the caller gave.
// No arithmetic of the method is done here: the walks touch tables and records, not K/V.
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "ukv_internal.h"

using namespace ukv;

extern "C" {
hipError_t hipHostMalloc(void **p, size_t n, unsigned) {
    *p = std::malloc(n ? n : 1);
    return *p ? hipSuccess : hipErrorOutOfMemory;
}
hipError_t hipHostFree(void *p) {
    std::free(p);
    return hipSuccess;
}
hipError_t hipHostGetDevicePointer(void **d, void *h, unsigned) {
    *d = h;
    return hipSuccess;
}
hipError_t hipEventCreate(hipEvent_t *e) {
    *e = (hipEvent_t)std::malloc(8);
    return hipSuccess;
}
hipError_t hipEventCreateWithFlags(hipEvent_t *e, unsigned) { return hipEventCreate(e); }
hipError_t hipEventDestroy(hipEvent_t e) {
    std::free((void *)e);
    return hipSuccess;
}
hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
hipError_t hipEventElapsedTime(float *ms, hipEvent_t, hipEvent_t) {
    *ms = 0.25f;
    return hipSuccess;
}
hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
hipError_t hipMalloc(void **p, size_t n) {
    *p = std::malloc(n ? n : 1);
    return *p ? hipSuccess : hipErrorOutOfMemory;
}
hipError_t hipFree(void *p) {
    std::free(p);
    return hipSuccess;
}
hipError_t hipMemsetAsync(void *p, int v, size_t n, hipStream_t) {
    std::memset(p, v, n);
    return hipSuccess;
}
const char *hipGetErrorString(hipError_t) { return "fake hip error"; }
}

// What the driver tells the walks about the caller's buffers (set before each call).
struct FakeDevice {
    uint64_t n_pages = 0;
    uint32_t log2_page = 0;
    uint64_t checked_entries = 0, items = 0, appended = 0;
} g_fake;

static void die(const char *what) {
    std::fprintf(stderr, "fake launch: %s\n", what);
    std::abort();
}

namespace ukv {

int decode_resident_workgroups(uint32_t) { return 256; }
uint32_t decode_grid(uint32_t n_spans, uint32_t, uint32_t, uint32_t) { return n_spans < 256 ? n_spans : 256; }

hipError_t launch_stage_copy(void *dst, const void *src, size_t bytes, int32_t *page_table, const uint64_t *pe,
                             const int32_t *pp, uint32_t n_patches, hipStream_t) {
    std::memcpy(dst, src, (bytes + 15) / 16 * 16); // the kernel moves whole 16-byte pieces
    for (uint32_t i = 0; i < n_patches; ++i)
        page_table[pe[i]] = pp[i];
    return hipSuccess;
}

hipError_t launch_validate(const int32_t *page_table, const ValRec *recs, uint32_t n, uint64_t n_pages,
                           ValReport *report, uint32_t *flag_dev, hipStream_t) {
    for (uint32_t i = 0; i < n; ++i)
        for (uint64_t e = 0; e < recs[i].n_entries; ++e) {
            const int64_t pg = page_table[recs[i].table_off + e];
            if (pg < 0 || (uint64_t)pg >= n_pages)
                *flag_dev = 1;
            if ((pg < 0 || (uint64_t)pg >= n_pages) && !report->bad) {
                report->bad = 1;
                report->req = recs[i].req;
                report->entry = recs[i].table_off + e;
                report->page = pg;
            }
        }
    return hipSuccess;
}

hipError_t launch_patch(int32_t *page_table, const uint64_t *entry, const int32_t *page, uint32_t n, hipStream_t) {
    for (uint32_t i = 0; i < n; ++i)
        page_table[entry[i]] = page[i];
    return hipSuccess;
}

// The table entries an item reads (tokens [t0, t1) of the slice's heads), as the kernel addresses them; entries
// the step adds come from the kernel arguments and are written to the table.
static void walk_item(const DecodeArgs &a, const StepPages &sp, const ItemRec &r0) {
    ItemRec r = r0;
    if (r.it.t1 == r.s.ctx_len)
        r.it.t1 += a.delta;
    r.s.ctx_len += a.delta;
    if (r.it.t0 > r.it.t1 || r.it.t1 > r.s.ctx_len)
        die("item outside its sequence");
    const uint64_t T = r.c.token_bytes, lg = a.log2_page;
    const bool appends = a.new_k != nullptr && r.s.ctx_len > 0 && r.it.t1 == r.s.ctx_len;
    uint64_t new_lo = 0, new_n = 0, new_first = 0;
    if (appends && sp.n_req) {
        if (r.s.req >= sp.n_req)
            die("request index outside the step's page list");
        new_first = sp.first[r.s.req];
        new_n = sp.first[r.s.req + 1] - new_first;
        new_lo = ((uint64_t)(r.s.ctx_len - 1) * T + ((1ull << lg) - 1)) >> lg;
    }
    int32_t *tab = const_cast<int32_t *>(a.page_table) + r.s.table_off;
    const uint64_t lo = (uint64_t)r.s.head0 * r.c.row_bytes, hi = (uint64_t)(r.s.head0 + r.c.hs) * r.c.row_bytes;
    for (uint64_t t = r.it.t0; t < r.it.t1; ++t)
        for (uint64_t e = (t * T + lo) >> lg; e <= (t * T + hi - 1) >> lg; ++e) {
            if (e - new_lo < new_n)
                tab[e] = sp.page[new_first + (e - new_lo)];
            const int32_t pg = tab[e];
            if (pg < 0 || (uint64_t)pg >= g_fake.n_pages)
                die("page id out of range in a table entry the launch reads");
            ++g_fake.checked_entries;
        }
    g_fake.appended += appends;
    ++g_fake.items;
}

hipError_t launch_decode(const DecodeArgs &a, const StepPages *sp_in, uint32_t grid, uint32_t, uint32_t, hipStream_t,
                         hipEvent_t, hipEvent_t) {
    static const StepPages none{};
    const StepPages &sp = sp_in ? *sp_in : none;
    if (a.bad && *a.bad)
        return hipSuccess;
    if (grid == 0 || grid > a.n_spans)
        die("grid must be in [1, n_spans]");
    if (a.log2_page != g_fake.log2_page)
        die("page size");
    uint32_t q = *a.queue - a.queue_base; // as the workgroups would find it
    if (q != 0)
        die("span queue does not start at the launch's base");
    for (uint32_t span = 0; span < a.n_spans; ++span)
        for (uint32_t i = a.span_first[span]; i < a.span_first[span + 1]; ++i)
            walk_item(a, sp, a.recs[i]);
    *a.queue += a.n_spans; // every workgroup takes until it fails once
    if (a.counters)        // the last part of every cut sequence resets its counter
        for (uint32_t i = 0; i < a.span_first[a.n_spans]; ++i)
            if (a.counters[a.recs[i].it.seq] != 0)
                die("a sequence's part counter is not zero at launch");
    return hipSuccess;
}

hipError_t launch_reduce(const ReduceRec *recs, uint32_t n_recs, uint32_t n_many, uint32_t, uint32_t, const float *,
                         float *, hipStream_t, hipEvent_t, hipEvent_t) {
    for (uint32_t i = 0; i < n_recs; ++i)
        if ((i < n_many) != (recs[i].n_parts > kReduceFewParts) || recs[i].n_parts < 2)
            die("merge list");
    return hipSuccess;
}
hipError_t launch_reduce_counted(const ReduceRec *, const uint32_t *, uint32_t, const ReduceRec *, const uint32_t *,
                                 uint32_t, uint32_t, uint32_t, const float *, float *, hipStream_t) {
    return hipSuccess;
}

hipError_t launch_append(unsigned char *, uint32_t lg, int32_t *page_table, const AppendRec *recs, uint32_t n,
                         const ClassRec *classes, const void *, const void *, const uint64_t *pe, const int32_t *pp,
                         uint32_t n_patches, const uint32_t *bad, hipStream_t, hipEvent_t, hipEvent_t) {
    if (bad && *bad)
        return hipSuccess;
    for (uint32_t i = 0; i < n; ++i) {
        const AppendRec &r = recs[i];
        if (r.ctx_len == 0)
            continue;
        const ClassRec &c = classes[r.cls];
        const uint64_t first = ((uint64_t)(r.ctx_len - 1) * c.token_bytes) >> lg,
                       last = ((uint64_t)r.ctx_len * c.token_bytes - 1) >> lg;
        for (uint64_t e = first; e <= last; ++e) {
            int32_t pg = e - first < 4 ? r.page[e - first] : -1;
            if (pg < 0)
                pg = page_table[r.table_off + e];
            if (pg < 0 || (uint64_t)pg >= g_fake.n_pages)
                die("append through a page id out of range");
        }
    }
    for (uint32_t i = 0; i < n_patches; ++i)
        page_table[pe[i]] = pp[i];
    return hipSuccess;
}

// The copy pass of the one-part weights: writes (zeros) exactly the bytes the kernel would write, so that the
// sanitizer sees a record that reaches past the workspace.
hipError_t launch_v16(const unsigned char *, uint32_t lg, const int32_t *page_table, const V16Rec *recs, uint32_t n_recs,
                      unsigned char *v16, const uint32_t *bad, hipStream_t) {
    if (bad && *bad)
        return hipSuccess;
    for (uint32_t i = 0; i < n_recs; ++i) {
        const V16Rec &r = recs[i];
        if (r.t0 >= r.t1 || r.t1 > r.ctx_len || (r.d != 64 && r.d != 128) || r.n_kv == 0)
            die("fp16 copy record");
        const uint64_t last = ((uint64_t)r.t1 * r.token_bytes - 1) >> lg;
        for (uint64_t e = ((uint64_t)r.t0 * r.token_bytes) >> lg; e <= last; ++e)
            if (page_table[r.table_off + e] < 0 || (uint64_t)page_table[r.table_off + e] >= g_fake.n_pages)
                die("fp16 copy through a page id out of range");
        for (uint32_t h = 0; h < r.n_kv; ++h)
            std::memset(v16 + r.v16_off + ((uint64_t)h * r.ctx_len + r.t0) * 2 * r.d, 0, (size_t)(r.t1 - r.t0) * 2 * r.d);
    }
    return hipSuccess;
}

hipError_t launch_prefill(const PrefillArgs &a, uint32_t n_recs, uint32_t head_dim, uint32_t parts, hipStream_t,
                          hipEvent_t, hipEvent_t) {
    if (a.bad && *a.bad)
        return hipSuccess;
    if (parts != 1 && parts != 2)
        die("prefill parts");
    for (uint32_t i = 0; i < n_recs; ++i) {
        const PrefillRec &r = a.recs[i];
        if (r.q_len == 0)
            continue; // filler
        if (r.q_len > r.ctx_len || r.r0 >= r.q_len)
            die("prefill record");
        if (r.t0 >= r.t1 || r.t1 > r.ctx_len || (r.t0 % 32) != 0)
            die("prefill record: stretch of tokens");
        if (r.part != kPrefillDirect) // the partial this record leaves: written, so that the sanitizer sees its bounds
            std::memset(a.partials + (uint64_t)r.part * kPrefillPartFloats, 0, kPrefillPartFloats * sizeof(float));
        if (parts == 1) { // the rows this record reads from the fp16 copy: first and last byte
            const volatile unsigned char *v = a.v16 + r.v16_off;
            (void)v[0];
            (void)v[(uint64_t)r.ctx_len * 2 * head_dim - 1];
        }
        const uint64_t last = ((uint64_t)r.ctx_len * r.token_bytes - 1) >> a.log2_page;
        for (uint64_t e = 0; e <= last; ++e)
            if (a.page_table[r.table_off + e] < 0 || (uint64_t)a.page_table[r.table_off + e] >= g_fake.n_pages)
                die("prefill through a page id out of range");
    }
    return hipSuccess;
}

hipError_t launch_prefill_merge(const PrefillMergeRec *recs, uint32_t n_recs, const float *partials, float *,
                                const uint32_t *bad, hipStream_t) {
    if (bad && *bad)
        return hipSuccess;
    for (uint32_t i = 0; i < n_recs; ++i) {
        const PrefillMergeRec &r = recs[i];
        if (r.n_parts < 2 || r.r0 >= r.q_len || (r.d != 64 && r.d != 128))
            die("prefill merge record");
        const volatile float *v = partials + (uint64_t)r.part0 * kPrefillPartFloats;
        (void)v[0];
        (void)v[(uint64_t)r.n_parts * kPrefillPartFloats - 1];
    }
    return hipSuccess;
}

hipError_t launch_copy_tokens(bool, unsigned char *, uint32_t lg, const int32_t *page_table, const GatherRec *recs,
                              uint32_t n, const ClassRec *classes, void *, void *, const uint32_t *bad, hipStream_t) {
    if (bad && *bad)
        return hipSuccess;
    for (uint32_t i = 0; i < n; ++i) {
        const GatherRec &r = recs[i];
        if (r.t0 >= r.t1 || r.flat_t0 > r.t0)
            die("copy record");
        const uint64_t T = classes[r.cls].token_bytes;
        for (uint64_t e = ((uint64_t)r.t0 * T) >> lg; e <= ((uint64_t)r.t1 * T - 1) >> lg; ++e)
            if (page_table[r.table_off + e] < 0 || (uint64_t)page_table[r.table_off + e] >= g_fake.n_pages)
                die("copy through a page id out of range");
    }
    return hipSuccess;
}

} // namespace ukv

extern "C" void fake_device_set(uint64_t n_pages, uint32_t log2_page) {
    g_fake.n_pages = n_pages;
    g_fake.log2_page = log2_page;
}
extern "C" void fake_device_counts(uint64_t *entries, uint64_t *items, uint64_t *appended) {
    *entries = g_fake.checked_entries;
    *items = g_fake.items;
    *appended = g_fake.appended;
}
