// Decode attention for callers that cannot allocate: ukv_decode_attention_static.
//
// The existing entry points plan on the host (from host arrays) and carry the plan to the device through pinned
// staging buffers that they allocate on first use; the caller brings the workspace.  Code under HIP graph capture,
// tight serving loops and harnesses that forbid hipMalloc can do neither.  Here every array of the batch
// descriptor lives in device memory, the launch is planned ON the device by static_plan_kernel, and everything the
// kernels need beyond the caller's inputs and outputs -- the plan and the split-KV partials -- lives in one
// file-scope device array of fixed size.  The call enqueues four launches (plan, decode, two merge kernels) and calls
// no allocating routine.  Decode and merge kernels are those of ukv_decode_attention.
#include <algorithm>
#include <string>

#include "ukv_device.h"

namespace ukv {

// ---- the scratch array: one copy per device, held until the process ends -------------------------------------
static constexpr size_t kStaticScratchBytes = (size_t)UKV_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

static constexpr uint32_t kStaticMaxRequests = UKV_STATIC_MAX_REQUESTS;
static constexpr uint32_t kStaticMaxSeqs = 8192;  // (request, head-slice) sequences
static constexpr uint32_t kStaticMaxSpans = 1024; // decode workgroups = threads of the plan kernel
static constexpr uint32_t kPlanThreads = 1024;

constexpr size_t up256(size_t x) { return (x + 255) / 256 * 256; }
// layout of the array (byte offsets)
static constexpr size_t kOffSeqs = 0;
static constexpr size_t kOffItems = up256(kOffSeqs + kStaticMaxSeqs * sizeof(SeqRec));
static constexpr size_t kOffSpans = up256(kOffItems + (kStaticMaxSeqs + kStaticMaxSpans) * sizeof(ItemRec));
static constexpr size_t kOffMany = up256(kOffSpans + (kStaticMaxSpans + 1) * sizeof(uint32_t));
static constexpr size_t kOffFew = up256(kOffMany + kStaticMaxSpans * sizeof(ReduceRec));
static constexpr size_t kOffCounts = up256(kOffFew + kStaticMaxSpans * sizeof(ReduceRec));
static constexpr size_t kOffStart = up256(kOffCounts + 4 * sizeof(uint32_t)); // two list lengths, the span queue, the span count
static constexpr size_t kOffPartials = up256(kOffStart + (kStaticMaxSeqs + 1) * sizeof(uint64_t));
static_assert(kOffPartials + (1u << 20) < kStaticScratchBytes, "scratch too small for its plan area");

struct StaticPlanArgs {
    ClassTable classes;
    uint32_t n_services;
    uint32_t n_requests;
    const uint32_t *service_id; // DEVICE [n]
    const uint32_t *ctx_len;
    const uint64_t *table_off;
    const uint64_t *q_off;
    const uint64_t *out_off;
    uint32_t max_spans;      // what the partial area holds for this pool's largest partial, <= kStaticMaxSpans
    uint32_t slots;          // compute units of the device
    uint64_t min_span_bytes; // tunable of the pool
    uint32_t gqa_cost_pct;
    unsigned char *scratch;
};

// Exclusive prefix sum over the workgroup's threads (kPlanThreads = 16 waves); every thread gets its prefix and the
// total.  tmp: 17 values in LDS.
__device__ __forceinline__ uint64_t block_scan(uint64_t v, uint64_t *tmp, uint64_t &total) {
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint64_t inc = v;
    for (int o = 1; o < 64; o <<= 1) {
        const uint64_t up = __shfl_up(inc, o);
        if ((int)lane >= o)
            inc += up;
    }
    __syncthreads(); // tmp may still be read from the previous scan
    if (lane == 63)
        tmp[wave] = inc;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint64_t run = 0;
        for (uint32_t w = 0; w < kPlanThreads / 64; ++w) {
            const uint64_t x = tmp[w];
            tmp[w] = run;
            run += x;
        }
        tmp[kPlanThreads / 64] = run;
    }
    __syncthreads();
    total = tmp[kPlanThreads / 64];
    return tmp[wave] + inc - v;
}

// The split-KV plan of ukv_decode_attention, made by one workgroup on the device.  Cost is counted as on the host
// (KV bytes of a head-slice per token, weighted for the matrix-core kind, plus a fixed amount per sequence); the
// sequences are laid end to end in request order on a cost axis, the axis is cut into equal spans (one decode
// workgroup each), and a span's work items are its intersections with the sequences.  A sequence that lies in
// several spans gets one partial per span and a record in one of the two merge lists.  Every cut is a valid plan:
// results differ from the host-planned call's only in fp32 summation order.
__global__ void __launch_bounds__(kPlanThreads) static_plan_kernel(StaticPlanArgs a) {
    __shared__ uint64_t s_tmp[kPlanThreads / 64 + 1];
    const uint32_t tid = threadIdx.x;
    unsigned char *w = a.scratch;
    SeqRec *seqs = reinterpret_cast<SeqRec *>(w + kOffSeqs);
    ItemRec *items = reinterpret_cast<ItemRec *>(w + kOffItems); // one record per work item, in span order
    uint32_t *span_first = reinterpret_cast<uint32_t *>(w + kOffSpans);
    ReduceRec *many = reinterpret_cast<ReduceRec *>(w + kOffMany);
    ReduceRec *few = reinterpret_cast<ReduceRec *>(w + kOffFew);
    uint32_t *counts = reinterpret_cast<uint32_t *>(w + kOffCounts);
    uint64_t *start = reinterpret_cast<uint64_t *>(w + kOffStart); // start[k] = first cost unit of sequence k

    auto token_cost = [&](const ClassRec &c) -> uint64_t {
        const uint64_t bytes = (uint64_t)c.hs * c.row_bytes;
        return kind_is_gqa(c.kind) ? bytes * a.gqa_cost_pct / 100 : bytes;
    };

    // sequences of request `tid`: one per head-slice; a request with a service id outside the pool has none
    uint32_t cls = 0, n_sl = 0;
    if (tid < a.n_requests) {
        cls = a.service_id[tid];
        if (cls < a.n_services)
            n_sl = a.classes.c[cls].n_kv / a.classes.c[cls].hs;
    }
    uint64_t total = 0;
    const uint32_t k0 = (uint32_t)block_scan(n_sl, s_tmp, total);
    const uint32_t n_seqs = (uint32_t)total; // <= kStaticMaxSeqs: checked on the host against the widest service
    if (n_sl) {
        const ClassRec &c = a.classes.c[cls];
        SeqRec s{};
        s.table_off = a.table_off[tid];
        s.q_off = a.q_off[tid];
        s.out_off = a.out_off[tid];
        s.ctx_len = a.ctx_len[tid];
        s.cls = cls;
        s.req = tid;
        s.part_stride = part_stride_of(c);
        const uint64_t wk = kItemOverheadBytes + (uint64_t)s.ctx_len * token_cost(c);
        for (uint32_t sl = 0; sl < n_sl; ++sl) {
            s.head0 = sl * c.hs;
            seqs[k0 + sl] = s; // n_parts and part_off follow below
            start[k0 + sl] = wk;
        }
    }
    __syncthreads();

    // cost axis: start[k] = sum of the costs before sequence k, start[n_seqs] = all of it
    const uint32_t per = (n_seqs + kPlanThreads - 1) / kPlanThreads; // consecutive sequences per thread
    const uint32_t c0 = min(tid * per, n_seqs), c1 = min(c0 + per, n_seqs);
    uint64_t mine = 0;
    for (uint32_t k = c0; k < c1; ++k)
        mine += start[k];
    uint64_t C = 0;
    uint64_t run = block_scan(mine, s_tmp, C);
    for (uint32_t k = c0; k < c1; ++k) {
        const uint64_t wk = start[k];
        start[k] = run;
        run += wk;
    }
    if (tid == 0)
        start[n_seqs] = C;
    __syncthreads();

    // equal spans.  As on the host: no span below min_span_bytes, except that a batch too small to give every
    // compute unit that much is cut finer, down to 64 KiB a span.
    uint32_t n_spans = 0;
    uint64_t span = 1;
    if (n_seqs) {
        uint64_t min_span = a.min_span_bytes < C / a.slots ? a.min_span_bytes : C / a.slots;
        if (min_span < kSmallBatchSpanBytes)
            min_span = kSmallBatchSpanBytes;
        uint64_t n = C / min_span;
        n = n < 1 ? 1 : (n > a.max_spans ? a.max_spans : n);
        span = (C + n - 1) / n;
        n_spans = (uint32_t)((C + span - 1) / span);
    }

    // per sequence: the spans it lies in, its partials, its place in a merge list
    uint64_t floats_mine = 0;
    uint32_t many_mine = 0, few_mine = 0;
    auto parts_of = [&](uint32_t k) { return (uint32_t)((start[k + 1] - 1) / span - start[k] / span) + 1; };
    for (uint32_t k = c0; k < c1; ++k) {
        const uint32_t np = parts_of(k);
        if (np > 1) {
            floats_mine += (uint64_t)np * seqs[k].part_stride;
            const ClassRec &c = a.classes.c[seqs[k].cls];
            if (np > kReduceFewParts || !reduce_few_takes(kind_is_gqa(c.kind) ? c.g : 0, c.d))
                ++many_mine;
            else
                ++few_mine;
        }
    }
    uint64_t t_floats, t_many, t_few;
    uint64_t f_run = block_scan(floats_mine, s_tmp, t_floats);
    uint32_t m_run = (uint32_t)block_scan(many_mine, s_tmp, t_many);
    uint32_t w_run = (uint32_t)block_scan(few_mine, s_tmp, t_few);
    for (uint32_t k = c0; k < c1; ++k) {
        const uint32_t np = parts_of(k);
        SeqRec &s = seqs[k];
        s.n_parts = np;
        if (np <= 1)
            continue;
        s.part_off = f_run;
        f_run += (uint64_t)np * s.part_stride;
        const ClassRec &c = a.classes.c[s.cls];
        ReduceRec r{};
        r.part_off = s.part_off;
        r.out_off = s.out_off + (uint64_t)s.head0 * c.g * c.d;
        r.n_parts = np;
        r.part_stride = s.part_stride;
        r.n_heads = c.hs * c.g;
        r.d = c.d;
        r.layout_g = kind_is_gqa(c.kind) ? c.g : 0;
        if (np > kReduceFewParts || !reduce_few_takes(r.layout_g, r.d))
            many[m_run++] = r;
        else
            few[w_run++] = r;
    }
    if (tid == 0) {
        counts[0] = (uint32_t)t_many;
        counts[1] = (uint32_t)t_few;
        counts[2] = 0; // the decode launch's span queue starts at zero
        counts[3] = n_spans;
    }

    // per span (one thread each): the sequences it meets, then its items
    uint32_t first = 0, n_it = 0;
    uint64_t lo = 0, hi = 0;
    if (tid < n_spans) {
        lo = (uint64_t)tid * span;
        hi = lo + span < C ? lo + span : C;
        auto seq_at = [&](uint64_t x) { // the sequence that holds cost unit x: largest k with start[k] <= x
            uint32_t l = 0, r = n_seqs; // start[l] <= x < start[r]
            while (r - l > 1) {
                const uint32_t m = (l + r) / 2;
                if (start[m] <= x)
                    l = m;
                else
                    r = m;
            }
            return l;
        };
        first = seq_at(lo);
        n_it = seq_at(hi - 1) - first + 1;
    }
    uint64_t t_items;
    const uint32_t i0 = (uint32_t)block_scan(n_it, s_tmp, t_items);
    span_first[tid] = i0; // spans past n_spans are empty: their workgroups leave at once
    if (tid == kPlanThreads - 1)
        span_first[kPlanThreads] = (uint32_t)t_items;
    for (uint32_t e = 0; e < n_it; ++e) {
        const uint32_t k = first + e;
        const uint64_t sk = start[k], ek = start[k + 1];
        const uint32_t n_tok = seqs[k].ctx_len;
        const uint64_t tc = token_cost(a.classes.c[seqs[k].cls]);
        // token boundary at cost unit x of the axis: the sequence's fixed cost comes first, then its tokens in order
        auto cut = [&](uint64_t x) -> uint32_t {
            if (x >= ek)
                return n_tok;
            const uint64_t rel = x > sk ? x - sk : 0;
            if (rel <= kItemOverheadBytes)
                return 0;
            const uint64_t t = (rel - kItemOverheadBytes) / tc;
            return t < n_tok ? (uint32_t)t : n_tok;
        };
        const uint32_t f_k = (uint32_t)(sk / span), np = (uint32_t)((ek - 1) / span) - f_k + 1;
        ItemRec &r = items[i0 + e];
        r.it = Item{k, cut(lo), cut(hi), np > 1 ? tid - f_k : kDirect};
        r.s = seqs[k]; // complete: n_parts and part_off were written before the last workgroup barrier
        r.c = a.classes.c[seqs[k].cls];
    }
}

// ---- host side --------------------------------------------------------------------------------------------
static constexpr int kMaxDevices = 64;
static unsigned char *g_scratch_ptr[kMaxDevices]; // device address of `scratch` on each device, taken once
static int g_cus[kMaxDevices];

// Device address of this device's copy of the array.  In host code `scratch` is only a handle for the symbol:
// kernels and copies get the address looked up here.
static int scratch_of_current_device(unsigned char **out, int *cus) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        set_error(std::string("hipGetDevice: ") + (e != hipSuccess ? hipGetErrorString(e) : "device index out of range"));
        return UKV_EHIP;
    }
    if (g_scratch_ptr[dev] == nullptr) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || ptr == nullptr) {
            set_error(std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e));
            return UKV_EHIP;
        }
        int n = 0;
        e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess || n <= 0) {
            set_error(std::string("hipDeviceGetAttribute: ") + hipGetErrorString(e));
            return UKV_EHIP;
        }
        g_cus[dev] = n;
        g_scratch_ptr[dev] = static_cast<unsigned char *>(ptr);
    }
    *out = g_scratch_ptr[dev];
    *cus = g_cus[dev];
    return UKV_OK;
}

} // namespace ukv

using namespace ukv;

extern "C" int ukv_decode_attention_static(ukv_pool_t *p, const ukv_device_batch_t *b, void *stream) {
    Trace trace("ukv_decode_attention_static"); // (a fixed buffer and stderr: nothing is allocated)
    if (b)
        trace.add("requests", b->n_requests);
    if (!p || !b) {
        set_error("null pool or batch");
        return UKV_EINVAL;
    }
    const uint32_t n = b->n_requests;
    if (n == 0)
        return UKV_OK;
    if (!b->service_id || !b->ctx_len || !b->table_off || !b->page_table || !b->q || !b->q_off || !b->out ||
        !b->out_off) {
        set_error("every array of the device batch must be a non-null device pointer");
        return UKV_EINVAL;
    }
    // sizes against the fixed scratch array
    uint32_t max_sl = 1, max_stride = 32, max_heads = 1, max_units = 1;
    bool all_few = true; // no service whose cut sequences all go to the many-parts merge kernel (see reduce_few_takes)
    for (uint32_t s = 0; s < p->n_services; ++s) {
        const ClassRec &c = p->classes.c[s];
        max_sl = std::max(max_sl, c.n_kv / c.hs);
        max_stride = std::max(max_stride, part_stride_of(c));
        max_heads = std::max(max_heads, c.hs * c.g);
        max_units = std::max(max_units, kind_is_gqa(c.kind) ? c.hs : c.hs * c.g);
        all_few = all_few && reduce_few_takes(kind_is_gqa(c.kind) ? c.g : 0, c.d);
    }
    if (n > kStaticMaxRequests || (uint64_t)n * max_sl > kStaticMaxSeqs) {
        set_error("batch too large for the static scratch array: at most " + std::to_string(kStaticMaxRequests) +
                  " requests and " + std::to_string(kStaticMaxSeqs) + " (request, head-slice) sequences, got " +
                  std::to_string(n) + " requests x " + std::to_string(max_sl) + " slices");
        return UKV_ENOSPC;
    }
    // Equal spans cut at most one sequence per boundary, so S spans leave at most 2 S partials.
    const uint64_t part_bytes = kStaticScratchBytes - kOffPartials;
    const uint32_t max_spans =
        (uint32_t)std::min<uint64_t>(kStaticMaxSpans, part_bytes / (2ull * max_stride * sizeof(float)));
    if (max_spans == 0) {
        set_error("a split partial of this pool's widest service does not fit the static scratch array");
        return UKV_ENOSPC;
    }
    unsigned char *sp = nullptr;
    int cus = 0;
    int rc = scratch_of_current_device(&sp, &cus);
    if (rc != UKV_OK)
        return rc;
    hipStream_t s = (hipStream_t)stream;

    StaticPlanArgs pa{};
    pa.classes = p->classes;
    pa.n_services = p->n_services;
    pa.n_requests = n;
    pa.service_id = b->service_id;
    pa.ctx_len = b->ctx_len;
    pa.table_off = b->table_off;
    pa.q_off = b->q_off;
    pa.out_off = b->out_off;
    pa.max_spans = max_spans;
    pa.slots = (uint32_t)cus;
    pa.min_span_bytes = (uint64_t)p->tun.min_span_bytes;
    pa.gqa_cost_pct = (uint32_t)p->tun.gqa_cost_pct;
    pa.scratch = sp;
    hipLaunchKernelGGL(static_plan_kernel, dim3(1), dim3(kPlanThreads), 0, s, pa);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error(std::string("launch plan kernel: ") + hipGetErrorString(e));
        return UKV_EHIP;
    }

    DecodeArgs a{};
    a.pool_base = p->base;
    a.log2_page = p->log2_page;
    a.page_table = b->page_table;
    a.q = b->q;
    a.out = (float *)b->out;
    a.recs = (const ItemRec *)(sp + kOffItems);
    a.span_first = (const uint32_t *)(sp + kOffSpans);
    a.partials = (float *)(sp + kOffPartials);
    a.counters = nullptr; // cut sequences are merged by the two launches below
    a.merge_acq_rel = 0;
    a.new_k = nullptr;
    a.new_v = nullptr;
    a.delta = 0;
    a.bad = nullptr; // (UKV_PARAM_VALIDATE does not cover this entry point: its check needs staging memory)
    a.queue = (uint32_t *)(sp + kOffCounts) + 2;
    a.queue_base = 0;
    a.n_spans = kStaticMaxSpans;
    a.n_spans_dev = (const uint32_t *)(sp + kOffCounts) + 3; // what the plan kernel made of the batch
    // (every place of the device: this plan's spans are all of one small size, there is no first round)
    e = launch_decode(a, nullptr, decode_grid(kStaticMaxSpans, (uint32_t)p->tun.block_threads, p->kinds, 0),
                      (uint32_t)p->tun.block_threads, p->kinds, s, nullptr, nullptr);
    if (e != hipSuccess) {
        set_error(std::string("launch decode kernel: ") + hipGetErrorString(e));
        return UKV_EHIP;
    }
    // At most max_spans - 1 sequences are cut; one of more than kReduceFewParts parts uses up that many boundaries.
    const uint32_t few_bound = max_spans - 1, many_bound = all_few ? (max_spans - 1) / kReduceFewParts : max_spans - 1;
    const uint32_t *counts = (const uint32_t *)(sp + kOffCounts);
    e = launch_reduce_counted((const ReduceRec *)(sp + kOffMany), counts, many_bound, (const ReduceRec *)(sp + kOffFew),
                              counts + 1, few_bound, max_heads, max_units, a.partials, a.out, s);
    if (e != hipSuccess) {
        set_error(std::string("launch merge kernels: ") + hipGetErrorString(e));
        return UKV_EHIP;
    }
    return UKV_OK;
}
