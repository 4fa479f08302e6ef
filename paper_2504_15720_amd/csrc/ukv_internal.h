// Internal declarations shared by the host code and the HIP kernels of libukv.
#pragma once

#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>
#include <string>
#include <utility>
#include <vector>

#include "ukv.h"

namespace ukv {

// ---- records copied to the device with every decode call (plain data, 16-byte aligned) ----

// One (request, head-slice) sequence.
struct SeqRec {
    uint64_t table_off;   // first page-table entry of the request
    uint64_t q_off;       // element offset of the request's q (head 0)
    uint64_t out_off;     // element offset of the request's out (head 0)
    uint64_t part_off;    // float offset of this sequence's first partial (n_parts > 1)
    uint64_t new_off;     // element offset of the request's new K/V token (fused append only)
    uint32_t ctx_len;
    uint32_t cls;         // service index
    uint32_t head0;       // first kv head of the slice
    uint32_t n_parts;     // work items this sequence was cut into
    uint32_t part_stride; // floats per partial: n_heads_q * (head_dim + 2), rounded up to 32 (one line)
    uint32_t req;         // index of the request in the batch
};
static_assert(sizeof(SeqRec) == 64, "SeqRec layout");

// One work item: tokens [t0, t1) of a sequence.  part == kDirect: the item is the whole
// sequence and writes the final output.
struct Item {
    uint32_t seq, t0, t1, part;
};
static constexpr uint32_t kDirect = 0xffffffffu;
// A sequence whose partials add up to more than this many floats (256 KiB) is never merged inside the decode
// launch: one workgroup walking that much is a long serial chain (hundreds of microseconds for a long request
// alone on the device); the second launch spreads the work over (query head, part) instead.
static constexpr uint64_t kFusedMergeMaxFloats = 64 * 1024;
__host__ __device__ inline bool merges_in_launch(uint32_t n_parts, uint32_t part_stride) {
    return (uint64_t)n_parts * part_stride <= kFusedMergeMaxFloats;
}
// The second launch takes sequences of up to this many parts with one wave per (sequence, query head), part
// after part, and longer ones with four waves that share the parts.
static constexpr uint32_t kReduceFewParts = 24;
// reduce_few_kernel gives a lane 64-float strides of one partial and one query head's (m, l): in the matrix-core layout
// that needs the group size to divide 32 and G d / 64 <= 16 elements per lane.  Other shapes go to reduce_many_kernel.
__host__ __device__ inline bool reduce_few_takes(uint32_t layout_g, uint32_t d) {
    return layout_g == 0 || (32 % layout_g == 0 && layout_g * d <= 16 * 64);
}

// Per-service constants used by the kernels.
struct ClassRec {
    uint32_t n_q, n_kv, d, g;
    uint32_t row_bytes, token_bytes;
    uint32_t hs, ti;      // kv heads per slice, token lanes (for the configured block size)
    float scale_log2e;    // softmax scale * log2(e)
    uint32_t kind;        // index of the compiled (head_dim, group) variant
    uint32_t pad_[2];
};
struct ClassTable {
    ClassRec c[UKV_MAX_SERVICES];
};

// What a decode workgroup needs to start an item, in one 128-byte record (one load, fetched while the previous item
// is still being worked on): the item, its sequence and the constants of the sequence's service.
struct ItemRec {
    Item it;
    SeqRec s;
    ClassRec c;
};
static_assert(sizeof(ItemRec) == 128 && offsetof(ItemRec, it.t1) == 8 && offsetof(ItemRec, s.ctx_len) == 56,
              "ItemRec layout (the kernel patches t1 and ctx_len by position)");

// kD64GQA: groups of 3 to 16 query heads at head_dim 64, on the matrix-core path like kD128GQA; not a shape of the
// workloads, and kept out of the kernels that their pools use (kWorkloadKinds).
enum Kind : uint32_t { kD64G1, kD64G2, kD128G1, kD128GQA, kD64GQA, kNumKinds };
static constexpr uint32_t kWorkloadKinds = (1u << kD64G1) | (1u << kD64G2) | (1u << kD128G1) | (1u << kD128GQA);
__host__ __device__ inline bool kind_is_gqa(uint32_t kind) { return kind == kD128GQA || kind == kD64GQA; }
static constexpr uint32_t kAllKinds = (1u << kNumKinds) - 1;

// floats of one split partial of a (request, head-slice) sequence: accumulators and (m, l) pairs of its query heads,
// rounded up so that partials of different items never share a 128-byte line
__host__ __device__ inline uint32_t part_stride_of(const ClassRec &c) { return (c.hs * c.g * (c.d + 2) + 31u) & ~31u; }
// planner cost of one item beyond its KV bytes (q load, merge and output), in KV bytes
static constexpr uint64_t kItemOverheadBytes = 16 * 1024;
static constexpr uint64_t kSmallBatchSpanBytes = 64 * 1024; // batches too small to fill the device are cut down to this

struct DecodeArgs {
    const unsigned char *pool_base;
    uint32_t log2_page;
    const int32_t *page_table;
    const void *q;      // bf16
    float *out;
    const ItemRec *recs;        // one per work item, in span order
    const uint32_t *span_first; // [n_spans + 1]
    float *partials;
    uint32_t *counters; // per sequence: finished items (fused merge); null = merge in a second launch
    uint32_t merge_acq_rel; // fused merge: count items with an agent-scope acquire-release instead of relaxed + waits
    // Fused append (null = attention only): the item that holds a request's last token takes that
    // token's K/V from here and stores it into the request's pages.
    const uint16_t *new_k;
    const uint16_t *new_v;
    // A plan that outlives its step: every sequence has grown by `delta` tokens since the plan was made; the growth
    // goes to the sequence's last item (the one whose t1 equals the planned ctx_len).  0 for a plan made for this call.
    uint32_t delta;
    const uint32_t *bad; // null, or the flag of the page-table check: set = leave at once
    // Spans are handed out through a queue in device memory: the launch has one workgroup per place the device
    // offers (grid <= n_spans); workgroup w starts with span w, and a workgroup that has finished a span takes the
    // next one, whichever XCD it runs on.  (The hardware deals the workgroups of a grid out to the XCDs in turn, and
    // the XCDs do not run at the same speed: with one workgroup per span the slowest XCD finished its fixed share
    // long after the fastest.)  A take is grid + atomic_add(queue, 1) - queue_base; values >= n_spans end the
    // workgroup.  Every workgroup takes until it fails once, so a launch leaves the counter n_spans higher, which
    // the host adds to queue_base of the next launch of the same plan.  n_spans_dev (may be null): the number of
    // spans if only the device knows it; n_spans is then an upper bound and empty spans may follow the last one.
    uint32_t *queue;
    uint32_t queue_base;
    uint32_t n_spans;
    const uint32_t *n_spans_dev;
};

// The page ids of the table entries a step adds, carried in the kernel arguments (no upload of their own): request r
// gets page[first[r]] .. page[first[r + 1] - 1] for the entries ceil((c - 1) T / P) .. ceil(c T / P) - 1 of its table,
// c its length after the step.  n_req == 0: nothing rides here (the entries are in the table already).
static constexpr uint32_t kStepMaxReq = 766, kStepMaxPages = 576;
struct StepPages {
    uint32_t n_req;
    uint16_t first[kStepMaxReq + 2];
    int32_t page[kStepMaxPages];
};
static_assert(sizeof(DecodeArgs) + sizeof(StepPages) <= 4096, "decode kernel arguments exceed 4 KiB");

// Opt-in check of the page tables a call is about to use (UKV_PARAM_VALIDATE): one record per request.
struct ValRec {
    uint64_t table_off;
    uint64_t n_entries; // entries [0, n_entries) of the request's table are checked
    uint32_t req;
    uint32_t pad_;
};
// What the check reports, in pinned host memory that the device writes: the first bad entry found.  (The kernels
// of a checked call read a flag in device memory instead, set together with `bad`: a read of host memory at the
// start of every workgroup was measured at a third of the decode launch.)
struct ValReport {
    uint32_t bad; // 0 = nothing found
    uint32_t req;
    uint64_t entry; // index into page_table
    int64_t page;
};

struct ReduceRec {
    uint64_t part_off;
    uint64_t out_off;     // element offset of the slice's first q head in out
    uint32_t n_parts, part_stride, n_heads, d;
    uint32_t layout_g; // 0 = ALU-path partial layout, else the group size of the matrix-core path
    uint32_t pad_[3];
};

struct AppendRec {
    uint64_t table_off;
    uint64_t new_off;
    uint32_t ctx_len;
    uint32_t cls;
    int32_t page[4]; // page ids of the first four pages the new token touches, where the same call
                     // patches those table entries; -1 = read the table
};

// Prefill: one workgroup = a tile of query rows of one (request, kv head).
struct PrefillRec {
    uint64_t table_off;
    uint64_t q_off;   // element offset of the request's first query row
    uint64_t out_off; // element offset of the request's first output row
    uint32_t ctx_len; // tokens in the cache, the chunk's own included
    uint32_t q_len;   // query rows of the request; row r is the token at position ctx_len - q_len + r;
                      // q_len == 0: filler workgroup (keeps the XCD interleave regular)
    uint64_t v16_off; // one-part weights only: byte offset, in the workspace, of this (request, kv head)'s V rows as fp16
    uint32_t r0;      // first query row of the tile
    // what the kernel needs of the service's class, copied here so that a workgroup starts with one load
    uint32_t g; // low half: query heads per kv head; high half: that number rounded up to a power of two, the number
                // of columns a query row takes up in a block of 16 (columns past the group stay empty)
    uint32_t n_q, token_bytes;
    float scale_log2e;
    uint32_t kvh;
    // The tokens this workgroup walks: all its rows can see (0 .. position of its last row), or, where few
    // workgroups would each walk a long context, one stretch [t0, t1) of them (multiples of 32 but for the end), the
    // result then going to partial `part` of the workspace (kPrefillDirect: straight to the output).
    uint32_t t0, t1;
    uint32_t part;
    uint32_t pad_;
};
static constexpr uint32_t kPrefillDirect = 0xffffffffu;
inline uint32_t prefill_group_columns(uint32_t g) { // 1, 2, 4, 8 or 16
    uint32_t gl = 1;
    while (gl < g)
        gl *= 2;
    return gl;
}
static_assert(sizeof(PrefillRec) == 80, "PrefillRec layout");

struct PrefillArgs {
    const unsigned char *pool_base;
    uint32_t log2_page;
    const int32_t *page_table;
    const uint16_t *q; // bf16
    float *out;
    const PrefillRec *recs;
    const uint32_t *bad; // null, or the flag of the page-table check: set = leave at once
    const unsigned char *v16; // one-part weights only: the workspace that holds the V rows as fp16
    float *partials;          // results of workgroups that walk a stretch of their tokens (see prefill_part_floats)
};
// One partial: kPrefillCols columns x head_dim accumulators (not yet divided by the sum of weights), then the columns'
// (reference point, sum of weights) pairs; every slot has the size the larger head_dim needs.
static constexpr uint32_t kPrefillPartFloats = 128u * (128u + 2u);
static constexpr uint32_t kPrefillMinStretch = 1024; // tokens: a shorter stretch is not worth a partial and a merge
static constexpr uint32_t kPrefillMaxParts = 2048;   // partial slots a call may use (about 136 MB of workspace)

// Merge of the partials of one tile of query rows that was walked in stretches: n_parts partials from slot part0 on.
struct PrefillMergeRec {
    uint64_t out_off;
    uint32_t part0, n_parts;
    uint32_t q_len, r0;
    uint32_t g; // as PrefillRec::g
    uint32_t n_q, kvh, d;
    uint32_t pad_[2];
};
static_assert(sizeof(PrefillMergeRec) == 48, "PrefillMergeRec layout");

// Work item of the pass that copies V rows out of the pool as fp16 (one-part weights): tokens [t0, t1) of one
// request, all kv heads; head h's row of token t goes to v16_off + (h ctx_len + t) * 2 head_dim.
struct V16Rec {
    uint64_t table_off;
    uint64_t v16_off;
    uint32_t t0, t1;
    uint32_t ctx_len;
    uint32_t token_bytes;
    uint32_t n_kv, d;
    uint32_t pad_[2];
};
static_assert(sizeof(V16Rec) == 48, "V16Rec layout");
static constexpr uint32_t kPrefillBlocks = 2; // 16-column blocks per wave
static constexpr uint32_t kPrefillWaves = 4;  // waves per workgroup (8 was measured: slower, one workgroup per CU)
static constexpr uint32_t kPrefillCols = 16 * kPrefillBlocks * kPrefillWaves; // (query row, query head) pairs per workgroup

struct GatherRec { // tokens [t0, t1) of one request
    uint64_t table_off;
    uint64_t kv_off;  // element offset of token `flat_t0` in the contiguous arrays
    uint32_t t0, t1;
    uint32_t cls;
    uint32_t flat_t0; // first token the contiguous arrays hold (0, or the first token of a chunk)
};

// ---- kernel launchers (ukv_decode.hip, ukv_prefill.hip, ukv_copy.hip) ----
int decode_resident_workgroups(uint32_t block_threads); // spans of the planner's first round: one per compute unit; 0 on failure
// workgroups to launch for n_spans spans: one per place the device offers the kernel instantiation, at most n_spans
uint32_t decode_grid(uint32_t n_spans, uint32_t block_threads, uint32_t kinds, uint32_t first_round);
hipError_t launch_stage_copy(void *dst, const void *src_mapped, size_t bytes, int32_t *page_table,
                             const uint64_t *patch_entry, const int32_t *patch_page, uint32_t n_patches,
                             hipStream_t s);
hipError_t launch_decode(const DecodeArgs &a, const StepPages *sp, uint32_t grid, uint32_t block_threads,
                         uint32_t kinds, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1);
hipError_t launch_reduce(const ReduceRec *recs, uint32_t n_recs, uint32_t n_many, uint32_t max_heads, uint32_t max_units,
                         const float *partials, float *out, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1);
hipError_t launch_reduce_counted(const ReduceRec *many, const uint32_t *n_many_dev, uint32_t many_bound,
                                 const ReduceRec *few, const uint32_t *n_few_dev, uint32_t few_bound, uint32_t max_heads,
                                 uint32_t max_units, const float *partials, float *out, hipStream_t s);
hipError_t launch_validate(const int32_t *page_table, const ValRec *recs, uint32_t n, uint64_t n_pages,
                           ValReport *report, uint32_t *flag_dev, hipStream_t s);
hipError_t launch_patch(int32_t *page_table, const uint64_t *entry, const int32_t *page, uint32_t n,
                        hipStream_t s);
hipError_t launch_append(unsigned char *pool_base, uint32_t log2_page, int32_t *page_table, const AppendRec *recs,
                         uint32_t n, const ClassRec *classes, const void *new_k, const void *new_v,
                         const uint64_t *patch_entry, const int32_t *patch_page, uint32_t n_patches,
                         const uint32_t *bad, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1);
hipError_t launch_prefill_merge(const PrefillMergeRec *recs, uint32_t n_recs, const float *partials, float *out,
                                const uint32_t *bad, hipStream_t s);
hipError_t launch_v16(const unsigned char *pool_base, uint32_t log2_page, const int32_t *page_table, const V16Rec *recs,
                      uint32_t n_recs, unsigned char *v16, const uint32_t *bad, hipStream_t s);
// parts: 2 = weights as two bf16 parts, 1 = as one fp16 part (a.v16 and the records' v16_off are then set)
hipError_t launch_prefill(const PrefillArgs &a, uint32_t n_recs, uint32_t head_dim, uint32_t parts, hipStream_t s, hipEvent_t ev0,
                          hipEvent_t ev1);
hipError_t launch_copy_tokens(bool to_pool, unsigned char *pool_base, uint32_t log2_page, const int32_t *page_table,
                              const GatherRec *recs, uint32_t n, const ClassRec *classes, void *k_io, void *v_io,
                              const uint32_t *bad, hipStream_t s);

// ---- host planner (ukv_planner.cpp) ----
struct Plan {
    std::vector<SeqRec> seqs;
    std::vector<Item> items;
    std::vector<uint32_t> span_first;
    std::vector<ReduceRec> reduce;   // sequences the second launch merges: those of many parts first
    uint32_t n_reduce_many = 0;      // how many of them have more than kReduceFewParts parts
    std::vector<uint32_t> item_span; // span index of each item (inspection only)
    std::vector<uint32_t> seq_req;   // request index of each sequence
    uint64_t partial_floats = 0;
    uint64_t kv_bytes = 0;
    uint32_t max_reduce_heads = 0;  // second launch, sequences of many parts: workgroups per sequence (query heads)
    uint32_t max_reduce_units = 0;  // sequences of few parts: waves per sequence (query heads, or kv heads on the matrix-core path)
};

struct Tunables {
    int64_t max_spans = 2048;
    int64_t min_span_bytes = 512 * 1024;
    bool min_span_auto = true; // until the caller sets it: small batches get smaller spans (see build_plan)
    int64_t block_threads = 512;
    int64_t heads_per_slice = 0;
    int64_t profile = 0;
    int64_t fused_merge = 1;
    int64_t slots = 512; // workgroups resident at once (refreshed from the device at the first launch)
    int64_t taper = 1;
    int64_t gqa_cost_pct = 150; // planner weight of a matrix-core (grouped-query) KV byte, percent
    int64_t prefill_xcd = 1;
    int64_t merge_acq_rel = 0;
    int64_t validate = 0; // check the page tables a call uses before its kernels run
    int64_t prefill_weights = 0; // 0 = chosen per call, 1 = one fp16 part, 2 = two bf16 parts
    int64_t prefill_form_used = 0; // what the last prefill call took
    int64_t prefill_partials_used = 0;
    int64_t replan_every = 64; // a kept plan is remade after its requests have grown by this many tokens
    bool slots_auto = true;
    bool grid_is_first_round = false; // launches of more spans than the device holds get `slots` workgroups (decode_grid)
};

void set_error(const std::string &msg);

// UKV_TRACE=1 in the environment: every compute call leaves one line on stderr when it returns --
//   ukv_trace call=<entry point> t_us=<host time since the first traced call> host_us=<time spent in the call>
//   status=ok|error key=value ...
// with the call's work-list figures (requests, KV bytes, spans, items, workgroups, ...).  Host side only; nothing is
// measured on the device (UKV_PARAM_PROFILE does that).  The line is built in a fixed buffer: tracing allocates nothing.
struct Trace {
    explicit Trace(const char *call);
    ~Trace();
    void add(const char *key, uint64_t value);
    Trace(const Trace &) = delete;
    Trace &operator=(const Trace &) = delete;

  private:
    const char *call_;
    bool on_;
    uint64_t t0_ns_, errors_at_start_;
    char kv_[384];
    size_t len_ = 0;
};

} // namespace ukv

// ---- the opaque pool object ----
struct ukv_pool {
    unsigned char *base = nullptr;
    uint64_t n_pages = 0;
    uint32_t page_bytes = 0, log2_page = 0;
    uint32_t n_services = 0;
    ukv_service_t services[UKV_MAX_SERVICES];
    ukv::ClassTable classes;
    ukv::Tunables tun;

    uint64_t tun_epoch = 0; // bumped by every ukv_set_param that changes how a launch is planned
    uint32_t kinds = 0; // bit k: a service of kind k exists (chooses the decode kernel instantiation)

    // LIFO free list
    std::vector<int32_t> free_stack;
    std::vector<uint8_t> is_free;

    // pinned, device-mapped staging ring (created lazily on the first compute call)
    struct Stage {
        void *host = nullptr;
        void *mapped = nullptr; // device-side address of the same pinned memory
        size_t cap = 0;
        hipEvent_t ev = nullptr;
        bool pending = false;
    };
    static constexpr int kStages = 8;
    Stage stage[kStages];
    int next_stage = 0;

    ukv::Plan plan_scratch;
    ukv::ValReport *val_host = nullptr; // pinned; val_dev is the device's address of the same memory
    ukv::ValReport *val_dev = nullptr;
    uint32_t *val_flag = nullptr; // device memory (256 bytes, allocated when the check is first used): set = leave
    std::vector<std::pair<uint64_t, int32_t>> patch_scratch; // ukv_append: the call's table patches, sorted by entry
    std::vector<ukv::GatherRec> chunk_scratch;               // gather / scatter: the call's chunk records

    // profiling
    struct EvPair {
        hipEvent_t a, b;
        int which;
    };
    std::vector<EvPair> ev_used, ev_free;
    uint64_t prof_seq[4] = {0, 0, 0, 0}; // launches seen per kind (decode, reduce, append, prefill)
};

namespace ukv {
int derive_classes(ukv_pool *p);
int build_plan(const ukv_pool *p, const ukv_batch_t *b, Plan &plan);
uint64_t max_partial_floats(const ukv_pool *p, uint32_t n_requests);
} // namespace ukv
