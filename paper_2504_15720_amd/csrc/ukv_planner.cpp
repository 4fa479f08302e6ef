// Host planner for the split-KV decode launch: cuts a mixed-service batch into work items of
// (request, head-slice, token range) and groups them into equal-cost spans, one per workgroup.
// The decode phase reads every cached K/V byte once per step (section 2.1), so cost is counted
// in KV bytes; long-tailed context lengths are balanced by cutting at token granularity.
#include <algorithm>

#include "ukv_internal.h"

namespace ukv {

static constexpr uint64_t kMinItemTokens = 16;
static constexpr uint64_t kDefaultTaperPct = 88;

static uint32_t spans_bound(const ukv_pool *p) { return (uint32_t)(2 * p->tun.max_spans + 2); }

uint64_t max_partial_floats(const ukv_pool *p, uint32_t /*n_requests*/) {
    uint32_t stride = 0;
    for (uint32_t s = 0; s < p->n_services; ++s)
        stride = std::max(stride, part_stride_of(p->classes.c[s]));
    // every span boundary cuts at most one sequence, adding at most two partials
    return (uint64_t)2 * spans_bound(p) * stride;
}

int build_plan(const ukv_pool *p, const ukv_batch_t *b, Plan &plan) {
    if (!p || !b) {
        set_error("null pool or batch");
        return UKV_EINVAL;
    }
    const uint32_t n = b->n_requests;
    if (n && (!b->service_id || !b->ctx_len || !b->table_off || !b->q_off || !b->out_off)) {
        set_error("batch host arrays must be non-null");
        return UKV_EINVAL;
    }
    plan.seqs.clear();
    plan.items.clear();
    plan.span_first.clear();
    plan.reduce.clear();
    plan.item_span.clear();
    plan.seq_req.clear();
    plan.partial_floats = 0;
    plan.kv_bytes = 0;
    plan.max_reduce_units = 0;
    plan.max_reduce_heads = 0;
    plan.n_reduce_many = 0;
    // planner cost of one token of one head-slice: its KV bytes, weighted by the kernel kind
    auto token_cost = [&](const ClassRec &c) {
        const uint64_t bytes = (uint64_t)c.hs * c.row_bytes;
        return kind_is_gqa(c.kind) ? bytes * (uint64_t)p->tun.gqa_cost_pct / 100 : bytes;
    };
    uint64_t total_cost = 0;
    for (uint32_t i = 0; i < n; ++i) {
        const uint32_t cls = b->service_id[i];
        if (cls >= p->n_services) {
            set_error("service_id out of range");
            return UKV_EINVAL;
        }
        if ((b->q_off[i] & 7) || (b->out_off[i] & 3)) {
            set_error("q_off must be a multiple of 8 elements and out_off of 4");
            return UKV_EINVAL;
        }
        const ClassRec &c = p->classes.c[cls];
        const uint64_t ctx = b->ctx_len[i];
        if (ukv_pages_for_tokens(p, cls, ctx) > p->n_pages) {
            set_error("ctx_len exceeds what the pool can hold");
            return UKV_EINVAL;
        }
        plan.kv_bytes += ctx * c.token_bytes;
        for (uint32_t h0 = 0; h0 < c.n_kv; h0 += c.hs) {
            SeqRec s{};
            s.table_off = b->table_off[i];
            s.q_off = b->q_off[i];
            s.out_off = b->out_off[i];
            s.ctx_len = (uint32_t)ctx;
            s.cls = cls;
            s.head0 = h0;
            s.req = i;
            s.part_stride = part_stride_of(c);
            plan.seqs.push_back(s);
            plan.seq_req.push_back(i);
            total_cost += kItemOverheadBytes + ctx * token_cost(c);
        }
    }
    if (plan.seqs.empty()) {
        plan.span_first.push_back(0);
        return UKV_OK;
    }
    {
        // Longest sequences first: they are cut into the most parts, and their merge should run
        // while other workgroups still have work, not at the tail of the launch.  Stable, so the
        // slices of one request stay adjacent (they read the same pages).
        std::vector<uint32_t> order(plan.seqs.size());
        for (uint32_t k = 0; k < order.size(); ++k)
            order[k] = k;
        auto cost_of = [&](uint32_t k) {
            const ClassRec &c = p->classes.c[plan.seqs[k].cls];
            return (uint64_t)plan.seqs[k].ctx_len * token_cost(c);
        };
        std::stable_sort(order.begin(), order.end(), [&](uint32_t x, uint32_t y) { return cost_of(x) > cost_of(y); });
        static thread_local std::vector<SeqRec> seqs;
        static thread_local std::vector<uint32_t> req;
        seqs.resize(order.size());
        req.resize(order.size());
        for (uint32_t k = 0; k < order.size(); ++k) {
            seqs[k] = plan.seqs[order[k]];
            req[k] = plan.seq_req[order[k]];
        }
        plan.seqs.swap(seqs);
        plan.seq_req.swap(req);
    }

    // Span sizes.  Workgroups are dispatched in order onto `slots` resident positions, so equal
    // spans would leave the last round partly empty.  With tapering, each batch of `slots` spans
    // takes a fixed share of the remaining cost (factoring self-scheduling): rounds shrink
    // geometrically down to min_span_bytes and the tail of the launch is one small round.  A large
    // share keeps the number of cuts (each costs an item start and a partial to merge) low; what
    // the first round's uneven finish leaves is evened out by the small rounds after it.
    std::vector<uint64_t> targets;
    {
        const uint64_t max_spans = (uint64_t)p->tun.max_spans;
        const uint64_t slots = (uint64_t)std::max<int64_t>(1, p->tun.slots);
        // A batch too small to give every resident workgroup min_span_bytes is latency-bound, not
        // bandwidth-bound: it is cut finer (down to 64 KiB a span), so that more CUs share the tokens of each
        // request (8 requests of a few hundred tokens: 12 -> 118 workgroups, 19 -> 12 us).
        uint64_t min_span = (uint64_t)p->tun.min_span_bytes;
        if (p->tun.min_span_auto)
            min_span = std::max<uint64_t>(std::min<uint64_t>(min_span, total_cost / slots), kSmallBatchSpanBytes);
        if (!p->tun.taper) {
            uint64_t n = std::max<uint64_t>(1, std::min<uint64_t>(total_cost / min_span, max_spans));
            targets.assign(1, (total_cost + n - 1) / n);
        } else {
            uint64_t R = total_cost;
            const uint64_t pct = p->tun.taper == 1 ? kDefaultTaperPct : (uint64_t)p->tun.taper;
            // Less than two rounds of min_span spans in all: one round of equal spans.  (Tapered, the second round
            // would be a few spans of min_span bytes that take almost as long as the first.)
            if (R <= 2 * slots * min_span && slots <= max_spans) {
                const uint64_t c = std::max<uint64_t>(min_span, (R + slots - 1) / slots);
                targets.assign((size_t)((R + c - 1) / c), c);
                R = 0;
            }
            while (R > 0 && targets.size() < max_spans) {
                const uint64_t c = std::max<uint64_t>(min_span, R * pct / (100 * slots));
                uint64_t batch = std::min<uint64_t>(slots, (R + c - 1) / c);
                batch = std::min<uint64_t>(batch, max_spans - targets.size());
                targets.insert(targets.end(), batch, c);
                R -= std::min<uint64_t>(R, batch * c);
            }
            if (R > 0) { // span budget exhausted: spread what is left over the last batch
                const uint64_t tail = std::min<uint64_t>(slots, targets.size());
                for (uint64_t j = targets.size() - tail; j < targets.size(); ++j)
                    targets[j] += (R + tail - 1) / tail;
            }
        }
    }
    uint64_t C = targets[0];

    std::vector<uint32_t> seq_first_item(plan.seqs.size() + 1, 0);
    plan.span_first.push_back(0);
    int64_t fill = 0;
    auto close_span = [&](bool carry) {
        if (plan.span_first.back() != plan.items.size())
            plan.span_first.push_back((uint32_t)plan.items.size());
        fill = carry ? std::max<int64_t>(0, fill - (int64_t)C) : 0;
        C = targets[std::min<size_t>(plan.span_first.size() - 1, targets.size() - 1)];
        // The workspace is sized for 2 * max_spans + 2 spans.  Spans can outnumber the targets (an item's overhead
        // is not part of the budget); should they get that far, everything left goes into one last span, uncut.
        if (plan.span_first.size() + 1 >= spans_bound(p)) {
            C = UINT64_MAX / 4;
            fill = 0;
        }
    };
    for (uint32_t k = 0; k < plan.seqs.size(); ++k) {
        const SeqRec &s = plan.seqs[k];
        const ClassRec &c = p->classes.c[s.cls];
        const uint64_t cost = token_cost(c);
        seq_first_item[k] = (uint32_t)plan.items.size();
        uint64_t t = 0, rem = s.ctx_len;
        if (rem == 0) {
            plan.items.push_back(Item{k, 0, 0, kDirect});
            plan.item_span.push_back((uint32_t)plan.span_first.size() - 1);
            fill += (int64_t)kItemOverheadBytes;
            if (fill >= (int64_t)C)
                close_span(true);
            continue;
        }
        while (rem > 0) {
            const int64_t avail = (int64_t)C - fill - (int64_t)kItemOverheadBytes;
            if (fill > 0 && avail < (int64_t)(std::min<uint64_t>(kMinItemTokens, rem) * cost)) {
                close_span(false); // too little room left: start the next span instead of a sliver
                continue;
            }
            uint64_t take = avail > 0 ? (uint64_t)avail / cost : 0;
            take = std::max<uint64_t>(take, std::min<uint64_t>(kMinItemTokens, rem)); // also where a span is smaller than an item's overhead
            if (take >= rem || rem - take < kMinItemTokens)
                take = rem;
            plan.items.push_back(Item{k, (uint32_t)t, (uint32_t)(t + take), 0});
            plan.item_span.push_back((uint32_t)plan.span_first.size() - 1);
            fill += (int64_t)(kItemOverheadBytes + take * cost);
            t += take;
            rem -= take;
            if (fill >= (int64_t)C)
                close_span(true);
        }
    }
    seq_first_item[plan.seqs.size()] = (uint32_t)plan.items.size();
    if (plan.span_first.back() != plan.items.size())
        plan.span_first.push_back((uint32_t)plan.items.size());

    // partial slots and the merge list
    for (uint32_t k = 0; k < plan.seqs.size(); ++k) {
        SeqRec &s = plan.seqs[k];
        const ClassRec &c = p->classes.c[s.cls];
        const uint32_t i0 = seq_first_item[k], i1 = seq_first_item[k + 1];
        s.n_parts = i1 - i0;
        if (s.n_parts <= 1) {
            plan.items[i0].part = kDirect;
            continue;
        }
        s.part_off = plan.partial_floats;
        for (uint32_t it = i0; it < i1; ++it)
            plan.items[it].part = it - i0;
        plan.partial_floats += (uint64_t)s.n_parts * s.part_stride;
        if (p->tun.fused_merge && merges_in_launch(s.n_parts, s.part_stride))
            continue; // merged inside the decode launch by the workgroup that finishes it last
        ReduceRec r{};
        r.part_off = s.part_off;
        r.out_off = s.out_off + (uint64_t)s.head0 * c.g * c.d;
        r.n_parts = s.n_parts;
        r.part_stride = s.part_stride;
        r.n_heads = c.hs * c.g;
        r.d = c.d;
        r.layout_g = kind_is_gqa(c.kind) ? c.g : 0;
        plan.reduce.push_back(r);
        plan.max_reduce_heads = std::max(plan.max_reduce_heads, r.n_heads);
        plan.max_reduce_units = std::max(plan.max_reduce_units, r.layout_g ? r.n_heads / r.layout_g : r.n_heads);
    }
    const auto many = std::stable_partition(plan.reduce.begin(), plan.reduce.end(),
                                            [](const ReduceRec &r) {
                                                return r.n_parts > kReduceFewParts || !reduce_few_takes(r.layout_g, r.d);
                                            });
    plan.n_reduce_many = (uint32_t)(many - plan.reduce.begin());
    return UKV_OK;
}

} // namespace ukv
