// Decode attention over the unified pool: decode_kernel (split-KV decode over a mixed-service batch in
// one launch, fused merge of split partials, fused append) and reduce_few_kernel / reduce_many_kernel (the merge as a second
// launch).
//
// Decode is bound by HBM: every cached K/V byte is read once per step (decode phase, section
// 2.1; merged blocks are chosen for read locality, section 4.4).  The design therefore keeps
// every load a fully used 128-bit access: a row (one kv head of one token, K[d] | V[d]) is
// read by d/8 adjacent lanes, 16 bytes each, so one wave instruction covers whole 128-byte
// lines, and the lanes of a workgroup cover `hs` consecutive heads of `ti` consecutive
// tokens, i.e. contiguous stretches of the request's byte stream inside 16 KiB pages.
#include "ukv_device.h"

namespace ukv {

static constexpr int kTabWindow = 2048; // page-table entries staged in LDS at a time

// Workgroup state in LDS.  The kernel body only picks items and publishes them in s_ctx; the
// per-kind item functions take their (workgroup-uniform) inputs from there and move them to
// SGPRs, so that nothing of one item stays live in registers across the next.
static constexpr int kMaxBlock = 512;
struct ItemCtx {
    DecodeArgs a;
    alignas(16) Item it; // it, s, c: the item's record as it lies in memory (ItemRec), written in 16-byte pieces
    SeqRec s;
    ClassRec c;
};
static_assert(offsetof(ItemCtx, s) == offsetof(ItemCtx, it) + offsetof(ItemRec, s) &&
                  offsetof(ItemCtx, c) == offsetof(ItemCtx, it) + offsetof(ItemRec, c),
              "ItemCtx mirrors ItemRec");
__shared__ int32_t s_tab[kTabWindow];                                  // page-table window
__shared__ __align__(16) float s_mbuf[kMaxBlock * 8 + (kMaxBlock / 8) * 2]; // merge buffer
__shared__ __align__(16) ItemCtx s_ctx;

// Fused append: an item appends when the launch carries new tokens and it ends at the request's
// last token.  That token is then not read from the pool: lanes take its row from new_k/new_v,
// store it into the request's page and use it from registers, so the store side of the step
// costs no launch and no wait.  Workgroup-uniform.
__device__ __forceinline__ bool item_appends(const SeqRec &s, const Item &it) {
    return uni(reinterpret_cast<uint64_t>(s_ctx.a.new_k)) != 0 && s.ctx_len > 0 && it.t1 == s.ctx_len;
}
// new_k / new_v rows of kv head kvh of the item's request (element pointers)
__device__ __forceinline__ void new_token_rows(uint32_t kvh, uint32_t D, const uint16_t *&nk, const uint16_t *&nv) {
    const uint64_t e0 = uni(s_ctx.s.new_off) + (uint64_t)kvh * D;
    nk = reinterpret_cast<const uint16_t *>(uni(reinterpret_cast<uint64_t>(s_ctx.a.new_k))) + e0;
    nv = reinterpret_cast<const uint16_t *>(uni(reinterpret_cast<uint64_t>(s_ctx.a.new_v))) + e0;
}

__device__ __forceinline__ DecodeArgs ctx_args() {
    DecodeArgs a;
    a.pool_base = reinterpret_cast<const unsigned char *>(uni(reinterpret_cast<uint64_t>(s_ctx.a.pool_base)));
    a.log2_page = uni(s_ctx.a.log2_page);
    a.page_table = reinterpret_cast<const int32_t *>(uni(reinterpret_cast<uint64_t>(s_ctx.a.page_table)));
    a.q = reinterpret_cast<const void *>(uni(reinterpret_cast<uint64_t>(s_ctx.a.q)));
    a.out = reinterpret_cast<float *>(uni(reinterpret_cast<uint64_t>(s_ctx.a.out)));
    a.recs = nullptr;
    a.span_first = nullptr;
    a.partials = reinterpret_cast<float *>(uni(reinterpret_cast<uint64_t>(s_ctx.a.partials)));
    a.counters = reinterpret_cast<uint32_t *>(uni(reinterpret_cast<uint64_t>(s_ctx.a.counters)));
    a.merge_acq_rel = uni(s_ctx.a.merge_acq_rel);
    a.new_k = nullptr; // the fused-append inputs are fetched where they are used (new_token_rows)
    a.new_v = nullptr;
    a.delta = 0;       // already applied to the item and the sequence in LDS
    a.bad = nullptr;
    return a;
}
__device__ __forceinline__ SeqRec ctx_seq() {
    SeqRec s;
    s.table_off = uni(s_ctx.s.table_off);
    s.q_off = uni(s_ctx.s.q_off);
    s.out_off = uni(s_ctx.s.out_off);
    s.part_off = uni(s_ctx.s.part_off);
    s.new_off = 0;
    s.ctx_len = uni(s_ctx.s.ctx_len);
    s.cls = uni(s_ctx.s.cls);
    s.head0 = uni(s_ctx.s.head0);
    s.n_parts = uni(s_ctx.s.n_parts);
    s.part_stride = uni(s_ctx.s.part_stride);
    s.req = 0; // read from LDS where it is needed (step_entries)
    return s;
}
__device__ __forceinline__ ClassRec ctx_class() {
    ClassRec c;
    c.n_q = uni(s_ctx.c.n_q);
    c.n_kv = uni(s_ctx.c.n_kv);
    c.d = uni(s_ctx.c.d);
    c.g = uni(s_ctx.c.g);
    c.row_bytes = uni(s_ctx.c.row_bytes);
    c.token_bytes = uni(s_ctx.c.token_bytes);
    c.hs = uni(s_ctx.c.hs);
    c.ti = uni(s_ctx.c.ti);
    c.scale_log2e = uni(s_ctx.c.scale_log2e);
    c.kind = uni(s_ctx.c.kind);
    return c;
}
__device__ __forceinline__ Item ctx_item() {
    Item it;
    it.seq = uni(s_ctx.it.seq);
    it.t0 = uni(s_ctx.it.t0);
    it.t1 = uni(s_ctx.it.t1);
    it.part = uni(s_ctx.it.part);
    return it;
}

// Online-softmax update of one kv head's G query heads with U tokens.  MASKED: token u only
// counts if bit u of `valid` is set (bit 0 always is: the running maximum stays finite).
template <int G, int U, int LPR, bool MASKED = false>
__device__ __forceinline__ void update(const float (&qf)[G][8], const uint4 (&kr)[U], const uint4 (&vr)[U],
                                       float (&m)[G], float (&l)[G], float (&acc)[G][8], uint32_t valid = ~0u) {
    float kf[U][8], vf[U][8];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        unpack8(kr[u], kf[u]);
        unpack8(vr[u], vf[u]);
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
        float sc[U];
        float mx = m[g];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float d = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e)
                d = fmaf(qf[g][e], kf[u][e], d);
            sc[u] = row_sum<LPR>(d);
            if (MASKED && !((valid >> u) & 1u))
                sc[u] = -INFINITY;
            mx = fmaxf(mx, sc[u]);
        }
        const float alpha = fast_exp2(m[g] - mx); // m = -inf on the first batch gives 0
        float psum = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e)
            acc[g][e] *= alpha;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float p = fast_exp2(sc[u] - mx);
            psum += p;
#pragma unroll
            for (int e = 0; e < 8; ++e)
                acc[g][e] = fmaf(p, vf[u][e], acc[g][e]);
        }
        l[g] = fmaf(l[g], alpha, psum);
        m[g] = mx;
    }
}

// Partials cross workgroups (and therefore XCDs, each with its own L2) inside one launch.  They
// are written and read with device-scope relaxed atomics, which go through to the point of
// coherence, so no cache-wide write-back/invalidate fence is needed: the writer waits for its
// stores to complete before it counts the item, the reader starts after it has seen the count.
__device__ __forceinline__ void st_part2(float *p, float a, float b) {
    const uint64_t v = ((uint64_t)__float_as_uint(b) << 32) | __float_as_uint(a);
    __hip_atomic_store(as_global(reinterpret_cast<uint64_t *>(p)), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 ld_part2(const float *p) {
    const uint64_t v = __hip_atomic_load(as_global(reinterpret_cast<const uint64_t *>(p)), __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_AGENT);
    return make_float2(__uint_as_float((uint32_t)v), __uint_as_float((uint32_t)(v >> 32)));
}

// Layout of the accumulators inside one partial.  It follows the writers' register layouts so
// that every 64-bit store instruction of a wave covers contiguous memory (whole 128-byte lines):
//   layout_g == 0 (ALU path): per query head D floats; lane lir of the row group holds columns
//     8*lir + 2k + {0,1} and stores pair k at  hq*D + k*(D/4) + 2*lir.
//   layout_g == G (matrix-core path): per kv head G*D floats; lane (j, q), q < D/32, holds columns
//     32q + 8r + 2pp + {0,1} of head j and stores pair (r, pp) at  hh*G*D + ((4r+pp)*(D/32)*G + q*G + j)*2.
// Returns the float offset of the pair holding columns 4*c4 + 2h, 4*c4 + 2h + 1 of query head hq.
__device__ __forceinline__ uint32_t part_pair_off(uint32_t layout_g, uint32_t D, uint32_t hq, uint32_t c4,
                                                  uint32_t h) {
    if (layout_g == 0) {
        const uint32_t lir = c4 >> 1, k = ((c4 & 1) << 1) + h;
        return hq * D + k * (D >> 2) + 2 * lir;
    }
    const uint32_t G = layout_g, hh = hq / G, j = hq % G;
    const uint32_t q = c4 >> 3, r = (c4 & 7) >> 1, pp = ((c4 & 1) << 1) + h;
    return hh * (G * D) + (((r << 2) + pp) * ((D >> 5) * G) + q * G + j) * 2;
}

// The inverse: float e of a partial's accumulators, in memory order, is column `col` of query head `head` (of
// the sequence's n_heads).  Readers walk partials in memory order, so that a wave's load covers whole lines.
struct AccElem {
    uint32_t head, col;
};
__device__ __forceinline__ AccElem acc_elem(uint32_t layout_g, uint32_t D, uint32_t e) {
    if (layout_g == 0) {
        const uint32_t q4 = D >> 2, o = e % D, k = o / q4, rem = o % q4;
        return AccElem{e / D, 8 * (rem >> 1) + 2 * k + (rem & 1)};
    }
    const uint32_t G = layout_g, hh = e / (G * D), t = (e % (G * D)) >> 1, nq = D >> 5;
    const uint32_t j = t % G, t2 = t / G, q = t2 % nq, t3 = t2 / nq;
    return AccElem{hh * G + j, 32 * q + 8 * (t3 >> 2) + 2 * (t3 & 3) + (e & 1)};
}

// Merge of the partials of one cut sequence (all its query heads), executed by the workgroup
// that finished the sequence's last item:  with M = max_c m_c,
//   out = sum_c acc_c 2^(m_c - M) / sum_c l_c 2^(m_c - M).
// The (m, l) pairs are staged in LDS a chunk of parts at a time, so that each output element
// only streams its accumulators, several parts in flight; chunks combine by the same rule.
static constexpr uint32_t kMergeBatch = 8; // parts whose accumulators are in flight per thread

// One pair of adjacent output columns of query head hq (the two floats at xa in every part) from the parts
// [c0, c0+nc) whose (m, l) pairs are staged in lds[2*(c*n_heads + hq)]; (Mr, Lr, o) carry the running maximum,
// sum and accumulator across chunks of parts.
__device__ __forceinline__ void merge_unit(const float *xa, uint32_t part_stride, const float *lds, uint32_t n_heads,
                                           uint32_t nc, uint32_t hq, float &Mr, float &Lr, float2 &o) {
    float Mc = Mr;
    for (uint32_t c = 0; c < nc; ++c)
        Mc = fmaxf(Mc, lds[2 * (c * n_heads + hq)]);
    if (Mc == -INFINITY)
        return;
    const float f = fast_exp2(Mr - Mc);
    Lr *= f;
    o.x *= f;
    o.y *= f;
    Mr = Mc;
    for (uint32_t c = 0; c < nc; c += kMergeBatch) {
        float2 x[kMergeBatch];
#pragma unroll
        for (uint32_t k = 0; k < kMergeBatch; ++k)
            x[k] = ld_part2(xa + (uint64_t)min(c + k, nc - 1) * part_stride); // clamp: a repeated load, skipped below
#pragma unroll
        for (uint32_t k = 0; k < kMergeBatch; ++k) {
            if (c + k >= nc)
                break;
            const uint32_t i = (c + k) * n_heads + hq;
            const float w = fast_exp2(lds[2 * i] - Mr);
            Lr = fmaf(lds[2 * i + 1], w, Lr);
            o.x = fmaf(x[k].x, w, o.x);
            o.y = fmaf(x[k].y, w, o.y);
        }
    }
}

// The units are the pairs of a partial in memory order (adjacent lanes read adjacent 8 bytes); only the output
// stores are scattered.
template <int NT>
__device__ void merge_parts(const DecodeArgs &a, const SeqRec &s, uint32_t n_heads, uint32_t D, uint32_t q_head0,
                            uint32_t layout_g, float *lds) {
    constexpr uint32_t kPairs = NT * 4; // (m, l) pairs that fit the LDS buffer
    const float *base = a.partials + s.part_off;
    const float *ml_base = base + (uint64_t)n_heads * D;
    const uint32_t units = n_heads * D / 2;
    const uint32_t cmax = kPairs / n_heads;
    auto stage_ml = [&](uint32_t c0, uint32_t nc) {
        __syncthreads();
        for (uint32_t i = threadIdx.x; i < nc * n_heads; i += NT) {
            const uint32_t c = i / n_heads, h = i % n_heads;
            const float2 p = ld_part2(ml_base + (uint64_t)(c0 + c) * s.part_stride + h * 2);
            lds[2 * i] = p.y > 0.f ? p.x : -INFINITY; // an empty part carries no weight
            lds[2 * i + 1] = p.y;
        }
        __syncthreads();
    };
    auto write_out = [&](const AccElem &el, float Lr, const float2 &o) {
        const float inv = Lr > 0.f ? 1.f / Lr : 0.f;
        st_g8(a.out + s.out_off + (uint64_t)(q_head0 + el.head) * D + el.col, o.x * inv, o.y * inv);
    };
    if (s.n_parts <= cmax) { // usual case: all (m, l) pairs fit, staged once for every output element
        stage_ml(0, s.n_parts);
        for (uint32_t u = threadIdx.x; u < units; u += NT) {
            const AccElem el = acc_elem(layout_g, D, 2 * u);
            float Mr = -INFINITY, Lr = 0.f;
            float2 o = make_float2(0.f, 0.f);
            merge_unit(base + 2 * u, s.part_stride, lds, n_heads, s.n_parts, el.head, Mr, Lr, o);
            write_out(el, Lr, o);
        }
        return;
    }
    for (uint32_t u0 = 0; u0 < units; u0 += NT) { // workgroup-uniform
        const uint32_t u = u0 + threadIdx.x;
        const bool act = u < units;
        const AccElem el = acc_elem(layout_g, D, act ? 2 * u : 0);
        float Mr = -INFINITY, Lr = 0.f;
        float2 o = make_float2(0.f, 0.f);
        for (uint32_t c0 = 0; c0 < s.n_parts; c0 += cmax) {
            const uint32_t nc = min(cmax, s.n_parts - c0);
            stage_ml(c0, nc);
            if (act)
                merge_unit(base + (uint64_t)c0 * s.part_stride + 2 * u, s.part_stride, lds, n_heads, nc, el.head, Mr, Lr, o);
        }
        if (act)
            write_out(el, Lr, o);
    }
}

// After an item's partials are written: count the item, and if it was the sequence's last one,
// merge.  Workgroup-uniform; no-op for whole-sequence items and for the two-launch variant.
template <int NT>
__device__ __forceinline__ void finish_item(const DecodeArgs &a, const SeqRec &s, const Item &it, uint32_t n_heads,
                                            uint32_t D, uint32_t q_head0, uint32_t layout_g, int32_t *tab,
                                            float *mbuf) {
    if (it.part == kDirect || a.counters == nullptr || !merges_in_launch(s.n_parts, s.part_stride))
        return;
    // Publication of the partial.  Every access to a partial or a counter is an agent-scope atomic, which the
    // hardware performs at the level that is coherent across XCDs (cache policy sc1: stores are written through to
    // it and acknowledged from there, loads are served from it).  (1) Each wave waits for the acknowledgement of its
    // own partial stores (vmcnt(0)); (2) the workgroup barrier, whose release/acquire fences also keep the compiler
    // from moving the stores below it or the increment above it; (3) one lane counts the item; (4) whoever reads
    // n_parts - 1 knows that every other part was counted, hence acknowledged, before, and reads the partials with
    // agent-scope loads after the next barrier.  This is the instruction sequence of an agent-scope release on the
    // increment and acquire on the read, minus the write-back and invalidation of the whole L2 (buffer_wbl2 /
    // buffer_inv), which serve accesses that are not agent-scope atomics: there are none here.  In the language's
    // memory model, though, relaxed atomics plus a barrier promise no such ordering; merge_acq_rel makes the
    // increment an acquire-release at agent scope (measured: 4 to 8 % of the launch), for whoever prefers the model's
    // word over the hardware's.
    __builtin_amdgcn_s_waitcnt(0x0F70); // vmcnt(0)
    __syncthreads();
    uint32_t *flag = reinterpret_cast<uint32_t *>(tab);
    if (threadIdx.x == 0)
        flag[0] = a.merge_acq_rel ? __hip_atomic_fetch_add(as_global(a.counters + it.seq), 1u, __ATOMIC_ACQ_REL,
                                                           __HIP_MEMORY_SCOPE_AGENT)
                                  : __hip_atomic_fetch_add(as_global(a.counters + it.seq), 1u, __ATOMIC_RELAXED,
                                                           __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (flag[0] == s.n_parts - 1) {
        if (threadIdx.x == 0) // the last one to count: nobody touches the counter again in this launch; a later
                              // launch that reuses the plan finds it at zero
            __hip_atomic_store(as_global(a.counters + it.seq), 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        merge_parts<NT>(a, s, n_heads, D, q_head0, layout_g, mbuf);
    }
}

// Page-table window of an item into LDS.  In a step whose new table entries ride in the kernel arguments, the
// entries the request gains in this step are taken from there (they are not in memory yet; only the items that hold
// the request's last token can meet them) and written to the table, for the launches to come.  Every head-slice
// writes the entries its own window covers: each new page holds bytes of the new token, so some slice covers it
// (slices that share a page store the same value).  Workgroup-uniform arguments; `new_n` == 0 otherwise.
template <int NT>
__device__ __forceinline__ void load_table_window(int32_t *tab, const DecodeArgs &a, const SeqRec &s, uint64_t s_lo,
                                                  uint32_t n_ent, const StepPages &sp, uint64_t new_lo, uint32_t new_n,
                                                  uint32_t new_first) {
    const int32_t *tp = a.page_table + s.table_off;
    for (uint32_t e = threadIdx.x; e < n_ent; e += NT) {
        const uint64_t ent = s_lo + e;
        int32_t pg;
        if (ent - new_lo < (uint64_t)new_n) {
            pg = sp.page[new_first + (uint32_t)(ent - new_lo)];
            as_global(const_cast<int32_t *>(tp))[ent] = pg;
        } else {
            pg = as_global(tp)[ent];
        }
        tab[e] = pg;
    }
}

// Which table entries of the item's request ride in the kernel arguments (see StepPages).
__device__ __forceinline__ void step_entries(bool appends, const StepPages &sp, const SeqRec &s, uint64_t T, uint32_t lg,
                                             uint64_t &new_lo, uint32_t &new_n, uint32_t &new_first) {
    new_lo = 0;
    new_n = 0;
    new_first = 0;
    if (appends && sp.n_req != 0) {
        const uint32_t r = uni(s_ctx.s.req);
        new_first = sp.first[r];
        new_n = (uint32_t)sp.first[r + 1] - new_first;
        new_lo = ((uint64_t)(s.ctx_len - 1) * T + ((1ull << lg) - 1)) >> lg;
    }
}

template <int D, int G, int NT>
__device__ __forceinline__ void process_item(const StepPages &sp) {
    const DecodeArgs a = ctx_args();
    const SeqRec s = ctx_seq();
    const ClassRec c = ctx_class();
    const Item it = ctx_item();
    int32_t *tab = s_tab;
    float *mbuf = s_mbuf;
    constexpr int LPR = D / 8;   // lanes per row
    constexpr int NG = NT / LPR; // row groups in the workgroup
    constexpr int U = 4;
    const int tid = threadIdx.x;
    const int lir = tid % LPR, grp = tid / LPR;
    const uint32_t HS = c.hs, TI = c.ti;
    const uint32_t hh = grp % HS, tl = grp / HS;
    const bool live = tl < TI;
    const uint32_t kvh = s.head0 + hh;
    const uint32_t lg = a.log2_page;
    const uint64_t page_mask = (1ull << lg) - 1;

    // q is only unpacked after the first page-table window is in LDS: its loads, the window's and
    // (fused append) the new token's are then in flight together, one round trip for all three.
    float qf[G][8];
    uint4 qraw[G];
    {
        const uint4 *qp = reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(a.q) + s.q_off +
                                                          (uint64_t)(kvh * G) * D + lir * 8);
#pragma unroll
        for (int g = 0; g < G; ++g)
            qraw[g] = ld_g16(qp + g * LPR);
    }
    float m[G], l[G], acc[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m[g] = -INFINITY;
        l[g] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e)
            acc[g][e] = 0.f;
    }

    const uint64_t T = c.token_bytes;
    const uint64_t row0 = (uint64_t)kvh * c.row_bytes + (uint64_t)lir * 16;
    const uint64_t slice_lo = (uint64_t)s.head0 * c.row_bytes;
    const uint64_t slice_hi = (uint64_t)(s.head0 + HS) * c.row_bytes;

    const bool appends = item_appends(s, it);
    const uint32_t t_pool = appends ? it.t1 - 1 : it.t1; // tokens below this are read from the pool
    uint64_t new_lo;
    uint32_t new_n, new_first;
    step_entries(appends, sp, s, T, lg, new_lo, new_n, new_first);
    uint4 nkr[1], nvr[1]; // the new token's K and V pieces of this lane (fused append)
    uint4 *new_dst = nullptr;
    uint32_t w0 = it.t0;
    while (w0 < it.t1) { // workgroup-uniform: one pass per page-table window
        const uint64_t s_lo = ((uint64_t)w0 * T + slice_lo) >> lg;
        const uint64_t lim = (s_lo + kTabWindow) << lg;
        const uint64_t tmax = (lim - slice_hi) / T; // last token whose slice ends inside the window
        const uint32_t w1 = (uint32_t)(tmax + 1 < (uint64_t)it.t1 ? tmax + 1 : (uint64_t)it.t1);
        const uint32_t n_ent = (uint32_t)((((uint64_t)(w1 - 1) * T + slice_hi - 1) >> lg) - s_lo) + 1;
        const uint32_t r1 = w1 < t_pool ? w1 : t_pool;
        // The new token is handled in the window that holds it, ahead of that window's pool tokens:
        // its loads are issued here, so that they are in flight together with the table window's.
        const bool new_here = appends && w1 == it.t1 && live && tl == 0;
        if (new_here) {
            const uint16_t *nk, *nv;
            new_token_rows(kvh, D, nk, nv);
            nkr[0] = ld_g16(nk + lir * 8);
            nvr[0] = ld_g16(nv + lir * 8);
        }
        if (w0 != it.t0)
            __syncthreads(); // later windows: every wave is done with the previous one (the first
                             // follows the workgroup barrier that published the item)
        load_table_window<NT>(tab, a, s, s_lo, n_ent, sp, new_lo, new_n, new_first);
        __syncthreads();
        if (w0 == it.t0) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                unpack8(qraw[g], qf[g]);
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    qf[g][e] *= c.scale_log2e;
            }
        }

        if (live) {
            auto row_ptr = [&](uint32_t t) -> const uint4 * {
                const uint64_t off = (uint64_t)t * T + row0;
                const int32_t pg = tab[(uint32_t)((off >> lg) - s_lo)];
                return reinterpret_cast<const uint4 *>(a.pool_base + ((uint64_t)(uint32_t)pg << lg) +
                                                       (off & page_mask));
            };
            if (new_here) { // into the softmax from registers; into the pool once the item's loads are done
                new_dst = const_cast<uint4 *>(row_ptr(it.t1 - 1));
                update<G, 1, LPR>(qf, nkr, nvr, m, l, acc);
            }
            uint32_t t = w0 + tl;
            for (; (uint64_t)t + (uint64_t)(U - 1) * TI < r1; t += U * TI) {
                uint4 kr[U], vr[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const uint4 *p = row_ptr(t + u * TI);
                    kr[u] = ld_kv(p);
                    vr[u] = ld_kv(p + LPR);
                }
                update<G, U, LPR>(qf, kr, vr, m, l, acc);
            }
            if (t < r1) { // the last, partly filled batch in one round trip: missing tokens are masked
                uint4 kr[U], vr[U];
                uint32_t valid = 0;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const bool ok = t + u * TI < r1;
                    valid |= (uint32_t)ok << u;
                    const uint4 *p = row_ptr(ok ? t + u * TI : t);
                    kr[u] = ld_kv(p);
                    vr[u] = ld_kv(p + LPR);
                }
                update<G, U, LPR, true>(qf, kr, vr, m, l, acc, valid);
            }
        }
        w0 = w1;
    }

    // merge the token lanes of each head (LDS), then write the final output or a partial
    float *accb = mbuf;               // [NG][LPR*8]
    float *mlb = mbuf + NG * LPR * 8; // [NG][2]
    const bool direct = it.part == kDirect;
    float *pbase = direct ? nullptr : a.partials + s.part_off + (uint64_t)it.part * s.part_stride;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        if (TI > 1) {
            __syncthreads();
            if (live && tl > 0) {
                float4 *dst = reinterpret_cast<float4 *>(accb + grp * (LPR * 8) + lir * 8);
                dst[0] = make_float4(acc[g][0], acc[g][1], acc[g][2], acc[g][3]);
                dst[1] = make_float4(acc[g][4], acc[g][5], acc[g][6], acc[g][7]);
                if (lir == 0) {
                    mlb[grp * 2] = m[g];
                    mlb[grp * 2 + 1] = l[g];
                }
            }
            __syncthreads();
            if (live && tl == 0) {
                for (uint32_t j = 1; j < TI; ++j) {
                    const uint32_t og = j * HS + hh;
                    const float mo = mlb[og * 2], lo = mlb[og * 2 + 1];
                    const float mx = fmaxf(m[g], mo);
                    const float mxs = (mx == -INFINITY) ? 0.f : mx;
                    const float wa = fast_exp2(m[g] - mxs), wb = fast_exp2(mo - mxs);
                    const float4 *src = reinterpret_cast<const float4 *>(accb + og * (LPR * 8) + lir * 8);
                    const float4 x0 = src[0], x1 = src[1];
                    acc[g][0] = acc[g][0] * wa + x0.x * wb;
                    acc[g][1] = acc[g][1] * wa + x0.y * wb;
                    acc[g][2] = acc[g][2] * wa + x0.z * wb;
                    acc[g][3] = acc[g][3] * wa + x0.w * wb;
                    acc[g][4] = acc[g][4] * wa + x1.x * wb;
                    acc[g][5] = acc[g][5] * wa + x1.y * wb;
                    acc[g][6] = acc[g][6] * wa + x1.z * wb;
                    acc[g][7] = acc[g][7] * wa + x1.w * wb;
                    l[g] = l[g] * wa + lo * wb;
                    m[g] = mx;
                }
            }
        }
        if (live && tl == 0) {
            if (direct) {
                const float inv = l[g] > 0.f ? 1.f / l[g] : 0.f;
                float *dst = a.out + s.out_off + (uint64_t)(kvh * G + g) * D + lir * 8;
                st_g16(dst, acc[g][0] * inv, acc[g][1] * inv, acc[g][2] * inv, acc[g][3] * inv);
                st_g16(dst + 4, acc[g][4] * inv, acc[g][5] * inv, acc[g][6] * inv, acc[g][7] * inv);
            } else {
                const uint32_t hq = hh * G + g;
                float *dst = pbase + (uint64_t)hq * D + lir * 2; // pair k at + k*(D/4): see part_pair_off
                st_part2(dst, acc[g][0], acc[g][1]);
                st_part2(dst + (D / 4), acc[g][2], acc[g][3]);
                st_part2(dst + 2 * (D / 4), acc[g][4], acc[g][5]);
                st_part2(dst + 3 * (D / 4), acc[g][6], acc[g][7]);
                if (lir == 0)
                    st_part2(pbase + (uint64_t)HS * G * D + hq * 2, m[g], l[g]);
            }
        }
    }

    // The store of the new token waits until here: loads (and barriers) issued after a store have
    // to wait for its acknowledgement too, and nothing in this item reads it back.
    if (new_dst != nullptr) {
        st_g16v(new_dst, nkr[0]);
        st_g16v(new_dst + LPR, nvr[0]);
    }
    finish_item<NT>(a, s, it, HS * G, D, s.head0 * G, 0, tab, mbuf);
}


// ---------------------------------------------------------------------------------------------
// Grouped-query path (head_dim D = 128, or 64 for groups of three and more; G = 2 .. 16 query heads per kv head:
// whatever fits the 16 columns of a product) on the matrix cores.  (The text below is written for D = 128; at D = 64 a
// K row is two 64-byte steps instead of four, a V row 8 chunks instead of 16 -- lanes j >= 8 fetch chunk j - 8 again and
// their output rows d = 8i + m >= 64, held by the lanes q >= 2, are never stored.)
//
// With G query heads sharing one kv head the path does G flop per KV byte and the plain-ALU
// formulation above becomes ALU-bound.  Here one wave owns one kv head and walks the item's
// tokens in tiles of 32, with v_mfma_f32_16x16x32_bf16 (lane l: column j = l%16, k-block q = l/16):
//   S^T[token][head]  = K[token][:] . Q[head][:]      A = K rows (16 tokens), B = Q^T (heads padded to 16)
//   O^T[d][head]     += V^T[d][token] . P^T[token][head]
// The S^T results leave lane (j, q) with 8 scores of head j (tokens 4q..4q+3 of each 16-token
// half), which is exactly the k-block the second product wants from that lane once its token
// order is taken as tau(q, e) = e < 4 ? 4q+e : 16+4q+(e-4); so P needs no cross-lane movement.
// V is loaded row-major (lane (i, q): 16-byte chunk i of the 8 tokens tau(q, .), i.e. whole
// 256-byte rows per 16 lanes) and transposed inside the lane with byte permutes; output row
// (MFMA m, lane i) is d = 8i + m.  P is split into bf16 high and low parts (two products), so the
// weights keep 16 mantissa bits: a single bf16 P would cost up to ~1e-2 absolute error.

template <int NT, int D>
__device__ __forceinline__ void process_item_gqa(const StepPages &sp) {
    const DecodeArgs a = ctx_args();
    const SeqRec s = ctx_seq();
    const ClassRec c = ctx_class();
    const Item it = ctx_item();
    int32_t *tab = s_tab;
    float *mbuf = s_mbuf;
    constexpr int KS = D / 32;  // products of 32 along head_dim for one score tile
    constexpr int VCH = D / 8;  // 16-byte chunks of a V row
    const int tid = threadIdx.x, lane = tid & 63;
    const uint32_t wave = uni((uint32_t)(tid >> 6));
    const uint32_t HS = c.hs, G = c.g;
    const bool live = wave < HS; // one wave per kv head of the slice; further waves idle
    const uint32_t kvh = s.head0 + (live ? wave : 0);
    const uint32_t j = lane & 15, q = lane >> 4;
    const uint32_t lg = a.log2_page;
    const uint64_t page_mask = (1ull << lg) - 1;

    const uint32_t jv = j % VCH; // the V chunk this lane fetches
    bf16x8_t qB[KS];
    {
        const uint4 *qp = reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(a.q) + s.q_off +
                                                          (uint64_t)(kvh * G + (j < G ? j : 0)) * D) + q;
#pragma unroll
        for (int st = 0; st < KS; ++st) {
            uint4 w = ld_g16(qp + st * 4);
            if (j >= G)
                w = make_uint4(0, 0, 0, 0);
            qB[st] = as_bf16x8(w);
        }
    }
    f32x4_t oacc[8];
#pragma unroll
    for (int mm = 0; mm < 8; ++mm)
        oacc[mm] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
    float m = -INFINITY, l = 0.f;

    const uint64_t T = c.token_bytes;
    const uint64_t row0 = (uint64_t)kvh * c.row_bytes;
    const uint64_t slice_lo = (uint64_t)s.head0 * c.row_bytes;
    const uint64_t slice_hi = (uint64_t)(s.head0 + HS) * c.row_bytes;

    const bool appends = item_appends(s, it);
    const uint32_t t_pool = appends ? it.t1 - 1 : it.t1; // tokens below this are read from the pool
    uint64_t new_lo;
    uint32_t new_n, new_first;
    step_entries(appends, sp, s, T, lg, new_lo, new_n, new_first);
    u32x4 nK[KS], nV; // the new token's K and V pieces of this lane (fused append)
    unsigned char *new_dst = nullptr;
    uint32_t w0 = it.t0;
    while (w0 < it.t1) { // workgroup-uniform: one pass per page-table window
        const uint64_t s_lo = ((uint64_t)w0 * T + slice_lo) >> lg;
        const uint64_t lim = (s_lo + kTabWindow) << lg;
        const uint64_t tmax = (lim - slice_hi) / T;
        const uint32_t w1 = (uint32_t)(tmax + 1 < (uint64_t)it.t1 ? tmax + 1 : (uint64_t)it.t1);
        const uint32_t n_ent = (uint32_t)((((uint64_t)(w1 - 1) * T + slice_hi - 1) >> lg) - s_lo) + 1;
        const uint32_t r1 = w1 < t_pool ? w1 : t_pool;
        // The new token is handled in the window that holds it, ahead of that window's pool tokens:
        // its loads are issued here, so that they are in flight together with the table window's.
        const bool new_here = appends && w1 == it.t1 && live;
        if (new_here) {
            const uint16_t *nk16, *nv16;
            new_token_rows(kvh, D, nk16, nv16);
            const unsigned char *nk = reinterpret_cast<const unsigned char *>(nk16) + q * 16;
#pragma unroll
            for (int st = 0; st < KS; ++st)
                nK[st] = ld_g16v(nk + st * 64);
            nV = ld_g16v(reinterpret_cast<const unsigned char *>(nv16) + jv * 16);
        }
        if (w0 != it.t0)
            __syncthreads(); // later windows only: see process_item
        load_table_window<NT>(tab, a, s, s_lo, n_ent, sp, new_lo, new_n, new_first);
        __syncthreads();

        if (live) {
            const uint32_t last = r1 - 1; // only used when the window holds a pool token
            // Window-relative byte offsets fit 32 bits (a window spans at most kTabWindow pages of at most 1 MiB).
            const uint32_t c0 = (uint32_t)(((uint64_t)w0 * T + row0) - (s_lo << lg));
            const uint32_t T32 = (uint32_t)T, mask32 = (uint32_t)page_mask;
            auto row_ptr = [&](uint32_t t) -> const unsigned char * { // head-row of (token t, this kv head)
                const uint32_t off = (t - w0) * T32 + c0;
                const int32_t pg = tab[off >> lg];
                return a.pool_base + (((uint64_t)(uint32_t)pg << lg) + (off & mask32));
            };
            // K rows: tokens tb+j and tb+16+j, chunk (step*4 + q) -> kA[half*4 + step]; V: chunk j of the
            // 8 tokens tau(q, e) -> vr[e].  Tokens past the range are clamped to its last token (and
            // masked in the scores of the range's last tile).
            auto tau = [&](uint32_t tb, int e) { return tb + (e < 4 ? 4 * q + e : 16 + 4 * q + (e - 4)); };
            auto load_k = [&](uint32_t tb, u32x4 (&kA)[2 * KS]) {
                const unsigned char *p0 = row_ptr(min(tb + j, last)) + q * 16;
                const unsigned char *p1 = row_ptr(min(tb + 16 + j, last)) + q * 16;
#pragma unroll
                for (int st = 0; st < KS; ++st) {
                    kA[st] = ld_kv4(p0 + st * 64);
                    kA[KS + st] = ld_kv4(p1 + st * 64);
                }
            };
            auto load_v = [&](uint32_t tb, u32x4 (&vr)[8]) {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    vr[e] = ld_kv4(row_ptr(min(tau(tb, e), last)) + 2 * D + jv * 16);
            };
            // raw scores q . K of the tile: s0 = tokens tb + 4q + r, s1 = tokens tb + 16 + 4q + r
            auto scores = [&](const u32x4 (&kA)[2 * KS], f32x4_t &s0, f32x4_t &s1) {
                s0 = (f32x4_t){0.f, 0.f, 0.f, 0.f};
                s1 = (f32x4_t){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int st = 0; st < KS; ++st) {
                    s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kA[st]), qB[st], s0, 0, 0, 0);
                    s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kA[KS + st]), qB[st], s1, 0, 0, 0);
                }
            };
            // Online softmax of the tile's scores and O^T += V^T P^T.  MASKED: only tokens below t_lim
            // count (the range's last tile, the new token's tile); the tile's first token always counts,
            // so the tile's maximum is finite.  Scores are scaled before the maximum is taken, so that
            // the largest one gets the weight 1 exactly (a one-token context returns that token's V).
            auto softmax_pv = [&](uint32_t tb, uint32_t t_lim, const f32x4_t &s0, const f32x4_t &s1,
                                  const u32x4 (&vr)[8], auto masked) {
// The scaled score must be rounded before the maximum is subtracted from it: fused into the
// subtraction, the largest score would no longer get the weight 1 exactly.
#pragma clang fp contract(off)
                constexpr bool MASKED = decltype(masked)::value;
                float sr[8];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    sr[r] = s0[r] * c.scale_log2e;
                    sr[4 + r] = s1[r] * c.scale_log2e;
                    if (MASKED) {
                        sr[r] = (tb + 4 * q + r < t_lim) ? sr[r] : -INFINITY;
                        sr[4 + r] = (tb + 16 + 4 * q + r < t_lim) ? sr[4 + r] : -INFINITY;
                    }
                }
                const float mt = max_over_kblocks(fmaxf(fmaxf(fmaxf(sr[0], sr[1]), fmaxf(sr[2], sr[3])),
                                                        fmaxf(fmaxf(sr[4], sr[5]), fmaxf(sr[6], sr[7]))));
                const float mn = fmaxf(m, mt);
                const float alpha = fast_exp2(m - mn);
                m = mn;
                // P as two bf16 parts by truncation: hi = upper 16 bits of p, lo = upper 16 bits of the
                // exact remainder p - hi; hi + lo carries 16 mantissa bits.  One byte permute packs a pair.
                uint32_t ph[4], pl[4];
                float psum = 0.f;
#pragma unroll
                for (int e = 0; e < 8; e += 2) {
                    const float p0 = fast_exp2(sr[e] - mn), p1 = fast_exp2(sr[e + 1] - mn);
                    psum += p0 + p1;
                    const uint32_t u0 = __float_as_uint(p0), u1 = __float_as_uint(p1);
                    const float x0 = p0 - __uint_as_float(u0 & 0xffff0000u);
                    const float x1 = p1 - __uint_as_float(u1 & 0xffff0000u);
                    ph[e / 2] = __builtin_amdgcn_perm(u1, u0, 0x07060302u);
                    pl[e / 2] = __builtin_amdgcn_perm(__float_as_uint(x1), __float_as_uint(x0), 0x07060302u);
                }
                l = fmaf(l, alpha, psum);
                if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0) {
#pragma unroll
                    for (int mm = 0; mm < 8; ++mm)
                        oacc[mm] *= alpha;
                }
                const bf16x8_t Ph = as_bf16x8(make_uint4(ph[0], ph[1], ph[2], ph[3]));
                const bf16x8_t Pl = as_bf16x8(make_uint4(pl[0], pl[1], pl[2], pl[3]));
#pragma unroll
                for (int mm = 0; mm < 8; ++mm) {
                    // element mm of each token's chunk: dword mm/2, low or high half
                    const uint32_t sel = (mm & 1) ? 0x07060302u : 0x05040100u;
                    uint32_t vt[4];
#pragma unroll
                    for (int pr = 0; pr < 4; ++pr)
                        vt[pr] = __builtin_amdgcn_perm(vr[2 * pr + 1][mm / 2], vr[2 * pr][mm / 2], sel);
                    const bf16x8_t Vt = as_bf16x8(make_uint4(vt[0], vt[1], vt[2], vt[3]));
                    oacc[mm] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Vt, Ph, oacc[mm], 0, 0, 0);
                    oacc[mm] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Vt, Pl, oacc[mm], 0, 0, 0);
                }
            };
            if (new_here) {
                // The new token as a tile of its own: every row of the tile is that token (all but
                // the first masked).  It goes into the pool once the item's loads are done.
                new_dst = const_cast<unsigned char *>(row_ptr(it.t1 - 1));
                u32x4 kA[2 * KS], vr[8];
#pragma unroll
                for (int st = 0; st < KS; ++st) {
                    kA[st] = nK[st];
                    kA[KS + st] = nK[st];
                }
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    vr[e] = nV;
                f32x4_t s0, s1;
                scores(kA, s0, s1);
                softmax_pv(it.t1 - 1, it.t1, s0, s1, vr, std::true_type{});
            }
            if (w0 < r1) {
                // The K registers of a tile are free once its scores are taken, the V registers once the
                // second product has read them: the next tile's K loads are issued right after the
                // first, its V loads right after the second, so one of the two is always in flight
                // behind the arithmetic without a second set of registers.  All tiles but the last are
                // whole, so only the last one takes the masked path.
                u32x4 kA[2 * KS], vr[8];
                load_k(w0, kA);
                load_v(w0, vr);
                uint32_t tb = w0;
                for (; tb + 32 < r1; tb += 32) {
                    f32x4_t s0, s1;
                    scores(kA, s0, s1);
                    load_k(tb + 32, kA);
                    softmax_pv(tb, r1, s0, s1, vr, std::false_type{});
                    load_v(tb + 32, vr);
                }
                f32x4_t s0, s1;
                scores(kA, s0, s1);
                softmax_pv(tb, r1, s0, s1, vr, std::true_type{});
            }
        }
        w0 = w1;
    }

    // lane (j, q) holds O[head j][d = 32q + 8r + mm] in oacc[mm][r]; l is a per-lane partial sum
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    const bool direct = it.part == kDirect;
    if (live && j < G && q < (uint32_t)KS) { // (at head_dim 64 the lanes q >= 2 hold rows past the head's end)
        if (direct) {
            const float inv = l > 0.f ? 1.f / l : 0.f;
            float *dst = a.out + s.out_off + (uint64_t)(kvh * G + j) * D + 32 * q;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                st_g16(dst + 8 * r, oacc[0][r] * inv, oacc[1][r] * inv, oacc[2][r] * inv, oacc[3][r] * inv);
                st_g16(dst + 8 * r + 4, oacc[4][r] * inv, oacc[5][r] * inv, oacc[6][r] * inv, oacc[7][r] * inv);
            }
        } else {
            float *pbase = a.partials + s.part_off + (uint64_t)it.part * s.part_stride;
            const uint32_t hq = wave * G + j;
            float *dst = pbase + (uint64_t)wave * (G * D) + (q * G + j) * 2; // pair (r, pp): see part_pair_off
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int pp = 0; pp < 4; ++pp)
                    st_part2(dst + (r * 4 + pp) * (2 * KS * G), oacc[2 * pp][r], oacc[2 * pp + 1][r]);
            if (q == 0)
                st_part2(pbase + (uint64_t)HS * G * D + hq * 2, m, l);
        }
    }
    if (new_dst != nullptr) { // K: D/8 pieces over lanes (j = 0, q) x D/32; V: D/8 pieces over lanes (j < D/8, q = 0)
        if (j == 0) {
#pragma unroll
            for (int st = 0; st < KS; ++st)
                st_g16v(new_dst + q * 16 + st * 64, nK[st]);
        }
        if (q == 0 && j < (uint32_t)VCH)
            st_g16v(new_dst + 2 * D + j * 16, nV);
    }
    finish_item<NT>(a, s, it, HS * G, D, s.head0 * G, G, tab, mbuf);
}

// KINDS: bit k set = the launch may meet items of kind k.  A pool's launches use the instantiation for the kinds of
// its services, so that the register count (and with it the number of workgroups a compute unit holds) is that of
// the kinds present, not of the most demanding kind compiled.
// (No second launch-bound argument: asking for two waves per SIMD outright gave the 256-lane kernel a
// register assignment that measured 0.5-1 % slower; the variants fit their register classes as they are.)
__shared__ uint32_t s_span; // the span the workgroup takes next

// Spans past the first of a workgroup come from the queue (see DecodeArgs).  The take is an atomic on one word in
// memory for the whole device, a few hundred nanoseconds each when many arrive together, and the loads its wave
// issues afterwards return behind it.  So the first span is the workgroup's own index (no take: all workgroups start
// at once), and the take for the next span is issued when the current span's last item begins: spans end at
// different times, and the round trip hides behind that item.
// (Returns the counter's value as fetched; the span is grid + value - queue_base, worked out where the span is
// needed, so that the fetch stays in flight until then.)
__device__ __forceinline__ uint32_t take_span(const DecodeArgs &a) {
    return __hip_atomic_fetch_add(as_global(a.queue), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int NT, uint32_t KINDS>
__device__ __forceinline__ void decode_body(const DecodeArgs &a, const StepPages &sp) {
    // a checked call (UKV_PARAM_VALIDATE) whose page tables hold an id outside the pool does nothing
    if (a.bad != nullptr && uni(*reinterpret_cast<const volatile uint32_t *>(a.bad)) != 0)
        return;
    if (threadIdx.x == 0)
        s_ctx.a = a;
    const uint32_t grid = gridDim.x;
    const uint32_t n_spans = a.n_spans_dev != nullptr ? uni(*as_global(a.n_spans_dev)) : a.n_spans;
    uint32_t span = blockIdx.x;
    // The first eight lanes of the workgroup hold one 16-byte piece each of an item's record.
    const bool rec_lane = threadIdx.x < sizeof(ItemRec) / 16;
    auto rec_piece = [&](uint32_t i) {
        return ld_g16(reinterpret_cast<const unsigned char *>(a.recs + i) + 16 * threadIdx.x);
    };
    while (span < n_spans) { // workgroup-uniform
        uint32_t next = 0;   // thread 0 only
        const uint32_t i0 = uni(a.span_first[span]), i1 = uni(a.span_first[span + 1]);
        if (i0 == i1 && threadIdx.x == 0)
            next = take_span(a);
        uint4 rec = make_uint4(0, 0, 0, 0), rec_next = make_uint4(0, 0, 0, 0);
        if (i0 < i1 && rec_lane)
            rec = rec_piece(i0);
        for (uint32_t i = i0; i < i1; ++i) {
            __syncthreads(); // the previous item is done with s_ctx
            if (threadIdx.x < 64) { // the first wave publishes the record
                // A plan that outlives its step: the sequence has grown by delta tokens since it was made, and the
                // growth belongs to the sequence's last item (t1 == ctx_len).  t1 is word 2 of piece 0, ctx_len
                // word 2 of piece 3 (see ItemRec).
                const uint32_t t1 = (uint32_t)__builtin_amdgcn_readlane((int)rec.z, 0);
                const uint32_t ctx = (uint32_t)__builtin_amdgcn_readlane((int)rec.z, 3);
                if ((threadIdx.x == 0 && t1 == ctx) || threadIdx.x == 3)
                    rec.z += a.delta;
                if (rec_lane)
                    reinterpret_cast<uint4 *>(&s_ctx.it)[threadIdx.x] = rec;
                if (threadIdx.x == 0 && i == i1 - 1)
                    next = take_span(a); // in flight while the span's last item is worked on
                if (rec_lane && i + 1 < i1)
                    rec_next = rec_piece(i + 1); // in flight while this item is worked on
            }
            __syncthreads();
            const uint32_t kind = uni(s_ctx.c.kind); // workgroup-uniform: one compiled function per (head_dim, group) kind
            if ((KINDS & (1u << kD64G1)) && kind == kD64G1)
                process_item<64, 1, NT>(sp);
            else if ((KINDS & (1u << kD64G2)) && kind == kD64G2)
                process_item<64, 2, NT>(sp);
            else if ((KINDS & (1u << kD128G1)) && kind == kD128G1)
                process_item<128, 1, NT>(sp);
            else if ((KINDS & (1u << kD128GQA)) && kind == kD128GQA)
                process_item_gqa<NT, 128>(sp);
            else if ((KINDS & (1u << kD64GQA)) && kind == kD64GQA)
                process_item_gqa<NT, 64>(sp);
            rec = rec_next;
        }
        __syncthreads(); // every wave has read the previous s_span
        if (threadIdx.x == 0)
            s_span = grid + next - a.queue_base;
        __syncthreads();
        span = uni(s_span);
    }
}

template <int NT, uint32_t KINDS>
__global__ void __launch_bounds__(NT) decode_kernel(DecodeArgs a, StepPages sp) {
    decode_body<NT, KINDS>(a, sp);
}

// The merge as a launch of its own:  out = sum_c acc_c 2^(m_c-M) / sum_c l_c 2^(m_c-M), in two kernels; the
// planner says which sequences go to which.
//
// reduce_few_kernel: sequences of a few parts.  One wave per (cut sequence, unit), a unit being a stretch of a
// partial that is contiguous in memory: the D accumulators of one query head (ALU-path layout) or the G*128 of
// one kv head's query group (matrix-core layout).  Lanes read a unit in memory order, 64 consecutive floats per
// load instruction (taken query head by query head in column order, the matrix-core layout costs a cache line
// for every 8 bytes: 20 against 11 us on the GQA workload), four parts per round trip.  Which (query head,
// column) a float is: acc_elem; all floats of a lane belong to one query head.
static constexpr uint32_t kReduceMaxPerLane = 16;
__global__ void __launch_bounds__(64) reduce_few_kernel(const ReduceRec *recs, const uint32_t *n_recs_dev,
                                                        const float *partials, float *out) {
    if (n_recs_dev != nullptr && blockIdx.x >= *n_recs_dev) // list length known only on the device: the grid is an upper bound
        return;
    const ReduceRec r = recs[blockIdx.x];
    const uint32_t gx = r.layout_g ? r.layout_g : 1;             // query heads per unit
    const uint32_t unit = blockIdx.y, unit_floats = gx * r.d;
    if (unit >= r.n_heads / gx)
        return;
    const uint32_t lane = threadIdx.x;
    const uint32_t ni = unit_floats / 64;                         // elements per lane: 1, 2 or G d / 64 <= 16 (reduce_few_takes)
    const uint32_t data_off = unit * unit_floats + lane;          // this lane's first float of every part
    const uint32_t head = acc_elem(r.layout_g, r.d, data_off).head; // its query head, the same for all its floats
    const float *base = partials + r.part_off;
    const uint32_t ml_off = r.n_heads * r.d + head * 2;
    float o[kReduceMaxPerLane];
#pragma unroll
    for (uint32_t i = 0; i < kReduceMaxPerLane; ++i)
        o[i] = 0.f;
    float M = -INFINITY, L = 0.f; // of this lane's query head
    constexpr uint32_t kGroup = 4;
    for (uint32_t c = 0; c < r.n_parts; c += kGroup) {
        float mc[kGroup], lc[kGroup], x[kGroup][kReduceMaxPerLane];
#pragma unroll
        for (uint32_t k = 0; k < kGroup; ++k) {
            const float *pc = base + (uint64_t)min(c + k, r.n_parts - 1) * r.part_stride;
            const float2 ml = *reinterpret_cast<const float2 *>(pc + ml_off);
            const bool live = c + k < r.n_parts && ml.y > 0.f; // an empty part carries no weight
            mc[k] = live ? ml.x : -INFINITY;
            lc[k] = live ? ml.y : 0.f;
#pragma unroll
            for (uint32_t i = 0; i < kReduceMaxPerLane; ++i)
                x[k][i] = i < ni ? pc[data_off + 64 * i] : 0.f;
        }
        float Mn = M;
#pragma unroll
        for (uint32_t k = 0; k < kGroup; ++k)
            Mn = fmaxf(Mn, mc[k]);
        const float Ms = Mn == -INFINITY ? 0.f : Mn;
        const float keep = fast_exp2(M - Ms);
        L *= keep;
#pragma unroll
        for (uint32_t i = 0; i < kReduceMaxPerLane; ++i)
            o[i] *= keep;
        M = Mn;
#pragma unroll
        for (uint32_t k = 0; k < kGroup; ++k) {
            const float w = fast_exp2(mc[k] - Ms); // 0 for a part that does not count
            L = fmaf(lc[k], w, L);
#pragma unroll
            for (uint32_t i = 0; i < kReduceMaxPerLane; ++i)
                o[i] = fmaf(x[k][i], w, o[i]);
        }
    }
    const float inv = L > 0.f ? 1.f / L : 0.f;
    float *dst = out + r.out_off + (uint64_t)head * r.d;
#pragma unroll
    for (uint32_t i = 0; i < kReduceMaxPerLane; ++i)
        if (i < ni)
            dst[acc_elem(r.layout_g, r.d, data_off + 64 * i).col] = o[i] * inv;
}

// reduce_many_kernel: sequences of many parts (one long request alone on the device is cut into hundreds), where
// part after part would be a chain of hundreds of dependent round trips.  One workgroup of four waves per (cut
// sequence, query head): the (m, l) pairs are fetched by all lanes at once, the weights are worked out in LDS,
// and the waves share the parts, each with several accumulator rows in flight.  (Here the data is small and
// there are few sequences: more workgroups matter more than whole cache lines.)
static constexpr uint32_t kReduceWaves = 4, kReduceChunk = 1024, kReduceAhead = 8;
__global__ void __launch_bounds__(64 * kReduceWaves) reduce_many_kernel(const ReduceRec *recs,
                                                                       const uint32_t *n_recs_dev,
                                                                       const float *partials, float *out) {
    if (n_recs_dev != nullptr && blockIdx.x >= *n_recs_dev) // workgroup-uniform
        return;
    const ReduceRec r = recs[blockIdx.x];
    const uint32_t hq = blockIdx.y;
    if (hq >= r.n_heads)
        return;
    const float *base = partials + r.part_off;
    const uint32_t ml_off = r.n_heads * r.d + hq * 2;
    const uint32_t tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
    const bool one = lane < r.d, two = r.d > 64;
    // this lane's output elements are lane and 64 + lane: where they sit inside a part
    const uint32_t off0 = part_pair_off(r.layout_g, r.d, hq, lane >> 2, (lane >> 1) & 1) + (lane & 1);
    const uint32_t off1 = part_pair_off(r.layout_g, r.d, hq, (64 + lane) >> 2, (lane >> 1) & 1) + (lane & 1);
    float *dst = out + r.out_off + (uint64_t)hq * r.d;
    __shared__ float s_m[kReduceChunk], s_l[kReduceChunk];
    __shared__ float s_red[kReduceWaves], s_o[kReduceWaves][128], s_L[kReduceWaves];
    float M = -INFINITY, L = 0.f, o0 = 0.f, o1 = 0.f; // M is the same in every lane of the workgroup; L, o0, o1 are this wave's shares
    for (uint32_t c0 = 0; c0 < r.n_parts; c0 += kReduceChunk) { // workgroup-uniform
        const uint32_t nc = min(kReduceChunk, r.n_parts - c0);
        float mx = -INFINITY;
        for (uint32_t c = tid; c < nc; c += 64 * kReduceWaves) {
            const float2 ml = *reinterpret_cast<const float2 *>(base + (uint64_t)(c0 + c) * r.part_stride + ml_off);
            const bool live = ml.y > 0.f; // an empty part carries no weight
            s_m[c] = live ? ml.x : -INFINITY;
            s_l[c] = live ? ml.y : 0.f;
            mx = fmaxf(mx, s_m[c]);
        }
        for (int o = 32; o > 0; o >>= 1)
            mx = fmaxf(mx, __shfl_xor(mx, o));
        if (lane == 0)
            s_red[wave] = mx;
        __syncthreads();
        float Mn = M;
        for (uint32_t w = 0; w < kReduceWaves; ++w)
            Mn = fmaxf(Mn, s_red[w]);
        const float Ms = Mn == -INFINITY ? 0.f : Mn;
        const float keep = fast_exp2(M - Ms); // what the sums so far are worth against the new maximum
        L *= keep;
        o0 *= keep;
        o1 *= keep;
        M = Mn;
        for (uint32_t c = wave * kReduceAhead; c < nc; c += kReduceWaves * kReduceAhead) { // wave-uniform
            float x0[kReduceAhead], x1[kReduceAhead];
#pragma unroll
            for (uint32_t k = 0; k < kReduceAhead; ++k) {
                const float *pc = base + (uint64_t)(c0 + min(c + k, nc - 1)) * r.part_stride;
                x0[k] = one && c + k < nc ? pc[off0] : 0.f;
                x1[k] = two && c + k < nc ? pc[off1] : 0.f;
            }
#pragma unroll
            for (uint32_t k = 0; k < kReduceAhead; ++k) {
                if (c + k >= nc)
                    break;
                const float w = fast_exp2(s_m[c + k] - Ms);
                L = fmaf(s_l[c + k], w, L);
                o0 = fmaf(x0[k], w, o0);
                o1 = fmaf(x1[k], w, o1);
            }
        }
        __syncthreads(); // s_m, s_l and s_red are rewritten by the next chunk
    }
    s_o[wave][lane] = o0;
    s_o[wave][64 + lane] = o1;
    if (lane == 0)
        s_L[wave] = L;
    __syncthreads();
    if (wave == 0) {
        float Lt = 0.f, t0 = 0.f, t1 = 0.f;
        for (uint32_t w = 0; w < kReduceWaves; ++w) {
            Lt += s_L[w];
            t0 += s_o[w][lane];
            t1 += s_o[w][64 + lane];
        }
        const float inv = Lt > 0.f ? 1.f / Lt : 0.f;
        if (one)
            dst[lane] = t0 * inv;
        if (two)
            dst[64 + lane] = t1 * inv;
    }
}

// ------------------------------------------------------------------ launchers
// How many spans the planner makes its first (largest) round of: one per compute unit.  Where two workgroups
// fit a CU (the 256-lane kernel at 256 registers or fewer), a first round of two spans per CU was measured 2-3 %
// slower on the grouped-query workload: twice the cuts, partials and merges, and no higher a rate while they stream.
int decode_resident_workgroups(uint32_t block_threads) {
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        return 0;
    hipError_t e = block_threads == 512
                       ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_kernel<512, kWorkloadKinds>, 512, 0)
                       : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_kernel<256, kWorkloadKinds>, 256, 0);
    if (e != hipSuccess || per_cu <= 0 || cus <= 0) // (a kernel that does not fit a CU at all)
        return 0;
    return cus;
}

// The compiled sets of kinds, smallest first; a launch takes the first one that covers the pool's kinds.
static constexpr uint32_t kKindSets[] = {1u << kD128G1, (1u << kD64G1) | (1u << kD64G2),
                                         (1u << kD64G1) | (1u << kD64G2) | (1u << kD128G1), 1u << kD128GQA,
                                         kWorkloadKinds, kAllKinds};
static constexpr int kNumKindSets = 6;

static int kind_set_of(uint32_t kinds) {
    if (kinds == 0 || (kinds & ~kAllKinds))
        kinds = kAllKinds;
    int set = 0;
    while ((kinds & ~kKindSets[set]) != 0)
        ++set; // ends at kAllKinds at the latest
    return set;
}

typedef void (*DecodeKernelFn)(DecodeArgs, StepPages);
static DecodeKernelFn decode_kernel_fn(int set, bool big) {
    switch (set) {
    case 0: return big ? decode_kernel<512, kKindSets[0]> : decode_kernel<256, kKindSets[0]>;
    case 1: return big ? decode_kernel<512, kKindSets[1]> : decode_kernel<256, kKindSets[1]>;
    case 2: return big ? decode_kernel<512, kKindSets[2]> : decode_kernel<256, kKindSets[2]>;
    case 3: return big ? decode_kernel<512, kKindSets[3]> : decode_kernel<256, kKindSets[3]>;
    case 4: return big ? decode_kernel<512, kKindSets[4]> : decode_kernel<256, kKindSets[4]>;
    default: return big ? decode_kernel<512, kAllKinds> : decode_kernel<256, kAllKinds>;
    }
}

// Workgroups of a launch: as many as the device keeps resident of this instantiation (compute units x workgroups
// per unit), so that none waits for a place; each takes spans from the queue until it is empty.  `first_round` (0 =
// no such limit): a plan with more spans than places gets at most this many workgroups -- the spans of the planner's
// first round.  Workgroups beyond those would start with the small spans of the later rounds and use them up in the
// launch's first quarter, when nothing needs evening out; at the end, where the first round's spans finish 5-8 %
// apart, the queue would be empty.
uint32_t decode_grid(uint32_t n_spans, uint32_t block_threads, uint32_t kinds, uint32_t first_round) {
    static int places[2][kNumKindSets]; // per device kind this would differ; all devices of a process are alike
    const int set = kind_set_of(kinds);
    const bool big = block_threads == 512;
    int &cached = places[big ? 1 : 0][set];
    if (cached == 0) {
        int dev = 0, cus = 0, per_cu = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess &&
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_kernel_fn(set, big), big ? 512 : 256, 0) ==
                hipSuccess &&
            cus > 0 && per_cu > 0)
            cached = cus * per_cu;
        else
            cached = -1;
    }
    const uint32_t cap = cached > 0 ? (uint32_t)cached : 256u;
    if (n_spans <= cap)
        return n_spans; // every span has a workgroup of its own from the start
    return first_round != 0 && first_round < cap ? first_round : cap;
}

// grid: decode_grid() of the plan's spans.  sp: the step's new page ids for the kernel arguments, or null.
// ev0/ev1 (may be null) receive the kernel's own start/stop timestamps.
hipError_t launch_decode(const DecodeArgs &a, const StepPages *sp_in, uint32_t grid, uint32_t block_threads,
                         uint32_t kinds, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1) {
    if (grid == 0)
        return hipSuccess;
    static const StepPages no_pages{}; // n_req == 0
    const StepPages &sp = sp_in ? *sp_in : no_pages;
    const bool big = block_threads == 512;
    hipExtLaunchKernelGGL(decode_kernel_fn(kind_set_of(kinds), big), dim3(grid), dim3(big ? 512 : 256), 0, s, ev0, ev1, 0,
                          a, sp);
    return hipGetLastError();
}

// recs: the n_many sequences of many parts first, then the others; ev0/ev1 bracket both launches.
hipError_t launch_reduce(const ReduceRec *recs, uint32_t n_recs, uint32_t n_many, uint32_t max_heads, uint32_t max_units,
                         const float *partials, float *out, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1) {
    if (n_recs == 0)
        return hipSuccess;
    const uint32_t n_few = n_recs - n_many;
    if (n_many)
        hipExtLaunchKernelGGL(reduce_many_kernel, dim3(n_many, max_heads), dim3(64 * kReduceWaves), 0, s, ev0,
                              n_few ? nullptr : ev1, 0, recs, (const uint32_t *)nullptr, partials, out);
    if (n_few)
        hipExtLaunchKernelGGL(reduce_few_kernel, dim3(n_few, max_units), dim3(64), 0, s, n_many ? nullptr : ev0, ev1, 0,
                              recs + n_many, (const uint32_t *)nullptr, partials, out);
    return hipGetLastError();
}

// The same two kernels over lists whose lengths only the device knows (a plan made on the device): the grids are
// upper bounds, workgroups past *n_many_dev / *n_few_dev leave at once.
hipError_t launch_reduce_counted(const ReduceRec *many, const uint32_t *n_many_dev, uint32_t many_bound,
                                 const ReduceRec *few, const uint32_t *n_few_dev, uint32_t few_bound, uint32_t max_heads,
                                 uint32_t max_units, const float *partials, float *out, hipStream_t s) {
    if (many_bound && max_heads)
        hipLaunchKernelGGL(reduce_many_kernel, dim3(many_bound, max_heads), dim3(64 * kReduceWaves), 0, s, many,
                           n_many_dev, partials, out);
    if (few_bound && max_units)
        hipLaunchKernelGGL(reduce_few_kernel, dim3(few_bound, max_units), dim3(64), 0, s, few, n_few_dev, partials, out);
    return hipGetLastError();
}

} // namespace ukv
