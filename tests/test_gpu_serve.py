"""Scheduler-driven serving loop on the GPU against the oracle, iteration by iteration (section 4.2, Equation 6, the
DB algorithm of the appendix; prefill and decode of section 2.1 over the unified cache of section 4.4).

The loop (paper_2504_15720_amd.serving: C++ scheduler, library free list, HIP kernels) runs on the model clock, so
its decisions are reproducible.  An observer replays every iteration on the CPU with oracle/db_scheduler.py, a
synthetic LIFO page stack and a host image of the pool kept by oracle.scatter / oracle.append, and compares:
  * every batch: (ids, service, queue), the free-page count it was chosen under, the pages taken (bit-exact ids),
    the charged time and clock (equal doubles), the finished flags;
  * budgets, priorities, doublings and lengths of the batch's requests after every iteration, of all live requests
    every 50 iterations (equal doubles);
  * sampled decode iterations against oracle.attention and the first prefill batches against oracle.prefill on
    sampled rows (max |err| <= 2e-3); finished requests' caches read back with ukv_gather against oracle.gather of
    the host image; the whole pool image, byte for byte, at checkpoints and at the end.
"""
import sys
from types import SimpleNamespace

import numpy as np
import pytest

from oracle import db_scheduler as dbs
from oracle import oracle
from synth import PageStack
from synth.serving import draw_serve_workload, modelled_time, tiled

ATOL = 2e-3


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


class Replay:
    """The oracle side of the loop.  Fed with the GPU loop's events it checks them; without a loop (drive()) it runs
    the same policy alone, which shows on the CPU that the workload completes."""

    def __init__(self, wl, policy):
        self.wl, self.policy = wl, policy
        prof = [dbs.ServiceProfile(m, s, thr, wl.services[k].token_bytes) for k, (m, s, thr) in enumerate(wl.profiles)]
        n_sched = 1 if policy == "db" else len(wl.services)
        self.scheds = [dbs.DBScheduler(prof, wl.page_bytes, wl.max_batch) for _ in range(n_sched)]
        for r in range(wl.n):
            self.scheds[0 if policy == "db" else int(wl.svc[r])].add_request(r, int(wl.svc[r]), int(wl.prompt[r]), 0.0)
        self.stack = PageStack(wl.n_pages)
        self.table = np.full(int(wl.cap.sum()), -1, np.int32)
        self.ctx = np.zeros(wl.n, np.int64)
        self.owned = [[] for _ in range(wl.n)]
        self.now = 0.0
        self.slot_off = (np.arange(wl.n) * wl.row_max).astype(np.uint64)
        self.pool = None          # host image of the pool: only with a GPU loop to compare against
        self.stats = dict(iterations=0, decode_checked=0, prefill_checked=0, caches=0, pool_images=0, doublings=0,
                          starved_first=0, page_limited=0, worst=0.0)

    def with_pool_image(self):
        wl = self.wl
        n_el = wl.n_pages * wl.page_bytes // 2
        blk = wl.noise_block(3)
        self.pool = np.tile(blk, -(-n_el // blk.size))[:n_el].copy()
        self.blocks = [wl.noise_block(w) for w in (0, 1, 2)]
        self.dq, self.dnk, self.dnv = wl.decode_inputs()
        return self

    # ---- the oracle's own decisions for the next iteration
    def decide(self):
        free = self.stack.free_pages
        batches = []
        for k, sc in enumerate(self.scheds):
            ids, s_, queue = sc.next_batch(self.now, free)
            if ids:
                if sc._starved_service(self.now) is not None:
                    self.stats["starved_first"] += 1
                if sc.next_batch(self.now, 10 ** 9)[0] != ids:     # with unlimited pages the batch would differ
                    self.stats["page_limited"] += 1
                free -= sum(sc.pages_needed(sc.requests[i]) for i in ids)
                batches.append((k, [int(i) for i in ids], int(s_), int(queue)))
        return batches

    def table_of(self, r):
        o = int(self.wl.table_off[r])
        return self.table[o:o + int(self.wl.cap[r])]

    def take_pages(self, ids, new_ctx):
        wl = self.wl
        entry, page = [], []
        for r, c in zip(ids, new_ctx):
            have = len(self.owned[r])
            need = int(-(-int(c) * int(wl.tok_b[r]) // wl.page_bytes)) - have
            if need > 0:
                got = self.stack.alloc(need)
                for k in range(need):
                    self.table[int(wl.table_off[r]) + have + k] = got[k]
                entry.extend(int(wl.table_off[r]) + have + k for k in range(need))
                page.extend(int(x) for x in got)
                self.owned[r].extend(int(x) for x in got)
        return np.array(entry, np.uint64), np.array(page, np.int32)

    def duck(self, ids):
        wl = self.wl
        ids = np.asarray(ids)
        so = self.slot_off[ids]
        return SimpleNamespace(services=wl.services, service_id=wl.svc[ids], ctx_len=self.ctx[ids].astype(np.uint32),
                               table_off=wl.table_off[ids], table_cap=wl.cap[ids], page_table=self.table,
                               new_off=so, q_off=so, out_off=so, out_elems=wl.n * wl.row_max, page_bytes=wl.page_bytes,
                               q=getattr(self, "dq", None))

    # ---- one iteration: the oracle's decision, executed on the host image; checked against `ev` if given
    def __call__(self, ev=None):
        wl, st = self.wl, self.stats
        it = st["iterations"]
        batches = self.decide()
        assert batches, "oracle: nothing fits the pool"
        if ev is not None:
            assert ev["free_pages"] == self.stack.free_pages, f"iteration {it}: free pages differ"
            assert ev["now"] == self.now, f"iteration {it}: clocks differ"
            got = [(k, [int(i) for i in ids], int(s_), int(q_)) for k, ids, s_, q_ in ev["batches"]]
            assert got == batches, f"iteration {it}: batch decision differs\n GPU loop {got}\n oracle   {batches}"
        work = iter(ev["work"]) if ev is not None else None
        elapsed, kv_base, q_base = 0.0, 0, 0                  # every prefill batch of an iteration has a buffer region of its own
        for _, ids, s_, queue in batches:                    # prefill batches first, in scheduler order
            if queue != dbs.WAIT:
                continue
            ids_a = np.array(ids)
            entry, page = self.take_pages(ids, wl.prompt[ids_a])
            sizes_kv, sizes_q = wl.prompt[ids_a] * wl.tok_el[ids_a], wl.prompt[ids_a] * wl.row_el[ids_a]
            kv_off, q_off = kv_base + np.cumsum(sizes_kv) - sizes_kv, q_base + np.cumsum(sizes_q) - sizes_q
            kv_base, q_base = kv_base + int(sizes_kv.sum()), q_base + int(sizes_q.sum())
            self.ctx[ids_a] = wl.prompt[ids_a]
            elapsed += modelled_time(True, wl.prompt[ids_a], wl.tok_b[ids_a])
            if ev is None:
                continue
            w = next(work)
            assert w["kind"] == "prefill" and np.array_equal(w["entry"], entry) and np.array_equal(w["page"], page), \
                f"iteration {it}: prefill pages differ"
            assert np.array_equal(w["kv_off"], kv_off) and np.array_equal(w["q_off"], q_off)
            for r, ko in zip(ids, kv_off):
                sv, p = wl.services[int(wl.svc[r])], int(wl.prompt[r])
                shape = (p, sv.n_kv_heads, sv.head_dim)
                oracle.scatter(self.pool, wl.page_bytes, self.table_of(r),
                               tiled(self.blocks[0], int(ko), p * int(wl.tok_el[r])).reshape(shape),
                               tiled(self.blocks[1], int(ko), p * int(wl.tok_el[r])).reshape(shape))
            if st["prefill_checked"] < 6:                     # the first prefill batches, on sampled rows
                out = ev["loop"].pf_out.cpu().numpy()
                for r, qo in zip(ids, q_off):
                    sv, p, re_ = wl.services[int(wl.svc[r])], int(wl.prompt[r]), int(wl.row_el[r])
                    pos = sorted({0, p // 3, p - 2 if p > 1 else 0, p - 1})
                    q_rows = np.stack([tiled(self.blocks[2], int(qo) + t * re_, re_) for t in pos])
                    ref = oracle.prefill(self.pool, wl.page_bytes, self.table_of(r), sv.n_q_heads, sv.n_kv_heads,
                                         sv.head_dim, sv.softmax_scale, p, pos, q_rows)
                    for j, t in enumerate(pos):
                        g = out[int(qo) + t * re_: int(qo) + (t + 1) * re_].astype(np.float64)
                        err = float(np.max(np.abs(g - ref[j].reshape(-1))))
                        st["worst"] = max(st["worst"], err)
                        assert err <= ATOL, f"iteration {it}: prefill request {r} row {t}: max |err| {err}"
                st["prefill_checked"] += 1
        dec = [i for _, ids, _, queue in batches if queue == dbs.DECODING for i in ids]
        if dec:
            dec_a = np.array(dec)
            self.ctx[dec_a] += 1
            entry, page = self.take_pages(dec, self.ctx[dec_a])
            elapsed += modelled_time(False, self.ctx[dec_a], wl.tok_b[dec_a])
            if ev is not None:
                w = next(work)
                assert w["kind"] == "decode" and np.array_equal(w["entry"], entry) and np.array_equal(w["page"], page), \
                    f"iteration {it}: decode pages differ"
                d = self.duck(dec)
                oracle.append(d, self.pool, self.dnk, self.dnv)
                if it % 40 == 7 or st["decode_checked"] < 3:  # sampled iterations: every output of the batch
                    ref = oracle.attention(d, self.pool)
                    out = ev["loop"].dout.cpu().numpy().astype(np.float64)
                    for r in dec:
                        o, re_ = int(self.slot_off[r]), int(wl.row_el[r])
                        err = float(np.max(np.abs(out[o:o + re_] - ref[o:o + re_])))
                        st["worst"] = max(st["worst"], err)
                        assert err <= ATOL, f"iteration {it}: decode request {r}: max |err| {err}"
                    st["decode_checked"] += 1
        self.now = self.now + elapsed
        if ev is not None:
            assert ev["elapsed"] == elapsed and ev["now_end"] == self.now, f"iteration {it}: charged time differs"
        fins = []
        for k, ids, _, _ in batches:
            fin = [bool(self.ctx[i] >= wl.prompt[i] + wl.out_len[i]) for i in ids]
            fins.append(fin)
            self.scheds[k].complete(ids, fin, elapsed, self.now)
            for i in ids:
                if i in self.scheds[k].requests:
                    st["doublings"] = max(st["doublings"], self.scheds[k].requests[i].doublings)
        if ev is not None:
            import paper_2504_15720_amd as U
            loop = ev["loop"]
            assert [list(f) for f in ev["finished"]] == fins, f"iteration {it}: finished flags differ"
            live = [(k, i) for k, ids, _, _ in batches for i in ids if i in self.scheds[k].requests]
            if it % 50 == 0:
                live = [(k, i) for k, sc in enumerate(self.scheds) for i in sc.requests]
            for k, i in live:
                o, g = self.scheds[k].requests[i], U.ukv_sched_request_info(loop.scheds[k], i)
                assert (g.budget, g.priority, g.doublings, g.ctx_len, g.queue, g.service) == \
                    (o.budget, o.priority, o.doublings, o.ctx_len, o.queue, o.service), f"iteration {it}: request {i}"
            for (k, ids, _, _), fin in zip(batches, fins):   # caches of finished requests, while they still own pages
                for i, f in zip(ids, fin):
                    if f and st["caches"] < 8:
                        self.check_cache(loop, i)
            if it % 150 == 149:
                self.check_pool_image(loop)
        for (k, ids, _, _), fin in zip(batches, fins):
            for i, f in zip(ids, fin):
                if f:
                    self.stack.free(np.array(self.owned[i], np.int32))
                    self.owned[i] = []
        st["iterations"] += 1

    def check_cache(self, loop, r):
        import paper_2504_15720_amd as U
        wl, torch = self.wl, loop.torch
        sv, c = wl.services[int(wl.svc[r])], int(self.ctx[r])
        n_el = c * int(wl.tok_el[r])
        k = torch.zeros(n_el, dtype=torch.int16, device=loop.dev)
        v = torch.zeros(n_el, dtype=torch.int16, device=loop.dev)
        d1 = U.BatchDesc([wl.svc[r]], [c], [wl.table_off[r]], loop.table_t.data_ptr())
        U.ukv_gather(loop.pool, d1, k.data_ptr(), v.data_ptr(), np.zeros(1, np.uint64), loop.stream)
        rk, rv = oracle.gather(self.pool, wl.page_bytes, self.table_of(r), sv.n_kv_heads, sv.head_dim, c)
        assert np.array_equal(k.cpu().numpy().view(np.uint16), rk.reshape(-1)), f"cache K of request {r} differs"
        assert np.array_equal(v.cpu().numpy().view(np.uint16), rv.reshape(-1)), f"cache V of request {r} differs"
        self.stats["caches"] += 1

    def check_pool_image(self, loop):
        got = loop.pool_t.cpu().numpy().view(np.uint16)
        assert np.array_equal(got, self.pool), "pool image differs from the oracle's"
        assert np.array_equal(loop.table_t.cpu().numpy()[self.table >= 0], self.table[self.table >= 0]), "page tables differ"
        self.stats["pool_images"] += 1

    def pending(self):
        return any(sc.requests for sc in self.scheds)

    def drive(self):
        while self.pending():
            self()
        return self.stats


def _workload():
    # 8 requests per service; a pool that holds a quarter of what all requests need at their final lengths (so
    # page-counted admission decides batches), budgets short enough to double twice and a starvation threshold short
    # enough to trigger on the model clock.  (The loop has no preemption or swap-out: a pool in which every admitted
    # request needs a page to grow and none is free stops it; this workload was chosen to complete under both policies.)
    return draw_serve_workload(8, max_batch=6, starvation_threshold=1.5e-3, headroom=0.25, time_unit=2.5e-4)


@pytest.mark.parametrize("policy", ["db", "mixed"])
def test_replay_alone_completes_and_exercises_the_rules(policy):
    """CPU: the oracle-side replay, driven by its own decisions, serves the test workload to completion and meets
    budget doublings and page-limited choices on the way, and starvation under the paper's rule (so the GPU
    comparison below covers those rules)."""
    st = Replay(_workload(), policy).drive()
    assert st["iterations"] > 100 and st["doublings"] >= 2
    assert st["page_limited"] > 0
    if policy == "db":
        assert st["starved_first"] > 0


@pytest.mark.gpu
@pytest.mark.parametrize("policy", ["db", "mixed"])
def test_serving_loop_matches_oracle_every_iteration(policy):
    from paper_2504_15720_amd.serving import ServingLoop
    wl = _workload()
    say(f"serving loop, policy {policy}: {wl.n} requests, {wl.n_pages} pages, prompts {int(wl.prompt.sum())} tokens, "
        f"{int(wl.out_len.sum())} tokens to generate")
    loop = ServingLoop(wl, modelled_time)
    rep = Replay(wl, policy).with_pool_image()
    res = loop.run(policy, clock="model", observer=rep)
    assert not rep.pending(), "the oracle still has requests queued"
    rep.check_pool_image(loop)
    st = rep.stats
    say(f"  {res['iterations']} iterations identical; decode outputs checked on {st['decode_checked']} iterations, "
        f"prefill on {st['prefill_checked']} batches, worst |err| {st['worst']:.2e}; {st['caches']} caches and "
        f"{st['pool_images']} pool images bit-exact; budgets doubled up to {st['doublings']} times")
    assert res["iterations"] == st["iterations"]
    assert st["decode_checked"] >= 3 and st["prefill_checked"] >= 3 and st["caches"] >= 4 and st["doublings"] >= 2
