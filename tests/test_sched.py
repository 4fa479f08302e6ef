"""Doubling-budget scheduler (section 4.2 and the DB algorithm of the appendix): pins of the Python
oracle, planted mistakes, and decision-by-decision parity of the C++ scheduler behind
include/ukv_sched.h with the oracle on seeded traces.  Host code only: no GPU."""
import itertools
import os

import numpy as np
import pytest

import paper_2504_15720_amd as U
from oracle import db_scheduler as dbs
from synth import SHAPES

PAGE = 16384
FAKE_BASE = 1 << 40


def _profiles(times, stds=None, thr=None, token_bytes=None):
    n = len(times)
    stds = stds or [0.0] * n
    thr = thr or [1e30] * n
    token_bytes = token_bytes or [4096] * n
    return [dbs.ServiceProfile(times[i], stds[i], thr[i], token_bytes[i]) for i in range(n)]


def _run_single_slot(sched, iters_of, tau, arrivals=()):
    """One request per iteration (max_batch = 1), every iteration takes tau; request r needs iters_of[r]
    iterations.  arrivals: (time, id, service) added when the clock reaches them.  Returns completion times."""
    now, done_iters, completion = 0.0, {}, {}
    pending = sorted(arrivals)
    while sched.requests or pending:
        while pending and pending[0][0] <= now + 1e-12:
            _, rid, svc = pending.pop(0)
            sched.add_request(rid, svc, 1, now)
        ids, _, _ = sched.next_batch(now, 10 ** 9)
        if not ids:
            now = pending[0][0]
            continue
        assert len(ids) == 1
        now += tau
        rid = ids[0]
        done_iters[rid] = done_iters.get(rid, 0) + 1
        fin = done_iters[rid] == iters_of[rid]
        if fin:
            completion[rid] = now
        sched.complete(ids, [fin], tau, now)
    return completion


def test_order_is_optimal_for_summed_normalized_latency_when_the_theorem_applies():
    """First theorem of section 4.2: with equal execution times within a service (and requests that
    can be preempted between iterations) the priority order minimises the sum of latency / profiled
    time.  Everything queued at time 0, one request per iteration: brute force over all run-to-completion
    orders (for this objective without release times an optimal order needs no preemption)."""
    tau = 1.0
    for n_iters, counts in (((2, 5), (3, 3)), ((4, 3, 7), (2, 2, 2)), ((1, 6), (4, 2))):
        prof = _profiles([k * tau for k in n_iters])
        sched = dbs.DBScheduler(prof, PAGE, max_batch=1)
        svc_of, iters_of = {}, {}
        rid = 0
        for s, c in enumerate(counts):
            for _ in range(c):
                svc_of[rid], iters_of[rid] = s, n_iters[s]
                rid += 1
        # interleave the arrival order so that the queue order is not already the answer
        for r in sorted(svc_of, key=lambda x: (x * 7) % len(svc_of)):
            sched.add_request(r, svc_of[r], 1, 0.0)
        comp = _run_single_slot(sched, iters_of, tau)
        got = sum(comp[r] / prof[svc_of[r]].mean_time for r in comp)
        best = min(
            sum(c / prof[svc_of[r]].mean_time
                for r, c in zip(order, itertools.accumulate(iters_of[r] * tau for r in order)))
            for order in itertools.permutations(svc_of))
        assert abs(got - best) < 1e-9, (got, best)


def test_priority_uses_remaining_budget_times_profiled_time():
    """Equation 6 with a partly executed request: A (profiled 10, 2 left) against a new B (profiled 3).
    O_A = 2 * 10 = 20 > O_B = 3 * 3 = 9, so B preempts A; that is also the better of the two possible
    schedules (2.3 against 2.67 summed normalized latency, worked by hand)."""
    prof = _profiles([10.0, 3.0])
    sched = dbs.DBScheduler(prof, PAGE, max_batch=1)
    sched.add_request(0, 0, 1, 0.0)
    comp = _run_single_slot(sched, {0: 10, 1: 3}, 1.0, arrivals=[(8.0, 1, 1)])
    assert comp == {1: 11.0, 0: 13.0}
    assert abs((comp[1] - 8.0) / 3.0 + comp[0] / 10.0 - 2.3) < 1e-12


def test_budget_doubles_each_time_it_is_used_up():
    prof = _profiles([2.0], stds=[1.0])          # Q = L + Var = 3
    sched = dbs.DBScheduler(prof, PAGE, max_batch=4)
    sched.add_request(7, 0, 5, 0.0)
    seen = []
    now = 0.0
    for _ in range(12):
        ids, svc, queue = sched.next_batch(now, 100)
        assert ids == [7]
        now += 1.0
        sched.complete(ids, [False], 1.0, now)
        r = sched.requests[7]
        seen.append((r.budget, r.doublings, r.priority))
    budgets = [b for b, _, _ in seen]
    assert budgets == [2.0, 1.0, 6.0, 5.0, 4.0, 3.0, 2.0, 1.0, 12.0, 11.0, 10.0, 9.0]      # Q, then 2Q, then 4Q
    assert [k for _, k, _ in seen] == [0, 0, 1, 1, 1, 1, 1, 1, 2, 2, 2, 2]
    assert all(p == b * 2.0 for b, _, p in seen)                                           # O = Q_r * L_s
    assert sched.requests[7].queue == dbs.DECODING and sched.requests[7].ctx_len == 5 + 11


def test_starved_service_is_served_first():
    prof = _profiles([1.0, 50.0], thr=[1e30, 5.0])
    sched = dbs.DBScheduler(prof, PAGE, max_batch=1)
    sched.add_request(100, 1, 1, 0.0)            # low priority: O = 2500
    now, served_at = 0.0, None
    for k in range(20):
        sched.add_request(k, 0, 1, now)          # a steady stream of short requests, O = 1
        ids, svc, _ = sched.next_batch(now, 100)
        now += 1.0
        if svc == 1:
            served_at = now - 1.0
            sched.complete(ids, [True], 1.0, now)
            break
        sched.complete(ids, [True], 1.0, now)
    assert served_at is not None and 5.0 < served_at <= 6.0 + 1e-9


def test_batches_hold_one_service_one_phase_and_fit_the_free_pages():
    rng = np.random.default_rng(5)
    shapes = [SHAPES["7b"], SHAPES["8b"], SHAPES["13b"]]
    prof = _profiles([1.0, 0.4, 2.0], stds=[0.5, 0.1, 1.0], thr=[8.0, 8.0, 8.0],
                     token_bytes=[s.token_bytes for s in shapes])
    sched = dbs.DBScheduler(prof, PAGE, max_batch=8)
    now, rid, free = 0.0, 0, 400
    owned = {}
    for step in range(300):
        for _ in range(rng.integers(0, 3)):
            sched.add_request(rid, int(rng.integers(0, 3)), int(rng.integers(1, 40)), now)
            rid += 1
        ids, svc, queue = sched.next_batch(now, free)
        if not ids:
            now += 0.1
            continue
        reqs = [sched.requests[i] for i in ids]
        assert all(r.service == svc and r.queue == queue for r in reqs) and len(ids) <= 8
        assert [sched._key(r) for r in reqs[1:]] == sorted(sched._key(r) for r in reqs[1:])
        need = [sched.pages_needed(r) for r in reqs]
        assert sum(need) <= free
        for r, n in zip(reqs, need):
            owned[r.id] = owned.get(r.id, 0) + n
        free -= sum(need)
        fin = [bool(rng.random() < 0.08) and queue == dbs.DECODING for _ in ids]
        now += 0.05 * len(ids)
        sched.complete(ids, fin, 0.05 * len(ids), now)
        for i, f in zip(ids, fin):
            if f:
                free += owned.pop(i)
    assert free + sum(owned.values()) == 400


# ------------------------------------------------------------------ planted mistakes (in a copy of the oracle)

MUTATIONS = {
    "priority without the profiled time": ("r.priority = r.budget * s.mean_time", "r.priority = r.budget"),
    "budget reset instead of doubled": ("float(2 ** r.doublings)", "1.0"),
    "largest priority value first": ("return (r.priority, r.arrival, r.id)", "return (-r.priority, r.arrival, r.id)"),
    "starvation ignored": ("if over > 0.0 and", "if False and"),
    "batch mixes services": ("if r.service != first.service:\n                continue", "if False:\n                continue"),
}


def _pins(mod, monkeypatch):
    monkeypatch.setattr(dbs, "DBScheduler", mod.DBScheduler)
    test_order_is_optimal_for_summed_normalized_latency_when_the_theorem_applies()
    test_priority_uses_remaining_budget_times_profiled_time()
    test_budget_doubles_each_time_it_is_used_up()
    test_starved_service_is_served_first()
    test_batches_hold_one_service_one_phase_and_fit_the_free_pages()


def _load_copy(text):
    import types
    mod = types.ModuleType("db_scheduler_copy")
    mod.__dict__["__name__"] = "db_scheduler_copy"
    import sys
    sys.modules["db_scheduler_copy"] = mod           # dataclasses looks the module up by name
    exec(compile(text, "db_scheduler_copy.py", "exec"), mod.__dict__)
    return mod


def test_unmutated_copy_passes(monkeypatch):
    _pins(_load_copy(open(dbs.__file__).read()), monkeypatch)


@pytest.mark.parametrize("name", list(MUTATIONS))
def test_planted_scheduler_mistake_is_caught(name, monkeypatch):
    old, new = MUTATIONS[name]
    text = open(dbs.__file__).read()
    assert text.count(old) == 1, name
    mod = _load_copy(text.replace(old, new))
    with pytest.raises(AssertionError):
        _pins(mod, monkeypatch)


# ------------------------------------------------------------------ the C++ scheduler against the oracle


def _trace_parity(seed, n_steps, services, profiles, max_batch, n_pages):
    """Drive both schedulers with the same seeded arrivals, execution times and finishes; pages come from
    the library's real free list.  Every decision must be identical."""
    rng = np.random.default_rng(seed)
    pool = U.ukv_pool_create(FAKE_BASE, n_pages * PAGE, PAGE, services)
    sched = U.ukv_sched_create(pool, profiles, max_batch)
    ref = dbs.DBScheduler([dbs.ServiceProfile(m, s, t, sv.token_bytes) for (m, s, t), sv in zip(profiles, services)],
                          PAGE, max_batch)
    owned, now, rid = {}, 0.0, 0
    n_batches = n_empty = n_prefill = 0
    try:
        for _ in range(n_steps):
            for _ in range(int(rng.integers(0, 3))):
                svc, plen = int(rng.integers(0, len(services))), int(rng.integers(1, 300))
                U.ukv_sched_add_request(sched, rid, svc, plen, now)
                ref.add_request(rid, svc, plen, now)
                rid += 1
            free = int(U.ukv_pool_info(pool, 0).free_pages)
            got = U.ukv_sched_next_batch(sched, now, free, cap=max_batch)
            want = ref.next_batch(now, free)
            assert got == (want[0], want[1], want[2]), (got, want)
            ids, svc, queue = got
            if not ids:
                n_empty += 1
                now += 0.05
                # make room: finish the request that owns the most pages
                if owned and U.ukv_sched_pending(sched):
                    victim = max(owned, key=lambda k: len(owned[k]))
                    info = U.ukv_sched_request_info(sched, victim)
                    if info.queue == U.UKV_SCHED_DECODING:
                        U.ukv_sched_complete(sched, [victim], [1], 0.0, now)
                        ref.complete([victim], [True], 0.0, now)
                        U.ukv_pages_free(pool, owned.pop(victim))
                continue
            n_batches += 1
            n_prefill += queue == U.UKV_SCHED_WAIT
            for i in ids:                                   # take the pages the iteration needs
                need = U.ukv_sched_pages_needed(sched, i)
                assert need == ref.pages_needed(ref.requests[i])
                if need:
                    owned.setdefault(i, []).extend(U.ukv_pages_alloc(pool, need).tolist())
            elapsed = float(rng.uniform(0.01, 0.3))
            now += elapsed
            fin = [bool(queue == U.UKV_SCHED_DECODING and rng.random() < 0.03) for _ in ids]
            U.ukv_sched_complete(sched, ids, fin, elapsed, now)
            ref.complete(ids, fin, elapsed, now)
            for i, f in zip(ids, fin):
                if f and i in owned:
                    U.ukv_pages_free(pool, owned.pop(i))
            for i, f in zip(ids, fin):                     # state of the survivors
                if not f:
                    a, b = U.ukv_sched_request_info(sched, i), ref.requests[i]
                    assert (a.queue, a.ctx_len, a.doublings, a.budget, a.priority) == \
                           (b.queue, b.ctx_len, b.doublings, b.budget, b.priority)
        assert U.ukv_sched_pending(sched) == len(ref.requests)
    finally:
        U.ukv_sched_destroy(sched)
        U.ukv_pool_destroy(pool)
    return n_batches, n_empty, n_prefill


def test_cpp_scheduler_matches_the_oracle_decision_by_decision():
    services = [SHAPES["7b"], SHAPES["8b"], SHAPES["13b"], SHAPES["h12"]]
    profiles = [(1.0, 0.5, 4.0), (0.3, 0.1, 4.0), (2.5, 2.0, 6.0), (0.1, 0.05, 2.0)]
    n_batches, n_empty, n_prefill = _trace_parity(11, 1500, services, profiles, max_batch=16, n_pages=6000)
    assert n_batches > 1000 and n_prefill > 100
    # a small pool: EnoughResource() cuts batches short and sometimes nothing fits
    n_batches, n_empty, _ = _trace_parity(12, 1200, services, profiles, max_batch=8, n_pages=700)
    assert n_batches > 300 and n_empty > 10
    # no starvation thresholds in reach, one request per batch
    _trace_parity(13, 600, services[:2], [(1.0, 0.0, 1e30), (3.0, 1.0, 1e30)], max_batch=1, n_pages=4000)


def test_cpp_scheduler_rejects_bad_arguments():
    services = [SHAPES["7b"], SHAPES["8b"]]
    pool = U.ukv_pool_create(FAKE_BASE, 64 * PAGE, PAGE, services)
    try:
        with pytest.raises(U.UkvError):
            U.ukv_sched_create(pool, [(1.0, 0.0, 1.0)], 4)                      # one profile per service
        with pytest.raises(U.UkvError):
            U.ukv_sched_create(pool, [(0.0, 0.0, 1.0), (1.0, 0.0, 1.0)], 4)     # mean_time must be positive
        with pytest.raises(U.UkvError):
            U.ukv_sched_create(pool, [(1.0, 0.0, 1.0), (1.0, 0.0, 1.0)], 0)
        sched = U.ukv_sched_create(pool, [(1.0, 0.0, 1.0), (1.0, 0.0, 1.0)], 4)
        U.ukv_sched_add_request(sched, 5, 1, 10, 0.0)
        for bad in ((5, 0, 10), (6, 2, 10), (7, 0, 0)):                         # duplicate id, bad service, empty prompt
            with pytest.raises(U.UkvError):
                U.ukv_sched_add_request(sched, *bad, 0.0)
        with pytest.raises(U.UkvError):
            U.ukv_sched_complete(sched, [99], [0], 1.0, 1.0)
        with pytest.raises(U.UkvError) as e:
            U.ukv_sched_next_batch(sched, 0.0, 100, cap=2)
        assert e.value.code == U.UKV_ENOSPC
        assert U.ukv_sched_next_batch(sched, 0.0, 0, cap=4) == ([], 1, U.UKV_SCHED_WAIT)   # nothing fits
        assert U.ukv_sched_next_batch(sched, 0.0, 100, cap=4) == ([5], 1, U.UKV_SCHED_WAIT)
        U.ukv_sched_destroy(sched)
    finally:
        U.ukv_pool_destroy(pool)
