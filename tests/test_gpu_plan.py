"""GPU parity of the decode plan that outlives its step (ukv_plan_create / ukv_plan_step): every step against the
oracle -- pool image and page tables bit for bit, attention within 2e-3 -- on steps served by the resident plan
(one launch, new page ids in the kernel arguments) and on steps that remake it.
"""
import sys

import numpy as np
import pytest

import paper_2504_15720_amd as U
from oracle import oracle
from paper_2504_15720_amd.device_batch import DeviceBatch
from synth import SHAPES, Service, make_batch, make_config

pytestmark = pytest.mark.gpu
ATOL = 2e-3


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _plan_steps(db, b, steps, seed, check_every=1, tag=""):
    """steps x (grow, ukv_plan_step) with the oracle mirroring the pool image on the host."""
    rng = np.random.default_rng(seed)
    worst = 0.0
    for step in range(steps):
        entry, ids = b.grow_one_token()
        lib_ids = U.ukv_pages_alloc(db.pool, ids.size) if ids.size else np.zeros(0, np.int32)
        assert np.array_equal(lib_ids, ids), "library free list diverged from the synthetic stack"
        q, nk, nv = b.draw_step_inputs(rng)
        b.q = q
        db.set_q(q)
        db.set_new(nk, nv)
        oracle.append(b, b.pool, nk, nv)
        db.plan_step(ids)
        if step % check_every == 0 or step == steps - 1:
            got = db.out_host().astype(np.float64)
            ref = oracle.attention(b, b.pool)
            assert np.all(np.isfinite(got)), f"{tag} step {step}: non-finite output"
            err = float(np.max(np.abs(got - ref)))
            worst = max(worst, err)
            assert err <= ATOL, f"{tag} step {step}: max |err| {err}"
    say(f"  {tag}: {steps} steps, worst max|err| = {worst:.3e}")
    assert np.array_equal(U.ukv_plan_lengths(db.plan, b.n_requests), b.ctx_len), "plan lengths differ"
    assert np.array_equal(db.table_t.cpu().numpy(), b.page_table), "device page table differs"
    assert np.array_equal(db.pool_host(), b.pool), "pool image differs after the steps"


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("fused_merge", [1, 0])
def test_kept_plan_mini_configs(cfg, fused_merge):
    say(f"kept plan, mini cfg {cfg}, fused merge {fused_merge}")
    b = make_config(cfg, mini=True, reserve_tokens=40)
    db = DeviceBatch(b)
    try:
        U.ukv_set_param(db.pool, U.UKV_PARAM_FUSED_MERGE, fused_merge)
        U.ukv_set_param(db.pool, U.UKV_PARAM_MIN_SPAN_BYTES, 48 * 1024)     # many cuts: growing last parts, merges
        U.ukv_set_param(db.pool, U.UKV_PARAM_REPLAN_EVERY, 5)
        db.resize_workspace()
        db.make_plan()
        _plan_steps(db, b, 14, seed=200 + cfg, tag="48 KiB spans, remade every 5 tokens")   # plans at steps 0, 6, 12
        U.ukv_set_param(db.pool, U.UKV_PARAM_MERGE_ACQ_REL, 1)
        _plan_steps(db, b, 3, seed=250 + cfg, tag="48 KiB spans, acquire-release count")
        U.ukv_set_param(db.pool, U.UKV_PARAM_MERGE_ACQ_REL, 0)
        U.ukv_set_param(db.pool, U.UKV_PARAM_MIN_SPAN_BYTES, 512 * 1024)    # set_param: the next step remakes the plan
        U.ukv_set_param(db.pool, U.UKV_PARAM_REPLAN_EVERY, 64)
        _plan_steps(db, b, 12, seed=300 + cfg, tag="512 KiB spans, one plan")
    finally:
        db.close()


def test_kept_plan_small_pages_several_new_entries_per_token():
    """1 KiB pages: a token row takes 4 to 20 pages, so every step adds several table entries per request, across
    page-table windows; group sizes outside the workloads; lengths that start at 0 and 1."""
    say("kept plan, 1 KiB pages")
    services = [SHAPES["13b"], SHAPES["70b"], Service(16, 8, 128), Service(8, 4, 64), SHAPES["h12"], Service(4, 1, 128)]
    sid = np.array([0, 1, 2, 3, 4, 5, 0, 1, 2, 3, 4, 5])
    ctx = np.array([37, 1200, 515, 64, 3, 700, 1, 0, 16, 0, 300, 31])
    rng = np.random.default_rng(321)
    b = make_batch(services, sid, ctx, 64 * 1024, "permutation", rng, page_bytes=1024, reserve_tokens=24, pool_seed=9)
    db = DeviceBatch(b)
    try:
        db.make_plan()
        _plan_steps(db, b, 10, seed=21, tag="block 512")
        U.ukv_set_param(db.pool, U.UKV_PARAM_BLOCK_THREADS, 256)
        U.ukv_set_param(db.pool, U.UKV_PARAM_MIN_SPAN_BYTES, 16 * 1024)
        db.resize_workspace()
        db.make_plan()
        _plan_steps(db, b, 10, seed=22, tag="block 256, 16 KiB spans")
    finally:
        db.close()


def test_kept_plan_full_size_config5_sixteen_steps():
    say("kept plan, full cfg 5, 16 x (append + attention), one plan")
    b = make_config(5)
    db = DeviceBatch(b)
    try:
        db.make_plan()
        _plan_steps(db, b, 16, seed=405, check_every=5, tag="cfg 5")
    finally:
        db.close()


def test_kept_plan_full_size_config3():
    say("kept plan, full cfg 3, 6 steps, one plan")
    b = make_config(3, reserve_tokens=8)
    db = DeviceBatch(b)
    try:
        db.make_plan()
        _plan_steps(db, b, 6, seed=403, check_every=3, tag="cfg 3")
    finally:
        db.close()


def test_kept_plan_too_many_requests_for_the_kernel_arguments():
    """800 short requests: more than the step's page ids can ride with in the kernel arguments, so every step takes
    the plan-and-upload route; results are the same."""
    say("kept plan, 800 requests")
    rng = np.random.default_rng(77)
    sid = rng.integers(0, 2, 800)
    ctx = rng.integers(0, 40, 800)
    b = make_batch([SHAPES["8b"], SHAPES["h12"]], sid, ctx, 8192, "permutation", rng, reserve_tokens=6, pool_seed=2)
    db = DeviceBatch(b)
    try:
        db.make_plan()
        _plan_steps(db, b, 4, seed=31, tag="800 requests")
    finally:
        db.close()


def test_kept_plan_two_tables_of_one_iteration():
    """Two page tables for the same requests (two layers of one engine): the second is stepped through the io
    argument without advancing the lengths, with its own page ids, inputs and outputs."""
    say("kept plan, two tables per request")
    import copy
    import torch
    rng = np.random.default_rng(55)
    services = [SHAPES["7b"], SHAPES["8b"], SHAPES["h12"]]
    sid = np.array([0, 1, 2, 0, 1, 2, 1])
    ctx = np.array([700, 1500, 90, 33, 1, 0, 2049])
    b0 = make_batch(services, sid, ctx, 16384, "permutation", rng, reserve_tokens=12, pool_seed=6)
    b1 = copy.copy(b0)                                  # second table: same requests, other pages of the same pool
    b1.page_table = np.full_like(b0.page_table, -1)
    b1.ctx_len = np.zeros_like(b0.ctx_len)
    # bring the second table to the same lengths: pages from the same stack, content scattered by the oracle
    db = DeviceBatch(b0)
    try:
        tb = b0.token_bytes()
        need = -(-ctx.astype(np.int64) * tb // b0.page_bytes)
        for i in range(b0.n_requests):
            if need[i]:
                ids = b0.stack.alloc(int(need[i]))
                assert np.array_equal(U.ukv_pages_alloc(db.pool, ids.size), ids)
                b1.page_table[int(b1.table_off[i]):int(b1.table_off[i]) + ids.size] = ids
        b1.ctx_len = b0.ctx_len.copy()
        # the pool image under the second table is whatever the fill put there: fine, both sides read the same bytes
        table1_t = torch.from_numpy(b1.page_table.copy()).to(db.dev)
        q1_t, out1_t = torch.zeros_like(db.q_t), torch.full_like(db.out_t, float("nan"))
        nk1_t, nv1_t = torch.zeros_like(db.newk_t), torch.zeros_like(db.newv_t)
        io1 = (table1_t.data_ptr(), q1_t.data_ptr(), out1_t.data_ptr(), nk1_t.data_ptr(), nv1_t.data_ptr())
        db.make_plan()
        for step in range(7):
            _, ids0 = b0.grow_one_token()
            if ids0.size:
                assert np.array_equal(U.ukv_pages_alloc(db.pool, ids0.size), ids0)
            _, ids1 = b1.grow_one_token()               # same stack object: the next pages
            if ids1.size:
                assert np.array_equal(U.ukv_pages_alloc(db.pool, ids1.size), ids1)
            q0, nk0, nv0 = b0.draw_step_inputs(rng)
            q1, nk1, nv1 = b0.draw_step_inputs(rng)
            b0.q, b1.q = q0, q1
            db.set_q(q0)
            db.set_new(nk0, nv0)
            q1_t.copy_(torch.from_numpy(q1.view(np.int16)))
            nk1_t.copy_(torch.from_numpy(nk1.view(np.int16)))
            nv1_t.copy_(torch.from_numpy(nv1.view(np.int16)))
            oracle.append(b0, b0.pool, nk0, nv0)
            oracle.append(b1, b0.pool, nk1, nv1)
            U.ukv_plan_step(db.plan, ids0, True, None, db.stream())
            U.ukv_plan_step(db.plan, ids1, False, io1, db.stream())
            e0 = float(np.max(np.abs(db.out_host().astype(np.float64) - oracle.attention(b0, b0.pool))))
            e1 = float(np.max(np.abs(out1_t.cpu().numpy().astype(np.float64) - oracle.attention(b1, b0.pool))))
            say(f"  step {step}: max|err| first table {e0:.2e}, second table {e1:.2e}")
            assert e0 <= ATOL and e1 <= ATOL
        assert np.array_equal(db.table_t.cpu().numpy(), b0.page_table)
        assert np.array_equal(table1_t.cpu().numpy(), b1.page_table)
        assert np.array_equal(db.pool_host(), b0.pool)
    finally:
        db.close()


def test_kept_plan_rejects_wrong_page_lists_and_changes_nothing():
    say("kept plan, error paths")
    b = make_config(3, mini=True, reserve_tokens=6)
    db = DeviceBatch(b)
    try:
        db.make_plan()
        _plan_steps(db, b, 2, seed=1, tag="two good steps")
        before = U.ukv_plan_lengths(db.plan, b.n_requests).copy()
        tb = b.token_bytes()
        n_new = int((-(-(b.ctx_len.astype(np.int64) + 1) * tb // b.page_bytes) - -(-b.ctx_len.astype(np.int64) * tb // b.page_bytes)).sum())
        assert n_new > 0
        with pytest.raises(U.UkvError) as ei:
            db.plan_step(np.zeros(n_new + 1, np.int32))                       # one page id too many
        assert ei.value.code == U.UKV_EINVAL
        with pytest.raises(U.UkvError) as ei:
            db.plan_step(np.full(n_new, b.n_pages, np.int32))                 # page id out of range
        assert ei.value.code == U.UKV_EINVAL
        assert np.array_equal(U.ukv_plan_lengths(db.plan, b.n_requests), before)
        _plan_steps(db, b, 2, seed=2, tag="two more good steps")
    finally:
        db.close()
