"""Opt-in check of device page tables (UKV_PARAM_VALIDATE) on the GPU.  The check only reads the table, and a call
whose table holds a page id outside the pool does nothing (its kernels leave at once), so nothing here can make the
device read or write through a bad id; with the check off such a table is never used."""
import sys

import numpy as np
import pytest

import paper_2504_15720_amd as U
from oracle import oracle
from paper_2504_15720_amd.device_batch import DeviceBatch
from synth import make_config

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def test_bad_table_entries_stop_the_call_and_are_reported():
    say("page-table check")
    b = make_config(3, mini=True, reserve_tokens=6)
    db = DeviceBatch(b)
    torch = db.torch
    try:
        U.ukv_set_param(db.pool, U.UKV_PARAM_VALIDATE, 1)
        db.decode()                                              # good tables: results as without the check
        got = db.out_host().astype(np.float64)
        assert float(np.max(np.abs(got - oracle.attention(b, b.pool)))) <= 2e-3
        pool_before = db.pool_host().copy()

        victim = 2
        entry = int(b.table_off[victim]) + 1
        good = int(b.page_table[entry])
        for bad_id in (b.n_pages, -1):
            db.table_t[entry] = bad_id
            db.out_t.fill_(float("nan"))
            db.decode()                                          # enqueued; the kernels find the flag and leave
            torch.cuda.synchronize()
            assert bool(torch.isnan(db.out_t).all()), "a checked call with a bad table wrote outputs"
            with pytest.raises(U.UkvError) as ei:                # the next call reports it
                db.decode()
            assert ei.value.code == U.UKV_EINVAL and f"page id {bad_id}" in str(ei.value) and \
                f"page_table[{entry}]" in str(ei.value) and f"request {victim}" in str(ei.value), str(ei.value)
            # the store side too: nothing is written through the table
            rng = np.random.default_rng(3)
            _, nk, nv = b.draw_step_inputs(rng)
            db.set_new(nk, nv)
            db.append(db.desc())
            torch.cuda.synchronize()
            assert np.array_equal(db.pool_host(), pool_before), "a checked append with a bad table wrote to the pool"
            with pytest.raises(U.UkvError):
                db.decode()
            db.table_t[entry] = good
            torch.cuda.synchronize()
        db.out_t.fill_(float("nan"))
        db.decode()                                              # repaired: works again
        got = db.out_host().astype(np.float64)
        assert float(np.max(np.abs(got - oracle.attention(b, b.pool)))) <= 2e-3

        # a kept plan under the check: steps match the oracle, new entries ride in the kernel arguments
        db.make_plan()
        rng = np.random.default_rng(4)
        for step in range(4):
            entry_, ids = b.grow_one_token()
            if ids.size:
                assert np.array_equal(U.ukv_pages_alloc(db.pool, ids.size), ids)
            q, nk, nv = b.draw_step_inputs(rng)
            b.q = q
            db.set_q(q)
            db.set_new(nk, nv)
            oracle.append(b, b.pool, nk, nv)
            db.plan_step(ids)
            err = float(np.max(np.abs(db.out_host().astype(np.float64) - oracle.attention(b, b.pool))))
            assert err <= 2e-3, f"step {step}: {err}"
        assert np.array_equal(db.pool_host(), b.pool)
        say("  bad ids reported, outputs and pool untouched; good tables: same results")
    finally:
        db.close()
