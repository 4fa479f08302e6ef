"""ukv_decode_attention_static (the entry point for callers that cannot allocate) against ukv_decode_attention.

Runs last (file name) because a failure here must not hide the other GPU tests; it must pass alone in a fresh
process and after the others.  Bar as for every attention output: max |difference| <= 2e-3 (the two entry points
cut the batch differently, so results differ in fp32 summation order only); the oracle is checked beside it.
"""
import sys

import numpy as np
import pytest

import paper_2504_15720_amd as U
from oracle import oracle
from synth import SHAPES, make_batch, make_config
from paper_2504_15720_amd.device_batch import DeviceBatch

pytestmark = pytest.mark.gpu
ATOL = 2e-3


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


class DeviceArrays:
    """The descriptor arrays of (a prefix of) a batch in device memory."""

    def __init__(self, db, n=None):
        torch = db.torch
        b = db.b
        n = b.n_requests if n is None else n
        self.n = n
        put = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a[:n]).astype(dt).view(np.int64 if dt == np.uint64 else np.int32)).to(db.dev)
        self.service_id = put(b.service_id, np.uint32)
        self.ctx_len = put(b.ctx_len, np.uint32)
        self.table_off = put(b.table_off, np.uint64)
        self.q_off = put(b.q_off, np.uint64)
        self.out_off = put(b.out_off, np.uint64)

    def call(self, db, out_t):
        U.ukv_decode_attention_static(db.pool, self.n, self.service_id.data_ptr(), self.ctx_len.data_ptr(),
                                      self.table_off.data_ptr(), db.table_t.data_ptr(), db.q_t.data_ptr(),
                                      self.q_off.data_ptr(), out_t.data_ptr(), self.out_off.data_ptr(), db.stream())


def _compare(db, b, n, tag):
    """Static call on the first n requests against ukv_decode_attention on the same requests, and the oracle."""
    torch = db.torch
    db.out_t.fill_(float("nan"))
    db.decode()                                              # existing entry point, whole batch
    want = db.out_host().astype(np.float64)
    out_t = torch.full_like(db.out_t, float("nan"))
    DeviceArrays(db, n).call(db, out_t)
    got = out_t.cpu().numpy().astype(np.float64)
    end = int(b.out_off[n]) if n < b.n_requests else b.out_elems
    assert np.all(np.isfinite(got[:end])), f"{tag}: non-finite output"
    assert np.all(np.isnan(got[end:])), f"{tag}: wrote outside the requests of the call"
    d = float(np.max(np.abs(got[:end] - want[:end]))) if end else 0.0
    ref = oracle.attention(b, b.pool)
    e = float(np.max(np.abs(got[:end] - ref[:end]))) if end else 0.0
    say(f"  {tag}: {n} requests, max|static - ukv_decode_attention| = {d:.3e}, max|static - oracle| = {e:.3e}")
    assert d <= ATOL and e <= ATOL, tag


@pytest.mark.parametrize("cfg", [5, 3, 4])
def test_static_entry_matches_decode_attention_twice_in_a_row(cfg):
    """Two calls in a row on one GPU's scratch array, the second with a smaller input."""
    say(f"static entry point, miniature workload {cfg}")
    b = make_config(cfg, mini=True)
    db = DeviceBatch(b)
    try:
        _compare(db, b, b.n_requests, f"cfg{cfg} mini, whole batch")
        _compare(db, b, max(1, b.n_requests // 3), f"cfg{cfg} mini, second call, smaller")
        _compare(db, b, b.n_requests, f"cfg{cfg} mini, third call, whole batch again")
    finally:
        db.close()


def test_static_entry_long_requests_and_edge_lengths():
    """One long request is cut into many parts (the many-parts merge kernel); lengths 0 and 1; then a small batch."""
    say("static entry point, long request + edge lengths")
    rng = np.random.default_rng(5)
    services = [SHAPES["70b"], SHAPES["7b"], SHAPES["h12"]]
    sid = np.array([0, 1, 2, 0, 1, 2, 1], np.uint32)
    ctx = np.array([9000, 5000, 3001, 0, 1, 17, 0], np.uint32)
    b = make_batch(services, sid, ctx, 8192, "permutation", rng, pool_seed=3)
    db = DeviceBatch(b)
    try:
        U.ukv_set_param(db.pool, U.UKV_PARAM_MIN_SPAN_BYTES, 64 * 1024)   # many spans, many parts per sequence
        db.resize_workspace()
        _compare(db, b, b.n_requests, "long + edge lengths, 64 KiB spans")
        _compare(db, b, 1, "the long request alone")
        _compare(db, b, 2, "two requests")
    finally:
        db.close()


def test_static_entry_more_sequences_than_plan_threads():
    """300 short requests of the 32- and 40-head services: about 1350 (request, head-slice) sequences, more than the
    plan kernel has threads, so every thread scans several; then a prefix of 7 requests."""
    say("static entry point, 300 short requests")
    rng = np.random.default_rng(9)
    services = [SHAPES["7b"], SHAPES["13b"]]
    sid = rng.integers(0, 2, 300).astype(np.uint32)
    ctx = rng.integers(0, 65, 300).astype(np.uint32)
    b = make_batch(services, sid, ctx, 16384, "permutation", rng, pool_seed=4)
    db = DeviceBatch(b)
    try:
        _compare(db, b, b.n_requests, "300 short requests")
        _compare(db, b, 7, "then 7 of them")
    finally:
        db.close()


def test_static_entry_rejects_what_does_not_fit():
    say("static entry point, size limits")
    b = make_config(1, mini=True)
    db = DeviceBatch(b)
    try:
        da = DeviceArrays(db)
        da.n = U.UKV_STATIC_MAX_REQUESTS + 1                 # refused on the host, before anything is enqueued
        with pytest.raises(U.UkvError) as ei:
            da.call(db, db.out_t)
        assert ei.value.code == U.UKV_ENOSPC and "static scratch" in str(ei.value)
        da.n = 0                                             # an empty batch is fine and does nothing
        da.call(db, db.out_t)
        with pytest.raises(U.UkvError) as ei:
            U.ukv_decode_attention_static(db.pool, 1, 0, 0, 0, 0, 0, 0, 0, 0, db.stream())
        assert ei.value.code == U.UKV_EINVAL
    finally:
        db.close()
