"""Query groups that are not a power of two (and the largest one, 16) at head_dim 128 -- 24/8, 40/8, 12/2, 28/4, 48/4
and 32/2 heads -- and groups of 3 and more at head_dim 64 (24/8, 32/8, 14/2, 32/4 and 32/2 heads: the matrix-core path
at half the row width) through every call that takes a service: decode attention whole and cut (merge inside the launch,
as a second launch with the many-parts kernel these group sizes are sent to), decode steps, a kept plan, the entry
point that allocates nothing, and prefill attention in both forms of the weights; all against the CPU oracle."""
import numpy as np
import pytest

import paper_2504_15720_amd as U
from synth import SHAPES, Service, draw_prefill_inputs, make_batch
from tests.test_gpu_parity import _check_attention, _check_gather, _decode_steps, say
from tests.test_gpu_plan import _plan_steps
from tests.test_gpu_prefill import _check_rows
from paper_2504_15720_amd.device_batch import DeviceBatch

pytestmark = pytest.mark.gpu

GROUPS = [Service(24, 8, 128), Service(40, 8, 128), Service(12, 2, 128), Service(28, 4, 128), Service(48, 4, 128),
          Service(32, 2, 128),                                        # G = 3, 5, 6, 7, 12, 16
          Service(32, 8, 64), Service(32, 4, 64),                     # G = 4, 8 at head_dim 64
          Service(24, 8, 64), Service(14, 2, 64), Service(32, 2, 64)]  # G = 3, 7, 16 at head_dim 64


def _batch(rng, page_bytes=16384, with_others=True, reserve=12):
    services = GROUPS + ([SHAPES["7b"], SHAPES["70b"], SHAPES["h12"]] if with_others else [])
    sid = np.arange(len(services)).repeat(2)
    ctx = rng.integers(1, 1400, size=sid.size)
    ctx[:4] = [1, 33, 513, 2050]
    need = sum(-(-int(c + reserve) * services[int(s)].token_bytes // page_bytes) for c, s in zip(ctx, sid))
    return make_batch(services, sid, ctx, int(need * 1.3) + 64, "permutation", rng, page_bytes=page_bytes,
                      reserve_tokens=reserve, pool_seed=21)


@pytest.mark.parametrize("with_others", [True, False], ids=["mixed pool", "odd groups only"])
def test_decode_attention_and_steps(with_others):
    say(f"group sizes 3, 5, 6, 7, 12, 16; other services in the pool: {with_others}")
    b = _batch(np.random.default_rng(61), with_others=with_others)
    db = DeviceBatch(b)
    try:
        for block in (512, 256):
            U.ukv_set_param(db.pool, U.UKV_PARAM_BLOCK_THREADS, block)
            for fused in (1, 0):
                U.ukv_set_param(db.pool, U.UKV_PARAM_FUSED_MERGE, fused)
                db.resize_workspace()
                _check_attention(db, b, f"block {block}, fused merge {fused}")
                U.ukv_set_param(db.pool, U.UKV_PARAM_MIN_SPAN_BYTES, 32 * 1024)
                _check_attention(db, b, f"block {block}, fused merge {fused}, many cuts")
                U.ukv_set_param(db.pool, U.UKV_PARAM_MIN_SPAN_BYTES, 512 * 1024)
        _check_gather(db, b)
        U.ukv_set_param(db.pool, U.UKV_PARAM_MIN_SPAN_BYTES, 32 * 1024)
        _decode_steps(db, b, 3, seed=62, fused="alternate")
        db.make_plan()
        _plan_steps(db, b, 6, seed=63, tag="kept plan")
    finally:
        db.close()


def test_small_pages_and_one_long_request_in_many_parts():
    rng = np.random.default_rng(64)
    b = _batch(rng, page_bytes=1024, with_others=False, reserve=4)
    db = DeviceBatch(b)
    try:
        _check_attention(db, b, "1 KiB pages")
        U.ukv_set_param(db.pool, U.UKV_PARAM_MIN_SPAN_BYTES, 16 * 1024)
        _check_attention(db, b, "1 KiB pages, many cuts")
    finally:
        db.close()
    for sv in (GROUPS[3], GROUPS[5], GROUPS[7], GROUPS[9]):            # G = 7 and 16, and 8 and 7 at head_dim 64: one request alone on the device
        b = make_batch([sv], np.array([0]), np.array([30000]), 30000 * sv.token_bytes // 16384 + 64, "permutation", rng,
                       pool_seed=22)
        db = DeviceBatch(b)
        try:
            for fused in (1, 0):
                U.ukv_set_param(db.pool, U.UKV_PARAM_FUSED_MERGE, fused)
                db.resize_workspace()
                _check_attention(db, b, f"{sv.n_q_heads}/{sv.n_kv_heads} heads, 30000 tokens, fused merge {fused}")
        finally:
            db.close()


def test_entry_point_that_allocates_nothing():
    from tests.test_zz_no_alloc import _compare
    b = _batch(np.random.default_rng(65))
    db = DeviceBatch(b)
    try:
        _compare(db, b, b.n_requests, "odd groups, whole batch")
        _compare(db, b, 5, "odd groups, five requests")
    finally:
        db.close()


@pytest.mark.parametrize("weights", [2, 1], ids=["two-part", "one-part"])
def test_prefill(weights):
    rng = np.random.default_rng(66)
    services = GROUPS + [SHAPES["8b"]]
    sid = np.array([0, 1, 2, 3, 4, 5, 6, 3, 0, 7, 11, 6, 8, 9, 10])
    ctx = np.array([130, 257, 96, 700, 33, 300, 64, 1, 1500, 200, 64, 513, 300, 129, 77])
    q_len = np.array([130, 100, 96, 700, 33, 1, 64, 1, 300, 200, 17, 513, 300, 100, 77])
    b = make_batch(services, sid, ctx, 8192, "permutation", rng, pool_seed=23)
    db = DeviceBatch(b)
    try:
        U.ukv_set_param(db.pool, U.UKV_PARAM_PREFILL_WEIGHTS, weights)
        q_bits, q_off, out_off, n_el = draw_prefill_inputs(b, q_len, rng)
        out_t, _ = db.prefill(q_len, q_bits, q_off, out_off, n_el)
        out = out_t.cpu().numpy()
        _check_rows(b, out, q_bits, q_len, q_off, out_off, tag="odd groups", weights=weights)
        touched = np.zeros(n_el, bool)                                 # nothing outside the rows of the call is written
        for i in range(b.n_requests):
            s = b.service_of(i)
            touched[int(out_off[i]):int(out_off[i]) + int(q_len[i]) * s.n_q_heads * s.head_dim] = True
        assert np.all(np.isnan(out[~touched]))
    finally:
        db.close()
