"""Seeded random batches (services, page sizes, lengths around tile and page-table-window edges) through
prefill attention, decode attention, sequences of decode steps and the bulk copies, against the CPU oracle."""
import numpy as np
import pytest

import paper_2504_15720_amd as U
from synth import SHAPES, Service, draw_prefill_inputs, make_batch
from tests.test_gpu_parity import _check_attention, _check_gather, _decode_steps
from tests.test_gpu_prefill import _check_rows, say
from paper_2504_15720_amd.device_batch import DeviceBatch

pytestmark = pytest.mark.gpu

SHAPE_POOL = [SHAPES["7b"], SHAPES["13b"], SHAPES["8b"], SHAPES["70b"], Service(16, 8, 128), SHAPES["h12"],
              SHAPES["tiny"], Service(8, 4, 64), Service(4, 1, 128)]
EDGES = [31, 32, 33, 63, 64, 65, 95, 96, 97, 127, 128, 129, 255, 256, 257, 511, 512, 513]


def _sampled_rows(m):
    """First and last rows of a chunk and a few in between."""
    return np.unique(np.concatenate([np.arange(min(m, 3)), np.arange(max(0, m - 3), m), np.arange(0, m, max(1, m // 7))]))


@pytest.mark.parametrize("seed", range(12))
def test_random_batches_match_oracle(seed):
    rng = np.random.default_rng(1000 + seed)
    page = int(rng.choice([1024, 4096, 16384]))
    k = int(rng.integers(2, 5))
    services = [SHAPE_POOL[i] for i in rng.choice(len(SHAPE_POOL), size=k, replace=False)]
    n = int(rng.integers(3, 9))
    sid = rng.integers(0, k, size=n)
    ctx = rng.integers(1, 700 if page == 1024 else 1500, size=n)
    for i in range(n):
        if rng.random() < 0.3:
            ctx[i] = int(rng.choice(EDGES))
    q_len = np.array([int(rng.integers(0, c + 1)) if rng.random() < 0.5 else int(c) for c in ctx])
    need = sum(-(-int(c) * services[int(s)].token_bytes // page) for c, s in zip(ctx, sid))
    say(f"random batch {seed}: page {page}, ctx {ctx.tolist()}, q_len {q_len.tolist()}")
    b = make_batch(services, sid, ctx, int(need * 1.3) + 64, "permutation", rng, page_bytes=page, pool_seed=seed)
    db = DeviceBatch(b)
    try:
        q_bits, q_off, out_off, n_el = draw_prefill_inputs(b, q_len, rng)
        out_t, _ = db.prefill(q_len, q_bits, q_off, out_off, n_el)
        _check_rows(b, out_t.cpu().numpy(), q_bits, q_len, q_off, out_off, rows_of=_sampled_rows, tag=f"prefill {seed}")
        for block in (512, 256):
            U.ukv_set_param(db.pool, U.UKV_PARAM_BLOCK_THREADS, block)
            db.resize_workspace()
            U.ukv_set_param(db.pool, U.UKV_PARAM_MIN_SPAN_BYTES, int(rng.choice([16 * 1024, 64 * 1024, 512 * 1024])))
            _check_attention(db, b, f"decode {seed}, block {block}")
    finally:
        db.close()


STEP_SHAPES = SHAPE_POOL + [Service(2, 1, 64), Service(48, 6, 128)]
STEP_EDGES = [0, 1, 2, 15, 16, 17] + EDGES


@pytest.mark.parametrize("seed", range(16))
def test_random_step_sequences_match_oracle(seed):
    """A few decode iterations (new pages from the library's free list, append and attention as two calls, as
    one launch, or alternating; merge fused or not), then gather, then a chunked scatter of the pool's own
    last tokens, which must leave the pool image as it is."""
    rng = np.random.default_rng(5000 + seed)
    page = int(rng.choice([1024, 2048, 4096, 16384, 65536]))
    k = int(rng.integers(1, 5))
    services = [STEP_SHAPES[i] for i in rng.choice(len(STEP_SHAPES), size=k, replace=False)]
    n = int(rng.integers(1, 12))
    sid = rng.integers(0, k, size=n)
    ctx = rng.integers(0, 600 if page <= 2048 else 1400, size=n)
    for i in range(n):
        if rng.random() < 0.35:
            ctx[i] = int(rng.choice(STEP_EDGES))
    steps = int(rng.integers(2, 7))
    reserve = steps * 3 + 2
    need = sum(-(-(int(c) + reserve) * services[int(s)].token_bytes // page) for c, s in zip(ctx, sid))
    say(f"random steps {seed}: page {page}, ctx {ctx.tolist()}, steps {steps}")
    b = make_batch(services, sid, ctx, int(need * 1.2) + 64, "permutation", rng, page_bytes=page, pool_seed=seed,
                   reserve_tokens=reserve)
    db = DeviceBatch(b)
    try:
        U.ukv_set_param(db.pool, U.UKV_PARAM_BLOCK_THREADS, int(rng.choice([256, 512])))
        U.ukv_set_param(db.pool, U.UKV_PARAM_MIN_SPAN_BYTES, int(rng.choice([16 * 1024, 64 * 1024, 512 * 1024])))
        U.ukv_set_param(db.pool, U.UKV_PARAM_FUSED_MERGE, int(rng.choice([0, 1])))
        db.resize_workspace()
        _decode_steps(db, b, steps, seed=seed, fused=str(rng.choice(["no", "yes", "alternate"])))
        _check_gather(db, b)
        k_t, v_t, kv_off, _ = db.gather_device()
        n_new = np.array([int(rng.integers(0, c + 1)) for c in b.ctx_len], np.uint32)
        tok = np.array([b.services[s].n_kv_heads * b.services[s].head_dim for s in b.service_id], np.int64)
        first = (kv_off.astype(np.int64) + (b.ctx_len.astype(np.int64) - n_new) * tok).astype(np.uint64)
        db.scatter_tokens(n_new, k_t, v_t, first)
        assert np.array_equal(db.pool_host(), b.pool), "chunked scatter of the pool's own tokens changed the pool"
    finally:
        db.close()


def test_sixteen_services_in_one_pool():
    """The largest number of services a pool takes: every supported (head_dim, group) kind, several head
    counts and explicit scales, one launch for decode and one per head_dim for prefill."""
    services = [Service(32, 32, 128), Service(40, 40, 128, 0.11), Service(32, 8, 128), Service(64, 8, 128, 0.07),
                Service(16, 8, 128), Service(4, 1, 128), Service(8, 8, 64), Service(12, 12, 64, 0.2),
                Service(8, 4, 64), Service(2, 1, 64), Service(1, 1, 128, 0.5), Service(8, 1, 128),
                Service(16, 16, 64), Service(24, 12, 64), Service(2, 2, 128), Service(48, 6, 128)]
    assert len(services) == U.UKV_MAX_SERVICES
    rng = np.random.default_rng(77)
    sid = np.concatenate([np.arange(16), rng.integers(0, 16, size=16)])
    ctx = rng.integers(1, 900, size=sid.size)
    need = sum(-(-int(c) * services[int(s)].token_bytes // 16384) for c, s in zip(ctx, sid))
    b = make_batch(services, sid, ctx, int(need * 1.3) + 64, "permutation", rng, pool_seed=7)
    db = DeviceBatch(b)
    try:
        _check_attention(db, b, "16 services, decode")
        q_len = np.minimum(ctx, rng.integers(0, 200, size=sid.size))
        q_bits, q_off, out_off, n_el = draw_prefill_inputs(b, q_len, rng)
        out_t, _ = db.prefill(q_len, q_bits, q_off, out_off, n_el)
        _check_rows(b, out_t.cpu().numpy(), q_bits, q_len, q_off, out_off, rows_of=_sampled_rows, tag="16 services, prefill")
    finally:
        db.close()
