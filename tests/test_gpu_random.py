"""Seeded random batches (services, page sizes, lengths around tile and page-table-window edges) through
prefill attention and decode attention, against the CPU oracle."""
import numpy as np
import pytest

import paper_2504_15720_amd as U
from synth import SHAPES, Service, draw_prefill_inputs, make_batch
from tests.test_gpu_parity import _check_attention
from tests.test_gpu_prefill import _check_rows, say
from tests.ukv_harness import DeviceBatch

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
