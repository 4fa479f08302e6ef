"""CPU-only checks of the C-ABI library: exported symbols, pool validation, block manager,
and the split-KV planner (no device work is launched)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2504_15720_amd as U
from synth import SHAPES, PageStack, Service, make_config, pages_for_tokens

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE_BASE = 1 << 32          # never dereferenced on the host


def _pool(services, n_pages=1024, page_bytes=16384, base=FAKE_BASE):
    return U.ukv_pool_create(base, n_pages * page_bytes, page_bytes, services)


def test_library_exports_every_declared_symbol():
    header = "".join(open(os.path.join(ROOT, "include", h)).read()
                     for h in sorted(os.listdir(os.path.join(ROOT, "include"))) if h.endswith(".h"))
    declared = set(re.findall(r"\b(ukv_[a-z_]+)\s*\(", header))
    assert declared == set(U.EXPORTS), declared ^ set(U.EXPORTS)
    L = C.CDLL(U.LIB_PATH)
    for name in declared:
        assert hasattr(L, name), name


def test_pool_info_matches_the_paper_closed_form():
    p = _pool([SHAPES["7b"], SHAPES["13b"], SHAPES["8b"], SHAPES["tiny"], SHAPES["h12"]])
    i7 = U.ukv_pool_info(p, 0)
    assert i7.token_bytes == 16384 and i7.head_row_bytes == 512 and i7.group == 1
    assert 8192 * 32 * i7.token_bytes == 4 << 30             # one 4096+4096-token request: 4 GB (section 2.3)
    assert U.ukv_pool_info(p, 1).token_bytes == 20480
    assert U.ukv_pool_info(p, 2).token_bytes == 4096 and U.ukv_pool_info(p, 2).group == 4
    for s, shape in enumerate(["7b", "13b", "8b", "tiny", "h12"]):
        for n in (0, 1, 3, 4, 5, 1000, 32768):
            assert U.ukv_pages_for_tokens(p, s, n) == int(pages_for_tokens(n, SHAPES[shape].token_bytes))
        inf = U.ukv_pool_info(p, s)
        assert inf.heads_per_slice * inf.n_slices == inf.n_kv_heads
    # split (per-head) blocks would need n_kv_heads x the table entries of merged blocks: 32 x per layer,
    # x 32 layers = the 1024 x of section 4.4
    assert (i7.token_bytes // i7.head_row_bytes) * 32 == 1024
    U.ukv_pool_destroy(p)


@pytest.mark.parametrize("kwargs,services", [
    (dict(page_bytes=1000), [SHAPES["7b"]]),
    (dict(page_bytes=512), [SHAPES["tiny"]]),
    (dict(page_bytes=2 << 20, n_pages=8), [SHAPES["7b"]]),   # above the 1 MiB page limit
    (dict(base=FAKE_BASE + 64), [SHAPES["7b"]]),
    (dict(), [Service(32, 32, 96)]),            # unsupported head_dim
    (dict(), [Service(30, 4, 128)]),            # q heads not a multiple of kv heads
    (dict(), [Service(34, 2, 128)]),            # group 17: more query heads than a product has columns
    (dict(), [Service(34, 2, 64)]),             # the same at head_dim 64
    (dict(), []),
    (dict(n_pages=0), [SHAPES["7b"]]),
])
def test_pool_create_rejects_bad_descriptors(kwargs, services):
    with pytest.raises(U.UkvError) as e:
        _pool(services, **kwargs)
    assert e.value.code == U.UKV_EINVAL


def test_free_list_is_lifo_and_matches_the_synthetic_stack():
    b = make_config(5, mini=True, fill_pool=False)
    p = _pool(b.services, n_pages=b.n_pages)
    ref = PageStack(b.n_pages)
    for op, arg in b.stack.log:
        if op == "alloc":
            assert np.array_equal(U.ukv_pages_alloc(p, arg), ref.alloc(arg))
        else:
            U.ukv_pages_free(p, arg)
            ref.free(arg)
    assert U.ukv_pool_info(p, 0).free_pages == b.stack.free_pages
    nxt = U.ukv_pages_alloc(p, 10)
    assert np.array_equal(nxt, b.stack.peek_order()[:10])
    U.ukv_pool_destroy(p)


def test_free_list_error_paths_leave_state_unchanged():
    p = _pool([SHAPES["7b"]], n_pages=8)
    a = U.ukv_pages_alloc(p, 5)
    assert list(a) == [0, 1, 2, 3, 4]
    with pytest.raises(U.UkvError) as e:
        U.ukv_pages_alloc(p, 4)
    assert e.value.code == U.UKV_ENOMEM
    for bad in ([5], [8], [-1], [1, 1], [2, 6]):
        with pytest.raises(U.UkvError) as e:
            U.ukv_pages_free(p, bad)
        assert e.value.code == U.UKV_EINVAL
    assert U.ukv_pool_info(p, 0).free_pages == 3
    U.ukv_pages_free(p, [3, 1])
    assert list(U.ukv_pages_alloc(p, 3)) == [1, 3, 5]
    U.ukv_pool_destroy(p)


def _check_plan(b, p):
    d = U.BatchDesc(b.service_id, b.ctx_len, b.table_off, q_off=b.q_off, out_off=b.out_off)
    info, items = U.ukv_plan_decode(p, d)
    assert info.kv_bytes == b.kv_bytes()
    # every (request, kv head, token) is covered exactly once
    for i in range(b.n_requests):
        s = b.service_of(i)
        rows = items[items[:, 0] == i]
        cover = np.zeros((s.n_kv_heads, max(int(b.ctx_len[i]), 1)), np.int32)
        for (_, h0, nh, t0, t1, _) in rows:
            assert t0 <= t1 <= b.ctx_len[i]
            cover[h0:h0 + nh, t0:t1] += 1
        if b.ctx_len[i]:
            assert np.all(cover == 1), i
        else:
            assert rows.shape[0] >= 1 and np.all(cover == 0)
    spans = items[:, 5]
    assert np.all(np.diff(spans.astype(np.int64)) >= 0) and spans.max() + 1 == info.n_spans
    ws = U.ukv_decode_workspace_bytes(p, b.n_requests)
    assert info.plan_bytes + 256 + 4 * info.partial_floats <= ws
    return info, items


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("block", [256, 512])
def test_plan_covers_every_token_once(cfg, block):
    b = make_config(cfg, mini=True, fill_pool=False)
    p = _pool(b.services, n_pages=b.n_pages)
    U.ukv_set_param(p, U.UKV_PARAM_BLOCK_THREADS, block)
    _check_plan(b, p)
    U.ukv_set_param(p, U.UKV_PARAM_MIN_SPAN_BYTES, 64 * 1024)     # force many cuts
    for fused in (1, 0):
        # the second launch merges every cut sequence, or (merge inside the decode launch) only those whose
        # partials add up to more than 64 Ki floats
        U.ukv_set_param(p, U.UKV_PARAM_FUSED_MERGE, fused)
        info, items = _check_plan(b, p)
        key = items[:, 0].astype(np.int64) * 4096 + items[:, 1]
        _, first, parts = np.unique(key, return_index=True, return_counts=True)
        assert np.any(parts > 1)
        stride = []
        for row in items[first]:
            si = U.ukv_pool_info(p, int(b.service_id[row[0]]))
            stride.append(-(-(int(row[2]) * si.group * (si.head_dim + 2)) // 32) * 32)
        big = parts * np.array(stride) > 64 * 1024
        assert info.n_reduce == int(np.sum((parts > 1) & (big if fused else True)))
    U.ukv_set_param(p, U.UKV_PARAM_MAX_SPANS, 3)
    info, _ = _check_plan(b, p)
    assert info.n_spans <= 8
    # spans smaller than an item's overhead and a small span limit: the plan still covers everything, stays within
    # 2 * limit + 2 spans (what the workspace is sized for) and within the workspace bound (checked by _check_plan)
    U.ukv_set_param(p, U.UKV_PARAM_MIN_SPAN_BYTES, 16 * 1024)
    U.ukv_set_param(p, U.UKV_PARAM_MAX_SPANS, 16)
    info, items = _check_plan(b, p)
    assert info.n_spans <= 2 * 16 + 2
    assert np.all((items[:, 4] - items[:, 3] >= 16) | (items[:, 4] == b.ctx_len[items[:, 0]]) | (items[:, 3] == 0))
    U.ukv_pool_destroy(p)


def test_plan_full_size_configs_balance_and_fit_workspace():
    for cfg in (3, 4):
        b = make_config(cfg, fill_pool=False)
        p = _pool(b.services, n_pages=b.n_pages)
        tb = np.array([U.ukv_pool_info(p, int(s)).head_row_bytes for s in b.service_id], np.int64)

        def per_span_cost():
            info, items = _check_plan(b, p)
            cost = (items[:, 4] - items[:, 3]).astype(np.int64) * items[:, 2] * tb[items[:, 0]]
            return np.bincount(items[:, 5], weights=cost, minlength=info.n_spans)

        U.ukv_set_param(p, U.UKV_PARAM_TAPER, 0)          # equal spans
        per_span = per_span_cost()
        assert per_span.max() < 1.25 * per_span.mean()
        U.ukv_set_param(p, U.UKV_PARAM_TAPER, 50)         # batches of `slots` spans, each half the rest
        U.ukv_set_param(p, U.UKV_PARAM_SLOTS, 512)
        U.ukv_set_param(p, U.UKV_PARAM_GQA_COST_PCT, 100)
        per_span = per_span_cost()
        first, second = per_span[:512], per_span[512:1024]
        assert 0.4 < second.mean() / first.mean() < 0.6
        assert per_span[-256:].mean() < 0.5 * first.mean()
        assert abs(first.sum() / per_span.sum() - 0.5) < 0.05
        U.ukv_set_param(p, U.UKV_PARAM_TAPER, 1)          # default share of the first batch
        per_span = per_span_cost()
        assert abs(per_span[:512].sum() / per_span.sum() - 0.88) < 0.03
        for bad in (-1, 3, 96):
            with pytest.raises(U.UkvError):
                U.ukv_set_param(p, U.UKV_PARAM_TAPER, bad)
        U.ukv_pool_destroy(p)


def test_plan_cost_weight_of_matrix_core_services():
    """A grouped-query (d = 128) byte counts gqa_cost_pct percent of another byte.  With equal spans of
    a fixed minimum size, doubling the weight doubles the span count of an all-grouped-query batch
    and leaves an all-multi-head batch alone."""
    counts = {}
    for cfg in (3, 4):
        b = make_config(cfg, fill_pool=False)
        p = _pool(b.services, n_pages=b.n_pages)
        assert U.ukv_get_param(p, U.UKV_PARAM_GQA_COST_PCT) == 150
        U.ukv_set_param(p, U.UKV_PARAM_TAPER, 0)
        U.ukv_set_param(p, U.UKV_PARAM_MIN_SPAN_BYTES, 8 << 20)
        for w in (100, 200):
            U.ukv_set_param(p, U.UKV_PARAM_GQA_COST_PCT, w)
            info, _ = _check_plan(b, p)
            counts[cfg, w] = info.n_spans
        with pytest.raises(U.UkvError):
            U.ukv_set_param(p, U.UKV_PARAM_GQA_COST_PCT, 10)
        U.ukv_pool_destroy(p)
    assert counts[3, 100] == counts[3, 200]
    assert abs(counts[4, 200] / counts[4, 100] - 2.0) < 0.05


def test_plan_handles_empty_contexts_and_bad_batches():
    svc = [SHAPES["7b"], SHAPES["8b"]]
    p = _pool(svc)
    d = U.BatchDesc([0, 1, 0], [0, 5, 0], [0, 1, 3], q_off=[0, 4096, 8192], out_off=[0, 4096, 8192])
    info, items = U.ukv_plan_decode(p, d)
    assert info.n_items == info.n_seqs and info.n_reduce == 0
    with pytest.raises(U.UkvError):
        U.ukv_plan_decode(p, U.BatchDesc([2], [5], [0]))
    with pytest.raises(U.UkvError):
        U.ukv_plan_decode(p, U.BatchDesc([0], [5], [0], q_off=[4]))
    with pytest.raises(U.UkvError):
        U.ukv_plan_decode(p, U.BatchDesc([0], [5000], [0]))      # more tokens than the pool holds
    U.ukv_pool_destroy(p)


def test_params_roundtrip_and_validation():
    p = _pool([SHAPES["13b"]])
    assert U.ukv_get_param(p, U.UKV_PARAM_BLOCK_THREADS) == 512
    assert U.ukv_pool_info(p, 0).heads_per_slice == 8 and U.ukv_pool_info(p, 0).token_lanes == 4
    U.ukv_set_param(p, U.UKV_PARAM_BLOCK_THREADS, 256)
    assert U.ukv_pool_info(p, 0).heads_per_slice == 8 and U.ukv_pool_info(p, 0).token_lanes == 2
    U.ukv_set_param(p, U.UKV_PARAM_BLOCK_THREADS, 512)
    U.ukv_set_param(p, U.UKV_PARAM_HEADS_PER_SLICE, 20)
    assert U.ukv_pool_info(p, 0).heads_per_slice == 20
    with pytest.raises(U.UkvError):
        U.ukv_set_param(p, U.UKV_PARAM_BLOCK_THREADS, 128)
    with pytest.raises(U.UkvError):
        U.ukv_set_param(p, 99, 1)
    U.ukv_pool_destroy(p)
    # pools of grouped-query (d = 128) services only start with four-wave workgroups
    p = _pool([SHAPES["8b"], SHAPES["70b"]])
    assert U.ukv_get_param(p, U.UKV_PARAM_BLOCK_THREADS) == 256
    assert U.ukv_pool_info(p, 1).heads_per_slice == 4
    assert U.ukv_get_param(p, U.UKV_PARAM_FUSED_MERGE) == 0       # ... and merge their (large) partials in a second launch
    U.ukv_pool_destroy(p)
    p = _pool([SHAPES["8b"], SHAPES["7b"]])
    assert U.ukv_get_param(p, U.UKV_PARAM_BLOCK_THREADS) == 512
    assert U.ukv_get_param(p, U.UKV_PARAM_FUSED_MERGE) == 1
    U.ukv_pool_destroy(p)
