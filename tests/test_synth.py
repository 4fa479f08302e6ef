"""Properties of the seeded input generators (structure only, no attention math)."""
import numpy as np
import pytest

from synth import (CONFIGS, PageStack, SHAPES, bf16_bits_to_f32, f32_to_bf16_bits, lockstep_order, make_config,
                   pages_for_tokens)


def test_bf16_rounding_is_nearest_even_and_exact_roundtrip():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e-5], np.float32)   # 1+2^-8 ties to even (1.0)
    b = f32_to_bf16_bits(x)
    assert b[0] == 0x3F80 and b[1] == 0x3F80 and b[2] == 0x3F82
    back = bf16_bits_to_f32(b)
    assert np.array_equal(f32_to_bf16_bits(back), b)
    assert np.all(np.abs(back - x) <= np.abs(x) * 2.0 ** -8)


def test_page_stack_is_lifo_and_logs():
    s = PageStack(8)
    a = s.alloc(3)
    assert list(a) == [0, 1, 2]
    s.free(np.array([1, 0]))
    assert list(s.alloc(3)) == [0, 1, 3]
    assert [op for op, _ in s.log] == ["alloc", "free", "alloc"]
    with pytest.raises(MemoryError):
        s.alloc(6)


def test_lockstep_order_interleaves_services():
    # 7B-shaped (1 page per token) and 13B-shaped (1.25 pages per token), three tokens each
    tb = np.array([16384, 20480])
    order = lockstep_order(pages_for_tokens([3, 3], tb), tb)
    # token 0: seq0 page0, seq1 pages 0 and 1 (its first row is 20480 B); token 1: seq0, seq1 ...
    assert list(order[:3]) == [0, 1, 1]
    assert np.bincount(order).tolist() == [3, 4]


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_config_tables_are_disjoint_and_sized(cfg):
    b = make_config(cfg, mini=True, fill_pool=False)
    owned = b.pages_owned()
    seen = []
    for i in range(b.n_requests):
        t = b.table_of(i)
        assert np.all(t[:owned[i]] >= 0) and np.all(t[owned[i]:] == -1)
        seen.append(t[:owned[i]])
    allp = np.concatenate(seen)
    assert allp.size == np.unique(allp).size and allp.max() < b.n_pages
    assert b.stack.used_pages == allp.size
    assert set(b.stack.peek_order().tolist()).isdisjoint(allp.tolist())


def test_full_size_configs_fit_and_match_stated_shapes():
    for cfg, n_req in ((1, 8), (2, 64), (3, 128), (4, 256), (5, 512)):
        b = make_config(cfg, fill_pool=False)
        assert b.n_requests == n_req
        assert b.notes["pages_needed"] <= b.n_pages
        law = CONFIGS[cfg]["law"]
        hi = law.get("hi", law.get("max"))
        assert b.ctx_len.max() <= hi and b.ctx_len.min() >= 1
    b3 = make_config(3, fill_pool=False)
    assert [s for s in b3.services] == [SHAPES["7b"], SHAPES["13b"]]
    assert np.array_equal(b3.service_id, np.arange(128) % 2)


def test_churn_scrambles_free_list_and_is_deterministic():
    a = make_config(4, mini=True, fill_pool=False)
    b = make_config(4, mini=True, fill_pool=False)
    assert np.array_equal(a.page_table, b.page_table)
    first = a.table_of(0)[:4]
    assert not np.array_equal(np.sort(first), first) or np.any(np.diff(first) != 1)


def test_grow_one_token_allocates_when_a_page_boundary_is_crossed():
    b = make_config(5, mini=True, fill_pool=False)
    for _ in range(16):
        before = b.pages_owned().copy()
        entry, ids = b.grow_one_token()
        after = b.pages_owned()
        assert ids.size == int((after - before).sum())
        assert np.array_equal(b.page_table[entry.astype(np.int64)], ids)


def test_as_stated_pool_admits_a_prefix_that_fits():
    """Workloads whose stated pool is smaller than the drawn batch: with as_stated the pool keeps the stated size
    and the requests are admitted in draw order while pages remain."""
    for cfg in (1, 2, 3):
        full = make_config(cfg, fill_pool=False)
        b = make_config(cfg, fill_pool=False, as_stated=True)
        assert b.n_pages == b.notes["stated_pages"] < full.n_pages
        assert 0 < b.n_requests < full.n_requests == b.notes["drawn_requests"]
        n = b.n_requests
        assert np.array_equal(b.ctx_len, full.ctx_len[:n]) and np.array_equal(b.service_id, full.service_id[:n])
        assert int(b.pages_owned().sum()) <= b.n_pages
        # with room for the tokens the run will add, the admitted requests fit and one more would not
        reserve = int(b.notes["reserve_tokens"])
        tb = np.array([s.token_bytes for s in full.services], np.int64)[full.service_id]
        held = np.cumsum(pages_for_tokens(full.ctx_len + reserve, tb, full.page_bytes))
        assert held[n - 1] <= b.n_pages < held[n]
    for cfg in (4, 5):  # these fit as stated: nothing changes
        a, b = make_config(cfg, fill_pool=False, mini=True), make_config(cfg, fill_pool=False, mini=True, as_stated=True)
        assert a.n_requests == b.n_requests and a.n_pages == b.n_pages
