"""Pins for the CPU oracle: what the paper and the mathematics fix, independent of the oracle.

Decode attention is softmax(q K^T scale) V over the whole cached context (decode phase,
section 2.1); the merged-block layout is section 4.4.  Each test is chosen so that one class
of mistake in the oracle (wrong head mapping, K/V swapped, wrong stride, missing scale, wrong
normalisation, wrong page slot / second index) makes it fail.
"""
import math
import os

import numpy as np
import pytest

from oracle import oracle
from synth import Service, SHAPES, make_batch, make_config, to_split_layout
from tests.reference_math import (contiguous_causal_attention, torch_sdpa_causal, bits_to_f64, build_paged_pool, contiguous_attention, copy_logical_kv_to_split,
                                  f32_to_bits, torch_sdpa_attention)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "address_map.txt")

CASES = {
    "A": dict(page_bytes=256, H=3, d=8, table=[5, 2, 7, 0], n_pages=8),
    "B": dict(page_bytes=16384, H=32, d=128, table=[9, 4, 6, 1], n_pages=10),
    "C": dict(page_bytes=16384, H=8, d=64, table=[3, 0], n_pages=4),
    "D": dict(page_bytes=16384, H=8, d=128, table=[2, 5], n_pages=6),
    "E": dict(page_bytes=16384, H=40, d=128, table=[1, 0, 3], n_pages=4),
}


def _golden_rows():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            c, t, h, kv, j, addr = line.split()
            rows.append((c, int(t), int(h), int(kv), int(j), int(addr)))
    return rows


def test_address_map_matches_hand_worked_fixture():
    """Pool elements are numbered by their own byte address; gather must return those numbers."""
    rows = _golden_rows()
    assert len(rows) >= 20
    for name, c in CASES.items():
        P = c["page_bytes"]
        n_el = c["n_pages"] * P // 2
        # 16-bit tag of the element index, plus the page number in the high bits of a second image
        idx = np.arange(n_el, dtype=np.int64)
        lo = (idx & 0xFFFF).astype(np.uint16)
        hi = (idx >> 16).astype(np.uint16)
        T = c["H"] * c["d"] * 4
        n_tok = len(c["table"]) * P // T
        klo, vlo = oracle.gather(lo, P, np.array(c["table"]), c["H"], c["d"], n_tok)
        khi, vhi = oracle.gather(hi, P, np.array(c["table"]), c["H"], c["d"], n_tok)
        for (cn, t, h, kv, j, addr) in rows:
            if cn != name:
                continue
            got_lo = (vlo if kv else klo)[t, h, j]
            got_hi = (vhi if kv else khi)[t, h, j]
            assert (int(got_hi) << 16 | int(got_lo)) * 2 == addr, (cn, t, h, kv, j)


def test_token_bytes_closed_form_4gib():
    """One request of 4096+4096 tokens on Llama2-7B needs 4 GB (section 2.3): 32 layers of token_bytes."""
    s = SHAPES["7b"]
    assert s.token_bytes == 32 * 128 * 2 * 2
    assert 8192 * 32 * s.token_bytes == 4 << 30


@pytest.mark.parametrize("shape,tpp", [("tiny", 8), ("7b", 1), ("8b", 4), ("70b", 4)])
def test_integral_tokens_per_page_rule(shape, tpp):
    """Where token_bytes divides the page, token t sits in table[t // tpp] at (t % tpp) * token_bytes."""
    s = SHAPES[shape]
    P = 16384
    assert P // s.token_bytes == tpp
    n_pages, n_tok = 6, 4 * tpp + 1
    table = np.array([4, 1, 5, 0, 2], np.int32)
    pool = (np.arange(n_pages * P // 2) % 65521).astype(np.uint16)
    k, v = oracle.gather(pool, P, table, s.n_kv_heads, s.head_dim, n_tok)
    for t in (0, tpp - 1, tpp, n_tok - 1):
        base = (int(table[t // tpp]) * P + (t % tpp) * s.token_bytes) // 2
        row = pool[base:base + s.token_bytes // 2].reshape(s.n_kv_heads, 2, s.head_dim)
        assert np.array_equal(k[t], row[:, 0, :])
        assert np.array_equal(v[t], row[:, 1, :])


def _random_case(rng, shape: Service, n, page_bytes, n_pages):
    k = f32_to_bits(rng.standard_normal((n, shape.n_kv_heads, shape.head_dim)).astype(np.float32))
    v = f32_to_bits(rng.standard_normal((n, shape.n_kv_heads, shape.head_dim)).astype(np.float32))
    q = f32_to_bits(rng.standard_normal((shape.n_q_heads, shape.head_dim)).astype(np.float32))
    need = -(-n * shape.token_bytes // page_bytes)
    table = rng.permutation(n_pages)[:need].astype(np.int32)
    pool = f32_to_bits(rng.standard_normal(n_pages * page_bytes // 2).astype(np.float32))
    build_paged_pool(pool, page_bytes, table, k, v)
    return q, k, v, table, pool


class _OneRequest:
    """Minimal batch-shaped object for the oracle front end."""

    def __init__(self, shape, n, table, q, page_bytes):
        self.page_bytes = page_bytes
        self.services = [shape]
        self.service_id = np.zeros(1, np.uint32)
        self.ctx_len = np.array([n], np.uint32)
        self.table_off = np.zeros(1, np.uint64)
        self.table_cap = np.array([len(table)], np.int64)
        self.page_table = np.asarray(table, np.int32)
        self.q = q.reshape(-1)
        self.q_off = np.zeros(1, np.uint64)
        self.out_off = np.zeros(1, np.uint64)
        self.out_elems = shape.n_q_heads * shape.head_dim
        self.new_off = np.zeros(1, np.uint64)


SMALL_SHAPES = [Service(4, 4, 16), Service(8, 2, 16), Service(6, 3, 8), Service(16, 2, 32), Service(5, 5, 24)]


@pytest.mark.parametrize("si", range(len(SMALL_SHAPES)))
@pytest.mark.parametrize("n", [1, 2, 7, 33])
def test_oracle_equals_bruteforce_and_torch_on_small_shapes(si, n):
    shape = SMALL_SHAPES[si]
    rng = np.random.default_rng(1000 * si + n)
    page_bytes = 4 * shape.head_dim * 3          # 3 head-rows per page: token rows straddle pages
    n_pages = 2 * (-(-n * shape.token_bytes // page_bytes)) + 3
    q, k, v, table, pool = _random_case(rng, shape, n, page_bytes, n_pages)
    got = oracle.attention(_OneRequest(shape, n, table, q, page_bytes), pool).reshape(shape.n_q_heads, -1)
    ref = contiguous_attention(q, k, v, shape.softmax_scale)
    ref_t = torch_sdpa_attention(q, k, v, shape.softmax_scale)
    assert np.max(np.abs(got - ref)) < 1e-12
    assert np.max(np.abs(got - ref_t)) < 1e-12


@pytest.mark.parametrize("name", ["tiny", "h12", "7b", "13b", "8b", "70b"])
def test_oracle_equals_bruteforce_on_service_shapes(name):
    shape = SHAPES[name]
    rng = np.random.default_rng(abs(hash(name)) % 2**31)
    n = 9
    P = 16384
    n_pages = 2 * (-(-n * shape.token_bytes // P)) + 2
    q, k, v, table, pool = _random_case(rng, shape, n, P, n_pages)
    got = oracle.attention(_OneRequest(shape, n, table, q, P), pool).reshape(shape.n_q_heads, -1)
    assert np.max(np.abs(got - contiguous_attention(q, k, v, shape.softmax_scale))) < 1e-12
    gk, gv = oracle.gather(pool, P, table, shape.n_kv_heads, shape.head_dim, n)
    assert np.array_equal(gk, k) and np.array_equal(gv, v)


def test_explicit_scale_is_used():
    shape = Service(4, 2, 16, scale=0.37)
    rng = np.random.default_rng(5)
    q, k, v, table, pool = _random_case(rng, shape, 12, 192, 20)
    got = oracle.attention(_OneRequest(shape, 12, table, q, 192), pool).reshape(4, 16)
    assert np.max(np.abs(got - contiguous_attention(q, k, v, 0.37))) < 1e-12
    other = contiguous_attention(q, k, v, 0.25)
    assert np.max(np.abs(got - other)) > 1e-4


# ---------------------------------------------------------------- closed forms
def _closed_form_setup(shape, n, rng, k=None, v=None, q=None, page_bytes=None):
    page_bytes = page_bytes or 4 * shape.head_dim * 4
    H, d, Q = shape.n_kv_heads, shape.head_dim, shape.n_q_heads
    k = f32_to_bits(rng.standard_normal((n, H, d)).astype(np.float32)) if k is None else k
    v = f32_to_bits(rng.standard_normal((n, H, d)).astype(np.float32)) if v is None else v
    q = f32_to_bits(rng.standard_normal((Q, d)).astype(np.float32)) if q is None else q
    need = -(-n * shape.token_bytes // page_bytes)
    n_pages = need + 5
    table = rng.permutation(n_pages)[:need].astype(np.int32)
    pool = np.full(n_pages * page_bytes // 2, 0x7FC0, np.uint16)      # NaN everywhere else
    build_paged_pool(pool, page_bytes, table, k, v)
    out = oracle.attention(_OneRequest(shape, n, table, q, page_bytes), pool).reshape(Q, d)
    return out, q, k, v


def test_constant_v_per_kv_head_returns_it_and_pins_gqa_mapping():
    shape = Service(8, 2, 16)
    rng = np.random.default_rng(11)
    n = 19
    consts = f32_to_bits(rng.standard_normal((2, 16)).astype(np.float32))
    v = np.broadcast_to(consts[None], (n, 2, 16)).copy()
    out, *_ = _closed_form_setup(shape, n, rng, v=v)
    expect = bits_to_f64(consts)
    for a in range(8):
        assert np.max(np.abs(out[a] - expect[a // 4])) < 1e-14     # head a reads kv head a // G


def test_single_token_returns_its_value_exactly():
    shape = Service(6, 3, 8)
    rng = np.random.default_rng(12)
    out, q, k, v = _closed_form_setup(shape, 1, rng)
    for a in range(6):
        assert np.array_equal(out[a], bits_to_f64(v[0, a // 2]))


def test_equal_keys_and_zero_query_give_mean_of_values():
    shape = Service(4, 4, 16)
    rng = np.random.default_rng(13)
    n = 23
    krow = f32_to_bits(rng.standard_normal((1, 4, 16)).astype(np.float32))
    out, q, k, v = _closed_form_setup(shape, n, rng, k=np.repeat(krow, n, axis=0))
    assert np.max(np.abs(out - bits_to_f64(v).mean(axis=0))) < 1e-13
    out0, q, k, v = _closed_form_setup(shape, n, rng, q=np.zeros((4, 16), np.uint16))
    assert np.max(np.abs(out0 - bits_to_f64(v).mean(axis=0))) < 1e-13


def test_two_token_logistic_closed_form():
    """q = c e1, K0 = e1, K1 = 0  =>  out = s V0 + (1 - s) V1 with s = 1 / (1 + exp(-c * scale))."""
    shape = Service(1, 1, 16)
    rng = np.random.default_rng(14)
    c = 3.5
    q = np.zeros((1, 16), np.float32); q[0, 0] = c
    k = np.zeros((2, 1, 16), np.float32); k[0, 0, 0] = 1.0
    out, qb, kb, v = _closed_form_setup(shape, 2, rng, k=f32_to_bits(k), q=f32_to_bits(q))
    s = 1.0 / (1.0 + math.exp(-c / math.sqrt(16)))
    vf = bits_to_f64(v)
    assert np.max(np.abs(out[0] - (s * vf[0, 0] + (1 - s) * vf[1, 0]))) < 1e-14


def test_bytes_past_ctx_len_do_not_matter():
    """The pool outside the request's valid tokens holds NaN patterns in _closed_form_setup."""
    shape = Service(4, 2, 8)
    out, *_ = _closed_form_setup(shape, 5, np.random.default_rng(15), page_bytes=32 * 5)
    assert np.all(np.isfinite(out))


def test_empty_context_gives_zeros():
    shape = Service(4, 2, 8)
    b = _OneRequest(shape, 0, np.array([0], np.int32), np.zeros((4, 8), np.uint16), 256)
    out = oracle.attention(b, np.full(1024, 0x7FC0, np.uint16))
    assert np.array_equal(out, np.zeros(32))


# ---------------------------------------------------------------- invariances
def test_page_renaming_is_bit_identical():
    b = make_config(3, mini=True)
    ref = oracle.attention(b, b.pool)
    rng = np.random.default_rng(3)
    perm = rng.permutation(b.n_pages)
    pool2 = np.empty_like(b.pool)
    epp = b.page_bytes // 2
    pool2.reshape(b.n_pages, epp)[perm] = b.pool.reshape(b.n_pages, epp)
    old = b.page_table.copy()
    b.page_table = np.where(old >= 0, perm[np.maximum(old, 0)], -1).astype(np.int32)
    got = oracle.attention(b, pool2)
    assert np.array_equal(ref, got)


def test_token_order_and_score_shift_invariance():
    shape = Service(4, 2, 16)
    rng = np.random.default_rng(21)
    n = 29
    k = rng.standard_normal((n, 2, 16)).astype(np.float32); k[:, :, 5] = 0.0
    out, q, kb, v = _closed_form_setup(shape, n, rng, k=f32_to_bits(k))
    p = rng.permutation(n)
    out_p, *_ = _closed_form_setup(shape, n, rng, k=kb[p], v=v[p], q=q)
    assert np.max(np.abs(out - out_p)) < 1e-13
    k2 = k.copy(); k2[:, :, 5] = 2.0           # adds q[a,5]*2*scale to every score of head a
    out_s, *_ = _closed_form_setup(shape, n, rng, k=f32_to_bits(k2), v=v, q=q)
    assert np.max(np.abs(out - out_s)) < 1e-12


def test_result_is_independent_of_batch_composition():
    b = make_config(5, mini=True)
    full = oracle.attention(b, b.pool)
    for i in (0, 7, b.n_requests - 1):
        one = oracle.attention(b, b.pool, requests=[i])
        o = int(b.out_off[i]); s = b.service_of(i)
        e = s.n_q_heads * s.head_dim
        assert np.array_equal(one[o:o + e], full[o:o + e])


def test_split_and_merge_equals_whole():
    b = make_config(4, mini=True)
    full = oracle.attention(b, b.pool)
    i = int(np.argmax(b.ctx_len))
    s = b.service_of(i)
    n = int(b.ctx_len[i])
    q = b.q[int(b.q_off[i]):int(b.q_off[i]) + s.n_q_heads * s.head_dim]
    cuts = [0, 1, n // 3, n // 3, n - 1, n]       # includes an empty range
    parts = [oracle.attention_range(b.pool, b.page_bytes, b.table_of(i), s.n_q_heads, s.n_kv_heads, s.head_dim,
                                    s.softmax_scale, cuts[c], cuts[c + 1], q) for c in range(len(cuts) - 1)]
    o = int(b.out_off[i])
    for a in range(s.n_q_heads):
        m = np.array([p[0][a] for p in parts]); l = np.array([p[1][a] for p in parts])
        acc = np.stack([p[2][a] for p in parts])
        merged = oracle.merge(m, l, acc)
        assert np.max(np.abs(merged - full[o + a * s.head_dim:o + (a + 1) * s.head_dim])) < 1e-12


# ---------------------------------------------------------------- append
@pytest.mark.parametrize("cfg", [2, 5])
def test_append_touches_exactly_the_new_token(cfg):
    b = make_config(cfg, mini=True)
    rng = np.random.default_rng(77)
    before = b.pool.copy()
    b.grow_one_token()
    _, nk, nv = b.draw_step_inputs(rng)
    oracle.append(b, b.pool, nk, nv)
    changed = np.flatnonzero(before != b.pool)
    kv_elems = sum(2 * b.service_of(i).n_kv_heads * b.service_of(i).head_dim for i in range(b.n_requests))
    assert changed.size <= kv_elems and changed.size > 0.99 * kv_elems   # equal unless a value repeats
    for i in range(b.n_requests):
        s = b.service_of(i)
        n = int(b.ctx_len[i])
        k, v = oracle.gather(b.pool, b.page_bytes, b.table_of(i), s.n_kv_heads, s.head_dim, n)
        o = int(b.new_off[i]); e = s.n_kv_heads * s.head_dim
        assert np.array_equal(k[n - 1].reshape(-1), nk[o:o + e])
        assert np.array_equal(v[n - 1].reshape(-1), nv[o:o + e])
        kb, vb = oracle.gather(before, b.page_bytes, b.table_of(i), s.n_kv_heads, s.head_dim, n - 1)
        assert np.array_equal(k[:n - 1], kb) and np.array_equal(v[:n - 1], vb)
    # element-wise placement, independently: rebuild the new token with the per-element scatter
    ref = before.copy()
    for i in range(b.n_requests):
        s = b.service_of(i)
        o = int(b.new_off[i]); e = s.n_kv_heads * s.head_dim
        build_paged_pool(ref, b.page_bytes, b.table_of(i), nk[o:o + e].reshape(1, s.n_kv_heads, s.head_dim),
                         nv[o:o + e].reshape(1, s.n_kv_heads, s.head_dim), first_token=int(b.ctx_len[i]) - 1)
    assert np.array_equal(ref, b.pool)


@pytest.mark.parametrize("name", ["h12", "13b", "8b"])
def test_scatter_places_every_element_and_inverts_gather(name):
    shape = SHAPES[name]
    rng = np.random.default_rng(77)
    n, P = 11, 16384
    need = -(-n * shape.token_bytes // P)
    table = rng.permutation(need + 4)[:need].astype(np.int32)
    k = f32_to_bits(rng.standard_normal((n, shape.n_kv_heads, shape.head_dim)).astype(np.float32))
    v = f32_to_bits(rng.standard_normal((n, shape.n_kv_heads, shape.head_dim)).astype(np.float32))
    pool = np.full((need + 4) * P // 2, 0xABCD, np.uint16)
    ref = pool.copy()
    oracle.scatter(pool, P, table, k, v)
    build_paged_pool(ref, P, table, k, v)                 # element-by-element placement, test-side
    assert np.array_equal(pool, ref)
    gk, gv = oracle.gather(pool, P, table, shape.n_kv_heads, shape.head_dim, n)
    assert np.array_equal(gk, k) and np.array_equal(gv, v)


@pytest.mark.parametrize("name", ["h12", "13b", "70b"])
def test_scatter_of_a_chunk_is_a_bulk_append(name):
    """Chunks written one after the other give the image of the whole prompt written at once; a chunk touches
    only its own tokens' bytes (sentinel elsewhere); each element sits where the test-side placement puts it;
    a chunk of one token is the single-token append."""
    shape = SHAPES[name]
    rng = np.random.default_rng(78)
    n, P = 23, 16384
    need = -(-n * shape.token_bytes // P)
    table = rng.permutation(need + 3)[:need].astype(np.int32)
    k = f32_to_bits(rng.standard_normal((n, shape.n_kv_heads, shape.head_dim)).astype(np.float32))
    v = f32_to_bits(rng.standard_normal((n, shape.n_kv_heads, shape.head_dim)).astype(np.float32))
    whole = np.full((need + 3) * P // 2, 0xABCD, np.uint16)
    oracle.scatter(whole, P, table, k, v)
    pieces = np.full_like(whole, 0xABCD)
    for lo, hi in ((0, 7), (7, 8), (8, 20), (20, 23)):
        before = pieces.copy()
        oracle.scatter(pieces, P, table, k[lo:hi], v[lo:hi], first_token=lo)
        ref = before.copy()
        build_paged_pool(ref, P, table, k[lo:hi], v[lo:hi], first_token=lo)   # element by element, test-side
        assert np.array_equal(pieces, ref)
        changed = np.flatnonzero(pieces != before)
        assert changed.size <= (hi - lo) * shape.token_bytes // 2             # nothing outside the chunk's bytes
    assert np.array_equal(pieces, whole)
    gk, gv = oracle.gather(pieces, P, table, shape.n_kv_heads, shape.head_dim, n)
    assert np.array_equal(gk, k) and np.array_equal(gv, v)
    # a chunk of one token == the decode step's append of that token
    b = _OneRequest(shape, 8, table, np.zeros((shape.n_q_heads, shape.head_dim), np.uint16), P)
    img = np.full_like(whole, 0xABCD)
    oracle.append(b, img, k[7].reshape(-1), v[7].reshape(-1))
    one = np.full_like(whole, 0xABCD)
    oracle.scatter(one, P, table, k[7:8], v[7:8], first_token=7)
    assert np.array_equal(img, one)


def test_oracle_rejects_missing_pages():
    shape = Service(2, 2, 8)
    b = _OneRequest(shape, 20, np.array([0, -1, 1], np.int32), np.zeros((2, 8), np.uint16), 256)
    with pytest.raises(RuntimeError):
        oracle.attention(b, np.zeros(4 * 128, np.uint16))


# ---------------------------------------------------------------- split-block layout
@pytest.mark.parametrize("page_bytes", [None, 1024])
def test_split_block_layout_gives_the_same_attention(page_bytes):
    """Section 4.4's alternative (a block stream per kv head) changes where bytes live, not the result."""
    b = make_config(3, mini=True)
    s = to_split_layout(b, page_bytes=page_bytes)
    assert s.kv_bytes() == b.kv_bytes() and s.n_requests == sum(b.service_of(i).n_kv_heads for i in range(b.n_requests))
    copy_logical_kv_to_split(b, s, oracle.gather)
    ref = oracle.attention(b, b.pool)
    got = oracle.attention(s, s.pool)
    assert np.max(np.abs(ref - got)) < 1e-13
    # Table accounting for one layer of the 7B shape.  Equal tokens per block (2 tokens: a merged
    # block of 32 KiB against per-head blocks of 1 KiB): the split table is n_kv_heads = 32 times
    # larger; over 32 layers that is the 1024 x of section 4.4.  Equal block BYTES instead (the
    # workloads here: 16 KiB either way) gives tables of practically equal size.
    from synth import pages_for_tokens
    sv = SHAPES["7b"]
    n = 4096
    merged_entries = int(pages_for_tokens(n, sv.token_bytes, 32768))
    split_entries = sv.n_kv_heads * int(pages_for_tokens(n, sv.head_row_bytes, 1024))
    assert split_entries == 32 * merged_entries and 32 * 32 == 1024
    if page_bytes is None:
        assert abs(int(s.pages_owned().sum()) / int(b.pages_owned().sum()) - 1.0) < 0.2


# ---------------------------------------------------------------- prefill phase (section 2.1), causal


def _prefill_case(rng, shape, n, page_bytes):
    n_pages = 2 * (-(-n * shape.token_bytes // page_bytes)) + 3
    _, k, v, table, pool = _random_case(rng, shape, n, page_bytes, n_pages)
    q = f32_to_bits(rng.standard_normal((n, shape.n_q_heads, shape.head_dim)).astype(np.float32))
    return q, k, v, table, pool


@pytest.mark.parametrize("si", range(len(SMALL_SHAPES)))
@pytest.mark.parametrize("n", [1, 2, 19])
def test_prefill_equals_masked_matrix_and_torch_causal(si, n):
    shape = SMALL_SHAPES[si]
    rng = np.random.default_rng(7000 + 10 * si + n)
    P = 4 * shape.head_dim * 3
    q, k, v, table, pool = _prefill_case(rng, shape, n, P)
    got = oracle.prefill(pool, P, table, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.softmax_scale,
                         n, np.arange(n), q)
    assert np.max(np.abs(got - contiguous_causal_attention(q, k, v, shape.softmax_scale))) < 1e-12
    assert np.max(np.abs(got - torch_sdpa_causal(q, k, v, shape.softmax_scale))) < 1e-12


def test_prefill_chunk_of_the_last_positions_and_service_shapes():
    """A chunk: only the last m positions are queried (chunked prefill); real head shapes and 16 KiB pages."""
    for name, n, m in (("8b", 11, 4), ("13b", 6, 6), ("h12", 13, 5)):
        shape = SHAPES[name]
        rng = np.random.default_rng(len(name) * 100 + n)
        q, k, v, table, pool = _prefill_case(rng, shape, n, 16384)
        pos = np.arange(n - m, n)
        got = oracle.prefill(pool, 16384, table, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                             shape.softmax_scale, n, pos, q[pos])
        ref = contiguous_causal_attention(q[pos], k, v, shape.softmax_scale, first_pos=n - m)
        assert np.max(np.abs(got - ref)) < 1e-12


def test_prefill_closed_forms_and_causality():
    shape = Service(8, 2, 16)
    rng = np.random.default_rng(77)
    n, P = 12, 4 * 16 * 3
    q, k, v, table, pool = _prefill_case(rng, shape, n, P)
    args = (P, table, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.softmax_scale, n)
    got = oracle.prefill(pool, *args, np.arange(n), q)
    # position 0 sees one token: its value, exactly, for every query head of the group
    v0 = bits_to_f64(v[0])                                                       # [H, d]
    assert np.array_equal(got[0], np.repeat(v0, shape.group, axis=0))
    # the last position is a decode step over the whole context (a different entry point)
    dec = oracle.attention(_OneRequest(shape, n, table, q[n - 1], P), pool).reshape(shape.n_q_heads, -1)
    assert np.max(np.abs(got[n - 1] - dec)) < 1e-15
    # zero queries: position p returns the mean of values 0..p
    zq = np.zeros_like(q)
    gz = oracle.prefill(pool, *args, np.arange(n), zq)
    vf = bits_to_f64(v)
    for p_ in (0, 3, n - 1):
        assert np.max(np.abs(gz[p_] - np.repeat(vf[:p_ + 1].mean(axis=0), shape.group, axis=0))) < 1e-12
    # causality: rewriting the cache of tokens after p does not change position p
    pool2 = pool.copy()
    k2, v2 = k.copy(), v.copy()
    k2[7:], v2[7:] = k2[7:] ^ 0x8000, v2[7:] ^ 0x8000                            # flip signs of tokens 7..
    build_paged_pool(pool2, P, table, k2, v2)
    g2 = oracle.prefill(pool2, *args, np.arange(n), q)
    assert np.array_equal(g2[:7], got[:7]) and not np.allclose(g2[7:], got[7:])
    # positions are looked up, not assumed consecutive; rows follow the order of the list
    pick = np.array([9, 2, 2, 11])
    gp = oracle.prefill(pool, *args, pick, q[pick])
    assert np.array_equal(gp, got[pick])
    with pytest.raises(RuntimeError):
        oracle.prefill(pool, *args, np.array([n]), q[:1])                        # position outside the context
