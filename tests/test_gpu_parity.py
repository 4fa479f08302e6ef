"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bars: append, page-table patches and gather are bit-exact; attention outputs (fp32 accumulation
over bf16 K/V) agree with the fp64 oracle within max |err| <= 2e-3.
"""
import sys

import numpy as np
import pytest

import paper_2504_15720_amd as U
from oracle import oracle
from synth import SHAPES, Service, make_batch, make_config, to_split_layout
from tests.reference_math import copy_logical_kv_to_split
from paper_2504_15720_amd.device_batch import DeviceBatch

pytestmark = pytest.mark.gpu
ATOL = 2e-3


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _check_attention(db, b, tag, run=None):
    (run or db.decode)()
    got = db.out_host().astype(np.float64)
    ref = oracle.attention(b, b.pool)
    assert np.all(np.isfinite(got)), f"{tag}: non-finite output"
    err = float(np.max(np.abs(got - ref)))
    say(f"  {tag}: max|err| = {err:.3e}")
    assert err <= ATOL, f"{tag}: max |err| {err}"
    return err


def _check_gather(db, b):
    k, v, kv_off, sizes = db.gather()
    for i in range(b.n_requests):
        s = b.service_of(i)
        n = int(b.ctx_len[i])
        if n == 0:
            continue
        rk, rv = oracle.gather(b.pool, b.page_bytes, b.table_of(i), s.n_kv_heads, s.head_dim, n)
        o = int(kv_off[i])
        assert np.array_equal(k[o:o + int(sizes[i])], rk.reshape(-1)), f"gather K mismatch, request {i}"
        assert np.array_equal(v[o:o + int(sizes[i])], rv.reshape(-1)), f"gather V mismatch, request {i}"


def _decode_steps(db, b, steps, seed, check_every=1, fused="no"):
    """steps x (grow, append, attention) with the oracle mirroring the pool image on the host.
    fused: "no" = ukv_append then ukv_decode_attention; "yes" = ukv_decode_step (one launch);
    "alternate" = odd steps fused."""
    rng = np.random.default_rng(seed)
    for step in range(steps):
        one_launch = fused == "yes" or (fused == "alternate" and step % 2 == 1)
        entry, ids = b.grow_one_token()
        lib_ids = U.ukv_pages_alloc(db.pool, ids.size) if ids.size else np.zeros(0, np.int32)
        assert np.array_equal(lib_ids, ids), "library free list diverged from the synthetic stack"
        q, nk, nv = b.draw_step_inputs(rng)
        b.q = q
        db.set_q(q)
        db.set_new(nk, nv)
        oracle.append(b, b.pool, nk, nv)
        if one_launch:
            desc = db.desc(entry, ids)
            if step % check_every == 0 or step == steps - 1:
                _check_attention(db, b, f"step {step} (one launch)", run=lambda: db.step(desc))
            else:
                db.step(desc)
            continue
        db.append(db.desc(entry, ids))
        if step % check_every == 0 or step == steps - 1:
            _check_attention(db, b, f"step {step}")
    assert np.array_equal(db.table_t.cpu().numpy(), b.page_table), "device page table differs"
    assert np.array_equal(db.pool_host(), b.pool), "pool image differs after append"


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("block", [256, 512])
def test_mini_configs_match_oracle(cfg, block):
    say(f"mini cfg {cfg} block {block}")
    b = make_config(cfg, mini=True, reserve_tokens=12)
    db = DeviceBatch(b)
    try:
        U.ukv_set_param(db.pool, U.UKV_PARAM_BLOCK_THREADS, block)
        db.resize_workspace()
        _check_attention(db, b, "whole-request items")
        _check_gather(db, b)
        U.ukv_set_param(db.pool, U.UKV_PARAM_MIN_SPAN_BYTES, 48 * 1024)      # many cuts -> merge of partials
        U.ukv_set_param(db.pool, U.UKV_PARAM_FUSED_MERGE, 1)                 # (the default except for all-GQA pools)
        _check_attention(db, b, "cut into many items, merge fused into the decode launch")
        U.ukv_set_param(db.pool, U.UKV_PARAM_MERGE_ACQ_REL, 1)               # items counted with acquire-release
        _check_attention(db, b, "cut into many items, merge fused, acquire-release count")
        U.ukv_set_param(db.pool, U.UKV_PARAM_MERGE_ACQ_REL, 0)
        U.ukv_set_param(db.pool, U.UKV_PARAM_FUSED_MERGE, 0)
        _check_attention(db, b, "cut into many items, merge in a second launch")
        U.ukv_set_param(db.pool, U.UKV_PARAM_FUSED_MERGE, 1)
        steps = max(1, int(b.notes["steps"]))
        _decode_steps(db, b, min(steps, 4), seed=cfg)
        _decode_steps(db, b, 2, seed=50 + cfg, fused="yes")                    # last items are cut parts
        U.ukv_set_param(db.pool, U.UKV_PARAM_MIN_SPAN_BYTES, 512 * 1024)
        _decode_steps(db, b, 2, seed=60 + cfg, fused="yes")                    # mostly whole requests
        U.ukv_set_param(db.pool, U.UKV_PARAM_FUSED_MERGE, 0)
        U.ukv_set_param(db.pool, U.UKV_PARAM_MIN_SPAN_BYTES, 48 * 1024)
        _decode_steps(db, b, 1, seed=70 + cfg, fused="yes")
    finally:
        db.close()


def test_edge_cases_empty_single_and_ragged():
    say("edge cases")
    services = [SHAPES["7b"], SHAPES["13b"], SHAPES["8b"], SHAPES["70b"], SHAPES["tiny"], SHAPES["h12"]]
    sid = np.array([0, 1, 2, 3, 4, 5, 0, 1, 2, 3, 4, 5, 1, 5])
    ctx = np.array([0, 0, 0, 0, 0, 0, 1, 1, 1, 1, 1, 1, 257, 1031])
    rng = np.random.default_rng(99)
    b = make_batch(services, sid, ctx, 2048, "permutation", rng, reserve_tokens=2, pool_seed=5)
    db = DeviceBatch(b)
    try:
        _check_attention(db, b, "ctx 0/1/ragged")
        got = db.out_host()
        for i in range(6):
            s = b.service_of(i); o = int(b.out_off[i])
            assert np.all(got[o:o + s.n_q_heads * s.head_dim] == 0.0)
        for i in range(6, 12):        # one token: output is that token's V exactly
            s = b.service_of(i); o = int(b.out_off[i])
            _, v = oracle.gather(b.pool, b.page_bytes, b.table_of(i), s.n_kv_heads, s.head_dim, 1)
            vf = (v.astype(np.uint32) << 16).view(np.float32)[0]
            assert np.array_equal(got[o:o + s.n_q_heads * s.head_dim].reshape(s.n_kv_heads, s.group, s.head_dim),
                                  np.repeat(vf[:, None, :], s.group, axis=1))
        _decode_steps(db, b, 2, seed=3)       # 0 -> 1 -> 2 tokens, including first-page allocation
    finally:
        db.close()
    b = make_batch(services, sid, ctx, 2048, "permutation", np.random.default_rng(99), reserve_tokens=2, pool_seed=5)
    db = DeviceBatch(b)
    try:
        _decode_steps(db, b, 2, seed=3, fused="yes")   # the same, store and attention in one launch
    finally:
        db.close()


def test_small_pages_and_group_sizes_outside_the_workloads():
    """1 KiB pages (token rows of 4 to 20 pages: page-table windows, the two-launch append) and the
    group sizes the five workloads do not use (G = 2 at both head dims)."""
    say("small pages, G=2 shapes")
    services = [SHAPES["13b"], SHAPES["70b"], Service(16, 8, 128), Service(8, 4, 64), SHAPES["h12"],
                Service(4, 1, 128)]
    sid = np.array([0, 1, 2, 3, 4, 5, 0, 1, 2, 3, 4, 5])
    ctx = np.array([37, 1200, 515, 64, 3, 700, 1, 33, 16, 17, 300, 31])
    rng = np.random.default_rng(123)
    b = make_batch(services, sid, ctx, 64 * 1024, "permutation", rng, page_bytes=1024, reserve_tokens=9,
                   pool_seed=9)
    db = DeviceBatch(b)
    try:
        for block in (512, 256):
            U.ukv_set_param(db.pool, U.UKV_PARAM_BLOCK_THREADS, block)
            db.resize_workspace()
            _check_attention(db, b, f"block {block}")
            U.ukv_set_param(db.pool, U.UKV_PARAM_MIN_SPAN_BYTES, 16 * 1024)
            _check_attention(db, b, f"block {block}, many cuts")
            U.ukv_set_param(db.pool, U.UKV_PARAM_MIN_SPAN_BYTES, 512 * 1024)
        _check_gather(db, b)
        _decode_steps(db, b, 3, seed=11)
        _decode_steps(db, b, 3, seed=12, fused="yes")     # several new pages per token and request
        U.ukv_set_param(db.pool, U.UKV_PARAM_MIN_SPAN_BYTES, 16 * 1024)
        _decode_steps(db, b, 2, seed=13, fused="alternate")
    finally:
        db.close()


def test_bytes_past_ctx_len_are_never_read_into_the_result():
    say("poison test")
    b = make_config(5, mini=True)
    ref = oracle.attention(b, b.pool)
    # poison every element that is not a valid token of some request with NaN / Inf patterns
    valid = np.zeros(b.pool.size, bool)
    for i in range(b.n_requests):
        s = b.service_of(i)
        n_bytes = int(b.ctx_len[i]) * s.token_bytes
        tab = b.table_of(i)
        for slot in range(-(-n_bytes // b.page_bytes)):
            lo = int(tab[slot]) * b.page_bytes // 2
            cnt = min(b.page_bytes, n_bytes - slot * b.page_bytes) // 2
            valid[lo:lo + cnt] = True
    poison = np.where(np.arange(b.pool.size) % 2 == 0, 0x7FC0, 0xFF80).astype(np.uint16)
    b.pool = np.where(valid, b.pool, poison)
    assert np.array_equal(oracle.attention(b, b.pool), ref)
    db = DeviceBatch(b)
    try:
        for block in (256, 512):
            U.ukv_set_param(db.pool, U.UKV_PARAM_BLOCK_THREADS, block)
            _check_attention(db, b, f"poisoned pool, block {block}")
        U.ukv_set_param(db.pool, U.UKV_PARAM_MIN_SPAN_BYTES, 32 * 1024)
        _check_attention(db, b, "poisoned pool, many cuts")
    finally:
        db.close()


def test_append_changes_only_the_new_token_bytes():
    say("append sentinel test")
    b = make_config(5, mini=True)
    b.pool[:] = 0xABCD
    db = DeviceBatch(b)
    try:
        _decode_steps_no_attention(db, b, 3)
    finally:
        db.close()
    b = make_config(5, mini=True)
    b.pool[:] = 0xABCD
    db = DeviceBatch(b)
    try:
        _decode_steps_no_attention(db, b, 3, fused=True)      # the store fused into the decode launch
    finally:
        db.close()


def _decode_steps_no_attention(db, b, steps, fused=False):
    rng = np.random.default_rng(8)
    for _ in range(steps):
        entry, ids = b.grow_one_token()
        assert np.array_equal(U.ukv_pages_alloc(db.pool, ids.size) if ids.size else ids, ids)
        _, nk, nv = b.draw_step_inputs(rng)
        db.set_new(nk, nv)
        oracle.append(b, b.pool, nk, nv)
        if fused:
            db.step(db.desc(entry, ids))
        else:
            db.append(db.desc(entry, ids))
    got = db.pool_host()
    assert np.array_equal(got, b.pool)
    untouched = got == 0xABCD
    expected_new = sum(2 * b.service_of(i).n_kv_heads * b.service_of(i).head_dim for i in range(b.n_requests)) * steps
    assert abs(int((~untouched).sum()) - expected_new) <= expected_new // 1000 + 4


def test_page_renaming_gives_bit_identical_output():
    say("page renaming")
    b = make_config(3, mini=True)
    db = DeviceBatch(b)
    db.decode()
    first = db.out_host().copy()
    db.close()
    perm = np.random.default_rng(4).permutation(b.n_pages)
    epp = b.page_bytes // 2
    pool2 = np.empty_like(b.pool)
    pool2.reshape(b.n_pages, epp)[perm] = b.pool.reshape(b.n_pages, epp)
    b.pool = pool2
    b.page_table = np.where(b.page_table >= 0, perm[np.maximum(b.page_table, 0)], -1).astype(np.int32)
    db2 = DeviceBatch(b)
    try:
        db2.decode()
        assert np.array_equal(db2.out_host(), first)
    finally:
        db2.close()


@pytest.mark.parametrize("page_bytes", [None, 1024])
def test_split_block_layout_matches_oracle_and_merged_layout(page_bytes):
    """The split-block alternative of section 4.4, run through the same entry points: one request
    per (request, kv head) of a one-kv-head service."""
    say(f"split layout, page_bytes {page_bytes}")
    b = make_config(5, mini=True)
    s = to_split_layout(b, page_bytes=page_bytes)
    copy_logical_kv_to_split(b, s, oracle.gather)
    merged_ref = oracle.attention(b, b.pool)
    db = DeviceBatch(s)
    try:
        _check_attention(db, s, "split layout")
        got = db.out_host().astype(np.float64)
        assert float(np.max(np.abs(got - merged_ref))) <= ATOL      # same logical K/V, other layout
        _check_gather(db, s)
        _decode_steps(db, s, 3, seed=17)
    finally:
        db.close()


def test_migration_gather_then_scatter_into_another_pool():
    """Request migration (section 5): gather every request out of one pool and scatter it into a
    differently fragmented pool; the new pool image is bit-exact and attention is unchanged."""
    say("migration: gather -> scatter")
    src = make_config(5, mini=True)
    dst = make_config(5, mini=True, seed=991)            # same recipe, other draw: other lengths and pages
    # the destination takes over the source's requests (service, length, q) but keeps its own placement
    rng = np.random.default_rng(5)
    dst = make_batch(src.services, src.service_id, src.ctx_len, src.n_pages, "permutation", rng, reserve_tokens=4,
                     pool_seed=3)
    dst.q = src.q.copy()
    dst.pool[:] = 0xABCD
    a, bdev = DeviceBatch(src), DeviceBatch(dst)
    try:
        k, v, kv_off, sizes = a.gather_device()
        bdev.scatter(k, v, kv_off)
        expect = dst.pool.copy()
        for i in range(src.n_requests):
            sv = src.service_of(i)
            n = int(src.ctx_len[i])
            gk, gv = oracle.gather(src.pool, src.page_bytes, src.table_of(i), sv.n_kv_heads, sv.head_dim, n)
            oracle.scatter(expect, dst.page_bytes, dst.table_of(i), gk, gv)
        assert np.array_equal(bdev.pool_host(), expect), "scattered pool image differs"
        dst.pool = expect
        bdev.decode()
        ref = oracle.attention(src, src.pool)
        assert float(np.max(np.abs(bdev.out_host().astype(np.float64) - ref))) <= ATOL
    finally:
        a.close()
        bdev.close()


def test_swap_out_to_pinned_host_memory_and_back():
    """Swapping a batch's cache out and in again (a preempted or migrating request, sections 4.2 and 5):
    ukv_gather writes straight into pinned host memory, the pages are overwritten, ukv_scatter reads the
    host copy back.  The host copy and the restored pool image are bit-exact against the oracle."""
    import torch
    say("swap: gather -> pinned host -> scatter")
    b = make_config(5, mini=True)
    db = DeviceBatch(b)
    try:
        kv_off, sizes = db.kv_layout()
        total = int(sizes.sum())
        hk = torch.zeros(total, dtype=torch.int16).pin_memory()
        hv = torch.zeros(total, dtype=torch.int16).pin_memory()
        U.ukv_gather(db.pool, db.desc(), hk.data_ptr(), hv.data_ptr(), kv_off, db.stream())
        torch.cuda.synchronize()
        expect = np.full_like(b.pool, 0xDEAD)
        for i in range(b.n_requests):
            sv = b.service_of(i)
            n = int(b.ctx_len[i])
            gk, gv = oracle.gather(b.pool, b.page_bytes, b.table_of(i), sv.n_kv_heads, sv.head_dim, n)
            o, e = int(kv_off[i]), int(kv_off[i] + sizes[i])
            assert np.array_equal(hk.numpy().view(np.uint16)[o:e], gk.reshape(-1)), f"host K copy differs, request {i}"
            assert np.array_equal(hv.numpy().view(np.uint16)[o:e], gv.reshape(-1)), f"host V copy differs, request {i}"
            oracle.scatter(expect, b.page_bytes, b.table_of(i), gk, gv)
        db.pool_t.fill_(np.array(0xDEAD, np.uint16).view(np.int16).item())     # the pages now hold something else
        U.ukv_scatter(db.pool, db.desc(), hk.data_ptr(), hv.data_ptr(), kv_off, db.stream())
        assert np.array_equal(db.pool_host(), expect), "restored pool image differs"
        db.decode()
        ref = oracle.attention(b, b.pool)
        assert float(np.max(np.abs(db.out_host().astype(np.float64) - ref))) <= ATOL
    finally:
        db.close()


@pytest.mark.parametrize("shape", ["70b", "13b", "h12"])
def test_one_long_request_cut_into_very_many_parts(shape):
    """A request alone on the device is cut into hundreds of parts per sequence: the merge of that many partials
    (spread over query heads and parts by the second launch, also when merging inside the decode launch is on)
    against the oracle; then a few parts more than, and exactly, what the in-launch merge still takes."""
    say(f"one long request, {shape}")
    sv = SHAPES[shape]
    rng = np.random.default_rng(41)
    b = make_batch([sv], np.array([0]), np.array([6000]), 6000 * sv.token_bytes // 16384 + 64, "permutation", rng,
                   reserve_tokens=4, pool_seed=9)
    db = DeviceBatch(b)
    try:
        for fused in (1, 0):
            U.ukv_set_param(db.pool, U.UKV_PARAM_FUSED_MERGE, fused)
            for span in (16 * 1024, 256 * 1024, 4 * 1024 * 1024):
                U.ukv_set_param(db.pool, U.UKV_PARAM_MIN_SPAN_BYTES, span)
                info, _ = U.ukv_plan_decode(db.pool, db.desc(), want_items=False)
                db.resize_workspace()
                db.out_t.fill_(float("nan"))
                _check_attention(db, b, f"fused {fused}, spans of {span} B: {info.n_items} items, "
                                        f"{info.n_reduce} sequences for the second launch")
    finally:
        db.close()


def test_one_sequence_of_more_than_a_thousand_parts():
    """One kv head, 40 000 tokens, spans of 16 KiB: a single sequence of about 1250 parts, more than the merge
    launch stages at a time (it goes through its parts in chunks of 1024)."""
    say("one sequence, > 1024 parts")
    sv = Service(4, 1, 128)
    rng = np.random.default_rng(43)
    b = make_batch([sv], np.array([0]), np.array([40000]), 40000 * sv.token_bytes // 16384 + 64, "permutation", rng,
                   reserve_tokens=4, pool_seed=10)
    db = DeviceBatch(b)
    try:
        U.ukv_set_param(db.pool, U.UKV_PARAM_MAX_SPANS, 4096)
        U.ukv_set_param(db.pool, U.UKV_PARAM_MIN_SPAN_BYTES, 16 * 1024)
        db.resize_workspace()
        info, _ = U.ukv_plan_decode(db.pool, db.desc(), want_items=False)
        assert info.n_seqs == 1 and info.n_items > 1024 and info.n_reduce == 1
        for fused in (1, 0):
            U.ukv_set_param(db.pool, U.UKV_PARAM_FUSED_MERGE, fused)
            db.out_t.fill_(float("nan"))
            _check_attention(db, b, f"fused {fused}: {info.n_items} parts")
    finally:
        db.close()


def test_many_calls_in_flight_on_a_side_stream():
    """More calls than staging slots are enqueued without synchronising, on a non-default stream;
    every call's output must still be that call's (plans and records are not overwritten early)."""
    import torch
    say("24 calls in flight on a side stream")
    b = make_config(5, mini=True)
    db = DeviceBatch(b, profile=True)
    try:
        rng = np.random.default_rng(31)
        qs = [b.draw_step_inputs(rng)[0] for _ in range(24)]
        q_dev = [torch.from_numpy(q.view(np.int16)).to(db.dev) for q in qs]
        outs = []
        side = torch.cuda.Stream()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            for k in range(24):
                db.q_t.copy_(q_dev[k], non_blocking=True)
                db.decode()
                outs.append(db.out_t.clone())
        torch.cuda.synchronize()
        prof = U.ukv_profile_read(db.pool)
        assert prof.n_decode == 24 and prof.decode_ms > 0.0
        for k in (0, 7, 8, 9, 23):
            ref = oracle.attention(b, b.pool, q=qs[k])
            err = float(np.max(np.abs(outs[k].cpu().numpy().astype(np.float64) - ref)))
            assert err <= ATOL, f"call {k}: max |err| {err}"
    finally:
        db.close()


def test_errors_from_the_compute_calls():
    b = make_config(1, mini=True)
    db = DeviceBatch(b)
    try:
        with pytest.raises(U.UkvError) as e:
            U.ukv_decode_attention(db.pool, db.desc(), db.ws_t.data_ptr(), 1024, db.stream())
        assert e.value.code == U.UKV_ENOSPC
        with pytest.raises(U.UkvError) as e:
            U.ukv_decode_attention(db.pool, db.desc(), db.ws_t.data_ptr() + 8, db.ws_bytes - 8, db.stream())
        assert e.value.code == U.UKV_EINVAL
        with pytest.raises(U.UkvError) as e:
            db.append(db.desc([0], [b.n_pages + 5]))
        assert e.value.code == U.UKV_EINVAL
        with pytest.raises(U.UkvError) as e:
            db.step(db.desc([0], [b.n_pages + 5]))
        assert e.value.code == U.UKV_EINVAL
        with pytest.raises(U.UkvError) as e:
            U.ukv_decode_step(db.pool, db.desc(), db.ws_t.data_ptr(), 1024, db.stream())
        assert e.value.code == U.UKV_ENOSPC
    finally:
        db.close()


@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
def test_full_size_configs_match_oracle(cfg):
    say(f"full cfg {cfg}")
    b = make_config(cfg)
    say(f"  generated: {b.n_requests} requests, {b.kv_bytes() / 1e9:.2f} GB of KV, pool {b.n_pages} pages")
    db = DeviceBatch(b)
    try:
        steps = int(b.notes["steps"])
        if steps:
            _decode_steps(db, b, steps, seed=100 + cfg, fused="alternate")
        else:
            _check_attention(db, b, "attention")
    finally:
        db.close()


def test_full_size_config5_sixteen_steps():
    say("full cfg 5, 16 x (append + attention)")
    b = make_config(5)
    say(f"  generated: {b.n_requests} requests, {b.kv_bytes() / 1e9:.2f} GB of KV, pool {b.n_pages} pages")
    db = DeviceBatch(b)
    try:
        _decode_steps(db, b, 16, seed=105, check_every=5, fused="alternate")
    finally:
        db.close()
