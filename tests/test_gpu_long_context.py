"""Decode and prefill attention at the largest page size over very long contexts, checked by a closed form.

The oracle cannot follow at this size (gigabytes of K/V per request), so the inputs are chosen to make the
answer known: every K is zero, so all scores are equal and the output is the plain mean of V over the tokens a
query may see; V[t][h][e] = (37 (t div 64) + h + e) mod 128 (small integers, exact in bf16), whose running mean
is summed exactly on the host: reading a page twice, or one that is not the request's, moves it far beyond the bar.  1 MiB pages
put a 2048-entry page-table window at 2 GiB, the largest byte offset the kernels' 32-bit window-relative
arithmetic has to hold; pages are placed by a seeded permutation and everything outside the requests' tokens
(the tail of each last page included) is NaN.
"""
import numpy as np
import pytest

import paper_2504_15720_amd as U
from synth import SHAPES
from synth.workloads import normal_bf16

ATOL = 2e-3
PAGE = 1 << 20


def _pattern(t, c):
    """V of token t at head + element index c: changes every 64 tokens, values 0..127 (exact in bf16)."""
    return ((t // 64) * 37 + c) % 128


def _mean_of_pattern(n_tokens: int, c: np.ndarray) -> np.ndarray:
    """mean over t in [0, n_tokens) of _pattern(t, c), exactly (float64 sums of small integers)."""
    blocks = np.arange(-(-n_tokens // 64), dtype=np.int64)
    count = np.minimum(64, n_tokens - 64 * blocks).astype(np.float64)
    flat = c.reshape(-1)
    total = (count[:, None] * ((blocks[:, None] * 37 + flat[None, :]) % 128)).sum(axis=0)
    return (total / n_tokens).reshape(c.shape)


def test_closed_form_mean_matches_brute_force():
    """The host-side expectation of the GPU test below, against the sum written out (CPU)."""
    c = np.arange(40).reshape(5, 8)
    for n in (1, 63, 64, 65, 1003, 12345):
        t = np.arange(n)
        brute = np.array([[_pattern(t, int(x)).mean() for x in row] for row in c])
        assert np.max(np.abs(brute - _mean_of_pattern(n, c))) < 1e-12


@pytest.mark.gpu
def test_million_token_context_in_one_mebibyte_pages():
    import torch
    dev = torch.device("cuda:0")
    services = [SHAPES["70b"], SHAPES["7b"]]
    ctx = np.array([1_000_003, 200_005], np.int64)
    sid = np.array([0, 1])
    tok_b = np.array([services[s].token_bytes for s in sid], np.int64)
    n_pg = -(-ctx * tok_b // PAGE)
    n_pages = int(n_pg.sum()) + 37
    print(f"long context: {ctx.tolist()} tokens, {n_pg.tolist()} pages of 1 MiB", flush=True)
    rng = np.random.default_rng(123)
    perm = rng.permutation(n_pages)[:int(n_pg.sum())].astype(np.int64)
    table_off = (np.cumsum(n_pg) - n_pg).astype(np.uint64)

    raw = torch.full((n_pages * PAGE // 2 + PAGE // 2,), 0x7FC0, dtype=torch.int16, device=dev)   # NaN everywhere
    skip = (-raw.data_ptr() % PAGE) // 2
    pool_t = raw[skip:skip + n_pages * PAGE // 2]
    pool_pages = pool_t.view(n_pages, PAGE // 2)
    for i in range(2):
        sv = services[sid[i]]
        H, d, n = sv.n_kv_heads, sv.head_dim, int(ctx[i])
        stream = torch.full((int(n_pg[i]) * PAGE // 2,), 0x7FC0, dtype=torch.int16, device=dev)
        rows = stream[:n * H * 2 * d].view(n, H, 2, d)
        rows[:, :, 0, :] = 0                                                                  # K = 0
        he = (torch.arange(H, device=dev)[:, None] + torch.arange(d, device=dev)[None, :])   # h + e
        for t0 in range(0, n, 1 << 16):
            t = torch.arange(t0, min(n, t0 + (1 << 16)), device=dev)
            v = _pattern(t[:, None, None], he[None]).to(torch.bfloat16)
            rows[t0:t0 + t.numel(), :, 1, :] = v.view(torch.int16)
        ids = torch.from_numpy(perm[int(table_off[i]):int(table_off[i]) + int(n_pg[i])]).to(dev)
        pool_pages[ids] = stream.view(int(n_pg[i]), PAGE // 2)
        del stream, rows
    table_t = torch.from_numpy(perm.astype(np.int32)).to(dev)

    pool = U.ukv_pool_create(pool_t.data_ptr(), n_pages * PAGE, PAGE, services)
    try:
        row_el = np.array([services[s].n_q_heads * services[s].head_dim for s in sid], np.int64)
        stream_h = torch.cuda.current_stream().cuda_stream

        def expected(i, n_seen):
            sv = services[sid[i]]
            a = np.arange(sv.n_q_heads) // sv.group                                   # kv head of every query head
            c = a[:, None] + np.arange(sv.head_dim)[None, :]
            return _mean_of_pattern(n_seen, c)

        # decode: one query token per request sees every token
        q_off = (np.cumsum(row_el) - row_el).astype(np.uint64)
        q_t = torch.from_numpy(normal_bf16(int(row_el.sum()), rng).view(np.int16)).to(dev)
        out_t = torch.full((int(row_el.sum()),), float("nan"), dtype=torch.float32, device=dev)
        ws = U.ukv_decode_workspace_bytes(pool, 2)
        ws_t = torch.empty(ws, dtype=torch.uint8, device=dev)
        desc = U.BatchDesc(sid, ctx, table_off, table_t.data_ptr(), q_t.data_ptr(), q_off, out_t.data_ptr(), q_off)
        for block in (512, 256):
            U.ukv_set_param(pool, U.UKV_PARAM_BLOCK_THREADS, block)
            out_t.fill_(float("nan"))
            U.ukv_decode_attention(pool, desc, ws_t.data_ptr(), ws, stream_h)
            got = out_t.cpu().numpy().astype(np.float64)
            for i in range(2):
                sv = services[sid[i]]
                g = got[int(q_off[i]):int(q_off[i]) + int(row_el[i])].reshape(sv.n_q_heads, sv.head_dim)
                err = float(np.max(np.abs(g - expected(i, int(ctx[i])))))
                print(f"  decode, block {block}, request {i}: max|err| = {err:.3e}", flush=True)
                assert np.all(np.isfinite(g)) and err <= ATOL

        # prefill: the last 64 tokens of each request, causal
        q_len = np.array([64, 64], np.uint32)
        pq_off = (np.cumsum(q_len * row_el) - q_len * row_el).astype(np.uint64)
        n_el = int((q_len * row_el).sum())
        pq_t = torch.from_numpy(normal_bf16(n_el, rng).view(np.int16)).to(dev)
        pout_t = torch.full((n_el,), float("nan"), dtype=torch.float32, device=dev)
        # both forms of the softmax weights; the one-part form keeps an fp16 copy of every V row in the workspace
        pws = U.ukv_prefill_workspace_bytes_one_part(pool, 2, int(q_len.sum()), int(ctx.sum()))
        pws_t = torch.empty(pws, dtype=torch.uint8, device=dev)
        pdesc = U.BatchDesc(sid, ctx, table_off, table_t.data_ptr(), pq_t.data_ptr(), pq_off, pout_t.data_ptr(), pq_off)
        for form in (2, 1):
            U.ukv_set_param(pool, U.UKV_PARAM_PREFILL_WEIGHTS, form)
            pout_t.fill_(float("nan"))
            U.ukv_prefill_attention(pool, pdesc, q_len, pws_t.data_ptr(), pws, stream_h)
            assert U.ukv_get_param(pool, U.UKV_PARAM_PREFILL_FORM_USED) == form
            got = pout_t.cpu().numpy().astype(np.float64)
            for i in range(2):
                sv = services[sid[i]]
                g = got[int(pq_off[i]):int(pq_off[i]) + 64 * int(row_el[i])].reshape(64, sv.n_q_heads, sv.head_dim)
                worst = 0.0
                for r in (0, 1, 31, 62, 63):
                    worst = max(worst, float(np.max(np.abs(g[r] - expected(i, int(ctx[i]) - 64 + r + 1)))))
                print(f"  prefill, weights in {form} part(s), request {i}: max|err| = {worst:.3e}", flush=True)
                assert np.all(np.isfinite(g)) and worst <= ATOL
        torch.cuda.synchronize()
    finally:
        torch.cuda.synchronize()
        U.ukv_pool_destroy(pool)
