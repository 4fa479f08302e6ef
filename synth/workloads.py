"""Seeded synthetic workloads: service shapes, context lengths, page placement.

Everything here is input *structure*: which request belongs to which service,
how long its context is, which physical pages its table names, and random
bf16 payloads.  The layout facts it needs are the two the unified cache
fixes for its callers (unified KV cache, section 4.4): a token of a service
occupies ``n_kv_heads * head_dim * 2 * sizeof(bf16)`` bytes of the request's
byte stream, and a request of ``n`` tokens therefore owns
``ceil(n * token_bytes / page_bytes)`` pages.

The five workloads stand in for the paper's ShareGPT / LongBench request
lengths and Llama-2 / OPT models (evaluation set-up, section 6.1), which are
not available offline: only layer shapes and a long-tailed length law are
borrowed.
"""
from __future__ import annotations

import math
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

PAGE_BYTES = 16384
BASE_SEED = 20250415


# --------------------------------------------------------------------------
# bf16 helpers (bit-level; no arithmetic of the method)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(n: int, rng: np.random.Generator) -> np.ndarray:
    """n samples of N(0,1) drawn in fp32 and rounded to bf16 bit patterns."""
    return f32_to_bf16_bits(rng.standard_normal(n, dtype=np.float32))


def _fill_normal_bf16_parallel(out: np.ndarray, seed: int, threads: Optional[int] = None) -> None:
    """Fill a large uint16 array with N(0,1) bf16 bits using independent per-chunk streams."""
    chunk = 1 << 23
    n = out.size
    n_chunks = (n + chunk - 1) // chunk
    seqs = np.random.SeedSequence(seed).spawn(max(n_chunks, 1))
    if threads is None:
        threads = min(16, os.cpu_count() or 1)

    def work(c: int) -> None:
        lo = c * chunk
        hi = min(n, lo + chunk)
        out[lo:hi] = normal_bf16(hi - lo, np.random.default_rng(seqs[c]))

    if n_chunks <= 1 or threads <= 1:
        for c in range(n_chunks):
            work(c)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(work, range(n_chunks)))


# --------------------------------------------------------------------------
# services
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Service:
    """One co-located LLM service, reduced to the shape of one attention layer."""

    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    scale: float = 0.0  # 0 means 1/sqrt(head_dim)

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def head_row_bytes(self) -> int:
        return 4 * self.head_dim  # K[d] then V[d], bf16

    @property
    def token_bytes(self) -> int:
        return self.n_kv_heads * self.head_dim * 2 * 2

    @property
    def softmax_scale(self) -> float:
        return self.scale if self.scale != 0.0 else 1.0 / math.sqrt(self.head_dim)


SHAPES: Dict[str, Service] = {
    "tiny": Service(8, 8, 64),
    "h12": Service(12, 12, 64),
    "7b": Service(32, 32, 128),
    "13b": Service(40, 40, 128),
    "8b": Service(32, 8, 128),
    "70b": Service(64, 8, 128),
}


def pages_for_tokens(n_tokens, token_bytes, page_bytes=PAGE_BYTES):
    """Pages a request of n_tokens owns: ceil(n * token_bytes / page_bytes)."""
    n = np.asarray(n_tokens, dtype=np.int64) * np.asarray(token_bytes, dtype=np.int64)
    return (n + page_bytes - 1) // page_bytes


# --------------------------------------------------------------------------
# LIFO page stack with an operation log (so another allocator can replay it)
# --------------------------------------------------------------------------
class PageStack:
    """LIFO free list; a fresh stack hands out 0, 1, 2, ...  Every operation is logged."""

    def __init__(self, n_pages: int):
        self.n_pages = int(n_pages)
        self._s = np.arange(n_pages - 1, -1, -1, dtype=np.int32)
        self._top = self.n_pages
        self.log: List[Tuple[str, object]] = []

    @property
    def free_pages(self) -> int:
        return self._top

    @property
    def used_pages(self) -> int:
        return self.n_pages - self._top

    def alloc(self, n: int) -> np.ndarray:
        n = int(n)
        if n > self._top:
            raise MemoryError(f"page stack exhausted: want {n}, have {self._top}")
        ids = self._s[self._top - n:self._top][::-1].copy()
        self._top -= n
        self.log.append(("alloc", n))
        return ids

    def free(self, ids: np.ndarray) -> None:
        ids = np.asarray(ids, dtype=np.int32)
        n = ids.size
        assert self._top + n <= self.n_pages
        self._s[self._top:self._top + n] = ids
        self._top += n
        self.log.append(("free", ids.copy()))

    def peek_order(self) -> np.ndarray:
        """Ids in the order future allocations will return them."""
        return self._s[:self._top][::-1].copy()


def lockstep_order(n_pages_per_seq: np.ndarray, token_bytes_per_seq: np.ndarray,
                   page_bytes: int = PAGE_BYTES) -> np.ndarray:
    """Order in which sequences take pages when all grow one token per round.

    Sequence i asks for its k-th page in the round of the first token whose
    bytes reach past k pages, i.e. token floor(k*page_bytes/token_bytes); ties
    go to the lower sequence index.  Returns the sequence index of every
    allocation event, in order.
    """
    n_pages_per_seq = np.asarray(n_pages_per_seq, dtype=np.int64)
    tb = np.asarray(token_bytes_per_seq, dtype=np.int64)
    seq = np.repeat(np.arange(n_pages_per_seq.size, dtype=np.int64), n_pages_per_seq)
    starts = np.cumsum(n_pages_per_seq) - n_pages_per_seq
    k = np.arange(seq.size, dtype=np.int64) - np.repeat(starts, n_pages_per_seq)
    t = (k * page_bytes) // tb[seq]
    order = np.lexsort((k, seq, t))
    return seq[order]


def _alloc_lockstep(stack: PageStack, n_pages_per_seq: np.ndarray, token_bytes_per_seq: np.ndarray,
                    page_bytes: int, budget: Optional[int] = None) -> List[np.ndarray]:
    ev = lockstep_order(n_pages_per_seq, token_bytes_per_seq, page_bytes)
    if budget is not None and ev.size > budget:
        ev = ev[:budget]
    ids = stack.alloc(ev.size)
    by_seq = np.argsort(ev, kind="stable")
    counts = np.bincount(ev, minlength=len(n_pages_per_seq))
    sorted_ids = ids[by_seq]
    out, pos = [], 0
    for c in counts:
        out.append(sorted_ids[pos:pos + c])
        pos += c
    return out


# --------------------------------------------------------------------------
# batch container
# --------------------------------------------------------------------------
@dataclass
class Batch:
    """A mixed-service decode batch plus the pool it lives in (all host arrays)."""

    page_bytes: int
    n_pages: int
    services: List[Service]
    service_id: np.ndarray      # uint32 [n]
    ctx_len: np.ndarray         # uint32 [n]  tokens valid for attention
    table_off: np.ndarray       # uint64 [n]  entry offset of each request's table
    table_cap: np.ndarray       # int64  [n]  entries reserved per request
    page_table: np.ndarray      # int32  [sum(table_cap)]  (-1 = not yet allocated)
    q: np.ndarray               # uint16 bf16 bits, concatenated [Q_s, d_s] per request
    q_off: np.ndarray           # uint64 [n]  element offsets into q
    out_off: np.ndarray         # uint64 [n]  element offsets into the fp32 output
    out_elems: int
    new_off: np.ndarray         # uint64 [n]  element offsets into new_k / new_v
    new_elems: int
    stack: PageStack
    pool: Optional[np.ndarray] = None   # uint16 [n_pages * page_bytes / 2]
    name: str = ""
    notes: Dict[str, object] = field(default_factory=dict)

    @property
    def n_requests(self) -> int:
        return int(self.service_id.size)

    def service_of(self, i: int) -> Service:
        return self.services[int(self.service_id[i])]

    def table_of(self, i: int) -> np.ndarray:
        o = int(self.table_off[i])
        return self.page_table[o:o + int(self.table_cap[i])]

    def token_bytes(self) -> np.ndarray:
        tb = np.array([s.token_bytes for s in self.services], dtype=np.int64)
        return tb[self.service_id]

    def kv_bytes(self) -> int:
        return int((self.ctx_len.astype(np.int64) * self.token_bytes()).sum())

    def pages_owned(self) -> np.ndarray:
        return pages_for_tokens(self.ctx_len, self.token_bytes(), self.page_bytes)

    def draw_step_inputs(self, rng: np.random.Generator):
        """Fresh q, new_k, new_v (bf16 bits) for one decode step."""
        return (normal_bf16(self.q.size, rng), normal_bf16(self.new_elems, rng),
                normal_bf16(self.new_elems, rng))

    def grow_one_token(self) -> Tuple[np.ndarray, np.ndarray]:
        """Bump every ctx_len by one, taking pages off the stack where the new token needs them.

        Returns (entry_index, page_id) of the table entries written, in request order.
        """
        tb = self.token_bytes()
        have = pages_for_tokens(self.ctx_len, tb, self.page_bytes)
        self.ctx_len = (self.ctx_len + 1).astype(np.uint32)
        need = pages_for_tokens(self.ctx_len, tb, self.page_bytes)
        extra = need - have
        assert np.all(need <= self.table_cap), "table capacity exceeded; raise reserve_tokens"
        total = int(extra.sum())
        if total == 0:
            return np.zeros(0, np.uint64), np.zeros(0, np.int32)
        ids = self.stack.alloc(total)
        req = np.repeat(np.arange(self.n_requests), extra)
        first = np.cumsum(extra) - extra
        k = np.arange(total) - np.repeat(first, extra)
        entry = (self.table_off[req].astype(np.int64) + have[req] + k).astype(np.uint64)
        self.page_table[entry.astype(np.int64)] = ids
        return entry, ids


def draw_prefill_inputs(b: "Batch", q_len: np.ndarray, rng: np.random.Generator):
    """Query rows for the prefill phase: request i gets q_len[i] rows of [n_q_heads, head_dim] bf16 bits.

    Returns (q_bits flat, q_off, out_off, n_elems): element offsets of each request's first row in the flat
    q array and in the (same-shaped) output array.  The requests' K/V are whatever the pool image holds."""
    q_len = np.asarray(q_len, np.int64)
    row = np.array([b.services[s].n_q_heads * b.services[s].head_dim for s in b.service_id], np.int64)
    sizes = q_len * row
    off = (np.cumsum(sizes) - sizes).astype(np.uint64)
    n_elems = int(sizes.sum())
    return normal_bf16(max(n_elems, 8), rng), off, off.copy(), max(n_elems, 8)


def draw_lengths(law: dict, n: int, rng: np.random.Generator) -> np.ndarray:
    if law["kind"] == "uniform":
        return rng.integers(law["lo"], law["hi"] + 1, size=n).astype(np.int64)
    if law["kind"] == "lognormal":
        x = np.exp(rng.normal(math.log(law["median"]), law["sigma"], size=n))
        return np.clip(np.rint(x), 1, law["max"]).astype(np.int64)
    raise ValueError(law["kind"])


def _churn(stack: PageStack, services: Sequence[Service], mix: Optional[Sequence[float]], law: dict,
           rng: np.random.Generator, page_bytes: int, rounds: int = 8, fill: float = 0.9,
           group: int = 64) -> None:
    """Fragment the free list: rounds of fill-to-90% with dummy sequences, then free a random half."""
    live: List[np.ndarray] = []
    limit = int(fill * stack.n_pages)
    tb_all = np.array([s.token_bytes for s in services], dtype=np.int64)
    for _ in range(rounds):
        while stack.used_pages < limit:
            sid = rng.choice(len(services), size=group, p=mix)
            lens = draw_lengths(law, group, rng)
            npg = pages_for_tokens(lens, tb_all[sid], page_bytes)
            got = _alloc_lockstep(stack, npg, tb_all[sid], page_bytes, budget=limit - stack.used_pages)
            live.extend(g for g in got if g.size)
        perm = rng.permutation(len(live))
        half = len(live) // 2
        if half:
            stack.free(np.concatenate([live[j] for j in perm[:half]]))
        live = [live[j] for j in perm[half:]]
    if live:
        perm = rng.permutation(len(live))
        stack.free(np.concatenate([live[j] for j in perm]))
    assert stack.used_pages == 0


def make_batch(services: Sequence[Service], service_id: np.ndarray, ctx_len: np.ndarray, n_pages: int,
               placement: str, rng: np.random.Generator, *, page_bytes: int = PAGE_BYTES,
               reserve_tokens: int = 0, churn: Optional[dict] = None, fill_pool: bool = True,
               pool_seed: int = 0, name: str = "") -> Batch:
    """Build a batch: allocate pages per the placement rule and draw payloads.

    placement: "permutation" (free pages handed out in a seeded random order, request after
    request) or "lockstep" (all requests grow one token per round from the LIFO stack).
    churn: if given, dict(mix=..., law=...) used to scramble the free list first.
    """
    services = list(services)
    service_id = np.asarray(service_id, dtype=np.uint32)
    ctx_len = np.asarray(ctx_len, dtype=np.uint32)
    n = service_id.size
    tb = np.array([s.token_bytes for s in services], dtype=np.int64)[service_id]
    stack = PageStack(n_pages)
    if churn is not None:
        _churn(stack, services, churn.get("mix"), churn["law"], rng, page_bytes)
    npg = pages_for_tokens(ctx_len, tb, page_bytes)
    cap = pages_for_tokens(ctx_len.astype(np.int64) + reserve_tokens, tb, page_bytes)
    cap = np.maximum(cap, 1)
    table_off = (np.cumsum(cap) - cap).astype(np.uint64)
    page_table = np.full(int(cap.sum()), -1, dtype=np.int32)
    if int(npg.sum()) > stack.free_pages:
        raise MemoryError(f"batch needs {int(npg.sum())} pages, pool has {stack.free_pages}")
    if placement == "permutation":
        perm = rng.permutation(n_pages).astype(np.int32)
        all_ids = stack.alloc(n_pages)
        del all_ids
        stack.free(perm[::-1])          # next allocations now come out in perm order
        for i in range(n):
            ids = stack.alloc(int(npg[i]))
            page_table[int(table_off[i]):int(table_off[i]) + ids.size] = ids
    elif placement == "lockstep":
        got = _alloc_lockstep(stack, npg, tb, page_bytes)
        for i in range(n):
            page_table[int(table_off[i]):int(table_off[i]) + got[i].size] = got[i]
    else:
        raise ValueError(placement)

    q_elems = np.array([services[s].n_q_heads * services[s].head_dim for s in service_id], dtype=np.int64)
    kv_elems = np.array([services[s].n_kv_heads * services[s].head_dim for s in service_id], dtype=np.int64)
    q_off = (np.cumsum(q_elems) - q_elems).astype(np.uint64)
    new_off = (np.cumsum(kv_elems) - kv_elems).astype(np.uint64)
    q = normal_bf16(int(q_elems.sum()), rng)
    pool = None
    if fill_pool:
        pool = np.empty(n_pages * page_bytes // 2, dtype=np.uint16)
        _fill_normal_bf16_parallel(pool, pool_seed)
    return Batch(page_bytes=page_bytes, n_pages=n_pages, services=services, service_id=service_id,
                 ctx_len=ctx_len, table_off=table_off, table_cap=cap, page_table=page_table, q=q,
                 q_off=q_off, out_off=q_off.copy(), out_elems=int(q_elems.sum()), new_off=new_off,
                 new_elems=int(kv_elems.sum()), stack=stack, pool=pool, name=name)


# --------------------------------------------------------------------------
# the five workloads (and scaled-down "mini" versions of the same recipes)
# --------------------------------------------------------------------------
GIB_PAGES = (1 << 30) // PAGE_BYTES

CONFIGS: Dict[int, dict] = {
    1: dict(name="cfg1-single-service", services=["tiny"], n=8, mix="alternate",
            law=dict(kind="uniform", lo=64, hi=512), n_pages=256, grow_pool_if_needed=512,
            placement="permutation", churn=False, steps=0,
            mini=dict(n=4, law=dict(kind="uniform", lo=5, hi=70), n_pages=64)),
    2: dict(name="cfg2-llama7b-layer", services=["7b"], n=64, mix="alternate",
            law=dict(kind="uniform", lo=128, hi=4096), n_pages=4 * GIB_PAGES, stated_pages=1 * GIB_PAGES,
            placement="permutation", churn=False, steps=1,
            mini=dict(n=6, law=dict(kind="uniform", lo=16, hi=300), n_pages=2048)),
    3: dict(name="cfg3-two-services", services=["7b", "13b"], n=128, mix="alternate",
            law=dict(kind="lognormal", median=1024, sigma=0.75, max=8192), n_pages=4 * GIB_PAGES,
            stated_pages=2 * GIB_PAGES, placement="lockstep", churn=False, steps=0,
            mini=dict(n=10, law=dict(kind="lognormal", median=96, sigma=0.75, max=700), n_pages=4096)),
    4: dict(name="cfg4-gqa-mix", services=["8b", "70b"], n=256, mix="alternate",
            law=dict(kind="lognormal", median=2048, sigma=1.0, max=32768), n_pages=4 * GIB_PAGES,
            placement="lockstep", churn=True, steps=0,
            mini=dict(n=12, law=dict(kind="lognormal", median=160, sigma=1.0, max=2500), n_pages=2048)),
    5: dict(name="cfg5-four-services", services=["h12", "7b", "13b", "8b"], n=512, mix=[0.4, 0.3, 0.2, 0.1],
            law=dict(kind="lognormal", median=1024, sigma=0.75, max=16384), n_pages=8 * GIB_PAGES,
            placement="lockstep", churn=True, steps=16,
            mini=dict(n=24, law=dict(kind="lognormal", median=80, sigma=0.75, max=1200), n_pages=4096)),
}


def make_config(index: int, *, mini: bool = False, fill_pool: bool = True, seed: Optional[int] = None,
                reserve_tokens: Optional[int] = None, as_stated: bool = False) -> Batch:
    """Draw workload `index` (1..5).  mini=True shrinks counts and lengths, same recipe.

    reserve_tokens: table entries are reserved for this many future tokens per request
    (default: the workload's own decode steps, at least 4).
    as_stated: keep the pool at the size the workload states even where the drawn batch does not fit, and
    admit the requests in draw order while pages remain (the admission gate of the paper's scheduler,
    appendix algorithm: a request only joins the batch if the block manager has room for it)."""
    c = dict(CONFIGS[index])
    if mini:
        c.update(c["mini"])
    seed = BASE_SEED + index if seed is None else seed
    rng = np.random.default_rng(seed)
    services = [SHAPES[s] for s in c["services"]]
    n = c["n"]
    if c["mix"] == "alternate":
        sid = np.arange(n) % len(services)
        mix = None
    else:
        mix = c["mix"]
        sid = rng.choice(len(services), size=n, p=mix)
    lens = draw_lengths(c["law"], n, rng)
    n_pages = c["n_pages"]
    tb = np.array([s.token_bytes for s in services], dtype=np.int64)[sid]
    need = int(pages_for_tokens(lens + c["steps"], tb).sum())
    notes = {"stated_pages": c.get("stated_pages", c["n_pages"])}
    notes["drawn_requests"] = n
    if as_stated and not mini:
        n_pages = notes["stated_pages"]
        keep_tokens = max(c["steps"], 4) if reserve_tokens is None else reserve_tokens
        per_req = pages_for_tokens(lens + keep_tokens, tb)  # what a request may hold by the end of the run
        admitted = int(np.searchsorted(np.cumsum(per_req), n_pages, side="right"))
        sid, lens, tb = sid[:admitted], lens[:admitted], tb[:admitted]
        need = int(pages_for_tokens(lens + c["steps"], tb).sum())
    elif need > n_pages and "grow_pool_if_needed" in c and not mini:
        n_pages = c["grow_pool_if_needed"]
    notes["pages_needed"] = need
    churn = dict(mix=mix, law=c["law"]) if c["churn"] else None
    b = make_batch(services, sid, lens, n_pages, c["placement"], rng,
                   reserve_tokens=max(c["steps"], 4) if reserve_tokens is None else reserve_tokens, churn=churn,
                   fill_pool=fill_pool, pool_seed=seed + 1000, name=c["name"] + ("-mini" if mini else ""))
    b.notes.update(notes)
    b.notes["steps"] = c["steps"]
    b.notes["seed"] = seed
    b.notes["reserve_tokens"] = max(c["steps"], 4) if reserve_tokens is None else reserve_tokens
    return b


# --------------------------------------------------------------------------
# the split-block alternative (section 4.4): one block stream per (request, kv head)
# --------------------------------------------------------------------------
def to_split_layout(b: Batch, *, fill_pool: bool = True, pool_seed: int = 0,
                    page_bytes: Optional[int] = None) -> Batch:
    """The same requests laid out with split cache blocks: every kv head of every request owns
    its own blocks and its own block table (what section 4.4 calls the split method).

    Expressed with the same descriptor: request i of a service (Q, H, d) becomes H requests of a
    one-kv-head service (Q/H, 1, d); q, out and new-token offsets point into the same arrays as
    before, so results are comparable element by element.  Pages are handed out from a fresh LIFO
    stack over a pool of the same byte size with all (request, head) streams growing in lock-step.
    page_bytes: block size of the split layout (default: the merged layout's page size).
    """
    page_bytes = b.page_bytes if page_bytes is None else page_bytes
    n_pages = b.n_pages * b.page_bytes // page_bytes
    services = [Service(s.group, 1, s.head_dim, s.scale) for s in b.services]
    H = np.array([s.n_kv_heads for s in b.services], dtype=np.int64)[b.service_id]
    G = np.array([s.group for s in b.services], dtype=np.int64)[b.service_id]
    d = np.array([s.head_dim for s in b.services], dtype=np.int64)[b.service_id]
    req = np.repeat(np.arange(b.n_requests), H)
    first = np.cumsum(H) - H
    head = np.arange(req.size) - np.repeat(first, H)
    sid = b.service_id[req]
    ctx = b.ctx_len[req]
    tb = (4 * d)[req]
    reserve = int(b.notes.get("reserve_tokens", 4))
    npg = pages_for_tokens(ctx, tb, page_bytes)
    cap = np.maximum(pages_for_tokens(ctx.astype(np.int64) + reserve, tb, page_bytes), 1)
    table_off = (np.cumsum(cap) - cap).astype(np.uint64)
    page_table = np.full(int(cap.sum()), -1, dtype=np.int32)
    stack = PageStack(n_pages)
    if int(npg.sum()) > stack.free_pages:
        raise MemoryError(f"split layout needs {int(npg.sum())} pages, pool has {stack.free_pages}")
    got = _alloc_lockstep(stack, npg, tb, page_bytes)
    for k in range(req.size):
        page_table[int(table_off[k]):int(table_off[k]) + got[k].size] = got[k]
    q_off = (b.q_off[req].astype(np.int64) + head * (G * d)[req]).astype(np.uint64)
    new_off = (b.new_off[req].astype(np.int64) + head * d[req]).astype(np.uint64)
    pool = None
    if fill_pool:
        pool = np.empty(n_pages * page_bytes // 2, dtype=np.uint16)
        _fill_normal_bf16_parallel(pool, pool_seed)
    out = Batch(page_bytes=page_bytes, n_pages=n_pages, services=services, service_id=sid.astype(np.uint32),
                ctx_len=ctx.astype(np.uint32), table_off=table_off, table_cap=cap, page_table=page_table,
                q=b.q, q_off=q_off, out_off=q_off.copy(), out_elems=b.out_elems, new_off=new_off,
                new_elems=b.new_elems, stack=stack, pool=pool, name=b.name + "-split")
    out.notes.update(b.notes)
    out.notes["split_of"] = (req, head)
    return out
