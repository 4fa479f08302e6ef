"""Seeded synthetic input of the scheduler-driven serving loop: requests of three co-located services with prompt
and output lengths from long-tailed laws, the execution-time profiles the scheduler is given, the bf16 payloads,
and the clock model that stands in for measured execution times.

Like the rest of this package it only draws inputs and holds none of the method's arithmetic (no scheduling rule,
no attention); the GPU loop and the oracle-side replay of a test are both fed from it.  The lengths stand in for
the chat / summarization / code mixes of the paper's evaluation (section 6.1), which are not available here.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence, Tuple

import numpy as np

from .workloads import PAGE_BYTES, SHAPES, Service, draw_lengths, normal_bf16

# (prompt law, output law) per service: short chat-like, long-prompt, medium
SERVE_LAWS = [
    (dict(kind="lognormal", median=256, sigma=0.6, max=2048), dict(kind="lognormal", median=32, sigma=0.5, max=128)),
    (dict(kind="lognormal", median=1024, sigma=0.5, max=2048), dict(kind="lognormal", median=96, sigma=0.5, max=256)),
    (dict(kind="lognormal", median=512, sigma=0.6, max=2048), dict(kind="lognormal", median=64, sigma=0.5, max=192)),
]
NOISE_BLOCK = 1 << 24   # elements of the random block that the large buffers repeat


@dataclass
class ServeWorkload:
    services: List[Service]
    svc: np.ndarray          # int64 [n] service of each request
    prompt: np.ndarray       # int64 [n] prompt tokens
    out_len: np.ndarray      # int64 [n] tokens to generate
    page_bytes: int
    max_batch: int
    tok_b: np.ndarray        # int64 [n] token bytes
    tok_el: np.ndarray       # int64 [n] K (or V) elements per token
    row_el: np.ndarray       # int64 [n] q / out elements per token
    row_max: int             # widest q row over the services (slot size of the per-request decode inputs)
    cap: np.ndarray          # int64 [n] page-table entries reserved per request
    table_off: np.ndarray    # uint64 [n]
    n_pages: int
    profiles: List[Tuple[float, float, float]]   # (mean_time, std_time, starvation_threshold) per service
    seed: int

    @property
    def n(self) -> int:
        return int(self.svc.size)

    def noise_block(self, which: int) -> np.ndarray:
        """Random bf16 block number `which` (0: prefill K source, 1: prefill V source, 2: prefill q, 3: pool fill)."""
        return normal_bf16(NOISE_BLOCK, np.random.default_rng([self.seed, 100 + which]))

    def decode_inputs(self):
        """Per-request decode inputs, [n * row_max] bf16 bits each: q, new K token, new V token (request r uses the
        slot starting at r * row_max; the same rows every step)."""
        rng = np.random.default_rng([self.seed, 200])
        n_el = self.n * self.row_max
        return normal_bf16(n_el, rng), normal_bf16(n_el, rng), normal_bf16(n_el, rng)


def tiled(block: np.ndarray, start: int, n: int) -> np.ndarray:
    """Elements [start, start + n) of the buffer that repeats `block` end to end."""
    return block[(start + np.arange(n, dtype=np.int64)) % block.size]


def modelled_time(queue_is_prefill: bool, lens: Sequence[int], token_bytes: Sequence[int]) -> float:
    """Execution time charged for one iteration when the loop runs on the model clock instead of the wall clock
    (reproducible decisions): a fixed launch cost plus the iteration's KV traffic at a nominal rate; a prefill
    batch is charged its causal KV reads, sum of p (p + 1) / 2 token rows, at a rate 64 times higher (cache reuse)."""
    lens = np.asarray(lens, dtype=np.int64)
    tb = np.asarray(token_bytes, dtype=np.int64)
    if queue_is_prefill:
        return 30e-6 + float((lens * (lens + 1) // 2 * tb).sum()) / (64 * 5e12)
    return 20e-6 + float((lens * tb).sum()) / 5e12


def draw_serve_workload(per_service: int, seed: int = 20250415 + 99, max_batch: int = 32,
                        starvation_threshold: float = 0.05, headroom: float = 1.05,
                        names: Sequence[str] = ("7b", "13b", "8b"), time_unit: float = 1e-3) -> ServeWorkload:
    """per_service requests of each of three services, all queued at time 0.  The pool is sized for every request
    at its final length plus `headroom`; a smaller headroom (< 1) makes page-counted admission bite.  time_unit: the
    profiled execution time given for the shortest service (the others in proportion to their KV traffic)."""
    services = [SHAPES[x] for x in names]
    rng = np.random.default_rng(seed)
    ns = len(services)
    svc = np.repeat(np.arange(ns), per_service)
    prompt = np.concatenate([np.maximum(draw_lengths(SERVE_LAWS[s][0], per_service, rng), 16) for s in range(ns)])
    out_len = np.concatenate([np.maximum(draw_lengths(SERVE_LAWS[s][1], per_service, rng), 4) for s in range(ns)])
    tok_b = np.array([services[s].token_bytes for s in svc], np.int64)
    row_el = np.array([services[s].n_q_heads * services[s].head_dim for s in svc], np.int64)
    cap = -(-(prompt + out_len + 1) * tok_b // PAGE_BYTES)
    table_off = (np.cumsum(cap) - cap).astype(np.uint64)
    n_pages = int(cap.sum() * headroom) + 64
    # profiled execution times: proportional to the KV bytes a request of the service streams over its life
    life = np.array([np.mean((prompt[svc == s] + out_len[svc == s] / 2) * out_len[svc == s] * services[s].token_bytes)
                     for s in range(ns)])
    std = np.array([np.std((prompt[svc == s] + out_len[svc == s] / 2) * out_len[svc == s] * services[s].token_bytes)
                    for s in range(ns)])
    unit = time_unit / life.min()
    profiles = [(float(life[s] * unit), float(std[s] * unit), float(starvation_threshold)) for s in range(ns)]
    return ServeWorkload(services, svc, prompt, out_len, PAGE_BYTES, max_batch, tok_b, tok_b // 4, row_el,
                         int(row_el.max()), cap, table_off, n_pages, profiles, seed)
