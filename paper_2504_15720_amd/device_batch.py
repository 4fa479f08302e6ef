"""A batch on the device: copies a host-side batch description (pool image, page tables, q) into torch tensors,
creates the pool and drives the C-ABI binding with their pointers.  Used by the benchmark, the smoke check and the
GPU tests.  It performs no arithmetic of the method."""
from __future__ import annotations

import numpy as np

from . import binding as U


def replay_stack_log(pool: int, log) -> None:
    """Bring the library's free list to the state of a synthetic PageStack by replaying its operations."""
    for op, arg in log:
        if op == "alloc":
            U.ukv_pages_alloc(pool, int(arg))
        else:
            U.ukv_pages_free(pool, arg)


class DeviceBatch:
    """Device copies of a synthetic batch + the pool handle."""

    def __init__(self, b, device="cuda:0", profile=False):
        import torch
        self.torch = torch
        self.b = b
        self.dev = torch.device(device)
        assert b.pool is not None
        n_el = b.n_pages * b.page_bytes // 2
        self._pool_raw = torch.empty(n_el + b.page_bytes // 2, dtype=torch.int16, device=self.dev)
        skip = (-self._pool_raw.data_ptr() % b.page_bytes) // 2          # page-align the pool base
        self.pool_t = self._pool_raw[skip:skip + n_el]
        self.pool_t.copy_(torch.from_numpy(b.pool.view(np.int16)))
        assert self.pool_t.data_ptr() % b.page_bytes == 0
        self.pool = U.ukv_pool_create(self.pool_t.data_ptr(), b.n_pages * b.page_bytes, b.page_bytes, b.services)
        replay_stack_log(self.pool, b.stack.log)
        self.table_t = torch.from_numpy(b.page_table.copy()).to(self.dev)
        self.q_t = torch.from_numpy(b.q.view(np.int16).copy()).to(self.dev)
        self.out_t = torch.full((b.out_elems,), float("nan"), dtype=torch.float32, device=self.dev)
        self.newk_t = torch.zeros(b.new_elems, dtype=torch.int16, device=self.dev)
        self.newv_t = torch.zeros(b.new_elems, dtype=torch.int16, device=self.dev)
        self.ws_bytes = U.ukv_decode_workspace_bytes(self.pool, b.n_requests)
        self.ws_t = torch.empty(self.ws_bytes, dtype=torch.uint8, device=self.dev)
        if profile:  # True = every launch; an integer n = every n-th launch of each kernel
            U.ukv_set_param(self.pool, U.UKV_PARAM_PROFILE, int(profile))

    def close(self):
        if self.pool:
            self.torch.cuda.synchronize()
            if getattr(self, "plan", 0):
                U.ukv_plan_destroy(self.plan)
                self.plan = 0
            U.ukv_pool_destroy(self.pool)
            self.pool = 0

    def make_plan(self):
        """A plan kept across steps for the batch as it is now (it owns the workspace from here on)."""
        if getattr(self, "plan", 0):
            U.ukv_plan_destroy(self.plan)
        self.plan = U.ukv_plan_create(self.pool, self.desc(), self.ws_t.data_ptr(), self.ws_bytes)
        return self.plan

    def plan_step(self, new_pages, advance=True):
        """One decode step of the kept plan: every request grows by one token (append + attention, one launch)."""
        U.ukv_plan_step(self.plan, new_pages, advance, None, self.stream())

    def resize_workspace(self):
        self.ws_bytes = U.ukv_decode_workspace_bytes(self.pool, self.b.n_requests)
        self.ws_t = self.torch.empty(self.ws_bytes, dtype=self.torch.uint8, device=self.dev)

    def stream(self) -> int:
        return self.torch.cuda.current_stream().cuda_stream

    def desc(self, patch_entry=None, patch_page=None) -> "U.BatchDesc":
        b = self.b
        return U.BatchDesc(b.service_id, b.ctx_len, b.table_off, self.table_t.data_ptr(), self.q_t.data_ptr(),
                           b.q_off, self.out_t.data_ptr(), b.out_off, self.newk_t.data_ptr(),
                           self.newv_t.data_ptr(), b.new_off, patch_entry, patch_page)

    def set_q(self, q_bits: np.ndarray):
        self.q_t.copy_(self.torch.from_numpy(q_bits.view(np.int16)))

    def set_new(self, k_bits: np.ndarray, v_bits: np.ndarray):
        self.newk_t.copy_(self.torch.from_numpy(k_bits.view(np.int16)))
        self.newv_t.copy_(self.torch.from_numpy(v_bits.view(np.int16)))

    def decode(self, desc=None):
        U.ukv_decode_attention(self.pool, desc or self.desc(), self.ws_t.data_ptr(), self.ws_bytes, self.stream())

    def append(self, desc):
        U.ukv_append(self.pool, desc, self.stream())

    def step(self, desc):
        """append + attention as one launch"""
        U.ukv_decode_step(self.pool, desc, self.ws_t.data_ptr(), self.ws_bytes, self.stream())

    def prefill(self, q_len, q_bits: np.ndarray, q_off, out_off, n_elems: int):
        """Causal attention of the last q_len[i] tokens of every request; returns (fp32 output tensor, desc)."""
        torch = self.torch
        b = self.b
        q_len = np.ascontiguousarray(q_len, np.uint32)
        q_t = torch.from_numpy(q_bits.view(np.int16).copy()).to(self.dev)
        out_t = torch.full((n_elems,), float("nan"), dtype=torch.float32, device=self.dev)
        # room for the fp16 copy of V as well, so that the call may take the one-part weights
        ws = U.ukv_prefill_workspace_bytes_one_part(self.pool, b.n_requests, int(q_len.sum()),
                                                    int(b.ctx_len[q_len > 0].astype(np.int64).sum()))
        if getattr(self, "pf_ws_t", None) is None or self.pf_ws_t.numel() < ws:
            self.pf_ws_t = torch.empty(ws, dtype=torch.uint8, device=self.dev)
        desc = U.BatchDesc(b.service_id, b.ctx_len, b.table_off, self.table_t.data_ptr(), q_t.data_ptr(), q_off,
                           out_t.data_ptr(), out_off, self.newk_t.data_ptr(), self.newv_t.data_ptr(), b.new_off,
                           None, None)
        self._pf_keep = (q_t, out_t, desc)

        def run():
            U.ukv_prefill_attention(self.pool, desc, q_len, self.pf_ws_t.data_ptr(), ws, self.stream())
        run()
        return out_t, run

    def out_host(self) -> np.ndarray:
        return self.out_t.cpu().numpy()

    def pool_host(self) -> np.ndarray:
        return self.pool_t.cpu().numpy().view(np.uint16)

    def kv_layout(self):
        """Element offsets / sizes of every request in the contiguous K (or V) array of gather/scatter."""
        b = self.b
        tok_elems = np.array([b.services[s].n_kv_heads * b.services[s].head_dim for s in b.service_id], np.int64)
        sizes = b.ctx_len.astype(np.int64) * tok_elems
        return (np.cumsum(sizes) - sizes).astype(np.uint64), sizes

    def scatter(self, k_t, v_t, kv_off):
        U.ukv_scatter(self.pool, self.desc(), k_t.data_ptr(), v_t.data_ptr(), kv_off, self.stream())

    def scatter_tokens(self, n_new, k_t, v_t, kv_off):
        U.ukv_scatter_tokens(self.pool, self.desc(), n_new, k_t.data_ptr(), v_t.data_ptr(), kv_off, self.stream())

    def gather_device(self):
        kv_off, sizes = self.kv_layout()
        total = int(sizes.sum())
        k = self.torch.zeros(max(total, 8), dtype=self.torch.int16, device=self.dev)
        v = self.torch.zeros(max(total, 8), dtype=self.torch.int16, device=self.dev)
        U.ukv_gather(self.pool, self.desc(), k.data_ptr(), v.data_ptr(), kv_off, self.stream())
        return k, v, kv_off, sizes

    def gather(self):
        b = self.b
        tok_elems = np.array([b.services[s].n_kv_heads * b.services[s].head_dim for s in b.service_id], np.int64)
        sizes = b.ctx_len.astype(np.int64) * tok_elems
        kv_off = (np.cumsum(sizes) - sizes).astype(np.uint64)
        total = int(sizes.sum())
        k = self.torch.zeros(max(total, 8), dtype=self.torch.int16, device=self.dev)
        v = self.torch.zeros(max(total, 8), dtype=self.torch.int16, device=self.dev)
        U.ukv_gather(self.pool, self.desc(), k.data_ptr(), v.data_ptr(), kv_off, self.stream())
        return k.cpu().numpy().view(np.uint16), v.cpu().numpy().view(np.uint16), kv_off, sizes
