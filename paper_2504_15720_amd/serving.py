"""Serving loop over the unified cache, driven by the doubling-budget scheduler of include/ukv_sched.h (section 4.2
and the DB algorithm of the appendix): requests of several services are prefilled (page-table patch, bulk store,
prefill attention) and decoded (ukv_decode_step) to their output lengths; pages come from the pool's free list and
go back when a request finishes.

  policy "db"     one scheduler over all services: an iteration runs ONE batch of one service in one phase (the
                  paper's batching rule);
  policy "mixed"  one scheduler per service: an iteration takes every service's batch, and all decode batches run
                  as ONE mixed-service launch (what the decode kernel here is built for).
  clock "wall"    iterations are charged their measured wall time;
  clock "model"   iterations are charged workload.modelled_time(...) of the batch, so every decision is reproducible.

One attention layer, no model around it; this module only sequences calls of the binding (no arithmetic of the
method on the host).  The workload object comes from synth.serving (duck-typed here).
"""
from __future__ import annotations

import time

import numpy as np

from . import binding as U


class ServingLoop:
    def __init__(self, wl, modelled_time, device="cuda:0"):
        import torch
        self.torch, self.wl, self.modelled_time = torch, wl, modelled_time
        self.dev = dev = torch.device(device)
        P = wl.page_bytes
        self.pool_raw = torch.empty(wl.n_pages * P // 2 + P // 2, dtype=torch.int16, device=dev)
        skip = (-self.pool_raw.data_ptr() % P) // 2
        self.pool_t = self.pool_raw[skip:skip + wl.n_pages * P // 2]
        self.max_prompt = int(wl.prompt.max())
        # worst case of one iteration's prefill batches (one per service under the mixed policy, each with a region
        # of its own in the q / out / source buffers): the max_batch longest prompts of every service
        self.pf_elems = int(sum(np.sort((wl.prompt * wl.row_el)[wl.svc == s])[::-1][:wl.max_batch].sum()
                                for s in range(len(wl.services))))

        def tiled_dev(which, n_el):
            blk = torch.from_numpy(wl.noise_block(which).view(np.int16)).to(dev)
            return blk.repeat(-(-n_el // blk.numel()))[:n_el].contiguous()

        self.src_k, self.src_v, self.pf_q = (tiled_dev(w, self.pf_elems) for w in (0, 1, 2))
        self.pool_fill = tiled_dev(3, self.pool_t.numel())
        self.pf_out = torch.empty(self.pf_elems, dtype=torch.float32, device=dev)
        dq, dnk, dnv = wl.decode_inputs()
        self.dq, self.dnk, self.dnv = (torch.from_numpy(a.view(np.int16)).to(dev) for a in (dq, dnk, dnv))
        self.dout = torch.empty(wl.n * wl.row_max, dtype=torch.float32, device=dev)
        self.slot_off = (np.arange(wl.n) * wl.row_max).astype(np.uint64)
        self.table_t = torch.full((int(wl.cap.sum()),), -1, dtype=torch.int32, device=dev)
        self.stream = torch.cuda.current_stream().cuda_stream

    def run(self, policy: str, clock: str = "wall", observer=None) -> dict:
        """Serve every request of the workload to completion.  observer(event), if given, is called at the end of
        every iteration (after the device has finished it and the scheduler has been told), with the iteration's
        decisions and inputs; the iteration's outputs are still in self.dout / self.pf_out at that point."""
        torch, wl = self.torch, self.wl
        n, P, ns = wl.n, wl.page_bytes, len(wl.services)
        svc, prompt, out_len, tok_b, tok_el, row_el = wl.svc, wl.prompt, wl.out_len, wl.tok_b, wl.tok_el, wl.row_el
        table_off, table_t, stream = wl.table_off, self.table_t, self.stream
        self.pool_t.copy_(self.pool_fill)
        table_t.fill_(-1)
        pool = self.pool = U.ukv_pool_create(self.pool_t.data_ptr(), wl.n_pages * P, P, wl.services)
        scheds = self.scheds = ([U.ukv_sched_create(pool, wl.profiles, wl.max_batch)] if policy == "db"
                                else [U.ukv_sched_create(pool, wl.profiles, wl.max_batch) for _ in range(ns)])
        ws_bytes = max(U.ukv_decode_workspace_bytes(pool, n),
                       U.ukv_prefill_workspace_bytes_one_part(pool, wl.max_batch, wl.max_batch * self.max_prompt,
                                                              wl.max_batch * self.max_prompt))
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device=self.dev)
        self.ctx = ctx = np.zeros(n, np.int64)
        owned = [[] for _ in range(n)]
        finish = np.zeros(n)
        for r in range(n):
            U.ukv_sched_add_request(scheds[0 if policy == "db" else int(svc[r])], r, int(svc[r]), int(prompt[r]), 0.0)
        n_iter = n_launch = 0

        def take_pages(ids, new_ctx):
            entry, page = [], []
            for r, c in zip(ids, new_ctx):
                have = len(owned[r])
                need = int(-(-c * tok_b[r] // P)) - have
                if need > 0:
                    got = U.ukv_pages_alloc(pool, need)
                    entry.extend(int(table_off[r]) + have + k for k in range(need))
                    page.extend(got.tolist())
                    owned[r].extend(got.tolist())
            return np.array(entry, np.uint64), np.array(page, np.int32)

        def prefill(ids, base):
            """base: (K/V source elements, q/out elements) already used by this iteration's earlier prefill batches"""
            ids = np.array(ids)
            entry, page = take_pages(ids, prompt[ids])
            kv_off = (base[0] + np.cumsum(prompt[ids] * tok_el[ids]) - prompt[ids] * tok_el[ids]).astype(np.uint64)
            q_off = (base[1] + np.cumsum(prompt[ids] * row_el[ids]) - prompt[ids] * row_el[ids]).astype(np.uint64)
            base[0] += int((prompt[ids] * tok_el[ids]).sum())
            base[1] += int((prompt[ids] * row_el[ids]).sum())
            assert len(ids) <= wl.max_batch and base[1] <= self.pf_elems
            desc = U.BatchDesc(svc[ids], prompt[ids], table_off[ids], table_t.data_ptr(), self.pf_q.data_ptr(), q_off,
                               self.pf_out.data_ptr(), q_off, 0, 0, None, entry, page)
            U.ukv_append(pool, U.BatchDesc([], [], [], table_t.data_ptr(), 0, None, 0, None, 0, 0, None, entry, page),
                         stream)                                     # the new table entries only
            U.ukv_scatter(pool, desc, self.src_k.data_ptr(), self.src_v.data_ptr(), kv_off, stream)
            U.ukv_prefill_attention(pool, desc, prompt[ids], ws.data_ptr(), ws_bytes, stream)
            ctx[ids] = prompt[ids]
            return dict(kind="prefill", ids=ids, entry=entry, page=page, kv_off=kv_off, q_off=q_off, keep=desc)

        def decode(ids):
            ids = np.array(ids)
            ctx[ids] += 1
            entry, page = take_pages(ids, ctx[ids])
            so = self.slot_off[ids]
            desc = U.BatchDesc(svc[ids], ctx[ids], table_off[ids], table_t.data_ptr(), self.dq.data_ptr(), so,
                               self.dout.data_ptr(), so, self.dnk.data_ptr(), self.dnv.data_ptr(), so, entry, page)
            U.ukv_decode_step(pool, desc, ws.data_ptr(), ws_bytes, stream)
            return dict(kind="decode", ids=ids, entry=entry, page=page, keep=desc)

        t0 = time.perf_counter()
        model_now = 0.0
        while any(U.ukv_sched_pending(sc) for sc in scheds):
            now = model_now if clock == "model" else time.perf_counter() - t0
            free0 = free = int(U.ukv_pool_info(pool, 0).free_pages)
            batches = []
            for k, sc in enumerate(scheds):
                ids, s_, queue = U.ukv_sched_next_batch(sc, now, free, cap=wl.max_batch)
                if ids:
                    free -= sum(U.ukv_sched_pages_needed(sc, i) for i in ids)
                    batches.append((k, ids, s_, queue))
            assert batches, "nothing fits the pool"
            t_it = time.perf_counter()
            dec_ids = [i for _, ids, _, queue in batches if queue == U.UKV_SCHED_DECODING for i in ids]
            work, elapsed_model, base = [], 0.0, [0, 0]
            for _, ids, _, queue in batches:
                if queue == U.UKV_SCHED_WAIT:
                    work.append(prefill(ids, base))
                    elapsed_model += self.modelled_time(True, prompt[np.array(ids)], tok_b[np.array(ids)])
                    n_launch += 1
            if dec_ids:
                work.append(decode(dec_ids))
                elapsed_model += self.modelled_time(False, ctx[np.array(dec_ids)], tok_b[np.array(dec_ids)])
                n_launch += 1
            torch.cuda.synchronize()
            if clock == "model":
                elapsed = elapsed_model
                model_now = now_end = now + elapsed
            else:
                elapsed = time.perf_counter() - t_it
                now_end = time.perf_counter() - t0
            n_iter += 1
            fins = []
            for k, ids, _, queue in batches:
                fin = [bool(ctx[i] >= prompt[i] + out_len[i]) for i in ids]
                fins.append(fin)
                U.ukv_sched_complete(scheds[k], ids, fin, elapsed, now_end)
            if observer is not None:   # before the finished requests' pages go back: their caches can still be read
                observer(dict(iteration=n_iter - 1, now=now, now_end=now_end, elapsed=elapsed, free_pages=free0,
                              batches=batches, finished=fins, work=work, loop=self))
            for (k, ids, _, queue), fin in zip(batches, fins):
                for i, f in zip(ids, fin):
                    if f:
                        finish[i] = now_end
                        U.ukv_pages_free(pool, np.array(owned[i], np.int32))
                        owned[i] = []
        wall = time.perf_counter() - t0
        torch.cuda.synchronize()
        for sc in scheds:
            U.ukv_sched_destroy(sc)
        U.ukv_pool_destroy(pool)
        self.pool, self.scheds = 0, []
        tokens = int(out_len.sum())
        norm = finish / out_len
        return {"wall_s": wall, "iterations": n_iter, "launch_groups": n_launch, "generated_tokens": tokens,
                "prompt_tokens": int(prompt.sum()), "clock": clock, "policy": policy,
                "mean_latency_per_output_token_ms": {str(s): round(float(norm[svc == s].mean() * 1e3), 4)
                                                     for s in range(ns)}}
