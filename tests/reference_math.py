"""Independent reference routines used to pin the oracle.

Nothing here looks at pages: attention is computed on contiguous arrays, by a
different formulation (vectorised numpy, and torch's fp64 SDPA) from the
oracle's scalar C loops.  The paged images the oracle reads are built by
`build_paged_pool`, which places every bf16 element individually from the
statement of the layout (token-major, kv-head-major, K then V), one Python
integer computation per element.
"""
import numpy as np


def bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return (np.asarray(bits, np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def f32_to_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bits, round to nearest even (test-local copy; used only to make exact inputs)."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def contiguous_attention(q_bits, k_bits, v_bits, scale):
    """q [Q,d], k/v [n,H,d] as bf16 bits -> fp64 [Q,d]; query head a uses kv head a // (Q//H)."""
    q, k, v = bits_to_f64(q_bits), bits_to_f64(k_bits), bits_to_f64(v_bits)
    Q, d = q.shape
    n, H, _ = k.shape
    G = Q // H
    out = np.zeros((Q, d))
    for a in range(Q):
        h = a // G
        s = (k[:, h, :] @ q[a]) * scale           # [n]
        w = np.exp(s - s.max())
        w /= w.sum()
        out[a] = w @ v[:, h, :]
    return out


def torch_sdpa_attention(q_bits, k_bits, v_bits, scale):
    import torch
    q = torch.from_numpy(bits_to_f64(q_bits))                       # [Q,d]
    k = torch.from_numpy(bits_to_f64(k_bits)).permute(1, 0, 2)      # [H,n,d]
    v = torch.from_numpy(bits_to_f64(v_bits)).permute(1, 0, 2)
    G = q.shape[0] // k.shape[0]
    k = k.repeat_interleave(G, dim=0)
    v = v.repeat_interleave(G, dim=0)
    o = torch.nn.functional.scaled_dot_product_attention(q[None, :, None, :], k[None], v[None], scale=scale)
    return o[0, :, 0, :].numpy()


def contiguous_causal_attention(q_bits, k_bits, v_bits, scale, first_pos=0):
    """Prefill by the masked-matrix formulation: q [m,Q,d] are the queries of positions first_pos..first_pos+m-1,
    k/v [n,H,d]; scores of tokens beyond a query's own position are set to -inf.  Returns fp64 [m,Q,d]."""
    q, k, v = bits_to_f64(q_bits), bits_to_f64(k_bits), bits_to_f64(v_bits)
    m, Q, d = q.shape
    n, H, _ = k.shape
    G = Q // H
    allowed = np.arange(n)[None, :] <= (first_pos + np.arange(m))[:, None]      # [m, n]
    out = np.zeros((m, Q, d))
    for a in range(Q):
        h = a // G
        s = (q[:, a, :] @ k[:, h, :].T) * scale                                  # [m, n]
        s = np.where(allowed, s, -np.inf)
        w = np.exp(s - s.max(axis=1, keepdims=True))
        w /= w.sum(axis=1, keepdims=True)
        out[:, a, :] = w @ v[:, h, :]
    return out


def torch_sdpa_causal(q_bits, k_bits, v_bits, scale):
    """torch's fp64 SDPA with is_causal=True (square case: as many queries as tokens)."""
    import torch
    q = torch.from_numpy(bits_to_f64(q_bits)).permute(1, 0, 2)      # [Q,n,d]
    k = torch.from_numpy(bits_to_f64(k_bits)).permute(1, 0, 2)      # [H,n,d]
    v = torch.from_numpy(bits_to_f64(v_bits)).permute(1, 0, 2)
    G = q.shape[0] // k.shape[0]
    k = k.repeat_interleave(G, dim=0)
    v = v.repeat_interleave(G, dim=0)
    o = torch.nn.functional.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True, scale=scale)
    return o[0].permute(1, 0, 2).numpy()                             # [n,Q,d]


def build_paged_pool(pool_u16, page_bytes, table, k_bits, v_bits, first_token=0):
    """Place K/V [n,H,d] into the pool image element by element."""
    n, H, d = k_bits.shape
    for t in range(n):
        for h in range(H):
            for which, src in ((0, k_bits), (1, v_bits)):
                for j in range(d):
                    stream_byte = ((first_token + t) * H + h) * (4 * d) + which * 2 * d + 2 * j
                    page = int(table[stream_byte // page_bytes])
                    assert page >= 0
                    byte = page * page_bytes + stream_byte % page_bytes
                    pool_u16[byte // 2] = src[t, h, j]


def copy_logical_kv_to_split(merged, split, gather):
    """Fill the split-layout pool with the K/V the merged-layout batch holds (test-side data movement).

    gather(pool, page_bytes, table, H, d, n) -> (K[n,H,d], V[n,H,d]) reads the merged layout; every
    (request, head) stream of the split batch is then written row by row: token t of a one-head
    stream sits at stream byte t * 4d.
    """
    req, head = split.notes["split_of"]
    cache = {}
    P = split.page_bytes
    for k in range(split.n_requests):
        i, h = int(req[k]), int(head[k])
        n = int(split.ctx_len[k])
        if n == 0:
            continue
        if i not in cache:
            sv = merged.service_of(i)
            cache = {i: gather(merged.pool, merged.page_bytes, merged.table_of(i), sv.n_kv_heads, sv.head_dim, n)}
        K, V = cache[i]
        d = K.shape[2]
        rows = np.concatenate([K[:, h, :], V[:, h, :]], axis=1)          # [n, 2d] bf16 bits
        stream = np.arange(n, dtype=np.int64) * (4 * d)
        page = split.table_of(k)[stream // P].astype(np.int64)
        base = (page * P + stream % P) // 2
        split.pool[base[:, None] + np.arange(2 * d)[None, :]] = rows
