"""The error model behind the two forms of the prefill attention's softmax weights (UKV_PARAM_PREFILL_WEIGHTS),
checked on the CPU in numpy against the plain definition: what rounding the weights to two bf16 parts, or to one
fp16 part that also feeds the denominator, can cost -- the figures the GPU tests hold the kernel to
(tests/test_gpu_prefill.py: EXPECTED) and the bound the header states."""
import numpy as np

from synth import normal_bf16


def _bf16_to_f64(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def _trunc_bf16(x32):
    return (x32.view(np.uint32) & 0xFFFF0000).view(np.float32)


def _rows(n_tok, d, seed):
    rng = np.random.default_rng(seed)
    q = _bf16_to_f64(normal_bf16(d, rng))
    k = _bf16_to_f64(normal_bf16(n_tok * d, rng)).reshape(n_tok, d)
    v = _bf16_to_f64(normal_bf16(n_tok * d, rng)).reshape(n_tok, d)
    return q, k, v


def _weights(q, k, n_seen, d):
    s = (k[:n_seen] @ q) / np.sqrt(d) * np.log2(np.e)
    return np.exp2(s - s.max())                         # in (0, 1], the reference the kernel uses (up to its lazy 2^6)


def test_two_bf16_parts_keep_sixteen_bits_and_one_fp16_part_eleven():
    d = 128
    worst2 = worst1 = 0.0
    for seed, n_tok in ((1, 3), (2, 40), (3, 300), (4, 2000)):
        q, k, v = _rows(n_tok, d, seed)
        for n_seen in sorted({1, 2, 3, n_tok // 2 + 1, n_tok}):
            p = _weights(q, k, n_seen, d)
            exact = (p[:, None] * v[:n_seen]).sum(0) / p.sum()
            p32 = p.astype(np.float32)
            hi = _trunc_bf16(p32)
            lo = _trunc_bf16(p32 - hi)
            p2 = hi.astype(np.float64) + lo.astype(np.float64)
            out2 = (p2[:, None] * v[:n_seen]).sum(0) / p2.sum()
            p1 = (p32 * np.float32(256.0)).astype(np.float16).astype(np.float64)    # 2^8 higher, round to nearest
            out1 = (p1[:, None] * v[:n_seen]).sum(0) / p1.sum()
            e2, e1 = np.abs(out2 - exact).max(), np.abs(out1 - exact).max()
            worst2, worst1 = max(worst2, e2), max(worst1, e1)
            # the stated bound: every weight off by at most 2^-11 of itself (fp16 keeps 11 significant bits), the same
            # weights in the denominator, so a result moves by at most twice that times the spread of V
            spread = np.abs(v[:n_seen] - exact[None, :]).max()
            assert e1 <= 2.0 ** -10 * spread + 1e-12
            assert np.all(np.abs(p1 / 256.0 - p)[p > 2.0 ** -22] <= 2.0 ** -11 * p[p > 2.0 ** -22] * (1 + 1e-6))
            assert np.all(np.abs(p2 - p) <= 2.0 ** -15 * p + 1e-45)
    assert worst2 <= 1e-5          # the kernel adds its fp32 accumulation on top: measured 3e-5, held to 1e-4
    assert 1e-5 < worst1 <= 8e-4   # the one-part form's error is the weights' rounding: measured 4.7e-4, held to 8e-4


def test_fp16_copy_of_v_is_exact_in_range_saturates_beyond_and_drops_what_is_below_two_to_minus_24():
    bits = np.arange(0, 1 << 16, dtype=np.uint32).astype(np.uint16)                # every bf16 pattern
    x = (bits.astype(np.uint32) << 16).view(np.float32)
    finite = np.isfinite(x)
    with np.errstate(over="ignore"):
        y = np.clip(x[finite], -65504.0, 65504.0).astype(np.float16).astype(np.float32)
    xf = x[finite]
    in_range = (np.abs(xf) <= 65504.0) & (np.abs(xf) >= 2.0 ** -14)
    assert np.array_equal(y[in_range], xf[in_range])                                # 8 significant bits fit 11
    assert np.all(np.abs(y[np.abs(xf) > 65504.0]) == 65504.0)
    sub = np.abs(xf) < 2.0 ** -14
    assert np.all(np.abs(y[sub] - xf[sub]) <= 2.0 ** -25)                           # fp16 subnormal spacing 2^-24
    assert np.all(y[np.abs(xf) < 2.0 ** -25] == 0.0)
