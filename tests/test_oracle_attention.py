"""Pins for the oracle's decode attention over the compressed cache (Figure 1; Section 3.3.2).

The fused path must equal plain softmax attention on the dequantized tensors (the paper's multi-kernel pipeline
computes exactly that, Section 4.3), which numpy evaluates here independently; closed forms cover the softmax
(zero query -> uniform average) and the limit of a tiny error bound (-> attention on the raw fp16 cache).
"""
import numpy as np
import pytest

import workloads as W

K, V = 0, 1


def _softmax_attention(q, Kd, Vd, scale):
    s = scale * (Kd @ q)
    p = np.exp(s - s.max())
    p /= p.sum()
    return p @ Vd


def _dequantized(oracle, oc, which, b, h):
    rows = [oracle.dequantize_block(which, *oracle.decode_block_serial(which, oc.get_block(which, b, h, j),
                                                                       oc.len[which]), oc.rel_eb[which])
            for j in range(oc.n_blocks)]
    rows.append(oc.res[which][b, : oc.n_res, h].astype(np.float64))
    return np.concatenate(rows, axis=0)


@pytest.mark.parametrize("B,H,Hq,S", [(1, 1, 1, 256), (2, 2, 8, 200), (1, 3, 3, 40)])
def test_equals_numpy_attention_on_dequantized_cache(oracle, B, H, Hq, S):
    Kx, Vx = W.make_kv(B, H, max(S, 64), 12)
    oc = oracle.OracleCache(B, H, Hq, 512, 1e-2, 1e-2)
    oc.build_codebook(Kx, Vx)
    oc.compress_blocks(Kx[:, :S], Vx[:, :S])
    q = W.make_queries(B, Hq, 1, 12)[0]
    scale = 1 / np.sqrt(128)
    out = oc.attn_decode(q, scale)
    G = Hq // H
    for b in range(B):
        for hq in range(Hq):
            Kd, Vd = _dequantized(oracle, oc, K, b, hq // G), _dequantized(oracle, oc, V, b, hq // G)
            assert Kd.shape == (S, 128)
            ref = _softmax_attention(q[b, hq].astype(np.float64), Kd, Vd, scale)
            np.testing.assert_allclose(out[b, hq], ref, rtol=1e-12, atol=1e-14)


def test_zero_query_gives_the_mean_of_v(oracle):
    Kx, Vx = W.make_kv(1, 1, 192, 13)
    oc = oracle.OracleCache(1, 1, 1, 192, 1e-2, 1e-2)
    oc.build_codebook(Kx, Vx)
    oc.compress_blocks(Kx, Vx)
    out = oc.attn_decode(np.zeros((1, 1, 128), np.float16), 0.3)
    Vd = _dequantized(oracle, oc, V, 0, 0)
    np.testing.assert_allclose(out[0, 0], Vd.mean(axis=0), rtol=1e-12, atol=1e-14)
    # and the mean of V' is within the per-token error bound of the mean of V
    v64 = Vx[0, :, 0].astype(np.float64)
    eb = 1e-2 * (v64.max(axis=1) - v64.min(axis=1))
    assert np.all(np.abs(out[0, 0] - v64.mean(axis=0)) <= eb.mean() * (1 + 1e-4))


def test_a_dominant_key_selects_its_value_row(oracle):
    Kx, Vx = W.make_kv(1, 1, 128, 14)
    q = W.make_queries(1, 1, 1, 14)[0]
    Kx[0, 77, 0] = (q[0, 0].astype(np.float32) * 40).astype(np.float16)  # score of token 77 dwarfs the rest
    oc = oracle.OracleCache(1, 1, 1, 128, 5e-3, 5e-3)
    oc.build_codebook(Kx, Vx)
    oc.compress_blocks(Kx, Vx)
    out = oc.attn_decode(q, 1.0)
    Vd = _dequantized(oracle, oc, V, 0, 0)
    np.testing.assert_allclose(out[0, 0], Vd[77], rtol=0, atol=1e-9)


def test_small_error_bound_converges_to_raw_attention(oracle):
    Kx, Vx = W.make_kv(1, 2, 256, 15)
    q = W.make_queries(1, 2, 1, 15)[0]
    scale = 1 / np.sqrt(128)
    raw = np.stack([_softmax_attention(q[0, h].astype(np.float64), Kx[0, :, h].astype(np.float64),
                                       Vx[0, :, h].astype(np.float64), scale) for h in range(2)])
    errs = []
    for rel_eb in (2e-2, 1e-2, 2.5e-3, 2e-3):
        oc = oracle.OracleCache(1, 2, 2, 256, rel_eb, rel_eb)
        oc.build_codebook(Kx, Vx)
        oc.compress_blocks(Kx, Vx)
        err = np.abs(oc.attn_decode(q, scale)[0] - raw).max(axis=1)
        errs.append(err.max())
        # propagation bound: |ds_t| <= scale * sum_c |q_c| eb_c =: d;  ||p' - p||_1 <= exp(2d) - 1;
        # |do_c| <= (exp(2d) - 1) * max|V| + max eb_v
        for h in range(2):
            k64 = Kx[0, :, h].astype(np.float64).reshape(4, 64, 128)
            eb_k = rel_eb * (k64.max(axis=1) - k64.min(axis=1))  # [block, channel]
            d = scale * (np.abs(q[0, h].astype(np.float64))[None, :] * eb_k).sum(axis=1).max()
            v64 = Vx[0, :, h].astype(np.float64)
            eb_v = rel_eb * (v64.max(axis=1) - v64.min(axis=1)).max()
            assert err[h] <= (np.exp(2 * d) - 1) * np.abs(v64).max() + eb_v
    assert errs[0] > errs[1] > errs[2]
    assert errs[3] < errs[0] / 4


def test_tokens_in_the_buffer_take_part_unquantized(oracle):
    # Section 3.2.3: the buffered fp16 vectors take part in attention as they are.  With a buffer larger than the
    # sequence nothing is compressed and the result is plain softmax attention on the raw fp16 cache, whatever the
    # codebook; with a window of 128 the newest tokens are exact and only the older ones carry quantization error.
    B, H, Hq, S = 2, 2, 4, 300
    Kx, Vx = W.make_kv(B, H, S, 16)
    q = W.make_queries(B, Hq, 1, 16)[0]
    scale = 1 / np.sqrt(128)
    oc = oracle.OracleCache(B, H, Hq, 512, 2e-2, 2e-2, buffer_tokens=320)
    oc.build_codebook(Kx, Vx)
    oc.compress_blocks(Kx[:, :280], Vx[:, :280])
    for t in range(280, S):
        oc.append_token(Kx[:, t], Vx[:, t])
    assert oc.n_blocks == 0 and oc.n_res == S
    out = oc.attn_decode(q, scale)
    for b in range(B):
        for hq in range(Hq):
            h = hq // 2
            ref = _softmax_attention(q[b, hq].astype(np.float64), Kx[b, :, h].astype(np.float64),
                                     Vx[b, :, h].astype(np.float64), scale)
            np.testing.assert_allclose(out[b, hq], ref, rtol=1e-12, atol=1e-14)
    win = oracle.OracleCache(B, H, Hq, 512, 2e-2, 2e-2, buffer_tokens=128)
    win.build_codebook(Kx, Vx)
    win.compress_blocks(Kx, Vx)
    assert win.n_blocks == 3 and win.n_res == 108
    out = win.attn_decode(q, scale)
    for b in range(B):
        for hq in range(Hq):
            Kd, Vd = _dequantized(oracle, win, K, b, hq // 2), _dequantized(oracle, win, V, b, hq // 2)
            np.testing.assert_array_equal(Kd[192:], Kx[b, 192:, hq // 2].astype(np.float64))
            ref = _softmax_attention(q[b, hq].astype(np.float64), Kd, Vd, scale)
            np.testing.assert_allclose(out[b, hq], ref, rtol=1e-12, atol=1e-14)


def test_factored_dot_product_is_an_identity(oracle):
    # q . (min + code*step) == q.min + (q*step).code per channel-wise unit; sum_t p (vmin + vstep code) likewise
    rng = np.random.default_rng(16)
    x = rng.standard_normal((64, 128)).astype(np.float16)
    q = rng.standard_normal(128)
    codes, mm = oracle.quantize_block(K, x, 1e-2)
    Kd = oracle.dequantize_block(K, codes, mm, 1e-2)
    mn = mm[:, 0].view(np.float16).astype(np.float64)
    # the bin width comes from two dequantized grid points
    g0 = oracle.dequantize_block(K, np.zeros((64, 128), np.uint8), mm, 1e-2)[0]
    g1 = oracle.dequantize_block(K, np.ones((64, 128), np.uint8), mm, 1e-2)[0]
    width = g1 - g0
    np.testing.assert_array_equal(g0, mn)
    lhs = Kd @ q
    rhs = q @ mn + codes.astype(np.float64) @ (q * width)
    np.testing.assert_allclose(lhs, rhs, rtol=1e-12, atol=1e-12)


def test_single_head_routine_against_numpy(oracle):
    rng = np.random.default_rng(18)
    Kd, Vd = rng.standard_normal((37, 128)), rng.standard_normal((37, 128))
    q = rng.standard_normal(128).astype(np.float16)
    np.testing.assert_allclose(oracle.attention_head(Kd, Vd, q, 0.2),
                               _softmax_attention(q.astype(np.float64), Kd, Vd, 0.2), rtol=1e-12, atol=1e-14)
