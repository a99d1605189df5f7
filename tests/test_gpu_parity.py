"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Bit-exact for codes, min/max metadata, histograms, codebooks, records, offsets and the fp16 buffer; attention within
max|o_gpu - o_oracle| <= 1e-3 * max(1, max|o_oracle|).
"""
import sys

import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu

K, V = 0, 1
SCALE = 1.0 / np.sqrt(128.0)


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2509_00579_amd import binding
    binding.load()
    return binding


def _dev(x):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0")


def _attn_close(o_gpu, o_ref):
    o_ref = np.asarray(o_ref, np.float64)
    err = np.abs(o_gpu.astype(np.float64) - o_ref).max()
    tol = 1e-3 * max(1.0, np.abs(o_ref).max())
    assert np.isfinite(o_gpu).all()
    assert err <= tol, f"max abs err {err:.3e} > {tol:.3e}"
    return err


def _both(gpu, oracle, B, H, Hq, S_book, S, max_seq, rel_k, rel_v, seed, limit=12):
    """Build codebooks on the first S_book tokens and compress S tokens on both sides (code words of up to `limit`
    bits; 12 is the library's default)."""
    Kx, Vx = W.make_kv(B, H, max(S_book, S), seed)
    oc = oracle.OracleCache(B, H, Hq, max_seq, rel_k, rel_v, 0, limit)
    oc.build_codebook(Kx[:, :S_book], Vx[:, :S_book])
    oc.compress_blocks(Kx[:, :S], Vx[:, :S])
    gc = gpu.KVCompCache(B, H, Hq, max_seq, rel_k, rel_v, max_code_len=limit)
    gc.build_codebook(_dev(Kx[:, :S_book]), _dev(Vx[:, :S_book]))
    gc.compress_blocks(_dev(Kx[:, :S]), _dev(Vx[:, :S]))
    return Kx, Vx, oc, gc


def _assert_same_cache(oc, gc, sample=None):
    st_o, st_g = oc.stats(), gc.stats()
    for key in ("n_blocks", "n_res", "raw_bytes", "record_bytes_k", "record_bytes_v", "header_bytes", "offsets_bytes",
                "residual_bytes", "payload_bits_k", "payload_bits_v", "stored_bytes"):
        assert st_o[key] == st_g[key], key
    assert abs(st_o["compression_ratio"] - st_g["compression_ratio"]) < 1e-12
    blocks = [(w, b, h, j) for w in (K, V) for b in range(oc.B) for h in range(oc.H) for j in range(oc.n_blocks)]
    if sample is not None and len(blocks) > sample:
        rng = np.random.default_rng(0)
        keep = rng.choice(len(blocks), sample, replace=False)
        blocks = [blocks[i] for i in keep]
    for w, b, h, j in blocks:
        bh = b * oc.H + h
        assert gc.block_entry(w, b, h, j) == (int(oc.off16[w][bh, j]), int(oc.size16[w][bh, j])), (w, b, h, j)
        np.testing.assert_array_equal(gc.get_block(w, b, h, j), oc.get_block(w, b, h, j), err_msg=str((w, b, h, j)))
    for w in (K, V):
        res, n = gc.residual(w)
        assert n == oc.n_res
        np.testing.assert_array_equal(res.view(np.uint16), oc.res[w][:, : oc.n_res].view(np.uint16))


@pytest.mark.parametrize("B,H,S,rel", [(1, 1, 1024, 1e-2), (2, 3, 200, 5e-3), (1, 2, 320, 2e-2)])
def test_codes_minmax_histogram_codebook(gpu, oracle, B, H, S, rel):
    _say(f"codes/hist B={B} H={H} S={S} rel={rel}")
    Kx, Vx = W.make_kv(B, H, S, 21)
    Kx[0, 64:128, 0, 5] = np.float16(0.75)   # a constant K unit
    Vx[0, 70, 0, :] = np.float16(-0.0)       # a constant V unit of negative zeros
    gc = gpu.KVCompCache(B, H, H, S, rel, rel)
    gc.build_codebook(_dev(Kx), _dev(Vx))
    for which, X in ((K, Kx), (V, Vx)):
        codes_o, mm_o = oracle.tensor_quantize(which, X, rel)
        codes_g, mm_g = gc.debug_codes(which, _dev(X))
        np.testing.assert_array_equal(mm_g, mm_o)
        np.testing.assert_array_equal(codes_g, codes_o)
        hist_o = oracle.histogram(codes_o)
        np.testing.assert_array_equal(gc.histogram(which).astype(np.uint64), hist_o)
        ln_o, cd_o, _ = oracle.build_codebook(hist_o, oracle.n_sym(rel), 12)
        ln_g, cd_g = gc.codebook(which)
        np.testing.assert_array_equal(ln_g, ln_o)
        np.testing.assert_array_equal(cd_g, cd_o)
    gc.close()


def test_config0_end_to_end(gpu, oracle):
    w = W.CONFIGS["c0"]
    _say("config 0: compress + one decode step")
    Kx, Vx, oc, gc = _both(gpu, oracle, w.batch, w.n_kv_heads, w.n_q_heads, w.seq, w.seq, w.seq, w.rel_eb, w.rel_eb, w.seed,
                           limit=W.CODE_LEN_LIMIT[w.rel_eb])
    _assert_same_cache(oc, gc)
    q = W.make_queries(w.batch, w.n_q_heads, 1, w.seed)[0]
    out = gc.attn_decode(_dev(q), SCALE).cpu().numpy()
    err = _attn_close(out, oc.attn_decode(q, SCALE))
    _say(f"  attention max abs err {err:.3e}; CR {gc.stats()['compression_ratio']:.3f}")
    gc.close()


@pytest.mark.parametrize("B,H,Hq,S,rel_k,rel_v", [
    (2, 2, 2, 520, 1e-2, 2e-2),     # ragged tail of 8 tokens, several blocks per wave
    (1, 2, 8, 333, 5e-3, 1e-2),     # GQA group of 4
    (1, 1, 8, 192, 2e-2, 2e-2),     # GQA group of 8, no residual
    (3, 2, 4, 129, 1e-2, 1e-2),     # GQA group of 2, one-token tail
    (1, 1, 8, 200, 2e-3, 2e-3),     # 251 quantization levels: symbols above 127 through the int8 products of a group
    (1, 2, 8, 136, 2e-3, 4e-3),     # the same for a group of 4
])
def test_records_and_attention(gpu, oracle, B, H, Hq, S, rel_k, rel_v):
    _say(f"records+attention B={B} H={H} Hq={Hq} S={S}")
    Kx, Vx, oc, gc = _both(gpu, oracle, B, H, Hq, S, S, S + 64, rel_k, rel_v, 22)
    _assert_same_cache(oc, gc)
    for step in range(2):
        q = W.make_queries(B, Hq, 2, 22)[step]
        out = gc.attn_decode(_dev(q), SCALE).cpu().numpy()
        _attn_close(out, oc.attn_decode(q, SCALE))
    gc.close()


@pytest.mark.parametrize("B,H,Hq,S,rel_k,rel_v,k_mode,limit,window", [
    (2, 2, 2, 520, 1e-2, 2e-2, 0, 12, 64),     # ragged tail
    (1, 3, 3, 333, 5e-3, 1e-2, 1, 9, 64),      # K BlockQuant: one {min,max} pair per block in the workspace
    (1, 2, 8, 700, 1e-2, 1e-2, 0, 6, 256),     # buffer of 256 tokens: fewer blocks are encoded than were quantized
    (2, 1, 4, 64, 2e-2, 2e-2, 0, 6, 64),       # a single block
])
def test_prefill_with_one_quantization_pass(gpu, oracle, B, H, Hq, S, rel_k, rel_v, k_mode, limit, window):
    """kvcomp_prefill = kvcomp_build_codebook + kvcomp_compress_blocks with the codes kept in a workspace between the
    histogram pass and the encoder: histograms, codebooks, records, offsets, buffer and attention against the oracle,
    and the arena byte for byte against the two separate calls."""
    _say(f"prefill B={B} H={H} Hq={Hq} S={S} rel {rel_k}/{rel_v} k_mode={k_mode} limit {limit} buffer {window}")
    import torch
    Kx, Vx = W.make_kv(B, H, S, 38)
    Kx[0, 0:64, 0, 7] = np.float16(1.25)      # a constant K unit
    oc = oracle.OracleCache(B, H, Hq, S + 64, rel_k, rel_v, k_mode, limit, buffer_tokens=window)
    oc.build_codebook(Kx, Vx)
    oc.compress_blocks(Kx, Vx)
    gc = gpu.KVCompCache(B, H, Hq, S + 64, rel_k, rel_v, k_mode=k_mode, max_code_len=limit, buffer_tokens=window)
    dK, dV = _dev(Kx), _dev(Vx)
    ws = torch.full((gc.prefill_workspace_bytes(S) + 64,), 0xAB, dtype=torch.uint8, device="cuda:0")
    gc.prefill(dK, dV, ws[: gc.prefill_workspace_bytes(S)])
    assert (ws[gc.prefill_workspace_bytes(S):] == 0xAB).all()      # nothing written past the stated size
    for which in (K, V):
        np.testing.assert_array_equal(gc.histogram(which).astype(np.uint64), oc.hist[which])
        ln_g, cd_g = gc.codebook(which)
        np.testing.assert_array_equal(ln_g, oc.len[which])
        np.testing.assert_array_equal(cd_g, oc.code[which])
    _assert_same_cache(oc, gc)
    q = W.make_queries(B, Hq, 1, 38)[0]
    _attn_close(gc.attn_decode(_dev(q), SCALE).cpu().numpy(), oc.attn_decode(q, SCALE))
    one_pass = [gc.get_block(w, b, h, j) for w in (K, V) for b in range(B) for h in range(H) for j in range(oc.n_blocks)]
    gc.reset(keep_codebook=False)
    gc.build_codebook(dK, dV)
    gc.compress_blocks(dK, dV)
    two_calls = [gc.get_block(w, b, h, j) for w in (K, V) for b in range(B) for h in range(H) for j in range(oc.n_blocks)]
    for a, b_ in zip(one_pass, two_calls):
        np.testing.assert_array_equal(a, b_)
    # errors: too small a workspace, a cache that is not empty, non-finite input
    with pytest.raises(gpu.KvcompError) as e:
        gc.prefill(dK, dV, ws)
    assert e.value.status == gpu.ERR_STATE
    gc.reset(keep_codebook=False)
    with pytest.raises(gpu.KvcompError) as e:
        gc.prefill(dK, dV, ws[:1024])
    assert e.value.status == gpu.ERR_CAPACITY
    bad = Kx.copy()
    bad[0, 3, 0, 5] = np.nan
    with pytest.raises(gpu.KvcompError) as e:
        gc.prefill(_dev(bad), dV, ws)
    assert e.value.status == gpu.ERR_NONFINITE
    gc.prefill(dK, dV, ws)
    _assert_same_cache(oc, gc)
    gc.close()


def test_one_context_two_prompts_with_different_codebooks(gpu, oracle):
    """A context that is reset and filled again builds new codebooks: the tables that the second prompt is encoded and
    decoded with must be the second prompt's (the tables travel from a pinned host block that is rewritten in place).
    Second prompt: values on a coarse grid, so that most quantization levels are never used and the code lengths
    differ from the first prompt's in almost every symbol."""
    _say("one context, two prompts")
    B, H, Hq, S = 1, 2, 2, 384
    Ka, Va = W.make_kv(B, H, S, 61)
    rng = np.random.default_rng(62)
    Kb = (rng.integers(-3, 4, size=Ka.shape) * 0.5).astype(np.float16)
    Vb = (rng.integers(0, 2, size=Va.shape) * 2.0 - 1.0).astype(np.float16)
    gc = gpu.KVCompCache(B, H, Hq, S + 64, 1e-2, 1e-2, max_code_len=6)
    q = W.make_queries(B, Hq, 1, 61)[0]
    books = []
    for Kx, Vx in ((Ka, Va), (Kb, Vb), (Ka, Va)):
        oc = oracle.OracleCache(B, H, Hq, S + 64, 1e-2, 1e-2, 0, 6)
        oc.build_codebook(Kx, Vx)
        oc.compress_blocks(Kx, Vx)
        gc.reset(keep_codebook=False)
        gc.prefill(_dev(Kx), _dev(Vx))
        for which in (K, V):
            ln_g, cd_g = gc.codebook(which)
            np.testing.assert_array_equal(ln_g, oc.len[which])
            np.testing.assert_array_equal(cd_g, oc.code[which])
        _assert_same_cache(oc, gc)
        _attn_close(gc.attn_decode(_dev(q), SCALE).cpu().numpy(), oc.attn_decode(q, SCALE))
        for which in (K, V):   # the stand-alone decompressor reads the single-symbol tables and the tree
            ref = oc.decompress(which)
            np.testing.assert_array_equal(gc.decompress(which, S).cpu().numpy().view(np.uint16), ref.view(np.uint16))
            np.testing.assert_array_equal(gc.decompress(which, S, tree_walk=True).cpu().numpy().view(np.uint16), ref.view(np.uint16))
        books.append(np.asarray(oc.len[K]).copy())
    assert (books[0] != books[1]).sum() > 8    # the two prompts really have different codebooks
    gc.close()


def test_all_residual_and_tiny_sequences(gpu, oracle):
    _say("seq < 64: everything stays in the fp16 buffer")
    B, H, Hq = 2, 2, 4
    for S in (1, 40, 63, 64, 65):
        Kx, Vx, oc, gc = _both(gpu, oracle, B, H, Hq, 128, S, 128, 1e-2, 1e-2, 23)
        _assert_same_cache(oc, gc)
        q = W.make_queries(B, Hq, 1, 23)[0]
        _attn_close(gc.attn_decode(_dev(q), SCALE).cpu().numpy(), oc.attn_decode(q, SCALE))
        gc.close()


@pytest.mark.parametrize("G", [1, 4, 8])
def test_symbols_unseen_at_codebook_build(gpu, oracle, G):
    _say(f"codebook from a narrow prefix, later data uses every level; {G} query heads per KV head")
    B, H, S = 1, 2, 256
    Kx, Vx = W.make_kv(B, H, S, 24)
    # the first 64 tokens use only three distinct values per unit -> the histogram sees few levels
    Kx[:, :64] = np.float16(0.0); Kx[:, 0:64:2] = np.float16(1.0); Kx[:, 1:64:7] = np.float16(0.5)
    Vx[:, :64] = np.float16(0.0); Vx[:, :64, :, ::2] = np.float16(1.0); Vx[:, :64, :, 1::7] = np.float16(0.5)
    oc = oracle.OracleCache(B, H, G * H, S, 1e-2, 1e-2)
    oc.build_codebook(Kx[:, :64], Vx[:, :64])
    oc.compress_blocks(Kx, Vx)
    gc = gpu.KVCompCache(B, H, G * H, S, 1e-2, 1e-2)
    gc.build_codebook(_dev(Kx[:, :64]), _dev(Vx[:, :64]))
    gc.compress_blocks(_dev(Kx), _dev(Vx))
    assert int(oc.len[K].max()) > 8  # rare levels got long code words
    _assert_same_cache(oc, gc)
    q = W.make_queries(B, G * H, 1, 24)[0]
    _attn_close(gc.attn_decode(_dev(q), SCALE).cpu().numpy(), oc.attn_decode(q, SCALE))
    # the same cache decoded with a staging area smaller than its records (global-memory path)
    assert gc.stats()["max_record_bytes"] > 4608
    gc.set_tuning(stage_bytes=4608)
    _attn_close(gc.attn_decode(_dev(q), SCALE).cpu().numpy(), oc.attn_decode(q, SCALE))
    gc.set_tuning(n_splits=3)
    _attn_close(gc.attn_decode(_dev(q), SCALE).cpu().numpy(), oc.attn_decode(q, SCALE))
    gc.close()


def test_append_path(gpu, oracle):
    _say("append: 150 tokens one by one, two flushes")
    B, H, Hq, S0, extra = 2, 2, 4, 100, 150
    Kx, Vx, oc, gc = _both(gpu, oracle, B, H, Hq, S0, S0, 256, 1e-2, 1e-2, 25)
    kn, vn = W.make_new_tokens(B, H, extra, 25)
    qs = W.make_queries(B, Hq, extra, 25)
    dkn, dvn, dq = _dev(kn), _dev(vn), _dev(qs)
    for t in range(extra):
        oc.append_token(kn[t], vn[t])
        gc.append_token(dkn[t], dvn[t])
        if t % 37 == 0 or t in (27, 28, 91, 92, extra - 1):   # around the flushes at t = 27 and t = 91
            _attn_close(gc.attn_decode(dq[t], SCALE).cpu().numpy(), oc.attn_decode(qs[t], SCALE))
    assert oc.n_blocks == 3 and oc.n_res == (S0 + extra) % 64
    _assert_same_cache(oc, gc)
    # running the whole sequence again after a reset gives the byte-identical arena (no atomics in the placement)
    first = [gc.get_block(w, b, h, j) for w in (K, V) for b in range(B) for h in range(H) for j in range(3)]
    gc.reset(keep_codebook=True)
    gc.compress_blocks(_dev(Kx[:, :S0]), _dev(Vx[:, :S0]))
    for t in range(extra):
        gc.append_token(dkn[t], dvn[t])
    _assert_same_cache(oc, gc)
    second = [gc.get_block(w, b, h, j) for w in (K, V) for b in range(B) for h in range(H) for j in range(3)]
    for a, b_ in zip(first, second):
        np.testing.assert_array_equal(a, b_)
    gc.close()


@pytest.mark.parametrize("B,H,Hq,window,S0,extra", [(2, 2, 2, 192, 200, 260), (1, 2, 8, 128, 70, 200),
                                                    (1, 1, 8, 1024, 1100, 80), (2, 1, 1, 320, 40, 100)])
def test_larger_buffer_window(gpu, oracle, B, H, Hq, window, S0, extra):
    """A buffer of `window` > 64 tokens (Section 3.2.1, maximum buffer size of Section 4.2): the newest tokens stay
    fp16, the oldest block of a full buffer is compressed.  Records, offsets, buffer contents (oldest first), the
    decompressed cache and the attention output against the oracle, across several wrap-arounds of the ring."""
    _say(f"buffer window {window}: B={B} H={H} Hq={Hq}, prompt {S0} + {extra} appended tokens")
    max_seq = (S0 + extra + 63) // 64 * 64
    Kx, Vx = W.make_kv(B, H, max(S0, 64), 27)
    oc = oracle.OracleCache(B, H, Hq, max_seq, 1e-2, 1e-2, buffer_tokens=window)
    gc = gpu.KVCompCache(B, H, Hq, max_seq, 1e-2, 1e-2, buffer_tokens=window)
    oc.build_codebook(Kx, Vx)
    gc.build_codebook(_dev(Kx), _dev(Vx))
    oc.compress_blocks(Kx[:, :S0], Vx[:, :S0])
    gc.compress_blocks(_dev(Kx[:, :S0]), _dev(Vx[:, :S0]))
    _assert_same_cache(oc, gc)
    kn, vn = W.make_new_tokens(B, H, extra, 27)
    qs = W.make_queries(B, Hq, extra, 27)
    dkn, dvn, dq = _dev(kn), _dev(vn), _dev(qs)
    worst = 0.0
    for t in range(extra):
        oc.append_token(kn[t], vn[t])
        gc.append_token(dkn[t], dvn[t])
        if t % 23 == 0 or oc.n_res in (window - 64, window - 1) or t == extra - 1:   # before and after every flush
            worst = max(worst, _attn_close(gc.attn_decode(dq[t], SCALE).cpu().numpy(), oc.attn_decode(qs[t], SCALE)))
    tokens = S0 + extra
    assert oc.n_blocks * 64 + oc.n_res == tokens
    _assert_same_cache(oc, gc)
    for which in (K, V):
        got = gc.decompress(which, tokens).cpu().numpy()
        np.testing.assert_array_equal(got.view(np.uint16), oc.decompress(which).view(np.uint16))
    _say(f"  blocks {oc.n_blocks}, buffered {oc.n_res}, worst attention error {worst:.2e}")
    gc.close()
    for bad in (100, 32, 8192):
        with pytest.raises(gpu.KvcompError):
            gpu.KVCompCache(B, H, Hq, max_seq, 1e-2, 1e-2, buffer_tokens=bad)


@pytest.mark.parametrize("B,H,Hq,window,S0,extra", [(2, 2, 2, 64, 100, 150), (1, 2, 8, 128, 70, 200),
                                                    (1, 1, 4, 192, 30, 260)])
def test_append_fused_into_the_attention_launch(gpu, oracle, B, H, Hq, window, S0, extra):
    """kvcomp_append_attn_decode = append_token then attn_decode: every step's output against the oracle's two calls,
    and the cache afterwards (buffer contents included: the kernel stores the token it read from the caller's tensor)
    bit for bit, across flushes and ring wrap-arounds; interleaved with the two separate calls."""
    _say(f"append fused into attention: B={B} H={H} Hq={Hq} buffer {window}, prompt {S0} + {extra} tokens")
    max_seq = (S0 + extra + 63) // 64 * 64
    Kx, Vx = W.make_kv(B, H, max(S0, 64), 28)
    oc = oracle.OracleCache(B, H, Hq, max_seq, 1e-2, 1e-2, buffer_tokens=window)
    gc = gpu.KVCompCache(B, H, Hq, max_seq, 1e-2, 1e-2, buffer_tokens=window)
    oc.build_codebook(Kx, Vx)
    gc.build_codebook(_dev(Kx), _dev(Vx))
    oc.compress_blocks(Kx[:, :S0], Vx[:, :S0])
    gc.compress_blocks(_dev(Kx[:, :S0]), _dev(Vx[:, :S0]))
    kn, vn = W.make_new_tokens(B, H, extra, 28)
    qs = W.make_queries(B, Hq, extra, 28)
    dkn, dvn, dq = _dev(kn), _dev(vn), _dev(qs)
    worst = 0.0
    for t in range(extra):
        oc.append_token(kn[t], vn[t])
        if t % 11 == 5:   # the two separate calls in between
            gc.append_token(dkn[t], dvn[t])
            out = gc.attn_decode(dq[t], SCALE)
        else:
            out = gc.append_attn_decode(dkn[t], dvn[t], dq[t], SCALE)
        if t % 3 == 0 or oc.n_res in (window - 64, window - 63, window - 1):
            worst = max(worst, _attn_close(out.cpu().numpy(), oc.attn_decode(qs[t], SCALE)))
        if t in (0, 17, extra // 2):
            _assert_same_cache(oc, gc)
    _assert_same_cache(oc, gc)
    _say(f"  blocks {oc.n_blocks}, buffered {oc.n_res}, worst attention error {worst:.2e}")
    for _ in range(max_seq - S0 - extra):
        gc.append_attn_decode(dkn[0], dvn[0], dq[0], SCALE)
    with pytest.raises(gpu.KvcompError) as e:
        gc.append_attn_decode(dkn[0], dvn[0], dq[0], SCALE)
    assert e.value.status == gpu.ERR_CAPACITY
    gc.close()


def test_many_sequence_splits(gpu, oracle):
    """One long sequence with a single KV head: the library splits it 128 ways (its maximum) so that the chip is
    filled; every split count gives the oracle's result, also when the last split is short or the buffer holds
    more 16-token units than there are splits."""
    _say("one head, 20000 tokens: 128 splits (automatic), then 97, 5 and 1")
    B, H, Hq, S = 1, 1, 2, 20000
    Kx, Vx = W.make_kv(B, H, S, 29)
    oc = oracle.OracleCache(B, H, Hq, S + 64, 1e-2, 1e-2, 0, 7, buffer_tokens=256)
    gc = gpu.KVCompCache(B, H, Hq, S + 64, 1e-2, 1e-2, max_code_len=7, buffer_tokens=256)
    oc.build_codebook(Kx, Vx)
    oc.compress_blocks(Kx, Vx)
    gc.build_codebook(_dev(Kx), _dev(Vx))
    gc.compress_blocks(_dev(Kx), _dev(Vx))
    assert oc.n_blocks == 309 and oc.n_res == 224
    q = W.make_queries(B, Hq, 1, 29)[0]
    ref = oc.attn_decode(q, SCALE)
    for n_splits in (0, 97, 5, 1):
        gc.set_tuning(n_splits=n_splits)
        err = _attn_close(gc.attn_decode(_dev(q), SCALE).cpu().numpy(), ref)
        _say(f"  n_splits {n_splits}: max abs err {err:.2e}")
    gc.close()


def _random_cases(n):
    rng = np.random.default_rng(2024)
    cases = []
    for i in range(n):
        H = int(rng.choice([1, 2, 3]))
        G = int(rng.choice([1, 2, 4, 8]))
        rel_k, rel_v = (float(x) for x in rng.choice([4e-3, 1e-2, 2e-2, 5e-2, 0.1], 2))
        levels = int(np.rint(1.0 / (2.0 * np.float32(min(rel_k, rel_v))))) + 1
        lo = int(np.ceil(np.log2(levels)))
        cases.append((int(rng.choice([1, 2])), H, H * G, int(rng.integers(64, 700)), rel_k, rel_v,
                      int(rng.choice([0, 1])), int(rng.integers(lo, 13)), int(rng.choice([64, 64, 128, 256])),
                      int(rng.integers(0, 150)), 100 + i))
    return cases


@pytest.mark.parametrize("B,H,Hq,S,rel_k,rel_v,k_mode,max_len,window,extra,seed", _random_cases(12))
def test_random_small_configs(gpu, oracle, B, H, Hq, S, rel_k, rel_v, k_mode, max_len, window, extra, seed):
    """Seeded random combinations of batch, heads, group size, length, error bounds, K unit, code word limit, buffer
    size and appended tokens: whole cache and decompressed tensors bit for bit, attention within tolerance."""
    _say(f"random case: B={B} H={H} Hq={Hq} S={S} rel {rel_k}/{rel_v} k_mode={k_mode} limit {max_len} "
         f"buffer {window} +{extra} tokens")
    max_seq = (S + extra + 63) // 64 * 64
    Kx, Vx = W.make_kv(B, H, S, seed)
    oc = oracle.OracleCache(B, H, Hq, max_seq, rel_k, rel_v, k_mode, max_len, buffer_tokens=window)
    gc = gpu.KVCompCache(B, H, Hq, max_seq, rel_k, rel_v, k_mode=k_mode, max_code_len=max_len, buffer_tokens=window)
    oc.build_codebook(Kx, Vx)
    gc.build_codebook(_dev(Kx), _dev(Vx))
    oc.compress_blocks(Kx, Vx)
    gc.compress_blocks(_dev(Kx), _dev(Vx))
    kn, vn = W.make_new_tokens(B, H, max(extra, 1), seed)
    qs = W.make_queries(B, Hq, max(extra, 1), seed)
    for t in range(extra):
        oc.append_token(kn[t], vn[t])
        if t % 5 == 4:
            gc.append_token(_dev(kn[t]), _dev(vn[t]))
        else:
            out = gc.append_attn_decode(_dev(kn[t]), _dev(vn[t]), _dev(qs[t]), SCALE)
            if t % 16 == 0:
                _attn_close(out.cpu().numpy(), oc.attn_decode(qs[t], SCALE))
    _assert_same_cache(oc, gc)
    _attn_close(gc.attn_decode(_dev(qs[0]), SCALE).cpu().numpy(), oc.attn_decode(qs[0], SCALE))
    tokens = S + extra
    for which in (K, V):
        got = gc.decompress(which, tokens).cpu().numpy()
        np.testing.assert_array_equal(got.view(np.uint16), oc.decompress(which).view(np.uint16))
    gc.close()


def test_decode_loop_in_a_hip_graph(gpu, oracle):
    """The decode loop (append + attention per step, one flush inside) captured in a HIP graph, as bench.py times it:
    every replay -- with an eager reset and prefill of the cache in between -- must give the eager loop's outputs bit
    for bit; the last step is also checked against the oracle."""
    import torch
    _say("decode loop of 20 steps in a HIP graph, three replays")
    B, H, Hq, S0, T = 2, 2, 4, 180, 20      # 180 = 2 blocks + 52 buffered: the 12th append completes a block
    Kx, Vx, oc, gc = _both(gpu, oracle, B, H, Hq, S0, S0, 256, 1e-2, 1e-2, 33)
    kn, vn = W.make_new_tokens(B, H, T, 33)
    qs = W.make_queries(B, Hq, T, 33)
    dK, dV, dkn, dvn, dq = _dev(Kx[:, :S0]), _dev(Vx[:, :S0]), _dev(kn), _dev(vn), _dev(qs)
    outs = torch.empty((T, B, Hq, 128), dtype=torch.float32, device="cuda:0")

    def loop():
        for t in range(T):
            gc.append_attn_decode(dkn[t], dvn[t], dq[t], SCALE, outs[t])

    def prefill():
        gc.reset(keep_codebook=True)
        gc.compress_blocks(dK, dV)

    loop()
    torch.cuda.synchronize()
    eager = outs.cpu().numpy().copy()
    for t in range(T):
        oc.append_token(kn[t], vn[t])
    _attn_close(eager[T - 1], oc.attn_decode(qs[T - 1], SCALE))
    _assert_same_cache(oc, gc)
    prefill()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        loop()
    for replay in range(3):
        prefill()                      # eager work and a synchronisation between the replays
        outs.zero_()
        graph.replay()
        torch.cuda.synchronize()
        np.testing.assert_array_equal(outs.cpu().numpy(), eager, err_msg=f"replay {replay}")
    # a replay runs the device work only: the context's host-side counters are where the last eager call left them
    # (the prefill), so the cache is brought back to a consistent state eagerly before it is used again
    prefill()
    loop()
    torch.cuda.synchronize()
    np.testing.assert_array_equal(outs.cpu().numpy(), eager)
    _assert_same_cache(oc, gc)
    gc.close()


def test_on_a_side_stream(gpu, oracle):
    """Every call takes the caller's stream: the whole path on a non-default stream (default priority), with the
    default stream kept busy by unrelated work, gives the same cache and attention."""
    import torch
    _say("the path on a side stream")
    B, H, Hq, S = 1, 2, 4, 300
    Kx, Vx = W.make_kv(B, H, S, 34)
    oc = oracle.OracleCache(B, H, Hq, 384, 1e-2, 1e-2)
    oc.build_codebook(Kx, Vx)
    oc.compress_blocks(Kx, Vx)
    kn, vn = W.make_new_tokens(B, H, 30, 34)
    q = W.make_queries(B, Hq, 1, 34)[0]
    for t in range(30):
        oc.append_token(kn[t], vn[t])
    dK, dV, dkn, dvn, dq = _dev(Kx), _dev(Vx), _dev(kn), _dev(vn), _dev(q)
    busy = torch.empty(64 << 20, dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        gc = gpu.KVCompCache(B, H, Hq, 384, 1e-2, 1e-2)
        gc.build_codebook(dK, dV)
        torch.cuda.default_stream().wait_stream(side)   # unrelated work on the default stream, ordered after this point
        with torch.cuda.stream(torch.cuda.default_stream()):
            for _ in range(4):
                busy.fill_(1)
        gc.compress_blocks(dK, dV)
        for t in range(30):
            if t % 2:
                gc.append_token(dkn[t], dvn[t])
            else:
                gc.append_attn_decode(dkn[t], dvn[t], dq, SCALE)
        out = gc.attn_decode(dq, SCALE)
        side.synchronize()
        _assert_same_cache(oc, gc)
        _attn_close(out.cpu().numpy(), oc.attn_decode(q, SCALE))
        gc.close()


@pytest.mark.parametrize("Hq,scale", [(2, 4.0), (8, 4.0), (2, 1e-4), (16, 30.0)])
def test_sharp_and_flat_softmax(gpu, oracle, Hq, scale):
    """Softmax scales far from 1/sqrt(128): with a large scale one token takes nearly all the weight (scores of the
    order of +-10^3, partial maxima that differ by hundreds between waves and splits), with a tiny one the weights
    are uniform.  Buffered tokens take part, so the sharpest token may sit in the fp16 buffer."""
    _say(f"softmax scale {scale}, Hq={Hq}")
    B, H, S = 1, 2, 1500
    Kx, Vx = W.make_kv(B, H, S, 35)
    oc = oracle.OracleCache(B, H, Hq, 1536, 1e-2, 1e-2, 0, 7, buffer_tokens=128)
    gc = gpu.KVCompCache(B, H, Hq, 1536, 1e-2, 1e-2, max_code_len=7, buffer_tokens=128)
    oc.build_codebook(Kx, Vx)
    oc.compress_blocks(Kx, Vx)
    gc.build_codebook(_dev(Kx), _dev(Vx))
    gc.compress_blocks(_dev(Kx), _dev(Vx))
    q = W.make_queries(B, Hq, 1, 35)[0]
    for n_splits in (0, 1, 7):
        gc.set_tuning(n_splits=n_splits)
        err = _attn_close(gc.attn_decode(_dev(q), scale).cpu().numpy(), oc.attn_decode(q, scale))
    _say(f"  max abs err {err:.2e}")
    gc.close()


@pytest.mark.parametrize("G,limit", [(4, 6), (8, 6), (8, 7), (2, 6)])
def test_heads_of_a_group_with_different_sharpness(gpu, oracle, G, limit):
    """The query heads that share a KV head differ by orders of magnitude in how sharp their softmax is, and K grows
    along the sequence so that the largest score of nearly every block exceeds the one before: the running softmax
    reference of the group path (which moves lazily, and whose integer weights share one scale per block across the
    heads) must not cost the other heads their resolution beyond what 22-bit weights under a 30000-fold spread of |q|
    leave: half of the 1e-3 bar (measured 2.7e-4 for groups of 4 and 8, 5e-6 for the per-head path of groups of 2)."""
    _say(f"heads of different sharpness, G={G}, code words <= {limit} bits")
    B, H, S = 1, 2, 64 * 40
    Hq = H * G
    Kx, Vx = W.make_kv(B, H, S, 71)
    ramp = np.linspace(0.25, 2.0, S, dtype=np.float32)[None, :, None, None]
    Kx = (Kx.astype(np.float32) * ramp).astype(np.float16)
    q = W.make_queries(B, Hq, 1, 71)[0].astype(np.float32)
    sharp = np.array([30.0, 0.01, 1.0, 8.0, 0.1, 3.0, 0.001, 15.0], np.float32)[:G]
    q = (q.reshape(B, H, G, 128) * sharp[None, None, :, None]).reshape(B, Hq, 128).astype(np.float16)
    oc = oracle.OracleCache(B, H, Hq, S + 64, 1e-2, 1e-2, 0, limit)
    gc = gpu.KVCompCache(B, H, Hq, S + 64, 1e-2, 1e-2, max_code_len=limit)
    oc.build_codebook(Kx, Vx)
    oc.compress_blocks(Kx, Vx)
    gc.prefill(_dev(Kx), _dev(Vx))
    ref = np.asarray(oc.attn_decode(q, SCALE), np.float64)
    for n_splits in (0, 1, 5):
        gc.set_tuning(n_splits=n_splits)
        out = gc.attn_decode(_dev(q), SCALE).cpu().numpy()
        err = np.abs(out - ref).max()
        assert err <= 5e-4 * max(1.0, np.abs(ref).max()), (n_splits, err)
    _say(f"  max abs err {err:.2e}")
    gc.close()


def test_layers_have_their_own_codebooks(gpu, oracle):
    """One context per layer in a single allocation (Section 3: codebooks are per layer): every layer matches an oracle
    cache of its own data, appends to one layer leave the others untouched, and the codebooks differ between layers
    whose value distributions differ."""
    _say("three layers in one arena, different data and error bounds per call order")
    B, H, Hq, S = 1, 2, 4, 200
    layers = gpu.KVCompLayers(3, B, H, Hq, 320, 1e-2, 2e-2, buffer_tokens=128)
    assert len(layers) == 3
    data, ocs = [], []
    for i in range(3):
        Kx, Vx = W.make_kv(B, H, S, 70 + i)
        if i == 1:   # a layer with a narrow bell inside each unit's range: a different histogram, hence codebook
            Kx = (Kx.astype(np.float32) ** 3 / 64).astype(np.float16)
            Vx = (Vx.astype(np.float32) ** 3 / 64).astype(np.float16)
        data.append((Kx, Vx))
        oc = oracle.OracleCache(B, H, Hq, 320, 1e-2, 2e-2, buffer_tokens=128)
        oc.build_codebook(Kx, Vx)
        oc.compress_blocks(Kx, Vx)
        ocs.append(oc)
    for i in (2, 0, 1):   # any order
        layers[i].build_codebook(_dev(data[i][0]), _dev(data[i][1]))
        layers[i].compress_blocks(_dev(data[i][0]), _dev(data[i][1]))
    kn, vn = W.make_new_tokens(B, H, 70, 70)
    for t in range(70):   # layer 1 grows by 70 tokens (one more block), the others stay
        ocs[1].append_token(kn[t], vn[t])
        layers[1].append_token(_dev(kn[t]), _dev(vn[t]))
    q = W.make_queries(B, Hq, 1, 70)[0]
    for i in range(3):
        _assert_same_cache(ocs[i], layers[i])
        for w in (K, V):
            ln, cd = layers[i].codebook(w)
            np.testing.assert_array_equal(ln, ocs[i].len[w])
            np.testing.assert_array_equal(cd, ocs[i].code[w])
        _attn_close(layers[i].attn_decode(_dev(q), SCALE).cpu().numpy(), ocs[i].attn_decode(q, SCALE))
    assert not np.array_equal(layers[0].codebook(K)[0], layers[1].codebook(K)[0])
    tot = layers.stats()
    assert tot["stored_bytes"] == sum(oc.stats()["stored_bytes"] for oc in ocs)
    assert abs(tot["compression_ratio"] - sum(oc.stats()["raw_bytes"] for oc in ocs) / tot["stored_bytes"]) < 1e-12
    layers.close()


def test_error_paths(gpu):
    import torch
    _say("error paths (all detected on the host or by the kernels' own checks)")
    B, H, S = 1, 2, 128
    Kx, Vx = W.make_kv(B, H, S, 26)
    gc = gpu.KVCompCache(B, H, H, S, 1e-2, 1e-2)
    dK, dV = _dev(Kx), _dev(Vx)
    with pytest.raises(gpu.KvcompError) as e:
        gc.compress_blocks(dK, dV)
    assert e.value.status == gpu.ERR_STATE
    with pytest.raises(gpu.KvcompError) as e:
        gc.attn_decode(_dev(W.make_queries(B, H, 1, 26)[0]), SCALE)
    assert e.value.status == gpu.ERR_STATE
    with pytest.raises(gpu.KvcompError) as e:
        gc.build_codebook(dK[:, :32].contiguous(), dV[:, :32].contiguous())
    assert e.value.status == gpu.ERR_INVALID_ARG
    bad = Kx.copy()
    bad[0, 5, 1, 7] = np.inf
    with pytest.raises(gpu.KvcompError) as e:
        gc.build_codebook(_dev(bad), dV)
    assert e.value.status == gpu.ERR_NONFINITE
    gc.build_codebook(dK, dV)
    big = torch.zeros((B, S + 64, H, 128), dtype=torch.float16, device="cuda:0")
    with pytest.raises(gpu.KvcompError) as e:
        gc.compress_blocks(big, big)
    assert e.value.status == gpu.ERR_CAPACITY
    gc.compress_blocks(dK, dV)
    with pytest.raises(gpu.KvcompError) as e:
        gc.compress_blocks(dK, dV)
    assert e.value.status == gpu.ERR_STATE
    with pytest.raises(gpu.KvcompError) as e:
        gc.append_token(dK[:, 0].contiguous(), dV[:, 0].contiguous())
    assert e.value.status == gpu.ERR_CAPACITY
    with pytest.raises(gpu.KvcompError) as e:   # new codebooks under existing records would invalidate them
        gc.build_codebook(dK, dV)
    assert e.value.status == gpu.ERR_STATE
    gc.reset(keep_codebook=False)
    gc.build_codebook(dK, dV)
    with pytest.raises(gpu.KvcompError):
        gpu.KVCompCache(1, 2, 6, 128, 1e-2, 1e-2)
    gc.close()


def test_nonfinite_token_is_reported_after_its_flush(gpu):
    """An Inf in an appended token: the appends never synchronise, so the flag that the flush's size pass sets is
    reported by the next synchronising call (statistics, decompression), once, and the cache stays usable."""
    _say("Inf in an appended token, reported at the next synchronising call")
    B, H, S = 1, 2, 100
    Kx, Vx = W.make_kv(B, H, S, 36)
    gc = gpu.KVCompCache(B, H, H, 256, 1e-2, 1e-2)
    gc.build_codebook(_dev(Kx), _dev(Vx))
    gc.compress_blocks(_dev(Kx), _dev(Vx))
    kn, vn = W.make_new_tokens(B, H, 40, 36)
    kn[5, 0, 1, 17] = np.inf
    for t in range(27):           # 100 = one block + 36 buffered: the 28th append completes the second block
        gc.append_token(_dev(kn[t]), _dev(vn[t]))
    assert gc.stats()["n_blocks"] == 1     # still buffered: nothing has looked at the token yet
    gc.append_token(_dev(kn[27]), _dev(vn[27]))
    with pytest.raises(gpu.KvcompError) as e:
        gc.stats()
    assert e.value.status == gpu.ERR_NONFINITE
    assert gc.stats()["n_blocks"] == 2     # reported once; the cache goes on
    vn[30, 0, 0, 3] = np.nan
    for t in range(28, 40):
        gc.append_token(_dev(kn[t]), _dev(vn[t]))
    gc.stats()                             # the NaN is still in the fp16 buffer
    for t in range(52):
        gc.append_token(_dev(kn[t % 20 + 6]), _dev(vn[t % 20 + 6]))   # rows without Inf/NaN; flushes the NaN's block
    with pytest.raises(gpu.KvcompError) as e:
        gc.decompress(V, 256)
    assert e.value.status == gpu.ERR_NONFINITE
    gc.close()


def test_flush_replayed_past_the_arena_is_refused(gpu):
    """The interface forbids replaying a captured flush without the eager calls in between: every replay advances the
    arena tail on the device.  The placement kernel bounds it: once the records would run past the arena it writes
    nothing, the next synchronising call reports KVCOMP_ERR_CAPACITY, and after a reset the context works again."""
    import torch
    _say("captured flush replayed until the arena is full")
    B, H, S = 1, 1, 64
    Kx, Vx = W.make_kv(B, H, 128, 37)
    gc = gpu.KVCompCache(B, H, H, 128, 1e-2, 1e-2)
    dK, dV = _dev(Kx), _dev(Vx)
    gc.build_codebook(dK, dV)
    gc.compress_blocks(dK[:, :S].contiguous(), dV[:, :S].contiguous())
    kn, vn = W.make_new_tokens(B, H, 64, 37)
    dkn, dvn = _dev(kn), _dev(vn)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for t in range(64):
            gc.append_token(dkn[t], dvn[t])      # the 64th append compresses the block
    # the arena holds two blocks at the worst case of 12 bits per symbol (about 52 KiB); a replay adds about 12 KiB
    for _ in range(12):
        graph.replay()
    torch.cuda.synchronize()
    with pytest.raises(gpu.KvcompError) as e:
        gc.stats()
    assert e.value.status == gpu.ERR_CAPACITY
    gc.reset(keep_codebook=True)
    gc.compress_blocks(dK, dV)
    assert gc.stats()["n_blocks"] == 2
    gc.close()


@pytest.mark.parametrize("B,H,Hq,S", [(1, 2, 2, 1000), (2, 2, 8, 300), (1, 1, 8, 64), (1, 4, 8, 4100)])
def test_fp16_baseline_attention(gpu, oracle, B, H, Hq, S):
    """The uncompressed comparison kernel (Section 4.3) against the oracle's attention on the raw fp16 values
    (K' = K, V' = V), to the same bar as the fused kernel; and against an oracle cache whose buffer holds the whole
    sequence, so that nothing is quantized and the oracle's own decode-attention call is the reference."""
    _say(f"fp16 baseline attention B={B} H={H} Hq={Hq} S={S}")
    Kx, Vx = W.make_kv(B, H, S, 27)
    q = W.make_queries(B, Hq, 1, 27)[0]
    G = Hq // H
    ref = np.zeros((B, Hq, 128))
    for b in range(B):
        for hq in range(Hq):
            ref[b, hq] = oracle.attention_head(Kx[b, :, hq // G], Vx[b, :, hq // G], q[b, hq], SCALE)
    if S < 4096:   # the largest buffer the oracle cache takes is 4096 tokens
        window = (S + 64) // 64 * 64
        oc = oracle.OracleCache(B, H, Hq, window, 1e-2, 1e-2, buffer_tokens=window)
        oc.build_codebook(Kx[:, :64] if S >= 64 else np.zeros((B, 64, H, 128), np.float16), Vx[:, :64] if S >= 64
                          else np.zeros((B, 64, H, 128), np.float16))
        oc.compress_blocks(Kx, Vx)
        assert oc.n_blocks == 0 and oc.n_res == S
        np.testing.assert_allclose(oc.attn_decode(q, SCALE), ref, rtol=0, atol=1e-12)
    base = gpu.BaselineFp16Attention(B, H, Hq)
    for n_splits in (0, 1, 5):
        out = base(_dev(Kx), _dev(Vx), _dev(q), SCALE, n_splits=n_splits).cpu().numpy()
        _attn_close(out, ref)


def test_config1_full_size_sampled(gpu, oracle):
    """The benchmark workload (32 heads x 4096 tokens) in the launch configuration bench.py times."""
    w = W.CONFIGS["c1"]
    _say("config 1 full size: records sampled, attention on every head")
    Kx, Vx, oc, gc = _both(gpu, oracle, w.batch, w.n_kv_heads, w.n_q_heads, w.seq, w.seq, w.seq, w.rel_eb, w.rel_eb, w.seed,
                           limit=W.CODE_LEN_LIMIT[w.rel_eb])
    _assert_same_cache(oc, gc, sample=200)
    qs = W.make_queries(w.batch, w.n_q_heads, 2, w.seed)
    for i in range(2):
        err = _attn_close(gc.attn_decode(_dev(qs[i]), SCALE).cpu().numpy(), oc.attn_decode(qs[i], SCALE))
        _say(f"  step {i}: max abs err {err:.3e}")
    _say(f"  stats {gc.stats()}")
    gc.close()


@pytest.mark.parametrize("max_len,rel,Hq", [(6, 1e-2, 4), (7, 1e-2, 4), (7, 5e-3, 4), (8, 5e-3, 4), (10, 1e-2, 4),
                                            (12, 1e-2, 4), (6, 1e-2, 2), (5, 2e-2, 2), (5, 2e-2, 4), (6, 1e-2, 8),
                                            (6, 1e-2, 16), (8, 5e-3, 8), (10, 1e-2, 8), (12, 1e-2, 16), (8, 5e-3, 16),
                                            (10, 5e-3, 16)])
def test_code_length_limits_select_every_decoder_variant(gpu, oracle, max_len, rel, Hq):
    """Shorter maximum code words: more symbols per decode window (5, 4, 3, 3, 2 for limits up to 6, 7, 8, 10, 12;
    for every size of query-head group)."""
    _say(f"max_code_len={max_len} rel={rel} Hq={Hq}")
    B, H, S = 1, 2, 330
    Kx, Vx = W.make_kv(B, H, S, 31)
    oc = oracle.OracleCache(B, H, Hq, S + 64, rel, rel, max_code_len=max_len)
    oc.build_codebook(Kx, Vx)
    oc.compress_blocks(Kx, Vx)
    gc = gpu.KVCompCache(B, H, Hq, S + 64, rel, rel, max_code_len=max_len)
    gc.build_codebook(_dev(Kx), _dev(Vx))
    gc.compress_blocks(_dev(Kx), _dev(Vx))
    for which in (K, V):
        ln_g, cd_g = gc.codebook(which)
        np.testing.assert_array_equal(ln_g, oc.len[which])
        np.testing.assert_array_equal(cd_g, oc.code[which])
        assert int(ln_g.max()) <= max_len
    _assert_same_cache(oc, gc)
    q = W.make_queries(B, Hq, 1, 31)[0]
    _attn_close(gc.attn_decode(_dev(q), SCALE).cpu().numpy(), oc.attn_decode(q, SCALE))
    gc.close()


@pytest.mark.parametrize("G", [1, 4, 8])
def test_long_code_words_and_length_limit(gpu, oracle, G):
    """A geometric code histogram at prefill drives the code words to the 12-bit limit (count halving on both sides);
    the later blocks then use every level, so records are large (above the 8 KiB that the first stage of the record
    staging moves) and the two-symbols-per-window decoder runs, for one query head per KV head and for groups."""
    _say(f"geometric prefill histogram -> 12-bit code words, {G} query heads per KV head")
    B, H, S = 1, 2, 256
    rng = np.random.default_rng(32)
    Kx, Vx = W.make_kv(B, H, S, 32)
    geo = np.minimum(rng.geometric(0.5, size=(B, 64, H, 128)) - 1, 50)   # code k with probability 2^-(k+1)
    kp = geo.astype(np.float16)
    kp[:, 0], kp[:, 1] = 0, 50          # every K unit (channel over the block's tokens) spans [0, 50] -> code == value
    vp = geo.astype(np.float16)
    vp[..., 0], vp[..., 1] = 0, 50      # every V unit (token over the channels) spans [0, 50]
    Kx[:, :64], Vx[:, :64] = kp, vp
    oc = oracle.OracleCache(B, H, G * H, S, 1e-2, 1e-2)
    oc.build_codebook(Kx[:, :64], Vx[:, :64])
    assert oc.halvings[K] > 0 and int(oc.len[K].max()) == 12 and int(oc.len[V].max()) == 12
    oc.compress_blocks(Kx, Vx)
    gc = gpu.KVCompCache(B, H, G * H, S, 1e-2, 1e-2)
    gc.build_codebook(_dev(Kx[:, :64]), _dev(Vx[:, :64]))
    gc.compress_blocks(_dev(Kx), _dev(Vx))
    for which in (K, V):
        ln_g, cd_g = gc.codebook(which)
        np.testing.assert_array_equal(ln_g, oc.len[which])
        np.testing.assert_array_equal(cd_g, oc.code[which])
    _assert_same_cache(oc, gc)
    q = W.make_queries(B, G * H, 1, 32)[0]
    _attn_close(gc.attn_decode(_dev(q), SCALE).cpu().numpy(), oc.attn_decode(q, SCALE))
    _say(f"  largest record {gc.stats()['max_record_bytes']} B, CR {gc.stats()['compression_ratio']:.3f}")
    gc.close()


@pytest.mark.parametrize("H,Hq", [(2, 2), (1, 4), (1, 8)])
@pytest.mark.parametrize("k_scale,q_scale,v_scale", [(256.0, 1.0 / 256.0, 64.0), (1.0 / 64.0, 64.0, 1.0 / 32.0)])
def test_attention_with_large_and_small_magnitudes(gpu, oracle, H, Hq, k_scale, q_scale, v_scale):
    """K, q and V scaled by powers of two: the scores do not change, the folded weights (q step, p step) move by
    several binades (the query-group path keeps them as scaled fp16 pairs)."""
    _say(f"scaled inputs H={H} Hq={Hq} k x{k_scale} q x{q_scale} v x{v_scale}")
    B, S = 1, 777
    Kx, Vx = W.make_kv(B, H, S, 41)
    Kx = (Kx.astype(np.float32) * k_scale).astype(np.float16)
    Vx = (Vx.astype(np.float32) * v_scale).astype(np.float16)
    q = (W.make_queries(B, Hq, 1, 41)[0].astype(np.float32) * q_scale).astype(np.float16)
    assert np.isfinite(Kx.astype(np.float32)).all() and np.isfinite(Vx.astype(np.float32)).all()
    oc = oracle.OracleCache(B, H, Hq, 1024, 1e-2, 1e-2, 0, 7)
    oc.build_codebook(Kx, Vx)
    oc.compress_blocks(Kx, Vx)
    gc = gpu.KVCompCache(B, H, Hq, 1024, 1e-2, 1e-2, max_code_len=7)
    gc.build_codebook(_dev(Kx), _dev(Vx))
    gc.compress_blocks(_dev(Kx), _dev(Vx))
    _assert_same_cache(oc, gc)
    err = _attn_close(gc.attn_decode(_dev(q), SCALE).cpu().numpy(), oc.attn_decode(q, SCALE))
    _say(f"  max abs err {err:.3e}")
    gc.close()


@pytest.mark.parametrize("H,Hq,max_len", [(2, 2, 12), (1, 4, 9), (1, 8, 7)])
def test_block_quant_k(gpu, oracle, H, Hq, max_len):
    """K with one quantization range per 2D block (BlockQuant, Section 4.2): codes, range, codebook, records (their
    header holds one {min,max} pair), attention, and the append path with a flush."""
    _say(f"BlockQuant K: H={H} Hq={Hq} max code word {max_len}")
    B, S, rel = 2, 200, 1e-2
    Kx, Vx = W.make_kv(B, H, S, 51)
    Kx[1, 64:128, 0, :] = np.float16(-2.5)  # a constant K block
    oc = oracle.OracleCache(B, H, Hq, 320, rel, rel, 1, max_len)
    gc = gpu.KVCompCache(B, H, Hq, 320, rel, rel, k_mode=1, max_code_len=max_len)
    oc.build_codebook(Kx, Vx)
    gc.build_codebook(_dev(Kx), _dev(Vx))
    codes_o, mm_o = oracle.tensor_quantize(K, Kx, rel, k_mode=1)
    codes_g, mm_g = gc.debug_codes(K, _dev(Kx))
    assert mm_g.shape == mm_o.shape == (B * H * (S // 64), 1, 2)
    np.testing.assert_array_equal(mm_g, mm_o)
    np.testing.assert_array_equal(codes_g, codes_o)
    for which in (K, V):
        ln_g, cd_g = gc.codebook(which)
        np.testing.assert_array_equal(ln_g, oc.len[which])
        np.testing.assert_array_equal(cd_g, oc.code[which])
    oc.compress_blocks(Kx, Vx)
    gc.compress_blocks(_dev(Kx), _dev(Vx))
    _assert_same_cache(oc, gc)
    kn, vn = W.make_new_tokens(B, H, 70, 51)
    qs = W.make_queries(B, Hq, 70, 51)
    for t in range(70):
        oc.append_token(kn[t], vn[t])
        gc.append_token(_dev(kn[t]), _dev(vn[t]))
        if t in (0, 55, 56, 69):  # the flush happens at t = 55
            err = _attn_close(gc.attn_decode(_dev(qs[t]), SCALE).cpu().numpy(), oc.attn_decode(qs[t], SCALE))
            _say(f"  step {t}: max abs err {err:.3e}")
    _assert_same_cache(oc, gc)
    st = gc.stats()
    _say(f"  CR {st['compression_ratio']:.3f}, K bits/symbol {st['payload_bits_k'] / (B * H * oc.n_blocks * 8192.0):.2f}")
    gc.close()


@pytest.mark.parametrize("B,H,S,k_mode,max_len", [(2, 2, 200, 0, 7), (1, 3, 333, 1, 10), (1, 1, 64, 0, 12)])
def test_stand_alone_decompression(gpu, oracle, B, H, S, k_mode, max_len):
    """The decompressed cache (blocks reconstructed in fp16, then the buffered tokens) is bit-identical to the
    oracle's, and the fp16 attention kernel on it (the multi-kernel pipeline) agrees with the oracle's attention up
    to the fp16 rounding of the reconstructed values."""
    _say(f"decompress B={B} H={H} S={S} k_mode={k_mode} max code word {max_len}")
    Kx, Vx = W.make_kv(B, H, S, 61)
    oc = oracle.OracleCache(B, H, H, S + 64, 1e-2, 2e-2, k_mode, max_len)
    gc = gpu.KVCompCache(B, H, H, S + 64, 1e-2, 2e-2, k_mode=k_mode, max_code_len=max_len)
    oc.build_codebook(Kx, Vx)
    oc.compress_blocks(Kx, Vx)
    gc.build_codebook(_dev(Kx), _dev(Vx))
    gc.compress_blocks(_dev(Kx), _dev(Vx))
    kn, vn = W.make_new_tokens(B, H, 5, 61)
    for t in range(5):
        oc.append_token(kn[t], vn[t])
        gc.append_token(_dev(kn[t]), _dev(vn[t]))
    tokens = S + 5
    dec = {}
    for which in (K, V):
        ref = oc.decompress(which)
        got = gc.decompress(which, tokens)
        assert tuple(got.shape) == ref.shape == (B, tokens, H, 128)
        np.testing.assert_array_equal(got.cpu().numpy().view(np.uint16), ref.view(np.uint16))
        walked = gc.decompress(which, tokens, tree_walk=True)   # the bit-serial tree walk gives the same bits
        np.testing.assert_array_equal(walked.cpu().numpy().view(np.uint16), ref.view(np.uint16))
        dec[which] = got
    with pytest.raises(gpu.KvcompError) as e:
        gc.decompress(K, tokens - 1)
    assert e.value.status == gpu.ERR_CAPACITY
    q = W.make_queries(B, H, 1, 61)[0]
    out = gpu.BaselineFp16Attention(B, H, H)(dec[K], dec[V], _dev(q), SCALE).cpu().numpy()
    ref = np.asarray(oc.attn_decode(q, SCALE))
    assert np.abs(out - ref).max() <= 2e-3 * max(1.0, np.abs(ref).max())   # values rounded to fp16: 2^-11 relative each
    gc.close()


@pytest.mark.parametrize("name,rel", [("c2", 1e-2), ("c2", 5e-3), ("c2", 2e-2), ("c3", 1e-2), ("c4", 1e-2)])
def test_large_configs_full_size_sampled(gpu, oracle, name, rel):
    """The long-context (with its error-bound sweep), grouped-query and 70B-shaped workloads at their full prompt
    size, in the launch configuration bench.py times (automatic splits, the code word limit of workloads.CODE_LEN_LIMIT).  The oracle quantizes
    the whole tensors (the codebooks depend on all of it); records are compared on a sample of blocks and the
    attention output on five (batch, kv head) pairs -- the two ends and three from the middle of the range, so that
    every part of the kernel's workgroup numbering is covered -- which the oracle recomputes from its own compressed
    copy of those heads."""
    w = W.CONFIGS[name]
    assert rel in W.C2_REL_EB_SWEEP and (name == "c2" or rel == w.rel_eb)
    B, H, Hq, S = w.batch, w.n_kv_heads, w.n_q_heads, w.seq
    G = Hq // H
    limit = W.CODE_LEN_LIMIT[rel]
    _say(f"{name} full size: B={B} H={H} Hq={Hq} S={S} rel_eb={rel} code words <= {limit} bits")
    Kx, Vx = W.make_kv(B, H, S, w.seed)
    gc = gpu.KVCompCache(B, H, Hq, S + 64, rel, rel, max_code_len=limit)
    dK, dV = _dev(Kx), _dev(Vx)
    gc.build_codebook(dK, dV)
    gc.compress_blocks(dK, dV)
    # the same prompt through the one-pass entry point that bench.py times (sizes from block histograms, placement in
    # several chunks, K written before V is sized): must give the same cache
    gp = gpu.KVCompCache(B, H, Hq, S + 64, rel, rel, max_code_len=limit)
    gp.prefill(dK, dV)
    del dK, dV
    st_c, st_p = gc.stats(), gp.stats()
    for key in ("n_blocks", "n_res", "record_bytes_k", "record_bytes_v", "payload_bits_k", "payload_bits_v", "stored_bytes"):
        assert st_c[key] == st_p[key], key
    _say("  gpu compressed; oracle quantizes")
    NB = S // 64
    book, codes, mms = {}, {}, {}
    for which, X in ((K, Kx), (V, Vx)):
        codes[which], mms[which] = oracle.tensor_quantize(which, X, rel)
        hist = oracle.histogram(codes[which])
        np.testing.assert_array_equal(gc.histogram(which).astype(np.uint64), hist)
        ln, cd, _ = oracle.build_codebook(hist, oracle.n_sym(rel), limit)
        ln_g, cd_g = gc.codebook(which)
        np.testing.assert_array_equal(ln_g, ln)
        np.testing.assert_array_equal(cd_g, cd)
        book[which] = (ln, cd)
    # Placement at full size: the record size of EVERY block from the oracle's codes and code lengths (the sampled
    # records below pin this size against oracle.encode_block), offsets by a running sum in (tensor, batch, head,
    # block) order; the device's Block Offsets Array is compared on the sample and on the very last entry.
    hdr = {K: 4 * 128 + 2 * 128, V: 4 * 64 + 2 * 128}
    size16 = {}
    for which in (K, V):
        ln8 = book[which][0].astype(np.uint8)
        bits = ln8[codes[which].reshape(B * H * NB, -1)].sum(axis=1, dtype=np.int64)
        size16[which] = (hdr[which] + 4 * ((bits + 31) // 32) + 15) // 16
    off16 = np.concatenate([[0], np.cumsum(np.concatenate([size16[K], size16[V]]))])
    rng = np.random.default_rng(5)
    picks = [(int(rng.integers(2)), int(rng.integers(B)), int(rng.integers(H)), int(rng.integers(NB))) for _ in range(48)]
    picks += [(K, 0, 0, 0), (K, B - 1, H - 1, NB - 1), (V, 0, 0, 0), (V, B - 1, H - 1, NB - 1)]
    for which, b, h, j in picks:
        i = (b * H + h) * NB + j
        rec = oracle.encode_block(which, codes[which][i], mms[which][i], *book[which])
        assert (len(rec) + 15) // 16 == size16[which][i]
        want = (int(off16[which * B * H * NB + i]), int(size16[which][i]))
        assert gc.block_entry(which, b, h, j) == want, (which, b, h, j)
        assert gp.block_entry(which, b, h, j) == want, (which, b, h, j)
        for cache in (gc, gp):
            got = cache.get_block(which, b, h, j)
            assert len(got) == (len(rec) + 15) // 16 * 16
            np.testing.assert_array_equal(got[: len(rec)], rec)
            assert not got[len(rec):].any()
    gp.close()
    del codes, mms
    q = W.make_queries(B, Hq, 1, w.seed)[0]
    out = gc.attn_decode(_dev(q), SCALE).cpu().numpy()
    sampled = {}
    BH = B * H
    pairs = sorted({0, BH - 1, BH // 2, BH // 3 + 1, (5 * BH) // 8 + 2})
    for b, h in ((i // H, i % H) for i in pairs):
        oc = oracle.OracleCache(1, 1, G, S + 64 + w.append_steps, rel, rel, 0, limit)
        oc.len, oc.code = [book[K][0], book[V][0]], [book[K][1], book[V][1]]
        oc.compress_blocks(np.ascontiguousarray(Kx[b:b + 1, :, h:h + 1]), np.ascontiguousarray(Vx[b:b + 1, :, h:h + 1]))
        ref = oc.attn_decode(np.ascontiguousarray(q[b:b + 1, h * G:(h + 1) * G]), SCALE)
        err = _attn_close(out[b:b + 1, h * G:(h + 1) * G], ref)
        # well inside the 1e-3 bar: the kernels' own error is a few 1e-5 at most (integer weights of 22 bits, fp32
        # accumulation); a tenfold loss of weight resolution would still pass the bar on these inputs and is caught here
        assert err <= 2e-4 * max(1.0, float(np.abs(np.asarray(ref)).max())), err
        _say(f"  (b={b}, h={h}): attention max abs err {err:.3e}")
        sampled[(b, h)] = oc
    gc.close()
    if not w.append_steps:
        return
    # the streaming phase at full size: every decode step appends one token per sequence (a full buffer is compressed
    # with the prompt's codebooks) and attends; the sampled heads are followed by oracle caches of their own
    T = w.append_steps
    _say(f"  streaming: {T} decode steps")
    gc = gpu.KVCompCache(B, H, Hq, S + T, rel, rel, max_code_len=limit)
    dK, dV = _dev(Kx), _dev(Vx)
    gc.build_codebook(dK, dV)
    gc.compress_blocks(dK, dV)
    del dK, dV
    kn, vn = W.make_new_tokens(B, H, T, w.seed)
    qs = W.make_queries(B, Hq, T, w.seed)
    dkn, dvn, dq = _dev(kn), _dev(vn), _dev(qs)
    check = {0, 62, 63, 64, 255, 256, T - 1}
    outs = {}
    for t in range(T):
        o = gc.append_attn_decode(dkn[t], dvn[t], dq[t], SCALE)
        if t in check:
            outs[t] = o.cpu().numpy()
    st = gc.stats()
    assert st["n_blocks"] == (S + T) // 64 and st["n_res"] == (S + T) % 64
    for (b, h), oc in sampled.items():
        worst = 0.0
        for t in range(T):
            oc.append_token(kn[t][b:b + 1, h:h + 1], vn[t][b:b + 1, h:h + 1])
            if t in check:
                ref = oc.attn_decode(np.ascontiguousarray(qs[t][b:b + 1, h * G:(h + 1) * G]), SCALE)
                worst = max(worst, _attn_close(outs[t][b:b + 1, h * G:(h + 1) * G], ref))
                assert worst <= 2e-4 * max(1.0, float(np.abs(np.asarray(ref)).max())), worst
        for which in (K, V):
            for j in range(NB, oc.n_blocks):   # the blocks compressed while streaming
                np.testing.assert_array_equal(gc.get_block(which, b, h, j), oc.get_block(which, 0, 0, j))
        _say(f"  (b={b}, h={h}): {oc.n_blocks - NB} streamed blocks bit-exact, attention max abs err {worst:.3e}")
    gc.close()
