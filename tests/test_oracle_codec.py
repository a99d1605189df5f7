"""Pins for the oracle's block encoder and its two decoders (Section 3.2.2, Figure 4; Section 3.3.1).

Slices are written from both ends (two decodable chains per slice); with 1-bit code words the two directions
coincide, which the first test uses to expose the plain bit and slice order.

The record layout is checked against an independent bit packer (numpy.packbits, little bit order) on streams
whose bits are known by construction, against the closed-form sizes, and by lossless round trips through two
structurally different decoders (canonical bit-serial; the paper's array-tree walk).
"""
import numpy as np
import pytest

import workloads as W

K, V = 0, 1


def _hist(counts):
    h = np.zeros(256, np.uint64)
    h[: len(counts)] = counts
    return h


def _slice_order(which, codes):
    """Symbols in stream order, [128 slices][64 symbols]: K -> half token rows; V -> channel columns."""
    return codes.reshape(128, 64) if which == K else codes.reshape(64, 128).T


def _pack_reference(which, codes, ln, cd, hdr):
    """Independent encoder for tiny cases: code words as '0'/'1' strings -> numpy.packbits(bitorder='little')."""
    sl = _slice_order(which, codes)
    slice_bits, bits = [], []
    for s in range(sl.shape[0]):
        words = [format(int(cd[x]), "b").zfill(int(ln[x])) for x in sl[s]]
        # symbols 0..31 first-bit-first, symbols 32..63 last-bit-first (read downwards from the slice end they are
        # the code words of 63, 62, .., 32 first-bit-first)
        w = "".join(words[:32]) + "".join(x[::-1] for x in words[32:])
        slice_bits.append(len(w))
        bits.extend(int(ch) for ch in w)
    payload = np.packbits(np.array(bits, np.uint8), bitorder="little")
    words = (len(bits) + 31) // 32
    payload = np.concatenate([payload, np.zeros(words * 4 - len(payload), np.uint8)])
    total = hdr + len(payload)
    pad = (-total) % 16
    return np.array(slice_bits, np.uint16), np.concatenate([payload, np.zeros(pad, np.uint8)])


@pytest.mark.parametrize("which", [K, V])
def test_one_bit_codes_expose_bit_and_slice_order(oracle, which):
    # two levels -> code words '0' and '1': the payload is the code matrix itself, in stream order
    rng = np.random.default_rng(1)
    codes = rng.integers(0, 2, (64, 128)).astype(np.uint8)
    ln, cd, _ = oracle.build_codebook(_hist([5, 5]), 2, 12)
    assert list(ln[:2]) == [1, 1] and list(cd[:2]) == [0, 1]
    mm = np.arange(2 * oracle.n_units(which), dtype=np.uint16).reshape(-1, 2)
    rec = oracle.encode_block(which, codes, mm, ln, cd)
    hdr = oracle.header_bytes(which)
    assert hdr == (512 + 256 if which == K else 256 + 256)
    assert len(rec) == hdr + 1024 and len(rec) % 16 == 0
    expect = np.packbits(_slice_order(which, codes).reshape(-1), bitorder="little")
    np.testing.assert_array_equal(rec[hdr:], expect)
    # the first 32 symbols of slice 0 are the bits of little-endian word 0, least significant bit first
    w0 = int(rec[hdr:hdr + 4].view("<u4")[0])
    first = _slice_order(which, codes)[0, :32]
    assert [(w0 >> i) & 1 for i in range(32)] == list(first)
    # header: min/max pairs as little-endian binary16 patterns, then u16 bit counts
    np.testing.assert_array_equal(rec[: 4 * mm.shape[0]].view("<u2").reshape(-1, 2), mm)
    nsl = 128
    np.testing.assert_array_equal(rec[hdr - 2 * nsl:hdr].view("<u2"), np.full(nsl, 8192 // nsl, np.uint16))


@pytest.mark.parametrize("which", [K, V])
@pytest.mark.parametrize("nsym", [3, 26, 51, 101])
def test_record_matches_independent_packer(oracle, which, nsym):
    rng = np.random.default_rng(nsym)
    counts = (rng.integers(1, 60, nsym) ** 2)
    ln, cd, _ = oracle.build_codebook(_hist(counts), nsym, 12)
    p = counts / counts.sum()
    codes = rng.choice(nsym, size=(64, 128), p=p).astype(np.uint8)
    mm = rng.integers(0, 0x7bff, (oracle.n_units(which), 2)).astype(np.uint16)
    rec = oracle.encode_block(which, codes, mm, ln, cd)
    hdr = oracle.header_bytes(which)
    sb, payload = _pack_reference(which, codes, ln, cd, hdr)
    nsl = len(sb)
    np.testing.assert_array_equal(rec[hdr - 2 * nsl:hdr].view("<u2"), sb)
    np.testing.assert_array_equal(rec[hdr:], payload)
    # sizes: sum of slice bit counts == sum of code lengths; record = header + whole words, padded to 16 bytes
    total_bits = int(ln[codes].astype(np.int64).sum())
    assert int(sb.astype(np.int64).sum()) == total_bits
    assert len(rec) == -(-(hdr + 4 * -(-total_bits // 32)) // 16) * 16


@pytest.mark.parametrize("which", [K, V])
@pytest.mark.parametrize("k_mode", [0, 1])
def test_round_trip_through_both_decoders(oracle, which, k_mode):
    if which == V and k_mode == 1:
        pytest.skip("block mode exists for K only")
    rng = np.random.default_rng(17)
    for nsym, skew in ((2, 1), (5, 3), (51, 2), (101, 4), (256, 6)):
        counts = rng.integers(1, 50, nsym) ** skew
        ln, cd, _ = oracle.build_codebook(_hist(counts), nsym, 12)
        codes = rng.choice(nsym, size=(64, 128), p=counts / counts.sum()).astype(np.uint8)
        codes[0, :5] = nsym - 1
        mm = rng.integers(0, 0x7bff, (oracle.n_units(which, k_mode), 2)).astype(np.uint16)
        rec = oracle.encode_block(which, codes, mm, ln, cd, k_mode)
        ca, ma = oracle.decode_block_serial(which, rec, ln, k_mode)
        cb, mb = oracle.decode_block_tree(which, rec, ln, cd, k_mode)
        np.testing.assert_array_equal(ca, codes)
        np.testing.assert_array_equal(cb, codes)
        np.testing.assert_array_equal(ma, mm)
        np.testing.assert_array_equal(mb, mm)


def test_decoders_reject_a_wrong_slice_length(oracle):
    rng = np.random.default_rng(3)
    counts = rng.integers(1, 50, 51)
    ln, cd, _ = oracle.build_codebook(_hist(counts), 51, 12)
    codes = rng.integers(0, 51, (64, 128)).astype(np.uint8)
    mm = np.zeros((128, 2), np.uint16)
    rec = oracle.encode_block(K, codes, mm, ln, cd)
    bad = rec.copy()
    bad[512] ^= 1  # bit count of slice 0 (the K header is 512 bytes of min/max pairs, then the counts)
    with pytest.raises(ValueError):
        oracle.decode_block_serial(K, bad, ln)
    with pytest.raises(ValueError):
        oracle.decode_block_tree(K, bad, ln, cd)


def test_metadata_overhead_closed_form(oracle):
    # Section 3.2.2: one unsigned 16-bit bit count per encoded vector -> 16 / (vector_len * avg_bits) of the payload
    # (the paper's vector is head_dim symbols; here a K vector is half a token row, 64 symbols)
    Kx, Vx = W.make_kv(1, 2, 512, 5)
    oc = oracle.OracleCache(1, 2, 2, 512, 1e-2, 1e-2)
    oc.build_codebook(Kx, Vx)
    oc.compress_blocks(Kx, Vx)
    st = oc.stats()
    nblk = 2 * 8
    avg_bits_k = st["payload_bits_k"] / (nblk * 8192)
    slice_meta_k = nblk * 128 * 2
    assert abs(slice_meta_k / (st["payload_bits_k"] / 8) - 16 / (64 * avg_bits_k)) < 1e-12
    assert st["header_bytes"] == nblk * (768 + 512)
    assert st["raw_bytes"] == 2 * 2 * 512 * 128 * 2
    # record bytes = header + payload words (+ < 16 B pad) for every block
    assert 0 <= st["record_bytes_k"] - nblk * 768 - st["payload_bits_k"] / 8 < nblk * 20


def test_cache_layout_and_determinism(oracle):
    Kx, Vx = W.make_kv(2, 2, 300, 6)  # 4 full blocks + 44 residual tokens
    caches = []
    for _ in range(2):
        oc = oracle.OracleCache(2, 2, 2, 512, 1e-2, 2e-2)
        oc.build_codebook(Kx, Vx)
        oc.compress_blocks(Kx, Vx)
        caches.append(oc)
    a, b = caches
    assert bytes(a.arena) == bytes(b.arena)
    assert a.n_blocks == 4 and a.n_res == 44
    np.testing.assert_array_equal(a.res[K][:, :44], Kx[:, 256:])
    np.testing.assert_array_equal(a.res[V][:, :44], Vx[:, 256:])
    # placement: all K records in (b,h,j) order from offset 0, then all V records in the same order
    at = 0
    for which in (K, V):
        for bh in range(4):
            for j in range(4):
                assert a.off16[which][bh, j] == at
                at += int(a.size16[which][bh, j])
    assert at * 16 == len(a.arena)
    # every record decodes back to the codes of its own block with its own tensor's codebook
    for which, X in ((K, Kx), (V, Vx)):
        codes, mm = oracle.tensor_quantize(which, X, a.rel_eb[which])
        i = 0
        for bb in range(2):
            for h in range(2):
                for j in range(4):
                    c, m = oracle.decode_block_serial(which, a.get_block(which, bb, h, j), a.len[which])
                    np.testing.assert_array_equal(c, codes[i])
                    np.testing.assert_array_equal(m, mm[i])
                    i += 1


def test_append_equals_prefill_of_the_longer_sequence(oracle):
    # Section 3.2.3: blocks are independent, so appending token by token must give the same records as
    # compressing the longer sequence at once (same codebook), and the same fp16 tail
    B, H, S0, extra = 2, 2, 100, 130
    Kx, Vx = W.make_kv(B, H, S0 + extra, 8)
    ref = oracle.OracleCache(B, H, H, 256, 1e-2, 1e-2)
    ref.build_codebook(Kx[:, :S0], Vx[:, :S0])
    inc = oracle.OracleCache(B, H, H, 256, 1e-2, 1e-2)
    inc.build_codebook(Kx[:, :S0], Vx[:, :S0])
    ref.compress_blocks(Kx, Vx)
    inc.compress_blocks(Kx[:, :S0], Vx[:, :S0])
    for t in range(S0, S0 + extra):
        inc.append_token(Kx[:, t], Vx[:, t])
    assert inc.n_blocks == ref.n_blocks == 3 and inc.n_res == ref.n_res == 38
    for which in (K, V):
        for b in range(B):
            for h in range(H):
                for j in range(3):
                    np.testing.assert_array_equal(inc.get_block(which, b, h, j), ref.get_block(which, b, h, j))
        np.testing.assert_array_equal(inc.res[which][:, :38], ref.res[which][:, :38])
    q = W.make_queries(B, H, 1, 8)[0]
    np.testing.assert_allclose(inc.attn_decode(q, 0.1), ref.attn_decode(q, 0.1), rtol=0, atol=1e-15)
    with pytest.raises(RuntimeError):
        for _ in range(64):
            inc.append_token(Kx[:, 0], Vx[:, 0])


@pytest.mark.parametrize("window", [128, 256])
def test_larger_buffer_keeps_a_recent_window_uncompressed(oracle, window):
    # Section 3.2.1 / Section 4.2 (maximum buffer size): the buffer holds up to `window` tokens; when it is full its
    # oldest block is cut off and compressed.  Blocks are independent of the buffer size (same codebook), so block j
    # must be the very record that the cache with the 64-token buffer holds; the buffer must hold the newest tokens
    # in order, and storing a prompt must equal appending its tokens one by one.
    B, H, S0, extra = 1, 2, 200, 250
    S = S0 + extra
    Kx, Vx = W.make_kv(B, H, S, 9)
    small = oracle.OracleCache(B, H, H, 512, 1e-2, 1e-2)
    small.build_codebook(Kx[:, :S0], Vx[:, :S0])
    small.compress_blocks(Kx, Vx)
    assert small.n_blocks == 7 and small.n_res == 2
    inc = oracle.OracleCache(B, H, H, 512, 1e-2, 1e-2, buffer_tokens=window)
    one = oracle.OracleCache(B, H, H, 512, 1e-2, 1e-2, buffer_tokens=window)
    for oc in (inc, one):
        oc.build_codebook(Kx[:, :S0], Vx[:, :S0])
    one.compress_blocks(Kx, Vx)
    inc.compress_blocks(Kx[:, :S0], Vx[:, :S0])
    for t in range(S0, S):
        inc.append_token(Kx[:, t], Vx[:, t])
        # a warm buffer keeps between window-64 and window-1 tokens
        tokens = t + 1
        assert inc.n_blocks * 64 + inc.n_res == tokens
        assert inc.n_res == tokens if tokens < window else window - 64 <= inc.n_res <= window - 1
    nb = (S - window) // 64 + 1
    for oc in (inc, one):
        assert oc.n_blocks == nb and oc.n_res == S - 64 * nb
        for which, X in ((K, Kx), (V, Vx)):
            np.testing.assert_array_equal(oc.res[which][:, : oc.n_res], X[:, 64 * nb:])
            for h in range(H):
                for j in range(nb):
                    np.testing.assert_array_equal(oc.get_block(which, 0, h, j), small.get_block(which, 0, h, j))
            np.testing.assert_array_equal(oc.decompress(which)[:, : 64 * nb], small.decompress(which)[:, : 64 * nb])
            np.testing.assert_array_equal(oc.decompress(which)[:, 64 * nb:], X[:, 64 * nb:])
    assert bytes(inc.arena) != b"" and inc.stats()["residual_bytes"] == 2 * B * H * inc.n_res * 128 * 2
    with pytest.raises(ValueError):
        oracle.OracleCache(B, H, H, 512, 1e-2, 1e-2, buffer_tokens=100)


def test_a_slice_decodes_from_both_ends_by_hand(oracle):
    # An independent, bit-by-bit prefix decoder written here (dictionary of code words) reads slice 0 of a K record
    # upwards from its start for symbols 0..31 and downwards from its end for symbols 63..32.
    rng = np.random.default_rng(23)
    counts = rng.integers(1, 40, 26) ** 2
    ln, cd, _ = oracle.build_codebook(_hist(counts), 26, 12)
    book = {format(int(cd[s]), "b").zfill(int(ln[s])): s for s in range(26)}
    codes = rng.choice(26, size=(64, 128), p=counts / counts.sum()).astype(np.uint8)
    rec = oracle.encode_block(K, codes, np.zeros((128, 2), np.uint16), ln, cd)
    hdr = oracle.header_bytes(K)
    bits = np.unpackbits(rec[hdr:], bitorder="little")
    sb = rec[512:hdr].view("<u2").astype(np.int64)
    for s in (0, 1, 77, 127):
        start, end = int(sb[:s].sum()), int(sb[: s + 1].sum())
        want = _slice_order(K, codes)[s]
        pos, got_up = start, []
        while len(got_up) < 32:
            w = ""
            while w not in book:
                w += str(bits[pos]); pos += 1
            got_up.append(book[w])
        pos_dn, got_dn = end, []
        while len(got_dn) < 32:
            w = ""
            while w not in book:
                pos_dn -= 1; w += str(bits[pos_dn])
            got_dn.append(book[w])
        assert got_up == list(want[:32])
        assert got_dn == list(want[:31:-1])
        assert pos == pos_dn  # the two chains meet: no gap, no overlap
