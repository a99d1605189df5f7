"""ctypes/numpy wrapper around the C oracle (kvcomp_oracle.c).  TEST INFRASTRUCTURE ONLY.

The arithmetic of every step lives in the C file; this module only marshals numpy arrays, and keeps the
bookkeeping of the growing cache (Section 3.2.1 buffering, Section 3.2.3 appending): which blocks exist, where their
records sit in the compressed data buffer (the Block Offsets Array of Section 3) and which tokens are still in the
fp16 buffer.  It never imports, loads or calls the HIP library.
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from . import build as _build

D = 128
BT = 64

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(str(path))
        u8p, u16p, u32p, u64p, f64p = (C.POINTER(C.c_uint8), C.POINTER(C.c_uint16), C.POINTER(C.c_uint32),
                                       C.POINTER(C.c_uint64), C.POINTER(C.c_double))
        L.orc_n_units.restype = C.c_int
        L.orc_n_units.argtypes = [C.c_int, C.c_int]
        L.orc_n_slices.restype = C.c_int
        L.orc_n_slices.argtypes = [C.c_int]
        L.orc_minmax_bytes.restype = C.c_int
        L.orc_minmax_bytes.argtypes = [C.c_int, C.c_int]
        L.orc_header_bytes.restype = C.c_int
        L.orc_header_bytes.argtypes = [C.c_int, C.c_int]
        L.orc_n_sym.restype = C.c_int
        L.orc_n_sym.argtypes = [C.c_float]
        L.orc_quantize_block.restype = C.c_int
        L.orc_quantize_block.argtypes = [C.c_int, C.c_int, u16p, C.c_float, u8p, u16p]
        L.orc_dequantize_block.restype = None
        L.orc_dequantize_block.argtypes = [C.c_int, C.c_int, u8p, u16p, C.c_float, f64p]
        L.orc_reconstruct_block_fp16.restype = None
        L.orc_reconstruct_block_fp16.argtypes = [C.c_int, C.c_int, u8p, u16p, C.c_float, u16p]
        L.orc_float_to_half.restype = C.c_uint16
        L.orc_float_to_half.argtypes = [C.c_float]
        L.orc_histogram.restype = None
        L.orc_histogram.argtypes = [u8p, C.c_size_t, u64p]
        L.orc_build_codebook.restype = C.c_int
        L.orc_build_codebook.argtypes = [u64p, C.c_int, C.c_int, u8p, u32p]
        L.orc_encode_block.restype = C.c_size_t
        L.orc_encode_block.argtypes = [C.c_int, C.c_int, u8p, u16p, u8p, u32p, u8p, C.c_size_t]
        L.orc_decode_block_serial.restype = C.c_int
        L.orc_decode_block_serial.argtypes = [C.c_int, C.c_int, u8p, u8p, u8p, u16p]
        L.orc_decode_block_tree.restype = C.c_int
        L.orc_decode_block_tree.argtypes = [C.c_int, C.c_int, u8p, u8p, u32p, u8p, u16p]
        L.orc_attention_head.restype = None
        L.orc_attention_head.argtypes = [f64p, f64p, C.c_long, u16p, C.c_double, f64p]
        L.orc_tensor_quantize.restype = C.c_int
        L.orc_tensor_quantize.argtypes = [C.c_int, C.c_int, u16p, C.c_int, C.c_long, C.c_int, C.c_float, u8p, u16p]
        L.orc_tensor_encode.restype = C.c_size_t
        L.orc_tensor_encode.argtypes = [C.c_int, C.c_int, u8p, u16p, C.c_long, u8p, u32p, u8p, C.c_size_t, u32p]
        L.orc_attn_decode.restype = C.c_int
        L.orc_attn_decode.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_float, C.c_float, C.c_long, C.c_long,
                                      u8p, u32p, u32p, u8p, u8p, u16p, u16p, C.c_int, C.c_int, u16p, C.c_double,
                                      f64p]
        L.orc_num_threads.restype = C.c_int
        _lib = L
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(C.POINTER(ct))


def _bits(x):
    """float16 array -> contiguous uint16 bit patterns."""
    x = np.ascontiguousarray(x)
    assert x.dtype == np.float16
    return x.view(np.uint16)


K, V = 0, 1

# worst-case record: header + 64*128 symbols at 16 bits each
MAX_RECORD_BYTES = 768 + BT * D * 2 + 16


def n_sym(rel_eb):
    return lib().orc_n_sym(np.float32(rel_eb))


def n_units(which, k_mode=0):
    return lib().orc_n_units(which, k_mode)


def header_bytes(which, k_mode=0):
    return lib().orc_header_bytes(which, k_mode)


def quantize_block(which, tile, rel_eb, k_mode=0):
    """tile: float16 [64,128] -> (codes uint8 [64,128], minmax uint16 [n_units,2])."""
    t = _bits(tile).reshape(BT, D)
    codes = np.zeros((BT, D), np.uint8)
    mm = np.zeros((n_units(which, k_mode), 2), np.uint16)
    r = lib().orc_quantize_block(which, k_mode, _p(t, C.c_uint16), np.float32(rel_eb), _p(codes, C.c_uint8),
                                 _p(mm, C.c_uint16))
    if r:
        raise ValueError(f"orc_quantize_block failed: {r}")
    return codes, mm


def dequantize_block(which, codes, minmax, rel_eb, k_mode=0):
    codes = np.ascontiguousarray(codes, np.uint8)
    minmax = np.ascontiguousarray(minmax, np.uint16)
    out = np.zeros((BT, D), np.float64)
    lib().orc_dequantize_block(which, k_mode, _p(codes, C.c_uint8), _p(minmax, C.c_uint16), np.float32(rel_eb),
                               _p(out, C.c_double))
    return out


def reconstruct_block_fp16(which, codes, minmax, rel_eb, k_mode=0):
    """Reconstructed block as float16 [64,128]: binary32 code * width + min, rounded once to binary16."""
    codes = np.ascontiguousarray(codes, np.uint8)
    minmax = np.ascontiguousarray(minmax, np.uint16)
    out = np.zeros((BT, D), np.uint16)
    lib().orc_reconstruct_block_fp16(which, k_mode, _p(codes, C.c_uint8), _p(minmax, C.c_uint16), np.float32(rel_eb),
                                     _p(out, C.c_uint16))
    return out.view(np.float16)


def float_to_half_bits(x):
    """binary32 -> binary16 bit pattern, round to nearest even (the oracle's own conversion)."""
    return int(lib().orc_float_to_half(float(x)))


def histogram(codes):
    codes = np.ascontiguousarray(codes, np.uint8)
    h = np.zeros(256, np.uint64)
    lib().orc_histogram(_p(codes, C.c_uint8), codes.size, _p(h, C.c_uint64))
    return h


def build_codebook(hist, nsym, max_len=12):
    """-> (len uint8[256], code uint32[256], halvings)."""
    hist = np.ascontiguousarray(hist, np.uint64)
    ln = np.zeros(256, np.uint8)
    cd = np.zeros(256, np.uint32)
    r = lib().orc_build_codebook(_p(hist, C.c_uint64), nsym, max_len, _p(ln, C.c_uint8), _p(cd, C.c_uint32))
    if r < 0:
        raise ValueError("orc_build_codebook: bad argument")
    return ln, cd, r


def encode_block(which, codes, minmax, ln, cd, k_mode=0):
    codes = np.ascontiguousarray(codes, np.uint8)
    minmax = np.ascontiguousarray(minmax, np.uint16)
    rec = np.zeros(MAX_RECORD_BYTES, np.uint8)
    n = lib().orc_encode_block(which, k_mode, _p(codes, C.c_uint8), _p(minmax, C.c_uint16), _p(ln, C.c_uint8),
                               _p(cd, C.c_uint32), _p(rec, C.c_uint8), rec.size)
    if n == 0:
        raise ValueError("orc_encode_block failed (symbol without a code word?)")
    return rec[:n].copy()


def decode_block_serial(which, rec, ln, k_mode=0):
    rec = np.ascontiguousarray(rec, np.uint8)
    codes = np.zeros((BT, D), np.uint8)
    mm = np.zeros((n_units(which, k_mode), 2), np.uint16)
    r = lib().orc_decode_block_serial(which, k_mode, _p(rec, C.c_uint8), _p(ln, C.c_uint8), _p(codes, C.c_uint8),
                                      _p(mm, C.c_uint16))
    if r:
        raise ValueError("malformed stream")
    return codes, mm


def decode_block_tree(which, rec, ln, cd, k_mode=0):
    rec = np.ascontiguousarray(rec, np.uint8)
    codes = np.zeros((BT, D), np.uint8)
    mm = np.zeros((n_units(which, k_mode), 2), np.uint16)
    r = lib().orc_decode_block_tree(which, k_mode, _p(rec, C.c_uint8), _p(ln, C.c_uint8), _p(cd, C.c_uint32),
                                    _p(codes, C.c_uint8), _p(mm, C.c_uint16))
    if r:
        raise ValueError("malformed stream")
    return codes, mm


def attention_head(Kd, Vd, q, scale):
    Kd = np.ascontiguousarray(Kd, np.float64)
    Vd = np.ascontiguousarray(Vd, np.float64)
    qb = _bits(q).reshape(D)
    out = np.zeros(D, np.float64)
    lib().orc_attention_head(_p(Kd, C.c_double), _p(Vd, C.c_double), Kd.shape[0], _p(qb, C.c_uint16), float(scale),
                             _p(out, C.c_double))
    return out


def tensor_quantize(which, X, rel_eb, k_mode=0):
    """X: float16 [B,S,H,128] -> (codes [B*H*NB,64,128], minmax [B*H*NB,n_units,2]) over the S//64 full blocks."""
    Xb = _bits(X)
    B, S, H, _ = Xb.shape
    nblk = B * H * (S // BT)
    nu = n_units(which, k_mode)
    codes = np.zeros((nblk, BT, D), np.uint8)
    mm = np.zeros((nblk, nu, 2), np.uint16)
    r = lib().orc_tensor_quantize(which, k_mode, _p(Xb, C.c_uint16), B, S, H, np.float32(rel_eb), _p(codes, C.c_uint8),
                                  _p(mm, C.c_uint16))
    if r:
        raise ValueError(f"orc_tensor_quantize failed: {r}")
    return codes, mm


def tensor_encode(which, codes, minmax, ln, cd, k_mode=0):
    """-> (bytes uint8[total], sizes16 uint32[nblk]); records compact, in block order."""
    nblk = codes.shape[0]
    cap = nblk * MAX_RECORD_BYTES
    out = np.zeros(cap, np.uint8)
    sizes = np.zeros(nblk, np.uint32)
    n = lib().orc_tensor_encode(which, k_mode, _p(codes, C.c_uint8), _p(minmax, C.c_uint16), nblk, _p(ln, C.c_uint8),
                                _p(cd, C.c_uint32), _p(out, C.c_uint8), cap, _p(sizes, C.c_uint32))
    if n == 0 and nblk > 0:
        raise ValueError("orc_tensor_encode failed")
    return out[:n].copy(), sizes


class OracleCache:
    """The growing compressed cache of one layer, CPU side (mirror of the four library calls).

    buffer_tokens is the maximum buffer size of Section 3.2.1 / Section 4.2 (a multiple of the block size): new
    tokens stay uncompressed in the buffer, oldest first; the append that brings the buffer to buffer_tokens
    tokens cuts its oldest block of 64 tokens off and compresses it, so a warm cache keeps the newest
    buffer_tokens-64 .. buffer_tokens-1 tokens as fp16.  A prompt is stored as if its tokens had been appended
    one by one.
    """

    def __init__(self, batch, n_kv_heads, n_q_heads, max_seq, rel_eb_k, rel_eb_v, k_mode=0, max_code_len=12,
                 buffer_tokens=BT):
        if buffer_tokens < BT or buffer_tokens % BT:
            raise ValueError("buffer_tokens must be a positive multiple of the block size")
        self.W = buffer_tokens
        self.B, self.H, self.Hq = batch, n_kv_heads, n_q_heads
        self.max_blocks = max_seq // BT
        self.max_seq = max_seq
        self.rel_eb = (np.float32(rel_eb_k), np.float32(rel_eb_v))
        self.k_mode = k_mode
        self.max_code_len = max_code_len
        self.hist = [None, None]
        self.len = [None, None]
        self.code = [None, None]
        self.halvings = [0, 0]
        self.arena = bytearray()
        self.off16 = [np.zeros((batch * n_kv_heads, self.max_blocks), np.uint32) for _ in range(2)]
        self.size16 = [np.zeros((batch * n_kv_heads, self.max_blocks), np.uint32) for _ in range(2)]
        self.n_blocks = 0
        self.n_res = 0
        self.res = [np.zeros((batch, buffer_tokens, n_kv_heads, D), np.float16) for _ in range(2)]
        self.payload_bits = [0, 0]

    def _mode(self, which):
        return self.k_mode if which == K else 0

    def build_codebook(self, Kx, Vx):
        for which, X in ((K, Kx), (V, Vx)):
            codes, _ = tensor_quantize(which, X, self.rel_eb[which], self._mode(which))
            self.hist[which] = histogram(codes)
            self.len[which], self.code[which], self.halvings[which] = build_codebook(
                self.hist[which], n_sym(self.rel_eb[which]), self.max_code_len)

    def _place(self, which, recs, sizes, idx):
        """Append records (already compact, in order) at the arena tail; idx: list of (bh, j) in the same order."""
        base16 = len(self.arena) // 16
        self.arena += recs.tobytes()
        at = base16
        hdr = header_bytes(which, self._mode(which))
        mmb = lib().orc_minmax_bytes(which, self._mode(which))
        for (bh, j), s16 in zip(idx, sizes):
            self.off16[which][bh, j] = at
            self.size16[which][bh, j] = s16
            rec = np.frombuffer(self.arena, np.uint8, int(s16) * 16, at * 16)
            sb = rec[mmb:hdr].view(np.uint16)
            self.payload_bits[which] += int(sb.astype(np.int64).sum())
            at += int(s16)

    def compress_blocks(self, Kx, Vx):
        if self.len[0] is None:
            raise RuntimeError("codebook not built")
        if self.n_blocks or self.n_res:
            raise RuntimeError("cache not empty")
        B, S, H, _ = Kx.shape
        if S > self.max_seq:
            raise RuntimeError("capacity")
        NB = 0 if S < self.W else (S - self.W) // BT + 1  # blocks cut off by S appends to an empty buffer
        for which, X in ((K, Kx), (V, Vx)):
            if NB:
                m = self._mode(which)
                codes, mm = tensor_quantize(which, np.ascontiguousarray(X[:, : NB * BT]), self.rel_eb[which], m)
                recs, sizes = tensor_encode(which, codes, mm, self.len[which], self.code[which], m)
                idx = [(bh, j) for bh in range(B * H) for j in range(NB)]
                self._place(which, recs, sizes, idx)
            self.res[which][:, : S - NB * BT] = X[:, NB * BT:]
        self.n_blocks = NB
        self.n_res = S - NB * BT

    def append_token(self, k_new, v_new):
        """k_new, v_new: float16 [B,H,128].  The call that fills the buffer compresses its oldest block at once."""
        if self.n_blocks * BT + self.n_res + 1 > self.max_seq:
            raise RuntimeError("capacity")
        self.res[K][:, self.n_res] = k_new
        self.res[V][:, self.n_res] = v_new
        self.n_res += 1
        if self.n_res == self.W:
            for which in (K, V):
                m = self._mode(which)
                oldest = np.ascontiguousarray(self.res[which][:, :BT])
                codes, mm = tensor_quantize(which, oldest, self.rel_eb[which], m)
                recs, sizes = tensor_encode(which, codes, mm, self.len[which], self.code[which], m)
                idx = [(bh, self.n_blocks) for bh in range(self.B * self.H)]
                self._place(which, recs, sizes, idx)
                self.res[which][:, : self.W - BT] = self.res[which][:, BT:].copy()
            self.n_blocks += 1
            self.n_res -= BT

    def attn_decode(self, q, scale):
        """q: float16 [B,Hq,128] -> float64 [B,Hq,128]."""
        qb = _bits(q)
        out = np.zeros((self.B, self.Hq, D), np.float64)
        arena = np.frombuffer(bytes(self.arena) + b"\0" * 16, np.uint8)
        rk, rv = _bits(self.res[K]), _bits(self.res[V])
        r = lib().orc_attn_decode(self.B, self.H, self.Hq, self.k_mode, self.rel_eb[K], self.rel_eb[V], self.n_blocks,
                                  self.max_blocks, _p(arena, C.c_uint8), _p(self.off16[K], C.c_uint32),
                                  _p(self.off16[V], C.c_uint32), _p(self.len[K], C.c_uint8), _p(self.len[V], C.c_uint8),
                                  _p(rk, C.c_uint16), _p(rv, C.c_uint16), self.W, self.n_res, _p(qb, C.c_uint16), float(scale),
                                  _p(out, C.c_double))
        if r:
            raise RuntimeError(f"orc_attn_decode failed: {r}")
        return out

    def decompress(self, which):
        """The whole cache of one tensor as float16 [B, tokens, H, 128]: reconstructed blocks, then the buffered tokens."""
        tokens = self.n_blocks * BT + self.n_res
        out = np.zeros((self.B, tokens, self.H, D), np.float16)
        for b in range(self.B):
            for h in range(self.H):
                for j in range(self.n_blocks):
                    codes, mm = decode_block_serial(which, self.get_block(which, b, h, j), self.len[which],
                                                    self._mode(which))
                    out[b, j * BT:(j + 1) * BT, h] = reconstruct_block_fp16(which, codes, mm, self.rel_eb[which],
                                                                            self._mode(which))
        out[:, self.n_blocks * BT:] = self.res[which][:, : self.n_res]
        return out

    def get_block(self, which, b, h, j):
        bh = b * self.H + h
        o, s = int(self.off16[which][bh, j]) * 16, int(self.size16[which][bh, j]) * 16
        return np.frombuffer(self.arena, np.uint8, s, o).copy()

    def stats(self):
        nblk = self.B * self.H * self.n_blocks
        tokens = self.n_blocks * BT + self.n_res
        raw = 2 * self.B * self.H * tokens * D * 2
        rec = [int(self.size16[w][:, : self.n_blocks].astype(np.int64).sum()) * 16 for w in (K, V)]
        header = sum(header_bytes(w, self._mode(w)) for w in (K, V)) * nblk
        offsets = 2 * nblk * 8
        residual = 2 * self.B * self.H * self.n_res * D * 2
        stored = rec[0] + rec[1] + offsets + residual
        return dict(n_blocks=self.n_blocks, n_res=self.n_res, raw_bytes=raw, record_bytes_k=rec[0],
                    record_bytes_v=rec[1], header_bytes=header, offsets_bytes=offsets, residual_bytes=residual,
                    payload_bits_k=self.payload_bits[K], payload_bits_v=self.payload_bits[V],
                    stored_bytes=stored, compression_ratio=(raw / stored) if stored else 0.0)


def num_threads():
    return lib().orc_num_threads()


def set_num_threads(n):
    lib().orc_set_num_threads.restype = None
    lib().orc_set_num_threads.argtypes = [C.c_int]
    lib().orc_set_num_threads(int(n))
