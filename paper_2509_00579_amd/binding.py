"""Thin ctypes binding over libkvcomp.so (argument marshalling only; every step runs in the HIP kernels).

PyTorch is used for device memory and streams.  The library must have been built (paper_2509_00579_amd/build.py or
__graft_entry__.build()); importing this module without it raises.
"""
from __future__ import annotations

import ctypes as C
import os
import pathlib

import numpy as np
import torch

HERE = pathlib.Path(__file__).resolve().parent
LIB_PATH = HERE / "libkvcomp.so"

K, V = 0, 1
D, BT = 128, 64

OK, ERR_INVALID_ARG, ERR_STATE, ERR_CAPACITY, ERR_HIP, ERR_NONFINITE = 0, -1, -2, -3, -4, -5


class Config(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_kv_heads", C.c_int32), ("n_q_heads", C.c_int32), ("head_dim", C.c_int32),
                ("block_tokens", C.c_int32), ("max_seq", C.c_int32), ("rel_eb_k", C.c_float), ("rel_eb_v", C.c_float),
                ("k_mode", C.c_int32), ("max_code_len", C.c_int32), ("buffer_tokens", C.c_int32)]


class Stats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in (
        "n_blocks", "n_res", "raw_bytes", "record_bytes_k", "record_bytes_v", "header_bytes", "offsets_bytes",
        "residual_bytes", "payload_bits_k", "payload_bits_v", "stored_bytes", "max_record_bytes")] + [
        ("compression_ratio", C.c_double)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


# every symbol include/kvcomp.h declares: name -> (restype, argtypes)
_vp, _i, _f = C.c_void_p, C.c_int, C.c_float
_cfgp = C.POINTER(Config)
SIGNATURES = {
    "kvcomp_arena_bytes": (C.c_size_t, [_cfgp]),
    "kvcomp_create": (_i, [_cfgp, _vp, C.c_size_t, _vp, C.POINTER(_vp)]),
    "kvcomp_destroy": (_i, [_vp]),
    "kvcomp_reset": (_i, [_vp, _i, _vp]),
    "kvcomp_build_codebook": (_i, [_vp, _vp, _vp, _i, _vp]),
    "kvcomp_compress_blocks": (_i, [_vp, _vp, _vp, _i, _vp]),
    "kvcomp_prefill_workspace_bytes": (C.c_size_t, [_cfgp, _i]),
    "kvcomp_prefill": (_i, [_vp, _vp, _vp, _i, _vp, C.c_size_t, _vp]),
    "kvcomp_append_token": (_i, [_vp, _vp, _vp, _vp]),
    "kvcomp_attn_decode": (_i, [_vp, _vp, _f, _vp, _vp]),
    "kvcomp_append_attn_decode": (_i, [_vp, _vp, _vp, _vp, _f, _vp, _vp]),
    "kvcomp_get_stats": (_i, [_vp, C.POINTER(Stats), _vp]),
    "kvcomp_debug_codes": (_i, [_vp, _i, _vp, _i, _vp, C.c_size_t, _vp, _vp, _vp]),
    "kvcomp_get_histogram": (_i, [_vp, _i, _vp, _vp]),
    "kvcomp_get_codebook": (_i, [_vp, _i, _vp, _vp]),
    "kvcomp_get_block_entry": (_i, [_vp, _i, _i, _i, _i, C.POINTER(C.c_uint32), C.POINTER(C.c_uint32), _vp]),
    "kvcomp_get_block": (_i, [_vp, _i, _i, _i, _i, _vp, C.c_size_t, C.POINTER(C.c_size_t), _vp]),
    "kvcomp_get_residual": (_i, [_vp, _i, _vp, C.POINTER(_i), _vp]),
    "kvcomp_decompress": (_i, [_vp, _i, _vp, _i, _vp]),
    "kvcomp_decompress_tree_walk": (_i, [_vp, _i, _vp, _i, _vp]),
    "kvcomp_set_tuning": (_i, [_vp, _i, _i, _i]),
    "kvcomp_set_profiling": (_i, [_vp, _i]),
    "kvcomp_get_profile": (_i, [_vp, C.POINTER(_i), C.POINTER(C.c_double)]),
    "kvcomp_probe_read_stream": (_i, [_vp, C.c_size_t, _vp, C.POINTER(C.c_size_t), _vp]),
    "kvcomp_baseline_workspace_bytes": (C.c_size_t, [_cfgp]),
    "kvcomp_baseline_fp16_attn": (_i, [_cfgp, _vp, _vp, _i, _vp, _f, _vp, _vp, C.c_size_t, _i, _vp]),
    "kvcomp_baseline_fp16_attn_noalloc": (_i, [_cfgp, _vp, _vp, _i, _vp, _f, _vp, _i, _vp]),
    "kvcomp_last_error": (C.c_char_p, []),
}

_lib = None


def load():
    """Load libkvcomp.so; fails loudly when the HIP extension has not been built."""
    global _lib
    if _lib is None:
        path = pathlib.Path(os.environ.get("KVCOMP_LIB", LIB_PATH))  # KVCOMP_LIB: try another build of the library
        if not path.exists():
            raise RuntimeError(f"{path} is missing: build it with `python -m paper_2509_00579_amd.build` "
                               "(there is no CPU fallback)")
        lib = C.CDLL(str(path))
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


class KvcompError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"kvcomp status {status}: {msg}")
        self.status = status


def _check(st):
    if st != OK:
        raise KvcompError(st, load().kvcomp_last_error().decode())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev_fp16(t, shape):
    assert t.is_cuda and t.dtype == torch.float16 and t.is_contiguous(), "expected a contiguous CUDA fp16 tensor"
    assert tuple(t.shape) == tuple(shape), f"expected shape {tuple(shape)}, got {tuple(t.shape)}"
    return C.c_void_p(t.data_ptr())


def make_config(batch, n_kv_heads, n_q_heads, max_seq, rel_eb_k, rel_eb_v, k_mode=0, max_code_len=0,
                buffer_tokens=0):
    return Config(batch, n_kv_heads, n_q_heads, D, BT, max_seq, rel_eb_k, rel_eb_v, k_mode, max_code_len,
                  buffer_tokens)


class KVCompCache:
    """One layer's compressed KV cache on the GPU: the four calls of the hot path plus the parity exports."""

    def __init__(self, batch, n_kv_heads, n_q_heads, max_seq, rel_eb_k, rel_eb_v, k_mode=0, max_code_len=0,
                 buffer_tokens=0, device="cuda:0", arena=None):
        self.lib = load()
        self.cfg = make_config(batch, n_kv_heads, n_q_heads, max_seq, rel_eb_k, rel_eb_v, k_mode, max_code_len,
                               buffer_tokens)
        self.buffer_tokens = buffer_tokens or BT
        self.B, self.H, self.Hq, self.max_seq = batch, n_kv_heads, n_q_heads, max_seq
        self.device = torch.device(device)
        nbytes = self.lib.kvcomp_arena_bytes(C.byref(self.cfg))
        if nbytes == 0:
            raise KvcompError(ERR_INVALID_ARG, "invalid configuration")
        if arena is None:
            arena = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        assert arena.is_cuda and arena.dtype == torch.uint8 and arena.is_contiguous() and arena.numel() >= nbytes
        assert arena.data_ptr() % 256 == 0
        self.arena = arena
        h = C.c_void_p()
        _check(self.lib.kvcomp_create(C.byref(self.cfg), C.c_void_p(self.arena.data_ptr()), nbytes, _stream(), C.byref(h)))
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            self.lib.kvcomp_destroy(self.h)
            self.h = None

    __del__ = close

    # ---- hot path ----
    def build_codebook(self, Kt, Vt):
        S = Kt.shape[1]
        shape = (self.B, S, self.H, D)
        _check(self.lib.kvcomp_build_codebook(self.h, _dev_fp16(Kt, shape), _dev_fp16(Vt, shape), S, _stream()))

    def compress_blocks(self, Kt, Vt):
        S = Kt.shape[1]
        shape = (self.B, S, self.H, D)
        _check(self.lib.kvcomp_compress_blocks(self.h, _dev_fp16(Kt, shape), _dev_fp16(Vt, shape), S, _stream()))

    def prefill_workspace_bytes(self, S):
        return self.lib.kvcomp_prefill_workspace_bytes(C.byref(self.cfg), S)

    def prefill(self, Kt, Vt, workspace=None):
        """build_codebook + compress_blocks with one quantization pass; `workspace`: a uint8 CUDA tensor of at least
        prefill_workspace_bytes(S) bytes (allocated here if None)."""
        S = Kt.shape[1]
        shape = (self.B, S, self.H, D)
        if workspace is None:
            workspace = torch.empty(self.prefill_workspace_bytes(S), dtype=torch.uint8, device=self.device)
        assert workspace.is_cuda and workspace.dtype == torch.uint8 and workspace.is_contiguous()
        _check(self.lib.kvcomp_prefill(self.h, _dev_fp16(Kt, shape), _dev_fp16(Vt, shape), S,
                                       C.c_void_p(workspace.data_ptr()), workspace.numel(), _stream()))

    def append_token(self, k_new, v_new):
        shape = (self.B, self.H, D)
        _check(self.lib.kvcomp_append_token(self.h, _dev_fp16(k_new, shape), _dev_fp16(v_new, shape), _stream()))

    def attn_decode(self, q, scale, out=None):
        if out is None:
            out = torch.empty((self.B, self.Hq, D), dtype=torch.float32, device=self.device)
        assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous()
        _check(self.lib.kvcomp_attn_decode(self.h, _dev_fp16(q, (self.B, self.Hq, D)), float(scale),
                                           C.c_void_p(out.data_ptr()), _stream()))
        return out

    def append_attn_decode(self, k_new, v_new, q, scale, out=None):
        """append_token followed by attn_decode, in one launch whenever no block has to be compressed."""
        if out is None:
            out = torch.empty((self.B, self.Hq, D), dtype=torch.float32, device=self.device)
        assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous()
        shape = (self.B, self.H, D)
        _check(self.lib.kvcomp_append_attn_decode(self.h, _dev_fp16(k_new, shape), _dev_fp16(v_new, shape),
                                                  _dev_fp16(q, (self.B, self.Hq, D)), float(scale),
                                                  C.c_void_p(out.data_ptr()), _stream()))
        return out

    def reset(self, keep_codebook=True):
        _check(self.lib.kvcomp_reset(self.h, int(keep_codebook), _stream()))

    # ---- metrics / parity exports ----
    def stats(self):
        st = Stats()
        _check(self.lib.kvcomp_get_stats(self.h, C.byref(st), _stream()))
        return st.as_dict()

    def debug_codes(self, which, X):
        S = X.shape[1]
        nblk = self.B * self.H * (S // BT)
        units = (1 if self.cfg.k_mode == 1 else D) if which == K else BT
        scratch = torch.empty(nblk * (BT * D + 4 * units), dtype=torch.uint8, device=self.device)
        codes = np.zeros((nblk, BT, D), np.uint8)
        mm = np.zeros((nblk, units, 2), np.uint16)
        _check(self.lib.kvcomp_debug_codes(self.h, which, _dev_fp16(X, (self.B, S, self.H, D)), S,
                                           C.c_void_p(scratch.data_ptr()), scratch.numel(),
                                           codes.ctypes.data_as(C.c_void_p), mm.ctypes.data_as(C.c_void_p), _stream()))
        return codes, mm

    def histogram(self, which):
        h = np.zeros(256, np.uint32)
        _check(self.lib.kvcomp_get_histogram(self.h, which, h.ctypes.data_as(C.c_void_p), _stream()))
        return h

    def codebook(self, which):
        ln, cd = np.zeros(256, np.uint8), np.zeros(256, np.uint32)
        _check(self.lib.kvcomp_get_codebook(self.h, which, ln.ctypes.data_as(C.c_void_p), cd.ctypes.data_as(C.c_void_p)))
        return ln, cd

    def block_entry(self, which, b, h, blk):
        o, s = C.c_uint32(), C.c_uint32()
        _check(self.lib.kvcomp_get_block_entry(self.h, which, b, h, blk, C.byref(o), C.byref(s), _stream()))
        return o.value, s.value

    def get_block(self, which, b, h, blk):
        buf = np.zeros(16384, np.uint8)
        n = C.c_size_t()
        _check(self.lib.kvcomp_get_block(self.h, which, b, h, blk, buf.ctypes.data_as(C.c_void_p), buf.size, C.byref(n),
                                         _stream()))
        return buf[: n.value].copy()

    def residual(self, which):
        buf = np.zeros((self.B, self.buffer_tokens, self.H, D), np.uint16)
        n = C.c_int()
        _check(self.lib.kvcomp_get_residual(self.h, which, buf.ctypes.data_as(C.c_void_p), C.byref(n), _stream()))
        return buf.view(np.float16)[:, : n.value], n.value

    def decompress(self, which, tokens, out=None, tree_walk=False):
        """The cache of one tensor as fp16 [B, tokens, H, 128] (stand-alone decompression; tree_walk: with the
        bit-serial decoder instead of the table decoder)."""
        if out is None:
            out = torch.empty((self.B, tokens, self.H, D), dtype=torch.float16, device=self.device)
        assert out.is_cuda and out.is_contiguous() and out.dtype == torch.float16
        fn = self.lib.kvcomp_decompress_tree_walk if tree_walk else self.lib.kvcomp_decompress
        _check(fn(self.h, which, C.c_void_p(out.data_ptr()), int(out.shape[1]), _stream()))
        return out

    def set_tuning(self, n_splits=0, stage_bytes=0, waves=0):
        _check(self.lib.kvcomp_set_tuning(self.h, n_splits, stage_bytes, waves))

    def set_profiling(self, enable):
        _check(self.lib.kvcomp_set_profiling(self.h, int(enable)))

    def get_profile(self):
        n, ms = C.c_int(), C.c_double()
        _check(self.lib.kvcomp_get_profile(self.h, C.byref(n), C.byref(ms)))
        return n.value, ms.value


class KVCompLayers:
    """The caches of all layers of a model: one context per layer (Section 3: buffers and codebooks are per layer,
    the K and the V codebook of a layer are built from that layer's prompt), carved out of a single device
    allocation.  `layers[i]` is the KVCompCache of layer i; nothing is computed here."""

    def __init__(self, n_layers, batch, n_kv_heads, n_q_heads, max_seq, rel_eb_k, rel_eb_v, device="cuda:0", **kw):
        lib = load()
        cfg = make_config(batch, n_kv_heads, n_q_heads, max_seq, rel_eb_k, rel_eb_v, kw.get("k_mode", 0),
                          kw.get("max_code_len", 0), kw.get("buffer_tokens", 0))
        per_layer = lib.kvcomp_arena_bytes(C.byref(cfg))
        if per_layer == 0 or n_layers < 1:
            raise KvcompError(ERR_INVALID_ARG, "invalid configuration")
        per_layer = (per_layer + 255) // 256 * 256
        self.arena = torch.empty(n_layers * per_layer, dtype=torch.uint8, device=torch.device(device))
        self.layers = [KVCompCache(batch, n_kv_heads, n_q_heads, max_seq, rel_eb_k, rel_eb_v, device=device,
                                   arena=self.arena[i * per_layer:(i + 1) * per_layer], **kw) for i in range(n_layers)]

    def __len__(self):
        return len(self.layers)

    def __getitem__(self, i):
        return self.layers[i]

    def stats(self):
        """Byte counts summed over the layers, and the overall compression ratio."""
        per = [c.stats() for c in self.layers]
        tot = {k: sum(p[k] for p in per) for k in ("raw_bytes", "record_bytes_k", "record_bytes_v", "header_bytes",
                                                    "offsets_bytes", "residual_bytes", "stored_bytes")}
        tot["compression_ratio"] = tot["raw_bytes"] / tot["stored_bytes"] if tot["stored_bytes"] else 0.0
        return tot

    def close(self):
        for c in self.layers:
            c.close()


def probe_read_stream(buf, sink):
    """One plain streaming read of the uint8 CUDA tensor `buf` (measurement aid); returns the bytes it reads."""
    assert buf.is_cuda and buf.is_contiguous() and sink.is_cuda and sink.numel() * sink.element_size() >= 4
    n = C.c_size_t()
    _check(load().kvcomp_probe_read_stream(C.c_void_p(buf.data_ptr()), buf.numel() * buf.element_size(),
                                           C.c_void_p(sink.data_ptr()), C.byref(n), _stream()))
    return n.value


class BaselineFp16Attention:
    """Decode attention on the uncompressed fp16 cache (the comparison kernel)."""

    def __init__(self, batch, n_kv_heads, n_q_heads, device="cuda:0"):
        self.lib = load()
        self.cfg = make_config(batch, n_kv_heads, n_q_heads, 64, 0.01, 0.01)
        self.B, self.H, self.Hq = batch, n_kv_heads, n_q_heads
        self.device = torch.device(device)
        self.ws = torch.zeros(self.lib.kvcomp_baseline_workspace_bytes(C.byref(self.cfg)), dtype=torch.uint8,
                              device=self.device)  # zero-filled once: it holds the split tickets

    def __call__(self, Kt, Vt, q, scale, out=None, n_splits=0):
        S = Kt.shape[1]
        shape = (self.B, S, self.H, D)
        if out is None:
            out = torch.empty((self.B, self.Hq, D), dtype=torch.float32, device=self.device)
        _check(self.lib.kvcomp_baseline_fp16_attn(C.byref(self.cfg), _dev_fp16(Kt, shape), _dev_fp16(Vt, shape), S,
                                                  _dev_fp16(q, (self.B, self.Hq, D)), float(scale),
                                                  C.c_void_p(out.data_ptr()), C.c_void_p(self.ws.data_ptr()),
                                                  self.ws.numel(), n_splits, _stream()))
        return out

    def noalloc(self, Kt, Vt, q, scale, out, n_splits=0):
        """The same through kvcomp_baseline_fp16_attn_noalloc: no workspace, the library's static scratch; `out` is
        the caller's."""
        S = Kt.shape[1]
        shape = (self.B, S, self.H, D)
        assert out.is_cuda and out.dtype == torch.float32 and out.is_contiguous()
        _check(self.lib.kvcomp_baseline_fp16_attn_noalloc(C.byref(self.cfg), _dev_fp16(Kt, shape), _dev_fp16(Vt, shape), S,
                                                          _dev_fp16(q, (self.B, self.Hq, D)), float(scale),
                                                          C.c_void_p(out.data_ptr()), n_splits, _stream()))
        return out
