"""Seeded synthetic KV-cache workloads (inputs only; none of the method's arithmetic lives here).

Both the CPU oracle's tests and the HIP path's tests/bench draw their inputs from this module so that the two
sides see byte-identical fp16 tensors.  The shapes follow the paper's evaluation setting (fp16 KV cache of shape
[context_len, head_num, head_dim], head_dim 128, context 2K-32K; Section 4.1 and Section 4.3) with a batch
dimension added outermost.  The value distributions are synthetic stand-ins for KV caches captured from real
model inference, which are not available here:

  for each (batch b, kv head h), in that order, from numpy.random.default_rng(seed):
      s_c      = lognormal(mean 0, sigma 0.5, size 128)              per-channel K scale
      outliers = choice(128, size 4, replace=False); s_c[outliers] *= 10
      K[b,:,h,:] = standard_normal((S,128)) * s_c  -> fp16 (round to nearest even)
      V[b,:,h,:] = standard_normal((S,128))        -> fp16
  queries / appended tokens: standard_normal -> fp16, from a second generator seeded (seed, 1) / (seed, 2).

Layout of every returned array: K, V -> uint16 view-compatible float16 arrays [B, S, H, 128]; q -> [B, Hq, 128].
"""
from __future__ import annotations

import dataclasses

import numpy as np

HEAD_DIM = 128
BLOCK_TOKENS = 64


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    n_kv_heads: int
    n_q_heads: int
    seq: int
    rel_eb: float
    seed: int
    decode_steps: int = 1
    append_steps: int = 0

    @property
    def max_seq(self) -> int:
        return self.seq + self.append_steps

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


# The five benchmark configurations (single transformer layer each).
CONFIGS = {
    "c0": Workload("c0", batch=1, n_kv_heads=1, n_q_heads=1, seq=1024, rel_eb=1e-2, seed=0, decode_steps=1),
    "c1": Workload("c1", batch=1, n_kv_heads=32, n_q_heads=32, seq=4096, rel_eb=1e-2, seed=1, decode_steps=32),
    "c2": Workload("c2", batch=1, n_kv_heads=32, n_q_heads=32, seq=32768, rel_eb=1e-2, seed=2, decode_steps=1),
    "c3": Workload("c3", batch=16, n_kv_heads=8, n_q_heads=32, seq=8192, rel_eb=1e-2, seed=3, decode_steps=1),
    "c4": Workload("c4", batch=8, n_kv_heads=8, n_q_heads=64, seq=16384, rel_eb=1e-2, seed=4, decode_steps=512,
                   append_steps=512),
}
C2_REL_EB_SWEEP = (5e-3, 1e-2, 2e-2)
# Longest Huffman code word that bench.py and the full-size parity tests allow for each error bound of the workloads
# (a parameter of the codec like the error bound itself; the library's own default is 12): the width of a fixed-length
# code of that bound's quantization levels (101, 51, 26 levels), but at least 6 bits.
CODE_LEN_LIMIT = {5e-3: 7, 1e-2: 6, 2e-2: 6}


def make_kv(batch: int, n_kv_heads: int, seq: int, seed: int):
    """Return (K, V) float16 arrays of shape [batch, seq, n_kv_heads, 128] following the module recipe."""
    rng = np.random.default_rng(seed)
    K = np.empty((batch, seq, n_kv_heads, HEAD_DIM), dtype=np.float16)
    V = np.empty((batch, seq, n_kv_heads, HEAD_DIM), dtype=np.float16)
    for b in range(batch):
        for h in range(n_kv_heads):
            s_c = rng.lognormal(0.0, 0.5, HEAD_DIM)
            outliers = rng.choice(HEAD_DIM, size=4, replace=False)
            s_c[outliers] *= 10.0
            K[b, :, h, :] = (rng.standard_normal((seq, HEAD_DIM), dtype=np.float32) * s_c.astype(np.float32)).astype(
                np.float16)
            V[b, :, h, :] = rng.standard_normal((seq, HEAD_DIM), dtype=np.float32).astype(np.float16)
    return K, V


def make_queries(batch: int, n_q_heads: int, steps: int, seed: int):
    """Return fp16 queries [steps, batch, n_q_heads, 128], N(0,1)."""
    rng = np.random.default_rng((seed, 1))
    return rng.standard_normal((steps, batch, n_q_heads, HEAD_DIM), dtype=np.float32).astype(np.float16)


def make_new_tokens(batch: int, n_kv_heads: int, steps: int, seed: int):
    """Return (k_new, v_new) fp16 arrays [steps, batch, n_kv_heads, 128] for the streaming-append path.

    k_new uses a per-(b,h) channel scale drawn the same way as in make_kv (but from its own generator), so the
    appended K rows keep a channel structure; v_new is N(0,1).
    """
    rng = np.random.default_rng((seed, 2))
    s_c = rng.lognormal(0.0, 0.5, (batch, n_kv_heads, HEAD_DIM)).astype(np.float32)
    k_new = (rng.standard_normal((steps, batch, n_kv_heads, HEAD_DIM), dtype=np.float32) * s_c).astype(np.float16)
    v_new = rng.standard_normal((steps, batch, n_kv_heads, HEAD_DIM), dtype=np.float32).astype(np.float16)
    return k_new, v_new


def make_workload(w: Workload, seq: int | None = None):
    """Materialise (K, V, q[steps]) for a Workload; `seq` may override the prefill length (tests use short ones)."""
    s = w.seq if seq is None else seq
    K, V = make_kv(w.batch, w.n_kv_heads, s, w.seed)
    q = make_queries(w.batch, w.n_q_heads, w.decode_steps, w.seed)
    return K, V, q
