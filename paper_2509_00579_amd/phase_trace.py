"""Phase timeline of the fused decode-attention kernel (developer tool, needs a GPU).

Builds a variant of the library with -DKVC_TRACE (every wave records the 100 MHz wall clock at eight points of the
kernel), runs a few decode steps on a seeded workload and prints, per point, when the waves reach it.

    python -m paper_2509_00579_amd.phase_trace [c1|c2|c3|c4] [max_code_len]
"""
from __future__ import annotations

import ctypes as C
import os
import pathlib
import sys

import numpy as np


def main():
    here = pathlib.Path(__file__).resolve().parent
    sys.path.insert(0, str(here.parent))
    from paper_2509_00579_amd import build as B

    lib_path = here / "_build" / "libkvcomp_trace.so"
    if not lib_path.exists():
        B.build(extra_flags=["-DKVC_TRACE"], out=lib_path)
    os.environ["KVCOMP_LIB"] = str(lib_path)
    import torch

    import workloads
    from paper_2509_00579_amd import binding

    name = sys.argv[1] if len(sys.argv) > 1 else "c1"
    mcl = int(sys.argv[2]) if len(sys.argv) > 2 else 7
    w = workloads.CONFIGS[name]
    Kx, Vx = workloads.make_kv(w.batch, w.n_kv_heads, w.seq, w.seed)
    dK, dV = torch.from_numpy(Kx).cuda(), torch.from_numpy(Vx).cuda()
    cache = binding.KVCompCache(w.batch, w.n_kv_heads, w.n_q_heads, w.seq + 64, w.rel_eb, w.rel_eb, max_code_len=mcl)
    cache.build_codebook(dK, dV)
    cache.compress_blocks(dK, dV)
    q = torch.from_numpy(workloads.make_queries(w.batch, w.n_q_heads, 1, w.seed)[0]).cuda()
    out = torch.empty(w.batch, w.n_q_heads, 128, dtype=torch.float32, device="cuda")
    for _ in range(5):
        cache.attn_decode(q, 1.0 / np.sqrt(128.0), out)
    torch.cuda.synchronize()
    lib = binding.load()
    n = (1 << 15) * 8
    buf = (C.c_ulonglong * n)()
    lib.kvcomp_trace_read.argtypes = [C.c_void_p, C.c_size_t]
    rc = lib.kvcomp_trace_read(buf, n)
    assert rc == 0, rc
    t = np.frombuffer(buf, dtype=np.uint64).reshape(-1, 8).astype(np.int64)
    t = t[t[:, 0] > 0]
    where = t[:, 1].copy()  # point 1: HW_ID register (low half) and accelerator die (high half)
    t[:, 1] = t[:, 0]
    t[:, 5] = t[:, 4]       # point 5: shader clock, not the wall clock
    rel = (t - t[:, 0].min()) * 0.01  # microseconds
    names = ["entry", "(tables, q)", "first K record staged", "first K block done", "first V block done",
             "(all blocks)", "partials written", "exit"]
    print(f"{name}: {len(t)} waves traced, last decode launch")
    for k, nm in enumerate(names):
        if k in (1, 5):
            continue
        col = rel[:, k]
        print("%-22s min %6.2f  p10 %6.2f  median %6.2f  p90 %6.2f  max %6.2f us" %
              (nm, col.min(), np.percentile(col, 10), np.median(col), np.percentile(col, 90), col.max()))
    # placement: waves per SIMD and per CU, and how the last exit of a CU depends on its load
    hw = where & 0xFFFFFFFF
    cu = ((where >> 32) & 15) * 1024 + ((hw >> 13) & 7) * 32 + ((hw >> 12) & 1) * 16 + ((hw >> 8) & 15)
    simd = cu * 4 + ((hw >> 4) & 3)
    ids, per_cu = np.unique(cu, return_counts=True)
    _, per_simd = np.unique(simd, return_counts=True)
    print(f"{len(ids)} CUs in use; waves per CU: " +
          ", ".join(f"{v}: {c} CUs" for v, c in zip(*np.unique(per_cu, return_counts=True))))
    print("waves per SIMD: " + ", ".join(f"{v}: {c}" for v, c in zip(*np.unique(per_simd, return_counts=True))))
    last = np.array([rel[cu == i, 7].max() for i in ids])
    for v in np.unique(per_cu):
        sel = last[per_cu == v]
        print(f"  CUs with {v:2d} waves: last exit median {np.median(sel):6.2f}  max {sel.max():6.2f} us")
    if hasattr(lib, "kvcomp_ticks_read") and w.n_q_heads // w.n_kv_heads >= 4:
        # tile path: shader-clock cycles between points inside the last block pair of every wave
        m = (1 << 15) * 16
        tb = (C.c_ulonglong * m)()
        lib.kvcomp_ticks_read.argtypes = [C.c_void_p, C.c_size_t]
        assert lib.kvcomp_ticks_read(tb, m) == 0
        tk = np.frombuffer(tb, dtype=np.uint64).reshape(-1, 16).astype(np.int64)
        tk = tk[tk[:, 0] > 0]
        steps = ["K weights", "K first half", "K second half + products", "K softmax", "(staging wait)", "V weights",
                 "V first half", "V first products", "V second half + products"]
        for k, nm in enumerate(steps):
            dcol = tk[:, k + 1] - tk[:, k]
            print("%-26s median %7.0f  p90 %7.0f cycles" % (nm, np.median(dcol), np.percentile(dcol, 90)))
        print("%-26s median %7.0f cycles" % ("block pair", np.median(tk[:, 9] - tk[:, 0])))
    cache.close()


if __name__ == "__main__":
    main()
