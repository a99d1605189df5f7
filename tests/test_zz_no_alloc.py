"""kvcomp_baseline_fp16_attn_noalloc, the entry point for callers that cannot allocate: it keeps the split tickets and
partials of the fp16 comparison kernel in a static device array of the library instead of a caller's workspace.  Its
output is checked against the workspace entry point's (and the oracle's attention on the raw fp16 values) on two calls
in a row, the second with a smaller input, and its size limit is checked from the host."""
import ctypes as C
import sys

import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu
SCALE = 1.0 / np.sqrt(128.0)


def _dev(x):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0")


def _close(got, ref):
    ref = np.asarray(ref, np.float64)
    err = np.abs(got.astype(np.float64) - ref).max()
    tol = 1e-3 * max(1.0, np.abs(ref).max())
    assert np.isfinite(got).all() and err <= tol, f"max abs err {err:.3e} > {tol:.3e}"
    return err


def test_no_alloc_entry_point_matches_the_workspace_entry_point(oracle):
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2509_00579_amd import binding
    binding.load()
    # the first call with groups of 4 query heads and many splits, the second smaller in every dimension (fewer
    # tickets, fewer and shorter partials: it runs on what the first call left in the array), then the first again
    cases = [(2, 2, 8, 3000, 0), (1, 2, 2, 500, 3), (2, 2, 8, 3000, 7), (1, 1, 8, 64, 0)]
    for B, H, Hq, S, n_splits in cases:
        print(f"no-alloc fp16 attention B={B} H={H} Hq={Hq} S={S} n_splits={n_splits}", flush=True)
        sys.stdout.flush()
        Kx, Vx = W.make_kv(B, H, S, 91)
        q = W.make_queries(B, Hq, 1, 91)[0]
        dK, dV, dq = _dev(Kx), _dev(Vx), _dev(q)
        base = binding.BaselineFp16Attention(B, H, Hq)
        want = base(dK, dV, dq, SCALE, n_splits=n_splits).cpu().numpy()
        out = torch.full((B, Hq, 128), float("nan"), dtype=torch.float32, device="cuda:0")
        got = base.noalloc(dK, dV, dq, SCALE, out, n_splits=n_splits).cpu().numpy()
        _close(got, want)
        np.testing.assert_array_equal(got, want)   # same kernel, same splits, same merge order
        G = Hq // H
        ref = np.zeros((B, Hq, 128))
        for b in range(B):
            for hq in range(Hq):
                ref[b, hq] = oracle.attention_head(Kx[b, :, hq // G], Vx[b, :, hq // G], q[b, hq], SCALE)
        _close(got, ref)
    # beyond the static array: refused on the host, nothing is launched (the pointers are never used)
    lib = binding.load()
    dummy = torch.zeros(64, dtype=torch.float16, device="cuda:0")
    out = torch.zeros(64, dtype=torch.float32, device="cuda:0")
    ptr, optr = C.c_void_p(dummy.data_ptr()), C.c_void_p(out.data_ptr())
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    big = binding.make_config(64, 8, 64, 1 << 20, 0.01, 0.01)        # 4096 query-head rows x 128 splits x 520 B
    assert lib.kvcomp_baseline_fp16_attn_noalloc(C.byref(big), ptr, ptr, 1 << 20, ptr, 1.0, optr, 128, stream) == binding.ERR_CAPACITY
    many = binding.make_config(4096, 8, 8, 64, 0.01, 0.01)           # 32768 (batch, kv head) pairs
    assert lib.kvcomp_baseline_fp16_attn_noalloc(C.byref(many), ptr, ptr, 64, ptr, 1.0, optr, 1, stream) == binding.ERR_CAPACITY
    assert b"static scratch" in lib.kvcomp_last_error()
    torch.cuda.synchronize()
