"""The store kernels form the quantizer's quotient as (x - min) * rcp(width), round it by adding 2^23, and redo it with
the correctly rounded division only when the product lies within 2^-12 of k + 1/2, which they test as
(q - rint(q))^2 > (1/2 - 2^-12)^2 (csrc/tile_quant.cuh, quant_codes).  This checks the
error analysis behind that rule on the CPU, in numpy binary32: for every reciprocal within 1 ulp of the exact one
(the accuracy of v_rcp_f32), a product that is NOT near a rounding boundary rounds to the same integer as the
correctly rounded quotient (numpy's binary32 division), on random fp16-grid inputs and on quotients constructed
right next to every k + 1/2.  The bit-exact parity of the codes themselves is a GPU test."""
import numpy as np

FAR_SQ = (np.float32(0.5) - np.float32(2.0 ** -12)) * (np.float32(0.5) - np.float32(2.0 ** -12))
MAGIC = np.float32(2.0 ** 23)


def _mismatches(d, step):
    bad = near_any = 0
    with np.errstate(all="ignore"):
        q_exact = (d / step).astype(np.float32)
        inv0 = (np.float32(1.0) / step).astype(np.float32)
        for direction in (-np.inf, None, np.inf):
            inv = inv0 if direction is None else np.nextafter(inv0, np.float32(direction))
            q = (d * inv).astype(np.float32)
            r = (q + MAGIC).astype(np.float32)                  # the kernel's rounding: the sum's low bits are the code
            k_fast = r.view(np.uint32).astype(np.int64) - 0x4B000000
            off = (q - (r - MAGIC)).astype(np.float32)
            near = ~((off * off).astype(np.float32) <= FAR_SQ)  # NaN counts as near
            keep = ~near & (q_exact < 300)
            bad += int((k_fast[keep] != np.rint(q_exact)[keep].astype(np.int64)).sum())
            near_any += int(near.sum())
    return bad, near_any


def test_product_rounds_like_the_quotient_away_from_boundaries():
    rng = np.random.default_rng(1)
    n = 3_000_000
    mn = (rng.standard_normal(n) * rng.choice([1, 10, 0.01], n)).astype(np.float16).astype(np.float32)
    span = np.abs(rng.standard_normal(n) * rng.choice([1, 10, 0.001], n)).astype(np.float32) + np.float32(1e-4)
    mx = (mn + span).astype(np.float16).astype(np.float32)
    x = (mn + rng.random(n).astype(np.float32) * (mx - mn)).astype(np.float16).astype(np.float32)
    x = np.minimum(np.maximum(x, mn), mx)
    rel = rng.choice([5e-3, 1e-2, 2e-2, 1 / 510, 0.0371, 0.25], n).astype(np.float32)
    ok = mx > mn
    step = (np.float32(2.0) * rel * (mx - mn))[ok]
    bad, _ = _mismatches((x - mn)[ok], step)
    assert bad == 0


def test_quotients_next_to_every_half_integer():
    rng = np.random.default_rng(2)
    for k in range(256):
        step = np.float32((rng.random() + 0.5) * 2.0 ** int(rng.integers(-20, 4)))
        centre = np.float32(k + 0.5) * step
        up, down = [centre], [centre]
        for _ in range(40):
            up.append(np.nextafter(up[-1], np.float32(np.inf)))
            down.append(np.nextafter(down[-1], np.float32(-np.inf)))
        d = np.array(up + down[1:], np.float32)
        bad, near = _mismatches(d, np.full_like(d, step))
        assert bad == 0 and near > 0   # the neighbourhood is recognised as such, everything outside agrees
