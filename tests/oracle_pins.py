"""Pins for the CPU oracle: checks against what the paper and the mathematics fix.

Every function takes ``lib`` (a loaded oracle library, None = the committed
one) and raises AssertionError when the oracle disagrees with

  * the hand-derived worked examples under tests/golden/,
  * exact rational arithmetic (tests/exact_ref.py) on small tensors,
  * library routines in the special cases that reduce to them
    (numpy min/max, numpy rint/clip, torch's bfloat16 conversion),
  * invariants that follow from Eq. 1, 2, 6 (code range, end codes,
    monotonicity, half-step error bound, idempotence, equivariances,
    collapse to layer-wise, power-of-two covariance).

``test_oracle_pins.py`` runs them on the real oracle; ``test_oracle_mutants.py``
runs them on copies of the oracle with one planted mistake each and expects a
failure, which shows the set is tight enough to notice such mistakes.
"""
from fractions import Fraction as F

import numpy as np
import torch

import oracle
import workloads
from exact_ref import (f32_to_fraction, real_fakequant, real_prescale, rn_bf16, soft_fakequant,
                       soft_prescale)
from golden_cases import from_storage, load_cases, to_storage


def _eq(a, b, what):
    a = np.asarray(a)
    b = np.asarray(b)
    assert a.shape == b.shape, "%s: shape %s vs %s" % (what, a.shape, b.shape)
    bad = np.nonzero(~(a == b))
    assert bad[0].size == 0, "%s: %d mismatches, first at %s: %r vs %r" % (
        what, bad[0].size, tuple(ix[0] for ix in bad), a[bad][0], b[bad][0])


# ---------------------------------------------------------------------------
# P1: hand-derived worked examples
# ---------------------------------------------------------------------------

def check_golden(lib=None):
    cases = load_cases()
    assert len(cases) >= 9
    for cs in cases:
        name, bits, dt = cs["name"], cs["bits"], cs["dtype"]
        x = to_storage(cs["x"], dt).reshape(cs["shape"])
        if "given_scale" in cs:
            s = cs["given_scale"].astype(np.float32)
            z = cs["given_zero_point"].astype(np.float32)
        else:
            mn, mx = oracle.range_reduce(x, lib)
            _eq(mn, cs["min"].astype(np.float32), name + ": min")
            _eq(mx, cs["max"].astype(np.float32), name + ": max")
            s, z = oracle.prescale(mn, mx, bits, lib)
            _eq(s, cs["scale"].astype(np.float32), name + ": scale")
            _eq(z, cs["zero_point"].astype(np.float32), name + ": zero_point")
            assert not np.any(np.signbit(z) & (z == 0)), name + ": zero_point must not be -0"
        xhat, codes = oracle.fakequant_fwd(x, s, z, bits, lib)
        _eq(codes.ravel(), cs["codes"].astype(np.uint8), name + ": codes")
        _eq(from_storage(xhat).ravel(), cs["xhat"].astype(np.float32), name + ": xhat")
        # backward with dy = 1 + index/8 (bf16-exact for the small cases), mask from the fixture
        dyv = 1.0 + np.arange(x.size) / 8.0
        dy = to_storage(dyv, dt).reshape(cs["shape"])
        dx = oracle.fakequant_bwd(x, dy, s, z, bits, lib)
        _eq(from_storage(dx).ravel(), (dyv * cs["mask"]).astype(np.float32), name + ": dx")
        # the packed gate bits: numpy's little-endian bit packing of the fixture's mask row
        packed = oracle.gate_mask(x, s, z, bits, lib)
        _eq(packed, np.packbits(cs["mask"].astype(np.uint8), bitorder="little"), name + ": packed gate bits")
        _eq(from_storage(oracle.bwd_from_mask(dy, packed, lib)).ravel(),
            (dyv * cs["mask"]).astype(np.float32), name + ": dx from gate bits")


# ---------------------------------------------------------------------------
# P2: exact rational arithmetic
# ---------------------------------------------------------------------------

def check_dyadic_grid_exhaustive(lib=None):
    """Every grid point of dyadic ranges, against the formulas over the rationals.

    Channel = (min, step): max = min + (2^b - 1) * step, values = all multiples
    of 1/8 in [min, max].  step is a power of two, so s = step exactly, x / s is
    exact and nothing is rounded except by the bracket of Eq. 1 / Eq. 2."""
    for bits in (1, 2, 3, 4):
        qmax = 2 ** bits - 1
        chans = [(F(mn8, 8), F(1, 2 ** k)) for mn8 in (-16, -10, -6, -3, 0, 4, 9) for k in (0, 1, 2)]
        length = max(int((qmax * st) * 8) + 1 for _, st in chans)
        vals = []
        for mn, st in chans:
            grid = [mn + F(i, 8) for i in range(int(qmax * st * 8) + 1)]
            grid += [grid[-1]] * (length - len(grid))
            # keep min first and max last, shuffle nothing: order must not matter
            vals.append(grid)
        # layout (N=2, C, HW): split every channel's list over two samples
        half = (length + 1) // 2
        for g in vals:
            g += [g[0]] * (2 * half - len(g))
        x = np.empty((2, len(chans), half), np.float32)
        for c, g in enumerate(vals):
            x[0, c, :] = [float(v) for v in g[:half]]
            x[1, c, :] = [float(v) for v in g[half:]]
        mn, mx = oracle.range_reduce(x, lib)
        s, z = oracle.prescale(mn, mx, bits, lib)
        xhat, codes = oracle.fakequant_fwd(x, s, z, bits, lib)
        dy = np.full(x.shape, 3.0, np.float32)
        dx = oracle.fakequant_bwd(x, dy, s, z, bits, lib)
        for c, (cmin, st) in enumerate(chans):
            es, ez = real_prescale(cmin, cmin + qmax * st, bits)
            assert es == st
            assert f32_to_fraction(mn[c]) == cmin and f32_to_fraction(mx[c]) == cmin + qmax * st
            assert f32_to_fraction(s[c]) == es and f32_to_fraction(z[c]) == ez, (bits, c)
            for n in range(2):
                for k in range(half):
                    q, xh, inr = real_fakequant(f32_to_fraction(x[n, c, k]), es, ez, bits)
                    assert codes[n, c, k] == q, (bits, c, n, k)
                    assert f32_to_fraction(xhat[n, c, k]) == xh, (bits, c, n, k)
                    assert dx[n, c, k] == (3.0 if inr else 0.0), (bits, c, n, k)


def check_tiny_shapes_softfloat(lib=None):
    """All shapes N,C,H,W <= 3 and awkward scales, against per-operation binary32
    rounding done with integers; ranges reduced in Python over (n,h,w)."""
    rng = np.random.default_rng(1234)
    shapes = [(n, c, h, w) for n in (1, 2, 3) for c in (1, 2, 3) for h in (1, 3) for w in (1, 2)]
    for i, shp in enumerate(shapes):
        bits = (1, 2, 3, 4, 5, 8)[i % 6]
        kind = i % 3
        if kind == 0:
            x = rng.integers(-24, 40, size=shp).astype(np.float32) / 8.0
        elif kind == 1:
            x = np.abs(rng.standard_normal(shp)).astype(np.float32) * (10.0 ** rng.uniform(-2, 2))
        else:
            x = rng.standard_normal(shp).astype(np.float32) * 3.0 + 1.0
        mn, mx = oracle.range_reduce(x, lib)
        s, z = oracle.prescale(mn, mx, bits, lib)
        xhat, codes = oracle.fakequant_fwd(x, s, z, bits, lib)
        dy = rng.standard_normal(shp).astype(np.float32)
        dx = oracle.fakequant_bwd(x, dy, s, z, bits, lib)
        for c in range(shp[1]):
            col = [f32_to_fraction(v) for v in x[:, c].ravel()]
            emn, emx = min(col), max(col)
            assert f32_to_fraction(mn[c]) == emn and f32_to_fraction(mx[c]) == emx, (shp, c)
            es, ez = soft_prescale(emn, emx, bits)
            assert f32_to_fraction(s[c]) == es and f32_to_fraction(z[c]) == ez, (shp, c, bits)
            for n in range(shp[0]):
                for h in range(shp[2]):
                    for w in range(shp[3]):
                        q, xh, inr = soft_fakequant(f32_to_fraction(x[n, c, h, w]), es, ez, bits)
                        assert codes[n, c, h, w] == q, (shp, n, c, h, w)
                        assert f32_to_fraction(xhat[n, c, h, w]) == xh, (shp, n, c, h, w)
                        assert dx[n, c, h, w] == (dy[n, c, h, w] if inr else 0.0)


def check_stale_ranges_softfloat(lib=None):
    """Scale / zero-point handed in (not from x): both clamp sides and the mask."""
    rng = np.random.default_rng(99)
    x = (rng.standard_normal((2, 3, 2, 5)) * 4).astype(np.float32)
    s = np.array([0.37, 1.0 / 7.0, 2.5], np.float32)
    z = np.array([3.0, 0.0, -2.0], np.float32)
    for bits in (2, 3, 5):
        xhat, codes = oracle.fakequant_fwd(x, s, z, bits, lib)
        dy = rng.standard_normal(x.shape).astype(np.float32)
        dx = oracle.fakequant_bwd(x, dy, s, z, bits, lib)
        seen = set()
        for idx in np.ndindex(*x.shape):
            c = idx[1]
            q, xh, inr = soft_fakequant(f32_to_fraction(x[idx]), f32_to_fraction(s[c]),
                                        int(z[c]), bits)
            assert codes[idx] == q and f32_to_fraction(xhat[idx]) == xh, (bits, idx)
            assert dx[idx] == (dy[idx] if inr else 0.0), (bits, idx)
            seen.add(inr)
        assert seen == {True, False}


def check_near_ties_softfloat(lib=None):
    """Inputs built to sit on or next to a rounding tie of Eq. 1: x ~ s * (k + 1/2).
    There the code depends on the quotient being the correctly rounded binary32
    one: a reciprocal-multiply, a fused multiply-add or a double-precision
    intermediate moves x / s by an ulp and flips the code.  numpy only searches
    for such inputs; the expected values come from integer arithmetic."""
    rng = np.random.default_rng(77)
    bits = 5
    s_all = (rng.uniform(0.01, 3.0, size=40000)).astype(np.float32)
    k_all = rng.integers(0, 31, size=40000).astype(np.float32)
    x_all = (s_all * (k_all + np.float32(0.5))).astype(np.float32)
    exact = (x_all / s_all)                                        # correctly rounded
    recip = (x_all * (np.float32(1.0) / s_all)).astype(np.float32)
    wide = (x_all.astype(np.float64) / s_all.astype(np.float64))
    pick = np.nonzero((np.rint(exact) != np.rint(recip)) | (np.rint(exact) != np.rint(wide)))[0]
    assert pick.size >= 64, "search found too few near-tie inputs"
    pick = pick[:160]
    c = pick.size
    x = np.stack([x_all[pick], x_all[pick] * np.float32(0.5)], axis=0).reshape(2, c, 1, 1).copy()
    s = s_all[pick].copy()
    z = np.zeros(c, np.float32)
    xhat, codes = oracle.fakequant_fwd(x, s, z, bits, lib)
    dy = np.ones_like(x)
    dx = oracle.fakequant_bwd(x, dy, s, z, bits, lib)
    for n in range(2):
        for j in range(c):
            q, xh, inr = soft_fakequant(f32_to_fraction(x[n, j, 0, 0]), f32_to_fraction(s[j]), 0, bits)
            assert codes[n, j, 0, 0] == q, (n, j, float(x[n, j, 0, 0]), float(s[j]))
            assert f32_to_fraction(xhat[n, j, 0, 0]) == xh
            assert dx[n, j, 0, 0] == (1.0 if inr else 0.0)


# ---------------------------------------------------------------------------
# P4: special cases that reduce to library routines
# ---------------------------------------------------------------------------

def check_minmax_vs_numpy(lib=None):
    rng = np.random.default_rng(5)
    for shp in [(4, 5, 3, 7), (1, 9, 1, 1), (7, 1, 2, 2), (3, 4, 7, 7)]:
        x = rng.standard_normal(shp).astype(np.float32)
        mn, mx = oracle.range_reduce(x, lib)
        _eq(mn, x.min(axis=(0, 2, 3)), "min vs numpy %s" % (shp,))
        _eq(mx, x.max(axis=(0, 2, 3)), "max vs numpy %s" % (shp,))


def check_unit_scale_is_clip_rint(lib=None):
    """min 0 and max 2^b - 1 give s = 1, z = 0: forward = clip(rint(x)) (numpy's
    rint is round-half-to-even)."""
    rng = np.random.default_rng(6)
    for bits in (1, 3, 4, 8):
        qmax = float(2 ** bits - 1)
        x = (rng.uniform(0, qmax, size=(3, 2, 4, 8))).astype(np.float32)
        x[..., 0] = np.arange(2 * 3 * 4).reshape(3, 2, 4) % (qmax + 1) + 0.5   # plant ties
        x = np.minimum(x, qmax).astype(np.float32)
        x[0, :, 0, 1] = 0.0
        x[0, :, 0, 2] = qmax
        mn, mx = oracle.range_reduce(x, lib)
        s, z = oracle.prescale(mn, mx, bits, lib)
        _eq(s, np.ones(2, np.float32), "unit scale")
        _eq(z, np.zeros(2, np.float32), "zero zero-point")
        xhat, codes = oracle.fakequant_fwd(x, s, z, bits, lib)
        want = np.clip(np.rint(x), 0, qmax)
        _eq(xhat, want, "xhat vs clip(rint)")
        _eq(codes, want.astype(np.uint8), "codes vs clip(rint)")


def check_bf16_vs_torch(lib=None):
    """bfloat16 storage: loads widen exactly and stores round to nearest even,
    checked against torch's own float32 <-> bfloat16 conversion."""
    g = torch.Generator().manual_seed(3)
    xt = (torch.randn(3, 4, 5, 6, generator=g) * 3).to(torch.bfloat16)
    xb = xt.view(torch.int16).numpy().view(np.uint16)
    x32 = xt.to(torch.float32).numpy()
    mnb, mxb = oracle.range_reduce(xb, lib)
    _eq(mnb, x32.min(axis=(0, 2, 3)), "bf16 min")
    _eq(mxb, x32.max(axis=(0, 2, 3)), "bf16 max")
    for bits in (3, 8):
        s, z = oracle.prescale(mnb, mxb, bits, lib)
        xh_b, codes_b = oracle.fakequant_fwd(xb, s, z, bits, lib)
        xh_32, codes_32 = oracle.fakequant_fwd(x32, s, z, bits, lib)
        _eq(codes_b, codes_32, "bf16 codes == f32 codes on the same values")
        want = torch.from_numpy(xh_32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        _eq(xh_b, want, "bf16 xhat == torch RNE narrowing of the f32 xhat")
        dyt = torch.randn(3, 4, 5, 6, generator=g).to(torch.bfloat16)
        dyb = dyt.view(torch.int16).numpy().view(np.uint16)
        dxb = oracle.fakequant_bwd(xb, dyb, s, z, bits, lib)
        dx32 = oracle.fakequant_bwd(x32, dyt.to(torch.float32).numpy(), s, z, bits, lib)
        _eq(oracle.f32_from_bf16_bits(dxb), dx32, "bf16 dx")
    # narrowing alone, against integer arithmetic, on values that need rounding
    s = np.array([1.0 / 3.0], np.float32)
    z = np.array([0.0], np.float32)
    q = np.arange(0, 256, dtype=np.float32).reshape(1, 1, 16, 16)
    xq = torch.from_numpy(q * s[0]).to(torch.bfloat16)     # any input that lands on code ~q
    xb = xq.view(torch.int16).numpy().view(np.uint16)
    xh_b, codes = oracle.fakequant_fwd(xb, s, z, 8, lib)
    for cb, hb in zip(codes.ravel(), xh_b.ravel()):
        exact = f32_to_fraction(np.float32(s[0]) * np.float32(cb))
        assert f32_to_fraction(oracle.f32_from_bf16_bits(np.array([hb]))[0]) == rn_bf16(exact)


def check_f16_vs_numpy(lib=None):
    """binary16 storage: the oracle's own widening and round-to-nearest-even narrowing against
    numpy's float16 (an independent implementation) on every binary16 pattern, on every exact
    midpoint between neighbouring binary16 values, around the overflow threshold and the
    subnormal range; then the quantizer on binary16 data against the same values held in binary32."""
    h = np.arange(65536, dtype=np.uint16)
    ref = h.view(np.float16).astype(np.float32)
    got = oracle.f16_widen(h, lib)
    fin = ~np.isnan(ref)
    _eq(got.view(np.uint32)[fin], ref.view(np.uint32)[fin], "binary16 -> binary32")
    assert np.isnan(got[~fin]).all()
    rng = np.random.default_rng(0)
    pos = h[:0x7C00].view(np.float16).astype(np.float64)                     # 0 .. 65504 ascending
    mids = ((pos[:-1] + pos[1:]) / 2).astype(np.float32)                     # exact in binary32
    f = np.concatenate([
        (rng.standard_normal(400000) * np.exp(rng.uniform(-20, 12, 400000))).astype(np.float32),
        mids, np.nextafter(mids, np.float32(0)), np.nextafter(mids, np.float32(np.inf)),
        np.array([65504, 65519.996, 65520, 65536, 1e9, np.inf, 0.0, 2.0 ** -24, 2.0 ** -25,
                  np.nextafter(np.float32(2.0 ** -25), np.float32(1)), 3 * 2.0 ** -25, 2.0 ** -14,
                  2.0 ** -14 - 2.0 ** -25], np.float32)])
    f = np.concatenate([f, -f])
    with np.errstate(over="ignore"):
        want = f.astype(np.float16).view(np.uint16)
    _eq(oracle.f16_narrow(f, lib), want, "binary32 -> binary16, ties to even")
    # the quantizer on binary16 storage
    x16 = (rng.standard_normal((3, 4, 5, 6)) * 3).astype(np.float16)
    x32 = x16.astype(np.float32)
    mn, mx = oracle.range_reduce(x16, lib)
    _eq(mn, x32.min(axis=(0, 2, 3)), "f16 min")
    _eq(mx, x32.max(axis=(0, 2, 3)), "f16 max")
    for bits in (3, 8):
        s, z = oracle.prescale(mn, mx, bits, lib)
        xh16, c16 = oracle.fakequant_fwd(x16, s, z, bits, lib)
        xh32, c32 = oracle.fakequant_fwd(x32, s, z, bits, lib)
        _eq(c16, c32, "f16 codes == f32 codes on the same values")
        _eq(xh16.view(np.uint16), xh32.astype(np.float16).view(np.uint16), "f16 xhat == numpy narrowing of the f32 xhat")
        dy16 = rng.standard_normal((3, 4, 5, 6)).astype(np.float16)
        dx16 = oracle.fakequant_bwd(x16, dy16, s, z, bits, lib)
        dx32 = oracle.fakequant_bwd(x32, dy16.astype(np.float32), s, z, bits, lib)
        _eq(dx16.astype(np.float32), dx32, "f16 dx")


# ---------------------------------------------------------------------------
# P3 / P5: invariants on workload-like tensors
# ---------------------------------------------------------------------------

def _workload_tensor(law, shape, seed):
    return workloads.make_activation(shape, law, (0.05, 20.0), seed).numpy()


def check_invariants(lib=None):
    rng = np.random.default_rng(11)
    for law, shape, bits in [("relu", (8, 16, 32, 32), 3), ("relu", (4, 32, 7, 7), 4),
                             ("linear", (4, 24, 14, 14), 4), ("laplace", (4, 64, 7, 7), 3),
                             ("relu6", (4, 32, 8, 8), 5)]:
        x = _workload_tensor(law, shape, seed=bits)
        if law == "relu":
            x[0, :, 0, 0] = 0.0             # real ReLU outputs contain exact zeros
        qmax = 2 ** bits - 1
        mn, mx = oracle.range_reduce(x, lib)
        s, z = oracle.prescale(mn, mx, bits, lib)
        xhat, codes = oracle.fakequant_fwd(x, s, z, bits, lib)
        sb = s.reshape(1, -1, 1, 1)
        # (a) code range
        assert codes.min() >= 0 and codes.max() <= qmax
        # (b) the channel minimum always maps to code 0
        cmin_codes = np.where(x == mn.reshape(1, -1, 1, 1), codes, 0)
        assert cmin_codes.max() == 0
        # (c) with min == 0 (post-ReLU) the channel maximum maps to the top code
        if law == "relu":
            assert np.all(mn == 0) and np.all(z == 0)
            top = np.where(x == mx.reshape(1, -1, 1, 1), codes, qmax)
            assert top.min() == qmax
        # (d) codes are monotone in x within a channel
        for c in range(shape[1]):
            xs = x[:, c].ravel()
            order = np.argsort(xs, kind="stable")
            assert np.all(np.diff(codes[:, c].ravel()[order].astype(np.int32)) >= 0)
        # (e) half-step error bound wherever the clamp was inactive
        dy = np.ones_like(x)
        mask = oracle.fakequant_bwd(x, dy, s, z, bits, lib)
        assert set(np.unique(mask).tolist()) <= {0.0, 1.0}
        err = np.abs(xhat.astype(np.float64) - x.astype(np.float64))
        bound = 0.5 * sb.astype(np.float64) * (1 + 1e-5) + 1e-30
        assert np.all((err <= bound) | (mask == 0))
        # the clamp only ever bites at the top, by one step at most
        assert np.all(err <= 1.0 * sb.astype(np.float64) * (1 + 1e-5) + 1e-30)
        assert np.all(codes[mask == 0] == qmax)
        assert (mask == 0).mean() < 0.01
        # (f) idempotence with the same (s, z)
        xhat2, codes2 = oracle.fakequant_fwd(xhat, s, z, bits, lib)
        _eq(codes2, codes, "idempotent codes")
        _eq(xhat2, xhat, "idempotent xhat")
        # (g) channel permutation equivariance, batch permutation invariance
        perm = rng.permutation(shape[1])
        xp = np.ascontiguousarray(x[:, perm])
        xh_p, codes_p, s_p, z_p = oracle.fakequant(xp, bits, lib)
        _eq(s_p, s[perm], "perm scale")
        _eq(codes_p, codes[:, perm], "perm codes")
        _eq(xh_p, xhat[:, perm], "perm xhat")
        bperm = rng.permutation(shape[0])
        xh_b, codes_b, s_b, z_b = oracle.fakequant(np.ascontiguousarray(x[bperm]), bits, lib)
        _eq(s_b, s, "batch perm scale")
        _eq(codes_b, codes[bperm], "batch perm codes")
        # (i) scaling the input by 2^k scales the output by 2^k and keeps the codes
        for k in (-3, 5):
            xh_k, codes_k, s_k, z_k = oracle.fakequant((x * np.float32(2.0 ** k)), bits, lib)
            _eq(codes_k, codes, "pow2 codes")
            _eq(xh_k, xhat * np.float32(2.0 ** k), "pow2 xhat")
            _eq(z_k, z, "pow2 zero-point")
        # the packed gate bits are the same gate (numpy's bit packing as the reference layout)
        packed = oracle.gate_mask(x, s, z, bits, lib)
        _eq(packed, np.packbits((mask.ravel() != 0).astype(np.uint8), bitorder="little"), "packed gate bits")
        # (j) backward returns dy or 0, bitwise
        dyr = rng.standard_normal(shape).astype(np.float32)
        dx = oracle.fakequant_bwd(x, dyr, s, z, bits, lib)
        assert np.all((dx == dyr) | (dx == 0))
        _eq(dx, dyr * mask, "dx == dy * mask")
        _eq(oracle.bwd_from_mask(dyr, packed, lib), dx, "backward from gate bits == backward from x")
        # every code value is used somewhere on these wide tensors, in every channel with spread
        assert len(np.unique(codes)) == qmax + 1


def check_collapse_to_layerwise(lib=None):
    """Channels that all contain the same extremes: per-channel == per-layer."""
    x = _workload_tensor("linear", (3, 6, 5, 5), seed=2)
    x = np.clip(x, -4.0, 9.0)
    x[0, :, 0, 0] = -4.0
    x[1, :, 2, 3] = 9.0
    for bits in (3, 4):
        xh_c, codes_c, s_c, z_c = oracle.fakequant(x, bits, lib)
        flat = x.reshape(1, 1, 1, -1)
        xh_l, codes_l, s_l, z_l = oracle.fakequant(flat, bits, lib)
        assert np.all(s_c == s_l[0]) and np.all(z_c == z_l[0])
        _eq(codes_c.ravel(), codes_l.ravel(), "collapse codes")
        _eq(xh_c.ravel(), xh_l.ravel(), "collapse xhat")


def check_per_sample_view(lib=None):
    """Ranges per sample and channel (the paper's C x H x W tensor without a
    batch) are the batch-level call on the (1, N*C, H, W) view."""
    x = _workload_tensor("relu", (3, 4, 5, 5), seed=8)
    xh_v, codes_v, s_v, z_v = oracle.fakequant(x.reshape(1, 12, 5, 5), 3, lib)
    for n in range(3):
        xh_n, codes_n, s_n, z_n = oracle.fakequant(x[n:n + 1].copy(), 3, lib)
        _eq(s_n, s_v[n * 4:(n + 1) * 4], "per-sample scale")
        _eq(codes_n.ravel(), codes_v.reshape(3, -1)[n], "per-sample codes")


def check_error_halves_per_bit(lib=None):
    x = _workload_tensor("relu", (8, 16, 16, 16), seed=4)
    prev = None
    for bits in range(2, 9):
        xh, _, s, _ = oracle.fakequant(x, bits, lib)
        rel = np.linalg.norm((xh - x).astype(np.float64)) / np.linalg.norm(x.astype(np.float64))
        if prev is not None:
            assert 0.35 < rel / prev < 0.65, (bits, rel, prev)
        prev = rel


def check_channelwise_beats_layerwise(lib=None):
    """Direction of the paper's Table 2 on channels with very different spreads:
    per-channel ranges give higher cosine similarity and lower relative error."""
    x = _workload_tensor("relu", (8, 16, 32, 32), seed=0)
    xd = x.astype(np.float64).ravel()

    def metrics(xh):
        q = xh.astype(np.float64).ravel()
        return (xd @ q) / (np.linalg.norm(xd) * np.linalg.norm(q)), \
            np.linalg.norm(xd - q) / np.linalg.norm(xd)

    xh_c = oracle.fakequant(x, 3, lib)[0]
    xh_l = oracle.fakequant(x.reshape(1, 1, 1, -1), 3, lib)[0]
    cos_c, rel_c = metrics(xh_c)
    cos_l, rel_l = metrics(xh_l)
    assert cos_c > cos_l and rel_c < rel_l
    # per channel the gap is large: small-sigma channels are wiped out layer-wise
    per_c = np.linalg.norm((xh_c - x).reshape(8, 16, -1).transpose(1, 0, 2).reshape(16, -1), axis=1)
    per_l = np.linalg.norm((xh_l.reshape(x.shape) - x).reshape(8, 16, -1).transpose(1, 0, 2)
                           .reshape(16, -1), axis=1)
    assert np.all(per_c <= per_l * (1 + 1e-6))


def check_accumulation_forms(lib=None):
    """Eq. 3 (scale inside the loop) and Eq. 6 (pre-scaled) compute the same sum.
    On dyadic data both are exact and equal to the rational sum; on general data
    they agree with a float64 einsum to rounding."""
    # dyadic: s in {1/2, 1, 2}, integer z, weights multiples of 1/4
    rng = np.random.default_rng(21)
    n, c, hw = 2, 5, 6
    codes = rng.integers(0, 8, size=(n, c, hw)).astype(np.uint8)
    s = np.array([0.5, 1, 2, 0.25, 1], np.float32)
    z = np.array([0, 2, 3, 1, 7], np.float32)
    w = np.array([0.25, -1.5, 2, 0.75, -0.5], np.float32)
    xhat = (s.reshape(1, c, 1) * (codes.astype(np.float32) - z.reshape(1, c, 1))).astype(np.float32)
    y3 = oracle.accumulate_inloop(codes, s, z, w, lib)
    y6 = oracle.accumulate_prescaled(xhat, w, lib)
    for i in range(n):
        for k in range(hw):
            exact = sum(F(float(w[j])) * F(float(s[j])) * (int(codes[i, j, k]) - int(z[j]))
                        for j in range(c))
            assert F(float(y3[i, k])) == exact and F(float(y6[i, k])) == exact
    # general
    x = _workload_tensor("linear", (3, 12, 4, 4), seed=5)
    xh, cd, s, z = oracle.fakequant(x, 4, lib)
    w = rng.standard_normal(12).astype(np.float32)
    y3 = oracle.accumulate_inloop(cd, s, z, w, lib)
    y6 = oracle.accumulate_prescaled(xh, w, lib)
    ref = np.einsum("c,nchw->nhw", w.astype(np.float64), xh.astype(np.float64))
    scale = np.abs(w).astype(np.float64) @ np.abs(xh.astype(np.float64)).max(axis=(0, 2, 3))
    assert np.max(np.abs(y3 - ref)) <= 1e-5 * scale
    assert np.max(np.abs(y6 - ref)) <= 1e-5 * scale


def check_distortion_metrics(lib=None):
    """Table 2's cosine similarity and relative error against numpy's dot / norm on the
    oracle's own x_hat, exact cases, and the direction of the table."""
    x = _workload_tensor("linear", (4, 6, 9, 9), seed=12)
    mn, mx = oracle.range_reduce(x, lib)
    for bits in (3, 6):
        s, z = oracle.prescale(mn, mx, bits, lib)
        xh, _ = oracle.fakequant_fwd(x, s, z, bits, lib)
        ch, layer = oracle.distortion(x, s, z, bits, lib)
        xd, qd = x.astype(np.float64), xh.astype(np.float64)
        for c in range(6):
            a, b = xd[:, c].ravel(), qd[:, c].ravel()
            want = np.array([a @ b, a @ a, b @ b, (a - b) @ (a - b)])
            assert np.allclose(ch[c], want, rtol=1e-12, atol=0), (bits, c, ch[c], want)
        assert np.allclose(layer[:4], ch.sum(axis=0), rtol=1e-13)
        cos = (xd.ravel() @ qd.ravel()) / (np.linalg.norm(xd.ravel()) * np.linalg.norm(qd.ravel()))
        rel = np.linalg.norm((xd - qd).ravel()) / np.linalg.norm(xd.ravel())
        assert abs(layer[4] - cos) <= 1e-12 and abs(layer[5] - rel) <= 1e-12 * max(rel, 1e-30)
        assert 0 < layer[5] < 1 and 0 < layer[4] <= 1
    # exact: a tensor that is already on the grid has cosine 1 and error 0
    g = np.arange(16, dtype=np.float32).reshape(1, 1, 4, 4)
    ch, layer = oracle.distortion(g, np.ones(1, np.float32), np.zeros(1, np.float32), 4, lib)
    assert layer[3] == 0.0 and layer[5] == 0.0 and layer[4] == 1.0
    assert ch[0, 0] == ch[0, 1] == ch[0, 2] == float((np.arange(16.0) ** 2).sum())
    # hand case: x = (1, 2.4) with s = 1, z = 0, b = 3 -> q = (1, 2): x.q = 5.8, x.x = 6.76,
    # q.q = 5, |x-q|^2 = 0.16 (up to the binary32 representation of 2.4)
    h = np.array([1.0, 2.4], np.float32).reshape(1, 1, 1, 2)
    ch, layer = oracle.distortion(h, np.ones(1, np.float32), np.zeros(1, np.float32), 3, lib)
    x24 = float(np.float32(2.4))
    assert np.allclose(ch[0], [1 + 2 * x24, 1 + x24 * x24, 5.0, (x24 - 2) ** 2], rtol=1e-15)
    assert abs(layer[4] - (1 + 2 * x24) / np.sqrt((1 + x24 * x24) * 5.0)) < 1e-15
    assert abs(layer[5] - (x24 - 2) / np.sqrt(1 + x24 * x24)) < 1e-15
    # direction of Table 2: channel-wise ranges distort less than one range per layer
    xr = _workload_tensor("relu", (8, 16, 16, 16), seed=0)
    s, z = oracle.prescale(*oracle.range_reduce(xr, lib), 3, lib)
    _, lay_c = oracle.distortion(xr, s, z, 3, lib)
    flat = xr.reshape(1, 1, 1, -1)
    sl, zl = oracle.prescale(*oracle.range_reduce(flat, lib), 3, lib)
    _, lay_l = oracle.distortion(flat, sl, zl, 3, lib)
    assert lay_c[4] > lay_l[4] and lay_c[5] < lay_l[5]


def check_integer_accumulation(lib=None):
    """Eq. 3 with the scale folded into int8 weights: the integer sum against numpy's integer
    einsum, the fold against its defining properties, and the whole against Eq. 6 within the
    bound that the rounding of the folded weights allows."""
    rng = np.random.default_rng(31)
    x = _workload_tensor("linear", (3, 16, 5, 4), seed=7)
    xh, codes, s, z = oracle.fakequant(x, 4, lib)
    w = (rng.standard_normal((6, 16)) * rng.uniform(0.1, 3, size=(6, 1))).astype(np.float32)
    w[4] = 0.0
    wq, corr, a = oracle.fold_weights(w, s, z, lib)
    ws = (w * s.reshape(1, -1)).astype(np.float32)
    assert wq.dtype == np.int8 and np.abs(wq.astype(np.int32)).max() <= 127
    live = [0, 1, 2, 3, 5]
    assert np.all(np.abs(wq[live].astype(np.int32)).max(axis=1) == 127)      # the largest entry maps to +-127
    assert np.all(wq[4] == 0) and a[4] == 1.0 and corr[4] == 0
    _eq(a[live], (np.abs(ws[live]).max(axis=1) / np.float32(127)).astype(np.float32), "row step")
    assert np.all(np.abs(a.reshape(-1, 1) * wq - ws) <= 0.5 * a.reshape(-1, 1) * (1 + 1e-6))
    _eq(corr, wq.astype(np.int64) @ z.astype(np.int64), "zero-point correction")
    # integer sum: numpy's int64 einsum is exact
    y = oracle.conv1x1_int8(codes, wq, corr, a, lib)
    acc = np.einsum("oc,nchw->nohw", wq.astype(np.int64), codes.astype(np.int64)) - corr.reshape(1, -1, 1, 1)
    _eq(y, (a.reshape(1, -1, 1, 1) * acc.astype(np.float32)).astype(np.float32), "int8 convolution")
    # against Eq. 6 (float weights on x_hat): off by at most the weight rounding times |code - z|
    ref = np.einsum("oc,nchw->nohw", w.astype(np.float64), xh.astype(np.float64))
    bound = 0.5 * a.astype(np.float64).reshape(1, -1, 1, 1) * \
        np.abs(codes.astype(np.float64) - z.reshape(1, -1, 1, 1)).sum(axis=1, keepdims=True)
    assert np.all(np.abs(y - ref) <= bound * (1 + 1e-4) + 1e-4 * np.abs(ref).max())
    # a dyadic case that is exact end to end: w = +-1, 127 entries per row irrelevant -> use s = 1
    codes2 = rng.integers(0, 8, size=(2, 4, 3, 3)).astype(np.uint8)
    w2 = np.array([[127, -127, 64, 0], [1, 2, 3, 127]], np.float32)
    wq2, corr2, a2 = oracle.fold_weights(w2, np.ones(4, np.float32), np.array([0, 1, 2, 3], np.float32), lib)
    _eq(wq2, w2.astype(np.int8), "integer weights fold to themselves")
    _eq(a2, np.ones(2, np.float32), "unit step")
    y2 = oracle.conv1x1_int8(codes2, wq2, corr2, a2, lib)
    want2 = np.einsum("oc,nchw->nohw", w2.astype(np.int64), codes2.astype(np.int64) - np.arange(4).reshape(1, 4, 1, 1))
    _eq(y2, want2.astype(np.float32), "exact integer case")


def check_large_zero_point_term(lib=None):
    """A channel range far from zero ([1000, 1001] at 4 bits: z = -15000) over many channels:
    the zero-point term of Eq. 3 exceeds 32 bits and must still be exact."""
    c = 2048
    s = np.full(c, 1.0 / 15.0, np.float32)
    z = np.full(c, -15000.0, np.float32)
    w = np.full((2, c), 1.0, np.float32)
    w[1] = -1.0
    wq, corr, a = oracle.fold_weights(w, s, z, lib)
    assert np.all(wq[0] == 127) and np.all(wq[1] == -127)
    assert corr[0] == 127 * -15000 * c and corr[1] == -127 * -15000 * c and abs(int(corr[0])) > 2 ** 31
    codes = np.full((1, c, 1, 2), 3, np.uint8)
    codes[0, :, 0, 1] = 12
    y = oracle.conv1x1_int8(codes, wq, corr, a, lib)
    exact = np.array([[127 * c * (3 + 15000), 127 * c * (12 + 15000)], [-127 * c * (3 + 15000), -127 * c * (12 + 15000)]], np.int64)
    _eq(y.reshape(2, 2), (a.reshape(2, 1) * exact.astype(np.float32)).astype(np.float32), "zero-point term beyond 32 bits")


def check_packed_codes(lib=None):
    """Two codes per byte: a hand-written example, the round trip on random codes of every
    width up to four bits and odd counts, and the layout against numpy bit operations."""
    _eq(oracle.pack4(np.array([0, 7, 3, 5, 1], np.uint8), lib), np.array([0x70, 0x53, 0x01], np.uint8), "hand-packed example")
    _eq(oracle.unpack4(np.array([0x70, 0x53, 0x01], np.uint8), 5, lib), np.array([0, 7, 3, 5, 1], np.uint8), "hand-unpacked example")
    rng = np.random.default_rng(5)
    for bits in (1, 2, 3, 4):
        for total in (1, 2, 7, 64, 1001):
            codes = rng.integers(0, 2 ** bits, size=total).astype(np.uint8)
            packed = oracle.pack4(codes, lib)
            assert packed.size == (total + 1) // 2
            padded = np.concatenate([codes, np.zeros(total % 2, np.uint8)])
            _eq(packed, padded[0::2] | (padded[1::2] << 4), "nibble layout")
            _eq(oracle.unpack4(packed, total, lib), codes, "round trip")
    # on a quantized tensor: the packed codes are the forward's codes, nothing else
    x = _workload_tensor("linear", (2, 5, 3, 3), seed=9)
    _, codes, _, _ = oracle.fakequant(x, 4, lib)
    _eq(oracle.unpack4(oracle.pack4(codes, lib), codes.size, lib), codes.ravel(), "codes of a tensor")


def check_float_convolution(lib=None):
    """Eq. 6's accumulation with a full weight matrix: a hand-worked case, exact rational sums on
    dyadic data, identity and permutation weights, numpy's float64 einsum, the one-weight-per-
    channel sum it reduces to, Eq. 3's sum from the codes, and 16-bit storage."""
    # by hand: x_hat (1,2,1,2) = [[1, 2], [3, 4]] (channel rows), w = [[1, 10], [0.5, -1]]
    xh = np.array([[[[1.0, 2.0]], [[3.0, 4.0]]]], np.float32)
    w = np.array([[1.0, 10.0], [0.5, -1.0]], np.float32)
    y = oracle.conv1x1_float(xh, w, lib)
    assert y.shape == (1, 2, 1, 2) and y.dtype == np.float64
    _eq(y.ravel(), np.array([31.0, 42.0, -2.5, -3.0]), "hand-worked 2x2")
    # dyadic values: every partial sum is exact, so the result is the rational sum
    rng = np.random.default_rng(33)
    n, c, hw, o = 2, 5, 3, 4
    xh = (rng.integers(-64, 64, size=(n, c, hw)) / 8.0).astype(np.float32)
    w = (rng.integers(-32, 32, size=(o, c)) / 4.0).astype(np.float32)
    y = oracle.conv1x1_float(xh, w, lib)
    for i in range(n):
        for j in range(o):
            for k in range(hw):
                exact = sum(F(float(w[j, q])) * F(float(xh[i, q, k])) for q in range(c))
                assert F(float(y[i, j, k])) == exact
    # identity weights return x_hat, a permutation matrix permutes the channels, exactly
    x = _workload_tensor("linear", (3, 6, 4, 5), seed=4)
    xh, cd, s, z = oracle.fakequant(x, 4, lib)
    _eq(oracle.conv1x1_float(xh, np.eye(6, dtype=np.float32), lib), xh.astype(np.float64), "identity")
    perm = np.array([3, 0, 5, 1, 4, 2])
    _eq(oracle.conv1x1_float(xh, np.eye(6, dtype=np.float32)[perm], lib), xh[:, perm].astype(np.float64), "permutation")
    # numpy's own contraction in float64 (another summation order: equal to rounding)
    w = rng.standard_normal((7, 6)).astype(np.float32)
    y = oracle.conv1x1_float(xh, w, lib)
    ref = np.einsum("oc,nchw->nohw", w.astype(np.float64), xh.astype(np.float64))
    mag = np.einsum("oc,nchw->nohw", np.abs(w).astype(np.float64), np.abs(xh).astype(np.float64))
    assert np.all(np.abs(y - ref) <= 8 * 2.0 ** -53 * mag)
    # one output row is the one-weight-per-channel sum of Eq. 6 (binary32 there: to its rounding)
    y6 = oracle.accumulate_prescaled(xh, w[2], lib)
    assert np.all(np.abs(y6 - y[:, 2]) <= 8 * 2.0 ** -24 * mag[:, 2])
    # Eq. 3 from the codes, sum_c w s_c (q - z_c), is the same sum: x_hat = s_c (q - z_c) rounded once
    deq = s.astype(np.float64).reshape(1, -1, 1, 1) * (cd.astype(np.float64) - z.astype(np.float64).reshape(1, -1, 1, 1))
    y3 = np.einsum("oc,nchw->nohw", w.astype(np.float64), deq)
    assert np.all(np.abs(y - y3) <= 2.0 ** -23 * mag)
    # linear in the weights
    w2 = rng.standard_normal((7, 6)).astype(np.float32)
    both = oracle.conv1x1_float(xh, (w + w2).astype(np.float32), lib)
    wsum = (w + w2).astype(np.float32).astype(np.float64)
    assert np.all(np.abs(both - np.einsum("oc,nchw->nohw", wsum, xh.astype(np.float64))) <= 8 * 2.0 ** -53 * 4 * mag + 1e-300)
    # 16-bit storage: the stored values widen exactly, the sum is over the widened values
    xb = (xh.view(np.uint32) >> 16).astype(np.uint16)      # truncated to bfloat16: any bfloat16 values do
    wb = (w.view(np.uint32) >> 16).astype(np.uint16)
    yb = oracle.conv1x1_float(xb, wb, lib)
    refb = np.einsum("oc,nchw->nohw", oracle.f32_from_bf16_bits(wb).astype(np.float64),
                     oracle.f32_from_bf16_bits(xb).astype(np.float64))
    assert np.all(np.abs(yb - refb) <= 8 * 2.0 ** -53 * mag * 1.1)
    xf, wf = xh.astype(np.float16), w.astype(np.float16)
    yf = oracle.conv1x1_float(xf, wf, lib)
    reff = np.einsum("oc,nchw->nohw", wf.astype(np.float64), xf.astype(np.float64))
    assert np.all(np.abs(yf - reff) <= 8 * 2.0 ** -53 * mag * 1.1)


ALL_CHECKS = [
    check_golden,
    check_dyadic_grid_exhaustive,
    check_tiny_shapes_softfloat,
    check_stale_ranges_softfloat,
    check_near_ties_softfloat,
    check_minmax_vs_numpy,
    check_unit_scale_is_clip_rint,
    check_bf16_vs_torch,
    check_f16_vs_numpy,
    check_invariants,
    check_collapse_to_layerwise,
    check_per_sample_view,
    check_error_halves_per_bit,
    check_channelwise_beats_layerwise,
    check_accumulation_forms,
    check_distortion_metrics,
    check_integer_accumulation,
    check_large_zero_point_term,
    check_packed_codes,
    check_float_convolution,
]
