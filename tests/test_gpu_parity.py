"""HIP library vs CPU oracle, element by element, through the C ABI (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_18339_amd as G
import workloads
from golden_cases import load_cases
from parity import assert_parity, gpu_path, oracle_path, to_numpy

pytestmark = pytest.mark.gpu

DEV = "cuda"


def _loaded_native_library():
    with open("/proc/self/maps") as fh:
        return any("libgranq.so" in line for line in fh)


def test_native_library_is_what_runs():
    G.load()
    assert _loaded_native_library(), "libgranq.so is not mapped into this process"
    assert torch.cuda.is_available()


def _check(x, bits, seed=0, desc=None, view_shape=None, what=""):
    dy = workloads.make_grad(x.shape, seed, x.device, x.dtype)
    got = gpu_path(x, bits, dy, desc=desc)
    want = oracle_path(to_numpy(x), bits, to_numpy(dy), view_shape=view_shape)
    assert_parity(got, want, what)
    return got, want


def test_config1_resnet20_first_layer():
    wl = workloads.resnet20_first_layer()
    a = wl.acts[0]
    x = workloads.make_activation(a.shape(wl.batch), a.law, wl.sigma, 0, DEV)
    got, want = _check(x, 3, 0, what="config1")
    assert np.all(got["min"] >= 0)
    assert got["codes"].max() == 7


# Shapes chosen to span several column tiles (2048 elements per tile), ragged
# last tiles, channels straddling tiles and vectors, tiny and unit dimensions.
SMALL = [
    (8, 16, 32, 32), (5, 37, 9, 8), (6, 100, 7, 7), (3, 40, 1, 1), (9, 24, 14, 14), (4, 3000, 1, 1),
    (1, 1, 1, 16384), (2, 1, 5, 4), (1, 64, 1, 1152), (7, 12, 14, 14), (1, 2048, 7, 7), (13, 8, 7, 7),
    (17, 520, 2, 2), (4, 4, 64, 65), (1, 1, 1, 4), (1, 4, 1, 1), (31, 8, 1, 3),
    # more rows than the grid's second dimension holds (row groups are capped at 65535)
    (200001, 4, 1, 4), (70001, 3, 2, 2),
    # no 16-byte structure: element-wise kernels
    (2, 3, 7, 7), (5, 7, 3, 3), (1, 1, 1, 5), (3, 1, 7, 3), (1, 1, 1, 1), (2, 5, 1, 1), (4, 9, 5, 5),
]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16], ids=["f32", "bf16", "f16"])
@pytest.mark.parametrize("shape", SMALL, ids=lambda s: "x".join(map(str, s)))
def test_small_shapes(shape, dtype):
    for i, (law, bits) in enumerate([("relu", 3), ("linear", 4), ("laplace", 8), ("relu6", 1)]):
        x = workloads.make_activation(shape, law, (0.05, 20.0), seed=i, device=DEV, dtype=dtype)
        _check(x, bits, i, what="%s %s b%d" % (shape, law, bits))


@pytest.mark.parametrize("bits", range(1, 9))
def test_every_bit_width(bits):
    x = workloads.make_activation((6, 20, 12, 12), "linear", (0.05, 20.0), seed=bits, device=DEV)
    got, _ = _check(x, bits, bits, what="bits=%d" % bits)
    assert got["codes"].max() == 2 ** bits - 1 and got["codes"].min() == 0


def test_golden_examples_on_gpu():
    """The hand-derived worked examples, through the HIP library."""
    for cs in load_cases():
        shape = cs["shape"]
        dt = torch.float32 if cs["dtype"] == "f32" else torch.bfloat16
        x = torch.tensor(cs["x"], dtype=torch.float32).reshape(shape).to(dt).to(DEV)
        dyv = 1.0 + np.arange(x.numel()) / 8.0
        dy = torch.tensor(dyv, dtype=torch.float32).reshape(shape).to(dt).to(DEV)
        kw = {}
        if "given_scale" in cs:
            kw = dict(scale=cs["given_scale"].astype(np.float32), zero_point=cs["given_zero_point"].astype(np.float32))
        got = gpu_path(x, cs["bits"], dy, **kw)
        name = cs["name"]
        if not kw:
            assert np.array_equal(got["min"], cs["min"].astype(np.float32)), name
            assert np.array_equal(got["max"], cs["max"].astype(np.float32)), name
            assert np.array_equal(got["scale"], cs["scale"].astype(np.float32)), name
            assert np.array_equal(got["zero_point"], cs["zero_point"].astype(np.float32)), name
            assert not np.any(np.signbit(got["zero_point"]) & (got["zero_point"] == 0)), name
        assert np.array_equal(got["codes"].ravel(), cs["codes"].astype(np.uint8)), name
        from parity import values
        assert np.array_equal(values(got["xhat"]).ravel(), cs["xhat"].astype(np.float32)), name
        assert np.array_equal(values(got["dx"]).ravel(), (dyv * cs["mask"]).astype(np.float32)), name


def test_stale_ranges_clamp_both_sides():
    """Scale / zero-point from another tensor: both clamp sides and the gate are exercised."""
    for dtype in (torch.float32, torch.bfloat16, torch.float16):
        ref = workloads.make_activation((4, 24, 14, 14), "linear", (0.5, 2.0), seed=1, device=DEV, dtype=dtype)
        x = workloads.make_activation((4, 24, 14, 14), "linear", (0.5, 6.0), seed=2, device=DEV, dtype=dtype)
        dy = workloads.make_grad(x.shape, 3, DEV, dtype)
        base = gpu_path(ref, 4)
        got = gpu_path(x, 4, dy, scale=base["scale"], zero_point=base["zero_point"])
        want = oracle_path(to_numpy(x), 4, to_numpy(dy), scale=base["scale"], zero_point=base["zero_point"])
        assert_parity(got, want, "stale ranges")
        from parity import values
        gated = (values(got["dx"]) == 0) & (values(to_numpy(dy)) != 0)
        assert 0.01 < gated.mean() < 0.9
        assert (got["codes"] == 0).any() and (got["codes"] == 15).any()


def test_dead_and_constant_channels():
    x = workloads.make_activation((4, 8, 7, 8), "relu", (0.05, 20.0), seed=5, device=DEV)
    x[:, 2] = 0.0
    x[:, 5] = 2.5
    x[:, 6] = -1e-30
    got, want = _check(x, 4, 5, what="degenerate")
    assert got["scale"][2] == 1.0 and got["zero_point"][2] == 0.0
    assert np.all(got["xhat"][:, 2] == 0) and np.all(got["codes"][:, 2] == 0)
    assert got["scale"][5] == 1.0 and np.all(got["xhat"][:, 5] == 2.0)


def test_subnormal_and_huge_values():
    x = torch.empty(2, 4, 4, 4, device=DEV)
    g = torch.Generator(device=DEV).manual_seed(0)
    x[:, 0] = torch.rand(2, 4, 4, generator=g, device=DEV) * 1e-38          # subnormal range
    x[:, 1] = torch.rand(2, 4, 4, generator=g, device=DEV) * 1e-36
    x[:, 2] = (torch.rand(2, 4, 4, generator=g, device=DEV) - 0.5) * 1e37   # range near overflow
    x[:, 3] = torch.rand(2, 4, 4, generator=g, device=DEV) * 1e-44
    _check(x, 4, 0, what="extreme magnitudes")


def test_layerwise_and_per_sample_views():
    x = workloads.make_activation((6, 12, 16, 16), "relu", (0.05, 20.0), seed=9, device=DEV)
    e = x.numel()
    _check(x, 3, 1, desc=G.make_desc(1, 1, 1, e, G.GRANQ_F32), view_shape=(1, 1, 1, e), what="layer-wise view")
    _check(x, 3, 2, desc=G.make_desc(1, 6 * 12, 16, 16, G.GRANQ_F32), view_shape=(1, 72, 16, 16), what="per-sample view")
    w = workloads.make_activation((1, 64, 1, 32 * 9), "linear", (0.01, 0.2), seed=4, device=DEV)
    _check(w, 4, 3, what="weight view")


def test_in_place_forward_and_gradient():
    x = workloads.make_activation((4, 16, 14, 14), "linear", (0.05, 20.0), seed=3, device=DEV)
    dy = workloads.make_grad(x.shape, 3, DEV)
    ref = gpu_path(x, 4, dy)
    s = torch.tensor(ref["scale"], device=DEV)
    z = torch.tensor(ref["zero_point"], device=DEV)
    x2, dy2 = x.clone(), dy.clone()
    G.granq_fakequant_bwd(x2, dy2, s, z, 4, dy2)       # dx aliases dy
    G.granq_fakequant_fwd(x2, s, z, 4, x2)             # x_hat aliases x
    torch.cuda.synchronize()
    assert np.array_equal(x2.cpu().numpy(), ref["xhat"])
    assert np.array_equal(dy2.cpu().numpy(), ref["dx"])


def _misaligned_like(t, off_elems):
    """A copy of t that starts off_elems elements into a fresh allocation."""
    buf = torch.zeros(t.numel() + 16, dtype=t.dtype, device=t.device)
    v = buf[off_elems:off_elems + t.numel()].view(t.shape)
    v.copy_(t)
    return v


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16], ids=["f32", "bf16", "f16"])
@pytest.mark.parametrize("shape,misaligned", [
    ((4, 16, 14, 14), False),     # every 16-byte vector inside one channel
    ((5, 24, 7, 7), False),       # H*W = 49: vectors straddle two channels
    ((64, 96, 1, 1), False),      # H*W = 1: every element its own channel
    ((3, 8, 8, 8), True),         # pointer aligned to the element only: element-wise kernels
    ((2, 3, 7, 7), False),        # rows that are no whole number of vectors: element-wise kernels
    ((1, 1, 1, 4096), False),     # layer-wise view
], ids=["one", "two", "each", "misaligned", "ragged", "layer"])
def test_in_place_every_kernel_family(shape, misaligned, dtype):
    """x_hat == x and dx == dy, which the header allows, in every kernel variant: results equal
    the oracle's (the out-of-place ones), also for the one-call forward and the gate-bit pair."""
    x = workloads.make_activation(shape, "linear", (0.05, 20.0), seed=11, device=DEV, dtype=dtype)
    dy = workloads.make_grad(shape, 11, DEV, dtype)
    ref = workloads.make_activation(shape, "linear", (0.05, 5.0), seed=12, device=DEV, dtype=dtype)
    off = (1 if dtype == torch.float32 else 2) if misaligned else 0
    mk = (lambda t: _misaligned_like(t, off)) if misaligned else (lambda t: t.clone())
    c = G.desc_of(x).c
    for stale in (False, True):            # stale ranges make the gate and both clamp sides bite
        src = to_numpy(ref if stale else x)
        mn, mx = oracle.range_reduce(src)
        s_np, z_np = oracle.prescale(mn, mx, 4)
        want = oracle_path(to_numpy(x), 4, to_numpy(dy), scale=s_np, zero_point=z_np)
        s, z = torch.tensor(s_np, device=DEV), torch.tensor(z_np, device=DEV)
        x2, dy2 = mk(x), mk(dy)
        if misaligned:
            assert x2.data_ptr() % 16 != 0
        G.granq_fakequant_bwd(x2, dy2, s, z, 4, dy2)
        G.granq_fakequant_fwd(x2, s, z, 4, x2)
        torch.cuda.synchronize()
        got = {"scale": s_np, "zero_point": z_np, "xhat": to_numpy(x2), "dx": to_numpy(dy2)}
        assert_parity(got, want, "in place %s stale=%s" % (shape, stale))
        # gate-bit pair, both in place
        x3, dy3 = mk(x), mk(dy)
        mask = torch.zeros(G.granq_mask_bytes(G.desc_of(x)), dtype=torch.uint8, device=DEV)
        G.granq_fakequant_fwd_mask(x3, s, z, 4, x3, mask)
        G.granq_fakequant_bwd_mask(dy3, mask, dy3)
        torch.cuda.synchronize()
        got = {"scale": s_np, "zero_point": z_np, "xhat": to_numpy(x3), "dx": to_numpy(dy3)}
        assert_parity(got, want, "in place, gate bits %s stale=%s" % (shape, stale))
    # ranges, parameters and forward in one call, x_hat == x
    want = oracle_path(to_numpy(x), 4)
    x4 = mk(x)
    vec = [torch.full((c,), float("nan"), device=DEV) for _ in range(4)]
    ws = torch.empty(max(16, G.granq_workspace_bytes(G.desc_of(x))), dtype=torch.uint8, device=DEV)
    G.granq_calibrate_fakequant_fwd(x4, 4, vec[0], vec[1], vec[2], vec[3], x4, None, ws)
    torch.cuda.synchronize()
    got = {"min": vec[0].cpu().numpy(), "max": vec[1].cpu().numpy(), "scale": vec[2].cpu().numpy(),
           "zero_point": vec[3].cpu().numpy(), "xhat": to_numpy(x4)}
    assert_parity(got, want, "one-call forward in place %s" % (shape,))


# Channels of more than 128 KB: the one-call forward takes two launches, the second one finishing
# the reduction in its leading blocks while the others wait for their channels' parameters.
TWO_LAUNCH = [
    ((64, 24, 28, 28), torch.float32),      # one channel per vector
    ((700, 100, 7, 7), torch.float32),      # vectors straddle two channels
    ((40000, 40, 1, 1), torch.float32),     # every element its own channel, glued rows
    ((96, 16, 32, 32), torch.bfloat16),
    ((1500, 36, 7, 7), torch.float16),
    ((1, 1, 1, 1 << 20), torch.float32),    # layer-wise view
    ((300, 3, 40, 40), torch.float32),      # channels that span many column tiles
]


@pytest.mark.parametrize("spin_limit", [None, "0", "3"], ids=["default", "nowait", "shortwait"])
@pytest.mark.parametrize("shape,dtype", TWO_LAUNCH, ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v)[6:])
def test_one_call_forward_in_two_launches(shape, dtype, spin_limit, monkeypatch):
    """All six outputs of granq_calibrate_fakequant_fwd against the oracle, with the default
    wait, with no wait at all (every wavefront that finds its parameters pending derives them
    from the partials itself) and with a wait of three polls."""
    if spin_limit is None:
        monkeypatch.delenv("GRANQ_SPIN_LIMIT", raising=False)
    else:
        monkeypatch.setenv("GRANQ_SPIN_LIMIT", spin_limit)
    for i, (law, bits) in enumerate([("relu", 4), ("linear", 3)]):
        x = workloads.make_activation(shape, law, (0.05, 20.0), seed=20 + i, device=DEV, dtype=dtype)
        d = G.desc_of(x)
        vec = [torch.full((d.c,), float("nan"), device=DEV) for _ in range(4)]
        ws = torch.full((max(16, G.granq_workspace_bytes(d)),), 0xA5, dtype=torch.uint8, device=DEV)
        xh = torch.empty_like(x)
        codes = torch.full(x.shape, 255, dtype=torch.uint8, device=DEV)
        for rep in range(2):                 # the second call finds the first one's hand-over slots filled
            G.granq_calibrate_fakequant_fwd(x, bits, vec[0], vec[1], vec[2], vec[3], xh, codes, ws)
        torch.cuda.synchronize()
        got = {"min": vec[0].cpu().numpy(), "max": vec[1].cpu().numpy(), "scale": vec[2].cpu().numpy(),
               "zero_point": vec[3].cpu().numpy(), "xhat": to_numpy(xh), "codes": codes.cpu().numpy()}
        want = oracle_path(to_numpy(x), bits)
        assert_parity(got, want, "two launches %s %s spin=%s" % (shape, law, spin_limit))
        # codes alone, and x_hat alone
        only = torch.full(x.shape, 254, dtype=torch.uint8, device=DEV)
        G.granq_calibrate_fakequant_fwd(x, bits, vec[0], vec[1], vec[2], vec[3], None, only, ws)
        xh2 = torch.empty_like(x)
        G.granq_calibrate_fakequant_fwd(x, bits, vec[0], vec[1], vec[2], vec[3], xh2, None, ws)
        torch.cuda.synchronize()
        assert torch.equal(only, codes)
        ib = torch.int32 if dtype == torch.float32 else torch.int16
        assert torch.equal(xh2.view(ib), xh.view(ib))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("shape", [(1, 1, 1, 10_000_001), (2, 3, 1, 1_000_003), (1, 5, 3, 333_337)],
                         ids=lambda s: "x".join(map(str, s)))
def test_long_slabs_without_vector_structure(shape, dtype):
    """Element-wise kernels on slabs of millions of elements (a layer-wise view of odd size, a
    few long channels): the slabs are cut into pieces so that every compute unit gets work;
    results as everywhere."""
    x = workloads.make_activation(shape, "linear", (0.05, 20.0), seed=31, device=DEV, dtype=dtype)
    _check(x, 4, 31, what="long slabs %s" % (shape,))


def test_misaligned_pointers_take_the_elementwise_path():
    """A tensor that starts 4 bytes into an allocation: same results, no fault."""
    for dtype in (torch.float32, torch.bfloat16, torch.float16):
        shape = (3, 8, 8, 8)
        n = 3 * 8 * 8 * 8
        off = 1 if dtype == torch.float32 else 2
        xbuf = torch.zeros(n + 8, dtype=dtype, device=DEV)
        x = xbuf[off:off + n].view(shape)
        x.copy_(workloads.make_activation(shape, "linear", (0.05, 20.0), seed=6, device=DEV, dtype=dtype))
        assert x.data_ptr() % 16 != 0
        dybuf = torch.zeros(n + 8, dtype=dtype, device=DEV)
        dy = dybuf[off:off + n].view(shape)
        dy.copy_(workloads.make_grad(shape, 6, DEV, dtype))
        got = gpu_path(x, 4, dy)
        want = oracle_path(to_numpy(x), 4, to_numpy(dy))
        assert_parity(got, want, "misaligned %s" % dtype)


def test_non_default_stream_and_reuse_of_workspace():
    st = torch.cuda.Stream()
    x1 = workloads.make_activation((8, 32, 14, 14), "relu", (0.05, 20.0), seed=1, device=DEV)
    x2 = workloads.make_activation((8, 32, 14, 14), "linear", (0.05, 20.0), seed=2, device=DEV)
    q = G.ActivationQuantizer(x1.shape, x1.dtype, 4, DEV)
    outs = []
    torch.cuda.synchronize()
    with torch.cuda.stream(st):
        for x in (x1, x2, x1):
            xh = torch.empty_like(x)
            q.forward(x, xh)
            outs.append(xh)
    st.synchronize()
    for x, xh in zip((x1, x2, x1), outs):
        want = oracle_path(to_numpy(x), 4)
        assert np.array_equal(xh.cpu().numpy(), want["xhat"])


def test_near_ties_at_scale():
    """Millions of inputs sitting on or next to a rounding tie of Eq. 1
    (x ~ s * (k + 1/2) and its neighbouring floats): the quotient must be the
    correctly rounded one for the codes to agree."""
    g = torch.Generator(device=DEV).manual_seed(11)
    c, n, hw = 96, 16, 1024
    for bits in (4, 5, 8):
        qmax = 2 ** bits - 1
        s_true = torch.exp(torch.rand(c, generator=g, device=DEV) * 12 - 6)          # 2.5e-3 .. 400
        k = torch.randint(0, qmax, (n, c, hw), generator=g, device=DEV).float()
        x = (s_true.view(1, c, 1) * (k + 0.5)).contiguous()
        bump = torch.randint(-2, 3, (n, c, hw), generator=g, device=DEV, dtype=torch.int32)
        x = (x.view(torch.int32) + bump).view(torch.float32)
        x[0, :, 0] = 0.0
        x[0, :, 1] = s_true * qmax                                                   # range [0, s*qmax]
        x = torch.minimum(x, (s_true * qmax).view(1, c, 1)).view(n, c, 32, 32).contiguous()
        got, want = _check(x, bits, bits, what="near ties b%d" % bits)
        # the scales the library derived are close to the planted ones, so the inputs are near ties
        frac = np.abs((to_numpy(x).astype(np.float64) / want["scale"].reshape(1, c, 1, 1)) % 1.0 - 0.5)
        assert np.median(frac) < 1e-5


def test_channels_outside_the_fast_quotient_window():
    """Scales below 2^-30, above 2^60, huge zero-points and ordinary channels mixed
    in one tensor: lanes fall back to the general division per channel."""
    g = torch.Generator(device=DEV).manual_seed(12)
    for shape in [(4, 12, 8, 8), (3, 12, 7, 7), (2, 12, 1, 2048)]:
        c = shape[1]
        mag = torch.tensor([1e-12, 1e-11, 1.0, 1e20, 1e25, 3e-10, 1e-3, 1e19, 5.0, 1e-9, 1e30, 2.0], device=DEV)
        x = torch.rand(shape, generator=g, device=DEV) * mag.view(1, c, 1, 1)
        x[:, 8] += 3e8                       # offset range: zero-point ~ -1e9 (beyond 2^26)
        for bits in (3, 8):
            got, want = _check(x, bits, 1, what="window %s b%d" % (shape, bits))
        assert (want["scale"] < 2.0 ** -30).any() and (want["scale"] > 2.0 ** 60).any()
        assert (np.abs(want["zero_point"]) > 2.0 ** 26).any()
        # stale parameters too: huge inputs against small scales, tiny inputs against large ones
        s = np.array([2.0 ** -30, 2.0 ** 60, 1.0, 2.0 ** -29, 2.0 ** 59, 1e-5, 1e5, 3.0, 0.1, 7.0, 2.0 ** -31, 2.0 ** 61], np.float32)
        z = np.array([0, 3, -5, 2.0 ** 26, -2.0 ** 26, 2.0 ** 27, 1, 0.3, 0.49999997, 100, 0, 1], np.float32)
        xs = (torch.randn(shape, generator=g, device=DEV) * torch.exp(torch.randn(shape, generator=g, device=DEV) * 30)).clamp(-3e38, 3e38).contiguous()
        xs[0, :, 0, 0] = 3.0e38
        xs[0, :, 0, 1] = -3.0e38
        xs[0, :, 0, 2] = 1e-45
        xs[0, :, 0, 3] = 0.0
        dy = workloads.make_grad(shape, 2, DEV)
        got = gpu_path(xs, 4, dy, scale=s, zero_point=z)
        want = oracle_path(to_numpy(xs), 4, to_numpy(dy), scale=s, zero_point=z)
        assert_parity(got, want, "stale extreme %s" % (shape,))


def test_binary16_overflow_subnormals_and_ties():
    """binary16 storage where its narrowing matters: dequantized values beyond 65504 become
    infinity, tiny ones become subnormals, and products that fall exactly between two binary16
    values go to the even one -- as in the oracle's own conversion."""
    g = torch.Generator(device=DEV).manual_seed(11)
    x = torch.empty(4, 6, 8, 8, dtype=torch.float16, device=DEV)
    scales = torch.tensor([6.0e4, 3.0e-6, 1.0e-7, 1.0, 255.0, 0.37], device=DEV).view(1, 6, 1, 1)
    x.copy_((torch.rand(4, 6, 8, 8, generator=g, device=DEV) * 2 - 1) * scales)
    x[0, 0, 0, 0] = 65504.0
    x[1, 0, 0, 0] = -65504.0
    dy = workloads.make_grad(x.shape, 5, DEV, torch.float16)
    for bits in (2, 3, 8):
        got = gpu_path(x, bits, dy)
        want = oracle_path(to_numpy(x), bits, to_numpy(dy))
        assert_parity(got, want, "binary16 edge values b%d" % bits)
    # given scale 17/16: x_hat = q * 17/16 has exactly 12 significant bits for odd q in [121, 240],
    # i.e. lies exactly between two binary16 values (11 significant bits)
    s = np.full(6, 17.0 / 16.0, np.float32)
    z = np.zeros(6, np.float32)
    xq = torch.arange(0, 4 * 6 * 8 * 8, device=DEV, dtype=torch.float32).remainder(256).view(4, 6, 8, 8).to(torch.float16)
    got = gpu_path(xq, 8, None, scale=s, zero_point=z)
    want = oracle_path(to_numpy(xq), 8, None, scale=s, zero_point=z)
    assert_parity(got, want, "binary16 midpoints")
    odd = got["codes"][(got["codes"] % 2 == 1) & (got["codes"] >= 121)]
    assert odd.size > 300


def test_binary16_store_rounds_twice():
    """x_hat is a binary32 product that is then narrowed: two roundings.  Scales s = RN(m / 3) for
    binary16 midpoints m make RN32(3 s) land exactly on m while the exact product 3 s does not, so a
    narrowing fused with the multiply (one rounding from the exact product) gives the other
    neighbour in about half of the channels.  Both the vector kernels and the element-wise ones."""
    h = np.arange(0x3C00, 0x6C00, dtype=np.uint16)                     # binary16 values 1 .. 4096
    lo = h.view(np.float16).astype(np.float64)
    mids = ((lo[:-1] + lo[1:]) / 2)[::3][:4096]                        # 4096 exact midpoints
    s = (mids / 3.0).astype(np.float32)
    hit = (s.astype(np.float32) * np.float32(3.0)).astype(np.float64) == mids     # RN32(3 s) is the midpoint
    inexact = s.astype(np.float64) * 3.0 != mids                                   # the exact product is not
    assert (hit & inexact).sum() > 1000
    c = s.size
    z = np.zeros(c, np.float32)
    for offset in (0, 1):                                              # aligned: vector path; +1 element: element-wise
        buf = torch.zeros(2 * c * 4 + 16, dtype=torch.float16, device=DEV)
        x = buf[offset:offset + 2 * c * 4].view(2, c, 2, 2)
        x.copy_(torch.from_numpy(mids.astype(np.float32)).to(DEV).view(1, c, 1, 1).expand(2, c, 2, 2))
        got = gpu_path(x, 4, None, scale=s, zero_point=z)
        want = oracle_path(to_numpy(x), 4, None, scale=s, zero_point=z)
        assert np.all(want["codes"] == 3)
        assert_parity(got, want, "binary16 double rounding, offset %d" % offset)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("shape", [(6, 64, 14, 14), (3, 24, 7, 5), (16, 256, 4, 4), (5, 3, 9, 8)],
                         ids=lambda s: "x".join(map(str, s)))
def test_channels_last_is_the_view_with_unit_maps(shape, dtype):
    """A channels-last (N,H,W,C) tensor is the NCHW call on {N*H*W, C, 1, 1}: the results must be
    those of the oracle on the ordinary NCHW tensor, element for element after the permutation."""
    n, c, h, w = shape
    x = workloads.make_activation(shape, "linear", (0.05, 20.0), seed=4, device=DEV, dtype=dtype)
    dy = workloads.make_grad(shape, 4, DEV, dtype)
    want = oracle_path(to_numpy(x), 4, to_numpy(dy))
    x_cl = x.permute(0, 2, 3, 1).contiguous().view(n * h * w, c, 1, 1)
    dy_cl = dy.permute(0, 2, 3, 1).contiguous().view(n * h * w, c, 1, 1)
    got = gpu_path(x_cl, 4, dy_cl)

    def back(a):
        return np.ascontiguousarray(a.reshape(n, h, w, c).transpose(0, 3, 1, 2))
    got = dict(got, xhat=back(got["xhat"]), codes=back(got["codes"]), dx=back(got["dx"]))
    assert_parity(got, want, "channels-last %s" % (shape,))
