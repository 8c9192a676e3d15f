"""Ranges, parameters and forward in ONE launch (granq_calibrate_fakequant_fwd_resident) against
the CPU oracle: every output, several calls in a row on one state (the arrival counters and the
parameter slots carry an epoch), and with the wait switched off, so that every wavefront computes
its channels' ranges from the tensor itself (needs an MI355X)."""
import numpy as np
import pytest
import torch

import paper_2503_18339_amd as G
import workloads
from parity import assert_parity, oracle_path, to_numpy

pytestmark = pytest.mark.gpu
DEV = "cuda"

SHAPES = [
    ((8, 16, 32, 32), torch.float32),       # one channel per vector, whole channels per tile
    ((64, 24, 28, 28), torch.float32),
    ((37, 100, 7, 7), torch.float32),       # vectors straddle two channels
    ((4000, 40, 1, 1), torch.float32),      # every element its own channel, glued rows
    ((96, 16, 32, 32), torch.bfloat16),
    ((150, 40, 7, 7), torch.float16),
    ((1, 1, 1, 1 << 20), torch.float32),    # layer-wise view
    ((30, 3, 40, 40), torch.float32),       # channels that span several column tiles
    ((5, 37, 9, 8), torch.bfloat16),
    ((3, 5, 1, 4), torch.float32),          # a single, ragged tile
]


def _call(x, bits, state, want_codes=True):
    d = G.desc_of(x)
    vec = [torch.full((d.c,), float("nan"), device=DEV) for _ in range(4)]
    xh = torch.empty_like(x)
    codes = torch.full(x.shape, 255, dtype=torch.uint8, device=DEV) if want_codes else None
    took = G.granq_calibrate_fakequant_fwd_resident(x, bits, vec[0], vec[1], vec[2], vec[3], xh, codes, state)
    torch.cuda.synchronize()
    assert took
    got = {"min": vec[0].cpu().numpy(), "max": vec[1].cpu().numpy(), "scale": vec[2].cpu().numpy(),
           "zero_point": vec[3].cpu().numpy(), "xhat": to_numpy(xh)}
    if want_codes:
        got["codes"] = codes.cpu().numpy()
    return got


@pytest.mark.parametrize("spin_limit", [None, "0", "2"], ids=["default", "nowait", "shortwait"])
@pytest.mark.parametrize("shape,dtype", SHAPES, ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v)[6:])
def test_resident_forward_against_oracle(shape, dtype, spin_limit, monkeypatch):
    if spin_limit is None:
        monkeypatch.delenv("GRANQ_SPIN_LIMIT", raising=False)
    else:
        monkeypatch.setenv("GRANQ_SPIN_LIMIT", spin_limit)
    d = G.make_desc(shape[0], shape[1], shape[2], shape[3], G.binding.dtype_code(dtype))
    nbytes = G.granq_resident_state_bytes(d)
    assert nbytes > 0
    state = torch.full((nbytes,), 0xCD, dtype=torch.uint8, device=DEV)
    G.granq_resident_state_init(state)
    print("case", shape, dtype, spin_limit, flush=True)
    # five calls on one state, the data changing from call to call: epochs 0..4
    for i, (law, bits) in enumerate([("relu", 4), ("linear", 3), ("laplace", 8), ("linear", 4), ("relu", 1)]):
        x = workloads.make_activation(shape, law, (0.05, 20.0), seed=40 + i, device=DEV, dtype=dtype)
        got = _call(x, bits, state, want_codes=(i % 2 == 0))
        want = oracle_path(to_numpy(x), bits)
        assert_parity(got, want, "resident %s %s call %d spin=%s" % (shape, law, i, spin_limit))


def test_resident_refuses_what_it_does_not_take():
    big = G.make_desc(256, 64, 56, 56, G.GRANQ_F32)              # 206 MB
    ragged = G.make_desc(2, 3, 7, 7, G.GRANQ_F32)
    assert G.granq_resident_state_bytes(big) == 0 and G.granq_resident_state_bytes(ragged) == 0
    x = workloads.make_activation((8, 16, 32, 32), "relu", (0.05, 20.0), seed=1, device=DEV)
    d = G.desc_of(x)
    state = torch.zeros(G.granq_resident_state_bytes(d), dtype=torch.uint8, device=DEV)
    vec = [torch.full((16,), 7.0, device=DEV) for _ in range(4)]
    before = x.clone()
    assert G.granq_calibrate_fakequant_fwd_resident(x, 4, vec[0], vec[1], vec[2], vec[3], x, None, state) is False
    torch.cuda.synchronize()
    assert torch.equal(x, before) and all(bool((v == 7.0).all()) for v in vec)      # nothing ran
    small = torch.zeros(16, dtype=torch.uint8, device=DEV)
    with pytest.raises(G.GranqError) as err:
        G.granq_calibrate_fakequant_fwd_resident(x, 4, vec[0], vec[1], vec[2], vec[3], torch.empty_like(x), None, small)
    assert err.value.status == G.GRANQ_ERR_WORKSPACE


def test_resident_config_tensors_full_size():
    """The tensors of the benchmark's workloads that take this form, full size."""
    for shape in [(256, 16, 32, 32), (256, 32, 16, 16), (256, 64, 8, 8), (256, 512, 7, 7), (256, 256, 14, 14)]:
        d = G.make_desc(*shape, G.GRANQ_F32)
        state = torch.zeros(G.granq_resident_state_bytes(d), dtype=torch.uint8, device=DEV)
        for rep in range(2):
            x = workloads.make_activation(shape, "relu", (0.05, 20.0), seed=rep, device=DEV)
            got = _call(x, 4, state)
            want = oracle_path(to_numpy(x), 4)
            assert_parity(got, want, "resident full size %s call %d" % (shape, rep))
