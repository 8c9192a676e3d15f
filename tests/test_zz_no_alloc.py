"""The entry point that allocates nothing: granq_range_reduce_noalloc keeps the reduction's
partials in a scratch array the library owns statically on the GPU.  Called through the C ABI
and compared with granq_range_reduce (bit for bit) and with the CPU oracle, on two calls in a
row, the second on a smaller tensor (the array keeps the first call's contents)."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2503_18339_amd as G
import workloads
from parity import to_numpy

pytestmark = pytest.mark.gpu

DEV = "cuda"


def _ranges_with_workspace(x):
    d = G.desc_of(x)
    mn = torch.full((d.c,), float("nan"), device=DEV)
    mx = torch.full((d.c,), float("nan"), device=DEV)
    ws = torch.empty(max(16, G.granq_workspace_bytes(d)), dtype=torch.uint8, device=DEV)
    G.granq_range_reduce(x, mn, mx, ws)
    return mn, mx


def _ranges_noalloc_raw(x, check_memory=False):
    """Straight through ctypes: pointers, descriptor, stream."""
    lib = G.load()
    d = G.desc_of(x)
    mn = torch.full((d.c,), float("nan"), device=DEV)
    mx = torch.full((d.c,), float("nan"), device=DEV)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    st = lib.granq_range_reduce_noalloc(ctypes.c_void_p(x.data_ptr()), ctypes.byref(d),
                                        ctypes.c_void_p(mn.data_ptr()), ctypes.c_void_p(mx.data_ptr()),
                                        ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert st == G.GRANQ_OK, G.status_string(st)
    torch.cuda.synchronize()
    if check_memory:
        assert torch.cuda.mem_get_info()[0] == free_before, "device memory changed hands during the call"
    return mn, mx


def _same_bits(a, b):
    return torch.equal(a.view(torch.int32), b.view(torch.int32))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_two_calls_in_a_row_second_smaller(dtype):
    big = workloads.make_activation((16, 96, 28, 28), "linear", (0.05, 20.0), seed=1, device=DEV, dtype=dtype)
    small = workloads.make_activation((3, 24, 7, 7), "relu", (0.05, 20.0), seed=2, device=DEV, dtype=dtype)
    ragged = workloads.make_activation((2, 5, 3, 3), "laplace", (0.05, 20.0), seed=3, device=DEV, dtype=dtype)
    _ranges_noalloc_raw(small)               # the first call on a device looks the array up
    for x in (big, small, ragged, big):
        got = _ranges_noalloc_raw(x, check_memory=True)
        ref = _ranges_with_workspace(x)
        torch.cuda.synchronize()
        assert _same_bits(got[0], ref[0]) and _same_bits(got[1], ref[1]), tuple(x.shape)
        mn, mx = oracle.range_reduce(to_numpy(x))
        assert np.array_equal(got[0].cpu().numpy(), mn) and np.array_equal(got[1].cpu().numpy(), mx)


def test_binding_wrapper_and_stream():
    x = workloads.make_activation((8, 64, 14, 14), "relu", (0.05, 20.0), seed=4, device=DEV)
    st = torch.cuda.Stream()
    mn = torch.empty(64, device=DEV)
    mx = torch.empty(64, device=DEV)
    torch.cuda.synchronize()
    with torch.cuda.stream(st):
        G.granq_range_reduce_noalloc(x, mn, mx)
    st.synchronize()
    ref = _ranges_with_workspace(x)
    torch.cuda.synchronize()
    assert _same_bits(mn, ref[0]) and _same_bits(mx, ref[1])


def test_size_beyond_the_scratch_is_refused():
    """Host-side refusal: nothing is launched, the outputs keep their contents."""
    d = G.make_desc(1, 1 << 20, 1, 4, G.GRANQ_F32)
    assert G.granq_workspace_bytes(d) > (4 << 20)
    x = torch.zeros(4 << 20, device=DEV)
    mn = torch.full((1 << 20,), 7.0, device=DEV)
    mx = torch.full((1 << 20,), 7.0, device=DEV)
    with pytest.raises(G.GranqError) as err:
        G.granq_range_reduce_noalloc(x, mn, mx, desc=d)
    assert err.value.status == G.GRANQ_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((mn == 7.0).all()) and bool((mx == 7.0).all())
