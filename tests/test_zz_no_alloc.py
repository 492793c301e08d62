"""gq_global_norm_static, the entry point that allocates nothing: its block partials live in a static
device array of the library instead of a caller-provided workspace.  Called through the C ABI and compared
with gq_global_norm (same kernels, so the same bits) and with the oracle, on two calls in a row, the second
on a smaller input, so that what the first call left in the shared array cannot leak into the second."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import gq_oracle as O

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2305_18627_amd as gq
    DEV = torch.device("cuda:0")
else:
    gq = None
    DEV = None


def _call_static(xs, kind, norm_out, flags):
    """Straight through the C ABI: host array of device pointers, raw device pointers, the current stream."""
    lib = gq.lib()
    arr = (C.c_void_p * len(xs))(*[x.data_ptr() for x in xs])
    st = lib.gq_global_norm_static(arr, len(xs), xs[0].numel(), int(kind), C.c_void_p(norm_out.data_ptr()),
                                   C.c_void_p(flags.data_ptr()), C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert st == gq.GQ_OK, gq.status_string(st)


def _call_workspace(xs, kind, norm_out, flags):
    lib = gq.lib()
    K, d = len(xs), xs[0].numel()
    nbytes = lib.gq_norm_workspace_bytes(K, d)
    ws = torch.full((max(nbytes, 8),), 0xEE, dtype=torch.uint8, device=DEV)
    arr = (C.c_void_p * K)(*[x.data_ptr() for x in xs])
    st = lib.gq_global_norm(arr, K, d, int(kind), C.c_void_p(norm_out.data_ptr()), C.c_void_p(flags.data_ptr()),
                            C.c_void_p(ws.data_ptr()), ws.numel(), C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert st == gq.GQ_OK, gq.status_string(st)


def _inputs(K, d, seed, scale):
    g = torch.Generator(device="cpu").manual_seed(seed)
    return [(torch.randn(d, generator=g) * scale).to(DEV) for _ in range(K)]


@pytest.mark.parametrize("kind", [0, 1, 2])
def test_static_scratch_norm_equals_workspace_norm_on_two_calls_in_a_row(kind):
    # the first input fills many partials with LARGE values; the second, smaller input has a much smaller norm:
    # a stale partial of the first call read by the second would show at once
    big = _inputs(5, 3_000_003, seed=11, scale=5.0)
    small = _inputs(3, 70_001, seed=12, scale=1e-3)
    for xs in (big, small):
        got = torch.full((1,), -1.0, device=DEV)
        gfl = torch.full((1,), 77, dtype=torch.int32, device=DEV)
        _call_static(xs, kind, got, gfl)
        want = torch.full((1,), -2.0, device=DEV)
        wfl = torch.full((1,), 78, dtype=torch.int32, device=DEV)
        _call_workspace(xs, kind, want, wfl)
        torch.cuda.synchronize()
        assert got.item() == want.item() and gfl.item() == wfl.item() == 0            # same kernels: same bits
        ne, nf, fl = O.global_norm([x.cpu().numpy() for x in xs], kind)
        if kind == 0:
            assert np.float32(got.item()) == nf                                       # the max norm is exact
        else:
            assert abs(got.item() - ne) <= 1e-5 * ne
    # and once more after an input that sets the status flags (zero gradient, then a NaN)
    zeros = [torch.zeros(4099, device=DEV)]
    got = torch.full((1,), -1.0, device=DEV)
    gfl = torch.full((1,), 77, dtype=torch.int32, device=DEV)
    _call_static(zeros, kind, got, gfl)
    torch.cuda.synchronize()
    assert got.item() == 0.0 and gfl.item() == 2
    zeros[0][4098] = float("nan")
    _call_static(zeros, kind, got, gfl)
    torch.cuda.synchronize()
    assert gfl.item() & 1
    _call_static(small, kind, got, gfl)
    want = torch.full((1,), -2.0, device=DEV)
    wfl = torch.full((1,), 78, dtype=torch.int32, device=DEV)
    _call_workspace(small, kind, want, wfl)
    torch.cuda.synchronize()
    assert got.item() == want.item() and gfl.item() == 0


def test_static_scratch_norm_allocates_nothing_and_takes_every_size():
    # the largest partial counts the library ever uses: K = 64 per-worker partials and a long gradient
    xs = [torch.full((1 << 20,), 0.5, device=DEV)] * 64
    got = torch.zeros(1, device=DEV)
    fl = torch.zeros(1, dtype=torch.int32, device=DEV)
    for kind in (0, 1, 2):
        _call_static(xs[:1], kind, got, fl)                    # first call on the device has been made
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    free_before, _ = torch.cuda.mem_get_info()
    for kind, want in ((0, 0.5), (1, 0.5 * np.sqrt(64.0 * (1 << 20))), (2, 0.5 * np.sqrt(float(1 << 20)))):
        _call_static(xs, kind, got, fl)
        torch.cuda.synchronize()
        assert abs(got.item() - want) <= 1e-6 * want and fl.item() == 0
    free_after, _ = torch.cuda.mem_get_info()
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before and free_after == free_before
    assert gq.lib().gq_norm_workspace_bytes(64, 1 << 40) <= 512 * 1024   # every size fits the static array
