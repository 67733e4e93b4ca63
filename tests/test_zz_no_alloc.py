"""lc_encode_static (the entry point that allocates nothing: its scratch is an array in the library's device image)
against lc_encode, through the C ABI: the same bytes in `out`, on calls in a row that share the array, the later
ones with smaller inputs; and against the oracle."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import lc_oracle as orc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def lc():
    from paper_2009_13003_amd import lc as mod
    return mod


def laplace_case(n, seed, scale=1e-3):
    g = torch.Generator(device=DEV); g.manual_seed(seed)
    w_ref = 0.05 * torch.randn(n, generator=g, device=DEV)
    u = torch.rand(n, generator=g, device=DEV) - 0.5
    return w_ref - scale * torch.sign(u) * torch.log1p(-2 * u.abs().clamp_(max=0.49999997)), w_ref


def header_size_status(out):
    h = out[:64].cpu().numpy()
    return int(h[40:48].view(np.uint64)[0]), int(h[48:52].view(np.uint32)[0])


def static_against_plain(lc, w, w_ref, nbits, label):
    n = w.numel()
    print("static case", label, "n=%d nbits=%d" % (n, nbits), flush=True)
    bound = lc.lc_encode_bound(n, nbits)
    out_s = torch.full((bound,), 0xA5, dtype=torch.uint8, device=DEV)
    out_p = torch.full((bound,), 0x5A, dtype=torch.uint8, device=DEV)
    lc.lc_encode_static(w, w_ref, nbits, out_s)
    torch.cuda.synchronize()
    size, status = header_size_status(out_s)
    assert status == 0
    assert lc.lc_encode(w, w_ref, nbits, out_p) == size
    assert torch.equal(out_s[:size], out_p[:size]), label
    blob_cpu = orc.encode(w.cpu().numpy(), w_ref.cpu().numpy(), nbits)
    assert blob_cpu.size == size and np.array_equal(out_s[:size].cpu().numpy(), blob_cpu), label
    return size


def test_static_encode_equals_encode_on_calls_in_a_row(lc):
    # the first call on the device, then smaller inputs that find the array as the call before left it
    w, r = laplace_case(37 * 16384 + 1234, seed=7)
    static_against_plain(lc, w, r, 4, "first")
    w2, r2 = laplace_case(5 * 16384 + 77, seed=8)
    static_against_plain(lc, w2, r2, 3, "smaller")
    w3, r3 = laplace_case(700, seed=9, scale=1e-5)
    static_against_plain(lc, w3, r3, 2, "less than a chunk")
    # quiet stretches (whole chunks below every kept bucket, chunks coded part by part), then a larger input again
    w4, r4 = laplace_case(64 * 16384 + 5, seed=10)
    w4[3 * 16384:40 * 16384] = r4[3 * 16384:40 * 16384] + 2.0 ** -30
    w4[41 * 16384 + 100] += 0.01
    static_against_plain(lc, w4, r4, 3, "quiet chunks")
    static_against_plain(lc, w, r, 4, "first again")
    z = torch.empty(0, device=DEV)
    static_against_plain(lc, z, z, 3, "empty")


def test_static_encode_back_to_back_without_waiting(lc):
    """Two calls enqueued on one stream with no wait between them: the second starts from what the first leaves."""
    wa, ra = laplace_case(20 * 16384 + 9, seed=11)
    wb, rb = laplace_case(3 * 16384 + 1, seed=12)
    oa, ob = lc.alloc_out(wa.numel(), 3, DEV), lc.alloc_out(wb.numel(), 4, DEV)
    lc.lc_encode_static(wa, ra, 3, oa)
    lc.lc_encode_static(wb, rb, 4, ob)
    torch.cuda.synchronize()
    for w, r, nbits, o in ((wa, ra, 3, oa), (wb, rb, 4, ob)):
        size, status = header_size_status(o)
        blob_cpu = orc.encode(w.cpu().numpy(), r.cpu().numpy(), nbits)
        assert status == 0 and size == blob_cpu.size and np.array_equal(o[:size].cpu().numpy(), blob_cpu)


def test_static_encode_limits_and_errors(lc):
    n = lc.STATIC_MAX_N
    w, r = laplace_case(n, seed=13)
    static_against_plain(lc, w, r, 4, "largest n")
    vp = lambda t: ctypes.c_void_p(t.data_ptr())
    out = lc.alloc_out(n, 4, DEV)
    assert lc._lib.lc_encode_static(vp(w), vp(r), n + 1, 4, vp(out), None) == lc.ERR_WORKSPACE
    assert lc._lib.lc_encode_static(vp(w), vp(r), n, 5, vp(out), None) == lc.ERR_BADARG
    assert lc._lib.lc_encode_static(None, vp(r), n, 3, vp(out), None) == lc.ERR_BADARG
    assert lc._lib.lc_encode_static(vp(w), vp(r), n, 3, None, None) == lc.ERR_BADARG
    # a non-finite delta: the header-only blob lc_encode leaves, status 2
    bad = w[:50000].clone(); bad[123] = float("inf")
    lc.lc_encode_static(bad, r[:50000], 3, out)
    torch.cuda.synchronize()
    assert header_size_status(out) == (512, 2)
    out_p = lc.alloc_out(50000, 3, DEV)
    with pytest.raises(lc.LcError):
        lc.lc_encode(bad, r[:50000], 3, out_p)
    assert torch.equal(out[:512], out_p[:512])
    # and the call after it is fine
    static_against_plain(lc, w[:50000], r[:50000], 3, "after an error")
