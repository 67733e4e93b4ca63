"""The five benchmark workloads at their full sizes, HIP path against the CPU oracle, in the
launch configuration bench.py times (one call per 2^28-element slice).  Blobs byte-identical,
recovered weights bit-identical."""
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


def bits(a):
    return np.ascontiguousarray(a).view(np.uint32)


def full_check(lc, w, w_ref, nbits, label):
    n = w.numel()
    print("full-size case", label, "n=%d nbits=%d" % (n, nbits), flush=True)
    out = lc.alloc_out(n, nbits, DEV)
    size = lc.lc_encode(w, w_ref, nbits, out)
    w_h, ref_h = w.cpu().numpy(), w_ref.cpu().numpy()
    blob_cpu = orc.encode(w_h, ref_h, nbits)
    blob_gpu = out[:size].cpu().numpy()
    assert blob_gpu.size == blob_cpu.size, (blob_gpu.size, blob_cpu.size)
    diff = np.nonzero(blob_gpu != blob_cpu)[0]
    assert diff.size == 0, "first differing byte %d" % diff[0]
    rec = w_ref.clone()
    assert lc.lc_decode(out, rec) == size
    orc.decode(blob_cpu, ref_h)
    bad = np.nonzero(bits(rec.cpu().numpy()) != bits(ref_h))[0]
    assert bad.size == 0, "first differing element %d of %d" % (bad[0], bad.size)
    return size


def test_config1_single_tensor(lc):
    from paper_2009_13003_amd import workloads
    w, w_ref, nbits = workloads.single_tensor(device=DEV)
    size = full_check(lc, w, w_ref, nbits, "config 1")
    assert w.numel() == 1 << 20 and 10 < 4.0 * w.numel() / size < 32


def test_config2_resnet50(lc):
    from paper_2009_13003_amd import workloads
    w, w_ref, nbits = workloads.resnet50(device=DEV)
    assert w.numel() == 25_557_032
    full_check(lc, w, w_ref, nbits, "config 2")


def test_config3_vgg16(lc):
    from paper_2009_13003_amd import workloads
    w, w_ref, nbits = workloads.vgg16(device=DEV)
    assert w.numel() == 138_357_544
    size = full_check(lc, w, w_ref, nbits, "config 3")
    assert float((w == w_ref).float().mean()) > 0.09          # the exactly-unchanged tenth
    assert 4.0 * w.numel() / size > 20


def test_config4_gpt2_chain_full_size_first_steps(lc):
    """Full-size vector, the first 3 of the 32 steps checked against the oracle step by step
    (the whole 32-step chain runs at 1/64 size in test_gpu_parity.py)."""
    from paper_2009_13003_amd import workloads
    chain = workloads.Gpt2Chain(device=DEV)
    assert chain.nel == 354_823_168
    tracked = chain.w0.clone()
    tracked_h = tracked.cpu().numpy()
    out = lc.alloc_out(chain.nel, chain.nbits, DEV)
    cache_gpu, cache_cpu = lc.new_cache(DEV), orc.new_cache()
    used_any = False
    for t in range(3):
        print("chain step", t, flush=True)
        w = chain.step()
        # with the code table cache (Section 3.2): blob and hit/miss verdict as the oracle's
        size_c, used = lc.lc_encode_cached(w, tracked, chain.nbits, out, cache_gpu)
        blob_c, used_cpu = orc.encode_cached(w.cpu().numpy(), tracked_h, chain.nbits, cache_cpu)
        assert used == used_cpu and np.array_equal(out[:size_c].cpu().numpy(), blob_c), "cached, step %d" % t
        used_any = used_any or used
        size = lc.lc_encode(w, tracked, chain.nbits, out)
        blob_cpu = orc.encode(w.cpu().numpy(), tracked_h, chain.nbits)
        assert np.array_equal(out[:size].cpu().numpy(), blob_cpu), "step %d" % t
        lc.lc_decode(out, tracked)
        orc.decode(blob_cpu, tracked_h)
        assert np.array_equal(bits(tracked.cpu().numpy()), bits(tracked_h)), "step %d" % t
    assert used_any                                      # step 2 finds step 1's kept set again


def test_config5_llama7b_slices(lc):
    """All 6.7e9 parameters generated on the device; the first, a middle and the ragged last slice
    of 2^28 elements are checked in full against the oracle, every other slice by round-trip
    properties that hold at any size."""
    from paper_2009_13003_amd import workloads
    w, w_ref, nbits = workloads.llama7b(device=DEV)
    n = w.numel()
    assert n == 6_738_415_616
    S = workloads.SLICE
    slices = [(lo, min(n, lo + S)) for lo in range(0, n, S)]
    assert len(slices) == 26 and slices[-1][1] - slices[-1][0] == 27_529_216
    for k in (0, 13, 25):
        lo, hi = slices[k]
        full_check(lc, w[lo:hi], w_ref[lo:hi], nbits, "config 5 slice %d" % k)
    out = lc.alloc_out(S, nbits, DEV)
    for k, (lo, hi) in enumerate(slices):
        if k in (0, 13, 25):
            continue
        print("config 5 slice", k, flush=True)
        size = lc.lc_encode(w[lo:hi], w_ref[lo:hi], nbits, out)
        hdr = out[:512].cpu().numpy()
        info = lc.lc_blob_info(hdr.tobytes())
        assert info == dict(n=hi - lo, nbits=nbits, total_bytes=size, status=0)
        rec = w_ref[lo:hi].clone()
        assert lc.lc_decode(out, rec) == size
        d = (w[lo:hi] - w_ref[lo:hi])
        dq = rec - w_ref[lo:hi]
        # kept elements land in their own binade (error <= half the bucket width), dropped ones are unchanged
        changed = rec.view(torch.int32) != w_ref[lo:hi].view(torch.int32)
        err = (d - dq).abs()
        assert bool((err[changed] <= d[changed].abs()).all())
        K = int(hdr[20])
        cnt = np.frombuffer(hdr[64:64 + 16 * 16].tobytes(), dtype=np.uint64)[1::2]
        assert int(cnt.sum()) == hi - lo and int(changed.sum()) <= int(cnt[:K].sum())
        del rec, d, dq, changed, err


def test_single_call_past_4gib_offsets(lc):
    """One call whose arrays are larger than 4 GiB (byte offsets and chunk indices beyond 32-bit
    element arithmetic), ragged tail included, in full against the oracle."""
    n = (1 << 30) + 100_000_007
    g = torch.Generator(device=DEV); g.manual_seed(123)
    w_ref = torch.empty(n, device=DEV)
    w = torch.empty(n, device=DEV)
    piece = 1 << 27
    for lo in range(0, n, piece):
        hi = min(n, lo + piece)
        w_ref[lo:hi] = 0.05 * torch.randn(hi - lo, generator=g, device=DEV)
        u = torch.rand(hi - lo, generator=g, device=DEV) - 0.5
        scale = 1e-4 * (1 + 9 * (lo // piece % 3))               # three alternating scales
        w[lo:hi] = w_ref[lo:hi] - scale * torch.sign(u) * torch.log1p(-2 * u.abs().clamp_(max=0.49999997))
        del u
    full_check(lc, w, w_ref, 4, "n = 2^30 + 100,000,007")


def test_largest_n_one_call_takes(lc):
    """n = LC_MAX_N = 2^32 elements in one call (2^18 chunks, 4096 groups: every per-chunk and per-group array of the
    scratch area at its full size), in full against the oracle; one element more is refused."""
    n = 1 << 32
    g = torch.Generator(device=DEV); g.manual_seed(321)
    w_ref = torch.empty(n, device=DEV)
    w = torch.empty(n, device=DEV)
    piece = 1 << 28
    for lo in range(0, n, piece):
        hi = lo + piece
        w_ref[lo:hi] = 0.05 * torch.randn(piece, generator=g, device=DEV)
        u = torch.rand(piece, generator=g, device=DEV) - 0.5
        k = lo // piece
        scale = 1e-3 * 10.0 ** -(k % 4)                                   # four alternating scales
        w[lo:hi] = w_ref[lo:hi] - scale * torch.sign(u) * torch.log1p(-2 * u.abs().clamp_(max=0.49999997))
        if k % 5 == 4:
            w[lo + piece // 2:hi] = w_ref[lo + piece // 2:hi]                  # long unchanged stretches
        del u
    full_check(lc, w, w_ref, 3, "n = 2^32")
    import ctypes
    assert lc.lc_encode_bound(n + 1, 3) == 0 and lc.lc_workspace_bytes(n + 1, 3) == 0
    out = lc.alloc_out(1 << 20, 3, DEV)
    vp = lambda t: ctypes.c_void_p(t.data_ptr())
    assert lc._lib.lc_encode(vp(w), vp(w_ref), n + 1, 3, vp(out), None) == -lc.ERR_BADARG
