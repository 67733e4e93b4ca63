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


class OracleJobs:
    """Oracle comparisons of host copies, a few at a time on worker threads beside the GPU work (the oracle's C
    routines run without the interpreter lock); `drain` re-raises the first failure."""

    def __init__(self, workers=6, in_flight=6):
        from concurrent.futures import ThreadPoolExecutor
        self.pool, self.pending, self.in_flight = ThreadPoolExecutor(workers), [], in_flight

    def submit(self, fn, *args):
        while len(self.pending) >= self.in_flight:
            self.pending.pop(0).result()
        self.pending.append(self.pool.submit(fn, *args))

    def drain(self):
        try:
            while self.pending:
                self.pending.pop(0).result()
        finally:
            self.pool.shutdown(wait=True)


def oracle_step(label, w_h, before_h, nbits, blob_gpu, after_gpu_h, cached=None):
    """One encode + restore of the oracle on host copies of what the GPU path was given, against what it produced:
    blob bytes, restored bits and (cached = (cache before, blob, used, cache after)) the cached encode's."""
    blob_cpu = orc.encode(w_h, before_h, nbits)
    assert blob_gpu.size == blob_cpu.size, (label, blob_gpu.size, blob_cpu.size)
    diff = np.nonzero(blob_gpu != blob_cpu)[0]
    assert diff.size == 0, "%s: first differing byte %d" % (label, diff[0])
    if cached is not None:
        cache_cpu, blob_c_gpu, used_gpu, cache_after_gpu = cached
        blob_c, used_cpu = orc.encode_cached(w_h, before_h, nbits, cache_cpu)
        assert used_gpu == used_cpu, label
        assert blob_c_gpu.size == blob_c.size and np.array_equal(blob_c_gpu, blob_c), label + " (cached)"
        assert np.array_equal(cache_after_gpu, cache_cpu), label + " (cache)"
    restored = before_h                                   # (this job's own copy)
    assert orc.decode(blob_cpu, restored) == blob_cpu.size
    bad = np.nonzero(bits(restored) != bits(after_gpu_h))[0]
    assert bad.size == 0, "%s: first differing element %d of %d" % (label, bad[0], bad.size)


def test_config4_gpt2_chain_all_32_steps_full_size(lc):
    """Algorithm 1's loop at full size: all 32 checkpoints, each encoded against the recovered state and restored
    into it, every blob (plain and with the code table cache of Section 3.2) and every recovered state against
    the oracle; then the restore from u_0 and all 32 blobs in one lc_decode_many call (Section 3, C1).
    The oracle is given the state the GPU path recovered at the step before, which that step's own comparison has
    shown to be the oracle's, so this is the oracle's chain step by step while its steps run side by side."""
    from paper_2009_13003_amd import workloads
    chain = workloads.Gpt2Chain(device=DEV)
    n, nbits = chain.nel, chain.nbits
    assert n == 354_823_168
    tracked = chain.w0.clone()
    out = lc.alloc_out(n, nbits, DEV)
    out_c = lc.alloc_out(n, nbits, DEV)
    cache_gpu = lc.new_cache(DEV)
    words = lambda c: c.cpu().numpy()[:4 * orc.CACHE_WORDS].view(np.uint32).copy()
    jobs = OracleJobs()
    blobs, hits = [], 0
    try:
        for t in range(32):
            print("chain step", t, flush=True)
            w = chain.step()
            w_h, before_h = w.cpu().numpy(), tracked.cpu().numpy()
            cache_before = words(cache_gpu)
            size_c, used = lc.lc_encode_cached(w, tracked, nbits, out_c, cache_gpu)
            size = lc.lc_encode(w, tracked, nbits, out)
            blob = out[:size].clone()
            assert lc.lc_decode(blob, tracked) == size
            hits += int(used)
            blobs.append(blob)
            jobs.submit(oracle_step, "step %d" % t, w_h, before_h, nbits, blob.cpu().numpy(), tracked.cpu().numpy(),
                        (cache_before, out_c[:size_c].cpu().numpy(), used, words(cache_gpu)))
            del w_h, before_h
    finally:
        jobs.drain()
    assert hits >= 16                                     # successive checkpoints mostly keep their buckets
    # crash after step 32: u_32 = u_0 + the 32 decoded deltas, in one call; `tracked` is the oracle's state (above)
    print("fused restore of 32 blobs", flush=True)
    restored = chain.w0.clone()
    assert lc.lc_decode_many(blobs, restored) == sum(b.numel() for b in blobs)
    assert torch.equal(restored.view(torch.int32), tracked.view(torch.int32))


def test_config5_llama7b_all_slices(lc):
    """All 6.7e9 parameters generated on the device; every one of the 26 slices of 2^28 elements (the calls bench.py
    times) in full against the oracle: blob bytes and restored bits."""
    from paper_2009_13003_amd import workloads
    w, w_ref, nbits = workloads.llama7b(device=DEV)
    n = w.numel()
    assert n == 6_738_415_616
    S = workloads.SLICE
    slices = [(lo, min(n, lo + S)) for lo in range(0, n, S)]
    assert len(slices) == 26 and slices[-1][1] - slices[-1][0] == 27_529_216
    out = lc.alloc_out(S, nbits, DEV)
    jobs = OracleJobs()
    try:
        for k, (lo, hi) in enumerate(slices):
            print("config 5 slice", k, flush=True)
            size = lc.lc_encode(w[lo:hi], w_ref[lo:hi], nbits, out)
            hdr = out[:512].cpu().numpy()
            assert lc.lc_blob_info(hdr.tobytes()) == dict(n=hi - lo, nbits=nbits, total_bytes=size, status=0)
            rec = w_ref[lo:hi].clone()
            assert lc.lc_decode(out, rec) == size
            jobs.submit(oracle_step, "slice %d" % k, w[lo:hi].cpu().numpy(), w_ref[lo:hi].cpu().numpy(), nbits,
                        out[:size].cpu().numpy(), rec.cpu().numpy())
            del rec
    finally:
        jobs.drain()


def test_staged_keys_at_full_size(lc):
    """The encode with staged keys (what a dense vector's second and later encodes take) on config 3 and on the first and
    the ragged last slice of config 5, in full against the oracle."""
    from paper_2009_13003_amd import workloads
    lc.lc_set_option(lc.OPT_KEY_STAGING, lc.STAGING_ALWAYS)
    try:
        w, w_ref, nbits = workloads.vgg16(device=DEV)
        full_check(lc, w, w_ref, nbits, "config 3, staged keys")
        del w, w_ref
        w, w_ref, nbits = workloads.llama7b_head(device=DEV)
        full_check(lc, w, w_ref, nbits, "config 5 slice 0, staged keys")
        n_last = 27_529_216
        full_check(lc, w[:n_last], w_ref[:n_last], nbits, "a slice of config 5's last length, staged keys")
    finally:
        lc.lc_set_option(lc.OPT_KEY_STAGING, lc.STAGING_AUTO)


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
