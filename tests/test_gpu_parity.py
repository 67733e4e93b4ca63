"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle, bit for bit.

Bar: blobs (header, code tables, offsets, lane lengths, packed bits) byte-identical;
recovered weights bit-identical (tighter than the 1e-6 relative the target allows: both
sides do one IEEE fp32 subtract and one fp32 add per element, and the representatives
are integer-exact)."""
import numpy as np
import pytest
import torch

from oracle import lc_oracle as orc
from tests import lcb1_reader

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def lc():
    from paper_2009_13003_amd import lc as mod
    return mod


def bits(a):
    return np.ascontiguousarray(a).view(np.uint32)


def first_diff(a, b):
    m = min(a.size, b.size)
    d = np.nonzero(a[:m] != b[:m])[0]
    return "sizes %d/%d, first differing byte %s" % (a.size, b.size, d[0] if d.size else None)


def check_case(lc, w, w_ref, nbits, label=""):
    """Encode on both sides, compare blobs; decode on both sides, compare weights. Returns the blob."""
    n = w.numel()
    print("case", label, "n=%d nbits=%d" % (n, nbits), flush=True)
    out = lc.alloc_out(n, nbits, DEV)
    out.fill_(0xA5)                                   # stale bytes must never leak into the blob
    size = lc.lc_encode(w, w_ref, nbits, out)
    w_h, ref_h = w.cpu().numpy(), w_ref.cpu().numpy()
    blob_cpu = orc.encode(w_h, ref_h, nbits)
    blob_gpu = out[:size].cpu().numpy()
    assert blob_gpu.size == blob_cpu.size and np.array_equal(blob_gpu, blob_cpu), first_diff(blob_gpu, blob_cpu)
    assert lc.lc_verify(out[:size], n) == size            # (the check that reads the blob only accepts it, too)
    rec = w_ref.clone()
    assert lc.lc_decode(out, rec) == size
    orc.decode(blob_cpu, ref_h)
    rec_h = rec.cpu().numpy()
    bad = np.nonzero(bits(rec_h) != bits(ref_h))[0]
    assert bad.size == 0, "first differing element %d of %d" % (bad[0], bad.size)
    # the 1e-6 relative bar of the target, stated explicitly (implied by bit equality)
    assert np.all(np.abs(rec_h - ref_h) <= 1e-6 * np.abs(ref_h))
    return blob_cpu


def laplace_case(n, seed, scale=1e-3, zero_frac=0.0):
    g = torch.Generator(device=DEV); g.manual_seed(seed)
    w_ref = 0.05 * torch.randn(n, generator=g, device=DEV)
    u = torch.rand(n, generator=g, device=DEV) - 0.5
    d = -scale * torch.sign(u) * torch.log1p(-2 * u.abs().clamp_(max=0.49999997))
    if zero_frac:
        d = d * (torch.rand(n, generator=g, device=DEV) >= zero_frac)
    return w_ref + d, w_ref


SIZES = [0, 1, 3, 4, 5, 255, 256, 257, 1000, 16383, 16384, 16385, 5 * 16384 + 77, 37 * 16384, (1 << 20) + 13]


@pytest.mark.parametrize("n", SIZES)
@pytest.mark.parametrize("nbits", [1, 2, 3, 4])
def test_sizes_and_bit_budgets(lc, n, nbits):
    w, w_ref = laplace_case(n, seed=n * 4 + nbits, zero_frac=0.05)
    check_case(lc, w, w_ref, nbits)


def test_unaligned_pointers(lc):
    for off_w, off_r in ((1, 0), (0, 3), (2, 2), (1, 3)):
        n = 3 * 16384 + 100
        w, w_ref = laplace_case(n + 8, seed=off_w * 10 + off_r)
        check_case(lc, w[off_w:off_w + n], w_ref[off_r:off_r + n], 3, "unaligned %d/%d" % (off_w, off_r))


def test_degenerate_deltas(lc):
    n = 2 * 16384 + 500
    w_ref = 0.05 * torch.randn(n, device=DEV)
    check_case(lc, w_ref.clone(), w_ref, 3, "all zero delta")                      # only the zero symbol
    check_case(lc, w_ref * 0 + 1.0, w_ref * 0, 2, "one bucket, one value")         # one kept symbol, no zero symbol
    d = torch.zeros(n, device=DEV); d[12345] = 0.5
    check_case(lc, d, torch.zeros(n, device=DEV), 3, "single non-zero")
    # subnormal deltas, negative zeros in delta and in w_ref
    w = w_ref.clone(); w[::3] = 0.0; ref = w_ref.clone(); ref[::3] = -0.0
    w[1::3] = w_ref[1::3] + 0.01
    ref[2::9] = 1e-39; w[2::9] = 3e-39
    check_case(lc, w, ref, 3, "zeros / subnormals")
    # subnormal inputs with a normal difference
    a = torch.full((4096,), 1.1e-38, device=DEV); b = torch.full((4096,), -0.9e-38, device=DEV)
    check_case(lc, a, b, 2, "subnormal operands")


def test_flat_symbol_distribution_long_and_short_codes(lc):
    n = 20 * 16384 + 9
    g = torch.Generator(device=DEV); g.manual_seed(5)
    e = torch.randint(-8, 0, (n,), generator=g, device=DEV).float()
    sgn = torch.randint(0, 2, (n,), generator=g, device=DEV).float() * 2 - 1
    d = sgn * torch.exp2(e) * (1 + torch.rand(n, generator=g, device=DEV))
    check_case(lc, d, torch.zeros(n, device=DEV), 4, "16 flat symbols")
    # geometric populations: the deepest possible tree (code lengths up to 15)
    e = torch.floor(torch.log2(torch.rand(n, generator=g, device=DEV).clamp_(min=2.0 ** -20)))  # P(e=-k) = 2^-k
    d = torch.exp2(-20 - e) * (1 + 0.5 * torch.rand(n, generator=g, device=DEV))               # rare = large exponent
    blob = check_case(lc, d, torch.zeros(n, device=DEV), 4, "geometric populations")
    assert lcb1_reader.parse_header(blob)["max_len"] >= 12


def test_heterogeneous_tensors_have_locally_long_codes(lc):
    from paper_2009_13003_amd import workloads
    w, w_ref, nbits = workloads.llama7b(seed=3, device=DEV, shrink_by=4096)      # 291 tensors, ~1.6M elements
    check_case(lc, w, w_ref, nbits, "llama7b / 4096")
    w, w_ref, nbits = workloads.resnet50(seed=3, device=DEV, shrink_by=16)
    check_case(lc, w, w_ref, nbits, "resnet50 / 16")


def test_encode_is_deterministic_and_leaves_inputs_alone(lc):
    n = 50 * 16384 + 3
    w, w_ref = laplace_case(n, seed=99)
    w0, r0 = w.clone(), w_ref.clone()
    out1, out2 = lc.alloc_out(n, 3, DEV), lc.alloc_out(n, 3, DEV)
    s1 = lc.lc_encode(w, w_ref, 3, out1)
    s2 = lc.lc_encode(w, w_ref, 3, out2)
    assert s1 == s2 and torch.equal(out1[:s1], out2[:s2])
    assert torch.equal(w.view(torch.int32), w0.view(torch.int32)) and torch.equal(w_ref.view(torch.int32), r0.view(torch.int32))


def test_non_default_stream(lc):
    s = torch.cuda.Stream()
    n = 9 * 16384 + 1
    with torch.cuda.stream(s):
        w, w_ref = laplace_case(n, seed=4)
        check_case(lc, w, w_ref, 3, "side stream")


def test_nonfinite_is_rejected(lc):
    n = 3 * 16384
    w, w_ref = laplace_case(n, seed=8)
    out = lc.alloc_out(n, 3, DEV)
    for bad in (float("inf"), float("-inf"), float("nan")):
        wb = w.clone(); wb[n // 2 + 5] = bad
        with pytest.raises(lc.LcError) as e:
            lc.lc_encode(wb, w_ref, 3, out)
        assert e.value.status == lc.ERR_NONFINITE
        hdr = out[:512].cpu().numpy()
        with pytest.raises(orc.OracleError) as eo:
            orc.encode(wb.cpu().numpy(), w_ref.cpu().numpy(), 3)
        assert np.array_equal(hdr, eo.value.header)
        info = lc.lc_blob_info(hdr.tobytes())
        assert info["status"] == lc.ERR_NONFINITE and info["total_bytes"] == 512 and info["n"] == n
        rec = w_ref.clone()
        with pytest.raises(lc.LcError) as e:
            lc.lc_decode(out, rec)
        assert e.value.status == lc.ERR_BAD_BLOB and torch.equal(rec, w_ref)
    # and the library works again afterwards
    check_case(lc, w, w_ref, 3, "after an error")


def test_bad_arguments(lc):
    n = 1000
    w, w_ref = laplace_case(n, seed=1)
    out = lc.alloc_out(n, 3, DEV)
    for nb in (0, 5, -2):
        with pytest.raises(lc.LcError) as e:
            lc.lc_encode(w, w_ref, nb, out)
        assert e.value.status == lc.ERR_BADARG
    roomy = torch.empty(out.numel() + 16, dtype=torch.uint8, device=DEV)
    with pytest.raises(lc.LcError) as e:
        lc.lc_encode(w, w_ref, 3, roomy[4:])           # out must be 16-byte aligned
    assert e.value.status == lc.ERR_BADARG
    size = lc.lc_encode(w, w_ref, 3, out)
    with pytest.raises(lc.LcError) as e:
        lc.lc_decode(out, w_ref.clone()[:n - 1])       # n does not match the header
    assert e.value.status == lc.ERR_BADARG
    assert lc.lc_blob_info(out[:64].cpu().numpy().tobytes()) == dict(n=n, nbits=3, total_bytes=size, status=0)


def test_decode_rejects_damaged_blobs(lc):
    n = 6 * 16384 + 321
    w, w_ref = laplace_case(n, seed=77)
    out = lc.alloc_out(n, 3, DEV)
    size = lc.lc_encode(w, w_ref, 3, out)
    good = out[:size].clone()
    area = 512 + (4 * (7 + 1) + 15) // 16 * 16

    def damaged(off, xor):
        b = good.clone(); b[off] ^= xor
        return b
    structural = [damaged(0, 1), damaged(4, 3), damaged(16, 8), damaged(20, 8), damaged(24, 1), damaged(36, 1),
                  damaged(40, 4), damaged(48, 2), damaged(66, 8), damaged(64 + 8, 1), damaged(512 + 4, 1),
                  damaged(512 + 4 * 7, 2), damaged(area, 64), damaged(area + 3, 0x40)]
    for i, b in enumerate(structural):
        print("structural damage", i, flush=True)
        rec = w_ref.clone()
        with pytest.raises(lc.LcError) as e:
            lc.lc_decode(b, rec)
        assert e.value.status == lc.ERR_BAD_BLOB
        assert torch.equal(rec.view(torch.int32), w_ref.view(torch.int32)), "w_ref touched"
        with pytest.raises(orc.OracleError):
            orc.decode(b.cpu().numpy(), w_ref.cpu().numpy())
    # damage inside the streams: both sides must agree on the outcome (a flipped bit may also
    # turn one code into another of the same length, which no decoder can notice)
    outcomes = []
    for i, b in enumerate([damaged(area, 1)] + [damaged(area + 128 + 41 + 4 * k, 0x10) for k in range(6)]):
        print("stream damage", i, flush=True)
        rec, rec_h = w_ref.clone(), w_ref.cpu().numpy()
        try:
            lc.lc_decode(b, rec); gpu_ok = True
        except lc.LcError as e:
            assert e.status == lc.ERR_BAD_BLOB; gpu_ok = False
        try:
            orc.decode(b.cpu().numpy(), rec_h); cpu_ok = True
        except orc.OracleError:
            cpu_ok = False
        assert gpu_ok == cpu_ok
        if gpu_ok:
            assert np.array_equal(bits(rec.cpu().numpy()), bits(rec_h))
        outcomes.append(gpu_ok)
    assert not all(outcomes)
    rec = w_ref.clone()
    assert lc.lc_decode(good, rec) == size


@pytest.fixture
def verify_first(lc):
    lc.lc_set_option(lc.OPT_VERIFY_FIRST, 1)
    yield
    lc.lc_set_option(lc.OPT_VERIFY_FIRST, 0)


def payload_damage_cases(blob_t, nchunks, count, seed):
    """`count` copies of the blob with one bit flipped somewhere in the chunk area (lane lengths or lane strings)."""
    area = 512 + (4 * (nchunks + 1) + 15) // 16 * 16
    rng = np.random.RandomState(seed)
    out = []
    for _ in range(count):
        b = blob_t.clone()
        at = int(rng.randint(area, b.numel()))
        b[at] ^= 1 << int(rng.randint(0, 8))
        out.append((at, b))
    return out


@pytest.mark.parametrize("nbits,scale", [(3, 1e-3), (4, 1e-3), (2, 1e-5)])
def test_verify_gives_the_oracles_verdict_on_damaged_payloads(lc, nbits, scale):
    """lc_verify reads the blob only: on 60 blobs with one bit flipped in the chunk area (a lane length, a lane string,
    the padding) it says what the oracle's decoder says; a truncated buffer and a blob for another vector are refused."""
    n = 7 * 16384 + 4321
    w, w_ref = laplace_case(n, seed=700 + nbits, scale=scale)
    out = lc.alloc_out(n, nbits, DEV)
    size = lc.lc_encode(w, w_ref, nbits, out)
    good = out[:size].clone()
    assert lc.lc_verify(good, n) == size
    verdicts = []
    for k, (at, b) in enumerate(payload_damage_cases(good, 8, 60, 40 + nbits)):
        print("verify: damaged byte", at, flush=True)
        try:
            orc.decode(b.cpu().numpy(), w_ref.cpu().numpy()); cpu_ok = True
        except orc.OracleError as e:
            assert e.status == 4; cpu_ok = False
        try:
            assert lc.lc_verify(b, n) == size; gpu_ok = True
        except lc.LcError as e:
            assert e.status == lc.ERR_BAD_BLOB; gpu_ok = False
        assert gpu_ok == cpu_ok, (k, at)
        verdicts.append(gpu_ok)
    assert not all(verdicts) and any(verdicts)            # (a flip inside a code can give another valid code; one in the padding is refused)
    with pytest.raises(lc.LcError) as e:
        lc.lc_verify(good, n, blob_bytes=size - 4)
    assert e.value.status == lc.ERR_BAD_BLOB
    with pytest.raises(lc.LcError) as e:
        lc.lc_verify(good, n + 1)
    assert e.value.status == lc.ERR_BADARG
    with pytest.raises(lc.LcError) as e:
        lc.lc_verify(good, n, torch.bfloat16)
    assert e.value.status == lc.ERR_BADARG
    z = torch.empty(0, device=DEV)
    oz = lc.alloc_out(0, nbits, DEV)
    empty = lc.lc_encode(z, z, nbits, oz)
    assert lc.lc_verify(oz[:empty], 0) == empty


def test_restore_that_verifies_first_leaves_w_ref_alone(lc, verify_first):
    """With LC_OPT_VERIFY_FIRST a blob whose payload is damaged leaves w_ref untouched (without the option the sweep
    finds the damage half way); good blobs restore as always; in lc_decode_many one damaged blob among good ones stops
    the whole restore before the first sweep.  16-bit and binary64 parameters too."""
    n = 9 * 16384 + 100
    w, w_ref = laplace_case(n, seed=750)
    blob = torch.from_numpy(check_case(lc, w, w_ref, 3, "verify first, good blob")).to(DEV)
    refused = 0
    for at, b in payload_damage_cases(blob, 10, 30, 51):
        try:
            orc.decode(b.cpu().numpy(), w_ref.cpu().numpy()); cpu_ok = True
        except orc.OracleError:
            cpu_ok = False
        rec = w_ref.clone()
        if cpu_ok:
            assert lc.lc_decode(b, rec) == blob.numel()
            ref_h = w_ref.cpu().numpy(); orc.decode(b.cpu().numpy(), ref_h)
            assert np.array_equal(bits(rec.cpu().numpy()), bits(ref_h))
        else:
            refused += 1
            with pytest.raises(lc.LcError) as e:
                lc.lc_decode(b, rec)
            assert e.value.status == lc.ERR_BAD_BLOB
            assert torch.equal(rec.view(torch.int32), w_ref.view(torch.int32)), "w_ref touched (damage at byte %d)" % at
    assert refused >= 5
    # several checkpoints: the third blob's payload damaged
    g = torch.Generator(device=DEV); g.manual_seed(751)
    deltas = [1e-3 * torch.randn(n, generator=g, device=DEV) for _ in range(5)]
    tracked, blobs = encode_chain(lc, w_ref, deltas, [3] * 5)
    rec = w_ref.clone()
    lc.lc_decode_many(blobs, rec)
    assert np.array_equal(bits(rec.cpu().numpy()), bits(oracle_restore(w_ref, blobs)))
    area = 512 + (4 * 11 + 15) // 16 * 16
    bad = [b.clone() for b in blobs]
    bad[2][area + 60] ^= 0x7F                           # lane 30's length in chunk 0: its string no longer ends where it says
    with pytest.raises(orc.OracleError):
        orc.decode(bad[2].cpu().numpy(), w_ref.cpu().numpy())
    rec = w_ref.clone()
    with pytest.raises(lc.LcError) as e:
        lc.lc_decode_many(bad, rec)
    assert e.value.status == lc.ERR_BAD_BLOB and torch.equal(rec.view(torch.int32), w_ref.view(torch.int32))
    # other element types
    for tdt in (torch.bfloat16, torch.float64):
        wt, rt = w.to(tdt), w_ref.to(tdt)
        out = lc.alloc_out(n, 3, DEV)
        size = lc.lc_encode_t(wt, rt, 3, out)
        rec = rt.clone()
        assert lc.lc_decode_t(out, rec) == size
        plain = rt.clone()
        lc.lc_set_option(lc.OPT_VERIFY_FIRST, 0)
        assert lc.lc_decode_t(out, plain) == size
        lc.lc_set_option(lc.OPT_VERIFY_FIRST, 1)
        assert torch.equal(rec.view(torch.int16 if tdt == torch.bfloat16 else torch.int64), plain.view(torch.int16 if tdt == torch.bfloat16 else torch.int64))
        b = out[:size].clone(); b[area + 60] ^= 0x7F
        rec = rt.clone()
        with pytest.raises(lc.LcError):
            lc.lc_decode_t(b, rec)
        assert torch.equal(rec.view(torch.int16 if tdt == torch.bfloat16 else torch.int64), rt.view(torch.int16 if tdt == torch.bfloat16 else torch.int64))


def test_calls_with_stated_buffer_sizes(lc):
    """lc_encode_sized refuses an `out` below lc_encode_bound without touching it; lc_decode_sized restores from a
    buffer of exactly the blob's size and refuses, with w_ref untouched, a blob whose header claims more bytes than
    the caller's buffer holds (truncated buffer; forged size field with a matching last offset)."""
    n, nbits = 3 * 16384 + 500, 3
    w, w_ref = laplace_case(n, seed=77)
    bound = lc.lc_encode_bound(n, nbits)
    small = torch.full((bound - 1,), 0x77, dtype=torch.uint8, device=DEV)
    with pytest.raises(lc.LcError) as e:
        lc.lc_encode_sized(w, w_ref, nbits, small)
    assert e.value.status == lc.ERR_OUT_TOO_SMALL and bool((small == 0x77).all())
    out = lc.alloc_out(n, nbits, DEV)
    size = lc.lc_encode_sized(w, w_ref, nbits, out)
    blob_cpu = orc.encode(w.cpu().numpy(), w_ref.cpu().numpy(), nbits)
    assert size == blob_cpu.size and np.array_equal(out[:size].cpu().numpy(), blob_cpu)
    exact = out[:size].clone()
    rec = w_ref.clone()
    assert lc.lc_decode_sized(exact, rec) == size
    ref_h = w_ref.cpu().numpy(); orc.decode(blob_cpu, ref_h)
    assert np.array_equal(bits(rec.cpu().numpy()), bits(ref_h))
    for cut in (4, size - 600, size - 100):                     # the buffer ends inside the payload / the header
        rec = w_ref.clone()
        with pytest.raises(lc.LcError) as e:
            lc.lc_decode_sized(exact[:size - cut], rec)
        assert e.value.status == lc.ERR_BAD_BLOB and torch.equal(rec, w_ref)
    # a forged blob that claims 64 more bytes (size field and last offset agree): lc_decode's own checks pass the
    # header, the stated buffer size does not
    nchunks = (n + 16383) // 16384
    forged = exact.clone()
    forged[40:48] = torch.tensor(np.frombuffer(np.uint64(size + 64).tobytes(), np.uint8).copy(), device=DEV)
    last = 512 + 4 * nchunks
    words = int(exact[last:last + 4].cpu().numpy().view(np.uint32)[0]) + 16
    forged[last:last + 4] = torch.tensor(np.frombuffer(np.uint32(words).tobytes(), np.uint8).copy(), device=DEV)
    rec = w_ref.clone()
    with pytest.raises(lc.LcError) as e:
        lc.lc_decode_sized(forged, rec)
    assert e.value.status == lc.ERR_BAD_BLOB and torch.equal(rec, w_ref)


def test_caller_workspace(lc):
    n = 4 * 16384
    w, w_ref = laplace_case(n, seed=12)
    need = lc.lc_workspace_bytes(n, 3)
    ws = torch.empty(need + 256, dtype=torch.uint8, device=DEV)
    ws = ws[(-ws.data_ptr()) % 256:][:need]
    try:
        assert lc.lc_set_workspace(ws) == lc.OK
        check_case(lc, w, w_ref, 3, "caller workspace")
        big = laplace_case(40 * 16384, seed=13)
        with pytest.raises(lc.LcError) as e:
            lc.lc_encode(big[0], big[1], 3, lc.alloc_out(40 * 16384, 3, DEV))
        assert e.value.status == lc.ERR_WORKSPACE
    finally:
        assert lc.lc_set_workspace(None) == lc.OK
    check_case(lc, w, w_ref, 3, "library workspace again")


def test_checkpoint_chain_small(lc):
    """Config 4 at 1/64 size, all 32 steps: encode against the recovered state, decode into it (Algorithm 1)."""
    from paper_2009_13003_amd import workloads
    chain = workloads.Gpt2Chain(seed=0, device=DEV, shrink_by=64)
    tracked = chain.w0.clone()
    tracked_h = tracked.cpu().numpy()
    out = lc.alloc_out(chain.nel, chain.nbits, DEV)
    blobs = []
    for t in range(32):
        w = chain.step()
        size = lc.lc_encode(w, tracked, chain.nbits, out)
        blob_cpu = orc.encode(w.cpu().numpy(), tracked_h, chain.nbits)
        blob_gpu = out[:size].cpu().numpy()
        assert np.array_equal(blob_gpu, blob_cpu), "step %d: %s" % (t, first_diff(blob_gpu, blob_cpu))
        lc.lc_decode(out, tracked)
        orc.decode(blob_cpu, tracked_h)
        assert np.array_equal(bits(tracked.cpu().numpy()), bits(tracked_h)), "step %d" % t
        blobs.append(out[:size].clone())
    # a crash now: restore from u_0 and the blobs alone
    restored = chain.w0.clone()
    for b in blobs:
        lc.lc_decode(b, restored)
    assert torch.equal(restored.view(torch.int32), tracked.view(torch.int32))


def make_chain(lc, n, steps, seed, nbits=3):
    """`steps` checkpoints of a drifting vector, each encoded against the recovered state (Algorithm 1)."""
    g = torch.Generator(device=DEV); g.manual_seed(seed)
    w = 0.05 * torch.randn(n, generator=g, device=DEV)
    w0 = w.clone(); tracked = w.clone()
    d = torch.zeros(n, device=DEV)
    out = lc.alloc_out(n, nbits, DEV)
    blobs = []
    for t in range(steps):
        u = torch.rand(n, generator=g, device=DEV) - 0.5
        d = 0.9 * d - 5e-5 * (1 + t % 3) * torch.sign(u) * torch.log1p(-2 * u.abs().clamp_(max=0.49999997))
        w = w + d
        size = lc.lc_encode(w, tracked, nbits, out)
        blobs.append(out[:size].clone())
        lc.lc_decode(blobs[-1], tracked)
    return w0, tracked, blobs


@pytest.mark.parametrize("steps", [1, 2, 3, 8, 9, 17])
def test_fused_restore_equals_successive_restores(lc, steps):
    """Section 3 (C1): restoring from u_0 and all the blobs at once gives, bit for bit, what the oracle gives
    applying them one after the other."""
    n = 7 * 16384 + 4321
    w0, tracked, blobs = make_chain(lc, n, steps, seed=steps, nbits=3 + steps % 2)
    restored = w0.clone()
    consumed = lc.lc_decode_many(blobs, restored)
    assert consumed == sum(b.numel() for b in blobs)
    ref = w0.cpu().numpy()
    for b in blobs:
        orc.decode(b.cpu().numpy(), ref)
    assert np.array_equal(bits(restored.cpu().numpy()), bits(ref))
    assert torch.equal(restored.view(torch.int32), tracked.view(torch.int32))


def test_fused_restore_edge_cases(lc):
    # unaligned w_ref, tiny and empty vectors
    for n in (0, 5, 300, 16384 + 1):
        w0, tracked, blobs = make_chain(lc, n, 3, seed=n)
        buf = torch.zeros(n + 4, device=DEV)
        view = buf[1:1 + n]
        view.copy_(w0)
        lc.lc_decode_many(blobs, view)
        assert torch.equal(view.view(torch.int32), tracked.view(torch.int32)), n
    # a damaged blob anywhere in the list: error, w_ref untouched (also across more than one sweep)
    n = 3 * 16384 + 77
    w0, tracked, blobs = make_chain(lc, n, 11, seed=5)
    for bad_at in (0, 4, 10):
        damaged = [b.clone() for b in blobs]
        damaged[bad_at][512 + 4] ^= 1
        rec = w0.clone()
        with pytest.raises(lc.LcError) as e:
            lc.lc_decode_many(damaged, rec)
        assert e.value.status == lc.ERR_BAD_BLOB
        assert torch.equal(rec.view(torch.int32), w0.view(torch.int32))
    with pytest.raises(lc.LcError) as e:
        lc.lc_decode_many(blobs, w0.clone()[:n - 1])
    assert e.value.status == lc.ERR_BADARG
    with pytest.raises(lc.LcError) as e:
        lc.lc_decode_many(blobs * 6, w0.clone())             # 66 > LC_MAX_MANY
    assert e.value.status == lc.ERR_BADARG
    rec = w0.clone()
    lc.lc_decode_many(blobs, rec)
    assert torch.equal(rec.view(torch.int32), tracked.view(torch.int32))


def encode_chain(lc, w0, deltas, nbits_list):
    """Blobs of successive checkpoints w0 + d_1, w0 + d_1 + d_2, ..., each against the recovered state."""
    n = w0.numel()
    tracked = w0.clone()
    w = w0.clone()
    out = lc.alloc_out(n, 4, DEV)
    blobs = []
    for d, nbits in zip(deltas, nbits_list):
        w = w + d
        size = lc.lc_encode(w, tracked, nbits, out)
        blobs.append(out[:size].clone())
        lc.lc_decode(blobs[-1], tracked)
    return tracked, blobs


def oracle_restore(w0, blobs):
    ref = w0.cpu().numpy()
    for b in blobs:
        orc.decode(b.cpu().numpy(), ref)
    return ref


def test_fused_restore_mixed_code_lengths_and_whole_chunks(lc):
    """Blobs with codes of at most 7 bits and blobs with longer codes alternate in one call (they go through
    different forms of the fused sweep); n is a whole number of chunks, so the last chunk is staged too."""
    n = 6 * 16384
    g = torch.Generator(device=DEV); g.manual_seed(77)
    w0 = 0.05 * torch.randn(n, generator=g, device=DEV)
    nbits_list = [3, 2, 4, 4, 1, 3, 3, 4, 2, 3, 3, 3]
    # wide spread of magnitudes: with nbits = 4 the rare top buckets get codes longer than 7 bits
    deltas = [torch.randn(n, generator=g, device=DEV) * torch.exp2(-6 - 12 * torch.rand(n, generator=g, device=DEV)) for _ in nbits_list]
    tracked, blobs = encode_chain(lc, w0, deltas, nbits_list)
    max_lens = [lcb1_reader.parse_header(b.cpu().numpy())["max_len"] for b in blobs]
    assert max(max_lens) > 7 and min(max_lens) <= 7, max_lens      # both forms take part
    restored = w0.clone()
    assert lc.lc_decode_many(blobs, restored) == sum(b.numel() for b in blobs)
    assert np.array_equal(bits(restored.cpu().numpy()), bits(oracle_restore(w0, blobs)))
    assert torch.equal(restored.view(torch.int32), tracked.view(torch.int32))


def test_fused_restore_uneven_chunks(lc):
    """Most chunks unchanged, one dense chunk per blob: where it lies, the payloads of the sweep's blobs
    exceed the LDS area (sized to 1.1 x the sum of the blobs' average chunk payloads) and are read from
    memory instead."""
    nchunks = 24
    n = nchunks * 16384 + 100
    g = torch.Generator(device=DEV); g.manual_seed(78)
    w0 = 0.05 * torch.randn(n, generator=g, device=DEV)
    deltas = []
    for t in range(5):
        d = torch.zeros(n, device=DEV)
        lo = (5 * t + 1) * 16384
        d[lo - 50:lo + 16384 + 50] = 1e-3 * torch.randn(16384 + 100, generator=g, device=DEV)
        deltas.append(d)
    tracked, blobs = encode_chain(lc, w0, deltas, [3] * 5)
    # payload words per chunk, from the offset tables
    words = []
    for b in blobs:
        h = b.cpu().numpy()
        off = h[512:512 + 4 * (nchunks + 2)].view(np.uint32).astype(np.int64)
        words.append(np.diff(off) - 32)
    words = np.array(words)                             # [blob, chunk]
    area_words = 1.1 * (words.mean(axis=1) + 6).sum()
    assert words[:, :nchunks].sum(axis=0).max() > area_words + 64, "no chunk overflows: the test misses its path"
    restored = w0.clone()
    lc.lc_decode_many(blobs, restored)
    assert np.array_equal(bits(restored.cpu().numpy()), bits(oracle_restore(w0, blobs)))


def test_fused_restore_stream_damage_matches_oracle(lc):
    """A flipped payload bit is found, if at all, during the sweep: same verdict as the oracle's decoder, and
    where both accept the blob, the same weights."""
    n = 4 * 16384
    w0, tracked, blobs = make_chain(lc, n, 4, seed=31, nbits=3)
    for k, byte in enumerate((600, 1200, 2500, 4000)):
        damaged = [b.clone() for b in blobs]
        nchunks = lcb1_reader.parse_header(blobs[k].cpu().numpy())["num_chunks"]
        at = 512 + (4 * (nchunks + 1) + 15) // 16 * 16 + 128 + byte    # inside the first chunk's payload
        damaged[k][at] ^= 0x10
        ref = w0.cpu().numpy()
        ok = True
        for b in damaged:
            try:
                orc.decode(b.cpu().numpy(), ref)
            except orc.OracleError as e:
                assert e.status == 4
                ok = False
                break
        rec = w0.clone()
        if ok:
            lc.lc_decode_many(damaged, rec)
            assert np.array_equal(bits(rec.cpu().numpy()), bits(ref))
        else:
            with pytest.raises(lc.LcError) as e:
                lc.lc_decode_many(damaged, rec)
            assert e.value.status == lc.ERR_BAD_BLOB


FUSED_WIDE = r"""
import sys, numpy as np, torch
sys.path.insert(0, %r)
from paper_2009_13003_amd import lc
from oracle import lc_oracle as orc
n = 5 * 16384 + 999
g = torch.Generator(device="cuda:0"); g.manual_seed(5)
w0 = 0.05 * torch.randn(n, generator=g, device="cuda:0")
tracked, w, blobs = w0.clone(), w0.clone(), []
out = lc.alloc_out(n, 3, "cuda:0")
for t in range(15):
    w = w + 1e-4 * torch.randn(n, generator=g, device="cuda:0") * (torch.rand(n, generator=g, device="cuda:0") < 0.3)
    size = lc.lc_encode(w, tracked, 3, out); blobs.append(out[:size].clone()); lc.lc_decode(blobs[-1], tracked)
for count in (5, 6, 7, 8, 15):
    rec = w0.clone(); lc.lc_decode_many(blobs[:count], rec)
    ref = w0.cpu().numpy()
    for b in blobs[:count]: orc.decode(b.cpu().numpy(), ref)
    assert np.array_equal(rec.cpu().numpy().view(np.uint32), ref.view(np.uint32)), count
prof_on = lc.lc_profile(True); rec = w0.clone(); lc.lc_decode_many(blobs[:8], rec); p = lc.lc_profile_read(); lc.lc_profile(False)
assert p["k_decode_fused"][1] == 1, p                  # all 8 blobs in one sweep
print("ok")
"""


def test_fused_restore_eight_blobs_per_sweep():
    """With the occupancy floor lowered (a launch-shape knob read once per process, hence the child process)
    a sweep takes up to 8 blobs: every width of the fused kernel against the oracle."""
    import os, subprocess, sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    env = dict(os.environ, LC_TUNE_FUSED_MIN_WAVES_PER_CU="2")
    r = subprocess.run([sys.executable, "-c", FUSED_WIDE % root], env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout + r.stderr


OTHER_SHAPES = """
import sys, numpy as np, torch
sys.path.insert(0, %r)
from oracle import lc_oracle as orc
from paper_2009_13003_amd import lc
DEV = "cuda:0"
g = torch.Generator(device=DEV); g.manual_seed(77)
def pair(n, dtype):
    ref = 0.05 * torch.randn(n, generator=g, device=DEV, dtype=torch.float64 if dtype == torch.float64 else torch.float32)
    d = 1e-3 * torch.randn(n, generator=g, device=DEV, dtype=ref.dtype) * (torch.rand(n, generator=g, device=DEV) < 0.4)
    d[n // 3] = 0.3; d[n // 2 + 5] = -0.2                  # a few large deltas: most chunks lie below the kept buckets
    return (ref + d).to(dtype), ref.to(dtype)
# sweep 1 with one wavefront per compute unit: 150 batches per wavefront, so its per-batch maxima are written out in
# several rounds; the other sweeps with launch shapes of their own as well
for dtype, n, nbits in ((torch.float32, 256 * 1024 * 150 + 4321, 3), (torch.bfloat16, 256 * 2048 * 70 + 77, 4), (torch.float64, 256 * 512 * 150 + 3, 2)):
    w, ref = pair(n, dtype)
    out = lc.alloc_out(n, nbits, DEV)
    size = lc.lc_encode_t(w, ref, nbits, out)
    if dtype == torch.float64:
        e = orc.encode64(w.cpu().numpy(), ref.cpu().numpy(), nbits)
    elif dtype == torch.float32:
        e = orc.encode(w.cpu().numpy(), ref.cpu().numpy(), nbits)
    else:
        e = orc.encode_t(w.view(torch.int16).cpu().numpy().view(np.uint16), ref.view(torch.int16).cpu().numpy().view(np.uint16), nbits, orc.DT_BF16)
    got = out[:size].cpu().numpy()
    assert got.size == e.size and np.array_equal(got, e), (str(dtype), got.size, e.size)
    rec = ref.clone()
    assert lc.lc_decode_t(out[:size], rec) == size
    again = lc.alloc_out(n, nbits, DEV)
    assert lc.lc_encode_t(w, rec, nbits, again) > 0        # (the restored state is a valid reference for the next checkpoint)
    print("ok", dtype, flush=True)
print("ok")
"""


def test_sweeps_under_other_launch_shapes():
    """The launch-shape knobs are read once per process, hence the child process: sweep 1 with a single wavefront per
    compute unit (every wavefront then walks 150 batches and hands in its per-batch maxima in several rounds), the
    coding and restoring sweeps with fewer wavefronts than they take by themselves; fp32, bf16 and fp64 blobs against the oracle."""
    import os, subprocess, sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    env = dict(os.environ, LC_TUNE_HIST_THREADS="64", LC_TUNE_HIST_BLOCKS_PER_CU="1", LC_TUNE_PACK_WAVES_PER_CU="3",
               LC_TUNE_DECODE_BLOCKS_PER_CU="2")
    r = subprocess.run([sys.executable, "-c", OTHER_SHAPES % root], env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout + r.stderr


# ---------------------------------------------------------------- code table caching (Section 3.2)
def cached_step(lc, w, ref, nbits, out, cache_gpu, cache_cpu):
    """One lc_encode_cached on both sides with their own caches; compares blob, verdict and cache."""
    size, used = lc.lc_encode_cached(w, ref, nbits, out, cache_gpu)
    blob_cpu, used_cpu = orc.encode_cached(w.cpu().numpy(), ref.cpu().numpy(), nbits, cache_cpu)
    blob_gpu = out[:size].cpu().numpy()
    assert used == used_cpu
    assert blob_gpu.size == blob_cpu.size and np.array_equal(blob_gpu, blob_cpu), first_diff(blob_gpu, blob_cpu)
    assert np.array_equal(cache_gpu.cpu().numpy()[:4 * orc.CACHE_WORDS].view(np.uint32), cache_cpu)
    return out[:size].clone(), used


@pytest.mark.parametrize("nbits,n", [(3, 9 * 16384 + 1234), (4, 5 * 16384), (2, 16384 + 3), (3, 700)])
def test_cached_encode_chain_matches_oracle(lc, nbits, n):
    """A chain of checkpoints through lc_encode_cached: blob, hit/miss verdict and cache content equal the
    oracle's at every step; hits and misses both occur; the restored state equals that of plain encodes."""
    g = torch.Generator(device=DEV); g.manual_seed(100 + nbits)
    w = 0.05 * torch.randn(n, generator=g, device=DEV)
    tracked = w.clone()
    plain_tracked = w.clone()
    out = lc.alloc_out(n, nbits, DEV)
    out2 = lc.alloc_out(n, nbits, DEV)
    cache_gpu, cache_cpu = lc.new_cache(DEV), orc.new_cache()
    verdicts = []
    for t in range(8):
        u = torch.rand(n, generator=g, device=DEV) - 0.5
        d = -1e-3 * torch.sign(u) * torch.log1p(-2 * u.abs().clamp_(max=0.49999997))
        d[:4] = torch.tensor([0.02, -0.02, 0.011, -0.011], device=DEV)      # same top of the range every step
        if t == 5:
            d[9] = 0.4                                                        # a new largest exponent: miss
        w = w + d
        blob, used = cached_step(lc, w, tracked, nbits, out, cache_gpu, cache_cpu)
        verdicts.append(used)
        # the plain encode of the same checkpoint restores the same weights
        size2 = lc.lc_encode(w, plain_tracked, nbits, out2)
        lc.lc_decode(blob, tracked)
        lc.lc_decode(out2[:size2], plain_tracked)
        assert torch.equal(tracked.view(torch.int32), plain_tracked.view(torch.int32)), t
    assert verdicts[0] is False and verdicts[5] is False and any(verdicts[1:5]), verdicts


@pytest.mark.parametrize("tdt", [torch.bfloat16, torch.float16])
def test_cached_and_async_encode_of_16_bit_parameters(lc, tdt):
    """lc_encode_cached_t / lc_encode_async_t: a chain of bf16 / fp16 checkpoints, blob, verdict and cache as the
    oracle's at every step, hits and a miss both occur; the asynchronous form gives the same blobs."""
    code = orc.DT_BF16 if tdt == torch.bfloat16 else orc.DT_F16
    nbits, n = 3, 7 * 16384 + 321
    g = torch.Generator(device=DEV); g.manual_seed(321)
    w = (0.05 * torch.randn(n, generator=g, device=DEV)).to(tdt)
    tracked = w.clone()
    out, out2 = lc.alloc_out(n, nbits, DEV), lc.alloc_out(n, nbits, DEV)
    cache_gpu, cache_cpu, cache_async = lc.new_cache(DEV), orc.new_cache(), lc.new_cache(DEV)
    verdicts = []
    for t in range(6):
        d = 2e-3 * torch.randn(n, generator=g, device=DEV)
        d[:4] = torch.tensor([0.02, -0.02, 0.011, -0.011], device=DEV)
        if t == 4:
            d[9] = 0.4                                                        # a new largest exponent: miss
        w = (w.float() + d).to(tdt)
        size, used = lc.lc_encode_cached_t(w, tracked, nbits, out, cache_gpu)
        blob_cpu, used_cpu = orc.encode_cached_t(raw16(w), raw16(tracked), nbits, code, cache_cpu)
        blob_gpu = out[:size].cpu().numpy()
        assert used == used_cpu, t
        assert blob_gpu.size == blob_cpu.size and np.array_equal(blob_gpu, blob_cpu), first_diff(blob_gpu, blob_cpu)
        assert np.array_equal(cache_gpu.cpu().numpy()[:4 * orc.CACHE_WORDS].view(np.uint32), cache_cpu)
        verdicts.append(used)
        ticket = lc.lc_encode_async_t(w, tracked, nbits, out2, cache_async)
        size2, used2 = lc.lc_encode_wait(ticket)
        assert size2 == size and used2 == used and torch.equal(out2[:size2], out[:size])
        ref_h = raw16(tracked)
        orc.decode_t(blob_cpu, ref_h, code)
        assert lc.lc_decode_t(out, tracked) == size
        assert np.array_equal(raw16(tracked).view(np.uint16), ref_h.view(np.uint16))
    assert verdicts[0] is False and verdicts[4] is False and any(verdicts[1:4]), verdicts
    ticket = lc.lc_encode_async_t(w, tracked, nbits, out2)                    # without a cache: lc_encode_t's blob
    size2, used2 = lc.lc_encode_wait(ticket)
    assert not used2 and size2 == lc.lc_encode_t(w, tracked, nbits, out) and torch.equal(out2[:size2], out[:size2])


def test_cached_encode_edge_cases(lc):
    nbits, n = 3, 2 * 16384 + 99
    w, w_ref = laplace_case(n, seed=41)
    out = lc.alloc_out(n, nbits, DEV)
    cache_gpu, cache_cpu = lc.new_cache(DEV), orc.new_cache()
    cached_step(lc, w, w_ref, nbits, out, cache_gpu, cache_cpu)
    _, used = cached_step(lc, w, w_ref, nbits, out, cache_gpu, cache_cpu)          # same checkpoint again: hit
    assert used
    _, used = cached_step(lc, w, w_ref, 2, out, cache_gpu, cache_cpu)              # other nbits: miss
    assert not used
    # unaligned inputs take the plain path of the sweep
    buf_w, buf_r = torch.zeros(n + 4, device=DEV), torch.zeros(n + 4, device=DEV)
    buf_w[1:1 + n] = w; buf_r[1:1 + n] = w_ref
    cached_step(lc, buf_w[1:1 + n], buf_r[1:1 + n], 2, out, cache_gpu, cache_cpu)
    _, used = cached_step(lc, buf_w[1:1 + n], buf_r[1:1 + n], 2, out, cache_gpu, cache_cpu)
    assert used
    # a damaged cache is not used, and is repaired
    good = cache_gpu.clone()
    for word, value in ((0, 2), (4, int(good[16:20].view(torch.int32).item()) ^ 1), (20, 9)):
        cache_gpu.copy_(good)
        cache_gpu.view(torch.int32)[word] = value
        cache_cpu[:] = cache_gpu.cpu().numpy()[:4 * orc.CACHE_WORDS].view(np.uint32)
        _, used = cached_step(lc, buf_w[1:1 + n], buf_r[1:1 + n], 2, out, cache_gpu, cache_cpu)
        assert not used
        assert torch.equal(cache_gpu, good)
    # non-finite delta: error, cache untouched
    bad = w.clone(); bad[5] = float("nan")
    cache_gpu.copy_(good)
    with pytest.raises(lc.LcError) as e:
        lc.lc_encode_cached(bad, w_ref, 2, out, cache_gpu)
    assert e.value.status == lc.ERR_NONFINITE and torch.equal(cache_gpu, good)
    # the call after an error, and plain encodes in between, are unaffected
    check_case(lc, w, w_ref, 3, "plain after cached")
    cache_cpu[:] = good.cpu().numpy()[:4 * orc.CACHE_WORDS].view(np.uint32)
    _, used = cached_step(lc, buf_w[1:1 + n], buf_r[1:1 + n], 2, out, cache_gpu, cache_cpu)
    assert used
    # empty vector, and bad arguments
    z = torch.empty(0, device=DEV)
    c0, c0_cpu = lc.new_cache(DEV), orc.new_cache()
    cached_step(lc, z, z, 3, lc.alloc_out(0, 3, DEV), c0, c0_cpu)
    cached_step(lc, z, z, 3, lc.alloc_out(0, 3, DEV), c0, c0_cpu)
    with pytest.raises(lc.LcError) as e:
        lc.lc_encode_cached(w, w_ref, 3, out, torch.zeros(lc.CACHE_BYTES + 16, dtype=torch.uint8, device=DEV)[4:])   # misaligned cache
    assert e.value.status == lc.ERR_BADARG


def test_cached_encode_stale_table_never_outgrows_the_bound(lc):
    """A table cached on skewed populations, then the same buckets with the populations reversed: under the cached
    lengths the blob would need about 7 bits per element where lc_encode_bound promises 3, so the reuse is refused
    (blob = lc_encode's, used = 0), as in the oracle; nothing is written behind the stated bound."""
    n, nbits = 4 * 16384, 3
    mags = [2.0 ** -e for e in range(1, 8)]
    skew = [n >> (j + 1) for j in range(7)]
    skew.append(n - sum(skew))

    def delta(counts, seed):
        d = torch.cat([torch.full((c,), m) for c, m in zip(counts[:-1], mags)] + [torch.zeros(counts[-1])])
        g = torch.Generator(); g.manual_seed(seed)
        return d[torch.randperm(n, generator=g)].to(DEV)

    zero = torch.zeros(n, device=DEV)
    bound = lc.lc_encode_bound(n, nbits)
    buf = torch.full((bound + 65536,), 0x5A, dtype=torch.uint8, device=DEV)     # guard bytes behind the bound
    out = buf[:bound]
    cache_gpu, cache_cpu = lc.new_cache(DEV), orc.new_cache()
    _, used = cached_step(lc, delta(skew, 0), zero, nbits, out, cache_gpu, cache_cpu)
    assert not used and [int(x) for x in cache_cpu[20:28]] == [1, 2, 3, 4, 5, 6, 7, 7]
    d2 = delta(skew[::-1], 1)
    blob, used = cached_step(lc, d2, zero, nbits, out, cache_gpu, cache_cpu)
    assert not used and blob.numel() <= bound
    assert bool((buf[bound:] == 0x5A).all())
    size = lc.lc_encode(d2, zero, nbits, out)
    assert size == blob.numel() and torch.equal(out[:size], blob)
    # the asynchronous form takes the same decision
    cache_async = lc.new_cache(DEV)
    for counts, seed in ((skew, 0), (skew[::-1], 1)):
        ticket = lc.lc_encode_async(delta(counts, seed), zero, nbits, out, cache_async)
        size2, used2 = lc.lc_encode_wait(ticket)
        assert not used2
    assert size2 == size and torch.equal(out[:size], blob) and bool((buf[bound:] == 0x5A).all())


# ---------------------------------------------------------------- asynchronous encode (Section 3.2)
def test_async_encode_equals_sync_and_releases_inputs(lc):
    """lc_encode_async + lc_encode_wait give lc_encode's blob; after lc_encode_release_inputs the caller may
    overwrite w on another stream at once (the overwrite is enqueued while the encode is still running)."""
    n, nbits = 4096 * 16384 + 321, 3                    # 67 M elements: the encode (~0.25 ms) outlasts the host's next enqueue
    w, w_ref = laplace_case(n, seed=51)
    out_sync = lc.alloc_out(n, nbits, DEV)
    size_sync = lc.lc_encode(w, w_ref, nbits, out_sync)
    expected = out_sync[:size_sync].clone()
    enc_stream, other = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for rep in range(3):
        w_live = w.clone()
        out = lc.alloc_out(n, nbits, DEV)
        torch.cuda.synchronize()
        ticket = lc.lc_encode_async(w_live, w_ref, nbits, out, stream=enc_stream)
        lc.lc_encode_release_inputs(ticket, other)
        with torch.cuda.stream(other):
            w_live.add_(1.0)                            # the "optimizer step"
        size, used = lc.lc_encode_wait(ticket)
        torch.cuda.synchronize()
        assert size == size_sync and not used and torch.equal(out[:size], expected), rep
        assert torch.equal(w_live, w + 1.0)


def test_async_encode_many_in_flight_and_mixed_with_other_calls(lc):
    nbits = 3
    cases = [laplace_case(16384 * k + 7 * k, seed=60 + k) for k in range(1, 7)]
    outs = [lc.alloc_out(w.numel(), nbits, DEV) for w, _ in cases]
    streams = [torch.cuda.Stream() for _ in range(3)]
    torch.cuda.synchronize()
    tickets = [lc.lc_encode_async(w, r, nbits, o, stream=streams[i % 3]) for i, ((w, r), o) in enumerate(zip(cases, outs))]
    assert len(set(tickets)) == len(tickets)
    # a synchronous call on yet another stream while those are in flight: ordered after them, scratch intact
    w0, r0 = cases[0]
    blob0 = check_case(lc, w0, r0, nbits, "sync while async in flight")
    for t, (w, r), o in reversed(list(zip(tickets, cases, outs))):
        size, used = lc.lc_encode_wait(t)
        ref = orc.encode(w.cpu().numpy(), r.cpu().numpy(), nbits)
        assert size == ref.size and np.array_equal(o[:size].cpu().numpy(), ref)
    # with a cache: first call fills, second hits; verdict comes back through the ticket
    w, r = cases[3]
    cache, cache_cpu = lc.new_cache(DEV), orc.new_cache()
    for expect_used in (False, True):
        t = lc.lc_encode_async(w, r, nbits, outs[3], cache=cache)
        size, used = lc.lc_encode_wait(t)
        ref, used_cpu = orc.encode_cached(w.cpu().numpy(), r.cpu().numpy(), nbits, cache_cpu)
        assert used == used_cpu == expect_used and np.array_equal(outs[3][:size].cpu().numpy(), ref)
    # errors: a finished ticket cannot be waited for twice; more calls in flight than tickets
    with pytest.raises(lc.LcError) as e:
        lc.lc_encode_wait(tickets[0])
    assert e.value.status == lc.ERR_BADARG
    with pytest.raises(lc.LcError) as e:
        lc.lc_encode_release_inputs(99)
    assert e.value.status == lc.ERR_BADARG
    held = [lc.lc_encode_async(w, r, nbits, outs[3]) for _ in range(lc.MAX_TICKETS)]
    with pytest.raises(lc.LcError) as e:
        lc.lc_encode_async(w, r, nbits, outs[3])
    assert e.value.status == lc.ERR_BADARG
    for t in held:
        lc.lc_encode_wait(t)
    # non-finite delta: the error arrives at the wait
    bad = w.clone(); bad[11] = float("inf")
    t = lc.lc_encode_async(bad, r, nbits, outs[3])
    with pytest.raises(lc.LcError) as e:
        lc.lc_encode_wait(t)
    assert e.value.status == lc.ERR_NONFINITE
    check_case(lc, w, r, nbits, "after async error")


# ---------------------------------------------------------------- bf16 / fp16 parameters
def raw16(t):
    """The oracle's view of a 16-bit tensor: uint16 bit patterns for bf16, numpy float16 for fp16."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16).copy()
    return t.cpu().numpy().copy()


@pytest.mark.parametrize("tdt", [torch.bfloat16, torch.float16])
@pytest.mark.parametrize("n,nbits,offset", [(5 * 16384 + 777, 3, 0), (16384, 4, 0), (3 * 16384 + 5, 2, 1), (100, 3, 3), (0, 3, 0)])
def test_16_bit_parameters_match_oracle(lc, tdt, n, nbits, offset):
    """bf16 / fp16 parameters: blob byte-identical to the oracle's, restored 16-bit values bit-identical;
    `offset` elements of misalignment take the guarded paths."""
    code = orc.DT_BF16 if tdt == torch.bfloat16 else orc.DT_F16
    g = torch.Generator(device=DEV); g.manual_seed(200 + n % 97 + nbits)
    buf_r = (0.05 * torch.randn(n + 8, generator=g, device=DEV)).to(tdt)
    buf_w = (buf_r.float() + 2e-3 * torch.randn(n + 8, generator=g, device=DEV)).to(tdt)
    buf_w[::7] = buf_r[::7]                                              # some exactly unchanged
    w, w_ref = buf_w[offset:offset + n], buf_r[offset:offset + n]
    out = lc.alloc_out(n, nbits, DEV); out.fill_(0x5A)
    size = lc.lc_encode_t(w, w_ref, nbits, out)
    blob_cpu = orc.encode_t(raw16(w), raw16(w_ref), nbits, code)
    blob_gpu = out[:size].cpu().numpy()
    assert blob_gpu.size == blob_cpu.size and np.array_equal(blob_gpu, blob_cpu), first_diff(blob_gpu, blob_cpu)
    rec = buf_r.clone()
    assert lc.lc_decode_t(out, rec[offset:offset + n]) == size
    ref_h = raw16(w_ref)
    orc.decode_t(blob_cpu, ref_h, code)
    assert np.array_equal(raw16(rec[offset:offset + n]).view(np.uint16), ref_h.view(np.uint16))
    assert torch.equal(rec[:offset].view(torch.int16), buf_r[:offset].view(torch.int16))          # nothing outside the range
    assert torch.equal(rec[offset + n:].view(torch.int16), buf_r[offset + n:].view(torch.int16))


@pytest.mark.parametrize("offset", [0, 1])
def test_bf16_restore_rounds_ties_subnormals_and_overflow_like_the_oracle(lc, offset):
    """Restored bf16 values that land exactly between two neighbours (both parities), on half the smallest
    subnormal (either sign) and above the largest finite value: the vector path narrows with the hardware
    conversion, the guarded path (offset 1) with integers, the oracle with integers."""
    def bf(bits):
        return torch.tensor(bits, dtype=torch.int16).view(torch.bfloat16)
    # (w_ref, [w choices]) as bf16 bit patterns
    one, one1 = 0x3F80, 0x3F81                    # 1, 1 + 2^-7
    groups = [
        (one, [0x3F82, 0x3F83]),                  # delta 2^-6, 3*2^-7 -> rep 5*2^-8: 1 + 5*2^-8 is a tie, even neighbour below
        (one1, [0x3F83, 0x3F84]),                 # same deltas from an odd mantissa: tie, even neighbour above
        (0x8080, [0x0000, 0x0001]),               # w_ref = -2^-126, w in {0, 2^-133}: rep 2^-126 (1 + 2^-8) -> +2^-134
        (0x8081, [0x8001, 0x0000]),               # w_ref = -2^-126 (1 + 2^-7): restored -2^-134
        (0x7F7D, [0x7F7F]),                       # largest finite minus 2 ulp, delta 2 ulp
        (0x0000, [0x7C60]),                       # delta 1.75 * 2^121 in the same bucket: rep 2.75 ulp -> above the largest finite
    ]
    reps = 2600
    r_bits, w_bits = [], []
    for k in range(reps):
        for ref, ws in groups:
            r_bits.append(ref); w_bits.append(ws[k % len(ws)])
    n = len(r_bits)
    to_i16 = lambda v: [x - 65536 if x >= 32768 else x for x in v]
    buf_r = torch.zeros(n + 8, dtype=torch.bfloat16); buf_w = torch.zeros(n + 8, dtype=torch.bfloat16)
    buf_r[offset:offset + n] = bf(to_i16(r_bits)); buf_w[offset:offset + n] = bf(to_i16(w_bits))
    buf_r, buf_w = buf_r.to(DEV), buf_w.to(DEV)
    w, w_ref = buf_w[offset:offset + n], buf_r[offset:offset + n]
    nbits = 3
    out = lc.alloc_out(n, nbits, DEV)
    size = lc.lc_encode_t(w, w_ref, nbits, out)
    blob_cpu = orc.encode_t(raw16(w), raw16(w_ref), nbits, orc.DT_BF16)
    assert np.array_equal(out[:size].cpu().numpy(), blob_cpu)
    rec = buf_r.clone()
    assert lc.lc_decode_t(out, rec[offset:offset + n]) == size
    ref_h = raw16(w_ref)
    orc.decode_t(blob_cpu, ref_h, orc.DT_BF16)
    got = raw16(rec[offset:offset + n])
    assert np.array_equal(got, ref_h)
    per_group = got[:len(groups) * 2].reshape(2, len(groups))
    assert per_group[0].tolist() == [0x3F82, 0x3F84, 0x0000, 0x8000, 0x7F80, 0x7C30]      # the cases the groups aim at do occur
    assert torch.equal(rec[:offset].view(torch.int16), buf_r[:offset].view(torch.int16))
    assert torch.equal(rec[offset + n:].view(torch.int16), buf_r[offset + n:].view(torch.int16))


def test_element_type_mismatch_is_refused(lc):
    n, nbits = 16384 + 9, 3
    w, w_ref = laplace_case(n, seed=70)
    out = lc.alloc_out(n, nbits, DEV)
    lc.lc_encode(w, w_ref, nbits, out)
    as_bf16 = w_ref.to(torch.bfloat16)
    before = as_bf16.clone()
    with pytest.raises(lc.LcError) as e:
        lc.lc_decode_t(out, as_bf16)                        # an fp32 blob into bf16 parameters
    assert e.value.status == lc.ERR_BADARG and torch.equal(as_bf16.view(torch.int16), before.view(torch.int16))
    lc.lc_encode_t(w.to(torch.bfloat16), as_bf16, nbits, out)
    rec = w_ref.clone()
    with pytest.raises(lc.LcError) as e:
        lc.lc_decode(out, rec)                              # a bf16 blob into fp32 parameters
    assert e.value.status == lc.ERR_BADARG and torch.equal(rec, w_ref)
    with pytest.raises(lc.LcError) as e:
        lc.lc_decode_many([out], rec)
    assert e.value.status == lc.ERR_BADARG and torch.equal(rec, w_ref)


# ---------------------------------------------------------------- batched per-tensor encode
def batch_case(seed, sizes, scales, offsets=None):
    g = torch.Generator(device=DEV); g.manual_seed(seed)
    ws, refs = [], []
    for i, (n, sc) in enumerate(zip(sizes, scales)):
        off = 0 if offsets is None else offsets[i]
        buf_r = 0.05 * torch.randn(n + off, generator=g, device=DEV)
        u = torch.rand(n + off, generator=g, device=DEV) - 0.5
        buf_w = buf_r - sc * torch.sign(u) * torch.log1p(-2 * u.abs().clamp_(max=0.49999997))
        ws.append(buf_w[off:]); refs.append(buf_r[off:])
    return ws, refs


def check_batch(lc, ws, refs, nbits, expect_status=None):
    outs = [lc.alloc_out(w.numel(), nbits, DEV) for w in ws]
    for o in outs:
        o.fill_(0x3C)
    sizes = lc.lc_encode_batch(ws, refs, nbits, outs)
    for t, (w, r, o, size) in enumerate(zip(ws, refs, outs, sizes)):
        if expect_status and t in expect_status:
            assert size == -expect_status[t], (t, size)
            hdr = o[:512].cpu().numpy()
            assert lc.lc_blob_info(hdr.tobytes())["status"] == expect_status[t]
            continue
        blob_cpu = orc.encode(w.cpu().numpy(), r.cpu().numpy(), nbits)
        blob_gpu = o[:size].cpu().numpy()
        assert size == blob_cpu.size and np.array_equal(blob_gpu, blob_cpu), "tensor %d: %s" % (t, first_diff(blob_gpu, blob_cpu))
        rec = r.clone()
        assert lc.lc_decode(o, rec) == size
        ref_h = r.cpu().numpy()
        orc.decode(blob_cpu, ref_h)
        assert np.array_equal(bits(rec.cpu().numpy()), bits(ref_h)), t
    # the batched restore of the same list: every tensor as its own lc_decode would leave it
    good = [t for t in range(len(ws)) if not (expect_status and t in expect_status)]
    recs = [refs[t].clone() for t in good]
    used = lc.lc_decode_batch([outs[t] for t in good], recs)
    assert used == [sizes[t] for t in good]
    for t, rec in zip(good, recs):
        ref_h = refs[t].cpu().numpy()
        orc.decode(outs[t][:sizes[t]].cpu().numpy(), ref_h)
        assert np.array_equal(bits(rec.cpu().numpy()), bits(ref_h)), t
    return sizes


@pytest.mark.parametrize("nbits", [2, 3, 4])
def test_batched_encode_one_table_per_tensor(lc, nbits):
    """Every tensor of a batched call gets exactly the blob a call of its own would give (oracle, byte for byte):
    sizes from empty to several groups of chunks, scales over four decades, so that every tensor keeps its own buckets."""
    sizes = [5 * 16384 + 777, 0, 1, 100, 16384, 16385, 70 * 16384 + 5, 3 * 16384, 2 * 16384 + 1, 130 * 16384, 64, 16384 * 64]
    scales = [10.0 ** (-6 + 4 * (i % 5) / 4) for i in range(len(sizes))]
    ws, refs = batch_case(300 + nbits, sizes, scales)
    check_batch(lc, ws, refs, nbits)
    # a different table per tensor is really in play: the kept buckets of a small-scale and a large-scale tensor differ
    outs = [lc.alloc_out(w.numel(), nbits, DEV) for w in ws]
    lc.lc_encode_batch(ws, refs, nbits, outs)
    k0 = lcb1_reader.parse_header(outs[0][:512].cpu().numpy())
    k4 = lcb1_reader.parse_header(outs[4][:512].cpu().numpy())
    assert k0["slots"][0]["bucket"] != k4["slots"][0]["bucket"]


def test_batched_encode_edge_cases(lc):
    nbits = 3
    # unaligned tensors, a single tensor, many tiny tensors
    ws, refs = batch_case(310, [3 * 16384 + 9, 16384, 5000], [1e-3, 1e-4, 1e-2], offsets=[1, 3, 2])
    check_batch(lc, ws, refs, nbits)
    ws, refs = batch_case(311, [9 * 16384 + 1], [1e-3])
    check_batch(lc, ws, refs, nbits)
    ws, refs = batch_case(312, [37 + 11 * i for i in range(200)], [1e-3] * 200)
    check_batch(lc, ws, refs, nbits)
    # a tensor with a non-finite delta: its blob is a header that says so, the others are untouched by it
    ws, refs = batch_case(313, [2 * 16384 + 5, 4 * 16384, 999], [1e-3, 1e-4, 1e-2])
    ws[1] = ws[1].clone(); ws[1][12345] = float("nan")
    sizes = check_batch(lc, ws, refs, nbits, expect_status={1: 2})
    assert sizes[0] > 512 and sizes[2] > 512
    # calls of the other kinds afterwards find their scratch in order
    w, r = laplace_case(3 * 16384 + 5, seed=314)
    check_case(lc, w, r, 3, "single after batch")
    # bad arguments
    with pytest.raises(lc.LcError) as e:
        lc.lc_encode_batch([w], [r], 5, [lc.alloc_out(w.numel(), 4, DEV)])
    assert e.value.status == lc.ERR_BADARG


def test_batched_decode_bad_blobs_leave_their_tensor_alone(lc):
    nbits = 3
    ws, refs = batch_case(320, [3 * 16384 + 9, 2 * 16384, 777, 5 * 16384], [1e-3, 1e-4, 1e-2, 1e-3])
    outs = [lc.alloc_out(w.numel(), nbits, DEV) for w in ws]
    sizes = lc.lc_encode_batch(ws, refs, nbits, outs)
    blobs = [o[:s].clone() for o, s in zip(outs, sizes)]
    blobs[1][512 + 4] ^= 1                               # offset table of tensor 1
    blobs[2][20] ^= 3                                    # K in the header of tensor 2
    recs = [r.clone() for r in refs]
    used = lc.lc_decode_batch(blobs, recs)
    assert used[1] == -lc.ERR_BAD_BLOB and used[2] == -lc.ERR_BAD_BLOB and used[0] == sizes[0] and used[3] == sizes[3]
    assert torch.equal(recs[1], refs[1]) and torch.equal(recs[2], refs[2])
    for t in (0, 3):
        ref_h = refs[t].cpu().numpy()
        orc.decode(blobs[t].cpu().numpy(), ref_h)
        assert np.array_equal(bits(recs[t].cpu().numpy()), bits(ref_h))
    # a blob for a vector of another length
    recs = [refs[0].clone(), refs[1].clone()]
    used = lc.lc_decode_batch([outs[1][:sizes[1]], outs[1][:sizes[1]]], recs)
    assert used[0] == -lc.ERR_BADARG and used[1] == sizes[1] and torch.equal(recs[0], refs[0])
    # a payload bit flipped: same verdict and, if accepted, same weights as the oracle
    damaged = outs[3][:sizes[3]].clone()
    damaged[512 + 16 * 2 + 128 + 700] ^= 0x20
    ref_h = refs[3].cpu().numpy()
    try:
        orc.decode(damaged.cpu().numpy(), ref_h); ok = True
    except orc.OracleError:
        ok = False
    recs = [refs[3].clone()]
    used = lc.lc_decode_batch([damaged], recs)
    if ok:
        assert used[0] == sizes[3] and np.array_equal(bits(recs[0].cpu().numpy()), bits(ref_h))
    else:
        assert used[0] == -lc.ERR_BAD_BLOB


def test_chunks_of_merged_symbols_only(lc):
    """Deltas that touch a few chunks only: the other chunks hold the merged symbol throughout and are left
    alone by the restore (plain, batched, several blobs at once).  Same weights as the oracle's, and a bit
    flipped inside such a chunk's payload gives the oracle's verdict."""
    nbits, nchunks = 3, 40
    n = nchunks * 16384 + 77
    g = torch.Generator(device=DEV); g.manual_seed(91)
    w0 = 0.05 * torch.randn(n, generator=g, device=DEV)
    deltas = []
    for t in range(5):
        d = torch.zeros(n, device=DEV)
        lo = (7 * t + 3) * 16384 + 100
        d[lo:lo + 20000] = 1e-3 * torch.randn(20000, generator=g, device=DEV)
        deltas.append(d)
    tracked, blobs = encode_chain(lc, w0, deltas, [nbits] * 5)
    hdr = lcb1_reader.parse_header(blobs[0].cpu().numpy())
    K = hdr["K"]
    assert hdr["slots"][K]["len"] == 1 and all(s["len"] > 1 for s in hdr["slots"][:K])       # the merged symbol codes as "0"
    ref = oracle_restore(w0, blobs)
    rec = w0.clone()
    for b in blobs:
        lc.lc_decode(b, rec)
    assert np.array_equal(bits(rec.cpu().numpy()), bits(ref))
    rec = w0.clone()
    lc.lc_decode_many(blobs, rec)
    assert np.array_equal(bits(rec.cpu().numpy()), bits(ref))
    rec = [w0.clone()]
    lc.lc_decode_batch([blobs[0]], rec)
    ref0 = w0.cpu().numpy(); orc.decode(blobs[0].cpu().numpy(), ref0)
    assert np.array_equal(bits(rec[0].cpu().numpy()), bits(ref0))
    # damage inside a chunk of merged symbols: chunk 0 of blob 0 (the delta starts in chunk 3)
    area = 512 + (4 * (nchunks + 2) + 15) // 16 * 16
    for byte in (128 + 5, 128 + 1000):
        damaged = blobs[0].clone()
        damaged[area + byte] ^= 0x40
        ref_h = w0.cpu().numpy()
        try:
            orc.decode(damaged.cpu().numpy(), ref_h); ok = True
        except orc.OracleError as e:
            assert e.status == 4; ok = False
        for call in ("one", "many", "batch"):
            rec = w0.clone()
            try:
                if call == "one":
                    lc.lc_decode(damaged, rec)
                elif call == "many":
                    lc.lc_decode_many([damaged], rec)
                else:
                    assert lc.lc_decode_batch([damaged], [rec])[0] == (damaged.numel() if ok else -lc.ERR_BAD_BLOB)
                got_ok = True
            except lc.LcError as e:
                assert e.status == lc.ERR_BAD_BLOB; got_ok = False
            if call != "batch":
                assert got_ok == ok, call
            if ok:
                assert np.array_equal(bits(rec.cpu().numpy()), bits(ref_h)), call


def quiet_chunk_case(n, seed, quiet, tiny=2.0 ** -30):
    """Deltas of four binades (eight buckets) everywhere, except in the chunks listed in `quiet`, whose
    deltas are far smaller (or zero): those chunks lie below every kept bucket."""
    g = torch.Generator(device=DEV); g.manual_seed(seed)
    w_ref = 0.05 * torch.randn(n, generator=g, device=DEV)
    e = torch.randint(10, 14, (n,), generator=g, device=DEV).float()
    d = torch.exp2(-e) * (1 + torch.rand(n, generator=g, device=DEV))
    d = d * (2 * torch.randint(0, 2, (n,), generator=g, device=DEV).float() - 1)
    for k, c in enumerate(quiet):
        lo, hi = c * 16384, min(n, (c + 1) * 16384)
        if k % 3 == 2:
            d[lo:hi] = 0
        else:
            d[lo:hi] = tiny * (1 + torch.rand(hi - lo, generator=g, device=DEV)) * (1 - 2 * (k % 2))
    # w - w_ref must reproduce d's bucket: use a reference of zeros where d is tiny
    w_ref = torch.where(d.abs() < 1e-6, torch.zeros_like(w_ref), w_ref)
    return w_ref + d, w_ref


@pytest.mark.parametrize("nbits", [2, 3, 4])
def test_fp64_encode_of_quiet_chunks_and_parts(lc, nbits):
    """binary64 parameters: whole chunks below every kept bucket are passed over, and a chunk of which only a few
    4 KiB parts (512 doubles) hold a kept element is coded part by part: loud elements in the first, the last and a
    middle part of otherwise quiet chunks, more loud parts than the quarter that still goes by parts, a quiet ragged
    tail with one loud element, an unaligned vector.  Blob and restore as the oracle's."""
    nchunks = 70
    n = nchunks * 16384 + 1500
    quiet = [0, 1, 5, 63, 64, 65] + list(range(20, 40)) + [69, 70]
    w, w_ref = quiet_chunk_case(n, 500 + nbits, quiet)
    w, w_ref = w.double(), w_ref.double()
    loud = lambda i: float(w_ref[i]) + 2.0 ** -11
    for c, offs in ((1, [3]), (5, [0, 16383]), (22, [512 * 7 + 5, 512 * 8 - 1]), (25, [512 * k + 17 for k in range(8)]),
                    (26, [512 * k + 17 for k in range(9)]), (30, [512 * k for k in range(32)]), (70, [1499]), (69, [16384 - 512, 100])):
        for o in offs:
            w[c * 16384 + o] = loud(c * 16384 + o)
    check_case64(lc, w, w_ref, nbits, "fp64 quiet chunks and parts")
    check_case64(lc, w[1:], w_ref[1:], nbits, "fp64 quiet chunks, unaligned")
    check_case64(lc, w[:3 * 16384 + 700], w_ref[:3 * 16384 + 700], nbits, "fp64 quiet, short ragged tail")


@pytest.mark.parametrize("nbits", [2, 3, 4])
def test_batched_encode_of_chunks_below_their_tensors_kept_buckets(lc, nbits):
    """A batched call passes over full chunks whose largest delta lies below every kept bucket of *their own* tensor
    (the counting sweep notes every chunk's maximum, a list kernel tells them apart once the tables exist): quiet
    chunks at the start and the end of tensors, at group borders, whole quiet tensors (all deltas zero; all tiny but
    one), a tensor whose quiet level is another tensor's kept range, a ragged last chunk that is quiet (read anyway),
    an unaligned tensor, 16-bit tensors, and a non-finite tensor in between."""
    C = 16384
    specs = [  # (chunks, extra elements, quiet chunks, tiny level, offset)
        (70, 123, [0, 1, 2, 63, 64, 65, 69, 70], 2.0 ** -30, 0),
        (3, 0, [0, 1, 2], 2.0 ** -30, 0),                     # all tiny: the tiny values are this tensor's own kept buckets
        (5, 17, [4, 5], 2.0 ** -30, 0),                       # last full chunk and the ragged tail quiet
        (9, 0, [1, 2, 3, 4, 5, 6, 7], 2.0 ** -13, 0),         # quiet level inside the first tensors' kept range
        (6, 999, [0, 2, 4], 2.0 ** -30, 3),                   # unaligned
        (130, 1, list(range(3, 128)), 2.0 ** -28, 0),
    ]
    ws, refs = [], []
    for i, (nc, extra, quiet, tiny, off) in enumerate(specs):
        w, r = quiet_chunk_case(nc * C + extra + off, 900 + 10 * nbits + i, quiet, tiny=tiny)
        ws.append(w[off:]); refs.append(r[off:])
    # a tensor that does not change at all, and one with a single changed element in its last chunk
    z = 0.05 * torch.randn(4 * C + 5, device=DEV)
    ws.append(z.clone()); refs.append(z)
    one = z.clone(); one[3 * C + 77] += 0.25
    ws.append(one); refs.append(z)
    check_batch(lc, ws, refs, nbits)
    # the coding sweep really passed over chunks: tensor 5's blob holds 125 chunks of the merged code only
    outs = [lc.alloc_out(w.numel(), nbits, DEV) for w in ws]
    sizes = lc.lc_encode_batch(ws, refs, nbits, outs)
    hdr = lcb1_reader.parse_header(outs[5][:sizes[5]].cpu().numpy())
    K = hdr["K"]
    rec_words = 32 + C * hdr["slots"][K]["len"] // 32
    offs = outs[5][512:512 + 4 * 132].cpu().numpy().view(np.uint32)
    assert all(int(offs[c + 1]) - int(offs[c]) == rec_words for c in range(3, 128))
    # with a non-finite tensor between them the others still come out the same
    bad = ws[2].clone(); bad[C + 5] = float("inf")
    check_batch(lc, [ws[0], bad, ws[3]], [refs[0], refs[2], refs[3]], nbits, expect_status={1: 2})
    # 16-bit tensors
    for tdt in (torch.bfloat16, torch.float16):
        w16 = [w.to(tdt) for w in ws[:4]]
        r16 = [r.to(tdt) for r in refs[:4]]
        outs = [lc.alloc_out(w.numel(), nbits, DEV) for w in w16]
        sizes = lc.lc_encode_batch(w16, r16, nbits, outs)
        for t, (w, r, o, size) in enumerate(zip(w16, r16, outs, sizes)):
            blob_cpu = orc.encode_t(raw16(w), raw16(r), nbits, orc.DT_BF16 if tdt == torch.bfloat16 else orc.DT_F16)
            assert size == blob_cpu.size and np.array_equal(o[:size].cpu().numpy(), blob_cpu), (tdt, t)


@pytest.mark.parametrize("nbits", [2, 3, 4])
def test_encode_of_chunks_below_every_kept_bucket(lc, nbits):
    """Whole chunks whose deltas all fall into the merged bucket are coded without being read again, from the
    per-chunk exponent maxima of the first sweep: at the start, at group borders (63, 64), in a run, as the
    last full chunk and in the ragged tail (which is read as usual).  The merged symbol's code has one bit
    (nbits = 2) or several (nbits = 3, 4), so the repeated code does not line up with 32-bit words."""
    nchunks = 150
    n = nchunks * 16384 + 1234
    quiet = [0, 5, 63, 64] + list(range(100, 111)) + [149, 150]
    w, w_ref = quiet_chunk_case(n, 300 + nbits, quiet)
    blob = check_case(lc, w, w_ref, nbits, "quiet chunks")
    hdr = lcb1_reader.parse_header(blob)
    K = hdr["K"]
    merged_len = hdr["slots"][K]["len"]
    print("merged symbol's code length", merged_len, flush=True)
    assert merged_len == 1 if nbits == 2 else merged_len >= 2
    # unaligned arrays: the quiet chunks are still recognised, the others take the guarded path
    check_case(lc, w[3:], w_ref[3:], nbits, "quiet chunks, unaligned")
    # every full chunk quiet, and nothing but quiet chunks plus one loud element in the tail
    w2, ref2 = quiet_chunk_case(n, 310 + nbits, list(range(nchunks + 1)))
    check_case(lc, w2, ref2, nbits, "all quiet")
    w2[-5] = ref2[-5] + 0.25
    check_case(lc, w2, ref2, nbits, "all quiet but one")
    # the caller's scratch area and a second call right after (the per-chunk maxima are left cleared)
    check_case(lc, w, w_ref, nbits, "quiet chunks again")


@pytest.mark.parametrize("nbits", [2, 3, 4])
@pytest.mark.parametrize("tdt", [torch.float32, torch.bfloat16])
def test_mostly_quiet_chunks_are_coded_part_by_part(lc, nbits, tdt):
    """Chunks that lie below every kept bucket except for a few elements: the second sweep reads only the 4 KiB
    parts that the first one marked (first, middle and last part; two elements in one part; exactly a quarter of
    the parts, and one more, which takes the usual path; a ragged last chunk with a loud element in a whole part,
    in its last rows, or nowhere).  Blob and restored values as the oracle's; the decoder meets chunks with few
    kept symbols in every one of these shapes."""
    nchunks = 24
    n = nchunks * 16384 + 9 * 1024 + 300
    w, w_ref = quiet_chunk_case(n, 400 + nbits, list(range(4, nchunks + 1)), tiny=2.0 ** -22)
    part = 1024 if tdt == torch.float32 else 2048
    loud = {4: [0], 5: [7 * part + 5], 6: [16384 - 1], 7: [3 * part + 1, 3 * part + 900],
            8: [p * (16384 // 4) + 17 for p in range(4)],                        # a quarter of the parts (fp32) or more
            9: [p * part + 3 for p in range(16384 // part // 4)],                 # exactly a quarter
            10: [p * part + 3 for p in range(16384 // part // 4 + 1)],            # one more: the usual path
            11: list(range(0, 16384, 64)), 12: [8191, 8192],
            nchunks: [2 * part + 77, 9 * 1024 + 299, 8 * 1024 + 1]}            # the ragged chunk
    for c, offs in loud.items():
        for k, o in enumerate(offs):
            i = c * 16384 + o
            w[i] = w_ref[i] + (2.0 ** -10) * (1.25 + 0.5 * (k % 2)) * (1 - 2 * (k % 3 == 1))
    if tdt == torch.float32:
        check_case(lc, w, w_ref, nbits, "part by part")
        w[nchunks * 16384:] = w_ref[nchunks * 16384:]                            # a ragged chunk without a loud element
        check_case(lc, w, w_ref, nbits, "part by part, quiet tail")
        return
    rt = w_ref.to(tdt)
    wt = (rt.float() + (w - w_ref)).to(tdt)
    out = lc.alloc_out(n, nbits, DEV)
    size = lc.lc_encode_t(wt, rt, nbits, out)
    blob_cpu = orc.encode_t(raw16(wt), raw16(rt), nbits, orc.DT_BF16)
    blob_gpu = out[:size].cpu().numpy()
    assert blob_gpu.size == blob_cpu.size and np.array_equal(blob_gpu, blob_cpu), first_diff(blob_gpu, blob_cpu)
    rec = rt.clone()
    assert lc.lc_decode_t(out, rec) == size
    ref_h = raw16(rt)
    orc.decode_t(blob_cpu, ref_h, orc.DT_BF16)
    assert np.array_equal(raw16(rec).view(np.uint16), ref_h.view(np.uint16))


@pytest.mark.parametrize("tdt", [torch.bfloat16, torch.float16])
def test_encode_of_quiet_chunks_16_bit(lc, tdt):
    code = orc.DT_BF16 if tdt == torch.bfloat16 else orc.DT_F16
    nbits, n = 3, 40 * 16384 + 99
    g = torch.Generator(device=DEV); g.manual_seed(77)
    w_ref = (0.05 * torch.randn(n, generator=g, device=DEV)).to(tdt)
    w = (w_ref.float() + 2e-3 * torch.randn(n, generator=g, device=DEV)).to(tdt)
    for c in (0, 7, 8, 9, 31, 39):
        w[c * 16384:(c + 1) * 16384] = w_ref[c * 16384:(c + 1) * 16384]         # unchanged chunks
    out = lc.alloc_out(n, nbits, DEV); out.fill_(0x5A)
    size = lc.lc_encode_t(w, w_ref, nbits, out)
    blob_cpu = orc.encode_t(raw16(w), raw16(w_ref), nbits, code)
    blob_gpu = out[:size].cpu().numpy()
    assert blob_gpu.size == blob_cpu.size and np.array_equal(blob_gpu, blob_cpu), first_diff(blob_gpu, blob_cpu)
    rec = w_ref.clone()
    assert lc.lc_decode_t(out, rec) == size
    ref_h = raw16(w_ref)
    orc.decode_t(blob_cpu, ref_h, code)
    assert np.array_equal(raw16(rec).view(np.uint16), ref_h.view(np.uint16))


# ---------------------------------------------------------------- binary64 parameters
def bits64(a):
    return np.ascontiguousarray(a, dtype=np.float64).view(np.uint64)


def check_case64(lc, w, w_ref, nbits, label=""):
    """fp64 parameters: blob byte-identical to the oracle's, restored values bit-identical."""
    n = w.numel()
    print("fp64 case", label, "n=%d nbits=%d" % (n, nbits), flush=True)
    out = lc.alloc_out(n, nbits, DEV); out.fill_(0xA5)
    size = lc.lc_encode_t(w, w_ref, nbits, out)
    w_h, ref_h = w.cpu().numpy(), w_ref.cpu().numpy()
    blob_cpu = orc.encode64(w_h, ref_h, nbits)
    blob_gpu = out[:size].cpu().numpy()
    assert blob_gpu.size == blob_cpu.size and np.array_equal(blob_gpu, blob_cpu), first_diff(blob_gpu, blob_cpu)
    assert lc.lc_verify(out[:size], n, torch.float64) == size
    rec = w_ref.clone()
    assert lc.lc_decode_t(out, rec) == size
    orc.decode64(blob_cpu, ref_h)
    bad = np.nonzero(bits64(rec.cpu().numpy()) != bits64(ref_h))[0]
    assert bad.size == 0, "first differing element %d of %d" % (bad[0], bad.size)
    return blob_cpu


@pytest.mark.parametrize("n,nbits,offset", [(5 * 16384 + 777, 3, 0), (16384, 4, 0), (3 * 16384 + 5, 2, 1), (100, 3, 1),
                                            (0, 3, 0), (1, 1, 0), (40 * 16384 + 99, 1, 0), (70 * 16384 + 4097, 4, 0)])
def test_fp64_parameters_match_oracle(lc, n, nbits, offset):
    """`offset` = 1 element leaves the arrays 8-byte aligned only: the guarded paths."""
    g = torch.Generator(device=DEV); g.manual_seed(400 + n % 89 + nbits)
    buf_r = 0.05 * torch.randn(n + 8, generator=g, device=DEV, dtype=torch.float64)
    buf_w = buf_r + 2e-3 * torch.randn(n + 8, generator=g, device=DEV, dtype=torch.float64)
    buf_w[::7] = buf_r[::7]                                              # some exactly unchanged
    keep = buf_r.clone()
    w, w_ref = buf_w[offset:offset + n], buf_r[offset:offset + n]
    check_case64(lc, w, w_ref, nbits, "offset %d" % offset)
    assert torch.equal(buf_r.view(torch.int64), keep.view(torch.int64))   # check_case64 restores into a clone


def test_fp64_wide_exponent_range_and_quiet_chunks(lc):
    """Exponents far outside binary32's range; whole chunks below every kept bucket (not read again by the second
    sweep, written by the placement kernel); a merged code of several bits."""
    nchunks = 70
    n = nchunks * 16384 + 321
    g = torch.Generator(device=DEV); g.manual_seed(41)
    w_ref = torch.zeros(n, device=DEV, dtype=torch.float64)
    e = torch.randint(0, 4, (n,), generator=g, device=DEV).double()
    d = torch.exp2(600 - e) * (1 + torch.rand(n, generator=g, device=DEV, dtype=torch.float64))
    d = d * (2 * torch.randint(0, 2, (n,), generator=g, device=DEV).double() - 1)
    for k, c in enumerate([0, 5, 63, 64, 65, 69, 70]):
        lo, hi = c * 16384, min(n, (c + 1) * 16384)
        d[lo:hi] = 0 if k % 3 == 2 else 1e-250 * (1 + torch.rand(hi - lo, generator=g, device=DEV, dtype=torch.float64))
    w = w_ref + d
    for nbits in (2, 3, 4):
        blob = check_case64(lc, w, w_ref, nbits, "wide range")
        hdr = lcb1_reader.parse_header(blob)
        assert hdr["dtype"] == 3 and (hdr["slots"][0]["bucket"] & 2047) == 1023 + 600
    check_case64(lc, w, w_ref, 3, "again")                               # the scratch state was left clean
    # and the fp32 path right after, on the same scratch area
    w32, ref32 = laplace_case(3 * 16384 + 11, seed=5)
    check_case(lc, w32, ref32, 3, "fp32 after fp64")


def test_fp64_errors(lc):
    n, nbits = 16384 + 9, 3
    g = torch.Generator(device=DEV); g.manual_seed(43)
    w_ref = 0.05 * torch.randn(n, generator=g, device=DEV, dtype=torch.float64)
    w = w_ref + 1e-3 * torch.randn(n, generator=g, device=DEV, dtype=torch.float64)
    out = lc.alloc_out(n, nbits, DEV)
    size = lc.lc_encode_t(w, w_ref, nbits, out)
    rec32 = w_ref.float()
    before = rec32.clone()
    with pytest.raises(lc.LcError) as e:
        lc.lc_decode(out, rec32)                                         # an fp64 blob into fp32 parameters
    assert e.value.status == lc.ERR_BADARG and torch.equal(rec32, before)
    out32 = lc.alloc_out(n, nbits, DEV)
    lc.lc_encode(w.float(), w_ref.float(), nbits, out32)
    rec = w_ref.clone()
    with pytest.raises(lc.LcError) as e:
        lc.lc_decode_t(out32, rec)                                       # an fp32 blob into fp64 parameters
    assert e.value.status == lc.ERR_BADARG and torch.equal(rec, w_ref)
    # damage in the high half of a representative: the oracle's verdict, parameters untouched
    damaged = out[:size].clone(); damaged[320 + 3] ^= 0x10
    with pytest.raises(lc.LcError) as e:
        lc.lc_decode_t(damaged, rec)
    assert e.value.status == lc.ERR_BAD_BLOB and torch.equal(rec, w_ref)
    with pytest.raises(orc.OracleError) as eo:
        orc.decode64(damaged.cpu().numpy(), w_ref.cpu().numpy())
    assert eo.value.status == orc.BAD_BLOB
    # a non-finite delta (the difference overflows)
    w2 = w.clone(); ref2 = w_ref.clone(); w2[7] = 1.7e308; ref2[7] = -1.7e308
    with pytest.raises(lc.LcError) as e:
        lc.lc_encode_t(w2, ref2, nbits, out)
    assert e.value.status == lc.ERR_NONFINITE
    hdr = lcb1_reader.parse_header(out[:512].cpu().numpy())
    assert hdr["status"] == 2 and hdr["dtype"] == 3 and hdr["total_bytes"] == 512
    check_case64(lc, w, w_ref, nbits, "after a failed call")


# ---------------------------------------------------------------- many small seeded cases
def seeded_delta(kind, n, g, dtype):
    """Deltas of different shapes: the paper's workloads have skewed exponent histograms, many near-zero
    updates, sparse updates and heavy tails (Section 3.1.1, Section 4)."""
    rnd = lambda: torch.rand(n, generator=g, device=DEV, dtype=dtype)
    if kind == "laplace":
        u = rnd() - 0.5
        return -1e-3 * torch.sign(u) * torch.log1p(-2 * u.abs().clamp(max=0.4999999))
    if kind == "sparse":                                     # most entries unchanged, the rest spread over many binades
        d = torch.exp2(-20 * rnd()) * torch.sign(rnd() - 0.5)
        return d * (rnd() < 0.02)
    if kind == "heavy":                                      # a few huge outliers
        d = 1e-5 * torch.randn(n, generator=g, device=DEV, dtype=dtype)
        return torch.where(rnd() < 1e-3, 1e3 * d, d)
    if kind == "blocks":                                     # scale changes every 5000 elements
        scale = torch.exp2(-torch.floor(torch.arange(n, device=DEV, dtype=dtype) / 5000) % 12 - 6)
        return scale * torch.randn(n, generator=g, device=DEV, dtype=dtype)
    assert kind == "two_values"
    return torch.where(rnd() < 0.5, 0.25, -0.125).to(dtype) * (rnd() < 0.7)


@pytest.mark.parametrize("seed", range(24))
def test_seeded_cases_all_types(lc, seed):
    kinds = ["laplace", "sparse", "heavy", "blocks", "two_values"]
    rng = np.random.RandomState(1000 + seed)
    kind = kinds[seed % len(kinds)]
    n = int(rng.choice([1, 63, 4095, 16384, 16385, 50001, 5 * 16384 - 1, 9 * 16384 + 4097]))
    nbits = int(rng.randint(1, 5))
    offset = int(rng.choice([0, 0, 1, 2, 3]))
    tdt = [torch.float32, torch.float64, torch.bfloat16, torch.float16][seed % 4]
    print("seeded case", seed, kind, "n=%d nbits=%d offset=%d" % (n, nbits, offset), tdt, flush=True)
    g = torch.Generator(device=DEV); g.manual_seed(seed)
    work = torch.float64 if tdt == torch.float64 else torch.float32
    buf_r = (0.05 * torch.randn(n + 8, generator=g, device=DEV, dtype=work)).to(tdt)
    buf_w = (buf_r.to(work) + seeded_delta(kind, n + 8, g, work)).to(tdt)
    w, w_ref = buf_w[offset:offset + n], buf_r[offset:offset + n]
    if tdt == torch.float32:
        check_case(lc, w, w_ref, nbits, kind)
    elif tdt == torch.float64:
        check_case64(lc, w, w_ref, nbits, kind)
    else:
        code = orc.DT_BF16 if tdt == torch.bfloat16 else orc.DT_F16
        out = lc.alloc_out(n, nbits, DEV)
        size = lc.lc_encode_t(w, w_ref, nbits, out)
        blob_cpu = orc.encode_t(raw16(w), raw16(w_ref), nbits, code)
        assert np.array_equal(out[:size].cpu().numpy(), blob_cpu)
        rec = w_ref.clone()
        assert lc.lc_decode_t(out, rec) == size
        ref_h = raw16(w_ref)
        orc.decode_t(blob_cpu, ref_h, code)
        assert np.array_equal(raw16(rec).view(np.uint16), ref_h.view(np.uint16))


def seeded_quiet_tensor(rng, g, tdt):
    """A tensor of 0..8 chunks and a ragged end, deltas over 1..6 binades at a random scale; whole chunks made quiet
    (zero, or scaled down by 2^8..2^29) with none, a few or many loud elements left in them."""
    C = 16384
    nchunks = int(rng.randint(0, 9))
    n = nchunks * C + int(rng.choice([0, 0, 1, 77, 1023, 4096, 4097, 16383]))
    off = int(rng.choice([0, 0, 0, 1, 2]))
    scale_exp, binades = int(rng.randint(5, 20)), int(rng.randint(1, 7))
    r = 0.05 * torch.randn(n + off, generator=g, device=DEV)
    e = torch.randint(scale_exp, scale_exp + binades, (n + off,), generator=g, device=DEV).float()
    d = torch.exp2(-e) * (1 + torch.rand(n + off, generator=g, device=DEV))
    d = d * (2 * torch.randint(0, 2, (n + off,), generator=g, device=DEV).float() - 1)
    for c in rng.choice(nchunks + 1, size=int(rng.randint(0, nchunks + 2)), replace=False):
        lo, hi = off + int(c) * C, min(n + off, off + (int(c) + 1) * C)
        if lo >= hi:
            continue
        keep = d[lo:hi].clone()
        d[lo:hi] = 0 if int(rng.randint(0, 3)) == 0 else keep * 2.0 ** -int(rng.randint(8, 30))
        k = int(rng.choice([0, 0, 1, 3, 40]))
        if k:
            idx = torch.from_numpy(rng.randint(0, hi - lo, size=k)).to(DEV)
            d[lo:hi][idx] = keep[idx]
    r = torch.where(d.abs() < 1e-7, torch.zeros_like(r), r)      # tiny deltas survive the subtraction only next to a zero
    if tdt == torch.float32:
        return (r + d)[off:], r[off:]
    r = r.to(tdt)
    return (r.float() + d).to(tdt)[off:], r[off:]


@pytest.mark.parametrize("seed", range(40))
def test_seeded_batches_single_calls_and_verdicts(lc, seed):
    """Seeded lists of 1..8 tensors with quiet stretches: every blob of the batched call is the oracle's and the
    single call's; lc_verify accepts it; restores agree with the oracle; one flipped bit in the chunk area gets the
    oracle's verdict from lc_verify and lc_decode, and with LC_OPT_VERIFY_FIRST (odd seeds) a refused blob leaves
    the parameters alone; the batched restore equals the single ones."""
    C = 16384
    rng = np.random.RandomState(9000 + seed)
    g = torch.Generator(device=DEV); g.manual_seed(9000 + seed)
    tdt = [torch.float32, torch.float32, torch.bfloat16, torch.float16][seed % 4]
    code = {torch.float32: orc.DT_F32, torch.bfloat16: orc.DT_BF16, torch.float16: orc.DT_F16}[tdt]
    view = torch.int32 if tdt == torch.float32 else torch.int16
    host = (lambda t: t.cpu().numpy()) if tdt == torch.float32 else raw16
    oracle_encode = (lambda a, b, x: orc.encode(a, b, x)) if tdt == torch.float32 else (lambda a, b, x: orc.encode_t(a, b, x, code))
    oracle_decode = (lambda blob, a: orc.decode(blob, a)) if tdt == torch.float32 else (lambda blob, a: orc.decode_t(blob, a, code))
    count, nbits = int(rng.randint(1, 9)), int(rng.randint(1, 5))
    print("seeded batch", seed, tdt, "tensors=%d nbits=%d" % (count, nbits), flush=True)
    ws, rs = zip(*[seeded_quiet_tensor(rng, g, tdt) for _ in range(count)])
    outs = [lc.alloc_out(w.numel(), nbits, DEV) for w in ws]
    sizes = lc.lc_encode_batch(list(ws), list(rs), nbits, outs)
    lc.lc_set_option(lc.OPT_VERIFY_FIRST, seed & 1)
    try:
        for t, (w, r, o, size) in enumerate(zip(ws, rs, outs, sizes)):
            n = w.numel()
            rh = host(r)
            blob_cpu = oracle_encode(host(w), rh, nbits)
            assert size == blob_cpu.size and np.array_equal(o[:size].cpu().numpy(), blob_cpu), (t, "batched blob")
            assert lc.lc_verify(o[:size], n, tdt) == size
            o2 = lc.alloc_out(n, nbits, DEV)
            assert lc.lc_encode_t(w, r, nbits, o2) == size and torch.equal(o2[:size], o[:size]), (t, "single blob")
            rec = r.clone()
            assert lc.lc_decode_t(o[:size], rec) == size
            oracle_decode(blob_cpu, rh)
            assert np.array_equal(host(rec).view(np.uint8), rh.view(np.uint8)), (t, "restore")
            if size > 700:
                area = 512 + (4 * ((n + C - 1) // C + 1) + 15) // 16 * 16
                b = o[:size].clone()
                at = int(rng.randint(area, size)); b[at] ^= 1 << int(rng.randint(0, 8))
                try:
                    oracle_decode(b.cpu().numpy(), host(r)); ok = True
                except orc.OracleError:
                    ok = False
                try:
                    lc.lc_verify(b, n, tdt); verified = True
                except lc.LcError:
                    verified = False
                rec = r.clone()
                try:
                    lc.lc_decode_t(b, rec); decoded = True
                except lc.LcError:
                    decoded = False
                assert verified == ok and decoded == ok, (t, at)
                if not ok and (seed & 1):
                    assert torch.equal(rec.view(view), r.view(view)), (t, at, "parameters touched")
    finally:
        lc.lc_set_option(lc.OPT_VERIFY_FIRST, 0)
    recs = [r.clone() for r in rs]
    assert lc.lc_decode_batch(outs, recs) == sizes
    for t, (rec, r, o, size) in enumerate(zip(recs, rs, outs, sizes)):
        single = r.clone()
        lc.lc_decode_t(o[:size], single)
        assert torch.equal(rec.view(view), single.view(view)), (t, "batched restore")


@pytest.mark.parametrize("steps,offset", [(2, 0), (5, 0), (8, 0), (3, 1)])
def test_fused_restore_long_codes(lc, steps, offset):
    """Every blob has codes of up to 15 bits (nbits = 4, magnitudes spread geometrically over many binades, so the
    rare buckets get long codes): several blobs per sweep, ragged tail, an unaligned vector, and a damaged lane
    string, each with the oracle's result."""
    n = 9 * 16384 + 1234
    g = torch.Generator(device=DEV); g.manual_seed(500 + steps)
    buf = 0.05 * torch.randn(n + 4, generator=g, device=DEV)
    w0 = buf[offset:offset + n]
    # P(binade e) halves with every binade down: code lengths 1, 2, 3, ... up to 15
    deltas = []
    for _ in range(steps):
        e = torch.floor(-torch.log2(torch.rand(n, generator=g, device=DEV).clamp_(min=2.0 ** -18)))
        deltas.append(torch.exp2(-4 - e) * (1 + torch.rand(n, generator=g, device=DEV)))
    tracked, blobs = encode_chain(lc, w0.clone(), deltas, [4] * steps)
    max_lens = [lcb1_reader.parse_header(b.cpu().numpy())["max_len"] for b in blobs]
    assert min(max_lens) > 7 and max(max_lens) >= 12, max_lens
    restored = buf.clone()
    assert lc.lc_decode_many(blobs, restored[offset:offset + n]) == sum(b.numel() for b in blobs)
    assert np.array_equal(bits(restored[offset:offset + n].cpu().numpy()), bits(oracle_restore(w0, blobs)))
    assert torch.equal(restored[:offset], buf[:offset]) and torch.equal(restored[offset + n:], buf[offset + n:])
    # a flipped payload bit in the last blob: same verdict as the oracle's
    nchunks = (n + 16383) // 16384
    area = 512 + (4 * (nchunks + 1) + 15) // 16 * 16
    damaged = [b.clone() for b in blobs]
    damaged[-1][area + 128 + 777] ^= 0x08
    ref_h = w0.cpu().numpy().copy()
    try:
        for b in damaged:
            orc.decode(b.cpu().numpy(), ref_h)
        oracle_ok = True
    except orc.OracleError as e:
        assert e.status == 4
        oracle_ok = False
    rec = w0.clone()
    if oracle_ok:
        lc.lc_decode_many(damaged, rec)
        assert np.array_equal(bits(rec.cpu().numpy()), bits(ref_h))
    else:
        with pytest.raises(lc.LcError) as e:
            lc.lc_decode_many(damaged, rec)
        assert e.value.status == lc.ERR_BAD_BLOB


@pytest.mark.parametrize("tdt", [torch.bfloat16, torch.float16])
@pytest.mark.parametrize("steps,nbits,offset", [(1, 3, 0), (5, 3, 0), (11, 2, 1), (6, 4, 0)])
def test_fused_restore_of_16_bit_parameters(lc, tdt, steps, nbits, offset):
    """lc_decode_many_t on bf16 / fp16 parameters: bit for bit the oracle's successive restores (the running value
    is rounded to the storage type after every blob), ragged tail, an offset that takes the guarded path, more
    blobs than one sweep takes; nbits 4 spreads the magnitudes so that long codes occur; fp64 is refused."""
    code = orc.DT_BF16 if tdt == torch.bfloat16 else orc.DT_F16
    n = 7 * 16384 + 4321
    g = torch.Generator(device=DEV); g.manual_seed(900 + steps)
    buf0 = (0.05 * torch.randn(n + 8, generator=g, device=DEV)).to(tdt)
    w0 = buf0[offset:offset + n]
    tracked, w, blobs = w0.clone(), w0.clone(), []
    out = lc.alloc_out(n, nbits, DEV)
    ref_h = raw16(w0)
    for t in range(steps):
        if nbits == 4:
            e = torch.floor(-torch.log2(torch.rand(n, generator=g, device=DEV).clamp_(min=2.0 ** -18)))
            d = torch.exp2(-4 - e) * (1 + torch.rand(n, generator=g, device=DEV)) * torch.sign(torch.randn(n, generator=g, device=DEV))
        else:
            d = 2e-3 * torch.randn(n, generator=g, device=DEV)
            d[::5] = 0
        w = (w.float() + d).to(tdt)
        size = lc.lc_encode_t(w, tracked, nbits, out)
        blobs.append(out[:size].clone())
        assert lc.lc_decode_t(blobs[-1], tracked) == size
        orc.decode_t(blobs[-1].cpu().numpy(), ref_h, code)
    assert np.array_equal(raw16(tracked).view(np.uint16), ref_h.view(np.uint16))
    restored = buf0.clone()
    assert lc.lc_decode_many_t(blobs, restored[offset:offset + n]) == sum(b.numel() for b in blobs)
    assert np.array_equal(raw16(restored[offset:offset + n]).view(np.uint16), ref_h.view(np.uint16))
    assert torch.equal(restored[:offset].view(torch.int16), buf0[:offset].view(torch.int16))
    assert torch.equal(restored[offset + n:].view(torch.int16), buf0[offset + n:].view(torch.int16))
    # a blob of another element type in the list: refused, parameters untouched
    other = torch.bfloat16 if tdt == torch.float16 else torch.float16
    wo = w.float().to(other)
    so = lc.lc_encode_t(wo, wo.clone(), nbits, out)
    rec = w0.clone()
    with pytest.raises(lc.LcError) as e:
        lc.lc_decode_many_t(blobs + [out[:so].clone()], rec)
    assert e.value.status == lc.ERR_BADARG and torch.equal(rec.view(torch.int16), w0.view(torch.int16))
    with pytest.raises(lc.LcError) as e:
        lc.lc_decode_many_t(blobs, w0.double())
    assert e.value.status == lc.ERR_BADARG


@pytest.mark.parametrize("tdt", [torch.bfloat16, torch.float16])
def test_batched_encode_and_restore_of_16_bit_tensors(lc, tdt):
    """lc_encode_batch_t / lc_decode_batch_t: every bf16 / fp16 tensor gets the blob lc_encode_t gives it alone (the
    oracle's, byte for byte) and is restored as lc_decode_t restores it; aligned and unaligned tensors, empty and
    ragged ones, a non-finite delta in one tensor, a blob of another element type in the restore list."""
    code = orc.DT_BF16 if tdt == torch.bfloat16 else orc.DT_F16
    nbits = 3
    sizes_n = [5 * 16384 + 777, 0, 1, 100, 16384, 16385, 20 * 16384 + 5, 3 * 16384, 64]
    scales = [10.0 ** (-4 + 2 * (i % 5) / 4) for i in range(len(sizes_n))]
    offsets = [0, 0, 1, 3, 0, 2, 0, 1, 0]
    ws32, refs32 = batch_case(700, sizes_n, scales, offsets)
    refs = [r.to(tdt) for r in refs32]                                   # (.to makes fresh, aligned tensors)
    ws = [(r.float() + (w - r0)).to(tdt) for w, r0, r in zip(ws32, refs32, refs)]
    # bring the misalignment back: element offsets into 16-bit buffers
    def shifted(t, off):
        buf = torch.zeros(t.numel() + off, dtype=tdt, device=DEV)
        buf[off:] = t
        return buf[off:]
    ws = [shifted(w, o) for w, o in zip(ws, offsets)]
    refs = [shifted(r, o) for r, o in zip(refs, offsets)]
    ws[7] = ws[7].clone(); ws[7][4321] = float("inf")
    outs = [lc.alloc_out(w.numel(), nbits, DEV) for w in ws]
    sizes = lc.lc_encode_batch_t(ws, refs, nbits, outs)
    good = []
    for t, (w, r, o, size) in enumerate(zip(ws, refs, outs, sizes)):
        if t == 7:
            assert size == -lc.ERR_NONFINITE
            assert lc.lc_blob_info(o[:512].cpu().numpy().tobytes())["status"] == lc.ERR_NONFINITE
            continue
        blob_cpu = orc.encode_t(raw16(w), raw16(r), nbits, code)
        blob_gpu = o[:size].cpu().numpy()
        assert size == blob_cpu.size and np.array_equal(blob_gpu, blob_cpu), "tensor %d: %s" % (t, first_diff(blob_gpu, blob_cpu))
        good.append(t)
    recs = [refs[t].clone() if offsets[t] == 0 else shifted(refs[t], offsets[t]) for t in good]
    used = lc.lc_decode_batch_t([outs[t] for t in good], recs)
    assert used == [sizes[t] for t in good]
    for t, rec in zip(good, recs):
        ref_h = raw16(refs[t])
        orc.decode_t(outs[t][:sizes[t]].cpu().numpy(), ref_h, code)
        assert np.array_equal(raw16(rec).view(np.uint16), ref_h.view(np.uint16)), t
    # a blob of the other 16-bit type in the list: that tensor fails and stays as it was, the others are restored
    other = torch.bfloat16 if tdt == torch.float16 else torch.float16
    wo, ro = ws[0].float().to(other), refs[0].float().to(other)
    oo = lc.alloc_out(wo.numel(), nbits, DEV)
    lc.lc_encode_t(wo, ro, nbits, oo)
    recs = [refs[0].clone(), refs[4].clone()]
    used = lc.lc_decode_batch_t([oo, outs[4]], recs)
    assert used[0] == -lc.ERR_BADARG and used[1] == sizes[4]
    assert torch.equal(recs[0].view(torch.int16), refs[0].view(torch.int16))
    ref_h = raw16(refs[4]); orc.decode_t(outs[4][:sizes[4]].cpu().numpy(), ref_h, code)
    assert np.array_equal(raw16(recs[1]).view(np.uint16), ref_h.view(np.uint16))


def test_seeded_mixtures_of_loud_and_quiet_chunks_all_types(lc):
    """Sixty seeded vectors (1 to 13 chunks, sometimes 60 to 140, ragged ends, offsets, nbits 1 to 4, all four element
    types): deltas over one to six binades, a random set of chunks quiet (tiny or zero deltas), some of those with 1 to
    40 loud elements put back.  Every mixture of the sweeps' paths (whole-chunk skips, part-by-part coding, symbols-first
    decode, the pipelined and the guarded paths) in one vector; blob and restored values as the oracle's."""
    for seed in range(60):
        rng = np.random.RandomState(5000 + seed)
        g = torch.Generator(device=DEV); g.manual_seed(5000 + seed)
        nchunks = int(rng.randint(1, 14)) if seed % 7 else int(rng.randint(60, 140))
        n = nchunks * 16384 + int(rng.choice([0, 1, 255, 256, 1023, 1024, 4097, 9000, 16383]))
        nbits = int(rng.randint(1, 5))
        tdt = [torch.float32, torch.float32, torch.bfloat16, torch.float16, torch.float64][seed % 5]
        off = int(rng.choice([0, 0, 0, 1, 2]))
        work = torch.float64 if tdt == torch.float64 else torch.float32
        binades = int(rng.randint(1, 7))
        e = torch.randint(8, 8 + binades, (n + 8,), generator=g, device=DEV).to(work)
        d = torch.exp2(-e) * (1 + torch.rand(n + 8, generator=g, device=DEV, dtype=work))
        d = d * (2 * torch.randint(0, 2, (n + 8,), generator=g, device=DEV).to(work) - 1)
        nq = int(rng.randint(0, nchunks + 2))
        for c in rng.choice(nchunks + 1, size=min(nq, nchunks + 1), replace=False):
            lo, hi = int(c) * 16384, min(n + 8, (int(c) + 1) * 16384)
            if lo >= hi:
                continue
            loud = d[lo:hi].clone()
            d[lo:hi] = (2.0 ** -20) * (1 + torch.rand(hi - lo, generator=g, device=DEV, dtype=work)) if rng.rand() < 0.7 else 0
            k = int(rng.choice([0, 1, 2, 5, 40]))
            if k:
                idx = torch.from_numpy(rng.randint(0, hi - lo, size=k)).to(DEV)
                d[lo:hi][idx] = loud[idx]
        rt = torch.zeros(n + 8, device=DEV, dtype=tdt)
        wt = d.to(tdt)                                                   # (w_ref = 0: every delta is its own value, exactly)
        w, r = wt[off:off + n], rt[off:off + n]
        tag = "seed %d n=%d nbits=%d %s off=%d" % (seed, n, nbits, str(tdt), off)
        if tdt == torch.float32:
            check_case(lc, w, r, nbits, tag)
        elif tdt == torch.float64:
            check_case64(lc, w, r, nbits, tag)
        else:
            print("case", tag, flush=True)
            code = orc.DT_BF16 if tdt == torch.bfloat16 else orc.DT_F16
            out = lc.alloc_out(n, nbits, DEV)
            size = lc.lc_encode_t(w, r, nbits, out)
            blob_cpu = orc.encode_t(raw16(w), raw16(r), nbits, code)
            assert np.array_equal(out[:size].cpu().numpy(), blob_cpu), tag
            rec = rt.clone()
            assert lc.lc_decode_t(out, rec[off:off + n]) == size
            ref_h = raw16(r)
            orc.decode_t(blob_cpu, ref_h, code)
            assert np.array_equal(raw16(rec[off:off + n]).view(np.uint16), ref_h.view(np.uint16)), tag


@pytest.mark.parametrize("n", [1, 100, 1023, 1024, 1025, 4096, 5000, 16384, 16384 + 1024, 3 * 16384 + 2048 + 7])
def test_vectors_in_which_no_element_is_merged(lc, n):
    """Every delta lies in a kept bucket (three buckets, nbits 2), so the merged symbol has no code at all: short
    vectors, vectors of exactly one or a few 4 KiB parts, whole chunks and ragged ends, fp32 and bf16."""
    g = torch.Generator(device=DEV); g.manual_seed(n)
    w_ref = torch.zeros(n, device=DEV)
    pick = torch.randint(0, 3, (n,), generator=g, device=DEV)
    mag = torch.where(pick == 2, 0.25, 0.5) * (1 + 0.5 * torch.rand(n, generator=g, device=DEV))
    w = torch.where(pick == 1, -mag, mag)                       # buckets (+, -1), (-, -1), (+, -2) once n is large enough
    blob = check_case(lc, w, w_ref, 2, "no merged element")
    hdr = lcb1_reader.parse_header(blob)
    assert hdr["slots"][hdr["K"]]["len"] == 0 and hdr["slots"][hdr["K"]]["cnt"] == 0
    wt, rt = w.to(torch.bfloat16), w_ref.to(torch.bfloat16)
    out = lc.alloc_out(n, 2, DEV)
    size = lc.lc_encode_t(wt, rt, 2, out)
    assert np.array_equal(out[:size].cpu().numpy(), orc.encode_t(raw16(wt), raw16(rt), 2, orc.DT_BF16))


def test_calls_from_two_host_threads(lc):
    """Two host threads, each with its own stream, vectors and outputs, calling lc_encode / lc_decode at the same time
    (ctypes drops the interpreter lock during a call): every call returns its own vector's blob and restore, the ones
    a single thread gets."""
    import threading
    cases = []
    for k, (n, nbits) in enumerate([(5 * 16384 + 99, 3), (11 * 16384 + 4097, 4)]):
        w, w_ref = laplace_case(n, seed=900 + k)
        out = lc.alloc_out(n, nbits, DEV)
        size = lc.lc_encode(w, w_ref, nbits, out)
        rec = w_ref.clone()
        lc.lc_decode(out, rec)
        cases.append((w, w_ref, nbits, out[:size].clone(), rec))
    errors = []

    def work(k):
        try:
            w, w_ref, nbits, want_blob, want_rec = cases[k]
            stream = torch.cuda.Stream()
            out = lc.alloc_out(w.numel(), nbits, DEV)
            torch.cuda.synchronize()
            for _ in range(40):
                size = lc.lc_encode(w, w_ref, nbits, out, stream=stream)
                assert size == want_blob.numel() and torch.equal(out[:size], want_blob)
                rec = w_ref.clone()
                torch.cuda.synchronize()
                assert lc.lc_decode(out, rec, stream=stream) == size
                assert torch.equal(rec.view(torch.int32), want_rec.view(torch.int32))
        except Exception as e:                                      # noqa: BLE001  (reported by the main thread)
            errors.append((k, repr(e)))

    threads = [threading.Thread(target=work, args=(k,)) for k in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=100)
    assert not any(t.is_alive() for t in threads) and not errors, errors


def test_chunks_with_very_long_payloads(lc):
    """A chunk made of the vector's rarest symbols only: its payload (about 7 bits per element, 3,400 words) is more than
    the placement kernel assembles in one go, in the single-vector call and in the batched call (which use different
    window sizes); the chunks around it are ordinary.  Blob and restore as the oracle's."""
    nbits, nchunks = 4, 40
    n = nchunks * 16384 + 777
    g = torch.Generator(device=DEV); g.manual_seed(4242)
    # binade e with probability ~ 2^-(e+1): code lengths 1, 2, 3, ... for the 15 kept buckets
    e = torch.floor(-torch.log2(torch.rand(n, generator=g, device=DEV).clamp_(min=2.0 ** -13)))
    for c in (3, 17, 39):                                          # chunks of rare binades only
        lo, hi = c * 16384, (c + 1) * 16384
        e[lo:hi] = torch.randint(7, 13, (hi - lo,), generator=g, device=DEV).float()
    d = torch.exp2(-4 - e) * (1 + torch.rand(n, generator=g, device=DEV))
    w_ref = torch.zeros(n, device=DEV)
    w = w_ref + d
    blob = check_case(lc, w, w_ref, nbits, "very long payloads")
    hdr = lcb1_reader.parse_header(blob)
    offs = np.frombuffer(bytes(blob[512:512 + 4 * (nchunks + 2)]), dtype="<u4")
    words = [int(offs[c + 1]) - int(offs[c]) - 32 for c in (3, 17, 39)]
    assert min(words) > 3000 and hdr["max_len"] >= 7, (words, hdr["max_len"])
    check_batch(lc, [w, w[:5 * 16384].clone()], [w_ref, w_ref[:5 * 16384].clone()], nbits)


def test_many_chunks_with_long_payloads(lc):
    """More than 4096 chunks in one vector (the placement kernel then works with its smaller windows) with payloads
    of 1,000 to 3,500 words per chunk: blob and restore as the oracle's, in full."""
    nbits, nchunks = 4, 4200
    n = nchunks * 16384 + 5
    g = torch.Generator(device=DEV); g.manual_seed(nbits)
    e = torch.floor(-torch.log2(torch.rand(n, generator=g, device=DEV).clamp_(min=2.0 ** -13)))
    for c in (3, 1700, nchunks - 1):
        lo, hi = c * 16384, (c + 1) * 16384
        e[lo:hi] = torch.randint(5, 12, (hi - lo,), generator=g, device=DEV).float()
    d = torch.exp2(-4 - e) * (1 + torch.rand(n, generator=g, device=DEV))
    w_ref = torch.zeros(n, device=DEV)
    check_case(lc, w_ref + d, w_ref, nbits, "many chunks, long payloads")


# ---------------------------------------------------------------- encode with staged keys
@pytest.fixture
def staged(lc):
    """lc_encode stages keys wherever that applies (fp32, aligned arrays, at least one chunk) for the test's duration."""
    lc.lc_set_option(lc.OPT_KEY_STAGING, lc.STAGING_ALWAYS)
    yield
    lc.lc_set_option(lc.OPT_KEY_STAGING, lc.STAGING_AUTO)


def staged_launches(lc, fn):
    """Runs fn with the library's kernel timing on; returns how often the key-staging sweep ran."""
    lc.lc_profile(True)
    try:
        fn()
        return lc.lc_profile_read()["k_hist_keys"][1]
    finally:
        lc.lc_profile(False)


@pytest.mark.parametrize("nbits", [1, 2, 3, 4])
def test_staged_keys_sizes_and_bit_budgets(lc, staged, nbits):
    """The second sweep coding from the 9-bit keys of the first: blobs and restored weights as the oracle's, for
    vectors of whole chunks, with ragged tails shorter and longer than a batch of keys, and below one chunk (where
    nothing is staged)."""
    for n in (16384, 16385, 2 * 16384 + 1023, 2 * 16384 + 1024, 5 * 16384 + 77, 37 * 16384, 64 * 16384 + 4097, (1 << 20) + 13, 1000):
        w, w_ref = laplace_case(n, seed=n * 4 + nbits, zero_frac=0.05)
        ran = staged_launches(lc, lambda: check_case(lc, w, w_ref, nbits, "staged keys"))
        assert ran == (1 if n >= 16384 else 0), n


def test_staged_keys_degenerate_and_long_codes(lc, staged):
    n = 2 * 16384 + 500
    w_ref = 0.05 * torch.randn(n, device=DEV)
    check_case(lc, w_ref.clone(), w_ref, 3, "all zero delta")
    check_case(lc, w_ref * 0 + 1.0, w_ref * 0, 2, "one bucket, one value")
    d = torch.zeros(n, device=DEV); d[12345] = 0.5
    check_case(lc, d, torch.zeros(n, device=DEV), 3, "single non-zero")
    w = w_ref.clone(); w[::3] = 0.0; ref = w_ref.clone(); ref[::3] = -0.0
    w[1::3] = w_ref[1::3] + 0.01
    ref[2::9] = 1e-39; w[2::9] = 3e-39
    check_case(lc, w, ref, 3, "zeros / subnormals")
    # both signs of many exponents, flat and geometric populations (codes of 12 and more bits)
    n = 20 * 16384 + 9
    g = torch.Generator(device=DEV); g.manual_seed(5)
    e = torch.randint(-8, 0, (n,), generator=g, device=DEV).float()
    sgn = torch.randint(0, 2, (n,), generator=g, device=DEV).float() * 2 - 1
    d = sgn * torch.exp2(e) * (1 + torch.rand(n, generator=g, device=DEV))
    check_case(lc, d, torch.zeros(n, device=DEV), 4, "16 flat symbols")
    e = torch.floor(torch.log2(torch.rand(n, generator=g, device=DEV).clamp_(min=2.0 ** -20)))
    d = torch.exp2(-20 - e) * (1 + 0.5 * torch.rand(n, generator=g, device=DEV))
    blob = check_case(lc, d, torch.zeros(n, device=DEV), 4, "geometric populations")
    assert lcb1_reader.parse_header(blob)["max_len"] >= 12
    # extremes of a bucket that sit in the ragged tail behind the last whole batch of keys, and in the last element
    n = 3 * 16384 + 1024 + 37
    w, w_ref = laplace_case(n, seed=808)
    w[-1] = w_ref[-1] + 0.0312; w[-20] = w_ref[-20] - 0.0623; w[3 * 16384 + 1024 + 3] = w_ref[3 * 16384 + 1024 + 3] + 0.03126
    check_case(lc, w, w_ref, 3, "extremes in the tail")
    # non-finite delta: rejected as ever, and the call after it is sound
    bad = w.clone(); bad[777] = float("nan")
    out = lc.alloc_out(n, 3, DEV)
    with pytest.raises(lc.LcError) as e:
        lc.lc_encode(bad, w_ref, 3, out)
    assert e.value.status == lc.ERR_NONFINITE
    check_case(lc, w, w_ref, 3, "after a rejected call")


@pytest.mark.parametrize("nbits", [2, 3, 4])
def test_staged_keys_quiet_chunks_and_other_paths(lc, staged, nbits):
    """Chunks below every kept bucket are passed over by the key sweep too; unaligned arrays, 16-bit parameters and the
    cached encode do not stage and still give their blobs; a plain call after staged ones finds the scratch state clean."""
    nchunks = 150
    n = nchunks * 16384 + 1234
    quiet = [0, 5, 63, 64] + list(range(100, 111)) + [149, 150]
    w, w_ref = quiet_chunk_case(n, 300 + nbits, quiet)
    assert staged_launches(lc, lambda: check_case(lc, w, w_ref, nbits, "quiet chunks, staged")) == 1
    assert staged_launches(lc, lambda: check_case(lc, w[3:], w_ref[3:], nbits, "unaligned: not staged")) == 0
    w2, ref2 = quiet_chunk_case(n, 310 + nbits, list(range(nchunks + 1)))
    check_case(lc, w2, ref2, nbits, "all quiet")
    w2[-5] = ref2[-5] + 0.25
    check_case(lc, w2, ref2, nbits, "all quiet but one")
    cache_gpu, cache_cpu = lc.new_cache(DEV), orc.new_cache()
    out = lc.alloc_out(n, nbits, DEV)
    cached_step(lc, w, w_ref, nbits, out, cache_gpu, cache_cpu)
    _, used = cached_step(lc, w, w_ref, nbits, out, cache_gpu, cache_cpu)
    assert used
    ticket = lc.lc_encode_async(w, w_ref, nbits, out)
    size, _ = lc.lc_encode_wait(ticket)
    assert np.array_equal(out[:size].cpu().numpy(), orc.encode(w.cpu().numpy(), w_ref.cpu().numpy(), nbits))
    lc.lc_set_option(lc.OPT_KEY_STAGING, lc.STAGING_NEVER)
    assert staged_launches(lc, lambda: check_case(lc, w, w_ref, nbits, "plain after staged")) == 0


@pytest.mark.parametrize("nbits", [3, 4])
def test_staged_keys_kept_buckets_spread_over_many_binades(lc, staged, nbits):
    """Kept buckets far apart: the keys carry the whole exponent byte, so a kept set that reaches 28 and more binades
    below the largest delta is coded from the keys like any other; chunks of a narrow range far below sit beside
    chunks of the wide one; and exponents 13 to 16 binades under the largest, around where a four-bit distance
    would run out, each land in their own bucket."""
    n = 24 * 16384 + 777
    g = torch.Generator(device=DEV); g.manual_seed(77 + nbits)
    k = torch.randint(0, 8, (n,), generator=g, device=DEV).float()
    sgn = torch.randint(0, 2, (n,), generator=g, device=DEV).float() * 2 - 1
    wide = sgn * torch.exp2(-4 * k) * (1 + 0.5 * torch.rand(n, generator=g, device=DEV))
    zero = torch.zeros(n, device=DEV)
    assert staged_launches(lc, lambda: check_case(lc, wide, zero, nbits, "kept buckets 4 binades apart")) == 1
    # the upper half of the vector in a narrow range far below the lower half's
    mixed = wide.clone()
    mixed[12 * 16384:] = sgn[12 * 16384:] * 2.0 ** -30 * (1 + torch.rand(n - 12 * 16384, generator=g, device=DEV))
    check_case(lc, mixed, zero, nbits, "wide and narrow chunks")
    # exponents 0, -1 .. -3 and -13 .. -16 in every batch, seven or fifteen buckets kept from the top
    e = torch.tensor([0.0, -14.0, -15.0, -1.0, -2.0, -3.0, -13.0, -16.0], device=DEV)[torch.randint(0, 8, (n,), generator=g, device=DEV)]
    edge = sgn * torch.exp2(e) * (1 + 0.25 * torch.rand(n, generator=g, device=DEV))
    check_case(lc, edge, zero, nbits, "far exponents")
    check_case(lc, edge.abs(), zero, nbits, "far exponents, one sign")


def test_staged_keys_follow_the_vectors_last_encode(lc):
    """The default: a vector's first encode takes the plain second sweep; the next stages keys iff the one before had
    to read more than 30 % of the chunks (vectors of 2^26 elements and more); the blob never depends on it."""
    lc.lc_set_option(lc.OPT_KEY_STAGING, lc.STAGING_AUTO)
    small_w, small_r = laplace_case(40 * 16384 + 5, seed=900)                 # below 2^26 elements: never staged by default
    out = lc.alloc_out(small_w.numel(), 3, DEV)
    for _ in range(2):
        assert staged_launches(lc, lambda: lc.lc_encode(small_w, small_r, 3, out)) == 0
    n = (1 << 26) + 5
    dense_w, dense_r = laplace_case(n, seed=901)
    sparse_w, sparse_r = quiet_chunk_case(n, 902, list(range(1000, 4096)))    # 1001 loud chunks of 4097
    out = lc.alloc_out(n, 3, DEV)
    for w, r, expect in ((dense_w, dense_r, [0, 1, 1]), (sparse_w, sparse_r, [0, 0, 0])):
        blob_cpu = orc.encode(w.cpu().numpy(), r.cpu().numpy(), 3)
        got = []
        for _ in range(3):
            sizes = []
            got.append(staged_launches(lc, lambda: sizes.append(lc.lc_encode(w, r, 3, out))))
            assert np.array_equal(out[:sizes[0]].cpu().numpy(), blob_cpu)
        assert got == expect, got
    # the same buffers with new content: the hint is a guess about performance only
    dense_w.copy_(sparse_w); dense_r.copy_(sparse_r)
    for expect in (1, 0):
        sizes = []
        assert staged_launches(lc, lambda: sizes.append(lc.lc_encode(dense_w, dense_r, 3, out))) == expect
        assert np.array_equal(out[:sizes[0]].cpu().numpy(), orc.encode(sparse_w.cpu().numpy(), sparse_r.cpu().numpy(), 3))
    with pytest.raises(lc.LcError):
        lc.lc_set_option(lc.OPT_KEY_STAGING, 3)
    with pytest.raises(lc.LcError):
        lc.lc_set_option(7, 0)


# ---------------------------------------------------------------- binary64 parameters through the other entry points
def test_fp64_cached_async_many_and_batch(lc):
    """The cached, asynchronous, several-blob and batched calls on binary64 parameters (Section 3.1.1, footnote on the
    bucket count): a chain of checkpoints through lc_encode_cached_t with blob, verdict and cache as the oracle's (hits
    and a miss), the asynchronous form with and without a cache, the restore from all blobs in one lc_decode_many_t call
    against the oracle's successive restores, and lists of tensors through lc_encode_batch_t / lc_decode_batch_t."""
    nbits, n = 3, 6 * 16384 + 321
    g = torch.Generator(device=DEV); g.manual_seed(640)
    w = 0.05 * torch.randn(n, generator=g, device=DEV, dtype=torch.float64)
    w0 = w.clone()
    tracked = w.clone()
    out, out2 = lc.alloc_out(n, nbits, DEV), lc.alloc_out(n, nbits, DEV)
    cache_gpu, cache_cpu, cache_async = lc.new_cache(DEV), orc.new_cache(), lc.new_cache(DEV)
    verdicts, blobs = [], []
    tracked_h = tracked.cpu().numpy()
    for t in range(6):
        d = 2e-3 * torch.randn(n, generator=g, device=DEV, dtype=torch.float64)
        d[:4] = torch.tensor([0.02, -0.02, 0.011, -0.011], device=DEV, dtype=torch.float64)
        if t == 4:
            d[9] = 0.4                                                        # a new largest exponent: miss
        w = w + d
        size, used = lc.lc_encode_cached_t(w, tracked, nbits, out, cache_gpu)
        blob_cpu, used_cpu = orc.encode_cached64(w.cpu().numpy(), tracked_h, nbits, cache_cpu)
        blob_gpu = out[:size].cpu().numpy()
        assert used == used_cpu, t
        assert blob_gpu.size == blob_cpu.size and np.array_equal(blob_gpu, blob_cpu), first_diff(blob_gpu, blob_cpu)
        assert np.array_equal(cache_gpu.cpu().numpy()[:4 * orc.CACHE_WORDS].view(np.uint32), cache_cpu)
        verdicts.append(used)
        ticket = lc.lc_encode_async_t(w, tracked, nbits, out2, cache_async)
        size2, used2 = lc.lc_encode_wait(ticket)
        assert size2 == size and used2 == used and torch.equal(out2[:size2], out[:size])
        ticket = lc.lc_encode_async_t(w, tracked, nbits, out2)              # without a cache: lc_encode_t's blob
        size2, used2 = lc.lc_encode_wait(ticket)
        assert not used2 and np.array_equal(out2[:size2].cpu().numpy(), orc.encode64(w.cpu().numpy(), tracked_h, nbits))
        blobs.append(out[:size].clone())
        orc.decode64(blob_cpu, tracked_h)
        assert lc.lc_decode_t(out, tracked) == size
        assert np.array_equal(bits64(tracked.cpu().numpy()), bits64(tracked_h))
    assert verdicts[0] is False and verdicts[4] is False and any(verdicts[1:4]), verdicts
    # restore from u_0 and all blobs in one call
    rec = w0.clone()
    assert lc.lc_decode_many_t(blobs, rec) == sum(b.numel() for b in blobs)
    assert np.array_equal(bits64(rec.cpu().numpy()), bits64(tracked_h))
    # a damaged blob anywhere in the list leaves the parameters alone
    bad = [b.clone() for b in blobs]
    bad[3][66] ^= 0x01                                                         # a code length: the lengths stop being a prefix code
    rec = w0.clone()
    with pytest.raises(lc.LcError) as e:
        lc.lc_decode_many_t(bad, rec)
    assert e.value.status == lc.ERR_BAD_BLOB and torch.equal(rec, w0)
    # lists of tensors
    sizes_n = [5 * 16384 + 3, 100, 0, 16384, 2 * 16384 + 999]
    ws, refs = [], []
    for k, m in enumerate(sizes_n):
        r = 0.05 * torch.randn(m, generator=g, device=DEV, dtype=torch.float64)
        ws.append(r + 10.0 ** -(2 + k) * torch.randn(m, generator=g, device=DEV, dtype=torch.float64)); refs.append(r)
    outs = [lc.alloc_out(m, 4, DEV) for m in sizes_n]
    got = lc.lc_encode_batch_t(ws, refs, 4, outs)
    expect = [orc.encode64(a.cpu().numpy(), b.cpu().numpy(), 4) for a, b in zip(ws, refs)]
    assert got == [e.size for e in expect]
    for o, e in zip(outs, expect):
        assert np.array_equal(o[:e.size].cpu().numpy(), e)
    recs = [r.clone() for r in refs]
    outs[1][80] ^= 0x01                                                       # tensor 1's blob is damaged: reported, left alone
    used = lc.lc_decode_batch_t(outs, recs)
    assert used == [e.size if k != 1 else -lc.ERR_BAD_BLOB for k, e in enumerate(expect)]
    for k, (rec, r, e) in enumerate(zip(recs, refs, expect)):
        ref_h = r.cpu().numpy()
        if k != 1:
            orc.decode64(e, ref_h)
        assert np.array_equal(bits64(rec.cpu().numpy()), bits64(ref_h)), k


# ---------------------------------------------------------------- calls on different streams run side by side
def test_scratch_areas_that_grow_under_calls_on_side_streams(lc):
    """Every call here needs more scratch than the one before it, so the library allocates and sets up a new area each
    time, on a side stream that does not wait for the null stream: the set-up must be ordered with the call's own
    kernels (a fill that landed behind them once left every bucket's smallest mantissa at zero: blobs of the right
    size with wrong representatives).  Checked against the oracle, representatives included."""
    nbits = 4
    streams = [torch.cuda.Stream() for _ in range(4)]
    cases = [laplace_case(16384 * (40 + 48 * k) + 7 * k, seed=760 + k, scale=10.0 ** -(2 + k % 3)) for k in range(10)]
    expect = [orc.encode(w.cpu().numpy(), r.cpu().numpy(), nbits) for w, r in cases]
    outs = [lc.alloc_out(w.numel(), nbits, DEV) for w, _ in cases]
    torch.cuda.synchronize()
    tickets = [lc.lc_encode_async(w, r, nbits, o, stream=streams[i % len(streams)]) for i, ((w, r), o) in enumerate(zip(cases, outs))]
    for t, o, e in zip(tickets, outs, expect):
        size, _ = lc.lc_encode_wait(t)
        g = o[:size].cpu().numpy()
        assert size == e.size and np.array_equal(g, e), first_diff(g, e)


def test_encodes_on_different_streams_have_their_own_scratch(lc):
    """Section 3.2, asynchronous execution in a trainer with many tensors: asynchronous encodes issued on several
    streams at once (more streams than the library keeps scratch areas, so some share), slices of one vector enqueued
    on one stream and waited for once, with restores and synchronous encodes on yet other streams between them: every
    blob is the oracle's."""
    nbits = 4
    cases = [laplace_case(16384 * (3 + 5 * k) + 11 * k, seed=700 + k, scale=10.0 ** -(2 + k % 3)) for k in range(12)]
    outs = [lc.alloc_out(w.numel(), nbits, DEV) for w, _ in cases]
    streams = [torch.cuda.Stream() for _ in range(10)]
    expect = [orc.encode(w.cpu().numpy(), r.cpu().numpy(), nbits) for w, r in cases]
    torch.cuda.synchronize()
    for rnd in range(3):
        for o in outs:
            o.zero_()
        torch.cuda.synchronize()
        tickets = [lc.lc_encode_async(w, r, nbits, o, stream=streams[(i + rnd) % len(streams)])
                   for i, ((w, r), o) in enumerate(zip(cases, outs))]
        # a restore and a synchronous encode on the default stream while those are in flight
        w0, r0 = cases[0]
        rec = r0.clone()
        tmp = lc.alloc_out(w0.numel(), nbits, DEV)
        size0 = lc.lc_encode(w0, r0, nbits, tmp)
        assert lc.lc_decode(tmp, rec) == size0 == expect[0].size
        for t, o, e in zip(tickets, outs, expect):
            size, _ = lc.lc_encode_wait(t)
            assert size == e.size and np.array_equal(o[:size].cpu().numpy(), e)
    # the slices of one vector on one stream, one wait at the end (the tickets are collected afterwards)
    w, r = laplace_case(8 * 65536 + 777, seed=720)
    cuts = list(range(0, w.numel(), 65536)) + [w.numel()]
    souts = [lc.alloc_out(b - a, nbits, DEV) for a, b in zip(cuts[:-1], cuts[1:])]
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    tickets = [lc.lc_encode_async(w[a:b], r[a:b], nbits, o, stream=s) for (a, b), o in zip(zip(cuts[:-1], cuts[1:]), souts)]
    s.synchronize()
    for t, (a, b), o in zip(tickets, zip(cuts[:-1], cuts[1:]), souts):
        size, _ = lc.lc_encode_wait(t)
        assert np.array_equal(o[:size].cpu().numpy(), orc.encode(w[a:b].cpu().numpy(), r[a:b].cpu().numpy(), nbits))
