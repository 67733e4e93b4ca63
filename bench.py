#!/usr/bin/env python3
"""Benchmark of the compress / restore hot path on one MI355X.

A step = one pass of the whole path over the workload: lc_encode(w, w_ref) followed by
lc_decode(blob) accumulating into a recovered-state buffer.  Inputs are synthetic, seeded
and resident in HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload vgg16|resnet50|single|gpt2_medium|llama7b]
                  [--no-also] [--no-cpu]

What the figures mean.  `*_GBps` of a call = bytes of fp32 parameters (4 n) per second.  `alg_GBps` = the bytes the
two-sweep algorithm has to move by the formula (encode 16 + c/8, decode 8 + c/8 bytes per element, c = stored bits per
element) per second: a design-neutral rate "of parameters", which passes the HBM peak when the sweeps pass over chunks
that hold the merged symbol only, and is therefore never called a fraction of peak.  `frac` (of the 8 TB/s HBM peak) is
given only where the bytes are known to have moved: from rocprofv3's FETCH_SIZE / WRITE_SIZE counters of the same
kernel on the same workload (profiles/*_hbm_traffic_pmc.txt, measured in a run of their own and named as the source),
or, for the kernels that read every element by construction (k_hist, k_spec_sweep), from the formula.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E, published


def make_workload(name, device):
    from paper_2009_13003_amd import workloads as W
    if name == "single":
        w, r, nbits = W.single_tensor(device=device)
    elif name == "resnet50":
        w, r, nbits = W.resnet50(device=device)
    elif name == "vgg16":
        w, r, nbits = W.vgg16(device=device)
    elif name == "llama7b":
        w, r, nbits = W.llama7b(device=device)
    elif name == "llama7b_slice0":
        w, r, nbits = W.llama7b_head(device=device)
    elif name == "gpt2_medium":
        chain = W.Gpt2Chain(device=device)
        r = chain.w0
        w = chain.step().clone()
        nbits = chain.nbits
    else:
        raise SystemExit("unknown workload " + name)
    return w, r, nbits


def slices_of(n):
    from paper_2009_13003_amd.workloads import SLICE
    return [(lo, min(n, lo + SLICE)) for lo in range(0, n, SLICE)]


class Job:
    """Device buffers for one workload; every slice of 2^28 elements is an independent call."""

    def __init__(self, name, device):
        import torch
        from paper_2009_13003_amd import lc
        self.lc, self.torch, self.name = lc, torch, name
        self.w, self.w_ref, self.nbits = make_workload(name, device)
        self.n = self.w.numel()
        self.rec = self.w_ref.clone()
        self.sl = slices_of(self.n)
        self.outs = [lc.alloc_out(hi - lo, self.nbits, device) for lo, hi in self.sl]
        self.sizes = [0] * len(self.sl)
        torch.cuda.synchronize()

    def encode(self):
        for k, (lo, hi) in enumerate(self.sl):
            self.sizes[k] = self.lc.lc_encode(self.w[lo:hi], self.w_ref[lo:hi], self.nbits, self.outs[k])

    def decode(self):
        for k, (lo, hi) in enumerate(self.sl):
            self.lc.lc_decode(self.outs[k], self.rec[lo:hi])

    def verify(self):
        """lc_verify on every blob of the workload: the end-to-end check that reads the blobs only."""
        for k, (lo, hi) in enumerate(self.sl):
            self.lc.lc_verify(self.outs[k][:self.sizes[k]], hi - lo)

    def step(self):
        t0 = time.perf_counter(); self.encode()
        t1 = time.perf_counter(); self.decode()
        t2 = time.perf_counter()
        return t1 - t0, t2 - t1

    def encode_one_wait(self):
        """The same encodes enqueued behind each other through lc_encode_async, then one wait for the stream (the
        tickets are collected afterwards): no host round trip between the slices."""
        lc = self.lc
        tickets = [lc.lc_encode_async(self.w[lo:hi], self.w_ref[lo:hi], self.nbits, self.outs[k]) for k, (lo, hi) in enumerate(self.sl)]
        self.torch.cuda.current_stream().synchronize()
        for k, t in enumerate(tickets):
            self.sizes[k] = lc.lc_encode_wait(t)[0]

    def encode_two_streams(self, streams):
        """The same, the calls dealt in turn to two streams (each stream's calls work in a scratch area of their own):
        the short kernels of one call (table, header) run beside the sweeps of the other."""
        lc, torch = self.lc, self.torch
        tickets = []
        for k, (lo, hi) in enumerate(self.sl):
            with torch.cuda.stream(streams[k & 1]):
                tickets.append(lc.lc_encode_async(self.w[lo:hi], self.w_ref[lo:hi], self.nbits, self.outs[k]))
        for st in streams:
            st.synchronize()
        for k, t in enumerate(tickets):
            self.sizes[k] = lc.lc_encode_wait(t)[0]

    def blob_bytes(self):
        return sum(self.sizes)

    def size_accounting(self):
        """Checkpoint size after each stage of the method (Section 3.1.1 formulas; the E / E+P / E+P+H of Section 4.3),
        summed over the calls of the workload, as fractions of the 32 n bits of the full checkpoint, and the stored
        bits per element against the Shannon entropy of the symbol populations in the headers."""
        E = EP = EPH = 0
        ent_bits = 0.0
        for k in range(len(self.sl)):
            hdr = self.outs[k][:512].cpu().numpy()
            b = self.lc.lc_blob_sizes(hdr.tobytes())
            E += b["E"]; EP += b["EP"]; EPH += b["EPH"]
            _, cnt, _ = header_fields(hdr)
            m = sum(cnt)
            ent_bits += -sum(c * math.log2(c / m) for c in cnt if c)
        full = 32.0 * self.n
        return dict(E_frac=round(E / full, 5), EP_frac=round(EP / full, 5), EPH_frac=round(EPH / full, 5),
                    stored_bits_per_elem=round(EPH / self.n, 4), entropy_bits_per_elem=round(ent_bits / self.n, 4),
                    note="fractions of the full fp32 checkpoint after exponent quantization, + priority promotion, "
                         "+ Huffman coding with all indices")

    def mean_code_bits(self):
        """Payload + index bits per element as stored (everything after the headers)."""
        return 8.0 * (self.blob_bytes() - 512 * len(self.sl)) / self.n


# bytes per element these kernels move whatever the data (k_spec_sweep: see cached_leg); the key-staging sweep reads w and
# w_ref and writes a byte and a bit per element
READS_EVERYTHING = {"k_hist": 8.0, "k_hist_keys": 9.125}
ENCODE_KERNELS = ("k_hist", "k_hist_keys", "k_table", "k_pack", "k_pack_keys", "k_place")
DECODE_KERNELS = ("k_dec_check", "k_decode")


def run(job, steps, warmup, with_cached=True):
    """Times `steps` steps with per-kernel events off (they cost ~60 us per step), then repeats the
    same steps with the library's HIP-event timing on to get each kernel's average duration."""
    torch, lc = job.torch, job.lc
    for _ in range(warmup):
        job.step()
    torch.cuda.synchronize()
    enc = dec = 0.0
    t0 = time.perf_counter()
    for _ in range(steps):
        e, d = job.step()
        enc += e; dec += d
    torch.cuda.synchronize()
    total = time.perf_counter() - t0
    one_wait_ms = two_streams_ms = None
    if 1 < len(job.sl) <= lc.MAX_TICKETS:
        job.encode_one_wait()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(steps):
            job.encode_one_wait()
        one_wait_ms = 1e3 * (time.perf_counter() - t1) / steps
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        for st in streams:
            st.wait_stream(torch.cuda.current_stream())
        job.encode_two_streams(streams)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(steps):
            job.encode_two_streams(streams)
        two_streams_ms = 1e3 * (time.perf_counter() - t1) / steps
    job.verify()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(steps):
        job.verify()
    verify_ms = 1e3 * (time.perf_counter() - t1) / steps
    lc.lc_profile(True)
    for _ in range(steps):
        job.step()
    torch.cuda.synchronize()
    prof = lc.lc_profile_read()
    lc.lc_profile(False)
    gb = 4.0 * job.n / 1e9
    bits = job.mean_code_bits()
    cached = None
    if with_cached:
        cached = cached_leg(job, steps, bits)
    alg = {"k_hist": 8.0, "k_pack": 8.0 + bits / 8.0, "k_decode": 8.0 + bits / 8.0,     # bytes per element by the formula
           "k_hist_keys": 9.125, "k_pack_keys": 1.125 + bits / 8.0}
    traffic, source = traffic_from_profiles(job.name)
    kernels = {}
    for name, (ms, launches) in prof.items():
        if launches == 0:
            continue
        per_step_ms = ms / steps
        per_launch_ms = ms / launches
        ent = {"ms_per_step": round(per_step_ms, 4), "launches_per_step": round(launches / steps, 2),
               "avg_launch_ms": round(per_launch_ms, 4)}
        # Rates only for a kernel that ran in every call of every step, so that it saw all n elements per step (with the
        # choice left to the library, the two forms of the encode, with and without staged keys, share a workload's
        # calls between them, and the calls are not all of one size).
        seen = job.n
        if launches != steps * len(job.sl):
            ent["note"] = "ran in %d of %d calls" % (launches, steps * len(job.sl))
            kernels[name] = ent
            continue
        if name in alg:
            ent.update(alg_bytes_per_elem=round(alg[name], 4),
                       alg_GBps=round(alg[name] * seen / 1e9 / (per_step_ms / 1e3), 1))
        if name in traffic:                              # counter bytes of this kernel on this workload, per launch
            ach = traffic[name] / 1e9 / (per_launch_ms / 1e3)
            ent.update(traffic_bytes_per_launch=traffic[name], hbm_GBps=round(ach, 1), frac=round(ach / HBM_PEAK_GBPS, 4),
                       frac_basis="counters: " + source)
        elif name in READS_EVERYTHING:
            ach = READS_EVERYTHING[name] * seen / 1e9 / (per_step_ms / 1e3)
            ent.update(hbm_GBps=round(ach, 1), frac=round(ach / HBM_PEAK_GBPS, 4), frac_basis="formula (reads every element)")
        kernels[name] = ent

    def call_frac(names, call_s):
        """Counter bytes of a call's kernels over the call's wall time, if every one of its big kernels was counted."""
        if not all(k in traffic for k in names if k in kernels and k in ("k_hist", "k_hist_keys", "k_pack", "k_pack_keys", "k_decode", "k_place")):
            return None, None
        moved = sum(traffic[k] * kernels[k]["launches_per_step"] for k in names if k in traffic and k in kernels)
        return moved, round(moved / 1e9 / call_s / HBM_PEAK_GBPS, 4)

    enc_moved, enc_frac = call_frac(ENCODE_KERNELS, enc / steps)
    dec_moved, dec_frac = call_frac(DECODE_KERNELS, dec / steps)
    return dict(ms_per_step=1e3 * total / steps, value=gb / (total / steps),
                encode_GBps=gb / (enc / steps), decode_GBps=gb / (dec / steps),
                encode_ms=1e3 * enc / steps, decode_ms=1e3 * dec / steps, encode_ms_slices_enqueued_one_wait=one_wait_ms, encode_ms_slices_on_two_streams=two_streams_ms, verify_ms=verify_ms,
                encode_alg_GBps=(16.0 + bits / 8.0) * job.n / 1e9 / (enc / steps),
                decode_alg_GBps=(8.0 + bits / 8.0) * job.n / 1e9 / (dec / steps),
                encode_hbm_bytes=enc_moved, encode_hbm_frac=enc_frac, decode_hbm_bytes=dec_moved, decode_hbm_frac=dec_frac,
                hbm_frac_basis=("counters: " + source) if source else None,
                ratio=4.0 * job.n / job.blob_bytes(), bits_per_elem=bits, blob_bytes=job.blob_bytes(), kernels=kernels,
                sizes=job.size_accounting(), encode_cached=cached)


def cached_leg(job, steps, bits):
    """Section 3.2 table caching: the same checkpoint again through lc_encode_cached.  Every call after the first finds
    its kept set and symbols in the cache, so this times the single-sweep path; the blobs equal lc_encode's."""
    torch, lc = job.torch, job.lc
    gb = 4.0 * job.n / 1e9
    caches = [lc.new_cache(job.w.device) for _ in job.sl]
    def encode_cached():
        used = 0
        for k, (lo, hi) in enumerate(job.sl):
            size, u = lc.lc_encode_cached(job.w[lo:hi], job.w_ref[lo:hi], job.nbits, job.outs[k], caches[k])
            assert size == job.sizes[k]
            used += int(u)
        return used
    encode_cached()
    torch.cuda.synchronize()
    rank_report = ranking_report([job.outs[k][:512].cpu().numpy() for k in range(len(job.sl))])
    tc = time.perf_counter()
    hits = sum(encode_cached() for _ in range(steps))
    t_cached = (time.perf_counter() - tc) / steps
    lc.lc_profile(True)
    for _ in range(steps):
        encode_cached()
    prof_c = lc.lc_profile_read()
    lc.lc_profile(False)
    sweep_ms = prof_c["k_spec_sweep"][0] / max(1, prof_c["k_spec_sweep"][1])
    sweep_alg = (8.0 + bits / 8.0) * job.n / len(job.sl)
    # the single sweep reads every element and writes every code word whatever the data, so 8 + c/8 is what it moves
    # (counters: 1.001 x that on config 3) and its fraction of peak may be taken from the formula
    cached = dict(encode_ms=round(1e3 * t_cached, 4), encode_GBps=round(gb / t_cached, 1), hits=hits, calls=steps * len(job.sl),
                  hbm_frac=round((8.0 + bits / 8.0) * job.n / 1e9 / t_cached / HBM_PEAK_GBPS, 4),
                  k_spec_sweep_ms=round(sweep_ms, 4), k_spec_sweep_GBps=round(sweep_alg / 1e9 / (sweep_ms / 1e3), 1),
                  k_spec_sweep_frac=round(sweep_alg / 1e9 / (sweep_ms / 1e3) / HBM_PEAK_GBPS, 4),
                  frac_basis="formula (reads every element)", ranking=rank_report)
    traffic, source = traffic_from_profiles(job.name)
    if "k_spec_sweep" in traffic:
        cached.update(k_spec_sweep_traffic_bytes=traffic["k_spec_sweep"],
                      k_spec_sweep_traffic_frac=round(traffic["k_spec_sweep"] / 1e9 / (sweep_ms / 1e3) / HBM_PEAK_GBPS, 4),
                      traffic_source=source.replace("_hbm_", "_cached_hbm_"))
    return cached


def typed_leg(device, steps, workload, tdt_name):
    """A workload's shapes and deltas with the parameters stored as bf16 or fp64 (lc_encode_t / lc_decode_t)."""
    import torch
    from paper_2009_13003_amd import lc, workloads
    tdt = dict(bf16=torch.bfloat16, fp64=torch.float64)[tdt_name]
    if workload == "vgg16":
        w, r, nbits = workloads.vgg16(device=device)
    else:
        w, r, nbits = workloads.llama7b_head(device=device)
    rt = r.to(tdt)
    wt = (rt.float() + (w - r)).to(tdt) if tdt_name == "bf16" else rt + (w - r).double()
    del w, r
    n, esize = wt.numel(), wt.element_size()
    out = lc.alloc_out(n, nbits, device)
    rec = rt.clone()
    for _ in range(2):
        size = lc.lc_encode_t(wt, rt, nbits, out); lc.lc_decode_t(out, rec)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        size = lc.lc_encode_t(wt, rt, nbits, out)
    t1 = time.perf_counter()
    for _ in range(steps):
        lc.lc_decode_t(out, rec)
    t2 = time.perf_counter()
    enc, dec, gb = (t1 - t0) / steps, (t2 - t1) / steps, esize * n / 1e9
    bits = 8.0 * (size - 512) / n
    return dict(n=n, nbits=nbits, dtype=tdt_name, encode_ms=round(1e3 * enc, 4), decode_ms=round(1e3 * dec, 4),
                encode_GBps=round(gb / enc, 1), decode_GBps=round(gb / dec, 1), ratio=round(esize * n / size, 3),
                # bytes by the two-sweep formulas over time: a rate "of parameters", above what moves (and above the HBM
                # peak) where the second sweep and the restore pass over chunks; no fraction of peak is claimed from it
                encode_alg_GBps=round((4.0 * esize + bits / 8.0) * n / 1e9 / enc, 1),
                decode_alg_GBps=round((2.0 * esize + bits / 8.0) * n / 1e9 / dec, 1))


def per_tensor_leg(device, steps, workload="resnet50"):
    """One table per tensor (lc_encode_batch / lc_decode_batch) against one lc_encode / lc_decode call per tensor, and
    against the flat vector with one table: config 2's tensors (ResNet-50: 161 tensors, 25.6 M parameters, every tensor
    dense in its own kept buckets) or config 3's (VGG-16: 32 tensors, 138 M, heavy-tailed: most chunks of a tensor lie
    below its kept buckets and the coding sweep passes over them)."""
    import math
    import torch
    from paper_2009_13003_amd import lc, workloads
    if workload == "vgg16":
        shapes = workloads.vgg16_shapes()
        w, r, nbits = workloads.vgg16(device=device)
    else:
        shapes = workloads.resnet50_shapes()
        w, r, nbits = workloads.resnet50(device=device)
    offs = [0]
    for sh in shapes:
        offs.append(offs[-1] + math.prod(sh))
    ws = [w[offs[i]:offs[i + 1]].clone() for i in range(len(shapes))]
    rs = [r[offs[i]:offs[i + 1]].clone() for i in range(len(shapes))]
    outs = [lc.alloc_out(t.numel(), nbits, device) for t in ws]
    recs = [t.clone() for t in rs]
    n = w.numel()
    # the argument lists are marshalled once, as a training loop that checkpoints the same tensors would do
    # (checking and converting 161 tensors costs the host more than the call)
    enc_args, dec_args = lc.EncodeBatch(ws, rs, nbits, outs), lc.DecodeBatch(outs, recs)
    for _ in range(2):
        sizes = enc_args.run(); dec_args.run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        sizes = enc_args.run()
    t1 = time.perf_counter()
    for _ in range(steps):
        dec_args.run()
    t2 = time.perf_counter()
    for a, b, o in zip(ws, rs, outs):
        lc.lc_encode(a, b, nbits, o)
    t3 = time.perf_counter()
    for a, o in zip(recs, outs):
        lc.lc_decode(o, a)
    t4 = time.perf_counter()
    # the flat vector with one table, for scale
    out_flat = lc.alloc_out(n, nbits, device)
    rec_flat = r.clone()
    for _ in range(2):
        flat = lc.lc_encode(w, r, nbits, out_flat); lc.lc_decode(out_flat, rec_flat)
    t5 = time.perf_counter()
    for _ in range(steps):
        lc.lc_encode(w, r, nbits, out_flat)
    t6 = time.perf_counter()
    for _ in range(steps):
        lc.lc_decode(out_flat, rec_flat)
    t7 = time.perf_counter()
    enc, dec, gb = (t1 - t0) / steps, (t2 - t1) / steps, 4.0 * n / 1e9
    return dict(n=n, tensors=len(ws), nbits=nbits, encode_ms=round(1e3 * enc, 4), decode_ms=round(1e3 * dec, 4),
                encode_GBps=round(gb / enc, 1), decode_GBps=round(gb / dec, 1), ratio=round(4.0 * n / sum(sizes), 3),
                encode_ms_one_call_per_tensor=round(1e3 * (t3 - t2), 3), decode_ms_one_call_per_tensor=round(1e3 * (t4 - t3), 3),
                flat_vector=dict(encode_ms=round(1e3 * (t6 - t5) / steps, 4), decode_ms=round(1e3 * (t7 - t6) / steps, 4),
                                 ratio=round(4.0 * n / flat, 3)))


def chain_leg(device, steps):
    """Config 4: `steps` successive checkpoints of the GPT-2-medium-shaped vector, each encoded against the
    recovered state and decoded into it (Algorithm 1); then the restore from u_0 (Section 3, C1) timed two
    ways: one lc_decode per blob, and lc_decode_many over all blobs."""
    import torch
    from paper_2009_13003_amd import lc, workloads
    chain = workloads.Gpt2Chain(device=device)
    n, nbits = chain.nel, chain.nbits
    tracked = chain.w0.clone()
    out = lc.alloc_out(n, nbits, device)
    out_c = lc.alloc_out(n, nbits, device)
    cache = lc.new_cache(device)
    blobs, enc, dec, enc_c, hits, bytes_c = [], 0.0, 0.0, 0.0, 0, 0
    hit_headers, hit_extra_bytes = [], 0
    for _ in range(steps):
        w = chain.step()
        torch.cuda.synchronize()
        tc = time.perf_counter(); size_c, used = lc.lc_encode_cached(w, tracked, nbits, out_c, cache)   # Section 3.2 table caching
        t0 = time.perf_counter(); size = lc.lc_encode(w, tracked, nbits, out)
        t1 = time.perf_counter(); lc.lc_decode(out, tracked)
        t2 = time.perf_counter()
        enc_c += t0 - tc; enc += t1 - t0; dec += t2 - t1
        hits += int(used); bytes_c += size_c
        if used:
            hit_headers.append(out_c[:512].cpu().numpy())
            hit_extra_bytes += size_c - size
        blobs.append(out[:size].clone())
    gb = 4.0 * n / 1e9
    restored = chain.w0.clone()
    lc.lc_decode(blobs[0], restored)                      # untimed, as for the fused restore below
    restored.copy_(chain.w0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for b in blobs:
        lc.lc_decode(b, restored)
    t_seq = time.perf_counter() - t0
    same_seq = bool(torch.equal(restored.view(torch.int32), tracked.view(torch.int32)))
    restored.copy_(chain.w0)
    lc.lc_decode_many(blobs, restored)                    # untimed: the first launch of these kernels in the process
    restored.copy_(chain.w0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    lc.lc_decode_many(blobs, restored)
    t_many = time.perf_counter() - t0
    same_many = bool(torch.equal(restored.view(torch.int32), tracked.view(torch.int32)))
    total_blob = sum(b.numel() for b in blobs)
    return dict(n=n, nbits=nbits, steps=steps, encode_ms=round(1e3 * enc / steps, 4), decode_ms=round(1e3 * dec / steps, 4),
                encode_GBps=round(gb / (enc / steps), 1), decode_GBps=round(gb / (dec / steps), 1),
                ratio=round(4.0 * n * steps / total_blob, 3),
                encode_cached_ms=round(1e3 * enc_c / steps, 4), encode_cached_GBps=round(gb / (enc_c / steps), 1),
                cache_hits=hits, ratio_cached=round(4.0 * n * steps / bytes_c, 3),
                cache_hit_ranking=ranking_report(hit_headers), cache_hit_extra_bytes_vs_own_huffman=hit_extra_bytes,
                restore_ms_one_call_per_blob=round(1e3 * t_seq, 3), restore_ms_fused=round(1e3 * t_many, 3),
                fused_speedup=round(t_seq / t_many, 3), restored_equals_tracked=same_seq and same_many)


def traffic_from_profiles(workload):
    """({kernel: HBM bytes per launch}, source file) as rocprofv3 --pmc counted them for this workload in a run of its
    own (profiles/<workload>_hbm_traffic_pmc.txt: lines `traffic_bytes_per_launch <kernel> <bytes>`), or ({}, None).
    These are constants of the committed summary, not measurements of this run: the summary names the library
    build it was taken from."""
    name = "%s_hbm_traffic_pmc.txt" % workload
    out = {}
    try:
        for line in open(os.path.join(ROOT, "profiles", name)):
            f = line.split()
            if len(f) == 3 and f[0] == "traffic_bytes_per_launch":
                out[f[1]] = float(f[2])
    except OSError:
        return {}, None
    try:                                         # the kernels of the cached encode: counted in a run of their own
        for line in open(os.path.join(ROOT, "profiles", "%s_cached_hbm_traffic_pmc.txt" % workload)):
            f = line.split()
            if len(f) == 3 and f[0] == "traffic_bytes_per_launch":
                out.setdefault(f[1], float(f[2]))
    except OSError:
        pass
    return out, "profiles/" + name


def header_fields(hdr):
    """K, counts and code lengths of the symbols from a blob header (numpy uint8[512])."""
    import numpy as np
    K = int(hdr[20:24].view(np.uint32)[0])
    cnt = [int(hdr[64 + 16 * j + 8:64 + 16 * j + 16].view(np.uint64)[0]) for j in range(K + 1)]
    length = [int(hdr[64 + 16 * j + 2]) for j in range(K + 1)]
    return K, cnt, length


def ranking_report(headers):
    """Section 3.2 hands out a cached table after sorting the buckets by population.  For blobs coded with a cached
    table as it stood (no sort): in how many of them do the lengths still follow the populations (no symbol with
    more entries has a longer code than one with fewer), i.e. the blob is what the sort would have given; and the
    payload bits the others spend beyond the best assignment of the same lengths."""
    same, extra_bits, payload_bits = 0, 0, 0
    for hdr in headers:
        K, cnt, length = header_fields(hdr)
        used = sum(c * l for c, l in zip(cnt, length))
        best = sum(c * l for c, l in zip(sorted(cnt, reverse=True), sorted(length)))
        same += int(used == best)
        extra_bits += used - best
        payload_bits += used
    return dict(blobs=len(headers), lengths_follow_populations=same,
                extra_payload_frac=round(extra_bits / max(1, payload_bits), 6))


def host_description():
    model = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count() or 1
    # the harness gives a one-GPU machine a share of its host: thread pools are sized to that share, whatever nproc says
    share = int(os.environ.get("OMP_NUM_THREADS", "0") or 0)
    threads = max(1, min(usable, share) if share > 0 else usable)
    return model, os.cpu_count() or 1, threads


def oracle_pass(w_h, r_h, nbits):
    """One encode + one restore of the oracle; returns (encode s, decode s, blob)."""
    from oracle import lc_oracle
    t0 = time.perf_counter()
    blob = lc_oracle.encode(w_h, r_h, nbits)
    t1 = time.perf_counter()
    rec = r_h.copy()
    t2 = time.perf_counter()
    lc_oracle.decode(blob, rec)
    t3 = time.perf_counter()
    return t1 - t0, t3 - t2, blob


def oracle_all_cores(w_h, r_h, nbits, threads):
    """The same oracle, unchanged, on all host cores: the sample cut into `threads` contiguous pieces, one oracle
    encode + restore per piece, each on a thread of its own (the C routines run without the interpreter lock).
    A piece is a call with its own table, which is how this path shards (config 5 is cut into calls the same way)."""
    from concurrent.futures import ThreadPoolExecutor
    n = w_h.size
    cuts = [n * i // threads for i in range(threads + 1)]
    pieces = [(w_h[a:b], r_h[a:b]) for a, b in zip(cuts[:-1], cuts[1:]) if b > a]
    with ThreadPoolExecutor(len(pieces)) as pool:
        t0 = time.perf_counter()
        res = list(pool.map(lambda p: oracle_pass(p[0], p[1], nbits)[:2], pieces))
        wall = time.perf_counter() - t0
    # encode and restore of a piece run back to back on its thread: split the wall time in their proportion
    e, d = sum(r[0] for r in res), sum(r[1] for r in res)
    return wall * e / (e + d), wall * d / (e + d), len(pieces)


def cpu_baseline(job, dense_sample=None):
    """The oracle as it stands on the host of the GPU machine, on the first slice of the workload (<= 2^28 elements):
    one thread, then all cores; and the same two legs on `dense_sample` = (name, w, w_ref, nbits), config 5's first slice."""
    import numpy as np
    model, nproc, threads = host_description()
    legs = {}

    def leg(name, w_h, r_h, nbits, gpu_blob=None):
        gb = 4.0 * w_h.size / 1e9
        e1, d1, blob = oracle_pass(w_h, r_h, nbits)
        eN, dN, pieces = oracle_all_cores(w_h, r_h, nbits, threads)
        ent = dict(n=int(w_h.size), one_thread=dict(encode_GBps=round(gb / e1, 4), decode_GBps=round(gb / d1, 4),
                                                    GBps=round(gb / (e1 + d1), 4)),
                   all_cores=dict(threads=pieces, encode_GBps=round(gb / eN, 4), decode_GBps=round(gb / dN, 4),
                                  GBps=round(gb / (eN + dN), 4)))
        if gpu_blob is not None:
            ent["gpu_blob_identical"] = bool(gpu_blob.size == blob.size and np.array_equal(gpu_blob, blob))
        legs[name] = ent
        return ent

    lo, hi = job.sl[0]
    head = leg(job.name, job.w[lo:hi].cpu().numpy(), job.w_ref[lo:hi].cpu().numpy(), job.nbits,
               job.outs[0][:job.sizes[0]].cpu().numpy())
    if dense_sample is not None:
        name, w, r, nbits = dense_sample
        leg(name, w.cpu().numpy(), r.cpu().numpy(), nbits)
    return dict(value=head["all_cores"]["GBps"], unit="GB/s", cores=head["all_cores"]["threads"], kind="oracle",
                sample="%s elements [%d, %d): 1 encode + 1 restore; all cores = the sample cut into %d contiguous pieces, "
                       "one unchanged oracle call pair per piece and thread" % (job.name, lo, hi, head["all_cores"]["threads"]),
                host_cpu=model, host_nproc=nproc, threads_used=threads,
                one_thread_GBps=head["one_thread"]["GBps"], gpu_blob_identical=head.get("gpu_blob_identical"), legs=legs)


PAPER_CONTEXT = {
    "note": "figures the paper prints, on its own hardware and workloads: context, not targets",
    "hardware": "40-core Xeon Gold 6138 @ 2.0 GHz, 192 GB, one Tesla P100 16 GB (Section 4.1)",
    "workloads": "MLR / LeNet-5 / AlexNet on MNIST and FashionMNIST, matrix factorization on Jester and MovieLens (fp32)",
    "compression_rate_best": "up to 28x (abstract, Section 5)",
    "size_after_E_P_H": {"2-bit": "below 5 % of the full checkpoint", "3-bit": "below 10 %", "source": "Section 4.3"},
    "size_breakdown_avg": {"E": "about 15 % of full size (85 % off), so fewer than 2^5 buckets",
                           "P_extra": {"2-bit": "9.26 %", "3-bit": "6.23 %"}, "H_extra": {"2-bit": "2 %", "3-bit": "1.6 %"},
                           "source": "Section 4.3"},
    "recovery_speedup_in_rework_iterations": {"vs SCAR": "2.88x-5.77x at 5 % size, 1.9x-4.82x at 10 %",
                                              "vs TOPN": "2.17x-4.06x at 5 %, 1.52x-2.17x at 10 %", "source": "Section 4.2"},
    "overhead": "under 4 s per 91 s iteration (about 4 %), 3-bit, MF on MovieLens25M; no encode or decode throughput is printed (Section 4.5)",
}


def two_streams_leg(device, steps):
    """Section 3.2, asynchronous execution: two lc_encode_async calls (the two halves of config 3's vector) issued on two
    streams, where they work in scratch areas of their own and overlap on the device, against the same two calls on one
    stream, where the second runs behind the first."""
    import torch
    from paper_2009_13003_amd import lc, workloads
    w, r, nbits = workloads.vgg16(device=device)
    n = w.numel() // 2
    a = (w[:n].clone(), r[:n].clone()); b = (w[n:2 * n].clone(), r[n:2 * n].clone())
    oa, ob = lc.alloc_out(n, nbits, device), lc.alloc_out(n, nbits, device)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    out = {"n_each": n, "nbits": nbits, "pairs": steps}
    for rnd in range(2):                                   # (the first round pays for the second scratch area)
        for mode, sb in (("two_streams", s2), ("one_stream", s1)):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                t1 = lc.lc_encode_async(a[0], a[1], nbits, oa, stream=s1)
                t2 = lc.lc_encode_async(b[0], b[1], nbits, ob, stream=sb)
                lc.lc_encode_wait(t1); lc.lc_encode_wait(t2)
            out["ms_per_pair_" + mode] = round(1e3 * (time.perf_counter() - t0) / steps, 4)
    return out


def rounded(r, job):
    out = {k: (round(v, 4) if isinstance(v, float) else v) for k, v in r.items()}
    out["n"], out["nbits"] = job.n, job.nbits
    return out


def roofline_of(res, job):
    """The kernel with the largest share of the step among those whose HBM bytes are known (counters, or a kernel
    that reads every element).  achieved = algorithmic bytes per launch / average launch duration (HIP events on the
    stream the kernel runs on); traffic = counter bytes per launch, from the committed summary it names, or null."""
    ks = res["kernels"]
    if not any("frac" in v for v in ks.values()):
        return {"bound": "hbm", "kernel": None, "workload": job.name, "note": "no kernel of this run has known HBM bytes"}
    dom = max((k for k in ks if "frac" in ks[k]), key=lambda k: ks[k]["ms_per_step"])
    kd = ks[dom]
    alg = kd.get("alg_bytes_per_elem", READS_EVERYTHING.get(dom)) * job.n / len(job.sl)      # one launch = one call's elements
    avg_ms = kd["avg_launch_ms"]
    ach = alg / 1e9 / (avg_ms / 1e3)
    out = {"bound": "hbm", "kernel": dom, "workload": job.name, "achieved": round(ach, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
           "frac": round(ach / HBM_PEAK_GBPS, 4), "traffic": kd.get("traffic_bytes_per_launch"),
           "traffic_source": kd["frac_basis"] if "traffic_bytes_per_launch" in kd else None,
           "alg_bytes_per_launch": alg, "avg_launch_ms": round(avg_ms, 4)}
    if out["traffic"] is not None:
        out["traffic_frac"] = kd["frac"]                 # counter bytes / duration / peak
        # a sweep that passes over all-merged chunks moves fewer bytes than the formula: its rate is the counters'
        if out["frac"] > 1.0 or alg > 1.05 * out["traffic"]:
            out.update(achieved=kd["hbm_GBps"], frac=kd["frac"], note="sparse input: achieved taken from counter bytes")
    return out


def next_checkpoint_leg(job):
    """Section 3.2 table caching across two successive checkpoints of config 5's first slice: checkpoint 1 fills the
    cache; checkpoint 2 (fresh noise of the same per-tensor scales, against the state recovered from checkpoint 1)
    is encoded with it.  Reports the verdict, how the blob compares with lc_encode's, and whether the cached lengths
    still follow the populations (then the blob is what Section 3.2's sort of the buckets would have given)."""
    torch, lc = job.torch, job.lc
    from paper_2009_13003_amd import workloads
    n, nbits, dev = job.n, job.nbits, job.w.device
    cache = lc.new_cache(dev)
    out = job.outs[0]
    lc.lc_encode_cached(job.w, job.w_ref, nbits, out, cache)
    rec = job.w_ref.clone()
    lc.lc_decode(out, rec)
    w2, r2, _ = workloads.llama7b_head(nel=n, device=str(dev), noise_seed=12345)
    w2 -= r2; w2 += job.w                                 # the next live state: the old one plus a fresh delta
    del r2
    size_c, used = lc.lc_encode_cached(w2, rec, nbits, out, cache)
    hdr = out[:512].cpu().numpy()
    size_p = lc.lc_encode(w2, rec, nbits, out)
    return dict(n=n, nbits=nbits, cache_used=bool(used), blob_bytes_cached=size_c, blob_bytes_plain=size_p,
                ranking=ranking_report([hdr]) if used else None)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="vgg16")
    ap.add_argument("--no-also", action="store_true", help="skip the secondary workloads")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--chain-steps", type=int, default=32, help="checkpoints in the config-4 chain leg (0 = skip)")
    ap.add_argument("--no-cached", action="store_true", help="skip the lc_encode_cached leg")
    ap.add_argument("--chain-only", action="store_true", help="run only the config-4 chain leg and print its result")
    ap.add_argument("--per-tensor", choices=("resnet50", "vgg16"),
                    help="run only the batched per-tensor leg on that model's tensors and print its result")
    ap.add_argument("--two-streams", action="store_true",
                    help="run only the pair of asynchronous encodes (the two halves of config 3) on two streams and on one")
    ap.add_argument("--calibrate", action="store_true",
                    help="run only a plain elementwise copy kernel of known size (553,430,176 bytes read and "
                         "written per launch): the reference for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py: this build runs on one GPU only (--gpus 1); more GPUs would each take "
                         "independent slices of the parameter vector, with no exchange between them")
    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = "cuda:0"

    if args.calibrate:
        src = torch.zeros(138_357_544, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate": "elementwise add, out-of-place", "bytes_read_per_launch": 4 * src.numel(),
                          "bytes_written_per_launch": 4 * src.numel(), "launches": 5}))
        return

    if args.chain_only:
        print(json.dumps(chain_leg(dev, args.chain_steps)))
        return

    if args.per_tensor:
        print(json.dumps(per_tensor_leg(dev, args.steps, args.per_tensor)))
        return
    if args.two_streams:
        print(json.dumps(two_streams_leg(dev, args.steps)))
        return

    job = Job(args.workload, dev)
    res = run(job, args.steps, args.warmup, not args.no_cached)
    roofline = roofline_of(res, job)
    config = {"workload": args.workload, "n": job.n, "nbits": job.nbits, "calls_per_step": 2 * len(job.sl),
              "slice_elems": min(job.n, 1 << 28)}

    also = {}
    dense = None
    if not args.no_also and args.workload != "llama7b_slice0":
        # config 5's first 2^28-element slice, where every chunk holds kept elements: the sweeps' dense rate
        dense = Job("llama7b_slice0", dev)
        # (three warm-up calls: the first encode of a vector takes the plain second sweep, the second allocates the larger
        # scratch area of the staged one)
        r = run(dense, max(2, args.steps // 2), 3, not args.no_cached)
        also["llama7b_slice0"] = rounded(r, dense)
        roofline["dense"] = roofline_of(r, dense)
        if not args.no_cached:
            also["llama7b_slice0_next_checkpoint"] = next_checkpoint_leg(dense)
    cpu = None
    if not args.no_cpu:
        cpu = cpu_baseline(job, None if dense is None else ("llama7b_slice0", dense.w, dense.w_ref, dense.nbits))
    del dense
    if not args.no_also:
        del job
        torch.cuda.empty_cache()
        for name in ("llama7b", "resnet50", "single"):
            if name == args.workload:
                continue
            j = Job(name, dev)
            r = run(j, max(2, args.steps // 4) if name == "llama7b" else args.steps, 2, not args.no_cached)
            also[name] = rounded(r, j)
            del j
            torch.cuda.empty_cache()
        also["vgg16_bf16"] = typed_leg(dev, args.steps, "vgg16", "bf16")
        torch.cuda.empty_cache()
        also["llama7b_slice0_bf16"] = typed_leg(dev, max(2, args.steps // 2), "llama7b_slice0", "bf16")
        torch.cuda.empty_cache()
        also["vgg16_fp64"] = typed_leg(dev, args.steps, "vgg16", "fp64")
        torch.cuda.empty_cache()
        also["llama7b_slice0_fp64"] = typed_leg(dev, max(2, args.steps // 2), "llama7b_slice0", "fp64")
        torch.cuda.empty_cache()
        also["resnet50_per_tensor"] = per_tensor_leg(dev, args.steps)
        also["vgg16_per_tensor"] = per_tensor_leg(dev, args.steps, "vgg16")
        torch.cuda.empty_cache()
        if args.chain_steps > 0:
            also["gpt2_medium_chain"] = chain_leg(dev, args.chain_steps)
            torch.cuda.empty_cache()

    line = {
        "metric": "encode+decode GB/s of fp32 params (one compress + one restore per step)",
        "value": round(res["value"], 3), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(res["ms_per_step"], 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": config,
        "encode_GBps": round(res["encode_GBps"], 2), "decode_GBps": round(res["decode_GBps"], 2),
        "encode_ms": round(res["encode_ms"], 4), "decode_ms": round(res["decode_ms"], 4),
        "encode_alg_GBps": round(res["encode_alg_GBps"], 1), "decode_alg_GBps": round(res["decode_alg_GBps"], 1),
        "encode_hbm_frac": res["encode_hbm_frac"], "decode_hbm_frac": res["decode_hbm_frac"],
        "encode_hbm_bytes": res["encode_hbm_bytes"], "decode_hbm_bytes": res["decode_hbm_bytes"],
        "hbm_frac_basis": res["hbm_frac_basis"],
        "compression_ratio": round(res["ratio"], 3), "bits_per_elem": round(res["bits_per_elem"], 4),
        "sizes": res["sizes"],
        "roofline": roofline, "kernels": res["kernels"], "encode_cached": res["encode_cached"], "cpu_baseline": cpu,
        "paper_context": PAPER_CONTEXT, "also": also,
    }
    for key in ("encode_ms_slices_enqueued_one_wait", "encode_ms_slices_on_two_streams", "verify_ms"):
        if res.get(key) is not None:
            line[key] = round(res[key], 4)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
