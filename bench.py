#!/usr/bin/env python3
"""Benchmark of the compress / restore hot path on one MI355X.

A step = one pass of the whole path over the workload: lc_encode(w, w_ref) followed by
lc_decode(blob) accumulating into a recovered-state buffer.  Inputs are synthetic, seeded
and resident in HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload vgg16|resnet50|single|gpt2_medium|llama7b]
                  [--no-also] [--no-cpu]
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

    def step(self):
        t0 = time.perf_counter(); self.encode()
        t1 = time.perf_counter(); self.decode()
        t2 = time.perf_counter()
        return t1 - t0, t2 - t1

    def blob_bytes(self):
        return sum(self.sizes)

    def mean_code_bits(self):
        """Payload + index bits per element as stored (everything after the headers)."""
        return 8.0 * (self.blob_bytes() - 512 * len(self.sl)) / self.n


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
    alg = {"k_hist": 8.0, "k_pack": 8.0 + bits / 8.0, "k_decode": 8.0 + bits / 8.0}   # bytes per element
    kernels = {}
    for name, (ms, launches) in prof.items():
        if launches == 0:
            continue
        per_step_ms = ms / steps
        ent = {"ms_per_step": round(per_step_ms, 4), "launches_per_step": launches // steps}
        if name in alg:
            ach = alg[name] * job.n / 1e9 / (per_step_ms / 1e3)
            ent.update(alg_bytes_per_elem=round(alg[name], 4), achieved_GBps=round(ach, 1), frac=round(ach / HBM_PEAK_GBPS, 4))
            # k_pack and k_decode pass over chunks that hold the merged symbol only, so on sparse updates they move
            # fewer bytes than the formula (frac can pass 1); the counter-based traffic, where a summary is committed,
            # is what moved
            tr = traffic_from_profiles(name, job.name)
            if tr is not None:
                per_launch_ms = per_step_ms / max(1, launches // steps)
                ent.update(traffic_bytes_per_launch=tr, traffic_GBps=round(tr / 1e9 / (per_launch_ms / 1e3), 1))
        kernels[name] = ent
    return dict(ms_per_step=1e3 * total / steps, value=gb / (total / steps),
                encode_GBps=gb / (enc / steps), decode_GBps=gb / (dec / steps),
                encode_ms=1e3 * enc / steps, decode_ms=1e3 * dec / steps,
                encode_hbm_frac=(16.0 + bits / 8.0) * job.n / 1e9 / (enc / steps) / HBM_PEAK_GBPS,
                decode_hbm_frac=(8.0 + bits / 8.0) * job.n / 1e9 / (dec / steps) / HBM_PEAK_GBPS,
                ratio=4.0 * job.n / job.blob_bytes(), bits_per_elem=bits, blob_bytes=job.blob_bytes(), kernels=kernels,
                encode_cached=cached)


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
    cached = dict(encode_ms=round(1e3 * t_cached, 4), encode_GBps=round(gb / t_cached, 1), hits=hits, calls=steps * len(job.sl),
                  hbm_frac=round((8.0 + bits / 8.0) * job.n / 1e9 / t_cached / HBM_PEAK_GBPS, 4),
                  k_spec_sweep_ms=round(sweep_ms, 4), k_spec_sweep_GBps=round(sweep_alg / 1e9 / (sweep_ms / 1e3), 1),
                  k_spec_sweep_frac=round(sweep_alg / 1e9 / (sweep_ms / 1e3) / HBM_PEAK_GBPS, 4))
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
                encode_hbm_frac=round((4.0 * esize + bits / 8.0) * n / 1e9 / enc / HBM_PEAK_GBPS, 4),
                decode_hbm_frac=round((2.0 * esize + bits / 8.0) * n / 1e9 / dec / HBM_PEAK_GBPS, 4))


def per_tensor_leg(device, steps):
    """Config 2's tensors (ResNet-50: 161 tensors, 25.6 M parameters) with one table per tensor: lc_encode_batch /
    lc_decode_batch against one lc_encode / lc_decode call per tensor."""
    import math
    import torch
    from paper_2009_13003_amd import lc, workloads
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
    enc, dec, gb = (t1 - t0) / steps, (t2 - t1) / steps, 4.0 * n / 1e9
    return dict(n=n, tensors=len(ws), nbits=nbits, encode_ms=round(1e3 * enc, 4), decode_ms=round(1e3 * dec, 4),
                encode_GBps=round(gb / enc, 1), decode_GBps=round(gb / dec, 1), ratio=round(4.0 * n / sum(sizes), 3),
                encode_ms_one_call_per_tensor=round(1e3 * (t3 - t2), 3), decode_ms_one_call_per_tensor=round(1e3 * (t4 - t3), 3))


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
    for _ in range(steps):
        w = chain.step()
        torch.cuda.synchronize()
        tc = time.perf_counter(); size_c, used = lc.lc_encode_cached(w, tracked, nbits, out_c, cache)   # Section 3.2 table caching
        t0 = time.perf_counter(); size = lc.lc_encode(w, tracked, nbits, out)
        t1 = time.perf_counter(); lc.lc_decode(out, tracked)
        t2 = time.perf_counter()
        enc_c += t0 - tc; enc += t1 - t0; dec += t2 - t1
        hits += int(used); bytes_c += size_c
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
                restore_ms_one_call_per_blob=round(1e3 * t_seq, 3), restore_ms_fused=round(1e3 * t_many, 3),
                fused_speedup=round(t_seq / t_many, 3), restored_equals_tracked=same_seq and same_many)


def traffic_from_profiles(kernel, workload):
    """HBM bytes per launch measured with rocprofv3 --pmc, if a summary for this kernel/workload is committed."""
    path = os.path.join(ROOT, "profiles", "%s_%s_pmc.txt" % (kernel, workload))
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch"):
                return float(line.split()[1])
    except OSError:
        pass
    return None


def cpu_baseline(job):
    """The oracle as it stands, single thread, on the first slice of the workload (<= 2^28 elements)."""
    import numpy as np
    from oracle import lc_oracle
    lo, hi = job.sl[0]
    w_h, r_h = job.w[lo:hi].cpu().numpy(), job.w_ref[lo:hi].cpu().numpy()
    t0 = time.perf_counter()
    blob = lc_oracle.encode(w_h, r_h, job.nbits)
    t1 = time.perf_counter()
    rec = r_h.copy()
    t2 = time.perf_counter()
    lc_oracle.decode(blob, rec)
    t3 = time.perf_counter()
    gpu_blob = job.outs[0][:job.sizes[0]].cpu().numpy()
    same = bool(gpu_blob.size == blob.size and np.array_equal(gpu_blob, blob))
    gb = 4.0 * (hi - lo) / 1e9
    return dict(value=round(gb / ((t1 - t0) + (t3 - t2)), 4), unit="GB/s", cores=1, kind="oracle",
                sample="%s elements [%d, %d): 1 encode + 1 decode, single thread" % (job.name, lo, hi),
                encode_GBps=round(gb / (t1 - t0), 4), decode_GBps=round(gb / (t3 - t2), 4),
                gpu_blob_identical=same)


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

    job = Job(args.workload, dev)
    res = run(job, args.steps, args.warmup, not args.no_cached)
    dom = max((k for k in res["kernels"] if "achieved_GBps" in res["kernels"][k]),
              key=lambda k: res["kernels"][k]["ms_per_step"])
    kd = res["kernels"][dom]
    launches = kd["launches_per_step"]
    roofline = {"bound": "hbm", "kernel": dom,
                "achieved": kd["achieved_GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": kd["frac"],
                "traffic": traffic_from_profiles(dom, args.workload),
                "alg_bytes_per_launch": kd["alg_bytes_per_elem"] * job.n / launches,
                "avg_launch_ms": round(kd["ms_per_step"] / launches, 4)}
    cpu = None if args.no_cpu else cpu_baseline(job)
    config = {"workload": args.workload, "n": job.n, "nbits": job.nbits, "calls_per_step": 2 * len(job.sl),
              "slice_elems": min(job.n, 1 << 28)}

    also = {}
    if not args.no_also:
        del job
        torch.cuda.empty_cache()
        for name in ("llama7b", "resnet50", "single"):
            if name == args.workload:
                continue
            j = Job(name, dev)
            r = run(j, max(2, args.steps // 4) if name == "llama7b" else args.steps, 1, not args.no_cached)
            also[name] = {k: (round(v, 4) if isinstance(v, float) else v) for k, v in r.items()}
            also[name]["n"] = j.n
            also[name]["nbits"] = j.nbits
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
        "encode_hbm_frac": round(res["encode_hbm_frac"], 4), "decode_hbm_frac": round(res["decode_hbm_frac"], 4),
        "compression_ratio": round(res["ratio"], 3), "bits_per_elem": round(res["bits_per_elem"], 4),
        "roofline": roofline, "kernels": res["kernels"], "encode_cached": res["encode_cached"], "cpu_baseline": cpu, "also": also,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
