"""Seeded synthetic inputs for the compress / restore path.

Input generation only: nothing of the method's arithmetic lives here, so both
the HIP path and the CPU oracle may be fed from this module.  The five
workloads have the parameter counts and tensor shapes of real models and
delta distributions with the structure the paper reports for real training
deltas (skewed exponent histograms, many near-zero updates, drift plus noise:
Section 2 eq. (1), Section 3.1, Figure 2).
"""
import math

import numpy as np
import torch


# ---------------------------------------------------------------- model shapes
def resnet50_shapes():
    shapes = [(64, 3, 7, 7), (64,), (64,)]
    inplanes = 64
    for planes, blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for blk in range(blocks):
            shapes += [(planes, inplanes, 1, 1), (planes,), (planes,),
                       (planes, planes, 3, 3), (planes,), (planes,),
                       (planes * 4, planes, 1, 1), (planes * 4,), (planes * 4,)]
            if blk == 0:
                shapes += [(planes * 4, inplanes, 1, 1), (planes * 4,), (planes * 4,)]
            inplanes = planes * 4
    shapes += [(1000, 2048), (1000,)]
    return shapes


def vgg16_shapes():
    shapes, cin = [], 3
    for cout in (64, 64, 128, 128, 256, 256, 256, 512, 512, 512, 512, 512, 512):
        shapes += [(cout, cin, 3, 3), (cout,)]
        cin = cout
    shapes += [(4096, 25088), (4096,), (4096, 4096), (4096,), (1000, 4096), (1000,)]
    return shapes


def gpt2_medium_shapes():
    d, shapes = 1024, [(50257, 1024), (1024, 1024)]
    for _ in range(24):
        shapes += [(d,), (d,), (d, 3 * d), (3 * d,), (d, d), (d,),
                   (d,), (d,), (d, 4 * d), (4 * d,), (4 * d, d), (d,)]
    shapes += [(d,), (d,)]
    return shapes


def llama7b_shapes():
    d, f, shapes = 4096, 11008, [(32000, 4096)]
    for _ in range(32):
        shapes += [(d, d)] * 4 + [(f, d), (f, d), (d, f), (d,), (d,)]
    shapes += [(d,), (32000, 4096)]
    return shapes


def numel(shapes):
    return sum(math.prod(s) for s in shapes)


def shrink(shapes, factor):
    """Same tensor list with every tensor's element count divided by `factor` (at least 1)."""
    return [(max(1, math.prod(s) // factor),) for s in shapes]


EXPECTED_NUMEL = {"resnet50": 25_557_032, "vgg16": 138_357_544,
                  "gpt2_medium": 354_823_168, "llama7b": 6_738_415_616}
SHAPES = {"resnet50": resnet50_shapes, "vgg16": vgg16_shapes,
          "gpt2_medium": gpt2_medium_shapes, "llama7b": llama7b_shapes}


# ---------------------------------------------------------------- distributions
_PIECE = 1 << 26   # generate at most this many elements at a time (bounds temporaries)


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _laplace(nel, b, g, device):
    u = torch.rand(nel, generator=g, device=device, dtype=torch.float32) - 0.5
    return -b * torch.sign(u) * torch.log1p(-2.0 * u.abs().clamp_(max=0.49999997))


def _student_t3(nel, g, device):
    z = torch.randn(nel, generator=g, device=device, dtype=torch.float32)
    chi = torch.zeros(nel, device=device, dtype=torch.float32)
    for _ in range(3):
        chi += torch.randn(nel, generator=g, device=device, dtype=torch.float32) ** 2
    return z / torch.sqrt(chi / 3.0 + 1e-30)


def _fill(out, fn):
    for lo in range(0, out.numel(), _PIECE):
        hi = min(out.numel(), lo + _PIECE)
        out[lo:hi] = fn(hi - lo)


def reference_weights(nel, seed, device):
    """w_ref ~ N(0, 0.05^2), fp32."""
    g = _gen(seed, device)
    w_ref = torch.empty(nel, device=device, dtype=torch.float32)
    _fill(w_ref, lambda m: 0.05 * torch.randn(m, generator=g, device=device, dtype=torch.float32))
    return w_ref


# ---------------------------------------------------------------- the five workloads
def single_tensor(n=1 << 20, seed=0, device="cpu"):
    """Config 1: one tensor, delta ~ Laplace(0, 1e-3), nbits = 3."""
    w_ref = reference_weights(n, seed, device)
    g = _gen(seed + 1, device)
    w = torch.empty_like(w_ref)
    _fill(w, lambda m: _laplace(m, 1e-3, g, device))
    w += w_ref
    return w, w_ref, 3


def per_tensor_laplace(shapes, lo_exp, hi_exp, nbits, seed=0, device="cpu"):
    """Configs 2 and 5: flat concatenation, per-tensor Laplace scale 10^U(lo_exp, hi_exp)."""
    nel = numel(shapes)
    w_ref = reference_weights(nel, seed, device)
    g = _gen(seed + 1, device)
    scales = 10.0 ** np.random.RandomState(seed + 2).uniform(lo_exp, hi_exp, size=len(shapes))
    w = torch.empty_like(w_ref)
    off = 0
    for s, b in zip(shapes, scales):
        m = math.prod(s)
        _fill(w[off:off + m], lambda k, b=float(b): _laplace(k, b, g, device))
        off += m
    w += w_ref
    return w, w_ref, nbits


def resnet50(seed=0, device="cpu", shrink_by=1):
    """Config 2: ResNet-50 shapes, scale 10^U(-5,-2), nbits = 4."""
    return per_tensor_laplace(shrink(resnet50_shapes(), shrink_by), -5, -2, 4, seed, device)


def llama7b(seed=0, device="cpu", shrink_by=1):
    """Config 5: LLaMA-7B shapes, scale 10^U(-6,-3), nbits = 4 (callers slice at 2^28 elements)."""
    return per_tensor_laplace(shrink(llama7b_shapes(), shrink_by), -6, -3, 4, seed, device)


def llama7b_head(nel=1 << 28, seed=0, device="cpu", noise_seed=None):
    """The first `nel` elements of config 5 (same values as llama7b()[:nel]): enough leading tensors, then cut.
    noise_seed: draw the deltas from a generator seeded with it instead (same reference weights, same per-tensor
    scales): the delta of another iteration of the same model."""
    shapes, total = [], 0
    for s in llama7b_shapes():
        shapes.append(s)
        total += math.prod(s)
        if total >= nel:
            break
    nfull = len(llama7b_shapes())
    scales = 10.0 ** np.random.RandomState(seed + 2).uniform(-6, -3, size=nfull)[:len(shapes)]
    w_ref = reference_weights(total, seed, device)
    g = _gen(seed + 1 if noise_seed is None else noise_seed, device)
    w = torch.empty_like(w_ref)
    off = 0
    for s, b in zip(shapes, scales):
        m = math.prod(s)
        _fill(w[off:off + m], lambda k, b=float(b): _laplace(k, b, g, device))
        off += m
    w += w_ref
    return w[:nel].clone(), w_ref[:nel].clone(), 4


def vgg16(seed=0, device="cpu", shrink_by=1):
    """Config 3: VGG-16 shapes, delta = 1e-4 * Student-t(3), 10 % of entries exactly unchanged, nbits = 3."""
    nel = numel(shrink(vgg16_shapes(), shrink_by))
    w_ref = reference_weights(nel, seed, device)
    g = _gen(seed + 1, device)
    w = torch.empty_like(w_ref)

    def piece(m):
        d = 1e-4 * _student_t3(m, g, device)
        keep = torch.rand(m, generator=g, device=device) >= 0.1
        return d * keep
    _fill(w, piece)
    w += w_ref          # masked entries: w == w_ref bit for bit
    return w, w_ref, 3


class Gpt2Chain:
    """Config 4: chain of checkpoints, d_t = 0.9 d_{t-1} + Laplace(0, 5e-5), w_t = w_{t-1} + d_t, nbits = 3.

    `w0` is the initial state (also the first recovered state); `step()` advances
    the live weights in place and returns them.
    """

    def __init__(self, seed=0, device="cpu", shrink_by=1):
        self.nel = numel(shrink(gpt2_medium_shapes(), shrink_by))
        self.device = device
        self.nbits = 3
        self.w = reference_weights(self.nel, seed, device)
        self.w0 = self.w.clone()
        self.d = torch.zeros_like(self.w)
        self.g = _gen(seed + 1, device)

    def step(self):
        for lo in range(0, self.nel, _PIECE):
            hi = min(self.nel, lo + _PIECE)
            self.d[lo:hi].mul_(0.9).add_(_laplace(hi - lo, 5e-5, self.g, self.device))
        self.w += self.d
        return self.w


SLICE = 1 << 28   # config 5 is encoded in slices of this many elements
