"""Seeded synthetic gradient profiles shared by the tests, the benchmark and the smoke check.

This module only *describes inputs*: tensor element counts in forward registration order,
per-tensor backward times, the (a, b) pair of the all-reduce cost model, and random gradient /
weight / momentum arrays.  It contains none of the method's arithmetic (no plan, no offsets, no
pack / reduce / update), so both the CPU oracle's tests and the HIP path can draw the very same
bytes from it without sharing any code of the method.

Index convention: position i = 0..L-1 is paper layer l = i+1 (forward order); the gradient of
i = L-1 is the first to become ready during backpropagation.

The five profiles stand in for the paper's workloads (its DNN table, Table 4, lists ResNet-50 with
161 tensors and about 25.5 M parameters); no dataset, trained weight or trace is used.
Backward times follow one stated rule (see `_bwd_flops_*`): they are proportional to the
backward FLOPs charged to each tensor.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

BASE_SEED = 191209268

# ---------------------------------------------------------------------------------------------
# profile container
# ---------------------------------------------------------------------------------------------


@dataclass
class Profile:
    name: str
    n_elems: np.ndarray          # uint64 [L], element count of every gradient tensor
    t_backward: np.ndarray       # float64 [L], seconds
    a: float                     # all-reduce startup time, seconds          (Eq. 10)
    b: float                     # all-reduce time per byte, seconds / byte  (Eq. 10)
    P: int                       # number of simulated workers
    grad_dtype: str              # "f32", "bf16" or "f16"
    grad_sigma: float            # std-dev of the gradient draw
    lr: float = 0.1
    momentum: float = 0.9
    labels: List[str] = field(default_factory=list)

    @property
    def L(self) -> int:
        return int(self.n_elems.shape[0])

    @property
    def elem_bytes(self) -> int:
        return 4 if self.grad_dtype == "f32" else 2

    @property
    def size_bytes(self) -> np.ndarray:
        return (self.n_elems * np.uint64(self.elem_bytes)).astype(np.uint64)

    @property
    def total_elems(self) -> int:
        return int(self.n_elems.sum())


# ---------------------------------------------------------------------------------------------
# FLOP bookkeeping used to shape backward times
#   weight of a conv / linear layer : 2 x (2 x forward MACs x batch)   (grad wrt input + wrt weight)
#   bias                            : batch x outputs
#   norm scale and shift            : 4 x batch x activations, each
#   embedding table                 : tokens x hidden
# Work that owns no parameter (attention score/context products) is charged to the tensor whose
# gradient becomes ready next, which is how a ready-time profiler would see it.
# ---------------------------------------------------------------------------------------------


def _resnet50() -> Tuple[List[str], List[int], List[float]]:
    batch = 64
    names: List[str] = []
    sizes: List[int] = []
    flops: List[float] = []

    def conv(name, cin, cout, k, hout):
        macs = cin * cout * k * k * hout * hout
        names.append(name + ".weight")
        sizes.append(cout * cin * k * k)
        flops.append(2.0 * 2.0 * macs * batch)

    def bn(name, c, hout):
        act = c * hout * hout
        for part in ("weight", "bias"):
            names.append(f"{name}.{part}")
            sizes.append(c)
            flops.append(4.0 * batch * act)

    conv("conv1", 3, 64, 7, 112)
    bn("bn1", 64, 112)
    inplanes = 64
    h = 56
    for stage, (planes, blocks) in enumerate(((64, 3), (128, 4), (256, 6), (512, 3)), start=1):
        for blk in range(blocks):
            stride = 2 if (stage > 1 and blk == 0) else 1
            h_in = h
            h_out = h // stride
            p = f"layer{stage}.{blk}"
            conv(p + ".conv1", inplanes, planes, 1, h_in)
            bn(p + ".bn1", planes, h_in)
            conv(p + ".conv2", planes, planes, 3, h_out)
            bn(p + ".bn2", planes, h_out)
            conv(p + ".conv3", planes, planes * 4, 1, h_out)
            bn(p + ".bn3", planes * 4, h_out)
            if blk == 0:
                conv(p + ".downsample.0", inplanes, planes * 4, 1, h_out)
                bn(p + ".downsample.1", planes * 4, h_out)
            inplanes = planes * 4
            h = h_out
    names.append("fc.weight")
    sizes.append(2048 * 1000)
    flops.append(2.0 * 2.0 * 2048 * 1000 * batch)
    names.append("fc.bias")
    sizes.append(1000)
    flops.append(float(batch * 1000))
    return names, sizes, flops


def _vgg16() -> Tuple[List[str], List[int], List[float]]:
    batch = 32
    names: List[str] = []
    sizes: List[int] = []
    flops: List[float] = []
    cfg = [(3, 64, 224), (64, 64, 224), (64, 128, 112), (128, 128, 112),
           (128, 256, 56), (256, 256, 56), (256, 256, 56),
           (256, 512, 28), (512, 512, 28), (512, 512, 28),
           (512, 512, 14), (512, 512, 14), (512, 512, 14)]
    for j, (cin, cout, hw) in enumerate(cfg):
        macs = cin * cout * 9 * hw * hw
        names.append(f"features.conv{j}.weight")
        sizes.append(cout * cin * 9)
        flops.append(2.0 * 2.0 * macs * batch)
        names.append(f"features.conv{j}.bias")
        sizes.append(cout)
        flops.append(float(batch * cout * hw * hw))
    for j, (fin, fout) in enumerate(((25088, 4096), (4096, 4096), (4096, 1000))):
        names.append(f"classifier.fc{j}.weight")
        sizes.append(fin * fout)
        flops.append(2.0 * 2.0 * fin * fout * batch)
        names.append(f"classifier.fc{j}.bias")
        sizes.append(fout)
        flops.append(float(batch * fout))
    return names, sizes, flops


def _transformer_encoder() -> Tuple[List[str], List[int], List[float]]:
    H, F, V, S, NL, batch = 1024, 4096, 30522, 512, 24, 8
    tokens = batch * S
    names: List[str] = []
    sizes: List[int] = []
    flops: List[float] = []

    def add(name, n, fl):
        names.append(name)
        sizes.append(n)
        flops.append(float(fl))

    def linear(name, fin, fout, extra_on_bias=0.0):
        add(name + ".weight", fin * fout, 2.0 * 2.0 * fin * fout * tokens)
        add(name + ".bias", fout, tokens * fout + extra_on_bias)

    def norm(name):
        add(name + ".weight", H, 4.0 * tokens * H)
        add(name + ".bias", H, 4.0 * tokens * H)

    add("emb.word", V * H, tokens * H)
    add("emb.position", S * H, tokens * H)
    add("emb.token_type", 2 * H, tokens * H)
    norm("emb.norm")
    attn_core = 8.0 * S * H * tokens  # QK^T and PV, forward+backward, no parameters of their own
    for j in range(NL):
        p = f"layer{j}"
        linear(p + ".attn.q", H, H)
        linear(p + ".attn.k", H, H)
        linear(p + ".attn.v", H, H, extra_on_bias=attn_core)
        linear(p + ".attn.out", H, H)
        norm(p + ".attn.norm")
        linear(p + ".ffn.in", H, F)
        linear(p + ".ffn.out", F, H)
        norm(p + ".ffn.norm")
    add("pooler.weight", H * H, 2.0 * 2.0 * H * H * batch)
    add("pooler.bias", H, batch * H)
    return names, sizes, flops


def _device_seconds_per_flop() -> float:
    """One device-speed constant: the ResNet-50-shaped backward pass lasts 100 ms."""
    _, _, fl = _resnet50()
    return 0.100 / float(np.sum(np.asarray(fl, dtype=np.float64)))


# ---------------------------------------------------------------------------------------------
# the five profiles
# ---------------------------------------------------------------------------------------------

PROFILE_NAMES = ("toy_mlp", "resnet50", "tiny_layers", "vgg16", "transformer")


def make_profile(name: str, seed: int = BASE_SEED) -> Profile:
    rng = np.random.default_rng(seed)
    if name == "toy_mlp":
        sizes = [784 * 256, 256, 256 * 256, 256, 256 * 128, 128, 128 * 10, 10]
        t_b = rng.uniform(50e-6, 500e-6, size=len(sizes))
        return Profile(name, np.asarray(sizes, np.uint64), t_b, a=10e-6, b=1e-9, P=4,
                       grad_dtype="f32", grad_sigma=1.0,
                       labels=[f"fc{j // 2}.{'weight' if j % 2 == 0 else 'bias'}" for j in range(8)])
    if name == "resnet50":
        names, sizes, fl = _resnet50()
        k = _device_seconds_per_flop()
        t_b = np.asarray(fl, np.float64) * k
        return Profile(name, np.asarray(sizes, np.uint64), t_b, a=20e-6, b=1.0 / 10e9, P=8,
                       grad_dtype="f32", grad_sigma=1e-2, labels=names)
    if name == "tiny_layers":
        raw = rng.lognormal(mean=np.log(4096.0), sigma=1.5, size=1000)
        sizes = np.clip(np.rint(raw), 16, 262144).astype(np.uint64)
        t_b = rng.uniform(20e-6, 200e-6, size=1000)
        return Profile(name, sizes, t_b, a=50e-6, b=1.0 / 5e9, P=16,
                       grad_dtype="f32", grad_sigma=1.0,
                       labels=[f"t{j}" for j in range(1000)])
    if name == "vgg16":
        names, sizes, fl = _vgg16()
        k = _device_seconds_per_flop()
        t_b = np.asarray(fl, np.float64) * k
        return Profile(name, np.asarray(sizes, np.uint64), t_b, a=20e-6, b=1.0 / 12.5e9, P=8,
                       grad_dtype="f32", grad_sigma=1e-2, labels=names)
    if name == "transformer":
        names, sizes, fl = _transformer_encoder()
        k = _device_seconds_per_flop()
        t_b = np.asarray(fl, np.float64) * k
        return Profile(name, np.asarray(sizes, np.uint64), t_b, a=10e-6, b=1.0 / 25e9, P=8,
                       grad_dtype="bf16", grad_sigma=1e-3, labels=names)
    raise KeyError(f"unknown profile {name!r}; choose from {PROFILE_NAMES}")


def make_random_profile(rng: np.random.Generator, L: int, *, size_lo: int = 1, size_hi: int = 5000,
                        tb_lo: float = 1e-6, tb_hi: float = 500e-6, a: float | None = None,
                        b: float | None = None, P: int = 4, grad_dtype: str = "f32",
                        allow_empty: bool = False) -> Profile:
    """A small random profile for property tests (sizes log-uniform, times uniform)."""
    lo = np.log(max(size_lo, 1))
    hi = np.log(size_hi)
    sizes = np.maximum(np.rint(np.exp(rng.uniform(lo, hi, size=L))), 1).astype(np.uint64)
    if allow_empty and L > 2:
        sizes[rng.integers(0, L)] = 0
    t_b = rng.uniform(tb_lo, tb_hi, size=L)
    if a is None:
        a = float(10.0 ** rng.uniform(-6, -3))
    if b is None:
        b = float(10.0 ** rng.uniform(-11, -8))
    return Profile(f"random{L}", sizes, t_b, a=a, b=b, P=P, grad_dtype=grad_dtype, grad_sigma=1.0)


# ---------------------------------------------------------------------------------------------
# tensors
# ---------------------------------------------------------------------------------------------


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even conversion of float32 values to bfloat16 bit patterns (uint16).

    Input preparation only: the method itself never narrows a value."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = u + np.uint32(0x7FFF) + lsb
    return (rounded >> np.uint32(16)).astype(np.uint16)


def worker_gradient_flat(profile: Profile, worker: int, seed: int = BASE_SEED) -> np.ndarray:
    """All gradients of one simulated worker, concatenated in forward order i = 0..L-1.

    float32 array for "f32" profiles, uint16 bfloat16 bit patterns for "bf16" profiles, float16 array
    (IEEE binary16, rounded to nearest even from the float32 draw) for "f16" profiles."""
    rng = np.random.default_rng(seed + 1 + worker)
    g = rng.standard_normal(profile.total_elems, dtype=np.float32)
    g *= np.float32(profile.grad_sigma)
    if profile.grad_dtype == "bf16":
        return f32_to_bf16_bits(g)
    if profile.grad_dtype == "f16":
        return g.astype(np.float16)
    return g


def initial_weights_flat(profile: Profile, seed: int = BASE_SEED) -> np.ndarray:
    rng = np.random.default_rng(seed + 100)
    return rng.standard_normal(profile.total_elems, dtype=np.float32)


def initial_momentum_flat(profile: Profile, seed: int = BASE_SEED, zero: bool = False) -> np.ndarray:
    """Momentum buffers: zero for a first step, or a seeded draw to exercise the mu*v term."""
    if zero:
        return np.zeros(profile.total_elems, dtype=np.float32)
    rng = np.random.default_rng(seed + 200)
    v = rng.standard_normal(profile.total_elems, dtype=np.float32)
    v *= np.float32(profile.grad_sigma)
    return v


def split_by_layer(flat: np.ndarray, n_elems: np.ndarray) -> List[np.ndarray]:
    """Views of a forward-order flat array, one per tensor."""
    out = []
    pos = 0
    for n in n_elems.tolist():
        out.append(flat[pos:pos + int(n)])
        pos += int(n)
    return out
