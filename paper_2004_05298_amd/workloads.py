"""Seeded synthetic inputs for the DEF / DEF-A compression-and-update step.

This module only *generates inputs*: tensor-size tables shaped like the models
the paper trains (Sec. 5, "Settings": VGG-16, ResNet-18/50/56-style networks),
initial parameters, and per-worker gradient sets with the value distributions
described below.  It contains none of the method's arithmetic (no momentum, no
error feedback, no block selection), so the CPU oracle and the HIP path can both
be fed from it without sharing any part of the method.

The paper's experiments use CIFAR-10/100 and ImageNet gradients; those datasets
are not available, so every gradient here is a seeded random stand-in with the
same shape (W workers x d parameters, fp32) and a documented distribution.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import Callable, List, Optional, Sequence

import numpy as np

MASTER_SEED = 200405298


# --------------------------------------------------------------------------- #
# Tensor-size tables (flattened model = concatenation of these tensors).
# --------------------------------------------------------------------------- #
def _conv(cout: int, cin: int, k: int) -> int:
    return cout * cin * k * k


def single_tensor(d: int) -> List[int]:
    return [d]


def resnet56_cifar_sizes() -> List[int]:
    """57 tensors, 853,018 parameters: a 56-layer CIFAR residual network with
    16/32/64 channels and 3x3 kernels.  Each convolution tensor carries its
    normalisation scale and shift (2*cout values) appended, followed by the
    64x10 classifier and its bias."""
    sizes = [_conv(16, 3, 3) + 2 * 16]
    cin = 16
    for cout in (16, 32, 64):
        for _ in range(18):
            sizes.append(_conv(cout, cin, 3) + 2 * cout)
            cin = cout
    sizes += [64 * 10, 10]
    return sizes


def _bn(c: int) -> List[int]:
    return [c, c]


def resnet18_sizes() -> List[int]:
    """62 tensors, 11,689,512 parameters: basic-block residual network, 64-512
    channels, 3x3 and 1x1 kernels, one 512x1000 classifier."""
    sizes = [_conv(64, 3, 7)] + _bn(64)
    cin = 64
    for cout in (64, 128, 256, 512):
        for blk in range(2):
            sizes += [_conv(cout, cin, 3)] + _bn(cout)
            sizes += [_conv(cout, cout, 3)] + _bn(cout)
            if blk == 0 and cin != cout:
                sizes += [_conv(cout, cin, 1)] + _bn(cout)
            cin = cout
    sizes += [512 * 1000, 1000]
    return sizes


def resnet50_sizes() -> List[int]:
    """161 tensors, 25,557,032 parameters: bottleneck (1x1 / 3x3 / 1x1) residual
    network with stage depths 3-4-6-3 and one 2048x1000 classifier."""
    sizes = [_conv(64, 3, 7)] + _bn(64)
    cin = 64
    for planes, depth in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for blk in range(depth):
            sizes += [_conv(planes, cin, 1)] + _bn(planes)
            sizes += [_conv(planes, planes, 3)] + _bn(planes)
            sizes += [_conv(4 * planes, planes, 1)] + _bn(4 * planes)
            if blk == 0:
                sizes += [_conv(4 * planes, cin, 1)] + _bn(4 * planes)
            cin = 4 * planes
    sizes += [2048 * 1000, 1000]
    return sizes


def vgg16_sizes() -> List[int]:
    """32 tensors, 138,357,544 parameters: 13 3x3 convolutions with biases and
    three fully connected layers (25088x4096, 4096x4096, 4096x1000)."""
    sizes: List[int] = []
    cin = 3
    for cout in (64, 64, 128, 128, 256, 256, 256, 512, 512, 512, 512, 512, 512):
        sizes += [_conv(cout, cin, 3), cout]
        cin = cout
    for fin, fout in ((25088, 4096), (4096, 4096), (4096, 1000)):
        sizes += [fin * fout, fout]
    return sizes


def ragged_sizes(d: int, n_tensors: int, seed: int) -> List[int]:
    """n_tensors positive sizes summing to d, most of them NOT multiples of 4,
    so that tensor boundaries fall on every residue of a 4-element vector."""
    if n_tensors < 1 or d < n_tensors:
        raise ValueError("need 1 <= n_tensors <= d")
    rng = np.random.default_rng([MASTER_SEED, 77, seed, d, n_tensors])
    if n_tensors == 1:
        return [d]
    cuts = np.sort(rng.choice(np.arange(1, d), size=n_tensors - 1, replace=False))
    edges = np.concatenate(([0], cuts, [d]))
    return [int(v) for v in np.diff(edges)]


# --------------------------------------------------------------------------- #
# Workload description.
# --------------------------------------------------------------------------- #
@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    index: int                 # position in the list of configurations (seeds derive from it)
    d: int
    W: int
    R: int
    lr: float
    momentum: float
    weight_decay: float
    T: int
    variant: str               # "def", "def_a" or "both"
    tensor_sizes: Sequence[int]
    grad_kind: str             # see gradient_set()
    pool: int                  # number of distinct gradient sets, cycled t mod pool
    wrap_every: int = 0        # >0: force a block that crosses the end on steps t % wrap_every == wrap_every-1

    @property
    def seed(self) -> int:
        return MASTER_SEED + self.index

    @property
    def B(self) -> int:
        return -(-self.d // self.R)

    @property
    def n_tensors(self) -> int:
        return len(self.tensor_sizes)

    def tensor_offsets(self) -> np.ndarray:
        off = np.zeros(self.n_tensors + 1, dtype=np.uint64)
        off[1:] = np.cumsum(np.asarray(self.tensor_sizes, dtype=np.uint64))
        assert int(off[-1]) == self.d, (int(off[-1]), self.d)
        return off

    def forced_start(self, t: int) -> Optional[int]:
        """Start index to force at step t, or None.  Used by the VGG-16-shaped
        workload: every wrap_every-th step the block straddles index d-1 -> 0."""
        if self.wrap_every > 0 and t % self.wrap_every == self.wrap_every - 1:
            return self.d - self.B // 2
        return None

    def replace(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


def _mk(name, index, sizes, W, R, lr, mu, wd, T, variant, grad_kind, pool, wrap_every=0):
    sizes = list(sizes)
    return Workload(name=name, index=index, d=int(sum(sizes)), W=W, R=R, lr=lr, momentum=mu,
                    weight_decay=wd, T=T, variant=variant, tensor_sizes=tuple(sizes),
                    grad_kind=grad_kind, pool=pool, wrap_every=wrap_every)


def tiny() -> Workload:
    return _mk("tiny", 0, single_tensor(65536), 4, 16, 0.1, 0.9, 0.0, 10, "def", "normal_1e-2", 10)


def resnet56_shaped() -> Workload:
    return _mk("resnet56_shaped", 1, resnet56_cifar_sizes(), 8, 32, 0.1, 0.9, 0.0, 100, "def",
               "per_tensor_sigma", 10)


def resnet18_shaped() -> Workload:
    return _mk("resnet18_shaped", 2, resnet18_sizes(), 16, 64, 0.1, 0.9, 0.0, 50, "def_a",
               "student_t3_1e-3", 3)


def resnet50_shaped() -> Workload:
    return _mk("resnet50_shaped", 3, resnet50_sizes(), 16, 128, 0.1, 0.9, 1e-4, 50, "def",
               "normal_1e-3_spiky", 2)


def vgg16_shaped() -> Workload:
    return _mk("vgg16_shaped", 4, vgg16_sizes(), 32, 256, 0.01, 0.9, 0.0, 20, "both",
               "normal_1e-3", 2, wrap_every=4)


ALL: List[Callable[[], Workload]] = [tiny, resnet56_shaped, resnet18_shaped, resnet50_shaped,
                                     vgg16_shaped]


def by_name(name: str) -> Workload:
    for f in ALL:
        w = f()
        if w.name == name:
            return w
    raise KeyError(name)


def shrunk(base: Workload, d: int, n_tensors: int, W: Optional[int] = None,
           R: Optional[int] = None, T: Optional[int] = None, pool: Optional[int] = None
           ) -> Workload:
    """A small relative of `base` with the same hyper-parameters and gradient
    distribution but d parameters in n_tensors ragged tensors; for parity cases
    the CPU oracle finishes in seconds."""
    sizes = ragged_sizes(d, n_tensors, base.index)
    return dataclasses.replace(
        base, name=f"{base.name}_d{d}", d=d, tensor_sizes=tuple(sizes),
        W=base.W if W is None else W, R=base.R if R is None else R,
        T=base.T if T is None else T, pool=base.pool if pool is None else pool)


# --------------------------------------------------------------------------- #
# Values.
# --------------------------------------------------------------------------- #
def initial_params(w: Workload) -> np.ndarray:
    """x_0 ~ N(0, 0.05^2), fp32, length d."""
    rng = np.random.default_rng([w.seed, 1])
    return (rng.standard_normal(w.d, dtype=np.float32) * np.float32(0.05)).astype(np.float32)


def _fill_row(w: Workload, slot: int, k: int, out: np.ndarray, sigma_flat) -> None:
    rng = np.random.default_rng([w.seed, 2, slot, k])
    d = w.d
    kind = w.grad_kind
    if kind == "normal_1e-2":
        out[:d] = rng.standard_normal(d, dtype=np.float32) * np.float32(0.01)
    elif kind == "normal_1e-3":
        out[:d] = rng.standard_normal(d, dtype=np.float32) * np.float32(1e-3)
    elif kind == "per_tensor_sigma":
        out[:d] = rng.standard_normal(d, dtype=np.float32) * sigma_flat
    elif kind == "student_t3_1e-3":
        # heavy tails: Student-t with 3 degrees of freedom, scale 1e-3
        chunk = 1 << 22
        for a in range(0, d, chunk):
            b = min(d, a + chunk)
            out[a:b] = (rng.standard_t(3.0, size=b - a) * 1e-3).astype(np.float32)
    elif kind == "normal_1e-3_spiky":
        # N(0, 1e-3^2) with 1 % of the entries, at seeded positions, scaled x100
        v = rng.standard_normal(d, dtype=np.float32) * np.float32(1e-3)
        spikes = rng.random(d, dtype=np.float32) < np.float32(0.01)
        v[spikes] *= np.float32(100.0)
        out[:d] = v
    else:
        raise ValueError(kind)
    out[d:] = 0.0


def per_tensor_sigma(w: Workload) -> np.ndarray:
    """sigma_l log-uniform in [1e-4, 1e-1], one per tensor."""
    rng = np.random.default_rng([w.seed, 3])
    return np.exp(rng.uniform(np.log(1e-4), np.log(1e-1), size=w.n_tensors)).astype(np.float32)


def gradient_set(w: Workload, slot: int, ld: Optional[int] = None, threads: int = 8,
                 out: Optional[np.ndarray] = None) -> np.ndarray:
    """One set of per-worker gradients: fp32 array [W][ld], worker k's flat
    gradient in row k, columns d..ld-1 zero.  Rows are independent streams
    keyed by (workload seed, slot, k)."""
    ld = w.d if ld is None else int(ld)
    if ld < w.d:
        raise ValueError("ld < d")
    if out is None:
        out = np.empty((w.W, ld), dtype=np.float32)
    assert out.shape == (w.W, ld) and out.dtype == np.float32
    sigma_flat = None
    if w.grad_kind == "per_tensor_sigma":
        sigma_flat = np.repeat(per_tensor_sigma(w), np.asarray(w.tensor_sizes))
    if threads <= 1 or w.W == 1:
        for k in range(w.W):
            _fill_row(w, slot, k, out[k], sigma_flat)
    else:
        with ThreadPoolExecutor(max_workers=min(threads, w.W)) as ex:
            list(ex.map(lambda k: _fill_row(w, slot, k, out[k], sigma_flat), range(w.W)))
    return out


def gradient_pool(w: Workload, ld: Optional[int] = None, threads: int = 8) -> List[np.ndarray]:
    return [gradient_set(w, slot, ld, threads) for slot in range(w.pool)]


def padded_ld(d: int, multiple: int = 256) -> int:
    """Row stride for a worker-major gradient buffer: d rounded up so that every
    row starts on a 1 KiB boundary (the library's fastest case)."""
    return -(-d // multiple) * multiple


def device_gradient_pool(w: Workload, ld: int, device="cuda", threads: int = 16):
    """The same gradient sets as gradient_pool(), generated row by row on the host
    and copied straight into device tensors [W][ld], so that the host never holds
    more than `threads` rows (the VGG-16-shaped set is 17.7 GB)."""
    import torch

    sigma_flat = None
    if w.grad_kind == "per_tensor_sigma":
        sigma_flat = np.repeat(per_tensor_sigma(w), np.asarray(w.tensor_sizes))
    pool = []
    for slot in range(w.pool):
        dev = torch.empty((w.W, ld), dtype=torch.float32, device=device)

        def make_row(k, slot=slot):
            row = np.empty(ld, dtype=np.float32)
            _fill_row(w, slot, k, row, sigma_flat)
            return k, row

        with ThreadPoolExecutor(max_workers=max(1, min(threads, w.W))) as ex:
            for k, row in ex.map(make_row, range(w.W)):
                dev[k].copy_(torch.from_numpy(row))
        pool.append(dev)
    return pool
