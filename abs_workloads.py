"""Seeded synthetic inputs for the ABS-SGD hot path.

This module only MAKES inputs: parameter vectors, micro-batch gradient vectors,
per-step micro-batch counts m_k, ragged tensor layouts.  It holds none of the
method's arithmetic (no accumulation, averaging or update), so both the CPU
oracle's tests and the GPU library's tests may draw the same bytes from it.

The paper trains ResNet18 on CIFAR10 with 4 workers whose speeds differ by a
fixed ratio, by a per-iteration random factor, or both (Section "Experimental
settings").  The hot path never sees images, only gradient vectors, so these
inputs take the shapes of that setting: flat vectors as long as the model,
reference batch size 32, and per-step micro-batch counts with the static /
dynamic / combined heterogeneity structure.

All normals are N(0, sigma) with sigma a STANDARD DEVIATION.
"""
from dataclasses import dataclass, field
from typing import Optional, Tuple

import numpy as np

BASE_SEED = 0x15164


@dataclass(frozen=True)
class Workload:
    name: str
    index: int                 # seed offset
    P: int                     # total number of parameters
    K: int                     # number of workers (the paper's N)
    grad_dtype: str            # "f32" | "bf16"
    n: int                     # samples per micro-batch (the paper's M_r)
    sigma_x: float
    sigma_g: float
    lr: float
    mu: float
    wd: float
    steps: int
    schedule: str              # how m_k is drawn, see schedule()
    ratio: Tuple[int, ...] = ()
    tensor_sizes: Optional[Tuple[int, ...]] = None   # ragged layout, sums to P
    pool: int = 8              # number of distinct gradient vectors
    notes: str = field(default="", compare=False)

    @property
    def seed(self):
        return BASE_SEED + self.index


def _gpt2_small_sizes():
    """Tensor sizes of a 12-layer, width-768 decoder with a 50,257-token
    vocabulary and 1,024 positions: 148 tensors, 124,439,808 parameters."""
    d, layers, vocab, ctx = 768, 12, 50257, 1024
    per_layer = [d, d,                 # norm 1 weight, bias
                 d * 3 * d, 3 * d,     # qkv weight, bias
                 d * d, d,             # attention projection weight, bias
                 d, d,                 # norm 2 weight, bias
                 d * 4 * d, 4 * d,     # mlp up weight, bias
                 4 * d * d, d]         # mlp down weight, bias
    sizes = [vocab * d, ctx * d] + per_layer * layers + [d, d]
    assert len(sizes) == 148 and sum(sizes) == 124_439_808
    return sizes


def _permuted(sizes, seed):
    rng = np.random.Generator(np.random.Philox(seed))
    order = rng.permutation(len(sizes))
    return tuple(int(sizes[i]) for i in order)


def _odd_sizes(seed, count=37, lo=1, hi=300_000):
    """Ragged sizes that are mostly NOT multiples of 4 or 8, including tiny
    ones, to exercise vector tails; log-uniform between lo and hi."""
    rng = np.random.Generator(np.random.Philox(seed))
    s = np.exp(rng.uniform(np.log(lo), np.log(hi), size=count)).astype(np.int64)
    s = np.maximum(s, 1)
    s[0], s[1], s[2], s[3] = 1, 3, 5, 7
    s[4] = 65_537
    return tuple(int(v) for v in s)


_GPT2 = _permuted(_gpt2_small_sizes(), BASE_SEED + 5)
_ODD = _odd_sizes(BASE_SEED + 6)

WORKLOADS = {w.name: w for w in [
    Workload("cfg1_small", 1, 1_048_576, 4, "f32", 32, 0.05, 0.01, 0.1, 0.9, 5e-4, 5,
             "uniform_1_4", pool=16,
             notes="correctness/latency case; the oracle finishes it in seconds"),
    Workload("cfg2_resnet18", 2, 11_689_512, 4, "f32", 32, 0.05, 0.01, 0.1, 0.9, 5e-4, 20,
             "fixed", ratio=(2, 2, 4, 8),
             notes="static speed ratio 1:1:2:4"),
    Workload("cfg3_resnet50_bf16", 3, 25_557_032, 8, "bf16", 32, 0.05, 0.01, 0.1, 0.9, 5e-4,
             20, "poisson4_plus1", notes="dynamic heterogeneity"),
    Workload("cfg4_vgg16", 4, 138_357_544, 4, "f32", 64, 0.05, 0.005, 0.1, 0.9, 5e-4, 10,
             "ratio_jitter", ratio=(1, 2, 3, 6),
             notes="static ratio times U(0.5,1.5) jitter per (step, worker)"),
    Workload("cfg5_gpt2_ragged_bf16", 5, sum(_GPT2), 16, "bf16", 32, 0.05, 0.01, 0.1, 0.9,
             5e-4, 10, "uniform_1_8", tensor_sizes=_GPT2,
             notes="148 separately allocated tensors in a seeded order"),
    # extras beyond the five stated configurations
    Workload("ragged_odd_f32", 6, sum(_ODD), 3, "f32", 32, 0.05, 0.01, 0.1, 0.9, 5e-4, 4,
             "uniform_1_4", tensor_sizes=_ODD, pool=12,
             notes="odd tensor sizes: vector tails, tiny tensors"),
    Workload("ragged_odd_bf16", 7, sum(_ODD), 5, "bf16", 32, 0.05, 0.01, 0.1, 0.9, 5e-4, 4,
             "uniform_1_4", tensor_sizes=_ODD, pool=12),
    Workload("tiny_tail_f32", 8, 100_003, 2, "f32", 32, 0.05, 0.01, 0.1, 0.9, 5e-4, 4,
             "uniform_1_4", pool=8, notes="flat vector with a ragged tail"),
    Workload("tiny_tail_bf16", 9, 100_003, 7, "bf16", 32, 0.05, 0.01, 0.1, 0.9, 5e-4, 4,
             "uniform_1_4", pool=8),
    Workload("vgg16_k8_bf16", 13, 138_357_544, 8, "bf16", 32, 0.05, 0.01, 0.1, 0.9, 5e-4, 6,
             "poisson4_plus1", notes="measurement only: the K = 8 kernels with every buffer far beyond the "
                                     "memory-side cache"),
    Workload("vgg16_k16_bf16", 14, 138_357_544, 16, "bf16", 32, 0.05, 0.01, 0.1, 0.9, 5e-4, 6,
             "uniform_1_8", notes="measurement only: the flat K = 16 kernels at a large size"),
    Workload("paper_static", 10, 11_689_512, 4, "f32", 32, 0.05, 0.01, 0.01, 0.0, 0.0, 20,
             "fixed", ratio=(12, 6, 4, 3),
             notes="the paper's own setting: plain SGD, lr 0.01, iteration-time ratio "
                   "1:2:3:4 hence micro-batch counts 12:6:4:3"),
    Workload("paper_dynamic", 11, 11_689_512, 4, "f32", 32, 0.05, 0.01, 0.01, 0.0, 0.0, 20,
             "speed_jitter", ratio=(1, 1, 1, 1),
             notes="the paper's dynamic-only cluster: equal workers, each iteration prolonged by "
                   "U(0, 50 %); a worker fits rint(6 / (1 + u)) reference batches in the window"),
    Workload("paper_static_dynamic", 12, 11_689_512, 4, "f32", 32, 0.05, 0.01, 0.01, 0.0, 0.0, 20,
             "speed_jitter", ratio=(1, 2, 3, 4),
             notes="the paper's third cluster: iteration-time ratio 1:2:3:4, each prolonged by "
                   "U(0, 50 %); a worker fits max(1, rint(12 / (r (1 + u)))) reference batches"),
]}


def schedule(w: Workload, steps: Optional[int] = None) -> np.ndarray:
    """m[t, k] >= 1: how many micro-batches worker k accumulates in step t."""
    T = w.steps if steps is None else steps
    rng = np.random.Generator(np.random.Philox(w.seed * 7919 + 1))
    if w.schedule == "fixed":
        m = np.tile(np.asarray(w.ratio, dtype=np.int64), (T, 1))
    elif w.schedule == "uniform_1_4":
        m = rng.integers(1, 5, size=(T, w.K))
    elif w.schedule == "uniform_1_8":
        m = rng.integers(1, 9, size=(T, w.K))
    elif w.schedule == "poisson4_plus1":
        m = rng.poisson(4.0, size=(T, w.K)) + 1
    elif w.schedule == "speed_jitter":
        # iteration time of worker k = r_k (1 + u), u ~ U(0, 0.5) per (step, worker); the number
        # of reference batches that fit in a fixed window is inversely proportional to it
        u = rng.uniform(0.0, 0.5, size=(T, w.K))
        r = np.asarray(w.ratio, dtype=np.float64)
        base = 6.0 * r.max() if r.max() == r.min() else 12.0
        m = np.maximum(1, np.rint(base / (r * (1.0 + u))))
    elif w.schedule == "ratio_jitter":
        u = rng.uniform(0.5, 1.5, size=(T, w.K))
        m = np.maximum(1, np.rint(np.asarray(w.ratio, dtype=np.float64) * u))
    else:
        raise ValueError(w.schedule)
    m = np.asarray(m, dtype=np.int64)
    assert m.shape == (T, w.K) and m.min() >= 1
    return m


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even.
    A storage-format conversion of the INPUT; inputs here are finite."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def _normal_f32(rng, size, sigma):
    a = rng.standard_normal(size, dtype=np.float32)
    a *= np.float32(sigma)
    return a


def initial_params(w: Workload, P: Optional[int] = None) -> np.ndarray:
    """x_0 ~ N(0, sigma_x), float32, flat (ragged layouts: the concatenation)."""
    rng = np.random.Generator(np.random.Philox(w.seed * 7919 + 2))
    return _normal_f32(rng, w.P if P is None else P, w.sigma_x)


def gradient_pool(w: Workload, P: Optional[int] = None, pool: Optional[int] = None):
    """R distinct micro-batch MEAN gradients ~ N(0, sigma_g): float32 arrays, or
    uint16 bf16 bit patterns when the workload's gradients are bf16."""
    R = w.pool if pool is None else pool
    size = w.P if P is None else P
    out = []
    for r in range(R):
        rng = np.random.Generator(np.random.Philox(w.seed * 7919 + 100 + r))
        g = _normal_f32(rng, size, w.sigma_g)
        out.append(to_bf16_bits(g) if w.grad_dtype == "bf16" else g)
    return out


def _mix64(z: int) -> int:
    z = (z + 0x9E3779B97F4A7C15) & 0xFFFFFFFFFFFFFFFF
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & 0xFFFFFFFFFFFFFFFF
    return z ^ (z >> 31)


def pool_index(w: Workload, t: int, k: int, j: int, pool: Optional[int] = None) -> int:
    """Which pool vector serves as micro-batch j of worker k in step t: a seeded start
    per (step, worker), then consecutive pool entries, so the gradients one worker
    takes in one step are distinct vectors as long as it takes no more than the pool
    holds (a vector read twice by one launch would be served from cache the second
    time, which no real sequence of micro-batch gradients offers)."""
    R = w.pool if pool is None else pool
    return (_mix64(_mix64(_mix64(w.seed) ^ t) ^ (k << 20)) + j) % R


def tensor_offsets(sizes):
    """Start of each tensor in the flat concatenation."""
    off = np.zeros(len(sizes) + 1, dtype=np.int64)
    np.cumsum(np.asarray(sizes, dtype=np.int64), out=off[1:])
    return off


def sample_indices(P: int, count: int, seed: int) -> np.ndarray:
    """Sorted sample of element indices that always includes both ends and
    positions around power-of-two block boundaries."""
    rng = np.random.Generator(np.random.Philox(seed))
    idx = set(int(i) for i in rng.integers(0, P, size=count))
    for b in (0, 1, 3, 4, 7, 8, 255, 256, 1023, 1024, 4095, 4096, 16383, 16384, 65535, 65536):
        for base in (b, P - 1 - b, P // 2 + b):
            if 0 <= base < P:
                idx.add(int(base))
    return np.array(sorted(idx), dtype=np.int64)
