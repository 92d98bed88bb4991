"""Seeded synthetic parameter stores shaped like the paper's MLR / MF / LDA / CNN
workloads (Section 5.1) plus a large flat store.

This module only *makes inputs*: live parameters x, a running checkpoint c, the
checkpoint size k and a lost block set S.  It holds none of the method's arithmetic
(no scores, no selection, no norms) so that both the GPU library's tests and the CPU
oracle can be fed from it without sharing any computation.

The paper's datasets (MNIST, CoverType, MovieLens, Jester, 20 Newsgroups, Reuters,
ClueWeb12) are not reproduced; these stores stand in for their parameter shapes and
for the rough structure of how much each block moves between checkpoints.
"""
from dataclasses import dataclass, field
import math

import numpy as np

F32, BF16, I32, F32_BF16C = 0, 1, 2, 3      # F32_BF16C: float32 x, bfloat16 checkpoint c
ELEM_BYTES = {F32: 4, BF16: 2, I32: 4}
NUMPY_DTYPE = {F32: np.float32, BF16: np.uint16, I32: np.int32}


@dataclass
class Workload:
    name: str
    dtype: int               # F32 / BF16 / I32
    block_len: int           # elements per block ("parameter" unit of the paper)
    x: np.ndarray            # live parameters, flat
    c: np.ndarray            # running checkpoint, flat, same dtype and size
    k: int                   # blocks saved per checkpoint
    lost: np.ndarray         # uint32 ascending indices of the lost blocks
    note: str = ""
    extra: dict = field(default_factory=dict)

    @property
    def n_elems(self) -> int:
        return int(self.x.size)

    @property
    def n_blocks(self) -> int:
        return (self.n_elems + self.block_len - 1) // self.block_len


def n_blocks_of(n_elems: int, block_len: int) -> int:
    return (n_elems + block_len - 1) // block_len


def k_of_fraction(r: float, n_blocks: int) -> int:
    """Checkpoint size for a fraction r of the blocks: ceil(r * n_blocks), at most n_blocks."""
    return min(n_blocks, int(math.ceil(r * n_blocks - 1e-9)))


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round to nearest, ties to even); returns the uint16 bits."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    nan = (u & 0x7FFFFFFF) > 0x7F800000
    lsb = (u >> 16) & 1
    r = (u + (0x7FFF + lsb)) >> 16
    r = np.where(nan, (u >> 16) | 0x0040, r)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32 (for building inputs only)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def random_lost_blocks(n_blocks: int, n_lost: int, seed: int) -> np.ndarray:
    """A uniformly random lost set of n_lost blocks (random partitioning, Section 4.1)."""
    rng = np.random.default_rng(seed)
    return np.sort(rng.choice(n_blocks, size=n_lost, replace=False)).astype(np.uint32)


def random_partitions(n_blocks: int, n_parts: int, seed: int):
    """Blocks dealt uniformly at random to n_parts near-equal partitions (PS nodes)."""
    rng = np.random.default_rng(seed)
    perm = rng.permutation(n_blocks)
    return [np.sort(p).astype(np.uint32) for p in np.array_split(perm, n_parts)]


def mlr_like(seed: int = 0, rows: int = 1000, cols: int = 784) -> Workload:
    """MLR-like fp32 weight matrix; block = row; log-normal per-row change scale."""
    rng = np.random.default_rng(seed)
    c = rng.normal(0.0, 0.1, size=(rows, cols)).astype(np.float32)
    s_r = rng.lognormal(-3.0, 1.0, size=(rows, 1))
    x = (c + rng.normal(0.0, 1.0, size=(rows, cols)) * s_r).astype(np.float32)
    k = k_of_fraction(0.25, rows)
    lost = random_lost_blocks(rows, rows // 2, seed + 1000)
    return Workload("mlr_like", F32, cols, x.reshape(-1), c.reshape(-1), k, lost,
                    "top 25% rows, random 50% rows lost")


def mf_like(seed: int = 1, u_rows: int = 138_000, v_rows: int = 27_000, rank: int = 100) -> Workload:
    """MF-like stacked factor table [U; V]; per-row change follows a rank^-1.1 law."""
    rng = np.random.default_rng(seed)
    rows = u_rows + v_rows
    c = rng.normal(0.0, 0.05, size=(rows, rank)).astype(np.float32)
    scale = np.empty(rows)
    for lo, n in ((0, u_rows), (u_rows, v_rows)):
        ranks = rng.permutation(n) + 1
        scale[lo:lo + n] = 0.05 * ranks.astype(np.float64) ** -1.1
    x = np.empty_like(c)
    step = 16384
    for lo in range(0, rows, step):
        hi = min(rows, lo + step)
        x[lo:hi] = c[lo:hi] + rng.normal(0.0, 1.0, size=(hi - lo, rank)) * scale[lo:hi, None]
    k = k_of_fraction(0.10, rows)
    lost = np.arange(0, u_rows // 4, dtype=np.uint32)
    return Workload("mf_like", F32, rank, x.reshape(-1), c.reshape(-1), k, lost,
                    "top 10% rows, first quarter of U lost")


def lda_like(seed: int = 2, words: int = 100_000, topics: int = 1000, tokens: float = 2e9,
             moved_fraction: float = 0.02) -> Workload:
    """LDA-like int32 count table; Zipf word frequencies; sparse signed count moves."""
    rng = np.random.default_rng(seed)
    ranks = rng.permutation(words) + 1
    f = ranks.astype(np.float64) ** -1.07
    f /= f.sum()
    lam = tokens * f / topics
    c = np.empty((words, topics), dtype=np.int32)
    step = 8192
    for lo in range(0, words, step):
        hi = min(words, lo + step)
        c[lo:hi] = rng.poisson(np.broadcast_to(lam[lo:hi, None], (hi - lo, topics))).astype(np.int32)
    x = c.copy()
    n_pairs = moved_fraction * words * topics / 2.0
    w = np.sqrt(f)
    w /= w.sum()
    cap = min(250, topics // 2)
    pairs = np.minimum(cap, rng.poisson(n_pairs * w))
    for r in np.nonzero(pairs)[0]:
        p = int(pairs[r])
        cols = rng.choice(topics, size=2 * p, replace=False)
        src, dst = cols[:p], cols[p:]
        m = np.minimum(c[r, src], 1 + rng.poisson(1.0, size=p)).astype(np.int32)
        x[r, src] -= m
        x[r, dst] += m
    k = k_of_fraction(0.05, words)
    lost = random_partitions(words, 8, seed + 1000)[0]
    return Workload("lda_like", I32, topics, x.reshape(-1), c.reshape(-1), k, lost,
                    "top 5% rows, one of 8 random partitions lost")


def doc_topic_like(seed: int = 7, docs: int = 20_000, topics: int = 100, resampled: float = 0.05,
                   dtype: int = F32):
    """Document-topic distributions as an LDA trainer holds them (Section 5.1): row d is the
    topic proportions of a document of N_d tokens (N_d log-normal, median about 150),
    checkpoint c = the proportions at the last checkpoint, x = after a fraction `resampled`
    of every document's tokens has been re-assigned to another topic.  Returns the workload
    with extra["lengths"] = float32 N_d, the weights of the scaled total variation."""
    rng = np.random.default_rng(seed)
    lengths = np.maximum(5, rng.lognormal(5.0, 1.0, size=docs)).astype(np.int64)
    theta = rng.dirichlet(np.full(topics, 0.1), size=docs)
    counts_c = np.stack([rng.multinomial(int(n), p) for n, p in zip(lengths, theta)]).astype(np.int64)
    counts_x = counts_c.copy()
    moves = rng.binomial(lengths, resampled)
    for d in np.nonzero(moves)[0]:
        for _ in range(int(moves[d])):
            src = rng.choice(topics, p=counts_x[d] / counts_x[d].sum())
            dst = int(rng.integers(0, topics))
            counts_x[d, src] -= 1
            counts_x[d, dst] += 1
    c = (counts_c / lengths[:, None]).astype(np.float32)
    x = (counts_x / lengths[:, None]).astype(np.float32)
    if dtype == BF16:
        x, c = f32_to_bf16_bits(x), f32_to_bf16_bits(c)
    k = k_of_fraction(0.125, docs)
    lost = random_partitions(docs, 4, seed + 1000)[0]
    return Workload("doc_topic_like", dtype, topics, x.reshape(-1), c.reshape(-1), k, lost,
                    "top 1/8 of the documents, one of 4 random partitions lost",
                    {"lengths": lengths.astype(np.float32)})


def cnn_like(seed: int = 3, n_elems: int = 25_000_000, block_len: int = 4096,
             fraction: float = 0.10) -> Workload:
    """CNN-like flat fp32 vector in fixed-size shards (ragged tail), per-shard change scale."""
    rng = np.random.default_rng(seed)
    nb = n_blocks_of(n_elems, block_len)
    c = rng.normal(0.0, 0.02, size=n_elems).astype(np.float32)
    u_b = rng.uniform(0.1, 10.0, size=nb)
    x = np.empty_like(c)
    step = 256
    for b0 in range(0, nb, step):
        b1 = min(nb, b0 + step)
        lo, hi = b0 * block_len, min(n_elems, b1 * block_len)
        sc = np.repeat(u_b[b0:b1], block_len)[: hi - lo]
        x[lo:hi] = c[lo:hi] + rng.normal(0.0, 1e-3, size=hi - lo) * sc
    k = k_of_fraction(fraction, nb)
    parts = random_partitions(nb, 16, seed + 1000)
    which = np.random.default_rng(seed + 2000).choice(16, size=3, replace=False)
    lost = np.sort(np.concatenate([parts[i] for i in which])).astype(np.uint32)
    return Workload("cnn_like", F32, block_len, x, c, k, lost,
                    "top %g%% shards, 3 of 16 random partitions lost" % (100 * fraction),
                    {"fraction": fraction})


@dataclass
class VarWorkload:
    name: str
    dtype: int
    offsets: np.ndarray      # uint64, n_blocks + 1 element offsets
    x: np.ndarray
    c: np.ndarray
    k: int
    lost: np.ndarray
    note: str = ""

    @property
    def n_blocks(self) -> int:
        return int(self.offsets.size - 1)


# The paper's CNN (Section 5.1): two 5x5 convolutions and three fully-connected layers,
# weights and biases as separate parameters ("by-layer").  Sizes are those of a common
# MNIST network of that shape.
CNN_LAYER_SIZES = (5 * 5 * 1 * 32, 32, 5 * 5 * 32 * 64, 64, 7 * 7 * 64 * 1024, 1024,
                   1024 * 512, 512, 512 * 10, 10)


def layers_like(sizes=CNN_LAYER_SIZES, seed: int = 5, fraction: float = 0.25, n_lost: int = 3,
                dtype: int = F32) -> VarWorkload:
    """A store cut "by layer": one block per tensor, sizes as given (zero allowed)."""
    rng = np.random.default_rng(seed)
    sizes = np.asarray(sizes, dtype=np.int64)
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.uint64)
    n, nb = int(off[-1]), sizes.size
    if dtype == I32:
        c = rng.integers(0, 1000, size=n).astype(np.int32)
        x = c + (rng.integers(-3, 4, size=n) * (rng.random(n) < 0.05)).astype(np.int32)
    else:
        c = rng.normal(0.0, 0.02, size=n).astype(np.float32)
        u = rng.uniform(0.1, 10.0, size=nb)
        x = (c + rng.normal(0.0, 1e-3, size=n) * np.repeat(u, sizes)).astype(np.float32)
        if dtype == BF16:
            x, c = f32_to_bf16_bits(x), f32_to_bf16_bits(c)
    k = k_of_fraction(fraction, nb)
    lost = random_lost_blocks(nb, min(n_lost, nb), seed + 1000)
    return VarWorkload("layers_like", dtype, off, x, c, k, lost,
                       "%d tensors of %d..%d elements" % (nb, sizes.min(), sizes.max()))


def mixed_layer_sizes(n_layers: int, total: int, seed: int = 6):
    """n_layers tensor sizes spread over four orders of magnitude that add up to about
    `total` elements, a few of them empty or tiny, none aligned to anything."""
    rng = np.random.default_rng(seed)
    w = rng.lognormal(0.0, 2.5, size=n_layers)
    sizes = np.maximum(1, (w / w.sum() * total)).astype(np.int64)
    sizes[rng.choice(n_layers, size=max(1, n_layers // 16), replace=False)] = 0
    sizes[rng.choice(n_layers, size=max(1, n_layers // 16), replace=False)] = 3
    return sizes


def student_t3(rng: np.random.Generator, n: int) -> np.ndarray:
    """Student-t with 3 degrees of freedom: Z0 / sqrt((Z1^2 + Z2^2 + Z3^2) / 3)."""
    z = rng.standard_normal(size=(4, n))
    return z[0] / np.sqrt((z[1] ** 2 + z[2] ** 2 + z[3] ** 2) / 3.0)


def flat_like(seed: int = 4, n_elems: int = 1 << 30, block_len: int = 1024,
              dtype: int = F32) -> Workload:
    """Large flat store on the host (numpy): heavy-tailed deltas.  Use flat_like_torch for
    the full 2^30-element size, which is generated on the device."""
    rng = np.random.default_rng(seed)
    c = np.empty(n_elems, dtype=np.float32)
    x = np.empty(n_elems, dtype=np.float32)
    step = 1 << 22
    for lo in range(0, n_elems, step):
        hi = min(n_elems, lo + step)
        c[lo:hi] = rng.normal(0.0, 0.02, size=hi - lo)
        x[lo:hi] = c[lo:hi] + 1e-3 * student_t3(rng, hi - lo)
    nb = n_blocks_of(n_elems, block_len)
    k = k_of_fraction(0.10, nb)
    lost = random_lost_blocks(nb, nb // 8, seed + 1000)
    if dtype == BF16:
        x, c = f32_to_bf16_bits(x), f32_to_bf16_bits(c)
    elif dtype == F32_BF16C:
        c = f32_to_bf16_bits(c)
    return Workload("flat_like", dtype, block_len, x, c, k, lost,
                    "top 10% blocks, random 1/8 of blocks lost")


def flat_like_torch(device, seed: int = 4, n_elems: int = 1 << 30, chunk: int = 1 << 26):
    """The large flat store generated chunk by chunk on `device` with torch's seeded
    generator.  Returns float32 tensors (x, c).  A bfloat16 copy is x.to(bfloat16),
    c.to(bfloat16) (round to nearest even)."""
    import torch

    g = torch.Generator(device=device)
    g.manual_seed(seed)
    c = torch.empty(n_elems, dtype=torch.float32, device=device)
    x = torch.empty(n_elems, dtype=torch.float32, device=device)
    for lo in range(0, n_elems, chunk):
        hi = min(n_elems, lo + chunk)
        m = hi - lo
        c[lo:hi].normal_(0.0, 0.02, generator=g)
        z = torch.empty((4, m), dtype=torch.float32, device=device).normal_(generator=g)
        t3 = z[0] / torch.sqrt((z[1] * z[1] + z[2] * z[2] + z[3] * z[3]) / 3.0)
        x[lo:hi] = c[lo:hi] + 1e-3 * t3
        del z, t3
    return x, c


def drift_torch(x, seed: int, fraction: float = 0.10, block_len: int = 1024):
    """Stand-in for the training iterations between two checkpoints: add a fresh
    heavy-tailed delta to a random `fraction` of the blocks of the float32 tensor x, in place."""
    import torch

    g = torch.Generator(device=x.device)
    g.manual_seed(seed)
    nb = x.numel() // block_len
    m = max(1, int(nb * fraction))
    start = int(torch.randint(0, max(1, nb - m + 1), (1,), generator=g, device=x.device).item())
    view = x[start * block_len:(start + m) * block_len]
    z = torch.empty((4, view.numel()), dtype=torch.float32, device=x.device).normal_(generator=g)
    view += 1e-3 * z[0] / torch.sqrt((z[1] * z[1] + z[2] * z[2] + z[3] * z[3]) / 3.0)
