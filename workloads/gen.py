"""Seeded synthetic workloads shaped like the paper's draft-step microbenchmark.

The paper benchmarks its subset-logits kernel on synthetic activations and
weights at each model's dimensions (Section 6, the paragraph on the kernel's speed-up).  The
same is done here: weights ~ N(0, 0.02^2), hidden states ~ N(0, 1), and index
sets biased towards frequent tokens (Zipf, exponent 1.1) because the candidate
vocabulary of a language model is dominated by frequent tokens (Section 1).

Nothing in this file computes any step of the method; it only draws numbers and
converts dtypes.  Both the CPU oracle's tests and the HIP tests import it.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

SEED_BASE = 13836 * 1000

# stream ids used for the per-config seeds
STREAM_WEIGHTS = 0
STREAM_HIDDEN = 1
STREAM_INDICES = 2
STREAM_SELECTOR = 3


def make_rng(config: int, stream: int) -> np.random.Generator:
    """PCG64 generator for (config number, stream id)."""
    return np.random.Generator(np.random.PCG64(SEED_BASE + 100 * config + stream))


# --------------------------------------------------------------------------
# dtype conversion (storage formats only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even), returned as uint16 bit patterns.

    Finite inputs only (the generators never produce inf/nan).
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns (uint16) to float32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_matrix(rng: np.random.Generator, shape, std: float, dtype: str,
                  chunk_rows: int = 4096, workers: int = 8) -> np.ndarray:
    """N(0, std^2) matrix. dtype 'f32' -> float32 array; 'bf16' -> uint16 bit patterns.

    Matrices are drawn in blocks of `chunk_rows` rows, block i from the i-th child generator
    spawned from `rng`, so the result does not depend on how many threads fill the blocks."""
    shape = tuple(int(s) for s in shape)
    if dtype not in ("f32", "bf16"):
        raise ValueError(f"unknown dtype {dtype!r}")
    if len(shape) == 1:
        x = rng.standard_normal(shape, dtype=np.float32) * np.float32(std)
        return x if dtype == "f32" else f32_to_bf16_bits(x)
    rows = shape[0]
    starts = list(range(0, rows, chunk_rows))
    children = rng.spawn(len(starts))
    out = np.empty(shape, dtype=np.float32 if dtype == "f32" else np.uint16)

    def fill(i):
        r0 = starts[i]
        r1 = min(rows, r0 + chunk_rows)
        blk = children[i].standard_normal((r1 - r0,) + shape[1:], dtype=np.float32)
        blk *= np.float32(std)
        out[r0:r1] = blk if dtype == "f32" else f32_to_bf16_bits(blk)

    if len(starts) == 1:
        fill(0)
    else:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=workers) as pool:
            list(pool.map(fill, range(len(starts))))
    return out


def hidden_rows(rng: np.random.Generator, rows: int, d: int, dtype: str) -> np.ndarray:
    """Hidden states h ~ N(0,1), [rows x d], in the storage dtype of the weights."""
    return normal_matrix(rng, (rows, d), 1.0, dtype)


# --------------------------------------------------------------------------
# Zipf-biased index sets
# --------------------------------------------------------------------------
def _zipf_keys(rng: np.random.Generator, V: int, s: float,
               rank_of_id: Optional[np.ndarray]) -> np.ndarray:
    """Gumbel-perturbed log-weights: the k largest are a weighted sample without replacement
    with P(token) proportional to rank^-s."""
    if rank_of_id is None:
        rank = np.arange(1, V + 1, dtype=np.float64)
    else:
        rank = np.asarray(rank_of_id, dtype=np.float64) + 1.0
    g = rng.gumbel(size=V)
    return -s * np.log(rank) + g


def zipf_subset(rng: np.random.Generator, V: int, k: int, s: float = 1.1,
                rank_of_id: Optional[np.ndarray] = None,
                exclude: Optional[np.ndarray] = None) -> np.ndarray:
    """k unique token ids in [0,V), sampled without replacement with weight rank^-s,
    returned sorted ascending as int32.  `rank_of_id[v]` is the 0-based frequency rank of
    token v (identity when None: low ids are the frequent tokens).  Ids in `exclude` are
    never drawn."""
    if not (1 <= k <= V):
        raise ValueError("need 1 <= k <= V")
    keys = _zipf_keys(rng, V, s, rank_of_id)
    if exclude is not None and len(exclude):
        if k > V - len(exclude):
            raise ValueError("k exceeds the number of drawable ids")
        keys[np.asarray(exclude, dtype=np.int64)] = -np.inf
    if k == V:
        return np.arange(V, dtype=np.int32)
    top = np.argpartition(keys, V - k)[V - k:]
    top.sort()
    return top.astype(np.int32)


def zipf_subsets(rng: np.random.Generator, V: int, k: int, n: int, s: float = 1.1,
                 rank_of_id: Optional[np.ndarray] = None) -> np.ndarray:
    """n independent subsets, [n x k] int32, each row sorted ascending."""
    out = np.empty((n, k), dtype=np.int32)
    for i in range(n):
        out[i] = zipf_subset(rng, V, k, s, rank_of_id)
    return out


def tree_subsets(rng: np.random.Generator, V: int, rows: int, k: int, shared: int,
                 s: float = 1.1, rank_of_id: Optional[np.ndarray] = None):
    """Per-row index sets for a draft tree: every row holds the same step-level set S
    (|S| = shared, a Zipf draw) plus k-shared row-private Zipf draws outside S.
    Returns (idx [rows x k] int32, each row sorted ascending; S sorted ascending)."""
    if not (0 <= shared <= k):
        raise ValueError("need 0 <= shared <= k")
    S = zipf_subset(rng, V, shared, s, rank_of_id) if shared else np.empty(0, np.int32)
    idx = np.empty((rows, k), dtype=np.int32)
    for r in range(rows):
        if k > shared:
            priv = zipf_subset(rng, V, k - shared, s, rank_of_id, exclude=S)
            row = np.concatenate([S, priv])
            row.sort()
        else:
            row = S.copy()
        idx[r] = row
    return idx, S


# --------------------------------------------------------------------------
# workload table
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    """Shapes of one benchmark / parity configuration."""
    number: int
    name: str
    d: int
    V: int
    dtype: str            # storage dtype of h, U, W_down, W_vocab: 'f32' or 'bf16'
    rows: int             # hidden-state rows per draft step
    k: int                # subset size per row
    kd: int               # draft tokens per row
    idx_mode: str         # 'per_row' or 'per_step'
    d_prime: int = 0      # selector width (0: the config has no selector)
    steps: int = 1
    shared: int = 0       # size of the step-level shared set (tree configs)
    k_sweep: tuple = field(default_factory=tuple)

    def esize(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def weights(self) -> np.ndarray:
        """Output embedding U [V x d] ~ N(0, 0.02^2)."""
        return normal_matrix(make_rng(self.number, STREAM_WEIGHTS), (self.V, self.d), 0.02, self.dtype)

    def selector(self, d_prime: Optional[int] = None):
        """Seeded random-init selector (W_down [d' x d], W_vocab [V x d']) ~ N(0, 0.02^2)."""
        dp = int(d_prime or self.d_prime)
        rng = make_rng(self.number, STREAM_SELECTOR)
        w_down = normal_matrix(rng, (dp, self.d), 0.02, self.dtype)
        w_vocab = normal_matrix(rng, (self.V, dp), 0.02, self.dtype)
        return w_down, w_vocab

    def hidden(self, steps: Optional[int] = None) -> np.ndarray:
        """[steps x rows x d] hidden states."""
        n = int(steps or self.steps)
        rng = make_rng(self.number, STREAM_HIDDEN)
        return normal_matrix(rng, (n * self.rows, self.d), 1.0, self.dtype).reshape(n, self.rows, self.d)

    def indices(self, steps: Optional[int] = None, k: Optional[int] = None) -> np.ndarray:
        """Index sets for `steps` draft steps: [steps x rows x k] (per_row) or [steps x k] (per_step)."""
        n = int(steps or self.steps)
        kk = int(k or self.k)
        rng = make_rng(self.number, STREAM_INDICES)
        if self.idx_mode == "per_step":
            return zipf_subsets(rng, self.V, kk, n)
        out = np.empty((n, self.rows, kk), dtype=np.int32)
        for t in range(n):
            if self.shared:
                sh = (self.shared * kk) // self.k
                out[t], _ = tree_subsets(rng, self.V, self.rows, kk, sh)
            else:
                out[t] = zipf_subsets(rng, self.V, kk, self.rows)
        return out


CONFIGS = {
    # tiny CPU-checkable case
    1: Workload(1, "tiny-fp32", d=256, V=8192, dtype="f32", rows=1, k=512, kd=8,
                idx_mode="per_row", d_prime=32, steps=4),
    # Llama-3-8B-shaped chain drafting (the headline workload)
    2: Workload(2, "llama3-8b-chain", d=4096, V=128256, dtype="bf16", rows=1, k=8192, kd=10,
                idx_mode="per_row", d_prime=256, steps=1000),
    # tree drafting: 60 rows, own k=4096 subset each, half of it shared step-wide
    3: Workload(3, "llama3-8b-tree60", d=4096, V=128256, dtype="bf16", rows=60, k=4096, kd=10,
                idx_mode="per_row", d_prime=256, steps=4, shared=2048),
    # large-vocabulary Gemma-style head, 8 rows, k sweep
    4: Workload(4, "gemma-262k", d=3840, V=262144, dtype="bf16", rows=8, k=8192, kd=10,
                idx_mode="per_step", d_prime=240, steps=4, k_sweep=(2048, 8192, 32768)),
    # full draft step with the selector, Qwen3-8B shape, 16 requests x 32 tree rows
    5: Workload(5, "qwen3-8b-select", d=4096, V=151936, dtype="bf16", rows=512, k=8192, kd=10,
                idx_mode="per_row", d_prime=256, steps=1),
}
