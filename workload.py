"""Seeded synthetic workloads for the DASGD/SGNS worker step.

This module produces *data only*: token streams, unigram counts, the batch
schedule (which slice of the stream each worker sees at each step) and the
staleness draws for peer snapshots.  It contains none of the method's
arithmetic (no Philox, no alias table, no gradients), so both the HIP path and
the CPU oracle may be fed from it without sharing any computation; it belongs to
neither (it sits at the repository root, outside the product package and outside
``oracle/``) and imports neither.

The paper trains its word-embedding model on a 1 % sample of English Wikipedia
(Section 4, "Sparse vs. Dense Models"); that corpus is not available here, so
Zipf-distributed token streams stand in for it: natural-language word
frequencies are Zipf-like with exponent close to 1.  Token id 0 is the most
frequent word (frequency-sorted vocabulary).
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Config:
    """One synthetic workload.  Field names follow the paper's vocabulary where it
    has one (mini-batch, peers = other Model instances, Algorithm 1)."""

    idx: int            # 1..5, order of the benchmark configurations
    name: str
    vocab: int          # V
    dim: int            # D
    dtype: str          # "f32" | "bf16" (table element type)
    tokens: int         # T, stream length
    zipf_s: float       # Zipf exponent of the stream
    window: int         # w
    negatives: int      # N per (center, context) pair
    batch: int          # B centers per mini-batch
    peers: int          # K peer gradients applied per step
    max_stale: int      # peer snapshots are 0..max_stale steps old
    lr: float           # alpha of Eq. 1
    parity_steps: int   # steps the multi-step parity runs use
    grad_buffer: int = 1   # maxGradBuffer of Algorithm 1: own gradients summed per broadcast
    resample: bool = False   # variant: a negative equal to the pair's center or context is drawn once more
    stochastic_rounding: bool = False   # variant: bf16 tables are rounded stochastically by the table update

    # seeds: one per purpose so that changing one input does not move another
    @property
    def stream_seed(self) -> int:
        return 1000 + self.idx

    @property
    def seed(self) -> int:
        """Key of the model's counter-based generator (table init and negative draws)."""
        return 3000 + self.idx

    @property
    def stale_seed(self) -> int:
        return 4000 + self.idx

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def n_batches(self) -> int:
        """Mini-batches in one pass over the stream (tumbling window, last one partial)."""
        return -(-self.tokens // self.batch)

    def scaled(self, **kw) -> "Config":
        """A smaller or otherwise modified copy (tests use these)."""
        return dataclasses.replace(self, **kw)


CONFIGS = {
    1: Config(1, "cfg1_v1k_d32", 1_000, 32, "f32", 10_000, 1.0, 2, 5, 64, 0, 0, 0.025, 157),
    2: Config(2, "cfg2_v50k_d128_k3", 50_000, 128, "f32", 5_000_000, 1.0, 5, 5, 1_024, 3, 0, 0.025, 50),
    3: Config(3, "cfg3_v1m_d300_k7", 1_000_000, 300, "f32", 50_000_000, 1.1, 5, 10, 4_096, 7, 3, 0.025, 20),
    4: Config(4, "cfg4_hot_v10k_d256_k7", 10_000, 256, "f32", 20_000_000, 1.5, 8, 15, 16_384, 7, 0, 0.025, 20),
    5: Config(5, "cfg5_v2m_d512_bf16_k15", 2_000_000, 512, "bf16", 100_000_000, 1.05, 5, 10, 8_192, 15, 4, 0.025, 5),
}


def zipf_stream(vocab: int, s: float, n_tokens: int, seed: int, chunk: int = 1 << 23) -> np.ndarray:
    """int32[n_tokens] with P(token = r) proportional to (r+1)^-s, r in [0, vocab).

    Inverse-CDF sampling from a float64 cumulative table; the uniforms come from
    numpy's Philox bit generator keyed by ``seed`` (a data generator, unrelated
    to the negative-sampling generator of the method)."""
    ranks = np.arange(1, vocab + 1, dtype=np.float64)
    cdf = np.cumsum(ranks ** (-float(s)))
    cdf /= cdf[-1]
    rng = np.random.Generator(np.random.Philox(key=int(seed)))
    out = np.empty(n_tokens, dtype=np.int32)
    for lo in range(0, n_tokens, chunk):
        hi = min(n_tokens, lo + chunk)
        u = rng.random(hi - lo)
        idx = np.searchsorted(cdf, u, side="right")
        np.minimum(idx, vocab - 1, out=idx)
        out[lo:hi] = idx
    return out


def unigram_counts(tokens: np.ndarray, vocab: int) -> np.ndarray:
    """uint64[vocab] exact histogram of the stream."""
    return np.bincount(tokens, minlength=vocab).astype(np.uint64)


def make_stream(cfg: Config):
    """(tokens int32[T], counts uint64[V]) of a configuration."""
    tok = zipf_stream(cfg.vocab, cfg.zipf_s, cfg.tokens, cfg.stream_seed)
    return tok, unigram_counts(tok, cfg.vocab)


def batch_slice(cfg: Config, j: int):
    """Global mini-batch ``j`` of the tumbling window -> (center_begin, n_centers, epoch).

    Batches are consecutive runs of ``batch`` center positions; the last batch of a
    pass is partial; after the last batch the stream is iterated again and
    ``epoch`` goes up by one (the paper re-iterates its datasets to simulate an
    unbounded stream, Section 4 "Event Generation")."""
    nb = cfg.n_batches
    epoch, b = divmod(int(j), nb)
    begin = b * cfg.batch
    return begin, min(cfg.batch, cfg.tokens - begin), epoch


def worker_batch(cfg: Config, step: int, worker: int):
    """Mini-batch of ``worker`` (0 = this worker, 1..K = peers) at ``step``.

    Mini-batches are dealt round-robin to the K+1 Model instances (step (4) of the
    paper's dataflow sends each mini-batch to one instance)."""
    return batch_slice(cfg, step * (cfg.peers + 1) + worker)


def stale_draws(cfg: Config, n_steps: int) -> np.ndarray:
    """int64[n_steps, K]: how many of this worker's steps old the model snapshot is
    on which peer k computed the gradient applied at step t (uniform 0..max_stale)."""
    rng = np.random.Generator(np.random.Philox(key=int(cfg.stale_seed)))
    k = max(cfg.peers, 1)
    d = rng.integers(0, cfg.max_stale + 1, size=(n_steps, k), dtype=np.int64)
    return d[:, : cfg.peers]


def pairs_in_batch(cfg: Config, center_begin: int, n_centers: int) -> int:
    """Number of (center, context) pairs of a batch, by direct counting (harness
    bookkeeping for the pairs/s metric; both implementations count on their own)."""
    p = np.arange(center_begin, center_begin + n_centers, dtype=np.int64)
    left = np.minimum(p, cfg.window)
    right = np.minimum(cfg.tokens - 1 - p, cfg.window)
    return int((left + right).sum())
