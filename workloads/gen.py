"""Synthetic, seeded stand-ins for production behaviour-sequence logs.

Every array the embedding path consumes is produced here: raw (untagged) feature
IDs per feature field, per-sample list lengths, the feature declarations a
caller would hand to the table-merging planner, and upstream gradients.  The
shapes follow the five benchmark configurations (tiny / long-sequence lookup /
table merging / insert-delete stress / large bf16 table).

Nothing in this file is part of the method under test.  In particular the
rank -> raw-ID scramble below is *workload* arithmetic (it only decides which
64-bit values the synthetic users and items carry) and is unrelated to the
table's slot hash or to row initialisation.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

SEED_BASE = 0x2505_1266_3000
_U64 = np.uint64


# --------------------------------------------------------------------------- #
# rank -> raw ID bijection on [0, 2^bits)
# --------------------------------------------------------------------------- #
def _odd_constants(seed: int, bits: int) -> List[int]:
    """Three odd multipliers derived from the seed (plain LCG stepping)."""
    out, s = [], (seed * 0x9E3779B97F4A7C15 + 0x7F4A7C15) & (2**64 - 1)
    for _ in range(3):
        s = (s * 6364136223846793005 + 1442695040888963407) & (2**64 - 1)
        out.append(((s >> 11) | 1) & ((1 << bits) - 1) | 1)
    return out


def scramble_bits(rank: np.ndarray, bits: int, seed: int) -> np.ndarray:
    """Seeded bijection on [0, 2^bits): odd multiply + xor-shift rounds.

    Makes popularity (rank) uncorrelated with the numeric key value."""
    assert 2 <= bits <= 63
    mask = _U64((1 << bits) - 1)
    sh = _U64((bits + 1) // 2)
    x = (np.asarray(rank, dtype=_U64) + _U64(seed & ((1 << bits) - 1))) & mask
    for c in _odd_constants(seed, bits):
        x = (x * _U64(c)) & mask
        x = x ^ (x >> sh)
    return x


def unscramble_bits(x: np.ndarray, bits: int, seed: int) -> np.ndarray:
    """Inverse of :func:`scramble_bits` (used to test that it is a bijection)."""
    mask_i = (1 << bits) - 1
    mask = _U64(mask_i)
    sh = (bits + 1) // 2
    x = np.asarray(x, dtype=_U64) & mask
    for c in reversed(_odd_constants(seed, bits)):
        # undo x ^= x >> sh: since 2*sh >= bits the map is its own inverse
        y = x ^ (x >> _U64(sh))
        x = (y * _U64(pow(c, -1, 1 << bits))) & mask
    return (x - _U64(seed & mask_i)) & mask


# --------------------------------------------------------------------------- #
# bounded Zipf ranks
# --------------------------------------------------------------------------- #
_HEAD = 1 << 18
_head_cache: Dict[Tuple[int, float], np.ndarray] = {}


def _head_cdf(k: int, alpha: float) -> np.ndarray:
    key = (k, alpha)
    if key not in _head_cache:
        w = np.arange(1, k + 1, dtype=np.float64) ** (-alpha)
        _head_cache[key] = np.cumsum(w)
    return _head_cache[key]


def bounded_zipf_ranks(rng: np.random.Generator, n: int, R: int, alpha: float) -> np.ndarray:
    """n draws of a 0-based rank r in [0, R) with P(r) ~ (r+1)^-alpha.

    Exact for the 2^18 most popular ranks (CDF table + binary search); beyond
    that the discrete tail is replaced by its continuous envelope on
    [K+1/2, R+1/2) and inverted in closed form."""
    R = int(R)
    K = min(R, _HEAD)
    cdf = _head_cdf(K, alpha)
    head_mass = cdf[-1]
    a, b = K + 0.5, R + 0.5
    if R > K:
        if abs(alpha - 1.0) < 1e-12:
            tail_mass = math.log(b / a)
        else:
            tail_mass = (b ** (1 - alpha) - a ** (1 - alpha)) / (1 - alpha)
    else:
        tail_mass = 0.0
    u = rng.random(n) * (head_mass + tail_mass)
    out = np.empty(n, dtype=np.int64)
    in_head = u < head_mass
    out[in_head] = np.searchsorted(cdf, u[in_head], side="right")
    if tail_mass > 0.0:
        v = u[~in_head] - head_mass
        if abs(alpha - 1.0) < 1e-12:
            x = a * np.exp(v)
        else:
            x = (v * (1 - alpha) + a ** (1 - alpha)) ** (1.0 / (1 - alpha))
        out[~in_head] = np.clip(np.rint(x).astype(np.int64) - 1, K, R - 1)
    np.clip(out, 0, R - 1, out=out)
    return out


# --------------------------------------------------------------------------- #
# declarations
# --------------------------------------------------------------------------- #
@dataclass
class FeatureDecl:
    """What a user declares per feature: name, vocabulary, dim, lookup table."""
    name: str
    table: int          # logical lookup-table id, 0-based (features may share one)
    vocab: int          # vocabulary of that logical table at step 0
    dim: int
    dtype: str = "f32"  # "f32" | "bf16"


@dataclass
class StepBatch:
    step: int
    ids: List[np.ndarray]        # per feature: raw IDs, uint64, sample-major
    ranks: List[np.ndarray]      # per feature: the popularity rank behind each ID
    lengths: List[np.ndarray]    # per feature: int32[batch] list length per sample
    fresh: List[np.ndarray]      # per feature: bool, rank was never issued before


@dataclass
class Workload:
    name: str
    config_id: int
    features: List[FeatureDecl]
    batch: int
    alpha: float
    id_bits: int
    len_mode: str                 # "per_field_uniform" | "per_sample_uniform" | "fixed"
    len_lo: int
    len_hi: int
    fresh_frac: float = 0.0       # share of a step's distinct keys never seen before
    prepopulated: Optional[List[int]] = None   # per logical table: ranks [0,P) exist at start
    lr: float = 0.01
    eps: float = 1e-8
    tag_bits: Optional[int] = None
    steps: int = 3
    seed: int = 0
    # eviction policy knobs (only the stress configuration uses them)
    ttl: int = 0
    min_freq: int = 0
    grace: int = 0
    evict_every: int = 0
    max_load_factor: float = 0.75
    _issued: List[int] = field(default_factory=list)   # per logical table: ranks issued so far

    def __post_init__(self):
        self.seed = SEED_BASE + self.config_id
        self.reset()

    # -- bookkeeping ------------------------------------------------------- #
    @property
    def n_tables(self) -> int:
        return 1 + max(f.table for f in self.features)

    def table_vocab(self, t: int) -> int:
        return next(f.vocab for f in self.features if f.table == t)

    def table_dim(self, t: int) -> int:
        return next(f.dim for f in self.features if f.table == t)

    def table_dtype(self, t: int) -> str:
        return next(f.dtype for f in self.features if f.table == t)

    def reset(self) -> None:
        self._issued = [self.table_vocab(t) for t in range(self.n_tables)]

    def table_seed(self, t: int) -> int:
        return (self.seed * 1000003 + 7919 * (t + 1)) & (2**63 - 1)

    def raw_ids_of_ranks(self, t: int, ranks: np.ndarray) -> np.ndarray:
        return scramble_bits(ranks, self.id_bits, self.table_seed(t))

    def prepopulated_ids(self, t: int, lo: int, hi: int) -> np.ndarray:
        """Raw IDs of ranks [lo, hi) of logical table t (for bulk loading)."""
        return self.raw_ids_of_ranks(t, np.arange(lo, hi, dtype=np.uint64))

    # -- one step of input ------------------------------------------------- #
    def _lengths(self, rng: np.random.Generator) -> List[np.ndarray]:
        B, F = self.batch, len(self.features)
        if self.len_mode == "fixed":
            return [np.full(B, self.len_lo, dtype=np.int32) for _ in range(F)]
        if self.len_mode == "per_sample_uniform":
            L = rng.integers(self.len_lo, self.len_hi + 1, size=B).astype(np.int32)
            return [L.copy() for _ in range(F)]
        return [rng.integers(self.len_lo, self.len_hi + 1, size=B).astype(np.int32) for _ in range(F)]

    def next_step(self, step: int) -> StepBatch:
        """Generate the batch of one step.  Steps must be drawn in order 0,1,2,...
        after :meth:`reset` because fresh keys advance a per-table counter."""
        rng = np.random.Generator(np.random.Philox(key=(self.seed + 0x9E37 * (step + 1)) & (2**64 - 1)))
        lengths = self._lengths(rng)
        ids, ranks_out, fresh_out = [], [], []
        for fi, f in enumerate(self.features):
            n = int(lengths[fi].sum())
            R = self._issued[f.table]
            r = bounded_zipf_ranks(rng, n, R, self.alpha)
            fresh = np.zeros(n, dtype=bool)
            if self.fresh_frac > 0.0 and n > 0:
                u_old = len(np.unique(r))
                n_fresh = int(round(self.fresh_frac / (1.0 - self.fresh_frac) * u_old))
                n_fresh = min(n_fresh, n)
                if n_fresh > 0:
                    pos = rng.choice(n, size=n_fresh, replace=False)
                    r[pos] = R + np.arange(n_fresh, dtype=np.int64)
                    fresh[pos] = True
                    self._issued[f.table] = R + n_fresh
            ranks_out.append(r)
            fresh_out.append(fresh)
            ids.append(self.raw_ids_of_ranks(f.table, r.astype(np.uint64)))
        return StepBatch(step=step, ids=ids, ranks=ranks_out, lengths=lengths, fresh=fresh_out)


# --------------------------------------------------------------------------- #
# the five configurations
# --------------------------------------------------------------------------- #
_FIELDS8 = ["item", "category", "shop", "brand", "price_bucket", "time_bucket", "action", "scene"]


def make_config(config_id: int, *, batch: Optional[int] = None, vocab_scale: float = 1.0,
                len_hi: Optional[int] = None, len_lo: Optional[int] = None,
                steps: Optional[int] = None, field_vocab: Optional[Sequence[int]] = None) -> Workload:
    """Build configuration 1..5.  ``batch``/``vocab_scale``/``len_*`` shrink a
    configuration for quick checks; defaults give the full published shape.
    ``field_vocab`` (configuration 2 only) replaces the per-field vocabulary sizes, e.g. a few
    fields with under a thousand values (action, scene, hour) next to item-like ones."""
    vs = lambda v: max(16, int(v * vocab_scale))
    if config_id == 1:
        feats = [FeatureDecl(f"f{i}", 0, vs(100_000), 32) for i in range(4)]
        # one logical table shared by four fields, 100k-key space
        w = Workload("tiny", 1, feats, batch or 256, 1.1, 17, "per_field_uniform", len_lo or 1, len_hi or 64,
                     steps=steps or 3)
        return w
    if config_id == 2:
        fv = list(field_vocab) if field_vocab is not None else [vs(6_250_000)] * len(_FIELDS8)
        assert len(fv) == len(_FIELDS8)
        feats = [FeatureDecl(n, i, int(fv[i]), 64) for i, n in enumerate(_FIELDS8)]
        w = Workload("grm_seq_lookup", 2, feats, batch or 512, 1.05, 40, "per_sample_uniform",
                     len_lo or 256, len_hi or 4096, steps=steps or 3)
        w.prepopulated = [f.vocab for f in feats]
        return w
    if config_id == 3:
        rng = np.random.Generator(np.random.Philox(key=SEED_BASE + 3))
        m = 32
        dims = rng.choice([16, 32, 64, 128], size=m)
        vocab = np.exp(rng.uniform(math.log(1e4), math.log(1e7), size=m)).astype(np.int64)
        owners = list(range(m)) + [int(t) for t in rng.choice(m, size=8, replace=False)]
        feats = [FeatureDecl(f"feat{j}", t, vs(int(vocab[t])), int(dims[t])) for j, t in enumerate(owners)]
        w = Workload("table_merging", 3, feats, batch or 1024, 1.1, 24, "per_field_uniform",
                     len_lo or 1, len_hi or 200, tag_bits=8, steps=steps or 6)
        return w
    if config_id == 4:
        feats = [FeatureDecl(f"f{i}", i, vs(400_000), 64) for i in range(4)]
        w = Workload("insert_delete_stress", 4, feats, batch or 512, 1.05, 40, "fixed",
                     len_lo or 1024, len_lo or 1024, fresh_frac=0.20, steps=steps or 1000,
                     ttl=200, min_freq=3, grace=20, evict_every=20, max_load_factor=0.85)
        return w
    if config_id == 5:
        feats = [FeatureDecl(f"f{i}", i, vs(100_000_000), 128, "bf16") for i in range(4)]
        w = Workload("large_bf16", 5, feats, batch or 2048, 1.0, 48, "fixed",
                     len_lo or 2048, len_lo or 2048, fresh_frac=0.05, steps=steps or 3)
        w.prepopulated = [f.vocab for f in feats]
        return w
    raise ValueError(f"unknown config {config_id}")


# --------------------------------------------------------------------------- #
# upstream gradients
# --------------------------------------------------------------------------- #
def normal_grads(seed: int, step: int, n: int, dim: int) -> np.ndarray:
    """N(0,1) float32 upstream gradients, row-major [n, dim]."""
    rng = np.random.Generator(np.random.Philox(key=(seed ^ 0xA5A5_0000) + step))
    return rng.standard_normal((n, dim), dtype=np.float32)


def small_int_grads(n: int, dim: int, seed: int, device: str = "cpu"):
    """Integer-valued gradients in [-8, 8] as a float32 torch tensor [n, dim].

    Sums of up to 2^20 such values are exact in fp32 in any order, so a
    segment reduction over them has exactly one correct fp32 answer.  The same
    integer formula runs on whichever device is asked for."""
    import torch

    i = torch.arange(n, dtype=torch.int64, device=device).unsqueeze(1)
    j = torch.arange(dim, dtype=torch.int64, device=device).unsqueeze(0)
    h = (i * 2654435761 + j * 40503 + (seed & 0xFFFF) * 97) & 0x7FFFFFFF
    h = (h ^ (h >> 13)) * 1274126177 & 0x7FFFFFFF
    return ((h >> 9) % 17 - 8).to(torch.float32)
