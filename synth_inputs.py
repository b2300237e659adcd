"""Seeded synthetic inputs for the Adamas decode path.

This module only draws random numbers and lays them out as a KV cache; it holds none of
the method's arithmetic (no transform, no codes, no distances, no attention), so both the
CPU oracle's tests and the GPU library's tests may use it.

The inputs stand in for the KV caches of the paper's 32K / 100K LongChat and Yarn-Llama
workloads (Section 4.1), which need model weights and datasets that are not available:
keys and values are i.i.d. N(0,1) in bf16 with four fixed "outlier" channels per KV head
scaled by 8 (the large-magnitude feature channels that motivate the Hadamard transform,
Section 3.1), and queries are noisy copies of "needle" key rows planted at seeded
positions, the synthetic counterpart of the passkey retrieval test (Table 1).

bf16 data is carried as uint16 bit patterns in numpy arrays.
"""

from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

D = 128
BASE_SEED = 20251018
OUTLIER_CHANNELS = 4
OUTLIER_SCALE = 8.0
NEEDLE_SIGMA = 0.1
FLUSH_BELOW = 2.0 ** -24          # magnitudes below this become +0 (keeps sums exact in fp64)
DEFAULT_THRESHOLDS = (-1.0, 0.0, 1.0)   # on the orthonormal transform scale
SEQ_GAP_ROWS = 64                 # unused pool rows between packed sequences


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns, round-to-nearest-even, tiny magnitudes flushed to +0."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    x = np.where(np.abs(x) < np.float32(FLUSH_BELOW), np.float32(0.0), x)
    u = x.view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class DecodeCase:
    """One decode step's inputs.  Pools hold the cache BEFORE the step's append."""
    name: str
    B: int
    Hq: int
    Hkv: int
    pool_tokens: int
    budgets: List[int]
    q: np.ndarray                 # uint16 [B, Hq, 128]
    K: np.ndarray                 # uint16 [Hkv, pool_tokens, 128]
    V: np.ndarray                 # uint16 [Hkv, pool_tokens, 128]
    seq_start: np.ndarray         # int64 [B]
    seq_len: np.ndarray           # int32 [B], lengths AFTER the append if k_new is set
    k_new: Optional[np.ndarray] = None   # uint16 [B, Hkv, 128]
    v_new: Optional[np.ndarray] = None
    needles: List[List[List[int]]] = field(default_factory=list)  # [B][Hq] -> token positions
    thresholds: Sequence[float] = DEFAULT_THRESHOLDS

    @property
    def group(self) -> int:
        return self.Hq // self.Hkv

    @property
    def max_seq_len(self) -> int:
        return int(self.seq_len.max())


def _rows(rng: np.random.Generator, n: int, scale: np.ndarray) -> np.ndarray:
    """n rows of N(0,1) float32 with the per-channel outlier scale applied."""
    return rng.standard_normal((n, scale.shape[0]), dtype=np.float32) * scale


def make_case(name: str, seed: int, B: int, Hq: int, Hkv: int, seq_len: Sequence[int],
              budgets: Sequence[int], needle_positions, append: bool = False,
              gap: int = SEQ_GAP_ROWS, head_dim: int = D) -> DecodeCase:
    """Builds a ragged KV cache with planted needles.

    needle_positions(b, L, kv_head, rng) -> int array [G, n_needles] of distinct token
    positions in [0, L_cached) for the G query heads of that KV head's group.
    With append=True the cache holds seq_len[b]-1 rows and k_new/v_new carry one more.
    head_dim: 128 (the paper's models) unless a test of other head dimensions says otherwise.
    """
    assert Hq % Hkv == 0
    D = head_dim      # shadows the module constant inside this function
    G = Hq // Hkv
    rng = np.random.default_rng(seed)
    seq_len = np.asarray(seq_len, dtype=np.int32)
    assert seq_len.shape == (B,)
    starts = np.zeros(B, dtype=np.int64)
    pos = 0
    for b in range(B):
        starts[b] = pos
        pos += int(seq_len[b]) + gap
    pool_tokens = max(pos - gap, 1) if B else 1
    K = np.zeros((Hkv, pool_tokens, D), dtype=np.uint16)
    V = np.zeros((Hkv, pool_tokens, D), dtype=np.uint16)
    q = np.zeros((B, Hq, D), dtype=np.uint16)
    k_new = np.zeros((B, Hkv, D), dtype=np.uint16) if append else None
    v_new = np.zeros((B, Hkv, D), dtype=np.uint16) if append else None
    needles: List[List[List[int]]] = [[[] for _ in range(Hq)] for _ in range(B)]

    for h in range(Hkv):
        scale_k = np.ones(D, dtype=np.float32)
        scale_k[rng.choice(D, OUTLIER_CHANNELS, replace=False)] = OUTLIER_SCALE
        scale_v = np.ones(D, dtype=np.float32)
        scale_v[rng.choice(D, OUTLIER_CHANNELS, replace=False)] = OUTLIER_SCALE
        for b in range(B):
            L = int(seq_len[b])
            cached = L - 1 if append else L
            s = int(starts[b])
            if cached > 0:
                K[h, s:s + cached] = f32_to_bf16_bits(_rows(rng, cached, scale_k))
                V[h, s:s + cached] = f32_to_bf16_bits(_rows(rng, cached, scale_v))
            if append and L > 0:
                k_new[b, h] = f32_to_bf16_bits(_rows(rng, 1, scale_k))[0]
                v_new[b, h] = f32_to_bf16_bits(_rows(rng, 1, scale_v))[0]
            base = []
            for g in range(G):
                hq = h * G + g
                u = _rows(rng, 1, scale_k)[0]
                base.append(u)
                q[b, hq] = f32_to_bf16_bits(
                    u + NEEDLE_SIGMA * rng.standard_normal(D, dtype=np.float32))
            if cached > 0:
                where = np.asarray(needle_positions(b, cached, h, rng), dtype=np.int64)
                assert where.shape[0] == G
                flat = where.reshape(-1)
                assert len(set(flat.tolist())) == flat.size, "needle positions must be distinct"
                assert flat.size == 0 or (flat.min() >= 0 and flat.max() < cached)
                for g in range(G):
                    hq = h * G + g
                    for p in where[g]:
                        row = base[g] + NEEDLE_SIGMA * rng.standard_normal(D, dtype=np.float32)
                        K[h, s + int(p)] = f32_to_bf16_bits(row)
                        needles[b][hq].append(int(p))
    return DecodeCase(name=name, B=B, Hq=Hq, Hkv=Hkv, pool_tokens=pool_tokens,
                      budgets=list(budgets), q=q, K=K, V=V, seq_start=starts, seq_len=seq_len,
                      k_new=k_new, v_new=v_new, needles=needles)


# --------------------------------------------------------------------------- named configs

def _distinct(rng: np.random.Generator, L: int, G: int, n: int) -> np.ndarray:
    return rng.choice(L, size=(G, n), replace=False)


def config_seed(config: int, layer: int = 0) -> int:
    return BASE_SEED + 1000 * config + layer


def tiny_single_head(layer: int = 0, L: int = 1024, k: int = 64) -> DecodeCase:
    """Config 0: batch 1, one head, context 1024, budget 64, one needle."""
    return make_case("cfg0_tiny", config_seed(0, layer), 1, 1, 1, [L], [k],
                     lambda b, Lc, h, rng: _distinct(rng, Lc, 1, 1))


def mha_32k(layer: int = 0, L: int = 32768, heads: int = 32,
            budgets: Sequence[int] = (64, 128, 256)) -> DecodeCase:
    """Config 1: Llama-style MHA layer, 32 query = 32 KV heads, context 32768, 8 needles/head."""
    return make_case("cfg1_mha32k", config_seed(1, layer), 1, heads, heads, [L], budgets,
                     lambda b, Lc, h, rng: _distinct(rng, Lc, 1, 8))


def gqa_32k(layer: int = 0, L: int = 32768, Hq: int = 32, Hkv: int = 8, k: int = 128) -> DecodeCase:
    """Config 2: GQA layer, 32 query heads over 8 KV heads, one needle per query head."""
    G = Hq // Hkv
    return make_case("cfg2_gqa32k", config_seed(2, layer), 1, Hq, Hkv, [L], [k],
                     lambda b, Lc, h, rng: _distinct(rng, Lc, G, 1))


def long_128k_append(layer: int = 0, L: int = 131072, Hq: int = 32, Hkv: int = 8,
                     budgets: Sequence[int] = (256, 1024)) -> DecodeCase:
    """Config 3: context 131072 after appending one token; needles at depths 10/50/90 %."""
    G = Hq // Hkv

    def depths(b, Lc, h, rng):
        rows = [int(0.1 * Lc), int(0.5 * Lc), int(0.9 * Lc)]
        return np.array([[r + g for r in rows] for g in range(G)])

    return make_case("cfg3_long128k", config_seed(3, layer), 1, Hq, Hkv, [L], budgets, depths,
                     append=True)


def batched_ragged(layer: int = 0, B: int = 16, lo: int = 8192, hi: int = 32768, Hq: int = 32,
                   Hkv: int = 8, k: int = 128) -> DecodeCase:
    """Config 4: 16 sequences, lengths uniform in [lo, hi], packed back to back with gaps."""
    G = Hq // Hkv
    lens = np.random.default_rng(config_seed(4, layer) + 500).integers(lo, hi + 1, size=B)
    return make_case("cfg4_batched", config_seed(4, layer), B, Hq, Hkv, lens, [k],
                     lambda b, Lc, h, rng: _distinct(rng, Lc, G, 1))


@dataclass
class PagedCase:
    """A DecodeCase whose cache rows were scattered over fixed-size pages.  Token t of sequence b
    lives in pool row page_table[b, t // page_tokens] * page_tokens + t % page_tokens of every
    KV head; rows of pages that no sequence owns hold other (random) data."""
    case: DecodeCase              # the contiguous original (its pools are not used on the device)
    page_tokens: int
    pool_tokens: int              # n_pages * page_tokens
    K: np.ndarray                 # uint16 [Hkv, pool_tokens, 128], BEFORE the step's append
    V: np.ndarray
    page_table: np.ndarray        # int32 [B, max_pages]; -1 where a sequence has no page


def paginate(case: DecodeCase, page_tokens: int, seed: int, spare_pages: int = 3) -> PagedCase:
    """Scatters the sequences of `case` over randomly chosen pages (a pure re-layout: no value
    changes).  Each sequence gets the pages its length AFTER the append needs."""
    rng = np.random.default_rng(seed)
    need = [(int(L) + page_tokens - 1) // page_tokens for L in case.seq_len]
    n_pages = sum(need) + spare_pages
    max_pages = max(1, max(need))
    order = rng.permutation(n_pages)
    pool = n_pages * page_tokens
    d = case.K.shape[-1]
    K = f32_to_bf16_bits(rng.standard_normal((case.Hkv, pool, d), dtype=np.float32))
    V = f32_to_bf16_bits(rng.standard_normal((case.Hkv, pool, d), dtype=np.float32))
    table = np.full((case.B, max_pages), -1, dtype=np.int32)
    at = 0
    for b in range(case.B):
        s, L = int(case.seq_start[b]), int(case.seq_len[b])
        for pg in range(need[b]):
            phys = int(order[at])
            at += 1
            table[b, pg] = phys
            n = min(page_tokens, L - pg * page_tokens)
            src = slice(s + pg * page_tokens, s + pg * page_tokens + n)
            dst = slice(phys * page_tokens, phys * page_tokens + n)
            K[:, dst] = case.K[:, src]
            V[:, dst] = case.V[:, src]
    return PagedCase(case, page_tokens, pool, K, V, table)
