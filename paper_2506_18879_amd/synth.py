"""Seeded synthetic workloads shaped like the paper's LLaMA-3.1-8B long-context runs.

This module only *generates inputs* (codes, codebooks, queries, positions) and
converts storage formats; it holds none of the method's arithmetic, so both the
HIP path and the CPU oracle may be fed from it.  The paper evaluates on
LLaMA-3.1-8B-Instruct (Sec. 5.1) at 8K-128K context (Table "speedup"); those
weights, caches and trained codebooks are not available, so these stand in for
them with the same layer shapes.

Storage conventions
  * bf16 tensors are carried as ``uint16`` bit patterns (numpy has no bf16).
  * key/value codes: flat ``uint8``; sequence ``b`` holds ``[Hkv][L_b][M]``,
    sequences concatenated in batch order.
  * codebooks: ``[Hkv][M][K][d]``; a key codeword row is the sequence of first
    rows ``(x, y)`` of its d/2 RoPE-commuting blocks ``[[x, y], [-y, x]]``
    (Property 1, Eq. C_struct), so the free parameters are exactly the row.
  * paired key format (App. A.1): per token and KV head ``R`` pairs ``(a_r, b_r)``
    of 6-bit indices, packed little endian into ``ceil(12 R / 8)`` bytes with
    pair ``r`` at bits ``12 r .. 12 r + 11`` (``a`` low, ``b`` high); one tied
    table ``[Hkv][R][64][d]`` serves both indices of a level.
  * binary value format (Sec. 4.1): per token ONE record of ``Nc / 8`` bytes for all KV
    heads together (bit ``c`` = bit ``c % 8`` of byte ``c // 8``), sequence ``b`` holds
    ``[L_b][Nc / 8]``; one value codebook ``[Nc][Hkv * d]``.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

BASE_SEED = 250618879
ROPE_BASE = 500000.0


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even) and return the uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns exactly to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Workload:
    name: str
    B: int
    Hq: int
    Hkv: int
    d: int
    Mk: int
    Mv: int
    K: int
    dtype: str  # "f32" or "bf16": storage type of q and of both codebooks
    rope_base: float
    q: np.ndarray  # [B][Hq][d] float32, or uint16 bf16 bits
    key_codes: np.ndarray  # uint8 flat
    val_codes: np.ndarray  # uint8 flat
    key_codebooks: np.ndarray  # [Hkv][Mk][K][d]
    val_codebooks: np.ndarray  # [Hkv][Mv][K][d]
    cu_seqlens: np.ndarray  # int32 [B+1]
    q_pos: np.ndarray  # int32 [B]
    key_pos: Optional[np.ndarray] = None  # int32 [T] or None (token i at position i)
    seed: int = 0
    code_dist: str = "uniform"
    extras: dict = field(default_factory=dict)
    key_format: str = "indexed"  # "indexed": Mk uint8 indices per token; "paired": key_levels packed 12-bit pairs
    key_levels: int = 0          # R of the paired format (then key_codebooks is the tied table [Hkv][R][64][d])
    val_format: str = "indexed"  # "indexed": Mv uint8 indices per token and KV head; "binary": val_bits bits per token
    val_bits: int = 0            # N_c of the binary format (then val_codebooks is [Nc][Hkv * d] and Mv is unused)

    @property
    def total_tokens(self) -> int:
        return int(self.cu_seqlens[-1])

    @property
    def max_seqlen(self) -> int:
        return int(np.max(np.diff(self.cu_seqlens)))

    def as_f64(self, name: str) -> np.ndarray:
        """Exact fp64 widening of q / key_codebooks / val_codebooks (for the oracle)."""
        a = getattr(self, name)
        if a.dtype == np.uint16:
            a = bf16_bits_to_f32(a)
        return a.astype(np.float64)

    def seq_codes(self, which: str, b: int) -> np.ndarray:
        """View of one sequence's codes as [Hkv][L_b][M] (index-form keys or values only)."""
        M = self.Mk if which == "key" else self.Mv
        flat = self.key_codes if which == "key" else self.val_codes
        o, e = int(self.cu_seqlens[b]), int(self.cu_seqlens[b + 1])
        return flat[o * self.Hkv * M:e * self.Hkv * M].reshape(self.Hkv, e - o, M)


def _zipf_codes(rng: np.random.Generator, Hkv: int, L: int, M: int, K: int, s: float) -> np.ndarray:
    """Codes with P(rank r) proportional to (r+1)^-s, r < K; rank -> codeword id by an
    independent random permutation per (KV head, codebook) so hot codewords differ."""
    p = (np.arange(1, K + 1, dtype=np.float64)) ** (-s)
    cdf = np.cumsum(p / p.sum())
    cdf[-1] = 1.0
    out = np.empty((Hkv, L, M), dtype=np.uint8)
    for g in range(Hkv):
        ranks = np.searchsorted(cdf, rng.random((L, M)), side="right").astype(np.int64)
        np.clip(ranks, 0, K - 1, out=ranks)
        perms = np.stack([rng.permutation(K) for _ in range(M)], axis=0)  # [M][K]
        out[g] = perms[np.arange(M)[None, :], ranks].astype(np.uint8)
    return out


def make_workload(name: str, *, B: int, Hq: int, Hkv: int, seqlens, Mk: int, Mv: int, dtype: str,
                  seed: int, d: int = 128, K: int = 256, code_dist: str = "uniform",
                  zipf_s: float = 1.1, rope_base: float = ROPE_BASE) -> Workload:
    """Generate every tensor of one workload from a single seed."""
    assert dtype in ("f32", "bf16") and Hq % Hkv == 0 and d % 2 == 0
    rng = np.random.Generator(np.random.PCG64(seed))
    seqlens = np.asarray(seqlens, dtype=np.int64)
    assert seqlens.shape == (B,) and np.all(seqlens >= 0) and seqlens.max() >= 1  # a sequence may be empty
    cu = np.zeros(B + 1, dtype=np.int32)
    cu[1:] = np.cumsum(seqlens)

    def codebook(M):
        # block parameters (x, y) ~ N(0, M^-1/2): decoded coordinates have unit variance
        params = rng.standard_normal((Hkv, M, K, d // 2, 2), dtype=np.float32) * np.float32(M ** -0.5)
        cb = params.reshape(Hkv, M, K, d)
        return f32_to_bf16_bits(cb) if dtype == "bf16" else cb

    key_cb = codebook(Mk)
    val_cb = codebook(Mv)
    q = rng.standard_normal((B, Hq, d), dtype=np.float32)
    if dtype == "bf16":
        q = f32_to_bf16_bits(q)

    def codes(M):
        parts = []
        for L in seqlens:
            if code_dist == "uniform":
                parts.append(rng.integers(0, K, size=(Hkv, int(L), M), dtype=np.uint8 if K == 256 else np.int64)
                             .astype(np.uint8).reshape(-1))
            elif code_dist == "zipf":
                parts.append(_zipf_codes(rng, Hkv, int(L), M, K, zipf_s).reshape(-1))
            else:
                raise ValueError(code_dist)
        return np.concatenate(parts)

    key_codes = codes(Mk)
    val_codes = codes(Mv)
    q_pos = np.maximum(seqlens - 1, 0).astype(np.int32)  # the query's own key is the last cached row
    return Workload(name=name, B=B, Hq=Hq, Hkv=Hkv, d=d, Mk=Mk, Mv=Mv, K=K, dtype=dtype, rope_base=rope_base,
                    q=q, key_codes=key_codes, val_codes=val_codes, key_codebooks=key_cb, val_codebooks=val_cb,
                    cu_seqlens=cu, q_pos=q_pos, key_pos=None, seed=seed, code_dist=code_dist)


def pack_key_pairs(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """[..., R] 6-bit indices a, b -> [..., ceil(12 R / 8)] bytes (pair r at bits 12 r .. 12 r + 11, a low)."""
    a = np.asarray(a, dtype=np.uint64)
    b = np.asarray(b, dtype=np.uint64)
    assert a.shape == b.shape and a.max(initial=0) < 64 and b.max(initial=0) < 64
    R = a.shape[-1]
    pb = (12 * R + 7) // 8
    out = np.zeros(a.shape[:-1] + (pb,), dtype=np.uint8)
    for r in range(R):
        pair = a[..., r] | (b[..., r] << np.uint64(6))   # 12 bits
        bit = 12 * r
        for k in range(3):                                # a pair touches at most 2 bytes, 3 covers any shift
            byte = bit // 8 + k
            if byte >= pb:
                break
            shift = 8 * k - bit % 8
            chunk = (pair >> np.uint64(shift)) if shift >= 0 else (pair << np.uint64(-shift))
            out[..., byte] |= (chunk & np.uint64(0xFF)).astype(np.uint8)
    return out


def make_pair_workload(name: str, *, B: int, Hq: int, Hkv: int, seqlens, R: int, Mv: int, seed: int,
                       d: int = 128, code_dist: str = "uniform", zipf_s: float = 1.1,
                       rope_base: float = ROPE_BASE) -> Workload:
    """A workload whose keys are in the paper's paired format: N_c' = 64 centres per level, R levels
    (R = 11: 1.03 bit per scalar, R = 21: 1.97), bf16 storage; values as in make_workload."""
    base = make_workload(name, B=B, Hq=Hq, Hkv=Hkv, seqlens=seqlens, Mk=16, Mv=Mv, dtype="bf16", seed=seed, d=d,
                         code_dist=code_dist, zipf_s=zipf_s, rope_base=rope_base)
    rng = np.random.Generator(np.random.PCG64(seed ^ 0xA11CE))
    # block parameters ~ N(0, (2R)^-1/2): a decoded coordinate is a sum of 2R of them
    table = rng.standard_normal((Hkv, R, 64, d), dtype=np.float32) * np.float32((2 * R) ** -0.5)
    parts = []
    for L in np.diff(base.cu_seqlens):
        if code_dist == "zipf":
            ab = _zipf_codes(rng, Hkv, int(L), 2 * R, 64, zipf_s)
        else:
            ab = rng.integers(0, 64, size=(Hkv, int(L), 2 * R)).astype(np.uint8)
        parts.append(pack_key_pairs(ab[..., 0::2], ab[..., 1::2]).reshape(-1))
    base.key_codes = np.concatenate(parts)
    base.key_codebooks = f32_to_bf16_bits(table)
    base.key_format, base.key_levels, base.Mk = "paired", R, 2 * R
    return base


def with_binary_values(base: Workload, Nc: int, *, density: float = 0.5, seed: Optional[int] = None) -> Workload:
    """Replace base's values by the paper's binary value code: every token stores Nc bits for all KV heads
    together, each bit set with probability `density` (the trained encoder's statistics are not published), and
    one codebook [Nc][Hkv * d] with entries ~ N(0, (density Nc)^-1/2), so that a decoded coordinate has about unit
    variance."""
    assert Nc % 8 == 0 and 0.0 <= density <= 1.0
    rng = np.random.Generator(np.random.PCG64((base.seed if seed is None else seed) ^ 0xB175))
    T = base.total_tokens
    rows = []
    for lo in range(0, T, 1 << 16):  # in pieces: the unpacked bits of a long context would not fit comfortably
        n = min(1 << 16, T - lo)
        rows.append(np.packbits(rng.random((n, Nc)) < density, axis=1, bitorder="little"))
    base.val_codes = np.concatenate(rows).reshape(-1) if rows else np.zeros(0, np.uint8)
    cb = rng.standard_normal((Nc, base.Hkv * base.d), dtype=np.float32) * np.float32(max(density * Nc, 1.0) ** -0.5)
    base.val_codebooks = f32_to_bf16_bits(cb) if base.dtype == "bf16" else cb
    base.val_format, base.val_bits, base.Mv = "binary", Nc, 0
    base.name += f"_vbits{Nc}"
    return base


def config(idx: int, *, seed: Optional[int] = None, max_len: Optional[int] = None) -> Workload:
    """The five benchmark configurations (1-based ``idx``).

    ``max_len`` shrinks every context length to at most that many tokens (ragged
    lengths are scaled down proportionally) so parity tests can run the same
    shapes at sizes the oracle finishes quickly; the full sizes are the default.
    """
    s = BASE_SEED + (idx - 1) if seed is None else seed

    def cap(L):
        return int(L) if max_len is None else int(min(L, max_len))

    if idx == 1:  # single head, fp32, 2-bit
        return make_workload("c1_1head_f32_L4096_2bit", B=1, Hq=1, Hkv=1, seqlens=[cap(4096)], Mk=32, Mv=32,
                             dtype="f32", seed=s)
    if idx == 2:  # 8B-shaped layer, 32K, 2-bit
        return make_workload("c2_8b_L32768_2bit", B=1, Hq=32, Hkv=8, seqlens=[cap(32768)], Mk=32, Mv=32,
                             dtype="bf16", seed=s)
    if idx == 3:  # 8B-shaped layer, 128K, 1-bit, skewed code usage
        return make_workload("c3_8b_L131072_1bit_zipf", B=1, Hq=32, Hkv=8, seqlens=[cap(131072)], Mk=16, Mv=16,
                             dtype="bf16", seed=s, code_dist="zipf")
    if idx == 4:  # batch of 8 ragged sequences, 2-bit
        lens = np.random.Generator(np.random.PCG64(s ^ 0x5EED)).integers(8192, 65536, size=8, endpoint=True)
        if max_len is not None:
            lens = np.maximum(1, (lens.astype(np.float64) * (max_len / 65536.0)).astype(np.int64))
        return make_workload("c4_8b_B8_ragged_2bit", B=8, Hq=32, Hkv=8, seqlens=lens, Mk=32, Mv=32,
                             dtype="bf16", seed=s)
    if idx == 5:  # 70B-shaped layer, batch 4, 128K, 2-bit keys / 1-bit values
        return make_workload("c5_70b_B4_L131072_k2v1", B=4, Hq=64, Hkv=8, seqlens=[cap(131072)] * 4, Mk=32, Mv=16,
                             dtype="bf16", seed=s)
    if idx in (6, 7):  # 8B-shaped layer, 128K, keys in the paper's own paired format: 1-bit (R = 11) / 2-bit (R = 21)
        R = 11 if idx == 6 else 21
        return make_pair_workload(f"c{idx}_8b_L131072_paired_R{R}", B=1, Hq=32, Hkv=8, seqlens=[cap(131072)], R=R,
                                  Mv=16 if idx == 6 else 32, seed=s)
    if idx in (8, 9):  # 8B-shaped layer, 128K, values in the paper's binary form: N_c = 1024 (1 bit) / 2048 (2 bit)
        base = make_workload(f"c{idx}_8b_L131072", B=1, Hq=32, Hkv=8, seqlens=[cap(131072)], Mk=16 if idx == 8 else 32,
                             Mv=16, dtype="bf16", seed=s)
        return with_binary_values(base, 1024 if idx == 8 else 2048)
    if idx in (10, 11):  # the paper's own formats on both sides (App., Table codebook_conf): 1 bit = (R 11, N_c 1024), 2 bit = (21, 2048)
        R, Nc = (11, 1024) if idx == 10 else (21, 2048)
        base = make_pair_workload(f"c{idx}_8b_L131072_paired_R{R}", B=1, Hq=32, Hkv=8, seqlens=[cap(131072)], R=R, Mv=16, seed=s)
        return with_binary_values(base, Nc)
    raise ValueError(f"config index {idx} not in 1..11")
