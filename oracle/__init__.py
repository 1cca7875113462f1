"""CPU oracle for CommVQ decode attention -- TEST INFRASTRUCTURE ONLY.

Thin ctypes binding over ``commvq_oracle.c`` (plain C, fp64), which writes out
the paper's naive decode-then-attend definition (Sec. 3.1, Eq. v1_formula).
Only the tests, the smoke check and the benchmark's ``cpu_baseline`` leg may
import this package; the product path (``paper_2506_18879_amd``) never does and
shares no code with it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "commvq_oracle.c")
_LIB = os.path.join(_HERE, "libcommvq_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no fast-math) into this directory."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-pthread", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        lib.commvq_oracle_rope.argtypes = [dp, ctypes.c_int, ctypes.c_double, ctypes.c_double]
        lib.commvq_oracle_rope.restype = None
        lib.commvq_oracle_decode.argtypes = [ctypes.c_void_p, dp, ctypes.c_int, ctypes.c_int, ctypes.c_int, dp]
        lib.commvq_oracle_decode.restype = None
        lib.commvq_oracle_decode_attn.argtypes = (
            [ctypes.c_int] * 7 + [ctypes.c_void_p] * 8 + [ctypes.c_double] * 2 + [ctypes.c_void_p] * 4 + [ctypes.c_int]
        )
        lib.commvq_oracle_decode_attn.restype = ctypes.c_int
        lib.commvq_oracle_encode_keys.argtypes = [ctypes.c_int] * 5 + [ctypes.c_void_p] * 6
        lib.commvq_oracle_encode_keys.restype = ctypes.c_int
        _lib = lib
    return _lib


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def rope(u, pos, rope_base):
    """Return u R_pos (Sec. 3.2, Eq. rope_ri) for a 1-D vector of even length."""
    u = _f64(u).copy()
    _load().commvq_oracle_rope(u.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), u.size, float(pos), float(rope_base))
    return u


def decode(codes, codebooks):
    """Return s C: the sum of the selected codeword rows (Eq. vanilla_decode).

    codes: uint8[M]; codebooks: [M][K][d].
    """
    cb = _f64(codebooks)
    M, K, d = cb.shape
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    assert codes.shape == (M,)
    out = np.empty(d, dtype=np.float64)
    dp = ctypes.POINTER(ctypes.c_double)
    _load().commvq_oracle_decode(_ptr(codes), cb.ctypes.data_as(dp), M, K, d, out.ctypes.data_as(dp))
    return out


def decode_attn(q, key_codes, val_codes, key_codebooks, val_codebooks, cu_seqlens, q_pos,
                key_pos=None, rope_base=500000.0, scale=None, unit_mask=None, n_threads=1,
                return_intermediates=False):
    """Naive decode-then-attend attention in fp64 (Sec. 3.1, Eq. v1_formula).

    q [B][Hq][d]; key_codes/val_codes flat uint8, per sequence [Hkv][L_b][M];
    codebooks [Hkv][M][K][d]; cu_seqlens int32[B+1]; q_pos int32[B];
    key_pos int32[T] or None (token i at position i).  Float inputs of any
    width are widened exactly to fp64.  unit_mask (bool [B][Hkv]) restricts the
    work to some (sequence, KV head) units; other output rows are NaN.
    Returns out [B][Hq][d], or (out, scores, weights) with the ragged
    [T*Hq] intermediates (sequence b, head h, token i at cu[b]*Hq + h*L_b + i).
    """
    q = _f64(q)
    kcb, vcb = _f64(key_codebooks), _f64(val_codebooks)
    B, Hq, d = q.shape
    Hkv, Mk, K, d2 = kcb.shape
    Mv = vcb.shape[1]
    assert d2 == d and vcb.shape == (Hkv, Mv, K, d)
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    qp = np.ascontiguousarray(q_pos, dtype=np.int32)
    assert cu.shape == (B + 1,) and qp.shape == (B,) and cu[0] == 0
    T = int(cu[-1])
    kc = np.ascontiguousarray(key_codes, dtype=np.uint8).reshape(-1)
    vc = np.ascontiguousarray(val_codes, dtype=np.uint8).reshape(-1)
    assert kc.size == T * Hkv * Mk and vc.size == T * Hkv * Mv
    kp = None if key_pos is None else np.ascontiguousarray(key_pos, dtype=np.int32)
    assert kp is None or kp.shape == (T,)
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    out = np.full((B, Hq, d), np.nan, dtype=np.float64)
    scores = np.full(T * Hq, np.nan, dtype=np.float64) if return_intermediates else None
    weights = np.full(T * Hq, np.nan, dtype=np.float64) if return_intermediates else None
    um = None if unit_mask is None else np.ascontiguousarray(unit_mask, dtype=np.uint8).reshape(B * Hkv)
    rc = _load().commvq_oracle_decode_attn(
        B, Hq, Hkv, d, Mk, Mv, K, _ptr(q), _ptr(kc), _ptr(vc), _ptr(kcb), _ptr(vcb), _ptr(cu), _ptr(qp), _ptr(kp),
        float(rope_base), float(scale), _ptr(out), _ptr(scores), _ptr(weights), _ptr(um), int(n_threads))
    if rc != 0:
        raise ValueError(f"commvq_oracle_decode_attn failed with code {rc}")
    if return_intermediates:
        return out, scores, weights
    return out


def unpack_key_pairs(records, R):
    """Paired key format (App. A.1): records uint8 [..., ceil(12 R / 8)] -> (a, b), each uint8 [..., R].

    Pair r of a record is its bits 12 r .. 12 r + 11 (little endian); a_r is the low 6 bits, b_r the high 6.
    """
    rec = np.ascontiguousarray(records, dtype=np.uint8)
    pb = (12 * R + 7) // 8
    assert rec.shape[-1] == pb
    bits = np.unpackbits(rec, axis=-1, bitorder="little")[..., :12 * R].reshape(rec.shape[:-1] + (R, 12))
    w = (1 << np.arange(6)).astype(np.uint8)
    a = (bits[..., :6] * w).sum(axis=-1).astype(np.uint8)
    b = (bits[..., 6:] * w).sum(axis=-1).astype(np.uint8)
    return a, b


def tied_table_as_codebooks(table, K=None):
    """Tied pair table [Hkv][R][N][d] -> index-form codebooks [Hkv][2R][K][d] (Eq. def_center).

    Level r decodes to C[r][a] + (second rows of the blocks of C[r][b]); a block [[x, y], [-y, x]] has second
    row (-y, x).  So codebook 2r holds the rows themselves and codebook 2r + 1 the same rows with every
    (x, y) replaced by (-y, x).  Rows N .. K-1 (never selected) are zero.
    """
    t = _f64(table)
    Hkv, R, N, d = t.shape
    K = N if K is None else K
    out = np.zeros((Hkv, 2 * R, K, d), dtype=np.float64)
    out[:, 0::2, :N, :] = t
    out[:, 1::2, :N, 0::2] = -t[..., 1::2]
    out[:, 1::2, :N, 1::2] = t[..., 0::2]
    return out


def paired_as_indexed(records, R, cu_seqlens, Hkv):
    """Flat packed records (per sequence [Hkv][L_b][PB]) -> flat index-form codes (per sequence [Hkv][L_b][2R]),
    index 2r = a_r, index 2r + 1 = b_r, matching tied_table_as_codebooks."""
    pb = (12 * R + 7) // 8
    rec = np.ascontiguousarray(records, dtype=np.uint8).reshape(-1, pb)
    a, b = unpack_key_pairs(rec, R)
    out = np.empty((rec.shape[0], 2 * R), dtype=np.uint8)
    out[:, 0::2], out[:, 1::2] = a, b
    return out.reshape(-1)


def encode_keys(keys, codebooks, paired=False, given=None):
    """Residual nearest-centre encoding of key vectors of ONE KV head (Sec. 4.2 E step, level by level).

    keys [n][d]; codebooks [levels][K][d] (index form) or the tied table [R][K][d] (paired, centres
    C[r][a] + second rows of C[r][b], Eq. def_center).  Returns (codes, best, taken): codes uint8
    [n][levels] (or [n][levels][2] = (a, b) when paired) = the nearest centre at every level; best[n][levels]
    its squared distance to the residual searched; taken[n][levels] the squared residual norm after the
    level.  With `given` (same shape as codes) the residual is updated with those codes instead, so that
    another encoder's choices can be judged level by level.
    """
    keys = _f64(keys)
    cb = _f64(codebooks)
    n, d = keys.shape
    levels, K, d2 = cb.shape
    assert d2 == d
    per = 2 if paired else 1
    codes = np.zeros((n, levels, per), dtype=np.uint8)
    best = np.zeros((n, levels), dtype=np.float64)
    taken = np.zeros((n, levels), dtype=np.float64)
    g = None
    if given is not None:
        g = np.ascontiguousarray(given, dtype=np.uint8).reshape(n, levels, per)
    rc = _load().commvq_oracle_encode_keys(n, d, levels, K, 1 if paired else 0, _ptr(keys), _ptr(cb), _ptr(g),
                                           _ptr(codes), _ptr(best), _ptr(taken))
    if rc != 0:
        raise ValueError(f"commvq_oracle_encode_keys failed with code {rc}")
    return (codes if paired else codes[:, :, 0]), best, taken
