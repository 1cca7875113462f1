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
        lib.commvq_oracle_decode_attn_bits.argtypes = lib.commvq_oracle_decode_attn.argtypes
        lib.commvq_oracle_decode_attn_bits.restype = ctypes.c_int
        lib.commvq_oracle_decode_bits.argtypes = [ctypes.c_void_p, dp] + [ctypes.c_int] * 4 + [dp]
        lib.commvq_oracle_decode_bits.restype = None
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


def decode_bits(bits, codebook, first=0, n=None):
    """Return columns first .. first + n - 1 of s C for a binary code s (Sec. 4.1, Eq. vanilla_decode).

    bits: uint8[Nc / 8], bit c of the code = bit c % 8 of byte c / 8; codebook: [Nc][width].
    """
    cb = _f64(codebook)
    Nc, width = cb.shape
    n = width - first if n is None else n
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    assert Nc % 8 == 0 and bits.shape == (Nc // 8,) and 0 <= first and first + n <= width
    out = np.empty(n, dtype=np.float64)
    dp = ctypes.POINTER(ctypes.c_double)
    _load().commvq_oracle_decode_bits(_ptr(bits), cb.ctypes.data_as(dp), Nc, width, int(first), int(n), out.ctypes.data_as(dp))
    return out


def decode_attn_binary_values(q, key_codes, val_bits, key_codebooks, val_codebook, cu_seqlens, q_pos,
                              key_pos=None, rope_base=500000.0, scale=None, unit_mask=None, n_threads=1,
                              return_intermediates=False):
    """decode_attn with the values in the paper's own binary form (Sec. 4.1; Eq. decode_v, Eq. v1_formula).

    val_bits flat uint8, per sequence [L_b][Nc / 8]: one record per token for all KV heads together;
    val_codebook [Nc][Hkv * d]: the token's whole value vector (the KV heads' values side by side) is the sum of
    the rows whose bit is set, and query head h attends over columns g d .. g d + d - 1 of it, g = h / (Hq / Hkv).
    Everything else as decode_attn.
    """
    q = _f64(q)
    kcb, vcb = _f64(key_codebooks), _f64(val_codebook)
    B, Hq, d = q.shape
    Hkv, Mk, K, d2 = kcb.shape
    Nc = vcb.shape[0]
    assert d2 == d and vcb.shape == (Nc, Hkv * d) and Nc % 8 == 0
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    qp = np.ascontiguousarray(q_pos, dtype=np.int32)
    assert cu.shape == (B + 1,) and qp.shape == (B,) and cu[0] == 0
    T = int(cu[-1])
    kc = np.ascontiguousarray(key_codes, dtype=np.uint8).reshape(-1)
    vb = np.ascontiguousarray(val_bits, dtype=np.uint8).reshape(-1)
    assert kc.size == T * Hkv * Mk and vb.size == T * (Nc // 8)
    kp = None if key_pos is None else np.ascontiguousarray(key_pos, dtype=np.int32)
    assert kp is None or kp.shape == (T,)
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    out = np.full((B, Hq, d), np.nan, dtype=np.float64)
    scores = np.full(T * Hq, np.nan, dtype=np.float64) if return_intermediates else None
    weights = np.full(T * Hq, np.nan, dtype=np.float64) if return_intermediates else None
    um = None if unit_mask is None else np.ascontiguousarray(unit_mask, dtype=np.uint8).reshape(B * Hkv)
    rc = _load().commvq_oracle_decode_attn_bits(
        B, Hq, Hkv, d, Mk, Nc, K, _ptr(q), _ptr(kc), _ptr(vb), _ptr(kcb), _ptr(vcb), _ptr(cu), _ptr(qp), _ptr(kp),
        float(rope_base), float(scale), _ptr(out), _ptr(scores), _ptr(weights), _ptr(um), int(n_threads))
    if rc != 0:
        raise ValueError(f"commvq_oracle_decode_attn_bits failed with code {rc}")
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
    rec = np.ascontiguousarray(records, dtype=np.uint8).reshape(-1)
    assert rec.size == int(np.asarray(cu_seqlens)[-1]) * Hkv * pb, "records do not match cu_seqlens x Hkv x record bytes"
    rec = rec.reshape(-1, pb)
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


def em_centres(phi):
    """All N_c'^2 clustering centres of one 2-D sub-space (Eq. def_center): phi [Nc][2] = (x_l, y_l);
    centre (a, b) = (x_a - y_b, y_a + x_b), returned as [Nc*Nc][2] with index a * Nc + b."""
    phi = _f64(phi)
    x, y = phi[:, 0], phi[:, 1]
    cx = x[:, None] - y[None, :]
    cy = y[:, None] + x[None, :]
    return np.stack([cx.reshape(-1), cy.reshape(-1)], axis=1)


def _em_assign(D, temperature):
    """Assignment weights of Eq. W from a distance matrix D [N][centres]: softmax(-D / T) per point, or the
    indicator of the nearest centre when temperature is None (Algorithm 1's E step as printed)."""
    if temperature is None:
        W = np.zeros_like(D)
        W[np.arange(D.shape[0]), np.argmin(D, axis=1)] = 1.0
        return W
    Z = -D / float(temperature)
    Z -= Z.max(axis=1, keepdims=True)
    W = np.exp(Z)
    W /= W.sum(axis=1, keepdims=True)
    return W


def _em_mstep(W, data, Nc):
    """M step of App. A.2 for one 2-D sub-space: phi* = (T^T S T)^-1 T^T S m with the constant matrix T written
    out entry by entry, S = diag of every centre's assigned weight (one entry per coordinate), m the weighted
    mean of the points assigned to it.  W [N][Nc^2], data [N][2]; returns phi [Nc][2]."""
    Nij = W.sum(axis=0)                                                          # weight of every centre
    sums = W.T @ data                                                            # [Nc^2][2]
    mean = np.where(Nij[:, None] > 0, sums / np.maximum(Nij[:, None], 1e-300), 0.0)
    # T: (2 Nc^2) x (2 Nc); row 2(a Nc + b) is the x coordinate of centre (a, b) = x_a - y_b,
    # row 2(a Nc + b) + 1 its y coordinate = y_a + x_b; phi is ordered x_0, y_0, x_1, y_1, ...
    Tm = np.zeros((2 * Nc * Nc, 2 * Nc))
    for a in range(Nc):
        for b in range(Nc):
            r = 2 * (a * Nc + b)
            Tm[r, 2 * a] += 1.0
            Tm[r, 2 * b + 1] += -1.0
            Tm[r + 1, 2 * b] += 1.0
            Tm[r + 1, 2 * a + 1] += 1.0
    S = np.repeat(Nij, 2)
    m = mean.reshape(-1)
    A = Tm.T @ (S[:, None] * Tm)
    rhs = Tm.T @ (S * m)
    return np.linalg.solve(A, rhs).reshape(Nc, 2)


def em_step_shared(data, phi, temperature=None):
    """One EM iteration when a group of g sub-spaces shares its quantized value (Sec. 4.2: s^0 = ... = s^{g-1};
    g = 64 = the whole head in the paper's configurations).

    data [N][g][2]: the calibration vectors, cut into their g sub-vectors; phi [g][Nc][2]: every sub-space's
    (x_l, y_l).  A clustering centre is the pair (a, b) applied in all g sub-spaces at once, so the E step
    measures the distance of the whole vector to the whole centre, D_i,ab = sqrt(sum_j ||k_i^j - c_ab^j||^2),
    and gives one weight matrix W (Eq. W) for the group; the M step is App. A.2's closed form in every
    sub-space with that common W.  Returns (phi_new [g][Nc][2], weighted squared error before the update).
    """
    data = _f64(data)
    phi = _f64(phi)
    g, Nc = phi.shape[0], phi.shape[1]
    D2 = np.zeros((data.shape[0], Nc * Nc))
    for j in range(g):
        cen = em_centres(phi[j])
        D2 += ((data[:, j, None, :] - cen[None, :, :]) ** 2).sum(axis=2)
    D = np.sqrt(D2)
    W = _em_assign(D, temperature)
    new = np.stack([_em_mstep(W, data[:, j, :], Nc) for j in range(g)])
    return new, float((W * D2).sum())


def em_step(data, phi, temperature=None):
    """One iteration of the EM-like codebook learner for ONE 2-D sub-space (Sec. 4.2 Alg. 1, App. A.2).

    data [N][2]: calibration points; phi [Nc][2]: current (x_l, y_l).  E step: soft assignment
    W_ij = softmax_j(-D_ij / T) over the Nc^2 centres, D the Euclidean distance (Eq. W); temperature None
    means hard assignment to the nearest centre.  M step: the closed form phi* = (T^T S T)^-1 T^T S m
    (_em_mstep).  Returns (phi_new [Nc][2], weighted squared error before the update).
    """
    data = _f64(data)
    phi = _f64(phi)
    Nc = phi.shape[0]
    cen = em_centres(phi)
    D = np.sqrt(((data[:, None, :] - cen[None, :, :]) ** 2).sum(axis=2))        # [N][Nc^2]
    W = _em_assign(D, temperature)
    return _em_mstep(W, data, Nc), float((W * D ** 2).sum())
