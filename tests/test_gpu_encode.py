"""GPU parity of the key encoder (cache append) against the fp64 oracle.

The encoder decides integers (nearest centre per level) from fp32 distances; the oracle decides them in
fp64.  A different choice is correct when the two centres are equidistant up to rounding, and from then
on the residuals differ, so the comparison is: (i) almost all records are identical, and (ii) for EVERY
record, at every level, the centre the GPU took is as near to the residual left by its own earlier
choices as the nearest centre the oracle finds for that residual, within fp32 rounding.
"""
import numpy as np
import pytest

from paper_2506_18879_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2506_18879_amd as cv
    cv.load_library()
    from paper_2506_18879_amd import device
    return device


def encode_on_gpu(gpu, w, keys_host, L_cap):
    """Encode keys [n][Hkv][d] (bf16 bits as uint16, or float32, matching w.dtype) straight into a cache-shaped
    buffer [Hkv][L_cap][record]."""
    import torch
    import paper_2506_18879_amd as cv
    n = keys_host.shape[0]
    bf = w.dtype == "bf16"
    assert keys_host.dtype == (np.uint16 if bf else np.float32)
    paired = w.key_format == "paired"
    rec = (12 * w.key_levels + 7) // 8 if paired else w.Mk
    op = gpu.DecodeAttention(w)
    kcb = gpu.to_device(w.key_codebooks, bf)
    keys = gpu.to_device(keys_host, bf)
    tables = torch.empty(cv.commvq_encoder_table_bytes(op.handle), dtype=torch.uint8, device="cuda")
    cache = torch.full((w.Hkv, L_cap, rec), 0xEE, dtype=torch.uint8, device="cuda")
    cv.commvq_encoder_prepare(op.handle, kcb, tables)
    cv.commvq_encode_keys(op.handle, keys, n, kcb, tables, cache, rec, L_cap * rec)
    torch.cuda.synchronize()
    out = cache.cpu().numpy()
    assert (out[:, n:] == 0xEE).all()          # nothing written past the n appended tokens
    op.close()
    return out[:, :n]                           # [Hkv][n][rec]


# fp32 rounding of a candidate's score ||c||^2 - 2 res.c (index form: one 128-term dot product; paired form: two of
# them plus three table terms) relative to the magnitudes that enter it.  128 terms x 2^-24, times 2 for the factor
# in front of the dot product and a little room for the table terms; observed differences are ~50x smaller.
FP32_SCORE_EPS = 2.0 * 128 * 2.0 ** -24 * 1.5


def judge(oracle, keys_f64, cb_f64, gpu_codes, paired):
    """keys [n][d], cb [levels][K][d], gpu_codes [n][levels(,2)] of one head.

    The GPU compares fp32 scores; the oracle fp64 distances.  Level by level, on the residual that the GPU's own
    earlier choices leave (oracle.encode_keys(given=...)), the centre the GPU took may be farther than the nearest
    one only by the fp32 error bound of that level: FP32_SCORE_EPS x (|res| |c| + |c|^2) with |res| the norm of the
    residual searched and |c| the largest centre norm of the level.  A record that differs from the oracle's own
    must differ first at such a near tie (implied, since every level passes the bound).  Returns which records are
    identical to the oracle's.
    """
    want, _, _ = oracle.encode_keys(keys_f64, cb_f64, paired=paired)
    _, best, taken = oracle.encode_keys(keys_f64, cb_f64, paired=paired, given=gpu_codes)
    same = np.all((want == gpu_codes).reshape(len(keys_f64), -1), axis=1)
    levels = cb_f64.shape[0]
    res_before = np.concatenate([(keys_f64 ** 2).sum(axis=1, keepdims=True), taken[:, :-1]], axis=1)   # [n][levels]
    row = np.sqrt((cb_f64 ** 2).sum(axis=-1).max(axis=-1))                                             # [levels]
    cmax = 2.0 * row if paired else row                                  # |C[a] + i C[b]| <= |C[a]| + |C[b]|
    tol = FP32_SCORE_EPS * (np.sqrt(res_before) * cmax[None, :] + cmax[None, :] ** 2)
    excess = taken - best
    assert excess.min() >= -1e-9 * (1 + best.max())                       # nothing beats the exhaustive search
    worst = float((excess / tol).max())
    assert worst <= 1.0, f"a chosen centre is {worst:.2f} x the fp32 bound farther than the nearest one"
    # a differing record differs FIRST at a level where its choice is not the oracle's nearest for the common residual
    for t in np.nonzero(~same)[0]:
        l = int(np.argmax((want[t] != gpu_codes[t]).reshape(levels, -1).any(axis=1)))
        assert 0.0 <= excess[t, l] <= tol[t, l]
    return same


def _keys(rng, n, w):
    k = rng.standard_normal((n, w.Hkv, w.d)).astype(np.float32)
    if w.dtype == "bf16":
        bits = synth.f32_to_bf16_bits(k)
        return bits, synth.bf16_bits_to_f32(bits).astype(np.float64)
    return k, k.astype(np.float64)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("n", [5, 96, 200])
@pytest.mark.parametrize("Mk", [16, 32])
def test_encode_index_form(gpu, oracle, Mk, n, dtype):
    # bf16, n < 64: one workgroup per token (decode-step append); n >= 64: 64 tokens per workgroup on the matrix
    # cores; fp32 keys and codebooks: one thread per centre, rows straight from L2, any n
    w = synth.make_workload(f"enc_m{Mk}", B=1, Hq=4, Hkv=2, seqlens=[8], Mk=Mk, Mv=16, dtype=dtype, seed=200 + Mk)
    rng = np.random.default_rng(Mk + n)
    keys, kf = _keys(rng, n, w)
    got = encode_on_gpu(gpu, w, keys, L_cap=n + 5)
    cb = w.as_f64("key_codebooks")
    same = np.concatenate([judge(oracle, kf[:, g], cb[g], got[g], False) for g in range(w.Hkv)])
    print(f"  identical records: {same.mean():.4f}", flush=True)
    assert same.mean() >= 0.99


def test_encode_fp32_single_head_feeds_attention(gpu, oracle):
    """The fp32 single-head configuration end to end: append 300 keys with the fp32 encoder, then attend over the
    records it wrote (fp32 codebooks take the row-gather score kernel)."""
    import torch
    L = 300
    w = synth.make_workload("enc_attn_f32", B=1, Hq=1, Hkv=1, seqlens=[L], Mk=32, Mv=32, dtype="f32", seed=77)
    rng = np.random.default_rng(5)
    keys, kf = _keys(rng, L, w)
    got = encode_on_gpu(gpu, w, keys, L_cap=L)
    same = judge(oracle, kf[:, 0], w.as_f64("key_codebooks")[0], got[0], False)
    assert same.mean() >= 0.99
    w.key_codes = np.ascontiguousarray(got).reshape(-1)
    dw = gpu.DeviceWorkload(w)
    op = gpu.DecodeAttention(w)
    out = op(dw)
    torch.cuda.synchronize()
    ref = oracle.decode_attn(w.as_f64("q"), w.key_codes, w.val_codes, w.as_f64("key_codebooks"), w.as_f64("val_codebooks"),
                             w.cu_seqlens, w.q_pos, rope_base=w.rope_base)
    err = np.abs(out.cpu().numpy() - ref).max(axis=-1) / np.abs(ref).max(axis=-1)
    assert err.max() <= 2e-5
    op.close()


@pytest.mark.parametrize("n", [40, 130])
@pytest.mark.parametrize("R", [11, 21, 2])
def test_encode_paired_format(gpu, oracle, R, n):
    # n < 64: one workgroup per token; n >= 64: 64 tokens per workgroup, dot products on the matrix cores
    w = synth.make_pair_workload(f"enc_R{R}", B=1, Hq=4, Hkv=2, seqlens=[8], R=R, Mv=16, seed=300 + R)
    rng = np.random.default_rng(R + n)
    keys, kf = _keys(rng, n, w)
    got = encode_on_gpu(gpu, w, keys, L_cap=n)
    tab = w.as_f64("key_codebooks")
    sames = []
    for g in range(w.Hkv):
        a, b = oracle.unpack_key_pairs(got[g], R)                       # the same bytes the attention call reads
        codes = np.stack([a, b], axis=-1)
        sames.append(judge(oracle, kf[:, g], tab[g], codes, True))
    same = np.concatenate(sames)
    print(f"  identical records: {same.mean():.4f}", flush=True)
    assert same.mean() >= 0.98


def test_encode_recovers_exact_centres_and_feeds_attention(gpu, oracle):
    """Keys that ARE first-level centres come back as that centre; and records written by the encoder are
    consumed by commvq_decode_attn (append, then attend) with the oracle agreeing on the result."""
    import torch
    R = 11
    L = 300
    w = synth.make_pair_workload("enc_attn", B=1, Hq=8, Hkv=2, seqlens=[L], R=R, Mv=16, seed=42)
    tab_bits = w.key_codebooks                                           # [Hkv][R][64][d] bf16 bits
    keys = np.stack([tab_bits[g, 0, np.arange(L) % 64] for g in range(w.Hkv)], axis=1)   # [L][Hkv][d]
    got = encode_on_gpu(gpu, w, keys, L_cap=L)
    tab = w.as_f64("key_codebooks")
    for g in range(w.Hkv):
        a, b = oracle.unpack_key_pairs(got[g], R)
        # the first level must reproduce the key up to the best partner b: distance <= that of (a = own index, any b)
        codes = np.stack([a, b], axis=-1)
        judge(oracle, synth.bf16_bits_to_f32(keys[:, g]).astype(np.float64), tab[g], codes, True)
    # append -> attend
    w.key_codes = np.ascontiguousarray(got).reshape(-1)                  # [Hkv][L][PB] of the single sequence
    dw = gpu.DeviceWorkload(w)
    op = gpu.DecodeAttention(w)
    out = op(dw)
    torch.cuda.synchronize()
    kc = oracle.paired_as_indexed(w.key_codes, R, w.cu_seqlens, w.Hkv)
    ref = oracle.decode_attn(w.as_f64("q"), kc, w.val_codes, oracle.tied_table_as_codebooks(tab, K=w.K),
                             w.as_f64("val_codebooks"), w.cu_seqlens, w.q_pos, rope_base=w.rope_base, n_threads=8)
    err = np.abs(out.cpu().numpy() - ref).max(axis=-1) / np.abs(ref).max(axis=-1)
    assert err.max() <= 2e-5
    op.close()


@pytest.mark.parametrize("dtype,Mv,n", [("bf16", 16, 7), ("bf16", 32, 150), ("f32", 32, 40)])
def test_encode_values_greedy_residual_assignment(gpu, oracle, dtype, Mv, n):
    """The stand-in value encoder: same residual nearest-row search as the key encoder in index form, over the VALUE
    codebooks (which have no block structure); and the records it writes are what commvq_decode_attn reads."""
    import torch
    import paper_2506_18879_amd as cv
    w = synth.make_workload(f"encv_{dtype}_{Mv}", B=1, Hq=4, Hkv=2, seqlens=[n], Mk=16, Mv=Mv, dtype=dtype, seed=900 + Mv + n)
    bf = dtype == "bf16"
    rng = np.random.default_rng(Mv + n)
    vals, vf = _keys(rng, n, w)
    op = gpu.DecodeAttention(w)
    vcb = gpu.to_device(w.val_codebooks, bf)
    tables = torch.empty(cv.commvq_value_encoder_table_bytes(op.handle), dtype=torch.uint8, device="cuda")
    cache = torch.full((w.Hkv, n, Mv), 0xEE, dtype=torch.uint8, device="cuda")
    cv.commvq_value_encoder_prepare(op.handle, vcb, tables)
    cv.commvq_encode_values(op.handle, gpu.to_device(vals, bf), n, vcb, tables, cache, Mv, n * Mv)
    torch.cuda.synchronize()
    got = cache.cpu().numpy()
    cb = w.as_f64("val_codebooks")
    same = np.concatenate([judge(oracle, vf[:, g], cb[g], got[g], False) for g in range(w.Hkv)])
    assert same.mean() >= 0.99
    # append -> attend: the cache's value codes are the encoder's records
    w.val_codes = np.ascontiguousarray(got).reshape(-1)
    dw = gpu.DeviceWorkload(w)
    out = op(dw)
    torch.cuda.synchronize()
    ref = oracle.decode_attn(w.as_f64("q"), w.key_codes, w.val_codes, w.as_f64("key_codebooks"), cb, w.cu_seqlens, w.q_pos,
                             rope_base=w.rope_base)
    err = np.abs(out.cpu().numpy() - ref).max(axis=-1) / np.abs(ref).max(axis=-1)
    assert err.max() <= 2e-5
    op.close()


def test_encode_rejects_overlapping_records(gpu):
    import torch
    import paper_2506_18879_amd as cv
    w = synth.make_workload("enc_err", B=1, Hq=4, Hkv=2, seqlens=[8], Mk=16, Mv=16, dtype="bf16", seed=1)
    op = gpu.DecodeAttention(w)
    buf = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    with pytest.raises(cv.CommVQError) as e:
        cv.commvq_encode_keys(op.handle, buf, 1, buf, buf, buf, 8, 16)
    assert e.value.status == 3
    with pytest.raises(cv.CommVQError) as e:
        cv.commvq_encode_keys(op.handle, buf, 0, buf, buf, buf, 16, 16)
    assert e.value.status == 3
    with pytest.raises(cv.CommVQError) as e:        # misaligned tables
        cv.commvq_encode_keys(op.handle, buf, 1, buf, buf.data_ptr() + 4, buf, 16, 16)
    assert e.value.status == 3
    op.close()
