"""The codebook learner end to end, as the paper runs it (Sec. 4.2 Algorithm 1's loop, residual refinement over
the levels, App. A.2's annealed temperature): level by level, iterate commvq_em_step_shared with a decaying
temperature, store the learnt level in the tied key table, encode the calibration vectors with commvq_encode_keys,
subtract what the level explains and learn the next level on the residuals; finally attend over a cache encoded
with the learnt table.  Every GPU step is checked against the fp64 oracle started from the same state
(oracle.em_step_shared, oracle.encode_keys, oracle.decode_attn); residuals are formed on the host, as a caller of
the library does.

N_c' = 16 centres per level are learnt (the oracle's literal T-matrix M step costs (2 N_c'^2) x (2 N_c') per
sub-space); the key format addresses 64 rows per level, so rows 16..63 of the table are parked far away and are
never the nearest centre.
"""
import numpy as np
import pytest

from paper_2506_18879_amd import synth

pytestmark = pytest.mark.gpu

D, J, NC, ROWS, LEVELS = 128, 64, 16, 64, 2
FAR = 64.0          # parked rows: every coordinate 64, squared distance to any calibration vector > 1e5


def hidden_vectors(n, seed):
    """Vectors that are sums over two levels of tied centres z_a + i z_b (Eq. def_center) plus a little noise; the
    second level is four times smaller than the first, as a residual level is."""
    rng = np.random.default_rng(seed)
    out = np.zeros((n, J), complex)
    tables = []
    for lev in range(LEVELS):
        z = (rng.standard_normal((J, NC)) + 1j * rng.standard_normal((J, NC))) * (0.5 / 4 ** lev)
        a, b = rng.integers(0, NC, n), rng.integers(0, NC, n)
        out += (z[:, a] + 1j * z[:, b]).T
        tables.append(z)
    out += 0.01 * (rng.standard_normal((n, J)) + 1j * rng.standard_normal((n, J)))
    data = np.stack([out.real, out.imag], axis=2).astype(np.float32)                   # [n][J][2]
    return data, tables


def table_rows(phi):
    """phi [J][NC][2] -> table rows [ROWS][D] in fp32: row c holds (x, y) of every sub-space; rows >= NC parked."""
    rows = np.full((ROWS, D), FAR, np.float32)
    rows[:NC] = np.ascontiguousarray(phi.transpose(1, 0, 2)).reshape(NC, D)
    return rows


def decode_level(rows_f64, ab):
    """Centres C[a] + i C[b] of one level for codes ab [n][2] (Eq. def_center): (x_a - y_b, y_a + x_b) per sub-space."""
    a, b = rows_f64[ab[:, 0]], rows_f64[ab[:, 1]]
    out = a.copy()
    out[:, 0::2] -= b[:, 1::2]
    out[:, 1::2] += b[:, 0::2]
    return out


def test_two_levels_learnt_encoded_and_attended(oracle):
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2506_18879_amd as cv
    from paper_2506_18879_amd import device
    import test_gpu_encode as enc                                   # the encoder's judge and GPU driver

    n = 640
    data, hidden = hidden_vectors(n, seed=2024)
    keys_bits = synth.f32_to_bf16_bits(data.reshape(n, 1, D))      # what the encoder is fed: bf16 keys, one KV head
    keys = synth.bf16_bits_to_f32(keys_bits).astype(np.float64).reshape(n, D)
    rng = np.random.default_rng(7)
    residual = keys.copy()
    table_bits = np.zeros((1, LEVELS, ROWS, D), np.uint16)
    err_before = float((keys ** 2).sum())
    for lev in range(LEVELS):
        # ---- learn the level on the current residuals, temperature annealed per iteration (App. A.2)
        res32 = residual.reshape(n, J, 2).astype(np.float32)
        start = np.stack([hidden[lev].real, hidden[lev].imag], axis=2) + 0.05 / 4 ** lev * rng.standard_normal((J, NC, 2))
        d_dev = torch.from_numpy(res32).cuda()
        phi_dev = torch.from_numpy(start.astype(np.float32)).cuda()
        nb = cv.commvq_em_shared_workspace_bytes(J, n, NC)
        ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
        T = 0.5 / 4 ** lev
        objective = []
        for it in range(4):
            before = phi_dev.cpu().numpy().astype(np.float64)
            cv.commvq_em_step_shared(d_dev, J, n, NC, T, phi_dev, ws, nb)
            torch.cuda.synchronize()
            got = phi_dev.cpu().numpy().astype(np.float64)
            want, _ = oracle.em_step_shared(res32, before, temperature=T)      # one oracle step from the same state
            dev = np.abs(got - want).max() / np.abs(want).max()
            print(f"level {lev} iteration {it} T={T:.4f}: phi deviation {dev:.2e}", flush=True)
            assert dev <= 2e-5                                                    # observed ~1e-6
            objective.append(oracle.em_step_shared(res32, got, temperature=None)[1])   # hard-assignment squared error
            T *= 0.6
        assert objective[-1] <= objective[0] * 1.0001, objective
        # ---- the level goes into the tied table (bf16 storage of the key format)
        table_bits[0, lev] = synth.f32_to_bf16_bits(table_rows(phi_dev.cpu().numpy()))
        rows = synth.bf16_bits_to_f32(table_bits[0, lev]).astype(np.float64)
        # ---- encode with the levels learnt so far; the new level's codes are judged against the oracle's search
        w = synth.make_pair_workload(f"learn_l{lev}", B=1, Hq=4, Hkv=1, seqlens=[8], R=lev + 1, Mv=16, seed=5)
        w.key_codebooks = np.ascontiguousarray(table_bits[:, :lev + 1])
        rec = enc.encode_on_gpu(device, w, keys_bits, L_cap=n)[0]                        # [n][record bytes]
        a, b = oracle.unpack_key_pairs(rec, lev + 1)
        codes = np.stack([a, b], axis=-1)                                                # [n][levels][2]
        assert codes.max() < NC                                                          # parked rows are never chosen
        tab = synth.bf16_bits_to_f32(table_bits[0, :lev + 1]).astype(np.float64)
        same = enc.judge(oracle, keys, tab, codes, True)
        print(f"level {lev}: records identical to the oracle's {same.mean():.4f}", flush=True)
        assert same.mean() >= 0.98
        # ---- residuals for the next level: what this level's chosen centres leave (formed by the caller)
        residual = residual - decode_level(rows, codes[:, lev])
        err_after = float((residual ** 2).sum())
        print(f"level {lev}: squared error {err_before:.2f} -> {err_after:.2f}", flush=True)
        assert err_after < 0.5 * err_before                                             # every level explains most of what is left
        err_before = err_after
    # the residual the host tracked is what the oracle's own residual bookkeeping gives for the GPU's records
    _, _, taken = oracle.encode_keys(keys, tab, paired=True, given=codes)
    assert abs(taken[:, -1].sum() - err_after) <= 1e-6 * err_after

    # ---- attend over a cache that holds these records, with the learnt table
    L = 500
    w = synth.make_pair_workload("learn_attend", B=1, Hq=4, Hkv=1, seqlens=[L], R=LEVELS, Mv=16, seed=9)
    w.key_codebooks = table_bits
    w.key_codes = np.ascontiguousarray(rec[:L]).reshape(-1)
    dw = device.DeviceWorkload(w)
    op = device.DecodeAttention(w)
    out = op(dw)
    torch.cuda.synchronize()
    ref = oracle.decode_attn(w.as_f64("q"), oracle.paired_as_indexed(w.key_codes, LEVELS, w.cu_seqlens, 1), w.val_codes,
                             oracle.tied_table_as_codebooks(w.as_f64("key_codebooks"), K=w.K), w.as_f64("val_codebooks"),
                             w.cu_seqlens, w.q_pos, rope_base=w.rope_base)
    err = np.abs(out.cpu().numpy() - ref).max(axis=-1) / np.abs(ref).max(axis=-1)
    print(f"attention over the learnt table: max row error {err.max():.2e}", flush=True)
    assert err.max() <= 2e-5
    op.close()
