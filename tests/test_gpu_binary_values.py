"""GPU parity for the paper's binary value code (Sec. 4.1): libcommvq through its C ABI against the fp64 oracle.

Same bars as the index-form parity tests: 2e-3 per output row as the contract, 2e-5 per row and 2e-2 element by
element (floor 1e-3 of the row maximum) as regression bars.
"""
import numpy as np
import pytest

from paper_2506_18879_amd import synth

pytestmark = pytest.mark.gpu

TOL_OUT, TOL_REGRESS, ELEM_FLOOR = 2e-3, 2e-5, 1e-3


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2506_18879_amd as cv
    cv.load_library()
    from paper_2506_18879_amd import device
    return device


def oracle_out(oracle, w, **kw):
    return oracle.decode_attn_binary_values(w.as_f64("q"), w.key_codes, w.val_codes, w.as_f64("key_codebooks"),
                                            w.as_f64("val_codebooks"), w.cu_seqlens, w.q_pos, key_pos=w.key_pos,
                                            rope_base=w.rope_base, n_threads=16, **kw)


def errors(got, ref):
    got = np.asarray(got, np.float64)
    row = np.abs(got - ref).max(axis=-1) / np.abs(ref).max(axis=-1)
    floor = ELEM_FLOOR * np.abs(ref).max(axis=-1, keepdims=True)
    return float(row.max()), float((np.abs(got - ref) / np.maximum(np.abs(ref), floor)).max())


def run_gpu(gpu, w, staged=False, **kw):
    import torch
    dw = gpu.DeviceWorkload(w)
    op = gpu.DecodeAttention(w, **kw)
    out = op.staged(dw) if staged else op(dw)
    torch.cuda.synchronize()
    res = out.cpu().numpy()
    op.close()
    return res


def check(gpu, oracle, w, **kw):
    print(f"case {w.name} B={w.B} Hq={w.Hq} Hkv={w.Hkv} Mk={w.Mk} Nc={w.val_bits} lens={np.diff(w.cu_seqlens)[:8]}", flush=True)
    got = run_gpu(gpu, w, **kw)
    ref = oracle_out(oracle, w)
    assert np.isfinite(got).all()
    row, el = errors(got, ref)
    print(f"  max row error {row:.3e}, element-wise {el:.3e}", flush=True)
    assert row <= TOL_OUT, ("contract", row)
    assert row <= TOL_REGRESS, ("regression bar", row)
    assert el <= 1e3 * TOL_REGRESS, ("element-wise regression bar", el)
    return got, ref


def make(B, Hq, Hkv, lens, Nc, *, Mk=16, dtype="bf16", seed=1, density=0.5, code_dist="uniform"):
    base = synth.make_workload("vb", B=B, Hq=Hq, Hkv=Hkv, seqlens=lens, Mk=Mk, Mv=16, dtype=dtype, seed=seed,
                               code_dist=code_dist)
    return synth.with_binary_values(base, Nc, density=density)


@pytest.mark.parametrize("Nc", [1024, 2048, 4096])
@pytest.mark.parametrize("Hq,Hkv", [(32, 8), (8, 8), (16, 8), (64, 8), (8, 1), (4, 2)])
def test_binary_values_group_sizes_and_code_widths(gpu, oracle, Nc, Hq, Hkv):
    # G = 4, 1, 2, 8 (32 and 64 query heads: one and two head groups), 8 heads on one KV head, and a head count below
    # the matrix instruction's 16 rows; lengths with a ragged tail inside a 128-token stage and inside a 64-token step
    check(gpu, oracle, make(2, Hq, Hkv, [1500, 333], Nc, seed=Nc + Hq))


@pytest.mark.parametrize("density", [0.0, 0.02, 0.9, 1.0])
def test_binary_values_bit_densities(gpu, oracle, density):
    w = make(1, 32, 8, [2100], 1024, seed=11, density=density)
    if density == 0.0:  # no bit set anywhere: every value is the zero vector
        got = run_gpu(gpu, w)
        assert np.array_equal(got, np.zeros_like(got))
    else:
        check(gpu, oracle, w)


def test_binary_values_fp32_storage_and_two_bit_keys(gpu, oracle):
    check(gpu, oracle, make(1, 4, 1, [3000], 1024, Mk=32, dtype="f32", seed=5))
    check(gpu, oracle, make(1, 32, 8, [2500], 2048, Mk=32, seed=6))


def test_binary_values_many_splits_and_empty_sequences(gpu, oracle):
    # 9000 tokens: several value ranges, each several stages; an empty batch slot gives zero rows
    w = make(3, 32, 8, [9000, 0, 1], 1024, seed=21)
    got = run_gpu(gpu, w)
    ref = oracle_out(oracle, synth_without_empty(w))
    assert np.array_equal(got[1], np.zeros_like(got[1]))
    for b_ref, b in enumerate([0, 2]):
        row, el = errors(got[b], ref[b_ref])
        assert row <= TOL_REGRESS and el <= 1e3 * TOL_REGRESS, (b, row, el)


def test_binary_values_one_long_range_per_sequence(gpu, oracle):
    # 130 sequences: more than the chip has workgroup slots, so every sequence is ONE token range; the long one runs
    # 47 stages through the same accumulators
    check(gpu, oracle, make(130, 32, 8, [6000] + [3] * 129, 1024, seed=81))


def synth_without_empty(w):
    """The same workload without its empty sequences (the oracle's softmax needs at least one token)."""
    import copy
    keep = np.flatnonzero(np.diff(w.cu_seqlens) > 0)
    v = copy.copy(w)
    v.B = len(keep)
    v.q = w.q[keep]
    v.q_pos = w.q_pos[keep]
    lens = np.diff(w.cu_seqlens)[keep]
    v.cu_seqlens = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    return v  # codes of empty sequences occupy no bytes, so the flat code arrays are already right


def test_binary_values_peaked_and_flat_attention(gpu, oracle):
    # one dominant token (weights of the others far below the fixed-point unit of a naive scaling) and an all-zero query
    # (uniform weights: the closed form (1 / L) colsum(S_V) C_V)
    w = make(1, 32, 8, [4000], 1024, seed=31)
    w.q = synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(w.q) * np.float32(6.0))
    check(gpu, oracle, w)
    w0 = make(1, 32, 8, [4000], 1024, seed=32)
    w0.q = np.zeros_like(w0.q)
    got, _ = check(gpu, oracle, w0)
    S = np.unpackbits(w0.val_codes.reshape(4000, 128), axis=1, bitorder="little").astype(np.float64)
    full = (S.sum(axis=0) / 4000.0) @ w0.as_f64("val_codebooks")
    for h in range(32):
        g = h // 4
        assert np.abs(got[0, h] - full[g * 128:(g + 1) * 128]).max() <= 2e-5 * np.abs(full).max()


def test_binary_value_bins_through_an_identity_codebook(gpu, oracle):
    # With C_V = a cyclically shifted identity the output row of head h IS a run of 128 of its normalised bins
    # (out[h][e] = bins[h][(g d + e + shift) mod N_c] / sum): every code bit's bin is read off directly, with no codebook
    # arithmetic in between, and must match the oracle far inside the usual bar.
    w = make(1, 32, 8, [1900], 1024, seed=41)
    for shift in (0, 128, 640):
        eye = np.roll(np.eye(1024, dtype=np.float32), -shift, axis=0)  # row c has its 1 in column (c - shift) mod 1024
        w.val_codebooks = synth.f32_to_bf16_bits(eye)
        got = run_gpu(gpu, w)
        ref = oracle_out(oracle, w)
        row, _ = errors(got, ref)
        print(f"  shift {shift}: max row error {row:.3e}", flush=True)
        assert row <= 2e-6, (shift, row)


def test_binary_values_staged_and_repeatable(gpu):
    w = make(2, 32, 8, [3000, 1200], 1024, seed=51)
    a = run_gpu(gpu, w)
    b = run_gpu(gpu, w, staged=True)
    c = run_gpu(gpu, w)
    assert np.array_equal(a, b) and np.array_equal(a, c)  # integer bins: no dependence on the order of arrival


def test_binary_values_batched_output_kernel_and_packing(gpu, oracle):
    # 8 sequences x 4 heads per KV head = 32 output rows per KV head: the product with the value codebook runs on the
    # matrix cores; packing the codebook ahead of time must not change a bit
    import torch
    w = make(8, 32, 8, [600, 50, 1300, 7, 64, 129, 1024, 2], 1024, seed=61)
    got, _ = check(gpu, oracle, w)
    dw = gpu.DeviceWorkload(w)
    op = gpu.DecodeAttention(w)
    op.pack_value_codebooks(dw)
    op.pack_key_codebooks(dw)
    out = op(dw)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), got)
    op.close()


def test_binary_values_with_paired_keys(gpu, oracle):
    # the paper's own formats on both sides: paired 12-bit key records (R = 11) and 1024 value bits per token
    base = synth.make_pair_workload("pv", B=1, Hq=32, Hkv=8, seqlens=[2300], R=11, Mv=16, seed=71)
    w = synth.with_binary_values(base, 1024)
    got = run_gpu(gpu, w)
    kc = oracle.paired_as_indexed(w.key_codes, 11, w.cu_seqlens, w.Hkv)
    kcb = oracle.tied_table_as_codebooks(w.as_f64("key_codebooks"), K=256)
    ref = oracle.decode_attn_binary_values(w.as_f64("q"), kc, w.val_codes, kcb, w.as_f64("val_codebooks"), w.cu_seqlens,
                                           w.q_pos, rope_base=w.rope_base, n_threads=16)
    row, el = errors(got, ref)
    assert row <= TOL_REGRESS and el <= 1e3 * TOL_REGRESS, (row, el)


def test_binary_values_full_size_sampled_heads(gpu, oracle):
    # the bench shape (8B layer, 131072 tokens, N_c = 1024) in the launch configuration bench.py times; the oracle
    # computes two of the eight KV heads (8 of the 32 output rows)
    w = synth.config(8)
    got = run_gpu(gpu, w)
    mask = np.zeros((1, 8), bool)
    mask[0, [1, 6]] = True
    ref = oracle_out(oracle, w, unit_mask=mask)
    rows = [h for h in range(32) if mask[0, h // 4]]
    row, el = errors(got[0, rows], ref[0, rows])
    print(f"  full size: max row error {row:.3e}, element-wise {el:.3e}", flush=True)
    assert row <= TOL_REGRESS and el <= 1e3 * TOL_REGRESS


def test_binary_values_static_scratch_entry_and_graph_replay(gpu):
    # the entry point that allocates nothing, and a captured call, must give the eager call's bits
    import torch
    import paper_2506_18879_amd as cv
    w = synth.config(8, max_len=20000)
    dw = gpu.DeviceWorkload(w)
    op = gpu.DecodeAttention(w)
    eager = op(dw).clone()
    torch.cuda.synchronize()
    out = torch.full_like(eager, float("nan"))
    cv.commvq_decode_attn_static(op.handle, dw.q, dw.key_codes, dw.val_codes, dw.key_codebooks, dw.val_codebooks,
                                 dw.positions, out, op.stream_ptr())
    torch.cuda.synchronize()
    assert torch.equal(out, eager)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        op(dw)
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            op(dw)
    torch.cuda.synchronize()
    for rep in range(3):
        op.out.zero_()
        graph.replay()
        torch.cuda.synchronize()
        replayed = op.out.clone()
        again = op(dw).clone()      # eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(replayed, eager) and torch.equal(again, eager), rep
    op.close()


def test_paper_one_bit_setting_full_size_sampled_head(gpu, oracle):
    # workload 10: the paper's 1-bit setting on both sides (paired keys R = 11, 1024 value bits) at 131072 tokens, in the
    # launch configuration bench.py times; the oracle computes one of the eight KV heads (4 of the 32 output rows)
    w = synth.config(10)
    got = run_gpu(gpu, w)
    kc = oracle.paired_as_indexed(w.key_codes, w.key_levels, w.cu_seqlens, w.Hkv)
    kcb = oracle.tied_table_as_codebooks(w.as_f64("key_codebooks"), K=256)
    mask = np.zeros((1, 8), bool)
    mask[0, 5] = True
    ref = oracle.decode_attn_binary_values(w.as_f64("q"), kc, w.val_codes, kcb, w.as_f64("val_codebooks"), w.cu_seqlens,
                                           w.q_pos, rope_base=w.rope_base, unit_mask=mask, n_threads=1)
    row, el = errors(got[0, 20:24], ref[0, 20:24])
    print(f"  c10 full size: max row error {row:.3e}, element-wise {el:.3e}", flush=True)
    assert row <= TOL_REGRESS and el <= 1e3 * TOL_REGRESS


def _random_shape(case):
    """One seeded shape within the documented limits (as the index-form random-shape test draws them)."""
    rng = np.random.Generator(np.random.PCG64(9500 + case))
    G = int(rng.choice([1, 2, 4, 8]))
    Hkv = int(rng.integers(1, 9))
    kind = ["short", "mixed", "many", "long"][case % 4]
    if kind == "short":
        lens = rng.integers(1, 700, size=int(rng.integers(1, 7)))
    elif kind == "mixed":
        lens = rng.integers(1, 6000, size=int(rng.integers(2, 6)))
    elif kind == "many":     # a serving batch: many short sequences
        lens = rng.integers(1, 300, size=int(rng.integers(20, 40)))
    else:
        lens = rng.integers(5000, 14000, size=int(rng.integers(1, 3)))
    return G, Hkv, [int(x) for x in lens], rng


@pytest.mark.parametrize("case", range(12))
def test_random_shapes_binary_values(gpu, oracle, case):
    G, Hkv, lens, rng = _random_shape(case)
    Nc = int(rng.choice([1024, 2048, 4096]))
    density = float(rng.choice([0.05, 0.3, 0.5, 0.8]))
    w = make(len(lens), G * Hkv, Hkv, lens, Nc, Mk=int(rng.choice([16, 32])), dtype="f32" if case % 5 == 4 else "bf16",
             seed=9600 + case, density=density, code_dist="zipf" if case % 3 == 0 else "uniform")
    print(f"G={G} Hkv={Hkv} Nc={Nc} density={density}", flush=True)
    check(gpu, oracle, w)
