"""The workload generator: shapes, layouts, determinism and the bf16 helpers."""
import numpy as np

from paper_2506_18879_amd import synth


def test_bf16_round_trip_and_rounding():
    x = np.array([1.0, -2.5, 3.140625, 1e-3, 0.0], np.float32)
    b = synth.f32_to_bf16_bits(x)
    y = synth.bf16_bits_to_f32(b)
    assert np.all(np.abs(y - x) <= np.abs(x) * 2.0 ** -8)
    assert np.array_equal(synth.f32_to_bf16_bits(y), b)  # idempotent
    # round to nearest even on the dropped 16 bits
    assert synth.f32_to_bf16_bits(np.array([1.0 + 2.0 ** -8], np.float32))[0] == 0x3F80
    assert synth.f32_to_bf16_bits(np.array([1.0 + 3 * 2.0 ** -8], np.float32))[0] == 0x3F82


def test_config_shapes_small():
    for idx, (B, Hq, Hkv, Mk, Mv, dt) in {1: (1, 1, 1, 32, 32, "f32"), 2: (1, 32, 8, 32, 32, "bf16"),
                                          3: (1, 32, 8, 16, 16, "bf16"), 4: (8, 32, 8, 32, 32, "bf16"),
                                          5: (4, 64, 8, 32, 16, "bf16")}.items():
        w = synth.config(idx, max_len=300)
        assert (w.B, w.Hq, w.Hkv, w.Mk, w.Mv, w.dtype) == (B, Hq, Hkv, Mk, Mv, dt)
        T = w.total_tokens
        assert w.key_codes.size == T * Hkv * Mk and w.val_codes.size == T * Hkv * Mv
        assert w.key_codebooks.shape == (Hkv, Mk, 256, 128) and w.val_codebooks.shape == (Hkv, Mv, 256, 128)
        assert w.q.shape == (B, Hq, 128) and w.cu_seqlens[0] == 0 and np.all(w.q_pos == np.diff(w.cu_seqlens) - 1)
        assert w.seq_codes("key", B - 1).shape == (Hkv, int(np.diff(w.cu_seqlens)[-1]), Mk)


def test_deterministic_and_seed_sensitive():
    a, b, c = synth.config(2, max_len=64), synth.config(2, max_len=64), synth.config(2, max_len=64, seed=1)
    assert np.array_equal(a.key_codes, b.key_codes) and np.array_equal(a.key_codebooks, b.key_codebooks)
    assert not np.array_equal(a.key_codes, c.key_codes)


def test_codebook_scale_and_zipf_skew():
    w = synth.config(3, max_len=4096)
    cb = w.as_f64("key_codebooks")
    assert abs(cb.std() - 16 ** -0.5) < 0.01  # N(0, M^-1/2)
    kc = w.seq_codes("key", 0)
    top = max(np.bincount(kc[0, :, 0], minlength=256)) / kc.shape[1]
    assert 0.15 < top < 0.28  # the hottest codeword takes ~21 % under Zipf(1.1) over 256 ranks
    # the hot codeword differs between codebooks (independent rank permutations)
    hot = [int(np.argmax(np.bincount(kc[0, :, m], minlength=256))) for m in range(16)]
    assert len(set(hot)) > 4


def test_ragged_lengths_config4():
    w = synth.config(4, max_len=65536 // 64)
    lens = np.diff(w.cu_seqlens)
    assert len(lens) == 8 and lens.min() >= 8192 // 64 and lens.max() <= 65536 // 64
