"""Host-only checks of the C-ABI boundary: the library loads, exports what the header declares,
and rejects bad configurations before touching a device."""
import os
import re

import pytest

import paper_2506_18879_amd as cv

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "commvq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(commvq_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = cv.load_library()
    names = header_functions()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(cv.binding.EXPORTS) == names


def good_cfg(**kw):
    c = dict(n_q_heads=32, n_kv_heads=8, head_dim=128, m_key=16, m_val=32, k=256, q_dtype=1, codebook_dtype=1,
             rope_base=500000.0, softmax_scale=0.0, max_position=131072)
    c.update(kw)
    return cv.Config(**c)


def test_validate_config_accepts_the_benchmark_shapes():
    for kw in (dict(), dict(n_q_heads=1, n_kv_heads=1, q_dtype=0, codebook_dtype=0, m_key=32),
               dict(n_q_heads=64, m_key=32, m_val=16)):
        assert cv.commvq_validate_config(good_cfg(**kw)) == 0


@pytest.mark.parametrize("kw", [
    dict(head_dim=64), dict(head_dim=127), dict(k=128), dict(m_key=8), dict(m_val=24), dict(n_q_heads=33),
    dict(n_q_heads=24), dict(n_kv_heads=0), dict(q_dtype=2), dict(codebook_dtype=-1), dict(rope_base=1.0),
    dict(softmax_scale=-1.0), dict(max_position=-1), dict(max_position=1 << 25)])
def test_validate_config_rejects(kw):
    assert cv.commvq_validate_config(good_cfg(**kw)) == 2  # COMMVQ_ERR_CONFIG


def test_validate_config_paired_key_format():
    ok = dict(key_format=cv.COMMVQ_KEYS_PAIRED, key_levels=11, m_key=0)   # m_key is ignored with paired keys
    assert cv.commvq_validate_config(good_cfg(**ok)) == 0
    assert cv.commvq_validate_config(good_cfg(**dict(ok, key_levels=21))) == 0
    for bad in (dict(ok, key_levels=0), dict(ok, key_levels=22), dict(ok, codebook_dtype=0, q_dtype=0),
                dict(key_format=2, key_levels=11)):
        assert cv.commvq_validate_config(good_cfg(**bad)) == 2


def test_validate_config_position_free():
    assert cv.commvq_validate_config(good_cfg(position_free=1)) == 0
    assert cv.commvq_validate_config(good_cfg(position_free=2)) == 2
    assert cv.commvq_validate_config(good_cfg(position_free=1, key_format=cv.COMMVQ_KEYS_PAIRED, key_levels=11)) == 2


def test_status_strings_are_distinct():
    s = {cv.commvq_status_string(i) for i in range(7)}
    assert len(s) == 7 and "ok" in s


def test_create_without_gpu_reports_no_device_not_a_crash():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(cv.CommVQError) as e:
        cv.commvq_create(good_cfg())
    assert e.value.status == 6
    with pytest.raises(cv.CommVQError) as e:
        cv.commvq_create(good_cfg(head_dim=64))
    assert e.value.status == 2  # configuration errors come first


def test_no_cpu_fallback():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    from paper_2506_18879_amd import synth
    from paper_2506_18879_amd.device import DeviceWorkload
    w = synth.make_workload("t", B=1, Hq=4, Hkv=1, seqlens=[8], Mk=16, Mv=16, dtype="bf16", seed=1)
    with pytest.raises(RuntimeError):
        DeviceWorkload(w)


# ---------------------------------------------------------------- planner handle: host logic without a GPU
@pytest.fixture()
def planner():
    made = []

    def make(**kw):
        h = cv.commvq_create_planner(good_cfg(**kw))
        made.append(h)
        return h

    yield make
    for h in made:
        cv.commvq_destroy(h)


def status_of(fn, *a, **kw):
    try:
        fn(*a, **kw)
    except cv.CommVQError as e:
        return e.status
    return 0


def test_planner_plans_the_five_configurations(planner):
    # (config kwargs, batch, total tokens, longest sequence) -> tile of the slice-streaming kernel, one value
    # workgroup per compute unit, bins x codebook chunks of 64 rows
    cases = [
        (dict(n_q_heads=1, n_kv_heads=1, m_key=32, m_val=32, q_dtype=0, codebook_dtype=0, max_position=4096), 1, 4096, 4096),
        (dict(m_key=32, m_val=32), 1, 32768, 32768),
        (dict(m_key=16, m_val=16), 1, 131072, 131072),
        (dict(m_key=32, m_val=32), 8, 300000, 65536),
        (dict(n_q_heads=64, m_key=32, m_val=16), 4, 4 * 131072, 131072),
    ]
    for kw, B, T, L in cases:
        h = planner(**kw)
        p = cv.commvq_plan_query(h, B, T, L)
        assert p.score_split_len in (16, 32, 64, 128, 256, 512, 1024, 2048, 4096)
        assert p.score_splits == -(-L // p.score_split_len)
        assert p.value_splits == -(-L // p.value_split_len) and 1 <= p.value_splits <= 256
        # a value split is a whole number of statistics tiles (score tiles, or 1024 tokens when the tiles are also cut
        # along the slices) or a power-of-two fraction of one, never under 1024 tokens
        stat = 1024 if p.score_slice_groups > 1 else p.score_split_len
        assert (p.value_split_len % max(stat, 1024) == 0 or p.score_kernel == 0
                or (stat % p.value_split_len == 0 and p.value_split_len >= 1024))
        assert p.out_chunks == kw.get("m_val", 32) * 256 // 64
        assert p.score_kernel == (0 if kw.get("codebook_dtype", 1) == 0 else 1)
        ws = cv.commvq_workspace_bytes(h, B, T, L)
        assert ws % 256 == 0 and ws >= 4 * T * kw.get("n_q_heads", 32)          # at least the logits
    # the workspace grows with the batch
    h = planner()
    assert cv.commvq_workspace_bytes(h, 2, 20000, 10000) > cv.commvq_workspace_bytes(h, 1, 10000, 10000)


@pytest.mark.parametrize("B,T,L", [(0, 10, 10), (1, 0, 0), (1, 10, 11), (2, 30, 10), (1, (1 << 30) + 1, (1 << 30) + 1)])
def test_planner_rejects_inconsistent_shapes(planner, B, T, L):
    h = planner(max_position=1 << 24)
    assert status_of(cv.commvq_plan_query, h, B, T, L) == 3
    assert status_of(cv.commvq_workspace_bytes, h, B, T, L) == 3


def test_one_head_stream_must_fit_32_bit_offsets(planner):
    # 2^27 tokens x 32 code bytes = 2^32: one past what a 32-bit byte offset reaches
    h = planner(m_key=32, m_val=32, max_position=1 << 24)
    assert status_of(cv.commvq_plan_query, h, 1, 1 << 27, 1 << 27) == 3
    assert status_of(cv.commvq_plan_query, h, 1, (1 << 27) - 1, (1 << 27) - 1) == 0
    h16 = planner(m_key=16, m_val=16, n_q_heads=8, n_kv_heads=8, max_position=1 << 24)
    assert status_of(cv.commvq_plan_query, h16, 1, 1 << 27, 1 << 27) == 0
    # eight heads of fp32 logits per token are 32 bytes as well
    h8 = planner(m_key=16, m_val=16, n_q_heads=64, n_kv_heads=8, max_position=1 << 24)
    assert status_of(cv.commvq_plan_query, h8, 1, 1 << 27, 1 << 27) == 3


class _Buf:
    """Stands in for a device buffer: the planner handle only looks at the address."""

    def __init__(self, addr):
        self.addr = addr

    def data_ptr(self):
        return self.addr


def _call_args(h, B=1, T=5000, L=5000, key_pos=None, ws_slack=0, ws_addr=1 << 20, code_addr=1 << 21):
    ws = cv.commvq_workspace_bytes(h, B, T, L)
    pos = cv.binding.make_positions(B, _Buf(4096), _Buf(8192), key_pos, T, L)
    return dict(q=_Buf(1 << 16), key_codes=_Buf(code_addr), val_codes=_Buf(1 << 22), key_codebooks=_Buf(1 << 23),
                val_codebooks=_Buf(1 << 24), positions=pos, out=_Buf(1 << 25), workspace=_Buf(ws_addr),
                workspace_bytes=ws + ws_slack)


def test_decode_attn_argument_checks_run_before_any_launch(planner):
    h = planner()
    call = lambda **a: status_of(cv.commvq_decode_attn, h, a["q"], a["key_codes"], a["val_codes"], a["key_codebooks"],
                                 a["val_codebooks"], a["positions"], a["out"], a["workspace"], a["workspace_bytes"])
    assert call(**_call_args(h)) == 6                                   # all fine: a full handle would launch here
    for missing in ("q", "key_codes", "val_codes", "key_codebooks", "val_codebooks", "out"):
        a = _call_args(h)
        a[missing] = None
        assert call(**a) == 1, missing
    a = _call_args(h)
    a["positions"] = cv.binding.make_positions(1, None, _Buf(8192), None, 5000, 5000)
    assert call(**a) == 1
    assert call(**_call_args(h, code_addr=(1 << 21) + 8)) == 3          # codes not 16-byte aligned
    assert call(**_call_args(h, ws_slack=-1)) == 4                      # one byte short
    assert call(**_call_args(h, ws_addr=(1 << 20) + 128)) == 4          # not 256-byte aligned
    a = _call_args(h)
    a["workspace"] = None
    assert call(**a) == 4
    a = _call_args(h)
    a["positions"] = cv.binding.make_positions(2, _Buf(4096), _Buf(8192), None, 5000, 2000)   # 5000 > 2 x 2000
    assert call(**a) == 3


def test_context_longer_than_the_phase_tables_is_refused(planner):
    h = planner(max_position=4095)
    call = lambda **a: status_of(cv.commvq_decode_attn, h, a["q"], a["key_codes"], a["val_codes"], a["key_codebooks"],
                                 a["val_codebooks"], a["positions"], a["out"], a["workspace"], a["workspace_bytes"])
    assert call(**_call_args(h, T=4096, L=4096)) == 6
    assert call(**_call_args(h, T=4097, L=4097)) == 3                   # token 0 would be 4096 away from the query
    # explicit key positions are the caller's to bound; the position-free variant has no rotation at all
    assert call(**_call_args(h, T=4097, L=4097, key_pos=_Buf(1 << 26))) == 6
    hf = planner(max_position=0, position_free=1)
    assert status_of(cv.commvq_plan_query, hf, 1, 9000, 9000) == 0


def test_paired_keys_refuse_explicit_positions_and_size_their_tables(planner):
    h = planner(key_format=cv.COMMVQ_KEYS_PAIRED, key_levels=11, m_key=0)
    a = _call_args(h, key_pos=_Buf(1 << 26))
    assert status_of(cv.commvq_decode_attn, h, a["q"], a["key_codes"], a["val_codes"], a["key_codebooks"],
                     a["val_codebooks"], a["positions"], a["out"], a["workspace"], a["workspace_bytes"]) == 2
    assert cv.commvq_packed_key_codebook_bytes(h) == 8 * 16 * 1 * 64 * 256        # 16 planes x 1 block of 16 KiB per head
    assert cv.commvq_encoder_table_bytes(h) == 8 * 11 * 64 * 4 * (1 + 64)         # norms + cross terms
    assert cv.commvq_value_encoder_table_bytes(h) == 8 * 32 * 256 * 4              # values are in index form whatever the keys
    hi = planner(m_key=16)
    assert cv.commvq_packed_key_codebook_bytes(hi) == 8 * 16 * 256 * 128 * 2
    assert cv.commvq_encoder_table_bytes(hi) == 8 * 16 * 256 * 4
    assert status_of(cv.commvq_encode_keys, hi, _Buf(1 << 20), 4, _Buf(1 << 21), _Buf(1 << 22), _Buf(1 << 23), 8, 16) == 3
    assert status_of(cv.commvq_encode_keys, hi, _Buf(1 << 20), 4, _Buf(1 << 21), _Buf(1 << 22), _Buf(1 << 23), 128, 16) == 6
    assert status_of(cv.commvq_encode_keys, hi, _Buf(1 << 20), 0, _Buf(1 << 21), _Buf(1 << 22), _Buf(1 << 23), 128, 16) == 3
    hv = planner(m_key=16, m_val=32)
    assert cv.commvq_value_encoder_table_bytes(hv) == 8 * 32 * 256 * 4
    # value codebooks re-laid for the batched output kernel: the size of the codebook itself; bf16 only; a batch with 16 or
    # more output rows per KV head reserves room for the per-call re-layout in its workspace
    assert cv.commvq_packed_value_codebook_bytes(hv) == 8 * 32 * 256 * 128 * 2
    assert cv.commvq_packed_value_codebook_bytes(hi) == 8 * 32 * 256 * 128 * 2
    h32 = planner(n_q_heads=1, n_kv_heads=1, q_dtype=0, codebook_dtype=0)
    assert status_of(cv.commvq_packed_value_codebook_bytes, h32) == 2
    assert status_of(cv.commvq_pack_value_codebooks, hv, _Buf(1 << 22), _Buf(1 << 26)) == 6
    cv.commvq_forget_packed_value_codebooks(hv)
    assert (cv.commvq_workspace_bytes(hv, 4, 4000, 1000) - cv.commvq_workspace_bytes(hv, 3, 3000, 1000)) > 8 * 32 * 256 * 128 * 2

    assert status_of(cv.commvq_encode_values, hv, _Buf(1 << 20), 4, _Buf(1 << 21), _Buf(1 << 22), _Buf(1 << 23), 256, 16) == 3   # 32-byte records
    assert status_of(cv.commvq_encode_values, hv, _Buf(1 << 20), 4, _Buf(1 << 21), _Buf(1 << 22), _Buf(1 << 23), 256, 32) == 6
    assert status_of(cv.commvq_value_encoder_prepare, hv, _Buf(1 << 21), _Buf((1 << 22) + 4)) == 3


def test_em_sizes_are_bounded():
    assert cv.commvq_em_workspace_bytes(64, 8192, 64) > 0
    for bad in ((0, 10, 4), (65536, 10, 4), (4, 0, 4), (4, (1 << 24) + 1, 4), (4, 10, 0), (4, 10, 65)):
        assert status_of(cv.commvq_em_workspace_bytes, *bad) == 3, bad
    for bad in ((0, 10, 4), (65, 10, 4), (4, 0, 4), (4, 10, 65)):
        assert status_of(cv.commvq_em_shared_workspace_bytes, *bad) == 3, bad


def test_static_scratch_entry_point_checks_its_arguments(planner):
    h = planner(max_position=1 << 23)
    a = _call_args(h)
    call = lambda pos, **kw: status_of(cv.commvq_decode_attn_static, h, kw.get("q", a["q"]), a["key_codes"], a["val_codes"],
                                       a["key_codebooks"], a["val_codebooks"], pos, a["out"])
    assert cv.commvq_static_scratch_bytes() == 48 << 20
    assert call(a["positions"]) == 6                                     # acceptable: a full handle would launch
    assert call(a["positions"], q=None) == 1
    big = cv.binding.make_positions(1, _Buf(4096), _Buf(8192), None, 4_000_000, 4_000_000)
    assert cv.commvq_workspace_bytes(h, 1, 4_000_000, 4_000_000) > cv.commvq_static_scratch_bytes()
    assert call(big) == 4                                                # more than the static array holds
    assert call(cv.binding.make_positions(1, _Buf(4096), _Buf(8192), None, 0, 0)) == 3


def test_bench_refuses_more_than_one_gpu():
    # one GPU per box in this build: --gpus N > 1 exits with a message and prints no result line
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and not r.stdout.strip()


def test_binary_value_format_config_plan_and_sizes(planner):
    ok = dict(value_format=cv.COMMVQ_VALUES_BINARY, value_bits=1024, m_val=0)   # m_val is ignored with binary values
    assert cv.commvq_validate_config(good_cfg(**ok)) == 0
    for bits in (2048, 4096):
        assert cv.commvq_validate_config(good_cfg(**dict(ok, value_bits=bits))) == 0
    for bad in (dict(ok, value_bits=0), dict(ok, value_bits=512), dict(ok, value_bits=1000), dict(ok, value_bits=8192),
                dict(value_format=2, value_bits=1024)):
        assert cv.commvq_validate_config(good_cfg(**bad)) == 2
    # the 8B-shaped layer at 128K: a value workgroup is 16 heads x 1024 code bits of a token range -> 2 head groups,
    # 128 ranges of 1024 tokens; the output stage sees N_c / 256 = 4 "codebooks" of 256 rows (16 chunks of 64 rows)
    h = planner(**ok)
    p = cv.commvq_plan_query(h, 1, 131072, 131072)
    assert (p.value_splits, p.value_split_len, p.out_chunks) == (128, 1024, 16)
    h70 = planner(**dict(ok, n_q_heads=64, m_key=32, value_bits=2048))
    p = cv.commvq_plan_query(h70, 4, 4 * 131072, 131072)
    assert p.value_splits * 4 * 2 * 4 <= 256 and p.value_splits * p.value_split_len >= 131072 and p.out_chunks == 32
    # bins: [B * Hkv * ranges][G * N_c] words are part of the workspace
    assert cv.commvq_workspace_bytes(h, 1, 131072, 131072) >= 131072 * 32 * 4 + 8 * 128 * 4 * 1024 * 4
    # records of N_c / 8 bytes per token must stay inside 32-bit offsets: 2^23 tokens x 512 bytes = 2^32
    h4k = planner(**dict(ok, value_bits=4096, max_position=1 << 24))
    assert status_of(cv.commvq_plan_query, h4k, 1, 1 << 23, 1 << 23) == 3
    assert status_of(cv.commvq_plan_query, h4k, 1, (1 << 23) - 1, (1 << 23) - 1) == 0
    # the packed value codebook has the size of the codebook; the greedy value encoder does not apply
    assert cv.commvq_packed_value_codebook_bytes(h) == 1024 * 8 * 128 * 2
    assert status_of(cv.commvq_value_encoder_table_bytes, h) == 2
    assert status_of(cv.commvq_encode_values, h, _Buf(1 << 20), 4, _Buf(1 << 21), _Buf(1 << 22), _Buf(1 << 23), 256, 32) == 2
    a = _call_args(h)
    assert status_of(cv.commvq_decode_attn, h, a["q"], a["key_codes"], a["val_codes"], a["key_codebooks"], a["val_codebooks"],
                     a["positions"], a["out"], a["workspace"], a["workspace_bytes"]) == 6


def test_binary_value_ranges_stay_within_the_32_bit_digit_sums(planner):
    # one sequence per workgroup-row of a big batch would give ranges as long as the context; they are capped at 2^16 tokens
    h = planner(value_format=cv.COMMVQ_VALUES_BINARY, value_bits=1024, m_val=0, max_position=1 << 24)
    p = cv.commvq_plan_query(h, 512, 512 << 20 >> 9 << 9, 1 << 20)
    assert p.value_split_len == 1 << 16 and p.value_splits == 16
