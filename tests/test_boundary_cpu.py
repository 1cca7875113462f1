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
