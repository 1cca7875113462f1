"""ctypes marshalling for libcommvq (see include/commvq.h for the contract)."""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, Structure, byref, c_double, c_float, c_int32, c_int64, c_size_t, c_void_p

from . import build as _build

COMMVQ_F32, COMMVQ_BF16 = 0, 1
COMMVQ_KEYS_INDEXED, COMMVQ_KEYS_PAIRED = 0, 1
COMMVQ_VALUES_INDEXED, COMMVQ_VALUES_BINARY = 0, 1
_lib = None


class CommVQError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({commvq_status_string(status)})")


class Config(Structure):
    _fields_ = [("n_q_heads", c_int32), ("n_kv_heads", c_int32), ("head_dim", c_int32), ("m_key", c_int32),
                ("m_val", c_int32), ("k", c_int32), ("q_dtype", c_int32), ("codebook_dtype", c_int32),
                ("rope_base", c_double), ("softmax_scale", c_double), ("max_position", c_int32),
                ("key_format", c_int32), ("key_levels", c_int32), ("position_free", c_int32),
                ("value_format", c_int32), ("value_bits", c_int32)]


class Positions(Structure):
    _fields_ = [("batch", c_int32), ("cu_seqlens", c_void_p), ("q_pos", c_void_p), ("key_pos", c_void_p),
                ("total_tokens", c_int64), ("max_seqlen", c_int32)]


class Plan(Structure):
    _fields_ = [("score_split_len", c_int32), ("score_splits", c_int32), ("value_split_len", c_int32),
                ("value_splits", c_int32), ("out_chunks", c_int32), ("score_kernel", c_int32),
                ("score_slice_groups", c_int32)]


Handle = c_void_p

EXPORTS = ("commvq_create", "commvq_create_planner", "commvq_destroy", "commvq_validate_config", "commvq_plan_query", "commvq_workspace_bytes",
           "commvq_decode_attn", "commvq_decode_attn_static", "commvq_static_scratch_bytes", "commvq_stage_scores", "commvq_stage_bins", "commvq_stage_output",
           "commvq_packed_key_codebook_bytes", "commvq_pack_key_codebooks", "commvq_forget_packed_key_codebooks",
           "commvq_packed_value_codebook_bytes", "commvq_pack_value_codebooks", "commvq_forget_packed_value_codebooks",
           "commvq_encoder_table_bytes", "commvq_encoder_prepare", "commvq_encode_keys",
           "commvq_value_encoder_table_bytes", "commvq_value_encoder_prepare", "commvq_encode_values",
           "commvq_em_workspace_bytes", "commvq_em_step", "commvq_em_shared_workspace_bytes", "commvq_em_step_shared",
           "commvq_profile_enable", "commvq_profile_read", "commvq_status_string")


def library_path() -> str:
    return _build.LIB


def load_library():
    """Load libcommvq.so (building it first only if it is not there); raises if that fails."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build()
    lib = ctypes.CDLL(_build.LIB)
    lib.commvq_status_string.restype = ctypes.c_char_p
    lib.commvq_status_string.argtypes = [ctypes.c_int]
    lib.commvq_validate_config.argtypes = [POINTER(Config)]
    lib.commvq_create.argtypes = [POINTER(Config), POINTER(c_void_p)]
    lib.commvq_create_planner.argtypes = [POINTER(Config), POINTER(c_void_p)]
    lib.commvq_destroy.argtypes = [c_void_p]
    lib.commvq_plan_query.argtypes = [c_void_p, c_int32, c_int64, c_int32, POINTER(Plan)]
    lib.commvq_workspace_bytes.argtypes = [c_void_p, c_int32, c_int64, c_int32, POINTER(c_size_t)]
    lib.commvq_decode_attn.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, POINTER(Positions),
                                       c_void_p, c_void_p, c_size_t, c_void_p]
    lib.commvq_decode_attn_static.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, POINTER(Positions),
                                              c_void_p, c_void_p]
    lib.commvq_static_scratch_bytes.argtypes = [POINTER(c_size_t)]
    lib.commvq_stage_scores.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, POINTER(Positions), c_void_p, c_size_t,
                                        c_void_p, c_void_p]
    lib.commvq_stage_bins.argtypes = [c_void_p, c_void_p, POINTER(Positions), c_void_p, c_size_t, c_void_p]
    lib.commvq_stage_output.argtypes = [c_void_p, c_void_p, POINTER(Positions), c_void_p, c_void_p, c_size_t, c_void_p]
    lib.commvq_packed_key_codebook_bytes.argtypes = [c_void_p, POINTER(c_size_t)]
    lib.commvq_pack_key_codebooks.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p]
    lib.commvq_forget_packed_key_codebooks.argtypes = [c_void_p, c_void_p]
    lib.commvq_packed_value_codebook_bytes.argtypes = [c_void_p, POINTER(c_size_t)]
    lib.commvq_pack_value_codebooks.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p]
    lib.commvq_forget_packed_value_codebooks.argtypes = [c_void_p, c_void_p]
    lib.commvq_encoder_table_bytes.argtypes = [c_void_p, POINTER(c_size_t)]
    lib.commvq_encoder_prepare.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p]
    lib.commvq_encode_keys.argtypes = [c_void_p, c_void_p, c_int32, c_void_p, c_void_p, c_void_p, c_int64, c_int64, c_void_p]
    lib.commvq_value_encoder_table_bytes.argtypes = [c_void_p, POINTER(c_size_t)]
    lib.commvq_value_encoder_prepare.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p]
    lib.commvq_encode_values.argtypes = [c_void_p, c_void_p, c_int32, c_void_p, c_void_p, c_void_p, c_int64, c_int64, c_void_p]
    lib.commvq_em_workspace_bytes.argtypes = [c_int32, c_int32, c_int32, POINTER(c_size_t)]
    lib.commvq_em_step.argtypes = [c_void_p, c_int32, c_int32, c_int32, c_float, c_void_p, c_void_p, c_size_t, c_void_p]
    lib.commvq_em_shared_workspace_bytes.argtypes = [c_int32, c_int32, c_int32, POINTER(c_size_t)]
    lib.commvq_em_step_shared.argtypes = [c_void_p, c_int32, c_int32, c_int32, c_float, c_void_p, c_void_p, c_size_t, c_void_p]
    lib.commvq_profile_enable.argtypes = [c_void_p, c_int32]
    lib.commvq_profile_read.argtypes = [c_void_p, POINTER(c_float), POINTER(c_int32)]
    for name in EXPORTS:
        if name != "commvq_status_string":
            getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def _ptr(x):
    """Device/host address of a torch tensor, an int address, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _check(status: int, where: str):
    if status != 0:
        raise CommVQError(status, where)


def commvq_status_string(status: int) -> str:
    return load_library().commvq_status_string(int(status)).decode()


def commvq_validate_config(cfg: Config) -> int:
    return load_library().commvq_validate_config(byref(cfg))


def commvq_create(cfg: Config) -> Handle:
    h = c_void_p()
    _check(load_library().commvq_create(byref(cfg), byref(h)), "commvq_create")
    return h


def commvq_create_planner(cfg: Config) -> Handle:
    h = c_void_p()
    _check(load_library().commvq_create_planner(byref(cfg), byref(h)), "commvq_create_planner")
    return h


def commvq_destroy(handle: Handle) -> None:
    _check(load_library().commvq_destroy(handle), "commvq_destroy")


def commvq_plan_query(handle: Handle, batch: int, total_tokens: int, max_seqlen: int) -> Plan:
    p = Plan()
    _check(load_library().commvq_plan_query(handle, batch, total_tokens, max_seqlen, byref(p)), "commvq_plan_query")
    return p


def commvq_workspace_bytes(handle: Handle, batch: int, total_tokens: int, max_seqlen: int) -> int:
    n = c_size_t()
    _check(load_library().commvq_workspace_bytes(handle, batch, total_tokens, max_seqlen, byref(n)),
           "commvq_workspace_bytes")
    return int(n.value)


def make_positions(batch, cu_seqlens, q_pos, key_pos, total_tokens, max_seqlen) -> Positions:
    return Positions(int(batch), _ptr(cu_seqlens), _ptr(q_pos), _ptr(key_pos), int(total_tokens), int(max_seqlen))


def commvq_decode_attn(handle, q, key_codes, val_codes, key_codebooks, val_codebooks, positions: Positions, out,
                       workspace, workspace_bytes: int, stream: int = 0) -> None:
    _check(load_library().commvq_decode_attn(handle, _ptr(q), _ptr(key_codes), _ptr(val_codes), _ptr(key_codebooks),
                                             _ptr(val_codebooks), byref(positions), _ptr(out), _ptr(workspace),
                                             int(workspace_bytes), stream or None), "commvq_decode_attn")


def commvq_decode_attn_static(handle, q, key_codes, val_codes, key_codebooks, val_codebooks, positions: Positions, out,
                              stream: int = 0) -> None:
    _check(load_library().commvq_decode_attn_static(handle, _ptr(q), _ptr(key_codes), _ptr(val_codes), _ptr(key_codebooks),
                                                    _ptr(val_codebooks), byref(positions), _ptr(out), stream or None),
           "commvq_decode_attn_static")


def commvq_static_scratch_bytes() -> int:
    n = c_size_t()
    _check(load_library().commvq_static_scratch_bytes(byref(n)), "commvq_static_scratch_bytes")
    return int(n.value)


def commvq_packed_key_codebook_bytes(handle) -> int:
    n = c_size_t()
    _check(load_library().commvq_packed_key_codebook_bytes(handle, byref(n)), "commvq_packed_key_codebook_bytes")
    return int(n.value)


def commvq_pack_key_codebooks(handle, key_codebooks, packed, stream: int = 0) -> None:
    _check(load_library().commvq_pack_key_codebooks(handle, _ptr(key_codebooks), _ptr(packed), stream or None),
           "commvq_pack_key_codebooks")


def commvq_forget_packed_key_codebooks(handle, key_codebooks=None) -> None:
    _check(load_library().commvq_forget_packed_key_codebooks(handle, _ptr(key_codebooks)),
           "commvq_forget_packed_key_codebooks")


def commvq_packed_value_codebook_bytes(handle) -> int:
    n = c_size_t(0)
    _check(load_library().commvq_packed_value_codebook_bytes(handle, byref(n)), "commvq_packed_value_codebook_bytes")
    return int(n.value)


def commvq_pack_value_codebooks(handle, val_codebooks, packed, stream: int = 0) -> None:
    _check(load_library().commvq_pack_value_codebooks(handle, _ptr(val_codebooks), _ptr(packed), stream or None),
           "commvq_pack_value_codebooks")


def commvq_forget_packed_value_codebooks(handle, val_codebooks=None) -> None:
    _check(load_library().commvq_forget_packed_value_codebooks(handle, _ptr(val_codebooks)),
           "commvq_forget_packed_value_codebooks")


def commvq_encoder_table_bytes(handle) -> int:
    n = c_size_t()
    _check(load_library().commvq_encoder_table_bytes(handle, byref(n)), "commvq_encoder_table_bytes")
    return int(n.value)


def commvq_encoder_prepare(handle, key_codebooks, tables, stream: int = 0) -> None:
    _check(load_library().commvq_encoder_prepare(handle, _ptr(key_codebooks), _ptr(tables), stream or None),
           "commvq_encoder_prepare")


def commvq_encode_keys(handle, keys, n_tokens: int, key_codebooks, tables, codes_out, token_stride: int,
                       head_stride: int, stream: int = 0) -> None:
    _check(load_library().commvq_encode_keys(handle, _ptr(keys), int(n_tokens), _ptr(key_codebooks), _ptr(tables),
                                             _ptr(codes_out), int(token_stride), int(head_stride), stream or None),
           "commvq_encode_keys")


def commvq_value_encoder_table_bytes(handle) -> int:
    n = c_size_t()
    _check(load_library().commvq_value_encoder_table_bytes(handle, byref(n)), "commvq_value_encoder_table_bytes")
    return int(n.value)


def commvq_value_encoder_prepare(handle, val_codebooks, tables, stream: int = 0) -> None:
    _check(load_library().commvq_value_encoder_prepare(handle, _ptr(val_codebooks), _ptr(tables), stream or None),
           "commvq_value_encoder_prepare")


def commvq_encode_values(handle, values, n_tokens: int, val_codebooks, tables, codes_out, token_stride: int,
                         head_stride: int, stream: int = 0) -> None:
    _check(load_library().commvq_encode_values(handle, _ptr(values), int(n_tokens), _ptr(val_codebooks), _ptr(tables),
                                               _ptr(codes_out), int(token_stride), int(head_stride), stream or None),
           "commvq_encode_values")


def commvq_em_workspace_bytes(n_subspaces: int, n_points: int, n_centres: int) -> int:
    n = c_size_t()
    _check(load_library().commvq_em_workspace_bytes(int(n_subspaces), int(n_points), int(n_centres), byref(n)),
           "commvq_em_workspace_bytes")
    return int(n.value)


def commvq_em_step(data, n_subspaces: int, n_points: int, n_centres: int, temperature: float, phi, workspace,
                   workspace_bytes: int, stream: int = 0) -> None:
    _check(load_library().commvq_em_step(_ptr(data), int(n_subspaces), int(n_points), int(n_centres), float(temperature),
                                         _ptr(phi), _ptr(workspace), int(workspace_bytes), stream or None),
           "commvq_em_step")


def commvq_em_shared_workspace_bytes(group: int, n_points: int, n_centres: int) -> int:
    n = c_size_t()
    _check(load_library().commvq_em_shared_workspace_bytes(int(group), int(n_points), int(n_centres), byref(n)),
           "commvq_em_shared_workspace_bytes")
    return int(n.value)


def commvq_em_step_shared(data, group: int, n_points: int, n_centres: int, temperature: float, phi, workspace,
                          workspace_bytes: int, stream: int = 0) -> None:
    _check(load_library().commvq_em_step_shared(_ptr(data), int(group), int(n_points), int(n_centres), float(temperature),
                                                _ptr(phi), _ptr(workspace), int(workspace_bytes), stream or None),
           "commvq_em_step_shared")


def commvq_stage_scores(handle, q, key_codes, key_codebooks, positions: Positions, workspace, workspace_bytes: int,
                        scores_out=None, stream: int = 0) -> None:
    _check(load_library().commvq_stage_scores(handle, _ptr(q), _ptr(key_codes), _ptr(key_codebooks), byref(positions),
                                              _ptr(workspace), int(workspace_bytes), _ptr(scores_out), stream or None),
           "commvq_stage_scores")


def commvq_stage_bins(handle, val_codes, positions: Positions, workspace, workspace_bytes: int, stream: int = 0) -> None:
    _check(load_library().commvq_stage_bins(handle, _ptr(val_codes), byref(positions), _ptr(workspace),
                                            int(workspace_bytes), stream or None), "commvq_stage_bins")


def commvq_stage_output(handle, val_codebooks, positions: Positions, out, workspace, workspace_bytes: int,
                        stream: int = 0) -> None:
    _check(load_library().commvq_stage_output(handle, _ptr(val_codebooks), byref(positions), _ptr(out),
                                              _ptr(workspace), int(workspace_bytes), stream or None),
           "commvq_stage_output")


def commvq_profile_enable(handle, every) -> None:
    """Stage events on every `every`-th call (True = every call, 0 / False = off)."""
    _check(load_library().commvq_profile_enable(handle, int(every)), "commvq_profile_enable")


def commvq_profile_read(handle):
    """Mean milliseconds of the [scores, bins, output] stages and the number of calls averaged."""
    ms = (c_float * 3)()
    n = c_int32()
    _check(load_library().commvq_profile_read(handle, ms, byref(n)), "commvq_profile_read")
    return [float(v) for v in ms], int(n.value)
