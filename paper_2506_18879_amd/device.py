"""Device-side plumbing around libcommvq: torch tensors for memory, nothing of the method itself."""
from __future__ import annotations

from typing import Optional

import numpy as np

from . import binding as B


def _torch():
    import torch

    if not torch.cuda.is_available():
        raise RuntimeError("libcommvq needs a GPU (gfx950); no CPU fallback exists")
    return torch


def to_device(arr: np.ndarray, bf16: bool = False):
    """Upload a numpy array; uint16 arrays flagged bf16 become torch.bfloat16 views of the same bits."""
    torch = _torch()
    if bf16:
        assert arr.dtype == np.uint16
        return torch.from_numpy(np.ascontiguousarray(arr).view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(arr)).cuda()


class DeviceWorkload:
    """A synth.Workload resident in HBM (one copy of every input buffer)."""

    def __init__(self, w):
        bf = w.dtype == "bf16"
        self.w = w
        self.q = to_device(w.q, bf)
        self.key_codes = to_device(w.key_codes)
        self.val_codes = to_device(w.val_codes)
        self.key_codebooks = to_device(w.key_codebooks, bf)
        self.val_codebooks = to_device(w.val_codebooks, bf)
        self.cu_seqlens = to_device(w.cu_seqlens)
        self.q_pos = to_device(w.q_pos)
        self.key_pos = None if w.key_pos is None else to_device(w.key_pos)
        self.positions = B.make_positions(w.B, self.cu_seqlens, self.q_pos, self.key_pos, w.total_tokens, w.max_seqlen)


class DecodeAttention:
    """Owns a libcommvq handle, a workspace and an output buffer for one batch shape."""

    def __init__(self, w, max_position: Optional[int] = None, softmax_scale: float = 0.0, position_free: bool = False,
                 q_dtype: Optional[str] = None):
        torch = _torch()
        dt = B.COMMVQ_BF16 if w.dtype == "bf16" else B.COMMVQ_F32
        qdt = dt if q_dtype is None else (B.COMMVQ_BF16 if q_dtype == "bf16" else B.COMMVQ_F32)
        if max_position is None:
            max_position = max(int(w.q_pos.max()), w.max_seqlen, 0 if w.key_pos is None else int(w.key_pos.max()))
        paired = getattr(w, "key_format", "indexed") == "paired"
        vbin = getattr(w, "val_format", "indexed") == "binary"
        self.cfg = B.Config(w.Hq, w.Hkv, w.d, 16 if paired else w.Mk, 16 if vbin else w.Mv, w.K, qdt, dt, float(w.rope_base),
                            float(softmax_scale), int(max_position),
                            B.COMMVQ_KEYS_PAIRED if paired else B.COMMVQ_KEYS_INDEXED, w.key_levels if paired else 0,
                            1 if position_free else 0,
                            B.COMMVQ_VALUES_BINARY if vbin else B.COMMVQ_VALUES_INDEXED, w.val_bits if vbin else 0)
        self.handle = B.commvq_create(self.cfg)
        self.plan = B.commvq_plan_query(self.handle, w.B, w.total_tokens, w.max_seqlen)
        self.workspace_bytes = B.commvq_workspace_bytes(self.handle, w.B, w.total_tokens, w.max_seqlen)
        self.workspace = torch.empty(self.workspace_bytes, dtype=torch.uint8, device="cuda")
        assert self.workspace.data_ptr() % 256 == 0
        self.out = torch.empty((w.B, w.Hq, w.d), dtype=torch.float32, device="cuda")
        self.n_scores = w.total_tokens * w.Hq
        self._packed = {}

    def pack_key_codebooks(self, dw: DeviceWorkload):
        """One-time re-layout of dw's (static) key codebooks; later calls with dw skip the per-call re-layout."""
        torch = _torch()
        buf = torch.empty(B.commvq_packed_key_codebook_bytes(self.handle), dtype=torch.uint8, device="cuda")
        B.commvq_pack_key_codebooks(self.handle, dw.key_codebooks, buf, self.stream_ptr())
        self._packed[dw.key_codebooks.data_ptr()] = (buf, dw.key_codebooks)  # keep both alive while registered

    def pack_value_codebooks(self, dw: DeviceWorkload):
        """One-time re-layout of dw's (static) value codebooks for the batched output kernel."""
        torch = _torch()
        buf = torch.empty(B.commvq_packed_value_codebook_bytes(self.handle), dtype=torch.uint8, device="cuda")
        B.commvq_pack_value_codebooks(self.handle, dw.val_codebooks, buf, self.stream_ptr())
        self._packed[("v", dw.val_codebooks.data_ptr())] = (buf, dw.val_codebooks)

    def close(self):
        if self.handle is not None:
            B.commvq_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def stream_ptr(self) -> int:
        return int(_torch().cuda.current_stream().cuda_stream)

    def __call__(self, dw: DeviceWorkload, out=None):
        """Enqueue commvq_decode_attn on torch's current stream; returns the (asynchronous) output tensor."""
        out = self.out if out is None else out
        B.commvq_decode_attn(self.handle, dw.q, dw.key_codes, dw.val_codes, dw.key_codebooks, dw.val_codebooks,
                             dw.positions, out, self.workspace, self.workspace_bytes, self.stream_ptr())
        return out

    def scores(self, dw: DeviceWorkload):
        """Run the score stage alone and return the logits [T*Hq] (ragged (b, h, i) layout)."""
        torch = _torch()
        s = torch.empty(self.n_scores, dtype=torch.float32, device="cuda")
        B.commvq_stage_scores(self.handle, dw.q, dw.key_codes, dw.key_codebooks, dw.positions, self.workspace,
                              self.workspace_bytes, s, self.stream_ptr())
        return s

    def staged(self, dw: DeviceWorkload):
        """scores -> bins -> output through the three stage entry points."""
        st = self.stream_ptr()
        B.commvq_stage_scores(self.handle, dw.q, dw.key_codes, dw.key_codebooks, dw.positions, self.workspace,
                              self.workspace_bytes, None, st)
        B.commvq_stage_bins(self.handle, dw.val_codes, dw.positions, self.workspace, self.workspace_bytes, st)
        B.commvq_stage_output(self.handle, dw.val_codebooks, dw.positions, self.out, self.workspace,
                              self.workspace_bytes, st)
        return self.out
