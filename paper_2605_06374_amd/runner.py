"""Device-side harness: puts a synthetic workload into HBM (torch tensors), calls the C-ABI
entry points, and copies results back.  Plumbing only; no attention arithmetic."""
from __future__ import annotations

import numpy as np
import torch

from . import binding
from .workloads import Workload, bf16_bits_to_f32


def _to_device_bf16(bits: np.ndarray, device) -> torch.Tensor:
    t = torch.from_numpy(bits.view(np.int16).copy()).to(device)
    return t.view(torch.bfloat16)


def _to_host_f64(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        bits = t.view(torch.int16).cpu().numpy().view(np.uint16)
        return bf16_bits_to_f32(bits).astype(np.float64)
    return t.cpu().numpy().astype(np.float64)


class DeviceProblem:
    """One packed microbatch resident on the GPU with its outputs and workspace."""

    def __init__(self, w: Workload, device="cuda:0", values=None, flags=0):
        self.w = w
        self.device = torch.device(device)
        vals = values if values is not None else w.values()
        self.q = _to_device_bf16(vals["q"], self.device)
        self.k = _to_device_bf16(vals["k"], self.device)
        self.v = _to_device_bf16(vals["v"], self.device)
        self.d_o = _to_device_bf16(vals["do"], self.device)
        cu = w.cu_seqlens
        self.cu = torch.from_numpy(cu.copy()).to(self.device)
        self.params = binding.make_params(w.n_tokens, len(cu) - 1, w.n_q_heads, w.n_kv_heads,
                                          w.head_dim, w.softmax_scale, flags)
        self.o = torch.empty_like(self.q)
        self.lse = torch.empty((w.n_q_heads, w.n_tokens), dtype=torch.float32, device=self.device)
        self.dq = torch.empty_like(self.q)
        self.dk = torch.empty_like(self.k)
        self.dv = torch.empty_like(self.v)
        nbytes = binding.varlen_attn_workspace_bytes(self.params)
        if nbytes == 0:
            raise ValueError("invalid parameters")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)

    def poison_outputs(self):
        for t in (self.o, self.dq, self.dk, self.dv):
            t.view(torch.int16).fill_(0x7FC0)   # bf16 NaN
        self.lse.fill_(float("nan"))

    def plan(self, stream=None):
        binding.check(binding.varlen_attn_plan(self.params, self.cu, self.workspace, stream=stream))

    def forward(self, stream=None, reuse_plan=False):
        p = self.params
        if reuse_plan:
            p = binding.make_params(p.total_tokens, p.num_docs, p.num_q_heads, p.num_kv_heads,
                                    p.head_dim, p.softmax_scale, p.flags | binding.FLAG_REUSE_PLAN)
        binding.check(binding.varlen_attn_fwd(p, self.q, self.k, self.v, self.cu, self.o,
                                              self.lse, self.workspace, stream=stream))

    def backward(self, stream=None, reuse_plan=False):
        p = self.params
        if reuse_plan:
            p = binding.make_params(p.total_tokens, p.num_docs, p.num_q_heads, p.num_kv_heads,
                                    p.head_dim, p.softmax_scale, p.flags | binding.FLAG_REUSE_PLAN)
        binding.check(binding.varlen_attn_bwd(p, self.q, self.k, self.v, self.o, self.lse, self.d_o,
                                              self.cu, self.dq, self.dk, self.dv, self.workspace,
                                              stream=stream))

    def read_plan(self):
        """Header, unit lists and combine lists as numpy arrays (synchronises).
        Units: columns row0, doc_start, doc_end, step_begin, step_end, slot, cost, reserved;
        combine items: row0, doc_end, slot0, n_chunks."""
        import ctypes
        torch.cuda.synchronize(self.device)
        L = binding.varlen_attn_workspace_regions(self.params)
        nbytes = max(L.col_combine_offset + 16 * L.max_combine, 64)
        raw = self.workspace[:nbytes].cpu().numpy()
        hdr = binding.PlanHeader.from_buffer_copy(raw[:ctypes.sizeof(binding.PlanHeader)].tobytes())

        def table(off, n, width):
            return np.frombuffer(raw[off:off + 4 * width * n].tobytes(), dtype=np.int32).reshape(-1, width)

        return {"header": hdr,
                "row_units": table(L.row_units_offset, hdr.n_row_units, 8),
                "col_units": table(L.col_units_offset, hdr.n_col_units, 8),
                "row_combine": table(L.row_combine_offset, hdr.n_row_combine, 4),
                "col_combine": table(L.col_combine_offset, hdr.n_col_combine, 4),
                "layout": L}

    def results(self):
        torch.cuda.synchronize(self.device)
        return {"o": _to_host_f64(self.o), "lse": _to_host_f64(self.lse),
                "dq": _to_host_f64(self.dq), "dk": _to_host_f64(self.dk),
                "dv": _to_host_f64(self.dv)}

    def result_bits(self):
        torch.cuda.synchronize(self.device)
        out = {n: getattr(self, n).view(torch.int16).cpu().numpy().view(np.uint16)
               for n in ("o", "dq", "dk", "dv")}
        out["lse"] = self.lse.cpu().numpy().view(np.uint32)
        return out
