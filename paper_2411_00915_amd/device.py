"""Move a seeded workload into HBM in the layout the C ABI expects.

Pure marshalling: transposes to contraction-index-fastest storage, narrows to
the workload's dtype (exact: the generators only emit representable values),
packs all adapters of a layer into one buffer and builds the device pointer
tables.  torch is used for device memory only.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

from . import binding as B
from .workloads import Workload


@dataclass
class DeviceLayer:
    dtype: int
    x: torch.Tensor                 # [T, K]
    Wt: Optional[torch.Tensor]      # [N, K]
    At_buf: torch.Tensor            # all At_a back to back, each 256-byte aligned
    Bt_buf: torch.Tensor
    At_ptrs: torch.Tensor           # int64 [n_a] device addresses
    Bt_ptrs: torch.Tensor
    At_off: np.ndarray              # element offsets of each adapter in At_buf
    Bt_off: np.ndarray


def torch_dtype(w: Workload):
    return torch.float32 if w.dtype == "f32" else torch.bfloat16


def abi_dtype(w: Workload) -> int:
    return B.LORA_F32 if w.dtype == "f32" else B.LORA_BF16


def _pack(mats, tdt, device, align_elems):
    offs, total = [], 0
    for m in mats:
        offs.append(total)
        total += (m.size + align_elems - 1) // align_elems * align_elems
    buf = torch.empty(max(total, align_elems), dtype=tdt, device=device)
    for off, m in zip(offs, mats):
        if m.size:
            buf[off:off + m.size].copy_(torch.from_numpy(np.ascontiguousarray(m)).reshape(-1).to(tdt))
    base = buf.data_ptr()
    es = buf.element_size()
    ptrs = torch.tensor([base + o * es for o in offs], dtype=torch.int64, device=device)
    return buf, ptrs, np.asarray(offs, dtype=np.int64)


def to_device(w: Workload, device="cuda:0", with_w: bool = True) -> DeviceLayer:
    tdt = torch_dtype(w)
    x = torch.from_numpy(w.x).to(device=device, dtype=tdt).contiguous()
    Wt = None
    if with_w and w.W is not None:
        Wt = torch.from_numpy(np.ascontiguousarray(w.W.T)).to(device=device, dtype=tdt).contiguous()
    align = 256 // (4 if w.dtype == "f32" else 2)
    At_buf, At_ptrs, At_off = _pack([a.T for a in w.A], tdt, device, align)   # [r, K]
    Bt_buf, Bt_ptrs, Bt_off = _pack([b.T for b in w.B], tdt, device, align)   # [N, r]
    return DeviceLayer(abi_dtype(w), x, Wt, At_buf, Bt_buf, At_ptrs, Bt_ptrs, At_off, Bt_off)


def make_plan(w: Workload, variant: int = B.LORA_VARIANT_AUTO, tuning=None, merged_adapter=None) -> B.Plan:
    return B.lora_plan(w.T, w.seg_indptr, w.seg_adapter, w.adapter_rank, w.adapter_scale,
                       w.K, w.N, abi_dtype(w), variant, tuning, merged_adapter)
