"""Host arrays of a synthetic workload (workloads.py) -> device tensors, as the C ABI takes them.
Copies only; used by the benchmark, the smoke check and the GPU tests."""
from __future__ import annotations

import numpy as np
import torch


def bf16_tensor(bits: np.ndarray, device="cuda") -> torch.Tensor:
    """uint16 bf16 bit patterns -> a torch.bfloat16 tensor with the same bits."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device).view(torch.bfloat16)


def attention_device_inputs(inp, device="cuda"):
    return dict(
        q=bf16_tensor(inp.q, device),
        k_pages=bf16_tensor(inp.k_pages, device),
        v_pages=None if inp.v_pages is None else bf16_tensor(inp.v_pages, device),
        block_table=torch.from_numpy(inp.block_table).to(device),
        ctx_len=torch.from_numpy(inp.ctx_len).to(device),
        tree_mask=None if inp.tree_mask is None else torch.from_numpy(inp.tree_mask.view(np.int64)).to(device),
    )


def accept_device_inputs(inp, device="cuda"):
    return dict(
        logits=torch.from_numpy(inp.logits).to(device),
        draft_tokens=torch.from_numpy(inp.draft_tokens).to(device),
        tree_parent=None if inp.tree_parent is None else torch.from_numpy(inp.tree_parent).to(device),
    )
