"""GPU-side test plumbing: torch allocates device memory and supplies the stream; the work itself is
done by libtpx through its C ABI."""
from __future__ import annotations

import torch

import paper_2312_05181_amd as tpx
from tests import helpers as H


def alloc(nbytes: int, fill=None) -> torch.Tensor:
    t = torch.empty(max(nbytes, 1), dtype=torch.uint8, device="cuda")[:nbytes]
    if fill is not None:
        t.fill_(fill)
    return t


def execute(plan, src_bufs, dst_bufs=None, workspace=None, poison=True):
    """Run plan on the current torch stream; returns (dst_bufs, workspace)."""
    if dst_bufs is None:
        dst_bufs = [alloc(plan.buffer_bytes(1, r), H.POISON if poison else None) for r in range(plan.num_buffers(1))]
    if workspace is None:
        workspace = alloc(plan.workspace_bytes())
        tpx.tpx_workspace_forget(workspace.data_ptr())   # fresh memory: whatever the library once copied to this address is gone
    stream = torch.cuda.current_stream().cuda_stream
    tpx.tpx_execute(plan, [b.data_ptr() if b.numel() else 0 for b in src_bufs],
                    [b.data_ptr() if b.numel() else 0 for b in dst_bufs], workspace.data_ptr(), stream)
    return dst_bufs, workspace
