"""Stand-in for the expert FFNs on the device (harness code: torch ops, outside the library, untimed).

The workloads define the expert as ``Yexp[row] = round_to_storage(f32(window[row]) * scale[expert of row])``.
The benchmark and the smoke check need that on the GPU between dispatch and combine; the parity tests use
the oracle's own stand-in instead.  Nothing of the dispatch / combine path is computed here.
"""
from __future__ import annotations


def standin_expert(layer, scale) -> None:
    """Fills ``layer.expert_out`` from ``layer.window``: every row of an expert's sub-block (this source rank's
    rows, as the plan tables describe them) times that expert's scalar; rows outside keep scale 0."""
    import torch
    E = layer.shape.E
    rows = layer.rows
    if rows == 0 or layer.shape.T == 0:
        return
    off = layer.plan.expert_offset[:E].long()
    cnt = layer.plan.expert_count.long()
    row_scale = torch.zeros(rows, dtype=torch.float32, device=layer.window.device)
    ids = torch.repeat_interleave(torch.arange(E, device=off.device), cnt)
    first = torch.cumsum(cnt, 0) - cnt
    pos = torch.repeat_interleave(off, cnt) + (torch.arange(ids.numel(), device=off.device)
                                               - torch.repeat_interleave(first, cnt))
    keep = pos < rows
    row_scale[pos[keep]] = scale[ids[keep]]
    step = max(1, (1 << 27) // layer.shape.H)
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        layer.expert_out[r0:r1] = (layer.window[r0:r1].float() * row_scale[r0:r1, None]).to(layer.torch_dtype)
