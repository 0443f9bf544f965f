"""Head-pipelined K/V staging on one GPU (paper section 4.3: keys and values
are gathered along the head dimension and the attention of the heads already
gathered overlaps the transfers of the next ones).

Stream choreography only.  A copy stream stands in for the arrival of the
gathered K/V: it moves one window of KV heads after the other from a source
buffer into the staging buffer the attention reads; the compute stream waits
for each window's event and runs mmattn_fwd_heads on it.  The share's tile
plan is built by the first call and reused by the others.

A launch over one or two KV heads has few work items and leaves CUs idle
towards its end; with `compute_streams` > 1 the windows are dealt round-robin
to that many streams (each with its own workspace and plan), so the next
window's kernel fills the CUs the previous one no longer uses -- the
multiple-stream execution of the paper's appendix on context parallelism.
"""
from __future__ import annotations

from typing import Optional

import torch

from . import binding as mb


def fwd_head_pipelined(q_loc: torch.Tensor, k_src: torch.Tensor, v_src: torch.Tensor,
                       bits: torch.Tensor, blocks: torch.Tensor, block: int,
                       heads_per_stage: int = 1, k_stage: Optional[torch.Tensor] = None,
                       v_stage: Optional[torch.Tensor] = None,
                       copy_stream: Optional[torch.cuda.Stream] = None,
                       ws: Optional[torch.Tensor] = None, out=None, scale: Optional[float] = None,
                       compute_streams: int = 1, side_streams=None, side_ws=None):
    """Forward for one rank share with K/V arriving window by window.

    k_src, v_src [S,Hkv,D]: where the gathered heads come from; k_stage,
    v_stage: the buffers the kernels read (allocated if not given).  Returns
    (o_loc, lse) on the current stream, like binding.fwd.  compute_streams > 1
    adds side streams (side_streams / side_ws: reuse these instead of creating
    compute_streams - 1 streams and workspaces per call)."""
    n_loc, Hq, D = q_loc.shape
    S, Hkv, _ = k_src.shape
    dev = q_loc.device
    if heads_per_stage < 1 or Hkv % heads_per_stage:
        raise ValueError("heads_per_stage must divide Hkv")
    k_stage = torch.empty_like(k_src) if k_stage is None else k_stage
    v_stage = torch.empty_like(v_src) if v_stage is None else v_stage
    if out is None:
        out = (torch.empty_like(q_loc), torch.empty((Hq, n_loc), dtype=torch.float32, device=dev))
    if ws is None:
        ws = torch.empty(max(mb.workspace_size(mb.OP_FWD_HEADS, S, blocks.numel(), block, Hq, Hkv, D), 256),
                         dtype=torch.uint8, device=dev)
    compute = torch.cuda.current_stream()
    copy = torch.cuda.Stream(device=dev) if copy_stream is None else copy_stream
    copy.wait_stream(compute)                       # sources and staging buffers are ready
    arrived = []
    with torch.cuda.stream(copy):
        for g0 in range(0, Hkv, heads_per_stage):
            g1 = g0 + heads_per_stage
            k_stage[:, g0:g1].copy_(k_src[:, g0:g1], non_blocking=True)
            v_stage[:, g0:g1].copy_(v_src[:, g0:g1], non_blocking=True)
            ev = torch.cuda.Event()
            ev.record(copy)
            arrived.append(ev)
    n_side = max(0, compute_streams - 1)
    if side_streams is None:
        side_streams = [torch.cuda.Stream(device=dev) for _ in range(n_side)]
    if side_ws is None:
        side_ws = [torch.empty_like(ws) for _ in range(n_side)]
    lanes = [(compute, ws)] + list(zip(side_streams[:n_side], side_ws[:n_side]))
    for st, _ in lanes[1:]:
        st.wait_stream(compute)                     # q_loc, bits, blocks, outputs are ready
    used = [False] * len(lanes)
    for i, g0 in enumerate(range(0, Hkv, heads_per_stage)):
        j = i % len(lanes)
        st, w = lanes[j]
        st.wait_event(arrived[i])
        mb.fwd_heads(q_loc, k_stage, v_stage, bits, blocks, block, g0, heads_per_stage,
                     plan_ready=used[j], out=out, ws=w, scale=scale, stream=st)
        used[j] = True
    for st, w in lanes[1:]:
        compute.wait_stream(st)
        for t in (q_loc, bits, blocks, k_stage, v_stage, out[0], out[1], w):
            t.record_stream(st)
    for t in (k_src, v_src, k_stage, v_stage):
        t.record_stream(copy)
    return out
