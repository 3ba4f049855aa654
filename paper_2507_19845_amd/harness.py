"""Schedules of stage calls over micro-batches (host-side sequencing only).

Two schedules, both built from the C entry points:
  * coupled   -- for each micro-batch: gpt_stage_fwd then gpt_stage_bwd on one stream;
  * decoupled -- every micro-batch's forward first on a forward stream, each into
    its own stash slot, then every backward on a separate backward stream that
    waits on an event recorded after the last forward: the breadth-first order
    of the paper's section 5.2 run as the two decoupled phases of section 4.1.
"""
from __future__ import annotations

import json
from typing import Dict, List, Optional, Sequence

import torch

from . import binding as B


class StageRunner:
    def __init__(self, bufs: B.StageBuffers):
        self.b = bufs
        self.fwd_stream = torch.cuda.Stream()
        self.bwd_stream = torch.cuda.Stream()
        self.event = torch.cuda.Event()
        # torch creates the underlying hipEvent lazily, on the first record
        self.event.record(self.fwd_stream)

    def coupled(self, xs: Sequence[torch.Tensor], dys: Sequence[torch.Tensor],
                ys: Sequence[torch.Tensor], dxs: Sequence[torch.Tensor],
                stream: Optional[torch.cuda.Stream] = None) -> None:
        b = self.b
        p = b.params()
        for x, dy, y, dx in zip(xs, dys, ys, dxs):
            B.gpt_stage_fwd(p, x, b.stash[0], y, stream)
            B.gpt_stage_bwd(p, b.stash[0], dy, dx, b.dparams, stream)

    def decoupled(self, xs, dys, ys, dxs, split_wgrad: bool = False) -> None:
        """All forwards on fwd_stream, then all backwards on bwd_stream.  The
        caller's current stream is joined on both sides.  split_wgrad: the backward
        calls run the data phase only and one weight phase over all micro-batches
        follows on bwd_stream (section 5.2: a chunk's gradients are due once all its
        micro-batches have passed)."""
        b = self.b
        assert len(b.stash) >= len(xs), "one stash slot per in-flight micro-batch"
        cur = torch.cuda.current_stream()
        self.fwd_stream.wait_stream(cur)
        n = len(xs)
        p = b.params()
        for i in range(n):
            B.gpt_stage_fwd_only(p, xs[i], b.stash[i], ys[i],
                                 self.fwd_stream, self.event if i == n - 1 else None)
        if split_wgrad:
            b.alloc_grad_stash(n)
            for i in range(n):
                B.gpt_stage_bwd_data_only(p, b.stash[i], dys[i], dxs[i], b.dparams, b.grad_stash[i],
                                          self.bwd_stream, self.event if i == 0 else None)
            B.gpt_stage_wgrad_flush(p, b.stash[:n], b.grad_stash[:n], b.dparams, self.bwd_stream)
        else:
            for i in range(n):
                B.gpt_stage_bwd_only(p, b.stash[i], dys[i], dxs[i],
                                     b.dparams, self.bwd_stream, self.event if i == 0 else None)
        cur.wait_stream(self.bwd_stream)


_LINEAR = ("qkv", "out_proj", "fc1", "fc2")


def chrome_trace(records: List[Dict], path: Optional[str] = None) -> Dict:
    """Operator records of the tracer as a Chrome Tracing / Perfetto JSON object
    (the trace format of the paper's section 3.2): one complete event ("ph": "X") per
    operator, forward and backward phases as two thread rows, the operator's metadata
    in "args".  Written to `path` when given."""
    events = []
    for r in records:
        name = r["op"]
        if name.startswith("gemm") or name == "bias_grad":
            name += "." + _LINEAR[r["sub"]]
        elif name.startswith("layernorm"):
            name += ".%d" % (r["sub"] + 1)
        args = {"layer": r["layer"], "flops": r["flops"], "bytes": r["bytes"]}
        if r["dur_ms"] > 0:
            args["TFLOP/s"] = r["flops"] / r["dur_ms"] / 1e9
            args["GB/s"] = r["bytes"] / r["dur_ms"] / 1e6
        events.append({"name": name, "cat": "fwd" if r["phase"] == 0 else "bwd", "ph": "X",
                       "ts": r["start_ms"] * 1e3, "dur": r["dur_ms"] * 1e3, "pid": 0,
                       "tid": r["phase"], "args": args})
    doc = {"traceEvents": events, "displayTimeUnit": "ms"}
    if path:
        with open(path, "w") as f:
            json.dump(doc, f)
    return doc
