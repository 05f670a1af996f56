"""The binarized VGG-small stack as a sequence of C-ABI calls (orchestration only).

Block order (every step runs in a HIP kernel of libbnn):
  conv -> int32 accumulators -> (2x2 max-pool on int32 when the block pools)
       -> fma(scale, acc, bias) -> fp32 map whose sign the next binarized layer takes.
Un-pooled blocks get the affine map from the GEMM store itself; pooled blocks from
the pool kernel.  The binarized FC flattens in NCHW order.
"""
from __future__ import annotations

from typing import Dict, List, Sequence

import numpy as np
import torch

from . import binding as B


class VggStack:
    def __init__(self, layers: Sequence, params: Sequence[Dict[str, np.ndarray]], batch: int, device="cuda:0"):
        self.layers = list(layers)
        self.batch = batch
        self.dev = torch.device(device)
        self.p: List[Dict[str, torch.Tensor]] = []
        ws_bytes = 16
        for L, prm in zip(self.layers, params):
            d = {k: torch.from_numpy(np.ascontiguousarray(v)).to(self.dev) for k, v in prm.items()}
            if L.kind == "bconv":
                d["wp"] = B.bnn_pack_conv_weight(d["w"])
                ws_bytes = max(ws_bytes, B.conv2d_workspace_bytes((batch, L.cin, L.hw, L.hw), 3, 3, (1, 1), (1, 1)))
            elif L.kind == "bfc":
                d["wp"] = B.bnn_encode(d["w"])
            self.p.append(d)
        self.ws = torch.empty(ws_bytes, dtype=torch.uint8, device=self.dev)
        # activation buffers, allocated once
        self.buf: List[Dict[str, torch.Tensor]] = []
        for L in self.layers:
            b: Dict[str, torch.Tensor] = {}
            if L.kind == "conv_f32":
                b["y"] = torch.empty((batch, L.cout, L.hw, L.hw), dtype=torch.float32, device=self.dev)
            elif L.kind == "bconv":
                if L.pool:
                    b["acc"] = torch.empty((batch, L.cout, L.hw, L.hw), dtype=torch.int32, device=self.dev)
                    b["y"] = torch.empty((batch, L.cout, L.hw // 2, L.hw // 2), dtype=torch.float32, device=self.dev)
                else:
                    b["y"] = torch.empty((batch, L.cout, L.hw, L.hw), dtype=torch.float32, device=self.dev)
            elif L.kind == "bfc":
                b["xp"] = torch.empty((batch, B.packed_words(L.cin)), dtype=torch.int64, device=self.dev)
                b["y"] = torch.empty((batch, L.cout), dtype=torch.float32, device=self.dev)
            elif L.kind == "fc_f32":
                b["y"] = torch.empty((batch, L.cout), dtype=torch.float32, device=self.dev)
            self.buf.append(b)
        torch.cuda.synchronize(self.dev)

    def forward(self, x: torch.Tensor, keep: bool = False):
        h = x
        acts = []
        for L, p, b in zip(self.layers, self.p, self.buf):
            if L.kind == "conv_f32":
                h = B.bnn_conv2d_f32(h, p["w"], (1, 1), (1, 1), p["scale"], p["bias"], out=b["y"])
            elif L.kind == "bconv":
                if L.pool:
                    B.bnn_conv2d(h, p["wp"], L.cout, 3, 3, (1, 1), (1, 1), want_int=True, workspace=self.ws,
                                 out_i32=b["acc"])
                    _, h = B.bnn_maxpool2x2(b["acc"], p["scale"], p["bias"], want_int=False, out_f32=b["y"])
                else:
                    _, h = B.bnn_conv2d(h, p["wp"], L.cout, 3, 3, (1, 1), (1, 1), p["scale"], p["bias"],
                                        want_int=False, workspace=self.ws, out_f32=b["y"])
            elif L.kind == "bfc":
                xp = B.bnn_encode(h.view(self.batch, -1), b["xp"])
                _, h = B.bnn_xnor_gemm_epilogue(xp, p["wp"], L.cin, p["scale"], p["bias"], B.CH_COL, out_y=b["y"])
            elif L.kind == "fc_f32":
                h = B.bnn_fc_f32(h.view(self.batch, -1), p["w"], p["bias"], sign_input=True, out=b["y"])
            else:
                raise ValueError(L.kind)
            if keep:
                acts.append(h.clone())
        return (h, acts) if keep else h


class VggStackFused:
    """The same stack with activations kept packed between layers (1 bit per activation):
    real-valued first layer with binarized output, binarized convolutions whose GEMM store
    does max-pool + affine + sign + pack, and the binarized FC on the packed map with its
    weight re-ordered to the (h, w, c) bit order.  Same arithmetic, same results."""

    def __init__(self, layers: Sequence, params: Sequence[Dict[str, np.ndarray]], batch: int, device="cuda:0"):
        self.layers = list(layers)
        self.batch = batch
        self.dev = torch.device(device)
        self.p: List[Dict[str, torch.Tensor]] = []
        self.buf: List[Dict[str, torch.Tensor]] = []
        hw_c = None  # (C, H, W) of the map entering the binarized FC
        for L, prm in zip(self.layers, params):
            d = {k: torch.from_numpy(np.ascontiguousarray(v)).to(self.dev) for k, v in prm.items()}
            b: Dict[str, torch.Tensor] = {}
            if L.kind == "conv_f32":
                b["yp"] = torch.empty((batch, L.hw, L.hw, B.packed_words(L.cout)), dtype=torch.int64, device=self.dev)
                hw_c = (L.cout, L.hw, L.hw)
            elif L.kind == "bconv":
                d["wp"] = B.bnn_pack_conv_weight(d["w"])
                o = L.hw // 2 if L.pool else L.hw
                b["yp"] = torch.empty((batch, o, o, B.packed_words(L.cout)), dtype=torch.int64, device=self.dev)
                hw_c = (L.cout, o, o)
            elif L.kind == "bfc":
                C, H, W = hw_c
                assert C * H * W == L.cin
                d["wp"] = B.bnn_pack_fc_weight_nhwc(d["w"], C, H, W)
                d["kbits"] = H * W * B.packed_words(C) * 64
                d["ktrue"] = L.cin
                b["y"] = torch.empty((batch, L.cout), dtype=torch.float32, device=self.dev)
            elif L.kind == "fc_f32":
                b["y"] = torch.empty((batch, L.cout), dtype=torch.float32, device=self.dev)
            self.p.append(d)
            self.buf.append(b)
        self._graph = None
        torch.cuda.synchronize(self.dev)

    def capture(self, x: torch.Tensor) -> None:
        """Record one forward pass reading x (its storage, not its present contents) into a HIP
        graph.  Every buffer of the pass is preallocated and the library neither allocates nor
        synchronises, so the graph holds exactly the pass's kernel launches; replay() re-issues
        them with one submission, which is what matters at batch sizes where a pass is shorter
        than its eight launches take to submit."""
        side = torch.cuda.Stream(device=self.dev)  # default priority
        side.wait_stream(torch.cuda.current_stream(self.dev))
        with torch.cuda.stream(side):
            self.forward(x)  # every code path has run once before capture
        torch.cuda.current_stream(self.dev).wait_stream(side)
        torch.cuda.synchronize(self.dev)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            self._graph_out = self.forward(x)
        self._graph = g

    def replay(self) -> torch.Tensor:
        """Re-run the captured pass on the current contents of the captured input."""
        if self._graph is None:
            raise RuntimeError("capture() first")
        self._graph.replay()
        return self._graph_out

    def forward(self, x: torch.Tensor, keep: bool = False):
        h = x
        acts = []
        for L, p, b in zip(self.layers, self.p, self.buf):
            if L.kind == "conv_f32":
                h = B.bnn_conv2d_f32_sign(h, p["w"], p["scale"], p["bias"], (1, 1), (1, 1), out=b["yp"])
            elif L.kind == "bconv":
                h = B.bnn_conv2d_packed(h, p["wp"], L.cin, L.cout, 3, 3, (1, 1), (1, 1), pool=2 if L.pool else 0,
                                        scale=p["scale"], bias=p["bias"], out="packed", out_buf=b["yp"])
            elif L.kind == "bfc":
                # pad bits are 0 in both operands, so the GEMM runs over whole words and the
                # formula takes the true K through the epilogue entry point's K argument
                rows = h.view(self.batch, -1)
                assert rows.shape[1] * 64 == p["kbits"] == p["ktrue"], "channel counts here are multiples of 64"
                _, h = B.bnn_xnor_gemm_epilogue(rows, p["wp"], p["ktrue"], p["scale"], p["bias"], B.CH_COL,
                                                out_y=b["y"])
            elif L.kind == "fc_f32":
                h = B.bnn_fc_f32(h.view(self.batch, -1), p["w"], p["bias"], sign_input=True, out=b["y"])
            else:
                raise ValueError(L.kind)
            if keep:
                acts.append(h.clone())
        return (h, acts) if keep else h

    def conv_launches(self):
        """One closure per binarized convolution that re-issues exactly that layer's launch on the
        buffers the last forward() left behind (for timing a launch in isolation)."""
        out = []
        prev = None
        for L, p, b in zip(self.layers, self.p, self.buf):
            if L.kind == "bconv":
                src = prev

                def call(L=L, p=p, b=b, src=src):
                    B.bnn_conv2d_packed(src, p["wp"], L.cin, L.cout, 3, 3, (1, 1), (1, 1), pool=2 if L.pool else 0,
                                        scale=p["scale"], bias=p["bias"], out="packed", out_buf=b["yp"])
                out.append(call)
            prev = b.get("yp", None)
        return out


class SplitBatch:
    """The fused stack on `parts` equal slices of the batch, each on its own HIP stream (default
    priority).  Images are independent, so the slices need no exchange; while one slice drains
    the tail of a kernel the other's next kernel fills the idle compute units."""

    def __init__(self, layers, params, batch: int, parts: int = 2, device="cuda:0"):
        assert batch % parts == 0
        self.parts = parts
        self.bs = batch // parts
        self.nets = [VggStackFused(layers, params, batch=self.bs, device=device) for _ in range(parts)]
        self.streams = [torch.cuda.Stream(device=device) for _ in range(parts)]

    def fork(self):
        """Make the slice streams wait for what has been enqueued on the current stream."""
        main = torch.cuda.current_stream()
        for st in self.streams:
            st.wait_stream(main)

    def join(self):
        """Make the current stream wait for everything enqueued on the slice streams."""
        main = torch.cuda.current_stream()
        for st in self.streams:
            main.wait_stream(st)

    def forward(self, x: torch.Tensor, sync: bool = True):
        """sync=False only enqueues the slices (successive batches then overlap freely; the caller
        forks before the first and joins after the last)."""
        if sync:
            self.fork()
        outs = []
        for i, (net, st) in enumerate(zip(self.nets, self.streams)):
            with torch.cuda.stream(st):
                outs.append(net.forward(x[i * self.bs:(i + 1) * self.bs]))
        if sync:
            self.join()
        return outs
