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
                _, h = B.bnn_xnor_gemm_epilogue(xp, p["wp"], L.cin, p["scale"], p["bias"], B.CH_COL)
            elif L.kind == "fc_f32":
                h = B.bnn_fc_f32(h.view(self.batch, -1), p["w"], p["bias"], sign_input=True, out=b["y"])
            else:
                raise ValueError(L.kind)
            if keep:
                acts.append(h.clone())
        return (h, acts) if keep else h
