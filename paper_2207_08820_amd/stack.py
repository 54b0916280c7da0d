"""Layer-list harness: chains packed convolutions on the GPU through the C ABI.

A stand-in for the graph runtime that the paper's product has around its kernels (Section VI):
just enough to run a list of quantized conv layers back to back.  Each layer is
pack (activations) -> dlrt_bitserial_conv2d -> dlrt_epilogue_f32 with requantization, and the
uint8 result feeds the layers that name it as their source.  All arithmetic happens in the
library's kernels; this module only owns the buffers and the call order.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import torch

from . import binding


@dataclass
class PackedLayer:
    spec: object                 # inputs.ConvLayer
    wp: torch.Tensor             # packed weights [Co, wbits, KH*KW*Cw]
    scale: torch.Tensor          # fp32 [Co]
    bias: torch.Tensor | None    # fp32 [Co]
    # buffers, allocated once so that the timed chain allocates nothing
    xp: torch.Tensor = field(default=None)
    acc: torch.Tensor = field(default=None)
    q: torch.Tensor = field(default=None)


class ConvStack:
    def __init__(self, layers, weights_i8, scales, biases, abits: int, wbits: int, enc_w: int, device="cuda:0"):
        self.abits, self.wbits, self.enc_w = abits, wbits, enc_w
        self.device = torch.device(device)
        self.layers = []
        for L, w, s, b in zip(layers, weights_i8, scales, biases):
            wt = torch.as_tensor(w, device=self.device)
            wp = binding.dlrt_pack_conv_weights(wt, wbits, enc_w)
            pl = PackedLayer(L, wp, torch.as_tensor(s, device=self.device),
                             None if b is None else torch.as_tensor(b, device=self.device))
            Cw = (L.Ci + 31) // 32
            pl.xp = torch.empty((L.H * L.W, abits, Cw), dtype=torch.int32, device=self.device)
            pl.acc = torch.empty((1, L.Ho, L.Wo, L.Co), dtype=torch.int32, device=self.device)
            pl.q = torch.empty((1, L.Ho, L.Wo, L.Co), dtype=torch.uint8, device=self.device)
            self.layers.append(pl)

    def run_layer(self, i: int, x_u8: torch.Tensor):
        """x_u8: NHWC uint8 activations of layer i.  Fills the layer's acc and q buffers."""
        pl = self.layers[i]
        L = pl.spec
        binding.dlrt_pack_bitplanes(x_u8, self.abits, binding.UNSIGNED, out=pl.xp)
        binding.dlrt_bitserial_conv2d(pl.xp, pl.wp, 1, L.H, L.W, L.Ci, L.Co, L.k, L.k, (L.stride, L.stride),
                                      (L.pad, L.pad), self.abits, self.wbits, binding.UNSIGNED, self.enc_w,
                                      out=pl.acc)
        binding.dlrt_epilogue_f32(pl.acc, pl.scale, pl.bias, want_f32=False, qbits=self.abits, out_q=pl.q)
        return pl.acc, pl.q

    def run(self, x0_u8: torch.Tensor):
        """Enqueue the whole chain; returns nothing (results stay in the per-layer buffers)."""
        for i, pl in enumerate(self.layers):
            src = pl.spec.src
            self.run_layer(i, x0_u8 if src < 0 else self.layers[src].q)
