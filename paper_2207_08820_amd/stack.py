"""Layer-list harness: chains packed convolutions on the GPU through the C ABI.

A stand-in for the graph runtime that the paper's product has around its kernels (Section VI):
just enough to run a list of quantized conv layers back to back.  Two ways to run a layer:

* ``fused=True`` (default): one ``dlrt_bitserial_conv2d_fused`` launch per layer, which writes the
  NEXT layer's packed activations directly (conv -> scale/bias -> requant -> bitplanes); only the
  stack input goes through ``dlrt_pack_bitplanes``.
* ``fused=False``: ``dlrt_pack_bitplanes`` -> ``dlrt_bitserial_conv2d`` -> ``dlrt_epilogue_f32`` per layer.

``capture()`` records the chain once into a HIP graph so that replays cost one launch from the host.
All arithmetic happens in the library's kernels; this module only owns the buffers and the call order.
"""
from __future__ import annotations

from dataclasses import dataclass

import torch

from . import binding


@dataclass
class PackedLayer:
    spec: object                 # inputs.ConvLayer
    wp: torch.Tensor             # packed weights [Co, wbits, KH*KW*Cw]
    scale: torch.Tensor          # fp32 [Co]
    bias: torch.Tensor | None    # fp32 [Co]
    # buffers, allocated once so that the timed chain allocates nothing
    xp: torch.Tensor = None      # unfused: this layer's packed input
    acc: torch.Tensor = None     # int32 accumulators (unfused, or fused with keep_outputs)
    q: torch.Tensor = None       # uint8 requantized output (unfused, or fused with keep_outputs)
    out_packed: torch.Tensor = None  # fused: packed requantized output = input of the consumers


def _per_layer(v, n):
    return list(v) if isinstance(v, (list, tuple)) else [v] * n


class ConvStack:
    """abits / wbits / enc_w are one value for the whole stack or one per layer (mixed precision, as in
    the paper's per-layer precision choice).  A layer's output is requantized to the activation width
    of the layers that read it (they must agree); a layer nobody reads keeps its own width."""

    def __init__(self, layers, weights_i8, scales, biases, abits, wbits, enc_w, device="cuda:0",
                 fused: bool = True, keep_outputs: bool = True, pair_launches: bool = True, batch: int = 1):
        n = len(layers)
        self.pair_launches = pair_launches
        self.batch = B = int(batch)  # images per pass; the layer list describes one image
        self.abits, self.wbits, self.enc_w = _per_layer(abits, n), _per_layer(wbits, n), _per_layer(enc_w, n)
        self.qbits = list(self.abits)
        for i in range(n):
            readers = {self.abits[j] for j in range(n) if layers[j].src == i}
            if len(readers) > 1:
                raise ValueError(f"layers reading layer {i} disagree on its activation width: {readers}")
            if readers:
                self.qbits[i] = readers.pop()
        self.fused, self.keep = fused, keep_outputs
        self.device = torch.device(device)
        self.layers = []
        self.graph = None
        for i, (L, w, s, b) in enumerate(zip(layers, weights_i8, scales, biases)):
            wt = torch.as_tensor(w, device=self.device)
            wp = binding.dlrt_pack_conv_weights(wt, self.wbits[i], self.enc_w[i])
            pl = PackedLayer(L, wp, torch.as_tensor(s, device=self.device),
                             None if b is None else torch.as_tensor(b, device=self.device))
            if fused:
                pl.out_packed = torch.empty((B * L.Ho * L.Wo, self.qbits[i], (L.Co + 31) // 32), dtype=torch.int32,
                                            device=self.device)
            else:
                pl.xp = torch.empty((B * L.H * L.W, self.abits[i], (L.Ci + 31) // 32), dtype=torch.int32,
                                    device=self.device)
            if keep_outputs or not fused:
                pl.acc = torch.empty((B, L.Ho, L.Wo, L.Co), dtype=torch.int32, device=self.device)
                pl.q = torch.empty((B, L.Ho, L.Wo, L.Co), dtype=torch.uint8, device=self.device)
            self.layers.append(pl)
        L0 = layers[0]
        self.x0_packed = torch.empty((B * L0.H * L0.W, self.abits[0], (L0.Ci + 31) // 32), dtype=torch.int32,
                                     device=self.device)

    # ---- unfused: three launches per layer ----
    def run_layer(self, i: int, x_u8: torch.Tensor):
        pl = self.layers[i]
        L = pl.spec
        binding.dlrt_pack_bitplanes(x_u8, self.abits[i], binding.UNSIGNED, out=pl.xp)
        binding.dlrt_bitserial_conv2d(pl.xp, pl.wp, self.batch, L.H, L.W, L.Ci, L.Co, L.k, L.k, (L.stride, L.stride),
                                      (L.pad, L.pad), self.abits[i], self.wbits[i], binding.UNSIGNED, self.enc_w[i],
                                      out=pl.acc)
        binding.dlrt_epilogue_f32(pl.acc, pl.scale, pl.bias, want_f32=False, qbits=self.qbits[i], out_q=pl.q)

    # ---- fused: one launch per layer ----
    def run_layer_fused(self, i: int, x_packed: torch.Tensor, tile_rows: int = 0, ksplit: int = 0):
        pl = self.layers[i]
        L = pl.spec
        binding.dlrt_bitserial_conv2d_fused(pl.xp if x_packed is None else x_packed, pl.wp, pl.scale, pl.bias,
                                            self.batch, L.H, L.W, L.Ci, L.Co, L.k, L.k, (L.stride, L.stride),
                                            (L.pad, L.pad), self.abits[i], self.wbits[i], binding.UNSIGNED, self.enc_w[i],
                                            qbits=self.qbits[i],
                                            out_acc=pl.acc if self.keep else None, out_q=pl.q if self.keep else None,
                                            out_packed=pl.out_packed, tile_rows=tile_rows, ksplit=ksplit)

    def problem(self, i: int):
        pl = self.layers[i]
        L = pl.spec
        return binding.conv_problem(self.layer_input(i), pl.wp, pl.scale, pl.bias, self.batch, L.H, L.W, L.Ci, L.Co, L.k, L.k,
                                    (L.stride, L.stride), (L.pad, L.pad), qbits=self.qbits[i],
                                    out_acc=pl.acc if self.keep else None, out_q=pl.q if self.keep else None,
                                    out_packed=pl.out_packed)

    def pairs(self):
        """Launch schedule of the fused chain: a layer goes out together with a later layer that reads the
        same input and has the same bit widths (a stride-2 conv with the 1x1 conv beside it, two 1x1 convs
        on one tensor); the later one simply runs early, its readers still come after it.  Everything else
        is a launch of its own."""
        plan, done, n = [], set(), len(self.layers)
        for i in range(n):
            if i in done:
                continue
            key = (self.layers[i].spec.src, self.abits[i], self.wbits[i], self.enc_w[i])
            mate = next((j for j in range(i + 1, n) if j not in done and
                         (self.layers[j].spec.src, self.abits[j], self.wbits[j], self.enc_w[j]) == key), None)
            if mate is None:
                plan.append((i,))
            else:
                plan.append((i, mate))
                done.add(mate)
        return plan

    def layer_input(self, i: int):
        src = self.layers[i].spec.src
        return self.x0_packed if src < 0 else self.layers[src].out_packed

    def run(self, x0_u8: torch.Tensor):
        """Enqueue the whole chain; results stay in the per-layer buffers."""
        if self.fused:
            # one stream on purpose: forking the side-branch 1x1 convs onto a second stream was
            # measured slower (0.170 against 0.128 ms), the cross-queue waits cost more than they hide
            binding.dlrt_pack_bitplanes(x0_u8, self.abits[0], binding.UNSIGNED, out=self.x0_packed)
            for group in self.pairs() if self.pair_launches else [(i,) for i in range(len(self.layers))]:
                if len(group) == 2:
                    i, j = group
                    binding.dlrt_bitserial_conv2d_fused_pair(self.problem(i), self.problem(j), self.abits[i],
                                                             self.wbits[i], binding.UNSIGNED, self.enc_w[i])
                else:
                    self.run_layer_fused(group[0], self.layer_input(group[0]))
        else:
            for i, pl in enumerate(self.layers):
                src = pl.spec.src
                self.run_layer(i, x0_u8 if src < 0 else self.layers[src].q)

    # ---- HIP graph ----
    def capture(self, x0_u8: torch.Tensor):
        """Record run(x0_u8) into a HIP graph (x0_u8 is read in place on every replay)."""
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            self.run(x0_u8)  # warm-up outside capture
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph):
            self.run(x0_u8)
        return self.graph

    def replay(self):
        self.graph.replay()
