"""Layer-list harness: chains packed convolutions on the GPU through the C ABI.

A stand-in for the graph runtime that the paper's product has around its kernels (Section VI):
just enough to run a list of quantized conv layers back to back.  Two ways to run a layer:

* ``fused=True`` (default): one ``dlrt_bitserial_conv2d_fused`` launch per layer, which writes the
  NEXT layer's packed activations directly (conv -> scale/bias -> requant -> bitplanes); only the
  stack input goes through ``dlrt_pack_bitplanes``.
* ``fused=False``: ``dlrt_pack_bitplanes`` -> ``dlrt_bitserial_conv2d`` -> ``dlrt_epilogue_f32`` per layer.

A layer listed in ``f32_layers`` keeps its output in float32 (the dequantized ``y``), the way the paper
leaves precision-sensitive layers unquantized (Section VII-D); its readers get it through the quantizer of
Section IV fused into ``dlrt_pack_bitplanes`` (float32 source, the activation step size in ``act_scales``).

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
    y: torch.Tensor = None       # float32 output of a layer that stays unquantized
    act_scale: torch.Tensor = None   # step size its readers quantize y with (one value)


def _per_layer(v, n):
    return list(v) if isinstance(v, (list, tuple)) else [v] * n


class ConvStack:
    """abits / wbits / enc_w are one value for the whole stack or one per layer (mixed precision, as in
    the paper's per-layer precision choice).  A layer's output is requantized to the activation width
    of the layers that read it (they must agree); a layer nobody reads keeps its own width."""

    def __init__(self, layers, weights_i8, scales, biases, abits, wbits, enc_w, device="cuda:0",
                 fused: bool = True, keep_outputs: bool = True, pair_launches: bool = True, batch: int = 1,
                 f32_layers=(), act_scales=None):
        n = len(layers)
        self.f32_layers = set(f32_layers)
        act_scales = act_scales or {}
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
            if i in self.f32_layers:
                pl.y = torch.empty((B, L.Ho, L.Wo, L.Co), dtype=torch.float32, device=self.device)
                pl.act_scale = torch.tensor([act_scales[i]], dtype=torch.float32, device=self.device)
            if fused or i in self.f32_layers:
                pl.out_packed = torch.empty((B * L.Ho * L.Wo, self.qbits[i], (L.Co + 31) // 32), dtype=torch.int32,
                                            device=self.device)
            if not fused:
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
    def requantize_f32(self, i: int):
        """Quantize layer i's float32 output to its readers' activation width and pack it (one launch)."""
        pl = self.layers[i]
        binding.dlrt_pack_bitplanes(pl.y, self.qbits[i], binding.UNSIGNED, scale=pl.act_scale, out=pl.out_packed)

    def run_layer(self, i: int, x_u8: torch.Tensor):
        pl = self.layers[i]
        L = pl.spec
        if L.src >= 0 and L.src in self.f32_layers:
            xp = self.layers[L.src].out_packed  # quantized and packed from float32 when the source ran
        else:
            xp = binding.dlrt_pack_bitplanes(x_u8, self.abits[i], binding.UNSIGNED, out=pl.xp)
        binding.dlrt_bitserial_conv2d(xp, pl.wp, self.batch, L.H, L.W, L.Ci, L.Co, L.k, L.k, (L.stride, L.stride),
                                      (L.pad, L.pad), self.abits[i], self.wbits[i], binding.UNSIGNED, self.enc_w[i],
                                      out=pl.acc)
        if i in self.f32_layers:
            binding.dlrt_epilogue_f32(pl.acc, pl.scale, pl.bias, want_f32=True, out_f32=pl.y)
            self.requantize_f32(i)
        else:
            binding.dlrt_epilogue_f32(pl.acc, pl.scale, pl.bias, want_f32=False, qbits=self.qbits[i], out_q=pl.q)

    # ---- fused: one launch per layer ----
    def run_layer_fused(self, i: int, x_packed: torch.Tensor, tile_rows: int = 0, ksplit: int = 0):
        pl = self.layers[i]
        L = pl.spec
        if i in self.f32_layers:
            binding.dlrt_bitserial_conv2d_fused(x_packed, pl.wp, pl.scale, pl.bias, self.batch, L.H, L.W, L.Ci, L.Co,
                                                L.k, L.k, (L.stride, L.stride), (L.pad, L.pad), self.abits[i],
                                                self.wbits[i], binding.UNSIGNED, self.enc_w[i], qbits=self.qbits[i],
                                                out_acc=pl.acc if self.keep else None, out_f32=pl.y,
                                                tile_rows=tile_rows, ksplit=ksplit)
            self.requantize_f32(i)
            return
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
                                    (L.stride, L.stride), (L.pad, L.pad), self.abits[i], self.wbits[i], qbits=self.qbits[i],
                                    out_acc=pl.acc if self.keep else None, out_q=pl.q if self.keep else None,
                                    out_packed=pl.out_packed)

    def pairs(self):
        """Launch schedule of the fused chain.  Layers go out in list order, each as soon as its input exists, and
        two layers of the same bit widths that are both ready share a launch: first choice a later layer that
        reads the same input (a stride-2 conv with the 1x1 conv beside it, two 1x1 convs on one tensor), else the
        next ready layer on another tensor (the inner 1x1 conv of one stage beside the stride-2 conv that opens the
        next).  The later one simply runs early; its readers still come after it.  Whether the two really share a
        launch is the library's decision (layers that fill the chip on their own go out one after the other)."""
        plan, done, n = [], set(), len(self.layers)
        widths = lambda i: (self.abits[i], self.wbits[i], self.enc_w[i])
        ready = lambda j: self.layers[j].spec.src < 0 or self.layers[j].spec.src in done
        for i in range(n):
            if i in done:
                continue
            if i in self.f32_layers:
                plan.append((i,))
                done.add(i)
                continue
            later = [j for j in range(i + 1, n) if j not in done and j not in self.f32_layers and ready(j) and
                     widths(j) == widths(i)]
            same = [j for j in later if self.layers[j].spec.src == self.layers[i].spec.src]
            mate = same[0] if same else later[0] if later else None
            if mate is None:
                plan.append((i,))
            else:
                plan.append((i, mate))
                done.add(mate)
            done.add(i)
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
