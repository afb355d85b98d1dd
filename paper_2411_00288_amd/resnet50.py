"""The convolution trunk of ResNet-50 (the paper's main architecture, Sec. 4) as a chain of library calls with real
dataflow: 7x7 stem -> max pool -> 16 bottleneck blocks, every block closed by the fused add + ReLU tail.

48 of the 53 convolutions carry a 2:4 mask and run on the sparse path (or, with ``sparse=False``, on the dense twin
with the same masked weights); the stem and the four shortcut convolutions stay dense.  The image is handed over with
a fourth, all-zero channel (the column-wise augmentation that Sec. 3.3 suggests for a reduction length that is no
multiple of 4: K = 7*7*4 = 196 instead of 147), so that every pixel is 8 aligned bytes and the stem's staging loads
one whole 2:4 block at a time; ``image_channels=3`` keeps the unpadded form.
Batch norm is folded into the bias.  Weights, masks and biases are synthetic (``workloads``); this module only wires
buffers and launches -- every arithmetic step runs in the library's kernels.
"""
from __future__ import annotations

import dataclasses

import numpy as np
import torch

from . import binding as ss
from . import workloads as wl

STAGES = [(64, 3, 1), (128, 4, 2), (256, 6, 2), (512, 3, 2)]      # (width, blocks, stride of the first block)


@dataclasses.dataclass
class Op:
    kind: str                 # "conv" | "pool"
    name: str
    src: int                  # activation buffer ids
    dst: int
    layer: wl.Layer | None = None
    residual: int | None = None


def build_ops(batch: int, image: int, dtype: int = wl.BF16, seed: int = 7000, image_channels: int = 4):
    """The op list and the activation shapes {buffer id: (N, H, W, C)}."""
    ops: list[Op] = []
    shapes = {0: (batch, image, image, image_channels)}
    nxt = [1]

    def new_buf(shape):
        i = nxt[0]
        nxt[0] += 1
        shapes[i] = shape
        return i

    def conv(name, src, cout, k, stride, act, mask, residual=None, relu_input=True, korder=wl.K_CRS):
        N, H, W, C = shapes[src]
        L = wl.Layer(name, N=N, H=H, W=W, cin=C, cout=cout, kh=k, kw=k, stride=stride, pad=k // 2, dtype=dtype, act=act,
                     korder=korder, mask=mask, relu_input=relu_input, seed=seed + len(ops))
        dst = new_buf((N, L.Ho, L.Wo, cout))
        ops.append(Op("conv", name, src, dst, L, residual))
        return dst

    a = conv("stem", 0, 64, 7, 2, wl.ACT_RELU, "none", relu_input=False,
             korder=wl.K_RSC if image_channels % 4 == 0 else wl.K_CRS)
    N, H, W, C = shapes[a]
    p = new_buf((N, (H + 2 - 3) // 2 + 1, (W + 2 - 3) // 2 + 1, C))
    ops.append(Op("pool", "maxpool", a, p))
    cur = p
    for si, (width, blocks, stride) in enumerate(STAGES, start=1):
        for b in range(blocks):
            s = stride if b == 0 else 1
            c1 = conv(f"s{si}b{b}_c1", cur, width, 1, 1, wl.ACT_RELU, "top2")
            c2 = conv(f"s{si}b{b}_c2", c1, width, 3, s, wl.ACT_RELU, "top2")
            short = conv(f"s{si}b{b}_ds", cur, 4 * width, 1, s, wl.ACT_NONE, "none") if b == 0 else cur
            cur = conv(f"s{si}b{b}_c3", c2, 4 * width, 1, 1, wl.ACT_RELU, "top2", residual=short)
    return ops, shapes


class Trunk:
    """Device-resident weights and activation buffers of the trunk, and a ``forward()`` that enqueues every kernel
    on the current stream (capturable in a HIP graph)."""

    def __init__(self, batch: int, image: int = 224, dtype: int = wl.BF16, sparse: bool = True, seed: int = 7000,
                 c3_scale: float = 0.25, keep_host: bool = False, image_channels: int = 4, fuse_pairs: bool = True):
        """fuse_pairs: run a block's 3x3 and the 1x1 expansion after it as one kernel where that is faster (widths up
        to 128 on the sparse path, 64 on the dense twin); the 3x3's own output buffer is then never written."""
        self.ops, self.shapes = build_ops(batch, image, dtype, seed, image_channels)
        self.dtype, self.sparse = dtype, sparse
        tdt = ss.torch_dtype(dtype)
        self.bufs = {i: torch.zeros(shp, dtype=tdt, device="cuda") for i, shp in self.shapes.items()}
        self.host = {}
        self.launches = []
        self.fused = []                                     # names of the 3x3 layers that run fused with their successor
        prepared = {}
        for op in self.ops:
            if op.kind != "conv":
                continue
            L = op.layer
            d = wl.make_weights(L, scale=c3_scale if op.residual is not None else 1.0)
            if keep_host:
                self.host[op.name] = d
            desc = ss.make_desc(L.cout, L.cin, L.kh, L.kw, L.dtype, L.korder)
            W = torch.from_numpy(d["W"].view(np.int16)).cuda().view(tdt)
            M = None if d["M"] is None else torch.from_numpy(d["M"]).cuda()
            bias = torch.from_numpy(d["bias"]).cuda()
            use_sparse = sparse and M is not None
            wbuf = ss.ss_mask_compress(desc, W, M) if use_sparse else ss.ss_dense_pack(desc, W, M)
            prepared[op.name] = (desc, wbuf, bias, use_sparse)
        by_dst = {op.dst: op for op in self.ops}
        pos = {}                                            # op name -> index of its launch
        for op in self.ops:
            if op.kind == "pool":
                x, y = self.bufs[op.src], self.bufs[op.dst]
                self.launches.append(lambda x=x, y=y: ss.ss_maxpool2d(x, 3, 2, 1, y=y))
                continue
            L = op.layer
            desc, wbuf, bias, use_sparse = prepared[op.name]
            prev = by_dst.get(op.src)
            res = None if op.residual is None else self.bufs[op.residual]
            if (fuse_pairs and op.name.endswith("_c3") and prev is not None and prev.name.endswith("_c2") and
                    prepared[prev.name][3] == use_sparse and
                    all(ss.ss_conv2d_pw_fused_query(prepared[prev.name][0], (prev.layer.stride,) * 2, (prev.layer.pad,) * 2,
                                                    desc, use_sparse))):      # the library says: supported, and expected to pay
                # (decided here, at the 1x1's position in the order: its residual is ready by now)
                d1, w1, b1, _ = prepared[prev.name]
                P = prev.layer
                launch, _ = ss.prepare_conv2d_pw_fused(d1, self.bufs[prev.src], w1, b1, (P.stride,) * 2, (P.pad,) * 2, P.act,
                                                       desc, wbuf, bias, res, L.act, y=self.bufs[op.dst], sparse=use_sparse)
                self.fused.append(prev.name)
                self.launches[pos[prev.name]] = None        # the 3x3 runs inside this launch
                self.launches.append(launch)
                continue
            launch, _ = ss.prepare_conv2d(desc, self.bufs[op.src], wbuf, bias, (L.stride,) * 2, (L.pad,) * 2, L.act,
                                          y=self.bufs[op.dst], sparse=use_sparse, residual=res)
            pos[op.name] = len(self.launches)
            self.launches.append(launch)
        self.launches = [l for l in self.launches if l is not None]
        torch.cuda.synchronize()

    @property
    def input(self) -> torch.Tensor:
        return self.bufs[0]

    @property
    def output(self) -> torch.Tensor:
        return self.bufs[self.ops[-1].dst]

    def forward(self):
        for launch in self.launches:
            launch()
        return self.output

    def dense_equiv_flop(self) -> float:
        """Dense-equivalent FLOP of one forward pass; the stem counts its three real channels, not the padding."""
        total = 0.0
        for op in self.ops:
            if op.kind == "conv":
                f = op.layer.dense_equiv_flop
                total += f * 3 / op.layer.cin if op.name == "stem" else f
        return total
