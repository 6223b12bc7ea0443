"""Harness for a sequential stack of linear layers evaluated on Shamir shares.

Two ways through the stack:
  * `forward_prepare` / `forward_timed`: every layer's result is opened and the
    activation applied to the plain integers (see below);
  * `secure_prepare` / `secure_timed`: ReLU runs on the shares (SSS-NonLinear,
    Sec. VI-C, order Linear - Truncation - NonLinear of Sec. VII-A), so a layer's
    output shares are the next layer's input and nothing is opened.  The two
    pooling points of the stack (max-pool after the stem, global average before
    the classifier) go through the plain route, or, with
    `secure_setup(pool_on_shares=True)`, stay on shares as well: ReLU and pooling
    under a mask that is equal inside a pooling kernel, the division of the
    average moved into the truncation before it (Sec. VI-C); then only the
    logits are opened.

Per layer, on the GPU library (Sec. VI, order Linear -> Truncation):
    share the layer input (GEN) -> conv / dense on shares -> degree reduction
    with re-randomisation -> truncation by 2^f -> reconstruct (REC).
Between layers the harness applies the plaintext steps (ReLU, pooling) to the
reconstructed integers and hands the result to the next layer; that part is
outside the share arithmetic and outside any timed region.  Weight shares and
their int8 limb tiles are prepared once (offline preprocessing of the model).
"""
from __future__ import annotations

from typing import List, Optional

import torch

from ssnet_inputs import Layer, gaussian, he_normal, pooling_of

from . import fixedpoint as fx
from .binding import SSNet

WEIGHT_STREAM_BASE = 1 << 20      # stream ids of the weight sharings, apart from the per-layer ones


def pool_spec(L: Layer):
    """-> (kernel, stride, pad, mode, kdiv) of the pooling that follows layer L, or None.  An average is a sum
    here: its division (kdiv = kernel elements) moves into the truncation before it (Sec. VI-C)."""
    spec = pooling_of(L)
    if spec is None:
        return None
    kind, k, s, pad = spec
    if kind == "max":
        return (k, k), (s, s), (pad, pad), SSNet.POOL_MAX, 1
    return (k, k), (s, s), (pad, pad), SSNet.POOL_SUM, k * k


def post_plain(y: torch.Tensor, L: Layer) -> torch.Tensor:
    """Plaintext step after layer L, on signed integers [B, C, H, W] (int64): ReLU, then its pooling (an
    average is the floor of sum / kernel elements)."""
    if L.post is None:
        return y
    y = torch.clamp(y, min=0)
    spec = pooling_of(L)
    if spec is None:
        return y
    kind, k, s, pad = spec
    z = y.to(torch.float64)      # values are below 2^53, so the float64 detour is exact
    if kind == "max":
        return torch.nn.functional.max_pool2d(z, kernel_size=k, stride=s, padding=pad).to(torch.int64)
    sums = (torch.nn.functional.avg_pool2d(z, kernel_size=k, stride=s, padding=pad) * (k * k)).round().to(torch.int64)
    return torch.div(sums, k * k, rounding_mode="floor")


class Chain:
    def __init__(self, ss: SSNet, layers: List[Layer], batch: int = 1, image_seed: int = 5,
                 weight_seed_base: int = 100, keep_weight_shares: bool = False, weights_of: "Optional[Chain]" = None,
                 deferred: bool = True):
        """weights_of: another harness over the same layers and context whose prepared weight tiles are
        reused (they do not depend on the batch size).
        deferred: a layer's product shares stay in the workspace as a sum of planes and the reduction
        that follows adds them up (ssnet_*_product_*); otherwise the product kernel writes them out whole."""
        self.ss, self.layers, self.batch, self.deferred = ss, layers, batch, deferred
        dev = ss.device
        # k x k layers whose channel count allows it read their input from channel-innermost limb planes
        # instead of an im2col matrix; their weights are packed in (tap, channel) order
        self.on_planes = [L.kind == "conv" and L.ksize > 1 and ss.planes_supported(batch, L.cin, L.hin, L.hin)
                          for L in layers]
        self.packed: List[torch.Tensor] = [] if weights_of is None else list(weights_of.packed)
        self.wshares: List[Optional[torch.Tensor]] = [] if weights_of is None else list(weights_of.wshares)
        for l, L in enumerate(layers if weights_of is None else []):
            shape = (L.cout, L.cin, L.ksize, L.ksize) if L.kind == "conv" else (L.cin, L.cout)
            w = he_normal(shape, L.K, weight_seed_base + l)
            we = fx.encode(torch.from_numpy(w).to(dev), ss.f, ss.p)
            wsh = ss.share(we, stream_id=WEIGHT_STREAM_BASE + l)
            if self.on_planes[l]:
                self.packed.append(ss.pack_weights_conv_taps(wsh))
            else:
                self.packed.append(ss.pack_weights_conv(wsh) if L.kind == "conv" else ss.pack_weights_linear(wsh))
            self.wshares.append(wsh if keep_weight_shares else None)
        L0 = layers[0]
        img = gaussian((batch, L0.cin, L0.hin, L0.hin), image_seed)
        self.image = fx.encode(torch.from_numpy(img).to(dev), ss.f, ss.p)
        self.ids = list(range(1, ss.k + 1))
        # per-layer buffers so that the timed loop allocates nothing
        self.x_plain: List[Optional[torch.Tensor]] = [None] * len(layers)
        self.x_shares = [torch.empty((ss.n,) + self._in_shape(L), dtype=torch.int64, device=dev) for L in layers]
        self.y = [torch.empty((ss.n,) + self._out_shape(L), dtype=torch.int64, device=dev) for L in layers]
        self.rec = [torch.empty(self._out_shape(L), dtype=torch.int64, device=dev) for L in layers]
        # dense and 1x1 / stride 1 / unpadded layers take their input tiles straight from the share kernel
        self.pointwise = [L.kind == "fc" or (L.ksize == 1 and L.stride == 1 and L.pad == 0) for L in layers]
        tiles = max([ss.n * ss.lib.ssnet_packed_weight_bytes(batch * (L.hin * L.hin if L.kind == "conv" else 1), L.cin)
                     for L, pw in zip(layers, self.pointwise) if pw] + [16])
        self.x_tiles = torch.empty(tiles, dtype=torch.uint8, device=dev)
        planes = max([ss.n * ss.lib.ssnet_conv_planes_bytes(batch, L.cin, L.hin, L.hin)
                      for L, pl in zip(layers, self.on_planes) if pl] + [16])
        self.x_planes = torch.empty(planes, dtype=torch.uint8, device=dev)
        need = 0
        for L in layers:
            count = batch * L.cout * L.M
            need = max(need, ss.workspace_bytes_stream(count))
            if L.kind == "conv":
                need = max(need, ss.workspace_bytes_conv(batch, L.cin, L.hin, L.hin, L.cout, L.ksize, L.ksize,
                                                         L.stride, L.pad))
                tail = (batch, L.cout, L.M)
                product = ss.lib.ssnet_product_bytes_conv(ss._ctx, batch, L.cin, L.hin, L.hin, L.cout, L.ksize, L.ksize,
                                                          L.stride, L.pad)
            else:
                need = max(need, ss.workspace_bytes_linear(batch, L.cin, L.cout))
                tail = (batch, L.cout, 1)
                product = ss.lib.ssnet_product_bytes_linear(ss._ctx, batch, L.cin, L.cout)
            # a pending product sits behind the messages of the call that consumes it
            need = max(need, product + max(ss.workspace_bytes_stream(count),
                                           ss.lib.ssnet_workspace_bytes_layer_tail(ss._ctx, *tail)))
        ss.reserve(need)

    def _in_shape(self, L: Layer):
        return (self.batch, L.cin, L.hin, L.hin) if L.kind == "conv" else (self.batch, L.cin)

    def _out_shape(self, L: Layer):
        return (self.batch, L.cout, L.hout, L.hout) if L.kind == "conv" else (self.batch, L.cout)

    def run_layer(self, l: int, x_plain: torch.Tensor, stages: str = "sgdtr") -> torch.Tensor:
        """All share arithmetic of layer l.  `stages` selects steps for timing
        breakdowns: s=share, g=gemm/conv, d=degree_reduce, t=truncate, r=reconstruct;
        D = the outputs of d, t, r by the no-message shortcut (reported separately);
        p = leave the product pending although no reduction is asked for (timing of the product alone)."""
        ss, L = self.ss, self.layers[l]
        xs, y = self.x_shares[l], self.y[l]
        # the product stays in the workspace if a reduction follows in this call
        defer = self.deferred and "g" in stages and any(c in stages for c in "dDp")
        pending = False
        if self.pointwise[l] and "s" in stages and "g" in stages:
            ss.share_packed(x_plain, stream_id=l, out=xs, packed=self.x_tiles)
            if L.kind == "conv":
                if defer:
                    ss.conv1x1_product_prepacked(self.x_tiles, self.packed[l], self.batch, L.cin, L.hin, L.hin, L.cout)
                else:
                    ss.conv1x1_mod_prepacked(self.x_tiles, self.packed[l], self.batch, L.cin, L.hin, L.hin, L.cout, out=y)
            elif defer:
                ss.linear_product_prepacked(self.x_tiles, self.packed[l], self.batch, L.cin, L.cout)
            else:
                ss.linear_mod_prepacked(self.x_tiles, self.packed[l], self.batch, L.cin, L.cout, out=y)
            pending = defer
            stages = stages.replace("s", "").replace("g", "")
        if self.on_planes[l] and "g" in stages:
            if "s" in stages:
                ss.share_planes(x_plain, stream_id=l, out=xs, planes=self.x_planes)
            else:
                ss.split_planes(xs, planes=self.x_planes)
            geom = (self.batch, L.cin, L.hin, L.hin, L.cout, L.ksize, L.ksize, L.stride, L.pad)
            if defer:
                ss.conv_product_planes(self.x_planes, self.packed[l], *geom)
            else:
                ss.conv_mod_planes(self.x_planes, self.packed[l], *geom, out=y)
            pending = defer
            stages = stages.replace("s", "").replace("g", "")
        if "s" in stages:
            ss.share(x_plain, stream_id=l, out=xs)
        if "g" in stages:
            if L.kind == "conv":
                ss.conv_mod_packed(xs, self.packed[l], L.cout, L.ksize, L.ksize, L.stride, L.pad, out=y)
            else:
                ss.linear_mod_packed(xs, self.packed[l], L.cout, out=y)
        yv = y.view(ss.n, -1)
        c = None if pending else yv    # None: the pending product
        if "D" in stages:   # the outputs of reduction, truncation and opening without the protocol's messages
            ss.reduce_truncate_direct(c, stream_id=l, ids=self.ids, out=yv, secret=self.rec[l])
            return self.rec[l]
        if "d" in stages and "t" in stages and "r" in stages:   # one launch for the three steps
            ss.degree_reduce_truncate_reconstruct(c, stream_id=l, ids=self.ids, out=yv, secret=self.rec[l])
            return self.rec[l]
        if "d" in stages and "t" in stages:
            ss.degree_reduce_truncate(c, stream_id=l, out=yv)
        elif "d" in stages:
            ss.degree_reduce(c, stream_id=l, out=yv)
        elif "t" in stages:
            ss.truncate(yv, stream_id=l, out=yv)
        if "r" in stages:
            ss.reconstruct(y, self.ids, out=self.rec[l])
        return self.rec[l]

    def forward_prepare(self):
        """One full pass with the plaintext steps in between; records every
        layer's plaintext input so that timed passes can replay the share
        arithmetic back to back.  Returns the last layer's output (field elements)."""
        x = self.image
        out = None
        for l, L in enumerate(self.layers):
            if L.kind == "fc":
                x = x.reshape(self.batch, -1)
            self.x_plain[l] = x.contiguous()
            out = self.run_layer(l, self.x_plain[l])
            if L.post is not None:
                x = fx.from_signed(post_plain(fx.lift(out, self.ss.p), L), self.ss.p)
        return out

    def forward_timed(self, stages: str = "sgdtr"):
        """Share arithmetic of every layer on the recorded inputs, nothing else."""
        for l in range(len(self.layers)):
            self.run_layer(l, self.x_plain[l], stages)

    def total_field_macs(self) -> int:
        return self.ss.n * self.batch * sum(L.macs for L in self.layers)

    # ------------------------------------------------------------------ ReLU on shares
    MASK_STREAM_BASE = 1 << 21     # stream ids of the non-linear masks, apart from the others

    def secure_setup(self, pool_on_shares: bool = False):
        """Offline part of SSS-NonLinear: the trusted source's mask shares for every layer whose
        activation is a plain ReLU (Sec. VII-B) and, with pool_on_shares, for the layers followed
        by ReLU and pooling (masks equal inside a pooling kernel, Sec. VI-C)."""
        ss = self.ss
        dev = ss.device or "cuda"
        self.pool_on_shares = pool_on_shares
        self.masks, self.pooled = [], []
        for l, L in enumerate(self.layers):
            spec = pool_spec(L) if pool_on_shares else None
            if L.post == "relu":
                self.masks.append(ss.nonlinear_masks(self._out_shape(L), stream_id=self.MASK_STREAM_BASE + l, device=dev))
            elif spec is not None:
                kern, stride, pad, _, _ = spec
                b, bi = ss.pool_masks(self.batch * L.cout, L.hout, L.hout, kern, stride, pad,
                                      stream_id=self.MASK_STREAM_BASE + l, device=dev)
                self.masks.append((b, bi))
            else:
                self.masks.append(None)
            self.pooled.append(torch.empty((ss.n, self.batch, L.cout) + tuple(self.masks[l][1].shape[-2:]),
                                           dtype=torch.int64, device=dev) if spec is not None else None)
        # here every convolution whose channel count allows it reads limb planes, 1x1 ones included: the
        # tail of the layer before writes them.  For a 1x1 kernel the tap-major tiles are the ordinary ones.
        self.sec_planes = [L.kind == "conv" and ss.planes_supported(self.batch, L.cin, L.hin, L.hin)
                           for L in self.layers]
        self.sec_packed = list(self.packed)
        need = max([ss.n * ss.lib.ssnet_conv_planes_bytes(self.batch, L.cin, L.hin, L.hin)
                    for L, pl in zip(self.layers, self.sec_planes) if pl] + [16])
        if self.x_planes.numel() < need:
            self.x_planes = torch.empty(need, dtype=torch.uint8, device=self.x_planes.device)

    def secure_layer(self, l: int, x_plain: Optional[torch.Tensor], x_shares: Optional[torch.Tensor],
                     planes_ready: bool = False, direct: bool = False):
        """Layer l from its plain input (shared here) or from the previous layer's output shares
        (planes_ready: their limb planes already are in self.x_planes).
        -> (output shares after the activation, or None; opened result, or None)"""
        ss, L = self.ss, self.layers[l]
        y = self.y[l]
        if x_shares is None:
            x_shares = ss.share(x_plain, stream_id=l, out=self.x_shares[l])
        elif L.kind == "fc":
            x_shares = x_shares.view(ss.n, self.batch, -1)
        pending = False
        if self.sec_planes[l]:
            if not planes_ready:
                ss.split_planes(x_shares, planes=self.x_planes)
            geom = (self.batch, L.cin, L.hin, L.hin, L.cout, L.ksize, L.ksize, L.stride, L.pad)
            if self.deferred:   # every branch below starts with a reduction, which adds the product's planes up
                ss.conv_product_planes(self.x_planes, self.sec_packed[l], *geom)
                pending = True
            else:
                ss.conv_mod_planes(self.x_planes, self.sec_packed[l], *geom, out=y)
        elif L.kind == "conv":
            ss.conv_mod_packed(x_shares, self.packed[l], L.cout, L.ksize, L.ksize, L.stride, L.pad, out=y)
        else:
            ss.linear_mod_packed(x_shares, self.packed[l], L.cout, out=y)
        yv = y.view(ss.n, -1)
        c = None if pending else yv
        if L.post == "relu":
            # reduce + truncate + ReLU in one launch, which also leaves the next layer's limb planes
            b, bi = self.masks[l]
            nxt = l + 1 < len(self.layers) and self.sec_planes[l + 1]
            if direct:   # the same shares and planes in one pass without the protocol's messages
                ss.reduce_truncate_relu_direct(None if pending else y, b, bi, out=y, planes=self.x_planes if nxt else None)
            else:
                ss.reduce_truncate_relu(None if pending else y, l, b, bi, out=y, planes=self.x_planes if nxt else None)
            return y, None
        if self.pooled[l] is not None:
            # reduce + truncate (with the division of an average), then ReLU and pooling under the mask
            kern, stride, pad, mode, kdiv = pool_spec(L)
            b, bi = self.masks[l]
            if kdiv > 1:
                ss.degree_reduce_truncate_div(c, kdiv, stream_id=l, out=yv)
            else:
                ss.degree_reduce_truncate(c, stream_id=l, out=yv)
            return ss.relu_pool(y, b, bi, kern, stride, pad, mode, out=self.pooled[l]), None
        ss.degree_reduce_truncate_reconstruct(c, stream_id=l, ids=self.ids, out=yv, secret=self.rec[l])
        return None, self.rec[l]

    def _planes_ready(self, l: int, x_shares) -> bool:
        """the tail of a layer with a plain ReLU has left the limb planes of layer l's input"""
        return x_shares is not None and self.sec_planes[l] and l > 0 and self.layers[l - 1].post == "relu"

    def secure_prepare(self, pool_on_shares: bool = False):
        """One pass; records the plain inputs of the layers that follow an opened pooling point.
        Returns the last layer's opened output."""
        if not hasattr(self, "masks") or self.pool_on_shares != pool_on_shares:
            self.secure_setup(pool_on_shares)
        self.secure_plain: List[Optional[torch.Tensor]] = [None] * len(self.layers)
        x_plain, x_shares, out = self.image, None, None
        for l, L in enumerate(self.layers):
            if x_shares is None:
                if L.kind == "fc":
                    x_plain = x_plain.reshape(self.batch, -1)
                self.secure_plain[l] = x_plain.contiguous()
            x_shares, out = self.secure_layer(l, self.secure_plain[l], x_shares, planes_ready=self._planes_ready(l, x_shares))
            if x_shares is None and L.post is not None:
                x_plain = fx.from_signed(post_plain(fx.lift(out, self.ss.p), L), self.ss.p)
        return out

    def secure_timed(self, direct: bool = False):
        """The share arithmetic of the whole stack, layer feeding layer.  direct: the tails of the layers with
        a plain ReLU in their one-pass form without messages (same shares)."""
        x_shares = None
        for l in range(len(self.layers)):
            x_shares, _ = self.secure_layer(l, self.secure_plain[l], x_shares,
                                            planes_ready=self._planes_ready(l, x_shares), direct=direct)
