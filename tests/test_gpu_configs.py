"""Parity at the benchmark's full sizes, in the launch configuration bench.py
times (same classes, same packed weights, same buffers).

The oracle side is a plain numpy/ctypes chain that shares no code with the
harness in paper_2406_02629_amd/chain.py: it draws the same seeded floats,
encodes, shares and evaluates every layer with the CPU oracle, and applies the
plaintext steps (ReLU, max-pool, global average) in numpy.
"""
import time

import numpy as np
import pytest
import torch

import oracle as orc
from paper_2406_02629_amd import SSNet
from paper_2406_02629_amd import fixedpoint as fx
from paper_2406_02629_amd.chain import WEIGHT_STREAM_BASE, Chain, post_plain
from ssnet_inputs import (alexnet_chain, gaussian, he_normal, lenet_chain, pooling_of, resnet_basic_chain, resnet_chain, uniform_below,
                          vgg16_chain)
from util import P61, to_dev, to_np

pytestmark = pytest.mark.gpu


def say(*a):
    """progress line (visible with pytest -s)"""
    print(*a, flush=True)


# ------------------------------------------------------------------ oracle-side plaintext steps
def np_post(y, L):
    """y: signed int64 [B, C, H, W] -> ReLU, then the layer's pooling (average = floor of sum / kernel elements)"""
    if L.post is None:
        return y
    y = np.maximum(y, 0)
    spec = pooling_of(L)
    if spec is None:
        return y
    kind, k, s, pad = spec
    B, C, H, W = y.shape
    Ho, Wo = (H + 2 * pad - k) // s + 1, (W + 2 * pad - k) // s + 1
    padded = np.zeros((B, C, H + 2 * pad, W + 2 * pad), np.int64)      # values are >= 0 after ReLU
    padded[:, :, pad:pad + H, pad:pad + W] = y
    out = np.zeros((B, C, Ho, Wo), np.int64)
    for r in range(k):
        for c in range(k):
            win = padded[:, :, r:r + s * Ho:s, c:c + s * Wo:s]
            out = np.maximum(out, win) if kind == "max" else out + win
    return out if kind == "max" else out // (k * k)


def np_signed_to_field(v, p=P61):
    return np.where(v < 0, v + p, v).astype(np.uint64)


def oracle_layer(L, l, x_plain, n, t, f, seed, wseed_base=100):
    """-> dict of the oracle's tensors for layer l given its plaintext input (field elements)"""
    shape = (L.cout, L.cin, L.ksize, L.ksize) if L.kind == "conv" else (L.cin, L.cout)
    w = orc.encode(he_normal(shape, L.K, wseed_base + l), f, P61)
    ws = orc.share(w, n, t, P61, seed, WEIGHT_STREAM_BASE + l)
    xs = orc.share(x_plain, n, t, P61, seed, l)
    if L.kind == "conv":
        y2 = orc.conv(xs, ws, L.stride, L.pad, P61)
    else:
        y2 = orc.linear(xs, ws, P61)
    yr = orc.degree_reduce(y2.reshape(n, -1), n, t, P61, seed, l)
    yt = orc.truncate(yr, n, t, f, P61, seed, l)
    rec = orc.reconstruct(yt, list(range(1, t + 2)), P61).reshape(y2.shape[1:])
    return {"xs": xs, "y2": y2, "yr": yr, "yt": yt, "rec": rec}


def run_chain_parity(depth, n, t, f, seed, full_every=1, batch=1):
    layers = resnet_chain(depth)
    ss = SSNet(n, t, f=f, seed=seed)
    chain = Chain(ss, layers, batch=batch)
    x_gpu = chain.image
    x_orc = orc.encode(gaussian((batch, 3, 224, 224), 5), f, P61)
    assert np.array_equal(to_np(x_gpu), x_orc)
    worst_float = 0.0
    t0 = time.time()
    for l, L in enumerate(layers):
        if L.kind == "fc":
            x_gpu = x_gpu.reshape(batch, -1)
            x_orc = x_orc.reshape(batch, -1)
        x_gpu = x_gpu.contiguous()
        o = oracle_layer(L, l, x_orc, n, t, f, seed)
        # the GPU layer, stage by stage, so that every intermediate share tensor can be compared
        chain.run_layer(l, x_gpu, "sg")
        assert np.array_equal(to_np(chain.x_shares[l]), o["xs"]), f"layer {l}: input shares"
        assert np.array_equal(to_np(chain.y[l]), o["y2"]), f"layer {l}: conv/dense output"
        chain.run_layer(l, x_gpu, "d")
        if l % full_every == 0:
            assert np.array_equal(to_np(chain.y[l]).reshape(n, -1), o["yr"]), f"layer {l}: degree_reduce"
        chain.run_layer(l, x_gpu, "t")
        assert np.array_equal(to_np(chain.y[l]).reshape(n, -1), o["yt"]), f"layer {l}: truncate"
        rec = chain.run_layer(l, x_gpu, "r")
        assert np.array_equal(to_np(rec), o["rec"]), f"layer {l}: reconstruct"
        # the same layer as the timed step runs it: all stages in one go, the product left in the workspace
        # as a sum of planes and added up by the reduction
        chain.y[l].fill_(-1)
        rec = chain.run_layer(l, x_gpu)
        assert np.array_equal(to_np(chain.y[l]).reshape(n, -1), o["yt"]), f"layer {l}: truncated shares, timed form"
        assert np.array_equal(to_np(rec), o["rec"]), f"layer {l}: opened value, timed form"
        # decoded output vs a float64 pass of this layer on the decoded (dequantised) input
        xin = orc.decode(x_orc, f, P61)
        shape = (L.cout, L.cin, L.ksize, L.ksize) if L.kind == "conv" else (L.cin, L.cout)
        wq = orc.decode(orc.encode(he_normal(shape, L.K, 100 + l), f, P61), f, P61)
        if L.kind == "conv":
            ref = torch.nn.functional.conv2d(torch.from_numpy(xin), torch.from_numpy(wq), stride=L.stride,
                                             padding=L.pad).numpy()
        else:
            ref = xin @ wq
        err = ref - orc.decode(o["rec"], f, P61)
        lo, hi = float(err.min()), float(err.max())
        assert lo > -2.0 ** -20 and hi < 2.0 ** -f + 2.0 ** -20, f"layer {l}: not a floor truncation {lo} {hi}"
        worst_float = max(worst_float, float(np.abs(err).max()))
        assert int(np.abs(orc.lift(o["rec"], P61)).max()) < 1 << 40       # fixed-point range is respected
        # plaintext step between layers, on each side with its own code
        if L.post is not None:
            x_gpu = fx.from_signed(post_plain(fx.lift(rec), L))
            x_orc = np_signed_to_field(np_post(orc.lift(o["rec"], P61), L))
            assert np.array_equal(to_np(x_gpu), x_orc), f"layer {l}: plaintext step"
        if l % 10 == 0:
            say(f"resnet{depth} layer {l}/{len(layers)} ok ({time.time() - t0:.0f} s)")
    assert worst_float < 2.0 ** -8
    # the timed path (all stages back to back on the recorded inputs) reproduces the same outputs
    chain.forward_prepare()
    last = to_np(chain.rec[-1]).copy()
    chain.forward_timed()
    torch.cuda.synchronize()
    assert np.array_equal(to_np(chain.rec[-1]), last)
    assert np.array_equal(last, o["rec"])
    return worst_float


def run_secure_chain_parity(depth, n, t, f, seed, pool_on_shares=False, p=P61, layers=None, batch=1):
    """The stack with ReLU on shares (SSS-NonLinear): every layer's output shares against an
    oracle chain of its own, and the opened logits against the chain that opens every layer.
    With pool_on_shares the two pooling points stay on shares too (mask equal inside a pooling
    kernel, division of the average inside the truncation): nothing but the logits is opened."""
    layers = resnet_chain(depth) if layers is None else layers
    B = batch
    ss = SSNet(n, t, f=f, seed=seed, p=p)
    chain = Chain(ss, layers, batch=B)
    chain.secure_setup(pool_on_shares)
    x_plain_g, x_sh_g = chain.image, None
    x_plain_o, x_sh_o = orc.encode(gaussian((B, layers[0].cin, layers[0].hin, layers[0].hin), 5), f, p), None
    t0 = time.time()
    rec_g = rec_o = None
    for l, L in enumerate(layers):
        shape = (L.cout, L.cin, L.ksize, L.ksize) if L.kind == "conv" else (L.cin, L.cout)
        ws = orc.share(orc.encode(he_normal(shape, L.K, 100 + l), f, p), n, t, p, seed, WEIGHT_STREAM_BASE + l)
        if x_sh_o is None:
            if L.kind == "fc":
                x_plain_g, x_plain_o = x_plain_g.reshape(B, -1), x_plain_o.reshape(B, -1)
            assert np.array_equal(to_np(x_plain_g), x_plain_o), f"layer {l}: plain input"
            x_sh_o = orc.share(x_plain_o, n, t, p, seed, l)
        elif L.kind == "fc":
            x_sh_o = x_sh_o.reshape(n, B, -1)
        y2 = orc.conv(x_sh_o, ws, L.stride, L.pad, p) if L.kind == "conv" else orc.linear(x_sh_o, ws, p)
        spec = pooling_of(L) if pool_on_shares else None
        pooled = spec is not None
        kdiv = spec[1] * spec[1] if pooled and spec[0] == "avg" else 1
        yr = orc.degree_reduce(y2.reshape(n, -1), n, t, p, seed, l)
        yt = orc.truncate_div(yr, n, t, f, kdiv, p, seed, l) if kdiv > 1 else orc.truncate(yr, n, t, f, p, seed, l)
        x_sh_g, rec_g = chain.secure_layer(l, None if x_sh_g is not None else x_plain_g.contiguous(), x_sh_g)
        if L.post is not None:
            # the multiplicative mask must not wrap: (elements summed by the pooling) * |x| * 2^28 < p/2
            peak = int(np.abs(orc.lift(orc.reconstruct(yt, list(range(1, t + 2)), p), p)).max())
            assert peak * (kdiv << 28) < p // 2, f"layer {l}: activation {peak} outside the mask's range"
        if L.post == "relu":
            sb, sbi = orc.nonlinear_masks(yt[0].size, n, t, 28, p, seed, Chain.MASK_STREAM_BASE + l)
            x_sh_o = orc.relu(yt, sb, sbi, n, t, p).reshape(y2.shape)
            assert np.array_equal(to_np(x_sh_g), x_sh_o), f"layer {l}: shares after ReLU"
        elif pooled:
            kind, pk, ps, pp = spec
            geo = (L.hout, L.hout, pk, pk, ps, ps, pp, pp, orc.POOL_MAX if kind == "max" else orc.POOL_SUM)
            sb, sbi = orc.pool_masks(B * L.cout, *geo[:8], n, t, 28, p, seed, Chain.MASK_STREAM_BASE + l)
            x_sh_o = orc.relu_pool(yt, sb, sbi, B * L.cout, *geo, n, t, p)
            ho = orc.pool_out_size(L.hout, geo[2], geo[4], geo[6])
            x_sh_o = x_sh_o.reshape(n, B, L.cout, ho, ho)
            assert np.array_equal(to_np(x_sh_g), x_sh_o), f"layer {l}: shares after ReLU and pooling"
        else:
            rec_o = orc.reconstruct(yt, list(range(1, t + 2)), p).reshape(y2.shape[1:])
            assert x_sh_g is None and np.array_equal(to_np(rec_g), rec_o), f"layer {l}: opened result"
            x_sh_o = None
            if L.post is not None:
                x_plain_g = fx.from_signed(post_plain(fx.lift(rec_g, p), L), p)
                x_plain_o = np_signed_to_field(np_post(orc.lift(rec_o, p), L), p)
        if l % 10 == 0:
            say(f"secure resnet{depth} layer {l}/{len(layers)} ok ({time.time() - t0:.0f} s)")
    logits = to_np(chain.secure_prepare(pool_on_shares)).copy()
    assert np.array_equal(logits, rec_o)
    chain.secure_timed()
    torch.cuda.synchronize()
    assert np.array_equal(to_np(chain.rec[-1]), logits)
    # the pass whose layer tails take the one-pass form without messages ends in the same shares
    last_shares = [y.clone() for y in chain.y[-3:]]
    chain.secure_timed(direct=True)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(chain.rec[-1]), logits)
    assert all(bool(torch.equal(a, b)) for a, b in zip(last_shares, chain.y[-3:]))
    plain = to_np(chain.forward_prepare())
    if not pool_on_shares:
        # the same logits as the chain that opens every layer (truncation and ReLU are exact)
        assert np.array_equal(plain, logits)
    else:
        # the average folded into the truncation rounds every element before the sum (App. C): each of
        # the 2048 pooled inputs of the classifier moves by a few units of 2^-f, the logits by little
        assert all(p is None for p in chain.secure_plain[1:])          # nothing was opened on the way
        dev = np.abs(orc.decode(plain, f, p) - orc.decode(logits, f, p)).max()
        say(f"resnet{depth} pooling on shares: max |logit - logit of the opened chain| = {dev:.3g}")
        assert dev < 2.0 ** -6


@pytest.mark.timeout(900)
def test_resnet50_stack_with_relu_on_shares():
    run_secure_chain_parity(50, 5, 2, 13, seed=20240602)


@pytest.mark.timeout(900)
def test_resnet50_stack_with_relu_and_pooling_on_shares():
    run_secure_chain_parity(50, 5, 2, 13, seed=20240602, pool_on_shares=True)


@pytest.mark.parametrize("n,t,p", [(3, 1, P61), (5, 2, P61), (7, 3, P61), (5, 1, P61), (8, 2, P61), (5, 2, (1 << 45) - 55),
                                   (3, 1, (1 << 45) - 55), (6, 2, (1 << 45) - 55)])
def test_small_stack_batch_3_with_pooling_on_shares(n, t, p):
    """Three images through a short stack (stem with overlapping max-pool, 1x1 and 3x3 layers on limb planes,
    global average, classifier), everything on shares: batched planes for masks and pooling, other schemes."""
    from ssnet_inputs import Layer
    layers = [Layer("conv", 3, 64, 7, 2, 3, 30, 15, "relu+maxpool3s2"), Layer("conv", 64, 64, 1, 1, 0, 8, 8, "relu"),
              Layer("conv", 64, 128, 3, 2, 1, 8, 4, "relu"), Layer("conv", 128, 70, 1, 1, 0, 4, 4, "relu+gap"),
              Layer("fc", 70, 10, 1, 1, 0, 1, 1, None)]
    run_secure_chain_parity(0, n, t, 12, seed=77, pool_on_shares=True, p=p, layers=layers, batch=3)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("batch,pool", [(1, True), (2, True), (1, False)])
def test_vgg16_stack_three_parties(batch, pool):
    """VGG16-shaped stack on 32 x 32 images, the paper's 3-party setting: 2 x 2 max-pools (one mask per kernel
    position), dense layers with ReLU on share vectors."""
    run_secure_chain_parity(0, 3, 1, 13, seed=16, pool_on_shares=pool, layers=vgg16_chain(32, 10, 512), batch=batch)


@pytest.mark.parametrize("n,t,f,p,batch", [(3, 1, 13, P61, 1), (3, 1, 13, P61, 4), (5, 2, 12, (1 << 45) - 55, 2)])
def test_lenet_stack_average_pools_on_shares(n, t, f, p, batch):
    """LeNet-5-shaped stack on 28 x 28 images: 5 x 5 convolutions through the im2col matrix (6 and 16 channels),
    2 x 2 average pools as sums behind a truncation with the rounding division by 4, dense layers with ReLU."""
    run_secure_chain_parity(0, n, t, f, seed=5, pool_on_shares=True, p=p, layers=lenet_chain(), batch=batch)


@pytest.mark.parametrize("n,t,batch", [(3, 1, 1), (5, 2, 2)])
def test_alexnet_stack_on_shares(n, t, batch):
    """AlexNet-shaped stack on 67 x 67 images: a strided 11 x 11 stem, a 5 x 5 layer with 96 input channels
    (im2col route), 384-channel layers on limb planes, overlapping max-pools without padding (one mask per
    plane), dense layers."""
    run_secure_chain_parity(0, n, t, 13, seed=12, pool_on_shares=True, layers=alexnet_chain(67, 10, 512), batch=batch)


@pytest.mark.timeout(900)
def test_resnet18_stack_on_shares():
    """basic-block ResNet-18 shapes (3 x 3 convolutions on limb planes throughout), five parties"""
    run_secure_chain_parity(18, 5, 2, 13, seed=18, pool_on_shares=True, layers=resnet_basic_chain(18))


@pytest.mark.timeout(900)
def test_resnet50_stack_over_the_45_bit_prime():
    """The library built for p = 2^45 - 55 (Sec. VII-A): the whole stack on shares, only the logits opened.
    f = 12 keeps every activation inside the 16-bit budget the masks of Sec. VII-B assume."""
    run_secure_chain_parity(50, 5, 2, 12, seed=20240602, pool_on_shares=True, p=(1 << 45) - 55)


@pytest.mark.timeout(900)
def test_config2_bulk_share_reconstruct_full_size():
    """n=5, t=2, 2^28 uniform field elements: every one of the 5 x 2^28 share words against the oracle
    (in chunks of 2^24 elements, so that host memory stays bounded), both reconstructions equal to the
    secret everywhere."""
    n, t, count, seed = 5, 2, 1 << 28, 2
    secret_np = uniform_below(count, P61, 2)
    secret = torch.from_numpy(secret_np.view(np.int64)).cuda()
    ss = SSNet(n, t, seed=seed)
    shares = ss.share(secret, stream_id=0)
    chunk = 1 << 24
    for start in range(0, count, chunk):
        eidx = np.arange(start, start + chunk, dtype=np.uint64)
        want = orc.share(secret_np[start:start + chunk], n, t, P61, seed, 0, eidx=eidx)
        got = to_np(shares[:, start:start + chunk])
        assert np.array_equal(got, want), start
        if start % (chunk * 4) == 0:
            say("config2 shares equal up to element", start + chunk)
    del want, got
    idx = np.concatenate([np.arange(2048), np.arange(count - 2048, count)]).astype(np.uint64)
    want = orc.share(secret_np[idx.astype(np.int64)], n, t, P61, seed, 0, eidx=idx)
    for ids in ([1, 2, 3], [3, 4, 5]):
        rec = ss.reconstruct(shares, ids)
        assert bool(torch.equal(rec, secret))
        assert np.array_equal(to_np(rec[torch.from_numpy(idx.astype(np.int64)).cuda()]),
                              orc.reconstruct(want, ids, P61))
    # a corrupted share plane is detected by disagreement between subsets
    shares[3, 12345] ^= 1
    assert int(ss.reconstruct(shares, [3, 4, 5])[12345]) != int(secret[12345])
    assert int(ss.reconstruct(shares, [1, 2, 3])[12345]) == int(secret[12345])


@pytest.mark.timeout(600)
def test_config3_resnet_conv_layer_full_size():
    """n=3, t=1, f=13: batch 8 x 64x56x56, 3x3 64->64 stride 1 pad 1, then degree
    reduction and truncation; every share plane against the oracle."""
    n, t, f, seed = 3, 1, 13, 3
    X = gaussian((8, 64, 56, 56), 3)
    Wt = he_normal((64, 64, 3, 3), 576, 4)
    ss = SSNet(n, t, f=f, seed=seed)
    xe, we = orc.encode(X, f, P61), orc.encode(Wt, f, P61)
    assert np.array_equal(to_np(fx.encode(torch.from_numpy(X).cuda(), f)), xe)
    xs, ws = ss.share(to_dev(xe), stream_id=1), ss.share(to_dev(we), stream_id=2)
    oxs, ows = orc.share(xe, n, t, P61, seed, 1), orc.share(we, n, t, P61, seed, 2)
    assert np.array_equal(to_np(xs), oxs) and np.array_equal(to_np(ws), ows)
    y2 = ss.conv_mod(xs, ws, 1, 1)
    oy2 = orc.conv(oxs, ows, 1, 1, P61)
    say("config3 oracle conv done")
    assert np.array_equal(to_np(y2), oy2)
    y2p = ss.conv_mod_packed(xs, ss.pack_weights_conv(ws), 64, 3, 3, 1, 1)
    assert bool(torch.equal(y2, y2p))
    yr = ss.degree_reduce(y2.view(n, -1), stream_id=3)
    oyr = orc.degree_reduce(oy2.reshape(n, -1), n, t, P61, seed, 3)
    assert np.array_equal(to_np(yr), oyr)
    yt = ss.truncate(yr, stream_id=4)
    oyt = orc.truncate(oyr, n, t, f, P61, seed, 4)
    assert np.array_equal(to_np(yt), oyt)
    rec = ss.reconstruct(yt, [1, 2])
    assert np.array_equal(to_np(rec), orc.reconstruct(oyt, [1, 2], P61))
    dec = fx.decode(rec, f).cpu().numpy().reshape(8, 64, 56, 56)
    exact = torch.nn.functional.conv2d(torch.from_numpy(orc.decode(xe, f, P61)), torch.from_numpy(orc.decode(we, f, P61)),
                                       padding=1).numpy()
    # the gate: against float64 on the dequantised operands the result is the exact product floored
    # to f fraction bits, far inside 2^-8
    err = exact - dec
    lo, hi = float(err.min()), float(err.max())
    assert lo > -2.0 ** -20 and hi < 2.0 ** -f + 2.0 ** -20, (lo, hi)
    # reported, not gated: against the un-quantised floats the input rounding alone (2^-14 per operand,
    # 576 terms) already reaches about 2^-8 in the worst of 1.6 M outputs
    plain = torch.nn.functional.conv2d(torch.from_numpy(X), torch.from_numpy(Wt), padding=1).numpy()
    say("config3 max |decoded - unquantised float64| =", float(np.abs(dec - plain).max()))


@pytest.mark.timeout(900)
def test_config4_resnet50_stack():
    worst = run_chain_parity(50, 5, 2, 13, seed=20240602)
    say("resnet50 worst per-layer |decoded - float64| =", worst)


@pytest.mark.timeout(1500)
def test_resnet50_stack_batch_8():
    """the batched setting of Sec. VIII (ImageNet, batch 8) that bench.py times beside the headline: eight
    images through the ResNet-50 shapes, every layer's shares and opened values against the oracle chain"""
    worst = run_chain_parity(50, 5, 2, 13, seed=20240602, batch=8)
    say("resnet50 batch 8 worst per-layer |decoded - float64| =", worst)


@pytest.mark.timeout(1500)
def test_resnet50_stack_batch_8_everything_on_shares():
    """the same eight images with ReLU and pooling on shares, only the logits opened"""
    run_secure_chain_parity(50, 5, 2, 13, seed=20240602, pool_on_shares=True, batch=8)


@pytest.mark.timeout(1500)
def test_config5_resnet152_stack():
    worst = run_chain_parity(152, 5, 2, 13, seed=20240602)
    say("resnet152 worst per-layer |decoded - float64| =", worst)
