"""Products left in the workspace as a sum of planes (ssnet_*_product_*) and the calls that consume
them with d_c = NULL: every output, opened value and message against the oracle's chain
convolution / dense layer -> degree reduction -> truncation (-> ReLU, -> REC), bit for bit.
Shapes cover one whole tile per workgroup, contractions split over several workgroups (several
planes), ragged edges, operands of at most 16 rows, and tensors on both sides of the size limits at
which the reduction changes kernels."""
import numpy as np
import pytest
import torch

import oracle as orc
from paper_2406_02629_amd import SSNet, SSNetError, binding
from util import field_uniform, to_dev, to_np

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


def small_secrets(shape, seed, bits, p):
    """signed values below 2^bits as field elements"""
    v = np.random.default_rng(seed).integers(-(1 << bits), 1 << bits, size=shape, dtype=np.int64)
    return np.where(v < 0, v + p, v).astype(np.uint64)


def check_consumers(s, p, y, shape, leave_product, f=12, seed=0):
    """y: the oracle's product shares [n, B, C, H, W] (degree 2t); leave_product() makes the library's
    product pending.  Runs the consuming calls one after the other, each on a fresh pending product."""
    n, t = s.n, s.t
    k, nr = t + 1, 2 * t + 1
    B, C, H, W = shape
    count = B * C * H * W
    yf = y.reshape(n, count)
    ids = list(range(1, k + 1))
    yr, m1, m2, _ = orc.degree_reduce(yf, n, t, p, seed, 3, full=True)
    yt, u, wsh = orc.truncate(yr, n, t, f, p, seed, 3, full=True)
    rec = orc.reconstruct(yt, ids, p)
    o = np.cumsum([0, nr * k, k * n, k, n]) * count

    # reduction alone, with its two message arrays
    leave_product()
    out = torch.empty((n, count), dtype=torch.int64, device="cuda")
    s.degree_reduce(None, stream_id=3, out=out)
    ws = to_np(s.messages()[: o[2]])
    assert np.array_equal(to_np(out), yr)
    assert np.array_equal(ws[: o[1]].reshape(nr, k, count), m1) and np.array_equal(ws[o[1]:].reshape(k, n, count), m2)

    # reduction + truncation + opening in one launch, all four message arrays
    leave_product()
    out2, got_rec = s.degree_reduce_truncate_reconstruct(None, stream_id=3, ids=ids, out=out)
    ws = to_np(s.messages()[: o[4]])
    for got, ref in zip([ws[o[i]:o[i + 1]] for i in range(4)], (m1, m2, u, wsh)):
        assert np.array_equal(got, ref.reshape(-1))
    assert np.array_equal(to_np(out2), yt) and np.array_equal(to_np(got_rec).reshape(-1), rec)

    # the same pending product again (it stays until the next product call), truncation with the rounding division
    yd = orc.truncate_div(yr, n, t, f, 4, p, seed, 3)
    s.degree_reduce_truncate_div(None, 4, stream_id=3, out=out)
    assert np.array_equal(to_np(out), yd)

    # the shortcut without messages: same residues as the protocol
    leave_product()
    out3, rec3 = s.reduce_truncate_direct(None, stream_id=3, ids=ids, out=out)
    assert np.array_equal(to_np(out3), yt) and np.array_equal(to_np(rec3).reshape(-1), rec)

    # Linear - Truncation - NonLinear tail in one call
    sb, sbi = s.nonlinear_masks((B, C, H, W), stream_id=21)
    osb, osbi = orc.nonlinear_masks(count, n, t, 28, p, seed, 21)
    want = orc.relu(yt, osb, osbi, n, t, p)
    leave_product()
    out5 = torch.empty((n, B, C, H, W), dtype=torch.int64, device="cuda")
    _, planes = s.reduce_truncate_relu(None, 3, sb, sbi, out=out5, want_planes=(C % 64 == 0))
    assert np.array_equal(to_np(out5).reshape(n, -1), want)
    if planes is not None:
        per = planes.numel() // n
        data = (8 if p == binding.P61 else 6) * count + 16
        ref = s.split_planes(to_dev(want.reshape(n, B, C, H, W)))
        assert bool(torch.equal(planes.view(n, per)[:, :data], ref.view(n, per)[:, :data]))

    # the same tail in one pass without messages: the protocol's residues, shares and planes
    leave_product()
    out6 = torch.empty_like(out5)
    _, planes6 = s.reduce_truncate_relu_direct(None, sb, sbi, out=out6, want_planes=(C % 64 == 0))
    assert np.array_equal(to_np(out6).reshape(n, -1), want)
    if planes6 is not None:
        assert bool(torch.equal(planes6.view(n, per)[:, :data], ref.view(n, per)[:, :data]))


CONV_CASES = [
    # B, C, H, W, Co, k, stride, pad
    (1, 256, 14, 14, 256, 3, 1, 1),     # 80 tiles of 36 k blocks: every tile split over several workgroups
    (1, 64, 14, 14, 1024, 1, 1, 0),     # more tiles than workgroups, one k block
    (1, 256, 14, 14, 64, 1, 1, 0),      # few tiles, four k blocks
    (1, 512, 7, 7, 128, 3, 1, 1),       # 49 pixels: one ragged column tile
    (2, 128, 9, 7, 65, 3, 2, 1),        # ragged rows and columns, stride 2
    (1, 64, 5, 5, 7, 3, 1, 1),          # at most 16 output channels
]


@pytest.mark.parametrize("n,t,p", [(5, 2, binding.P61), (3, 1, binding.P61), (7, 3, binding.P61), (5, 2, binding.P45)])
def test_conv_product_on_planes_then_every_consumer(n, t, p):
    s = SSNet(n, t, f=12, seed=91, p=p)
    bits = 11 if p == binding.P45 else 15
    cases = CONV_CASES if (n, t, p) == (5, 2, binding.P61) else CONV_CASES[:1] + CONV_CASES[3:5]
    for (B, C, H, W, Co, k, stride, pad) in cases:
        say("conv product", n, t, hex(p), B, C, H, W, Co, k, stride, pad)
        xs = orc.share(small_secrets((B, C, H, W), 1, bits, p), n, t, p, 91, 5)
        ws = orc.share(small_secrets((Co, C, k, k), 2, bits - 2, p), n, t, p, 91, 6)
        y = orc.conv(xs, ws, stride, pad, p)
        Ho, Wo = y.shape[-2:]
        planes = s.split_planes(to_dev(xs))
        wp = s.pack_weights_conv_taps(to_dev(ws))
        check_consumers(s, p, y, (B, Co, Ho, Wo),
                        lambda: s.conv_product_planes(planes, wp, B, C, H, W, Co, k, k, stride, pad), seed=91)


@pytest.mark.parametrize("n,t,p", [(5, 2, binding.P61), (3, 1, binding.P45)])
def test_prepacked_products_then_every_consumer(n, t, p):
    s = SSNet(n, t, f=12, seed=92, p=p)
    bits = 11 if p == binding.P45 else 15
    for (B, C, H, W, Co) in [(1, 1024, 14, 14, 256), (1, 70, 9, 9, 33), (2, 512, 7, 7, 2048)]:
        say("1x1 product", n, t, hex(p), B, C, H, W, Co)
        x = small_secrets((B, C, H, W), 3, bits, p)
        xs_o = orc.share(x, n, t, p, 92, 6)
        ws = orc.share(small_secrets((Co, C, 1, 1), 4, bits - 2, p), n, t, p, 92, 7)
        y = orc.conv(xs_o, ws, 1, 0, p)
        xs, tiles = s.share_packed(to_dev(x), stream_id=6)
        assert np.array_equal(to_np(xs), xs_o)
        wp = s.pack_weights_conv(to_dev(ws))
        check_consumers(s, p, y, (B, Co, H, W), lambda: s.conv1x1_product_prepacked(tiles, wp, B, C, H, W, Co), seed=92)
    for (M, K, N) in [(1, 2048, 1000), (5, 100, 9), (130, 4096, 65)]:
        say("dense product", n, t, hex(p), M, K, N)
        x = small_secrets((M, K), 5, bits, p)
        xs_o = orc.share(x, n, t, p, 92, 8)
        ws = orc.share(small_secrets((K, N), 6, bits - 2, p), n, t, p, 92, 9)
        y = orc.linear(xs_o, ws, p)
        xs, tiles = s.share_packed(to_dev(x), stream_id=8)
        wp = s.pack_weights_linear(to_dev(ws))
        check_consumers(s, p, y, (M, N, 1, 1), lambda: s.linear_product_prepacked(tiles, wp, M, K, N), seed=92)


def test_pending_product_full_range_operands_and_plane_sums():
    """Uniform field elements as operands (what shares are), a contraction long enough that every tile is
    shared: the reduction of the pending product equals the reduction of the oracle's product."""
    n, t, p = 5, 2, binding.P61
    s = SSNet(n, t, f=13, seed=93)
    B, C, H, W, Co, k = 1, 512, 7, 7, 96, 3
    xs, ws = field_uniform((n, B, C, H, W), 7), field_uniform((n, Co, C, k, k), 8)
    y = orc.conv(xs, ws, 1, 1, p)
    s.conv_product_planes(s.split_planes(to_dev(xs)), s.pack_weights_conv_taps(to_dev(ws)), B, C, H, W, Co, k, k, 1, 1)
    out = torch.empty((n, B * Co * H * W), dtype=torch.int64, device="cuda")
    s.degree_reduce(None, stream_id=1, out=out)
    assert np.array_equal(to_np(out), orc.degree_reduce(y.reshape(n, -1), n, t, p, 93, 1))
    # repeated launches give the same bits (planes are rewritten in full every time)
    for _ in range(20):
        s.conv_product_planes(s.split_planes(to_dev(xs)), s.pack_weights_conv_taps(to_dev(ws)), B, C, H, W, Co, k, k, 1, 1)
        again = torch.empty_like(out)
        s.degree_reduce(None, stream_id=1, out=again)
        assert bool(torch.equal(again, out))


def test_pending_product_errors():
    s = SSNet(5, 2, f=13, seed=1)
    out = torch.empty((5, 64), dtype=torch.int64, device="cuda")
    s.reserve(1 << 20)
    with pytest.raises(SSNetError) as ei:            # nothing pending
        s.degree_reduce(None, stream_id=0, out=out)
    assert ei.value.code == binding.EINVAL
    x = field_uniform((5, 1, 64, 4, 4), 1)
    w = field_uniform((5, 4, 64, 1, 1), 2)
    planes, wp = s.split_planes(to_dev(x)), s.pack_weights_conv_taps(to_dev(w))
    s.conv_product_planes(planes, wp, 1, 64, 4, 4, 4, 1, 1, 1, 0)      # 64 elements per party
    with pytest.raises(SSNetError) as ei:            # another element count than the pending product's
        s.degree_reduce(None, stream_id=0, out=torch.empty((5, 63), dtype=torch.int64, device="cuda"))
    assert ei.value.code == binding.EINVAL
    s.degree_reduce(None, stream_id=0, out=out)
    assert np.array_equal(to_np(out), orc.degree_reduce(orc.conv(x, w, 1, 0, binding.P61).reshape(5, -1), 5, 2, binding.P61, 1, 0))
    # a new workspace drops the pending product
    s._ws = None
    s.reserve(1 << 20)
    with pytest.raises(SSNetError) as ei:
        s.degree_reduce(None, stream_id=0, out=out)
    assert ei.value.code == binding.EINVAL
