"""Parity of the library built for the paper's own prime p = 2^45 - 55 (Sec. VII-A) against the
oracle (which takes any prime): every entry point, element by element, at sizes that span the
kernels' size classes, several tiles and ragged tails."""
import numpy as np
import pytest
import torch

import oracle as orc
from paper_2406_02629_amd import P45, SSNet
from util import to_dev, to_np

pytestmark = pytest.mark.gpu

SCHEMES = [(3, 1), (5, 2), (7, 3), (5, 1)]


def say(*a):
    print(*a, flush=True)


def uniform(shape, seed):
    """uniform field elements with extreme values planted"""
    a = np.random.default_rng(seed).integers(0, P45, size=shape, dtype=np.uint64)
    flat = a.reshape(-1)
    if flat.size >= 6:
        flat[:4] = [0, P45 - 1, 1, (P45 - 1) // 2]
        flat[-2:] = [P45 - 1, (P45 + 1) // 2]
    return a


def signed(xs):
    return np.where(xs < 0, xs + P45, xs).astype(np.uint64)


@pytest.mark.parametrize("n,t", SCHEMES)
def test_p45_share_and_reconstruct(n, t):
    s = SSNet(n, t, seed=5, p=P45)
    for count in (1, 255, 4099, 65538, (1 << 20) + 2):
        say("p45 share", n, t, count)
        secret = uniform(count, count)
        for degree in (t, 2 * t):
            got = s.share(to_dev(secret), stream_id=3, degree=degree)
            want = orc.share(secret, n, degree, P45, 5, 3)
            assert np.array_equal(to_np(got), want)
            ids = list(range(n, n - degree - 1, -1))
            assert np.array_equal(to_np(s.reconstruct(got, ids, degree=degree)), secret)
            assert np.array_equal(orc.reconstruct(want, ids, P45), secret)


@pytest.mark.parametrize("n,t", SCHEMES)
def test_p45_reduce_truncate_and_fused_forms(n, t):
    f = 13
    s = SSNet(n, t, f=f, seed=9, p=P45)
    k, nr = t + 1, 2 * t + 1
    for count in (1, 100, 8191, 9000, 170001, (1 << 20) + 2):      # lanes kernel, fixed / general kernels, two per thread
        say("p45 reduce/truncate", n, t, count)
        xs = np.random.default_rng(count).integers(-(1 << 42), 1 << 42, count, dtype=np.int64)
        xs[: min(count, 4)] = [0, -1, (1 << f) - 1, -(1 << f) - 1][: min(count, 4)]
        c = orc.share(signed(xs), n, 2 * t, P45, 9, 1)
        yr_o, m1, m2, _ = orc.degree_reduce(c, n, t, P45, 9, 2, full=True)
        yr = s.degree_reduce(to_dev(c), stream_id=2)
        ws = to_np(s.messages()[: (nr * k + k * n) * count])
        assert np.array_equal(ws[: nr * k * count].reshape(nr, k, count), m1)
        assert np.array_equal(ws[nr * k * count:].reshape(k, n, count), m2)
        assert np.array_equal(to_np(yr), yr_o)
        yt_o, u, wsh = orc.truncate(yr_o, n, t, f, P45, 9, 2, full=True)
        yt = s.truncate(yr, stream_id=2)
        ws = to_np(s.messages()[: (k + n) * count])
        assert np.array_equal(ws[: k * count].reshape(k, count), u) and np.array_equal(ws[k * count:].reshape(n, count), wsh)
        assert np.array_equal(to_np(yt), yt_o)
        assert np.array_equal(orc.lift(orc.reconstruct(yt_o, list(range(1, k + 1)), P45), P45), xs >> f)
        assert np.array_equal(to_np(s.degree_reduce_truncate(to_dev(c), stream_id=2)), yt_o)
        ids = list(range(n - t, n + 1))
        out, rec = s.degree_reduce_truncate_reconstruct(to_dev(c), stream_id=2, ids=ids)
        assert np.array_equal(to_np(out), yt_o) and np.array_equal(to_np(rec), signed(xs >> f))
        out, rec = s.reduce_truncate_direct(to_dev(c), stream_id=2, ids=ids)
        assert np.array_equal(to_np(out), yt_o) and np.array_equal(to_np(rec), signed(xs >> f))
        if count <= 170001:
            want = orc.truncate_div(yr_o, n, t, f, 49, P45, 9, 2)
            assert np.array_equal(to_np(s.truncate_div(yr, 49, stream_id=2)), want)
            assert np.array_equal(to_np(s.degree_reduce_truncate_div(to_dev(c), 49, stream_id=2)), want)


P45_LINEAR_SHAPES = [(1, 1, 1), (3, 5, 7), (17, 65, 33), (64, 256, 128), (100, 300, 70), (1, 2048, 100), (49, 700, 80),
                     (130, 1000, 200), (256, 4608, 49), (1, 9216, 300), (16, 1000, 257), (8, 64, 128), (2, 16383, 130)]


@pytest.mark.parametrize("n,t", [(3, 1), (5, 2), (7, 3)])
def test_p45_linear_and_conv(n, t):
    """six-limb product kernel: uniform field elements (every limb busy), ragged tiles, tiles shared
    between workgroups, long contractions"""
    s = SSNet(n, t, seed=1, p=P45)
    for M, K, N in P45_LINEAR_SHAPES:
        say("p45 linear", n, M, K, N)
        x, w = uniform((n, M, K), M * 7 + K), uniform((n, K, N), N * 3 + K)
        want = orc.linear(x, w, P45)
        assert np.array_equal(to_np(s.linear_mod(to_dev(x), to_dev(w))), want)
        wp = s.pack_weights_linear(to_dev(w))
        assert np.array_equal(to_np(s.linear_mod_packed(to_dev(x), wp, N)), want)
    # worst case for the int32 diagonal sums: every digit at its extreme over the longest contraction
    K = 16383
    ext = np.full((n, 2, K), int("0x808080808080", 16) % P45, np.uint64)
    ext[:, 1, :] = int("0x7f7f7f7f7f7f", 16) % P45
    w = np.ascontiguousarray(np.transpose(ext, (0, 2, 1)))
    assert np.array_equal(to_np(s.linear_mod(to_dev(ext), to_dev(w))), orc.linear(ext, w, P45))
    for (B, C, H, W, Co, ksz, stride, pad) in [(1, 3, 9, 9, 5, 3, 1, 1), (2, 16, 12, 10, 20, 3, 2, 1),
                                               (1, 64, 14, 14, 64, 1, 1, 0), (1, 8, 15, 15, 4, 7, 2, 3)]:
        say("p45 conv", n, B, C, H, W, Co, ksz, stride, pad)
        x, w = uniform((n, B, C, H, W), 3), uniform((n, Co, C, ksz, ksz), 4)
        want = orc.conv(x, w, stride, pad, P45)
        assert np.array_equal(to_np(s.conv_mod(to_dev(x), to_dev(w), stride, pad)), want)
        wp = s.pack_weights_conv(to_dev(w))
        assert np.array_equal(to_np(s.conv_mod_packed(to_dev(x), wp, Co, ksz, ksz, stride, pad)), want)


@pytest.mark.parametrize("n,t", [(3, 1), (5, 2), (7, 3)])
def test_p45_limb_tiles_and_planes_paths(n, t):
    """GEN fused with the limb split (tiles for dense / 1x1 layers, channel-innermost planes for k x k
    convolutions) and the convolution that gathers from the planes"""
    s = SSNet(n, t, seed=17, p=P45)
    for (B, C, H, W, Co) in [(1, 3, 5, 7, 2), (2, 70, 9, 9, 33), (1, 128, 14, 14, 64)]:
        say("p45 share_packed conv", n, t, B, C, H, W, Co)
        x = uniform((B, C, H, W), C)
        xs_o = orc.share(x, n, t, P45, 17, 1)
        xs, tiles = s.share_packed(to_dev(x), stream_id=1)
        assert np.array_equal(to_np(xs), xs_o)
        w = orc.share(uniform((Co, C, 1, 1), Co), n, t, P45, 17, 2)
        y = s.conv1x1_mod_prepacked(tiles, s.pack_weights_conv(to_dev(w)), B, C, H, W, Co)
        assert np.array_equal(to_np(y), orc.conv(xs_o, w, 1, 0, P45))
    for (M, K, N) in [(1, 1, 1), (5, 100, 9), (8, 2048, 1000), (130, 64, 65)]:
        say("p45 share_packed dense", n, t, M, K, N)
        x = uniform((M, K), K)
        xs_o = orc.share(x, n, t, P45, 17, 3)
        xs, tiles = s.share_packed(to_dev(x), stream_id=3)
        assert np.array_equal(to_np(xs), xs_o)
        w = orc.share(uniform((K, N), N), n, t, P45, 17, 4)
        y = s.linear_mod_prepacked(tiles, s.pack_weights_linear(to_dev(w)), M, K, N)
        assert np.array_equal(to_np(y), orc.linear(xs_o, w, P45))
    cases = [(1, 64, 5, 5, 7, 3, 1, 1), (2, 128, 9, 7, 65, 3, 2, 1), (1, 64, 14, 14, 64, 1, 1, 0),
             (1, 192, 6, 6, 10, 5, 1, 2), (1, 256, 14, 14, 256, 3, 1, 1), (2, 64, 72, 72, 8, 3, 1, 1)]
    for (B, C, H, W, Co, ksz, stride, pad) in cases:
        say("p45 planes conv", n, B, C, H, W, Co, ksz, stride, pad)
        x = uniform((B, C, H, W), 3)
        xs_o = orc.share(x, n, t, P45, 17, 5)
        w = orc.share(uniform((Co, C, ksz, ksz), 4), n, t, P45, 17, 6)
        want = orc.conv(xs_o, w, stride, pad, P45)
        wp = s.pack_weights_conv_taps(to_dev(w))
        xs, planes = s.share_planes(to_dev(x), stream_id=5)
        assert np.array_equal(to_np(xs), xs_o)
        assert np.array_equal(to_np(s.conv_mod_planes(planes, wp, B, C, H, W, Co, ksz, ksz, stride, pad)), want)
        planes2 = s.split_planes(xs)
        per = s.lib.ssnet_conv_planes_bytes(B, C, H, W)
        live = 6 * B * C * H * W + 16
        a, b = planes.view(n, per)[:, :live], planes2.view(n, per)[:, :live]
        assert bool(torch.equal(a, b))


@pytest.mark.parametrize("n,t", SCHEMES)
def test_p45_nonlinear(n, t):
    """ReLU, ReLU + pooling and the one-launch layer tail under the masks of Sec. VII-B (beta up to 2^28:
    inputs within 16 bits)"""
    f = 13
    s = SSNet(n, t, f=f, seed=55, p=P45)
    nr = 2 * t + 1
    for count in (1, 255, 4099, 65538, (1 << 20) + 2):
        say("p45 relu", n, t, count)
        sb, sbi = s.nonlinear_masks(count, stream_id=12)
        osb, osbi = orc.nonlinear_masks(count, n, t, 28, P45, 55, 12)
        assert np.array_equal(to_np(sb), osb) and np.array_equal(to_np(sbi), osbi)
        xs = np.random.default_rng(count).integers(-(1 << 15), 1 << 15, count, dtype=np.int64)
        xs[: min(count, 5)] = [0, (1 << 16) - 1, -((1 << 16) - 1), 1, -1][: min(count, 5)]
        x = orc.share(signed(xs), n, t, P45, 55, 13)
        want, msg, y = orc.relu(x, osb, osbi, n, t, P45, full=True)
        got = s.relu(to_dev(x), sb, sbi)
        ws = to_np(s.messages()[: (nr + 1) * count])
        assert np.array_equal(ws[: nr * count].reshape(nr, count), msg) and np.array_equal(ws[nr * count:], y)
        assert np.array_equal(to_np(got), want)
        assert np.array_equal(orc.lift(to_np(s.reconstruct(got, list(range(n, n - t - 1, -1)))), P45), np.maximum(xs, 0))
    for gi, (planes, H, W, kern, stride, pad) in enumerate([(5, 7, 5, (2, 2), (2, 2), (0, 0)), (64, 33, 31, (3, 3), (2, 2), (1, 1)),
                                                            (70, 7, 7, (7, 7), (7, 7), (0, 0))]):
        say("p45 relu_pool", n, t, planes, H, W, kern)
        geo = (H, W) + kern + stride + pad
        sb, sbi = s.pool_masks(planes, H, W, kern, stride, pad, stream_id=40 + gi)
        osb, osbi = orc.pool_masks(planes, *geo, n, t, 28, P45, 55, 40 + gi)
        assert np.array_equal(to_np(sb).reshape(n, -1), osb) and np.array_equal(to_np(sbi).reshape(n, -1), osbi)
        lim = (1 << 15) // (kern[0] * kern[1])
        xs = np.random.default_rng(gi).integers(-lim, lim, planes * H * W, dtype=np.int64)
        x = orc.share(signed(xs), n, t, P45, 55, 13)
        for mode in (SSNet.POOL_MAX, SSNet.POOL_SUM):
            want = orc.relu_pool(x, osb, osbi, planes, *geo, mode, n, t, P45)
            got = s.relu_pool(to_dev(x).view(n, planes, H, W), sb, sbi, kern, stride, pad, mode)
            assert np.array_equal(to_np(got).reshape(n, -1), want)
    for (B, C, HW) in [(1, 64, 49), (2, 128, 196), (1, 20, 17)]:
        say("p45 layer tail", n, t, B, C, HW)
        count = B * C * HW
        xs = np.random.default_rng(C).integers(-(1 << 28), 1 << 28, count, dtype=np.int64)      # before truncation
        c = orc.share(signed(xs), n, 2 * t, P45, 55, 1).reshape(n, B, C, HW)
        sb, sbi = s.nonlinear_masks((B, C, HW), stream_id=21)
        osb, osbi = orc.nonlinear_masks(count, n, t, 28, P45, 55, 21)
        yt = orc.truncate(orc.degree_reduce(c.reshape(n, -1), n, t, P45, 55, 7), n, t, f, P45, 55, 7)
        want = orc.relu(yt, osb, osbi, n, t, P45)
        got, planes = s.reduce_truncate_relu(to_dev(c), 7, sb, sbi, want_planes=(C % 64 == 0))
        assert np.array_equal(to_np(got).reshape(n, -1), want)
        if planes is not None:
            ref = s.split_planes(got.view(n, B, C, HW, 1))
            per = s.lib.ssnet_conv_planes_bytes(B, C, HW, 1)
            live = 6 * count + 16
            assert bool(torch.equal(planes.view(n, per)[:, :live], ref.view(n, per)[:, :live]))
