"""GPU-vs-oracle parity, element by element and bit-exact, through the C ABI.
Sizes span several workgroup tiles plus ragged tails; the oracle finishes each
case in well under a second."""
import itertools

import numpy as np
import pytest
import torch

import oracle as orc
from paper_2406_02629_amd import SSNet, SSNetError, binding
from util import P61, field_uniform, to_dev, to_np

pytestmark = pytest.mark.gpu

SCHEMES = [(3, 1), (5, 2), (7, 3), (5, 1), (8, 2)]
COUNTS = [1, 2, 7, 255, 256, 513, 1000, 4099, 65538]


def say(*a):
    print(*a, flush=True)


@pytest.mark.parametrize("n,t", SCHEMES)
def test_share_parity(n, t):
    s = SSNet(n, t, seed=1234)
    for count in COUNTS:
        for degree in (t, 2 * t, 0):
            if degree > n - 1:
                continue
            say("share", n, t, count, degree)
            secret = field_uniform(count, seed=count + degree)
            got = to_np(s.share(to_dev(secret), stream_id=count, degree=degree))
            want = orc.share(secret, n, degree, P61, 1234, count)
            assert np.array_equal(got, want)


@pytest.mark.parametrize("n,t", SCHEMES)
def test_reconstruct_parity(n, t):
    s = SSNet(n, t, seed=5)
    for count in (1, 513, 4099, 65538):
        shares = field_uniform((n, count), seed=count)
        d = to_dev(shares)
        subsets = list(itertools.combinations(range(1, n + 1), t + 1))[:6] + [tuple(range(1, 2 * t + 2)),
                                                                            tuple(range(n, n - t - 1, -1))]
        for ids in subsets:
            say("reconstruct", n, t, count, ids)
            deg = t if len(ids) == t + 1 else 2 * t
            got = to_np(s.reconstruct(d, list(ids), degree=deg))
            assert np.array_equal(got, orc.reconstruct(shares, list(ids), P61))


@pytest.mark.parametrize("n,t", SCHEMES)
def test_share_then_reconstruct_roundtrip(n, t):
    s = SSNet(n, t, seed=77)
    secret = field_uniform(10001, seed=3)
    sh = s.share(to_dev(secret), stream_id=9)
    for ids in ([1 + i for i in range(t + 1)], [n - i for i in range(t + 1)]):
        assert np.array_equal(to_np(s.reconstruct(sh, ids)), secret)


@pytest.mark.parametrize("n,t", SCHEMES)
def test_degree_reduce_parity_with_messages(n, t):
    s = SSNet(n, t, seed=42)
    k, nr = t + 1, 2 * t + 1
    for count in (1, 2, 513, 1000, 4099, 65538):
        say("degree_reduce", n, t, count)
        c = field_uniform((n, count), seed=count + 1)
        got = to_np(s.degree_reduce(to_dev(c), stream_id=count))
        want, msg1, msg2, red = orc.degree_reduce(c, n, t, P61, 42, count, full=True)
        ws = to_np(s.messages()[: (nr * k + k * n) * count])
        assert np.array_equal(ws[: nr * k * count].reshape(nr, k, count), msg1)
        assert np.array_equal(ws[nr * k * count:].reshape(k, n, count), msg2)
        assert np.array_equal(got, want)


@pytest.mark.parametrize("n,t", [(3, 1), (5, 2)])
def test_large_tensors_take_the_one_thread_per_element_kernels(n, t):
    # degree reduction switches kernels at 160 K elements, truncation vector width at 2^20
    s = SSNet(n, t, seed=31)
    count = (1 << 20) + 6
    c = field_uniform((n, count), seed=11)
    d = to_dev(c)
    got = to_np(s.degree_reduce(d, stream_id=2))
    want, msg1, msg2, red = orc.degree_reduce(c, n, t, P61, 31, 2, full=True)
    k, nr = t + 1, 2 * t + 1
    ws = to_np(s.messages()[: (nr * k + k * n) * count])
    assert np.array_equal(ws[: nr * k * count].reshape(nr, k, count), msg1)
    assert np.array_equal(ws[nr * k * count:].reshape(k, n, count), msg2)
    assert np.array_equal(got, want)
    xs = np.random.default_rng(4).integers(-(1 << 50), 1 << 50, count, dtype=np.int64)
    xsh = orc.share(np.where(xs < 0, xs + P61, xs).astype(np.uint64), n, t, P61, 31, 1)
    assert np.array_equal(to_np(s.truncate(to_dev(xsh), stream_id=3)), orc.truncate(xsh, n, t, 13, P61, 31, 3))


@pytest.mark.parametrize("n,t", SCHEMES)
def test_fused_reduce_truncate_equals_the_two_calls(n, t):
    s = SSNet(n, t, f=13, seed=77)
    k, nr = t + 1, 2 * t + 1
    for count in (1, 33, 4099, 65538, 200001, (1 << 20) + 2 if n == 3 else 300000):
        say("reduce+truncate", n, t, count)
        rng = np.random.default_rng(count)
        # degree-2t shares of moderate secrets, so that the truncation precondition holds
        xs = rng.integers(-(1 << 55), 1 << 55, count, dtype=np.int64)
        c = orc.share(np.where(xs < 0, xs + P61, xs).astype(np.uint64), n, 2 * t if 2 * t < n else t, P61, 5, 0)
        want_r, m1, m2, _ = orc.degree_reduce(c, n, t, P61, 77, 9, full=True)
        want, u, wsh = orc.truncate(want_r, n, t, 13, P61, 77, 9, full=True)
        d = to_dev(c)
        got = to_np(s.degree_reduce_truncate(d, stream_id=9, out=d))      # in place
        ws = to_np(s.messages()[: (nr * k + k * n + k + n) * count])
        o1, o2, o3 = nr * k * count, (nr * k + k * n) * count, (nr * k + k * n + k) * count
        assert np.array_equal(ws[:o1].reshape(nr, k, count), m1)
        assert np.array_equal(ws[o1:o2].reshape(k, n, count), m2)
        assert np.array_equal(ws[o2:o3].reshape(k, count), u)
        assert np.array_equal(ws[o3:].reshape(n, count), wsh)
        assert np.array_equal(got, want)
        assert np.array_equal(orc.lift(orc.reconstruct(got, list(range(1, t + 2)), P61), P61), xs >> 13)


@pytest.mark.parametrize("n,t", [(3, 1), (5, 2), (7, 3), (5, 1)])
def test_fused_reduce_truncate_reconstruct(n, t):
    """One launch for degree reduction, truncation and REC: shares, messages and the
    opened value against the oracle's three functions, for both kernel families."""
    s = SSNet(n, t, f=13, seed=31)
    k = t + 1
    subsets = [list(range(1, k + 1)), list(range(n, n - k, -1)), list(range(1, n + 1))]
    for count, ids in zip((1, 37, 4099, 170001, 262146), subsets + subsets):
        say("reduce+truncate+reconstruct", n, t, count, ids)
        rng = np.random.default_rng(count)
        xs = rng.integers(-(1 << 55), 1 << 55, count, dtype=np.int64)
        c = orc.share(np.where(xs < 0, xs + P61, xs).astype(np.uint64), n, 2 * t if 2 * t < n else t, P61, 6, 0)
        want = orc.truncate(orc.degree_reduce(c, n, t, P61, 31, 4), n, t, 13, P61, 31, 4)
        want_rec = orc.reconstruct(want, ids, P61)
        d = to_dev(c)
        out, rec = s.degree_reduce_truncate_reconstruct(d, stream_id=4, ids=ids, out=d)
        assert np.array_equal(to_np(out), want)
        assert np.array_equal(to_np(rec), want_rec)
        assert np.array_equal(orc.lift(want_rec, P61), xs >> 13)
        # the same residues as the two separate entry points
        sep = s.degree_reduce_truncate(to_dev(c), stream_id=4)
        assert bool(torch.equal(sep, out)) and bool(torch.equal(s.reconstruct(sep, ids), rec))
    d = to_dev(orc.share(field_uniform(8, 1), n, t, P61, 6, 0))
    for bad, code in (([1, 1] + list(range(2, k)), "EID"), ([0] + list(range(2, k + 1)), "EID"), (list(range(1, k)), "ESHARES")):
        with pytest.raises(SSNetError) as ei:
            s.degree_reduce_truncate_reconstruct(d, stream_id=1, ids=bad)
        assert ei.value.code == {"EID": -4, "ESHARES": -3}[code]


@pytest.mark.parametrize("n,t", SCHEMES)
def test_reduce_truncate_direct_gives_the_protocol_outputs(n, t):
    """The no-message shortcut writes the very residues of the protocol path (oracle: the three
    steps of RED, RERAND, the three steps of truncation), whatever the reshare randomness was."""
    s = SSNet(n, t, f=13, seed=91)
    for count in (1, 2, 4099, 65538, (1 << 20) + 2):
        say("direct", n, t, count)
        rng = np.random.default_rng(count)
        xs = rng.integers(-(1 << 55), 1 << 55, count, dtype=np.int64)
        c = orc.share(np.where(xs < 0, xs + P61, xs).astype(np.uint64), n, 2 * t if 2 * t < n else t, P61, 2, 0)
        want = orc.truncate(orc.degree_reduce(c, n, t, P61, 91, 7), n, t, 13, P61, 91, 7)
        ids = list(range(n, n - t - 1, -1))
        d = to_dev(c)
        out, rec = s.reduce_truncate_direct(d, stream_id=7, ids=ids, out=d)
        assert np.array_equal(to_np(out), want)
        assert np.array_equal(to_np(rec), orc.reconstruct(want, ids, P61))
        assert np.array_equal(orc.lift(to_np(rec), P61), xs >> 13)
        out2, none = s.reduce_truncate_direct(to_dev(c), stream_id=7)
        assert none is None and bool(torch.equal(out2, out))


def test_degree_reduce_in_place_and_on_real_products():
    n, t = 5, 2
    s = SSNet(n, t, seed=8)
    a, b = field_uniform(3000, 1), field_uniform(3000, 2)
    sa, sb = orc.share(a, n, t, P61, 8, 0), orc.share(b, n, t, P61, 8, 1)
    prod = np.array([[int(x) * int(y) % P61 for x, y in zip(ra, rb)] for ra, rb in zip(sa, sb)], np.uint64)
    d = to_dev(prod)
    out = s.degree_reduce(d, stream_id=5, out=d)                     # aliasing allowed
    want = orc.degree_reduce(prod, n, t, P61, 8, 5)
    assert np.array_equal(to_np(out), want)
    ab = np.array([int(x) * int(y) % P61 for x, y in zip(a, b)], np.uint64)
    assert np.array_equal(to_np(s.reconstruct(out, [2, 4, 5])), ab)


@pytest.mark.parametrize("n,t,f", [(3, 1, 13), (5, 2, 13), (7, 3, 8), (5, 1, 16), (3, 1, 1), (3, 1, 31)])
def test_truncate_parity(n, t, f):
    s = SSNet(n, t, f=f, seed=99)
    for count in (1, 2, 513, 4099, 65538):
        say("truncate", n, t, f, count)
        rng = np.random.default_rng(count)
        xs = rng.integers(-(1 << 58), 1 << 58, count, dtype=np.int64)
        xs[: min(count, 6)] = [0, -1, 1, (1 << f) - 1, -(1 << f), -(1 << f) - 1][: min(count, 6)]
        secret = np.where(xs < 0, xs + P61, xs).astype(np.uint64)
        xsh = orc.share(secret, n, t, P61, 99, 1)
        got = to_np(s.truncate(to_dev(xsh), stream_id=count))
        want, u, wsh = orc.truncate(xsh, n, t, f, P61, 99, count, full=True)
        ws = to_np(s.messages()[: (t + 1 + n) * count])
        assert np.array_equal(ws[: (t + 1) * count].reshape(t + 1, count), u)
        assert np.array_equal(ws[(t + 1) * count:].reshape(n, count), wsh)
        assert np.array_equal(got, want)
        rec = to_np(s.reconstruct(to_dev(got), list(range(1, t + 2))))
        assert np.array_equal(orc.lift(rec, P61), xs >> f)


LINEAR_SHAPES = [(1, 1, 1), (3, 5, 7), (16, 64, 16), (17, 65, 33), (32, 128, 32), (33, 129, 31), (64, 256, 128),
                 (100, 300, 70), (1, 2048, 100), (49, 700, 80),
                 # at most 16 rows: the 16 x 128 tile form, whole and shared tiles, ragged column tiles
                 (1, 9216, 300), (16, 1000, 257), (8, 64, 128), (2, 16383, 130), (5, 130, 1000), (16, 4096, 4096)]


@pytest.mark.parametrize("n,t", [(3, 1), (5, 2)])
def test_linear_parity(n, t):
    s = SSNet(n, t, seed=1)
    for M, K, N in LINEAR_SHAPES:
        say("linear", n, M, K, N)
        x = field_uniform((n, M, K), seed=M * 7 + K)
        w = field_uniform((n, K, N), seed=N * 3 + K)
        got = to_np(s.linear_mod(to_dev(x), to_dev(w)))
        assert np.array_equal(got, orc.linear(x, w, P61))


def test_linear_random_shapes_cover_the_unit_dealing():
    """Seeded sweep of ragged shapes: whole tiles and tiles cut between 2 to 8 workgroups, light last
    column tiles of 1 to 3 blocks, fewer units than workgroups, one party to eight."""
    rng = np.random.default_rng(2024)
    cases = [(3, 1, 1, 1, 1), (3, 1, 1, 16383, 1), (5, 2, 64, 64, 64), (5, 2, 65, 65, 65), (8, 2, 17, 700, 49),
             (3, 1, 200, 129, 3), (5, 2, 1, 2048, 1000), (7, 3, 130, 1000, 196)]
    for _ in range(24):
        n, t = [(3, 1), (5, 2), (7, 3), (5, 1)][int(rng.integers(4))]
        cases.append((n, t, int(rng.integers(1, 400)), int(rng.integers(1, 2500)), int(rng.integers(1, 400))))
    for (n, t, M, K, N) in cases:
        say("linear", n, t, M, K, N)
        s = SSNet(n, t, seed=3)
        x, w = field_uniform((n, M, K), M + K), field_uniform((n, K, N), N + K)
        y = s.linear_mod(to_dev(x), to_dev(w))
        assert np.array_equal(to_np(y), orc.linear(x, w, P61)), (n, t, M, K, N)


def test_linear_many_tiles_one_whole_tile_per_workgroup():
    # 3 * 130 * 130 output tiles: many more than compute units, so every workgroup takes one whole tile (one plane)
    n, t = 3, 1
    s = SSNet(n, t, seed=1)
    M, K, N = 8320, 64, 8320
    x, w = field_uniform((n, M, K), 41), field_uniform((n, K, N), 42)
    y = s.linear_mod(to_dev(x), to_dev(w))
    rows = np.r_[0:24, 4000:4024, M - 24:M]
    got = to_np(y[:, torch.from_numpy(rows).cuda()])
    assert np.array_equal(got, orc.linear(np.ascontiguousarray(x[:, rows]), w, P61))


def test_linear_extreme_operands():
    # all digits at their extremes: p-1 everywhere, and the values whose balanced
    # digits are all -128 / all +127, at the longest contraction the int32
    # accumulators are sized for
    n, t = 3, 1
    s = SSNet(n, t, seed=1)
    all_neg = 0x007F7F7F7F7F7F80        # digits: seven times -128, then +1
    all_pos = 0x1F7F7F7F7F7F7F7F        # digits: seven times +127, then +31
    for K in (64, 4608, 16383):
        for xv, wv in ((P61 - 1, P61 - 1), (all_neg, all_neg), (all_pos, all_pos), (all_neg, all_pos)):
            say("linear extreme", K, hex(xv), hex(wv))
            x = np.full((n, 2, K), xv, np.uint64)
            w = np.full((n, K, 3), wv, np.uint64)
            got = to_np(s.linear_mod(to_dev(x), to_dev(w)))
            assert np.all(got == np.uint64(K * xv * wv % P61))


def test_linear_packed_weights_identical():
    n, t = 5, 2
    s = SSNet(n, t, seed=1)
    M, K, N = 37, 190, 45
    x, w = field_uniform((n, M, K), 5), field_uniform((n, K, N), 6)
    wd = to_dev(w)
    packed = s.pack_weights_linear(wd)
    a = to_np(s.linear_mod_packed(to_dev(x), packed, N))
    assert np.array_equal(a, orc.linear(x, w, P61))
    assert np.array_equal(a, to_np(s.linear_mod(to_dev(x), wd)))


CONV_CASES = [  # B, C, H, W, Co, k, stride, pad
    (1, 3, 8, 8, 4, 3, 1, 1), (2, 5, 9, 7, 6, 3, 2, 1), (1, 16, 14, 14, 32, 1, 1, 0), (1, 8, 15, 15, 8, 1, 2, 0),
    (1, 3, 20, 20, 16, 7, 2, 3), (3, 4, 6, 6, 40, 3, 1, 1), (1, 70, 5, 5, 33, 3, 1, 1), (2, 2, 4, 4, 2, 4, 1, 0),
    (1, 64, 14, 14, 64, 3, 1, 1)]


@pytest.mark.parametrize("n,t", [(3, 1), (5, 2)])
def test_conv_parity(n, t):
    s = SSNet(n, t, seed=1)
    for (B, Ci, H, W, Co, k, stride, pad) in CONV_CASES:
        say("conv", n, B, Ci, H, W, Co, k, stride, pad)
        x = field_uniform((n, B, Ci, H, W), seed=H + Ci)
        w = field_uniform((n, Co, Ci, k, k), seed=Co + k)
        got = to_np(s.conv_mod(to_dev(x), to_dev(w), stride, pad))
        want = orc.conv(x, w, stride, pad, P61)
        assert got.shape == want.shape
        assert np.array_equal(got, want)
        packed = s.pack_weights_conv(to_dev(w))
        got2 = to_np(s.conv_mod_packed(to_dev(x), packed, Co, k, k, stride, pad))
        assert np.array_equal(got2, want)


@pytest.mark.parametrize("n,t", [(3, 1), (5, 2), (7, 3)])
def test_share_packed_and_prepacked_layers(n, t):
    """GEN fused with the limb split: shares against the oracle, tiles against the
    separate pack call (through identical layer outputs), dense and 1x1 conv."""
    s = SSNet(n, t, seed=21)
    # conv input [B][C][H][W], ragged in every direction
    for (B, C, H, W, Co) in [(1, 3, 5, 7, 2), (2, 70, 9, 9, 33), (1, 128, 14, 14, 64), (3, 64, 1, 1, 17)]:
        say("share_packed conv", n, t, B, C, H, W, Co)
        x = field_uniform(B * C * H * W, 3).reshape(B, C, H, W)
        want = orc.share(x, n, t, P61, 21, 6)
        xs, tiles = s.share_packed(to_dev(x), stream_id=6)
        assert np.array_equal(to_np(xs), want)
        assert bool(torch.equal(xs, s.share(to_dev(x), stream_id=6)))
        w = orc.share(field_uniform(Co * C, 4).reshape(Co, C, 1, 1), n, t, P61, 21, 7)
        wp = s.pack_weights_conv(to_dev(w))
        y = s.conv1x1_mod_prepacked(tiles, wp, B, C, H, W, Co)
        assert np.array_equal(to_np(y), orc.conv(want, w, 1, 0, P61))
        assert bool(torch.equal(y, s.conv_mod_packed(xs, wp, Co, 1, 1, 1, 0)))
    for (M, K, N) in [(1, 1, 1), (5, 100, 9), (1, 2048, 1000), (130, 64, 65)]:
        say("share_packed dense", n, t, M, K, N)
        x = field_uniform(M * K, 5).reshape(M, K)
        want = orc.share(x, n, t, P61, 21, 8)
        xs, tiles = s.share_packed(to_dev(x), stream_id=8)
        assert np.array_equal(to_np(xs), want)
        w = orc.share(field_uniform(K * N, 6).reshape(K, N), n, t, P61, 21, 9)
        y = s.linear_mod_prepacked(tiles, s.pack_weights_linear(to_dev(w)), M, K, N)
        assert np.array_equal(to_np(y), orc.linear(want, w, P61))


@pytest.mark.parametrize("n,t", SCHEMES)
def test_relu_parity_with_masks_and_messages(n, t):
    """SSS-NonLinear: the trusted source's mask shares, the 2t+1 masked products, the elite
    party's plain value and the output shares, all against the oracle."""
    s = SSNet(n, t, seed=55)
    nr = 2 * t + 1
    for count in (1, 2, 255, 4099, 65538):
        say("relu", n, t, count)
        sb, sbi = s.nonlinear_masks(count, stream_id=12)
        osb, osbi = orc.nonlinear_masks(count, n, t, 28, P61, 55, 12)
        assert np.array_equal(to_np(sb), osb) and np.array_equal(to_np(sbi), osbi)
        rng = np.random.default_rng(count)
        xs = rng.integers(-(1 << 31), 1 << 31, count, dtype=np.int64)
        xs[: min(count, 5)] = [0, (1 << 32) - 1, -((1 << 32) - 1), 1, -1][: min(count, 5)]
        x = orc.share(np.where(xs < 0, xs + P61, xs).astype(np.uint64), n, t, P61, 55, 13)
        want, msg, y = orc.relu(x, osb, osbi, n, t, P61, full=True)
        d = to_dev(x)
        got = s.relu(d, sb, sbi, out=d)                                  # in place
        ws = to_np(s.messages()[: (nr + 1) * count])
        assert np.array_equal(ws[: nr * count].reshape(nr, count), msg)
        assert np.array_equal(ws[nr * count:], y)
        assert np.array_equal(to_np(got), want)
        assert np.array_equal(to_np(s.reconstruct(got, list(range(n, n - t - 1, -1)))).astype(np.int64),
                              np.maximum(xs, 0))


@pytest.mark.parametrize("n,t", [(3, 1), (5, 2), (7, 3)])
def test_conv_on_limb_planes(n, t):
    """Convolution that gathers its input from channel-innermost limb planes (no im2col matrix):
    the same residues as the oracle's convolution, for planes made from shares and for planes
    made together with the shares; strides, paddings, ragged pixel counts, several images."""
    s = SSNet(n, t, seed=17)
    cases = [(1, 64, 5, 5, 7, 3, 1, 1), (2, 128, 9, 7, 65, 3, 2, 1), (1, 64, 14, 14, 64, 1, 1, 0),
             (1, 192, 6, 6, 10, 5, 1, 2), (3, 64, 4, 4, 130, 3, 1, 1), (1, 256, 14, 14, 256, 3, 1, 1),
             (1, 64, 8, 8, 16, 2, 2, 0), (1, 64, 3, 3, 5, 3, 1, 0),
             (2, 64, 72, 72, 8, 3, 1, 1)]            # > 2^19 elements: the four-channels-per-thread kernels
    for (B, C, H, W, Co, k, stride, pad) in cases:
        say("planes conv", n, t, B, C, H, W, Co, k, stride, pad)
        x = field_uniform(B * C * H * W, 3).reshape(B, C, H, W)
        xs_o = orc.share(x, n, t, P61, 17, 5)
        w = orc.share(field_uniform(Co * C * k * k, 4).reshape(Co, C, k, k), n, t, P61, 17, 6)
        want = orc.conv(xs_o, w, stride, pad, P61)
        wp = s.pack_weights_conv_taps(to_dev(w))
        xs, planes = s.share_planes(to_dev(x), stream_id=5)
        assert np.array_equal(to_np(xs), xs_o)
        y = s.conv_mod_planes(planes, wp, B, C, H, W, Co, k, k, stride, pad)
        assert np.array_equal(to_np(y), want)
        planes2 = s.split_planes(to_dev(xs_o))                          # planes of existing shares: same bytes
        per = planes.numel() // n
        data = 8 * B * C * H * W + 16                                   # the rest of the pad is unspecified
        assert bool(torch.equal(planes2.view(n, per)[:, :data], planes.view(n, per)[:, :data]))
        # extreme digits everywhere: all limbs at -128 / +127, and p - 1
    for v in (P61 - 1, 0x0080808080808080, 0x007F7F7F7F7F7F7F):
        B, C, H, W, Co, k = 1, 64 * 8, 6, 6, 33, 3        # K = 4608
        x = np.full((n, B, C, H, W), v, np.uint64)
        w = np.full((n, Co, C, k, k), v, np.uint64)
        y = s.conv_mod_planes(s.split_planes(to_dev(x)), s.pack_weights_conv_taps(to_dev(w)), B, C, H, W, Co, k, k, 1, 1)
        assert np.array_equal(to_np(y), orc.conv(x, w, 1, 1, P61))
    assert not s.planes_supported(1, 3, 8, 8) and not s.planes_supported(1, 96, 8, 8)


@pytest.mark.parametrize("n,t", [(3, 1), (5, 2), (7, 3)])
def test_layer_tail_in_one_launch(n, t):
    """Reduction + RERAND + truncation + ReLU of a layer's product shares in one launch: output shares,
    every message of the three protocols, and the limb planes (through the next convolution) against the
    oracle's separate steps.  (7,3) takes the library's three-launch route behind the same entry point."""
    s = SSNet(n, t, f=13, seed=63)
    k, nr = t + 1, 2 * t + 1
    # the last case is past half a million elements, where the planes are written by a launch of their own
    for (B, C, H, W) in [(1, 64, 3, 5), (2, 128, 7, 7), (1, 20, 4, 4), (1, 64, 40, 40), (1, 64, 96, 96)]:
        say("layer tail", n, t, B, C, H, W)
        count = B * C * H * W
        rng = np.random.default_rng(count)
        xs = rng.integers(-(1 << 43), 1 << 43, count, dtype=np.int64)
        c = orc.share(np.where(xs < 0, xs + P61, xs).astype(np.uint64), n, 2 * t if 2 * t < n else t, P61, 8, 0)
        sb, sbi = s.nonlinear_masks((B, C, H, W), stream_id=21)
        osb, osbi = orc.nonlinear_masks(count, n, t, 28, P61, 63, 21)
        yr, m1, m2, _ = orc.degree_reduce(c, n, t, P61, 63, 5, full=True)
        yt, u, wsh = orc.truncate(yr, n, t, 13, P61, 63, 5, full=True)
        want, rmsg, yplain = orc.relu(yt, osb, osbi, n, t, P61, full=True)
        d = to_dev(c.reshape(n, B, C, H, W))
        out, planes = s.reduce_truncate_relu(d, 5, sb, sbi, out=d, want_planes=(C % 64 == 0))
        assert np.array_equal(to_np(out).reshape(n, -1), want)
        assert np.array_equal(orc.lift(orc.reconstruct(want, list(range(1, k + 1)), P61), P61), np.maximum(xs >> 13, 0))
        # message planes of P positions; for the one-kernel schemes in the order of that kernel's threads
        P = s.lib.ssnet_layer_tail_message_plane(s._ctx, B, C, H * W)
        cc, pix = np.meshgrid(np.arange(C), np.arange(B * H * W), indexing="ij")
        bb, hw = pix // (H * W), pix % (H * W)
        elem = ((bb * C + cc) * (H * W) + hw).reshape(-1)
        if (n, t) not in ((3, 1), (5, 2)):          # three launches, element order
            assert P == count
            pos = elem
        else:
            pos = (((cc // 16) * ((B * H * W + 15) // 16) + pix // 16) * 256 + (cc % 16 // 4) * 64 + (cc % 4) * 16
                   + pix % 16).reshape(-1)
        ws = to_np(s.messages()[: (nr * k + k * n + k + n + nr + 1) * P])
        o = np.cumsum([0, nr * k, k * n, k, n, nr, 1]) * P
        for got, ref in zip([ws[o[i]:o[i + 1]] for i in range(6)], (m1, m2, u, wsh, rmsg, yplain)):
            got, ref = got.reshape(-1, P), ref.reshape(-1, count)
            assert np.array_equal(got[:, pos], ref[:, elem])
        if planes is not None:   # the planes feed a convolution: same result as the convolution on the shares
            w = orc.share(field_uniform(9 * C * 9, 4).reshape(9, C, 3, 3), n, t, P61, 63, 6)
            y = s.conv_mod_planes(planes, s.pack_weights_conv_taps(to_dev(w)), B, C, H, W, 9, 3, 3, 1, 1)
            assert np.array_equal(to_np(y), orc.conv(want.reshape(n, B, C, H, W), w, 1, 1, P61))
        # the one-pass form without messages gives the protocol's residues, in place as well
        d2 = to_dev(c.reshape(n, B, C, H, W))
        out2, planes2 = s.reduce_truncate_relu_direct(d2, sb, sbi, out=d2, want_planes=(C % 64 == 0))
        assert np.array_equal(to_np(out2).reshape(n, -1), want)
        if planes is not None:
            data = 8 * count + 16
            per = planes.numel() // n
            assert bool(torch.equal(planes2.view(n, per)[:, :data], planes.view(n, per)[:, :data]))


def test_config1_tiny_secure_gemm_end_to_end():
    """n=3, t=1, f=13, X 64x256 ~ N(0,1), W 256x128 ~ N(0,1): share, multiply,
    reduce, truncate, reconstruct, decode."""
    from paper_2406_02629_amd import fixedpoint as fx
    from ssnet_inputs import gaussian
    n, t, f, seed = 3, 1, 13, 2024
    X, Wt = gaussian((64, 256), 1), gaussian((256, 128), 2)
    s = SSNet(n, t, f=f, seed=seed)
    xe = fx.encode(torch.from_numpy(X).cuda(), f)
    we = fx.encode(torch.from_numpy(Wt).cuda(), f)
    assert np.array_equal(to_np(xe), orc.encode(X, f, P61)) and np.array_equal(to_np(we), orc.encode(Wt, f, P61))
    xs, ws = s.share(xe, stream_id=1), s.share(we, stream_id=2)
    y2 = s.linear_mod(xs, ws)
    yr = s.degree_reduce(y2.view(n, -1), stream_id=3)
    yt = s.truncate(yr, stream_id=4)
    rec = s.reconstruct(yt, [1, 2]).view(64, 128)
    # oracle pipeline on the same seeds
    oxs, ows = orc.share(orc.encode(X, f, P61), n, t, P61, seed, 1), orc.share(orc.encode(Wt, f, P61), n, t, P61, seed, 2)
    assert np.array_equal(to_np(xs), oxs) and np.array_equal(to_np(ws), ows)
    oy2 = orc.linear(oxs, ows, P61)
    assert np.array_equal(to_np(y2), oy2)
    oyr = orc.degree_reduce(oy2.reshape(n, -1), n, t, P61, seed, 3)
    assert np.array_equal(to_np(yr), oyr)
    oyt = orc.truncate(oyr, n, t, f, P61, seed, 4)
    assert np.array_equal(to_np(yt), oyt)
    orec = orc.reconstruct(oyt, [1, 2], P61)
    assert np.array_equal(to_np(rec).reshape(-1), orec)
    # every pair of parties agrees
    for ids in ([2, 3], [1, 3]):
        assert torch.equal(s.reconstruct(yt, ids).view(64, 128), rec)
    dec = fx.decode(rec, f).cpu().numpy()
    exact = orc.decode(orc.encode(X, f, P61), f, P61) @ orc.decode(orc.encode(Wt, f, P61), f, P61)
    err = exact - dec
    assert err.min() >= 0 and err.max() < 2.0 ** -f                  # floor truncation of exact product
    assert np.max(np.abs(dec - X @ Wt)) < 2.0 ** -8                  # vs float64 plaintext


def test_errors_surface_as_codes_not_crashes():
    s = SSNet(3, 1, seed=1)
    x = to_dev(field_uniform((3, 16), 1))
    with pytest.raises(SSNetError) as ei:
        s.reconstruct(x, [1], degree=1)
    assert ei.value.code == binding.ESHARES
    with pytest.raises(SSNetError) as ei:
        s.reconstruct(x, [1, 4], degree=1)
    assert ei.value.code == binding.EID


@pytest.mark.parametrize("n,t", SCHEMES)
def test_truncate_div_parity(n, t):
    """Truncation with the rounding division of average pooling (Sec. VI-C, App. C): result and
    messages against the oracle, alone and fused behind the degree reduction."""
    f = 13
    s = SSNet(n, t, f=f, seed=31)
    for count, kdiv in ((1, 4), (513, 1), (4099, 9), (65538, 49), (70001, 4096), (300001, 4), ((1 << 20) + 2, 49)):
        say("truncate_div", n, t, count, kdiv)
        rng = np.random.default_rng(count)
        xs = rng.integers(-(1 << 57), 1 << 57, count, dtype=np.int64)
        edge = [0, -1, 1, (kdiv << f) // 2 - 1, (kdiv << f) // 2, -((kdiv << f) // 2), -((kdiv << f) // 2) - 1]
        xs[: min(count, 7)] = edge[: min(count, 7)]
        xsh = orc.share(np.where(xs < 0, xs + P61, xs).astype(np.uint64), n, t, P61, 31, 1)
        got = to_np(s.truncate_div(to_dev(xsh), kdiv, stream_id=count))
        want, u, wsh = orc.truncate_div(xsh, n, t, f, kdiv, P61, 31, count, full=True)
        ws = to_np(s.messages()[: (t + 1 + n) * count])
        assert np.array_equal(ws[: (t + 1) * count].reshape(t + 1, count), u)
        assert np.array_equal(ws[(t + 1) * count:].reshape(n, count), wsh)
        assert np.array_equal(got, want)
        rec = orc.lift(to_np(s.reconstruct(to_dev(got), list(range(n - t, n + 1)))), P61)
        assert np.array_equal(rec, ((xs >> f) + kdiv // 2) // kdiv)
        if count > 100000 and (n, t) not in ((3, 1), (5, 2)):
            continue
        # behind the reduction: product-degree shares in, one launch
        c = orc.share(np.where(xs < 0, xs + P61, xs).astype(np.uint64), n, 2 * t, P61, 31, 2)
        got2 = to_np(s.degree_reduce_truncate_div(to_dev(c), kdiv, stream_id=7))
        want2 = orc.truncate_div(orc.degree_reduce(c, n, t, P61, 31, 7), n, t, f, kdiv, P61, 31, 7)
        assert np.array_equal(got2, want2)


POOL_GEOMS = [
    # planes, H, W, kernel, stride, pad
    (3, 6, 6, (2, 2), (2, 2), (0, 0)),
    (5, 7, 5, (2, 2), (2, 2), (0, 0)),           # ragged edges
    (4, 9, 9, (3, 3), (2, 2), (1, 1)),           # overlapping kernels
    (70, 7, 7, (7, 7), (7, 7), (0, 0)),          # global pooling
    (2, 8, 6, (3, 2), (1, 2), (0, 1)),           # unequal per axis
    (1, 1, 1, (1, 1), (1, 1), (0, 0)),
    (64, 33, 31, (3, 3), (2, 2), (1, 1)),        # several blocks, ragged
    (16, 40, 40, (2, 2), (2, 2), (0, 0)),
]


@pytest.mark.parametrize("n,t", [(3, 1), (5, 2), (7, 3), (5, 1)])
def test_relu_pool_parity_with_masks_and_messages(n, t):
    """SSS-NonLinear with pooling: mask shares (beta equal inside a pooling kernel), masked
    products, the elite party's rectified and pooled plain values, output shares; against the
    oracle and, opened, against torch's pooling of the plain input."""
    s = SSNet(n, t, seed=77)
    nr = 2 * t + 1
    for gi, (planes, H, W, kern, stride, pad) in enumerate(POOL_GEOMS):
        say("relu_pool", n, t, planes, H, W, kern, stride, pad)
        geo = (H, W) + kern + stride + pad
        sb, sbi = s.pool_masks(planes, H, W, kern, stride, pad, stream_id=40 + gi)
        osb, osbi = orc.pool_masks(planes, *geo, n, t, 28, P61, 77, 40 + gi)
        assert np.array_equal(to_np(sb).reshape(n, -1), osb) and np.array_equal(to_np(sbi).reshape(n, -1), osbi)
        Ho, Wo = sbi.shape[-2], sbi.shape[-1]
        cin, cout = planes * H * W, planes * Ho * Wo
        rng = np.random.default_rng(gi)
        xs = rng.integers(-(1 << 25), 1 << 25, (planes, H, W), dtype=np.int64)
        xs.reshape(-1)[: min(cin, 3)] = [0, 1, -1][: min(cin, 3)]
        x = orc.share(np.where(xs < 0, xs + P61, xs).astype(np.uint64).reshape(-1), n, t, P61, 77, 13)
        xt = torch.from_numpy(xs).clamp(min=0).to(torch.float64)[None]
        for mode in (SSNet.POOL_MAX, SSNet.POOL_SUM):
            want, msg, y = orc.relu_pool(x, osb, osbi, planes, *geo, mode, n, t, P61, full=True)
            got = s.relu_pool(to_dev(x).view(n, planes, H, W), sb, sbi, kern, stride, pad, mode)
            assert tuple(got.shape) == (n, planes, Ho, Wo)
            ws = to_np(s.messages()[: (nr + 1) * cin + cout])
            assert np.array_equal(ws[: nr * cin].reshape(nr, cin), msg)
            # the rectified products before pooling: the elementwise protocol's plain value
            _, _, r = orc.relu(x, osb, np.zeros_like(osb), n, t, P61, full=True)
            assert np.array_equal(ws[nr * cin: (nr + 1) * cin], r)
            assert np.array_equal(ws[(nr + 1) * cin:], y)
            assert np.array_equal(to_np(got).reshape(n, -1), want)
            if mode == SSNet.POOL_MAX:
                ref = torch.nn.functional.max_pool2d(xt, kern, stride, pad)[0]
            else:
                ref = torch.nn.functional.avg_pool2d(xt, kern, stride, pad)[0] * (kern[0] * kern[1])
            opened = orc.lift(to_np(s.reconstruct(got, list(range(n, n - t - 1, -1)))), P61)
            assert np.array_equal(opened.reshape(planes, Ho, Wo), ref.round().to(torch.int64).numpy())


def test_relu_pool_stem_size():
    """The two pooling points of the ResNet stacks at full size (n = 5, t = 2): 3x3 / 2 padding 1 on
    64 x 112 x 112 and the global sum on 2048 x 7 x 7 after the truncation with kdiv = 49."""
    n, t, f = 5, 2, 13
    s = SSNet(n, t, f=f, seed=8)
    for planes, H, kern, stride, pad, mode, kdiv in ((64, 112, (3, 3), (2, 2), (1, 1), SSNet.POOL_MAX, 1),
                                                     (2048, 7, (7, 7), (7, 7), (0, 0), SSNet.POOL_SUM, 49)):
        say("relu_pool full size", planes, H, kern)
        geo = (H, H) + kern + stride + pad
        rng = np.random.default_rng(planes)
        xs = rng.integers(-(1 << 39), 1 << 39, planes * H * H, dtype=np.int64)       # before truncation
        c = orc.share(np.where(xs < 0, xs + P61, xs).astype(np.uint64), n, 2 * t, P61, 8, 1)
        xt = s.degree_reduce_truncate_div(to_dev(c), kdiv, stream_id=2)
        oxt = orc.truncate_div(orc.degree_reduce(c, n, t, P61, 8, 2), n, t, f, kdiv, P61, 8, 2)
        assert np.array_equal(to_np(xt), oxt)
        sb, sbi = s.pool_masks(planes, H, H, kern, stride, pad, stream_id=3)
        osb, osbi = orc.pool_masks(planes, *geo, n, t, 28, P61, 8, 3)
        assert np.array_equal(to_np(sb).reshape(n, -1), osb) and np.array_equal(to_np(sbi).reshape(n, -1), osbi)
        got = s.relu_pool(xt.view(n, planes, H, H), sb, sbi, kern, stride, pad, mode)
        want = orc.relu_pool(oxt, osb, osbi, planes, *geo, mode, n, t, P61)
        assert np.array_equal(to_np(got).reshape(n, -1), want)
        q = torch.from_numpy(((xs >> f) + kdiv // 2) // kdiv).clamp(min=0).to(torch.float64).view(1, planes, H, H)
        ref = (torch.nn.functional.max_pool2d(q, kern, stride, pad) if mode == SSNet.POOL_MAX
               else torch.nn.functional.avg_pool2d(q, kern, stride, pad) * (kern[0] * kern[1]))
        opened = orc.lift(to_np(s.reconstruct(got, [1, 3, 5])), P61)
        assert np.array_equal(opened.reshape(-1), ref.round().to(torch.int64).numpy().reshape(-1))
