"""CPU-only checks of the GPU library: it loads, exports the whole C ABI, and
its host-side logic (tables, generator, argument checks) is right.  No kernel
is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle as orc
from paper_2406_02629_amd import SSNet, SSNetError, binding

P61 = (1 << 61) - 1
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "ssnet.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(ssnet_[a-z0-9_]+)\s*\(", header))
    assert len(declared) >= 20
    lib = binding.load_library()
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(binding.SIGNATURES), declared ^ set(binding.SIGNATURES)


def test_create_rejects_bad_parameters():
    for args, code in [((3, 1, 11, 13, 0), binding.EPRIME), ((2, 1, P61, 13, 0), binding.EINVAL),
                       ((4, 2, P61, 13, 0), binding.EINVAL), ((9, 1, P61, 13, 0), binding.EINVAL),
                       ((3, 0, P61, 13, 0), binding.EINVAL), ((3, 1, P61, 0, 0), binding.EINVAL),
                       ((3, 1, P61, 32, 0), binding.EINVAL), ((9, 4, P61, 13, 0), binding.EINVAL)]:
        n, t, p, f, seed = args
        with pytest.raises(SSNetError) as ei:
            SSNet(n, t, f=f, seed=seed, p=p, device=None)
        assert ei.value.code == code, args
    assert binding.load_library().ssnet_create(None, 3, 1, P61, 13, 0, None) == binding.EINVAL


def test_null_and_range_checks_before_any_launch():
    s = SSNet(5, 2, device=None)
    lib, ctx = s.lib, s._ctx
    ids = (C.c_int * 3)(1, 2, 3)
    assert lib.ssnet_share(ctx, None, 8, 2, 0, None) == binding.EINVAL
    assert lib.ssnet_share(ctx, 16, 0, 2, 0, 16) == binding.EINVAL
    assert lib.ssnet_share(ctx, 16, 8, 5, 0, 16) == binding.EINVAL            # degree > 2t
    assert lib.ssnet_reconstruct(ctx, 16, 8, ids, 3, 4, 16) == binding.ESHARES   # 3 shares, degree 4
    assert lib.ssnet_reconstruct(ctx, 16, 8, (C.c_int * 3)(1, 2, 6), 3, 2, 16) == binding.EID
    assert lib.ssnet_reconstruct(ctx, 16, 8, (C.c_int * 3)(1, 2, 2), 3, 2, 16) == binding.EID
    assert lib.ssnet_reconstruct(ctx, 16, 8, (C.c_int * 3)(0, 1, 2), 3, 2, 16) == binding.EID
    assert lib.ssnet_degree_reduce(ctx, 16, 8, 0, 16) == binding.EWORKSPACE
    assert lib.ssnet_truncate(ctx, 16, 8, 0, 16) == binding.EWORKSPACE
    # the entry point with the fixed message array: (8 MiB / 8) / 30 words per element at n = 5, t = 2
    assert lib.ssnet_degree_reduce_static(ctx, 16, 34953, 0, 16) == binding.ESCRATCH
    assert lib.ssnet_degree_reduce_static(ctx, None, 8, 0, 16) == binding.EINVAL
    assert b"fixed scratch" in lib.ssnet_strerror(binding.ESCRATCH)
    assert lib.ssnet_linear_mod(ctx, 16, 16, 4, 4, 4, 16) == binding.EWORKSPACE
    assert lib.ssnet_linear_mod(ctx, 16, 16, 4, 16384, 4, 16) == binding.EINVAL   # K too long for int32
    assert lib.ssnet_linear_mod(ctx, 16, 16, 0, 4, 4, 16) == binding.EINVAL
    assert lib.ssnet_conv_mod(ctx, 16, 16, 1, 3, 4, 4, 2, 5, 5, 1, 0, 16) == binding.EINVAL  # kernel > input
    assert lib.ssnet_conv_mod(ctx, 16, 16, 1, 3, 8, 8, 2, 3, 3, 1, 1, 16) == binding.EWORKSPACE
    assert lib.ssnet_set_workspace(ctx, 8, 64) == binding.EINVAL                   # misaligned
    assert lib.ssnet_strerror(binding.ESHARES) == b"too few shares for this degree"


def test_workspace_sizes():
    s = SSNet(5, 2, device=None)
    # RED messages: [2t+1][k][count] + [k][n][count] field elements
    hdr = binding.WS_HEADER_BYTES
    assert s.workspace_bytes_stream(1000) >= hdr + (5 * 3 + 3 * 5) * 1000 * 8
    s3 = SSNet(3, 1, device=None)
    # reduction messages [3][2] + [2][3] and truncation messages [2] + [3] planes of 2^20 elements
    assert s3.workspace_bytes_stream(1 << 20) == hdr + ((3 * 2 + 2 * 3 + 2 + 3) * 8 << 20)
    # limb tiles: 8 bytes per element, rows padded to 16 and K to 64
    assert s3.lib.ssnet_packed_weight_bytes(16, 64) == 8192
    assert s3.lib.ssnet_packed_weight_bytes(17, 65) == 4 * 8192
    # limb tiles of both operands, plus room for the residues of tiles shared between workgroups
    assert s3.workspace_bytes_linear(64, 256, 128) >= hdr + 3 * (64 * 256 * 8 + 128 * 256 * 8)
    assert s3.workspace_bytes_linear(64, 64, 64) >= hdr + 3 * (64 * 64 * 8 + 64 * 64 * 8)
    assert s3.workspace_bytes_linear(64, 64, 64) < hdr + (1 << 20)


@pytest.mark.parametrize("n,t", [(3, 1), (5, 2), (7, 3), (5, 1), (8, 3)])
def test_host_tables_match_oracle(n, t):
    s = SSNet(n, t, device=None)
    assert s.host_reduction_matrix() == [[int(v) for v in r] for r in orc.red_matrix(n, t, P61)]
    import itertools
    for m in (t + 1, 2 * t + 1):
        for ids in list(itertools.combinations(range(1, n + 1), m))[:12]:
            assert s.host_lagrange(ids) == [int(v) for v in orc.lagrange(list(ids), P61)]
    perm = list(range(n, 0, -1))[: t + 1]
    assert s.host_lagrange(perm) == [int(v) for v in orc.lagrange(perm, P61)]


def test_generator_matches_golden_vectors():
    path = os.path.join(ROOT, "tests", "golden", "rng_vectors.txt")
    nkeys = ndraws = 0
    for line in open(path):
        parts = line.split()
        if not parts or parts[0].startswith("#"):
            continue
        if parts[0] == "key":
            vals = [int(v) for v in parts[1:]]
            assert binding.rng_key(*vals[:5]) == vals[5]
            nkeys += 1
        elif parts[0] == "draw":
            key, e, out, fld = (int(v) for v in parts[1:])
            assert binding.rng_draw(key, e) == out
            assert binding.rng_field(key, e) == fld
            ndraws += 1
    assert nkeys == 8 and ndraws == 32
    want = [int(l, 16) for l in open(os.path.join(ROOT, "tests", "golden", "splitmix64.txt")) if l.startswith("0x")]
    assert [binding.rng_draw(0, e) for e in range(3)] == want


def test_bench_refuses_more_than_one_gpu():
    """every box has one GPU: bench.py --gpus N with N > 1 exits with a message, before touching a device"""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "one GPU" in (r.stderr + r.stdout)


def test_new_entry_points_check_their_arguments():
    lib = binding.load_library()
    s = SSNet(5, 2, device=None)
    ctx = s._ctx
    # limb planes need a channel count that is a multiple of 64
    assert lib.ssnet_conv_planes_bytes(1, 64, 8, 8) == 8 * 64 * 64 + 256
    assert lib.ssnet_conv_planes_bytes(1, 3, 8, 8) == 0 and lib.ssnet_conv_planes_bytes(1, 96, 8, 8) == 0
    assert lib.ssnet_share_planes(ctx, 16, 1, 3, 8, 8, 0, 16, 16) == binding.EINVAL
    assert lib.ssnet_conv_mod_planes(ctx, 16, 16, 1, 64, 8, 8, 4, 3, 3, 1, 1, 16) == binding.EWORKSPACE
    assert lib.ssnet_conv_mod_planes(ctx, 16, 16, 1, 64, 2, 2, 4, 3, 3, 1, 0, 16) == binding.EINVAL   # kernel > input
    assert lib.ssnet_share_packed(ctx, 16, 0, 4, 4, 0, 16, 16) == binding.EINVAL
    assert lib.ssnet_relu(ctx, 16, 16, 16, 0, 16) == binding.EINVAL
    assert lib.ssnet_relu(ctx, 16, 16, 16, 100, 16) == binding.EWORKSPACE
    assert lib.ssnet_nonlinear_masks(ctx, 0, 1, 16, 16) == binding.EINVAL
    assert lib.ssnet_reduce_truncate_relu(ctx, 16, 1, 64, 16, 0, 16, 16, 16, 8) == binding.EINVAL    # misaligned planes
    assert lib.ssnet_reduce_truncate_relu(ctx, 16, 1, 32, 16, 0, 16, 16, 16, 16) == binding.EINVAL   # planes need C % 64 == 0
    assert lib.ssnet_reduce_truncate_relu(ctx, 16, 1, 32, 16, 0, 16, 16, 16, None) == binding.EWORKSPACE
    # message planes of the one-launch layer tail count padded 16 x 16 blocks
    assert lib.ssnet_layer_tail_message_plane(ctx, 1, 20, 17) == 2 * 2 * 256
    s7 = SSNet(7, 3, device=None)
    assert s7.lib.ssnet_layer_tail_message_plane(s7._ctx, 1, 20, 17) == 20 * 17
    ids = (C.c_int * 3)(1, 1, 2)
    assert lib.ssnet_reduce_truncate_direct(ctx, 16, 8, 0, 16, ids, 3, 16) == binding.EID


def test_product_entry_points_check_their_arguments():
    lib = binding.load_library()
    s = SSNet(5, 2, device=None)
    ctx = s._ctx
    # a product that one workgroup per tile computes whole is one plane of n * count elements
    assert lib.ssnet_product_bytes_linear(ctx, 64, 64, 64) == 5 * 64 * 64 * 8
    # 196 x 2304 x 256: 80 tiles of 36 k blocks for 256 workgroups, so several planes
    one = 5 * 196 * 256 * 8
    assert lib.ssnet_product_bytes_conv(ctx, 1, 256, 14, 14, 256, 3, 3, 1, 1) % 256 == 0
    assert 2 * one <= lib.ssnet_product_bytes_conv(ctx, 1, 256, 14, 14, 256, 3, 3, 1, 1) <= 8 * one
    assert lib.ssnet_product_bytes_linear(ctx, 0, 4, 4) == 0 and lib.ssnet_product_bytes_linear(ctx, 4, 16384, 4) == 0
    assert lib.ssnet_product_bytes_conv(ctx, 1, 3, 4, 4, 2, 5, 5, 1, 0) == 0                  # kernel > input
    assert lib.ssnet_linear_product_prepacked(ctx, 16, 16, 4, 4, 4) == binding.EWORKSPACE
    assert lib.ssnet_linear_product_prepacked(ctx, None, 16, 4, 4, 4) == binding.EINVAL
    assert lib.ssnet_conv1x1_product_prepacked(ctx, 16, 16, 1, 4, 0, 4) == binding.EINVAL
    assert lib.ssnet_conv1x1_product_prepacked(ctx, 16, 16, 1, 4, 9, 4) == binding.EWORKSPACE
    assert lib.ssnet_conv_product_planes(ctx, 16, 16, 1, 3, 8, 8, 4, 3, 3, 1, 1) == binding.EINVAL   # C % 64 != 0
    assert lib.ssnet_conv_product_planes(ctx, 16, 16, 1, 64, 8, 8, 4, 3, 3, 1, 1) == binding.EWORKSPACE
    # d_c = NULL means the pending product; there is none
    assert lib.ssnet_degree_reduce(ctx, None, 8, 0, 16) == binding.EINVAL
    assert lib.ssnet_degree_reduce_truncate(ctx, None, 8, 0, 16) == binding.EINVAL
    assert lib.ssnet_reduce_truncate_direct(ctx, None, 8, 0, 16, None, 0, None) == binding.EINVAL
    assert lib.ssnet_reduce_truncate_relu(ctx, None, 1, 64, 16, 0, 16, 16, 16, None) == binding.EINVAL
    assert lib.ssnet_reduce_truncate_relu_direct(ctx, None, 1, 64, 16, 16, 16, 16, None) == binding.EINVAL
    assert lib.ssnet_reduce_truncate_relu_direct(ctx, 16, 1, 32, 16, 16, 16, 16, 16) == binding.EINVAL    # planes need C % 64 == 0
    assert lib.ssnet_reduce_truncate_relu_direct(ctx, 16, 1, 64, 16, None, 16, 16, None) == binding.EINVAL


def test_pooling_entry_points_check_their_arguments():
    lib = binding.load_library()
    s = SSNet(5, 2, device=None)
    ctx = s._ctx
    assert lib.ssnet_pool_out_size(112, 3, 2, 1) == 56 and lib.ssnet_pool_out_size(7, 7, 7, 0) == 1
    assert lib.ssnet_pool_out_size(5, 2, 2, 0) == 2 and lib.ssnet_pool_out_size(2, 3, 1, 0) == 0
    geom = lambda H, W, kh, kw, sh, sw, ph, pw: (H, W, kh, kw, sh, sw, ph, pw)
    bad = [geom(2, 2, 3, 3, 1, 1, 0, 0),      # kernel larger than the image
           geom(8, 8, 2, 2, 2, 2, 2, 0),      # padding as large as the kernel
           geom(8, 8, 2, 2, 0, 2, 0, 0),      # zero stride
           geom(8, 8, 2, 2, 2, 2, -1, 0),
           geom(1 << 16, 8, 2, 2, 2, 2, 0, 0),
           geom(100, 100, 65, 64, 1, 1, 0, 0)]   # more than SSNET_MAX_KDIV kernel elements
    for g in bad:
        assert lib.ssnet_pool_masks(ctx, 1, *g, 0, 16, 16) == binding.EINVAL, g
        assert lib.ssnet_relu_pool(ctx, 16, 16, 16, 1, *g, 0, 16) == binding.EINVAL, g
    ok = geom(8, 8, 2, 2, 2, 2, 0, 0)
    assert lib.ssnet_pool_masks(ctx, 0, *ok, 0, 16, 16) == binding.EINVAL
    assert lib.ssnet_relu_pool(ctx, 16, 16, 16, 1, *ok, 2, 16) == binding.EINVAL         # unknown mode
    assert lib.ssnet_relu_pool(ctx, 16, 16, None, 1, *ok, 0, 16) == binding.EINVAL
    assert lib.ssnet_relu_pool(ctx, 16, 16, 16, 1, *ok, 0, 16) == binding.EINVAL        # output overlaps the input
    assert lib.ssnet_relu_pool(ctx, 16, 16, 16, 1, *ok, 0, 1 << 20) == binding.EWORKSPACE
    for kdiv in (0, -1, 4097):
        assert lib.ssnet_truncate_div(ctx, 16, 8, kdiv, 0, 16) == binding.EINVAL
        assert lib.ssnet_degree_reduce_truncate_div(ctx, 16, 8, kdiv, 0, 16) == binding.EINVAL
    assert lib.ssnet_truncate_div(ctx, 16, 8, 4, 0, 16) == binding.EWORKSPACE
    # the divisor must leave a value of e: kdiv <= 2^(32-f) (Sec. VII-B)
    keep = SSNet(3, 1, f=24, device=None)
    wide = keep._ctx
    assert lib.ssnet_truncate_div(wide, 16, 8, 257, 0, 16) == binding.EINVAL
    assert lib.ssnet_degree_reduce_truncate_div(wide, 16, 8, 257, 0, 16) == binding.EINVAL
    assert lib.ssnet_truncate_div(wide, 16, 8, 256, 0, 16) == binding.EWORKSPACE


# ----------------------------------------------------------------- the second library, over p = 2^45 - 55
P45 = (1 << 45) - 55


def test_p45_library_exports_the_same_abi_and_knows_its_prime():
    lib61, lib45 = binding.load_library(), binding.load_library(P45)
    assert lib61 is not lib45
    for name in binding.SIGNATURES:
        assert hasattr(lib45, name), name
    assert lib61.ssnet_field_prime() == P61 and lib45.ssnet_field_prime() == P45 == binding.P45
    assert SSNet(5, 2, p=P45, device=None).lib is lib45
    for lib, other in ((lib61, P45), (lib45, P61)):
        ctx = C.c_void_p()
        assert lib.ssnet_create(C.byref(ctx), 3, 1, other, 13, 0, None) == binding.EPRIME
    # six limbs per element: tiles and planes are three quarters the size
    assert lib45.ssnet_packed_weight_bytes(16, 64) == 6 * 1024 and lib61.ssnet_packed_weight_bytes(16, 64) == 8 * 1024
    assert lib45.ssnet_conv_planes_bytes(1, 64, 8, 8) == 6 * 64 * 64 + 256


@pytest.mark.parametrize("n,t", [(3, 1), (5, 2), (7, 3), (8, 2)])
def test_p45_host_tables_and_generator_match_oracle(n, t):
    import itertools
    s = SSNet(n, t, p=P45, device=None)
    assert s.host_reduction_matrix() == [[int(v) for v in r] for r in orc.red_matrix(n, t, P45)]
    for m in (t + 1, 2 * t + 1):
        for ids in list(itertools.combinations(range(1, n + 1), m))[:8]:
            assert s.host_lagrange(ids) == [int(v) for v in orc.lagrange(list(ids), P45)]
    # a field element is (draw >> 3) mod p
    key = binding.rng_key(7, 1, 2, 3, 4)
    for e in range(64):
        d = binding.rng_draw(key, e)
        assert binding.rng_field(key, e, P45) == (d >> 3) % P45 == orc.draw_field(key, e, P45)
