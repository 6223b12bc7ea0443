"""Pins for the CPU oracle: what the paper prints, closed forms, invariants and
brute force over tiny fields.  None of these re-types the oracle's formulas;
big-integer checks use Python's own arbitrary-precision `%`.
"""
import itertools
import os
import random
from fractions import Fraction
from math import comb

import numpy as np
import pytest

import oracle as orc

P61 = (1 << 61) - 1
GOLD = os.path.join(os.path.dirname(__file__), "golden")


def frac_mod(fr, p):
    fr = Fraction(fr)
    return fr.numerator * pow(fr.denominator, -1, p) % p


def read_kv(name):
    out = {}
    for line in open(os.path.join(GOLD, name)):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *vals = line.split()
        out[key] = [int(v) for v in vals]
    return out


# ----------------------------------------------------------------- field
def test_division_distortion_F11():
    # Sec. IV-A: 5 * 2^-1 = 8 in F_11
    assert orc.mul(5, orc.inv(2, 11), 11) == 8


def test_inverse_closed_forms_mersenne61():
    assert orc.inv(2, P61) == 1 << 60                 # 2 * 2^60 = 2^61 = 1 (mod p)
    assert orc.inv(3, P61) == (2 * P61 + 1) // 3      # 3 * (2p+1)/3 = 2p + 1
    assert orc.inv(P61 - 1, P61) == P61 - 1           # (-1)^-1 = -1


def test_field_ops_against_python_bigints():
    rnd = random.Random(7)
    edge = [0, 1, 2, P61 - 1, P61 - 2, (P61 - 1) // 2, (P61 + 1) // 2, 1 << 60, (1 << 60) - 1]
    vals = edge + [rnd.randrange(P61) for _ in range(200)]
    for a in vals:
        for b in vals[:24]:
            assert orc.add(a, b, P61) == (a + b) % P61
            assert orc.sub(a, b, P61) == (a - b) % P61
            assert orc.mul(a, b, P61) == (a * b) % P61
    for a in vals:
        if a:
            assert orc.mul(a, orc.inv(a, P61), P61) == 1
    for p in (11, 13, 97, 35184372088777):             # the last is the paper's 2^45 - 55
        for _ in range(50):
            a, b = rnd.randrange(p), rnd.randrange(1, p)
            assert orc.mul(a, b, p) == a * b % p
            assert orc.mul(b, orc.inv(b, p), p) == 1


def test_paper_prime_constants():
    # Sec. VII-A / App. D: p = 2^45 - 55 = 35184372088777 and 2^46 mod p = 110
    p = 35184372088777
    assert p == 2 ** 45 - 55
    assert orc.power(2, 46, p) == 110


def test_lift_and_signed_roundtrip():
    # Sec. II-B: F_11 stands for [-5, 5]
    assert list(orc.lift(np.arange(11, dtype=np.uint64), 11)) == [0, 1, 2, 3, 4, 5, -5, -4, -3, -2, -1]
    for v in (-5, -1, 0, 1, 5):
        assert orc.lift(np.array([orc.from_signed(v, 11)], np.uint64), 11)[0] == v
    half = (P61 - 1) // 2
    assert list(orc.lift(np.array([half, half + 1, P61 - 1], np.uint64), P61)) == [half, -half, -1]


def test_encode_round_half_even_and_decode():
    x = np.array([0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 0.49, -0.51, 3.0], dtype=np.float64)
    enc = orc.encode(x, 0, P61)
    assert list(orc.lift(enc, P61)) == [0, 2, 2, 0, -2, -2, 0, -1, 3]
    y = np.array([1.0, -1.0, 0.123456789, -7.75], dtype=np.float64)
    enc = orc.encode(y, 13, P61)
    assert list(orc.lift(enc, P61)) == [8192, -8192, round(0.123456789 * 8192), -63488]
    dec = orc.decode(enc, 13, P61)
    assert np.max(np.abs(dec - y)) <= 2.0 ** -14
    with pytest.raises(ValueError):
        orc.encode(np.array([2.0 ** 30]), 13, P61)


# ----------------------------------------------------------------- generator
def test_generator_core_is_splitmix64():
    want = [int(l, 16) for l in open(os.path.join(GOLD, "splitmix64.txt")) if l.startswith("0x")]
    assert [orc.draw(0, e) for e in range(3)] == want


def test_generator_second_published_stream():
    """draw(key, e) is output e of the SplitMix64 stream started at state `key`: checked on the published
    vector for state 1234567, so the counter stepping and the key entering as the state are pinned too."""
    want = [int(l) for l in open(os.path.join(GOLD, "splitmix64.txt")) if l.strip().isdigit()]
    assert len(want) == 5 and [orc.draw(1234567, e) for e in range(5)] == want


def test_key_is_a_chain_of_first_outputs_and_field_draw_is_the_top_bits():
    """The key absorbs its five words one by one, h <- first output of the stream at state (h ^ word), from
    h = 0 (draw(s, 0) is that first output, pinned above); the field element is (draw >> 3) mod p."""
    for words in [(0, 1, 0, 0, 1), (7, 2, 151, 3, 2), (2 ** 64 - 1, 10, 2 ** 40, 5, 0)]:
        h = 0
        for w in words:
            h = orc.draw(h ^ w, 0)
        assert orc.key(*words) == h
    k = orc.key(5, orc.DOM_ZERO, 9, 0, 2)
    for e in (0, 1, 2 ** 33 + 5):
        for p in (P61, P45, 11, 97):
            assert orc.draw_field(k, e, p) == (orc.draw(k, e) >> 3) % p


def test_oracle_generator_matches_the_golden_vectors():
    """tests/golden/rng_vectors.txt pins both implementations of the generator: the library's host code
    (tests/test_host_logic.py) and, here, the oracle that wrote it."""
    nkeys = ndraws = 0
    for line in open(os.path.join(GOLD, "rng_vectors.txt")):
        parts = line.split()
        if not parts or parts[0].startswith("#"):
            continue
        if parts[0] == "key":
            vals = [int(v) for v in parts[1:]]
            assert orc.key(*vals[:5]) == vals[5]
            nkeys += 1
        else:
            key, e, out, fld = (int(v) for v in parts[1:])
            assert orc.draw(key, e) == out and orc.draw_field(key, e, P61) == fld
            ndraws += 1
    assert nkeys == 8 and ndraws == 32


def test_keys_separate_streams_and_field_range():
    keys = {orc.key(s, d, sid, pty, j) for s in (0, 1) for d in range(1, 8) for sid in (0, 1, 2)
            for pty in range(0, 6) for j in range(0, 3)}
    assert len(keys) == 2 * 7 * 3 * 6 * 3
    k = orc.key(42, orc.DOM_SHARE, 0, 0, 1)
    draws = [orc.draw_field(k, e, P61) for e in range(2000)]
    assert all(0 <= d < P61 for d in draws) and len(set(draws)) == 2000
    mean = sum(draws) / len(draws) / P61
    assert 0.45 < mean < 0.55
    small = [orc.draw_field(k, e, 11) for e in range(2200)]
    counts = np.bincount(small, minlength=11)
    assert counts.min() > 140 and counts.max() < 260


# ----------------------------------------------------------------- Lagrange / REC
def test_lagrange_hand_values():
    for line in open(os.path.join(GOLD, "lagrange_multipliers.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        ids, vals = line.split("|")
        ids = [int(v) for v in ids.strip().split(",")]
        vals = [Fraction(v) for v in vals.split()]
        assert sum(vals) == 1
        for p in (11, 13, 97, P61):
            if any(v.denominator % p == 0 for v in vals):
                continue
            got = [int(v) for v in orc.lagrange(ids, p)]
            assert got == [frac_mod(v, p) for v in vals], (ids, p)


def test_lagrange_closed_form_first_m_ids():
    # for IDs 1..m: lambda_i = (-1)^(i-1) C(m, i)
    for m in range(1, 9):
        got = [int(v) for v in orc.lagrange(list(range(1, m + 1)), P61)]
        assert got == [((-1) ** (i - 1) * comb(m, i)) % P61 for i in range(1, m + 1)]


def test_lagrange_sum_is_one_any_subset():
    for m in (2, 3, 4):
        for ids in itertools.combinations(range(1, 8), m):
            assert sum(int(v) for v in orc.lagrange(list(ids), P61)) % P61 == 1


@pytest.mark.parametrize("p,t,n", [(11, 1, 3), (13, 1, 3), (11, 2, 5), (13, 2, 5)])
def test_share_reconstruct_bruteforce_all_polynomials(p, t, n):
    # every polynomial of degree <= t over F_p: any t+1 shares give the secret
    # (Sec. II-B property 1) and any t shares are consistent with every secret
    # (property 2: for each candidate secret the same number of polynomials
    # produce those t shares)
    combos = list(itertools.product(range(p), repeat=t + 1))
    secrets = np.array([c[0] for c in combos], np.uint64)
    coef = np.array([[c[j] for c in combos] for j in range(1, t + 1)], np.uint64)
    sh = orc.share_explicit(secrets, coef, n, t, p)
    # against direct evaluation with Python ints
    for idx in range(0, len(combos), 7):
        for i in range(1, n + 1):
            assert int(sh[i - 1, idx]) == sum(c * i ** j for j, c in enumerate(combos[idx])) % p
    for ids in itertools.combinations(range(1, n + 1), t + 1):
        assert np.array_equal(orc.reconstruct(sh, list(ids), p), secrets)
    for ids in itertools.combinations(range(1, n + 1), t):
        seen = {}
        for idx, c in enumerate(combos):
            view = tuple(int(sh[i - 1, idx]) for i in ids)
            seen.setdefault(view, []).append(c[0])
        for view, secs in seen.items():
            assert sorted(secs) == list(range(p)), "t shares must not narrow down the secret"


def test_appendix_B_truncation_case():
    g = read_kv("appB_truncation.txt")
    p = g["p"][0]
    sh = np.array(g["shares"], np.uint64).reshape(3, 1)
    assert int(orc.reconstruct(sh, [1, 2], p)[0]) == g["rec_first_two"][0] == 5
    halved = np.array(g["halved_shares"], np.uint64).reshape(3, 1)
    assert int(orc.reconstruct(halved, [1, 2], p)[0]) == g["rec_halved_first_two"][0] == 8


def test_sharing_is_linear():
    rng = np.random.default_rng(3)
    a = rng.integers(0, P61, 64, dtype=np.uint64)
    b = rng.integers(0, P61, 64, dtype=np.uint64)
    sa = orc.share(a, 5, 2, P61, seed=1, stream_id=0)
    sb = orc.share(b, 5, 2, P61, seed=1, stream_id=1)
    ssum = np.array([[(int(x) + int(y)) % P61 for x, y in zip(ra, rb)] for ra, rb in zip(sa, sb)], np.uint64)
    sdiff = np.array([[(int(x) - int(y)) % P61 for x, y in zip(ra, rb)] for ra, rb in zip(sa, sb)], np.uint64)
    want_sum = [(int(x) + int(y)) % P61 for x, y in zip(a, b)]
    want_diff = [(int(x) - int(y)) % P61 for x, y in zip(a, b)]
    for ids in ([1, 2, 3], [3, 4, 5], [1, 3, 5], [2, 4, 5], [1, 2, 3, 4, 5]):
        assert [int(v) for v in orc.reconstruct(ssum, ids, P61)] == want_sum
        assert [int(v) for v in orc.reconstruct(sdiff, ids, P61)] == want_diff
        assert np.array_equal(orc.reconstruct(sa, ids, P61), a)


def test_seeded_share_uses_same_coefficients_for_all_parties():
    # Eq. 1: a_1..a_t are identical in all shares -> second differences of a
    # degree-2 sharing at consecutive IDs are constant (= 2 a_2)
    a = np.arange(10, dtype=np.uint64)
    sh = orc.share(a, 5, 2, P61, seed=9, stream_id=4)
    coef = orc.draw_coeffs(9, orc.DOM_SHARE, 4, 0, 2, 10, P61)
    for e in range(10):
        s = [int(sh[i, e]) for i in range(5)]
        d2 = {(s[i + 2] - 2 * s[i + 1] + s[i]) % P61 for i in range(3)}
        assert d2 == {2 * int(coef[1, e]) % P61}
        assert (s[0] - int(a[e]) - int(coef[0, e]) - int(coef[1, e])) % P61 == 0
    # sampled element indices draw the same coefficients as the full call
    sub = orc.share(a[[2, 7]], 5, 2, P61, seed=9, stream_id=4, eidx=[2, 7])
    assert np.array_equal(sub, sh[:, [2, 7]])


# ----------------------------------------------------------------- products
def test_fig2_product_needs_all_three_shares():
    g = read_kv("fig2_example.txt")
    p = g["p"][0]
    a, b = g["a_shares"], g["b_shares"]
    assert int(orc.reconstruct(np.array(a, np.uint64).reshape(3, 1), [1, 2], p)[0]) == 2
    assert int(orc.reconstruct(np.array(b, np.uint64).reshape(3, 1), [2, 3], p)[0]) == 3
    prod = np.array([orc.mul(x, y, p) for x, y in zip(a, b)], np.uint64).reshape(3, 1)
    assert [int(v) for v in prod[:, 0]] == g["product_shares"] == [2, 6, 7]
    assert int(orc.reconstruct(prod, [1, 2, 3], p)[0]) == g["product"][0] == 6
    for ids in ([1, 2], [1, 3], [2, 3]):
        assert int(orc.reconstruct(prod, ids, p)[0]) != 6


def test_product_of_sharings_has_degree_2t():
    rng = np.random.default_rng(5)
    for n, t in ((3, 1), (5, 2)):
        a = rng.integers(0, P61, 32, dtype=np.uint64)
        b = rng.integers(0, P61, 32, dtype=np.uint64)
        sa = orc.share(a, n, t, P61, 11, 0)
        sb = orc.share(b, n, t, P61, 11, 1)
        prod = np.array([[int(x) * int(y) % P61 for x, y in zip(ra, rb)] for ra, rb in zip(sa, sb)], np.uint64)
        want = np.array([int(x) * int(y) % P61 for x, y in zip(a, b)], np.uint64)
        assert np.array_equal(orc.reconstruct(prod, list(range(1, 2 * t + 2)), P61), want)
        short = orc.reconstruct(prod, list(range(1, 2 * t + 1)), P61)
        assert not np.any(short == want)


# ----------------------------------------------------------------- R matrix
def read_rational_R():
    mats, cur = {}, None
    for line in open(os.path.join(GOLD, "reduction_matrix.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line.startswith("t="):
            cur = int(line[2:])
            mats[cur] = []
        else:
            mats[cur].append([Fraction(v) for v in line.split()])
    return mats


@pytest.mark.parametrize("p", [11, 13, 97, P61])
def test_reduction_matrix_matches_rational_form(p):
    for t, rows in read_rational_R().items():
        n = 2 * t + 1
        if any(v.denominator % p == 0 for r in rows for v in r):
            continue
        got = orc.red_matrix(n, t, p)
        want = [[frac_mod(v, p) for v in r] for r in rows]
        assert [[int(v) for v in r] for r in got] == want


def test_reduction_matrix_mod_11():
    assert orc.red_matrix(3, 1, 11).tolist() == [[6, 9, 1], [1, 5, 9], [5, 9, 2]]


@pytest.mark.parametrize("t", [1, 2, 3])
def test_reduction_matrix_invariants(t):
    p, n = P61, 2 * t + 1
    R = [[int(v) for v in r] for r in orc.red_matrix(n, t, p)]
    R2 = [[sum(R[i][l] * R[l][j] for l in range(n)) % p for j in range(n)] for i in range(n)]
    assert R2 == R                                                  # projector
    # fixes every share vector of degree <= t, drops the monomials above t
    for deg in range(0, 2 * t + 1):
        vec = [pow(i, deg, p) for i in range(1, n + 1)]
        img = [sum(vec[i] * R[i][j] for i in range(n)) % p for j in range(n)]
        assert img == (vec if deg <= t else [0] * n)


def test_reduction_matrix_with_extra_parties():
    # n > 2t+1: the first 2t+1 parties reduce, the truncated polynomial is
    # evaluated at all n IDs
    p, t, n = P61, 1, 5
    R = [[int(v) for v in r] for r in orc.red_matrix(n, t, p)]
    assert [r[:3] for r in R] == [[int(v) for v in r] for r in orc.red_matrix(3, t, p)]
    coeffs = [123456789, 987654321, 555]                             # degree 2t polynomial
    c = [sum(a * i ** j for j, a in enumerate(coeffs)) % p for i in range(1, 4)]
    img = [sum(c[i] * R[i][j] for i in range(3)) % p for j in range(n)]
    assert img == [(coeffs[0] + coeffs[1] * i) % p for i in range(1, n + 1)]


# ----------------------------------------------------------------- RED + RERAND
def test_fig2_degree_reduction_and_rerandomisation():
    g = read_kv("fig2_example.txt")
    p = g["p"][0]
    c = np.array(g["product_shares"], np.uint64).reshape(3, 1)
    zc = np.array(g["zero_coeff"], np.uint64).reshape(1, 1)
    for r1, r2, r3 in itertools.product(range(p), repeat=3):        # every reshare randomness
        rc = np.array([r1, r2, r3], np.uint64).reshape(3, 1, 1)
        out, msg1, msg2, red = orc.degree_reduce_explicit(c, rc, zc, 3, 1, p, full=True)
        assert [int(v) for v in red[:, 0]] == g["red_shares"] == [9, 1, 4]
        assert [int(v) for v in out[:, 0]] == g["final_shares"] == [2, 9, 5]
    assert [int(v) for v in out[:2, 0]] == [2, 9]                   # Sec. IV-C: "(i.e., 2,9)"
    for ids in ([1, 2], [1, 3], [2, 3]):
        assert int(orc.reconstruct(out, ids, p)[0]) == 6
    zsh = orc.share_explicit(np.zeros(1, np.uint64), zc, 3, 1, p)
    assert [int(v) for v in zsh[:, 0]] == g["zero_shares"]


def test_degree_reduce_messages_are_sharings_of_the_inputs():
    # step 1 messages of party i reconstruct (from parties 1..k) to c_i;
    # step 2 messages towards party m reconstruct to the reduced share of m
    rng = np.random.default_rng(8)
    n, t, count = 5, 2, 16
    c = rng.integers(0, P61, (n, count), dtype=np.uint64)
    out, msg1, msg2, red = orc.degree_reduce(c, n, t, P61, seed=5, stream_id=2, full=True)
    ids = list(range(1, t + 2))
    for i in range(2 * t + 1):
        assert np.array_equal(orc.reconstruct(msg1[i], ids, P61), c[i])
    for m in range(n):
        assert np.array_equal(orc.reconstruct(np.ascontiguousarray(msg2[:, m, :]), ids, P61), red[m])


@pytest.mark.parametrize("n,t", [(3, 1), (5, 2), (7, 3), (5, 1), (7, 2)])
def test_degree_reduce_equals_truncated_product_polynomial(n, t):
    # multiply two degree-t polynomials coefficient-wise with Python ints,
    # cut above degree t, evaluate at 1..n: RED must give exactly that,
    # whatever the reshare randomness; RERAND adds a degree-t sharing of 0
    rnd = random.Random(n * 10 + t)
    p, count = P61, 6
    A = [[rnd.randrange(p) for _ in range(t + 1)] for _ in range(count)]
    Bc = [[rnd.randrange(p) for _ in range(t + 1)] for _ in range(count)]
    prodc = []
    for a, b in zip(A, Bc):
        pc = [0] * (2 * t + 1)
        for i, x in enumerate(a):
            for j, y in enumerate(b):
                pc[i + j] = (pc[i + j] + x * y) % p
        prodc.append(pc)
    c = np.array([[sum(co * i ** j for j, co in enumerate(pc)) % p for pc in prodc]
                  for i in range(1, n + 1)], np.uint64)
    want_red = [[sum(co * i ** j for j, co in enumerate(pc[:t + 1])) % p for pc in prodc]
                for i in range(1, n + 1)]
    outs = []
    for seed in (1, 2):
        out, msg1, msg2, red = orc.degree_reduce(c, n, t, p, seed=seed, stream_id=0, full=True)
        assert [[int(v) for v in r] for r in red] == want_red
        zc = orc.draw_coeffs(seed, orc.DOM_ZERO, 0, 0, t, count, p)
        want_out = [[(want_red[i - 1][e] + sum(int(zc[j - 1, e]) * i ** j for j in range(1, t + 1))) % p
                     for e in range(count)] for i in range(1, n + 1)]
        assert [[int(v) for v in r] for r in out] == want_out
        outs.append(out)
        for ids in itertools.combinations(range(1, n + 1), t + 1):
            got = orc.reconstruct(out, list(ids), p)
            assert [int(v) for v in got] == [pc[0] for pc in prodc]
    assert not np.array_equal(outs[0], outs[1])                      # re-randomised
    assert not np.array_equal(outs[0], np.array(want_red, np.uint64))


# ----------------------------------------------------------------- truncation
@pytest.mark.parametrize("p,f,n,t", [(97, 1, 3, 1), (97, 2, 3, 1), (251, 2, 5, 2)])
def test_truncation_bruteforce_small_field(p, f, n, t):
    # every secret whose masked value stays inside the signed range, every
    # admissible mask e: the output shares are a degree-t sharing of
    # floor(x / 2^f) (Sec. VI-B), independent of e
    r = 1 << f
    half = (p - 1) // 2
    rnd = random.Random(p * 10 + f)
    for e_val in (1, 2, 3):
        xs = [x for x in range(-half, half + 1) if -half <= x + e_val * r <= half]
        count = len(xs)
        secret = np.array([x % p for x in xs], np.uint64)
        mk = lambda: np.array([[rnd.randrange(p) for _ in range(count)] for _ in range(t)], np.uint64)
        xsh = orc.share_explicit(secret, mk(), n, t, p)
        ev = np.full(count, e_val, np.uint64)
        out, u, wsh = orc.truncate_explicit(xsh, ev, mk(), mk(), mk(), n, t, f, p, full=True)
        want = [(x // r) % p for x in xs]                           # Python // floors toward -inf
        for ids in itertools.combinations(range(1, n + 1), t + 1):
            assert [int(v) for v in orc.reconstruct(out, list(ids), p)] == want
        # what the elite party sees is x + alpha, and what it re-shares is y + e
        seen = orc.reconstruct(np.vstack([u, np.zeros((n - t - 1, count), np.uint64)]), list(range(1, t + 2)), p)
        assert [int(v) for v in seen] == [(x + e_val * r) % p for x in xs]
        assert [int(v) for v in orc.reconstruct(wsh, list(range(1, t + 2)), p)] == [(x // r + e_val) % p for x in xs]


def test_truncation_seeded_mersenne61():
    rng = np.random.default_rng(12)
    n, t, f = 5, 2, 13
    xs = rng.integers(-(1 << 45), 1 << 45, 200, dtype=np.int64)
    xs[:4] = [0, -1, 8191, -8193]
    secret = np.array([int(x) % P61 for x in xs], np.uint64)
    xsh = orc.share(secret, n, t, P61, seed=3, stream_id=0)
    out, u, wsh = orc.truncate(xsh, n, t, f, P61, seed=3, stream_id=77, full=True)
    want = [(int(x) >> f) % P61 for x in xs]
    for ids in ([1, 2, 3], [3, 4, 5], [1, 3, 5]):
        assert [int(v) for v in orc.reconstruct(out, ids, P61)] == want
    # masks: alpha in (0, 2^32], a multiple of 2^f
    masked = orc.reconstruct(np.vstack([u, np.zeros((2, 200), np.uint64)]), [1, 2, 3], P61)
    alpha = [(int(m) - int(s)) % P61 for m, s in zip(masked, secret)]
    assert all(0 < a <= 1 << 32 and a % (1 << f) == 0 for a in alpha)
    assert len(set(alpha)) > 150


# ----------------------------------------------------------------- linear / conv
def test_linear_lazy_equals_strict_and_bigints():
    rng = np.random.default_rng(21)
    n, M, K, N = 2, 3, 70, 4
    x = rng.integers(0, P61, (n, M, K), dtype=np.uint64)
    w = rng.integers(0, P61, (n, K, N), dtype=np.uint64)
    x[0, 0, :] = P61 - 1
    w[0, :, 0] = P61 - 1
    y = orc.linear(x, w, P61)
    assert np.array_equal(y, orc.linear(x, w, P61, strict=True))
    for i in range(n):
        for m in range(M):
            for c in range(N):
                assert int(y[i, m, c]) == sum(int(x[i, m, k]) * int(w[i, k, c]) for k in range(K)) % P61


def test_linear_small_prime_against_numpy_matmul():
    rng = np.random.default_rng(22)
    for p in (97, 65521):
        x = rng.integers(0, p, (3, 9, 33), dtype=np.uint64)
        w = rng.integers(0, p, (3, 33, 7), dtype=np.uint64)
        want = np.stack([(x[i].astype(np.int64) @ w[i].astype(np.int64)) % p for i in range(3)])
        assert np.array_equal(orc.linear(x, w, p).astype(np.int64), want)
    # a transposed operand must fail: non-square, non-symmetric data
    assert not np.array_equal(orc.linear(x, w, p)[0].astype(np.int64),
                              (w[0].astype(np.int64).T[:, :9] @ x[0].astype(np.int64).T[:9, :7]) % p)


def test_linear_signed_small_values_match_integer_gemm():
    rng = np.random.default_rng(23)
    xs = rng.integers(-2 ** 15, 2 ** 15, (1, 8, 64), dtype=np.int64)
    ws = rng.integers(-2 ** 15, 2 ** 15, (1, 64, 5), dtype=np.int64)
    x = np.where(xs < 0, xs + P61, xs).astype(np.uint64)
    w = np.where(ws < 0, ws + P61, ws).astype(np.uint64)
    assert np.array_equal(orc.lift(orc.linear(x, w, P61), P61), xs @ ws)


@pytest.mark.parametrize("stride,pad,k", [(1, 1, 3), (2, 1, 3), (1, 0, 1), (2, 3, 7), (2, 0, 1)])
def test_conv_matches_torch_int64(stride, pad, k):
    import torch
    rng = np.random.default_rng(31 + k + stride)
    B, Ci, H, W, Co = 2, 3, 9, 8, 4
    xs = rng.integers(-2 ** 12, 2 ** 12, (B, Ci, H, W), dtype=np.int64)
    ws = rng.integers(-2 ** 12, 2 ** 12, (Co, Ci, k, k), dtype=np.int64)
    want = torch.nn.functional.conv2d(torch.from_numpy(xs), torch.from_numpy(ws), stride=stride, padding=pad).numpy()
    x = np.where(xs < 0, xs + P61, xs).astype(np.uint64)[None]
    w = np.where(ws < 0, ws + P61, ws).astype(np.uint64)[None]
    got = orc.conv(x, w, stride, pad, P61)
    assert got.shape[1:] == want.shape
    assert np.array_equal(orc.lift(got, P61)[0], want)
    flat = np.array([0, 5, got.size - 1, got.size // 2], np.uint64)
    assert np.array_equal(orc.conv_points(x, w, stride, pad, P61, flat), got.reshape(-1)[flat.astype(np.int64)])


def test_conv_full_range_against_bigints_and_per_party_independence():
    rng = np.random.default_rng(33)
    n, B, Ci, H, W, Co, k = 2, 1, 2, 4, 5, 2, 3
    x = rng.integers(0, P61, (n, B, Ci, H, W), dtype=np.uint64)
    w = rng.integers(0, P61, (n, Co, Ci, k, k), dtype=np.uint64)
    y = orc.conv(x, w, 1, 1, P61)
    for i in range(n):
        for co in range(Co):
            for ho in range(H):
                for wo in range(W):
                    acc = 0
                    for c in range(Ci):
                        for r in range(k):
                            for s in range(k):
                                hi, wi = ho - 1 + r, wo - 1 + s
                                if 0 <= hi < H and 0 <= wi < W:
                                    acc += int(x[i, 0, c, hi, wi]) * int(w[i, co, c, r, s])
                    assert int(y[i, 0, co, ho, wo]) == acc % P61
    # party 1's output only depends on party 1's operands
    x2, w2 = x.copy(), w.copy()
    x2[0] = 1
    w2[0] = 2
    assert np.array_equal(orc.conv(x2, w2, 1, 1, P61)[1], y[1])


# ----------------------------------------------------------------- end to end
def test_tiny_secure_gemm_matches_float64_on_dequantised_operands():
    # share X and W, local product, degree reduction, truncation, reconstruct:
    # the decoded result is floor-truncated, so it lies in (exact - 2^-f, exact]
    from ssnet_inputs import gaussian
    n, t, f, p = 3, 1, 13, P61
    M, K, N = 8, 32, 6
    X, Wt = gaussian((M, K), 1), gaussian((K, N), 2)
    xe, we = orc.encode(X, f, p), orc.encode(Wt, f, p)
    xs = orc.share(xe, n, t, p, seed=7, stream_id=1)
    ws = orc.share(we, n, t, p, seed=7, stream_id=2)
    y2 = orc.linear(xs, ws, p)                                       # degree 2t
    # the untruncated product reconstructs exactly from all 2t+1 parties
    exact = orc.decode(xe, f, p) @ orc.decode(we, f, p)
    assert np.array_equal(orc.decode(orc.reconstruct(y2, [1, 2, 3], p), 2 * f, p), exact)
    yr = orc.degree_reduce(y2.reshape(n, -1), n, t, p, seed=7, stream_id=3)
    yt = orc.truncate(yr, n, t, f, p, seed=7, stream_id=4)
    for ids in ([1, 2], [2, 3], [1, 3]):
        got = orc.decode(orc.reconstruct(yt, ids, p), f, p).reshape(M, N)
        err = exact - got
        assert err.min() >= 0 and err.max() < 2.0 ** -f
    assert np.max(np.abs(got - X @ Wt)) < 2.0 ** -8


# ----------------------------------------------------------------- SSS-NonLinear (ReLU), Sec. VI-C
def _poly_shares(a0, coefs, n, p):
    """shares of the polynomial a0 + c1 x + ... at IDs 1..n, with Python integers"""
    return [(a0 + sum(c * pow(i, j + 1, p) for j, c in enumerate(coefs))) % p for i in range(1, n + 1)]


@pytest.mark.parametrize("n,t", [(3, 1), (5, 2)])
def test_relu_bruteforce_small_field(n, t):
    """Every x in [-15, 15] and every mask beta in [1, 8] over F_251 (|x| beta < p/2): the output
    shares open to max(x, 0) from every k-subset, the messages are the products of the shares,
    and the elite party sees exactly x * beta."""
    p, k, nr = 251, t + 1, 2 * t + 1
    rng = random.Random(7)
    xs = [x for x in range(-15, 16) for _ in range(8)]
    betas = [b for _ in range(-15, 16) for b in range(1, 9)]
    count = len(xs)
    cx = [[rng.randrange(p) for _ in range(count)] for _ in range(t)]
    cb = [[rng.randrange(p) for _ in range(count)] for _ in range(t)]
    cbi = [[rng.randrange(p) for _ in range(count)] for _ in range(t)]
    x_sh = np.array([_poly_shares(x % p, [c[e] for c in cx], n, p) for e, x in enumerate(xs)], np.uint64).T.copy()
    sb, sbi = orc.nonlinear_masks_explicit(np.array(betas, np.uint64), np.array(cb, np.uint64),
                                           np.array(cbi, np.uint64), n, t, p)
    # the dealer's masks: degree-t sharings of beta and of its inverse
    for e in range(count):
        assert [int(v) for v in sb[:, e]] == _poly_shares(betas[e], [c[e] for c in cb], n, p)
        assert [int(v) for v in sbi[:, e]] == _poly_shares(pow(betas[e], -1, p), [c[e] for c in cbi], n, p)
    out, msg, y = orc.relu(x_sh, sb, sbi, n, t, p, full=True)
    for e in range(count):
        for i in range(nr):
            assert int(msg[i, e]) == int(x_sh[i, e]) * int(sb[i, e]) % p
        assert int(y[e]) == max(xs[e] * betas[e], 0)
    for ids in itertools.combinations(range(1, n + 1), k):
        rec = orc.reconstruct(out, list(ids), p)
        assert [int(v) for v in rec] == [max(x, 0) for x in xs], ids
    # the product sharing has degree 2t: 2t+1 points open it, 2t points in general do not
    full = orc.reconstruct(np.vstack([msg, np.zeros((n - nr, count), np.uint64)]), list(range(1, nr + 1)), p)
    assert [int(v) for v in full] == [x * b % p for x, b in zip(xs, betas)]
    short = orc.reconstruct(np.vstack([msg, np.zeros((n - nr, count), np.uint64)]), list(range(1, nr)), p)
    assert sum(int(a) != int(b) for a, b in zip(short, full)) > count // 2


def test_relu_seeded_masks_mersenne61():
    """p = 2^61 - 1, beta in [1, 2^28] as in Sec. VII-B: mask invariants and the opened result for
    16-bit-scale and extreme inputs."""
    n, t, count, seed = 5, 2, 4096, 11
    sb, sbi = orc.nonlinear_masks(count, n, t, 28, P61, seed, 3)
    for ids in ([1, 2, 3], [2, 4, 5], [3, 4, 5]):
        beta = orc.reconstruct(sb, ids, P61)
        binv = orc.reconstruct(sbi, ids, P61)
        assert int(beta.min()) >= 1 and int(beta.max()) <= 1 << 28
        assert all(int(b) * int(bi) % P61 == 1 for b, bi in zip(beta, binv))
    assert len(set(int(b) for b in orc.reconstruct(sb, [1, 2, 3], P61))) > count - 8     # not a constant
    # sampled element indices draw the same masks as the full run
    idx = np.array([0, 5, 77, 4095], np.uint64)
    sb2, sbi2 = orc.nonlinear_masks(4, n, t, 28, P61, seed, 3, eidx=idx)
    assert np.array_equal(sb2, sb[:, idx.astype(np.int64)]) and np.array_equal(sbi2, sbi[:, idx.astype(np.int64)])
    rng = np.random.default_rng(5)
    xs = rng.integers(-(1 << 31), 1 << 31, count, dtype=np.int64)
    xs[:6] = [0, 1, -1, (1 << 32) - 1, -((1 << 32) - 1), 12345]
    x_sh = orc.share(np.where(xs < 0, xs + P61, xs).astype(np.uint64), n, t, P61, seed, 9)
    out = orc.relu(x_sh, sb, sbi, n, t, P61)
    for ids in ([1, 2, 3], [1, 3, 5]):
        assert np.array_equal(orc.reconstruct(out, ids, P61).astype(np.int64), np.maximum(xs, 0))
    # degree of the result stays t: k = 3 shares determine the other two
    assert np.array_equal(orc.reconstruct(out, [1, 2, 3], P61), orc.reconstruct(out, [3, 4, 5], P61))


# ----------------------------------------------------------------- truncation with rounding division (Sec. VI-C, App. C)
def _round_half_up(a, b):
    """nearest integer to a/b for b > 0, halves going up, with Python's exact rationals"""
    fr = Fraction(a, b)
    lo = fr.numerator // fr.denominator
    return lo + 1 if fr - lo >= Fraction(1, 2) else lo


@pytest.mark.parametrize("n,t", [(3, 1), (5, 2)])
def test_truncate_div_is_rounding_division_whatever_the_mask(n, t):
    """y = [floor(x / 2^f) / kdiv] for every x of a signed range, every kdiv of the usual pooling
    kernels and several e: the opened result never depends on e, and kdiv = 1 is the plain truncation."""
    p, f = P61, 3
    rng = random.Random(3)
    xs = list(range(-700, 701))
    count = len(xs)
    x_sh = orc.share(np.array([x % p for x in xs], np.uint64), n, t, p, 5, 1)
    coefs = [np.array([[rng.randrange(p) for _ in range(count)] for _ in range(t)], np.uint64) for _ in range(3)]
    for kdiv in (1, 4, 9, 49):
        want = [_round_half_up(x >> f, kdiv) for x in xs]
        for evals in ([1] * count, [rng.randrange(1, 1 << 19) for _ in range(count)]):
            out, u, wsh = orc.truncate_div_explicit(x_sh, np.array(evals, np.uint64), *coefs, n, t, f, kdiv, p, full=True)
            for ids in ([1, 2, 3][:t + 1], list(range(n - t, n + 1))):
                got = orc.lift(orc.reconstruct(out, ids, p), p)
                assert [int(v) for v in got] == want, (kdiv, ids)
            # what the elite party opens is x + e * 2^f * kdiv, what it re-shares is the result + e
            opened = orc.reconstruct(np.vstack([u, np.zeros((n - t - 1, count), np.uint64)]), list(range(1, t + 2)), p)
            assert [int(v) for v in opened] == [(x + e * (1 << f) * kdiv) % p for x, e in zip(xs, evals)]
            shared = orc.reconstruct(wsh, list(range(1, t + 2)), p)
            assert [int(v) for v in shared] == [(w + e) % p for w, e in zip(want, evals)]
        if kdiv == 1:
            assert np.array_equal(out, orc.truncate_explicit(x_sh, np.array(evals, np.uint64), *coefs, n, t, f, p))
    # seeded form: kdiv = 1 draws the same masks as the plain truncation
    assert np.array_equal(orc.truncate_div(x_sh, n, t, f, 1, p, 5, 2), orc.truncate(x_sh, n, t, f, p, 5, 2))
    got = orc.lift(orc.reconstruct(orc.truncate_div(x_sh, n, t, f, 4, p, 5, 2), [1, 2, 3][:t + 1], p), p)
    assert [int(v) for v in got] == [_round_half_up(x >> f, 4) for x in xs]


def test_truncation_mask_range_with_pooling_divisor_sec_vii_b():
    """Sec. VII-B: before a pooling kernel of kh*kw elements the mask is a multiple of 2^f * kh*kw and still lies in
    (0, 2^32], i.e. e comes from [1, floor(2^32 / 2^f / (kh*kw))].  The mask is read off what the elite party opens
    (x + alpha with x = 0); without a divisor the range is that of the plain truncation."""
    for p, n, t, f in ((P61, 5, 2, 13), (P45, 3, 1, 12), (P61, 3, 1, 24)):
        count = 4096
        zeros = orc.share(np.zeros(count, np.uint64), n, t, p, 3, 1)
        for kdiv in (1, 4, 9, 49, 255, 4096):
            if kdiv > (1 << (32 - f)):
                continue
            _, u, _ = orc.truncate_div(zeros, n, t, f, kdiv, p, 77, kdiv, full=True)
            alpha = orc.reconstruct(u[:t + 1], list(range(1, t + 2)), p)
            step = kdiv << f
            e = alpha // np.uint64(step)
            assert np.all(alpha % np.uint64(step) == 0) and int(alpha.min()) > 0 and int(alpha.max()) <= 1 << 32, (p, kdiv)
            assert int(e.max()) <= (1 << (32 - f)) // kdiv
            if (1 << (32 - f)) // kdiv >= 64:   # the whole range is used, not a corner of it
                assert int(e.max()) > 0.9 * ((1 << (32 - f)) // kdiv) and int(e.min()) < 0.1 * ((1 << (32 - f)) // kdiv) + 2


def test_avgpool_fold_worst_case_and_bound_appendix_c():
    """App. C: with every element of a 2x2 kernel equal to g*4 + 2 the folded form gives (g+1)*4
    against the true 4g + 2: off by exactly 2; and over every 2x2 kernel of a small range the
    sum of rounded quarters is never further than 2 from the rounded mean.  Run through the
    oracle: truncation with kdiv = 4 (f = 0 keeps the values), then ReLU + sum pooling."""
    n, t, p = 3, 1, P61
    vals = list(range(-3, 10))
    kernels = list(itertools.product(vals, repeat=4))
    kernels += [(g * 4 + 2,) * 4 for g in range(0, 50)]            # the printed worst case
    planes = len(kernels)
    x = np.array([[v % p for v in ker] for ker in kernels], np.uint64)          # [planes, 2*2]
    x_sh = orc.share(x.reshape(-1), n, t, p, 9, 1)
    q_sh = orc.truncate_div(x_sh, n, t, 0, 4, p, 9, 2)
    sb, sbi = orc.pool_masks(planes, 2, 2, 2, 2, 2, 2, 0, 0, n, t, 28, p, 9, 3)
    out = orc.relu_pool(q_sh, sb, sbi, planes, 2, 2, 2, 2, 2, 2, 0, 0, orc.POOL_SUM, n, t, p)
    folded = [int(v) for v in orc.lift(orc.reconstruct(out, [2, 3], p), p)]
    worst = 0
    for ker, got in zip(kernels, folded):
        true = _round_half_up(sum(max(v, 0) for v in ker), 4)
        assert got == sum(max(_round_half_up(v, 4), 0) for v in ker)
        worst = max(worst, abs(got - true))
        if len(set(ker)) == 1 and ker[0] % 4 == 2 and ker[0] > 0:
            assert got - ker[0] == 2 and true == ker[0]
    assert worst == 2


# ----------------------------------------------------------------- SSS-NonLinear with pooling (Sec. VI-C)
@pytest.mark.parametrize("geom", [
    (6, 6, 2, 2, 2, 2, 0, 0),      # 2x2 / 2: kernels tile the image
    (7, 5, 2, 2, 2, 2, 0, 0),      # ragged right and bottom edges
    (9, 9, 3, 3, 2, 2, 1, 1),      # 3x3 / 2, padding 1: overlapping kernels (the ResNet stem)
    (7, 7, 7, 7, 7, 7, 0, 0),      # global pooling
    (8, 6, 3, 2, 1, 2, 0, 1),      # unequal kernel, stride and padding per axis
])
@pytest.mark.parametrize("n,t", [(3, 1), (5, 2)])
def test_relu_pool_against_torch_and_mask_constancy(geom, n, t):
    import torch
    H, W, kh, kw, sh, sw, ph, pw = geom
    p, planes, seed = P61, 5, 21
    Ho, Wo = (H + 2 * ph - kh) // sh + 1, (W + 2 * pw - kw) // sw + 1
    assert (orc.pool_out_size(H, kh, sh, ph), orc.pool_out_size(W, kw, sw, pw)) == (Ho, Wo)
    rng = np.random.default_rng(4)
    xs = rng.integers(-(1 << 20), 1 << 20, (planes, H, W), dtype=np.int64)
    xs[0, 0, :3] = [0, -1, 1]
    x_sh = orc.share(np.where(xs < 0, xs + p, xs).astype(np.uint64).reshape(-1), n, t, p, seed, 1)
    sb, sbi = orc.pool_masks(planes, H, W, kh, kw, sh, sw, ph, pw, n, t, 28, p, seed, 2)
    # the masks: beta in [1, 2^28], equal inside every pooling kernel, and the pooled element's
    # beta^-1 inverts the beta of its kernel
    beta = np.array([int(v) for v in orc.reconstruct(sb, list(range(1, t + 2)), p)], object).reshape(planes, H, W)
    binv = np.array([int(v) for v in orc.reconstruct(sbi, list(range(n - t, n + 1)), p)], object).reshape(planes, Ho, Wo)
    assert beta.min() >= 1 and beta.max() <= 1 << 28
    for pl in range(planes):
        for oh in range(Ho):
            for ow in range(Wo):
                win = [beta[pl, h, w] for h in range(oh * sh - ph, oh * sh - ph + kh)
                       for w in range(ow * sw - pw, ow * sw - pw + kw) if 0 <= h < H and 0 <= w < W]
                assert len(set(win)) == 1 and win[0] * binv[pl, oh, ow] % p == 1
    tiled = (sh, sw, ph, pw) == (kh, kw, 0, 0)
    distinct = len(set(beta.reshape(-1)))
    assert distinct == (planes * Ho * Wo if tiled else planes)          # no coarser than needed
    # the share polynomials differ from element to element even where beta is equal
    assert len(set(int(v) for v in sb[0])) == planes * H * W
    xt = torch.from_numpy(xs).clamp(min=0).to(torch.float64)[None]
    want_max = torch.nn.functional.max_pool2d(xt, (kh, kw), (sh, sw), (ph, pw))[0].to(torch.int64).numpy()
    want_sum = (torch.nn.functional.avg_pool2d(xt, (kh, kw), (sh, sw), (ph, pw), count_include_pad=True)[0]
                * (kh * kw)).round().to(torch.int64).numpy()
    for mode, want in ((orc.POOL_MAX, want_max), (orc.POOL_SUM, want_sum)):
        out, msg, y = orc.relu_pool(x_sh, sb, sbi, planes, H, W, kh, kw, sh, sw, ph, pw, mode, n, t, p, full=True)
        for ids in (list(range(1, t + 2)), list(range(n - t, n + 1))):
            got = orc.lift(orc.reconstruct(out, ids, p), p).reshape(planes, Ho, Wo)
            assert np.array_equal(got, want), (mode, ids)
        # messages: products of the shares; the plain result is the pooled value times its kernel's beta
        assert all(int(msg[i, e]) == int(x_sh[i, e]) * int(sb[i, e]) % p
                   for i in range(2 * t + 1) for e in range(0, planes * H * W, 7))
        b_out = np.array([pow(int(v), -1, p) for v in binv.reshape(-1)], object)
        assert [int(v) for v in y] == [int(w) * int(b) for w, b in zip(want.reshape(-1), b_out)]


# ----------------------------------------------------------------- the paper's own prime, p = 2^45 - 55 (Sec. VII-A, App. D)
P45 = (1 << 45) - 55


def test_p45_split_product_of_appendix_d():
    """App. D multiplies two 46-bit operands through 23-bit halves: C = (C_HH + hi(C_HL) + hi(C_LH)) 2^46 +
    (lo(C_HL) + lo(C_LH)) 2^23 + C_LL with 2^46 = 110 (mod p).  (As printed the middle term has lost its
    weight 2^23.)  Restated with Python integers, it agrees with the oracle's product."""
    rng = random.Random(45)
    ops = [(rng.randrange(P45), rng.randrange(P45)) for _ in range(2000)]
    ops += [(P45 - 1, P45 - 1), (0, 5), (1, P45 - 1), ((1 << 44), (1 << 44) + 12345)]
    for a, b in ops:
        ah, al, bh, bl = a >> 23, a & 0x7FFFFF, b >> 23, b & 0x7FFFFF
        chh, chl, clh, cll = ah * bh, ah * bl, al * bh, al * bl
        c_h = chh + (chl >> 23) + (clh >> 23)
        c_m = (chl & 0x7FFFFF) + (clh & 0x7FFFFF)
        want = ((c_h % P45) * 110 + c_m * (1 << 23) + cll) % P45
        assert orc.mul(a, b, P45) == want == a * b % P45


def test_p45_bit_budget_of_a_layer():
    """Sec. VII-A: 16-bit operands leave 13 bits for the accumulation of a dot product in a 45-bit
    signed range.  A dot product of K = 2^13 - 1 worst-case 16-bit terms on shares over p = 2^45 - 55
    reconstructs to the exact signed integer; one more doubling of K wraps."""
    n, t, p = 3, 1, P45
    for K, fits in ((1 << 13) - 1, True), (1 << 14, False):
        x = np.full((1, K), -(1 << 15), np.int64)          # the extreme of the signed 16-bit range
        w = np.full((K, 1), -(1 << 15), np.int64)
        exact = int((x.astype(object) @ w.astype(object))[0, 0])
        xs = orc.share(np.where(x < 0, x + p, x).astype(np.uint64), n, t, p, 3, 1)
        ws = orc.share(np.where(w < 0, w + p, w).astype(np.uint64), n, t, p, 3, 2)
        got = int(orc.lift(orc.reconstruct(orc.linear(xs, ws, p), [1, 2, 3], p), p)[0, 0])
        assert (got == exact) == fits
        assert (abs(exact) <= (p - 1) // 2) == fits


def test_p45_tiny_secure_layer_with_relu_matches_float64():
    """Linear - Truncation - NonLinear over the paper's prime with its mask ranges (alpha below 2^32,
    beta below 2^28, Sec. VII-B): floor-truncated product, then max(., 0)."""
    from ssnet_inputs import gaussian
    n, t, f, p = 5, 2, 13, P45
    M, K, N = 6, 48, 5
    X, Wt = gaussian((M, K), 11), gaussian((K, N), 12) / np.sqrt(K)
    xe, we = orc.encode(X, f, p), orc.encode(Wt, f, p)
    y2 = orc.linear(orc.share(xe, n, t, p, 7, 1), orc.share(we, n, t, p, 7, 2), p)
    exact = orc.decode(xe, f, p) @ orc.decode(we, f, p)
    yt = orc.truncate(orc.degree_reduce(y2.reshape(n, -1), n, t, p, 7, 3), n, t, f, p, 7, 3)
    sb, sbi = orc.nonlinear_masks(M * N, n, t, 28, p, 7, 4)
    out = orc.relu(yt, sb, sbi, n, t, p)
    for ids in ([1, 2, 3], [3, 4, 5], [1, 3, 5]):
        tr = orc.decode(orc.reconstruct(yt, ids, p), f, p).reshape(M, N)
        err = exact - tr
        assert err.min() >= 0 and err.max() < 2.0 ** -f
        got = orc.decode(orc.reconstruct(out, ids, p), f, p).reshape(M, N)
        assert np.array_equal(got, np.maximum(tr, 0))
