"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the GPU library.  Each pins a piece of the oracle to something
other than itself: exact algebra of the group 2T, a library routine (numpy / scipy), a closed
form, a brute-force evaluation written differently, or numbers the paper prints.
"""
import math
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
SEEDS = [0, 1, 7, 42, 1337]  # the seeds the paper's seed-variance study uses


# ---------------------------------------------------------------------------------------
# independent helpers (textbook constructions, not the oracle's formulas)
# ---------------------------------------------------------------------------------------

def as_complex_matrix(q):
    """Standard 2x2 complex representation of a quaternion a + bi + cj + dk."""
    a, b, c, d = q
    return np.array([[a + 1j * b, c + 1j * d], [-c + 1j * d, a - 1j * b]])


def from_complex_matrix(m):
    return np.array([m[0, 0].real, m[0, 0].imag, m[0, 1].real, m[0, 1].imag])


def matmul_product(a, b):
    return from_complex_matrix(as_complex_matrix(a) @ as_complex_matrix(b))


def f16(x):
    return np.asarray(x, np.float16).view(np.uint16)


# ---------------------------------------------------------------------------------------
# fp16 conversions against numpy's
# ---------------------------------------------------------------------------------------

def test_half_to_double_all_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.half_to_double(bits)
    want = bits.view(np.float16).astype(np.float64)
    finite = np.isfinite(want)
    assert np.array_equal(got[finite], want[finite])
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.array_equal(np.isinf(got), np.isinf(want))
    assert np.array_equal(np.signbit(got[finite]), np.signbit(want[finite]))


def test_double_to_half_matches_numpy_rne():
    rng = np.random.default_rng(3)
    v = np.concatenate([
        rng.standard_normal(4000) * np.exp(rng.uniform(-20, 11, 4000)),
        # exact ties between neighbouring halves, normal and subnormal
        (np.arange(1, 4000) + 0.5) * 2.0 ** -24,
        (2048 + np.arange(0, 2000) + 0.5) * 2.0 ** -5,
        [0.0, -0.0, 65504.0, 65519.9, 2.0 ** -25, 2.0 ** -25 * 1.0000001, 2.0 ** -24, 6.1e-5],
    ])
    v = v[np.abs(v) < 65520.0]  # numpy overflows to inf beyond; the oracle saturates
    with np.errstate(over="ignore"):
        want = v.astype(np.float16).view(np.uint16)
    got = oracle.double_to_half(v)
    assert np.array_equal(got, want)


def test_double_to_half_saturates():
    got = oracle.double_to_half(np.array([65520.0, 1e9, -1e9, np.inf, -np.inf]))
    assert list(got) == [0x7BFF, 0x7BFF, 0xFBFF, 0x7BFF, 0xFBFF]


# ---------------------------------------------------------------------------------------
# 2T and the Hamilton product
# ---------------------------------------------------------------------------------------

def test_hamilton_matches_matrix_representation():
    rng = np.random.default_rng(0)
    for _ in range(200):
        a, b = rng.standard_normal(4), rng.standard_normal(4)
        assert np.allclose(oracle.hamilton(a, b), matmul_product(a, b), rtol=0, atol=1e-14)


def test_hamilton_matches_scipy_rotation_composition():
    from scipy.spatial.transform import Rotation as R
    rng = np.random.default_rng(1)
    for _ in range(50):
        a, b = rng.standard_normal(4), rng.standard_normal(4)
        a /= np.linalg.norm(a)
        b /= np.linalg.norm(b)
        # scipy stores (x, y, z, w); composition r_a * r_b is the quaternion product a (x) b
        ra, rb = R.from_quat(np.roll(a, -1)), R.from_quat(np.roll(b, -1))
        q = np.roll((ra * rb).as_quat(), 1)
        mine = oracle.hamilton(a, b)
        assert min(np.abs(q - mine).max(), np.abs(q + mine).max()) < 1e-12


def test_sign_convention_ij_k():
    one, i, j, k = np.eye(4)
    assert np.array_equal(oracle.hamilton(i, j), k)
    assert np.array_equal(oracle.hamilton(j, i), -k)
    assert np.array_equal(oracle.hamilton(i, i), -one)
    assert np.array_equal(oracle.hamilton(j, k), i)
    assert np.array_equal(oracle.hamilton(k, i), j)



def test_primary_index_outside_the_group_names_no_element():
    """2T has exactly 24 elements (App. D "The Hurwitz primary codebook"): any other index yields NaNs,
    so a codeword index k >= 24 S can never score as a valid pick."""
    for p in (-1, 24, 25, 39, 47):
        assert np.isnan(oracle.primary(p)).all()
    sec = oracle.build_codebooks(0, 1, 1, 4)[0, 0, 0]
    x = np.array([1.0, 0.5, -0.25, 2.0], np.float16).view(np.uint16)
    assert np.isnan(oracle.score(x, sec, 24 * 4 + 1))
    assert np.isfinite(oracle.score(x, sec, 24 * 4 - 1))

def test_2T_elements_and_order():
    P = oracle.primaries()
    assert P.shape == (24, 4)
    assert np.array_equal((P * P).sum(1), np.ones(24))          # unit, exactly
    assert len({tuple(p) for p in P}) == 24                      # distinct
    # the set is {+-1, +-i, +-j, +-k, (+-1 +-i +-j +-k)/2} (Sec. 2, App. D)
    want = {tuple(s * e) for e in np.eye(4) for s in (1.0, -1.0)}
    want |= {tuple(0.5 * np.array(sg)) for sg in np.ndindex(2, 2, 2, 2) for sg in [[1 - 2 * t for t in sg]]}
    assert {tuple(p) for p in P} == want
    # the order this build fixes
    assert np.array_equal(P[0], [1, 0, 0, 0]) and np.array_equal(P[1], [-1, 0, 0, 0])
    assert np.array_equal(P[2], [0, 1, 0, 0]) and np.array_equal(P[7], [0, 0, 0, -1])
    assert np.array_equal(P[8], [0.5, 0.5, 0.5, 0.5]) and np.array_equal(P[9], [0.5, 0.5, 0.5, -0.5])
    assert np.array_equal(P[8 + 8], [-0.5, 0.5, 0.5, 0.5]) and np.array_equal(P[23], [-0.5] * 4)


def test_2T_group_axioms_and_geometry():
    P = oracle.primaries()
    elems = {tuple(p): n for n, p in enumerate(P)}
    table = np.zeros((24, 24), int)
    for a in range(24):
        for b in range(24):
            prod = oracle.hamilton(P[a], P[b])
            assert tuple(prod) in elems                          # closure (exact: multiples of 1/4 -> 1/2)
            table[a, b] = elems[tuple(prod)]
    assert all(sorted(table[a]) == list(range(24)) for a in range(24))  # Latin square
    assert np.array_equal(table[0], np.arange(24)) and np.array_equal(table[:, 0], np.arange(24))
    conj = P * np.array([1, -1, -1, -1])
    for a in range(24):
        assert table[a, elems[tuple(conj[a])]] == 0              # inverse = conjugate
    # element orders of the binary tetrahedral group: 1, 1, 6, 8, 8 elements of order 1, 2, 4, 3, 6
    orders = []
    for a in range(24):
        n, cur = 1, a
        while cur != 0:
            cur, n = table[cur, a], n + 1
        orders.append(n)
    assert sorted(orders) == sorted([1] + [2] + [4] * 6 + [3] * 8 + [6] * 8)
    # 24-cell: every vertex sees inner products {1:1, 1/2:8, 0:6, -1/2:8, -1:1}
    G = P @ P.T
    for a in range(24):
        vals, counts = np.unique(G[a], return_counts=True)
        assert dict(zip(vals, counts)) == {-1.0: 1, -0.5: 8, 0.0: 6, 0.5: 8, 1.0: 1}
    off = G[~np.eye(24, dtype=bool)]
    assert math.degrees(math.acos(off.max())) == pytest.approx(60.0, abs=1e-12)  # min angle 60 deg


# ---------------------------------------------------------------------------------------
# codebooks
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("seed", SEEDS)
def test_joint_codebook_has_24S_distinct_unit_codewords(seed):
    S = 24
    sec = oracle.build_codebooks(seed, 2, 2, S)
    for l in range(2):
        for m in range(2):
            for h in range(2):
                Cb = oracle.joint_codebook(sec[l, m, h])
                assert Cb.shape == (24 * S, 4)
                assert np.abs(np.linalg.norm(Cb, axis=1) - 1).max() < 1e-6
                G = Cb @ Cb.T
                np.fill_diagonal(G, -1)
                assert G.max() < 1 - 1e-9                        # pairwise distinct: |C| = 24 S
                # codeword k = p*S + s is P[p] (x) sec[s], primary on the left (Eq. 1)
                P = oracle.primaries()
                k = 5 * S + 7
                assert np.allclose(Cb[k], matmul_product(P[5], sec[l, m, h, 7].astype(np.float64)), atol=1e-15)


def test_codebook_generator_properties():
    a = oracle.build_codebooks(0, 3, 4, 64)
    assert a.shape == (3, 2, 4, 64, 4) and a.dtype == np.float32
    assert np.array_equal(a, oracle.build_codebooks(0, 3, 4, 64))            # deterministic
    assert not np.array_equal(a, oracle.build_codebooks(1, 3, 4, 64))        # seed matters
    n = np.linalg.norm(a.astype(np.float64), axis=-1)
    assert np.abs(n - 1).max() < 1e-7                                        # unit after fp32 rounding
    flat = oracle.build_codebooks(0, 8, 8, 256).reshape(-1, 4).astype(np.float64)   # 32768 draws
    # Haar on S^3: zero mean, E[q_i^2] = 1/4, uncorrelated components, distinct per (layer, role, head)
    assert np.abs(flat.mean(0)).max() < 0.012
    assert np.abs((flat ** 2).mean(0) - 0.25).max() < 0.005
    cov = np.cov(flat.T)
    assert np.abs(cov - np.diag(np.diag(cov))).max() < 0.006
    assert len({tuple(r) for r in flat.round(6)}) == flat.shape[0]
    # a single coordinate of a Haar point on S^3 has density (2/pi) sqrt(1 - t^2): P(|t| < 1/2)
    want = (2 / math.pi) * (math.asin(0.5) + 0.5 * math.sqrt(0.75))
    assert abs((np.abs(flat[:, 0]) < 0.5).mean() - want) < 0.01


def test_isometry_of_left_and_right_multiplication():
    rng = np.random.default_rng(5)
    for _ in range(100):
        q, a, b = (rng.standard_normal(4) for _ in range(3))
        q /= np.linalg.norm(q)
        assert abs(oracle.hamilton(q, a) @ oracle.hamilton(q, b) - a @ b) < 1e-13
        assert abs(oracle.hamilton(a, q) @ oracle.hamilton(b, q) - a @ b) < 1e-13


def test_score_rewrites_agree_for_all_24S_pairs():
    """<u, P q_s> = <conj(P) u, q_s> = <u conj(q_s), P> (isometry, Sec. 3)."""
    rng = np.random.default_rng(6)
    S = 16
    sec = oracle.build_codebooks(7, 1, 1, S)[0, 0, 0]
    P = oracle.primaries()
    cj = np.array([1, -1, -1, -1.0])
    x = f16(rng.standard_normal(4))
    xf = x.view(np.float16).astype(np.float64)
    u = xf / np.linalg.norm(xf)
    for p in range(24):
        for s in range(S):
            q = sec[s].astype(np.float64)
            sc = oracle.score(x, sec, p * S + s)
            assert abs(sc - oracle.hamilton(P[p] * cj, u) @ q) < 1e-14
            assert abs(sc - oracle.hamilton(u, q * cj) @ P[p]) < 1e-14


# ---------------------------------------------------------------------------------------
# search
# ---------------------------------------------------------------------------------------

def numpy_bruteforce(xf, sec_head):
    """Second, differently-written search: codewords by complex 2x2 matmul, scores by one
    matrix product, np.argmax (first maximum = lowest index)."""
    P = oracle.primaries()
    S = sec_head.shape[0]
    Cb = np.array([matmul_product(P[p], sec_head[s].astype(np.float64)) for p in range(24) for s in range(S)])
    u = xf / np.linalg.norm(xf, axis=-1, keepdims=True)
    sc = u @ Cb.T
    return sc.argmax(-1), sc


@pytest.mark.parametrize("S", [1, 5, 16, 24])
def test_search_matches_numpy_bruteforce(S):
    rng = np.random.default_rng(S)
    sec = oracle.build_codebooks(42, 1, 1, S)[0, 0, 0]
    x = f16(rng.standard_normal((300, 4)) * np.exp(rng.normal(0, 1, (300, 1))))
    xf = x.view(np.float16).astype(np.float64)
    kk, sc = numpy_bruteforce(xf, sec)
    for n in range(x.shape[0]):
        k, best, second = oracle.search_chunk(x[n], sec)
        srt = np.sort(sc[n])
        if srt[-1] - srt[-2] > 1e-12:
            assert k == kk[n]
        assert best == pytest.approx(srt[-1], abs=1e-14)
        assert second == pytest.approx(srt[-2], abs=1e-14)
        assert best - second >= 0


def test_search_plant_returns_planted_pair():
    rng = np.random.default_rng(11)
    S = 16
    sec = oracle.build_codebooks(1, 1, 1, S)[0, 0, 0]
    P = oracle.primaries()
    for _ in range(100):
        p, s = rng.integers(24), rng.integers(S)
        c = matmul_product(P[p], sec[s].astype(np.float64))
        x = f16(3.0 * c)                    # fp16 rounding moves the direction by < 1e-3
        k, best, _ = oracle.search_chunk(x, sec)
        assert k == p * S + s and best > 1 - 1e-6


def test_search_S1_identity_is_nearest_24cell_vertex_closed_form():
    """With one secondary equal to 1 the codebook is 2T itself and the best score is
    max(max|u_i|, (|u_0|+|u_1|+|u_2|+|u_3|)/2); it never falls below cos 45 deg."""
    rng = np.random.default_rng(12)
    sec = np.array([[1, 0, 0, 0]], np.float32)
    for _ in range(500):
        x = f16(rng.standard_normal(4))
        xf = x.view(np.float16).astype(np.float64)
        u = np.abs(xf) / np.linalg.norm(xf)
        _, best, _ = oracle.search_chunk(x, sec)
        assert best == pytest.approx(max(u.max(), 0.5 * u.sum()), abs=1e-15)
        assert best >= math.sqrt(0.5) - 1e-12


@pytest.mark.parametrize("S", [1, 16, 64])
def test_search_covering_bound(S):
    rng = np.random.default_rng(13 + S)
    sec = oracle.build_codebooks(0, 1, 1, S)[0, 0, 0]
    for _ in range(300):
        _, best, _ = oracle.search_chunk(f16(rng.standard_normal(4)), sec)
        assert best >= math.sqrt(0.5) - 1e-7


def test_search_exact_tie_takes_lowest_index():
    sec = np.array([[1, 0, 0, 0]], np.float32)
    k, best, second = oracle.search_chunk(f16([1, 1, 0, 0]), sec)
    # six vertices at the same distance: +1, +i and the four (1,1,+-1,+-1)/2
    P = oracle.primaries()
    u = np.array([1, 1, 0, 0]) / math.sqrt(2)
    tied = [p for p in range(24) if abs(P[p] @ u - best) < 1e-15]
    assert tied == [0, 2, 8, 9, 10, 11]
    assert k == 0 and best - second == 0.0


def test_search_zero_chunk():
    sec = oracle.build_codebooks(0, 1, 1, 4)[0, 0, 0]
    assert oracle.search_chunk(f16([0, -0.0, 0, 0]), sec) == (0, 0.0, 0.0)


@pytest.mark.parametrize("S,deg", [(1, 25.7), (16, 11.9), (64, 7.1)])
def test_mean_angular_error_trend(S, deg):
    """Haar-uniform directions: the mean angle to the nearest codeword falls like
    (24 S)^(-1/3) (Prop. 1); the values are Monte-Carlo figures for this construction."""
    rng = np.random.default_rng(99)
    sec = oracle.build_codebooks(0, 1, 1, S)[0, 0, 0]
    best = [oracle.search_chunk(f16(rng.standard_normal(4)), sec)[1] for _ in range(1500)]
    mean = np.degrees(np.arccos(np.clip(best, -1, 1))).mean()
    assert mean == pytest.approx(deg, rel=0.10)
    assert mean == pytest.approx(25.7 * S ** (-1 / 3), rel=0.25)


# ---------------------------------------------------------------------------------------
# norms, median, mask, outliers
# ---------------------------------------------------------------------------------------

def test_norm2_fixed_order_fp64():
    rng = np.random.default_rng(20)
    x = f16(rng.standard_normal((1000, 4)) * np.exp(rng.normal(0, 3, (1000, 1))))
    xf = x.view(np.float16).astype(np.float64)
    want = ((xf[:, 0] ** 2 + xf[:, 1] ** 2) + xf[:, 2] ** 2) + xf[:, 3] ** 2
    got = oracle.norm2(x).reshape(-1)
    assert np.array_equal(got, want)
    # exact value from integers: every fp16 is an integer multiple of 2^-24
    from fractions import Fraction
    for n in range(50):
        exact = sum(Fraction(float(v)) ** 2 for v in xf[n])
        assert abs(Fraction(float(got[n])) - exact) <= exact * Fraction(1, 2 ** 51)


def test_lower_median_against_numpy_sort_and_properties():
    rng = np.random.default_rng(21)
    for n in [1, 2, 3, 10, 11, 1000, 4097]:
        v = rng.standard_normal(n) ** 2
        v[rng.integers(0, n, n // 3)] = v[0]                  # duplicates
        m = oracle.lower_median(v)
        assert m == np.sort(v)[(n - 1) // 2]
        assert (v < m).sum() <= (n - 1) // 2 <= (v <= m).sum() - 1
        assert oracle.lower_median(rng.permutation(v)) == m


def _encode_small(x, S=4, **kw):
    B, H, T, D = x.shape
    sec = oracle.build_codebooks(0, 1, H, S)[0, 0]
    return oracle.encode(x, sec, **kw), sec


def test_median_is_per_head_over_batch_and_tokens():
    rng = np.random.default_rng(22)
    B, H, T = 2, 3, 8
    scale = np.array([1.0, 10.0, 0.1]).reshape(1, H, 1, 1)
    x = f16(rng.standard_normal((B, H, T, 128)) * scale)
    e, _ = _encode_small(x)
    r2 = oracle.norm2(x)                                        # [B, H, T, 32]
    for h in range(H):
        v = np.sort(r2[:, h].reshape(-1))
        assert e.m2[h] == v[(v.size - 1) // 2]


def test_mask_invariants():
    rng = np.random.default_rng(23)
    x = rng.standard_normal((1, 2, 64, 128)) * np.exp(rng.normal(0, 1.5, (1, 2, 64, 128)))
    e, _ = _encode_small(f16(x))
    n_h = 64 * 32
    assert e.n_out[2] == e.flag.sum() == e.n_out[:2].sum() and e.n_out[2] > 0
    assert (e.n_out[:2] <= n_h // 2).all()
    # strict inequality on squares against 9 * median
    for h in range(2):
        rows = slice(h * 64, (h + 1) * 64)
        assert np.array_equal(e.flag[rows].astype(bool), e.r2[rows] > 9.0 * e.m2[h])
    # scaling by a power of two changes nothing in the mask
    e2, _ = _encode_small(f16(2.0 * x.astype(np.float16).astype(np.float64)))
    assert np.array_equal(e.flag, e2.flag)
    # equal norms -> no outliers; extraction off -> no outliers
    e3, _ = _encode_small(f16(np.ones((1, 2, 16, 128))))
    assert e3.n_out[2] == 0 and not e3.flag.any()
    e4, _ = _encode_small(f16(x), use_outliers=False)
    assert e4.n_out[2] == 0 and not e4.flags.any()


def test_mask_fraction_gaussian_closed_form():
    """i.i.d. N(0,1) chunks: r^2 ~ chi^2_4, so P(r > C r_med) = exp(-t/2)(1 + t/2) at
    t = C^2 * median(chi^2_4).  Checked at C = 1.5 where the fraction is ~11 %."""
    from scipy.stats import chi2
    rng = np.random.default_rng(24)
    T = 8192
    x = f16(rng.standard_normal((1, 1, T, 128)))
    e, _ = _encode_small(x, S=1, Cmul=1.5, rows=[0])
    t = 1.5 ** 2 * chi2.median(4)
    want = math.exp(-t / 2) * (1 + t / 2)
    assert want == pytest.approx(chi2.sf(t, 4), rel=1e-12)
    assert e.n_out[1] / (T * 32) == pytest.approx(want, rel=0.02)


def test_outlier_list_layout():
    rng = np.random.default_rng(25)
    B, H, T = 2, 2, 16
    x = rng.standard_normal((B, H, T, 128)).astype(np.float16)
    x[0, 1, 3, 8:12] = [100, -0.0, 7, 1]
    x[1, 0, 0, 0:4] = [-300, 1, 1, 1]
    x[1, 0, 0, 124:128] = [0, 0, 0, 90]
    xb = x.view(np.uint16)
    e, _ = _encode_small(xb)
    chunks = xb.reshape(-1, 4)
    idx = np.flatnonzero(e.flag.reshape(-1))                   # ascending linear chunk index
    assert np.array_equal(e.outliers, chunks[idx])              # verbatim bits, incl. -0
    counts = e.flag.sum(1)
    assert np.array_equal(e.row_off, np.concatenate([[0], np.cumsum(counts)]))
    assert np.array_equal(e.flags, (e.flag.astype(np.uint64) << np.arange(32, dtype=np.uint64)).sum(1).astype(np.uint32))
    row = (0 * H + 1) * T + 3
    assert (e.flags[row] >> 2) & 1 and e.k[row, 2] == -1 and e.rq[row, 2] == -1
    per_head = [e.flag.reshape(B, H, T * 32)[:, h].sum() for h in range(H)]
    assert list(e.n_out) == per_head + [sum(per_head)]


# ---------------------------------------------------------------------------------------
# radius quantiser, packing, decode
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("b_r", [3, 4, 6, 8])
def test_radius_quantiser_bounds(b_r):
    rng = np.random.default_rng(30 + b_r)
    x = f16(rng.standard_normal((1, 2, 64, 128)) * np.exp(rng.normal(0, 1.0, (1, 2, 64, 128))))
    e, sec = _encode_small(x, b_r=b_r)
    L = 2 ** b_r - 1
    sig = e.sigma.view(np.float16).astype(np.float64)
    ok = e.flag == 0
    assert ((e.rq[ok] >= 0) & (e.rq[ok] <= L)).all()
    r = np.sqrt(e.r2)
    smax = np.where(ok, r, 0).max(1)
    assert np.array_equal(e.sigma, smax.astype(np.float16).view(np.uint16))   # numpy's RNE cast
    r_hat = e.rq * sig[:, None] / L
    err = np.abs(r - r_hat)[ok]
    bound = (sig[:, None] / (2 * L) + 2.0 ** -11 * sig[:, None]) * np.ones_like(r)
    assert (err <= bound[ok] * (1 + 1e-12)).all()
    # the largest unflagged chunk of every row takes the top code
    top = np.where(ok, r, -1).argmax(1)
    assert (e.rq[np.arange(e.rq.shape[0]), top] == L).all()
    # rounding is half-to-even: a value exactly between two codes
    assert oracle.radius_code(((2.5 / L) * 4.0) ** 2, int(f16(4.0)), b_r) == 2
    assert oracle.radius_code(((3.5 / L) * 4.0) ** 2, int(f16(4.0)), b_r) == 4
    assert oracle.radius_code(1.0, 0, b_r) == 0


@pytest.mark.parametrize("w", list(range(12, 22)))
def test_pack_layout_and_roundtrip(w):
    rng = np.random.default_rng(w)
    codes = rng.integers(0, 1 << w, 32, dtype=np.uint64).astype(np.uint32)
    words = oracle.pack_row(codes, w)
    assert words.shape == (w,)                                   # a row is exactly w dwords
    big = sum(int(c) << (i * w) for i, c in enumerate(codes))    # LSB-first concatenation
    assert [int(v) for v in words] == [(big >> (32 * i)) & 0xFFFFFFFF for i in range(w)]
    assert np.array_equal(oracle.unpack_row(words, w), codes)


def test_index_bits():
    for S, want in [(1, 5), (16, 9), (24, 10), (48, 11), (64, 11), (96, 12), (192, 13), (256, 13), (2730, 16), (2731, 17)]:
        assert oracle.index_bits(S) == want == math.ceil(math.log2(24 * S))


def test_decode_planted_codewords_and_outliers_roundtrip():
    rng = np.random.default_rng(40)
    B, H, T, S, b_r = 1, 2, 8, 8, 6
    L = 63
    sec = oracle.build_codebooks(3, 1, H, S)[0, 1]
    P = oracle.primaries()
    x = np.zeros((B, H, T, 128), np.float16)
    kk = rng.integers(0, 24 * S, (B, H, T, 32))
    qq = rng.integers(1, L + 1, (B, H, T, 32))
    qq[..., 0] = L                                               # sigma = 2.0 exactly on every row
    for h in range(H):
        for t in range(T):
            for c in range(32):
                k = kk[0, h, t, c]
                cw = matmul_product(P[k // S], sec[h, k % S].astype(np.float64))
                x[0, h, t, 4 * c:4 * c + 4] = (qq[0, h, t, c] * 2.0 / L) * cw
    # two outliers with awkward payloads
    x[0, 0, 2, 4:8] = [500, -0.0, 3, -7]
    x[0, 1, 5, 0:4] = [1000, 2, np.float16(6e-8), 0]
    xb = x.view(np.uint16).copy()
    e = oracle.encode(xb, sec, b_r=b_r)
    assert e.n_out[H] == 2
    ok = e.flag.reshape(B, H, T, 32) == 0
    # fp16 rounding of x perturbs directions by ~5e-4: the planted pair must still win
    assert (e.k.reshape(B, H, T, 32)[ok] == kk[ok]).mean() > 0.99
    out, r_hat = oracle.decode(e.codes, e.sigma, e.flags, e.row_off, e.outliers, sec, B, H, T, b_r, True)
    of = out.view(np.float16).astype(np.float64)
    xf = x.astype(np.float64)
    same = ok & (e.k.reshape(B, H, T, 32) == kk) & (e.rq.reshape(B, H, T, 32) == qq)
    assert same.mean() > 0.95
    err = np.abs(of - xf).reshape(B, H, T, 32, 4).max(-1)
    rn = np.linalg.norm(xf.reshape(B, H, T, 32, 4), axis=-1)
    assert (err[same] <= 1.5e-3 * rn[same]).all()                # two fp16 roundings + sigma rounding
    flagged = ~ok
    assert np.array_equal(out.reshape(B, H, T, 32, 4)[flagged], xb.reshape(B, H, T, 32, 4)[flagged])
    assert (r_hat.reshape(B, H, T, 32)[flagged] == 0).all()


def test_decode_formula_against_numpy():
    rng = np.random.default_rng(41)
    B, H, T, S, b_r = 1, 1, 4, 24, 4
    w_idx, L = 10, 15
    sec = oracle.build_codebooks(9, 1, H, S)[0, 0]
    k = rng.integers(0, 24 * S, (T, 32))
    q = rng.integers(0, L + 1, (T, 32))
    codes = np.stack([oracle.pack_row(((q[t] << w_idx) | k[t]).astype(np.uint32), w_idx + b_r) for t in range(T)])
    sigma = f16(rng.uniform(0.5, 4, T))
    flags = np.zeros(T, np.uint32)
    row_off = np.zeros(T + 1, np.uint32)
    out = oracle.decode(codes, sigma, flags, row_off, np.zeros((0, 4), np.uint16), sec, B, H, T, b_r)
    P = oracle.primaries()
    sf = sigma.view(np.float16).astype(np.float64)
    for t in range(T):
        for c in range(32):
            cw = matmul_product(P[k[t, c] // S], sec[0, k[t, c] % S].astype(np.float64))
            want = ((q[t, c] * sf[t] / L) * cw).astype(np.float16)
            got = out[0, 0, t, 4 * c:4 * c + 4].view(np.float16)
            # identical up to one fp16 ulp where the fp64 value sits on a rounding boundary
            assert np.allclose(got.astype(np.float64), want.astype(np.float64), rtol=1e-3, atol=1e-7)


def test_reconstruction_error_matches_angular_error():
    """decode(encode(x)) : relative error ~ sin(angle to codeword), radius error <= sigma/(2L)."""
    rng = np.random.default_rng(42)
    B, H, T, S = 1, 2, 32, 64
    x = f16(rng.standard_normal((B, H, T, 128)))
    sec = oracle.build_codebooks(0, 1, H, S)[0, 0]
    e = oracle.encode(x, sec)
    out = oracle.decode(e.codes, e.sigma, e.flags, e.row_off, e.outliers, sec, B, H, T, 6)
    xf = x.view(np.float16).astype(np.float64).reshape(-1, 4)
    of = out.view(np.float16).astype(np.float64).reshape(-1, 4)
    ok = e.flag.reshape(-1) == 0
    cosang = (xf * of).sum(1)[ok] / (np.linalg.norm(xf, axis=1) * np.linalg.norm(of, axis=1))[ok]
    assert np.allclose(cosang, e.best.reshape(-1)[ok], atol=2e-3)
    rel = np.linalg.norm(xf - of) / np.linalg.norm(xf)
    assert 0.08 < rel < 0.16                                     # ~ sin(7.1 deg) = 0.124 at S = 64


# ---------------------------------------------------------------------------------------
# single-query attention over the reconstructed cache
# ---------------------------------------------------------------------------------------

def test_attend_matches_numpy_softmax_einsum_with_gqa():
    from scipy.special import softmax
    rng = np.random.default_rng(50)
    B, Hq, H, T, D = 2, 6, 2, 37, 128
    q = rng.standard_normal((B, Hq, D)).astype(np.float16)
    K = rng.standard_normal((B, H, T, D))
    V = rng.standard_normal((B, H, T, D))
    scale = 1 / math.sqrt(D)
    o16, o64 = oracle.attend(q.view(np.uint16), K, V, scale)
    kv = np.repeat(np.arange(H), Hq // H)                       # query head -> kv head (grouped)
    s = np.einsum("bqd,bqtd->bqt", q.astype(np.float64), K[:, kv]) * scale
    want = np.einsum("bqt,bqtd->bqd", softmax(s, axis=-1), V[:, kv])
    assert np.allclose(o64, want, rtol=0, atol=1e-13)
    assert np.array_equal(o16, o64.astype(np.float16).view(np.uint16))      # numpy's RNE cast


def test_attend_lse_against_scipy_and_the_segment_merge_identity():
    """lse = logsumexp of the scaled scores; attention over a token range split in two equals the
    lse-weighted combination of the two parts (the identity a caller uses to combine segments)."""
    from scipy.special import logsumexp
    rng = np.random.default_rng(53)
    B, Hq, H, T, D = 2, 4, 2, 61, 128
    q = rng.standard_normal((B, Hq, D)).astype(np.float16)
    K = rng.standard_normal((B, H, T, D)) * 3
    V = rng.standard_normal((B, H, T, D))
    scale = 0.2
    _, o, lse = oracle.attend(q.view(np.uint16), K, V, scale, want_lse=True)
    kv = np.repeat(np.arange(H), Hq // H)
    s = np.einsum("bqd,bqtd->bqt", q.astype(np.float64), K[:, kv]) * scale
    assert np.allclose(lse, logsumexp(s, axis=-1), rtol=0, atol=1e-12)
    cut = 23
    _, o1, l1 = oracle.attend(q.view(np.uint16), K[:, :, :cut], V[:, :, :cut], scale, want_lse=True)
    _, o2, l2 = oracle.attend(q.view(np.uint16), K[:, :, cut:], V[:, :, cut:], scale, want_lse=True)
    L = np.logaddexp(l1, l2)
    merged = np.exp(l1 - L)[..., None] * o1 + np.exp(l2 - L)[..., None] * o2
    assert np.allclose(L, lse, atol=1e-12) and np.allclose(merged, o, atol=1e-12)


def test_attend_causal_limit_equals_attention_over_the_truncated_cache():
    """Query head hq with visible = v must equal plain attention over the first v tokens; v = 0 gives zeros
    and lse = -inf, v >= T the unmasked result."""
    rng = np.random.default_rng(54)
    B, Hq, H, T, D = 2, 6, 2, 40, 64
    q = rng.standard_normal((B, Hq, D)).astype(np.float16).view(np.uint16)
    K = rng.standard_normal((B, H, T, D))
    V = rng.standard_normal((B, H, T, D))
    vis = np.array([[0, 1, 7, 39, 40, 1000], [40, 3, 0, 25, 12, 41]], np.int32)
    _, o, lse = oracle.attend(q, K, V, 0.3, want_lse=True, visible=vis)
    for b in range(B):
        for hq_ in range(Hq):
            v = min(int(vis[b, hq_]), T)
            if v == 0:
                assert not o[b, hq_].any() and lse[b, hq_] == -np.inf
                continue
            h = hq_ // (Hq // H)
            _, o1, l1 = oracle.attend(q[b:b + 1, hq_:hq_ + 1], K[b:b + 1, h:h + 1, :v], V[b:b + 1, h:h + 1, :v], 0.3,
                                      want_lse=True)
            assert np.array_equal(o[b, hq_], o1[0, 0]) and lse[b, hq_] == l1[0, 0]


def test_attend_invariants():
    rng = np.random.default_rng(51)
    B, Hq, H, T, D = 1, 4, 1, 50, 128
    q = rng.standard_normal((B, Hq, D)).astype(np.float16).view(np.uint16)
    K = rng.standard_normal((B, H, T, D))
    V = rng.standard_normal((B, H, T, D))
    _, o = oracle.attend(q, K, V, 0.1)
    # a convex combination of the value rows
    assert (o <= V.max(2) + 1e-12).all() and (o >= V.min(2) - 1e-12).all()
    # permuting the tokens changes nothing; zero scale gives the plain mean
    perm = rng.permutation(T)
    _, o2 = oracle.attend(q, K[:, :, perm], V[:, :, perm], 0.1)
    assert np.allclose(o, o2, atol=1e-13)
    _, o3 = oracle.attend(q, K, V, 0.0)
    assert np.allclose(o3, np.broadcast_to(V.mean(2), o3.shape), atol=1e-13)
    # a key aligned with the query and a huge scale picks that token's value
    K2 = K.copy()
    K2[0, 0, 7] = 50 * q.view(np.float16).astype(np.float64)[0, 2]
    _, o4 = oracle.attend(q, K2, V, 5.0)
    assert np.allclose(o4[0, 2], V[0, 0, 7], atol=1e-9)


def test_decode64_rounds_to_decode():
    rng = np.random.default_rng(52)
    x = f16(rng.standard_normal((1, 2, 16, 128)) * np.exp(rng.normal(0, 1.2, (1, 2, 16, 128))))
    e, sec = _encode_small(x, S=16)
    d16 = oracle.decode(e.codes, e.sigma, e.flags, e.row_off, e.outliers, sec, 1, 2, 16, 6)
    d64 = oracle.decode64(e.codes, e.sigma, e.flags, e.row_off, e.outliers, sec, 1, 2, 16, 6)
    assert e.n_out[-1] > 0
    assert np.array_equal(d64.astype(np.float16).view(np.uint16), d16)      # numpy's RNE cast


# ---------------------------------------------------------------------------------------
# numbers the paper prints
# ---------------------------------------------------------------------------------------

def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_bit_accounting_table():
    for name, S, b_r, lg, per_chunk, per_elem, with_scale in _rows("bit_accounting.txt"):
        S, b_r = int(S), int(b_r)
        assert round(math.log2(24 * S), 2) == float(lg)
        bare = oracle.bits_per_element(S, b_r, d_h=10 ** 12)
        assert round(4 * bare, 2) == float(per_chunk)
        assert round(bare, 2) == float(per_elem)
        assert round(oracle.bits_per_element(S, b_r, 128), 2) == float(with_scale)


def test_memory_table_and_headlines():
    for name, S, b_r, bits, ratio in _rows("memory_table.txt"):
        b = oracle.bits_per_element(int(S), int(b_r), 128)
        assert round(b, 2) == float(bits)
        assert round(16.0 / b, 2) == pytest.approx(float(ratio), abs=0.011)
    b = oracle.bits_per_element(24, 3, 128)
    llama70 = 2 * 80 * 8 * 128 * 131072 * 2                     # K and V, 80 layers, 8 KV heads, fp16
    assert round(llama70 / 1e9) == 43 and round(llama70 * b / 16 / 1e9, 1) == 8.5
    mistral = 2 * 32 * 8 * 128 * 32768 * 2
    assert round(mistral / 1e9, 1) == 4.3 and round(mistral * b / 16 / 1e6, -1) == 850
    # Eq. (2) and the stored (ceil) width
    assert oracle.bits_per_element(256, 6, 128, p=0.02) == pytest.approx(
        0.98 * oracle.bits_per_element(256, 6, 128) + 0.32 + 0.25)
    assert oracle.bits_per_element(256, 6, 128, stored=True) == (13 + 6) / 4 + 0.125


# ---------------------------------------------------------------------------------------
# head dimensions other than 128: rows of 1..32 chunks, and the padding wrapper
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("nc", [1, 5, 11, 16, 24, 31, 32])
@pytest.mark.parametrize("w", [10, 13, 17, 22])
def test_pack_row_any_chunk_count_against_big_integer(nc, w):
    """The packed row read as one little-endian integer is sum(code_c << (c w))."""
    rng = np.random.default_rng(100 * nc + w)
    code = rng.integers(0, 1 << w, nc, dtype=np.uint64).astype(np.uint32)
    words = oracle.pack_row(code, w)
    assert words.size == -(-nc * w // 32)
    big = sum(int(c) << (i * w) for i, c in enumerate(code))
    want = [(big >> (32 * i)) & 0xFFFFFFFF for i in range(words.size)]
    assert [int(v) for v in words] == want
    assert np.array_equal(oracle.unpack_row(words, w, nc), code)


def _embed(x_bits, D_to):
    out = np.zeros(x_bits.shape[:-1] + (D_to,), np.uint16)
    out[..., : x_bits.shape[-1]] = x_bits
    return out


@pytest.mark.parametrize("D", [64, 96, 45, 4])
@pytest.mark.parametrize("with_thresholds", [False, True])
def test_short_heads_equal_the_zero_padded_128_wide_tensor(D, with_thresholds):
    """Zero chunks have no direction, no radius and are never flagged, so a head of D < 128
    elements must encode exactly like the same rows padded with zeros to 128, chunk by chunk
    (thresholds supplied, or extraction off, so that the padding does not move the median)."""
    rng = np.random.default_rng(D)
    B, H, T, S, b_r = 2, 2, 5, 24, 4
    x = (rng.standard_normal((B, H, T, D)) * np.exp(rng.normal(0, 1.0, (B, H, T, D)))).astype(np.float16)
    x[0, 0, 1] = 0  # a zero row
    xb = x.view(np.uint16)
    sec = oracle.build_codebooks(7, 1, H, S)[0, 0]
    thr = np.array([2.0, 0.7]) if with_thresholds else None
    kw = dict(b_r=b_r, thresholds=thr) if with_thresholds else dict(b_r=b_r, use_outliers=False)
    e = oracle.encode(xb, sec, **kw)
    full = oracle.encode(_embed(xb, 128), sec, **kw)
    nc = oracle.chunks_per_row(D)
    assert e.k.shape == (B * H * T, nc) and e.codes.shape[1] == oracle.row_words(D, oracle.index_bits(S) + b_r)
    assert np.array_equal(e.k, full.k[:, :nc]) and np.array_equal(e.rq, full.rq[:, :nc])
    assert np.array_equal(e.flag, full.flag[:, :nc]) and not full.flag[:, nc:].any()
    assert np.array_equal(e.sigma, full.sigma) and np.array_equal(e.flags, full.flags)
    assert np.array_equal(e.row_off, full.row_off) and np.array_equal(e.n_out, full.n_out)
    assert np.array_equal(e.outliers, full.outliers)
    if with_thresholds:
        assert e.flag.any()
    k2, rq2 = oracle.unpack_rows(e.codes, S, b_r, nc)
    keep = e.flag == 0
    assert np.array_equal(k2[keep], e.k[keep]) and np.array_equal(rq2[keep], e.rq[keep])
    assert not k2[~keep].any() and not rq2[~keep].any()
    out = oracle.decode(e.codes, e.sigma, e.flags, e.row_off, e.outliers, sec, B, H, T, b_r, D=D)
    out_full = oracle.decode(full.codes, full.sigma, full.flags, full.row_off, full.outliers, sec, B, H, T, b_r)
    assert out.shape == (B, H, T, D)
    assert np.array_equal(out, out_full[..., :D])
    # what lies beyond D decodes to zeros in the padded tensor (code 0 with r_q = 0)
    assert not (out_full[..., 4 * nc:] & 0x7FFF).any()


@pytest.mark.parametrize("D", [64, 96, 45])
def test_median_of_short_heads_against_numpy_sort(D):
    rng = np.random.default_rng(5 + D)
    B, H, T = 2, 3, 7
    x = rng.standard_normal((B, H, T, D)).astype(np.float16)
    sec = oracle.build_codebooks(0, 1, H, 4)[0, 0]
    e = oracle.encode(x.view(np.uint16), sec, b_r=3, rows=np.zeros(B * H * T, bool))
    nc = oracle.chunks_per_row(D)
    xp = np.zeros((B, H, T, 4 * nc)); xp[..., :D] = x.astype(np.float64)
    r2 = (xp.reshape(B, H, T, nc, 4) ** 2).sum(-1)
    for h in range(H):
        v = np.sort(r2[:, h].reshape(-1))
        assert e.m2[h] == pytest.approx(v[(v.size - 1) // 2], rel=1e-15)
        want_flag = r2[:, h] > 9.0 * e.m2[h]
        got = e.flag.reshape(B, H, T, nc)[:, h].astype(bool)
        assert np.array_equal(got, want_flag)


def test_padding_overhead_printed_example():
    for line in open(os.path.join(GOLDEN, "padding_overhead.txt")):
        if line.startswith("#") or not line.strip():
            continue
        d_h, padded, pct = line.split()
        assert 4 * oracle.chunks_per_row(int(d_h)) == int(padded)
        assert round(100 * oracle.padding_overhead(int(d_h)), 1) == float(pct)
    for d in (64, 96, 128):  # the paper's models need no padding
        assert oracle.padding_overhead(d) == 0.0


def test_scale_term_of_the_bit_accounting_follows_the_head_dimension():
    # b = (log2(24 S) + b_r) / 4 + 16 / d_h: only the last term depends on d_h
    for S, b_r in ((24, 3), (192, 4)):
        b128 = oracle.bits_per_element(S, b_r, 128)
        assert oracle.bits_per_element(S, b_r, 64) - b128 == pytest.approx(16 / 64 - 16 / 128)
        assert oracle.bits_per_element(S, b_r, 96) - b128 == pytest.approx(16 / 96 - 16 / 128)
