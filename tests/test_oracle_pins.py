"""Pins of the float64 oracle against what the paper and the mathematics fix.

None of these tests touches the HIP library.  Each names the passage or the
closed form it pins and is chosen so that a plausible slip in the oracle (wrong
index, dropped term, swapped side, transposed operand) fails it.
"""
import math

import numpy as np
import pytest
from scipy import integrate, stats

import oracle


# ----------------------------------------------------------------- constants
def test_pilot_k_printed_values(golden):
    # Remark 3.1 prints k = 11 at d = 128; the appendix remark gives ~7 at d = 64
    assert oracle.pilot_k(128) == int(golden["pilot_k_d128"][0])
    assert oracle.pilot_k(64) == int(golden["pilot_k_d64"][0])


def test_edge_constant():
    assert abs(oracle.EDGE_COEF - 1.7024143839193153) < 1e-15
    assert abs(oracle.rank_threshold(128) - 128 ** (-1 / 3)) < 1e-16
    assert abs(oracle.rank_threshold(128) - 0.19842513149602492) < 1e-15


# ------------------------------------------------------------------ codebook
def test_lloyd_max_known_centroids(golden):
    c1 = oracle.lloyd_max_gaussian(1)
    assert np.allclose(c1.centroids, [-golden["lloyd_1bit"][0], golden["lloyd_1bit"][0]], atol=1e-9)
    assert abs(c1.centroids[1] - math.sqrt(2 / math.pi)) < 1e-14
    c2 = oracle.lloyd_max_gaussian(2)
    a, b = golden["lloyd_2bit"]
    assert np.allclose(c2.centroids, [-b, -a, a, b], atol=6e-4)   # printed to 4 significant digits


@pytest.mark.parametrize("bits", [1, 2, 3, 4])
def test_lloyd_max_fixed_point_by_quadrature(bits):
    """Centroid = conditional mean of its cell, boundary = midpoint: checked with
    numerical integration of the density, not with the erf formula the oracle uses."""
    cb = oracle.lloyd_max_gaussian(bits)
    assert cb.centroids.shape == (1 << bits,) and cb.bounds.shape == ((1 << bits) - 1,)
    assert np.all(np.diff(cb.centroids) > 0)
    assert np.allclose(cb.bounds, 0.5 * (cb.centroids[:-1] + cb.centroids[1:]), atol=1e-15)
    assert np.allclose(cb.centroids, -cb.centroids[::-1], atol=1e-15)
    edges = np.r_[-np.inf, cb.bounds, np.inf]
    pdf = stats.norm.pdf
    dist = 0.0
    for i, c in enumerate(cb.centroids):
        lo, hi = max(edges[i], -40.0), min(edges[i + 1], 40.0)
        mass = integrate.quad(pdf, lo, hi, epsabs=1e-14, epsrel=1e-13)[0]
        mean = integrate.quad(lambda x: x * pdf(x), lo, hi, epsabs=1e-14, epsrel=1e-13)[0] / mass
        assert abs(mean - c) < 1e-10
        dist += integrate.quad(lambda x: (x - c) ** 2 * pdf(x), lo, hi, epsabs=1e-14, epsrel=1e-13)[0]
    assert abs(dist - cb.distortion) < 1e-10
    assert cb.centroids_f32.dtype == np.float32 and cb.bounds_f32.dtype == np.float32
    assert np.array_equal(cb.centroids_f32, cb.centroids.astype(np.float32))


def test_lloyd_max_distortion_matches_paper_tables(golden):
    """sqrt(D_b) is the relative L2 error of TQ_MSE on isotropic rows; Tables 1-4
    print 34.1-34.2 / 18.4-18.5 / 9.7 percent for b = 2, 3, 4."""
    for key in ("table1_tqmse_l2", "table2_tqmse_l2", "table3_tqmse_l2", "table4_tqmse_l2"):
        for bits, printed in zip((2, 3, 4), golden[key]):
            assert abs(100 * math.sqrt(oracle.lloyd_max_gaussian(bits).distortion) - printed) < 0.25


def test_nearest_centroid_equals_boundary_count():
    rng = np.random.default_rng(3)
    d = 128
    Pi = np.eye(d)
    for bits in (1, 2, 3, 4):
        cb = oracle.lloyd_max_gaussian(bits)
        x = rng.standard_normal((16, d))
        codes, rho, z = oracle.tq_mse_encode(x, Pi, cb)
        t = z * math.sqrt(d)
        brute = np.argmin(np.abs(t[:, :, None] - cb.centroids[None, None, :]), axis=2)
        margin = np.min(np.abs(t[:, :, None] - cb.bounds[None, None, :]), axis=2)
        ok = margin > 1e-6     # away from ties the two definitions agree
        assert ok.mean() > 0.999 and np.array_equal(codes[ok], brute[ok])
        assert codes.min() == 0 and codes.max() == (1 << bits) - 1


# ------------------------------------------------------------------ rotation
def test_gaussian_stream_is_standard_normal():
    g = oracle.gaussian_stream(12345, 200000)
    assert abs(g.mean()) < 0.01 and abs(g.var() - 1.0) < 0.01
    assert stats.kstest(g, "norm").pvalue > 1e-3
    # counter based: a prefix of a longer stream is the shorter stream
    assert np.array_equal(g[:1000], oracle.gaussian_stream(12345, 1000))
    assert not np.array_equal(g[:1000], oracle.gaussian_stream(12346, 1000))


def test_splitmix64_reference_vector():
    # first outputs of SplitMix64 seeded with 0 (published test vector of the generator)
    out = oracle.splitmix64(0, np.arange(3, dtype=np.uint64))
    assert [int(x) for x in out] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


@pytest.mark.parametrize("d", [8, 128])
def test_haar_rotation_orthogonal_and_sign_fixed(d):
    seed = 260502906
    Pi = oracle.haar_rotation(d, seed)
    assert np.abs(Pi.T @ Pi - np.eye(d)).max() < 1e-13
    assert np.abs(Pi @ Pi.T - np.eye(d)).max() < 1e-13
    assert abs(abs(np.linalg.det(Pi)) - 1.0) < 1e-10
    u = np.random.default_rng(0).standard_normal(d)
    assert abs(np.linalg.norm(Pi @ u) - np.linalg.norm(u)) < 1e-12
    # Q^T G must be upper triangular with a positive diagonal (the Haar sign convention)
    G = oracle.gaussian_stream(seed, d * d).reshape(d, d)
    R = Pi.T @ G
    assert np.abs(np.tril(R, -1)).max() < 1e-10
    assert np.all(np.diag(R) > 0)


# ------------------------------------------------------------------ SVD step
def _jacobi_eigh(A, sweeps=50):
    """Textbook cyclic Jacobi on a small symmetric matrix, pure Python loops."""
    A = A.copy()
    m = A.shape[0]
    V = np.eye(m)
    for _ in range(sweeps):
        for p in range(m - 1):
            for q in range(p + 1, m):
                if abs(A[p, q]) < 1e-300:
                    continue
                th = 0.5 * math.atan2(2 * A[p, q], A[q, q] - A[p, p])
                c, s = math.cos(th), math.sin(th)
                J = np.eye(m)
                J[p, p] = c; J[q, q] = c; J[p, q] = s; J[q, p] = -s
                A = J.T @ A @ J
                V = V @ J
    return np.diag(A), V


@pytest.mark.parametrize("shape", [(8, 4), (6, 5), (12, 6)])
def test_svd_against_brute_force_on_tiny_blocks(shape):
    rng = np.random.default_rng(shape[0])
    S = rng.standard_normal(shape)
    es = oracle.eoptshrink(S, r_max=1)
    lam_bf, V_bf = _jacobi_eigh(S.T @ S)
    order = np.argsort(-lam_bf)
    assert np.allclose(es.lam, lam_bf[order], rtol=1e-10)
    # Sec. 2.3: lambda_i = sigma_i^2 are the eigenvalues of S S^T as well
    assert np.allclose(np.sort(np.linalg.eigvalsh(S @ S.T))[::-1][:shape[1]], es.lam, rtol=1e-9)
    # plant a strong direction so that at least one component is retained and its vectors can be checked
    S2 = S + 8.0 * np.outer(rng.standard_normal(shape[0]), np.eye(shape[1])[0])
    full = oracle.eoptshrink(S2, r_max=shape[1])
    lam_bf, V_bf = _jacobi_eigh(S2.T @ S2)
    order = np.argsort(-lam_bf)
    assert full.rank >= 1 or shape[1] - 2 * full.k - 1 == 0
    S = S2
    for i in range(full.rank):
        v_bf = V_bf[:, order[i]]
        assert abs(abs(v_bf @ full.V[:, i]) - 1.0) < 1e-8
        assert np.allclose(S @ full.V[:, i], full.sigma[i] * full.U[:, i], atol=1e-10)


# ------------------------------------------------------- Alg. 2 Step 1: edge
def _spiked(rng, n, d, strengths, channel=None):
    r = len(strengths)
    Z = rng.standard_normal((n, r))
    W, _ = np.linalg.qr(rng.standard_normal((d, r)))
    sig = (Z * np.asarray(strengths)) @ W.T if r else np.zeros((n, d))
    E = rng.standard_normal((n, d))
    if channel is not None:
        E = E * channel
    return sig + E, sig, E


@pytest.mark.parametrize("n,d,tol", [(512, 128, 0.03), (1024, 128, 0.03), (128, 128, 0.09)])
def test_bulk_edge_on_white_noise_is_marchenko_pastur_edge(n, d, tol):
    """Sec. 2.3: for iid noise the bulk edge is sigma^2 (1 + sqrt(beta))^2, i.e.
    (sqrt(n) + sqrt(d))^2 for unit-variance entries."""
    k = oracle.pilot_k(d)
    vals = []
    for seed in range(24):
        S = np.random.default_rng(1000 + seed).standard_normal((n, d))
        lam = np.linalg.svd(S, compute_uv=False) ** 2
        vals.append(oracle.bulk_edge(lam, k))
    exact = (math.sqrt(n) + math.sqrt(d)) ** 2
    # (the estimator extrapolates from the k+1-th and 2k+1-th of only 128 eigenvalues: a few percent of
    # finite-size bias, largest for the square block whose spectrum is widest)
    assert abs(np.mean(vals) / exact - 1.0) < tol
    assert np.max(np.abs(np.array(vals) / exact - 1.0)) < tol + 0.08


def test_bulk_edge_uses_the_printed_indices():
    """Alg. 2 Step 1 on an exact square-root-edge spectrum lam_j = L - c j^{2/3}:
    extrapolating from j = k+1 and 2k+1 must return L + c(k+1)^{2/3} ... exactly
    the printed formula; with j measured from the edge itself (lam_j = L - c (j-1/2... )
    it would not.  Use the model the constant 2^{2/3}-1 is exact for: positions k and 2k."""
    k = 11
    L, c = 100.0, 0.37
    j = np.arange(0, 64, dtype=float)        # 0-based index i holds lam_{i+1}
    # place the law so that entry k (lam_{k+1}) sits at offset k^{2/3}, entry 2k at (2k)^{2/3}
    lam = L - c * j ** (2.0 / 3.0)
    assert abs(oracle.bulk_edge(lam, k) - L) < 1e-12
    # an off-by-one in either index breaks exactness
    a, b = lam[k + 1], lam[2 * k]
    assert abs(a + oracle.EDGE_COEF * (a - b) - L) > 1e-3


# ------------------------------------------------------- Alg. 2 Step 1: rank
def test_planted_rank_recovered_above_bbp_and_none_below():
    n, d = 512, 128
    u_bbp = (n * d) ** 0.25        # white-noise detection threshold on the singular-value scale
    for seed in range(12):
        rng = np.random.default_rng(seed)
        S, _, _ = _spiked(rng, n, d, (6.0, 4.0, 2.5))         # singular values ~ (136, 90, 57) >> 16
        assert oracle.eoptshrink(S).rank == 3
    for seed in range(40):
        S = np.random.default_rng(500 + seed).standard_normal((n, d))
        assert oracle.eoptshrink(S).rank == 0                  # Remark 3.1: isotropic block -> r = 0
    for seed in range(12):
        rng = np.random.default_rng(900 + seed)
        weak = 0.5 * u_bbp / math.sqrt(n)                      # half the BBP threshold: sticks to the bulk
        S, _, _ = _spiked(rng, n, d, (6.0, weak, weak))
        assert oracle.eoptshrink(S).rank == 1


def test_rank_threshold_is_strict_and_relative():
    d, k = 128, 11
    lam = np.linspace(2.0, 1.0, 128)
    lp = oracle.bulk_edge(lam, k)
    thr = (1.0 + oracle.rank_threshold(d)) * lp
    lam2 = lam.copy()
    lam2[0] = thr * (1 + 1e-9)
    assert oracle.estimate_rank(lam2, d, k)[0] == 1
    lam2[0] = thr * (1 - 1e-9)
    lam2[:2] = np.sort(lam2[:2])[::-1]
    assert oracle.estimate_rank(lam2, d, k)[0] == 0
    r1, _ = oracle.estimate_rank(lam2 * 37.0, d, k)           # scale free
    assert r1 == 0


# ------------------------------------------------ Alg. 2 Step 2: imputation
def test_imputation_follows_the_square_root_edge_law_exactly():
    """Alg. 2 Step 2 is the square-root edge law lam_j ~ L - c (j-1)^{2/3} of the noise bulk, extrapolated from its
    (k+1)-th and (2k+1)-th atoms.  On a spectrum that obeys the law exactly -- r outliers in front, noise atom j
    (1-based) at L - c (j-1)^{2/3}, so the first noise atom sits on the edge L -- the printed rule must return
    L - c j^{2/3} for j = 1..k: imputed atom j is the true atom j+1 (the printed indices, kept as they are), whatever
    r, L and c.  This is the closed form of the law, not the rule's own expression; reading either eigenvalue one
    position off misses it by far more than the bar."""
    N = 128
    for k, r, L, c in [(11, 3, 50.0, 0.2), (11, 0, 7.0, 0.01), (7, 5, 1e4, 30.0), (11, 32, 2.5, 0.004)]:
        jj = np.arange(1, N - r + 1, dtype=float)
        noise = L - c * (jj - 1.0) ** (2.0 / 3.0)
        lam = np.r_[L * (10.0 + np.arange(r, 0, -1)), noise]
        atoms = oracle.impute_noise_spectrum(lam, r, k)
        assert atoms.shape == (N - r,)
        want = L - c * np.arange(1, k + 1, dtype=float) ** (2.0 / 3.0)
        assert np.max(np.abs(atoms[:k] - want)) < 1e-12 * L
        assert np.max(np.abs(atoms[:k] - noise[1:k + 1])) < 1e-12 * L       # imputed atom j = true atom j + 1
        assert np.array_equal(atoms[k:], lam[r + k:])                        # the rest is copied
        # non-increasing; the single tie is atom k, which the printed rule places on the first copied atom
        dd = np.diff(atoms)
        assert np.all(dd[:k - 1] < 0) and abs(dd[k - 1]) < 1e-12 * L and np.all(dd[k:] < 0)
        # the same rule fed with a neighbouring eigenvalue (an off-by-one in either index, or r forgotten) is off by
        # more than 1e-3 c in some atom
        def rule(a, b):
            j = np.arange(1, k + 1, dtype=float)
            return a + (1.0 - (j / k) ** (2.0 / 3.0)) * oracle.EDGE_COEF * (a - b)
        for da, db in [(-1, 0), (1, 0), (0, -1), (0, 1), (-1, -1), (1, 1)]:
            wrong = rule(lam[k + r + da], lam[2 * k + r + db])
            assert np.max(np.abs(wrong - want)) > 1e-3 * c, (k, r, da, db)
        if r:
            assert np.max(np.abs(rule(lam[k], lam[2 * k]) - want)) > 1e-3 * c


# --------------------------------------------------- Alg. 2 Step 3: shrinker
def test_shrinker_matches_white_noise_closed_form_and_true_overlaps():
    """White noise (A = B = I) is the special case with a textbook answer: for an observed singular value y
    of an n x d matrix with unit-variance noise the Frobenius-optimal value is
    sqrt((y^2 - n - d)^2 - 4 n d) / y.  The D-transform estimates must also recover the planted strengths
    and the *measured* overlaps |<u_i, xi_i>|^2 (left, a_1) and |<v_i, zeta_i>|^2 (right, a_2) of Eq. (overlaps)."""
    n, d = 512, 128
    rows = []
    for seed in range(24):
        rng = np.random.default_rng(seed)
        S, sig, _ = _spiked(rng, n, d, (6.0, 4.0, 2.5))
        Us, ss, Vts = np.linalg.svd(sig, full_matrices=False)
        es = oracle.eoptshrink(S)
        assert es.rank == 3 and es.flags == 0
        y = es.sigma
        closed = np.sqrt((y ** 2 - n - d) ** 2 - 4 * n * d) / y
        o1 = np.array([(Us[:, i] @ es.U[:, i]) ** 2 for i in range(3)])
        o2 = np.array([(Vts[i] @ es.V[:, i]) ** 2 for i in range(3)])
        rows.append(np.r_[es.phi / closed, es.d_hat / ss[:3], es.a1 - o1, es.a2 - o2])
        assert np.all(es.phi < es.sigma) and np.all(es.phi > 0)
    m = np.mean(rows, axis=0)
    assert np.all(np.abs(m[0:3] - 1.0) < 0.006)        # shrunk values vs closed form
    assert np.all(np.abs(m[3:6] - 1.0) < 0.01)         # d_hat vs planted strength
    assert np.all(np.abs(m[6:9]) < 0.01)               # a_1 vs measured left overlap
    assert np.all(np.abs(m[9:12]) < 0.01)              # a_2 vs measured right overlap
    # the two overlaps differ by much more than the tolerance, so a swapped labelling fails
    assert np.all(np.array(rows)[:, 9:12].mean(0) + 0.0 < 0.01)
    assert (es.a2 - es.a1).min() > 0.015


def test_noise_measure_is_normalised_by_its_number_of_atoms():
    """Eq. (Fe) prints a sum over n ^ d indices with 1/(n ^ d) in front although the r outliers have been discarded:
    either the weight is 1/(n ^ d) and the measure has mass 1 - r/(n ^ d), or it is 1/M over the M = n ^ d - r atoms
    that exist.  What decides: the estimator must recover a planted strength without bias.  Over 96 independent
    white-noise blocks with three planted components the mean of d_hat / (true singular value of the signal) is 1 to
    a quarter of a percent with 1/M, and 1.5 % high (about ten standard errors) with 1/(n ^ d).  The alternative is
    written out here from Eq. (d_transform); the oracle's own d_hat must be the 1/M one."""
    n, d = 512, 128
    beta = d / n

    def strength(z, atoms, weight):
        m_s = weight * np.sum(1.0 / (atoms - z))
        m_l = beta * m_s - (1.0 - beta) / z
        return 1.0 / math.sqrt(z * m_s * m_l)

    by_atoms, by_size = [], []
    for seed in range(96):
        rng = np.random.default_rng(seed)
        S, sig, _ = _spiked(rng, n, d, (6.0, 4.0, 2.5))
        true = np.linalg.svd(sig, compute_uv=False)[:3]
        es = oracle.eoptshrink(S)
        assert es.rank == 3
        lam = np.linalg.svd(S, compute_uv=False) ** 2
        atoms = oracle.impute_noise_spectrum(lam, 3, oracle.pilot_k(d))
        assert atoms.shape[0] == d - 3
        dm = np.array([strength(z, atoms, 1.0 / atoms.shape[0]) for z in lam[:3]])
        dn = np.array([strength(z, atoms, 1.0 / d) for z in lam[:3]])
        assert np.allclose(dm, es.d_hat, rtol=1e-10)
        by_atoms.append(dm / true - 1.0)
        by_size.append(dn / true - 1.0)
    by_atoms, by_size = np.array(by_atoms), np.array(by_size)
    sem = by_atoms.std(axis=0) / math.sqrt(by_atoms.shape[0])
    assert np.all(sem < 0.0025)
    assert np.all(np.abs(by_atoms.mean(axis=0)) < 3.0 * sem + 5e-4), by_atoms.mean(axis=0)
    assert np.all(by_size.mean(axis=0) > 0.012) and np.all(by_size.mean(axis=0) > 6.0 * sem), by_size.mean(axis=0)


def _white_noise_closed_forms(y, n, d):
    """Textbook white-noise (A = B = I) quantities for an observed singular value y of an n x d matrix, n >= d, with
    unit-variance noise: the signal strength x behind y, the asymptotic overlaps on the long side (left vectors, R^n)
    and on the short side (right vectors, R^d), with beta = d / n and everything in units of sqrt(n):
      y^2 = (x^2 + 1)(x^2 + beta) / x^2,   a_long = (x^4 - beta)/(x^4 + x^2),   a_short = (x^4 - beta)/(x^4 + beta x^2)."""
    beta = d / n
    y2 = y * y / n
    x2 = 0.5 * ((y2 - beta - 1.0) + np.sqrt((y2 - beta - 1.0) ** 2 - 4.0 * beta))
    a_long = (x2 * x2 - beta) / (x2 * x2 + x2)
    a_short = (x2 * x2 - beta) / (x2 * x2 + beta * x2)
    return np.sqrt(x2 * n), a_long, a_short


def test_operator_and_nuclear_shrinkers_match_their_white_noise_closed_forms():
    """Eq. (shrinkers), cases 2 and 3, in the white-noise special case where strength and overlaps have closed forms:
    operator  x sqrt(a_long / a_short)  (the long side has the smaller overlap), nuclear
    x (sqrt(a_long a_short) - sqrt((1 - a_long)(1 - a_short))).  Also what holds for any spectrum:
    phi_op <= d_hat, phi_nuc <= phi_fro <= phi_op, and all three share d_hat, a_1, a_2."""
    n, d = 512, 128
    ratios = {"operator": [], "nuclear": []}
    for seed in range(24):
        rng = np.random.default_rng(seed)
        S, _, _ = _spiked(rng, n, d, (6.0, 4.0, 2.5))
        fro = oracle.eoptshrink(S)
        x, a_long, a_short = _white_noise_closed_forms(fro.sigma, n, d)
        closed = {"operator": x * np.sqrt(a_long / a_short),
                  "nuclear": x * (np.sqrt(a_long * a_short) - np.sqrt((1 - a_long) * (1 - a_short)))}
        # the closed forms themselves reproduce the Frobenius pin of the test above
        y = fro.sigma
        assert np.allclose(x * np.sqrt(a_long * a_short), np.sqrt((y ** 2 - n - d) ** 2 - 4 * n * d) / y, rtol=1e-12)
        for loss in ("operator", "nuclear"):
            es = oracle.eoptshrink(S, loss=loss)
            assert es.rank == 3 and es.flags == 0
            assert np.array_equal(es.d_hat, fro.d_hat) and np.array_equal(es.a1, fro.a1) and np.array_equal(es.a2, fro.a2)
            ratios[loss].append(es.phi / closed[loss])
            if loss == "operator":
                assert np.all(es.phi <= es.d_hat) and np.all(es.phi >= fro.phi)
                # the printed ratio is min/max: with the overlaps swapped or the root dropped it moves by several percent
                assert np.all(np.abs(es.phi / (es.d_hat * np.sqrt(es.a1 / es.a2)) - 1.0) < 1e-12) and np.all(es.a1 < es.a2)
            else:
                assert np.all(es.phi <= fro.phi) and np.all(es.phi > 0)
    for loss in ratios:
        m = np.mean(ratios[loss], axis=0)
        assert np.all(np.abs(m - 1.0) < 0.008), (loss, m)
    # a component whose overlaps are small gets a negative nuclear expression: shrunk to zero, not below
    phi, dh, a1, a2, ok = oracle.shrink(1.02 * 1152.0, np.linspace(1152.0, 100.0, 125), 512, 128, "nuclear")
    assert ok and phi == 0.0 and a1 * a2 < (1 - a1) * (1 - a2)
    with pytest.raises(ValueError):
        oracle.shrink(2000.0, np.linspace(1152.0, 100.0, 125), 512, 128, "huber")


def test_shrinker_tall_and_wide_blocks_agree():
    """A block and its transpose have the same singular values; the shrunk values must agree and the
    overlap estimates swap sides."""
    rng = np.random.default_rng(5)
    S, _, _ = _spiked(rng, 256, 128, (5.0, 3.0))
    es = oracle.eoptshrink(S)
    lam = es.lam
    for i in range(es.rank):
        p1, d1, a1, a2, ok1 = oracle.shrink(lam[i], es.atoms, 256, 128)
        p2, d2, b1, b2, ok2 = oracle.shrink(lam[i], es.atoms, 128, 256)
        assert ok1 and ok2
        assert abs(p1 - p2) < 1e-12 * p1 and abs(d1 - d2) < 1e-12 * d1
        assert abs(a1 - b2) < 1e-12 and abs(a2 - b1) < 1e-12


def test_shrinker_identity_and_scale_equivariance():
    rng = np.random.default_rng(11)
    ch = np.exp(0.7 * rng.standard_normal(128))
    S, _, _ = _spiked(rng, 512, 128, (9.0, 6.0, 4.0, 3.0), channel=ch)
    es = oracle.eoptshrink(S)
    assert es.rank >= 3
    es2 = oracle.eoptshrink(3.5 * S)
    assert es2.rank == es.rank
    assert np.allclose(es2.phi, 3.5 * es.phi, rtol=1e-10)
    assert np.allclose(es2.a1, es.a1, rtol=1e-9) and np.allclose(es2.a2, es.a2, rtol=1e-9)
    # phi = d sqrt(a1 a2) must equal -T / (sigma T'), with T' taken by central differences of T here
    n, d = S.shape
    beta = d / n
    for i in range(es.rank):
        z = es.lam[i]

        def T(zz):
            ms = np.mean(1.0 / (es.atoms - zz))
            return zz * ms * (beta * ms - (1 - beta) / zz)
        h = 1e-5 * z
        dT = (T(z + h) - T(z - h)) / (2 * h)
        assert abs(-T(z) / (math.sqrt(z) * dT) - es.phi[i]) < 1e-6 * es.phi[i]
        assert abs(1.0 / math.sqrt(T(z)) - es.d_hat[i]) < 1e-12 * es.d_hat[i]


def test_shrinker_guard_on_degenerate_input():
    atoms = np.linspace(10.0, 1.0, 100)
    phi, dh, a1, a2, ok = oracle.shrink(5.05, atoms, 512, 128)     # "outlier" inside the bulk
    assert (phi == 0.0 and not ok) or (0.0 <= phi <= math.sqrt(5.05))
    with np.errstate(divide="ignore", invalid="ignore"):
        phi, dh, a1, a2, ok = oracle.shrink(5.0, np.r_[atoms, 5.0], 512, 128)   # exactly on an atom
    assert phi == 0.0 and not ok


# -------------------------------------------------- Prop. 6.1 and Cor. 6.3
def test_residual_has_no_outliers_and_noise_energy():
    n, d = 512, 128
    k = oracle.pilot_k(d)
    ratios = []
    for seed in range(10):
        rng = np.random.default_rng(40 + seed)
        S, sig, E = _spiked(rng, n, d, (12.0, 8.0, 6.0))
        es = oracle.eoptshrink(S)
        assert es.rank == 3
        R = S - (es.U * es.phi) @ es.V.T
        lamR = np.linalg.svd(R, compute_uv=False) ** 2
        # Prop. 6.1(1): the residual's spectrum is the noise bulk, nothing sticks out of it
        assert oracle.estimate_rank(lamR, d, k)[0] == 0
        assert math.sqrt(lamR[0]) < 1.1 * (math.sqrt(n) + math.sqrt(d))
        # the leftover of each shrunk component, sigma - phi, lies inside the bulk (proof of Prop. 6.1, Part 1)
        assert np.all(es.sigma - es.phi < math.sqrt(es.lam_plus))
        ratios.append(np.sum(R * R) / np.sum(E * E))
        # Cor. 6.3: no coordinate of a residual row carries disproportionate energy
        assert np.max(np.abs(R).max(1) / np.linalg.norm(R, axis=1)) < 3.0 * math.sqrt(math.log(d) / d)
        assert np.sum(R * R) < 0.5 * np.sum(S * S)
    # Prop. 6.1(2): ||R||_F^2 = ||Z||_F^2 up to O(d^{-1/2}) (~0.09 here); the three removed directions carry
    # about 3 (n + d) / (n d) = 2.9 % of the noise energy, which is the deficit seen
    assert abs(np.mean(ratios) - (1.0 - 3 * (n + d) / (n * d))) < 0.01
    # separable (per-channel) noise covariance: the energy statement still holds
    ratios = []
    for seed in range(10):
        rng = np.random.default_rng(80 + seed)
        ch = np.exp(0.3 * rng.standard_normal(d))
        S, sig, E = _spiked(rng, n, d, (12.0, 8.0, 6.0), channel=ch)
        es = oracle.eoptshrink(S)
        R = S - (es.U * es.phi) @ es.V.T
        ratios.append(np.sum(R * R) / np.sum(E * E))
    assert abs(np.mean(ratios) - 1.0) < 0.06


# ------------------------------------------------------------ Alg. 1, Alg. 3
@pytest.mark.parametrize("bits", [2, 3, 4])
def test_tq_mse_distortion_on_isotropic_rows(bits, golden):
    d = 128
    rng = np.random.default_rng(bits)
    X = rng.standard_normal((512, d))
    Pi = oracle.haar_rotation(d, 77)
    cb = oracle.lloyd_max_gaussian(bits)
    codes, rho, z = oracle.tq_mse_encode(X, Pi, cb)
    Xh = oracle.tq_mse_decode(codes, rho, Pi, cb)
    rel = np.linalg.norm(X - Xh) / np.linalg.norm(X)
    # (coordinates of a rotated unit vector have slightly lighter tails than N(0,1/d): up to ~2 % below sqrt(D_b))
    assert abs(rel / math.sqrt(cb.distortion) - 1.0) < 0.03
    assert abs(100 * rel - golden["table1_tqmse_l2"][bits - 2]) < 0.5
    assert np.allclose(np.linalg.norm(z, axis=1), 1.0, atol=1e-12)     # rotation keeps the unit norm
    # decoding with the transpose of the wrong orientation would not invert the rotation
    bad = rho[:, None] * ((cb.centroids[codes] / math.sqrt(d)) @ Pi.T)
    assert np.linalg.norm(X - bad) / np.linalg.norm(X) > 1.0


def test_bit_accounting(golden):
    assert abs(16 / 128 - golden["norm_overhead_d128"][0]) < 1e-12
    f = lambda r: r * (128 + 128) * 4 / (128 * 128)
    assert round(f(1), 2) == golden["factor_overhead_r1"][0]
    assert round(f(5.6), 2) == golden["factor_overhead_r5p6"][0]
    for b, printed in zip((2, 3, 4), golden["table1_bits_rank5p6"]):
        assert round(b + f(5.6), 2) == printed
    for b, printed in zip((2, 3, 4), golden["table2_bits_rank5p0"]):
        assert round(b + f(5.0), 2) == printed
    # the record this build stores keeps binary16 factors: b_s = 16
    assert abs(oracle.bits_per_entry(128, 128, 2, 1, b_s=4) - (2 + f(1) + 0.125 + 16 / 16384)) < 1e-12
    assert abs(oracle.bits_per_entry(512, 128, 2, 5) - (2 + 5 * 640 * 16 / 65536 + 0.125 + 80 / 65536)) < 1e-12


def test_pipeline_closed_loop_and_rank0_bypass():
    n, d = 512, 128
    Pi = oracle.haar_rotation(d, 260502906)
    cb = oracle.lloyd_max_gaussian(2)
    rng = np.random.default_rng(8)
    S, _, _ = _spiked(rng, n, d, (6.0, 4.0, 2.5))
    S = S.astype(np.float16).astype(np.float64)
    rec = oracle.compress_block(S, Pi, cb)
    X = oracle.decompress_block(rec, Pi, cb)
    assert rec.rank == 3 and rec.lfac.shape == (3, n) and rec.rfac.shape == (3, d)
    # stored factors are binary16 values
    assert np.array_equal(rec.lfac, rec.lfac.astype(np.float16).astype(np.float64))
    # closed loop: S - X_hat = R - R_hat, so the total error is the residual's quantisation error
    Rh = oracle.tq_mse_decode(rec.codes, rec.rho16, Pi, cb)
    assert np.allclose(S - X, rec.R - Rh, atol=1e-9)
    rel_res = np.linalg.norm(rec.R - Rh) / np.linalg.norm(rec.R)
    assert abs(rel_res / math.sqrt(cb.distortion) - 1.0) < 0.02
    assert np.linalg.norm(S - X) / np.linalg.norm(S) < 0.85 * math.sqrt(cb.distortion)   # better than TQ alone
    # Alg. 3 else-branch: pure noise goes to TQ_MSE unchanged
    N0 = np.random.default_rng(9).standard_normal((n, d))
    rec0 = oracle.compress_block(N0, Pi, cb)
    assert rec0.rank == 0 and rec0.lfac.shape[0] == 0 and np.array_equal(rec0.R, N0)
    c0, rho0, _ = oracle.tq_mse_encode(N0, Pi, cb)
    assert np.array_equal(rec0.codes, c0)
    assert np.allclose(rec0.rho16, rho0, rtol=1e-3)


def test_zero_row_and_norm_saturation():
    d = 128
    Pi = oracle.haar_rotation(d, 1)
    cb = oracle.lloyd_max_gaussian(2)
    X = np.zeros((3, d))
    X[1, 0] = 1e6
    X[2] = 1e-3
    codes, rho, _ = oracle.tq_mse_encode(X, Pi, cb)
    assert rho[0] == 0 and np.all(codes[0] == 2)        # 0 sits in the first non-negative cell
    assert oracle.fp16_round(rho)[1] == 65504.0
    assert oracle.fp16_bits(np.array([1.0]))[0] == 0x3C00


def test_scores_equal_fused_form():
    """Remark 6.5: <q, x_hat> = <q, s_hat> + <q, r_hat>, and <q, Pi^T z> = <Pi q, z>."""
    n, d = 512, 128
    Pi = oracle.haar_rotation(d, 260502906)
    cb = oracle.lloyd_max_gaussian(2)
    rng = np.random.default_rng(21)
    S, _, _ = _spiked(rng, n, d, (6.0, 4.0, 2.5))
    rec = oracle.compress_block(S, Pi, cb)
    q = rng.standard_normal((64, d))
    sc = oracle.score_block(q, rec, Pi, cb)
    qp = q @ Pi.T                                         # rows are Pi q
    zhat = cb.centroids_f32.astype(np.float64)[rec.codes] / math.sqrt(d)
    fused = (qp @ zhat.T) * rec.rho16[None, :] + (q @ rec.rfac.T) @ rec.lfac
    assert np.allclose(sc, fused / math.sqrt(d), atol=1e-10)
    exact = q @ S.T / math.sqrt(d)
    assert np.corrcoef(sc.ravel(), exact.ravel())[0, 1] > 0.9


# ------------------------------------------------------------------ encoding
@pytest.mark.parametrize("bits", [1, 2, 3, 4])
def test_pack_unpack_exhaustive(bits):
    d = 128
    L = 1 << bits
    # every code value at every coordinate, all other coordinates at a different value
    for other in (0, L - 1):
        codes = np.full((d * L, d), other, dtype=np.uint8)
        for j in range(d):
            for v in range(L):
                codes[j * L + v, j] = v
        pk = oracle.pack_codes(codes, bits)
        assert pk.shape == (d * L, bits * d // 8) and pk.dtype == np.uint8
        assert np.array_equal(oracle.unpack_codes(pk, bits, d), codes)
    # layout: coordinate j, bit p of its code -> plane p, byte j // 8, bit j % 8
    one = np.zeros((1, d), dtype=np.uint8)
    one[0, 77] = L - 1
    pk = oracle.pack_codes(one, bits).reshape(bits, d // 8)
    for p in range(bits):
        expect = np.zeros(d // 8, dtype=np.uint8)
        expect[77 // 8] = 1 << (77 % 8)
        assert np.array_equal(pk[p], expect)
    rng = np.random.default_rng(bits)
    codes = rng.integers(0, L, (64, d), dtype=np.uint8)
    assert np.array_equal(oracle.unpack_codes(oracle.pack_codes(codes, bits), bits, d), codes)


# ---------------------------------------------------------------------------------------------
# SVD factors at 4 bits (Alg. 3 line 3, Sec. 3.1): data-adaptive Lloyd-Max codebooks
# ---------------------------------------------------------------------------------------------
def test_adaptive_codebook_converges_to_the_gaussian_lloyd_max_levels():
    """On a large Gaussian sample Lloyd's iteration on |x| must reach the 16-level Lloyd-Max codebook of N(0,1)
    (whose values are pinned above to the printed table): a wrong update rule or boundary would settle elsewhere."""
    rng = np.random.default_rng(11)
    x = rng.standard_normal(400_000) * 3.0
    m = oracle.adaptive_magnitudes(x, iters=200, round16=False)
    ref = 3.0 * oracle.lloyd_max_gaussian(4).centroids[8:]
    assert np.max(np.abs(m - ref) / ref) < 0.02, (m, ref)
    # on data that is not Gaussian it leaves the Gaussian start for that data's own fixed point: every level
    # with a non-empty cell is the mean of its cell (levels above max|y| keep their start: their cells are empty)
    y = rng.uniform(-1.0, 1.0, 200_000)
    my = oracle.adaptive_magnitudes(y, iters=300, round16=False)
    cell = np.searchsorted(0.5 * (my[:-1] + my[1:]), np.abs(y), side="right")
    for k_ in range(8):
        if np.any(cell == k_):
            assert abs(my[k_] - np.abs(y)[cell == k_].mean()) < 1e-3
    assert np.count_nonzero(np.bincount(cell, minlength=8)) >= 6


def test_adaptive_codebook_lloyd_steps_never_increase_the_distortion():
    rng = np.random.default_rng(12)
    x = rng.standard_normal(5000) * 0.09
    prev = np.inf
    for it in range(0, 10):
        m = oracle.adaptive_magnitudes(x, iters=it, round16=False)
        xq = oracle.factor_decode(oracle.factor_encode(x, m), m)
        dist = float(np.mean((x - xq) ** 2))
        assert dist <= prev * (1 + 1e-12)
        prev = dist
    # after the fixed 8 iterations the distortion is close to the 4-bit optimum D_4 = 0.009497 sigma^2
    assert prev / np.var(x) < 1.03 * 0.009497
    # brute force: every entry is coded to the nearest of the 16 levels
    m = oracle.adaptive_magnitudes(x)
    levels = np.concatenate([-m[::-1], m])
    codes = oracle.factor_encode(x, m)
    xq = oracle.factor_decode(codes, m)
    nearest = levels[np.argmin(np.abs(x[:, None] - levels[None, :]), axis=1)]
    assert np.allclose(np.abs(x - xq), np.abs(x - nearest), rtol=0, atol=1e-15)


def test_factor_codes_do_not_depend_on_the_sign_of_a_singular_vector():
    rng = np.random.default_rng(13)
    U, _ = np.linalg.qr(rng.standard_normal((128, 3)))
    m1, m2 = oracle.adaptive_magnitudes(U), oracle.adaptive_magnitudes(U * np.array([1.0, -1.0, 1.0]))
    assert np.array_equal(m1, m2)
    c1, c2 = oracle.factor_encode(U, m1), oracle.factor_encode(U * np.array([1.0, -1.0, 1.0]), m1)
    assert np.array_equal(c1 & 7, c2 & 7) and np.array_equal(c1[:, 1] ^ c2[:, 1], np.full(128, 8))
    assert np.array_equal(oracle.unpack_nibbles(oracle.pack_nibbles(c1.T)), c1.T)


def test_factor_overhead_matches_the_printed_figure():
    """Sec. 3.3: r(n + d) b_s / (n d) with r = 5.6, n = d = 128, b_s = 4 is 'approximately 0.35 bits'; with r = 1
    'approximately 0.06'."""
    assert abs(5.6 * 256 * 4 / 16384 - 0.35) < 1e-12
    assert abs(oracle.bits_per_entry(128, 128, 2, 1, b_s=4) - (2 + 0.0625 + 0.125 + 16.0 / 16384)) < 1e-12


def test_four_bit_factors_closed_loop_and_expansion():
    """The residual is taken against the stored 4-bit factors (closed loop): decompress reproduces S up to the
    TQ error of the residual, the record's binary16 factors are exactly what the codes expand to, and the
    low-rank part keeps ~99 % of what binary16 factors keep (4-bit distortion 0.95 % per factor)."""
    S, _, _ = _spiked(np.random.default_rng(21), 512, 128, (6.0, 4.0, 2.5))
    Pi = oracle.haar_rotation(128, 7)
    cb = oracle.lloyd_max_gaussian(2)
    r16 = oracle.compress_block(S, Pi, cb)
    r4 = oracle.compress_block(S, Pi, cb, factor_bits=4)
    assert r4.rank == r16.rank == 3 and r4.factor_bits == 4
    lf = oracle.fp16_round(oracle.factor_decode(r4.lcodes, r4.fbook[0]) * r4.phi16[:, None])
    assert np.array_equal(lf, r4.lfac) and np.array_equal(oracle.factor_decode(r4.rcodes, r4.fbook[1]), r4.rfac)
    x4 = oracle.decompress_block(r4, Pi, cb)
    e4 = np.linalg.norm(S - x4) / np.linalg.norm(r4.R)
    assert abs(e4 - math.sqrt(0.117482)) < 0.02          # TQ error of the residual, 2 bits
    low16, low4 = r16.lfac.T @ r16.rfac, r4.lfac.T @ r4.rfac
    assert np.linalg.norm(low16 - low4) / np.linalg.norm(low16) < 0.2
    # 4-bit factors leave sqrt(2 D_4) = 14 % of the low-rank part in the residual: here 1 % more residual energy
    assert np.linalg.norm(r4.R) < 1.02 * np.linalg.norm(r16.R)


def test_score_stream_is_the_logit_of_the_concatenated_cache():
    """A cache of two compressed blocks and an uncompressed tail: the streamed logits are the logits of the
    reconstructed cache [x_hat_0; x_hat_1; tail] (Sec. 2.1), and with an empty tail those of the blocks alone."""
    rng = np.random.default_rng(11)
    Pi = oracle.haar_rotation(128, 5)
    cb = oracle.lloyd_max_gaussian(2)
    blocks = [rng.standard_normal((128, 128)) + 3.0 * np.outer(rng.standard_normal(128), rng.standard_normal(128)) / 11.0
              for _ in range(2)]
    recs = [oracle.compress_block(S, Pi, cb) for S in blocks]
    tail = rng.standard_normal((37, 128))
    q = rng.standard_normal((4, 128))
    cache = np.concatenate([oracle.decompress_block(r, Pi, cb) for r in recs] + [tail])
    want = q @ cache.T / math.sqrt(128.0)
    got = oracle.score_stream(q, recs, tail, Pi, cb)
    assert got.shape == (4, 2 * 128 + 37) and np.allclose(got, want, rtol=0, atol=1e-12)
    assert np.array_equal(oracle.score_stream(q, recs, tail[:0], Pi, cb), got[:, :256])
    # the tail part alone is the exact logit of the uncompressed keys
    assert np.allclose(oracle.score_stream(q, [], tail, Pi, cb), q @ tail.T / math.sqrt(128.0), rtol=0, atol=1e-13)


def test_softmax_rows_against_scipy_and_its_invariants():
    from scipy import special
    rng = np.random.default_rng(2)
    s = rng.standard_normal((5, 300)) * 6.0
    p = oracle.softmax_rows(s)
    assert np.allclose(p, special.softmax(s, axis=-1), rtol=1e-13, atol=0)
    assert np.allclose(p.sum(-1), 1.0, rtol=0, atol=1e-14) and np.all(p > 0)
    assert np.allclose(oracle.softmax_rows(s + 1000.0), p, rtol=1e-12, atol=0)         # shift invariance, no overflow
    assert np.allclose(np.log(p[:, 1:] / p[:, :1]), s[:, 1:] - s[:, :1], rtol=0, atol=1e-10)


def test_attend_blocks_is_the_weighted_sum_of_the_reconstructed_values():
    """One-hot weights pick single reconstructed rows; general weights agree with the split the fused kernel
    uses (rotated-codebook term through one inverse rotation of the summed codes plus the low-rank term), written
    out here independently of decompress_block."""
    rng = np.random.default_rng(4)
    Pi = oracle.haar_rotation(128, 9)
    cb = oracle.lloyd_max_gaussian(2)
    blocks = [rng.standard_normal((128, 128)) + np.outer(rng.standard_normal(128), rng.standard_normal(128)) * 0.4
              for _ in range(3)]
    recs = [oracle.compress_block(S, Pi, cb) for S in blocks]
    assert all(r.rank >= 1 for r in recs)
    x = np.concatenate([oracle.decompress_block(r, Pi, cb) for r in recs])
    onehot = np.zeros((2, 384))
    onehot[0, 5] = 1.0
    onehot[1, 300] = 1.0
    got = oracle.attend_blocks(onehot, recs, Pi, cb)
    assert np.array_equal(got[0], x[5]) and np.array_equal(got[1], x[300])
    w = oracle.softmax_rows(rng.standard_normal((4, 384)) * 3.0)
    got = oracle.attend_blocks(w, recs, Pi, cb)
    acc_rot = np.zeros((4, 128))
    acc_lin = np.zeros((4, 128))
    for j, r in enumerate(recs):
        wj = w[:, 128 * j:128 * (j + 1)]
        zhat = cb.centroids_f32.astype(np.float64)[r.codes] / math.sqrt(128.0)   # the stored table, rotated domain
        acc_rot += (wj * r.rho16[None, :]) @ zhat
        acc_lin += (wj @ r.lfac.T) @ r.rfac
    want = acc_rot @ Pi + acc_lin                                           # x_hat = rho Pi^T z_hat + C V
    assert np.allclose(got, want, rtol=0, atol=1e-12 * np.max(np.abs(want)) + 1e-13)
    assert np.allclose(got, w @ x, rtol=0, atol=1e-13)
    with pytest.raises(ValueError):
        oracle.attend_blocks(w[:, :-1], recs, Pi, cb)


# ---- TQ_prod / QJL (Alg. 1 lines "TQ_prod", Eq. (qjl)) ------------------------------------------------------------
def test_qjl_identity_behind_the_estimator():
    """For g ~ N(0, I): E[sign(<g, a>) <g, y>] = sqrt(2/pi) <a, y> / |a|, which is why Eq. (qjl) scales by
    sqrt(pi/2)/d.  Checked by the closed form in 2 dimensions (numerical integration over the angle) and by brute
    force over many rows of Phi."""
    a = np.array([0.3, -1.1])
    y = np.array([0.7, 0.2])
    # in polar form g = rho (cos t, sin t): E = E[rho] * mean over t of sign(cos(t - ta)) (y . unit(t)), E[rho] = sqrt(pi/2)
    f = lambda t: np.sign(a[0] * np.cos(t) + a[1] * np.sin(t)) * (y[0] * np.cos(t) + y[1] * np.sin(t)) / (2 * np.pi)
    val, _ = integrate.quad(f, 0.0, 2 * np.pi, points=[np.arctan2(a[1], a[0]) + np.pi / 2, np.arctan2(a[1], a[0]) + 1.5 * np.pi],
                            limit=200)
    assert abs(math.sqrt(math.pi / 2) * val - math.sqrt(2 / math.pi) * (a @ y) / np.linalg.norm(a)) < 1e-9
    rng = np.random.default_rng(0)
    d = 16
    a, y = rng.standard_normal(d), rng.standard_normal(d)
    g = rng.standard_normal((400000, d))
    mc = np.mean(np.sign(g @ a) * (g @ y))
    assert abs(mc - math.sqrt(2 / math.pi) * (a @ y) / np.linalg.norm(a)) < 4 * np.linalg.norm(y) / math.sqrt(400000)


def test_qjl_estimator_is_unbiased_over_the_projection():
    """Eq. (qjl): averaged over independent Phi the corrected inner product equals <y, x>; the MSE reconstruction
    alone is biased low in magnitude along x (the quantiser shrinks)."""
    Pi = oracle.haar_rotation(128, 3)
    cb = oracle.lloyd_max_gaussian(2)
    rng = np.random.default_rng(1)
    S = rng.standard_normal((128, 128))
    rec = oracle.compress_block(S, Pi, cb, force_rank0=True)
    q = S[:4] / np.linalg.norm(S[:4], axis=1, keepdims=True) + 0.3 * rng.standard_normal((4, 128)) / math.sqrt(128)
    exact = q @ S.T
    mse = oracle.score_block(q, rec, Pi, cb) * math.sqrt(128.0)
    acc = np.zeros_like(exact)
    reps = 300
    for s in range(reps):
        Phi = oracle.gaussian_projection(128, 1000 + s)
        acc += oracle.qjl_correction(q, oracle.qjl_encode(S, rec, Pi, cb, Phi), Phi)
    est = mse + acc / reps
    rx = S - oracle.decompress_block(rec, Pi, cb)
    # standard error of the mean of one correction: |r_x| sqrt(pi/2)/d * sqrt(d) |q| at most
    se = np.linalg.norm(rx, axis=1)[None, :] * math.sqrt(math.pi / 2 / 128) * np.linalg.norm(q, axis=1)[:, None] / math.sqrt(reps)
    assert np.all(np.abs(est - exact) < 5 * se + 2e-3 * np.abs(exact))
    diag = np.arange(4)
    assert np.all(np.abs(mse[diag, diag]) < np.abs(exact[diag, diag]))                 # shrinkage bias of TQ_MSE
    assert np.mean(np.abs(est[diag, diag] - exact[diag, diag])) < 0.3 * np.mean(np.abs(mse[diag, diag] - exact[diag, diag]))


def test_qjl_record_definition_and_packing():
    Pi = oracle.haar_rotation(128, 3)
    cb = oracle.lloyd_max_gaussian(3)
    Phi = oracle.gaussian_projection(128, 4)
    assert Phi.shape == (128, 128) and abs(Phi.mean()) < 0.03 and abs(Phi.std() - 1.0) < 0.02
    assert np.array_equal(Phi.ravel()[:5], oracle.gaussian_stream(4, 5))
    rng = np.random.default_rng(6)
    S = rng.standard_normal((128, 128)) + 2.0 * np.outer(rng.standard_normal(128), rng.standard_normal(128)) / 11.3
    rec = oracle.compress_block(S, Pi, cb)
    assert rec.rank >= 1
    qj = oracle.qjl_encode(S, rec, Pi, cb, Phi)
    rx = S - oracle.decompress_block(rec, Pi, cb)
    t = 17
    assert np.array_equal(qj.signs[t], (Phi @ rx[t] >= 0).astype(np.uint8))            # one row, written out
    assert qj.gamma16[t] == float(np.float16(np.linalg.norm(rx[t])))
    # the residual of the stored record is the quantisation residual of the residual row (Alg. 3 + Alg. 1)
    R = S - rec.lfac.T @ rec.rfac
    Rhat = oracle.tq_mse_decode(rec.codes, rec.rho16, Pi, cb)
    assert np.allclose(rx, R - Rhat, rtol=0, atol=1e-12)
    packed = oracle.pack_signs(qj.signs)
    assert packed.shape == (128, 16) and np.array_equal(oracle.unpack_signs(packed, 128), qj.signs)
    assert packed[t, 0] == sum(int(qj.signs[t, j]) << j for j in range(8))
    # bits per entry of TQ_prod: b + 1 + 16/d (Alg. 1 last line), one more bit-plane than TQ_MSE
    assert oracle.bits_per_entry(128, 128, 3, 0) + 1.0 == 3 + 1 + 16 / 128
    # zero residual row: sign(0) = +1, norm 0, no correction
    q = rng.standard_normal((2, 128))
    z = oracle.QjlRecord(np.ones((1, 128), np.uint8), np.zeros(1))
    assert not np.any(oracle.qjl_correction(q, z, Phi))


def test_attend_stream_is_attention_over_the_concatenated_values():
    rng = np.random.default_rng(8)
    Pi = oracle.haar_rotation(128, 9)
    cb = oracle.lloyd_max_gaussian(2)
    recs = [oracle.compress_block(rng.standard_normal((128, 128)), Pi, cb) for _ in range(2)]
    tail = rng.standard_normal((19, 128))
    w = oracle.softmax_rows(rng.standard_normal((3, 256 + 19)))
    vals = np.concatenate([oracle.decompress_block(r, Pi, cb) for r in recs] + [tail])
    assert np.allclose(oracle.attend_stream(w, recs, tail, Pi, cb), w @ vals, rtol=0, atol=1e-13)
    assert np.allclose(oracle.attend_stream(w[:, 256:], [], tail, Pi, cb), w[:, 256:] @ tail, rtol=0, atol=1e-14)
    with pytest.raises(ValueError):
        oracle.attend_stream(w[:, :-1], recs, tail, Pi, cb)
