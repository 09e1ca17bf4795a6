"""Plain float64 reference of the eOptShrinkQ hot path (NumPy, one block at a time).

TEST INFRASTRUCTURE ONLY -- slow on purpose, written to be checked against the
paper by eye.  It shares no code with the HIP library and the product path never
imports it.

Every function cites the passage of the paper (arXiv 2605.02905) it follows.
Where the paper is silent the reading taken is stated next to the code; the full
list of readings lives in the design notes of the repository.

Parity pins (tests/test_oracle_pins.py): pilot k (Remark 3.1), Gaussian Lloyd-Max
centroids, Haar-rotation orthogonality and sign convention, brute-force SVD on
tiny blocks, Marchenko-Pastur bulk edge, planted-rank recovery, the exact
square-root-edge law behind the bulk-edge and imputation rules of Alg. 2 Steps
1-2, the white-noise closed forms of the Frobenius, operator-norm and
nuclear-norm shrinkers with measured overlaps, Prop. 6.1 / Cor. 6.3 residual
properties, the sqrt(D_b) distortion the paper's Tables 1-4 print for TQ_MSE,
bit accounting of Alg. 3 and Sec. 4.1, and the score identity of Remark 6.5.
The 1/M normalisation of the imputed noise measure (Eq. (Fe) prints 1/(n ^ d)
over atoms of which r have been discarded) is pinned by unbiasedness: over 96
white-noise blocks d_hat recovers the planted strengths to a quarter of a percent
with 1/M and comes out 1.5 % high with 1/(n ^ d).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

__all__ = [
    "pilot_k", "rank_threshold", "EDGE_COEF",
    "lloyd_max_gaussian", "Codebook",
    "splitmix64", "gaussian_stream", "haar_rotation",
    "bulk_edge", "estimate_rank", "impute_noise_spectrum", "shrink", "LOSSES",
    "EOptShrinkResult", "eoptshrink",
    "tq_mse_encode", "tq_mse_decode",
    "BlockRecord", "compress_block", "decompress_block", "score_block", "score_stream", "softmax_rows", "attend_blocks", "attend_stream",
    "gaussian_projection", "QjlRecord", "qjl_encode", "qjl_correction", "score_block_prod", "pack_signs", "unpack_signs",
    "pack_codes", "unpack_codes", "fp16_round", "fp16_bits", "bits_per_entry",
    "FLAG_RANK_CLAMPED", "FLAG_SHRINK_GUARD",
    "FACTOR_LEVELS", "FACTOR_LLOYD_ITERS", "adaptive_magnitudes", "factor_encode", "factor_decode",
    "pack_nibbles", "unpack_nibbles", "quantize_factors",
]

FLAG_RANK_CLAMPED = 1
FLAG_SHRINK_GUARD = 2

# 1 / (2^{2/3} - 1): the constant of the square-root-edge extrapolation in
# Alg. 2, Steps 1 and 2.
EDGE_COEF = 1.0 / (2.0 ** (2.0 / 3.0) - 1.0)


# --------------------------------------------------------------------------
# constants of Alg. 2
# --------------------------------------------------------------------------
def pilot_k(d: int) -> int:
    """k = floor(d^c), c = min(1/2.01, 1/log log d), natural logarithms.

    Alg. 2 REQUIRE and Step 1; Remark 3.1 prints k = 11 for d = 128 and the
    remark after Prop. 6.1's proof gives k ~ 7 for d = 64.
    """
    c = min(1.0 / 2.01, 1.0 / math.log(math.log(d)))
    return int(math.floor(d ** c))


def rank_threshold(d: int) -> float:
    """d^{-1/3}, the relative margin above the bulk edge in Alg. 2 Step 1."""
    return float(d) ** (-1.0 / 3.0)


# --------------------------------------------------------------------------
# Lloyd-Max codebook for a Gaussian marginal (Sec. 2.2 item 3, Alg. 1 REQUIRE)
# --------------------------------------------------------------------------
@dataclass
class Codebook:
    bits: int
    centroids: np.ndarray      # float64, ascending, for N(0,1)
    bounds: np.ndarray         # float64, ascending midpoints, 2^b - 1 of them
    centroids_f32: np.ndarray  # the stored table
    bounds_f32: np.ndarray
    distortion: float          # E (x - Q(x))^2 for x ~ N(0,1)


def _phi(x):
    return math.exp(-0.5 * x * x) / math.sqrt(2.0 * math.pi)


def _Phi(x):
    return 0.5 * math.erfc(-x / math.sqrt(2.0))


def lloyd_max_gaussian(bits: int, tol: float = 1e-15, max_iter: int = 200000) -> Codebook:
    """MSE-optimal 2^b-level scalar quantizer of N(0,1) by the Lloyd iteration.

    Sec. 2.2 item 3: the codebook is optimised for the N(0,1/d) marginal of a
    rotated unit vector; that codebook is this one scaled by 1/sqrt(d).
    Fixed point: boundaries are midpoints of neighbouring centroids, centroids
    are conditional means  (phi(a) - phi(b)) / (Phi(b) - Phi(a))  of their cell.
    """
    L = 1 << bits
    # start from equiprobable-cell means (any sorted start converges: the
    # Gaussian density is log-concave, so the fixed point is unique)
    c = np.array([(i + 0.5) / L * 6.0 - 3.0 for i in range(L)], dtype=np.float64)
    for _ in range(max_iter):
        b = 0.5 * (c[:-1] + c[1:])
        edges = [-math.inf] + list(b) + [math.inf]
        new = np.empty(L)
        for i in range(L):
            lo, hi = edges[i], edges[i + 1]
            plo = 0.0 if lo == -math.inf else _phi(lo)
            phi_ = 0.0 if hi == math.inf else _phi(hi)
            if i >= L // 2:
                # upper tail: use complementary CDFs so the mass keeps its
                # relative accuracy
                mass = 0.5 * (math.erfc(lo / math.sqrt(2.0)) - (0.0 if hi == math.inf else math.erfc(hi / math.sqrt(2.0))))
            else:
                mass = (1.0 if hi == math.inf else _Phi(hi)) - (0.0 if lo == -math.inf else _Phi(lo))
            new[i] = (plo - phi_) / mass
        # the optimum is symmetric; enforce it so both halves carry the same bits
        new = 0.5 * (new - new[::-1])
        delta = float(np.max(np.abs(new - c)))
        c = new
        if delta < tol:
            break
    b = 0.5 * (c[:-1] + c[1:])
    # distortion  E x^2 - sum_i mass_i c_i^2  (centroid condition)
    edges = [-math.inf] + list(b) + [math.inf]
    ec2 = 0.0
    for i in range(L):
        lo, hi = edges[i], edges[i + 1]
        mass = (1.0 if hi == math.inf else _Phi(hi)) - (0.0 if lo == -math.inf else _Phi(lo))
        ec2 += mass * c[i] * c[i]
    return Codebook(bits, c, b, c.astype(np.float32), b.astype(np.float32), 1.0 - ec2)


# --------------------------------------------------------------------------
# seeded Haar rotation (Sec. 2.2 item 2; Alg. 1 REQUIRE "shared Haar rotation")
# --------------------------------------------------------------------------
_M64 = (1 << 64) - 1


def splitmix64(seed: int, counter: np.ndarray) -> np.ndarray:
    """SplitMix64 output for state seed + (counter+1)*golden, vectorised.

    Counter-based: value number `counter` of the stream `seed` (public-domain
    generator of Steele, Lea & Flood / Vigna).
    """
    with np.errstate(over="ignore"):
        z = (np.uint64(seed & _M64) + (counter.astype(np.uint64) + np.uint64(1)) * np.uint64(0x9E3779B97F4A7C15))
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    return z


def gaussian_stream(seed: int, count: int) -> np.ndarray:
    """`count` iid N(0,1) draws: Box-Muller cosine branch on counters (2e, 2e+1)."""
    e = np.arange(count, dtype=np.uint64)
    a = splitmix64(seed, 2 * e)
    b = splitmix64(seed, 2 * e + 1)
    u1 = ((a >> np.uint64(11)).astype(np.float64) + 0.5) * (2.0 ** -53)
    u2 = ((b >> np.uint64(11)).astype(np.float64) + 0.5) * (2.0 ** -53)
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * math.pi * u2)


def haar_rotation(d: int, seed: int) -> np.ndarray:
    """Haar-distributed orthogonal Pi (float64): QR of a d x d Gaussian matrix
    filled row-major from `gaussian_stream`, columns of Q re-signed so that R
    has a positive diagonal (this makes the law of Q exactly Haar).
    """
    g = gaussian_stream(seed, d * d).reshape(d, d)
    q, r = np.linalg.qr(g)
    s = np.sign(np.diag(r))
    s[s == 0] = 1.0
    return q * s[None, :]


# --------------------------------------------------------------------------
# Alg. 2 (eOptShrink)
# --------------------------------------------------------------------------
def bulk_edge(lam: np.ndarray, k: int) -> float:
    """Alg. 2 Step 1: lambda_+ = lam_{k+1} + (lam_{k+1} - lam_{2k+1}) / (2^{2/3} - 1).

    `lam` holds the eigenvalues sigma_i^2 in descending order; the paper's
    subscripts are 1-based.  (Alg. 2 prints a square on the eigenvalue symbol;
    Sec. 2.3 defines lambda_i := sigma_i^2 and Sec. 4.1 counts singular values
    above sqrt(lambda_+), so the quantity is the eigenvalue itself.)
    """
    a = lam[k]          # lam_{k+1}
    b = lam[2 * k]      # lam_{2k+1}
    return a + EDGE_COEF * (a - b)


def estimate_rank(lam: np.ndarray, d: int, k: int) -> tuple[int, float]:
    """Alg. 2 Step 1: r^+ = #{ i : lam_i / lambda_+ - 1 > d^{-1/3} } (strict)."""
    lp = bulk_edge(lam, k)
    thr = rank_threshold(d)
    r = int(np.count_nonzero(lam / lp - 1.0 > thr))
    return r, lp


def impute_noise_spectrum(lam: np.ndarray, r: int, k: int) -> np.ndarray:
    """Alg. 2 Step 2 and Eq. (Fe): the estimated noise eigenvalues.

    The r outliers are dropped; the next k values are replaced by
        lam_{k+r+1} + (1 - (j/k)^{2/3}) / (2^{2/3}-1) * (lam_{k+r+1} - lam_{2k+r+1}),
    j = 1..k; the rest are the observed eigenvalues.  Returns the N - r atoms
    in descending order.
    """
    N = lam.shape[0]
    a = lam[k + r]        # lam_{k+r+1}
    b = lam[2 * k + r]    # lam_{2k+r+1}
    atoms = np.empty(N - r)
    for j in range(1, k + 1):
        atoms[j - 1] = a + (1.0 - (j / k) ** (2.0 / 3.0)) * EDGE_COEF * (a - b)
    atoms[k:] = lam[r + k:]
    return atoms


LOSSES = ("frobenius", "operator", "nuclear")


def shrink(lam_i: float, atoms: np.ndarray, n: int, d: int, loss: str = "frobenius"):
    """Alg. 2 Step 3 for one outlier eigenvalue z = lam_i (Eqs. d_transform,
    d_a_estimates, shrinkers).

    m_s, m_s' : Stieltjes transform (and derivative) of the empirical measure of
    the M = len(atoms) noise atoms, i.e. of the min(n,d)-sided Gram matrix.
    m_l       : the transform of the max(n,d)-sided Gram matrix, which has the
    same non-zero spectrum plus |n-d| zeros:  m_l = beta m_s - (1-beta)/z.
    m_1 is the transform on the n x n side (Z Z^T, left vectors), m_2 on the
    d x d side (Z^T Z, right vectors): (m_1, m_2) = (m_l, m_s) when n >= d.
    T = z m_1 m_2;  d = T^{-1/2};  a_1 = m_1/(d^2 T'),  a_2 = m_2/(d^2 T');
    the shrunk value is the case of Eq. (shrinkers) that `loss` names:
      frobenius  d sqrt(a_1 a_2)
      operator   d sqrt(min(a_1, a_2) / max(a_1, a_2))
      nuclear    d (sqrt(a_1 a_2) - sqrt((1 - a_1)(1 - a_2)))
    (all experiments of the paper use the Frobenius case, Remark 3.1).

    Readings (the paper defers the estimators to its reference): the measure is
    normalised by the number of atoms M; beta = min(n,d)/max(n,d); an overlap
    estimate outside [0, 1] is clipped into it before the operator and nuclear
    formulas take roots of a_x and 1 - a_x; the result is clipped to [0, sigma]
    (the nuclear expression is negative for weak components: those get 0).
    Returns (phi, d_hat, a_1, a_2, ok).
    """
    if loss not in LOSSES:
        raise ValueError("loss must be one of " + ", ".join(LOSSES))
    z = float(lam_i)
    beta = min(n, d) / max(n, d)
    diff = atoms - z
    m_s = float(np.mean(1.0 / diff))
    dm_s = float(np.mean(1.0 / (diff * diff)))
    m_l = beta * m_s - (1.0 - beta) / z
    dm_l = beta * dm_s + (1.0 - beta) / (z * z)
    if n >= d:
        m_1, dm_1, m_2, dm_2 = m_l, dm_l, m_s, dm_s
    else:
        m_1, dm_1, m_2, dm_2 = m_s, dm_s, m_l, dm_l
    T = z * m_1 * m_2
    dT = m_1 * m_2 + z * dm_1 * m_2 + z * m_1 * dm_2
    sigma = math.sqrt(z)
    ok = math.isfinite(T) and math.isfinite(dT) and T > 0.0 and dT < 0.0
    if not ok:
        return 0.0, 0.0, 0.0, 0.0, False
    d_hat = 1.0 / math.sqrt(T)
    a1 = m_1 / (d_hat * d_hat * dT)
    a2 = m_2 / (d_hat * d_hat * dT)
    if loss == "frobenius":
        phi = d_hat * math.sqrt(a1 * a2)
    else:
        if not (math.isfinite(a1) and math.isfinite(a2)):
            return 0.0, 0.0, 0.0, 0.0, False
        c1, c2 = min(max(a1, 0.0), 1.0), min(max(a2, 0.0), 1.0)
        if loss == "operator":
            hi = max(c1, c2)
            phi = d_hat * math.sqrt(min(c1, c2) / hi) if hi > 0.0 else 0.0
        else:
            phi = d_hat * (math.sqrt(c1 * c2) - math.sqrt((1.0 - c1) * (1.0 - c2)))
    if not math.isfinite(phi):
        return 0.0, 0.0, 0.0, 0.0, False
    phi = min(max(phi, 0.0), sigma)
    return phi, d_hat, a1, a2, True


@dataclass
class EOptShrinkResult:
    lam: np.ndarray            # all min(n,d) eigenvalues sigma^2, descending
    k: int
    lam_plus: float
    rank: int                  # r^+ after clamping to r_max
    rank_unclamped: int
    atoms: np.ndarray          # estimated noise eigenvalues
    sigma: np.ndarray          # observed singular values of the outliers [rank]
    phi: np.ndarray            # shrunk singular values [rank]
    d_hat: np.ndarray
    a1: np.ndarray
    a2: np.ndarray
    U: np.ndarray              # [n, rank] left singular vectors
    V: np.ndarray              # [d, rank] right singular vectors
    flags: int


def eoptshrink(S: np.ndarray, r_max: int = 32, loss: str = "frobenius") -> EOptShrinkResult:
    """Alg. 2 on one block S (n x d) from the direct SVD; `loss` picks the case of
    Eq. (shrinkers) (Alg. 2 REQUIRE "loss function L")."""
    S = np.asarray(S, dtype=np.float64)
    n, d = S.shape
    U, s, Vt = np.linalg.svd(S, full_matrices=False)
    lam = s * s                                   # Sec. 2.3: lambda_i = sigma_i^2
    k = pilot_k(d)
    N = lam.shape[0]
    if 2 * k + 1 > N:
        raise ValueError("block too small for the pilot parameter: 2k+1 > min(n,d)")
    r_raw, lp = estimate_rank(lam, d, k)
    flags = 0
    r = r_raw
    # Step 2 reads lam_{2k+r+1}: the retained rank is cut so that this index exists
    # (the paper assumes k >> r^+ and is silent about larger ranks)
    r_cap = min(r_max, N - 2 * k - 1)
    if r > r_cap:
        r = r_cap
        flags |= FLAG_RANK_CLAMPED
    atoms = impute_noise_spectrum(lam, r, k)
    phi = np.zeros(r)
    dh = np.zeros(r)
    a1 = np.zeros(r)
    a2 = np.zeros(r)
    for i in range(r):
        phi[i], dh[i], a1[i], a2[i], ok = shrink(lam[i], atoms, n, d, loss)
        if not ok:
            flags |= FLAG_SHRINK_GUARD
    return EOptShrinkResult(lam, k, lp, r, r_raw, atoms, s[:r].copy(), phi, dh, a1, a2,
                            U[:, :r].copy(), Vt[:r].T.copy(), flags)


# --------------------------------------------------------------------------
# Alg. 1 (TQ_MSE)
# --------------------------------------------------------------------------
def fp16_round(x: np.ndarray) -> np.ndarray:
    """Round to nearest-even binary16, saturating at +-65504; returned as float64."""
    x = np.clip(np.asarray(x, dtype=np.float64), -65504.0, 65504.0)
    return x.astype(np.float16).astype(np.float64)


def fp16_bits(x: np.ndarray) -> np.ndarray:
    x = np.clip(np.asarray(x, dtype=np.float64), -65504.0, 65504.0)
    return x.astype(np.float16).view(np.uint16)


def tq_mse_encode(R: np.ndarray, Pi: np.ndarray, cb: Codebook):
    """Alg. 1 lines 3-5 for every row of R.

    rho = ||x||, u = x/rho, z = Pi u, code_j = index of the nearest centroid of
    the N(0,1/d) codebook = number of N(0,1) boundaries <= z_j sqrt(d).
    The comparison is taken in binary32 (the precision of the stored boundary
    table): value and boundaries are both rounded to float32 first.
    A zero row gets u = 0.  Returns (codes uint8 [n,d], rho float64 [n], z [n,d]).
    """
    R = np.asarray(R, dtype=np.float64)
    n, d = R.shape
    rho = np.sqrt(np.sum(R * R, axis=1))
    safe = np.where(rho > 0.0, rho, 1.0)
    u = R / safe[:, None]
    z = u @ Pi.T                                   # row form of z = Pi u
    t = (z * math.sqrt(d)).astype(np.float32)
    codes = np.zeros((n, d), dtype=np.uint8)
    for bm in cb.bounds_f32:
        codes += (bm <= t).astype(np.uint8)
    return codes, rho, z


def tq_mse_decode(codes: np.ndarray, rho16: np.ndarray, Pi: np.ndarray, cb: Codebook) -> np.ndarray:
    """Alg. 1 line 6: x_hat = rho * Pi^T z_hat, z_hat = centroid[code]/sqrt(d)
    (stored float32 table), rho the stored binary16 norm."""
    d = codes.shape[1]
    zhat = cb.centroids_f32.astype(np.float64)[codes] / math.sqrt(d)
    return rho16[:, None] * (zhat @ Pi)            # row form of Pi^T z_hat


# --------------------------------------------------------------------------
# Alg. 3 (eOptShrinkQ) on one block, decompression and scoring
# --------------------------------------------------------------------------
@dataclass
class BlockRecord:
    """What Alg. 3 line "Store" keeps for one block (factors in binary16)."""
    n: int
    d: int
    bits: int
    rank: int
    flags: int
    phi: np.ndarray      # [rank] float64 shrunk singular values
    sigma: np.ndarray    # [rank] observed singular values
    lfac: np.ndarray     # [rank, n] binary16 values (as float64) of U diag(phi)
    rfac: np.ndarray     # [rank, d] binary16 values (as float64) of V
    codes: np.ndarray    # [n, d] uint8
    rho16: np.ndarray    # [n] stored norms (binary16 values as float64)
    # diagnostics
    lam: np.ndarray = field(default=None, repr=False)
    lam_plus: float = 0.0
    rho: np.ndarray = field(default=None, repr=False)
    z: np.ndarray = field(default=None, repr=False)
    R: np.ndarray = field(default=None, repr=False)
    # SVD factors stored at 4 bits (Alg. 3 line 3, Sec. 3.1); None when the factors are kept in binary16
    factor_bits: int = 16
    lcodes: np.ndarray = field(default=None, repr=False)   # [rank, n] uint8, 4-bit codes of U
    rcodes: np.ndarray = field(default=None, repr=False)   # [rank, d] uint8, 4-bit codes of V
    fbook: np.ndarray = field(default=None, repr=False)    # [2, 8] binary16 magnitudes (as float64): U's, V's
    phi16: np.ndarray = field(default=None, repr=False)    # [rank] binary16 shrunk singular values


# --------------------------------------------------------------------------
# SVD factors at b_s = 4 bits (Alg. 3 line 3; Sec. 3.1 "data-adaptive Lloyd-Max codebooks")
# --------------------------------------------------------------------------
FACTOR_LEVELS = 8        # magnitudes; with the sign bit 16 levels = 4 bits
FACTOR_LLOYD_ITERS = 8


def adaptive_magnitudes(x: np.ndarray, levels: int = FACTOR_LEVELS, iters: int = FACTOR_LLOYD_ITERS,
                        round16: bool = True) -> np.ndarray:
    """Lloyd's algorithm on the magnitudes |x| of the entries of one factor matrix.
    Start: the Lloyd-Max levels of a Gaussian with the entries' root mean square
    (entries of singular vectors are close to Gaussian, so this start is already
    near the fixed point); then `iters` times assign every |x| to the nearest level
    (midpoint boundaries, a tie goes to the upper cell) and move every level to the
    mean of its cell (an empty cell keeps its level).  The codebook is {+-m_k}:
    symmetric, so it does not depend on the arbitrary sign of a singular vector.
    Returned ascending, in binary16."""
    a = np.abs(np.asarray(x, dtype=np.float64)).ravel()
    rms = math.sqrt(float(np.mean(a * a))) if a.size else 0.0
    nbits = int(round(math.log2(2 * levels)))
    m = lloyd_max_gaussian(nbits).centroids[levels:] * rms
    for _ in range(iters):
        cell = np.searchsorted(0.5 * (m[:-1] + m[1:]), a, side="right")
        for k in range(levels):
            sel = cell == k
            if sel.any():
                m[k] = a[sel].mean()
    return fp16_round(m) if round16 else m


def factor_encode(x: np.ndarray, mags: np.ndarray) -> np.ndarray:
    """4-bit code of every entry: bits 0-2 = index of the nearest magnitude (tie ->
    upper cell), bit 3 = 1 for x >= 0."""
    x = np.asarray(x, dtype=np.float64)
    cell = np.searchsorted(0.5 * (mags[:-1] + mags[1:]), np.abs(x), side="right").astype(np.uint8)
    return (cell | ((x >= 0).astype(np.uint8) << 3)).astype(np.uint8)


def factor_decode(codes: np.ndarray, mags: np.ndarray) -> np.ndarray:
    v = np.asarray(mags, dtype=np.float64)[codes & 7]
    return np.where(codes & 8, v, -v)


def pack_nibbles(codes: np.ndarray) -> np.ndarray:
    """[..., m] 4-bit codes -> [..., m/2] bytes, entry e in the low (e even) or high nibble of byte e // 2."""
    c = np.asarray(codes, dtype=np.uint8)
    return (c[..., 0::2] | (c[..., 1::2] << 4)).astype(np.uint8)


def unpack_nibbles(packed: np.ndarray) -> np.ndarray:
    p = np.asarray(packed, dtype=np.uint8)
    out = np.empty(p.shape[:-1] + (2 * p.shape[-1],), dtype=np.uint8)
    out[..., 0::2] = p & 15
    out[..., 1::2] = p >> 4
    return out


def quantize_factors(U: np.ndarray, V: np.ndarray, phi: np.ndarray):
    """U [n, r], V [d, r] (orthonormal columns), phi [r] -> codes, codebooks and the
    binary16 factors every later step uses: lfac = fp16(U_hat * phi16), rfac = V_hat."""
    mu, mv = adaptive_magnitudes(U), adaptive_magnitudes(V)
    lcodes, rcodes = factor_encode(U.T, mu), factor_encode(V.T, mv)          # [r, n], [r, d]
    phi16 = fp16_round(phi)
    lfac = fp16_round(factor_decode(lcodes, mu) * phi16[:, None])
    rfac = factor_decode(rcodes, mv)
    return lcodes, rcodes, np.stack([mu, mv]), phi16, lfac, rfac


def compress_block(S: np.ndarray, Pi: np.ndarray, cb: Codebook, r_max: int = 32,
                   force_rank0: bool = False, factor_bits: int = 16, loss: str = "frobenius") -> BlockRecord:
    """Alg. 3: eOptShrink, residual against the *stored* factors (binary16, or
    4-bit codes with per-block codebooks), TQ_MSE per row.  With r^+ = 0 the block
    goes to TQ_MSE unchanged."""
    if factor_bits not in (16, 4):
        raise ValueError("factor_bits must be 16 or 4")
    S = np.asarray(S, dtype=np.float64)
    n, d = S.shape
    es = eoptshrink(S, r_max, loss)
    r = 0 if force_rank0 else es.rank
    extra = {}
    if r > 0 and factor_bits == 4:
        lcodes, rcodes, fbook, phi16, lfac, rfac = quantize_factors(es.U[:, :r], es.V[:, :r], es.phi[:r])
        extra = dict(factor_bits=4, lcodes=lcodes, rcodes=rcodes, fbook=fbook, phi16=phi16)
        R = S - lfac.T @ rfac
    elif r > 0:
        lfac = fp16_round((es.U[:, :r] * es.phi[None, :r]).T)   # [r, n]
        rfac = fp16_round(es.V[:, :r].T)                        # [r, d]
        R = S - lfac.T @ rfac
    else:
        lfac = np.zeros((0, n))
        rfac = np.zeros((0, d))
        R = S
        if factor_bits == 4:
            extra = dict(factor_bits=4, lcodes=np.zeros((0, n), np.uint8), rcodes=np.zeros((0, d), np.uint8),
                         fbook=np.zeros((2, FACTOR_LEVELS)), phi16=np.zeros(0))
    codes, rho, z = tq_mse_encode(R, Pi, cb)
    return BlockRecord(n, d, cb.bits, r, es.flags, es.phi[:r], es.sigma[:r], lfac, rfac, codes,
                       fp16_round(rho), lam=es.lam, lam_plus=es.lam_plus, rho=rho, z=z, R=R, **extra)


def decompress_block(rec: BlockRecord, Pi: np.ndarray, cb: Codebook) -> np.ndarray:
    """x_hat_t = rho_t Pi^T z_hat_t + (U diag(phi) V^T)[t, :]  (Alg. 1 line 6 plus
    the stored low-rank part of Alg. 2's Return), float64, before any rounding."""
    x = tq_mse_decode(rec.codes, rec.rho16, Pi, cb)
    if rec.rank > 0:
        x = x + rec.lfac.T @ rec.rfac
    return x


def score_block(q: np.ndarray, rec: BlockRecord, Pi: np.ndarray, cb: Codebook) -> np.ndarray:
    """<q, x_hat_t> / sqrt(d) for every query row of q and every token of the
    block (Sec. 2.1 attention logits; Remark 6.5 split into low-rank + residual)."""
    x = decompress_block(rec, Pi, cb)
    return (np.asarray(q, dtype=np.float64) @ x.T) / math.sqrt(rec.d)


def score_stream(q: np.ndarray, recs, tail: np.ndarray, Pi: np.ndarray, cb: Codebook) -> np.ndarray:
    """Logits of one KV head whose cache is still being filled (Sec. 3.1: blocks are
    compressed as they complete; Sec. 7: the newest fewer-than-n tokens stay in
    FP16): the compressed blocks `recs` in token order, then the uncompressed
    tail [t, d], whose logits are the plain <q, k_t> / sqrt(d) of Sec. 2.1."""
    q = np.asarray(q, dtype=np.float64)
    parts = [score_block(q, r, Pi, cb) for r in recs]
    tail = np.asarray(tail, dtype=np.float64)
    if tail.shape[0]:
        parts.append((q @ tail.T) / math.sqrt(tail.shape[1]))
    return np.concatenate(parts, axis=-1) if parts else np.zeros(q.shape[:-1] + (0,))


# --------------------------------------------------------------------------
# TQ_prod: the 1-bit QJL correction of Alg. 1 (lines "TQ_prod") and Eq. (qjl)
# --------------------------------------------------------------------------
def gaussian_projection(d: int, seed: int) -> np.ndarray:
    """Phi of Alg. 1 REQUIRE: d x d with iid N(0,1) entries, filled row-major
    from `gaussian_stream` (the generator that also feeds the rotation)."""
    return gaussian_stream(seed, d * d).reshape(d, d)


@dataclass
class QjlRecord:
    """Alg. 1 "Store" of TQ_prod for the rows of one block."""
    signs: np.ndarray    # [n, d] uint8 in {0, 1}: 1 where (Phi r_x)_i >= 0
    gamma16: np.ndarray  # [n] stored residual norms |r_x| (binary16 values as float64)
    gamma: np.ndarray = field(default=None, repr=False)   # unrounded norms (diagnostic)
    proj: np.ndarray = field(default=None, repr=False)    # Phi r_x (diagnostic: distance of every sign decision from 0)


def qjl_encode(S: np.ndarray, rec: BlockRecord, Pi: np.ndarray, cb: Codebook, Phi: np.ndarray) -> QjlRecord:
    """Alg. 1 lines "r_x <- x - x_hat_MSE" and "Store |r_x| and sign(Phi r_x)",
    applied where Alg. 3 applies TurboQuant: to the rows of the residual R.  The
    quantisation residual of row t is r_x = R_t - R_hat_t = S_t - x_hat_t with
    x_hat the reconstruction of the stored record (stored norm, stored factors).
    sign(0) counts as +1; the norm is stored in binary16 like the row norms."""
    S = np.asarray(S, dtype=np.float64)
    rx = S - decompress_block(rec, Pi, cb)
    proj = rx @ Phi.T
    gamma = np.linalg.norm(rx, axis=1)
    return QjlRecord((proj >= 0).astype(np.uint8), fp16_round(gamma), gamma=gamma, proj=proj)


def qjl_correction(q: np.ndarray, qjl: QjlRecord, Phi: np.ndarray) -> np.ndarray:
    """Second term of Eq. (qjl) for every query row of q and every token:
    |r_x| sqrt(pi/2)/d <Phi y, sign(Phi r_x)>, with the stored norm."""
    q = np.asarray(q, dtype=np.float64)
    d = Phi.shape[1]
    sgn = 2.0 * qjl.signs.astype(np.float64) - 1.0
    return (q @ Phi.T) @ sgn.T * (math.sqrt(math.pi / 2.0) / d) * qjl.gamma16[None, :]


def score_block_prod(q: np.ndarray, rec: BlockRecord, qjl: QjlRecord, Pi: np.ndarray, cb: Codebook,
                     Phi: np.ndarray) -> np.ndarray:
    """Attention logits with the TQ_prod estimator of Eq. (qjl) in place of the
    MSE reconstruction: (<q, x_hat_t> + correction) / sqrt(d)."""
    return score_block(q, rec, Pi, cb) + qjl_correction(q, qjl, Phi) / math.sqrt(rec.d)


def pack_signs(signs: np.ndarray) -> np.ndarray:
    """[n, d] sign bits -> [n, d/8] bytes, coordinate j in bit (j mod 8) of byte j // 8 (one more bit-plane)."""
    return np.packbits(np.asarray(signs, dtype=np.uint8), axis=1, bitorder="little")


def unpack_signs(packed: np.ndarray, d: int) -> np.ndarray:
    return np.unpackbits(np.asarray(packed, dtype=np.uint8), axis=1, bitorder="little")[:, :d]


def softmax_rows(scores: np.ndarray) -> np.ndarray:
    """softmax along the last axis (the attention weights of Sec. 2.1, Eq. for
    Attention(Q, K, V)), with the row maximum subtracted first."""
    s = np.asarray(scores, dtype=np.float64)
    e = np.exp(s - np.max(s, axis=-1, keepdims=True))
    return e / np.sum(e, axis=-1, keepdims=True)


def attend_blocks(weights: np.ndarray, recs, Pi: np.ndarray, cb: Codebook) -> np.ndarray:
    """Attention output of one KV head on compressed values (Sec. 2.1:
    softmax(QK^T / sqrt(d)) V with V replaced by its reconstruction): weights
    [h, T] over the tokens of the blocks `recs` in order, T = sum of their n;
    returns sum_t weights[:, t] x_hat_t, [h, d]."""
    w = np.asarray(weights, dtype=np.float64)
    out = np.zeros((w.shape[0], recs[0].d if recs else 0))
    t0 = 0
    for r in recs:
        out += w[:, t0:t0 + r.n] @ decompress_block(r, Pi, cb)
        t0 += r.n
    if t0 != w.shape[1]:
        raise ValueError("weights do not cover the blocks' tokens")
    return out


def attend_stream(weights: np.ndarray, recs, tail: np.ndarray, Pi: np.ndarray, cb: Codebook) -> np.ndarray:
    """attend_blocks over a cache that is still being filled: the weights cover
    the compressed blocks' tokens and then the uncompressed tail values [t, d]
    (Sec. 7: the newest tokens stay in FP16), which enter as they are."""
    w = np.asarray(weights, dtype=np.float64)
    tail = np.asarray(tail, dtype=np.float64)
    T = sum(r.n for r in recs)
    if w.shape[1] != T + tail.shape[0]:
        raise ValueError("weights do not cover the blocks' tokens plus the tail")
    out = attend_blocks(w[:, :T], recs, Pi, cb) if recs else np.zeros((w.shape[0], tail.shape[1]))
    return out + w[:, T:] @ tail


# --------------------------------------------------------------------------
# storage encoding of the codes (builder's format; the paper only says "indices")
# --------------------------------------------------------------------------
def pack_codes(codes: np.ndarray, bits: int) -> np.ndarray:
    """[n, d] codes -> [n, d*bits/8] bytes.

    Each row is stored as `bits` bit-planes of d/8 bytes: plane p holds bit p of
    the d codes, coordinate j in bit (j mod 8) of byte j // 8.
    """
    n, d = codes.shape
    out = np.zeros((n, bits, d // 8), dtype=np.uint8)
    for p in range(bits):
        plane = (codes >> p) & 1
        for j in range(d):
            out[:, p, j // 8] |= (plane[:, j] << (j % 8)).astype(np.uint8)
    return out.reshape(n, bits * d // 8)


def unpack_codes(packed: np.ndarray, bits: int, d: int) -> np.ndarray:
    n = packed.shape[0]
    pk = packed.reshape(n, bits, d // 8)
    codes = np.zeros((n, d), dtype=np.uint8)
    for p in range(bits):
        for j in range(d):
            codes[:, j] |= (((pk[:, p, j // 8] >> (j % 8)) & 1) << p).astype(np.uint8)
    return codes


def bits_per_entry(n: int, d: int, bits: int, rank: int, b_s: int = 16) -> float:
    """Alg. 3 last line plus the two shared costs of Remark 3.1: the binary16
    norm per row (16/d) and the binary16 shrunk values (16 r / (n d))."""
    return bits + rank * (n + d) * b_s / (n * d) + 16.0 / d + 16.0 * rank / (n * d)
