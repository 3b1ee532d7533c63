"""Step-by-step CPU reference of Winograd convolution over a residue number system.

TEST INFRASTRUCTURE ONLY (see the package docstring).  Plain numpy int64 and
`fractions.Fraction`; every function follows one passage of the paper and is
written so it can be checked against that passage by eye.  Nothing is blocked,
fused or reordered: each stage materialises its full tensor.

Notation follows the paper: F(M x M, R x R) produces an M x M output tile from
an N x N input tile, N = M + R - 1, with transform matrices A^T (M x N),
G (N x R), B^T (N x N) built from N interpolation points S_0..S_{N-1} of which
the last is the point at infinity (section 4).  In the code below the paper's
M, R, N are spelled m, r, t because N, K, C are taken by the tensor shapes.

Readings where the paper leaves a choice (each also listed in the design notes):
  * points: 0, +1, -1, +2, -2, ..., infinity -- the pattern of the printed
    F(2,3), F(4,3) and F(10,3) examples, continued for other sizes;
  * the point at infinity contributes the row (0,...,0,1) to the Vandermonde
    matrix (it evaluates the leading coefficient);
  * the fractions of B^T are moved into G (section 4 says so without giving the rule): row j of V^{-T} is
    multiplied by |prod_{l != j}(S_j - S_l)| and row j of G divided by it,
    which reproduces every matrix printed in the paper;
  * residues are kept in the symmetric range [-(p-1)/2, (p-1)/2] (the remark
    after the matrices modulo 253);
  * signed results are recovered by mixed-radix conversion with symmetric
    digits, which lands in [-(P-1)/2, (P-1)/2], P the product of the moduli --
    the dynamic ranges quoted in sections 5 and 8.
"""
from __future__ import annotations

from fractions import Fraction
from math import gcd

import numpy as np


# --------------------------------------------------------------------------
# Residue number system (section 3)
# --------------------------------------------------------------------------

def sym(v, p: int):
    """Representative of v modulo p in [-(p-1)/2, (p-1)/2] (p odd); int or int64 array."""
    h = (p - 1) // 2
    return (v + h) % p - h


def to_rns(v, moduli):
    """Forward conversion x -> (x mod m_0, ..., x mod m_{n-1}), least non-negative residues."""
    return [v % p for p in moduli]


def modinv(a: int, p: int) -> int:
    """Multiplicative inverse of a modulo p (p need not be prime; a must be a unit)."""
    a %= p
    if gcd(a, p) != 1:
        raise ZeroDivisionError(f"{a} has no inverse modulo {p}")
    return pow(a, -1, p)


def mrc(residues, moduli, signed: bool = True):
    """Mixed-radix conversion of residues (one int or int64 array per modulus) back to integers.

    Digits: v_0 = x_0;  v_j = ((..((x_j - v_0)/m_0 - v_1)/m_1 ..) - v_{j-1})/m_{j-1}  (mod m_j);
    value: x = v_0 + m_0 (v_1 + m_1 (v_2 + ...)).  For two moduli this is the
    worked example of section 3, x = 6 + 7*[((3-6)/7) mod 9] = 48.
    With signed=False the digits are least non-negative (0 <= x < P, the
    section-3 statement); with signed=True they are symmetric and the value is
    the representative in [-(P-1)/2, (P-1)/2].
    """
    n = len(moduli)
    digits = []
    for j in range(n):
        pj = moduli[j]
        tmp = residues[j]
        for l in range(j):
            tmp = ((tmp - digits[l]) * modinv(moduli[l], pj)) % pj
        tmp = tmp % pj
        digits.append(sym(tmp, pj) if signed else tmp)
    value = digits[n - 1]
    for j in range(n - 2, -1, -1):
        value = digits[j] + moduli[j] * value
    return value


def dynamic_range(moduli) -> int:
    """Largest magnitude representable with symmetric residues: (prod m_i - 1) / 2."""
    P = 1
    for p in moduli:
        P *= p
    return (P - 1) // 2


# --------------------------------------------------------------------------
# Winograd transform matrices (section 4) and their residues (section 5)
# --------------------------------------------------------------------------

INF = "inf"


def interpolation_points(t: int):
    """t points 0, 1, -1, 2, -2, ..., infinity (t - 1 finite ones)."""
    pts = [0]
    a = 1
    while len(pts) < t - 1:
        pts.append(a)
        if len(pts) < t - 1:
            pts.append(-a)
        a += 1
    return pts + [INF]


def vandermonde(points):
    """t x t Vandermonde matrix over Q; the infinite point gives the row (0,..,0,1)."""
    t = len(points)
    V = [[Fraction(0)] * t for _ in range(t)]
    for i, s in enumerate(points):
        if s == INF:
            V[i][t - 1] = Fraction(1)
        else:
            for j in range(t):
                V[i][j] = Fraction(s) ** j
    return V


def _invert(Mx):
    """Gauss-Jordan inverse over Q."""
    t = len(Mx)
    aug = [list(row) + [Fraction(int(i == j)) for j in range(t)] for i, row in enumerate(Mx)]
    for col in range(t):
        piv = next(rw for rw in range(col, t) if aug[rw][col] != 0)
        aug[col], aug[piv] = aug[piv], aug[col]
        inv = 1 / aug[col][col]
        aug[col] = [v * inv for v in aug[col]]
        for rw in range(t):
            if rw != col and aug[rw][col] != 0:
                f = aug[rw][col]
                aug[rw] = [a - f * b for a, b in zip(aug[rw], aug[col])]
    return [row[t:] for row in aug]


def row_denominators(points):
    """|prod_{l != j} (S_j - S_l)| over the finite points, per finite point j; 1 for infinity."""
    fin = [s for s in points if s != INF]
    out = []
    for j, sj in enumerate(fin):
        d = 1
        for l, sl in enumerate(fin):
            if l != j:
                d *= (sj - sl)
        out.append(abs(d))
    return out + [1] * (len(points) - len(fin))


def matrices_Q(m: int, r: int):
    """(A^T, G, B^T) of F(m, r) over Q as nested lists of Fraction.

    A^T = V^T[0:m, :],  G = V[:, 0:r],  B^T = V^{-T}, then the per-row
    fractions of B^T are moved into G (see the module docstring).
    """
    t = m + r - 1
    pts = interpolation_points(t)
    V = vandermonde(pts)
    Vinv = _invert(V)
    den = row_denominators(pts)
    AT = [[V[j][i] for j in range(t)] for i in range(m)]
    # the infinite point evaluates the leading coefficient of each factor of
    # the product polynomial: degree r-1 for the filter, m-1 for the output
    G = [[V[j][k] for k in range(r)] for j in range(t)]
    for k in range(r):
        G[t - 1][k] = Fraction(int(k == r - 1))
    for i in range(m):
        AT[i][t - 1] = Fraction(int(i == m - 1))
    BT = [[Vinv[i][j] for i in range(t)] for j in range(t)]      # transpose of V^{-1}
    for j in range(t):
        BT[j] = [v * den[j] for v in BT[j]]
        G[j] = [v / den[j] for v in G[j]]
    return AT, G, BT


def residue_matrix(MQ, p: int) -> np.ndarray:
    """Entry-wise a/b -> a * b^{-1} mod p, symmetric range, as an int64 array."""
    rows = []
    for row in MQ:
        rows.append([sym((f.numerator % p) * modinv(f.denominator, p), p) for f in row])
    return np.array(rows, dtype=np.int64)


def matrices_mod(m: int, r: int, p: int):
    """(A^T_p, G_p, B^T_p) as int64 arrays with symmetric entries."""
    AT, G, BT = matrices_Q(m, r)
    return residue_matrix(AT, p), residue_matrix(G, p), residue_matrix(BT, p)


def check_moduli(m: int, r: int, moduli) -> None:
    """Conditions of sections 3 and 5: pairwise coprime moduli, each coprime to
    every difference of two finite interpolation points (so that every
    denominator of the inverse Vandermonde matrix is a unit)."""
    t = m + r - 1
    fin = [s for s in interpolation_points(t) if s != INF]
    for a in range(len(moduli)):
        for b in range(a + 1, len(moduli)):
            if gcd(moduli[a], moduli[b]) != 1:
                raise ValueError(f"moduli {moduli[a]} and {moduli[b]} are not coprime")
    for p in moduli:
        for j, sj in enumerate(fin):
            for sl in fin[j + 1:]:
                if gcd(p, abs(sj - sl)) != 1:
                    raise ValueError(f"modulus {p} shares a factor with the point difference {sj}-({sl})")


def arithmetic_reduction(m: int, r: int, n: int) -> float:
    """Section 7: multiplications of the direct method over those of F(m x m, r x r) in an n-residue RNS."""
    t = m + r - 1
    return (m * m * r * r) / (t * t) / n


# --------------------------------------------------------------------------
# Layer algorithm (section 6)
# --------------------------------------------------------------------------

def tile_grid(H: int, W: int, r: int, m: int, pad: int):
    Ho, Wo = H + 2 * pad - r + 1, W + 2 * pad - r + 1
    return Ho, Wo, -(-Ho // m), -(-Wo // m)


def input_tiles(x: np.ndarray, r: int, m: int, pad: int) -> np.ndarray:
    """Overlapping t x t patches with stride m of the zero-extended input: d[T, C, t, t], T = N*th*tw.

    Tile (n, ty, tx) starts at input row m*ty - pad, column m*tx - pad; pixels
    outside the plane (padding, and the overhang of ragged last tiles) are 0.
    """
    N, C, H, W = x.shape
    t = m + r - 1
    Ho, Wo, th, tw = tile_grid(H, W, r, m, pad)
    ext_h, ext_w = (th - 1) * m + t, (tw - 1) * m + t
    xe = np.zeros((N, C, ext_h, ext_w), dtype=np.int64)
    xe[:, :, pad:pad + H, pad:pad + W] = x
    d = np.empty((N * th * tw, C, t, t), dtype=np.int64)
    for n in range(N):
        for ty in range(th):
            for tx in range(tw):
                d[(n * th + ty) * tw + tx] = xe[n, :, ty * m:ty * m + t, tx * m:tx * m + t]
    return d


def filter_transform(w: np.ndarray, m: int, moduli) -> np.ndarray:
    """U[i, xi, nu, k, c] = (G_p g^{(c)(k)} G_p^T)[xi, nu] mod p_i  (pre-computable, section 6)."""
    K, C, r, _ = w.shape
    t = m + r - 1
    U = np.empty((len(moduli), t, t, K, C), dtype=np.int64)
    w64 = w.astype(np.int64)
    for i, p in enumerate(moduli):
        _, G, _ = matrices_mod(m, r, p)
        half = np.einsum("xa,kcab->kcxb", G, w64 % p) % p
        full = np.einsum("kcxb,yb->xykc", half, G) % p
        U[i] = sym(full, p)
    return U


def input_transform(x: np.ndarray, r: int, m: int, pad: int, moduli) -> np.ndarray:
    """V[i, xi, nu, tau, c] = (B^T_p d_tau^{(c)} B_p)[xi, nu] mod p_i  (shared by all K filters)."""
    d = input_tiles(x, r, m, pad)
    t = m + r - 1
    V = np.empty((len(moduli), t, t, d.shape[0], d.shape[1]), dtype=np.int64)
    for i, p in enumerate(moduli):
        _, _, BT = matrices_mod(m, r, p)
        half = np.einsum("xa,tcab->tcxb", BT, d % p) % p
        full = np.einsum("tcxb,yb->xytc", half, BT) % p
        V[i] = sym(full, p)
    return V


def residue_gemm(U: np.ndarray, V: np.ndarray, moduli) -> np.ndarray:
    """O[i, xi, nu, k, tau] = (sum_c U[i,xi,nu,k,c] V[i,xi,nu,tau,c]) mod p_i -- one GEMM per
    transform point and residue, the modulo taken after the sum over C (section 6, eq. "gemm")."""
    n, t = U.shape[0], U.shape[1]
    O = np.empty((n, t, t, U.shape[3], V.shape[3]), dtype=np.int64)
    for i, p in enumerate(moduli):
        for a in range(t):
            for b in range(t):
                O[i, a, b] = sym(U[i, a, b] @ V[i, a, b].T, p)
    return O


def inverse_transform(O: np.ndarray, m: int, r: int, moduli) -> np.ndarray:
    """Y[i, k, tau, u, v] = (A^T_p O[i,:,:,k,tau] A_p)[u, v] mod p_i, after the reduction over C."""
    n = O.shape[0]
    Y = np.empty((n, O.shape[3], O.shape[4], m, m), dtype=np.int64)
    for i, p in enumerate(moduli):
        AT, _, _ = matrices_mod(m, r, p)
        half = np.einsum("ux,xykt->ktuy", AT, O[i]) % p
        Y[i] = sym(np.einsum("ktuy,vy->ktuv", half, AT) % p, p)
    return Y


def assemble(tiles: np.ndarray, N: int, Ho: int, Wo: int, m: int) -> np.ndarray:
    """Place the m x m output tiles [K, T, m, m] into y[N, K, Ho, Wo], cropping ragged tiles."""
    K = tiles.shape[0]
    th, tw = -(-Ho // m), -(-Wo // m)
    full = np.zeros((N, K, th * m, tw * m), dtype=np.int64)
    for n in range(N):
        for ty in range(th):
            for tx in range(tw):
                full[n, :, ty * m:(ty + 1) * m, tx * m:(tx + 1) * m] = tiles[:, (n * th + ty) * tw + tx]
    return full[:, :, :Ho, :Wo]


def conv2d(x: np.ndarray, w: np.ndarray, m: int, pad: int, moduli, return_stages: bool = False):
    """The whole pipeline: residues -> transforms -> GEMM -> inverse -> mixed-radix conversion."""
    N, C, H, W = x.shape
    K, _, r, _ = w.shape
    check_moduli(m, r, moduli)
    Ho, Wo, _, _ = tile_grid(H, W, r, m, pad)
    U = filter_transform(w, m, moduli)
    V = input_transform(x, r, m, pad, moduli)
    O = residue_gemm(U, V, moduli)
    Y = inverse_transform(O, m, r, moduli)
    tiles = mrc([Y[i] for i in range(len(moduli))], list(moduli), signed=True)
    y = assemble(tiles, N, Ho, Wo, m)
    if return_stages:
        return y, dict(U=U, V=V, O=O, Y=Y)
    return y
