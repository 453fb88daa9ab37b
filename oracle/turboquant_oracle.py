"""CPU oracle for TurboQuant (arxiv 2504.19874).  TEST INFRASTRUCTURE ONLY.

This module is the slow, plain, obviously-correct statement of what the
method computes.  It exists so that the GPU library can be checked against
something that was written from the paper and pinned to the paper's own
numbers.  It is NOT part of the product: nothing in the package may import
it, and it imports nothing from the package.  Only the tests, the smoke
check and the benchmark's cpu_baseline leg call it.

Arithmetic: float64 everywhere, with float32 rounding at exactly these
points: the stored parameters (Pi, S, centroids, bounds), the rotated
coordinates y just before the bucket decision, and the stored per-vector
scalars (norm, gamma).  The bucket decision itself is an fp32 compare of
fp32 y against the fp32 boundary table, so that it is a bit-deterministic
function of y.

Readings taken where the paper is silent (each listed in the design notes):
  * a coordinate exactly on a bucket boundary goes to the upper bucket;
  * sign(0) = +1 (bit 1);
  * a zero input vector keeps x_hat = 0 and stored norm 0;
  * bits_mse = 0 means a one-entry codebook {0} and no index bits;
  * gamma is the residual norm of the unit-normalised vector;
  * the packed layout is groups of 32 coordinates stored as bit planes.

The split into two instances over the channels (Sec. 4.3) is a composition
of the functions above and nothing else; its bookkeeping is pinned by the
per-instance distortion and variance it must show (tests/test_oracle_quant.py).
The attention read-out over a quantised cache (attend) is softmax of the
scores times the dequantised values; pinned in tests/test_oracle_attend.py by a
scalar-loop brute force and by the cases with a known answer (equal logits, one
dominant key, a common shift of the logits, a single key).

The optimal prefix code for the indices (Sec. 3.1, last paragraph) is Huffman's
construction; pinned in tests/test_oracle_entropy.py by Kraft's equality, exact
lengths for dyadic laws, brute force over every complete code of small
alphabets, and the paper's two figures for b = 4.

Pinned by tests/test_oracle_*.py (closed forms, the paper's printed values,
brute force).  The only part with no external pin is the exact index vector
of one particular input under one particular Pi ("parity unpinned" for that
alone): it is fixed only through the definition argmin_k |y_j - c_k|, which
the tests do check by brute force.
"""
from __future__ import annotations

import math

import numpy as np
from scipy import special as _sp

# --------------------------------------------------------------------------
# Lemma 1: law of one coordinate of a uniform point on the unit sphere
# --------------------------------------------------------------------------


def coord_log_norm_const(d: int) -> float:
    """log of Gamma(d/2) / (sqrt(pi) Gamma((d-1)/2))  (Lemma 1)."""
    return _sp.gammaln(d / 2.0) - 0.5 * math.log(math.pi) - _sp.gammaln((d - 1) / 2.0)


def coord_pdf(x, d: int):
    """f_X(x) = C_d (1 - x^2)^((d-3)/2) on [-1, 1]  (Lemma 1)."""
    x = np.asarray(x, dtype=np.float64)
    return np.exp(coord_log_norm_const(d) + 0.5 * (d - 3) * np.log1p(-x * x))


def coord_cdf(x, d: int):
    """F_X(x).  (1+X)/2 is Beta(a, a) with a = (d-1)/2, so F is a regularised
    incomplete beta function."""
    x = np.asarray(x, dtype=np.float64)
    a = 0.5 * (d - 1)
    return _sp.betainc(a, a, 0.5 * (1.0 + x))


def coord_partial_mean(lo, hi, d: int):
    """int_lo^hi x f_X(x) dx = -C_d/(d-1) [ (1-x^2)^((d-1)/2) ]_lo^hi."""
    lo = np.asarray(lo, dtype=np.float64)
    hi = np.asarray(hi, dtype=np.float64)
    lc = coord_log_norm_const(d) - math.log(d - 1)

    def g(t):
        with np.errstate(divide="ignore"):
            return np.exp(lc + 0.5 * (d - 1) * np.log1p(-t * t))

    return g(lo) - g(hi)


def coord_partial_second_moment(lo, hi, d: int):
    """int_lo^hi x^2 f_X dx.  Uses x^2 f_d = f_d - (1-x^2) f_d and
    (1-x^2) f_d = ((d-1)/d) f_{d+2}."""
    m0 = coord_cdf(hi, d) - coord_cdf(lo, d)
    m0_up = coord_cdf(hi, d + 2) - coord_cdf(lo, d + 2)
    return m0 - (d - 1.0) / d * m0_up


# --------------------------------------------------------------------------
# eq. (4): Lloyd-Max codebook for f_X
# --------------------------------------------------------------------------


def lloyd_max_codebook(d: int, bits: int, tol: float = 1e-13, max_iter: int = 200000):
    """Solve the 1-D continuous k-means problem of eq. (4) for f_X at this d.

    Returns (centroids[2^bits] float64 ascending, bounds[2^bits - 1] float64,
    cost) where bounds are the midpoints of consecutive centroids (Voronoi
    cells, Sec. 3.1) and cost = C(f_X, bits), the per-coordinate MSE.
    """
    if d < 3:
        raise ValueError("d must be >= 3")
    if bits < 0 or bits > 8:
        raise ValueError("bits must be in [0, 8]")
    K = 1 << bits
    if K == 1:
        return np.zeros(1), np.zeros(0), 1.0 / d
    a = 0.5 * (d - 1)
    # start from the quantiles at (k + 1/2)/K
    c = 2.0 * _sp.betaincinv(a, a, (np.arange(K) + 0.5) / K) - 1.0
    c = 0.5 * (c - c[::-1])
    scale = 1.0 / math.sqrt(d)
    for _ in range(max_iter):
        t = 0.5 * (c[:-1] + c[1:])
        edges = np.concatenate(([-1.0], t, [1.0]))
        mass = coord_cdf(edges[1:], d) - coord_cdf(edges[:-1], d)
        mean = coord_partial_mean(edges[:-1], edges[1:], d)
        c_new = mean / mass
        c_new = 0.5 * (c_new - c_new[::-1])  # the law is symmetric about 0
        delta = np.max(np.abs(c_new - c))
        c = c_new
        if delta < tol * scale:
            break
    t = 0.5 * (c[:-1] + c[1:])
    return c, t, codebook_cost(c, d)


def codebook_cost(c, d: int) -> float:
    """sum_k int_{cell k} (x - c_k)^2 f_X dx for an ascending codebook c with
    midpoint cell boundaries (the objective of eq. (4))."""
    c = np.asarray(c, dtype=np.float64)
    if c.size == 1:
        edges = np.array([-1.0, 1.0])
    else:
        edges = np.concatenate(([-1.0], 0.5 * (c[:-1] + c[1:]), [1.0]))
    lo, hi = edges[:-1], edges[1:]
    m0 = coord_cdf(hi, d) - coord_cdf(lo, d)
    m1 = coord_partial_mean(lo, hi, d)
    m2 = coord_partial_second_moment(lo, hi, d)
    return float(np.sum(m2 - 2.0 * c * m1 + c * c * m0))


def bucket_masses(c, d: int):
    """p_l = mass of f_X in Voronoi cell l (the entropy-coding paragraph of
    Sec. 3.1)."""
    c = np.asarray(c, dtype=np.float64)
    edges = np.concatenate(([-1.0], 0.5 * (c[:-1] + c[1:]), [1.0]))
    return coord_cdf(edges[1:], d) - coord_cdf(edges[:-1], d)


def codebook_fp32(d: int, bits: int):
    """The stored tables: fp32 centroids, and fp32 roundings of the fp64
    midpoints of the fp64 centroids."""
    c, t, cost = lloyd_max_codebook(d, bits)
    return c.astype(np.float32), t.astype(np.float32), cost


# --------------------------------------------------------------------------
# Alg. 1 setup: random rotation; Alg. 2 setup uses a plain Gaussian matrix
# --------------------------------------------------------------------------


def rotation_from_gaussian(G):
    """Pi = orthogonal factor of the QR decomposition of a Gaussian matrix
    (Sec. 3.1), with the sign choice that makes diag(R) positive, so that Pi
    is a deterministic function of G and Haar distributed.  Rounded to fp32
    once; everything later uses the rounded matrix."""
    G = np.asarray(G, dtype=np.float64)
    Q, R = np.linalg.qr(G)
    sgn = np.where(np.diag(R) < 0.0, -1.0, 1.0)
    return (Q * sgn[None, :]).astype(np.float32)


# --------------------------------------------------------------------------
# input handling
# --------------------------------------------------------------------------


def bf16_bits_to_f64(u16):
    """Exact value of bfloat16 bit patterns (the top half of an fp32)."""
    u = np.asarray(u16, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def unit_normalise(x, normalise: bool = True):
    """Norm handling of Sec. 1.3: returns (x_hat float64, norm float32).
    With normalise=False the caller asserts unit norm: x is used as is and
    the stored norm is 1."""
    x = np.asarray(x, dtype=np.float64)
    if not normalise:
        return x, np.ones(x.shape[0], dtype=np.float32)
    nu = np.sqrt(np.sum(x * x, axis=1))
    safe = np.where(nu > 0.0, nu, 1.0)
    xh = np.where(nu[:, None] > 0.0, x / safe[:, None], 0.0)
    return xh, nu.astype(np.float32)


# --------------------------------------------------------------------------
# Alg. 1: TurboQuant_mse
# --------------------------------------------------------------------------


def rotate(xh, Pi):
    """y = Pi x for every row x of xh, rounded to fp32 (Alg. 1, Quant: the rotation step)."""
    P = np.asarray(Pi, dtype=np.float32).astype(np.float64)
    return (np.asarray(xh, dtype=np.float64) @ P.T).astype(np.float32)


def nearest_centroid(y32, bounds32):
    """idx_j = argmin_k |y_j - c_k| (Alg. 1, Quant: the nearest-centroid step), evaluated as the
    number of cell boundaries that y_j is >= to, in fp32."""
    y32 = np.asarray(y32, dtype=np.float32)
    b = np.asarray(bounds32, dtype=np.float32)
    idx = np.zeros(y32.shape, dtype=np.int32)
    for k in range(b.size):
        idx += (y32 >= b[k]).astype(np.int32)
    return idx


def quant_mse(x, Pi, bounds32, normalise: bool = True):
    """Quant_mse of Alg. 1 on every row.  Returns (idx int32 [n,d],
    norm float32 [n], y float32 [n,d])."""
    xh, nu = unit_normalise(x, normalise)
    y = rotate(xh, Pi)
    return nearest_centroid(y, bounds32), nu, y


def dequant_mse(idx, Pi, centroids32, norm=None):
    """DeQuant_mse of Alg. 1: x~ = Pi^T c[idx], rescaled by the stored norm."""
    c = np.asarray(centroids32, dtype=np.float32).astype(np.float64)
    P = np.asarray(Pi, dtype=np.float32).astype(np.float64)
    yt = c[np.asarray(idx)]
    xt = yt @ P  # row form of Pi^T y~
    if norm is not None:
        xt = xt * np.asarray(norm, dtype=np.float32).astype(np.float64)[:, None]
    return xt


# --------------------------------------------------------------------------
# Def. 1 (QJL) and Alg. 2: TurboQuant_prod
# --------------------------------------------------------------------------


def qjl_scale(d: int) -> float:
    """sqrt(pi/2) / d  (Def. 1, inverse map)."""
    return math.sqrt(math.pi / 2.0) / d


def residual_and_sketch(xh, idx, Pi, S, centroids32):
    """Lines 2-3 of Quant_prod (Alg. 2) for given MSE-stage indices:
    r = x_hat - DeQuant_mse(idx), u = S r.  Returns (r, gamma64, u)."""
    r = np.asarray(xh, dtype=np.float64) - dequant_mse(idx, Pi, centroids32)
    gamma = np.sqrt(np.sum(r * r, axis=1))
    S64 = np.asarray(S, dtype=np.float32).astype(np.float64)
    u = r @ S64.T
    return r, gamma, u


def quant_prod(x, Pi, S, centroids32, bounds32, normalise: bool = True):
    """Quant_prod of Alg. 2 with the MSE stage at len(centroids32) levels.
    Returns dict(idx, qjl (bool: True = +1), gamma float32, norm float32,
    y float32, u float64)."""
    xh, nu = unit_normalise(x, normalise)
    y = rotate(xh, Pi)
    idx = nearest_centroid(y, bounds32)
    _, gamma, u = residual_and_sketch(xh, idx, Pi, S, centroids32)
    return dict(idx=idx, qjl=(u >= 0.0), gamma=gamma.astype(np.float32), norm=nu, y=y, u=u)


def dequant_prod(idx, qjl, gamma, Pi, S, centroids32, norm=None):
    """DeQuant_prod of Alg. 2: x~_mse + sqrt(pi/2)/d * gamma * S^T z."""
    d = np.asarray(idx).shape[1]
    S64 = np.asarray(S, dtype=np.float32).astype(np.float64)
    z = np.where(np.asarray(qjl, dtype=bool), 1.0, -1.0)
    g = np.asarray(gamma, dtype=np.float32).astype(np.float64)
    xt = dequant_mse(idx, Pi, centroids32) + qjl_scale(d) * g[:, None] * (z @ S64)
    if norm is not None:
        xt = xt * np.asarray(norm, dtype=np.float32).astype(np.float64)[:, None]
    return xt


# --------------------------------------------------------------------------
# Sec. 4.3: two independent instances over a split of the channels
# (outlier channels at a higher bit-width)
# --------------------------------------------------------------------------


def split_channels(d: int, hi_channels):
    """(hi, lo): the outlier channels and the others, each ascending."""
    hi = np.sort(np.asarray(hi_channels, dtype=np.int64))
    return hi, np.setdiff1d(np.arange(d), hi)


def quant_split(x, hi_channels, inst_hi, inst_lo, prod: bool):
    """Quantise x[:, hi] with instance hi and x[:, lo] with instance lo, each an
    ordinary Quant_mse / Quant_prod of its own dimension.  An instance is a dict
    Pi, S (None for mse), c32, t32.  Returns (result_hi, result_lo)."""
    x = np.asarray(x)
    hi, lo = split_channels(x.shape[1], hi_channels)
    out = []
    for ch, inst in ((hi, inst_hi), (lo, inst_lo)):
        if prod:
            out.append(quant_prod(x[:, ch], inst["Pi"], inst["S"], inst["c32"], inst["t32"]))
        else:
            idx, nu, y = quant_mse(x[:, ch], inst["Pi"], inst["t32"])
            out.append(dict(idx=idx, y=y, norm=nu))
    return out[0], out[1]


def dequant_split(d: int, hi_channels, res_hi, res_lo, inst_hi, inst_lo, prod: bool):
    """The two dequantised parts put back at their channels."""
    hi, lo = split_channels(d, hi_channels)
    n = np.asarray(res_hi["idx"]).shape[0]
    xt = np.zeros((n, d), dtype=np.float64)
    for ch, r, inst in ((hi, res_hi, inst_hi), (lo, res_lo, inst_lo)):
        if prod:
            xt[:, ch] = dequant_prod(r["idx"], r["qjl"], r["gamma"], inst["Pi"], inst["S"], inst["c32"], r["norm"])
        else:
            xt[:, ch] = dequant_mse(r["idx"], inst["Pi"], inst["c32"], r["norm"])
    return xt


def score(q, x_tilde):
    """Inner-product estimates <q, Q^-1(Q(x))> for every (query, code) pair
    (Sec. 3.2, the displayed estimator), through the dequantised vectors."""
    return np.asarray(q, dtype=np.float64) @ np.asarray(x_tilde, dtype=np.float64).T


def attend(q, k_tilde, v_tilde, scale: float):
    """Decoder attention of a few queries over a quantised key/value cache
    (the use of Sec. 4.3: keys AND values of past tokens are kept as codes):
        logits_i = scale * <q, k~_i>      (the estimator of Sec. 3.2 on the keys)
        p        = softmax(logits)
        out      = sum_i p_i v~_i         (v~ = DeQuant of the value codes)
    The paper states nothing about the value side beyond DeQuant, so this is
    the textbook attention read-out applied to the dequantised cache.  The
    maximum is subtracted before exp (no effect on the value in exact
    arithmetic)."""
    logits = float(scale) * score(q, k_tilde)
    logits = logits - logits.max(axis=1, keepdims=True)
    w = np.exp(logits)
    p = w / w.sum(axis=1, keepdims=True)
    return p @ np.asarray(v_tilde, dtype=np.float64)


def topk(scores, k: int):
    """Indices of the k largest scores per row; equal scores order by lower
    index first."""
    s = np.asarray(scores)
    order = np.argsort(-s, axis=1, kind="stable")
    return order[:, :k]


# --------------------------------------------------------------------------
# the B = b*d bit string (Sec. 1.1): layout chosen by this build
# --------------------------------------------------------------------------


def pack_planes(idx, bits: int):
    """Group-of-32 bit planes: for vector i, coordinate group g (coordinates
    32g..32g+31) and plane p < bits, word [i, g*bits + p] has bit l equal to
    bit p of idx[i, 32g + l]."""
    idx = np.asarray(idx)
    n, d = idx.shape
    assert d % 32 == 0
    out = np.zeros((n, (d // 32) * bits), dtype=np.uint32)
    for g in range(d // 32):
        for p in range(bits):
            w = np.zeros(n, dtype=np.uint64)
            for l in range(32):
                w |= ((idx[:, 32 * g + l].astype(np.uint64) >> np.uint64(p)) & np.uint64(1)) << np.uint64(l)
            out[:, g * bits + p] = w.astype(np.uint32)
    return out


def unpack_planes(words, bits: int, d: int):
    words = np.asarray(words, dtype=np.uint32)
    n = words.shape[0]
    idx = np.zeros((n, d), dtype=np.int32)
    for g in range(d // 32):
        for p in range(bits):
            w = words[:, g * bits + p]
            for l in range(32):
                idx[:, 32 * g + l] |= (((w >> np.uint32(l)) & np.uint32(1)).astype(np.int32)) << p
    return idx


def pack_signs(qjl):
    """qjl word [i, g] bit l = 1 iff sign is +1 at coordinate 32g + l."""
    return pack_planes(np.asarray(qjl, dtype=bool).astype(np.int32), 1)


def unpack_signs(words, d: int):
    return unpack_planes(words, 1, d).astype(bool)


# --------------------------------------------------------------------------
# entropy coding of the indices (Sec. 3.1, last paragraph): an optimal prefix
# code for the bucket probabilities p_l.  The paper names the technique and
# its gain and declines to use it; the bit stream below is this build's
# choice: the codewords of coordinates 0..d-1 of a vector, most significant
# bit first, vectors back to back.
# --------------------------------------------------------------------------


def index_entropy(p):
    """Entropy in bits of the index distribution {p_l}."""
    p = np.asarray(p, dtype=np.float64)
    nz = p[p > 0]
    return float(-(nz * np.log2(nz)).sum())


def huffman_lengths(p):
    """Codeword lengths of an optimal prefix code for probabilities p
    (Huffman's construction: merge the two least probable nodes until one
    is left; every merge makes the codewords below it one bit longer).
    Ties go to the node that was made first / has the lower symbol."""
    p = [float(v) for v in p]
    K = len(p)
    if K == 1:
        return np.zeros(1, dtype=np.int64)
    nodes = [(p[s], s, [s]) for s in range(K)]  # (probability, age, symbols below)
    lengths = np.zeros(K, dtype=np.int64)
    age = K
    while len(nodes) > 1:
        nodes.sort(key=lambda t: (t[0], t[1]))
        a, b = nodes[0], nodes[1]
        for s in a[2] + b[2]:
            lengths[s] += 1
        nodes = nodes[2:] + [(a[0] + b[0], age, a[2] + b[2])]
        age += 1
    return lengths


def canonical_codewords(lengths):
    """Codewords of the canonical prefix code with the given lengths:
    symbols ordered by (length, symbol) take consecutive binary numbers,
    shifted left whenever the length grows."""
    lengths = np.asarray(lengths, dtype=np.int64)
    code = np.zeros(lengths.size, dtype=np.int64)
    nxt, prev = 0, 0
    for s in sorted(range(lengths.size), key=lambda s: (lengths[s], s)):
        nxt <<= int(lengths[s] - prev)
        code[s] = nxt
        nxt += 1
        prev = int(lengths[s])
    return code


def prefix_encode(idx, lengths, codewords):
    """Bit list of the rows of idx (one codeword per coordinate, most
    significant bit first) and the bit offset at which every row starts."""
    bits, starts = [], []
    for row in np.asarray(idx):
        starts.append(len(bits))
        for v in row:
            L, c = int(lengths[v]), int(codewords[v])
            bits.extend((c >> (L - 1 - k)) & 1 for k in range(L))
    starts.append(len(bits))
    return bits, starts


def prefix_decode(bits, lengths, codewords, n: int, d: int):
    """Inverse of prefix_encode by matching codewords bit by bit."""
    table = {(int(lengths[s]), int(codewords[s])): s for s in range(len(lengths))}
    out = np.zeros((n, d), dtype=np.int32)
    pos = 0
    for i in range(n):
        for j in range(d):
            L, c = 0, 0
            while (L, c) not in table:
                c = (c << 1) | bits[pos]
                pos += 1
                L += 1
            out[i, j] = table[(L, c)]
    return out
