"""CPU oracle for the certified sub-vocabulary LM-head path (CSV-Decode).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference the GPU path is
checked against.  It may be imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg, and by nothing else; it shares no code with the HIP
path and never receives a value computed there.

Everything is float64 on the values the method is given: bf16 weights W and hidden
states h (as 16-bit patterns), float32 bias b, and the float32 index arrays
(centroids, radii, per-cluster bias maxima).  A BLAS matrix product serves as the
"inner product for all rows" step; nothing is blocked, fused or reordered beyond
what the cited definition states.

Pins (tests/test_oracle_*.py):
  full_logits        head-FLOP arithmetic of Section I (GPT-3 example); linearity; long-double on tiny V
  topk_bruteforce    three independent selections on tiny V
  build_index        partition/permutation invariants, radius >= every member distance, footprint of Section IV
  cluster_bounds     Cauchy-Schwarz invariant (Section III-A), homogeneity, singleton clusters, single cluster
  angular_bounds     two hand-computed planar clusters (tight at the cone's edge, ||w|| ||h|| inside it), every logit dominated
  spherical_kmeans   planted directions recovered; assignment is the largest cosine with ties to the smaller id
  bias_table         a hand-computed cluster; every logit still dominated; never looser than the max-bias bound; m = 1 is that bound
  topk certificate   Theorem 1 against brute force; minimal prefix = {U_c >= true k-th logit}
  eps certificate    proof identity TV = R/(Z_S+R) (Theorem 2), cluster-wise tail <= loose tail
  alg1_step          brute-force enumeration of all prefixes on small C (certificates written out on sets, linear domain)
  csv2r_step         contains Algorithm 1's minimal prefix; monotone thresholds; budget extremes; the softmax prefix of
                     round 1 traced by hand; equal bounds open the smaller cluster id first
  fallback levels    two hand-traced one-dimensional examples (a rescue by one more cluster, an acceptance between eps
                     and 2 eps); Theorems 1 and 2 by brute force over V; levels only ever remove fallbacks
  kmax_update        the printed expression evaluated by hand; a closed loop with a monotone rate model
  nucleus_holds      agrees with the step's flag and with brute-force coverage over V
  certified_distribution   brackets the true probabilities over V; running sums and nucleus length against their definitions
  lloyd_kmeans       planted clusters recovered; assignment is the nearest centroid with ties to the smaller id
  centroid_bf16      the bound stays sound with rounded centroids and costs little
Parity unpinned: the choices K_max = V/4, radius slack 2^-14 and the angular slacks, the tie tolerance, the default of
requiring both certificates, the order and triggers of the fallback levels, the sign of the budget update, which tokens
get their own bias-table entry and the seeding rule are readings of this build, not values the paper fixes.
"""
from __future__ import annotations

import math

import numpy as np

FLAG_TOPK_CERT = 1
FLAG_SOFTMAX_CERT = 2
FLAG_FALLBACK = 4
FLAG_INVALID = 8
FLAG_SOFTMAX_RELAXED = 16   # softmax tail bound met only at the relaxed tolerance 2*eps (Section IV, fallback levels)

COMBINE_ALL = 0   # a step is certified when every enabled certificate holds
COMBINE_ANY = 1   # Algorithm 1's literal "break on either certificate"

NEG_INF = -math.inf


# ----------------------------------------------------------------------------- arithmetic pins
def head_flops(V: int, d: int) -> int:
    """Multiply-adds x2 of one full output-layer product (Section I, the GPT-3 example)."""
    return 2 * V * d


def metadata_bytes_bf16(C: int, d: int) -> int:
    """Footprint with bfloat16 centroids and float32 radius / bias maximum / size: C (2d + 4 + 4 + 4)."""
    return C * (2 * d + 12)


def metadata_bytes(C: int, d: int) -> int:
    """Index metadata footprint C*(4d + 8 + 4) bytes (Section IV, offline preprocessing)."""
    return C * (d * 4 + 8 + 4)


# ----------------------------------------------------------------------------- plain definitions
def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns -> float64 (exact)."""
    return (np.asarray(bits).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def full_logits(W64: np.ndarray, b, h64: np.ndarray) -> np.ndarray:
    """l[s,i] = <W_i, h_s> + b_i for every token i (Eq. "logit", Section II-A)."""
    out = h64 @ W64.T
    if b is not None:
        out = out + np.asarray(b, dtype=np.float64)[None, :]
    return out


def logsumexp(x: np.ndarray) -> float:
    """log sum_i exp(x_i): log of the partition function of Eq. "softmax"."""
    x = np.asarray(x, dtype=np.float64)
    if x.size == 0:
        return NEG_INF
    m = float(np.max(x))
    if m == NEG_INF:
        return NEG_INF
    return m + math.log(float(np.sum(np.exp(x - m))))


def topk_bruteforce(logits: np.ndarray, k: int, ids: np.ndarray | None = None):
    """Largest k by full sort; order (logit descending, token id ascending)."""
    logits = np.asarray(logits, dtype=np.float64)
    if ids is None:
        ids = np.arange(logits.shape[0], dtype=np.int64)
    order = np.lexsort((ids, -logits))[:k]
    return ids[order], logits[order]


# ----------------------------------------------------------------------------- offline index
class OracleIndex:
    """Cluster metadata of Section III-A.1 / Section IV: centroids, radii, bias maxima, row permutation."""

    def __init__(self, mu, R, bmax, n, perm, bias_table=None, ang=None):
        self.mu = np.ascontiguousarray(mu, dtype=np.float32)      # [C,d] stored centroids
        self.R = np.ascontiguousarray(R, dtype=np.float32)        # [C]   stored radii (rounded up)
        self.bmax = np.ascontiguousarray(bmax, dtype=np.float32)  # [C]   max bias in cluster (-inf if empty)
        # [C,m,2] or None: per cluster m pairs (radius, bias) of the top-m bias table; unused entries (0, -inf)
        self.bias_table = None if bias_table is None else np.ascontiguousarray(bias_table, dtype=np.float32)
        # [C,4] or None: angular index (spherical clustering): (cos theta_c, sin theta_c, largest row norm, smallest row
        # norm) with their slack; mu then holds the unit centroid directions and R is unused
        self.ang = None if ang is None else np.ascontiguousarray(ang, dtype=np.float32)
        self.n = np.ascontiguousarray(n, dtype=np.int64)          # [C]   rows per cluster
        self.off = np.concatenate([[0], np.cumsum(self.n)]).astype(np.int64)
        self.perm = np.ascontiguousarray(perm, dtype=np.int64)    # [V]   permuted row -> original token id
        self.C = int(self.n.shape[0])
        self.V = int(self.perm.shape[0])
        self.d = int(self.mu.shape[1])

    def rows(self, c: int) -> np.ndarray:
        """idx(c): original token ids of cluster c."""
        return self.perm[self.off[c]:self.off[c + 1]]


def _round_bf16(x: np.ndarray) -> np.ndarray:
    """float32 -> nearest bfloat16 (ties to even), returned as float32 values."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def _round_up_f32(x: np.ndarray) -> np.ndarray:
    x = np.asarray(x, dtype=np.float64)
    y = x.astype(np.float32)
    low = y.astype(np.float64) < x
    y[low] = np.nextafter(y[low], np.float32(np.inf))
    return y


def build_index(W_bits: np.ndarray, b, labels: np.ndarray, C: int, radius_slack: float = 2.0 ** -14,
                centroid_bf16: bool = False, bias_table_m: int = 0) -> OracleIndex:
    """Index from a cluster assignment.

    mu_c = mean of the cluster's rows, stored as float32;  R_c = max_i ||W_i - mu_c||_2 measured to the
    STORED centroid (Section III-A.1).  The stored radius is R_c(1+rho) + rho*||mu_c||, rounded up to
    float32, so that float32 evaluation of the bound stays above float32 evaluation of the logits.
    Rows are permuted so each cluster is contiguous (Algorithm 1, "contiguous by reordering"):
    clusters in id order, tokens inside a cluster by ascending original id.
    centroid_bf16: the stored centroid is the mean rounded to bfloat16 (nearest even); the radius is measured to
    that stored value, so the bound of Eq. "cluster_bound" stays valid and the centroids take half the bytes.
    bias_table_m >= 2: also build the top-m bias table of Section III ("Advanced Theoretical Improvements", bias
    binning), see bias_table().
    """
    labels = np.asarray(labels, dtype=np.int64)
    V, d = W_bits.shape
    n = np.bincount(labels, minlength=C).astype(np.int64)
    perm = np.argsort(labels, kind="stable").astype(np.int64)
    off = np.concatenate([[0], np.cumsum(n)])
    mu = np.zeros((C, d), dtype=np.float32)
    R = np.zeros(C, dtype=np.float64)
    bmax = np.full(C, -np.inf, dtype=np.float32)
    bb = None if b is None else np.asarray(b, dtype=np.float32)
    for c in range(C):
        rows = perm[off[c]:off[c + 1]]
        if rows.size == 0:
            continue
        Wc = bf16_to_f64(W_bits[rows])
        mu[c] = Wc.mean(axis=0).astype(np.float32)
        if centroid_bf16:
            mu[c] = _round_bf16(mu[c])
        diff = Wc - mu[c].astype(np.float64)[None, :]
        R[c] = math.sqrt(float(np.max(np.einsum("ij,ij->i", diff, diff))))
        bmax[c] = np.float32(0.0) if bb is None else bb[rows].max()
    mun = np.sqrt(np.einsum("ij,ij->i", mu.astype(np.float64), mu.astype(np.float64)))
    Rt = _round_up_f32(R * (1.0 + radius_slack) + radius_slack * mun)
    Rt[n == 0] = 0.0
    table = None
    if bias_table_m >= 2:
        table = bias_table(W_bits, bb, mu, n, perm, bias_table_m, radius_slack)
    return OracleIndex(mu, Rt, bmax, n, perm, table)


def bias_table(W_bits: np.ndarray, bb, mu: np.ndarray, n: np.ndarray, perm: np.ndarray, m: int,
               radius_slack: float) -> np.ndarray:
    """Top-m bias table of a cluster (Section III, "Advanced Theoretical Improvements": bias binning).

    The bound of Eq. "cluster_bound" charges every token of a cluster with the largest radius AND the largest bias,
    which is loose when one token has an outlying bias.  Reading used here: the m-1 tokens with the largest biases
    (equal biases: smaller token id first) are bounded one by one, each with its own distance to the centroid and its
    own bias, <W_i,h> + b_i <= <mu_c,h> + ||W_i - mu_c|| ||h|| + b_i (the Cauchy-Schwarz step of Section III-A for
    that token alone); all other tokens of the cluster share the largest radius and the largest bias among THEM.
    The cluster bound is the largest of these m bounds:
        U_c(h) = <mu_c,h> + max_j (rho_j ||h|| + beta_j).
    Every token is covered by one of the m terms, so Theorems 1 and 2 hold unchanged; no term exceeds
    R_c ||h|| + max_i b_i, so the bound is never looser; m = 1 is Eq. "cluster_bound" itself.
    Returns float32 [C, m, 2] = (rho_j, beta_j); radii get the same slack and upward rounding as R_c; entries a
    cluster does not need are (0, -inf)."""
    C = n.shape[0]
    off = np.concatenate([[0], np.cumsum(n)])
    out = np.zeros((C, m, 2), dtype=np.float32)
    out[:, :, 1] = -np.inf
    mun = np.sqrt(np.einsum("ij,ij->i", mu.astype(np.float64), mu.astype(np.float64)))
    for c in range(C):
        rows = perm[off[c]:off[c + 1]]                 # ascending token id
        if rows.size == 0:
            continue
        diff = bf16_to_f64(W_bits[rows]) - mu[c].astype(np.float64)[None, :]
        dist = np.sqrt(np.einsum("ij,ij->i", diff, diff))
        bias = np.zeros(rows.size, dtype=np.float32) if bb is None else bb[rows]
        order = np.lexsort((rows, -bias.astype(np.float64)))      # bias descending, token id ascending
        ne = min(m - 1, rows.size)
        pick = order[:ne]
        rest = order[ne:]
        rho = list(dist[pick])
        beta = list(bias[pick])
        if rest.size:
            rho.append(dist[rest].max())
            beta.append(bias[rest].max())
        rho = _round_up_f32(np.array(rho) * (1.0 + radius_slack) + radius_slack * mun[c])
        out[c, :len(rho), 0] = rho
        out[c, :len(rho), 1] = np.array(beta, dtype=np.float32)
    return out


def lloyd_assign(W64: np.ndarray, cent64: np.ndarray) -> np.ndarray:
    """Nearest centroid in squared Euclidean distance; ties go to the smaller cluster id."""
    out = np.empty(W64.shape[0], dtype=np.int64)
    step = max(1, int(2e7) // (cent64.shape[0] * cent64.shape[1]))
    for lo in range(0, W64.shape[0], step):
        x = W64[lo:lo + step]
        d2 = ((x[:, None, :] - cent64[None, :, :]) ** 2).sum(-1)
        out[lo:lo + step] = np.argmin(d2, axis=1)      # argmin returns the first (smallest id) minimum
    return out


def _round_down_f32(x: np.ndarray) -> np.ndarray:
    x = np.asarray(x, dtype=np.float64)
    y = x.astype(np.float32)
    high = y.astype(np.float64) > x
    y[high] = np.nextafter(y[high], np.float32(-np.inf))
    return y


def build_index_angular(W_bits: np.ndarray, b, labels: np.ndarray, C: int, slack: float = 2.0 ** -14,
                        angle_slack: float = 2.0 ** -12) -> OracleIndex:
    """Angular index for spherical clustering (Section III, "Advanced Theoretical Improvements", spherical metrics).

    Per cluster: the unit centroid direction m_c = normalise(sum_i W_i / ||W_i||), stored as float32; the angular radius
    theta_c = max_i angle(W_i, m_c) measured to the STORED direction; the largest and smallest row norm.
    Stored with slack so that a float32 evaluation of the bound stays above the logits: theta_c + theta_c*slack +
    angle_slack (its cosine and sine are what is kept), the largest norm times (1 + slack) rounded up, the smallest
    times (1 - slack) rounded down.  Rows of zero norm count as having the centroid's own direction."""
    labels = np.asarray(labels, dtype=np.int64)
    V, d = W_bits.shape
    n = np.bincount(labels, minlength=C).astype(np.int64)
    perm = np.argsort(labels, kind="stable").astype(np.int64)
    off = np.concatenate([[0], np.cumsum(n)])
    mu = np.zeros((C, d), dtype=np.float32)
    ang = np.zeros((C, 4), dtype=np.float32)
    ang[:, 0] = 1.0
    bmax = np.full(C, -np.inf, dtype=np.float32)
    bb = None if b is None else np.asarray(b, dtype=np.float32)
    for c in range(C):
        rows = perm[off[c]:off[c + 1]]
        if rows.size == 0:
            continue
        Wc = bf16_to_f64(W_bits[rows])
        nrm = np.sqrt(np.einsum("ij,ij->i", Wc, Wc))
        unit = Wc / np.where(nrm > 0, nrm, 1.0)[:, None]
        m = unit.sum(axis=0)
        mn = math.sqrt(float(m @ m))
        mu[c] = (m / mn if mn > 0 else m).astype(np.float32)
        ms = mu[c].astype(np.float64)
        msn = math.sqrt(float(ms @ ms))
        cosv = np.where(nrm > 0, (Wc @ ms) / (np.where(nrm > 0, nrm, 1.0) * (msn if msn > 0 else 1.0)), 1.0)
        theta = math.acos(float(np.clip(cosv.min(), -1.0, 1.0)))
        theta = min(math.pi, theta * (1.0 + slack) + angle_slack)
        ang[c, 0] = _round_down_f32(np.array([math.cos(theta)]))[0] if theta < math.pi else np.float32(-1.0)
        ang[c, 1] = _round_up_f32(np.array([math.sin(theta)]))[0]
        ang[c, 2] = _round_up_f32(np.array([nrm.max() * (1.0 + slack)]))[0]
        ang[c, 3] = _round_down_f32(np.array([nrm.min() * (1.0 - slack)]))[0]
        bmax[c] = np.float32(0.0) if bb is None else bb[rows].max()
    return OracleIndex(mu, np.zeros(C, dtype=np.float32), bmax, n, perm, None, ang)


def angular_bounds(index: OracleIndex, h64: np.ndarray):
    """Angular cluster bound.  For a row w of cluster c, angle(w,h) >= phi - theta_c with phi = angle(m_c,h), so
        <w,h> <= ||w|| ||h|| cos(phi - theta_c)          when phi > theta_c,        <w,h> <= ||w|| ||h||  otherwise,
    and with t = <m_c,h> = ||h|| cos(phi):  ||h|| cos(phi - theta_c) = t cos(theta_c) + sqrt(||h||^2 - t^2) sin(theta_c).
    The row norm is replaced by the cluster's largest (when that factor is positive) or smallest (when negative).
    The paper prints ||h|| (||mu_c|| cos(theta_c) + sin(theta_c)), which does not depend on the direction of h and so
    cannot order clusters; it follows from the form used here with cos(phi) and sin(phi) replaced by 1."""
    h64 = np.atleast_2d(h64)
    hn = np.sqrt(np.einsum("ij,ij->i", h64, h64))
    t = h64 @ index.mu.astype(np.float64).T                       # [B,C]
    a = index.ang.astype(np.float64)
    ct, st, rmax, rmin = a[:, 0][None, :], a[:, 1][None, :], a[:, 2][None, :], a[:, 3][None, :]
    perp = np.sqrt(np.maximum(hn[:, None] ** 2 - t ** 2, 0.0))
    inside = t >= hn[:, None] * ct                                # phi <= theta_c: the cone contains the direction of h
    g = t * ct + perp * st
    val = np.where(inside, rmax * hn[:, None], np.where(g >= 0, rmax * g, rmin * g))
    U = val + index.bmax.astype(np.float64)[None, :]
    U[:, index.n == 0] = NEG_INF
    return U, hn


def spherical_assign(W64: np.ndarray, dirs64: np.ndarray) -> np.ndarray:
    """Largest cosine to a unit direction (rows of zero norm go to cluster 0); ties go to the smaller cluster id."""
    out = np.empty(W64.shape[0], dtype=np.int64)
    nrm = np.sqrt(np.einsum("ij,ij->i", W64, W64))
    step = max(1, int(2e7) // max(1, dirs64.shape[0]))
    for lo in range(0, W64.shape[0], step):
        x = W64[lo:lo + step]
        cosv = (x @ dirs64.T) / np.where(nrm[lo:lo + step] > 0, nrm[lo:lo + step], 1.0)[:, None]
        out[lo:lo + step] = np.argmax(cosv, axis=1)             # argmax returns the first (smallest id) maximum
    return out


def spherical_kmeans(W_bits: np.ndarray, init_rows: np.ndarray, iters: int):
    """Spherical K-means (Section III, spherical clustering metrics): directions start at the given rows (normalised);
    each iteration assigns every row to the direction of largest cosine and replaces each direction by the
    float32-rounded normalised sum of its rows' unit vectors (an empty cluster keeps its direction)."""
    W64 = bf16_to_f64(W_bits)
    nrm = np.sqrt(np.einsum("ij,ij->i", W64, W64))
    unit = W64 / np.where(nrm > 0, nrm, 1.0)[:, None]
    dirs = unit[np.asarray(init_rows, dtype=np.int64)].astype(np.float32)
    labels = spherical_assign(W64, dirs.astype(np.float64))
    for _ in range(iters):
        for c in range(dirs.shape[0]):
            m = labels == c
            if m.any():
                v = unit[m].sum(axis=0)
                vn = math.sqrt(float(v @ v))
                dirs[c] = (v / vn if vn > 0 else v).astype(np.float32)
        labels = spherical_assign(W64, dirs.astype(np.float64))
    return labels, dirs


def strided_seed_rows(V: int, C: int) -> np.ndarray:
    """Seeding rule used when the caller names no starting rows: C tokens evenly spread over the vocabulary,
    token floor(c V / C) for cluster c (the paper leaves the seeding of its K-means to a library)."""
    return (np.arange(C, dtype=np.int64) * V) // C


def lloyd_kmeans(W_bits: np.ndarray, init_rows: np.ndarray, iters: int):
    """Plain Lloyd iteration (Section III-A.1: K-means over the rows of W).

    Centroids start at the given rows; each iteration assigns every row to its nearest centroid and
    replaces each centroid by the float32-rounded mean of its rows (an empty cluster keeps its centroid).
    Returns (labels after the last assignment, float32 centroids used for that assignment).
    """
    W64 = bf16_to_f64(W_bits)
    cent = W64[np.asarray(init_rows, dtype=np.int64)].astype(np.float32)
    labels = lloyd_assign(W64, cent.astype(np.float64))
    for _ in range(iters):
        for c in range(cent.shape[0]):
            m = labels == c
            if m.any():
                cent[c] = W64[m].mean(axis=0).astype(np.float32)
        labels = lloyd_assign(W64, cent.astype(np.float64))
    return labels, cent


# ----------------------------------------------------------------------------- bounds
def cluster_bounds(index: OracleIndex, h64: np.ndarray):
    """U_c(h) = <mu_c,h> + R_c ||h||_2 + max_{i in c} b_i  (Eq. "cluster_bound"); with a top-m bias table the last
    two terms are replaced by max_j (rho_j ||h|| + beta_j).  Empty clusters get -inf."""
    h64 = np.atleast_2d(h64)
    if index.ang is not None:
        return angular_bounds(index, h64)
    hn = np.sqrt(np.einsum("ij,ij->i", h64, h64))
    dots = h64 @ index.mu.astype(np.float64).T
    if index.bias_table is None:
        U = dots + hn[:, None] * index.R.astype(np.float64)[None, :] + index.bmax.astype(np.float64)[None, :]
    else:       # top-m bias table: the largest of the m (radius, bias) terms of each cluster, see bias_table()
        t = index.bias_table.astype(np.float64)
        U = dots + np.max(hn[:, None, None] * t[None, :, :, 0] + t[None, :, :, 1], axis=2)
    U[:, index.n == 0] = NEG_INF
    return U, hn


def cluster_order(U_row: np.ndarray) -> np.ndarray:
    """Clusters by descending bound; equal bounds -> smaller cluster id first."""
    return np.lexsort((np.arange(U_row.shape[0]), -U_row))


def _lam(eps: float) -> float:
    """ln(eps/(1-eps)): R-hat/(e^Z + R-hat) <= eps  <=>  log R-hat - Z <= ln(eps/(1-eps))."""
    if eps >= 1.0:
        return math.inf
    if eps <= 0.0:
        return NEG_INF
    return math.log(eps / (1.0 - eps))


def tail_log_mass(index: OracleIndex, U_row: np.ndarray, order: np.ndarray) -> np.ndarray:
    """T[m] = log sum_{j>m} n_{o(j)} exp(U_{o(j)}), m = 0..C: log of the cluster-wise tail bound R-hat
    of Theorem 2's proof when the first m clusters of the order are open.  T[C] = -inf."""
    C = order.shape[0]
    with np.errstate(divide="ignore"):
        v = np.log(index.n[order].astype(np.float64)) + U_row[order]
    T = np.full(C + 1, NEG_INF)
    acc = NEG_INF
    for m in range(C - 1, -1, -1):
        acc = np.logaddexp(acc, v[m]) if v[m] != NEG_INF else acc
        T[m] = acc
    return T


def _kth_largest(vals: np.ndarray, k: int) -> float:
    if k <= 0 or vals.size < k:
        return NEG_INF
    return float(np.sort(vals)[::-1][k - 1])


# ----------------------------------------------------------------------------- minimal certifying prefix (Algorithm 1)
def prefix_certificates(index: OracleIndex, U_row: np.ndarray, logits_row: np.ndarray, opened: np.ndarray, k: int,
                        eps: float):
    """Both certificates for the open set `opened` (cluster ids), straight from their definitions.

    Definition 1: the top-k of S is certified when every unopened non-empty cluster's bound lies strictly below the
    k-th largest logit of S (S must hold at least k rows).  Theorem 2, with the cluster-wise tail of its proof:
    R-hat = sum over unopened clusters of n_c e^{U_c}; certified when R-hat / (e^{Z_S} + R-hat) <= eps, evaluated in
    the log domain as log R-hat - Z_S <= ln(eps / (1 - eps)) (S must be non-empty).  With nothing left unopened both hold.
    Returns (topk_ok, softmax_ok, k-th largest logit of S, Z_S)."""
    mask = index.n > 0
    mask[np.asarray(opened, dtype=np.int64)] = False
    rest = np.flatnonzero(mask)
    rows = np.concatenate([index.rows(c) for c in opened]) if len(opened) else np.empty(0, dtype=np.int64)
    vals = logits_row[rows]
    theta = _kth_largest(vals, k) if k >= 1 else NEG_INF
    Z = logsumexp(vals)
    if rest.size == 0:
        return True, True, theta, Z
    tk = bool(vals.size >= k and np.max(U_row[rest]) < theta)
    log_Rhat = logsumexp(np.log(index.n[rest].astype(np.float64)) + U_row[rest])
    sm = bool(vals.size > 0 and log_Rhat - Z <= _lam(eps))
    return tk, sm, theta, Z


def alg1_step(index: OracleIndex, U_row: np.ndarray, logits_row: np.ndarray, k: int, eps: float,
              K_max: int, combine: int = COMBINE_ANY) -> dict:
    """What Algorithm 1 returns for one decoding step: the shortest prefix of the bound order that certifies.

    Clusters are opened in descending bound order (equal bounds: smaller id first; empty clusters are never queued).
    The result is the smallest m such that the first m clusters satisfy the stopping rule of Section III-C - under
    combine=ANY either certificate (Algorithm 1 stops on the first that holds), under combine=ALL every enabled one -
    unless a prefix on the way holds more than K_max rows, in which case the step falls back to the full vocabulary
    (Algorithm 1 tests the budget after each opening).  logits_row holds the exact logits by ORIGINAL token id;
    scoring a cluster means reading its rows' entries."""
    order = cluster_order(U_row)
    order = order[index.n[order] > 0]
    use_k, use_s = k >= 1, eps > 0
    P = np.concatenate([[0], np.cumsum(index.n[order])])
    for m in range(order.shape[0] + 1):
        if m > 0 and P[m] > K_max:
            return {"fallback": True, "opened": m, "n_rows": int(P[m])}
        tk, sm, theta, Z = prefix_certificates(index, U_row, logits_row, order[:m], k, eps)
        tk_ok = tk if use_k else (combine == COMBINE_ALL)
        sm_ok = sm if use_s else (combine == COMBINE_ALL)
        if (tk_ok and sm_ok) if combine == COMBINE_ALL else (tk_ok or sm_ok):
            return {"fallback": False, "opened": m, "n_rows": int(P[m]), "topk_cert": tk, "soft_cert": sm,
                    "clusters": order[:m].copy(), "theta": theta, "Z": Z}
    raise AssertionError("with every cluster open both certificates hold")


# ----------------------------------------------------------------------------- two-round schedule
def csv2r_step(index: OracleIndex, U_row: np.ndarray, logits_row: np.ndarray, k: int, eps: float,
               K_max: int, combine: int = COMBINE_ALL, max_rounds: int = 2, delta_clusters: int = 0,
               relax: bool = False) -> dict:
    """Round-based batched schedule of Algorithm 1 (the selection rule the GPU path is graded on).

    The same two tests as Algorithm 1, evaluated only at round boundaries:
      round 0  open the shortest prefix of the bound order holding >= max(k,1) rows; theta0 = k-th largest
               scored logit, Z0 = log-sum-exp of scored logits; test both certificates.
      round 1  a = number of clusters with U_c >= theta0 (all that could still reach the top-k, Definition 1);
               s = shortest prefix >= m0 whose tail satisfies Theorem 2 against Z0;
               open up to max(a,s) (ALL) or min(a,s) (ANY); test again.
    The budget |S| > K_max is tested on the planned size before scoring; failing tests after round 1 -> fallback.

    With the defaults that is the whole schedule.  The three fallback levels of Section IV ("Runtime
    Optimization") extend it:
      max_rounds      scoring rounds allowed (>= 2); every later round plans exactly as round 1 does, from the
                      theta and Z of the rows scored so far;
      delta_clusters  partial expansion S' = S + Delta C: when a planned set exceeds K_max, open instead the next
                      clusters of the bound order - at most delta_clusters of them, not past the planned set, and
                      only while the rows stay within K_max - and test again (theta and Z grow, so the next plan
                      may fit); 0 switches the level off;
      relax           relaxed tolerance eps' = 2 eps: when no further expansion is possible, the step is accepted
                      if the softmax tail bound holds at 2 eps (flag SOFTMAX_RELAXED instead of SOFTMAX_CERT);
    and the full vocabulary remains the last level.
    Returns decisions, outputs and, for every comparison that decided something, the pair
    (|x - y|, max(1,|x|,|y|)) under "margins" (tie-band accounting in parity tests).
    """
    C = index.C
    order = cluster_order(U_row)
    su = U_row[order]
    P = np.concatenate([[0], np.cumsum(index.n[order])])          # P[m] rows in first m clusters
    T = tail_log_mass(index, U_row, order)
    lam = _lam(eps)
    use_k, use_s = k >= 1, eps > 0
    if not (use_k or use_s):
        raise ValueError("both certificates disabled")
    margins: dict[str, tuple] = {}

    def gap(x, y):
        x, y = float(x), float(y)
        return (abs(x - y), max(1.0, abs(x), abs(y)))

    def gap_soft(t, z):            # T - Z against lam: the rounding scale is that of T and Z themselves
        return (abs(float(t) - z - lam), max(1.0, abs(float(t)), abs(z), abs(lam)))

    def result(flags, m, rounds, ids, vals, Z, theta):
        return {"flags": flags, "fallback": bool(flags & FLAG_FALLBACK), "m0": m0, "m1": m, "rounds": rounds,
                "n_rows": int(P[m]) if not flags & FLAG_FALLBACK else index.V,
                "n_clusters": int(m) if not flags & FLAG_FALLBACK else C,
                "clusters": order[:m].copy(), "order": order, "ids": ids, "logits": vals, "lse": Z,
                "theta": theta, "margins": margins}

    def fallback(m, rounds):
        ids, vals = topk_bruteforce(logits_row, k)
        f = FLAG_FALLBACK | FLAG_TOPK_CERT | FLAG_SOFTMAX_CERT
        if vals.size > k - 1 and logits_row.size > k >= 1:
            srt = np.sort(logits_row)[::-1]
            margins["id_gap"] = gap(srt[k - 1], srt[k])
        return result(f, m, rounds, ids, vals, logsumexp(logits_row), float(vals[-1]) if k >= 1 else NEG_INF)

    def score(m):
        rows = index.perm[:0] if m == 0 else np.concatenate([index.rows(c) for c in order[:m]])
        vals = logits_row[rows]
        ids, top = topk_bruteforce(vals, k, rows)
        theta = float(top[-1]) if use_k else NEG_INF
        return rows, vals, ids, top, theta, logsumexp(vals)

    def tests(m, theta, Z, tag):
        if m == C or su[m] == NEG_INF:
            tk = True
        else:
            tk = bool(su[m] < theta)
            if use_k:
                margins["tk" + tag] = gap(su[m], theta)
        sm = bool(T[m] - Z <= lam)
        if use_s and math.isfinite(T[m]) and math.isfinite(lam):
            margins["sm" + tag] = gap_soft(T[m], Z)
        return tk, sm

    def combine_ok(tk, sm):
        if combine == COMBINE_ALL:
            return (tk or not use_k) and (sm or not use_s)
        return (tk and use_k) or (sm and use_s)

    need = max(k, 1)
    m0 = int(np.searchsorted(P, need, side="left"))              # min m with P[m] >= need
    if m0 < C and su[m0] != NEG_INF:
        margins["seed"] = gap(su[m0 - 1], su[m0])
    if P[m0] > K_max:
        return fallback(m0, 0)
    lam2 = _lam(2.0 * eps) if use_s else NEG_INF
    if max_rounds < 2:
        raise ValueError("max_rounds must be at least 2")
    m, r, theta_prev, Z_prev = m0, 0, NEG_INF, NEG_INF
    m_plan = m0
    while True:
        tag = str(r)
        rows, vals, ids, top, theta, Z = score(m)
        assert theta >= theta_prev and Z >= Z_prev          # both only grow with S
        theta_prev, Z_prev = theta, Z
        tk, sm = tests(m, theta, Z, tag)
        if combine_ok(tk, sm):
            f = (FLAG_TOPK_CERT if tk and use_k else 0) | (FLAG_SOFTMAX_CERT if sm and use_s else 0)
            _id_margin(margins, vals, k)
            return result(f, m, r + 1, ids, top, Z, theta)
        if r + 1 >= max_rounds:
            break
        # target of the next round
        if tk or not use_k:
            a = m
        else:
            a = int(np.sum(su >= theta))
            fin = su[np.isfinite(su)]
            near = fin[np.argmin(np.abs(fin - theta))]
            margins["a" + ("" if r == 0 else tag)] = gap(near, theta)
        if sm or not use_s:
            sp = m
        else:
            sp = m + int(np.argmax(T[m:] - Z <= lam))
            sfx = "" if r == 0 else tag
            if math.isfinite(T[sp]):
                margins["s_hi" + sfx] = gap_soft(T[sp], Z)
            margins["s_lo" + sfx] = gap_soft(T[sp - 1], Z)
            if sp < C and su[sp] != NEG_INF:
                margins["s_order" + sfx] = gap(su[sp - 1], su[sp])
        cands = ([a] if use_k else []) + ([sp] if use_s else [])
        m_plan = max(cands) if combine == COMBINE_ALL else min(cands)
        if 0 < m_plan < C and su[m_plan] != NEG_INF:
            margins["m1_order" + ("" if r == 0 else tag)] = gap(su[m_plan - 1], su[m_plan])
        if P[m_plan] <= K_max:
            m_next = m_plan
        else:
            m_next = m
            while m_next < min(m + max(delta_clusters, 0), m_plan) and P[m_next + 1] <= K_max:
                m_next += 1
            if m_next == m:
                break
            if su[m_next] != NEG_INF and m_next < C:
                margins["mp_order" + tag] = gap(su[m_next - 1], su[m_next])
        m = m_next
        r += 1
    # no further expansion: relaxed tolerance, else the full vocabulary
    if relax and use_s:
        sm2 = bool(T[m] - Z <= lam2)
        if math.isfinite(T[m]) and math.isfinite(lam2):
            margins["sm_relaxed"] = (abs(float(T[m]) - Z - lam2), max(1.0, abs(float(T[m])), abs(Z), abs(lam2)))
        if combine_ok(tk, sm2):
            f = (FLAG_TOPK_CERT if tk and use_k else 0) | (FLAG_SOFTMAX_CERT if sm else (FLAG_SOFTMAX_RELAXED if sm2 else 0))
            _id_margin(margins, vals, k)
            return result(f, m, r + 1, ids, top, Z, theta)
    return fallback(max(m, m_plan), r + 1)


def _id_margin(margins: dict, vals: np.ndarray, k: int) -> None:
    if k >= 1 and vals.size > k:
        srt = np.sort(vals)[::-1]
        x, y = float(srt[k - 1]), float(srt[k])
        margins["id_gap"] = (x - y, max(1.0, abs(x), abs(y)))


# ----------------------------------------------------------------------------- one batch step
def decode_step(W64: np.ndarray, b, index: OracleIndex, h_bits: np.ndarray, k: int, eps: float, K_max: int,
                combine: int = COMBINE_ALL, logits: np.ndarray | None = None, max_rounds: int = 2,
                delta_clusters: int = 0, relax: bool = False) -> list:
    """All sequences of one batch step.  Full logits are formed once by definition; the selection
    rule then reads the entries of the rows it opens (identical to scoring those rows alone)."""
    h64 = bf16_to_f64(np.atleast_2d(h_bits))
    if logits is None:
        logits = full_logits(W64, b, h64)
    U, hn = cluster_bounds(index, h64)
    out = []
    for s in range(h64.shape[0]):
        if not np.isfinite(hn[s]):
            out.append({"flags": FLAG_INVALID, "fallback": False})
            continue
        r = csv2r_step(index, U[s], logits[s], k, eps, K_max, combine, max_rounds, delta_clusters, relax)
        r["U"] = U[s]
        r["hnorm"] = hn[s]
        out.append(r)
    return out


# ----------------------------------------------------------------------------- top-p (nucleus) form
def nucleus_eps(delta: float) -> float:
    """Top-p certification (Section III, "Advanced Theoretical Improvements"): when the unopened clusters satisfy
    sum_c n_c e^{U_c} <= delta e^{Z_S}, the probability mass outside S is at most delta / (1 + delta).  That is the
    softmax test of Theorem 2 read with eps = delta / (1 + delta), since ln(eps / (1 - eps)) = ln(delta): a step
    run with this eps carries the top-p coverage certificate 1 - eps; the stopping rule delta <= eps / (1 - eps)
    is the same statement solved for delta."""
    return delta / (1.0 + delta)


def certified_distribution(logits: np.ndarray, lse: float, top_p: float = 0.0):
    """Sub-vocabulary distribution over a returned list (Section III, top-p certification): p~_t = exp(l_t - Z_S) in
    list order, its running sums, and the length of the shortest prefix whose running sum reaches top_p (0 when
    top_p is 0 or the list ends first).  With the eps-softmax certificate at most eps of the mass lies outside S, so
    the full-vocabulary probability of token t is within [(1 - eps) p~_t, p~_t] and a prefix with running sum >= top_p
    covers at least (1 - eps) top_p of the full-vocabulary mass."""
    p = np.exp(np.asarray(logits, dtype=np.float64) - lse)
    cum = np.cumsum(p)
    nucleus = 0
    if top_p > 0:
        hit = np.flatnonzero(cum >= top_p)
        nucleus = int(hit[0]) + 1 if hit.size else 0
    return p, cum, nucleus


def nucleus_holds(index: OracleIndex, U_row: np.ndarray, opened: np.ndarray, Z_S: float, delta: float) -> bool:
    """The delta-form written out: sum over unopened, non-empty clusters of n_c e^{U_c} <= delta e^{Z_S}."""
    mask = np.ones(index.C, dtype=bool)
    mask[np.asarray(opened, dtype=np.int64)] = False
    mask &= index.n > 0
    if not mask.any():
        return True
    terms = np.log(index.n[mask].astype(np.float64)) + U_row[mask].astype(np.float64)
    return bool(logsumexp(terms) <= math.log(delta) + Z_S)


# ----------------------------------------------------------------------------- adaptive budget
def kmax_update(K_max: float, rho_fall: float, alpha: float = 0.01, rho_target: float = 0.02,
                literal: bool = False) -> float:
    """One update of the row budget from the fallback rate of the step just taken (Section IV, "Runtime
    Optimization": K_max(t+1) = K_max(t) (1 + alpha (rho_target - rho_fall(t))), alpha = 0.01, target 0.02).

    As printed the factor shrinks the budget when fallbacks are above the target, which drives the rate away from
    the target it is said to maintain (a larger budget means fewer fallbacks).  literal=True evaluates the printed
    expression; the default takes the sign that makes the update a negative feedback,
    K_max (1 + alpha (rho_fall - rho_target)).  The value is returned unrounded and unclamped."""
    err = (rho_target - rho_fall) if literal else (rho_fall - rho_target)
    return K_max * (1.0 + alpha * err)


def kmax_rows(K_max: float, K_min: int, K_cap: int) -> int:
    """Row budget handed to a step: the controller's value rounded down and kept inside [K_min, K_cap]."""
    return int(min(max(math.floor(K_max), K_min), K_cap))
