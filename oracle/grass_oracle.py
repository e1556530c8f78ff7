"""Plain CPU oracle for per-sample gradient compression (GraSS / FactGraSS).

TEST INFRASTRUCTURE ONLY: a slow, obviously-correct NumPy float64 statement of
what the compression path computes, written from the paper.  It shares no code
with the HIP kernels and must never be imported by the product package.

Every function cites the passage of the paper it follows.  Where the paper
leaves a choice to the implementer (which random generator, how ties and
orders are resolved, normalisation) the choice is stated in the docstring as a
"reading"; the same readings bind the GPU path.

Pins (see tests/test_oracle_*.py): published splitmix64 outputs; brute force
on tiny inputs; an explicitly materialised dense projection matrix; linearity;
the Kronecker/vec identity of Eq. (2)/(3); closed-form first and second
moments of the count-sketch norm; limits k'=p and k'=k of Sec. 3.3.1; the
Gaussian matrix against the normal distribution (Kolmogorov-Smirnov, moments)
and the norm-preservation property of Sec. 2.2.
Parity unpinned: absolute output values (the paper prints no worked example).
"""
from __future__ import annotations

import numpy as np

# ----------------------------------------------------------------------------
# Counter-based random numbers.
#
# Reading (the paper only says indices and signs are "sampled", App. B.4.1):
# all randomness comes from the splitmix64 generator (Steele, Lea, Flood,
# "Fast splittable pseudorandom number generators", OOPSLA 2014; the constants
# are those of the public-domain reference).  Its n-th output depends only on
# seed + (n+1)*gamma, so any output can be computed without the earlier ones.
# ----------------------------------------------------------------------------
_U64 = np.uint64
GOLDEN_GAMMA = _U64(0x9E3779B97F4A7C15)
_MUL_A = _U64(0xBF58476D1CE4E5B9)
_MUL_B = _U64(0x94D049BB133111EB)


def _as_u64(a):
    return np.atleast_1d(np.asarray(a, dtype=np.uint64))


def _finalise(z):
    """The splitmix64 output function (two xor-shift-multiply rounds and a
    final xor-shift), on a uint64 array, arithmetic modulo 2**64."""
    with np.errstate(over="ignore"):
        z = (z ^ (z >> _U64(30))) * _MUL_A
        z = (z ^ (z >> _U64(27))) * _MUL_B
        return z ^ (z >> _U64(31))


def splitmix64_sequence(seed: int, count: int) -> np.ndarray:
    """First `count` outputs of the sequential splitmix64 generator whose
    state starts at `seed`: state += gamma; output = finalise(state)."""
    out = np.empty(count, dtype=np.uint64)
    state = _as_u64(seed).copy()
    with np.errstate(over="ignore"):
        for i in range(count):
            state = state + GOLDEN_GAMMA
            out[i] = _finalise(state)[0]
    return out


def sm(seed, counter) -> np.ndarray:
    """Counter form: the `counter`-th (0-based) output of splitmix64 seeded
    with `seed`, i.e. finalise(seed + (counter+1)*gamma)."""
    seed = _as_u64(seed)
    counter = _as_u64(counter)
    with np.errstate(over="ignore"):
        return _finalise(seed + (counter + _U64(1)) * GOLDEN_GAMMA)


def stream_hash(seed: int, stream: int, counter) -> np.ndarray:
    """H(seed, stream, c) = sm(sm(seed, stream), c): an independent
    sub-generator per `stream` id (mask, SJLT, per-layer roles)."""
    sub = sm(seed, stream)[0]
    return sm(sub, counter)


# Stream ids (a reading; the paper names no generator).  General vectors use
# 0 for the mask and 1 for the SJLT; linear layer l uses 16+4l (input mask),
# 17+4l (output-gradient mask) and 18+4l (SJLT).
STREAM_MASK = 0
STREAM_SJLT = 1


def layer_streams(layer: int):
    return 16 + 4 * layer, 17 + 4 * layer, 18 + 4 * layer


# ----------------------------------------------------------------------------
# Random Mask (Sec. 3.2, "Random Mask"): a random subset of k' of the p
# coordinates; as a matrix, a binary selection matrix with one non-repeating
# non-zero per row.
# ----------------------------------------------------------------------------
def mask_indices(seed: int, stream: int, p: int, kprime: int) -> np.ndarray:
    """Indices kept by the Random Mask, ascending, int32.

    Reading: coordinate j draws key_j = H(seed, stream, j); the k' coordinates
    with the smallest (key_j, j) pairs are kept (ties on the key go to the
    smaller j), reported in ascending order of j.  This is a uniform draw
    without replacement, independent of any evaluation order, and k' = p
    returns 0..p-1 (the GraSS -> SJLT limit of Sec. 3.3.1).
    """
    if not (0 < kprime <= p):
        raise ValueError("need 0 < k' <= p")
    j = np.arange(p, dtype=np.uint64)
    key = stream_hash(seed, stream, j)
    order = np.lexsort((j, key))          # primary key, secondary j
    kept = np.sort(order[:kprime])
    return kept.astype(np.int32)


def mask(g: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """Mask_k'(g) = M g: the sub-vector g[idx] of every row (Sec. 3.2).  No
    rescaling is applied: the paper's M is binary."""
    g = np.asarray(g)
    return g[..., np.asarray(idx, dtype=np.int64)]


# ----------------------------------------------------------------------------
# SJLT (Sec. 3.1, "Sparse Johnson-Lindenstrauss Transform"): P has s non-zero
# +-1 entries per column; equivalently scan g and let each g(j) add itself to,
# or subtract itself from, s chosen output coordinates.
# ----------------------------------------------------------------------------
def sjlt_tables(seed: int, stream: int, d: int, k: int, s: int):
    """bucket[j, r] in [0, k) and sign[j, r] in {+1, -1} for input position j
    and r in [0, s).

    Reading (block construction of the sparser-JL paper the text cites): s
    divides k, m = k/s, and the r-th non-zero of column j falls in block r:
        h      = H(seed, stream, j*s + r)
        bucket = r*m + floor((h >> 32) * m / 2**32)
        sign   = +1 if the lowest bit of h is 0, else -1
    so that every column has exactly s non-zeros in distinct rows.
    """
    return sjlt_entries(seed, stream, np.arange(d, dtype=np.uint64), k, s)


def sjlt_entries(seed: int, stream: int, positions, k: int, s: int):
    """The rows of `sjlt_tables` for the given input positions only (any
    order, any subset): bucket[q, r], sign[q, r] of position positions[q]."""
    if s <= 0 or k <= 0 or k % s:
        raise ValueError("need s >= 1 dividing k")
    m = k // s
    j = _as_u64(positions).reshape(-1)
    c = j[:, None] * _U64(s) + np.arange(s, dtype=np.uint64)[None, :]
    h = stream_hash(seed, stream, c.reshape(-1)).reshape(j.size, s)
    hi = h >> _U64(32)
    within = (hi * _U64(m)) >> _U64(32)                      # < m, no overflow: hi, m < 2**32
    bucket = within + (np.arange(s, dtype=np.uint64) * _U64(m))[None, :]
    sign = np.where((h & _U64(1)) == 0, 1, -1).astype(np.int8)
    return bucket.astype(np.uint32), sign


def sjlt_scan(g_row, bucket, sign, k: int) -> np.ndarray:
    """The scan of Sec. 3.1 written out for one vector: start from zero, visit
    j = 0..d-1, add sign*g(j)/sqrt(s) to each of its s buckets.  Pure Python:
    small inputs only."""
    d, s = bucket.shape
    out = [0.0] * k
    scale = 1.0 / np.sqrt(float(s))
    for j in range(d):
        v = float(g_row[j])
        for r in range(s):
            out[int(bucket[j, r])] += float(sign[j, r]) * v * scale
    return np.asarray(out, dtype=np.float64)


def sjlt(g: np.ndarray, k: int, s: int, seed: int, stream: int = STREAM_SJLT) -> np.ndarray:
    """SJLT_k of every row of g (n x d) -> n x k float64, scale 1/sqrt(s) so
    that squared norms are preserved in expectation.  Same scan as
    `sjlt_scan`, carried out by NumPy's in-order unbuffered add."""
    g = np.asarray(g, dtype=np.float64)
    if g.ndim == 1:
        return sjlt(g[None, :], k, s, seed, stream)[0]
    n, d = g.shape
    bucket, sign = sjlt_tables(seed, stream, d, k, s)
    out = np.zeros((n, k), dtype=np.float64)
    scale = 1.0 / np.sqrt(float(s))
    for i in range(n):
        for r in range(s):
            np.add.at(out[i], bucket[:, r], sign[:, r] * g[i] * scale)
    return out


def grass(g: np.ndarray, idx: np.ndarray, k: int, s: int, seed: int,
          stream: int = STREAM_SJLT) -> np.ndarray:
    """GraSS = SJLT_k o Mask_k' (Sec. 3.3.1): sparsify to g' = g[idx], then
    SJLT g'.  The SJLT sees only the k'-vector, so its hash key is the
    position inside g', not the original coordinate."""
    return sjlt(mask(g, idx), k, s, seed, stream)


# ----------------------------------------------------------------------------
# The compressors as explicit matrices (Sec. 3.1: P has s non-zeros +-1/sqrt(s)
# per column; Sec. 3.3.1: GraSS is the product of that matrix and the binary
# selection matrix of the mask).  Used for the factorised baselines of
# Sec. 3.3.2, where P_in and P_out of Eq. (3) may be any compressor.
# ----------------------------------------------------------------------------
def projection_matrix(seed: int, stream: int, p: int, k: int, s: int, idx=None) -> np.ndarray:
    """k x p matrix P with P g = sjlt(g) (idx None) or P g = grass(g, idx)."""
    cols = np.arange(p) if idx is None else np.asarray(idx, dtype=np.int64)
    bucket, sign = sjlt_tables(seed, stream, cols.size, k, s)
    P = np.zeros((k, p), dtype=np.float64)
    for jp in range(cols.size):
        for r in range(s):
            P[int(bucket[jp, r]), int(cols[jp])] += float(sign[jp, r]) / np.sqrt(float(s))
    return P


# ----------------------------------------------------------------------------
# FactGraSS (Sec. 3.3.2, "Factorized GraSS"; Eq. (2), Eq. (3)).
# ----------------------------------------------------------------------------
def factgrass_sparsified_gradient(x: np.ndarray, gout: np.ndarray,
                                  idx_in: np.ndarray, idx_out: np.ndarray) -> np.ndarray:
    """Stages 1 and 2: mask every token's layer input x_t (d_in) and
    pre-activation gradient g_t (d_out) separately, then sum over tokens the
    Kronecker products (masked x_t) (x) (masked g_t).  x is (n, T, d_in), gout
    is (n, T, d_out); returns n x (k_in' * k_out') with flat index
    a'*k_out' + b' -- the order Eq. (2) gives vec(DW)."""
    xs = np.asarray(x, dtype=np.float64)[..., np.asarray(idx_in, dtype=np.int64)]
    gs = np.asarray(gout, dtype=np.float64)[..., np.asarray(idx_out, dtype=np.int64)]
    n, T, ka = xs.shape
    kb = gs.shape[-1]
    v = np.zeros((n, ka * kb), dtype=np.float64)
    for i in range(n):
        for t in range(T):
            v[i] += np.kron(xs[i, t], gs[i, t])
    return v


def factgrass_linear(x, gout, idx_in, idx_out, k: int, s: int, seed: int, stream: int) -> np.ndarray:
    """FactGraSS for one linear layer: SJLT_k of the sparsified gradient; the
    layer gradient itself (d_out x d_in) is never formed."""
    v = factgrass_sparsified_gradient(x, gout, idx_in, idx_out)
    return sjlt(v, k, s, seed, stream)


# ----------------------------------------------------------------------------
# LoGra baseline (Sec. 3.3.2, "Recap on LoGra"; Eq. (3)): the factorised dense
# projection Gauss_{k_in (x) k_out} that FactGraSS is compared with.
# ----------------------------------------------------------------------------
def logra_linear(x: np.ndarray, gout: np.ndarray, P_in: np.ndarray, P_out: np.ndarray) -> np.ndarray:
    """out_i = sum_t (P_in x_t) (x) (P_out g_t) = (P_in (x) P_out) vec(DW_i), flat index a*k_out + b.
    x is (n, T, d_in), gout is (n, T, d_out), P_in is k_in x d_in, P_out is k_out x d_out (handed in as data)."""
    xs = np.asarray(x, dtype=np.float64)
    gs = np.asarray(gout, dtype=np.float64)
    Pi = np.asarray(P_in, dtype=np.float64)
    Po = np.asarray(P_out, dtype=np.float64)
    n, T, _ = xs.shape
    out = np.zeros((n, Pi.shape[0] * Po.shape[0]), dtype=np.float64)
    for i in range(n):
        for t in range(T):
            out[i] += np.kron(Pi @ xs[i, t], Po @ gs[i, t])
    return out


# ----------------------------------------------------------------------------
# Attribute stage (Sec. 2.1): all-pair inner products of compressed gradients,
# without a preconditioner (GradDot).
# ----------------------------------------------------------------------------
def score(train: np.ndarray, test: np.ndarray) -> np.ndarray:
    """scores[m, i] = <test_m, train_i>; train is N x K, test is M x K."""
    return np.asarray(test, dtype=np.float64) @ np.asarray(train, dtype=np.float64).T


# ----------------------------------------------------------------------------
# Cache stage after compression (Sec. 2.1 steps 2 and 3, applied to compressed
# gradients as in Sec. 2.2 / Sec. 3.3.2): the projected FIM of a block of k
# compressed coordinates and the inverse-FIM-vector product with the damping
# term of App. B ("damping lambda used for the Hessian/FIM inverse").
#
# Reading: the damped inverse is (F + lambda*I)^{-1} with lambda an absolute
# number (the grid of App. B lists absolute values); the paper prints F^{-1}
# only.  A block-diagonal FIM (Sec. 3.3.2) is this function applied to each
# layer's k_l columns separately.
# ----------------------------------------------------------------------------
def fim(G: np.ndarray) -> np.ndarray:
    """F = (1/n) sum_i g_i g_i^T for the rows g_i of G (n x k)."""
    G = np.asarray(G, dtype=np.float64)
    return G.T @ G / G.shape[0]


def ifvp(G: np.ndarray, F: np.ndarray, lam: float) -> np.ndarray:
    """Row i of the result is (F + lam*I)^{-1} g_i."""
    G = np.asarray(G, dtype=np.float64)
    F = np.asarray(F, dtype=np.float64)
    return np.linalg.solve(F + lam * np.eye(F.shape[0]), G.T).T


def influence(train: np.ndarray, test: np.ndarray, lam: float) -> np.ndarray:
    """I[m, i] = <test_m, (F + lam*I)^{-1} train_i> with F the FIM of the train rows (Sec. 2.1)."""
    return score(ifvp(train, fim(train), lam), test)


# ----------------------------------------------------------------------------
# Selective Mask (Sec. 3.2, Eq. (1); practical notes in App. B.4 "Selective
# Mask"): the mask logits S in R^p maximise the average, over test points, of
# the Pearson correlation between the exact GradDot scores <g_i, g_test> and
# the soft-masked ones <sigma(S) * g_i, sigma(S) * g_test>, minus
# lambda * ||sigma(S)||_1.  App. B.4 replaces S by S / T (inverse temperature).
#
# Readings: the expectation over test points is the mean over the rows handed
# in; corr is the Pearson correlation over the n training points with
# population (1/n) moments; ||sigma||_1 is the plain sum (sigma > 0).  The paper
# names no optimiser, step size or schedule: `selective_mask_train` is plain
# gradient ascent with a caller-supplied temperature per step.
# ----------------------------------------------------------------------------
def _sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def selective_mask_objective(S, G, Gt, lam: float, temperature: float = 1.0) -> float:
    """Eq. (1) for train rows G (n x p), test rows Gt (m x p) and logits S (p)."""
    S = np.asarray(S, dtype=np.float64)
    G = np.asarray(G, dtype=np.float64)
    Gt = np.asarray(Gt, dtype=np.float64)
    sig = _sigmoid(S / temperature)
    total = 0.0
    for t in range(Gt.shape[0]):
        exact = G @ Gt[t]                                  # <g_i, g_test>, i = 1..n
        masked = (G * sig) @ (Gt[t] * sig)                 # <sigma*g_i, sigma*g_test>
        da, db = exact - exact.mean(), masked - masked.mean()
        total += (da @ db) / np.sqrt((da @ da) * (db @ db))
    return total / Gt.shape[0] - lam * sig.sum()


def selective_mask_gradient(S, G, Gt, lam: float, temperature: float = 1.0) -> np.ndarray:
    """Gradient of selective_mask_objective with respect to S, by the chain rule:
    d corr / d masked_i = (da_i / (|da||db|) - corr * db_i / |db|^2), masked_i = sum_j sigma_j^2 G_ij Gt_j,
    d sigma_j / d S_j = sigma_j (1 - sigma_j) / T."""
    S = np.asarray(S, dtype=np.float64)
    G = np.asarray(G, dtype=np.float64)
    Gt = np.asarray(Gt, dtype=np.float64)
    sig = _sigmoid(S / temperature)
    dsig = sig * (1.0 - sig) / temperature
    grad_w = np.zeros_like(S)                              # with respect to w_j = sigma_j^2
    for t in range(Gt.shape[0]):
        exact = G @ Gt[t]
        masked = (G * sig) @ (Gt[t] * sig)
        da, db = exact - exact.mean(), masked - masked.mean()
        na, nb = np.sqrt(da @ da), np.sqrt(db @ db)
        corr = (da @ db) / (na * nb)
        c = da / (na * nb) - corr * db / (nb * nb)         # sums to zero, so centring needs no extra term
        grad_w += (c @ G) * Gt[t]
    grad_w /= Gt.shape[0]
    return grad_w * 2.0 * sig * dsig - lam * dsig


def selective_mask_factorized(S_in, S_out, Z_in, Z_out, Zt_in, Zt_out, lam: float, temperature: float = 1.0):
    """Factorised Selective Mask of a linear layer (App. B.4 "Linear Layer"): gradients are z_in (x) z_out, the mask is
    sigma(S_in) (x) sigma(S_out), the penalty lam * (|sigma(S_in)|_1 + |sigma(S_out)|_1), and every inner product of
    Kronecker products factorises, <a (x) b, c (x) d> = <a, c> <b, d>.  One token per sample, as in the paper's formula.
    Returns (objective, d objective / d S_in, d objective / d S_out)."""
    S_in, S_out = np.asarray(S_in, np.float64), np.asarray(S_out, np.float64)
    Z_in, Z_out = np.asarray(Z_in, np.float64), np.asarray(Z_out, np.float64)
    Zt_in, Zt_out = np.asarray(Zt_in, np.float64), np.asarray(Zt_out, np.float64)
    si, so = _sigmoid(S_in / temperature), _sigmoid(S_out / temperature)
    dsi, dso = si * (1 - si) / temperature, so * (1 - so) / temperature
    m = Zt_in.shape[0]
    total, gi, go = 0.0, np.zeros_like(S_in), np.zeros_like(S_out)
    for t in range(m):
        exact = (Z_in @ Zt_in[t]) * (Z_out @ Zt_out[t])
        b_in = (Z_in * si) @ (Zt_in[t] * si)
        b_out = (Z_out * so) @ (Zt_out[t] * so)
        masked = b_in * b_out
        da, db = exact - exact.mean(), masked - masked.mean()
        na, nb = np.sqrt(da @ da), np.sqrt(db @ db)
        corr = (da @ db) / (na * nb)
        total += corr
        c = da / (na * nb) - corr * db / (nb * nb)
        gi += ((c * b_out) @ Z_in) * Zt_in[t]              # d masked_i / d w_in_j = b_out_i Z_in[i, j] Zt_in[t, j]
        go += ((c * b_in) @ Z_out) * Zt_out[t]
    obj = total / m - lam * (si.sum() + so.sum())
    return obj, gi / m * 2 * si * dsi - lam * dsi, go / m * 2 * so * dso - lam * dso


def graddot_factorized_seq(X_in, X_out, Xt_in, Xt_out) -> np.ndarray:
    """Exact GradDot scores of a linear layer on sequences without forming the layer gradients: with per-sample
    gradients sum_t x_t (x) g_t (Eq. (2)) and <a (x) b, c (x) d> = <a, c> <b, d> (App. B.4 "Linear Layer"),
        score[test][i] = sum_{t, t'} <x_{i,t}, x_{test,t'}> <g_{i,t}, g_{test,t'}>.
    X_in (n, T, d_in), X_out (n, T, d_out) train; Xt_in (m, T', d_in), Xt_out (m, T', d_out) test.  Returns (m, n)."""
    X_in, X_out = np.asarray(X_in, np.float64), np.asarray(X_out, np.float64)
    Xt_in, Xt_out = np.asarray(Xt_in, np.float64), np.asarray(Xt_out, np.float64)
    m, n = Xt_in.shape[0], X_in.shape[0]
    out = np.zeros((m, n))
    for te in range(m):
        for i in range(n):
            k_in = X_in[i] @ Xt_in[te].T            # (T, T') token-pair inner products of the input factor
            k_out = X_out[i] @ Xt_out[te].T
            out[te, i] = np.sum(k_in * k_out)
    return out


def selective_mask_factorized_seq(S_in, S_out, X_in, X_out, Xt_in, Xt_out, lam: float, temperature: float = 1.0):
    """Factorised Selective Mask of a linear layer (App. B.4 "Linear Layer") for samples that are sequences of tokens.
    Reading: the paper writes the factorised problem for one token per sample; for T tokens the layer gradient is
    sum_t x_t (x) g_t (Eq. (2)), the mask sigma(S_in) (x) sigma(S_out) acts on it, and every inner product of two such
    gradients is the sum over all token pairs of the product of the two factors' (masked) inner products.
    Returns (objective, d objective / d S_in, d objective / d S_out)."""
    S_in, S_out = np.asarray(S_in, np.float64), np.asarray(S_out, np.float64)
    X_in, X_out = np.asarray(X_in, np.float64), np.asarray(X_out, np.float64)
    Xt_in, Xt_out = np.asarray(Xt_in, np.float64), np.asarray(Xt_out, np.float64)
    si, so = _sigmoid(S_in / temperature), _sigmoid(S_out / temperature)
    dsi, dso = si * (1 - si) / temperature, so * (1 - so) / temperature
    m, n = Xt_in.shape[0], X_in.shape[0]
    exact_all = graddot_factorized_seq(X_in, X_out, Xt_in, Xt_out)
    total, gi, go = 0.0, np.zeros_like(S_in), np.zeros_like(S_out)
    for te in range(m):
        masked = np.zeros(n)
        k_in, k_out = [], []
        for i in range(n):
            k_in.append((X_in[i] * si) @ (Xt_in[te] * si).T)        # (T, T'), weights sigma^2 in total
            k_out.append((X_out[i] * so) @ (Xt_out[te] * so).T)
            masked[i] = np.sum(k_in[i] * k_out[i])
        exact = exact_all[te]
        da, db = exact - exact.mean(), masked - masked.mean()
        na, nb = np.sqrt(da @ da), np.sqrt(db @ db)
        corr = (da @ db) / (na * nb)
        total += corr
        c = da / (na * nb) - corr * db / (nb * nb)
        for i in range(n):
            # d masked_i / d w_in_j = sum_{t,t'} k_out[t,t'] x_in[i,t,j] xt_in[te,t',j], w = sigma^2
            gi += c[i] * np.einsum("ab,aj,bj->j", k_out[i], X_in[i], Xt_in[te])
            go += c[i] * np.einsum("ab,aj,bj->j", k_in[i], X_out[i], Xt_out[te])
    obj = total / m - lam * (si.sum() + so.sum())
    return obj, gi / m * 2 * si * dsi - lam * dsi, go / m * 2 * so * dso - lam * dso


def selective_mask_train(S0, G, Gt, lam: float, lr: float, temperatures):
    """Solves Eq. (1) by first-order ascent on the logits, with the inverse-temperature annealing of App. B.4
    ("Ensuring Exact k": S is replaced by S / T and T decreases as training progresses).

    Reading: the paper names no optimiser, step size, batching or schedule.  Here every step is one plain gradient
    ascent step over all train and test rows handed in,
        S_{i+1} = S_i + lr * grad L(S_i; T_i),      i = 0 .. len(temperatures) - 1,
    with the temperature of each step given by the caller (a constant list is training without annealing).
    Returns (S_final, history) with history[i] = L(S_i; T_i), the objective before step i."""
    S = np.array(S0, dtype=np.float64, copy=True)
    history = []
    for T in temperatures:
        history.append(selective_mask_objective(S, G, Gt, lam, T))
        S = S + lr * selective_mask_gradient(S, G, Gt, lam, T)
    return S, np.asarray(history, dtype=np.float64)


def selective_mask_train_factorized(S_in0, S_out0, Z_in, Z_out, Zt_in, Zt_out, lam: float, lr: float, temperatures):
    """The factorised Selective Mask problem of a linear layer (App. B.4 "Linear Layer") solved the same way as the
    plain one (same reading: plain gradient ascent over all rows, one caller-given temperature per step): both logit
    vectors move together,
        S_in  <- S_in  + lr * dL/dS_in,      S_out <- S_out + lr * dL/dS_out,
    with both derivatives taken at the logits before the step.
    Returns (S_in, S_out, history) with history[i] the objective before step i."""
    S_in = np.array(S_in0, dtype=np.float64, copy=True)
    S_out = np.array(S_out0, dtype=np.float64, copy=True)
    history = []
    for T in temperatures:
        obj, g_in, g_out = selective_mask_factorized(S_in, S_out, Z_in, Z_out, Zt_in, Zt_out, lam, T)
        history.append(obj)
        S_in = S_in + lr * g_in
        S_out = S_out + lr * g_out
    return S_in, S_out, np.asarray(history, dtype=np.float64)


def selective_mask_train_factorized_seq(S_in0, S_out0, X_in, X_out, Xt_in, Xt_out, lam: float, lr: float, temperatures):
    """The training loop of the factorised Selective Mask for samples that are sequences of tokens: the loop of
    selective_mask_train_factorized with the objective and derivatives of selective_mask_factorized_seq (same readings:
    plain gradient ascent, one caller-given temperature per step, both derivatives taken at the logits before the step).
    X_in (n, T, d_in), X_out (n, T, d_out) train; Xt_in (m, T', d_in), Xt_out (m, T', d_out) test.
    Returns (S_in, S_out, history) with history[i] the objective before step i."""
    S_in = np.array(S_in0, dtype=np.float64, copy=True)
    S_out = np.array(S_out0, dtype=np.float64, copy=True)
    history = []
    for T in temperatures:
        obj, g_in, g_out = selective_mask_factorized_seq(S_in, S_out, X_in, X_out, Xt_in, Xt_out, lam, T)
        history.append(obj)
        S_in = S_in + lr * g_in
        S_out = S_out + lr * g_out
    return S_in, S_out, np.asarray(history, dtype=np.float64)


def graddot_correlation(G, Gt, idx) -> float:
    """First term of Eq. (1) for a binary mask: the mean over test rows of the Pearson correlation between the exact
    GradDot scores <g_i, g_test> and those of the masked gradients <g_i[idx], g_test[idx]> (Sec. 3.2)."""
    G = np.asarray(G, dtype=np.float64)
    Gt = np.asarray(Gt, dtype=np.float64)
    idx = np.asarray(idx, dtype=np.int64)
    total = 0.0
    for t in range(Gt.shape[0]):
        exact = G @ Gt[t]
        masked = G[:, idx] @ Gt[t, idx]
        da, db = exact - exact.mean(), masked - masked.mean()
        total += (da @ db) / np.sqrt((da @ da) * (db @ db))
    return total / Gt.shape[0]


def selective_mask_indices(S, k: int | None = None) -> np.ndarray:
    """Index extraction (Sec. 3.2): all j with sigma(S_j) >= 1/2, i.e. S_j >= 0, ascending.  With k given, the
    'ensuring exact k' rule of App. B.4: the k largest logits (ties towards the smaller index), ascending."""
    S = np.asarray(S, dtype=np.float64)
    if k is None:
        return np.nonzero(S >= 0.0)[0].astype(np.int32)
    order = np.lexsort((np.arange(S.size), -S))            # by -S, then by index
    return np.sort(order[:k]).astype(np.int32)


# ----------------------------------------------------------------------------
# Dense random projection baseline (Sec. 2.2): g_hat = P g with P (k x p),
# P_ab ~ N(0, 1/k) i.i.d.
#
# Reading (the paper says "Gaussian" and leaves out both the generator and the
# 1/sqrt(k) that makes E||Pg||^2 = ||g||^2): entry (a, b) is one Box-Muller
# normal from the hash of the flat index a*p + b.  Bits 63..41 of the hash give
# u1 = (x + 1/2) / 2^23 in (0, 1) and bits 39..16 give u2 = y / 2^24 in [0, 1),
# both exactly representable in fp32, and z = sqrt(-2 ln u1) cos(2 pi u2).
# ----------------------------------------------------------------------------
def gauss_matrix(seed: int, stream: int, p: int, k: int, p0: int = 0, pc: int | None = None, rows=None) -> np.ndarray:
    """Columns [p0, p0+pc) of P as a k x pc float64 matrix (only the listed rows if `rows` is given)."""
    pc = p - p0 if pc is None else pc
    rows = (np.arange(k, dtype=np.uint64) if rows is None else np.asarray(rows, dtype=np.uint64))[:, None]
    cols = (np.uint64(p0) + np.arange(pc, dtype=np.uint64))[None, :]
    h = stream_hash(seed, stream, rows * np.uint64(p) + cols)
    u1 = ((h >> _U64(41)).astype(np.float64) + 0.5) / 8388608.0
    u2 = ((h >> _U64(16)) & _U64(0xFFFFFF)).astype(np.float64) / 16777216.0
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2) / np.sqrt(float(k))


def gauss_project(g: np.ndarray, P: np.ndarray) -> np.ndarray:
    """g_hat = g P^T for a materialised P (k x p)."""
    return np.asarray(g, dtype=np.float64) @ np.asarray(P, dtype=np.float64).T


# ----------------------------------------------------------------------------
# Error measure used by every parity test: per row, the largest absolute
# difference divided by the largest absolute oracle value of that row.
# (Element-wise relative error is meaningless for a signed sum that can cancel
# to ~0 in individual buckets.)
# ----------------------------------------------------------------------------
def max_rel_err(got: np.ndarray, want: np.ndarray) -> float:
    got = np.asarray(got, dtype=np.float64).reshape(-1, want.shape[-1])
    want = np.asarray(want, dtype=np.float64).reshape(-1, want.shape[-1])
    denom = np.abs(want).max(axis=1)
    denom = np.where(denom == 0.0, 1.0, denom)
    return float((np.abs(got - want).max(axis=1) / denom).max())
