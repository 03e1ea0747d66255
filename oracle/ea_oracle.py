"""fp64 CPU oracle for Expected-Attention KV-cache compression.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this module.
It shares no code with the HIP library and imports neither it nor the input generator; it is
never a fallback for the product path.

Every function follows the paper's steps in the paper's order and notation, with numpy
library routines (matmul, einsum, stable sort) as single steps and no blocking, fusion or
re-ordering.  All arithmetic is IEEE double.  Inputs are the stored tensors widened exactly
to fp64 by the caller.

Shapes:  q_win [B, Hq, w, d]   the w most recent queries, row s at position q_pos0 + s
         k, v  [B, Hkv, n, d]  cached keys (post-rotary, Eq. 1) and values
         group of KV head h = query heads h*G .. h*G+G-1,  G = Hq / Hkv

Readings of the paper where it is silent (each is listed in the design notes too):
  * statistics come from the queries themselves: un-rotate each window query with its own
    position (inverse of Eq. 1), take mean and covariance, then apply R-bar (Eq. 5-6);
  * covariance divisor w - ddof with ddof = 0 unless told otherwise;
  * R-bar averages the rotary matrices of positions t_next .. t_next+T-1 (Eq. 6 with the
    paper's 1-based t = last cached token);
  * GQA: each query head has its own softmax over keys; the normalised attentions are
    averaged over the group, then (a + eps) * ||v||  (Eq. 9 with ||v|| for ||W_o v||, as the
    implementation-details paragraph of Sec. 3.1 states);
  * kept pairs stay in cache order (ascending position); ties go to the lower index.

Pins (tests/test_oracle_pins.py): rotary matrix vs the textbook 2-D rotation and the
relative-position identity; R-bar vs the Dirichlet-kernel closed form; statistics vs
numpy.mean / numpy.cov and vs Eq. 5's linear-map statement; Eq. 7 vs Monte-Carlo sampling of
Gaussian queries (also end-to-end through the rotary maps at T = 1); Sigma = 0 reduction;
variance identity for the quadratic term; softmax vs scipy; Eq. 9 invariants; selection vs
brute force with planted ties; compaction vs fancy indexing; the scalar re-implementation
in ea_scalar.py.  Downstream task accuracy (Tables 1-3) needs the paper's models and
datasets: parity unpinned, and not computed here.
"""
import math

import numpy as np

HALF_SPLIT, INTERLEAVED = 0, 1


# ----------------------------------------------------------------------------- rotary maps
def rope_matrix(p, inv_freq, layout=HALF_SPLIT):
    """R_p of Eq. 1 as a dense d x d matrix: on channel pair (a, b) it is the plane rotation
    [[cos, -sin], [sin, cos]] by the angle p * inv_freq[c]; (a, b) = (c, c + d/2) for the
    half-split layout, (2c, 2c + 1) for the interleaved one."""
    half = len(inv_freq)
    d = 2 * half
    R = np.zeros((d, d))
    for c in range(half):
        a, b = (c, c + half) if layout == HALF_SPLIT else (2 * c, 2 * c + 1)
        ang = float(p) * float(inv_freq[c])
        co, si = math.cos(ang), math.sin(ang)
        R[a, a] = co
        R[a, b] = -si
        R[b, a] = si
        R[b, b] = co
    return R


def averaged_rope_matrix(t_next, T, inv_freq, layout=HALF_SPLIT):
    """R-bar = (1/T) * sum of the rotary matrices of the next T positions (Eq. 6, text below
    it).  The first future position is t_next."""
    d = 2 * len(inv_freq)
    acc = np.zeros((d, d))
    for j in range(int(T)):
        acc += rope_matrix(t_next + j, inv_freq, layout)
    return acc / float(T)


# ------------------------------------------------------------------------------ statistics
def query_stats(q_win, q_pos0, inv_freq, t_next, T=512, ddof=0, q_is_rotated=True,
                layout=HALF_SPLIT):
    """Mean and covariance of the position-averaged query distribution (Eq. 5-6).

    u_s   = R_{p_s}^T q_s                       (queries back to the un-rotated frame, Eq. 1)
    m, S  = mean_s u_s,  cov_s u_s              ("compute_statistics" of Listing 1)
    mu    = R-bar m,   Sigma = R-bar S R-bar^T  (Eq. 6)
    Returns mu [B, Hq, d], Sigma [B, Hq, d, d]."""
    q_win = np.asarray(q_win, dtype=np.float64)
    B, Hq, w, d = q_win.shape
    if w - ddof < 1:
        raise ValueError("window must exceed ddof")
    Rbar = averaged_rope_matrix(t_next, T, inv_freq, layout)
    if q_is_rotated:
        Rt = np.stack([rope_matrix(q_pos0 + s, inv_freq, layout).T for s in range(w)])
    mu = np.empty((B, Hq, d))
    sigma = np.empty((B, Hq, d, d))
    for b in range(B):
        for h in range(Hq):
            q = q_win[b, h]
            u = np.einsum("sij,sj->si", Rt, q) if q_is_rotated else q
            m = u.sum(axis=0) / w
            c = u - m
            S = (c.T @ c) / (w - ddof)
            mu[b, h] = Rbar @ m
            sigma[b, h] = Rbar @ S @ Rbar.T
    return mu, sigma


# ---------------------------------------------------------------------------------- scores
def logits(k, mu, sigma):
    """log z-hat of Eq. 7 for every (query head, key):
         l[g, i] = mu_g . k_i / sqrt(d)  +  k_i^T Sigma_g k_i / (2 d).
    Returns [B, Hq, n]; query head g reads the keys of KV head g // G."""
    k = np.asarray(k, dtype=np.float64)
    B, Hkv, n, d = k.shape
    Hq = mu.shape[1]
    G = Hq // Hkv
    out = np.empty((B, Hq, n))
    for b in range(B):
        for g in range(Hq):
            kk = k[b, g // G]
            lin = (kk @ mu[b, g]) / math.sqrt(d)
            quad = ((kk @ sigma[b, g]) * kk).sum(axis=1) / (2.0 * d)   # k_i^T (Sigma k_i)
            out[b, g] = lin + quad
    return out


def expected_attention(lg):
    """a-hat of Eq. 8: z-hat normalised over all n cached keys (max-subtracted exp)."""
    mx = lg.max(axis=-1, keepdims=True)
    z = np.exp(lg - mx)
    return z / z.sum(axis=-1, keepdims=True)


def scores(k, v, mu, sigma, epsilon=0.02):
    """Eq. 9 per KV pair with ||v|| in place of ||W_o v||, averaged over the GQA group:
         score[h, i] = ( (1/G) sum_{g in group(h)} a-hat[g, i] + eps ) * ||v_i||_2 .
    Returns [B, Hkv, n]."""
    v = np.asarray(v, dtype=np.float64)
    B, Hkv, n, d = v.shape
    a = expected_attention(logits(k, mu, sigma))            # [B, Hq, n]
    G = a.shape[1] // Hkv
    a_group = a.reshape(B, Hkv, G, n).sum(axis=2) / G
    vnorm = np.sqrt((v * v).sum(axis=-1))
    return (a_group + epsilon) * vnorm


# ------------------------------------------------------------------- selection, compaction
def n_keep(n, compression_ratio):
    """Listing 1: int(n * (1 - r)) evaluated in IEEE double, truncated toward zero."""
    return int(float(n) * (1.0 - float(compression_ratio)))


def select(sc, n_kept):
    """The n_kept highest-scoring pairs of every KV head (Sec. 2.2, compression paragraph;
    Listing 1 top-k); equal scores go to the lower index; returned in ascending position.
    sc [B, Hkv, n] -> int64 [B, Hkv, n_kept]."""
    B, H, n = sc.shape
    if not 0 <= n_kept <= n:
        raise ValueError("n_kept out of range")
    idx = np.empty((B, H, n_kept), np.int64)
    for b in range(B):
        for h in range(H):
            order = np.argsort(-sc[b, h], kind="stable")      # descending, ties by index
            idx[b, h] = np.sort(order[:n_kept])
    return idx


def compact(k, v, idx):
    """keys[indices], values[indices] of Listing 1, per KV head."""
    kk = np.take_along_axis(k, idx[..., None], axis=2)
    vv = np.take_along_axis(v, idx[..., None], axis=2)
    return kk, vv


def compress_layer(q_win, k, v, q_pos0, inv_freq, t_next, n_kept, T=512, epsilon=0.02,
                   ddof=0, q_is_rotated=True, layout=HALF_SPLIT, k_store=None, v_store=None):
    """Listing 1 end to end.  k, v are the fp64 values of the cache; k_store / v_store, when
    given, are the stored tensors (any dtype, e.g. bf16 bit patterns) the gather is taken from,
    so that compacted bytes can be compared bit for bit.
    Returns dict(mu, sigma, scores, idx, k, v)."""
    mu, sigma = query_stats(q_win, q_pos0, inv_freq, t_next, T, ddof, q_is_rotated, layout)
    sc = scores(k, v, mu, sigma, epsilon)
    idx = select(sc, n_kept)
    kk, vv = compact(k if k_store is None else k_store, v if v_store is None else v_store, idx)
    return dict(mu=mu, sigma=sigma, scores=sc, idx=idx, k=kk, v=vv)
