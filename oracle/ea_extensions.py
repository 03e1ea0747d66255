"""fp64 CPU oracle for the extensions around the Expected-Attention compress step.
TEST INFRASTRUCTURE ONLY (same rules as ea_oracle.py: only tests/, smoke() and bench.py's
cpu_baseline leg may import it; it shares nothing with the HIP library).

  compact_unordered      order-free compaction: attention over the cache is a sum over cached pairs
                         (Eq. 2-3), so the order of the kept pairs does not matter; kept rows
                         beyond the new length move into the holes in front of it
  select_adaptive        head-adaptive budgets (Sec. 2.2, "Head-Adaptive Compression"): one budget
                         per layer shared by its KV heads
  compact_ragged         the gather of Listing 1 with a different kept count per head
  query_stats_hidden     Eq. 5 as printed: statistics of the hidden states, pushed through W_Q
  scores_wo              Eq. 9 as printed: ||W_o v|| instead of ||v||
  paged_rows             block-table ("paged") cache layout: which pool row holds a logical row
  fp8_e4m3_decode        caches stored as OCP e4m3 bytes: the value of every byte
  knorm / streaming / keydiff scores   the comparison scorers of Sec. 3.1 ("Baselines"), from the one
                         sentence the paper gives each, on the same select + compact back half

Readings where the paper is silent (each is listed in the design notes too):
  * head-adaptive: the paper only cites the idea.  Here: per (sequence, layer) the
    Hkv * n_kept pairs of highest score over ALL the KV heads of the layer are kept, after every
    head has been given its own `floor` best pairs; equal scores go to the lower head, then to
    the lower position.
  * Eq. 9 with W_o under GQA: query head g sends value head h = g // G through its own d columns
    of W_o, so  score[h, i] = (1/G) sum_{g in group(h)} (a-hat[g, i] + eps) * ||W_o^(g) v_i||.
  * KNorm "preserves keys with the lowest L2 norm": score = 1 / ||k||  (larger = kept first).
  * StreamingLLM "maintains initial sink tokens": the first n_sink pairs are always kept, the
    rest of the budget goes to the most recent pairs: score = +inf for sinks, position + 1 else.
  * KeyDiff "employs distance metrics between key embeddings": score = 1 - cos(k_i, a) with a the
    mean of the head's unit-normalised keys (keys least like the average key are kept first).

Pins (tests/test_oracle_extensions.py): order-free compaction vs brute force over all kept
sets of small caches (the rows in front are exactly the kept set, untouched rows stay, the move
count is the minimum possible); adaptive selection vs a flat stable sort and its invariants
(sum of lengths = budget, every head's list is its own top-length, floor honoured, uniform
scores reduce to the per-head rule); hidden-state statistics vs the projected-query route of
ea_oracle.query_stats (Eq. 5's linearity); ||W_o v|| vs numpy.linalg.norm of the explicit product
and the W_o = I reduction to ea_oracle.scores; the scorers vs their one-line definitions on
hand-made keys; the paged layout vs a pool written out by hand and vs the input generator's
separately coded scatter; the e4m3 decoding vs values written out from the format's definition
and vs torch's float8_e4m3fn for all 256 codes.
"""
import math

import numpy as np

from . import ea_oracle as O


# ------------------------------------------------------------------ order-free compaction (f3)
def unordered_perm(idx, n_kept):
    """Which source row ends up at each position < n_kept when the kept rows idx (ascending)
    are compacted without keeping their order: a kept row below n_kept stays where it is; the
    kept rows at or beyond n_kept fill, in ascending order, the evicted positions below n_kept,
    in ascending order.  Returns int64 [n_kept]."""
    idx = np.asarray(idx, np.int64)
    perm = np.full(n_kept, -1, np.int64)
    stay = idx[idx < n_kept]
    perm[stay] = stay
    movers = idx[idx >= n_kept]
    holes = np.nonzero(perm < 0)[0]
    assert len(holes) == len(movers)
    perm[holes] = movers
    return perm


def compact_unordered(k, v, idx):
    """Order-free compaction of every KV head: rows [0, n_kept) of the result hold exactly the
    kept rows; rows from n_kept on are not part of the result.
    Returns (k[:, :, :n_kept], v[:, :, :n_kept], perm [B, Hkv, n_kept])."""
    B, H, n_kept = idx.shape
    perm = np.empty((B, H, n_kept), np.int64)
    for b in range(B):
        for h in range(H):
            perm[b, h] = unordered_perm(idx[b, h], n_kept)
    kk = np.take_along_axis(k, perm[..., None], axis=2)
    vv = np.take_along_axis(v, perm[..., None], axis=2)
    return kk, vv, perm


# ------------------------------------------------------------------ head-adaptive budgets (f1)
def select_adaptive(sc, n_kept, floor=0):
    """One budget of Hkv * n_kept pairs per (sequence, layer), shared by its KV heads.
    Step 1: every head keeps its own `floor` best pairs (ties to the lower position).
    Step 2: the rest of the budget goes to the best remaining pairs of the whole layer
            (ties to the lower head, then to the lower position).
    sc [B, Hkv, n] -> (lengths int64 [B, Hkv], list over b of list over h of ascending int64 arrays)."""
    B, H, n = sc.shape
    if not 0 <= floor <= n_kept <= n:
        raise ValueError("need 0 <= floor <= n_kept <= n")
    lengths = np.zeros((B, H), np.int64)
    kept = []
    for b in range(B):
        taken = np.zeros((H, n), bool)
        for h in range(H):
            order = np.argsort(-sc[b, h], kind="stable")
            taken[h, order[:floor]] = True
        rest = H * n_kept - H * floor
        flat = np.where(taken, -np.inf, sc[b]).reshape(-1)       # pairs already kept are out of the pool
        order = np.argsort(-flat, kind="stable")                 # (head, position) order among equals
        taken.reshape(-1)[order[:rest]] = True
        kept.append([np.nonzero(taken[h])[0].astype(np.int64) for h in range(H)])
        lengths[b] = taken.sum(axis=1)
    return lengths, kept


def compact_ragged(k, v, kept):
    """Listing 1's gather with a kept list per head: returns lists [b][h] of (k rows, v rows)."""
    return [[(k[b, h][ix], v[b, h][ix]) for h, ix in enumerate(row)] for b, row in enumerate(kept)]


# ------------------------------------------------------------------ Eq. 5 / Eq. 9 as printed (f2)
def query_stats_hidden(hidden, w_q, inv_freq, t_next, T=512, ddof=0, layout=O.HALF_SPLIT):
    """Eq. 5-6 literally: mu_h, Sigma_h = mean / covariance of the buffered hidden states
    hidden [B, w, dm]; per query head  mu = R-bar W_Q mu_h,  Sigma = R-bar W_Q Sigma_h W_Q^T R-bar^T
    with W_Q [Hq, d, dm].  Returns mu [B, Hq, d], Sigma [B, Hq, d, d]."""
    hidden = np.asarray(hidden, np.float64)
    w_q = np.asarray(w_q, np.float64)
    B, w, dm = hidden.shape
    Hq, d, _ = w_q.shape
    Rbar = O.averaged_rope_matrix(t_next, T, inv_freq, layout)
    mu = np.empty((B, Hq, d))
    sigma = np.empty((B, Hq, d, d))
    for b in range(B):
        m_h = hidden[b].sum(axis=0) / w
        c = hidden[b] - m_h
        S_h = (c.T @ c) / (w - ddof)
        for g in range(Hq):
            mu[b, g] = Rbar @ (w_q[g] @ m_h)
            sigma[b, g] = Rbar @ (w_q[g] @ S_h @ w_q[g].T) @ Rbar.T
    return mu, sigma


def wo_value_norms(v, w_o):
    """||W_o^(g) v_i||_2 for every query head g and cached value i: v [B, Hkv, n, d],
    w_o [Hq, dm, d] (the d columns of W_o that query head g feeds).  Returns [B, Hq, n]."""
    v = np.asarray(v, np.float64)
    w_o = np.asarray(w_o, np.float64)
    B, Hkv, n, d = v.shape
    Hq = w_o.shape[0]
    G = Hq // Hkv
    out = np.empty((B, Hq, n))
    for b in range(B):
        for g in range(Hq):
            y = v[b, g // G] @ w_o[g].T                           # [n, dm]
            out[b, g] = np.sqrt((y * y).sum(axis=1))
    return out


def scores_wo(k, v, mu, sigma, w_o, epsilon=0.02):
    """Eq. 9 as printed, per query head, averaged over the GQA group:
         score[h, i] = (1/G) sum_{g in group(h)} (a-hat[g, i] + eps) * ||W_o^(g) v_i||.
    Returns [B, Hkv, n]."""
    a = O.expected_attention(O.logits(k, mu, sigma))              # [B, Hq, n]
    wn = wo_value_norms(v, w_o)
    B, Hq, n = a.shape
    Hkv = np.asarray(v).shape[1]
    G = Hq // Hkv
    return ((a + epsilon) * wn).reshape(B, Hkv, G, n).sum(axis=2) / G


# ------------------------------------------------------------------ comparison scorers (f4)
def knorm_scores(k):
    """KNorm keeps the keys of lowest L2 norm: score = 1 / ||k_i||_2.  k [B, Hkv, n, d]."""
    k = np.asarray(k, np.float64)
    with np.errstate(divide="ignore"):
        return 1.0 / np.sqrt((k * k).sum(axis=-1))


def streaming_scores(B, Hkv, n, n_sink):
    """StreamingLLM keeps the first n_sink pairs and, with the rest of the budget, the most
    recent ones: score = +inf for i < n_sink, i + 1 otherwise."""
    s = np.arange(1, n + 1, dtype=np.float64)
    s[:n_sink] = np.inf
    return np.broadcast_to(s, (B, Hkv, n)).copy()


def keydiff_scores(k):
    """KeyDiff ranks keys by a distance between key embeddings: here 1 - cos(k_i, a), a = the mean
    of the head's unit-normalised keys.  Keys of zero norm count as the zero vector."""
    k = np.asarray(k, np.float64)
    nrm = np.sqrt((k * k).sum(axis=-1, keepdims=True))
    with np.errstate(invalid="ignore", divide="ignore"):
        u = np.where(nrm > 0, k / nrm, 0.0)
    a = u.sum(axis=2, keepdims=True) / k.shape[2]
    an = np.sqrt((a * a).sum(axis=-1, keepdims=True))
    with np.errstate(invalid="ignore", divide="ignore"):
        cos = np.where(an > 0, (u * a).sum(axis=-1, keepdims=True) / an, 0.0)
    return 1.0 - cos[..., 0]


# ------------------------------------------------------------------ paged cache layout (f3)
def paged_rows(pool, table, n):
    """Logical view of a paged cache: pool [num_blocks, Hkv, block_size, d], table [B, max_blocks]
    (pool block of every logical block of every sequence) -> [B, Hkv, n, d], where logical row i of
    sequence b and head h is pool[table[b, i // block_size], h, i % block_size]."""
    pool, table = np.asarray(pool), np.asarray(table)
    B, bs = table.shape[0], pool.shape[2]
    out = np.empty((B, pool.shape[1], n, pool.shape[3]), pool.dtype)
    for b in range(B):
        for i in range(n):
            out[b, :, i] = pool[table[b, i // bs], :, i % bs]
    return out


# ------------------------------------------------------------------ caches stored as e4m3 bytes (f3)
def fp8_e4m3_decode(b):
    """Value of OCP e4m3 ("float8_e4m3fn") bytes as float64: 1 sign bit, 4 exponent bits (bias 7),
    3 mantissa bits; exponent 0 is subnormal ((m / 8) * 2^-6); there are no infinities and
    S.1111.111 is NaN, so the largest magnitude is 1.75 * 2^8 = 448."""
    b = np.asarray(b, np.uint8).astype(np.int64)
    sign = np.where(b >> 7, -1.0, 1.0)
    e, m = (b >> 3) & 15, b & 7
    mag = np.where(e == 0, (m / 8.0) * 2.0 ** -6, (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64)))
    return np.where((e == 15) & (m == 7), np.nan, sign * mag)
