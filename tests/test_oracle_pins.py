"""Pins for the fp64 oracle: each test checks it against something other than itself -- a
textbook identity, a library routine, a closed form, Monte-Carlo sampling of the definition,
brute force -- chosen so that a dropped term, a wrong sign / index or a transposed operand
fails at least one of them.  The paper prints no worked numeric example, so there are no
paper-given golden values to compare with."""
import itertools
import math

import numpy as np
import pytest
import scipy.special

from oracle import ea_oracle as O
from oracle import ea_scalar as S
from ea_inputs import CONFIGS, make_layer, widen, inv_freq_table
from ea_inputs.host import _embed_positions


def _rng(seed):
    return np.random.default_rng(seed)


# ------------------------------------------------------------------ rotary matrix (Eq. 1)
@pytest.mark.parametrize("layout", [O.HALF_SPLIT, O.INTERLEAVED])
def test_rope_matrix_is_textbook_rotation(layout):
    # d = 2: one pair, both layouts coincide with the plane rotation by p*theta
    R = O.rope_matrix(3, np.array([0.25]), layout)
    a = 0.75
    assert np.allclose(R, [[math.cos(a), -math.sin(a)], [math.sin(a), math.cos(a)]], atol=1e-15)
    inv = inv_freq_table(16, 1e4)
    Ra, Rb = O.rope_matrix(5, inv, layout), O.rope_matrix(11, inv, layout)
    assert np.allclose(Ra.T @ Ra, np.eye(16), atol=1e-14)             # orthogonal
    assert np.allclose(Ra @ Rb, O.rope_matrix(16, inv, layout), atol=1e-14)  # angles add
    x = _rng(0).standard_normal(16)
    assert abs(np.linalg.norm(Ra @ x) - np.linalg.norm(x)) < 1e-14


@pytest.mark.parametrize("layout", [O.HALF_SPLIT, O.INTERLEAVED])
def test_rope_relative_position_identity(layout):
    # defining property of the rotary embedding: (R_m q).(R_n k) depends on n - m only
    inv = inv_freq_table(32, 5e5)
    q, k = _rng(1).standard_normal(32), _rng(2).standard_normal(32)
    base = (O.rope_matrix(7, inv, layout) @ q) @ (O.rope_matrix(19, inv, layout) @ k)
    for shift in (1, 1000, 123456):
        val = (O.rope_matrix(7 + shift, inv, layout) @ q) @ (O.rope_matrix(19 + shift, inv, layout) @ k)
        assert abs(val - base) < 1e-9


@pytest.mark.parametrize("interleaved", [False, True])
def test_rope_matrix_matches_generator_embedding(interleaved):
    # the input generator's own rotary code (separate coding) applies the same map
    inv = inv_freq_table(16, 1e4)
    x = _rng(3).standard_normal((4, 16))
    pos = np.array([0, 5, 77, 1030])
    y = _embed_positions(x, pos, inv, interleaved)
    for i, p in enumerate(pos):
        R = O.rope_matrix(int(p), inv, O.INTERLEAVED if interleaved else O.HALF_SPLIT)
        assert np.allclose(R @ x[i], y[i], atol=1e-13)


# ------------------------------------------------------------------------- R-bar (Eq. 6)
def _dirichlet(t_next, T, theta):
    # closed form of (1/T) sum_{j<T} exp(i (t_next + j) theta)
    if abs(math.sin(theta / 2)) < 1e-300:
        return 1.0, 0.0
    amp = math.sin(T * theta / 2) / (T * math.sin(theta / 2))
    ph = theta * (t_next + (T - 1) / 2)
    return amp * math.cos(ph), amp * math.sin(ph)


@pytest.mark.parametrize("t_next,T", [(1024, 512), (131072, 512), (17, 1), (4608, 7)])
def test_averaged_rope_closed_form(t_next, T):
    inv = inv_freq_table(64, 5e5)
    Rb = O.averaged_rope_matrix(t_next, T, inv)
    for c in range(32):
        cb, sb = _dirichlet(t_next, T, inv[c])
        blk = Rb[np.ix_([c, c + 32], [c, c + 32])]
        assert np.allclose(blk, [[cb, -sb], [sb, cb]], atol=1e-12)
        sc, ss = S.averaged_rotation(t_next, T, inv[c])
        assert abs(sc - cb) < 1e-12 and abs(ss - sb) < 1e-12
    # nothing outside the 2x2 blocks; contraction (spectral radius <= 1)
    mask = np.ones_like(Rb, bool)
    for c in range(32):
        mask[np.ix_([c, c + 32], [c, c + 32])] = False
    assert np.all(Rb[mask] == 0)
    assert np.linalg.norm(Rb, 2) <= 1 + 1e-12


def test_averaged_rope_special_cases():
    inv = inv_freq_table(32, 1e4)
    assert np.allclose(O.averaged_rope_matrix(41, 1, inv), O.rope_matrix(41, inv), atol=0)
    tiny = np.full(4, 1e-12)
    assert np.allclose(O.averaged_rope_matrix(1000, 512, tiny), np.eye(8), atol=1e-8)
    assert np.allclose(O.averaged_rope_matrix(3, 5, inv, O.INTERLEAVED),
                       sum(O.rope_matrix(3 + j, inv, O.INTERLEAVED) for j in range(5)) / 5)


# -------------------------------------------------------------------- statistics (Eq. 5-6)
@pytest.mark.parametrize("ddof", [0, 1])
def test_stats_match_numpy_mean_cov(ddof):
    # pre-rotary queries, T=1 at position 0 => R-bar = I: plain sample mean / covariance
    q = _rng(4).standard_normal((1, 2, 40, 16)) * 3 + 1
    inv = inv_freq_table(16, 1e4)
    mu, sg = O.query_stats(q, 0, inv, 0, T=1, ddof=ddof, q_is_rotated=False)
    for h in range(2):
        assert np.allclose(mu[0, h], np.mean(q[0, h], axis=0), atol=1e-13)
        assert np.allclose(sg[0, h], np.cov(q[0, h].T, ddof=ddof), atol=1e-12)


def test_stats_unrotation_and_eq5_linear_map():
    # queries built as in Eq. 1, q_s = R_{p_s} W h_s.  Eq. 5-6 then say
    #   mu = R-bar W mean(h),  Sigma = R-bar W cov(h) W^T R-bar^T.
    r = _rng(5)
    d, hdim, w, p0, t_next, T = 16, 24, 50, 300, 350, 9
    inv = inv_freq_table(d, 1e4)
    W = r.standard_normal((d, hdim))
    h = r.standard_normal((w, hdim)) * 2 + r.standard_normal(hdim)
    q = np.stack([O.rope_matrix(p0 + s, inv) @ (W @ h[s]) for s in range(w)])
    mu, sg = O.query_stats(q[None, None], p0, inv, t_next, T=T)
    Rb = O.averaged_rope_matrix(t_next, T, inv)
    assert np.allclose(mu[0, 0], Rb @ W @ h.mean(axis=0), atol=1e-11)
    assert np.allclose(sg[0, 0], Rb @ W @ np.cov(h.T, ddof=0) @ W.T @ Rb.T, atol=1e-10)


def test_stats_psd_rank_and_degenerate_window():
    lay = make_layer(CONFIGS["c1"], n=256, window=24)
    mu, sg = O.query_stats(widen(lay["q_win"]), lay["q_pos0"], lay["inv_freq"], lay["t_next"], T=512)
    for h in range(4):
        A = sg[0, h]
        assert np.allclose(A, A.T, atol=1e-13)
        ev = np.linalg.eigvalsh(A)
        assert ev.min() > -1e-12 * max(1.0, np.trace(A))
        assert np.linalg.matrix_rank(A, tol=1e-9 * ev.max()) <= 23
    q1 = widen(lay["q_win"])[:, :, :1]
    mu1, sg1 = O.query_stats(q1, lay["q_pos0"], lay["inv_freq"], lay["t_next"], T=512)
    assert np.all(sg1 == 0)                         # one sample: zero covariance
    with pytest.raises(ValueError):
        O.query_stats(q1, 0, lay["inv_freq"], 1, ddof=1)


# --------------------------------------------------------------------- closed form (Eq. 7)
def test_closed_form_vs_monte_carlo():
    # z-hat_i = E_q exp(q.k_i / sqrt d) for q ~ N(mu, Sigma): sample the definition
    r = _rng(6)
    d, n, N = 16, 6, 1_000_000
    A = r.standard_normal((d, d)) * 0.15
    sigma = A @ A.T
    mu = r.standard_normal(d) * 0.5
    k = r.standard_normal((n, d))
    lg = O.logits(k[None, None], mu[None, None], sigma[None, None])[0, 0]
    q = r.multivariate_normal(mu, sigma, size=N, method="cholesky")
    x = np.exp(q @ k.T / math.sqrt(d))
    for i in range(n):
        s2 = k[i] @ sigma @ k[i] / d
        assert s2 < 0.8
        rel_se = math.sqrt((math.exp(s2) - 1) / N)
        assert abs(x[:, i].mean() / math.exp(lg[i]) - 1) < 4.5 * rel_se


def test_closed_form_end_to_end_through_rotary_maps_T1():
    # exact Gaussian pre-rotary queries -> window at positions p0.. -> query_stats with T=1.
    # Fresh queries drawn from the fitted Gaussian and embedded at t_next by the *generator's*
    # rotary code must reproduce z-hat: pins un-rotation direction, R-bar direction, Eq. 7.
    r = _rng(7)
    d, w, p0, N = 8, 4000, 100, 400_000
    inv = inv_freq_table(d, 1e2)
    t_next = p0 + w
    A = r.standard_normal((d, d)) * 0.5
    m_true = r.standard_normal(d)
    u = r.standard_normal((w, d)) @ A.T + m_true
    q = _embed_positions(u, p0 + np.arange(w), inv, False)
    mu, sg = O.query_stats(q[None, None], p0, inv, t_next, T=1)
    m_hat, S_hat = u.mean(axis=0), np.cov(u.T, ddof=0)
    fresh = r.multivariate_normal(m_hat, S_hat, size=N, method="cholesky")
    qf = _embed_positions(fresh, np.full(N, t_next), inv, False)
    k = r.standard_normal((3, d))
    lg = O.logits(k[None, None], mu, sg)[0, 0]
    for i in range(3):
        s2 = k[i] @ sg[0, 0] @ k[i] / d
        rel_se = math.sqrt((math.exp(s2) - 1) / N)
        mc = np.exp(qf @ k[i] / math.sqrt(d)).mean()
        assert abs(mc / math.exp(lg[i]) - 1) < 4.5 * rel_se


def test_sigma_zero_reduces_to_mean_query_dot():
    r = _rng(8)
    d, n = 32, 50
    mu, k = r.standard_normal(d), r.standard_normal((n, d))
    lg = O.logits(k[None, None], mu[None, None], np.zeros((1, 1, d, d)))[0, 0]
    assert np.allclose(np.exp(lg), np.exp(k @ mu / math.sqrt(d)), rtol=1e-14)


def test_quadratic_term_variance_identity():
    # k^T Sigma-bar k = var_s(u~_s . k) and mu-bar . k = mean_s(u~_s . k) with u~_s = R-bar u_s:
    # a second computation that never forms a covariance matrix
    lay = make_layer(CONFIGS["c1"], n=128, window=32)
    q, k = widen(lay["q_win"]), widen(lay["k"])
    inv, T = lay["inv_freq"], 512
    mu, sg = O.query_stats(q, lay["q_pos0"], inv, lay["t_next"], T=T)
    lg = O.logits(k, mu, sg)
    Rb = O.averaged_rope_matrix(lay["t_next"], T, inv)
    d = 64
    for g in range(4):
        ut = np.stack([Rb @ O.rope_matrix(lay["q_pos0"] + s, inv).T @ q[0, g, s] for s in range(32)])
        proj = ut @ k[0, g // 2].T                                   # [w, n]
        ref = proj.mean(axis=0) / math.sqrt(d) + proj.var(axis=0) / (2 * d)
        assert np.allclose(lg[0, g], ref, rtol=1e-10, atol=1e-10)
        assert np.all(proj.var(axis=0) >= 0)


# ------------------------------------------------------------------------ softmax (Eq. 8)
def test_expected_attention_is_softmax():
    lg = _rng(9).standard_normal((2, 3, 100)) * 30
    a = O.expected_attention(lg)
    assert np.allclose(a.sum(axis=-1), 1.0, atol=1e-12)
    assert np.allclose(a, scipy.special.softmax(lg, axis=-1), rtol=1e-12, atol=0)
    assert np.allclose(a, O.expected_attention(lg + 123.0), rtol=1e-10)
    assert np.allclose(np.log(a), lg - scipy.special.logsumexp(lg, axis=-1, keepdims=True), atol=1e-9)
    perm = _rng(10).permutation(100)
    assert np.allclose(O.expected_attention(lg[..., perm]), a[..., perm], rtol=1e-12)


# --------------------------------------------------------------------- final score (Eq. 9)
def test_score_invariants():
    lay = make_layer(CONFIGS["c1"], n=200, window=16)
    q, k, v = widen(lay["q_win"]), widen(lay["k"]), widen(lay["v"])
    mu, sg = O.query_stats(q, lay["q_pos0"], lay["inv_freq"], lay["t_next"])
    eps = 0.02
    sc = O.scores(k, v, mu, sg, eps)
    vn = np.linalg.norm(v, axis=-1)
    assert sc.shape == (1, 2, 200)
    assert np.all(sc >= eps * vn - 1e-15)
    assert np.allclose((sc / vn).sum(axis=-1), 1 + 200 * eps, rtol=1e-12)   # sum_i a-hat = 1
    assert np.allclose(O.scores(k, 3 * v, mu, sg, eps), 3 * sc, rtol=1e-13)
    # eps = 0, unit value norms, G = 1: ranking is the ranking of the logits
    vu = v / vn[..., None]
    s0 = O.scores(k[:, :1], vu[:, :1], mu[:, :1], sg[:, :1], 0.0)
    lg = O.logits(k[:, :1], mu[:, :1], sg[:, :1])
    assert np.array_equal(np.argsort(s0[0, 0]), np.argsort(lg[0, 0]))
    # a group of identical query heads scores like a single head
    mu2, sg2 = np.repeat(mu[:, :1], 2, axis=1), np.repeat(sg[:, :1], 2, axis=1)
    assert np.allclose(O.scores(k[:, :1], v[:, :1], mu2, sg2, eps),
                       O.scores(k[:, :1], v[:, :1], mu[:, :1], sg[:, :1], eps), rtol=1e-13)
    # group average: mean of the per-head scores (||v|| and eps are per-pair constants)
    per_head = [O.scores(k[:, :1], v[:, :1], mu[:, g:g + 1], sg[:, g:g + 1], eps) for g in (0, 1)]
    assert np.allclose(sc[:, :1], (per_head[0] + per_head[1]) / 2, rtol=1e-13)
    # query heads 2,3 belong to KV head 1, not 0
    other = O.scores(k[:, 1:], v[:, 1:], mu[:, 2:], sg[:, 2:], eps)
    assert np.allclose(sc[:, 1:], other, rtol=1e-13)


# ------------------------------------------------------------- selection and compaction
def test_n_keep_is_listing_truncation():
    assert O.n_keep(1024, 0.5) == 512 and O.n_keep(131072, 0.25) == 98304
    assert O.n_keep(131072, 0.75) == 32768 and O.n_keep(7, 0.5) == 3
    assert O.n_keep(1000, 0.9) == int(1000 * (1 - 0.9)) == 99      # double rounding of 1-0.9
    assert O.n_keep(10, 0.0) == 10 and O.n_keep(10, 1.0) == 0


def test_select_vs_brute_force_with_ties():
    r = _rng(11)
    for n in (1, 2, 7, 12):
        sc = r.integers(0, 4, size=(1, 3, n)).astype(np.float64)     # many planted ties
        for kk in range(n + 1):
            idx = O.select(sc, kk)
            for h in range(3):
                s = sc[0, h]
                got = idx[0, h]
                assert list(got) == sorted(set(got)) and len(got) == kk
                # brute force: the subset of size kk maximising (sum of scores, then
                # lexicographically smallest index tuple among maximisers)
                if n <= 7:
                    best = max(itertools.combinations(range(n), kk),
                               key=lambda c: (s[list(c)].sum(), [-i for i in c]))
                    assert list(got) == list(best)
                assert list(got) == S.select(list(s), kk)
                if 0 < kk < n:
                    rest = np.setdiff1d(np.arange(n), got)
                    assert s[got].min() >= s[rest].max()
                    tie = s[got].min()
                    # among pairs tied at the threshold the lower indices are the kept ones
                    tied_kept = [i for i in got if s[i] == tie]
                    tied_left = [i for i in rest if s[i] == tie]
                    assert not tied_left or max(tied_kept) < min(tied_left)


def test_compact_is_fancy_index_gather():
    r = _rng(12)
    k = r.integers(0, 2**16, size=(2, 3, 20, 8)).astype(np.uint16)
    v = r.integers(0, 2**16, size=(2, 3, 20, 8)).astype(np.uint16)
    idx = np.sort(r.permuted(np.tile(np.arange(20), (2, 3, 1)), axis=-1)[..., :9], axis=-1)
    kk, vv = O.compact(k, v, idx)
    for b in range(2):
        for h in range(3):
            assert np.array_equal(kk[b, h], k[b, h][idx[b, h]])
            assert np.array_equal(vv[b, h], v[b, h][idx[b, h]])
    full = np.tile(np.arange(20), (2, 3, 1))
    k2, v2 = O.compact(k, v, full)
    assert np.array_equal(k2, k) and np.array_equal(v2, v)


# ------------------------------------------------------------- scalar re-implementation
def test_vectorised_oracle_matches_scalar_restatement():
    cfg = CONFIGS["c1"].with_(head_dim=8, n_q_heads=4, n_kv_heads=2)
    for interleaved in (False, True):
        lay = make_layer(cfg, n=24, window=6, pos0=1000, interleaved=interleaved)
        q, k, v = widen(lay["q_win"]), widen(lay["k"]), widen(lay["v"])
        layout = O.INTERLEAVED if interleaved else O.HALF_SPLIT
        for ddof in (0, 1):
            res = O.compress_layer(q, k, v, lay["q_pos0"], lay["inv_freq"], lay["t_next"], 10,
                                   T=16, epsilon=0.02, ddof=ddof, layout=layout)
            for h in range(2):
                mus, sgs = [], []
                for g in (2 * h, 2 * h + 1):
                    m, s = S.query_stats(q[0, g].tolist(), lay["q_pos0"], list(lay["inv_freq"]),
                                         lay["t_next"], 16, ddof, True, interleaved)
                    assert np.allclose(res["mu"][0, g], m, rtol=1e-11, atol=1e-12)
                    assert np.allclose(res["sigma"][0, g], s, rtol=1e-10, atol=1e-12)
                    mus.append(m)
                    sgs.append(s)
                sc = S.scores(k[0, h].tolist(), v[0, h].tolist(), mus, sgs, 0.02)
                assert np.allclose(res["scores"][0, h], sc, rtol=1e-10)
                assert list(res["idx"][0, h]) == S.select(sc, 10)


def test_pre_rope_queries_flag():
    # un-rotating rotated queries equals taking the pre-rotary queries as they are
    cfg = CONFIGS["c1"].with_(head_dim=16)
    a = make_layer(cfg, n=64, window=20)
    b = make_layer(cfg, n=64, window=20, pre_rope_queries=True)
    mu_a, sg_a = O.query_stats(a["q_win"].astype(np.float64), a["q_pos0"], a["inv_freq"], a["t_next"])
    mu_b, sg_b = O.query_stats(b["q_win"].astype(np.float64), b["q_pos0"], b["inv_freq"], b["t_next"],
                               q_is_rotated=False)
    assert np.allclose(mu_a, mu_b, atol=2e-5) and np.allclose(sg_a, sg_b, atol=2e-4)  # fp32 storage
