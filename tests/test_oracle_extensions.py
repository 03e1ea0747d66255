"""Pins of oracle/ea_extensions.py against things other than itself: brute force on tiny inputs,
invariants, library routines and reductions to the already pinned ea_oracle.py (CPU only)."""
import itertools

import numpy as np
import pytest

from oracle import ea_oracle as O
from oracle import ea_extensions as X


# ---------------------------------------------------------------- order-free compaction (Eq. 2-3)
@pytest.mark.parametrize("n", [1, 2, 5, 7])
def test_unordered_perm_brute_force_over_all_kept_sets(n):
    """Every subset of a small cache: the rows in front are exactly the kept set, kept rows that
    are already in front do not move, and the number of moved rows is the minimum any order-free
    compaction needs (a kept row at or beyond the new length has to move, nothing else does)."""
    for m in range(n + 1):
        for kept in itertools.combinations(range(n), m):
            perm = X.unordered_perm(np.array(kept, np.int64), m)
            assert sorted(perm.tolist()) == list(kept)
            for p in range(m):
                if p in kept:
                    assert perm[p] == p
            moved = int((perm != np.arange(m)).sum())
            assert moved == sum(1 for i in kept if i >= m)
            # movers and holes are paired in ascending order
            mv = perm[perm != np.arange(m)]
            assert np.all(np.diff(mv) > 0)


def test_compact_unordered_attention_output_is_unchanged():
    """The reason the order may be given up: softmax attention over the kept pairs (Eq. 2-3) is a
    sum over pairs, so ordered and order-free compaction give the same attention output."""
    r = np.random.default_rng(5)
    k, v = r.standard_normal((2, 3, 40, 8)), r.standard_normal((2, 3, 40, 8))
    idx = np.stack([[np.sort(r.choice(40, 17, replace=False)) for _ in range(3)] for _ in range(2)])
    ko, vo = O.compact(k, v, idx)
    ku, vu, perm = X.compact_unordered(k, v, idx)
    assert np.array_equal(np.sort(perm, axis=-1), idx)
    q = r.standard_normal(8)
    for b in range(2):
        for h in range(3):
            def attn(kk, vv):
                z = np.exp(kk @ q / np.sqrt(8.0))
                return (z / z.sum()) @ vv
            assert np.allclose(attn(ko[b, h], vo[b, h]), attn(ku[b, h], vu[b, h]), rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------- head-adaptive budgets
def _flat_reference(sc_b, budget):
    """Top-`budget` of the flattened [H, n] scores: full stable sort (ties: head, then position)."""
    H, n = sc_b.shape
    order = np.argsort(-sc_b.reshape(-1), kind="stable")[:budget]
    return [np.sort(order[(order // n) == h] % n) for h in range(H)]


def test_select_adaptive_without_floor_is_a_flat_top_k():
    r = np.random.default_rng(1)
    sc = r.random((2, 4, 50))
    sc[0, 1, ::3] = sc[0, 0, 0]                       # ties across heads and positions
    sc[1] = np.round(sc[1], 1)                        # few distinct values
    for n_kept in (0, 1, 13, 50):
        lengths, kept = X.select_adaptive(sc, n_kept)
        for b in range(2):
            ref = _flat_reference(sc[b], 4 * n_kept)
            assert lengths[b].sum() == 4 * n_kept
            for h in range(4):
                assert np.array_equal(kept[b][h], ref[h])
                assert lengths[b, h] == len(ref[h])


def test_select_adaptive_invariants_with_floor():
    r = np.random.default_rng(2)
    sc = np.exp(2.0 * r.standard_normal((3, 5, 64)))
    sc[:, 0] *= 50.0                                   # one dominant head
    n_kept, floor = 20, 6
    lengths, kept = X.select_adaptive(sc, n_kept, floor)
    per_head = O.select(sc, floor)
    for b in range(3):
        assert lengths[b].sum() == 5 * n_kept
        assert lengths[b].min() >= floor and lengths[b, 0] == lengths[b].max() > n_kept   # the dominant head keeps more
        for h in range(5):
            ix = kept[b][h]
            assert np.all(np.diff(ix) > 0)
            # every head's list is that head's own top-`length`
            assert np.array_equal(ix, O.select(sc[b:b + 1, h:h + 1], len(ix))[0, 0])
            assert set(per_head[b, h]) <= set(ix)
        # nothing evicted beats anything kept beyond the floors
        pool_kept = [sc[b, h, i] for h in range(5) for i in kept[b][h] if i not in set(per_head[b, h])]
        evicted = [sc[b, h, i] for h in range(5) for i in range(64) if i not in set(kept[b][h])]
        if pool_kept and evicted:
            assert min(pool_kept) >= max(evicted)


def test_select_adaptive_reduces_to_the_per_head_rule():
    """floor = n_kept leaves nothing to share; so does a layer whose heads have the same scores."""
    r = np.random.default_rng(3)
    sc = r.random((1, 3, 30))
    lengths, kept = X.select_adaptive(sc, 10, floor=10)
    ref = O.select(sc, 10)
    assert np.all(lengths == 10)
    for h in range(3):
        assert np.array_equal(kept[0][h], ref[0, h])
    same = np.broadcast_to(sc[:, :1], (1, 3, 30)).copy()
    lengths, kept = X.select_adaptive(same, 10)
    assert lengths.sum() == 30 and lengths.max() - lengths.min() <= 1


def test_compact_ragged_is_fancy_indexing():
    r = np.random.default_rng(4)
    k, v = r.integers(0, 1000, (1, 2, 9, 4)), r.integers(0, 1000, (1, 2, 9, 4))
    kept = [[np.array([0, 3, 8]), np.array([], np.int64)]]
    out = X.compact_ragged(k, v, kept)
    assert np.array_equal(out[0][0][0], k[0, 0][[0, 3, 8]]) and out[0][1][1].shape == (0, 4)


# ---------------------------------------------------------------- Eq. 5 and Eq. 9 as printed
def test_hidden_state_statistics_equal_projected_query_statistics():
    """Eq. 5's statement: queries are a fixed linear map of the hidden states, so the statistics of
    the hidden states pushed through W_Q are the statistics of the projected (un-rotated) queries.
    The right-hand side is ea_oracle.query_stats, pinned on its own."""
    r = np.random.default_rng(6)
    B, w, dm, Hq, d = 2, 24, 20, 3, 8
    hidden = r.standard_normal((B, w, dm)) + 0.5
    w_q = r.standard_normal((Hq, d, dm)) / np.sqrt(dm)
    inv_freq = 10000.0 ** (-np.arange(d // 2) / (d // 2))
    q = np.einsum("gdm,bwm->bgwd", w_q, hidden)
    for ddof in (0, 1):
        mu, sg = X.query_stats_hidden(hidden, w_q, inv_freq, 100, T=16, ddof=ddof)
        rmu, rsg = O.query_stats(q, 0, inv_freq, 100, T=16, ddof=ddof, q_is_rotated=False)
        assert np.allclose(mu, rmu, rtol=1e-11, atol=1e-13)
        assert np.allclose(sg, rsg, rtol=1e-10, atol=1e-13)


def test_wo_norms_and_scores():
    r = np.random.default_rng(7)
    B, Hkv, G, n, d, dm = 1, 2, 2, 30, 8, 12
    k, v = r.standard_normal((B, Hkv, n, d)), r.standard_normal((B, Hkv, n, d))
    mu = r.standard_normal((B, Hkv * G, d))
    a = r.standard_normal((B, Hkv * G, d, d))
    sigma = a @ a.transpose(0, 1, 3, 2) / d
    w_o = r.standard_normal((Hkv * G, dm, d))
    wn = X.wo_value_norms(v, w_o)
    for g in range(Hkv * G):
        for i in (0, 7, 29):
            assert np.isclose(wn[0, g, i], np.linalg.norm(w_o[g] @ v[0, g // G, i]), rtol=1e-13)
    # an orthonormal W_o (here: identity padded with zero rows) leaves the norms alone: Eq. 9 with ||v||
    eye = np.zeros((Hkv * G, dm, d))
    eye[:, :d, :] = np.eye(d)
    assert np.allclose(X.scores_wo(k, v, mu, sigma, eye, 0.02), O.scores(k, v, mu, sigma, 0.02), rtol=1e-12)
    # scaling W_o scales the scores; the sum over keys of score / norm is 1 + n eps for G = 1
    assert np.allclose(X.scores_wo(k, v, mu, sigma, 3.0 * w_o, 0.02), 3.0 * X.scores_wo(k, v, mu, sigma, w_o, 0.02))
    s1 = X.scores_wo(k, v, mu[:, ::2], sigma[:, ::2], w_o[::2], 0.02)
    assert np.allclose((s1 / X.wo_value_norms(v, w_o[::2])).sum(axis=-1), 1 + n * 0.02)


# ---------------------------------------------------------------- comparison scorers
def test_scorers_on_hand_made_keys():
    k = np.zeros((1, 1, 5, 4))
    k[0, 0, :, 0] = [3.0, 1.0, 2.0, 0.5, 4.0]          # norms 3, 1, 2, .5, 4
    s = X.knorm_scores(k)
    assert np.array_equal(O.select(s, 2)[0, 0], [1, 3])            # the two keys of lowest norm
    assert np.allclose(s[0, 0], 1.0 / np.array([3.0, 1.0, 2.0, 0.5, 4.0]))
    st = X.streaming_scores(1, 1, 10, 2)
    assert np.array_equal(O.select(st, 5)[0, 0], [0, 1, 7, 8, 9])  # two sinks and the three most recent
    assert np.array_equal(O.select(X.streaming_scores(1, 1, 10, 0), 3)[0, 0], [7, 8, 9])
    kd = np.zeros((1, 1, 4, 2))
    kd[0, 0] = [[1, 0], [2, 0], [0, 1], [5, 0]]        # three keys along x, one along y
    sd = X.keydiff_scores(kd)
    a = np.array([3.0, 1.0]) / 4.0
    cos = np.array([a[0], a[0], a[1], a[0]]) / np.linalg.norm(a)
    assert np.allclose(sd[0, 0], 1.0 - cos)
    assert O.select(sd, 1)[0, 0, 0] == 2               # the odd one out is kept first
    # scale invariance of the cosine and the range [0, 2]
    r = np.random.default_rng(8)
    kk = r.standard_normal((2, 2, 50, 16))
    assert np.allclose(X.keydiff_scores(kk), X.keydiff_scores(7.0 * kk))
    assert X.keydiff_scores(kk).min() >= 0 and X.keydiff_scores(kk).max() <= 2


def test_paged_rows_on_a_hand_made_pool_and_against_the_generator_scatter():
    # two sequences, one head, blocks of 2 rows, d = 1: pool rows written out by hand
    pool = np.array([[[[10.], [11.]]], [[[20.], [21.]]], [[[30.], [31.]]], [[[40.], [41.]]]])   # [4, 1, 2, 1]
    table = np.array([[2, 0], [3, 1]])
    got = X.paged_rows(pool, table, 3)
    assert got[0, 0, :, 0].tolist() == [30., 31., 10.] and got[1, 0, :, 0].tolist() == [40., 41., 20.]
    # the generator's scatter is coded separately (block slices, not row by row): round trip
    from ea_inputs import make_block_pools
    rng = np.random.default_rng(5)
    k = rng.standard_normal((2, 3, 75, 4))
    v = rng.standard_normal((2, 3, 75, 4))
    kp, vp, tab, nb = make_block_pools(k, v, 32, seed=11)
    assert kp.shape == (nb, 3, 32, 4) and len(set(tab.ravel().tolist())) == tab.size
    np.testing.assert_array_equal(X.paged_rows(kp, tab, 75), k)
    np.testing.assert_array_equal(X.paged_rows(vp, tab, 75), v)


def test_fp8_e4m3_decode_against_the_format_and_a_library_conversion():
    # codes written out from the format's definition
    known = {0x00: 0.0, 0x01: 2.0 ** -9, 0x07: 7 * 2.0 ** -9, 0x08: 2.0 ** -6, 0x38: 1.0, 0x3C: 1.5, 0x40: 2.0,
             0x7E: 448.0, 0xB8: -1.0, 0xFE: -448.0, 0x80: -0.0}
    for code, val in known.items():
        assert X.fp8_e4m3_decode(np.array([code], np.uint8))[0] == val, hex(code)
    assert np.isnan(X.fp8_e4m3_decode(np.array([0x7F, 0xFF], np.uint8))).all()
    import torch
    codes = np.arange(256, dtype=np.uint8)
    lib = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    got = X.fp8_e4m3_decode(codes)
    assert np.array_equal(np.isnan(lib), np.isnan(got))
    ok = ~np.isnan(lib)
    assert np.array_equal(lib[ok], got[ok])
    # the generator's quantiser (torch's rounding) lands on codes whose decoded value is the nearest one
    from ea_inputs import quantize_fp8
    x = np.random.default_rng(2).standard_normal((1, 2, 50, 8)) * 3
    q, sc = quantize_fp8(x)
    back = X.fp8_e4m3_decode(q) * sc.astype(np.float64)[:, :, None, None]
    grid = np.sort(got[ok])
    y = x / sc.astype(np.float64)[:, :, None, None]
    nearest = np.abs(y[..., None] - grid).min(axis=-1)
    # (the quantiser rounds the float32 image of y: allow that rounding on top of the grid distance)
    assert np.all(np.abs(back / sc.astype(np.float64)[:, :, None, None] - y) <= nearest + 1e-6 * np.abs(y))
