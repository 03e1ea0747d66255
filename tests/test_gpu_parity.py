"""GPU parity: every C-ABI entry point against the fp64 oracle on the same seeded inputs.

Tolerances (from the benchmark spec): scores within 2e-3 relative for bf16 caches (fp32
accumulation), 1e-5 for fp32 caches; kept-index sets equal to the oracle's except where oracle
scores lie within that tolerance of the threshold, and bit-exact top-k of the kernel's own
scores; compacted bytes bit-exact given the indices."""
import numpy as np
import pytest

from ea_inputs import CONFIGS, make_layer, widen
from oracle import ea_oracle as O
from tests import parity as P
import paper_2510_00636_amd as ea

pytestmark = pytest.mark.gpu

TOL = {"bf16": 2e-3, "f32": 1e-5}
MINI = {
    "c1": (CONFIGS["c1"], dict()),                                            # the tiny fp32 config as it is
    "c2mini": (CONFIGS["c2"], dict(n=3000, window=128)),                      # ragged tail, several tiles
    "c4mini": (CONFIGS["c4"].with_(batch=2), dict(n=1500, window=128)),       # d=256, G=2, batch 2
    "c5mini": (CONFIGS["c5"], dict(n=1100, window=512, pos0=30000)),          # G=5, window 512, offset positions
    "d64bf16": (CONFIGS["c2"].with_(head_dim=64, n_q_heads=16, n_kv_heads=2), dict(n=700, window=40)),  # G=8
}


def _oracle_stats(cfg, lay, **kw):
    return O.query_stats(widen(lay["q_win"]), lay["q_pos0"], lay["inv_freq"], lay["t_next"],
                         T=cfg.horizon_T, **kw)


# ------------------------------------------------------------------------- ea_query_stats
@pytest.mark.parametrize("name", list(MINI))
def test_query_stats(name):
    cfg, kw = MINI[name]
    lay = make_layer(cfg, **kw)
    mu, sg = P.run_query_stats(cfg, lay)
    rmu, rsg = _oracle_stats(cfg, lay)
    P.check_stats(mu, sg, rmu, rsg)


@pytest.mark.parametrize("w", [2, 63, 64, 65, 131, 4096])
@pytest.mark.parametrize("dt", ["bf16", "f32"])
def test_query_stats_window_sizes(w, dt):
    """Odd tails of the two-samples-per-instruction loop, chunk boundaries of the 64-sample
    staging, and the largest window the entry point accepts."""
    cfg = (CONFIGS["c2"] if dt == "bf16" else CONFIGS["c1"]).with_(n_q_heads=3, n_kv_heads=1)
    lay = make_layer(cfg, n=max(w, 8) + 5, window=w)
    for ddof in (0, 1):
        mu, sg = P.run_query_stats(cfg, lay, ddof=ddof)
        rmu, rsg = _oracle_stats(cfg, lay, ddof=ddof)
        P.check_stats(mu, sg, rmu, rsg)


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("w", [40, 130])
def test_query_stats_many_heads(w, layout):
    """With several hundred query heads per call one workgroup takes a whole d = 128 head (all ten
    covariance tiles) instead of half of it: the decode-time shape, 40 query heads x many layers."""
    cfg = CONFIGS["c2"].with_(head_dim=128, n_q_heads=40, n_kv_heads=8, batch=10)
    lay = make_layer(cfg, n=w + 9, window=w, interleaved=bool(layout))
    mu, sg = P.run_query_stats(cfg, lay, rope_layout=layout)
    rmu, rsg = _oracle_stats(cfg, lay, **({"layout": O.INTERLEAVED} if layout else {}))
    P.check_stats(mu, sg, rmu, rsg)


@pytest.mark.parametrize("variant", ["interleaved", "ddof1", "pre_rope", "T1", "w1"])
def test_query_stats_variants(variant):
    cfg = CONFIGS["c2"].with_(n_q_heads=4, n_kv_heads=2)
    if variant == "interleaved":
        lay = make_layer(cfg, n=500, window=48, interleaved=True)
        mu, sg = P.run_query_stats(cfg, lay, rope_layout=1)
        rmu, rsg = _oracle_stats(cfg, lay, layout=O.INTERLEAVED)
    elif variant == "ddof1":
        lay = make_layer(cfg, n=500, window=48)
        mu, sg = P.run_query_stats(cfg, lay, ddof=1)
        rmu, rsg = _oracle_stats(cfg, lay, ddof=1)
    elif variant == "pre_rope":
        lay = make_layer(cfg, n=500, window=48, pre_rope_queries=True)
        mu, sg = P.run_query_stats(cfg, lay, q_is_rotated=0)
        rmu, rsg = _oracle_stats(cfg, lay, q_is_rotated=False)
    elif variant == "T1":
        lay = make_layer(cfg, n=500, window=48)
        mu, sg = P.run_query_stats(cfg, lay, T=1)
        rmu, rsg = O.query_stats(widen(lay["q_win"]), lay["q_pos0"], lay["inv_freq"], lay["t_next"], T=1)
    else:   # a single query: zero covariance
        lay = make_layer(cfg, n=500, window=1)
        mu, sg = P.run_query_stats(cfg, lay)
        rmu, rsg = _oracle_stats(cfg, lay)
        assert np.all(sg == 0)
    P.check_stats(mu, sg, rmu, rsg)


@pytest.mark.parametrize("factor", [2.0 ** 10, 2.0 ** -10, 2.0 ** 40])
def test_query_stats_bf16_is_scale_free(factor):
    """The bf16 path splits the shifted samples into fp16 halves after scaling them by a power of
    two taken from the data: windows a thousand times larger or smaller than the generator's (and
    far outside fp16 range) give the same relative accuracy."""
    from ea_inputs import bf16_bits_from_f64
    cfg = CONFIGS["c5"].with_(n_q_heads=5, n_kv_heads=1)
    lay = make_layer(cfg, n=700, window=300, pos0=12345)
    lay = dict(lay, q_win=bf16_bits_from_f64(widen(lay["q_win"]) * factor))     # exact: a power of two
    mu, sg = P.run_query_stats(cfg, lay)
    rmu, rsg = _oracle_stats(cfg, lay)
    P.check_stats(mu, sg, rmu, rsg)


# ------------------------------------------------------------------------------- ea_score
@pytest.mark.parametrize("eps", [0.02, 0.0])
@pytest.mark.parametrize("name", list(MINI))
def test_score(name, eps):
    cfg, kw = MINI[name]
    lay = make_layer(cfg, **kw)
    rmu, rsg = _oracle_stats(cfg, lay)
    mu32, sg32 = rmu.astype(np.float32), rsg.astype(np.float32)    # the call's inputs are fp32
    got = P.run_score(cfg, lay, mu32, sg32, eps)
    ref = O.scores(widen(lay["k"]), widen(lay["v"]), mu32.astype(np.float64), sg32.astype(np.float64), eps)
    P.check_scores(got, ref, TOL[cfg.dtype])


@pytest.mark.parametrize("n", [1, 31, 32, 33, 255, 257, 2049])
def test_score_ragged_sizes_and_capacity(n):
    cfg = CONFIGS["c2"].with_(n_q_heads=8, n_kv_heads=2)
    lay = make_layer(cfg, n=max(n, 8), window=8)
    lay = dict(lay, n=n, k=np.ascontiguousarray(lay["k"][:, :, :n]), v=np.ascontiguousarray(lay["v"][:, :, :n]))
    rmu, rsg = _oracle_stats(cfg, lay)
    mu32, sg32 = rmu.astype(np.float32), rsg.astype(np.float32)
    got = P.run_score(cfg, lay, mu32, sg32, 0.0, n_cap=n + 37)      # rows beyond n hold NaN
    ref = O.scores(widen(lay["k"]), widen(lay["v"]), mu32.astype(np.float64), sg32.astype(np.float64), 0.0)
    P.check_scores(got, ref, 2e-3)


@pytest.mark.parametrize("hq,hkv", [(8, 1), (16, 2), (3, 1)])
def test_score_group_shapes(hq, hkv):
    """One KV head scored by the whole grid (several tile counters), groups larger than one pass
    holds (two passes over K for 8 query heads per KV head at d = 128), and an odd group."""
    cfg = CONFIGS["c2"].with_(n_q_heads=hq, n_kv_heads=hkv)
    lay = make_layer(cfg, n=9000 + 13, window=16)
    rmu, rsg = _oracle_stats(cfg, lay)
    mu32, sg32 = rmu.astype(np.float32), rsg.astype(np.float32)
    for eps in (0.02, 0.0):
        got = P.run_score(cfg, lay, mu32, sg32, eps)
        ref = O.scores(widen(lay["k"]), widen(lay["v"]), mu32.astype(np.float64), sg32.astype(np.float64), eps)
        P.check_scores(got, ref, 2e-3)


@pytest.mark.parametrize("hq,hkv,n", [(2, 1, 4100), (3, 1, 2077), (8, 2, 1300), (2, 1, 20)])
def test_score_d256_two_heads_per_pass(hq, hkv, n):
    """Head dimension 256 with both query heads of a pair in one pass over K (extra tile's
    fragments in registers): a full pair, an odd group (last pass half empty), two passes of pairs,
    and a head shorter than one tile."""
    cfg = CONFIGS["c4"].with_(batch=1, n_q_heads=hq, n_kv_heads=hkv)
    lay = make_layer(cfg, n=max(n, 40), window=16)
    lay = dict(lay, n=n, k=np.ascontiguousarray(lay["k"][:, :, :n]), v=np.ascontiguousarray(lay["v"][:, :, :n]))
    rmu, rsg = _oracle_stats(cfg, lay)
    mu32, sg32 = rmu.astype(np.float32), rsg.astype(np.float32)
    for eps in (0.02, 0.0):
        got = P.run_score(cfg, lay, mu32, sg32, eps, n_cap=n + 5)
        ref = O.scores(widen(lay["k"]), widen(lay["v"]), mu32.astype(np.float64), sg32.astype(np.float64), eps)
        P.check_scores(got, ref, 2e-3)


def test_score_zero_covariance_and_zero_mean():
    cfg = CONFIGS["c2"].with_(n_q_heads=4, n_kv_heads=1)
    lay = make_layer(cfg, n=600, window=8)
    rmu, _ = _oracle_stats(cfg, lay)
    mu32 = rmu.astype(np.float32)
    z = np.zeros((1, 4, 128, 128), np.float32)
    got = P.run_score(cfg, lay, mu32, z, 0.0)
    ref = O.scores(widen(lay["k"]), widen(lay["v"]), mu32.astype(np.float64), z.astype(np.float64), 0.0)
    P.check_scores(got, ref, 2e-3)
    got0 = P.run_score(cfg, lay, np.zeros_like(mu32), z, 0.02)      # uniform attention 1/n
    vn = np.linalg.norm(widen(lay["v"]), axis=-1)
    P.check_scores(got0, (1.0 / 600 + 0.02) * vn, 2e-3)


@pytest.mark.parametrize("d,hq,hkv,n,kscale,decades", [(128, 8, 2, 5000, 1e3, 3), (128, 4, 1, 3000, 3e3, 5),
                                                       (64, 4, 2, 2000, 300.0, 4), (256, 2, 1, 1500, 1e3, 3),
                                                       (128, 4, 1, 3000, 1.0, 6)])
def test_score_large_keys_and_wide_range_sigma(d, hq, hkv, n, kscale, decades):
    """Keys of magnitude 1e3 (entries beyond 4096, where the squared keys of the diagonal
    correction leave fp16 range) and a covariance whose diagonal spans several decades, scaled so
    that the logits stay within a few tens."""
    import torch
    from ea_inputs import bf16_bits_from_f64
    r = np.random.default_rng(d + n)
    cfg = CONFIGS["c2"].with_(head_dim=d, n_q_heads=hq, n_kv_heads=hkv, batch=1)
    p = P.params_for(cfg, epsilon=0.02)
    sig_c = 10.0 ** (-decades * r.permutation(d) / d)
    s = np.sqrt(5.0 * 2 * d / (kscale ** 2 * (sig_c ** 2).sum()))
    q = (r.standard_normal((1, hq, 64, d)) + 0.3) * sig_c * s
    mu = q.mean(axis=2)
    c = q - mu[:, :, None]
    mu32 = mu.astype(np.float32)
    sg32 = (np.einsum("bgsi,bgsj->bgij", c, c) / 64).astype(np.float32)
    kb = bf16_bits_from_f64(r.standard_normal((1, hkv, n, d)) * kscale)
    vb = bf16_bits_from_f64(r.standard_normal((1, hkv, n, d)))
    assert np.abs(widen(kb)).max() > (4096 if kscale >= 1e3 else 0)
    ws = P.workspace(p, n, 64)
    sc = torch.empty(1, hkv, n, dtype=torch.float32, device="cuda")
    ea.score(p, P.to_dev(kb), P.to_dev(vb), n, n, P.to_dev(mu32), P.to_dev(sg32), sc, ws)
    torch.cuda.synchronize()
    ref = O.scores(widen(kb), widen(vb), mu32.astype(np.float64), sg32.astype(np.float64), 0.02)
    P.check_scores(sc.cpu().numpy(), ref, 2e-3)


def test_score_c2_full_size():
    cfg = CONFIGS["c2"]
    lay = make_layer(cfg)
    rmu, rsg = _oracle_stats(cfg, lay)
    mu32, sg32 = rmu.astype(np.float32), rsg.astype(np.float32)
    for eps in (0.02, 0.0):
        got = P.run_score(cfg, lay, mu32, sg32, eps)
        ref = O.scores(widen(lay["k"]), widen(lay["v"]), mu32.astype(np.float64), sg32.astype(np.float64), eps)
        P.check_scores(got, ref, 2e-3)


# ------------------------------------------------------------------------------ ea_select
@pytest.mark.parametrize("n,n_keep", [(1, 1), (1, 0), (5, 3), (4096, 2048), (4097, 1), (5000, 4999),
                                      (5000, 5000), (16384, 9000), (16385, 1), (16385, 16384), (20000, 7),
                                      (32768, 30000), (32769, 1), (32769, 32768),
                                      (70000, 35000), (70001, 69999)])
def test_select_exact(n, n_keep):
    # heads of up to 16384 scores are selected by one workgroup out of LDS, longer ones by the
    # multi-launch histogram path: sizes on both sides of the switch
    cfg = CONFIGS["c2"].with_(batch=2, n_kv_heads=3, n_q_heads=3)
    r = np.random.default_rng(n * 7 + n_keep)
    sc = np.exp(r.standard_normal((2, 3, n))).astype(np.float32)
    sc[0, 0] = np.float32(0.5)                                       # every score equal
    sc[0, 1] = r.integers(0, 5, n).astype(np.float32)                # few distinct values, zeros
    sc[1, 0, ::3] = sc[1, 0, 0]                                      # ties at one value
    sc[1, 1] = np.sort(sc[1, 1])                                     # best pairs at the tail
    sc[1, 2] = np.sort(sc[1, 2])[::-1]                               # best pairs at the head
    got = P.run_select(cfg, sc, n_keep)
    assert np.array_equal(got.astype(np.int64), O.select(sc.astype(np.float64), n_keep))


def test_select_denormal_and_huge_scores():
    cfg = CONFIGS["c2"].with_(batch=1, n_kv_heads=1, n_q_heads=1)
    r = np.random.default_rng(3)
    sc = np.concatenate([r.random(3000) * 1e-42, r.random(3000) * 3e38, [0.0] * 50]).astype(np.float32)
    sc = r.permutation(sc)[None, None]
    for kk in (1, 3000, 3025, 6049):
        got = P.run_select(cfg, sc, kk)
        assert np.array_equal(got.astype(np.int64), O.select(sc.astype(np.float64), kk))
    # the same values repeated past the single-workgroup limit: the multi-launch path
    sc = np.tile(sc, (1, 1, 6))
    for kk in (1, 18000, 18150, 36299):
        got = P.run_select(cfg, sc, kk)
        assert np.array_equal(got.astype(np.int64), O.select(sc.astype(np.float64), kk))


# ----------------------------------------------------------------------------- ea_compact
def _masks(n, r):
    yield "half_random", np.sort(r.choice(n, n // 2, replace=False))
    yield "tail_only", np.arange(n - n // 3, n)
    yield "head_only", np.arange(n // 3)
    yield "everything", np.arange(n)
    yield "alternate", np.arange(1, n, 2)
    yield "shift_by_one", np.arange(1, n)
    yield "prefix_then_gap", np.concatenate([np.arange(n // 4), np.arange(n // 2, n)])
    yield "single_last", np.array([n - 1])


@pytest.mark.parametrize("inplace", [True, False])
@pytest.mark.parametrize("shape", ["d128bf16", "d256bf16", "d64f32", "d64bf16"])
def test_compact_bit_exact(shape, inplace):
    cfg = {"d128bf16": CONFIGS["c2"].with_(n_kv_heads=2, n_q_heads=2),
           "d256bf16": CONFIGS["c4"].with_(batch=1, n_kv_heads=2, n_q_heads=2),
           "d64f32": CONFIGS["c1"],
           "d64bf16": CONFIGS["c2"].with_(head_dim=64, n_kv_heads=2, n_q_heads=2)}[shape]
    n, n_cap = 3001, 3100
    r = np.random.default_rng(11)
    B, H, d = cfg.batch, cfg.n_kv_heads, cfg.head_dim
    if cfg.dtype == "bf16":
        k = r.integers(0, 2 ** 16, (B, H, n_cap, d)).astype(np.uint16)
        v = r.integers(0, 2 ** 16, (B, H, n_cap, d)).astype(np.uint16)
    else:
        k = r.standard_normal((B, H, n_cap, d)).astype(np.float32)
        v = r.standard_normal((B, H, n_cap, d)).astype(np.float32)
    for name, m in _masks(n, r):
        idx = np.broadcast_to(m, (B, H, len(m))).copy()
        if name == "half_random":                       # a different mask per head
            for b in range(B):
                for h in range(H):
                    idx[b, h] = np.sort(r.choice(n, len(m), replace=False))
        ko, vo = P.run_compact(cfg, k, v, n, idx, inplace=inplace)
        # rows past n_keep are left alone: the old rows in place, the fresh buffers' zeros otherwise
        P.check_compaction(ko, vo, k, v, idx, len(m), rest="same" if inplace else "zero")


@pytest.mark.parametrize("n_keep", [1, 95, 96, 97, 191, 192, 193, 959, 960, 961])
def test_compact_kept_counts_around_chunk_multiples(n_keep):
    # in place, kept counts just below, at and just above whole chunks of destination rows
    cfg = CONFIGS["c2"].with_(n_kv_heads=3, n_q_heads=3)
    n = 1500
    r = np.random.default_rng(1000 + n_keep)
    k = r.integers(0, 2 ** 16, (1, 3, n, 128)).astype(np.uint16)
    v = r.integers(0, 2 ** 16, (1, 3, n, 128)).astype(np.uint16)
    idx = np.stack([np.sort(r.choice(n, n_keep, replace=False)),          # scattered
                    np.arange(n - n_keep, n),                             # the tail, moved to the front
                    np.arange(n_keep)])[None]                             # identity: nothing moves
    ko, vo = P.run_compact(cfg, k, v, n, idx, inplace=True)
    P.check_compaction(ko, vo, k, v, idx, n_keep)
    assert np.array_equal(ko[:, 2], k[:, 2]) and np.array_equal(vo[:, 2], v[:, 2])
    assert np.array_equal(ko[:, :, n_keep:][:, 0], k[:, :, n_keep:][:, 0])


def test_compact_large_in_place_hazards():
    # many chunks, strongly overlapping source/destination ranges
    cfg = CONFIGS["c2"].with_(n_kv_heads=4, n_q_heads=4)
    n = 40000
    r = np.random.default_rng(12)
    k = r.integers(0, 2 ** 16, (1, 4, n, 128)).astype(np.uint16)
    v = r.integers(0, 2 ** 16, (1, 4, n, 128)).astype(np.uint16)
    idx = np.stack([np.arange(100, n),                                    # shift by 100
                    np.sort(r.choice(n, n - 100, replace=False)),         # sparse holes
                    np.arange(n - (n - 100), n),                          # same as shift
                    np.concatenate([np.arange(20000), np.arange(20100, n)])])[None]
    ko, vo = P.run_compact(cfg, k, v, n, idx, inplace=True)
    P.check_compaction(ko, vo, k, v, idx, n - 100)


# ---------------------------------------------------------------------- ea_compress_layer
@pytest.mark.parametrize("eps", [0.02, 0.0])
@pytest.mark.parametrize("name", list(MINI))
def test_compress_layer(name, eps):
    cfg, kw = MINI[name]
    lay = make_layer(cfg, **kw)
    n = lay["n"]
    n_keep = int(n * cfg.keep)
    got = P.run_compress_layer(cfg, lay, n_keep, epsilon=eps)
    ref = O.compress_layer(widen(lay["q_win"]), widen(lay["k"]), widen(lay["v"]), lay["q_pos0"],
                           lay["inv_freq"], lay["t_next"], n_keep, T=cfg.horizon_T, epsilon=eps,
                           k_store=lay["k"], v_store=lay["v"])
    P.check_layer(cfg, lay, got, ref, n_keep, TOL[cfg.dtype])


@pytest.mark.parametrize("n_keep", [0, 1, 999, 1000])
def test_compress_layer_edge_budgets(n_keep):
    cfg = CONFIGS["c2"].with_(n_q_heads=8, n_kv_heads=2)
    lay = make_layer(cfg, n=1000, window=32)
    got = P.run_compress_layer(cfg, lay, n_keep)
    ref = O.compress_layer(widen(lay["q_win"]), widen(lay["k"]), widen(lay["v"]), lay["q_pos0"],
                           lay["inv_freq"], lay["t_next"], n_keep, T=cfg.horizon_T,
                           epsilon=cfg.epsilon, k_store=lay["k"], v_store=lay["v"])
    P.check_layer(cfg, lay, got, ref, n_keep, 2e-3)
    if n_keep in (0, 1000):                         # nothing moves
        assert np.array_equal(got["k"], lay["k"]) and np.array_equal(got["v"], lay["v"])


def test_compress_layer_without_optional_outputs_matches():
    """The softmax sums are combined in a fixed order, so two calls on the same input give the
    same bits: the compacted cache of a call without the optional outputs equals that of a call
    with them."""
    cfg = CONFIGS["c2"].with_(n_q_heads=8, n_kv_heads=2)
    lay = make_layer(cfg, n=2000, window=64)
    a = P.run_compress_layer(cfg, lay, 1000)
    b = P.run_compress_layer(cfg, lay, 1000, want_scores=False, want_idx=False)
    assert np.array_equal(a["k"], b["k"]) and np.array_equal(a["v"], b["v"])
    P.check_compaction(b["k"], b["v"], lay["k"], lay["v"], a["idx"], 1000)


@pytest.mark.parametrize("shape", ["g4_long", "g5", "d256"])
def test_compress_layer_is_bit_reproducible(shape):
    """Tiles are dealt to workgroups at run time; scores, kept sets and bytes must not depend on
    how.  Five calls on the same input, on a device kept busy differently each time."""
    import torch
    cfg, kw = {"g4_long": (CONFIGS["c2"], dict(n=50000, window=128)),
               "g5": (CONFIGS["c5"], dict(n=4608, window=512, pos0=30000)),
               "d256": (CONFIGS["c4"].with_(batch=1), dict(n=9000, window=128))}[shape]
    lay = make_layer(cfg, **kw)
    n_keep = lay["n"] // 2
    first = None
    side = torch.cuda.Stream()
    junk = torch.empty(1 << 26, dtype=torch.float32, device="cuda")
    for rep in range(5):
        with torch.cuda.stream(side):               # unrelated load on another stream
            for _ in range(rep):
                junk.mul_(1.0001)
        got = P.run_compress_layer(cfg, lay, n_keep, epsilon=0.0)
        torch.cuda.synchronize()
        if first is None:
            first = got
        else:
            for key in ("scores", "idx", "k", "v"):
                assert np.array_equal(first[key], got[key]), (shape, rep, key)


def test_compress_layer_c2_full_size():
    cfg = CONFIGS["c2"]
    lay = make_layer(cfg)
    n_keep = cfg.n_keep
    for eps in (0.02, 0.0):
        got = P.run_compress_layer(cfg, lay, n_keep, epsilon=eps)
        ref = O.compress_layer(widen(lay["q_win"]), widen(lay["k"]), widen(lay["v"]), lay["q_pos0"],
                               lay["inv_freq"], lay["t_next"], n_keep, T=cfg.horizon_T, epsilon=eps,
                               k_store=lay["k"], v_store=lay["v"])
        P.check_layer(cfg, lay, got, ref, n_keep, 2e-3)


def test_layers_on_concurrent_streams_match_sequential():
    """Layers are independent: compressing them on several streams, each with its own workspace
    (the launch configuration bench.py times), gives what the one-stream order gives."""
    import torch
    cfg = CONFIGS["c2"].with_(n_q_heads=8, n_kv_heads=2)
    n, w, n_keep, L = 6000, 64, 3000, 6
    lays = [make_layer(cfg, layer=l, n=n, window=w) for l in range(L)]
    seq = [P.run_compress_layer(cfg, lay, n_keep) for lay in lays]
    p = P.params_for(cfg)
    ns = 3
    streams = [torch.cuda.Stream() for _ in range(ns)]
    wss = [P.workspace(p, n, w) for _ in range(ns)]
    dev = [dict(q=P.to_dev(lay["q_win"]), k=P.to_dev(lay["k"]), v=P.to_dev(lay["v"]),
                f=P.to_dev(lay["inv_freq"])) for lay in lays]
    idx = [torch.full((cfg.batch, cfg.n_kv_heads, n_keep), -1, dtype=torch.int32, device="cuda")
           for _ in range(L)]
    scs = [torch.zeros(cfg.batch, cfg.n_kv_heads, n, dtype=torch.float32, device="cuda") for _ in range(L)]
    torch.cuda.synchronize()
    for rep in range(2):                            # second round: workspaces are reused dirty
        if rep == 1:
            for l, lay in enumerate(lays):
                dev[l]["k"].copy_(P.to_dev(lay["k"]))
                dev[l]["v"].copy_(P.to_dev(lay["v"]))
            torch.cuda.synchronize()
        for l, lay in enumerate(lays):
            ea.compress_layer(p, dev[l]["q"], w, lay["q_pos0"], dev[l]["f"], lay["t_next"], dev[l]["k"],
                              dev[l]["v"], n, n, n_keep, scs[l], idx[l], wss[l % ns], stream=streams[l % ns])
        torch.cuda.synchronize()
        # the softmax sums are combined in a fixed order whatever the scheduling: same bits
        for l, lay in enumerate(lays):
            got_idx, got_sc = idx[l].cpu().numpy(), scs[l].cpu().numpy()
            assert np.array_equal(got_sc, seq[l]["scores"]), (rep, l)
            assert np.array_equal(got_idx, seq[l]["idx"]), (rep, l)
            assert np.array_equal(P.to_host(dev[l]["k"]), seq[l]["k"]), (rep, l)
            assert np.array_equal(P.to_host(dev[l]["v"]), seq[l]["v"]), (rep, l)


def test_compress_layer_replayed_from_a_graph_matches_eager():
    """The library only enqueues kernels (its counters are cleared by a kernel, not a memset
    node), so a call can be captured in a HIP graph as it is.  The graph is replayed several
    times, with eager work and synchronisation in between and the cache restored each time;
    every replay must give what the eager call gives.  Two shapes: a long head (multi-launch
    selection) and a short one (single-launch selection)."""
    import torch
    for n, w, n_keep in ((40000, 64, 17000), (3000, 64, 1100)):
        cfg = CONFIGS["c2"].with_(n_q_heads=8, n_kv_heads=2)
        lay = make_layer(cfg, layer=3, n=n, window=w)
        ref = P.run_compress_layer(cfg, lay, n_keep)
        p = P.params_for(cfg)
        ws = P.workspace(p, n, w)
        q, f = P.to_dev(lay["q_win"]), P.to_dev(lay["inv_freq"])
        k, v = P.to_dev(lay["k"]), P.to_dev(lay["v"])
        k0, v0 = k.clone(), v.clone()
        idx = torch.full((cfg.batch, cfg.n_kv_heads, n_keep), -1, dtype=torch.int32, device="cuda")
        sc = torch.zeros(cfg.batch, cfg.n_kv_heads, n, dtype=torch.float32, device="cuda")
        cap = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=cap):
            ea.compress_layer(p, q, w, lay["q_pos0"], f, lay["t_next"], k, v, n, n, n_keep, sc, idx, ws,
                              stream=cap)
        torch.cuda.synchronize()
        for rep in range(3):
            k.copy_(k0)
            v.copy_(v0)
            idx.fill_(-1)
            sc.zero_()
            ws.random_(0, 255)                      # the workspace may hold anything between calls
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            got_sc, got_idx = sc.cpu().numpy(), idx.cpu().numpy()
            assert np.array_equal(got_sc, ref["scores"]), (n, rep)
            assert np.array_equal(got_idx, ref["idx"]), (n, rep)
            assert np.array_equal(P.to_host(k), ref["k"]) and np.array_equal(P.to_host(v), ref["v"]), (n, rep)


# ------------------------------------------------------- fp32 caches at d = 128 and d = 256
@pytest.mark.parametrize("d", [128, 256])
def test_fp32_path_at_larger_head_dims(d):
    """The fp32 instances of the statistics, score and compaction kernels beyond the d = 64 of
    the small fp32 configuration."""
    cfg = CONFIGS["c1"].with_(head_dim=d, n_q_heads=4, n_kv_heads=2)
    lay = make_layer(cfg, n=700, window=48)
    mu, sg = P.run_query_stats(cfg, lay)
    rmu, rsg = _oracle_stats(cfg, lay)
    P.check_stats(mu, sg, rmu, rsg)
    n_keep = 333
    for eps in (0.02, 0.0):
        got = P.run_compress_layer(cfg, lay, n_keep, epsilon=eps)
        ref = O.compress_layer(widen(lay["q_win"]), widen(lay["k"]), widen(lay["v"]), lay["q_pos0"],
                               lay["inv_freq"], lay["t_next"], n_keep, T=cfg.horizon_T, epsilon=eps,
                               k_store=lay["k"], v_store=lay["v"])
        P.check_layer(cfg, lay, got, ref, n_keep, 1e-5)


# ---------------------------------------------------------------- out-of-domain inputs are visible
def test_status_word_reports_bad_scores_and_bad_indices():
    import torch
    cfg = CONFIGS["c2"].with_(batch=1, n_kv_heads=2, n_q_heads=2)
    p = P.params_for(cfg)
    for n in (3000, 40000):                          # one-launch and multi-launch selection
        ws = P.workspace(p, n, 1)
        r = np.random.default_rng(n)
        sc = r.random((1, 2, n)).astype(np.float32)
        idx = torch.zeros(1, 2, n // 2, dtype=torch.int32, device="cuda")
        ea.select(p, P.to_dev(sc), n, n // 2, idx, ws)
        assert ea.debug_status(p, n, 1, ws) == 0
        bad = sc.copy()
        bad[0, 1, n // 3] = np.nan
        bad[0, 0, 7] = -1.0
        ea.select(p, P.to_dev(bad), n, n // 2, idx, ws)
        assert ea.debug_status(p, n, 1, ws) & ea.STATUS_BAD_SCORE
        ea.select(p, P.to_dev(sc), n, n // 2, idx, ws)          # the next call starts clean
        assert ea.debug_status(p, n, 1, ws) == 0
    n, n_keep = 3000, 1000
    ws = P.workspace(p, n, 1)
    k = r.integers(0, 2 ** 16, (1, 2, n, 128)).astype(np.uint16)
    good = np.sort(r.choice(n, n_keep, replace=False)).astype(np.int32)
    twisted = good.copy()
    twisted[500], twisted[501] = twisted[501], twisted[500]     # not ascending
    for inplace in (False, True):
        kd, vd = P.to_dev(k), P.to_dev(k[:, :, ::-1].copy())
        ko, vo = (kd, vd) if inplace else (torch.zeros_like(kd), torch.zeros_like(vd))
        ea.compact(p, kd, vd, n, n, P.to_dev(np.broadcast_to(good, (1, 2, n_keep)).copy()), n_keep, ko, vo, ws)
        assert ea.debug_status(p, n, 1, ws) == 0
        kd, vd = P.to_dev(k), P.to_dev(k[:, :, ::-1].copy())
        ko, vo = (kd, vd) if inplace else (torch.zeros_like(kd), torch.zeros_like(vd))
        ea.compact(p, kd, vd, n, n, P.to_dev(np.broadcast_to(twisted, (1, 2, n_keep)).copy()), n_keep, ko, vo, ws)
        assert ea.debug_status(p, n, 1, ws) & ea.STATUS_BAD_INDEX


# ------------------------------------------------------------------- order-free compaction
@pytest.mark.parametrize("shape", ["d128bf16", "d256bf16", "d64f32"])
def test_compact_unordered_bit_exact(shape):
    """Rows in front are exactly the oracle's permutation of the kept rows (so also the same set),
    rows from n_keep on are untouched, and perm_out names the source of every position."""
    import torch
    from oracle import ea_extensions as X
    cfg = {"d128bf16": CONFIGS["c2"].with_(n_kv_heads=2, n_q_heads=2),
           "d256bf16": CONFIGS["c4"].with_(batch=1, n_kv_heads=2, n_q_heads=2),
           "d64f32": CONFIGS["c1"]}[shape]
    p = P.params_for(cfg)
    n, n_cap = 3001, 3050
    r = np.random.default_rng(21)
    B, H, d = cfg.batch, cfg.n_kv_heads, cfg.head_dim
    if cfg.dtype == "bf16":
        k = r.integers(0, 2 ** 16, (B, H, n_cap, d)).astype(np.uint16)
        v = r.integers(0, 2 ** 16, (B, H, n_cap, d)).astype(np.uint16)
    else:
        k = r.standard_normal((B, H, n_cap, d)).astype(np.float32)
        v = r.standard_normal((B, H, n_cap, d)).astype(np.float32)
    for name, m in _masks(n, r):
        idx = np.broadcast_to(m, (B, H, len(m))).copy()
        if name == "half_random":
            for b in range(B):
                for h in range(H):
                    idx[b, h] = np.sort(r.choice(n, len(m), replace=False))
        nk = len(m)
        kd, vd = P.to_dev(k), P.to_dev(v)
        perm = torch.full((B, H, nk), -1, dtype=torch.int32, device="cuda")
        ea.compact_unordered(p, kd, vd, n, n_cap, P.to_dev(idx.astype(np.int32)), nk, perm)
        torch.cuda.synchronize()
        ko, vo = P.to_host(kd), P.to_host(vd)
        rk, rv, rperm = X.compact_unordered(k, v, idx.astype(np.int64))
        assert np.array_equal(perm.cpu().numpy(), rperm), name
        assert np.array_equal(ko[:, :, :nk], rk) and np.array_equal(vo[:, :, :nk], rv), name
        assert np.array_equal(ko[:, :, nk:], k[:, :, nk:]) and np.array_equal(vo[:, :, nk:], v[:, :, nk:]), name


def test_compress_layer_unordered_decode_shape():
    """The decode-time pass (4608 -> 4096 pairs) with the order-free last step: same scores and kept
    set as the ordered call, rows in front = the oracle's permutation."""
    import torch
    from oracle import ea_extensions as X
    cfg = CONFIGS["c5"]
    lay = make_layer(cfg, n=4608, window=512, pos0=20000)
    n, w, n_keep = 4608, 512, 4096
    ref = P.run_compress_layer(cfg, lay, n_keep)
    p = P.params_for(cfg)
    ws = P.workspace(p, n, w)
    kd, vd = P.to_dev(lay["k"]), P.to_dev(lay["v"])
    sc = torch.empty(cfg.batch, cfg.n_kv_heads, n, dtype=torch.float32, device="cuda")
    idx = torch.empty(cfg.batch, cfg.n_kv_heads, n_keep, dtype=torch.int32, device="cuda")
    perm = torch.empty_like(idx)
    ea.compress_layer_unordered(p, P.to_dev(lay["q_win"]), w, lay["q_pos0"], P.to_dev(lay["inv_freq"]),
                                lay["t_next"], kd, vd, n, n, n_keep, sc, idx, perm, ws)
    torch.cuda.synchronize()
    assert np.array_equal(sc.cpu().numpy(), ref["scores"]) and np.array_equal(idx.cpu().numpy(), ref["idx"])
    rk, rv, rperm = X.compact_unordered(lay["k"], lay["v"], ref["idx"].astype(np.int64))
    assert np.array_equal(perm.cpu().numpy(), rperm)
    assert np.array_equal(P.to_host(kd)[:, :, :n_keep], rk) and np.array_equal(P.to_host(vd)[:, :, :n_keep], rv)


# ------------------------------------------------------------------- comparison scorers
@pytest.mark.parametrize("name", ["c1", "c2mini", "c4mini", "d64bf16"])
def test_baseline_scorers(name):
    """KNorm, StreamingLLM and KeyDiff scores against their oracle definitions, and the kept sets
    they lead to through ea_select."""
    import torch
    from oracle import ea_extensions as X
    cfg, kw = MINI[name]
    lay = make_layer(cfg, **kw)
    n = lay["n"]
    p = P.params_for(cfg)
    ws = P.workspace(p, n, 1)
    kd = P.to_dev(lay["k"])
    k64 = widen(lay["k"])
    sc = torch.empty(cfg.batch, cfg.n_kv_heads, n, dtype=torch.float32, device="cuda")
    n_keep = n // 3
    idx = torch.empty(cfg.batch, cfg.n_kv_heads, n_keep, dtype=torch.int32, device="cuda")
    for scorer, ref, tol, atol in ((ea.SCORER_KNORM, X.knorm_scores(k64), 1e-5, 0.0),
                                   (ea.SCORER_STREAMING, X.streaming_scores(cfg.batch, cfg.n_kv_heads, n, 4), 0.0, 0.0),
                                   (ea.SCORER_KEYDIFF, X.keydiff_scores(k64), 1e-5, 2e-6)):
        ea.score_baseline(p, scorer, kd, n, n, 4, sc, ws)
        ea.select(p, sc, n, n_keep, idx, ws)
        torch.cuda.synchronize()
        got = sc.cpu().numpy().astype(np.float64)
        if scorer != ea.SCORER_STREAMING:
            assert np.all(np.abs(got - ref) <= tol * np.abs(ref) + atol)
        if scorer == ea.SCORER_STREAMING:
            assert np.array_equal(got, ref)
            assert np.array_equal(idx.cpu().numpy().astype(np.int64), O.select(ref, n_keep))
        else:
            P.check_idx_exact_given_scores(idx.cpu().numpy(), sc.cpu().numpy(), n_keep)
            # kept set vs the oracle's, up to scores within the tolerance band of the threshold
            for b in range(cfg.batch):
                for h in range(cfg.n_kv_heads):
                    s = ref[b, h]
                    thr = np.sort(s)[n - n_keep]
                    band = tol * abs(thr) + atol
                    kept = np.zeros(n, bool)
                    kept[idx[b, h].cpu().numpy()] = True
                    assert kept[s > thr + 2 * band].all() and not kept[s < thr - 2 * band].any()


# ------------------------------------------------------------------- head-adaptive budgets
@pytest.mark.parametrize("n,n_keep,floor", [(700, 300, 0), (700, 300, 40), (700, 300, 300), (700, 0, 0),
                                            (20000, 9000, 0), (20000, 9000, 500), (5, 3, 1)])
def test_select_adaptive_and_ragged_compaction(n, n_keep, floor):
    """Pooled selection over the KV heads of every sequence against the oracle's flat stable sort
    (bit-exact lists and lengths), then the ragged in-place gather against fancy indexing."""
    import torch
    from oracle import ea_extensions as X
    cfg = CONFIGS["c2"].with_(batch=2, n_kv_heads=4, n_q_heads=4)
    p = P.params_for(cfg)
    r = np.random.default_rng(n + n_keep + floor)
    sc = np.exp(1.5 * r.standard_normal((2, 4, n))).astype(np.float32)
    sc[:, 1] *= 8.0                                        # a head that earns more than its share
    sc[0, 2, ::4] = sc[0, 2, 0]                            # ties inside a head
    sc[1, 0] = sc[1, 3]                                    # ties across heads
    ws = P.workspace(p, n, 1)
    idx = torch.full((2, 4, n), -7, dtype=torch.int32, device="cuda")
    lengths = torch.full((2, 4), -1, dtype=torch.int32, device="cuda")
    ea.select_adaptive(p, P.to_dev(sc), n, n_keep, floor, idx, lengths, ws)
    torch.cuda.synchronize()
    rl, rk = X.select_adaptive(sc.astype(np.float64), n_keep, floor)
    gl, gi = lengths.cpu().numpy(), idx.cpu().numpy()
    assert np.array_equal(gl, rl)
    for b in range(2):
        for h in range(4):
            assert np.array_equal(gi[b, h, :gl[b, h]], rk[b][h]), (b, h)
            assert np.all(gi[b, h, gl[b, h]:] == -7)
    k = r.integers(0, 2 ** 16, (2, 4, n + 9, 128)).astype(np.uint16)
    v = r.integers(0, 2 ** 16, (2, 4, n + 9, 128)).astype(np.uint16)
    kd, vd = P.to_dev(k), P.to_dev(v)
    ea.compact_ragged(p, kd, vd, n, n + 9, idx, lengths, ws)
    torch.cuda.synchronize()
    assert ea.debug_status(p, n, 1, ws) == 0
    ko, vo = P.to_host(kd), P.to_host(vd)
    ref = X.compact_ragged(k, v, rk)
    for b in range(2):
        for h in range(4):
            m = gl[b, h]
            assert np.array_equal(ko[b, h, :m], ref[b][h][0]) and np.array_equal(vo[b, h, :m], ref[b][h][1])
            assert np.array_equal(ko[b, h, m:], k[b, h, m:]) and np.array_equal(vo[b, h, m:], v[b, h, m:])


# ------------------------------------------------------------------- hidden-state front end (Eq. 5 as printed)
@pytest.mark.parametrize("dt,d,w,dm", [("bf16", 128, 128, 512), ("f32", 64, 40, 200), ("bf16", 256, 70, 96),
                                      ("bf16", 128, 300, 4096), ("bf16", 64, 33, 72), ("bf16", 128, 50, 130),
                                      ("bf16", 128, 2, 64)])
def test_query_stats_from_hidden_states(dt, d, w, dm):
    """mu, Sigma from a hidden-state buffer and W_Q against the oracle's literal Eq. 5 (mean and
    covariance of the hidden states, then W_Q, then R-bar)."""
    import torch
    from oracle import ea_extensions as X
    from ea_inputs import bf16_bits_from_f64, inv_freq_table
    cfg = (CONFIGS["c2"] if dt == "bf16" else CONFIGS["c1"]).with_(head_dim=d, n_q_heads=4, n_kv_heads=2, batch=2)
    p = P.params_for(cfg)
    r = np.random.default_rng(d + w + dm)
    hidden = r.standard_normal((2, w, dm)) * 1.5 + r.standard_normal(dm)          # channels with offsets
    w_q = r.standard_normal((4, d, dm)) / np.sqrt(dm)
    if dt == "bf16":
        hb, wb = bf16_bits_from_f64(hidden), bf16_bits_from_f64(w_q)
        h64, w64 = widen(hb), widen(wb)
    else:
        hb, wb = hidden.astype(np.float32), w_q.astype(np.float32)
        h64, w64 = hb.astype(np.float64), wb.astype(np.float64)
    inv = inv_freq_table(d, cfg.rope_base)
    t_next = 70000
    ws = P.workspace(p, 8, w)
    mu = torch.empty(2, 4, d, dtype=torch.float32, device="cuda")
    sg = torch.empty(2, 4, d, d, dtype=torch.float32, device="cuda")
    ea.query_stats_hidden(p, P.to_dev(hb), P.to_dev(wb), dm, w, P.to_dev(inv), t_next, mu, sg, ws)
    torch.cuda.synchronize()
    rmu, rsg = X.query_stats_hidden(h64, w64, inv, t_next, T=cfg.horizon_T)
    P.check_stats(mu.cpu().numpy(), sg.cpu().numpy(), rmu, rsg)


# ------------------------------------------------------------------- Eq. 9 as printed: ||W_o v||
@pytest.mark.parametrize("dt,d,hq,hkv,n,dm", [("bf16", 128, 8, 2, 3000, 256), ("bf16", 128, 5, 1, 700, 96),
                                              ("bf16", 64, 4, 2, 1100, 130), ("bf16", 256, 2, 1, 900, 64),
                                              ("f32", 64, 4, 2, 500, 72)])
def test_scores_with_output_projection(dt, d, hq, hkv, n, dm):
    """ea_wo_gram + ea_value_norms_wo + ea_score_wo against the oracle's explicit W_o v products."""
    import torch
    from oracle import ea_extensions as X
    from ea_inputs import bf16_bits_from_f64
    cfg = (CONFIGS["c2"] if dt == "bf16" else CONFIGS["c1"]).with_(head_dim=d, n_q_heads=hq, n_kv_heads=hkv, batch=2)
    lay = make_layer(cfg, n=n, window=16)
    p = P.params_for(cfg, epsilon=0.02)
    rmu, rsg = _oracle_stats(cfg, lay)
    mu32, sg32 = rmu.astype(np.float32), rsg.astype(np.float32)
    r = np.random.default_rng(n + dm)
    w_o = r.standard_normal((hq, dm, d)) / np.sqrt(d) * (1.0 + np.arange(hq))[:, None, None]
    if dt == "bf16":
        wb = bf16_bits_from_f64(w_o)
        w64 = widen(wb)
    else:
        wb = w_o.astype(np.float32)
        w64 = wb.astype(np.float64)
    ws = P.workspace(p, n, 16)
    gram = torch.empty(hq, d, d, dtype=torch.float32, device="cuda")
    wnorm = torch.empty(2, hq, n, dtype=torch.float32, device="cuda")
    scores = torch.empty(2, hkv, n, dtype=torch.float32, device="cuda")
    kd, vd = P.to_dev(lay["k"]), P.to_dev(lay["v"])
    ea.wo_gram(p, P.to_dev(wb), dm, gram)
    ea.value_norms_wo(p, vd, n, n, gram, wnorm, ws)
    ea.score_wo(p, kd, vd, n, n, P.to_dev(mu32), P.to_dev(sg32), wnorm, scores, ws)
    torch.cuda.synchronize()
    g_ref = np.einsum("gma,gmb->gab", w64, w64)
    got_g = gram.cpu().numpy().astype(np.float64)
    assert np.abs(got_g - g_ref).max() <= 1e-5 * np.abs(g_ref).max()
    wn_ref = X.wo_value_norms(widen(lay["v"]), w64)
    tol = TOL[cfg.dtype]
    P.check_scores(wnorm.cpu().numpy(), wn_ref, tol)
    ref = X.scores_wo(widen(lay["k"]), widen(lay["v"]), mu32.astype(np.float64), sg32.astype(np.float64), w64, 0.02)
    P.check_scores(scores.cpu().numpy(), ref, 2 * tol)


# ------------------------------------------------------------------- paged (block-table) caches
def _paged_setup(cfg, lay, bs, seed):
    import torch
    from ea_inputs import make_block_pools
    kp, vp, tab, nb = make_block_pools(lay["k"], lay["v"], bs, seed)
    tabd = torch.from_numpy(tab).cuda()
    return kp, vp, tab, nb, P.to_dev(kp), P.to_dev(vp), tabd, ea.make_paged(tabd, bs, nb)


@pytest.mark.parametrize("name,n,bs", [("c2mini", 3000, 32), ("c2mini", 2049, 256), ("c4mini", 1500, 64),
                                      ("c5mini", 1100, 128), ("d64bf16", 700, 1024), ("c2mini", 17, 32),
                                      ("c2mini", 3000, 16), ("c4mini", 1511, 16), ("d64bf16", 700, 16),
                                      ("c5mini", 1097, 16), ("c2mini", 15, 16), ("c2mini", 48, 16)])
def test_score_paged(name, n, bs):
    """ea_score over block pools behind a shuffled block table: same scores as the oracle gives for
    the logical rows (the rows of a sequence's last block beyond n, and the pool's spare blocks,
    hold NaN)."""
    import torch
    from oracle import ea_extensions as X
    cfg, kw = MINI[name]
    lay = make_layer(cfg, **dict(kw, n=max(n, kw.get("window", 1) + 8)))
    lay = dict(lay, n=n, k=np.ascontiguousarray(lay["k"][:, :, :n]), v=np.ascontiguousarray(lay["v"][:, :, :n]))
    kp, vp, tab, nb, kd, vd, tabd, pg = _paged_setup(cfg, lay, bs, seed=n + bs)
    assert np.array_equal(X.paged_rows(kp, tab, n), lay["k"])
    rmu, rsg = _oracle_stats(cfg, lay)
    mu32, sg32 = rmu.astype(np.float32), rsg.astype(np.float32)
    p = P.params_for(cfg, epsilon=0.02)
    ws = P.workspace(p, n, 1)
    sc = torch.empty(cfg.batch, cfg.n_kv_heads, n, dtype=torch.float32, device="cuda")
    ea.score_paged(p, kd, vd, pg, n, P.to_dev(mu32), P.to_dev(sg32), sc, ws)
    torch.cuda.synchronize()
    ref = O.scores(widen(lay["k"]), widen(lay["v"]), mu32.astype(np.float64), sg32.astype(np.float64), 0.02)
    P.check_scores(sc.cpu().numpy(), ref, 2e-3)
    # and agrees with the contiguous call far inside the tolerance (the two may run different
    # kernels, which add the same fp16 products in different orders)
    got_c = P.run_score(cfg, lay, mu32, sg32, 0.02)
    np.testing.assert_allclose(sc.cpu().numpy(), got_c, rtol=2e-5, atol=0)


@pytest.mark.parametrize("order_free", [0, 1])
@pytest.mark.parametrize("name,n,bs", [("c2mini", 3000, 32), ("c4mini", 1500, 64), ("c5mini", 1100, 128),
                                      ("c2mini", 2990, 16), ("c4mini", 1500, 16)])
def test_compress_layer_paged(name, n, bs, order_free):
    """The whole path over a paged cache: scores, kept set and the compacted logical rows equal
    what the oracle gives on the contiguous view; pool rows outside the kept prefix are untouched."""
    import torch
    from oracle import ea_extensions as X
    cfg, kw = MINI[name]
    lay = make_layer(cfg, **dict(kw, n=n))
    w = lay["window"]
    n_keep = int(n * 0.6)
    kp, vp, tab, nb, kd, vd, tabd, pg = _paged_setup(cfg, lay, bs, seed=7 * n + bs)
    p = P.params_for(cfg, epsilon=0.02)
    ws = P.workspace(p, n, w)
    sc = torch.empty(cfg.batch, cfg.n_kv_heads, n, dtype=torch.float32, device="cuda")
    idx = torch.empty(cfg.batch, cfg.n_kv_heads, n_keep, dtype=torch.int32, device="cuda")
    perm = torch.empty_like(idx)
    ea.compress_layer_paged(p, P.to_dev(lay["q_win"]), w, lay["q_pos0"], P.to_dev(lay["inv_freq"]), lay["t_next"],
                            kd, vd, pg, n, n_keep, order_free, sc, idx, perm, ws)
    torch.cuda.synchronize()
    ref = O.compress_layer(widen(lay["q_win"]), widen(lay["k"]), widen(lay["v"]), lay["q_pos0"], lay["inv_freq"],
                           lay["t_next"], n_keep, T=cfg.horizon_T, epsilon=0.02, k_store=lay["k"], v_store=lay["v"])
    gi = idx.cpu().numpy()
    P.check_scores(sc.cpu().numpy(), ref["scores"], 2e-3)
    P.check_idx_vs_oracle_scores(gi, ref["scores"], n_keep, 2e-3)
    P.check_idx_exact_given_scores(gi, sc.cpu().numpy(), n_keep)
    ka, va = X.paged_rows(P.to_host(kd), tab, n), X.paged_rows(P.to_host(vd), tab, n)
    if order_free:
        for b in range(cfg.batch):
            for h in range(cfg.n_kv_heads):
                rperm = X.unordered_perm(gi[b, h], n_keep)
                assert np.array_equal(perm.cpu().numpy()[b, h], rperm)
                assert np.array_equal(ka[b, h, :n_keep], lay["k"][b, h][rperm])
                assert np.array_equal(va[b, h, :n_keep], lay["v"][b, h][rperm])
        assert np.array_equal(ka[:, :, n_keep:], lay["k"][:, :, n_keep:])
    else:
        P.check_compaction(ka, va, lay["k"], lay["v"], gi, n_keep)
    # nothing outside the sequences' own rows was written: spare blocks and block tails keep their marker
    used = np.zeros(kp.shape[:1] + kp.shape[2:3], bool)
    for b in range(cfg.batch):
        for i in range(n):
            used[tab[b, i // bs], i % bs] = True
    assert np.array_equal(P.to_host(kd)[~used[:, None, :].repeat(cfg.n_kv_heads, 1)],
                          kp[~used[:, None, :].repeat(cfg.n_kv_heads, 1)])


def test_compact_paged_matches_contiguous_compaction():
    """ea_compact_paged (in place, order-preserving) on adversarial kept sets: the logical rows
    equal those of ea_compact on the contiguous cache."""
    import torch
    from oracle import ea_extensions as X
    cfg = CONFIGS["c2"].with_(n_q_heads=8, n_kv_heads=2, batch=2)
    n, bs = 5000, 64
    lay = make_layer(cfg, n=n, window=8)
    r = np.random.default_rng(3)
    for name, keep in (("random", np.sort(r.choice(n, 2100, replace=False))), ("tail", np.arange(n - 1900, n)),
                       ("head", np.arange(0, 1234)), ("stride", np.arange(1, n, 3))):
        nk = len(keep)
        idx = np.broadcast_to(keep.astype(np.int32), (cfg.batch, cfg.n_kv_heads, nk)).copy()
        kp, vp, tab, nb, kd, vd, tabd, pg = _paged_setup(cfg, lay, bs, seed=nk)
        p = P.params_for(cfg)
        ws = P.workspace(p, n, 1)
        ea.compact_paged(p, kd, vd, pg, n, P.to_dev(idx), nk, 0, None, ws)
        torch.cuda.synchronize()
        ka, va = X.paged_rows(P.to_host(kd), tab, n), X.paged_rows(P.to_host(vd), tab, n)
        P.check_compaction(ka, va, lay["k"], lay["v"], idx, nk)
        assert ea.debug_status(p, n, 1, ws) == 0, name


# ------------------------------------------------------------------- caches stored as e4m3 bytes
def _fp8_layer(cfg, n, window, pos0=None):
    """A generated layer whose K and V are then stored as e4m3 bytes with per-head scales; the
    oracle sees the dequantised values (its own decoding of the bytes times the scales)."""
    from ea_inputs import quantize_fp8
    from oracle import ea_extensions as X
    kw = dict(n=n, window=window)
    if pos0 is not None:
        kw["pos0"] = pos0
    lay = make_layer(cfg, **kw)
    k8, ks = quantize_fp8(widen(lay["k"]))
    v8, vs = quantize_fp8(widen(lay["v"]))
    kd = X.fp8_e4m3_decode(k8) * ks.astype(np.float64)[:, :, None, None]
    vd = X.fp8_e4m3_decode(v8) * vs.astype(np.float64)[:, :, None, None]
    return lay, k8, v8, ks, vs, kd, vd


@pytest.mark.parametrize("name,hq,hkv,n", [("c2", 8, 2, 3000), ("c2", 5, 1, 1100), ("c2", 3, 1, 2049), ("c2", 2, 2, 700),
                                           ("c2", 1, 1, 20), ("c4", 2, 1, 1500), ("c4", 1, 1, 900), ("c4", 3, 1, 777)])
def test_score_fp8(name, hq, hkv, n):
    """ea_score_fp8 against the oracle on the dequantised cache: every group size the kernels
    instantiate at d = 128 and 256, ragged sizes, a head shorter than a tile; NaN rows beyond n."""
    import torch
    cfg = CONFIGS[name].with_(batch=2 if n > 1000 else 1, n_q_heads=hq, n_kv_heads=hkv)
    lay, k8, v8, ks, vs, kd, vd = _fp8_layer(cfg, max(n, 40), 16)
    k8, v8, kd, vd = k8[:, :, :n], v8[:, :, :n], kd[:, :, :n], vd[:, :, :n]
    lay = dict(lay, n=n)
    rmu, rsg = _oracle_stats(cfg, lay)
    mu32, sg32 = rmu.astype(np.float32), rsg.astype(np.float32)
    n_cap = n + 11
    pad = [(0, 0), (0, 0), (0, n_cap - n), (0, 0)]
    k8p, v8p = np.pad(k8, pad, constant_values=0x7F), np.pad(v8, pad, constant_values=0x7F)     # NaN codes
    p = P.params_for(cfg, epsilon=0.02)
    ws = P.workspace(p, n, 1)
    sc = torch.empty(cfg.batch, hkv, n, dtype=torch.float32, device="cuda")
    ea.score_fp8(p, torch.from_numpy(k8p).cuda(), torch.from_numpy(v8p).cuda(), torch.from_numpy(ks).cuda(),
                 torch.from_numpy(vs).cuda(), n, n_cap, P.to_dev(mu32), P.to_dev(sg32), sc, ws)
    torch.cuda.synchronize()
    ref = O.scores(kd, vd, mu32.astype(np.float64), sg32.astype(np.float64), 0.02)
    P.check_scores(sc.cpu().numpy(), ref, 2e-3)


@pytest.mark.parametrize("order_free", [0, 1])
@pytest.mark.parametrize("name,n,w", [("c2", 3000, 128), ("c4", 1500, 64), ("c5", 1100, 512)])
def test_compress_layer_fp8(name, n, w, order_free):
    import torch
    from oracle import ea_extensions as X
    cfg = CONFIGS[name].with_(batch=1) if name == "c4" else CONFIGS[name]
    lay, k8, v8, ks, vs, kd, vd = _fp8_layer(cfg, n, w, pos0=30000 if name == "c5" else None)
    n_keep = int(n * 0.55)
    p = P.params_for(cfg, epsilon=0.02)
    ws = P.workspace(p, n, w)
    k8d, v8d = torch.from_numpy(k8).cuda(), torch.from_numpy(v8).cuda()
    sc = torch.empty(cfg.batch, cfg.n_kv_heads, n, dtype=torch.float32, device="cuda")
    idx = torch.empty(cfg.batch, cfg.n_kv_heads, n_keep, dtype=torch.int32, device="cuda")
    perm = torch.empty_like(idx)
    ea.compress_layer_fp8(p, P.to_dev(lay["q_win"]), w, lay["q_pos0"], P.to_dev(lay["inv_freq"]), lay["t_next"],
                          k8d, v8d, torch.from_numpy(ks).cuda(), torch.from_numpy(vs).cuda(), n, n, n_keep,
                          order_free, sc, idx, perm, ws)
    torch.cuda.synchronize()
    ref = O.compress_layer(widen(lay["q_win"]), kd, vd, lay["q_pos0"], lay["inv_freq"], lay["t_next"], n_keep,
                           T=cfg.horizon_T, epsilon=0.02, k_store=k8, v_store=v8)
    gi = idx.cpu().numpy()
    P.check_scores(sc.cpu().numpy(), ref["scores"], 2e-3)
    P.check_idx_vs_oracle_scores(gi, ref["scores"], n_keep, 2e-3)
    P.check_idx_exact_given_scores(gi, sc.cpu().numpy(), n_keep)
    ka, va = k8d.cpu().numpy(), v8d.cpu().numpy()
    if order_free:
        for b in range(cfg.batch):
            for h in range(cfg.n_kv_heads):
                rperm = X.unordered_perm(gi[b, h], n_keep)
                assert np.array_equal(perm.cpu().numpy()[b, h], rperm)
                assert np.array_equal(ka[b, h, :n_keep], k8[b, h][rperm]) and np.array_equal(va[b, h, :n_keep], v8[b, h][rperm])
        assert np.array_equal(ka[:, :, n_keep:], k8[:, :, n_keep:])
    else:
        P.check_compaction(ka, va, k8, v8, gi, n_keep)


def test_compact_moves_fp8_rows():
    """ea_compact and ea_compact_unordered with p->dtype = EA_FP8_E4M3: rows of d bytes."""
    import torch
    from oracle import ea_extensions as X
    r = np.random.default_rng(9)
    for d in (128, 256):
        B, H, n = 2, 3, 4000
        k8 = r.integers(0, 256, (B, H, n, d), dtype=np.uint8)
        v8 = r.integers(0, 256, (B, H, n, d), dtype=np.uint8)
        keep = np.sort(r.choice(n, 1700, replace=False)).astype(np.int32)
        idx = np.broadcast_to(keep, (B, H, len(keep))).copy()
        p = ea.make_params(B, H, H, d, ea.EA_FP8_E4M3)
        ws = P.workspace(p, n, 1)
        kd, vd = torch.from_numpy(k8).cuda(), torch.from_numpy(v8).cuda()
        ea.compact(p, kd, vd, n, n, torch.from_numpy(idx).cuda(), len(keep), kd, vd, ws)
        torch.cuda.synchronize()
        P.check_compaction(kd.cpu().numpy(), vd.cpu().numpy(), k8, v8, idx, len(keep))
        kd, vd = torch.from_numpy(k8).cuda(), torch.from_numpy(v8).cuda()
        ea.compact_unordered(p, kd, vd, n, n, torch.from_numpy(idx).cuda(), len(keep))
        torch.cuda.synchronize()
        rperm = X.unordered_perm(keep, len(keep))
        assert np.array_equal(kd.cpu().numpy()[:, :, :len(keep)], k8[:, :, rperm])
        assert np.array_equal(vd.cpu().numpy()[:, :, :len(keep)], v8[:, :, rperm])


# ------------------------------------------------------------------- fused pass with head-adaptive budgets
@pytest.mark.parametrize("name,n,floor", [("c2mini", 3000, 0), ("c2mini", 3000, 200), ("c4mini", 1500, 64),
                                          ("c5mini", 1100, 0), ("c1", 1024, 100)])
def test_compress_layer_adaptive(name, n, floor):
    """statistics -> scores -> pooled selection with a floor -> ragged compaction in one call: scores
    against the oracle, lists and lengths bit-exact against the oracle's rule applied to the call's
    own scores, bytes against the ragged gather."""
    import torch
    from oracle import ea_extensions as X
    cfg, kw = MINI[name]
    lay = make_layer(cfg, **dict(kw, n=n))
    w = lay["window"]
    n_keep = int(n * 0.4)
    B, H = cfg.batch, cfg.n_kv_heads
    p = P.params_for(cfg, epsilon=0.02)
    ws = P.workspace(p, n, w)
    kd, vd = P.to_dev(lay["k"]), P.to_dev(lay["v"])
    sc = torch.empty(B, H, n, dtype=torch.float32, device="cuda")
    idx = torch.full((B, H, n), -7, dtype=torch.int32, device="cuda")
    lengths = torch.full((B, H), -1, dtype=torch.int32, device="cuda")
    ea.compress_layer_adaptive(p, P.to_dev(lay["q_win"]), w, lay["q_pos0"], P.to_dev(lay["inv_freq"]), lay["t_next"],
                               kd, vd, n, n, n_keep, floor, sc, idx, lengths, ws)
    torch.cuda.synchronize()
    assert ea.debug_status(p, n, w, ws) == 0
    rmu, rsg = _oracle_stats(cfg, lay)
    ref_sc = O.scores(widen(lay["k"]), widen(lay["v"]), rmu, rsg, 0.02)
    gs = sc.cpu().numpy()
    P.check_scores(gs, ref_sc, TOL[cfg.dtype])
    rl, rk = X.select_adaptive(gs.astype(np.float64), n_keep, floor)
    gl, gi = lengths.cpu().numpy(), idx.cpu().numpy()
    assert np.array_equal(gl, rl) and gl.sum(axis=1).tolist() == [H * n_keep] * B
    ko, vo = P.to_host(kd), P.to_host(vd)
    ref = X.compact_ragged(lay["k"], lay["v"], rk)
    for b in range(B):
        for h in range(H):
            m = gl[b, h]
            assert m >= floor
            assert np.array_equal(gi[b, h, :m], rk[b][h]), (b, h)
            assert np.array_equal(ko[b, h, :m], ref[b][h][0]) and np.array_equal(vo[b, h, :m], ref[b][h][1])
            assert np.array_equal(ko[b, h, m:], lay["k"][b, h, m:])
    # the same call without the optional scores gives the same cache
    kd2, vd2 = P.to_dev(lay["k"]), P.to_dev(lay["v"])
    idx2, len2 = torch.empty_like(idx), torch.empty_like(lengths)
    ea.compress_layer_adaptive(p, P.to_dev(lay["q_win"]), w, lay["q_pos0"], P.to_dev(lay["inv_freq"]), lay["t_next"],
                               kd2, vd2, n, n, n_keep, floor, None, idx2, len2, ws)
    torch.cuda.synchronize()
    assert torch.equal(len2, lengths) and torch.equal(kd2, kd) and torch.equal(vd2, vd)
