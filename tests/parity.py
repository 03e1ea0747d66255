"""Helpers for the GPU parity tests and smoke(): upload seeded inputs, call the C ABI through
the Python binding, download, and compare with the fp64 oracle."""
import numpy as np

import paper_2510_00636_amd as ea
from ea_inputs.torch_io import to_dev, to_host          # noqa: F401  (re-exported for the tests)
from oracle import ea_oracle as O


def params_for(cfg, epsilon=None, rope_layout=0, q_is_rotated=1, ddof=0, T=None):
    return ea.make_params(cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                          ea.EA_BF16 if cfg.dtype == "bf16" else ea.EA_F32, rope_layout,
                          q_is_rotated, ddof, cfg.horizon_T if T is None else T,
                          cfg.epsilon if epsilon is None else epsilon)


def workspace(p, n, window):
    import torch
    nbytes = ea.workspace_bytes(p, n, window)
    assert nbytes > 0
    return torch.empty(nbytes, dtype=torch.uint8, device="cuda")


def run_query_stats(cfg, lay, **pk):
    import torch
    p = params_for(cfg, **pk)
    B, Hq, d, w = cfg.batch, cfg.n_q_heads, cfg.head_dim, lay["window"]
    ws = workspace(p, lay["n"], w)
    mu = torch.empty(B, Hq, d, dtype=torch.float32, device="cuda")
    sigma = torch.empty(B, Hq, d, d, dtype=torch.float32, device="cuda")
    ea.query_stats(p, to_dev(lay["q_win"]), w, lay["q_pos0"], to_dev(lay["inv_freq"]),
                   lay["t_next"], mu, sigma, ws)
    torch.cuda.synchronize()
    return mu.cpu().numpy(), sigma.cpu().numpy()


def run_score(cfg, lay, mu32, sigma32, epsilon, n_cap=None):
    import torch
    p = params_for(cfg, epsilon=epsilon)
    n = lay["n"]
    n_cap = n if n_cap is None else n_cap
    k, v = lay["k"], lay["v"]
    if n_cap != n:
        pad = [(0, 0), (0, 0), (0, n_cap - n), (0, 0)]
        k = np.pad(k, pad, constant_values=0x7FC0 if k.dtype == np.uint16 else np.nan)  # NaN rows
        v = np.pad(v, pad, constant_values=0x7FC0 if v.dtype == np.uint16 else np.nan)
    ws = workspace(p, n, 1)
    sc = torch.empty(cfg.batch, cfg.n_kv_heads, n, dtype=torch.float32, device="cuda")
    ea.score(p, to_dev(k), to_dev(v), n, n_cap, to_dev(mu32), to_dev(sigma32), sc, ws)
    torch.cuda.synchronize()
    return sc.cpu().numpy()


def run_select(cfg, scores32, n_keep):
    import torch
    p = params_for(cfg)
    B, H, n = scores32.shape
    ws = workspace(p, n, 1)
    idx = torch.full((B, H, max(n_keep, 1)), -1, dtype=torch.int32, device="cuda")
    ea.select(p, to_dev(scores32), n, n_keep, idx, ws)
    torch.cuda.synchronize()
    return idx.cpu().numpy()[:, :, :n_keep]


def run_compact(cfg, k, v, n, idx, inplace=True):
    import torch
    p = params_for(cfg)
    n_cap = k.shape[2]
    n_keep = idx.shape[2]
    ws = workspace(p, n, 1)
    kd, vd = to_dev(k), to_dev(v)
    if inplace:
        ko, vo = kd, vd
    else:
        ko, vo = torch.zeros_like(kd), torch.zeros_like(vd)
    ea.compact(p, kd, vd, n, n_cap, to_dev(idx.astype(np.int32)) if n_keep else None, n_keep, ko, vo, ws)
    torch.cuda.synchronize()
    return to_host(ko), to_host(vo)


def run_compress_layer(cfg, lay, n_keep, epsilon=None, want_scores=True, want_idx=True, **pk):
    import torch
    p = params_for(cfg, epsilon=epsilon, **pk)
    n, w = lay["n"], lay["window"]
    ws = workspace(p, n, w)
    kd, vd = to_dev(lay["k"]), to_dev(lay["v"])
    sc = torch.empty(cfg.batch, cfg.n_kv_heads, n, dtype=torch.float32, device="cuda") if want_scores else None
    idx = torch.full((cfg.batch, cfg.n_kv_heads, max(n_keep, 1)), -1, dtype=torch.int32,
                     device="cuda") if want_idx else None
    ea.compress_layer(p, to_dev(lay["q_win"]), w, lay["q_pos0"], to_dev(lay["inv_freq"]),
                      lay["t_next"], kd, vd, n, n, n_keep, sc, idx, ws)
    torch.cuda.synchronize()
    return dict(scores=sc.cpu().numpy() if want_scores else None,
                idx=idx.cpu().numpy()[:, :, :n_keep] if want_idx else None,
                k=to_host(kd), v=to_host(vd))


# ------------------------------------------------------------------------------- checks
def rel_err(got, ref):
    ref = np.asarray(ref, np.float64)
    return np.abs(np.asarray(got, np.float64) - ref) / np.maximum(np.abs(ref), 1e-300)


def check_scores(got, ref, tol):
    got = np.asarray(got, np.float64)
    assert np.all(np.isfinite(got))
    bad = np.abs(got - ref) > tol * np.abs(ref) + 1e-37
    assert not bad.any(), "scores: %d of %d beyond %g, worst rel err %g" % (
        bad.sum(), bad.size, tol, rel_err(got, ref).max())


def check_stats(mu, sigma, ref_mu, ref_sigma, tol=2e-5):
    for b in range(ref_mu.shape[0]):
        for h in range(ref_mu.shape[1]):
            sm, ss = np.abs(ref_mu[b, h]).max(), np.abs(ref_sigma[b, h]).max()
            assert np.abs(mu[b, h] - ref_mu[b, h]).max() <= tol * sm + 1e-30, ("mu", b, h)
            assert np.abs(sigma[b, h] - ref_sigma[b, h]).max() <= tol * ss + 1e-30, ("sigma", b, h)


def check_idx_vs_oracle_scores(idx, ref_scores, n_keep, tol):
    """Kept sets equal the oracle's except where oracle scores lie within tol of the threshold."""
    B, H, n = ref_scores.shape
    assert idx.shape == (B, H, n_keep)
    if n_keep == 0 or n_keep == n:
        if n_keep == n:
            assert np.array_equal(idx, np.broadcast_to(np.arange(n), idx.shape))
        return
    for b in range(B):
        for h in range(H):
            got = idx[b, h].astype(np.int64)
            assert np.all(np.diff(got) > 0) and got[0] >= 0 and got[-1] < n, "not ascending / range"
            s = ref_scores[b, h]
            thr = np.sort(s)[n - n_keep]                     # n_keep-th largest
            must_keep = np.nonzero(s > thr * (1 + tol))[0]
            must_drop = np.nonzero(s < thr * (1 - tol))[0]
            kept = np.zeros(n, bool)
            kept[got] = True
            assert kept[must_keep].all(), ("evicted a pair well above the threshold", b, h)
            assert not kept[must_drop].any(), ("kept a pair well below the threshold", b, h)


def check_idx_exact_given_scores(idx, gpu_scores32, n_keep):
    """Bit-exact: the kernel's indices are the top-k (ties to lower index) of its own scores."""
    ref = O.select(gpu_scores32.astype(np.float64), n_keep)
    assert np.array_equal(idx.astype(np.int64), ref)


def check_compaction(k_after, v_after, k_before, v_before, idx, n_keep, rest="same"):
    """Bytes bit-exact given the indices.  Rows >= n_keep: rest="same" -- what they were before
    (in place); rest="zero" -- still the zeros the output buffers were created with (out of
    place); rest=None -- not looked at."""
    i = idx.astype(np.int64)[..., None]
    assert np.array_equal(k_after[:, :, :n_keep], np.take_along_axis(k_before, i, axis=2))
    assert np.array_equal(v_after[:, :, :n_keep], np.take_along_axis(v_before, i, axis=2))
    if rest == "same":
        assert np.array_equal(k_after[:, :, n_keep:], k_before[:, :, n_keep:]), "K rows past n_keep changed"
        assert np.array_equal(v_after[:, :, n_keep:], v_before[:, :, n_keep:]), "V rows past n_keep changed"
    elif rest == "zero":
        assert not k_after[:, :, n_keep:].any() and not v_after[:, :, n_keep:].any()


def check_layer(cfg, lay, got, ref, n_keep, tol):
    check_scores(got["scores"], ref["scores"], tol)
    check_idx_vs_oracle_scores(got["idx"], ref["scores"], n_keep, tol)
    check_idx_exact_given_scores(got["idx"], got["scores"], n_keep)
    check_compaction(got["k"], got["v"], lay["k"], lay["v"], got["idx"], n_keep)
