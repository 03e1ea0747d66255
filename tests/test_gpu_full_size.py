"""Full-size parity in the launch configuration bench.py times: one layer of the
Llama-3.1-8B-shaped 131072-token cache (8 KV heads, 32 query heads, d 128, window 128, keep
25 / 50 / 75 %), four such layers as one batch on side streams, one layer of the d-256 four-sequence
shape and one decode-time pass, all generated on the device and downloaded so the oracle sees the
same bits.  The oracle is fast enough here to check every score, the kept sets and the compacted
bytes, not just a sample."""
import numpy as np
import pytest

from ea_inputs import CONFIGS, widen
from oracle import ea_oracle as O
from tests import parity as P

pytestmark = pytest.mark.gpu


def _layer_full_size(cfg, layer, n_keep, eps):
    import torch
    import paper_2510_00636_amd as ea
    from ea_inputs.device import make_layer_device
    lay = make_layer_device(cfg, layer=layer)
    n, w = lay["n"], lay["window"]
    host = dict(q_win=P.to_host(lay["q_win"]), k=P.to_host(lay["k"]), v=P.to_host(lay["v"]))
    p = ea.make_params(cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, ea.EA_BF16,
                       horizon_T=cfg.horizon_T, epsilon=eps)
    ws = torch.empty(ea.workspace_bytes(p, n, w), dtype=torch.uint8, device="cuda")
    sc = torch.empty(cfg.batch, cfg.n_kv_heads, n, dtype=torch.float32, device="cuda")
    idx = torch.empty(cfg.batch, cfg.n_kv_heads, n_keep, dtype=torch.int32, device="cuda")
    ea.compress_layer(p, lay["q_win"], w, lay["q_pos0"], lay["inv_freq"], lay["t_next"], lay["k"],
                      lay["v"], n, n, n_keep, sc, idx, ws)
    torch.cuda.synchronize()
    got = dict(scores=sc.cpu().numpy(), idx=idx.cpu().numpy(), k=P.to_host(lay["k"]), v=P.to_host(lay["v"]))
    inv = lay["inv_freq"].cpu().numpy()
    ref = O.compress_layer(widen(host["q_win"]), widen(host["k"]), widen(host["v"]), lay["q_pos0"], inv,
                           lay["t_next"], n_keep, T=cfg.horizon_T, epsilon=eps)
    P.check_scores(got["scores"], ref["scores"], 2e-3)
    P.check_idx_vs_oracle_scores(got["idx"], ref["scores"], n_keep, 2e-3)
    P.check_idx_exact_given_scores(got["idx"], got["scores"], n_keep)
    P.check_compaction(got["k"], got["v"], host["k"], host["v"], got["idx"], n_keep)
    # rows past n_keep are untouched
    assert np.array_equal(got["k"][:, :, n_keep:], host["k"][:, :, n_keep:])


@pytest.mark.parametrize("ratio,eps", [(0.5, 0.02), (0.75, 0.0), (0.25, 0.02)])
def test_c3_layer_full_size(ratio, eps):
    import paper_2510_00636_amd as ea
    cfg = CONFIGS["c3"]
    _layer_full_size(cfg, int(ratio * 100) % 32, ea.n_keep(cfg.n, ratio), eps)


def test_c4_layer_full_size():
    """Head dimension 256, four sequences, two query heads per KV head (two passes over K)."""
    cfg = CONFIGS["c4"]
    _layer_full_size(cfg, 47, cfg.n // 2, 0.02)


def test_c5_layer_full_size():
    """The decode-time pass: 4608 cached tokens back to 4096, statistics over 512 queries,
    five query heads per KV head."""
    cfg = CONFIGS["c5"]
    _layer_full_size(cfg, 0, 4096, 0.02)


def test_c3_four_layers_as_one_batch_on_side_streams():
    """The configuration bench.py times by default: four consecutive layers handed to one call
    as a batch (same shape and positions, contiguous in memory), calls issued on side streams
    with a workspace each.  Every layer is checked in full against the oracle."""
    import torch
    import paper_2510_00636_amd as ea
    from ea_inputs.device import make_layer_device
    cfg = CONFIGS["c3"]
    LB, NCALL, ratio, eps = 4, 2, 0.5, 0.02
    B, Hq, Hkv, d, n, w = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.n, cfg.window
    L = LB * NCALL
    k = torch.empty(L, B, Hkv, n, d, dtype=torch.bfloat16, device="cuda")
    v = torch.empty_like(k)
    q = torch.empty(L, B, Hq, w, d, dtype=torch.bfloat16, device="cuda")
    for l in range(L):
        lay = make_layer_device(cfg, l, out_k=k[l], out_v=v[l], out_q=q[l])
    inv = lay["inv_freq"]
    host_k, host_v, host_q = P.to_host(k), P.to_host(v), P.to_host(q)
    n_keep = ea.n_keep(n, ratio)
    p = ea.make_params(B * LB, Hq, Hkv, d, ea.EA_BF16, horizon_T=cfg.horizon_T, epsilon=eps)
    streams = [torch.cuda.Stream() for _ in range(NCALL)]
    wss = [torch.empty(ea.workspace_bytes(p, n, w), dtype=torch.uint8, device="cuda") for _ in range(NCALL)]
    sc = torch.empty(L, B, Hkv, n, dtype=torch.float32, device="cuda")
    idx = torch.empty(L, B, Hkv, n_keep, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    for c in range(NCALL):
        sl = slice(c * LB, (c + 1) * LB)
        ea.compress_layer(p, q[sl], w, n - w, inv, n, k[sl], v[sl], n, n, n_keep, sc[sl], idx[sl], wss[c],
                          stream=streams[c])
    torch.cuda.synchronize()
    got_k, got_v = P.to_host(k), P.to_host(v)
    got_sc, got_idx = sc.cpu().numpy(), idx.cpu().numpy()
    invh = inv.cpu().numpy()
    for l in range(L):
        ref = O.compress_layer(widen(host_q[l]), widen(host_k[l]), widen(host_v[l]), n - w, invh, n, n_keep,
                               T=cfg.horizon_T, epsilon=eps)
        P.check_scores(got_sc[l], ref["scores"], 2e-3)
        P.check_idx_vs_oracle_scores(got_idx[l], ref["scores"], n_keep, 2e-3)
        P.check_idx_exact_given_scores(got_idx[l], got_sc[l], n_keep)
        P.check_compaction(got_k[l], got_v[l], host_k[l], host_v[l], got_idx[l], n_keep)
