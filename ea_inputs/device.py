"""Device-side (torch, ROCm) generator for the large throughput / full-size parity runs.

Same recipe as host.py (per-channel mean N(0, var 2) and log-normal(0, 0.5) scale, outlier
channels shared by a KV head and its query group, rotary embedding at positions 0..n-1,
values N(0,1) times a per-token log-normal(0, 0.5) scale), with two differences that do not
matter to the method: the normal draws come from torch's Philox generator on the GPU, and the
arithmetic is fp32 (rotary angles in fp64) before rounding to bf16.  The per-channel
statistics are drawn on the host with the same numpy streams as host.py.  Tests that use
these tensors download them, so the oracle always sees the exact bits the kernels saw.
"""
import numpy as np

from .configs import CacheConfig
from .host import _rng, _KIND_KCHAN, _KIND_QCHAN, _KIND_OUTL, inv_freq_table, layer_seed


def _rotate(x, pos, inv_freq):
    """half-split rotary embedding of x [n, d] (fp32) at integer positions pos [n] (int64)."""
    import torch
    d = x.shape[-1]
    ang = pos.to(torch.float64)[:, None] * inv_freq[None, :]
    co, si = torch.cos(ang).float(), torch.sin(ang).float()
    xa, xb = x[:, : d // 2], x[:, d // 2:]
    return torch.cat([xa * co - xb * si, xa * si + xb * co], dim=1)


def make_layer_device(cfg: CacheConfig, layer: int = 0, *, n: int = None, window: int = None,
                      out_k=None, out_v=None, out_q=None, device="cuda"):
    """Returns dict(q_win [B,Hq,w,d], k, v [B,Hkv,n,d] bf16 CUDA tensors, inv_freq fp64 CUDA,
    q_pos0, t_next, n, window).  out_* may be preallocated destinations."""
    import torch
    assert cfg.dtype == "bf16"
    n = cfg.n if n is None else int(n)
    w = cfg.window if window is None else int(window)
    d, B, Hq, Hkv, G = cfg.head_dim, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.group
    inv_np = inv_freq_table(d, cfg.rope_base)
    inv = torch.from_numpy(inv_np).to(device)
    k = out_k if out_k is not None else torch.empty(B, Hkv, n, d, dtype=torch.bfloat16, device=device)
    v = out_v if out_v is not None else torch.empty(B, Hkv, n, d, dtype=torch.bfloat16, device=device)
    q = out_q if out_q is not None else torch.empty(B, Hq, w, d, dtype=torch.bfloat16, device=device)
    kpos = torch.arange(n, device=device, dtype=torch.int64)
    qpos = kpos[n - w:]
    for b in range(B):
        seed = layer_seed(cfg, layer, b)
        gen = torch.Generator(device=device)
        gen.manual_seed(int(seed))
        for h in range(Hkv):
            outl = _rng(seed, b, _KIND_OUTL, h).choice(d, size=cfg.n_outliers, replace=False) \
                if cfg.n_outliers else np.zeros(0, np.int64)
            r = _rng(seed, b, _KIND_KCHAN, h)
            m = r.normal(0.0, np.sqrt(2.0), d)
            s = np.exp(0.5 * r.normal(0.0, 1.0, d))
            m[outl] += cfg.outlier_offset
            mt = torch.from_numpy(m.astype(np.float32)).to(device)
            st = torch.from_numpy(s.astype(np.float32)).to(device)
            z = torch.randn(n, d, generator=gen, device=device, dtype=torch.float32)
            k[b, h].copy_(_rotate(z * st + mt, kpos, inv))
            tau = torch.exp(0.5 * torch.randn(n, 1, generator=gen, device=device, dtype=torch.float32))
            v[b, h].copy_(tau * torch.randn(n, d, generator=gen, device=device, dtype=torch.float32))
            for g in range(G):
                hq = h * G + g
                r = _rng(seed, b, _KIND_QCHAN, hq)
                m = r.normal(0.0, np.sqrt(2.0), d)
                s = np.exp(0.5 * r.normal(0.0, 1.0, d))
                m[outl] += cfg.outlier_offset
                mt = torch.from_numpy(m.astype(np.float32)).to(device)
                st = torch.from_numpy(s.astype(np.float32)).to(device)
                z = torch.randn(w, d, generator=gen, device=device, dtype=torch.float32)
                q[b, hq].copy_(_rotate(z * st + mt, qpos, inv))
    return dict(q_win=q, k=k, v=v, inv_freq=inv, q_pos0=int(n - w), t_next=int(n), n=n, window=w)
