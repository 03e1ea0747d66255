"""Host (numpy) generator: the canonical bits for the small and medium parity cases.

Recipe, per (sequence b, head), all in fp64 then rounded to the storage dtype:
  * per-channel mean  m_c ~ N(0, variance 2), per-channel scale s_c = exp(0.5 * N(0,1)),
    drawn independently for every query head and every KV head;
  * `n_outliers` channels per KV head (a seeded choice shared by the key head and the query
    heads of its group) get m_c += outlier_offset;
  * pre-rotary activation x[i, c] = s_c * z[i, c] + m_c with z ~ N(0,1);
  * the rotary embedding at the token's position turns x into the cached key (all n tokens)
    and into the query (only the last `window` tokens are materialised);
  * values v[i, c] = tau_i * z[i, c] with tau_i = exp(0.5 * N(0,1)) per token per KV head.
Random streams are numpy Philox generators keyed by (seed, b, kind, head).
"""
import numpy as np

from .configs import CacheConfig

_KIND_KCHAN, _KIND_QCHAN, _KIND_OUTL, _KIND_KZ, _KIND_QZ, _KIND_V = range(6)


def _rng(seed, b, kind, head):
    ss = np.random.SeedSequence([int(seed), int(b), int(kind), int(head)])
    return np.random.Generator(np.random.Philox(ss))


def layer_seed(cfg: CacheConfig, layer: int = 0, b: int = 0) -> int:
    """c3: seed+layer; c4: seed + layers*b + layer (per-sequence seeds); others: seed+layer."""
    if cfg.batch > 1:
        return cfg.seed + cfg.layers * b + layer
    return cfg.seed + layer


def inv_freq_table(head_dim: int, base: float) -> np.ndarray:
    """theta_c = base^(-2c/d), c = 0 .. d/2-1, fp64."""
    c = np.arange(head_dim // 2, dtype=np.float64)
    return np.power(float(base), -2.0 * c / head_dim)


def bf16_bits_from_f64(x: np.ndarray) -> np.ndarray:
    """Round to bfloat16 (via fp32, round-to-nearest-even at both steps); returns uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float64).astype(np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def f64_from_bf16_bits(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to fp64."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def widen(a: np.ndarray) -> np.ndarray:
    """Exact fp64 view of a stored tensor (uint16 = bf16 bits, float32 = itself)."""
    if a.dtype == np.uint16:
        return f64_from_bf16_bits(a)
    return a.astype(np.float64)


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return bf16_bits_from_f64(x)
    if dtype == "f32":
        return x.astype(np.float32)
    raise ValueError(dtype)


def _embed_positions(x: np.ndarray, positions: np.ndarray, inv_freq: np.ndarray,
                     interleaved: bool) -> np.ndarray:
    """Rotary embedding of rows x[i, :] at integer positions[i] (fp64).

    Channel pair (a, b) = (c, c + d/2) [half-split] or (2c, 2c+1) [interleaved] is turned by
    the angle positions[i] * inv_freq[c], counter-clockwise."""
    d = x.shape[-1]
    ang = positions.astype(np.float64)[:, None] * inv_freq[None, :]
    co, si = np.cos(ang), np.sin(ang)
    out = np.empty_like(x)
    if interleaved:
        xa, xb = x[:, 0::2], x[:, 1::2]
        out[:, 0::2] = xa * co - xb * si
        out[:, 1::2] = xa * si + xb * co
    else:
        xa, xb = x[:, : d // 2], x[:, d // 2:]
        out[:, : d // 2] = xa * co - xb * si
        out[:, d // 2:] = xa * si + xb * co
    return out


def make_layer(cfg: CacheConfig, layer: int = 0, *, n: int = None, window: int = None,
               pos0: int = 0, interleaved: bool = False, pre_rope_queries: bool = False):
    """One layer of synthetic cache.

    Returns a dict with
      q_win  [B, Hq, w, d]   the last w queries (positions pos0+n-w .. pos0+n-1)
      k, v   [B, Hkv, n, d]  keys (rotary-embedded at pos0 .. pos0+n-1) and values
      inv_freq [d/2] fp64, q_pos0 = pos0+n-w, t_next = pos0+n
    Tensors are float32 arrays (dtype "f32") or uint16 bfloat16 bit patterns ("bf16")."""
    n = cfg.n if n is None else int(n)
    w = cfg.window if window is None else int(window)
    d, B, Hq, Hkv, G = cfg.head_dim, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.group
    inv_freq = inv_freq_table(d, cfg.rope_base)
    kpos = pos0 + np.arange(n, dtype=np.int64)
    qpos = kpos[n - w:]
    np_dt = np.uint16 if cfg.dtype == "bf16" else np.float32
    q_win = np.empty((B, Hq, w, d), np_dt)
    k = np.empty((B, Hkv, n, d), np_dt)
    v = np.empty((B, Hkv, n, d), np_dt)
    for b in range(B):
        seed = layer_seed(cfg, layer, b)
        for h in range(Hkv):
            outl = _rng(seed, b, _KIND_OUTL, h).choice(d, size=cfg.n_outliers, replace=False) \
                if cfg.n_outliers else np.zeros(0, np.int64)
            r = _rng(seed, b, _KIND_KCHAN, h)
            m = r.normal(0.0, np.sqrt(2.0), d)
            s = np.exp(0.5 * r.normal(0.0, 1.0, d))
            m[outl] += cfg.outlier_offset
            z = _rng(seed, b, _KIND_KZ, h).standard_normal((n, d))
            k[b, h] = _store(_embed_positions(s * z + m, kpos, inv_freq, interleaved), cfg.dtype)
            rv = _rng(seed, b, _KIND_V, h)
            tau = np.exp(0.5 * rv.standard_normal(n))
            v[b, h] = _store(tau[:, None] * rv.standard_normal((n, d)), cfg.dtype)
            for g in range(G):
                hq = h * G + g
                r = _rng(seed, b, _KIND_QCHAN, hq)
                m = r.normal(0.0, np.sqrt(2.0), d)
                s = np.exp(0.5 * r.normal(0.0, 1.0, d))
                m[outl] += cfg.outlier_offset
                x = s * _rng(seed, b, _KIND_QZ, hq).standard_normal((w, d)) + m
                if not pre_rope_queries:
                    x = _embed_positions(x, qpos, inv_freq, interleaved)
                q_win[b, hq] = _store(x, cfg.dtype)
    return dict(q_win=q_win, k=k, v=v, inv_freq=inv_freq, q_pos0=int(qpos[0]),
                t_next=int(pos0 + n), n=n, window=w)


def make_block_pools(k, v, block_size, seed, spare_blocks=3):
    """Scatters contiguous caches k, v [B, Hkv, n, d] into block pools [num_blocks, Hkv, block_size, d]
    through a seeded random block table [B, max_blocks] (every logical block gets a pool block of
    its own; the pool holds `spare_blocks` blocks more than needed, filled with a marker pattern,
    as are the unused rows of each sequence's last block).  Returns (k_pool, v_pool, table, num_blocks)."""
    B, H, n, d = k.shape
    mb = -(-n // block_size)
    num_blocks = B * mb + spare_blocks
    rng = np.random.Generator(np.random.Philox(key=[seed & 0xFFFFFFFF, 0x9A6ED]))
    table = rng.permutation(num_blocks)[:B * mb].reshape(B, mb).astype(np.int32)
    marker = 0x7FC0 if k.dtype == np.uint16 else np.nan          # NaN in either storage type
    pools = []
    for t in (k, v):
        pool = np.full((num_blocks, H, block_size, d), marker, dtype=t.dtype)
        for b in range(B):
            for j in range(mb):
                rows = t[b, :, j * block_size:(j + 1) * block_size]
                pool[table[b, j], :, :rows.shape[1]] = rows
        pools.append(pool)
    return pools[0], pools[1], table, num_blocks


def quantize_fp8(x, headroom=0.9):
    """Stores x [B, H, n, d] (float64) as OCP e4m3 bytes with one fp32 scale per (b, h): the head's
    largest magnitude lands at `headroom` x 448.  The rounding is torch's float8_e4m3fn conversion
    (a library routine; the oracle decodes the bytes with code of its own).  Returns (uint8 bytes,
    float32 scales [B, H])."""
    import torch
    amax = np.abs(x).max(axis=(2, 3))
    scale = (np.maximum(amax, 1e-30) / (448.0 * headroom)).astype(np.float32)
    y = torch.from_numpy(x / scale.astype(np.float64)[:, :, None, None]).to(torch.float32)
    return y.to(torch.float8_e4m3fn).view(torch.uint8).numpy(), scale
