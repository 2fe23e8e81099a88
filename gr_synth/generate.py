"""Seeded generators.  numpy only; every array is produced on the host from PCG64 streams."""
import numpy as np

from .configs import GRConfig

# stream ids (seed = 1000 * config_id + stream id [+ 10 * step for per-step streams])
_STREAM_LENGTHS = 1
_STREAM_ITEMS = 2
_STREAM_KV_SHARED = 3
_STREAM_STEP_ATTN = 100      # + step
_STREAM_STEP_LOGITS = 200    # + step


def rng_for(cfg: GRConfig, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(1000 * cfg.config_id + stream))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (round-to-nearest-even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def e4m3_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Decode OCP FP8 E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa bits; no infinities, 0x7f / 0xff = NaN)."""
    codes = np.arange(256, dtype=np.uint32)
    sign = np.where(codes & 0x80, -1.0, 1.0)
    e = ((codes >> 3) & 0xF).astype(np.int32)
    m = (codes & 0x7).astype(np.float64)
    val = np.where(e == 0, m / 8.0 * 2.0 ** -6, (1.0 + m / 8.0) * 2.0 ** (e - 7).astype(np.float64))
    val = np.where((codes & 0x7F) == 0x7F, np.nan, val) * sign
    return val.astype(np.float32)[np.ascontiguousarray(b, dtype=np.uint8)]


def f32_to_e4m3_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to OCP FP8 E4M3 (round-to-nearest-even on the representable grid, saturating at +-448)."""
    grid = e4m3_bits_to_f32(np.arange(0, 0x7F, dtype=np.uint8)).astype(np.float64)      # the 127 non-negative finite values, ascending
    a = np.minimum(np.abs(np.ascontiguousarray(x, dtype=np.float32)).astype(np.float64), 448.0)
    hi = np.clip(np.searchsorted(grid, a, side="left"), 1, len(grid) - 1)
    lo = hi - 1
    d_lo, d_hi = a - grid[lo], grid[hi] - a
    pick_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0))                          # ties go to the even code
    code = np.where(pick_hi, hi, lo).astype(np.uint8)
    return np.where(np.signbit(x), code | np.uint8(0x80), code).astype(np.uint8)


def _randn_bf16(rng: np.random.Generator, shape) -> np.ndarray:
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    chunk = 1 << 24
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        out[s:e] = f32_to_bf16_bits(rng.standard_normal(e - s, dtype=np.float32))
    return out.reshape(shape)


def make_prompt_lengths(cfg: GRConfig) -> np.ndarray:
    """Prompt length per request -> cu_seqlens int32 [B+1]."""
    if cfg.L_min == cfg.L_max:
        lens = np.full(cfg.B, cfg.L_min, dtype=np.int64)
    else:
        lens = rng_for(cfg, _STREAM_LENGTHS).integers(cfg.L_min, cfg.L_max + 1, size=cfg.B)
    cu = np.zeros(cfg.B + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    return cu


def make_item_table(cfg: GRConfig) -> np.ndarray:
    """Sorted (lexicographic), distinct table of valid items, int32 [n_items, ND]."""
    rng = rng_for(cfg, _STREAM_ITEMS)
    V, N, depth = cfg.V, cfg.n_items, cfg.ND
    assert V ** depth >= N
    if cfg.zipf_a > 0:
        ranks = np.arange(1, V + 1, dtype=np.float64)
        p = ranks ** (-cfg.zipf_a)
        p /= p.sum()
        rank_to_token = rng.permutation(V)
    keys = np.empty(0, dtype=np.uint64)
    while keys.size < N:
        m = int((N - keys.size) * 1.05) + 1024
        if cfg.zipf_a > 0:
            t0 = rank_to_token[rng.choice(V, size=m, p=p)].astype(np.uint64)
        else:
            t0 = rng.integers(0, V, size=m, dtype=np.int64).astype(np.uint64)
        k = t0
        for _ in range(depth - 1):
            k = k * np.uint64(V) + rng.integers(0, V, size=m, dtype=np.int64).astype(np.uint64)
        keys = np.unique(np.concatenate([keys, k]))
    if keys.size > N:
        keep = np.sort(rng.choice(keys.size, size=N, replace=False))
        keys = keys[keep]
    items = np.empty((N, depth), dtype=np.int32)
    rem = keys.copy()
    for c in range(depth - 1, -1, -1):
        items[:, c] = (rem % np.uint64(V)).astype(np.int32)
        rem //= np.uint64(V)
    return items


def make_kv_shared(cfg: GRConfig, cu_seqlens: np.ndarray):
    """Prompt K and V as bf16 bit patterns, packed [total_L, Hkv, d]."""
    rng = rng_for(cfg, _STREAM_KV_SHARED)
    total = int(cu_seqlens[-1])
    k = _randn_bf16(rng, (total, cfg.Hkv, cfg.d))
    v = _randn_bf16(rng, (total, cfg.Hkv, cfg.d))
    return k, v


def make_attention_inputs(cfg: GRConfig, step: int, kv_shared=None):
    """Everything one attention call needs at decode step `step` (u = step + 1 own tokens per beam).

    Returns a dict of numpy arrays; bf16 tensors are uint16 bit patterns.
    """
    cu = make_prompt_lengths(cfg)
    if kv_shared is None:
        kv_shared = make_kv_shared(cfg, cu)
    rng = rng_for(cfg, _STREAM_STEP_ATTN + step)
    q = _randn_bf16(rng, (cfg.B, cfg.W, cfg.Hq, cfg.d))
    k_un = _randn_bf16(rng, (cfg.B, cfg.W, cfg.ND, cfg.Hkv, cfg.d))
    v_un = _randn_bf16(rng, (cfg.B, cfg.W, cfg.ND, cfg.Hkv, cfg.d))
    return dict(q=q, k_shared=kv_shared[0], v_shared=kv_shared[1], cu_seqlens=cu,
                k_unshared=k_un, v_unshared=v_un, u=step + 1)


def make_logits(cfg: GRConfig, step: int) -> np.ndarray:
    """fp32 logits [B, W, V] for decode step `step`."""
    rng = rng_for(cfg, _STREAM_STEP_LOGITS + step)
    x = rng.standard_normal((cfg.B, cfg.W, cfg.V), dtype=np.float32)
    x *= np.float32(cfg.logit_sigma)
    return x


def initial_beam_state(B: int, W: int, depth: int):
    """Single live root per request: scores [0, -inf, ...], empty prefixes and ranges."""
    scores = np.full((B, W), -np.inf, dtype=np.float32)
    scores[:, 0] = 0.0
    prefix = np.full((B, W, depth), -1, dtype=np.int32)
    rng_ = np.zeros((B, W, 2), dtype=np.int32)
    return scores, prefix, rng_
