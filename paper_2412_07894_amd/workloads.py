"""Seeded synthetic workloads: sequence-length structure and tensor values of the benchmark
configurations.  This module holds no attention arithmetic; it only draws lengths, packs them into
fixed-size buffers and fills tensors with seeded normal values.  It is the one module that both
the GPU path's tests and the CPU oracle's tests may use, so that both see the same bytes.

The length distributions are long-tailed stand-ins for the corpora of the paper's Sec. 8.1 (short
sequences dominate, long ones are rare: Sec. 3.1); buffers are filled the way the paper's
max-length packing baseline fills them (Sec. 3.2 and App. A.2: first-fit-decreasing bin packing
to the context length).
"""
from dataclasses import dataclass

import numpy as np

TENSOR_IDS = {"lengths": 0, "q": 1, "k": 2, "v": 3, "do": 4}


@dataclass(frozen=True)
class Config:
    cid: int
    name: str
    dtype: str          # "bf16" or "fp32"
    hq: int
    hkv: int
    d: int
    n_buffers: int
    buffer_tokens: int

    @property
    def total_tokens(self):
        return self.n_buffers * self.buffer_tokens

    @property
    def scale(self):
        return 1.0 / float(np.sqrt(self.d))


CONFIGS = {
    1: Config(1, "tiny-fp32", "fp32", 2, 2, 64, 1, 256),
    2: Config(2, "7b-lognormal-16k", "bf16", 32, 32, 128, 1, 16384),
    3: Config(3, "13b-pareto-4x32k", "bf16", 40, 40, 128, 4, 32768),
    4: Config(4, "imbalance-gqa-8x32k", "bf16", 32, 8, 128, 8, 32768),
    5: Config(5, "longctx-gqa-2x64k", "bf16", 64, 8, 128, 2, 65536),
}


def _rng(cid, tensor_id, stream=0):
    return np.random.Generator(np.random.Philox(key=[1000 * cid + tensor_id, stream]))


def _first_fit_decreasing(lengths, n_bins, cap):
    """Sort decreasing, put each length into the first bin with room; lengths that fit nowhere
    are dropped.  Returns the per-bin lists."""
    bins = [[] for _ in range(n_bins)]
    room = [cap] * n_bins
    for L in sorted((int(x) for x in lengths), reverse=True):
        for b in range(n_bins):
            if L <= room[b]:
                bins[b].append(L)
                room[b] -= L
                break
    return bins, room


def _top_up(bins, room, draw):
    """Fill every bin exactly: append one more draw truncated to the room left (repeat while the
    truncated draw still leaves room)."""
    for b in range(len(bins)):
        while room[b] > 0:
            L = min(int(draw()), room[b])
            bins[b].append(L)
            room[b] -= L


def seqlens(cid):
    """Sequence lengths of configuration `cid`, buffer after buffer, every buffer exactly full."""
    cfg = CONFIGS[cid]
    rng = _rng(cid, TENSOR_IDS["lengths"])
    cap = cfg.buffer_tokens
    if cid == 1:
        return [1, 7, 64, 184]
    if cid == 2:
        out, room = [], cap
        while room > 0:
            L = int(np.clip(np.rint(np.exp(rng.normal(np.log(1024.0), 1.0))), 32, cap))
            L = min(L, room)
            out.append(L)
            room -= L
        return out
    if cid == 3:
        def draw():
            u = 1.0 - rng.random()          # (0, 1]
            return max(1, min(int(np.floor(128.0 * u ** (-1.0 / 1.2))), cap))
        drawn = []
        while sum(drawn) < cfg.total_tokens:
            drawn.append(draw())
        bins, room = _first_fit_decreasing(drawn, cfg.n_buffers, cap)
        _top_up(bins, room, draw)
        return [L for b in bins for L in b]
    if cid == 4:
        out = [cap]
        for _ in range(1, cfg.n_buffers):
            room = cap
            while room > 0:
                L = min(int(rng.integers(64, 1025)), room)
                out.append(L)
                room -= L
        return out
    if cid == 5:
        def draw():
            u = rng.random()
            if u < 0.70:
                return int(rng.integers(32, 2049))
            if u < 0.95:
                return int(rng.integers(2048, 16385))
            return int(rng.integers(16384, 65537))
        drawn = []
        while sum(drawn) < cfg.total_tokens:
            drawn.append(draw())
        bins, room = _first_fit_decreasing(drawn, cfg.n_buffers, cap)
        _top_up(bins, room, draw)
        return [L for b in bins for L in b]
    raise KeyError(cid)


def cu_seqlens(lengths):
    cu = np.zeros(len(lengths) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(np.asarray(lengths, dtype=np.int64))
    return cu


def causal_pairs(lengths):
    """Number of (query, key) pairs with key <= query, summed over sequences."""
    return int(sum(int(L) * (int(L) + 1) // 2 for L in lengths))


def f32_to_bf16_bits(x):
    """Round float32 to bfloat16 (round to nearest, ties to even); returns the uint16 patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_tensor(cid, name, T, H, d, dtype, heads=None):
    """Seeded N(0,1) tensor [T, H, d].  Every head has its own stream, so any subset of heads can
    be regenerated alone (`heads`: list of head indices -> [T, len(heads), d]).  Returns float32
    holding exactly the values the GPU sees (bf16 configs: already rounded to bf16)."""
    heads = list(range(H)) if heads is None else list(heads)
    out = np.empty((T, len(heads), d), dtype=np.float32)
    for n, h in enumerate(heads):
        x = _rng(cid, TENSOR_IDS[name], stream=h + 1).standard_normal((T, d), dtype=np.float32)
        if dtype == "bf16":
            x = bf16_bits_to_f32(f32_to_bf16_bits(x))
        out[:, n, :] = x
    return out


def custom(lengths, hq, hkv, d, dtype, seed):
    """Free-form seeded case for tests: returns (cu_seqlens, q, k, v, do) as float32 arrays that
    hold exactly representable values of `dtype`."""
    cu = cu_seqlens(lengths)
    T = int(cu[-1])
    rng = np.random.Generator(np.random.Philox(key=[seed, 7]))
    def t(H):
        x = rng.standard_normal((T, H, d), dtype=np.float32)
        return bf16_bits_to_f32(f32_to_bf16_bits(x)) if dtype == "bf16" else x
    return cu, t(hq), t(hkv), t(hkv), t(hq)
