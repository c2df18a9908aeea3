"""Seeded synthetic workloads shaped like the paper's pre-ranking traffic.

This module only makes inputs (shapes, distributions, storage rounding).  It
holds none of the scoring arithmetic and is the one module both the GPU tests
and the CPU oracle tests draw their inputs from.

The paper's traffic (Sec. 5.1, production logs) is not public; requests here
follow its stated scale -- about 10^4 retrieved candidates per request cut to
about 10^2, 1,000-item mini-batches (Sec. 1) -- with sizes per configuration
C1..C5 below.  Values are N(0, 0.1^2) rounded once to the storage type;
weights are Xavier-uniform with zero biases.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional, Tuple

import numpy as np

CROSS_NONE, CROSS_HADAMARD, CROSS_SEGDOT, CROSS_BEA = 0, 1, 2, 3
SEED_BASE = 0xA1F0000


@dataclass(frozen=True)
class Config:
    name: str
    index: int                  # 1..5, enters the seed
    dtype: str                  # "f32" | "bf16": storage type of table, user tensors, weights
    n_users: int
    n_cand: int
    n_items: int
    d_item: int
    id_dist: str                # "uniform" | "zipf"
    seq_len: int
    d_attn: int
    n_heads: int
    use_wq: bool
    cross_mode: int
    n_cross: int
    d_cross_vec: int
    d_user: int
    mlp_dims: Tuple[int, ...]
    top_k: int
    zipf_s: float = 1.1

    @property
    def d_cross(self) -> int:
        if self.cross_mode == CROSS_HADAMARD:
            return self.d_item
        if self.cross_mode == CROSS_SEGDOT:
            return self.n_cross * (self.d_item // self.d_cross_vec)
        if self.cross_mode == CROSS_BEA:
            return self.d_cross_vec
        return 0

    @property
    def d_in(self) -> int:
        return self.d_user + self.d_item + self.d_attn + self.d_cross

    @property
    def seed(self) -> int:
        return SEED_BASE + self.index

    def scaled(self, **kw) -> "Config":
        return replace(self, **kw)


CONFIGS: Dict[str, Config] = {
    "C1": Config("C1", 1, "f32", 1, 1_000, 100_000, 64, "uniform", 50, 32, 1, True,
                 CROSS_HADAMARD, 0, 0, 64, (224, 128, 64, 1), 100),
    "C2": Config("C2", 2, "bf16", 1, 10_000, 1_000_000, 64, "zipf", 1_000, 64, 1, False,
                 CROSS_HADAMARD, 0, 0, 64, (256, 256, 128, 1), 200),
    "C3": Config("C3", 3, "bf16", 64, 10_000, 10_000_000, 64, "zipf", 500, 64, 1, False,
                 CROSS_HADAMARD, 0, 0, 64, (256, 512, 256, 1), 100),
    "C4": Config("C4", 4, "bf16", 16, 20_000, 50_000_000, 128, "uniform", 200, 128, 4, False,
                 CROSS_HADAMARD, 0, 0, 128, (512, 256, 1), 100),
    "C5": Config("C5", 5, "bf16", 32, 10_000, 10_000_000, 256, "zipf", 2_000, 128, 8, True,
                 CROSS_SEGDOT, 16, 64, 576, (1024, 1024, 512, 256, 1), 150),
    # C3 with its cross block formed by the Bridge Embedding Approximation (Sec. 4.1): 16 bridges (the
    # paper's quality plateau is at about 10), the item row = 48-wide vector + 16 bridge weights, the user
    # side brings 16 vectors of width 64.
    "B3": Config("B3", 6, "bf16", 64, 10_000, 10_000_000, 64, "zipf", 500, 64, 1, False,
                 CROSS_BEA, 16, 64, 64, (256, 512, 256, 1), 100),
    # C3 fed by the asynchronous user-side network (Sec. 3.1): the cached user vector is
    # [U_self_attention | U_profile_attention] (2 x 64), keys = values = the projected sequence, the Hadamard
    # operand is U_profile_attention.  See USER_CONFIGS["U3"] for the network that produces them.
    "A3": Config("A3", 7, "bf16", 64, 10_000, 10_000_000, 64, "zipf", 500, 64, 1, False,
                 CROSS_HADAMARD, 0, 0, 128, (320, 512, 256, 1), 100),
}
for _c in CONFIGS.values():
    assert _c.d_in == _c.mlp_dims[0], (_c.name, _c.d_in)


# ----------------------------------------------------------------------------
# storage rounding
# ----------------------------------------------------------------------------
def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    nan = (u & 0x7FFFFFFF) > 0x7F800000
    r = (u + (0x7FFF + ((u >> 16) & 1))) >> 16
    r = np.where(nan, (u >> 16) | 0x40, r)
    return r.astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32)


def round_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float32 values once to the storage type; result is float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "bf16":
        return bf16_to_f32(bf16_bits(x)).reshape(x.shape)
    raise ValueError(dtype)


# ----------------------------------------------------------------------------
# model weights
# ----------------------------------------------------------------------------
@dataclass
class Model:
    dims: Tuple[int, ...]
    weights: List[np.ndarray]           # W_l [out, in], float32 holding storage-rounded values
    biases: List[np.ndarray]            # b_l [out]
    w_q: Optional[np.ndarray]           # [d_attn, d_item] or None


def _xavier(rng: np.random.Generator, fan_out: int, fan_in: int) -> np.ndarray:
    lim = np.sqrt(6.0 / (fan_in + fan_out))
    return rng.uniform(-lim, lim, size=(fan_out, fan_in)).astype(np.float32)


def make_model(cfg: Config, seed: Optional[int] = None, bias_scale: float = 0.0) -> Model:
    """Xavier-uniform weights; biases zero unless ``bias_scale`` is given (tests)."""
    rng = np.random.default_rng((cfg.seed if seed is None else seed) ^ 0x5EED)
    ws, bs = [], []
    for l in range(len(cfg.mlp_dims) - 1):
        ws.append(round_storage(_xavier(rng, cfg.mlp_dims[l + 1], cfg.mlp_dims[l]), cfg.dtype))
        b = rng.standard_normal(cfg.mlp_dims[l + 1]).astype(np.float32) * bias_scale
        bs.append(round_storage(b, cfg.dtype))
    wq = round_storage(_xavier(rng, cfg.d_attn, cfg.d_item), cfg.dtype) if cfg.use_wq else None
    return Model(tuple(cfg.mlp_dims), ws, bs, wq)


# ----------------------------------------------------------------------------
# user side
# ----------------------------------------------------------------------------
@dataclass
class User:
    user_vec: np.ndarray                # [d_user]
    seq_keys: np.ndarray                # [L, d_attn]
    seq_vals: np.ndarray                # [L, d_attn]
    cross_vecs: Optional[np.ndarray]    # SEGDOT, BEA: [n_cross, d_cross_vec]; HADAMARD: None (= user_vec)


def make_user(cfg: Config, rng: np.random.Generator, sigma: float = 0.1,
              seq_len: Optional[int] = None) -> User:
    L = cfg.seq_len if seq_len is None else seq_len
    g = lambda *s: round_storage(rng.standard_normal(s).astype(np.float32) * sigma, cfg.dtype)
    u = g(cfg.d_user)
    k = g(L, cfg.d_attn)
    v = g(L, cfg.d_attn)
    cv = g(cfg.n_cross, cfg.d_cross_vec) if cfg.cross_mode in (CROSS_SEGDOT, CROSS_BEA) else None
    if cfg.cross_mode == CROSS_HADAMARD and cfg.d_user != cfg.d_item:
        cv = u[cfg.d_user - cfg.d_item:].copy()         # the trailing d_item entries of the user vector
    return User(u, k, v, cv)


# ----------------------------------------------------------------------------
# item table
# ----------------------------------------------------------------------------
def make_table_host(cfg: Config, rng: np.random.Generator, n_items: Optional[int] = None,
                    sigma: float = 0.1) -> np.ndarray:
    """Whole table on the host (small configurations only).  With the BEA cross block (Sec. 4.1) the
    last n_cross entries of a row are the item's bridge weights as the nearline pipeline would have
    left them: non-negative, summing to one (normalised exponentials, i.e. uniform on the simplex)."""
    n = cfg.n_items if n_items is None else n_items
    t = rng.standard_normal((n, cfg.d_item), dtype=np.float32) * np.float32(sigma)
    if cfg.cross_mode == CROSS_BEA:
        w = rng.exponential(size=(n, cfg.n_cross))
        t[:, cfg.d_item - cfg.n_cross:] = (w / w.sum(axis=1, keepdims=True)).astype(np.float32)
    return round_storage(t, cfg.dtype)


def make_table_device(cfg: Config, device, n_items: Optional[int] = None, sigma: float = 0.1,
                      chunk_rows: int = 4_000_000):
    """Whole table filled on the device in chunks (tables too large for the host)."""
    import torch

    n = cfg.n_items if n_items is None else n_items
    tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    gen = torch.Generator(device=device)
    gen.manual_seed(cfg.seed)
    out = torch.empty((n, cfg.d_item), dtype=tdt, device=device)
    for lo in range(0, n, chunk_rows):
        hi = min(n, lo + chunk_rows)
        blk = torch.randn((hi - lo, cfg.d_item), dtype=torch.float32, device=device, generator=gen) * sigma
        if cfg.cross_mode == CROSS_BEA:         # bridge weights in the row's tail, as in make_table_host
            w = torch.empty((hi - lo, cfg.n_cross), dtype=torch.float32, device=device).exponential_(generator=gen)
            blk[:, cfg.d_item - cfg.n_cross:] = w / w.sum(dim=1, keepdim=True)
            del w
        out[lo:hi] = blk.to(tdt)
        del blk
    return out


# ----------------------------------------------------------------------------
# candidate ids
# ----------------------------------------------------------------------------
class IdSampler:
    """Candidate ids of one request: ``n`` distinct rows (a retrieval stage
    returns a set), uniform or Zipf(s) over the table.  Zipf: P(rank r) ~ r^-s
    on r in [1, n_items] by inverse CDF with the exact truncated normaliser;
    rank -> row through a fixed seeded permutation so hot rows are scattered.
    Ids repeat across users (the cross-request reuse of Sec. 1)."""

    def __init__(self, cfg: Config, n_items: Optional[int] = None):
        self.n_items = cfg.n_items if n_items is None else n_items
        self.dist = cfg.id_dist
        if self.dist == "zipf":
            r = np.arange(1, self.n_items + 1, dtype=np.float64)
            self.cdf = np.cumsum(r ** (-cfg.zipf_s))
            self.cdf /= self.cdf[-1]
            prng = np.random.default_rng(cfg.seed ^ 0x9E3779B9)
            self.perm = prng.permutation(self.n_items).astype(np.int32)

    def _draw(self, rng: np.random.Generator, m: int) -> np.ndarray:
        if self.dist == "uniform":
            return rng.integers(0, self.n_items, size=m, dtype=np.int64).astype(np.int32)
        ranks = np.searchsorted(self.cdf, rng.random(m), side="left")
        ranks = np.minimum(ranks, self.n_items - 1)
        return self.perm[ranks]

    def sample(self, rng: np.random.Generator, n: int) -> np.ndarray:
        if n > self.n_items:
            raise ValueError("more distinct candidates than table rows")
        if n <= 0:
            return np.zeros(0, np.int32)
        got: List[np.ndarray] = []
        seen = set()
        have = 0
        while have < n:
            d = self._draw(rng, max(2 * (n - have), 64))
            _, first = np.unique(d, return_index=True)
            d = d[np.sort(first)]
            keep = np.fromiter((x not in seen for x in d.tolist()), dtype=bool, count=d.size)
            d = d[keep][: n - have]
            seen.update(d.tolist())
            got.append(d)
            have += d.size
        return np.concatenate(got).astype(np.int32)


@dataclass
class Request:
    user: User
    ids: np.ndarray


def make_requests(cfg: Config, n_users: Optional[int] = None, n_cand: Optional[int] = None,
                  n_items: Optional[int] = None, seed: Optional[int] = None,
                  sigma: float = 0.1) -> List[Request]:
    rng = np.random.default_rng(cfg.seed if seed is None else seed)
    sampler = IdSampler(cfg, n_items)
    nu = cfg.n_users if n_users is None else n_users
    nc = cfg.n_cand if n_cand is None else n_cand
    return [Request(make_user(cfg, rng, sigma), sampler.sample(rng, nc)) for _ in range(nu)]


def make_id_lists(cfg: Config, set_index: int, n_users: Optional[int] = None, n_cand: Optional[int] = None,
                  n_items: Optional[int] = None) -> List[np.ndarray]:
    """Another candidate list per user, same sampler, its own seed (set 0 is make_requests' own)."""
    rng = np.random.default_rng(cfg.seed + 7919 * set_index)
    sampler = IdSampler(cfg, n_items)
    nu = cfg.n_users if n_users is None else n_users
    nc = cfg.n_cand if n_cand is None else n_cand
    return [sampler.sample(rng, nc) for _ in range(nu)]


# ----------------------------------------------------------------------------
# LSH behaviour modelling (Sec. 4.3): synthetic signatures and history embeddings
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class LshConfig:
    """Shapes of one LSH workload.  Signatures are stand-ins for hashed multi-modal embeddings: items
    belong to clusters and an item's signature is its cluster's prototype with every bit flipped with
    probability ``flip`` (so similarities spread over the tiers as those of related and unrelated items
    do); nothing of the method is computed here."""
    name: str
    index: int
    dtype: str            # storage of the projected history embeddings
    n_users: int
    n_cand: int
    n_items: int
    d_bits: int           # d' of Eq. 5
    d_out: int            # d of Eq. 8
    n_tiers: int          # N of Eq. 9
    seq_len: int
    n_clusters: int = 64
    flip: float = 0.15

    @property
    def seed(self) -> int:
        return SEED_BASE + 100 + self.index

    def scaled(self, **kw) -> "LshConfig":
        return replace(self, **kw)


LSH_CONFIGS: Dict[str, LshConfig] = {
    # small: the oracle finishes it in seconds
    "L1": LshConfig("L1", 1, "f32", 1, 1_000, 100_000, 64, 64, 8, 2_000),
    # the long-sequence case: 64 users x 10^4 candidates, 10^4 history items each, 64-bit signatures
    # (d_lsh = 8 bytes = d / 8, Sec. 5.2.3), 64-wide bf16 history embeddings, 8 tiers
    "L2": LshConfig("L2", 2, "bf16", 64, 10_000, 10_000_000, 64, 64, 8, 10_000),
    # wider signatures and outputs, fewer users, l = 10^5 (the scale Sec. 4.3 quotes)
    "L3": LshConfig("L3", 3, "bf16", 8, 10_000, 10_000_000, 128, 128, 8, 100_000),
}


def _flip_bits(rng: np.random.Generator, proto: np.ndarray, flip: float) -> np.ndarray:
    """proto [n, nbytes] uint8 -> each bit flipped with probability flip."""
    n, nb = proto.shape
    mask = np.packbits(rng.random((n, nb * 8)) < flip, axis=1)
    return np.bitwise_xor(proto, mask)


def make_lsh_prototypes(cfg: LshConfig) -> np.ndarray:
    rng = np.random.default_rng(cfg.seed)
    return rng.integers(0, 256, (cfg.n_clusters, cfg.d_bits // 8), dtype=np.uint8)


def make_sig_table_host(cfg: LshConfig, n_items: Optional[int] = None, chunk: int = 1 << 18) -> np.ndarray:
    """Signature table [n_items, d_bits / 8] uint8 (item i belongs to cluster i mod n_clusters)."""
    n = cfg.n_items if n_items is None else n_items
    protos = make_lsh_prototypes(cfg)
    rng = np.random.default_rng(cfg.seed + 1)
    out = np.empty((n, cfg.d_bits // 8), dtype=np.uint8)
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        out[lo:hi] = _flip_bits(rng, protos[np.arange(lo, hi) % cfg.n_clusters], cfg.flip)
    return out


@dataclass
class LshUser:
    seq_sigs: np.ndarray      # [L, d_bits / 8] uint8
    seq_emb: np.ndarray       # [L, d_out] float32 holding storage-rounded values


def make_lsh_user(cfg: LshConfig, rng: np.random.Generator, seq_len: Optional[int] = None, sigma: float = 0.1) -> LshUser:
    """A user's history: items drawn from a few favoured clusters, their signatures and embeddings."""
    L = cfg.seq_len if seq_len is None else seq_len
    protos = make_lsh_prototypes(cfg)
    fav = rng.choice(cfg.n_clusters, size=min(8, cfg.n_clusters), replace=False)
    cl = fav[rng.integers(0, fav.size, L)]
    sigs = _flip_bits(rng, protos[cl], cfg.flip) if L else np.zeros((0, cfg.d_bits // 8), np.uint8)
    emb = round_storage(rng.standard_normal((L, cfg.d_out)).astype(np.float32) * sigma, cfg.dtype)
    return LshUser(sigs, emb)


@dataclass
class LshRequestHost:
    user: LshUser
    ids: np.ndarray


def make_lsh_requests(cfg: LshConfig, n_users: Optional[int] = None, n_cand: Optional[int] = None,
                      n_items: Optional[int] = None, seq_len: Optional[int] = None) -> List[LshRequestHost]:
    rng = np.random.default_rng(cfg.seed + 2)
    nu = cfg.n_users if n_users is None else n_users
    nc = cfg.n_cand if n_cand is None else n_cand
    ni = cfg.n_items if n_items is None else n_items
    out = []
    for _ in range(nu):
        user = make_lsh_user(cfg, rng, seq_len)
        ids = rng.choice(ni, size=nc, replace=False).astype(np.int32) if nc <= ni else rng.integers(0, ni, nc).astype(np.int32)
        out.append(LshRequestHost(user, ids))
    return out


# ----------------------------------------------------------------------------
# user-side asynchronous network (Sec. 3.1, Eq. 1-3): raw embeddings and weights
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class UserNetConfig:
    name: str
    index: int
    dtype: str
    n_users: int
    seq_len: int
    d_raw: int            # d^U: width of the profile / behaviour embeddings
    d: int                # common width after Eq. 1

    @property
    def seed(self) -> int:
        return SEED_BASE + 200 + self.index

    def scaled(self, **kw) -> "UserNetConfig":
        return replace(self, **kw)


USER_CONFIGS: Dict[str, UserNetConfig] = {
    # small, fp32: the user side of C1 (L = 50, attention width 32)
    "U1": UserNetConfig("U1", 1, "f32", 1, 50, 48, 32),
    # the user side of C3 / A3: 64 concurrent users, L = 500, 128-wide raw embeddings projected to 64
    "U3": UserNetConfig("U3", 3, "bf16", 64, 500, 128, 64),
}


@dataclass
class UserNetModel:
    w_profile: np.ndarray     # [d, d_raw]
    w_seq: np.ndarray         # [d, d_raw]
    w_ffn: np.ndarray         # [d, d]
    b_ffn: np.ndarray         # [d]


def make_user_net_model(cfg: UserNetConfig, seed: Optional[int] = None, bias_scale: float = 0.0) -> UserNetModel:
    """Xavier-uniform weights; the FFN bias is zero unless ``bias_scale`` is given (tests)."""
    rng = np.random.default_rng((cfg.seed if seed is None else seed) ^ 0x5EED)
    r = lambda a: round_storage(a, cfg.dtype)
    return UserNetModel(r(_xavier(rng, cfg.d, cfg.d_raw)), r(_xavier(rng, cfg.d, cfg.d_raw)), r(_xavier(rng, cfg.d, cfg.d)),
                        r(rng.standard_normal(cfg.d).astype(np.float32) * bias_scale))


@dataclass
class RawUser:
    profile: np.ndarray       # [d_raw]
    seq: np.ndarray           # [L, d_raw]


def make_raw_user(cfg: UserNetConfig, rng: np.random.Generator, sigma: float = 0.1, seq_len: Optional[int] = None) -> RawUser:
    L = cfg.seq_len if seq_len is None else seq_len
    g = lambda *s: round_storage(rng.standard_normal(s).astype(np.float32) * sigma, cfg.dtype)
    return RawUser(g(cfg.d_raw), g(L, cfg.d_raw))


def make_raw_users(cfg: UserNetConfig, n_users: Optional[int] = None, seed: Optional[int] = None, sigma: float = 0.1) -> List[RawUser]:
    rng = np.random.default_rng(cfg.seed if seed is None else seed)
    return [make_raw_user(cfg, rng, sigma) for _ in range(cfg.n_users if n_users is None else n_users)]
