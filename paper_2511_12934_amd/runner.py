"""Host-side plumbing shared by the tests, the smoke check and the benchmark:
moves a synthetic workload into device memory and drives the C ABI through
``binding``.  No scoring arithmetic lives here.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Tuple, List, Optional, Sequence

import numpy as np

from . import binding as B
from . import workloads as wl


def torch_dtype(dtype: str):
    import torch
    return torch.float32 if dtype == "f32" else torch.bfloat16


def to_device(a: Optional[np.ndarray], dtype: str, device="cuda:0"):
    """float32 host array holding storage-rounded values -> device tensor of the storage type."""
    import torch
    if a is None:
        return None
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device).to(torch_dtype(dtype)).contiguous()


def from_device_f32(t) -> np.ndarray:
    import torch
    return t.detach().to(torch.float32).cpu().numpy()


@dataclass
class DeviceRequest:
    req: B.Request
    ids_host: np.ndarray
    logits: object          # torch fp32 [n]
    scores: object          # torch fp32 [n]
    keep: tuple             # device tensors kept alive


def upload_request(cfg: wl.Config, user: wl.User, ids: np.ndarray, device="cuda:0",
                   with_scores: bool = True) -> DeviceRequest:
    import torch
    u = to_device(user.user_vec, cfg.dtype, device)
    k = to_device(user.seq_keys, cfg.dtype, device)
    v = to_device(user.seq_vals, cfg.dtype, device)
    cv = to_device(user.cross_vecs, cfg.dtype, device)
    idt = torch.from_numpy(np.ascontiguousarray(ids, dtype=np.int32)).to(device)
    z = torch.full((ids.size,), float("nan"), dtype=torch.float32, device=device)
    y = torch.full((ids.size,), float("nan"), dtype=torch.float32, device=device) if with_scores else None
    return DeviceRequest(B.Request(u, k, v, idt, z, y, cv), np.asarray(ids, np.int32), z, y, (u, k, v, cv, idt))


def slice_request(cfg: wl.Config, dr: DeviceRequest, lo: int, hi: int) -> DeviceRequest:
    """A mini-batch slice [lo, hi) of a request: same user tensors, views of ids and outputs."""
    q = dr.req
    z = dr.logits[lo:hi]
    y = dr.scores[lo:hi] if dr.scores is not None else None
    ids = q.cand_ids[lo:hi]
    return DeviceRequest(B.Request(q.user_vec, q.seq_keys, q.seq_vals, ids, z, y, q.cross_vecs, q.seq_len),
                         dr.ids_host[lo:hi], z, y, dr.keep)


class DeviceModel:
    def __init__(self, cfg: wl.Config, model: wl.Model, device="cuda:0"):
        self.weights = [to_device(w, cfg.dtype, device) for w in model.weights]
        self.biases = [to_device(b, cfg.dtype, device) for b in model.biases]
        self.w_q = to_device(model.w_q, cfg.dtype, device)


def make_context(cfg: wl.Config, dmodel: DeviceModel, table_dev, *, max_users: Optional[int] = None,
                 max_candidates: Optional[int] = None, max_seq_len: Optional[int] = None,
                 with_biases: bool = True) -> B.Context:
    return B.Context(dtype=B.AIF_F32 if cfg.dtype == "f32" else B.AIF_BF16, table=table_dev,
                     d_user=cfg.d_user, d_attn=cfg.d_attn, n_heads=cfg.n_heads,
                     max_seq_len=cfg.seq_len if max_seq_len is None else max_seq_len,
                     layer_dims=list(cfg.mlp_dims), weights=dmodel.weights,
                     biases=dmodel.biases if with_biases else None, w_q=dmodel.w_q,
                     cross_mode=cfg.cross_mode, n_cross=cfg.n_cross, d_cross_vec=cfg.d_cross_vec,
                     max_candidates=cfg.n_cand if max_candidates is None else max_candidates,
                     max_users=cfg.n_users if max_users is None else max_users)


def peek_features(ctx: B.Context, cfg: wl.Config, req_index: int, n_rows: int) -> np.ndarray:
    """Rows of the feature matrix [e | attention | cross] of request ``req_index`` as float32."""
    import torch
    torch.cuda.synchronize()
    ld = cfg.d_item + cfg.d_attn + cfg.d_cross
    host = np.empty(n_rows * ld, dtype=np.float32 if cfg.dtype == "f32" else np.uint16)
    ctx.aif_peek_features(req_index, 0, n_rows, host.ctypes.data)
    if cfg.dtype == "f32":
        return host.reshape(n_rows, ld)
    return wl.bf16_to_f32(host).reshape(n_rows, ld)


class Workload:
    """One configuration resident on the device, in the launch configuration the
    benchmark times: ``step()`` = aif_score_topk over all users (aif_score_batch + aif_topk when the
    requests are cut into mini-batches).

    With ``n_sets`` > 1 the same users arrive with ``n_sets`` different candidate
    lists and ``step()`` takes them in turn, so that consecutive steps do not
    gather the same table rows out of the caches (set 0 is the configuration's
    own list; the others are drawn by the same sampler with later seeds)."""

    def __init__(self, cfg: wl.Config, device="cuda:0", n_users: Optional[int] = None,
                 n_cand: Optional[int] = None, n_items: Optional[int] = None, host_table: bool = False,
                 minibatch: Optional[int] = None, n_sets: int = 1):
        import torch
        self.cfg = cfg
        self.torch = torch
        self.n_users = cfg.n_users if n_users is None else n_users
        self.n_cand = cfg.n_cand if n_cand is None else n_cand
        self.n_items = cfg.n_items if n_items is None else n_items
        self.model = wl.make_model(cfg)
        self.dmodel = DeviceModel(cfg, self.model, device)
        if host_table:
            rng = np.random.default_rng(cfg.seed)
            self.table_host = wl.make_table_host(cfg, rng, self.n_items)
            self.table = to_device(self.table_host, cfg.dtype, device)
        else:
            self.table_host = None
            self.table = wl.make_table_device(cfg, device, self.n_items)
        self.requests = wl.make_requests(cfg, self.n_users, self.n_cand, self.n_items)
        self.dev = [upload_request(cfg, r.user, r.ids, device) for r in self.requests]
        # the launch list: whole requests, or each cut into mini-batches
        self.launch: List[DeviceRequest] = []
        for d in self.dev:
            if minibatch:
                self.launch += [slice_request(cfg, d, lo, min(lo + minibatch, self.n_cand))
                                for lo in range(0, self.n_cand, minibatch)]
            else:
                self.launch.append(d)
        self.ctx = make_context(cfg, self.dmodel, self.table, max_users=len(self.launch),
                                max_candidates=max(d.ids_host.size for d in self.launch))
        self.packed = B.pack_requests([d.req for d in self.launch])
        # further candidate lists for the same users: only ids differ, outputs and user tensors are shared
        self.sets = [(self.launch, self.packed)]
        for si in range(1, n_sets):
            if minibatch:
                raise ValueError("n_sets > 1 is for whole requests")
            lst = []
            for d, ids in zip(self.dev, wl.make_id_lists(cfg, si, self.n_users, self.n_cand, self.n_items)):
                idt = torch.from_numpy(np.ascontiguousarray(ids, dtype=np.int32)).to(device)
                q = d.req
                lst.append(DeviceRequest(B.Request(q.user_vec, q.seq_keys, q.seq_vals, idt, d.logits, d.scores,
                                                   q.cross_vecs, q.seq_len), ids, d.logits, d.scores,
                                         d.keep + (idt,)))
            self.sets.append((lst, B.pack_requests([x.req for x in lst])))
        self._turn = 0
        self.whole_requests = not minibatch
        self.k = cfg.top_k
        self.idx = torch.empty((self.n_users, self.k), dtype=torch.int32, device=device)
        self.val = torch.empty((self.n_users, self.k), dtype=torch.float32, device=device)
        self._logits = [d.logits for d in self.dev]

    @property
    def total_candidates(self) -> int:
        return self.n_users * self.n_cand

    def step(self):
        launch, packed = self.sets[self._turn % len(self.sets)]
        self._turn += 1
        if self.whole_requests:             # one request per user: scoring and selection as one call
            self.ctx.aif_score_topk(launch, self.k, self.idx, self.val, packed=packed)
        else:                               # mini-batch slices: one selection over each user's whole list
            self.ctx.aif_score_batch(launch, packed=packed)
            self.ctx.aif_topk(self._logits, self.k, self.idx, self.val)

    def rows_of(self, user: int, positions: np.ndarray) -> np.ndarray:
        """Item rows of some candidates of a user, fetched with torch indexing (not the library)."""
        import torch
        ids = torch.from_numpy(self.requests[user].ids[positions].astype(np.int64)).to(self.table.device)
        return from_device_f32(self.table.index_select(0, ids))


# ---------------------------------------------------------------------------
# LSH behaviour modelling (include/aif_lsh.h)
# ---------------------------------------------------------------------------
@dataclass
class LshDeviceRequest:
    req: B.LshRequest
    ids_host: np.ndarray
    din: object             # torch fp32 [n, d_out]
    tiers: object           # torch int32 [n, n_tiers]
    keep: tuple


def upload_lsh_request(cfg: wl.LshConfig, user: wl.LshUser, ids: np.ndarray, device="cuda:0") -> LshDeviceRequest:
    import torch
    sig = torch.from_numpy(np.ascontiguousarray(user.seq_sigs)).to(device)
    emb = to_device(user.seq_emb, cfg.dtype, device) if user.seq_emb.size else torch.empty((0, cfg.d_out), dtype=torch_dtype(cfg.dtype), device=device)
    idt = torch.from_numpy(np.ascontiguousarray(ids, dtype=np.int32)).to(device)
    din = torch.full((ids.size, cfg.d_out), float("nan"), dtype=torch.float32, device=device)
    tiers = torch.full((ids.size, cfg.n_tiers), -7, dtype=torch.int32, device=device)
    return LshDeviceRequest(B.LshRequest(sig, emb, idt, din, tiers, seq_len=user.seq_sigs.shape[0]),
                            np.asarray(ids, np.int32), din, tiers, (sig, emb, idt))


def slice_lsh_request(dr: LshDeviceRequest, lo: int, hi: int) -> LshDeviceRequest:
    q = dr.req
    return LshDeviceRequest(B.LshRequest(q.seq_sigs, q.seq_emb, q.cand_ids[lo:hi], dr.din[lo:hi], dr.tiers[lo:hi], q.seq_len),
                            dr.ids_host[lo:hi], dr.din[lo:hi], dr.tiers[lo:hi], dr.keep)


def make_lsh_context(cfg: wl.LshConfig, sig_table_dev, *, max_users: Optional[int] = None,
                     max_candidates: Optional[int] = None, max_seq_len: Optional[int] = None) -> B.LshContext:
    return B.LshContext(sig_table=sig_table_dev, d_out=cfg.d_out, n_tiers=cfg.n_tiers,
                        dtype=B.AIF_F32 if cfg.dtype == "f32" else B.AIF_BF16,
                        max_seq_len=cfg.seq_len if max_seq_len is None else max_seq_len,
                        max_candidates=cfg.n_cand if max_candidates is None else max_candidates,
                        max_users=cfg.n_users if max_users is None else max_users)


class LshWorkload:
    """One LSH configuration resident on the device; ``step()`` = one aif_lsh_batch over all users."""

    def __init__(self, cfg: wl.LshConfig, device="cuda:0", n_users: Optional[int] = None,
                 n_cand: Optional[int] = None, n_items: Optional[int] = None, seq_len: Optional[int] = None):
        import torch
        self.cfg = cfg
        self.n_users = cfg.n_users if n_users is None else n_users
        self.n_cand = cfg.n_cand if n_cand is None else n_cand
        self.n_items = cfg.n_items if n_items is None else n_items
        self.seq_len = cfg.seq_len if seq_len is None else seq_len
        self.table_host = wl.make_sig_table_host(cfg, self.n_items)
        self.table = torch.from_numpy(self.table_host).to(device)
        self.requests = wl.make_lsh_requests(cfg, self.n_users, self.n_cand, self.n_items, self.seq_len)
        self.dev = [upload_lsh_request(cfg, r.user, r.ids, device) for r in self.requests]
        self.ctx = make_lsh_context(cfg, self.table, max_users=self.n_users, max_candidates=self.n_cand,
                                    max_seq_len=self.seq_len)
        self.packed = B.pack_lsh_requests([d.req for d in self.dev])

    @property
    def total_candidates(self) -> int:
        return self.n_users * self.n_cand

    def step(self):
        self.ctx.aif_lsh_batch([d.req for d in self.dev], packed=self.packed)


# ---------------------------------------------------------------------------
# user-side asynchronous network (include/aif_user.h)
# ---------------------------------------------------------------------------
@dataclass
class UserNetDevice:
    req: B.UserRequest
    user_vec: "object"       # torch [2 d]
    seq_out: "object"        # torch [L, d]
    keep: Tuple = ()


def make_user_context(cfg: wl.UserNetConfig, model: wl.UserNetModel, *, max_users: Optional[int] = None,
                      max_seq_len: Optional[int] = None, device="cuda:0") -> B.UserContext:
    w = [to_device(a, cfg.dtype, device) for a in (model.w_profile, model.w_seq, model.w_ffn, model.b_ffn)]
    return B.UserContext(dtype=B.AIF_F32 if cfg.dtype == "f32" else B.AIF_BF16, d_raw=cfg.d_raw, d=cfg.d,
                         w_profile=w[0], w_seq=w[1], w_ffn=w[2], b_ffn=w[3],
                         max_seq_len=cfg.seq_len if max_seq_len is None else max_seq_len,
                         max_users=cfg.n_users if max_users is None else max_users)


def upload_raw_user(cfg: wl.UserNetConfig, user: wl.RawUser, device="cuda:0") -> UserNetDevice:
    import torch
    p = to_device(user.profile, cfg.dtype, device)
    sq = to_device(user.seq, cfg.dtype, device)
    L = user.seq.shape[0]
    uv = torch.zeros(2 * cfg.d, dtype=torch_dtype(cfg.dtype), device=device)
    so = torch.zeros((max(L, 1), cfg.d), dtype=torch_dtype(cfg.dtype), device=device)
    return UserNetDevice(B.UserRequest(p, sq, uv, so, L), uv, so, (p, sq))


class UserNetWorkload:
    """The user side of one configuration resident on the device: ``step()`` = aif_user_precompute over all users."""

    def __init__(self, cfg: wl.UserNetConfig, device="cuda:0", n_users: Optional[int] = None):
        self.cfg = cfg
        self.n_users = cfg.n_users if n_users is None else n_users
        self.model = wl.make_user_net_model(cfg)
        self.users = wl.make_raw_users(cfg, self.n_users)
        self.dev = [upload_raw_user(cfg, u, device) for u in self.users]
        self.ctx = make_user_context(cfg, self.model, max_users=self.n_users, device=device)
        self.packed = B.pack_user_requests([d.req for d in self.dev])

    def step(self, stream: Optional[int] = None):
        self.ctx.aif_user_precompute([d.req for d in self.dev], packed=self.packed, stream=stream)


class AsyncPipeline:
    """Steady state of the two phases of Sec. 3.1 on one device: while the real-time phase scores the candidates
    of one batch of users (stream ``s_score``), the pre-computation phase runs the user-side network for the next
    batch (stream ``s_user``), as it would beside retrieval.  The cached user tensors are double-buffered; a
    scoring call waits for the event that marks its buffer complete, a pre-computation waits until the scoring
    call that last read its buffer has finished.  ``step(i, overlap=False)`` runs the same work on one stream."""

    def __init__(self, cfg: wl.Config, ucfg: wl.UserNetConfig, device="cuda:0", n_items: Optional[int] = None,
                 n_cand: Optional[int] = None, n_users: Optional[int] = None):
        import torch
        assert cfg.d_user == 2 * ucfg.d and cfg.d_attn == ucfg.d and cfg.d_item == ucfg.d and cfg.dtype == ucfg.dtype
        self.cfg, self.ucfg, self.torch = cfg, ucfg, torch
        self.n_users = cfg.n_users if n_users is None else n_users
        self.n_cand = cfg.n_cand if n_cand is None else n_cand
        self.n_items = cfg.n_items if n_items is None else n_items
        self.model = wl.make_model(cfg)
        self.dmodel = DeviceModel(cfg, self.model, device)
        self.umodel = wl.make_user_net_model(ucfg)
        self.table = wl.make_table_device(cfg, device, self.n_items)
        self.uctx = make_user_context(ucfg, self.umodel, max_users=self.n_users, device=device)
        self.ctx = make_context(cfg, self.dmodel, self.table, max_users=self.n_users, max_candidates=self.n_cand,
                                max_seq_len=ucfg.seq_len)
        self.raw, self.udev, self.upacked, self.ids, self.reqs, self.packed, self.logits = [], [], [], [], [], [], []
        for b in range(2):
            raw = wl.make_raw_users(ucfg, self.n_users, seed=ucfg.seed + 31 * b)
            udev = [upload_raw_user(ucfg, u, device) for u in raw]
            ids = wl.make_id_lists(cfg, b, self.n_users, self.n_cand, self.n_items)
            reqs, zs = [], []
            for d, idl in zip(udev, ids):
                idt = torch.from_numpy(np.ascontiguousarray(idl, dtype=np.int32)).to(device)
                z = torch.full((idl.size,), float("nan"), dtype=torch.float32, device=device)
                reqs.append(B.Request(d.user_vec, d.seq_out, d.seq_out, idt, z, None, d.user_vec[ucfg.d:], d.req.seq_len))
                zs.append(z)
            self.raw.append(raw)
            self.udev.append(udev)
            self.upacked.append(B.pack_user_requests([d.req for d in udev]))
            self.ids.append(ids)
            self.reqs.append(reqs)
            self.packed.append(B.pack_requests(reqs))
            self.logits.append(zs)
        self.k = cfg.top_k
        self.idx = torch.empty((self.n_users, self.k), dtype=torch.int32, device=device)
        self.val = torch.empty((self.n_users, self.k), dtype=torch.float32, device=device)
        self.s_score = torch.cuda.Stream(device=device)
        self.s_user = torch.cuda.Stream(device=device)
        self.u_done = [torch.cuda.Event() for _ in range(2)]
        self.s_done = [torch.cuda.Event() for _ in range(2)]
        self._s_recorded = [False, False]

    @property
    def total_candidates(self) -> int:
        return self.n_users * self.n_cand

    def _precompute(self, b: int):
        self.uctx.aif_user_precompute([d.req for d in self.udev[b]], packed=self.upacked[b])

    def _score(self, b: int):
        self.ctx.aif_score_batch(self.reqs[b], packed=self.packed[b])
        self.ctx.aif_topk(self.logits[b], self.k, self.idx, self.val)

    def prime(self):
        """User tensors of buffer 0, before the first overlapped step."""
        torch = self.torch
        with torch.cuda.stream(self.s_user):
            self._precompute(0)
            self.u_done[0].record()

    def step(self, i: int, overlap: bool = True):
        torch = self.torch
        b, nb = i % 2, 1 - i % 2
        if not overlap:
            with torch.cuda.stream(self.s_score):
                self._precompute(b)
                self._score(b)
            return
        with torch.cuda.stream(self.s_user):
            if self._s_recorded[nb]:
                self.s_user.wait_event(self.s_done[nb])
            self._precompute(nb)
            self.u_done[nb].record()
        with torch.cuda.stream(self.s_score):
            self.s_score.wait_event(self.u_done[b])
            self._score(b)
            self.s_done[b].record()
            self._s_recorded[b] = True
