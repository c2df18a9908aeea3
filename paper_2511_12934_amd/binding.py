"""Thin ctypes binding of ``libaif.so`` (see ``include/aif.h``).

Argument marshalling only: every step of the scoring path runs in the HIP
kernels behind the C ABI.  Tensors are torch tensors used purely as device
memory (``data_ptr()``) and the current torch stream is the HIP stream the
work is enqueued on.  A missing library raises; there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libaif.so")

AIF_OK, AIF_EINVAL, AIF_ESHAPE, AIF_ENOMEM, AIF_EDEVICE, AIF_ERANGE = range(6)
AIF_F32, AIF_BF16 = 0, 1
AIF_CROSS_NONE, AIF_CROSS_HADAMARD, AIF_CROSS_SEGDOT, AIF_CROSS_BEA = 0, 1, 2, 3

EXPORTS = ("aif_score_init", "aif_score_request", "aif_score_batch", "aif_topk", "aif_score_destroy",
           "aif_last_error", "aif_poll_device_errors", "aif_peek_features", "aif_profile_begin",
           "aif_profile_end", "aif_stage_kind", "aif_update_rows", "aif_swap_table", "aif_score_topk",
           "aif_profile_begin_stages", "aif_profile_begin_sampled", "aif_last_user_slots", "aif_score_topk_static",
           "aif_mlp_layer1_width")
STAGES = ("gather", "user_fold", "attention", "mlp", "topk")
LSH_EXPORTS = ("aif_lsh_init", "aif_lsh_batch", "aif_lsh_destroy", "aif_lsh_last_error",
               "aif_lsh_poll_device_errors", "aif_lsh_simtier_kind", "aif_lsh_din_kind", "aif_lsh_profile_begin", "aif_lsh_profile_end")
LSH_STAGES = ("user", "din", "simtier")
USER_EXPORTS = ("aif_user_init", "aif_user_precompute", "aif_user_destroy", "aif_user_last_error",
                "aif_user_attention_kind", "aif_user_profile_begin", "aif_user_profile_end")
USER_STAGES = ("project", "attention", "ffn_pool")


class aif_config(C.Structure):
    _fields_ = [("dtype", C.c_int), ("n_items", C.c_int64), ("d_item", C.c_int32), ("d_user", C.c_int32),
                ("d_attn", C.c_int32), ("n_heads", C.c_int32), ("max_seq_len", C.c_int32),
                ("cross_mode", C.c_int), ("n_cross", C.c_int32), ("d_cross_vec", C.c_int32),
                ("n_layers", C.c_int32), ("layer_dims", C.POINTER(C.c_int32)),
                ("max_candidates", C.c_int32), ("max_users", C.c_int32), ("flags", C.c_uint32)]


class aif_weights(C.Structure):
    _fields_ = [("item_table", C.c_void_p), ("w_q", C.c_void_p),
                ("w", C.POINTER(C.c_void_p)), ("b", C.POINTER(C.c_void_p))]


class aif_request(C.Structure):
    _fields_ = [("user_vec", C.c_void_p), ("cross_vecs", C.c_void_p), ("seq_keys", C.c_void_p),
                ("seq_vals", C.c_void_p), ("seq_len", C.c_int32), ("cand_ids", C.c_void_p),
                ("n_cand", C.c_int32), ("logits_out", C.c_void_p), ("scores_out", C.c_void_p)]


class aif_lsh_config(C.Structure):
    _fields_ = [("n_items", C.c_int64), ("d_bits", C.c_int32), ("d_out", C.c_int32), ("n_tiers", C.c_int32),
                ("dtype", C.c_int), ("max_seq_len", C.c_int32), ("max_candidates", C.c_int32),
                ("max_users", C.c_int32)]


class aif_lsh_request(C.Structure):
    _fields_ = [("seq_sigs", C.c_void_p), ("seq_emb", C.c_void_p), ("seq_len", C.c_int32),
                ("cand_ids", C.c_void_p), ("n_cand", C.c_int32), ("din_out", C.c_void_p),
                ("tier_out", C.c_void_p)]


class aif_user_config(C.Structure):
    _fields_ = [("dtype", C.c_int), ("d_raw", C.c_int32), ("d", C.c_int32), ("max_seq_len", C.c_int32),
                ("max_users", C.c_int32)]


class aif_user_weights(C.Structure):
    _fields_ = [("w_profile", C.c_void_p), ("w_seq", C.c_void_p), ("w_ffn", C.c_void_p), ("b_ffn", C.c_void_p)]


class aif_user_request(C.Structure):
    _fields_ = [("profile", C.c_void_p), ("seq", C.c_void_p), ("seq_len", C.c_int32),
                ("user_vec_out", C.c_void_p), ("seq_out", C.c_void_p)]


_lib = None


def load():
    """Load libaif.so (built by ``python -m paper_2511_12934_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2511_12934_amd.build` "
                           "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    vp = C.c_void_p
    lib.aif_score_init.restype = C.c_int
    lib.aif_score_init.argtypes = [C.POINTER(aif_config), C.POINTER(aif_weights), C.POINTER(vp)]
    lib.aif_score_request.restype = C.c_int
    lib.aif_score_request.argtypes = [vp, C.POINTER(aif_request), vp]
    lib.aif_score_batch.restype = C.c_int
    lib.aif_score_batch.argtypes = [vp, C.POINTER(aif_request), C.c_int32, vp]
    lib.aif_topk.restype = C.c_int
    lib.aif_topk.argtypes = [vp, C.POINTER(vp), C.POINTER(C.c_int32), C.c_int32, C.c_int32, vp, vp, vp]
    lib.aif_score_destroy.restype = None
    lib.aif_score_destroy.argtypes = [vp]
    lib.aif_last_error.restype = C.c_char_p
    lib.aif_last_error.argtypes = [vp]
    lib.aif_poll_device_errors.restype = C.c_int
    lib.aif_poll_device_errors.argtypes = [vp, C.POINTER(C.c_int32)]
    lib.aif_peek_features.restype = C.c_int
    lib.aif_peek_features.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32, vp]
    lib.aif_profile_begin.restype = C.c_int
    lib.aif_profile_begin.argtypes = [vp, C.c_int32]
    lib.aif_profile_begin_stages.restype = C.c_int
    lib.aif_profile_begin_stages.argtypes = [vp, C.c_int32, C.c_uint32]
    lib.aif_profile_begin_sampled.restype = C.c_int
    lib.aif_profile_begin_sampled.argtypes = [vp, C.c_int32, C.c_uint32, C.c_int32]
    lib.aif_profile_end.restype = C.c_int
    lib.aif_profile_end.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int32)]
    lib.aif_stage_kind.restype = C.c_int32
    lib.aif_stage_kind.argtypes = [vp, C.c_int32]
    lib.aif_score_topk_static.restype = C.c_int
    lib.aif_score_topk_static.argtypes = [vp, C.POINTER(aif_request), C.c_int32, vp, vp, vp]
    lib.aif_last_user_slots.restype = C.c_int32
    lib.aif_last_user_slots.argtypes = [vp]
    lib.aif_mlp_layer1_width.restype = C.c_int32
    lib.aif_mlp_layer1_width.argtypes = [vp]
    lib.aif_score_topk.restype = C.c_int
    lib.aif_score_topk.argtypes = [vp, C.POINTER(aif_request), C.c_int32, C.c_int32, vp, vp, vp]
    lib.aif_update_rows.restype = C.c_int
    lib.aif_update_rows.argtypes = [vp, vp, vp, C.c_int32, vp]
    lib.aif_swap_table.restype = C.c_int
    lib.aif_swap_table.argtypes = [vp, vp, C.c_int64]
    lib.aif_lsh_init.restype = C.c_int
    lib.aif_lsh_init.argtypes = [C.POINTER(aif_lsh_config), vp, C.POINTER(vp)]
    lib.aif_lsh_batch.restype = C.c_int
    lib.aif_lsh_batch.argtypes = [vp, C.POINTER(aif_lsh_request), C.c_int32, vp]
    lib.aif_lsh_destroy.restype = None
    lib.aif_lsh_destroy.argtypes = [vp]
    lib.aif_lsh_last_error.restype = C.c_char_p
    lib.aif_lsh_last_error.argtypes = [vp]
    lib.aif_lsh_poll_device_errors.restype = C.c_int
    lib.aif_lsh_poll_device_errors.argtypes = [vp, C.POINTER(C.c_int32)]
    lib.aif_lsh_simtier_kind.restype = C.c_int32
    lib.aif_lsh_simtier_kind.argtypes = [vp]
    lib.aif_lsh_din_kind.restype = C.c_int32
    lib.aif_lsh_din_kind.argtypes = [vp]
    lib.aif_lsh_profile_begin.restype = C.c_int
    lib.aif_lsh_profile_begin.argtypes = [vp, C.c_int32]
    lib.aif_lsh_profile_end.restype = C.c_int
    lib.aif_lsh_profile_end.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int32)]
    lib.aif_user_init.restype = C.c_int
    lib.aif_user_init.argtypes = [C.POINTER(aif_user_config), C.POINTER(aif_user_weights), C.POINTER(vp)]
    lib.aif_user_precompute.restype = C.c_int
    lib.aif_user_precompute.argtypes = [vp, C.POINTER(aif_user_request), C.c_int32, vp]
    lib.aif_user_destroy.restype = None
    lib.aif_user_destroy.argtypes = [vp]
    lib.aif_user_last_error.restype = C.c_char_p
    lib.aif_user_last_error.argtypes = [vp]
    lib.aif_user_attention_kind.restype = C.c_int32
    lib.aif_user_attention_kind.argtypes = [vp]
    lib.aif_user_profile_begin.restype = C.c_int
    lib.aif_user_profile_begin.argtypes = [vp, C.c_int32]
    lib.aif_user_profile_end.restype = C.c_int
    lib.aif_user_profile_end.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int32)]
    _lib = lib
    return lib


class AifError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"aif status {status}: {msg}")
        self.status = status


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> Optional[int]:
    import torch
    return torch.cuda.current_stream().cuda_stream or None


class Request:
    """Device tensors of one request (or mini-batch slice)."""

    def __init__(self, user_vec, seq_keys, seq_vals, cand_ids, logits_out, scores_out=None, cross_vecs=None,
                 seq_len: Optional[int] = None):
        self.user_vec, self.seq_keys, self.seq_vals = user_vec, seq_keys, seq_vals
        self.cand_ids, self.logits_out, self.scores_out, self.cross_vecs = cand_ids, logits_out, scores_out, cross_vecs
        self.seq_len = int(seq_keys.shape[0]) if seq_len is None else int(seq_len)
        self.n_cand = int(cand_ids.numel())

    def fill(self, r: aif_request):
        r.user_vec = _ptr(self.user_vec)
        r.cross_vecs = _ptr(self.cross_vecs)
        r.seq_keys = _ptr(self.seq_keys)
        r.seq_vals = _ptr(self.seq_vals)
        r.seq_len = self.seq_len
        r.cand_ids = _ptr(self.cand_ids)
        r.n_cand = self.n_cand
        r.logits_out = _ptr(self.logits_out)
        r.scores_out = _ptr(self.scores_out)


def pack_requests(reqs: Sequence[Request]):
    arr = (aif_request * max(len(reqs), 1))()
    for i, q in enumerate(reqs):
        q.fill(arr[i])
    return arr


class Context:
    """Owns one ``aif_ctx``.  Methods carry the names of the C entry points."""

    def __init__(self, *, dtype: int, table, d_user: int, d_attn: int, n_heads: int, max_seq_len: int,
                 layer_dims: Sequence[int], weights: Sequence, biases: Optional[Sequence] = None, w_q=None,
                 cross_mode: int = AIF_CROSS_HADAMARD, n_cross: int = 0, d_cross_vec: int = 0,
                 max_candidates: int, max_users: int = 1, n_items: Optional[int] = None,
                 d_item: Optional[int] = None):
        self._lib = load()
        self._h = C.c_void_p()
        nl = len(layer_dims) - 1
        dims = (C.c_int32 * (nl + 1))(*layer_dims)
        cfg = aif_config(dtype, int(table.shape[0]) if n_items is None else n_items,
                         int(table.shape[1]) if d_item is None else d_item, d_user, d_attn, n_heads, max_seq_len,
                         cross_mode, n_cross, d_cross_vec, nl, dims, max_candidates, max_users, 0)
        w_arr = (C.c_void_p * nl)(*[_ptr(w) for w in weights])
        b_arr = None
        if biases is not None:
            b_arr = (C.c_void_p * nl)(*[_ptr(b) for b in biases])
        wt = aif_weights(_ptr(table), _ptr(w_q), w_arr, b_arr)
        self._keep = (table,)                      # the table is borrowed for the life of the context
        st = self._lib.aif_score_init(C.byref(cfg), C.byref(wt), C.byref(self._h))
        if st != AIF_OK:
            self._h = C.c_void_p()
            raise AifError(st, self._lib.aif_last_error(None).decode())

    def _check(self, st: int):
        if st != AIF_OK:
            raise AifError(st, self._lib.aif_last_error(self._h).decode())

    def aif_last_error(self) -> str:
        return self._lib.aif_last_error(self._h).decode()

    def aif_score_request(self, req: Request):
        arr = pack_requests([req])
        self._check(self._lib.aif_score_request(self._h, arr, _stream()))

    def aif_score_batch(self, reqs: Sequence[Request], packed=None):
        arr = pack_requests(reqs) if packed is None else packed
        self._check(self._lib.aif_score_batch(self._h, arr, len(reqs), _stream()))

    def aif_score_topk(self, reqs: Sequence[Request], k: int, idx_out, val_out, packed=None):
        arr = pack_requests(reqs) if packed is None else packed
        self._check(self._lib.aif_score_topk(self._h, arr, len(reqs), k, _ptr(idx_out), _ptr(val_out), _stream()))

    def aif_score_topk_static(self, req: Request, k: int, idx_out=None, val_out=None):
        arr = pack_requests([req])
        self._check(self._lib.aif_score_topk_static(self._h, arr, k, _ptr(idx_out), _ptr(val_out), _stream()))

    def aif_topk(self, logits: Sequence, k: int, idx_out, val_out, n_cand: Optional[Sequence[int]] = None):
        n = len(logits)
        ptrs = (C.c_void_p * max(n, 1))(*[_ptr(t) for t in logits])
        counts = (C.c_int32 * max(n, 1))(*([int(t.numel()) for t in logits] if n_cand is None else n_cand))
        self._check(self._lib.aif_topk(self._h, ptrs, counts, n, k, _ptr(idx_out), _ptr(val_out), _stream()))

    def aif_poll_device_errors(self) -> int:
        n = C.c_int32(0)
        self._check(self._lib.aif_poll_device_errors(self._h, C.byref(n)))
        return n.value

    def aif_update_rows(self, ids, rows, n: Optional[int] = None):
        self._check(self._lib.aif_update_rows(self._h, _ptr(ids), _ptr(rows), int(ids.numel()) if n is None else n, _stream()))

    def aif_swap_table(self, new_table, n_items: Optional[int] = None):
        self._check(self._lib.aif_swap_table(self._h, _ptr(new_table), int(new_table.shape[0]) if n_items is None else n_items))
        self._keep = self._keep + (new_table,)     # the old table may still be read by enqueued work

    def aif_peek_features(self, request: int, first_row: int, n_rows: int, out_ptr: int):
        """Rows of the last batch's [e | attention | cross] matrix of one request into a host buffer."""
        self._check(self._lib.aif_peek_features(self._h, request, first_row, n_rows, out_ptr))

    def aif_profile_begin(self, max_calls: int):
        self._check(self._lib.aif_profile_begin(self._h, max_calls))

    def aif_profile_begin_stages(self, max_calls: int, stages):
        mask = 0
        for s in stages:
            mask |= 1 << STAGES.index(s)
        self._check(self._lib.aif_profile_begin_stages(self._h, max_calls, mask))

    def aif_profile_begin_sampled(self, max_calls: int, stages, every: int):
        mask = 0
        for s in stages:
            mask |= 1 << STAGES.index(s)
        self._check(self._lib.aif_profile_begin_sampled(self._h, max_calls, mask, every))

    def aif_profile_end(self):
        """{stage: (summed ms, recorded calls)}"""
        ms = (C.c_double * len(STAGES))()
        n = (C.c_int32 * len(STAGES))()
        self._check(self._lib.aif_profile_end(self._h, ms, n))
        return {s: (ms[i], n[i]) for i, s in enumerate(STAGES)}

    def aif_stage_kind(self, stage: str) -> int:
        return int(self._lib.aif_stage_kind(self._h, STAGES.index(stage)))

    def aif_last_user_slots(self) -> int:
        return int(self._lib.aif_last_user_slots(self._h))

    def aif_mlp_layer1_width(self) -> int:
        return int(self._lib.aif_mlp_layer1_width(self._h))

    def close(self):
        if self._h:
            self._lib.aif_score_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class LshRequest:
    """Device tensors of one request of the LSH path."""

    def __init__(self, seq_sigs, seq_emb, cand_ids, din_out, tier_out, seq_len: Optional[int] = None):
        self.seq_sigs, self.seq_emb, self.cand_ids, self.din_out, self.tier_out = seq_sigs, seq_emb, cand_ids, din_out, tier_out
        self.seq_len = int(seq_sigs.shape[0]) if seq_len is None else int(seq_len)
        self.n_cand = int(cand_ids.numel())

    def fill(self, r: aif_lsh_request):
        r.seq_sigs = _ptr(self.seq_sigs)
        r.seq_emb = _ptr(self.seq_emb)
        r.seq_len = self.seq_len
        r.cand_ids = _ptr(self.cand_ids)
        r.n_cand = self.n_cand
        r.din_out = _ptr(self.din_out)
        r.tier_out = _ptr(self.tier_out)


def pack_lsh_requests(reqs: Sequence[LshRequest]):
    arr = (aif_lsh_request * max(len(reqs), 1))()
    for i, q in enumerate(reqs):
        q.fill(arr[i])
    return arr


class LshContext:
    """Owns one ``aif_lsh_ctx``.  Methods carry the names of the C entry points."""

    def __init__(self, *, sig_table, d_out: int, n_tiers: int, dtype: int, max_seq_len: int, max_candidates: int,
                 max_users: int = 1):
        self._lib = load()
        self._h = C.c_void_p()
        cfg = aif_lsh_config(int(sig_table.shape[0]), 8 * int(sig_table.shape[1]), d_out, n_tiers, dtype, max_seq_len,
                             max_candidates, max_users)
        self._keep = (sig_table,)
        st = self._lib.aif_lsh_init(C.byref(cfg), _ptr(sig_table), C.byref(self._h))
        if st != AIF_OK:
            self._h = C.c_void_p()
            raise AifError(st, self._lib.aif_lsh_last_error(None).decode())

    def _check(self, st: int):
        if st != AIF_OK:
            raise AifError(st, self._lib.aif_lsh_last_error(self._h).decode())

    def aif_lsh_batch(self, reqs: Sequence[LshRequest], packed=None):
        arr = pack_lsh_requests(reqs) if packed is None else packed
        self._check(self._lib.aif_lsh_batch(self._h, arr, len(reqs), _stream()))

    def aif_lsh_poll_device_errors(self) -> int:
        n = C.c_int32(0)
        self._check(self._lib.aif_lsh_poll_device_errors(self._h, C.byref(n)))
        return n.value

    def aif_lsh_simtier_kind(self) -> int:
        return int(self._lib.aif_lsh_simtier_kind(self._h))

    def aif_lsh_din_kind(self) -> int:
        return int(self._lib.aif_lsh_din_kind(self._h))

    def aif_lsh_profile_begin(self, max_calls: int):
        self._check(self._lib.aif_lsh_profile_begin(self._h, max_calls))

    def aif_lsh_profile_end(self):
        ms = (C.c_double * len(LSH_STAGES))()
        n = (C.c_int32 * len(LSH_STAGES))()
        self._check(self._lib.aif_lsh_profile_end(self._h, ms, n))
        return {s: (ms[i], n[i]) for i, s in enumerate(LSH_STAGES)}

    def close(self):
        if self._h:
            self._lib.aif_lsh_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class UserRequest:
    """Device tensors of one user of the user-side network (include/aif_user.h)."""

    def __init__(self, profile, seq, user_vec_out, seq_out, seq_len: Optional[int] = None):
        self.profile, self.seq, self.user_vec_out, self.seq_out = profile, seq, user_vec_out, seq_out
        self.seq_len = int(seq.shape[0]) if seq_len is None else int(seq_len)

    def fill(self, r: aif_user_request):
        r.profile = _ptr(self.profile)
        r.seq = _ptr(self.seq)
        r.seq_len = self.seq_len
        r.user_vec_out = _ptr(self.user_vec_out)
        r.seq_out = _ptr(self.seq_out)


def pack_user_requests(reqs: Sequence[UserRequest]):
    arr = (aif_user_request * max(len(reqs), 1))()
    for i, q in enumerate(reqs):
        q.fill(arr[i])
    return arr


class UserContext:
    """Owns one ``aif_user_ctx``.  Methods carry the names of the C entry points."""

    def __init__(self, *, dtype: int, d_raw: int, d: int, w_profile, w_seq, w_ffn, b_ffn=None, max_seq_len: int,
                 max_users: int = 1):
        self._lib = load()
        self._h = C.c_void_p()
        cfg = aif_user_config(dtype, d_raw, d, max_seq_len, max_users)
        wts = aif_user_weights(_ptr(w_profile), _ptr(w_seq), _ptr(w_ffn), _ptr(b_ffn))
        st = self._lib.aif_user_init(C.byref(cfg), C.byref(wts), C.byref(self._h))
        if st != AIF_OK:
            self._h = C.c_void_p()
            raise AifError(st, self._lib.aif_user_last_error(None).decode())

    def _check(self, st: int):
        if st != AIF_OK:
            raise AifError(st, self._lib.aif_user_last_error(self._h).decode())

    def aif_user_precompute(self, reqs: Sequence[UserRequest], packed=None, stream: Optional[int] = None):
        arr = pack_user_requests(reqs) if packed is None else packed
        self._check(self._lib.aif_user_precompute(self._h, arr, len(reqs), _stream() if stream is None else stream))

    def aif_user_attention_kind(self) -> int:
        return int(self._lib.aif_user_attention_kind(self._h))

    def aif_user_profile_begin(self, max_calls: int):
        self._check(self._lib.aif_user_profile_begin(self._h, max_calls))

    def aif_user_profile_end(self):
        ms = (C.c_double * len(USER_STAGES))()
        n = (C.c_int32 * len(USER_STAGES))()
        self._check(self._lib.aif_user_profile_end(self._h, ms, n))
        return {s: (ms[i], n[i]) for i, s in enumerate(USER_STAGES)}

    def close(self):
        if self._h:
            self._lib.aif_user_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
