"""ctypes front end of the CPU oracle (``aif_oracle.c``).

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the benchmark's
``cpu_baseline`` leg import this; the product package never does.

All array arguments are NumPy arrays: float32 for anything that is stored in
fp32 or bf16 (both widen to float32 exactly), int32 for ids.  Results come
back as float64.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "aif_oracle.c")
_SRCS = [_SRC, os.path.join(_HERE, "aif_lsh_oracle.c"), os.path.join(_HERE, "aif_bea_oracle.c"),
         os.path.join(_HERE, "aif_user_oracle.c")]
_LIB = os.path.join(_HERE, "libaif_oracle.so")

OK, EINVAL, ESHAPE, ENOMEM, ERANGE = 0, 1, 2, 3, 5
CROSS_NONE, CROSS_HADAMARD, CROSS_SEGDOT, CROSS_BEA = 0, 1, 2, 3


_LIB_SAN = os.path.join(_HERE, "libaif_oracle_san.so")


def sanitized() -> bool:
    """True when this process was asked (AIF_ORACLE_SANITIZE=1) to run the oracle's AddressSanitizer +
    UndefinedBehaviorSanitizer build; the process must then have been started with the sanitizer runtime
    preloaded (see sanitizer_env)."""
    return os.environ.get("AIF_ORACLE_SANITIZE", "") == "1"


def build(force: bool = False, sanitize: bool = False) -> str:
    """Compile the oracle with gcc -O2 (no fast-math) into a shared object; with ``sanitize`` the
    -fsanitize=address,undefined flavour (-O1, frame pointers, any finding aborts) into a second one."""
    out = _LIB_SAN if sanitize else _LIB
    stale = (not os.path.exists(out)) or os.path.getmtime(out) < max(os.path.getmtime(f) for f in _SRCS)
    if force or stale:
        flags = (["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                  "-fno-sanitize-recover=all"] if sanitize else ["-O2"])
        subprocess.check_call(["gcc", *flags, "-std=c99", "-fopenmp", "-shared", "-fPIC", "-o", out, *_SRCS, "-lm"])
    return out


def sanitizer_env(env=None) -> dict:
    """Environment for a child Python process that loads the sanitized oracle: the AddressSanitizer runtime goes
    in front of whatever is already preloaded (an instrumented shared object cannot be loaded into a process
    that started without it); leak reports are off (the interpreter itself never frees everything)."""
    e = dict(os.environ if env is None else env)
    rt = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    e["LD_PRELOAD"] = rt + (":" + e["LD_PRELOAD"] if e.get("LD_PRELOAD") else "")
    e["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    e["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    e["AIF_ORACLE_SANITIZE"] = "1"
    return e


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build(sanitize=sanitized()))
        _lib.aifo_sigmoid.restype = C.c_double
        _lib.aifo_sigmoid.argtypes = [C.c_double]
    return _lib


def _f32(a) -> Optional[np.ndarray]:
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def _p(a, ty):
    return None if a is None else a.ctypes.data_as(C.POINTER(ty))


class OracleError(RuntimeError):
    def __init__(self, code: int):
        super().__init__(f"oracle status {code}")
        self.code = code


def _check(rc: int):
    if rc != OK:
        raise OracleError(rc)


def gather(table, ids) -> np.ndarray:
    table = _f32(table)
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    out = np.empty((ids.size, table.shape[1]), dtype=np.float64)
    _check(lib().aifo_gather(_p(table, C.c_float), C.c_int64(table.shape[0]), table.shape[1],
                             _p(ids, C.c_int32), ids.size, _p(out, C.c_double)))
    return out


def update_rows(table, ids, rows, inplace: bool = False):
    """Incremental update of the index table (Sec. 3.4): returns (updated copy, number of skipped ids);
    ``inplace`` updates a C-contiguous float32 table itself."""
    t = table if inplace else np.array(table, dtype=np.float32, order="C", copy=True)
    assert t.dtype == np.float32 and t.flags.c_contiguous
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    rows = _f32(rows)
    assert rows.shape == (ids.size, t.shape[1])
    skipped = C.c_int(0)
    f = lib().aifo_update_rows
    f.restype = None
    f(_p(t, C.c_float), C.c_int64(t.shape[0]), C.c_int(t.shape[1]), _p(ids, C.c_int32), _p(rows, C.c_float),
      C.c_int(ids.size), C.byref(skipped))
    return t, skipped.value


def query(e, w_q, d_attn: int) -> np.ndarray:
    e = np.ascontiguousarray(e, dtype=np.float64)
    w_q = _f32(w_q)
    q = np.empty(d_attn, dtype=np.float64)
    lib().aifo_query(_p(e, C.c_double), _p(w_q, C.c_float), e.size, d_attn, _p(q, C.c_double))
    return q


def attention(q, K, V, n_heads: int = 1, return_weights: bool = False):
    q = np.ascontiguousarray(q, dtype=np.float64)
    K = _f32(K)
    V = _f32(V)
    L = K.shape[0]
    d_attn = q.size
    a = np.empty(d_attn, dtype=np.float64)
    p = np.empty((n_heads, L), dtype=np.float64) if return_weights else None
    lib().aifo_attention(_p(q, C.c_double), _p(K, C.c_float), _p(V, C.c_float), L, d_attn, n_heads,
                         _p(a, C.c_double), _p(p, C.c_double))
    return (a, p) if return_weights else a


def cross(mode: int, user_operand, e, n_cross: int = 0, d_c: int = 0) -> np.ndarray:
    e = np.ascontiguousarray(e, dtype=np.float64)
    uc = _f32(user_operand)
    width = lib().aifo_cross_width(mode, e.size, n_cross, d_c)
    if width < 0:
        raise OracleError(ESHAPE)
    c = np.empty(width, dtype=np.float64)
    _check(lib().aifo_cross(mode, _p(uc, C.c_float), n_cross, d_c, _p(e, C.c_double), e.size,
                            _p(c, C.c_double)))
    return c


def _cat(arrs: Sequence[Optional[np.ndarray]], shapes) -> Optional[np.ndarray]:
    if arrs is None:
        return None
    parts = []
    for a, shp in zip(arrs, shapes):
        if a is None:
            parts.append(np.zeros(int(np.prod(shp)), dtype=np.float32))
        else:
            a = _f32(a)
            assert tuple(a.shape) == tuple(shp), (a.shape, shp)
            parts.append(a.reshape(-1))
    return np.concatenate(parts) if parts else np.zeros(0, np.float32)


def mlp(x, dims: Sequence[int], weights, biases=None) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float64)
    dims_a = np.ascontiguousarray(dims, dtype=np.int32)
    nl = len(dims) - 1
    w = _cat(weights, [(dims[l + 1], dims[l]) for l in range(nl)])
    b = _cat(biases, [(dims[l + 1],) for l in range(nl)]) if biases is not None else None
    z = np.empty(dims[-1], dtype=np.float64)
    _check(lib().aifo_mlp(_p(x, C.c_double), nl, _p(dims_a, C.c_int32), _p(w, C.c_float),
                          _p(b, C.c_float), _p(z, C.c_double)))
    return z


def sigmoid(z: float) -> float:
    return float(lib().aifo_sigmoid(float(z)))


@dataclass
class Scores:
    logits: np.ndarray            # [n] float64
    scores: np.ndarray            # [n] float64, sigmoid(logit)
    attn: np.ndarray              # [n, d_attn]
    cross: np.ndarray             # [n, d_cross]


def score(*, table, ids, user_vec, seq_keys, seq_vals, dims, weights, biases=None, w_q=None,
          n_heads: int = 1, cross_mode: int = CROSS_HADAMARD, cross_vecs=None,
          n_threads: int = 1) -> Scores:
    """Steps 1-6 for the candidates ``ids`` of one request."""
    table = _f32(table)
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    user_vec = _f32(user_vec)
    K = _f32(seq_keys)
    V = _f32(seq_vals)
    w_q = _f32(w_q)
    cv = _f32(cross_vecs)
    d_item = table.shape[1]
    d_attn = K.shape[1]
    L = K.shape[0]
    assert V.shape == K.shape
    n_cross, d_c = (cv.shape if (cv is not None and cross_mode in (CROSS_SEGDOT, CROSS_BEA)) else (0, 0))
    d_cross = lib().aifo_cross_width(cross_mode, d_item, n_cross, d_c)
    if d_cross < 0:
        raise OracleError(ESHAPE)
    nl = len(dims) - 1
    dims_a = np.ascontiguousarray(dims, dtype=np.int32)
    w = _cat(weights, [(dims[l + 1], dims[l]) for l in range(nl)])
    b = _cat(biases, [(dims[l + 1],) for l in range(nl)]) if biases is not None else None
    n = ids.size
    z = np.empty(n, np.float64)
    y = np.empty(n, np.float64)
    a = np.empty((n, d_attn), np.float64)
    c = np.empty((n, max(d_cross, 0)), np.float64)
    _check(lib().aifo_score(
        _p(table, C.c_float), C.c_int64(table.shape[0]), d_item,
        _p(w_q, C.c_float), d_attn, n_heads,
        _p(user_vec, C.c_float), user_vec.size,
        cross_mode, _p(cv, C.c_float), n_cross, d_c,
        _p(K, C.c_float), _p(V, C.c_float), L,
        nl, _p(dims_a, C.c_int32), _p(w, C.c_float), _p(b, C.c_float),
        _p(ids, C.c_int32), n,
        _p(z, C.c_double), _p(y, C.c_double), _p(a, C.c_double), _p(c, C.c_double),
        n_threads))
    return Scores(z, y, a, c)


def bea_attention_weights(X, Y) -> np.ndarray:
    """Algorithm 1, steps 1 and 3: Softmax over the rows of Y of <X_r, Y_j> / sqrt(d); X [rows, d], Y [cols, d]."""
    X, Y = _f32(X), _f32(Y)
    rows, d = X.shape
    cols = Y.shape[0]
    assert Y.shape[1] == d
    out = np.empty((rows, cols), dtype=np.float64)
    f = lib().aifo_bea_attention_weights
    f.restype = C.c_int
    _check(f(_p(X, C.c_float), C.c_int(rows), _p(Y, C.c_float), C.c_int(cols), C.c_int(d), _p(out, C.c_double)))
    return out


def bea_weighted_sum(w_hat, V) -> np.ndarray:
    """Algorithm 1, step 4: v^ = w^ V; w^ [b, n], V [n, d']."""
    w_hat = np.ascontiguousarray(w_hat, dtype=np.float64)
    V = _f32(V)
    b, n = w_hat.shape
    assert V.shape[0] == n
    out = np.empty((b, V.shape[1]), dtype=np.float64)
    f = lib().aifo_bea_weighted_sum
    f.restype = None
    f(_p(w_hat, C.c_double), C.c_int(b), C.c_int(n), _p(V, C.c_float), C.c_int(V.shape[1]), _p(out, C.c_double))
    return out


# ---------------------------------------------------------------------------
# user-side asynchronous network (aif_user_oracle.c; Sec. 3.1, Eq. 1-3)
# ---------------------------------------------------------------------------
def user_project(x, W) -> np.ndarray:
    """Eq. 1: rows of x [rows, d_raw] times W^T, W [d, d_raw]."""
    x, W = _f32(x), _f32(W)
    rows, d_raw = x.shape
    d = W.shape[0]
    assert W.shape[1] == d_raw
    out = np.empty((rows, d), dtype=np.float64)
    f = lib().aifo_user_project
    f.restype = None
    f(_p(x, C.c_float), C.c_int(rows), C.c_int(d_raw), _p(W, C.c_float), C.c_int(d), _p(out, C.c_double))
    return out


def user_attend(Q, S) -> np.ndarray:
    """Attention core of Eq. 2 / Eq. 3: Softmax(Q S^T / sqrt(d)) S; Q [rows, d], S [l, d] (float64)."""
    Q = np.ascontiguousarray(Q, dtype=np.float64)
    S = np.ascontiguousarray(S, dtype=np.float64)
    rows, d = Q.shape
    l = S.shape[0]
    out = np.empty((rows, d), dtype=np.float64)
    f = lib().aifo_user_attend
    f.restype = C.c_int
    _check(f(_p(Q, C.c_double), C.c_int(rows), _p(S, C.c_double), C.c_int(l), C.c_int(d), _p(out, C.c_double)))
    return out


def user_ffn(x, W, b=None) -> np.ndarray:
    """FFN of Eq. 2 (one layer, ReLU): max(0, W x + b) per row; x [rows, d] float64."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    W, b = _f32(W), _f32(b)
    rows, d = x.shape
    y = np.empty((rows, d), dtype=np.float64)
    f = lib().aifo_user_ffn
    f.restype = None
    f(_p(x, C.c_double), C.c_int(rows), C.c_int(d), _p(W, C.c_float), _p(b, C.c_float), _p(y, C.c_double))
    return y


def user_pool(y) -> np.ndarray:
    """Pooling of Eq. 2 (mean over positions)."""
    y = np.ascontiguousarray(y, dtype=np.float64)
    rows, d = y.shape
    out = np.empty(d, dtype=np.float64)
    f = lib().aifo_user_pool
    f.restype = None
    f(_p(y, C.c_double), C.c_int(rows), C.c_int(d), _p(out, C.c_double))
    return out


def user_network(*, profile, seq, w_profile, w_seq, w_ffn, b_ffn=None):
    """Eq. 1-3 for one user: (user_vec [2 d] = [self-attention | profile-attention], seq_hat [l, d])."""
    profile, seq = _f32(profile).reshape(-1), _f32(seq)
    w_profile, w_seq, w_ffn, b_ffn = _f32(w_profile), _f32(w_seq), _f32(w_ffn), _f32(b_ffn)
    l, d_raw = seq.shape
    d = w_seq.shape[0]
    assert profile.size == d_raw and w_profile.shape == (d, d_raw) and w_seq.shape == (d, d_raw) and w_ffn.shape == (d, d)
    uv = np.empty(2 * d, dtype=np.float64)
    sh = np.empty((l, d), dtype=np.float64)
    f = lib().aifo_user_network
    f.restype = C.c_int
    _check(f(_p(profile, C.c_float), _p(seq, C.c_float), C.c_int(l), C.c_int(d_raw), C.c_int(d),
             _p(w_profile, C.c_float), _p(w_seq, C.c_float), _p(w_ffn, C.c_float), _p(b_ffn, C.c_float),
             _p(uv, C.c_double), _p(sh, C.c_double)))
    return uv, sh


def topk(z, k: int):
    z = np.ascontiguousarray(z, dtype=np.float64)
    idx = np.empty(max(k, 0), np.int32)
    val = np.empty(max(k, 0), np.float64)
    _check(lib().aifo_topk(_p(z, C.c_double), z.size, k, _p(idx, C.c_int32), _p(val, C.c_double)))
    return idx, val


# ---------------------------------------------------------------------------
# LSH behaviour modelling (aif_lsh_oracle.c; Sec. 4.3, Eq. 5-9, Table 3)
# ---------------------------------------------------------------------------
def _u8(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.uint8)


def lsh_pack_bits(bits) -> np.ndarray:
    """d' bits (0/1) -> d'/8 bytes, first bit most significant."""
    bits = _u8(bits)
    out = np.empty(bits.size // 8, dtype=np.uint8)
    lib().aifo_lsh_pack_bits(_p(bits, C.c_uint8), C.c_int(bits.size), _p(out, C.c_uint8))
    return out


def lsh_sign(M, w_hash) -> np.ndarray:
    """Eq. 5: signatures [n, d'/8] of embeddings M [n, d] under hyperplanes w_hash [d', d]."""
    M, w_hash = _f32(M), _f32(w_hash)
    n, d = M.shape
    d_bits = w_hash.shape[0]
    sig = np.empty((n, d_bits // 8), dtype=np.uint8)
    rc = lib().aifo_lsh_sign(_p(M, C.c_float), C.c_int(n), C.c_int(d), _p(w_hash, C.c_float), C.c_int(d_bits),
                             _p(sig, C.c_uint8))
    if rc:
        raise OracleError(rc)
    return sig


def lsh_equal_bits(a, b) -> int:
    """Eq. 6 numerator: number of equal bits of two signatures."""
    a, b = _u8(a), _u8(b)
    f = lib().aifo_lsh_equal_bits
    f.restype = C.c_int
    return int(f(_p(a, C.c_uint8), _p(b, C.c_uint8), C.c_int(a.size)))


def lsh_din(equal, d_bits: int, u_seq) -> np.ndarray:
    """Eq. 8 for one candidate from its equal-bit counts [L] and U~ [L, d]."""
    equal = np.ascontiguousarray(equal, dtype=np.int32)
    u_seq = _f32(u_seq)
    L, d = u_seq.shape
    a = np.empty(d, dtype=np.float64)
    lib().aifo_lsh_din(_p(equal, C.c_int32), C.c_int(L), C.c_int(d_bits), _p(u_seq, C.c_float), C.c_int(d),
                       _p(a, C.c_double))
    return a


def simtier(equal, d_bits: int, n_tiers: int) -> np.ndarray:
    """Eq. 9 for one candidate: counts per tier."""
    equal = np.ascontiguousarray(equal, dtype=np.int32)
    out = np.empty(n_tiers, dtype=np.int32)
    lib().aifo_simtier(_p(equal, C.c_int32), C.c_int(equal.size), C.c_int(d_bits), C.c_int(n_tiers),
                       _p(out, C.c_int32))
    return out


@dataclass
class LshResult:
    din: np.ndarray         # [n, d] float64
    tiers: np.ndarray       # [n, n_tiers] int32
    equal: Optional[np.ndarray]   # [n, L] int32 when asked for


def lsh_request(*, sig_table, ids, seq_sig, u_seq, n_tiers: int, want_equal: bool = False,
                n_threads: int = 1) -> LshResult:
    """One request of the LSH path: signature lookup, Eq. 7, Eq. 8 and Eq. 9 for every candidate."""
    sig_table, seq_sig, u_seq = _u8(sig_table), _u8(seq_sig), _f32(u_seq)
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    n_items, nb = sig_table.shape
    L, d = u_seq.shape
    assert seq_sig.shape == (L, nb)
    n = ids.size
    din = np.empty((n, d), dtype=np.float64)
    tiers = np.empty((n, n_tiers), dtype=np.int32)
    eq = np.empty((n, L), dtype=np.int32) if want_equal else None
    f = lib().aifo_lsh_request
    f.restype = C.c_int
    rc = f(_p(sig_table, C.c_uint8), C.c_int64(n_items), C.c_int(8 * nb), _p(ids, C.c_int32), C.c_int(n),
           _p(seq_sig, C.c_uint8), _p(u_seq, C.c_float), C.c_int(L), C.c_int(d), C.c_int(n_tiers),
           _p(din, C.c_double), _p(tiers, C.c_int32), _p(eq, C.c_int32), C.c_int(n_threads))
    if rc:
        raise OracleError(rc)
    return LshResult(din, tiers, eq)


def lsh_similarity_cost(b: float, l: float, widths: Sequence[float]) -> float:
    """Table 3: b * l * (sum of the widths entering the attention / similarity modules)."""
    w = np.ascontiguousarray(widths, dtype=np.float64)
    f = lib().aifo_lsh_similarity_cost
    f.restype = C.c_double
    return float(f(C.c_double(b), C.c_double(l), _p(w, C.c_double), C.c_int(w.size)))
