"""ctypes front end of the CPU oracle (oracle/fc_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  It never touches the GPU library and the GPU
library never touches it.

All storage arrays are numpy float32 whose values are exactly representable in
the configured storage dtype ("f32" or "bf16"); see fc_oracle.c for layouts and
for the passages of the paper each function follows.
"""
import ctypes
import os
from dataclasses import dataclass

import numpy as np

from . import build as _build

F32, BF16 = 0, 1
_DTYPES = {"f32": F32, "bf16": BF16}


class _Cfg(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32),
        ("hidden", ctypes.c_int32),
        ("n_q_heads", ctypes.c_int32),
        ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("max_seq", ctypes.c_int32),
        ("dtype", ctypes.c_int32),
        ("rope_base", ctypes.c_double),
        ("softmax_scale", ctypes.c_double),
    ]


@dataclass
class OracleConfig:
    batch: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    max_seq: int
    dtype: str = "bf16"
    rope_base: float = 10000.0
    softmax_scale: float = 0.0  # 0 => 1/sqrt(head_dim)

    @property
    def qkv_width(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    def c(self) -> _Cfg:
        return _Cfg(self.batch, self.hidden, self.n_q_heads, self.n_kv_heads, self.head_dim,
                    self.max_seq, _DTYPES[self.dtype], self.rope_base, self.softmax_scale)


_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build()
        L = ctypes.CDLL(path)
        L.fco_round_to_storage.restype = ctypes.c_double
        L.fco_round_to_storage.argtypes = [ctypes.c_double, ctypes.c_int32]
        L.fco_round_array.restype = None
        for name in ("fco_project_rope", "fco_scatter", "fco_attend", "fco_layer_step", "fco_window",
                     "fco_rmsnorm", "fco_linear_residual", "fco_ffn_gate_up", "fco_full_layer_step",
                     "fco_lm_head_argmax", "fco_unmask_select", "fco_gather_rows",
                     "fco_guided_accept", "fco_kv_similarity"):
            getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def set_threads(n: int) -> None:
    """Set the OpenMP thread count used by the oracle's outer loops."""
    os.environ["OMP_NUM_THREADS"] = str(n)
    try:
        omp = ctypes.CDLL("libgomp.so.1")
        omp.omp_set_num_threads(int(n))
    except OSError:
        pass


def get_threads() -> int:
    try:
        omp = ctypes.CDLL("libgomp.so.1")
        return int(omp.omp_get_max_threads())
    except OSError:
        return 1


def _f32(a, shape=None):
    a = np.ascontiguousarray(a, dtype=np.float32)
    if shape is not None:
        assert a.shape == tuple(shape), (a.shape, shape)
    return a


def _p(a, ctype):
    if a is None:
        return None
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _check(rc, what):
    if rc != 0:
        raise ValueError("%s failed with oracle status %d" % (what, rc))


def round_to_storage(x, dtype: str):
    """Round doubles to the storage dtype (RNE); returns float64 array."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    out = np.empty_like(x)
    lib().fco_round_array(_p(x, ctypes.c_double), _p(out, ctypes.c_double),
                          ctypes.c_int64(x.size), ctypes.c_int32(_DTYPES[dtype]))
    return out


def project_rope(cfg: OracleConfig, X, W, bias, pos, want_pre=False):
    """Steps 1-2. Returns Q [B,Hq,A,Dh], Knew, Vnew [B,A,Hkv,Dh] (+ pre [B,A,N])."""
    B, A = pos.shape
    X = _f32(X, (B, A, cfg.hidden))
    W = _f32(W, (cfg.qkv_width, cfg.hidden))
    bias = None if bias is None else _f32(bias, (cfg.qkv_width,))
    pos = np.ascontiguousarray(pos, dtype=np.int32)
    Q = np.empty((B, cfg.n_q_heads, A, cfg.head_dim), np.float32)
    Kn = np.empty((B, A, cfg.n_kv_heads, cfg.head_dim), np.float32)
    Vn = np.empty_like(Kn)
    pre = np.empty((B, A, cfg.qkv_width), np.float64) if want_pre else None
    c = cfg.c()
    rc = lib().fco_project_rope(ctypes.byref(c), ctypes.c_int32(A), _p(X, ctypes.c_float),
                                _p(W, ctypes.c_float), _p(bias, ctypes.c_float),
                                _p(pos, ctypes.c_int32), _p(Q, ctypes.c_float),
                                _p(Kn, ctypes.c_float), _p(Vn, ctypes.c_float),
                                _p(pre, ctypes.c_double))
    _check(rc, "fco_project_rope")
    return (Q, Kn, Vn, pre) if want_pre else (Q, Kn, Vn)


def scatter(cfg: OracleConfig, Knew, Vnew, pos, Kc, Vc):
    """Step 3, in place on Kc, Vc [B,Hkv,Smax,Dh]."""
    B, A = pos.shape
    assert Kc.dtype == np.float32 and Vc.dtype == np.float32
    assert Kc.flags.c_contiguous and Vc.flags.c_contiguous
    assert Kc.shape == (B, cfg.n_kv_heads, cfg.max_seq, cfg.head_dim) == Vc.shape
    Knew = _f32(Knew, (B, A, cfg.n_kv_heads, cfg.head_dim))
    Vnew = _f32(Vnew, (B, A, cfg.n_kv_heads, cfg.head_dim))
    pos = np.ascontiguousarray(pos, dtype=np.int32)
    c = cfg.c()
    rc = lib().fco_scatter(ctypes.byref(c), ctypes.c_int32(A), _p(Knew, ctypes.c_float),
                           _p(Vnew, ctypes.c_float), _p(pos, ctypes.c_int32),
                           _p(Kc, ctypes.c_float), _p(Vc, ctypes.c_float))
    _check(rc, "fco_scatter")


def attend(cfg: OracleConfig, Q, Kc, Vc, kv_len, pos=None, want_probs=False):
    """Step 4. Returns O [B,A,Hq*Dh] (+ probs [B,Hq,A,kv_len])."""
    B, Hq, A, Dh = Q.shape
    Q = _f32(Q, (cfg.batch, cfg.n_q_heads, A, cfg.head_dim))
    Kc = _f32(Kc, (B, cfg.n_kv_heads, cfg.max_seq, Dh))
    Vc = _f32(Vc, (B, cfg.n_kv_heads, cfg.max_seq, Dh))
    if pos is not None:
        pos = np.ascontiguousarray(pos, dtype=np.int32)
        assert pos.shape == (B, A)
    O = np.empty((B, A, Hq * Dh), np.float32)
    probs = np.empty((B, Hq, A, kv_len), np.float64) if want_probs else None
    c = cfg.c()
    rc = lib().fco_attend(ctypes.byref(c), ctypes.c_int32(A), _p(Q, ctypes.c_float),
                          _p(Kc, ctypes.c_float), _p(Vc, ctypes.c_float),
                          _p(pos, ctypes.c_int32), ctypes.c_int32(kv_len),
                          _p(O, ctypes.c_float), _p(probs, ctypes.c_double))
    _check(rc, "fco_attend")
    return (O, probs) if want_probs else O


def layer_step(cfg: OracleConfig, X, W, bias, pos, kv_len, Kc, Vc):
    """One cached layer-step; Kc, Vc updated in place. Returns Q, O."""
    B, A = pos.shape
    X = _f32(X, (B, A, cfg.hidden))
    W = _f32(W, (cfg.qkv_width, cfg.hidden))
    bias = None if bias is None else _f32(bias, (cfg.qkv_width,))
    pos = np.ascontiguousarray(pos, dtype=np.int32)
    assert Kc.dtype == np.float32 and Vc.dtype == np.float32
    assert Kc.flags.c_contiguous and Vc.flags.c_contiguous
    assert Kc.shape == (B, cfg.n_kv_heads, cfg.max_seq, cfg.head_dim) == Vc.shape
    Q = np.empty((B, cfg.n_q_heads, A, cfg.head_dim), np.float32)
    O = np.empty((B, A, cfg.n_q_heads * cfg.head_dim), np.float32)
    c = cfg.c()
    rc = lib().fco_layer_step(ctypes.byref(c), ctypes.c_int32(A), _p(X, ctypes.c_float),
                              _p(W, ctypes.c_float), _p(bias, ctypes.c_float),
                              _p(pos, ctypes.c_int32), ctypes.c_int32(kv_len),
                              _p(Kc, ctypes.c_float), _p(Vc, ctypes.c_float),
                              _p(Q, ctypes.c_float), _p(O, ctypes.c_float))
    _check(rc, "fco_layer_step")
    return Q, O


def refresh(cfg: OracleConfig, X, W, bias, start, kv_len, Kc, Vc):
    """Full refresh of rows [start, start+R): the same step with a wide window."""
    B, R = X.shape[0], X.shape[1]
    pos = np.tile(np.arange(start, start + R, dtype=np.int32), (B, 1))
    return layer_step(cfg, X, W, bias, pos, kv_len, Kc, Vc)


def window(step, P, G, Bk, steps_per_block, refresh_every=0, mode=0):
    """Window schedule. Returns (win_start, rows, refresh_after)."""
    ws, rows, ra = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    rc = lib().fco_window(ctypes.c_int32(step), ctypes.c_int32(P), ctypes.c_int32(G),
                          ctypes.c_int32(Bk), ctypes.c_int32(steps_per_block),
                          ctypes.c_int32(refresh_every), ctypes.c_int32(mode),
                          ctypes.byref(ws), ctypes.byref(rows), ctypes.byref(ra))
    if rc == 2:
        raise IndexError("step past the last block")
    _check(rc, "fco_window")
    return ws.value, rows.value, ra.value


# --- the rest of the layer on the window rows (Table 1: W_out, FFN W_1, FFN W_2) ---------------

class _LayerWeights(ctypes.Structure):
    _fields_ = [(n, ctypes.POINTER(ctypes.c_float)) for n in
                ("norm1", "w_qkv", "b_qkv", "w_out", "norm2", "w_gate", "w_up", "w_down")] + [
        ("d_ff", ctypes.c_int32), ("eps", ctypes.c_double)]


def rmsnorm(X, w, eps: float, dtype: str):
    """Row-wise RMS normalisation of X [..., d] with weight w [d]; float32 array of X's shape."""
    X = _f32(X)
    d = X.shape[-1]
    w = _f32(w, (d,))
    out = np.empty_like(X)
    rc = lib().fco_rmsnorm(_p(X, ctypes.c_float), _p(w, ctypes.c_float), ctypes.c_double(eps),
                           ctypes.c_int64(X.size // d), ctypes.c_int32(d),
                           ctypes.c_int32(_DTYPES[dtype]), _p(out, ctypes.c_float))
    _check(rc, "fco_rmsnorm")
    return out


def linear_residual(X, W, res, dtype: str):
    """res + X W^T for X [M, K], W [N, K], res [M, N] or None."""
    X = _f32(X)
    M, K = X.shape
    W = _f32(W)
    N = W.shape[0]
    assert W.shape == (N, K)
    res = None if res is None else _f32(res, (M, N))
    out = np.empty((M, N), np.float32)
    rc = lib().fco_linear_residual(_p(X, ctypes.c_float), _p(W, ctypes.c_float), _p(res, ctypes.c_float),
                                   ctypes.c_int64(M), ctypes.c_int32(K), ctypes.c_int32(N),
                                   ctypes.c_int32(_DTYPES[dtype]), _p(out, ctypes.c_float))
    _check(rc, "fco_linear_residual")
    return out


def ffn_gate_up(X, Wg, Wu, dtype: str):
    """silu(X Wg^T) * (X Wu^T) for X [M, K], Wg, Wu [F, K]."""
    X = _f32(X)
    M, K = X.shape
    Wg, Wu = _f32(Wg), _f32(Wu)
    F = Wg.shape[0]
    assert Wg.shape == (F, K) == Wu.shape
    out = np.empty((M, F), np.float32)
    rc = lib().fco_ffn_gate_up(_p(X, ctypes.c_float), _p(Wg, ctypes.c_float), _p(Wu, ctypes.c_float),
                               ctypes.c_int64(M), ctypes.c_int32(K), ctypes.c_int32(F),
                               ctypes.c_int32(_DTYPES[dtype]), _p(out, ctypes.c_float))
    _check(rc, "fco_ffn_gate_up")
    return out


def full_layer_step(cfg: OracleConfig, X, weights: dict, pos, kv_len, Kc, Vc, eps: float, want_x2=False):
    """One cached step of the whole layer; Kc, Vc updated in place.  weights: dict with norm1,
    w_qkv, b_qkv (or None), w_out, norm2, w_gate, w_up, w_down as float32 arrays.
    Returns Y [B, A, d] (+ X2, the residual stream after attention)."""
    B, A = pos.shape
    d, E = cfg.hidden, cfg.n_q_heads * cfg.head_dim
    X = _f32(X, (B, A, d))
    F = weights["w_gate"].shape[0]
    keep = {
        "norm1": _f32(weights["norm1"], (d,)), "w_qkv": _f32(weights["w_qkv"], (cfg.qkv_width, d)),
        "b_qkv": None if weights.get("b_qkv") is None else _f32(weights["b_qkv"], (cfg.qkv_width,)),
        "w_out": _f32(weights["w_out"], (d, E)), "norm2": _f32(weights["norm2"], (d,)),
        "w_gate": _f32(weights["w_gate"], (F, d)), "w_up": _f32(weights["w_up"], (F, d)),
        "w_down": _f32(weights["w_down"], (d, F)),
    }
    lw = _LayerWeights(*[_p(keep[n], ctypes.c_float) for n in
                         ("norm1", "w_qkv", "b_qkv", "w_out", "norm2", "w_gate", "w_up", "w_down")],
                       F, eps)
    pos = np.ascontiguousarray(pos, dtype=np.int32)
    assert Kc.dtype == np.float32 and Vc.dtype == np.float32
    assert Kc.flags.c_contiguous and Vc.flags.c_contiguous
    assert Kc.shape == (B, cfg.n_kv_heads, cfg.max_seq, cfg.head_dim) == Vc.shape
    Y = np.empty((B, A, d), np.float32)
    X2 = np.empty((B, A, d), np.float32) if want_x2 else None
    c = cfg.c()
    rc = lib().fco_full_layer_step(ctypes.byref(c), ctypes.c_int32(A), _p(X, ctypes.c_float),
                                   ctypes.byref(lw), _p(pos, ctypes.c_int32), ctypes.c_int32(kv_len),
                                   _p(Kc, ctypes.c_float), _p(Vc, ctypes.c_float),
                                   _p(Y, ctypes.c_float), _p(X2, ctypes.c_float))
    _check(rc, "fco_full_layer_step")
    return (Y, X2) if want_x2 else Y


# --- unmasking step on the window rows (section 3.1: M_t, z_t, arg-max fill of U_t) ---------------

def lm_head_argmax(X, Wv, want_logits=False):
    """Vocabulary projection of X [M, K] with Wv [V, K]: (tok int32 [M], conf float64 [M]) (+ logits)."""
    X, Wv = _f32(X), _f32(Wv)
    M, K = X.shape
    V = Wv.shape[0]
    assert Wv.shape == (V, K)
    tok = np.empty((M,), np.int32)
    conf = np.empty((M,), np.float64)
    logits = np.empty((M, V), np.float64) if want_logits else None
    rc = lib().fco_lm_head_argmax(_p(X, ctypes.c_float), _p(Wv, ctypes.c_float), ctypes.c_int64(M),
                                  ctypes.c_int32(K), ctypes.c_int32(V), _p(tok, ctypes.c_int32),
                                  _p(conf, ctypes.c_double), _p(logits, ctypes.c_double))
    _check(rc, "fco_lm_head_argmax")
    return (tok, conf, logits) if want_logits else (tok, conf)


def unmask_select(tok, conf, pos, n_unmask, mask_id, tokens):
    """One confidence-ranked unmasking step; tokens [B, L] int32 updated in place.
    Returns (pos_next [B, A] int32 padded with -1, count_next [B] int32)."""
    pos = np.ascontiguousarray(pos, dtype=np.int32)
    B, A = pos.shape
    tok = np.ascontiguousarray(tok, dtype=np.int32).reshape(B, A)
    conf = np.ascontiguousarray(conf, dtype=np.float64).reshape(B, A)
    assert tokens.dtype == np.int32 and tokens.flags.c_contiguous and tokens.shape[0] == B
    L = tokens.shape[1]
    pos_next = np.empty((B, A), np.int32)
    count = np.empty((B,), np.int32)
    rc = lib().fco_unmask_select(_p(tok, ctypes.c_int32), _p(conf, ctypes.c_double), _p(pos, ctypes.c_int32),
                                 ctypes.c_int32(B), ctypes.c_int32(A), ctypes.c_int32(n_unmask),
                                 ctypes.c_int32(mask_id), _p(tokens, ctypes.c_int32), ctypes.c_int32(L),
                                 _p(pos_next, ctypes.c_int32), _p(count, ctypes.c_int32))
    if rc == 2:
        raise IndexError("position beyond the sequence")
    _check(rc, "fco_unmask_select")
    return pos_next, count


def gather_rows(table, idx):
    """out[i] = table[idx[i]] (zeros for a negative index); table [R, d] float32, idx int32 [n]."""
    table = _f32(table)
    R, d = table.shape
    idx = np.ascontiguousarray(idx, dtype=np.int32).reshape(-1)
    out = np.empty((idx.size, d), np.float32)
    rc = lib().fco_gather_rows(_p(table, ctypes.c_float), ctypes.c_int64(R), ctypes.c_int32(d),
                               _p(idx, ctypes.c_int32), ctypes.c_int64(idx.size), _p(out, ctypes.c_float))
    if rc == 2:
        raise IndexError("row index beyond the table")
    _check(rc, "fco_gather_rows")
    return out


def guided_accept(dlm, ar, pos, topk, tau, mask_id, tokens):
    """Guided Diffusion acceptance (Algorithm 1 with Top-K match and threshold tau); tokens [B, L] int32
    updated in place.  dlm, ar: float32 logits [B, A, V].  Returns (n_accept [B], pos_next [B, A], count [B])."""
    pos = np.ascontiguousarray(pos, dtype=np.int32)
    B, A = pos.shape
    dlm, ar = _f32(dlm), _f32(ar)
    V = dlm.shape[-1]
    assert dlm.shape == (B, A, V) == ar.shape
    assert tokens.dtype == np.int32 and tokens.flags.c_contiguous and tokens.shape[0] == B
    L = tokens.shape[1]
    n_acc = np.empty((B,), np.int32)
    pos_next = np.empty((B, A), np.int32)
    count = np.empty((B,), np.int32)
    rc = lib().fco_guided_accept(_p(dlm, ctypes.c_float), _p(ar, ctypes.c_float), _p(pos, ctypes.c_int32),
                                 ctypes.c_int32(B), ctypes.c_int32(A), ctypes.c_int32(V), ctypes.c_int32(topk),
                                 ctypes.c_float(tau), ctypes.c_int32(mask_id), _p(tokens, ctypes.c_int32),
                                 ctypes.c_int32(L), _p(n_acc, ctypes.c_int32), _p(pos_next, ctypes.c_int32),
                                 _p(count, ctypes.c_int32))
    if rc == 2:
        raise IndexError("position beyond the sequence")
    _check(rc, "fco_guided_accept")
    return n_acc, pos_next, count


def kv_similarity(cfg: OracleConfig, Kc, Vc, k_prev, v_prev, start):
    """Cosine similarity of cache rows [start, start+rows) to an earlier snapshot [B, Hkv, rows, Dh].
    Returns (sim_k, sim_v), float64 [B, Hkv, rows]."""
    B, Hkv, Dh = cfg.batch, cfg.n_kv_heads, cfg.head_dim
    Kc, Vc = _f32(Kc, (B, Hkv, cfg.max_seq, Dh)), _f32(Vc, (B, Hkv, cfg.max_seq, Dh))
    k_prev, v_prev = _f32(k_prev), _f32(v_prev)
    rows = k_prev.shape[2]
    assert k_prev.shape == (B, Hkv, rows, Dh) == v_prev.shape
    sk = np.empty((B, Hkv, rows), np.float64)
    sv = np.empty((B, Hkv, rows), np.float64)
    c = cfg.c()
    rc = lib().fco_kv_similarity(ctypes.byref(c), _p(Kc, ctypes.c_float), _p(Vc, ctypes.c_float),
                                 _p(k_prev, ctypes.c_float), _p(v_prev, ctypes.c_float), ctypes.c_int32(start),
                                 ctypes.c_int32(rows), _p(sk, ctypes.c_double), _p(sv, ctypes.c_double))
    if rc == 2:
        raise IndexError("rows outside the cache")
    _check(rc, "fco_kv_similarity")
    return sk, sv
