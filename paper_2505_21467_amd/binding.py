"""Thin ctypes binding of libfreecache.so: same names as include/freecache.h.

Argument marshalling only: torch tensors are used for device memory and streams,
every step of the path runs in the library's HIP kernels.  There is no fallback:
if the shared library is missing, loading raises.
"""
import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libfreecache.so")

FC_OK, FC_ERR_INVALID_ARG, FC_ERR_BOUNDS, FC_ERR_UNSUPPORTED, FC_ERR_OOM, FC_ERR_WORKSPACE, FC_ERR_HIP = range(7)
FC_F32, FC_BF16 = 0, 1
DTYPE_CODE = {"f32": FC_F32, "bf16": FC_BF16, torch.float32: FC_F32, torch.bfloat16: FC_BF16}
TORCH_DTYPE = {FC_F32: torch.float32, FC_BF16: torch.bfloat16}

EXPORTS = (
    "fc_last_error", "fc_tuning_set", "fc_attention_plan", "fc_cache_storage_bytes", "fc_cache_alloc", "fc_cache_free", "fc_cache_ptrs",
    "fc_cache_write_rows", "fc_cache_read_rows", "fc_window", "fc_qkv_project_scatter",
    "fc_workspace_bytes", "fc_active_attention", "fc_refresh",
    "fc_active_attention_static_max_bytes", "fc_active_attention_static",
    "fc_rmsnorm", "fc_linear_workspace_bytes", "fc_linear_residual", "fc_ffn_gate_up",
    "fc_full_layer_workspace_bytes", "fc_full_layer_step",
    "fc_lm_head_workspace_bytes", "fc_lm_head_argmax", "fc_unmask_select", "fc_gather_rows",
    "fc_guided_accept_workspace_bytes", "fc_guided_accept", "fc_kv_similarity",
)


class fc_config(ctypes.Structure):
    _fields_ = [
        ("n_layers", ctypes.c_int32), ("batch", ctypes.c_int32), ("hidden", ctypes.c_int32),
        ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("max_seq", ctypes.c_int32), ("dtype", ctypes.c_int32), ("rope_base", ctypes.c_float),
        ("softmax_scale", ctypes.c_float),
    ]


class fc_layer_weights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("norm1", "w_qkv", "b_qkv", "w_out", "norm2", "w_gate", "w_up", "w_down")] + [
        ("d_ff", ctypes.c_int32), ("eps", ctypes.c_float)]


class FreeCacheError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("fc_status %d: %s" % (status, text))
        self.status = status


_lib = None


def lib():
    """Load libfreecache.so (built by paper_2505_21467_amd.build); raises if it is absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                "%s not found: run `python -m paper_2505_21467_amd.build` first" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        cfgp = ctypes.POINTER(fc_config)
        L.fc_last_error.restype = ctypes.c_char_p
        L.fc_last_error.argtypes = []
        L.fc_tuning_set.restype = ctypes.c_int
        L.fc_tuning_set.argtypes = [ctypes.c_char_p, ctypes.c_char_p]
        L.fc_attention_plan.restype = ctypes.c_int
        L.fc_attention_plan.argtypes = [cfgp, i32, i32, ctypes.POINTER(i32)]
        L.fc_cache_storage_bytes.restype = sz
        L.fc_cache_storage_bytes.argtypes = [cfgp]
        L.fc_cache_alloc.restype = ctypes.c_int
        L.fc_cache_alloc.argtypes = [cfgp, vp, vp, ctypes.POINTER(vp)]
        L.fc_cache_free.restype = ctypes.c_int
        L.fc_cache_free.argtypes = [vp]
        L.fc_cache_ptrs.restype = ctypes.c_int
        L.fc_cache_ptrs.argtypes = [vp, i32, ctypes.POINTER(vp), ctypes.POINTER(vp)]
        for name in ("fc_cache_write_rows", "fc_cache_read_rows"):
            getattr(L, name).restype = ctypes.c_int
            getattr(L, name).argtypes = [vp, i32, vp, vp, i32, i32, vp]
        L.fc_window.restype = ctypes.c_int
        L.fc_window.argtypes = [i32] * 7 + [ctypes.POINTER(i32)] * 3
        L.fc_qkv_project_scatter.restype = ctypes.c_int
        L.fc_qkv_project_scatter.argtypes = [vp, i32, vp, vp, vp, i32, i32, vp, vp, vp]
        L.fc_workspace_bytes.restype = sz
        L.fc_workspace_bytes.argtypes = [cfgp, i32]
        L.fc_active_attention.restype = ctypes.c_int
        L.fc_active_attention.argtypes = [vp, i32, vp, i32, i32, vp, vp, vp, sz, vp]
        L.fc_active_attention_static_max_bytes.restype = sz
        L.fc_active_attention_static_max_bytes.argtypes = []
        L.fc_active_attention_static.restype = ctypes.c_int
        L.fc_active_attention_static.argtypes = [vp, i32, vp, i32, i32, vp, vp, vp]
        L.fc_refresh.restype = ctypes.c_int
        L.fc_refresh.argtypes = [vp, i32, vp, vp, vp, i32, i32, i32, vp, vp, vp, sz, vp]
        L.fc_rmsnorm.restype = ctypes.c_int
        L.fc_rmsnorm.argtypes = [i32, vp, vp, ctypes.c_float, i32, i32, vp, vp]
        L.fc_linear_workspace_bytes.restype = sz
        L.fc_linear_workspace_bytes.argtypes = [i32, i32, i32, i32]
        L.fc_linear_residual.restype = ctypes.c_int
        L.fc_linear_residual.argtypes = [i32, vp, vp, vp, i32, i32, i32, vp, vp, sz, vp]
        L.fc_ffn_gate_up.restype = ctypes.c_int
        L.fc_ffn_gate_up.argtypes = [i32, vp, vp, vp, i32, i32, i32, vp, vp, sz, vp]
        L.fc_full_layer_workspace_bytes.restype = sz
        L.fc_full_layer_workspace_bytes.argtypes = [cfgp, i32, i32]
        L.fc_full_layer_step.restype = ctypes.c_int
        L.fc_full_layer_step.argtypes = [vp, i32, ctypes.POINTER(fc_layer_weights), vp, i32, i32, vp, i32, vp,
                                         vp, sz, vp]
        L.fc_lm_head_workspace_bytes.restype = sz
        L.fc_lm_head_workspace_bytes.argtypes = [i32, i32, i32, i32]
        L.fc_lm_head_argmax.restype = ctypes.c_int
        L.fc_lm_head_argmax.argtypes = [i32, vp, vp, i32, i32, i32, vp, vp, vp, sz, vp]
        L.fc_unmask_select.restype = ctypes.c_int
        L.fc_unmask_select.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, vp, i32, vp, vp, vp]
        L.fc_gather_rows.restype = ctypes.c_int
        L.fc_gather_rows.argtypes = [i32, vp, i32, i32, vp, i32, vp, vp]
        L.fc_guided_accept_workspace_bytes.restype = sz
        L.fc_guided_accept_workspace_bytes.argtypes = [i32, i32, i32]
        L.fc_guided_accept.restype = ctypes.c_int
        L.fc_guided_accept.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, ctypes.c_float, i32, vp, i32, vp, vp, vp, vp,
                                       sz, vp]
        L.fc_kv_similarity.restype = ctypes.c_int
        L.fc_kv_similarity.argtypes = [vp, i32, vp, vp, i32, i32, vp, vp, vp]
        _lib = L
    return _lib


def fc_last_error() -> str:
    return lib().fc_last_error().decode()


def _check(status):
    if status != FC_OK:
        raise FreeCacheError(status, fc_last_error())


def _ptr(t):
    """Device (or raw) pointer of a tensor / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def make_config(n_layers, batch, hidden, n_q_heads, n_kv_heads, head_dim, max_seq, dtype,
                rope_base=10000.0, softmax_scale=0.0) -> fc_config:
    return fc_config(n_layers, batch, hidden, n_q_heads, n_kv_heads, head_dim, max_seq,
                     DTYPE_CODE[dtype], rope_base, softmax_scale)


def fc_tuning_set(name: str, value=None) -> None:
    """Set a tuning knob (value None restores the default)."""
    _check(lib().fc_tuning_set(name.encode(), None if value is None else str(value).encode()))


def fc_attention_plan(cfg: fc_config, A: int, kv_len: int) -> dict:
    out = (ctypes.c_int32 * 6)()
    _check(lib().fc_attention_plan(ctypes.byref(cfg), A, kv_len, out))
    return dict(zip(("kind", "splits", "keys_per_split", "row_tiles", "tiles_per_wg", "waves"), list(out)))


def fc_cache_storage_bytes(cfg: fc_config) -> int:
    return int(lib().fc_cache_storage_bytes(ctypes.byref(cfg)))


def fc_cache_alloc(cfg: fc_config, k_storage=None, v_storage=None):
    """Returns an opaque handle (int). Storage tensors, if given, are borrowed: keep them alive."""
    out = ctypes.c_void_p()
    _check(lib().fc_cache_alloc(ctypes.byref(cfg), _ptr(k_storage), _ptr(v_storage), ctypes.byref(out)))
    return out.value


def fc_cache_free(cache) -> None:
    _check(lib().fc_cache_free(cache))


def fc_cache_ptrs(cache, layer: int):
    k, v = ctypes.c_void_p(), ctypes.c_void_p()
    _check(lib().fc_cache_ptrs(cache, layer, ctypes.byref(k), ctypes.byref(v)))
    return k.value, v.value


def fc_cache_write_rows(cache, layer, k_rows, v_rows, start, rows, stream=None) -> None:
    _check(lib().fc_cache_write_rows(cache, layer, _ptr(k_rows), _ptr(v_rows), start, rows, _stream(stream)))


def fc_cache_read_rows(cache, layer, k_rows, v_rows, start, rows, stream=None) -> None:
    _check(lib().fc_cache_read_rows(cache, layer, _ptr(k_rows), _ptr(v_rows), start, rows, _stream(stream)))


def fc_window(step, P, G, Bk, steps_per_block, refresh_every=0, mode=0):
    ws, rows, ra = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    _check(lib().fc_window(step, P, G, Bk, steps_per_block, refresh_every, mode,
                           ctypes.byref(ws), ctypes.byref(rows), ctypes.byref(ra)))
    return ws.value, rows.value, ra.value


def fc_qkv_project_scatter(cache, layer, x, w_qkv, b_qkv, win_start, A, pos, q_out, stream=None) -> None:
    _check(lib().fc_qkv_project_scatter(cache, layer, _ptr(x), _ptr(w_qkv), _ptr(b_qkv), win_start, A,
                                        _ptr(pos), _ptr(q_out), _stream(stream)))


def fc_workspace_bytes(cfg: fc_config, max_rows: int) -> int:
    return int(lib().fc_workspace_bytes(ctypes.byref(cfg), max_rows))


def fc_active_attention(cache, layer, q, A, kv_len, pos, out, workspace, workspace_bytes=None,
                        stream=None) -> None:
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().fc_active_attention(cache, layer, _ptr(q), A, kv_len, _ptr(pos), _ptr(out),
                                     _ptr(workspace), workspace_bytes, _stream(stream)))


def fc_active_attention_static_max_bytes() -> int:
    return int(lib().fc_active_attention_static_max_bytes())


def fc_active_attention_static(cache, layer, q, A, kv_len, pos, out, stream=None) -> None:
    _check(lib().fc_active_attention_static(cache, layer, _ptr(q), A, kv_len, _ptr(pos), _ptr(out),
                                            _stream(stream)))


def fc_refresh(cache, layer, x, w_qkv, b_qkv, start, R, kv_len, q_scratch, out, workspace,
               workspace_bytes=None, stream=None) -> None:
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().fc_refresh(cache, layer, _ptr(x), _ptr(w_qkv), _ptr(b_qkv), start, R, kv_len,
                            _ptr(q_scratch), _ptr(out), _ptr(workspace), workspace_bytes, _stream(stream)))


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def fc_rmsnorm(dtype, x, weight, eps, rows, hidden, out, stream=None) -> None:
    _check(lib().fc_rmsnorm(DTYPE_CODE[dtype], _ptr(x), _ptr(weight), eps, rows, hidden, _ptr(out),
                            _stream(stream)))


def fc_linear_workspace_bytes(dtype, M, K, N) -> int:
    return int(lib().fc_linear_workspace_bytes(DTYPE_CODE[dtype], M, K, N))


def fc_linear_residual(dtype, x, w, residual, M, K, N, out, workspace, workspace_bytes=None,
                       stream=None) -> None:
    if workspace_bytes is None:
        workspace_bytes = _nbytes(workspace)
    _check(lib().fc_linear_residual(DTYPE_CODE[dtype], _ptr(x), _ptr(w), _ptr(residual), M, K, N, _ptr(out),
                                    _ptr(workspace), workspace_bytes, _stream(stream)))


def fc_ffn_gate_up(dtype, x, w_gate, w_up, M, K, F, out, workspace, workspace_bytes=None, stream=None) -> None:
    if workspace_bytes is None:
        workspace_bytes = _nbytes(workspace)
    _check(lib().fc_ffn_gate_up(DTYPE_CODE[dtype], _ptr(x), _ptr(w_gate), _ptr(w_up), M, K, F, _ptr(out),
                                _ptr(workspace), workspace_bytes, _stream(stream)))


def make_layer_weights(norm1, w_qkv, b_qkv, w_out, norm2, w_gate, w_up, w_down, d_ff, eps) -> fc_layer_weights:
    """Pointers only: the caller keeps the tensors alive."""
    return fc_layer_weights(_ptr(norm1), _ptr(w_qkv), _ptr(b_qkv), _ptr(w_out), _ptr(norm2), _ptr(w_gate),
                            _ptr(w_up), _ptr(w_down), d_ff, eps)


def fc_full_layer_workspace_bytes(cfg: fc_config, d_ff: int, max_rows: int) -> int:
    return int(lib().fc_full_layer_workspace_bytes(ctypes.byref(cfg), d_ff, max_rows))


def fc_full_layer_step(cache, layer, weights: fc_layer_weights, x, win_start, A, pos, kv_len, y, workspace,
                       workspace_bytes=None, stream=None) -> None:
    if workspace_bytes is None:
        workspace_bytes = _nbytes(workspace)
    _check(lib().fc_full_layer_step(cache, layer, ctypes.byref(weights), _ptr(x), win_start, A, _ptr(pos),
                                    kv_len, _ptr(y), _ptr(workspace), workspace_bytes, _stream(stream)))


def fc_lm_head_workspace_bytes(dtype, M, K, V) -> int:
    return int(lib().fc_lm_head_workspace_bytes(DTYPE_CODE[dtype], M, K, V))


def fc_lm_head_argmax(dtype, x, w_vocab, M, K, V, tok, conf, workspace, workspace_bytes=None, stream=None) -> None:
    if workspace_bytes is None:
        workspace_bytes = _nbytes(workspace)
    _check(lib().fc_lm_head_argmax(DTYPE_CODE[dtype], _ptr(x), _ptr(w_vocab), M, K, V, _ptr(tok), _ptr(conf),
                                   _ptr(workspace), workspace_bytes, _stream(stream)))


def fc_unmask_select(tok, conf, pos, win_start, B, A, n_unmask, mask_id, tokens, L, pos_next, count_next,
                     stream=None) -> None:
    _check(lib().fc_unmask_select(_ptr(tok), _ptr(conf), _ptr(pos), win_start, B, A, n_unmask, mask_id,
                                  _ptr(tokens), L, _ptr(pos_next), _ptr(count_next), _stream(stream)))


def fc_gather_rows(dtype, table, rows, width, idx, n, out, stream=None) -> None:
    _check(lib().fc_gather_rows(DTYPE_CODE[dtype], _ptr(table), rows, width, _ptr(idx), n, _ptr(out), _stream(stream)))


def fc_guided_accept_workspace_bytes(B, A, V) -> int:
    return int(lib().fc_guided_accept_workspace_bytes(B, A, V))


def fc_guided_accept(dlm, ar, pos, win_start, B, A, V, topk, tau, mask_id, tokens, L, n_accept, pos_next, count_next,
                     workspace, workspace_bytes=None, stream=None) -> None:
    if workspace_bytes is None:
        workspace_bytes = _nbytes(workspace)
    _check(lib().fc_guided_accept(_ptr(dlm), _ptr(ar), _ptr(pos), win_start, B, A, V, topk, tau, mask_id, _ptr(tokens),
                                  L, _ptr(n_accept), _ptr(pos_next), _ptr(count_next), _ptr(workspace),
                                  workspace_bytes, _stream(stream)))


def fc_kv_similarity(cache, layer, k_prev, v_prev, start, rows, sim_k, sim_v, stream=None) -> None:
    _check(lib().fc_kv_similarity(cache, layer, _ptr(k_prev), _ptr(v_prev), start, rows, _ptr(sim_k), _ptr(sim_v),
                                  _stream(stream)))
