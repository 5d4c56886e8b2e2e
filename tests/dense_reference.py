"""Brute-force uncached bidirectional attention layer, used only to pin the oracle.

Written independently of oracle/fc_oracle.c: BLAS matmuls in float64, rotary
embedding as a complex multiplication, scipy's softmax, storage rounding through
torch's own dtype casts.  There is no cache object here: every row of the
sequence is projected and every row attends to every row, which is what a
vanilla diffusion-LM layer does at each denoising step (paper, section 3.1.1).
"""
import numpy as np
import torch
from scipy.special import expit, softmax


def round_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float64))
    if dtype == "bf16":
        # torch casts float64 -> float32 -> bf16, both to nearest even; that differs from a
        # single rounding only for values within 2^-24 (relative) of a bf16 tie
        return t.to(torch.bfloat16).to(torch.float64).numpy()
    return t.to(torch.float32).to(torch.float64).numpy()


def rope_complex(x: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """x [..., S, H, Dh], pos [..., S]; pairs (i, i + Dh/2) rotate by pos * base^(-2i/Dh)."""
    dh = x.shape[-1]
    half = dh // 2
    freqs = base ** (-np.arange(half, dtype=np.float64) * 2.0 / dh)
    ang = pos[..., None, None].astype(np.float64) * freqs
    z = (x[..., :half] + 1j * x[..., half:]) * np.exp(1j * ang)
    return np.concatenate([z.real, z.imag], axis=-1)


def dense_layer(X, W, bias, Hq, Hkv, Dh, base, dtype, scale=None, pos=None):
    """X [B,S,d] -> (Q [B,Hq,S,Dh], K [B,Hkv,S,Dh], V [B,Hkv,S,Dh], O [B,S,Hq*Dh]) as float64."""
    X = np.asarray(X, np.float64)
    W = np.asarray(W, np.float64)
    B, S, _ = X.shape
    Y = X @ W.T
    if bias is not None:
        Y = Y + np.asarray(bias, np.float64)
    q = Y[..., : Hq * Dh].reshape(B, S, Hq, Dh)
    k = Y[..., Hq * Dh: (Hq + Hkv) * Dh].reshape(B, S, Hkv, Dh)
    v = Y[..., (Hq + Hkv) * Dh:].reshape(B, S, Hkv, Dh)
    if pos is None:
        pos = np.tile(np.arange(S), (B, 1))
    q = round_storage(rope_complex(q, pos, base), dtype)
    k = round_storage(rope_complex(k, pos, base), dtype)
    v = round_storage(v, dtype)
    g = Hq // Hkv
    k_rep = np.repeat(k, g, axis=2)
    v_rep = np.repeat(v, g, axis=2)
    if scale is None:
        scale = 1.0 / np.sqrt(Dh)
    s = np.einsum("bshd,bthd->bhst", q, k_rep) * scale
    p = softmax(s, axis=-1)
    o = np.einsum("bhst,bthd->bshd", p, v_rep)
    O = round_storage(o.reshape(B, S, Hq * Dh), dtype)
    return (q.transpose(0, 2, 1, 3).copy(), k.transpose(0, 2, 1, 3).copy(),
            v.transpose(0, 2, 1, 3).copy(), O)


def rmsnorm_np(x, w, eps):
    x = np.asarray(x, np.float64)
    return x / np.sqrt(np.mean(np.square(x), axis=-1, keepdims=True) + eps) * np.asarray(w, np.float64)


def dense_full_layer(X, wts, Hq, Hkv, Dh, base, dtype, eps, pos=None):
    """Uncached pre-normalised transformer layer over all rows of X [B,S,d]: RMSNorm, bidirectional
    attention (dense_layer), output projection + residual, RMSNorm, SiLU-gated feed-forward network +
    residual (Table 1 of the paper lists these modules).  wts: dict of float arrays norm1, w_qkv,
    b_qkv (or None), w_out, norm2, w_gate, w_up, w_down.  Returns (X2, Y, K, V) as float64; every
    tensor handed from one module to the next is rounded to the storage dtype."""
    f = lambda a: np.asarray(a, np.float64)
    X = f(X)
    h1 = round_storage(rmsnorm_np(X, wts["norm1"], eps), dtype)
    _, k, v, O = dense_layer(h1, wts["w_qkv"], wts.get("b_qkv"), Hq, Hkv, Dh, base, dtype, pos=pos)
    X2 = round_storage(X + O @ f(wts["w_out"]).T, dtype)
    h2 = round_storage(rmsnorm_np(X2, wts["norm2"], eps), dtype)
    g = h2 @ f(wts["w_gate"]).T
    u = h2 @ f(wts["w_up"]).T
    act = round_storage(g * expit(g) * u, dtype)
    Y = round_storage(X2 + act @ f(wts["w_down"]).T, dtype)
    return X2, Y, k, v
