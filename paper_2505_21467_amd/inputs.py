"""Seeded synthetic inputs shared by the tests, the bench and the smoke check.

This module holds no arithmetic of the method: it only draws random numbers on
the CPU, casts them once to the storage dtype, and names the workload shapes.
The same bits are handed to the CPU oracle (as float32 numpy arrays, exact for
both f32 and bf16 values) and to the GPU library (as torch tensors).

The shapes stand in for Dream-7B (Qwen2.5-7B geometry: hidden 3584, 28 query
heads, 4 KV heads, head_dim 128) and LLaDA-8B (hidden 4096, 32/32 heads,
head_dim 128); weights ~ N(0, 0.02), activations ~ N(0, 1).  Block sizes 32 and
64 and generation length 256 follow the paper's configuration table.
"""
import zlib
from dataclasses import dataclass, replace

import numpy as np
import torch

TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str
    batch: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    cached_len: int       # L: rows already in the cache before the window
    active: int           # A: rows of the active window
    n_layers: int = 1
    gen_len: int = 0      # G, when the workload is a block schedule
    block: int = 0        # Bk
    steps_per_block: int = 0
    refresh_every: int = 0
    rope_base: float = 10000.0
    d_ff: int = 0         # width of the feed-forward network (whole-layer workloads)
    norm_eps: float = 1e-6

    @property
    def qkv_width(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    @property
    def kv_len(self) -> int:
        """Attended length S."""
        return self.cached_len + (self.gen_len if self.gen_len else self.active)

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


# The five configurations of the measurement plan.
# d_ff: 18944 for the Dream-7B geometry (Qwen2.5-7B), 12288 for LLaDA-8B.
C1 = Workload("c1_tiny_f32", "f32", 1, 256, 4, 4, 64, 256, 32, d_ff=512)
C2 = Workload("c2_dream7b_L1024_A32", "bf16", 1, 3584, 28, 4, 128, 1024, 32, d_ff=18944)
C3 = Workload("c3_llada8b_B4_L4096_A64", "bf16", 4, 4096, 32, 32, 128, 4096, 64, d_ff=12288,
              norm_eps=1e-5)
C4 = Workload("c4_dream7b_long_L16384_A32", "bf16", 1, 3584, 28, 4, 128, 16384, 32,
              gen_len=416, block=32, steps_per_block=8, d_ff=18944)
C5 = Workload("c5_dream7b_28layers_B8_P2048_G256", "bf16", 8, 3584, 28, 4, 128, 2048, 32,
              n_layers=28, gen_len=256, block=32, steps_per_block=8, refresh_every=8, d_ff=18944)
CONFIGS = {w.name: w for w in (C1, C2, C3, C4, C5)}


def _gen(seed: int, tag: str) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed((int(seed) * 1000003 + zlib.crc32(tag.encode())) % (2 ** 63))
    return g


def normal(seed: int, tag: str, shape, std: float, dtype: str) -> torch.Tensor:
    """CPU tensor ~ N(0, std) drawn in fp32 from (seed, tag), cast once to dtype."""
    t = torch.randn(tuple(shape), generator=_gen(seed, tag), dtype=torch.float32)
    if std != 1.0:
        t = t * std
    return t.to(TORCH_DTYPE[dtype]).contiguous()


def integers(seed: int, tag: str, shape, low: int, high: int) -> torch.Tensor:
    """CPU int32 tensor uniform in [low, high)."""
    return torch.randint(low, high, tuple(shape), generator=_gen(seed, tag), dtype=torch.int32)


def as_oracle(t: torch.Tensor) -> np.ndarray:
    """The same values as a float32 numpy array (exact for f32 and bf16)."""
    if t.dtype in (torch.int32, torch.int64):
        return t.cpu().numpy().astype(np.int32)
    return t.detach().cpu().to(torch.float32).numpy()


def weights(w: Workload, seed: int, layer: int = 0) -> torch.Tensor:
    """W_qkv [N, hidden] ~ N(0, 0.02); rows = q heads | k heads | v heads."""
    return normal(seed, "w_qkv.%d" % layer, (w.qkv_width, w.hidden), 0.02, w.dtype)


def bias(w: Workload, seed: int, layer: int = 0) -> torch.Tensor:
    return normal(seed, "b_qkv.%d" % layer, (w.qkv_width,), 0.02, w.dtype)


def hidden_states(w: Workload, seed: int, rows: int, tag: str = "x") -> torch.Tensor:
    """X [B, rows, hidden] ~ N(0, 1)."""
    return normal(seed, tag, (w.batch, rows, w.hidden), 1.0, w.dtype)


def kv_fill(w: Workload, seed: int, rows: int, tag: str = "kv"):
    """Direct N(0,1) cache fill: K, V as [B, Hkv, rows, Dh] (canonical row layout)."""
    shape = (w.batch, w.n_kv_heads, rows, w.head_dim)
    return normal(seed, tag + ".k", shape, 1.0, w.dtype), normal(seed, tag + ".v", shape, 1.0, w.dtype)


def window_positions(batch: int, start: int, rows: int) -> torch.Tensor:
    """pos [B, rows] = start + a."""
    return torch.arange(start, start + rows, dtype=torch.int32).repeat(batch, 1).contiguous()


def layer_weights(w: Workload, seed: int, layer: int = 0, with_bias: bool = False, std: float = 0.02) -> dict:
    """All weights of one pre-normalised layer: matrices ~ N(0, std), norm weights ~ 1 + N(0, 0.1)."""
    e = w.n_q_heads * w.head_dim
    t = lambda name, shape: normal(seed, "%s.%d" % (name, layer), shape, std, w.dtype)
    n = lambda name: (1.0 + 0.1 * torch.randn((w.hidden,), generator=_gen(seed, "%s.%d" % (name, layer)),
                                              dtype=torch.float32)).to(TORCH_DTYPE[w.dtype]).contiguous()
    return {
        "norm1": n("norm1"), "w_qkv": t("w_qkv", (w.qkv_width, w.hidden)),
        "b_qkv": bias(w, seed, layer) if with_bias else None,
        "w_out": t("w_out", (w.hidden, e)), "norm2": n("norm2"),
        "w_gate": t("w_gate", (w.d_ff, w.hidden)), "w_up": t("w_up", (w.d_ff, w.hidden)),
        "w_down": t("w_down", (w.hidden, w.d_ff)),
    }
