"""Seeded synthetic inputs for one GPT pipeline stage.

This module only *describes* workloads (shapes, value distributions) and draws
random tensors for them.  It contains none of the layer arithmetic: the CPU
oracle and the HIP library both receive the buffers produced here and neither
generates inputs of its own.

The paper (MegaFBD section 4.1 "forward and backward phases", MegaDPP
section 5.2 "a task = one model chunk on one micro-batch") names no dataset
for the stage computation, so every workload is dense Gaussian data of the
shape of a GPT stage:  weights N(0, w_std), output projections optionally
N(0, out_std), biases 0 (or N(0, bias_std) in tests that exercise the bias
paths), LayerNorm gamma = 1 and beta = 0 (optionally jittered), activations x
and upstream gradients dy N(0, 1).

Random numbers come from numpy's counter-based Philox generator keyed by
(seed, stream id), one stream per (tensor, layer, micro-batch), so any tensor
can be regenerated on its own and in any order.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Tuple

import numpy as np

# Per-layer tensor order of the flat parameter buffer (and of the fp32 gradient
# buffer).  The C header declares the same order as the GPTS_* tensor ids.
TENSOR_NAMES: Tuple[str, ...] = (
    "ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
    "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2",
)


@dataclass(frozen=True)
class StageShape:
    """Shape and input recipe of one stage workload."""
    name: str
    n_layers: int
    hidden: int          # H
    n_heads: int         # a (heads held by this GPU)
    head_dim: int        # d ; attention width P = a*d may differ from H
    ffn: int             # F
    seq: int             # S
    batch: int           # B (micro-batch size)
    dtype: str           # "fp32" or "bf16" (storage type of activations/weights)
    n_microbatches: int = 1
    gelu: str = "tanh"   # "tanh" or "erf"
    ln_eps: float = 1e-5
    w_std: float = 0.02
    out_std: float = 0.02   # std of w_o and w_fc2
    bias_std: float = 0.0
    ln_jitter: float = 0.0  # gamma = 1 + N(0, j), beta = N(0, j)
    recompute: int = 0       # 1: backward rebuilds the LayerNorm and GeLU outputs; 2: the stash keeps
                             # only each layer's input and backward re-runs the layer's forward
    fwd_fp16: bool = False   # bf16 stage whose forward activations are kept in fp16

    @property
    def attn_width(self) -> int:
        return self.n_heads * self.head_dim

    @property
    def tokens(self) -> int:
        return self.batch * self.seq

    def with_(self, **kw) -> "StageShape":
        return replace(self, **kw)


# The five stage workloads.  Index i here is "workload i+1" in the docs.
WORKLOADS: Tuple[StageShape, ...] = (
    StageShape("tiny_fp32", n_layers=1, hidden=128, n_heads=4, head_dim=32, ffn=512,
               seq=64, batch=2, dtype="fp32"),
    StageShape("gpt_medium_bf16", n_layers=4, hidden=1024, n_heads=16, head_dim=64, ffn=4096,
               seq=1024, batch=4, dtype="bf16"),
    # 0.02/sqrt(2*layers) with layers = the stage's own 2 layers -> 0.01
    StageShape("gpt13b_bf16", n_layers=2, hidden=5120, n_heads=40, head_dim=128, ffn=20480,
               seq=2048, batch=1, dtype="bf16", out_std=0.02 / np.sqrt(2 * 2)),
    StageShape("decoupled_bf16", n_layers=4, hidden=4096, n_heads=32, head_dim=128, ffn=16384,
               seq=4096, batch=1, dtype="bf16", n_microbatches=8),
    # hidden 12288 with N(0, 0.02) weights gives attention logits of standard deviation ~5: the
    # softmax amplifies the rounding of the forward activations, so they are kept in fp16
    StageShape("tp_share_175b_bf16", n_layers=2, hidden=12288, n_heads=12, head_dim=128, ffn=6144,
               seq=2048, batch=1, dtype="bf16", fwd_fp16=True),
)


def param_shapes(s: StageShape) -> Dict[str, Tuple[int, ...]]:
    """Shape of each per-layer tensor.  Weights are stored [out, in]."""
    P, H, F = s.attn_width, s.hidden, s.ffn
    return {
        "ln1_g": (H,), "ln1_b": (H,),
        "w_qkv": (3 * P, H), "b_qkv": (3 * P,),
        "w_o": (H, P), "b_o": (H,),
        "ln2_g": (H,), "ln2_b": (H,),
        "w_fc1": (F, H), "b_fc1": (F,),
        "w_fc2": (H, F), "b_fc2": (H,),
    }


def params_per_layer(s: StageShape) -> int:
    return int(sum(int(np.prod(v)) for v in param_shapes(s).values()))


# ---------------------------------------------------------------- rounding ---
def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result is fp32
    holding exactly bf16-representable values."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """Upper 16 bits of fp32 values that are already bf16-representable."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round an array to the workload's storage type; returned as fp32."""
    a = np.asarray(a, dtype=np.float32)
    return round_to_bf16(a) if dtype == "bf16" else a


# ------------------------------------------------------------------ drawing ---
_KIND_PARAM, _KIND_X, _KIND_DY, _KIND_AUX = 1, 2, 3, 4


def _normal(seed: int, kind: int, a: int, b: int, shape, std: float) -> np.ndarray:
    stream = (kind << 48) | ((a & 0xFFFFFF) << 24) | (b & 0xFFFFFF)
    rng = np.random.Generator(np.random.Philox(key=[seed & (2**64 - 1), stream]))
    out = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        out *= np.float32(std)
    return out


def make_layer_params(s: StageShape, layer: int, seed: int = 0) -> Dict[str, np.ndarray]:
    """One layer's tensors as fp32 arrays already rounded to the storage type."""
    out: Dict[str, np.ndarray] = {}
    for tid, (name, shp) in enumerate(param_shapes(s).items()):
        if name in ("ln1_g", "ln2_g"):
            v = np.ones(shp, np.float32)
            if s.ln_jitter:
                v += _normal(seed, _KIND_PARAM, layer, tid, shp, s.ln_jitter)
        elif name in ("ln1_b", "ln2_b"):
            v = (_normal(seed, _KIND_PARAM, layer, tid, shp, s.ln_jitter)
                 if s.ln_jitter else np.zeros(shp, np.float32))
        elif name.startswith("b_"):
            v = (_normal(seed, _KIND_PARAM, layer, tid, shp, s.bias_std)
                 if s.bias_std else np.zeros(shp, np.float32))
        else:
            std = s.out_std if name in ("w_o", "w_fc2") else s.w_std
            v = _normal(seed, _KIND_PARAM, layer, tid, shp, std)
        out[name] = to_storage(v, s.dtype)
    return out


def make_params(s: StageShape, seed: int = 0) -> List[Dict[str, np.ndarray]]:
    return [make_layer_params(s, l, seed) for l in range(s.n_layers)]


def make_x(s: StageShape, seed: int = 0, microbatch: int = 0) -> np.ndarray:
    """Stage input x, [B, S, H]."""
    return to_storage(_normal(seed, _KIND_X, microbatch, 0, (s.batch, s.seq, s.hidden), 1.0), s.dtype)


def make_dy(s: StageShape, seed: int = 0, microbatch: int = 0) -> np.ndarray:
    """Upstream gradient dy, [B, S, H]."""
    return to_storage(_normal(seed, _KIND_DY, microbatch, 0, (s.batch, s.seq, s.hidden), 1.0), s.dtype)


def make_aux(seed: int, tag: int, shape, std: float = 1.0) -> np.ndarray:
    """Extra seeded Gaussian tensor for unit tests of single kernels."""
    return _normal(seed, _KIND_AUX, tag, 0, shape, std)
