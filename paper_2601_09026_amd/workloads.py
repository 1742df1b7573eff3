"""Seeded synthetic workloads for the layer-parallel (MGRIT) transformer ODE.

This module only *draws inputs*: shapes, seeds, distributions, and the rounding
of weight matrices to bf16-representable values for the mixed-precision
configurations.  It contains none of the method's arithmetic (no layer step,
no MGRIT logic) so that the CPU oracle and the HIP library can both be fed
from it without sharing any of the code under test.

The five named workloads mirror the benchmark configurations: model shapes
follow the paper's Table 2 families (BERT / GPT-2 / ViT: d=768 or 384, MT:
d=512), the MGRIT knobs follow its Table 3 (c_f in {2,4}, 2-3 levels, a few
iterations).  Data are synthetic stand-ins for the paper's corpora: token or
patch embeddings are i.i.d. N(0,1), every weight matrix i.i.d. N(0,0.02^2).

Weight convention: a projection computes ``y = x @ W.T + b`` with ``W`` stored
``[out_features, in_features]`` (reduction dimension contiguous).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np
import torch

ARCH_ENCODER = 0      # self-attention without mask (paper eq. for the encoder step)
ARCH_CAUSAL = 1       # decoder-only: causal self-attention
ARCH_CROSS = 2        # enc-dec decoder: causal self-attention + cross-attention

DTYPE_F32 = 0         # fp32 weights, operands and state
DTYPE_BF16 = 1        # bf16 weight matrices / matmul operands, fp32 state and vectors


@dataclass(frozen=True)
class Workload:
    name: str
    arch: int
    d_model: int
    n_heads: int
    d_ff: int
    batch: int
    seq: int
    mem_seq: int          # cross-attention memory length (0 unless arch == ARCH_CROSS)
    N: int                # number of layers (fine time steps)
    h: float              # fine step size
    cf: int
    levels: int
    iters: int
    dtype: int
    seed: int
    adjoint: bool = False
    ln_eps: float = 1e-5
    relax: int = 1        # 0 = F-relaxation, 1 = FCF-relaxation

    @property
    def tokens(self) -> int:
        return self.batch * self.seq

    def scaled(self, **kw) -> "Workload":
        """Same shape family with some fields replaced (used for reduced test cases)."""
        return replace(self, **kw)


def named_workloads() -> Dict[str, Workload]:
    """The five benchmark configurations (index i of the list = ``configs[i]``), followed by the
    deep-narrow shape of the paper's own scaling study (its "MC" example: one head of width 128,
    sequences of 2048 tokens, hundreds of layers, F-relaxation, more levels)."""
    w = [
        Workload("tiny_encoder", ARCH_ENCODER, 64, 4, 256, 2, 32, 0, 16, 1.0 / 16, 4, 2, 2,
                 DTYPE_F32, seed=0, adjoint=True),
        Workload("bert_base", ARCH_ENCODER, 768, 12, 3072, 32, 128, 0, 64, 1.0 / 64, 4, 2, 2,
                 DTYPE_BF16, seed=1),
        Workload("gpt2_small", ARCH_CAUSAL, 768, 12, 3072, 8, 512, 0, 128, 1.0 / 128, 4, 3, 2,
                 DTYPE_BF16, seed=2, adjoint=True),
        Workload("vit_small", ARCH_ENCODER, 384, 6, 1536, 64, 197, 0, 32, 1.0 / 32, 2, 2, 3,
                 DTYPE_BF16, seed=3),
        Workload("mt_encoder", ARCH_ENCODER, 512, 8, 2048, 64, 64, 0, 32, 1.0 / 32, 4, 2, 2,
                 DTYPE_BF16, seed=4),
        Workload("mt_decoder", ARCH_CROSS, 512, 8, 2048, 64, 64, 64, 32, 1.0 / 32, 4, 2, 2,
                 DTYPE_BF16, seed=5),
        Workload("mc_deep_narrow", ARCH_ENCODER, 128, 1, 128, 8, 2048, 0, 256, 1.0 / 256, 4, 3, 2,
                 DTYPE_BF16, seed=6, relax=0),
    ]
    return {x.name: x for x in w}


# Names and shapes of the per-layer parameters, in drawing order.
def param_shapes(wl: Workload) -> Dict[str, tuple]:
    d, f = wl.d_model, wl.d_ff
    shapes = {
        "ln1_g": (d,), "ln1_b": (d,),
        "Wqkv": (3 * d, d), "bqkv": (3 * d,),
        "Wo": (d, d), "bo": (d,),
        "ln2_g": (d,), "ln2_b": (d,),
        "W1": (f, d), "b1": (f,),
        "W2": (d, f), "b2": (d,),
    }
    if wl.arch == ARCH_CROSS:
        shapes.update({
            "ln3_g": (d,), "ln3_b": (d,),
            "Wq_c": (d, d), "bq_c": (d,),
            "Wkv_c": (2 * d, d), "bkv_c": (2 * d,),
            "Wo_c": (d, d), "bo_c": (d,),
        })
    return shapes


def _round_bf16(t: torch.Tensor) -> torch.Tensor:
    """Round to the nearest bf16-representable value (ties to even), keep fp32 storage."""
    return t.to(torch.bfloat16).to(torch.float32)


def layer_params(wl: Workload, layer: int, weight_std: float = 0.02) -> Dict[str, np.ndarray]:
    """Parameters of one layer as fp32 numpy arrays.

    Each layer has its own generator seeded from (seed, layer) so that layers
    can be drawn independently and lazily.  Matrices ~ N(0, weight_std^2);
    biases and LayerNorm offsets ~ N(0, weight_std^2); LayerNorm gains
    ~ 1 + N(0, weight_std^2), so that every parameter influences the result.
    In the bf16 configurations matrices are rounded to bf16-representable
    values here, before either implementation sees them.
    """
    gen = torch.Generator(device="cpu")
    gen.manual_seed(wl.seed * 1_000_003 + 7919 * (layer + 1))
    out: Dict[str, np.ndarray] = {}
    for name, shape in param_shapes(wl).items():
        t = torch.randn(shape, generator=gen, dtype=torch.float32) * weight_std
        if name.endswith("_g"):
            t = t + 1.0
        if len(shape) == 2 and wl.dtype == DTYPE_BF16:
            t = _round_bf16(t)
        out[name] = t.numpy()
    return out


def initial_state(wl: Workload) -> np.ndarray:
    """Z_0: [batch*seq, d_model] fp32, i.i.d. N(0,1) (embeddings stand-in)."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(wl.seed * 1_000_003 + 11)
    return torch.randn((wl.tokens, wl.d_model), generator=gen, dtype=torch.float32).numpy()


def terminal_adjoint(wl: Workload) -> np.ndarray:
    """lambda_N = dL/dZ_N for the loss L = <C, Z_N>, C i.i.d. N(0,1): [tokens, d] fp32."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(wl.seed * 1_000_003 + 13)
    return torch.randn((wl.tokens, wl.d_model), generator=gen, dtype=torch.float32).numpy()


def cross_memory(wl: Workload) -> Optional[np.ndarray]:
    """Encoder output stand-in for the cross-attention: [batch*mem_seq, d] fp32, or None."""
    if wl.arch != ARCH_CROSS:
        return None
    gen = torch.Generator(device="cpu")
    gen.manual_seed(wl.seed * 1_000_003 + 17)
    return torch.randn((wl.batch * wl.mem_seq, wl.d_model), generator=gen,
                       dtype=torch.float32).numpy()


def select_sequences(wl: Workload, x: np.ndarray, seqs, seq_len: Optional[int] = None) -> np.ndarray:
    """Rows of a [batch*seq, d] array that belong to the listed sequences, in order."""
    s = wl.seq if seq_len is None else seq_len
    idx = np.concatenate([np.arange(b * s, (b + 1) * s) for b in seqs])
    return x[idx]


# ----------------------------------------------------------------------------
# stacked encoder-decoder system: one time axis, encoder layers first (paper section 3.1)
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class StackedWorkload:
    """An encoder and a cross-attention decoder of the same width and batch on one grid of
    enc.N + dec.N layers.  State rows: the encoder's tokens, then the decoder's.  The decoder
    workload carries the grid's step size and MGRIT knobs; dec.mem_seq == enc.seq."""
    name: str
    enc: Workload
    dec: Workload

    def __post_init__(self):
        e, d = self.enc, self.dec
        assert e.arch == ARCH_ENCODER and d.arch == ARCH_CROSS
        assert (e.d_model, e.n_heads, e.d_ff, e.batch, e.dtype) == (d.d_model, d.n_heads, d.d_ff, d.batch, d.dtype)
        assert d.mem_seq == e.seq

    @property
    def N(self) -> int:
        return self.enc.N + self.dec.N

    @property
    def n_enc(self) -> int:
        return self.enc.N

    @property
    def tokens(self) -> int:
        return self.enc.tokens + self.dec.tokens


def stacked_workloads() -> Dict[str, StackedWorkload]:
    """The machine-translation configuration as one grid: 32 encoder + 32 decoder layers."""
    w = named_workloads()
    dec = w["mt_decoder"].scaled(h=1.0 / 64)
    return {"mt_stacked": StackedWorkload("mt_stacked", w["mt_encoder"].scaled(h=1.0 / 64), dec)}


def stacked_layer_params(sw: StackedWorkload, layer: int, weight_std: float = 0.02) -> Dict[str, np.ndarray]:
    """Layer `layer` of the stacked grid: an encoder layer below n_enc, a decoder layer from there."""
    if layer < sw.n_enc:
        return layer_params(sw.enc, layer, weight_std)
    return layer_params(sw.dec, layer - sw.n_enc, weight_std)


def stacked_initial_state(sw: StackedWorkload) -> np.ndarray:
    """[X_0 ; Y_0]: source embeddings, then target embeddings."""
    return np.concatenate([initial_state(sw.enc), initial_state(sw.dec)])


def stacked_terminal_adjoint(sw: StackedWorkload) -> np.ndarray:
    """lambda_N for L = <C, Z_N> over both parts of the final state."""
    return np.concatenate([terminal_adjoint(sw.enc), terminal_adjoint(sw.dec)])
