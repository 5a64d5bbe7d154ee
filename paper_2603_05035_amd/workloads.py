"""Seeded synthetic inputs shaped like the paper's workloads.

Holds input generation only (hidden states H, weights W, workload shapes);
none of the method's arithmetic lives here, so both the GPU tests and the CPU
oracle can draw identical inputs from it.

The paper evaluates on Llama-2-7B hidden states and weights (Section 4.1,
Appendix A: d = 4096, each of Q/K/V/O is 4096 x 4096).  Those are not
available offline; the stand-ins keep the shapes (d = 4096, fused QKV width
p = 12288) and use N(0,1) activations with a few high-magnitude "outlier"
channels, and N(0, 0.02^2) weights.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

KIND_ORTHOGONAL = 0
KIND_GAUSSIAN = 1
KIND_CONDITIONED = 2
KIND_STRUCTURED = 3
KIND_BLOCK_ORTHOGONAL = 4
KIND_REFLECTOR_PRODUCT = 5


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str            # "f32" or "bf16"
    n_data: int           # plaintext rows of H
    k_shield: int         # shield rows appended
    d: int
    p: int
    kind: int
    outlier_channels: int
    seed: int
    shield_scale: float = 10.0
    cond_max: float = 1e3

    @property
    def n(self) -> int:
        return self.n_data + self.k_shield


WORKLOADS = {
    # tiny fp32 case a CPU reference finishes instantly
    "tiny_f32": Workload("tiny_f32", "f32", 16, 2, 64, 192, KIND_ORTHOGONAL, 0, 0xC0),
    # Llama-2-7B-shaped single layer, fp32, non-orthogonal Gaussian A with kappa rejection
    "llama7b_f32_gaussian": Workload("llama7b_f32_gaussian", "f32", 512, 0, 4096, 12288,
                                     KIND_GAUSSIAN, 8, 0xC1),
    # bf16 prefill, orthogonal A + 5% shields (102 rows on 2048 -> n = 2150)
    "llama7b_bf16_prefill": Workload("llama7b_bf16_prefill", "bf16", 2048, 102, 4096, 12288,
                                     KIND_ORTHOGONAL, 8, 0xC2),
    # one layer of the 32-layer sweep: 8 sequences x 512 tokens; even layers
    "sweep_bf16_orth": Workload("sweep_bf16_orth", "bf16", 4096, 205, 4096, 12288,
                                KIND_ORTHOGONAL, 8, 0xC3),
    # ... odd layers: well-conditioned non-orthogonal A, no shields
    "sweep_bf16_cond": Workload("sweep_bf16_cond", "bf16", 4096, 0, 4096, 12288,
                                KIND_CONDITIONED, 8, 0xC3),
    # decode-shaped: 64 tokens per step, 4 shields
    "decode_bf16": Workload("decode_bf16", "bf16", 64, 4, 4096, 12288, KIND_ORTHOGONAL, 8, 0xC4),
    # the attention output projection of the same layer shape (W_o is 4096 x 4096): the same chain with
    # p = d and a fresh A of its own (the method offloads every linear projection Q, K, V and O)
    "llama7b_bf16_oproj": Workload("llama7b_bf16_oproj", "bf16", 2048, 102, 4096, 4096,
                                   KIND_ORTHOGONAL, 8, 0xC5),
    # beyond Q/K/V/O: the MLP projections of the same model (the paper's Conclusion lists them as the next
    # layers to offload; Llama-2-7B: hidden 4096, intermediate 11008).  Gate and up share their input and
    # are fused like Q|K|V (p = 2 x 11008); down maps 11008 back to 4096.
    "llama7b_bf16_mlp_gate_up": Workload("llama7b_bf16_mlp_gate_up", "bf16", 2048, 102, 4096, 22016,
                                         KIND_STRUCTURED, 8, 0xC9),
    "llama7b_bf16_mlp_down": Workload("llama7b_bf16_mlp_down", "bf16", 2048, 102, 11008, 4096,
                                      KIND_STRUCTURED, 8, 0xCA),
    # the prefill batch again with the structured orthogonal A (permutations, sign flips and block
    # Walsh-Hadamard rounds: nothing to factorise, mix and unmix in O(n log n) per column)
    "llama7b_bf16_prefill_structured": Workload("llama7b_bf16_prefill_structured", "bf16", 2048, 102, 4096, 12288,
                                                KIND_STRUCTURED, 8, 0xC6),
    # ... the 4096 + 205 row layer of the sweep and the decode-shaped batch, same kind
    "sweep_bf16_structured": Workload("sweep_bf16_structured", "bf16", 4096, 205, 4096, 12288,
                                      KIND_STRUCTURED, 8, 0xC7),
    # ... and with the block-diagonal orthogonal A (dense orthogonal mixing inside blocks of 256 mixed rows)
    "llama7b_bf16_prefill_blocks": Workload("llama7b_bf16_prefill_blocks", "bf16", 2048, 102, 4096, 12288,
                                            KIND_BLOCK_ORTHOGONAL, 8, 0xCB),
    "sweep_bf16_blocks": Workload("sweep_bf16_blocks", "bf16", 4096, 205, 4096, 12288,
                                  KIND_BLOCK_ORTHOGONAL, 8, 0xCC),
    # ... and with the dense Haar-distributed A built as a product of directly drawn reflectors (nothing factorised)
    "llama7b_bf16_prefill_reflectors": Workload("llama7b_bf16_prefill_reflectors", "bf16", 2048, 102, 4096, 12288,
                                                KIND_REFLECTOR_PRODUCT, 8, 0xCD),
    "sweep_bf16_reflectors": Workload("sweep_bf16_reflectors", "bf16", 4096, 205, 4096, 12288,
                                      KIND_REFLECTOR_PRODUCT, 8, 0xCE),
    "decode_bf16_structured": Workload("decode_bf16_structured", "bf16", 64, 4, 4096, 12288,
                                       KIND_STRUCTURED, 8, 0xC8),
}


def make_hidden(rows: int, d: int, seed: int, outlier_channels: int = 8,
                outlier_scale: float = 20.0) -> np.ndarray:
    """rows x d float32 ~ N(0,1); `outlier_channels` distinct seeded columns are
    multiplied by `outlier_scale` (massive-activation channels of LLM hidden states)."""
    rng = np.random.default_rng([seed, 0x48])
    H = rng.standard_normal((rows, d), dtype=np.float32)
    if outlier_channels > 0:
        cols = rng.choice(d, size=min(outlier_channels, d), replace=False)
        H[:, cols] *= np.float32(outlier_scale)
    return H


def make_weight(d: int, p: int, seed: int, std: float = 0.02) -> np.ndarray:
    """d x p float32 ~ N(0, std^2) (std is a standard deviation, the usual LLM init)."""
    rng = np.random.default_rng([seed, 0x57])
    W = rng.standard_normal((d, p), dtype=np.float32)
    W *= np.float32(std)
    return W


def make_inputs(w: Workload, layer: int = 0):
    """(H, W) float32 host arrays for one batch of workload `w`."""
    H = make_hidden(w.n_data, w.d, w.seed * 1000 + layer, w.outlier_channels)
    W = make_weight(w.d, w.p, w.seed * 1000 + layer)
    return H, W
