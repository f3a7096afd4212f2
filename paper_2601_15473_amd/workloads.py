"""Seeded synthetic inputs for the SKLinear workloads.

This module holds NONE of the layer's arithmetic: it only draws random tensors
of the shapes and distributions of the benchmark configurations and rounds them
to the storage type, so that the HIP path and the CPU oracle can be fed the
very same numbers.  It imports neither of them.

The paper's only real workload for this layer is BERT on WikiText (Sec. 4.2);
neither the weights nor the data are available offline, and the layer's cost
does not depend on values, so dense Gaussian tensors at BERT's layer shapes
stand in for it.

Draw order for one workload (one numpy Generator seeded with ``seed``):
x, then S_0..S_{l-1}, then U_0..U_{l-1}, then b, then dY.  Normal draws are
made in fp32; the Student-t draw of the heavy-tailed workload is made in fp64
and cast.  The second argument of N(., .) is a variance:
S ~ N(0, 1/k), U ~ N(0, 1/(l k)), b ~ N(0, 0.01), x, dY ~ N(0, 1).
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    tokens: int
    d_in: int
    d_out: int
    l: int            # num_terms
    k: int            # low_rank
    dtype: str        # "f32" or "bf16": storage type of x, S, U, b, y, dY, dX
    x_dist: str = "normal"   # "normal" or "student_t3" (unit variance)
    seed: int = 0

    @property
    def R(self):
        return self.l * self.k


# The five benchmark configurations (index = configuration number).
TINY = Workload("c0_tiny_f32", 64, 256, 256, 1, 16, "f32")
BERT_BASE_FFN_UP = Workload("c1_bert_base_ffn_up", 4096, 768, 3072, 2, 64, "bf16")
BERT_BASE_PROJ = tuple(
    Workload(f"c2_bert_base_proj_k{k}", 4096, 768, 768, 2, k, "bf16")
    for k in (16, 32, 64, 128, 192))
BERT_LARGE_FFN_UP = Workload("c3_bert_large_ffn_up", 8192, 1024, 4096, 4, 128, "bf16")
BERT_LARGE_FFN_DOWN = Workload("c3_bert_large_ffn_down", 8192, 4096, 1024, 4, 128, "bf16")
LLM_MLP = Workload("c4_llm_mlp", 16384, 4096, 11008, 8, 256, "bf16", x_dist="student_t3")

ALL = (TINY, BERT_BASE_FFN_UP) + BERT_BASE_PROJ + (
    BERT_LARGE_FFN_UP, BERT_LARGE_FFN_DOWN, LLM_MLP)

# The paper's own runtime grid for this layer (Sec. 4.1, Fig. 1): square layers of
# 8192 features, l in {1, 2, 3}, k in {16 .. 512}; the text gives no batch size, so the
# token count is this repository's choice.  l = 3 makes the 1/l scale inexact in binary.
PAPER_GRID_FEATURES = 8192
PAPER_GRID_TOKENS = 4096
PAPER_GRID = tuple(
    Workload(f"grid8192_l{l}_k{k}", PAPER_GRID_TOKENS, PAPER_GRID_FEATURES, PAPER_GRID_FEATURES,
             l, k, "bf16")
    for l in (1, 2, 3) for k in (16, 32, 64, 128, 256, 512))

BY_NAME = {w.name: w for w in ALL + PAPER_GRID}


def scaled(w: Workload, **changes) -> Workload:
    """A copy of a workload with some fields replaced (e.g. fewer tokens)."""
    return replace(w, **changes)


# ---------------------------------------------------------------------------
# bf16 storage: round-to-nearest-even from fp32, kept as raw uint16 patterns.
# ---------------------------------------------------------------------------

def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns uint16 bit patterns.
    Inputs must be finite."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to fp32 exactly."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32)


@dataclass
class Tensors:
    """One workload's inputs.

    ``stored`` maps a name to the array in storage form -- fp32 values for
    "f32", uint16 bf16 bit patterns for "bf16" -- which is what goes to the GPU.
    ``value`` maps a name to the exactly equal fp32 values, which is what the
    oracle widens to fp64.  Shapes: x [T,in], S [l,in,k], U [l,k,out], b [out],
    dY [T,out]."""
    workload: Workload
    stored: dict
    value: dict

    def S_cat(self, which="stored"):
        """[in, l*k]: column i*k + j is column j of S_i (a re-layout, no arithmetic)."""
        S = getattr(self, which)["S"]
        l, d_in, k = S.shape
        return np.ascontiguousarray(np.transpose(S, (1, 0, 2)).reshape(d_in, l * k))

    def U_cat(self, which="stored"):
        """[l*k, out]: rows i*k .. i*k+k-1 are U_i (a plain reshape)."""
        U = getattr(self, which)["U"]
        l, k, d_out = U.shape
        return np.ascontiguousarray(U.reshape(l * k, d_out))


def _normal(rng, shape, var):
    a = rng.standard_normal(size=shape, dtype=np.float32)
    if var != 1.0:
        a *= np.float32(np.sqrt(var))
    return a


def _store(w: Workload, raw: dict):
    stored, value = {}, {}
    for name, a in raw.items():
        if w.dtype == "bf16":
            bits = f32_to_bf16_bits(a)
            stored[name] = bits
            value[name] = bf16_bits_to_f32(bits)
        elif w.dtype == "f32":
            stored[name] = a
            value[name] = a
        else:
            raise ValueError(w.dtype)
    return stored, value


def generate_two_sided(w: Workload) -> Tensors:
    """Inputs of the two-sided reading of the layer: ``w.l`` terms per side.  Draw order:
    x, S1 terms, U1 terms, U2 terms, S2 terms, b, dY.  Fixed sketches have variance 1/k,
    learned factors 1/(2 l k).  Shapes: S1 [l,in,k], U1 [l,k,out], U2 [l,in,k], S2 [l,out,k].
    ``A_cat``/``B_cat`` are the stage matrices of the equivalent chain of 2 l terms
    ([S1 | U2] and [U1 ; S2^T]) in storage form -- a re-layout, no arithmetic."""
    rng = np.random.default_rng(w.seed)
    T, d_in, d_out, l, k = w.tokens, w.d_in, w.d_out, w.l, w.k
    raw = {
        "x": _normal(rng, (T, d_in), 1.0),
        "S1": np.stack([_normal(rng, (d_in, k), 1.0 / k) for _ in range(l)]),
        "U1": np.stack([_normal(rng, (k, d_out), 1.0 / (2 * l * k)) for _ in range(l)]),
        "U2": np.stack([_normal(rng, (d_in, k), 1.0 / (2 * l * k)) for _ in range(l)]),
        "S2": np.stack([_normal(rng, (d_out, k), 1.0 / k) for _ in range(l)]),
        "b": _normal(rng, (d_out,), 0.01),
        "dY": _normal(rng, (T, d_out), 1.0),
    }
    stored, value = _store(w, raw)
    for d in (stored, value):
        first = np.concatenate([d["S1"], d["U2"]], axis=0)                            # [2l, in, k]
        second = np.concatenate([d["U1"], np.transpose(d["S2"], (0, 2, 1))], axis=0)  # [2l, k, out]
        d["A_cat"] = np.ascontiguousarray(np.transpose(first, (1, 0, 2)).reshape(d_in, 2 * l * k))
        d["B_cat"] = np.ascontiguousarray(second.reshape(2 * l * k, d_out))
    return Tensors(w, stored, value)


def generate(w: Workload, with_bias: bool = True) -> Tensors:
    rng = np.random.default_rng(w.seed)
    T, d_in, d_out, l, k = w.tokens, w.d_in, w.d_out, w.l, w.k
    if w.x_dist == "normal":
        x = _normal(rng, (T, d_in), 1.0)
    elif w.x_dist == "student_t3":
        # variance of Student-t with nu = 3 is nu / (nu - 2) = 3
        x = (rng.standard_t(3.0, size=(T, d_in)) / np.sqrt(3.0)).astype(np.float32)
    else:
        raise ValueError(w.x_dist)
    S = np.stack([_normal(rng, (d_in, k), 1.0 / k) for _ in range(l)])
    U = np.stack([_normal(rng, (k, d_out), 1.0 / (l * k)) for _ in range(l)])
    b = _normal(rng, (d_out,), 0.01)
    dY = _normal(rng, (T, d_out), 1.0)
    raw = {"x": x, "S": S, "U": U, "dY": dY}
    if with_bias:
        raw["b"] = b
    stored, value = _store(w, raw)
    return Tensors(w, stored, value)
