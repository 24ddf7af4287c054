"""Shapes and seeded random inputs for the synthetic DISCO workloads.

Every tensor is drawn from a counter-based generator keyed by (seed, tensor id), so a tensor's
bytes do not depend on the order in which tensors are generated.  Small models are drawn on the
host with NumPy's Philox generator; models too large for that to be practical (billions of
parameters) are drawn with PyTorch's seeded generator on the device that will hold them and are
copied to the host when the CPU oracle needs the same bytes.

The stand-in workloads mirror the model pairs of the paper's experiments section (a 13B-class
target with a 68M-class draft; a 15B-class multi-query code model with a small draft) in shape
only: matrices and embedding tables are N(0, 0.02^2) noise, norm gains are 1 and biases 0.
"""
from __future__ import annotations

import dataclasses
import zlib
from typing import Dict, List, Optional

import numpy as np
import torch

__all__ = [
    "ModelShape", "ClassifierShape", "CFG0_TARGET", "CFG0_DRAFT", "CFG1_DRAFT", "CFG2_TARGET",
    "CFG3_TARGET", "CFG3_DRAFT", "CLF_SHAPE", "weight_specs", "make_weights", "early_exit_draft",
    "make_classifier", "make_prompt", "make_tokens", "make_kv_fill", "make_force_mask",
    "scaled_shape", "bf16_round", "n_params", "make_uniforms",
]


@dataclasses.dataclass(frozen=True)
class ModelShape:
    """Decoder-only transformer shape.

    family "A": pre-LN LayerNorm, GELU MLP (w1, w2), learned position embeddings.
    family "B": RMSNorm, rotary embeddings (half-split pairing), SwiGLU MLP (wg, wu, wd).
    n_kv_heads == n_heads is multi-head attention; n_kv_heads == 1 is multi-query attention.
    """
    family: str
    n_layers: int
    d_model: int
    n_heads: int
    d_head: int
    n_kv_heads: int
    d_ff: int
    vocab: int
    max_pos: int = 4096          # rows of the learned position table (family A)
    ln_eps: float = 1e-5
    rms_eps: float = 1e-6
    rope_base: float = 10000.0

    @property
    def d_q(self) -> int:
        return self.n_heads * self.d_head

    @property
    def d_kv(self) -> int:
        return self.n_kv_heads * self.d_head

    @property
    def d_qkv(self) -> int:
        return self.d_q + 2 * self.d_kv


@dataclasses.dataclass(frozen=True)
class ClassifierShape:
    k: int = 10                  # top-k probabilities (the paper's footnote: k = 10)
    hidden: int = 64

    @property
    def n_feat(self) -> int:
        return self.k + 2        # top-k, entropy, position


CLF_SHAPE = ClassifierShape()

# tiny end-to-end pair (draft = first target layer + final LN + LM head)
CFG0_TARGET = ModelShape("A", 4, 256, 4, 64, 4, 1024, 4096, max_pos=128)
CFG0_DRAFT = dataclasses.replace(CFG0_TARGET, n_layers=1)
# 68M-class draft;  13B-class target
CFG1_DRAFT = ModelShape("B", 2, 768, 12, 64, 12, 3072, 32000)
CFG2_TARGET = ModelShape("B", 40, 5120, 40, 128, 40, 13824, 32000)
# multi-query code-model pair
CFG3_TARGET = ModelShape("A", 40, 6144, 48, 128, 1, 24576, 49152, max_pos=4096)
CFG3_DRAFT = ModelShape("A", 12, 768, 12, 64, 1, 3072, 49152, max_pos=4096)


def scaled_shape(shape: ModelShape, **kw) -> ModelShape:
    """A reduced copy of a shape (fewer layers, smaller vocab ...) for parity tests."""
    return dataclasses.replace(shape, **kw)


def weight_specs(shape: ModelShape) -> List[tuple]:
    """[(name, shape tuple, kind)] in a fixed order; kind in {"matrix", "gain", "bias"}."""
    d, s = shape.d_model, []
    s.append(("tok_emb", (shape.vocab, d), "matrix"))
    if shape.family == "A":
        s.append(("pos_emb", (shape.max_pos, d), "matrix"))
    for l in range(shape.n_layers):
        p = f"l{l}."
        s.append((p + "norm1_g", (d,), "gain"))
        if shape.family == "A":
            s.append((p + "norm1_b", (d,), "bias"))
        s.append((p + "wqkv", (shape.d_qkv, d), "matrix"))
        s.append((p + "wo", (d, shape.d_q), "matrix"))
        s.append((p + "norm2_g", (d,), "gain"))
        if shape.family == "A":
            s.append((p + "norm2_b", (d,), "bias"))
            s.append((p + "w1", (shape.d_ff, d), "matrix"))
            s.append((p + "w2", (d, shape.d_ff), "matrix"))
        else:
            s.append((p + "wg", (shape.d_ff, d), "matrix"))
            s.append((p + "wu", (shape.d_ff, d), "matrix"))
            s.append((p + "wd", (d, shape.d_ff), "matrix"))
    s.append(("normf_g", (d,), "gain"))
    if shape.family == "A":
        s.append(("normf_b", (d,), "bias"))
    s.append(("wlm", (shape.vocab, d), "matrix"))
    return s


def n_params(shape: ModelShape) -> int:
    return sum(int(np.prod(sh)) for _, sh, _ in weight_specs(shape))


def _tid(name: str) -> int:
    return zlib.crc32(name.encode())


def _normal_host(seed: int, name: str, n: int) -> torch.Tensor:
    g = np.random.Generator(np.random.Philox(key=[seed & 0xFFFFFFFF, _tid(name)]))
    return torch.from_numpy(g.standard_normal(n, dtype=np.float32))


def _normal_device(seed: int, name: str, n: int, device) -> torch.Tensor:
    g = torch.Generator(device=device)
    g.manual_seed(((seed & 0xFFFFFFFF) << 32) | _tid(name))
    return torch.randn(n, generator=g, device=device, dtype=torch.float32)


def bf16_round(x: torch.Tensor) -> torch.Tensor:
    """Round-to-nearest-even to bfloat16 and back to the input dtype."""
    return x.to(torch.bfloat16).to(x.dtype)


def make_weights(shape: ModelShape, seed: int, dtype: str = "bf16", device="cpu",
                 sigma: float = 0.02, gain_jitter: float = 0.0) -> Dict[str, torch.Tensor]:
    """Matrices/tables ~ N(0, sigma^2) stored as bf16 (dtype="bf16") or fp32 (dtype="f32").

    Norm gains are 1 and biases 0 (fp32) unless gain_jitter > 0, which adds N(0, gain_jitter^2)
    to both so that tests can tell a dropped gain or bias from a present one.
    """
    dev = torch.device(device)
    draw = _normal_host if dev.type == "cpu" else (lambda s, n_, c: _normal_device(s, n_, c, dev))
    out: Dict[str, torch.Tensor] = {}
    for name, sh, kind in weight_specs(shape):
        n = int(np.prod(sh))
        if kind == "matrix":
            w = draw(seed, name, n).mul_(sigma).view(*sh)
            out[name] = w.to(torch.bfloat16) if dtype == "bf16" else w.to(dev)
            if dtype == "bf16":
                out[name] = out[name].to(dev)
        else:
            base = torch.ones(n) if kind == "gain" else torch.zeros(n)
            if gain_jitter > 0.0:
                base = base + _normal_host(seed, name, n) * gain_jitter
            out[name] = base.to(torch.float32).to(dev)
    return out


def early_exit_draft(target_w: Dict[str, torch.Tensor], n_layers: int = 1) -> Dict[str, torch.Tensor]:
    """Draft = the target's first n_layers layers + its final norm + its LM head (shared tensors)."""
    keep = {}
    for k, v in target_w.items():
        if k.startswith("l"):
            if int(k[1:k.index(".")]) < n_layers:
                keep[k] = v
        else:
            keep[k] = v
    return keep


def make_classifier(seed: int, shape: ClassifierShape = CLF_SHAPE, sigma: float = 0.1
                    ) -> Dict[str, torch.Tensor]:
    """Halting classifier parameters, drawn in the order W1[h x f], b1[h], w2[h], b2[1]."""
    h, f = shape.hidden, shape.n_feat
    return {
        "W1": (_normal_host(seed, "clf.W1", h * f) * sigma).view(h, f),
        "b1": _normal_host(seed, "clf.b1", h) * sigma,
        "w2": _normal_host(seed, "clf.w2", h) * sigma,
        "b2": _normal_host(seed, "clf.b2", 1) * sigma,
    }


def make_tokens(seed: int, n: int, vocab: int, name: str = "tokens") -> torch.Tensor:
    g = np.random.Generator(np.random.Philox(key=[seed & 0xFFFFFFFF, _tid(name)]))
    return torch.from_numpy(g.integers(0, vocab, size=n, dtype=np.int64)).to(torch.int32)


def make_prompt(seed: int, n: int, vocab: int) -> torch.Tensor:
    """n token ids uniform on [0, vocab)."""
    return make_tokens(seed, n, vocab, "prompt")


def make_kv_fill(shape: ModelShape, ctx: int, seed: int, device="cpu") -> torch.Tensor:
    """N(0,1) keys and values for positions [0, ctx): bf16 [n_layers, 2, ctx, n_kv_heads, d_head]."""
    dev = torch.device(device)
    n = shape.n_layers * 2 * ctx * shape.d_kv
    x = _normal_host(seed, "kv", n) if dev.type == "cpu" else _normal_device(seed, "kv", n, dev)
    return x.view(shape.n_layers, 2, ctx, shape.n_kv_heads, shape.d_head).to(torch.bfloat16).to(dev)


def make_force_mask(seed: int, n: int, alpha: float) -> torch.Tensor:
    """Bernoulli(alpha) per generated position (bool[n]); a function of the position only."""
    g = np.random.Generator(np.random.Philox(key=[seed & 0xFFFFFFFF, _tid("force")]))
    return torch.from_numpy(g.random(n) < alpha)


def make_uniforms(seed: int, n: int, name: str) -> torch.Tensor:
    """n float32 uniforms on [0, 1), a function of (seed, name, index) only: the random numbers a
    sampling run consumes are inputs of the run, shared by the CPU oracle and the GPU path."""
    g = np.random.Generator(np.random.Philox(key=[seed & 0xFFFFFFFF, _tid("u." + name)]))
    return torch.from_numpy(g.random(n, dtype=np.float32))
