"""Seeded synthetic inputs for the HiFT step: workload shapes, token batches, labels and
initial weights.

This module holds no arithmetic of the method.  It only draws random numbers with numpy's
PCG64 generator and describes the five workload shapes.  Both the CPU oracle's tests and the
GPU path's tests call it so that the two sides see identical inputs; neither side's
implementation imports it.

Weights are drawn per tensor from a caller-supplied tensor list (name, shape, kind), so the
module does not know any model's parameter layout either.
"""
from __future__ import annotations

import numpy as np

# kind codes of a parameter tensor, shared vocabulary of the tensor lists
KIND_MATRIX = 0   # >= 2 dims: N(0, 0.02^2)
KIND_GAIN = 1     # norm gain: ones
KIND_BIAS = 2     # bias / norm shift: zeros

# Workload shapes.  C1..C5 follow the five configurations of the benchmark description;
# the *_L2 twins keep every width of C4 / C5 and cut the depth to two hidden layers so that
# a CPU implementation finishes a step in about a minute.
WORKLOADS = {
    "C1": dict(arch=0, n_layers=2, d_model=64, n_heads=4, d_ffn=256, vocab=256, max_seq=32,
               n_classes=0, norm_eps=1e-5, rope_base=10000.0, dtype=0, batch=2, seq=32,
               m=1, strategy="bottom2up",
               opt=dict(kind="adamw", lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8,
                        weight_decay=0.01, momentum=0.0)),
    "C2": dict(arch=1, n_layers=12, d_model=768, n_heads=12, d_ffn=3072, vocab=50265,
               max_seq=514, n_classes=2, norm_eps=1e-5, rope_base=10000.0, dtype=1,
               batch=8, seq=128, m=1, strategy="top2down",
               opt=dict(kind="adamw", lr=1e-5, beta1=0.9, beta2=0.999, eps=1e-8,
                        weight_decay=0.0, momentum=0.0)),
    "C3": dict(arch=1, n_layers=24, d_model=1024, n_heads=16, d_ffn=4096, vocab=50265,
               max_seq=514, n_classes=3, norm_eps=1e-5, rope_base=10000.0, dtype=1,
               batch=16, seq=128, m=2, strategy="random",
               opt=dict(kind="adamw", lr=1e-5, beta1=0.9, beta2=0.999, eps=1e-8,
                        weight_decay=0.0, momentum=0.0)),
    "C4": dict(arch=2, n_layers=32, d_model=4096, n_heads=32, d_ffn=11008, vocab=32000,
               max_seq=512, n_classes=0, norm_eps=1e-5, rope_base=10000.0, dtype=1,
               batch=4, seq=512, m=1, strategy="bottom2up",
               opt=dict(kind="adamw", lr=1e-5, beta1=0.9, beta2=0.999, eps=1e-8,
                        weight_decay=0.0, momentum=0.0)),
    "C5": dict(arch=2, n_layers=40, d_model=5120, n_heads=40, d_ffn=13824, vocab=32000,
               max_seq=1024, n_classes=0, norm_eps=1e-5, rope_base=10000.0, dtype=1,
               batch=2, seq=1024, m=4, strategy="bottom2up",
               opt=dict(kind="adamw", lr=1e-5, beta1=0.9, beta2=0.999, eps=1e-8,
                        weight_decay=0.0, momentum=0.0)),
}
# The second decoder family of the paper's model list (GPT-2 / OPT: learned positions, LayerNorm, GELU,
# biases, output matrix tied to the token table) at the OPT-13B shape, batch and grouping as C5.
WORKLOADS["OPT13B"] = dict(arch=0, n_layers=40, d_model=5120, n_heads=40, d_ffn=20480, vocab=50272,
                           max_seq=2048, n_classes=0, norm_eps=1e-5, rope_base=10000.0, dtype=1,
                           batch=2, seq=1024, m=4, strategy="bottom2up", tie_embeddings=1,
                           opt=dict(kind="adamw", lr=1e-5, beta1=0.9, beta2=0.999, eps=1e-8,
                                    weight_decay=0.0, momentum=0.0))
WORKLOADS["C4_L2"] = dict(WORKLOADS["C4"], n_layers=2)
WORKLOADS["C5_L2"] = dict(WORKLOADS["C5"], n_layers=2, m=2)

MODEL_KEYS = ("arch", "n_layers", "d_model", "n_heads", "d_ffn", "vocab", "max_seq",
              "n_classes", "norm_eps", "rope_base", "dtype")


def model_config(workload: dict, **overrides) -> dict:
    """The model-shape part of a workload, optionally with fields replaced."""
    cfg = {k: workload[k] for k in MODEL_KEYS}
    if workload.get("tie_embeddings"):
        cfg["tie_embeddings"] = 1
    cfg.update(overrides)
    return cfg


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([int(seed), int(stream)]))


def uniform_tokens(seed: int, step: int, batch: int, seq: int, vocab: int) -> np.ndarray:
    """int32 [batch, seq], uniform in [0, vocab)."""
    return _rng(seed, 1000 + step).integers(0, vocab, size=(batch, seq), dtype=np.int32)


def zipf_tokens(seed: int, step: int, batch: int, seq: int, vocab: int,
                exponent: float = 1.1) -> np.ndarray:
    """int32 [batch, seq] from the bounded Zipf law P(rank r) ~ r^-exponent, r = 1..vocab,
    token id = r - 1, by inverse-CDF sampling."""
    w = np.arange(1, vocab + 1, dtype=np.float64) ** (-exponent)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    u = _rng(seed, 2000 + step).random(size=(batch, seq))
    ids = np.searchsorted(cdf, u, side="left")
    return np.minimum(ids, vocab - 1).astype(np.int32)


def next_token_labels(tokens: np.ndarray) -> np.ndarray:
    """Labels of a causal language-model batch: position s is asked for token s+1; the last
    position of every sequence carries -1 (no target)."""
    lab = np.full_like(tokens, -1)
    lab[:, :-1] = tokens[:, 1:]
    return lab


def class_labels(seed: int, step: int, batch: int, n_classes: int) -> np.ndarray:
    """int32 [batch], uniform over the classes."""
    return _rng(seed, 3000 + step).integers(0, n_classes, size=(batch,), dtype=np.int32)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16-representable value (ties to even); result
    stays fp32.  Used so that both sides of a bf16 comparison start from equal weights."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + r) & np.uint32(0xFFFF0000)).view(np.float32)


def init_tensor(seed: int, index: int, shape, kind: int, bf16_exact: bool,
                std: float = 0.02, jitter: float = 0.0) -> np.ndarray:
    """One parameter tensor, fp32.  Matrices N(0, std^2); gains 1; biases 0.  `jitter` > 0
    adds N(0, jitter^2) to gains and biases so that gradient checks see generic values."""
    n = int(np.prod(shape))
    g = _rng(seed, 10 + index)
    if kind == KIND_MATRIX:
        t = g.standard_normal(n, dtype=np.float32) * np.float32(std)
    else:
        t = np.full(n, 1.0 if kind == KIND_GAIN else 0.0, dtype=np.float32)
        if jitter > 0.0:
            t += g.standard_normal(n, dtype=np.float32) * np.float32(jitter)
    if bf16_exact:
        t = round_to_bf16(t)
    return t


def init_params(seed: int, tensors, bf16_exact: bool, std: float = 0.02,
                jitter: float = 0.0) -> np.ndarray:
    """Flat fp32 parameter vector for a tensor list [(name, shape, kind), ...] in the
    order given; tensor i is drawn from its own random stream."""
    parts = [init_tensor(seed, i, shape, kind, bf16_exact, std, jitter)
             for i, (_name, shape, kind) in enumerate(tensors)]
    return np.concatenate(parts) if parts else np.zeros(0, np.float32)


def make_batch(workload: dict, seed: int, step: int, batch: int | None = None,
               seq: int | None = None):
    """(tokens, labels) of one step of a workload: uniform tokens for arch 0 and 1, bounded
    Zipf(1.1) tokens for arch 2; next-token labels for the decoders, class labels for the
    encoder."""
    b = batch or workload["batch"]
    s = seq or workload["seq"]
    if workload["arch"] == 2:
        tok = zipf_tokens(seed, step, b, s, workload["vocab"])
    else:
        tok = uniform_tokens(seed, step, b, s, workload["vocab"])
    if workload["arch"] == 1:
        lab = class_labels(seed, step, b, workload["n_classes"])
    else:
        lab = next_token_labels(tok)
    return tok, lab


def fill_weights_on_device(model, seed: int) -> None:
    """Initial weights for models too large to draw on the host (the 7B and 13B shapes at full depth): N(0, 0.02^2)
    matrices, unit gains, zero biases, drawn with torch's generator on the GPU unit by unit and handed to
    `model.write_params_device` (or, through the host, to `model.write_params`).  `model` needs `tensors` (name,
    shape, kind, unit, offset per tensor, in parameter order) and one of the two writers (unit_lo, unit_hi, values)."""
    import torch
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    per_unit = {}
    for _name, shape, kind, unit, _off in model.tensors:
        per_unit.setdefault(unit, []).append((shape, kind))
    for unit in sorted(per_unit):
        parts = []
        for shape, kind in per_unit[unit]:
            n = int(np.prod(shape))
            if kind == KIND_MATRIX:
                parts.append(torch.randn(n, generator=g, device="cuda", dtype=torch.float32) * 0.02)
            else:
                parts.append(torch.full((n,), 1.0 if kind == KIND_GAIN else 0.0, device="cuda"))
        flat = torch.cat(parts)
        if hasattr(model, "write_params_device"):
            model.write_params_device(unit, unit + 1, flat)
        else:
            model.write_params(unit, unit + 1, flat.cpu().numpy())
        del parts, flat
