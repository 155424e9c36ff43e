"""Seeded synthetic inputs shaped like the paper's models (Table 1; Appendix C model table).

This module only draws random tensors and rounds them to the storage format. It holds none of the
method's arithmetic: no binarisation, no quantiser, no GEMM.  Both the CPU oracle's tests and the
HIP path's tests/bench take their inputs from here so that the two sides see identical bytes.

All arrays are returned as float32.  When a tensor is stored as bf16 on the device its values are
first rounded to bf16 here (round-to-nearest-even on the bit pattern), so a float32 -> bf16 cast on
the device is exact and both sides start from the same numbers.
"""
from __future__ import annotations

import numpy as np


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result is float32 with 16 low zero bits."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    r = ((u >> np.uint64(16)) & np.uint64(1)) + np.uint64(0x7FFF)
    u2 = ((u + r) & np.uint64(0xFFFF0000)).astype(np.uint32)
    return u2.view(np.float32).reshape(x.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of bf16-representable float32 values (asserts representability)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "value not representable in bf16"
    return (u >> np.uint32(16)).astype(np.uint16).reshape(x.shape)


def _store(x: np.ndarray, bf16: bool) -> np.ndarray:
    x = x.astype(np.float32)
    return bf16_round(x) if bf16 else x


def activations(rng, tokens, d_in, outlier_frac=0.0, outlier_count=0, outlier_scale=1.0, bf16=False):
    """X ~ N(0,1) with a few input channels scaled up (the activation outliers of FFN inputs)."""
    X = rng.standard_normal((tokens, d_in))
    n_out = outlier_count if outlier_count else int(round(outlier_frac * d_in))
    if n_out:
        ch = rng.choice(d_in, size=n_out, replace=False)
        X[:, ch] *= outlier_scale
    return _store(X, bf16)


def normal(rng, shape, std, bf16=False):
    return _store(rng.standard_normal(shape) * std, bf16)


def linear_case(seed, tokens, d_in, d_out, hp_rank=0, n_experts=1, bf16=False,
                outlier_frac=0.0, outlier_count=0, outlier_scale=1.0, w_std=0.02):
    """One decoupled linear: latent W, X, dY, low-rank high-precision factors A/B and router Wr."""
    rng = np.random.default_rng(seed)
    case = {
        "tokens": tokens, "d_in": d_in, "d_out": d_out, "hp_rank": hp_rank,
        "n_experts": n_experts, "bf16": bf16,
        "W": normal(rng, (d_out, d_in), w_std, bf16),
        "X": activations(rng, tokens, d_in, outlier_frac, outlier_count, outlier_scale, bf16),
        "dY": normal(rng, (tokens, d_out), 1.0, bf16),
        "alpha": 2.0, "beta": 0.2,          # the paper's feature-scaling initialisation (Sec. 3.2)
    }
    if hp_rank:
        if n_experts == 1:
            case["A"] = normal(rng, (hp_rank, d_in), w_std, bf16)
            case["B"] = normal(rng, (d_out, hp_rank), w_std, bf16)
        else:
            case["A"] = normal(rng, (n_experts, hp_rank, d_in), w_std, bf16)
            case["B"] = normal(rng, (n_experts, d_out, hp_rank), w_std, bf16)
            case["Wr"] = normal(rng, (n_experts, d_in), w_std, bf16)
    return case


def config1():
    """Small fp32 case: T=64, 256x256, r=16, 4 outlier channels x10, seed 0."""
    return linear_case(0, 64, 256, 256, hp_rank=16, bf16=False, outlier_count=4, outlier_scale=10.0)


def config2(tokens=8192, seed=2):
    """1.3B-shaped attention projection, bf16: 2048x2048, r=128, 1 % of channels x20."""
    return linear_case(seed, tokens, 2048, 2048, hp_rank=128, bf16=True,
                       outlier_frac=0.01, outlier_scale=20.0)


def ffn_case(seed, tokens, d_model, d_ffn, n_experts, hp_rank, bf16=True,
             outlier_frac=0.01, outlier_scale=20.0, w_std=0.02):
    """Decoupled FFN: three 1-bit projections plus routed high-precision FFN experts of width r."""
    rng = np.random.default_rng(seed)
    return {
        "tokens": tokens, "d_model": d_model, "d_ffn": d_ffn, "n_experts": n_experts,
        "hp_rank": hp_rank, "bf16": bf16,
        "W_up": normal(rng, (d_ffn, d_model), w_std, bf16),
        "W_gate": normal(rng, (d_ffn, d_model), w_std, bf16),
        "W_down": normal(rng, (d_model, d_ffn), w_std, bf16),
        "Up": normal(rng, (n_experts, hp_rank, d_model), w_std, bf16),
        "Gate": normal(rng, (n_experts, hp_rank, d_model), w_std, bf16),
        "Down": normal(rng, (n_experts, d_model, hp_rank), w_std, bf16),
        "Wr": normal(rng, (n_experts, d_model), w_std, bf16),
        "X": activations(rng, tokens, d_model, outlier_frac, 0, outlier_scale, bf16),
        "dY": normal(rng, (tokens, d_model), 1.0, bf16),
        "alpha": 2.0, "beta": 0.2,
    }


def config3(tokens=8192, seed=3):
    """1.3B-shaped FFN triplet: d_model=2048, d_ffn=5504, E=8 experts of width 32, top-1."""
    return ffn_case(seed, tokens, 2048, 5504, 8, 32)


def decode_case(seed, batch, d_in=4096, d_out=11008, n_experts=8, hp_rank=64, n_layers=1, w_std=0.02):
    """Decode GEMV inputs: latent W (packed offline by the caller), token batch, bf16 low-rank experts."""
    rng = np.random.default_rng(seed)
    return {
        "batch": batch, "d_in": d_in, "d_out": d_out, "n_experts": n_experts, "hp_rank": hp_rank,
        "n_layers": n_layers,
        "W": normal(rng, (n_layers, d_out, d_in), w_std, True),
        "X": activations(rng, n_layers * batch, d_in, bf16=True).reshape(n_layers, batch, d_in),
        "A": normal(rng, (n_layers, n_experts, hp_rank, d_in), w_std, True),
        "B": normal(rng, (n_layers, n_experts, d_out, hp_rank), w_std, True),
        "Wr": normal(rng, (n_layers, n_experts, d_in), w_std, True),
        "alpha": 2.0, "beta": 0.2,
    }


def config4(batch=1, seed=4, n_layers=1):
    return decode_case(seed, batch, n_layers=n_layers)


# Feature scales of the trained 1.3B model (App. F, table of feature scaling after training), in the
# order the paper lists the layers; used cyclically as realistic per-layer alpha/beta.
TRAINED_ALPHA = [1.82, 1.73, 1.57, 1.59, 1.39, 1.33, 1.25, 1.22, 1.34, 1.49, 1.37, 1.27, 1.38, 1.45, 1.56, 1.61]
TRAINED_BETA = [0.78, 0.62, 0.48, 0.42, 0.38, 0.34, 0.31, 0.26, 0.29, 0.36, 0.43, 0.45, 0.41, 0.47, 0.52, 0.50]


def stack_case(seed, n_layers, tokens, d_model, d_ffn, n_experts, hp_rank, vocab=32000, w_std=0.02):
    """Token ids ~ U[0, vocab) gathering rows of an N(0,1) bf16 table, per-layer weights of a stack of
    {q,k,v,o pure 1-bit linears + decoupled FFN}, and an N(0,1) output gradient."""
    rng = np.random.default_rng(seed)
    layers = []
    for l in range(n_layers):
        w = {n: normal(rng, (d_model, d_model), w_std, True) for n in ("Wq", "Wk", "Wv", "Wo")}
        w.update(W_up=normal(rng, (d_ffn, d_model), w_std, True), W_gate=normal(rng, (d_ffn, d_model), w_std, True),
                 W_down=normal(rng, (d_model, d_ffn), w_std, True),
                 Up=normal(rng, (n_experts, hp_rank, d_model), w_std, True),
                 Gate=normal(rng, (n_experts, hp_rank, d_model), w_std, True),
                 Down=normal(rng, (n_experts, d_model, hp_rank), w_std, True),
                 Wr=normal(rng, (n_experts, d_model), w_std, True),
                 alpha=TRAINED_ALPHA[l % 16], beta=TRAINED_BETA[l % 16])
        layers.append(w)
    return {"layers": layers, "table": normal(rng, (vocab, d_model), 1.0, True),
            "ids": rng.integers(0, vocab, size=tokens).astype(np.int32),
            "dY": normal(rng, (tokens, d_model), 1.0, True),
            "tokens": tokens, "d_model": d_model, "d_ffn": d_ffn, "n_experts": n_experts, "hp_rank": hp_rank}
