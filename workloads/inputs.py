"""Seeded synthetic inputs for the five benchmark configurations.

No public dataset is involved: every configuration is synthetic by
construction.  RNG: numpy Generator(PCG64(seed)), seed = 1000 + configuration
number.  Sizes default to the full configuration; smaller sizes are used by
parity tests so the CPU oracle finishes in seconds.
"""
from __future__ import annotations

import numpy as np


def _rng(config: int, extra: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(1000 + config + 7919 * extra))


def c1_inputs(rows: int = 1024, cols: int = 1024, seed_extra: int = 0):
    """x, y [rows, cols] and bias [cols], uniform in [-1, 1), float32."""
    r = _rng(1, seed_extra)
    u = lambda *s: (r.random(s, dtype=np.float32) * 2.0 - 1.0).astype(np.float32)
    return {"x": u(rows, cols), "y": u(rows, cols), "bias": u(cols)}


def c2_inputs(batch: int = 128, dims=(784, 512, 512, 10), steps: int = 100, seed_extra: int = 0):
    """He-initialised weights (std sqrt(2/fan_in)), zero biases, `steps`
    batches of N(0,1) inputs with labels uniform in [0, classes)."""
    r = _rng(2, seed_extra)
    out = {}
    for i in range(len(dims) - 1):
        fan_in, fan_out = dims[i], dims[i + 1]
        out[f"W{i+1}"] = (r.standard_normal((fan_in, fan_out), dtype=np.float32)
                          * np.float32(np.sqrt(2.0 / fan_in))).astype(np.float32)
        out[f"b{i+1}"] = np.zeros((fan_out,), dtype=np.float32)
    out["X"] = r.standard_normal((steps, batch, dims[0]), dtype=np.float32)
    out["labels"] = r.integers(0, dims[-1], size=(steps, batch), dtype=np.int32)
    return out


def c3_inputs(batch: int = 32, seq: int = 256, d_model: int = 1024, ffn: int = 4096, seed_extra: int = 0):
    """Transformer encoder layer: activations and upstream gradient N(0,1),
    weights N(0, 0.02), biases 0, LayerNorm gain 1 and shift 0.  Values are
    float32 here; the caller rounds them to bf16."""
    r = _rng(3, seed_extra)
    n = lambda std, *s: (r.standard_normal(s, dtype=np.float32) * np.float32(std)).astype(np.float32)
    d = d_model
    return {
        "x": n(1.0, batch, seq, d), "dy": n(1.0, batch, seq, d),
        "Wq": n(0.02, d, d), "Wk": n(0.02, d, d), "Wv": n(0.02, d, d), "Wo": n(0.02, d, d),
        "W1": n(0.02, d, ffn), "W2": n(0.02, ffn, d),
        "bq": np.zeros(d, np.float32), "bk": np.zeros(d, np.float32), "bv": np.zeros(d, np.float32),
        "bo": np.zeros(d, np.float32), "b1": np.zeros(ffn, np.float32), "b2": np.zeros(d, np.float32),
        "g1": np.ones(d, np.float32), "be1": np.zeros(d, np.float32),
        "g2": np.ones(d, np.float32), "be2": np.zeros(d, np.float32),
    }


def c4_inputs(n: int = 268_435_456, seed_extra: int = 0):
    """Parameters, gradients and first moments N(0, std 1e-2); the second
    moment is |N(0, 1e-2)| because a negative second moment has no square
    root.  Generated in chunks to bound peak host memory."""
    r = _rng(4, seed_extra)
    out = {}
    for name in ("p", "g", "m", "v"):
        a = np.empty((n,), dtype=np.float32)
        step = 1 << 24
        for lo in range(0, n, step):
            hi = min(n, lo + step)
            a[lo:hi] = r.standard_normal((hi - lo,), dtype=np.float32)
        a *= np.float32(1e-2)
        if name == "v":
            np.abs(a, out=a)
        out[name] = a
    return out


C4_HYPER = {"lr": 1e-3, "beta1": 0.9, "beta2": 0.999, "eps": 1e-8, "t": 1, "max_norm": 1.0}


def c5_inputs(d: int = 2048, steps: int = 200, n_base: int = 4, n_res: int = 8,
              batches=(8, 16, 32, 64, 128, 256, 512, 1024), seed_extra: int = 0):
    """Weights N(0, 2/d) (std sqrt(2/d)), biases 0; per step a batch size drawn
    uniformly from `batches` and an int32 word w, from which the program
    derives the number of residual blocks 1 + (w mod n_res).  The activations
    of a step are generated from the step's own stream (see c5_batch)."""
    r = _rng(5, seed_extra)
    std = np.float32(np.sqrt(2.0 / d))
    out = {"W": [(r.standard_normal((d, d), dtype=np.float32) * std).astype(np.float32) for _ in range(n_base)],
           "Wr": [(r.standard_normal((d, d), dtype=np.float32) * std).astype(np.float32) for _ in range(n_res)],
           "b": [np.zeros(d, np.float32) for _ in range(n_base)],
           "br": [np.zeros(d, np.float32) for _ in range(n_res)],
           "batch": r.choice(np.array(batches), size=steps).astype(np.int64),
           "word": r.integers(0, 1 << 20, size=steps, dtype=np.int32)}
    return out


def c5_batch(step: int, batch: int, d: int = 2048, seed_extra: int = 0):
    r = _rng(5, 1000 + step + seed_extra)
    return r.standard_normal((batch, d), dtype=np.float32)
