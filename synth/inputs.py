"""Counter-based, seeded generators for layer shapes, masks, weights and activations.

Everything is drawn with numpy's Philox generator keyed by ``(seed, tensor_id)``
so a tensor can be regenerated anywhere from two integers.  The shapes and
distributions stand in for GPT-2 fully-connected layers fed with token batches
(Sec. A.2 "Model and Implementation Details", Table "Public hyperparameters":
embedding 768, sequence length 1024); no dataset is involved.
"""
from __future__ import annotations

import numpy as np

# (name, I, O) per transformer block; Y = X @ W.T with W of shape [O, I].
def _block(d_model: int, ffn: int):
    return [
        ("qkv", d_model, 3 * d_model),
        ("proj", d_model, d_model),
        ("fc1", d_model, ffn),
        ("fc2", ffn, d_model),
    ]


LAYER_SETS = {
    "small": _block(768, 3072),
    "medium": _block(1024, 4096),
    "large": _block(1280, 5120),
}

# The five workloads named for this build.  "densities" with more than one
# entry is a sweep produced by successive mask updates.
CONFIGS = {
    "C1": dict(layers=[("fc1", 768, 3072)], T=512, act="f32", densities=[0.05],
               mask="uniform", zeta=0.3, R=0.25),
    "C2": dict(layers=LAYER_SETS["small"], T=8 * 1024, act="f32", densities=[0.10],
               mask="uniform", zeta=0.3, R=0.25),
    "C3": dict(layers=LAYER_SETS["small"], T=16 * 1024, act="f32", densities=[0.02],
               mask="powerlaw", zeta=0.3, R=0.25),
    "C4": dict(layers=LAYER_SETS["medium"], T=16 * 1024, act="bf16", densities=[0.05],
               mask="uniform", zeta=0.3, R=0.25),
    "C5": dict(layers=LAYER_SETS["large"], T=8 * 1024, act="f32",
               densities=[1.0, 0.5, 0.1, 0.02, 0.1, 0.5], mask="uniform", zeta=0.3, R=0.25,
               n_blocks=36),
}


def _rng(seed: int, tensor_id: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), int(tensor_id)]))


def normal(seed: int, tensor_id: int, shape, sigma: float = 1.0) -> np.ndarray:
    """fp32 draws from N(0, sigma^2)."""
    x = _rng(seed, tensor_id).standard_normal(size=shape, dtype=np.float32)
    if sigma != 1.0:
        x *= np.float32(sigma)
    return x


def active_count(n_total: int, density: float) -> int:
    """Number of active positions for a requested density: nearest integer, halves up."""
    return int(np.floor(float(density) * n_total + 0.5))


def uniform_mask(seed: int, tensor_id: int, O: int, I: int, density: float) -> np.ndarray:
    """uint8 [O, I] mask with exactly ``active_count`` ones, uniform without replacement."""
    n = O * I
    k = active_count(n, density)
    m = np.zeros(n, dtype=np.uint8)
    if k >= n:
        m[:] = 1
    elif k > 0:
        m[_rng(seed, tensor_id).permutation(n)[:k]] = 1
    return m.reshape(O, I)


def nested_uniform_masks(seed: int, tensor_id: int, O: int, I: int, densities) -> list:
    """One uniform mask per density from a single random order of the positions: the mask of
    density d is the first ``active_count(O*I, d)`` positions of that order (so the masks are
    nested).  Each is uniform without replacement; drawing the order once makes a whole sweep
    of densities cheap."""
    n = O * I
    order = _rng(seed, tensor_id).permutation(n)
    out = []
    for d in densities:
        m = np.zeros(n, dtype=np.uint8)
        m[order[: min(n, active_count(n, d))]] = 1
        out.append(m.reshape(O, I))
    return out


def powerlaw_row_lengths(seed: int, tensor_id: int, O: int, I: int, density: float,
                         alpha: float = 1.5) -> np.ndarray:
    """Per-row active counts with a Pareto tail (pdf ~ len^-alpha), summing exactly to the target.

    raw_r = (1-u)^(-1/(alpha-1)); a scale c is found by bisection so that
    sum_r min(I, c*raw_r) hits the target (so the heaviest rows are completely full);
    floors are taken and the remainder goes to the rows with the largest fractional
    parts (lowest row first on ties).
    """
    total = active_count(O * I, density)
    u = _rng(seed, tensor_id).random(O)
    raw = (1.0 - u) ** (-1.0 / (alpha - 1.0))
    lo, hi = 0.0, float(I)
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if np.minimum(float(I), mid * raw).sum() < total:
            lo = mid
        else:
            hi = mid
    real = np.minimum(float(I), hi * raw)
    base = np.floor(real).astype(np.int64)
    rem = total - int(base.sum())
    if rem > 0:
        frac = real - base
        frac[base >= I] = -1.0
        order = np.lexsort((np.arange(O), -frac))
        base[order[:rem]] += 1
    elif rem < 0:
        order = np.lexsort((np.arange(O), -base))
        base[order[:-rem]] -= 1
    assert int(base.sum()) == total and base.max() <= I and base.min() >= 0
    return base


def powerlaw_mask(seed: int, tensor_id: int, O: int, I: int, density: float,
                  alpha: float = 1.5) -> np.ndarray:
    """uint8 [O, I] mask whose row lengths follow ``powerlaw_row_lengths``; columns uniform."""
    lens = powerlaw_row_lengths(seed, tensor_id, O, I, density, alpha)
    keys = _rng(seed, tensor_id + (1 << 20)).random((O, I))
    rank = np.argsort(np.argsort(keys, axis=1, kind="stable"), axis=1, kind="stable")
    return (rank < lens[:, None]).astype(np.uint8)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (nearest, ties to even) and return the uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    b = b + 0x7FFF + ((b >> 16) & 1)
    return (b >> 16).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to fp32."""
    return (bits.astype(np.uint32) << 16).view(np.float32)


def make_layer(seed: int, layer_id: int, I: int, O: int, density: float, mask: str = "uniform",
               sigma: float = 0.02):
    """(W fp32 [O, I] with zeros at inactive positions, M uint8 [O, I])."""
    tid = 1000 * layer_id
    if mask == "uniform":
        M = uniform_mask(seed, tid + 1, O, I, density)
    elif mask == "powerlaw":
        M = powerlaw_mask(seed, tid + 1, O, I, density)
    else:
        raise ValueError(mask)
    W = normal(seed, tid + 2, (O, I), sigma)
    W *= M
    return W, M


def make_activations(seed: int, layer_id: int, T: int, I: int, O: int, act: str = "f32"):
    """(X [T, I], dY [T, O]) ~ N(0, 1).  For ``act='bf16'`` the values are rounded to
    bfloat16 and returned as (X_f32_exact, dY_f32_exact, X_bits, dY_bits)."""
    tid = 1000 * layer_id
    X = normal(seed, tid + 3, (T, I))
    dY = normal(seed, tid + 4, (T, O))
    if act == "f32":
        return X, dY
    if act == "bf16":
        xb, yb = to_bf16_bits(X), to_bf16_bits(dY)
        return bf16_bits_to_f32(xb), bf16_bits_to_f32(yb), xb, yb
    raise ValueError(act)
