"""Seeded synthetic inputs for the degraded-block backward (no method arithmetic here).

This module only draws random numbers and lays them out.  It is the one piece
shared by the CPU oracle's tests and the GPU path: both consume the same host
arrays.  Nothing in it computes any step of the method (no norm, no SwiGLU, no
projection of gradients, no SVD).

Shapes follow the paper's model table (App. E, architecture table: hidden /
intermediate / heads) and its sequence length (App. E, "maximum sequence length
256"); the paper trains on a public text corpus that is not available here, so
token ids are drawn uniformly over a 32000-entry vocabulary and activations are
Gaussian, as the workload description of each config states.

Values of the bf16 configs are rounded once, here, to the bf16 grid (round to
nearest even) and returned as float32 arrays holding exactly representable
values, so that the fp64 oracle and the bf16 GPU path start from identical
numbers.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

BASE_SEED = 20251016
VOCAB = 32000


@dataclass(frozen=True)
class Config:
    name: str
    index: int          # position in the benchmark's config list (seed offset)
    d_model: int        # d
    d_ff: int           # f
    heads: int
    batch: int
    seq: int
    rank: int           # r
    layers: int
    dtype: str          # "f32" or "bf16"
    micro_batches: int = 1
    stack: bool = False  # True: H and dOut come from a forward through a token stack

    @property
    def tokens(self) -> int:  # b = batch x seq
        return self.batch * self.seq


CONFIGS = {
    "C1": Config("C1", 0, 256, 688, 4, 2, 128, 32, 1, "f32"),
    "C2": Config("C2", 1, 512, 1376, 8, 8, 256, 128, 8, "bf16", stack=True),
    "C3": Config("C3", 2, 1024, 2736, 16, 16, 256, 256, 24, "bf16", micro_batches=2, stack=True),
    "C4": Config("C4", 3, 2048, 5461, 32, 8, 256, 512, 24, "bf16", stack=True),
    "C5": Config("C5", 4, 4096, 11008, 32, 4, 2048, 1024, 1, "bf16"),
}


def round_to_bf16_grid(x: np.ndarray) -> np.ndarray:
    """float32 array -> float32 array whose values are bf16-representable (RNE)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).copy()
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    u += np.uint32(0x7FFF)
    u += lsb                      # finite inputs cannot carry out of the exponent field
    u &= np.uint32(0xFFFF0000)
    return u.view(np.float32).reshape(x.shape)


def _cast(x: np.ndarray, dtype: str) -> np.ndarray:
    x = x.astype(np.float32, copy=False)
    return round_to_bf16_grid(x) if dtype == "bf16" else x


def _normal(rng: np.random.Generator, shape, std: float = 1.0) -> np.ndarray:
    x = rng.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return x


def rng_for(cfg_index: int, *stream: int) -> np.random.Generator:
    """Independent generator per (config, purpose...) tuple."""
    return np.random.default_rng([BASE_SEED + cfg_index, *stream])


def ffn_weights(rng: np.random.Generator, d: int, f: int, dtype: str, std: float = 0.02):
    """Wg, Wu [f x d], Wd [d x f] ~ N(0, std^2); gamma = 1 (fresh RMSNorm gain)."""
    Wg = _cast(_normal(rng, (f, d), std), dtype)
    Wu = _cast(_normal(rng, (f, d), std), dtype)
    Wd = _cast(_normal(rng, (d, f), std), dtype)
    gamma = np.ones(d, dtype=np.float32)
    return Wg, Wu, Wd, gamma


def mha_weights(rng: np.random.Generator, d: int, dtype: str, std: float = 0.02):
    """Wq, Wk, Wv, Wo [d x d] ~ N(0, std^2); attention-norm gain = 1."""
    Ws = [_cast(_normal(rng, (d, d), std), dtype) for _ in range(4)]
    return (*Ws, np.ones(d, dtype=np.float32))


def gaussian_block_io(rng: np.random.Generator, b: int, d: int, dtype: str):
    """Block input / stored FFN input and upstream gradient ~ N(0,1), [b x d] each."""
    X = _cast(_normal(rng, (b, d)), dtype)
    dOut = _cast(_normal(rng, (b, d)), dtype)
    return X, dOut


def perturbed_gain(rng: np.random.Generator, d: int, dtype: str):
    """A non-trivial norm gain (1 + 0.1 N(0,1)) so that tests exercise gamma."""
    return _cast(1.0 + 0.1 * _normal(rng, d), dtype)


def token_ids(rng: np.random.Generator, batch: int, seq: int) -> np.ndarray:
    return rng.integers(0, VOCAB, size=(batch, seq), dtype=np.int64)


def stack_params(cfg: Config, layers: int | None = None):
    """Embedding, per-layer MHA+FFN weights, final gain and untied LM head of a stack config.

    Every layer draws from a generator of its own (seeded by config and layer index), so the layers of
    a deep stack can be drawn by several host threads and a layer's values do not depend on the depth."""
    from concurrent.futures import ThreadPoolExecutor
    import os
    L = cfg.layers if layers is None else layers
    d, f = cfg.d_model, cfg.d_ff
    rng = rng_for(cfg.index, 1)
    emb = _cast(_normal(rng, (VOCAB, d), 0.02), cfg.dtype)
    lm_head = _cast(_normal(rng, (VOCAB, d), 0.02), cfg.dtype)

    def draw(layer: int):
        r = rng_for(cfg.index, 1, layer + 1)
        Wq, Wk, Wv, Wo, g_attn = mha_weights(r, d, cfg.dtype)
        Wg, Wu, Wd, g_ffn = ffn_weights(r, d, f, cfg.dtype)
        return dict(Wq=Wq, Wk=Wk, Wv=Wv, Wo=Wo, g_attn=g_attn, Wg=Wg, Wu=Wu, Wd=Wd, g_ffn=g_ffn)

    with ThreadPoolExecutor(max_workers=max(1, min(16, os.cpu_count() or 1, L))) as ex:
        blocks = list(ex.map(draw, range(L)))
    return dict(emb=emb, lm_head=lm_head, g_final=np.ones(d, dtype=np.float32), blocks=blocks)


def random_orthonormal(rng: np.random.Generator, n: int, r: int, dtype: str) -> np.ndarray:
    """[n x r] matrix with orthonormal columns (QR of a Gaussian), then cast.

    Used where only the cost of the path matters (timing runs): the path treats
    the projection as opaque data, so any full-column-rank P exercises it.
    """
    q, _ = np.linalg.qr(rng.standard_normal((n, r)))
    return _cast(q, dtype)


def pad_cols(x: np.ndarray, ld: int) -> np.ndarray:
    """Copy a [rows x cols] array into a zero-filled [rows x ld] buffer (ld >= cols)."""
    out = np.zeros((x.shape[0], ld), dtype=x.dtype)
    out[:, : x.shape[1]] = x
    return out


def planted_spectrum_matrix(rng: np.random.Generator, m: int, n: int, sigma: np.ndarray, dtype: str):
    """W [m x n] = U diag(sigma) V^T with orthonormal U [m x k], V [n x k] (QR of Gaussians),
    k = len(sigma) <= min(m, n), sigma in descending order.  Returns (W cast to dtype, U, V) so
    that tests know the singular subspaces by construction (before the cast's rounding)."""
    k = len(sigma)
    U, _ = np.linalg.qr(rng.standard_normal((m, k)))
    V, _ = np.linalg.qr(rng.standard_normal((n, k)))
    W = (U * np.asarray(sigma, dtype=np.float64)[None, :]) @ V.T
    return _cast(W.astype(np.float32), dtype), U, V


def spectrum_with_gap(k: int, r: int, decay: float = 0.98, gap: float = 0.5) -> np.ndarray:
    """Geometric spectrum sigma_i = decay^i with one extra factor `gap` between index r-1 and r."""
    s = decay ** np.arange(k, dtype=np.float64)
    s[r:] *= gap
    return s
