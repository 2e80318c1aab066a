"""Seeded synthetic inputs for the mini-sequence LM-head + cross-entropy path
and for the mini-sequence MLP path.

This module is the only code shared by the CPU oracle's tests and the GPU
harness.  It holds no arithmetic of the method itself: it draws hidden states
H, the output-embedding matrix W and the labels with the shapes and value
distributions of the five benchmark configurations (Llama3-8B, Gemma-2 and
Mistral-7B shaped LM heads; the shapes are the ones the paper's model listing
and evaluation section name), rounds H and W to bfloat16 and hands them back
as raw bit patterns plus exact float widenings.  For the MLP block it draws
the block input X, the three projection matrices and an upstream gradient dO
with the Llama shapes of the paper's model listing.

bfloat16 is carried as ``numpy.uint16`` bit patterns (numpy has no bf16 type).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

IGNORE_INDEX = -100
BASE_SEED = 20240715

# tensor ids fed into the Philox key so every tensor has its own stream
_T_H, _T_W, _T_LABEL, _T_IGNORE, _T_PERM = 1, 2, 3, 4, 5
_T_X, _T_WG, _T_WU, _T_WD, _T_DO = 11, 12, 13, 14, 15


# ----------------------------------------------------------------------------
# bfloat16 <-> float conversions (format handling only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); return uint16 bits."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + (np.uint32(0x7FFF) + lsb)
    out = (r >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out[nan] = np.uint16(0x7FC0)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float64."""
    return bf16_bits_to_f32(b).astype(np.float64)


def to_device_bf16(bits: np.ndarray):
    """bfloat16 bit patterns -> a torch bf16 tensor on the current GPU (a copy of the bits, no arithmetic)."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def bf16_tensor_to_f64(t) -> np.ndarray:
    """A torch bf16 tensor (any device) -> float64 numpy array, exact."""
    import torch
    return bf16_bits_to_f64(t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16))


# ----------------------------------------------------------------------------
# configurations
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class Config:
    name: str
    index: int          # 1-based index of the benchmark configuration
    S: int              # tokens (batch folded into the sequence)
    d: int              # hidden size
    V: int              # vocabulary size
    M: int              # number of mini-sequences
    h_std: float        # std of H entries
    w_std: float        # std of W entries
    label_dist: str     # "uniform" | "zipf"
    ignore: str         # "every16" | "fraction"
    ignore_frac: float  # used when ignore == "fraction"

    @property
    def C(self) -> int:
        return -(-self.S // self.M)

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index


CONFIGS = {
    1: Config("tiny", 1, 512, 256, 4096, 4, 1.0, 0.02, "uniform", "every16", 0.0),
    2: Config("llama3-8b", 2, 8192, 4096, 128256, 8, 4.0 / 64.0, 0.02, "uniform", "fraction", 0.01),
    3: Config("llama3-8b-long", 3, 32768, 4096, 128256, 32, 4.0 / 64.0, 0.02, "zipf", "fraction", 0.01),
    4: Config("gemma2-largevocab", 4, 16384, 3584, 256000, 16, 1.0, 0.02, "uniform", "fraction", 0.02),
    5: Config("mistral-7b-verylong", 5, 131072, 4096, 32768, 64, 1.0, 0.02, "zipf", "fraction", 0.05),
}


def custom_config(S, d, V, M, *, index=100, h_std=1.0, w_std=0.02, label_dist="uniform",
                  ignore="fraction", ignore_frac=0.05, name="custom") -> Config:
    """A configuration of arbitrary shape for parity tests (ragged tiles, odd M)."""
    return Config(name, index, S, d, V, M, h_std, w_std, label_dist, ignore, ignore_frac)


def _rng(seed: int, tensor_id: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed & 0xFFFFFFFFFFFFFFFF, tensor_id]))


def _normal_bf16(rng: np.random.Generator, rows: int, cols: int, std: float) -> np.ndarray:
    """rows x cols N(0, std^2) values rounded to bf16, generated in row blocks."""
    out = np.empty((rows, cols), dtype=np.uint16)
    blk = max(1, (1 << 24) // max(cols, 1))
    for r0 in range(0, rows, blk):
        r1 = min(rows, r0 + blk)
        x = rng.standard_normal((r1 - r0, cols), dtype=np.float32)
        x *= np.float32(std)
        out[r0:r1] = f32_to_bf16_bits(x)
    return out


def _zipf_labels(rng_lab, rng_perm, n: int, V: int, s: float = 1.1) -> np.ndarray:
    """Zipf(s) over ranks 1..V (inverse-CDF + binary search); ranks are sent to
    class ids through a seeded permutation so hot classes scatter over vocab tiles."""
    w = 1.0 / np.power(np.arange(1, V + 1, dtype=np.float64), s)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    u = rng_lab.random(n)
    rank = np.searchsorted(cdf, u, side="left")
    rank = np.minimum(rank, V - 1)
    perm = rng_perm.permutation(V)
    return perm[rank].astype(np.int32)


def make_labels(cfg: Config) -> np.ndarray:
    rng_lab = _rng(cfg.seed, _T_LABEL)
    if cfg.label_dist == "uniform":
        labels = rng_lab.integers(0, cfg.V, size=cfg.S, dtype=np.int64).astype(np.int32)
    elif cfg.label_dist == "zipf":
        labels = _zipf_labels(rng_lab, _rng(cfg.seed, _T_PERM), cfg.S, cfg.V)
    else:
        raise ValueError(cfg.label_dist)
    if cfg.ignore == "every16":
        labels[15::16] = IGNORE_INDEX
    elif cfg.ignore == "fraction":
        k = int(round(cfg.ignore_frac * cfg.S))
        if k > 0:
            pos = _rng(cfg.seed, _T_IGNORE).choice(cfg.S, size=k, replace=False)
            labels[pos] = IGNORE_INDEX
    else:
        raise ValueError(cfg.ignore)
    return labels


@dataclass
class Inputs:
    cfg: Config
    H_bits: np.ndarray   # uint16 [S, d]  bf16 bit patterns
    W_bits: np.ndarray   # uint16 [V, d]
    labels: np.ndarray   # int32  [S]
    ignore_index: int = IGNORE_INDEX

    def H_f64(self, rows=None) -> np.ndarray:
        return bf16_bits_to_f64(self.H_bits if rows is None else self.H_bits[rows])

    def W_f64(self, rows=None) -> np.ndarray:
        return bf16_bits_to_f64(self.W_bits if rows is None else self.W_bits[rows])

    @property
    def n_valid(self) -> int:
        return int((self.labels != self.ignore_index).sum())


def make_inputs(cfg) -> Inputs:
    """Draw the tensors of a configuration (an int 1..5 or a Config)."""
    if not isinstance(cfg, Config):
        cfg = CONFIGS[int(cfg)]
    H = _normal_bf16(_rng(cfg.seed, _T_H), cfg.S, cfg.d, cfg.h_std)
    W = _normal_bf16(_rng(cfg.seed, _T_W), cfg.V, cfg.d, cfg.w_std)
    return Inputs(cfg, H, W, make_labels(cfg))


# ----------------------------------------------------------------------------
# mini-sequence MLP (three bias-free linear layers and SiLU)
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class MlpConfig:
    name: str
    index: int          # 1-based index among the MLP configurations
    S: int              # tokens (batch folded into the sequence)
    d: int              # hidden size
    I: int              # intermediate size
    M: int              # number of mini-sequences
    x_std: float = 1.0      # block input (after the normalisation layer)
    w_std: float = 0.02     # all three projections
    do_std: float = 1.0     # upstream gradient of the block output

    @property
    def C(self) -> int:
        return -(-self.S // self.M)

    @property
    def seed(self) -> int:
        return BASE_SEED + 1000 + self.index


# chunk size C = d (the constant chunk size the paper's chunk-based variant uses for MLP blocks)
MLP_CONFIGS = {
    1: MlpConfig("tiny", 1, 512, 256, 896, 2),
    2: MlpConfig("llama3-8b-mlp", 2, 8192, 4096, 14336, 2),
    3: MlpConfig("llama3-8b-mlp-long", 3, 32768, 4096, 14336, 8),
    4: MlpConfig("llama2-7b-mlp", 4, 16384, 4096, 11008, 4),
}


def custom_mlp_config(S, d, I, M, *, index=100, x_std=1.0, w_std=0.02, do_std=1.0, name="custom") -> MlpConfig:
    return MlpConfig(name, index, S, d, I, M, x_std, w_std, do_std)


@dataclass
class MlpInputs:
    cfg: MlpConfig
    X_bits: np.ndarray    # uint16 [S, d]
    Wg_bits: np.ndarray   # uint16 [I, d]   gate projection, stored [out, in]
    Wu_bits: np.ndarray   # uint16 [I, d]   up projection
    Wd_bits: np.ndarray   # uint16 [d, I]   down projection
    dO_bits: np.ndarray   # uint16 [S, d]   upstream gradient of the block output

    def f64(self, name: str, rows=None) -> np.ndarray:
        b = getattr(self, name + "_bits")
        return bf16_bits_to_f64(b if rows is None else b[rows])


def make_mlp_inputs(cfg) -> MlpInputs:
    """Draw the tensors of an MLP configuration (an int 1..4 or an MlpConfig)."""
    if not isinstance(cfg, MlpConfig):
        cfg = MLP_CONFIGS[int(cfg)]
    return MlpInputs(
        cfg,
        _normal_bf16(_rng(cfg.seed, _T_X), cfg.S, cfg.d, cfg.x_std),
        _normal_bf16(_rng(cfg.seed, _T_WG), cfg.I, cfg.d, cfg.w_std),
        _normal_bf16(_rng(cfg.seed, _T_WU), cfg.I, cfg.d, cfg.w_std),
        _normal_bf16(_rng(cfg.seed, _T_WD), cfg.d, cfg.I, cfg.w_std),
        _normal_bf16(_rng(cfg.seed, _T_DO), cfg.S, cfg.d, cfg.do_std),
    )
