"""Seeded synthetic inputs shaped like the paper's FFN workloads.

This module holds no arithmetic of the method: it only draws the random tensors (and the bias that
dials the activation sparsity) that both the CPU oracle and the GPU library are fed with.
Shapes follow the paper's appendix table (model dimension 2048 / 4096, FFN hidden dimension
8192 / 16384); the sparsity range follows Fig. 1 (84-98 % zeros after Squared-ReLU).

All tensors are float32 numpy arrays; each consumer rounds them to its own storage type.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
from scipy.special import ndtri


@dataclass(frozen=True)
class Workload:
    name: str
    T: int          # tokens
    D: int          # model dimension
    F: int          # FFN hidden dimension
    sparsity: object  # float target fraction of zeros, or the string "per_feature"
    seed: int


WORKLOADS = {
    # small case the oracle finishes in well under a second
    "c1": Workload("c1", 256, 512, 2048, 0.90, 1000),
    # 1B-model FFN dims, per-feature positive fraction uniform in [2 %, 15 %]
    "c2": Workload("c2", 8192, 2048, 8192, "per_feature", 2000),
    # 7B-model FFN dims, four layers at 85 / 90 / 95 / 98 % zeros
    "c3_85": Workload("c3_85", 16384, 4096, 16384, 0.85, 3000),
    "c3_90": Workload("c3_90", 16384, 4096, 16384, 0.90, 3001),
    "c3_95": Workload("c3_95", 16384, 4096, 16384, 0.95, 3002),
    "c3_98": Workload("c3_98", 16384, 4096, 16384, 0.98, 3003),
    # forward + backward at the 7B dims, 90 % zeros
    "c4": Workload("c4", 16384, 4096, 16384, 0.90, 4000),
    # fp8 shape
    "c5": Workload("c5", 8192, 8192, 32768, 0.95, 5000),
}


def bias_for(F: int, sparsity, rng: np.random.Generator) -> np.ndarray:
    """Per-feature bias b1 such that, for pre-activations ~ N(0, 1), the wanted fraction is negative."""
    if isinstance(sparsity, str):
        if sparsity != "per_feature":
            raise ValueError(sparsity)
        p = rng.uniform(0.02, 0.15, size=F)           # positive fraction of each feature
        return (-ndtri(1.0 - p)).astype(np.float32)
    return np.full(F, -ndtri(float(sparsity)), dtype=np.float32)


def make_inputs(T: int, D: int, F: int, sparsity, seed: int, with_dy: bool = False, token_corr=None) -> dict:
    """X ~ N(0,1) [T,D]; W1 ~ N(0,1/D) [D,F]; W2 ~ N(0,1/F) [F,D]; b1 [F]; optionally dY ~ N(0,1) [T,D].
    token_corr = (L, rho): consecutive tokens are correlated in runs of L (what the paper reports of real activations:
    a feature is often non-zero on a stretch of consecutive tokens): x_t = sqrt(rho) base_{t // L} + sqrt(1 - rho) e_t,
    still N(0,1) marginally."""
    rng = np.random.Generator(np.random.Philox(seed))
    X = rng.standard_normal((T, D), dtype=np.float32)
    if token_corr is not None:
        L, rho = token_corr
        base = np.random.Generator(np.random.Philox(seed + 7919)).standard_normal(((T + L - 1) // L, D), dtype=np.float32)
        X = np.float32(np.sqrt(rho)) * np.repeat(base, L, axis=0)[:T] + np.float32(np.sqrt(1.0 - rho)) * X
    out = {
        "X": X,
        "W1": rng.standard_normal((D, F), dtype=np.float32) * np.float32(1.0 / np.sqrt(D)),
        "W2": rng.standard_normal((F, D), dtype=np.float32) * np.float32(1.0 / np.sqrt(F)),
        "b1": bias_for(F, sparsity, rng),
    }
    if with_dy:
        out["dY"] = rng.standard_normal((T, D), dtype=np.float32)
    return out


def make_workload(name: str, with_dy: bool = False, T: int | None = None) -> dict:
    """Inputs of a named workload; T overrides the token count (a token slice of the same recipe)."""
    w = WORKLOADS[name]
    return make_inputs(T or w.T, w.D, w.F, w.sparsity, w.seed, with_dy)


def random_activation_words(rows: int, cols: int, p_nonzero: float, seed: int) -> np.ndarray:
    """bf16 words of a non-negative activation-like matrix: each entry is zero with probability
    1 - p_nonzero, else the square of a half-normal draw (what max(0, z)^2 looks like).  The float32
    draw is truncated to its upper 16 bits, so the words are exact and no rounding rule is involved."""
    rng = np.random.Generator(np.random.Philox(seed))
    z = rng.standard_normal((rows, cols), dtype=np.float32)
    keep = rng.random((rows, cols), dtype=np.float32) < np.float32(p_nonzero)
    h = np.where(keep, z * z, np.float32(0)).astype(np.float32)
    return (h.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def make_inputs_fp8(T: int, D: int, F: int, sparsity, seed: int, sh: float = 16.0 / 448.0) -> dict:
    """fp8 workload: the bf16 recipe's tensors quantised per tensor to OCP e4m3 codes (uint8) with fp32 scales
    s = amax / 448 (so nothing saturates and torch's CPU cast is the plain round-to-nearest-even conversion).
    The activation scale sh is static and handed in: the default puts the format's largest value, 448, at a
    squared-ReLU activation of 16 (pre-activation 4 standard deviations above zero); larger activations saturate."""
    import torch
    inp = make_inputs(T, D, F, sparsity, seed)
    out = {"b1": inp["b1"], "sh": float(sh)}
    for k in ("X", "W1", "W2"):
        s = float(np.abs(inp[k]).max() / 448.0)
        out["s" + k.lower()] = s
        q = torch.from_numpy(inp[k] / np.float32(s)).to(torch.float8_e4m3fn)
        out[k] = q.view(torch.uint8).numpy()
    return out


def make_inputs_fp8_rowwise(T: int, D: int, F: int, sparsity, seed: int, token_corr=None) -> dict:
    """fp8 workload with row-wise scales: X quantised per token row, W1 and W2 per output channel (column), each with
    s = amax / 448 of its row / column (1 where that is zero), by torch's CPU cast.  Returns codes X [T,D], W1 [D,F],
    W2 [F,D] (uint8), scales sx [T], sw1 [F], sw2 [D] (float32) and b1.  token_corr as in make_inputs."""
    import torch
    inp = make_inputs(T, D, F, sparsity, seed, token_corr=token_corr)

    def quant(x, axis):
        amax = np.abs(x).max(axis=axis, keepdims=True).astype(np.float32)
        s = np.where(amax > 0, amax / np.float32(448.0), np.float32(1.0)).astype(np.float32)
        q = torch.from_numpy(np.ascontiguousarray(x / s)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        return q, s.reshape(-1)
    out = {"b1": inp["b1"]}
    out["X"], out["sx"] = quant(inp["X"], 1)
    out["W1"], out["sw1"] = quant(inp["W1"], 0)
    out["W2"], out["sw2"] = quant(inp["W2"], 0)
    return out


def make_bwd_operands_fp8_rowwise(T: int, D: int, F: int, sparsity, seed: int, token_corr=None) -> dict:
    """The operands of the row-wise-scaled fp8 backward for the workload of make_inputs_fp8_rowwise(T, D, F, sparsity, seed):
    dY ~ N(0, 1) (seeded) and the float X, W1, W2 of that workload, each quantised with one scale per index of the
    dimension its backward GEMM does NOT reduce (s = amax / 448 along the reduced one, 1 where that is zero), by torch's CPU cast:
    dY8r, sdy_t (per token);  dY8c, sdy_d and X8c, sx_d (per model dimension);  W2_8r, sw2_f (per hidden feature);
    W1_8c, sw1_d (per model dimension).  Codes are uint8 in the tensors' own layouts ([T,D], [F,D], [D,F])."""
    import torch
    inp = make_inputs(T, D, F, sparsity, seed, with_dy=True, token_corr=token_corr)

    def quant(x, axis):
        amax = np.abs(x).max(axis=axis, keepdims=True).astype(np.float32)
        s = np.where(amax > 0, amax / np.float32(448.0), np.float32(1.0)).astype(np.float32)
        q = torch.from_numpy(np.ascontiguousarray(x / s)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        return q, s.reshape(-1)
    out = {}
    out["dY8r"], out["sdy_t"] = quant(inp["dY"], 1)
    out["dY8c"], out["sdy_d"] = quant(inp["dY"], 0)
    out["X8c"], out["sx_d"] = quant(inp["X"], 0)
    out["W2_8r"], out["sw2_f"] = quant(inp["W2"], 1)
    out["W1_8c"], out["sw1_d"] = quant(inp["W1"], 1)
    return out


def token_permutation(T: int, seed: int) -> np.ndarray:
    """A fixed pseudo-random permutation of the tokens (int32 [T]): position p inside the FFN holds token perm[p]."""
    return np.random.Generator(np.random.Philox(seed)).permutation(T).astype(np.int32)
