"""CPU oracle for the 2:4-activation-sparse Squared-ReLU FFN.  TEST INFRASTRUCTURE ONLY.

This module is the slow, plain definition that the GPU library is checked against.  Only the
tests, the smoke check and the benchmark's cpu_baseline leg may import it; the GPU product
path never does, and this file shares no code with it.

Everything is numpy.  Matrix products are taken in float64 (products of bf16/fp8 operands are
exact there and the summation error is far below the storage precision; stricter than the plain
float32 a CPU reference would need); pointwise steps that decide a pruning pick are taken in the
precision the kernels use (float32 arithmetic followed by round-to-nearest-even to the storage
type), so that a pick depends on the same number on both sides.

What the paper defines, and where (Haziza et al., "Accelerating Transformer Inference and
Training with 2:4 Activation Sparsity"):
  * Squared-ReLU FFN  Y3 = max(0, X1 W1)^2 W2                      -- Sec. 1, "Squared ReLU"
  * 2:4 sparsity: at most 2 non-zeros in every 4 consecutive values -- Sec. 1, "Hardware-accelerated (2:4) sparsity"
  * keep the 2 largest-magnitude scalars of each block of 4 of Y2    -- Sec. 2 (Approach), first paragraph
  * A.B is accelerated when A is 2:4 along the features of a token ("token-wise"),
    A^T.B when A is 2:4 along the tokens of a feature ("feature-wise") -- Fig. 2 caption
  * backward graph: 6 GEMMs, those touching y2 or dy1 are the sparse ones -- Fig. 4 caption
  * the feature-wise picks are made on top of the forward's token-wise mask -- Sec. 2, last paragraph
  * forward order: activation, then sparsification, then FP8 quantisation -- Sec. 2, the paragraph on the two new kernels

Readings where the paper is silent:
  * ties in magnitude go to the lower index; zeros take part like any value, so a group always
    yields exactly two kept slots with i0 < i1;
  * magnitude = the storage word with its sign bit cleared, compared as an unsigned integer;
  * the pick is made on the activation after rounding to the storage type (bf16);
  * metadata: one nibble i0 | (i1 << 2) per group, two groups per byte, even group in the low nibble;
  * a per-feature bias b1 is added before the ReLU (a synthetic sparsity dial; b1 = None is the paper's FFN);
  * one feature-wise mask, ranked on |H24|, is applied to both H24^T and dZ^T;
  * dX uses only the token-wise mask;
  * dZ is rounded to the storage type before the three GEMMs that consume it.

The backward takes the derivative of the activation by its definition, 2 max(0, Z), from the Z of the
oracle's own forward.  A GPU context keeps only the rounded, pruned activation; for checks that start from
such saved tensors, staged_state_from_saved() offers the derivative re-derived from them, 2 sqrt(h), under
that explicit name, and a CPU test bounds its distance from the definition.

Parity pins live in tests/test_oracle_*.py.  Absolute output values for the benchmark shapes have
no external pin (the paper prints none): "parity unpinned" beyond the invariants tested there.
"""
from __future__ import annotations

import numpy as np

# --------------------------------------------------------------------------------------
# storage-type rounding helpers (bf16, OCP fp8 e4m3)
# --------------------------------------------------------------------------------------


def f32_to_bf16_bits(x) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even), returning the 16-bit words.

    NaN maps to a quiet NaN with the sign preserved; infinities stay infinities.
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    r = ((u + np.uint64(0x7FFF) + lsb) >> np.uint64(16)).astype(np.uint32)
    nan = np.isnan(x)
    if nan.any():
        r = np.where(nan, (x.view(np.uint32) >> np.uint32(16)) | np.uint32(0x0040), r)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_bf16(x) -> np.ndarray:
    """float32 -> nearest bf16 value, returned as float32."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x))


_E4M3_MAX = 448.0


def _e4m3_table() -> np.ndarray:
    """Value of each of the 256 OCP e4m3 codes (bias 7, no infinities, S.1111.111 = NaN)."""
    t = np.empty(256, dtype=np.float64)
    for c in range(256):
        s = -1.0 if c & 0x80 else 1.0
        e = (c >> 3) & 0xF
        m = c & 7
        if e == 0xF and m == 7:
            t[c] = np.nan
        elif e == 0:
            t[c] = s * (m / 8.0) * 2.0 ** (-6)
        else:
            t[c] = s * (1.0 + m / 8.0) * 2.0 ** (e - 7)
    return t


E4M3_VALUES = _e4m3_table()


def f32_to_e4m3_bits(x) -> np.ndarray:
    """Saturating round-to-nearest-even conversion float32 -> OCP e4m3 code.

    Finite inputs beyond +-448 clamp to +-448 (codes 0x7E / 0xFE); NaN gives 0x7F | sign.
    Written as a search over the non-negative code values (a 127-entry table), which is the
    definition of round-to-nearest with ties to the even code.
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    a = np.abs(x.astype(np.float64))
    pos = E4M3_VALUES[:0x7F]  # codes 0x00..0x7E, ascending, 0 .. 448
    a_c = np.minimum(a, _E4M3_MAX)
    hi = np.searchsorted(pos, a_c, side="left")  # first code with value >= a
    hi = np.minimum(hi, 0x7E)
    lo = np.maximum(hi - 1, 0)
    d_hi = pos[hi] - a_c
    d_lo = a_c - pos[lo]
    pick_lo = (d_lo < d_hi) | ((d_lo == d_hi) & ((lo & 1) == 0))
    code = np.where(pick_lo, lo, hi).astype(np.uint8)
    code = np.where(np.isnan(x), np.uint8(0x7F), code)
    sign = (x.view(np.uint32) >> np.uint32(31)).astype(np.uint8) << np.uint8(7)
    return (code | sign).astype(np.uint8)


def e4m3_bits_to_f32(b) -> np.ndarray:
    return E4M3_VALUES[np.ascontiguousarray(b, dtype=np.uint8)].astype(np.float32)


def round_e4m3(x) -> np.ndarray:
    return e4m3_bits_to_f32(f32_to_e4m3_bits(x))


# --------------------------------------------------------------------------------------
# 2:4 pruning (Sec. 2, first paragraph: of each group of 4 the two entries of largest magnitude stay)
# --------------------------------------------------------------------------------------

_MAG_MASK = {2: 0x7FFF, 1: 0x7F}


def _as_words(h):
    h = np.ascontiguousarray(h)
    if h.dtype not in (np.uint16, np.uint8):
        raise TypeError("sparsify24 works on storage words: uint16 (bf16) or uint8 (e4m3)")
    return h


def pick24(words: np.ndarray):
    """For storage words of shape [rows, cols] (cols % 4 == 0) return (i0, i1), each [rows, cols/4].

    Inside every group of 4 consecutive columns the entries are ordered by (magnitude descending,
    index ascending); the first two of that order are kept and reported as i0 < i1.
    """
    w = _as_words(words)
    rows, cols = w.shape
    if cols % 4:
        raise ValueError("cols must be a multiple of 4")
    mag = (w & w.dtype.type(_MAG_MASK[w.dtype.itemsize])).astype(np.int64).reshape(rows, cols // 4, 4)
    # stable sort on the negated magnitude = magnitude descending, index ascending among equals
    order = np.argsort(-mag, axis=-1, kind="stable")
    kept = np.sort(order[..., :2], axis=-1)
    return kept[..., 0].astype(np.uint8), kept[..., 1].astype(np.uint8)


def sparsify24(words: np.ndarray):
    """2:4-compress storage words [rows, cols] along the columns.

    Returns (values [rows, cols/2] of the same dtype, meta [rows, cols/8] uint8).
    values[:, 2g], values[:, 2g+1] are the kept entries of group g in index order;
    the nibble of group g is i0 | (i1 << 2), stored in the low half of byte g//2 for even g.
    cols must be a multiple of 8 so that every metadata byte is whole.
    """
    w = _as_words(words)
    rows, cols = w.shape
    if cols % 8:
        raise ValueError("cols must be a multiple of 8")
    i0, i1 = pick24(w)
    g = w.reshape(rows, cols // 4, 4)
    v0 = np.take_along_axis(g, i0[..., None].astype(np.int64), axis=-1)[..., 0]
    v1 = np.take_along_axis(g, i1[..., None].astype(np.int64), axis=-1)[..., 0]
    values = np.stack([v0, v1], axis=-1).reshape(rows, cols // 2)
    nib = (i0 | (i1 << np.uint8(2))).astype(np.uint8)
    meta = (nib[:, 0::2] | (nib[:, 1::2] << np.uint8(4))).astype(np.uint8)
    return values, meta


def unpack_meta(meta: np.ndarray):
    """meta [rows, cols/8] -> (i0, i1) each [rows, cols/4]."""
    meta = np.ascontiguousarray(meta, dtype=np.uint8)
    rows, nb = meta.shape
    nib = np.empty((rows, nb * 2), dtype=np.uint8)
    nib[:, 0::2] = meta & 0xF
    nib[:, 1::2] = meta >> 4
    return nib & 3, (nib >> 2) & 3


def mask_from_meta(meta: np.ndarray) -> np.ndarray:
    """Boolean keep-mask [rows, cols] described by the metadata."""
    i0, i1 = unpack_meta(meta)
    rows, ng = i0.shape
    m = np.zeros((rows, ng, 4), dtype=bool)
    np.put_along_axis(m, i0[..., None].astype(np.int64), True, axis=-1)
    np.put_along_axis(m, i1[..., None].astype(np.int64), True, axis=-1)
    return m.reshape(rows, ng * 4)


def decompress24(values: np.ndarray, meta: np.ndarray) -> np.ndarray:
    """Inverse of sparsify24 on the kept entries: a dense [rows, cols] array with zeros elsewhere."""
    i0, i1 = unpack_meta(meta)
    rows, ng = i0.shape
    v = np.ascontiguousarray(values).reshape(rows, ng, 2)
    out = np.zeros((rows, ng, 4), dtype=v.dtype)
    np.put_along_axis(out, i0[..., None].astype(np.int64), v[..., 0:1], axis=-1)
    np.put_along_axis(out, i1[..., None].astype(np.int64), v[..., 1:2], axis=-1)
    return out.reshape(rows, ng * 4)


def compress_with_meta(dense: np.ndarray, meta: np.ndarray) -> np.ndarray:
    """Gather the entries of `dense` [rows, cols] at the positions the metadata names -> [rows, cols/2]."""
    i0, i1 = unpack_meta(meta)
    rows, ng = i0.shape
    g = np.ascontiguousarray(dense).reshape(rows, ng, 4)
    v0 = np.take_along_axis(g, i0[..., None].astype(np.int64), axis=-1)[..., 0]
    v1 = np.take_along_axis(g, i1[..., None].astype(np.int64), axis=-1)[..., 0]
    return np.stack([v0, v1], axis=-1).reshape(rows, ng * 2)


def gather_matmul24(values_f: np.ndarray, meta: np.ndarray, B: np.ndarray) -> np.ndarray:
    """(compressed A) . B computed straight from (values, metadata): for each kept entry,
    add value * B[4*group + index, :].  float64.  Must equal decompress24(...) @ B (Fig. 2)."""
    i0, i1 = unpack_meta(meta)
    rows, ng = i0.shape
    v = np.asarray(values_f, dtype=np.float64).reshape(rows, ng, 2)
    B = np.asarray(B, dtype=np.float64)
    base = (4 * np.arange(ng, dtype=np.int64))[None, :]
    k0 = base + i0.astype(np.int64)
    k1 = base + i1.astype(np.int64)
    out = np.zeros((rows, B.shape[1]), dtype=np.float64)
    for r in range(rows):
        out[r] = v[r, :, 0] @ B[k0[r]] + v[r, :, 1] @ B[k1[r]]
    return out


# --------------------------------------------------------------------------------------
# quantisers
# --------------------------------------------------------------------------------------


class Bf16:
    """Storage type bf16: q() rounds float32 to the nearest bf16 value; words()/from_words() expose the bits."""

    name = "bf16"

    @staticmethod
    def q(x):
        return round_bf16(np.asarray(x, dtype=np.float32))

    @staticmethod
    def words(x):
        return f32_to_bf16_bits(np.asarray(x, dtype=np.float32))

    @staticmethod
    def from_words(w):
        return bf16_bits_to_f32(w)


class Exact:
    """No storage rounding (used to pin the calculus against finite differences); words() are the
    bf16 bits of the value, which is lossless for the small-integer test inputs it is used with."""

    name = "exact"

    @staticmethod
    def q(x):
        return np.asarray(x, dtype=np.float64)

    words = staticmethod(Bf16.words)
    from_words = staticmethod(Bf16.from_words)


# --------------------------------------------------------------------------------------
# forward
# --------------------------------------------------------------------------------------


def _preact(X, W1, b1, st):
    Xq = st.q(X).astype(np.float64)
    W1q = st.q(W1).astype(np.float64)
    Z = Xq @ W1q
    if b1 is not None:
        Z = Z + np.asarray(b1, dtype=np.float64)[None, :]
    return Xq, W1q, Z


def _relu2(Z, st):
    """R = max(0, Z), H = R^2.  With a storage type the two pointwise steps run in float32, as the kernels do."""
    if st is Exact:
        R = np.maximum(Z, 0.0)
        return R, R * R
    Z32 = Z.astype(np.float32)
    R32 = np.maximum(Z32, np.float32(0))
    H32 = R32 * R32
    return R32, H32


def ffn_fwd(X, W1, b1, W2, st=Bf16):
    """Dense Squared-ReLU FFN (Sec. 1): Y = max(0, X W1 + b1)^2 W2, with H stored in the storage type."""
    Xq, W1q, Z = _preact(X, W1, b1, st)
    R, H = _relu2(Z, st)
    Hq = st.q(H)
    W2q = st.q(W2).astype(np.float64)
    Y = Hq.astype(np.float64) @ W2q
    return {"Z": Z, "R": R, "Rq": st.q(R), "Hq": Hq, "Y": Y, "Xq": Xq, "W1q": W1q, "W2q": W2q, "dAct": relu2_derivative(Z)}


def ffn24_fwd(X, W1, b1, W2, st=Bf16):
    """Squared-ReLU FFN whose second GEMM sees the 2:4-pruned activation (Sec. 2, first paragraph).

    Steps: Z = X W1 + b1;  H = max(0, Z)^2;  Hq = storage rounding of H;  per token and per group of
    4 consecutive features keep the top-2 of |Hq| (ties -> lower index);  Y = H24 W2.
    """
    Xq, W1q, Z = _preact(X, W1, b1, st)
    R, H = _relu2(Z, st)
    Hq = st.q(H)
    Hw = st.words(Hq)
    Hc_w, meta = sparsify24(Hw)
    Mtok = mask_from_meta(meta)
    H24 = np.where(Mtok, Hq, Hq.dtype.type(0))
    W2q = st.q(W2).astype(np.float64)
    Y = H24.astype(np.float64) @ W2q
    Rq = st.q(R)
    return {
        "Z": Z, "R": R, "Rq": Rq, "Hq": Hq, "H_words": Hw, "Hc_words": Hc_w, "meta": meta, "Mtok": Mtok,
        "H24": H24, "Hc": compress_with_meta(Hq, meta), "Rc": compress_with_meta(Rq, meta),
        "Y": Y, "Xq": Xq, "W1q": W1q, "W2q": W2q, "dAct": relu2_derivative(Z),
    }


# --------------------------------------------------------------------------------------
# backward
# --------------------------------------------------------------------------------------


def featurewise24(H24, st=Bf16):
    """2:4 picks along the tokens of each feature, made on the already token-wise-pruned H24
    (Sec. 2, last paragraph).  H24 is [T, F]; the same top-2 rule runs on H24^T [F, T] in groups of
    4 consecutive tokens.  Returns (Hc_t words [F, T/2], meta_t [F, T/8], M_T bool [T, F])."""
    Ht_words = st.words(np.ascontiguousarray(np.asarray(H24).T))
    Hc_t, meta_t = sparsify24(Ht_words)
    M_T = mask_from_meta(meta_t).T
    return Hc_t, meta_t, M_T


def relu2_derivative(Z) -> np.ndarray:
    """d/dz max(0, z)^2 = 2 max(0, z) (Fig. 4 caption: the backward graph of the Squared-ReLU FFN), float64."""
    return 2.0 * np.maximum(np.asarray(Z, dtype=np.float64), 0.0)


def relu2_derivative_from_stored_activation(Hq) -> np.ndarray:
    """The same derivative re-derived from a stored activation h = round(max(0, z)^2):  2 sqrt(h).
    NOT the definition: it differs from 2 max(0, z) by the storage rounding of h (relative 2^-9 for bf16, halved by
    the square root).  Only for checks that start from tensors a context saved, which no longer include Z."""
    return 2.0 * np.sqrt(np.asarray(Hq, dtype=np.float64))


def staged_state_from_saved(Hc_words, meta, X, W1, W2, st=Bf16):
    """Forward state rebuilt from the compressed activation (Hc words, metadata) that a forward pass saved, for
    staged checks of a backward pass on exactly those tensors.  Same keys as ffn24_fwd's result as far as ffn24_bwd
    reads them; dAct is relu2_derivative_from_stored_activation of the saved activation (see there)."""
    H24 = st.from_words(decompress24(np.asarray(Hc_words, dtype=np.uint16), meta))
    return {"H24": H24, "meta": np.asarray(meta, dtype=np.uint8), "Mtok": mask_from_meta(meta),
            "dAct": relu2_derivative_from_stored_activation(H24),
            "Xq": st.q(X).astype(np.float64), "W1q": st.q(W1).astype(np.float64), "W2q": st.q(W2).astype(np.float64)}


def dz_tokenwise(fwd: dict, dY, st=Bf16):
    """dH = dY W2^T;  dZ = dH * dAct on the positions the token-wise mask kept, zero elsewhere;  rounded to the storage
    type (Fig. 4 caption; Sec. 2, last paragraph).  Returns (dH, dZq).  Needs of `fwd`: W2q, dAct, Mtok."""
    dYq = st.q(dY).astype(np.float64)
    dH = dYq @ fwd["W2q"].T
    dZ = np.where(fwd["Mtok"], dH * fwd["dAct"], 0.0)
    return dH, st.q(dZ)


def feature_nnz(Hq) -> np.ndarray:
    """Column-level statistic of Sec. 2, "Optimization 1": for every hidden feature the number of tokens whose
    (storage-rounded, not yet pruned) activation is non-zero -- what the first GEMM's epilogue can count for free."""
    return np.count_nonzero(np.asarray(Hq), axis=0).astype(np.int64)


def split_features(nnz, n_dense: int) -> np.ndarray:
    """Partition of the features for the split weight-gradient GEMMs (Sec. 2, "Optimization 1"): the n_dense
    least sparse features (largest non-zero count; ties -> lower feature index) are kept dense, the rest is
    2:4-sparsified along tokens.  Returns a boolean array [F], True = dense feature.  (The paper sorts with an
    argsort kernel and takes 5 %; the count is a parameter here.)"""
    nnz = np.asarray(nnz, dtype=np.int64)
    F = nnz.shape[0]
    if not 0 <= n_dense <= F:
        raise ValueError("n_dense out of range")
    order = np.argsort(-nnz, kind="stable")        # count descending, index ascending among equals
    dense = np.zeros(F, dtype=bool)
    dense[order[:n_dense]] = True
    return dense


def ffn24_bwd(fwd: dict, dY, st=Bf16, wgrad_mask="featurewise", dense_features=None):
    """Backward of ffn24_fwd with the masks held fixed (Fig. 4 caption; Sec. 2, backward paragraphs).

      dH  = dY W2^T                                  (dense)
      dZ  = dH * 2 max(0, Z) * M_tok                  (ReLU^2 derivative on the kept positions; stored rounded)
      dX  = dZ W1^T                                  (sparse along features: token-wise mask only)
      dW2 = (H24 * M_T)^T dY,  dW1 = X^T (dZ * M_T)   (sparse along tokens: feature-wise mask on top)

    Needs of `fwd` only H24, meta, Mtok, dAct (= 2 max(0, Z) of the forward's own Z), Xq, W1q, W2q.
    wgrad_mask="tokenwise" replaces M_T by M_tok in the
    last line: the exact gradient of the pruned forward, used only to pin the calculus.
    dense_features (bool [F], optional): the split of Sec. 2, "Optimization 1" -- for these features the weight
    gradients use the token-wise mask only (a dense GEMM over them), for all others the feature-wise mask on top.
    """
    dYq = st.q(dY).astype(np.float64)
    Mtok = fwd["Mtok"]
    dH, dZq = dz_tokenwise(fwd, dY, st)
    dX = dZq.astype(np.float64) @ fwd["W1q"].T
    Hc_t, meta_t, M_T = featurewise24(fwd["H24"], st)
    Mw = M_T if wgrad_mask == "featurewise" else Mtok
    if dense_features is not None:
        Mw = np.where(np.asarray(dense_features, dtype=bool)[None, :], Mtok, Mw)
    H24m = np.where(Mw, fwd["H24"], fwd["H24"].dtype.type(0)).astype(np.float64)
    dZm = np.where(Mw, dZq, dZq.dtype.type(0)).astype(np.float64)
    dW2 = H24m.T @ dYq
    dW1 = fwd["Xq"].T @ dZm
    dZc_t = compress_with_meta(np.ascontiguousarray(dZq.T), meta_t)
    return {
        "dH": dH, "dZq": dZq, "dZc": compress_with_meta(dZq, fwd["meta"]), "dX": dX, "dW1": dW1, "dW2": dW2,
        "Hc_t_words": Hc_t, "meta_t": meta_t, "M_T": M_T, "dZc_t": dZc_t,
    }


def ffn24_fwd_bwd_permuted(X, W1, b1, W2, dY, perm, st=Bf16, wgrad_mask="featurewise", dense_features=None):
    """Forward + backward with a fixed token permutation around the FFN (Sec. 2, "Optimization 2": permute the tokens
    before entering the FFN and shuffle them back after).  Position p inside the FFN holds token perm[p]: the FFN runs
    on X[perm] and dY[perm]; Y and dX are scattered back to token order; the weight gradients are sums over tokens and
    keep their layout, but their feature-wise 2:4 groups are now made of the tokens the permutation puts side by side."""
    perm = np.asarray(perm, dtype=np.int64)
    T = np.asarray(X).shape[0]
    if sorted(perm.tolist()) != list(range(T)):
        raise ValueError("perm is not a permutation of the tokens")
    f = ffn24_fwd(np.asarray(X)[perm], W1, b1, W2, st)
    g = ffn24_bwd(f, np.asarray(dY)[perm], st, wgrad_mask, dense_features)
    Y = np.empty_like(f["Y"]); Y[perm] = f["Y"]
    dX = np.empty_like(g["dX"]); dX[perm] = g["dX"]
    return {"fwd": f, "bwd": g, "Y": Y, "dX": dX, "dW1": g["dW1"], "dW2": g["dW2"]}


def featurewise_drop_fraction(H24, M_T) -> float:
    """Fraction of the non-zero entries of the token-wise-pruned activation that the feature-wise 2:4 drops."""
    nz = np.asarray(H24) != 0
    return float((nz & ~np.asarray(M_T, dtype=bool)).sum() / max(1, nz.sum()))


def sparsity_counts(Hq, H24=None, M_T=None, dense_features=None) -> dict:
    """The counts behind the paper's sparsity figures (Sec. 1, the sparsity-level figure; Sec. 2, first paragraph: the share
    of non-zero values that 2:4 drops), for one FFN call:
      elements        T F
      nonzero         non-zero entries of the stored activation H
      kept_tokenwise  of those, the entries that survive the token-wise 2:4 (None for a dense forward)
      kept_featurewise  of those, the entries the weight-gradient GEMMs still see: the feature-wise 2:4 on top, except
                        on `dense_features` (Sec. 2, "Optimization 1"), which keep the token-wise set (None without M_T)
    """
    Hq = np.asarray(Hq)
    out = {"elements": int(Hq.size), "nonzero": int(np.count_nonzero(Hq)), "kept_tokenwise": None, "kept_featurewise": None}
    if H24 is not None:
        H24 = np.asarray(H24)
        out["kept_tokenwise"] = int(np.count_nonzero(H24))
        if M_T is not None:
            Mw = np.asarray(M_T, dtype=bool)
            if dense_features is not None:
                Mw = Mw | np.asarray(dense_features, dtype=bool)[None, :]
            out["kept_featurewise"] = int(np.count_nonzero(np.where(Mw, H24, H24.dtype.type(0))))
    return out


def use_sparse_path(counts: dict, min_sparsity: float) -> bool:
    """The dense <-> 2:4 switch behind the paper's dense warm-up (Sec. 2, last paragraph: training starts dense because
    the activation is only about half zeros at initialisation, and 2:4 is switched on once it is sparse enough): run
    the 2:4 path iff the measured share of zeros, 1 - nonzero / elements, has reached min_sparsity."""
    return (1.0 - counts["nonzero"] / counts["elements"]) >= min_sparsity


def ffn_bwd(fwd: dict, dY, st=Bf16):
    """Textbook backward of the dense FFN: dZ = (dY W2^T) * 2 max(0, Z); dX = dZ W1^T; dW2 = H^T dY; dW1 = X^T dZ.
    Needs of `fwd` only Hq, dAct (= 2 max(0, Z) of the forward's own Z), Xq, W1q, W2q."""
    dYq = st.q(dY).astype(np.float64)
    dH = dYq @ fwd["W2q"].T
    dZq = st.q(dH * fwd["dAct"])
    dX = dZq.astype(np.float64) @ fwd["W1q"].T
    dW2 = np.asarray(fwd["Hq"], dtype=np.float64).T @ dYq
    dW1 = fwd["Xq"].T @ dZq.astype(np.float64)
    return {"dZq": dZq, "dX": dX, "dW1": dW1, "dW2": dW2}


# --------------------------------------------------------------------------------------
# fp8 forward (order of Sec. 2: activation, sparsification, then FP8 quantisation)
# --------------------------------------------------------------------------------------


def ffn24_fwd_fp8_codes(X8, W1_8, b1, W2_8, sx, sw1, sh, sw2):
    """The fp8 forward on operands that are already e4m3 codes (uint8): X8 [T,D], W1_8 [D,F], W2_8 [F,D].
    Z = sx sw1 (X8 W1_8) + b1;  the 2:4 pick is made on bf16(H) exactly as in ffn24_fwd;  the kept values are then
    quantised, Hc8 = e4m3(Hc / sh);  Y = sh sw2 (Hc8 . W2_8)."""
    Xq = E4M3_VALUES[np.ascontiguousarray(X8, dtype=np.uint8)]
    W1q = E4M3_VALUES[np.ascontiguousarray(W1_8, dtype=np.uint8)]
    Z = (Xq @ W1q) * (float(sx) * float(sw1))
    if b1 is not None:
        Z = Z + np.asarray(b1, dtype=np.float64)[None, :]
    R, H = _relu2(Z, Bf16)
    Hq = round_bf16(H)
    Hc_w, meta = sparsify24(f32_to_bf16_bits(Hq))
    Hc = bf16_bits_to_f32(Hc_w)
    Hc8_bits = f32_to_e4m3_bits(Hc / np.float32(sh))
    Hc8 = E4M3_VALUES[Hc8_bits]
    W2q = E4M3_VALUES[np.ascontiguousarray(W2_8, dtype=np.uint8)]
    H24_8 = decompress24(Hc8, meta)
    Y = (H24_8 @ W2q) * (float(sh) * float(sw2))
    return {"Z": Z, "Hq": Hq, "meta": meta, "Hc8_bits": Hc8_bits, "Y": Y}


def ffn24_fwd_fp8(X, W1, b1, W2, sx, sw1, sh, sw2):
    """Per-tensor-scaled e4m3 variant (order of Sec. 2: activation, sparsification, then FP8 quantisation).
    Xq = e4m3(X / sx), W1q = e4m3(W1 / sw1), W2q = e4m3(W2 / sw2), then ffn24_fwd_fp8_codes."""
    X8 = f32_to_e4m3_bits(np.asarray(X, np.float32) / np.float32(sx))
    W1_8 = f32_to_e4m3_bits(np.asarray(W1, np.float32) / np.float32(sw1))
    W2_8 = f32_to_e4m3_bits(np.asarray(W2, np.float32) / np.float32(sw2))
    return ffn24_fwd_fp8_codes(X8, W1_8, b1, W2_8, sx, sw1, sh, sw2)


def ffn24_bwd_fp8_codes(fwd, X8, W1_8, W2_8, dY8, sx, sw1, sh, sw2, sdy, sdz, wgrad_mask="featurewise", quantise_dz=True, dAct=None):
    """Backward of ffn24_fwd_fp8_codes with every GEMM operand in e4m3 (abstract: FP8 "in both the forwards and backwards
    pass"; Sec. 2, the paragraph on the fused backward pointwise kernel: it includes the FP8 scaling).  Per-tensor scales.
      dY8 [T,D] codes with scale sdy;  fwd = the result of ffn24_fwd_fp8_codes on the same X8, W1_8, W2_8 and scales.
      dH  = sdy sw2 (dY8 . W2_8^T)
      dZ  = dH * 2 max(0, Z) on the positions the token-wise mask kept (Fig. 4 caption), Z = the forward's own
      dZ8 = e4m3(dZ / sdz), saturating, stored compressed with the forward's metadata
      dX  = sdz sw1 (dZ8 . W1_8^T)                                       (token-wise mask only)
      feature-wise picks on top of the token-wise mask (Sec. 2, last paragraph), ranked on the stored activation's
      codes H24_8 (the e4m3 words with the sign cleared, as integers; ties -> lower token), one mask for H and dZ
      dW2 = sh sdy ((H24_8 * M_T)^T . dY8);   dW1 = sx sdz (X8^T . (dZ8 * M_T))
    Switches for pinning only: wgrad_mask="tokenwise" uses M_tok in the last line; quantise_dz=False keeps dZ / sdz
    unrounded.  dAct (optional) replaces 2 max(0, Z) for checks that start from a context's saved tensors."""
    Xv = E4M3_VALUES[np.ascontiguousarray(X8, dtype=np.uint8)]
    W1v = E4M3_VALUES[np.ascontiguousarray(W1_8, dtype=np.uint8)]
    W2v = E4M3_VALUES[np.ascontiguousarray(W2_8, dtype=np.uint8)]
    dYv = E4M3_VALUES[np.ascontiguousarray(dY8, dtype=np.uint8)]
    meta = np.asarray(fwd["meta"], dtype=np.uint8)
    Mtok = mask_from_meta(meta)
    dH = (dYv @ W2v.T) * (float(sdy) * float(sw2))
    dA = relu2_derivative(fwd["Z"]) if dAct is None else np.asarray(dAct, dtype=np.float64)
    dZ = np.where(Mtok, dH * dA, 0.0)
    if quantise_dz:
        dZ8_bits = f32_to_e4m3_bits((dZ / float(sdz)).astype(np.float32))
        dZ8v = E4M3_VALUES[dZ8_bits]
    else:
        dZ8_bits = None
        dZ8v = dZ / float(sdz)
    dX = (dZ8v @ W1v.T) * (float(sdz) * float(sw1))
    H24_bits = decompress24(np.asarray(fwd["Hc8_bits"], dtype=np.uint8), meta)
    Hc8_t, meta_t = sparsify24(np.ascontiguousarray(H24_bits.T))
    M_T = mask_from_meta(meta_t).T
    Mw = M_T if wgrad_mask == "featurewise" else Mtok
    H24v = E4M3_VALUES[H24_bits]
    dW2 = (np.where(Mw, H24v, 0.0).T @ dYv) * (float(sh) * float(sdy))
    dW1 = (Xv.T @ np.where(Mw, dZ8v, 0.0)) * (float(sx) * float(sdz))
    out = {"dH": dH, "dZ": dZ, "dX": dX, "dW1": dW1, "dW2": dW2, "Hc8_t_bits": Hc8_t, "meta_t": meta_t, "M_T": M_T, "Mtok": Mtok}
    if quantise_dz:
        out["dZ8_bits"] = dZ8_bits
        out["dZc8_bits"] = compress_with_meta(dZ8_bits, meta)
        out["dZc8_t_bits"] = compress_with_meta(np.ascontiguousarray(dZ8_bits.T), meta_t)
    return out


def ffn_fwd_fp8_codes(X8, W1_8, b1, W2_8, sx, sw1, sh, sw2):
    """ffn_fwd_fp8 on operands that are already e4m3 codes; also returns Z for the backward."""
    Xq = E4M3_VALUES[np.ascontiguousarray(X8, dtype=np.uint8)]
    W1q = E4M3_VALUES[np.ascontiguousarray(W1_8, dtype=np.uint8)]
    Z = (Xq @ W1q) * (float(sx) * float(sw1))
    if b1 is not None:
        Z = Z + np.asarray(b1, dtype=np.float64)[None, :]
    R, H = _relu2(Z, Bf16)
    Hq = round_bf16(H)
    H8_bits = f32_to_e4m3_bits(Hq / np.float32(sh))
    W2q = E4M3_VALUES[np.ascontiguousarray(W2_8, dtype=np.uint8)]
    Y = (E4M3_VALUES[H8_bits] @ W2q) * (float(sh) * float(sw2))
    return {"Z": Z, "Hq": Hq, "H8_bits": H8_bits, "Y": Y}


def ffn_bwd_fp8_codes(fwd, X8, W1_8, W2_8, dY8, sx, sw1, sh, sw2, sdy, sdz, quantise_dz=True, dAct=None):
    """Dense counterpart of ffn24_bwd_fp8_codes (no masks): the textbook backward of the dense FFN with every GEMM operand
    in e4m3.  dH = sdy sw2 (dY8 . W2_8^T);  dZ8 = e4m3(dH * 2 max(0, Z) / sdz);  dX = sdz sw1 (dZ8 . W1_8^T);
    dW2 = sh sdy (H8^T . dY8);  dW1 = sx sdz (X8^T . dZ8).  fwd = the result of ffn_fwd_fp8_codes."""
    Xv = E4M3_VALUES[np.ascontiguousarray(X8, dtype=np.uint8)]
    W1v = E4M3_VALUES[np.ascontiguousarray(W1_8, dtype=np.uint8)]
    W2v = E4M3_VALUES[np.ascontiguousarray(W2_8, dtype=np.uint8)]
    dYv = E4M3_VALUES[np.ascontiguousarray(dY8, dtype=np.uint8)]
    dH = (dYv @ W2v.T) * (float(sdy) * float(sw2))
    dZ = dH * (relu2_derivative(fwd["Z"]) if dAct is None else np.asarray(dAct, dtype=np.float64))
    if quantise_dz:
        dZ8_bits = f32_to_e4m3_bits((dZ / float(sdz)).astype(np.float32))
        dZ8v = E4M3_VALUES[dZ8_bits]
    else:
        dZ8_bits, dZ8v = None, dZ / float(sdz)
    dX = (dZ8v @ W1v.T) * (float(sdz) * float(sw1))
    dW2 = (E4M3_VALUES[np.asarray(fwd["H8_bits"], dtype=np.uint8)].T @ dYv) * (float(sh) * float(sdy))
    dW1 = (Xv.T @ dZ8v) * (float(sx) * float(sdz))
    return {"dH": dH, "dZ": dZ, "dZ8_bits": dZ8_bits, "dX": dX, "dW1": dW1, "dW2": dW2}


def ffn24_fwd_fp8_rowwise_codes(X8, sx, W1_8, sw1, b1, W2_8, sw2):
    """fp8 forward with row-wise scaling (the paper's precision recipe, Sec. 2: "FP8 rowwise scaling"): the
    activation operand of each GEMM carries one scale per token row, the weight operand one per output channel.
      X8 [T,D] codes, sx [T];  W1_8 [D,F] codes, sw1 [F];  W2_8 [F,D] codes, sw2 [D]
      Z[t,f] = sx[t] sw1[f] (X8 W1_8)[t,f] + b1[f];  H = bf16(max(0,Z)^2);  2:4 pick on the bf16 words;
      sh[t] = max_f H24[t,f] / 448 (1 if the row is all zero), computed in float32;  Hc8 = e4m3(Hc / sh[t]);
      Y[t,d] = sh[t] sw2[d] (Hc8 . W2_8)[t,d]."""
    Xq = E4M3_VALUES[np.ascontiguousarray(X8, dtype=np.uint8)]
    W1q = E4M3_VALUES[np.ascontiguousarray(W1_8, dtype=np.uint8)]
    sx = np.asarray(sx, dtype=np.float32); sw1 = np.asarray(sw1, dtype=np.float32); sw2 = np.asarray(sw2, dtype=np.float32)
    Z = (Xq @ W1q) * sx.astype(np.float64)[:, None] * sw1.astype(np.float64)[None, :]
    if b1 is not None:
        Z = Z + np.asarray(b1, dtype=np.float64)[None, :]
    R, H = _relu2(Z, Bf16)
    Hq = round_bf16(H)
    Hc_w, meta = sparsify24(f32_to_bf16_bits(Hq))
    Hc = bf16_bits_to_f32(Hc_w)
    rowmax = Hc.max(axis=1).astype(np.float32)                      # the largest entry of a group is always kept
    sh = np.where(rowmax > 0, rowmax / np.float32(448.0), np.float32(1.0)).astype(np.float32)
    Hc8_bits = f32_to_e4m3_bits(Hc / sh[:, None])
    W2q = E4M3_VALUES[np.ascontiguousarray(W2_8, dtype=np.uint8)]
    Y = (decompress24(E4M3_VALUES[Hc8_bits], meta) @ W2q) * sh.astype(np.float64)[:, None] * sw2.astype(np.float64)[None, :]
    return {"Z": Z, "Hq": Hq, "meta": meta, "Hc_words": Hc_w, "rowmax": rowmax, "sh": sh, "Hc8_bits": Hc8_bits, "Y": Y}


def ffn_fwd_fp8_rowwise_codes(X8, sx, W1_8, sw1, b1, W2_8, sw2):
    """Dense counterpart of ffn24_fwd_fp8_rowwise_codes (no pruning): the baseline of the paper's forward benchmark, whose
    FP8 GEMMs use row-wise scaling on both sides (caption of the forward-speed-up figure).  Every activation is stored:
    sh[t] = max_f H[t,f] / 448 (1 for an all-zero row);  H8 = e4m3(bf16(H) / sh[t]);  Y = sh[t] sw2[d] (H8 . W2_8)."""
    Xq = E4M3_VALUES[np.ascontiguousarray(X8, dtype=np.uint8)]
    W1q = E4M3_VALUES[np.ascontiguousarray(W1_8, dtype=np.uint8)]
    sx = np.asarray(sx, dtype=np.float32); sw1 = np.asarray(sw1, dtype=np.float32); sw2 = np.asarray(sw2, dtype=np.float32)
    Z = (Xq @ W1q) * sx.astype(np.float64)[:, None] * sw1.astype(np.float64)[None, :]
    if b1 is not None:
        Z = Z + np.asarray(b1, dtype=np.float64)[None, :]
    R, H = _relu2(Z, Bf16)
    Hq = round_bf16(H)
    rowmax = Hq.max(axis=1).astype(np.float32)
    sh = np.where(rowmax > 0, rowmax / np.float32(448.0), np.float32(1.0)).astype(np.float32)
    H8_bits = f32_to_e4m3_bits(Hq / sh[:, None])
    W2q = E4M3_VALUES[np.ascontiguousarray(W2_8, dtype=np.uint8)]
    Y = (E4M3_VALUES[H8_bits] @ W2q) * sh.astype(np.float64)[:, None] * sw2.astype(np.float64)[None, :]
    return {"Z": Z, "Hq": Hq, "sh": sh, "H8_bits": H8_bits, "Y": Y}


def ffn24_bwd_fp8_rowwise_codes(fwd, dY8r, sdy_t, W2_8r, sw2_f, W1_8c, sw1_d, dY8c, sdy_d, X8c, sx_d, wgrad_mask="featurewise", quantise_internal=True,
                                dense_features=None):
    """Backward of ffn24_fwd_fp8_rowwise_codes with row-wise scaling in every GEMM (the paper's precision recipe: the caption
    of the forward-speed-up figure has all FP8 matrix multiplications row-wise scaled; Sec. 2, the paragraph on the fused
    backward pointwise kernel: it includes the transposition and the FP8 scaling).  Row-wise scaling of a GEMM: each operand
    carries one scale per index of its non-reduced dimension, so the tensors that enter two GEMMs with different reduced
    dimensions are quantised twice, by the caller (from its higher-precision copies):
      dY8r [T,D] codes, sdy_t [T]: dY quantised per token (reduced over d in the dH GEMM)
      dY8c [T,D] codes, sdy_d [D]: dY quantised per model dimension (reduced over t in the dW2 GEMM)
      W2_8r [F,D] codes, sw2_f [F]: W2 quantised per hidden feature (dH GEMM);  W1_8c [D,F] codes, sw1_d [D]: W1 per model
      dimension (dX GEMM);  X8c [T,D] codes, sx_d [D]: X per model dimension (dW1 GEMM)
    and the tensors the backward makes itself are quantised where they are made, each scale = the largest magnitude / 448 in
    float32 (1 if all zero), as the forward does for the activation:
      dH[t,f] = sdy_t[t] sw2_f[f] (dY8r . W2_8r^T)[t,f]
      dZ      = bf16( dH * 2 max(0, Z) ) on the positions the token-wise mask kept (Fig. 4 caption), 0 elsewhere
      sdz_t[t] = max_f |dZ[t,f]| / 448;  dZ8r = e4m3(dZ / sdz_t[t]);   dX[t,d] = sdz_t[t] sw1_d[d] (dZ8r . W1_8c^T)[t,d]
      feature-wise picks on top of the token-wise mask (Sec. 2, last paragraph), ranked on the bf16 activation H24 as in
      ffn24_bwd (quantisation comes after the pick, as in the forward), one mask M_T for H and dZ
      the two transposed operands are quantised as they enter their GEMMs, i.e. after the second mask:
      sh_f[f] = max_t (H24 * M_T)[t,f] / 448;  H8c = e4m3(H24 * M_T / sh_f[f])   (the largest entry of a column always survives M_T)
      sdz_f[f] = max_t |(dZ * M_T)[t,f]| / 448;  dZ8c = e4m3(dZ * M_T / sdz_f[f])
      dW2[f,d] = sh_f[f] sdy_d[d] (H8c^T . dY8c)[f,d];   dW1[d,f] = sx_d[d] sdz_f[f] (X8c^T . dZ8c)[d,f]
    dense_features (bool [F], optional): the split of Sec. 2, "Optimization 1", as in ffn24_bwd -- for these features the two
    weight gradients use the token-wise mask only (their rows of the transposed operands stay dense and go through a dense
    GEMM), for all others the feature-wise mask on top; either way a feature's row is quantised with its own scale, taken
    over whatever of the row enters the GEMM.
    fwd = the result of ffn24_fwd_fp8_rowwise_codes.  Switches for pinning only: wgrad_mask="tokenwise" uses the token-wise
    mask in the last line; quantise_internal=False leaves dZ and H24 unrounded (neither bf16 nor e4m3) in all three GEMMs."""
    dec = lambda c: E4M3_VALUES[np.ascontiguousarray(c, dtype=np.uint8)]
    f64 = lambda v: np.asarray(v, dtype=np.float32).astype(np.float64)
    meta = np.asarray(fwd["meta"], dtype=np.uint8)
    Mtok = mask_from_meta(meta)
    dH = (dec(dY8r) @ dec(W2_8r).T) * f64(sdy_t)[:, None] * f64(sw2_f)[None, :]
    dZ = np.where(Mtok, dH * relu2_derivative(fwd["Z"]), 0.0)
    H24 = decompress24(bf16_bits_to_f32(np.asarray(fwd["Hc_words"], dtype=np.uint16)), meta)
    _, meta_t, M_T = featurewise24(H24)
    Mw = M_T if wgrad_mask == "featurewise" else Mtok
    if dense_features is not None:
        Mw = np.where(np.asarray(dense_features, dtype=bool)[None, :], Mtok, Mw)
    out = {"dH": dH, "Mtok": Mtok, "M_T": M_T, "meta_t": meta_t}
    if quantise_internal:
        dZ16 = round_bf16(dZ)
        dZ8r_bits, sdz_t = quantise_rows_e4m3(dZ16)
        dZ8c_bits_t, sdz_f = quantise_rows_e4m3(np.ascontiguousarray(np.where(Mw, dZ16, np.float32(0)).T))
        H8c_bits_t, sh_f = quantise_rows_e4m3(np.ascontiguousarray(np.where(Mw, H24, np.float32(0)).T))
        dZr = dec(dZ8r_bits) * sdz_t.astype(np.float64)[:, None]
        dZc = dec(dZ8c_bits_t).T * sdz_f.astype(np.float64)[None, :]
        Hc = dec(H8c_bits_t).T * sh_f.astype(np.float64)[None, :]
        out.update({"dZ16": dZ16, "sdz_t": sdz_t, "sdz_f": sdz_f, "sh_f": sh_f, "dZ8r_bits": dZ8r_bits,
                    "dZc8r_bits": compress_with_meta(dZ8r_bits, meta),
                    "Hc8_t_bits": compress_with_meta(H8c_bits_t, meta_t), "dZc8_t_bits": compress_with_meta(dZ8c_bits_t, meta_t),
                    "H8_t_bits": H8c_bits_t, "dZ8_t_bits": dZ8c_bits_t})
    else:
        dZr = dZc = dZ
        Hc = H24.astype(np.float64)
    out["dZ"] = dZ
    out["dX"] = (dZr @ dec(W1_8c).T) * f64(sw1_d)[None, :]
    out["dW2"] = (np.where(Mw, Hc, 0.0).T @ dec(dY8c)) * f64(sdy_d)[None, :]
    out["dW1"] = (dec(X8c).T * f64(sx_d)[:, None]) @ np.where(Mw, dZc, 0.0)
    return out


def ffn24_fwd_bwd_fp8_rowwise_permuted(X8, sx, W1_8, sw1, b1, W2_8, sw2, bw: dict, perm, wgrad_mask="featurewise", dense_features=None):
    """Row-wise fp8 forward + backward with the fixed token permutation of Sec. 2, "Optimization 2" around the FFN, as
    ffn24_fwd_bwd_permuted does it for bf16: position p inside the FFN holds token perm[p], so the FFN runs on the rows perm of
    every per-token operand (X8 and sx; dY8r and sdy_t; the token rows of the column-quantised dY8c and X8c, whose scales belong to
    model dimensions and stay), Y and dX are scattered back to token order, and the weight gradients keep their layout while
    their feature-wise 2:4 groups are made of the tokens the permutation puts side by side.  bw = the backward operands of
    ffn24_bwd_fp8_rowwise_codes by name."""
    perm = np.asarray(perm, dtype=np.int64)
    T = np.asarray(X8).shape[0]
    if sorted(perm.tolist()) != list(range(T)):
        raise ValueError("perm is not a permutation of the tokens")
    f = ffn24_fwd_fp8_rowwise_codes(np.asarray(X8)[perm], np.asarray(sx)[perm], W1_8, sw1, b1, W2_8, sw2)
    bwp = dict(bw)
    for k in ("dY8r", "sdy_t", "dY8c", "X8c"):
        bwp[k] = np.asarray(bw[k])[perm]
    g = ffn24_bwd_fp8_rowwise_codes(f, **bwp, wgrad_mask=wgrad_mask, dense_features=dense_features)
    Y = np.empty_like(f["Y"]); Y[perm] = f["Y"]
    dX = np.empty_like(g["dX"]); dX[perm] = g["dX"]
    return {"fwd": f, "bwd": g, "Y": Y, "dX": dX, "dW1": g["dW1"], "dW2": g["dW2"]}


def ffn_bwd_fp8_rowwise_codes(fwd, dY8r, sdy_t, W2_8r, sw2_f, W1_8c, sw1_d, dY8c, sdy_d, X8c, sx_d, quantise_internal=True):
    """Dense counterpart of ffn24_bwd_fp8_rowwise_codes (no masks): the backward of ffn_fwd_fp8_rowwise_codes with every GEMM
    scaled row-wise.  Same operands from the caller; the internal tensors are quantised where they are made:
      dH = sdy_t[t] sw2_f[f] (dY8r . W2_8r^T);  dZ = bf16(dH * 2 max(0, Z));
      sdz_t[t] = max_f |dZ[t,f]| / 448;  dX = sdz_t[t] sw1_d[d] (e4m3(dZ / sdz_t) . W1_8c^T)
      sh_f[f] = max_t H[t,f] / 448 on the bf16 activation;  sdz_f[f] = max_t |dZ[t,f]| / 448
      dW2 = sh_f[f] sdy_d[d] (e4m3(H / sh_f)^T . dY8c);   dW1 = sx_d[d] sdz_f[f] (X8c^T . e4m3(dZ / sdz_f))
    quantise_internal=False (pinning only) leaves dZ and H unrounded in all three GEMMs."""
    dec = lambda c: E4M3_VALUES[np.ascontiguousarray(c, dtype=np.uint8)]
    f64 = lambda v: np.asarray(v, dtype=np.float32).astype(np.float64)
    dH = (dec(dY8r) @ dec(W2_8r).T) * f64(sdy_t)[:, None] * f64(sw2_f)[None, :]
    dZ = dH * relu2_derivative(fwd["Z"])
    Hq = np.asarray(fwd["Hq"], dtype=np.float32)
    out = {"dH": dH, "dZ": dZ}
    if quantise_internal:
        dZ16 = round_bf16(dZ)
        dZ8r_bits, sdz_t = quantise_rows_e4m3(dZ16)
        dZ8c_bits_t, sdz_f = quantise_rows_e4m3(np.ascontiguousarray(dZ16.T))
        H8c_bits_t, sh_f = quantise_rows_e4m3(np.ascontiguousarray(Hq.T))
        dZr = dec(dZ8r_bits) * sdz_t.astype(np.float64)[:, None]
        dZc = dec(dZ8c_bits_t).T * sdz_f.astype(np.float64)[None, :]
        Hc = dec(H8c_bits_t).T * sh_f.astype(np.float64)[None, :]
        out.update({"dZ16": dZ16, "sdz_t": sdz_t, "sdz_f": sdz_f, "sh_f": sh_f, "dZ8r_bits": dZ8r_bits, "H8_t_bits": H8c_bits_t, "dZ8_t_bits": dZ8c_bits_t})
    else:
        dZr = dZc = dZ
        Hc = Hq.astype(np.float64)
    out["dX"] = (dZr @ dec(W1_8c).T) * f64(sw1_d)[None, :]
    out["dW2"] = (Hc.T @ dec(dY8c)) * f64(sdy_d)[None, :]
    out["dW1"] = (dec(X8c).T * f64(sx_d)[:, None]) @ dZc
    return out


def quantise_rows_e4m3(x):
    """Row-wise e4m3 quantisation of a float matrix: s[r] = max|x[r,:]| / 448 (1 for an all-zero row), codes of x / s."""
    x = np.asarray(x, dtype=np.float32)
    amax = np.abs(x).max(axis=1).astype(np.float32)
    s = np.where(amax > 0, amax / np.float32(448.0), np.float32(1.0)).astype(np.float32)
    return f32_to_e4m3_bits(x / s[:, None]), s


def ffn_fwd_fp8(X, W1, b1, W2, sx, sw1, sh, sw2):
    """Dense counterpart of ffn24_fwd_fp8 (no pruning): every activation is quantised, H8 = e4m3(bf16(H) / sh)."""
    Xq = round_e4m3(np.asarray(X, np.float32) / np.float32(sx)).astype(np.float64)
    W1q = round_e4m3(np.asarray(W1, np.float32) / np.float32(sw1)).astype(np.float64)
    Z = (Xq @ W1q) * (float(sx) * float(sw1))
    if b1 is not None:
        Z = Z + np.asarray(b1, dtype=np.float64)[None, :]
    R, H = _relu2(Z, Bf16)
    Hq = round_bf16(H)
    H8_bits = f32_to_e4m3_bits(Hq / np.float32(sh))
    W2q = round_e4m3(np.asarray(W2, np.float32) / np.float32(sw2)).astype(np.float64)
    Y = (e4m3_bits_to_f32(H8_bits).astype(np.float64) @ W2q) * (float(sh) * float(sw2))
    return {"Z": Z, "Hq": Hq, "H8_bits": H8_bits, "Y": Y}


# --------------------------------------------------------------------------------------
# error measure used by the parity tests
# --------------------------------------------------------------------------------------


def max_rel_err(y, y_ref) -> float:
    """max_i |y_i - ref_i| / max_i |ref_i|  (per tensor; element-wise ratios are unbounded at zeros)."""
    y = np.asarray(y, dtype=np.float64)
    y_ref = np.asarray(y_ref, dtype=np.float64)
    den = float(np.max(np.abs(y_ref)))
    if den == 0.0:
        return float(np.max(np.abs(y)))
    return float(np.max(np.abs(y - y_ref)) / den)


def row_rel_err(y, y_ref) -> float:
    """max over rows r of ||y_r - ref_r||_2 / ||ref_r||_2 (rows whose reference is all zero count by ||y_r||_2).
    Tighter than max_rel_err: every row is measured against its own size, so a small row that is wrong by its own
    magnitude shows, which the per-tensor maximum would hide."""
    y = np.asarray(y, dtype=np.float64)
    y_ref = np.asarray(y_ref, dtype=np.float64)
    y = y.reshape(y.shape[0], -1) if y.ndim > 1 else y.reshape(1, -1)
    y_ref = y_ref.reshape(y.shape)
    num = np.sqrt(np.sum((y - y_ref) ** 2, axis=1))
    den = np.sqrt(np.sum(y_ref ** 2, axis=1))
    return float(np.max(np.where(den > 0, num / np.where(den > 0, den, 1.0), num))) if y.size else 0.0


def fro_rel_err(y, y_ref) -> float:
    """||y - ref||_F / ||ref||_F over the whole tensor."""
    y = np.asarray(y, dtype=np.float64)
    y_ref = np.asarray(y_ref, dtype=np.float64)
    den = float(np.sqrt(np.sum(y_ref ** 2)))
    num = float(np.sqrt(np.sum((y - y_ref) ** 2)))
    return num if den == 0.0 else num / den

