"""CPU fp64 oracle for HMAR's Markovian next-scale attention (forward and backward).

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the tests, the smoke check and
the benchmark's cpu_baseline leg may call it.  It shares no code with the HIP path
and never imports it.

What it computes
----------------
HMAR (Sec. "Efficient Markovian Next-Scale Prediction", Eq. 4) makes next-scale prediction Markovian: the tokens of
resolution scale k are conditioned on one block of H_{k-1} x W_{k-1} tokens that
stands for everything before it, instead of on all earlier scales.  During training
the K scales are laid end to end, coarse to fine, in one sequence (Sec. "Background",
next-scale prediction), and the attention mask changes from VAR's lower
block-triangular pattern to a banded block pattern (Sec. "Efficient Markovian Next-Scale Prediction", appendix "Attention Patterns").  Inside a
scale attention stays bidirectional (Sec. "Background"), and the refinement module conditions
on the scale's own tokens plus the predecessor block (Sec. "The HMAR Architecture").  Hence

    allowed(i, j)  <=>  scale(j) == scale(i)  or  scale(j) == scale(i) - 1 .

The kernel the paper describes (Sec. "Efficient Markovian Next-Scale Prediction", appendix "Efficient Attention Performance") is an exact FlashAttention-style
evaluation of softmax attention under that mask, so the oracle is the plain
definition written out densely with an explicit L x L mask, per (batch, head) slice:

    S = sm_scale * Q K^T  (-inf where not allowed)
    P = softmax_rows(S),  O = P V,  LSE = log sum_j exp(S_ij)

and the backward is the analytic derivative of that definition.  All arithmetic is
float64.  numpy.matmul is the only library primitive used as a step.

Parity status: every function here is pinned by tests/test_oracle_pins.py (closed
forms, brute force, dense library attention on window slices, finite differences).
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "scale_token_counts",
    "scale_offsets",
    "token_scale_ids",
    "markov_mask",
    "block_causal_mask",
    "scale_ids_from_counts",
    "markov_mask_from_counts",
    "block_causal_mask_from_counts",
    "allowed_pairs",
    "attn_fwd",
    "attn_bwd",
    "attn_fwd_masked",
    "attn_bwd_masked",
    "attn_step_fwd",
]


# --------------------------------------------------------------------------- schedule
def scale_token_counts(side_lens):
    """n_k = s_k^2 tokens in scale k (Sec. "Background": scale k holds H_k x W_k tokens; square maps)."""
    sides = [int(s) for s in side_lens]
    if len(sides) == 0 or any(s < 1 for s in sides):
        raise ValueError("side lengths must be a non-empty list of positive integers")
    return [s * s for s in sides]


def scale_offsets(side_lens):
    """off_0 = 0, off_k = n_1 + ... + n_k; scale k (1-based) owns rows [off_{k-1}, off_k)."""
    offs = [0]
    for n in scale_token_counts(side_lens):
        offs.append(offs[-1] + n)
    return offs


def token_scale_ids(side_lens):
    """scale id (1-based) of every token of the concatenated coarse-to-fine sequence."""
    ids = []
    for k, n in enumerate(scale_token_counts(side_lens), start=1):
        ids.extend([k] * n)
    return np.asarray(ids, dtype=np.int64)


def markov_mask(side_lens):
    """L x L boolean mask of the Markovian pattern (Sec. "Efficient Markovian Next-Scale Prediction", Eq. 4; appendix "Attention Patterns").

    Built from per-token scale ids only: a query of scale k may look at keys of scale
    k (bidirectional inside a scale) and of its immediate predecessor k-1.  Scale 1
    has no predecessor and sees only itself.
    """
    sid = token_scale_ids(side_lens)
    qi = sid[:, None]
    kj = sid[None, :]
    return (kj == qi) | (kj == qi - 1)


def block_causal_mask(side_lens):
    """VAR's block-causal mask (Sec. "Background"): scale k sees every scale <= k."""
    sid = token_scale_ids(side_lens)
    return sid[None, :] <= sid[:, None]


def scale_ids_from_counts(token_counts):
    """scale id (1-based) of every token when scale k holds token_counts[k-1] = H_k * W_k tokens
    of a token map that need not be square (Sec. "Background")."""
    counts = [int(n) for n in token_counts]
    if len(counts) == 0 or any(n < 1 for n in counts):
        raise ValueError("token counts must be a non-empty list of positive integers")
    ids = []
    for k, n in enumerate(counts, start=1):
        ids.extend([k] * n)
    return np.asarray(ids, dtype=np.int64)


def markov_mask_from_counts(token_counts):
    """The Markovian mask (Sec. "Efficient Markovian Next-Scale Prediction", Eq. 4) for scales given by their token counts."""
    sid = scale_ids_from_counts(token_counts)
    return (sid[None, :] == sid[:, None]) | (sid[None, :] == sid[:, None] - 1)


def block_causal_mask_from_counts(token_counts):
    """VAR's block-causal mask (Sec. "Background") for scales given by their token counts."""
    sid = scale_ids_from_counts(token_counts)
    return sid[None, :] <= sid[:, None]


def allowed_pairs(side_lens):
    """Number of unmasked (query, key) pairs per head under the Markovian mask."""
    return int(markov_mask(side_lens).sum())


# --------------------------------------------------------------------------- dense masked attention
def _as_f64(x):
    return np.asarray(x, dtype=np.float64)


def attn_fwd_masked(Q, K, V, mask, sm_scale):
    """Dense softmax attention under an explicit boolean mask, float64.

    Q: [..., Lq, D], K, V: [..., Lk, D], mask: [Lq, Lk] (True = may attend).
    Returns O [..., Lq, D], LSE [..., Lq] (natural log of the row sum of
    exp(scaled scores)), and P [..., Lq, Lk].  Every row must have one allowed key.
    """
    Q, K, V = _as_f64(Q), _as_f64(K), _as_f64(V)
    mask = np.asarray(mask, dtype=bool)
    if not mask.any(axis=-1).all():
        raise ValueError("a query row has no allowed key")
    S = float(sm_scale) * np.matmul(Q, np.swapaxes(K, -1, -2))
    S = np.where(mask, S, -np.inf)
    m = S.max(axis=-1, keepdims=True)
    E = np.exp(S - m)                      # exp(-inf) = 0 on masked entries
    l = E.sum(axis=-1, keepdims=True)
    P = E / l
    O = np.matmul(P, V)
    LSE = (m + np.log(l))[..., 0]
    return O, LSE, P


def attn_bwd_masked(Q, K, V, dO, mask, sm_scale):
    """Analytic gradient of attn_fwd_masked's O with respect to Q, K, V, float64.

    With P the softmax of the masked scaled scores:
        dV = P^T dO
        dP = dO V^T
        Delta_i = sum_j P_ij dP_ij
        dS = P * (dP - Delta)            (softmax Jacobian applied row by row)
        dQ = sm_scale * dS K
        dK = sm_scale * dS^T Q
    """
    Q, K, V, dO = _as_f64(Q), _as_f64(K), _as_f64(V), _as_f64(dO)
    _, _, P = attn_fwd_masked(Q, K, V, mask, sm_scale)
    dV = np.matmul(np.swapaxes(P, -1, -2), dO)
    dP = np.matmul(dO, np.swapaxes(V, -1, -2))
    Delta = (P * dP).sum(axis=-1, keepdims=True)
    dS = P * (dP - Delta)
    dQ = float(sm_scale) * np.matmul(dS, K)
    dK = float(sm_scale) * np.matmul(np.swapaxes(dS, -1, -2), Q)
    return dQ, dK, dV


# --------------------------------------------------------------------------- the method
def _check_shapes(side_lens, *tensors):
    L = scale_offsets(side_lens)[-1]
    for t in tensors:
        if t.shape[-2] != L:
            raise ValueError(f"sequence length {t.shape[-2]} does not match schedule length {L}")
    return L


def attn_fwd(Q, K, V, side_lens, sm_scale=None):
    """Markovian next-scale attention forward (Sec. "Efficient Markovian Next-Scale Prediction").  Q, K, V: [B, H, L, D].

    Returns (O [B,H,L,D], LSE [B,H,L]) in float64.  sm_scale defaults to 1/sqrt(D).
    """
    Q, K, V = _as_f64(Q), _as_f64(K), _as_f64(V)
    _check_shapes(side_lens, Q, K, V)
    if sm_scale is None:
        sm_scale = 1.0 / np.sqrt(Q.shape[-1])
    O, LSE, _ = attn_fwd_masked(Q, K, V, markov_mask(side_lens), sm_scale)
    return O, LSE


def attn_bwd(Q, K, V, dO, side_lens, sm_scale=None):
    """Markovian next-scale attention backward.  Returns (dQ, dK, dV), float64."""
    Q, K, V, dO = _as_f64(Q), _as_f64(K), _as_f64(V), _as_f64(dO)
    _check_shapes(side_lens, Q, K, V, dO)
    if sm_scale is None:
        sm_scale = 1.0 / np.sqrt(Q.shape[-1])
    return attn_bwd_masked(Q, K, V, dO, markov_mask(side_lens), sm_scale)


def attn_step_fwd(Q, K, V, n_prev, sm_scale=None):
    """One KV-cache-free inference step (Sec. "Efficient Markovian Next-Scale Prediction", last paragraph; Sec. "Efficiency").

    The step that generates scale k holds only the predecessor block and the scale's
    own tokens: K, V have n_{k-1} + n_k rows (predecessor block first), Q has the
    n_k rows of the current scale.  Every query sees every key of the step, so this
    is ordinary dense attention of Q against K, V.  `n_prev` is only checked.
    """
    Q, K, V = _as_f64(Q), _as_f64(K), _as_f64(V)
    if K.shape[-2] != int(n_prev) + Q.shape[-2]:
        raise ValueError("step keys must be the predecessor block followed by the scale's own tokens")
    if sm_scale is None:
        sm_scale = 1.0 / np.sqrt(Q.shape[-1])
    mask = np.ones((Q.shape[-2], K.shape[-2]), dtype=bool)
    O, LSE, _ = attn_fwd_masked(Q, K, V, mask, sm_scale)
    return O, LSE
