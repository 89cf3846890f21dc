"""Pins for the CPU oracle: checks against things other than the oracle itself.

Each test names what a plausible mistake in oracle/hmar_attn_oracle.py it would catch.
None of these needs a GPU.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import hmar_attn_oracle as orc
import synth_inputs as si

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden_schedules():
    rows = []
    with open(os.path.join(GOLDEN, "schedule_arithmetic.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, sides, L, A = [x.strip() for x in line.split("|")]
            rows.append((name, tuple(int(s) for s in sides.split(",")), int(L), None if A == "-" else int(A)))
    return rows


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


# ------------------------------------------------------------------ schedule arithmetic
@pytest.mark.parametrize("name,sides,L,A", _golden_schedules())
def test_schedule_lengths_and_pair_counts_match_hand_worked_values(name, sides, L, A):
    # catches: wrong n_k (side instead of side^2), off-by-one in offsets, wrong mask family
    offs = orc.scale_offsets(sides)
    assert offs[0] == 0 and offs[-1] == L
    assert len(orc.token_scale_ids(sides)) == L
    if A is not None:
        assert orc.allowed_pairs(sides) == A


def test_sixteen_step_sequence_is_5p84_times_next_token_length():
    # Sec. "Introduction" (efficiency item): up to 5.84x longer than next-token prediction at 256x256
    L = orc.scale_offsets(range(1, 17))[-1]
    assert L == 1496
    assert round(L / 256, 2) == 5.84


def test_finest_scale_has_256x_tokens_of_coarsest():
    # Sec. "Training Dynamics": with K=10 the finest scale has 256x the tokens of the coarsest
    n = orc.scale_token_counts(si.SIDES_256)
    assert len(n) == 10 and n[-1] // n[0] == 256


# ------------------------------------------------------------------ mask
@pytest.mark.parametrize("sides", [si.SIDES_TINY, (3,), (2, 5), (1, 1, 1, 2), si.SIDES_256])
def test_mask_equals_independent_interval_construction(sides):
    # catches: wrong predecessor (k+1 instead of k-1), missing own block, causal triangle
    mask = orc.markov_mask(sides)
    n = [s * s for s in sides]
    L = sum(n)
    assert mask.shape == (L, L)
    # interval construction, written with explicit loops and running sums
    expect = np.zeros((L, L), dtype=bool)
    start = 0
    prev_start = 0
    for k, nk in enumerate(n):
        lo = prev_start if k > 0 else start
        hi = start + nk
        for i in range(start, start + nk):
            for j in range(lo, hi):
                expect[i, j] = True
        prev_start = start
        start += nk
    assert np.array_equal(mask, expect)


@pytest.mark.parametrize("counts", [(2, 6, 12, 20), (1, 3, 3, 7), (5,), (4, 9, 16)])
def test_masks_from_token_counts(counts):
    # scales as H_k x W_k maps that need not be square (Sec. "Background"): (2,6,12,20) = 1x2, 2x3, 3x4, 4x5.
    # catches: counts squared by mistake, predecessor taken two scales back, missing own block
    L = sum(counts)
    offs = [0]
    for n in counts:
        offs.append(offs[-1] + n)
    markov = np.zeros((L, L), dtype=bool)
    causal = np.zeros((L, L), dtype=bool)
    for k in range(len(counts)):
        for i in range(offs[k], offs[k + 1]):
            for j in range(L):
                markov[i, j] = offs[max(k - 1, 0)] <= j < offs[k + 1]
                causal[i, j] = j < offs[k + 1]
    assert np.array_equal(orc.markov_mask_from_counts(counts), markov)
    assert np.array_equal(orc.block_causal_mask_from_counts(counts), causal)
    # row sums: n_{k-1} + n_k keys per row of scale k
    rows = orc.markov_mask_from_counts(counts).sum(axis=1)
    for k in range(len(counts)):
        assert (rows[offs[k]:offs[k + 1]] == counts[k] + (counts[k - 1] if k else 0)).all()


def test_masks_from_counts_reduce_to_the_square_case():
    for sides in (si.SIDES_TINY, (2, 5), si.SIDES_256):
        counts = [s * s for s in sides]
        assert np.array_equal(orc.markov_mask_from_counts(counts), orc.markov_mask(sides))
        assert np.array_equal(orc.block_causal_mask_from_counts(counts), orc.block_causal_mask(sides))
        assert np.array_equal(orc.scale_ids_from_counts(counts), orc.token_scale_ids(sides))


def test_mask_row_and_column_counts_and_contiguity():
    sides = si.SIDES_256
    n = [s * s for s in sides]
    mask = orc.markov_mask(sides)
    offs = orc.scale_offsets(sides)
    for k in range(len(n)):
        rows = mask[offs[k]:offs[k + 1]]
        want = n[k] + (n[k - 1] if k > 0 else 0)
        assert (rows.sum(axis=1) == want).all()
        cols = mask[:, offs[k]:offs[k + 1]]
        wantc = n[k] + (n[k + 1] if k + 1 < len(n) else 0)
        assert (cols.sum(axis=0) == wantc).all()
    # each row's allowed set is one contiguous interval that contains the diagonal
    for i in range(mask.shape[0]):
        idx = np.flatnonzero(mask[i])
        assert idx[-1] - idx[0] + 1 == len(idx)
        assert mask[i, i]
    # last scale's window is 169 + 256 = 425 keys (the KV length of the last inference step)
    assert mask[-1].sum() == 425


def test_markov_mask_is_subset_of_block_causal_and_differs_from_other_readings():
    # catches: returning the block-causal (VAR) mask, or the {k} only / {k-1} only readings
    sides = si.SIDES_256
    m = orc.markov_mask(sides)
    bc = orc.block_causal_mask(sides)
    assert (m <= bc).all() and m.sum() < bc.sum()
    assert bc.sum() == 286434
    sid = orc.token_scale_ids(sides)
    only_self = sid[None, :] == sid[:, None]
    only_prev = sid[None, :] == sid[:, None] - 1
    assert np.array_equal(m, only_self | only_prev)
    assert m.sum() == only_self.sum() + only_prev.sum()
    assert only_self.sum() != m.sum() and only_prev.sum() != m.sum()


# ------------------------------------------------------------------ forward
def _brute_force_fwd(Q, K, V, sides, sm_scale):
    """Scalar triple loops, its own mask logic (scale index by scanning boundaries)."""
    n = [s * s for s in sides]
    L, D = Q.shape
    bounds = []
    acc = 0
    for nk in n:
        bounds.append((acc, acc + nk))
        acc += nk

    def scale_of(t):
        for k, (a, b) in enumerate(bounds):
            if a <= t < b:
                return k
        raise AssertionError

    O = [[0.0] * D for _ in range(L)]
    LSE = [0.0] * L
    for i in range(L):
        ki = scale_of(i)
        scores = []
        keys = []
        for j in range(L):
            kj = scale_of(j)
            if kj == ki or kj == ki - 1:
                s = 0.0
                for d in range(D):
                    s += float(Q[i, d]) * float(K[j, d])
                scores.append(s * sm_scale)
                keys.append(j)
        mx = max(scores)
        ex = [math.exp(s - mx) for s in scores]
        tot = sum(ex)
        LSE[i] = mx + math.log(tot)
        for e, j in zip(ex, keys):
            p = e / tot
            for d in range(D):
                O[i][d] += p * float(V[j, d])
    return np.array(O), np.array(LSE)


def test_forward_matches_scalar_brute_force_on_tiny():
    # catches: transposed operand, wrong scale factor placement, wrong normaliser, wrong LSE
    sides = si.SIDES_TINY
    D = 8
    L = sum(s * s for s in sides)
    Q, K, V = _rand((L, D), 1), _rand((L, D), 2), _rand((L, D), 3)
    sm = 0.37
    O, LSE = orc.attn_fwd(Q[None, None], K[None, None], V[None, None], sides, sm)
    Ob, LSEb = _brute_force_fwd(Q, K, V, sides, sm)
    assert np.abs(O[0, 0] - Ob).max() < 1e-12
    assert np.abs(LSE[0, 0] - LSEb).max() < 1e-12


@pytest.mark.parametrize("sides", [si.SIDES_256, si.SIDES_512])
def test_window_slice_identity_against_library_dense_attention(sides):
    # Every scale's output rows must equal ordinary dense softmax attention of that scale's
    # queries against the keys/values of scales k-1 and k.  The dense attention here is
    # torch's CPU scaled_dot_product_attention in float64, a library routine.
    D = 64
    L = sum(s * s for s in sides)
    Q, K, V = _rand((2, L, D), 11), _rand((2, L, D), 12), _rand((2, L, D), 13)
    sm = 1.0 / math.sqrt(D)
    O, LSE = orc.attn_fwd(Q[None], K[None], V[None], sides, sm)
    offs = np.concatenate([[0], np.cumsum([s * s for s in sides])])
    tq, tk, tv = (torch.from_numpy(x) for x in (Q, K, V))
    for k in range(len(sides)):
        q0, q1 = offs[k], offs[k + 1]
        k0 = offs[k - 1] if k > 0 else offs[k]
        ref = torch.nn.functional.scaled_dot_product_attention(
            tq[:, q0:q1], tk[:, k0:q1], tv[:, k0:q1], scale=sm).numpy()
        assert np.abs(O[0, :, q0:q1] - ref).max() < 1e-12
        # LSE against torch.logsumexp of the window's scaled scores
        s = sm * (tq[:, q0:q1] @ tk[:, k0:q1].transpose(-1, -2))
        assert np.abs(LSE[0, :, q0:q1] - torch.logsumexp(s, dim=-1).numpy()).max() < 1e-12


def test_single_scale_schedule_is_plain_softmax_attention():
    from scipy.special import softmax, logsumexp
    D, s = 16, 5
    L = s * s
    Q, K, V = _rand((3, 2, L, D), 21), _rand((3, 2, L, D), 22), _rand((3, 2, L, D), 23)
    O, LSE = orc.attn_fwd(Q, K, V, (s,), None)
    S = (Q @ np.swapaxes(K, -1, -2)) / math.sqrt(D)   # default scale is 1/sqrt(D)
    assert np.abs(O - softmax(S, axis=-1) @ V).max() < 1e-12
    assert np.abs(LSE - logsumexp(S, axis=-1)).max() < 1e-12


def test_two_scale_schedule_last_block_sees_all_keys():
    from scipy.special import softmax
    sides, D = (2, 3), 8
    L = 13
    Q, K, V = _rand((L, D), 31), _rand((L, D), 32), _rand((L, D), 33)
    O, _ = orc.attn_fwd(Q[None, None], K[None, None], V[None, None], sides, 0.5)
    ref = softmax(0.5 * Q[4:] @ K.T, axis=-1) @ V
    assert np.abs(O[0, 0, 4:] - ref).max() < 1e-12
    ref0 = softmax(0.5 * Q[:4] @ K[:4].T, axis=-1) @ V[:4]
    assert np.abs(O[0, 0, :4] - ref0).max() < 1e-12


def test_first_row_and_constant_keys_closed_forms():
    sides, D = si.SIDES_TINY, 64
    L = 30
    Q, K, V = _rand((L, D), 41), _rand((L, D), 42), _rand((L, D), 43)
    sm = 0.125
    O, LSE = orc.attn_fwd(Q[None, None], K[None, None], V[None, None], sides, sm)
    # scale 1 has one token that sees only itself
    assert np.abs(O[0, 0, 0] - V[0]).max() < 1e-14
    assert abs(LSE[0, 0, 0] - sm * float(Q[0] @ K[0])) < 1e-13
    # all keys equal -> uniform P over the window: O = window mean of V, LSE = s + ln(len)
    Kc = np.tile(K[:1], (L, 1))
    O, LSE = orc.attn_fwd(Q[None, None], Kc[None, None], V[None, None], sides, sm)
    offs = [0, 1, 5, 14, 30]
    for k in range(4):
        lo = offs[k - 1] if k > 0 else offs[k]
        hi = offs[k + 1]
        for i in range(offs[k], offs[k + 1]):
            assert np.abs(O[0, 0, i] - V[lo:hi].mean(axis=0)).max() < 1e-13
            assert abs(LSE[0, 0, i] - (sm * float(Q[i] @ K[0]) + math.log(hi - lo))) < 1e-12


def test_softmax_rows_sum_to_one_and_vanish_outside_window():
    sides, D = si.SIDES_256, 64
    L = 680
    Q, K, V = _rand((1, 1, L, D), 51), _rand((1, 1, L, D), 52), _rand((1, 1, L, D), 53)
    mask = orc.markov_mask(sides)
    O, LSE, P = orc.attn_fwd_masked(Q, K, V, mask, 0.125)
    assert np.abs(P.sum(axis=-1) - 1).max() < 1e-12
    assert (P[0, 0][~mask] == 0).all() and (P[0, 0][mask] > 0).all()
    S = 0.125 * Q[0, 0] @ K[0, 0].T
    recon = np.where(mask, np.exp(S - LSE[0, 0][:, None]), 0.0)
    assert np.abs(recon.sum(axis=-1) - 1).max() < 1e-12
    assert np.abs(recon - P[0, 0]).max() < 1e-12


def test_permuting_keys_inside_a_scale_leaves_output_unchanged():
    sides, D = si.SIDES_256, 32
    L = 680
    Q, K, V = _rand((1, 1, L, D), 61), _rand((1, 1, L, D), 62), _rand((1, 1, L, D), 63)
    O, LSE = orc.attn_fwd(Q, K, V, sides, 0.2)
    perm = np.arange(L)
    rng = np.random.default_rng(0)
    perm[155:255] = rng.permutation(np.arange(155, 255))   # scale 8 of the 256px schedule
    O2, LSE2 = orc.attn_fwd(Q, K[:, :, perm], V[:, :, perm], sides, 0.2)
    assert np.abs(O - O2).max() < 1e-12 and np.abs(LSE - LSE2).max() < 1e-12
    # a permutation that crosses a scale boundary must change the result
    perm2 = np.arange(L)
    perm2[[100, 600]] = perm2[[600, 100]]
    O3, _ = orc.attn_fwd(Q, K[:, :, perm2], V[:, :, perm2], sides, 0.2)
    assert np.abs(O - O3).max() > 1e-3


def test_inference_step_equals_rows_of_training_forward():
    # Sec. "Efficient Markovian Next-Scale Prediction": no prefix/KV cache; step k sees the predecessor block and its own tokens.
    sides, D = si.SIDES_256, 64
    L = 680
    Q, K, V = _rand((2, 3, L, D), 71), _rand((2, 3, L, D), 72), _rand((2, 3, L, D), 73)
    O, LSE = orc.attn_fwd(Q, K, V, sides)
    offs = orc.scale_offsets(sides)
    for k in (0, 1, 5, 9):
        q0, q1 = offs[k], offs[k + 1]
        k0 = offs[k - 1] if k > 0 else q0
        Ok, LSEk = orc.attn_step_fwd(Q[:, :, q0:q1], K[:, :, k0:q1], V[:, :, k0:q1], q0 - k0)
        assert np.abs(Ok - O[:, :, q0:q1]).max() < 1e-12
        assert np.abs(LSEk - LSE[:, :, q0:q1]).max() < 1e-12


# ------------------------------------------------------------------ backward
def _loss(Q, K, V, dO, sides, sm):
    O, _ = orc.attn_fwd(Q, K, V, sides, sm)
    return float((O * dO).sum())


def test_backward_matches_central_finite_differences_on_tiny_all_elements():
    # catches: dropped Delta term, missing sm_scale on dQ/dK, swapped dQ/dK operands
    sides, D = si.SIDES_TINY, 4
    L = 30
    Q, K, V, dO = (_rand((1, 1, L, D), s) for s in (81, 82, 83, 84))
    sm = 0.41
    dQ, dK, dV = orc.attn_bwd(Q, K, V, dO, sides, sm)
    h = 1e-6
    for name, X, G in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV)):
        num = np.zeros_like(X)
        it = np.nditer(X, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = X[idx]
            X[idx] = old + h
            fp = _loss(Q, K, V, dO, sides, sm)
            X[idx] = old - h
            fm = _loss(Q, K, V, dO, sides, sm)
            X[idx] = old
            num[idx] = (fp - fm) / (2 * h)
        err = np.abs(num - G).max() / max(1.0, np.abs(G).max())
        assert err < 1e-7, (name, err)


def test_backward_matches_finite_differences_on_random_coordinates_at_680():
    sides, D = si.SIDES_256, 64
    L = 680
    Q, K, V, dO = (_rand((1, 1, L, D), s) for s in (91, 92, 93, 94))
    sm = 0.125
    dQ, dK, dV = orc.attn_bwd(Q, K, V, dO, sides, sm)
    rng = np.random.default_rng(5)
    h = 1e-5
    for X, G in ((Q, dQ), (K, dK), (V, dV)):
        for _ in range(6):
            idx = (0, 0, int(rng.integers(L)), int(rng.integers(D)))
            old = X[idx]
            X[idx] = old + h
            fp = _loss(Q, K, V, dO, sides, sm)
            X[idx] = old - h
            fm = _loss(Q, K, V, dO, sides, sm)
            X[idx] = old
            num = (fp - fm) / (2 * h)
            assert abs(num - G[idx]) < 1e-6 * max(1.0, abs(G[idx]))


@pytest.mark.parametrize("sides,D", [(si.SIDES_TINY, 64), (si.SIDES_256, 64)])
def test_backward_matches_library_autograd_through_dense_masked_softmax(sides, D):
    # torch float64 autograd through softmax(masked scores) @ V -- a library derivative
    L = sum(s * s for s in sides)
    Qn, Kn, Vn, dOn = (_rand((2, L, D), s) for s in (101, 102, 103, 104))
    sm = 1.0 / math.sqrt(D)
    dQ, dK, dV = orc.attn_bwd(Qn[None], Kn[None], Vn[None], dOn[None], sides, sm)
    Q, K, V = (torch.from_numpy(x.copy()).requires_grad_(True) for x in (Qn, Kn, Vn))
    # mask built here from intervals, not from the oracle
    n = [s * s for s in sides]
    offs = np.concatenate([[0], np.cumsum(n)])
    bias = torch.full((L, L), float("-inf"), dtype=torch.float64)
    for k in range(len(n)):
        lo = offs[k - 1] if k > 0 else offs[k]
        bias[offs[k]:offs[k + 1], lo:offs[k + 1]] = 0.0
    P = torch.softmax(sm * Q @ K.transpose(-1, -2) + bias, dim=-1)
    (P @ V * torch.from_numpy(dOn)).sum().backward()
    assert np.abs(dQ[0] - Q.grad.numpy()).max() < 1e-12
    assert np.abs(dK[0] - K.grad.numpy()).max() < 1e-12
    assert np.abs(dV[0] - V.grad.numpy()).max() < 1e-12


def test_backward_markov_locality():
    # keys of the last scale receive gradient only from last-scale queries; keys of scale k
    # only from queries of scales k and k+1
    sides, D = si.SIDES_256, 16
    L = 680
    Q, K, V, dO = (_rand((1, 1, L, D), s) for s in (111, 112, 113, 114))
    offs = orc.scale_offsets(sides)
    dO2 = dO.copy()
    dO2[:, :, offs[9]:] = 0.0            # silence the last scale's queries
    _, dK, dV = orc.attn_bwd(Q, K, V, dO2, sides)
    assert np.abs(dK[:, :, offs[9]:]).max() == 0 and np.abs(dV[:, :, offs[9]:]).max() == 0
    dO3 = np.zeros_like(dO)
    dO3[:, :, offs[9]:] = dO[:, :, offs[9]:]   # only the last scale's queries
    dQ, dK, dV = orc.attn_bwd(Q, K, V, dO3, sides)
    assert np.abs(dK[:, :, :offs[8]]).max() == 0 and np.abs(dV[:, :, :offs[8]]).max() == 0
    assert np.abs(dK[:, :, offs[8]:]).min() > 0
    assert np.abs(dQ[:, :, :offs[9]]).max() == 0


def test_delta_identity_and_zero_row_sum_of_dS():
    sides, D = si.SIDES_TINY, 64
    Q, K, V, dO = (_rand((2, 2, 30, D), s) for s in (121, 122, 123, 124))
    mask = orc.markov_mask(sides)
    O, _, P = orc.attn_fwd_masked(Q, K, V, mask, 0.125)
    dP = dO @ np.swapaxes(V, -1, -2)
    delta_a = (P * dP).sum(-1)
    delta_b = (dO * O).sum(-1)
    assert np.abs(delta_a - delta_b).max() < 1e-12
    dS = P * (dP - delta_a[..., None])
    assert np.abs(dS.sum(-1)).max() < 1e-12


# ------------------------------------------------------------------ input generator
def test_inputs_are_seeded_and_bf16_exact():
    w = si.WORKLOADS["tiny"]
    a = si.make_inputs(w)
    b = si.make_inputs(w)
    assert all(torch.equal(x, y) for x, y in zip(a, b))
    assert a[0].shape == (2, 2, 30, 64) and a[0].dtype == torch.bfloat16
    assert not torch.equal(a[0], a[1])
    x64 = si.to_f64(a[0])
    assert x64.dtype == np.float64
    assert np.array_equal(x64, a[0].float().numpy().astype(np.float64))
