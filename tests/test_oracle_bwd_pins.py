"""Pins of the oracle's attention gradients (the paper trains through the block-wise causal
attention: Sec. 3.1 for the mask, Sec. 3.2 for training).  The gradient formulas are pinned by
things that do not contain them: central finite differences of the FORWARD oracle, reverse-mode
autodiff of a library (torch, fp64) through a dense attention with an explicit mask matrix,
and invariants of the mask and of the softmax Jacobian."""
import numpy as np
import pytest
import torch

from oracle import nfd_oracle as orc


def _case(B, H, T, D, kvf, qf, F, seed):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((B, H, qf * T, D))
    k = rng.standard_normal((B, H, F * T, D))
    v = rng.standard_normal((B, H, F * T, D))
    g = rng.standard_normal((B, H, qf * T, D))
    return q, k, v, g


SHAPES = [
    # B, H, T, D, kvf, qf, F
    (1, 2, 3, 4, 4, 4, 4),    # training form
    (2, 1, 2, 8, 5, 2, 6),    # cached form with spare capacity
    (1, 1, 1, 4, 6, 6, 6),    # T = 1: causal attention
    (1, 1, 5, 2, 1, 1, 1),    # one frame: full attention
]


@pytest.mark.parametrize("B,H,T,D,kvf,qf,F", SHAPES)
def test_gradients_match_central_differences_of_the_forward_oracle(B, H, T, D, kvf, qf, F):
    """L = sum(out * g).  dL/dx by (L(x + e) - L(x - e)) / 2e on every element of q, k, v."""
    q, k, v, g = _case(B, H, T, D, kvf, qf, F, 11)
    dq, dk, dv, _ = orc.block_causal_attn_bwd(q, k, v, g, T, kv_frames=kvf, q_frames=qf, scale=0.7)
    loss = lambda q_, k_, v_: float((orc.block_causal_attn(q_, k_, v_, T, kv_frames=kvf, q_frames=qf, scale=0.7) * g).sum())
    eps = 1e-6
    for name, x, dx in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        num = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = x[idx]
            x[idx] = old + eps
            up = loss(q, k, v)
            x[idx] = old - eps
            dn = loss(q, k, v)
            x[idx] = old
            num[idx] = (up - dn) / (2 * eps)
        np.testing.assert_allclose(dx, num, rtol=0, atol=2e-8, err_msg=name)


@pytest.mark.parametrize("B,H,T,D,kvf,qf,F", SHAPES + [(1, 2, 7, 16, 6, 3, 7)])
def test_gradients_match_library_autodiff_through_dense_masked_attention(B, H, T, D, kvf, qf, F):
    q, k, v, g = _case(B, H, T, D, kvf, qf, F, 12)
    dq, dk, dv, lse = orc.block_causal_attn_bwd(q, k, v, g, T, kv_frames=kvf, q_frames=qf)
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, k, v))
    Sq, Sk, P = qf * T, kvf * T, kvf - qf
    i = torch.arange(Sq)[:, None] // T
    j = torch.arange(Sk)[None, :] // T
    mask = j <= P + i
    s = (tq @ tk[:, :, :Sk].transpose(-1, -2)) / np.sqrt(D)
    s = s.masked_fill(~mask, float("-inf"))
    out = torch.softmax(s, dim=-1) @ tv[:, :, :Sk]
    (out * torch.tensor(g)).sum().backward()
    np.testing.assert_allclose(dq, tq.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dk, tk.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dv, tv.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(lse, torch.logsumexp(s, dim=-1).detach().numpy(), atol=1e-12)
    assert np.all(dk[:, :, Sk:] == 0) and np.all(dv[:, :, Sk:] == 0)  # capacity rows get no gradient


def test_keys_of_a_frame_get_gradient_only_from_rows_of_that_frame_onwards():
    """dk_j, dv_j gather over the rows that see key j: zeroing dout for all frames >= f leaves the
    keys of frames >= f with exactly zero gradient; changing dout of earlier frames does not matter."""
    B, H, T, D, Fr = 1, 2, 4, 8, 5
    q, k, v, g = _case(B, H, T, D, Fr, Fr, Fr, 13)
    f = 3
    g2 = g.copy()
    g2[:, :, f * T:] = 0.0
    dq, dk, dv, _ = orc.block_causal_attn_bwd(q, k, v, g2, T)
    assert np.all(dk[:, :, f * T:] == 0) and np.all(dv[:, :, f * T:] == 0) and np.all(dq[:, :, f * T:] == 0)
    assert np.abs(dk[:, :, :f * T]).min() > 0


def test_scores_gradient_sums_to_zero_per_row_so_dq_ignores_a_common_key_shift():
    """The softmax Jacobian annihilates constants: adding one vector c to every VISIBLE key changes
    every score of a row by the same amount, so out, dv and dq are unchanged when all keys a row can
    see are shifted - true for the last frame's rows when every key is shifted."""
    B, H, T, D, Fr = 1, 1, 3, 6, 4
    q, k, v, g = _case(B, H, T, D, Fr, Fr, Fr, 14)
    c = np.random.default_rng(15).standard_normal(D)
    dq0, dk0, dv0, lse0 = orc.block_causal_attn_bwd(q, k, v, g, T)
    dq1, dk1, dv1, lse1 = orc.block_causal_attn_bwd(q, k + c, v, g, T)
    np.testing.assert_allclose(dv1, dv0, atol=1e-12)
    # dq_i = scale * sum_j ds_ij (k_j + c) = dq_i + scale * c * sum_j ds_ij, and sum_j ds_ij = 0
    np.testing.assert_allclose(dq1, dq0, atol=1e-12)
    np.testing.assert_allclose(dk1, dk0, atol=1e-12)


def test_dv_is_linear_in_dout_and_dq_dk_vanish_for_constant_values():
    """If every value row is the same vector the output does not depend on the scores: dq = dk = 0;
    and dv_j = sum_i p_ij dout_i is the transposed attention applied to dout."""
    B, H, T, D, Fr = 1, 2, 3, 4, 4
    q, k, v, g = _case(B, H, T, D, Fr, Fr, Fr, 16)
    vconst = np.broadcast_to(np.arange(1.0, D + 1.0), v.shape).copy()
    dq, dk, dv, _ = orc.block_causal_attn_bwd(q, k, vconst, g, T)
    assert np.abs(dq).max() < 1e-13 and np.abs(dk).max() < 1e-13
    # column sums of P are the weights: sum_j dv_j = sum_i dout_i (rows of P sum to one)
    np.testing.assert_allclose(dv.sum(axis=2), g.sum(axis=2), atol=1e-12)


def test_cached_form_gradients_equal_training_form_with_zero_upstream_on_past_rows():
    """Queries = last q_frames frames: same dk, dv as the full form whose upstream gradient is zero
    on the earlier frames' rows; dq equals the tail rows."""
    B, H, T, D, Fr, qf = 1, 2, 3, 4, 5, 2
    q, k, v, g = _case(B, H, T, D, Fr, Fr, Fr, 17)
    g_full = g.copy()
    g_full[:, :, :(Fr - qf) * T] = 0.0
    dq_f, dk_f, dv_f, _ = orc.block_causal_attn_bwd(q, k, v, g_full, T)
    dq_c, dk_c, dv_c, _ = orc.block_causal_attn_bwd(q[:, :, (Fr - qf) * T:], k, v, g[:, :, (Fr - qf) * T:], T,
                                                    kv_frames=Fr, q_frames=qf)
    np.testing.assert_allclose(dq_c, dq_f[:, :, (Fr - qf) * T:], atol=1e-13)
    np.testing.assert_allclose(dk_c, dk_f, atol=1e-13)
    np.testing.assert_allclose(dv_c, dv_f, atol=1e-13)
