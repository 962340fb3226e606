"""Pins of the CPU oracle against what the paper and the mathematics fix.

The paper prints no worked numeric example of the attention, so the oracle is
pinned by special cases that reduce to textbook / library routines, brute force
over an explicit mask matrix, closed forms and invariants (Sec. 3.1 "Block-wise
Causal Attention"; Sec. 4.2 and Appendix A for the speculative form; Appendix B
for the cached form).  Every check here is independent of the oracle's own
code path: the references are numpy expressions written differently (dense
matrix form) or a library SDPA.
"""
import numpy as np
import pytest
import torch

from oracle import nfd_oracle as orc


def rnd(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def dense_reference(q, k, v, mask, scale):
    """Dense-matrix softmax attention with an explicit boolean mask [Sq,Sk] (numpy, fp64)."""
    s = np.einsum("bhid,bhjd->bhij", q, k) * scale
    s = np.where(mask[None, None], s, -np.inf)
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    return np.einsum("bhij,bhjd->bhid", e / e.sum(axis=-1, keepdims=True), v)


def frame_mask(T, kv_frames, q_frames):
    """Explicit mask built frame by frame from the sentence in Sec. 3.1: the tokens of
    query frame a (absolute frame P+a) see all tokens of frames 0..P+a."""
    P = kv_frames - q_frames
    M = np.zeros((q_frames * T, kv_frames * T), dtype=bool)
    for a in range(q_frames):
        M[a * T:(a + 1) * T, : (P + a + 1) * T] = True
    return M


# ---- P1: T = 1 reduces to standard causal attention -------------------------------------
def test_T1_is_causal_attention():
    B, H, S, D = 2, 3, 37, 16
    q, k, v = rnd((B, H, S, D), 1), rnd((B, H, S, D), 2), rnd((B, H, S, D), 3)
    got = orc.block_causal_attn(q, k, v, T=1)
    ref = dense_reference(q, k, v, np.tril(np.ones((S, S), dtype=bool)), 1 / np.sqrt(D))
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-13)
    lib = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q), torch.from_numpy(k), torch.from_numpy(v), is_causal=True).numpy()
    np.testing.assert_allclose(got, lib, rtol=1e-10, atol=1e-12)


# ---- P2: one frame reduces to full bidirectional attention ------------------------------
def test_single_frame_is_full_attention():
    B, H, T, D = 1, 2, 29, 8
    q, k, v = rnd((B, H, T, D), 4), rnd((B, H, T, D), 5), rnd((B, H, T, D), 6)
    got = orc.block_causal_attn(q, k, v, T=T)
    lib = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q), torch.from_numpy(k), torch.from_numpy(v)).numpy()
    np.testing.assert_allclose(got, lib, rtol=1e-10, atol=1e-12)


# ---- P3: brute force with an explicit mask matrix ----------------------------------------
@pytest.mark.parametrize("T,kvf,qf,D", [(16, 4, 4, 64), (3, 5, 5, 8), (3, 5, 2, 8), (7, 6, 1, 4), (5, 4, 3, 12)])
def test_brute_force_explicit_mask(T, kvf, qf, D):
    B, H = 2, 2
    q, k, v = rnd((B, H, qf * T, D), 7), rnd((B, H, kvf * T, D), 8), rnd((B, H, kvf * T, D), 9)
    got = orc.block_causal_attn(q, k, v, T=T, kv_frames=kvf, q_frames=qf, scale=0.3)
    ref = dense_reference(q, k, v, frame_mask(T, kvf, qf), 0.3)
    np.testing.assert_allclose(got, ref, rtol=1e-11, atol=1e-13)


def test_capacity_rows_beyond_kv_frames_are_ignored():
    """k, v hold F frames but only kv_frames are valid: the rest must not be read into the result."""
    B, H, T, D, F, kvf, qf = 1, 2, 4, 8, 7, 5, 2
    q, k, v = rnd((B, H, qf * T, D), 10), rnd((B, H, F * T, D), 11), rnd((B, H, F * T, D), 12)
    got = orc.block_causal_attn(q, k, v, T=T, kv_frames=kvf, q_frames=qf)
    ref = dense_reference(q, k[:, :, : kvf * T], v[:, :, : kvf * T], frame_mask(T, kvf, qf), 1 / np.sqrt(D))
    np.testing.assert_allclose(got, ref, rtol=1e-11, atol=1e-13)
    k2, v2 = k.copy(), v.copy()
    k2[:, :, kvf * T:] = 1e6
    v2[:, :, kvf * T:] = np.nan
    assert np.array_equal(got, orc.block_causal_attn(q, k2, v2, T=T, kv_frames=kvf, q_frames=qf))


# ---- P4: causality: later frames cannot influence earlier outputs -------------------------
def test_future_perturbation_leaves_past_bit_identical():
    B, H, T, D, F = 1, 2, 6, 8, 5
    q, k, v = rnd((B, H, F * T, D), 13), rnd((B, H, F * T, D), 14), rnd((B, H, F * T, D), 15)
    base = orc.block_causal_attn(q, k, v, T=T)
    for f in range(F - 1):
        k2, v2 = k.copy(), v.copy()
        k2[:, :, (f + 1) * T:] += rnd(k2[:, :, (f + 1) * T:].shape, 16 + f) * 10
        v2[:, :, (f + 1) * T:] -= 3.0
        pert = orc.block_causal_attn(q, k2, v2, T=T)
        assert np.array_equal(base[:, :, : (f + 1) * T], pert[:, :, : (f + 1) * T])
        assert not np.allclose(base[:, :, (f + 1) * T:], pert[:, :, (f + 1) * T:])


def test_own_frame_is_bidirectional():
    """Changing the LAST token's K/V of a frame changes the FIRST token's output of that frame."""
    B, H, T, D, F = 1, 1, 5, 4, 3
    q, k, v = rnd((B, H, F * T, D), 21), rnd((B, H, F * T, D), 22), rnd((B, H, F * T, D), 23)
    base = orc.block_causal_attn(q, k, v, T=T)
    v2 = v.copy()
    v2[0, 0, 2 * T - 1] += 5.0  # last token of frame 1
    pert = orc.block_causal_attn(q, k, v2, T=T)
    assert np.array_equal(base[0, 0, :T], pert[0, 0, :T])          # frame 0 untouched
    assert np.all(np.abs(base[0, 0, T] - pert[0, 0, T]) > 0)         # first token of frame 1 changed
    assert np.all(np.abs(base[0, 0, 2 * T] - pert[0, 0, 2 * T]) > 0)  # frame 2 sees it too


# ---- P5: equal scores => mean of visible V -------------------------------------------------
@pytest.mark.parametrize("mode", ["q_zero", "k_const"])
def test_uniform_scores_give_mean_of_visible_v(mode):
    B, H, T, D, kvf, qf = 1, 2, 4, 8, 6, 3
    q, k, v = rnd((B, H, qf * T, D), 24), rnd((B, H, kvf * T, D), 25), rnd((B, H, kvf * T, D), 26)
    if mode == "q_zero":
        q = np.zeros_like(q)
    else:
        k = np.broadcast_to(rnd((B, H, 1, D), 27), k.shape).copy()
    got = orc.block_causal_attn(q, k, v, T=T, kv_frames=kvf, q_frames=qf)
    P = kvf - qf
    for a in range(qf):
        mean = v[:, :, : (P + a + 1) * T].mean(axis=2, keepdims=True)
        np.testing.assert_allclose(got[:, :, a * T:(a + 1) * T], np.broadcast_to(mean, (B, H, T, D)),
                                   rtol=1e-12, atol=1e-13)


# ---- P6: visible-pair count closed form, and the ~50 % claim of Sec. 3.1 --------------------
@pytest.mark.parametrize("T,kvf,qf", [(1, 1, 1), (3, 5, 5), (3, 5, 2), (16, 4, 4), (7, 9, 1), (4, 8, 3)])
def test_visible_pairs_closed_form(T, kvf, qf):
    P = kvf - qf
    assert orc.visible_pairs(T, kvf, qf) == T * T * (qf * P + qf * (qf + 1) // 2)
    assert orc.visible_pairs(T, kvf, qf) == int(frame_mask(T, kvf, qf).sum())


def test_half_cost_claim():
    for F, want in [(16, 17 / 32), (64, 65 / 128)]:
        frac = orc.visible_pairs(2, F, F) / float((2 * F) ** 2)
        assert abs(frac - want) < 1e-15
    assert abs(orc.visible_pairs(1, 400, 400) / 400.0 ** 2 - 0.5) < 2e-3


# ---- P7: cached form == tail rows of the full form ----------------------------------------
@pytest.mark.parametrize("qf", [1, 2, 4])
def test_cached_form_equals_tail_of_full_form(qf):
    B, H, T, D, F = 1, 2, 5, 8, 6
    q, k, v = rnd((B, H, F * T, D), 28), rnd((B, H, F * T, D), 29), rnd((B, H, F * T, D), 30)
    full = orc.block_causal_attn(q, k, v, T=T)
    tail = orc.block_causal_attn(q[:, :, (F - qf) * T:], k, v, T=T, kv_frames=F, q_frames=qf)
    assert np.array_equal(full[:, :, (F - qf) * T:], tail)


# ---- P8: speculative k-frame call == k single-frame calls with a growing cache ------------
def test_speculative_equals_sequential():
    B, H, T, D, past, kq = 1, 2, 4, 8, 3, 3
    F = past + kq
    q, k, v = rnd((B, H, kq * T, D), 31), rnd((B, H, F * T, D), 32), rnd((B, H, F * T, D), 33)
    spec = orc.block_causal_attn(q, k, v, T=T, kv_frames=F, q_frames=kq)
    for a in range(kq):
        one = orc.block_causal_attn(q[:, :, a * T:(a + 1) * T], k, v, T=T, kv_frames=past + a + 1, q_frames=1)
        assert np.array_equal(spec[:, :, a * T:(a + 1) * T], one)


# ---- P9: permutation invariants within a frame --------------------------------------------
def test_intra_frame_permutations():
    B, H, T, D, F = 1, 2, 6, 8, 4
    q, k, v = rnd((B, H, F * T, D), 34), rnd((B, H, F * T, D), 35), rnd((B, H, F * T, D), 36)
    base = orc.block_causal_attn(q, k, v, T=T)
    rng = np.random.default_rng(37)
    perm = np.concatenate([f * T + rng.permutation(T) for f in range(F)])
    np.testing.assert_allclose(orc.block_causal_attn(q, k[:, :, perm], v[:, :, perm], T=T), base,
                               rtol=1e-12, atol=1e-14)
    assert np.array_equal(orc.block_causal_attn(q[:, :, perm], k, v, T=T), base[:, :, perm])
    # a permutation ACROSS frames must change the result (the mask is not permutation invariant)
    cross = np.arange(F * T)
    cross[[0, F * T - 1]] = cross[[F * T - 1, 0]]
    assert not np.allclose(orc.block_causal_attn(q, k[:, :, cross], v[:, :, cross], T=T), base)


# ---- P10: convexity / linearity in V --------------------------------------------------------
def test_convexity_and_linearity_in_v():
    B, H, T, D, kvf, qf = 1, 2, 5, 8, 5, 3
    q, k = rnd((B, H, qf * T, D), 38), rnd((B, H, kvf * T, D), 39)
    v1, v2 = rnd((B, H, kvf * T, D), 40), rnd((B, H, kvf * T, D), 41)
    f = lambda vv: orc.block_causal_attn(q, k, vv, T=T, kv_frames=kvf, q_frames=qf)
    o1, o2 = f(v1), f(v2)
    np.testing.assert_allclose(f(2.0 * v1 - 3.0 * v2), 2.0 * o1 - 3.0 * o2, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(f(np.full_like(v1, 1.75)), 1.75, rtol=1e-13)
    P = kvf - qf
    for a in range(qf):
        vis = v1[:, :, : (P + a + 1) * T]
        blk = o1[:, :, a * T:(a + 1) * T]
        assert np.all(blk <= vis.max(axis=2, keepdims=True) + 1e-12)
        assert np.all(blk >= vis.min(axis=2, keepdims=True) - 1e-12)


# ---- P11: one-hot limit --------------------------------------------------------------------
def test_one_hot_key_and_invisible_future_key():
    B, H, T, D, F = 1, 1, 4, 8, 4
    q = rnd((B, H, F * T, D), 42)
    q[..., 0] = 1.0
    k = 0.01 * rnd((B, H, F * T, D), 43)
    v = rnd((B, H, F * T, D), 44)
    scale = 1.0
    hot = 1 * T + 2  # a key in frame 1
    k[0, 0, hot] = 0.0
    k[0, 0, hot, 0] = 200.0
    out = orc.block_causal_attn(q, k, v, T=T, scale=scale)
    # frames >= 1 see the hot key and return its V row; frame 0 does not see it
    np.testing.assert_allclose(out[0, 0, T:], np.broadcast_to(v[0, 0, hot], ((F - 1) * T, D)), atol=1e-9)
    k0 = k.copy()
    k0[0, 0, hot] = 0.01
    base0 = orc.block_causal_attn(q, k0, v, T=T, scale=scale)
    assert np.array_equal(out[0, 0, :T], base0[0, 0, :T])


# ---- P12: large magnitudes ------------------------------------------------------------------
def test_large_scores_are_stable():
    B, H, T, D, F = 1, 2, 5, 16, 3
    q, k, v = 30 * rnd((B, H, F * T, D), 45), 30 * rnd((B, H, F * T, D), 46), rnd((B, H, F * T, D), 47)
    got = orc.block_causal_attn(q, k, v, T=T)
    assert np.all(np.isfinite(got))
    # log-sum-exp reference through scipy
    from scipy.special import logsumexp
    s = np.einsum("bhid,bhjd->bhij", q, k) / np.sqrt(D)
    s = np.where(frame_mask(T, F, F)[None, None], s, -np.inf)
    w = np.exp(s - logsumexp(s, axis=-1, keepdims=True))
    np.testing.assert_allclose(got, np.einsum("bhij,bhjd->bhid", w, v), rtol=1e-9, atol=1e-12)


# ---- row-sampled mode is the same computation on a subset -----------------------------------
def test_row_sampled_mode_matches_full():
    B, H, T, D, kvf, qf = 2, 2, 6, 8, 5, 3
    q, k, v = rnd((B, H, qf * T, D), 48), rnd((B, H, kvf * T, D), 49), rnd((B, H, kvf * T, D), 50)
    full = orc.block_causal_attn(q, k, v, T=T, kv_frames=kvf, q_frames=qf)
    rows = np.array([0, 5, 6, 11, 17, 3], dtype=np.int64)
    assert np.array_equal(orc.block_causal_attn(q, k, v, T=T, kv_frames=kvf, q_frames=qf, rows=rows),
                          full[:, :, rows])


def test_default_scale_is_inverse_sqrt_d():
    B, H, T, D, F = 1, 1, 4, 64, 2
    q, k, v = rnd((B, H, F * T, D), 51), rnd((B, H, F * T, D), 52), rnd((B, H, F * T, D), 53)
    assert np.array_equal(orc.block_causal_attn(q, k, v, T=T), orc.block_causal_attn(q, k, v, T=T, scale=0.125))


def test_argument_errors():
    q = rnd((1, 1, 8, 4), 54)
    with pytest.raises(ValueError):
        orc.block_causal_attn(q, q, q, T=4, kv_frames=1, q_frames=2)   # q_frames > kv_frames
    with pytest.raises(ValueError):
        orc.block_causal_attn(q, q, q, T=4, kv_frames=3, q_frames=2)   # kv_frames > capacity
    with pytest.raises(ValueError):
        orc.block_causal_attn(q, q, q, T=3)                            # rows not a multiple of T


# ---- cache append ---------------------------------------------------------------------------
def test_kvcache_append_places_frames():
    B, H, T, D, F = 2, 2, 3, 4, 5
    cache = rnd((B, H, F * T, D), 55)
    fresh = rnd((B, H, 2 * T, D), 56)
    got = orc.kvcache_append(cache, fresh, T=T, frame_pos=2)
    want = cache.copy()
    want[:, :, 2 * T:4 * T] = fresh
    assert np.array_equal(got, want)
    with pytest.raises(ValueError):
        orc.kvcache_append(cache, fresh, T=T, frame_pos=4)


def test_paper_stated_cost_reduction_fixture():
    """tests/golden/cost_reduction.txt holds the paper's statement (Sec. 3.1) that the mask halves the cost:
    the oracle's enumerated visible fraction of the training form agrees with it within the stated slack."""
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "cost_reduction.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 2
    for frames, claim, slack in rows:
        F, T = int(frames), 3
        frac = orc.visible_pairs(T, F, F) / float((F * T) ** 2)
        assert abs(frac - float(claim)) <= float(slack), (F, frac)
        assert abs(frac - (F + 1) / (2.0 * F)) < 1e-12
