"""Pins of the oracle's 3D rotary embedding + cache write (Sec. 3.1 "3D Positional Embedding";
Appendix B "KV Caching").  The paper prints no numbers for it, so the oracle is pinned by what
the mathematics fixes: the complex-multiplication form of textbook 1-D RoPE, the identity at
the origin, norm preservation, dependence of rotated dot products on position differences
only, independence of the three sections, and closed-form quarter turns."""
import numpy as np
import pytest

from oracle import nfd_oracle as orc


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def _run(B=1, H=2, grid=(3, 4), n_new=2, F=5, frame_pos=1, sections=(4, 6, 6), theta=10000.0,
         t_offset=0, seed=1, q=None, k=None, v=None):
    T, D = grid[0] * grid[1], sum(sections)
    q = _rand((B, H, n_new * T, D), seed) if q is None else q
    k = _rand((B, H, n_new * T, D), seed + 1) if k is None else k
    v = _rand((B, H, n_new * T, D), seed + 2) if v is None else v
    kc = np.full((B, H, F * T, D), 7.0)
    vc = np.full((B, H, F * T, D), -7.0)
    qo, kc2, vc2 = orc.rope_kvcache_append(q, kc, vc, k, v, T, frame_pos, grid, sections, theta, t_offset)
    return q, k, v, qo, kc2, vc2, T, D


def test_time_only_section_is_textbook_1d_rope_by_complex_multiplication():
    """n_h = n_w = 0: every feature pair (2i, 2i+1) is the complex number a + ib multiplied by
    exp(i * t * theta^(-2i/D)), the textbook rotary embedding over the frame index."""
    grid, D, n_new, F, fp = (2, 3), 8, 3, 6, 2
    q, k, v, qo, kc, vc, T, _ = _run(grid=grid, n_new=n_new, F=F, frame_pos=fp, sections=(D, 0, 0), theta=100.0)
    t = fp + np.arange(n_new * T) // T
    freq = 100.0 ** (-np.arange(0, D, 2) / D)
    rot = np.exp(1j * t[:, None] * freq[None, :])  # [rows, D/2]
    for x, y in ((q, qo), (k, kc[:, :, fp * T:(fp + n_new) * T])):
        z = (x[..., 0::2] + 1j * x[..., 1::2]) * rot
        np.testing.assert_allclose(y[..., 0::2], z.real, rtol=0, atol=1e-12)
        np.testing.assert_allclose(y[..., 1::2], z.imag, rtol=0, atol=1e-12)


def test_width_only_section_uses_column_index_and_height_only_the_row_index():
    grid, D = (3, 5), 6
    T = 15
    for sections, pos in (((0, 0, D), np.arange(T) % 5), ((0, D, 0), np.arange(T) // 5)):
        q, k, v, qo, kc, vc, _, _ = _run(grid=grid, n_new=1, F=2, frame_pos=1, sections=sections, theta=50.0)
        freq = 50.0 ** (-np.arange(0, D, 2) / D)
        rot = np.exp(1j * pos[:, None] * freq[None, :])
        z = (q[..., 0::2] + 1j * q[..., 1::2]) * rot
        np.testing.assert_allclose(qo[..., 0::2], z.real, atol=1e-12)
        np.testing.assert_allclose(qo[..., 1::2], z.imag, atol=1e-12)


def test_origin_is_the_identity_and_values_and_other_frames_are_untouched():
    q, k, v, qo, kc, vc, T, D = _run(grid=(1, 1), n_new=1, F=3, frame_pos=0)
    np.testing.assert_array_equal(qo, q)  # position (0, 0, 0): every angle is zero
    np.testing.assert_array_equal(kc[:, :, :T], k)
    np.testing.assert_array_equal(vc[:, :, :T], v)
    assert np.all(kc[:, :, T:] == 7.0) and np.all(vc[:, :, T:] == -7.0)
    # general case: v copied bit for bit into the right frames, nothing else written
    q, k, v, qo, kc, vc, T, D = _run(n_new=2, F=5, frame_pos=1)
    np.testing.assert_array_equal(vc[:, :, T:3 * T], v)
    assert np.all(vc[:, :, :T] == -7.0) and np.all(vc[:, :, 3 * T:] == -7.0)
    assert np.all(kc[:, :, :T] == 7.0) and np.all(kc[:, :, 3 * T:] == 7.0)


def test_every_pair_keeps_its_norm():
    q, k, v, qo, kc, vc, T, D = _run(seed=5)
    n_in = q[..., 0::2] ** 2 + q[..., 1::2] ** 2
    n_out = qo[..., 0::2] ** 2 + qo[..., 1::2] ** 2
    np.testing.assert_allclose(n_out, n_in, rtol=1e-12)


def test_rotated_dot_products_depend_on_position_differences_only():
    """<rope(q, p), rope(k, p')> is a function of p - p': shifting every temporal position by the
    same offset leaves all query-key dot products unchanged, per section and in total."""
    grid, sections = (3, 4), (4, 6, 6)
    q, k, v, qo_a, kc_a, _, T, D = _run(grid=grid, n_new=2, F=4, frame_pos=0, sections=sections, t_offset=0, seed=9)
    _, _, _, qo_b, kc_b, _, _, _ = _run(grid=grid, n_new=2, F=4, frame_pos=0, sections=sections, t_offset=11, seed=9)
    ka, kb = kc_a[:, :, :2 * T], kc_b[:, :, :2 * T]
    assert np.abs(qo_a - qo_b).max() > 1e-3  # the embeddings themselves do change
    np.testing.assert_allclose(qo_a @ ka.transpose(0, 1, 3, 2), qo_b @ kb.transpose(0, 1, 3, 2), atol=1e-10)
    # and a spatial shift: token (y, x) against token (y, x + 1) gives the same product wherever x is
    one = np.ones((1, 1, T, D))
    _, _, _, qo, kc, _, _, _ = _run(B=1, H=1, grid=grid, n_new=1, F=1, frame_pos=0, sections=sections, q=one, k=one, v=one)
    s = (qo @ kc.transpose(0, 1, 3, 2))[0, 0]
    tok = lambda y, x: y * grid[1] + x
    assert abs(s[tok(0, 0), tok(0, 1)] - s[tok(2, 2), tok(2, 3)]) < 1e-10
    assert abs(s[tok(0, 1), tok(1, 1)] - s[tok(1, 3), tok(2, 3)]) < 1e-10
    assert abs(s[tok(0, 0), tok(0, 1)] - s[tok(0, 0), tok(0, 2)]) > 1e-6  # one step and two steps differ


def test_sections_are_independent_and_ordered_t_h_w():
    """Moving a token along one axis changes only that axis's slice of the head dimension."""
    grid, sections = (3, 4), (4, 6, 8)
    T, D = 12, 18
    x = _rand((1, 1, T, D), 3)
    _, _, _, q0, _, _, _, _ = _run(B=1, H=1, grid=grid, n_new=1, F=9, frame_pos=0, sections=sections, q=x, k=x, v=x)
    _, _, _, q5, _, _, _, _ = _run(B=1, H=1, grid=grid, n_new=1, F=9, frame_pos=5, sections=sections, q=x, k=x, v=x)
    assert np.abs(q0[..., :4] - q5[..., :4]).max() > 1e-3       # frame index: T section only
    np.testing.assert_array_equal(q0[..., 4:], q5[..., 4:])
    same = np.repeat(x[:, :, :1], T, axis=2)                     # one vector at every grid position
    _, _, _, qs, _, _, _, _ = _run(B=1, H=1, grid=grid, n_new=1, F=1, frame_pos=0, sections=sections, q=same, k=same, v=same)
    row0, row1 = qs[0, 0, 0:4], qs[0, 0, 4:8]                    # y = 0 and y = 1
    np.testing.assert_array_equal(row0[:, 4:10], np.repeat(row0[:1, 4:10], 4, axis=0))  # H section constant along x
    assert np.abs(row0[1, 10:] - row0[0, 10:]).max() > 1e-3      # W section moves along x
    np.testing.assert_array_equal(row0[:, 10:], row1[:, 10:])    # W section constant along y
    assert np.abs(row1[0, 4:10] - row0[0, 4:10]).max() > 1e-3    # H section moves along y
    np.testing.assert_array_equal(qs[0, 0, :, :4], np.repeat(qs[0, 0, :1, :4], T, axis=0))  # T section constant in a frame


def test_first_pair_of_each_axis_turns_by_the_position_in_radians_counter_clockwise():
    """Pair 0 of a section has frequency theta^0 = 1: the unit vector (1, 0) at position p becomes
    (cos p, sin p).  Fixes the rotation sense and that positions are not scaled."""
    grid, sections = (2, 3), (2, 2, 2)
    T, D = 6, 6
    x = np.zeros((1, 1, T, D))
    x[..., 0::2] = 1.0
    _, _, _, qo, _, _, _, _ = _run(B=1, H=1, grid=grid, n_new=1, F=4, frame_pos=3, sections=sections, q=x, k=x, v=x)
    for tok in range(T):
        for ax, p in enumerate((3, tok // 3, tok % 3)):
            assert abs(qo[0, 0, tok, 2 * ax] - np.cos(p)) < 1e-14
            assert abs(qo[0, 0, tok, 2 * ax + 1] - np.sin(p)) < 1e-14


def test_later_pairs_turn_slower_by_the_geometric_frequency_ladder():
    """Pair i of a section of width n at position 1 turns by theta^(-2i/n): with theta = 16 and
    n = 8 the angles are 1, 1/2, 1/4, 1/8 radians."""
    x = np.zeros((1, 1, 1, 8))
    x[..., 0::2] = 1.0
    _, _, _, qo, _, _, _, _ = _run(B=1, H=1, grid=(1, 1), n_new=1, F=2, frame_pos=1, sections=(8, 0, 0), theta=16.0, q=x, k=x, v=x)
    for i, ang in enumerate((1.0, 0.5, 0.25, 0.125)):
        assert abs(qo[0, 0, 0, 2 * i] - np.cos(ang)) < 1e-14 and abs(qo[0, 0, 0, 2 * i + 1] - np.sin(ang)) < 1e-14


def test_rejects_bad_arguments():
    with pytest.raises(ValueError):
        _run(sections=(4, 6, 7))          # odd width (and wrong sum)
    with pytest.raises(ValueError):
        _run(sections=(3, 7, 6))          # odd widths
    with pytest.raises(ValueError):
        _run(F=2, frame_pos=1, n_new=2)   # beyond the capacity
    q = _rand((1, 1, 12, 16), 1)
    kc = np.zeros((1, 1, 24, 16))
    with pytest.raises(ValueError):
        orc.rope_kvcache_append(q, kc, kc, q, q, 12, 0, (3, 5), (4, 6, 6))  # grid does not match T
