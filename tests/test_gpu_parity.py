"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle on
the same seeded inputs.  Bounds are the ones the task states: bf16 max-abs <= 2e-2 and
relative L2 <= 1e-2; fp32 max-abs <= 1e-4.  A tighter internal bar on relative L2 catches
bugs that the loose max-abs bound would hide (outputs shrink like 1/sqrt(keys))."""
import numpy as np
import pytest
import torch

from oracle import nfd_oracle as orc
from paper_2506_01380_amd import binding as nb
from paper_2506_01380_amd import workloads as wl

pytestmark = pytest.mark.gpu

from parity_bounds import (BF16_MAX_ABS, BF16_REL_L2, BF16_REL_L2_INTERNAL, BF16_ROW_REL_L2, FP32_MAX_ABS, worst_row)


@pytest.fixture(scope="module")
def attn_bf16():
    a = nb.Attention("bf16")
    yield a
    a.close()


@pytest.fixture(scope="module")
def attn_fp32():
    a = nb.Attention("fp32")
    yield a
    a.close()


def to_dev(x, dtype):
    t = torch.from_numpy(x).cuda()
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def run_hip(attn, q, k, v, T, kvf, qf, dtype, scale=0.0):
    out = attn.forward(to_dev(q, dtype), to_dev(k, dtype), to_dev(v, dtype), T, kv_frames=kvf, q_frames=qf, scale=scale)
    torch.cuda.synchronize()
    return out.float().cpu().numpy().astype(np.float64)


def errors(got, ref):
    d = got - ref
    return float(np.abs(d).max()), float(np.linalg.norm(d) / np.linalg.norm(ref))


def check_bf16(got, ref, tag, row_bound=BF16_ROW_REL_L2):
    assert np.all(np.isfinite(got)), tag
    max_abs, rel = errors(got, ref)
    worst, where = worst_row(got, ref)
    print("%s: max_abs=%.3e rel_l2=%.3e row=%.3e" % (tag, max_abs, rel, worst), flush=True)
    assert max_abs <= BF16_MAX_ABS and rel <= BF16_REL_L2, (tag, max_abs, rel)
    assert rel <= BF16_REL_L2_INTERNAL, (tag, rel)
    assert worst <= row_bound, (tag, worst, where)


# ---- config c1: tiny fp32 -------------------------------------------------------------------
def test_c1_tiny_fp32(attn_fp32):
    cfg, q, k, v = wl.make_config("c1_tiny_fp32")
    got = run_hip(attn_fp32, q, k, v, cfg["T"], cfg["kv_frames"], cfg["q_frames"], "fp32")
    ref = orc.block_causal_attn(q, k, v, cfg["T"])
    max_abs, rel = errors(got, ref)
    print("c1: max_abs=%.3e rel_l2=%.3e" % (max_abs, rel), flush=True)
    assert max_abs <= FP32_MAX_ABS


@pytest.mark.parametrize("B,H,T,D,kvf,qf,F", [
    (1, 2, 5, 8, 6, 3, 7),       # odd T, narrow head, spare capacity
    (2, 3, 48, 128, 5, 5, 5),    # wide head
    (1, 1, 1, 64, 130, 130, 130),  # T = 1: plain causal attention over > 2 key chunks
    (1, 2, 200, 64, 1, 1, 1),    # one frame: full attention
    (1, 2, 37, 65, 4, 2, 4),     # odd head width
])
def test_general_kernel_fp32_shapes(attn_fp32, B, H, T, D, kvf, qf, F):
    q, k, v = wl.make_qkv(B, H, D, T, kvf, qf, F, "fp32", seed=wl.BASE_SEED + 100 + T)
    got = run_hip(attn_fp32, q, k, v, T, kvf, qf, "fp32")
    ref = orc.block_causal_attn(q, k, v, T, kv_frames=kvf, q_frames=qf)
    assert errors(got, ref)[0] <= FP32_MAX_ABS


def test_general_kernel_bf16_other_width(attn_bf16):
    B, H, T, D, kvf, qf = 1, 2, 24, 128, 6, 6
    q, k, v = wl.make_qkv(B, H, D, T, kvf, qf, kvf, "bf16", seed=wl.BASE_SEED + 120)
    got = run_hip(attn_bf16, q, k, v, T, kvf, qf, "bf16")
    check_bf16(got, orc.block_causal_attn(q, k, v, T), "generic bf16 D=128")


# ---- matrix-core kernel, every element, sizes spanning several tiles and ragged tails ----------
MFMA_CASES = [
    # B, H, T,   kvf, qf, F
    (1, 2, 16, 4, 4, 4),       # c1's shape in bf16: one partial tile
    (1, 3, 48, 7, 7, 7),       # 336 rows: 2 query tiles, ragged second; BH not a multiple of 8
    (2, 5, 40, 9, 9, 9),       # frames not aligned to the 64-key tiles; 10 heads over 8 XCDs
    (1, 2, 336, 3, 3, 3),      # the paper's frame size
    (1, 9, 100, 6, 1, 8),      # single-frame decode over a cache with spare capacity
    (1, 2, 336, 5, 2, 6),      # speculative, 2 frames
    (1, 1, 72, 12, 4, 12),     # speculative, 4 frames, key splits
    (1, 2, 1, 300, 300, 300),  # T = 1: causal attention, every tile on the diagonal is masked per row
    (1, 1, 7, 50, 50, 50),     # tiny odd frames
    (1, 2, 576, 2, 1, 2),      # long-context frame size, decode
]


@pytest.mark.parametrize("B,H,T,kvf,qf,F", MFMA_CASES)
def test_mfma_kernel_every_element(attn_bf16, B, H, T, kvf, qf, F):
    D = 64
    q, k, v = wl.make_qkv(B, H, D, T, kvf, qf, F, "bf16", seed=wl.BASE_SEED + 200 + T + kvf)
    if F > kvf:  # rows past kv_frames must never be read
        k[:, :, kvf * T:] = np.nan
        v[:, :, kvf * T:] = np.nan
    got = run_hip(attn_bf16, q, k, v, T, kvf, qf, "bf16")
    ref = orc.block_causal_attn(q, k, v, T, kv_frames=kvf, q_frames=qf)
    check_bf16(got, ref, "mfma B%d H%d T%d kv%d q%d" % (B, H, T, kvf, qf))


def test_mfma_custom_scale_and_large_scores(attn_bf16):
    B, H, T, D, F = 1, 2, 64, 64, 5
    q, k, v = wl.make_qkv(B, H, D, T, F, F, F, "bf16", seed=wl.BASE_SEED + 300)
    q = wl.round_to_bf16(q * 6.0)  # scores with std ~6: peaked softmax, frequent max updates
    got = run_hip(attn_bf16, q, k, v, T, F, F, "bf16", scale=0.2)
    ref = orc.block_causal_attn(q, k, v, T, scale=0.2)
    assert np.all(np.isfinite(got))
    max_abs, rel = errors(got, ref)
    print("peaked: max_abs=%.3e rel_l2=%.3e" % (max_abs, rel), flush=True)
    assert rel <= BF16_REL_L2


def _ramp_case(top, seed):
    """Scores that drift with the key index: q has a constant component, k the same component
    scaled by a ramp over the keys, so the row max moves by many powers of two from tile to tile."""
    B, H, T, D, F = 1, 2, 96, 64, 6
    q, k, v = wl.make_qkv(B, H, D, T, F, F, F, "bf16", seed=seed)
    ramp = np.linspace(0.0, top, F * T)  # score drift of `top` natural units over 576 keys (9 tiles)
    q[..., 0] = 8.0
    k[..., 0] = ramp[None, None, :]
    return B, H, T, D, F, wl.round_to_bf16(q), wl.round_to_bf16(k), v


def test_mfma_scores_rising_with_key_index(attn_bf16):
    """Every later tile outgrows the reference max of the earlier ones: the exact pass (tile max,
    rescale of the accumulators, P formed again) runs on every tile."""
    B, H, T, D, F, q, k, v = _ramp_case(100.0, wl.BASE_SEED + 310)  # 16 powers of two per tile
    got = run_hip(attn_bf16, q, k, v, T, F, F, "bf16")
    ref = orc.block_causal_attn(q, k, v, T)
    check_bf16(got, ref, "rising scores")


def test_mfma_scores_falling_with_key_index(attn_bf16):
    """The first tile holds the max; later tiles are formed against a reference far above them and
    their weights underflow towards zero without ever triggering the exact pass."""
    B, H, T, D, F, q, k, v = _ramp_case(-40.0, wl.BASE_SEED + 311)
    got = run_hip(attn_bf16, q, k, v, T, F, F, "bf16")
    ref = orc.block_causal_attn(q, k, v, T)
    check_bf16(got, ref, "falling scores")


def test_mfma_scores_just_below_and_above_the_redo_limit(attn_bf16):
    """One key per row sits 2^14..2^16 above the reference set by the first tile: tile sums land on
    both sides of the limit that decides between the stale reference and the exact pass."""
    B, H, T, D, F = 1, 1, 64, 64, 4
    q, k, v = wl.make_qkv(B, H, D, T, F, F, F, "bf16", seed=wl.BASE_SEED + 312)
    q[:] = 0.0
    k[:] = 0.0
    q[..., 0] = 1.0
    # scores are scale * k[...,0] = k/8; a score of x natural units is x*log2(e) powers of two
    for j, pw in zip((70, 135, 200), (14.0, 15.0, 16.0)):
        k[0, 0, j, 0] = 8.0 * pw / np.log2(np.e)
    q, k = wl.round_to_bf16(q), wl.round_to_bf16(k)
    got = run_hip(attn_bf16, q, k, v, T, F, F, "bf16")
    ref = orc.block_causal_attn(q, k, v, T)
    check_bf16(got, ref, "redo limit")


def test_mfma_uniform_scores_mean_of_visible_v(attn_bf16):
    """Q = 0: the output is the mean of the visible V rows (closed form), checked on the device path."""
    B, H, T, D, kvf, qf = 1, 2, 48, 64, 6, 3
    q, k, v = wl.make_qkv(B, H, D, T, kvf, qf, kvf, "bf16", seed=wl.BASE_SEED + 301)
    q[:] = 0
    got = run_hip(attn_bf16, q, k, v, T, kvf, qf, "bf16")
    for a in range(qf):
        mean = v[:, :, : (kvf - qf + a + 1) * T].astype(np.float64).mean(axis=2, keepdims=True)
        assert np.abs(got[:, :, a * T:(a + 1) * T] - mean).max() <= 2e-3


def test_future_frames_do_not_influence_past_rows_bitwise(attn_bf16):
    B, H, T, D, F = 1, 2, 80, 64, 6
    q, k, v = wl.make_qkv(B, H, D, T, F, F, F, "bf16", seed=wl.BASE_SEED + 302)
    base = run_hip(attn_bf16, q, k, v, T, F, F, "bf16")
    k2, v2 = k.copy(), v.copy()
    k2[:, :, 4 * T:] *= -3.0
    v2[:, :, 4 * T:] += 7.0
    pert = run_hip(attn_bf16, q, k2, v2, T, F, F, "bf16")
    assert np.array_equal(base[:, :, : 4 * T], pert[:, :, : 4 * T])
    assert not np.array_equal(base[:, :, 4 * T:], pert[:, :, 4 * T:])


# ---- the paper-shaped configs at full size --------------------------------------------------------
# Every element of every output, in the launch configuration the benchmark times.  Only the long training form is
# row-sampled (its oracle would take minutes): first and last row of each of its 64 frames + 64 random rows per frame.
FULL = ["c2_train", "c3_decode", "c4_spec_k2", "c4_spec_k4", "c4_spec_k8", "c5a_long_train", "c5b_batch_decode",
        "x_train_h12", "x_train_h24", "x_decode_h12", "x_decode_h24", "x_spec_k3"]  # x_: other model sizes, N = 3
SAMPLED = {"c5a_long_train": 64}


@pytest.mark.parametrize("name", FULL)
def test_full_size_configs(attn_bf16, name):
    cfg, q, k, v = wl.make_config(name)
    T, kvf, qf = cfg["T"], cfg["kv_frames"], cfg["q_frames"]
    got = run_hip(attn_bf16, q, k, v, T, kvf, qf, "bf16")
    if name in SAMPLED:
        rows = wl.sample_rows(T, qf, SAMPLED[name], cfg["seed"])
        ref = orc.block_causal_attn(q, k, v, T, kv_frames=kvf, q_frames=qf, rows=rows)
        check_bf16(got[:, :, rows], ref, name + " (%d sampled rows/head)" % len(rows))
    else:
        ref = orc.block_causal_attn(q, k, v, T, kv_frames=kvf, q_frames=qf)
        check_bf16(got, ref, name + " (every element)")
    # convexity holds at any size: every output lies inside the range of V (bf16 rounding slack)
    assert np.abs(got).max() <= np.abs(v[:, :, : kvf * T]).max() * 1.01


def test_cached_and_speculative_forms_equal_training_tail(attn_bf16):
    """Appendix B / Sec. 4.2: the cached forms are the tail rows of the full form."""
    cfg, q, k, v = wl.make_config("c4_spec_k4")
    T, kvf = cfg["T"], cfg["kv_frames"]
    B, H, D = cfg["B"], cfg["H"], cfg["D"]
    qfull = wl.randn((B, H, kvf * T, D), cfg["seed"] + 7, "bf16")
    kk, vv = k[:, :, : kvf * T].copy(), v[:, :, : kvf * T].copy()
    full = run_hip(attn_bf16, qfull, kk, vv, T, kvf, kvf, "bf16")
    for qf in (1, 4):
        tail = run_hip(attn_bf16, qfull[:, :, (kvf - qf) * T:].copy(), kk, vv, T, kvf, qf, "bf16")
        d = tail - full[:, :, (kvf - qf) * T:]
        assert np.linalg.norm(d) / np.linalg.norm(tail) <= 4e-3


# ---- KV cache append ----------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,T,D", [("bf16", 336, 64), ("fp32", 16, 64), ("bf16", 5, 3)])
def test_kvcache_append_bit_exact(attn_bf16, attn_fp32, dtype, T, D):
    attn = attn_bf16 if dtype == "bf16" else attn_fp32
    B, H, F, n, pos = 2, 3, 6, 2, 3
    kc = wl.randn((B, H, F * T, D), 1, dtype)
    vc = wl.randn((B, H, F * T, D), 2, dtype)
    kn = wl.randn((B, H, n * T, D), 3, dtype)
    vn = wl.randn((B, H, n * T, D), 4, dtype)
    dk, dv = to_dev(kc, dtype), to_dev(vc, dtype)
    attn.append(dk, dv, to_dev(kn, dtype), to_dev(vn, dtype), T, pos)
    torch.cuda.synchronize()
    assert np.array_equal(dk.float().cpu().numpy().astype(np.float64), orc.kvcache_append(kc, kn, T, pos))
    assert np.array_equal(dv.float().cpu().numpy().astype(np.float64), orc.kvcache_append(vc, vn, T, pos))
    with pytest.raises(nb.NfdError) as e:
        attn.append(dk, dv, to_dev(kn, dtype), to_dev(vn, dtype), T, F - 1)
    assert e.value.code == nb.NFD_ERR_CAPACITY


def test_decode_loop_with_append_and_rollback(attn_bf16):
    """Appendix A listing: frames are appended to the cache, a speculative chunk is attended,
    part of it is rejected, and generation resumes from the last accepted frame."""
    B, H, T, D, F = 1, 2, 48, 64, 8
    kc = torch.zeros((B, H, F * T, D), dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    ks = wl.randn((B, H, F * T, D), 11, "bf16")
    vs = wl.randn((B, H, F * T, D), 12, "bf16")
    past = 3
    attn_bf16.append(kc, vc, to_dev(ks[:, :, : past * T], "bf16"), to_dev(vs[:, :, : past * T], "bf16"), T, 0)
    # speculative chunk of 3 frames
    attn_bf16.append(kc, vc, to_dev(ks[:, :, past * T:(past + 3) * T], "bf16"),
                     to_dev(vs[:, :, past * T:(past + 3) * T], "bf16"), T, past)
    q3 = wl.randn((B, H, 3 * T, D), 13, "bf16")
    out3 = attn_bf16.forward(to_dev(q3, "bf16"), kc, vc, T, kv_frames=past + 3, q_frames=3)
    ref3 = orc.block_causal_attn(q3, ks, vs, T, kv_frames=past + 3, q_frames=3)
    check_bf16(out3.float().cpu().numpy().astype(np.float64), ref3, "spec chunk")
    # reject the last two: next frame overwrites position past+1 with different content
    k_alt = wl.randn((B, H, T, D), 14, "bf16")
    v_alt = wl.randn((B, H, T, D), 15, "bf16")
    attn_bf16.append(kc, vc, to_dev(k_alt, "bf16"), to_dev(v_alt, "bf16"), T, past + 1)
    q1 = wl.randn((B, H, T, D), 16, "bf16")
    out1 = attn_bf16.forward(to_dev(q1, "bf16"), kc, vc, T, kv_frames=past + 2, q_frames=1)
    ks2, vs2 = ks.copy(), vs.copy()
    ks2[:, :, (past + 1) * T:(past + 2) * T] = k_alt
    vs2[:, :, (past + 1) * T:(past + 2) * T] = v_alt
    ref1 = orc.block_causal_attn(q1, ks2, vs2, T, kv_frames=past + 2, q_frames=1)
    check_bf16(out1.float().cpu().numpy().astype(np.float64), ref1, "after rollback")


def test_error_codes_on_device(attn_bf16):
    t = torch.zeros((1, 1, 16, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(nb.NfdError) as e:
        nb.nfd_block_causal_attn_fwd(attn_bf16.h, t, t, None, t, 1, 1, 1, 16, 64, 1, 1)
    assert e.value.code == nb.NFD_ERR_NULL
    with pytest.raises(nb.NfdError) as e:
        nb.nfd_block_causal_attn_fwd(attn_bf16.h, t, t, t, t, 1, 1, 1, 16, 64, 2, 1)
    assert e.value.code == nb.NFD_ERR_CAPACITY
    with pytest.raises(nb.NfdError) as e:
        nb.nfd_block_causal_attn_fwd(attn_bf16.h, t, t, t, t, 1, 1, 1, 16, 64, 1, 2)
    assert e.value.code == nb.NFD_ERR_SHAPE


def test_empty_appends_are_no_ops(attn_bf16):
    """n_frames == 0: nothing is launched, nothing changes - for the plain and the rotary append."""
    B, H, T, D, F = 1, 2, 16, 64, 3
    kc = torch.randn(B, H, F * T, D, device="cuda").to(torch.bfloat16)
    vc = torch.randn(B, H, F * T, D, device="cuda").to(torch.bfloat16)
    k0, v0 = kc.clone(), vc.clone()
    empty = torch.empty(B, H, 0, D, device="cuda", dtype=torch.bfloat16)
    dummy = torch.zeros(8, device="cuda", dtype=torch.bfloat16)  # a valid pointer for the zero-row tensors
    nb.nfd_kvcache_append(attn_bf16.h, kc, vc, dummy, dummy, B, H, F, T, D, 1, 0)
    nb.nfd_rope_kvcache_append(attn_bf16.h, dummy, dummy, kc, vc, dummy, dummy, B, H, F, T, D, 3, 0, 0, 4, 4, 16, 24, 24)
    nb.nfd_kvcache_shift(attn_bf16.h, kc, vc, B, H, F, T, D, 0, 0)
    torch.cuda.synchronize()
    assert torch.equal(kc, k0) and torch.equal(vc, v0) and empty.numel() == 0


def test_misaligned_views_are_refused_not_faulted(attn_bf16):
    """A bf16 view that starts 2 bytes into a 16-byte vector must come back as an error code."""
    B, H, T, D, F = 1, 1, 16, 64, 2
    buf = torch.zeros(B * H * F * T * D + 8, dtype=torch.bfloat16, device="cuda")
    q = buf[1:1 + B * H * F * T * D].view(B, H, F * T, D)
    ok = buf[:B * H * F * T * D].view(B, H, F * T, D)
    assert q.data_ptr() % 16 != 0
    with pytest.raises(nb.NfdError) as e:
        nb.nfd_block_causal_attn_fwd(attn_bf16.h, q, ok, ok, torch.empty_like(ok), B, H, F, T, D, F, F)
    assert e.value.code == nb.NFD_ERR_UNSUPPORTED


def test_runs_are_bit_reproducible(attn_bf16):
    cfg, q, k, v = wl.make_config("c4_spec_k2")
    a = run_hip(attn_bf16, q, k, v, cfg["T"], cfg["kv_frames"], cfg["q_frames"], "bf16")
    b = run_hip(attn_bf16, q, k, v, cfg["T"], cfg["kv_frames"], cfg["q_frames"], "bf16")
    assert np.array_equal(a, b)


def test_wrapper_methods_validate_their_tensors(attn_bf16):
    """A wrong dtype, a strided view, a host tensor or a length that is not a multiple of T must raise in the
    binding instead of reaching the device as a wrong stride."""
    B, H, T, D, F = 1, 2, 16, 64, 3
    mk = lambda *s: torch.zeros(*s, dtype=torch.bfloat16, device="cuda")
    q, k, v = mk(B, H, F * T, D), mk(B, H, F * T, D), mk(B, H, F * T, D)
    out, lse = attn_bf16.forward_lse(q, k, v, T)
    bad_sets = [
        dict(k=k.float()),                                       # dtype of the handle
        dict(k=mk(B, H, F * T, 2 * D)[..., ::2]),                # not contiguous
        dict(v=v.cpu()),                                         # not on the device
        dict(k=mk(B, H, F * T + 1, D), v=mk(B, H, F * T + 1, D)),  # cache length not a multiple of T
        dict(v=mk(B, H, 2 * F * T, D)),                          # k and v disagree
        dict(q=mk(B, H + 1, F * T, D)),                          # heads disagree
    ]
    for bad in bad_sets:
        a = dict(q=q, k=k, v=v)
        a.update(bad)
        for call in (lambda: attn_bf16.forward(a["q"], a["k"], a["v"], T),
                     lambda: attn_bf16.forward_lse(a["q"], a["k"], a["v"], T),
                     lambda: attn_bf16.backward(a["q"], a["k"], a["v"], out, out, lse, T)):
            with pytest.raises(ValueError):
                call()
    with pytest.raises(ValueError):
        attn_bf16.backward(q, k, v, out, out, lse.double(), T)
    kn = mk(B, H, T, D)
    for bad in (dict(k_new=kn.float()), dict(k_new=mk(B, H, T + 1, D), v_new=mk(B, H, T + 1, D)), dict(v_cache=v.cpu()),
                dict(k_new=mk(B, H + 1, T, D), v_new=mk(B, H + 1, T, D))):
        a = dict(k_cache=k, v_cache=v, k_new=kn, v_new=kn)
        a.update(bad)
        with pytest.raises(ValueError):
            attn_bf16.append(a["k_cache"], a["v_cache"], a["k_new"], a["v_new"], T, 0)
        with pytest.raises(ValueError):
            attn_bf16.rope_append(kn, a["k_cache"], a["v_cache"], a["k_new"], a["v_new"], T, 0, (4, 4), (16, 24, 24))
    with pytest.raises(ValueError):
        attn_bf16.rope_append(mk(B, H, 2 * T, D), k, v, kn, kn, T, 0, (4, 4), (16, 24, 24))  # q and the new frames disagree
    torch.cuda.synchronize()


# ---- append fused into the attention launch ---------------------------------------------------------
@pytest.mark.parametrize("name,B,H,T,D,kvf,qf,F,dtype", [
    ("c3_decode", None, None, None, None, None, None, None, "bf16"),   # one launch: copy by the attention workgroups
    ("c4_spec_k4", None, None, None, None, None, None, None, "bf16"),
    ("c4_spec_k2", None, None, None, None, None, None, None, "bf16"),
    ("c4_spec_k8", None, None, None, None, None, None, None, "bf16"),
    ("c5b_batch_decode", None, None, None, None, None, None, None, "bf16"),  # the batched step bench.py times
    (None, 2, 3, 40, 64, 9, 3, 11, "bf16"),     # odd frames, spare capacity, heads not a multiple of 8
    (None, 1, 2, 48, 64, 5, 5, 6, "bf16"),      # no past frames: everything is "new"
    (None, 1, 1, 16, 64, 40, 39, 40, "bf16"),   # many new rows for few workgroups: the two-launch path
    (None, 1, 2, 24, 128, 6, 2, 7, "bf16"),     # general kernel (other head width): two launches
    (None, 1, 2, 16, 64, 4, 1, 4, "fp32"),      # fp32 handle: two launches
])
def test_fused_append_equals_append_then_forward(attn_bf16, attn_fp32, name, B, H, T, D, kvf, qf, F, dtype):
    """nfd_kvcache_append_attn_fwd against the two calls it replaces: out and both caches bit for bit; the rows of
    the cache that the call overwrites hold NaN beforehand, so reading them would show; and against the oracle."""
    attn = attn_bf16 if dtype == "bf16" else attn_fp32
    if name:
        cfg, q, k, v = wl.make_config(name)
        B, H, T, D, kvf, qf, F = (cfg[x] for x in ("B", "H", "T", "D", "kv_frames", "q_frames", "F"))
    else:
        q, k, v = wl.make_qkv(B, H, D, T, kvf, qf, F, dtype, seed=wl.BASE_SEED + 800 + T + kvf)
    P = kvf - qf
    kn, vn = k[:, :, P * T: kvf * T].copy(), v[:, :, P * T: kvf * T].copy()
    k0, v0 = k.copy(), v.copy()
    k0[:, :, P * T:] = np.nan   # the new frames' slots and the spare capacity: never to be read
    v0[:, :, P * T:] = np.nan
    qd, knd, vnd = to_dev(q, dtype), to_dev(kn, dtype), to_dev(vn, dtype)
    # two calls
    ka, va = to_dev(k0, dtype), to_dev(v0, dtype)
    want = torch.empty_like(qd)
    nb.nfd_kvcache_append(attn.h, ka, va, knd, vnd, B, H, F, T, D, P, qf)
    nb.nfd_block_causal_attn_fwd(attn.h, qd, ka, va, want, B, H, F, T, D, kvf, qf)
    # one call
    kb, vb = to_dev(k0, dtype), to_dev(v0, dtype)
    got = torch.full_like(qd, float("nan"))
    nb.nfd_kvcache_append_attn_fwd(attn.h, qd, kb, vb, knd, vnd, got, B, H, F, T, D, kvf, qf)
    torch.cuda.synchronize()
    assert torch.equal(got, want)
    same = lambda a, b: torch.equal(a.view(torch.int16 if dtype == "bf16" else torch.int32), b.view(torch.int16 if dtype == "bf16" else torch.int32))
    assert same(ka, kb) and same(va, vb)          # NaN rows past kv_frames compare by bit pattern
    hk = kb.float().cpu().numpy()
    assert np.array_equal(hk[:, :, : kvf * T], k[:, :, : kvf * T])
    assert np.all(np.isnan(hk[:, :, kvf * T:]))
    del hk
    g = got.float().cpu().numpy().astype(np.float64)
    if name == "c5b_batch_decode":
        # every row of two of the eight sequences against the oracle here (test_full_size_configs checks all eight on the
        # two-call form, to which this call's output is compared bit for bit above)
        ref = orc.block_causal_attn(q[:2], k[:2], v[:2], T, kv_frames=kvf, q_frames=qf)
        g = g[:2]
    else:
        ref = orc.block_causal_attn(q, k, v, T, kv_frames=kvf, q_frames=qf)
    if dtype == "bf16":
        check_bf16(g, ref, "fused append %s" % (name or "B%d H%d T%d D%d" % (B, H, T, D)))
    else:
        assert errors(g, ref)[0] <= FP32_MAX_ABS
    with pytest.raises(nb.NfdError) as e:
        nb.nfd_kvcache_append_attn_fwd(attn.h, qd, kb, vb, None, vnd, got, B, H, F, T, D, kvf, qf)
    assert e.value.code == nb.NFD_ERR_NULL
