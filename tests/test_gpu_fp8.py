"""GPU parity of the 8-bit (E4M3) KV cache through the C ABI: the quantising append bit for bit against the
oracle's codes, the attention over the 8-bit cache against the fp64 oracle on the values those codes
stand for (same bound as the bf16 cache: the codes widen to bf16 exactly, so the arithmetic between the
operands is the bf16 kernel's)."""
import numpy as np
import pytest
from parity_bounds import BF16_ROW_REL_L2, worst_row
import torch

from oracle import fp8_cache as f8
from paper_2506_01380_amd import binding as nb
from paper_2506_01380_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL_MAX_ABS, TOL_REL_L2 = 2e-2, 1e-2
NAN_CODE = 0x7F


@pytest.fixture(scope="module")
def attn():
    a = nb.Attention("bf16")
    yield a
    a.close()


def _bf16(x):
    return torch.from_numpy(x).cuda().to(torch.bfloat16)


def _spad(F, T):
    return (F * T + 63) // 64 * 64


def _caches(B, H, F, T, D=64, fill=NAN_CODE):
    n = nb.nfd_fp8_cache_bytes(B, H, F, T, D)
    assert n == B * H * _spad(F, T) * D
    k8 = torch.full((n,), fill, dtype=torch.uint8, device="cuda")
    v8 = torch.full((n,), fill, dtype=torch.uint8, device="cuda")
    return k8, v8


def _scales(B, H, seed, lo=0.01, hi=0.05):
    rng = np.random.default_rng(seed)
    return (rng.uniform(lo, hi, size=(B, H)).astype(np.float32), rng.uniform(lo, hi, size=(B, H)).astype(np.float32))


def _v_position(j, s):
    """Byte position of key j inside a feature row of the library's V cache (s = bit 4 of the feature index): keys
    are permuted inside aligned groups of 16 so that keys 4h..4h+3 and 8+4h..8+4h+3 sit in 8 consecutive bytes
    at byte 8 * (h ^ s) of the group (see include/nfd_attn.h)."""
    q = j & 15
    return (j & ~15) | (8 * (((q >> 2) & 1) ^ s) + 4 * (q >> 3) + (q & 3))


def _v_logical(hv):
    """Device bytes [B, H, D, S] -> plain key order."""
    S = hv.shape[3]
    j = np.arange(S)
    out = np.empty_like(hv)
    for d in range(hv.shape[2]):
        out[:, :, d, :] = hv[:, :, d, _v_position(j, (d >> 4) & 1)]
    return out


def _v_physical(lv):
    S = lv.shape[3]
    j = np.arange(S)
    out = np.empty_like(lv)
    for d in range(lv.shape[2]):
        out[:, :, d, _v_position(j, (d >> 4) & 1)] = lv[:, :, d, :]
    return out


def _host_views(k8, v8, B, H, F, T, D=64):
    S = _spad(F, T)
    return k8.cpu().numpy().reshape(B, H, S, D), _v_logical(v8.cpu().numpy().reshape(B, H, D, S))


def _append(attn, k8, v8, ks, vs, kn, vn, B, H, F, T, pos):
    ksd, vsd = torch.from_numpy(ks).cuda(), torch.from_numpy(vs).cuda()
    nb.nfd_kvcache_append_fp8(attn.h, k8, v8, ksd, vsd, _bf16(kn), _bf16(vn), B, H, F, T, 64, pos, kn.shape[2] // T)
    torch.cuda.synchronize()
    return ksd, vsd


@pytest.mark.parametrize("B,H,T,F,pos,n", [(1, 2, 16, 4, 1, 2), (2, 3, 5, 7, 0, 7), (1, 16, 336, 3, 2, 1), (1, 1, 1, 70, 3, 64),
                                           (1, 9, 37, 5, 1, 3)])
def test_append_codes_are_bit_exact(attn, B, H, T, F, pos, n):
    D = 64
    rng = np.random.default_rng(wl.BASE_SEED + 40 + T)
    kn = wl.round_to_bf16(rng.standard_normal((B, H, n * T, D)).astype(np.float32))
    vn = wl.round_to_bf16((rng.standard_normal((B, H, n * T, D)) * rng.choice([1e-3, 0.05, 1.0, 40.0], size=(B, H, n * T, D)))
                          .astype(np.float32))  # subnormal codes up to saturation
    ks, vs = _scales(B, H, T)
    k8, v8 = _caches(B, H, F, T)
    _append(attn, k8, v8, ks, vs, kn, vn, B, H, F, T, pos)
    gk, gv = _host_views(k8, v8, B, H, F, T)
    rk = np.full_like(gk, NAN_CODE)
    rv = np.full_like(gv, NAN_CODE)
    f8.kvcache_append_fp8(rk, rv, kn, vn, T, pos, ks, vs)
    assert np.array_equal(gk, rk), "K codes differ at %d places" % int((gk != rk).sum())
    assert np.array_equal(gv, rv), "V codes differ at %d places" % int((gv != rv).sum())
    assert (rv == 0x7E).any() or (rv == 0xFE).any()  # the saturating branch was exercised


def test_append_rounds_every_tie_to_even(attn):
    """Scale 1 and inputs that are exact midpoints between neighbouring codes (bf16 holds them all)."""
    B, H, T, D, F = 1, 1, 64, 64, 2
    codes = np.arange(0, 0x7E, dtype=np.uint8)
    mids = ((f8.e4m3_decode(codes) + f8.e4m3_decode(codes + 1)) / 2).astype(np.float32)
    assert np.array_equal(wl.round_to_bf16(mids), mids)
    x = np.resize(np.concatenate([mids, -mids]), (B, H, T, D)).astype(np.float32)
    one = np.ones((B, H), dtype=np.float32)
    k8, v8 = _caches(B, H, F, T)
    _append(attn, k8, v8, one, one, x, x, B, H, F, T, 0)
    gk, gv = _host_views(k8, v8, B, H, F, T)
    want = f8.e4m3_encode(x)
    assert np.array_equal(gk[:, :, :T], want)
    assert np.array_equal(gv[:, :, :, :T], np.swapaxes(want, 2, 3))


def _run(attn, B, H, T, kvf, qf, F, seed, scale=0.0):
    D = 64
    q, k, v = wl.make_qkv(B, H, D, T, kvf, qf, kvf, "bf16", seed=seed)
    ks, vs = _scales(B, H, seed)
    k8, v8 = _caches(B, H, F, T)                       # everything outside the appended frames holds NaN codes
    ksd, vsd = _append(attn, k8, v8, ks, vs, k, v, B, H, F, T, 0)
    qd = _bf16(q)
    out = torch.empty_like(qd)
    nb.nfd_block_causal_attn_fwd_fp8kv(attn.h, qd, k8, v8, ksd, vsd, out, B, H, F, T, D, kvf, qf, scale)
    torch.cuda.synchronize()
    hk, hv = _host_views(k8, v8, B, H, F, T)
    ref = f8.block_causal_attn_fp8kv(q, hk, hv, ks, vs, T, kvf, qf, scale=None if scale <= 0 else scale)
    return out.float().cpu().numpy().astype(np.float64), ref


def _check(got, ref, tag):
    assert np.all(np.isfinite(got)), tag
    d = got - ref
    mx, rel = float(np.abs(d).max()), float(np.linalg.norm(d) / np.linalg.norm(ref))
    print("%s: max_abs=%.3e rel_l2=%.3e" % (tag, mx, rel), flush=True)
    assert mx <= TOL_MAX_ABS and rel <= TOL_REL_L2, (tag, mx, rel)
    worst, where = worst_row(got, ref)
    assert worst <= BF16_ROW_REL_L2, (tag, worst, where)


CASES = [
    # B, H, T,  kvf, qf, F
    (1, 2, 16, 4, 4, 4),        # one tile, part of it past the end of the cache
    (1, 3, 48, 7, 7, 7),        # 336 keys: ragged last tile, heads not a multiple of 8
    (2, 5, 40, 9, 9, 10),       # frames not aligned to tiles, spare capacity
    (1, 2, 336, 3, 3, 3),       # the paper's frame size
    (1, 8, 100, 12, 2, 14),     # cached form with key splits
    (1, 16, 336, 5, 1, 6),      # single-frame decode: the 32-row workgroup shape
    (1, 1, 1, 300, 300, 300),   # T = 1: plain causal attention
    (1, 1, 7, 50, 50, 50),      # tiny odd frames: the cache end falls inside a 4-key word
    (1, 2, 576, 2, 2, 2),       # long-context frame size
]


@pytest.mark.parametrize("B,H,T,kvf,qf,F", CASES)
def test_attention_over_the_8bit_cache(attn, B, H, T, kvf, qf, F):
    got, ref = _run(attn, B, H, T, kvf, qf, F, wl.BASE_SEED + 500 + T + kvf)
    _check(got, ref, "fp8kv B%d H%d T%d kv%d q%d" % (B, H, T, kvf, qf))


@pytest.mark.parametrize("name", ["c3_decode", "c4_spec_k4"])
def test_attention_over_the_8bit_cache_full_size(attn, name):
    """The decode and speculative configurations at their full size, every element."""
    c = wl.CONFIGS[name]
    got, ref = _run(attn, c["B"], c["H"], c["T"], c["kv_frames"], c["q_frames"], c["F"], c["seed"] + 77)
    _check(got, ref, "fp8kv " + name)


def test_custom_scale_and_plan_shapes(attn):
    got, ref = _run(attn, 1, 4, 64, 6, 3, 6, wl.BASE_SEED + 590, scale=0.2)
    _check(got, ref, "fp8kv custom scale")
    assert nb.nfd_attn_plan(nb.NFD_BF16, 1, 16, 6, 336, 64, 5, 1)["block_m"] == 128
    assert nb.nfd_attn_plan(nb.NFD_BF16, 1, 8, 14, 100, 64, 12, 2)["n_splits"] > 1


@pytest.mark.parametrize("B,H,T,F,kvf,drop,ws", [
    (1, 2, 16, 6, 6, 4, 0),      # keep <= drop: one disjoint copy; 16-byte vectors
    (2, 3, 48, 8, 7, 2, 0),      # overlapping: through the workspace
    (1, 2, 5, 9, 9, 2, 0),       # T not a multiple of 16: V moves key by key through the workspace
    (1, 2, 5, 9, 9, 2, 4096),    # ... in two batches of feature rows (117 + 11)
    (1, 3, 37, 6, 5, 1, 0),
    (1, 2, 48, 8, 8, 3, 4096),   # a workspace too small for staging: runs of n_drop frames
    (1, 1, 7, 5, 4, 4, 0),       # everything dropped: nothing moves
])
def test_shift_of_the_8bit_cache(B, H, T, F, kvf, drop, ws):
    """Integer work: bit-exact.  Expected values: the frames kept, moved to the front (frames at and after
    the kept count are unspecified, as for the bf16 cache)."""
    D = 64
    a = nb.Attention("bf16", workspace_bytes=ws) if ws else nb.Attention("bf16")
    try:
        S = _spad(F, T)
        rng = np.random.default_rng(T + F)
        hk = rng.integers(0, 256, size=(B, H, S, D), dtype=np.uint8)
        hv = rng.integers(0, 256, size=(B, H, D, S), dtype=np.uint8)  # in plain key order
        k8, v8 = torch.from_numpy(hk.reshape(-1)).cuda(), torch.from_numpy(_v_physical(hv).reshape(-1)).cuda()
        nb.nfd_kvcache_shift_fp8(a.h, k8, v8, B, H, F, T, D, kvf, drop)
        torch.cuda.synchronize()
        gk, gv = _host_views(k8, v8, B, H, F, T)
        keep = kvf - drop
        assert np.array_equal(gk[:, :, :keep * T], hk[:, :, drop * T: kvf * T])
        assert np.array_equal(gv[:, :, :, :keep * T], hv[:, :, :, drop * T: kvf * T])
        assert np.array_equal(gk[:, :, kvf * T:], hk[:, :, kvf * T:]) and np.array_equal(gv[:, :, :, kvf * T:], hv[:, :, :, kvf * T:])
    finally:
        a.close()


def test_error_codes(attn):
    B, H, T, D, F = 1, 1, 16, 64, 2
    k8, v8 = _caches(B, H, F, T)
    s = torch.ones((B, H), dtype=torch.float32, device="cuda")
    x = torch.zeros((B, H, T, D), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(nb.NfdError) as e:
        nb.nfd_kvcache_append_fp8(attn.h, k8, v8, s, s, x, x, B, H, F, T, D, 2, 1)
    assert e.value.code == nb.NFD_ERR_CAPACITY
    with pytest.raises(nb.NfdError) as e:
        nb.nfd_kvcache_append_fp8(attn.h, k8, v8, None, s, x, x, B, H, F, T, D, 0, 1)
    assert e.value.code == nb.NFD_ERR_NULL
    with pytest.raises(nb.NfdError) as e:
        nb.nfd_kvcache_append_fp8(attn.h, k8, v8, s, s, x, x, B, H, F, T, 32, 0, 1)
    assert e.value.code == nb.NFD_ERR_UNSUPPORTED
    with pytest.raises(nb.NfdError) as e:
        nb.nfd_block_causal_attn_fwd_fp8kv(attn.h, x, k8, v8, s, None, x, B, H, F, T, D, 1, 1)
    assert e.value.code == nb.NFD_ERR_NULL
    with pytest.raises(nb.NfdError) as e:
        nb.nfd_block_causal_attn_fwd_fp8kv(attn.h, x, k8, v8, s, s, x, B, H, F, T, D, 3, 1)
    assert e.value.code == nb.NFD_ERR_CAPACITY
    with pytest.raises(nb.NfdError) as e:
        nb.nfd_block_causal_attn_fwd_fp8kv(attn.h, x, k8, v8, s, s, x, B, H, F, T, 128, 1, 1)
    assert e.value.code == nb.NFD_ERR_UNSUPPORTED
    a32 = nb.Attention("fp32")
    try:
        with pytest.raises(nb.NfdError) as e:
            nb.nfd_kvcache_append_fp8(a32.h, k8, v8, s, s, x, x, B, H, F, T, D, 0, 1)
        assert e.value.code == nb.NFD_ERR_UNSUPPORTED
    finally:
        a32.close()
    # key-wise V move (T not a multiple of 16) with a workspace that cannot hold one feature row
    tiny = nb.Attention("bf16", workspace_bytes=16)
    try:
        k8b, v8b = _caches(1, 1, 4, 7)
        with pytest.raises(nb.NfdError) as e:
            nb.nfd_kvcache_shift_fp8(tiny.h, k8b, v8b, 1, 1, 4, 7, D, 4, 1)
        assert e.value.code == nb.NFD_ERR_ALLOC
        with pytest.raises(nb.NfdError) as e:
            nb.nfd_kvcache_shift_fp8(tiny.h, k8b, v8b, 1, 1, 4, 7, D, 5, 1)
        assert e.value.code == nb.NFD_ERR_CAPACITY
        nb.nfd_kvcache_shift_fp8(tiny.h, k8b, v8b, 1, 1, 4, 7, D, 3, 0)  # nothing to drop: no launch, no error
    finally:
        tiny.close()


@pytest.mark.parametrize("T", [48, 20])  # 48: whole 16-key groups move; 20: V moves key by key
def test_speculative_decode_loop_over_the_8bit_cache(T):
    """The library's speculative bookkeeping driving the 8-bit cache: eviction (shift), quantising append of the
    generated frames, attention, accept/reject with rollback.  A host mirror of the codes is kept with the
    oracle's quantiser; codes are compared bit for bit and every step's attention with the fp64 oracle."""
    from oracle import spec_driver as sd
    B, H, D = 1, 3, 64
    total, n_prompt, nframe, window, F = 18, 2, 3, 5, 8
    rng = np.random.default_rng(500 + T)
    actions = np.repeat(rng.integers(0, 3, size=(total, 1)), rng.integers(1, 5, size=total), axis=0)[:total].astype(np.int32)
    mk = lambda: wl.round_to_bf16(rng.standard_normal((total, B, H, T, D)).astype(np.float32))
    Q, K, V = mk(), mk(), mk()
    frames = lambda X, idx: np.ascontiguousarray(np.concatenate([X[f] for f in idx], axis=2))
    ks, vs = _scales(B, H, T, 0.01, 0.02)
    a = nb.Attention("bf16")
    try:
        k8, v8 = _caches(B, H, F, T)
        S = _spad(F, T)
        hk = np.full((B, H, S, D), NAN_CODE, dtype=np.uint8)
        hv = np.full((B, H, D, S), NAN_CODE, dtype=np.uint8)
        prompt = list(range(n_prompt))
        ksd, vsd = _append(a, k8, v8, ks, vs, frames(K, prompt), frames(V, prompt), B, H, F, T, 0)
        f8.kvcache_append_fp8(hk, hv, frames(K, prompt), frames(V, prompt), T, 0, ks, vs)
        s = nb.nfd_spec_init(F, window, nframe, n_prompt, total)
        expect = sd.run(actions, n_prompt, nframe, window, F)
        n_steps = 0
        while True:
            st = nb.nfd_spec_next(s)
            if st is None:
                break
            ex = expect[n_steps]
            n_steps += 1
            if st.n_drop:
                kv_before = st.frame_pos + st.n_drop
                nb.nfd_kvcache_shift_fp8(a.h, k8, v8, B, H, F, T, D, kv_before, st.n_drop)
                keep = (kv_before - st.n_drop) * T
                hk[:, :, :keep] = hk[:, :, st.n_drop * T: kv_before * T].copy()
                hv[:, :, :, :keep] = hv[:, :, :, st.n_drop * T: kv_before * T].copy()
            gen = ex["generated"]
            qn, kn, vn = frames(Q, gen), frames(K, gen), frames(V, gen)
            nb.nfd_kvcache_append_fp8(a.h, k8, v8, ksd, vsd, _bf16(kn), _bf16(vn), B, H, F, T, D, st.frame_pos, st.n_frames)
            f8.kvcache_append_fp8(hk, hv, kn, vn, T, st.frame_pos, ks, vs)
            qd = _bf16(qn)
            out = torch.empty_like(qd)
            nb.nfd_block_causal_attn_fwd_fp8kv(a.h, qd, k8, v8, ksd, vsd, out, B, H, F, T, D, st.kv_frames, st.q_frames)
            torch.cuda.synchronize()
            n_valid = st.kv_frames * T
            gk, gv = _host_views(k8, v8, B, H, F, T)
            assert np.array_equal(gk[:, :, :n_valid], hk[:, :, :n_valid]), "step %d: K codes" % n_steps
            assert np.array_equal(gv[:, :, :, :n_valid], hv[:, :, :, :n_valid]), "step %d: V codes" % n_steps
            ref = f8.block_causal_attn_fp8kv(qn, hk, hv, ks, vs, T, st.kv_frames, st.q_frames)
            d = out.float().cpu().numpy() - ref
            assert np.abs(d).max() <= TOL_MAX_ABS and np.linalg.norm(d) / np.linalg.norm(ref) <= 5e-3, n_steps
            assert nb.nfd_spec_accept(s, st, actions) == ex["kept"]
        assert n_steps == len(expect) and s.done == total
    finally:
        a.close()


@pytest.mark.parametrize("B,H,grid,F,pos,n", [(1, 2, (6, 8), 5, 1, 2), (2, 3, (5, 7), 4, 0, 3), (1, 16, (24, 14), 3, 2, 1)])
def test_fused_rotary_and_quantising_append(attn, B, H, grid, F, pos, n):
    """One call (rotate q and k, quantise k and v into the 8-bit caches) against the two calls it replaces: rotary
    pre-op into a bf16 buffer, then the quantising append - identical codes and identical rotated queries, and
    untouched bytes everywhere else.  The two-call path is itself checked against the oracle: rotated keys within
    one bf16 step, and the codes the oracle's quantiser gives for the device's rotated keys, bit for bit."""
    from oracle import nfd_oracle as orc
    D, sections = 64, (16, 24, 24)
    T = grid[0] * grid[1]
    rng = np.random.default_rng(900 + T)
    qn, kn, vn = (wl.round_to_bf16(rng.standard_normal((B, H, n * T, D)).astype(np.float32)) for _ in range(3))
    ks, vs = _scales(B, H, T, 0.01, 0.03)
    ksd, vsd = torch.from_numpy(ks).cuda(), torch.from_numpy(vs).cuda()
    qd, kd, vd = _bf16(qn), _bf16(kn), _bf16(vn)
    # two calls
    kt = torch.zeros((B, H, n * T, D), dtype=torch.bfloat16, device="cuda")
    vt = torch.zeros_like(kt)
    q_two = attn.rope_append(qd, kt, vt, kd, vd, T, 0, grid, sections, t_offset=pos)  # temporal position = pos + frame
    k8a, v8a = _caches(B, H, F, T)
    nb.nfd_kvcache_append_fp8(attn.h, k8a, v8a, ksd, vsd, kt, vt, B, H, F, T, D, pos, n)
    # one call
    k8b, v8b = _caches(B, H, F, T)
    q_one = torch.empty_like(qd)
    nb.nfd_rope_kvcache_append_fp8(attn.h, qd, q_one, k8b, v8b, ksd, vsd, kd, vd, B, H, F, T, D, pos, n, 0,
                                   grid[0], grid[1], sections[0], sections[1], sections[2])
    torch.cuda.synchronize()
    assert torch.equal(q_one, q_two)
    assert torch.equal(k8a, k8b) and torch.equal(v8a, v8b)
    # the two-call path against the oracle
    zeros = np.zeros((B, H, n * T, D))
    rq, rk, rv = orc.rope_kvcache_append(qn, zeros, zeros.copy(), kn, vn, T, 0, grid, sections, t_offset=pos)
    dk = kt.float().cpu().numpy().astype(np.float64)
    assert np.all(np.abs(dk - rk) <= np.abs(rk) * 2.0 ** -8 + 1e-6)
    gk, gv = _host_views(k8b, v8b, B, H, F, T)
    assert np.array_equal(gk[:, :, pos * T:(pos + n) * T], f8.quantize(dk, ks[:, :, None, None]))
    assert np.array_equal(gv[:, :, :, pos * T:(pos + n) * T], np.swapaxes(f8.quantize(vn, vs[:, :, None, None]), 2, 3))
    assert np.all(gk[:, :, :pos * T] == NAN_CODE) and np.all(gk[:, :, (pos + n) * T:] == NAN_CODE)
    assert np.all(gv[:, :, :, :pos * T] == NAN_CODE) and np.all(gv[:, :, :, (pos + n) * T:] == NAN_CODE)
