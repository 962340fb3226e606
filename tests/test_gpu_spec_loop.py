"""GPU: the sliding-window cache move (bit-exact against the plain statement) and a whole
speculative decode loop driven by the library's bookkeeping - eviction, rotary embedding +
cache write, attention, accept/reject, rollback - with every kept frame's attention output
checked against the fp64 oracle run on a host copy of the same cache."""
import numpy as np
import pytest
from parity_bounds import BF16_ROW_REL_L2, worst_row
import torch

from oracle import nfd_oracle as orc
from oracle import spec_driver as sd
from paper_2506_01380_amd import binding as nb
from paper_2506_01380_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _dev(x):
    return torch.from_numpy(x).cuda().to(torch.bfloat16)


def _host(t):
    return t.float().cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("workspace,kv,drop", [
    (0, 7, 5),          # kept frames fit in the dropped range: one disjoint copy
    (0, 7, 2),          # overlapping: through the workspace
    (4096, 7, 2),       # workspace too small: runs of n_drop frames
    (4096, 6, 1),       # ... one frame at a time
    (0, 5, 0), (0, 5, 5),  # nothing to do
])
def test_kvcache_shift_bit_exact(workspace, kv, drop):
    B, H, T, D, F = 2, 3, 24, 64, 8
    a = nb.Attention("bf16", workspace_bytes=workspace) if workspace else nb.Attention("bf16")
    rng = np.random.default_rng(kv * 10 + drop)
    k = wl.round_to_bf16(rng.standard_normal((B, H, F * T, D)).astype(np.float32))
    v = wl.round_to_bf16(rng.standard_normal((B, H, F * T, D)).astype(np.float32))
    kd, vd = _dev(k), _dev(v)
    nb.nfd_kvcache_shift(a.h, kd, vd, B, H, F, T, D, kv, drop)
    torch.cuda.synchronize()
    keep = kv - drop
    rk, rv = sd.kvcache_shift(k, T, kv, drop), sd.kvcache_shift(v, T, kv, drop)
    # the kept frames sit at the front, bit for bit; frames past them are unspecified up to kv, untouched beyond
    np.testing.assert_array_equal(_host(kd)[:, :, : keep * T], rk[:, :, : keep * T])
    np.testing.assert_array_equal(_host(vd)[:, :, : keep * T], rv[:, :, : keep * T])
    np.testing.assert_array_equal(_host(kd)[:, :, kv * T:], k[:, :, kv * T:].astype(np.float64))
    np.testing.assert_array_equal(_host(vd)[:, :, kv * T:], v[:, :, kv * T:].astype(np.float64))
    a.close()


def test_speculative_decode_loop_with_window_and_rollback():
    B, H, D, grid, sections = 1, 2, 64, (6, 8), (16, 24, 24)
    T = grid[0] * grid[1]
    total, n_prompt, nframe, window, F = 22, 3, 3, 6, 9
    rng = np.random.default_rng(77)
    actions = np.repeat(rng.integers(0, 3, size=(total, 1)), rng.integers(1, 5, size=total), axis=0)[:total].astype(np.int32)
    # per-frame q, k, v "projections" of a stand-in model: fixed random tensors per absolute frame
    mk = lambda: wl.round_to_bf16(rng.standard_normal((total, B, H, T, D)).astype(np.float32))
    Q, K, V = mk(), mk(), mk()
    a = nb.Attention("bf16")
    kc = torch.zeros((B, H, F * T, D), dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    frames = lambda X, idx: np.ascontiguousarray(np.concatenate([X[f] for f in idx], axis=2))

    # prompt frames into the cache (rotated keys), and a host mirror kept by the oracle
    hk = np.zeros((B, H, F * T, D))
    hv = np.zeros((B, H, F * T, D))
    prompt = list(range(n_prompt))
    a.rope_append(_dev(frames(Q, prompt)), kc, vc, _dev(frames(K, prompt)), _dev(frames(V, prompt)), T, 0, grid, sections)
    torch.cuda.synchronize()
    _, rk, rv = orc.rope_kvcache_append(frames(Q, prompt), hk, hv, frames(K, prompt), frames(V, prompt), T, 0, grid, sections)
    assert np.all(np.abs(_host(kc) - rk) <= np.abs(rk) * 2.0 ** -8 + 1e-6) and np.array_equal(_host(vc), rv)
    hk, hv = _host(kc), _host(vc)  # the mirror continues from the device's bf16 values

    s = nb.nfd_spec_init(F, window, nframe, n_prompt, total)
    expect = sd.run(actions, n_prompt, nframe, window, F)
    n_steps = 0
    while True:
        st = nb.nfd_spec_next(s)
        if st is None:
            break
        ex = expect[n_steps]
        n_steps += 1
        assert st.n_drop == ex["evict"]
        if st.n_drop:
            kv_before = st.frame_pos + st.n_drop
            nb.nfd_kvcache_shift(a.h, kc, vc, B, H, F, T, D, kv_before, st.n_drop)
            hk, hv = sd.kvcache_shift(hk, T, kv_before, st.n_drop), sd.kvcache_shift(hv, T, kv_before, st.n_drop)
        gen = ex["generated"]
        assert len(gen) == st.n_frames
        qn, kn, vn = frames(Q, gen), frames(K, gen), frames(V, gen)
        qr = a.rope_append(_dev(qn), kc, vc, _dev(kn), _dev(vn), T, st.frame_pos, grid, sections, t_offset=st.t_offset)
        out = a.forward(qr, kc, vc, T, kv_frames=st.kv_frames, q_frames=st.q_frames)
        torch.cuda.synchronize()
        # oracle on the host mirror: same positions, same rounded cache contents
        rq, rk, rv = orc.rope_kvcache_append(qn, hk, hv, kn, vn, T, st.frame_pos, grid, sections, t_offset=st.t_offset)
        n_valid = st.kv_frames * T
        dk_, dv_ = _host(kc)[:, :, :n_valid], _host(vc)[:, :, :n_valid]
        assert np.all(np.abs(dk_ - rk[:, :, :n_valid]) <= np.abs(rk[:, :, :n_valid]) * 2.0 ** -8 + 1e-6)
        assert np.array_equal(dv_, rv[:, :, :n_valid])
        assert np.all(np.abs(_host(qr) - rq) <= np.abs(rq) * 2.0 ** -8 + 1e-6)
        hk[:, :, :n_valid], hv[:, :, :n_valid] = dk_, dv_  # continue from the device's bf16 values
        ref = orc.block_causal_attn(_host(qr), hk, hv, T, kv_frames=st.kv_frames, q_frames=st.q_frames)
        d = _host(out) - ref
        assert np.abs(d).max() <= 2e-2 and np.linalg.norm(d) / np.linalg.norm(ref) <= 5e-3
        assert worst_row(_host(out), ref)[0] <= BF16_ROW_REL_L2
        kept = nb.nfd_spec_accept(s, st, actions)
        assert kept == ex["kept"]
        # absolute temporal positions: cache slot 0 holds frame t_offset
        assert st.t_offset == ex["cache_frames"][0]
    assert n_steps == len(expect) and s.done == total
    a.close()
