"""GPU parity on seeded random shapes: forward (every call form), forward with log-sum-exp and
backward against the fp64 oracle, every element.  The shapes are drawn to hit ragged query tiles,
ragged key blocks, frames that straddle tiles, head counts that do not divide by the number of
XCDs, spare cache capacity and key splits."""
import numpy as np
import pytest
from parity_bounds import BF16_LSE_ABS, BF16_ROW_REL_L2, worst_row
import torch

from oracle import nfd_oracle as orc
from paper_2506_01380_amd import binding as nb
from paper_2506_01380_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _shapes(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        T = int(rng.choice([1, 3, 8, 17, 33, 64, 65, 100, 127, 130, 200]))
        kvf = int(rng.integers(1, 9))
        if kvf * T > 1600:
            continue
        qf = int(rng.integers(1, kvf + 1))
        F = kvf + int(rng.integers(0, 3))
        out.append((int(rng.integers(1, 3)), int(rng.integers(1, 10)), T, kvf, qf, F))
    return out


@pytest.fixture(scope="module")
def attn():
    a = nb.Attention("bf16")
    yield a
    a.close()


def _dev(x):
    return torch.from_numpy(x).cuda().to(torch.bfloat16)


def _host(t):
    return t.float().cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("B,H,T,kvf,qf,F", _shapes(24, 20260613))
def test_forward_and_backward_on_random_shapes(attn, B, H, T, kvf, qf, F):
    D = 64
    seed = wl.BASE_SEED + 1000 + 7 * T + 31 * kvf + qf
    q, k, v = wl.make_qkv(B, H, D, T, kvf, qf, F, "bf16", seed=seed)
    g = wl.round_to_bf16(np.random.default_rng(seed + 1).standard_normal(q.shape).astype(np.float32))
    if F > kvf:
        k[:, :, kvf * T:] = np.nan
        v[:, :, kvf * T:] = np.nan
    qd, kd, vd, gd = _dev(q), _dev(k), _dev(v), _dev(g)
    out_plain = attn.forward(qd, kd, vd, T, kv_frames=kvf, q_frames=qf)
    out, lse = attn.forward_lse(qd, kd, vd, T, kv_frames=kvf, q_frames=qf)
    dq, dk, dv = attn.backward(qd, kd, vd, out, gd, lse, T, kv_frames=kvf, q_frames=qf)
    torch.cuda.synchronize()
    # the forward of the training pair forms its scores from the queries as given, the plain forward from queries that
    # carry the softmax scale (one more bf16 rounding): two results, both checked against the oracle below
    kz, vz = np.nan_to_num(k), np.nan_to_num(v)
    ref = orc.block_causal_attn(q, kz, vz, T, kv_frames=kvf, q_frames=qf)
    rdq, rdk, rdv, rlse = orc.block_causal_attn_bwd(q, kz, vz, g, T, kv_frames=kvf, q_frames=qf)
    Sk = kvf * T

    def close(got, want, tag):
        assert np.all(np.isfinite(got)), tag
        d = got - want
        rel = np.linalg.norm(d) / np.linalg.norm(want)
        assert rel <= 5e-3 and np.abs(d).max() <= 2e-2 * max(1.0, np.abs(want).max()), (tag, rel, np.abs(d).max())

    close(_host(out), ref, "out")
    assert worst_row(_host(out), ref)[0] <= BF16_ROW_REL_L2
    close(_host(out_plain), ref, "out (plain forward)")
    assert worst_row(_host(out_plain), ref)[0] <= BF16_ROW_REL_L2
    close(_host(dq), rdq, "dq")
    close(_host(dk)[:, :, :Sk], rdk[:, :, :Sk], "dk")
    close(_host(dv)[:, :, :Sk], rdv[:, :, :Sk], "dv")
    assert np.abs(lse.cpu().numpy() - rlse).max() <= BF16_LSE_ABS
    assert np.all(_host(dk)[:, :, Sk:] == 0) and np.all(_host(dv)[:, :, Sk:] == 0)


def _shapes_many_heads(n, seed):
    """Enough (batch, head) units that the plan takes the 64-row wavefront shape (two interleaved row blocks per
    wavefront, two tile loops; with the 8-bit cache the tiles widened once per workgroup)."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        T = int(rng.choice([1, 3, 17, 40, 64, 100, 130, 200, 336]))
        kvf = int(rng.integers(1, 12))
        if kvf * T > 1400 or kvf * T < 200:
            continue
        qf = int(rng.integers(1, kvf + 1))
        out.append((int(rng.choice([4, 8, 9])), int(rng.choice([8, 16, 9])), T, kvf, qf, kvf + int(rng.integers(0, 2))))
    return out


_FIXED_MANY_HEADS = [
    (8, 8, 1, 300, 300, 300),    # T = 1: a frame boundary after every row
    (8, 8, 3, 150, 100, 150),    # cached form, tiny frames
    (4, 16, 17, 40, 40, 41),     # many boundaries inside one workgroup, ragged last tile
    (4, 16, 336, 4, 4, 4),       # the paper's frame size: one boundary in three of four workgroups
    (8, 8, 256, 3, 3, 3),        # frames = workgroups: no boundary inside any
    # query tiles of fewer than eight 32-row blocks (the blocks of a head are dealt evenly): wavefronts with one block
    (8, 8, 40, 5, 5, 5),         # 200 rows: one tile of 7 blocks, the last block 8 rows
    (8, 8, 36, 5, 5, 5),         # 180 rows: 6 blocks
    (8, 8, 30, 6, 5, 6),         # 150 rows: 5 blocks, cached form
    (4, 16, 52, 9, 8, 9),        # 416 rows: two tiles, 7 + 6 blocks
    (4, 16, 336, 6, 4, 6),       # four speculative frames of the paper's size: six tiles of 7 blocks
]


@pytest.mark.parametrize("B,H,T,kvf,qf,F", _shapes_many_heads(14, 20260614) + _FIXED_MANY_HEADS)
def test_forward_many_heads_both_caches(attn, B, H, T, kvf, qf, F):
    from oracle import fp8_cache as f8
    D = 64
    plan = nb.nfd_attn_plan(nb.NFD_BF16, B, H, F, T, D, kvf, qf)
    assert plan["block_m"] == 256, plan
    seed = wl.BASE_SEED + 2000 + 7 * T + 31 * kvf + qf
    q, k, v = wl.make_qkv(B, H, D, T, kvf, qf, F, "bf16", seed=seed)
    if F > kvf:
        k[:, :, kvf * T:] = np.nan
        v[:, :, kvf * T:] = np.nan
    qd = _dev(q)
    out = attn.forward(qd, _dev(k), _dev(v), T, kv_frames=kvf, q_frames=qf)
    # the same keys and values through the 8-bit cache
    Sk = kvf * T
    n8 = nb.nfd_fp8_cache_bytes(B, H, F, T, D)
    k8 = torch.full((n8,), 0x7F, dtype=torch.uint8, device="cuda")
    v8 = torch.full((n8,), 0x7F, dtype=torch.uint8, device="cuda")
    rng = np.random.default_rng(seed)
    ks, vs = (rng.uniform(0.01, 0.03, size=(B, H)).astype(np.float32) for _ in range(2))
    ksd, vsd = torch.from_numpy(ks).cuda(), torch.from_numpy(vs).cuda()
    nb.nfd_kvcache_append_fp8(attn.h, k8, v8, ksd, vsd, _dev(k[:, :, :Sk]), _dev(v[:, :, :Sk]), B, H, F, T, D, 0, kvf)
    out8 = torch.empty_like(qd)
    nb.nfd_block_causal_attn_fwd_fp8kv(attn.h, qd, k8, v8, ksd, vsd, out8, B, H, F, T, D, kvf, qf)
    torch.cuda.synchronize()

    def close(got, want, tag):
        assert np.all(np.isfinite(got)), tag
        d = got - want
        rel = np.linalg.norm(d) / np.linalg.norm(want)
        assert rel <= 5e-3 and np.abs(d).max() <= 2e-2, (tag, rel, np.abs(d).max())

    kz, vz = np.nan_to_num(k), np.nan_to_num(v)
    ref16 = orc.block_causal_attn(q, kz, vz, T, kv_frames=kvf, q_frames=qf)
    close(_host(out), ref16, "bf16 cache")
    assert worst_row(_host(out), ref16)[0] <= BF16_ROW_REL_L2
    kq = f8.e4m3_decode(f8.quantize(kz[:, :, :Sk], ks[:, :, None, None])) * ks[:, :, None, None].astype(np.float64)
    vq = f8.e4m3_decode(f8.quantize(vz[:, :, :Sk], vs[:, :, None, None])) * vs[:, :, None, None].astype(np.float64)
    ref8 = orc.block_causal_attn(q, kq, vq, T, kv_frames=kvf, q_frames=qf)
    close(_host(out8), ref8, "8-bit cache")
    assert worst_row(_host(out8), ref8)[0] <= BF16_ROW_REL_L2
