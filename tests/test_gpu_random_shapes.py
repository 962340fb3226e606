"""GPU parity on seeded random shapes: forward (every call form), forward with log-sum-exp and
backward against the fp64 oracle, every element.  The shapes are drawn to hit ragged query tiles,
ragged key blocks, frames that straddle tiles, head counts that do not divide by the number of
XCDs, spare cache capacity and key splits."""
import numpy as np
import pytest
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
    assert torch.equal(out, out_plain)  # writing the log-sum-exp does not change the output
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
    close(_host(dq), rdq, "dq")
    close(_host(dk)[:, :, :Sk], rdk[:, :, :Sk], "dk")
    close(_host(dv)[:, :, :Sk], rdv[:, :, :Sk], "dv")
    assert np.abs(lse.cpu().numpy() - rlse).max() <= 2e-4
    assert np.all(_host(dk)[:, :, Sk:] == 0) and np.all(_host(dv)[:, :, Sk:] == 0)
