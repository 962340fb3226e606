"""GPU parity of the attention backward (dq, dk, dv) and of the forward's log-sum-exp output
against the fp64 oracle, through the C ABI.  Tolerances for bf16 gradients: relative L2 <= 1e-2
per tensor (the forward's bound; P and dS are rounded to bf16 once each before their second
product, the results once more) and max-abs <= 2e-2 of the tensor's largest reference magnitude;
log-sum-exp within the bound derived in parity_bounds.py."""
import numpy as np
import pytest
from parity_bounds import BF16_LSE_ABS
import torch

from oracle import nfd_oracle as orc
from paper_2506_01380_amd import binding as nb
from paper_2506_01380_amd import workloads as wl

pytestmark = pytest.mark.gpu

REL_L2, MAX_REL = 1e-2, 2e-2


@pytest.fixture(scope="module")
def attn():
    a = nb.Attention("bf16")
    yield a
    a.close()


def _dev(x):
    return torch.from_numpy(x).cuda().to(torch.bfloat16)


def _host(t):
    return t.float().cpu().numpy().astype(np.float64)


def _check(got, ref, tag):
    assert np.all(np.isfinite(got)), tag
    d = got - ref
    rel = float(np.linalg.norm(d) / np.linalg.norm(ref))
    mx = float(np.abs(d).max() / np.abs(ref).max())
    print("%s: rel_l2=%.3e max_abs/max_ref=%.3e" % (tag, rel, mx), flush=True)
    assert rel <= REL_L2 and mx <= MAX_REL, (tag, rel, mx)


def _run(attn, B, H, T, kvf, qf, F, seed, scale=0.0, q_gain=1.0):
    D = 64
    q, k, v = wl.make_qkv(B, H, D, T, kvf, qf, F, "bf16", seed=seed)
    if q_gain != 1.0:
        q = wl.round_to_bf16(q * q_gain)
    g = wl.round_to_bf16(np.random.default_rng(seed + 1).standard_normal(q.shape).astype(np.float32))
    if F > kvf:  # rows past kv_frames must never be read
        k[:, :, kvf * T:] = np.nan
        v[:, :, kvf * T:] = np.nan
    qd, kd, vd, gd = _dev(q), _dev(k), _dev(v), _dev(g)
    out, lse = attn.forward_lse(qd, kd, vd, T, kv_frames=kvf, q_frames=qf, scale=scale)
    dq, dk, dv = attn.backward(qd, kd, vd, out, gd, lse, T, kv_frames=kvf, q_frames=qf, scale=scale)
    torch.cuda.synchronize()
    kz, vz = np.nan_to_num(k), np.nan_to_num(v)
    rdq, rdk, rdv, rlse = orc.block_causal_attn_bwd(q, kz, vz, g, T, kv_frames=kvf, q_frames=qf,
                                                    scale=None if scale <= 0 else scale)
    return (_host(dq), _host(dk), _host(dv), lse.cpu().numpy().astype(np.float64)), (rdq, rdk, rdv, rlse), _host(out)


CASES = [
    # B, H, T,  kvf, qf, F
    (1, 2, 16, 4, 4, 4),       # one partial tile
    (1, 3, 48, 7, 7, 7),       # 336 rows: ragged second query tile and key block; BH not a multiple of 8
    (2, 5, 40, 9, 9, 9),       # frames not aligned to tiles; 10 heads over 8 XCDs
    (1, 2, 336, 3, 3, 3),      # the paper's frame size, 1008 rows: four key blocks
    (1, 2, 100, 6, 2, 8),      # cached form (queries = last 2 frames), spare capacity
    (1, 1, 1, 300, 300, 300),  # T = 1: causal attention, mask on every diagonal tile
    (1, 1, 7, 50, 50, 50),     # tiny odd frames
    (1, 2, 576, 2, 2, 2),      # long-context frame size
]


@pytest.mark.parametrize("B,H,T,kvf,qf,F", CASES)
def test_backward_every_element(attn, B, H, T, kvf, qf, F):
    got, ref, _ = _run(attn, B, H, T, kvf, qf, F, wl.BASE_SEED + 800 + T + kvf)
    tag = "bwd B%d H%d T%d kv%d q%d" % (B, H, T, kvf, qf)
    Sk = kvf * T
    _check(got[0], ref[0], tag + " dq")
    _check(got[1][:, :, :Sk], ref[1][:, :, :Sk], tag + " dk")
    _check(got[2][:, :, :Sk], ref[2][:, :, :Sk], tag + " dv")
    assert np.all(got[1][:, :, Sk:] == 0) and np.all(got[2][:, :, Sk:] == 0)  # capacity rows untouched
    assert np.abs(got[3] - ref[3]).max() <= BF16_LSE_ABS, np.abs(got[3] - ref[3]).max()


def test_backward_full_size_training_config(attn):
    """c2 at its full size (B4 H16, 16 frames x 336 tokens), the launch configuration bench.py times;
    B is cut to one batch element for the oracle's sake (heads are independent), every element checked."""
    c = wl.CONFIGS["c2_train"]
    got, ref, _ = _run(attn, 1, c["H"], c["T"], c["kv_frames"], c["q_frames"], c["F"], c["seed"] + 31)
    _check(got[0], ref[0], "c2 dq")
    _check(got[1], ref[1], "c2 dk")
    _check(got[2], ref[2], "c2 dv")
    assert np.abs(got[3] - ref[3]).max() <= BF16_LSE_ABS


def test_forward_lse_on_split_and_general_paths(attn):
    """The log-sum-exp also comes out of the key-split launches (combine kernel) and of the general
    (fp32) kernel."""
    B, H, T, D, kvf, qf = 1, 2, 72, 64, 12, 2
    q, k, v = wl.make_qkv(B, H, D, T, kvf, qf, kvf, "bf16", seed=wl.BASE_SEED + 850)
    plan = nb.nfd_attn_plan(nb.NFD_BF16, B, H, kvf, T, D, kvf, qf)
    assert plan["n_splits"] > 1
    out, lse = attn.forward_lse(_dev(q), _dev(k), _dev(v), T, kv_frames=kvf, q_frames=qf)
    torch.cuda.synchronize()
    _, _, _, rlse = orc.block_causal_attn_bwd(q, k, v, np.zeros_like(q), T, kv_frames=kvf, q_frames=qf)
    assert np.abs(lse.cpu().numpy() - rlse).max() <= BF16_LSE_ABS
    a32 = nb.Attention("fp32")
    q32, k32, v32 = wl.make_qkv(1, 2, 32, 16, 4, 4, 4, "fp32", seed=wl.BASE_SEED + 851)
    o32, l32 = a32.forward_lse(torch.from_numpy(q32).cuda(), torch.from_numpy(k32).cuda(), torch.from_numpy(v32).cuda(), 16)
    torch.cuda.synchronize()
    _, _, _, r32 = orc.block_causal_attn_bwd(q32, k32, v32, np.zeros_like(q32), 16)
    assert np.abs(l32.cpu().numpy() - r32).max() <= 1e-5
    a32.close()


def test_backward_peaked_scores_and_custom_scale(attn):
    got, ref, _ = _run(attn, 1, 2, 64, 5, 5, 5, wl.BASE_SEED + 860, scale=0.2, q_gain=4.0)
    _check(got[0], ref[0], "peaked dq")
    _check(got[1], ref[1], "peaked dk")
    _check(got[2], ref[2], "peaked dv")


def test_backward_future_rows_do_not_reach_earlier_keys_and_is_reproducible(attn):
    """dout = 0 on the rows of frames < f: keys of frames < f still get gradient only through rows
    >= f ... and zeroing dout from frame f on leaves keys of frames >= f with exactly zero gradient."""
    B, H, T, D, Fr, f = 1, 2, 80, 64, 6, 4
    q, k, v = wl.make_qkv(B, H, D, T, Fr, Fr, Fr, "bf16", seed=wl.BASE_SEED + 870)
    g = wl.round_to_bf16(np.random.default_rng(5).standard_normal(q.shape).astype(np.float32))
    g[:, :, f * T:] = 0.0
    qd, kd, vd, gd = _dev(q), _dev(k), _dev(v), _dev(g)
    out, lse = attn.forward_lse(qd, kd, vd, T)
    dq, dk, dv = attn.backward(qd, kd, vd, out, gd, lse, T)
    dq2, dk2, dv2 = attn.backward(qd, kd, vd, out, gd, lse, T)
    torch.cuda.synchronize()
    assert torch.equal(dq, dq2) and torch.equal(dk, dk2) and torch.equal(dv, dv2)
    assert float(dk[:, :, f * T:].abs().max()) == 0.0 and float(dv[:, :, f * T:].abs().max()) == 0.0
    assert float(dq[:, :, f * T:].abs().max()) == 0.0
    assert float(dk[:, :, :f * T].abs().max()) > 0.0


def test_backward_error_codes(attn):
    B, H, T, D = 1, 1, 16, 64
    q, k, v = wl.make_qkv(B, H, D, T, 2, 2, 2, "bf16", seed=1)
    qd, kd, vd = _dev(q), _dev(k), _dev(v)
    out, lse = attn.forward_lse(qd, kd, vd, T)
    with pytest.raises(nb.NfdError) as e:
        nb.nfd_block_causal_attn_bwd(attn.h, qd, kd, vd, out, None, lse, qd, kd, vd, B, H, 2, T, D, 2, 2)
    assert e.value.code == nb.NFD_ERR_NULL
    with pytest.raises(nb.NfdError) as e:
        nb.nfd_block_causal_attn_bwd(attn.h, qd, kd, vd, out, out, lse, qd, kd, vd, B, H, 2, T, D, 3, 2)
    assert e.value.code == nb.NFD_ERR_CAPACITY
    with pytest.raises(nb.NfdError) as e:
        nb.nfd_block_causal_attn_bwd(attn.h, qd, kd, vd, out, out, lse, qd, kd, vd, B, H, 2, T, 512, 2, 2)
    assert e.value.code == nb.NFD_ERR_UNSUPPORTED  # head width beyond the general path's 256


GENERAL_CASES = [
    # dtype, B, H, T, D, kvf, qf, F
    ("fp32", 1, 2, 16, 64, 4, 4, 4),
    ("fp32", 2, 3, 40, 32, 5, 5, 5),     # rows and keys not multiples of 64
    ("fp32", 1, 2, 100, 64, 6, 2, 8),    # cached form with spare capacity
    ("fp32", 1, 1, 1, 48, 130, 130, 130),  # T = 1, D not a multiple of 64
    ("fp32", 1, 1, 336, 128, 2, 2, 2),   # the paper's frame size, two feature chunks per lane
    ("bf16", 1, 2, 24, 32, 6, 6, 6),     # bf16 storage at a head width the matrix-core path is not built for
    ("bf16", 1, 1, 50, 160, 3, 2, 3),
]


@pytest.mark.parametrize("dtype,B,H,T,D,kvf,qf,F", GENERAL_CASES)
def test_backward_general_path(dtype, B, H, T, D, kvf, qf, F):
    """fp32 storage, and head widths other than 64: the general kernels.  fp32 gradients within 1e-4
    max-abs of the fp64 oracle (fp32 sums of at most a few thousand terms of magnitude <= 1 each
    carry about 1e-6); bf16 storage to the bf16 bound of the other tests."""
    seed = wl.BASE_SEED + 900 + T + D
    q, k, v = wl.make_qkv(B, H, D, T, kvf, qf, F, dtype, seed=seed)
    g = np.random.default_rng(seed + 1).standard_normal(q.shape).astype(np.float32)
    tdt = torch.float32 if dtype == "fp32" else torch.bfloat16
    if dtype == "bf16":
        g = wl.round_to_bf16(g)
    if F > kvf:
        k[:, :, kvf * T:] = np.nan
        v[:, :, kvf * T:] = np.nan
    dev = lambda x: torch.from_numpy(x).cuda().to(tdt)
    a = nb.Attention(dtype)
    try:
        qd, kd, vd, gd = dev(q), dev(k), dev(v), dev(g)
        out, lse = a.forward_lse(qd, kd, vd, T, kv_frames=kvf, q_frames=qf)
        dq, dk, dv = a.backward(qd, kd, vd, out, gd, lse, T, kv_frames=kvf, q_frames=qf)
        dq2, dk2, dv2 = a.backward(qd, kd, vd, out, gd, lse, T, kv_frames=kvf, q_frames=qf)
        torch.cuda.synchronize()
    finally:
        a.close()
    assert torch.equal(dq, dq2) and torch.equal(dk, dk2) and torch.equal(dv, dv2)
    rdq, rdk, rdv, rlse = orc.block_causal_attn_bwd(q, np.nan_to_num(k), np.nan_to_num(v), g, T, kv_frames=kvf,
                                                    q_frames=qf)
    Sk = kvf * T
    tag = "general bwd %s T%d D%d" % (dtype, T, D)
    for name, got, ref in (("dq", dq, rdq), ("dk", dk[:, :, :Sk], rdk[:, :, :Sk]), ("dv", dv[:, :, :Sk], rdv[:, :, :Sk])):
        got = _host(got)
        if dtype == "fp32":
            err = float(np.abs(got - ref).max())
            print("%s %s: max_abs=%.3e" % (tag, name, err), flush=True)
            assert np.all(np.isfinite(got)) and err <= 1e-4, (tag, name, err)
        else:
            _check(got, ref, tag + " " + name)
    assert float(dk[:, :, Sk:].abs().max() if F > kvf else 0.0) == 0.0
    assert np.abs(lse.cpu().numpy() - rlse).max() <= (1e-5 if dtype == "fp32" else 2e-4)
