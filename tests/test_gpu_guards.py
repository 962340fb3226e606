"""Writes stay inside the tensors they are given: every tensor a call writes (out, lse, the caches, the gradients,
the rotated queries, the 8-bit caches) sits between two guard regions filled with a sentinel byte, the call goes
through the C ABI, and the guards are compared from the host afterwards.  Shapes are ragged on purpose (rows that
do not fill a tile, a last frame at the end of the capacity, key splits, both workgroup shapes).  Values are
checked by the parity tests; here only that the written tensors hold no sentinel leftovers where a result is due."""
import numpy as np
import pytest
import torch

from paper_2506_01380_amd import binding as nb

pytestmark = pytest.mark.gpu

GUARD = 8192       # elements on either side (a multiple of 16 bytes for every dtype used)
SENTINEL = 0xA5


class Guarded:
    """A dense tensor of `shape` in the middle of a larger allocation whose margins hold the sentinel."""

    def __init__(self, shape, dtype, value=None):
        self.n = int(np.prod(shape))
        self.base = torch.empty(self.n + 2 * GUARD, dtype=dtype, device="cuda")
        self.base.view(torch.uint8).fill_(SENTINEL)
        self.t = self.base[GUARD:GUARD + self.n].view(shape)
        if value is not None:
            self.t.copy_(value)

    def intact(self):
        raw = self.base.view(torch.uint8)
        es = self.base.element_size()
        return bool((raw[:GUARD * es] == SENTINEL).all()) and bool((raw[(GUARD + self.n) * es:] == SENTINEL).all())

    def written(self):
        """No element still holds the sentinel pattern (for tensors a call must fill completely)."""
        es = self.base.element_size()
        raw = self.t.reshape(-1).view(torch.uint8).view(-1, es)
        return not bool((raw == SENTINEL).all(dim=1).any())


def _rand(shape, dtype, seed):
    g = torch.Generator(device="cuda").manual_seed(seed)
    return torch.randn(*shape, device="cuda", generator=g, dtype=torch.float32).to(dtype)


@pytest.fixture(scope="module")
def attn():
    a = nb.Attention("bf16")
    yield a
    a.close()


@pytest.fixture(scope="module")
def attn32():
    a = nb.Attention("fp32")
    yield a
    a.close()


# (B, H, T, kv_frames, q_frames, F): training forms with ragged last tiles, cached forms with key splits, both
# workgroup shapes of the matrix-core kernel, a head count that is not a multiple of 8
FWD_CASES = [(1, 2, 7, 5, 5, 5), (1, 16, 336, 3, 3, 3), (2, 3, 50, 9, 9, 10), (1, 16, 336, 33, 1, 33), (1, 16, 336, 12, 4, 13),
             (1, 8, 21, 40, 2, 41), (3, 5, 1, 70, 70, 70), (1, 1, 300, 2, 2, 2)]


@pytest.mark.parametrize("B,H,T,kvf,qf,F", FWD_CASES)
def test_forward_forms_write_only_their_outputs(attn, B, H, T, kvf, qf, F):
    D, bf = 64, torch.bfloat16
    q, k, v = _rand((B, H, qf * T, D), bf, 1), _rand((B, H, F * T, D), bf, 2), _rand((B, H, F * T, D), bf, 3)
    out = Guarded((B, H, qf * T, D), bf)
    nb.nfd_block_causal_attn_fwd(attn.h, q, k, v, out.t, B, H, F, T, D, kvf, qf)
    torch.cuda.synchronize()
    assert out.intact() and out.written() and bool(torch.isfinite(out.t.float()).all())
    # training pair: out and the log-sum-exp
    out2, lse = Guarded((B, H, qf * T, D), bf), Guarded((B, H, qf * T), torch.float32)
    nb.nfd_block_causal_attn_fwd_lse(attn.h, q, k, v, out2.t, lse.t, B, H, F, T, D, kvf, qf)
    torch.cuda.synchronize()
    assert out2.intact() and lse.intact() and out2.written() and lse.written()
    # the handle-free entry point
    out3 = Guarded((B, H, qf * T, D), bf)
    nb.nfd_block_causal_attn_fwd_noalloc(nb.NFD_BF16, q, k, v, out3.t, B, H, F, T, D, kvf, qf)
    torch.cuda.synchronize()
    assert out3.intact() and torch.equal(out3.t, out.t)
    # gradients
    dq, dk, dv = Guarded(q.shape, bf), Guarded(k.shape, bf), Guarded(k.shape, bf)
    dk.t.zero_(); dv.t.zero_()
    nb.nfd_block_causal_attn_bwd(attn.h, q, k, v, out2.t, _rand(q.shape, bf, 4), lse.t, dq.t, dk.t, dv.t, B, H, F, T, D, kvf, qf)
    torch.cuda.synchronize()
    assert dq.intact() and dk.intact() and dv.intact() and dq.written()
    assert bool((dk.t[:, :, kvf * T:] == 0).all()) and bool((dv.t[:, :, kvf * T:] == 0).all())


@pytest.mark.parametrize("B,H,T,D,kvf,qf,F", [(1, 2, 16, 64, 4, 4, 4), (2, 3, 5, 24, 6, 2, 7), (1, 1, 9, 200, 3, 3, 3)])
def test_general_path_writes_only_its_outputs(attn32, B, H, T, D, kvf, qf, F):
    f32 = torch.float32
    q, k, v = _rand((B, H, qf * T, D), f32, 5), _rand((B, H, F * T, D), f32, 6), _rand((B, H, F * T, D), f32, 7)
    out, lse = Guarded(q.shape, f32), Guarded((B, H, qf * T), f32)
    nb.nfd_block_causal_attn_fwd_lse(attn32.h, q, k, v, out.t, lse.t, B, H, F, T, D, kvf, qf)
    dq, dk, dv = Guarded(q.shape, f32), Guarded(k.shape, f32), Guarded(k.shape, f32)
    dk.t.zero_(); dv.t.zero_()
    nb.nfd_block_causal_attn_bwd(attn32.h, q, k, v, out.t, _rand(q.shape, f32, 8), lse.t, dq.t, dk.t, dv.t, B, H, F, T, D, kvf, qf)
    torch.cuda.synchronize()
    for g in (out, lse, dq, dk, dv):
        assert g.intact()
    assert out.written() and lse.written() and dq.written()


@pytest.mark.parametrize("B,H,T,F,pos,n", [(1, 16, 336, 33, 32, 1), (2, 3, 5, 7, 4, 3), (1, 16, 336, 12, 8, 4), (1, 2, 21, 41, 39, 2)])
def test_cache_writes_stay_inside_the_caches(attn, B, H, T, F, pos, n):
    D, bf = 64, torch.bfloat16
    kn, vn, q = _rand((B, H, n * T, D), bf, 11), _rand((B, H, n * T, D), bf, 12), _rand((B, H, n * T, D), bf, 13)
    # plain append of the last frames the capacity allows for this position
    kc, vc = Guarded((B, H, F * T, D), bf), Guarded((B, H, F * T, D), bf)
    kc.t.zero_(); vc.t.zero_()
    nb.nfd_kvcache_append(attn.h, kc.t, vc.t, kn, vn, B, H, F, T, D, pos, n)
    torch.cuda.synchronize()
    assert kc.intact() and vc.intact()
    assert torch.equal(kc.t[:, :, pos * T:(pos + n) * T], kn) and not bool(kc.t[:, :, :pos * T].any())
    # one-call cached step: the attention's workgroups copy the new frames on the side
    kc2, vc2 = Guarded((B, H, F * T, D), bf, _rand((B, H, F * T, D), bf, 14)), Guarded((B, H, F * T, D), bf, _rand((B, H, F * T, D), bf, 15))
    k_before = kc2.t.clone()
    out = Guarded(q.shape, bf)
    nb.nfd_kvcache_append_attn_fwd(attn.h, q, kc2.t, vc2.t, kn, vn, out.t, B, H, F, T, D, pos + n, n)
    torch.cuda.synchronize()
    assert kc2.intact() and vc2.intact() and out.intact() and out.written()
    assert torch.equal(kc2.t[:, :, pos * T:(pos + n) * T], kn) and torch.equal(vc2.t[:, :, pos * T:(pos + n) * T], vn)
    assert torch.equal(kc2.t[:, :, :pos * T], k_before[:, :, :pos * T]) and torch.equal(kc2.t[:, :, (pos + n) * T:], k_before[:, :, (pos + n) * T:])
    # rotary embedding + cache write (needs a grid with grid_h * grid_w == T)
    gh = next(x for x in (24, 7, 5, 3, 1) if T % x == 0)
    qo = Guarded(q.shape, bf)
    nb.nfd_rope_kvcache_append(attn.h, q, qo.t, kc.t, vc.t, kn, vn, B, H, F, T, D, pos, n, 3, gh, T // gh, 16, 24, 24)
    torch.cuda.synchronize()
    assert kc.intact() and vc.intact() and qo.intact() and qo.written()
    # sliding window: drop the oldest frames (all three strategies are chosen by sizes; here whatever fits)
    for drop in (1, (pos + n) // 2, pos + n - 1):
        if 0 < drop < pos + n:
            nb.nfd_kvcache_shift(attn.h, kc.t, vc.t, B, H, F, T, D, pos + n, drop)
    torch.cuda.synchronize()
    assert kc.intact() and vc.intact()


@pytest.mark.parametrize("B,H,T,F,pos,n", [(1, 16, 336, 33, 32, 1), (2, 3, 20, 7, 4, 3), (1, 2, 48, 9, 5, 4)])
def test_8bit_cache_writes_stay_inside_the_caches(attn, B, H, T, F, pos, n):
    D, bf = 64, torch.bfloat16
    nbytes = nb.nfd_fp8_cache_bytes(B, H, F, T, D)
    k8, v8 = Guarded((nbytes,), torch.uint8), Guarded((nbytes,), torch.uint8)
    k8.t.zero_(); v8.t.zero_()
    ks = torch.full((B, H), 0.05, dtype=torch.float32, device="cuda")
    vs = torch.full((B, H), 0.04, dtype=torch.float32, device="cuda")
    past_k, past_v = _rand((B, H, pos * T, D), bf, 21), _rand((B, H, pos * T, D), bf, 22)
    kn, vn, q = _rand((B, H, n * T, D), bf, 23), _rand((B, H, n * T, D), bf, 24), _rand((B, H, n * T, D), bf, 25)
    nb.nfd_kvcache_append_fp8(attn.h, k8.t, v8.t, ks, vs, past_k, past_v, B, H, F, T, D, 0, pos)
    nb.nfd_kvcache_append_fp8(attn.h, k8.t, v8.t, ks, vs, kn, vn, B, H, F, T, D, pos, n)
    out = Guarded(q.shape, bf)
    nb.nfd_block_causal_attn_fwd_fp8kv(attn.h, q, k8.t, v8.t, ks, vs, out.t, B, H, F, T, D, pos + n, n)
    torch.cuda.synchronize()
    assert k8.intact() and v8.intact() and out.intact() and out.written() and bool(torch.isfinite(out.t.float()).all())
    gh = next(x for x in (24, 6, 5, 4) if T % x == 0)
    qo = Guarded(q.shape, bf)
    nb.nfd_rope_kvcache_append_fp8(attn.h, q, qo.t, k8.t, v8.t, ks, vs, kn, vn, B, H, F, T, D, pos, n, 2, gh, T // gh, 16, 24, 24)
    for drop in (1, pos + n - 1):
        nb.nfd_kvcache_shift_fp8(attn.h, k8.t, v8.t, B, H, F, T, D, pos + n, drop)
    torch.cuda.synchronize()
    assert k8.intact() and v8.intact() and qo.intact() and qo.written()
