"""GPU: the decode step (rotary embedding + cache write, attention with key splits, combine) is
capturable into a HIP graph - the calls allocate nothing, never synchronise and use no memset -
and every replay gives the eager result bit for bit, with eager work and synchronisations between
the replays."""
import numpy as np
import pytest
import torch

from paper_2506_01380_amd import binding as nb
from paper_2506_01380_amd import workloads as wl

pytestmark = pytest.mark.gpu


def test_decode_step_replays_bit_identically_from_a_graph():
    B, H, D, grid, sections = 1, 4, 64, (24, 14), (16, 24, 24)
    T, F, past = 336, 8, 6
    a = nb.Attention("bf16")
    gen = torch.Generator(device="cuda").manual_seed(wl.BASE_SEED + 900)
    mk = lambda *s: torch.randn(*s, device="cuda", generator=gen, dtype=torch.float32).to(torch.bfloat16)
    kc, vc = mk(B, H, F * T, D), mk(B, H, F * T, D)
    q, kn, vn = mk(B, H, T, D), mk(B, H, T, D), mk(B, H, T, D)   # static input buffers of the graph
    qr, out = torch.empty_like(q), torch.empty_like(q)
    plan = nb.nfd_attn_plan(nb.NFD_BF16, B, H, F, T, D, past + 1, 1)
    assert plan["n_splits"] > 1  # the captured step includes the combine launch

    def step():
        nb.nfd_rope_kvcache_append(a.h, q, qr, kc, vc, kn, vn, B, H, F, T, D, past, 1, 0, grid[0], grid[1], *sections)
        nb.nfd_block_causal_attn_fwd(a.h, qr, kc, vc, out, B, H, F, T, D, past + 1, 1)

    step()  # eager warm-up outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        with torch.cuda.graph(g, stream=s):
            step()
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()

    for rep in range(4):
        # new inputs in the static buffers, eager reference first
        q.copy_(mk(B, H, T, D)); kn.copy_(mk(B, H, T, D)); vn.copy_(mk(B, H, T, D))
        step()
        torch.cuda.synchronize()
        ref_out, ref_q, ref_k = out.clone(), qr.clone(), kc.clone()
        out.zero_(); qr.zero_()
        kc[:, :, past * T:(past + 1) * T].zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref_out) and torch.equal(qr, ref_q) and torch.equal(kc, ref_k), rep
    a.close()
