"""CPU-side checks of the C-ABI library: it loads, exports what the header declares,
validates arguments with the documented codes, and plans a tile schedule that skips
future frames.  No compute call is made (there is no GPU here)."""
import os
import re

import pytest

from oracle import nfd_oracle as orc
from paper_2506_01380_amd import binding as nb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "nfd_attn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(nfd_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"nfd_attn_create", "nfd_block_causal_attn_fwd", "nfd_kvcache_append", "nfd_attn_destroy"} <= set(names)
    L = nb.lib()
    for n in names:
        assert hasattr(L, n), n
    assert set(names) == set(nb.EXPORTS)


@pytest.mark.parametrize("args,code", [
    (dict(B=1, H=2, F=4, T=16, D=64, kv_frames=4, q_frames=4), nb.NFD_OK),
    (dict(B=0, H=2, F=4, T=16, D=64, kv_frames=4, q_frames=4), nb.NFD_ERR_SHAPE),
    (dict(B=1, H=2, F=4, T=0, D=64, kv_frames=4, q_frames=4), nb.NFD_ERR_SHAPE),
    (dict(B=1, H=2, F=4, T=16, D=64, kv_frames=4, q_frames=0), nb.NFD_ERR_SHAPE),
    (dict(B=1, H=2, F=4, T=16, D=64, kv_frames=3, q_frames=4), nb.NFD_ERR_SHAPE),
    (dict(B=1, H=2, F=4, T=16, D=64, kv_frames=5, q_frames=4), nb.NFD_ERR_CAPACITY),
    (dict(B=1, H=2, F=4, T=16, D=512, kv_frames=4, q_frames=4), nb.NFD_ERR_UNSUPPORTED),
])
def test_check_args_codes(args, code):
    assert nb.nfd_attn_check_args(nb.NFD_BF16, **args) == code


@pytest.mark.parametrize("args,code", [
    (dict(B=1, H=16, F=40, T=336, D=64, frame_pos=32, n_frames=1, grid_h=24, grid_w=14, n_t=16, n_h=24, n_w=24), nb.NFD_OK),
    (dict(B=1, H=16, F=40, T=336, D=64, frame_pos=32, n_frames=0, grid_h=24, grid_w=14, n_t=64, n_h=0, n_w=0), nb.NFD_OK),
    (dict(B=1, H=16, F=40, T=336, D=64, frame_pos=32, n_frames=1, grid_h=24, grid_w=13, n_t=16, n_h=24, n_w=24), nb.NFD_ERR_SHAPE),
    (dict(B=1, H=16, F=40, T=336, D=64, frame_pos=32, n_frames=1, grid_h=24, grid_w=14, n_t=15, n_h=25, n_w=24), nb.NFD_ERR_SHAPE),
    (dict(B=1, H=16, F=40, T=336, D=64, frame_pos=32, n_frames=1, grid_h=24, grid_w=14, n_t=16, n_h=24, n_w=22), nb.NFD_ERR_SHAPE),
    (dict(B=1, H=16, F=40, T=336, D=64, frame_pos=-1, n_frames=1, grid_h=24, grid_w=14, n_t=16, n_h=24, n_w=24), nb.NFD_ERR_SHAPE),
    (dict(B=1, H=16, F=40, T=336, D=64, frame_pos=39, n_frames=2, grid_h=24, grid_w=14, n_t=16, n_h=24, n_w=24), nb.NFD_ERR_CAPACITY),
    (dict(B=1, H=1, F=2, T=4, D=512, frame_pos=0, n_frames=1, grid_h=2, grid_w=2, n_t=512, n_h=0, n_w=0), nb.NFD_ERR_UNSUPPORTED),
])
def test_rope_check_args_codes(args, code):
    assert nb.nfd_rope_check_args(nb.NFD_BF16, **args) == code


def test_bad_dtype_is_unsupported():
    assert nb.nfd_attn_check_args(7, 1, 1, 1, 1, 64, 1, 1) == nb.NFD_ERR_UNSUPPORTED


@pytest.mark.parametrize("T,kvf,qf", [(16, 4, 4), (3, 5, 2), (336, 33, 1), (7, 9, 9)])
def test_visible_pairs_matches_enumeration(T, kvf, qf):
    assert nb.nfd_attn_visible_pairs(T, kvf, qf) == orc.visible_pairs(T, kvf, qf)


def test_plan_training_form_skips_future_tiles():
    # Sec. 3.1: about half of the dense attention cost
    pl = nb.nfd_attn_plan(nb.NFD_BF16, 4, 16, 16, 336, 64, 16, 16)
    assert pl["kernel"] == 1 and pl["n_splits"] == 1
    frac = pl["key_tiles_visited"] / pl["key_tiles_dense"]
    assert 0.5 < frac < 0.60
    pl = nb.nfd_attn_plan(nb.NFD_BF16, 2, 16, 64, 576, 64, 64, 64)
    assert 0.5 < pl["key_tiles_visited"] / pl["key_tiles_dense"] < 0.53


def test_plan_cached_forms_split_keys_and_fit_workspace():
    pl = nb.nfd_attn_plan(nb.NFD_BF16, 1, 16, 40, 336, 64, 33, 1)
    assert pl["n_splits"] > 1 and pl["workspace_bytes"] <= 128 << 20
    assert pl["workspace_bytes"] == 16 * 336 * pl["n_splits"] * (64 * 2 + 8)
    small = nb.nfd_attn_plan(nb.NFD_BF16, 1, 16, 40, 336, 64, 33, 1, 256, 3 * 16 * 336 * (64 * 2 + 8))
    assert small["n_splits"] == 3
    none = nb.nfd_attn_plan(nb.NFD_BF16, 1, 16, 40, 336, 64, 33, 1, 256, 1000)
    assert none["n_splits"] == 1 and none["workspace_bytes"] == 0


def test_plan_general_kernel_for_fp32_and_other_widths():
    assert nb.nfd_attn_plan(nb.NFD_FP32, 1, 2, 4, 16, 64, 4, 4)["kernel"] == 0
    assert nb.nfd_attn_plan(nb.NFD_BF16, 1, 2, 4, 16, 128, 4, 4)["kernel"] == 0


def test_create_without_gpu_reports_an_error_code():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(nb.NfdError) as e:
        nb.nfd_attn_create(nb.NFD_BF16, 0)
    assert e.value.code in (nb.NFD_ERR_HIP, nb.NFD_ERR_ALLOC)


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_plan_refuses_a_launch_beyond_the_grid_limit():
    # 2^24 heads x 2^22 query tiles would overflow the workgroup count
    rc = nb.lib().nfd_attn_plan(nb.NFD_BF16, 1 << 12, 1 << 12, 1 << 14, 1 << 16, 64, 1 << 14, 1 << 14, 0, 0,
                                __import__("ctypes").byref(nb.Plan()))
    assert rc == nb.NFD_ERR_UNSUPPORTED


@pytest.mark.parametrize("BH,nq,ns", [(16, 2, 16), (16, 6, 5), (128, 3, 4), (5, 3, 7), (9, 4, 1), (64, 21, 1), (3, 1, 2),
                                      (1, 1, 1), (17, 2, 3), (12, 3, 16), (24, 21, 1), (8, 1, 1), (256, 21, 1), (136, 2, 1),
                                      (20, 3, 1), (72, 5, 2)])
@pytest.mark.parametrize("group", [0, 1])
def test_every_work_item_is_dealt_exactly_once(BH, nq, ns, group):
    """The workgroup -> (head, query tile, split) map of the forward launch is a bijection onto all items;
    with a head count that is a multiple of 8 a head stays on one XCD (block id mod 8)."""
    n = BH * nq * ns
    seen = {}
    for blk in range(n):
        item = nb.nfd_attn_work_item(BH, nq, ns, group, blk)
        assert item is not None and 0 <= item[0] < BH and 0 <= item[1] < nq and 0 <= item[2] < ns
        assert item not in seen
        seen[item] = blk
    assert len(seen) == n and nb.nfd_attn_work_item(BH, nq, ns, group, n) is None
    if BH % 8 == 0:
        assert all(blk % 8 == bh % 8 for (bh, _, _), blk in seen.items())
    if not group:  # heaviest (last) query tiles first
        order = [nb.nfd_attn_work_item(BH, nq, ns, 0, b)[1] for b in range(n)]
        first_of = {q: order.index(q) for q in range(nq)}
        assert all(first_of[q + 1] <= first_of[q] for q in range(nq - 1))
        # heads go in groups of 8 per id stream (one stream per XCD when heads are pinned, else one in all): every
        # item of a group is dealt before the next group starts
        stream = (lambda bh: bh // 8) if BH % 8 == 0 else (lambda bh: bh)
        for x in range(8 if BH % 8 == 0 else 1):
            groups = [stream(nb.nfd_attn_work_item(BH, nq, ns, 0, b)[0]) // 8 for b in range(n) if BH % 8 != 0 or b % 8 == x]
            assert groups == sorted(groups)


def test_fp8_cache_bytes_rounds_the_key_count_to_whole_tiles():
    assert nb.nfd_fp8_cache_bytes(1, 16, 40, 336, 64) == 16 * 13440 * 64          # 40 * 336 = 210 tiles exactly
    assert nb.nfd_fp8_cache_bytes(2, 3, 5, 7, 64) == 2 * 3 * 64 * 64              # 35 keys -> one tile
    assert nb.nfd_fp8_cache_bytes(1, 1, 1, 65, 64) == 128 * 64
    import ctypes
    n = ctypes.c_size_t(0)
    assert nb.lib().nfd_fp8_cache_bytes(1, 1, 1, 16, 128, ctypes.byref(n)) == nb.NFD_ERR_UNSUPPORTED
    assert nb.lib().nfd_fp8_cache_bytes(0, 1, 1, 16, 64, ctypes.byref(n)) == nb.NFD_ERR_SHAPE
    assert nb.lib().nfd_fp8_cache_bytes(1, 1, 1, 16, 64, None) == nb.NFD_ERR_NULL


@pytest.mark.parametrize("T,qf,B,H", [(336, 4, 1, 16), (336, 2, 1, 16), (336, 1, 1, 16), (336, 16, 4, 16), (576, 1, 8, 16), (7, 5, 1, 2),
                                      (1, 300, 8, 8), (50, 9, 2, 3), (100, 3, 4, 16), (33, 5, 8, 8), (130, 7, 9, 9)])
def test_query_tiles_cover_every_row_once_and_evenly(T, qf, B, H):
    """The rows of a head are cut into the plan's query tiles without gap or overlap; the 32-row blocks are dealt
    evenly, so no tile is larger than block_m and tile sizes differ by at most one block."""
    pl = nb.nfd_attn_plan(nb.NFD_BF16, B, H, qf + 3, T, 64, qf + 3, qf)
    rows, nq = qf * T, pl["n_q_tiles"]
    nxt, sizes = 0, []
    for qt in range(nq):
        r0, n = nb.nfd_attn_q_tile_rows(rows, nq, qt)
        assert r0 == nxt and 1 <= n <= pl["block_m"] and r0 % 32 == 0
        nxt += n
        sizes.append(n)
    assert nxt == rows
    assert max(sizes[:-1] + [sizes[-1]]) - min(sizes[:-1] or sizes) <= 32   # the last tile may also lose a partial block
    assert nb.nfd_attn_q_tile_rows(rows, nq, nq) is None and nb.nfd_attn_q_tile_rows(0, nq, 0) is None
    # the plan's count of visited key tiles follows from these tiles: the last row of a tile sets its chain
    visited = 0
    P = 3
    for qt in range(nq):
        r0, n = nb.nfd_attn_q_tile_rows(rows, nq, qt)
        visited += -(-((P + (r0 + n - 1) // T + 1) * T) // 64)
    assert pl["key_tiles_visited"] == visited * B * H
