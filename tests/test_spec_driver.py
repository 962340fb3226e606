"""Speculative-sampling bookkeeping of the library (host only) against the plain statement of the
loop in oracle/spec_driver.py (Sec. 4.2; Appendix A), and pins of that statement by what the
paper's description fixes: constant actions keep every chunk whole, ever-changing actions keep
one frame per call, kept frames are exactly the leading run of the current action, every frame
is produced once, the context never exceeds the window.  The window eviction as an array operation
(kvcache_shift) is pinned by a cache whose every element encodes its own (frame, token, feature)."""
import numpy as np
import pytest

from oracle import spec_driver as sd
from paper_2506_01380_amd import binding as nb


def _drive(actions, n_prompt, nframe, window, capacity):
    total = actions.shape[0]
    s = nb.nfd_spec_init(capacity, window, nframe, n_prompt, total)
    cache = list(range(n_prompt))
    out = []
    while True:
        st = nb.nfd_spec_next(s)
        if st is None:
            break
        cache = cache[st.n_drop:]
        assert st.frame_pos == len(cache) and st.kv_frames == len(cache) + st.n_frames and st.q_frames == st.n_frames
        assert st.t_offset == (cache[0] if cache else s.done)
        gen = list(range(s.done, s.done + st.n_frames))
        kept = nb.nfd_spec_accept(s, st, actions)
        out.append(dict(evict=st.n_drop, cache_frames=list(cache), generated=gen, kept=kept))
        cache += gen[:kept]
        assert s.cached == len(cache) and s.done == gen[0] + kept
    return out


# ---- pins of the plain statement ------------------------------------------------------------------
def test_constant_actions_keep_every_chunk_whole():
    a = np.zeros((30, 2), dtype=np.int32)
    steps = sd.run(a, n_prompt=4, nframe=4, window=32, capacity=40)
    assert [s["kept"] for s in steps] == [4] * 6 + [2]          # ceil(26 / 4) calls, the last one short
    assert sum(s["kept"] for s in steps) == 26


def test_ever_changing_actions_keep_one_frame_per_call():
    a = np.arange(20, dtype=np.int32)[:, None]
    steps = sd.run(a, n_prompt=2, nframe=3, window=32, capacity=40)
    assert [s["kept"] for s in steps] == [1] * 18
    assert [s["generated"][0] for s in steps] == list(range(2, 20))


def test_kept_frames_are_the_leading_run_of_the_current_action():
    #           prompt | chunk of 4 generated under action 5: frames 2,3 match, frame 4 has action 7
    a = np.array([9, 9, 5, 5, 7, 7, 7, 7, 7, 1], dtype=np.int32)[:, None]
    steps = sd.run(a, n_prompt=2, nframe=4, window=32, capacity=40)
    assert steps[0]["generated"] == [2, 3, 4, 5] and steps[0]["kept"] == 2
    assert steps[1]["generated"] == [4, 5, 6, 7] and steps[1]["kept"] == 4      # resumes after the last verified frame
    assert steps[2]["generated"] == [8, 9] and steps[2]["kept"] == 1
    assert steps[3]["generated"] == [9] and steps[3]["kept"] == 1
    kept = [f for s in steps for f in s["generated"][:s["kept"]]]
    assert kept == list(range(2, 10))                                          # every frame produced exactly once


def test_context_never_exceeds_the_window_and_is_contiguous():
    rng = np.random.default_rng(3)
    a = rng.integers(0, 2, size=(80, 1)).astype(np.int32)
    for s in sd.run(a, n_prompt=3, nframe=4, window=8, capacity=12):
        c = s["cache_frames"]
        assert len(c) <= 8 and c == list(range(c[0], c[0] + len(c))) and c[-1] + 1 == s["generated"][0]


def test_valid_prefix_hand_worked():
    col = lambda *a: np.array(a, dtype=np.int32)[:, None]
    assert sd.valid_prefix(col(3)) == 1                       # a chunk of one frame is always kept
    assert sd.valid_prefix(col(3, 3, 3, 3)) == 4
    assert sd.valid_prefix(col(3, 4, 3, 3)) == 1              # a later return to the action does not rescue frames
    assert sd.valid_prefix(col(3, 3, 4, 3)) == 2
    # multi-component actions differ if any component differs
    assert sd.valid_prefix(np.array([[1, 2], [1, 2], [1, 3], [1, 2]], dtype=np.int32)) == 2
    assert sd.valid_prefix(np.array([[1, 2], [0, 2]], dtype=np.int32)) == 1


# ---- the window eviction as an array operation (Sec. 5 Limitations: fixed context window) ----------
def _labelled_cache(B, H, F, T, D):
    """cache[b, h, f*T + t, d] = a number from which (b, h, f, t, d) can be read back."""
    b, h, f, t, d = np.meshgrid(np.arange(B), np.arange(H), np.arange(F), np.arange(T), np.arange(D), indexing="ij")
    lab = ((((b * 7 + h) * 100 + f) * 100 + t) * 100 + d).astype(np.float64)
    return lab.reshape(B, H, F * T, D)


@pytest.mark.parametrize("B,H,F,T,D,kv,drop", [
    (1, 1, 5, 3, 2, 5, 2),    # full cache
    (2, 3, 9, 5, 7, 6, 1),    # odd sizes, spare capacity behind the cached frames
    (1, 2, 8, 1, 3, 7, 5),    # one token per frame; more dropped than kept
    (2, 1, 6, 4, 1, 4, 0),    # nothing dropped
    (1, 2, 6, 4, 3, 4, 4),    # everything dropped
    (1, 1, 4, 2, 2, 0, 0),    # empty cache
])
def test_kvcache_shift_against_labelled_frames(B, H, F, T, D, kv, drop):
    cache = _labelled_cache(B, H, F, T, D)
    before = cache.copy()
    out = sd.kvcache_shift(cache, T, kv, drop)
    assert np.array_equal(cache, before)                      # the input is not modified
    assert out.shape == cache.shape
    keep = kv - drop
    for b in range(B):
        for h in range(H):
            for f in range(F):
                src = f + drop if f < keep else f              # kept frames move down; the rest stays
                for t in range(T):
                    for d in range(D):
                        want = (((b * 7 + h) * 100 + src) * 100 + t) * 100 + d
                        assert out[b, h, f * T + t, d] == want, (b, h, f, t, d)


def test_kvcache_shift_composes():
    """Dropping a then b frames equals dropping a + b at once on the frames that remain."""
    cache = _labelled_cache(1, 2, 10, 3, 2)
    one = sd.kvcache_shift(sd.kvcache_shift(cache, 3, 9, 2), 3, 7, 3)
    both = sd.kvcache_shift(cache, 3, 9, 5)
    assert np.array_equal(one[:, :, : 4 * 3], both[:, :, : 4 * 3])
    assert np.array_equal(both[:, :, 9 * 3:], cache[:, :, 9 * 3:])


# ---- the library's bookkeeping against the statement -----------------------------------------------
@pytest.mark.parametrize("seed,total,n_prompt,nframe,window,capacity,adim,n_act", [
    (1, 40, 4, 4, 32, 40, 1, 2), (2, 100, 1, 2, 8, 10, 3, 2), (3, 64, 8, 3, 8, 11, 2, 3), (4, 33, 32, 8, 32, 40, 1, 5),
    (5, 50, 2, 1, 4, 5, 1, 2), (6, 30, 4, 4, 32, 40, 4, 1),
])
def test_library_bookkeeping_equals_the_plain_loop(seed, total, n_prompt, nframe, window, capacity, adim, n_act):
    rng = np.random.default_rng(seed)
    # actions that persist for a few frames, as the paper observes for gameplay
    runs = rng.integers(1, 7, size=total)
    vals = rng.integers(0, n_act, size=(total, adim))
    a = np.repeat(vals, runs, axis=0)[:total].astype(np.int32)
    assert _drive(a, n_prompt, nframe, window, capacity) == sd.run(a, n_prompt, nframe, window, capacity)


def test_spec_init_rejects_bad_arguments():
    with pytest.raises(nb.NfdError) as e:
        nb.nfd_spec_init(40, 38, 4, 4, 100)   # window + n_spec > capacity
    assert e.value.code == nb.NFD_ERR_CAPACITY
    with pytest.raises(nb.NfdError) as e:
        nb.nfd_spec_init(40, 32, 0, 4, 100)
    assert e.value.code == nb.NFD_ERR_SHAPE
    with pytest.raises(nb.NfdError) as e:
        nb.nfd_spec_init(40, 32, 4, 4, 3)     # fewer frames than the prompt
    assert e.value.code == nb.NFD_ERR_SHAPE
