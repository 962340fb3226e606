"""Plain statement of the speculative-sampling loop and of the sliding context window.

TEST INFRASTRUCTURE ONLY (imported by tests/ alone).  It follows the control flow of the
paper's speculative sampling (Sec. 4.2; Appendix A, "Detailed Algorithm of Speculative
Sampling") in the paper's notation: ``i`` is the number of frames verified so far, every
iteration generates ``nframe`` frames under the action of frame ``i`` repeated, and then
advances ``i`` by ``nframe`` when the true actions of the chunk are all the same, otherwise by
the number of leading frames whose action still equals that of frame ``i``.  The model itself is
outside: only which frames are generated, kept and cached is tracked.

The context kept for the next call is limited to ``window`` frames (Sec. 5, Limitations): the
oldest frames are evicted before a call when more than ``window`` verified frames are cached.
"""
import numpy as np


def run(actions, n_prompt, nframe, window, capacity):
    """actions: int array [total, action_dim].  Returns the list of steps, each a dict with the
    frames generated (absolute indices), the number kept, and the cache picture before the call:
    ``evict`` oldest frames dropped, ``cache_frames`` = absolute indices of the verified frames in
    the cache after the eviction (slot order)."""
    actions = np.asarray(actions)
    total = actions.shape[0]
    assert window + nframe <= capacity and n_prompt <= capacity
    cache = list(range(n_prompt))  # absolute frame indices, oldest first
    i = n_prompt
    steps = []
    while i < total:
        evict = max(0, len(cache) - window)
        cache = cache[evict:]
        n = min(nframe, total - i)
        chunk = actions[i:i + n]
        same_action = bool(np.all(chunk == chunk[0]))
        if same_action:
            kept = n
        else:
            first_change = next(j for j in range(1, n) if np.any(chunk[j] != chunk[0]))
            kept = first_change
        steps.append(dict(evict=evict, cache_frames=list(cache), generated=list(range(i, i + n)), kept=kept))
        cache += list(range(i, i + kept))
        i += kept
    return steps


def kvcache_shift(cache, T, kv_frames, n_drop):
    """Drop the oldest n_drop of the kv_frames cached frames: returns a new array."""
    out = np.array(cache, copy=True)
    keep = kv_frames - n_drop
    out[:, :, : keep * T] = cache[:, :, n_drop * T: kv_frames * T]
    return out
