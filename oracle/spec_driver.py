"""Plain statement of the speculative-sampling bookkeeping and of the sliding context window.

TEST INFRASTRUCTURE ONLY (imported by tests/ alone).

What Sec. 4.2 describes, stated as a rule on the action sequence: a model call is conditioned on
the action of the first frame it has to produce, repeated for every frame of the chunk; a
produced frame is valid exactly when the action it was really due under equals that
conditioning action and every frame before it in the chunk was valid as well; the first
mismatch invalidates everything after it; the next call starts right after the last valid
frame.  The chunk's first frame is produced under its own action, so every call yields at least
one frame.  The model itself is outside: only which frames are produced, kept and cached is
tracked.

The context kept for the next call is limited to ``window`` frames (Sec. 5, Limitations): the
oldest frames are evicted before a call when more than ``window`` verified frames are cached.

``kvcache_shift`` is the eviction as an array operation.  Both functions are pinned by
tests/test_spec_driver.py (hand-worked sequences, per-frame slicing).
"""
import numpy as np


def valid_prefix(chunk_actions):
    """Number of leading frames of a chunk whose true action equals the action the chunk was
    conditioned on (the action of its first frame).  Always >= 1."""
    conditioned_on = chunk_actions[0]
    valid = 0
    for true_action in chunk_actions:
        if not np.array_equal(true_action, conditioned_on):
            break
        valid += 1
    return valid


def run(actions, n_prompt, nframe, window, capacity):
    """actions: int array [total, action_dim].  Returns the list of model calls, each a dict with
    the frames generated (absolute indices), the number kept, and the cache picture before the
    call: ``evict`` oldest frames dropped, ``cache_frames`` = absolute indices of the verified
    frames in the cache after the eviction (slot order)."""
    actions = np.asarray(actions)
    total = actions.shape[0]
    assert window + nframe <= capacity and n_prompt <= capacity
    context = list(range(n_prompt))  # verified frames held as context, oldest first
    calls = []
    verified = n_prompt              # frames of the video that are final
    while verified < total:
        evict = max(0, len(context) - window)
        del context[:evict]
        produced = list(range(verified, min(verified + nframe, total)))
        kept = valid_prefix(actions[produced[0]: produced[-1] + 1])
        calls.append(dict(evict=evict, cache_frames=list(context), generated=produced, kept=kept))
        context.extend(produced[:kept])
        verified += kept
    return calls


def kvcache_shift(cache, T, kv_frames, n_drop):
    """Drop the oldest n_drop of the kv_frames cached frames of a [B, H, F*T, D] cache: frame
    n_drop + f becomes frame f; everything from frame kv_frames - n_drop on is left as it was.
    Returns a new array."""
    frames = [cache[:, :, f * T:(f + 1) * T] for f in range(cache.shape[2] // T)]
    moved = frames[n_drop:kv_frames] + frames[kv_frames - n_drop:]
    assert len(moved) == len(frames)
    return np.concatenate(moved, axis=2) if moved else np.array(cache, copy=True)
