"""Which waveforms of a full-size batch the oracle checks.

The STFT kernel deals its workgroups round-robin to the 8 XCDs; each XCD walks its own contiguous range of
128-frame tiles in groups of 64 (the last group partial).  A mistake in that walk would drop, repeat or
misplace whole tiles of some XCD's range only, so the sample is taken from the walk itself: for every XCD
a tile inside its first group, the tile on a group boundary and the last tile of its (partial) last group,
each mapped to the waveform that holds the tile's first frame; plus the first two, the middle and the last
two waveforms, plus three seeded random ones.  These constants restate the kernel's; they are not imported
from it.
"""
import numpy as np

TILE_FRAMES = 128
N_XCD = 8
GROUP = 64
FIXED = [0, 1, 885, 1768, 1769]


def sampled_waveforms(B=1770, T=345, seed=2055):
    n_frames = B * T
    n_ft = -(-n_frames // TILE_FRAMES)
    per_xcd = -(-n_ft // N_XCD)
    picks = set(b for b in FIXED if b < B)
    for xcd in range(N_XCD):
        first = xcd * per_xcd
        last = min(n_ft, first + per_xcd) - 1
        if last < first:
            continue
        n_groups = -(-(last - first + 1) // GROUP)
        mid_group = max(1, n_groups // 2)
        for ft in (first + 17, first + mid_group * GROUP, last):
            ft = min(max(ft, first), last)
            picks.add(min(B - 1, ft * TILE_FRAMES // T))
    rng = np.random.default_rng(seed)
    while len(picks) < min(B, 24 + len(FIXED) + 3):
        picks.add(int(rng.integers(0, B)))
    return sorted(picks)
