"""The bucket path of the row sort leaves every key inside the slot range of its value bin and then orders the row
with a fixed number of register passes: 16-slot windows sorted, then 8+8 merges of neighbouring half windows at
alternating alignments.  How many passes a largest bin of a given size needs is a property of that pass structure,
not of the GPU code; it is checked here on a model of the passes (CPU, no library involved): two passes for bins of
at most 9 keys, three for at most 17, the limits the kernel uses; one key more per bin defeats the same number of passes."""
import random

import pytest


def run_passes(arr, npass):
    a = list(arr)
    n = len(a)
    for s in range(0, n, 16):                     # pass 1: every window [16t, 16t+16) sorted
        a[s:s + 16] = sorted(a[s:s + 16])
    off = 8
    for _ in range(1, npass):                     # later passes: merges of two ordered halves = a sort of 16 slots
        for s in range(off, n, 16):
            a[s:s + 16] = sorted(a[s:s + 16])
        off = 0 if off == 8 else 8
    return a


def arrangement(rng, n, maxbin):
    """Consecutive bins of at most maxbin slots; inside a bin the keys in reversed, rotated or random order."""
    pos, arr = 0, []
    while pos < n:
        sz = min(rng.choice([1, 1, 2, 3, maxbin, maxbin - 1, maxbin // 2 + 1]), n - pos)
        ks = list(range(pos, pos + sz))
        mode = rng.randrange(3)
        if mode == 0:
            ks.reverse()
        elif mode == 1:
            rng.shuffle(ks)
        else:
            ks = ks[sz // 2:] + ks[:sz // 2]
        arr += ks
        pos += sz
    return arr


@pytest.mark.parametrize("maxbin,npass", [(8, 2), (9, 2), (16, 3), (17, 3)])
def test_passes_order_every_arrangement_within_the_bin_limit(maxbin, npass):
    rng = random.Random(100 * maxbin + npass)
    for n in (40, 250, 256):
        for _ in range(1500):
            arr = arrangement(rng, n, maxbin)
            assert run_passes(arr, npass) == sorted(arr)
    # one bin of exactly maxbin keys in reversed order at every alignment to the windows
    for start in range(0, 33):
        arr = list(range(96))
        arr[start:start + maxbin] = arr[start:start + maxbin][::-1]
        assert run_passes(arr, npass) == sorted(arr)


@pytest.mark.parametrize("maxbin,npass", [(10, 2), (18, 3)])
def test_one_key_more_per_bin_needs_another_pass(maxbin, npass):
    rng = random.Random(7 * maxbin)
    failures = 0
    for _ in range(3000):
        arr = arrangement(rng, 256, maxbin)
        failures += run_passes(arr, npass) != sorted(arr)
    assert failures > 0
