"""Where the range pass leaves the parts of a sequence: sd_range_parts (closed form, shared with the merge
kernel) against a replay of what the waves do.  Host only: no kernel is launched.

The replay follows the range pass step by step.  A line of T tiles is cut into ranges of `per` tiles; range r
is walked by wave r % 4 of workgroup r // 4.  A wave goes through the segments of its piece in order and
stores the result of every segment but the last at once (the whole sequence -> finished rows, a part -> a
partial).  The last segment is stored after the workgroup's barrier, unless the wave hands it to the wave
before it: that happens when the segment began before the piece and the wave is not the workgroup's first.
A wave that keeps its last segment adds the handed-over ones of the waves right after it.
"""
import os
import random

import pytest

import paper_2508_11553_amd as sd
from paper_2508_11553_amd import build as sd_build


@pytest.fixture(scope="module", autouse=True)
def lib():
    if not os.path.exists(sd.lib_path()):
        sd_build.build()
    return sd.load()


def replay(offsets, per):
    """offsets: tile offsets of the sequences (len B + 1).  Returns {b: sorted ranges that store a partial of b}
    and the set of sequences whose rows the range pass finishes itself."""
    T = offsets[-1]
    ranges = (T + per - 1) // per
    partial_in = {}
    finished = set()

    def segments(r):
        g0, g1 = r * per, min(T, (r + 1) * per)
        out = []
        for b in range(len(offsets) - 1):
            o0, o1 = offsets[b], offsets[b + 1]
            if o1 > o0 and o0 < g1 and o1 > g0:
                out.append((b, max(g0, o0) - o0, min(g1, o1) - o0, o1 - o0))
        return out

    def store(b, lt0, lt1, n, r):
        if lt0 == 0 and lt1 == n:
            finished.add(b)
        else:
            partial_in.setdefault(b, []).append(r)

    for wg in range((ranges + 3) // 4):
        last = {}
        for w in range(4):
            r = 4 * wg + w
            if r >= ranges:
                continue
            segs = segments(r)
            for s in segs[:-1]:
                store(*s, r)
            last[w] = segs[-1]
        hands_over = {w: w > 0 and last[w][1] > 0 for w in last}
        for w in sorted(last):
            if hands_over[w]:
                continue
            b, lt0, lt1, n = last[w]
            v = w + 1
            while v in last and hands_over[v]:
                assert last[v][0] == b and last[v][1] == lt1   # it continues where the run ends
                lt1 = last[v][2]
                v += 1
            store(b, lt0, lt1, n, 4 * wg + w)
    return partial_in, finished


@pytest.mark.parametrize("seed", range(40))
def test_parts_of_random_batches(seed):
    rng = random.Random(seed)
    B = rng.randint(1, 40)
    tiles = [rng.choice([0, 0, 1, 1, 2, 3, 5, 8, 13, 21, 40, 90]) + rng.randint(0, 3) for _ in range(B)]
    offsets = [0]
    for t in tiles:
        offsets.append(offsets[-1] + t)
    if offsets[-1] == 0:
        return
    per = rng.choice([1, 2, 3, 4, 5, 7, 8, 16, 33])
    partial_in, finished = replay(offsets, per)
    for b in range(B):
        o0, o1 = offsets[b], offsets[b + 1]
        if o1 == o0:
            continue
        got = sd.range_parts(o0, o1, offsets[-1], per)
        if b in finished:
            assert b not in partial_in and len(got) == 1, (b, got)
        else:
            assert got == sorted(partial_in[b]) and len(got) >= 2, (b, got, partial_in.get(b))


def test_a_sequence_inside_one_workgroup_is_finished_there():
    # ranges of 8 tiles; tiles [0, 32) are the four ranges of workgroup 0
    assert sd.range_parts(0, 32, 100, 8) == [0]
    # tiles [5, 40): starts inside range 0, runs through workgroup 0 and into the first range of workgroup 1
    assert sd.range_parts(5, 40, 100, 8) == [0, 4]
    # ends inside range 2 while another sequence follows there: range 2 stored its part before going on
    assert sd.range_parts(0, 20, 100, 8) == [0, 2]
    # ends inside range 2 and nothing follows on the line: range 2's part is its last segment and is handed over
    assert sd.range_parts(0, 20, 20, 8) == [0]


def test_bad_geometry_is_refused():
    for args in [(5, 5, 100, 8), (-1, 4, 100, 8), (0, 101, 100, 8), (0, 4, 100, 0)]:
        with pytest.raises(sd.SeamDecodeError):
            sd.range_parts(*args)
