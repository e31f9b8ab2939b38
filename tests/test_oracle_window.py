"""Pins for the window-bookkeeping oracle (Sec. 4.2 four regions, Sec. 5.1 frame counts) -- CPU only."""
import random

import oracle
from oracle.window import RollingWindow, update_slots


def test_paper_frame_counts():
    # Sec. 5.1: 18 latent frames = sink 3 + retrieval 9 + recent 3 + denoising 3, chunks of 3 frames,
    # compressed chunks of 1.5 frames: the retrieval region holds 6 of them
    T = 880
    n_out, n_keep = oracle.keep_count(0.25, oracle.RATIO_NONANCHOR, oracle.ANCHOR_FIRST_FRAME, 3, T)
    assert 2 * n_out == 3 * T
    sink, recent, denoise, retrieval = 3 * T, 3 * T, 3 * T, 9 * T
    assert sink + recent + denoise + retrieval == 18 * T
    assert retrieval // n_out == 6 and retrieval % n_out == 0
    # uncompressed chunks: 3 fit (the "3 -> 3.0" row of Tab. 2)
    assert retrieval // (3 * T) == 3


def test_rolling_window_keeps_every_chunk_in_exactly_one_place():
    for sink_chunks, recent_chunks in [(1, 1), (1, 2), (2, 1), (0, 1), (1, 0)]:
        w = RollingWindow(sink_chunks, recent_chunks)
        for c in range(40):
            region, slot, evicted = w.step(c)
            everywhere = list(w.sink) + list(w.ring) + list(w.store)
            assert sorted(everywhere) == list(range(c + 1))                 # nothing lost, nothing doubled
            assert w.sink == list(range(min(c + 1, sink_chunks)))
            assert list(w.ring) == list(range(max(sink_chunks, c - recent_chunks), c + 1)) if c >= sink_chunks else not w.ring
            # the store receives chunks oldest first: store id i is generated chunk sink_chunks + i
            assert w.store == list(range(sink_chunks, sink_chunks + len(w.store)))
            if c >= sink_chunks:
                assert region == "ring" and w.ring_slots[slot] == c
                # the physical ring holds exactly the logical ring
                assert sorted(x for x in w.ring_slots if x is not None) == list(w.ring)
                # eviction starts when the ring is full and then happens at every step
                assert (evicted is not None) == (c >= sink_chunks + recent_chunks + 1)
                if evicted is not None:
                    assert evicted == c - recent_chunks - 1
                # slots fill in ascending order, then rotate
                assert slot == (c - sink_chunks) % (recent_chunks + 1)
            else:
                assert region == "sink" and slot == c and evicted is None


def test_update_slots_hand_cases():
    ok = lambda i: 0 <= i < 100
    # first fill, short of the budget
    s, f = update_slots([-1] * 4, [7, 3], 4, ok)
    assert s == [7, 3, -1, -1] and f == [(0, 7), (1, 3)]
    # the store grew: residents stay, the newcomer is appended
    s, f = update_slots(s, [3, 9, 7], 4, ok)
    assert s == [7, 3, 9, -1] and f == [(2, 9)]
    # full budget, one chunk swapped: only that slot is fetched; rank order does not move residents
    s, f = update_slots([7, 3, 9, 1], [1, 5, 7, 9], 4, ok)
    assert s == [7, 5, 9, 1] and f == [(1, 5)]
    # nothing changed
    s, f = update_slots([7, 5, 9, 1], [9, 1, 5, 7], 4, ok)
    assert s == [7, 5, 9, 1] and f == []
    # two leave, two enter: free slots ascending get the newcomers in rank order
    s, f = update_slots([7, 5, 9, 1], [20, 9, 30, 5], 4, ok)
    assert s == [20, 5, 9, 30] and f == [(0, 20), (3, 30)]
    # the wanted list shrank below a resident's slot: rebuild in rank order, fetching what is not in place
    s, f = update_slots([7, 5, 9, 1], [1, 5], 4, ok)
    assert s == [1, 5, -1, -1] and f == [(0, 1)]
    # invalid and repeated ids are dropped
    s, f = update_slots([-1] * 3, [4, -1, 4, 200, 6], 3, ok)
    assert s == [4, 6, -1] and f == [(0, 4), (1, 6)]
    # empty request clears the region
    s, f = update_slots([4, 6, -1], [], 3, ok)
    assert s == [-1, -1, -1] and f == []


def test_update_slots_invariants_brute_force():
    rng = random.Random(5)
    for trial in range(3000):
        R = rng.randint(1, 6)
        M = rng.randint(1, 9)
        n_old = rng.randint(0, min(R, M))
        old = rng.sample(range(M), n_old) + [-1] * (R - n_old)
        ids = [rng.randint(-1, M) for _ in range(rng.randint(0, R + 2))]
        valid = lambda i: 0 <= i < M
        want = []
        for i in ids:
            if valid(i) and i not in want:
                want.append(i)
        want = want[:R]
        new, fetched = update_slots(list(old), ids, R, valid)
        n = len(want)
        assert sorted(new[:n]) == sorted(want) and all(x == -1 for x in new[n:])   # exactly the wanted set, as a prefix
        for s, i in fetched:
            assert new[s] == i and old[s] != i                                  # only what is not in place moves
        moved = {s for s, _ in fetched}
        for s in range(n):
            if s not in moved:
                assert new[s] == old[s]                                         # everything else stayed
        resident = set(x for x in old if x >= 0) & set(want)
        if all(old.index(i) < n for i in resident):
            assert len(fetched) == n - len(resident)                            # minimal traffic when nothing must move
            for i in resident:
                assert new.index(i) == old.index(i)
        assert [s for s, _ in fetched] == sorted(s for s, _ in fetched)
