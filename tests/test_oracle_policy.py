"""Pins of the index oracle (oracle/policy.py): hand-worked fixtures, the printed form of Eq. 4
evaluated in exact rationals, set-membership brute force, and structural invariants."""
from fractions import Fraction
import math

import numpy as np
import pytest

from oracle import policy as P
from paper_2605_13111_amd import synth
import helpers
from helpers import read_policy_fixture


def test_hand_worked_selections():
    n = 0
    for pol, T, expect, source in read_policy_fixture("policy_cases.txt"):
        want = [int(x) for x in expect.split()]
        scores = {f: 0.0 for f in range(T)}
        assert P.selected_frames(pol, T, scores) == want, source
        n += 1
    assert n >= 14


def test_counts_stated_by_the_workloads():
    for pol, T, expect, source in read_policy_fixture("policy_counts.txt"):
        scores = {f: float((f * 37) % 101) for f in range(T)}
        assert len(P.selected_frames(pol, T, scores)) == int(expect), source


@pytest.mark.parametrize("t", range(1, 81))
def test_eq4_printed_form_in_exact_rationals(t):
    """Eq. 4 prints 1-indexed positions t - i*(t/Cap) - floor(t/(2Cap)) with a real stride.  The oracle's
    integer form must be that position rounded up to a whole frame, converted to 0-based ids."""
    middle = list(range(t))
    for cap in range(1, 12):
        got = P.anchor_strided(middle, cap)
        if t <= cap:
            assert got == set(middle)
            continue
        want = set()
        for i in range(cap):
            pos = Fraction(t) - i * Fraction(t, cap) - (t // (2 * cap))
            want.add(math.ceil(pos) - 1)
        assert got == want
        assert len(got) == cap and min(got) >= 0 and max(got) <= t - 1
        if t % cap == 0 and (t // cap) % 2 == 1:
            s = t // cap                                  # odd stride: picks are exact window centres
            assert got == {w * s + s // 2 for w in range(cap)}


def test_wave_by_membership_brute_force():
    """Eq. 5 / Observation 2 restated as a membership test: a middle frame f is picked iff its distance
    to the chunk's first frame is a positive multiple of P; with a cap, the nearest ones win."""
    for T in range(0, 70):
        for S in (0, 1, 3):
            for R in (0, 2, 4):
                middle = P.middle_frames(T, S, R)
                for period in (1, 2, 3, 4, 6, 7):
                    hits = [f for f in middle if (T - f) % period == 0 and T - f > 0]
                    for cap in (0, 1, 4):
                        want = set(sorted(hits, reverse=True)[:cap] if cap else hits)
                        assert P.wave_periodic(T, middle, period, cap) == want


def test_topk_by_counting_brute_force():
    rng = np.random.default_rng(5)
    for trial in range(200):
        n = int(rng.integers(1, 30))
        cap = int(rng.integers(1, 12))
        middle = sorted(rng.choice(100, size=n, replace=False).tolist())
        # coarse scores so that ties occur
        score = {f: np.float32(rng.integers(0, 6)) / np.float32(4) for f in middle}
        got = P.anchor_topk(middle, cap, score)
        if n <= cap:
            assert got == set(middle)
            continue
        # f is kept iff fewer than cap frames beat it (higher score, or equal score and smaller id)
        want = {f for f in middle
                if sum(1 for g in middle if score[g] > score[f] or (score[g] == score[f] and g < f)) < cap}
        assert got == want and len(got) == cap


def _all_policies():
    pols = []
    for S in (0, 1, 3):
        for R in (0, 2, 4):
            pols.append(synth.HeadPolicy(synth.ANCHOR, synth.MODE_ALL, S, R, 0, 1, 10 ** 6))
            pols.append(synth.HeadPolicy(synth.VEIL, 0, S, R, 0, 1, 10 ** 6))
            for cap in (0, 2, 4, 18):
                pols.append(synth.HeadPolicy(synth.ANCHOR, synth.MODE_STRIDED, S, R, cap, 1, 10 ** 6))
                pols.append(synth.HeadPolicy(synth.ANCHOR, synth.MODE_TOPK, S, R, cap, 1, 10 ** 6))
                for period in (2, 3, 6):
                    pols.append(synth.HeadPolicy(synth.WAVE, 0, S, R, cap, period, 10 ** 6))
    return pols


def test_selection_invariants():
    rng = np.random.default_rng(11)
    score = {f: np.float32(rng.random()) for f in range(100)}
    for pol in _all_policies():
        for T in range(0, 81):
            sel = P.selected_frames(pol, T, {f: score[f] for f in range(T)})
            assert sel == sorted(set(sel)), "strictly ascending"
            assert all(0 <= f < T for f in sel), "history frames only (Sec. 2.2: I(t) is a subset of H(t))"
            assert P.sink_frames(T, pol.sink) <= set(sel) and P.recent_frames(T, pol.recent) <= set(sel)
            middle = P.middle_frames(T, pol.sink, pol.recent)
            typed = set(sel) - P.sink_frames(T, pol.sink) - P.recent_frames(T, pol.recent)
            assert typed <= set(middle)
            if pol.type == synth.VEIL:
                assert not typed
            if pol.cap > 0 and pol.type != synth.VEIL and not (pol.type == synth.ANCHOR and pol.mode == synth.MODE_ALL):
                assert len(typed) <= pol.cap
            if pol.sink == 0 and pol.recent == 0 and pol.type == synth.ANCHOR and pol.mode == synth.MODE_ALL:
                assert sel == list(range(T))


def test_selection_is_always_retained_when_streaming():
    """Whatever chunk sizes the history is appended in, the frames a head selects are frames the
    retention rule has kept (Sec. 2.2: I(t) is chosen from the candidate history H(t))."""
    rng = np.random.default_rng(3)
    score = {f: np.float32(rng.integers(0, 50)) / np.float32(7) for f in range(200)}
    for pol in _all_policies():
        for chunks in ([1] * 60, [3] * 25, [1, 3, 2, 5, 1, 1, 4] * 6):
            resident, T = [], 0
            for n_new in chunks:
                cand = resident + list(range(T, T + n_new))
                T += n_new
                resident = P.retained_frames(pol, T, cand, score)
                assert resident == sorted(resident)
                sel = P.selected_frames(pol, T, {f: score[f] for f in resident})
                assert set(sel) <= set(resident)
                # streaming == batch: same selection as with the whole history at hand
                assert sel == P.selected_frames(pol, T, {f: score[f] for f in range(T)})
                # and the retained set equals one retention pass over the whole history
                assert resident == P.retained_frames(pol, T, list(range(T)), score)


def test_hand_worked_retained_sets():
    """tests/golden/retained_cases.txt: the exact retained set, worked out by hand from Eq. 5 / Observation 1."""
    n = 0
    for pol, T, expect, source in read_policy_fixture("retained_cases.txt"):
        want = [int(x) for x in expect.split()]
        assert P.retained_frames(pol, T, range(T)) == want, (pol, T, source)
        n += 1
    assert n >= 6


def test_retention_keeps_exactly_what_a_later_step_can_select():
    """For the policies that evict (capped Wave, Veil with and without merging, Anchor top-k with static scores) the
    retained set at history length T equals the union, over this and every later step, of the history frames below
    T that the step attends to: nothing is missing (sufficiency) and nothing is kept in vain (no over-retention)."""
    rng = np.random.default_rng(11)
    score = {f: np.float32(rng.integers(0, 40)) / np.float32(3) for f in range(400)}
    pols = []
    for S in (0, 1, 3):
        for R in (0, 2, 4):
            pols.append(synth.HeadPolicy(synth.VEIL, 0, S, R, 0, 1, 10 ** 6))
            for cap in (1, 2, 4):
                for period in (1, 2, 3, 6):
                    pols.append(synth.HeadPolicy(synth.WAVE, 0, S, R, cap, period, 10 ** 6))
                    pols.append(synth.HeadPolicy(synth.VEIL, 0, S, R, cap, period, 10 ** 6))
                pols.append(synth.HeadPolicy(synth.ANCHOR, synth.MODE_TOPK, S, R, cap, 1, 10 ** 6))
    M = P.MERGED
    for pol in pols:
        horizon = pol.recent + (pol.cap + 1) * max(pol.period, 1) + pol.sink + 2     # later steps that can still reach below T
        for T in (0, 1, 5, 13, 30):
            needed = set()
            for T2 in range(T, T + horizon + 1):
                for f in P.selected_frames(pol, T2, {g: score[g] for g in range(T2)}):
                    if f & M:                                  # a merged window needs its m source frames
                        needed |= {g for g in range(f & ~M, (f & ~M) + pol.period) if g < T}
                    elif f < T:
                        needed.add(f)
            kept = P.retained_frames(pol, T, range(T), {g: score[g] for g in range(T)})
            assert set(kept) == needed, (pol, T, sorted(needed), kept)


def test_cu_seqlens_is_an_exclusive_prefix_sum():
    """Sec. 4.3: cu_seqlens_i = sum of the lengths before sequence i; sequence i occupies [cu_i, cu_{i+1})."""
    assert P.cu_seqlens([12, 4, 3, 3], 16) == [0, 192, 256, 304, 352]
    assert P.cu_seqlens([], 7) == [0]
    rng = np.random.default_rng(0)
    counts = rng.integers(0, 60, size=40).tolist()
    cu = P.cu_seqlens(counts, 1560)
    assert cu[0] == 0 and cu[-1] == 1560 * sum(counts)
    assert all(cu[i + 1] - cu[i] == counts[i] * 1560 for i in range(40))


# ---------------------------------------------------------------- Veil cache merging (Sec. 4.2)
def test_veil_merging_windows_and_key_sequence():
    """Paper defaults for Veil heads: sink 3, forced recent 4, 2 merged frames, window 2.  At T = 20 the recent
    frames are 16..19, so the windows are [14,16) and [12,14); each is ONE entry of the key sequence."""
    pol = helpers.veil_merged(3, 4, 2, 2)
    M = P.MERGED
    assert P.selected_frames(pol, 20) == [0, 1, 2, M | 12, M | 14, 16, 17, 18, 19]
    # a window exists only if it lies entirely between the sink and the recent frames
    assert P.selected_frames(pol, 9) == [0, 1, 2, M | 3, 5, 6, 7, 8]            # [3,5) fits, [1,3) does not
    assert P.selected_frames(pol, 8) == [0, 1, 2, 4, 5, 6, 7]                   # [2,4) overlaps the sink
    assert P.selected_frames(pol, 5) == [0, 1, 2, 3, 4]                         # sink and recent overlap
    assert P.selected_frames(pol, 0) == []
    # without forced recent frames the window is the m frames before the current one: merged(t-m : t)
    assert P.selected_frames(helpers.veil_merged(1, 0, 1, 3), 10) == [0, M | 7]
    # retention: sink, recent, and the Cap*m frames the windows of this and any later step are made of
    assert P.retained_frames(pol, 20, range(20)) == [0, 1, 2] + list(range(12, 20))
    # cap = 0 is the plain Veil policy
    assert P.selected_frames(synth.veil(3, 4), 20) == [0, 1, 2, 16, 17, 18, 19]


def test_merged_frame_composition():
    """Frame i of the window contributes the tokens congruent to i modulo m, in order; the pieces are
    concatenated in window order and add up to exactly one frame of tokens, also when m does not divide it."""
    assert P.merged_rows(2, 6) == [(0, 0), (0, 2), (0, 4), (1, 1), (1, 3), (1, 5)]
    assert P.merged_rows(3, 7) == [(0, 0), (0, 3), (0, 6), (1, 1), (1, 4), (2, 2), (2, 5)]
    for m in (1, 2, 3, 4, 5):
        for tpf in (1, 7, 16, 1560):
            rows = P.merged_rows(m, tpf)
            assert len(rows) == tpf and sorted(t for _, t in rows) == list(range(tpf))   # every token position once
            assert all(t % m == i for i, t in rows)
