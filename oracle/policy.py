"""Index oracle: the frames a head retains and the frames it attends to.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).

Notation.  History frames carry global ids ``0 .. T-1``; the chunk being
generated starts at id ``T`` (so ``T`` plays the role of the paper's current
frame index ``t``).  Every head has the parameters

    type    0 Anchor, 1 Wave, 2 Veil           (Sec. 4.1, the three head sets)
    mode    Anchor only: 0 ALL, 1 STRIDED, 2 TOPK
    sink    S  shared sink frames               (Sec. 4.2, last paragraph)
    recent  R  force-preserved recent frames    (Sec. 4.2, last paragraph)
    cap     Cap, 0 = unlimited                  (Eq. 4, Eq. 5); Veil: number of merged
                                                frames, 0 = no cache merging
    period  P, Wave                             (Eq. 5, Observation 2); Veil: size m of
                                                the local window that is merged (Sec. 4.2)

The head-type policy acts on the *intermediate* history between the sink and
the recent window (Sec. 4.2, last paragraph), written ``middle`` below.

Everything is written with Python sets and sorted lists so it can be checked
against the paper by eye.
"""

ANCHOR, WAVE, VEIL = 0, 1, 2
MODE_ALL, MODE_STRIDED, MODE_TOPK = 0, 1, 2
MERGED = 1 << 30        # flag of a merged-frame entry: MERGED | id of the window's first frame


def sink_frames(T, S):
    """The first S frames of the history (Sec. 2.2, sink frames)."""
    return set(range(0, min(S, T)))


def recent_frames(T, R):
    """The last R frames of the history (Sec. 2.2, recent frames)."""
    return set(range(max(0, T - R), T))


def middle_frames(T, S, R):
    """Ascending list of the intermediate ids S .. T-R-1 (may be empty)."""
    return list(range(S, max(S, T - R)))


def anchor_strided(middle, cap):
    """Adaptive strided sliding window (Eq. 4) on the intermediate history.

    With t' = len(middle) frames and Cap windows of (real) stride t'/Cap, the
    i-th pick counted back from the newest frame sits at 0-based offset
    (t'-1) - floor(i*t'/Cap) - floor(t'/(2*Cap)): the centre of its window.
    When the history is not longer than Cap every frame is kept.
    """
    t = len(middle)
    if cap <= 0 or t <= cap:
        return set(middle)
    picks = set()
    for i in range(cap):
        offset = (t - 1) - (i * t) // cap - t // (2 * cap)
        picks.add(middle[offset])
    return picks


def anchor_topk(middle, cap, score_of):
    """The Cap intermediate frames with the largest score; equal scores are
    ordered by smaller frame id first.  ``score_of`` maps id -> float32 score."""
    if cap <= 0 or len(middle) <= cap:
        return set(middle)
    ranked = sorted(middle, key=lambda f: (-float(score_of[f]), f))
    return set(ranked[:cap])


def wave_periodic(T, middle, period, cap):
    """Periodic sampling (Eq. 5, Observation 2): frames T - i*P, i >= 1, that
    fall in the intermediate history; the Cap nearest ones if Cap > 0."""
    inside = set(middle)
    picks = []
    i = 1
    while T - i * period >= 0:
        f = T - i * period
        if f in inside:
            picks.append(f)
        i += 1
    if cap > 0:
        picks = picks[:cap]
    return set(picks)


def veil_windows(T, S, R, cap, m):
    """Cache merging of Veil heads (Sec. 4.2): the local windows of m frames that are each compressed into one
    merged frame.  Window j (j = 0 nearest) covers the m frames right before the previous window, starting from
    the forced recent frames: ids T-R-(j+1)m .. T-R-jm-1; a window exists only if it lies entirely in the
    intermediate history.  Returns the first frame ids of the existing windows, ascending."""
    starts = []
    for j in range(cap):
        w0 = T - R - (j + 1) * m
        if m >= 1 and w0 >= S:
            starts.append(w0)
    return sorted(starts)


def merged_rows(m, tokens_per_frame):
    """Composition of a merged frame (Sec. 4.2, K_merged = Concat_i K[t-m+i, C_i]): list of (i, token) pairs, one
    per row, where frame i of the window contributes its i-th 1/m subset C_i = {token : token mod m == i}."""
    rows = []
    for i in range(m):
        for tok in range(tokens_per_frame):
            if tok % m == i:
                rows.append((i, tok))
    return rows


def selected_frames(pol, T, score_of=None):
    """List of the frames head ``pol`` attends to when the chunk starting at id T is generated, in the order of
    its key sequence: sink + type policy on the middle + recent, ascending ids.  A Veil head with cache merging
    has entries MERGED | w0 (one per merged window, ascending) between its sink and its recent frames."""
    middle = middle_frames(T, pol.sink, pol.recent)
    if pol.type == VEIL and pol.cap > 0:
        sink = sorted(sink_frames(T, pol.sink))
        recent = sorted(recent_frames(T, pol.recent) - set(sink))
        return sink + [MERGED | w0 for w0 in veil_windows(T, pol.sink, pol.recent, pol.cap, pol.period)] + recent
    if pol.type == ANCHOR:
        if pol.mode == MODE_ALL:
            typed = set(middle)
        elif pol.mode == MODE_STRIDED:
            typed = anchor_strided(middle, pol.cap)
        elif pol.mode == MODE_TOPK:
            # ranked over the candidate history: ids that still have a score
            typed = anchor_topk([f for f in middle if f in score_of], pol.cap, score_of)
        else:
            raise ValueError("bad anchor mode")
    elif pol.type == WAVE:
        typed = wave_periodic(T, middle, pol.period, pol.cap)
    elif pol.type == VEIL:
        typed = set()
    else:
        raise ValueError("bad head type")
    return sorted(sink_frames(T, pol.sink) | recent_frames(T, pol.recent) | typed)


def retained_frames(pol, T_new, candidates, score_of=None):
    """Ascending list of the candidate ids the pool keeps once the history has
    T_new frames (Sec. 2.2: the retained candidate set H(t+1)).

    The retained set must contain everything any later selection can ask for:
      Anchor ALL / STRIDED  every frame (the strided picks wander over all ids);
      Anchor TOPK           sink + recent + the Cap best-scored middle frames
                            (scores never change, so a frame that drops out of
                            the best Cap never re-enters);
      Wave, Cap = 0         every frame;
      Wave, Cap > 0         sink + recent + every id >= T_new - (floor(R/P)+Cap)*P,
                            the oldest id a later chunk can still pick;
      Veil                  sink + recent; with cache merging also the Cap*m frames before the recent
                            ones (the sources of this and every later step's merged windows).
    """
    cand = sorted(candidates)
    keep = sink_frames(T_new, pol.sink) | recent_frames(T_new, pol.recent)
    middle = [f for f in middle_frames(T_new, pol.sink, pol.recent) if f in set(cand)]
    if pol.type == ANCHOR and pol.mode in (MODE_ALL, MODE_STRIDED):
        keep |= set(cand)
    elif pol.type == ANCHOR and pol.mode == MODE_TOPK:
        keep |= anchor_topk(middle, pol.cap, score_of)
    elif pol.type == WAVE:
        if pol.cap <= 0:
            keep |= set(cand)
        else:
            oldest = T_new - (pol.recent // pol.period + pol.cap) * pol.period
            keep |= {f for f in cand if f >= oldest}
    elif pol.type == VEIL:
        if pol.cap > 0:
            keep |= {f for f in cand if f >= T_new - pol.recent - pol.cap * pol.period}
    else:
        raise ValueError("bad head policy")
    return [f for f in cand if f in keep]


def cu_seqlens(sel_counts, tokens_per_frame):
    """Boundary indices of the flattened ragged history (Sec. 4.3):
    cu[0] = 0, cu[i+1] = cu[i] + L_i with L_i the selected history tokens of
    sequence i, sequences in batch-head order."""
    cu = [0]
    for n in sel_counts:
        cu.append(cu[-1] + n * tokens_per_frame)
    return cu
