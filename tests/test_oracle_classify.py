"""Pins of the head-classification oracle (Sec. 4.1 + the appendix paragraph on the FFT analysis): closed forms,
invariances and hand-computed cases.  The paper prints no worked example for this step, so there is no golden file."""
import numpy as np
import pytest

from oracle import classify as C
from paper_2605_13111_amd import synth


def _tone(n, period, amp=1.0, phase=0.3):
    return amp * np.sin(2 * np.pi * np.arange(n) / period + phase)


@pytest.mark.parametrize("period", [4.0, 5.0, 6.0, 8.0, 10.0, 12.0])
def test_bin_centred_tone_gives_its_period_exactly(period):
    """121 points -> 120 differences; a period that divides 120 sits on a bin, the difference of a sinusoid is a
    sinusoid of the same period and the Hann window does not move a bin-centred peak: P = 120 / k exactly."""
    assert C.dominant_period(_tone(121, period)) == period


def test_constant_offset_and_linear_trend_do_not_change_the_period():
    """Difference + mean removal: an offset disappears in the difference, a trend becomes an offset of the
    difference and disappears in the mean removal.  Without them the trend's low bins would win (P = 120)."""
    a = _tone(121, 6.0)
    t = np.arange(121)
    assert C.dominant_period(a + 40.0) == 6.0
    assert C.dominant_period(a + 0.5 * t) == 6.0
    assert C.dominant_period(a + 40.0 - 0.2 * t) == 6.0


def test_harmonic_folding_moves_the_peak_to_the_fundamental():
    """x = 1.0 sin(2 pi t/12) + 0.7 sin(2 pi t/6).  The difference scales a tone of frequency f by 2 sin(pi f):
    0.5176 for period 12 and 0.7 for period 6, so the raw spectrum peaks at period 6; folded with weights 1/j
    the fundamental scores 0.5176 + 0.7/2 = 0.868 > 0.7 (both tones are bin-centred and windowed alike), so the
    estimate is 12.  Swapping the amplitudes' ratio below 1/2 of the harmonic keeps 6."""
    n = 121
    assert C.dominant_period(_tone(n, 12.0, 1.0) + _tone(n, 6.0, 0.7, phase=1.1)) == 12.0
    assert C.dominant_period(_tone(n, 12.0, 0.3) + _tone(n, 6.0, 0.7, phase=1.1)) == 6.0   # 0.155 + 0.35 < 0.7


def test_spectrum_amplitudes_are_those_of_the_dft_definition():
    """|rfft| of the pre-processed sequence = the O(N^2) sum of the definition; checks bins, window and folding
    weights through the first bin of a white sequence (score[0] = sum_j |X[j]| / j, j = 1..4)."""
    rng = np.random.default_rng(7)
    a = rng.standard_normal(40)
    d = np.diff(a)
    d = d - d.mean()
    n = len(d)
    w = 0.5 - 0.5 * np.cos(2 * np.pi * np.arange(n) / (n - 1))
    X = np.array([abs(sum(d[m] * w[m] * np.exp(-2j * np.pi * k * m / n) for m in range(n))) for k in range(n // 2 + 1)])
    score, N = C.folded_spectrum(a)
    assert N == 39 and len(score) == 19
    assert score[0] == pytest.approx(X[1] + X[2] / 2 + X[3] / 3 + X[4] / 4, rel=1e-12)
    assert score[7] == pytest.approx(X[8] + X[16] / 2, rel=1e-12)           # bins 24, 32 are past N/2 = 19
    assert score[18] == pytest.approx(X[19], rel=1e-12)


def test_sign_rate_thresholds_are_inclusive():
    base = np.array([1.0] * 8 + [-1.0] * 2)                      # r_pos = 0.8
    assert C.sign_rates(base) == (0.8, pytest.approx(0.2))
    assert C.classify_sequence(np.tile(base, 5))[0] == C.ANCHOR
    assert C.classify_sequence(np.tile(-base, 5))[0] == C.VEIL
    almost = np.array([1.0] * 79 + [-1.0] * 21)                 # r_pos = 0.79: not decided by the sign rate
    assert C.classify_sequence(almost)[0] == C.ANCHOR             # ... but by the mean fallback (no short period)
    assert np.isfinite(C.classify_sequence(almost)[1])            # the period was computed on the way
    assert C.classify_sequence(np.zeros(30) - 1e-3)[0] == C.VEIL  # zeros are not positive


def test_wave_needs_a_short_period_and_a_balanced_sign():
    t, p = C.classify_sequence(_tone(121, 6.0, 1.5))
    assert (t, p) == (C.WAVE, 6.0)
    # the same oscillation on a positive bias is one-sided: the sign rate decides first (the "pseudo-periodic" case)
    assert C.classify_sequence(_tone(121, 6.0, 1.0) + 2.0)[0] == C.ANCHOR
    assert C.classify_sequence(_tone(121, 6.0, 1.0) - 2.0)[0] == C.VEIL
    # period threshold is strict: 65 points -> N = 64; bin 10 is period 6.4 (not < 6.4), bin 11 is 5.82
    assert C.classify_sequence(_tone(65, 6.4, 1.5) + 0.01)[0] == C.ANCHOR     # falls through to the mean
    assert C.classify_sequence(_tone(65, 64.0 / 11.0, 1.5))[0] == C.WAVE
    # slow oscillation, balanced sign: not a wave, the mean decides
    assert C.classify_sequence(_tone(121, 40.0, 1.5) + 0.05)[0] == C.ANCHOR
    assert C.classify_sequence(_tone(121, 40.0, 1.5) - 0.05)[0] == C.VEIL


def test_degenerate_sequences():
    assert C.dominant_period([1.0, -1.0, 1.0]) == float("inf")     # 2 differences: no spectrum
    assert C.dominant_period(np.ones(50)) == float("inf")           # flat: nothing to pick
    # 4 alternating points: r_pos 0.5, 3 differences, one bin (period 3 < 6.4): a Wave like any other oscillation
    assert C.classify_sequence(np.array([1.0, -1.0, 1.0, -1.0])) == (C.WAVE, 3.0)


def test_majority_vote_and_ties():
    a_pos, a_neg, a_wave = np.ones(30), -np.ones(30), _tone(30 + 1, 6.0, 1.5)[:30]
    assert C.classify_sequence(a_wave)[0] == C.WAVE
    logits = np.stack([np.stack([a_pos, a_wave, a_neg, a_pos]),
                       np.stack([a_pos, a_wave, a_neg, a_neg]),
                       np.stack([a_neg, a_pos, a_neg, a_wave])])          # 3 prompts x 4 heads
    head, ptype, _ = C.classify_heads(logits)
    assert ptype.tolist() == [[0, 1, 2, 0], [0, 1, 2, 2], [2, 0, 2, 1]]
    assert head.tolist() == [0, 1, 2, 0]                                   # head 3: one vote each -> smallest code


def test_synthetic_kinds_are_recovered():
    """The seeded sequences used on the GPU side: Anchor-like, Wave-like and Veil-like heads come out as such, the
    one-sided oscillation is NOT a Wave (the paper's first failure case), the slow drifts go by their mean."""
    logits, kinds = synth.head_logits(16, 48, 69, seed=3)
    head, ptype, pper = C.classify_heads(logits.numpy())
    want = {0: C.ANCHOR, 1: C.WAVE, 2: C.VEIL, 3: C.ANCHOR, 4: C.ANCHOR, 5: C.VEIL}
    assert [int(x) for x in head] == [want[int(k)] for k in kinds]
    wave = np.nonzero(kinds.numpy() == 1)[0]
    assert len(wave) > 0 and np.all(np.abs(pper[:, wave] - 6.0) < 0.8)
