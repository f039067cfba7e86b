"""Oracle of the offline tri-pattern head classification (Sec. 4.1 and the appendix paragraph on the FFT
analysis stage).

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).

Input: for every sampled prompt p and head h (all layers' heads in one axis) the historical attention sequence
``a[p, h, t]``, the pre-softmax score of the newest frame towards history frame t (Sec. 4.1).  Everything is
fp64 numpy; the steps follow the paper's order:

  1. sign rates r_pos = mean(a > 0), r_neg = 1 - r_pos (the equation of Sec. 4.1);
     r_pos >= alpha -> Anchor, r_neg >= alpha -> Veil
  2. otherwise the dominant period P of the sequence: first-order difference, mean removal, Hann window, real
     FFT, zero-frequency bin dropped, harmonic folding, period = 1/f (appendix);  P < beta -> Wave
  3. otherwise the mean-score fallback: mean(a) > 0 -> Anchor, else Veil
  4. per head, majority vote over the prompts (caption of the classification-results figure)

Readings where the paper is silent (listed with the others in the design notes):
  * the Hann window is the symmetric one, w[n] = 0.5 - 0.5 cos(2 pi n / (N-1)), N = length of the difference
  * a bin's amplitude is |X[k]|; harmonic folding gives bin k the score sum_{j=1..J} |X[j k]| / j over the
    harmonics j k <= N/2, J = 4 (weights decaying as 1/j)
  * period = N / k for bin k of the length-N transform; equal folded scores (to a relative 1e-9) go to the
    lowest bin; a sequence with fewer than 4 points, or a flat one, has no period (P = inf)
  * equal vote counts go to the smaller type code (Anchor 0 < Wave 1 < Veil 2)
"""
import numpy as np

ANCHOR, WAVE, VEIL = 0, 1, 2
ALPHA, BETA = 0.8, 6.4          # sign-rate and period thresholds of the experimental setup
N_HARMONICS = 4
TIE_REL = 1e-9


def sign_rates(a):
    """(r_pos, r_neg) of one sequence (Sec. 4.1)."""
    a = np.asarray(a, np.float64)
    r_pos = float(np.count_nonzero(a > 0)) / len(a)
    return r_pos, 1.0 - r_pos


def folded_spectrum(a):
    """Folded score of every bin k = 1 .. N//2 of the pre-processed sequence; index 0 of the result is bin 1.
    Returns (scores, N)."""
    a = np.asarray(a, np.float64)
    d = np.diff(a)                                   # first-order difference
    N = len(d)
    if N < 3:
        return np.zeros(0), N
    d = d - d.mean()                                 # mean removal
    d = d * np.hanning(N)                            # Hann window
    amp = np.abs(np.fft.rfft(d))                     # bins 0 .. N//2
    nb = N // 2
    score = np.zeros(nb)
    for k in range(1, nb + 1):                       # harmonic folding onto the fundamental
        for j in range(1, N_HARMONICS + 1):
            if j * k <= nb:
                score[k - 1] += amp[j * k] / j
    return score, N


def dominant_period(a):
    """Top-1 period estimate of one sequence, in frames (inf when there is none)."""
    score, N = folded_spectrum(a)
    if len(score) == 0 or not np.isfinite(score).all() or score.max() <= 0.0:
        return float("inf")
    best = score.max()
    k = int(np.nonzero(score >= best * (1.0 - TIE_REL))[0][0]) + 1     # lowest bin among equals
    return N / k


def classify_sequence(a, alpha=ALPHA, beta=BETA):
    """(type, period) of one (prompt, head) sequence; period is inf when step 2 was not reached."""
    r_pos, r_neg = sign_rates(a)
    if r_pos >= alpha:
        return ANCHOR, float("inf")
    if r_neg >= alpha:
        return VEIL, float("inf")
    P = dominant_period(a)
    if P < beta:
        return WAVE, P
    return (ANCHOR if float(np.mean(np.asarray(a, np.float64))) > 0.0 else VEIL), P


def classify_heads(logits, alpha=ALPHA, beta=BETA):
    """logits: [n_prompts, n_heads, n_hist].  Returns (head_type [n_heads], prompt_type [n_prompts, n_heads],
    prompt_period [n_prompts, n_heads])."""
    logits = np.asarray(logits, np.float64)
    n_p, n_h, _ = logits.shape
    ptype = np.zeros((n_p, n_h), np.int32)
    pper = np.zeros((n_p, n_h), np.float64)
    for p in range(n_p):
        for h in range(n_h):
            ptype[p, h], pper[p, h] = classify_sequence(logits[p, h], alpha, beta)
    head = np.zeros(n_h, np.int32)
    for h in range(n_h):
        votes = np.bincount(ptype[:, h], minlength=3)
        head[h] = int(np.argmax(votes))               # argmax returns the first (smallest code) among equals
    return head, ptype, pper
