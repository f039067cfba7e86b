"""Shared helpers for the tests: fixture parsing, and an independent dense-mask attention."""
import os

import numpy as np

from paper_2605_13111_amd import synth

from oracle import policy as OP

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")

_TYPE = {"A": synth.ANCHOR, "W": synth.WAVE, "V": synth.VEIL}
_MODE = {"all": synth.MODE_ALL, "strided": synth.MODE_STRIDED, "topk": synth.MODE_TOPK, "-": 0}


def read_policy_fixture(name):
    """Yield (HeadPolicy, T, expected-field-string, source) for each case line of a golden file."""
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            head, expect, source = [p.strip() for p in line.split("|")]
            ty, mode, S, R, cap, P, T = head.split()
            pol = synth.HeadPolicy(_TYPE[ty], _MODE[mode], int(S), int(R), int(cap), int(P), 10 ** 6)
            yield pol, int(T), expect, source


def dense_masked_attention(q, k_all, v_all, mask, scale):
    """Brute-force check, independent of the oracle's code path: dense logits of every query against
    EVERY history + chunk token, then an explicit boolean mask (False -> -inf) per head.
    q [H,Lq,D], k_all/v_all [H,Ltot,D] float64, mask [H,Ltot] bool -> [H,Lq,D] float64."""
    logits = np.einsum("hid,hjd->hij", q, k_all) * scale
    logits = np.where(mask[:, None, :], logits, -np.inf)
    logits = logits - logits.max(axis=2, keepdims=True)
    w = np.exp(logits)
    w = w / w.sum(axis=2, keepdims=True)
    return np.einsum("hij,hjd->hid", w, v_all), w


def oracle_slots(max_T):
    """slots_of callable for ``synth.paper_default_policies``: the most frames the oracle's retention rule ever
    keeps for the head at history lengths 0 .. max_T, plus one slot per merged frame of a Veil head."""
    def slots_of(pol):
        big = pol._replace(slots=10 ** 6)
        need = max(len(OP.retained_frames(big, T, range(T))) for T in range(max_T + 1))
        return need + (pol.cap if pol.type == synth.VEIL and pol.cap > 0 else 0)
    return slots_of


def veil_merged(sink, recent, n_merged, window, slots=None, n_new=3):
    """Veil head with cache merging whose pool region holds sink + recent + the window sources + the frames of one
    append, plus one slot per merged frame at the end of the region."""
    need = sink + recent + n_merged * window + n_new + n_merged
    return synth.veil_merged(sink, recent, n_merged, window, slots if slots is not None else need)
