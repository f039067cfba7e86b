"""Shared helpers for the tests: fixture parsing, and an independent dense-mask attention."""
import os

import numpy as np

from paper_2605_13111_amd import synth

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
