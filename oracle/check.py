"""Comparison helpers around the oracle: assemble a head's key sequence from the pool oracle, evaluate the attention
oracle on it, and compare a candidate output with the result.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``): used by the GPU parity tests, the smoke check and the
benchmark's ``cpu_baseline`` leg.  Nothing of the method is computed here beyond calling ``oracle.attention`` and
``oracle.pool``; the candidate output is only ever an argument.
"""
import numpy as np

from . import attention as OA

MAX_ABS_TOL = 2e-2     # contract: bf16 inputs, fp32 accumulation, against the fp32 oracle
REL_L2_TOL = 1e-2      # self-imposed: the outputs are only O(1e-2..1), max-abs alone is too weak


def oracle_attention(pool_o, sel_count, sel_frames, q, k_cur, v_cur, rows=None, scale=None, heads=None):
    """q, k_cur, v_cur: CPU bf16 torch tensors [H, Lq, D]; pool_o: ``PoolOracle``; sel_* as ``build_index`` returns
    them.  Returns {head: float32 [n_rows, D]} (Eq. 1 over [selected frames || chunk] of every head)."""
    out = {}
    for h in (range(q.shape[0]) if heads is None else heads):
        Kb, Vb = pool_o.head_kv(h, sel_frames[h, :sel_count[h]].tolist())
        Kh = np.concatenate([OA.widen_bf16(Kb), k_cur[h].float().numpy()], 0)
        Vh = np.concatenate([OA.widen_bf16(Vb), v_cur[h].float().numpy()], 0)
        out[h] = OA.attn_head(q[h].float().numpy(), Kh, Vh, rows=rows, scale=scale)
    return out


def compare_attention(got_all, want, rows=None, label=""):
    """got_all: float32 array [H, Lq, D] (the candidate); want: {head: float32 [n_rows, D]}.  Asserts the
    tolerances, returns (worst max-abs error, worst relative L2 error)."""
    worst_abs, worst_rel = 0.0, 0.0
    for h, ref in want.items():
        got = got_all[h] if rows is None else got_all[h][rows]
        assert np.isfinite(got).all(), "%s head %d: non-finite output" % (label, h)
        err = np.abs(got - ref).max()
        rel = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30)
        worst_abs, worst_rel = max(worst_abs, err), max(worst_rel, rel)
        assert err <= MAX_ABS_TOL, "%s head %d: max-abs error %.3e" % (label, h, err)
        assert rel <= REL_L2_TOL, "%s head %d: relative L2 error %.3e" % (label, h, rel)
    return worst_abs, worst_rel


def sample_rows(Lq, n, seed, extra=()):
    """Seeded query rows incl. the first, the last and rows next to the 128/256-row tile boundaries."""
    fixed = {0, Lq - 1} | {r for r in (127, 128, 255, 256, Lq - 2) if 0 <= r < Lq} | {r for r in extra if 0 <= r < Lq}
    rng = np.random.default_rng(seed)
    while len(fixed) < min(n, Lq):
        fixed.add(int(rng.integers(0, Lq)))
    return np.array(sorted(fixed), np.int32)
