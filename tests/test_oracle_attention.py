"""Pins of the attention oracle (oracle/attention.c + attention.py): brute-force dense masked attention,
a library routine on the keep-everything case, closed forms and invariances."""
import math

import numpy as np
import pytest
import torch

from oracle import attention as A
from oracle import policy as P
from oracle.pool import PoolOracle
from paper_2605_13111_amd import synth
import helpers
from helpers import dense_masked_attention


def _tiny_case(seed=1, workload="c1_tiny", T=None):
    """History appended chunk by chunk into the pool oracle, then one query chunk."""
    w = synth.WORKLOADS[workload]
    T = w.history_frames if T is None else T
    pols = synth.policies(workload)
    H, D, tpf = w.n_heads, w.head_dim, w.tokens_per_frame
    Lq = w.chunk_frames * tpf
    k_hist = synth.randn_bf16((H, T, tpf, D), seed)
    v_hist = synth.randn_bf16((H, T, tpf, D), seed + 1)
    q = synth.randn_bf16((H, Lq, D), seed + 2)
    k_cur = synth.randn_bf16((H, Lq, D), seed + 3)
    v_cur = synth.randn_bf16((H, Lq, D), seed + 4)
    pool = PoolOracle(pols, tpf, D)
    for t0 in range(0, T, w.chunk_frames):
        t1 = min(T, t0 + w.chunk_frames)
        pool.append(synth.bits(k_hist[:, t0:t1]), synth.bits(v_hist[:, t0:t1]))
    return w, pols, pool, k_hist, v_hist, q, k_cur, v_cur


def _oracle_out(pool, pols, q, k_cur, v_cur, rows=None):
    hist = []
    for h, pol in enumerate(pols):
        sel = P.selected_frames(pol, pool.T, {f[0]: f[1] for f in pool.frames[h]})
        Kb, Vb = pool.head_kv(h, sel)
        hist.append((A.widen_bf16(Kb), A.widen_bf16(Vb)))
    return A.ragged_attention(q.float().numpy(), hist, k_cur.float().numpy(), v_cur.float().numpy(), rows=rows)


def test_against_dense_masked_brute_force():
    """Tiny configuration: 1 Anchor (all 12), 1 Wave (every 3rd), 2 Veil (frame 0 + last 2); the mask is
    written down frame by frame here, not taken from the oracle."""
    w, pols, pool, k_hist, v_hist, q, k_cur, v_cur = _tiny_case()
    H, D, tpf, T = w.n_heads, w.head_dim, w.tokens_per_frame, w.history_frames
    Lq = q.shape[1]
    out = _oracle_out(pool, pols, q, k_cur, v_cur)
    k_all = torch.cat([k_hist.reshape(H, T * tpf, D), k_cur], 1).double().numpy()
    v_all = torch.cat([v_hist.reshape(H, T * tpf, D), v_cur], 1).double().numpy()
    keep = {0: range(12), 1: (0, 3, 6, 9), 2: (0, 10, 11), 3: (0, 10, 11)}
    mask = np.zeros((H, T * tpf + Lq), bool)
    mask[:, T * tpf:] = True                                    # the chunk attends to itself
    for h, frames in keep.items():
        for f in frames:
            mask[h, f * tpf:(f + 1) * tpf] = True
    want, wts = dense_masked_attention(q.double().numpy(), k_all, v_all, mask, 1.0 / math.sqrt(D))
    assert [int(m.sum()) for m in mask] == [240, 112, 96, 96]   # per-head key counts of the tiny case
    assert np.abs(out - want).max() < 1e-6
    assert np.abs(wts.sum(2) - 1).max() < 1e-12


@pytest.mark.parametrize("D", [64, 128])
def test_keep_everything_is_plain_attention_over_history_plus_chunk(D):
    """All heads keep everything == standard attention of the chunk over [whole history || chunk]
    (no mask inside the chunk): checked against torch's scaled_dot_product_attention in float64."""
    H, tpf, T, Lq = 3, 5, 7, 11
    pols = [synth.anchor_all(T)] * H
    k_hist = synth.randn_bf16((H, T, tpf, D), 21)
    v_hist = synth.randn_bf16((H, T, tpf, D), 22)
    q, k_cur, v_cur = (synth.randn_bf16((H, Lq, D), s) for s in (23, 24, 25))
    pool = PoolOracle(pols, tpf, D)
    pool.append(synth.bits(k_hist), synth.bits(v_hist))
    out = _oracle_out(pool, pols, q, k_cur, v_cur)
    k_all = torch.cat([k_hist.reshape(H, T * tpf, D), k_cur], 1).double()
    v_all = torch.cat([v_hist.reshape(H, T * tpf, D), v_cur], 1).double()
    want = torch.nn.functional.scaled_dot_product_attention(q.double()[None], k_all[None], v_all[None])[0]
    assert np.abs(out - want.numpy()).max() < 1e-6


def test_rows_subset_matches_full():
    w, pols, pool, _, _, q, k_cur, v_cur = _tiny_case(seed=9)
    full = _oracle_out(pool, pols, q, k_cur, v_cur)
    rows = np.array([0, 5, 17, 47], np.int32)
    part = _oracle_out(pool, pols, q, k_cur, v_cur, rows=rows)
    assert np.array_equal(part, full[:, rows])


def test_softmax_weights_sum_to_one_and_ones_values_give_ones():
    rng = np.random.default_rng(2)
    q = rng.standard_normal((9, 16)).astype(np.float32) * 3
    K = rng.standard_normal((37, 16)).astype(np.float32) * 3
    out, wts = A.attn_head(q, K, np.ones((37, 16), np.float32), return_weights=True)
    assert np.abs(wts.sum(1) - 1).max() <= 1e-12 and (wts >= 0).all()
    assert np.abs(out - 1).max() <= 1e-6


def test_two_keys_closed_form():
    """D=2, one query, two keys: p_1 = 1/(1+exp(scale*(q.k2-q.k1)))."""
    q = np.array([[1.5, -0.5]], np.float32)
    K = np.array([[2.0, 1.0], [-1.0, 3.0]], np.float32)
    V = np.array([[10.0, 0.0], [0.0, -4.0]], np.float32)
    s1, s2 = (1.5 * 2 - 0.5 * 1), (-1.5 - 1.5)
    p1 = 1.0 / (1.0 + math.exp((s2 - s1) / math.sqrt(2)))
    out = A.attn_head(q, K, V)
    assert np.allclose(out, [[10 * p1, -4 * (1 - p1)]], atol=1e-6)
    # explicit scale argument
    out = A.attn_head(q, K, V, scale=0.25)
    p1 = 1.0 / (1.0 + math.exp((s2 - s1) * 0.25))
    assert np.allclose(out, [[10 * p1, -4 * (1 - p1)]], atol=1e-6)


def test_closed_forms():
    rng = np.random.default_rng(4)
    D, Lkv = 32, 50
    q = rng.standard_normal((6, D)).astype(np.float32)
    V = rng.standard_normal((Lkv, D)).astype(np.float32)
    # all keys equal -> uniform weights -> mean of the values
    K = np.tile(rng.standard_normal((1, D)).astype(np.float32), (Lkv, 1))
    assert np.abs(A.attn_head(q, K, V) - V.astype(np.float64).mean(0)).max() < 1e-6
    # one key only -> that value
    assert np.array_equal(A.attn_head(q, K[:1], V[:1]), np.tile(V[:1], (6, 1)))
    # zero queries, value of frame f constant c_f -> sum_f c_f * tokens_f / Lkv
    tpf, consts = 10, [3.0, -1.0, 7.0, 0.5, 2.0]
    Vf = np.concatenate([np.full((tpf, D), c, np.float32) for c in consts])
    out = A.attn_head(np.zeros((2, D), np.float32), rng.standard_normal((Lkv, D)).astype(np.float32), Vf)
    assert np.abs(out - sum(consts) / len(consts)).max() < 1e-6
    # one logit dominates -> the output is that key's value
    K = rng.standard_normal((Lkv, D)).astype(np.float32)
    qd = np.zeros((1, D), np.float32)
    qd[0] = K[17] * 40.0
    assert np.abs(A.attn_head(qd, K, V) - V[17]).max() < 1e-5


def test_duplicating_every_key_and_reordering_frames_change_nothing():
    """Softmax attention over a multiset: duplicating every key/value the same number of times, or
    permuting the frames, leaves the output unchanged (Eq. 2: the concatenation order is free)."""
    rng = np.random.default_rng(8)
    D, tpf, nf = 16, 6, 5
    q = rng.standard_normal((7, D)).astype(np.float32)
    K = rng.standard_normal((nf * tpf, D)).astype(np.float32)
    V = rng.standard_normal((nf * tpf, D)).astype(np.float32)
    base = A.attn_head(q, K, V)
    dup = A.attn_head(q, np.concatenate([K, K, K]), np.concatenate([V, V, V]))
    assert np.abs(dup - base).max() <= 1e-6
    perm = np.concatenate([np.arange(f * tpf, (f + 1) * tpf) for f in (3, 0, 4, 2, 1)])
    assert np.abs(A.attn_head(q, K[perm], V[perm]) - base).max() <= 1e-6
    # duplicating only a SUBSET is not invariant (guards against a vacuous test)
    sub = A.attn_head(q, np.concatenate([K, K[:tpf]]), np.concatenate([V, V[:tpf]]))
    assert np.abs(sub - base).max() > 1e-4


def test_float32_evaluation_agrees():
    """Self-check: a pure float32 numpy evaluation differs from the double-accumulating oracle by ~1e-6."""
    rng = np.random.default_rng(12)
    q, K, V = (rng.standard_normal(s).astype(np.float32) for s in ((8, 64), (300, 64), (300, 64)))
    s = (q @ K.T) * np.float32(1 / 8.0)
    p = np.exp(s - s.max(1, keepdims=True))
    want = (p / p.sum(1, keepdims=True)) @ V
    assert np.abs(A.attn_head(q, K, V) - want).max() < 2e-5


def test_widen_bf16_is_exact():
    x = synth.randn_bf16((1000,), 3)
    assert np.array_equal(A.widen_bf16(synth.bits(x)), x.float().numpy())


@pytest.mark.parametrize("m,tpf", [(2, 6), (3, 7)])
def test_veil_cache_merging_equals_a_token_level_mask(m, tpf):
    """A merged frame is a concatenation of token subsets of raw frames, and softmax attention does not depend on
    the order of its keys: attending to [sink | merged windows | recent | chunk] must equal dense attention over
    EVERY raw token with the mask 'token tok of frame w0+i is visible iff tok mod m == i' written down here."""
    H, D, T, Lq = 2, 64, 17, 5
    S, R, cap = 2, 3, 2
    pols = [helpers.veil_merged(S, R, cap, m), helpers.veil_merged(1, 0, 1, m)]
    k_hist = synth.randn_bf16((H, T, tpf, D), 71)
    v_hist = synth.randn_bf16((H, T, tpf, D), 72)
    q = synth.randn_bf16((H, Lq, D), 73)
    k_cur = synth.randn_bf16((H, Lq, D), 74)
    v_cur = synth.randn_bf16((H, Lq, D), 75)
    pool = PoolOracle(pols, tpf, D)
    for t in range(T):
        pool.append(synth.bits(k_hist[:, t:t + 1]), synth.bits(v_hist[:, t:t + 1]))
    out = _oracle_out(pool, pols, q, k_cur, v_cur)
    k_all = torch.cat([k_hist.reshape(H, T * tpf, D), k_cur], 1).double().numpy()
    v_all = torch.cat([v_hist.reshape(H, T * tpf, D), v_cur], 1).double().numpy()
    mask = np.zeros((H, T * tpf + Lq), bool)
    mask[:, T * tpf:] = True
    for h, (s_, r_, c_) in enumerate([(S, R, cap), (1, 0, 1)]):
        for f in list(range(s_)) + list(range(T - r_, T)):
            mask[h, f * tpf:(f + 1) * tpf] = True
        for j in range(c_):
            w0 = T - r_ - (j + 1) * m
            assert w0 >= s_
            for i in range(m):
                for tok in range(tpf):
                    if tok % m == i:
                        mask[h, (w0 + i) * tpf + tok] = True
    want, _ = dense_masked_attention(q.double().numpy(), k_all, v_all, mask, 1.0 / math.sqrt(D))
    assert [int(x.sum()) for x in mask] == [(S + R + cap) * tpf + Lq, (1 + 1) * tpf + Lq]
    assert np.abs(out - want).max() < 1e-6
