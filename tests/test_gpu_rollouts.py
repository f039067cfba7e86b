"""GPU parity along rollouts at model shape: the named workloads driven chunk by chunk through the C ABI, with
the pool and the index compared bit for bit with the oracle on the way and the attention output compared on
sampled query rows at several history lengths.  Inputs are drawn on the GPU from a seeded generator and copied
to the host for the oracle (one generator serves both sides)."""
import numpy as np
import pytest
import torch

from oracle.pool import PoolOracle
from paper_2605_13111_amd import binding as B
from paper_2605_13111_amd import synth
import gpu_common as G
import helpers

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _rollout(pols, tpf, D, n_new, n_chunks, seed, check_at, attn_at, rows_n, label, with_scores=True, append_last=True):
    """Chunk c (history length T = c * n_new): when T is in attn_at, build the index, compare it, run one attention
    pass of the chunk (q, k_cur, v_cur drawn for this chunk) and compare sampled rows; then write the chunk's
    k_cur / v_cur back as frames T .. T+n_new-1 (Sec. 2.2) on both sides.  After the append of every chunk whose
    new history length is in check_at the pool tables and payload are compared."""
    H, Lq = len(pols), n_new * tpf
    pool_o = PoolOracle(pols, tpf, D)
    pool_g = B.Pool(pols, tpf, D, device=DEV)
    B.pf_pool_reset(pool_g)
    index = B.Index(pool_g, Lq)
    ws = torch.empty(B.pf_attn_workspace_bytes(pool_g, Lq), dtype=torch.uint8, device=DEV)
    worst = (0.0, 0.0)
    for c in range(n_chunks):
        T = c * n_new
        k_cur = synth.randn_bf16((H, Lq, D), seed * 100000 + 3 * c, device=DEV)
        v_cur = synth.randn_bf16((H, Lq, D), seed * 100000 + 3 * c + 1, device=DEV)
        sc = synth.frame_scores(H, n_new, seed * 100000 + 3 * c + 2) if with_scores else None
        if T in attn_at:
            q = synth.randn_bf16((H, Lq, D), seed * 100000 + 90000 + c, device=DEV)
            B.pf_build_index(pool_g, index, Lq)
            sel_count, sel_frames = G.check_index(index, pool_o)
            assert B.pf_index_status(index) == 0
            out = torch.full((H, Lq, D), float("nan"), dtype=torch.bfloat16, device=DEV)
            B.pf_ragged_attn_fwd(pool_g, index, q, k_cur, v_cur, out, ws)
            torch.cuda.synchronize()
            rows = G.sample_rows(Lq, rows_n, seed + c, extra=(1559, 1560, 1535, 1536, 3119, 3120))
            want = G.oracle_attention(pool_o, sel_count, sel_frames, q.cpu(), k_cur.cpu(), v_cur.cpu(), rows=rows)
            a, r = G.compare_attention(out, want, rows=rows, label="%s T=%d" % (label, T))
            worst = (max(worst[0], a), max(worst[1], r))
        if c == n_chunks - 1 and not append_last:
            break
        # write-back: the chunk's keys and values become frames T .. T+n_new-1
        k_new, v_new = k_cur.view(H, n_new, tpf, D), v_cur.view(H, n_new, tpf, D)
        pool_o.append(synth.bits(k_new), synth.bits(v_new), None if sc is None else sc.numpy())
        B.pf_cache_append(pool_g, k_new, v_new, None if sc is None else sc.to(DEV))
        if T + n_new in check_at:
            G.check_pool(pool_g, pool_o)
            B.pf_build_index(pool_g, index, Lq)
            G.check_index(index, pool_o)
    print("%s: attention at T in %s: max-abs %.2e rel %.2e" % (label, sorted(attn_at), worst[0], worst[1]))
    return pool_g, pool_o


@pytest.mark.parametrize("layer", [0, 17])
def test_c5_streaming_rollout_attention_pool_index(layer):
    """The streaming workload: a layer's drawn policies (top-18 Anchor / Wave period 2-4 / Veil 1+3), one-frame
    chunks of 1560 tokens (six full 256-row query tiles and one with 24 rows), history 0 .. 39.  Attention against
    the oracle at T = 0, 1, 2, 7, 20, 39; pool and index bit-exact there and after every 8th append."""
    w = synth.WORKLOADS["c5_stream"]
    pols = synth.policies("c5_stream", layer=layer)
    attn_at = {0, 1, 2, 7, 20, 39}
    check_at = attn_at | set(range(8, 41, 8))
    _rollout(pols, w.tokens_per_frame, w.head_dim, 1, 40, 500 + layer, check_at, attn_at, 40, "c5_stream layer %d" % layer)


@pytest.mark.parametrize("group", [0, 1, 2])
def test_c3_step_every_layer_sampled_rows(group):
    """The 30-layer step: EVERY layer's drawn policies (each has its own per-head segment plan) filled to 57 frames;
    pool and index in full, attention on 16 sampled rows per head, in the launch configuration the bench times."""
    w = synth.WORKLOADS["c3_step"]
    for layer in range(group * 10, group * 10 + 10):
        pols = synth.policies("c3_step", layer=layer)
        T = w.history_frames
        _rollout(pols, w.tokens_per_frame, w.head_dim, 3, T // 3 + 1, 600 + layer, {T}, {T}, 16, "c3_step layer %d" % layer,
                 append_last=False)


@pytest.mark.parametrize("name", ["c6_paper", "c7_headwin"])
def test_paper_default_rollouts_to_240_frames(name):
    """The paper's own policy set (sink 3, recent 4, capacities 4/4/2: strided Anchor Eq. 4, capped Wave Eq. 5 with
    its sliding retention, Veil with merge window 2) and the head-window ablation (12 / 10 / 5), rolled out in
    three-frame chunks to 240 history frames: pool and index bit-exact after every 8th chunk, attention against
    the oracle at T = 120 and T = 237."""
    w = synth.WORKLOADS[name]
    pols = synth.policies(name, layer=1, slots_of=helpers.oracle_slots(w.history_frames))
    check_at = set(range(24, 241, 24)) | {3, 9}
    _rollout(pols, w.tokens_per_frame, w.head_dim, 3, 80, 700 + len(name), check_at, {120, 237}, 32, name)


def test_c3_step_layers_with_the_64_row_kernel():
    """Two layers of the 30-layer step (their own per-head segment plans) through kernel variant 2 (4 waves x 64 query
    rows): pool and index in full, attention on 16 sampled rows per head."""
    w = synth.WORKLOADS["c3_step"]
    B.pf_set_tuning(attn_variant=2)
    try:
        for layer in (5, 22):
            pols = synth.policies("c3_step", layer=layer)
            T = w.history_frames
            _rollout(pols, w.tokens_per_frame, w.head_dim, 3, T // 3 + 1, 800 + layer, {T}, {T}, 16,
                     "c3_step layer %d, 64-row kernel" % layer, append_last=False)
    finally:
        B.pf_set_tuning(attn_variant=1)
