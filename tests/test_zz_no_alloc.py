"""The entry point that allocates nothing and takes no workspace: pf_ragged_attn_fwd_static against
pf_ragged_attn_fwd on the same pool, index and inputs -- equal bit for bit (the same kernels, another scratch
address) and within the oracle's tolerance -- on two calls in a row, the second with a smaller input."""
import pytest
import torch

from oracle.pool import PoolOracle
from paper_2605_13111_amd import binding as B
from paper_2605_13111_amd import synth
import gpu_common as G

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _case(pols, tpf, D, chunks, Lq, seed, seg_tiles, rows_n):
    H = len(pols)
    pool_o = PoolOracle(pols, tpf, D)
    pool = B.Pool(pols, tpf, D, device=DEV)
    B.pf_pool_reset(pool)
    for ci, n_new in enumerate(chunks):
        k = synth.randn_bf16((H, n_new, tpf, D), seed * 1000 + 2 * ci, device=DEV)
        v = synth.randn_bf16((H, n_new, tpf, D), seed * 1000 + 2 * ci + 1, device=DEV)
        sc = synth.frame_scores(H, n_new, seed * 1000 + 500 + ci)
        pool_o.append(synth.bits(k), synth.bits(v), sc.numpy())
        B.pf_cache_append(pool, k, v, sc.to(DEV))
    index = B.Index(pool, Lq, seg_tiles=seg_tiles)
    B.pf_build_index(pool, index, Lq)
    sel_count, sel_frames = G.check_index(index, pool_o)
    assert index.c.n_partials > 0, "the case must use the scratch buffer"
    q, kc, vc = [synth.randn_bf16((H, Lq, D), seed * 1000 + 900 + i, device=DEV) for i in range(3)]
    ws = torch.empty(B.pf_attn_workspace_bytes(pool, Lq) if seg_tiles == 0 else (1 << 28), dtype=torch.uint8, device=DEV)
    want_bits = torch.full((H, Lq, D), float("nan"), dtype=torch.bfloat16, device=DEV)
    B.pf_ragged_attn_fwd(pool, index, q, kc, vc, want_bits, ws)
    got = torch.full((H, Lq, D), float("nan"), dtype=torch.bfloat16, device=DEV)
    before = torch.cuda.memory_allocated()
    B.pf_ragged_attn_fwd_static(pool, index, q, kc, vc, got)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(got.view(torch.int16), want_bits.view(torch.int16))
    rows = None if rows_n is None else G.sample_rows(Lq, rows_n, seed)
    want = G.oracle_attention(pool_o, sel_count, sel_frames, q.cpu(), kc.cpu(), vc.cpu(), rows=rows)
    return G.compare_attention(got, want, rows=rows, label="static scratch")


def test_static_scratch_entry_point_matches_the_workspace_entry_point():
    # first call: a layer of the 30-layer step in its planned launch configuration (about 100 MB of partial results)
    w = synth.WORKLOADS["c3_step"]
    a, r = _case(synth.policies("c3_step", layer=2), w.tokens_per_frame, w.head_dim, [3] * 19, 4680, seed=81, seg_tiles=0,
                 rows_n=16)
    # second call, smaller: mixed policies, short frames, short forced segments -- the array still holds the first call's partials
    pols = [synth.anchor_all(30), synth.anchor_topk(5, 5), synth.wave(2, 30), synth.veil(1, 3)]
    a2, r2 = _case(pols, 48, 128, [3] * 10, 200, seed=82, seg_tiles=16, rows_n=None)
    print("static scratch: max-abs %.2e / %.2e, relative L2 %.2e / %.2e" % (a, a2, r, r2))
