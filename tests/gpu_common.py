"""Driver shared by the GPU parity tests: runs one seeded case through the oracle and through libpf.so."""
import numpy as np
import torch

from oracle import check as OC
from oracle.check import MAX_ABS_TOL, REL_L2_TOL, oracle_attention, sample_rows
from oracle.pool import PoolOracle
from paper_2605_13111_amd import binding as B
from paper_2605_13111_amd import synth



def check_pool(pool_g, pool_o):
    """Bit-exact: T, resident counts, frame ids, scores, and the K/V payload of every resident slot."""
    torch.cuda.synchronize()
    n_frames, frame_ids, frame_score = pool_o.tables()
    assert int(pool_g.T_dev.item()) == pool_o.T == pool_g.T
    assert np.array_equal(pool_g.n_frames.cpu().numpy(), n_frames)
    assert np.array_equal(pool_g.frame_ids.cpu().numpy(), frame_ids)
    assert np.array_equal(pool_g.frame_score.cpu().numpy().view(np.uint32), frame_score.view(np.uint32))
    assert (pool_g.sync.cpu().numpy() == 0).all()
    res = list(pool_o.resident_kv())
    if not res:
        return
    slots = torch.tensor([r[0] for r in res], dtype=torch.long, device=pool_g.device)
    kg = synth.bits(pool_g.k_pool[slots])
    vg = synth.bits(pool_g.v_pool[slots])
    for i, (_, K, V) in enumerate(res):
        assert np.array_equal(kg[i], K), "K payload of slot %d" % res[i][0]
        assert np.array_equal(vg[i], V), "V payload of slot %d" % res[i][0]


def check_index(index_g, pool_o):
    torch.cuda.synchronize()
    sel_count, sel_frames, sel_slots, cu = pool_o.build_index(index_g.max_sel)
    assert np.array_equal(index_g.sel_count.cpu().numpy(), sel_count)
    assert np.array_equal(index_g.sel_frames.cpu().numpy(), sel_frames)
    assert np.array_equal(index_g.sel_slots.cpu().numpy(), sel_slots)
    assert np.array_equal(index_g.cu_seqlens.cpu().numpy(), cu)
    header = index_g.work[:64].cpu().numpy().view(np.int32)
    assert header[4] == 0, "index kernel reported a plan mismatch"
    assert header[0] == index_g.c.n_blocks and header[3] == index_g.c.n_partials
    return sel_count, sel_frames


def compare_attention(out_g, want, rows=None, label=""):
    """out_g: GPU bf16 [H, Lq, D]; want: {head: float32 [n_rows, D]}.  The whole output must be finite (a query
    row the kernel never wrote would still hold the NaN it was pre-filled with)."""
    got_all = out_g.float().cpu().numpy()
    assert np.isfinite(got_all).all(), "%s: non-finite values in the output" % label
    return OC.compare_attention(got_all, want, rows=rows, label=label)


def run_case(pols, tpf, D, chunks, Lq, seed, with_scores=True, q_gain=1.0, seg_tiles=0, rows=None,
             check_every_append=True, scale=0.0, device="cuda:0", label="case", layout="packed"):
    """Full path on both sides.  Returns (worst max-abs, worst relative L2) of the attention output.
    layout="model": the GPU side holds the new frames and the chunk tensors as [tokens][heads][D] and goes
    through the strided entry points (same values, so the oracle side does not change)."""
    model = layout == "model"

    def as_model(t):              # [H, ..., D] on the CPU -> heads-first view of a [tokens][H][D] device tensor
        flat = t.reshape(t.shape[0], -1, t.shape[-1]).to(device)
        return flat.permute(1, 0, 2).contiguous().permute(1, 0, 2).reshape(t.shape) if t.dim() == 3 else \
            flat.permute(1, 0, 2).contiguous().permute(1, 0, 2).unflatten(1, tuple(t.shape[1:-1]))

    H = len(pols)
    pool_o = PoolOracle(pols, tpf, D)
    pool_g = B.Pool(pols, tpf, D, device=device)
    B.pf_pool_reset(pool_g)
    T = 0
    for ci, n_new in enumerate(chunks):
        k_new = synth.randn_bf16((H, n_new, tpf, D), seed * 1000 + 2 * ci)
        v_new = synth.randn_bf16((H, n_new, tpf, D), seed * 1000 + 2 * ci + 1)
        sc = synth.frame_scores(H, n_new, seed * 1000 + 500 + ci) if with_scores else None
        pool_o.append(synth.bits(k_new), synth.bits(v_new), None if sc is None else sc.numpy())
        if model:
            B.pf_cache_append_strided(pool_g, as_model(k_new), as_model(v_new), None if sc is None else sc.to(device))
        else:
            B.pf_cache_append(pool_g, k_new.to(device), v_new.to(device), None if sc is None else sc.to(device))
        T += n_new
        if check_every_append or ci == len(chunks) - 1:
            check_pool(pool_g, pool_o)
    if not chunks:
        check_pool(pool_g, pool_o)
    index = B.Index(pool_g, Lq, seg_tiles=seg_tiles)
    B.pf_build_index(pool_g, index, Lq)
    sel_count, sel_frames = check_index(index, pool_o)
    q = synth.randn_bf16((H, Lq, D), seed * 1000 + 900) * q_gain
    k_cur = synth.randn_bf16((H, Lq, D), seed * 1000 + 901)
    v_cur = synth.randn_bf16((H, Lq, D), seed * 1000 + 902)
    out = torch.full((H, Lq, D), float("nan"), dtype=torch.bfloat16, device=device)
    attn = B.pf_ragged_attn_fwd
    qg, kg, vg = q.to(device), k_cur.to(device), v_cur.to(device)
    if model:
        attn = B.pf_ragged_attn_fwd_strided
        qg, kg, vg, out = as_model(q), as_model(k_cur), as_model(v_cur), as_model(out.cpu())
    ws = torch.empty(B.pf_attn_workspace_bytes(pool_g, Lq) if seg_tiles == 0 else (1 << 28), dtype=torch.uint8,
                     device=device)
    attn(pool_g, index, qg, kg, vg, out, ws, softmax_scale=scale)
    torch.cuda.synchronize()
    want = oracle_attention(pool_o, sel_count, sel_frames, q, k_cur, v_cur, rows=rows,
                            scale=None if scale == 0.0 else scale)
    res = compare_attention(out, want, rows=rows, label=label)
    # a second launch on the same index must give the same bits (arrival counters reset themselves)
    out2 = torch.full_like(out, float("nan"))           # keeps the strides
    attn(pool_g, index, qg, kg, vg, out2, ws, softmax_scale=scale)
    torch.cuda.synchronize()
    assert torch.equal(out.contiguous().view(torch.int16), out2.contiguous().view(torch.int16)), "%s: second launch differs" % label
    return res
