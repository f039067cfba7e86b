"""CPU-only tests of libpf.so: exported symbols, closed-form counts against the oracle, and argument
validation (all rejected before any device access, so fake device pointers are enough)."""
import ctypes
import os
import re

import pytest

from oracle import policy as P
from paper_2605_13111_amd import binding as B
from paper_2605_13111_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

pytestmark = pytest.mark.skipif(not os.path.exists(B.LIB_PATH), reason="libpf.so not built")


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "pf.h")).read()
    declared = set(re.findall(r"\b(pf_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    lib = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def _policies():
    out = []
    for S in (0, 1, 3):
        for R in (0, 2, 4):
            out.append(synth.HeadPolicy(synth.ANCHOR, synth.MODE_ALL, S, R, 0, 1, 100))
            out.append(synth.HeadPolicy(synth.VEIL, 0, S, R, 0, 1, 100))
            for cap in (0, 2, 4, 18):
                out.append(synth.HeadPolicy(synth.ANCHOR, synth.MODE_STRIDED, S, R, cap, 1, 100))
                out.append(synth.HeadPolicy(synth.ANCHOR, synth.MODE_TOPK, S, R, cap, 1, 100))
                for period in (1, 2, 3, 6):
                    out.append(synth.HeadPolicy(synth.WAVE, 0, S, R, cap, period, 100))
            for cap in (1, 2, 3):                      # Veil with cache merging: cap merged frames, window m
                for m in (1, 2, 3, 5):
                    out.append(synth.HeadPolicy(synth.VEIL, 0, S, R, cap, m, 100))
    return out


def test_closed_form_counts_match_the_oracle():
    """The host sizes launches and checks capacity from closed-form counts; they must equal the length of
    the oracle's frame lists for every policy and history length."""
    score = {f: float((f * 7919) % 97) for f in range(100)}
    for pol in _policies():
        for T in range(0, 90):
            sc = {f: score[f] for f in range(T)}
            assert B.pf_selected_count(pol, T) == len(P.selected_frames(pol, T, sc)), (pol, T)
            assert B.pf_retained_count(pol, T) == len(P.retained_frames(pol, T, list(range(T)), sc)), (pol, T)


def test_count_helpers_reject_bad_policies():
    bad = synth.HeadPolicy(7, 0, 0, 0, 0, 1, 4)
    assert B.pf_selected_count(bad, 3) == B.PF_ERR_INVALID_ARG
    assert B.pf_retained_count(synth.HeadPolicy(synth.WAVE, 0, 0, 0, 0, 0, 4), 3) == B.PF_ERR_INVALID_ARG
    assert B.pf_selected_count(synth.anchor_all(4), -1) == B.PF_ERR_INVALID_ARG
    # cache merging needs a window size and room for the merged frames next to the raw ones
    assert B.pf_selected_count(synth.HeadPolicy(synth.VEIL, 0, 1, 2, 2, 0, 16), 9) == B.PF_ERR_INVALID_ARG
    assert B.pf_selected_count(synth.HeadPolicy(synth.VEIL, 0, 1, 2, 2, 2, 2), 9) == B.PF_ERR_INVALID_ARG


def _fake_pool(policies, tpf=16, D=64):
    """A pf_pool whose device pointers are fake but non-null and aligned: good enough for every check
    that happens before a kernel launch."""
    H = len(policies)
    host = (B.pf_head_policy * H)(*[B.make_policy(p) for p in policies])
    total = sum(p.slots for p in policies)
    fake = 0x1000
    pool = B.pf_pool(H, D, tpf, 0, total, fake, fake, ctypes.cast(host, ctypes.POINTER(B.pf_head_policy)), fake,
                     fake, fake, fake, fake, fake, fake, 0, 0)
    pool._keep = host
    return pool


def test_argument_validation_without_a_device():
    lib = B.lib()
    pols = [synth.anchor_all(4), synth.veil(1, 2)]
    pool = _fake_pool(pols)
    fake = ctypes.c_void_p(0x1000)
    null = ctypes.c_void_p(0)
    # sizes
    assert lib.pf_index_work_bytes(ctypes.byref(pool), 48) > 0
    assert lib.pf_attn_workspace_bytes(ctypes.byref(pool), 48) > 0
    assert lib.pf_index_work_bytes(ctypes.byref(pool), 0) == 0
    assert lib.pf_index_work_bytes(None, 48) == 0
    # append: bad arguments
    assert lib.pf_cache_append(None, fake, fake, 1, null, null) == B.PF_ERR_INVALID_ARG
    assert lib.pf_cache_append(ctypes.byref(pool), null, fake, 1, null, null) == B.PF_ERR_INVALID_ARG
    assert lib.pf_cache_append(ctypes.byref(pool), fake, fake, 0, null, null) == B.PF_ERR_INVALID_ARG
    assert lib.pf_cache_append(ctypes.byref(pool), ctypes.c_void_p(0x1004), fake, 1, null, null) == B.PF_ERR_INVALID_ARG
    # append: Anchor/ALL has 4 slots, 5 frames do not fit -> capacity error, host mirror untouched
    assert lib.pf_cache_append(ctypes.byref(pool), fake, fake, 5, null, null) == B.PF_ERR_CAPACITY
    assert pool.T_host == 0
    # unsupported head_dim / dtype, inconsistent total_slots, bad policy
    p2 = _fake_pool(pols, D=96)
    assert lib.pf_cache_append(ctypes.byref(p2), fake, fake, 1, null, null) == B.PF_ERR_UNSUPPORTED
    p3 = _fake_pool(pols)
    p3.total_slots = 99
    assert lib.pf_pool_reset(ctypes.byref(p3), null) == B.PF_ERR_INVALID_ARG
    p4 = _fake_pool([synth.HeadPolicy(synth.WAVE, 0, 0, 0, 0, 0, 4)])
    assert lib.pf_pool_reset(ctypes.byref(p4), null) == B.PF_ERR_INVALID_ARG
    # index: null struct, max_sel too small for what the policies select at T = 4
    assert lib.pf_build_index(ctypes.byref(pool), None, 48, null) == B.PF_ERR_INVALID_ARG
    pool.T_host = 4
    idx = B.pf_index(2, 0, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 1 << 20, 0, 0, 0, 0, 0, 0)
    assert lib.pf_build_index(ctypes.byref(pool), ctypes.byref(idx), 48, null) == B.PF_ERR_CAPACITY
    idx = B.pf_index(8, 0, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 64, 0, 0, 0, 0, 0, 0)   # work buffer too small
    assert lib.pf_build_index(ctypes.byref(pool), ctypes.byref(idx), 48, null) == B.PF_ERR_CAPACITY
    # attention: stale index (built for another T / q_tokens) and null tensors
    idx = B.pf_index(8, 0, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 1 << 20, 48, 3, 8, 0, 0, 0)
    assert lib.pf_ragged_attn_fwd(ctypes.byref(pool), ctypes.byref(idx), fake, fake, fake, fake, 48, 0.0, null, 0,
                                  null) == B.PF_ERR_INVALID_ARG
    idx.T_built = 4
    assert lib.pf_ragged_attn_fwd(ctypes.byref(pool), ctypes.byref(idx), null, fake, fake, fake, 48, 0.0, null, 0,
                                  null) == B.PF_ERR_INVALID_ARG
    assert lib.pf_ragged_attn_fwd(ctypes.byref(pool), ctypes.byref(idx), fake, fake, fake, fake, 32, 0.0, null, 0,
                                  null) == B.PF_ERR_INVALID_ARG
    assert B.lib().pf_status_string(B.PF_ERR_CAPACITY) == b"capacity exceeded"


def test_static_scratch_entry_point_rejects_plans_that_do_not_fit():
    """pf_ragged_attn_fwd_static keeps partial results in a fixed 160 MiB array: a plan that needs more is refused
    on the host with a capacity error, before anything touches a device."""
    lib = B.lib()
    pool = _fake_pool([synth.anchor_all(4), synth.veil(1, 2)], tpf=1560, D=128)
    fake, null = ctypes.c_void_p(0x1000), ctypes.c_void_p(0)
    slot = 256 * (128 + 2) * 4
    too_many = (160 << 20) // slot + 1
    idx = B.pf_index(8, 0, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 1 << 20, 48, 0, 8, too_many, 1, 0)
    assert lib.pf_ragged_attn_fwd_static(ctypes.byref(pool), ctypes.byref(idx), fake, fake, fake, fake, 48, 0.0,
                                         null) == B.PF_ERR_CAPACITY
    assert lib.pf_ragged_attn_fwd_static(None, ctypes.byref(idx), fake, fake, fake, fake, 48, 0.0, null) == B.PF_ERR_INVALID_ARG
    idx.n_partials = -1
    assert lib.pf_ragged_attn_fwd_static(ctypes.byref(pool), ctypes.byref(idx), fake, fake, fake, fake, 48, 0.0,
                                         null) == B.PF_ERR_INVALID_ARG


def test_chunk_layout_validation_without_a_device():
    """Strided entry points: stride checks happen on the host, before any device access."""
    lib = B.lib()
    pols = [synth.anchor_all(4), synth.veil(1, 2)]
    pool = _fake_pool(pols)                                   # head_dim 64, 16 tokens per frame
    fake, null = ctypes.c_void_p(0x1000), ctypes.c_void_p(0)
    idx = B.pf_index(8, 0, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 1 << 20, 48, 0, 8, 0, 0, 0)
    lay = lambda ts, hs: ctypes.byref(B.pf_chunk_layout(ts, hs))
    bad = [(0, 64), (60, 64 * 48), (64, 60), (32, 64 * 48), (128, 100), (128, 64 * 8)]   # short, unaligned, overlapping rows
    for ts, hs in bad:
        assert lib.pf_ragged_attn_fwd_strided(ctypes.byref(pool), ctypes.byref(idx), fake, fake, fake, fake, 48, 0.0, null, 0,
                                              lay(ts, hs), null) == B.PF_ERR_INVALID_ARG, (ts, hs)
        assert lib.pf_cache_append_strided(ctypes.byref(pool), fake, fake, 3, null, lay(ts, hs), null) == B.PF_ERR_INVALID_ARG
    assert lib.pf_ragged_attn_fwd_strided(ctypes.byref(pool), ctypes.byref(idx), fake, fake, fake, fake, 48, 0.0, null, 0,
                                          None, null) == B.PF_ERR_INVALID_ARG
    assert lib.pf_cache_append_strided(ctypes.byref(pool), fake, fake, 3, null, None, null) == B.PF_ERR_INVALID_ARG
    # a good layout passes the stride check and fails later, on capacity (5 frames into 4 slots): nothing was launched
    assert lib.pf_cache_append_strided(ctypes.byref(pool), fake, fake, 5, null, lay(2 * 64, 64), null) == B.PF_ERR_CAPACITY
    assert pool.T_host == 0


def test_classify_argument_validation_without_a_device():
    lib = B.lib()
    fake, null = ctypes.c_void_p(0x1000), ctypes.c_void_p(0)
    call = lambda lg, n_p, n_h, n_t, al, be, ht, pt: lib.pf_classify_heads(lg, n_p, n_h, n_t, al, be, ht, pt, null, null)
    assert call(null, 2, 3, 10, 0.8, 6.4, fake, fake) == B.PF_ERR_INVALID_ARG
    assert call(fake, 2, 3, 10, 0.8, 6.4, null, fake) == B.PF_ERR_INVALID_ARG
    assert call(fake, 2, 3, 10, 0.8, 6.4, fake, null) == B.PF_ERR_INVALID_ARG
    assert call(fake, 0, 3, 10, 0.8, 6.4, fake, fake) == B.PF_ERR_INVALID_ARG
    assert call(fake, 2, 3, 0, 0.8, 6.4, fake, fake) == B.PF_ERR_INVALID_ARG
    assert call(fake, 2, 3, 10, 0.0, 6.4, fake, fake) == B.PF_ERR_INVALID_ARG
    assert call(fake, 2, 3, 10, 1.5, 6.4, fake, fake) == B.PF_ERR_INVALID_ARG
    assert call(fake, 2, 3, 10, 0.8, -1.0, fake, fake) == B.PF_ERR_INVALID_ARG
    assert call(fake, 2, 3, 2000, 0.8, 6.4, fake, fake) == B.PF_ERR_UNSUPPORTED


def _tiles(pol, T, tpf, q_tokens):
    return -(-(B.pf_selected_count(pol, T) * tpf + q_tokens) // 64)


def test_launch_plan_stays_inside_the_advertised_buffers():
    """pf_plan_segments (host only) returns the plan pf_build_index would launch.  For the bench workload's drawn
    policies at several history lengths, in both launch forms and with the per-head step switched off: every split
    head's segments are at least 48 tiles long, the block and partial counts follow from the segment lengths, and
    they fit what pf_index_work_bytes / pf_attn_workspace_bytes promise for any history length."""
    w = synth.WORKLOADS["c3_step"]
    tpf, D, Lq = w.tokens_per_frame, w.head_dim, w.chunk_frames * w.tokens_per_frame
    n_qt = -(-Lq // 256)
    for layer in (0, 7, 13):
        pols = synth.policies("c3_step", layer=layer)
        pool = _fake_pool(pols, tpf=tpf, D=D)
        work_bytes = B.lib().pf_index_work_bytes(ctypes.byref(pool), Lq)
        ws_bytes = B.lib().pf_attn_workspace_bytes(ctypes.byref(pool), Lq)
        for env in ({}, {"attn_queue": 0}, {"plan_uniform": 1}):
            B.pf_set_tuning(attn_variant=1, attn_queue=1, seg_tiles=0, plan_uniform=0)
            B.pf_set_tuning(**env)
            for T in (0, 3, 21, 57):
                seg, n_blocks, n_partials = B.pf_plan_segments(pool, T, Lq)
                assert B.pf_plan_segments(pool, T, Lq) == (seg, n_blocks, n_partials)       # remembered, same answer
                teams = parts = 0
                for pol, sg in zip(pols, seg):
                    n = _tiles(pol, T, tpf, Lq)
                    nseg = max(1, -(-n // sg))
                    assert sg >= 48 or nseg == 1, (layer, T, sg, n)
                    teams += nseg
                    parts += nseg * n_qt if nseg > 1 else 0
                assert n_blocks == -(-teams // 8) * 8 * n_qt and n_partials == parts
                assert n_partials * 256 * (D + 2) * 4 <= ws_bytes
                assert 64 + 4 * (len(pols) * n_qt + 16) + 16 * len(pols) + 32 * n_blocks <= work_bytes
                if env.get("plan_uniform"):
                    assert len(set(seg)) == 1
    B.pf_set_tuning(attn_variant=1, attn_queue=1, seg_tiles=0, plan_uniform=0)


def test_tuning_switches_validate_and_apply():
    assert B.lib().pf_set_tuning(7, -1, -1, -1) == B.PF_ERR_INVALID_ARG
    pool = _fake_pool(synth.policies("c3_step", layer=0), tpf=1560, D=128)
    B.pf_set_tuning(seg_tiles=64)
    seg, _, _ = B.pf_plan_segments(pool, 57, 4680)
    assert set(seg) == {64}
    B.pf_set_tuning(seg_tiles=0)
    seg, _, _ = B.pf_plan_segments(pool, 57, 4680)
    assert min(seg) >= 48


def test_planning_a_streaming_rollout_is_cheap_once_seen():
    """The one-frame-chunk rollout asks for 30 layers x 40 history lengths = 1200 different launch plans.  The
    library remembers all of them: a second rollout pays a table lookup per call (budget: 50 us mean, measured
    ~3 us), and a first-time plan stays in the low milliseconds."""
    import time
    w = synth.WORKLOADS["c5_stream"]
    pools = [_fake_pool(synth.policies("c5_stream", layer=l), tpf=w.tokens_per_frame, D=w.head_dim) for l in range(w.n_layers)]
    B.pf_set_tuning(attn_variant=1, attn_queue=1, seg_tiles=0, plan_uniform=0)

    def rollout():
        plans, worst = [], 0.0
        t0 = time.perf_counter()
        for T in range(w.history_frames):
            for pool in pools:
                t1 = time.perf_counter()
                plans.append(B.pf_plan_segments(pool, T, w.tokens_per_frame))
                worst = max(worst, time.perf_counter() - t1)
        return plans, (time.perf_counter() - t0) / len(plans), worst

    first, mean1, worst1 = rollout()
    again, mean2, worst2 = rollout()
    assert first == again
    print("plan per call: first rollout %.1f us mean / %.2f ms worst, second %.1f us mean" % (mean1 * 1e6, worst1 * 1e3, mean2 * 1e6))
    assert mean2 <= 50e-6
    assert mean1 <= 2e-3


def test_launch_plan_rejects_bad_arguments():
    pool = _fake_pool([synth.anchor_all(4), synth.veil(1, 2)], tpf=1560, D=128)
    lib = B.lib()
    assert lib.pf_plan_segments(None, 3, 4680, None, None, None) == B.PF_ERR_INVALID_ARG
    assert lib.pf_plan_segments(ctypes.byref(pool), -1, 4680, None, None, None) == B.PF_ERR_INVALID_ARG
    assert lib.pf_plan_segments(ctypes.byref(pool), 3, 0, None, None, None) == B.PF_ERR_INVALID_ARG
    assert lib.pf_plan_segments(ctypes.byref(pool), 9, 4680, None, None, None) == B.PF_ERR_INVALID_ARG   # 9 frames > 4 slots
    assert lib.pf_plan_segments(ctypes.byref(pool), 3, 4680, None, None, None) == B.PF_OK


def test_tuning_accepts_every_kernel_variant():
    for v in (0, 1, 2):
        assert B.lib().pf_set_tuning(v, -1, -1, -1) == B.PF_OK
    assert B.lib().pf_set_tuning(3, -1, -1, -1) == B.PF_ERR_INVALID_ARG
    B.pf_set_tuning(attn_variant=1)


def test_build_refuses_a_listing_where_the_compiler_uses_the_hidden_registers():
    """The 64-row attention kernel owns accumulation registers a64..a255 through asm statements; the build reads the device
    listing and must fail when an instruction outside those statements touches a register from a32 up."""
    from paper_2605_13111_amd import build as BLD

    def listing(body):
        return "\n".join(["other_kernel:", "\tv_accvgpr_write_b32 a200, v0", "\ts_endpgm", BLD.W64_KERNEL + ":"] + body + ["\ts_endpgm"])

    ok = ["\tv_accvgpr_write_b32 a3, v0", "\t;;#ASMSTART", "\tv_mfma_f32_32x32x16_bf16 a[64:79], v[0:3], v[4:7], a[64:79]",
          "\t;;#ASMEND", "\tv_accvgpr_read_b32 v1, a3 ; a77 in a comment does not count"]
    assert BLD.check_hidden_registers(listing(ok)) == 3
    assert BLD.check_hidden_registers(listing(["\tv_add_f32 v0, v1, v2"])) == -1
    for bad in ("\tv_accvgpr_write_b32 a64, v0", "\tscratch_load_dwordx4 a[40:43], off, off", "\tv_accvgpr_mov_b32 a32, a1"):
        with pytest.raises(RuntimeError):
            BLD.check_hidden_registers(listing(ok + [bad]))
    with pytest.raises(RuntimeError):
        BLD.check_hidden_registers("other_kernel:\n\ts_endpgm")


def test_stored_counter_summary_belongs_to_this_attention_kernel():
    """bench.py takes roofline.traffic from profiles/pf_attn_pp_kernel_c3_step.md only when that summary was made from
    this very pf_attn.hip (SHA-256 recorded in the summary); a summary of another version makes the field null."""
    sys_path_root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    import importlib.util
    spec = importlib.util.spec_from_file_location("pf_bench", os.path.join(sys_path_root, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    traffic, source = bench.profiled_traffic("c3_step", 1, "packed")
    assert traffic is not None and traffic > 100e6 and "profiles/pf_attn_pp_kernel_c3_step.md @" in source, source
    assert bench.profiled_traffic("c3_step", 2, "packed")[0] is None
    assert bench.profiled_traffic("c5_stream", 1, "packed")[0] is None
