"""Seeded synthetic inputs shared by the HIP path's tests, the oracle's tests and the benchmark.

This module holds shapes, policy tables and random tensors only -- none of the
method's arithmetic (no frame selection, no attention).  The workloads stand in
for the paper's evaluation inputs (a Wan-1.3B-class autoregressive video DiT:
30 layers x 12 heads, head_dim 128, 1560 tokens per latent frame, 3-frame
chunks), which need model weights and prompt sets that are not available here.
"""
from collections import namedtuple

import torch

ANCHOR, WAVE, VEIL = 0, 1, 2
MODE_ALL, MODE_STRIDED, MODE_TOPK = 0, 1, 2

HeadPolicy = namedtuple("HeadPolicy", "type mode sink recent cap period slots")

Workload = namedtuple("Workload", "name n_layers n_heads head_dim tokens_per_frame chunk_frames history_frames")

WORKLOADS = {
    # tiny case: 1 Anchor (all 12), 1 Wave (every 3rd), 2 Veil (frame 0 + last 2)
    "c1_tiny": Workload("c1_tiny", 1, 4, 64, 16, 3, 12),
    # one layer at model shape: 4 Anchor (all 18), 4 Wave (every 2nd), 4 Veil (frame 0 + last 3)
    "c2_layer": Workload("c2_layer", 1, 12, 128, 1560, 3, 18),
    # full 30-layer denoising step, 57 history frames, types drawn 40/30/30
    "c3_step": Workload("c3_step", 30, 12, 128, 1560, 3, 57),
    # skewed stress case: 8 Anchor keep all 60, 32 Veil keep 4
    "c4_skew": Workload("c4_skew", 1, 40, 128, 1560, 3, 60),
    # streaming rollout: 1-frame chunks, 40 chunks, 4 denoising passes per chunk
    "c5_stream": Workload("c5_stream", 30, 12, 128, 1560, 1, 40),
    # the paper's own policy set (sink 3, recent 4, capacities 4/4/2, strided Anchor, capped Wave) rolled out in
    # 3-frame chunks to a 240-frame history: mild raggedness, short key lists
    "c6_paper": Workload("c6_paper", 30, 12, 128, 1560, 3, 240),
    # the "Head Classification only" variant of the component ablation: every head keeps the sink frames and a
    # neighbouring window whose length depends on its type (12 / 10 / 5 frames for Anchor / Wave / Veil)
    "c7_headwin": Workload("c7_headwin", 30, 12, 128, 1560, 3, 240),
}


def _cpu_gen(seed):
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    return g


def anchor_all(slots):
    return HeadPolicy(ANCHOR, MODE_ALL, 0, 0, 0, 1, slots)


def anchor_strided(cap, slots, sink=0, recent=0):
    return HeadPolicy(ANCHOR, MODE_STRIDED, sink, recent, cap, 1, slots)


def anchor_topk(cap, slots, sink=0, recent=0):
    return HeadPolicy(ANCHOR, MODE_TOPK, sink, recent, cap, 1, slots)


def wave(period, slots, cap=0, sink=0, recent=0):
    return HeadPolicy(WAVE, 0, sink, recent, cap, period, slots)


def veil(sink, recent, slots=None):
    return HeadPolicy(VEIL, 0, sink, recent, 0, 1, slots if slots is not None else sink + recent)


def veil_merged(sink, recent, n_merged, window, slots):
    """Veil head with cache merging (Sec. 4.2): ``n_merged`` merged frames, each compressing a local window of
    ``window`` frames.  ``slots`` = capacity of the head's pool region, chosen by the caller."""
    return HeadPolicy(VEIL, 0, sink, recent, n_merged, window, slots)


def drawn_policies(n_heads, seed, max_frames, topk_cap=18, veil_recent=3):
    """Head types drawn 40/30/30 (Anchor/Wave/Veil) from the seed; Anchor = TOPK with ``topk_cap``,
    Wave period uniform in {2,3,4} and uncapped, Veil = 1 sink + ``veil_recent`` adjacent frames."""
    g = _cpu_gen(seed)
    u = torch.rand(n_heads, generator=g)
    periods = torch.randint(2, 5, (n_heads,), generator=g)
    pols = []
    for h in range(n_heads):
        if u[h] < 0.4:
            pols.append(anchor_topk(topk_cap, min(max_frames, topk_cap)))
        elif u[h] < 0.7:
            pols.append(wave(int(periods[h]), max_frames))
        else:
            pols.append(veil(1, veil_recent))
    return pols


def policies(workload, layer=0, extra_frames=0, slots_of=None):
    """Policy table of one layer.  ``extra_frames`` adds pool capacity beyond the workload's history.
    ``slots_of``: see ``paper_default_policies`` (needed by ``c6_paper`` only)."""
    w = WORKLOADS[workload] if isinstance(workload, str) else workload
    cap_frames = w.history_frames + extra_frames
    if w.name == "c1_tiny":
        return [anchor_all(cap_frames), wave(3, cap_frames), veil(1, 2), veil(1, 2)]
    if w.name == "c2_layer":
        return [anchor_all(cap_frames)] * 4 + [wave(2, cap_frames)] * 4 + [veil(1, 3)] * 4
    if w.name == "c4_skew":
        return [anchor_all(cap_frames)] * 8 + [veil(1, 3)] * 32
    if w.name in ("c3_step", "c5_stream"):
        return drawn_policies(w.n_heads, 7000 + layer, cap_frames)
    if w.name == "c6_paper":
        return paper_default_policies(w.n_heads, 8000 + layer, cap_frames, slots_of)
    if w.name == "c7_headwin":
        return head_window_policies(w.n_heads, 8000 + layer)
    raise KeyError(w.name)


def paper_default_policies(n_heads, seed, max_frames, slots_of, wave_period=6):
    """The paper's own hyper-parameters (experimental setup): sink 3, forced recent 4, capacities
    Anchor/Wave/Veil 4/4/2, Veil merge window 2.  Capped Wave heads and Veil heads with merging retain a sliding
    window of the history; how many pool slots that takes is the caller's to say: ``slots_of(policy) -> int`` is
    applied to those heads (the tests size from the oracle's retained sets, the benchmark from the library's
    closed-form count -- this module holds none of the method's arithmetic)."""
    g = _cpu_gen(seed)
    u = torch.rand(n_heads, generator=g)
    pols = []
    for h in range(n_heads):
        if u[h] < 0.4:
            pols.append(anchor_strided(4, max_frames, sink=3, recent=4))
        elif u[h] < 0.7:
            p = wave(wave_period, max_frames, cap=4, sink=3, recent=4)
            pols.append(p._replace(slots=min(max_frames, slots_of(p))))
        else:
            p = veil_merged(3, 4, 2, 2, max_frames)
            pols.append(p._replace(slots=slots_of(p)))
    return pols


def head_window_policies(n_heads, seed, windows=(12, 10, 5), sink=3):
    """Type-specific neighbouring windows (component ablation, "Head Classification" variant): a head of type
    Anchor / Wave / Veil keeps the sink frames plus its last 12 / 10 / 5 frames; types drawn 40/30/30 as in
    ``paper_default_policies``.  A sink + recent-window policy is what the library calls a Veil head without
    merging, whatever the head's type."""
    g = _cpu_gen(seed)
    u = torch.rand(n_heads, generator=g)
    pols = []
    for h in range(n_heads):
        win = windows[0] if u[h] < 0.4 else windows[1] if u[h] < 0.7 else windows[2]
        pols.append(veil(sink, win))
    return pols


def randn_bf16(shape, seed, device="cpu", std=1.0):
    """Seeded N(0, std^2) tensor rounded to bfloat16."""
    if str(device).startswith("cuda"):
        g = torch.Generator(device=device)
        g.manual_seed(int(seed))
        x = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    else:
        x = torch.randn(shape, generator=_cpu_gen(seed), dtype=torch.float32)
    if std != 1.0:
        x = x * std
    return x.to(torch.bfloat16)


def frame_scores(n_heads, n_frames, seed, device="cpu"):
    """Seeded U(0,1) float32 scores, one per (head, appended frame)."""
    s = torch.rand((n_heads, n_frames), generator=_cpu_gen(seed), dtype=torch.float32)
    return s.to(device)


def bits(t):
    """bfloat16 tensor -> numpy uint16 bit patterns (host copy)."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view("uint16")


# ---- historical attention sequences for the offline head classification (Sec. 4.1) --------------------
# Kinds of synthetic sequence (what the paper's observations describe, plus its two failure cases):
#   0 broadly positive scores (Anchor-like)        1 oscillation of period ~6 around zero (Wave-like)
#   2 suppressed history (Veil-like)               3 one-sided oscillation ("pseudo-periodic", positive bias)
#   4 slow drift around zero, no short period      5 the same with a negative mean
LOGIT_KINDS = 6


def head_logits(n_prompts, n_heads, n_hist, seed, wave_period=6.0):
    """Seeded float32 sequences [n_prompts, n_heads, n_hist] and the kind of every head [n_heads].  The kind is a
    property of the head; prompts differ by noise, phase and a small period jitter."""
    g = _cpu_gen(seed)
    kinds = torch.randint(0, LOGIT_KINDS, (n_heads,), generator=g)
    t = torch.arange(n_hist, dtype=torch.float64)[None, None, :]
    noise = torch.randn((n_prompts, n_heads, n_hist), generator=g, dtype=torch.float64)
    phase = torch.rand((n_prompts, n_heads, 1), generator=g, dtype=torch.float64) * 6.283185307179586
    jitter = 1.0 + 0.04 * (torch.rand((n_prompts, n_heads, 1), generator=g, dtype=torch.float64) - 0.5)
    osc = torch.sin(6.283185307179586 * t / (wave_period * jitter) + phase)
    slow = torch.sin(6.283185307179586 * t / (n_hist * 0.45) + phase)
    k = kinds[None, :, None]
    x = torch.where(k == 0, 1.6 + 0.9 * noise,
        torch.where(k == 1, 1.5 * osc + 0.35 * noise,
        torch.where(k == 2, -1.6 + 0.9 * noise,
        torch.where(k == 3, 2.2 + 1.2 * osc + 0.3 * noise,
        torch.where(k == 4, 0.25 + 1.4 * slow + 0.06 * noise, -0.25 + 1.4 * slow + 0.06 * noise)))))
    return x.to(torch.float32), kinds
