"""Thin ctypes binding of ``libpf.so`` (C ABI in ``include/pf.h``): argument marshalling only.

Every step of the path runs in the library's HIP kernels.  PyTorch is used for device memory and
for the current stream; there is no fallback -- if the library has not been built, importing the
functions raises.
"""
import ctypes
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libpf.so")

PF_OK, PF_ERR_INVALID_ARG, PF_ERR_CAPACITY, PF_ERR_UNSUPPORTED, PF_ERR_HIP = 0, -1, -2, -3, -4
PF_SYNC_STRIDE = 32            # int32 words between the per-head counters of pf_pool.sync

EXPORTS = ["pf_index_work_bytes", "pf_attn_workspace_bytes", "pf_selected_count", "pf_retained_count", "pf_plan_segments",
           "pf_pool_reset", "pf_cache_append", "pf_cache_append_strided", "pf_build_index", "pf_ragged_attn_fwd",
           "pf_ragged_attn_fwd_strided", "pf_classify_heads", "pf_status_string", "pf_set_tuning", "pf_index_status_dev", "pf_ragged_attn_fwd_static",
           "pf_set_block_trace"]


class pf_head_policy(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("type", "mode", "sink", "recent", "cap", "period", "slots", "reserved")]


class pf_chunk_layout(ctypes.Structure):
    _fields_ = [("token_stride", ctypes.c_int64), ("head_stride", ctypes.c_int64)]


class pf_pool(ctypes.Structure):
    _fields_ = [("n_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("tokens_per_frame", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("total_slots", ctypes.c_int64),
                ("k_pool", ctypes.c_void_p), ("v_pool", ctypes.c_void_p),
                ("policy_host", ctypes.POINTER(pf_head_policy)), ("policy_dev", ctypes.c_void_p),
                ("slot_base", ctypes.c_void_p), ("n_frames", ctypes.c_void_p), ("frame_ids", ctypes.c_void_p),
                ("frame_score", ctypes.c_void_p), ("T_dev", ctypes.c_void_p), ("sync", ctypes.c_void_p),
                ("T_host", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class pf_index(ctypes.Structure):
    _fields_ = [("max_sel", ctypes.c_int32), ("seg_tiles", ctypes.c_int32),
                ("sel_count", ctypes.c_void_p), ("sel_frames", ctypes.c_void_p), ("sel_slots", ctypes.c_void_p),
                ("cu_seqlens", ctypes.c_void_p), ("work", ctypes.c_void_p), ("work_bytes", ctypes.c_size_t),
                ("q_tokens", ctypes.c_int32), ("T_built", ctypes.c_int32), ("n_blocks", ctypes.c_int32),
                ("n_partials", ctypes.c_int32), ("variant", ctypes.c_int32), ("longest_seg", ctypes.c_int32)]


_lib = None


def lib():
    """The loaded library.  Raises if it has not been built (``python paper_2605_13111_amd/build.py``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libpf.so is not built: run __graft_entry__.build() "
                               "(there is no CPU or PyTorch fallback for the HIP path)")
        L = ctypes.CDLL(LIB_PATH)
        P, I, V = ctypes.POINTER, ctypes.c_int, ctypes.c_void_p
        L.pf_index_work_bytes.restype = ctypes.c_size_t
        L.pf_index_work_bytes.argtypes = [P(pf_pool), I]
        L.pf_attn_workspace_bytes.restype = ctypes.c_size_t
        L.pf_attn_workspace_bytes.argtypes = [P(pf_pool), I]
        L.pf_selected_count.restype = I
        L.pf_selected_count.argtypes = [P(pf_head_policy), I]
        L.pf_retained_count.restype = I
        L.pf_retained_count.argtypes = [P(pf_head_policy), I]
        L.pf_plan_segments.restype = I
        L.pf_plan_segments.argtypes = [P(pf_pool), I, I, P(ctypes.c_int32), P(ctypes.c_int32), P(ctypes.c_int32)]
        L.pf_pool_reset.restype = I
        L.pf_pool_reset.argtypes = [P(pf_pool), V]
        L.pf_cache_append.restype = I
        L.pf_cache_append.argtypes = [P(pf_pool), V, V, I, V, V]
        L.pf_cache_append_strided.restype = I
        L.pf_cache_append_strided.argtypes = [P(pf_pool), V, V, I, V, P(pf_chunk_layout), V]
        L.pf_build_index.restype = I
        L.pf_build_index.argtypes = [P(pf_pool), P(pf_index), I, V]
        L.pf_ragged_attn_fwd.restype = I
        L.pf_ragged_attn_fwd.argtypes = [P(pf_pool), P(pf_index), V, V, V, V, I, ctypes.c_float, V, ctypes.c_size_t, V]
        L.pf_ragged_attn_fwd_strided.restype = I
        L.pf_ragged_attn_fwd_strided.argtypes = [P(pf_pool), P(pf_index), V, V, V, V, I, ctypes.c_float, V, ctypes.c_size_t,
                                                 P(pf_chunk_layout), V]
        L.pf_ragged_attn_fwd_static.restype = I
        L.pf_ragged_attn_fwd_static.argtypes = [P(pf_pool), P(pf_index), V, V, V, V, I, ctypes.c_float, V]
        L.pf_classify_heads.restype = I
        L.pf_classify_heads.argtypes = [V, I, I, I, ctypes.c_double, ctypes.c_double, V, V, V, V]
        L.pf_set_block_trace.restype = I
        L.pf_set_block_trace.argtypes = [V, ctypes.c_size_t]
        L.pf_set_tuning.restype = I
        L.pf_set_tuning.argtypes = [I, I, I, I]
        L.pf_index_status_dev.restype = V
        L.pf_index_status_dev.argtypes = [P(pf_index)]
        L.pf_status_string.restype = ctypes.c_char_p
        L.pf_status_string.argtypes = [I]
        _lib = L
    return _lib


class PfError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__("%s: %s (%d)" % (what, lib().pf_status_string(status).decode(), status))


def _check(status, what):
    if status != PF_OK:
        raise PfError(status, what)


def _stream(stream):
    if stream is not None:
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def make_policy(p):
    return pf_head_policy(int(p.type), int(p.mode), int(p.sink), int(p.recent), int(p.cap), int(p.period),
                          int(p.slots), 0)


def pf_set_tuning(attn_variant=-1, attn_queue=-1, seg_tiles=-1, plan_uniform=-1):
    """Process-wide tuning switches; -1 leaves a switch unchanged."""
    _check(lib().pf_set_tuning(int(attn_variant), int(attn_queue), int(seg_tiles), int(plan_uniform)), "pf_set_tuning")


def pf_set_block_trace(buffer):
    """buffer: int64 CUDA tensor of at least 4 words per compute unit, or None to switch the diagnostics off."""
    if buffer is None:
        _check(lib().pf_set_block_trace(ctypes.c_void_p(0), 0), "pf_set_block_trace")
    else:
        assert buffer.dtype == torch.int64 and buffer.is_contiguous()
        _check(lib().pf_set_block_trace(_ptr(buffer), buffer.numel() * 8), "pf_set_block_trace")


def pf_index_status(index):
    """The index's device status word as a Python int (synchronises): 0 = the plan is valid."""
    addr = lib().pf_index_status_dev(ctypes.byref(index.c))
    off = addr - index.work.data_ptr()
    torch.cuda.synchronize()
    return int(index.work[off:off + 4].view(torch.int32).item())


def pf_selected_count(policy, T):
    c = make_policy(policy)
    return int(lib().pf_selected_count(ctypes.byref(c), int(T)))


def pf_plan_segments(pool_c, T, q_tokens):
    """(seg_tiles per head, n_blocks, n_partials) of the launch plan for history length T; pool_c is a pf_pool struct."""
    seg = (ctypes.c_int32 * pool_c.n_heads)()
    nb, npart = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(lib().pf_plan_segments(ctypes.byref(pool_c), int(T), int(q_tokens), seg, ctypes.byref(nb), ctypes.byref(npart)),
           "pf_plan_segments")
    return list(seg), nb.value, npart.value


def pf_retained_count(policy, T):
    c = make_policy(policy)
    return int(lib().pf_retained_count(ctypes.byref(c), int(T)))


def slots_needed(policy, max_T):
    """Pool capacity (frames) that keeps pf_cache_append within bounds for history lengths up to max_T: the
    library's closed-form retained count at its largest, plus one slot per merged frame of a Veil head."""
    big = policy._replace(slots=1 << 20)
    need = max(pf_retained_count(big, T) for T in range(max_T + 1))
    return need + (int(policy.cap) if int(policy.type) == 2 and int(policy.cap) > 0 else 0)


class Pool:
    """Caller-side owner of one layer's pool buffers (torch tensors) and its ``pf_pool`` struct."""

    def __init__(self, policies, tokens_per_frame, head_dim, device="cuda:0", kv=None):
        self.policies = list(policies)
        H = len(self.policies)
        self.n_heads, self.tpf, self.D, self.device = H, int(tokens_per_frame), int(head_dim), torch.device(device)
        self.host_policy = (pf_head_policy * H)(*[make_policy(p) for p in self.policies])
        base = [0]
        for p in self.policies:
            base.append(base[-1] + int(p.slots))
        self.slot_base_host = base
        total = base[-1]
        dev = self.device
        if kv is None:
            self.k_pool = torch.zeros((total, self.tpf, self.D), dtype=torch.bfloat16, device=dev)
            self.v_pool = torch.zeros((total, self.tpf, self.D), dtype=torch.bfloat16, device=dev)
        else:
            self.k_pool, self.v_pool = kv
        pol_words = torch.tensor([[p.type, p.mode, p.sink, p.recent, p.cap, p.period, p.slots, 0]
                                  for p in self.policies], dtype=torch.int32)
        self.policy_dev = pol_words.to(dev)
        self.slot_base = torch.tensor(base, dtype=torch.int32).to(dev)
        self.n_frames = torch.zeros(H, dtype=torch.int32, device=dev)
        self.frame_ids = torch.full((total,), -1, dtype=torch.int32, device=dev)
        self.frame_score = torch.zeros(total, dtype=torch.float32, device=dev)
        self.T_dev = torch.zeros(1, dtype=torch.int32, device=dev)
        self.sync = torch.zeros(H * PF_SYNC_STRIDE, dtype=torch.int32, device=dev)
        self.c = pf_pool(H, self.D, self.tpf, 0, total, self.k_pool.data_ptr(), self.v_pool.data_ptr(),
                         ctypes.cast(self.host_policy, ctypes.POINTER(pf_head_policy)), self.policy_dev.data_ptr(),
                         self.slot_base.data_ptr(), self.n_frames.data_ptr(), self.frame_ids.data_ptr(),
                         self.frame_score.data_ptr(), self.T_dev.data_ptr(), self.sync.data_ptr(), 0, 0)

    @property
    def T(self):
        return int(self.c.T_host)


class Index:
    """Caller-side owner of one layer's index buffers and its ``pf_index`` struct."""

    def __init__(self, pool, q_tokens, max_sel=None, seg_tiles=0):
        H, dev = pool.n_heads, pool.device
        if max_sel is None:
            max_sel = max(int(p.slots) for p in pool.policies)
        self.max_sel = int(max_sel)
        self.sel_count = torch.zeros(H, dtype=torch.int32, device=dev)
        self.sel_frames = torch.full((H, self.max_sel), -1, dtype=torch.int32, device=dev)
        self.sel_slots = torch.full((H, self.max_sel), -1, dtype=torch.int32, device=dev)
        self.cu_seqlens = torch.zeros(H + 1, dtype=torch.int32, device=dev)
        nbytes = int(lib().pf_index_work_bytes(ctypes.byref(pool.c), int(q_tokens)))
        if nbytes == 0:
            raise PfError(PF_ERR_INVALID_ARG, "pf_index_work_bytes")
        self.work = torch.zeros(nbytes, dtype=torch.uint8, device=dev)
        self.c = pf_index(self.max_sel, int(seg_tiles), self.sel_count.data_ptr(), self.sel_frames.data_ptr(),
                          self.sel_slots.data_ptr(), self.cu_seqlens.data_ptr(), self.work.data_ptr(), nbytes,
                          0, 0, 0, 0, 0, 0)


def pf_index_work_bytes(pool, q_tokens):
    return int(lib().pf_index_work_bytes(ctypes.byref(pool.c), int(q_tokens)))


def pf_attn_workspace_bytes(pool, q_tokens):
    return int(lib().pf_attn_workspace_bytes(ctypes.byref(pool.c), int(q_tokens)))


def pf_pool_reset(pool, stream=None):
    _check(lib().pf_pool_reset(ctypes.byref(pool.c), _stream(stream)), "pf_pool_reset")


def pf_cache_append(pool, k_new, v_new, scores=None, stream=None):
    """k_new, v_new: bf16 [n_heads, n_new, tokens_per_frame, head_dim] on the pool's device."""
    assert k_new.is_contiguous() and v_new.is_contiguous() and k_new.dtype == torch.bfloat16
    assert tuple(k_new.shape) == (pool.n_heads, k_new.shape[1], pool.tpf, pool.D) and v_new.shape == k_new.shape
    if scores is not None:
        assert scores.is_contiguous() and scores.dtype == torch.float32
        assert tuple(scores.shape) == (pool.n_heads, k_new.shape[1])
    _check(lib().pf_cache_append(ctypes.byref(pool.c), _ptr(k_new), _ptr(v_new), int(k_new.shape[1]), _ptr(scores),
                                 _stream(stream)), "pf_cache_append")


def pf_cache_append_strided(pool, k_new, v_new, scores=None, stream=None):
    """k_new, v_new: bf16 views of logical shape [n_heads, n_new, tokens_per_frame, head_dim] whose tokens are
    equally spaced (e.g. a [tokens, heads, head_dim] tensor seen as heads x frames x tokens); no copy is made."""
    assert k_new.dtype == torch.bfloat16 and v_new.dtype == torch.bfloat16
    assert tuple(k_new.shape) == (pool.n_heads, k_new.shape[1], pool.tpf, pool.D) and v_new.shape == k_new.shape
    assert k_new.stride() == v_new.stride() and k_new.stride(3) == 1 and k_new.stride(1) == pool.tpf * k_new.stride(2)
    if scores is not None:
        assert scores.is_contiguous() and scores.dtype == torch.float32
        assert tuple(scores.shape) == (pool.n_heads, k_new.shape[1])
    lay = pf_chunk_layout(k_new.stride(2), k_new.stride(0))
    _check(lib().pf_cache_append_strided(ctypes.byref(pool.c), _ptr(k_new), _ptr(v_new), int(k_new.shape[1]),
                                         _ptr(scores), ctypes.byref(lay), _stream(stream)), "pf_cache_append_strided")


def pf_build_index(pool, index, q_tokens, stream=None):
    _check(lib().pf_build_index(ctypes.byref(pool.c), ctypes.byref(index.c), int(q_tokens), _stream(stream)),
           "pf_build_index")


def pf_ragged_attn_fwd(pool, index, q, k_cur, v_cur, out, workspace, softmax_scale=0.0, stream=None):
    """q, k_cur, v_cur, out: bf16 [n_heads, q_tokens, head_dim]; workspace: uint8 tensor (or None)."""
    for t in (q, k_cur, v_cur, out):
        assert t.is_contiguous() and t.dtype == torch.bfloat16 and tuple(t.shape) == tuple(q.shape)
    assert q.shape[0] == pool.n_heads and q.shape[2] == pool.D
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().pf_ragged_attn_fwd(ctypes.byref(pool.c), ctypes.byref(index.c), _ptr(q), _ptr(k_cur), _ptr(v_cur),
                                    _ptr(out), int(q.shape[1]), float(softmax_scale), _ptr(workspace), ws_bytes,
                                    _stream(stream)), "pf_ragged_attn_fwd")


def pf_ragged_attn_fwd_static(pool, index, q, k_cur, v_cur, out, softmax_scale=0.0, stream=None):
    """pf_ragged_attn_fwd without a workspace argument: partial results go to the library's own fixed device array."""
    for t in (q, k_cur, v_cur, out):
        assert t.is_contiguous() and t.dtype == torch.bfloat16 and tuple(t.shape) == tuple(q.shape)
    assert q.shape[0] == pool.n_heads and q.shape[2] == pool.D
    _check(lib().pf_ragged_attn_fwd_static(ctypes.byref(pool.c), ctypes.byref(index.c), _ptr(q), _ptr(k_cur), _ptr(v_cur),
                                           _ptr(out), int(q.shape[1]), float(softmax_scale), _stream(stream)),
           "pf_ragged_attn_fwd_static")


def pf_ragged_attn_fwd_strided(pool, index, q, k_cur, v_cur, out, workspace, softmax_scale=0.0, stream=None):
    """q, k_cur, v_cur, out: bf16 views of logical shape [n_heads, q_tokens, head_dim] with one common stride
    pattern (e.g. [tokens, heads, head_dim] tensors permuted to heads first); no copy is made."""
    for t in (q, k_cur, v_cur, out):
        assert t.dtype == torch.bfloat16 and tuple(t.shape) == tuple(q.shape) and t.stride() == q.stride()
    assert q.shape[0] == pool.n_heads and q.shape[2] == pool.D and q.stride(2) == 1
    lay = pf_chunk_layout(q.stride(1), q.stride(0))
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().pf_ragged_attn_fwd_strided(ctypes.byref(pool.c), ctypes.byref(index.c), _ptr(q), _ptr(k_cur),
                                            _ptr(v_cur), _ptr(out), int(q.shape[1]), float(softmax_scale),
                                            _ptr(workspace), ws_bytes, ctypes.byref(lay), _stream(stream)),
           "pf_ragged_attn_fwd_strided")


def pf_classify_heads(logits, alpha=0.8, beta=6.4, with_periods=True, stream=None):
    """logits: float32 [n_prompts, n_heads, n_hist] on the GPU.  Returns (head_type [n_heads] int32,
    prompt_type [n_prompts, n_heads] int32, prompt_period [n_prompts, n_heads] float64 or None)."""
    assert logits.is_contiguous() and logits.dtype == torch.float32 and logits.dim() == 3
    n_p, n_h, n_t = logits.shape
    head_type = torch.empty(n_h, dtype=torch.int32, device=logits.device)
    prompt_type = torch.empty((n_p, n_h), dtype=torch.int32, device=logits.device)
    prompt_period = torch.empty((n_p, n_h), dtype=torch.float64, device=logits.device) if with_periods else None
    _check(lib().pf_classify_heads(_ptr(logits), n_p, n_h, n_t, float(alpha), float(beta), _ptr(head_type),
                                   _ptr(prompt_type), _ptr(prompt_period), _stream(stream)), "pf_classify_heads")
    return head_type, prompt_type, prompt_period
