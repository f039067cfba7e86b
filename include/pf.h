/*
 * pf.h -- C ABI of the ragged-cache attention library for MI355X (gfx950).
 *
 * The library implements the hot path of Pyramid Forcing's "Heterogeneous
 * KVCache Computation Optimization" (paper Sec. 4.3) on top of the per-head
 * cache policies of Sec. 4.2: every attention head of an autoregressive video
 * DiT layer attends from the tokens of the chunk being generated to its OWN
 * policy-selected set of history frames, so key/value lengths differ per head.
 *
 * Conventions
 *  - Plain C.  Every function returns an int status (PF_OK or a negative
 *    PF_ERR_* code), never throws, never allocates or frees device memory and
 *    never synchronises with the device: all work is enqueued on the caller's
 *    stream (a hipStream_t passed as void*; NULL = the default stream).
 *  - Every buffer is owned by the caller.  "dev" = device memory, "host" = host
 *    memory.  Device buffers must stay valid until the enqueued work has run.
 *    Host structures are read during the call only; pf_cache_append and
 *    pf_build_index update the host-side bookkeeping fields marked [lib].
 *  - A "head" is one of the N = B x H independent sequences of Sec. 4.3
 *    (batch-head order); the configurations used here have B = 1.
 *  - A "frame" is one latent frame = tokens_per_frame tokens; history frames
 *    carry global ids 0 .. T-1 and the chunk being generated starts at id T.
 *  - K/V/Q/out elements are bfloat16 (dtype 0).  head_dim is 64 or 128.
 *  - Calls that use the same pf_pool or pf_index must be ordered on one stream
 *    (or otherwise serialised by the caller); concurrent use is a data race.
 */
#ifndef PF_H
#define PF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PF_OK                 0
#define PF_ERR_INVALID_ARG   -1   /* null / misaligned pointer, bad size, bad policy      */
#define PF_ERR_CAPACITY      -2   /* a head's pool region or max_sel cannot hold the result */
#define PF_ERR_UNSUPPORTED   -3   /* head_dim / dtype the kernels do not implement        */
#define PF_ERR_HIP           -4   /* a HIP runtime call or kernel launch failed           */

/* head types: the three head sets of Sec. 4.1 (mutually exclusive, covering) */
#define PF_ANCHOR 0
#define PF_WAVE   1
#define PF_VEIL   2
/* Anchor modes */
#define PF_MODE_ALL     0   /* keep every intermediate frame                               */
#define PF_MODE_STRIDED 1   /* adaptive strided sliding window, Sec. 4.2 Eq. 4             */
#define PF_MODE_TOPK    2   /* the cap best-scored intermediate frames (static scores)     */

/*
 * Cache policy of one head (Sec. 4.2).  All heads share the meaning of `sink`
 * (S, first frames of the video) and `recent` (R, newest frames), which are
 * always attended; the type-specific rule acts on the intermediate frames
 * S .. T-R-1:
 *   Anchor/ALL      all of them;
 *   Anchor/STRIDED  if more than cap: the cap window centres
 *                   S + (t'-1) - floor(i*t'/cap) - floor(t'/(2cap)), i=0..cap-1,
 *                   t' = number of intermediate frames (Eq. 4 in 0-based ids);
 *   Anchor/TOPK     the cap frames with the largest score given at append time
 *                   (ties: smaller id first);
 *   Wave            T - i*period, i = 1,2,... (Eq. 5 / Observation 2), the cap
 *                   nearest ones if cap > 0;
 *   Veil            none if cap = 0.  With cap > 0, cache merging (Sec. 4.2): cap merged
 *                   frames, each compressing a local window of `period` = m frames.
 *                   Window j (0 = nearest) covers ids T-R-(j+1)m .. T-R-jm-1 and exists
 *                   if it lies entirely in the intermediate range; its merged frame is
 *                   the concatenation over i = 0..m-1 of the tokens of frame w0+i whose
 *                   index is congruent to i modulo m (tokens_per_frame tokens in all).
 *                   In the head's key sequence the merged frames stand between the sink
 *                   and the recent frames, oldest window first; sel_frames holds
 *                   PF_MERGED_FRAME | w0 for them (w0 = first frame of the window).
 *                   The pool keeps them in the LAST cap slots of the head's region
 *                   (window j in slot slots-1-j), rebuilt by every pf_cache_append; raw
 *                   frames may use slots - cap slots.
 * cap = 0 means unlimited (Anchor, Wave).  `slots` is the capacity, in frames, of this
 * head's region of the pool.
 */
#define PF_MERGED_FRAME (1 << 30)
#define PF_SYNC_STRIDE 32          /* int32 words between the per-head counters of pf_pool.sync (128 bytes) */
typedef struct pf_head_policy {
  int32_t type;      /* PF_ANCHOR | PF_WAVE | PF_VEIL */
  int32_t mode;      /* PF_MODE_*, Anchor only (0 otherwise) */
  int32_t sink;      /* S >= 0 */
  int32_t recent;    /* R >= 0 */
  int32_t cap;       /* Cap >= 0, 0 = unlimited */
  int32_t period;    /* Wave: P >= 1; Veil with cap > 0: window size m >= 1; ignored otherwise */
  int32_t slots;     /* >= 1 */
  int32_t reserved;  /* must be 0 */
} pf_head_policy;

/*
 * The per-head ragged KV pool: the retained candidate history H(t) of Sec. 2.2
 * stored as the flattened, unpadded layout of Sec. 4.3.  Head h owns pool
 * slots slot_base[h] .. slot_base[h+1]-1; its resident frames sit in the first
 * n_frames[h] of them in ascending frame id (left-packed), the rest are free
 * (frame_ids = -1, frame_score = 0, K/V bytes unspecified).
 * Slot s holds tokens_per_frame x head_dim elements at
 * k_pool + s*tokens_per_frame*head_dim (same for v_pool).
 */
typedef struct pf_pool {
  int32_t n_heads;
  int32_t head_dim;               /* 64 or 128 */
  int32_t tokens_per_frame;       /* >= 1 */
  int32_t dtype;                  /* 0 = bfloat16 */
  int64_t total_slots;            /* sum of policy[h].slots */
  void *k_pool;                   /* dev [total_slots][tokens_per_frame][head_dim], 16-byte aligned */
  void *v_pool;                   /* dev, same shape */
  const pf_head_policy *policy_host; /* host [n_heads] */
  const pf_head_policy *policy_dev;  /* dev  [n_heads], same contents */
  const int32_t *slot_base;       /* dev [n_heads+1], exclusive prefix sum of slots */
  int32_t *n_frames;              /* dev [n_heads]      resident frames per head */
  int32_t *frame_ids;             /* dev [total_slots]  global frame id, -1 = free */
  float   *frame_score;           /* dev [total_slots]  score of the resident frame, 0 = free */
  int32_t *T_dev;                 /* dev [1]            frames appended so far */
  int32_t *sync;                  /* dev [n_heads * PF_SYNC_STRIDE] library scratch (one arrival counter per head,
                                     each in a cache line of its own), zeroed by pf_pool_reset */
  int32_t T_host;                 /* [lib] host mirror of *T_dev (no device read-back needed) */
  int32_t reserved;
} pf_pool;

/*
 * The frame index of one layer: for each head the selected subset I(t) of the
 * pool (Sec. 2.2), as ascending frame ids and the pool slots that hold them,
 * plus the boundary indices of the flattened ragged history (Sec. 4.3):
 * cu_seqlens[0] = 0, cu_seqlens[h+1] = cu_seqlens[h] + sel_count[h]*tokens_per_frame.
 * The key/value sequence head h attends to is its selected frames in this
 * order followed by the current chunk: Lkv[h] = cu_seqlens[h+1]-cu_seqlens[h] + q_tokens.
 * `work` is library scratch (launch plan of pf_ragged_attn_fwd, private format).
 */
typedef struct pf_index {
  int32_t max_sel;                /* row length of sel_frames / sel_slots */
  int32_t seg_tiles;              /* tuning: key tiles per work item, 0 = chosen by the library per launch */
  int32_t *sel_count;             /* dev [n_heads] */
  int32_t *sel_frames;            /* dev [n_heads][max_sel], unused entries -1 */
  int32_t *sel_slots;             /* dev [n_heads][max_sel], global pool slots, unused -1 */
  int32_t *cu_seqlens;            /* dev [n_heads+1] */
  void *work;                     /* dev, >= pf_index_work_bytes(), 16-byte aligned */
  size_t work_bytes;
  /* [lib] host-side description of the plan written by pf_build_index */
  int32_t q_tokens;               /* chunk length the plan was built for */
  int32_t T_built;                /* pool->T_host at build time */
  int32_t n_blocks;               /* workgroups of the attention launch */
  int32_t n_partials;             /* partial-result slots the launch uses */
  int32_t variant;                /* kernel variant the plan was built for */
  int32_t longest_seg;            /* longest segment (64-key tiles per work item) the library planned; 0 when the caller fixed seg_tiles */
} pf_index;

/*
 * Layout of the chunk tensors when they are not packed per head.  The model keeps
 * its activations as [tokens][heads][head_dim] (the attention of Eq. 1 is applied
 * to projections of that shape), so the strided entry points read q / k_cur / v_cur
 * / k_new / v_new and write out in place, without a permute pass before or after
 * (the per-call packing the fused kernel of Sec. 4.3 removes).
 * Strides are in ELEMENTS: element (head h, token t, channel d) sits at
 * base + h*head_stride + t*token_stride + d.  Both must be multiples of 8
 * (16-byte rows), >= head_dim, and rows must not overlap: either
 * head_stride >= tokens*token_stride or token_stride >= n_heads*head_stride.
 */
typedef struct pf_chunk_layout {
  int64_t token_stride;
  int64_t head_stride;
} pf_chunk_layout;

/* ---- sizes (host only, no device access) -------------------------------- */

/* Bytes of pf_index.work needed for a pool with these policies, for any T the
 * pool's slot capacities allow.  0 on a bad argument. */
size_t pf_index_work_bytes(const pf_pool *pool, int q_tokens);

/* Upper bound of the workspace pf_ragged_attn_fwd needs for this pool and
 * chunk length (partial results of heads whose keys are split over several
 * workgroups), for any T the slot capacities allow.  Never 0 for valid input. */
size_t pf_attn_workspace_bytes(const pf_pool *pool, int q_tokens);

/* ---- host-side planning helpers (no device access) ---------------------- */

/* Number of frames head `pol` attends to / the pool retains when the history
 * has T frames.  Both are functions of T and the policy alone (for TOPK the
 * scores decide WHICH frames, not how many).  Negative = PF_ERR_INVALID_ARG. */
int pf_selected_count(const pf_head_policy *pol, int T);
int pf_retained_count(const pf_head_policy *pol, int T);

/* The launch plan pf_build_index would make for the pool's policies at history
 * length T (pool->T_host is not read) and a chunk of q_tokens tokens, with the
 * library's own choice of segment lengths: seg_tiles[h] = 64-key tiles per work item
 * of head h (>= its tile count when the head is not split), *n_blocks = work items
 * of the launch, *n_partials = partial-result slots.  The same figures as the ones
 * pf_index_work_bytes / pf_attn_workspace_bytes bound.  Host only; any pointer but
 * pool may be NULL.  PF_OK or PF_ERR_INVALID_ARG. */
int pf_plan_segments(const pf_pool *pool, int T, int q_tokens, int32_t *seg_tiles,
                     int32_t *n_blocks, int32_t *n_partials);

/* Process-wide tuning switches, for tests and A/B measurements.  Each argument: -1 = leave unchanged.
 *   attn_variant  attention kernel for head_dim 128: 0 = 4 waves x 32 query rows, staged through registers;
 *                 1 = 8 waves x 32 rows in two alternating groups (the default);
 *                 2 = 4 waves x 64 rows, one wave per SIMD (measured slower than 1; kept selectable)
 *   attn_queue    1 = resident workgroups fed from per-die work queues (default), 0 = one work item per workgroup
 *   seg_tiles     key tiles per work item for every head, 0 = planned per launch (default)
 *   plan_uniform  1 = the planner stops after choosing one segment length for all heads
 * The initial values come from the environment variables PF_ATTN_VARIANT, PF_ATTN_QUEUE, PF_SEG_TILES and
 * PF_PLAN_UNIFORM, read once at the library's first use.  Takes effect at the next pf_build_index (and the size
 * queries); an index must be rebuilt after a change.  Not synchronised with calls running on other threads. */
int pf_set_tuning(int attn_variant, int attn_queue, int seg_tiles, int plan_uniform);

/* Diagnostics (process-wide, off by default): while a buffer is set, every work-queue launch of the pipelined
 * attention kernel (variants 1 and 2) makes each of its resident workgroups -- one per compute unit -- write int64 words
 * at dev_buffer + 64 * workgroup: [0] ticks of the device's constant 100 MHz clock spent inside work items, [1] the
 * start of its first item and [2] the end of its last item on that clock, [3] the number of items it ran, [4] shader-clock
 * cycles spent inside work items ([4] / [0] x 100 MHz = the clock the compute unit really ran at); [5..7] unused.
 * A launch with more resident workgroups than bytes / 64 writes nothing.  Each launch overwrites the last one's
 * figures; NULL switches it off.  The buffer must stay valid while launches that were enqueued with it may run. */
int pf_set_block_trace(void *dev_buffer, size_t bytes);

/* ---- the hot path -------------------------------------------------------- */

/* Empty the pool: T = 0, n_frames = 0, frame_ids = -1, frame_score = 0,
 * sync = 0 (all n_heads * PF_SYNC_STRIDE words).  K/V bytes are left as they are. */
int pf_pool_reset(pf_pool *pool, void *stream);

/*
 * Write-back of Sec. 2.2: append n_new frames (ids T .. T+n_new-1) to every
 * head, evict what the head's policy no longer retains and left-pack the
 * survivors (stable: ascending frame id), in one launch for all heads
 * (the batched workspace packing of Sec. 4.3).
 *   k_new, v_new  dev [n_heads][n_new][tokens_per_frame][head_dim], 16-byte aligned
 *   scores        dev [n_heads][n_new] float, or NULL (= 0) -- used by Anchor/TOPK
 * PF_ERR_CAPACITY if any head would hold more than its `slots` frames after
 * eviction, or if a head's resident frames plus n_new exceed 1024 (the kernel's
 * per-head tables); PF_ERR_UNSUPPORTED if n_heads x the largest Veil merge capacity exceeds
 * 65535 (the merge launch's grid).  The pool is then untouched: every check happens before
 * the first launch.  On success pool->T_host += n_new.
 */
int pf_cache_append(pf_pool *pool, const void *k_new, const void *v_new,
                    int n_new, const float *scores, void *stream);

/* The same with k_new / v_new laid out by `layout` (token index = frame*tokens_per_frame
 * + token inside the frame, n_new*tokens_per_frame tokens): the write-back reads the
 * chunk's keys and values where the attention pass left them.  layout must not be NULL. */
int pf_cache_append_strided(pf_pool *pool, const void *k_new, const void *v_new,
                            int n_new, const float *scores,
                            const pf_chunk_layout *layout, void *stream);

/*
 * Select every head's frames for the chunk that starts at frame id T
 * (Sec. 4.2 policies), map them to pool slots, write cu_seqlens (Sec. 4.3) and
 * the private launch plan of pf_ragged_attn_fwd for a chunk of q_tokens tokens.
 * PF_ERR_CAPACITY if a head selects more than max_sel frames.
 */
int pf_build_index(const pf_pool *pool, pf_index *index, int q_tokens, void *stream);

/* Device address of the index's status word (one int32 inside index->work), written by pf_build_index's kernel:
 * 0 = the selection found on the device agrees with the launch plan the host made from the policies' closed-form
 * counts; non-zero = it does not (the pool was not filled through pf_cache_append, or tables were overwritten), the
 * plan is then left empty and pf_ragged_attn_fwd on this index writes nothing to `out`.  A caller that cannot
 * rule this out reads the word after the stream has run the build.  NULL on a bad argument. */
const int32_t *pf_index_status_dev(const pf_index *index);

/*
 * Ragged-cache attention (Sec. 4.3) = Eq. 1 evaluated per head over that
 * head's key/value sequence [selected history frames || current chunk]:
 *   out[h,i,:] = sum_j softmax_j( scale * q[h,i,:].K_h[j,:] ) * V_h[j,:]
 * Every chunk token sees all chunk tokens and all selected history (no mask
 * inside the chunk).  bf16 inputs, fp32 accumulation, bf16 output; ONE launch
 * for all heads of the layer.
 *   q, k_cur, v_cur, out  dev [n_heads][q_tokens][head_dim] bf16, 16-byte aligned
 *   softmax_scale         0 = 1/sqrt(head_dim)
 *   workspace             dev, >= pf_attn_workspace_bytes(), 16-byte aligned
 * `index` must have been built for this q_tokens and the pool's current T.
 * index->work (arrival counters, work-queue tickets) and the workspace are written
 * by the launch and left ready for the next one: launches that share either must
 * not overlap in time (same stream, or ordered by events).
 */
int pf_ragged_attn_fwd(const pf_pool *pool, const pf_index *index,
                       const void *q, const void *k_cur, const void *v_cur, void *out,
                       int q_tokens, float softmax_scale,
                       void *workspace, size_t workspace_bytes, void *stream);

/* The same with q, k_cur, v_cur and out laid out by `layout` (one layout for all
 * four; q_tokens tokens).  layout must not be NULL.  History tiles are unaffected;
 * chunk tiles are fetched with the same 16-byte copies, one token row at a time. */
int pf_ragged_attn_fwd_strided(const pf_pool *pool, const pf_index *index,
                               const void *q, const void *k_cur, const void *v_cur, void *out,
                               int q_tokens, float softmax_scale,
                               void *workspace, size_t workspace_bytes,
                               const pf_chunk_layout *layout, void *stream);

/*
 * pf_ragged_attn_fwd for callers that cannot allocate device memory or bring a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation.  The partial results of split heads go to a fixed
 * 160 MiB array inside the library's device image instead of `workspace` (each GPU the library runs on holds its
 * own copy until the process ends); everything else -- arguments, result, errors -- is as for pf_ragged_attn_fwd
 * with packed chunk tensors.  PF_ERR_CAPACITY when the launch plan of `index` needs more than 160 MiB of partial
 * results (n_partials x 256 rows x (head_dim + 2) floats; the 30-layer configuration's layers need up to 133 MiB).
 * The call allocates nothing and frees nothing; the array's address on the current device is looked up at the
 * first call on that device (so make one call per device before capturing a graph).  All calls on one GPU share
 * the array: launches that use it must not overlap in time (same stream, or ordered by events), whatever pool or
 * index they belong to.  Nothing in it needs clearing: every partial is written in full before it is read.
 */
int pf_ragged_attn_fwd_static(const pf_pool *pool, const pf_index *index,
                              const void *q, const void *k_cur, const void *v_cur, void *out,
                              int q_tokens, float softmax_scale, void *stream);

/* ---- before the hot path: which head gets which policy -------------------- */

/*
 * Offline tri-pattern head classification (Sec. 4.1).  For every sampled prompt p and
 * head h, logits[p][h][t] is the historical attention sequence a(t): the pre-softmax
 * score of the newest frame towards history frame t, t = 0 .. n_hist-1.  Per sequence:
 *   r_pos = fraction of positive scores; r_pos >= alpha -> PF_ANCHOR, 1 - r_pos >= alpha -> PF_VEIL;
 *   otherwise the dominant period P of the sequence (first-order difference, mean removal,
 *   Hann window, real spectrum without the zero-frequency bin, harmonic folding with weights
 *   1/j over 4 harmonics, P = length / bin; appendix on the FFT analysis): P < beta -> PF_WAVE;
 *   otherwise mean(a) > 0 -> PF_ANCHOR, else PF_VEIL.
 * head_type[h] is the majority vote over the prompts (equal counts: the smaller code).
 *   logits         dev [n_prompts][n_heads][n_hist] float, n_hist <= 1024
 *   head_type      dev [n_heads] int32 (out)
 *   prompt_type    dev [n_prompts][n_heads] int32 (out, also the vote's input)
 *   prompt_period  dev [n_prompts][n_heads] double (out) or NULL: P, +inf where it was not computed
 * The paper's thresholds are alpha = 0.8, beta = 6.4.  fp64 arithmetic throughout.
 */
int pf_classify_heads(const float *logits, int n_prompts, int n_heads, int n_hist,
                      double alpha, double beta, int32_t *head_type, int32_t *prompt_type,
                      double *prompt_period, void *stream);

/* Human-readable text for a status code (static storage). */
const char *pf_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* PF_H */
