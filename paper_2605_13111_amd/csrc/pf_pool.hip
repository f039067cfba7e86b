// Per-head ragged KV pool: reset and append / evict / left-pack (the write-back of Sec. 2.2 done as
// the batched packing of Sec. 4.3: one launch for all heads, no per-head host loop).
//
// Hazard-free in-place packing.  Survivors keep their ascending order, so a frame only ever moves to
// a lower slot, and the destination of the k-th kept frame can only coincide with the source of an
// EARLIER kept frame.  Every thread owns a fixed byte range of the frame payload and walks the kept
// frames in order, so all reads and writes of one byte range are issued by one thread in program
// order: no synchronisation between workgroups is needed and the copy streams at HBM speed.
#include "pf_internal.h"
#ifndef PF_STRICT_FENCES
#define PF_STRICT_FENCES 0   // 1: release fence in front of every arrival counter (the memory model's own form)
#endif

typedef __attribute__((ext_vector_type(4))) unsigned int pool_unit;   // one 16-byte unit of payload (a native vector: arrays of it stay in registers)
constexpr int POOL_THREADS = 256;
constexpr int POOL_UNITS_PER_THREAD = 2;                    // 16-byte units per thread per frame
constexpr int POOL_CHUNK_UNITS = POOL_THREADS * POOL_UNITS_PER_THREAD;
constexpr int POOL_MAX_CAND = 1024;                         // resident + new frames of one head (20 KB of tables per workgroup)
constexpr int POOL_MOVE_BATCH = 8;                          // frames in flight per thread
constexpr int POOL_PREFETCH = 4;                            // new frames whose payload is requested before the plan is made

__global__ void pf_pool_reset_kernel(int32_t *n_frames, int32_t *frame_ids, float *frame_score,
                                     int32_t *T_dev, int32_t *sync, int n_heads, long long total_slots) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < total_slots) {
    frame_ids[i] = -1;
    frame_score[i] = 0.0f;
  }
  if (i < n_heads) n_frames[i] = 0;
  if (i < (long long)n_heads * PF_SYNC_STRIDE) sync[i] = 0;
  if (i == 0) *T_dev = 0;
}

struct PoolAppendParams {
  uint4 *k_pool, *v_pool;
  const uint4 *k_new, *v_new;
  const float *scores;
  const pf_head_policy *policy;
  const int32_t *slot_base;
  int32_t *n_frames, *frame_ids, *T_dev, *sync;
  float *frame_score;
  int T, n_new, frame_units, blocks_per_head;
  // new frames: strides in 16-byte units between tokens and between heads (packed [heads][n_new][tokens][D]:
  // head_dim / 8 and n_new * frame_units)
  int row_shift;                        // log2 of the units per row (head_dim 64 -> 3, 128 -> 4)
  long long new_tok_units, new_head_units;
};

// Is candidate frame `f` (an intermediate frame of head p at history length T) kept by the type rule?
// rank = number of intermediate candidates that beat it (TOPK only).
__device__ __forceinline__ bool middle_kept(const pf_head_policy &p, int T, int f, int rank) {
  if (p.type == PF_ANCHOR) return (p.mode == PF_MODE_TOPK && p.cap > 0) ? rank < p.cap : true;
  if (p.type == PF_WAVE) return p.cap <= 0 ? true : f >= pf_wave_oldest(p, T);
  // Veil: sink + recent only; with cache merging also the frames the merged windows are (and will be) made of
  return p.cap > 0 && f >= T - p.recent - p.cap * p.period;
}

// Four or five workgroups share a compute unit, so a wave may take up to 128 registers: the batch of loads and the
// prefetched new frames stay in flight together instead of being parked (and waited for) early.
__global__ __launch_bounds__(POOL_THREADS) __attribute__((amdgpu_waves_per_eu(1, 4))) void pf_pool_append_kernel(PoolAppendParams P) {
  __shared__ int32_t s_id[POOL_MAX_CAND];
  __shared__ float s_score[POOL_MAX_CAND];
  __shared__ int32_t s_dest[POOL_MAX_CAND];     // destination slot or -1 (evicted)
  __shared__ int32_t s_move_src[POOL_MAX_CAND]; // >= 0: resident slot, < 0: -(new index)-1
  __shared__ int32_t s_move_dst[POOL_MAX_CAND];
  __shared__ int32_t s_counts[2];               // kept frames, moves
  __shared__ int32_t s_wave[POOL_THREADS / 64];
  __shared__ int32_t s_last;

  const int h = blockIdx.y;
  const bool is_v = blockIdx.z != 0;
  const int tid = threadIdx.x;
  const pf_head_policy pol = P.policy[h];
  const int base = P.slot_base[h];
  const int n_old = P.n_frames[h];
  const int n_cand = n_old + P.n_new;
  const int T_new = P.T + P.n_new;

  // ---- the new frames' payload does not depend on the plan (only its destination does): this thread's share of the
  // first POOL_PREFETCH new frames is requested before the tables are even read, so these loads travel while the
  // plan below is worked out ----
  const pool_unit *fresh = (const pool_unit *)(is_v ? P.v_new : P.k_new) + (size_t)h * P.new_head_units;
  const long long new_frame_units = (long long)(P.frame_units >> P.row_shift) * P.new_tok_units;   // tokens per frame x token stride
  const int u0 = blockIdx.x * POOL_CHUNK_UNITS + tid;
  bool valid[POOL_UNITS_PER_THREAD];
  int unit_c[POOL_UNITS_PER_THREAD];
  long long fresh_off[POOL_UNITS_PER_THREAD];
#pragma unroll
  for (int u = 0; u < POOL_UNITS_PER_THREAD; ++u) {
    const int unit = u0 + u * POOL_THREADS;
    valid[u] = unit < P.frame_units;
    unit_c[u] = valid[u] ? unit : 0;
    // a new frame's token rows may be strided: unit -> (token, 16-byte piece of its row)
    fresh_off[u] = (long long)(unit_c[u] >> P.row_shift) * P.new_tok_units + (unit_c[u] & ((1 << P.row_shift) - 1));
  }
  static_assert(POOL_PREFETCH == 4 && POOL_UNITS_PER_THREAD == 2, "the prefetched frames are held in named registers");
  pool_unit nf00, nf01, nf10, nf11, nf20, nf21, nf30, nf31;
  {
    const pool_unit *f0 = fresh, *f1 = fresh + (size_t)pf_min(1, P.n_new - 1) * new_frame_units;
    const pool_unit *f2 = fresh + (size_t)pf_min(2, P.n_new - 1) * new_frame_units, *f3 = fresh + (size_t)pf_min(3, P.n_new - 1) * new_frame_units;
    nf00 = f0[fresh_off[0]]; nf01 = f0[fresh_off[1]];
    nf10 = f1[fresh_off[0]]; nf11 = f1[fresh_off[1]];
    nf20 = f2[fresh_off[0]]; nf21 = f2[fresh_off[1]];
    nf30 = f3[fresh_off[0]]; nf31 = f3[fresh_off[1]];
  }

  for (int j = tid; j < n_cand; j += POOL_THREADS) {
    if (j < n_old) {
      s_id[j] = P.frame_ids[base + j];
      s_score[j] = P.frame_score[base + j];
    } else {
      s_id[j] = P.T + (j - n_old);
      s_score[j] = P.scores ? P.scores[(size_t)h * P.n_new + (j - n_old)] : 0.0f;
    }
  }
  __syncthreads();

  const int mid_lo = pol.sink, mid_hi = T_new - pol.recent;   // intermediate ids [mid_lo, mid_hi)
  const bool need_rank = pol.type == PF_ANCHOR && pol.mode == PF_MODE_TOPK && pol.cap > 0;
  for (int j = tid; j < n_cand; j += POOL_THREADS) {
    const int f = s_id[j];
    bool keep;
    if (f < mid_lo || f >= mid_hi) {
      keep = true;                                            // sink or recent
    } else {
      int rank = 0;
      if (need_rank) {
        const float sc = s_score[j];
        for (int g = 0; g < n_cand; ++g) {
          const int fg = s_id[g];
          if (fg < mid_lo || fg >= mid_hi) continue;
          const float sg = s_score[g];
          rank += (sg > sc || (sg == sc && fg < f)) ? 1 : 0;
        }
      }
      keep = middle_kept(pol, T_new, f, rank);
    }
    s_dest[j] = keep ? 0 : -1;
  }
  __syncthreads();
  // destination slots (stable left-pack = exclusive prefix count of the keep flags) and the move list
  // (new frames, and survivors that shift left), by ballots: 256 candidates per round
  {
    const int lane = tid & 63, wave = tid >> 6;
    const unsigned long long below = (1ull << lane) - 1ull;
    int kept_base = 0, move_base = 0;
    for (int j0 = 0; j0 < n_cand; j0 += POOL_THREADS) {
      const int j = j0 + tid;
      const bool keep = j < n_cand && s_dest[j] >= 0;
      const unsigned long long km = __builtin_amdgcn_ballot_w64(keep);
      if (lane == 0) s_wave[wave] = __builtin_popcountll(km);
      __syncthreads();
      int dest = kept_base + __builtin_popcountll(km & below), kept_round = 0;
      for (int w = 0; w < POOL_THREADS / 64; ++w) {
        if (w < wave) dest += s_wave[w];
        kept_round += s_wave[w];
      }
      const bool move = keep && (j >= n_old || dest != j);
      const unsigned long long mm = __builtin_amdgcn_ballot_w64(move);
      __syncthreads();
      if (lane == 0) s_wave[wave] = __builtin_popcountll(mm);
      __syncthreads();
      int mpos = move_base + __builtin_popcountll(mm & below), moves_round = 0;
      for (int w = 0; w < POOL_THREADS / 64; ++w) {
        if (w < wave) mpos += s_wave[w];
        moves_round += s_wave[w];
      }
      if (keep) s_dest[j] = dest;
      if (move) {
        s_move_src[mpos] = j < n_old ? j : -(j - n_old) - 1;
        s_move_dst[mpos] = dest;
      }
      kept_base += kept_round;
      move_base += moves_round;
      __syncthreads();
    }
    if (tid == 0) {
      s_counts[0] = kept_base;
      s_counts[1] = move_base;
    }
  }
  __syncthreads();
  const int n_kept = s_counts[0], n_moves = s_counts[1];

  // ---- payload: this workgroup owns 16-byte units [u0, u0+POOL_CHUNK_UNITS) of every frame.  The loads of a
  // batch are unconditional (indices clamped, the source chosen by a select) so that all of them are in flight
  // before the first store; only the stores are predicated. ----
  pool_unit *pool = (pool_unit *)(is_v ? P.v_pool : P.k_pool) + (size_t)base * P.frame_units;
  // moves of survivors come first in the list (ascending candidate order), the new frames last; the prefetched
  // new frames are stored after all of them (a new frame's slot may still hold a survivor that has to move)
  const int n_pref = pf_min(P.n_new, POOL_PREFETCH);
  int n_moves_loop = n_moves;
  for (int j = 0; j < n_pref; ++j) n_moves_loop -= s_dest[n_old + j] >= 0 ? 1 : 0;
  if (P.n_new > POOL_PREFETCH) n_moves_loop = n_moves;        // more new frames than registers: the general loop takes them all
  for (int m0 = 0; m0 < n_moves_loop; m0 += POOL_MOVE_BATCH) {
    pool_unit r[POOL_MOVE_BATCH][POOL_UNITS_PER_THREAD];
#pragma unroll
    for (int b = 0; b < POOL_MOVE_BATCH; ++b) {
      const int src = s_move_src[pf_min(m0 + b, n_moves_loop - 1)];
      const pool_unit *from_pool = pool + (size_t)pf_max(src, 0) * P.frame_units;
      const pool_unit *from_new = fresh + (size_t)pf_max(-src - 1, 0) * new_frame_units;
#pragma unroll
      for (int u = 0; u < POOL_UNITS_PER_THREAD; ++u) r[b][u] = src >= 0 ? from_pool[unit_c[u]] : from_new[fresh_off[u]];
    }
#pragma unroll
    for (int b = 0; b < POOL_MOVE_BATCH; ++b) {
      if (m0 + b < n_moves_loop) {
        pool_unit *dp = pool + (size_t)s_move_dst[m0 + b] * P.frame_units;
#pragma unroll
        for (int u = 0; u < POOL_UNITS_PER_THREAD; ++u)
          if (valid[u]) dp[unit_c[u]] = r[b][u];
      }
    }
  }

  if (P.n_new <= POOL_PREFETCH) {
    auto put = [&](int j, const pool_unit &a, const pool_unit &b) {
      const int d = j < P.n_new ? s_dest[n_old + j] : -1;
      if (d >= 0) {
        pool_unit *dp = pool + (size_t)d * P.frame_units;
        if (valid[0]) dp[unit_c[0]] = a;
        if (valid[1]) dp[unit_c[1]] = b;
      }
    };
    put(0, nf00, nf01);
    put(1, nf10, nf11);
    put(2, nf20, nf21);
    put(3, nf30, nf31);
  }

  // ---- tables: written by the last workgroup of this head to arrive, after every workgroup of the
  // head has read the old tables.  Each workgroup consumed the old tables (the plan above was computed from
  // them) before it signals its arrival, and nobody reads the new tables or the payload before the kernel
  // ends, so the arrival needs no memory fence (a device-scope release here would write back the die's
  // whole L2 once per workgroup).  The arrival comes after the payload on purpose: atomics and loads return
  // in order, so an early arrival would hold up the loads behind the atomics.  Every head's counter sits in a
  // cache line of its own (PF_SYNC_STRIDE), so the arrivals of different heads do not queue behind each other. ----
#if PF_STRICT_FENCES
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
#endif
  __syncthreads();
  if (tid == 0) {
#if PF_STRICT_FENCES
    const int arrived = __hip_atomic_fetch_add(&P.sync[h * PF_SYNC_STRIDE], 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
#else
    const int arrived = atomicAdd(&P.sync[h * PF_SYNC_STRIDE], 1);
#endif
    s_last = (arrived == 2 * P.blocks_per_head - 1) ? 1 : 0;
  }
  __syncthreads();
  if (!s_last) return;
  const int slots = pol.slots;
  for (int j = tid; j < n_cand; j += POOL_THREADS) {
    const int d = s_dest[j];
    if (d >= 0) {
      P.frame_ids[base + d] = s_id[j];
      P.frame_score[base + d] = s_score[j];
    }
  }
  for (int j = n_kept + tid; j < slots && j < n_cand; j += POOL_THREADS) {   // slots freed by this append
    P.frame_ids[base + j] = -1;
    P.frame_score[base + j] = 0.0f;
  }
  if (tid == 0) {
    P.n_frames[h] = n_kept;
    P.sync[h * PF_SYNC_STRIDE] = 0;
    if (h == 0) *P.T_dev = T_new;
  }
}

// ---------------------------------------------------------------------------------------------------
// Veil cache merging (Sec. 4.2): after an append, rebuild the merged frames of every Veil head that
// has them.  Window j (0 = nearest) of head h covers frames w0 .. w0+m-1 with w0 = T-R-(j+1)m and goes to the
// head's slot slots-1-j; row r of the merged frame is token `tok` of frame w0+i, where (i, tok) runs over
// i = 0..m-1 and, inside i, over the tokens congruent to i modulo m.  The sources are found in closed form:
// a head's resident raw frames are its sink frames followed by the ids lo .. T-1, lo = max(S, T-R-cap*m).
// grid: (16-byte units of a frame / 256, heads * max_cap, K|V).
// ---------------------------------------------------------------------------------------------------
struct PoolMergeParams {
  uint4 *k_pool, *v_pool;
  const pf_head_policy *policy;
  const int32_t *slot_base;
  int32_t *frame_ids;
  float *frame_score;
  int T, tpf, row_units, frame_units, max_cap;
};

__global__ __launch_bounds__(POOL_THREADS) void pf_pool_merge_kernel(PoolMergeParams P) {
  const int h = blockIdx.y / P.max_cap, j = blockIdx.y % P.max_cap;
  const pf_head_policy pol = P.policy[h];
  if (pol.type != PF_VEIL || j >= pol.cap) return;
  const int m = pol.period;
  const int w0 = P.T - pol.recent - (j + 1) * m;
  const bool exists = w0 >= pol.sink;
  const int base = P.slot_base[h];
  const int dst_slot = base + pol.slots - 1 - j;
  if (blockIdx.x == 0 && blockIdx.z == 0 && threadIdx.x == 0) {
    P.frame_ids[dst_slot] = exists ? (PF_MERGED_FRAME | w0) : -1;
    P.frame_score[dst_slot] = 0.0f;
  }
  if (!exists) return;
  const int u = blockIdx.x * POOL_THREADS + threadIdx.x;
  if (u >= P.frame_units) return;
  const int r = u / P.row_units, c = u - r * P.row_units;
  // row r -> (i, tok): subset i holds the tokens i, i+m, i+2m, ... below tpf
  int i = 0, first = 0;
  for (; i < m; ++i) {
    const int n_i = (P.tpf - i + m - 1) / m;
    if (r < first + n_i) break;
    first += n_i;
  }
  const int tok = (r - first) * m + i;
  const int f = w0 + i;
  const int n_sink = pf_min(pol.sink, P.T);
  const int lo = pf_max(pol.sink, P.T - pol.recent - pol.cap * m);
  const int src_slot = base + (f < pol.sink ? f : n_sink + (f - lo));
  uint4 *pool = blockIdx.z ? P.v_pool : P.k_pool;
  pool[(size_t)dst_slot * P.frame_units + u] = pool[(size_t)src_slot * P.frame_units + (size_t)tok * P.row_units + c];
}

extern "C" int pf_pool_reset(pf_pool *pool, void *stream) {
  const int rc = pf_validate_pool(pool);
  if (rc != PF_OK) return rc;
  const long long n_sync = (long long)pool->n_heads * PF_SYNC_STRIDE;
  const long long n = pool->total_slots > n_sync ? pool->total_slots : n_sync;
  const int threads = 256;
  const unsigned blocks = (unsigned)((n + threads - 1) / threads);
  hipLaunchKernelGGL(pf_pool_reset_kernel, dim3(blocks), dim3(threads), 0, (hipStream_t)stream, pool->n_frames,
                     pool->frame_ids, pool->frame_score, pool->T_dev, pool->sync, pool->n_heads, pool->total_slots);
  PF_HIP_CHECK(hipGetLastError());
  pool->T_host = 0;
  return PF_OK;
}

static int cache_append_impl(pf_pool *pool, const void *k_new, const void *v_new, int n_new, const float *scores,
                             const pf_chunk_layout *layout, void *stream) {
  const int rc = pf_validate_pool(pool);
  if (rc != PF_OK) return rc;
  if (!k_new || !v_new || n_new < 1) return PF_ERR_INVALID_ARG;
  if (n_new <= (1 << 20) && !pf_chunk_layout_ok(layout, pool->n_heads, n_new * pool->tokens_per_frame, pool->head_dim))
    return PF_ERR_INVALID_ARG;
  if ((((uintptr_t)k_new) & 15u) || (((uintptr_t)v_new) & 15u)) return PF_ERR_INVALID_ARG;
  if ((long long)pool->T_host + n_new > (1ll << 30)) return PF_ERR_INVALID_ARG;
  const int T_new = pool->T_host + n_new;
  for (int h = 0; h < pool->n_heads; ++h) {
    const pf_head_policy &p = pool->policy_host[h];
    if (pf_ret_count_impl(p, T_new) > p.slots - pf_veil_merged_slots(p)) return PF_ERR_CAPACITY;
    if (pf_ret_count_impl(p, pool->T_host) + n_new > POOL_MAX_CAND) return PF_ERR_CAPACITY;
  }
  // heads with cache merging need a second launch; its grid is checked before the first one is enqueued, so a
  // call that fails leaves host and device state as they were
  int max_cap = 0;
  for (int h = 0; h < pool->n_heads; ++h) max_cap = pf_max(max_cap, pf_veil_merged_slots(pool->policy_host[h]));
  if ((long long)pool->n_heads * max_cap > 65535) return PF_ERR_UNSUPPORTED;
  PoolAppendParams P;
  P.k_pool = (uint4 *)pool->k_pool;
  P.v_pool = (uint4 *)pool->v_pool;
  P.k_new = (const uint4 *)k_new;
  P.v_new = (const uint4 *)v_new;
  P.scores = scores;
  P.policy = pool->policy_dev;
  P.slot_base = pool->slot_base;
  P.n_frames = pool->n_frames;
  P.frame_ids = pool->frame_ids;
  P.frame_score = pool->frame_score;
  P.T_dev = pool->T_dev;
  P.sync = pool->sync;
  P.T = pool->T_host;
  P.n_new = n_new;
  P.frame_units = pool->tokens_per_frame * pool->head_dim / 8;   // bf16: 8 elements per 16 bytes
  P.blocks_per_head = pf_ceil_div(P.frame_units, POOL_CHUNK_UNITS);
  P.row_shift = pool->head_dim == 128 ? 4 : 3;
  P.new_tok_units = layout ? layout->token_stride / 8 : (1 << P.row_shift);
  P.new_head_units = layout ? layout->head_stride / 8 : (long long)n_new * P.frame_units;
  hipLaunchKernelGGL(pf_pool_append_kernel, dim3(P.blocks_per_head, pool->n_heads, 2), dim3(POOL_THREADS), 0,
                     (hipStream_t)stream, P);
  PF_HIP_CHECK(hipGetLastError());
  // heads with cache merging: a second launch rebuilds their merged frames from the frames just packed
  if (max_cap > 0) {
    PoolMergeParams M;
    M.k_pool = (uint4 *)pool->k_pool;
    M.v_pool = (uint4 *)pool->v_pool;
    M.policy = pool->policy_dev;
    M.slot_base = pool->slot_base;
    M.frame_ids = pool->frame_ids;
    M.frame_score = pool->frame_score;
    M.T = T_new;
    M.tpf = pool->tokens_per_frame;
    M.row_units = pool->head_dim / 8;
    M.frame_units = P.frame_units;
    M.max_cap = max_cap;
    hipLaunchKernelGGL(pf_pool_merge_kernel, dim3(pf_ceil_div(P.frame_units, POOL_THREADS), pool->n_heads * max_cap, 2),
                       dim3(POOL_THREADS), 0, (hipStream_t)stream, M);
    PF_HIP_CHECK(hipGetLastError());
  }
  pool->T_host = T_new;
  return PF_OK;
}

extern "C" int pf_cache_append(pf_pool *pool, const void *k_new, const void *v_new, int n_new,
                               const float *scores, void *stream) {
  return cache_append_impl(pool, k_new, v_new, n_new, scores, nullptr, stream);
}

extern "C" int pf_cache_append_strided(pf_pool *pool, const void *k_new, const void *v_new, int n_new,
                                       const float *scores, const pf_chunk_layout *layout, void *stream) {
  if (!layout) return PF_ERR_INVALID_ARG;
  return cache_append_impl(pool, k_new, v_new, n_new, scores, layout, stream);
}
