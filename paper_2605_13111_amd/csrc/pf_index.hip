// Frame-index build: per-head frame selection (Sec. 4.2), boundary indices of the flattened ragged
// history (Sec. 4.3) and the launch plan of the attention kernel.  One small launch per layer.
#include <stdlib.h>
#include <string.h>
#include "pf_internal.h"

constexpr int INDEX_THREADS = 256;
constexpr int INDEX_STAGE_SLOTS = 4096;     // pool slots whose tables are staged in LDS

struct IndexParams {
  const pf_head_policy *policy;
  const int32_t *slot_base, *n_frames, *frame_ids;
  const float *frame_score;
  int32_t *sel_count, *sel_frames, *sel_slots, *cu_seqlens;
  PfWorkHeader *header;
  int32_t *counters, *scratch;
  PfWorkItem *items;
  long long total_slots;
  int n_heads, T, tpf, max_sel, q_tokens, n_qt, bq, variant;
  int host_teams, host_blocks, host_partials;
  PfSegPlan plan;
};

// Does head `p` attend to resident frame f (history length T)?  `rank` = number of resident
// intermediate frames that beat f by score (needed for TOPK only).
__device__ __forceinline__ bool frame_selected(const pf_head_policy &p, int T, int f, int rank) {
  if (f < p.sink || f >= T - p.recent) return true;            // shared sink / forced recent frames
  const int mid = pf_middle_count(T, p.sink, p.recent);
  if (p.type == PF_ANCHOR) {
    if (p.mode == PF_MODE_ALL || p.cap <= 0 || mid <= p.cap) return true;
    if (p.mode == PF_MODE_TOPK) return rank < p.cap;
    // strided window centres (Eq. 4): offsets (mid-1) - floor(i*mid/cap) - floor(mid/(2cap))
    const int off = f - p.sink;
    const int half = mid / (2 * p.cap);
    for (int i = 0; i < p.cap; ++i) {
      const int pick = (mid - 1) - (int)(((long long)i * mid) / p.cap) - half;
      if (pick == off) return true;
      if (pick < off) break;                                    // picks decrease with i
    }
    return false;
  }
  if (p.type == PF_WAVE) {
    const int dist = T - f;                                     // Eq. 5: f = T - i*P
    if (dist % p.period != 0) return false;
    if (p.cap <= 0) return true;
    const int i = dist / p.period;
    return i - (p.recent / p.period + 1) < p.cap;               // the cap nearest intermediate picks
  }
  return false;                                                 // Veil
}

__global__ __launch_bounds__(INDEX_THREADS) void pf_build_index_kernel(IndexParams P) {
  __shared__ int32_t s_nseg[PF_MAX_HEADS];
  __shared__ int32_t s_nkvt[PF_MAX_HEADS];
  __shared__ int32_t s_team0[PF_MAX_HEADS];     // first team rank of the head (teams sorted by length)
  __shared__ int32_t s_part0[PF_MAX_HEADS];     // first partial slot of the head, -1 if unsplit
  __shared__ int32_t s_selcount[PF_MAX_HEADS];
  __shared__ int32_t s_ids[INDEX_STAGE_SLOTS];
  __shared__ float s_scores[INDEX_STAGE_SLOTS];
  __shared__ int32_t s_error;
  const int tid = threadIdx.x;
  if (tid == 0) s_error = 0;
  __syncthreads();

  // ---- stage the pool tables in LDS (one coalesced pass) so the per-head walks below do not pay a
  // global-memory round trip per frame; pools with more slots than fit are read in place ----
  const bool staged = P.total_slots <= INDEX_STAGE_SLOTS;
  if (staged) {
    for (int i = tid; i < (int)P.total_slots; i += INDEX_THREADS) {
      s_ids[i] = P.frame_ids[i];
      s_scores[i] = P.frame_score[i];
    }
  }
  for (int i = tid; i < P.n_heads * P.max_sel; i += INDEX_THREADS) {     // unused entries read -1
    P.sel_frames[i] = -1;
    P.sel_slots[i] = -1;
  }
  __syncthreads();
  const int32_t *ids = staged ? s_ids : P.frame_ids;
  const float *scores = staged ? s_scores : P.frame_score;

  // ---- selection: one wave per head, one lane per resident frame (ascending ids, 64 at a time); a lane
  // decides whether its frame is attended, the wave compacts the survivors with a ballot ----
  const int lane = tid & 63, wave = tid >> 6;
  for (int h = wave; h < P.n_heads; h += INDEX_THREADS / 64) {
    const pf_head_policy pol = P.policy[h];
    const int base = P.slot_base[h];
    const int n_res = P.n_frames[h];
    const int mid_lo = pol.sink, mid_hi = P.T - pol.recent;
    const bool need_rank = pol.type == PF_ANCHOR && pol.mode == PF_MODE_TOPK && pol.cap > 0 &&
                           pf_middle_count(P.T, pol.sink, pol.recent) > pol.cap;
    // Veil heads with cache merging: their merged frames (kept in the last slots of the region) stand between
    // the sink and the recent frames in the key sequence, oldest window first
    const int n_win = pf_veil_windows(pol, P.T);
    int n = 0;
    for (int j0 = 0; j0 < n_res; j0 += 64) {
      const int j = j0 + lane;
      bool sel = false;
      int f = -1;
      if (j < n_res) {
        f = ids[base + j];
        int rank = 0;
        if (need_rank && f >= mid_lo && f < mid_hi) {
          const float sc = scores[base + j];
          for (int g = 0; g < n_res; ++g) {
            const int fg = ids[base + g];
            if (fg < mid_lo || fg >= mid_hi) continue;
            const float sg = scores[base + g];
            rank += (sg > sc || (sg == sc && fg < f)) ? 1 : 0;
          }
        }
        sel = frame_selected(pol, P.T, f, rank);
      }
      const unsigned long long mask = __builtin_amdgcn_ballot_w64(sel);
      const int pos = n + __builtin_popcountll(mask & ((1ull << lane) - 1ull)) + (f >= pol.sink ? n_win : 0);
      if (sel && pos < P.max_sel) {
        P.sel_frames[(size_t)h * P.max_sel + pos] = f;
        P.sel_slots[(size_t)h * P.max_sel + pos] = base + j;
      }
      n += __builtin_popcountll(mask);
    }
    if (lane < n_win) {                                           // window j = lane, 0 = nearest
      const int pos = pf_min(pol.sink, P.T) + (n_win - 1 - lane);
      if (pos < P.max_sel) {
        P.sel_frames[(size_t)h * P.max_sel + pos] = PF_MERGED_FRAME | (P.T - pol.recent - (lane + 1) * pol.period);
        P.sel_slots[(size_t)h * P.max_sel + pos] = base + pol.slots - 1 - lane;
      }
    }
    n += n_win;
    if (lane == 0) {
      P.sel_count[h] = n;
      s_selcount[h] = n;
      // The host sized the launch from the closed-form count; a mismatch means the pool does not hold
      // what the policy asks for (it was not filled through pf_cache_append).
      if (n != pf_sel_count_impl(pol, P.T) || n > P.max_sel) atomicExch(&s_error, 1);
      const PfHeadPlan hp = pf_plan_head(n * P.tpf + P.q_tokens, P.plan.of(h));
      s_nseg[h] = hp.nseg;
      s_nkvt[h] = hp.n_kvt;
    }
  }
  for (int i = tid; i < P.n_heads * P.n_qt + PF_QUEUE_INTS; i += INDEX_THREADS) P.counters[i] = 0;
  __syncthreads();

  // ---- boundaries (exclusive prefix sum, batch-head order) and per-head plan offsets ----
  if (tid == 0) {
    int cu = 0, parts = 0;
    P.cu_seqlens[0] = 0;
    for (int h = 0; h < P.n_heads; ++h) {
      cu += s_selcount[h] * P.tpf;
      P.cu_seqlens[h + 1] = cu;
      s_part0[h] = s_nseg[h] > 1 ? parts : -1;
      if (s_nseg[h] > 1) parts += s_nseg[h] * P.n_qt;
    }
    P.header->n_partials = parts;
    if (parts != P.host_partials) s_error = 1;
  }
  // team order: heads by descending segment length (ties: head id), a head's segments consecutive
  for (int h = tid; h < P.n_heads; h += INDEX_THREADS) {
    const int len_h = pf_ceil_div(s_nkvt[h], s_nseg[h]);
    int first = 0;
    for (int g = 0; g < P.n_heads; ++g) {
      const int len_g = pf_ceil_div(s_nkvt[g], s_nseg[g]);
      if (len_g > len_h || (len_g == len_h && g < h)) first += s_nseg[g];
    }
    s_team0[h] = first;
  }
  __syncthreads();
  int n_teams = 0;
  for (int h = 0; h < P.n_heads; ++h) n_teams += s_nseg[h];
  const int n_blocks = pf_ceil_div(n_teams, PF_NUM_XCD) * PF_NUM_XCD * P.n_qt;
  if (tid == 0) {
    if (n_teams != P.host_teams || n_blocks != P.host_blocks) s_error = 1;
    P.header->n_blocks = P.host_blocks;
    P.header->n_teams = n_teams;
    P.header->n_qt = P.n_qt;
    P.header->variant = P.variant;
    P.header->seg_tiles = P.plan.per_head ? 0 : P.plan.uniform;
    P.header->q_tokens = P.q_tokens;
  }
  for (int b = tid; b < P.host_blocks; b += INDEX_THREADS) P.items[b].head = -1;
  __syncthreads();
  if (tid == 0) P.header->error = s_error;
  if (s_error) return;                           // leave an all-empty plan: the attention launch does nothing

  // ---- items: team k runs on die xcd(k) (boustrophedon over the sorted teams, so the dies' loads
  // stay level); its query tiles are consecutive in that die's queue, so they stream the same keys
  // through the die's L2 at the same time ----
  for (int h = 0; h < P.n_heads; ++h) {
    const int nseg = s_nseg[h], n_kvt = s_nkvt[h];
    for (int e = tid; e < nseg * P.n_qt; e += INDEX_THREADS) {
      const int s = e / P.n_qt, qi = e - s * P.n_qt;
      const int k = s_team0[h] + s;
      const int row = k / PF_NUM_XCD, col = k % PF_NUM_XCD;
      const int xcd = (row & 1) ? PF_NUM_XCD - 1 - col : col;
      PfWorkItem it;
      it.head = h;
      it.q0 = qi * P.bq;
      it.kt0 = pf_seg_begin(n_kvt, nseg, s);
      it.kt1 = pf_seg_begin(n_kvt, nseg, s + 1);
      it.nseg = nseg;
      it.seg = s;
      it.part0 = nseg > 1 ? s_part0[h] + qi : -1;
      it.group = h * P.n_qt + qi;
      P.items[(size_t)(row * P.n_qt + qi) * PF_NUM_XCD + xcd] = it;
    }
  }
}

extern "C" int pf_build_index(const pf_pool *pool, pf_index *index, int q_tokens, void *stream) {
  const int rc = pf_validate_pool(pool);
  if (rc != PF_OK) return rc;
  if (!index || q_tokens < 1 || q_tokens > (1 << 24)) return PF_ERR_INVALID_ARG;
  if (!index->sel_count || !index->sel_frames || !index->sel_slots || !index->cu_seqlens || !index->work)
    return PF_ERR_INVALID_ARG;
  if (index->max_sel < 1 || index->max_sel > PF_MAX_SEL) return PF_ERR_INVALID_ARG;
  if (((uintptr_t)index->work) & 15u) return PF_ERR_INVALID_ARG;
  if (index->seg_tiles < 0) return PF_ERR_INVALID_ARG;

  const int variant = pf_resolve_variant(pool->head_dim);
  // segment lengths: the caller's, else the PF_SEG_TILES override, else planned for this launch
  const bool fixed = index->seg_tiles > 0 || pf_tuned_seg_tiles() > 0;
  PfSegPlan plan;
  if (fixed) {
    memset(&plan, 0, sizeof(plan));
    plan.uniform = pf_resolve_seg_tiles(index->seg_tiles);
  } else {
    pf_auto_plan(pool, pool->T_host, q_tokens, variant, pf_attn_queue_mode(variant), &plan);
  }
  int n_teams, n_blocks, n_partials, max_sel_needed;
  pf_host_plan(pool, pool->T_host, q_tokens, variant, plan, &n_teams, &n_blocks, &n_partials, &max_sel_needed);
  if (max_sel_needed > index->max_sel) return PF_ERR_CAPACITY;
  const int n_qt = pf_ceil_div(q_tokens, pf_variant_bq(variant));
  const PfWorkLayout L = pf_work_layout(pool->n_heads, n_qt, n_blocks);
  if (L.total > index->work_bytes) return PF_ERR_CAPACITY;

  char *w = (char *)index->work;
  IndexParams P;
  P.policy = pool->policy_dev;
  P.slot_base = pool->slot_base;
  P.n_frames = pool->n_frames;
  P.frame_ids = pool->frame_ids;
  P.frame_score = pool->frame_score;
  P.sel_count = index->sel_count;
  P.sel_frames = index->sel_frames;
  P.sel_slots = index->sel_slots;
  P.cu_seqlens = index->cu_seqlens;
  P.header = (PfWorkHeader *)w;
  P.counters = (int32_t *)(w + L.counters_off);
  P.scratch = (int32_t *)(w + L.scratch_off);
  P.items = (PfWorkItem *)(w + L.items_off);
  P.total_slots = pool->total_slots;
  P.n_heads = pool->n_heads;
  P.T = pool->T_host;
  P.tpf = pool->tokens_per_frame;
  P.max_sel = index->max_sel;
  P.q_tokens = q_tokens;
  P.n_qt = n_qt;
  P.bq = pf_variant_bq(variant);
  P.plan = plan;
  P.variant = variant;
  P.host_teams = n_teams;
  P.host_blocks = n_blocks;
  P.host_partials = n_partials;
  hipLaunchKernelGGL(pf_build_index_kernel, dim3(1), dim3(INDEX_THREADS), 0, (hipStream_t)stream, P);
  PF_HIP_CHECK(hipGetLastError());
  index->q_tokens = q_tokens;
  index->T_built = pool->T_host;
  index->n_blocks = n_blocks;
  index->n_partials = n_partials;
  index->variant = variant;
  int longest = plan.uniform;
  if (plan.per_head) {
    longest = 0;
    for (int h = 0; h < pool->n_heads; ++h) longest = pf_max(longest, plan.of(h));
  }
  index->longest_seg = fixed ? 0 : longest;
  return PF_OK;
}

extern "C" const int32_t *pf_index_status_dev(const pf_index *index) {
  if (!index || !index->work) return nullptr;
  return &((const PfWorkHeader *)index->work)->error;
}
