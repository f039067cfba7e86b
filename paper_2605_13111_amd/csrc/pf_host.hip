// Host-side validation, sizing and planning of libpf.so (no kernels in this file).
#include <stdlib.h>
#include <string.h>
#include <algorithm>
#include <functional>
#include <queue>
#include <vector>
#include "pf_internal.h"

static bool aligned16(const void *p) { return (((uintptr_t)p) & 15u) == 0; }

static bool policy_ok(const pf_head_policy &p) {
  if (p.type != PF_ANCHOR && p.type != PF_WAVE && p.type != PF_VEIL) return false;
  if (p.type == PF_ANCHOR && (p.mode < PF_MODE_ALL || p.mode > PF_MODE_TOPK)) return false;
  if (p.sink < 0 || p.recent < 0 || p.cap < 0 || p.slots < 1) return false;
  if (p.type == PF_WAVE && p.period < 1) return false;
  if (p.type == PF_VEIL && p.cap > 0 && (p.cap > 64 || p.period < 1 || p.period > 64 || p.slots <= p.cap)) return false;
  return true;
}

int pf_validate_pool(const pf_pool *pool) {
  if (!pool) return PF_ERR_INVALID_ARG;
  if (pool->n_heads < 1 || pool->n_heads > PF_MAX_HEADS) return PF_ERR_INVALID_ARG;
  if (pool->tokens_per_frame < 1 || pool->total_slots < 1) return PF_ERR_INVALID_ARG;
  if (pool->dtype != 0) return PF_ERR_UNSUPPORTED;
  if (pool->head_dim != 64 && pool->head_dim != 128) return PF_ERR_UNSUPPORTED;
  if (!pool->k_pool || !pool->v_pool || !pool->policy_host || !pool->policy_dev || !pool->slot_base ||
      !pool->n_frames || !pool->frame_ids || !pool->frame_score || !pool->T_dev || !pool->sync)
    return PF_ERR_INVALID_ARG;
  if (!aligned16(pool->k_pool) || !aligned16(pool->v_pool)) return PF_ERR_INVALID_ARG;
  if (pool->T_host < 0) return PF_ERR_INVALID_ARG;
  long long total = 0;
  for (int h = 0; h < pool->n_heads; ++h) {
    if (!policy_ok(pool->policy_host[h])) return PF_ERR_INVALID_ARG;
    total += pool->policy_host[h].slots;
  }
  if (total != pool->total_slots) return PF_ERR_INVALID_ARG;
  // token offsets inside one head's key sequence are kept in 32-bit integers
  for (int h = 0; h < pool->n_heads; ++h)
    if ((long long)pool->policy_host[h].slots * pool->tokens_per_frame > (1ll << 30)) return PF_ERR_INVALID_ARG;
  return PF_OK;
}

int pf_resolve_seg_tiles(int seg_tiles) {
  if (seg_tiles <= 0) {
    const char *e = getenv("PF_SEG_TILES");
    seg_tiles = e ? atoi(e) : 0;
    if (seg_tiles <= 0) seg_tiles = PF_DEFAULT_SEG_TILES;
  }
  return seg_tiles < PF_MIN_SEG_TILES ? PF_MIN_SEG_TILES : seg_tiles;
}

// ---- automatic segment length --------------------------------------------------------------------
// The launch is a list of equal-priority blocks, one per (head, key segment, query tile).  Block i goes to
// die i % 8; a die starts its next block on the first compute unit that frees up.  With three or four
// blocks per compute unit the finish time depends strongly on how the block count per die divides by its 32
// compute units, so the segment length is chosen by replaying that schedule on the host for a few
// candidate lengths (costs: one key tile = 1, fixed cost per block, extra cost when a partial result has
// to be parked, and for a head's last segment the cost of reading back every partial it merges) and keeping
// the shortest finish.
static const int kSegCandidates[] = {48, 56, 64, 72, 80, 96, 112, 128, 144, 160, 176, 192, 224, 256, 320, 384};
constexpr int PF_AUTO_MIN_SEG = 48;                 // smallest candidate: bounds the partial-result workspace
constexpr double PF_BLOCK_COST = 8.0;               // set-up + first fetch + store, in key-tile times (fitted to timings)
constexpr double PF_SPLIT_COST = 2.0;               // parking a partial result
constexpr double PF_MERGE_COST = 2.0;               // per partial read back by the merging block (fitted to timings)

static double model_finish(const std::vector<int> &n_kvt, const std::vector<int> &order, int n_qt, int seg_tiles,
                           int slots_per_die) {
  typedef std::priority_queue<double, std::vector<double>, std::greater<double> > MinHeap;
  std::vector<MinHeap> die(PF_NUM_XCD);
  for (int x = 0; x < PF_NUM_XCD; ++x)
    for (int c = 0; c < slots_per_die; ++c) die[x].push(0.0);
  double finish = 0.0;
  int k = 0;                                         // team rank, as in the index kernel
  for (size_t o = 0; o < order.size(); ++o) {
    const int nk = n_kvt[order[o]];
    const int nseg = pf_max(1, pf_ceil_div(nk, seg_tiles));
    for (int sgi = 0; sgi < nseg; ++sgi, ++k) {
      const int row = k / PF_NUM_XCD, col = k % PF_NUM_XCD;
      const int xcd = (row & 1) ? PF_NUM_XCD - 1 - col : col;
      // the merge falls to whichever segment arrives last; the replay charges it to the last one launched
      const double cost = pf_seg_begin(nk, nseg, sgi + 1) - pf_seg_begin(nk, nseg, sgi) + PF_BLOCK_COST +
                          (nseg > 1 ? PF_SPLIT_COST : 0.0) + (nseg > 1 && sgi == nseg - 1 ? PF_MERGE_COST * nseg : 0.0);
      for (int q = 0; q < n_qt; ++q) {
        const double t = die[xcd].top() + cost;
        die[xcd].pop();
        die[xcd].push(t);
        finish = t > finish ? t : finish;
      }
    }
  }
  return finish;
}

int pf_auto_seg_tiles(const pf_pool *pool, int T, int q_tokens, int variant) {
  const int n_qt = pf_ceil_div(q_tokens, pf_variant_bq(variant));
  const int slots_per_die = 32 * (variant == 0 ? 2 : 1);          // workgroups resident per die
  std::vector<int> n_kvt(pool->n_heads);
  long long total = 0;
  for (int h = 0; h < pool->n_heads; ++h) {
    const int nsel = pf_sel_count_impl(pool->policy_host[h], T);
    n_kvt[h] = pf_ceil_div(nsel * pool->tokens_per_frame + q_tokens, PF_BK);
    total += pf_ceil_div(n_kvt[h], PF_AUTO_MIN_SEG);
  }
  if (total * n_qt > 50000) return PF_DEFAULT_SEG_TILES;          // keep the replay cheap on huge launches
  int best = PF_DEFAULT_SEG_TILES;
  double best_t = 0.0;
  std::vector<int> order(pool->n_heads);
  for (size_t ci = 0; ci < sizeof(kSegCandidates) / sizeof(kSegCandidates[0]); ++ci) {
    const int seg = kSegCandidates[ci];
    // heads by descending segment length (ties: head id), as the index kernel ranks them
    for (int h = 0; h < pool->n_heads; ++h) order[h] = h;
    std::vector<int> len(pool->n_heads);
    for (int h = 0; h < pool->n_heads; ++h) len[h] = pf_ceil_div(n_kvt[h], pf_max(1, pf_ceil_div(n_kvt[h], seg)));
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return len[a] > len[b]; });
    const double t = model_finish(n_kvt, order, n_qt, seg, slots_per_die);
    if (best_t == 0.0 || t < best_t * 0.995) {       // a longer segment must win clearly: it costs fewer partials
      best_t = best_t == 0.0 ? t : (t < best_t ? t : best_t);
      best = seg;
    }
  }
  return best;
}

int pf_resolve_variant(int head_dim) {
  const char *e = getenv("PF_ATTN_VARIANT");
  int v = e ? atoi(e) : PF_DEFAULT_VARIANT;
  if (v < 0 || v >= PF_NUM_VARIANTS) v = PF_DEFAULT_VARIANT;
  return head_dim == 128 ? v : 0;                   // kernel 1 exists for head_dim 128 only
}

void pf_host_plan(const pf_pool *pool, int T, int q_tokens, int variant, int seg_tiles,
                  int *n_teams, int *n_blocks, int *n_partials, int *max_sel_needed) {
  const int n_qt = pf_ceil_div(q_tokens, pf_variant_bq(variant));
  long long teams = 0, parts = 0;
  int max_sel = 0;
  for (int h = 0; h < pool->n_heads; ++h) {
    const int nsel = pf_sel_count_impl(pool->policy_host[h], T);
    max_sel = pf_max(max_sel, nsel);
    const PfHeadPlan hp = pf_plan_head(nsel * pool->tokens_per_frame + q_tokens, seg_tiles);
    teams += hp.nseg;
    if (hp.nseg > 1) parts += (long long)hp.nseg * n_qt;
  }
  *n_teams = (int)teams;
  *n_blocks = (int)(pf_ceil_div((int)teams, PF_NUM_XCD) * PF_NUM_XCD * (long long)n_qt);
  *n_partials = (int)parts;
  *max_sel_needed = max_sel;
}

// Worst case over every T the slot capacities allow: a head never selects more frames than it has slots.
static void worst_case(const pf_pool *pool, int q_tokens, int seg_tiles, int variant, long long *max_blocks,
                       long long *max_partials, int *n_qt_out) {
  const int n_qt = pf_ceil_div(q_tokens, pf_variant_bq(variant));
  long long teams = 0, parts = 0;
  for (int h = 0; h < pool->n_heads; ++h) {
    const long long lkv = (long long)pool->policy_host[h].slots * pool->tokens_per_frame + q_tokens;
    const PfHeadPlan hp = pf_plan_head((int)lkv, seg_tiles);
    teams += hp.nseg;
    if (hp.nseg > 1) parts += (long long)hp.nseg * n_qt;
  }
  *max_blocks = (teams + PF_NUM_XCD - 1) / PF_NUM_XCD * PF_NUM_XCD * n_qt;
  *max_partials = parts;
  *n_qt_out = n_qt;
}

extern "C" size_t pf_index_work_bytes(const pf_pool *pool, int q_tokens) {
  if (pf_validate_pool(pool) != PF_OK || q_tokens < 1) return 0;
  size_t need = 0;
  for (int v = 0; v < PF_NUM_VARIANTS; ++v) {
    long long mb, mp;
    int n_qt;
    worst_case(pool, q_tokens, PF_MIN_SEG_TILES, v, &mb, &mp, &n_qt);
    const size_t t = pf_work_layout(pool->n_heads, n_qt, mb).total;
    need = t > need ? t : need;
  }
  return need;
}

extern "C" size_t pf_attn_workspace_bytes(const pf_pool *pool, int q_tokens) {
  if (pf_validate_pool(pool) != PF_OK || q_tokens < 1) return 0;
  // The shortest automatic segment length (or the PF_SEG_TILES override) bounds the partial count unless the
  // caller asks for shorter segments through pf_index.seg_tiles; pf_ragged_attn_fwd checks the actual need
  // against workspace_bytes.
  size_t need = 0;
  for (int v = 0; v < PF_NUM_VARIANTS; ++v) {
    long long mb, mp;
    int n_qt;
    worst_case(pool, q_tokens, getenv("PF_SEG_TILES") ? pf_resolve_seg_tiles(0) : PF_AUTO_MIN_SEG, v, &mb, &mp, &n_qt);
    const size_t t = (size_t)mp * pf_partial_bytes(pf_variant_bq(v), pool->head_dim);
    need = t > need ? t : need;
  }
  return pf_align_up(need + 256, 256);
}

extern "C" int pf_selected_count(const pf_head_policy *pol, int T) {
  if (!pol || T < 0 || !policy_ok(*pol)) return PF_ERR_INVALID_ARG;
  return pf_sel_count_impl(*pol, T);
}

extern "C" int pf_retained_count(const pf_head_policy *pol, int T) {
  if (!pol || T < 0 || !policy_ok(*pol)) return PF_ERR_INVALID_ARG;
  return pf_ret_count_impl(*pol, T);
}

extern "C" const char *pf_status_string(int status) {
  switch (status) {
    case PF_OK: return "ok";
    case PF_ERR_INVALID_ARG: return "invalid argument";
    case PF_ERR_CAPACITY: return "capacity exceeded";
    case PF_ERR_UNSUPPORTED: return "unsupported head_dim or dtype";
    case PF_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}
