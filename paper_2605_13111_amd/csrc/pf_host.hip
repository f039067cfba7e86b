// Host-side validation, sizing and planning of libpf.so (no kernels in this file).
#include <stdlib.h>
#include <string.h>
#include <algorithm>
#include <functional>
#include <mutex>
#include <queue>
#include <unordered_map>
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

// ---- process-wide tuning switches ---------------------------------------------------------------
// Defaults come from the environment (PF_ATTN_VARIANT, PF_ATTN_QUEUE, PF_SEG_TILES, PF_PLAN_UNIFORM), read once at
// first use; pf_set_tuning changes them afterwards.  Plain ints: a change races with calls running on other threads.
namespace {
struct Tuning {
  int attn_variant, attn_queue, seg_tiles, plan_uniform;
};
int env_int(const char *name, int dflt) {
  const char *e = getenv(name);
  return e ? atoi(e) : dflt;
}
Tuning &tuning() {
  static Tuning t = {env_int("PF_ATTN_VARIANT", PF_DEFAULT_VARIANT), env_int("PF_ATTN_QUEUE", 1),
                     env_int("PF_SEG_TILES", 0), getenv("PF_PLAN_UNIFORM") ? 1 : 0};
  return t;
}
}  // namespace

extern "C" int pf_set_tuning(int attn_variant, int attn_queue, int seg_tiles, int plan_uniform) {
  if (attn_variant >= PF_NUM_VARIANTS || seg_tiles > (1 << 20)) return PF_ERR_INVALID_ARG;
  Tuning &t = tuning();
  if (attn_variant >= 0) t.attn_variant = attn_variant;
  if (attn_queue >= 0) t.attn_queue = attn_queue != 0;
  if (seg_tiles >= 0) t.seg_tiles = seg_tiles;
  if (plan_uniform >= 0) t.plan_uniform = plan_uniform != 0;
  return PF_OK;
}

int pf_tuned_seg_tiles() { return tuning().seg_tiles > 0 ? tuning().seg_tiles : 0; }

int pf_resolve_seg_tiles(int seg_tiles) {
  if (seg_tiles <= 0) {
    seg_tiles = pf_tuned_seg_tiles();
    if (seg_tiles <= 0) seg_tiles = PF_DEFAULT_SEG_TILES;
  }
  return seg_tiles < PF_MIN_SEG_TILES ? PF_MIN_SEG_TILES : seg_tiles;
}

// ---- automatic segment lengths ------------------------------------------------------------------
// The launch is a list of blocks, one per (head, key segment, query tile); block i belongs to die i % 8.
//   * one block per workgroup (kernel 0): the hardware sends block i to die i % 8, and a die starts its next
//     block on the first compute unit that frees up;
//   * work queue (kernel 1): one resident workgroup per compute unit takes the next block of its die's list, and
//     from the next die's list once its own is empty.
// With three or four blocks per compute unit the finish time depends strongly on how the blocks pack, so the
// plan is chosen by replaying the schedule on the host (costs: one key tile = 1, a fixed cost per block, an
// extra cost when a partial result has to be parked, and for a head's last segment the cost of reading back
// every partial it merges; the constants are fitted to per-layer timings of every candidate) and keeping
// the shortest finish:
//   1. one segment length for every head, from a list of candidates;
//   2. starting from that, heads with the same key count try every segment count of their own while the
//      others stay fixed, a few rounds (pools of up to PF_PLAN_HEADS heads).
// Plans are remembered per (key tiles of every head, query tiles, kernel, mode) in a hash table large enough for
// whole rollouts, so a step whose shape has been seen before pays a lookup.
static const int kSegCandidates[] = {48, 56, 64, 72, 80, 96, 112, 128, 144, 160, 176, 192, 224, 256, 320, 384};
constexpr int PF_AUTO_MIN_SEG = 48;                 // shortest planned segment: bounds the partial-result workspace
struct PlanCosts {
  double block, split, merge;                       // per block; per parked partial; per partial read back by the merging block
};
static const PlanCosts kCostsDirect = {8.0, 2.0, 2.0};
static const PlanCosts kCostsQueue = {4.0, 2.0, 3.0};
constexpr int PF_PLAN_ROUNDS = 3;
constexpr int PF_PLAN_MAX_NSEG = 16;                // segment counts tried per head in step 2
constexpr double PF_PLAN_MIN_GAIN = 0.01;           // step 2 must beat step 1 by this much to be used
constexpr size_t PF_PLAN_CACHE = 16384;            // remembered plans (about 300 bytes each)

// Finish time of the launch in which head h has key tiles n_kvt[h] cut into segments of at most seg[h] tiles.
static double model_finish(const std::vector<int> &n_kvt, const std::vector<int> &seg, int n_qt, int slots_per_die,
                           bool queue) {
  typedef std::priority_queue<double, std::vector<double>, std::greater<double> > MinHeap;
  const PlanCosts &C = queue ? kCostsQueue : kCostsDirect;
  const int H = (int)n_kvt.size();
  // heads by descending segment length (ties: head id), as the index kernel ranks them
  std::vector<int> order(H), nsegs(H), len(H);
  for (int h = 0; h < H; ++h) {
    order[h] = h;
    nsegs[h] = pf_max(1, pf_ceil_div(n_kvt[h], seg[h]));
    len[h] = pf_ceil_div(n_kvt[h], nsegs[h]);
  }
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return len[a] > len[b]; });
  // per die: the cost of each team (n_qt equal blocks), in launch order
  std::vector<std::vector<double> > teams(PF_NUM_XCD);
  int k = 0;                                         // team rank, as in the index kernel
  for (int o = 0; o < H; ++o) {
    const int nk = n_kvt[order[o]], nseg = nsegs[order[o]];
    for (int sgi = 0; sgi < nseg; ++sgi, ++k) {
      const int row = k / PF_NUM_XCD, col = k % PF_NUM_XCD;
      const int xcd = (row & 1) ? PF_NUM_XCD - 1 - col : col;
      // the merge falls to whichever segment arrives last; the replay charges it to the last one launched
      teams[xcd].push_back(pf_seg_begin(nk, nseg, sgi + 1) - pf_seg_begin(nk, nseg, sgi) + C.block +
                           (nseg > 1 ? C.split : 0.0) + (nseg > 1 && sgi == nseg - 1 ? C.merge * nseg : 0.0));
    }
  }
  double finish = 0.0;
  if (!queue) {
    for (int x = 0; x < PF_NUM_XCD; ++x) {
      MinHeap cu;
      for (int c = 0; c < slots_per_die; ++c) cu.push(0.0);
      for (size_t t = 0; t < teams[x].size(); ++t)
        for (int q = 0; q < n_qt; ++q) {
          const double e = cu.top() + teams[x][t];
          cu.pop();
          cu.push(e);
          finish = e > finish ? e : finish;
        }
    }
    return finish;
  }
  // work queue: the worker that frees up first takes the next block of its die's list, else of the next die's
  typedef std::pair<double, int> Worker;             // (time it is free, home die)
  std::priority_queue<Worker, std::vector<Worker>, std::greater<Worker> > workers;
  for (int w = 0; w < PF_NUM_XCD * slots_per_die; ++w) workers.push(Worker(0.0, w % PF_NUM_XCD));
  size_t next[PF_NUM_XCD] = {};
  while (!workers.empty()) {
    const Worker w = workers.top();
    workers.pop();
    for (int hop = 0; hop < PF_NUM_XCD; ++hop) {
      const int x = (w.second + hop) % PF_NUM_XCD;
      if (next[x] < teams[x].size() * (size_t)n_qt) {
        const double e = w.first + teams[x][next[x] / n_qt];
        ++next[x];
        finish = e > finish ? e : finish;
        workers.push(Worker(e, w.second));
        break;
      }
    }
  }
  return finish;
}

namespace {
// Remembered plans: key = key tiles of every head, then query tiles, then kernel / launch form / planning depth.
// Sized for whole rollouts (30 layers x a few hundred history lengths each have their own key); emptied when full.
struct KeyHash {
  size_t operator()(const std::vector<int> &k) const {
    unsigned long long h = 1469598103934665603ull;
    for (size_t i = 0; i < k.size(); ++i) h = (h ^ (unsigned)k[i]) * 1099511628211ull;
    return (size_t)h;
  }
};
std::mutex g_plan_mutex;
std::unordered_map<std::vector<int>, PfSegPlan, KeyHash> g_plan_cache;
}  // namespace

void pf_auto_plan(const pf_pool *pool, int T, int q_tokens, int variant, bool queue, PfSegPlan *plan) {
  const int H = pool->n_heads;
  const int n_qt = pf_ceil_div(q_tokens, pf_variant_bq(variant));
  const int slots_per_die = 32 * (variant == 0 ? 2 : 1);          // workgroups resident per die
  memset(plan, 0, sizeof(*plan));
  plan->uniform = PF_DEFAULT_SEG_TILES;
  std::vector<int> key(H + 2);
  long long total = 0;
  for (int h = 0; h < H; ++h) {
    const int nsel = pf_sel_count_impl(pool->policy_host[h], T);
    key[h] = pf_ceil_div(nsel * pool->tokens_per_frame + q_tokens, PF_BK);
    total += pf_ceil_div(key[h], PF_AUTO_MIN_SEG);
  }
  if (total * n_qt > 50000) return;                               // keep the replay cheap on huge launches
  const bool uniform_only = H > PF_PLAN_HEADS || tuning().plan_uniform != 0;
  key[H] = n_qt;
  key[H + 1] = variant * 4 + (queue ? 2 : 0) + (uniform_only ? 1 : 0);
  {
    std::lock_guard<std::mutex> lock(g_plan_mutex);
    auto hit = g_plan_cache.find(key);
    if (hit != g_plan_cache.end()) {
      *plan = hit->second;
      return;
    }
  }
  const std::vector<int> n_kvt(key.begin(), key.begin() + H);

  // Many candidate lengths cut the heads into the same segment counts: the replay runs once per distinct cut.
  std::unordered_map<std::vector<int>, double, KeyHash> seen;
  std::vector<int> cut(H);
  auto finish_of = [&](const std::vector<int> &seg) {
    for (int h = 0; h < H; ++h) cut[h] = pf_max(1, pf_ceil_div(n_kvt[h], seg[h]));
    auto f = seen.find(cut);
    if (f != seen.end()) return f->second;
    const double t = model_finish(n_kvt, seg, n_qt, slots_per_die, queue);
    seen.emplace(cut, t);
    return t;
  };

  // step 1: one length for all
  std::vector<int> seg(H);
  double best_t = 0.0;
  for (size_t ci = 0; ci < sizeof(kSegCandidates) / sizeof(kSegCandidates[0]); ++ci) {
    std::fill(seg.begin(), seg.end(), kSegCandidates[ci]);
    const double t = finish_of(seg);
    if (best_t == 0.0 || t < best_t * 0.995) {       // a longer segment must win clearly: it costs fewer partials
      best_t = best_t == 0.0 ? t : (t < best_t ? t : best_t);
      plan->uniform = kSegCandidates[ci];
    }
  }
  std::fill(seg.begin(), seg.end(), plan->uniform);
  const double uniform_t = finish_of(seg);

  // step 2: per key count, the segment count of its own
  if (!uniform_only) {
    std::vector<int> distinct(n_kvt);
    std::sort(distinct.begin(), distinct.end());
    distinct.erase(std::unique(distinct.begin(), distinct.end()), distinct.end());
    double cur_t = uniform_t;
    for (int round = 0; round < PF_PLAN_ROUNDS; ++round) {
      bool changed = false;
      for (size_t d = 0; d < distinct.size(); ++d) {
        const int nk = distinct[d];
        int cur_seg = 0;
        for (int h = 0; h < H; ++h)
          if (n_kvt[h] == nk) cur_seg = seg[h];
        int best_seg = cur_seg;
        for (int n = 1; n <= PF_PLAN_MAX_NSEG; ++n) {
          const int cand = pf_ceil_div(nk, n);
          if (cand < PF_AUTO_MIN_SEG && n > 1) break;
          if (cand == cur_seg) continue;
          for (int h = 0; h < H; ++h)
            if (n_kvt[h] == nk) seg[h] = pf_max(cand, PF_AUTO_MIN_SEG);
          const double t = finish_of(seg);
          if (t < cur_t * 0.998) {
            cur_t = t;
            best_seg = pf_max(cand, PF_AUTO_MIN_SEG);
          }
        }
        for (int h = 0; h < H; ++h)
          if (n_kvt[h] == nk) seg[h] = best_seg;
        changed = changed || best_seg != cur_seg;
      }
      if (!changed) break;
    }
    if (cur_t < uniform_t * (1.0 - PF_PLAN_MIN_GAIN)) {
      plan->per_head = 1;
      for (int h = 0; h < H; ++h) plan->seg[h] = (uint16_t)pf_min(seg[h], 65535);
    }
  }

  std::lock_guard<std::mutex> lock(g_plan_mutex);
  if (g_plan_cache.size() >= PF_PLAN_CACHE) g_plan_cache.clear();
  g_plan_cache.emplace(key, *plan);
}

bool pf_attn_queue_mode(int variant) { return variant >= 1 && tuning().attn_queue != 0; }

int pf_resolve_variant(int head_dim) {
  int v = tuning().attn_variant;
  if (v < 0 || v >= PF_NUM_VARIANTS) v = PF_DEFAULT_VARIANT;
  return head_dim == 128 ? v : 0;                   // the pipelined kernels exist for head_dim 128 only
}

void pf_host_plan(const pf_pool *pool, int T, int q_tokens, int variant, const PfSegPlan &plan,
                  int *n_teams, int *n_blocks, int *n_partials, int *max_sel_needed) {
  const int n_qt = pf_ceil_div(q_tokens, pf_variant_bq(variant));
  long long teams = 0, parts = 0;
  int max_sel = 0;
  for (int h = 0; h < pool->n_heads; ++h) {
    const int nsel = pf_sel_count_impl(pool->policy_host[h], T);
    max_sel = pf_max(max_sel, nsel);
    const PfHeadPlan hp = pf_plan_head(nsel * pool->tokens_per_frame + q_tokens, plan.of(h));
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
    worst_case(pool, q_tokens, pf_tuned_seg_tiles() ? pf_resolve_seg_tiles(0) : PF_AUTO_MIN_SEG, v, &mb, &mp, &n_qt);
    const size_t t = (size_t)mp * pf_partial_bytes(pf_variant_bq(v), pool->head_dim);
    need = t > need ? t : need;
  }
  return pf_align_up(need + 256, 256);
}

extern "C" int pf_plan_segments(const pf_pool *pool, int T, int q_tokens, int32_t *seg_tiles, int32_t *n_blocks,
                                int32_t *n_partials) {
  if (pf_validate_pool(pool) != PF_OK || T < 0 || q_tokens < 1 || q_tokens > (1 << 24)) return PF_ERR_INVALID_ARG;
  for (int h = 0; h < pool->n_heads; ++h)
    if (pf_sel_count_impl(pool->policy_host[h], T) > pool->policy_host[h].slots) return PF_ERR_INVALID_ARG;
  const int variant = pf_resolve_variant(pool->head_dim);
  PfSegPlan plan;
  if (pf_tuned_seg_tiles()) {
    memset(&plan, 0, sizeof(plan));
    plan.uniform = pf_resolve_seg_tiles(0);
  } else {
    pf_auto_plan(pool, T, q_tokens, variant, pf_attn_queue_mode(variant), &plan);
  }
  int teams, blocks, partials, max_sel;
  pf_host_plan(pool, T, q_tokens, variant, plan, &teams, &blocks, &partials, &max_sel);
  if (seg_tiles)
    for (int h = 0; h < pool->n_heads; ++h) seg_tiles[h] = plan.of(h);
  if (n_blocks) *n_blocks = blocks;
  if (n_partials) *n_partials = partials;
  return PF_OK;
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
