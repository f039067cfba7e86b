// Host-side validation, sizing and planning of libpf.so (no kernels in this file).
#include <stdlib.h>
#include <string.h>
#include "pf_internal.h"

static bool aligned16(const void *p) { return (((uintptr_t)p) & 15u) == 0; }

static bool policy_ok(const pf_head_policy &p) {
  if (p.type != PF_ANCHOR && p.type != PF_WAVE && p.type != PF_VEIL) return false;
  if (p.type == PF_ANCHOR && (p.mode < PF_MODE_ALL || p.mode > PF_MODE_TOPK)) return false;
  if (p.sink < 0 || p.recent < 0 || p.cap < 0 || p.slots < 1) return false;
  if (p.type == PF_WAVE && p.period < 1) return false;
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
  // The default segment length bounds the partial count unless the caller asks for shorter segments
  // through pf_index.seg_tiles; pf_ragged_attn_fwd checks the actual need against workspace_bytes.
  size_t need = 0;
  for (int v = 0; v < PF_NUM_VARIANTS; ++v) {
    long long mb, mp;
    int n_qt;
    worst_case(pool, q_tokens, pf_resolve_seg_tiles(0), v, &mb, &mp, &n_qt);
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
