// Internal declarations shared by the translation units of libpf.so (host and device code).
// Nothing here is part of the ABI; the ABI is include/pf.h.
#ifndef PF_INTERNAL_H
#define PF_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>
#include "pf.h"

#define PF_HD __host__ __device__ __forceinline__

// ---- tiling constants of the attention kernel ------------------------------------------------
constexpr int PF_BK = 64;               // keys per tile
constexpr int PF_MIN_SEG_TILES = 16;    // smallest allowed key-tile count per work item
constexpr int PF_DEFAULT_SEG_TILES = 128;
constexpr int PF_MAX_SEL = 1024;        // slot table kept in LDS by the attention kernel
constexpr int PF_MAX_HEADS = 1024;      // one index-kernel thread per head
constexpr int PF_NUM_XCD = 8;           // MI355X: 8 accelerator dies, workgroup i runs on die i % 8
constexpr int PF_NUM_VARIANTS = 3;
constexpr int PF_DEFAULT_VARIANT = 1;   // for head_dim 128; other head sizes always use variant 0

// query rows per workgroup of kernel variant v: 0 = 4 waves x 32 rows, 1 = 8 waves x 32 rows, 2 = 4 waves x 64 rows
PF_HD int pf_variant_bq(int variant) { return variant == 0 ? 128 : 256; }

PF_HD int pf_ceil_div(int a, int b) { return (a + b - 1) / b; }
PF_HD int pf_min(int a, int b) { return a < b ? a : b; }
PF_HD int pf_max(int a, int b) { return a > b ? a : b; }

// ---- closed-form frame counts (Sec. 4.2 policies) ---------------------------------------------
// Number of intermediate ids S .. T-R-1.
PF_HD int pf_middle_count(int T, int S, int R) { return pf_max(0, T - R - S); }

// Number of Wave picks T - i*P (i >= 1) that fall into the intermediate range, before the cap:
// i runs from floor(R/P)+1 (first distance beyond the recent window) to floor((T-S)/P).
PF_HD int pf_wave_middle_picks(int T, int S, int R, int P) {
  if (T - R - S <= 0) return 0;
  const int i_first = R / P + 1;
  const int i_last = (T - S) / P;
  return pf_max(0, i_last - i_first + 1);
}

// Veil cache merging (Sec. 4.2): slots at the end of the head's region that hold merged frames, and the number
// of merged windows (m = period frames each, stacked before the recent frames) that fit into the intermediate
// range at history length T.
PF_HD int pf_veil_merged_slots(const pf_head_policy &p) { return (p.type == PF_VEIL && p.cap > 0) ? p.cap : 0; }
PF_HD int pf_veil_windows(const pf_head_policy &p, int T) {
  if (p.type != PF_VEIL || p.cap <= 0) return 0;
  return pf_min(p.cap, pf_middle_count(T, p.sink, p.recent) / p.period);
}

// Frames head `p` attends to when the history has T frames.
PF_HD int pf_sel_count_impl(const pf_head_policy &p, int T) {
  const int mid = pf_middle_count(T, p.sink, p.recent);
  const int shared = T - mid;   // |sink U recent|
  int typed = 0;
  if (p.type == PF_ANCHOR) {
    typed = (p.mode == PF_MODE_ALL || p.cap <= 0) ? mid : pf_min(mid, p.cap);
  } else if (p.type == PF_WAVE) {
    typed = pf_wave_middle_picks(T, p.sink, p.recent, p.period);
    if (p.cap > 0) typed = pf_min(typed, p.cap);
  } else {
    typed = pf_veil_windows(p, T);                 // one merged frame per window
  }
  return shared + typed;
}

// Oldest id a capped Wave head may still pick at this or any later step.
PF_HD int pf_wave_oldest(const pf_head_policy &p, int T) {
  return T - (p.recent / p.period + p.cap) * p.period;
}

// Frames the pool retains for head `p` when the history has T frames.
PF_HD int pf_ret_count_impl(const pf_head_policy &p, int T) {
  const int mid = pf_middle_count(T, p.sink, p.recent);
  const int shared = T - mid;
  int kept = 0;
  if (p.type == PF_ANCHOR) {
    kept = (p.mode == PF_MODE_TOPK && p.cap > 0) ? pf_min(mid, p.cap) : mid;
  } else if (p.type == PF_WAVE) {
    if (p.cap <= 0) {
      kept = mid;
    } else {
      const int lo = pf_max(p.sink, pf_wave_oldest(p, T));
      kept = pf_max(0, (T - p.recent) - lo);
      kept = pf_min(kept, mid);
    }
  } else if (p.cap > 0) {
    kept = pf_min(mid, p.cap * p.period);          // the sources of this and every later step's windows
  }
  return shared + kept;
}

// ---- launch plan of the attention kernel -------------------------------------------------------
// A head with Lkv keys has n_kvt = ceil(Lkv/PF_BK) key tiles, cut into nseg nearly equal segments of
// at most seg_tiles tiles; segment s covers tiles [s*n_kvt/nseg, (s+1)*n_kvt/nseg).
struct PfHeadPlan {
  int n_kvt;
  int nseg;
};
PF_HD PfHeadPlan pf_plan_head(int lkv, int seg_tiles) {
  PfHeadPlan hp;
  hp.n_kvt = pf_ceil_div(lkv, PF_BK);
  hp.nseg = pf_max(1, pf_ceil_div(hp.n_kvt, seg_tiles));
  return hp;
}
// Segment lengths of a launch: one for every head, or one per head (small pools).
constexpr int PF_PLAN_HEADS = 64;
struct PfSegPlan {
  int32_t uniform;                 // key tiles per work item when per_head == 0
  int32_t per_head;
  uint16_t seg[PF_PLAN_HEADS];
  PF_HD int of(int h) const { return per_head ? (int)seg[h] : uniform; }
};
PF_HD int pf_seg_begin(int n_kvt, int nseg, int s) { return (int)(((long long)s * n_kvt) / nseg); }

// One workgroup's job.  head < 0 = nothing to do.
struct __attribute__((aligned(32))) PfWorkItem {
  int32_t head;
  int32_t q0;          // first query row
  int32_t kt0, kt1;    // key tiles [kt0, kt1)
  int32_t nseg;        // segments of this (head, query tile)
  int32_t seg;         // this item's segment
  int32_t part0;       // partial slot of segment 0 of this (head, query tile); segment s uses part0 + s*n_qt
  int32_t group;       // arrival counter index = head*n_qt + query tile
};

struct __attribute__((aligned(64))) PfWorkHeader {
  int32_t n_blocks;
  int32_t n_teams;
  int32_t n_qt;
  int32_t n_partials;
  int32_t error;       // set by the index kernel when the device disagrees with the host plan
  int32_t variant;
  int32_t seg_tiles;
  int32_t q_tokens;
  int32_t pad[8];
};

// Layout of pf_index.work: header | counters[n_heads*n_qt + PF_QUEUE_INTS] | head scratch[4*n_heads] | items[n_blocks]
// (the last PF_QUEUE_INTS counters are the attention kernel's work-queue tickets)
constexpr int PF_QUEUE_INTS = 16;
struct PfWorkLayout {
  size_t counters_off, scratch_off, items_off, total;
};
static inline size_t pf_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
static inline PfWorkLayout pf_work_layout(int n_heads, int n_qt, long long max_blocks) {
  PfWorkLayout L;
  L.counters_off = sizeof(PfWorkHeader);
  L.scratch_off = pf_align_up(L.counters_off + sizeof(int32_t) * ((size_t)n_heads * n_qt + PF_QUEUE_INTS), 64);
  L.items_off = pf_align_up(L.scratch_off + sizeof(int32_t) * 4 * (size_t)n_heads, 64);
  L.total = L.items_off + sizeof(PfWorkItem) * (size_t)max_blocks;
  return L;
}

// bytes of one partial-result slot: O [bq][D] fp32, then m [bq], l [bq]
PF_HD size_t pf_partial_bytes(int bq, int head_dim) { return (size_t)bq * (head_dim + 2) * sizeof(float); }

// ---- host helpers ---------------------------------------------------------------------------
int pf_validate_pool(const pf_pool *pool);                 // PF_OK or error
bool pf_chunk_layout_ok(const pf_chunk_layout *lay, int n_heads, int tokens, int head_dim);   // null = packed = ok
int pf_resolve_seg_tiles(int seg_tiles);                   // 0 -> default, else clamped to the minimum
int pf_tuned_seg_tiles();                                  // the process-wide segment-length override, 0 = none
int pf_resolve_variant(int head_dim);                      // kernel variant in use
// Segment length that a host replay of the launch schedule finds best for this history length.
void pf_auto_plan(const pf_pool *pool, int T, int q_tokens, int variant, bool queue, PfSegPlan *plan);
bool pf_attn_queue_mode(int variant);                      // does this kernel take its blocks from the work queue?
// Host plan for the pool's current T: per-launch block count and partial count.
void pf_host_plan(const pf_pool *pool, int T, int q_tokens, int variant, const PfSegPlan &plan,
                  int *n_teams, int *n_blocks, int *n_partials, int *max_sel_needed);

#define PF_HIP_CHECK(expr)                         \
  do {                                             \
    hipError_t _e = (expr);                        \
    if (_e != hipSuccess) return PF_ERR_HIP;       \
  } while (0)

#endif  // PF_INTERNAL_H
