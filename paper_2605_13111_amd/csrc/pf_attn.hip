// Ragged-cache attention forward (Sec. 4.3; Eq. 1 per head over [selected frames || chunk]).
//
// One launch per layer.  A work item is BQ query rows of one head and a run of 64-key tiles of that
// head's ragged key sequence; heads with many keys are cut into several runs whose partial results are
// merged by the last workgroup to finish (no spinning).  pf_attn_kernel runs one item per workgroup;
// pf_attn_pp_kernel keeps one workgroup per compute unit resident and lets it take items from per-die queues
// until all are empty.  Two kernels share the operand layouts below:
//   pf_attn_kernel     BQ = 128, 4 waves x 32 query rows, two workgroups per CU, tiles staged through
//                      registers into padded LDS rows; any head_dim in {64, 128}
//   pf_attn_pp_kernel  BQ = 256, 8 waves x 32 query rows in two groups that alternate between a matrix phase
//                      and a vector phase, tiles copied global -> LDS directly; head_dim 128 (the default there)
//
// Per tile, on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulate):
//   S^T = K . Q^T     A operand = K rows from LDS, B operand = Q^T held in registers
//   O^T += V^T . P^T  A operand = V^T via the LDS transpose read, B operand = P^T straight from the
//                     S^T accumulators (the key permutation of the accumulator layout is applied to
//                     the V rows instead, since a sum over keys has no order)
// so every lane owns ONE query column: the running maximum and sum of the online softmax live in
// one register each and need a single exchange with lane^32 per tile.
#include <stddef.h>
#include <stdlib.h>
#include "pf_internal.h"
#ifndef PF_STRICT_FENCES
#define PF_STRICT_FENCES 0
#endif
#include <mutex>
#include <utility>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;   // 16-byte register quad
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

constexpr int ATT_THREADS = 256;
constexpr int ATT_WAVES = 4;
// Exponent headroom (log2 units) a score may have over the reference maximum before the accumulators
// must be rescaled: weights stay below 2^8 (fp32 and bf16 share the 8-bit exponent, so both hold such
// weights without loss of relative precision).
constexpr float ATT_LAZY_LOG2 = 8.0f;

struct AttnParams {
  const __bf16 *q, *k_cur, *v_cur, *k_pool, *v_pool;
  __bf16 *out;
  const int32_t *sel_count, *sel_slots;
  const PfWorkItem *items;
  int32_t *counters;
  int32_t *tickets;     // work-queue mode: next entry of each die's queue [PF_NUM_XCD], then the count of workgroups done; null = one item per workgroup
  float *workspace;
  int max_sel, tpf, q_tokens, n_qt, queue_len;
  float scale_log2;     // softmax scale * log2(e)
  // chunk tensors (q, k_cur, v_cur, out): element strides between tokens of a head and between heads
  // (packed [heads][tokens][D]: D and q_tokens*D; the model's [tokens][heads][D]: heads*D and D)
  long long tok_stride, head_stride;
  // optional diagnostics (pf_set_block_trace): per resident workgroup {busy, first start, last end, items, busy shader cycles}, in ticks of the
  // constant 100 MHz clock; null = off
  long long *block_trace;
};

template <class T>
__device__ __forceinline__ T *as_global(T *p) {
  return (T *)(__attribute__((address_space(1))) T *)(unsigned long long)p;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// max / sum with the lane that holds the other half of the same query column (lane ^ 32)
__device__ __forceinline__ float partner_max(float x) {
  const int xi = __float_as_int(x);
  auto r = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
  return fmaxf(__int_as_float(r[0]), __int_as_float(r[1]));
}
__device__ __forceinline__ float partner_sum(float x) {
  const int xi = __float_as_int(x);
  auto r = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
  return __int_as_float(r[0]) + __int_as_float(r[1]);
}

// Partial results cross workgroups that may run on different dies, each with its own L2.  They are written
// and read with device-scope (relaxed atomic) accesses, which go through to the memory side that all dies
// share; no L2 write-back fence is needed, only the wait for the stores' completion before the arrival
// counter is bumped.  Building with -DPF_STRICT_FENCES=1 adds the release fence the memory model asks for in
// front of every arrival (here and in the pool append): the known-correct form, measured against this one.
__device__ __forceinline__ void st_dev2(float *p, float a, float b) {
  const unsigned long long v = (unsigned long long)__float_as_uint(a) | ((unsigned long long)__float_as_uint(b) << 32);
  __hip_atomic_store((unsigned long long *)p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 ld_dev2(const float *p) {
  const unsigned long long v = __hip_atomic_load((const unsigned long long *)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return make_float2(__uint_as_float((unsigned)v), __uint_as_float((unsigned)(v >> 32)));
}
__device__ __forceinline__ void st_dev1(float *p, float a) {
  __hip_atomic_store(p, a, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_dev1(const float *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---------------------------------------------------------------------------------------------------
// Tile addressing.  A head's key sequence is [selected frame 0 | selected frame 1 | ... | chunk]; frames
// sit anywhere in the pool (slot table), the chunk in k_cur / v_cur.  Tiles of 64 keys ignore frame borders.
// ---------------------------------------------------------------------------------------------------
struct TilePos {   // where a tile's first key lives: frame index (n_sel = the chunk) and offset in it
  int j, r;
};
__device__ __forceinline__ TilePos tile_pos_init(int kt, int hist_tokens, int n_sel, int tpf) {
  TilePos p;
  const int t0 = kt * PF_BK;
  if (t0 >= hist_tokens) { p.j = n_sel; p.r = t0 - hist_tokens; }
  else { p.j = t0 / tpf; p.r = t0 - p.j * tpf; }
  return p;
}
__device__ __forceinline__ void tile_pos_advance(TilePos &p, int n_sel, int tpf) {
  p.r += PF_BK;
  if (p.j < n_sel) {
    if (tpf >= PF_BK) { if (p.r >= tpf) { p.r -= tpf; ++p.j; } }
    else { const int adv = p.r / tpf; p.r -= adv * tpf; p.j += adv; }
    if (p.j > n_sel) { p.r += (p.j - n_sel) * tpf; p.j = n_sel; }
  }
}

struct HeadKV {     // everything a loader thread needs to find keys of one head
  const __bf16 *k_pool, *v_pool, *k_cur, *v_cur;
  // slot table of the head: written by the index kernel before this launch and constant during it, so it is
  // read through the constant address space (wave-uniform indices become scalar loads, which do not queue
  // behind outstanding vector-memory operations)
  const __attribute__((address_space(4))) int32_t *slots;
  int n_sel, tpf, hist_tokens, lkv;
  int lrow, lchunk;
  unsigned thread_off;
  long long cur_stride;   // elements between consecutive chunk tokens in k_cur / v_cur
};

// Global -> register load of one 64-key tile of one tensor.  Common case (tile inside one frame, no ragged
// tail): one wave-uniform base pointer plus a per-thread constant offset.  Otherwise every row is located
// on its own (branch-free: both candidate addresses, then a select).
template <int D, int NP, int RPP>
__device__ __forceinline__ void attn_load_rows(u32x4 (&reg)[NP], int kt, TilePos pos, const HeadKV &H, const __bf16 *pool,
                                               const __bf16 *cur) {
  constexpr unsigned PASS_BYTES = RPP * D * 2;
  const int last = H.lkv - 1 - kt * PF_BK;
  const bool in_hist = pos.j < H.n_sel;
  const bool simple = last >= PF_BK - 1 && (!in_hist || pos.r + PF_BK <= H.tpf);
  if (__builtin_expect(simple && (in_hist || H.cur_stride == D), 1)) {
    const char *b = in_hist ? (const char *)(pool + ((size_t)H.slots[pos.j] * H.tpf + pos.r) * D)
                            : (const char *)(cur + (size_t)pos.r * D);
#pragma unroll
    for (int p = 0; p < NP; ++p) reg[p] = *(const u32x4 *)(b + (H.thread_off + p * PASS_BYTES));
  } else if (simple) {                              // whole chunk tile, token rows apart by the caller's stride
    const __bf16 *b = cur + (size_t)pos.r * H.cur_stride + H.lchunk * 8;
#pragma unroll
    for (int p = 0; p < NP; ++p) reg[p] = *(const u32x4 *)(b + (size_t)(H.lrow + p * RPP) * H.cur_stride);
  } else {
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      const int t = kt * PF_BK + pf_min(H.lrow + p * RPP, last);    // rows past the end re-read the last key
      const bool in_chunk = t >= H.hist_tokens;
      const int th = in_chunk ? 0 : t;
      const int j = th / H.tpf;
      const size_t e_hist = ((size_t)pf_max(H.slots[j], 0) * H.tpf + (th - j * H.tpf)) * D;
      const size_t e = in_chunk ? (size_t)(t - H.hist_tokens) * H.cur_stride : e_hist;
      const __bf16 *b = in_chunk ? cur : pool;
      reg[p] = *(const u32x4 *)(b + e + H.lchunk * 8);
    }
  }
}

template <int NP, int RPP, int STRIDE>
__device__ __forceinline__ void attn_store_rows(const u32x4 (&reg)[NP], __bf16 *dst, int lrow, int lchunk) {
#pragma unroll
  for (int p = 0; p < NP; ++p) *(u32x4 *)(&dst[(lrow + p * RPP) * STRIDE + lchunk * 8]) = reg[p];
}

// Where a tile's rows come from, for the direct global -> LDS copies of the two-group kernel.
struct TileSrc {
  bool simple;            // tile inside one frame (or the chunk) and not ragged: base + row * stride
  bool strided;           // simple chunk tile whose rows are cur_stride elements apart instead of D
  bool split;             // whole tile made of two dense runs: rows below n1 end one frame, the others start the next
                          // frame (or the packed chunk); never together with simple
  const __bf16 *kb, *vb;  // first row of the tile (simple case); of the first run (split case)
  const __bf16 *kb2, *vb2; // split case: where row 0 of the tile WOULD sit if the second run began there (second run's
                          // first row minus n1 rows), so that both runs are addressed by the row number in the tile
  int n1;                 // split case: rows of the first run, 1 .. 63
  int kt;
};
__device__ __forceinline__ TileSrc tile_src(int kt, TilePos pos, const HeadKV &H, int D) {
  TileSrc t;
  const int last = H.lkv - 1 - kt * PF_BK;
  const bool in_hist = pos.j < H.n_sel;
  t.simple = last >= PF_BK - 1 && (!in_hist || pos.r + PF_BK <= H.tpf);
  t.strided = !in_hist && H.cur_stride != D;
  t.kt = kt;
  // a whole history tile that crosses exactly one border: frames of at least a tile, and the next run (a frame, or the
  // chunk with rows D apart) holds the rest of the tile
  t.n1 = H.tpf - pos.r;
  t.split = !t.simple && in_hist && last >= PF_BK - 1 && H.tpf >= PF_BK && t.n1 > 0 && t.n1 < PF_BK &&
            (pos.j + 1 < H.n_sel || H.cur_stride == D);
  size_t e = 0;
  if (t.simple) e = in_hist ? ((size_t)H.slots[pos.j] * H.tpf + pos.r) * D : (size_t)pos.r * H.cur_stride;
  if (t.split) e = ((size_t)H.slots[pos.j] * H.tpf + pos.r) * D;
  t.kb = (in_hist ? H.k_pool : H.k_cur) + e;
  t.vb = (in_hist ? H.v_pool : H.v_cur) + e;
  t.kb2 = t.kb;
  t.vb2 = t.vb;
  if (t.split) {
    const bool next_hist = pos.j + 1 < H.n_sel;
    const long long e2 = (next_hist ? (long long)H.slots[pos.j + 1] * H.tpf * D : 0ll) - (long long)t.n1 * D;
    t.kb2 = (next_hist ? H.k_pool : H.k_cur) + e2;
    t.vb2 = (next_hist ? H.v_pool : H.v_cur) + e2;
  }
  return t;
}
// V^T operand of O^T += V^T P^T for 16 keys x 32 channels: two LDS transpose reads whose row choice
// (4g+r and 8+4g+r) reproduces the key order of the S^T accumulator registers.
template <int VS>
__device__ __forceinline__ bf16x8 read_vt(const __bf16 *vp) {
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(vp));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(vp + 8 * VS));
  const s16x8 av = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, av);
}

// ---------------------------------------------------------------------------------------------------
// The rescaling ("classic") loop over key tiles [kt0, kt1): load tile -> S^T -> online softmax with
// running-maximum rescaling -> O^T.  Used by pf_attn_kernel.
// ---------------------------------------------------------------------------------------------------
template <int D, int NQB>
__device__ __forceinline__ void classic_loop(const HeadKV &H, int kt0, int kt1, const bf16x8 (&qf)[NQB][D / 16],
                                             f32x16 (&o)[NQB][D / 32], float (&m_run)[NQB], float (&l_run)[NQB],
                                             __bf16 (*sK)[PF_BK * (D + 8)], __bf16 (*sV)[PF_BK * (D + 32)], float c) {
  constexpr int BK = PF_BK;
  constexpr int KS = D + 8;            // K row stride in LDS (elements): +16 B so 32 rows spread over banks
  constexpr int VS = D + 32;           // V row stride: +64 B so the 4 rows of one transpose read do not collide
  constexpr int CPR = D / 8, RPP = ATT_THREADS / CPR, NP = BK / RPP;
  constexpr int NKS = D / 16, NDB = D / 32, NKB = BK / 32, NS16 = BK / 16;
  const int lane = threadIdx.x & 63;
  const int l32 = lane & 31, g = lane >> 5;
  const int k_lane = l32 * KS + 8 * g;                                           // K operand: row l32, d 8g..
  const int v_lane = (4 * g + ((lane & 15) >> 2)) * VS + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  const float thr = ATT_LAZY_LOG2 / c;

  u32x4 kreg[NP], vreg[NP];
  TilePos pos = tile_pos_init(kt0, H.hist_tokens, H.n_sel, H.tpf);
  attn_load_rows<D, NP, RPP>(kreg, kt0, pos, H, H.k_pool, H.k_cur);
  attn_load_rows<D, NP, RPP>(vreg, kt0, pos, H, H.v_pool, H.v_cur);
  attn_store_rows<NP, RPP, KS>(kreg, sK[0], H.lrow, H.lchunk);
  attn_store_rows<NP, RPP, VS>(vreg, sV[0], H.lrow, H.lchunk);
  __syncthreads();

  int buf = 0;
  for (int kt = kt0; kt < kt1; ++kt) {
    const bool more = kt + 1 < kt1;
    if (__builtin_expect(more, 1)) {
      tile_pos_advance(pos, H.n_sel, H.tpf);
      attn_load_rows<D, NP, RPP>(kreg, kt + 1, pos, H, H.k_pool, H.k_cur);
      attn_load_rows<D, NP, RPP>(vreg, kt + 1, pos, H, H.v_pool, H.v_cur);
    }

    // ---- S^T = K Q^T ----
    f32x16 s[NQB][NKB];
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
        for (int i = 0; i < 16; ++i) s[qb][kb][i] = 0.0f;
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) {
        const bf16x8 a = *(const bf16x8 *)(&sK[buf][k_lane + kb * 32 * KS + ks * 16]);
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb)
          s[qb][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[qb][ks], s[qb][kb], 0, 0, 0);
      }
    }
    // ragged tail: keys at or beyond lkv exist only in the last tile of the head
    const int valid = H.lkv - kt * BK;
    if (__builtin_expect(valid < BK, 0)) {
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int key = kb * 32 + 8 * (i >> 2) + 4 * g + (i & 3);
          if (key >= valid) {
#pragma unroll
            for (int qb = 0; qb < NQB; ++qb) s[qb][kb][i] = -INFINITY;
          }
        }
    }

    // ---- online softmax (per lane: one query column).  The reference maximum m_run only moves when a row's
    // tile maximum exceeds it by more than thr: exp2 arguments stay small and the accumulators are
    // rescaled on a few early tiles only. ----
    bf16x8 pf[NQB][NS16];
    float mx[NQB];
    bool need = false;
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      float a = s[qb][0][0];
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) a = fmaxf(a, s[qb][kb][i]);
      mx[qb] = partner_max(a);
      need = need || (mx[qb] > m_run[qb] + thr);
    }
    if (__builtin_expect(__builtin_amdgcn_ballot_w64(need) != 0, 0)) {
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
        const float m_new = fmaxf(m_run[qb], mx[qb]);
        const float alpha = fast_exp2((m_run[qb] - m_new) * c);
        m_run[qb] = m_new;
        l_run[qb] *= alpha;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[qb][db][i] *= alpha;
      }
    }
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      const float mc = m_run[qb] * c;
      // row sum with plain fp32 adds: dot-product instructions share the matrix pipe and queue behind MFMAs
      float ls0 = 0.f, ls1 = 0.f;
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
          const float e0 = fast_exp2(fmaf(s[qb][kb][i], c, -mc));
          const float e1 = fast_exp2(fmaf(s[qb][kb][i + 1], c, -mc));
          ls0 += e0;
          ls1 += e1;
          pf[qb][kb * 2 + (i >> 3)][i & 7] = (__bf16)e0;
          pf[qb][kb * 2 + (i >> 3)][(i & 7) + 1] = (__bf16)e1;
        }
      l_run[qb] += ls0 + ls1;
    }

    // ---- O^T += V^T P^T ----
#pragma unroll
    for (int s16 = 0; s16 < NS16; ++s16) {
#pragma unroll
      for (int db = 0; db < NDB; ++db) {
        const bf16x8 a = read_vt<VS>(&sV[buf][v_lane + s16 * 16 * VS + db * 32]);
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb)
          o[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[qb][s16], o[qb][db], 0, 0, 0);
      }
    }

    if (more) {
      attn_store_rows<NP, RPP, KS>(kreg, sK[buf ^ 1], H.lrow, H.lchunk);
      attn_store_rows<NP, RPP, VS>(vreg, sV[buf ^ 1], H.lrow, H.lchunk);
    }
    __syncthreads();
    buf ^= 1;
  }
}

// ---------------------------------------------------------------------------------------------------
// Final normalisation and store.  Unsplit heads write bf16 output directly; split heads park the
// unnormalised partial (O, m, l) and the last segment to arrive merges all partials of its (head, query tile).
// The accumulators hold O^T (one query column per lane); they go through LDS once so that every global
// access of the epilogue is a full row segment: 16 bytes per lane, consecutive lanes consecutive addresses.
// sStage: attn_stage_floats(BQ, D) floats of LDS that no wave reads any more (all passed the loop's last barrier).
// ---------------------------------------------------------------------------------------------------
constexpr int attn_stage_floats(int bq, int d) { return bq * (d + 4) + 2 * bq; }

// 16-byte device-scope store: written through to the memory all dies share (see st_dev2).
__device__ __forceinline__ void st_dev4(float *p, f32x4 v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc1" : : "v"(p), "v"(v) : "memory");
}

template <int D, int NQB, int NWAVES = ATT_WAVES>
__device__ __forceinline__ void attn_epilogue(const AttnParams &P, const PfWorkItem &it, f32x16 (&o)[NQB][D / 32],
                                              float (&m_run)[NQB], float (&l_run)[NQB], float *sStage, int32_t *sFlagp,
                                              int tid) {
  constexpr int BQ = NWAVES * 32 * NQB;
  constexpr int NT = NWAVES * 64;
  constexpr int NDB = D / 32;
  constexpr int LD = D + 4;                        // row stride of the staged tile: 16-byte writes of 16 rows hit all banks
  const int lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const int h = it.head;
  const float c = P.scale_log2;
  float *sO = sStage;                              // [BQ][LD]
  float *sM = sStage + BQ * LD, *sL = sM + BQ;     // [BQ] each

  // ---- accumulators -> LDS rows ----
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const int lrow_q = (wave * NQB + qb) * 32 + l32;
    const float lsum = partner_sum(l_run[qb]);
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4)
        *(float4 *)(sO + lrow_q * LD + db * 32 + 8 * i4 + 4 * g) =
            make_float4(o[qb][db][i4 * 4], o[qb][db][i4 * 4 + 1], o[qb][db][i4 * 4 + 2], o[qb][db][i4 * 4 + 3]);
    if (g == 0) { sM[lrow_q] = m_run[qb]; sL[lrow_q] = lsum; }
  }
  __syncthreads();

  __bf16 *oh = P.out + (size_t)h * P.head_stride;
  if (it.nseg == 1) {
    for (int e = tid; e < BQ * (D / 8); e += NT) {
      const int r = e / (D / 8), d0 = (e % (D / 8)) * 8;
      const int row = it.q0 + r;
      if (row >= P.q_tokens) continue;
      const float inv = 1.0f / sL[r];
      const float4 a = *(const float4 *)(sO + r * LD + d0), b = *(const float4 *)(sO + r * LD + d0 + 4);
      bf16x8 w;
      w[0] = (__bf16)(a.x * inv); w[1] = (__bf16)(a.y * inv); w[2] = (__bf16)(a.z * inv); w[3] = (__bf16)(a.w * inv);
      w[4] = (__bf16)(b.x * inv); w[5] = (__bf16)(b.y * inv); w[6] = (__bf16)(b.z * inv); w[7] = (__bf16)(b.w * inv);
      *(bf16x8 *)(oh + (size_t)row * P.tok_stride + d0) = w;
    }
    return;
  }

  // ---- split head: park the unnormalised partial (O, m, l), the last segment to arrive merges ----
  const size_t part_floats = (size_t)BQ * (D + 2);
  {
    float *po = P.workspace + (size_t)(it.part0 + it.seg * P.n_qt) * part_floats;
    float *pm = po + (size_t)BQ * D;                // m[BQ] then l[BQ]
    for (int e = tid; e < BQ * (D / 4); e += NT) {
      const int r = e / (D / 4), d0 = (e % (D / 4)) * 4;
      st_dev4(po + (size_t)r * D + d0, *(const f32x4 *)(sO + r * LD + d0));
    }
    for (int e = tid; e < 2 * BQ; e += NT) st_dev1(pm + e, sM[e]);      // sM and sL are adjacent
  }
  __builtin_amdgcn_s_waitcnt(0);             // this wave's partial stores have completed
#if PF_STRICT_FENCES
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");   // the memory model's own publication: release before the arrival
#endif
  __syncthreads();
  if (tid == 0) {
#if PF_STRICT_FENCES
    const int arrived = __hip_atomic_fetch_add(&P.counters[it.group], 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
#else
    const int arrived = atomicAdd(&P.counters[it.group], 1);
#endif
    *sFlagp = (arrived == it.nseg - 1) ? 1 : 0;
    if (*sFlagp) P.counters[it.group] = 0;     // ready for the next launch on this index
  }
  __syncthreads();
  if (!*sFlagp) return;

  // ---- merge.  The other segments' stores went through to memory before their arrival was counted; what
  // this die's L2 may still hold of these addresses is older (the workspace is reused by every launch), so
  // the L2 copies are dropped first (acquire at device scope: an invalidate, no write-back) and the partials
  // are then read with ordinary wide loads.
  // Phase A: per query row, the maximum M over the segments' reference maxima and the total denominator
  // L = sum_s 2^((m_s-M)c) l_s.  Phase B: out = sum_s 2^((m_s-M)c) O_s / L. ----
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  float *sInvL = sL;
  const float *base = P.workspace + (size_t)it.part0 * part_floats;
  const size_t seg_stride = (size_t)P.n_qt * part_floats;
  const int nseg = it.nseg;
  for (int r = tid; r < BQ; r += NT) {
    const float *pm = base + (size_t)BQ * D + r;
    float mmax = -3.0e38f;
#pragma unroll 8
    for (int sgi = 0; sgi < nseg; ++sgi) mmax = fmaxf(mmax, pm[sgi * seg_stride]);
    float lsum = 0.0f;
#pragma unroll 8
    for (int sgi = 0; sgi < nseg; ++sgi) lsum += fast_exp2((pm[sgi * seg_stride] - mmax) * c) * pm[sgi * seg_stride + BQ];
    sM[r] = mmax;
    sInvL[r] = 1.0f / lsum;
  }
  __syncthreads();
  constexpr int EG = 4;                                        // 8-channel output groups per thread in flight
  static_assert((BQ * (D / 8)) % (NT * EG) == 0, "merge tiling");
  for (int e0 = tid; e0 < BQ * (D / 8); e0 += NT * EG) {
    int r[EG], d0[EG];
    float mrow[EG];
    float4 acc[EG][2];
#pragma unroll
    for (int k = 0; k < EG; ++k) {
      const int e = e0 + k * NT;
      r[k] = e / (D / 8);
      d0[k] = (e % (D / 8)) * 8;
      mrow[k] = sM[r[k]];
      acc[k][0] = acc[k][1] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll 2
    for (int sgi = 0; sgi < nseg; ++sgi) {
      const float *ps = base + sgi * seg_stride;
#pragma unroll
      for (int k = 0; k < EG; ++k) {
        const float w = fast_exp2((ps[(size_t)BQ * D + r[k]] - mrow[k]) * c);
        const float4 va = *(const float4 *)(ps + (size_t)r[k] * D + d0[k]);
        const float4 vb = *(const float4 *)(ps + (size_t)r[k] * D + d0[k] + 4);
        acc[k][0].x += w * va.x; acc[k][0].y += w * va.y; acc[k][0].z += w * va.z; acc[k][0].w += w * va.w;
        acc[k][1].x += w * vb.x; acc[k][1].y += w * vb.y; acc[k][1].z += w * vb.z; acc[k][1].w += w * vb.w;
      }
    }
#pragma unroll
    for (int k = 0; k < EG; ++k) {
      const int row = it.q0 + r[k];
      if (row >= P.q_tokens) continue;
      const float inv = sInvL[r[k]];
      bf16x8 w;
      w[0] = (__bf16)(acc[k][0].x * inv); w[1] = (__bf16)(acc[k][0].y * inv);
      w[2] = (__bf16)(acc[k][0].z * inv); w[3] = (__bf16)(acc[k][0].w * inv);
      w[4] = (__bf16)(acc[k][1].x * inv); w[5] = (__bf16)(acc[k][1].y * inv);
      w[6] = (__bf16)(acc[k][1].z * inv); w[7] = (__bf16)(acc[k][1].w * inv);
      *(bf16x8 *)(oh + (size_t)row * P.tok_stride + d0[k]) = w;
    }
  }
}

// ---------------------------------------------------------------------------------------------------
// Common set-up of a workgroup: its work item, the head's key layout, its Q^T fragments.
// ---------------------------------------------------------------------------------------------------
template <int D>
__device__ __forceinline__ void attn_setup_head(const AttnParams &P, const PfWorkItem &it, HeadKV &H, int tid) {
  constexpr int CPR = D / 8;
  const int h = it.head;
  H.n_sel = P.sel_count[h];
  H.tpf = P.tpf;
  H.hist_tokens = H.n_sel * P.tpf;
  H.lkv = H.hist_tokens + P.q_tokens;
  H.k_pool = P.k_pool;
  H.v_pool = P.v_pool;
  H.k_cur = P.k_cur + (size_t)h * P.head_stride;
  H.v_cur = P.v_cur + (size_t)h * P.head_stride;
  H.cur_stride = P.tok_stride;
  H.slots = (const __attribute__((address_space(4))) int32_t *)(P.sel_slots + (size_t)h * P.max_sel);
  H.lrow = tid / CPR;
  H.lchunk = tid % CPR;
  H.thread_off = (unsigned)((H.lrow * D + H.lchunk * 8) * 2);
}
// Q^T fragments: lane (l32, g) holds, for its query row, d = 16*ks + 8*g .. +7
template <int D, int NQB>
__device__ __forceinline__ void attn_load_q(const AttnParams &P, const PfWorkItem &it, bf16x8 (&qf)[NQB][D / 16], int tid) {
  const int lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const __bf16 *qh = P.q + (size_t)it.head * P.head_stride;
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const int row = pf_min(it.q0 + (wave * NQB + qb) * 32 + l32, P.q_tokens - 1);
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) qf[qb][ks] = *(const bf16x8 *)(qh + (size_t)row * P.tok_stride + ks * 16 + 8 * g);
  }
}
template <int D, int NQB>
__device__ __forceinline__ void attn_setup(const AttnParams &P, const PfWorkItem &it, HeadKV &H, bf16x8 (&qf)[NQB][D / 16]) {
  attn_setup_head<D>(P, it, H, threadIdx.x);
  attn_load_q<D, NQB>(P, it, qf, threadIdx.x);
}

template <int D, int NQB>
__device__ __forceinline__ void attn_zero(f32x16 (&o)[NQB][D / 32], float (&m_run)[NQB], float (&l_run)[NQB]) {
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    m_run[qb] = -3.0e38f;
    l_run[qb] = 0.0f;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[qb][db][i] = 0.0f;
  }
}

// ---------------------------------------------------------------------------------------------------
// Kernel 0: 32 query rows per wave, two workgroups per CU.
// ---------------------------------------------------------------------------------------------------
// One work item done with the rescaling loop: set-up, loop, epilogue.
template <int D, int NQB>
__device__ __forceinline__ void attn_item_classic(const AttnParams &P, const PfWorkItem &it,
                                                  __bf16 (*sK)[PF_BK * (D + 8)], __bf16 (*sV)[PF_BK * (D + 32)],
                                                  int32_t *sFlag) {
  HeadKV H;
  bf16x8 qf[NQB][D / 16];
  attn_setup<D, NQB>(P, it, H, qf);
  f32x16 o[NQB][D / 32];
  float m_run[NQB], l_run[NQB];
  attn_zero<D, NQB>(o, m_run, l_run);
  classic_loop<D, NQB>(H, it.kt0, it.kt1, qf, o, m_run, l_run, sK, sV, P.scale_log2);
  attn_epilogue<D, NQB>(P, it, o, m_run, l_run, (float *)&sK[0][0], sFlag, threadIdx.x);
}

template <int D>
__global__ __launch_bounds__(ATT_THREADS, 2) void pf_attn_kernel(AttnParams P) {
  // two K and two V tile buffers; the epilogue reuses the same memory to stage the output rows
  constexpr int K_BYTES = 2 * PF_BK * (D + 8) * 2, V_BYTES = 2 * PF_BK * (D + 32) * 2;
  constexpr int STAGE_BYTES = attn_stage_floats(ATT_WAVES * 32, D) * 4;
  __shared__ __attribute__((aligned(16))) char smem[K_BYTES + V_BYTES > STAGE_BYTES ? K_BYTES + V_BYTES : STAGE_BYTES];
  __shared__ int32_t sFlag;
  const PfWorkItem it = P.items[blockIdx.x];
  if (it.head < 0) return;
  attn_item_classic<D, 1>(P, it, (__bf16 (*)[PF_BK * (D + 8)])smem, (__bf16 (*)[PF_BK * (D + 32)])(smem + K_BYTES), &sFlag);
}

// ---------------------------------------------------------------------------------------------------
// Kernel 1 (default for head_dim 128): 8 waves x 32 query rows (BQ = 256) in two groups of four that alternate between a matrix phase
// and a vector phase.  Waves w and w+4 share a SIMD; group 1 runs one phase behind group 0, so while one
// wave of a SIMD issues the 32 MFMAs of a tile (O^T += V^T P^T of the previous tile, then S^T = K Q^T of
// the current one) the other computes its softmax on the vector ALU.  A workgroup barrier ends every phase
// and keeps the groups in step.
//   phase M(u)   reads K of tile u and V of tile u-1, requests the first V^T fragments of tile u for the next
//                matrix phase and ends with the wait for this wave's copies of tile u+1
//   phase V(u)   sends the copies of tile u+3 into the stages tiles u-1 (K) and u-2 (V) lived in (their last
//                readers, both groups' M(u-1), are two barriers back), plans the copy after that, then scores of
//                tile u -> weights (masking of the ragged tail, lazy rescaling as in the rescaling loop)
// A wave is limited by its own instruction stream (about one instruction per 5 cycles, an MFMA ~16); where the
// copies and their address arithmetic sit was settled by measurement (in the vector phase: +3.5 % over the
// matrix phase, start, end or spread).
// K/V tiles travel global -> LDS three tiles ahead (K ring of 4 stages, V ring of 5: V of a tile is read one
// phase after its K) with 16-byte copies: one instruction
// moves four 256-byte rows (lane i -> bytes 16*i of the 1 KB destination), a quarter of the instructions the
// 4-byte form needs, and the cost of these copies is per instruction.  The destination of such a copy is
// contiguous, so rows cannot be padded; bank conflicts are avoided by permuting the 16-byte chunks of a row
// instead, which costs nothing because each lane picks the global chunk it fetches:
//   K tile   chunk c of row r sits at position c ^ (r & 15)        (16 rows x one chunk = all banks once)
//   V tile   chunk c of row r sits at position c ^ ((r & 3) << 2)  (a transpose read takes 64 bytes from each
//                                                                   of 4 rows per 32 lanes: 4 x 64 B = all banks once)
// ---------------------------------------------------------------------------------------------------
constexpr int PP_WAVES = 8;
constexpr int PP_KSTAGES = 4;                                   // K of tile u is read in phase M(u)
constexpr int PP_VSTAGES = 5;                                   // V of tile u is read one phase later, in M(u+1)
constexpr int PP_TILE_BYTES = PF_BK * 128 * 2;                  // one tensor's tile, head_dim 128, unpadded
struct TagT { static constexpr bool value = true; };
struct TagF { static constexpr bool value = false; };
template <int N>
struct IntC { static constexpr int value = N; };
template <int B, class F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>) {
  (f(IntC<B + I>()), ...);
}
template <int B, int E, class F>
__device__ __forceinline__ void static_for(F &&f) {
  static_for_impl<B>(f, std::make_integer_sequence<int, E - B>());
}
constexpr int PP_RING = 4;                                      // fragments requested ahead of their MFMA
// LDS reads that fragments i+1 .. last of a matrix phase take (see the kernel: V^T fragments two, K one)
constexpr int pp_reads_between(int i, int last) {
  int n = 0;
  for (int j = i + 1; j <= last; ++j) n += j < 16 ? 2 : 1;
  return n;
}

__device__ __forceinline__ int pp_swz(bool is_v, int row) { return is_v ? ((row & 3) << 2) : (row & 15); }

// Per-lane source offset inside a 4-row copy group whose first row is row0: lane i fetches the 16-byte chunk that
// belongs at bytes 16*i of the group's 1 KB destination (chunk permutation of the tile layouts above).
template <bool IS_V>
__device__ __forceinline__ unsigned pp_group_voff(int lane, int row0) {
  const int rr = lane >> 4, p = lane & 15;
  return (unsigned)(rr * 256 + ((p ^ pp_swz(IS_V, row0 + rr)) << 4));
}
template <bool IS_V, int RPW>
__device__ __forceinline__ int pp_copy_rows_slow(int kt, const HeadKV &H, char *stage, int wave, int lane) {
  typedef const __attribute__((address_space(1))) void *gptr_t;
  typedef __attribute__((address_space(3))) void *lptr_t;
  constexpr int D = 128;
  const int last = H.lkv - 1 - kt * PF_BK;
  asm volatile("" : "+v"(lane));                    // rare path: its per-lane offsets are worked out here, not held in registers through the loop
#pragma unroll
  for (int r = 0; r < RPW; ++r) {
    const int row = wave * RPW + r;
    const int t = kt * PF_BK + pf_min(row, last);                 // rows past the end re-read the last key
    const bool in_chunk = t >= H.hist_tokens;
    const int th = in_chunk ? 0 : t;
    const int j = th / H.tpf;
    const size_t e_hist = ((size_t)pf_max(H.slots[j], 0) * H.tpf + (th - j * H.tpf)) * D;
    const size_t e = in_chunk ? (size_t)(t - H.hist_tokens) * H.cur_stride : e_hist;
    const char *b = (const char *)((in_chunk ? (IS_V ? H.v_cur : H.k_cur) : (IS_V ? H.v_pool : H.k_pool)) + e);
    const unsigned off = (unsigned)((((lane >> 2) ^ pp_swz(IS_V, row)) << 4) | ((lane & 3) << 2));
    __builtin_amdgcn_global_load_lds((gptr_t)(b + off), (lptr_t)(stage + row * 256), 4, 0, 0);
  }
  return RPW;
}

// Request fragment I of a matrix phase (see the kernel): ak / av = this lane's K / V^T base address in the stage.
template <int I>
__device__ __forceinline__ void pp_issue_frag(u32x2 (&vl)[16], u32x2 (&vh)[16], u32x4 (&kf)[16], unsigned ak, unsigned av) {
  if constexpr (I < 16) {
    constexpr int OFF = (I / 4) * 4096;
    const unsigned a = av ^ ((I % 4) << 6);
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(vl[I]) : "v"(a), "n"(OFF));
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(vh[I]) : "v"(a), "n"(OFF + 2048));
  } else {
    constexpr int J = I - 16;
    const unsigned a = ak ^ ((J >> 1) << 5);
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(kf[J]) : "v"(a), "n"((J & 1) * 8192));
  }
}
// The wait is the compiler's own instruction fenced on both sides, not an asm statement tied to the fragment's
// registers: after an asm statement that writes a register the compiler puts a wait state in front of the MFMA
// that reads it (one issue slot per MFMA).
template <int I, int LAST>
__device__ __forceinline__ void pp_wait_frag(u32x2 (&vl)[16], u32x2 (&vh)[16], u32x4 (&kf)[16]) {
  constexpr int N = pp_reads_between(I, LAST) > 15 ? 15 : pp_reads_between(I, LAST);
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_waitcnt(0xC07F | (N << 8));                 // lgkmcnt(N), the other counters untouched
  __builtin_amdgcn_sched_barrier(0);
}

// ---- 4 waves x 64 query rows: one instruction stream per SIMD that carries the MFMAs of two half tiles (32 keys)
// and the softmax of the half tile between them (see the kernel).  A half step's operand fragments, in the order they
// are consumed: V^T of the previous half tile (8, if the half step has a PV part), K of the next half tile (8, if it
// has a QK part), and, when it prefetches, the first PP_RING V^T fragments of its own half tile, which the following
// half step consumes first.
template <bool PV, bool QK, bool PRE>
struct W64Stream {
  static constexpr int NV = PV ? 8 : 0, NK = QK ? 8 : 0, NC = NV + NK, L = NC + (PRE ? PP_RING : 0);
  static constexpr int NSLOT = NC > 0 ? 2 * NC : 1;              // MFMA slots: two per fragment (the query blocks)
  static constexpr int kind(int p) { return p < NV ? 0 : p < NC ? 1 : 2; }
  static constexpr int idx(int p) { return p < NV ? p : p < NC ? p - NV : p - NC; }
  static constexpr int reads(int p) { return kind(p) == 1 ? 1 : 2; }
  // LDS reads requested after fragment p's at the time its first MFMA is issued
  static constexpr int wait_n(int p) {
    int n = 0;
    for (int q = p + 1; q < p + PP_RING && q < L; ++q) n += reads(q);
    return n;
  }
};
// The softmax of one half tile (16 scores per lane and query block) as 65 small steps that are dealt out between the
// MFMAs in proportion to their instruction counts: 0..15 running maxima (two scores each; two chains per query block
// take turns, block 0 first), 16 the check against the reference maximum, which moves only when a score exceeds it by
// the lazy margin (then, and only then, the two lanes of a query column exchange their maxima), then for each of 16
// score pairs three steps a few instructions apart, so that none waits for the one before: "scale" (2 instructions),
// "exp2" (2), "add to the row sum, round to bf16" (3).
constexpr int W64_NSTEP = 65;
constexpr int W64_BSTEP0 = 17;                                   // first step of the exp2 part
// step W64_BSTEP0 + t -> kind (0 scale, 1 exp2, 2 sum and round) * 16 + score pair: pair u is scaled at time u, goes
// through exp2 at time u + 1 and is summed at time u + 2
constexpr int w64_bstep(int t) {
  int n = 0;
  for (int tau = 0; tau < 18; ++tau)
    for (int kind = 0; kind < 3; ++kind) {
      const int u = tau - kind;
      if (u < 0 || u > 15) continue;
      if (n == t) return kind * 16 + u;
      ++n;
    }
  return -1;
}
constexpr int w64_step_weight(int k) {
  if (k < 16) return 1;
  if (k == 16) return 6;
  return w64_bstep(k - W64_BSTEP0) / 16 == 2 ? 3 : 2;
}
constexpr int w64_weight_before(int k) {
  int w = 0;
  for (int i = 0; i < k; ++i) w += w64_step_weight(i);
  return w;
}
constexpr int w64_first_step(int slot, int nslot) {
  const int total = w64_weight_before(W64_NSTEP);
  for (int k = 0; k < W64_NSTEP; ++k)
    if (w64_weight_before(k) * nslot >= slot * total) return k;
  return W64_NSTEP;
}
// The 64-row form keeps its long-lived MFMA operands in accumulation registers that the compiler never sees: the output
// accumulators in a64..a191 (block n = 4*qb + db in a[64 + 16*n ..]) and the Q^T fragments in a192..a255 (fragment
// n = 8*qb + ks in a[192 + 4*n ..]) for the whole work item; the scores are ordinary vector registers, where the softmax
// reads them without copies.  All MFMAs of that form are asm statements that name these registers.  (Left to the
// compiler, a kernel that may use all 512 registers gets every MFMA result in accumulation registers, pays a copy per
// score and keeps moving the accumulators around.)  This only works because the compiler itself stays out of a64..a255
// in that kernel: it has no MFMA builtin there, the library is built with spilling of vector registers into
// accumulation registers switched off (-mllvm -amdgpu-spill-vgpr-to-agpr=0), the few values it still parks there go to
// the lowest registers, and the build reads the listing and fails if any instruction of the compiler's own touches a
// register from a32 up (build.py).
// The compiler does not know these statements are MFMAs and adds no wait states around them: the distances the
// hardware needs between an MFMA and a dependent instruction are kept by the order of the stream (see the kernel), and
// no operand of such a statement is written by a vector instruction right in front of it.
#define PF_A10(b) "a" #b "0", "a" #b "1", "a" #b "2", "a" #b "3", "a" #b "4", "a" #b "5", "a" #b "6", "a" #b "7", "a" #b "8", "a" #b "9"
#define PF_CLOBBER_A64_A191                                                                                                  \
  "a64", "a65", "a66", "a67", "a68", "a69", PF_A10(7), PF_A10(8), PF_A10(9), PF_A10(10), PF_A10(11), PF_A10(12), PF_A10(13), \
      PF_A10(14), PF_A10(15), PF_A10(16), PF_A10(17), PF_A10(18), "a190", "a191"
#define PF_CLOBBER_A192_A255 "a192", "a193", "a194", "a195", "a196", "a197", "a198", "a199", PF_A10(20), PF_A10(21), PF_A10(22), PF_A10(23), PF_A10(24), "a250", "a251", "a252", "a253", "a254", "a255"
template <int N> __device__ __forceinline__ void w64_mfma_o(u32x4 a, bf16x8 b);     // O^T block n += a . b
template <int N> __device__ __forceinline__ void w64_mfma_s(f32x16 &acc, u32x4 a);  // acc += a . Q^T fragment n
template <int N> __device__ __forceinline__ void w64_mfma_s0(f32x16 &acc, u32x4 a); // acc  = a . Q^T fragment n
template <int N> __device__ __forceinline__ void w64_set_q(u32x4 q);                // Q^T fragment n = q
template <int N> __device__ __forceinline__ f32x16 w64_get_o();                     // O^T block n
#define PF_W64_O(N, R0, R1, R2, R3, R4, R5, R6, R7, R8, R9, R10, R11, R12, R13, R14, R15)                                    \
  template <> __device__ __forceinline__ void w64_mfma_o<N>(u32x4 a, bf16x8 b) {                                             \
    asm volatile("v_mfma_f32_32x32x16_bf16 a[" #R0 ":" #R15 "], %0, %1, a[" #R0 ":" #R15 "]" : : "v"(a), "v"(b)              \
                 : PF_CLOBBER_A64_A191);                                                                                     \
  }                                                                                                                          \
  template <> __device__ __forceinline__ f32x16 w64_get_o<N>() {                                                             \
    float r[16];                                                                                                             \
    asm volatile("v_accvgpr_read_b32 %0, a" #R0 "\n\tv_accvgpr_read_b32 %1, a" #R1 "\n\tv_accvgpr_read_b32 %2, a" #R2       \
                 "\n\tv_accvgpr_read_b32 %3, a" #R3 "\n\tv_accvgpr_read_b32 %4, a" #R4 "\n\tv_accvgpr_read_b32 %5, a" #R5    \
                 "\n\tv_accvgpr_read_b32 %6, a" #R6 "\n\tv_accvgpr_read_b32 %7, a" #R7 "\n\tv_accvgpr_read_b32 %8, a" #R8    \
                 "\n\tv_accvgpr_read_b32 %9, a" #R9 "\n\tv_accvgpr_read_b32 %10, a" #R10 "\n\tv_accvgpr_read_b32 %11, a" #R11 \
                 "\n\tv_accvgpr_read_b32 %12, a" #R12 "\n\tv_accvgpr_read_b32 %13, a" #R13                                  \
                 "\n\tv_accvgpr_read_b32 %14, a" #R14 "\n\tv_accvgpr_read_b32 %15, a" #R15                                  \
                 : "=v"(r[0]), "=v"(r[1]), "=v"(r[2]), "=v"(r[3]), "=v"(r[4]), "=v"(r[5]), "=v"(r[6]), "=v"(r[7]), "=v"(r[8]), \
                   "=v"(r[9]), "=v"(r[10]), "=v"(r[11]), "=v"(r[12]), "=v"(r[13]), "=v"(r[14]), "=v"(r[15]));                \
    f32x16 v;                                                                                                                \
    _Pragma("unroll") for (int i = 0; i < 16; ++i) v[i] = r[i];                                                             \
    return v;                                                                                                                \
  }
PF_W64_O(0, 64, 65, 66, 67, 68, 69, 70, 71, 72, 73, 74, 75, 76, 77, 78, 79)
PF_W64_O(1, 80, 81, 82, 83, 84, 85, 86, 87, 88, 89, 90, 91, 92, 93, 94, 95)
PF_W64_O(2, 96, 97, 98, 99, 100, 101, 102, 103, 104, 105, 106, 107, 108, 109, 110, 111)
PF_W64_O(3, 112, 113, 114, 115, 116, 117, 118, 119, 120, 121, 122, 123, 124, 125, 126, 127)
PF_W64_O(4, 128, 129, 130, 131, 132, 133, 134, 135, 136, 137, 138, 139, 140, 141, 142, 143)
PF_W64_O(5, 144, 145, 146, 147, 148, 149, 150, 151, 152, 153, 154, 155, 156, 157, 158, 159)
PF_W64_O(6, 160, 161, 162, 163, 164, 165, 166, 167, 168, 169, 170, 171, 172, 173, 174, 175)
PF_W64_O(7, 176, 177, 178, 179, 180, 181, 182, 183, 184, 185, 186, 187, 188, 189, 190, 191)
#undef PF_W64_O
#define PF_W64_Q(N, R0, R1, R2, R3)                                                                                          \
  template <> __device__ __forceinline__ void w64_mfma_s<N>(f32x16 & acc, u32x4 a) {                                         \
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, a[" #R0 ":" #R3 "], %0" : "+v"(acc) : "v"(a));                            \
  }                                                                                                                          \
  template <> __device__ __forceinline__ void w64_mfma_s0<N>(f32x16 & acc, u32x4 a) {                                        \
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, a[" #R0 ":" #R3 "], 0" : "=&v"(acc) : "v"(a));                            \
  }                                                                                                                          \
  template <> __device__ __forceinline__ void w64_set_q<N>(u32x4 q) {                                                        \
    asm volatile("v_accvgpr_write_b32 a" #R0 ", %0\n\tv_accvgpr_write_b32 a" #R1 ", %1\n\tv_accvgpr_write_b32 a" #R2        \
                 ", %2\n\tv_accvgpr_write_b32 a" #R3 ", %3"                                                                  \
                 : : "v"(q[0]), "v"(q[1]), "v"(q[2]), "v"(q[3]) : PF_CLOBBER_A192_A255);                                     \
  }
PF_W64_Q(0, 192, 193, 194, 195) PF_W64_Q(1, 196, 197, 198, 199) PF_W64_Q(2, 200, 201, 202, 203) PF_W64_Q(3, 204, 205, 206, 207)
PF_W64_Q(4, 208, 209, 210, 211) PF_W64_Q(5, 212, 213, 214, 215) PF_W64_Q(6, 216, 217, 218, 219) PF_W64_Q(7, 220, 221, 222, 223)
PF_W64_Q(8, 224, 225, 226, 227) PF_W64_Q(9, 228, 229, 230, 231) PF_W64_Q(10, 232, 233, 234, 235) PF_W64_Q(11, 236, 237, 238, 239)
PF_W64_Q(12, 240, 241, 242, 243) PF_W64_Q(13, 244, 245, 246, 247) PF_W64_Q(14, 248, 249, 250, 251) PF_W64_Q(15, 252, 253, 254, 255)
#undef PF_W64_Q
// a64..a191 = 0, and a64..a191 *= alpha (a64..a127: query block 0, a128..a191: query block 1): a loop over the register
// NUMBER cannot be written (no indirect access to accumulation registers), so the text is spelled out, ten registers (one decade of numbers) at a time
#define PF_W64_Z10(b) "v_accvgpr_write_b32 a" #b "0, 0\n\tv_accvgpr_write_b32 a" #b "1, 0\n\tv_accvgpr_write_b32 a" #b "2, 0\n\tv_accvgpr_write_b32 a" #b "3, 0\n\tv_accvgpr_write_b32 a" #b "4, 0\n\tv_accvgpr_write_b32 a" #b "5, 0\n\tv_accvgpr_write_b32 a" #b "6, 0\n\tv_accvgpr_write_b32 a" #b "7, 0\n\tv_accvgpr_write_b32 a" #b "8, 0\n\tv_accvgpr_write_b32 a" #b "9, 0\n\t"
__device__ __forceinline__ void w64_zero_o() {
  asm volatile("v_accvgpr_write_b32 a64, 0\n\tv_accvgpr_write_b32 a65, 0\n\tv_accvgpr_write_b32 a66, 0\n\tv_accvgpr_write_b32 a67, 0\n\t"
               "v_accvgpr_write_b32 a68, 0\n\tv_accvgpr_write_b32 a69, 0\n\t"
               PF_W64_Z10(7) PF_W64_Z10(8) PF_W64_Z10(9) PF_W64_Z10(10) PF_W64_Z10(11) PF_W64_Z10(12) PF_W64_Z10(13) PF_W64_Z10(14)
               PF_W64_Z10(15) PF_W64_Z10(16) PF_W64_Z10(17) PF_W64_Z10(18) "v_accvgpr_write_b32 a190, 0\n\tv_accvgpr_write_b32 a191, 0"
               : : : PF_CLOBBER_A64_A191);
}
#undef PF_W64_Z10
#define PF_W64_R1(r, al) "v_accvgpr_read_b32 %2, a" #r "\n\tv_mul_f32 %2, %2, %" #al "\n\tv_accvgpr_write_b32 a" #r ", %2\n\t"
#define PF_W64_R10(b, al) PF_W64_R1(b##0, al) PF_W64_R1(b##1, al) PF_W64_R1(b##2, al) PF_W64_R1(b##3, al) PF_W64_R1(b##4, al) PF_W64_R1(b##5, al) PF_W64_R1(b##6, al) PF_W64_R1(b##7, al) PF_W64_R1(b##8, al) PF_W64_R1(b##9, al)
__device__ __forceinline__ void w64_rescale(float al0, float al1) {
  float t;
  asm volatile("s_nop 15\n\ts_nop 15\n\t"                          // the last MFMA into the accumulators has written them back
               PF_W64_R1(64, 0) PF_W64_R1(65, 0) PF_W64_R1(66, 0) PF_W64_R1(67, 0) PF_W64_R1(68, 0) PF_W64_R1(69, 0)
               PF_W64_R10(7, 0) PF_W64_R10(8, 0) PF_W64_R10(9, 0) PF_W64_R10(10, 0) PF_W64_R10(11, 0)
               PF_W64_R1(120, 0) PF_W64_R1(121, 0) PF_W64_R1(122, 0) PF_W64_R1(123, 0) PF_W64_R1(124, 0) PF_W64_R1(125, 0) PF_W64_R1(126, 0) PF_W64_R1(127, 0)
               PF_W64_R1(128, 1) PF_W64_R1(129, 1)
               PF_W64_R10(13, 1) PF_W64_R10(14, 1) PF_W64_R10(15, 1) PF_W64_R10(16, 1) PF_W64_R10(17, 1) PF_W64_R10(18, 1)
               PF_W64_R1(190, 1) PF_W64_R1(191, 1) "s_nop 7"
               : "+v"(al0), "+v"(al1), "=&v"(t) : : PF_CLOBBER_A64_A191);
}
#undef PF_W64_R10
#undef PF_W64_R1
template <int N>
__device__ __forceinline__ void pp_wait_lgkm() {
  __builtin_amdgcn_sched_barrier(0);
  __builtin_amdgcn_s_waitcnt(0xC07F | (N << 8));                 // lgkmcnt(N), the other counters untouched
  __builtin_amdgcn_sched_barrier(0);
}

template <int D, int NW>
__global__ __launch_bounds__(NW * 64, NW == 8 ? 2 : 1) void pf_attn_pp_kernel(AttnParams) {
  static_assert(D == 128, "tile layouts are written for 256-byte rows");
  static_assert(NW == 8 || NW == 4, "8 waves x 32 query rows, or 4 waves x 64");
  constexpr int RPW = PF_BK / NW;                              // rows of every tile that one wave copies
  constexpr int NG = RPW / 4;                                  // ... in groups of four rows, one copy instruction each
  constexpr int NQB = 256 / (NW * 32);                         // 32-row query blocks per wave
  constexpr int BK = PF_BK;
  constexpr int NKS = D / 16, NDB = D / 32;
  typedef const __attribute__((address_space(1))) void *gptr_t;
  typedef __attribute__((address_space(3))) void *lptr_t;

  // K ring, then V ring; the epilogue reuses the same memory to stage the output rows
  static_assert((PP_KSTAGES + PP_VSTAGES) * PP_TILE_BYTES >= attn_stage_floats(256, D) * 4, "output staging fits");
  __shared__ __attribute__((aligned(1024))) char smem[(PP_KSTAGES + PP_VSTAGES) * PP_TILE_BYTES];
  __shared__ int32_t sFlag;
  __shared__ int32_t sNext;
  __shared__ long long sTrace[6];                              // busy ticks, first start, this item's start, items, busy shader-clock cycles, this item's start in those (thread 0 only)
  char (*sK)[PP_TILE_BYTES] = (char (*)[PP_TILE_BYTES])smem;
  char (*sV)[PP_TILE_BYTES] = sK + PP_KSTAGES;
  const int tid0 = threadIdx.x;

  // ---- work queue.  The items of die x are entries x, x + 8, x + 16, ... of the list, in the order the plan
  // wants them started.  One workgroup per compute unit is launched; workgroup b runs on die b % 8 and takes
  // the next entry of that die's queue (so the query tiles of one key segment still run side by side on one
  // die and share its L2), and when that queue is empty it takes from the next die's, and so on: the dies do
  // not run at the same speed, and without this the launch ends when the slowest die does.  Every workgroup
  // leaves the loop after finding all eight queues empty; tickets only grow, so that always happens.  The last
  // workgroup to leave puts the tickets back to zero for the next launch. ----
  // The parameters are read again from the kernel-argument segment for every item (a few scalar loads): held in
  // registers across the loop they would crowd out the item's own state.
  typedef const __attribute__((address_space(4))) unsigned long long *karg_t;
  static_assert(sizeof(AttnParams) % 8 == 0, "parameters are copied as 8-byte words");
  struct ParamWords { unsigned long long w[sizeof(AttnParams) / 8]; };
  auto load_params = [&]() {
    int opaque_zero = 0;                       // hides from the compiler that every call reads the same words
    asm volatile("" : "+s"(opaque_zero));
    karg_t karg = (karg_t)__builtin_amdgcn_kernarg_segment_ptr() + __builtin_amdgcn_readfirstlane(opaque_zero);
    ParamWords pw;
#pragma unroll
    for (int i = 0; i < (int)(sizeof(AttnParams) / 8); ++i) pw.w[i] = karg[i];
    AttnParams R = __builtin_bit_cast(AttnParams, pw);
    // pointers rebuilt from raw words: say again that they point to global memory
    R.q = as_global(R.q), R.k_cur = as_global(R.k_cur), R.v_cur = as_global(R.v_cur), R.k_pool = as_global(R.k_pool);
    R.v_pool = as_global(R.v_pool), R.out = as_global(R.out), R.sel_count = as_global(R.sel_count);
    R.sel_slots = as_global(R.sel_slots), R.items = as_global(R.items), R.counters = as_global(R.counters);
    R.tickets = as_global(R.tickets), R.workspace = as_global(R.workspace);
    return R;
  };
  if (tid0 == 0) sTrace[0] = sTrace[1] = sTrace[2] = sTrace[3] = sTrace[4] = sTrace[5] = 0;
  int hop_v = 0;                               // dies given up so far; kept in a vector register between items
  while (true) {
  asm volatile("" : "+v"(hop_v));
  int hop = __builtin_amdgcn_readfirstlane(hop_v);
  const AttnParams P = load_params();
  int item_idx = -1;
  if (P.tickets == nullptr) {
    if (hop == 0) item_idx = blockIdx.x;
    hop = PF_NUM_XCD;
  } else {
    const int home = blockIdx.x % PF_NUM_XCD;
    while (hop < PF_NUM_XCD) {
      const int x = (home + hop) % PF_NUM_XCD;
      if (tid0 == 0) sNext = atomicAdd(&P.tickets[x], 1);
      __syncthreads();
      const int j = __builtin_amdgcn_readfirstlane(sNext);
      __syncthreads();
      if (j < P.queue_len) {
        item_idx = j * PF_NUM_XCD + x;
        break;
      }
      ++hop;
    }
  }
  hop_v = hop;
  if (item_idx < 0) break;
  const PfWorkItem it = P.items[item_idx];
  if (it.head < 0) continue;
  if (__builtin_expect(P.block_trace != nullptr, 0) && tid0 == 0) {
    const long long now = wall_clock64();
    if (sTrace[3] == 0) sTrace[1] = now;
    sTrace[2] = now;
    sTrace[5] = clock64();
  }
  int tid = tid0;
  asm volatile("" : "+v"(tid));               // per-lane constants are worked out anew for each item, not kept across the loop
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wave >> 2;
  const int l32 = lane & 31, g = lane >> 5;
  HeadKV H;
  attn_setup_head<D>(P, it, H, tid);
  f32x16 o[NQB][NDB];
  float m_run[NQB], l_run[NQB];
  attn_zero<D, NQB>(o, m_run, l_run);
  const float c = P.scale_log2;
  const float thr = ATT_LAZY_LOG2 / c;

  // LDS byte addresses of this lane's fragments inside stage 0 (other stages: + stage * PP_TILE_BYTES).  The
  // arrays are 1 KB aligned, so the chunk permutation and the k-step / channel-block index act on address
  // bits nothing else touches and one base register per tensor is enough:
  //   K: row l32 (+32 per key block), chunk (2*ks + g) ^ (l32 & 15)       -> ak ^ (ks << 5)
  //   V^T: row 4g + (lane & 15) / 4 (+8, +16 per chunk), chunk (c0 + 4*db) ^ swz  -> av ^ (db << 6)
  const unsigned ldsK = (unsigned)(uintptr_t)(const __attribute__((address_space(3))) char *)&sK[0][0];
  const unsigned ldsV = (unsigned)(uintptr_t)(const __attribute__((address_space(3))) char *)&sV[0][0];
  const unsigned ak = ldsK + l32 * 256 + ((g ^ (l32 & 15)) << 4);
  unsigned av;
  {
    const int rowv = 4 * g + ((lane & 15) >> 2);
    const int c0 = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
    av = ldsV + rowv * 256 + ((c0 ^ pp_swz(true, rowv)) << 4) + 8 * (lane & 1);
  }
  // per-lane source offsets inside a 4-row copy group.  The wave's later groups (rows + 4, + 8, + 12) permute the
  // K chunks by one more bit each and the V chunks not at all
  const unsigned vofK0 = pp_group_voff<false>(lane, wave * RPW), vofV = pp_group_voff<true>(lane, wave * RPW);
  const int wrow_bytes = wave * RPW * 256;                     // this wave's first row inside a tile

  // One 4-row group gi of K or of V.  The copies are buffer loads: the tile's first row is the base of a 16 KB
  // buffer descriptor (scalar registers), the wave's rows are a scalar offset, the lane's chunk a 32-bit vector
  // offset, and the group is the instruction's immediate offset (it moves the LDS destination along with the
  // source).  Next to MFMAs this form costs almost nothing, whereas a global load with a 64-bit address per lane
  // held up the SIMD for ~65 cycles per instruction (measured).
  auto copy_group_at = [&](const __bf16 *kbase, const __bf16 *vbase, int snk, int snv, auto is_v, auto gidx) __attribute__((always_inline)) {
    constexpr unsigned RSRC_FLAGS = 0x00020000u;               // raw buffer, 32-bit data format
    constexpr int GI = decltype(gidx)::value;
    if constexpr (!decltype(is_v)::value) {
      const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc((void *)kbase, 0, PP_TILE_BYTES, RSRC_FLAGS);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lptr_t)(&sK[snk][wrow_bytes]), 16, vofK0 ^ (unsigned)(GI << 6), wrow_bytes, GI * 1024, 0);
    } else {
      const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc((void *)vbase, 0, PP_TILE_BYTES, RSRC_FLAGS);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lptr_t)(&sV[snv][wrow_bytes]), 16, vofV, wrow_bytes, GI * 1024, 0);
    }
  };
  // a whole contiguous tile: K groups, then V groups
  auto copy_tile_dense = [&](const __bf16 *kbase, const __bf16 *vbase, int snk, int snv) __attribute__((always_inline)) {
    static_for<0, NG>([&](auto gi) { copy_group_at(kbase, vbase, snk, snv, TagF(), gi); });
    static_for<0, NG>([&](auto gi) { copy_group_at(kbase, vbase, snk, snv, TagT(), gi); });
  };
  // The same for a chunk tile whose token rows are cur_stride elements apart (the model's [tokens][heads][D]
  // layout): the lane's row is part of its vector offset, the wave's first row and the group are scalar
  // offsets, and the group's LDS destination moves by hand.
  const unsigned row_b = (unsigned)(H.cur_stride * 2);         // bytes between chunk token rows (< 2^25, checked on the host)
  auto copy_tile_strided = [&](const TileSrc &src, int snk, int snv) __attribute__((always_inline)) {
    constexpr unsigned RSRC_FLAGS = 0x00020000u;
    const unsigned lrow = (unsigned)(lane >> 4) * row_b;
    const __amdgpu_buffer_rsrc_t rk = __builtin_amdgcn_make_buffer_rsrc((void *)src.kb, 0, (int)(PF_BK * row_b), RSRC_FLAGS);
    const __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc((void *)src.vb, 0, (int)(PF_BK * row_b), RSRC_FLAGS);
    static_for<0, NG>([&](auto gi) {
      constexpr int GI = decltype(gi)::value;
      const unsigned soff = (unsigned)(wave * RPW + 4 * GI) * row_b;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rk, (lptr_t)(&sK[snk][wrow_bytes + GI * 1024]), 16,
                                               ((vofK0 ^ (unsigned)(GI << 6)) & 0xffu) + lrow, soff, 0, 0);
    });
    static_for<0, NG>([&](auto gi) {
      constexpr int GI = decltype(gi)::value;
      const unsigned soff = (unsigned)(wave * RPW + 4 * GI) * row_b;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rv, (lptr_t)(&sV[snv][wrow_bytes + GI * 1024]), 16, (vofV & 0xffu) + lrow, soff, 0, 0);
    });
  };
  // A tile made of two dense runs (it crosses a frame border): a 4-row group lies in the first run, in the second, or
  // (when the border is not a multiple of 4 rows into the tile) in both, and then each run's lanes copy under their
  // own execution mask: the LDS address of such a copy follows the lane number, so masked-off lanes leave their
  // 16 bytes to the other instruction.  Returns the number of copy instructions issued.
  auto copy_tile_split = [&](const TileSrc &src, int snk, int snv) __attribute__((always_inline)) -> int {
    int n = 0;
    const __bf16 *ka = src.kb, *va = src.vb, *kb2 = src.kb2, *vb2 = src.vb2;
    const int n1 = src.n1;
    auto one = [&](auto is_v, auto gi) __attribute__((always_inline)) {
      const int row0 = wave * RPW + decltype(gi)::value * 4;
      if (row0 + 4 <= n1) {
        copy_group_at(ka, va, snk, snv, is_v, gi);
        n += 1;
      } else if (row0 >= n1) {
        copy_group_at(kb2, vb2, snk, snv, is_v, gi);
        n += 1;
      } else {
        int lane_l = lane;
        asm volatile("" : "+v"(lane_l));                        // rare: its lane test is not held in a register through the loop
        if (row0 + (lane_l >> 4) < n1) copy_group_at(ka, va, snk, snv, is_v, gi);
        else copy_group_at(kb2, vb2, snk, snv, is_v, gi);
        n += 2;
      }
    };
    static_for<0, NG>([&](auto gi) { one(TagF(), gi); });
    static_for<0, NG>([&](auto gi) { one(TagT(), gi); });
    return n;
  };
  // whole tile at once (prologue; tiles that cross a frame border or hold the ragged end go row by row here)
  auto copy_tile_now = [&](int kt, const TilePos &tp, int snk, int snv) -> int {
    const TileSrc src = tile_src(kt, tp, H, D);
    if (src.simple) {
      if (src.strided) copy_tile_strided(src, snk, snv);
      else copy_tile_dense(src.kb, src.vb, snk, snv);
      return 2 * NG;
    }
    pp_copy_rows_slow<false, RPW>(kt, H, sK[snk], wave, lane);
    pp_copy_rows_slow<true, RPW>(kt, H, sV[snv], wave, lane);
    return 2 * RPW;
  };
  // "Everything but the copies of the last step has landed": at most 2*NG vector-memory operations may be
  // outstanding (a contiguous tile's copies).  When the last step sent a tile row by row (at a frame border) this
  // also waits for most of those, which were sent a whole step ago; when it sent nothing, the older copies are all
  // that is in flight.
  auto wait_copies = [&](int n) __attribute__((always_inline)) {
    __builtin_amdgcn_s_waitcnt(0x0F70 | (2 * NG));
    if (__builtin_expect(n == 0, 0)) __builtin_amdgcn_s_waitcnt(0x0F70);
  };
  // the copy planned for this step (see plan_copy), K into stage snk, V into stage snv; returns the instruction count
  auto copy_planned = [&](const TileSrc &src, int kt_copy, int snk, int snv) __attribute__((always_inline)) -> int {
    if (__builtin_expect(src.simple && !src.strided, 1)) {
      copy_tile_dense(src.kb, src.vb, snk, snv);
      return 2 * NG;
    }
    if (src.simple) {
      copy_tile_strided(src, snk, snv);
      return 2 * NG;
    }
    if (src.split) return copy_tile_split(src, snk, snv);
    pp_copy_rows_slow<false, RPW>(kt_copy, H, sK[snk], wave, lane);
    pp_copy_rows_slow<true, RPW>(kt_copy, H, sV[snv], wave, lane);
    return 2 * RPW;
  };

  // ---- prologue: tiles kt0 .. kt0+2 start travelling, then Q^T is fetched.  Vector-memory operations complete
  // in order, so once Q^T is in its registers (the empty asm makes the compiler wait here, not inside the loop,
  // where such a wait would drain the copies in flight) the three tiles have landed too. ----
  TilePos pos = tile_pos_init(it.kt0, H.hist_tokens, H.n_sel, H.tpf);
  copy_tile_now(it.kt0, pos, 0, 0);
  if (it.kt0 + 1 < it.kt1) {
    tile_pos_advance(pos, H.n_sel, H.tpf);
    copy_tile_now(it.kt0 + 1, pos, 1, 1);
  }
  if (it.kt0 + 2 < it.kt1) {
    tile_pos_advance(pos, H.n_sel, H.tpf);
    copy_tile_now(it.kt0 + 2, pos, 2, 2);
  }
  // ---- plan of the next copy (made in one vector phase and carried out at the start of the next, so the
  // scalar load of a frame's slot has a whole tile time to arrive) ----
  TileSrc nsrc;
  nsrc.kb = nsrc.vb = nsrc.kb2 = nsrc.vb2 = nullptr;
  nsrc.simple = nsrc.split = false;
  nsrc.n1 = 0;
  int ncopy_kt = -1;                                           // tile planned for the next copy, -1: none
  int run_left = 0;                                            // tiles after the planned one that continue its source run
  long long run_step = 0;                                      // elements from one tile of the run to the next
  auto plan_copy = [&](int kt_target) __attribute__((always_inline)) {
    if (__builtin_expect(run_left <= 0, 0)) {
      ncopy_kt = -1;
      if (kt_target < it.kt1) {
        tile_pos_advance(pos, H.n_sel, H.tpf);
        nsrc = tile_src(kt_target, pos, H, D);
        ncopy_kt = kt_target;
        if (nsrc.simple) {
          const int room = pos.j < H.n_sel ? H.tpf - pos.r : H.lkv - kt_target * PF_BK;   // keys from the tile's first row to the run's end
          run_left = pf_min(room / PF_BK - 1, it.kt1 - 1 - kt_target);
          run_step = (long long)PF_BK * (pos.j < H.n_sel ? D : H.cur_stride);
        }
      }
    } else {
      // common case: the tile follows a contiguous tile of the same frame (or of the chunk), is itself whole and
      // inside it, and belongs to this work item: both sources move on by one tile, no slot lookup
      --run_left;
      pos.r += PF_BK;
      nsrc.kb += run_step;
      nsrc.vb += run_step;
      ncopy_kt = kt_target;
    }
  };

  // A wave whose 32 query rows all lie beyond the chunk's end (the last query tile of a head) still sends its share
  // of the copies and meets every barrier, but skips the fragments, MFMAs and softmax: its partner on the SIMD then
  // has the issue slots to itself, and the matrix pipe does no work that is thrown away.
  const bool has_rows = it.q0 + wave * (32 * NQB) < P.q_tokens;

  if constexpr (NW == 8) {
  bf16x8 qf[1][NKS];
  attn_load_q<D, 1>(P, it, qf, tid);
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) asm volatile("" : "+v"(qf[0][ks]));
  __builtin_amdgcn_s_waitcnt(0x0F70);
  int n_last = 0;                                              // copy instructions sent in the last vector phase
  __builtin_amdgcn_s_barrier();
  if (grp == 1) __builtin_amdgcn_s_barrier();                  // group 1 trails by one phase

  // ---- fragments.  A matrix phase consumes 32 operand fragments from LDS, one per MFMA:
  //   0..15   V^T of the previous tile: 16-key chunk i/4, channel block i%4 (two 8-byte transpose reads)
  //   16..31  K of the current tile: key block (i-16)%2, k-step (i-16)/2 (one 16-byte read); the two key
  //           blocks alternate so consecutive MFMAs never wait for each other's accumulator
  // They are requested PP_RING fragments ahead of their MFMA (at most 15 LDS reads may be in flight per
  // wave) and waited for with counted waits: LDS reads of a wave complete in order.
  f32x16 s[2];
  bf16x8 pf[4];
  u32x2 vl[16], vh[16];
  u32x4 kf[16];
  auto issue_frag = [&](auto idx, unsigned offK, unsigned offV) {
    pp_issue_frag<decltype(idx)::value>(vl, vh, kf, ak + offK, av + offV);
  };
  // wait until fragment I has arrived, LAST being the newest fragment requested so far
  auto wait_frag = [&](auto idx, auto last) {
    pp_wait_frag<decltype(idx)::value, decltype(last)::value>(vl, vh, kf);
  };
  auto mfma_frag = [&](auto idx) {
    constexpr int I = decltype(idx)::value;
    if constexpr (I < 16) {
      const u32x4 a4 = __builtin_shufflevector(vl[I], vh[I], 0, 1, 2, 3);
      o[0][I % 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a4), pf[I / 4], o[0][I % 4], 0, 0, 0);
    } else {
      constexpr int J = I - 16, KB = J & 1, KSTEP = J >> 1;
      const f32x16 zero = {};
      s[KB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kf[J]), qf[0][KSTEP], KSTEP == 0 ? zero : s[KB], 0, 0, 0);
    }
  };

  float mthr = m_run[0] + thr, mc = m_run[0] * c, l_odd = 0.0f;   // reference maximum + lazy margin, * scale; odd scores' row sum
  // weights of two scores (key block kb, registers i and i+1): scale, exp2, add to the row sums (even scores into l_run,
  // odd ones into l_odd; plain fp32 adds: a dot-product instruction goes through the matrix pipe and queues there behind
  // the other group's MFMAs, measured ~54 cycles each next to a saturated MFMA stream, against 4 alone), round to bf16
  auto softmax_pair = [&](auto kbv, auto iv) __attribute__((always_inline)) {
    constexpr int kb = decltype(kbv)::value, i = decltype(iv)::value;
    const float e0 = fast_exp2(fmaf(s[kb][i], c, -mc));
    const float e1 = fast_exp2(fmaf(s[kb][i + 1], c, -mc));
    l_run[0] += e0;
    l_odd += e1;
    pf[kb * 2 + (i >> 3)][i & 7] = (__bf16)e0;
    pf[kb * 2 + (i >> 3)][(i & 7) + 1] = (__bf16)e1;
  };
  // ---- matrix phase: PV of the tile whose V sits in stage st_pv (its fragments 0 .. PP_RING-1 already
  // requested), QK of the tile whose K sits in stage st_qk ----
  auto m_phase = [&](auto has_pv, auto has_qk, int st_qk, int st_pv, int st_v_next) {
    constexpr bool HAS_PV = decltype(has_pv)::value, HAS_QK = decltype(has_qk)::value;
    constexpr int FIRST = HAS_PV ? 0 : 16, LAST = HAS_QK ? 31 : 15;
    const unsigned offK = st_qk * PP_TILE_BYTES, offV = st_pv * PP_TILE_BYTES;
    if (__builtin_expect(has_rows, 1)) {
    __builtin_amdgcn_s_setprio(3);                              // the matrix phase goes first on its SIMD
    if constexpr (!HAS_PV) static_for<16, 16 + PP_RING>([&](auto f) { issue_frag(f, offK, offV); });
    static_for<FIRST, LAST + 1>([&](auto f) {
      constexpr int I = decltype(f)::value;
      constexpr int NEWEST = I + PP_RING - 1 < LAST ? I + PP_RING - 1 : LAST;
      wait_frag(f, IntC<NEWEST>());
      mfma_frag(f);
      if constexpr (I + PP_RING <= LAST) issue_frag(IntC<I + PP_RING>(), offK, offV);
      __builtin_amdgcn_sched_barrier(0);                        // keep the hand-made order: wait, MFMA, next request
    });
    // the first V^T fragments of the QK tile (V stage st_v_next), for the next matrix phase: requested here, at the
    // end of the shorter of the two instruction streams
    if constexpr (HAS_QK) static_for<0, PP_RING>([&](auto f) { issue_frag(f, 0u, (unsigned)(st_v_next * PP_TILE_BYTES)); });
    __builtin_amdgcn_s_setprio(0);
    }
    // this wave's rows of the tile after the QK tile (sent two vector phases ago) have landed once only the
    // copies of its last vector phase are outstanding
    if (HAS_QK) wait_copies(n_last);
    __builtin_amdgcn_s_barrier();
  };

  // ---- vector phase: copies of tile kt+3, plan of the copy after that, scores of tile kt -> weights ----
  auto v_phase = [&](int kt, int sk_, int sv_) {
    // the copy planned one vector phase ago: tile kt+3, K into the stage tile kt-1 lived in, V into tile kt-2's
    // (their last readers, both groups' M(kt-1), are two barriers back)
    n_last = 0;
    if (__builtin_expect(ncopy_kt >= 0, 1)) {
      const int snk = (sk_ + 3) & (PP_KSTAGES - 1);
      const int snv = sv_ >= 2 ? sv_ - 2 : sv_ + PP_VSTAGES - 2;
      n_last = copy_planned(nsrc, ncopy_kt, snk, snv);
    }
    plan_copy(kt + 4);
    if (__builtin_expect(!has_rows, 0)) {
      __builtin_amdgcn_s_barrier();
      return;
    }
    const int valid = H.lkv - kt * BK;                          // ragged tail: only the head's last tile
    if (__builtin_expect(valid < BK, 0)) {
      int g_l = g;
      asm volatile("" : "+v"(g_l));                              // rare path: its per-lane constants are not held in registers
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (kb * 32 + 8 * (i >> 2) + 4 * g_l + (i & 3) >= valid) s[kb][i] = -INFINITY;
    }
    // maximum of this lane's 32 scores (two chains, one per key block); the check against the reference maximum is
    // local: the two lanes of a query column exchange their maxima only when one of them has to move it
    float mx0, mx1;
    asm("v_max_f32 %0, %1, %2" : "=v"(mx0) : "v"(s[0][0]), "v"(s[0][1]));   // asm: no canonicalising of the MFMA's results
    asm("v_max_f32 %0, %1, %2" : "=v"(mx1) : "v"(s[1][0]), "v"(s[1][1]));
#pragma unroll
    for (int i = 2; i < 16; i += 2) {
      mx0 = fmaxf(fmaxf(mx0, s[0][i]), s[0][i + 1]);
      mx1 = fmaxf(fmaxf(mx1, s[1][i]), s[1][i + 1]);
    }
    const float mxl = fmaxf(mx0, mx1);
    if (__builtin_expect(__builtin_amdgcn_fcmpf(mxl, mthr, 2 /* ogt */) != 0, 0)) {
      const float m_new = fmaxf(m_run[0], partner_max(mxl));
      const float alpha = fast_exp2((m_run[0] - m_new) * c);
      m_run[0] = m_new;
      mthr = m_new + thr;
      mc = m_new * c;
      l_run[0] *= alpha;
      l_odd *= alpha;
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[0][db][i] *= alpha;
    }
    static_for<0, 16>([&](auto j) { softmax_pair(IntC<decltype(j)::value / 8>(), IntC<2 * (decltype(j)::value % 8)>()); });
    __builtin_amdgcn_s_barrier();
  };

  int sk = 0, sv = 0;                                          // K and V stage of the tile whose scores are computed
  plan_copy(it.kt0 + 3);
  m_phase(TagF(), TagT(), 0, PP_VSTAGES - 1, 0);               // "the V stage before tile kt0's"
  v_phase(it.kt0, 0, 0);
  for (int kt = it.kt0 + 1; kt < it.kt1; ++kt) {
    const int sp = sv;
    sk = (sk + 1) & (PP_KSTAGES - 1);
    sv = sv + 1 == PP_VSTAGES ? 0 : sv + 1;
    m_phase(TagT(), TagT(), sk, sp, sv);
    v_phase(kt, sk, sv);
  }
  m_phase(TagT(), TagF(), 0, sv, 0);
  if (grp == 0) __builtin_amdgcn_s_barrier();                  // group 0 waits for group 1's last phase
  l_run[0] += l_odd;
  __syncthreads();
  } else {
    // ================= 4 waves x 64 query rows, one wave per SIMD =================
    // The wave's instruction stream is pipelined over half tiles of 32 keys.  Half step h issues, as ONE stream, the
    // 16 MFMAs of O^T += V^T P^T for half tile h-1, the 16 MFMAs of S^T = K Q^T for half tile h+1, and between
    // consecutive MFMAs a few instructions of the softmax of half tile h.  Every K / V^T fragment read from LDS feeds
    // two MFMAs (the wave's two 32-row query blocks), which halves the LDS traffic per MFMA of the 8-wave form, and
    // the matrix pipe of a SIMD is fed by one wave that never waits for a partner.  Scores and weights alternate
    // between two register sets (A: first half of a tile, B: second half).  One workgroup barrier per tile, between
    // its two half steps: the second one is the first to read the next tile's K.
    bf16x8 qf[2][NKS];
    attn_load_q<D, 2>(P, it, qf, tid);
    static_for<0, 16>([&](auto n) {                             // Q^T goes to its accumulation registers
      constexpr int N = decltype(n)::value;
      w64_set_q<N>(__builtin_bit_cast(u32x4, qf[N / 8][N % 8]));
    });
    w64_zero_o();
    __builtin_amdgcn_s_waitcnt(0x0F70);
    int n_last = 0;                                            // copy instructions sent at the last barrier
    __builtin_amdgcn_s_barrier();

    f32x16 sA[2], sB[2];                                       // S^T of a half tile, per query block
    bf16x8 pA[2][2], pB[2][2];                                 // P^T of a half tile: [query block][16-key chunk]
    u32x2 vl[16], vh[16];
    u32x4 kf[16];
    float alpha[2] = {1.0f, 1.0f};
    bool pending = false;                                      // the accumulators still have to be multiplied by alpha
    // running state per query block: reference maximum m_run, m_run + lazy margin, m_run * scale, and the row sum in two
    // halves (even and odd scores), all kept up to date where the reference maximum moves
    float mthr[2] = {m_run[0] + thr, m_run[1] + thr}, mc[2] = {m_run[0] * c, m_run[1] * c};
    float lsum[2][2] = {{0.0f, 0.0f}, {0.0f, 0.0f}};
    float mx[2][2], ex[16][2];

    auto rescale_pending = [&]() __attribute__((always_inline)) {
      if (__builtin_expect(pending, 0)) w64_rescale(alpha[0], alpha[1]);
      pending = false;
    };
    // softmax step K of the half tile whose scores are in s_cur; weights go to p_new
    auto sm_step = [&](auto kk, auto &s_cur, auto &p_new) __attribute__((always_inline)) {
      constexpr int K = decltype(kk)::value;
      if constexpr (K < 16) {
        constexpr int qb = K >> 3, ch = K & 1, j = (K & 7) >> 1, i = 8 * ch + 2 * j;   // block 0 first: block 1's last MFMA is the younger one
        if constexpr (j == 0) asm("v_max_f32 %0, %1, %2" : "=v"(mx[qb][ch]) : "v"(s_cur[qb][i]), "v"(s_cur[qb][i + 1]));
        else mx[qb][ch] = fmaxf(fmaxf(mx[qb][ch], s_cur[qb][i]), s_cur[qb][i + 1]);
        if constexpr (j == 3) asm volatile("" : "+v"(mx[qb][ch]));   // results stay near their step: the optimizer would sink them to their uses
      } else if constexpr (K == 16) {
        const float m0 = fmaxf(mx[0][0], mx[0][1]), m1 = fmaxf(mx[1][0], mx[1][1]);
        const unsigned long long over = __builtin_amdgcn_fcmpf(m0, mthr[0], 2 /* ogt */) | __builtin_amdgcn_fcmpf(m1, mthr[1], 2);
        if (__builtin_expect(over != 0, 0)) {
          const float mq[2] = {partner_max(m0), partner_max(m1)};
#pragma unroll
          for (int qb = 0; qb < 2; ++qb) {
            const float m_new = fmaxf(m_run[qb], mq[qb]);
            const float a = fast_exp2((m_run[qb] - m_new) * c);
            alpha[qb] = pending ? alpha[qb] * a : a;
            m_run[qb] = m_new;
            mthr[qb] = m_new + thr;
            mc[qb] = m_new * c;
            lsum[qb][0] *= a;
            lsum[qb][1] *= a;
          }
          pending = true;
        }
      } else {
        constexpr int code = w64_bstep(K - W64_BSTEP0), kind = code / 16, u = code % 16;
        constexpr int qb = u / 8, i = (u % 8) * 2;
        if constexpr (kind == 0) {
          ex[u][0] = fmaf(s_cur[qb][i], c, -mc[qb]);
          ex[u][1] = fmaf(s_cur[qb][i + 1], c, -mc[qb]);
          asm volatile("" : "+v"(ex[u][0]), "+v"(ex[u][1]));
        } else if constexpr (kind == 1) {
          ex[u][0] = fast_exp2(ex[u][0]);
          ex[u][1] = fast_exp2(ex[u][1]);
          asm volatile("" : "+v"(ex[u][0]), "+v"(ex[u][1]));
        } else {
          // row sum with plain fp32 adds: a dot-product instruction goes through the matrix pipe and queues there
          lsum[qb][0] += ex[u][0];
          lsum[qb][1] += ex[u][1];
          p_new[qb][i >> 3][i & 7] = (__bf16)ex[u][0];
          p_new[qb][i >> 3][(i & 7) + 1] = (__bf16)ex[u][1];
          asm volatile("" : "+v"(lsum[qb][0]), "+v"(lsum[qb][1]), "+v"(p_new[qb][i >> 3]));
        }
      }
    };
    // One stream: PV part (V^T fragments IV0.. at lane address aVp, weights p_old), QK part (K fragments of key block
    // KB at aK, scores to s_nxt), softmax of s_cur -> p_new spread over the MFMAs, prefetch of V^T fragments IVN.. at aVn.
    auto stream = [&](auto pv, auto qk, auto sm, auto pre, auto iv0, auto kbq, auto ivn, auto &s_cur, auto &s_nxt, auto &p_old,
                      auto &p_new, unsigned aK, unsigned aVp, unsigned aVn) __attribute__((always_inline)) {
      constexpr bool PV = decltype(pv)::value, QK = decltype(qk)::value, SM = decltype(sm)::value, PRE = decltype(pre)::value;
      constexpr int IV0 = decltype(iv0)::value, KB = decltype(kbq)::value, IVN = decltype(ivn)::value;
      using S = W64Stream<PV, QK, PRE>;
      constexpr int NC = S::NC, NSLOT = S::NSLOT;
      auto issue = [&](auto pos) __attribute__((always_inline)) {
        constexpr int PP = decltype(pos)::value;
        if constexpr (PP < S::L) {
          constexpr int kind = S::kind(PP), i = S::idx(PP);
          if constexpr (kind == 0) pp_issue_frag<IV0 + i>(vl, vh, kf, 0u, aVp);
          else if constexpr (kind == 1) pp_issue_frag<16 + i * 2 + KB>(vl, vh, kf, aK, 0u);
          else pp_issue_frag<IVN + i>(vl, vh, kf, 0u, aVn);
        }
      };
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (!PV) static_for<0, PP_RING>([&](auto f) { issue(f); });   // with a PV part the previous half step has sent these
      if constexpr (!PV && SM) asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");   // no MFMA ahead of the first read of the scores
      static_for<0, NSLOT>([&](auto sl) {
        constexpr int SL = decltype(sl)::value, qb = SL % 2;
        if constexpr (NC > 0) {
          constexpr int p = SL / 2;
          if constexpr (qb == 0) pp_wait_lgkm<S::wait_n(p)>();
          constexpr int kind = S::kind(p), i = S::idx(p);
          if constexpr (kind == 0) {
            constexpr int I = IV0 + i;
            const u32x4 a4 = __builtin_shufflevector(vl[I], vh[I], 0, 1, 2, 3);
            w64_mfma_o<qb * 4 + I % 4>(a4, p_old[qb][i / 4]);
          } else {
            if constexpr (i == 0) w64_mfma_s0<qb * 8 + i>(s_nxt[qb], kf[i * 2 + KB]);
            else w64_mfma_s<qb * 8 + i>(s_nxt[qb], kf[i * 2 + KB]);
          }
          if constexpr (qb == 1) issue(IntC<p + PP_RING>());
          __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (SM) {
          static_for<w64_first_step(SL, NSLOT), w64_first_step(SL + 1, NSLOT)>([&](auto kk) { sm_step(kk, s_cur, p_new); });
          __builtin_amdgcn_sched_barrier(0);
        }
      });
      // the PV part is long complete: the accumulators follow the moved maximum before the next half step adds to them
      if constexpr (SM) rescale_pending();
    };
    // Between a tile's two half steps: this wave's rows of tile kt+1 have landed once only the copies of its last such
    // point are outstanding; after the barrier that holds for every wave's rows, and every wave is done with K of tile
    // kt-1 and V of tile kt-2.  The copies of tile kt+3 go into those stages, and the copy after that is planned.
    int sk = 0, sv = 0;                                        // K and V stage of tile kt
    auto tile_sync = [&](int kt) __attribute__((always_inline)) {
      wait_copies(n_last);
      __builtin_amdgcn_s_barrier();
      n_last = 0;
      if (__builtin_expect(ncopy_kt >= 0, 1)) {
        const int snk = (sk + 3) & (PP_KSTAGES - 1);
        const int snv = sv >= 2 ? sv - 2 : sv + PP_VSTAGES - 2;
        n_last = copy_planned(nsrc, ncopy_kt, snk, snv);
      }
      plan_copy(kt + 4);
    };
    auto mask_tail = [&](auto &s_cur, int key0, int kt) __attribute__((always_inline)) {
      const int valid = H.lkv - kt * BK - key0;                 // ragged tail: only the head's last tile
      if (__builtin_expect(valid < 32, 0)) {
        int g_l = g;
        asm volatile("" : "+v"(g_l));                            // rare path: its per-lane constants are not held in registers
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (8 * (i >> 2) + 4 * g_l + (i & 3) >= valid) s_cur[0][i] = s_cur[1][i] = -INFINITY;
      }
    };
    // Every tile runs the same two half steps, so that the loop has one body and every register set one place where
    // it is written.  The ends of an item are absorbed by work whose result is not used: the first half step's PV part
    // multiplies weights that are all zero (with V rows of the item's first tile), the last one's QK part computes
    // scores of a tile that does not exist from whatever its K stage holds (16 MFMAs each, of ~64 per tile).
    // first half step of tile kt: softmax of its keys 0..31 (set A); PV of tile kt-1's keys 32..63; QK of its keys 32..63
    auto half0 = [&](int kt, bool first) __attribute__((always_inline)) {
      if (__builtin_expect(has_rows, 1)) {
        mask_tail(sA, 0, kt);
        const unsigned aK = ak + (unsigned)(sk * PP_TILE_BYTES);
        const unsigned aVn = av + (unsigned)(sv * PP_TILE_BYTES);
        const unsigned aVp = first ? aVn : av + (unsigned)((sv == 0 ? PP_VSTAGES - 1 : sv - 1) * PP_TILE_BYTES);
        stream(TagT(), TagT(), TagT(), TagT(), IntC<8>(), IntC<1>(), IntC<0>(), sA, sB, pB, pA, aK, aVp, aVn);
      }
    };
    // second half step of tile kt: softmax of its keys 32..63 (set B); PV of its keys 0..31; QK of tile kt+1's keys 0..31
    auto half1 = [&](int kt) __attribute__((always_inline)) {
      if (__builtin_expect(has_rows, 1)) {
        mask_tail(sB, 32, kt);
        const unsigned aK = ak + (unsigned)(((sk + 1) & (PP_KSTAGES - 1)) * PP_TILE_BYTES);
        const unsigned aV = av + (unsigned)(sv * PP_TILE_BYTES);
        stream(TagT(), TagT(), TagT(), TagT(), IntC<0>(), IntC<0>(), IntC<8>(), sB, sA, pA, pB, aK, aV, aV);
      }
      sk = (sk + 1) & (PP_KSTAGES - 1);
      sv = sv + 1 == PP_VSTAGES ? 0 : sv + 1;
    };

    plan_copy(it.kt0 + 3);
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
      for (int ch = 0; ch < 2; ++ch)
#pragma unroll
        for (int i = 0; i < 8; ++i) pB[qb][ch][i] = (__bf16)0.0f;
    if (__builtin_expect(has_rows, 1))                         // S^T of tile kt0's keys 0..31; V^T fragments for the first (empty) PV part
      stream(TagF(), TagT(), TagF(), TagT(), IntC<0>(), IntC<0>(), IntC<8>(), sA, sA, pA, pA, ak, 0u, av);
    for (int kt = it.kt0; kt < it.kt1; ++kt) {
      half0(kt, kt == it.kt0);
      tile_sync(kt);
      half1(kt);
    }
    if (__builtin_expect(has_rows, 1)) {                       // PV of the last tile's keys 32..63 (its V stage is the one before sv now)
      const unsigned aVp = av + (unsigned)((sv == 0 ? PP_VSTAGES - 1 : sv - 1) * PP_TILE_BYTES);
      stream(TagT(), TagF(), TagF(), TagF(), IntC<8>(), IntC<0>(), IntC<0>(), sA, sA, pB, pB, 0u, aVp, 0u);
    }
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");           // the last MFMA has written the accumulators back
    static_for<0, 8>([&](auto n) { o[decltype(n)::value / 4][decltype(n)::value % 4] = w64_get_o<decltype(n)::value>(); });
    l_run[0] = lsum[0][0] + lsum[0][1];
    l_run[1] = lsum[1][0] + lsum[1][1];
    __syncthreads();
  }
  const AttnParams Pe = load_params();                         // read again: nothing of it is held through the loop above
  attn_epilogue<D, NQB, NW>(Pe, it, o, m_run, l_run, (float *)&sK[0][0], &sFlag, tid);
  if (__builtin_expect(Pe.block_trace != nullptr, 0) && tid0 == 0) {
    const long long now = wall_clock64();
    sTrace[0] += now - sTrace[2];
    sTrace[2] = now;                                           // doubles as "last end"
    sTrace[3] += 1;
    sTrace[4] += clock64() - sTrace[5];
  }
  }
  {
    long long *bt = load_params().block_trace;
    if (__builtin_expect(bt != nullptr, 0) && tid0 == 0) {
      bt = as_global(bt) + (size_t)blockIdx.x * 8;
      bt[0] = sTrace[0]; bt[1] = sTrace[1]; bt[2] = sTrace[2]; bt[3] = sTrace[3]; bt[4] = sTrace[4];
    }
  }
  int32_t *tickets = load_params().tickets;
  if (tickets != nullptr && tid0 == 0) {
    const int done = atomicAdd(&tickets[PF_NUM_XCD], 1);
    if (done == (int)gridDim.x - 1) {
      for (int x = 0; x <= PF_NUM_XCD; ++x) atomicExch(&tickets[x], 0);
    }
  }
}

// Workgroups of the pipelined kernel that are resident at once: its LDS rings leave room for one per compute unit.
static int pp_resident_workgroups() {
  static int n_cu[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (n_cu[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
    n_cu[dev] = n;
  }
  return n_cu[dev];
}

// Diagnostics: where the resident workgroups of the pipelined kernel write their busy times (see pf_set_block_trace).
static long long *g_block_trace = nullptr;
static size_t g_block_trace_bytes = 0;
extern "C" int pf_set_block_trace(void *dev_buffer, size_t bytes) {
  if (dev_buffer && ((((uintptr_t)dev_buffer) & 7u) || bytes < 64)) return PF_ERR_INVALID_ARG;
  g_block_trace = (long long *)dev_buffer;
  g_block_trace_bytes = dev_buffer ? bytes : 0;
  return PF_OK;
}

static int launch_attn(const AttnParams &P, int head_dim, int variant, int n_blocks, hipStream_t stream) {
  if (head_dim == 128 && variant == 1)
    hipLaunchKernelGGL((pf_attn_pp_kernel<128, 8>), dim3(P.tickets ? pf_min(n_blocks, pp_resident_workgroups()) : n_blocks),
                       dim3(8 * 64), 0, stream, P);
  else if (head_dim == 128 && variant == 2)
    hipLaunchKernelGGL((pf_attn_pp_kernel<128, 4>), dim3(P.tickets ? pf_min(n_blocks, pp_resident_workgroups()) : n_blocks),
                       dim3(4 * 64), 0, stream, P);
  else if (head_dim == 128 && variant == 0)
    hipLaunchKernelGGL((pf_attn_kernel<128>), dim3(n_blocks), dim3(ATT_THREADS), 0, stream, P);
  else if (head_dim == 64 && variant == 0)
    hipLaunchKernelGGL((pf_attn_kernel<64>), dim3(n_blocks), dim3(ATT_THREADS), 0, stream, P);
  else
    return PF_ERR_UNSUPPORTED;                      // kernel 1 exists for head_dim 128 only
  return hipGetLastError() == hipSuccess ? PF_OK : PF_ERR_HIP;
}

// Strides of the chunk tensors are usable when rows are 16-byte aligned, at least head_dim long, and the
// (head, token) rows do not overlap: heads outermost or tokens outermost.
bool pf_chunk_layout_ok(const pf_chunk_layout *lay, int n_heads, int tokens, int head_dim) {
  if (!lay) return true;
  const long long ts = lay->token_stride, hs = lay->head_stride;
  if (ts < head_dim || hs < head_dim || (ts & 7) || (hs & 7)) return false;
  if (ts >= (1ll << 24) || hs > (1ll << 40)) return false;   // 64 rows of a tile stay inside a 32-bit byte offset
  return hs >= (long long)tokens * ts || ts >= (long long)n_heads * hs;
}

static int attn_fwd_impl(const pf_pool *pool, const pf_index *index, const void *q, const void *k_cur,
                         const void *v_cur, void *out, int q_tokens, float softmax_scale, void *workspace,
                         size_t workspace_bytes, const pf_chunk_layout *layout, void *stream) {
  const int rc = pf_validate_pool(pool);
  if (rc != PF_OK) return rc;
  if (q_tokens >= 1 && !pf_chunk_layout_ok(layout, pool->n_heads, q_tokens, pool->head_dim)) return PF_ERR_INVALID_ARG;
  if (!index || !q || !k_cur || !v_cur || !out || q_tokens < 1) return PF_ERR_INVALID_ARG;
  if ((((uintptr_t)q) | ((uintptr_t)k_cur) | ((uintptr_t)v_cur) | ((uintptr_t)out) | ((uintptr_t)workspace)) & 15u)
    return PF_ERR_INVALID_ARG;
  if (!index->sel_count || !index->sel_slots || !index->work) return PF_ERR_INVALID_ARG;
  if (index->q_tokens != q_tokens || index->T_built != pool->T_host) return PF_ERR_INVALID_ARG;  // stale index
  if (index->variant < 0 || index->variant >= PF_NUM_VARIANTS || index->n_blocks < 1) return PF_ERR_INVALID_ARG;
  if (!(softmax_scale >= 0.0f) || softmax_scale > 1.0e6f) return PF_ERR_INVALID_ARG;
  const int bq = pf_variant_bq(index->variant);
  const size_t need = (size_t)index->n_partials * pf_partial_bytes(bq, pool->head_dim);
  if (need > 0 && (!workspace || workspace_bytes < need)) return PF_ERR_INVALID_ARG;

  const int n_qt = pf_ceil_div(q_tokens, bq);
  const PfWorkLayout L = pf_work_layout(pool->n_heads, n_qt, index->n_blocks);
  char *w = (char *)index->work;
  AttnParams P;
  P.q = (const __bf16 *)q;
  P.k_cur = (const __bf16 *)k_cur;
  P.v_cur = (const __bf16 *)v_cur;
  P.k_pool = (const __bf16 *)pool->k_pool;
  P.v_pool = (const __bf16 *)pool->v_pool;
  P.out = (__bf16 *)out;
  P.sel_count = index->sel_count;
  P.sel_slots = index->sel_slots;
  P.items = (const PfWorkItem *)(w + L.items_off);
  P.counters = (int32_t *)(w + L.counters_off);
  const bool queue = pf_attn_queue_mode(index->variant);
  P.tickets = queue ? P.counters + (size_t)pool->n_heads * n_qt : nullptr;
  P.queue_len = index->n_blocks / PF_NUM_XCD;
  P.workspace = (float *)workspace;
  P.max_sel = index->max_sel;
  P.tpf = pool->tokens_per_frame;
  P.q_tokens = q_tokens;
  P.n_qt = n_qt;
  P.block_trace = (queue && g_block_trace_bytes >= (size_t)pf_min(index->n_blocks, pp_resident_workgroups()) * 64) ? g_block_trace : nullptr;
  P.tok_stride = layout ? layout->token_stride : pool->head_dim;
  P.head_stride = layout ? layout->head_stride : (long long)q_tokens * pool->head_dim;
  const float scale = softmax_scale > 0.0f ? softmax_scale : 1.0f / sqrtf((float)pool->head_dim);
  P.scale_log2 = scale * 1.4426950408889634f;
  hipStream_t st = (hipStream_t)stream;
  return launch_attn(P, pool->head_dim, index->variant, index->n_blocks, st);
}

extern "C" int pf_ragged_attn_fwd(const pf_pool *pool, const pf_index *index, const void *q, const void *k_cur,
                                  const void *v_cur, void *out, int q_tokens, float softmax_scale,
                                  void *workspace, size_t workspace_bytes, void *stream) {
  return attn_fwd_impl(pool, index, q, k_cur, v_cur, out, q_tokens, softmax_scale, workspace, workspace_bytes, nullptr, stream);
}

// ---------------------------------------------------------------------------------------------------
// The same launch for callers that cannot allocate device memory or bring a workspace (code under graph capture,
// tight serving loops): the partial results of split heads go to a fixed array in the library's own device image.
// Every GPU holds its own copy of the array at its own address, looked up once per device.
// ---------------------------------------------------------------------------------------------------
constexpr size_t PF_STATIC_SCRATCH_BYTES = 160ull << 20;
static __device__ __align__(256) unsigned char scratch[PF_STATIC_SCRATCH_BYTES];

static int static_scratch_ptr(void **out) {
  static std::mutex mu;
  static void *ptr_of[64] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return PF_ERR_HIP;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr_of[dev]) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return PF_ERR_HIP;
    ptr_of[dev] = p;
  }
  *out = ptr_of[dev];
  return PF_OK;
}

extern "C" int pf_ragged_attn_fwd_static(const pf_pool *pool, const pf_index *index, const void *q, const void *k_cur,
                                         const void *v_cur, void *out, int q_tokens, float softmax_scale, void *stream) {
  if (!pool || !index) return PF_ERR_INVALID_ARG;
  if (index->variant < 0 || index->variant >= PF_NUM_VARIANTS || index->n_partials < 0) return PF_ERR_INVALID_ARG;
  if (pool->head_dim != 64 && pool->head_dim != 128) return PF_ERR_UNSUPPORTED;
  const size_t need = (size_t)index->n_partials * pf_partial_bytes(pf_variant_bq(index->variant), pool->head_dim);
  if (need > PF_STATIC_SCRATCH_BYTES) return PF_ERR_CAPACITY;
  void *ws = nullptr;
  const int rc = static_scratch_ptr(&ws);
  if (rc != PF_OK) return rc;
  return attn_fwd_impl(pool, index, q, k_cur, v_cur, out, q_tokens, softmax_scale, ws, PF_STATIC_SCRATCH_BYTES, nullptr, stream);
}

extern "C" int pf_ragged_attn_fwd_strided(const pf_pool *pool, const pf_index *index, const void *q, const void *k_cur,
                                          const void *v_cur, void *out, int q_tokens, float softmax_scale,
                                          void *workspace, size_t workspace_bytes, const pf_chunk_layout *layout,
                                          void *stream) {
  if (!layout) return PF_ERR_INVALID_ARG;
  return attn_fwd_impl(pool, index, q, k_cur, v_cur, out, q_tokens, softmax_scale, workspace, workspace_bytes, layout, stream);
}
