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
  // optional diagnostics (pf_set_block_trace): per resident workgroup {busy, first start, last end, items}, in ticks of the
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

// Copies this wave's 8 rows (wave*8 ..) of tile kt of one tensor into the stage at LDS pointer `stage`.
// Returns the number of copy instructions issued (2 when the tile is contiguous in memory, else 8).
// voff[h]: per-lane source offset inside the 4-row group h of this wave, see pp_group_voff.
template <bool IS_V>
__device__ __forceinline__ unsigned pp_group_voff(int lane, int row0) {
  const int rr = lane >> 4, p = lane & 15;
  return (unsigned)(rr * 256 + ((p ^ pp_swz(IS_V, row0 + rr)) << 4));
}
template <bool IS_V>
__device__ __forceinline__ int pp_copy_rows_slow(int kt, const HeadKV &H, char *stage, int wave, int lane) {
  typedef const __attribute__((address_space(1))) void *gptr_t;
  typedef __attribute__((address_space(3))) void *lptr_t;
  constexpr int D = 128;
  const int last = H.lkv - 1 - kt * PF_BK;
  asm volatile("" : "+v"(lane));                    // rare path: its per-lane offsets are worked out here, not held in registers through the loop
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    const int row = wave * 8 + r;
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
  return 8;
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

template <int D>
__global__ __launch_bounds__(PP_WAVES * 64, 2) void pf_attn_pp_kernel(AttnParams) {
  static_assert(D == 128, "tile layouts are written for 256-byte rows");
  constexpr int BK = PF_BK;
  constexpr int NKS = D / 16, NDB = D / 32;
  typedef const __attribute__((address_space(1))) void *gptr_t;
  typedef __attribute__((address_space(3))) void *lptr_t;

  // K ring, then V ring; the epilogue reuses the same memory to stage the output rows
  static_assert((PP_KSTAGES + PP_VSTAGES) * PP_TILE_BYTES >= attn_stage_floats(PP_WAVES * 32, D) * 4, "output staging fits");
  __shared__ __attribute__((aligned(1024))) char smem[(PP_KSTAGES + PP_VSTAGES) * PP_TILE_BYTES];
  __shared__ int32_t sFlag;
  __shared__ int32_t sNext;
  __shared__ long long sTrace[4];                              // busy ticks, first start, this item's start, items (thread 0 only)
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
  if (tid0 == 0) sTrace[0] = sTrace[1] = sTrace[2] = sTrace[3] = 0;
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
  }
  int tid = tid0;
  asm volatile("" : "+v"(tid));               // per-lane constants are worked out anew for each item, not kept across the loop
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wave >> 2;
  const int l32 = lane & 31, g = lane >> 5;
  HeadKV H;
  attn_setup_head<D>(P, it, H, tid);
  f32x16 o[1][NDB];
  float m_run[1], l_run[1];
  attn_zero<D, 1>(o, m_run, l_run);
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
  // per-lane source offsets inside a 4-row copy group; the wave's second group (rows + 4) differs in one bit
  // for K and not at all for V
  const unsigned vofK0 = pp_group_voff<false>(lane, wave * 8), vofK1 = vofK0 ^ 64u, vofV = pp_group_voff<true>(lane, wave * 8);
  const int wrow_bytes = wave * 8 * 256;                       // this wave's first row inside a tile

  // One 4-row group: h = 0, 1 (K), 2, 3 (V).  The copies are buffer loads: the tile's first row is the base of a
  // 16 KB buffer descriptor (scalar registers), the wave's rows are a scalar offset, the lane's chunk a 32-bit
  // vector offset that never changes, and the second group is the instruction's immediate offset (it moves the
  // LDS destination along with the source).  Next to MFMAs this form costs almost nothing, whereas a global
  // load with a 64-bit address per lane held up the SIMD for ~65 cycles per instruction (measured).
  auto copy_group_at = [&](const __bf16 *kbase, const __bf16 *vbase, int snk, int snv, int h) {
    constexpr unsigned RSRC_FLAGS = 0x00020000u;               // raw buffer, 32-bit data format
    if (h < 2) {
      const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc((void *)kbase, 0, PP_TILE_BYTES, RSRC_FLAGS);
      lptr_t dst = (lptr_t)(&sK[snk][wrow_bytes]);
      if (h == 0) __builtin_amdgcn_raw_ptr_buffer_load_lds(r, dst, 16, vofK0, wrow_bytes, 0, 0);
      else __builtin_amdgcn_raw_ptr_buffer_load_lds(r, dst, 16, vofK1, wrow_bytes, 1024, 0);
    } else {
      const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc((void *)vbase, 0, PP_TILE_BYTES, RSRC_FLAGS);
      lptr_t dst = (lptr_t)(&sV[snv][wrow_bytes]);
      if (h == 2) __builtin_amdgcn_raw_ptr_buffer_load_lds(r, dst, 16, vofV, wrow_bytes, 0, 0);
      else __builtin_amdgcn_raw_ptr_buffer_load_lds(r, dst, 16, vofV, wrow_bytes, 1024, 0);
    }
  };
  auto copy_group = [&](const TileSrc &src, int snk, int snv, int h) { copy_group_at(src.kb, src.vb, snk, snv, h); };
  // The same for a chunk tile whose token rows are cur_stride elements apart (the model's [tokens][heads][D]
  // layout): the lane's row is part of its vector offset, the wave's first row and the second group are scalar
  // offsets, and the second group's LDS destination moves by hand.
  const unsigned row_b = (unsigned)(H.cur_stride * 2);         // bytes between chunk token rows (< 2^25, checked on the host)
  const unsigned sofK0 = (unsigned)(((vofK0 & 0xffu) + (lane >> 4) * row_b)), sofK1 = (unsigned)(((vofK1 & 0xffu) + (lane >> 4) * row_b));
  const unsigned sofV = (unsigned)(((vofV & 0xffu) + (lane >> 4) * row_b));
  auto copy_group_strided = [&](const TileSrc &src, int snk, int snv, int h) {
    constexpr unsigned RSRC_FLAGS = 0x00020000u;
    const unsigned soff = (unsigned)(wave * 8 + 4 * (h & 1)) * row_b;
    const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc((void *)(h < 2 ? src.kb : src.vb), 0, (int)(PF_BK * row_b), RSRC_FLAGS);
    lptr_t dst = h < 2 ? (lptr_t)(&sK[snk][wrow_bytes + (h & 1) * 1024]) : (lptr_t)(&sV[snv][wrow_bytes + (h & 1) * 1024]);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, dst, 16, h == 0 ? sofK0 : h == 1 ? sofK1 : sofV, soff, 0, 0);
  };
  // A tile made of two dense runs (it crosses a frame border): a 4-row group lies in the first run, in the second, or
  // (when the border is not a multiple of 4 rows into the tile) in both, and then each run's lanes copy under their
  // own execution mask: the LDS address of such a copy follows the lane number, so masked-off lanes leave their
  // 16 bytes to the other instruction.  Returns the number of copy instructions issued.
  auto copy_tile_split = [&](const TileSrc &src, int snk, int snv) __attribute__((always_inline)) -> int {
    int n = 0;
    const __bf16 *ka = src.kb, *va = src.vb, *kb2 = src.kb2, *vb2 = src.vb2;
    const int n1 = src.n1;
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      const int row0 = wave * 8 + (h & 1) * 4;
      if (row0 + 4 <= n1) {
        copy_group_at(ka, va, snk, snv, h);
        n += 1;
      } else if (row0 >= n1) {
        copy_group_at(kb2, vb2, snk, snv, h);
        n += 1;
      } else {
        int lane_l = lane;
        asm volatile("" : "+v"(lane_l));                        // rare: its lane test is not held in a register through the loop
        if (row0 + (lane_l >> 4) < n1) copy_group_at(ka, va, snk, snv, h);
        else copy_group_at(kb2, vb2, snk, snv, h);
        n += 2;
      }
    }
    return n;
  };
  // whole tile at once (prologue; tiles that cross a frame border or hold the ragged end go row by row here)
  auto copy_tile_now = [&](int kt, const TilePos &tp, int snk, int snv) -> int {
    const TileSrc src = tile_src(kt, tp, H, D);
    if (src.simple) {
#pragma unroll
      for (int h = 0; h < 4; ++h) {
        if (src.strided) copy_group_strided(src, snk, snv, h);
        else copy_group(src, snk, snv, h);
      }
      return 4;
    }
    pp_copy_rows_slow<false>(kt, H, sK[snk], wave, lane);
    pp_copy_rows_slow<true>(kt, H, sV[snv], wave, lane);
    return 16;
  };
  // "Everything but the copies of the last vector phase has landed": at most 4 vector-memory operations may be
  // outstanding (a contiguous tile's copies).  When the last vector phase sent a tile row by row (16 copies, at
  // a frame border) this also waits for 12 of those, which were sent a whole matrix phase ago; when it sent
  // nothing, the older copies are all that is in flight.
  auto wait_copies = [&](int n) {
    __builtin_amdgcn_s_waitcnt(0x0F70 | 4);
    if (__builtin_expect(n == 0, 0)) __builtin_amdgcn_s_waitcnt(0x0F70);
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

  // ---- plan of the next copy (made in one vector phase and carried out at the start of the next, so the
  // scalar load of a frame's slot has a whole tile time to arrive) ----
  TileSrc nsrc;
  nsrc.kb = nsrc.vb = nsrc.kb2 = nsrc.vb2 = nullptr;
  nsrc.simple = nsrc.split = false;
  nsrc.n1 = 0;
  int ncopy_kt = -1;                                           // tile planned for the next copy, -1: none
  int run_left = 0;                                            // tiles after the planned one that continue its source run
  long long run_step = 0;                                      // elements from one tile of the run to the next
  auto plan_copy = [&](int kt_target) {
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
  const bool has_rows = it.q0 + wave * 32 < P.q_tokens;

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
      if (__builtin_expect(nsrc.simple && !nsrc.strided, 1)) {
#pragma unroll
        for (int h = 0; h < 4; ++h) copy_group(nsrc, snk, snv, h);
        n_last = 4;
      } else if (nsrc.simple) {
#pragma unroll
        for (int h = 0; h < 4; ++h) copy_group_strided(nsrc, snk, snv, h);
        n_last = 4;
      } else if (nsrc.split) {
        n_last = copy_tile_split(nsrc, snk, snv);
      } else {
        pp_copy_rows_slow<false>(ncopy_kt, H, sK[snk], wave, lane);
        pp_copy_rows_slow<true>(ncopy_kt, H, sV[snv], wave, lane);
        n_last = 16;
      }
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
    float mx = s[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[kb][i]);
    mx = partner_max(mx);
    if (__builtin_expect(__builtin_amdgcn_ballot_w64(mx > m_run[0] + thr) != 0, 0)) {
      const float m_new = fmaxf(m_run[0], mx);
      const float alpha = fast_exp2((m_run[0] - m_new) * c);
      m_run[0] = m_new;
      l_run[0] *= alpha;
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[0][db][i] *= alpha;
    }
    const float mc = m_run[0] * c;
    // row sum with plain fp32 adds: a dot-product instruction goes through the matrix pipe and queues there
    // behind the other group's MFMAs (measured: ~54 cycles each next to a saturated MFMA stream, against 4 alone)
    float ls0 = 0.f, ls1 = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        const float e0 = fast_exp2(fmaf(s[kb][i], c, -mc));
        const float e1 = fast_exp2(fmaf(s[kb][i + 1], c, -mc));
        ls0 += e0;
        ls1 += e1;
        pf[kb * 2 + (i >> 3)][i & 7] = (__bf16)e0;
        pf[kb * 2 + (i >> 3)][(i & 7) + 1] = (__bf16)e1;
      }
    l_run[0] += ls0 + ls1;
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
  __syncthreads();
  const AttnParams Pe = load_params();                         // read again: nothing of it is held through the loop above
  attn_epilogue<D, 1, PP_WAVES>(Pe, it, o, m_run, l_run, (float *)&sK[0][0], &sFlag, tid);
  if (__builtin_expect(Pe.block_trace != nullptr, 0) && tid0 == 0) {
    const long long now = wall_clock64();
    sTrace[0] += now - sTrace[2];
    sTrace[2] = now;                                           // doubles as "last end"
    sTrace[3] += 1;
  }
  }
  {
    long long *bt = load_params().block_trace;
    if (__builtin_expect(bt != nullptr, 0) && tid0 == 0) {
      bt = as_global(bt) + (size_t)blockIdx.x * 4;
      bt[0] = sTrace[0]; bt[1] = sTrace[1]; bt[2] = sTrace[2]; bt[3] = sTrace[3];
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
  if (dev_buffer && ((((uintptr_t)dev_buffer) & 7u) || bytes < 32)) return PF_ERR_INVALID_ARG;
  g_block_trace = (long long *)dev_buffer;
  g_block_trace_bytes = dev_buffer ? bytes : 0;
  return PF_OK;
}

static int launch_attn(const AttnParams &P, int head_dim, int variant, int n_blocks, hipStream_t stream) {
  if (head_dim == 128 && variant == 1)
    hipLaunchKernelGGL((pf_attn_pp_kernel<128>), dim3(P.tickets ? pf_min(n_blocks, pp_resident_workgroups()) : n_blocks),
                       dim3(PP_WAVES * 64), 0, stream, P);
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
  P.block_trace = (queue && g_block_trace_bytes >= (size_t)pf_min(index->n_blocks, pp_resident_workgroups()) * 32) ? g_block_trace : nullptr;
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
