// Ragged-cache attention forward (Sec. 4.3; Eq. 1 per head over [selected frames || chunk]).
//
// One launch per layer.  A workgroup (4 waves) owns BQ = 128*NQB query rows of one head and a run of
// 64-key tiles of that head's ragged key sequence; heads with many keys are cut into several runs
// whose partial results are merged by the last workgroup to finish (no spinning).
//
// Per tile, on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulate):
//   S^T = K . Q^T     A operand = K rows from LDS, B operand = Q^T held in registers
//   O^T += V^T . P^T  A operand = V^T via the LDS transpose read, B operand = P^T straight from the
//                     S^T accumulators (the key permutation of the accumulator layout is applied to
//                     the V rows instead, since a sum over keys has no order)
// so every lane owns ONE query column: the running maximum and sum of the online softmax live in
// one register each and need a single exchange with lane^32 per tile.
#include "pf_internal.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;   // 16-byte register quad

constexpr int ATT_THREADS = 256;
constexpr int ATT_WAVES = 4;

struct AttnParams {
  const __bf16 *q, *k_cur, *v_cur, *k_pool, *v_pool;
  __bf16 *out;
  const int32_t *sel_count, *sel_slots;
  const PfWorkItem *items;
  int32_t *counters;
  float *workspace;
  int max_sel, tpf, q_tokens, n_qt;
  float scale_log2;     // softmax scale * log2(e)
};

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
// and read with device-scope (relaxed atomic) 64-bit accesses, which go through to the memory side that all
// dies share; no L2 write-back fence is needed, only the wait for the stores' completion before the arrival
// counter is bumped.
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

// Global -> register load of one 64-key tile of a head's ragged key sequence
// [selected frames || chunk].  (j0, r0) locate the tile's first key: frame index and offset in it, j0 = n_sel
// meaning the chunk.  Common case (tile inside one frame, no ragged tail): one wave-uniform base pointer plus
// a per-thread constant offset.  Otherwise each row is located on its own.
template <int D, int NP, int RPP>
__device__ __forceinline__ void attn_load_tile(u32x4 (&kreg)[NP], u32x4 (&vreg)[NP], int kt, int j0, int r0, int n_sel,
                                               int tpf, int lkv, int hist_tokens, int lrow, int lchunk,
                                               unsigned thread_off, const __bf16 *k_pool, const __bf16 *v_pool,
                                               const __bf16 *kcur, const __bf16 *vcur, const int32_t *slots_h) {
  constexpr unsigned PASS_BYTES = RPP * D * 2;
  const int last = lkv - 1 - kt * PF_BK;                     // last valid row of this tile
  const bool in_hist = j0 < n_sel;
  const bool simple = last >= PF_BK - 1 && (!in_hist || r0 + PF_BK <= tpf);
  if (simple) {
    const char *kb, *vb;
    if (in_hist) {
      const size_t e = ((size_t)slots_h[j0] * tpf + r0) * D;
      kb = (const char *)(k_pool + e);
      vb = (const char *)(v_pool + e);
    } else {
      kb = (const char *)(kcur + (size_t)r0 * D);
      vb = (const char *)(vcur + (size_t)r0 * D);
    }
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      kreg[p] = *(const u32x4 *)(kb + (thread_off + p * PASS_BYTES));
      vreg[p] = *(const u32x4 *)(vb + (thread_off + p * PASS_BYTES));
    }
  } else {
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      const int t = kt * PF_BK + pf_min(lrow + p * RPP, last);    // rows past the end re-read the last key
      size_t e;
      const __bf16 *kb = k_pool, *vb = v_pool;
      if (t >= hist_tokens) {
        e = (size_t)(t - hist_tokens) * D;
        kb = kcur;
        vb = vcur;
      } else {
        const int j = t / tpf;
        e = ((size_t)slots_h[j] * tpf + (t - j * tpf)) * D;
      }
      kreg[p] = *(const u32x4 *)(kb + e + lchunk * 8);
      vreg[p] = *(const u32x4 *)(vb + e + lchunk * 8);
    }
  }
}

template <int NP, int RPP, int KS, int VS>
__device__ __forceinline__ void attn_store_tile(const u32x4 (&kreg)[NP], const u32x4 (&vreg)[NP], __bf16 *sK, __bf16 *sV,
                                                int lrow, int lchunk) {
#pragma unroll
  for (int p = 0; p < NP; ++p) {
    const int row = lrow + p * RPP;
    *(u32x4 *)(&sK[row * KS + lchunk * 8]) = kreg[p];
    *(u32x4 *)(&sV[row * VS + lchunk * 8]) = vreg[p];
  }
}

template <int D, int NQB>
__global__ __launch_bounds__(ATT_THREADS, (NQB == 1 ? 2 : 1)) void pf_attn_kernel(AttnParams P) {
  constexpr int BQ = ATT_WAVES * 32 * NQB;
  constexpr int BK = PF_BK;
  constexpr int KS = D + 8;            // K row stride in LDS (elements): +16 B so 32 rows spread over banks
  constexpr int VS = D + 32;           // V row stride: +64 B so the 4 rows of one transpose read do not collide
  constexpr int CPR = D / 8;           // 16-byte chunks per row
  constexpr int RPP = ATT_THREADS / CPR;   // rows loaded per pass
  constexpr int NP = BK / RPP;         // passes per tile
  constexpr int NKS = D / 16;          // k-steps of S^T = K Q^T
  constexpr int NDB = D / 32;          // 32-row blocks of O^T
  constexpr int NKB = BK / 32;         // 32-key blocks of S^T
  constexpr int NS16 = BK / 16;        // k-steps of O^T += V^T P^T

  __shared__ __attribute__((aligned(16))) __bf16 sK[2][BK * KS];
  __shared__ __attribute__((aligned(16))) __bf16 sV[2][BK * VS];
  __shared__ int32_t sFlag;

  const PfWorkItem it = P.items[blockIdx.x];
  if (it.head < 0) return;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const int h = it.head;
  const int n_sel = P.sel_count[h];
  const int hist_tokens = n_sel * P.tpf;
  const int lkv = hist_tokens + P.q_tokens;
  const int tpf = P.tpf;

  // ---- Q^T fragments: lane (l32, g) holds, for its query row, d = 16*ks + 8*g .. +7 ----
  bf16x8 qf[NQB][NKS];
  const __bf16 *qh = P.q + (size_t)h * P.q_tokens * D;
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const int row = pf_min(it.q0 + (wave * NQB + qb) * 32 + l32, P.q_tokens - 1);
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) qf[qb][ks] = *(const bf16x8 *)(qh + (size_t)row * D + ks * 16 + 8 * g);
  }

  // ---- K/V tile loader: thread (lrow, lchunk) copies one 16-byte chunk of NP rows per tile ----
  // j0 / r0 (wave-uniform) = frame index (n_sel = the chunk) and offset in it of the tile's first key.
  const int lrow = tid / CPR, lchunk = tid % CPR;
  const __bf16 *kcur = P.k_cur + (size_t)h * P.q_tokens * D;
  const __bf16 *vcur = P.v_cur + (size_t)h * P.q_tokens * D;
  const int32_t *slots_h = P.sel_slots + (size_t)h * P.max_sel;
  u32x4 kreg[NP], vreg[NP];
  int j0, r0;
  {
    const int t0 = it.kt0 * BK;
    if (t0 >= hist_tokens) { j0 = n_sel; r0 = t0 - hist_tokens; }
    else { j0 = t0 / tpf; r0 = t0 - j0 * tpf; }
  }
  const unsigned thread_off = (unsigned)((lrow * D + lchunk * 8) * 2);      // bytes, row lrow of a tile
  constexpr unsigned PASS_BYTES = RPP * D * 2;
  // ---- accumulators ----
  f32x16 o[NQB][NDB];
  float m_run[NQB], l_run[NQB];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    m_run[qb] = -3.0e38f;
    l_run[qb] = 0.0f;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[qb][db][i] = 0.0f;
  }

  const int k_lane = l32 * KS + 8 * g;                                           // K operand: row l32, d 8g..
  const int v_lane = (4 * g + ((lane & 15) >> 2)) * VS + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  const float c = P.scale_log2;

  attn_load_tile<D, NP, RPP>(kreg, vreg, it.kt0, j0, r0, n_sel, tpf, lkv, hist_tokens, lrow, lchunk, thread_off,
                              P.k_pool, P.v_pool, kcur, vcur, slots_h);
  attn_store_tile<NP, RPP, KS, VS>(kreg, vreg, sK[0], sV[0], lrow, lchunk);
  __syncthreads();

  int buf = 0;
  for (int kt = it.kt0; kt < it.kt1; ++kt) {
    const bool more = kt + 1 < it.kt1;
    if (more) {
      r0 += BK;                                            // position of the next tile's first key
      if (j0 < n_sel) {
        if (tpf >= BK) { if (r0 >= tpf) { r0 -= tpf; ++j0; } }
        else { const int adv = r0 / tpf; r0 -= adv * tpf; j0 += adv; }
        if (j0 > n_sel) { r0 += (j0 - n_sel) * tpf; j0 = n_sel; }
      }
      attn_load_tile<D, NP, RPP>(kreg, vreg, kt + 1, j0, r0, n_sel, tpf, lkv, hist_tokens, lrow, lchunk, thread_off,
                                  P.k_pool, P.v_pool, kcur, vcur, slots_h);
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
    const int valid = lkv - kt * BK;
    if (valid < BK) {
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

    // ---- online softmax (per lane: one query column) ----
    bf16x8 pf[NQB][NS16];
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      float mx = s[qb][0][0];
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[qb][kb][i]);
      mx = partner_max(mx);
      const float m_new = fmaxf(m_run[qb], mx);
      const float alpha = fast_exp2((m_run[qb] - m_new) * c);
      m_run[qb] = m_new;
      const float mc = m_new * c;
      float rs = 0.0f;
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float p = fast_exp2(fmaf(s[qb][kb][i], c, -mc));
          rs += p;
          pf[qb][kb * 2 + (i >> 3)][i & 7] = (__bf16)p;
        }
      l_run[qb] = l_run[qb] * alpha + rs;
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[qb][db][i] *= alpha;
    }

    // ---- O^T += V^T P^T ----
#pragma unroll
    for (int s16 = 0; s16 < NS16; ++s16) {
#pragma unroll
      for (int db = 0; db < NDB; ++db) {
        const __bf16 *vp = &sV[buf][v_lane + s16 * 16 * VS + db * 32];
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(vp));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(vp + 8 * VS));
        const s16x8 av = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        const bf16x8 a = __builtin_bit_cast(bf16x8, av);
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb)
          o[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[qb][s16], o[qb][db], 0, 0, 0);
      }
    }

    if (more) attn_store_tile<NP, RPP, KS, VS>(kreg, vreg, sK[buf ^ 1], sV[buf ^ 1], lrow, lchunk);
    __syncthreads();
    buf ^= 1;
  }

  // ---- epilogue ----
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) l_run[qb] = partner_sum(l_run[qb]);

  if (it.nseg == 1) {
    __bf16 *oh = P.out + (size_t)h * P.q_tokens * D;
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      const int row = it.q0 + (wave * NQB + qb) * 32 + l32;
      if (row >= P.q_tokens) continue;
      const float inv = 1.0f / l_run[qb];
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          bf16x4 w;
#pragma unroll
          for (int e = 0; e < 4; ++e) w[e] = (__bf16)(o[qb][db][i4 * 4 + e] * inv);
          *(bf16x4 *)(oh + (size_t)row * D + db * 32 + 8 * i4 + 4 * g) = w;
        }
    }
    return;
  }

  // ---- split head: park the unnormalised partial (O, m, l), the last segment to arrive merges ----
  const size_t part_floats = (size_t)BQ * (D + 2);
  {
    float *po = P.workspace + (size_t)(it.part0 + it.seg * P.n_qt) * part_floats;
    float *pm = po + (size_t)BQ * D, *pl = pm + BQ;
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      const int lrow_q = (wave * NQB + qb) * 32 + l32;
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          float *dst = po + (size_t)lrow_q * D + db * 32 + 8 * i4 + 4 * g;
          st_dev2(dst, o[qb][db][i4 * 4], o[qb][db][i4 * 4 + 1]);
          st_dev2(dst + 2, o[qb][db][i4 * 4 + 2], o[qb][db][i4 * 4 + 3]);
        }
      if (g == 0) { st_dev1(pm + lrow_q, m_run[qb]); st_dev1(pl + lrow_q, l_run[qb]); }
    }
  }
  __builtin_amdgcn_s_waitcnt(0);             // this wave's partial stores have completed
  __syncthreads();
  if (tid == 0) {
    const int arrived = atomicAdd(&P.counters[it.group], 1);
    sFlag = (arrived == it.nseg - 1) ? 1 : 0;
    if (sFlag) P.counters[it.group] = 0;     // ready for the next launch on this index
  }
  __syncthreads();
  if (!sFlag) return;

  // ---- merge.  Phase A: per query row, the maximum M over the segments' running maxima and the total
  // denominator L = sum_s 2^((m_s-M)c) l_s.  Phase B: out = sum_s 2^((m_s-M)c) O_s / L.  Both phases keep
  // many independent loads in flight: the merge is pure memory latency otherwise. ----
  float *sM = (float *)&sK[0][0];            // the K/V tiles are dead: every wave passed the loop's last barrier
  float *sInvL = sM + BQ;
  const float *base = P.workspace + (size_t)it.part0 * part_floats;
  const size_t seg_stride = (size_t)P.n_qt * part_floats;
  const int nseg = it.nseg;
  for (int r = tid; r < BQ; r += ATT_THREADS) {
    const float *pm = base + (size_t)BQ * D + r;
    float mmax = -3.0e38f;
#pragma unroll 8
    for (int sgi = 0; sgi < nseg; ++sgi) mmax = fmaxf(mmax, ld_dev1(pm + sgi * seg_stride));
    float lsum = 0.0f;
#pragma unroll 8
    for (int sgi = 0; sgi < nseg; ++sgi)
      lsum += fast_exp2((ld_dev1(pm + sgi * seg_stride) - mmax) * c) * ld_dev1(pm + sgi * seg_stride + BQ);
    sM[r] = mmax;
    sInvL[r] = 1.0f / lsum;
  }
  __syncthreads();
  __bf16 *oh = P.out + (size_t)h * P.q_tokens * D;
  constexpr int EG = 4;                                        // output quads per thread in flight
  static_assert((BQ * (D / 4)) % (ATT_THREADS * EG) == 0, "merge tiling");
  for (int e0 = tid; e0 < BQ * (D / 4); e0 += ATT_THREADS * EG) {
    int r[EG], dc[EG];
    float mrow[EG];
    float4 acc[EG];
#pragma unroll
    for (int k = 0; k < EG; ++k) {
      const int e = e0 + k * ATT_THREADS;
      r[k] = e / (D / 4);
      dc[k] = (e % (D / 4)) * 4;
      mrow[k] = sM[r[k]];
      acc[k] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll 4
    for (int sgi = 0; sgi < nseg; ++sgi) {
      const float *ps = base + sgi * seg_stride;
#pragma unroll
      for (int k = 0; k < EG; ++k) {
        const float w = fast_exp2((ld_dev1(ps + (size_t)BQ * D + r[k]) - mrow[k]) * c);
        const float2 va = ld_dev2(ps + (size_t)r[k] * D + dc[k]);
        const float2 vb = ld_dev2(ps + (size_t)r[k] * D + dc[k] + 2);
        acc[k].x += w * va.x; acc[k].y += w * va.y; acc[k].z += w * vb.x; acc[k].w += w * vb.y;
      }
    }
#pragma unroll
    for (int k = 0; k < EG; ++k) {
      const int row = it.q0 + r[k];
      if (row >= P.q_tokens) continue;
      const float inv = sInvL[r[k]];
      bf16x4 w4;
      w4[0] = (__bf16)(acc[k].x * inv); w4[1] = (__bf16)(acc[k].y * inv);
      w4[2] = (__bf16)(acc[k].z * inv); w4[3] = (__bf16)(acc[k].w * inv);
      *(bf16x4 *)(oh + (size_t)row * D + dc[k]) = w4;
    }
  }
}

template <int D, int NQB>
static int launch_attn(const AttnParams &P, int n_blocks, hipStream_t stream) {
  hipLaunchKernelGGL((pf_attn_kernel<D, NQB>), dim3(n_blocks), dim3(ATT_THREADS), 0, stream, P);
  return hipGetLastError() == hipSuccess ? PF_OK : PF_ERR_HIP;
}

extern "C" int pf_ragged_attn_fwd(const pf_pool *pool, const pf_index *index, const void *q, const void *k_cur,
                                  const void *v_cur, void *out, int q_tokens, float softmax_scale,
                                  void *workspace, size_t workspace_bytes, void *stream) {
  const int rc = pf_validate_pool(pool);
  if (rc != PF_OK) return rc;
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
  P.workspace = (float *)workspace;
  P.max_sel = index->max_sel;
  P.tpf = pool->tokens_per_frame;
  P.q_tokens = q_tokens;
  P.n_qt = n_qt;
  const float scale = softmax_scale > 0.0f ? softmax_scale : 1.0f / sqrtf((float)pool->head_dim);
  P.scale_log2 = scale * 1.4426950408889634f;
  hipStream_t st = (hipStream_t)stream;
  if (pool->head_dim == 128)
    return index->variant == 1 ? launch_attn<128, 2>(P, index->n_blocks, st) : launch_attn<128, 1>(P, index->n_blocks, st);
  return index->variant == 1 ? launch_attn<64, 2>(P, index->n_blocks, st) : launch_attn<64, 1>(P, index->n_blocks, st);
}
