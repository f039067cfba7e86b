// Stand-alone micro-benchmarks behind the attention kernel's design choices (not part of libpf.so):
//   1. bf16 MFMA rate that one / two waves per SIMD sustain (the practical matrix roof on this board)
//   2. how much vector work a wave can hide behind its own MFMAs (same-wave overlap) vs across waves
//   3. LDS read bandwidth of the K operand pattern with padded (272 B) and unpadded (256 B) rows, and of the
//      V^T transpose-read pattern
//   4. one wave per SIMD issuing only MFMAs next to one issuing only vector work (the two-group kernel's
//      arrangement): what each of them loses
//   5. global -> LDS streaming with 16-byte direct copies: workgroups of one die reading the same stream
//      from HBM (what a team of query tiles does), at 1 to 4 tiles in flight, against private streams
//   6. which kinds of instruction of a second wave on the same SIMD slow a vector-ALU wave down (issue rates per
//      wave and per SIMD, cost of a taken branch)
//   7. the softmax's vector instructions next to a wave that issues MFMAs back to back: each kind alone and the
//      kernel's mix, with dot-product and with plain-add row sums, accumulators in VGPRs or AGPRs
//   8. global -> LDS copy instructions inside an MFMA + LDS-read loop: 64-bit-address form, buffer form, via registers
// Build:  python paper_2605_13111_amd/build.py --ubench     Run:  paper_2605_13111_amd/pf_ubench
#include <hip/hip_runtime.h>
#include <cstdio>
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef const __attribute__((address_space(1))) void *gptr_t;
typedef __attribute__((address_space(3))) void *lptr_t;
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 1; } } while (0)

// ---- 1 + 2: per iteration 8 MFMAs on 4 independent accumulators, each followed by NV independent FMAs ----
template <int NV>
__global__ __launch_bounds__(256, 1) void mfma_valu(float *out, int iters, float seed) {
  const int lane = threadIdx.x & 63;
  bf16x8 a, b;
  for (int j = 0; j < 8; ++j) { a[j] = (__bf16)(float)((lane + j) % 3 - 1); b[j] = (__bf16)(float)((lane * 2 + j) % 3 - 1); }
  f32x16 acc[4];
  for (int k = 0; k < 4; ++k) for (int i = 0; i < 16; ++i) acc[k][i] = 0.f;
  float x[16];
  for (int i = 0; i < 16; ++i) x[i] = seed + i * 0.001f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      acc[m & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[m & 3], 0, 0, 0);
#pragma unroll
      for (int v = 0; v < NV; ++v) { const int r = (m * NV + v) & 15; x[r] = fmaf(x[r], 0.999f, 0.001f); }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  float r = 0;
  for (int k = 0; k < 4; ++k) for (int i = 0; i < 16; ++i) r += acc[k][i];
  for (int i = 0; i < 16; ++i) r += x[i];
  if (r == 12345.678f) out[0] = r;
}

// ---- 3: LDS read patterns of the attention kernel (64-key tile, 128 channels) ----
// MODE 0: K operand reads (ds_read_b128, lane = row l%32, 16-byte column 2*ks + l/32), row stride KS elements
// MODE 1: V^T operand reads (ds_read_b64_tr_b16), row stride VS elements
template <int MODE, int STRIDE>
__global__ __launch_bounds__(256, 2) void lds_read(float *out, int iters) {
  __shared__ __attribute__((aligned(16))) __bf16 tile[64 * STRIDE];
  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, g = lane >> 5;
  for (int i = tid; i < 64 * STRIDE; i += 256) tile[i] = (__bf16)(float)((i * 7) % 5 - 2);
  __syncthreads();
  const int k_lane = l32 * STRIDE + 8 * g;
  const int v_lane = (4 * g + ((lane & 15) >> 2)) * STRIDE + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  for (int it = 0; it < iters; ++it) {
    if (MODE == 0) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          const u32x4 a = *(const u32x4 *)(&tile[k_lane + kb * 32 * STRIDE + ks * 16]);
          asm volatile("" ::"v"(a));
        }
    } else {
#pragma unroll
      for (int s16 = 0; s16 < 4; ++s16)
#pragma unroll
        for (int db = 0; db < 4; ++db) {
          const __bf16 *vp = &tile[v_lane + s16 * 16 * STRIDE + db * 32];
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(vp));
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(vp + 8 * STRIDE));
          asm volatile("" ::"v"(lo), "v"(hi));
        }
    }
  }
  if (iters < 0) out[0] = 1.f;
}

static int time_kernel(void (*launch)(float *, int), float *dout, int iters, float *ms) {
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  launch(dout, 10);
  CK(hipDeviceSynchronize());
  CK(hipEventRecord(e0));
  launch(dout, iters);
  CK(hipEventRecord(e1));
  CK(hipDeviceSynchronize());
  CK(hipEventElapsedTime(ms, e0, e1));
  return 0;
}

template <int NV, int BLOCKS> static void l_mfma(float *o, int it) { mfma_valu<NV><<<BLOCKS, 256>>>(o, it, 0.5f); }
template <int MODE, int STRIDE> static void l_lds(float *o, int it) { lds_read<MODE, STRIDE><<<512, 256>>>(o, it); }

template <int NV, int BLOCKS>
static int run_mfma(float *dout) {
  const int iters = 4000;
  float ms;
  if (time_kernel(l_mfma<NV, BLOCKS>, dout, iters, &ms)) return 1;
  const double mfmas = (double)BLOCKS * 4 * iters * 8;
  printf("MFMA + %2d FMA each, %d wave(s)/SIMD: %7.3f ms  %5.1f ns per MFMA per SIMD  matrix rate %6.0f TFLOP/s\n", NV,
         BLOCKS / 256, ms, ms * 1e6 / (iters * 8.0 * (BLOCKS / 256)), mfmas * 32768.0 / (ms * 1e-3) / 1e12);
  return 0;
}
template <int MODE, int STRIDE>
static int run_lds(float *dout, const char *name) {
  const int iters = 2000;
  float ms;
  if (time_kernel(l_lds<MODE, STRIDE>, dout, iters, &ms)) return 1;
  const double bytes = 512.0 * 4 * iters * 16384.0;          // 16 KB per wave per iteration
  printf("%-44s %7.3f ms  %6.1f TB/s aggregate  %5.1f GB/s per CU\n", name, ms, bytes / (ms * 1e-3) / 1e12,
         bytes / (ms * 1e-3) / 1e9 / 256);
  return 0;
}

// ---- 4: waves 0-3 (one per SIMD) run MFMAs only, waves 4-7 (the second wave of each SIMD) vector work only ----
template <int MODE>   // 0: second group idle, 1: FMA stream, 2: exp2 stream, 3: 3 FMA : 1 exp2
__global__ __launch_bounds__(512, 2) void split_roles(float *out, long long *cyc, int n) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const long long t0 = clock64();
  float res;
  if (wave < 4) {
    f32x16 a0 = {}, a1 = {}, a2 = {}, a3 = {};
    bf16x8 x, y;
    for (int i = 0; i < 8; ++i) { x[i] = (__bf16)(float)(lane + i); y[i] = (__bf16)(float)(lane - i); }
    for (int i = 0; i < n; ++i) {
      a0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, a0, 0, 0, 0);
      a1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, a1, 0, 0, 0);
      a2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, a2, 0, 0, 0);
      a3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, a3, 0, 0, 0);
    }
    res = 0;
    for (int i = 0; i < 16; ++i) res += a0[i] + a1[i] + a2[i] + a3[i];
  } else {
    float v[8];
    for (int i = 0; i < 8; ++i) v[i] = lane * 0.001f + i;
    if (MODE != 0) {
      for (int i = 0; i < n; ++i) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const bool ex = MODE == 2 || (MODE == 3 && (e & 3) == 3);
            v[e] = ex ? __builtin_amdgcn_exp2f(v[e]) : fmaf(v[e], 1.0001f, 0.5f);
          }
      }
    }
    res = 0;
    for (int i = 0; i < 8; ++i) res += v[i];
  }
  if (res == 12345.678f) out[0] = res;
  const long long t1 = clock64();
  if (lane == 0) cyc[blockIdx.x * 8 + wave] = t1 - t0;
}
template <int MODE>
static int run_split(long long *dcyc, float *dout, const char *name) {
  const int n = 20000;
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  for (int rep = 0; rep < 2; ++rep) {
    CK(hipEventRecord(e0));
    split_roles<MODE><<<256, 512>>>(dout, dcyc, n);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
  }
  float ms; CK(hipEventElapsedTime(&ms, e0, e1));
  static long long h[256 * 8];
  CK(hipMemcpy(h, dcyc, sizeof(h), hipMemcpyDeviceToHost));
  double m = 0, v = 0;
  for (int b = 0; b < 256; ++b) { for (int w = 0; w < 4; ++w) m += h[b * 8 + w]; for (int w = 4; w < 8; ++w) v += h[b * 8 + w]; }
  m /= 1024; v /= 1024;
  printf("%-34s %7.3f ms  matrix wave %5.1f cycles per MFMA   vector wave %5.2f cycles per instruction   clock %.2f GHz\n",
         name, ms, m / (4.0 * n), MODE ? v / (32.0 * n) : 0.0, m / (ms * 1e6));
  return 0;
}

// ---- 5: teams of workgroups on one die stream the same 32 KB tiles global -> LDS (16-byte direct copies) ----
constexpr int TILE = 32768;
template <int DEPTH>
__global__ __launch_bounds__(512, 2) void stream_kernel(const char *base, size_t team_stride, int team_size, int n_tiles, float *sink) {
  __shared__ __attribute__((aligned(1024))) char s[4][TILE];
  typedef const __attribute__((address_space(1))) void *gptr_t;
  typedef __attribute__((address_space(3))) void *lptr_t;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;     // workgroup i runs on die i % 8
  const int team = (slot / team_size) * 8 + xcd;
  const char *src = base + (size_t)team * team_stride + wave * 4096 + lane * 16;
  auto issue = [&](int t) {
    const char *p = src + (size_t)t * TILE;
    char *d = &s[t & 3][wave * 4096];
#pragma unroll
    for (int h = 0; h < 4; ++h) __builtin_amdgcn_global_load_lds((gptr_t)(p + h * 1024), (lptr_t)(d + h * 1024), 16, 0, 0);
  };
  for (int t = 0; t < DEPTH && t < n_tiles; ++t) issue(t);
  for (int t = 0; t < n_tiles; ++t) {
    __builtin_amdgcn_s_waitcnt(0x0F70 | (4 * (DEPTH - 1)));   // vmcnt: all but the DEPTH-1 newest tiles have landed
    __builtin_amdgcn_s_barrier();
    issue(t + DEPTH < n_tiles ? t + DEPTH : n_tiles - 1);     // constant number of copies per step
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);
  __syncthreads();
  if (threadIdx.x == 0 && s[0][0] == 123 && s[1][5] == 77) sink[0] = 1.0f;
}
template <int DEPTH>
static int run_stream(const char *name, const char *buf, size_t team_stride, int team_size, int n_tiles, float *sink) {
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  for (int rep = 0; rep < 2; ++rep) {
    CK(hipEventRecord(e0));
    stream_kernel<DEPTH><<<256, 512>>>(buf, team_stride, team_size, n_tiles, sink);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
  }
  float ms; CK(hipEventElapsedTime(&ms, e0, e1));
  printf("%-36s %d tile(s) in flight: %7.3f ms  %5.0f ns per 32 KB tile  %6.1f GB/s per CU  %6.2f TB/s into the CUs\n", name, DEPTH,
         ms, ms * 1e6 / n_tiles, (double)TILE / (ms * 1e6 / n_tiles), (double)TILE * n_tiles * 256 / (ms * 1e-3) / 1e12);
  return 0;
}

// ---- 6: two waves on every SIMD, each issuing one kind of instruction for a fixed number of cycles: which kinds
// compete (the timer is the shader clock, so the figures are cycles) ----
template <int AMODE, int BMODE>
__global__ __launch_bounds__(512, 2) void issue_types(float *out, long long *cnt, long long tfix, int zero) {
  __shared__ __attribute__((aligned(1024))) char lds[65536];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  for (int i = threadIdx.x; i < 65536 / 4; i += 512) ((float *)lds)[i] = 0.001f * i;
  __syncthreads();
  const long long t0 = clock64();
  long long done = 0;
  float res = 0;
  if (wave < 4) {                                   // wave A
    int sa = zero, sb = zero + 1, sc = zero + 2;
    const unsigned ra = (unsigned)(uintptr_t)(const __attribute__((address_space(3))) char *)&lds[0] + wave * 8192 + lane * 16;
    float v[8];
    for (int i = 0; i < 8; ++i) v[i] = lane + i;
    if (AMODE) {
      while (clock64() - t0 < tfix) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          if (AMODE == 1) {
            asm volatile("s_add_i32 %0, %0, %1\n s_lshl_b32 %1, %1, 1\n s_sub_i32 %2, %2, %0\n s_and_b32 %1, %1, 0xffff\n s_xor_b32 %2, %2, %1\n s_add_i32 %0, %0, 3\n s_max_i32 %1, %1, %2\n s_add_i32 %0, %0, 5"
                         : "+s"(sa), "+s"(sb), "+s"(sc));
          } else if (AMODE == 2) {
            asm volatile("s_nop 0\n s_nop 0\n s_nop 0\n s_nop 0\n s_nop 0\n s_nop 0\n s_nop 0\n s_nop 0");
          } else if (AMODE == 3) {
            u32x4 f[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f[j]) : "v"(ra), "n"(j * 1024));
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]), "+v"(f[4]), "+v"(f[5]), "+v"(f[6]), "+v"(f[7]));
          } else if (AMODE == 4) {
            asm volatile("s_branch 1f\n 1: s_branch 2f\n 2: s_branch 3f\n 3: s_branch 4f\n 4: s_branch 5f\n 5: s_branch 6f\n 6: s_branch 7f\n 7: s_branch 8f\n 8: s_nop 0");
          } else if (AMODE == 5) {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = fmaf(v[e], 1.0001f, 0.5f);
          } else if (AMODE == 6) {
            asm volatile("s_waitcnt lgkmcnt(0)\n s_waitcnt lgkmcnt(1)\n s_waitcnt lgkmcnt(0)\n s_waitcnt lgkmcnt(1)\n s_waitcnt lgkmcnt(0)\n s_waitcnt lgkmcnt(1)\n s_waitcnt lgkmcnt(0)\n s_waitcnt lgkmcnt(1)");
          }
        }
        done += 128;
      }
    }
    res = (float)(sa + sb + sc);
    for (int i = 0; i < 8; ++i) res += v[i];
  } else {                                          // wave B
    float v[8];
    for (int i = 0; i < 8; ++i) v[i] = lane * 0.001f + i;
    int sa = zero, sb = zero + 1, sc = zero + 2;
    while (clock64() - t0 < tfix) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        if (BMODE == 0) {
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] = fmaf(v[e], 1.0001f, 0.5f);
        } else {
          asm volatile("s_add_i32 %0, %0, %1\n s_lshl_b32 %1, %1, 1\n s_sub_i32 %2, %2, %0\n s_and_b32 %1, %1, 0xffff\n s_xor_b32 %2, %2, %1\n s_add_i32 %0, %0, 3\n s_max_i32 %1, %1, %2\n s_add_i32 %0, %0, 5"
                       : "+s"(sa), "+s"(sb), "+s"(sc));
        }
      }
      done += 128;
    }
    for (int i = 0; i < 8; ++i) res += v[i];
    res += (float)(sa + sb + sc);
  }
  if (res == 12345.678f) out[0] = res;
  if (lane == 0) cnt[blockIdx.x * 8 + wave] = done;
}
template <int AMODE, int BMODE>
static int run_issue(long long *dcnt, float *dout, const char *name) {
  const long long tfix = 3000000;
  CK(hipMemset(dcnt, 0, 256 * 8 * 8));
  for (int rep = 0; rep < 2; ++rep) { issue_types<AMODE, BMODE><<<256, 512>>>(dout, dcnt, tfix, 0); CK(hipDeviceSynchronize()); }
  static long long h[256 * 8];
  CK(hipMemcpy(h, dcnt, sizeof(h), hipMemcpyDeviceToHost));
  double a = 0, b = 0;
  for (int blk = 0; blk < 256; ++blk) { for (int w = 0; w < 4; ++w) a += h[blk * 8 + w]; for (int w = 4; w < 8; ++w) b += h[blk * 8 + w]; }
  a /= 1024; b /= 1024;
  printf("%-52s wave A %6.2f ticks per instr   wave B %6.2f ticks per instr\n", name, a > 0 ? tfix / a : 0.0, b > 0 ? tfix / b : 0.0);
  return 0;
}

// ---- 7: a wave issuing only MFMAs (accumulators in VGPRs or AGPRs) next to a wave issuing the softmax's vector
// instructions, each kind alone and as the mix the kernel runs; both run for a fixed number of cycles ----
template <int ACC, int MODE, int MROLE, int PRIO = 0>
__global__ __launch_bounds__(512, 2) void mfma_next_to(float *out, long long *cnt, long long tfix) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const long long t0 = clock64();
  float res = 0;
  long long done = 0;
  if (wave < 4) {
    if (MROLE) {
      if (PRIO) __builtin_amdgcn_s_setprio(3);
      f32x16 a0 = {}, a1 = {}, a2 = {}, a3 = {};
      bf16x8 x, y;
      for (int i = 0; i < 8; ++i) { x[i] = (__bf16)(float)(lane + i); y[i] = (__bf16)(float)(lane - i); }
      while (clock64() - t0 < tfix) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          if (ACC) {
            asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(a0) : "v"(x), "v"(y));
            asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(a1) : "v"(x), "v"(y));
            asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(a2) : "v"(x), "v"(y));
            asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(a3) : "v"(x), "v"(y));
          } else {
            asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(a0) : "v"(x), "v"(y));
            asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(a1) : "v"(x), "v"(y));
            asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(a2) : "v"(x), "v"(y));
            asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(a3) : "v"(x), "v"(y));
          }
        }
        done += 16;
      }
      asm volatile("s_nop 15\n s_nop 15");
      for (int i = 0; i < 16; ++i) res += a0[i] + a1[i] + a2[i] + a3[i];
    }
  } else {
    float v[8], w[8], u[8];
    for (int i = 0; i < 8; ++i) { v[i] = lane * 0.001f + i; w[i] = 1.0f + lane * 1e-6f * i; u[i] = 0.5f - i * 1e-3f; }
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    float l = 0, mx = 0;
    if (MODE != 0) {
      while (clock64() - t0 < tfix) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          if (MODE == 1) {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = fmaf(v[e], w[e], u[e]);
          } else if (MODE == 2) {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = __builtin_amdgcn_exp2f(v[e]);
          } else if (MODE == 4) {                 // max3 chain
#pragma unroll
            for (int e = 0; e < 8; e += 2) mx = fmaxf(fmaxf(mx, v[e]), v[e + 1]);
#pragma unroll
            for (int e = 0; e < 8; e += 2) l = fmaxf(fmaxf(l, w[e]), w[e + 1]);
            asm volatile("" : "+v"(mx), "+v"(l));
          } else if (MODE == 5) {                 // cvt_pk only
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              bf16x2 pk; pk[0] = (__bf16)v[e]; pk[1] = (__bf16)w[e];
              asm volatile("" : "+v"(pk));
              v[e] = __builtin_bit_cast(float, pk);
            }
          } else if (MODE == 11) {                // v_perm_b32 pack (truncation)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              unsigned pk = __builtin_amdgcn_perm(__builtin_bit_cast(unsigned, w[e]), __builtin_bit_cast(unsigned, v[e]), 0x07060302u);
              asm volatile("" : "+v"(pk));
              v[e] = __builtin_bit_cast(float, pk);
            }
          } else if (MODE == 12) {                // 16 independent cvt_pk per round (no chains)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              bf16x2 pk; pk[0] = (__bf16)w[e]; pk[1] = (__bf16)u[e];
              asm volatile("" : "+v"(pk));
            }
          } else if (MODE == 13) {                // independent exp2
#pragma unroll
            for (int e = 0; e < 8; ++e) { float t = __builtin_amdgcn_exp2f(w[e]); asm volatile("" : "+v"(t)); }
          } else if (MODE == 14) {                // independent fma
#pragma unroll
            for (int e = 0; e < 8; ++e) { float t = fmaf(w[e], u[e], v[e]); asm volatile("" : "+v"(t)); }
          } else if (MODE == 6) {                 // dot2 only, 8 chains
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w[e]), ones, v[e], false);
          } else if (MODE == 7) {                 // dot2 only, one chain (as the kernel's row sum)
#pragma unroll
            for (int e = 0; e < 8; ++e) l = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w[e]), ones, l, false);
            asm volatile("" : "+v"(l));
          } else {
            // the softmax mix: per 8 values 4 max3, 8 fma, 8 exp2, 4 cvt_pk, 4 row-sum steps
            float p[8];
#pragma unroll
            for (int e = 0; e < 8; e += 2) mx = fmaxf(fmaxf(mx, v[e]), v[e + 1]);
#pragma unroll
            for (int e = 0; e < 8; ++e) p[e] = __builtin_amdgcn_exp2f(fmaf(v[e], w[0], u[0]));
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
              bf16x2 pk; pk[0] = (__bf16)p[e]; pk[1] = (__bf16)p[e + 1];
              if (MODE == 3) l = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, l, false);
              else if (MODE == 8) l += p[e] + p[e + 1];               // fp32 adds instead of dot2 (2 instrs)
              else if (MODE == 9) { l = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, l, false); }
              if (MODE == 10) { l += p[e]; asm volatile("" : "+v"(p[e + 1])); }   // no cvt: pack skipped
              else asm volatile("" : "+v"(pk));
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) asm volatile("" : "+v"(v[e]));
          }
        }
        done += MODE == 3 || MODE == 9 ? 16 * 28 : MODE == 8 ? 16 * 32 : MODE == 10 ? 16 * 24 : 128;
      }
    }
    for (int i = 0; i < 8; ++i) res += v[i];
    res += l + mx;
  }
  if (res == 12345.678f) out[0] = res;
  if (lane == 0) cnt[blockIdx.x * 8 + wave] = done;
}
template <int ACC, int MODE, int MROLE, int PRIO = 0>
static int run_next_to(long long *dcnt, float *dout, const char *name) {
  const long long tfix = 4000000;
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  for (int rep = 0; rep < 2; ++rep) {
    CK(hipEventRecord(e0));
    mfma_next_to<ACC, MODE, MROLE, PRIO><<<256, 512>>>(dout, dcnt, tfix);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
  }
  float ms; CK(hipEventElapsedTime(&ms, e0, e1));
  static long long h[256 * 8];
  CK(hipMemcpy(h, dcnt, sizeof(h), hipMemcpyDeviceToHost));
  double m = 0, v = 0;
  for (int b = 0; b < 256; ++b) { for (int w = 0; w < 4; ++w) m += h[b * 8 + w]; for (int w = 4; w < 8; ++w) v += h[b * 8 + w]; }
  m /= 1024; v /= 1024;
  printf("%-44s %7.3f ms (timer ticks %.0f MHz)  ticks per MFMA %6.1f   ticks per vector instr %6.2f   MFMA rate %.0f TFLOP/s\n", name, ms,
         tfix / (ms * 1e3), m > 0 ? tfix / m : 0.0, v > 0 ? tfix / v : 0.0, m * 1024 * 32768.0 / (ms * 1e-3) / 1e12);
  return 0;
}

// ---- 8: global -> LDS copy instructions inside a loop of MFMAs and LDS reads: the 64-bit-address form, the buffer
// form (scalar base, 32-bit vector offset) and the way through registers ----
// NDMA copies per 32 MFMAs; READS: LDS reads per MFMA (0, 1); WAVES: active waves (4 = one per SIMD, 8 = two)
// DSIZE: bytes per lane per copy (4 or 16); REG: 1 = copy through registers (global load + ds_write) instead
template <int NDMA, int READS, int WAVES, int DSIZE, int REG>
__global__ __launch_bounds__(512, 2) void copy_forms(const char *src, float *out, long long *cnt, long long tfix) {
  __shared__ __attribute__((aligned(1024))) char lds[2][65536];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  for (int i = threadIdx.x; i < 65536 / 4; i += 512) ((float *)lds[0])[i] = 0.001f * i;
  __syncthreads();
  const long long t0 = clock64();
  long long done = 0;
  float res = 0;
  if (wave < WAVES) {
    f32x16 a0 = {}, a1 = {}, a2 = {}, a3 = {};
    bf16x8 y;
    for (int i = 0; i < 8; ++i) y[i] = (__bf16)(float)(lane - i);
    const unsigned ra = (unsigned)(uintptr_t)(const __attribute__((address_space(3))) char *)&lds[0][0] + wave * 8192 + lane * 16;
    const char *g = src + (size_t)blockIdx.x * 65536 + wave * 8192 + lane * DSIZE;
    u32x4 hold[4] = {};
    __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void *)(src + (size_t)blockIdx.x * 65536 + wave * 8192), 0, 8192, 0x00020000);
    int it = 0;
    while (clock64() - t0 < tfix) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        u32x4 f[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          if (READS) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f[j]) : "v"(ra), "n"(j * 1024));
          else asm volatile("" : "=v"(f[j]));
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          if (READS) asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(f[j]) : "n"(7 - j));
          const bf16x8 x = __builtin_bit_cast(bf16x8, f[j]);
          if ((j & 3) == 0) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(a0) : "v"(x), "v"(y));
          if ((j & 3) == 1) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(a1) : "v"(x), "v"(y));
          if ((j & 3) == 2) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(a2) : "v"(x), "v"(y));
          if ((j & 3) == 3) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(a3) : "v"(x), "v"(y));
        }
        // this quarter's share of the copies
#pragma unroll
        for (int d = 0; d < (REG == 3 ? 0 : NDMA / 4); ++d) {
          const int slot = (it * NDMA + q * (NDMA / 4) + d) & 7;
          if (REG == 2) {
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lptr_t)(&lds[1][wave * 8192 + slot * 1024]), 16, lane * 16, slot * 1024, 0, 0);
          } else if (REG) {
            hold[d & 3] = *(const u32x4 *)(g + slot * 1024);
          } else {
            if constexpr (DSIZE == 16) __builtin_amdgcn_global_load_lds((gptr_t)(g + slot * 1024), (lptr_t)(&lds[1][wave * 8192 + slot * 1024]), 16, 0, 0);
            else __builtin_amdgcn_global_load_lds((gptr_t)(g + slot * 256), (lptr_t)(&lds[1][wave * 8192 + slot * 256]), 4, 0, 0);
          }
        }
        if (REG == 1) {
#pragma unroll
          for (int d = 0; d < NDMA / 4; ++d) *(u32x4 *)(&lds[1][wave * 8192 + ((it + d) & 7) * 1024 + lane * 16]) = hold[d & 3];
        }
      }
      if (REG == 3) {
#pragma unroll
        for (int d = 0; d < NDMA; ++d) {
          const unsigned wa = (unsigned)(uintptr_t)(const __attribute__((address_space(3))) char *)&lds[1][0] + wave * 8192 + ((it + d) & 7) * 1024 + lane * 16;
          asm volatile("ds_write_b128 %0, %1" :: "v"(wa), "v"(hold[d & 3]) : "memory");
        }
#pragma unroll
        for (int d = 0; d < NDMA; ++d) {
          auto t = __builtin_amdgcn_raw_buffer_load_b128(rs, lane * 16, ((it * NDMA + d) & 7) * 1024, 0);
          hold[d & 3] = __builtin_bit_cast(u32x4, t);
        }
      }
      ++it;
      done += 32;
    }
    __builtin_amdgcn_s_waitcnt(0);
    asm volatile("s_nop 15\n s_nop 15");
    for (int i = 0; i < 16; ++i) res += a0[i] + a1[i] + a2[i] + a3[i];
  }
  __syncthreads();
  res += lds[1][threadIdx.x];
  if (res == 12345.678f) out[0] = res;
  if (lane == 0) cnt[blockIdx.x * 8 + wave] = done;
}
template <int NDMA, int READS, int WAVES, int DSIZE, int REG>
static int run_copy(const char *src, long long *dcnt, float *dout, const char *name) {
  const long long tfix = 3000000;
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  CK(hipMemset(dcnt, 0, 256 * 8 * 8));
  for (int rep = 0; rep < 2; ++rep) {
    CK(hipEventRecord(e0));
    copy_forms<NDMA, READS, WAVES, DSIZE, REG><<<256, 512>>>(src, dout, dcnt, tfix);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
  }
  float ms; CK(hipEventElapsedTime(&ms, e0, e1));
  static long long h[256 * 8];
  CK(hipMemcpy(h, dcnt, sizeof(h), hipMemcpyDeviceToHost));
  double m = 0;
  for (int b = 0; b < 256; ++b) for (int w = 0; w < WAVES; ++w) m += h[b * 8 + w];
  m /= 256.0 * WAVES;
  printf("%-58s ticks per 32 MFMAs %7.0f  (%5.1f per MFMA)   clock %.0f MHz\n", name, tfix / m * 32, tfix / m, tfix / (ms * 1e3));
  return 0;
}
int main() {
  float *dout;
  CK(hipMalloc(&dout, 4));
  if (run_mfma<0, 256>(dout) || run_mfma<2, 256>(dout) || run_mfma<4, 256>(dout) || run_mfma<6, 256>(dout) ||
      run_mfma<8, 256>(dout) || run_mfma<12, 256>(dout))
    return 1;
  if (run_mfma<0, 512>(dout) || run_mfma<4, 512>(dout) || run_mfma<6, 512>(dout) || run_mfma<8, 512>(dout) ||
      run_mfma<12, 512>(dout))
    return 1;
  if (run_lds<0, 136>(dout, "K reads, rows padded to 272 B") || run_lds<0, 128>(dout, "K reads, unpadded 256 B rows") ||
      run_lds<1, 160>(dout, "V^T transpose reads, rows padded to 320 B") ||
      run_lds<1, 128>(dout, "V^T transpose reads, unpadded 256 B rows"))
    return 1;
  long long *dcyc;
  CK(hipMalloc(&dcyc, 256 * 8 * sizeof(long long)));
  if (run_split<0>(dcyc, dout, "matrix waves alone") || run_split<1>(dcyc, dout, "matrix waves + FMA waves") ||
      run_split<2>(dcyc, dout, "matrix waves + exp2 waves") || run_split<3>(dcyc, dout, "matrix waves + 3 FMA : 1 exp2 waves"))
    return 1;
  {
    const int n_tiles = 400;
    const size_t stream = (size_t)n_tiles * TILE;             // 13 MB per stream: every tile comes from HBM
    char *buf;
    CK(hipMalloc(&buf, stream * 256));
    CK(hipMemset(buf, 1, stream * 256));
    if (run_stream<1>("team of 16 shares one HBM stream", buf, stream, 16, n_tiles, dout) ||
        run_stream<2>("team of 16 shares one HBM stream", buf, stream, 16, n_tiles, dout) ||
        run_stream<3>("team of 16 shares one HBM stream", buf, stream, 16, n_tiles, dout) ||
        run_stream<4>("team of 16 shares one HBM stream", buf, stream, 16, n_tiles, dout) ||
        run_stream<2>("every workgroup its own HBM stream", buf, stream, 1, n_tiles, dout) ||
        run_stream<4>("every workgroup its own HBM stream", buf, stream, 1, n_tiles, dout))
      return 1;
  }
  {
    long long *dcnt;
    CK(hipMalloc(&dcnt, 256 * 8 * 8));
    if (run_issue<0, 0>(dcnt, dout, "A idle            | B fma") || run_issue<5, 0>(dcnt, dout, "A fma             | B fma") ||
        run_issue<1, 0>(dcnt, dout, "A scalar ALU      | B fma") || run_issue<2, 0>(dcnt, dout, "A s_nop           | B fma") ||
        run_issue<3, 0>(dcnt, dout, "A LDS reads       | B fma") || run_issue<4, 0>(dcnt, dout, "A taken branches  | B fma") ||
        run_issue<6, 0>(dcnt, dout, "A s_waitcnt       | B fma") || run_issue<1, 1>(dcnt, dout, "A scalar ALU      | B scalar ALU"))
      return 1;
    if (run_next_to<0, 0, 1>(dcnt, dout, "matrix wave alone, VGPR accumulators") || run_next_to<1, 0, 1>(dcnt, dout, "matrix wave alone, AGPR accumulators") ||
        run_next_to<0, 1, 0>(dcnt, dout, "fma alone") || run_next_to<0, 2, 0>(dcnt, dout, "exp2 alone") ||
        run_next_to<0, 12, 0>(dcnt, dout, "cvt_pk_bf16 alone") || run_next_to<0, 11, 0>(dcnt, dout, "v_perm alone") ||
        run_next_to<0, 4, 0>(dcnt, dout, "max3 alone") || run_next_to<0, 6, 0>(dcnt, dout, "dot2 alone") ||
        run_next_to<0, 3, 0>(dcnt, dout, "softmax mix (dot2 row sums) alone") || run_next_to<0, 8, 0>(dcnt, dout, "softmax mix (fp32 add row sums) alone") ||
        run_next_to<0, 1, 1>(dcnt, dout, "matrix + fma") || run_next_to<0, 2, 1>(dcnt, dout, "matrix + exp2") ||
        run_next_to<0, 12, 1>(dcnt, dout, "matrix + cvt_pk_bf16") || run_next_to<0, 4, 1>(dcnt, dout, "matrix + max3") ||
        run_next_to<0, 6, 1>(dcnt, dout, "matrix + dot2") || run_next_to<0, 3, 1>(dcnt, dout, "matrix + softmax mix (dot2 row sums)") ||
        run_next_to<0, 8, 1>(dcnt, dout, "matrix + softmax mix (fp32 add row sums)") ||
        run_next_to<1, 8, 1>(dcnt, dout, "matrix (AGPR) + softmax mix (fp32 add row sums)"))
      return 1;
    char *src;
    CK(hipMalloc(&src, 256 * 65536 + 65536));
    CK(hipMemset(src, 0, 256 * 65536 + 65536));
    if (run_copy<0, 1, 4, 16, 0>(src, dcnt, dout, "1 wave/SIMD: MFMA + LDS reads") ||
        run_copy<4, 1, 4, 16, 0>(src, dcnt, dout, "1 wave/SIMD: MFMA + LDS reads + 4 x 16-byte global copies") ||
        run_copy<4, 1, 4, 16, 2>(src, dcnt, dout, "1 wave/SIMD: MFMA + LDS reads + 4 x 16-byte buffer copies") ||
        run_copy<16, 1, 4, 16, 0>(src, dcnt, dout, "1 wave/SIMD: MFMA + LDS reads + 16 x 16-byte global copies") ||
        run_copy<16, 1, 4, 4, 0>(src, dcnt, dout, "1 wave/SIMD: MFMA + LDS reads + 16 x 4-byte global copies") ||
        run_copy<4, 1, 4, 16, 3>(src, dcnt, dout, "1 wave/SIMD: MFMA + LDS reads + 4 x (buffer load, ds_write)") ||
        run_copy<0, 1, 8, 16, 0>(src, dcnt, dout, "2 waves/SIMD: MFMA + LDS reads") ||
        run_copy<4, 1, 8, 16, 0>(src, dcnt, dout, "2 waves/SIMD: MFMA + LDS reads + 4 x 16-byte global copies") ||
        run_copy<4, 1, 8, 16, 2>(src, dcnt, dout, "2 waves/SIMD: MFMA + LDS reads + 4 x 16-byte buffer copies") ||
        run_copy<4, 1, 8, 16, 3>(src, dcnt, dout, "2 waves/SIMD: MFMA + LDS reads + 4 x (buffer load, ds_write)"))
      return 1;
  }
  printf("UBENCH DONE\n");
  return 0;
}
