// Stand-alone micro-benchmarks behind the attention kernel's design choices (not part of libpf.so):
//   1. bf16 MFMA rate that one / two waves per SIMD sustain (the practical matrix roof on this board)
//   2. how much vector work a wave can hide behind its own MFMAs (same-wave overlap) vs across waves
//   3. LDS read bandwidth of the K operand pattern with padded (272 B) and unpadded (256 B) rows, and of the
//      V^T transpose-read pattern
//   4. one wave per SIMD issuing only MFMAs next to one issuing only vector work (the two-group kernel's
//      arrangement): what each of them loses
//   5. global -> LDS streaming with 16-byte direct copies: workgroups of one die reading the same stream
//      from HBM (what a team of query tiles does), at 1 to 4 tiles in flight, against private streams
// Build:  python paper_2605_13111_amd/build.py --ubench     Run:  paper_2605_13111_amd/pf_ubench
#include <hip/hip_runtime.h>
#include <cstdio>
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
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
  printf("UBENCH DONE\n");
  return 0;
}
