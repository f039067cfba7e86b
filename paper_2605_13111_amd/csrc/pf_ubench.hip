// Stand-alone micro-benchmarks behind the attention kernel's design choices (not part of libpf.so):
//   1. bf16 MFMA rate that one / two waves per SIMD sustain (the practical matrix roof on this board)
//   2. how much vector work a wave can hide behind its own MFMAs (same-wave overlap) vs across waves
//   3. LDS read bandwidth of the K operand pattern with padded (272 B) and unpadded (256 B) rows, and of the
//      V^T transpose-read pattern
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
  printf("UBENCH DONE\n");
  return 0;
}
