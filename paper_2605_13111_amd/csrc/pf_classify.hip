// Offline tri-pattern head classification (Sec. 4.1; pre-processing and harmonic folding as in the appendix
// paragraph on the FFT analysis stage): one workgroup per (prompt, head) sequence, then a vote per head.
// All arithmetic is fp64: the sequences are short (tens of frames), so a direct DFT from a twiddle table is
// cheaper than anything cleverer, and the decisions (thresholds, peak bin) are taken in the precision a host
// implementation would use.
#include <hip/hip_runtime.h>
#include <math.h>
#include "pf_internal.h"

constexpr int CLS_THREADS = 256;
constexpr int CLS_MAX_HIST = 1024;      // longest historical sequence (frames)
constexpr int CLS_HARMONICS = 4;        // harmonics folded onto a fundamental, weights 1/j
constexpr double CLS_TIE_REL = 1e-9;    // folded scores this close count as equal: the lowest bin wins

struct ClassifyParams {
  const float *logits;                  // [n_prompts][n_heads][n_hist]
  int32_t *prompt_type;                 // [n_prompts][n_heads]
  double *prompt_period;                // [n_prompts][n_heads] or null
  int n_hist;
  double alpha, beta;
};

__device__ __forceinline__ double block_sum(double v, double *s_red) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
  __syncthreads();
  if (lane == 0) s_red[wave] = v;
  __syncthreads();
  double t = 0.0;
  for (int w = 0; w < CLS_THREADS / 64; ++w) t += s_red[w];
  return t;
}

__global__ __launch_bounds__(CLS_THREADS) void pf_classify_kernel(ClassifyParams P) {
  __shared__ double s_a[CLS_MAX_HIST];           // the sequence, then the pre-processed difference
  __shared__ double s_cos[CLS_MAX_HIST], s_sin[CLS_MAX_HIST];
  __shared__ double s_amp[CLS_MAX_HIST / 2 + 1];
  __shared__ double s_score[CLS_MAX_HIST / 2 + 1];
  __shared__ double s_red[CLS_THREADS / 64];
  __shared__ int s_k;
  const int tid = threadIdx.x;
  const int n = P.n_hist;
  const float *a = P.logits + (size_t)blockIdx.x * n;

  // ---- sign rates and mean of the raw sequence ----
  double cnt = 0.0, sum = 0.0;
  for (int t = tid; t < n; t += CLS_THREADS) {
    const double v = (double)a[t];
    s_a[t] = v;
    cnt += v > 0.0 ? 1.0 : 0.0;
    sum += v;
  }
  const double n_pos = block_sum(cnt, s_red);
  const double total = block_sum(sum, s_red);
  const double r_pos = n_pos / (double)n, r_neg = 1.0 - r_pos;
  int type = -1;
  double period = INFINITY;
  if (r_pos >= P.alpha) type = PF_ANCHOR;
  else if (r_neg >= P.alpha) type = PF_VEIL;
  if (type < 0) {                                  // uniform over the workgroup
    // ---- dominant period: difference, mean removal, Hann window, spectrum, harmonic folding ----
    const int N = n - 1;
    if (N >= 3) {
      __syncthreads();
      double dsum = 0.0;
      double d_mine[CLS_MAX_HIST / CLS_THREADS];
      for (int m = tid, i = 0; m < N; m += CLS_THREADS, ++i) {
        d_mine[i] = s_a[m + 1] - s_a[m];
        dsum += d_mine[i];
      }
      const double dmean = block_sum(dsum, s_red) / (double)N;   // (the barriers inside also order the reads above)
      for (int m = tid, i = 0; m < N; m += CLS_THREADS, ++i) {
        const double w = 0.5 - 0.5 * cospi(2.0 * (double)m / (double)(N - 1));
        s_a[m] = (d_mine[i] - dmean) * w;
        double sn, cs;
        sincospi(2.0 * (double)m / (double)N, &sn, &cs);
        s_cos[m] = cs;
        s_sin[m] = sn;
      }
      __syncthreads();
      const int nb = N / 2;
      for (int k = tid; k <= nb; k += CLS_THREADS) {
        double re = 0.0, im = 0.0;
        int j = 0;                                 // (k * m) mod N
        for (int m = 0; m < N; ++m) {
          re += s_a[m] * s_cos[j];
          im -= s_a[m] * s_sin[j];
          j += k;
          if (j >= N) j -= N;
        }
        s_amp[k] = sqrt(re * re + im * im);
      }
      __syncthreads();
      double best = 0.0;
      for (int k = 1 + tid; k <= nb; k += CLS_THREADS) {
        double sc = 0.0;
        for (int h = 1; h <= CLS_HARMONICS; ++h)
          if (h * k <= nb) sc += s_amp[h * k] / (double)h;
        s_score[k] = sc;
        best = fmax(best, sc);
      }
      // maximum over the workgroup, then the lowest bin within the tie band
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) best = fmax(best, __shfl_down(best, o, 64));
      __syncthreads();
      if ((tid & 63) == 0) s_red[tid >> 6] = best;
      if (tid == 0) s_k = 0x7fffffff;
      __syncthreads();
      best = fmax(fmax(s_red[0], s_red[1]), fmax(s_red[2], s_red[3]));
      if (best > 0.0 && isfinite(best)) {
        int kmin = 0x7fffffff;
        for (int k = 1 + tid; k <= nb; k += CLS_THREADS)
          if (s_score[k] >= best * (1.0 - CLS_TIE_REL)) { kmin = k; break; }
        if (kmin != 0x7fffffff) atomicMin(&s_k, kmin);
        __syncthreads();
        period = (double)N / (double)s_k;
      }
    }
    if (period < P.beta) type = PF_WAVE;
    else type = (total / (double)n) > 0.0 ? PF_ANCHOR : PF_VEIL;   // mean-score fallback
  }
  if (tid == 0) {
    P.prompt_type[blockIdx.x] = type;
    if (P.prompt_period) P.prompt_period[blockIdx.x] = period;
  }
}

// Majority vote over the prompts; equal counts go to the smaller type code.
__global__ void pf_classify_vote_kernel(const int32_t *prompt_type, int32_t *head_type, int n_prompts, int n_heads) {
  const int h = blockIdx.x * blockDim.x + threadIdx.x;
  if (h >= n_heads) return;
  int votes[3] = {0, 0, 0};
  for (int p = 0; p < n_prompts; ++p) {
    const int t = prompt_type[(size_t)p * n_heads + h];
    if (t >= 0 && t < 3) ++votes[t];
  }
  int best = 0;
  if (votes[1] > votes[best]) best = 1;
  if (votes[2] > votes[best]) best = 2;
  head_type[h] = best;
}

extern "C" int pf_classify_heads(const float *logits, int n_prompts, int n_heads, int n_hist, double alpha, double beta,
                                 int32_t *head_type, int32_t *prompt_type, double *prompt_period, void *stream) {
  if (!logits || !head_type || !prompt_type) return PF_ERR_INVALID_ARG;
  if (n_prompts < 1 || n_heads < 1 || n_hist < 1) return PF_ERR_INVALID_ARG;
  if ((long long)n_prompts * n_heads > (1ll << 30)) return PF_ERR_INVALID_ARG;
  if (n_hist > CLS_MAX_HIST) return PF_ERR_UNSUPPORTED;
  if (!(alpha > 0.0) || !(alpha <= 1.0) || !(beta > 0.0)) return PF_ERR_INVALID_ARG;
  ClassifyParams P;
  P.logits = logits;
  P.prompt_type = prompt_type;
  P.prompt_period = prompt_period;
  P.n_hist = n_hist;
  P.alpha = alpha;
  P.beta = beta;
  hipLaunchKernelGGL(pf_classify_kernel, dim3(n_prompts * n_heads), dim3(CLS_THREADS), 0, (hipStream_t)stream, P);
  PF_HIP_CHECK(hipGetLastError());
  hipLaunchKernelGGL(pf_classify_vote_kernel, dim3(pf_ceil_div(n_heads, 256)), dim3(256), 0, (hipStream_t)stream,
                     prompt_type, head_type, n_prompts, n_heads);
  PF_HIP_CHECK(hipGetLastError());
  return PF_OK;
}
