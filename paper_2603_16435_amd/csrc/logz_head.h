// logz_head.h - the log-Z head: per-prompt log-partition estimate from the prompt's hidden states.
//
//   pooled_p = mean of the prompt's hidden-state rows        logz_pool_kernel   (HBM-bound: reads the rows once)
//   a_p = W1 pooled_p + b1,  g_p = gelu(a_p)                 gemm_nt_kernel<float, EpiMlpHidden>  (W1 streamed once)
//   logZ_p = w2 . g_p + b2                                   logz_out_kernel
//   backward from d_logZ: da, db1, dw2, db2                  logz_bwd_vec_kernel
//                         dW1 = sum_p da_p pooled_p^T        logz_bwd_w1_kernel  (HBM-bound: writes dW1 once)
//
// The hidden states are constants here (no gradient into the language model).  Parameters and
// activations are f32; the hidden states come in the model's dtype.  All of it is a few tens of
// microseconds next to the policy-loss path: the kernels are written to touch every byte once, not for MFMA peak.
#pragma once
#include "gemm_nt.h"

namespace rlk {

__device__ inline float gelu_f(float a) { return 0.5f * a * (1.f + erff(a * 0.70710678118654752f)); }
__device__ inline float gelu_grad_f(float a) {
  return 0.5f * (1.f + erff(a * 0.70710678118654752f)) + a * expf(-0.5f * a * a) * 0.3989422804014327f;
}

// grid (P, ceil(H / 256)): thread = one hidden column of one prompt, f32 sum over the prompt's rows
template <class T>
__global__ void logz_pool_kernel(const T* X, int64_t rows, int H, const int32_t* cu, float* pooled) {
  const int p = blockIdx.x, h = blockIdx.y * 256 + threadIdx.x;
  if (h >= H) return;
  int64_t a = cu[p], b = cu[p + 1];
  if (a < 0) a = 0;
  if (b > rows) b = rows;
  float s = 0.f;
  for (int64_t r = a; r < b; ++r) s += (float)X[r * H + h];
  pooled[(int64_t)p * H + h] = b > a ? s / (float)(b - a) : 0.f;
}

// epilogue of the hidden layer: C[m = unit][n = prompt] -> a[p][j] = acc + b1[j], g[p][j] = gelu(a)
struct EpiMlpHidden {
  typedef NoPre Pre;
  template <class L> __device__ Pre preload(const TileCtx&, const GemmDims&) const { return Pre(); }
  static constexpr bool kPermute = false;
  __device__ void keep_alive() const { a_out[0] = 0.f; }
  const float* b1; float* a_out; float* g_out; int M, P;

  template <class L, int MB, int NB, int BM, int BN, int WAVES_M, int WAVES_N, bool AGPR>
  __device__ __attribute__((always_inline)) void run(typename L::acc_t (&acc)[MB][NB], const TileCtx& c, unsigned char*, const GemmDims&, const Pre&) const {
#pragma unroll
    for (int bi = 0; bi < MB; ++bi)
#pragma unroll
      for (int i = 0; i < L::kRegs; ++i) {
        const int j = c.m0 + L::row(bi, i, c.lane);
        if (j >= M) continue;
        const float bias = b1[j];
#pragma unroll
        for (int bj = 0; bj < NB; ++bj) {
          const int p = c.n0 + L::col(bj, c.lane);
          if (p < P) {
            const float a = acc_read<AGPR>(acc[bi][bj], i) + bias;
            a_out[(int64_t)p * M + j] = a;
            g_out[(int64_t)p * M + j] = gelu_f(a);
          }
        }
      }
  }
};

// one workgroup per prompt: logZ_p = w2 . g_p + b2
__global__ void logz_out_kernel(const float* g, const float* w2, const float* b2, int M, float* log_z) {
  __shared__ float sh[4];
  const int p = blockIdx.x;
  float s = 0.f;
  for (int j = threadIdx.x; j < M; j += blockDim.x) s += w2[j] * g[(int64_t)p * M + j];
  for (int o = 32; o > 0; o >>= 1) s += __shfl_down(s, o);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) log_z[p] = sh[0] + sh[1] + sh[2] + sh[3] + b2[0];
}

// thread per hidden unit j: da[p][j] for every prompt, db1[j], dw2[j]; thread 0 also db2
__global__ void logz_bwd_vec_kernel(const float* d, const float* a, const float* g, const float* w2, int P, int M,
                                    float* da, float* db1, float* dw2, float* db2) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j == 0) { float s = 0.f; for (int p = 0; p < P; ++p) s += d[p]; db2[0] = s; }
  if (j >= M) return;
  const float w = w2[j];
  float sb = 0.f, sw = 0.f;
  for (int p = 0; p < P; ++p) {
    const float dp = d[p];
    const float v = dp * w * gelu_grad_f(a[(int64_t)p * M + j]);
    da[(int64_t)p * M + j] = v;
    sb += v;
    sw += dp * g[(int64_t)p * M + j];
  }
  db1[j] = sb; dw2[j] = sw;
}

// grid (ceil(H / 256), M): dW1[j][h] = sum_p da[p][j] pooled[p][h]
__global__ void logz_bwd_w1_kernel(const float* da, const float* pooled, int P, int M, int H, float* dW1) {
  const int j = blockIdx.y, h = blockIdx.x * 256 + threadIdx.x;
  if (h >= H) return;
  float s = 0.f;
  for (int p = 0; p < P; ++p) s += da[(int64_t)p * M + j] * pooled[(int64_t)p * H + h];
  dW1[(int64_t)j * H + h] = s;
}

struct LogzPlan { size_t off_pooled, off_a, off_g, off_da, total; };

static inline LogzPlan logz_plan(int P, int H, int M) {
  LogzPlan q; size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o += (bytes + 255) & ~(size_t)255; return at; };
  q.off_pooled = take(4 * (size_t)P * H); q.off_a = take(4 * (size_t)P * M); q.off_g = take(4 * (size_t)P * M);
  q.off_da = take(4 * (size_t)P * M); q.total = o;
  return q;
}

}  // namespace rlk
