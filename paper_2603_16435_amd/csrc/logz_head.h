// logz_head.h - the log-Z head: per-prompt log-partition estimate from the prompt's hidden states.
//
//   pooled_p = mean of the prompt's hidden-state rows        logz_pool_kernel   (HBM-bound: reads the rows once)
//   a_p = W1 pooled_p + b1,  g_p = gelu(a_p)                 logz_hidden_kernel (HBM-bound: W1 streamed once per 16 prompts)
//   logZ_p = w2 . g_p + b2                                   logz_out_kernel
//   backward from d_logZ: da, db1, dw2, db2                  logz_bwd_vec_kernel
//                         dW1 = sum_p da_p pooled_p^T        logz_bwd_w1_kernel  (HBM-bound: writes dW1 once)
//
// The hidden states are constants here (no gradient into the language model).  Parameters and
// activations are f32; the hidden states come in the model's dtype.  All of it is a few tens of
// microseconds next to the policy-loss path: with 16-32 prompts the layer is a matrix-vector product per
// prompt, bound by reading W1 and writing dW1 once, so these are plain bandwidth kernels, not MFMA ones.
#pragma once
#include "gemm_nt.h"

namespace rlk {

__device__ inline float gelu_f(float a) { return 0.5f * a * (1.f + erff(a * 0.70710678118654752f)); }
__device__ inline float gelu_grad_f(float a) {
  return 0.5f * (1.f + erff(a * 0.70710678118654752f)) + a * expf(-0.5f * a * a) * 0.3989422804014327f;
}

// grid (P, ceil(H / 64)): a workgroup pools 64 hidden columns of one prompt; its four wavefronts take every
// fourth row each (f32 sums), merged through LDS
template <class T>
__global__ void logz_pool_kernel(const T* X, int64_t rows, int H, const int32_t* cu, float* pooled) {
  __shared__ float part[4][64];
  const int p = blockIdx.x, c = threadIdx.x & 63, slice = threadIdx.x >> 6;
  const int h = blockIdx.y * 64 + c;
  int64_t a = cu[p], b = cu[p + 1];
  if (a < 0) a = 0;
  if (b > rows) b = rows;
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  if (h < H) {
    int64_t r = a + slice;
    for (; r + 12 < b; r += 16) {                       // four independent loads in flight per thread
      s0 += (float)X[r * H + h]; s1 += (float)X[(r + 4) * H + h];
      s2 += (float)X[(r + 8) * H + h]; s3 += (float)X[(r + 12) * H + h];
    }
    for (; r < b; r += 4) s0 += (float)X[r * H + h];
  }
  part[slice][c] = (s0 + s1) + (s2 + s3);
  __syncthreads();
  if (slice == 0 && h < H) {
    const float s = (part[0][c] + part[1][c]) + (part[2][c] + part[3][c]);
    pooled[(int64_t)p * H + h] = b > a ? s / (float)(b - a) : 0.f;
  }
}

// Hidden layer.  grid (ceil(M / 16), ceil(P / 16)): a workgroup computes 16 units for 16 prompts; each of its four
// wavefronts owns four units.  The pooled states of the 16 prompts go through LDS in chunks of 256 columns; a
// lane multiplies its four columns of the chunk into 4 x 16 accumulators, reduced across the wavefront at the end.
__global__ __launch_bounds__(256) void logz_hidden_kernel(const float* W1, const float* b1, const float* pooled, int P, int H, int M,
                                                          float* a_out, float* g_out) {
  __shared__ float ch[16][256];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j0 = blockIdx.x * 16 + wave * 4, p0 = blockIdx.y * 16;
  float acc[4][16];
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int q = 0; q < 16; ++q) acc[u][q] = 0.f;
  for (int h0 = 0; h0 < H; h0 += 256) {
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int p = p0 + q, h = h0 + threadIdx.x;
      ch[q][threadIdx.x] = (p < P && h < H) ? pooled[(int64_t)p * H + h] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int h = h0 + lane + 64 * k;
      float w[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) w[u] = (j0 + u < M && h < H) ? W1[(int64_t)(j0 + u) * H + h] : 0.f;
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const float x = ch[q][lane + 64 * k];
#pragma unroll
        for (int u = 0; u < 4; ++u) acc[u][q] = fmaf(w[u], x, acc[u][q]);
      }
    }
  }
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      float v = acc[u][q];
      for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o);
      acc[u][q] = v;
    }
  if (lane == 0) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = j0 + u;
      if (j >= M) continue;
      const float bias = b1[j];
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int p = p0 + q;
        if (p < P) { const float a = acc[u][q] + bias; a_out[(int64_t)p * M + j] = a; g_out[(int64_t)p * M + j] = gelu_f(a); }
      }
    }
  }
}

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

// grid (ceil(H / 256), ceil(M / 8)): dW1[j][h] = sum_p da[p][j] pooled[p][h] for eight units j per workgroup, so that a
// pooled value is loaded once for eight outputs; stores are coalesced along h
__global__ void logz_bwd_w1_kernel(const float* da, const float* pooled, int P, int M, int H, float* dW1) {
  const int j0 = blockIdx.y * 8, h = blockIdx.x * 256 + threadIdx.x;
  if (h >= H) return;
  float s[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) s[u] = 0.f;
  for (int p = 0; p < P; ++p) {
    const float x = pooled[(int64_t)p * H + h];
#pragma unroll
    for (int u = 0; u < 8; ++u) if (j0 + u < M) s[u] = fmaf(da[(int64_t)p * M + j0 + u], x, s[u]);
  }
#pragma unroll
  for (int u = 0; u < 8; ++u) if (j0 + u < M) dW1[(int64_t)(j0 + u) * H + h] = s[u];
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
