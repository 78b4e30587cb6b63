// rvq_encode.h - residual vector-quantisation encode of KV-cache vectors (the paper's compression step:
// method section, Eq. 1-2 and Eq. 5-8).  For every vector x (D = 128, bf16) and every one of N stages:
//
//     z_i = argmin_s || r_i - c_{i,s} ||^2 = argmax_s ( r_i . c_{i,s} - ||c_{i,s}||^2 / 2 ),   r_{i+1} = bf16( r_i - c_{i,z_i} )
//
// with the lowest index winning ties and the running residual kept in the cache's 16-bit storage precision.
//
// Mapping to the hardware.  A workgroup of four wavefronts takes 256 vectors of one codebook group and walks all N
// stages with the residuals in registers (already in MFMA operand layout: a lane holds row l%16, 8 consecutive k).
// A stage's codebook (S x 128 bf16) streams through LDS in chunks of 64 entries (16 KiB, double-buffered, fetched
// into registers one chunk ahead); per chunk a wavefront does 64 v_mfma_f32_16x16x32_bf16 (64 vectors x 64 entries
// x K = 128) and folds the 64 scores of each lane into a running (best score, index) pair per row.  Stage end: the
// 16 lanes that share rows merge their pairs (value first, then lower index), the winners go through LDS to the
// lanes that own those rows in operand layout, which fetch the chosen entry (16-byte gathers) and update the residual.
// LDS layout: entry e at 256 e, its 16-byte piece p at slot p ^ (e & 15): fragment reads are conflict-free.
#pragma once
#include "gemm_nt.h"

namespace rlk {

constexpr int kRvqD = 128;          // head dimension the kernel is written for
constexpr int kRvqChunk = 64;       // codebook entries per LDS chunk
constexpr int kRvqVecs = 256;       // vectors per workgroup

// squared norms of the entries, f32 (products of bf16 are exact in f32; summed in index order)
__global__ void rvq_norms_kernel(const bf16_t* cb, int64_t entries, float* cn) {
  const int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= entries) return;
  const uint4* p = reinterpret_cast<const uint4*>(cb + s * kRvqD);
  float acc = 0.f;
  for (int k = 0; k < kRvqD / 8; ++k) {
    const uint4 v = p[k];
    const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float a = __uint_as_float(w[j] << 16), b = __uint_as_float(w[j] & 0xffff0000u);
      acc = fmaf(a, a, acc); acc = fmaf(b, b, acc);
    }
  }
  cn[s] = acc;
}

__device__ inline u32x4_t rvq_sub_bf16(const u32x4_t& r, const u32x4_t& c) {   // bf16(r - c) on eight packed values
  u32x4_t o;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float lo = __uint_as_float(r[j] << 16) - __uint_as_float(c[j] << 16);
    const float hi = __uint_as_float(r[j] & 0xffff0000u) - __uint_as_float(c[j] & 0xffff0000u);
    bf16x2 p; p[0] = (bf16_t)lo; p[1] = (bf16_t)hi;
    o[j] = __builtin_bit_cast(unsigned, p);
  }
  return o;
}

// grid (ceil(L / 256), G).  x [G][L][128], cb [G][N][S][128] bf16, cn [G][N][S] f32, codes [G][L][N] int32,
// residual [G][L][128] bf16 or null.  S % 64 == 0.
__global__ __launch_bounds__(256, 2)
void rvq_encode_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ cb, const float* __restrict__ cn,
                       int L, int N, int S, int32_t* __restrict__ codes, bf16_t* __restrict__ residual) {
  __shared__ __attribute__((aligned(256))) unsigned char buf[2][kRvqChunk * 256];
  __shared__ int zbuf[4][64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int e16 = lane & 15, kq = lane >> 4;
  const int g = blockIdx.y;
  const int v0 = blockIdx.x * kRvqVecs + wave * 64;
  x += (int64_t)g * L * kRvqD; codes += (int64_t)g * L * N;
  cb += (int64_t)g * N * S * kRvqD; cn += (int64_t)g * N * S;
  if (residual) residual += (int64_t)g * L * kRvqD;

  // residuals in operand layout: ra[rb][ks] = row 16 rb + l%16, k = 32 ks + 8 (l/16) .. +7
  u32x4_t ra[4][4];
#pragma unroll
  for (int rb = 0; rb < 4; ++rb) {
    int v = v0 + rb * 16 + e16; v = v < L ? v : L - 1;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) ra[rb][ks] = *reinterpret_cast<const u32x4_t*>(x + (int64_t)v * kRvqD + ks * 32 + kq * 8);
  }

  const int nch = S / kRvqChunk, total = N * nch;
  // staging: thread t moves pieces q = t + 256 j (j = 0..3) of a chunk: entry q/16, LDS slot q%16, i.e. source piece slot ^ (entry & 15)
  u32x4_t st[4];
  float cnn[4], cnc[4];
  auto fetch = [&](int t) __attribute__((always_inline)) {      // chunk t of the linear sequence (stage t / nch, chunk t % nch)
    const bf16_t* base = cb + (int64_t)t * kRvqChunk * kRvqD;    // chunks of consecutive stages are consecutive in memory
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int q = tid + 256 * j, ent = q >> 4, piece = (q & 15) ^ (ent & 15);
      st[j] = *reinterpret_cast<const u32x4_t*>(base + ent * kRvqD + piece * 8);
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) cnn[c] = cn[(int64_t)t * kRvqChunk + c * 16 + e16];
  };
  auto stash = [&](int b) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < 4; ++j) *reinterpret_cast<u32x4_t*>(buf[b] + (tid + 256 * j) * 16) = st[j];
  };

  fetch(0);
  stash(0);
#pragma unroll
  for (int c = 0; c < 4; ++c) cnc[c] = cnn[c];
  __syncthreads();

  float best[4][4]; int bidx[4][4];
  for (int t = 0; t < total; ++t) {
    const int ch = t % nch, stage = t / nch;
    if (ch == 0) {
#pragma unroll
      for (int rb = 0; rb < 4; ++rb)
#pragma unroll
        for (int e = 0; e < 4; ++e) { best[rb][e] = -__builtin_inff(); bidx[rb][e] = 0; }
    }
    if (t + 1 < total) fetch(t + 1);
    const unsigned char* cur = buf[t & 1];
    // the accumulators start at -|c|^2/2 of their column, so the MFMAs leave the score r.c - |c|^2/2 directly
    floatx4 acc[4][4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const float h = -0.5f * cnc[c];
#pragma unroll
      for (int rb = 0; rb < 4; ++rb)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[rb][c][e] = h;
    }
    // codebook fragments are read one k-step ahead of the MFMAs that use them
    u32x4_t fb[2][4];
    auto frag = [&](int set, int ks) __attribute__((always_inline)) {
#pragma unroll
      for (int c = 0; c < 4; ++c) fb[set][c] = *reinterpret_cast<const u32x4_t*>(cur + (c * 16 + e16) * 256 + (((ks * 4 + kq) ^ e16) << 4));
    };
    frag(0, 0);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      if (ks < 3) frag((ks + 1) & 1, ks + 1);
#pragma unroll
      for (int rb = 0; rb < 4; ++rb)
#pragma unroll
        for (int c = 0; c < 4; ++c)
          acc[rb][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ra[rb][ks]), __builtin_bit_cast(bf16x8, fb[ks & 1][c]), acc[rb][c], 0, 0, 0);
    }
    // scores r.c - |c|^2/2 of rows 16 rb + 4 (l/16) + e against entries ch*64 + 16 c + l%16; candidates come in increasing index
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int idx = ch * kRvqChunk + c * 16 + e16;
#pragma unroll
      for (int rb = 0; rb < 4; ++rb)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float v = acc[rb][c][e];
          if (v > best[rb][e]) { best[rb][e] = v; bidx[rb][e] = idx; }
        }
    }
    if (ch == nch - 1) {
      // merge the 16 lanes that hold the same rows: higher score wins, equal scores go to the lower index
#pragma unroll
      for (int rb = 0; rb < 4; ++rb)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float bv = best[rb][e]; int bi = bidx[rb][e];
#pragma unroll
          for (int o = 1; o < 16; o <<= 1) {
            const float ov = __shfl_xor(bv, o); const int oi = __shfl_xor(bi, o);
            if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
          }
          if (e16 == 0) zbuf[wave][rb * 16 + kq * 4 + e] = bi;
        }
      __builtin_amdgcn_s_waitcnt(0xC07F);      // lgkmcnt(0): zbuf visible to the own wavefront (same-wave LDS ordering)
      const bf16_t* stage_cb = cb + (int64_t)stage * S * kRvqD;
#pragma unroll
      for (int rb = 0; rb < 4; ++rb) {
        const int z = zbuf[wave][rb * 16 + e16];
        const int v = v0 + rb * 16 + e16;
        if (kq == 0 && v < L) codes[(int64_t)v * N + stage] = z;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const u32x4_t cz = *reinterpret_cast<const u32x4_t*>(stage_cb + (int64_t)z * kRvqD + ks * 32 + kq * 8);
          ra[rb][ks] = rvq_sub_bf16(ra[rb][ks], cz);
        }
      }
    }
    if (t + 1 < total) {
      stash((t + 1) & 1);
#pragma unroll
      for (int c = 0; c < 4; ++c) cnc[c] = cnn[c];
    }
    __syncthreads();
  }
  if (residual) {
#pragma unroll
    for (int rb = 0; rb < 4; ++rb) {
      const int v = v0 + rb * 16 + e16;
      if (v < L) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) *reinterpret_cast<u32x4_t*>(residual + (int64_t)v * kRvqD + ks * 32 + kq * 8) = ra[rb][ks];
      }
    }
  }
}

}  // namespace rlk
