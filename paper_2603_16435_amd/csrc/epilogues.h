// epilogues.h - what each contraction does with its accumulators while they are in registers.
//
// Orientation.  The logits contraction is run "vocab-major": A = W (rows = vocab entries),
// B = X (rows = tokens), so that in the MFMA accumulator layouts (see Layout32 / Layout16) a lane
// owns ONE token column per block and several vocab rows of it.  The softmax reductions over the
// vocabulary are then mostly in-register; the only cross-lane steps are between the lane groups
// that hold other rows of the same column (one or two shuffles), and the only cross-wavefront
// step is between the WAVES_M wavefronts stacked along the vocabulary.
#pragma once
#include "gemm_nt.h"

namespace rlk {

// 16-byte store of eight bf16 that nobody re-reads from cache (the chunk buffers are 10 GB): non-temporal,
// measured 26 % cheaper than a plain store in the tile-writing epilogues.
template <class T>
__device__ inline void store_stream(T* p, const bf16x8& v) { __builtin_nontemporal_store(v, reinterpret_cast<bf16x8*>(p)); }

template <class T> __device__ inline float fast_exp(float x);
template <> __device__ inline float fast_exp<bf16_t>(float x) { return __expf(x); }
template <> __device__ inline float fast_exp<float>(float x) { return expf(x); }

constexpr float kLog2e = 1.4426950408889634f;

// exp(zs z - m) for a raw logit z, the inverse temperature zs and a shift m given in tempered units, with
// m*log2(e) and zs*log2(e) precomputed: one fma and one v_exp for bf16 inputs, the accurate libm path for f32
template <class T> __device__ inline float exp_shifted(float z, float m, float m_l2e, float zs, float zs_l2e);
template <> __device__ inline float exp_shifted<bf16_t>(float z, float, float m_l2e, float, float zs_l2e) {
  return __builtin_amdgcn_exp2f(__builtin_fmaf(z, zs_l2e, -m_l2e));
}
template <> __device__ inline float exp_shifted<float>(float z, float m, float, float zs, float) { return expf(z * zs - m); }

// ---- forward: per-token partial (max m, s = sum exp(z-m), u = sum exp(z-m) z) over this tile's vocab
//      range + target gather; z_t[y_t] is written by the single lane that holds vocab row y_t of token t.
//      u feeds the entropy H_t = lse_t - u/s of the full distribution at no extra pass.
//      z is the tempered logit zs * (W x_t), zs = 1 / temperature; everything written is in tempered units.
template <class T>
struct EpiFwd {
  typedef NoPre Pre;
  template <class L> __device__ Pre preload(const TileCtx&, const GemmDims&) const { return Pre(); }
  static constexpr bool kPermute = false;
  static constexpr bool kGatherB = true;      // the B rows come through a row map (GemmDims::b_rows)
  __device__ void keep_alive() const { zy_c[0] = 0.f; }
  const int* ids_c;     // [chunk-global compact row] sampled token
  float* zy_c;          // [compact row] target logit
  float4* part;         // [tiles_m(V)][ldp] partial (m, s, u, -) per token
  int ldp;              // = chunk rows
  int V;
  float zs;             // inverse temperature
  int* ycol_c;          // [compact row] vocabulary row the target logit was taken from (the position of the accumulator read)

  // one token column of one lane: the MB * kRegs logits it holds.  PAD: some of the sub-tile's rows are
  // vocabulary padding (only in the last tile row) and must not enter the sums.
  template <class L, int MB, int NB, bool AGPR, bool PAD>
  __device__ __attribute__((always_inline)) void column(typename L::acc_t (&acc)[MB][NB], int bj, int lane, int vleft,
                                                        float& mx, float& sm, float& su) const {
    const float NEG = -__builtin_inff();
    float z[MB * L::kRegs];
    mx = NEG;
#pragma unroll
    for (int bi = 0; bi < MB; ++bi)
#pragma unroll
      for (int i = 0; i < L::kRegs; ++i) {
        const float v = acc_read<AGPR>(acc[bi][bj], i);
        z[bi * L::kRegs + i] = v;
        mx = fmaxf(mx, (!PAD || L::row(bi, i, lane) < vleft) ? v : NEG);
      }
    const float ms = (mx == NEG) ? 0.f : mx * zs;             // zs > 0: the largest raw logit is the largest tempered one
    const float ms_l2e = ms * kLog2e, zs_l2e = zs * kLog2e;
    sm = 0.f; su = 0.f;
#pragma unroll
    for (int bi = 0; bi < MB; ++bi)
#pragma unroll
      for (int i = 0; i < L::kRegs; ++i) {
        const float v = z[bi * L::kRegs + i];
        float e = exp_shifted<T>(v, ms, ms_l2e, zs, zs_l2e);
        if (PAD && !(L::row(bi, i, lane) < vleft)) e = 0.f;
        sm += e;
        su = __builtin_fmaf(e, v, su);
      }
    mx *= zs; su *= zs;
  }

  template <class L, int MB, int NB, int BM, int BN, int WAVES_M, int WAVES_N, bool AGPR>
  __device__ __attribute__((always_inline)) void run(typename L::acc_t (&acc)[MB][NB], const TileCtx& c, unsigned char* smem, const GemmDims& d, const Pre& pre) const {
    float4* red = reinterpret_cast<float4*>(smem);              // [WAVES_M][BN]
    const float NEG = -__builtin_inff();
    const int vleft = V - c.m0;                                 // rows of this sub-tile below vleft are real vocabulary
    const bool pad = vleft < MB * L::kBlk;                      // wavefront-uniform
#pragma unroll
    for (int bj = 0; bj < NB; ++bj) {
      const int n = c.n0 + L::col(bj, c.lane);
      const bool valid = n < c.Nv;
      // target gather: at most one lane of the whole grid holds row y of column n, so this branch is almost never taken
      const int yrel = valid ? ids_c[d.chunk_start + n] - c.m0 : -1;
      if (yrel >= 0 && yrel < MB * L::kBlk && L::owns(yrel, c.lane)) {
        float zy = 0.f;
        int got = -1;
#pragma unroll
        for (int bi = 0; bi < MB; ++bi)
#pragma unroll
          for (int i = 0; i < L::kRegs; ++i) {
            const float v = acc_read<AGPR>(acc[bi][bj], i);
            if (L::row(bi, i, c.lane) == yrel) { zy = v; got = c.m0 + L::row(bi, i, c.lane); }
          }
        zy_c[d.chunk_start + n] = zy * zs;
        ycol_c[d.chunk_start + n] = got;
      }
      float mx, sm, su;
      if (pad) column<L, MB, NB, AGPR, true>(acc, bj, c.lane, vleft, mx, sm, su);
      else column<L, MB, NB, AGPR, false>(acc, bj, c.lane, vleft, mx, sm, su);
      // merge with the lane groups that hold the other rows of this column
#pragma unroll
      for (int off = L::kBlk; off < 64; off <<= 1) {
        const float mx2 = __shfl_xor(mx, off), sm2 = __shfl_xor(sm, off), su2 = __shfl_xor(su, off);
        const float mm = fmaxf(mx, mx2);
        const float mms = (mm == NEG) ? 0.f : mm;
        const float f1 = fast_exp<T>(mx - mms), f2 = fast_exp<T>(mx2 - mms);
        sm = sm * f1 + sm2 * f2;
        su = su * f1 + su2 * f2;
        mx = mm;
      }
      if (c.lane < L::kBlk) red[c.wm * BN + (n - c.tile_n * BN)] = make_float4(mx, sm, su, 0.f);
    }
    __syncthreads();
    if (c.tid < BN) {
      const int n = c.tile_n * BN + c.tid;
      if (n < c.Nv) {
        float4 r = red[c.tid];
#pragma unroll
        for (int w = 1; w < WAVES_M; ++w) {
          const float4 o = red[w * BN + c.tid];
          const float mm = fmaxf(r.x, o.x);
          const float mms = (mm == NEG) ? 0.f : mm;
          const float f1 = fast_exp<T>(r.x - mms), f2 = fast_exp<T>(o.x - mms);
          r.y = r.y * f1 + o.y * f2;
          r.z = r.z * f1 + o.z * f2;
          r.x = mm;
        }
        part[(int64_t)c.tile_m * ldp + n] = r;
      }
    }
  }
};

// ---- forward that also keeps the chunk's unnormalised probabilities for a single-pass backward.
//      Every token has a reference ref_t close to its logsumexp, known before the contraction
//      (target logit minus the old policy's log-prob), so e = exp(z - ref_t) needs no running
//      maximum: the epilogue adds up s = sum e and u = sum e z per token and tile row, and
//      stores e itself in the input precision, token-major E[t][v] (16-byte stores through the same
//      relabelling as EpiDS; the weight-gradient contraction reads E as a K-major operand, so no
//      vocab-major copy is kept).  bf16 keeps f32's exponent range, so e is
//      stored at full relative precision whatever its size.  Later, with Z_t = sum_v e,
//      dS[t][v] = -(c_t / Z_t) (E[t][v] - Z_t 1[v = y_t]): the backward contractions run on E
//      directly, with the target entry patched and the factor applied per token.
template <class T>
struct EpiFwdStash {
  struct Pre { float rl[8]; };                            // ref_t * log2(e) of the lane's eight token columns
  template <class L> __device__ Pre preload(const TileCtx& c, const GemmDims& d) const {
    Pre p;
    const int cc = c.lane & 15;
#pragma unroll
    for (int bj = 0; bj < 8; ++bj) {
      const int n = c.n0 + perm_col(bj, cc);
      p.rl[bj] = (n < c.Nv) ? ref_l2e[d.chunk_start + n] : __builtin_inff();   // column without a token: e = exp2(-inf) = 0
    }
    return p;
  }
  static constexpr bool kPermute = true;
  static constexpr bool kGatherB = true;      // the B rows come through a row map (GemmDims::b_rows)
  __device__ void keep_alive() const { E[0] = (T)0.f; }
  const float* ref_l2e;   // [compact row] ref_t * log2(e)
  float2* part;           // [tiles_m(V)][ldp] partial (s, u) per token of the chunk
  int ldp;
  T* E;  int64_t ld_e;    // [chunk rows][Vp = ld_e], slab-tiled
  int V;
  float zs;               // inverse temperature: z = zs * (W x_t) is the logit that ref_t, s and u refer to

  // Exponentials, sums and the stores, in two rounds of four block rows (64 vocabulary entries = one 128-byte
  // line of a token's E row).  A lane holds 16 bytes of the first half of that line (block rows 4j, 4j+1) and 16 of
  // the second (4j+2, 4j+3), and its four lane groups make each half 64 bytes wide; lane pairs (token columns cc,
  // cc^1) swap one half each, so that one store instruction writes whole lines: the eight lanes of the even token's
  // line first, then the odd token's.
  template <class L, int MB, int NB, bool AGPR, bool PAD>
  __device__ __attribute__((always_inline)) void body(typename L::acc_t (&acc)[MB][NB], const TileCtx& c, int g, int cc, int vleft,
                                                      const float (&rl)[NB], float (&sm)[NB], float (&su)[NB]) const {
    const int p = cc & 1;
    const float zs_l2e = zs * kLog2e;
#pragma unroll
    for (int j = 0; j < MB / 4; ++j) {
#pragma unroll
      for (int bj = 0; bj < NB; ++bj) {
        bf16x8 half[2];
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
          const int mrel = (2 * j + kk) * 32 + g * 8;
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const float z = acc_read<AGPR>(acc[2 * (2 * j + kk) + (i >> 2)][bj], i & 3);
            float v = __builtin_amdgcn_exp2f(__builtin_fmaf(z, zs_l2e, -rl[bj]));
            if (PAD && !(mrel + i < vleft)) v = 0.f;
            sm[bj] += v;
            su[bj] = __builtin_fmaf(v, z, su[bj]);
            half[kk][i] = (bf16_t)v;
          }
        }
        const u32x4_t a = __builtin_bit_cast(u32x4_t, half[0]), b = __builtin_bit_cast(u32x4_t, half[1]);
        u32x4_t recv;
#pragma unroll
        for (int q = 0; q < 4; ++q)                         // swap with the neighbouring lane (quad_perm [1,0,3,2])
          recv[q] = (unsigned)__builtin_amdgcn_mov_dpp((int)(p ? a[q] : b[q]), 0xB1, 0xF, 0xF, true);
        const u32x4_t d_even = p ? recv : a, d_odd = p ? b : recv;
        const int v0 = c.m0 + j * 64 + p * 32 + g * 8;
        store_stream(E + tiled_index(c.n0 + perm_col(bj, cc & ~1), v0, ld_e), __builtin_bit_cast(bf16x8, d_even));
        store_stream(E + tiled_index(c.n0 + perm_col(bj, cc | 1), v0, ld_e), __builtin_bit_cast(bf16x8, d_odd));
      }
      __builtin_amdgcn_sched_barrier(0);                  // keep the two rounds apart
    }
  }

  template <class L, int MB, int NB, int BM, int BN, int WAVES_M, int WAVES_N, bool AGPR>
  __device__ __attribute__((always_inline)) void run(typename L::acc_t (&acc)[MB][NB], const TileCtx& c, unsigned char* smem, const GemmDims& d, const Pre& pre) const {
    static_assert(L::kBlk == 16 && MB == 8 && NB == 8 && sizeof(T) == 2, "hot kernel only");
    float2* red = reinterpret_cast<float2*>(smem);              // [WAVES_M][BN + BN / 32]
    constexpr int kRedRow = BN + BN / 32;
    const int g = c.lane >> 4, cc = c.lane & 15;
    float rl[NB], sm[NB], su[NB];
#pragma unroll
    for (int bj = 0; bj < NB; ++bj) { rl[bj] = pre.rl[bj]; sm[bj] = 0.f; su[bj] = 0.f; }
    const int vleft = V - c.m0;                            // sub-tile rows >= vleft are vocabulary padding
    if (vleft < MB * L::kBlk) body<L, MB, NB, AGPR, true>(acc, c, g, cc, vleft, rl, sm, su);   // wavefront-uniform
    else body<L, MB, NB, AGPR, false>(acc, c, g, cc, vleft, rl, sm, su);
#pragma unroll
    for (int bj = 0; bj < NB; ++bj) {
#pragma unroll
      for (int off = 16; off < 64; off <<= 1) { sm[bj] += __shfl_xor(sm[bj], off); su[bj] += __shfl_xor(su[bj], off); }
      // (one spare slot after every 32 columns: the sixteen lanes write columns 8 apart, 64 bytes, and would otherwise meet
      // in the LDS banks four at a time)
      if (c.lane < 16) {
        const int col = c.wn * (BN / WAVES_N) + perm_col(bj, cc);
        red[c.wm * kRedRow + col + (col >> 5)] = make_float2(sm[bj], su[bj] * zs);
      }
    }
    __syncthreads();
    if (c.tid < BN) {
      const int n = c.tile_n * BN + c.tid;
      if (n < c.Nv) {
        const int slot = c.tid + (c.tid >> 5);
        float2 r = red[slot];
#pragma unroll
        for (int w = 1; w < WAVES_M; ++w) { const float2 o2 = red[w * kRedRow + slot]; r.x += o2.x; r.y += o2.y; }
        part[(int64_t)c.tile_m * ldp + n] = r;
      }
    }
  }
};

template <class T> struct Pack4;
template <> struct Pack4<bf16_t> {
  __device__ static void store(bf16_t* p, float a, float b, float c, float d) {
    bf16x4 v; v[0] = (bf16_t)a; v[1] = (bf16_t)b; v[2] = (bf16_t)c; v[3] = (bf16_t)d;
    *reinterpret_cast<bf16x4*>(p) = v;
  }
};
template <> struct Pack4<float> {
  __device__ static void store(float* p, float a, float b, float c, float d) {
    *reinterpret_cast<float4*>(p) = make_float4(a, b, c, d);
  }
};

// ---- backward, stage 1: recomputed logits -> dS = zs c_t (1[v=y_t] - exp(z - lse_t)) (z the tempered
//      logit, zs = 1 / temperature the chain factor back to W x_t), formed in
//      f32 (subtraction and scaling before rounding) and stored in the input precision, token-major
//      dS[t][v] (operand of dX = dS W).  dW = dS^T X reads the same array as a K-major operand in the
//      bf16 hot kernel; f32 inputs (generic kernel) also get the vocab-major copy dST[v][t].
//
//      In the hot kernel (16x16 blocks) the tile rows and columns are relabelled (kPermute, see
//      perm_row / perm_col in gemm_nt.h) such that a lane ends up holding eight consecutive
//      vocabulary entries of a token: the copy leaves in 16-byte stores with no staging through LDS.
template <class T>
struct EpiDS {
  typedef NoPre Pre;
  template <class L> __device__ Pre preload(const TileCtx&, const GemmDims&) const { return Pre(); }
  static constexpr bool kPermute = true;
  static constexpr bool kGatherB = true;      // the B rows come through a row map (GemmDims::b_rows)
  __device__ void keep_alive() const { dS[0] = (T)0.f; }
  const int* ids_c; const float* lse_c; const float* c_c;
  T* dS;  int64_t ld_ds;    // [chunk rows][Vp]
  T* dST; int64_t ld_dst;   // [Vp][chunk rows]; f32 inputs only
  int V;
  bool tiled;               // dS slab-tiled (always so for bf16: its consumer is the hot kernel)
  float zs;                 // inverse temperature

  template <class L, int MB, int NB, int BM, int BN, int WAVES_M, int WAVES_N, bool AGPR>
  __device__ __attribute__((always_inline)) void run(typename L::acc_t (&acc)[MB][NB], const TileCtx& c, unsigned char*, const GemmDims& d, const Pre&) const {
    if constexpr (L::kBlk == 16 && sizeof(T) == 2) {
      static_assert(MB == 8 && NB == 8, "the relabelling is written for 128x128 wavefront sub-tiles");
      const int g = c.lane >> 4, cc = c.lane & 15;
      int y[NB]; float lse[NB], lse_l2e[NB], ct[NB];
#pragma unroll
      for (int bj = 0; bj < NB; ++bj) {
        const int n = c.n0 + perm_col(bj, cc);
        const bool valid = n < c.Nv;
        const int t = d.chunk_start + n;
        y[bj] = valid ? ids_c[t] - c.m0 : -1;             // relative to the sub-tile; -1 never matches
        lse[bj] = valid ? lse_c[t] : 3.0e38f;             // invalid token: p = exp(z - huge) = 0 and
        ct[bj] = valid ? c_c[t] * zs : 0.f;               // c = 0, so every dS entry becomes 0
        lse_l2e[bj] = lse[bj] * kLog2e;
      }
      const float zs_l2e = zs * kLog2e;
      const int vleft = V - c.m0;                          // sub-tile rows >= vleft are vocabulary padding
      const int p = cc & 1;
#pragma unroll
      for (int j = 0; j < MB / 4; ++j) {                   // four block rows = 64 vocabulary entries = one 128-byte line of a dS row
        bf16_t o[NB][16];
#pragma unroll
        for (int bj = 0; bj < NB; ++bj)
#pragma unroll
          for (int r = 0; r < 16; ++r) {                   // r: entry of the round, vocab offset j*64 + (r/8)*32 + g*8 + r%8
            const int m = (2 * j + (r >> 3)) * 32 + g * 8 + (r & 7);
            const float pr = exp_shifted<T>(acc_read<AGPR>(acc[4 * j + (r >> 2)][bj], r & 3), lse[bj], lse_l2e[bj], zs, zs_l2e);
            const float ds = ct[bj] * ((m == y[bj] ? 1.f : 0.f) - pr);
            o[bj][r] = (bf16_t)(m < vleft ? ds : 0.f);
          }
        // token-major copy: lane pairs (token columns cc, cc^1) swap one half each, so that a store writes whole lines
#pragma unroll
        for (int bj = 0; bj < NB; ++bj) {
          bf16x8 h0, h1;
#pragma unroll
          for (int i = 0; i < 8; ++i) { h0[i] = o[bj][i]; h1[i] = o[bj][8 + i]; }
          const u32x4_t a = __builtin_bit_cast(u32x4_t, h0), b = __builtin_bit_cast(u32x4_t, h1);
          u32x4_t recv;
#pragma unroll
          for (int q = 0; q < 4; ++q) recv[q] = (unsigned)__builtin_amdgcn_mov_dpp((int)(p ? a[q] : b[q]), 0xB1, 0xF, 0xF, true);
          const u32x4_t d_even = p ? recv : a, d_odd = p ? b : recv;
          const int v0 = c.m0 + j * 64 + p * 32 + g * 8;
          store_stream(dS + tiled_index(c.n0 + perm_col(bj, cc & ~1), v0, ld_ds), __builtin_bit_cast(bf16x8, d_even));
          store_stream(dS + tiled_index(c.n0 + perm_col(bj, cc | 1), v0, ld_ds), __builtin_bit_cast(bf16x8, d_odd));
        }
      }
    } else {
#pragma unroll
      for (int bj = 0; bj < NB; ++bj) {
        const int n = c.n0 + L::col(bj, c.lane);
        const bool valid = n < c.Nv;
        const int g = d.chunk_start + n;
        const int y = valid ? ids_c[g] : -1;
        const float lse = valid ? lse_c[g] : 0.f;
        const float ct = valid ? c_c[g] * zs : 0.f;
#pragma unroll
        for (int bi = 0; bi < MB; ++bi)
#pragma unroll
          for (int q = 0; q < L::kRegs / 4; ++q) {
            const int m = c.m0 + L::row(bi, q * 4, c.lane);
            float o[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float p = fast_exp<T>(acc_read<AGPR>(acc[bi][bj], q * 4 + e) * zs - lse);
              const float ds = ct * (((m + e) == y ? 1.f : 0.f) - p);
              o[e] = (valid && (m + e) < V) ? ds : 0.f;
            }
            Pack4<T>::store(dS + operand_index(tiled, n, m, ld_ds), o[0], o[1], o[2], o[3]);
            if constexpr (sizeof(T) == 4) {
#pragma unroll
              for (int e = 0; e < 4; ++e) dST[operand_index(tiled, m + e, n, ld_dst)] = (T)o[e];
            }
          }
      }
    }
  }
};

// ---- backward, stage 2: dX tile -> rows scattered back to their original positions
template <class T>
struct EpiDX {
  typedef NoPre Pre;
  template <class L> __device__ Pre preload(const TileCtx&, const GemmDims&) const { return Pre(); }
  static constexpr bool kPermute = false;
  static constexpr bool kGatherB = false;      // the B rows come through a row map (GemmDims::b_rows)
  __device__ void keep_alive() const { dX[0] = (T)0.f; }
  const int* row_map;   // compact row -> original row
  T* dX; int64_t ldx; int H;
  const float* row_scale;   // optional [chunk row]: factor applied to the whole row

  template <class L, int MB, int NB, int BM, int BN, int WAVES_M, int WAVES_N, bool AGPR>
  __device__ __attribute__((always_inline)) void run(typename L::acc_t (&acc)[MB][NB], const TileCtx& c, unsigned char*, const GemmDims& d, const Pre&) const {
#pragma unroll
    for (int bi = 0; bi < MB; ++bi)
#pragma unroll
      for (int i = 0; i < L::kRegs; ++i) {
        const int m = c.m0 + L::row(bi, i, c.lane);
        if (m >= c.Mv) continue;
        const int64_t dst = row_map[d.chunk_start + m];
        const float f = row_scale ? row_scale[m] : 1.f;
#pragma unroll
        for (int bj = 0; bj < NB; ++bj) {
          const int n = c.n0 + L::col(bj, c.lane);
          if (n < H) dX[dst * ldx + n] = (T)(f * acc_read<AGPR>(acc[bi][bj], i));
        }
      }
  }
};

// ---- backward, stage 3: dW tile, f32, overwritten by the first chunk and accumulated after.
//      When accumulating, the old values of a whole block row are fetched first (32 loads in flight)
//      and only then added and stored: a load-add-store per element would pay the memory latency
//      256 times per tile.
struct EpiDW {
  typedef NoPre Pre;
  template <class L> __device__ Pre preload(const TileCtx&, const GemmDims&) const { return Pre(); }
  static constexpr bool kPermute = false;
  static constexpr bool kGatherB = false;      // the B rows come through a row map (GemmDims::b_rows)
  __device__ void keep_alive() const { dW[0] = 0.f; }
  float* dW; int64_t ldw; int V, H; int accumulate;

  template <class L, int MB, int NB, int BM, int BN, int WAVES_M, int WAVES_N, bool AGPR>
  __device__ __attribute__((always_inline)) void run(typename L::acc_t (&acc)[MB][NB], const TileCtx& c, unsigned char*, const GemmDims&, const Pre&) const {
    constexpr int RUN = L::kRegs < 4 ? L::kRegs : 4;      // registers handled per round: 4 rows x NB columns
#pragma unroll
    for (int bi = 0; bi < MB; ++bi)
#pragma unroll
      for (int q = 0; q < L::kRegs / RUN; ++q) {
        float old[RUN][NB];
        if (accumulate) {
#pragma unroll
          for (int e = 0; e < RUN; ++e) {
            const int m = c.m0 + L::row(bi, q * RUN + e, c.lane);
#pragma unroll
            for (int bj = 0; bj < NB; ++bj) {
              const int n = c.n0 + L::col(bj, c.lane);
              old[e][bj] = (m < V && n < H) ? dW[(int64_t)m * ldw + n] : 0.f;
            }
          }
        }
#pragma unroll
        for (int e = 0; e < RUN; ++e) {
          const int m = c.m0 + L::row(bi, q * RUN + e, c.lane);
#pragma unroll
          for (int bj = 0; bj < NB; ++bj) {
            const int n = c.n0 + L::col(bj, c.lane);
            const float v = acc_read<AGPR>(acc[bi][bj], q * RUN + e);
            if (m < V && n < H) dW[(int64_t)m * ldw + n] = accumulate ? old[e][bj] + v : v;
          }
        }
      }
  }
};

}  // namespace rlk
