// rvq_encode.h - residual vector-quantisation encode of KV-cache vectors (the paper's compression step:
// method section, Eq. 1-2 and Eq. 5-8).  For every vector x (D = 128, bf16) and every one of N stages:
//
//     z_i = argmin_s || r_i - c_{i,s} ||^2 = argmax_s ( r_i . c_{i,s} - ||c_{i,s}||^2 / 2 ),   r_{i+1} = bf16( r_i - c_{i,z_i} )
//
// with the lowest index winning ties and the running residual kept in the cache's 16-bit storage precision.
//
// Mapping to the hardware.  A workgroup of eight wavefronts (four when a group has at most 256 vectors) takes 64 vectors
// per wavefront of one codebook group and walks all N stages with the residuals in registers, already in MFMA operand
// layout (a lane holds vector l%16 of a block of 16, 8 consecutive k).  A stage's codebook (S x 128 bf16) streams through
// LDS in chunks of 64 entries (16 KiB; three stages, filled by global -> LDS loads two chunks ahead).  The scores are
// computed ENTRY-major: A = 16 entries, B = 16 vectors, so that in the accumulator layout a lane owns ONE vector per block
// and four entries of it.  The accumulators of a block of 16 entries start at -|c|^2/2 through the MFMA's C operand, and the
// blocks of a chunk are software-pipelined: the bookkeeping of block c runs under the MFMAs of block c+1.
// Running arg-max.  MFMA and vector instructions leave through the same issue port of a SIMD (4 cycles each, a 16x16x32 MFMA
// lasts 16), so the bookkeeping per score decides the speed.  A lane therefore keeps its state per BLOCK of four scores (its
// four entries of a 16-entry block): the three largest block maxima so far, each carrying the number of its block in its
// lowest mantissa bits, and the four scores of the best block - eleven vector operations per four scores, where a compare
// and two selects per score take sixteen.  Which of the four scores won is looked up once per stage, and the four lanes that
// share a vector merge with two row swaps; the winner's index is then already in the lanes that hold that vector's residual.
//
// Exactness.  The scores come out of f32 accumulation, the definition is exact.  Products of bf16 values are exact in
// f32, so a score differs from its exact value by at most g (|r| |c| + |c|^2 / 2) with g = 2^-16 (256 roundings of
// relative size 2^-24 would be needed to exceed it; a score goes through about 160); a block maximum moves by at most
// 2^(nb - 23) of itself more when the nb bits of its block number are written into it.  If the best score of a vector
// leads every other by more than the margin 2 (g + 2^(nb - 23)) (|r| c_max + c_max^2 / 2), the winner is the exact arg-max.
// Otherwise (about one decision in 400, and always for duplicated entries) the decision is taken in float64 straight from
// the definition, sum_d (r_d - c_d)^2 on the stored bf16 values, smallest distance first, lowest index on ties, among the
// entries whose score came within the margin: those are the only ones that can be the exact arg-min.  They are the near
// scores of the lanes' best blocks (entries known) and, where a lane's second-largest block maximum is that close, the four
// entries of that block: the wavefront settles the vector among them by itself.  Only when a lane's third-largest block
// maximum is within the margin as well are there entries nobody can name, and the workgroup looks at the whole stage again
// (below).  The codes therefore equal the float64 arg-min of the definition, not just a nearest entry up to rounding.  (The
// bound is relative: it assumes that products and partial sums stay in float32's normal range - no underflow, no overflow -
// which holds for any cache values of interest, |x| between 1e-15 and 1e15, say.  S <= 65536: block numbers of 12 bits.)
// LDS layout: entry e at 256 e, its 16-byte piece p at slot p ^ (e & 15): fragment reads are conflict-free.
#pragma once
#include "gemm_nt.h"

namespace rlk {

constexpr int kRvqD = 128;          // head dimension the kernel is written for
constexpr int kRvqChunk = 64;       // codebook entries per LDS chunk
// (a workgroup of kW wavefronts takes 64 kW vectors: kW = 8, one workgroup per CU, when there are more than 256 vectors
// in a group - the chunk in LDS then serves twice the vectors per load - else kW = 4, two workgroups per CU)
constexpr float kRvqGamma2 = 3.0517578125e-05f;   // 2 g = 2^-15: twice the bound on the relative error of an f32 score

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

// bf16(r - c) on eight packed values; ss += the squares of the eight differences before they are rounded (a bound on the new
// vector's squared norm to one part in 2^7, which is all the margin needs of it)
__device__ inline u32x4_t rvq_sub_bf16(const u32x4_t& r, const u32x4_t& c, float& ss) {
  u32x4_t o;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float lo = __uint_as_float(r[j] << 16) - __uint_as_float(c[j] << 16);
    const float hi = __uint_as_float(r[j] & 0xffff0000u) - __uint_as_float(c[j] & 0xffff0000u);
    ss = fmaf(lo, lo, ss); ss = fmaf(hi, hi, ss);
    bf16x2 p; p[0] = (bf16_t)lo; p[1] = (bf16_t)hi;
    o[j] = __builtin_bit_cast(unsigned, p);
  }
  return o;
}

__device__ inline float rvq_sumsq(const u32x4_t& r, float acc) {               // acc + sum of squares of eight packed bf16
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float lo = __uint_as_float(r[j] << 16), hi = __uint_as_float(r[j] & 0xffff0000u);
    acc = fmaf(lo, lo, acc); acc = fmaf(hi, hi, acc);
  }
  return acc;
}

// The four lanes that share a vector are 16 lanes (one row) apart.  v_permlane16_swap / v_permlane32_swap hand a lane its own
// value and that of its partner across rows (l ^ 16, l ^ 32) in an order that is the same for both partners, so any symmetric
// function of the pair leaves both with the same result - at vector-ALU speed, where a shuffle goes through LDS.
template <int kRows>
__device__ __attribute__((always_inline)) inline void rvq_pair(unsigned v, unsigned& a, unsigned& b) {
  if constexpr (kRows == 16) { const auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false); a = r[0]; b = r[1]; }
  else { const auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false); a = r[0]; b = r[1]; }
}
__device__ __attribute__((always_inline)) inline float rvq_sum4(float v) {       // sum over the vector's four lanes
  unsigned a, b;
  rvq_pair<16>(__float_as_uint(v), a, b); v = __uint_as_float(a) + __uint_as_float(b);
  rvq_pair<32>(__float_as_uint(v), a, b); return __uint_as_float(a) + __uint_as_float(b);
}
__device__ __attribute__((always_inline)) inline float rvq_max4(float v) {
  unsigned a, b;
  rvq_pair<16>(__float_as_uint(v), a, b); v = fmaxf(__uint_as_float(a), __uint_as_float(b));
  rvq_pair<32>(__float_as_uint(v), a, b); return fmaxf(__uint_as_float(a), __uint_as_float(b));
}

// ---- exact decisions by the whole workgroup, for the vectors with a near score whose entry nobody can name (rare: three
// block maxima of one lane within the margin).  At the end of a stage, up to 16 such vectors at a time:
//  1. The vectors become the 16 columns of an MFMA B operand and the float32 scores r . c - |c|^2 / 2 of all S entries
//     are recomputed on the matrix cores, an equal share of the entries per wavefront, fetched straight from memory in
//     operand layout, four groups of 16 entries in flight.
//  2. An entry within the vector's margin (twice the bound on a score's error) of the largest score could be the exact
//     arg-max; no other entry can.  The largest recomputed score is at least the main pass's best score minus the margin
//     (both are within the error bound of the same exact value), and no smaller than any running maximum; so every such
//     entry is within the margin of max(that floor, the lane's running maximum) when it arrives.  Those are listed per
//     vector (two or three), and the list is then cut down against the final maximum.
//  3. The survivors are evaluated from the definition in float64, sum_d (r_d - c_d)^2 from the stored bf16 values; the
//     smallest distance wins, the lowest index on ties.
constexpr int kRvqSlots = 16;       // vectors resolved per round
constexpr int kRvqCand = 32;        // listed entries per vector; more (that many scores within twice the margin): all S evaluated
struct RvqResolveLds {
  u32x4_t bits[kRvqSlots][kRvqD / 8];     // the vectors as stored: 16 pieces of eight bf16 each
  float margin[kRvqSlots];
  float best[kRvqSlots];                  // the main pass's best score
  int owner[kRvqSlots];                   // 64 * wavefront + 16 * vector block + vector: who gets the answer
  int count[kRvqSlots];                   // entries listed (may run past kRvqCand: then the list is not used)
  int cand[kRvqSlots][kRvqCand];
  float cscore[kRvqSlots][kRvqCand];
  float top[kRvqSlots][32];               // running maxima at the end of the pass, per wavefront and lane group
  int result[kRvqSlots];
  int n;                                  // vectors that asked for a slot this round (may exceed kRvqSlots: the rest go next round)
};

// Squared distance of the vector in slot j to one entry, straight from the definition in float64: lane l takes components
// 2 l and 2 l + 1, the 64 partial sums are added in a fixed tree (the same for every entry, so equal entries give equal sums).
__device__ __attribute__((always_inline)) inline double rvq_exact_distance(const u32x4_t* bits, const bf16_t* stage_cb, int ent, int lane) {
  const unsigned w = *reinterpret_cast<const unsigned*>(stage_cb + (int64_t)ent * kRvqD + 2 * lane);
  const unsigned r = reinterpret_cast<const unsigned*>(bits)[lane];
  const double d0 = (double)__uint_as_float(r << 16) - (double)__uint_as_float(w << 16);
  const double d1 = (double)__uint_as_float(r & 0xffff0000u) - (double)__uint_as_float(w & 0xffff0000u);
  double acc = fma(d1, d1, d0 * d0);
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) acc += __shfl_xor(acc, o);
  return acc;
}

// The same for four entries at once, one per group of 16 lanes: lane t of a group takes components 8 t .. 8 t + 7 in order,
// the 16 partial sums are added in a fixed tree.  ent < 0: no entry for this group (+inf).  All 64 lanes must call it.
__device__ __attribute__((always_inline)) inline double rvq_exact_distance16(const u32x4_t* bits, const bf16_t* stage_cb, int ent, int t) {
  double acc = __builtin_inf();
  if (ent >= 0) {
    const u32x4_t w = *reinterpret_cast<const u32x4_t*>(stage_cb + (int64_t)ent * kRvqD + 8 * t);
    const u32x4_t r = bits[t];
    acc = 0.0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const double d0 = (double)__uint_as_float(r[j] << 16) - (double)__uint_as_float(w[j] << 16);
      const double d1 = (double)__uint_as_float(r[j] & 0xffff0000u) - (double)__uint_as_float(w[j] & 0xffff0000u);
      acc = fma(d0, d0, acc); acc = fma(d1, d1, acc);
    }
  }
#pragma unroll
  for (int o = 1; o < 16; o <<= 1) acc += __shfl_xor(acc, o);
  return acc;
}

// grid 8 ceil(G / 8) ceil(L / 256) workgroups (see the kernel for who takes what).  x [G][L][128], cb [G][N][S][128] bf16, cn [G][N][S] f32, codes [G][L][N] int32,
// residual [G][L][128] bf16 or null.  S % 64 == 0.  stats (optional): [0] += decisions re-evaluated exactly.
template <int kW>
__global__ __launch_bounds__(64 * kW, 8 / kW)
void rvq_encode_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ cb, const float* __restrict__ cn,
                       int G, int L, int N, int S, int32_t* __restrict__ codes, bf16_t* __restrict__ residual, int32_t* __restrict__ stats) {
  // three stages of a chunk each: chunk t is computed on while chunks t+1 and t+2 are on their way (with one chunk ahead
  // only, the wait for it at the end of every chunk costs about a memory latency: the MFMA-only loop ran at half speed)
  // The fragment reads of the main loop are inline assembly with the wavefront's own waits (read1 / lds_wait below): the
  // compiler, seeing a read of an LDS array that loads in flight may write to, would wait for all of them before every read.
  __shared__ __attribute__((aligned(1024))) unsigned char bufs[3][kRvqChunk * 256];
  __shared__ __attribute__((aligned(256))) float nrms[3][kRvqChunk];
  __shared__ RvqResolveLds rq;                    // exact re-evaluation at the end of a stage
  __shared__ u32x4_t wvec[kW][kRvqD / 8];          // ... and one vector per wavefront for what it settles by itself
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int e16 = lane & 15, kq = lane >> 4;
  // Workgroups are handed to the eight XCDs in turn (w % 8), each with an L2 of its own.  The workgroups of one group read the
  // same codebooks at the same time, so they are given numbers w that agree modulo 8: on its XCD, workgroup q = w / 8 takes
  // block q % gx of group 8 (q / gx) + w % 8, and the codebooks come out of memory once instead of once per block.
  constexpr int kRvqVecs = 64 * kW;
  const int w = blockIdx.x, gx = (L + kRvqVecs - 1) / kRvqVecs;
  const int g = 8 * ((w >> 3) / gx) + (w & 7);
  if (g >= G) return;                             // (the whole workgroup: the grid covers ceil(G / 8) * 8 groups)
  const int v0 = ((w >> 3) % gx) * kRvqVecs + wave * 64;
  x += (int64_t)g * L * kRvqD; codes += (int64_t)g * L * N;
  cb += (int64_t)g * N * S * kRvqD; cn += (int64_t)g * N * S;
  if (residual) residual += (int64_t)g * L * kRvqD;

  // residuals in operand layout: ra[rb][ks] = vector 16 rb + l%16, k = 32 ks + 8 (l/16) .. +7
  u32x4_t ra[4][4];
  float rn2[4];                                   // squared norm of the lane's four vectors (f32, all 128 components)
#pragma unroll
  for (int rb = 0; rb < 4; ++rb) {
    int v = v0 + rb * 16 + e16; v = v < L ? v : L - 1;
    float a = 0.f;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      ra[rb][ks] = *reinterpret_cast<const u32x4_t*>(x + (int64_t)v * kRvqD + ks * 32 + kq * 8);
      a = rvq_sumsq(ra[rb][ks], a);
    }
    rn2[rb] = rvq_sum4(a);
  }

  const int nch = S / kRvqChunk, total = N * nch;
  // staging: chunk t of the linear sequence (stage t / nch, chunk t % nch; consecutive in memory) goes straight from
  // global memory into LDS in sixteen loads of 1 KiB, 16 / kW per wavefront.  Wavefront w, load j writes pieces
  // q = 64 (kW j + w) + l: entry q / 16 = 4 (kW j + w) + l/16, LDS slot q % 16, which holds source piece slot ^ (entry & 15).
  // (entry & 15 = (4 w + l/16) & 15 does not depend on j: one lane offset serves all of a wavefront's loads)
  const unsigned lane_off = (unsigned)((4 * wave + kq) * kRvqD + 8 * (e16 ^ ((4 * wave + kq) & 15)));
  // load j of chunk t; the loads of the chunk after next are issued one per block of the current one (kW = 8: in blocks 0
  // and 2), because a global -> LDS load stalls its wavefront longest when many wavefronts issue one at the same moment
  auto stage_in1 = [&](int t, int j, unsigned loff, unsigned ln, unsigned char* dst, float* ndst) __attribute__((always_inline)) {
    const bf16_t* base = cb + (int64_t)t * kRvqChunk * kRvqD;
    load16_to_lds(base + 4 * kW * j * kRvqD + loff, dst + 64 * (kW * j + wave) * 16);
    // the chunk's 64 squared norms: every wavefront brings them (the same bytes to the same place) rather than one of them
    // behind a branch - the chunk loop stays one straight line of code, which is what lets its instruction order be pinned
    if (j == 0) __builtin_amdgcn_global_load_lds((glb_ptr_t)(cn + (int64_t)t * kRvqChunk + ln), (lds_ptr_t)ndst, 4, 0, 0);
  };

#pragma unroll
  for (int j = 0; j < 16 / kW; ++j) stage_in1(0, j, lane_off, lane, bufs[0], nrms[0]);
  if (tid == 0) rq.n = 0;
  if (tid < kRvqSlots) rq.count[tid] = 0;
#pragma unroll
  for (int j = 0; j < 16 / kW; ++j) stage_in1(total > 1 ? 1 : 0, j, lane_off, lane, bufs[1], nrms[1]);
  // all but the five loads of the second chunk, i.e. the first chunk has landed; then everybody's part of it
  __builtin_amdgcn_s_waitcnt(kW == 4 ? 0x0075 : 0x0073);   // vmcnt(5 or 3) lgkmcnt(0)
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");

  // Running arg-max per vector block, kept per block of four scores (the lane's entries 16 b + 4 (l/16) + 0..3 of block b): the
  // largest block maximum so far, the second largest, the block that holds the largest, and that block's four scores.  Which
  // of the four won, and how close the others of that block came, is looked up once at the end of the stage: ten vector
  // operations per four scores instead of sixteen.
  float best[4], second[4], third[4], sv[4][4], cmax2 = 0.f;
  const float NEG = -__builtin_inff();
#pragma unroll
  for (int rb = 0; rb < 4; ++rb) {
    best[rb] = NEG; second[rb] = NEG; third[rb] = NEG;
#pragma unroll
    for (int e = 0; e < 4; ++e) sv[rb][e] = NEG;
  }
  // A block maximum carries the number of its block in its lowest mantissa bits (nb bits for S / 16 blocks): the three
  // largest block maxima a lane keeps then say where they came from, at one vector operation per block instead of selects
  // for each.  The price is a relative change of the value of at most 2^(nb - 23), which the margin allows for.
  const int nblk = S / 16;
  const int nb = 32 - __builtin_clz((unsigned)(nblk - 1));      // S / 16 >= 4 blocks
  const unsigned idmask = (1u << nb) - 1u, nidmask = ~idmask;
  const float gamma2 = kRvqGamma2 + __builtin_ldexpf(1.f, nb - 22);   // twice (the rounding bound + the block number's bits)

  // scores of the last block of a chunk: folded into the running best under the first MFMAs of the next chunk (at the
  // start of a stage they are a finite stand-in for -inf, below every score, which the first real block replaces; -inf
  // itself would turn into a NaN when a block number is written into its low bits)
  const float NEGF = -3.0e38f;
  floatx4 tail[4];
#pragma unroll
  for (int rb = 0; rb < 4; ++rb)
#pragma unroll
    for (int e = 0; e < 4; ++e) tail[rb][e] = NEGF;

  int t = 0, stg = 0;
  for (int stage = 0; stage < N; ++stage) {
   for (int ch = 0; ch < nch; ++ch, ++t) {
    // chunk t sits in stage t % 3 (= stg) and chunk t + 2 goes to stage (t + 2) % 3, which chunk t - 1 was the last to read
    const int stg2 = stg == 0 ? 2 : stg - 1;
    const unsigned cur_a = (unsigned)(uintptr_t)(lds_ptr_t)&bufs[0][0] + (unsigned)stg * (kRvqChunk * 256);     // LDS byte addresses
    const unsigned ncur_a = (unsigned)(uintptr_t)(lds_ptr_t)&nrms[0][0] + (unsigned)stg * (kRvqChunk * 4);
    unsigned char* nxt = bufs[stg2];
    float* nnxt = nrms[stg2];
    const int tn = t + 2 < total ? t + 2 : total - 1;   // past the end: a harmless re-load of the last chunk (no branch in the chunk body)

    // One block = 16 entries against the wavefront's 64 vectors: 16 MFMAs (4 k-steps x 4 vector blocks).  Accumulator
    // element e of acc[rb] is the score of entry 16 c + 4 (l/16) + e against vector 16 rb + l%16.
    // The four blocks of a chunk are software-pipelined by hand, one region per block (the scheduler may not move
    // instructions across a region border, which also keeps it from hoisting every read of the chunk to the top and running
    // out of registers): region c holds the fragment and norm reads of block c+1, one load of the chunk after next, the 16
    // MFMAs of block c and the bookkeeping of block c-1 (region 0: of the previous chunk's last block), and inside a region
    // the order is pinned to one MFMA, two or three vector operations, one MFMA, ...
    floatx4 acc[2][4];
    u32x4_t fa[2][4], nqr[2];
    // LDS offsets of the lane's fragment pieces, derived from the lane number inside the loop (a handful of operations per
    // chunk): kept across the loop they would be a dozen loop-invariant registers, which the register allocator spills
    int lq = lane;
    asm volatile("" : "+v"(lq));
    const int le16 = lq & 15, lkq = lq >> 4;
    const int frag0 = le16 * 256 + ((lkq ^ le16) << 4);          // k-step ks: frag0 ^ (ks << 6) (bits 6-7 hold (l%16)/4 ^ ks)
    const unsigned loff = (unsigned)((4 * wave + lkq) * kRvqD + 8 * (le16 ^ ((4 * wave + lkq) & 15)));   // = lane_off
    // read j (of five) of block c: four fragment pieces and the lane's four squared norms (raw: not to be used before lds_wait)
    unsigned fbase[4];                                           // this chunk's addresses of the lane's four pieces of block 0, and of its norms
#pragma unroll
    for (int j = 0; j < 4; ++j) fbase[j] = cur_a + (unsigned)(frag0 ^ (j << 6));
    const unsigned nbase = ncur_a + (unsigned)lkq * 16u;
    auto read1 = [&](int c, int j, u32x4_t (&f)[4], u32x4_t& nq) __attribute__((always_inline)) {
      if (j == 4) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(nq) : "v"(nbase), "n"(c * 64));
      else asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f[j]) : "v"(fbase[j]), "n"(c * 4096));
    };
    // ... and wait for them (everything this wavefront has asked of LDS): the registers go through the statement, so that no use moves above it
    auto lds_wait = [&](u32x4_t (&f)[4], u32x4_t& nq) __attribute__((always_inline)) {
      asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]), "+v"(nq));
    };
    // the four scores v of one block folded into the running state of vector block rb, in four parts u (one per MFMA step).
    // (Which of two equal maxima is kept does not matter: equal scores are always settled exactly.)
    float m4 = 0.f;
    bool gt = false;
    auto fold = [&](int rb, int u, const floatx4& v, int blk) __attribute__((always_inline)) {
#ifndef RVQ_PROBE_NO_UPDATE
      if (u == 0) {
        float m3, mx;
        asm("v_max3_f32 %0, %1, %2, %3" : "=v"(m3) : "v"(v[0]), "v"(v[1]), "v"(v[2]));
        asm("v_max_f32 %0, %1, %2" : "=v"(mx) : "v"(m3), "v"(v[3]));     // (written out: fmaxf would canonicalise both inputs first)
        m4 = __uint_as_float((__float_as_uint(mx) & nidmask) | (unsigned)blk);   // the block's number into the low bits
        gt = m4 > best[rb];
      } else if (u == 1) {
        sv[rb][0] = gt ? v[0] : sv[rb][0];
        sv[rb][1] = gt ? v[1] : sv[rb][1];
      } else if (u == 2) {
        sv[rb][2] = gt ? v[2] : sv[rb][2];
        sv[rb][3] = gt ? v[3] : sv[rb][3];
        third[rb] = __builtin_amdgcn_fmed3f(second[rb], third[rb], m4);   // (before the second largest moves)
      } else {
        second[rb] = __builtin_amdgcn_fmed3f(best[rb], second[rb], m4);
        asm("v_max_f32 %0, %0, %1" : "+v"(best[rb]) : "v"(m4));
      }
#else
      if (u == 0) asm("v_max_f32 %0, %0, %1" : "+v"(best[rb]) : "v"(v[0]));
#endif
    };
#pragma unroll
    for (int j = 0; j < 5; ++j) read1(0, j, fa[0], nqr[0]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      lds_wait(fa[c & 1], nqr[c & 1]);
      floatx4 h;
      {
        const floatx4 q = __builtin_bit_cast(floatx4, nqr[c & 1]);
#pragma unroll
        for (int e = 0; e < 4; ++e) h[e] = -0.5f * q[e];
        asm("v_max3_f32 %0, %0, %1, %2" : "+v"(cmax2) : "v"(q[0]), "v"(q[1]));
        asm("v_max3_f32 %0, %0, %1, %2" : "+v"(cmax2) : "v"(q[2]), "v"(q[3]));
      }
      int blkv = (ch * 4 + c - 1) & (int)idmask;     // the block whose scores this region folds in, in a register of its own
      asm volatile("" : "+v"(blkv));
      __builtin_amdgcn_sched_barrier(0);
      // 16 steps, each fenced off so that the order written is the order issued: one MFMA of block c (k-step i / 4, vector
      // block i % 4), a part of folding the previous block's scores into the running state (two or three vector operations),
      // and in the early steps one of the reads of block c + 1 or this region's load of the chunk after next
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int ks = i >> 2, rb = i & 3;
#ifdef RVQ_PROBE_NO_MFMA
        acc[c & 1][rb] = h;
#else
        acc[c & 1][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, fa[c & 1][ks]), __builtin_bit_cast(bf16x8, ra[rb][ks]),
                                                              ks == 0 ? h : acc[c & 1][rb], 0, 0, 0);
#endif
#ifndef RVQ_PROBE_NO_LDSREAD
        if (c < 3 && i < 5) read1(c + 1, i, fa[(c + 1) & 1], nqr[(c + 1) & 1]);
#endif
#ifndef RVQ_PROBE_NO_DMA
        if (i == 6 && (kW == 4 || (c & 1) == 0)) stage_in1(tn, kW == 4 ? c : c >> 1, loff, (unsigned)lq, nxt, nnxt);
#endif
        // part i % 4 of folding in the previous block's scores for vector block i / 4 (region 0: the previous chunk's last block)
        fold(i >> 2, i & 3, c == 0 ? tail[i >> 2] : acc[(c - 1) & 1][i >> 2], blkv);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
#pragma unroll
    for (int rb = 0; rb < 4; ++rb) tail[rb] = acc[1][rb];
    stg = stg == 2 ? 0 : stg + 1;
    // End of a chunk: all but this chunk's own five loads have landed (the next chunk is complete once everybody is here) and
    // the wavefront's fragment reads are done (the stage may be overwritten).  Written out instead of __syncthreads(), whose
    // fence would wait for the loads of the chunk after next as well; nothing but LDS is shared here.
    __builtin_amdgcn_s_waitcnt(kW == 4 ? 0x0075 : 0x0073);   // vmcnt(5 or 3) lgkmcnt(0)
#ifndef RVQ_PROBE_NO_SYNC
    __builtin_amdgcn_s_barrier();
#endif
    asm volatile("" ::: "memory");                // (the compiler keeps LDS accesses on their side of the barrier)
   }
    {
      // ---- end of a stage: the last block's scores, then merge the four lanes that share a vector (their entries differ
      // by 4 (l/16))
#pragma unroll
      for (int rb = 0; rb < 4; ++rb) {
        const floatx4 v = tail[rb];
        float m3;
        asm("v_max3_f32 %0, %1, %2, %3" : "=v"(m3) : "v"(v[0]), "v"(v[1]), "v"(v[2]));
        const float m4 = __uint_as_float((__float_as_uint(fmaxf(m3, v[3])) & nidmask) | (unsigned)(nch * 4 - 1));
        const bool gt = m4 > best[rb];
#pragma unroll
        for (int e = 0; e < 4; ++e) { sv[rb][e] = gt ? v[e] : sv[rb][e]; tail[rb][e] = NEGF; }
        third[rb] = __builtin_amdgcn_fmed3f(second[rb], third[rb], m4);
        second[rb] = __builtin_amdgcn_fmed3f(best[rb], second[rb], m4);
        best[rb] = fmaxf(best[rb], m4);
      }
      // the blocks of the largest and the second-largest block maximum (their low bits), and which of the kept block's four
      // scores is the maximum (the first, if several)
      int bidx[4], bblk[4], sblk[4];
#pragma unroll
      for (int rb = 0; rb < 4; ++rb) {
        bblk[rb] = (int)(__float_as_uint(best[rb]) & idmask);
        sblk[rb] = (int)(__float_as_uint(second[rb]) & idmask);
        if (bblk[rb] >= nblk) bblk[rb] = 0;               // (only if no score of the stage was a number)
        if (sblk[rb] >= nblk) sblk[rb] = 0;
        const float m = fmaxf(fmaxf(sv[rb][0], sv[rb][1]), fmaxf(sv[rb][2], sv[rb][3]));
        const int e = sv[rb][0] == m ? 0 : sv[rb][1] == m ? 1 : sv[rb][2] == m ? 2 : 3;
        bidx[rb] = 16 * bblk[rb] + e;
      }
      const float cm = rvq_max4(cmax2);
      const bf16_t* stage_cb = cb + (int64_t)stage * S * kRvqD;
      // The winner is certain when its lead over every other score exceeds what rounding (and the block number in the low
      // bits) can have done to two scores.  What comes within that margin is looked at exactly.  The scores of a lane's kept
      // block have known entries (bits 0-3 of near[rb]: one per score of the block).  A second-largest block maximum that
      // close (bit 4) puts the four entries of its block in play, whichever of them it was.  If these are all there is, the
      // wavefront settles the vector among them by itself.  A lane whose third-largest block maximum comes that close stands
      // for entries nobody can name: then the whole workgroup looks at the stage again.
      int z[4], near[4];
      bool amb_known[4], amb_any[4];
      float margin[4], bestm[4];
#pragma unroll
      for (int rb = 0; rb < 4; ++rb) {
        float b = best[rb];
        int bi = bidx[rb] + 4 * kq;
        {
          unsigned ba, bb, ia, ib;
          rvq_pair<16>(__float_as_uint(b), ba, bb); rvq_pair<16>((unsigned)bi, ia, ib);
          bool tb = __uint_as_float(bb) > __uint_as_float(ba) || (__uint_as_float(bb) == __uint_as_float(ba) && (int)ib < (int)ia);
          b = __uint_as_float(tb ? bb : ba); bi = (int)(tb ? ib : ia);
          rvq_pair<32>(__float_as_uint(b), ba, bb); rvq_pair<32>((unsigned)bi, ia, ib);
          tb = __uint_as_float(bb) > __uint_as_float(ba) || (__uint_as_float(bb) == __uint_as_float(ba) && (int)ib < (int)ia);
          b = __uint_as_float(tb ? bb : ba); bi = (int)(tb ? ib : ia);
        }
        z[rb] = bi;
        bestm[rb] = b;
        margin[rb] = gamma2 * (sqrtf(rn2[rb] * 1.02f * cm) + 0.5f * cm);   // (1.02: rn2 is known to one part in 2^7)
        int nr = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) nr |= (!(b - sv[rb][q] > margin[rb]) ? 1 : 0) << q;
        if (!(b - second[rb] > margin[rb])) nr |= 16;
        near[rb] = nr;
        int cnt = __builtin_popcount(nr & 15) + (nr & 16), unk = !(b - third[rb] > margin[rb]) ? 1 : 0;
        {                                                  // both at once: the count in the low half, the flag above it
          unsigned a2, b2;
          unsigned cu = (unsigned)cnt | ((unsigned)unk << 16);
          rvq_pair<16>(cu, a2, b2); cu = a2 + b2;
          rvq_pair<32>(cu, a2, b2); cu = a2 + b2;
          cnt = (int)(cu & 0xffffu); unk = (int)(cu >> 16);
        }
        amb_any[rb] = unk != 0;
        amb_known[rb] = unk == 0 && cnt != 1;
#ifdef RVQ_MEASURE_WITHOUT_EXACT_PATH                       // timing probes only: never defined in the library build
        amb_any[rb] = false; amb_known[rb] = false;
#endif
      }
      unsigned long long todo = 0, mine = 0;
#pragma unroll
      for (int rb = 0; rb < 4; ++rb) {                     // (the four lanes of a vector agree: bit 16 rb + l%16 comes from the lanes with l/16 = 0)
        todo |= (__ballot(amb_any[rb]) & 0xffffull) << (16 * rb);
        mine |= (__ballot(amb_known[rb]) & 0xffffull) << (16 * rb);
      }
      if (stats && lane == 0 && (todo | mine)) atomicAdd(stats, __builtin_popcountll(todo) + __builtin_popcountll(mine));
      // ---- vectors settled by their wavefront: the exact distance to each of the known near entries, the smallest wins
      while (mine) {
        const int bit = __builtin_ctzll(mine);
        mine &= mine - 1;
        const int rbs = bit >> 4, ev = bit & 15;
#pragma unroll
        for (int rb = 0; rb < 4; ++rb)
          if (rb == rbs && e16 == ev) {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) wvec[wave][ks * 4 + kq] = ra[rb][ks];
          }
        // its candidates: per lane group eight possible ones (the four scores of the best block, the four entries of the
        // second block), as one bit each, and the two block numbers
        unsigned cand = 0;
        int b1[4], b2[4];
#pragma unroll
        for (int kq2 = 0; kq2 < 4; ++kq2) {
          int m = 0;
#pragma unroll
          for (int rb = 0; rb < 4; ++rb) {                   // near bits, best block and second block of lane group kq2, in one word
            const int mm = __shfl(near[rb] | (bblk[rb] << 5) | (sblk[rb] << 18), ev + 16 * kq2);
            if (rb == rbs) m = mm;
          }
          m = __builtin_amdgcn_readfirstlane(m);
          b1[kq2] = (m >> 5) & 0x1fff; b2[kq2] = (m >> 18) & 0x1fff;
          cand |= (unsigned)((m & 15) | ((m & 16) ? 0xf0 : 0)) << (8 * kq2);
        }
        double dmin = __builtin_inf();
        int imin = 0x7fffffff;
        while (cand) {                                       // four at a time, one per group of 16 lanes
          int ce[4];
#pragma unroll
          for (int gq = 0; gq < 4; ++gq) {
            ce[gq] = -1;
            if (cand) {
              const int c = __builtin_ctz(cand);
              cand &= cand - 1;
              const int kq2 = c >> 3, q = c & 7;
              const int blk = q < 4 ? (kq2 == 0 ? b1[0] : kq2 == 1 ? b1[1] : kq2 == 2 ? b1[2] : b1[3])
                                    : (kq2 == 0 ? b2[0] : kq2 == 1 ? b2[1] : kq2 == 2 ? b2[2] : b2[3]);
              const int ent = 16 * blk + 4 * kq2 + (q & 3);
              ce[gq] = (unsigned)ent < (unsigned)S ? ent : -1;   // (always inside: block numbers come from the chunk loop)
            }
          }
          const int mine_c = kq == 0 ? ce[0] : kq == 1 ? ce[1] : kq == 2 ? ce[2] : ce[3];
          const double d = rvq_exact_distance16(&wvec[wave][0], stage_cb, mine_c, e16);
#pragma unroll
          for (int gq = 0; gq < 4; ++gq) {
            const double dg = __shfl(d, 16 * gq);
            if (ce[gq] >= 0 && (dg < dmin || (dg == dmin && ce[gq] < imin))) { dmin = dg; imin = ce[gq]; }
          }
        }
        if ((unsigned)imin < (unsigned)S) {
#pragma unroll
          for (int rb = 0; rb < 4; ++rb)
            if (rb == rbs && e16 == ev) z[rb] = imin;
        }
      }
      // ---- the others: exact re-evaluation by the whole workgroup, kRvqSlots vectors per round
      const float* stage_cn = cn + (int64_t)stage * S;
      // (rq.n and rq.count are zero on entry: cleared at the start of the kernel and at the end of every round that used them,
      // with a workgroup barrier between that and the next claim; the usual stage, with nothing to resolve, costs one barrier)
      for (;;) {
        // claim slots, lowest vector first; a vector that gets none this round keeps its bit
        unsigned long long rest = todo;
        while (rest) {
          const int bit = __builtin_ctzll(rest);
          rest &= rest - 1;
          int slot = 0;
          if (lane == 0) slot = atomicAdd(&rq.n, 1);
          slot = __shfl(slot, 0);
          if (slot >= kRvqSlots) continue;
          todo &= ~(1ull << bit);
          const int rbs = bit >> 4, e = bit & 15;
#pragma unroll
          for (int rb = 0; rb < 4; ++rb)
            if (rb == rbs && e16 == e) {
#pragma unroll
              for (int ks = 0; ks < 4; ++ks) rq.bits[slot][ks * 4 + kq] = ra[rb][ks];
              if (kq == 0) { rq.margin[slot] = margin[rb]; rq.best[slot] = bestm[rb]; rq.owner[slot] = 64 * wave + bit; }
            }
        }
        __syncthreads();
        const int asked = rq.n;
        if (asked == 0) break;                             // (the same for every wavefront)
        const int nslot = asked < kRvqSlots ? asked : kRvqSlots;
        {
          // 1. + 2.: column l%16 of the B operand is the vector of slot l%16; this wavefront takes a quarter of the entries
          const bool live = e16 < nslot;
          const float mg = live ? rq.margin[e16] : 0.f;
          u32x4_t bq[4];
#pragma unroll
          for (int ks = 0; ks < 4; ++ks) bq[ks] = rq.bits[e16][ks * 4 + kq];      // (stale data in unused slots: never looked at)
          float lmax = live ? rq.best[e16] - mg : NEG;
          const int nblk = S / 16, per = (nblk + kW - 1) / kW;
          const int blk_end = (wave + 1) * per < nblk ? (wave + 1) * per : nblk;
#ifndef RVQ_PROBE_NO_PASS
#pragma unroll 1
          for (int blk0 = wave * per; blk0 < blk_end; blk0 += 4) {
            u32x4_t a[4][4];
            floatx4 h[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              const int blk = blk0 + u < blk_end ? blk0 + u : blk0;         // per may not be a multiple of four: redo a group
              const bf16_t* ent = stage_cb + (int64_t)(blk * 16 + e16) * kRvqD + kq * 8;
#pragma unroll
              for (int ks = 0; ks < 4; ++ks) a[u][ks] = *reinterpret_cast<const u32x4_t*>(ent + ks * 32);
              h[u] = *reinterpret_cast<const floatx4*>(stage_cn + blk * 16 + 4 * kq);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              if (blk0 + u >= blk_end) break;
              floatx4 acc;
#pragma unroll
              for (int e = 0; e < 4; ++e) acc[e] = -0.5f * h[u][e];
#pragma unroll
              for (int ks = 0; ks < 4; ++ks)
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[u][ks]), __builtin_bit_cast(bf16x8, bq[ks]), acc, 0, 0, 0);
#pragma unroll
              for (int e = 0; e < 4; ++e) {                // element e: entry 16 (blk0 + u) + 4 (l/16) + e against the vector of slot l%16
                const float v = acc[e];
                lmax = fmaxf(lmax, v);
                if (live && !(lmax - v > mg)) {
                  const int pos = atomicAdd(&rq.count[e16], 1);
                  if (pos < kRvqCand) { rq.cand[e16][pos] = (blk0 + u) * 16 + 4 * kq + e; rq.cscore[e16][pos] = v; }
                }
              }
            }
          }
#endif
          rq.top[e16][wave * 4 + kq] = lmax;            // (a wavefront without entries writes its floor: the main pass's best minus the margin, or -inf)
        }
        __syncthreads();
        // 3.: wavefront w decides slots w, w + 4, ...
#ifndef RVQ_PROBE_NO_DECIDE
        for (int j = wave; j < nslot; j += kW) {
          float top = rq.top[j][lane & (4 * kW - 1)];
#pragma unroll
          for (int o = 1; o < 4 * kW; o <<= 1) top = fmaxf(top, __shfl_xor(top, o));
          const float mg = rq.margin[j];
          const int listed = rq.count[j];
          double dmin = __builtin_inf();
          int imin = 0x7fffffff;
          if (listed > kRvqCand) {                         // the list overflowed: every entry, one after the other
#pragma unroll 1
            for (int ent = 0; ent < S; ++ent) {
              const double d = rvq_exact_distance(&rq.bits[j][0], stage_cb, ent, lane);
              if (d < dmin) { dmin = d; imin = ent; }
            }
          } else {
#pragma unroll 1
            for (int i = 0; i < listed; ++i) {
              if (top - rq.cscore[j][i] > mg) continue;
              const int ent = rq.cand[j][i];
              const double d = rvq_exact_distance(&rq.bits[j][0], stage_cb, ent, lane);
              if (d < dmin || (d == dmin && ent < imin)) { dmin = d; imin = ent; }
            }
          }
          if (lane == 0) rq.result[j] = imin;
        }
#else
        if (tid < kRvqSlots) rq.result[tid] = 0;
#endif
        __syncthreads();
        for (int j = 0; j < nslot; ++j) {                  // the owners collect their answers
          const int o = rq.owner[j];
          if ((o >> 6) != wave) continue;
          const int rbs = (o >> 4) & 3, e = o & 15, zz = rq.result[j];
          if ((unsigned)zz >= (unsigned)S) continue;       // no survivor (scores that are not numbers): the main pass's index stands
#pragma unroll
          for (int rb = 0; rb < 4; ++rb)
            if (rb == rbs && e16 == e) z[rb] = zz;
        }
        __syncthreads();                                   // everybody has read this round's requests and answers
        if (tid == 0) rq.n = 0;
        if (tid < kRvqSlots) rq.count[tid] = 0;
        if (asked <= kRvqSlots) break;
        __syncthreads();                                   // cleared before the next round's claims
      }
      // ---- codes out, residual update, its squared norm for the next stage's margin
#pragma unroll
      for (int rb = 0; rb < 4; ++rb) {
        const int v = v0 + rb * 16 + e16;
        if (kq == 0 && v < L) codes[(int64_t)v * N + stage] = z[rb];
        float a = 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const u32x4_t cz = *reinterpret_cast<const u32x4_t*>(stage_cb + (int64_t)z[rb] * kRvqD + ks * 32 + kq * 8);
          ra[rb][ks] = rvq_sub_bf16(ra[rb][ks], cz, a);
        }
        rn2[rb] = rvq_sum4(a);
        best[rb] = NEG; second[rb] = NEG; third[rb] = NEG;
#pragma unroll
        for (int e = 0; e < 4; ++e) sv[rb][e] = NEG;
      }
      cmax2 = 0.f;
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);             // vmcnt(0): no load into LDS may be in flight when the workgroup gives its LDS back
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
