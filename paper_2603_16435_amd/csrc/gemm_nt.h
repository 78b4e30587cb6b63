// gemm_nt.h - the one contraction main loop of the library (gfx950 / CDNA4).
//
//   C[m,n] = sum_k A[m,k] * B[n,k]        A: [M,K] row-major, B: [N,K] row-major ("NT")
//
// Every contraction of the path is brought into this form (K contiguous in both operands)
// so that one MFMA main loop serves the forward logits, the recomputed logits, dX and dW;
// what differs is the epilogue functor that consumes the accumulators in registers.
//
// Tiling: a workgroup of WAVES_M x WAVES_N wavefronts (64 lanes each) owns a BM x BN tile of
// C and walks K in slabs of 128 bytes per row (64 bf16 or 32 f32).  Slabs are staged in LDS
// (double-buffered; global loads for slab k+1 are in flight while slab k feeds the MFMAs).
// LDS rows are 128 B = eight 16-byte chunks; chunk c of row r sits at slot c ^ ((r>>1)&7),
// which spreads both the 16-byte row-wise stores and the column-wise fragment loads over all
// 64 banks.  MFMA shape is 32x32 (x16 for bf16, x2 for f32); both have the same accumulator
// layout: lane l, register i hold  row = 8*(i/4) + 4*(l/32) + i%4,  col = l%32.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rlk {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kSlabBytes = 128;   // bytes of K per LDS row
constexpr int kXcds = 8;          // MI355X: 8 accelerator dies, workgroups dealt round-robin

template <class T> struct Elem;
template <> struct Elem<bf16_t> { static constexpr int kPerChunk = 8; static constexpr int kBK = 64; };
template <> struct Elem<float>  { static constexpr int kPerChunk = 4; static constexpr int kBK = 32; };

struct GemmDims {
  int M, N, K;            // upper bounds (static); the dynamic extent trims one of them
  int64_t lda, ldb;       // row strides in elements
  const int* a_rows;      // optional gather: logical row m of A lives at row a_rows[m]
  const int* b_rows;
  const int* n_real;      // device scalar: number of compacted rows in the whole batch
  int chunk_start;        // first compacted row of this chunk
  int dyn;                // which extent is min(max(*n_real - chunk_start,0), bound): 0 none, 1 M, 2 N, 3 K (rounded up to 256)
  int group_m;            // tile-order parameter: M-tiles per band
};

// Workgroup -> tile.  Workgroups are dealt to the 8 XCDs round-robin, and each XCD has its own
// L2, so ids are first regrouped such that one XCD receives a contiguous run of tile numbers;
// runs are then laid out in bands of group_m M-tiles by all N-tiles, N fastest inside a band
// column, so the workgroups resident on one XCD share A and B panels through its L2.
__device__ inline void tile_of_block(int pid, int tiles_m, int tiles_n, int group_m, int& tm, int& tn) {
  const int total = tiles_m * tiles_n;
  const int per = total / kXcds, rem = total % kXcds;
  const int xcd = pid % kXcds, q = pid / kXcds;
  const int t = xcd * per + (xcd < rem ? xcd : rem) + q;
  const int band = group_m * tiles_n;
  const int g = t / band;
  const int first_m = g * group_m;
  const int gsz = (tiles_m - first_m < group_m) ? (tiles_m - first_m) : group_m;
  const int r = t - g * band;
  tm = first_m + r % gsz;
  tn = r / gsz;
}

__device__ inline int lds_off(int row, int chunk) {           // byte offset inside one operand slab
  return row * kSlabBytes + ((chunk ^ ((row >> 1) & 7)) << 4);
}

template <class T>
__device__ inline void mma_step(const uint4& a, const uint4& b, floatx16& acc);

template <>
__device__ inline void mma_step<bf16_t>(const uint4& a, const uint4& b, floatx16& acc) {
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
}
template <>
__device__ inline void mma_step<float>(const uint4& a, const uint4& b, floatx16& acc) {
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a.x), __builtin_bit_cast(float, b.x), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a.y), __builtin_bit_cast(float, b.y), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a.z), __builtin_bit_cast(float, b.z), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a.w), __builtin_bit_cast(float, b.w), acc, 0, 0, 0);
}

// Coordinates handed to an epilogue: everything it needs to map acc[bi][bj][i] to (m,n).
struct TileCtx {
  int m0, n0;        // first row / col of this wavefront's sub-tile
  int Mv, Nv;        // valid extents (after dynamic trimming)
  int lane, wm, wn;  // lane id, wavefront coordinates inside the workgroup
  int tile_m, tile_n;// workgroup tile indices
  int tid;
};
template <int> struct Int {};

template <class T, class Epi, int BM, int BN, int WAVES_M, int WAVES_N>
__global__ __launch_bounds__(WAVES_M * WAVES_N * 64)
void gemm_nt_kernel(const T* __restrict__ A, const T* __restrict__ B, GemmDims d, Epi epi) {
  constexpr int NT = WAVES_M * WAVES_N * 64;
  constexpr int BK = Elem<T>::kBK;
  constexpr int EPC = Elem<T>::kPerChunk;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int MB = WM / 32, NB = WN / 32;
  constexpr int ROWS_PER_PASS = NT / 8;
  constexpr int PA = BM / ROWS_PER_PASS, PB = BN / ROWS_PER_PASS;
  static_assert(BM % ROWS_PER_PASS == 0 && BN % ROWS_PER_PASS == 0, "tile vs threads");
  constexpr int A_BYTES = BM * kSlabBytes, B_BYTES = BN * kSlabBytes;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  int M = d.M, N = d.N, K = d.K;
  if (d.dyn) {
    const int left = *d.n_real - d.chunk_start;
    if (left <= 0) {
      // nothing left for this chunk; the very first K-trimmed launch still has to produce zeros
      if (d.dyn == 3 && d.chunk_start == 0) K = 0; else return;
    } else if (d.dyn == 1) M = left < M ? left : M;
    else if (d.dyn == 2) N = left < N ? left : N;
    else { const int k = (left + 255) & ~255; K = k < K ? k : K; }
  }
  const int tiles_m = (d.M + BM - 1) / BM, tiles_n = (d.N + BN - 1) / BN;
  int tm, tn;
  tile_of_block(blockIdx.x, tiles_m, tiles_n, d.group_m, tm, tn);
  if (tm * BM >= M || tn * BN >= N) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;

  // ---- global -> register staging: thread owns chunk (tid&7) of rows (tid>>3) + p*ROWS_PER_PASS
  const int lchunk = tid & 7, lrow = tid >> 3;
  const T* ap[PA];
  const T* bp[PB];
#pragma unroll
  for (int p = 0; p < PA; ++p) {
    int r = tm * BM + lrow + p * ROWS_PER_PASS;
    r = r < M ? r : M - 1;
    if (d.a_rows) r = d.a_rows[r];
    ap[p] = A + (int64_t)r * d.lda + lchunk * EPC;
  }
#pragma unroll
  for (int p = 0; p < PB; ++p) {
    int r = tn * BN + lrow + p * ROWS_PER_PASS;
    r = r < N ? r : N - 1;
    if (d.b_rows) r = d.b_rows[r];
    bp[p] = B + (int64_t)r * d.ldb + lchunk * EPC;
  }
  uint4 ra[PA], rb[PB];
  auto gload = [&](int k0) {
    const bool ok = (k0 + lchunk * EPC) < K;
#pragma unroll
    for (int p = 0; p < PA; ++p) ra[p] = ok ? *reinterpret_cast<const uint4*>(ap[p] + k0) : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int p = 0; p < PB; ++p) rb[p] = ok ? *reinterpret_cast<const uint4*>(bp[p] + k0) : make_uint4(0, 0, 0, 0);
  };
  auto lstore = [&](int buf) {
    unsigned char* as = smem + buf * (A_BYTES + B_BYTES);
    unsigned char* bs = as + A_BYTES;
#pragma unroll
    for (int p = 0; p < PA; ++p) *reinterpret_cast<uint4*>(as + lds_off(lrow + p * ROWS_PER_PASS, lchunk)) = ra[p];
#pragma unroll
    for (int p = 0; p < PB; ++p) *reinterpret_cast<uint4*>(bs + lds_off(lrow + p * ROWS_PER_PASS, lchunk)) = rb[p];
  };

  floatx16 acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int nk = (K + BK - 1) / BK;
  gload(0);
  lstore(0);
  __syncthreads();
  const int frow = lane & 31, fhalf = lane >> 5;
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) gload((kt + 1) * BK);
    const unsigned char* as = smem + cur * (A_BYTES + B_BYTES);
    const unsigned char* bs = as + A_BYTES;
#pragma unroll
    for (int s = 0; s < 4; ++s) {                  // four 32-byte k-steps per slab
      uint4 af[MB], bf[NB];
#pragma unroll
      for (int i = 0; i < MB; ++i) af[i] = *reinterpret_cast<const uint4*>(as + lds_off(wm * WM + i * 32 + frow, s * 2 + fhalf));
#pragma unroll
      for (int j = 0; j < NB; ++j) bf[j] = *reinterpret_cast<const uint4*>(bs + lds_off(wn * WN + j * 32 + frow, s * 2 + fhalf));
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) mma_step<T>(af[i], bf[j], acc[i][j]);
    }
    if (kt + 1 < nk) lstore(cur ^ 1);
    __syncthreads();
  }

  TileCtx c;
  c.m0 = tm * BM + wm * WM; c.n0 = tn * BN + wn * WN;
  c.Mv = M; c.Nv = N; c.lane = lane; c.wm = wm; c.wn = wn; c.tile_m = tm; c.tile_n = tn; c.tid = tid;
  epi.template run<MB, NB, BM, BN, WAVES_M, WAVES_N>(acc, c, smem, d);
}

// accumulator coordinates inside a wavefront sub-tile
__device__ inline int acc_row(int bi, int i, int lane) { return bi * 32 + ((i >> 2) << 3) + ((lane >> 5) << 2) + (i & 3); }
__device__ inline int acc_col(int bj, int lane) { return bj * 32 + (lane & 31); }

}  // namespace rlk
