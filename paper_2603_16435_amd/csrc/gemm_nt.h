// gemm_nt.h - the contraction main loops of the library (gfx950 / CDNA4).
//
//   C[m,n] = sum_k A[m,k] * B[n,k]        A: [M,K] row-major, B: [N,K] row-major ("NT")
//
// Every contraction of the path is brought into this form (K contiguous in both operands)
// so that one MFMA main loop serves the forward logits, the recomputed logits, dX and dW;
// what differs is the epilogue functor that consumes the accumulators in registers.  One
// exception: the hot kernel can also take its A operand K-major (the stored array is A^T, rows = k),
// read through transposing LDS loads; dW uses that to contract dS^T X out of dS itself.
//
// Two kernels share tile order, LDS layout and epilogues:
//  * gemm_nt_bf16_kernel  - the hot one (bf16, K % 128 == 0).  256x256 tile, four wavefronts of
//    128x128 each (256 accumulator registers per lane live in AGPRs, one wavefront per SIMD),
//    K walked in slabs of 64, MFMA shape 16x16x32 (measured on this part: at the power limit it
//    sustains about 15 % more flops than 32x32x16 on random data).  Slabs go from global memory
//    straight into LDS (global_load ... lds, 16 bytes per lane) into two static 64 KiB stages.  A
//    slab is four phases of 32 MFMAs; its loads are spread over three phases so that no burst
//    blocks the MFMA issue, the fragments of a phase are read from LDS during the phase before,
//    and the last phase of a slab runs after the workgroup barrier so that it hides the first
//    fragment reads of the next slab.  The MFMAs are inline asm and every one is fenced with
//    sched_barrier, so the interleaving in the source is the interleaving issued.  A light
//    software prefetch (one 4-byte load per 128-byte line, two slabs ahead, shared between the
//    workgroups of an XCD; off for dX) pulls the next panels into that XCD's L2.
//  * gemm_nt_kernel       - generic fallback (f32 inputs, or K not a multiple of 128): eight
//    wavefronts of 128x64, 32x32 MFMA blocks, register-staged loads with a K-tail predicate.
//
// LDS rows are 128 B = eight 16-byte chunks; chunk c of row r sits at slot c ^ ((r>>1)&7),
// which spreads both the 16-byte row-wise stores and the column-wise fragment loads over all
// 64 banks (measured: zero bank conflicts).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rlk {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

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
  const int* chunk;       // if set, device pair {first compacted row, rows} of this chunk; replaces n_real / chunk_start,
                          // and the gather tables are then indexed from the chunk's first row
  int a_tiled, b_tiled;   // hot kernel only: operand stored slab-tiled (see tiled_index) instead of row-major; K is then its full K extent
  int dyn;                // which extent is min(rows left in the chunk, bound): 0 none, 1 M, 2 N, 3 K (rounded up to 256)
  int zero_if_empty;      // dyn == 3 only: an empty chunk still runs the epilogue (with K = 0) instead of returning
  int group_m;            // tile-order parameter: M-tiles per band
};

// Slab-tiled operand layout of the library's own bf16 work buffers: [row / 256][k / 64][256 rows][64 k].
// The 32 KiB that a workgroup loads per operand and slab are then contiguous in memory (one page, one DRAM
// row run) instead of 256 pieces of 128 bytes a whole matrix row apart; K is the buffer's full K extent.
__device__ __host__ inline int64_t tiled_index(int r, int k, int64_t K) {
  return (int64_t)(r >> 8) * (K * 256) + (int64_t)(k >> 6) * 16384 + ((r & 255) << 6) + (k & 63);
}
__device__ __host__ inline int64_t operand_index(bool tiled, int r, int k, int64_t ld) {
  return tiled ? tiled_index(r, k, ld) : (int64_t)r * ld + k;
}

// Apply the dynamic extent.  Returns false if this launch has nothing to do.
__device__ inline bool resolve_dims(GemmDims& d, int& M, int& N, int& K) {
  M = d.M; N = d.N; K = d.K;
  if (!d.dyn) return true;
  int left;
  if (d.chunk) {
    const int cs = d.chunk[0];
    left = d.chunk[1];
    d.chunk_start = cs;
    if (d.a_rows) d.a_rows += cs;
    if (d.b_rows) d.b_rows += cs;
  } else {
    left = *d.n_real - d.chunk_start;
  }
  if (left <= 0) {
    if (d.dyn == 3 && d.zero_if_empty) K = 0; else return false;
  } else if (d.dyn == 1) M = left < M ? left : M;
  else if (d.dyn == 2) N = left < N ? left : N;
  else { const int k = (left + 255) & ~255; K = k < K ? k : K; }
  return true;
}

// Workgroup -> tile.  Workgroups are dealt to the 8 XCDs round-robin (workgroup id % 8), and each XCD has
// its own L2.  Tiles are walked in bands of group_m M-tiles by all N-tiles, M fastest inside a band column,
// so that the workgroups resident on one XCD at a time (about group_m M-tiles by 32 / group_m N-tiles)
// share their A and B panels through its L2.  Two ways of giving each XCD its part of that sequence:
//
//  * runs (by_share = false): the sequence is cut into eight equal runs.  The XCDs are then at unrelated
//    N positions, which spreads their B-panel reads over the memory channels.  Best where the B panels
//    are short or few enough to live in the memory-side cache (logits: K = H; dW: B = X^T chunk).
//  * shares (by_share = true): an XCD owns a contiguous share of the M-tiles that exist (after dynamic
//    trimming; shares differ by at most one tile) and all XCDs are at the same N-tiles at the same
//    time, so a B panel comes out of memory once and reaches the other XCDs through the memory-side
//    cache.  Needed for dX, where both operands stream from memory over a very long K (B = W^T, a
//    1 GB panel set per sweep): equal runs there are 7 % slower unless they happen to start on band
//    boundaries, and with shares a partly filled chunk is spread over all XCDs instead of the first few.
//
// The launch has launch_tiles() workgroups of the static bounds; the ones without a tile get false.
__device__ __host__ inline int launch_tiles(int tiles_m, int tiles_n) {
  return (tiles_m + kXcds - 1) / kXcds * kXcds * tiles_n;
}
__device__ __host__ inline bool tile_of_block(int pid, int tiles_m, int tiles_n, int group_m, bool by_share, int& tm, int& tn) {
  const int xcd = pid % kXcds, q = pid / kXcds;
  int t, first = 0, rows = tiles_m;                // position in the band sequence of `rows` M-tiles starting at `first`
  if (by_share) {
    const int base = tiles_m / kXcds, rem = tiles_m % kXcds;
    rows = base + (xcd < rem ? 1 : 0);
    first = xcd * base + (xcd < rem ? xcd : rem);
    if (q >= rows * tiles_n) return false;
    t = q;
  } else {
    const int total = tiles_m * tiles_n;
    if (pid >= total) return false;
    const int per = total / kXcds, rem = total % kXcds;
    t = xcd * per + (xcd < rem ? xcd : rem) + q;
  }
  const int band = group_m * tiles_n;
  const int g = t / band;
  const int first_m = g * group_m;
  const int gsz = (rows - first_m < group_m) ? (rows - first_m) : group_m;
  const int r = t - g * band;
  tm = first + first_m + r % gsz;
  tn = r / gsz;
  return true;
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
struct NoPre {};      // epilogue with nothing to fetch ahead of the main loop

// Accumulator layouts: where register i of block (bi, bj) of a lane sits inside the wavefront's
// sub-tile.  Registers come in runs of four consecutive rows of one column.
struct Layout32 {   // 32x32 MFMA blocks, 16 registers per block: row = 8*(i/4) + 4*(l/32) + i%4, col = l%32
  typedef floatx16 acc_t;
  static constexpr int kBlk = 32, kRegs = 16;
  __device__ static int row(int bi, int i, int lane) { return bi * 32 + ((i >> 2) << 3) + ((lane >> 5) << 2) + (i & 3); }
  __device__ static int col(int bj, int lane) { return bj * 32 + (lane & 31); }
  __device__ static bool owns(int r, int lane) { return ((r >> 2) & 1) == (lane >> 5); }   // does this lane hold row r of its columns?
};
struct Layout16 {   // 16x16 MFMA blocks, 4 registers per block: row = 4*(l/16) + i, col = l%16
  typedef floatx4 acc_t;
  static constexpr int kBlk = 16, kRegs = 4;
  __device__ static int row(int bi, int i, int lane) { return bi * 16 + ((lane >> 4) << 2) + i; }
  __device__ static int col(int bj, int lane) { return bj * 16 + (lane & 15); }
  __device__ static bool owns(int r, int lane) { return ((r >> 2) & 3) == (lane >> 4); }
};

// Reading one accumulator element in an epilogue.  In the hot kernel the 256 accumulators of a lane
// live in AGPRs; left to itself the compiler copies all of them to VGPRs at loop exit and spills
// most of them to scratch (tens of GB of extra HBM traffic per launch).  Reading each element
// through an explicit v_accvgpr_read at its point of use keeps them where they are.
template <bool AGPR, class V>
__device__ inline float acc_read(const V& v, int i) {
  if constexpr (AGPR) {
    float r;
    const float e = v[i];
    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(r) : "a"(e));
    return r;
  } else {
    return v[i];
  }
}

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

  int M, N, K;
  if (!resolve_dims(d, M, N, K)) return;
  // dynamic M (dX): XCD shares of the M-tiles that exist; otherwise equal runs over the static grid
  const bool by_share = d.dyn == 1;
  const int tiles_m = ((by_share ? M : d.M) + BM - 1) / BM, tiles_n = (d.N + BN - 1) / BN;
  int tm, tn;
  if (!tile_of_block(blockIdx.x, tiles_m, tiles_n, d.group_m, by_share, tm, tn)) return;
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
  const typename Epi::Pre pre = epi.template preload<Layout32>(c, d);
  epi.template run<Layout32, MB, NB, BM, BN, WAVES_M, WAVES_N, false>(acc, c, smem, d, pre);
}

// ------------------------------------------------------------------ bf16 hot kernel
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* glb_ptr_t;

// The same load with its address given as a wavefront-uniform base (two scalar registers) plus a 32-bit lane offset in
// bytes: no vector operation goes into the address.  Written as inline assembly because the compiler, given base + offset,
// folds the offset into a per-lane 64-bit pointer outside the loop and adds the slab's stride to it with a vector add per
// load.  It keeps no count of such a load: the waits that cover it are the ones written out in the main loop.
__device__ __attribute__((always_inline)) inline void load16_to_lds_uniform(const void* base, unsigned lane_bytes, void* l) {
  const unsigned lds = (unsigned)(size_t)(lds_ptr_t)l;      // uniform
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" :: "v"(lane_bytes), "s"(base), "s"(lds) : "memory");
}
// ... and with a 64-bit address per lane, for rows that come through a row map.  (Every load of the hot kernel's main loop is
// one of these two, so that the compiler itself never sets M0 there.)
__device__ __attribute__((always_inline)) inline void load16_to_lds_lanes(const void* g, void* l) {
  const unsigned lds = (unsigned)(size_t)(lds_ptr_t)l;      // uniform
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" :: "v"(g), "s"(lds) : "memory");
}

__device__ inline void load16_to_lds(const void* g, void* l) {   // 64 lanes x 16 B -> 1 KiB of LDS at l
  __builtin_amdgcn_global_load_lds((glb_ptr_t)g, (lds_ptr_t)l, 16, 0, 0);
}

// Optional relabelling of the tile's rows and columns in the hot kernel (epilogues with kPermute).
// Which matrix row an LDS row holds is free to choose as long as the epilogue uses the same map.
// Inside each 128-row half of the tile, LDS row 16*b + 4*g + e (block b, lane group g, register e)
// holds matrix row 32*(b/2) + 8*g + 4*(b%2) + e, and LDS column-row 16*b + c holds matrix column
// 8*c + b: a lane (g, c) then owns runs of eight consecutive rows and of eight consecutive columns.
__device__ inline int perm_row(int b, int g, int e) { return ((b >> 1) << 5) + (g << 3) + ((b & 1) << 2) + e; }
__device__ inline int perm_col(int b, int c) { return (c << 3) + b; }
__device__ inline int perm_lds_row_a(int lr) { return (lr & 128) + perm_row((lr >> 4) & 7, (lr >> 2) & 3, lr & 3); }
__device__ inline int perm_lds_row_b(int lr) { return (lr & 128) + perm_col((lr >> 4) & 7, lr & 15); }

// One 16x16x32 bf16 MFMA, accumulator in place.  Written as inline asm so that the 64 accumulator
// blocks of a lane are pinned to the 256 AGPRs for the whole kernel: with the builtin the register
// allocator splits them between the two register files and fills the main loop with copies.  The
// compiler therefore does not know these are MFMAs: the required wait states before the epilogue
// reads the accumulators are inserted by hand (mfma_drain).
__device__ __attribute__((always_inline)) inline void mfma16(floatx4& acc, const u32x4_t& a, const u32x4_t& b) {
  asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
__device__ __attribute__((always_inline)) inline void mfma_drain() { asm volatile("s_nop 15\n\ts_nop 15" ::: "memory"); }

// PFD: L2 prefetch distance in slabs (0 = none).  VMG / VMO: inside a phase of 32 MFMAs the slab loads
// are issued after MFMA number VMO, VMO + VMG, VMO + 2 VMG, ...  LDA / LDB: how many of a slab's 16 loads go
// into the phase after the barrier and into the first phase of the next slab (the rest into its second phase);
// the earlier they go, the longer they have to land before the next barrier.
constexpr int kHotStageBytes = (256 + 256) * kSlabBytes;      // one LDS stage of the hot kernel: a slab of A and of B

// Transposing LDS read (ds_read_b64_tr_b16).  Within each group of 16 lanes, the four 16-bit values that lane
// 4e + j/4 fetched (8 bytes at its own address) are dealt to lanes 4(j/4).. : lane j receives, as element e,
// value j%4 of the piece fetched by lane 4e + j/4.  With lanes 4e..4e+3 pointing at sixteen consecutive m of
// k-row e, lane j ends up with (m = j, k = 0..3): an MFMA operand read out of a K-major slab.
typedef short tr16x4_t __attribute__((ext_vector_type(4)));
typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));
__device__ __attribute__((always_inline)) inline u32x2_t lds_read_tr16(const unsigned char* p) {
  typedef __attribute__((address_space(3))) tr16x4_t* lds_ptr;
  return __builtin_bit_cast(u32x2_t, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p)));
}

// The work of one workgroup of the hot kernel: tile number `pid` of the contraction (A, B, d) into epi.
// stage0 / stage1 are the caller's two LDS stages; they must be separate objects so that the compiler
// can tell the stage being filled by the DMA loads from the stage the fragments are read from and
// does not serialise them with a vmcnt(0).
//
// ATR: the A operand is given K-major, element (m, k) at tiled_index(k, m, d.lda) (the slab-tiled layout of its
// transpose, whose rows are k): C = A^T-stored x B without a transposed copy of A in memory.  Its LDS slab is
// 64 k-rows of 256 m (512 bytes a row, 32-byte pieces XOR-swizzled by a function of the row such that the eight
// rows a half-wavefront's transposing read touches fall into different banks) and its fragments come from two
// transposing reads each.
template <class Epi, int PFD, int VMG, int VMO, bool ATR = false, int LDA = 6, int LDB = 5>
__device__ __attribute__((always_inline)) inline void gemm_nt_bf16_tile(const bf16_t* __restrict__ A, const bf16_t* __restrict__ B, GemmDims d,
                                                                        const Epi& epi, int pid, unsigned char* stage0, unsigned char* stage1) {
  constexpr int BM = 256, BN = 256, BK = 64, WAVES_M = 2, WAVES_N = 2;
  constexpr int WM = 128, WN = 128, MB = 8, NB = 8;             // 8 x 8 blocks of 16 x 16 per wavefront
  constexpr int DSG = 2;                                        // one fragment read per DSG MFMAs
  constexpr int A_BYTES = BM * kSlabBytes, B_BYTES = BN * kSlabBytes, STAGE = A_BYTES + B_BYTES;
  constexpr int LDC = 16 - LDA - LDB;
  constexpr int LDMAX = LDA > LDB ? (LDA > LDC ? LDA : LDC) : (LDB > LDC ? LDB : LDC);
  static_assert(LDA >= 0 && LDB >= 0 && LDC >= 0 && VMO < VMG && (LDMAX - 1) * VMG + VMO < 32,
                "the slab loads of the fullest phase must fit into its 32 MFMAs");
  static_assert(STAGE == kHotStageBytes, "stage size");
  static_assert(!ATR || !Epi::kPermute, "the K-major A path loads rows in natural order");

  int M, N, K;
  if (!resolve_dims(d, M, N, K)) return;
  const int nk = K / BK;
  // dynamic M (dX): XCD shares of the M-tiles that exist; otherwise equal runs over the static grid
  const bool by_share = d.dyn == 1;
  const int tiles_m = ((by_share ? M : d.M) + BM - 1) / BM, tiles_n = (d.N + BN - 1) / BN;
  int tm, tn;
  if (!tile_of_block(pid, tiles_m, tiles_n, d.group_m, by_share, tm, tn)) return;
  if (tm * BM >= M || tn * BN >= N) return;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // uniform: LDS addresses stay scalar
  const int wm = wave >> 1, wn = wave & 1;

  // ---- slab staging.  Wavefront w fills rows [64w, 64w+64) of A and of B: eight loads of eight
  // rows each.  A load writes lane l's 16 bytes to LDS offset 16*l of its 1 KiB target, i.e. row
  // l/8, slot l%8; the swizzle is therefore applied on the global side (which chunk a lane fetches).
  // An operand whose rows are where they are numbered (every one but the hidden states, whose rows come through the row
  // map) is addressed as a wavefront-uniform base plus a 32-bit lane offset: the address of a load is then a scalar add per
  // slab and no vector operation (vector operations and MFMAs take turns on a SIMD).  All rows of a tile lie within
  // 256 rows of the tile's first, so the offsets fit.
  constexpr bool GB = Epi::kGatherB;
  const bf16_t* ap[8];
  const bf16_t* bp[8];
  unsigned aoff[8], boff[8];
  const bf16_t* const abase = ATR ? A + tiled_index(0, tm * BM, d.lda)
                                  : A + (d.a_tiled ? tiled_index(tm * BM, 0, d.K) : (int64_t)(tm * BM) * d.lda);
  const bf16_t* const bbase = B + (d.b_tiled ? tiled_index(tn * BN, 0, d.K) : (int64_t)(tn * BN) * d.ldb);
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int lr = wave * 64 + j * 8 + (lane >> 3);
    const int c = (lane & 7) ^ ((lr >> 1) & 7);
    int r;
    if constexpr (ATR) {
      const int p = (wave * 8 + j) * 64 + lane;                  // 16-byte unit of the A slab this lane fills
      const int row = p >> 5, u = p & 31;                        // k-row of the slab, unit inside the row
      const int f = (row & 3) | (((row >> 3) & 1) << 2);
      const int m = tm * BM + (((u >> 1) ^ f) << 4) + ((u & 1) << 3);
      ap[j] = A + tiled_index(row, m, d.lda);
    } else {
      r = tm * BM + (Epi::kPermute ? perm_lds_row_a(lr) : lr); r = r < M ? r : M - 1;
      if (d.a_rows) r = d.a_rows[r];
      ap[j] = A + (d.a_tiled ? tiled_index(r, 0, d.K) : (int64_t)r * d.lda) + c * 8;
    }
    r = tn * BN + (Epi::kPermute ? perm_lds_row_b(lr) : lr); r = r < N ? r : N - 1;
    if (d.b_rows) r = d.b_rows[r];
    bp[j] = B + (d.b_tiled ? tiled_index(r, 0, d.K) : (int64_t)r * d.ldb) + c * 8;
    aoff[j] = (unsigned)(ap[j] - abase) * 2u;                   // in bytes
    boff[j] = GB ? 0u : (unsigned)(bp[j] - bbase) * 2u;
  }
  const int a_ks = d.a_tiled ? 16384 : BK, b_ks = d.b_tiled ? 16384 : BK;     // elements from one slab to the next
  // K-major A: slab s is k-rows [64 s, 64 s + 64), i.e. quarter s%4 of row block s/4 of the tiled layout
  auto a_slab = [&](int slab) __attribute__((always_inline)) -> int64_t {
    return ATR ? (int64_t)(slab >> 2) * (d.lda * 256) + (slab & 3) * 4096 : (int64_t)slab * a_ks;
  };
  // load j of the 16 per slab (0..7 = A rows, 8..15 = B rows)
  auto issue1 = [&](int slab, unsigned char* stage, int j) __attribute__((always_inline)) {
    unsigned char* as = stage + wave * 64 * kSlabBytes;
    if (j < 8) {
      load16_to_lds_uniform(abase + a_slab(slab), aoff[j], as + j * 8 * kSlabBytes);   // (the hot kernel is not launched with gathered A rows)
    } else {
      if constexpr (GB) load16_to_lds_lanes(bp[j - 8] + (int64_t)slab * b_ks, as + A_BYTES + (j - 8) * 8 * kSlabBytes);
      else load16_to_lds_uniform(bbase + (int64_t)slab * b_ks, boff[j - 8], as + A_BYTES + (j - 8) * 8 * kSlabBytes);
    }
  };

  // ---- L2 prefetch.  The workgroups resident on one XCD at a time form (about) a block of 8 M-tiles
  // by 4 N-tiles that walks K in lock-step.  Wavefront 0 touches one quarter of the A panel rows,
  // wavefront 1 one eighth of the B panel rows, PFD slabs ahead, one 4-byte load per 128-byte line:
  // between them the block's workgroups cover every line once.  Wavefronts 2 and 3 execute the same
  // instruction on one fixed line (no divergent control flow around the accumulators).
  const unsigned char* pf_ptr;
  int pf_stride;
  const bool pf_atr = ATR && wave == 0;
  if (pf_atr) {                                    // K-major A: the slab's 256 lines are (k-row, 64-m block); a quarter per N-tile
    const int q = 64 * (tn & 3) + lane;
    pf_ptr = reinterpret_cast<const unsigned char*>(A + tiled_index(q >> 2, tm * BM + 64 * (q & 3), d.lda));
    pf_stride = 0;
  } else if (wave == 0) {
    int r = tm * BM + 64 * (tn & 3) + lane; r = r < M ? r : M - 1;
    if (d.a_rows) r = d.a_rows[r];
    pf_ptr = reinterpret_cast<const unsigned char*>(A + (d.a_tiled ? tiled_index(r, 0, d.K) : (int64_t)r * d.lda));
    pf_stride = a_ks * 2;
  } else if (wave == 1) {
    int r = tn * BN + 32 * (tm & 7) + (lane & 31); r = r < N ? r : N - 1;
    if (d.b_rows) r = d.b_rows[r];
    pf_ptr = reinterpret_cast<const unsigned char*>(B + (d.b_tiled ? tiled_index(r, 0, d.K) : (int64_t)r * d.ldb));
    pf_stride = b_ks * 2;
  } else {
    pf_ptr = reinterpret_cast<const unsigned char*>(A);
    pf_stride = 0;
  }
  unsigned pf0 = 0, pf1 = 0, pf_sink = 0;
  auto prefetch = [&](unsigned& slot, int kt) __attribute__((always_inline)) {
    if (PFD > 0) {
      pf_sink ^= slot;                                   // fetched two slabs ago: long since back
      const int k = kt + PFD < nk ? kt + PFD : nk - 1;
      slot = *reinterpret_cast<const unsigned*>(pf_ptr + (int64_t)k * pf_stride + (pf_atr ? a_slab(k) * 2 : 0));
    }
  };

  TileCtx c;
  c.m0 = tm * BM + wm * WM; c.n0 = tn * BN + wn * WN;
  c.Mv = M; c.Nv = N; c.lane = lane; c.wm = wm; c.wn = wn; c.tile_m = tm; c.tile_n = tn; c.tid = tid;
  // what the epilogue needs from memory per column or row (a few registers): fetched now, used after the main loop
  const typename Epi::Pre pre = epi.template preload<Layout16>(c, d);

  floatx4 acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;

  // ---- fragments.  Operand of a 16x16x32 MFMA: lane l holds row l%16, k = 8*(l/16) .. +7 of the
  // 32-wide k-step, i.e. 16-byte chunk 4*s + l/16 of its row in the slab.  A k-step is consumed in
  // two phases (all eight A blocks against B blocks 0..3, then against B blocks 4..7), so the
  // register sets are: A two sets of eight, B two sets of four.
  const int frow = lane & 15, fq = lane >> 4;
  const int arow = (wm * WM + frow) * kSlabBytes, brow = A_BYTES + (wn * WN + frow) * kSlabBytes;
  const int swz = (frow >> 1) & 7;                 // the other row blocks are 16 rows apart: same swizzle
  u32x4_t fa[2][MB], fb[2][NB / 2];
  // K-major A: byte offset, in the slab, of the 8-byte piece this lane points a transposing read of block bi at:
  // k-row 8 (l/16) + (l%16)/4 of the k-step, 32-byte chunk (8 wm + bi) ^ f(row), piece l%4
  int atr_base[MB];
  if constexpr (ATR) {
    const int f = ((frow >> 2) & 3) | ((fq & 1) << 2);
#pragma unroll
    for (int i = 0; i < MB; ++i) atr_base[i] = (8 * fq + (frow >> 2)) * 512 + (((wm * 8 + i) ^ f) << 5) + ((frow & 3) << 3);
  }
  // half h (k = 0..3 or 4..7 of the lane's eight) of A block i of k-step fs
  auto read_a_tr = [&](u32x4_t& dst, const unsigned char* fstage, int i, int fs, int h) __attribute__((always_inline)) {
    const u32x2_t v = lds_read_tr16(fstage + atr_base[i] + (32 * fs + 4 * h) * 512);
    dst[2 * h] = v[0]; dst[2 * h + 1] = v[1];
  };
  auto kof = [&](int k) __attribute__((always_inline)) { return k < nk ? k : nk - 1; };   // slab number; past the end: harmless re-load

  // One phase = 32 MFMAs on (fa[aset], fb[bset]) into column half `half`, with, at fixed places between them,
  //  * fragment reads for the next phase, one per DSG MFMAs.  kind 4: fb[bset^1] <- B blocks 4..7 of
  //    k-step fs in fstage; kind 12: fa[aset^1], fb[bset^1] <- A blocks 0..7 and B blocks 0..3 of k-step fs
  //  * slab loads lo .. lo+nvm-1 of the slab at k0 into wstage.
  // Every MFMA (with what follows it) is fenced off, so the order below is the order issued.
  auto phase = [&](int aset, int bset, int half, int kind, const unsigned char* fstage, int fs,
                   int k0, unsigned char* wstage, int lo, int nvm) __attribute__((always_inline)) {
    const int slot = ((fs * 4 + fq) ^ swz) << 4;
#pragma unroll
    for (int q = 0; q < 32; ++q) {
      mfma16(acc[q >> 2][half * 4 + (q & 3)], fa[aset][q >> 2], fb[bset][q & 3]);
      if (ATR && kind == 12) {                          // sixteen half-reads of A, one per MFMA, then the four of B
        if (q < 16) read_a_tr(fa[aset ^ 1][q >> 1], fstage, q >> 1, fs, q & 1);
        else if (q % DSG == 0 && q < 24) fb[bset ^ 1][(q - 16) / DSG] = *reinterpret_cast<const u32x4_t*>(fstage + brow + ((q - 16) / DSG) * 16 * kSlabBytes + slot);
      } else if (q % DSG == 0 && q / DSG < kind) {
        const int f = q / DSG;
        if (kind == 4) fb[bset ^ 1][f] = *reinterpret_cast<const u32x4_t*>(fstage + brow + (4 + f) * 16 * kSlabBytes + slot);
        else if (f < 8) fa[aset ^ 1][f] = *reinterpret_cast<const u32x4_t*>(fstage + arow + f * 16 * kSlabBytes + slot);
        else fb[bset ^ 1][f - 8] = *reinterpret_cast<const u32x4_t*>(fstage + brow + (f - 8) * 16 * kSlabBytes + slot);
      }
      if (q % VMG == VMO && q / VMG < nvm) issue1(k0, wstage, lo + q / VMG);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // Slab kt sits in `cur`.  On entry fa[0] / fb[0] hold its k-step 0 (A all, B blocks 0..3) and loads
  // 0..LDA-1 of slab kt+1 are in flight towards `nxt`.  The last phase runs from registers after the
  // workgroup barrier, so it covers the first fragment reads of slab kt+1 and the first loads of kt+2.
  auto slab = [&](unsigned char* cur, unsigned char* nxt, int kt, unsigned& pfslot) __attribute__((always_inline)) {
    prefetch(pfslot, kt);
    phase(0, 0, 0, 4, cur, 0, kof(kt + 1), nxt, LDA, LDB);
    phase(0, 1, 1, 12, cur, 1, kof(kt + 1), nxt, LDA + LDB, LDC);
    phase(1, 0, 0, 4, cur, 1, 0, nxt, 0, 0);
    __builtin_amdgcn_s_waitcnt(0x0070);     // vmcnt(0) lgkmcnt(0): own loads have landed, own fragment reads are done
    __syncthreads();                        // ... and so have everybody else's: `nxt` is complete, `cur` is free
    phase(1, 1, 1, 12, nxt, 0, kof(kt + 2), cur, 0, LDA);
  };

  if (nk > 0) {
#pragma unroll
    for (int j = 0; j < 16; ++j) issue1(0, stage0, j);
    __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0)
    __syncthreads();
#pragma unroll
    for (int j = 0; j < LDA; ++j) issue1(kof(1), stage1, j);
    {
      const int slot = (fq ^ swz) << 4;
#pragma unroll
      for (int i = 0; i < MB; ++i) {
        if constexpr (ATR) { read_a_tr(fa[0][i], stage0, i, 0, 0); read_a_tr(fa[0][i], stage0, i, 0, 1); }
        else fa[0][i] = *reinterpret_cast<const u32x4_t*>(stage0 + arow + i * 16 * kSlabBytes + slot);
      }
#pragma unroll
      for (int j = 0; j < NB / 2; ++j) fb[0][j] = *reinterpret_cast<const u32x4_t*>(stage0 + brow + j * 16 * kSlabBytes + slot);
    }
    for (int kt = 0; kt < nk; kt += 2) {    // nk is even (K % 128 == 0 is a launch condition)
      slab(stage0, stage1, kt, pf0);
      slab(stage1, stage0, kt + 1, pf1);
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0070);       // trailing re-loads must land before the epilogue reuses LDS
  __syncthreads();
  mfma_drain();

  epi.template run<Layout16, MB, NB, BM, BN, WAVES_M, WAVES_N, true>(acc, c, stage0, d, pre);
  if (PFD > 0 && (pf_sink ^ pf0 ^ pf1) == 0x9E3779B9u && K < 0) epi.keep_alive();   // never true: keeps the prefetch loads
}

template <class Epi, class Tune, bool ATR = false>
__global__ __launch_bounds__(256)
void gemm_nt_bf16_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ B, GemmDims d, Epi epi) {
  __shared__ __attribute__((aligned(1024))) unsigned char stage0[kHotStageBytes];
  __shared__ __attribute__((aligned(1024))) unsigned char stage1[kHotStageBytes];
  gemm_nt_bf16_tile<Epi, Tune::kPfd, Tune::kVmg, Tune::kVmo, ATR, Tune::kLdA, Tune::kLdB>(A, B, d, epi, blockIdx.x, stage0, stage1);
}

// Two independent contractions in one launch: workgroups [0, n1) work on the first, the rest on the
// second.  Used where one of them alone has too few tiles to fill the last round of the 256 CUs: the
// other's workgroups then fill the tail.  n1 = launch_tiles() of the first (a multiple of the XCD count).
// ATR2: the second contraction's A operand is given K-major (see gemm_nt_bf16_tile).
template <class Epi1, class Tune1, class Epi2, class Tune2, bool ATR2 = false>
__global__ __launch_bounds__(256)
void gemm_nt_bf16_pair_kernel(const bf16_t* __restrict__ A1, const bf16_t* __restrict__ B1, GemmDims d1, Epi1 epi1, int n1,
                              const bf16_t* __restrict__ A2, const bf16_t* __restrict__ B2, GemmDims d2, Epi2 epi2) {
  __shared__ __attribute__((aligned(1024))) unsigned char stage0[kHotStageBytes];
  __shared__ __attribute__((aligned(1024))) unsigned char stage1[kHotStageBytes];
  if ((int)blockIdx.x < n1)
    gemm_nt_bf16_tile<Epi1, Tune1::kPfd, Tune1::kVmg, Tune1::kVmo, false, Tune1::kLdA, Tune1::kLdB>(A1, B1, d1, epi1, blockIdx.x, stage0, stage1);
  else
    gemm_nt_bf16_tile<Epi2, Tune2::kPfd, Tune2::kVmg, Tune2::kVmo, ATR2, Tune2::kLdA, Tune2::kLdB>(A2, B2, d2, epi2, (int)blockIdx.x - n1, stage0, stage1);
}

}  // namespace rlk
