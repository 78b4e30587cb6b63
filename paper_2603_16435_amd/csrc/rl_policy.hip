// rl_policy.hip - kernels of the O(T) stages and the C ABI of the library.
//
// Pipeline of rl_policy_loss_fwd_bwd (all on the caller's stream, no host sync):
//   prep      : per-sequence counts -> scan -> ordered compaction of the rows that count
//               (row_map, ids_c), masked rows of the outputs zeroed
//   advantage : group mean / std of the rewards -> A_i
//   forward   : per chunk of compacted rows: logits tiles (MFMA) -> partial (max,sumexp) per
//               vocab tile + target logit -> combine -> lse_t, logp_t
//   loss      : one workgroup per sequence: length-normalised sums, loss_i, c_t; final reduce
//   backward  : W^T once; per chunk: X^T, recomputed logits -> dS (input precision; f32 inputs also dS^T),
//               dX = dS W (scattered to original rows), dW (+)= dS^T X (bf16: dS read as a K-major operand)
// The number of real rows is only known on the device, so grids are sized for the upper
// bound R and every kernel trims itself against the device-side count.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <string.h>

#include <mutex>
#include <utility>
#include <vector>

#include "../../include/rl_policy.h"
#include "../../include/rl_policy_diag.h"
#include "epilogues.h"
#include "logz_head.h"
#include "rvq_encode.h"
#include "gemm_nt.h"

namespace rlk {

constexpr int kDefaultChunkRows = 32768;        // recompute mode: 128 x 14 dX tiles = 7 full rounds of 256 CUs on the 7B shape
constexpr int kDefaultChunkRowsStash = 40960;   // single-pass mode: the step time is flat (+-0.7 %) from 24576 to 65536 rows
constexpr int kBM = 256, kBN = 256, kWavesM = 2, kWavesN = 4;
constexpr int kGemmThreads = kWavesM * kWavesN * 64;
constexpr int kGemmSmem = 2 * (kBM + kBN) * kSlabBytes;   // 128 KiB of the 160 KiB per CU
// Per-contraction tuning of the hot kernel, from sweeps on the 7B-shaped workload:
// tile-order band height (M-tiles per band), L2 prefetch distance in slabs (0 = off), where in a
// phase of 32 MFMAs the slab loads are issued (after MFMA kVmo, kVmo + kVmg, ...) and how many of a slab's 16 loads
// go into the phase after the barrier / the next phase (kLdA / kLdB; the rest into the phase after that).
// Measured on the 7B shape: with the XCDs sweeping N in step the dX prefetch only costs (-4 % of dX+dW when off; its
// band height then makes no difference between 1 and 8), dW is best with one M-tile per band (its A panel, the stored
// probabilities, then leaves memory once for all 14 N-tiles), the logits want the prefetch (off: +4 % on the forward).
// dX, whose operands both stream from memory, waits 17 % of its loop time for its slab loads with the 6/5/5 placement and
// 5 % with 8/8/0 (all loads at least two phases before the barrier); at the power limit that is worth 0.8 % of dX+dW.
// The other two lose with 8/8/0.
struct TuneLogits { static constexpr int kBand = 8, kPfd = 2, kVmg = 5, kVmo = 3, kLdA = 6, kLdB = 5; };
struct TuneDX     { static constexpr int kBand = 8, kPfd = 0, kVmg = 4, kVmo = 1, kLdA = 8, kLdB = 8; };
struct TuneDW     { static constexpr int kBand = 1, kPfd = 2, kVmg = 4, kVmo = 1, kLdA = 6, kLdB = 5; };

struct Ctrl {            // device control block at the head of the workspace
  int n_real;
  int too_long;          // single-pass backward: some sequence has more rows than the caller promised / a chunk holds
  int overflow;          // single-pass backward: rows whose stored probabilities left the range of the staging precision
  int pad[13];
};

struct ChunkDesc {       // device record of one sequence-aligned chunk (single-pass backward)
  int row_start, rows;   // compacted rows [row_start, row_start + rows)
  int seq_begin, seq_end;// sequences [seq_begin, seq_end) lie wholly inside
};

// ------------------------------------------------------------------ optional launch timing
// When enabled (benchmarks only), each group of launches is bracketed by a pair of HIP events
// on the caller's stream; rl_profile_read() folds the elapsed times per class.
struct ProfRec { hipEvent_t a, b; int cls; };
struct Profiler {
  bool on = false;
  std::vector<ProfRec> recs;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> pool;
};
static Profiler g_prof;

struct ProfScope {
  hipStream_t s; hipEvent_t a{}, b{}; int cls; bool live;
  ProfScope(int cls_, hipStream_t s_) : s(s_), cls(cls_), live(g_prof.on) {
    if (!live) return;
    if (!g_prof.pool.empty()) { a = g_prof.pool.back().first; b = g_prof.pool.back().second; g_prof.pool.pop_back(); }
    else { if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) { live = false; return; } }
    (void)hipEventRecord(a, s);
  }
  ~ProfScope() {
    if (!live) return;
    (void)hipEventRecord(b, s);
    g_prof.recs.push_back({a, b, cls});
  }
};

// ------------------------------------------------------------------ small utilities
__device__ inline int wave_prefix_count(bool flag, int lane, int& total) {
  const unsigned long long b = __ballot(flag);
  total = __popcll(b);
  return __popcll(b & ((1ull << lane) - 1ull));
}

template <class V>
__global__ void fill_kernel(V* p, int64_t n, V v) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t step = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += step) p[i] = v;
}

template <class V>
static void fill(V* p, int64_t n, V v, hipStream_t s) {
  if (!p || n <= 0) return;
  int64_t blocks = (n + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  fill_kernel<V><<<(int)blocks, 256, 0, s>>>(p, n, v);
}

__device__ inline double block_sum(double v, double* sh) {   // blockDim.x multiple of 64, <= 1024
  for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) sh[w] = v;
  __syncthreads();
  double r = 0.0;
  const int nw = blockDim.x >> 6;
  for (int i = 0; i < nw; ++i) r += sh[i];                   // same order in every thread
  return r;
}

// ------------------------------------------------------------------ prep
// Inclusive running maximum of the sequence offsets, hi[i] = max(cu[0..i]) for i < B (single workgroup of 1024).
// A sequence keeps its rows only if its first offset is not below any earlier offset: the kept row ranges are then
// pairwise disjoint whatever the offsets are, so no row can count twice and the compacted rows never exceed R.
__global__ void cu_running_max_kernel(const int32_t* cu, int B, int32_t* hi) {
  __shared__ int wmax[16];
  __shared__ int carry;
  if (threadIdx.x == 0) carry = INT32_MIN;
  __syncthreads();
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  for (int base = 0; base < B; base += 1024) {
    const int i = base + threadIdx.x;
    int x = i < B ? cu[i] : INT32_MIN;
    for (int o = 1; o < 64; o <<= 1) { const int y = __shfl_up(x, o); if (lane >= o) x = max(x, y); }
    if (lane == 63) wmax[w] = x;
    __syncthreads();
    int m = carry;
    for (int k = 0; k < w; ++k) m = max(m, wmax[k]);
    x = max(x, m);
    if (i < B) hi[i] = x;
    __syncthreads();
    if (threadIdx.x == 1023) carry = x;
    __syncthreads();
  }
}

// One workgroup per sequence: validate its row range and group index, count rows that count.
__global__ void seq_count_kernel(const uint8_t* mask, const int32_t* ids, const int32_t* cu, const int32_t* cu_hi,
                                 const int32_t* group_idx, int64_t R, int V, int P,
                                 int32_t* seq_len, rl_stats* stats) {
  const int i = blockIdx.x;
  __shared__ int sh_cnt, sh_bad;
  if (threadIdx.x == 0) { sh_cnt = 0; sh_bad = 0; }
  __syncthreads();
  const int64_t a = cu[i], b = cu[i + 1];
  const bool seq_ok = (a >= 0 && a <= b && b <= R && a >= cu_hi[i]);
  const bool grp_ok = (group_idx == nullptr) || (group_idx[i] >= 0 && group_idx[i] < P);
  int cnt = 0, bad = 0;
  if (seq_ok && grp_ok) {
    for (int64_t r = a + threadIdx.x; r < b; r += blockDim.x) {
      if (mask[r]) {
        const int y = ids[r];
        if (y >= 0 && y < V) ++cnt; else ++bad;
      }
    }
  }
  for (int o = 32; o > 0; o >>= 1) { cnt += __shfl_down(cnt, o); bad += __shfl_down(bad, o); }
  if ((threadIdx.x & 63) == 0) { atomicAdd(&sh_cnt, cnt); atomicAdd(&sh_bad, bad); }
  __syncthreads();
  if (threadIdx.x == 0) {
    seq_len[i] = sh_cnt;
    if (stats) {
      if (sh_bad) atomicAdd(&stats->n_bad_token, sh_bad);
      if (!seq_ok) atomicAdd(&stats->n_bad_seq, 1);
      if (!grp_ok) atomicAdd(&stats->n_bad_group, 1);
    }
  }
}

// Exclusive scan of seq_len over sequences (single workgroup of 1024), total -> ctrl.
__global__ void seq_scan_kernel(const int32_t* seq_len, int B, int32_t* cstart, Ctrl* ctrl, rl_stats* stats) {
  __shared__ int wsum[16];
  __shared__ int carry;
  if (threadIdx.x == 0) carry = 0;
  __syncthreads();
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  for (int base = 0; base < B; base += 1024) {
    const int i = base + threadIdx.x;
    const int v = i < B ? seq_len[i] : 0;
    int x = v;
    for (int o = 1; o < 64; o <<= 1) { const int y = __shfl_up(x, o); if (lane >= o) x += y; }
    if (lane == 63) wsum[w] = x;
    __syncthreads();
    int woff = 0;
    for (int k = 0; k < w; ++k) woff += wsum[k];
    if (i < B) cstart[i] = carry + woff + x - v;
    __syncthreads();
    if (threadIdx.x == 1023) carry += woff + x;
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    cstart[B] = carry;
    ctrl->n_real = carry;
    ctrl->too_long = 0;
    ctrl->overflow = 0;
    if (stats) stats->n_tokens = carry;
  }
}

// Ordered compaction, one workgroup per sequence: the k-th counting row of sequence i becomes
// compact row cstart[i]+k.  cpos[r] = compact position of original row r (left at -1 otherwise).
__global__ void compact_kernel(const uint8_t* mask, const int32_t* ids, const int32_t* cu,
                               const int32_t* seq_len, const int32_t* cstart, int V,
                               int32_t* row_map, int32_t* ids_c, int32_t* cpos, int32_t* row_map_out) {
  const int i = blockIdx.x;
  if (seq_len[i] == 0) return;
  __shared__ int wsum[16];
  __shared__ int carry;
  if (threadIdx.x == 0) carry = cstart[i];
  __syncthreads();
  const int64_t a = cu[i], b = cu[i + 1];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  for (int64_t base = a; base < b; base += blockDim.x) {
    const int64_t r = base + threadIdx.x;
    int y = 0;
    bool f = false;
    if (r < b && mask[r]) { y = ids[r]; f = (y >= 0 && y < V); }
    int tot;
    const int pre = wave_prefix_count(f, lane, tot);
    if (lane == 0) wsum[w] = tot;
    __syncthreads();
    int woff = 0, all = 0;
    for (int k = 0; k < nw; ++k) { if (k < w) woff += wsum[k]; all += wsum[k]; }
    if (f) {
      const int c = carry + woff + pre;
      row_map[c] = (int)r; ids_c[c] = y; cpos[r] = c;
      if (row_map_out) row_map_out[c] = (int)r;
    }
    __syncthreads();
    if (threadIdx.x == 0) carry += all;
    __syncthreads();
  }
}

template <class T>
__global__ void zero_masked_rows_kernel(const int32_t* cpos, T* dX, int64_t R, int H) {
  // one wavefront per row; rows that count are left alone (the dX epilogue writes them)
  const int64_t r = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (r >= R || cpos[r] >= 0) return;
  const int lane = threadIdx.x & 63;
  uint4* p = reinterpret_cast<uint4*>(dX + r * H);
  const int n16 = H * (int)sizeof(T) / 16;
  for (int k = lane; k < n16; k += 64) p[k] = make_uint4(0, 0, 0, 0);
}

// ------------------------------------------------------------------ advantage
// Thread per prompt p: mean and std of the rewards of its members, then A_i for each member.
__global__ void advantage_kernel(const float* rewards, const int32_t* group_idx, int B, int P,
                                 float adv_eps, int ddof, float* adv, int32_t* group_count) {
  const int p = blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= P) return;
  int n = 0; double s = 0.0;
  for (int i = 0; i < B; ++i) if (group_idx[i] == p) { ++n; s += (double)rewards[i]; }
  if (group_count) group_count[p] = n;
  if (n == 0) return;
  const double mu = s / n;
  double inv = 0.0;
  if (n - ddof > 0) {
    double q = 0.0;
    for (int i = 0; i < B; ++i) if (group_idx[i] == p) { const double e = (double)rewards[i] - mu; q += e * e; }
    inv = 1.0 / (sqrt(q / (n - ddof)) + (double)adv_eps);
  }
  for (int i = 0; i < B; ++i) if (group_idx[i] == p) adv[i] = (float)(((double)rewards[i] - mu) * inv);
}

// ------------------------------------------------------------------ single-pass backward: chunking and references
// Greedy packing of whole sequences into chunks of at most Tc compacted rows (one thread: B is small).
// Two consecutive chunks together hold more than Tc rows, so n_desc = 2 ceil(R / Tc) + 1 records
// always suffice; unused records are empty.  A sequence longer than max_len (<= Tc) raises the flag.
__global__ void chunk_build_kernel(const int32_t* seq_len, const int32_t* cstart, int B, int Tc, int max_len,
                                   ChunkDesc* desc, int n_desc, Ctrl* ctrl, rl_stats* stats) {
  if (blockIdx.x != 0 || threadIdx.x != 0) return;
  int k = 0, start = 0, rows = 0, sb = 0, bad = 0;
  for (int i = 0; i < B; ++i) {
    const int n = seq_len[i];
    if (n > max_len) ++bad;
    if (rows > 0 && rows + n > Tc && k < n_desc - 1) {
      desc[k].row_start = start; desc[k].rows = rows; desc[k].seq_begin = sb; desc[k].seq_end = i;
      ++k; start += rows; rows = 0; sb = i;
    }
    rows += n;
  }
  desc[k].row_start = start; desc[k].rows = rows; desc[k].seq_begin = sb; desc[k].seq_end = B;
  for (int j = k + 1; j < n_desc; ++j) { desc[j].row_start = start + rows; desc[j].rows = 0; desc[j].seq_begin = B; desc[j].seq_end = B; }
  if (bad) { ctrl->too_long = 1; if (stats) stats->n_seq_too_long = bad; }
}

// One wavefront per compacted row t: target logit zy_t = x_t . W[y_t] (f32 accumulation of bf16 products)
// (times the inverse temperature) and the reference of the stored probabilities, ref_t = zy_t - old_t, which is
// the logsumexp of the row up to the (small) drift between the old and the current policy (NaN-free for any finite old_t).
__global__ void target_logit_kernel(const bf16_t* X, const bf16_t* W, int H, const int32_t* row_map, const int32_t* ids_c,
                                    const float* old_lp, const Ctrl* ctrl, float inv_tau, float* zy, float* ref_l2e, int32_t* ycol) {
  const int t = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (t >= ctrl->n_real) return;
  const int lane = threadIdx.x & 63;
  const int r = row_map[t];
  const uint4* x = reinterpret_cast<const uint4*>(X + (int64_t)r * H);
  const int y = ids_c[t];
  const uint4* w = reinterpret_cast<const uint4*>(W + (int64_t)y * H);
  float acc = 0.f;
  for (int k = lane; k < H / 8; k += 64) {
    const uint4 a = x[k], b = w[k];
    const unsigned av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      acc = fmaf(__uint_as_float(av[j] << 16), __uint_as_float(bv[j] << 16), acc);
      acc = fmaf(__uint_as_float(av[j] & 0xffff0000u), __uint_as_float(bv[j] & 0xffff0000u), acc);
    }
  }
  for (int o = 32; o > 0; o >>= 1) acc += __shfl_down(acc, o);
  if (lane == 0) {
    // the old log-prob only steers the reference; clamped to [-40, 0] a wild value costs range, not correctness:
    // exp(z - ref) stays representable for current log-probs between about -120 and 0
    const float o = fminf(fmaxf(old_lp[r], -40.f), 0.f);
    acc *= inv_tau;
    zy[t] = acc; ref_l2e[t] = (acc - o) * 1.4426950408889634f;
    ycol[t] = y;                                   // the row of W the target logit was read from
  }
}

// Per-tile-row partial sums (s, u) of a chunk -> lse, logp, entropy and Z_t = sum_v exp(z - ref_t).
// A workgroup handles 64 rows x 16 slices of the tile range (1024 threads: the sums are chains of dependent f64 adds,
// so it takes many short chains to keep the memory system busy), merged through LDS in a fixed order.
constexpr int kSumSlices = 16;
__global__ __launch_bounds__(64 * kSumSlices) void lse_sum_kernel(const float2* part, int ldp, int tiles_v, const float* zy_c, const float* ref_l2e,
                               const int32_t* row_map, const ChunkDesc* desc, const int32_t* ycol_c, Ctrl* ctrl, rl_stats* stats,
                               float* lse_c, float* logp_c, float* zsum_c, float* lse_out, float* logp_out, float* ent_out,
                               float* zy_out, int32_t* ycol_out) {
  __shared__ double ss[kSumSlices][64], su[kSumSlices][64];
  const int left = desc->rows, chunk_start = desc->row_start;
  if ((int)blockIdx.x * 64 >= left) return;
  const int col = threadIdx.x & 63, slice = threadIdx.x >> 6;
  const int n = blockIdx.x * 64 + col;
  double s = 0.0, u = 0.0;
  if (n < left)
    for (int t = slice; t < tiles_v; t += kSumSlices) { const float2 v = part[(int64_t)t * ldp + n]; s += (double)v.x; u += (double)v.y; }
  ss[slice][col] = s; su[slice][col] = u;
  __syncthreads();
  if (slice == 0 && n < left) {
    double S = 0.0, U = 0.0;
    for (int k = 0; k < kSumSlices; ++k) { S += ss[k][col]; U += su[k][col]; }
    const int g = chunk_start + n;
    const double lse_d = (double)ref_l2e[g] * 0.6931471805599453 + log(S);
    const float lse = (float)lse_d;
    const float lp = zy_c[g] - lse;
    lse_c[g] = lse; logp_c[g] = lp; zsum_c[g] = (float)S;
    // Z_t = exp(lse_t - ref_t) is of order one when the old log-prob is anywhere near the current one.  A row whose
    // sum left [1e-30, 1e30] (or is not a number) had stored probabilities outside the staging precision's range:
    // counted, and the loss of the call comes back NaN.
    if (!(S >= 1e-30 && S <= 1e30)) { atomicAdd(&ctrl->overflow, 1); if (stats) atomicAdd(&stats->n_overflow_rows, 1); }
    const int r = row_map[g];
    if (lse_out) lse_out[r] = lse;
    if (logp_out) logp_out[r] = lp;
    if (ent_out) ent_out[r] = (float)fmax(lse_d - U / S, 0.0);
    if (zy_out) zy_out[r] = zy_c[g];
    if (ycol_out) ycol_out[r] = ycol_c[g];
  }
}

// After the loss: per row of the chunk the factor -c_t / (tau Z_t) of the backward contractions (1 / tau: from the
// tempered logit back to W x_t), and the target entry of the stored probabilities replaced by e_y - Z_t (so that
// the factor times the stored row is dS).
template <class T>
__global__ void stash_patch_kernel(const ChunkDesc* desc, const int32_t* ids_c, const float* zy_c, const float* ref_l2e,
                                   const float* zsum_c, const float* c_c, float inv_tau, float* row_scale,
                                   T* E, int64_t ld_e) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= desc->rows) return;
  const int g = desc->row_start + n;
  const float Z = zsum_c[g];
  row_scale[n] = -c_c[g] * inv_tau / Z;
  const float ey = exp2f(fmaf(zy_c[g], 1.4426950408889634f, -ref_l2e[g]));
  const T v = (T)(ey - Z);
  const int y = ids_c[g];
  E[tiled_index(n, y, ld_e)] = v;
}

// ------------------------------------------------------------------ forward combine
// Fold the per-vocab-tile partials (max, sumexp) of a chunk into lse, logp.  A workgroup handles 64
// compact rows x 4 slices of the tile range: one online (rescaling) pass per thread, coalesced
// along the rows, then the four slices are merged through LDS in a fixed order.
__global__ void lse_combine_kernel(const float4* part, int ldp, int tiles_v, const float* zy_c,
                                   const int32_t* row_map, const Ctrl* ctrl, int chunk_start, int chunk_rows, const int32_t* ycol_c,
                                   float* lse_c, float* logp_c, float* lse_out, float* logp_out, float* ent_out,
                                   float* zy_out, int32_t* ycol_out) {
  __shared__ float sm[4][64], ss[4][64], su[4][64];
  int left = ctrl->n_real - chunk_start;
  if (left > chunk_rows) left = chunk_rows;
  if ((int)blockIdx.x * 64 >= left) return;
  const int col = threadIdx.x & 63, slice = threadIdx.x >> 6;
  const int n = blockIdx.x * 64 + col;
  const float NEG = -__builtin_inff();
  float m = NEG, s = 0.f, u = 0.f;
  if (n < left) {
    for (int t = slice; t < tiles_v; t += 4) {
      const float4 v = part[(int64_t)t * ldp + n];
      const float mm = fmaxf(m, v.x);
      if (mm != NEG) {
        const float f1 = expf(m - mm), f2 = expf(v.x - mm);
        s = s * f1 + v.y * f2;
        u = u * f1 + v.z * f2;
      }
      m = mm;
    }
  }
  sm[slice][col] = m; ss[slice][col] = s; su[slice][col] = u;
  __syncthreads();
  if (slice == 0 && n < left) {
    float M = sm[0][col];
    for (int k = 1; k < 4; ++k) M = fmaxf(M, sm[k][col]);
    double S = 0.0, U = 0.0;
    for (int k = 0; k < 4; ++k)
      if (sm[k][col] != NEG) {
        const double f = exp((double)(sm[k][col] - M));
        S += (double)ss[k][col] * f; U += (double)su[k][col] * f;
      }
    const double lse_d = (double)M + log(S);
    const float lse = (float)lse_d;
    const int g = chunk_start + n;
    const float lp = zy_c[g] - lse;
    lse_c[g] = lse; logp_c[g] = lp;
    const int r = row_map[g];
    if (lse_out) lse_out[r] = lse;
    if (logp_out) logp_out[r] = lp;
    if (ent_out) ent_out[r] = (float)fmax(lse_d - U / S, 0.0);     // H = lse - sum_v p_v z_v
    if (zy_out) zy_out[r] = zy_c[g];
    if (ycol_out) ycol_out[r] = ycol_c[g];
  }
}

// ------------------------------------------------------------------ loss
struct LossOpts {
  float clip_lo, clip_hi;   // ratio / weight kept inside [1 - clip_lo, 1 + clip_hi]
  float kl_coef, beta;
  int token_agg;            // GRPO: loss = (1/T) sum of all token terms instead of the mean of per-sequence means
  int seq_ratio;            // GRPO: one ratio per sequence, exp(mean_t (logp - old))
  int w_mean;               // FLOW: weight from the mean instead of the sum of the token log-ratios
};

// One workgroup per sequence over its compact rows [cstart[i], cstart[i+1]).
__global__ void seq_loss_kernel(int objective, const float* logp_c, const float* old_lp, const float* ref_lp,
                                const int32_t* row_map, const int32_t* cstart, const float* adv,
                                const int32_t* group_idx, const float* log_z, int B, LossOpts o, const Ctrl* ctrl,
                                float* seq_loss, float* gterm, float* c_c, float* coeff_out, rl_stats* stats,
                                const ChunkDesc* desc) {
  __shared__ double sh[16];
  __shared__ int sh_hi, sh_lo;
  int i = blockIdx.x;
  if (desc) {                           // only the sequences of one chunk
    i += desc->seq_begin;
    if (i >= desc->seq_end) return;
  }
  const int a = cstart[i], b = cstart[i + 1], n = b - a;
  if (threadIdx.x == 0) { sh_hi = 0; sh_lo = 0; }
  if (n <= 0) {
    if (threadIdx.x == 0) { seq_loss[i] = 0.f; gterm[i] = 0.f; }
    return;
  }
  const float A = adv[i];
  const double Ad = (double)A;
  const double inv_bn = 1.0 / ((double)B * (double)n);
  const double lo_c = 1.0 - (double)o.clip_lo, hi_c = 1.0 + (double)o.clip_hi;
  if (objective == RL_OBJ_GRPO && !o.seq_ratio) {
    // weight of a token term in the loss: 1/(B n_i) (mean of per-sequence means) or 1/T (mean over all tokens)
    const double wt = o.token_agg ? 1.0 / (double)ctrl->n_real : inv_bn;
    double acc = 0.0; int hi = 0, lo = 0;
    for (int k = a + threadIdx.x; k < b; k += blockDim.x) {
      const int r = row_map[k];
      // per-token terms in f64: e^d - d - 1 cancels to ~d^2/2 and would lose digits in f32
      const double lp = (double)logp_c[k];
      const double rho = exp(lp - (double)old_lp[r]);
      const double dd = (double)ref_lp[r] - lp;
      const double ed = exp(dd);
      const double rc = fmin(fmax(rho, lo_c), hi_c);
      const double l = -fmin(rho * Ad, rc * Ad) + (double)o.kl_coef * (ed - dd - 1.0);
      const bool chi = (A > 0.f) && (rho > hi_c);
      const bool clo = (A < 0.f) && (rho < lo_c);
      hi += chi; lo += clo;
      const double g = ((chi || clo) ? 0.0 : -Ad * rho) + (double)o.kl_coef * (1.0 - ed);
      const float ct = (float)(g * wt);
      c_c[k] = ct;
      if (coeff_out) coeff_out[r] = ct;
      acc += l;
    }
    const double tot = block_sum(acc, sh);
    for (int q = 32; q > 0; q >>= 1) { hi += __shfl_down(hi, q); lo += __shfl_down(lo, q); }
    if ((threadIdx.x & 63) == 0) { if (hi) atomicAdd(&sh_hi, hi); if (lo) atomicAdd(&sh_lo, lo); }
    __syncthreads();
    if (threadIdx.x == 0) {
      // token aggregation reports (B/T) sum_t l_t, so that loss = mean_i seq_loss_i in both aggregations
      seq_loss[i] = (float)(o.token_agg ? tot * wt * (double)B : tot / n); gterm[i] = 0.f;
      if (stats) { if (sh_hi) atomicAdd(&stats->n_clip_hi, sh_hi); if (sh_lo) atomicAdd(&stats->n_clip_lo, sh_lo); }
    }
  } else if (objective == RL_OBJ_GRPO) {
    // sequence-level ratio s = exp(mean_t (logp - old)): first the mean and the KL sum, then the coefficients
    double s_old = 0.0, s_kl = 0.0;
    for (int k = a + threadIdx.x; k < b; k += blockDim.x) {
      const int r = row_map[k];
      const double lp = (double)logp_c[k];
      const double dd = (double)ref_lp[r] - lp;
      s_old += lp - (double)old_lp[r];
      s_kl += exp(dd) - dd - 1.0;
    }
    const double t_old = block_sum(s_old, sh);
    const double t_kl = block_sum(s_kl, sh);
    const double sr = exp(t_old / n);
    const double rc = fmin(fmax(sr, lo_c), hi_c);
    const bool chi = (A > 0.f) && (sr > hi_c);
    const bool clo = (A < 0.f) && (sr < lo_c);
    const double ds = (chi || clo) ? 0.0 : -Ad * sr;               // d(-surrogate)/d(mean log-ratio)
    for (int k = a + threadIdx.x; k < b; k += blockDim.x) {
      const int r = row_map[k];
      const double dd = (double)ref_lp[r] - (double)logp_c[k];
      const float ct = (float)((ds + (double)o.kl_coef * (1.0 - exp(dd))) * inv_bn);
      c_c[k] = ct;
      if (coeff_out) coeff_out[r] = ct;
    }
    if (threadIdx.x == 0) {
      seq_loss[i] = (float)(-fmin(sr * Ad, rc * Ad) + (double)o.kl_coef * t_kl / n); gterm[i] = 0.f;
      if (stats) { if (chi) atomicAdd(&stats->n_clip_hi, 1); if (clo) atomicAdd(&stats->n_clip_lo, 1); }
    }
  } else {
    double s_ref = 0.0, s_old = 0.0;
    for (int k = a + threadIdx.x; k < b; k += blockDim.x) {
      const int r = row_map[k];
      const float lp = logp_c[k];
      s_ref += (double)(lp - ref_lp[r]);
      s_old += (double)(lp - old_lp[r]);
    }
    const double t_ref = block_sum(s_ref, sh);
    double t_old = block_sum(s_old, sh);
    if (o.w_mean) t_old /= n;
    const double lo_b = log1p(-(double)o.clip_lo), hi_b = log1p((double)o.clip_hi);
    const double w = exp(fmin(fmax(t_old, lo_b), hi_b));
    const double delta = (double)log_z[group_idx[i]] + t_ref / n - (double)o.beta * Ad;
    const float ct = (float)(2.0 * w * delta * inv_bn);
    for (int k = a + threadIdx.x; k < b; k += blockDim.x) {
      c_c[k] = ct;
      if (coeff_out) coeff_out[row_map[k]] = ct;
    }
    if (threadIdx.x == 0) {
      seq_loss[i] = (float)(w * delta * delta);
      gterm[i] = (float)(2.0 * w * delta / (double)B);
      if (stats) { if (t_old > hi_b) atomicAdd(&stats->n_clip_hi, 1); if (t_old < lo_b) atomicAdd(&stats->n_clip_lo, 1); }
    }
  }
}

// loss = (1/B) sum_i seq_loss_i ;  d_logZ_p = sum over members of gterm  (single workgroup)
__global__ void finalize_kernel(const float* seq_loss, const float* gterm, const int32_t* group_idx,
                                const int32_t* seq_len, int B, int P, int objective, const Ctrl* ctrl,
                                float* loss, float* d_log_z, float* seq_loss_out) {
  __shared__ double sh[16];
  double acc = 0.0;
  for (int i = threadIdx.x; i < B; i += blockDim.x) {
    acc += (double)seq_loss[i];
    if (seq_loss_out) seq_loss_out[i] = seq_loss[i];
  }
  const double tot = block_sum(acc, sh);
  // a sequence longer than the caller promised: the single-pass backward dropped rows, say so loudly
  // ... or stored probabilities that left the representable range: the gradients of those rows are not numbers
  if (threadIdx.x == 0) *loss = (ctrl->too_long || ctrl->overflow) ? __builtin_nanf("") : (float)(tot / B);
  if (d_log_z) {
    for (int p = threadIdx.x; p < P; p += blockDim.x) {
      double s = 0.0;
      if (objective == RL_OBJ_FLOW)
        for (int i = 0; i < B; ++i) if (group_idx[i] == p && seq_len[i] > 0) s += (double)gterm[i];
      d_log_z[p] = (float)s;
    }
  }
}

// ------------------------------------------------------------------ transposes (K-contiguous operands)
// dst[c][r] = src[row_of(r)][c] for r < rows_valid, 0 for rows_valid <= r < ld_dst rows covered by the grid.
template <class T>
__global__ void transpose_kernel(const T* src, int64_t ld_src, int rows, int cols, const int32_t* row_idx,
                                 const Ctrl* ctrl, int chunk_start, int dyn_rows, const ChunkDesc* desc, const float* row_scale,
                                 T* dst, int64_t ld_dst, int rows_padded, bool dst_tiled) {
  __shared__ T tile[64][65];
  int rv = rows;
  if (dyn_rows) {
    int left;
    if (desc) { chunk_start = desc->row_start; left = desc->rows; } else left = ctrl->n_real - chunk_start;
    if (left <= 0) return;
    rv = left < rows ? left : rows;
  }
  const int r0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
  if (dyn_rows && r0 >= ((rv + 255) & ~255)) return;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;        // 256 threads: 4 rows per pass
  for (int k = ty; k < 64; k += 4) {
    const int r = r0 + k, c = c0 + tx;
    T v = (T)0.f;
    if (r < rv && c < cols) {
      const int64_t sr = row_idx ? (int64_t)row_idx[chunk_start + r] : (int64_t)r;
      v = src[sr * ld_src + c];
      if (row_scale) v = (T)((float)v * row_scale[r]);
    }
    tile[k][tx] = v;
  }
  __syncthreads();
  for (int k = ty; k < 64; k += 4) {
    const int c = c0 + k, r = r0 + tx;
    if (c < cols && r < rows_padded) dst[operand_index(dst_tiled, c, r, ld_dst)] = tile[tx][k];
  }
}

// The same for bf16 with 16-byte accesses on both sides (cols % 8 == 0, 16-byte aligned rows; rows_padded % 8 == 0, tiled
// destination): a thread loads two 16-byte pieces of source rows and stores two 16-byte pieces of destination rows, each
// gathered from eight consecutive source rows of one column in LDS (row stride 33 dwords: the gather is conflict-free).
__global__ __launch_bounds__(256)
void transpose_bf16_kernel(const bf16_t* src, int64_t ld_src, int rows, int cols, const int32_t* row_idx,
                           const Ctrl* ctrl, int chunk_start, int dyn_rows, const ChunkDesc* desc, const float* row_scale,
                           bf16_t* dst, int64_t ld_dst, int rows_padded) {
  __shared__ unsigned tile[64][33];
  int rv = rows;
  if (dyn_rows) {
    int left;
    if (desc) { chunk_start = desc->row_start; left = desc->rows; } else left = ctrl->n_real - chunk_start;
    if (left <= 0) return;
    rv = left < rows ? left : rows;
  }
  const int r0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
  if (dyn_rows && r0 >= ((rv + 255) & ~255)) return;
  const int ch = threadIdx.x & 7, k0 = threadIdx.x >> 3;
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int k = k0 + 32 * p, r = r0 + k, c = c0 + 8 * ch;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (r < rv && c < cols) {
      const int64_t sr = row_idx ? (int64_t)row_idx[chunk_start + r] : (int64_t)r;
      v = *reinterpret_cast<const uint4*>(src + sr * ld_src + c);
      if (row_scale) {
        const float f = row_scale[r];
        bf16x8 e = __builtin_bit_cast(bf16x8, v);
#pragma unroll
        for (int i = 0; i < 8; ++i) e[i] = (bf16_t)((float)e[i] * f);
        v = __builtin_bit_cast(uint4, e);
      }
    }
    tile[k][4 * ch] = v.x; tile[k][4 * ch + 1] = v.y; tile[k][4 * ch + 2] = v.z; tile[k][4 * ch + 3] = v.w;
  }
  __syncthreads();
  const unsigned short* t16 = reinterpret_cast<const unsigned short*>(&tile[0][0]);
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int k = k0 + 32 * p, c = c0 + k, r = r0 + 8 * ch;
    if (c < cols && r < rows_padded) {
      unsigned w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i)
        w[i] = (unsigned)t16[(8 * ch + 2 * i) * 66 + k] | ((unsigned)t16[(8 * ch + 2 * i + 1) * 66 + k] << 16);
      *reinterpret_cast<uint4*>(dst + tiled_index(c, r, ld_dst)) = make_uint4(w[0], w[1], w[2], w[3]);
    }
  }
}

// Host side: the 16-byte kernel where its conditions hold (always, for the library's own bf16 buffers and 16-byte aligned inputs).
template <class T>
static void launch_transpose(dim3 grid, hipStream_t s, const T* src, int64_t ld_src, int rows, int cols, const int32_t* row_idx,
                             const Ctrl* ctrl, int chunk_start, int dyn_rows, const ChunkDesc* desc, const float* row_scale,
                             T* dst, int64_t ld_dst, int rows_padded, bool dst_tiled) {
  if constexpr (sizeof(T) == 2) {
    if (dst_tiled && cols % 8 == 0 && ld_src % 8 == 0 && rows_padded % 8 == 0 && reinterpret_cast<uintptr_t>(src) % 16 == 0) {
      transpose_bf16_kernel<<<grid, 256, 0, s>>>(src, ld_src, rows, cols, row_idx, ctrl, chunk_start, dyn_rows, desc, row_scale,
                                                 dst, ld_dst, rows_padded);
      return;
    }
  }
  transpose_kernel<T><<<grid, 256, 0, s>>>(src, ld_src, rows, cols, row_idx, ctrl, chunk_start, dyn_rows, desc, row_scale,
                                           dst, ld_dst, rows_padded, dst_tiled);
}

// ------------------------------------------------------------------ MFMA ceiling probe (benchmark aid)
__global__ __launch_bounds__(256) void mfma_peak_kernel(float* out, int iters, long long* clk) {
  // the hot kernel's own instruction and register blocking: 8 x 8 blocks of v_mfma_f32_16x16x32_bf16
  floatx4 acc[64];
#pragma unroll
  for (int i = 0; i < 64; ++i)
#pragma unroll
    for (int e = 0; e < 4; ++e) acc[i][e] = 0.f;
  // operands: pseudo-random bf16 values in (-1,1) (constant or small-integer operands let the part hold
  // 2.4 GHz; real data does not: it is the values that cost power)
  bf16x8 a[8], b[8];
  unsigned h = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
  for (int k = 0; k < 8; ++k)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      h = h * 1664525u + 1013904223u; a[k][e] = (bf16_t)(((int)(h >> 8) & 0xffff) * (1.f / 32768.f) - 1.f);
      h = h * 1664525u + 1013904223u; b[k][e] = (bf16_t)(((int)(h >> 8) & 0xffff) * (1.f / 32768.f) - 1.f);
    }
  const long long t0 = clock64(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 64; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i >> 3], b[i & 7], acc[i], 0, 0, 0);
  }
  const long long t1 = clock64(), w1 = wall_clock64();
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 64; ++i)
#pragma unroll
    for (int e = 0; e < 4; ++e) s += acc[i][e];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
  if (threadIdx.x == 0) { clk[blockIdx.x * 2] = t1 - t0; clk[blockIdx.x * 2 + 1] = w1 - w0; }
}

// ------------------------------------------------------------------ host side
struct Plan {
  int64_t R; int H, V, B, P; int dtype; size_t esz;
  int Tc, Vp, tiles_v, n_chunks;
  bool bwd;
  bool tiled;            // bf16: the work buffers dS/E, W^T, X^T are slab-tiled (hot kernel operands)
  bool stash;            // single-pass backward (forward keeps each chunk's unnormalised probabilities)
  int n_desc, max_len;   // stash: number of chunk records, promised bound on rows per sequence
  float inv_tau;         // 1 / temperature
  size_t off_ctrl, off_seq_len, off_cstart, off_row_map, off_ids_c, off_cpos, off_zy, off_lse_c, off_logp_c,
      off_c_c, off_adv, off_seq_loss, off_gterm, off_part, off_wt, off_xt, off_ds, off_dst,
      off_desc, off_ref, off_zsum, off_scale, off_ycol, total;
};

static inline size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

static rl_status make_plan(const rl_batch* b, const rl_params* prm, bool bwd, Plan& p) {
  if (!b) return RL_ERR_NULL;
  if (b->R < 1 || b->R >= ((int64_t)1 << 31) - (1 << 16) || b->H < 1 || b->V < 1 || b->B < 1 || b->P < 1) return RL_ERR_SHAPE;
  if (b->dtype != RL_F32 && b->dtype != RL_BF16) return RL_ERR_DTYPE;
  if (b->dtype == RL_BF16 && (b->H % 8)) return RL_ERR_SHAPE;
  if (b->dtype == RL_F32 && (b->H % 4)) return RL_ERR_SHAPE;
  p.R = b->R; p.H = b->H; p.V = b->V; p.B = b->B; p.P = b->P; p.dtype = b->dtype;
  p.esz = b->dtype == RL_BF16 ? 2 : 4;
  p.inv_tau = 1.f;
  if (prm && prm->temperature != 0.f) {
    if (!(prm->temperature > 0.f) || !(prm->temperature <= 3.0e38f)) return RL_ERR_RANGE;
    p.inv_tau = 1.f / prm->temperature;
  }
  if (prm && prm->chunk_rows < 0) return RL_ERR_SHAPE;
  const int mode = prm ? prm->backward_mode : RL_BWD_AUTO;
  if (mode != RL_BWD_AUTO && mode != RL_BWD_RECOMPUTE && mode != RL_BWD_STASH) return RL_ERR_RANGE;
  if (prm && prm->max_seq_len < 0) return RL_ERR_RANGE;
  // Single-pass backward: bf16 hot-kernel shapes only, and only when the caller bounds the sequence length by a chunk.
  const int64_t rp = (b->R + 255) & ~(int64_t)255;
  auto chunk_rows = [&](int dflt) { int t = (prm && prm->chunk_rows > 0) ? prm->chunk_rows : dflt; t = (t + 255) & ~255; return t > rp ? (int)rp : t; };
  const bool stash_kernels = b->dtype == RL_BF16 && (b->H % 128 == 0) &&
                             ((reinterpret_cast<uintptr_t>(b->hidden) | reinterpret_cast<uintptr_t>(b->weight)) % 16 == 0);
  const bool stash_shape = bwd && stash_kernels && prm && prm->max_seq_len > 0 && mode != RL_BWD_RECOMPUTE;
  const bool can_stash = stash_shape && prm->max_seq_len <= chunk_rows(kDefaultChunkRowsStash);
  if (mode == RL_BWD_STASH && !stash_kernels) return RL_ERR_UNIMPLEMENTED;
  if (mode == RL_BWD_STASH && !can_stash) return RL_ERR_RANGE;
  const int tc = chunk_rows(can_stash ? kDefaultChunkRowsStash : kDefaultChunkRows);
  p.Tc = tc;
  p.Vp = (b->V + kBM - 1) / kBM * kBM;
  p.tiles_v = p.Vp / kBM;
  p.n_chunks = (int)((b->R + tc - 1) / tc);
  p.bwd = bwd;
  p.tiled = (b->dtype == RL_BF16);
  p.stash = can_stash;
  p.max_len = p.stash ? prm->max_seq_len : 0;
  // chunk records: two consecutive chunks hold more than Tc rows, and every chunk but the last more than Tc - max_len
  p.n_desc = 2 * p.n_chunks + 1;
  if (p.stash && p.max_len < tc) {
    const int64_t alt = (b->R + (tc - p.max_len)) / (tc - p.max_len + 1) + 1;
    if (alt < p.n_desc) p.n_desc = (int)alt;
  }
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o += up256(bytes); return at; };
  const size_t Rp = (size_t)rp + 256;
  p.off_ctrl = take(sizeof(Ctrl));
  p.off_seq_len = take(sizeof(int32_t) * (size_t)b->B);
  p.off_cstart = take(sizeof(int32_t) * ((size_t)b->B + 1));
  p.off_row_map = take(4 * Rp); p.off_ids_c = take(4 * Rp); p.off_cpos = take(4 * Rp);
  p.off_zy = take(4 * Rp); p.off_lse_c = take(4 * Rp); p.off_logp_c = take(4 * Rp); p.off_c_c = take(4 * Rp);
  p.off_ycol = take(4 * Rp);
  p.off_adv = take(4 * (size_t)b->B); p.off_seq_loss = take(4 * (size_t)b->B); p.off_gterm = take(4 * (size_t)b->B);
  p.off_part = take(sizeof(float4) * (size_t)p.tiles_v * (size_t)tc);
  p.off_wt = p.off_xt = p.off_ds = p.off_dst = 0;
  if (bwd) {
    const size_t Hp = ((size_t)b->H + 255) & ~(size_t)255;   // tiled layouts come in blocks of 256 rows
    p.off_wt = take(p.esz * Hp * (size_t)p.Vp);
    p.off_xt = take(p.esz * Hp * (size_t)tc);
    p.off_ds = take(p.esz * (size_t)tc * (size_t)p.Vp);
    if (b->dtype == RL_F32) p.off_dst = take(p.esz * (size_t)p.Vp * (size_t)tc);   // bf16: dW reads dS / E itself
  }
  p.off_desc = p.off_ref = p.off_zsum = p.off_scale = 0;
  if (p.stash) {
    p.off_desc = take(sizeof(ChunkDesc) * (size_t)p.n_desc);
    p.off_ref = take(4 * Rp); p.off_zsum = take(4 * Rp); p.off_scale = take(4 * (size_t)tc);
  }
  p.total = o;
  return RL_OK;
}

// The bf16 hot kernel needs an even number of whole 64-element slabs and 16-byte aligned rows; anything else (f32
// inputs, ragged K) takes the generic kernel.
template <class T, class Epi>
static void launch_generic(const T* A, const T* B, const GemmDims& d, const Epi& epi, int tiles, hipStream_t s) {
  auto kern = gemm_nt_kernel<T, Epi, kBM, kBN, kWavesM, kWavesN>;
  // 128 KiB of dynamic LDS needs the opt-in on every device the caller may be on: set on each launch (a host-side table
  // update, no device work) rather than remembered in a flag that is neither per device nor thread-safe
  (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, kGemmSmem);
  kern<<<tiles, kGemmThreads, kGemmSmem, s>>>(A, B, d, epi);
}

template <class Tune, class Epi>
static void launch_gemm(const bf16_t* A, const bf16_t* B, const GemmDims& d, const Epi& epi, hipStream_t s) {
  const int tiles = launch_tiles((d.M + kBM - 1) / kBM, (d.N + kBN - 1) / kBN);
  const bool fast = (d.K % 128 == 0) && (d.lda % 8 == 0) && (d.ldb % 8 == 0) &&
                    ((reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B)) % 16 == 0) &&
                    !d.a_rows && (d.b_rows != nullptr) == Epi::kGatherB;     // (how the hot kernel addresses its operands)
  if (!fast) { launch_generic<bf16_t, Epi>(A, B, d, epi, tiles, s); return; }
  gemm_nt_bf16_kernel<Epi, Tune><<<tiles, 256, 0, s>>>(A, B, d, epi);
}

template <class Tune, class Epi>
static void launch_gemm(const float* A, const float* B, const GemmDims& d, const Epi& epi, hipStream_t s) {
  const int tiles = launch_tiles((d.M + kBM - 1) / kBM, (d.N + kBN - 1) / kBN);
  launch_generic<float, Epi>(A, B, d, epi, tiles, s);
}

// Weight-gradient contraction of the recompute mode: bf16 reads dS (K-major A operand), f32 its stored transpose.
static void launch_dw(const bf16_t* dS, const bf16_t*, const bf16_t* XT, const GemmDims& d, const EpiDW& epi, hipStream_t s) {
  const int tiles = launch_tiles((d.M + kBM - 1) / kBM, (d.N + kBN - 1) / kBN);
  gemm_nt_bf16_kernel<EpiDW, TuneDW, true><<<tiles, 256, 0, s>>>(dS, XT, d, epi);
}
static void launch_dw(const float*, const float* dST, const float* XT, const GemmDims& d, const EpiDW& epi, hipStream_t s) {
  launch_gemm<TuneDW>(dST, XT, d, epi, s);
}

struct Ptrs {
  Ctrl* ctrl; int32_t *seq_len, *cstart, *row_map, *ids_c, *cpos;
  float *zy, *lse_c, *logp_c, *c_c, *adv, *seq_loss, *gterm; float4* part;
  void *wt, *xt, *ds, *dst;
  ChunkDesc* desc; float *ref, *zsum, *scale;
  int32_t* ycol;
};

static Ptrs carve(void* ws, const Plan& p) {
  unsigned char* w = static_cast<unsigned char*>(ws);
  Ptrs q;
  q.ctrl = (Ctrl*)(w + p.off_ctrl); q.seq_len = (int32_t*)(w + p.off_seq_len); q.cstart = (int32_t*)(w + p.off_cstart);
  q.row_map = (int32_t*)(w + p.off_row_map); q.ids_c = (int32_t*)(w + p.off_ids_c); q.cpos = (int32_t*)(w + p.off_cpos);
  q.zy = (float*)(w + p.off_zy); q.lse_c = (float*)(w + p.off_lse_c); q.logp_c = (float*)(w + p.off_logp_c);
  q.c_c = (float*)(w + p.off_c_c); q.adv = (float*)(w + p.off_adv); q.seq_loss = (float*)(w + p.off_seq_loss);
  q.gterm = (float*)(w + p.off_gterm); q.part = (float4*)(w + p.off_part);
  q.wt = w + p.off_wt; q.xt = w + p.off_xt; q.ds = w + p.off_ds;
  q.dst = p.off_dst ? w + p.off_dst : nullptr;          // f32 inputs only
  q.desc = (ChunkDesc*)(w + p.off_desc); q.ref = (float*)(w + p.off_ref); q.zsum = (float*)(w + p.off_zsum);
  q.scale = (float*)(w + p.off_scale);
  q.ycol = (int32_t*)(w + p.off_ycol);
  return q;
}

// prep: counts, scan, compaction; zero the per-row outputs so masked rows read 0
static void run_prep(const rl_batch* b, const Plan& p, const Ptrs& q, int32_t* seq_len_out, rl_stats* stats,
                     const int32_t* group_idx, float* logp_out, float* lse_out, float* coeff_out, int32_t* row_map_out,
                     hipStream_t s) {
  ProfScope ps(RL_PROF_PREP, s);
  if (stats) fill<int32_t>(reinterpret_cast<int32_t*>(stats), sizeof(rl_stats) / 4, 0, s);
  fill<int32_t>(q.cpos, p.R, -1, s);
  fill<int32_t>(row_map_out, p.R, -1, s);
  fill<float>(logp_out, p.R, 0.f, s); fill<float>(lse_out, p.R, 0.f, s); fill<float>(coeff_out, p.R, 0.f, s);
  // the running maximum of the offsets borrows cstart until the scan below overwrites it with the compacted starts
  cu_running_max_kernel<<<1, 1024, 0, s>>>(b->cu_seqlens, p.B, q.cstart);
  seq_count_kernel<<<p.B, 256, 0, s>>>(b->mask, b->token_ids, b->cu_seqlens, q.cstart, group_idx, p.R, p.V, p.P, q.seq_len, stats);
  seq_scan_kernel<<<1, 1024, 0, s>>>(q.seq_len, p.B, q.cstart, q.ctrl, stats);
  compact_kernel<<<p.B, 1024, 0, s>>>(b->mask, b->token_ids, b->cu_seqlens, q.seq_len, q.cstart, p.V, q.row_map, q.ids_c, q.cpos,
                                      row_map_out);
  if (seq_len_out) (void)hipMemcpyAsync(seq_len_out, q.seq_len, 4 * (size_t)p.B, hipMemcpyDeviceToDevice, s);
}

template <class T>
static void run_forward(const rl_batch* b, const Plan& p, const Ptrs& q, float* logp_out, float* lse_out, float* ent_out,
                        float* zy_out, int32_t* ycol_out, hipStream_t s) {
  const T* X = static_cast<const T*>(b->hidden);
  const T* W = static_cast<const T*>(b->weight);
  for (int ch = 0; ch < p.n_chunks; ++ch) {
    const int c0 = ch * p.Tc;
    GemmDims d{};
    d.M = p.V; d.N = p.Tc; d.K = p.H; d.lda = p.H; d.ldb = p.H;
    d.a_rows = nullptr; d.b_rows = q.row_map + c0; d.n_real = &q.ctrl->n_real; d.chunk_start = c0; d.dyn = 2; d.group_m = TuneLogits::kBand;
    EpiFwd<T> e{q.ids_c, q.zy, q.part, p.Tc, p.V, p.inv_tau, q.ycol};
    { ProfScope ps(RL_PROF_GEMM_FWD, s); launch_gemm<TuneLogits>(W, X, d, e, s); }
    ProfScope ps(RL_PROF_COMBINE, s);
    lse_combine_kernel<<<(p.Tc + 63) / 64, 256, 0, s>>>(q.part, p.Tc, p.tiles_v, q.zy, q.row_map, q.ctrl, c0, p.Tc, q.ycol,
                                                        q.lse_c, q.logp_c, lse_out, logp_out, ent_out, zy_out, ycol_out);
  }
}

template <class T>
static void run_backward(const rl_batch* b, const Plan& p, const Ptrs& q, void* d_hidden, float* d_weight, hipStream_t s) {
  const T* X = static_cast<const T*>(b->hidden);
  const T* W = static_cast<const T*>(b->weight);
  T* WT = static_cast<T*>(q.wt); T* XT = static_cast<T*>(q.xt);
  T* dS = static_cast<T*>(q.ds); T* dST = static_cast<T*>(q.dst);
  T* dX = static_cast<T*>(d_hidden);
  // masked rows of dX are zero; rows that count are written by the dX epilogue
  {
    ProfScope ps(RL_PROF_TRANSPOSE, s);
    const int rows_per_block = 4;
    zero_masked_rows_kernel<T><<<(unsigned)((p.R + rows_per_block - 1) / rows_per_block), 256, 0, s>>>(q.cpos, dX, p.R, p.H);
  }
  // W^T [H][Vp] with zero padding columns, once per call
  {
    ProfScope ps(RL_PROF_TRANSPOSE, s);
    dim3 g((p.Vp + 63) / 64, (p.H + 63) / 64);
    launch_transpose<T>(g, s, W, p.H, p.V, p.H, nullptr, q.ctrl, 0, 0, nullptr, nullptr, WT, p.Vp, p.Vp, p.tiled);
  }
  for (int ch = 0; ch < p.n_chunks; ++ch) {
    const int c0 = ch * p.Tc;
    {  // X^T chunk [H][Tc], gathered through row_map, zero beyond the valid rows
      ProfScope ps(RL_PROF_TRANSPOSE, s);
      dim3 g((p.Tc + 63) / 64, (p.H + 63) / 64);
      launch_transpose<T>(g, s, X, p.H, p.Tc, p.H, q.row_map, q.ctrl, c0, 1, nullptr, nullptr, XT, p.Tc, p.Tc, p.tiled);
    }
    {  // recompute logits, form dS (and dS^T for f32 inputs)
      GemmDims d{};
      d.M = p.V; d.N = p.Tc; d.K = p.H; d.lda = p.H; d.ldb = p.H;
      d.b_rows = q.row_map + c0; d.n_real = &q.ctrl->n_real; d.chunk_start = c0; d.dyn = 2; d.group_m = TuneLogits::kBand;
      EpiDS<T> e{q.ids_c, q.lse_c, q.c_c, dS, p.Vp, dST, p.Tc, p.V, p.tiled, p.inv_tau};
      ProfScope ps(RL_PROF_GEMM_DS, s);
      launch_gemm<TuneLogits>(W, X, d, e, s);
    }
    {  // dX = dS W  : A = dS [Tc][Vp], B = W^T [H][Vp]
      GemmDims d{};
      d.M = p.Tc; d.N = p.H; d.K = p.Vp; d.lda = p.Vp; d.ldb = p.Vp;
      d.n_real = &q.ctrl->n_real; d.chunk_start = c0; d.dyn = 1; d.group_m = TuneDX::kBand; d.a_tiled = d.b_tiled = p.tiled;
      EpiDX<T> e{q.row_map, dX, p.H, p.H, nullptr};
      ProfScope ps(RL_PROF_GEMM_DX, s);
      launch_gemm<TuneDX>(dS, WT, d, e, s);
    }
    {  // dW (+)= dS^T X : B = X^T [H][Tc]; A = dS^T, for bf16 read out of dS itself as a K-major operand
       // (K = Tc is a multiple of 256 and the workspace is aligned: always the hot kernel), for f32 the stored copy [Vp][Tc]
      GemmDims d{};
      d.M = p.V; d.N = p.H; d.K = p.Tc; d.lda = p.tiled ? p.Vp : p.Tc; d.ldb = p.Tc;
      d.n_real = &q.ctrl->n_real; d.chunk_start = c0; d.dyn = 3; d.group_m = TuneDW::kBand; d.a_tiled = d.b_tiled = p.tiled;
      d.zero_if_empty = (ch == 0);
      EpiDW e{d_weight, p.H, p.V, p.H, ch > 0 ? 1 : 0};
      ProfScope ps(RL_PROF_GEMM_DW, s);
      launch_dw(dS, dST, XT, d, e, s);
    }
  }
}

static LossOpts loss_opts(const rl_params* prm) {
  LossOpts o;
  o.clip_lo = prm->clip_eps;
  o.clip_hi = prm->clip_eps_high > 0.f ? prm->clip_eps_high : prm->clip_eps;
  o.kl_coef = prm->kl_coef; o.beta = prm->beta;
  o.token_agg = prm->aggregation == RL_AGG_TOKEN;
  o.seq_ratio = prm->ratio_level == RL_RATIO_SEQUENCE;
  o.w_mean = prm->flow_weight_norm == RL_WNORM_MEAN;
  return o;
}

// Single-pass variant of forward + loss + backward (bf16 hot kernels): chunks are made of whole
// sequences, so each chunk's loss coefficients are known as soon as its forward is; the forward
// keeps the chunk's unnormalised probabilities E and the backward contractions run on
// them directly: dX = diag(-c/Z) E' W and dW += E'^T diag(-c/Z) X, E' = E with the target entry
// patched (E' is the row-major A operand of the first and the K-major A operand of the second).  Three contractions per chunk instead of four; T x V is still never held, only Tc x V.
static void run_fused(const rl_batch* b, const rl_params* prm, int objective, const Plan& p, const Ptrs& q,
                      const rl_outputs* out, hipStream_t s) {
  typedef bf16_t T;
  const T* X = static_cast<const T*>(b->hidden);
  const T* W = static_cast<const T*>(b->weight);
  T* WT = static_cast<T*>(q.wt); T* XT = static_cast<T*>(q.xt);
  T* E = static_cast<T*>(q.ds);
  T* dX = static_cast<T*>(out->d_hidden);
  {
    ProfScope ps(RL_PROF_TRANSPOSE, s);
    const int rows_per_block = 4;
    zero_masked_rows_kernel<T><<<(unsigned)((p.R + rows_per_block - 1) / rows_per_block), 256, 0, s>>>(q.cpos, dX, p.R, p.H);
    dim3 g((p.Vp + 63) / 64, (p.H + 63) / 64);
    launch_transpose<T>(g, s, W, p.H, p.V, p.H, nullptr, q.ctrl, 0, 0, nullptr, nullptr, WT, p.Vp, p.Vp, p.tiled);
  }
  {
    ProfScope ps(RL_PROF_PREP, s);
    chunk_build_kernel<<<1, 64, 0, s>>>(q.seq_len, q.cstart, p.B, p.Tc, p.max_len, q.desc, p.n_desc, q.ctrl, out->stats);
    target_logit_kernel<<<(unsigned)((p.R + 3) / 4), 256, 0, s>>>(X, W, p.H, q.row_map, q.ids_c, b->old_logprob, q.ctrl, p.inv_tau, q.zy, q.ref, q.ycol);
  }
  float2* part = reinterpret_cast<float2*>(q.part);
  for (int k = 0; k < p.n_desc; ++k) {
    const ChunkDesc* dk = q.desc + k;
    const int* chunk = &dk->row_start;
    {  // forward: partial sums + E
      GemmDims d{};
      d.M = p.V; d.N = p.Tc; d.K = p.H; d.lda = p.H; d.ldb = p.H;
      d.b_rows = q.row_map; d.chunk = chunk; d.dyn = 2; d.group_m = TuneLogits::kBand;
      EpiFwdStash<T> e{q.ref, part, p.Tc, E, p.Vp, p.V, p.inv_tau};
      ProfScope ps(RL_PROF_GEMM_FWD, s);
      gemm_nt_bf16_kernel<EpiFwdStash<T>, TuneLogits>
          <<<launch_tiles((p.V + kBM - 1) / kBM, (p.Tc + kBN - 1) / kBN), 256, 0, s>>>(W, X, d, e);
    }
    {
      ProfScope ps(RL_PROF_COMBINE, s);
      lse_sum_kernel<<<(p.Tc + 63) / 64, 64 * kSumSlices, 0, s>>>(part, p.Tc, p.tiles_v, q.zy, q.ref, q.row_map, dk, q.ycol, q.ctrl, out->stats,
                                                      q.lse_c, q.logp_c, q.zsum, out->lse, out->logprob, out->entropy,
                                                      out->target_logit, out->target_col);
    }
    {
      ProfScope ps(RL_PROF_LOSS, s);
      seq_loss_kernel<<<p.B, 256, 0, s>>>(objective, q.logp_c, b->old_logprob, b->ref_logprob, q.row_map, q.cstart, q.adv,
                                         b->group_idx, b->log_z, p.B, loss_opts(prm), q.ctrl,
                                         q.seq_loss, q.gterm, q.c_c, out->coeff, out->stats, dk);
      stash_patch_kernel<T><<<(p.Tc + 255) / 256, 256, 0, s>>>(dk, q.ids_c, q.zy, q.ref, q.zsum, q.c_c, p.inv_tau, q.scale, E, p.Vp);
    }
    {  // X^T chunk scaled by -c/Z, zero beyond the valid rows
      ProfScope ps(RL_PROF_TRANSPOSE, s);
      dim3 g((p.Tc + 63) / 64, (p.H + 63) / 64);
      launch_transpose<T>(g, s, X, p.H, p.Tc, p.H, q.row_map, q.ctrl, 0, 1, dk, q.scale, XT, p.Tc, p.Tc, true);
    }
    {  // dX = diag(-c/Z) E' W  (A = E' [Tc][Vp], B = W^T [H][Vp]) and dW (+)= E'^T (diag(-c/Z) X)  (A = E'^T, read out
       // of E' itself as a K-major operand; B = scaled X^T [H][Tc]) in one launch: dX alone has too few (long) tiles
       // to fill its last round of CUs
      GemmDims dx{};
      dx.M = p.Tc; dx.N = p.H; dx.K = p.Vp; dx.lda = p.Vp; dx.ldb = p.Vp;
      dx.chunk = chunk; dx.dyn = 1; dx.group_m = TuneDX::kBand; dx.a_tiled = dx.b_tiled = 1;
      EpiDX<T> ex{q.row_map, dX, p.H, p.H, q.scale};
      GemmDims dw{};
      dw.M = p.V; dw.N = p.H; dw.K = p.Tc; dw.lda = p.Vp; dw.ldb = p.Tc;
      dw.chunk = chunk; dw.dyn = 3; dw.zero_if_empty = (k == 0); dw.group_m = TuneDW::kBand; dw.a_tiled = dw.b_tiled = 1;
      EpiDW ew{out->d_weight, p.H, p.V, p.H, k > 0 ? 1 : 0};
      const int tn = (p.H + kBN - 1) / kBN;
      const int n1 = launch_tiles((p.Tc + kBM - 1) / kBM, tn);
      const int n2 = launch_tiles((p.V + kBM - 1) / kBM, tn);
      ProfScope ps(RL_PROF_GEMM_BWD, s);
      gemm_nt_bf16_pair_kernel<EpiDX<T>, TuneDX, EpiDW, TuneDW, true>
          <<<n1 + n2, 256, 0, s>>>(E, WT, dx, ex, n1, E, XT, dw, ew);
    }
  }
  ProfScope ps(RL_PROF_LOSS, s);
  finalize_kernel<<<1, 1024, 0, s>>>(q.seq_loss, q.gterm, b->group_idx, q.seq_len, p.B, p.P, objective, q.ctrl,
                                    out->loss, out->d_log_z, out->seq_loss);
}

static rl_status check_ws(void* ws, size_t bytes, const Plan& p) {
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255) || bytes < p.total) return RL_ERR_WORKSPACE;
  return RL_OK;
}

}  // namespace rlk

using namespace rlk;

extern "C" {

const char* rl_status_string(int32_t s) {
  switch (s) {
    case RL_OK: return "ok";
    case RL_ERR_NULL: return "a required pointer is NULL";
    case RL_ERR_SHAPE: return "a size is non-positive, too large or misaligned";
    case RL_ERR_DTYPE: return "unknown dtype";
    case RL_ERR_RANGE: return "objective or a coefficient is out of range";
    case RL_ERR_WORKSPACE: return "workspace is NULL, misaligned or too small";
    case RL_ERR_HIP: return "a HIP launch failed";
    case RL_ERR_UNIMPLEMENTED: return "this build has no kernel for the request (single-pass backward needs bf16 inputs and H % 128 == 0)";
    default: return "unknown status";
  }
}

void rl_profile_enable(int32_t on) { g_prof.on = (on != 0); }

rl_status rl_profile_read(rl_profile* out) {
  if (!out) return RL_ERR_NULL;
  memset(out, 0, sizeof(*out));
  rl_status st = RL_OK;
  for (const ProfRec& r : g_prof.recs) {
    float ms = 0.f;
    if (hipEventSynchronize(r.b) != hipSuccess || hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) st = RL_ERR_HIP;
    else if (r.cls >= 0 && r.cls < RL_PROF_CLASSES) { out->ms[r.cls] += (double)ms; out->launches[r.cls] += 1; }
    g_prof.pool.push_back({r.a, r.b});
  }
  g_prof.recs.clear();
  return st;
}

int32_t rl_version(void) { return 107; }
int32_t rl_default_chunk_rows(void) { return kDefaultChunkRows; }
int32_t rl_default_chunk_rows_single_pass(void) { return kDefaultChunkRowsStash; }

rl_status rl_measure_mfma_peak(int32_t millis, void* scratch, size_t scratch_bytes, void* stream,
                               double* tflops, double* shader_mhz) {
  if (!scratch || !tflops || !shader_mhz) return RL_ERR_NULL;
  if (millis < 1 || millis > 5000) return RL_ERR_RANGE;
  constexpr int kBlocks = 1024;                                   // 4 workgroups of 4 wavefronts per CU
  if (scratch_bytes < (size_t)kBlocks * 256 * 4 + (size_t)kBlocks * 16 || (reinterpret_cast<uintptr_t>(scratch) & 15)) return RL_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  float* out = static_cast<float*>(scratch);
  long long* clk = reinterpret_cast<long long*>(out + kBlocks * 256);
  // one launch of `iters` rounds of 64 MFMAs per wavefront: ~16 cycles per MFMA, 4 workgroups share a CU
  const double cycles_per_round = 64.0 * 16.0 * 4.0;
  int iters = (int)(millis * 1e-3 * 2.0e9 / cycles_per_round);
  if (iters < 16) iters = 16;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return RL_ERR_HIP;
  mfma_peak_kernel<<<kBlocks, 256, 0, s>>>(out, 16, clk);        // warm-up
  (void)hipEventRecord(e0, s);
  mfma_peak_kernel<<<kBlocks, 256, 0, s>>>(out, iters, clk);
  (void)hipEventRecord(e1, s);
  rl_status st = RL_OK;
  float ms = 0.f;
  if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess || ms <= 0.f) st = RL_ERR_HIP;
  long long h[2] = {0, 0};
  if (st == RL_OK && hipMemcpy(h, clk, sizeof(h), hipMemcpyDeviceToHost) != hipSuccess) st = RL_ERR_HIP;
  (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
  if (st != RL_OK) return st;
  *tflops = (double)kBlocks * 4.0 * iters * 64.0 * 16384.0 / (ms * 1e-3) / 1e12;
  *shader_mhz = h[1] > 0 ? 100.0 * (double)h[0] / (double)h[1] : 0.0;   // wall clock ticks at 100 MHz
  return RL_OK;
}

rl_status rl_debug_tile_order(int32_t tiles_m, int32_t tiles_n, int32_t group_m, int32_t by_share,
                              int32_t* workgroups, int32_t* tile) {
  if (!workgroups) return RL_ERR_NULL;
  if (tiles_m < 1 || tiles_n < 1 || group_m < 1 || (int64_t)tiles_m * tiles_n > (1 << 24)) return RL_ERR_SHAPE;
  const int n = launch_tiles(tiles_m, tiles_n);
  *workgroups = n;
  if (!tile) return RL_OK;
  for (int w = 0; w < n; ++w) {
    int tm = -1, tn = -1;
    if (!tile_of_block(w, tiles_m, tiles_n, group_m, by_share != 0, tm, tn)) tm = tn = -1;
    tile[2 * w] = tm; tile[2 * w + 1] = tn;
  }
  return RL_OK;
}

rl_status rl_workspace_bytes(const rl_batch* batch, const rl_params* params, int32_t want_backward, size_t* bytes) {
  if (!batch || !bytes) return RL_ERR_NULL;
  Plan p;
  rl_status st = make_plan(batch, params, want_backward != 0, p);
  if (st != RL_OK) return st;
  *bytes = p.total;
  return RL_OK;
}

rl_status rl_token_logprob(const rl_batch* b, float* logprob, float* lse, void* ws, size_t ws_bytes, void* stream) {
  return rl_token_logprob_tempered(b, 1.f, logprob, lse, ws, ws_bytes, stream);
}

rl_status rl_token_logprob_tempered(const rl_batch* b, float temperature, float* logprob, float* lse,
                                    void* ws, size_t ws_bytes, void* stream) {
  if (!b) return RL_ERR_NULL;
  if (!b->hidden || !b->weight || !b->token_ids || !b->mask || !b->cu_seqlens) return RL_ERR_NULL;
  if (!logprob && !lse) return RL_ERR_NULL;
  if (!(temperature > 0.f) || !(temperature <= 3.0e38f)) return RL_ERR_RANGE;
  Plan p;
  rl_status st = make_plan(b, nullptr, false, p);
  if (st != RL_OK) return st;
  p.inv_tau = 1.f / temperature;
  st = check_ws(ws, ws_bytes, p);
  if (st != RL_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  (void)hipGetLastError();
  Ptrs q = carve(ws, p);
  run_prep(b, p, q, nullptr, nullptr, nullptr, logprob, lse, nullptr, nullptr, s);
  if (p.dtype == RL_BF16) run_forward<bf16_t>(b, p, q, logprob, lse, nullptr, nullptr, nullptr, s);
  else run_forward<float>(b, p, q, logprob, lse, nullptr, nullptr, nullptr, s);
  return hipGetLastError() == hipSuccess ? RL_OK : RL_ERR_HIP;
}

rl_status rl_policy_loss_fwd_bwd(const rl_batch* b, const rl_params* prm, int32_t objective, const rl_outputs* out,
                                 void* ws, size_t ws_bytes, void* stream) {
  if (!b || !prm || !out) return RL_ERR_NULL;
  if (!b->hidden || !b->weight || !b->token_ids || !b->mask || !b->cu_seqlens || !b->group_idx || !b->rewards ||
      !b->old_logprob || !b->ref_logprob || !out->loss)
    return RL_ERR_NULL;
  if (objective != RL_OBJ_GRPO && objective != RL_OBJ_FLOW) return RL_ERR_RANGE;
  if (objective == RL_OBJ_FLOW && !b->log_z) return RL_ERR_NULL;
  if (!(prm->clip_eps > 0.f && prm->clip_eps < 1.f)) return RL_ERR_RANGE;
  if (prm->adv_std_ddof != 0 && prm->adv_std_ddof != 1) return RL_ERR_RANGE;
  if (!(prm->adv_eps >= 0.f)) return RL_ERR_RANGE;
  if (!(prm->clip_eps_high >= 0.f)) return RL_ERR_RANGE;
  if ((prm->aggregation != RL_AGG_SEQUENCE && prm->aggregation != RL_AGG_TOKEN) ||
      (prm->ratio_level != RL_RATIO_TOKEN && prm->ratio_level != RL_RATIO_SEQUENCE) ||
      (prm->flow_weight_norm != RL_WNORM_SUM && prm->flow_weight_norm != RL_WNORM_MEAN))
    return RL_ERR_RANGE;
  if (prm->ratio_level == RL_RATIO_SEQUENCE && prm->aggregation == RL_AGG_TOKEN) return RL_ERR_RANGE;
  const bool bwd = out->d_hidden || out->d_weight;
  if (bwd && (!out->d_hidden || !out->d_weight)) return RL_ERR_NULL;
  Plan p;
  rl_status st = make_plan(b, prm, bwd, p);
  if (st != RL_OK) return st;
  st = check_ws(ws, ws_bytes, p);
  if (st != RL_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  (void)hipGetLastError();
  Ptrs q = carve(ws, p);

  run_prep(b, p, q, out->seq_len, out->stats, b->group_idx, out->logprob, out->lse, out->coeff, out->row_map, s);
  fill<float>(out->entropy, p.R, 0.f, s);
  fill<float>(out->target_logit, p.R, 0.f, s);
  fill<int32_t>(out->target_col, p.R, -1, s);
  {
  ProfScope ps(RL_PROF_LOSS, s);
  fill<float>(q.adv, p.B, 0.f, s);
  advantage_kernel<<<(p.P + 127) / 128, 128, 0, s>>>(b->rewards, b->group_idx, p.B, p.P, prm->adv_eps, prm->adv_std_ddof, q.adv, out->group_count);
  if (out->advantages) (void)hipMemcpyAsync(out->advantages, q.adv, 4 * (size_t)p.B, hipMemcpyDeviceToDevice, s);
  }

  if (p.stash) {
    run_fused(b, prm, objective, p, q, out, s);
    return hipGetLastError() == hipSuccess ? RL_OK : RL_ERR_HIP;
  }
  if (p.dtype == RL_BF16) run_forward<bf16_t>(b, p, q, out->logprob, out->lse, out->entropy, out->target_logit, out->target_col, s);
  else run_forward<float>(b, p, q, out->logprob, out->lse, out->entropy, out->target_logit, out->target_col, s);

  {
  ProfScope ps(RL_PROF_LOSS, s);
  seq_loss_kernel<<<p.B, 256, 0, s>>>(objective, q.logp_c, b->old_logprob, b->ref_logprob, q.row_map, q.cstart, q.adv,
                                     b->group_idx, b->log_z, p.B, loss_opts(prm), q.ctrl,
                                     q.seq_loss, q.gterm, q.c_c, out->coeff, out->stats, nullptr);
  finalize_kernel<<<1, 1024, 0, s>>>(q.seq_loss, q.gterm, b->group_idx, q.seq_len, p.B, p.P, objective, q.ctrl,
                                    out->loss, out->d_log_z, out->seq_loss);
  }
  if (bwd) {
    if (p.dtype == RL_BF16) run_backward<bf16_t>(b, p, q, out->d_hidden, out->d_weight, s);
    else run_backward<float>(b, p, q, out->d_hidden, out->d_weight, s);
  }
  return hipGetLastError() == hipSuccess ? RL_OK : RL_ERR_HIP;
}

// ------------------------------------------------------------------ scoring call that allocates nothing
// The forward-only call with its workspace in a file-scope device array instead of a caller's buffer.  Every GPU the
// library runs on holds its own copy of the array at its own address; the host-side name of the array is only a handle
// for hipGetSymbolAddress, never a device address, so the address is looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[RL_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mutex;

static rl_status static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return RL_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return RL_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return RL_OK;
}

rl_status rl_token_logprob_static(const rl_batch* b, float temperature, float* logprob, float* lse, void* stream) {
  if (!b) return RL_ERR_NULL;
  if (!b->hidden || !b->weight || !b->token_ids || !b->mask || !b->cu_seqlens) return RL_ERR_NULL;
  if (!logprob && !lse) return RL_ERR_NULL;
  if (!(temperature > 0.f) || !(temperature <= 3.0e38f)) return RL_ERR_RANGE;
  // the largest chunk (a power of two times 256 rows) whose plan fits the array; none fits: the batch is beyond the limit
  Plan p;
  bool fits = false;
  for (int tc = kDefaultChunkRows; tc >= 256 && !fits; tc >>= 1) {
    rl_params prm{};
    prm.chunk_rows = tc;
    const rl_status st = make_plan(b, &prm, false, p);
    if (st != RL_OK) return st;
    fits = p.total <= (size_t)RL_STATIC_SCRATCH_BYTES;
  }
  if (!fits) return RL_ERR_WORKSPACE;
  p.inv_tau = 1.f / temperature;
  void* ws = nullptr;
  const rl_status st = static_scratch(&ws);
  if (st != RL_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  (void)hipGetLastError();
  Ptrs q = carve(ws, p);
  run_prep(b, p, q, nullptr, nullptr, nullptr, logprob, lse, nullptr, nullptr, s);
  if (p.dtype == RL_BF16) run_forward<bf16_t>(b, p, q, logprob, lse, nullptr, nullptr, nullptr, s);
  else run_forward<float>(b, p, q, logprob, lse, nullptr, nullptr, nullptr, s);
  return hipGetLastError() == hipSuccess ? RL_OK : RL_ERR_HIP;
}

// ------------------------------------------------------------------ log-Z head
static rl_status logz_check(int32_t P, int32_t H, int32_t M) {
  if (P < 1 || H < 1 || M < 1 || P > (1 << 20) || (int64_t)((M + 7) / 8) > 65535) return RL_ERR_SHAPE;
  return RL_OK;
}

rl_status rl_logz_head_workspace_bytes(int32_t P, int32_t H, int32_t M, size_t* bytes) {
  if (!bytes) return RL_ERR_NULL;
  rl_status st = logz_check(P, H, M);
  if (st != RL_OK) return st;
  *bytes = logz_plan(P, H, M).total;
  return RL_OK;
}

rl_status rl_logz_head_forward(const void* prompt_hidden, int32_t dtype, int64_t rows, int32_t H,
                               const int32_t* cu_prompt, int32_t P, const float* W1, const float* b1,
                               const float* w2, const float* b2, int32_t M, float* log_z,
                               void* ws, size_t ws_bytes, void* stream) {
  if (!prompt_hidden || !cu_prompt || !W1 || !b1 || !w2 || !b2 || !log_z) return RL_ERR_NULL;
  if (dtype != RL_F32 && dtype != RL_BF16) return RL_ERR_DTYPE;
  rl_status st = logz_check(P, H, M);
  if (st != RL_OK) return st;
  if (rows < 0) return RL_ERR_SHAPE;
  const LogzPlan q = logz_plan(P, H, M);
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255) || ws_bytes < q.total) return RL_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  (void)hipGetLastError();
  unsigned char* w = static_cast<unsigned char*>(ws);
  float* pooled = (float*)(w + q.off_pooled); float* a = (float*)(w + q.off_a); float* g = (float*)(w + q.off_g);
  dim3 gp(P, (H + 63) / 64);
  if (dtype == RL_BF16) logz_pool_kernel<bf16_t><<<gp, 256, 0, s>>>(static_cast<const bf16_t*>(prompt_hidden), rows, H, cu_prompt, pooled);
  else logz_pool_kernel<float><<<gp, 256, 0, s>>>(static_cast<const float*>(prompt_hidden), rows, H, cu_prompt, pooled);
  dim3 gh((M + 15) / 16, (P + 15) / 16);
  logz_hidden_kernel<<<gh, 256, 0, s>>>(W1, b1, pooled, P, H, M, a, g);
  logz_out_kernel<<<P, 256, 0, s>>>(g, w2, b2, M, log_z);
  return hipGetLastError() == hipSuccess ? RL_OK : RL_ERR_HIP;
}

rl_status rl_logz_head_backward(const float* d_log_z, int32_t P, int32_t H, int32_t M, const float* w2,
                                float* dW1, float* db1, float* dw2, float* db2,
                                void* ws, size_t ws_bytes, void* stream) {
  if (!d_log_z || !w2 || !dW1 || !db1 || !dw2 || !db2) return RL_ERR_NULL;
  rl_status st = logz_check(P, H, M);
  if (st != RL_OK) return st;
  const LogzPlan q = logz_plan(P, H, M);
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255) || ws_bytes < q.total) return RL_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  (void)hipGetLastError();
  unsigned char* w = static_cast<unsigned char*>(ws);
  float* pooled = (float*)(w + q.off_pooled); float* a = (float*)(w + q.off_a); float* g = (float*)(w + q.off_g);
  float* da = (float*)(w + q.off_da);
  logz_bwd_vec_kernel<<<(M + 255) / 256, 256, 0, s>>>(d_log_z, a, g, w2, P, M, da, db1, dw2, db2);
  dim3 gw((H + 255) / 256, (M + 7) / 8);
  logz_bwd_w1_kernel<<<gw, 256, 0, s>>>(da, pooled, P, M, H, dW1);
  return hipGetLastError() == hipSuccess ? RL_OK : RL_ERR_HIP;
}

// ------------------------------------------------------------------ residual-VQ encode
static rl_status rvq_check(int32_t G, int64_t L, int32_t D, int32_t N, int32_t S) {
  if (G < 1 || G > 65535 || L < 1 || L > ((int64_t)1 << 24) || N < 1 || S < 1) return RL_ERR_SHAPE;
  if (D != kRvqD || (S % kRvqChunk) != 0 || S > 65536 || (int64_t)N * S > ((int64_t)1 << 26)) return RL_ERR_SHAPE;
  return RL_OK;
}

rl_status rl_rvq_codebook_norms(const void* codebooks, int32_t G, int32_t N, int32_t S, int32_t D, float* norms, void* stream) {
  if (!codebooks || !norms) return RL_ERR_NULL;
  rl_status st = rvq_check(G, 1, D, N, S);
  if (st != RL_OK) return st;
  if (reinterpret_cast<uintptr_t>(codebooks) & 15) return RL_ERR_SHAPE;
  (void)hipGetLastError();
  const int64_t entries = (int64_t)G * N * S;
  rvq_norms_kernel<<<(unsigned)((entries + 255) / 256), 256, 0, static_cast<hipStream_t>(stream)>>>(static_cast<const bf16_t*>(codebooks), entries, norms);
  return hipGetLastError() == hipSuccess ? RL_OK : RL_ERR_HIP;
}

rl_status rl_rvq_encode(const void* vectors, const void* codebooks, const float* norms, int32_t G, int64_t L, int32_t D,
                        int32_t N, int32_t S, int32_t* codes, void* residual, void* stream) {
  return rl_rvq_encode_counted(vectors, codebooks, norms, G, L, D, N, S, codes, residual, nullptr, stream);
}

rl_status rl_rvq_encode_counted(const void* vectors, const void* codebooks, const float* norms, int32_t G, int64_t L, int32_t D,
                                int32_t N, int32_t S, int32_t* codes, void* residual, int32_t* n_exact, void* stream) {
  if (!vectors || !codebooks || !norms || !codes) return RL_ERR_NULL;
  rl_status st = rvq_check(G, L, D, N, S);
  if (st != RL_OK) return st;
  if ((reinterpret_cast<uintptr_t>(vectors) | reinterpret_cast<uintptr_t>(codebooks) | reinterpret_cast<uintptr_t>(residual)) & 15) return RL_ERR_SHAPE;
  (void)hipGetLastError();
  const int kw = L > 256 ? 8 : 4;                                   // wavefronts per workgroup, 64 vectors each
  const int64_t n_wg = (L + 64 * kw - 1) / (64 * kw) * (8 * (((int64_t)G + 7) / 8));
  if (n_wg > 0x7fffffff) return RL_ERR_RANGE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (kw == 8)
    rvq_encode_kernel<8><<<(unsigned)n_wg, 512, 0, s>>>(static_cast<const bf16_t*>(vectors), static_cast<const bf16_t*>(codebooks), norms,
                                                        G, (int)L, N, S, codes, static_cast<bf16_t*>(residual), n_exact);
  else
    rvq_encode_kernel<4><<<(unsigned)n_wg, 256, 0, s>>>(static_cast<const bf16_t*>(vectors), static_cast<const bf16_t*>(codebooks), norms,
                                                        G, (int)L, N, S, codes, static_cast<bf16_t*>(residual), n_exact);
  return hipGetLastError() == hipSuccess ? RL_OK : RL_ERR_HIP;
}

}  // extern "C"
