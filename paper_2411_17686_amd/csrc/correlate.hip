// Correlate stage: correlation row of every discarded token over the preserved tokens,
// its eps-quantile threshold, the correlated targets and their weights
// (Sec. "Correlation-based Information Recycling", Eq. 4, Algorithm 1/2 stage 3, Eq. 2's
// alpha).  One wavefront per discarded token.  Values are evaluated on the fly in double
// precision and every comparison is on doubles.
//
//   tau_i = v[f] + g (v[f+1] - v[f]),  p = eps (n-1), f = floor(p), g = p - f, v = row sorted
//   J_i = { j : C_ij >= tau_i },  alpha_ij = C_ij / sum_{J_i} C_ij  (sum in ascending j)
//
// Only the m = n - f largest values of a row decide tau.  For m <= kSelMax they are kept in
// registers (per lane, then merged across the wavefront); otherwise the row is written to
// the workspace and the two order statistics are found bit by bit.
#include "common.hpp"
#include "gram_tile.hpp"

namespace ficoco {

enum CorrMode { kAttnV = 0, kAttnL = 1, kCosV = 2, kCosL = 3 };

struct CorrArgs {
  int B, N, n_keep, n_disc, M, k_max, Df, mode;
  const float* abar;     // [B][N][map_pitch] head-mean map, transposed: abar[b][key token i][query token j]
  int map_pitch;
  const double* ttext;   // [B][N][M]
  const bf16_t* xhat;    // [B][N][Df]
  double gamma, invM;
  const int32_t* S;
  const int32_t* T;
  int sel_m, sel_f;
  double sel_g;
  int dense;
  double* rowbuf;        // [B][n_disc][n_keep]
  int32_t* edge_cnt;
  int32_t* edge_tgt;
  double* edge_alpha;
  int32_t* overflow;
  const int32_t* slot_of; // [B][N] keep slot of a visual token, -1 if discarded
  float* ct;             // [ct_splits][B][n_disc][n_keep] approximate cosines from the matrix cores (partial sums)
  int ct_splits;
  double* cmax;          // [B][M]
  float delta;           // bound of |ct - exact dot|
  int fixed_k;           // > 0: ablation "fixed K" (sel_m = K, sel_g = 0): of the values equal to the threshold only
                         // the lowest positions are taken, K targets in all; -1: every value >= threshold
  double* gap;           // correlation-gap diagnostic output [B][n_disc] (its own kernel)
  int32_t* share_cnt;    // [B][shares][n_keep] edges written per (share of discarded rows, target), cleared by the
                         // filter stage of a fused step; null where the compress stage counts for itself
  int shares, share_rows;
  PairRec* pair_tab;     // [B][n_disc] first two edges of every row as one record (fused step, scanning merge), or null
};

// The record of discarded row `row` (source token i): written by one lane with two 16-byte stores.
__device__ __forceinline__ void write_pair(const CorrArgs& a, int64_t b, int row, int cnt, int i, int t0, int t1,
                                           double a0, double a1) {
  PairRec r;
  r.cnt = cnt; r.src = i; r.t0 = t0; r.t1 = t1; r.a0 = a0; r.a1 = a1;
  a.pair_tab[b * a.n_disc + row] = r;
}

// One more edge from discarded row `row` to keep slot `tgt`: counted for the compress stage, which
// buckets the edges by target (one workgroup per share of share_rows consecutive rows).
__device__ __forceinline__ void count_edge(const CorrArgs& a, int64_t b, int row, int tgt) {
  if (a.share_cnt && (unsigned)tgt < (unsigned)a.n_keep)
    atomicAdd(&a.share_cnt[(b * a.shares + row / a.share_rows) * a.n_keep + tgt], 1);
}

__device__ __forceinline__ double dot_bf16(const bf16_t* __restrict__ x, const bf16_t* __restrict__ y, int D) {
  double acc = 0.0;
  int d = 0;
  for (; d + kVec <= D; d += kVec) {
    double a[kVec], c[kVec];
    load8<bf16_t>(x + d, a);
    load8<bf16_t>(y + d, c);
#pragma unroll
    for (int k = 0; k < kVec; ++k) acc += a[k] * c[k];
  }
  for (; d < D; ++d) acc += widen(x[d]) * widen(y[d]);
  return acc;
}

// C[i][j] for discarded visual token i and preserved visual token j of image b.
__device__ __forceinline__ double corr_value(const CorrArgs& a, int64_t b, int i, int j) {
  double direct;
  if (a.mode == kAttnV || a.mode == kAttnL) {
    direct = (double)a.abar[(b * a.N + i) * a.map_pitch + j];
  } else {
    const double d = dot_bf16(a.xhat + (b * a.N + i) * a.Df, a.xhat + (b * a.N + j) * a.Df, a.Df);
    direct = d > 0.0 ? d : 0.0;
  }
  if (a.mode == kAttnV || a.mode == kCosV) return direct;
  const double* ti = a.ttext + (b * a.N + i) * a.M;
  const double* tj = a.ttext + (b * a.N + j) * a.M;
  double br = 0.0;
  for (int k = 0; k < a.M; ++k) br += ti[k] * tj[k];
  return a.gamma * direct + (1.0 - a.gamma) * (br * a.invM);
}

__device__ __forceinline__ double wave_max(double v) {
  return wave_reduce(v, [](double x, double y) { return y > x ? y : x; });
}
__device__ __forceinline__ float wave_max(float v) {
  return wave_reduce(v, [](float x, float y) { return y > x ? y : x; });
}
__device__ __forceinline__ int wave_sum(int v) {
  return wave_reduce(v, [](int x, int y) { return x + y; });
}

__device__ __forceinline__ uint64_t order_key(double x) {   // monotone double -> uint64
  const uint64_t u = (uint64_t)__double_as_longlong(x);
  return (u >> 63) ? ~u : (u | 0x8000000000000000ULL);
}
__device__ __forceinline__ double key_value(uint64_t k) {
  const uint64_t u = (k >> 63) ? (k & 0x7fffffffffffffffULL) : ~k;
  return __longlong_as_double((long long)u);
}

// Value of ascending rank `want` (0-based) among row[0..n): bitwise selection on the
// ordered keys, most significant bit first.  All lanes return the same value.
__device__ double select_rank(const double* __restrict__ row, int n, int want, int lane) {
  uint64_t prefix = 0;
  int rank = want;
  for (int bit = 63; bit >= 0; --bit) {
    const uint64_t hi_mask = bit == 63 ? 0ULL : (~0ULL << (bit + 1));
    int zeros = 0;
    for (int j = lane; j < n; j += kWave) {
      const uint64_t k = order_key(row[j]);
      zeros += ((k & hi_mask) == prefix && !((k >> bit) & 1ULL)) ? 1 : 0;
    }
    zeros = wave_sum(zeros);
    if (rank >= zeros) { rank -= zeros; prefix |= 1ULL << bit; }
  }
  return key_value(prefix);
}

__device__ __forceinline__ double threshold_of(double v_f, double v_f1, double g) {
#pragma clang fp contract(off)
  const double diff = v_f1 - v_f;
  const double step = g * diff;
  return v_f + step;
}

__global__ __launch_bounds__(256) void corr_fill_rows_kernel(CorrArgs a) {
  const int lane = threadIdx.x % kWave;
  const int row = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
  const int64_t b = blockIdx.y;
  if (row >= a.n_disc) return;
  const int i = a.S[b * a.n_disc + row];
  double* dst = a.rowbuf + (b * a.n_disc + row) * a.n_keep;
  for (int jj = lane; jj < a.n_keep; jj += kWave) {
    const int j = a.T[b * a.n_keep + jj];
    const bool ok = (unsigned)i < (unsigned)a.N && (unsigned)j < (unsigned)a.N;  // index sets are device data
    dst[jj] = ok ? corr_value(a, b, i, j) : -__builtin_huge_val();
  }
}

// One discarded row, exactly: every value of the row evaluated in double precision.
__device__ void corr_row_exact(const CorrArgs& a, const int64_t b, const int row, const int lane) {
  const int n = a.n_keep;
  const int i = a.S[b * a.n_disc + row];
  const int32_t* T = a.T + b * n;
  if ((unsigned)i >= (unsigned)a.N) {  // index sets are device data: never index with a bad one
    if (lane == 0) {
      a.edge_cnt[b * a.n_disc + row] = 0;
      if (a.pair_tab) write_pair(a, b, row, 0, 0, 0, 0, 0.0, 0.0);
    }
    return;
  }
  const double* rowv = a.dense ? a.rowbuf + (b * a.n_disc + row) * n : nullptr;
  const double NEG = -__builtin_huge_val();

  double v_f, v_f1;
  int n_gt = 0;                      // values strictly above v_f (used by the fixed-K form only)
  if (a.dense) {
    v_f = select_rank(rowv, n, a.sel_f, lane);
    v_f1 = a.sel_f + 1 <= n - 1 ? select_rank(rowv, n, a.sel_f + 1, lane) : v_f;
    if (a.fixed_k > 0) {
      for (int jj = lane; jj < n; jj += kWave) n_gt += rowv[jj] > v_f ? 1 : 0;
      n_gt = wave_sum(n_gt);
    }
  } else {
    // per-lane descending top list, then m rounds of "pop the wavefront maximum"
    double top[kSelMax];
#pragma unroll
    for (int k = 0; k < kSelMax; ++k) top[k] = NEG;
    for (int jj = lane; jj < n; jj += kWave) {
      const int j = T[jj];
      double c = (unsigned)j < (unsigned)a.N ? corr_value(a, b, i, j) : NEG;
      if (c > top[kSelMax - 1]) {
#pragma unroll
        for (int k = 0; k < kSelMax; ++k) {
          const bool sw = c > top[k];
          const double t = top[k];
          top[k] = sw ? c : t;
          c = sw ? t : c;
        }
      }
    }
    v_f = NEG; v_f1 = NEG;
    for (int r = 0; r < a.sel_m; ++r) {
      const double mx = wave_max(top[0]);
      const unsigned long long who = __ballot(top[0] == mx);
      const int first = __ffsll(who) - 1;
      if (lane == first) {
#pragma unroll
        for (int k = 0; k + 1 < kSelMax; ++k) top[k] = top[k + 1];
        top[kSelMax - 1] = NEG;
      }
      if (r == 0 || mx < v_f) n_gt = r;     // pops so far that are strictly above this one
      v_f1 = v_f;
      v_f = mx;
    }
    if (a.sel_m == 1) v_f1 = v_f;
  }
  const double tau = threshold_of(v_f, v_f1, a.sel_g);
  const int tie_quota = a.fixed_k > 0 ? a.sel_m - n_gt : 0x7fffffff;   // values equal to tau that are taken
  int ties_seen = 0;

  // Emit targets in ascending order; lane e of the wavefront ends up holding edge e.
  int cnt = 0;
  double denom = 0.0;
  int my_tgt = -1;
  double my_c = 0.0;
  const int64_t ebase = (b * a.n_disc + row) * a.k_max;
  for (int base = 0; base < n; base += kWave) {
    const int jj = base + lane;
    double c = NEG;
    if (jj < n) {
      if (a.dense) c = rowv[jj];
      else { const int j = T[jj]; if ((unsigned)j < (unsigned)a.N) c = corr_value(a, b, i, j); }
    }
    const bool is_eq = jj < n && c == tau;
    const unsigned long long eqm = __ballot(is_eq);
    const int eq_rank = ties_seen + __popcll(eqm & ((1ULL << lane) - 1ULL));
    ties_seen += __popcll(eqm);
    unsigned long long hit = __ballot(jj < n && (c > tau || (is_eq && eq_rank < tie_quota)));
    while (hit) {
      const int l = __ffsll(hit) - 1;
      hit &= hit - 1;
      const double cl = lane_value(c, l);
      denom += cl;
      if (a.k_max <= kWave) {
        if (lane == cnt) { my_tgt = base + l; my_c = cl; }
      } else if (lane == 0 && cnt < a.k_max) {
        a.edge_tgt[ebase + cnt] = base + l;
        a.edge_alpha[ebase + cnt] = cl;      // raw value, scaled below
      }
      ++cnt;
    }
  }
  const int stored = cnt < a.k_max ? cnt : a.k_max;
  const bool live = denom > 0.0;
  if (a.k_max <= kWave) {
    if (live && lane < stored) {
      const double al = my_c / denom;
      a.edge_tgt[ebase + lane] = my_tgt;
      a.edge_alpha[ebase + lane] = al;
      count_edge(a, b, row, my_tgt);
    }
  } else if (live && lane == 0) {
    for (int e = 0; e < stored; ++e) {
      const double al = a.edge_alpha[ebase + e] / denom;
      a.edge_alpha[ebase + e] = al;
      count_edge(a, b, row, a.edge_tgt[ebase + e]);
    }
  }
  if (a.pair_tab) {              // uniform (lists of at most 64 entries: lanes 0 and 1 hold the first two)
    const double al = live && lane < stored ? my_c / denom : 0.0;
    const int t0 = lane_value(my_tgt, 0), t1 = lane_value(my_tgt, 1);
    const double a0 = lane_value(al, 0), a1 = lane_value(al, 1);
    if (lane == 0) write_pair(a, b, row, live ? stored : 0, i, t0, t1, a0, a1);
  }
  if (lane == 0) {
    a.edge_cnt[b * a.n_disc + row] = live ? stored : 0;
    if (live && cnt > a.k_max) a.overflow[b] = 1;
  }
}

__global__ __launch_bounds__(256) void corr_rows_kernel(CorrArgs a) {
  const int lane = threadIdx.x % kWave;
  const int row = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
  if (row >= a.n_disc) return;  // whole wavefront leaves together
  corr_row_exact(a, blockIdx.y, row, lane);
}

// ---- cosine correlation through the matrix cores -------------------------------------------
// gram_tile_kernel (bf16 MFMA) has written approximate cosines ct[b][row][j].  They only
// propose candidates.  With |ct - exact dot| <= delta and, for FiCoCo-L, the indirect term of
// Eq. 4 inside [0, bound_i], every C_ij lies in [lo_ij, up_ij]; the m-th largest lo of the
// row is a lower bound of v[f], so a target with up_ij below it can neither be one of the
// order statistics that fix tau nor pass the threshold.  The remaining targets (a handful)
// are evaluated exactly in double precision and the row is finished on those.  A row with
// more than 64 candidates is evaluated exactly in full instead.
constexpr int kCandCap = 64;

__device__ __forceinline__ double wave_sum_f64(double v) {
  return wave_reduce(v, [](double x, double y) { return x + y; });
}

// exact C[i][j], the whole wavefront working on one pair (all lanes return the value)
__device__ __forceinline__ double corr_value_wave(const CorrArgs& a, int64_t b, int i, int j, int lane) {
  double direct;
  if (a.mode == kAttnL) {
    direct = (double)a.abar[(b * a.N + i) * a.map_pitch + j];
  } else {
    const bf16_t* x = a.xhat + (b * a.N + i) * a.Df;
    const bf16_t* y = a.xhat + (b * a.N + j) * a.Df;
    double acc = 0.0;
    const int Dv = a.Df - a.Df % kVec;
    for (int d = lane * kVec; d < Dv; d += kWave * kVec) {
      double u[kVec], w[kVec];
      load8<bf16_t>(x + d, u);
      load8<bf16_t>(y + d, w);
#pragma unroll
      for (int k = 0; k < kVec; ++k) acc += u[k] * w[k];
    }
    for (int d = Dv + lane; d < a.Df; d += kWave) acc += widen(x[d]) * widen(y[d]);
    acc = wave_sum_f64(acc);
    direct = acc > 0.0 ? acc : 0.0;
  }
  if (a.mode == kCosV) return direct;
  const double* ti = a.ttext + (b * a.N + i) * a.M;
  const double* tj = a.ttext + (b * a.N + j) * a.M;
  double br = 0.0;
  for (int k = lane; k < a.M; k += kWave) br += ti[k] * tj[k];
  br = wave_sum_f64(br);
  return a.gamma * direct + (1.0 - a.gamma) * (br * a.invM);
}

// cmax[b][k] = max over the visual tokens of the text profile entry k (bound of Eq. 4's indirect
// term).  A workgroup takes 64 consecutive text queries k of one image: thread (k, g) walks the
// tokens g, g+4, ... (16 independent loads per round), the four token groups meet in LDS.
__global__ __launch_bounds__(256) void text_colmax_kernel(CorrArgs a) {
  __shared__ double part[256];
  const int64_t b = blockIdx.y;
  const int tid = threadIdx.x;
  const int k = blockIdx.x * 64 + tid % 64, g = tid / 64;
  double mx = 0.0;
  if (k < a.M) {
    int i = g;
    for (; i + 4 * 15 < a.N; i += 4 * 16) {            // 16 independent loads per round
      double v[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) v[u] = a.ttext[(b * a.N + i + 4 * u) * a.M + k];
#pragma unroll
      for (int u = 0; u < 16; ++u) mx = v[u] > mx ? v[u] : mx;
    }
    for (; i < a.N; i += 4) { const double v = a.ttext[(b * a.N + i) * a.M + k]; mx = v > mx ? v : mx; }
  }
  part[tid] = mx;
  __syncthreads();
  if (g == 0 && k < a.M) {
    for (int q = 1; q < 4; ++q) mx = part[q * 64 + tid] > mx ? part[q * 64 + tid] : mx;
    a.cmax[b * a.M + k] = mx;
  }
}

constexpr int kCorrSteps = 2;   // 512-feature steps of the exact dot products loaded together

// Exact C[i][j_q] for up to CB targets at once, the whole wavefront working on them together
// (all lanes return the values).  The loads of all CB rows are issued before the first use, so
// a batch costs one memory round trip per 512 features instead of one per target.  Per target
// the arithmetic and its order are those of corr_value_wave.
template <int CB>
__device__ __forceinline__ void corr_values_wave(const CorrArgs& a, int64_t b, int i, const int (&j)[CB], int lane,
                                                 double (&out)[CB]) {
  double direct[CB];
  if (a.mode == kAttnL) {
#pragma unroll
    for (int q = 0; q < CB; ++q) direct[q] = (double)a.abar[(b * a.N + i) * a.map_pitch + j[q]];
  } else {
    const bf16_t* x = a.xhat + (b * a.N + i) * a.Df;
    const bf16_t* y[CB];
    double acc[CB];
#pragma unroll
    for (int q = 0; q < CB; ++q) { y[q] = a.xhat + (b * a.N + j[q]) * a.Df; acc[q] = 0.0; }
    const int Dv = a.Df - a.Df % kVec;
    // kCorrSteps steps of 512 features at a time: (1 + CB) * kCorrSteps loads in flight.  A lane
    // past the last whole vector reads vector 0 and clears it (straight-line batch).
    for (int d0 = lane * kVec; d0 - lane * kVec < Dv; d0 += kCorrSteps * kWave * kVec) {
      Raw8<bf16_t> xr[kCorrSteps], yr[kCorrSteps][CB];
#pragma unroll
      for (int t = 0; t < kCorrSteps; ++t) {
        const int d = d0 + t * kWave * kVec;
        const int off = d < Dv ? d : 0;
        load_raw(x + off, xr[t]);
#pragma unroll
        for (int q = 0; q < CB; ++q) load_raw(y[q] + off, yr[t][q]);
      }
      issue_fence();
#pragma unroll
      for (int t = 0; t < kCorrSteps; ++t) {
        keep_raw_if(xr[t], d0 + t * kWave * kVec < Dv);      // a cleared x vector adds zeros for every target
        double u[kVec];
        widen_raw(xr[t], u);
#pragma unroll
        for (int q = 0; q < CB; ++q) {
          double w[kVec];
          widen_raw(yr[t][q], w);
#pragma unroll
          for (int k = 0; k < kVec; ++k) acc[q] += u[k] * w[k];
        }
      }
    }
    for (int d = Dv + lane; d < a.Df; d += kWave) {
#pragma unroll
      for (int q = 0; q < CB; ++q) acc[q] += widen(x[d]) * widen(y[q][d]);
    }
#pragma unroll
    for (int q = 0; q < CB; ++q) {
      const double t = wave_sum_f64(acc[q]);
      direct[q] = t > 0.0 ? t : 0.0;
    }
  }
  if (a.mode == kCosV) {
#pragma unroll
    for (int q = 0; q < CB; ++q) out[q] = direct[q];
    return;
  }
  const double* ti = a.ttext + (b * a.N + i) * a.M;
  double br[CB];
#pragma unroll
  for (int q = 0; q < CB; ++q) br[q] = 0.0;
  for (int k = lane; k < a.M; k += kWave) {
    const double tik = ti[k];
    double tjk[CB];
#pragma unroll
    for (int q = 0; q < CB; ++q) tjk[q] = a.ttext[(b * a.N + j[q]) * a.M + k];
#pragma unroll
    for (int q = 0; q < CB; ++q) br[q] += tik * tjk[q];
  }
#pragma unroll
  for (int q = 0; q < CB; ++q) out[q] = a.gamma * direct[q] + (1.0 - a.gamma) * (wave_sum_f64(br[q]) * a.invM);
}

constexpr int kCandKeep = 32;                    // approximate values held per lane
constexpr int kCandChunk = kCandKeep * kWave;    // targets per pass over the row
static_assert(kCandChunk <= kCandPad, "the block's padding covers one pass");
constexpr int kCandBatch = 4;                    // targets evaluated exactly at a time

// Compiled for four wavefronts per SIMD (128 registers; it would take 132): the decoder shape has
// 3456 discarded rows, one wavefront each, and the chip holds 3072 of them at three per SIMD.
template <int MC>   // lower bounds kept per lane (>= sel_m: one lane may hold the m largest of the row)
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4))) void corr_cand_rows_kernel(CorrArgs a) {
  __shared__ int cand_j[4][kCandCap];
  const int lane = threadIdx.x % kWave, wv = threadIdx.x / kWave;
  const int row = blockIdx.x * (blockDim.x / kWave) + wv;
  const int64_t b = blockIdx.y;
  if (row >= a.n_disc) return;  // whole wavefront leaves together
  const int n = a.n_keep;
  const int i = a.S[b * a.n_disc + row];
  const int32_t* T = a.T + b * n;
  if ((unsigned)i >= (unsigned)a.N) {
    if (lane == 0) {
      a.edge_cnt[b * a.n_disc + row] = 0;
      if (a.pair_tab) write_pair(a, b, row, 0, 0, 0, 0, 0.0, 0.0);
    }
    return;
  }
  // approximate direct term of the row: the matrix-core cosines, or (FiCoCo-L with the
  // attention correlation) the token's row of the exact head-mean map, delta = 0
  const bool from_map = a.mode == kAttnL;
  const float* ct = from_map ? a.abar + (b * a.N + i) * a.map_pitch : a.ct + (b * a.n_disc + row) * n;
  const bool L = a.mode == kCosL || a.mode == kAttnL;
  const float gam = L ? (float)a.gamma : 1.0f;
  float extra = 0.0f;                      // upper bound of (1 - gamma) * indirect term of this row
  if (L) {
    double bd = 0.0;
    for (int k = lane; k < a.M; k += kWave) bd += a.ttext[(b * a.N + i) * a.M + k] * a.cmax[b * a.M + k];
    bd = wave_sum_f64(bd) * a.invM * (1.0 - a.gamma);
    extra = (float)bd * 1.000001f + 1e-30f;   // rounded up
  }
  const float delta = from_map ? 0.0f : a.delta;
  const float NEGF = -__builtin_huge_valf();
  const int64_t split_stride = (int64_t)a.B * a.n_disc * n;

  // One pass of the row: element u of a lane is target c0 + u*64 + lane.  All loads of a pass
  // are independent (the map gather takes the token indices first), absent targets read as -inf.
  float val[kCandKeep];
  auto load_pass = [&](int c0) {
    const int n_u = min(kCandKeep, (n - c0 + kWave - 1) / kWave);   // slots of this pass that hold targets (uniform)
    if (from_map) {
      int jt[kCandKeep];
#pragma unroll
      for (int u = 0; u < kCandKeep; ++u) {
        const int jj = c0 + u * kWave + lane;
        jt[u] = (u < n_u && jj < n) ? T[jj] : -1;
      }
#pragma unroll
      for (int u = 0; u < kCandKeep; ++u) {
        const bool ok = (unsigned)jt[u] < (unsigned)a.N;
        float v = 0.0f;
        if (u < n_u) v = ct[ok ? jt[u] : 0];
        val[u] = c0 + u * kWave + lane < n ? (ok ? v : 0.0f) : NEGF;
      }
    } else {
      // The block is followed by kCandChunk floats of padding, so a pass may read past the end
      // of the row (what it reads there is masked below): one address, constant offsets.
      const float* c = ct + c0 + lane;
#pragma unroll
      for (int ub = 0; ub < kCandKeep; ub += 8) {
        if (ub < n_u) {                                              // uniform: groups of 8 slots that hold targets
#pragma unroll
          for (int u = 0; u < 8; ++u) val[ub + u] = c[(ub + u) * kWave];
        } else {
#pragma unroll
          for (int u = 0; u < 8; ++u) val[ub + u] = 0.0f;
        }
      }
      // partial sums of the further K ranges, added in order; the loads of up to four ranges
      // are issued together (a range past the last one reads the last again and adds zero)
#pragma unroll 1
      for (int sp0 = 1; sp0 < a.ct_splits; sp0 += 4) {
#pragma unroll
        for (int ub = 0; ub < kCandKeep; ub += 8) {
          if (ub < n_u) {                                            // uniform
            float part[4][8];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const float* cq = c + (int64_t)min(sp0 + q, a.ct_splits - 1) * split_stride;
#pragma unroll
              for (int u = 0; u < 8; ++u) part[q][u] = cq[(ub + u) * kWave];
            }
            issue_fence();
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const bool in = sp0 + q < a.ct_splits;
#pragma unroll
              for (int u = 0; u < 8; ++u) val[ub + u] += in ? part[q][u] : 0.0f;
            }
          }
        }
      }
#pragma unroll
      for (int u = 0; u < kCandKeep; ++u) {
        if (c0 + u * kWave >= n) break;         // uniform: no reader looks at slots past the row
        if (c0 + u * kWave + lane >= n) val[u] = NEGF;
      }
    }
  };

  // lower bounds: per-lane top list, then m pops of the wavefront maximum -> lambda
  float top[MC];
#pragma unroll
  for (int k = 0; k < MC; ++k) top[k] = NEGF;
  for (int c0 = 0; c0 < n; c0 += kCandChunk) {
    load_pass(c0);
#pragma unroll
    for (int u = 0; u < kCandKeep; ++u) {
      if (c0 + u * kWave >= n) break;           // uniform: slots past the row hold nothing
      float lo = val[u] == NEGF ? NEGF : gam * fmaxf(val[u] - delta, 0.0f);
      if (lo > top[MC - 1]) {
#pragma unroll
        for (int k = 0; k < MC; ++k) {
          const bool sw = lo > top[k];
          const float t = top[k];
          top[k] = sw ? lo : t;
          lo = sw ? t : lo;
        }
      }
    }
  }
  float lambda = NEGF;
  for (int r = 0; r < a.sel_m; ++r) {
    const float mx = wave_max(top[0]);
    const unsigned long long who = __ballot(top[0] == mx);
    if (lane == __ffsll(who) - 1) {
#pragma unroll
      for (int k = 0; k + 1 < MC; ++k) top[k] = top[k + 1];
      top[MC - 1] = NEGF;
    }
    lambda = mx;
  }
  // candidates in ascending target order (a row of one pass is still in registers)
  int n_cand = 0;
  for (int c0 = 0; c0 < n; c0 += kCandChunk) {
    if (n > kCandChunk) load_pass(c0);
#pragma unroll
    for (int u = 0; u < kCandKeep; ++u) {
      if (c0 + u * kWave >= n) break;           // uniform
      const int jj = c0 + u * kWave + lane;
      const bool is = jj < n && gam * fmaxf(val[u] + delta, 0.0f) * 1.000001f + extra >= lambda;
      const unsigned long long m = __ballot(is);
      if (is) {
        const int slot = n_cand + __popcll(m & ((1ULL << lane) - 1ULL));
        if (slot < kCandCap) cand_j[wv][slot] = jj;
      }
      n_cand += __popcll(m);
    }
  }
  if (n_cand > kCandCap) {       // uniform per wavefront
    corr_row_exact(a, b, row, lane);
    return;
  }
  // exact values of the candidates: lane c keeps candidate c
  const double NEG = -__builtin_huge_val();
  const int myjj = lane < n_cand ? cand_j[wv][lane] : -1;
  const int myj = myjj >= 0 ? T[myjj] : -1;
  double myv = NEG;
  for (int c = 0; c < n_cand; c += kCandBatch) {
    int j[kCandBatch];
    bool ok[kCandBatch];
#pragma unroll
    for (int q = 0; q < kCandBatch; ++q) {
      const int jq = lane_value(myj, min(c + q, n_cand - 1));
      ok[q] = (unsigned)jq < (unsigned)a.N;
      j[q] = ok[q] ? jq : i;                   // a valid row to read; the value is dropped
    }
    double v[kCandBatch];
    corr_values_wave<kCandBatch>(a, b, i, j, lane, v);
#pragma unroll
    for (int q = 0; q < kCandBatch; ++q)
      if (lane == c + q && c + q < n_cand) myv = ok[q] ? v[q] : NEG;
  }
  // v[f], v[f+1] = m-th and (m-1)-th largest of the exact candidate values
  double v_f = NEG, v_f1 = NEG;
  int n_gt = 0;
  {
    double act = myv;
    for (int r = 0; r < a.sel_m; ++r) {
      const double mx = wave_max(act);
      const unsigned long long who = __ballot(act == mx);
      if (lane == __ffsll(who) - 1) act = NEG;
      if (r == 0 || mx < v_f) n_gt = r;
      v_f1 = v_f;
      v_f = mx;
    }
    if (a.sel_m == 1) v_f1 = v_f;
  }
  const double tau = threshold_of(v_f, v_f1, a.sel_g);
  const int tie_quota = a.fixed_k > 0 ? a.sel_m - n_gt : 0x7fffffff;
  const bool is_eq = myjj >= 0 && myv == tau;
  const int eq_rank = __popcll(__ballot(is_eq) & ((1ULL << lane) - 1ULL));   // candidates are in ascending target order
  unsigned long long hit = __ballot(myjj >= 0 && (myv > tau || (is_eq && eq_rank < tie_quota)));
  const unsigned long long hit_all = hit;
  const int cnt = __popcll(hit);
  const int my_pos = __popcll(hit & ((1ULL << lane) - 1ULL));
  const bool mine = (hit >> lane) & 1ULL;
  double denom = 0.0;
  while (hit) {                       // ascending target order
    const int l = __ffsll(hit) - 1;
    hit &= hit - 1;
    denom += lane_value(myv, l);
  }
  const bool live = denom > 0.0;
  const int stored = cnt < a.k_max ? cnt : a.k_max;
  const int64_t ebase = (b * a.n_disc + row) * a.k_max;
  if (live && mine && my_pos < stored) {
    const double al = myv / denom;
    a.edge_tgt[ebase + my_pos] = myjj;
    a.edge_alpha[ebase + my_pos] = al;
    count_edge(a, b, row, myjj);
  }
  if (a.pair_tab) {              // uniform; the lanes of the first two hits hold the first two edges
    const double al = live && mine ? myv / denom : 0.0;
    const unsigned long long rest = hit_all & (hit_all - 1);
    const int l0 = hit_all ? __ffsll(hit_all) - 1 : 0, l1 = rest ? __ffsll(rest) - 1 : 0;
    const int t0 = lane_value(myjj, l0), t1 = lane_value(myjj, l1);
    const double a0 = lane_value(al, l0), a1 = lane_value(al, l1);
    if (lane == 0) write_pair(a, b, row, live ? stored : 0, i, t0, t1, a0, a1);
  }
  if (lane == 0) {
    a.edge_cnt[b * a.n_disc + row] = live ? stored : 0;
    if (live && cnt > a.k_max) a.overflow[b] = 1;
  }
}

// ---- FiCoCo-V attention correlation ------------------------------------------------------------
// C[i][j] = Pbar[j][i] (Algorithm 1, stage 2).  The head-mean map is stored transposed, so the
// values of discarded token i are one contiguous row; slot_of tells which of its entries belong
// to preserved tokens.  One wavefront per discarded token: one pass keeps each lane's MC largest
// (value, slot) pairs, the m-th and (m-1)-th largest of the row (with multiplicity) are popped
// off the lanes' lists, and the targets at or above the threshold are taken from the lists in
// ascending order; the row is read a second time only if some lane's list could not hold all
// of its targets.  Values are compared as the floats they are stored as.
// kRowBatch = 64-entry steps of the row loaded together; a row that fits one batch stays in
// registers for the second pass (10 steps: the 576-token grid).  Longer rows take batches of
// kRowWide steps (measured at 2880 tokens: 16 is as good as 24, and 48 -- the whole row in
// registers, at a quarter of the resident wavefronts -- is slower).
constexpr int kRowWide = 16;
template <int MC, int kRowBatch>
__global__ __launch_bounds__(256) void corr_attn_rows_kernel(CorrArgs a) {
  const int lane = threadIdx.x % kWave;
  const int row = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
  const int64_t b = blockIdx.y;
  if (row >= a.n_disc) return;                 // whole wavefront leaves together
  const int i = a.S[b * a.n_disc + row];
  if ((unsigned)i >= (unsigned)a.N) {          // index sets are device data
    if (lane == 0) {
      a.edge_cnt[b * a.n_disc + row] = 0;
      if (a.pair_tab) write_pair(a, b, row, 0, 0, 0, 0, 0.0, 0.0);
    }
    return;
  }
  const float* mrow = a.abar + (b * a.N + i) * a.map_pitch;
  const int32_t* slot_of = a.slot_of + b * a.N;
  const float NEGF = -__builtin_huge_valf();

  // One batch of the row: entry u of a lane is query token r0 + 64 u + lane; entries past the
  // row or of discarded tokens read as -inf with slot -1.
  float vv[kRowBatch];
  int sv[kRowBatch];
  auto load_batch = [&](int r0) {
    // Rows of the map are padded to whole 64-entry steps and the slot table by one step, so the
    // steps that begin inside the row are read as they are (one address, constant offsets) and
    // masked below; steps that begin past the row are skipped.
    const int n_u = min(kRowBatch, (a.N - r0 + kWave - 1) / kWave);      // steps of this batch that begin inside the row
    const float* mp = mrow + r0 + lane;
    const int32_t* sp = slot_of + r0 + lane;
#pragma unroll
    for (int u = 0; u < kRowBatch; ++u) {
      vv[u] = 0.0f;
      sv[u] = -1;
      if (u < n_u) {                                       // uniform (a scalar branch): nothing is read past the row's last step
        vv[u] = mp[u * kWave];
        sv[u] = sp[u * kWave];
      }
    }
    issue_fence();
#pragma unroll
    for (int u = 0; u < kRowBatch; ++u) {
      const bool ok = r0 + u * kWave + lane < a.N && sv[u] >= 0;
      vv[u] = ok ? vv[u] : NEGF;
      sv[u] = ok ? sv[u] : -1;
    }
  };

  float top[MC];
  int topj[MC];
#pragma unroll
  for (int k = 0; k < MC; ++k) { top[k] = NEGF; topj[k] = -1; }
  for (int r0 = 0; r0 < a.N; r0 += kRowBatch * kWave) {
    load_batch(r0);
#pragma unroll
    for (int u = 0; u < kRowBatch; ++u) {
      float v = vv[u];
      int jq = sv[u];
#pragma unroll
      for (int k = 0; k < MC; ++k) {
        const bool sw = v > top[k];
        const float t = top[k];
        const int tj = topj[k];
        top[k] = sw ? v : t;
        topj[k] = sw ? jq : tj;
        v = sw ? t : v;
        jq = sw ? tj : jq;
      }
    }
  }
  // v[f], v[f+1]: pop the wavefront maximum m times (MC >= m, so one lane may hold them all)
  float vf = NEGF, vf1 = NEGF;
  int n_gt = 0;                                // pops strictly above vf
  int head = 0;                                // entries of this lane's list popped so far (the lists stay as they are)
  for (int r = 0; r < a.sel_m; ++r) {
    float cur = NEGF;
#pragma unroll
    for (int k = 0; k < MC; ++k) cur = k == head ? top[k] : cur;
    const float mx = wave_max(cur);
    const unsigned long long who = __ballot(cur == mx);
    if (lane == __ffsll(who) - 1) ++head;
    if (r == 0 || mx < vf) n_gt = r;
    vf1 = vf;
    vf = mx;
  }
  if (a.sel_m == 1) vf1 = vf;
  const double tau = threshold_of((double)vf, (double)vf1, a.sel_g);
  const int tie_quota = a.fixed_k > 0 ? a.sel_m - n_gt : 0x7fffffff;   // values equal to tau that are taken
  int ties_seen = 0;
  // a float at or below tau: v >= tau_below is a cheap necessary condition for (double)v >= tau
  float tau_below = (float)tau;
  if ((double)tau_below > tau) {             // rounded up: step to the next float below (finite here)
    const uint32_t u = __float_as_uint(tau_below);
    tau_below = tau_below > 0.0f ? __uint_as_float(u - 1u) : (tau_below < 0.0f ? __uint_as_float(u + 1u) : -1.401298464e-45f);
  }

  // Emit the targets in ascending order; lane e ends up holding edge e (k_max <= 64 on this path).
  int cnt = 0;
  double denom = 0.0;
  int my_tgt = -1;
  double my_c = 0.0;
  // A lane whose whole list is at or above tau may have seen more such values than it kept: only
  // then is the row read again.  Otherwise every target is in some lane's list, and the lists
  // are emptied in ascending slot order (slots are distinct) by repeated minimum search.
  const bool list_full = topj[MC - 1] >= 0 && (double)top[MC - 1] >= tau;
  const bool reread = __any(list_full);
  if (!reread) {
    bool open[MC];
#pragma unroll
    for (int k = 0; k < MC; ++k) open[k] = topj[k] >= 0 && (double)top[k] >= tau;
    for (;;) {
      int mine = 0x7fffffff, mk = 0;
#pragma unroll
      for (int k = 0; k < MC; ++k)
        if (open[k] && topj[k] < mine) { mine = topj[k]; mk = k; }
      const int mn = wave_reduce(mine, [](int x, int y) { return y < x ? y : x; });
      if (mn == 0x7fffffff) break;                               // uniform
      const bool owner = mine == mn;
      float vo = 0.0f;
#pragma unroll
      for (int k = 0; k < MC; ++k) {
        if (owner && k == mk) { vo = top[k]; open[k] = false; }
      }
      const int l = __ffsll(__ballot(owner)) - 1;
      const double cl = (double)lane_value(vo, l);
      const bool is_eq = cl == tau;
      const bool take = cl > tau || (is_eq && ties_seen < tie_quota);
      ties_seen += is_eq ? 1 : 0;
      if (take) {
        denom += cl;
        if (lane == cnt) { my_tgt = mn; my_c = cl; }
        ++cnt;
      }
    }
  }
  for (int r0 = 0; reread && r0 < a.N; r0 += kRowBatch * kWave) {
    if (a.N > kRowBatch * kWave || r0 > 0) load_batch(r0);     // a row of one batch is still in registers
    bool some = false;                                           // most batches hold no target at all
#pragma unroll
    for (int u = 0; u < kRowBatch; ++u) some |= sv[u] >= 0 && vv[u] >= tau_below;
    if (!__any(some)) continue;
#pragma unroll
    for (int u = 0; u < kRowBatch; ++u) {
      if (r0 + u * kWave >= a.N) break;                          // uniform; nothing is loaded past this point
      const double c = (double)vv[u];
      const bool in = sv[u] >= 0;
      const bool is_eq = in && c == tau;
      const unsigned long long eqm = __ballot(is_eq);
      const int eq_rank = ties_seen + __popcll(eqm & ((1ULL << lane) - 1ULL));
      ties_seen += __popcll(eqm);
      unsigned long long hit = __ballot(in && (c > tau || (is_eq && eq_rank < tie_quota)));
      while (hit) {
        const int l = __ffsll(hit) - 1;
        hit &= hit - 1;
        const double cl = lane_value(c, l);
        const int tl = lane_value(sv[u], l);
        denom += cl;
        if (lane == cnt) { my_tgt = tl; my_c = cl; }
        ++cnt;
      }
    }
  }
  const int stored = cnt < a.k_max ? cnt : a.k_max;
  const bool live = denom > 0.0;
  const int64_t ebase = (b * a.n_disc + row) * a.k_max;
  if (live && lane < stored) {
    const double al = my_c / denom;
    a.edge_tgt[ebase + lane] = my_tgt;
    a.edge_alpha[ebase + lane] = al;
    count_edge(a, b, row, my_tgt);
  }
  if (a.pair_tab) {              // uniform
    const double al = live && lane < stored ? my_c / denom : 0.0;
    const int t0 = lane_value(my_tgt, 0), t1 = lane_value(my_tgt, 1);
    const double a0 = lane_value(al, 0), a1 = lane_value(al, 1);
    if (lane == 0) write_pair(a, b, row, live ? stored : 0, i, t0, t1, a0, a1);
  }
  if (lane == 0) {
    a.edge_cnt[b * a.n_disc + row] = live ? stored : 0;
    if (live && cnt > a.k_max) a.overflow[b] = 1;
  }
}

// Pairwise token correlation gap: top-1 minus top-2 value of every discarded row, values
// evaluated exactly (one target per lane at a time), counted with multiplicity.
__global__ __launch_bounds__(256) void corr_gap_kernel(CorrArgs a) {
  const int lane = threadIdx.x % kWave;
  const int row = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
  const int64_t b = blockIdx.y;
  if (row >= a.n_disc) return;  // whole wavefront leaves together
  const int n = a.n_keep;
  const int i = a.S[b * a.n_disc + row];
  const double NEG = -__builtin_huge_val();
  double t1 = NEG, t2 = NEG;           // this lane's two largest values
  if ((unsigned)i < (unsigned)a.N) {
    for (int jj = lane; jj < n; jj += kWave) {
      const int j = a.T[b * n + jj];
      if ((unsigned)j >= (unsigned)a.N) continue;
      const double c = corr_value(a, b, i, j);
      if (c > t1) { t2 = t1; t1 = c; }
      else if (c > t2) t2 = c;
    }
  }
  const double m1 = wave_max(t1);
  const unsigned long long who = __ballot(t1 == m1);
  const bool owner = lane == __ffsll(who) - 1;
  const double m2 = wave_max(owner ? t2 : t1);   // the runner-up: the owner's second value or another lane's best
  if (lane == 0) a.gap[b * a.n_disc + row] = (n >= 2 && m2 > NEG) ? m1 - m2 : 0.0;
}

__global__ void zero_i32_kernel(int32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

static void launch_cand_rows(int sel_m, dim3 grid, dim3 block, hipStream_t s, const CorrArgs& a) {
  if (sel_m <= 2) hipLaunchKernelGGL(corr_cand_rows_kernel<2>, grid, block, 0, s, a);
  else if (sel_m <= 4) hipLaunchKernelGGL(corr_cand_rows_kernel<4>, grid, block, 0, s, a);
  else hipLaunchKernelGGL(corr_cand_rows_kernel<8>, grid, block, 0, s, a);
}

void launch_correlate(const ficoco_problem& p, const Plan& pl, char* ws, const int32_t* discard_idx,
                      const int32_t* keep_idx, int32_t* edge_cnt, int32_t* edge_tgt,
                      double* edge_alpha, int32_t* overflow, bool fused,
                      hipEvent_t gram_start, hipEvent_t gram_stop, hipStream_t s, int gram_repeat) {
  // fused: called from a fused step, whose filter stage cleared the overflow flags and whose
  // score stage formed the column maxima of the text profiles (text_stats_in_score)
  if (!fused)
    hipLaunchKernelGGL(zero_i32_kernel, dim3((p.B + 255) / 256), dim3(256), 0, s, overflow, p.B);
  const bool need_colmax = !(fused && text_stats_in_score(p));
  if (pl.n_disc == 0) return;
  if (pl.fixed_k == 0) {       // pruning / convergent form: no discarded token has a target
    const int n = p.B * pl.n_disc;
    hipLaunchKernelGGL(zero_i32_kernel, dim3((n + 255) / 256), dim3(256), 0, s, edge_cnt, n);
    return;
  }
  CorrArgs a{};
  a.B = p.B; a.N = p.N; a.n_keep = p.n_keep; a.n_disc = pl.n_disc; a.M = p.M; a.k_max = p.k_max; a.Df = pl.Df;
  const bool L = p.variant == FICOCO_VARIANT_L;
  a.mode = p.corr_src == FICOCO_C_ATTN ? (L ? kAttnL : kAttnV) : (L ? kCosL : kCosV);
  a.abar = (const float*)(ws + pl.abar);
  a.map_pitch = pl.map_pitch;
  a.ttext = (const double*)(ws + pl.ttext);
  a.xhat = (const bf16_t*)(ws + pl.xhat);
  a.gamma = (double)p.gamma;
  a.invM = p.M > 0 ? 1.0 / (double)p.M : 0.0;
  a.S = discard_idx; a.T = keep_idx;
  a.sel_m = pl.sel_m; a.sel_f = pl.sel_f; a.sel_g = pl.sel_g;
  a.dense = pl.dense_rows ? 1 : 0;
  a.rowbuf = (double*)(ws + pl.rowbuf);
  a.edge_cnt = edge_cnt; a.edge_tgt = edge_tgt; a.edge_alpha = edge_alpha; a.overflow = overflow;
  a.slot_of = (const int32_t*)(ws + pl.slot_of);
  a.ct = (float*)(ws + pl.ct);
  a.cmax = (double*)(ws + pl.cmax);
  a.fixed_k = pl.fixed_k;
  a.ct_splits = pl.gram_splits;
  a.delta = (float)(pl.Df + 4 * pl.gram_splits) * 2.384185791015625e-07f;   // (Df + 4 splits) * 2^-22
  if (fused && pair_records(p, pl)) a.pair_tab = (PairRec*)(ws + pl.pair_tab);
  if (fused && edges_inverted(pl)) {
    a.share_cnt = (int32_t*)(ws + pl.share_cnt);
    a.shares = invert_groups(pl);
    a.share_rows = invert_share_rows(pl);
  }
  dim3 grid((pl.n_disc + 3) / 4, p.B), block(256);
  if (a.mode == kAttnV && !pl.dense_rows && p.k_max <= kWave) {
    const bool wide = p.N > 10 * kWave;     // longer rows: wider batches (fewer dependent trips to memory)
    if (wide) {
      if (pl.sel_m <= 2) hipLaunchKernelGGL((corr_attn_rows_kernel<2, kRowWide>), grid, block, 0, s, a);
      else if (pl.sel_m <= 4) hipLaunchKernelGGL((corr_attn_rows_kernel<4, kRowWide>), grid, block, 0, s, a);
      else hipLaunchKernelGGL((corr_attn_rows_kernel<8, kRowWide>), grid, block, 0, s, a);
    } else {
      if (pl.sel_m <= 2) hipLaunchKernelGGL((corr_attn_rows_kernel<2, 10>), grid, block, 0, s, a);
      else if (pl.sel_m <= 4) hipLaunchKernelGGL((corr_attn_rows_kernel<4, 10>), grid, block, 0, s, a);
      else hipLaunchKernelGGL((corr_attn_rows_kernel<8, 10>), grid, block, 0, s, a);
    }
    return;
  }
  if (a.mode == kAttnL && !pl.dense_rows && p.k_max <= 64) {
    if (need_colmax) hipLaunchKernelGGL(text_colmax_kernel, dim3((p.M + 63) / 64, p.B), dim3(256), 0, s, a);
    launch_cand_rows(pl.sel_m, grid, block, s, a);
    return;
  }
  if (pl.use_gram) {
    GramArgs g{a.xhat, p.B, p.N, pl.Df, pl.n_disc, p.n_keep, discard_idx, keep_idx, a.ct, pl.gram_splits, pl.gram_st_per_split};
    const int tiles = pl.gram_splits * p.B * ((pl.n_disc + kGT - 1) / kGT) * ((p.n_keep + kGT - 1) / kGT);
    // large blocks (one K range, enough 256 x 192 tiles for most of the chip): the wide-tile form
    const int tiles2 = p.B * ((pl.n_disc + kG2M - 1) / kG2M) * ((p.n_keep + kG2N - 1) / kG2N);
    const bool wide = pl.gram_splits == 1 && tiles2 >= 128;
    if (gram_start) (void)hipEventRecord(gram_start, s);
    // gram_repeat > 1 (measurement only): the same launch again and again between the two events
    for (int rep = 0; rep < gram_repeat; ++rep) {
      if (wide) {
        const size_t lds = (size_t)2 * (kG2M + kG2N) * kG2Chunks * sizeof(uint4);
        (void)hipFuncSetAttribute((const void*)gram_tile2_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        hipLaunchKernelGGL(gram_tile2_kernel, dim3(xcd_padded_total(tiles2)), dim3(kG2Threads), lds, s, g);
      }
      else hipLaunchKernelGGL(gram_tile_kernel, dim3(xcd_padded_total(tiles)), dim3(256), 0, s, g);
    }
    if (gram_stop) (void)hipEventRecord(gram_stop, s);
    if (L && need_colmax) hipLaunchKernelGGL(text_colmax_kernel, dim3((p.M + 63) / 64, p.B), dim3(256), 0, s, a);
    launch_cand_rows(pl.sel_m, grid, block, s, a);
    return;
  }
  if (pl.dense_rows) hipLaunchKernelGGL(corr_fill_rows_kernel, grid, block, 0, s, a);
  hipLaunchKernelGGL(corr_rows_kernel, grid, block, 0, s, a);
}

void launch_corr_gap(const ficoco_problem& p, const Plan& pl, char* ws, const int32_t* discard_idx,
                     const int32_t* keep_idx, double* gap, hipStream_t s) {
  if (pl.n_disc == 0) return;
  CorrArgs a{};
  a.B = p.B; a.N = p.N; a.n_keep = p.n_keep; a.n_disc = pl.n_disc; a.M = p.M; a.k_max = p.k_max; a.Df = pl.Df;
  const bool L = p.variant == FICOCO_VARIANT_L;
  a.mode = p.corr_src == FICOCO_C_ATTN ? (L ? kAttnL : kAttnV) : (L ? kCosL : kCosV);
  a.abar = (const float*)(ws + pl.abar);
  a.map_pitch = pl.map_pitch;
  a.ttext = (const double*)(ws + pl.ttext);
  a.xhat = (const bf16_t*)(ws + pl.xhat);
  a.gamma = (double)p.gamma;
  a.invM = p.M > 0 ? 1.0 / (double)p.M : 0.0;
  a.S = discard_idx; a.T = keep_idx;
  a.gap = gap;
  hipLaunchKernelGGL(corr_gap_kernel, dim3((pl.n_disc + 3) / 4, p.B), dim3(256), 0, s, a);
}

}  // namespace ficoco

