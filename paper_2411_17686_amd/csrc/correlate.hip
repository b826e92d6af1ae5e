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

namespace ficoco {

enum CorrMode { kAttnV = 0, kAttnL = 1, kCosV = 2, kCosL = 3 };

struct CorrArgs {
  int N, n_keep, n_disc, M, k_max, Df, mode;
  const float* abar;     // [B][N][N]
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
};

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
    direct = (double)a.abar[(b * a.N + j) * a.N + i];
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
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const double o = __shfl_xor(v, off, kWave);
    v = o > v ? o : v;
  }
  return v;
}
__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
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

__global__ __launch_bounds__(256) void corr_rows_kernel(CorrArgs a) {
  const int lane = threadIdx.x % kWave;
  const int row = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
  const int64_t b = blockIdx.y;
  if (row >= a.n_disc) return;  // whole wavefront leaves together
  const int n = a.n_keep;
  const int i = a.S[b * a.n_disc + row];
  const int32_t* T = a.T + b * n;
  if ((unsigned)i >= (unsigned)a.N) {  // index sets are device data: never index with a bad one
    if (lane == 0) a.edge_cnt[b * a.n_disc + row] = 0;
    return;
  }
  const double* rowv = a.dense ? a.rowbuf + (b * a.n_disc + row) * n : nullptr;
  const double NEG = -__builtin_huge_val();

  double v_f, v_f1;
  if (a.dense) {
    v_f = select_rank(rowv, n, a.sel_f, lane);
    v_f1 = a.sel_f + 1 <= n - 1 ? select_rank(rowv, n, a.sel_f + 1, lane) : v_f;
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
      v_f1 = v_f;
      v_f = mx;
    }
    if (a.sel_m == 1) v_f1 = v_f;
  }
  const double tau = threshold_of(v_f, v_f1, a.sel_g);

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
    unsigned long long hit = __ballot(jj < n && c >= tau);
    while (hit) {
      const int l = __ffsll(hit) - 1;
      hit &= hit - 1;
      const double cl = __shfl(c, l, kWave);
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
      a.edge_tgt[ebase + lane] = my_tgt;
      a.edge_alpha[ebase + lane] = my_c / denom;
    }
  } else if (live && lane == 0) {
    for (int e = 0; e < stored; ++e) a.edge_alpha[ebase + e] = a.edge_alpha[ebase + e] / denom;
  }
  if (lane == 0) {
    a.edge_cnt[b * a.n_disc + row] = live ? stored : 0;
    if (live && cnt > a.k_max) a.overflow[b] = 1;
  }
}


// ---- FiCoCo-V attention correlation, tiled ----------------------------------------------------
// The generic kernel above gathers one column of the row-major head-mean map per wavefront
// (64 different rows per load).  For the plain attention correlation of Algorithm 1 this
// tile kernel is used instead: a workgroup owns kTileCols discarded columns, thread
// (c, jl) scans rows T[jl], T[jl + kTileLanes], ... of column S[c], so the threads of one
// row read neighbouring columns of the same row.  Pass 1 keeps the m largest values per
// thread, LDS merges them per column into v[f], v[f+1] and tau; pass 2 re-reads the (cache
// resident) column and collects the rows at or above tau.
constexpr int kTileCols = 8;
constexpr int kTileLanes = 32;
constexpr int kHitCap = 64;

__global__ __launch_bounds__(kTileCols * kTileLanes) void corr_attn_tile_kernel(CorrArgs a) {
  __shared__ float cand[kTileCols][kTileLanes][kSelMax];
  __shared__ double tau_s[kTileCols];
  __shared__ int hit_cnt[kTileCols];
  __shared__ int hit_j[kTileCols][kHitCap];
  __shared__ float hit_v[kTileCols][kHitCap];
  const int tid = threadIdx.x;
  const int c = tid % kTileCols, jl = tid / kTileCols;
  const int64_t b = blockIdx.y;
  const int row = blockIdx.x * kTileCols + c;
  const int n = a.n_keep;
  const int32_t* T = a.T + b * n;
  int i = row < a.n_disc ? a.S[b * a.n_disc + row] : -1;
  const bool valid = (unsigned)i < (unsigned)a.N;   // index sets are device data
  if (!valid) i = 0;
  const float* col = a.abar + b * a.N * (int64_t)a.N + i;
  const float NEGF = -__builtin_huge_valf();

  float top[kSelMax];
#pragma unroll
  for (int k = 0; k < kSelMax; ++k) top[k] = NEGF;
  if (valid) {
    for (int jj = jl; jj < n; jj += kTileLanes) {
      const int j = T[jj];
      float v = (unsigned)j < (unsigned)a.N ? col[(int64_t)j * a.N] : NEGF;
      if (v > top[kSelMax - 1]) {
#pragma unroll
        for (int k = 0; k < kSelMax; ++k) {
          const bool sw = v > top[k];
          const float t = top[k];
          top[k] = sw ? v : t;
          v = sw ? t : v;
        }
      }
    }
  }
#pragma unroll
  for (int k = 0; k < kSelMax; ++k) cand[c][jl][k] = top[k];
  __syncthreads();
  if (jl == 0) {
    float best[kSelMax];
#pragma unroll
    for (int k = 0; k < kSelMax; ++k) best[k] = NEGF;
    for (int l = 0; l < kTileLanes; ++l)
      for (int q = 0; q < a.sel_m; ++q) {
        float v = cand[c][l][q];
        if (v > best[kSelMax - 1]) {
#pragma unroll
          for (int k = 0; k < kSelMax; ++k) {
            const bool sw = v > best[k];
            const float t = best[k];
            best[k] = sw ? v : t;
            v = sw ? t : v;
          }
        }
      }
    float vf = NEGF, vf1 = NEGF;     // m-th and (m-1)-th largest
#pragma unroll
    for (int k = 0; k < kSelMax; ++k) {
      if (k == a.sel_m - 1) vf = best[k];
      if (k == a.sel_m - 2) vf1 = best[k];
    }
    if (a.sel_m == 1) vf1 = vf;
    tau_s[c] = threshold_of((double)vf, (double)vf1, a.sel_g);
    hit_cnt[c] = 0;
  }
  __syncthreads();
  if (valid) {
    const double tau = tau_s[c];
    for (int jj = jl; jj < n; jj += kTileLanes) {
      const int j = T[jj];
      if ((unsigned)j >= (unsigned)a.N) continue;
      const float v = col[(int64_t)j * a.N];
      if ((double)v >= tau) {
        const int slot = atomicAdd(&hit_cnt[c], 1);
        if (slot < kHitCap) { hit_j[c][slot] = jj; hit_v[c][slot] = v; }
      }
    }
  }
  __syncthreads();
  if (jl == 0 && row < a.n_disc) {
    const int cnt = valid ? hit_cnt[c] : 0;
    const int have = cnt < kHitCap ? cnt : kHitCap;
    for (int x = 1; x < have; ++x) {          // ascending target slot (arrival order is arbitrary)
      const int jx = hit_j[c][x];
      const float vx = hit_v[c][x];
      int y = x - 1;
      while (y >= 0 && hit_j[c][y] > jx) { hit_j[c][y + 1] = hit_j[c][y]; hit_v[c][y + 1] = hit_v[c][y]; --y; }
      hit_j[c][y + 1] = jx;
      hit_v[c][y + 1] = vx;
    }
    double denom = 0.0;
    for (int x = 0; x < have; ++x) denom += (double)hit_v[c][x];
    const bool live = denom > 0.0;
    const int stored = have < a.k_max ? have : a.k_max;
    const int64_t ebase = (b * a.n_disc + row) * a.k_max;
    if (live)
      for (int x = 0; x < stored; ++x) {
        a.edge_tgt[ebase + x] = hit_j[c][x];
        a.edge_alpha[ebase + x] = (double)hit_v[c][x] / denom;
      }
    a.edge_cnt[b * a.n_disc + row] = live ? stored : 0;
    if (live && cnt > a.k_max) a.overflow[b] = 1;
  }
}

__global__ void zero_i32_kernel(int32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

void launch_correlate(const ficoco_problem& p, const Plan& pl, char* ws, const int32_t* discard_idx,
                      const int32_t* keep_idx, int32_t* edge_cnt, int32_t* edge_tgt,
                      double* edge_alpha, int32_t* overflow, bool overflow_is_zero, hipStream_t s) {
  if (!overflow_is_zero)
    hipLaunchKernelGGL(zero_i32_kernel, dim3((p.B + 255) / 256), dim3(256), 0, s, overflow, p.B);
  if (pl.n_disc == 0) return;
  CorrArgs a{};
  a.N = p.N; a.n_keep = p.n_keep; a.n_disc = pl.n_disc; a.M = p.M; a.k_max = p.k_max; a.Df = pl.Df;
  const bool L = p.variant == FICOCO_VARIANT_L;
  a.mode = p.corr_src == FICOCO_C_ATTN ? (L ? kAttnL : kAttnV) : (L ? kCosL : kCosV);
  a.abar = (const float*)(ws + pl.abar);
  a.ttext = (const double*)(ws + pl.ttext);
  a.xhat = (const bf16_t*)(ws + pl.xhat);
  a.gamma = (double)p.gamma;
  a.invM = p.M > 0 ? 1.0 / (double)p.M : 0.0;
  a.S = discard_idx; a.T = keep_idx;
  a.sel_m = pl.sel_m; a.sel_f = pl.sel_f; a.sel_g = pl.sel_g;
  a.dense = pl.dense_rows ? 1 : 0;
  a.rowbuf = (double*)(ws + pl.rowbuf);
  a.edge_cnt = edge_cnt; a.edge_tgt = edge_tgt; a.edge_alpha = edge_alpha; a.overflow = overflow;
  if (a.mode == kAttnV && !pl.dense_rows && p.k_max <= kHitCap) {
    dim3 tgrid((pl.n_disc + kTileCols - 1) / kTileCols, p.B);
    hipLaunchKernelGGL(corr_attn_tile_kernel, tgrid, dim3(kTileCols * kTileLanes), 0, s, a);
    return;
  }
  dim3 grid((pl.n_disc + 3) / 4, p.B), block(256);
  if (pl.dense_rows) hipLaunchKernelGGL(corr_fill_rows_kernel, grid, block, 0, s, a);
  hipLaunchKernelGGL(corr_rows_kernel, grid, block, 0, s, a);
}

}  // namespace ficoco
