// Feature-derived terms: row norms and bfloat16 unit rows (cosine correlation), the
// equivalent-token term -cos(mu, F_i) of the appendix "Implementation of the Equivalent
// Token", and the mean-cosine redundancy term (1/N) sum_j cos(F_i, F_j), evaluated as
// u_i . mean_j u_j with u = F / |F|.  Double precision throughout; column sums use a fixed
// two-level order (row chunks, then chunks) so results do not depend on scheduling.
#include "common.hpp"
#include "feature_rows.hpp"
#include "text_rows.hpp"
#include "text_stats.hpp"

namespace ficoco {

template <typename T, int KB>
__global__ __launch_bounds__(256) void row_norm_kernel(FeatArgs a) {
  const int lane = threadIdx.x % kWave;
  const int i = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
  if (i >= a.N) return;      // whole wavefront leaves together
  row_norm_row<T, KB>(a, blockIdx.y, i, lane);
}

// The same rows with the text-profile kernel of FiCoCo-L in the same launch: the first
// `text_blocks` workgroups (x fastest, then y, then image: tg = the text kernel's grid) form text
// profiles, the others take four rows each.  Neither needs anything from the other; as two
// launches the short text kernel stood in line before this one.
template <typename T, int KB>
__global__ __launch_bounds__(256) void rows_text_kernel(FeatArgs a, AttnArgs t, int text_blocks, int tgx, int tgy,
                                                        int row_blocks) {
  if ((int)blockIdx.x < text_blocks) {
    const int q = blockIdx.x;
    text_reduce_block<T>(t, q % tgx, (q / tgx) % tgy, q / (tgx * tgy));
    return;
  }
  const int rb = (int)blockIdx.x - text_blocks;
  const int i = (rb % row_blocks) * (blockDim.x / kWave) + threadIdx.x / kWave;
  if (i >= a.N) return;      // whole wavefront leaves together
  row_norm_row<T, KB>(a, rb / row_blocks, i, threadIdx.x % kWave);
}

// Partial column sums over a chunk of rows: slot 0 adds unit rows (row times the reciprocal of
// its norm), slot 1 raw rows.  A workgroup covers 512 features: a lane owns 8 consecutive
// ones, each of its four wavefronts takes a quarter of the chunk's rows (16-byte loads of up
// to kColBatch rows in flight, added in row order) and the quarters are added in order.
constexpr int kColBatch = 8;
constexpr int kColSpan = kWave * kVec;
template <typename T>
__device__ __forceinline__ void col_sum_block(const FeatArgs& a, int chunk, int span, int64_t b) {
  __shared__ double part[3][2][kVec][kWave];
  const int lane = threadIdx.x % kWave, wv = threadIdx.x / kWave;
  const int d = span * kColSpan + lane * kVec;
  const int nd = max(min(kVec, a.Df - d), 0);
  const int c0 = chunk * a.f_rows_per_wg, c1 = min(c0 + a.f_rows_per_wg, a.N);
  const int quarter = (c1 - c0 + 3) / 4;
  const int r0 = min(c0 + wv * quarter, c1), r1 = min(r0 + quarter, c1);
  const T* base = (const T*)a.F + b * a.sb + d;
  double su[kVec], sr[kVec];
#pragma unroll
  for (int k = 0; k < kVec; ++k) { su[k] = 0.0; sr[k] = 0.0; }
  if (nd == kVec) {
    for (int i0 = r0; i0 < r1; i0 += kColBatch) {
      Raw8<T> raw[kColBatch];
      double nrm[kColBatch];
#pragma unroll
      for (int u = 0; u < kColBatch; ++u) {
        const int i = min(i0 + u, r1 - 1);                 // clamped: always a valid row
        load_raw(base + (int64_t)i * a.sn, raw[u]);
        nrm[u] = a.norm[b * a.N + i];
      }
      issue_fence();                                       // all loads of the batch are issued before the first use
      // past the last row the clamped load is cleared, not skipped: a branch around its use
      // lets the compiler move the load down to it, one memory round trip per row
#pragma unroll
      for (int u = 0; u < kColBatch; ++u) {
        keep_raw_if(raw[u], i0 + u < r1);
        const double inv = nrm[u] > 0.0 ? 1.0 / nrm[u] : 0.0;
        double v[kVec];
        widen_raw(raw[u], v);
        if (a.want_sim) {                                  // uniform: only the sums some term needs
#pragma unroll
          for (int k = 0; k < kVec; ++k) su[k] += v[k] * inv;
        }
        if (a.want_eq) {
#pragma unroll
          for (int k = 0; k < kVec; ++k) sr[k] += v[k];
        }
      }
    }
  } else {
    for (int i = r0; i < r1; ++i) {
      const double nrm = a.norm[b * a.N + i];
      const double inv = nrm > 0.0 ? 1.0 / nrm : 0.0;
      for (int k = 0; k < nd; ++k) {
        const double v = widen(base[(int64_t)i * a.sn + k]);
        su[k] += v * inv;
        sr[k] += v;
      }
    }
  }
  if (wv > 0) {
#pragma unroll
    for (int k = 0; k < kVec; ++k) { part[wv - 1][0][k][lane] = su[k]; part[wv - 1][1][k][lane] = sr[k]; }
  }
  __syncthreads();
  if (wv > 0 || nd == 0) return;
#pragma unroll
  for (int w = 0; w < 3; ++w)
#pragma unroll
    for (int k = 0; k < kVec; ++k) { su[k] += part[w][0][k][lane]; sr[k] += part[w][1][k][lane]; }
  const int64_t slot = (int64_t)a.B * a.f_chunks * a.Df;
  double* pu = a.colsum_part + (b * a.f_chunks + chunk) * a.Df + d;
  for (int k = 0; k < nd; ++k) { pu[k] = su[k]; pu[slot + k] = sr[k]; }
}

template <typename T>
__global__ __launch_bounds__(256) void col_sum_kernel(FeatArgs a) { col_sum_block<T>(a, blockIdx.x, blockIdx.y, blockIdx.z); }

// The column sums with the statistics of the text profiles (FiCoCo-L) in the same launch: the first
// `stat_blocks * B` workgroups take the statistics, the others the column sums (chunk fastest,
// then feature span, then image).
template <typename T>
__global__ __launch_bounds__(256) void colsum_stats_kernel(FeatArgs a, TextStatsArgs t, int stat_blocks, int spans) {
  const int n_stat = stat_blocks * a.B;
  if ((int)blockIdx.x < n_stat) {
    text_stats_block(t, (int)blockIdx.x % stat_blocks, (int)blockIdx.x / stat_blocks);
    return;
  }
  const int q = (int)blockIdx.x - n_stat;
  col_sum_block<T>(a, q % a.f_chunks, (q / a.f_chunks) % spans, q / (a.f_chunks * spans));
}

// Column means from the chunk partials (added in chunk order, 8 loads in flight).  Every
// workgroup also leaves the squared norm of its 256 features of the raw mean (the equivalent
// token): colmean[2][B][Df], then munorm2[B][workgroups] behind it.
__global__ __launch_bounds__(256) void col_mean_kernel(FeatArgs a) {
  __shared__ double red[256];
  const int d = blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t b = blockIdx.y;
  const int64_t slot = (int64_t)a.B * a.f_chunks * a.Df;
  double mm = 0.0;
  if (d < a.Df) {
    const double* p = a.colsum_part + b * a.f_chunks * (int64_t)a.Df + d;
    double su = 0.0, sr = 0.0;
    for (int c = 0; c < a.f_chunks; c += 8) {     // past the last chunk the last one is loaded again and counted as zero
      double vu[8], vr[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int64_t at = (int64_t)min(c + u, a.f_chunks - 1) * a.Df;
        vu[u] = p[at];
        vr[u] = p[slot + at];
      }
      issue_fence();
#pragma unroll
      for (int u = 0; u < 8; ++u) { su += c + u < a.f_chunks ? vu[u] : 0.0; sr += c + u < a.f_chunks ? vr[u] : 0.0; }
    }
    const double mu = sr / (double)a.N;
    a.colmean[b * a.Df + d] = su / (double)a.N;
    a.colmean[(int64_t)a.B * a.Df + b * a.Df + d] = mu;
    mm = mu * mu;
  }
  if (!a.want_eq) return;          // uniform: only the equivalent-token term reads the squared norm
  red[threadIdx.x] = mm;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = 0.0;
    for (int k0 = 0; k0 < (int)blockDim.x; k0 += 16) {          // fixed order, sixteen reads at a time
      double v[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) v[u] = red[k0 + u];
#pragma unroll
      for (int u = 0; u < 16; ++u) t += v[u];
    }
    a.colmean[2 * (int64_t)a.B * a.Df + b * gridDim.x + blockIdx.x] = t;
  }
}

// u_i . mean(u) and F_i . mu in double precision for kFtRows rows per workgroup.  The two mean
// vectors are 16 bytes per feature, eight times a bfloat16 row: read once per row they, not the
// rows, set the kernel's duration.  So the four wavefronts of a workgroup share them over four
// rows: wavefront w takes the 64-vector steps w, w + 4, ... of all four rows (two steps in flight),
// lanes are summed by a fixed butterfly and the wavefronts in order through LDS.
constexpr int kFtRows = 4;
constexpr int kFtSteps = 2;
template <typename T>
__global__ __launch_bounds__(256) void feature_terms_kernel(FeatArgs a) {
  __shared__ double part[4][2][kFtRows];
  const int lane = threadIdx.x % kWave, wv = threadIdx.x / kWave;
  const int i0 = blockIdx.x * kFtRows;
  const int64_t b = blockIdx.y;
  const double* ubar = a.colmean + b * a.Df;
  const double* mu = a.colmean + (int64_t)a.B * a.Df + b * a.Df;
  const int n_vec = a.Df / kVec, Dv = n_vec * kVec;
  const int n_t = (n_vec + kWave - 1) / kWave;
  const T* x[kFtRows];
#pragma unroll
  for (int r = 0; r < kFtRows; ++r)
    x[r] = (const T*)a.F + b * a.sb + (int64_t)min(i0 + r, a.N - 1) * a.sn;     // clamped: a valid row, dropped at the end
  double du[kFtRows], dm[kFtRows];
#pragma unroll
  for (int r = 0; r < kFtRows; ++r) { du[r] = 0.0; dm[r] = 0.0; }
  for (int t0 = wv; t0 < n_t; t0 += 4 * kFtSteps) {
    Raw8<T> raw[kFtSteps][kFtRows];
    double w[kFtSteps][kVec], m[kFtSteps][kVec];
#pragma unroll
    for (int q = 0; q < kFtSteps; ++q) {
      const int idx = (t0 + 4 * q) * kWave + lane;
      const int d = idx < n_vec ? idx * kVec : 0;          // past the row: vector 0, cleared below
#pragma unroll
      for (int r = 0; r < kFtRows; ++r) load_raw(x[r] + d, raw[q][r]);
#pragma unroll
      for (int k = 0; k < kVec; ++k) { w[q][k] = a.want_sim ? ubar[d + k] : 0.0; m[q][k] = a.want_eq ? mu[d + k] : 0.0; }
    }
    issue_fence();
#pragma unroll
    for (int q = 0; q < kFtSteps; ++q) {
      const bool in = (t0 + 4 * q) * kWave + lane < n_vec;
#pragma unroll
      for (int r = 0; r < kFtRows; ++r) {
        keep_raw_if(raw[q][r], in);
        double v[kVec];
        widen_raw(raw[q][r], v);
        if (a.want_sim) {
#pragma unroll
          for (int k = 0; k < kVec; ++k) du[r] += v[k] * w[q][k];
        }
        if (a.want_eq) {
#pragma unroll
          for (int k = 0; k < kVec; ++k) dm[r] += v[k] * m[q][k];
        }
      }
    }
  }
  if (wv == 0) {                                            // the features behind the last whole vector
    for (int d = Dv + lane; d < a.Df; d += kWave) {
#pragma unroll
      for (int r = 0; r < kFtRows; ++r) {
        const double v = widen(x[r][d]);
        du[r] += v * ubar[d];
        dm[r] += v * mu[d];
      }
    }
  }
#pragma unroll
  for (int r = 0; r < kFtRows; ++r) { du[r] = wave_sum_d(du[r]); dm[r] = wave_sum_d(dm[r]); }
  if (lane == 0) {
#pragma unroll
    for (int r = 0; r < kFtRows; ++r) { part[wv][0][r] = du[r]; part[wv][1][r] = dm[r]; }
  }
  __syncthreads();
  const int r = threadIdx.x;
  if (r >= kFtRows || i0 + r >= a.N) return;
  const int i = i0 + r;
  double su = 0.0, sm = 0.0;
  for (int w4 = 0; w4 < 4; ++w4) { su += part[w4][0][r]; sm += part[w4][1][r]; }      // wavefronts in order
  const double nrm = a.norm[b * a.N + i];
  if (a.want_sim) a.fterm_r[b * a.N + i] = nrm > 0.0 ? su / nrm : 0.0;
  if (a.want_eq) {
    const int n_part = (a.Df + 255) / 256;
    double mm = 0.0;
    for (int k = 0; k < n_part; ++k) mm += a.colmean[2 * (int64_t)a.B * a.Df + b * n_part + k];
    const double mn = sqrt(mm);
    a.fterm_g[b * a.N + i] = (nrm > 0.0 && mn > 0.0) ? -(sm / (mn * nrm)) : 0.0;
  }
}

void fill_row_args(const ficoco_problem& p, const Plan& pl, char* ws, FeatArgs& a) {
  if (p.F) { a.F = p.F; a.sb = p.f_stride_b; a.sn = p.f_stride_n; }
  else {
    const size_t es = p.dtype == FICOCO_BF16 ? 2 : 4;
    a.F = (const char*)p.X + (size_t)p.vis_begin * p.x_stride_n * es;
    a.sb = p.x_stride_b; a.sn = p.x_stride_n;
  }
  a.N = p.N; a.Df = pl.Df; a.f_chunks = pl.f_chunks; a.f_rows_per_wg = pl.f_rows_per_wg; a.B = p.B;
  a.norm = (double*)(ws + pl.inv_norm);
  a.xhat = p.corr_src == FICOCO_C_COSINE ? (bf16_t*)(ws + pl.xhat) : nullptr;
}

void launch_features(const ficoco_problem& p, const Plan& pl, char* ws, hipStream_t s, bool with_text, bool with_cmax) {
  if (rows_with_filter(p, pl)) return;      // norms and unit rows only: the filter kernel's launch takes them along
  FeatArgs a{};
  fill_row_args(p, pl, ws, a);
  a.colsum_part = (double*)(ws + pl.colsum_part);
  a.colmean = (double*)(ws + pl.colmean);
  a.fterm_r = (double*)(ws + pl.fterm);
  a.fterm_g = (double*)(ws + pl.fterm2);
  a.want_sim = p.red_src == FICOCO_R_SIM_MEAN;
  a.want_eq = p.sem_src == FICOCO_G_EQ_TOKEN;
  const bool bf16 = p.dtype == FICOCO_BF16;
  dim3 rows((p.N + 3) / 4, p.B), block(256);
  const int steps = (pl.Df / kVec + kWave - 1) / kWave;    // 16-byte vectors per lane and row
  const int kb = steps <= 2 ? 2 : (steps <= 4 || !bf16) ? 4 : 8;
  if (with_text) {
    AttnArgs t{};
    fill_text_args(p, pl, ws, t);
    const dim3 tg = text_grid(p);
    const int text_blocks = tg.x * tg.y * tg.z, row_blocks = rows.x;
    const dim3 grid(text_blocks + row_blocks * p.B);
    auto go = [&](auto kern) { hipLaunchKernelGGL(kern, grid, block, 0, s, a, t, text_blocks, (int)tg.x, (int)tg.y, row_blocks); };
    if (bf16) { if (kb == 2) go(rows_text_kernel<bf16_t, 2>); else if (kb == 4) go(rows_text_kernel<bf16_t, 4>); else go(rows_text_kernel<bf16_t, 8>); }
    else { if (kb == 2) go(rows_text_kernel<float, 2>); else go(rows_text_kernel<float, 4>); }
  } else if (bf16) {
    if (kb == 2) hipLaunchKernelGGL((row_norm_kernel<bf16_t, 2>), rows, block, 0, s, a);
    else if (kb == 4) hipLaunchKernelGGL((row_norm_kernel<bf16_t, 4>), rows, block, 0, s, a);
    else hipLaunchKernelGGL((row_norm_kernel<bf16_t, 8>), rows, block, 0, s, a);
  } else {
    if (kb == 2) hipLaunchKernelGGL((row_norm_kernel<float, 2>), rows, block, 0, s, a);
    else hipLaunchKernelGGL((row_norm_kernel<float, 4>), rows, block, 0, s, a);
  }
  if (!a.want_sim && !a.want_eq) return;
  const int spans = (pl.Df + kColSpan - 1) / kColSpan;
  if (with_text) {
    TextStatsArgs t{};
    fill_text_stats(p, pl, ws, t);
    const int stat_blocks = text_stats_blocks(t, with_cmax);
    const dim3 grid(stat_blocks * p.B + pl.f_chunks * spans * p.B);
    if (bf16) hipLaunchKernelGGL(colsum_stats_kernel<bf16_t>, grid, block, 0, s, a, t, stat_blocks, spans);
    else hipLaunchKernelGGL(colsum_stats_kernel<float>, grid, block, 0, s, a, t, stat_blocks, spans);
  } else {
    dim3 cgrid(pl.f_chunks, spans, p.B);
    if (bf16) hipLaunchKernelGGL(col_sum_kernel<bf16_t>, cgrid, block, 0, s, a);
    else hipLaunchKernelGGL(col_sum_kernel<float>, cgrid, block, 0, s, a);
  }
  hipLaunchKernelGGL(col_mean_kernel, dim3((pl.Df + 255) / 256, p.B), block, 0, s, a);
  const dim3 trows((p.N + kFtRows - 1) / kFtRows, p.B);
  if (bf16) hipLaunchKernelGGL(feature_terms_kernel<bf16_t>, trows, block, 0, s, a);
  else hipLaunchKernelGGL(feature_terms_kernel<float>, trows, block, 0, s, a);
}

}  // namespace ficoco
