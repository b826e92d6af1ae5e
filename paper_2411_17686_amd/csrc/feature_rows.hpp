// Row norms and bfloat16 unit rows of the feature rows: the body shared by the feature stage's own
// kernel (features.hip) and by the filter kernel's side workgroups (select.hip), which take this
// work along when no score term needs the features.
#pragma once
#include "common.hpp"

namespace ficoco {

struct FeatArgs {
  const void* F;
  int64_t sb, sn;
  int N, Df, f_chunks, f_rows_per_wg;
  double* norm;         // [B][N]
  bf16_t* xhat;         // [B][N][Df] or null
  double* colsum_part;  // [2][B][f_chunks][Df]  (0: unit rows, 1: raw rows)
  double* colmean;      // [2][B][Df]
  double* fterm_r;      // [B][N]
  double* fterm_g;      // [B][N]
  int want_sim, want_eq;
  int B;
};

__device__ __forceinline__ double wave_sum_d(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

// A row is read as 16-byte vectors, vector 64 * t + lane by lane `lane` in step t, KB steps in
// flight per lane.  Lanes past the last whole vector read vector 0 and clear what they got, so
// that the batch stays straight-line code.
template <typename T, int KB>
struct RowBatch {
  static constexpr int kVecs = KB;
  Raw8<T> raw[kVecs];
  __device__ __forceinline__ void load(const T* x, int t0, int n_vec, int lane) {
#pragma unroll
    for (int u = 0; u < kVecs; ++u) {
      const int idx = (t0 + u) * kWave + lane;
      load_raw(x + (idx < n_vec ? idx * kVec : 0), raw[u]);
    }
    issue_fence();
#pragma unroll
    for (int u = 0; u < kVecs; ++u) keep_raw_if(raw[u], (t0 + u) * kWave + lane < n_vec);
  }
};

// Feature source, norms and unit rows of a problem (the fields row_norm_row reads).
void fill_row_args(const ficoco_problem& p, const Plan& pl, char* ws, FeatArgs& a);

// One wavefront per row: |F_i| in double precision and, for the cosine correlation, the unit
// row rounded to bfloat16.  Rows of up to 64 * KB vectors are read once; longer ones are read
// again (from cache) for the unit row.  The launcher picks KB = 2, 4 or 8 by the row length (a
// batch wider than the row only adds loads that are thrown away).
template <typename T, int KB>
__device__ __forceinline__ void row_norm_row(const FeatArgs& a, int64_t b, int i, int lane) {
  const T* x = (const T*)a.F + b * a.sb + (int64_t)i * a.sn;
  const int n_vec = a.Df / kVec, Dv = n_vec * kVec;
  const int n_t = (n_vec + kWave - 1) / kWave;
  constexpr int kB = KB;
  RowBatch<T, KB> first, more;
  double ss = 0.0;
  auto add_squares = [&](const RowBatch<T, KB>& rb) {
#pragma unroll
    for (int u = 0; u < kB; ++u) {
      double v[kVec];
      widen_raw(rb.raw[u], v);
#pragma unroll
      for (int k = 0; k < kVec; ++k) ss += v[k] * v[k];
    }
  };
  if (n_t > 0) { first.load(x, 0, n_vec, lane); add_squares(first); }
  for (int t0 = kB; t0 < n_t; t0 += kB) { more.load(x, t0, n_vec, lane); add_squares(more); }
  for (int d = Dv + lane; d < a.Df; d += kWave) { const double v = widen(x[d]); ss += v * v; }
  ss = wave_sum_d(ss);
  const double nrm = sqrt(ss);
  if (lane == 0) a.norm[b * a.N + i] = nrm;
  if (a.xhat) {
    const double inv = nrm > 0.0 ? 1.0 / nrm : 0.0;
    bf16_t* o = a.xhat + (b * a.N + i) * (int64_t)a.Df;
    auto store_unit = [&](const RowBatch<T, KB>& rb, int t0) {
#pragma unroll
      for (int u = 0; u < kB; ++u) {
        const int idx = (t0 + u) * kWave + lane;
        if (idx < n_vec) {
          double v[kVec];
          widen_raw(rb.raw[u], v);
          Pack8<bf16_t> r;
#pragma unroll
          for (int k = 0; k < kVec; ++k) r.v[k] = to_bf16(v[k] * inv);
          __builtin_memcpy(o + idx * kVec, &r, sizeof(r));
        }
      }
    };
    if (n_t > 0) store_unit(first, 0);
    for (int t0 = kB; t0 < n_t; t0 += kB) { more.load(x, t0, n_vec, lane); store_unit(more, t0); }
    for (int d = Dv + lane; d < a.Df; d += kWave) o[d] = to_bf16(widen(x[d]) * inv);
  }
}

}  // namespace ficoco
