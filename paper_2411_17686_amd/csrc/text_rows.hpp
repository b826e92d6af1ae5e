// Text-query block of FiCoCo-L: the body of the kernel that forms the tokens' text profiles, shared
// by attn_reduce.hip (its own launch) and features.hip (the fused step lets it ride in the launch
// of the row-norm kernel, which does not depend on it).
#pragma once
#include "common.hpp"

namespace ficoco {

constexpr int kHeadBatch = 8;

struct AttnArgs {
  const void* A;
  int64_t sb, sh, sq;
  int H;
  int row0, nrows;  // rows [row0, row0+nrows) of the block are visited
  int col0;         // column of visual key 0
  int N;
  int vis_r0, n_vis;  // rows of the visual queries (n_vis = 0: none)
  int cls_r;          // row of the [CLS] query or -1
  int M;              // text queries (text block only)
  float* abar;
  double* recv_part;
  double* cls;
  double* ttext;
  int rows_per_wg, n_chunks, row_lanes, strip_groups, col_strips, B;
  int shift;          // rows by which chunk 0 is shortened (visual row 0 starts a chunk)
  int map_pitch;      // floats per row of abar
  double invH;
};

// The text block of a problem as AttnArgs (the fields text_reduce_block reads), and its grid.
void fill_text_args(const ficoco_problem& p, const Plan& pl, char* ws, AttnArgs& a);
inline dim3 text_grid(const ficoco_problem& p);

// Text-query block of FiCoCo-L (task term of Eq. 3, profiles of Eq. 4): the head mean of
// A_text[b][h][k][i], stored TRANSPOSED as the token's profile ttext[b][i][k].  A workgroup
// owns 8 consecutive text rows x 256 key columns: a thread forms the head mean of one row and
// 8 columns exactly as the kernel above does (heads added in order, in double), the tile is
// turned in LDS, and each thread then writes the 8 rows of one column as one 64-byte piece.
constexpr int kTextHeadBatch = 16;
constexpr int kTextRows = 8;
constexpr int kTextGroups = 256 / kTextRows;      // 8-column groups per workgroup
template <typename T>
__device__ __forceinline__ void text_reduce_block(const AttnArgs& a, int chunk, int strip, int64_t b) {
  __shared__ double tile[kTextGroups * kVec][kTextRows + 1];     // +1: rows of one column in different banks
  const int tid = threadIdx.x;
  const int cg = tid % kTextGroups, rl = tid / kTextGroups;
  const int row = chunk * kTextRows + rl;
  const int col0 = strip * kTextGroups * kVec;
  const int col = col0 + cg * kVec;
  const int ncol = max(min(kVec, a.N - col), 0);
  if (row < a.M && ncol > 0) {
    const T* base = (const T*)a.A + b * a.sb + (int64_t)row * a.sq + a.col0 + col;
    double p[kVec];
#pragma unroll
    for (int k = 0; k < kVec; ++k) p[k] = 0.0;
    if (ncol == kVec) {
      int h0 = 0;
      // the grid of this kernel is small (8 rows x 256 keys per workgroup), so each thread keeps
      // more loads in flight than the map kernel does: kTextHeadBatch heads at a time
      for (; h0 + kTextHeadBatch <= a.H; h0 += kTextHeadBatch) {
        Raw8<T> raw[kTextHeadBatch];
#pragma unroll
        for (int u = 0; u < kTextHeadBatch; ++u) load_raw(base + (int64_t)(h0 + u) * a.sh, raw[u]);
        issue_fence();
#pragma unroll
        for (int u = 0; u < kTextHeadBatch; ++u) add_raw(raw[u], p);
      }
      for (; h0 + kHeadBatch <= a.H; h0 += kHeadBatch) {
        Raw8<T> raw[kHeadBatch];
#pragma unroll
        for (int u = 0; u < kHeadBatch; ++u) load_raw(base + (int64_t)(h0 + u) * a.sh, raw[u]);
#pragma unroll
        for (int u = 0; u < kHeadBatch; ++u) add_raw(raw[u], p);
      }
      for (; h0 < a.H; ++h0) {
        Raw8<T> raw;
        load_raw(base + (int64_t)h0 * a.sh, raw);
        add_raw(raw, p);
      }
    } else {
      for (int h = 0; h < a.H; ++h)
        for (int k = 0; k < ncol; ++k) p[k] += widen(base[(int64_t)h * a.sh + k]);
    }
#pragma unroll
    for (int k = 0; k < kVec; ++k) tile[cg * kVec + k][rl] = p[k] * a.invH;
  }
  __syncthreads();
  const int c = col0 + tid;                        // this thread's column
  if (c >= a.N) return;
  const int r0 = chunk * kTextRows;
  const int nr = min(kTextRows, a.M - r0);
  double* dst = a.ttext + ((int64_t)b * a.N + c) * a.M + r0;
  if (nr == kTextRows && a.M % 2 == 0) {           // 16-byte aligned pieces
#pragma unroll
    for (int k = 0; k < kTextRows; k += 2) {
      double2 v = make_double2(tile[tid][k], tile[tid][k + 1]);
      *reinterpret_cast<double2*>(dst + k) = v;
    }
  } else {
    for (int k = 0; k < nr; ++k) dst[k] = tile[tid][k];
  }
}

inline dim3 text_grid(const ficoco_problem& p) {
  return dim3((p.M + kTextRows - 1) / kTextRows, (p.N + kTextGroups * kVec - 1) / (kTextGroups * kVec), p.B);
}

}  // namespace ficoco
