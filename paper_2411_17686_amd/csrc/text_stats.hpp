// Statistics of the tokens' text profiles (FiCoCo-L): the body shared by select.hip (its own launch
// before the filter kernel) and features.hip (the fused step lets it ride in the launch of the
// column-sum kernel, which does not depend on it).
#pragma once
#include "common.hpp"

namespace ficoco {

// From 32 text queries on: the task term of Eq. 3, the mean of a token's text profile, is formed
// by one wavefront per token on the whole chip (lane sums over k = lane, lane + 64, ..., then a
// fixed tree), so the per-image workgroup of select_kernel reads one value.  A thread of that
// workgroup walking its token's profile touches a cache line per lane and load, all on one
// compute unit (64 queries: 17 us for the select kernel against 9 + 4 us this way).
// In the fused step the same launch also forms cmax[b][k], the maximum over the visual tokens of
// profile entry k (the bound of Eq. 4's indirect term that the correlate stage needs): the
// workgroups behind the first `mean_blocks` take 64 text queries of one image each, thread
// (k, g) walking the tokens g, g + 4, ... with 16 independent loads per round, the four token
// groups meeting in LDS.  Both are short chains of dependent loads on few workgroups; in one
// launch they overlap instead of following each other.
struct TextStatsArgs {
  const double* ttext;   // [B][N][M]
  int N, M;
  double* out_g;         // [B][N]
  double* cmax;          // [B][M], written by the workgroups behind the first mean_blocks (if any are launched)
  int mean_blocks;
};
void fill_text_stats(const ficoco_problem& p, const Plan& pl, char* ws, TextStatsArgs& t);
inline int text_stats_blocks(const TextStatsArgs& a, bool with_cmax) { return a.mean_blocks + (with_cmax ? (a.M + 63) / 64 : 0); }

__device__ __forceinline__ void text_stats_block(const TextStatsArgs& a, int bx, int64_t b) {
  __shared__ double part[256];
  const double* __restrict__ ttext = a.ttext;
  double* __restrict__ out_g = a.out_g;
  double* __restrict__ cmax = a.cmax;
  const int N = a.N, M = a.M, mean_blocks = a.mean_blocks;
  if (bx < mean_blocks) {
    const int lane = threadIdx.x % kWave;
    const int i = bx * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (i >= N) return;      // whole wavefront leaves together
    const double* p = ttext + (b * N + i) * M;
    double acc = 0.0;
    for (int k = lane; k < M; k += kWave) acc += p[k];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, kWave);
    if (lane == 0) out_g[b * N + i] = acc / (double)M;
    return;
  }
  const int tid = threadIdx.x;
  const int k = (bx - mean_blocks) * 64 + tid % 64, g = tid / 64;
  double mx = 0.0;
  if (k < M) {
    int i = g;
    for (; i + 4 * 15 < N; i += 4 * 16) {              // 16 independent loads per round
      double v[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) v[u] = ttext[(b * N + i + 4 * u) * M + k];
#pragma unroll
      for (int u = 0; u < 16; ++u) mx = v[u] > mx ? v[u] : mx;
    }
    for (; i < N; i += 4) { const double v = ttext[(b * N + i) * M + k]; mx = v > mx ? v : mx; }
  }
  part[tid] = mx;
  __syncthreads();
  if (g == 0 && k < M) {
    for (int q = 1; q < 4; ++q) mx = part[q * 64 + tid] > mx ? part[q * 64 + tid] : mx;
    cmax[b * M + k] = mx;
  }
}

}  // namespace ficoco
