// bf16 MFMA tile kernel for the cosine correlation (the one dense contraction of the path):
//   Ct[b][a][j] = xh[b][S[b][a]] . xh[b][T[b][j]]      (float accumulation)
// for the discarded rows a and preserved columns j of every image, xh = unit rows rounded to
// bfloat16.  The result only PROPOSES candidates: every value that can decide a threshold
// is afterwards recomputed in double precision, so the order in which the matrix core adds
// does not matter for the outcome.
//
// 128 x 128 output tile per workgroup (4 wavefronts, 64 x 64 each = 2 x 2 blocks of
// v_mfma_f32_32x32x16_bf16), K staged through LDS 32 at a time,
// double buffered, rows gathered by index.  LDS rows are padded by 16 bytes so that the
// 16-byte fragment reads of a quarter wavefront fall on distinct banks.
#pragma once
#include "common.hpp"

namespace ficoco {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kGT = 128;           // tile rows = tile columns
constexpr int kGK = kGramStage;    // K elements per stage (32 measured best at 4096 tokens; 64 halves LDS occupancy)
constexpr int kGChunks = kGK / 16;  // 16-byte chunks per thread, operand and stage
constexpr int kGStride = kGK + 8;  // LDS row pitch in elements (row + 16 bytes)
constexpr int kGStages = 2;   // K-stages in flight per thread (register ring)

struct GramArgs {
  const bf16_t* xhat;  // [B][N][Df]
  int B, N, Df, n_disc, n_keep;
  const int32_t* S;    // [B][n_disc]
  const int32_t* T;    // [B][n_keep]
  float* ct;           // [splits][B][n_disc][n_keep]: partial sums over the K ranges of the splits
  int splits, st_per_split;   // K is cut into `splits` ranges of st_per_split stages (the last may be shorter)
};

__global__ __launch_bounds__(256) void gram_tile_kernel(GramArgs a) {
  __shared__ __attribute__((aligned(16))) bf16_t As[2][kGT * kGStride];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[2][kGT * kGStride];
  __shared__ int rowA[kGT];
  __shared__ int rowB[kGT];
  const int tid = threadIdx.x, lane = tid % kWave, wv = tid / kWave;
  const int tiles_m = (a.n_disc + kGT - 1) / kGT, tiles_n = (a.n_keep + kGT - 1) / kGT;
  const int per_split = a.B * tiles_m * tiles_n;
  const int total = per_split * a.splits;
  int logical = xcd_logical_id(blockIdx.x, total);
  if (logical >= total) return;   // padding workgroup
  const int split = logical / per_split;
  logical %= per_split;
  const int64_t b = logical / (tiles_m * tiles_n);
  const int tm = (logical % (tiles_m * tiles_n)) / tiles_n, tn = logical % tiles_n;

  if (tid < kGT) {
    const int r = tm * kGT + tid;
    const int i = r < a.n_disc ? a.S[b * a.n_disc + r] : -1;
    rowA[tid] = (unsigned)i < (unsigned)a.N ? i : -1;      // index sets are device data
  } else {
    const int c = tn * kGT + tid - kGT;
    const int j = c < a.n_keep ? a.T[b * a.n_keep + c] : -1;
    rowB[tid - kGT] = (unsigned)j < (unsigned)a.N ? j : -1;
  }
  __syncthreads();

  // this split's K range, [k_begin, k_begin + k_len)
  const int k_begin = split * a.st_per_split * kGK;
  const int k_len = max(min(a.Df - k_begin, a.st_per_split * kGK), 0);
  // loader: the stage is 128 rows x kGK/8 chunks of 8 elements per operand; thread -> kGChunks chunks each
  const bf16_t* Xb = a.xhat + b * a.N * (int64_t)a.Df + k_begin;
  int lrow[kGChunks], lkc[kGChunks];
  const bf16_t* srcA[kGChunks];
  const bf16_t* srcB[kGChunks];
#pragma unroll
  for (int u = 0; u < kGChunks; ++u) {
    const int q = tid + 256 * u;
    lrow[u] = q / (kGK / 8);
    lkc[u] = (q % (kGK / 8)) * 8;
    srcA[u] = rowA[lrow[u]] >= 0 ? Xb + (int64_t)rowA[lrow[u]] * a.Df + lkc[u] : nullptr;
    srcB[u] = rowB[lrow[u]] >= 0 ? Xb + (int64_t)rowB[lrow[u]] * a.Df + lkc[u] : nullptr;
  }
  // Register ring of kGStages K-stages in flight per thread: a stage is fetched kGStages
  // iterations before it is stashed into LDS.
  uint4 ra[kGStages][kGChunks], rb[kGStages][kGChunks];
  const int n_st = (k_len + kGK - 1) / kGK;
  auto fetch = [&](int slot, int st) {
    const int k0 = st * kGK;
#pragma unroll
    for (int u = 0; u < kGChunks; ++u) {
      const bool in = st < n_st && k0 + lkc[u] + 8 <= k_len;   // Df is a multiple of 8 on this path
      ra[slot][u] = make_uint4(0, 0, 0, 0);
      rb[slot][u] = make_uint4(0, 0, 0, 0);
      if (in && srcA[u]) __builtin_memcpy(&ra[slot][u], srcA[u] + k0, 16);
      if (in && srcB[u]) __builtin_memcpy(&rb[slot][u], srcB[u] + k0, 16);
    }
  };
  auto stash = [&](int slot, int buf) {
#pragma unroll
    for (int u = 0; u < kGChunks; ++u) {
      *reinterpret_cast<uint4*>(&As[buf][lrow[u] * kGStride + lkc[u]]) = ra[slot][u];
      *reinterpret_cast<uint4*>(&Bs[buf][lrow[u] * kGStride + lkc[u]]) = rb[slot][u];
    }
  };

  f32x16_t acc[2][2];
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;

  const int wm = wv / 2, wn = wv % 2;
  const int frow = lane % 32, fk = (lane / 32) * 8;   // fragment: row / column within the block, k offset
#pragma unroll
  for (int sl = 0; sl < kGStages; ++sl) fetch(sl, sl);
  stash(0, 0);
  __syncthreads();
  int cur = 0;
  for (int base = 0; base < n_st; base += kGStages) {
#pragma unroll
    for (int sl = 0; sl < kGStages; ++sl) {
      const int it = base + sl;
      if (it < n_st) {                          // uniform over the workgroup
        fetch(sl, it + kGStages);               // slot sl was stashed one iteration ago
#pragma unroll
        for (int kk = 0; kk < kGK; kk += 16) {
          bf16x8_t fa[2], fb[2];
#pragma unroll
          for (int mi = 0; mi < 2; ++mi)
            fa[mi] = *reinterpret_cast<const bf16x8_t*>(&As[cur][(wm * 64 + mi * 32 + frow) * kGStride + kk + fk]);
#pragma unroll
          for (int ni = 0; ni < 2; ++ni)
            fb[ni] = *reinterpret_cast<const bf16x8_t*>(&Bs[cur][(wn * 64 + ni * 32 + frow) * kGStride + kk + fk]);
#pragma unroll
          for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
              acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[mi], fb[ni], acc[mi][ni], 0, 0, 0);
        }
        if (it + 1 < n_st) {
          stash((sl + 1) % kGStages, cur ^ 1);  // the other buffer was last read before the previous barrier
          __syncthreads();
          cur ^= 1;
        }
      }
    }
  }

  // C block layout of the 32x32 MFMA: lane holds column lane%32; register v holds row
  // 8*(v/4) + 4*(lane/32) + v%4.
  float* ctb = a.ct + ((int64_t)split * a.B + b) * a.n_disc * (int64_t)a.n_keep;   // this split's block of image b
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
      const int col = tn * kGT + wn * 64 + ni * 32 + lane % 32;
      const int row0 = tm * kGT + wm * 64 + mi * 32 + 4 * (lane / 32);
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = row0 + 8 * (v / 4) + v % 4;
        if (row < a.n_disc && col < a.n_keep) ctb[row * a.n_keep + col] = acc[mi][ni][v];   // below 2^31: n_disc * n_keep < 12288^2
      }
    }
}

}  // namespace ficoco
