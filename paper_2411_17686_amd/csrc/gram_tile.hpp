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

// ---- the same product for large blocks ---------------------------------------------------------
// 256 x 192 output tile per workgroup of 8 wavefronts (4 x 2), 64 x 96 per wavefront = 2 x 3 blocks
// of v_mfma_f32_32x32x16_bf16: five fragment reads feed six matrix instructions (the 64 x 64 form
// above reads four for four), and every operand row is fetched by 6 (A) or 32 (B) workgroups
// instead of 9 and 63 at the 8064 x 1152 shape.  K is staged 64 features at a time (half the
// barriers of the 32-feature stages above).  LDS rows are the 128 bytes of a stage with no padding;
// the eight 16-byte chunks of row r sit at chunk ^ ((r >> 1) & 7), which makes both the loader's
// stores (consecutive lanes = consecutive chunks of consecutive rows) and the fragment reads
// (sixteen consecutive rows, one chunk) free of bank conflicts.
constexpr int kG2M = 256, kG2N = 192, kG2K = 64;
constexpr int kG2Threads = 512;
constexpr int kG2Chunks = kG2K / 8;        // 16-byte chunks per operand row and stage
__device__ __forceinline__ int g2_slot(int row, int chunk) { return row * kG2Chunks + (chunk ^ ((row >> 1) & 7)); }

__global__ __launch_bounds__(kG2Threads) void gram_tile2_kernel(GramArgs a) {
  static_assert(kG2Chunks == 8, "the swizzle spreads eight chunks");
  extern __shared__ uint4 g2_lds[];
  uint4* Abuf = g2_lds;                                   // [2][256 rows][8 chunks]
  uint4* Bbuf = g2_lds + 2 * kG2M * kG2Chunks;            // [2][192 rows][8 chunks]
  __shared__ int rowA[kG2M];
  __shared__ int rowB[kG2N];
  const int tid = threadIdx.x, lane = tid % kWave, wv = tid / kWave;
  const int tiles_m = (a.n_disc + kG2M - 1) / kG2M, tiles_n = (a.n_keep + kG2N - 1) / kG2N;
  const int total = a.B * tiles_m * tiles_n;
  const int logical = xcd_logical_id(blockIdx.x, total);     // the column tiles of the same rows share an XCD
  if (logical >= total) return;   // padding workgroup
  const int64_t b = logical / (tiles_m * tiles_n);
  const int tm = (logical % (tiles_m * tiles_n)) / tiles_n, tn = logical % tiles_n;

  if (tid < kG2M) {
    const int r = tm * kG2M + tid;
    const int i = r < a.n_disc ? a.S[b * a.n_disc + r] : -1;
    rowA[tid] = (unsigned)i < (unsigned)a.N ? i : -1;      // index sets are device data
  } else if (tid < kG2M + kG2N) {
    const int c = tn * kG2N + tid - kG2M;
    const int j = c < a.n_keep ? a.T[b * a.n_keep + c] : -1;
    rowB[tid - kG2M] = (unsigned)j < (unsigned)a.N ? j : -1;
  }
  __syncthreads();

  // loader: per stage 2048 chunks of A (four per thread) and 1536 of B (three per thread);
  // chunk q = (row q / 8, 16 bytes q % 8)
  const bf16_t* Xb = a.xhat + b * a.N * (int64_t)a.Df;
  constexpr int kSlotsA = kG2M * kG2Chunks / kG2Threads, kSlotsB = kG2N * kG2Chunks / kG2Threads;
  constexpr int kSlots = kSlotsA + kSlotsB;
  static_assert(kSlotsA * kG2Threads == kG2M * kG2Chunks && kSlotsB * kG2Threads == kG2N * kG2Chunks, "whole slots");
  // Every load of the loader is unconditional: a row past the block reads token 0 and a chunk past
  // the K range reads the row's first chunk (both valid addresses: N >= 1, Df >= 8), and what was
  // read is cleared when it is put into LDS.  Under a per-lane condition the loads sit in
  // branches, and the compiler then waits for ALL outstanding loads before it issues the next
  // stage's -- one stage in flight instead of two, and the wait at the head of every stage
  // (measured here: 33-35 -> 30-33 us; the 128 x 128 kernel above, with four loads per stage, is
  // no faster for it and keeps its conditional loads).
  const bf16_t* src[kSlots];
  bool row_ok[kSlots];
  int lds_at[kSlots], kc[kSlots];
#pragma unroll
  for (int u = 0; u < kSlots; ++u) {
    const bool aop = u < kSlotsA;
    const int q = tid + kG2Threads * (aop ? u : u - kSlotsA);
    const int row = q / kG2Chunks, chunk = q % kG2Chunks;
    const int tok = aop ? rowA[row] : rowB[row];
    kc[u] = chunk * 8;
    lds_at[u] = g2_slot(row, chunk);
    row_ok[u] = tok >= 0;
    src[u] = Xb + (int64_t)max(tok, 0) * a.Df;
  }
  uint4 rg[kGStages][kSlots];
  const int n_st = (a.Df + kG2K - 1) / kG2K;
  auto in_range = [&](int st, int u) { return st < n_st && st * kG2K + kc[u] + 8 <= a.Df; };   // Df is a multiple of 8 on this path
  auto fetch = [&](int slot, int st) {
#pragma unroll
    for (int u = 0; u < kSlots; ++u) __builtin_memcpy(&rg[slot][u], src[u] + (in_range(st, u) ? st * kG2K + kc[u] : 0), 16);
  };
  auto stash = [&](int slot, int buf, int st) {      // st: the stage that slot holds
#pragma unroll
    for (int u = 0; u < kSlots; ++u) {
      const uint4 v = row_ok[u] && in_range(st, u) ? rg[slot][u] : make_uint4(0, 0, 0, 0);
      if (u < kSlotsA) Abuf[buf * kG2M * kG2Chunks + lds_at[u]] = v;
      else Bbuf[buf * kG2N * kG2Chunks + lds_at[u]] = v;
    }
  };

  f32x16_t acc[2][3];
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 3; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;

  const int wm = wv / 2, wn = wv % 2;
  const int frow = lane % 32, fch = lane / 32;     // fragment: row within the block, 16-byte chunk within a 16-feature step
#pragma unroll
  for (int sl = 0; sl < kGStages; ++sl) fetch(sl, sl);
  stash(0, 0, 0);
  __syncthreads();
  int cur = 0;
  for (int base = 0; base < n_st; base += kGStages) {
#pragma unroll
    for (int sl = 0; sl < kGStages; ++sl) {
      const int it = base + sl;
      if (it < n_st) {                          // uniform over the workgroup
        fetch(sl, it + kGStages);               // slot sl was stashed one iteration ago
#pragma unroll
        for (int kk = 0; kk < kG2K / 16; ++kk) {
          bf16x8_t fa[2], fb[3];
#pragma unroll
          for (int mi = 0; mi < 2; ++mi) {
            const uint4 t = Abuf[cur * kG2M * kG2Chunks + g2_slot(wm * 64 + mi * 32 + frow, kk * 2 + fch)];
            __builtin_memcpy(&fa[mi], &t, 16);
          }
#pragma unroll
          for (int ni = 0; ni < 3; ++ni) {
            const uint4 t = Bbuf[cur * kG2N * kG2Chunks + g2_slot(wn * 96 + ni * 32 + frow, kk * 2 + fch)];
            __builtin_memcpy(&fb[ni], &t, 16);
          }
#pragma unroll
          for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int ni = 0; ni < 3; ++ni)
              acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[mi], fb[ni], acc[mi][ni], 0, 0, 0);
        }
        if (it + 1 < n_st) {
          stash((sl + 1) % kGStages, cur ^ 1, it + 1);  // the other buffer was last read before the previous barrier
          __syncthreads();
          cur ^= 1;
        }
      }
    }
  }

  // C block layout of the 32x32 MFMA: lane holds column lane%32; register v holds row
  // 8*(v/4) + 4*(lane/32) + v%4.
  float* ctb = a.ct + b * a.n_disc * (int64_t)a.n_keep;
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 3; ++ni) {
      const int col = tn * kG2N + wn * 96 + ni * 32 + lane % 32;
      const int row0 = tm * kG2M + wm * 64 + mi * 32 + 4 * (lane / 32);
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = row0 + 8 * (v / 4) + v % 4;
        if (row < a.n_disc && col < a.n_keep) ctb[(int64_t)row * a.n_keep + col] = acc[mi][ni][v];
      }
    }
}

}  // namespace ficoco
