// Attention-map reduction: the one pass over the [B,H,Nq,Nk] maps.
//
// For every query row that carries a role the head mean  Pbar[q][k] = (1/H) sum_h P[h][q][k]
// is formed in double precision, heads added in order (so the value does not depend on the
// launch shape), and consumed three ways:
//   visual query : added into the per-column received-attention partial of this row chunk
//                  (first term of Eq. 1 / Eq. 3) and stored in single precision as the map
//                  the correlate stage gathers from (Algorithm 1, stage 2);
//   [CLS] query  : stored as the semantic term of Eq. 1;
//   text query   : stored transposed as the token's text-attention profile (task term of
//                  Eq. 3 and indirect term of Eq. 4) -- by text_reduce_kernel below.
// HBM-bound: each lane streams 8 consecutive key columns of one row for all heads with
// 16-byte loads; rows of a dense map with an odd length are only element aligned, the
// hardware's unaligned dwordx4 access is relied on for those.
#include "common.hpp"
#include "text_rows.hpp"

namespace ficoco {

constexpr int kRowsAtOnce = 4;     // rows of one thread whose heads are added side by side ...
constexpr int kHeadsAtOnce = 2;    // ... this many heads of each per batch of loads (more where the thread has fewer rows)


// Three wavefronts per SIMD (170 registers): the four-row form keeps 32 double accumulators and 8
// raw vectors per thread, and its grids hold about three wavefronts per SIMD anyway.
template <typename T>
__global__ __launch_bounds__(kReduceThreads) __attribute__((amdgpu_waves_per_eu(3))) void attn_reduce_kernel(AttnArgs a) {
  extern __shared__ double lds[];
  // Workgroups that read neighbouring strips of the same rows share the cache lines at the
  // strip boundaries: they get consecutive logical ids, which run on the same XCD (one L2).
  const int total = a.n_chunks * a.col_strips * a.B;
  const int logical = xcd_logical_id(blockIdx.x, total);
  if (logical >= total) return;                   // padding workgroup (the whole block leaves)
  const int strip = logical % a.col_strips;
  const int chunk = (logical / a.col_strips) % a.n_chunks;
  const int b = logical / (a.col_strips * a.n_chunks);
  const int tid = threadIdx.x;
  const int cg = tid % a.strip_groups, rl = tid / a.strip_groups;
  const int col = (strip * a.strip_groups + cg) * kVec;
  const int ncol = min(kVec, a.N - col);
  const bool active = rl < a.row_lanes && ncol > 0;

  // Where this thread leaves its column partial for the combination of the row lanes.
  const int width = a.strip_groups * kVec;
  double* mine = lds + (rl < a.row_lanes ? rl : 0) * width + cg * kVec;

  // The head-mean map leaves transposed (abar[key token][query token], what the correlate stage
  // reads row by row): this workgroup's tile, strip columns x chunk rows, is turned in LDS and
  // written as one piece of rows_per_wg floats per key column.
  float* tile = (float*)(lds + a.row_lanes * width);
  const int tile_pitch = a.rows_per_wg + 1;           // odd: the 8 columns of a lane fall into different banks
  const int r_begin = a.row0 + chunk * a.rows_per_wg - a.shift;   // chunk 0 may begin before row0
  const int r_end = min(r_begin + a.rows_per_wg, a.row0 + a.nrows);

  // This thread's column partial over its rows (rows in ascending order, from zero): kept in
  // registers and handed to LDS once -- a read-modify-write of LDS per row sat on every
  // workgroup's critical path (2 us of the kernel at the batched ViT shape).
  double colsum[kVec];
#pragma unroll
  for (int k = 0; k < kVec; ++k) colsum[k] = 0.0;
  // What is done with the head mean of one (row, 8 columns) once its heads are added.
  auto finish_row = [&](int r, bool is_vis, bool is_cls, double (&p)[kVec]) __attribute__((always_inline)) {
#pragma unroll
    for (int k = 0; k < kVec; ++k) p[k] *= a.invH;
    if (is_vis) {
#pragma unroll
      for (int k = 0; k < kVec; ++k) colsum[k] += p[k];
      if (a.abar) {
        float* dst = tile + (cg * kVec) * tile_pitch + (r - r_begin);
#pragma unroll
        for (int k = 0; k < kVec; ++k) dst[k * tile_pitch] = (float)p[k];   // columns past N are never read back
      }
    }
    if (is_cls) {
      double* dst = a.cls + (int64_t)b * a.N + col;
      for (int k = 0; k < ncol; ++k) dst[k] = p[k];
    }
  };

  const int rows_per_thread = (a.rows_per_wg + a.row_lanes - 1) / a.row_lanes;
  if (sizeof(T) == 2 && rows_per_thread <= kRowsAtOnce) {     // uniform
    // All rows of this thread at once, heads outermost: a batch is a few heads of each of the
    // thread's rows.  The loads in flight then come from a few rows of one or two head
    // matrices -- neighbouring addresses -- instead of one row of eight matrices 665 KB apart,
    // which the memory system serves measurably faster; every (row, column) still adds its
    // heads in ascending order, so the sums are the same doubles.  Loads are unconditional and
    // from valid addresses (rows outside the chunk read its nearest row, heads past H read head
    // H-1) and what does not count is cleared with selects.
    if (active && ncol == kVec) {
      const T* Ab = (const T*)a.A + (int64_t)b * a.sb + a.col0 + col;
      // ROWS = rows of this thread (compile time: the accumulators are registers)
      auto run = [&](auto rows_c) __attribute__((always_inline)) {
        constexpr int ROWS = decltype(rows_c)::value;
        constexpr int HEADS = ROWS >= 3 ? kHeadsAtOnce : kHeadBatch / ROWS;   // about kHeadBatch loads in flight
        double p[ROWS][kVec];
        const T* base[ROWS];
#pragma unroll
        for (int q = 0; q < ROWS; ++q) {
          const int r = r_begin + rl + q * a.row_lanes;
          base[q] = Ab + (int64_t)min(max(r, a.row0), a.row0 + a.nrows - 1) * a.sq;
#pragma unroll
          for (int k = 0; k < kVec; ++k) p[q][k] = 0.0;
        }
        for (int h0 = 0; h0 < a.H; h0 += HEADS) {
          Raw8<T> raw[HEADS][ROWS];
#pragma unroll
          for (int u = 0; u < HEADS; ++u) {
            const int64_t hoff = (int64_t)min(h0 + u, a.H - 1) * a.sh;
#pragma unroll
            for (int q = 0; q < ROWS; ++q) load_raw(base[q] + hoff, raw[u][q]);
          }
          issue_fence();
#pragma unroll
          for (int u = 0; u < HEADS; ++u)
#pragma unroll
            for (int q = 0; q < ROWS; ++q) {
              keep_raw_if(raw[u][q], h0 + u < a.H);
              add_raw(raw[u][q], p[q]);
            }
        }
#pragma unroll
        for (int q = 0; q < ROWS; ++q) {
          const int r = r_begin + rl + q * a.row_lanes;
          const bool is_vis = r >= a.vis_r0 && r < a.vis_r0 + a.n_vis;
          const bool is_cls = r == a.cls_r;
          if (r < r_end && r >= a.row0 && (is_vis || is_cls)) {
#pragma unroll
            for (int k = 0; k < kVec; ++k) p[q][k] *= a.invH;
            if (is_vis) {
#pragma unroll
              for (int k = 0; k < kVec; ++k) colsum[k] += p[q][k];      // rows in ascending order, from zero
              if (a.abar) {
                float* dst = tile + (cg * kVec) * tile_pitch + (r - r_begin);
#pragma unroll
                for (int k = 0; k < kVec; ++k) dst[k * tile_pitch] = (float)p[q][k];
              }
            }
            if (is_cls) {
              double* dst = a.cls + (int64_t)b * a.N + col;
#pragma unroll
              for (int k = 0; k < kVec; ++k) dst[k] = p[q][k];
            }
          }
        }
      };
      if (rows_per_thread <= 1) run(std::integral_constant<int, 1>{});
      else if (rows_per_thread == 2) run(std::integral_constant<int, 2>{});
      else if (rows_per_thread == 3) run(std::integral_constant<int, 3>{});
      else run(std::integral_constant<int, 4>{});
    } else if (active) {
      const T* Ab = (const T*)a.A + (int64_t)b * a.sb + a.col0 + col;
      for (int r = r_begin + rl; r < r_end; r += a.row_lanes) {
        const bool is_vis = r >= a.vis_r0 && r < a.vis_r0 + a.n_vis;
        const bool is_cls = r == a.cls_r;
        if (r < a.row0 || !(is_vis || is_cls)) continue;
        double p[kVec];
#pragma unroll
        for (int k = 0; k < kVec; ++k) p[k] = 0.0;
        for (int h = 0; h < a.H; ++h)
          for (int k = 0; k < ncol; ++k) p[k] += widen(Ab[(int64_t)r * a.sq + (int64_t)h * a.sh + k]);
        finish_row(r, is_vis, is_cls, p);
      }
    }
  } else if (active) {
    const T* Ab = (const T*)a.A + (int64_t)b * a.sb + a.col0 + col;
    for (int r = r_begin + rl; r < r_end; r += a.row_lanes) {
      const bool is_vis = r >= a.vis_r0 && r < a.vis_r0 + a.n_vis;
      const bool is_cls = r == a.cls_r;
      if (r < a.row0 || !(is_vis || is_cls)) continue;
      const T* base = Ab + (int64_t)r * a.sq;
      double p[kVec];
#pragma unroll
      for (int k = 0; k < kVec; ++k) p[k] = 0.0;
      if (ncol == kVec) {
        // kHeadBatch independent 16-byte loads are issued before the first add; the adds
        // then run in head order.
        int h0 = 0;
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
      finish_row(r, is_vis, is_cls, p);
    }
  }

  if (rl < a.row_lanes) {
#pragma unroll
    for (int k = 0; k < kVec; ++k) mine[k] = colsum[k];
  }
  __syncthreads();
  if (a.abar) {
    // pieces of 4 query rows: thread -> (key column of the strip, piece), consecutive threads
    // on consecutive pieces of one column
    const int v_begin = r_begin - a.vis_r0;                 // query token of tile row 0 (a multiple of rows_per_wg, or negative)
    const int v_end = min(r_end - a.vis_r0, a.n_vis);       // query tokens of this chunk end here
    const int pieces = a.rows_per_wg / 4;
    const int strip_col0 = strip * width;
    const int n_cols = min(width, a.N - strip_col0);
    for (int q = tid; q < n_cols * pieces; q += (int)blockDim.x) {
      const int c = q / pieces, v0 = (q % pieces) * 4;
      const float* src = tile + c * tile_pitch + v0;
      float* dst = a.abar + ((int64_t)b * a.N + strip_col0 + c) * a.map_pitch + v_begin + v0;
      if (v_begin + v0 >= 0 && v_begin + v0 + 4 <= v_end) {
        const float4 o = make_float4(src[0], src[1], src[2], src[3]);
        __builtin_memcpy(dst, &o, 16);
      } else {
        for (int e = 0; e < 4; ++e)
          if (v_begin + v0 + e >= 0 && v_begin + v0 + e < v_end) dst[e] = src[e];
      }
    }
  }
  if (a.recv_part == nullptr) return;  // uniform for the whole grid
  // Combine the row lanes in a fixed order, then one partial per (image, chunk, column): one
  // thread per column of the strip (the workgroup's last act -- eight columns per thread would
  // keep its slot for eight times as many dependent LDS reads).
  const int strip_col0 = strip * width;
  for (int c = tid; c < width && strip_col0 + c < a.N; c += (int)blockDim.x) {
    double s = 0.0;
    for (int l = 0; l < a.row_lanes; ++l) s += lds[l * width + c];
    a.recv_part[((int64_t)b * a.n_chunks + chunk) * a.N + strip_col0 + c] = s;
  }
}

template <typename T>
__global__ __launch_bounds__(256) void text_reduce_kernel(AttnArgs a) {
  text_reduce_block<T>(a, blockIdx.x, blockIdx.y, blockIdx.z);
}

static void launch_block(const AttnArgs& a, int B, int col_strips, bool bf16, hipStream_t s) {
  AttnArgs g = a;
  g.col_strips = col_strips; g.B = B;
  dim3 grid(xcd_padded_total(a.n_chunks * col_strips * B)), block(std::min(kReduceThreads, (a.row_lanes * a.strip_groups + kWave - 1) / kWave * kWave));
  size_t lds = (size_t)a.row_lanes * a.strip_groups * kVec * sizeof(double);
  if (a.abar) lds += (size_t)a.strip_groups * kVec * (a.rows_per_wg + 1) * sizeof(float);   // the tile that is turned
  if (bf16)
    hipLaunchKernelGGL(attn_reduce_kernel<bf16_t>, grid, block, lds, s, g);
  else
    hipLaunchKernelGGL(attn_reduce_kernel<float>, grid, block, lds, s, g);
}

void launch_attn_reduce(const ficoco_problem& p, const Plan& pl, char* ws, hipStream_t s, bool text_elsewhere) {
  const bool bf16 = p.dtype == FICOCO_BF16;
  const bool want_recv = p.red_src == FICOCO_R_ATTN_RECV;
  const bool want_cls = p.sem_src == FICOCO_G_CLS_ATTN;
  const bool want_abar = p.corr_src == FICOCO_C_ATTN && pl.n_disc > 0;
  if (p.A && (want_recv || want_cls || want_abar)) {
    AttnArgs a{};
    a.A = p.A; a.sb = p.a_stride_b; a.sh = p.a_stride_h; a.sq = p.a_stride_q;
    a.H = p.H;
    a.row0 = pl.a_row0; a.nrows = pl.a_rows;
    a.col0 = p.vis_begin - p.a_k_begin;
    a.N = p.N;
    a.vis_r0 = p.vis_begin - p.a_q_begin;
    a.n_vis = (want_recv || want_abar) ? p.N : 0;
    a.cls_r = want_cls ? p.cls_index - p.a_q_begin : -1;
    a.M = 0;
    a.abar = want_abar ? (float*)(ws + pl.abar) : nullptr;
    a.recv_part = (double*)(ws + pl.recv_part);
    a.cls = (double*)(ws + pl.cls);
    a.ttext = nullptr;
    a.rows_per_wg = pl.rows_per_wg; a.n_chunks = pl.n_chunks;
    a.shift = pl.a_shift; a.map_pitch = pl.map_pitch;
    a.row_lanes = pl.row_lanes; a.strip_groups = pl.strip_groups;
    a.invH = 1.0 / (double)p.H;
    launch_block(a, p.B, pl.col_strips, bf16, s);
  }
  if (p.A_text && p.variant == FICOCO_VARIANT_L && !text_elsewhere) {
    AttnArgs a{};
    fill_text_args(p, pl, ws, a);
    if (bf16) hipLaunchKernelGGL(text_reduce_kernel<bf16_t>, text_grid(p), dim3(256), 0, s, a);
    else hipLaunchKernelGGL(text_reduce_kernel<float>, text_grid(p), dim3(256), 0, s, a);
  }
}

void fill_text_args(const ficoco_problem& p, const Plan& pl, char* ws, AttnArgs& a) {
  a.A = p.A_text; a.sb = p.at_stride_b; a.sh = p.at_stride_h; a.sq = p.at_stride_q;
  a.H = p.H;
  a.row0 = 0; a.nrows = p.M;
  a.col0 = p.vis_begin - p.at_k_begin;
  a.N = p.N;
  a.vis_r0 = 0; a.n_vis = 0; a.cls_r = -1;
  a.M = p.M;
  a.abar = nullptr; a.recv_part = nullptr; a.cls = nullptr;
  a.ttext = (double*)(ws + pl.ttext);
  a.invH = 1.0 / (double)p.H;
}

}  // namespace ficoco

