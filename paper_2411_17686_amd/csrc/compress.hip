// Compress stage: self-preserving compression (Eq. 2) and the removal of the discarded
// tokens (last lines of Algorithm 1/2).
//
// `merge_rows` is a pure pull: one wavefront per OUTPUT row (and per 1024-feature span of it)
// reads its own token plus its sources and writes
//     (X_j + sum_i alpha_ij X_i) / (1 + sum_i alpha_ij)
// accumulated in double precision in ascending i; rows without sources, and every token
// outside the visual span, are copied bit for bit.  No floating-point atomics anywhere.
// Where the sources come from: with few discarded tokens the wavefront scans the per-source
// edge records itself; otherwise `invert_edges` first buckets the edges by target with an
// integer counting sort in LDS (arrival order inside a bucket is arbitrary) and the merging
// wavefront puts its bucket into ascending source order before it adds, so the result never
// depends on scheduling.
#include "common.hpp"

namespace ficoco {

struct InvertArgs {
  int n_keep, n_disc, k_max;
  const int32_t* edge_cnt;
  const int32_t* edge_tgt;
  const double* edge_alpha;
  int32_t* tgt_ptr;    // [B][n_keep+1]
  int32_t* tgt_src;    // [B][n_disc*k_max]  discarded row index (position in S)
  double* tgt_alpha;
};

__global__ __launch_bounds__(kSelectThreads) void invert_edges_kernel(InvertArgs a) {
  extern __shared__ int lds_i[];
  int* cnt = lds_i;                       // [n_keep+1] counts, then exclusive offsets
  int* cursor = lds_i + (a.n_keep + 1);   // [n_keep]
  int* part = cursor + a.n_keep;          // [2][nt] scan scratch
  const int64_t b = blockIdx.x;
  const int tid = threadIdx.x, nt = blockDim.x;
  const int n = a.n_keep;
  for (int j = tid; j <= n; j += nt) cnt[j] = 0;
  __syncthreads();
  for (int r = tid; r < a.n_disc; r += nt) {
    const int c = min(a.edge_cnt[b * a.n_disc + r], a.k_max);
    for (int e = 0; e < c; ++e) {
      const int j = a.edge_tgt[(b * a.n_disc + r) * a.k_max + e];
      if (j >= 0 && j < n) atomicAdd(&cnt[j], 1);
    }
  }
  __syncthreads();
  // exclusive scan of cnt[0..n): thread t owns a contiguous slice
  const int per = (n + nt - 1) / nt;
  const int lo = min(tid * per, n), hi = min(lo + per, n);
  int local = 0;
  for (int j = lo; j < hi; ++j) local += cnt[j];
  int* cur = part;
  int* nxt = part + nt;
  cur[tid] = local;
  __syncthreads();
  for (int off = 1; off < nt; off <<= 1) {
    nxt[tid] = cur[tid] + (tid >= off ? cur[tid - off] : 0);
    __syncthreads();
    int* t = cur; cur = nxt; nxt = t;
  }
  int run = cur[tid] - local;
  const int total = cur[nt - 1];
  for (int j = lo; j < hi; ++j) {
    const int c = cnt[j];
    cnt[j] = run;
    cursor[j] = run;
    run += c;
  }
  if (tid == 0) cnt[n] = total;
  __syncthreads();
  for (int j = tid; j <= n; j += nt) a.tgt_ptr[b * (n + 1) + j] = cnt[j];
  const int64_t ebase = b * (int64_t)a.n_disc * a.k_max;
  for (int r = tid; r < a.n_disc; r += nt) {
    const int c = min(a.edge_cnt[b * a.n_disc + r], a.k_max);
    for (int e = 0; e < c; ++e) {
      const int64_t src = (b * a.n_disc + r) * a.k_max + e;
      const int j = a.edge_tgt[src];
      if (j >= 0 && j < n) {
        const int slot = atomicAdd(&cursor[j], 1);
        a.tgt_src[ebase + slot] = r;
        a.tgt_alpha[ebase + slot] = a.edge_alpha[src];
      }
    }
  }
}

struct MergeArgs {
  const void* X;
  int64_t xsb, xsn;
  void* X_out;
  int D, n_tot, n_out, vis_begin, N, n_keep, n_disc, k_max;
  const int32_t* S;
  const int32_t* T;
  const int32_t* tgt_ptr;
  const int32_t* tgt_src;
  const double* tgt_alpha;
  const int32_t* edge_cnt;
  const int32_t* edge_tgt;
  const double* edge_alpha;
  const EdgeRec* pack;   // null: read the caller's edge lists instead
  const int32_t* pos;
  int32_t* pos_out;
};

template <typename T>
__device__ __forceinline__ void copy8(const T* src, T* dst) {
  Pack8<T> v;
  __builtin_memcpy(&v, src, sizeof(v));
  __builtin_memcpy(dst, &v, sizeof(v));
}

constexpr int kMergeSlice = 2;    // 8-element vectors per lane per pass over the feature axis
constexpr int kMergeSpan = kWave * kVec * kMergeSlice;   // features handled by one wavefront
constexpr int kMatchCap = 64;     // sources of one target kept in LDS

// Accumulate w * X[src] into num (this lane's slices of the feature span starting at d0).
template <typename T>
__device__ __forceinline__ void add_source(const MergeArgs& a, const T* Xb, int i, double w, int d0, int lane,
                                           const bool (&full)[kMergeSlice], double (&num)[kMergeSlice][kVec]) {
  i = min(max(i, 0), a.N - 1);                 // index sets are device data: stay inside the span
  const T* xs = Xb + (int64_t)(a.vis_begin + i) * a.xsn;
#pragma unroll
  for (int u = 0; u < kMergeSlice; ++u) {
    const int d = d0 + (u * kWave + lane) * kVec;
    if (full[u]) {
      double v[kVec];
      load8<T>(xs + d, v);
#pragma unroll
      for (int k = 0; k < kVec; ++k) num[u][k] += w * v[k];
    } else {
      for (int k = 0; k < kVec; ++k)
        if (d + k < a.D) num[u][k] += w * widen(xs[d + k]);
    }
  }
}

// One wavefront per (output row, 1024-feature span).  MATCH = true (few discarded tokens):
// the wavefront scans the packed per-source edge records, 64 discarded rows per load, and
// keeps the rows that name its target in LDS in ascending row order.  MATCH = false: its
// sources are one bucket of the inverted lists, sorted here by rank counting.  Buckets /
// match lists longer than kMatchCap take a slower path that needs no list.
template <typename T, bool MATCH>
__global__ __launch_bounds__(256) void merge_rows_kernel(MergeArgs a) {
  DBG_SPAN(3);
  __shared__ int m_src[4][kMatchCap];
  __shared__ double m_w[4][kMatchCap];
  const int lane = threadIdx.x % kWave, wv = threadIdx.x / kWave;
  const int n_spans = (a.D + kMergeSpan - 1) / kMergeSpan;
  const int wave_id = blockIdx.x * (blockDim.x / kWave) + wv;
  const int r = wave_id / n_spans;
  const int d0 = (wave_id % n_spans) * kMergeSpan;
  const int64_t b = blockIdx.y;
  if (r >= a.n_out) return;
  const T* Xb = (const T*)a.X + b * a.xsb;
  T* out = (T*)a.X_out + (b * a.n_out + r) * (int64_t)a.D;
  int t, j = -1, e0 = 0, e1 = 0;
  if (r < a.vis_begin) {
    t = r;
  } else if (r < a.vis_begin + a.n_keep) {
    j = r - a.vis_begin;
    int tok = a.T[b * a.n_keep + j];
    tok = min(max(tok, 0), a.N - 1);   // index sets are device data: stay inside the span
    t = a.vis_begin + tok;
    if (!MATCH && a.n_disc > 0) {
      e0 = a.tgt_ptr[b * (a.n_keep + 1) + j];
      e1 = a.tgt_ptr[b * (a.n_keep + 1) + j + 1];
    }
    if (lane == 0 && d0 == 0 && a.pos_out) a.pos_out[b * a.n_keep + j] = a.pos ? a.pos[b * a.N + tok] : tok;
  } else {
    t = r + a.n_disc;
  }
  const T* x = Xb + (int64_t)t * a.xsn;
  const bool merged_row = j >= 0 && a.n_disc > 0;
  const int64_t ebase = b * (int64_t)a.n_disc * a.k_max;

  // ---- sources of this target -------------------------------------------------------------
  int n_src = 0;
  if (merged_row && MATCH) {
    for (int base = 0; base < a.n_disc; base += kWave) {
      const int row = base + lane;
      const bool in = row < a.n_disc;
      const int64_t rr = b * a.n_disc + (in ? row : 0);
      const int cnt = in ? min(a.edge_cnt[rr], a.k_max) : 0;
      int t0, src;
      double w;
      if (a.pack) {
        const EdgeRec e = a.pack[rr * a.k_max];
        t0 = e.tgt; src = e.src; w = e.alpha;
      } else {
        t0 = a.edge_tgt[rr * a.k_max];
        src = a.S[rr];
        w = 0.0;
      }
      int he = (cnt > 0 && t0 == j) ? 0 : -1;
      for (int e = 1; e < cnt; ++e)
        if (a.edge_tgt[rr * a.k_max + e] == j) he = e;
      const bool hit = he >= 0;
      if (hit && (he > 0 || !a.pack)) w = a.edge_alpha[rr * a.k_max + he];
      const unsigned long long m = __ballot(hit);
      if (hit) {
        const int slot = n_src + __popcll(m & ((1ULL << lane) - 1ULL));
        if (slot < kMatchCap) { m_src[wv][slot] = src; m_w[wv][slot] = w; }
      }
      n_src += __popcll(m);
    }
  } else if (merged_row) {
    n_src = e1 - e0;
    if (n_src > 0 && n_src <= kMatchCap) {
      // bucket -> ascending source row: rank of an entry = number of entries with a smaller row
      const bool in = lane < n_src;
      const int row = in ? a.tgt_src[ebase + e0 + lane] : 0x7fffffff;
      const double w = in ? a.tgt_alpha[ebase + e0 + lane] : 0.0;
      const int src = in ? a.S[b * a.n_disc + min(max(row, 0), a.n_disc - 1)] : 0;
      int rank = 0;
      for (int l = 0; l < n_src; ++l) rank += __shfl(row, l, kWave) < row ? 1 : 0;
      if (in) { m_src[wv][rank] = src; m_w[wv][rank] = w; }
    }
  }
  bool full[kMergeSlice];
#pragma unroll
  for (int u = 0; u < kMergeSlice; ++u) full[u] = d0 + (u * kWave + lane) * kVec + kVec <= a.D;
  if (!merged_row || n_src == 0) {  // nothing merged into this row: exact copy
#pragma unroll
    for (int u = 0; u < kMergeSlice; ++u) {
      const int d = d0 + (u * kWave + lane) * kVec;
      if (full[u]) copy8<T>(x + d, out + d);
      else
        for (int k = 0; k < kVec; ++k)
          if (d + k < a.D) out[d + k] = x[d + k];
    }
    return;
  }
  // this lane's slices of the row
  double num[kMergeSlice][kVec];
#pragma unroll
  for (int u = 0; u < kMergeSlice; ++u) {
    const int d = d0 + (u * kWave + lane) * kVec;
    if (full[u]) load8<T>(x + d, num[u]);
    else
      for (int k = 0; k < kVec; ++k) num[u][k] = d + k < a.D ? widen(x[d + k]) : 0.0;
  }

  double den = 1.0;
  if (n_src <= kMatchCap) {
    for (int e = 0; e < n_src; ++e) den += m_w[wv][e];
    for (int e = 0; e < n_src; ++e) add_source<T>(a, Xb, m_src[wv][e], m_w[wv][e], d0, lane, full, num);
  } else if (MATCH) {
    // more sources than the list holds: add while scanning
    for (int base = 0; base < a.n_disc; base += kWave) {
      const int row = base + lane;
      const bool in = row < a.n_disc;
      const int64_t rr = b * a.n_disc + (in ? row : 0);
      const int cnt = in ? min(a.edge_cnt[rr], a.k_max) : 0;
      int he = -1;
      for (int e = 0; e < cnt; ++e)
        if (a.edge_tgt[rr * a.k_max + e] == j) he = e;
      const double w = he >= 0 ? a.edge_alpha[rr * a.k_max + he] : 0.0;
      const int src = a.S[rr];
      unsigned long long m = __ballot(he >= 0);
      while (m) {
        const int l = __ffsll(m) - 1;
        m &= m - 1;
        const double wl = __shfl(w, l, kWave);
        den += wl;
        add_source<T>(a, Xb, __shfl(src, l, kWave), wl, d0, lane, full, num);
      }
    }
  } else {
    // long bucket: take its entries in ascending source row by repeated minimum search
    int last = -1;
    for (int k = 0; k < n_src; ++k) {
      int best = 0x7fffffff, best_e = -1;
      for (int e = e0 + lane; e < e1; e += kWave) {
        const int row = a.tgt_src[ebase + e];
        if (row > last && row < best) { best = row; best_e = e; }
      }
      int mn = best;
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) mn = min(mn, __shfl_xor(mn, off, kWave));
      const unsigned long long who = __ballot(best == mn && best_e >= 0);
      const int l = __ffsll(who) - 1;
      const int e = __shfl(best_e, l, kWave);
      const double w = a.tgt_alpha[ebase + e];
      den += w;
      add_source<T>(a, Xb, a.S[b * a.n_disc + min(max(mn, 0), a.n_disc - 1)], w, d0, lane, full, num);
      last = mn;
    }
  }
#pragma unroll
  for (int u = 0; u < kMergeSlice; ++u) {
    const int d = d0 + (u * kWave + lane) * kVec;
    if (full[u]) {
      Pack8<T> o;
#pragma unroll
      for (int k = 0; k < kVec; ++k) store_token(&o.v[k], num[u][k] / den);
      __builtin_memcpy(out + d, &o, sizeof(o));
    } else {
      for (int k = 0; k < kVec; ++k)
        if (d + k < a.D) store_token(out + d + k, num[u][k] / den);
    }
  }
}

constexpr int kMatchMaxRows = 1024;   // above this many discarded tokens the edge lists are inverted first

void launch_compress(const ficoco_problem& p, const Plan& pl, char* ws, const int32_t* discard_idx,
                     const int32_t* keep_idx, const int32_t* edge_cnt, const int32_t* edge_tgt,
                     const double* edge_alpha, void* X_out, int32_t* pos_out, bool use_pack,
                     hipStream_t s) {
  const bool match = pl.n_disc <= kMatchMaxRows;
  if (pl.n_disc > 0 && !match) {
    InvertArgs a{};
    a.n_keep = p.n_keep; a.n_disc = pl.n_disc; a.k_max = p.k_max;
    a.edge_cnt = edge_cnt; a.edge_tgt = edge_tgt; a.edge_alpha = edge_alpha;
    a.tgt_ptr = (int32_t*)(ws + pl.tgt_ptr);
    a.tgt_src = (int32_t*)(ws + pl.tgt_src);
    a.tgt_alpha = (double*)(ws + pl.tgt_alpha);
    const size_t lds = ((size_t)2 * p.n_keep + 1 + 2 * kSelectThreads) * sizeof(int);
    if (lds > 32768)
      (void)hipFuncSetAttribute((const void*)invert_edges_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipLaunchKernelGGL(invert_edges_kernel, dim3(p.B), dim3(kSelectThreads), lds, s, a);
  }
  MergeArgs m{};
  m.X = p.X; m.xsb = p.x_stride_b; m.xsn = p.x_stride_n; m.X_out = X_out;
  m.D = p.D; m.n_tot = p.n_tot; m.n_out = pl.n_out; m.vis_begin = p.vis_begin; m.N = p.N;
  m.n_keep = p.n_keep; m.n_disc = pl.n_disc; m.k_max = p.k_max;
  m.S = discard_idx; m.T = keep_idx;
  m.tgt_ptr = (const int32_t*)(ws + pl.tgt_ptr);
  m.tgt_src = (const int32_t*)(ws + pl.tgt_src);
  m.tgt_alpha = (const double*)(ws + pl.tgt_alpha);
  m.edge_cnt = edge_cnt; m.edge_tgt = edge_tgt; m.edge_alpha = edge_alpha;
  m.pack = use_pack ? (const EdgeRec*)(ws + pl.edge_pack) : nullptr;
  m.pos = p.pos; m.pos_out = pos_out;
  const int n_spans = (p.D + kMergeSpan - 1) / kMergeSpan;
  dim3 grid((pl.n_out * n_spans + 3) / 4, p.B), block(256);
  const bool bf16 = p.dtype == FICOCO_BF16;
  if (match) {
    if (bf16) hipLaunchKernelGGL((merge_rows_kernel<bf16_t, true>), grid, block, 0, s, m);
    else hipLaunchKernelGGL((merge_rows_kernel<float, true>), grid, block, 0, s, m);
  } else {
    if (bf16) hipLaunchKernelGGL((merge_rows_kernel<bf16_t, false>), grid, block, 0, s, m);
    else hipLaunchKernelGGL((merge_rows_kernel<float, false>), grid, block, 0, s, m);
  }
}

}  // namespace ficoco

FICOCO_DBG_READER(merge)
