// Compress stage: self-preserving compression (Eq. 2) and the removal of the discarded
// tokens (last lines of Algorithm 1/2).
//
// `merge_rows` is a pure pull: one wavefront per OUTPUT row (and per feature span of it) reads
// its own token plus its sources and writes
//     (X_j + sum_i alpha_ij X_i) / (1 + sum_i alpha_ij)
// accumulated in double precision in ascending i; rows without sources, and every token
// outside the visual span, are copied bit for bit.  No floating-point atomics anywhere.
// Where the sources come from: with few discarded tokens the workgroup stages the image's
// per-source edge lists in LDS and every wavefront scans them for its target; otherwise
// `invert_edges` first buckets the edges by target with an integer counting sort in LDS
// (order inside a bucket is arbitrary) and the merging wavefront puts its bucket into
// ascending source order before it adds, so the result never depends on scheduling.
#include "common.hpp"

// Products and sums of Eq. 2 are rounded separately everywhere in this file (no fused multiply-add):
// the weighted sums are then the very doubles the plain statement of the equation produces.
#pragma clang fp contract(off)

namespace ficoco {

struct InvertArgs {
  int n_keep, n_disc, k_max;
  const int32_t* edge_cnt;
  const int32_t* edge_tgt;
  const double* edge_alpha;
  int32_t* tgt_ptr;    // [B][n_keep+1]
  int32_t* tgt_src;    // [B][n_disc*k_max]  discarded row index (position in S)
  double* tgt_alpha;
  int32_t* hub_list;   // [B][n_keep]  preserved tokens with more than kHubMin sources (any order)
  int32_t* hub_cnt;    // [B]
  const int32_t* share_cnt;   // [B][gridDim.x][n_keep] edges per (share of rows, target) counted by the correlate stage, or null
  int share_rows;      // discarded rows per workgroup
};

constexpr int kHubMin = 32;        // buckets longer than this are merged by a whole workgroup

// Buckets the edges of one image by target.  gridDim.x workgroups share an image, each owning
// share_rows consecutive discarded rows.  Every workgroup needs, per target, the number of edges
// of the whole image and the number from rows before its own share: the prefix sum of the former
// gives the bucket offsets, and offset + "before" is where this workgroup's own rows start inside
// each bucket.  Then it scatters its rows.  The two numbers come from the counters the correlate
// stage kept per (share, target) while it wrote the lists (share_cnt, a fused step), or else from
// a pass of every workgroup over ALL lists of the image into an LDS histogram (it needs no
// exchange between workgroups and nothing cleared beforehand).  Bucket regions per workgroup
// are fixed either way; only the order inside a region depends on scheduling (the merge orders
// buckets itself).
template <int CH>   // consecutive list slots one thread loads at a time: 4 (rows of 4k slots, 16-byte aligned lists) or 1
__global__ __launch_bounds__(kSelectThreads) void invert_edges_kernel(InvertArgs a) {
  extern __shared__ int lds_i[];
  int* cnt = lds_i;                       // [n_keep+1] counts, then exclusive offsets
  int* cursor = lds_i + (a.n_keep + 1);   // [n_keep] edges from earlier shares, then write cursor
  int* part = cursor + a.n_keep;          // [2][nt] scan scratch
  const int64_t b = blockIdx.y;
  const int tid = threadIdx.x, nt = blockDim.x;
  const int n = a.n_keep;
  const int r_lo = min((int)blockIdx.x * a.share_rows, a.n_disc), r_hi = min(r_lo + a.share_rows, a.n_disc);
  const int64_t rbase = b * a.n_disc;
  const int32_t* tgt = a.edge_tgt + rbase * a.k_max;      // the image's lists as one flat array of slots
  const double* alp = a.edge_alpha + rbase * a.k_max;
  auto load_slots = [&](int f, int (&v)[CH]) {            // slots f .. f+CH-1 (inside one row)
    if constexpr (CH == 4) {
      const int4 q = *reinterpret_cast<const int4*>(tgt + f);
      v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
    } else {
      v[0] = tgt[f];
    }
  };
  if (a.share_cnt) {             // counted while the lists were written: add the shares up
    const int32_t* sc = a.share_cnt + b * (int64_t)gridDim.x * n;
    constexpr int kShareBatch = 8;      // counters one thread has in flight together
    const int shares = gridDim.x, mine = blockIdx.x;
    for (int j = tid; j < n; j += nt) {
      int all = 0, before = 0;
      for (int s0 = 0; s0 < shares; s0 += kShareBatch) {
        int c[kShareBatch];
#pragma unroll
        for (int u = 0; u < kShareBatch; ++u) c[u] = sc[(int64_t)min(s0 + u, shares - 1) * n + j];   // clamped: always a valid address
        issue_fence();
#pragma unroll
        for (int u = 0; u < kShareBatch; ++u) {
          if (s0 + u < shares) all += c[u];
          if (s0 + u < mine) before += c[u];
        }
      }
      cnt[j] = all;
      cursor[j] = before;
    }
    if (tid == 0) cnt[n] = 0;
  } else {
    // Count pass over every slot of the image.  Consecutive threads take consecutive slots, so a
    // wavefront's load covers whole cache lines (a thread per row would touch every line of the
    // lists once per slot position); kInvertBatch loads per thread are in flight together.
    for (int j = tid; j <= n; j += nt) cnt[j] = 0;
    for (int j = tid; j < n; j += nt) cursor[j] = 0;
    __syncthreads();
    constexpr int kInvertBatch = CH == 4 ? 8 : 16;     // loads of list slots one thread has in flight together
    const int n_chunks = a.n_disc * a.k_max / CH;
    for (int c0 = tid; c0 < n_chunks; c0 += nt * kInvertBatch) {
      int v[kInvertBatch][CH], have[kInvertBatch], row[kInvertBatch];
#pragma unroll
      for (int u = 0; u < kInvertBatch; ++u) {
        const int f = min(c0 + u * nt, n_chunks - 1) * CH;   // clamped: always a valid address
        row[u] = f / a.k_max;
        have[u] = min(a.edge_cnt[rbase + row[u]], a.k_max) - (f - row[u] * a.k_max);   // list entries from slot f on
        load_slots(f, v[u]);
      }
      issue_fence();
#pragma unroll
      for (int u = 0; u < kInvertBatch; ++u) {
        if (c0 + u * nt >= n_chunks) break;
        const bool before = row[u] < r_lo;
#pragma unroll
        for (int q = 0; q < CH; ++q) {
          const int j = v[u][q];
          if (q < have[u] && j >= 0 && j < n) {
            atomicAdd(&cnt[j], 1);
            if (before) atomicAdd(&cursor[j], 1);
          }
        }
      }
    }
  }
  __syncthreads();
  // exclusive scan of cnt[0..n): thread t owns a contiguous slice
  const int per = (n + nt - 1) / nt;
  const int lo = min(tid * per, n), hi = min(lo + per, n);
  int local = 0;
  for (int j = lo; j < hi; ++j) local += cnt[j];
  int total;
  int run = block_scan_inclusive(local, part, &total) - local;
  for (int j = lo; j < hi; ++j) {
    const int c = cnt[j];
    cnt[j] = run;
    cursor[j] += run;
    run += c;
  }
  if (tid == 0) cnt[n] = total;
  __syncthreads();
  if (blockIdx.x == 0) {       // uniform over the workgroup
    for (int j = tid; j <= n; j += nt) a.tgt_ptr[b * (n + 1) + j] = cnt[j];
    // targets with long buckets, for the workgroup-per-target pass of the merge
    int* hub_n = part;         // the scan scratch is free now
    if (tid == 0) *hub_n = 0;
    __syncthreads();
    for (int j = tid; j < n; j += nt)
      if (cnt[j + 1] - cnt[j] > kHubMin) a.hub_list[b * n + atomicAdd(hub_n, 1)] = j;
    __syncthreads();
    if (tid == 0) a.hub_cnt[b] = *hub_n;
  }
  const int64_t ebase = b * (int64_t)a.n_disc * a.k_max;
  const int cap = a.n_disc * a.k_max;
  // Scatter of the workgroup's own rows, slot by slot in the same flat order.
  const int f_lo = r_lo * a.k_max / CH, f_hi = r_hi * a.k_max / CH;
  for (int ci = f_lo + tid; ci < f_hi; ci += nt) {
    const int f = ci * CH;
    const int r = f / a.k_max;
    const int have = min(a.edge_cnt[rbase + r], a.k_max) - (f - r * a.k_max);
    int v[CH];
    double al[CH];
    load_slots(f, v);
    if constexpr (CH == 4) {
      const double2 a0 = *reinterpret_cast<const double2*>(alp + f);
      const double2 a1 = *reinterpret_cast<const double2*>(alp + f + 2);
      al[0] = a0.x; al[1] = a0.y; al[2] = a1.x; al[3] = a1.y;
    } else {
      al[0] = alp[f];
    }
    issue_fence();
#pragma unroll
    for (int q = 0; q < CH; ++q) {
      const int j = v[q];
      if (q < have && j >= 0 && j < n) {
        const int slot = atomicAdd(&cursor[j], 1);
        if (slot < cap) {                     // always true for consistent lists; they are device data
          a.tgt_src[ebase + slot] = r;
          a.tgt_alpha[ebase + slot] = al[q];
        }
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
  const int32_t* pos;
  int32_t* pos_out;
  const int32_t* hub_list;   // bucket mode: targets with more than kHubMin sources ...
  const int32_t* hub_cnt;    // ... and their number; null: no such split
  const PairRec* pair_tab;   // [B][n_disc] the staged fields of every discarded row as one record (fused step), or null
  int average;      // ablation "average compression": every weight counts as one
  int extra_row;    // output row of the additional token of the convergent form (mean of the discarded tokens), or -1
};

static __device__ int32_t g_no_token = 0;   // what the row's token index is read from when nothing is preserved

template <typename T>
__device__ __forceinline__ void copy8(const T* src, T* dst) {
  Pack8<T> v;
  __builtin_memcpy(&v, src, sizeof(v));
  __builtin_memcpy(dst, &v, sizeof(v));
}

constexpr int kMergeWaves = 8;    // wavefronts (= output row spans) per workgroup
// (kMatchMaxRows, common.hpp: above that many discarded tokens the edge lists are inverted first)
static_assert(kMatchMaxRows % (kMergeWaves * kWave) == 0, "a workgroup stages the edge table in whole rounds");
constexpr int kMatchCap = 64;     // scanning mode: sources of one target kept in LDS
constexpr int kBucketCap = 256;   // inverted lists: bucket entries put in order in LDS
constexpr int kBucketPer = kBucketCap / kWave;

// Accumulate w * X[src] into num (this lane's slices of the feature span starting at d0).
template <typename T, int SLICE>
__device__ __forceinline__ void add_source(const MergeArgs& a, const T* Xb, int i, double w, int d0, int lane,
                                           const bool (&full)[SLICE], double (&num)[SLICE][kVec]) {
  i = min(max(i, 0), a.N - 1);                 // index sets are device data: stay inside the span
  const T* xs = Xb + (int64_t)(a.vis_begin + i) * a.xsn;
#pragma unroll
  for (int u = 0; u < SLICE; ++u) {
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

// The same for a whole list held in LDS, in list order, with the row loads of kBatch sources
// issued before the first of them is added: a target with n sources then waits for
// ceil(n / kBatch) memory round trips instead of n.  The batch is straight-line code: a load
// under a per-lane condition makes the compiler wait for the previous load first (the
// registers it fills may still be awaited on the path that skipped their use), which would
// put the round trips back in series.  So lanes without a whole vector inside the row load the
// row's first vector instead, and what they loaded is cleared before it is added (adding
// w * 0 leaves the sum as it is).
template <typename T, int SLICE, int REGS>
__device__ __forceinline__ void add_sources(const MergeArgs& a, const T* Xb, const int* src, const double* w,
                                            int n_src, int d0, int lane, const bool (&full)[SLICE],
                                            double (&num)[SLICE][kVec]) {
  constexpr int kWant = REGS / (SLICE * (int)(sizeof(Raw8<T>) / 4));   // REGS registers of raw data in flight
  constexpr int kBatch = kWant < 1 ? 1 : kWant;
  if (a.D >= kVec) {                 // uniform; narrower rows have no whole vector at all
    int off[SLICE];
#pragma unroll
    for (int u = 0; u < SLICE; ++u) off[u] = full[u] ? d0 + (u * kWave + lane) * kVec : 0;
#pragma unroll 1
    for (int e = 0; e < n_src; e += kBatch) {
      Raw8<T> raw[kBatch][SLICE];
#pragma unroll
      for (int q = 0; q < kBatch; ++q) {
        const int i = min(max(src[min(e + q, n_src - 1)], 0), a.N - 1);   // device data: stay inside the span
        const T* xs = Xb + (int64_t)(a.vis_begin + i) * a.xsn;
#pragma unroll
        for (int u = 0; u < SLICE; ++u) load_raw(xs + off[u], raw[q][u]);
      }
      issue_fence();
      // past the end of the list the last row was loaded again and is cleared like the lanes
      // above: a branch around its use would let the compiler move the load down to it
#pragma unroll
      for (int q = 0; q < kBatch; ++q) {
        const double wq = w[min(e + q, n_src - 1)];
#pragma unroll
        for (int u = 0; u < SLICE; ++u) {
          keep_raw_if(raw[q][u], full[u] && e + q < n_src);
          fma_raw(raw[q][u], wq, num[u]);
        }
      }
    }
  }
  // The one lane whose vector straddles the end of a row (D not a multiple of 8) adds its
  // elements source by source: batching these guarded element loads as well would cost every
  // launch a third of its registers for a case that row widths in use never have.
  bool ragged = false;
#pragma unroll
  for (int u = 0; u < SLICE; ++u) ragged |= !full[u] && d0 + (u * kWave + lane) * kVec < a.D;
  if (ragged) {
#pragma unroll 1
    for (int e = 0; e < n_src; ++e) {
      const int i = min(max(src[e], 0), a.N - 1);
      const T* xs = Xb + (int64_t)(a.vis_begin + i) * a.xsn;
      const double wq = w[e];
#pragma unroll
      for (int u = 0; u < SLICE; ++u) {
        const int d = d0 + (u * kWave + lane) * kVec;
        if (!full[u]) {
#pragma unroll
          for (int k = 0; k < kVec; ++k)
            if (d + k < a.D) num[u][k] += wq * widen(xs[d + k]);
        }
      }
    }
  }
}

// Per-source edge table of one image in LDS (scanning mode): count, token, and the first two
// (target, weight) pairs of every discarded row; further pairs stay in global memory.
struct EdgeTable {
  double* a0;
  double* a1;
  int* cnt;
  int* src;
  int* t0;
  int* t1;
};

// Does discarded row `row` of the image name preserved token j as a target, and with which weight?
// The first two pairs of a row are in LDS (FULL = false looks at those only and reports in
// `more` whether the row has further pairs); the rest is read from global memory.
template <bool FULL>
__device__ __forceinline__ bool row_names_target(const MergeArgs& a, const EdgeTable& tb, int64_t ebase, int row,
                                                 bool in, int j, double& w, bool& more) {
  const int cnt = in ? tb.cnt[row] : 0;
  bool hit = false;
  if (cnt > 0 && tb.t0[row] == j) { hit = true; w = tb.a0[row]; }
  if (cnt > 1 && tb.t1[row] == j) { hit = true; w = tb.a1[row]; }
  more = cnt > 2;
  if (FULL) {
    for (int e = 2; e < cnt; ++e)
      if (a.edge_tgt[ebase + (int64_t)row * a.k_max + e] == j) {
        hit = true;
        w = a.average ? 1.0 : a.edge_alpha[ebase + (int64_t)row * a.k_max + e];
      }
  }
  return hit;
}

__device__ __forceinline__ EdgeTable edge_table(char* base, int n_disc) {
  EdgeTable tb;
  tb.a0 = (double*)base;
  tb.a1 = tb.a0 + n_disc;
  tb.cnt = (int*)(tb.a1 + n_disc);
  tb.src = tb.cnt + n_disc;
  tb.t0 = tb.src + n_disc;
  tb.t1 = tb.t0 + n_disc;
  return tb;
}

// LDS carve-up of merge_rows_kernel, shared by the kernel and its launcher.
template <bool MATCH, int SLICE, int WPU>
struct MergeLds {
  static constexpr int kCap = MATCH ? kMatchCap : kBucketCap;
  static constexpr int kUnits = kMergeWaves / WPU;
  static constexpr size_t kLists = (size_t)kMergeWaves * kCap * 12;
  static constexpr size_t kPartDoubles = WPU > 1 ? (size_t)kUnits * (WPU - 1) * SLICE * kVec * kWave : 0;
  static constexpr size_t kDen = WPU > 1 ? (size_t)kMergeWaves * 16 : 0;     // one (den, count) pair per wavefront
  static size_t bytes(int n_disc) { return kLists + kPartDoubles * 8 + kDen + (MATCH ? (size_t)n_disc * 32 : 0); }
};

// One UNIT = (output row, feature span of 512 * SLICE).  Rows without sources, and every token
// outside the visual span, are copied.  A unit is served by WPU wavefronts: wavefront w takes
// the sources whose discarded row lies in the w-th part of [0, n_disc), adds them in ascending
// row order in double precision, and the parts are then added in order by wavefront 0
// (WPU = 1: one plain ascending sum).  Where a wavefront's sources come from:
//   MATCH = true  (few discarded tokens): the workgroup stages the image's edge table in LDS
//     once; each wavefront scans its part of it, 64 discarded rows per pass, and keeps the rows
//     that name its target in a list in ascending row order;
//   MATCH = false: the sources are one bucket of the inverted lists (arbitrary order); the
//     wavefront takes the entries of its part and orders them by rank counting.
// The list is then added with several row loads in flight.  Buckets longer than the LDS holds
// take a slower path that needs no list; scanning-mode targets with more than kHubMin sources
// are left to merge_hub_targets.
// Returns the number of sources of a target that is left to the whole workgroup (scanning
// mode, more than kHubMin sources), else 0.
template <typename T, bool MATCH, int SLICE, int WPU>
__device__ __forceinline__ int merge_unit(const MergeArgs& a, char* lds_m, int blk) {
  using Lds = MergeLds<MATCH, SLICE, WPU>;
  constexpr int kCap = Lds::kCap;
  constexpr int kSpan = kWave * kVec * SLICE;
  constexpr int kRegs = (MATCH && WPU == 1) ? 16 : 32;   // registers of row data in flight per lane while a list is added
  const int lane = threadIdx.x % kWave, wv = threadIdx.x / kWave;
  const int unit_l = wv / WPU, sub = wv % WPU;
  double* l_w = (double*)lds_m + wv * kCap;
  int* l_src = (int*)((double*)lds_m + kMergeWaves * kCap) + wv * kCap;
  double* part = (double*)(lds_m + Lds::kLists);                 // [kUnits][WPU-1][SLICE*kVec][64]
  double* wden = part + Lds::kPartDoubles;                       // [kMergeWaves][2]: partial denominator, source count
  const EdgeTable tb = edge_table(lds_m + Lds::kLists + Lds::kPartDoubles * 8 + Lds::kDen, a.n_disc);
  const int n_spans = (a.D + kSpan - 1) / kSpan;
  const int unit = blk * Lds::kUnits + unit_l;      // blk: index of this workgroup among those of its pass
  const int64_t b = blockIdx.y;
  int r = unit / n_spans;
  const int d0 = (unit % n_spans) * kSpan;
  if (WPU > 1) {
    // workgroup-per-target pass: unit -> entry of the list of long buckets (one unit per
    // workgroup, so the whole workgroup leaves together past the end of the list)
    static_assert(WPU == 1 || Lds::kUnits == 1, "the long-bucket pass maps one workgroup to one target");
    const int h = unit / n_spans;
    const int n_hub = min(max(a.hub_cnt[b], 0), a.n_keep);
    if (h >= n_hub) return 0;
    r = a.vis_begin + min(max(a.hub_list[b * a.n_keep + h], 0), a.n_keep - 1);
  }
  const bool valid = r < a.n_out && r != a.extra_row;   // the additional token is written by extra_token_kernel

  // Order of the loads below: the row's token index first (its own row depends on it), then
  // this thread's share of the edge table, then -- once the index is there -- the row itself;
  // the table is put into LDS last.  Each of them is a memory round trip of its own if taken
  // one after the other.
  const T* Xb = (const T*)a.X + b * a.xsb;
  T* out = (T*)a.X_out + (b * a.n_out + (valid ? r : 0)) * (int64_t)a.D;
  const bool kept_row = valid && r >= a.vis_begin && r < a.vis_begin + a.n_keep;
  // (an unconditional load from an address that is always valid: under a condition the compiler
  // moves the first use of the value next to the load and waits for it there)
  const int32_t* tok_at = a.n_keep > 0 ? a.T + b * a.n_keep + min(max(r - a.vis_begin, 0), a.n_keep - 1) : &g_no_token;
  int tok = *tok_at;
  constexpr int kStage = MATCH ? kMatchMaxRows / (kMergeWaves * kWave) : 1;   // edge-table rows per thread
  int st_cnt[kStage], st_src[kStage], st_t0[kStage], st_t1[kStage];
  double st_a0[kStage], st_a1[kStage];
  if (MATCH && a.n_disc > 0 && a.pair_tab) {       // uniform: one record per row, two whole-line loads
#pragma unroll
    for (int q = 0; q < kStage; ++q) {
      const int row = min((int)threadIdx.x + q * kMergeWaves * kWave, a.n_disc - 1);   // clamped: a valid row
      const PairRec* rec = a.pair_tab + (b * a.n_disc + row);
      const int4 head = *reinterpret_cast<const int4*>(rec);
      const double2 wts = *reinterpret_cast<const double2*>(&rec->a0);
      st_cnt[q] = head.x; st_src[q] = head.y; st_t0[q] = head.z; st_t1[q] = head.w;
      st_a0[q] = a.average ? 1.0 : wts.x;
      st_a1[q] = a.average ? 1.0 : wts.y;
    }
  } else if (MATCH && a.n_disc > 0) {
    const int e1 = min(1, a.k_max - 1);
#pragma unroll
    for (int q = 0; q < kStage; ++q) {
      const int row = min((int)threadIdx.x + q * kMergeWaves * kWave, a.n_disc - 1);   // clamped: a valid row
      const int64_t rr = b * a.n_disc + row;
      st_cnt[q] = a.edge_cnt[rr];
      st_src[q] = a.S[rr];
      st_t0[q] = a.edge_tgt[rr * a.k_max];
      st_t1[q] = a.edge_tgt[rr * a.k_max + e1];
      st_a0[q] = a.average ? 1.0 : a.edge_alpha[rr * a.k_max];
      st_a1[q] = a.average ? 1.0 : a.edge_alpha[rr * a.k_max + e1];
    }
  }
  issue_fence();

  int t = 0, j = -1, e0 = 0, e1 = 0;
  if (valid) {
    if (r < a.vis_begin) {
      t = r;
    } else if (kept_row) {
      j = r - a.vis_begin;
      tok = min(max(tok, 0), a.N - 1);   // index sets are device data: stay inside the span
      t = a.vis_begin + tok;
      if (!MATCH && a.n_disc > 0) {
        // bucket bounds are device data: keep them inside the image's edge storage
        e0 = min(max(a.tgt_ptr[b * (a.n_keep + 1) + j], 0), a.n_disc * a.k_max);
        e1 = min(max(a.tgt_ptr[b * (a.n_keep + 1) + j + 1], e0), a.n_disc * a.k_max);
      }
    } else {
      t = r + a.n_disc - (a.extra_row >= 0 ? 1 : 0);
    }
  }
  const T* x = Xb + (int64_t)t * a.xsn;
  const bool merged_row = j >= 0 && a.n_disc > 0;
  const int64_t ebase = b * (int64_t)a.n_disc * a.k_max;
  bool full[SLICE];
#pragma unroll
  for (int u = 0; u < SLICE; ++u) full[u] = d0 + (u * kWave + lane) * kVec + kVec <= a.D;
  // this row's own slices, in flight while its sources are looked up
  Raw8<T> xr[SLICE];
  if (valid && sub == 0) {
#pragma unroll
    for (int u = 0; u < SLICE; ++u)
      if (full[u]) load_raw(x + d0 + (u * kWave + lane) * kVec, xr[u]);
  }
  if (MATCH && a.n_disc > 0) {
#pragma unroll
    for (int q = 0; q < kStage; ++q) {
      // threads past the last row hold a second copy of it and store that: no branch around the
      // use of what was loaded, so nothing stays "possibly in flight" for the code below
      const int row = min((int)threadIdx.x + q * kMergeWaves * kWave, a.n_disc - 1);
      tb.cnt[row] = min(st_cnt[q], a.k_max);
      tb.src[row] = st_src[q];
      tb.t0[row] = st_t0[q];
      tb.t1[row] = st_t1[q];
      tb.a0[row] = st_a0[q];
      tb.a1[row] = st_a1[q];
    }
  }
  if (MATCH) __syncthreads();   // the edge table is complete (every wavefront arrives here)
  if (WPU == 1 && !valid) return 0;

  // this wavefront's part of the discarded rows
  const int part_rows = WPU == 1 ? a.n_disc : ((a.n_disc + WPU - 1) / WPU + kWave - 1) / kWave * kWave;
  const int row_lo = min(sub * part_rows, a.n_disc), row_hi = min(row_lo + part_rows, a.n_disc);

  // ---- sources of this target within [row_lo, row_hi) ------------------------------------------
  int n_src = 0;
  bool long_bucket = false;
  if (valid && merged_row && MATCH) {
    // The common search touches LDS only, so it runs while the row's own load is in flight (a
    // global load inside this loop would make every pass wait for all loads issued before it).
    // Rows with more than two targets are rare: if the image has any, the search is done again
    // with the further pairs read from global memory.
    bool any_more = false;
    for (int base = row_lo; base < row_hi; base += kWave) {
      const int row = base + lane;
      double w = 0.0;
      bool more;
      const bool hit = row_names_target<false>(a, tb, ebase, row, row < row_hi, j, w, more);
      any_more |= more;
      const unsigned long long m = __ballot(hit);
      if (hit) {
        const int slot = n_src + __popcll(m & ((1ULL << lane) - 1ULL));
        if (slot < kCap) { l_src[slot] = tb.src[row]; l_w[slot] = w; }
      }
      n_src += __popcll(m);
    }
    if (__any(any_more)) {
      n_src = 0;
      for (int base = row_lo; base < row_hi; base += kWave) {
        const int row = base + lane;
        double w = 0.0;
        bool more;
        const bool hit = row_names_target<true>(a, tb, ebase, row, row < row_hi, j, w, more);
        const unsigned long long m = __ballot(hit);
        if (hit) {
          const int slot = n_src + __popcll(m & ((1ULL << lane) - 1ULL));
          if (slot < kCap) { l_src[slot] = tb.src[row]; l_w[slot] = w; }
        }
        n_src += __popcll(m);
      }
    }
    if (WPU == 1 && n_src > kHubMin) return n_src;   // added by the whole workgroup, see merge_hub_targets
  } else if (valid && merged_row) {
    const int n_all = e1 - e0;
    if (WPU == 1 && a.hub_cnt != nullptr && n_all > kHubMin) return 0;   // written by the workgroup-per-target pass
    long_bucket = n_all > kCap;
    if (n_all > 0 && !long_bucket) {
      // entries of the bucket that fall into this part -> ascending discarded row: rank of an
      // entry = number of entries of the part with a smaller row (rows read back from LDS)
      const int n_q = (n_all + kWave - 1) / kWave;
      int row[kBucketPer], rank[kBucketPer];
      double w[kBucketPer];
#pragma unroll
      for (int q = 0; q < kBucketPer; ++q) {
        const bool in = q * kWave + lane < n_all;
        const int rw = in ? a.tgt_src[ebase + e0 + q * kWave + lane] : 0x7fffffff;
        w[q] = in ? (a.average ? 1.0 : a.tgt_alpha[ebase + e0 + q * kWave + lane]) : 0.0;
        row[q] = (rw >= row_lo && rw < row_hi) ? rw : 0x7fffffff;
        rank[q] = 0;
      }
#pragma unroll
      for (int q = 0; q < kBucketPer; ++q) {
        if (q < n_q) l_src[q * kWave + lane] = row[q];
        n_src += __popcll(__ballot(row[q] != 0x7fffffff));
      }
      const int n_pad = n_q * kWave;
      for (int l0 = 0; l0 < n_pad; l0 += 8) {
        int v[8];
#pragma unroll
        for (int x8 = 0; x8 < 8; ++x8) v[x8] = l_src[l0 + x8];
#pragma unroll
        for (int x8 = 0; x8 < 8; ++x8)
#pragma unroll
          for (int q = 0; q < kBucketPer; ++q) rank[q] += v[x8] < row[q] ? 1 : 0;
      }
      int tok[kBucketPer];
#pragma unroll
      for (int q = 0; q < kBucketPer; ++q)
        tok[q] = row[q] != 0x7fffffff ? a.S[b * a.n_disc + min(max(row[q], 0), a.n_disc - 1)] : 0;
#pragma unroll
      for (int q = 0; q < kBucketPer; ++q) {
        if (row[q] != 0x7fffffff) {      // all reads of the rows above precede these writes
          l_src[rank[q]] = tok[q];
          l_w[rank[q]] = w[q];
        }
      }
    } else if (long_bucket) {
      n_src = sub == 0 ? n_all : 0;      // wavefront 0 takes the whole bucket on the slow path
    }
  }

  // ---- this wavefront's partial sum ----------------------------------------------------------------
  double num[SLICE][kVec];
  double den = sub == 0 ? 1.0 : 0.0;
#pragma unroll
  for (int u = 0; u < SLICE; ++u)
#pragma unroll
    for (int k = 0; k < kVec; ++k) num[u][k] = 0.0;
  if (WPU == 1 && n_src == 0) {  // nothing merged into this row: exact copy
#pragma unroll
    for (int u = 0; u < SLICE; ++u) {
      const int d = d0 + (u * kWave + lane) * kVec;
      if (full[u]) __builtin_memcpy(out + d, &xr[u], sizeof(xr[u]));
      else
        for (int k = 0; k < kVec; ++k)
          if (d + k < a.D) out[d + k] = x[d + k];
    }
    return 0;
  }
  // The row's own value is the first term of the sum.  Where a list follows, it is added after
  // the loads of the list's first batch have been issued: the row's load (issued long ago) and
  // those then share one wait instead of taking two memory round trips in a row.
  if (valid && sub == 0) {
#pragma unroll
    for (int u = 0; u < SLICE; ++u) {
      const int d = d0 + (u * kWave + lane) * kVec;
      if (full[u]) add_raw(xr[u], num[u]);
      else
        for (int k = 0; k < kVec; ++k) num[u][k] = d + k < a.D ? widen(x[d + k]) : 0.0;
    }
  }
  if (n_src > 0) {
    if (!long_bucket && n_src <= kCap) {
      int e = 0;
      for (; e + 8 <= n_src; e += 8) {
        double wv8[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) wv8[q] = l_w[e + q];
#pragma unroll
        for (int q = 0; q < 8; ++q) den += wv8[q];
      }
      for (; e < n_src; ++e) den += l_w[e];
      add_sources<T, SLICE, kRegs>(a, Xb, l_src, l_w, n_src, d0, lane, full, num);
    } else if (!MATCH) {
      // long bucket: take its entries in ascending discarded row by repeated minimum search
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
        if (who == 0) break;             // fewer distinct rows than entries: inconsistent device data
        const int l = __ffsll(who) - 1;
        const int e = __shfl(best_e, l, kWave);
        const double w = a.average ? 1.0 : a.tgt_alpha[ebase + e];
        den += w;
        add_source<T, SLICE>(a, Xb, a.S[b * a.n_disc + min(max(mn, 0), a.n_disc - 1)], w, d0, lane, full, num);
        last = mn;
      }
    }
  }

  // ---- parts added in order by wavefront 0 of the unit -----------------------------------------------
  if (WPU > 1) {
    if (sub > 0) {
      double* dst = part + ((size_t)(unit_l * (WPU - 1) + sub - 1) * SLICE * kVec) * kWave + lane;
#pragma unroll
      for (int u = 0; u < SLICE; ++u)
#pragma unroll
        for (int k = 0; k < kVec; ++k) dst[(u * kVec + k) * kWave] = num[u][k];
    }
    if (lane == 0) { wden[2 * wv] = den; wden[2 * wv + 1] = (double)n_src; }
    __syncthreads();              // every wavefront of the workgroup arrives here exactly once
    if (sub > 0 || !valid) return 0;
    double total = 0.0;
#pragma unroll
    for (int w = 0; w < WPU; ++w) total += wden[2 * (unit_l * WPU + w) + 1];
    if (total == 0.0) {           // nothing merged into this row: exact copy
#pragma unroll
      for (int u = 0; u < SLICE; ++u) {
        const int d = d0 + (u * kWave + lane) * kVec;
        if (full[u]) __builtin_memcpy(out + d, &xr[u], sizeof(xr[u]));
        else
          for (int k = 0; k < kVec; ++k)
            if (d + k < a.D) out[d + k] = x[d + k];
      }
      return 0;
    }
#pragma unroll
    for (int w = 1; w < WPU; ++w) {
      const double* src = part + ((size_t)(unit_l * (WPU - 1) + w - 1) * SLICE * kVec) * kWave + lane;
#pragma unroll
      for (int u = 0; u < SLICE; ++u)
#pragma unroll
        for (int k = 0; k < kVec; ++k) num[u][k] += src[(u * kVec + k) * kWave];
      den += wden[2 * (unit_l * WPU + w)];
    }
  }
#pragma unroll
  for (int u = 0; u < SLICE; ++u) {
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
  return 0;
}

// Scanning mode, targets with more than kHubMin sources (a token that most discarded tokens
// attend to): the eight wavefronts of the workgroup that holds such a unit add it together once
// their own units are done.  The discarded rows are taken 512 at a time: every wavefront scans
// 64 of them, the hits are packed in ascending row order into one list (the LDS of the
// per-wavefront lists), and every wavefront then adds the whole list, 16 row loads in flight,
// to its own 64 * SLICE features of the span: the sum of every output element still runs over
// ascending discarded rows.
template <typename T, int SLICE>
__device__ __forceinline__ void merge_hub_targets(const MergeArgs& a, char* lds_m, int deferred) {
  using Lds = MergeLds<true, SLICE, 1>;
  static_assert(Lds::kCap == kWave, "the shared list holds one hit per scanned row");
  constexpr int kSpan = kWave * kVec * SLICE;
  constexpr int kChunk = kMergeWaves * kWave;
  constexpr int kBatch = 16;
  __shared__ int hub_n[kMergeWaves];
  __shared__ int hit_n[kMergeWaves];
  const int lane = threadIdx.x % kWave, wv = threadIdx.x / kWave;
  if (lane == 0) hub_n[wv] = deferred;
  __syncthreads();            // every wavefront is done with its own list
  double* s_w = (double*)lds_m;
  int* s_src = (int*)((double*)lds_m + kMergeWaves * Lds::kCap);
  const EdgeTable tb = edge_table(lds_m + Lds::kLists + Lds::kPartDoubles * 8 + Lds::kDen, a.n_disc);
  const int n_spans = (a.D + kSpan - 1) / kSpan;
  const int64_t b = blockIdx.y;
  const int64_t ebase = b * (int64_t)a.n_disc * a.k_max;
  const T* Xb = (const T*)a.X + b * a.xsb;
  for (int u = 0; u < kMergeWaves; ++u) {
    if (hub_n[u] == 0) continue;                         // uniform over the workgroup
    const int unit = blockIdx.x * kMergeWaves + u;
    const int r = unit / n_spans;
    const int j = r - a.vis_begin;                       // a deferred unit is a preserved visual row
    const int dl = (unit % n_spans) * kSpan + (wv * kWave + lane) * SLICE;
    const bool whole = dl + SLICE <= a.D;
    const int tok = min(max(a.T[b * a.n_keep + j], 0), a.N - 1);
    const T* x = Xb + (int64_t)(a.vis_begin + tok) * a.xsn;
    T* out = (T*)a.X_out + (b * a.n_out + r) * (int64_t)a.D;
    double num[SLICE];
#pragma unroll
    for (int e = 0; e < SLICE; ++e) num[e] = dl + e < a.D ? widen(x[dl + e]) : 0.0;
    double den = 1.0;
    for (int c0 = 0; c0 < a.n_disc; c0 += kChunk) {
      const int row = c0 + wv * kWave + lane;
      double w = 0.0;
      bool more;
      const bool hit = row_names_target<true>(a, tb, ebase, row, row < a.n_disc, j, w, more);
      const unsigned long long m = __ballot(hit);
      if (lane == 0) hit_n[wv] = __popcll(m);
      __syncthreads();
      int off = 0, n_list = 0;
#pragma unroll
      for (int q = 0; q < kMergeWaves; ++q) {
        const int c = hit_n[q];
        off += q < wv ? c : 0;
        n_list += c;
      }
      if (hit) {
        const int slot = off + __popcll(m & ((1ULL << lane) - 1ULL));
        s_src[slot] = tb.src[row];
        s_w[slot] = w;
      }
      __syncthreads();
      auto row_of = [&](int e) {
        const int i = min(max(s_src[e], 0), a.N - 1);      // device data: stay inside the span
        return Xb + (int64_t)(a.vis_begin + i) * a.xsn;
      };
      if (a.D >= SLICE) {                                  // uniform; straight-line batches as in add_sources
        const int off = whole ? dl : 0;
#pragma unroll 1
        for (int e0 = 0; e0 < n_list; e0 += kBatch) {
          T v[kBatch][SLICE];
#pragma unroll
          for (int q = 0; q < kBatch; ++q)
            __builtin_memcpy(&v[q][0], row_of(min(e0 + q, n_list - 1)) + off, sizeof(T) * SLICE);
          issue_fence();
#pragma unroll
          for (int q = 0; q < kBatch; ++q) {
            const bool in = e0 + q < n_list;               // past the end: the last row again, not counted
            const double wq = s_w[min(e0 + q, n_list - 1)];
            den += in ? wq : 0.0;
#pragma unroll
            for (int e = 0; e < SLICE; ++e) num[e] += whole && in ? wq * widen(v[q][e]) : 0.0;
          }
        }
      } else {
        for (int e0 = 0; e0 < n_list; ++e0) den += s_w[e0];
      }
      if (!whole && dl < a.D) {                            // the lane at the end of a row of odd width
#pragma unroll 1
        for (int e0 = 0; e0 < n_list; ++e0) {
          const T* xs = row_of(e0);
          const double wq = s_w[e0];
#pragma unroll
          for (int e = 0; e < SLICE; ++e)
            if (dl + e < a.D) num[e] += wq * widen(xs[dl + e]);
        }
      }
      __syncthreads();        // the list and the counts are written again by the next chunk or unit
    }
#pragma unroll
    for (int e = 0; e < SLICE; ++e)
      if (dl + e < a.D) store_token(out + dl + e, num[e] / den);
  }
}

// Position ids of the preserved tokens: written last, by one thread per output row of the
// workgroup (two dependent loads that nothing before should wait for).
template <int SLICE>
__device__ __forceinline__ void write_pos_out(const MergeArgs& a, int blk) {
  if (a.pos_out && (int)threadIdx.x < kMergeWaves) {
    constexpr int kSpan = kWave * kVec * SLICE;
    const int n_spans = (a.D + kSpan - 1) / kSpan;
    const int unit = blk * kMergeWaves + threadIdx.x;
    const int r = unit / n_spans;
    const int64_t b = blockIdx.y;
    if (unit % n_spans == 0 && r >= a.vis_begin && r < a.vis_begin + a.n_keep) {
      const int j = r - a.vis_begin;
      const int tok = min(max(a.T[b * a.n_keep + j], 0), a.N - 1);
      a.pos_out[b * a.n_keep + j] = a.pos ? a.pos[b * a.N + tok] : tok;
    }
  }
}

template <typename T, bool MATCH, int SLICE, int WPU>
__global__ __launch_bounds__(kMergeWaves * kWave) void merge_rows_kernel(MergeArgs a) {
  extern __shared__ __attribute__((aligned(16))) char lds_m[];
  const int deferred = merge_unit<T, MATCH, SLICE, WPU>(a, lds_m, blockIdx.x);
  if (MATCH && WPU == 1) merge_hub_targets<T, SLICE>(a, lds_m, deferred);
  if (WPU == 1) write_pos_out<SLICE>(a, blockIdx.x);
}

// Bucket mode, both passes in one launch (no launch gap separates them): the first `hub_blocks`
// workgroups take the targets with long buckets, a whole workgroup per unit -- workgroup w takes
// entries w, w + hub_blocks, ... of the list of such targets (times the spans of a row), as far
// as the list goes -- the others eight units of the one-wavefront pass each.  How long the list
// is only the device knows, so most of the first kind leave at once; but the chip starts only a
// few hundred workgroups per microsecond, empty ones included: with one workgroup per POSSIBLE
// long target ahead of the row workgroups (2304 at 1152 preserved tokens) the rows started 10 to
// 16 us into the launch.  So there is one workgroup for every fourth possible entry (an image
// with more long targets than that takes them in a second trip).  They still come first: the
// long targets take longest, and with the rows ahead of them they wait for a place on the chip.
template <typename T, int SLICE>
__global__ __launch_bounds__(kMergeWaves * kWave) void merge_buckets_kernel(MergeArgs a, int hub_blocks) {
  extern __shared__ __attribute__((aligned(16))) char lds_m[];
  if ((int)blockIdx.x >= hub_blocks) {
    (void)merge_unit<T, false, SLICE, 1>(a, lds_m, blockIdx.x - hub_blocks);
    write_pos_out<SLICE>(a, blockIdx.x - hub_blocks);
  } else {
    constexpr int kSpan = kWave * kVec * SLICE;
    const int n_spans = (a.D + kSpan - 1) / kSpan;
    const int n_units = min(max(a.hub_cnt[blockIdx.y], 0), a.n_keep) * n_spans;     // uniform
    for (int u = (int)blockIdx.x; u < n_units; u += hub_blocks) {
      (void)merge_unit<T, false, SLICE, kMergeWaves>(a, lds_m, u);
      __syncthreads();          // the partial sums in LDS are written again by the next entry
    }
  }
}

// The additional token of the "convergent" ablation: the plain mean of the discarded tokens.
// A workgroup covers 512 features of one image; each of its kExtraWaves wavefronts adds one part
// of the discarded rows in ascending order (16-byte loads of 8 rows in flight), the parts are
// added in order and the sum is divided by N^S.
constexpr int kExtraWaves = 16;
template <typename T>
__global__ __launch_bounds__(kExtraWaves * kWave) void extra_token_kernel(MergeArgs a) {
  __shared__ double part[kExtraWaves - 1][kVec][kWave];
  const int lane = threadIdx.x % kWave, wv = threadIdx.x / kWave;
  const int d = (blockIdx.x * kWave + lane) * kVec;
  const int64_t b = blockIdx.y;
  const int nd = max(min(kVec, a.D - d), 0);
  const int share = (a.n_disc + kExtraWaves - 1) / kExtraWaves;
  const int r0 = min(wv * share, a.n_disc), r1 = min(r0 + share, a.n_disc);
  const T* Xb = (const T*)a.X + b * a.xsb + d;
  double acc[kVec];
#pragma unroll
  for (int k = 0; k < kVec; ++k) acc[k] = 0.0;
  for (int e0 = r0; e0 < r1; e0 += 8) {
    int tok[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int i = a.S[b * a.n_disc + min(e0 + u, r1 - 1)];
      tok[u] = a.vis_begin + min(max(i, 0), a.N - 1);     // index sets are device data: stay inside the span
    }
    if (nd == kVec) {
      Raw8<T> raw[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) load_raw(Xb + (int64_t)tok[u] * a.xsn, raw[u]);
      issue_fence();
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (e0 + u < r1) add_raw(raw[u], acc);
    } else {
      for (int u = 0; u < 8 && e0 + u < r1; ++u)
        for (int k = 0; k < nd; ++k) acc[k] += widen(Xb[(int64_t)tok[u] * a.xsn + k]);
    }
  }
  if (wv > 0) {
#pragma unroll
    for (int k = 0; k < kVec; ++k) part[wv - 1][k][lane] = acc[k];
  }
  __syncthreads();
  if (wv > 0 || nd == 0) return;
  for (int w = 0; w < kExtraWaves - 1; ++w)
#pragma unroll
    for (int k = 0; k < kVec; ++k) acc[k] += part[w][k][lane];
  T* out = (T*)a.X_out + (b * a.n_out + a.extra_row) * (int64_t)a.D + d;
  const double cnt = (double)a.n_disc;
  for (int k = 0; k < nd; ++k) store_token(out + k, acc[k] / cnt);
}


// Scanning mode (few discarded tokens): eight one-wavefront units per workgroup.
template <typename T, int SLICE>
static void launch_merge_scan(const MergeArgs& m, int B, hipStream_t s) {
  using Lds = MergeLds<true, SLICE, 1>;
  constexpr int kSpan = kWave * kVec * SLICE;
  const int n_spans = (m.D + kSpan - 1) / kSpan;
  const size_t lds = Lds::bytes(m.n_disc);
  const int units = m.n_out * n_spans;
  dim3 grid((units + Lds::kUnits - 1) / Lds::kUnits, B), block(kMergeWaves * kWave);
  if (lds > 32768)
    (void)hipFuncSetAttribute((const void*)merge_rows_kernel<T, true, SLICE, 1>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  hipLaunchKernelGGL((merge_rows_kernel<T, true, SLICE, 1>), grid, block, lds, s, m);
}

template <typename T, int SLICE>
static void launch_merge_buckets(const MergeArgs& m, int B, hipStream_t s) {
  using L1 = MergeLds<false, SLICE, 1>;
  using L8 = MergeLds<false, SLICE, kMergeWaves>;
  constexpr int kSpan = kWave * kVec * SLICE;
  const int n_spans = (m.D + kSpan - 1) / kSpan;
  const size_t lds = std::max(L1::bytes(m.n_disc), L8::bytes(m.n_disc));
  const int hub_units = m.n_keep * n_spans;                        // at most every preserved token has a long bucket
  const int hub_blocks = std::min(hub_units, std::max(64, (hub_units + 3) / 4));
  const int row_blocks = (m.n_out * n_spans + L1::kUnits - 1) / L1::kUnits;
  if (lds > 32768)
    (void)hipFuncSetAttribute((const void*)merge_buckets_kernel<T, SLICE>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  hipLaunchKernelGGL((merge_buckets_kernel<T, SLICE>), dim3(row_blocks + hub_blocks, B), dim3(kMergeWaves * kWave), lds, s, m,
                     hub_blocks);
}

void launch_compress(const ficoco_problem& p, const Plan& pl, char* ws, const int32_t* discard_idx,
                     const int32_t* keep_idx, const int32_t* edge_cnt, const int32_t* edge_tgt,
                     const double* edge_alpha, void* X_out, int32_t* pos_out,
                     hipStream_t s, bool targets_counted) {
  const bool match = !edges_inverted(pl);
  if (pl.n_disc > 0 && !match) {
    InvertArgs a{};
    a.n_keep = p.n_keep; a.n_disc = pl.n_disc; a.k_max = p.k_max;
    a.edge_cnt = edge_cnt; a.edge_tgt = edge_tgt; a.edge_alpha = edge_alpha;
    a.tgt_ptr = (int32_t*)(ws + pl.tgt_ptr);
    a.tgt_src = (int32_t*)(ws + pl.tgt_src);
    a.tgt_alpha = (double*)(ws + pl.tgt_alpha);
    a.hub_list = (int32_t*)(ws + pl.hub_list);
    a.hub_cnt = (int32_t*)(ws + pl.hub_cnt);
    const size_t lds = ((size_t)2 * p.n_keep + 1 + 2 * kSelectThreads) * sizeof(int);
    // four slots per load where every row of the lists starts on a 16-byte boundary
    const bool quads = p.k_max % 4 == 0 && reinterpret_cast<uintptr_t>(edge_tgt) % 16 == 0 &&
                       reinterpret_cast<uintptr_t>(edge_alpha) % 16 == 0;
    auto kern = quads ? invert_edges_kernel<4> : invert_edges_kernel<1>;
    if (lds > 32768)
      (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    a.share_cnt = targets_counted ? (const int32_t*)(ws + pl.share_cnt) : nullptr;
    a.share_rows = invert_share_rows(pl);
    hipLaunchKernelGGL(kern, dim3(invert_groups(pl), p.B), dim3(kSelectThreads), lds, s, a);
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
  m.pos = p.pos; m.pos_out = pos_out;
  m.average = p.compress_mode == FICOCO_COMPRESS_AVERAGE ? 1 : 0;
  m.pair_tab = targets_counted && match && pair_records(p, pl) ? (const PairRec*)(ws + pl.pair_tab) : nullptr;
  m.extra_row = pl.extra_token ? p.vis_begin + p.n_keep : -1;
  // Narrow spans (one 8-element vector per lane) double the number of wavefronts: taken when the
  // wide ones would not fill the chip.  Bucket mode has two kinds of workgroups in its one launch:
  // eight units with one wavefront each for the targets with at most kHubMin sources, and a whole
  // workgroup per unit (eight wavefronts, each adding the sources of one part of the discarded
  // rows, parts added in order) for the few targets with long buckets, whose serial row loads
  // would otherwise set the kernel's duration.
  const int slice = (int64_t)p.B * pl.n_out * ((p.D + 1023) / 1024) >= 4096 ? 2 : 1;
  const bool bf16 = p.dtype == FICOCO_BF16;
  if (match) {
    if (bf16) { if (slice == 1) launch_merge_scan<bf16_t, 1>(m, p.B, s); else launch_merge_scan<bf16_t, 2>(m, p.B, s); }
    else { if (slice == 1) launch_merge_scan<float, 1>(m, p.B, s); else launch_merge_scan<float, 2>(m, p.B, s); }
  } else {
    m.hub_list = (const int32_t*)(ws + pl.hub_list);
    m.hub_cnt = (const int32_t*)(ws + pl.hub_cnt);
    if (bf16) { if (slice == 1) launch_merge_buckets<bf16_t, 1>(m, p.B, s); else launch_merge_buckets<bf16_t, 2>(m, p.B, s); }
    else { if (slice == 1) launch_merge_buckets<float, 1>(m, p.B, s); else launch_merge_buckets<float, 2>(m, p.B, s); }
  }
  if (m.extra_row >= 0) {
    dim3 grid((p.D + kWave * kVec - 1) / (kWave * kVec), p.B);
    if (p.dtype == FICOCO_BF16) hipLaunchKernelGGL(extra_token_kernel<bf16_t>, grid, dim3(kExtraWaves * kWave), 0, s, m);
    else hipLaunchKernelGGL(extra_token_kernel<float>, grid, dim3(kExtraWaves * kWave), 0, s, m);
  }
}

// Row gather by the preserved sequence (key / value cache, position ids): one wavefront per
// (output row, span of 64 vectors), bytes copied unchanged.
struct GatherArgs {
  const char* in;
  int64_t sb, sn;
  char* out;
  int row_bytes, n_out, vis_begin, n_keep, n_disc, N;
  const int32_t* T;
};

template <typename V>
__global__ __launch_bounds__(256) void gather_rows_kernel(GatherArgs a) {
  const int lane = threadIdx.x % kWave, wv = threadIdx.x / kWave;
  const int per_row = (a.row_bytes + (int)sizeof(V) * kWave - 1) / ((int)sizeof(V) * kWave);
  const int unit = blockIdx.x * 4 + wv;
  const int r = unit / per_row;
  const int off = ((unit % per_row) * kWave + lane) * (int)sizeof(V);
  const int64_t b = blockIdx.y;
  if (r >= a.n_out || off >= a.row_bytes) return;
  int t;
  if (r < a.vis_begin) t = r;
  else if (r < a.vis_begin + a.n_keep) t = a.vis_begin + min(max(a.T[b * a.n_keep + r - a.vis_begin], 0), a.N - 1);
  else t = r + a.n_disc;
  const V v = *reinterpret_cast<const V*>(a.in + b * a.sb + (int64_t)t * a.sn + off);
  *reinterpret_cast<V*>(a.out + (b * a.n_out + r) * (int64_t)a.row_bytes + off) = v;
}

void launch_gather(const ficoco_problem& p, const Plan& pl, const int32_t* keep_idx, const void* in,
                   int64_t sb, int64_t sn, int row_bytes, void* out, hipStream_t s) {
  GatherArgs a{(const char*)in, sb, sn, (char*)out, row_bytes, pl.n_out, p.vis_begin, p.n_keep, pl.n_disc, p.N, keep_idx};
  const bool wide = row_bytes % 16 == 0 && sb % 16 == 0 && sn % 16 == 0 && ((uintptr_t)in % 16) == 0 &&
                    ((uintptr_t)out % 16) == 0;
  const int vec = wide ? 16 : 4;
  const int per_row = (row_bytes + vec * kWave - 1) / (vec * kWave);
  dim3 grid((pl.n_out * per_row + 3) / 4, p.B), block(256);
  if (wide) hipLaunchKernelGGL(gather_rows_kernel<uint4>, grid, block, 0, s, a);
  else hipLaunchKernelGGL(gather_rows_kernel<uint32_t>, grid, block, 0, s, a);
}

}  // namespace ficoco

