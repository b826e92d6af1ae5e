// Filter stage: redundancy score (Eq. 1 / Eq. 3), local penalty (Sec. "Redundancy-based
// Token Discard") and the top-K split into source set S and target set T (Algorithm 1/2,
// stage 1).  One workgroup per image; the per-image state lives in LDS.  All comparisons
// are on doubles (through order-preserving 64-bit keys); ties go to the lower token index
// (filter) / lower grid cell (penalty).
//
// The same kernel serves the staged entry points (score only / filter only) and the fused
// step (both phases in one launch: every dependent launch costs several microseconds).
//
// The top-K is a radix select: 8 passes over the key bytes, most significant first, find the
// key K* of the N^S-th largest token; tokens above K* are discarded, tokens equal to K* are
// discarded in index order until N^S is reached.  Integer LDS atomics only build histograms
// (their result does not depend on the order of arrival).
#include "common.hpp"

namespace ficoco {

struct SelectArgs {
  int N, H, M, n_chunks, dtype;
  int red_src, sem_src;
  int do_score, do_filter;
  const double* recv_part;  // [B][n_chunks][N]
  const double* cls;        // [B][N]
  const double* ttext;      // [B][N][M]
  const void* recv_vec;     // [B][H][N]
  const void* sem_vec;
  const double* fterm_r;    // [B][N] mean cosine
  const double* fterm_g;    // [B][N] equivalent-token term
  double w;
  const int32_t* pos;
  int grid_g, grid_h, grid_w, window;
  double coef;
  double* scores;           // out (do_score) / in (filter only)
  int n_disc;
  int32_t* discard_idx;
  int32_t* keep_idx;
  int32_t* slot_of;
  int32_t* overflow;        // zeroed here for the correlate stage (fused step only), may be null
};

// head mean of a pre-reduced per-head vector entry: 16 independent loads at a time, added in
// head order
template <typename T>
__device__ __forceinline__ double vec_head_sum(const T* p, int H, int N) {
  double acc = 0.0;
  int h = 0;
  for (; h + 16 <= H; h += 16) {
    T v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) v[u] = p[(int64_t)(h + u) * N];
#pragma unroll
    for (int u = 0; u < 16; ++u) acc += widen(v[u]);
  }
  for (; h < H; ++h) acc += widen(p[(int64_t)h * N]);
  return acc;
}
__device__ __forceinline__ double vec_head_mean(const void* v, int dtype, int64_t b, int H, int N, int i) {
  const double acc = dtype == FICOCO_BF16 ? vec_head_sum((const bf16_t*)v + b * H * (int64_t)N + i, H, N)
                                          : vec_head_sum((const float*)v + b * H * (int64_t)N + i, H, N);
  return acc * (1.0 / (double)H);
}

// Eq. 1 / Eq. 3 with both products rounded before the subtraction (no fused multiply-add): given
// the same R and G, the score is then the same double as in the plain statement.
__device__ __forceinline__ double combine_terms(double w, double R, double G) {
#pragma clang fp contract(off)
  const double first = w * R;
  const double second = (1.0 - w) * G;
  return first - second;
}

__device__ __forceinline__ uint64_t score_key(double s) {
  const uint64_t u = (uint64_t)__double_as_longlong(s + 0.0);   // -0 folded into +0
  return (u >> 63) ? ~u : (u | 0x8000000000000000ULL);
}

constexpr int kTokensPerThread = (kMaxSelectN + kSelectThreads - 1) / kSelectThreads;   // sequences longer than kSelectThreads run with kSelectThreads threads
constexpr int kBinCopies = 32;      // counters per histogram bin in the many-keys form: one per LDS bank
constexpr int kSpreadMinN = 4096;   // tokens from which that form is used (it costs one more barrier per pass)
static_assert(kSelectThreads == 4 * 256, "four threads fold the counters of one bin");

__global__ __launch_bounds__(kSelectThreads) void select_kernel(SelectArgs a) {
  DBG_SPAN(1);
  extern __shared__ double lds_d[];
  double* s = lds_d;                                   // [N] scores, then keys in place
  uint64_t* keys = (uint64_t*)lds_d;
  int* ibase = (int*)(lds_d + a.N);
  int* scan = ibase;                                   // [2][nt]
  int* hist = ibase + 2 * kSelectThreads;              // [256]
  int* bcast = hist + 256;                             // [4]
  int* owner = bcast + 4;                              // [cells] (penalty only)
  const int b = blockIdx.x, tid = threadIdx.x, nt = blockDim.x;
  const int N = a.N;

  DBG_PHASE(0);
  if (a.do_score) {
    // Both terms one stored value per token, and several tokens per thread: all of the thread's
    // loads are issued before the first use (the general loop below takes a trip to memory per token).
    const double* r_one = a.red_src == FICOCO_R_ATTN_RECV ? (a.n_chunks == 1 ? a.recv_part : nullptr)
                        : a.red_src == FICOCO_R_VECTOR ? nullptr : a.fterm_r;
    const double* g_one = a.sem_src == FICOCO_G_CLS_ATTN ? a.cls
                        : (a.sem_src == FICOCO_G_TEXT_ATTN || a.sem_src == FICOCO_G_VECTOR) ? nullptr : a.fterm_g;
    const bool one_each = r_one && g_one && N > nt;      // uniform
    if (one_each) {
      double r[kTokensPerThread], g[kTokensPerThread];
#pragma unroll
      for (int u = 0; u < kTokensPerThread; ++u) {
        const int i = min(tid + u * nt, N - 1);          // clamped: always a valid address
        r[u] = r_one[(int64_t)b * N + i];
        g[u] = g_one[(int64_t)b * N + i];
      }
      issue_fence();
#pragma unroll
      for (int u = 0; u < kTokensPerThread; ++u) {
        const int i = tid + u * nt;
        if (i < N) s[i] = combine_terms(a.w, a.red_src == FICOCO_R_ATTN_RECV ? (0.0 + r[u]) / (double)N : r[u], g[u]);
      }
    }
    for (int i = tid; i < (one_each ? 0 : N); i += nt) {
      double R, G;
      if (a.red_src == FICOCO_R_ATTN_RECV) {
        const double* p = a.recv_part + (int64_t)b * a.n_chunks * N + i;
        double acc = 0.0;
        int c = 0;
        for (; c + 32 <= a.n_chunks; c += 32) {          // 32 independent loads, added in order
          double v[32];
#pragma unroll
          for (int u = 0; u < 32; ++u) v[u] = p[(int64_t)(c + u) * N];
#pragma unroll
          for (int u = 0; u < 32; ++u) acc += v[u];
        }
        for (; c + 8 <= a.n_chunks; c += 8) {
          double v[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) v[u] = p[(int64_t)(c + u) * N];
#pragma unroll
          for (int u = 0; u < 8; ++u) acc += v[u];
        }
        for (; c < a.n_chunks; ++c) acc += p[(int64_t)c * N];
        R = acc / (double)N;
      } else if (a.red_src == FICOCO_R_VECTOR) {
        R = vec_head_mean(a.recv_vec, a.dtype, b, a.H, N, i);
      } else {
        R = a.fterm_r[(int64_t)b * N + i];
      }
      if (a.sem_src == FICOCO_G_CLS_ATTN) {
        G = a.cls[(int64_t)b * N + i];
      } else if (a.sem_src == FICOCO_G_TEXT_ATTN) {
        const double* p = a.ttext + ((int64_t)b * N + i) * a.M;
        double acc = 0.0;
        int k = 0;
        for (; k + 16 <= a.M; k += 16) {                  // 16 independent loads, added in order
          double v[16];
#pragma unroll
          for (int u = 0; u < 16; ++u) v[u] = p[k + u];
#pragma unroll
          for (int u = 0; u < 16; ++u) acc += v[u];
        }
        for (; k < a.M; ++k) acc += p[k];
        G = acc / (double)a.M;
      } else if (a.sem_src == FICOCO_G_VECTOR) {
        G = vec_head_mean(a.sem_vec, a.dtype, b, a.H, N, i);
      } else {
        G = a.fterm_g[(int64_t)b * N + i];
      }
      s[i] = combine_terms(a.w, R, G);
    }
    DBG_PHASE(1);
    if (a.window > 0) {
      const int cells = a.grid_g * a.grid_h * a.grid_w;
      for (int c = tid; c < cells; c += nt) owner[c] = -1;
      __syncthreads();
      for (int i = tid; i < N; i += nt) {
        const int c = a.pos ? a.pos[(int64_t)b * N + i] : i;
        if (c >= 0 && c < cells) owner[c] = i;
      }
      __syncthreads();
      const int W = a.window;
      const int wr = (a.grid_h + W - 1) / W, wc = (a.grid_w + W - 1) / W;
      const int n_win = a.grid_g * wr * wc;
      for (int w = tid; w < n_win; w += nt) {
        const int sub = w / (wr * wc), rem = w % (wr * wc);
        const int r0 = (rem / wc) * W, c0 = (rem % wc) * W;
        int best = -1;
        double best_s = 0.0;
        for (int r = r0; r < min(r0 + W, a.grid_h); ++r)
          for (int c = c0; c < min(c0 + W, a.grid_w); ++c) {
            const int t = owner[(sub * a.grid_h + r) * a.grid_w + c];
            if (t >= 0 && (best < 0 || s[t] > best_s)) { best = t; best_s = s[t]; }
          }
        if (best >= 0) s[best] = a.coef * best_s;   // windows are disjoint: no other reader
      }
    }
    __syncthreads();
    for (int i = tid; i < N; i += nt) a.scores[(int64_t)b * N + i] = s[i];
  } else {
    for (int i = tid; i < N; i += nt) s[i] = a.scores[(int64_t)b * N + i];
  }
  DBG_PHASE(2);
  if (!a.do_filter) return;
  if (a.overflow && tid == 0) a.overflow[b] = 0;
  __syncthreads();
  for (int i = tid; i < N; i += nt) keys[i] = score_key(s[i]);   // in place: same 8-byte slots
  __syncthreads();

  // ---- radix select of the n_disc-th largest key -------------------------------------------
  uint64_t kstar = 0;
  int need = a.n_disc;   // how many of the current candidates (keys matching the prefix) to take from the top
  if (a.n_disc > 0) {
    uint64_t* small = (uint64_t*)hist;   // candidate keys once at most 64 are left (after the histogram is spent)
    const bool spread = N >= kSpreadMinN;   // uniform
    int* hist_wide = owner;              // [256][kBinCopies]: the penalty's table is no longer needed
    for (int pass = 0; pass < 8; ++pass) {
      const int shift = 56 - 8 * pass;
      const uint64_t hi_mask = pass == 0 ? 0ULL : (~0ULL << (shift + 8));
      if (spread) {
        // Many keys per thread: scores of one image share their leading digits, so in the first
        // passes nearly all atomics would queue on one LDS address (one lane per cycle).  Every
        // bin has 32 counters here, one per bank, lane l adding to counter l % 32 -- no two
        // lanes of an instruction meet -- and four threads per bin fold them afterwards.
        for (int j = tid; j < 256 * kBinCopies; j += nt) hist_wide[j] = 0;
        __syncthreads();
        for (int i = tid; i < N; i += nt) {
          const uint64_t k = keys[i];
          if ((k & hi_mask) == kstar) atomicAdd(&hist_wide[(int)((k >> shift) & 255) * kBinCopies + tid % kBinCopies], 1);
        }
        __syncthreads();
        const int bin = tid / 4, part = tid % 4;           // 1024 threads: four per bin
        int sum = 0;
#pragma unroll
        for (int c = 0; c < kBinCopies / 4; ++c)           // rotated by the bin so that neighbouring bins read different banks
          sum += hist_wide[bin * kBinCopies + (part * (kBinCopies / 4) + c + bin) % kBinCopies];
        sum += __shfl_xor(sum, 1, kWave);
        sum += __shfl_xor(sum, 2, kWave);
        if (part == 0) hist[bin] = sum;
      } else {
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        for (int i = tid; i < N; i += nt) {
          const uint64_t k = keys[i];
          if ((k & hi_mask) == kstar) atomicAdd(&hist[(int)((k >> shift) & 255)], 1);
        }
      }
      __syncthreads();
      if (tid < kWave) {
        // Wavefront 0 walks the 256 bins from the top: lane l owns bins 4l .. 4l+3.
        int h[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) h[k] = hist[4 * tid + k];
        const int lsum = h[0] + h[1] + h[2] + h[3];
        int incl = lsum;                                   // sum over lanes >= this one
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
          const int t = __shfl_down(incl, off, kWave);
          if (tid + off < kWave) incl += t;
        }
        int above = incl - lsum;                           // tokens in bins above this lane's
        if (above < need && need <= above + lsum) {        // exactly one lane
#pragma unroll
          for (int k = 3; k >= 0; --k) {
            if (above < need && need <= above + h[k]) {
              bcast[0] = 4 * tid + k; bcast[1] = need - above; bcast[2] = h[k];
            }
            above += h[k];
          }
        }
      }
      __syncthreads();
      kstar |= (uint64_t)bcast[0] << shift;
      need = bcast[1];
      const int left = bcast[2];
      __syncthreads();
      if (left <= kWave && shift > 0) {
        // Few candidates left: rank them directly in one wavefront instead of more passes.
        if (tid == 0) bcast[3] = 0;
        __syncthreads();
        const uint64_t m2 = ~0ULL << shift;
        for (int i = tid; i < N; i += nt) {
          const uint64_t k = keys[i];
          if ((k & m2) == kstar) { const int slot = atomicAdd(&bcast[3], 1); if (slot < kWave) small[slot] = k; }
        }
        __syncthreads();
        if (tid < kWave) {
          const uint64_t mine = tid < left ? small[tid] : 0ULL;
          int greater = 0, equal = 0;
          for (int l = 0; l < left; ++l) {
            const uint64_t o = small[l];
            greater += o > mine ? 1 : 0;
            equal += o == mine ? 1 : 0;
          }
          if (tid < left && greater < need && need <= greater + equal) {   // all such lanes agree
            small[kWave] = mine;
            bcast[1] = need - greater;
          }
        }
        __syncthreads();
        kstar = small[kWave];
        need = bcast[1];
        __syncthreads();
        break;
      }
    }
  }
  DBG_PHASE(3);
  // need = how many tokens with key == kstar are discarded (lowest indices first)

  // ---- flags and ordered compaction -----------------------------------------------------------
  const int per = (N + nt - 1) / nt;
  const int lo = min(tid * per, N), hi = min(lo + per, N);
  // One scan carries both counts of this thread's tokens: keys above K* (upper half) and keys
  // equal to K* (lower half); neither total exceeds N <= 12288.  The discarded tokens before
  // `lo` are then the ones above K* plus the first `need` of the equal ones.
  int n_eq = 0, n_gt = 0;
  for (int i = lo; i < hi; ++i) {
    const uint64_t k = keys[i];
    n_eq += (a.n_disc > 0 && k == kstar) ? 1 : 0;
    n_gt += (a.n_disc > 0 && k > kstar) ? 1 : 0;
  }
  int tot;
  const int packed = block_scan_inclusive((n_gt << 16) | n_eq, scan, &tot) - ((n_gt << 16) | n_eq);
  int eq_before = packed & 0xffff;
  const int gt_before = packed >> 16;
  int d_pos = gt_before + min(eq_before, need);                   // discarded tokens before `lo`
  int k_pos = lo - d_pos;                                         // preserved tokens before `lo`
  uint32_t dis_mask = 0;  // per <= 12 tokens per thread (N <= kMaxSelectN)
  for (int i = lo; i < hi; ++i) {
    const uint64_t k = keys[i];
    bool dis = false;
    if (a.n_disc > 0) {
      if (k > kstar) dis = true;
      else if (k == kstar) { dis = eq_before < need; ++eq_before; }
    }
    if (dis) dis_mask |= 1u << (i - lo);
  }
  DBG_PHASE(4);
  const int n_keep = N - a.n_disc;
  for (int i = lo; i < hi; ++i) {
    if (dis_mask & (1u << (i - lo))) {
      if (d_pos < a.n_disc) a.discard_idx[(int64_t)b * a.n_disc + d_pos] = i;
      a.slot_of[(int64_t)b * N + i] = -1;
      ++d_pos;
    } else {
      if (k_pos < n_keep) a.keep_idx[(int64_t)b * n_keep + k_pos] = i;
      a.slot_of[(int64_t)b * N + i] = k_pos;
      ++k_pos;
    }
  }
  DBG_PHASE(5);
}

// Large problems (many row chunks and more columns than one workgroup has threads): the
// per-column partial sums are added up by a grid of workgroups first, in chunk order, so the
// single per-image workgroup of select_kernel reads one value per column.
__global__ __launch_bounds__(256) void combine_partials_kernel(const double* __restrict__ part, double* __restrict__ out,
                                                               int N, int n_chunks) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t b = blockIdx.y;
  if (i >= N) return;
  const double* p = part + b * n_chunks * (int64_t)N + i;
  double acc = 0.0;
  int c = 0;
  for (; c + 16 <= n_chunks; c += 16) {
    double v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) v[u] = p[(int64_t)(c + u) * N];
#pragma unroll
    for (int u = 0; u < 16; ++u) acc += v[u];
  }
  for (; c < n_chunks; ++c) acc += p[(int64_t)c * N];
  out[b * N + i] = acc;
}

// Long sequences with per-head vectors as score terms: their head means are formed by a grid
// of workgroups first (same arithmetic), so the per-image workgroup of select_kernel reads one
// value per token and term instead of 2 H strided ones.
__global__ __launch_bounds__(256) void vector_terms_kernel(const void* recv_vec, const void* sem_vec, int dtype, int H,
                                                           int N, double* __restrict__ out_r,
                                                           double* __restrict__ out_g) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t b = blockIdx.y;
  if (i >= N) return;
  if (recv_vec) out_r[b * N + i] = vec_head_mean(recv_vec, dtype, b, H, N, i);
  if (sem_vec) out_g[b * N + i] = vec_head_mean(sem_vec, dtype, b, H, N, i);
}

// From 32 text queries on: the task term of Eq. 3, the mean of a token's text profile, is formed
// by one wavefront per token on the whole chip (lane sums over k = lane, lane + 64, ..., then a
// fixed tree), so the per-image workgroup of select_kernel reads one value.  A thread of that
// workgroup walking its token's profile touches a cache line per lane and load, all on one
// compute unit (64 queries: 17 us for the select kernel against 9 + 4 us this way).
__global__ __launch_bounds__(256) void text_mean_kernel(const double* __restrict__ ttext, int N, int M,
                                                        double* __restrict__ out_g) {
  const int lane = threadIdx.x % kWave;
  const int i = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
  const int64_t b = blockIdx.y;
  if (i >= N) return;      // whole wavefront leaves together
  const double* p = ttext + (b * N + i) * M;
  double acc = 0.0;
  for (int k = lane; k < M; k += kWave) acc += p[k];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, kWave);
  if (lane == 0) out_g[b * N + i] = acc / (double)M;
}

static size_t select_lds(const ficoco_problem& p, bool penalty) {
  const size_t cells = penalty ? (size_t)p.grid_g * p.grid_h * p.grid_w : 0;
  const size_t wide = p.N >= kSpreadMinN ? 256 * kBinCopies : 0;   // shares the penalty table's space
  return (size_t)p.N * sizeof(double) + (2 * kSelectThreads + 256 + 4 + (cells > wide ? cells : wide)) * sizeof(int);
}

void launch_select(const ficoco_problem& p, const Plan& pl, char* ws, double* scores, bool do_score,
                   bool do_filter, int32_t* discard_idx, int32_t* keep_idx, int32_t* overflow,
                   hipStream_t s) {
  SelectArgs a{};
  a.N = p.N; a.H = p.H; a.M = p.M; a.n_chunks = pl.n_chunks; a.dtype = p.dtype;
  a.red_src = p.red_src; a.sem_src = p.sem_src;
  a.do_score = do_score; a.do_filter = do_filter;
  a.recv_part = (const double*)(ws + pl.recv_part);
  if (do_score && p.red_src == FICOCO_R_ATTN_RECV &&
      (int64_t)pl.n_chunks * ((p.N + kSelectThreads - 1) / kSelectThreads) > 128) {
    double* sums = (double*)(ws + pl.fterm);     // free in this mode (it holds the mean-cosine term otherwise)
    hipLaunchKernelGGL(combine_partials_kernel, dim3((p.N + 255) / 256, p.B), dim3(256), 0, s, a.recv_part, sums,
                       p.N, pl.n_chunks);
    a.recv_part = sums;
    a.n_chunks = 1;
  }
  a.cls = (const double*)(ws + pl.cls);
  a.ttext = (const double*)(ws + pl.ttext);
  a.recv_vec = p.recv_vec; a.sem_vec = p.sem_vec;
  a.fterm_r = (const double*)(ws + pl.fterm);
  a.fterm_g = (const double*)(ws + pl.fterm2);
  if (do_score && p.N > 2 * kSelectThreads && (p.red_src == FICOCO_R_VECTOR || p.sem_src == FICOCO_G_VECTOR)) {
    // the term buffers of the vector-sourced terms are free (the feature stage fills only the others)
    const bool vr = p.red_src == FICOCO_R_VECTOR, vg = p.sem_src == FICOCO_G_VECTOR;
    hipLaunchKernelGGL(vector_terms_kernel, dim3((p.N + 255) / 256, p.B), dim3(256), 0, s, vr ? p.recv_vec : nullptr,
                       vg ? p.sem_vec : nullptr, (int)p.dtype, p.H, p.N, (double*)(ws + pl.fterm),
                       (double*)(ws + pl.fterm2));
    if (vr) a.red_src = FICOCO_R_SIM_MEAN;     // "read the precomputed term"
    if (vg) a.sem_src = FICOCO_G_EQ_TOKEN;
  }
  if (do_score && p.sem_src == FICOCO_G_TEXT_ATTN && p.M >= 32) {
    // the equivalent-token buffer is free in FiCoCo-L
    hipLaunchKernelGGL(text_mean_kernel, dim3((p.N + 3) / 4, p.B), dim3(256), 0, s, a.ttext, p.N, p.M,
                       (double*)(ws + pl.fterm2));
    a.sem_src = FICOCO_G_EQ_TOKEN;             // "read the precomputed term"
  }
  a.w = (double)p.w_score;
  const bool penalty = p.variant == FICOCO_VARIANT_V && p.window > 0;
  a.pos = p.pos;
  a.grid_g = p.grid_g; a.grid_h = p.grid_h; a.grid_w = p.grid_w;
  a.window = penalty ? p.window : 0;
  a.coef = (double)p.penalty_coef;
  a.scores = scores;
  a.n_disc = pl.n_disc;
  a.discard_idx = discard_idx; a.keep_idx = keep_idx;
  a.slot_of = (int32_t*)(ws + pl.slot_of);
  a.overflow = overflow;
  const size_t lds = select_lds(p, penalty);
  if (lds > 32768)
    (void)hipFuncSetAttribute((const void*)select_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  // Short sequences: no more wavefronts than tokens need (every barrier of the kernel waits for
  // all of them); at least 256 threads, which the histogram walk assumes.
  const int threads = p.N >= kSelectThreads ? kSelectThreads : std::max(256, (p.N + kWave - 1) / kWave * kWave);
  hipLaunchKernelGGL(select_kernel, dim3(p.B), dim3(threads), lds, s, a);
}

void launch_score(const ficoco_problem& p, const Plan& pl, char* ws, double* scores, hipStream_t s) {
  launch_select(p, pl, ws, scores, true, false, nullptr, nullptr, nullptr, s);
}

void launch_filter(const ficoco_problem& p, const Plan& pl, char* ws, const double* scores,
                   int32_t* discard_idx, int32_t* keep_idx, hipStream_t s) {
  launch_select(p, pl, ws, const_cast<double*>(scores), false, true, discard_idx, keep_idx, nullptr, s);
}

}  // namespace ficoco

FICOCO_DBG_READER(select)
