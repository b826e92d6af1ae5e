// Filter stage: redundancy score (Eq. 1 / Eq. 3), local penalty (Sec. "Redundancy-based
// Token Discard") and the top-K split into source set S and target set T (Algorithm 1/2,
// stage 1).  One workgroup per image; the per-image state lives in LDS.  All comparisons
// are on doubles; ties go to the lower token index (filter) / lower grid cell (penalty).
#include "common.hpp"

namespace ficoco {

struct ScoreArgs {
  int N, H, M, n_chunks, dtype;
  int red_src, sem_src;
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
  double* scores;
};

__device__ __forceinline__ double vec_head_mean(const void* v, int dtype, int64_t b, int H, int N, int i) {
  double acc = 0.0;
  if (dtype == FICOCO_BF16) {
    const bf16_t* p = (const bf16_t*)v + b * H * (int64_t)N + i;
    for (int h = 0; h < H; ++h) acc += widen(p[(int64_t)h * N]);
  } else {
    const float* p = (const float*)v + b * H * (int64_t)N + i;
    for (int h = 0; h < H; ++h) acc += widen(p[(int64_t)h * N]);
  }
  return acc * (1.0 / (double)H);
}

__global__ __launch_bounds__(kSelectThreads) void score_kernel(ScoreArgs a) {
  extern __shared__ double lds_d[];
  double* s = lds_d;                              // [N]
  const int cells = a.grid_g * a.grid_h * a.grid_w;
  int* owner = (int*)(lds_d + a.N);               // [cells] (penalty only)
  const int b = blockIdx.x, tid = threadIdx.x, nt = blockDim.x;
  const int N = a.N;

  for (int i = tid; i < N; i += nt) {
    double R, G;
    if (a.red_src == FICOCO_R_ATTN_RECV) {
      const double* p = a.recv_part + (int64_t)b * a.n_chunks * N + i;
      double acc = 0.0;
      for (int c = 0; c < a.n_chunks; ++c) acc += p[(int64_t)c * N];
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
      for (int k = 0; k < a.M; ++k) acc += p[k];
      G = acc / (double)a.M;
    } else if (a.sem_src == FICOCO_G_VECTOR) {
      G = vec_head_mean(a.sem_vec, a.dtype, b, a.H, N, i);
    } else {
      G = a.fterm_g[(int64_t)b * N + i];
    }
    s[i] = a.w * R - (1.0 - a.w) * G;
  }
  if (a.window > 0) {
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
}

struct FilterArgs {
  int N, n_disc;
  const double* scores;
  int32_t* discard_idx;
  int32_t* keep_idx;
  int32_t* slot_of;
};

__global__ __launch_bounds__(kSelectThreads) void filter_kernel(FilterArgs a) {
  extern __shared__ double lds_d[];
  uint64_t* keys = (uint64_t*)lds_d;        // [N]
  int* scan = (int*)(lds_d + a.N);          // [2][nt]
  const int b = blockIdx.x, tid = threadIdx.x, nt = blockDim.x;
  const int N = a.N;
  for (int i = tid; i < N; i += nt) {
    const uint64_t u = (uint64_t)__double_as_longlong(a.scores[(int64_t)b * N + i] + 0.0);
    keys[i] = (u >> 63) ? ~u : (u | 0x8000000000000000ULL);
  }
  __syncthreads();

  // Thread t owns the contiguous tokens [t*per, (t+1)*per).  rank_i = number of tokens
  // that come before i in (score descending, index ascending) order.  The comparison runs
  // on order-preserving integer keys of the doubles (-0 folded into +0), which is the same
  // order for finite scores and stays a strict total order whatever the bits are, so
  // exactly n_disc tokens are flagged even for non-finite input.
  const int per = (N + nt - 1) / nt;
  const int lo = min(tid * per, N), hi = min(lo + per, N);
  int n_dis = 0;
  uint32_t dis_mask = 0;  // per <= 12 tokens per thread (N <= kMaxSelectN)
  for (int i = lo; i < hi; ++i) {
    const uint64_t ki = keys[i];
    int rank = 0;
    for (int j = 0; j < N; ++j) {
      const uint64_t kj = keys[j];
      rank += (kj > ki || (kj == ki && j < i)) ? 1 : 0;
    }
    if (rank < a.n_disc) { dis_mask |= 1u << (i - lo); ++n_dis; }
  }
  // exclusive scan of the per-thread discard counts
  int* cur = scan;
  int* nxt = scan + nt;
  cur[tid] = n_dis;
  __syncthreads();
  for (int off = 1; off < nt; off <<= 1) {
    nxt[tid] = cur[tid] + (tid >= off ? cur[tid - off] : 0);
    __syncthreads();
    int* t = cur; cur = nxt; nxt = t;
  }
  int d_pos = cur[tid] - n_dis;   // discarded tokens before `lo`
  int k_pos = lo - d_pos;         // preserved tokens before `lo`
  const int n_keep = N - a.n_disc;
  for (int i = lo; i < hi; ++i) {
    if (dis_mask & (1u << (i - lo))) {
      a.discard_idx[(int64_t)b * a.n_disc + d_pos] = i;
      a.slot_of[(int64_t)b * N + i] = -1;
      ++d_pos;
    } else {
      a.keep_idx[(int64_t)b * n_keep + k_pos] = i;
      a.slot_of[(int64_t)b * N + i] = k_pos;
      ++k_pos;
    }
  }
}

void launch_score(const ficoco_problem& p, const Plan& pl, char* ws, double* scores, hipStream_t s) {
  ScoreArgs a{};
  a.N = p.N; a.H = p.H; a.M = p.M; a.n_chunks = pl.n_chunks; a.dtype = p.dtype;
  a.red_src = p.red_src; a.sem_src = p.sem_src;
  a.recv_part = (const double*)(ws + pl.recv_part);
  a.cls = (const double*)(ws + pl.cls);
  a.ttext = (const double*)(ws + pl.ttext);
  a.recv_vec = p.recv_vec; a.sem_vec = p.sem_vec;
  a.fterm_r = (const double*)(ws + pl.fterm);
  a.fterm_g = (const double*)(ws + pl.fterm2);
  a.w = (double)p.w_score;
  const bool penalty = p.variant == FICOCO_VARIANT_V && p.window > 0;
  a.pos = p.pos;
  a.grid_g = p.grid_g; a.grid_h = p.grid_h; a.grid_w = p.grid_w;
  a.window = penalty ? p.window : 0;
  a.coef = (double)p.penalty_coef;
  a.scores = scores;
  const size_t cells = penalty ? (size_t)p.grid_g * p.grid_h * p.grid_w : 0;
  const size_t lds = (size_t)p.N * sizeof(double) + cells * sizeof(int);
  if (lds > 32768)
    (void)hipFuncSetAttribute((const void*)score_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  hipLaunchKernelGGL(score_kernel, dim3(p.B), dim3(kSelectThreads), lds, s, a);
}

void launch_filter(const ficoco_problem& p, const Plan& pl, char* ws, const double* scores,
                   int32_t* discard_idx, int32_t* keep_idx, hipStream_t s) {
  FilterArgs a{};
  a.N = p.N; a.n_disc = pl.n_disc;
  a.scores = scores; a.discard_idx = discard_idx; a.keep_idx = keep_idx;
  a.slot_of = (int32_t*)(ws + pl.slot_of);
  const size_t lds = (size_t)p.N * sizeof(double) + 2 * kSelectThreads * sizeof(int);
  if (lds > 32768)
    (void)hipFuncSetAttribute((const void*)filter_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  hipLaunchKernelGGL(filter_kernel, dim3(p.B), dim3(kSelectThreads), lds, s, a);
}

}  // namespace ficoco
