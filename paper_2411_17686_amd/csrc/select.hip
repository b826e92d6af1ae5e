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
#include "feature_rows.hpp"
#include "text_stats.hpp"

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
  int32_t* share_cnt;       // [B][share_n] edge counters of the correlate stage, zeroed here (fused step with inverted edge lists), or null
  int share_n;
  int32_t* pos_out;         // [B][n_keep] position ids of the preserved tokens (fused step: written here, beside keep_idx), or null
  // Exact re-evaluation of the cosine-derived terms for tokens whose decision is within the error
  // bound of the bulk evaluation (exact_r: the mean-cosine term, exact_g: the equivalent-token term)
  int exact_r, exact_g;
  const void* F;            // features [B][N][Df]
  int64_t fsb, fsn;         // strides in elements
  int Df;
  const double* norm;       // [B][N] row norms of the bulk pass
  const double* mu_parts;   // [B][mu_n_parts] parts of the squared norm of the bulk pass's mean feature row
  int mu_n_parts;
  double* fterm_r_w;        // the term buffers again, writable (exact values replace bulk ones)
  double* fterm_g_w;
  double* ex_nrm;           // [B][N]       row norms, squares added in feature order
  double* ex_mu;            // [B][Df + 1]  mean feature row, tokens added in order; then its norm
  double* ex_u;             // [B][kExactGroup][Df] unit rows of the tokens being re-evaluated
  double* ex_g;             // [B][kExactGroup][N]  their cosines with every token
  int32_t* ex_list;         // [B][N] tokens to re-evaluate in this pass
  // Side work (SIDE_KB > 0): the workgroups behind the first B take the row norms and unit rows of
  // the feature stage along, `side_chunks` workgroups per image with one wavefront per row.
  FeatArgs side;
  int B, side_chunks;
};

constexpr int kExactGroup = 8;    // tokens whose mean cosine is re-evaluated together

// head mean of a pre-reduced per-head vector entry: 16 independent loads at a time, added in
// head order
template <typename T>
__device__ __forceinline__ double vec_head_sum(const T* p, int H, int N) {
  double acc = 0.0;
  for (int h = 0; h < H; h += 16) {       // past the last head the last one is loaded again and counted as zero
    T v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) v[u] = p[(int64_t)min(h + u, H - 1) * N];
    issue_fence();
#pragma unroll
    for (int u = 0; u < 16; ++u) acc += h + u < H ? widen(v[u]) : 0.0;
  }
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

// x / d for 0 <= x < 2^14 and 1 <= d, given rd = 1.0f / (float)d: the float product is within
// 2^-9 of the quotient, so its integer part is off by at most one, which the remainder shows.
// (Token, cell and window counts are at most 12288; an integer division costs five times as many
// instructions, and the one workgroup of an image pays for every instruction of every token.)
static_assert(kMaxSelectN <= (1 << 14), "div_small's range");
__device__ __forceinline__ int div_small(int x, int d, float rd) {
  int q = (int)((float)x * rd);
  const int r = x - q * d;
  if (r < 0) --q; else if (r >= d) ++q;
  return q;
}

__device__ __forceinline__ uint64_t score_key(double s) {
  const uint64_t u = (uint64_t)__double_as_longlong(s + 0.0);   // -0 folded into +0
  return (u >> 63) ? ~u : (u | 0x8000000000000000ULL);
}

constexpr int kTokensPerThread = (kMaxSelectN + kSelectThreads - 1) / kSelectThreads;   // sequences longer than kSelectThreads run with kSelectThreads threads
constexpr int kBinCopies = 32;      // counters per histogram bin in the spread form: one per LDS bank
constexpr int kSpreadMinN = 4096;   // tokens from which that form is used (below, clearing and folding 8192 counters costs more than the queueing: measured at 576 and 2304 tokens)
constexpr int kRegsMinN = kSpreadMinN;   // tokens from which the keys of the selection live in registers (the workgroup then has kSelectThreads threads, and the spread counters exist)

__device__ __forceinline__ double key_score(uint64_t k) {       // inverse of score_key
  const uint64_t u = (k >> 63) ? (k & 0x7fffffffffffffffULL) : ~k;
  return __longlong_as_double((long long)u);
}

// Radix select of the n_disc-th largest key (n_disc >= 1): 8 passes over the key bytes, most
// significant first.  Returns K* and how many of the tokens with key == K* belong to the n_disc
// largest (lowest indices first).  Called by every thread of the workgroup.
// OPAQUE: the thread index is taken through an opaque move, so that the addresses derived from it
// are formed here and not ahead of a loop around the call (where they would occupy registers).
template <bool OPAQUE>
__device__ __forceinline__ void radix_select_kstar(const uint64_t* keys, int N, int n_disc, int* hist, int* bcast,
                                                   int* hist_wide, uint64_t& kstar_out, int& need_out) {
  int tid = threadIdx.x;
  if constexpr (OPAQUE) asm volatile("" : "+v"(tid));
  const int nt = blockDim.x;
  uint64_t kstar = 0;
  int need = n_disc;   // how many of the current candidates (keys matching the prefix) to take from the top
  uint64_t* small = (uint64_t*)hist;   // candidate keys once at most 64 are left (after the histogram is spent)
  const bool spread = N >= kSpreadMinN;   // uniform
  // The counters are cleared once here and, in every pass, by the threads that have just read them
  // (each barrier of the one workgroup costs a good part of a microsecond at sixteen wavefronts:
  // a pass has two of them, three in the many-keys form).
  if (spread) { for (int j = tid; j < 256 * kBinCopies; j += nt) hist_wide[j] = 0; }
  else if (tid < 256) hist[tid] = 0;
  __syncthreads();
  for (int pass = 0; pass < 8; ++pass) {
    const int shift = 56 - 8 * pass;
    const uint64_t hi_mask = pass == 0 ? 0ULL : (~0ULL << (shift + 8));
    if (spread) {
      // Many keys per thread: scores of one image share their leading digits, so in the first
      // passes nearly all atomics would queue on one LDS address (one lane at a time).  Every
      // bin has 32 counters here, one per bank, lane l adding to counter l % 32 -- only lanes
      // l and l + 32 of an instruction meet -- and four threads per bin fold them afterwards.
      for (int i = tid; i < N; i += nt) {
        const uint64_t k = keys[i];
        if ((k & hi_mask) == kstar) atomicAdd(&hist_wide[(int)((k >> shift) & 255) * kBinCopies + tid % kBinCopies], 1);
      }
      __syncthreads();
      // four threads per bin (neighbouring lanes: the thread count is a multiple of 64)
      for (int j = tid; j < 4 * 256; j += nt) {
        const int bin = j / 4, part = j % 4;
        int sum = 0;
#pragma unroll
        for (int c = 0; c < kBinCopies / 4; ++c) {       // rotated by the bin so that neighbouring bins read different banks
          int* ctr = &hist_wide[bin * kBinCopies + (part * (kBinCopies / 4) + c + bin) % kBinCopies];
          sum += *ctr;
          *ctr = 0;
        }
        sum += dpp_move<0xB1>(sum);                        // lane ^ 1
        sum += dpp_move<0x4E>(sum);                        // lane ^ 2
        if (part == 0) hist[bin] = sum;
      }
    } else {
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
      if (!spread) {
#pragma unroll
        for (int k = 0; k < 4; ++k) hist[4 * tid + k] = 0;
      }
      const int lsum = h[0] + h[1] + h[2] + h[3];
      const int upto = wave_scan_inclusive(lsum);        // lanes 0 .. this one; lane 63 holds the total
      int above = lane_value(upto, kWave - 1) - upto;    // tokens in bins above this lane's
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
    // (the next write of these three words lies behind the next pass's barriers)
    kstar |= (uint64_t)bcast[0] << shift;
    need = bcast[1];
    const int left = bcast[2];
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
  kstar_out = kstar;
  need_out = need;
}

// The same selection for long sequences, with the keys in registers.  One workgroup serves an image,
// so every instruction per token costs N / 64 cycles of the one compute unit (60 ns at 9216 tokens):
// here a thread holds the keys of its own contiguous run of tokens (the run the ordered compaction
// gives it anyway) and a bit per key that says whether the key still matches the digits chosen so
// far, and a pass is a shift, a mask and an LDS add per live key -- no key is read from LDS again,
// no 64-bit prefix is compared.  Histogram as in the many-keys form above (one counter per bank).
// valid: bit u set where kreg[u] is a token.  Needs blockDim.x == kSelectThreads.
template <int PER>
__device__ __forceinline__ void radix_select_regs(const uint64_t (&kreg)[PER], uint32_t valid, int n_disc, int* hist,
                                                  int* bcast, int* hist_wide, uint64_t& kstar_out, int& need_out) {
  const int tid = threadIdx.x, nt = blockDim.x;
  uint64_t kstar = 0;
  int need = n_disc;
  uint32_t alive = valid;
  uint64_t* small = (uint64_t*)hist;
  for (int j = tid; j < 256 * kBinCopies; j += nt) hist_wide[j] = 0;
  __syncthreads();
  for (int pass = 0; pass < 8; ++pass) {
    const int shift = 56 - 8 * pass;
#pragma unroll
    for (int u = 0; u < PER; ++u)
      if ((alive >> u) & 1u) atomicAdd(&hist_wide[(int)((kreg[u] >> shift) & 255) * kBinCopies + tid % kBinCopies], 1);
    __syncthreads();
    {
      const int bin = tid / 4, part = tid % 4;           // four threads per bin
      int sum = 0;
#pragma unroll
      for (int c = 0; c < kBinCopies / 4; ++c) {         // read and cleared for the next pass
        int* ctr = &hist_wide[bin * kBinCopies + (part * (kBinCopies / 4) + c + bin) % kBinCopies];
        sum += *ctr;
        *ctr = 0;
      }
      sum += dpp_move<0xB1>(sum);
      sum += dpp_move<0x4E>(sum);
      if (part == 0) hist[bin] = sum;
    }
    __syncthreads();
    if (tid < kWave) {
      int h[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) h[k] = hist[4 * tid + k];
      const int lsum = h[0] + h[1] + h[2] + h[3];
      const int upto = wave_scan_inclusive(lsum);
      int above = lane_value(upto, kWave - 1) - upto;
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
    const int digit = bcast[0];
    kstar |= (uint64_t)digit << shift;
    need = bcast[1];
    const int left = bcast[2];
#pragma unroll
    for (int u = 0; u < PER; ++u)
      if ((int)((kreg[u] >> shift) & 255) != digit) alive &= ~(1u << u);
    if (left <= kWave && shift > 0) {
      // Few candidates left: rank them directly in one wavefront instead of more passes.
      if (tid == 0) bcast[3] = 0;
      __syncthreads();
#pragma unroll
      for (int u = 0; u < PER; ++u)
        if ((alive >> u) & 1u) { const int slot = atomicAdd(&bcast[3], 1); if (slot < kWave) small[slot] = kreg[u]; }
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
  kstar_out = kstar;
  need_out = need;
}

// ---- exact re-evaluation of the cosine-derived score terms ----------------------------------------
// The bulk feature kernels evaluate the mean-cosine term as u_i . mean(u) and the equivalent-token
// term with chunked sums: fast, and within a provable distance of the value the terms are DEFINED
// as -- every sum in index order, products and sums rounded separately (mean cosine: the cosine of
// the token with every token, features added in order, then the cosines added in token order;
// equivalent token: mu = tokens added in order / N, dot product and norms with features added in
// order).  Collinear features make exact ties in that definition (and near-ties at rounding level)
// that the bulk values do not reproduce.  So the tokens whose decision -- maximum of a penalty
// window, side of the top-K cut -- lies within the error bound are evaluated again here, operation
// for operation as defined; their values then rank exactly.  Rare on real data, slow, and bounded.
template <typename T>
__device__ __forceinline__ void exact_terms_of(const SelectArgs& a, int b_in, const int32_t* list, int n_list, bool first) {
#pragma clang fp contract(off)
  // Opaque copies of the image and thread index: nothing below can then be computed ahead of
  // this point, in the registers of the code that runs for every problem.
  int b32 = b_in, tid = threadIdx.x;
  asm volatile("" : "+s"(b32));
  asm volatile("" : "+v"(tid));
  const int64_t b = b32;
  const int nt = blockDim.x;
  const int N = a.N, Df = a.Df;
  const T* Fb = (const T*)a.F + b * a.fsb;
  double* enrm = a.ex_nrm + b * N;
  double* emu = a.ex_mu + b * (Df + 1);
  if (first) {
    for (int j = tid; j < N; j += nt) {
      const T* x = Fb + (int64_t)j * a.fsn;
      double ss = 0.0;
      for (int d = 0; d < Df; ++d) { const double v = widen(x[d]); ss = ss + v * v; }
      enrm[j] = sqrt(ss);
    }
    if (a.exact_g) {
      for (int d = tid; d < Df; d += nt) {
        double acc = 0.0;
        for (int i = 0; i < N; ++i) acc = acc + widen(Fb[(int64_t)i * a.fsn + d]);
        emu[d] = acc / (double)N;
      }
      __syncthreads();
      if (tid == 0) {
        double mm = 0.0;
        for (int d = 0; d < Df; ++d) mm = mm + emu[d] * emu[d];
        emu[Df] = sqrt(mm);
      }
    }
    __syncthreads();
  }
  if (a.exact_g) {
    const double mu_n = emu[Df];
    for (int f = tid; f < n_list; f += nt) {
      const int i = list[f];
      const T* x = Fb + (int64_t)i * a.fsn;
      double dot = 0.0;
      for (int d = 0; d < Df; ++d) dot = dot + emu[d] * widen(x[d]);
      const double ni = enrm[i];
      a.fterm_g_w[b * N + i] = (mu_n > 0.0 && ni > 0.0) ? -(dot / (mu_n * ni)) : 0.0;
    }
  }
  if (a.exact_r) {
    double* eu = a.ex_u + b * (int64_t)kExactGroup * Df;
    double* eg = a.ex_g + b * (int64_t)kExactGroup * N;
    for (int f0 = 0; f0 < n_list; f0 += kExactGroup) {
      const int nf = min(kExactGroup, n_list - f0);
      for (int q = tid; q < nf * Df; q += nt) {          // unit rows of this group's tokens
        const int f = q / Df, d = q % Df;
        const int i = list[f0 + f];
        const double ni = enrm[i];
        eu[(int64_t)f * Df + d] = ni > 0.0 ? widen(Fb[(int64_t)i * a.fsn + d]) / ni : 0.0;
      }
      __syncthreads();
      for (int q = tid; q < nf * N; q += nt) {           // cos(token f, token j), features in order
        const int f = q / N, j = q % N;
        const T* y = Fb + (int64_t)j * a.fsn;
        const double nj = enrm[j];
        const double* u = eu + (int64_t)f * Df;
        double acc = 0.0;
        for (int d = 0; d < Df; ++d) {
          const double uj = nj > 0.0 ? widen(y[d]) / nj : 0.0;
          acc = acc + u[d] * uj;
        }
        eg[(int64_t)f * N + j] = acc;
      }
      __syncthreads();
      if (tid < nf) {                                     // the token's cosines added in token order
        const double* g = eg + (int64_t)tid * N;
        double acc = 0.0;
        for (int j = 0; j < N; ++j) acc = acc + g[j];
        a.fterm_r_w[b * N + list[f0 + tid]] = acc / (double)N;
      }
      __syncthreads();
    }
  }
  __syncthreads();
}

// EXACT: the instantiation for problems with a cosine-derived score term (the re-evaluation code
// costs registers that the common instantiation does not pay).
// SIDE_KB > 0: no score term needs the features, but the correlate stage needs their unit rows.
// That work depends on nothing the filter computes and the filter is one workgroup per image, so
// it rides in the same launch on workgroups of its own (row_norm_row with SIDE_KB steps in
// flight) instead of in a kernel before this one.
template <bool EXACT, typename TF, int SIDE_KB>     // TF: storage type of the features (EXACT or SIDE_KB > 0)
__global__ __launch_bounds__(kSelectThreads) void select_kernel(SelectArgs a) {
  if constexpr (SIDE_KB > 0) {
    if ((int)blockIdx.x >= a.B) {                       // uniform per workgroup
      const int sb = (int)blockIdx.x - a.B;
      const int i = (sb % a.side_chunks) * ((int)blockDim.x / kWave) + (int)threadIdx.x / kWave;
      if (i < a.N) row_norm_row<TF, SIDE_KB>(a.side, sb / a.side_chunks, i, threadIdx.x % kWave);
      return;
    }
  }
  extern __shared__ double lds_d[];
  double* s = lds_d;                                   // [N] scores, then keys in place
  uint64_t* keys = (uint64_t*)lds_d;
  int* ibase = (int*)(lds_d + a.N);
  int* scan = ibase;                                   // [2][nt]
  int* hist = ibase + 2 * kSelectThreads;              // [256]
  int* bcast = hist + 256;                             // [8]: 0-3 radix select, 4 tokens flagged in this pass
  uint32_t* exbits = (uint32_t*)(bcast + 8);           // [(N + 31) / 32] bit i: the terms of token i are exact (or about to be)
  int* owner = bcast + 8 + (a.N + 31) / 32;            // [cells] (penalty only)
  int* hist_wide = owner;                              // [256][kBinCopies]: used when the penalty's table is no longer needed
  const int b = blockIdx.x, tid = threadIdx.x, nt = blockDim.x;
  const int N = a.N;
  const bool exact_mode = EXACT && a.do_score && (a.exact_r || a.exact_g);    // uniform
  int32_t* ex_list = a.ex_list + (int64_t)b * N;
  auto is_exact = [&](int i) { return (exbits[i >> 5] >> (i & 31)) & 1u; };
  // marks token i; true if this call was the one that marked it (it then goes on the list)
  auto mark_exact = [&](int i) { return ((atomicOr(&exbits[i >> 5], 1u << (i & 31)) >> (i & 31)) & 1u) == 0u; };

  // Distance within which the bulk value of a cosine-derived term lies from its defined value.
  // Both are double-precision evaluations of the same real number: sums of at most Df + N terms
  // whose absolute values add up to at most 1 (cosines, unit rows), so each is within
  // (Df + N + c) 2^-53 of it; 16 times that is taken.  The equivalent-token term divides by |mu|,
  // which cancellation can make small against the rows that were averaged: its bound grows by
  // (mean row norm) / |mu|, and is unbounded when |mu| vanishes (every token is then re-evaluated).
  double delta = 0.0, delta_p = 0.0;
  if (exact_mode) {
    for (int i = tid; i < (N + 31) / 32; i += nt) exbits[i] = 0u;
    const double base = 16.0 * (double)(a.Df + N + 32) * 1.1102230246251565e-16;
    double dg = 0.0;
    if (a.exact_g) {
      double* red = (double*)scan;                     // the scan scratch is free here
      double part = 0.0;
      for (int i = tid; i < N; i += nt) part += a.norm[(int64_t)b * N + i];
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off, kWave);
      if (tid % kWave == 0) red[tid / kWave] = part;
      __syncthreads();
      if (tid == 0) {
        double tot = 0.0;
        for (int t = 0; t < nt / kWave; ++t) tot += red[t];
        double mm = 0.0;
        for (int k = 0; k < a.mu_n_parts; ++k) mm += a.mu_parts[(int64_t)b * a.mu_n_parts + k];
        const double mu_n = sqrt(mm), mean_nrm = tot / (double)N;
        double kappa = mu_n > 0.0 ? mean_nrm / mu_n : __builtin_huge_val();
        if (!(kappa < 1e8)) kappa = __builtin_huge_val();
        if (kappa < 1.0) kappa = 1.0;
        red[kSelectThreads / kWave] = kappa;
      }
      __syncthreads();
      dg = base * red[kSelectThreads / kWave];
      __syncthreads();
    }
    const double wr = a.w < 0.0 ? -a.w : a.w, wg = 1.0 - a.w < 0.0 ? a.w - 1.0 : 1.0 - a.w;
    delta = (a.exact_r ? wr * base : 0.0) + (a.exact_g ? wg * dg : 0.0);
    const double ac = a.coef < 0.0 ? -a.coef : a.coef;
    delta_p = a.window > 0 && ac > 1.0 ? ac * delta : delta;
  }

  uint64_t kstar = 0;
  int need = a.n_disc;      // how many tokens with key == kstar are discarded (lowest indices first)
  bool keys_ready = false;  // uniform
  if (a.do_score) {
    for (int pass = 0;; ++pass) {
      // Image and thread index go through an opaque move once per pass: the addresses below would
      // otherwise count as invariant across passes and be kept in registers around the whole
      // loop (dozens of them), which pushed the exact instantiation into scratch memory.
      int bq = b, tq = tid;
      if constexpr (EXACT) { asm volatile("" : "+s"(bq)); asm volatile("" : "+v"(tq)); }
      if (exact_mode) {
        if (tq == 0) bcast[4] = 0;
        __syncthreads();
      }
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
          const int i = min(tq + u * nt, N - 1);          // clamped: always a valid address
          r[u] = r_one[(int64_t)bq * N + i];
          g[u] = g_one[(int64_t)bq * N + i];
        }
        issue_fence();
#pragma unroll
        for (int u = 0; u < kTokensPerThread; ++u) {
          const int i = tq + u * nt;
          if (i < N) s[i] = combine_terms(a.w, a.red_src == FICOCO_R_ATTN_RECV ? (0.0 + r[u]) / (double)N : r[u], g[u]);
        }
      }
      for (int i = tq; i < (one_each ? 0 : N); i += nt) {
        double R, G;
        // the [CLS] term's load goes out first and is in flight together with the partials below
        const double g_cls = a.sem_src == FICOCO_G_CLS_ATTN ? a.cls[(int64_t)bq * N + i] : 0.0;
        if (a.red_src == FICOCO_R_ATTN_RECV) {
          // Column partials of the row chunks, added in chunk order.  32 loads are issued together
          // (one trip to memory per 32 chunks): past the last chunk the last one is loaded again and
          // counted as zero, so that the batch stays straight-line code.
          const double* p = a.recv_part + (int64_t)bq * a.n_chunks * N + i;
          double acc = 0.0;
          for (int c = 0; c < a.n_chunks; c += 32) {
            double v[32];
#pragma unroll
            for (int u = 0; u < 32; ++u) v[u] = p[(int64_t)min(c + u, a.n_chunks - 1) * N];
            issue_fence();
#pragma unroll
            for (int u = 0; u < 32; ++u) acc += c + u < a.n_chunks ? v[u] : 0.0;
          }
          R = acc / (double)N;
        } else if (a.red_src == FICOCO_R_VECTOR) {
          R = vec_head_mean(a.recv_vec, a.dtype, bq, a.H, N, i);
        } else {
          R = a.fterm_r[(int64_t)bq * N + i];
        }
        if (a.sem_src == FICOCO_G_CLS_ATTN) {
          G = g_cls;
        } else if (a.sem_src == FICOCO_G_TEXT_ATTN) {
          const double* p = a.ttext + ((int64_t)bq * N + i) * a.M;
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
          G = vec_head_mean(a.sem_vec, a.dtype, bq, a.H, N, i);
        } else {
          G = a.fterm_g[(int64_t)bq * N + i];
        }
        s[i] = combine_terms(a.w, R, G);
      }
      if (a.window > 0) {
        const int cells = a.grid_g * a.grid_h * a.grid_w;
        // Without position ids token i sits in cell i: no table of the cells' tokens is needed then.
        const bool table = a.pos != nullptr;     // uniform
        if (table) {
          for (int c = tq; c < cells; c += nt) owner[c] = -1;
          __syncthreads();
          for (int i = tq; i < N; i += nt) {
            const int c = a.pos[(int64_t)bq * N + i];
            if (c >= 0 && c < cells) owner[c] = i;
          }
        }
        __syncthreads();
        auto token_in = [&](int cell) { return table ? owner[cell] : (cell < N ? cell : -1); };
        const int W = a.window;
        const int wr = (a.grid_h + W - 1) / W, wc = (a.grid_w + W - 1) / W;
        const int n_win = a.grid_g * wr * wc;
        const float r_sub = 1.0f / (float)(wr * wc), r_wc = 1.0f / (float)wc;
        for (int w = tq; w < n_win; w += nt) {
          const int sub = div_small(w, wr * wc, r_sub), rem = w - sub * (wr * wc);
          const int wrow = div_small(rem, wc, r_wc);
          const int r0 = wrow * W, c0 = (rem - wrow * wc) * W;
          int best = -1;
          double best_s = 0.0;
          for (int r = r0; r < min(r0 + W, a.grid_h); ++r)
            for (int c = c0; c < min(c0 + W, a.grid_w); ++c) {
              const int t = token_in((sub * a.grid_h + r) * a.grid_w + c);
              if (t >= 0 && (best < 0 || s[t] > best_s)) { best = t; best_s = s[t]; }
            }
          if (exact_mode && best >= 0) {
            // Which token is the maximum is uncertain while another one is within the two tokens'
            // error bounds of it: all of those are evaluated exactly (a token that already is has
            // no error).  The flags of a window's tokens are touched by this thread alone.
            const double d_best = is_exact(best) ? 0.0 : delta;
            bool any = false;
            for (int r = r0; r < min(r0 + W, a.grid_h); ++r)
              for (int c = c0; c < min(c0 + W, a.grid_w); ++c) {
                const int t = token_in((sub * a.grid_h + r) * a.grid_w + c);
                if (t < 0 || t == best) continue;
                const double d_t = is_exact(t) ? 0.0 : delta;
                if (d_t + d_best > 0.0 && s[t] >= best_s - (d_t + d_best)) {
                  any = true;
                  if (mark_exact(t)) ex_list[atomicAdd(&bcast[4], 1)] = t;
                }
              }
            if (any && mark_exact(best)) ex_list[atomicAdd(&bcast[4], 1)] = best;
          }
          if (best >= 0) s[best] = a.coef * best_s;   // windows are disjoint: no other reader
        }
      }
      __syncthreads();
      for (int i = tq; i < N; i += nt) a.scores[(int64_t)bq * N + i] = s[i];
      if (!exact_mode) break;
      // the side of the top-K cut: tokens within the bound of the N^S-th largest score
      __syncthreads();
      for (int i = tq; i < N; i += nt) keys[i] = score_key(s[i]);   // in place: same 8-byte slots
      __syncthreads();
      if (a.n_disc > 0) {
        radix_select_kstar<EXACT>(keys, N, a.n_disc, hist, bcast, hist_wide, kstar, need);
        if (a.n_disc < N) {          // with every token discarded there is no cut to be on a side of
          // Tokens more than twice the bound above the N^S-th largest score are discarded whatever
          // the exact values are, tokens more than that below it are preserved; the others share
          // the places that are left.  Only if those places are fewer than these tokens (and more
          // than none) does it matter how they rank among themselves: then they are re-evaluated.
          const double cut = key_score(kstar);
          if (tq == 0) { bcast[5] = 0; bcast[6] = 0; }
          __syncthreads();
          int n_above = 0, n_band = 0;
          for (int i = tq; i < N; i += nt) {
            const double d = key_score(keys[i]) - cut;
            n_above += d > 2.0 * delta_p ? 1 : 0;
            n_band += (d < 0.0 ? -d : d) <= 2.0 * delta_p ? 1 : 0;
          }
          if (n_above) atomicAdd(&bcast[5], n_above);
          if (n_band) atomicAdd(&bcast[6], n_band);
          __syncthreads();
          const int places = a.n_disc - bcast[5];
          if (places > 0 && places < bcast[6]) {          // uniform
            for (int i = tq; i < N; i += nt) {
              const double d = key_score(keys[i]) - cut;
              if ((d < 0.0 ? -d : d) <= 2.0 * delta_p && mark_exact(i)) ex_list[atomicAdd(&bcast[4], 1)] = i;
            }
          }
        }
      }
      __syncthreads();
      const int n_flag = bcast[4];
      keys_ready = true;
      if (n_flag == 0 || pass == 3) break;
      if constexpr (EXACT) exact_terms_of<TF>(a, bq, ex_list, n_flag, pass == 0);
      keys_ready = false;
    }
  } else if (N > nt) {           // several tokens per thread: all loads issued before the first use
    double v[kTokensPerThread];
#pragma unroll
    for (int u = 0; u < kTokensPerThread; ++u) v[u] = a.scores[(int64_t)b * N + min(tid + u * nt, N - 1)];
    issue_fence();
#pragma unroll
    for (int u = 0; u < kTokensPerThread; ++u)
      if (tid + u * nt < N) s[tid + u * nt] = v[u];
  } else {
    for (int i = tid; i < N; i += nt) s[i] = a.scores[(int64_t)b * N + i];
  }
  if (!a.do_filter) return;
  if (a.overflow && tid == 0) a.overflow[b] = 0;
  if (a.share_cnt)
    for (int j = tid; j < a.share_n; j += nt) a.share_cnt[(int64_t)b * a.share_n + j] = 0;
  // ---- K*, flags and ordered compaction --------------------------------------------------------
  // Thread t owns the contiguous run [lo, hi) of tokens (at most kTokensPerThread of them).
  const int per = (N + nt - 1) / nt;
  const int lo = min(tid * per, N), hi = min(lo + per, N);
  uint32_t eq_mask = 0, gt_mask = 0;    // bit u: the key of token lo + u is equal to / above K*
  bool in_regs = false;                 // uniform: long sequence, keys not formed yet -> they live in registers
  if constexpr (!EXACT) in_regs = !keys_ready && N >= kRegsMinN;
  if (in_regs) {
    if constexpr (!EXACT) {
      __syncthreads();                  // the scores in LDS are final
      uint64_t kreg[kTokensPerThread];
#pragma unroll
      for (int u = 0; u < kTokensPerThread; ++u) kreg[u] = lo + u < hi ? score_key(s[lo + u]) : 0ULL;
      const uint32_t valid = (1u << (hi - lo)) - 1u;
      if (a.n_disc > 0) {
        radix_select_regs<kTokensPerThread>(kreg, valid, a.n_disc, hist, bcast, hist_wide, kstar, need);
#pragma unroll
        for (int u = 0; u < kTokensPerThread; ++u) {
          eq_mask |= kreg[u] == kstar ? 1u << u : 0u;
          gt_mask |= kreg[u] > kstar ? 1u << u : 0u;
        }
        eq_mask &= valid;
        gt_mask &= valid;
      }
    }
  } else {
    if (!keys_ready) {
      __syncthreads();
      for (int i = tid; i < N; i += nt) keys[i] = score_key(s[i]);   // in place: same 8-byte slots
      __syncthreads();
      if (a.n_disc > 0) radix_select_kstar<EXACT>(keys, N, a.n_disc, hist, bcast, hist_wide, kstar, need);
    }
    for (int i = lo; i < hi; ++i) {
      const uint64_t k = keys[i];
      eq_mask |= (a.n_disc > 0 && k == kstar) ? 1u << (i - lo) : 0u;
      gt_mask |= (a.n_disc > 0 && k > kstar) ? 1u << (i - lo) : 0u;
    }
  }
  // need = how many tokens with key == K* are discarded (lowest indices first).
  // One scan carries both counts of this thread's tokens: keys above K* (upper half) and keys
  // equal to K* (lower half); neither total exceeds N <= 12288.  The discarded tokens before
  // `lo` are then the ones above K* plus the first `need` of the equal ones.
  const int n_eq = __popc(eq_mask), n_gt = __popc(gt_mask);
  int tot;
  const int packed = block_scan_inclusive((n_gt << 16) | n_eq, scan, &tot) - ((n_gt << 16) | n_eq);
  int eq_before = packed & 0xffff;
  const int gt_before = packed >> 16;
  int d_pos = gt_before + min(eq_before, need);                   // discarded tokens before `lo`
  int k_pos = lo - d_pos;                                         // preserved tokens before `lo`
  uint32_t dis_mask = gt_mask;
  for (int u = 0; u < hi - lo; ++u) {
    if ((eq_mask >> u) & 1u) {
      if (eq_before < need) dis_mask |= 1u << u;
      ++eq_before;
    }
  }
  const int n_keep = N - a.n_disc;
  for (int i = lo; i < hi; ++i) {
    if (dis_mask & (1u << (i - lo))) {
      if (d_pos < a.n_disc) a.discard_idx[(int64_t)b * a.n_disc + d_pos] = i;
      a.slot_of[(int64_t)b * N + i] = -1;
      ++d_pos;
    } else {
      if (k_pos < n_keep) {
        a.keep_idx[(int64_t)b * n_keep + k_pos] = i;
        if (a.pos_out) a.pos_out[(int64_t)b * n_keep + k_pos] = a.pos ? a.pos[(int64_t)b * N + i] : i;
      }
      a.slot_of[(int64_t)b * N + i] = k_pos;
      ++k_pos;
    }
  }
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
  // 16 loads issued together; past the last chunk the last one is loaded again and counted as zero,
  // so that the tail is one more trip to memory and not one per chunk
  double acc = 0.0;
  for (int c = 0; c < n_chunks; c += 16) {
    double v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) v[u] = p[(int64_t)min(c + u, n_chunks - 1) * N];
    issue_fence();
#pragma unroll
    for (int u = 0; u < 16; ++u) acc += c + u < n_chunks ? v[u] : 0.0;
  }
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

// Both terms per-head vectors and the tokens in grid order (no position ids): nothing of the score
// stage then needs a step across the image -- head means, Eq. 1 and the local penalty concern the
// tokens of one window -- so a grid of workgroups forms the FINAL scores, one thread per penalty
// window (same arithmetic and the same order inside a window as select_kernel), and the per-image
// workgroup, where every instruction per token costs N / 64 cycles, only filters.  penalize == 0:
// no penalty; the caller then passes windows of one cell.
__global__ __launch_bounds__(256) void vector_scores_kernel(const void* recv_vec, const void* sem_vec, int dtype, int H,
                                                            int N, double w, int grid_g, int grid_h, int grid_w, int W,
                                                            int penalize, double coef, double* __restrict__ scores) {
  const int win = blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t b = blockIdx.y;
  const int wr = (grid_h + W - 1) / W, wc = (grid_w + W - 1) / W;
  if (win >= grid_g * wr * wc) return;
  const int sub = win / (wr * wc), rem = win % (wr * wc);
  const int r0 = (rem / wc) * W, c0 = (rem % wc) * W;
  int best = -1;
  double best_s = 0.0;
  for (int r = r0; r < min(r0 + W, grid_h); ++r)
    for (int c = c0; c < min(c0 + W, grid_w); ++c) {
      const int t = (sub * grid_h + r) * grid_w + c;       // token = cell
      if (t >= N) continue;
      const double R = vec_head_mean(recv_vec, dtype, b, H, N, t);
      const double G = vec_head_mean(sem_vec, dtype, b, H, N, t);
      const double st = combine_terms(w, R, G);
      scores[b * N + t] = st;
      if (best < 0 || st > best_s) { best = t; best_s = st; }
    }
  if (penalize && best >= 0) scores[b * N + best] = coef * best_s;
}

// The same with one thread per CELL (windows of at most 256 cells; a workgroup takes `wpb` whole
// windows, thread k of a window its k-th cell in row-major order): the head means of a window's
// tokens are then loaded side by side instead of one token after the other.  The window's first
// thread picks the maximum, scanning the cells in the same order as above.
__global__ __launch_bounds__(256) void vector_scores_cells_kernel(const void* recv_vec, const void* sem_vec, int dtype,
                                                                  int H, int N, double w, int grid_g, int grid_h,
                                                                  int grid_w, int W, int wpb, int penalize, double coef,
                                                                  double* __restrict__ scores) {
  __shared__ double sc[256];
  __shared__ int tok[256];
  __shared__ int best_of[256];
  const int64_t b = blockIdx.y;
  const int W2 = W * W;
  const int lw = threadIdx.x / W2, k = threadIdx.x % W2;
  const int wr = (grid_h + W - 1) / W, wc = (grid_w + W - 1) / W;
  const int win = blockIdx.x * wpb + lw;
  const bool active = lw < wpb && win < grid_g * wr * wc;
  int t = -1;
  if (active) {
    const int sub = win / (wr * wc), rem = win % (wr * wc);
    const int r = (rem / wc) * W + k / W, c = (rem % wc) * W + k % W;
    if (r < grid_h && c < grid_w) {
      const int cell = (sub * grid_h + r) * grid_w + c;
      if (cell < N) t = cell;
    }
  }
  double st = 0.0;
  if (t >= 0) {
    const double R = vec_head_mean(recv_vec, dtype, b, H, N, t);
    const double G = vec_head_mean(sem_vec, dtype, b, H, N, t);
    st = combine_terms(w, R, G);
  }
  sc[threadIdx.x] = st;
  tok[threadIdx.x] = t;
  __syncthreads();
  if (active && k == 0) {
    int best = -1;
    double best_s = 0.0;
    for (int j = 0; j < W2; ++j) {
      const int tj = tok[lw * W2 + j];
      const double sj = sc[lw * W2 + j];
      if (tj >= 0 && (best < 0 || sj > best_s)) { best = tj; best_s = sj; }
    }
    best_of[lw] = best;
  }
  __syncthreads();
  if (t >= 0) scores[b * N + t] = penalize && best_of[lw] == t ? coef * st : st;
}

__global__ __launch_bounds__(256) void text_stats_kernel(TextStatsArgs a) { text_stats_block(a, blockIdx.x, blockIdx.y); }

static size_t select_lds(const ficoco_problem& p, bool penalty) {
  const size_t cells = penalty ? (size_t)p.grid_g * p.grid_h * p.grid_w : 0;
  const size_t wide = p.N >= kSpreadMinN ? 256 * kBinCopies : 0;   // shares the penalty table's space
  return (size_t)p.N * sizeof(double) + (2 * kSelectThreads + 256 + 8 + (p.N + 31) / 32 + (cells > wide ? cells : wide)) * sizeof(int);
}

void fill_text_stats(const ficoco_problem& p, const Plan& pl, char* ws, TextStatsArgs& t) {
  t.ttext = (const double*)(ws + pl.ttext);
  t.N = p.N; t.M = p.M;
  t.out_g = (double*)(ws + pl.fterm2);
  t.cmax = (double*)(ws + pl.cmax);
  t.mean_blocks = (p.N + 3) / 4;
}

void launch_select(const ficoco_problem& p, const Plan& pl, char* ws, double* scores, bool do_score,
                   bool do_filter, int32_t* discard_idx, int32_t* keep_idx, int32_t* overflow,
                   hipStream_t s, bool text_stats_done, int32_t* pos_out) {
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
  const bool penalty = p.variant == FICOCO_VARIANT_V && p.window > 0;
  bool scored = false;       // the final scores are in `scores` before the kernel starts
  if (do_score && p.N > 2 * kSelectThreads && p.red_src == FICOCO_R_VECTOR && p.sem_src == FICOCO_G_VECTOR &&
      !(penalty && p.pos)) {
    const int g = penalty ? p.grid_g : 1, gh = penalty ? p.grid_h : 1, gw = penalty ? p.grid_w : p.N;
    const int W = penalty ? p.window : 1;
    const int n_win = g * ((gh + W - 1) / W) * ((gw + W - 1) / W);
    if (W <= 16) {                 // a thread per cell, 256 / W^2 whole windows per workgroup
      const int wpb = 256 / (W * W);
      hipLaunchKernelGGL(vector_scores_cells_kernel, dim3((n_win + wpb - 1) / wpb, p.B), dim3(256), 0, s, p.recv_vec,
                         p.sem_vec, (int)p.dtype, p.H, p.N, (double)p.w_score, g, gh, gw, W, wpb, penalty ? 1 : 0,
                         (double)p.penalty_coef, scores);
    } else {
      hipLaunchKernelGGL(vector_scores_kernel, dim3((n_win + 255) / 256, p.B), dim3(256), 0, s, p.recv_vec, p.sem_vec,
                         (int)p.dtype, p.H, p.N, (double)p.w_score, g, gh, gw, W, penalty ? 1 : 0,
                         (double)p.penalty_coef, scores);
    }
    scored = true;
  } else if (do_score && p.N > 2 * kSelectThreads && (p.red_src == FICOCO_R_VECTOR || p.sem_src == FICOCO_G_VECTOR)) {
    // the term buffers of the vector-sourced terms are free (the feature stage fills only the others)
    const bool vr = p.red_src == FICOCO_R_VECTOR, vg = p.sem_src == FICOCO_G_VECTOR;
    hipLaunchKernelGGL(vector_terms_kernel, dim3((p.N + 255) / 256, p.B), dim3(256), 0, s, vr ? p.recv_vec : nullptr,
                       vg ? p.sem_vec : nullptr, (int)p.dtype, p.H, p.N, (double*)(ws + pl.fterm),
                       (double*)(ws + pl.fterm2));
    if (vr) a.red_src = FICOCO_R_SIM_MEAN;     // "read the precomputed term"
    if (vg) a.sem_src = FICOCO_G_EQ_TOKEN;
  }
  if (do_score && p.sem_src == FICOCO_G_TEXT_ATTN && p.M >= 32) {
    // the equivalent-token buffer is free in FiCoCo-L; the column maxima ride along in the fused
    // step (text_stats_in_score), a staged correlate call forms them itself
    if (!text_stats_done) {
      const bool with_cmax = do_filter && text_stats_in_score(p);
      TextStatsArgs t{};
      fill_text_stats(p, pl, ws, t);
      hipLaunchKernelGGL(text_stats_kernel, dim3(text_stats_blocks(t, with_cmax), p.B), dim3(256), 0, s, t);
    }
    a.sem_src = FICOCO_G_EQ_TOKEN;             // "read the precomputed term"
  }
  if (do_score && (p.red_src == FICOCO_R_SIM_MEAN || p.sem_src == FICOCO_G_EQ_TOKEN)) {
    a.exact_r = p.red_src == FICOCO_R_SIM_MEAN;
    a.exact_g = p.sem_src == FICOCO_G_EQ_TOKEN;
    if (p.F) { a.F = p.F; a.fsb = p.f_stride_b; a.fsn = p.f_stride_n; }
    else {
      const size_t es = p.dtype == FICOCO_BF16 ? 2 : 4;
      a.F = (const char*)p.X + (size_t)p.vis_begin * p.x_stride_n * es;
      a.fsb = p.x_stride_b; a.fsn = p.x_stride_n;
    }
    a.Df = pl.Df;
    a.norm = (const double*)(ws + pl.inv_norm);
    a.mu_n_parts = (pl.Df + 255) / 256;
    a.mu_parts = (const double*)(ws + pl.colmean) + 2 * (size_t)p.B * pl.Df;
    a.fterm_r_w = (double*)(ws + pl.fterm);
    a.fterm_g_w = (double*)(ws + pl.fterm2);
    a.ex_nrm = (double*)(ws + pl.ex_nrm);
    a.ex_mu = (double*)(ws + pl.ex_mu);
    a.ex_u = (double*)(ws + pl.ex_u);
    a.ex_g = (double*)(ws + pl.ex_g);
    a.ex_list = (int32_t*)(ws + pl.ex_list);
  }
  a.w = (double)p.w_score;
  if (scored) a.do_score = 0;                    // the kernel reads the scores instead of forming them
  a.pos = p.pos;
  a.grid_g = p.grid_g; a.grid_h = p.grid_h; a.grid_w = p.grid_w;
  a.window = penalty ? p.window : 0;
  a.coef = (double)p.penalty_coef;
  a.scores = scores;
  a.n_disc = pl.n_disc;
  a.discard_idx = discard_idx; a.keep_idx = keep_idx;
  a.slot_of = (int32_t*)(ws + pl.slot_of);
  a.overflow = overflow;
  a.pos_out = do_filter ? pos_out : nullptr;
  if (overflow && edges_inverted(pl)) {      // a fused step: the correlate stage counts its edges per target
    a.share_cnt = (int32_t*)(ws + pl.share_cnt);
    a.share_n = invert_groups(pl) * p.n_keep;
  }
  const size_t lds = select_lds(p, penalty);
  const bool exact = a.exact_r || a.exact_g;
  // Short sequences: no more wavefronts than tokens need (every barrier of the kernel waits for
  // all of them); at least 256 threads, which the histogram walk assumes.
  const int threads = p.N >= kSelectThreads ? kSelectThreads : std::max(256, (p.N + kWave - 1) / kWave * kWave);
  const bool bf16 = p.dtype == FICOCO_BF16;
  int side_kb = 0;
  if (do_score && rows_with_filter(p, pl)) {
    fill_row_args(p, pl, ws, a.side);
    a.B = p.B;
    a.side_chunks = (p.N + threads / kWave - 1) / (threads / kWave);
    const int steps = (pl.Df / kVec + kWave - 1) / kWave;    // 16-byte vectors per lane and row
    side_kb = steps <= 2 ? 2 : (steps <= 4 || !bf16) ? 4 : 8;
  }
  const dim3 grid(p.B + (side_kb ? p.B * a.side_chunks : 0)), block(threads);
  auto go = [&](auto kern) {
    if (lds > 32768) (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipLaunchKernelGGL(kern, grid, block, lds, s, a);
  };
  if (exact) { if (bf16) go(select_kernel<true, bf16_t, 0>); else go(select_kernel<true, float, 0>); }
  else if (side_kb == 0) go(select_kernel<false, float, 0>);
  else if (bf16) {
    if (side_kb == 2) go(select_kernel<false, bf16_t, 2>);
    else if (side_kb == 4) go(select_kernel<false, bf16_t, 4>);
    else go(select_kernel<false, bf16_t, 8>);
  } else {
    if (side_kb == 2) go(select_kernel<false, float, 2>); else go(select_kernel<false, float, 4>);
  }
}

void launch_score(const ficoco_problem& p, const Plan& pl, char* ws, double* scores, hipStream_t s, bool text_stats_done) {
  launch_select(p, pl, ws, scores, true, false, nullptr, nullptr, nullptr, s, text_stats_done);
}

void launch_filter(const ficoco_problem& p, const Plan& pl, char* ws, const double* scores,
                   int32_t* discard_idx, int32_t* keep_idx, hipStream_t s) {
  launch_select(p, pl, ws, const_cast<double*>(scores), false, true, discard_idx, keep_idx, nullptr, s, false);
}

}  // namespace ficoco

