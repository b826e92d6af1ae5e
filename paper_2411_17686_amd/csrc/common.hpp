// Internal declarations shared by the kernels and the C-ABI layer of the FiCoCo library.
// gfx950 only (64-wide wavefronts).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/ficoco.h"

namespace ficoco {

constexpr int kWave = 64;
constexpr int kCandPad = 2048;     // floats of padding behind the approximate correlation block (one pass of its reader)
constexpr int kGramStage = 32;     // features per K stage of the matrix-core kernel (its K ranges are counted in stages)
constexpr int kVec = 8;            // elements per lane per load in the streaming kernels
constexpr int kSelMax = 8;         // order statistics kept in registers by the fast threshold path
constexpr int kReduceThreads = 256;
constexpr int kSelectThreads = 1024;
constexpr int kMaxSelectN = 12288; // visual tokens / grid cells the per-image select kernel holds in LDS

// Workspace layout: byte offsets from a 256-byte aligned base, 0 = absent.
struct Plan {
  int n_disc;            // N^S
  int n_out;             // n_tot - N^S
  // attention reduction
  int col_strips;        // column strips of the visual keys
  int strip_groups;      // 8-column groups per strip
  int row_lanes;         // rows processed concurrently by one workgroup
  int rows_per_wg;       // visual-block rows per workgroup
  int n_chunks;          // row chunks of the A block (partials of the received attention)
  int a_row0, a_rows;    // rows of A that carry a role (first, count)
  int a_shift;           // rows by which the first chunk is shortened so that visual row 0 starts a chunk
  int map_pitch;         // floats per row of the head-mean map (N rounded up to 64: read in whole 64-entry steps)
  // threshold selection
  int sel_m;             // order statistics needed: n_keep - floor(eps (n_keep-1))
  int sel_f;             // floor(p)
  double sel_g;          // fractional part of p
  bool dense_rows;       // sel_m > kSelMax: rows are materialised and selected bit by bit
  bool need_features;    // unit rows / norms
  size_t abar;           // float  [B][N][map_pitch]  head-mean visual x visual map, TRANSPOSED: [key token][query token]
  size_t recv_part;      // double [B][n_chunks][N]
  size_t cls;            // double [B][N]
  size_t ttext;          // double [B][N][M]      head-mean text->visual map, transposed
  size_t inv_norm;       // double [B][N]         1/|F_i| (0 for a zero row)
  size_t xhat;           // bf16   [B][N][Df]     unit rows rounded to bfloat16
  size_t colsum_part;    // double [B][f_chunks][Df]
  size_t colmean;        // double [2][B][Df] (mean unit row, mean raw row), then the parts of |mean raw row|^2
  size_t fterm;          // double [B][N]         feature-derived score term
  size_t fterm2;         // double [B][N]
  size_t slot_of;        // int32  [B][N]         keep slot of a preserved token, -1 if discarded
  size_t tgt_ptr;        // int32  [B][n_keep+1]
  size_t tgt_src;        // int32  [B][N^S*k_max] discarded token index per edge, by target
  size_t tgt_alpha;      // double [B][N^S*k_max]
  size_t hub_list, hub_cnt;   // int32 [B][n_keep], [B]: preserved tokens with long buckets (inverted lists only)
  size_t share_cnt;      // int32  [B][invert_groups][n_keep]  edges per target from each share of the discarded rows (fused step, inverted lists)
  size_t pair_tab;       // PairRec [B][N^S]     first two edges of every discarded row (fused step, lists not inverted)
  size_t rowbuf;         // double [B][N^S][n_keep] (dense_rows only)
  size_t ct;             // float  [splits][B][N^S][n_keep]  approximate cosines (matrix-core path)
  size_t cmax;           // double [B][M]
  // exact re-evaluation of the cosine-derived score terms (select stage), present with those terms only
  size_t ex_nrm;         // double [B][N]
  size_t ex_mu;          // double [B][Df + 1]
  size_t ex_u;           // double [B][8][Df]
  size_t ex_g;           // double [B][8][N]
  size_t ex_list;        // int32  [B][N]
  int fixed_k;           // >= 0: targets per discarded token fixed by the caller (0: no edges), -1: adaptive
  bool extra_token;      // the additional token of the convergent form is written
  bool qk;               // the maps are formed from queries and keys on the fly (attn_qk.hip)
  int qk_groups;         // two-sweep form: workgroups per query tile, each with a share of the heads (1: no split)
  size_t qk_part;        // float: the groups' head sums of map, text profiles, column partials, [CLS] row (qk_groups > 1)
  bool use_gram;         // cosine correlation proposed by the MFMA tile kernel
  int gram_splits, gram_st_per_split;   // K ranges of that kernel and their length in 32-feature stages
  int f_chunks, f_rows_per_wg, Df;
  size_t total;
};

int make_plan(const ficoco_problem& p, Plan& plan, const char** why);

// One edge of the correlate stage in the form the merge kernel scans: target slot, source
// visual token, weight.  16 bytes, one load.

// ---- launchers (all asynchronous on `s`) -----------------------------------------------
// text_elsewhere: the text-profile kernel is not launched here (text_with_features: it rides in the
// feature stage's launch)
void launch_attn_reduce(const ficoco_problem& p, const Plan& pl, char* ws, hipStream_t s, bool text_elsewhere = false);
void launch_attn_qk(const ficoco_problem& p, const Plan& pl, char* ws, hipStream_t s);
constexpr int kQkTile = 48;        // query rows per workgroup of the query/key form
constexpr int kQkMaxKeys = 640;    // keys it holds in registers (longer blocks: the keys in blocks of this size, two sweeps)
constexpr int kQkLongMaxHeads = 64; // heads whose softmax normalisers that form keeps in LDS
// with_text: the launch of the row-norm kernel also forms the text profiles and the launch of the
// column-sum kernel their statistics (with_cmax: the column maxima too), see text_with_features
void launch_features(const ficoco_problem& p, const Plan& pl, char* ws, hipStream_t s, bool with_text = false,
                     bool with_cmax = false);
// The feature stage is norms and unit rows only (no score term reads the features; the cosine
// correlation does): the score stage's launch of the filter kernel takes them along on workgroups
// of its own, and launch_features does nothing.
inline bool rows_with_filter(const ficoco_problem& p, const Plan& pl) {
  return pl.need_features && p.red_src != FICOCO_R_SIM_MEAN && p.sem_src != FICOCO_G_EQ_TOKEN;
}
// FiCoCo-L with 32 or more text queries: the fused step forms the column maxima of the text
// profiles in the score stage's launch (select.hip), and its correlate stage does not.
inline bool text_stats_in_score(const ficoco_problem& p) {
  return p.variant == FICOCO_VARIANT_L && p.sem_src == FICOCO_G_TEXT_ATTN && p.M >= 32;
}
// FiCoCo-L whose score reads both the features (column sums: four dependent launches) and the text
// profiles (two dependent launches): the two chains do not depend on each other, so where score
// and reduction are issued by the same call the text kernels ride in the launches of the feature
// kernels instead of standing in line before and after them.
inline bool text_with_features(const ficoco_problem& p, const Plan& pl) {
  return text_stats_in_score(p) && p.A_text != nullptr && pl.need_features && !rows_with_filter(p, pl);
}
// text_stats_done: the text statistics were formed by the feature stage's launches
void launch_score(const ficoco_problem& p, const Plan& pl, char* ws, double* scores, hipStream_t s,
                  bool text_stats_done = false);
void launch_filter(const ficoco_problem& p, const Plan& pl, char* ws, const double* scores,
                   int32_t* discard_idx, int32_t* keep_idx, hipStream_t s);
// pos_out: the filter also writes the position ids of the preserved tokens (a fused step: the
// compress stage is then called without them), or null
void launch_select(const ficoco_problem& p, const Plan& pl, char* ws, double* scores, bool do_score,
                   bool do_filter, int32_t* discard_idx, int32_t* keep_idx, int32_t* overflow,
                   hipStream_t s, bool text_stats_done = false, int32_t* pos_out = nullptr);
void launch_correlate(const ficoco_problem& p, const Plan& pl, char* ws, const int32_t* discard_idx,
                      const int32_t* keep_idx, int32_t* edge_cnt, int32_t* edge_tgt,
                      double* edge_alpha, int32_t* overflow, bool fused,
                      hipEvent_t gram_start, hipEvent_t gram_stop, hipStream_t s, int gram_repeat = 1);
void launch_gather(const ficoco_problem& p, const Plan& pl, const int32_t* keep_idx, const void* in,
                   int64_t sb, int64_t sn, int row_bytes, void* out, hipStream_t s);
void launch_corr_gap(const ficoco_problem& p, const Plan& pl, char* ws, const int32_t* discard_idx,
                     const int32_t* keep_idx, double* gap, hipStream_t s);
// targets_counted: the call follows the correlate stage of the same fused step, which counted the
// edges per target and share of rows (inverted lists) or wrote the pair records (scanning merge)
// while it wrote the lists; otherwise the compress stage works from the lists it is given alone
void launch_compress(const ficoco_problem& p, const Plan& pl, char* ws, const int32_t* discard_idx,
                     const int32_t* keep_idx, const int32_t* edge_cnt, const int32_t* edge_tgt,
                     const double* edge_alpha, void* X_out, int32_t* pos_out,
                     hipStream_t s, bool targets_counted = false);
// Above kMatchMaxRows discarded tokens the compress stage first buckets the edges by target
// (compress.hip).  The discarded rows are cut into invert_groups() shares of invert_share_rows()
// consecutive rows, one workgroup of the bucketing kernel per share.  In a fused step the filter
// stage clears a counter per (share, target) and the correlate stage adds one per edge it writes,
// so the bucketing kernel starts from the counts instead of reading every list in every workgroup.
// Up to kMatchMaxRows discarded tokens every workgroup of the merge stages the image's edges in LDS:
// count, source token and the first two (target, weight) pairs of each discarded row.  Gathered
// from the lists (rows of k_max slots) that is two or three cache lines per four rows and several
// strided loads per thread, in every workgroup; in a fused step the correlate stage therefore also
// writes those fields as one 32-byte record per row, which the merge reads with whole-line loads.
struct alignas(16) PairRec {
  int32_t cnt, src, t0, t1;
  double a0, a1;
};
static_assert(sizeof(PairRec) == 32, "two 16-byte loads per record");
constexpr int kMatchMaxRows = 1024;
constexpr int kInvertRows = 512;
inline bool pair_records(const ficoco_problem& p, const Plan& pl) {     // (lists of at most 64 entries: one wavefront holds a row's edges)
  return pl.n_disc > 0 && pl.n_disc <= kMatchMaxRows && p.k_max <= 64 && pl.fixed_k != 0;
}
inline bool edges_inverted(const Plan& pl) { return pl.n_disc > kMatchMaxRows; }
inline int invert_groups(const Plan& pl) { return (pl.n_disc + kInvertRows - 1) / kInvertRows; }
inline int invert_share_rows(const Plan& pl) {
  const int g = invert_groups(pl);
  return g > 0 ? (pl.n_disc + g - 1) / g : 1;
}

// ---- device helpers ----------------------------------------------------------------------
typedef uint16_t bf16_t;

template <typename T> struct __attribute__((packed, aligned(2))) Pack8 { T v[kVec]; };

__device__ __forceinline__ double widen(bf16_t x) {
  return (double)__uint_as_float(((uint32_t)x) << 16);
}
__device__ __forceinline__ double widen(float x) { return (double)x; }

// Raw bits of 8 consecutive elements, loaded from an address that is only element aligned
// (kept unconverted so that many loads can be in flight before the first use).
template <typename T> struct Raw8;
template <> struct Raw8<bf16_t> { uint4 a; };
template <> struct Raw8<float> { float4 a, b; };

__device__ __forceinline__ void load_raw(const bf16_t* __restrict__ p, Raw8<bf16_t>& r) {
  __builtin_memcpy(&r.a, p, 16);
}
__device__ __forceinline__ void load_raw(const float* __restrict__ p, Raw8<float>& r) {
  __builtin_memcpy(&r.a, p, 16);
  __builtin_memcpy(&r.b, p + 4, 16);
}
__device__ __forceinline__ void add_raw(const Raw8<bf16_t>& r, double (&acc)[kVec]) {
  const uint32_t w[4] = {r.a.x, r.a.y, r.a.z, r.a.w};
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    acc[2 * j] += (double)__uint_as_float(w[j] << 16);
    acc[2 * j + 1] += (double)__uint_as_float(w[j] & 0xffff0000u);
  }
}
__device__ __forceinline__ void add_raw(const Raw8<float>& r, double (&acc)[kVec]) {
  acc[0] += r.a.x; acc[1] += r.a.y; acc[2] += r.a.z; acc[3] += r.a.w;
  acc[4] += r.b.x; acc[5] += r.b.y; acc[6] += r.b.z; acc[7] += r.b.w;
}

// acc += w * (the 8 elements held raw): product and sum are rounded separately, as the plain
// statement of Eq. 2 does, so that the sums are the same doubles (a fused multiply-add differs in
// the last bit, which shows where a sum cancels)
__device__ __forceinline__ void fma_raw(const Raw8<bf16_t>& r, double w, double (&acc)[kVec]) {
#pragma clang fp contract(off)
  const uint32_t q[4] = {r.a.x, r.a.y, r.a.z, r.a.w};
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    acc[2 * j] += w * (double)__uint_as_float(q[j] << 16);
    acc[2 * j + 1] += w * (double)__uint_as_float(q[j] & 0xffff0000u);
  }
}
__device__ __forceinline__ void fma_raw(const Raw8<float>& r, double w, double (&acc)[kVec]) {
#pragma clang fp contract(off)
  acc[0] += w * r.a.x; acc[1] += w * r.a.y; acc[2] += w * r.a.z; acc[3] += w * r.a.w;
  acc[4] += w * r.b.x; acc[5] += w * r.b.y; acc[6] += w * r.b.z; acc[7] += w * r.b.w;
}

// Between the loads of a batch and their first use: the instruction scheduler moves nothing
// across this point.  Left to itself it may pull a load down to its use to save registers,
// which turns a batch of loads in flight back into one memory round trip after the other.
__device__ __forceinline__ void issue_fence() { __builtin_amdgcn_sched_barrier(0); }

// ---- reductions over the 64 lanes of a wavefront ----------------------------------------------------
// Every lane must be active and every lane gets the result.  The first four steps pair lanes inside
// a row of 16 with data-parallel-primitive moves (lane ^ 1, lane ^ 2, then the mirror images inside
// 8 and inside 16 lanes, which reach the other half because the halves are uniform by then), the
// four row results are read out by lane and combined as (r0 op r1) op (r2 op r3): a fixed tree,
// and no trip through the LDS permute path (a butterfly of six of those costs several hundred
// cycles in kernels that are chains of dependent steps).  `op` must be commutative.
template <int CTRL>
__device__ __forceinline__ int dpp_move(int x) { return __builtin_amdgcn_update_dpp(0, x, CTRL, 0xF, 0xF, false); }
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) { return __int_as_float(dpp_move<CTRL>(__float_as_int(x))); }
template <int CTRL>
__device__ __forceinline__ double dpp_move(double x) {
  return __hiloint2double(dpp_move<CTRL>(__double2hiint(x)), dpp_move<CTRL>(__double2loint(x)));
}
__device__ __forceinline__ int lane_value(int x, int l) { return __builtin_amdgcn_readlane(x, l); }
__device__ __forceinline__ float lane_value(float x, int l) { return __int_as_float(lane_value(__float_as_int(x), l)); }
__device__ __forceinline__ double lane_value(double x, int l) {
  return __hiloint2double(lane_value(__double2hiint(x), l), lane_value(__double2loint(x), l));
}
template <typename T, typename F>
__device__ __forceinline__ T wave_reduce(T v, F op) {
  v = op(v, dpp_move<0xB1>(v));      // quad_perm [1,0,3,2]: lane ^ 1
  v = op(v, dpp_move<0x4E>(v));      // quad_perm [2,3,0,1]: lane ^ 2
  v = op(v, dpp_move<0x141>(v));     // mirror inside 8 lanes
  v = op(v, dpp_move<0x140>(v));     // mirror inside 16 lanes
  return op(op(lane_value(v, 0), lane_value(v, 16)), op(lane_value(v, 32), lane_value(v, 48)));
}
// Inclusive prefix sum over the lanes of a wavefront (every lane active): four shifted adds inside
// each row of 16 (a lane whose source would lie before its row adds zero), then the totals of
// the rows before a lane's own, read out of lanes 15, 31 and 47.
template <int CTRL>
__device__ __forceinline__ int dpp_move_or_zero(int x) { return __builtin_amdgcn_update_dpp(0, x, CTRL, 0xF, 0xF, true); }
__device__ __forceinline__ int wave_scan_inclusive(int v) {
  v += dpp_move_or_zero<0x111>(v);   // row_shr:1
  v += dpp_move_or_zero<0x112>(v);   // row_shr:2
  v += dpp_move_or_zero<0x114>(v);   // row_shr:4
  v += dpp_move_or_zero<0x118>(v);   // row_shr:8
  const int r0 = lane_value(v, 15), r1 = lane_value(v, 31), r2 = lane_value(v, 47);
  const int row = (int)(threadIdx.x % kWave) / 16;
  return v + (row >= 1 ? r0 : 0) + (row >= 2 ? r1 : 0) + (row >= 3 ? r2 : 0);
}

// all bits cleared (eight zeros) unless `keep`: selects, no branch
__device__ __forceinline__ void keep_raw_if(Raw8<bf16_t>& r, bool keep) {
  r.a.x = keep ? r.a.x : 0u; r.a.y = keep ? r.a.y : 0u; r.a.z = keep ? r.a.z : 0u; r.a.w = keep ? r.a.w : 0u;
}
__device__ __forceinline__ void keep_raw_if(Raw8<float>& r, bool keep) {
  r.a.x = keep ? r.a.x : 0.0f; r.a.y = keep ? r.a.y : 0.0f; r.a.z = keep ? r.a.z : 0.0f; r.a.w = keep ? r.a.w : 0.0f;
  r.b.x = keep ? r.b.x : 0.0f; r.b.y = keep ? r.b.y : 0.0f; r.b.z = keep ? r.b.z : 0.0f; r.b.w = keep ? r.b.w : 0.0f;
}

// the 8 elements held raw, as doubles
__device__ __forceinline__ void widen_raw(const Raw8<bf16_t>& r, double (&out)[kVec]) {
  const uint32_t q[4] = {r.a.x, r.a.y, r.a.z, r.a.w};
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    out[2 * j] = (double)__uint_as_float(q[j] << 16);
    out[2 * j + 1] = (double)__uint_as_float(q[j] & 0xffff0000u);
  }
}
__device__ __forceinline__ void widen_raw(const Raw8<float>& r, double (&out)[kVec]) {
  out[0] = r.a.x; out[1] = r.a.y; out[2] = r.a.z; out[3] = r.a.w;
  out[4] = r.b.x; out[5] = r.b.y; out[6] = r.b.z; out[7] = r.b.w;
}

// 8 consecutive elements from an address that is only element aligned.
template <typename T>
__device__ __forceinline__ void load8(const T* __restrict__ p, double (&out)[kVec]);

template <>
__device__ __forceinline__ void load8<bf16_t>(const bf16_t* __restrict__ p, double (&out)[kVec]) {
  uint4 r;
  __builtin_memcpy(&r, p, 16);
  const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    out[2 * j] = (double)__uint_as_float(w[j] << 16);
    out[2 * j + 1] = (double)__uint_as_float(w[j] & 0xffff0000u);
  }
}
template <>
__device__ __forceinline__ void load8<float>(const float* __restrict__ p, double (&out)[kVec]) {
  float4 a, b;
  __builtin_memcpy(&a, p, 16);
  __builtin_memcpy(&b, p + 4, 16);
  out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w;
  out[4] = b.x; out[5] = b.y; out[6] = b.z; out[7] = b.w;
}

// Workgroups are handed to the 8 XCDs round-robin by their linear id, and every XCD has its
// own L2.  This maps the linear id to a logical id such that consecutive logical ids (the
// tiles of one image) run on the same XCD and share its L2.  Logical ids >= total are idle.
constexpr int kXcds = 8;
__device__ __forceinline__ int xcd_logical_id(int linear, int total) {
  const int per = (total + kXcds - 1) / kXcds;
  return (linear % kXcds) * per + linear / kXcds;
}
__host__ __device__ __forceinline__ int xcd_padded_total(int total) {
  return ((total + kXcds - 1) / kXcds) * kXcds;
}

// Inclusive scan of one int per thread over the workgroup (wavefront shuffles, then the
// wavefront totals through LDS); returns this thread's inclusive value, *total receives the
// sum.  scratch: at least blockDim.x / 64 ints.
__device__ __forceinline__ int block_scan_inclusive(int v, int* scratch, int* total) {
  const int tid = threadIdx.x, lane = tid % kWave, wv = tid / kWave, nw = blockDim.x / kWave;
  const int incl = wave_scan_inclusive(v);
  __syncthreads();
  if (lane == kWave - 1) scratch[wv] = incl;
  __syncthreads();
  int before = 0, tot = 0;
  for (int w = 0; w < nw; ++w) {
    const int t = scratch[w];
    before += w < wv ? t : 0;
    tot += t;
  }
  *total = tot;
  __syncthreads();
  return incl + before;
}

// Round a double to the nearest bfloat16, ties to even, straight from double (no
// intermediate float rounding).  The spacing at binary exponent e is 2^(max(e,-126)-7).
__device__ __forceinline__ bf16_t to_bf16(double x) {
  const uint64_t u = (uint64_t)__double_as_longlong(x);
  int e = (int)((u >> 52) & 0x7ff) - 1023;
  e = e < -126 ? -126 : e;
  const double r = ldexp(rint(ldexp(x, 7 - e)), e - 7);
  return (bf16_t)(__float_as_uint((float)r) >> 16);
}
__device__ __forceinline__ void store_token(bf16_t* p, double x) { *p = to_bf16(x); }
__device__ __forceinline__ void store_token(float* p, double x) { *p = (float)x; }

}  // namespace ficoco
