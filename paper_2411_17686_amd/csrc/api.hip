// C-ABI layer: argument checks, workspace plan and the stage / fused-step entry points
// declared in include/ficoco.h.  Host code only; every launch goes to the caller's stream.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>

#include "common.hpp"

// Scratch of the allocation-free entry point (ficoco_v_step_static): the workspace of a step
// lives in this file-scope device array instead of caller memory.  Every GPU the library runs
// on holds its own copy for the life of the process.  Host code never passes the array's name to
// a kernel (on the host it is a stand-in symbol, not a device address): ficoco_create asks the
// runtime for the array's address on the ctx's device and keeps it in g_static_ws.
constexpr size_t kStaticScratchBytes = FICOCO_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char g_static_scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static void* g_static_ws[kMaxDevices];    // per device, filled by ficoco_create (written once per device with the same value)

struct ficoco_ctx {
  int device;
  hipEvent_t probe_start, probe_stop;   // measurement hook, both null when off
  int probe_kernel;
  char err[512];
};

namespace ficoco {

// With the head-mean map to store, a reduction workgroup has at most 8 row lanes and chunks of a
// multiple of 8 rows (measured at the 576-token batched shape: 8 lanes x 32 rows, ~900 workgroups,
// gives the best pipelined step; 10 lanes x 24 rows is 10 % slower alone).
constexpr int kMapRowLanes = 8;
constexpr int kMapRowsAlign = 8;
// Workgroups the reduction aims at (half of it where the map tile is turned).  Measured: 1024 against
// 2048 changes nothing at the batched ViT shapes and gives the decoder shape (8 sequences, 32 heads)
// 32-row chunks instead of 16-row ones, 42.5 against 44.0 us.
constexpr int64_t kWgTarget = 1024;

static size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

int make_plan(const ficoco_problem& p, Plan& pl, const char** why) {
  static const char* kNone = "";
  *why = kNone;
  std::memset(&pl, 0, sizeof(pl));
#define REQUIRE(c, msg) do { if (!(c)) { *why = msg; return FICOCO_EINVAL; } } while (0)
  REQUIRE(p.variant == FICOCO_VARIANT_V || p.variant == FICOCO_VARIANT_L, "variant must be V or L");
  REQUIRE(p.dtype == FICOCO_F32 || p.dtype == FICOCO_BF16, "dtype must be F32 or BF16");
  REQUIRE(p.B >= 1 && p.D >= 1 && p.n_tot >= 1, "B, D, n_tot must be positive");
  REQUIRE(p.N >= 1 && p.vis_begin >= 0 && p.vis_begin + (int64_t)p.N <= p.n_tot,
          "visual span [vis_begin, vis_begin+N) must lie inside the sequence");
  REQUIRE(p.n_keep >= 0 && p.n_keep <= p.N, "n_keep must be in [0, N]");
  REQUIRE(p.n_keep >= 1 || p.N == 0, "n_keep must be >= 1 (nothing to recycle into)");
  REQUIRE(p.N <= kMaxSelectN, "N exceeds the per-image limit of the filter kernel (12288)");
  REQUIRE(p.X != nullptr, "X is NULL");
  REQUIRE(p.x_stride_n >= p.D && p.x_stride_b >= 0, "bad X strides");
  REQUIRE(p.eps >= 0.0f && p.eps <= 1.0f, "eps must be in [0, 1]");
  REQUIRE(p.k_max >= 1, "k_max must be >= 1");
  REQUIRE(p.k_max <= kMaxSelectN, "k_max exceeds 12288 (N^S * k_max is indexed with 32-bit integers)");
  REQUIRE(p.k_mode >= FICOCO_K_ADAPTIVE && p.k_mode <= FICOCO_K_CONVERGENT, "unknown k_mode");
  REQUIRE(p.compress_mode == FICOCO_COMPRESS_SELF || p.compress_mode == FICOCO_COMPRESS_AVERAGE,
          "unknown compress_mode");
  if (p.k_mode == FICOCO_K_FIXED)
    REQUIRE(p.fixed_k >= 0 && p.fixed_k <= p.k_max, "fixed_k must be in [0, k_max]");
  REQUIRE(p.red_src >= 0 && p.red_src <= 2 && p.sem_src >= 0 && p.sem_src <= 3 &&
              p.corr_src >= 0 && p.corr_src <= 1, "unknown source selector");
  const bool L = p.variant == FICOCO_VARIANT_L;
  const bool need_A = p.red_src == FICOCO_R_ATTN_RECV || p.sem_src == FICOCO_G_CLS_ATTN ||
                      p.corr_src == FICOCO_C_ATTN;
  // queries and keys in place of the maps: FiCoCo-V with an attention-derived term and no A;
  // FiCoCo-L with neither A nor A_text (the decoder's causal maps; the M text tokens follow the visual span)
  const bool qk = p.A == nullptr && p.Q != nullptr && p.K != nullptr && (L ? p.A_text == nullptr : need_A);
  if (qk) {
    REQUIRE(p.H >= 1 && p.qk_n >= 1 && p.qk_stride_n >= p.d_head && p.qk_stride_h >= 0 && p.qk_stride_b >= 0,
            "bad Q / K shape or strides");
    REQUIRE(p.qk_begin >= 0 && p.qk_begin <= p.vis_begin && p.vis_begin + p.N <= p.qk_begin + p.qk_n,
            "Q / K do not cover the visual tokens");
    if (L)
      REQUIRE(p.M >= 1 && p.vis_begin + p.N + (int64_t)p.M <= p.qk_begin + (int64_t)p.qk_n,
              "Q / K do not cover the M text tokens behind the visual span");
    if (p.sem_src == FICOCO_G_CLS_ATTN)
      REQUIRE(p.cls_index >= p.qk_begin && p.cls_index < p.qk_begin + p.qk_n &&
                  (p.cls_index < p.vis_begin || p.cls_index >= p.vis_begin + p.N),
              "cls_index must be a row of Q / K outside the visual span");
    REQUIRE(p.qk_scale > 0.0f && p.qk_scale < 1e30f, "qk_scale must be positive and finite");
    if (p.qk_dtype != FICOCO_BF16 || !(p.d_head == 32 || p.d_head == 64 || p.d_head == 128) ||
        ((L || p.qk_n > kQkMaxKeys) && p.H > kQkLongMaxHeads) || p.qk_stride_n % 8 != 0 || p.qk_stride_h % 8 != 0 ||
        p.qk_stride_b % 8 != 0 || ((uintptr_t)p.Q & 15) || ((uintptr_t)p.K & 15)) {
      *why = "queries / keys: bfloat16, 16-byte aligned rows and d_head in {32,64,128} are supported (beyond 640 rows and for FiCoCo-L: at most 64 heads)";
      return FICOCO_EUNSUPPORTED;
    }
  } else if (need_A) {
    REQUIRE(p.A != nullptr, "A is NULL but an attention-derived term is selected");
    REQUIRE(p.H >= 1, "H must be positive");
    REQUIRE(p.a_nq >= 1 && p.a_nk >= 1 && p.a_stride_q >= p.a_nk, "bad A shape / strides");
    REQUIRE(p.a_k_begin <= p.vis_begin && p.vis_begin + p.N <= p.a_k_begin + p.a_nk,
            "A does not cover the visual keys");
    if (p.red_src == FICOCO_R_ATTN_RECV || p.corr_src == FICOCO_C_ATTN)
      REQUIRE(p.a_q_begin <= p.vis_begin && p.vis_begin + p.N <= p.a_q_begin + p.a_nq,
              "A does not cover the visual queries");
    if (p.sem_src == FICOCO_G_CLS_ATTN)
      REQUIRE(p.cls_index >= p.a_q_begin && p.cls_index < p.a_q_begin + p.a_nq &&
                  (p.cls_index < p.vis_begin || p.cls_index >= p.vis_begin + p.N),
              "cls_index must be a query row of A outside the visual span");
  }
  if (L) {
    REQUIRE(p.sem_src == FICOCO_G_TEXT_ATTN, "FiCoCo-L uses the text-attention term (Eq. 3)");
    REQUIRE((qk || p.A_text != nullptr) && p.M >= 1 && p.H >= 1, "A_text / M missing for FiCoCo-L");
    REQUIRE(p.gamma >= 0.0f && p.gamma <= 1.0f, "gamma (Eq. 4) must be in [0, 1]");
    if (!qk)
      REQUIRE(p.at_stride_q >= p.at_nk && p.at_k_begin <= p.vis_begin &&
                  p.vis_begin + p.N <= p.at_k_begin + p.at_nk, "A_text does not cover the visual keys");
  } else {
    REQUIRE(p.sem_src != FICOCO_G_TEXT_ATTN, "the text-attention term belongs to FiCoCo-L");
  }
  if (p.red_src == FICOCO_R_VECTOR) REQUIRE(p.recv_vec != nullptr && p.H >= 1, "recv_vec is NULL");
  if (p.sem_src == FICOCO_G_VECTOR) REQUIRE(p.sem_vec != nullptr && p.H >= 1, "sem_vec is NULL");
  const bool penalty = !L && p.window > 0;
  if (penalty) {
    REQUIRE(p.grid_g >= 1 && p.grid_h >= 1 && p.grid_w >= 1, "grid dimensions must be positive");
    const int64_t cells = (int64_t)p.grid_g * p.grid_h * p.grid_w;
    REQUIRE(cells >= p.N && cells <= kMaxSelectN, "grid must have between N and 12288 cells");
    REQUIRE(p.pos != nullptr || cells == p.N, "pos is NULL but the grid has more cells than tokens");
  }
  pl.need_features = p.red_src == FICOCO_R_SIM_MEAN || p.sem_src == FICOCO_G_EQ_TOKEN ||
                     p.corr_src == FICOCO_C_COSINE;
  pl.Df = p.F ? p.Df : p.D;
  if (pl.need_features && p.F)
    REQUIRE(p.Df >= 1 && p.f_stride_n >= p.Df, "bad F shape / strides");
#undef REQUIRE

  pl.n_disc = p.N - p.n_keep;
  pl.extra_token = p.k_mode == FICOCO_K_CONVERGENT && pl.n_disc > 0;
  pl.n_out = p.n_tot - pl.n_disc + (pl.extra_token ? 1 : 0);
  // targets per discarded token fixed by the caller (ablation): 0 = no edges at all
  pl.fixed_k = p.k_mode == FICOCO_K_FIXED ? std::min(p.fixed_k, p.n_keep) : -1;
  if (p.k_mode == FICOCO_K_CONVERGENT) pl.fixed_k = 0;

  // attention reduction geometry
  // Column strips.  Up to 1024 key columns a strip has at most 24 8-column groups: a workgroup
  // is then (row lanes) x (groups of the strip) with several row lanes, covers many query rows
  // and leaves few per-chunk column partials behind (measured: 3 strips of 24 groups beat 1 strip
  // of 72 at 576 columns by 4 %).  Wider maps without a head-mean map to store take wide strips
  // (their partials are a small share of the traffic).  From there the fewest strips that keep at
  // least 80 % of the threads busy, else the busiest of the next 8 choices.
  const int groups = (p.N + kVec - 1) / kVec;
  // (with the head-mean map to store, strips stay narrow at any width: the workgroup turns its
  // tile of the map in LDS, strip columns x chunk rows)
  const bool map_tile = p.corr_src == FICOCO_C_ATTN;
  {
    const int max_groups = groups <= 128 ? 24 : (map_tile ? 32 : kReduceThreads);
    const int s_min = std::max((groups + kReduceThreads - 1) / kReduceThreads, (groups + max_groups - 1) / max_groups);
    int best_busy = -1;
    for (int sN = s_min; sN < s_min + 8; ++sN) {
      const int sg = (groups + sN - 1) / sN;
      int rl = kReduceThreads / sg;
      if (map_tile) rl = std::min(rl, kMapRowLanes);
      if (rl * sg > best_busy) { best_busy = rl * sg; pl.col_strips = sN; pl.strip_groups = sg; pl.row_lanes = rl; }
      if (best_busy * 5 >= kReduceThreads * 4) break;
    }
  }
  auto rows_per_wg = [&](int rows) {
    // aim at ~kWgTarget workgroups; half as many where the map tile is turned (longer chunks make
    // whole cache lines of the transposed pieces, and a reduction that does not fill every
    // wavefront slot leaves room for the short kernels of the neighbouring streams)
    const int64_t target = map_tile ? kWgTarget / 2 : kWgTarget;
    int64_t want = ((int64_t)p.B * pl.col_strips * rows + target - 1) / target;
    if (want < 1) want = 1;
    int r = (int)((want + pl.row_lanes - 1) / pl.row_lanes) * pl.row_lanes;
    return r;
  };
  pl.qk = qk;
  if (qk) {
    // one column partial per tile of query rows: all rows of the block, or (FiCoCo-L) the visual and
    // text rows, or the text rows alone where no visual-to-visual term is needed
    const int q_rows = !L ? p.qk_n : (p.red_src == FICOCO_R_ATTN_RECV || p.corr_src == FICOCO_C_ATTN) ? p.N + p.M : p.M;
    pl.n_chunks = (q_rows + kQkTile - 1) / kQkTile;
  } else if (need_A) {
    int lo = p.vis_begin - p.a_q_begin, hi = lo + p.N;  // visual query rows
    const bool vis_rows = p.red_src == FICOCO_R_ATTN_RECV || p.corr_src == FICOCO_C_ATTN;
    if (!vis_rows) { lo = hi = p.cls_index - p.a_q_begin; ++hi; }
    if (p.sem_src == FICOCO_G_CLS_ATTN) {
      const int c = p.cls_index - p.a_q_begin;
      if (c < lo) lo = c;
      if (c + 1 > hi) hi = c + 1;
    }
    pl.a_row0 = lo;
    pl.a_rows = hi - lo;
    pl.rows_per_wg = rows_per_wg(pl.a_rows);
    pl.a_shift = 0;
    if (p.corr_src == FICOCO_C_ATTN && vis_rows) {
      // The head-mean map is stored transposed, a chunk's rows of one key column as one piece:
      // chunks of a multiple of 8 rows that start at multiples of it, counted from visual row 0,
      // make every piece whole 32-byte sectors.
      pl.rows_per_wg = std::min((pl.rows_per_wg + kMapRowsAlign - 1) / kMapRowsAlign * kMapRowsAlign, 32);    // the tile is at most 256 columns x that many rows
      const int lead = (p.vis_begin - p.a_q_begin) - lo;             // role rows before visual row 0 (the [CLS] query)
      pl.a_shift = (pl.rows_per_wg - lead % pl.rows_per_wg) % pl.rows_per_wg;
    }
    pl.n_chunks = (pl.a_rows + pl.a_shift + pl.rows_per_wg - 1) / pl.rows_per_wg;
  } else {
    pl.n_chunks = 0;
  }

  // threshold selection: p = eps (n-1) evaluated in double from the float eps
  if (p.n_keep >= 1) {
    const double q = (double)p.eps * (double)(p.n_keep - 1);
    const double f = std::floor(q);
    pl.sel_f = (int)f;
    pl.sel_g = q - f;
    pl.sel_m = p.n_keep - pl.sel_f;
    if (pl.fixed_k > 0) {      // fixed K: the threshold is the K-th largest value itself
      pl.sel_m = pl.fixed_k;
      pl.sel_f = p.n_keep - pl.fixed_k;
      pl.sel_g = 0.0;
    }
    pl.dense_rows = pl.sel_m > kSelMax;
  }

  // feature pass geometry (column sums over the tokens)
  if (pl.need_features) {
    pl.f_rows_per_wg = 64;      // two batches of 8 rows per wavefront: half the workgroups (one round on the chip) and half the partials
    pl.f_chunks = (p.N + pl.f_rows_per_wg - 1) / pl.f_rows_per_wg;
  }

  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes ? bytes : 1); return o; };
  const size_t B = p.B, N = p.N;
  pl.map_pitch = (p.N + 63) / 64 * 64;     // whole 64-entry steps: a wavefront reads a row without clamping
  pl.abar = take(p.corr_src == FICOCO_C_ATTN ? B * N * (size_t)pl.map_pitch * sizeof(float) : 0);
  pl.recv_part = take(B * (size_t)pl.n_chunks * N * sizeof(double));
  pl.cls = take(B * N * sizeof(double));
  pl.ttext = take(L ? B * N * (size_t)p.M * sizeof(double) : 0);
  pl.inv_norm = take(pl.need_features ? B * N * sizeof(double) : 0);
  pl.xhat = take(p.corr_src == FICOCO_C_COSINE ? B * N * (size_t)pl.Df * sizeof(bf16_t) : 0);
  pl.colsum_part = take(pl.need_features ? 2 * B * (size_t)pl.f_chunks * pl.Df * sizeof(double) : 0);
  pl.colmean = take(pl.need_features ? (2 * B * (size_t)pl.Df + B * (size_t)((pl.Df + 255) / 256)) * sizeof(double) : 0);   // two means, then |mu|^2 in parts
  pl.fterm = take(B * N * sizeof(double));
  pl.fterm2 = take(B * N * sizeof(double));
  pl.slot_of = take((B * N + 64) * sizeof(int32_t));    // + one 64-entry step: rows of it are read in whole steps
  pl.tgt_ptr = take(B * (size_t)(p.n_keep + 1) * sizeof(int32_t));
  pl.tgt_src = take(B * (size_t)pl.n_disc * p.k_max * sizeof(int32_t));
  pl.tgt_alpha = take(B * (size_t)pl.n_disc * p.k_max * sizeof(double));
  pl.hub_list = take(B * (size_t)p.n_keep * sizeof(int32_t));
  pl.hub_cnt = take(B * sizeof(int32_t));
  pl.share_cnt = take(edges_inverted(pl) ? B * (size_t)invert_groups(pl) * p.n_keep * sizeof(int32_t) : 0);
  pl.pair_tab = take(pair_records(p, pl) ? B * (size_t)pl.n_disc * sizeof(PairRec) : 0);
  pl.qk_groups = 1;
  if (qk && (L || p.qk_n > kQkMaxKeys)) {
    // Few query tiles (a decoder's 64 text queries are two): the heads are split over up to sixteen
    // workgroups per tile until the chip has about one workgroup per compute unit.
    const int64_t base = (int64_t)pl.n_chunks * p.B;
    const int want = (int)std::max<int64_t>(1, std::min<int64_t>(std::min(p.H, 16), 256 / std::max<int64_t>(base, 1)));
    const int per = (p.H + want - 1) / want;
    pl.qk_groups = (p.H + per - 1) / per;            // no group without heads
  }
  {
    const size_t g = pl.qk_groups > 1 ? (size_t)pl.qk_groups : 0;
    const size_t map = p.corr_src == FICOCO_C_ATTN ? B * N * (size_t)pl.map_pitch : 0;
    pl.qk_part = take(g * (map + (L ? B * N * (size_t)p.M : 0) + B * (size_t)pl.n_chunks * N + B * N) * sizeof(float));
  }
  pl.rowbuf = take(pl.dense_rows ? B * (size_t)pl.n_disc * p.n_keep * sizeof(double) : 0);
  pl.use_gram = p.corr_src == FICOCO_C_COSINE && !pl.dense_rows && pl.Df % 8 == 0 && p.k_max <= 64 &&
                pl.n_disc > 0;
  pl.gram_splits = 1;
  pl.gram_st_per_split = (pl.Df + kGramStage - 1) / kGramStage;
  if (pl.use_gram) {
    // Few output tiles: cut K so that the matrix-core kernel still fills the chip (about two
    // workgroups per compute unit), each range at least 256 features long; the partial blocks are
    // added, in a fixed order, where they are read.
    const int64_t tiles = (int64_t)p.B * ((pl.n_disc + 127) / 128) * ((p.n_keep + 127) / 128);
    int splits = (int)((512 + tiles - 1) / tiles);
    splits = std::min(splits, std::min(8, pl.Df / 256));
    if (splits < 1) splits = 1;
    const int st_all = (pl.Df + kGramStage - 1) / kGramStage;
    pl.gram_st_per_split = (st_all + splits - 1) / splits;
    pl.gram_splits = (st_all + pl.gram_st_per_split - 1) / pl.gram_st_per_split;
  }
  // + padding: the row kernel reads whole 2048-target passes
  pl.ct = take(pl.use_gram ? (pl.gram_splits * B * (size_t)pl.n_disc * p.n_keep + kCandPad) * sizeof(float) : 0);
  pl.cmax = take(L ? B * (size_t)p.M * sizeof(double) : 0);
  const bool exact_terms = p.red_src == FICOCO_R_SIM_MEAN || p.sem_src == FICOCO_G_EQ_TOKEN;
  pl.ex_nrm = take(exact_terms ? B * N * sizeof(double) : 0);
  pl.ex_mu = take(exact_terms ? B * (size_t)(pl.Df + 1) * sizeof(double) : 0);
  pl.ex_u = take(exact_terms ? B * 8 * (size_t)pl.Df * sizeof(double) : 0);
  pl.ex_g = take(exact_terms ? B * 8 * N * sizeof(double) : 0);
  pl.ex_list = take(exact_terms ? B * N * sizeof(int32_t) : 0);
  pl.total = off;
  return FICOCO_OK;
}

static int fail(ficoco_ctx* ctx, int code, const char* what, const char* detail) {
  if (ctx) std::snprintf(ctx->err, sizeof(ctx->err), "%s: %s", what, detail ? detail : "");
  return code;
}

// The calling thread's current device must be the one the ctx was created for: every launch
// goes to the current device, and the caller's pointers and stream belong to it.
static int check_device(ficoco_ctx* ctx, const char* fn) {
  int cur = -1;
  if (hipGetDevice(&cur) != hipSuccess) return fail(ctx, FICOCO_EHIP, fn, "hipGetDevice failed");
  if (cur != ctx->device) return fail(ctx, FICOCO_EINVAL, fn, "the current device is not the device this ctx was created for");
  return FICOCO_OK;
}

// Do the byte ranges [a, a + na) and [b, b + nb) overlap?
static bool ranges_overlap(const void* a, size_t na, const void* b, size_t nb) {
  const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
  return a && b && na && nb && a0 < b0 + nb && b0 < a0 + na;
}

// Bytes from X to the end of its last row, and of the dense X_out.
static size_t x_extent(const ficoco_problem& p) {
  const size_t es = p.dtype == FICOCO_BF16 ? 2 : 4;
  return ((size_t)(p.B - 1) * (size_t)p.x_stride_b + (size_t)(p.n_tot - 1) * (size_t)p.x_stride_n + (size_t)p.D) * es;
}
static size_t x_out_extent(const ficoco_problem& p, const Plan& pl) {
  return (size_t)p.B * (size_t)pl.n_out * (size_t)p.D * (p.dtype == FICOCO_BF16 ? 2 : 4);
}

static int prepare(ficoco_ctx* ctx, const ficoco_problem* p, const void* ws, size_t ws_bytes,
                   Plan& pl, const char* fn) {
  if (!ctx) return FICOCO_EINVAL;
  if (!p) return fail(ctx, FICOCO_EINVAL, fn, "problem is NULL");
  const int dev_rc = check_device(ctx, fn);
  if (dev_rc != FICOCO_OK) return dev_rc;
  const char* why;
  const int rc = make_plan(*p, pl, &why);
  if (rc != FICOCO_OK) return fail(ctx, rc, fn, why);
  if (!ws || ((uintptr_t)ws & 255)) return fail(ctx, FICOCO_EINVAL, fn, "workspace is NULL or not 256-byte aligned");
  if (ws_bytes < pl.total) return fail(ctx, FICOCO_ENOMEM, fn, "workspace smaller than ficoco_workspace_bytes()");
  return FICOCO_OK;
}

static int finish(ficoco_ctx* ctx, const char* fn) {
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(ctx, FICOCO_EHIP, fn, hipGetErrorString(e));
  return FICOCO_OK;
}

static int run_step(ficoco_ctx* ctx, const ficoco_problem* p0, int variant, void* ws, size_t ws_bytes,
                    void* X_out, int32_t* pos_out, int32_t* keep_idx, int32_t* discard_idx,
                    int32_t* edge_cnt, int32_t* edge_tgt, double* edge_alpha, double* scores,
                    int32_t* overflow, void* stream, const char* fn) {
  if (!ctx) return FICOCO_EINVAL;
  if (!p0) return fail(ctx, FICOCO_EINVAL, fn, "problem is NULL");
  if (p0->variant != variant) return fail(ctx, FICOCO_EINVAL, fn, "problem.variant does not match the entry point");
  Plan pl;
  const int rc = prepare(ctx, p0, ws, ws_bytes, pl, fn);
  if (rc != FICOCO_OK) return rc;
  if (!X_out || !keep_idx || !scores || !overflow ||
      (pl.n_disc > 0 && (!discard_idx || !edge_cnt || !edge_tgt || !edge_alpha)))
    return fail(ctx, FICOCO_EINVAL, fn, "an output pointer is NULL");
  const ficoco_problem& p = *p0;
  if (ranges_overlap(X_out, x_out_extent(p, pl), p.X, x_extent(p)))
    return fail(ctx, FICOCO_EINVAL, fn, "X_out overlaps X (outputs may not alias inputs)");
  if (ranges_overlap(X_out, x_out_extent(p, pl), ws, pl.total))
    return fail(ctx, FICOCO_EINVAL, fn, "X_out overlaps the workspace");
  hipStream_t s = (hipStream_t)stream;
  char* w = (char*)ws;
  const bool pr = ctx->probe_start && ctx->probe_kernel == FICOCO_PROBE_REDUCE;
  const bool pg = ctx->probe_start && ctx->probe_kernel == FICOCO_PROBE_GRAM;
  if (pr) (void)hipEventRecord(ctx->probe_start, s);
  const bool tw = text_with_features(p, pl);
  if (pl.qk) launch_attn_qk(p, pl, w, s); else launch_attn_reduce(p, pl, w, s, tw);
  if (pr) (void)hipEventRecord(ctx->probe_stop, s);
  if (pl.need_features) launch_features(p, pl, w, s, tw, tw);
  launch_select(p, pl, w, scores, true, true, discard_idx, keep_idx, overflow, s, tw, pos_out);
  launch_correlate(p, pl, w, discard_idx, keep_idx, edge_cnt, edge_tgt, edge_alpha, overflow, true,
                   pg ? ctx->probe_start : nullptr, pg ? ctx->probe_stop : nullptr, s);
  // (the position ids of the preserved tokens were written by the filter, beside keep_idx)
  launch_compress(p, pl, w, discard_idx, keep_idx, edge_cnt, edge_tgt, edge_alpha, X_out, nullptr, s, true);
  return finish(ctx, fn);
}

}  // namespace ficoco

using namespace ficoco;

extern "C" {

int ficoco_create(ficoco_ctx** out, int device) {
  if (!out) return FICOCO_EINVAL;
  *out = nullptr;
  int count = 0;
  if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) return FICOCO_EHIP;
  if (device < kMaxDevices && g_static_ws[device] == nullptr) {
    // the scratch array's address on this device, asked for with that device current
    int prev = -1;
    if (hipGetDevice(&prev) != hipSuccess) return FICOCO_EHIP;
    if (prev != device && hipSetDevice(device) != hipSuccess) return FICOCO_EHIP;
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_static_scratch));
    if (prev != device) (void)hipSetDevice(prev);
    if (e != hipSuccess || ptr == nullptr) return FICOCO_EHIP;
    g_static_ws[device] = ptr;
  }
  ficoco_ctx* c = new (std::nothrow) ficoco_ctx;
  if (!c) return FICOCO_ENOMEM;
  c->device = device;
  c->probe_start = nullptr;
  c->probe_stop = nullptr;
  c->probe_kernel = FICOCO_PROBE_REDUCE;
  c->err[0] = 0;
  *out = c;
  return FICOCO_OK;
}

int ficoco_destroy(ficoco_ctx* ctx) {
  delete ctx;
  return FICOCO_OK;
}

const char* ficoco_last_error(const ficoco_ctx* ctx) { return ctx ? ctx->err : "ctx is NULL"; }

int ficoco_set_probe(ficoco_ctx* ctx, int kernel, void* start_event, void* stop_event) {
  if (!ctx || ((start_event == nullptr) != (stop_event == nullptr)) ||
      (kernel != FICOCO_PROBE_REDUCE && kernel != FICOCO_PROBE_GRAM && kernel != FICOCO_PROBE_GRAM_X16))
    return FICOCO_EINVAL;
  ctx->probe_kernel = kernel;
  ctx->probe_start = (hipEvent_t)start_event;
  ctx->probe_stop = (hipEvent_t)stop_event;
  return FICOCO_OK;
}

const char* ficoco_version(void) { return "ficoco-gfx950 0.1"; }

int ficoco_workspace_bytes(const ficoco_problem* p, size_t* out_bytes) {
  if (!p || !out_bytes) return FICOCO_EINVAL;
  Plan pl;
  const char* why;
  const int rc = make_plan(*p, pl, &why);
  if (rc != FICOCO_OK) return rc;
  *out_bytes = pl.total;
  return FICOCO_OK;
}

int ficoco_out_rows(const ficoco_problem* p, int32_t* out_rows) {
  if (!p || !out_rows) return FICOCO_EINVAL;
  Plan pl;
  const char* why;
  const int rc = make_plan(*p, pl, &why);
  if (rc != FICOCO_OK) return rc;
  *out_rows = pl.n_out;
  return FICOCO_OK;
}

int ficoco_reduce(ficoco_ctx* ctx, const ficoco_problem* p, void* ws, size_t ws_bytes, void* stream) {
  Plan pl;
  const int rc = prepare(ctx, p, ws, ws_bytes, pl, "ficoco_reduce");
  if (rc != FICOCO_OK) return rc;
  const bool pr = ctx->probe_start && ctx->probe_kernel == FICOCO_PROBE_REDUCE;
  if (pr) (void)hipEventRecord(ctx->probe_start, (hipStream_t)stream);
  if (pl.qk) launch_attn_qk(*p, pl, (char*)ws, (hipStream_t)stream);
  else launch_attn_reduce(*p, pl, (char*)ws, (hipStream_t)stream);
  if (pr) (void)hipEventRecord(ctx->probe_stop, (hipStream_t)stream);
  return finish(ctx, "ficoco_reduce");
}

int ficoco_score(ficoco_ctx* ctx, const ficoco_problem* p, void* ws, size_t ws_bytes, double* scores,
                 void* stream) {
  Plan pl;
  const int rc = prepare(ctx, p, ws, ws_bytes, pl, "ficoco_score");
  if (rc != FICOCO_OK) return rc;
  if (!scores) return fail(ctx, FICOCO_EINVAL, "ficoco_score", "scores is NULL");
  const bool tw = text_with_features(*p, pl);
  if (pl.qk) launch_attn_qk(*p, pl, (char*)ws, (hipStream_t)stream);
  else launch_attn_reduce(*p, pl, (char*)ws, (hipStream_t)stream, tw);
  if (pl.need_features) launch_features(*p, pl, (char*)ws, (hipStream_t)stream, tw, false);
  launch_score(*p, pl, (char*)ws, scores, (hipStream_t)stream, tw);
  return finish(ctx, "ficoco_score");
}

int ficoco_filter(ficoco_ctx* ctx, const ficoco_problem* p, void* ws, size_t ws_bytes,
                  const double* scores, int32_t* discard_idx, int32_t* keep_idx, void* stream) {
  Plan pl;
  const int rc = prepare(ctx, p, ws, ws_bytes, pl, "ficoco_filter");
  if (rc != FICOCO_OK) return rc;
  if (!scores || !keep_idx || (pl.n_disc > 0 && !discard_idx))
    return fail(ctx, FICOCO_EINVAL, "ficoco_filter", "a pointer is NULL");
  launch_filter(*p, pl, (char*)ws, scores, discard_idx, keep_idx, (hipStream_t)stream);
  return finish(ctx, "ficoco_filter");
}

int ficoco_correlate(ficoco_ctx* ctx, const ficoco_problem* p, void* ws, size_t ws_bytes,
                     const int32_t* discard_idx, const int32_t* keep_idx, int32_t* edge_cnt,
                     int32_t* edge_tgt, double* edge_alpha, int32_t* overflow, void* stream) {
  Plan pl;
  const int rc = prepare(ctx, p, ws, ws_bytes, pl, "ficoco_correlate");
  if (rc != FICOCO_OK) return rc;
  if (!keep_idx || !overflow || (pl.n_disc > 0 && (!discard_idx || !edge_cnt || !edge_tgt || !edge_alpha)))
    return fail(ctx, FICOCO_EINVAL, "ficoco_correlate", "a pointer is NULL");
  const bool pg = ctx->probe_start && (ctx->probe_kernel == FICOCO_PROBE_GRAM || ctx->probe_kernel == FICOCO_PROBE_GRAM_X16);
  launch_correlate(*p, pl, (char*)ws, discard_idx, keep_idx, edge_cnt, edge_tgt, edge_alpha, overflow,
                   false, pg ? ctx->probe_start : nullptr, pg ? ctx->probe_stop : nullptr,
                   (hipStream_t)stream, pg && ctx->probe_kernel == FICOCO_PROBE_GRAM_X16 ? FICOCO_PROBE_REPEAT : 1);
  return finish(ctx, "ficoco_correlate");
}

int ficoco_correlation_gap(ficoco_ctx* ctx, const ficoco_problem* p, void* ws, size_t ws_bytes,
                           const int32_t* discard_idx, const int32_t* keep_idx, double* gap, void* stream) {
  Plan pl;
  const int rc = prepare(ctx, p, ws, ws_bytes, pl, "ficoco_correlation_gap");
  if (rc != FICOCO_OK) return rc;
  if (!keep_idx || (pl.n_disc > 0 && (!discard_idx || !gap)))
    return fail(ctx, FICOCO_EINVAL, "ficoco_correlation_gap", "a pointer is NULL");
  launch_corr_gap(*p, pl, (char*)ws, discard_idx, keep_idx, gap, (hipStream_t)stream);
  return finish(ctx, "ficoco_correlation_gap");
}

int ficoco_gather_tokens(ficoco_ctx* ctx, const ficoco_problem* p, const int32_t* keep_idx, const void* in,
                         int64_t in_stride_b, int64_t in_stride_n, int32_t row_bytes, void* out, void* stream) {
  if (!ctx) return FICOCO_EINVAL;
  if (!p) return fail(ctx, FICOCO_EINVAL, "ficoco_gather_tokens", "problem is NULL");
  const int dev_rc = check_device(ctx, "ficoco_gather_tokens");
  if (dev_rc != FICOCO_OK) return dev_rc;
  Plan pl;
  const char* why;
  const int rc = make_plan(*p, pl, &why);
  if (rc != FICOCO_OK) return fail(ctx, rc, "ficoco_gather_tokens", why);
  if (pl.extra_token)
    return fail(ctx, FICOCO_EUNSUPPORTED, "ficoco_gather_tokens", "the convergent form's additional token has no row to gather");
  if (!keep_idx || !in || !out) return fail(ctx, FICOCO_EINVAL, "ficoco_gather_tokens", "a pointer is NULL");
  if (row_bytes < 4 || row_bytes % 4 != 0 || in_stride_n < row_bytes || in_stride_n % 4 != 0 || in_stride_b % 4 != 0 ||
      ((uintptr_t)in % 4) != 0 || ((uintptr_t)out % 4) != 0)
    return fail(ctx, FICOCO_EINVAL, "ficoco_gather_tokens", "row_bytes / strides / pointers must be multiples of 4 bytes");
  launch_gather(*p, pl, keep_idx, in, in_stride_b, in_stride_n, row_bytes, out, (hipStream_t)stream);
  return finish(ctx, "ficoco_gather_tokens");
}

int ficoco_compress(ficoco_ctx* ctx, const ficoco_problem* p, void* ws, size_t ws_bytes,
                    const int32_t* discard_idx, const int32_t* keep_idx, const int32_t* edge_cnt,
                    const int32_t* edge_tgt, const double* edge_alpha, void* X_out, int32_t* pos_out,
                    void* stream) {
  Plan pl;
  const int rc = prepare(ctx, p, ws, ws_bytes, pl, "ficoco_compress");
  if (rc != FICOCO_OK) return rc;
  if (!X_out || !keep_idx || (pl.n_disc > 0 && (!discard_idx || !edge_cnt || !edge_tgt || !edge_alpha)))
    return fail(ctx, FICOCO_EINVAL, "ficoco_compress", "a pointer is NULL");
  if (ranges_overlap(X_out, x_out_extent(*p, pl), p->X, x_extent(*p)))
    return fail(ctx, FICOCO_EINVAL, "ficoco_compress", "X_out overlaps X (outputs may not alias inputs)");
  launch_compress(*p, pl, (char*)ws, discard_idx, keep_idx, edge_cnt, edge_tgt, edge_alpha, X_out,
                  pos_out, (hipStream_t)stream);
  return finish(ctx, "ficoco_compress");
}

int ficoco_v_step(ficoco_ctx* ctx, const ficoco_problem* p, void* ws, size_t ws_bytes, void* X_out,
                  int32_t* pos_out, int32_t* keep_idx, int32_t* discard_idx, int32_t* edge_cnt,
                  int32_t* edge_tgt, double* edge_alpha, double* scores, int32_t* overflow,
                  void* stream) {
  return run_step(ctx, p, FICOCO_VARIANT_V, ws, ws_bytes, X_out, pos_out, keep_idx, discard_idx,
                  edge_cnt, edge_tgt, edge_alpha, scores, overflow, stream, "ficoco_v_step");
}

int ficoco_v_step_static(ficoco_ctx* ctx, const ficoco_problem* p, void* X_out, int32_t* pos_out,
                         int32_t* keep_idx, int32_t* discard_idx, int32_t* edge_cnt, int32_t* edge_tgt,
                         double* edge_alpha, double* scores, int32_t* overflow, void* stream) {
  const char* fn = "ficoco_v_step_static";
  if (!ctx) return FICOCO_EINVAL;
  if (!p) return fail(ctx, FICOCO_EINVAL, fn, "problem is NULL");
  Plan pl;
  const char* why;
  const int rc = make_plan(*p, pl, &why);
  if (rc != FICOCO_OK) return fail(ctx, rc, fn, why);
  if (pl.total > kStaticScratchBytes)
    return fail(ctx, FICOCO_ENOMEM, fn, "the step's workspace exceeds the 32 MiB static scratch: use ficoco_v_step with a caller workspace");
  void* ws = ctx->device < kMaxDevices ? g_static_ws[ctx->device] : nullptr;
  if (!ws) return fail(ctx, FICOCO_EHIP, fn, "no static scratch on this device");
  return run_step(ctx, p, FICOCO_VARIANT_V, ws, kStaticScratchBytes, X_out, pos_out, keep_idx, discard_idx,
                  edge_cnt, edge_tgt, edge_alpha, scores, overflow, stream, fn);
}

int ficoco_l_step(ficoco_ctx* ctx, const ficoco_problem* p, void* ws, size_t ws_bytes, void* X_out,
                  int32_t* pos_out, int32_t* keep_idx, int32_t* discard_idx, int32_t* edge_cnt,
                  int32_t* edge_tgt, double* edge_alpha, double* scores, int32_t* overflow,
                  void* stream) {
  return run_step(ctx, p, FICOCO_VARIANT_L, ws, ws_bytes, X_out, pos_out, keep_idx, discard_idx,
                  edge_cnt, edge_tgt, edge_alpha, scores, overflow, stream, "ficoco_l_step");
}

}  // extern "C"
