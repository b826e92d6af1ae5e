/* A caller written in plain C against include/ficoco.h: one tiny FiCoCo-V step whose result
 * has a closed form.  Built with gcc (no C++) and linked against libficoco.so, as a shared
 * object whose one function the GPU test calls in its own process (a process that has touched
 * the GPU must not start other programs on the test machines); -DSTEP_CHECK_MAIN adds a main().
 *
 * Workload: [CLS] + a 4 x 4 grid, D = 8, H = 2, float32; the attention map is uniform
 * (every entry 1/17).  Then every token has the same score s = (0.35 - 0.65)/17 < 0; the
 * local penalty doubles the first cell of every 2 x 2 window (ties go to the lowest cell),
 * which makes those four tokens (0, 2, 8, 10) the LEAST redundant; the top-K filter discards
 * the four lowest-indexed of the other twelve: S = {1, 3, 4, 5}.  Every correlation equals
 * 1/17, so every discarded token is recycled into all twelve preserved tokens with weight
 * 1/12, and Eq. 2 gives X'_j = (X_j + (X_1 + X_3 + X_4 + X_5)/12) / (1 + 4/12).
 */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>

#include "ficoco.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %d at line %d\n", (int)e_, __LINE__); return 2; } } while (0)
#define CHECK_FC(x) do { int s_ = (x); if (s_ != FICOCO_OK) { printf("ficoco status %d at line %d: %s\n", s_, __LINE__, ficoco_last_error(ctx)); return 3; } } while (0)

enum { G = 4, N = G * G, NTOT = N + 1, D = 8, H = 2, KEEP = 12, NDISC = N - KEEP, KMAX = 16 };

int ficoco_c_step_check(void) {
  static float X[NTOT][D], A[H][NTOT][NTOT], X_out[NTOT - NDISC][D];
  for (int t = 0; t < NTOT; ++t)
    for (int d = 0; d < D; ++d) X[t][d] = (float)(t * 3 + d) - 7.5f;
  for (int h = 0; h < H; ++h)
    for (int q = 0; q < NTOT; ++q)
      for (int k = 0; k < NTOT; ++k) A[h][q][k] = 1.0f / (float)NTOT;

  ficoco_ctx *ctx = NULL;
  if (ficoco_create(&ctx, 0) != FICOCO_OK) { printf("ficoco_create failed\n"); return 1; }

  float *dX, *dA, *dXo;
  int32_t *d_keep, *d_disc, *d_cnt, *d_tgt, *d_pos, *d_ovf;
  double *d_alpha, *d_scores;
  CHECK_HIP(hipMalloc((void **)&dX, sizeof X));
  CHECK_HIP(hipMalloc((void **)&dA, sizeof A));
  CHECK_HIP(hipMalloc((void **)&dXo, sizeof X_out));
  CHECK_HIP(hipMalloc((void **)&d_keep, KEEP * 4));
  CHECK_HIP(hipMalloc((void **)&d_disc, NDISC * 4));
  CHECK_HIP(hipMalloc((void **)&d_cnt, NDISC * 4));
  CHECK_HIP(hipMalloc((void **)&d_tgt, NDISC * KMAX * 4));
  CHECK_HIP(hipMalloc((void **)&d_alpha, NDISC * KMAX * 8));
  CHECK_HIP(hipMalloc((void **)&d_scores, N * 8));
  CHECK_HIP(hipMalloc((void **)&d_pos, KEEP * 4));
  CHECK_HIP(hipMalloc((void **)&d_ovf, 4));
  CHECK_HIP(hipMemcpy(dX, X, sizeof X, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(dA, A, sizeof A, hipMemcpyHostToDevice));

  ficoco_problem p;
  memset(&p, 0, sizeof p);
  p.variant = FICOCO_VARIANT_V; p.dtype = FICOCO_F32;
  p.B = 1; p.H = H; p.D = D; p.n_tot = NTOT; p.vis_begin = 1; p.N = N; p.n_keep = KEEP; p.cls_index = 0;
  p.X = dX; p.x_stride_b = NTOT * D; p.x_stride_n = D;
  p.A = dA; p.a_stride_b = H * NTOT * NTOT; p.a_stride_h = NTOT * NTOT; p.a_stride_q = NTOT;
  p.a_q_begin = 0; p.a_nq = NTOT; p.a_k_begin = 0; p.a_nk = NTOT;
  p.grid_g = 1; p.grid_h = G; p.grid_w = G; p.window = 2; p.penalty_coef = 2.0f;
  p.w_score = 0.35f; p.gamma = 0.6f; p.eps = 0.998f;
  p.red_src = FICOCO_R_ATTN_RECV; p.sem_src = FICOCO_G_CLS_ATTN; p.corr_src = FICOCO_C_ATTN; p.k_max = KMAX;

  size_t ws_bytes = 0;
  CHECK_FC(ficoco_workspace_bytes(&p, &ws_bytes));
  void *ws;
  CHECK_HIP(hipMalloc(&ws, ws_bytes));
  int32_t rows = 0;
  CHECK_FC(ficoco_out_rows(&p, &rows));
  if (rows != NTOT - NDISC) { printf("ficoco_out_rows: %d\n", rows); return 4; }

  /* an aliased output must be refused on the host */
  if (ficoco_v_step(ctx, &p, ws, ws_bytes, dX, d_pos, d_keep, d_disc, d_cnt, d_tgt, d_alpha, d_scores, d_ovf, NULL) != FICOCO_EINVAL) {
    printf("X_out == X was not refused\n");
    return 5;
  }
  CHECK_FC(ficoco_v_step(ctx, &p, ws, ws_bytes, dXo, d_pos, d_keep, d_disc, d_cnt, d_tgt, d_alpha, d_scores, d_ovf, NULL));
  CHECK_HIP(hipDeviceSynchronize());

  int32_t keep[KEEP], disc[NDISC], cnt[NDISC], ovf;
  CHECK_HIP(hipMemcpy(keep, d_keep, sizeof keep, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(disc, d_disc, sizeof disc, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(cnt, d_cnt, sizeof cnt, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(&ovf, d_ovf, 4, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(X_out, dXo, sizeof X_out, hipMemcpyDeviceToHost));

  const int32_t want_disc[NDISC] = {1, 3, 4, 5};
  const int32_t want_keep[KEEP] = {0, 2, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15};
  int bad = ovf != 0;
  for (int a = 0; a < NDISC; ++a) bad |= disc[a] != want_disc[a] || cnt[a] != KEEP;
  for (int j = 0; j < KEEP; ++j) bad |= keep[j] != want_keep[j];
  for (int d = 0; d < D; ++d) bad |= X_out[0][d] != X[0][d];               /* [CLS] is copied */
  for (int j = 0; j < KEEP && !bad; ++j)
    for (int d = 0; d < D; ++d) {
      double add = 0.0;
      for (int a = 0; a < NDISC; ++a) add += (double)X[1 + want_disc[a]][d] / 12.0;
      const double want = ((double)X[1 + want_keep[j]][d] + add) / (1.0 + 4.0 / 12.0);
      if (fabs((double)X_out[1 + j][d] - want) > 1e-5 * fabs(want) + 1e-6) bad = 1;
    }
  if (bad) { printf("FAIL: the step's result differs from the closed form\n"); return 6; }
  ficoco_destroy(ctx);
  printf("OK: ficoco_v_step called from C matches the closed form\n");
  return 0;
}

#ifdef STEP_CHECK_MAIN
int main(void) { return ficoco_c_step_check(); }
#endif
