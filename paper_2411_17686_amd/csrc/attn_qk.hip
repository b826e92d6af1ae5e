// Attention reduction from queries and keys (Sec. "Self-Attention": A = Softmax(Q K^T / sqrt(D))):
// the per-head maps are formed on the matrix cores and reduced on the fly, so the [B,H,n,n]
// maps never exist in memory.  Outputs are those of attn_reduce.hip -- per-tile column partials of
// the received attention (first term of Eq. 1), the [CLS] row (second term), and the head-mean
// map in single precision, transposed, for the correlate stage (Algorithm 1, stage 2).
//
// Single precision throughout (products of bfloat16 values are exact in it); the vector arithmetic
// of the softmax, not memory, bounds the kernel.
#include "common.hpp"

#include <algorithm>

namespace ficoco {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int kQkWaves = 8;                         // wavefronts per workgroup: they split the keys
constexpr int kQkKB = 5;                            // 16-key blocks per wavefront
constexpr int kQkQB = kQkTile / 16;                 // 16-query blocks per workgroup
static_assert(kQkWaves * kQkKB * 16 == kQkMaxKeys, "the wavefronts split the keys");
static_assert(kQkTile % 16 == 0, "whole 16-query blocks");

struct QkArgs {
  const bf16_t* Q;
  const bf16_t* K;
  int64_t sb, sh, sn;
  int H, n;             // heads, rows of the block (queries = keys)
  int N;                // visual tokens
  int vis0;             // block row of visual token 0
  int cls_r;            // block row of the [CLS] query, or -1
  float scale_log2e;    // qk_scale * log2(e): exponentials are taken as powers of two
  float* abar;          // [B][N][map_pitch] or null
  int map_pitch;
  double* recv_part;    // [B][n_tiles][N]
  double* cls;          // [B][N]
  int n_tiles, B;
  // the two-sweep kernel only:
  int q_begin, q_count; // block rows whose queries are needed (the tiles cover these)
  int text0, M;         // FiCoCo-L: block row of the first text query, number of text queries
  double* ttext;        // FiCoCo-L: [B][N][M] head-mean attention of the text queries on the visual keys, or null
  // Few tiles: the heads are split over `groups` workgroups per tile (heads_per_group consecutive
  // heads each), which leave head SUMS in single precision; a second kernel adds the groups in
  // order and divides by H.  groups == 1: the outputs are written directly.
  int groups, heads_per_group;
  float* part_map;      // [groups][B][N][map_pitch]
  float* part_text;     // [groups][B][N][M]
  float* part_recv;     // [groups][B][n_tiles][N]
  float* part_cls;      // [groups][B][N]
};

// v_mfma_f32_16x16x32_bf16: operand A is 16 rows x 32 features (lane: row lane % 16, features
// 8 (lane / 16) .. + 8), operand B 16 columns x 32 features (same), the result 16 x 16 (lane: column
// lane % 16, rows 4 (lane / 16) + v for its four registers v).  Rows are keys here, columns queries:
// a lane's 16-byte operand loads of one key cover 64 contiguous bytes of the key's row across the
// four lane groups, and a query's probabilities sit in the registers of four lanes.
//
// A workgroup owns kQkTile query rows of one image; its 8 wavefronts split the keys (80 each, 640 at
// most) and walk the heads in order, the operands of the next head being loaded while the current
// head's softmax is computed.
template <int KS>     // 32-feature steps of the head dimension
__global__ __launch_bounds__(kQkWaves * kWave) void attn_qk_kernel(QkArgs a) {
  __shared__ float xmax[2][kQkWaves][kQkTile];
  __shared__ float xsum[2][kQkWaves][kQkTile];
  const int total = a.n_tiles * a.B;
  const int logical = xcd_logical_id(blockIdx.x, total);     // the tiles of one image share an XCD and its L2 (the keys)
  if (logical >= total) return;
  const int tile = logical % a.n_tiles;
  const int64_t b = logical / a.n_tiles;
  const int lane = threadIdx.x % kWave;
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);   // the same in every lane: scalar, so tests on it are branches
  const int l16 = lane % 16, lg = lane / 16;
  const float NEG = -__builtin_huge_valf();
  const int key_base = wv * kQkKB * 16;             // first key of this wavefront

  // operand addresses (clamped to valid rows: what lies past the block is masked later)
  int64_t q_off[kQkQB], k_off[kQkKB];
#pragma unroll
  for (int qb = 0; qb < kQkQB; ++qb) q_off[qb] = (int64_t)min(tile * kQkTile + qb * 16 + l16, a.n - 1) * a.sn + lg * 8;
#pragma unroll
  for (int kb = 0; kb < kQkKB; ++kb) k_off[kb] = (int64_t)min(key_base + kb * 16 + l16, a.n - 1) * a.sn + lg * 8;

  bf16x8_t kf[kQkKB][KS], qf[kQkQB][KS];
  auto load_head = [&](int h) {
    const bf16_t* Qh = a.Q + b * a.sb + (int64_t)h * a.sh;
    const bf16_t* Kh = a.K + b * a.sb + (int64_t)h * a.sh;
#pragma unroll
    for (int kb = 0; kb < kQkKB; ++kb)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) __builtin_memcpy(&kf[kb][ks], Kh + k_off[kb] + ks * 32, 16);
#pragma unroll
    for (int qb = 0; qb < kQkQB; ++qb)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) __builtin_memcpy(&qf[qb][ks], Qh + q_off[qb] + ks * 32, 16);
  };

  f32x4_t P[kQkKB][kQkQB];
#pragma unroll
  for (int kb = 0; kb < kQkKB; ++kb)
#pragma unroll
    for (int qb = 0; qb < kQkQB; ++qb) P[kb][qb] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};

  load_head(0);
#pragma unroll 1
  for (int h = 0; h < a.H; ++h) {
    // logits of this head: S[kb][qb][v] = key (key_base + 16 kb + 4 lg + v) . query (16 qb + l16)
    f32x4_t S[kQkKB][kQkQB];
#pragma unroll
    for (int kb = 0; kb < kQkKB; ++kb)
#pragma unroll
      for (int qb = 0; qb < kQkQB; ++qb) {
        S[kb][qb] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          S[kb][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[kb][ks], qf[qb][ks], S[kb][qb], 0, 0, 0);
      }
    // the next head's operands are on their way while this head's softmax is computed (past the
    // last head the last one is loaded again)
    load_head(min(h + 1, a.H - 1));
    issue_fence();                  // the loads go out here, not where the next head first uses them
    // keys past the block read as -inf (only the last wavefronts can hold any: a scalar test, so the
    // others skip the selects altogether)
    if (key_base + kQkKB * 16 > a.n) {
#pragma unroll
    for (int kb = 0; kb < kQkKB; ++kb) {
      if (key_base + (kb + 1) * 16 > a.n) {
#pragma unroll
        for (int v = 0; v < 4; ++v)
          if (key_base + kb * 16 + lg * 4 + v >= a.n) {
#pragma unroll
            for (int qb = 0; qb < kQkQB; ++qb) S[kb][qb][v] = NEG;
          }
      }
    }
    }
    // Softmax of every query's row with ONE exchange between the wavefronts: a wavefront takes the
    // exponentials relative to a reference at or above the maximum of ITS keys (the maximum in
    // units of log2, rounded up to a whole number) and sums them; the (reference, sum) pairs are
    // exchanged, and its probabilities are its exponentials times 2^(own reference - largest
    // reference) / row sum.  scale_log2e > 0.
    const int par = h & 1;          // two sets of slots: the next head's writes do not wait for this head's reads
    // The three query blocks go through every stage side by side (maxima, their two exchanges
    // between the lane groups, exponentials, sums, their exchanges, one write): taken one block
    // after the other, each of the twelve lane exchanges of a head waits out its own trip
    // through the permute path.
    float mc[kQkQB], mw[kQkQB], lw[kQkQB];
    bool any_key[kQkQB];
#pragma unroll
    for (int qb = 0; qb < kQkQB; ++qb) {
      mw[qb] = NEG;
#pragma unroll
      for (int kb = 0; kb < kQkKB; ++kb)
#pragma unroll
        for (int v = 0; v < 4; ++v) mw[qb] = fmaxf(mw[qb], S[kb][qb][v]);
    }
    {
      float o[kQkQB];
#pragma unroll
      for (int qb = 0; qb < kQkQB; ++qb) o[qb] = __shfl_xor(mw[qb], 16, kWave);
#pragma unroll
      for (int qb = 0; qb < kQkQB; ++qb) mw[qb] = fmaxf(mw[qb], o[qb]);
#pragma unroll
      for (int qb = 0; qb < kQkQB; ++qb) o[qb] = __shfl_xor(mw[qb], 32, kWave);
#pragma unroll
      for (int qb = 0; qb < kQkQB; ++qb) mw[qb] = fmaxf(mw[qb], o[qb]);
    }
#pragma unroll
    for (int qb = 0; qb < kQkQB; ++qb) {
      any_key[qb] = mw[qb] > NEG;                   // a wavefront whose keys all lie past the block has none
      mc[qb] = any_key[qb] ? ceilf(mw[qb] * a.scale_log2e) : 0.0f;  // a whole number: rescaling between wavefronts is exact
      lw[qb] = 0.0f;
#pragma unroll
      for (int kb = 0; kb < kQkKB; ++kb)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const float e = __builtin_amdgcn_exp2f(fmaf(S[kb][qb][v], a.scale_log2e, -mc[qb]));
          S[kb][qb][v] = e;
          lw[qb] += e;
        }
    }
    {
      float o[kQkQB];
#pragma unroll
      for (int qb = 0; qb < kQkQB; ++qb) o[qb] = __shfl_xor(lw[qb], 16, kWave);
#pragma unroll
      for (int qb = 0; qb < kQkQB; ++qb) lw[qb] += o[qb];
#pragma unroll
      for (int qb = 0; qb < kQkQB; ++qb) o[qb] = __shfl_xor(lw[qb], 32, kWave);
#pragma unroll
      for (int qb = 0; qb < kQkQB; ++qb) lw[qb] += o[qb];
    }
    if (lg == 0) {
#pragma unroll
      for (int qb = 0; qb < kQkQB; ++qb) {
        xmax[par][wv][qb * 16 + l16] = any_key[qb] ? mc[qb] : NEG;
        xsum[par][wv][qb * 16 + l16] = lw[qb];
      }
    }
    __syncthreads();
#pragma unroll
    for (int qb = 0; qb < kQkQB; ++qb) {
      const int qi = qb * 16 + l16;
      float m = NEG;
#pragma unroll
      for (int w = 0; w < kQkWaves; ++w) m = fmaxf(m, xmax[par][w][qi]);          // finite: key 0 is valid
      float l = 0.0f;
#pragma unroll
      for (int w = 0; w < kQkWaves; ++w)                                         // wavefronts in order; 2^(whole number) is exact
        l += xsum[par][w][qi] * __builtin_amdgcn_exp2f(fmaxf(xmax[par][w][qi] - m, -150.0f));
      // the quotient is taken by every lane (l > 0: key 0 is valid) and dropped where the wavefront
      // has no key: as the value of a choice it would sit in a branch of its own
      const float q = __builtin_amdgcn_exp2f(fmaxf(mc[qb] - m, -150.0f)) / l;
      const float inv = any_key[qb] ? q : 0.0f;
#pragma unroll
      for (int kb = 0; kb < kQkKB; ++kb)
#pragma unroll
        for (int v = 0; v < 4; ++v) P[kb][qb][v] = fmaf(S[kb][qb][v], inv, P[kb][qb][v]);
    }
  }

  const float invH = 1.0f / (float)a.H;
#pragma unroll
  for (int kb = 0; kb < kQkKB; ++kb) {
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int ik = key_base + kb * 16 + lg * 4 + v - a.vis0;      // visual key index
      const bool k_vis = ik >= 0 && ik < a.N;
      float cs = 0.0f;                                              // received from this tile's visual queries
#pragma unroll
      for (int qb = 0; qb < kQkQB; ++qb) {
        const int q = tile * kQkTile + qb * 16 + l16;
        const int jq = q - a.vis0;                                  // visual query index
        const bool q_vis = q < a.n && jq >= 0 && jq < a.N;
        const float pm = P[kb][qb][v] * invH;                       // head-mean probability P[q][key]
        if (a.abar && q_vis && k_vis) a.abar[(b * a.N + ik) * a.map_pitch + jq] = pm;
        if (q == a.cls_r && k_vis) a.cls[b * a.N + ik] = (double)pm;
        cs += q_vis ? pm : 0.0f;
      }
      // sum over the 16 lanes that hold the tile's other queries of this key (a fixed butterfly)
#pragma unroll
      for (int off = 8; off > 0; off >>= 1) cs += __shfl_xor(cs, off, kWave);
      if (l16 == 0 && k_vis) a.recv_part[(b * a.n_tiles + tile) * a.N + ik] = (double)cs;
    }
  }
}

// More keys than one workgroup holds in registers (kQkMaxKeys): the keys are taken in blocks of
// kQkMaxKeys (each wavefront 80 of a block, as above), in two sweeps.  Sweep 1, head by head: the
// row maximum and the row sum of every query over all key blocks, kept per wavefront as a running
// (reference, sum) pair -- the reference a whole number in units of log2, so that rescaling the sum
// when a later block raises it is exact -- and combined across the wavefronts once per head; the
// results (reference, 1 / sum) of all heads wait in LDS.  Sweep 2, key block by key block: the
// logits of every head are formed again, turned into probabilities with the stored pair and
// accumulated over the heads in registers; the block's piece of the head-mean map, of the [CLS] row
// and of the column partials is written as above.  The logits are computed twice; the maps still
// never exist in memory.  The same kernel serves the decoder of FiCoCo-L (DEC: a key behind
// its query reads as -inf like a key past the sequence; the tiles cover the visual and the text
// queries, or the text queries alone where no visual-to-visual term is needed; the rows of the text
// queries leave as the text profiles of Eq. 3 / Eq. 4).
template <int KS, int KBU, bool DEC>     // KBU: groups of 16 keys a wavefront holds of a key block (<= kQkKB); DEC: the decoder's causal maps
__global__ __launch_bounds__(kQkWaves * kWave) void attn_qk_long_kernel(QkArgs a) {
  extern __shared__ float norm[];                    // [heads of this workgroup][kQkTile][2]: reference, 1 / row sum
  __shared__ float xmax[kQkWaves][kQkTile];
  __shared__ float xsum[kQkWaves][kQkTile];
  const int total = a.n_tiles * a.B * a.groups;
  const int logical = xcd_logical_id(blockIdx.x, total);
  if (logical >= total) return;
  const int grp = logical % a.groups;               // the groups of a tile are neighbours: same operands
  const int tile = (logical / a.groups) % a.n_tiles;
  const int64_t b = logical / (a.groups * a.n_tiles);
  const int h_lo = grp * a.heads_per_group, h_hi = min(h_lo + a.heads_per_group, a.H);
  if (h_lo >= h_hi) return;                         // (the launcher leaves no group without heads)
  const int lane = threadIdx.x % kWave;
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int l16 = lane % 16, lg = lane / 16;
  const float NEG = -__builtin_huge_valf();
  // A key block is KBU groups of 16 keys per wavefront: 640 keys with five groups, 384 with three
  // (675 keys are two blocks of 384 instead of 640 + 35, with three fifths of the registers).
  constexpr int kbu = KBU;
  constexpr int blk_keys = kQkWaves * KBU * 16;
  const int key_base = wv * KBU * 16;               // first key of this wavefront inside a key block
  const int n_blocks = (a.n + blk_keys - 1) / blk_keys;
  const int q_first = a.q_begin + tile * kQkTile;   // block row of this tile's first query
  const int q_end = min(a.q_begin + a.q_count, a.n);
  // decoder: key blocks that begin behind the tile's last query hold no key any of its queries
  // attends -- they are not computed (their pieces of the outputs are written as zeros)
  const int nb = DEC ? min(n_blocks, min(q_first + kQkTile - 1, q_end - 1) / blk_keys + 1) : n_blocks;

  int q_row[kQkQB];
  int64_t q_off[kQkQB];
#pragma unroll
  for (int qb = 0; qb < kQkQB; ++qb) {
    q_row[qb] = q_first + qb * 16 + l16;
    q_off[qb] = (int64_t)min(q_row[qb], a.n - 1) * a.sn + lg * 8;
  }

  // Operands of head h and key block blk (rows clamped to valid ones), and the logits between this
  // tile's queries and this wavefront's keys of the block (keys past the sequence read as -inf).
  // The operands of the next (head, block) are loaded right after the matrix instructions of the
  // current one, so that they arrive while its softmax is computed.
  bf16x8_t kf[KBU][KS], qf[kQkQB][KS];
  auto load_ops = [&](int h, int blk) {
    const bf16_t* Qh = a.Q + b * a.sb + (int64_t)h * a.sh;
    const bf16_t* Kh = a.K + b * a.sb + (int64_t)h * a.sh;
    const int k0 = blk * blk_keys + key_base;
#pragma unroll
    for (int kb = 0; kb < KBU; ++kb) {
      const int64_t off = (int64_t)min(k0 + kb * 16 + l16, a.n - 1) * a.sn + lg * 8;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) __builtin_memcpy(&kf[kb][ks], Kh + off + ks * 32, 16);
    }
#pragma unroll
    for (int qb = 0; qb < kQkQB; ++qb)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) __builtin_memcpy(&qf[qb][ks], Qh + q_off[qb] + ks * 32, 16);
  };
  auto logits = [&](int blk, f32x4_t (&S)[KBU][kQkQB], int h_next, int blk_next) {
    const int k0 = blk * blk_keys + key_base;
#pragma unroll
    for (int kb = 0; kb < KBU; ++kb)
#pragma unroll
      for (int qb = 0; qb < kQkQB; ++qb) {
        S[kb][qb] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          S[kb][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[kb][ks], qf[qb][ks], S[kb][qb], 0, 0, 0);
      }
    load_ops(h_next, blk_next);
    issue_fence();                                   // the loads go out here, not where they are first used
    if (k0 + kbu * 16 > a.n) {                       // scalar: only the last wavefronts of the last block
#pragma unroll
      for (int kb = 0; kb < KBU; ++kb)
#pragma unroll
        for (int v = 0; v < 4; ++v)
          if (k0 + kb * 16 + lg * 4 + v >= a.n) {
#pragma unroll
            for (int qb = 0; qb < kQkQB; ++qb) S[kb][qb][v] = NEG;
          }
    }
    if (DEC && k0 + kbu * 16 - 1 > q_first) {         // scalar: some key of this wavefront may lie behind some query
#pragma unroll
      for (int kb = 0; kb < KBU; ++kb)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int key = k0 + kb * 16 + lg * 4 + v;
#pragma unroll
          for (int qb = 0; qb < kQkQB; ++qb)
            if (key > q_row[qb]) S[kb][qb][v] = NEG;
        }
    }
  };

  // ---- sweep 1: (reference, 1 / sum) of every head and query ---------------------------------------
  load_ops(h_lo, 0);
#pragma unroll 1
  for (int h = h_lo; h < h_hi; ++h) {
    float mref[kQkQB], lsum[kQkQB];
#pragma unroll
    for (int qb = 0; qb < kQkQB; ++qb) { mref[qb] = NEG; lsum[qb] = 0.0f; }
#pragma unroll 1
    for (int blk = 0; blk < nb; ++blk) {
      f32x4_t S[KBU][kQkQB];
      {
        // next: the following block of this head, then block 0 of the next head; after the last of
        // sweep 1 the first of sweep 2 (head 0, block 0)
        const bool last_blk = blk + 1 == nb;
        logits(blk, S, last_blk ? (h + 1 < h_hi ? h + 1 : h_lo) : h, last_blk ? 0 : blk + 1);
      }
      float mw[kQkQB];
#pragma unroll
      for (int qb = 0; qb < kQkQB; ++qb) {
        mw[qb] = NEG;
#pragma unroll
        for (int kb = 0; kb < KBU; ++kb)
#pragma unroll
          for (int v = 0; v < 4; ++v) mw[qb] = fmaxf(mw[qb], S[kb][qb][v]);
      }
      {
        float o[kQkQB];
#pragma unroll
        for (int qb = 0; qb < kQkQB; ++qb) o[qb] = __shfl_xor(mw[qb], 16, kWave);
#pragma unroll
        for (int qb = 0; qb < kQkQB; ++qb) mw[qb] = fmaxf(mw[qb], o[qb]);
#pragma unroll
        for (int qb = 0; qb < kQkQB; ++qb) o[qb] = __shfl_xor(mw[qb], 32, kWave);
#pragma unroll
        for (int qb = 0; qb < kQkQB; ++qb) mw[qb] = fmaxf(mw[qb], o[qb]);
      }
#pragma unroll
      for (int qb = 0; qb < kQkQB; ++qb) {
        // the block's maximum in units of log2, rounded up to a whole number; -inf: no key of it here
        const float mc = mw[qb] > NEG ? ceilf(mw[qb] * a.scale_log2e) : NEG;
        const float ref = fmaxf(mref[qb], mc);
        const bool some = ref > NEG;                 // a key of this wavefront has been seen by now
        lsum[qb] *= some && mref[qb] > NEG ? __builtin_amdgcn_exp2f(fmaxf(mref[qb] - ref, -150.0f)) : 0.0f;
        mref[qb] = ref;
        const float sub = some ? ref : 0.0f;
#pragma unroll
        for (int kb = 0; kb < KBU; ++kb)
#pragma unroll
          for (int v = 0; v < 4; ++v) lsum[qb] += __builtin_amdgcn_exp2f(fmaf(S[kb][qb][v], a.scale_log2e, -sub));
      }
    }
    {
      float o[kQkQB];
#pragma unroll
      for (int qb = 0; qb < kQkQB; ++qb) o[qb] = __shfl_xor(lsum[qb], 16, kWave);
#pragma unroll
      for (int qb = 0; qb < kQkQB; ++qb) lsum[qb] += o[qb];
#pragma unroll
      for (int qb = 0; qb < kQkQB; ++qb) o[qb] = __shfl_xor(lsum[qb], 32, kWave);
#pragma unroll
      for (int qb = 0; qb < kQkQB; ++qb) lsum[qb] += o[qb];
    }
    if (lg == 0) {
#pragma unroll
      for (int qb = 0; qb < kQkQB; ++qb) {
        xmax[wv][qb * 16 + l16] = mref[qb];
        xsum[wv][qb * 16 + l16] = lsum[qb];
      }
    }
    __syncthreads();
    if ((int)threadIdx.x < kQkTile) {
      const int qi = threadIdx.x;
      float m = NEG;
#pragma unroll
      for (int w = 0; w < kQkWaves; ++w) m = fmaxf(m, xmax[w][qi]);               // finite: key 0 is valid
      float l = 0.0f;
#pragma unroll
      for (int w = 0; w < kQkWaves; ++w)                                          // wavefronts in order
        l += xmax[w][qi] > NEG ? xsum[w][qi] * __builtin_amdgcn_exp2f(fmaxf(xmax[w][qi] - m, -150.0f)) : 0.0f;
      norm[((h - h_lo) * kQkTile + qi) * 2] = m;
      norm[((h - h_lo) * kQkTile + qi) * 2 + 1] = 1.0f / l;
    }
    __syncthreads();              // the pairs are read back below; the exchange slots are written again by the next head
  }

  // ---- sweep 2: probabilities, head mean, outputs, key block by key block --------------------------
  const float invH = 1.0f / (float)a.H;
#pragma unroll 1
  for (int blk = 0; blk < n_blocks; ++blk) {
    f32x4_t P[KBU][kQkQB];
#pragma unroll
    for (int kb = 0; kb < KBU; ++kb)
#pragma unroll
      for (int qb = 0; qb < kQkQB; ++qb) P[kb][qb] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll 1
    for (int h = h_lo; h < (blk < nb ? h_hi : h_lo); ++h) {
      f32x4_t S[KBU][kQkQB];
      {
        // next: the following head of this block, then the first head of the next block (past the end: the last again)
        const bool last_h = h + 1 == h_hi;
        logits(blk, S, last_h ? h_lo : h + 1, last_h ? min(blk + 1, nb - 1) : blk);
      }
#pragma unroll
      for (int qb = 0; qb < kQkQB; ++qb) {
        const float m = norm[((h - h_lo) * kQkTile + qb * 16 + l16) * 2];
        const float inv = norm[((h - h_lo) * kQkTile + qb * 16 + l16) * 2 + 1];
#pragma unroll
        for (int kb = 0; kb < KBU; ++kb)
#pragma unroll
          for (int v = 0; v < 4; ++v)
            P[kb][qb][v] = fmaf(__builtin_amdgcn_exp2f(fmaf(S[kb][qb][v], a.scale_log2e, -m)), inv, P[kb][qb][v]);
      }
    }
#pragma unroll
    for (int kb = 0; kb < KBU; ++kb) {
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int key = blk * blk_keys + key_base + kb * 16 + lg * 4 + v;
        const int ik = key - a.vis0;                                  // visual key index
        const bool k_vis = key < a.n && ik >= 0 && ik < a.N;
        float cs = 0.0f;                                              // received from this tile's visual queries
#pragma unroll
        for (int qb = 0; qb < kQkQB; ++qb) {
          const int q = q_row[qb];
          const int jq = q - a.vis0;                                  // visual query index
          const bool q_vis = q < q_end && jq >= 0 && jq < a.N;
          const int mq = q - a.text0;                                 // text query index
          const bool q_txt = DEC && a.ttext && q < q_end && mq >= 0 && mq < a.M;
          if (a.groups > 1) {            // uniform: head sums of this group, combined by qk_combine_kernel
            const float ps = P[kb][qb][v];
            const int64_t gb = (int64_t)grp * a.B + b;
            if (a.abar && q_vis && k_vis) a.part_map[(gb * a.N + ik) * a.map_pitch + jq] = ps;
            if (q == a.cls_r && k_vis) a.part_cls[gb * a.N + ik] = ps;
            if (q_txt && k_vis) a.part_text[(gb * a.N + ik) * a.M + mq] = ps;
            cs += q_vis ? ps : 0.0f;
            continue;
          }
          const float pm = P[kb][qb][v] * invH;                       // head-mean probability P[q][key]
          if (a.abar && q_vis && k_vis) a.abar[(b * a.N + ik) * a.map_pitch + jq] = pm;
          if (q == a.cls_r && k_vis) a.cls[b * a.N + ik] = (double)pm;
          if (q_txt && k_vis) a.ttext[(b * a.N + ik) * a.M + mq] = (double)pm;
          cs += q_vis ? pm : 0.0f;
        }
#pragma unroll
        for (int off = 8; off > 0; off >>= 1) cs += __shfl_xor(cs, off, kWave);
        if (a.recv_part && l16 == 0 && k_vis) {
          if (a.groups > 1) a.part_recv[(((int64_t)grp * a.B + b) * a.n_tiles + tile) * a.N + ik] = cs;
          else a.recv_part[(b * a.n_tiles + tile) * a.N + ik] = (double)cs;
        }
      }
    }
  }
}

// The groups' head sums added in group order and divided by H: one thread per output element.
// The grid is the four outputs one after the other (map, text profiles, column partials, [CLS]
// row), each with exactly the workgroups it needs (an empty workgroup still costs its start).
struct QkCombineBlocks { int map, text, recv, cls; };
__global__ __launch_bounds__(256) void qk_combine_kernel(QkArgs a, QkCombineBlocks nb) {
  int blk = blockIdx.x, part = 0;
  if (blk >= nb.map) { blk -= nb.map; part = 1; if (blk >= nb.text) { blk -= nb.text; part = 2; if (blk >= nb.recv) { blk -= nb.recv; part = 3; } } }
  const int64_t i = (int64_t)blk * blockDim.x + threadIdx.x;
  const float invH = 1.0f / (float)a.H;
  auto total = [&](const float* part, int64_t at, int64_t stride) {
    float t = 0.0f;
    for (int g = 0; g < a.groups; ++g) t += part[at + g * stride];
    return t * invH;
  };
  if (part == 0) {
    if (!a.abar || i >= (int64_t)a.B * a.N * a.N) return;
    const int64_t at = (i / a.N) * a.map_pitch + i % a.N;           // [b][key][query < N]
    a.abar[at] = total(a.part_map, at, (int64_t)a.B * a.N * a.map_pitch);
  } else if (part == 1) {
    if (!a.ttext || i >= (int64_t)a.B * a.N * a.M) return;
    a.ttext[i] = (double)total(a.part_text, i, (int64_t)a.B * a.N * a.M);
  } else if (part == 2) {
    if (!a.recv_part || i >= (int64_t)a.B * a.n_tiles * a.N) return;
    a.recv_part[i] = (double)total(a.part_recv, i, (int64_t)a.B * a.n_tiles * a.N);
  } else {
    if (a.cls_r < 0 || i >= (int64_t)a.B * a.N) return;
    a.cls[i] = (double)total(a.part_cls, i, (int64_t)a.B * a.N);
  }
}

void launch_attn_qk(const ficoco_problem& p, const Plan& pl, char* ws, hipStream_t s) {
  QkArgs a{};
  a.Q = (const bf16_t*)p.Q; a.K = (const bf16_t*)p.K;
  a.sb = p.qk_stride_b; a.sh = p.qk_stride_h; a.sn = p.qk_stride_n;
  a.H = p.H; a.n = p.qk_n; a.N = p.N;
  a.vis0 = p.vis_begin - p.qk_begin;
  a.cls_r = p.sem_src == FICOCO_G_CLS_ATTN ? p.cls_index - p.qk_begin : -1;
  a.scale_log2e = p.qk_scale * 1.4426950408889634f;
  a.abar = (p.corr_src == FICOCO_C_ATTN && pl.n_disc > 0) ? (float*)(ws + pl.abar) : nullptr;
  a.map_pitch = pl.map_pitch;
  a.recv_part = (double*)(ws + pl.recv_part);
  a.cls = (double*)(ws + pl.cls);
  a.n_tiles = pl.n_chunks; a.B = p.B;
  a.q_begin = 0; a.q_count = p.qk_n;
  const bool L = p.variant == FICOCO_VARIANT_L;
  if (L) {                            // decoder: causal; the text queries follow the visual span
    const bool need_vv = p.red_src == FICOCO_R_ATTN_RECV || p.corr_src == FICOCO_C_ATTN;
    a.text0 = a.vis0 + p.N;
    a.M = p.M;
    a.ttext = (double*)(ws + pl.ttext);
    a.q_begin = need_vv ? a.vis0 : a.text0;
    a.q_count = need_vv ? p.N + p.M : p.M;
    if (!need_vv) a.recv_part = nullptr;
  }
  const dim3 grid(xcd_padded_total(a.n_tiles * a.B)), block(kQkWaves * kWave);
  if (L || p.qk_n > kQkMaxKeys) {     // keys in blocks, two sweeps
    // key groups per wavefront that cut the keys evenly over as many blocks as blocks of 640 would take
    const int blocks = (p.qk_n + kQkMaxKeys - 1) / kQkMaxKeys;
    // (heads of 128 always take three: with five the kernel spills 41 registers)
    const bool three = p.d_head == 128 || (p.qk_n + blocks * kQkWaves * 16 - 1) / (blocks * kQkWaves * 16) <= 3;
    a.groups = pl.qk_groups;
    a.heads_per_group = (p.H + a.groups - 1) / a.groups;
    if (a.groups > 1) {
      float* part = (float*)(ws + pl.qk_part);
      a.part_map = part;
      part += a.abar ? (size_t)a.groups * p.B * p.N * pl.map_pitch : 0;
      a.part_text = part;
      part += a.ttext ? (size_t)a.groups * p.B * p.N * p.M : 0;
      a.part_recv = part;
      part += (size_t)a.groups * p.B * a.n_tiles * p.N;
      a.part_cls = part;
    }
    const dim3 grid2(xcd_padded_total(a.n_tiles * a.B * a.groups));
    const size_t lds = (size_t)a.heads_per_group * kQkTile * 2 * sizeof(float);
    auto go = [&](auto kern) { hipLaunchKernelGGL(kern, grid2, block, lds, s, a); };
    const int ks = p.d_head / 32;       // (heads of 128 always take three key groups)
    if (L) {
      if (ks == 1) { if (three) go(attn_qk_long_kernel<1, 3, true>); else go(attn_qk_long_kernel<1, kQkKB, true>); }
      else if (ks == 2) { if (three) go(attn_qk_long_kernel<2, 3, true>); else go(attn_qk_long_kernel<2, kQkKB, true>); }
      else go(attn_qk_long_kernel<4, 3, true>);
    } else {
      if (ks == 1) { if (three) go(attn_qk_long_kernel<1, 3, false>); else go(attn_qk_long_kernel<1, kQkKB, false>); }
      else if (ks == 2) { if (three) go(attn_qk_long_kernel<2, 3, false>); else go(attn_qk_long_kernel<2, kQkKB, false>); }
      else go(attn_qk_long_kernel<4, 3, false>);
    }
    if (a.groups > 1) {
      auto blocks = [](int64_t n) { return (int)((n + 255) / 256); };
      QkCombineBlocks nb;
      nb.map = a.abar ? blocks((int64_t)p.B * p.N * p.N) : 0;
      nb.text = a.ttext ? blocks((int64_t)p.B * p.N * p.M) : 0;
      nb.recv = a.recv_part ? blocks((int64_t)p.B * a.n_tiles * p.N) : 0;
      nb.cls = a.cls_r >= 0 ? blocks((int64_t)p.B * p.N) : 0;
      const int all = nb.map + nb.text + nb.recv + nb.cls;
      if (all > 0) hipLaunchKernelGGL(qk_combine_kernel, dim3(all), dim3(256), 0, s, a, nb);
    }
    return;
  }
  switch (p.d_head / 32) {
    case 1: hipLaunchKernelGGL(attn_qk_kernel<1>, grid, block, 0, s, a); break;
    case 2: hipLaunchKernelGGL(attn_qk_kernel<2>, grid, block, 0, s, a); break;
    default: hipLaunchKernelGGL(attn_qk_kernel<4>, grid, block, 0, s, a); break;
  }
}

}  // namespace ficoco
