/*
 * vsa_oracle.c -- slow, plain CPU oracle for Video Sparse Attention (VSA).
 *
 * TEST INFRASTRUCTURE ONLY.  This file defines what the GPU library must compute; it is
 * called by the tests, by the smoke check and by the benchmark's CPU-baseline leg, and by
 * nothing else.  It shares no code with the HIP path and is deliberately naive: plain
 * loops, no blocking, no fusion, no reordering beyond what the definitions state.
 *
 * One source, two builds: -DREAL=double (fp64, used to pin the oracle against closed
 * forms / brute force / finite differences) and -DREAL=float (fp32, the precision the
 * GPU path's coarse stage decides its top-K in).
 *
 * What is computed (paper sections in brackets):
 *   geometry / tile map   [Sec. 2.2, cube partition and the index equation]
 *   mean pooling          [Sec. 2.2 coarse stage; App. B pseudocode "mean(dim=3)"]
 *   coarse attention      [Sec. 2.2: A_c = softmax(Q_c K_c^T / sqrt d), O_c = A_c V_c]
 *   row-wise top-K        [Sec. 2.2: top-K entries per row of A_c -> block index list]
 *   fine attention        [Sec. 2.1 attention equation with the block-sparse mask M]
 *   gated combine         [Sec. 2.2: O = O_c * G_c + O_f * G_f]
 *   backward              [Sec. 2.4 only says it exists; here: the chain rule applied to
 *                          the steps above with the index sets held constant]
 *
 * Readings taken where the paper is silent (same list as the design document):
 *   - top-K is taken on the coarse logits (softmax is monotone per row, same set);
 *     ties go to the lower cube index; the list is stored ascending.
 *   - grids that are not cube multiples are padded up; pad tokens are never keys, are
 *     excluded from pooled means (divide by the number of valid tokens), produce zero
 *     output rows and zero gradients.  Every cube of a padded grid holds >= 1 valid token.
 *   - a partially filled cube has the same weight in the coarse softmax as a full one.
 *   - gate_f == NULL means a gate of ones [Sec. 2.3].
 *   - no gradient flows through the top-K selection.
 *   - the 64 x 16 row of the tile-size tables [Sec. 3.2] is read as: query cubes (4,4,4), key cubes
 *     (2,4,2) nested in them (the table writes 16x64, the text 64 x 16; see the section on key
 *     cubes below).  A key cube with no valid token is dead: never in the softmax, never selected.
 *
 * Parity pins: see tests/test_oracle_*.py.  Unpinned by anything outside this file: the
 * pad conventions above that are ours by fiat (equal weighting of partial cubes in the
 * coarse softmax; zero rows for pad queries; and, with key cubes of 16 tokens, leaving a
 * dead key cube out of the coarse softmax) -- "parity unpinned" for those three.
 *
 * Layout: every tensor is [B,H,Np,d] in TILED order (each cube = Bk consecutive rows),
 * Np = padded token count, row-major, contiguous.  Pooled tensors are [B,H,Nc,d].
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef REAL
#define REAL double
#endif
typedef REAL real;

#define EXP(x) ((real)exp((double)(x)))
#define LOG(x) ((real)log((double)(x)))

static int cdiv(int a, int b) { return (a + b - 1) / b; }

typedef struct {
  int T, Hh, W;    /* valid grid */
  int Ct, Ch, Cw;  /* cube */
  int Nt, Nh, Nw;  /* cubes per axis of the padded grid */
  int Bk;          /* tokens per cube */
  int Nc;          /* cubes */
  int64_t Np;      /* padded tokens = Nc * Bk */
} grid_t;

static grid_t make_grid(int T, int Hh, int W, int Ct, int Ch, int Cw) {
  grid_t g;
  g.T = T; g.Hh = Hh; g.W = W; g.Ct = Ct; g.Ch = Ch; g.Cw = Cw;
  g.Nt = cdiv(T, Ct); g.Nh = cdiv(Hh, Ch); g.Nw = cdiv(W, Cw);
  g.Bk = Ct * Ch * Cw;
  g.Nc = g.Nt * g.Nh * g.Nw;
  g.Np = (int64_t)g.Nc * g.Bk;
  return g;
}

/* [Sec. 2.2, index equation]  n = (floor(t/Ct) Nh Nw + floor(h/Ch) Nw + floor(w/Cw)) B
 *                                 + (t mod Ct) Ch Cw + (h mod Ch) Cw + (w mod Cw)        */
static int64_t tiled_index(const grid_t* g, int t, int h, int w) {
  int64_t cube = (int64_t)(t / g->Ct) * g->Nh * g->Nw + (int64_t)(h / g->Ch) * g->Nw + (w / g->Cw);
  int64_t in = (int64_t)(t % g->Ct) * g->Ch * g->Cw + (int64_t)(h % g->Ch) * g->Cw + (w % g->Cw);
  return cube * g->Bk + in;
}

void vsa_oracle_dims(int T, int Hh, int W, int Ct, int Ch, int Cw, int64_t* Np, int32_t* Nc, int32_t* Bk) {
  grid_t g = make_grid(T, Hh, W, Ct, Ch, Cw);
  *Np = g.Np; *Nc = g.Nc; *Bk = g.Bk;
}

int64_t vsa_oracle_tiled_index(int T, int Hh, int W, int Ct, int Ch, int Cw, int t, int h, int w) {
  grid_t g = make_grid(T, Hh, W, Ct, Ch, Cw);
  return tiled_index(&g, t, h, w);
}

/* valid[n] = 1 iff tiled slot n holds a token of the valid grid; cnt[c] = valid tokens in cube c. */
void vsa_oracle_valid(int T, int Hh, int W, int Ct, int Ch, int Cw, uint8_t* valid, int32_t* cnt) {
  grid_t g = make_grid(T, Hh, W, Ct, Ch, Cw);
  memset(valid, 0, (size_t)g.Np);
  memset(cnt, 0, sizeof(int32_t) * (size_t)g.Nc);
  for (int t = 0; t < T; ++t)
    for (int h = 0; h < Hh; ++h)
      for (int w = 0; w < W; ++w) {
        int64_t n = tiled_index(&g, t, h, w);
        valid[n] = 1;
        cnt[n / g.Bk] += 1;
      }
}

/* Raster -> tiled permutation of `rows` independent [L,d] matrices of 16-bit elements
 * (inverse != 0: tiled -> raster).  Pad slots of the tiled tensor are zero-filled.
 * [Sec. 2.2 index equation; App. B tile()/untile()] */
void vsa_oracle_tile_u16(int T, int Hh, int W, int Ct, int Ch, int Cw, int64_t rows, int d,
                         const uint16_t* src, uint16_t* dst, int inverse) {
  grid_t g = make_grid(T, Hh, W, Ct, Ch, Cw);
  int64_t L = (int64_t)T * Hh * W;
  if (!inverse) memset(dst, 0, sizeof(uint16_t) * (size_t)(rows * g.Np * d));
  for (int64_t r = 0; r < rows; ++r)
    for (int t = 0; t < T; ++t)
      for (int h = 0; h < Hh; ++h)
        for (int w = 0; w < W; ++w) {
          int64_t n_r = ((int64_t)t * Hh + h) * W + w; /* [Sec. 2.1] n = tHW + hW + w */
          int64_t n_t = tiled_index(&g, t, h, w);
          const uint16_t* s = inverse ? src + (r * g.Np + n_t) * d : src + (r * L + n_r) * d;
          uint16_t* o = inverse ? dst + (r * L + n_r) * d : dst + (r * g.Np + n_t) * d;
          memcpy(o, s, sizeof(uint16_t) * (size_t)d);
        }
}

/* ------------------------------------------------------------------------------------ */
/* Per-(b,h) building blocks                                                            */
/* ------------------------------------------------------------------------------------ */

/* Mean over the valid tokens of every cube.  x: [Np,d] -> xc: [Nc,d] */
static void pool_mean(const grid_t* g, int d, const uint8_t* valid, const int32_t* cnt, const real* x, real* xc) {
  for (int c = 0; c < g->Nc; ++c)
    for (int e = 0; e < d; ++e) {
      real s = 0;
      for (int p = 0; p < g->Bk; ++p) {
        int64_t n = (int64_t)c * g->Bk + p;
        if (valid[n]) s += x[n * d + e];
      }
      xc[(int64_t)c * d + e] = s / (real)cnt[c];
    }
}

/* Coarse logits row c: Sc[c,j] = scale * Qc[c] . Kc[j] */
static void coarse_logits_row(const grid_t* g, int d, real scale, const real* Qc, const real* Kc, int c, real* row) {
  for (int j = 0; j < g->Nc; ++j) {
    real s = 0;
    for (int e = 0; e < d; ++e) s += Qc[(int64_t)c * d + e] * Kc[(int64_t)j * d + e];
    row[j] = s * scale;
  }
}

/* softmax over a row of n logits; returns logsumexp */
static real softmax_row(int n, const real* logits, real* prob) {
  real m = logits[0];
  for (int j = 1; j < n; ++j) if (logits[j] > m) m = logits[j];
  real l = 0;
  for (int j = 0; j < n; ++j) { prob[j] = EXP(logits[j] - m); l += prob[j]; }
  for (int j = 0; j < n; ++j) prob[j] /= l;
  return m + LOG(l);
}

typedef struct { real v; int32_t i; } vi_t;
static int cmp_vi(const void* a, const void* b) {
  const vi_t* x = (const vi_t*)a; const vi_t* y = (const vi_t*)b;
  if (x->v > y->v) return -1;
  if (x->v < y->v) return 1;
  return (x->i < y->i) ? -1 : (x->i > y->i);
}
static int cmp_i32(const void* a, const void* b) {
  int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
  return (x < y) ? -1 : (x > y);
}
/* The K largest logits of a row, ties to the lower index, emitted in ascending index order. */
static void topk_row(int n, const real* logits, int K, int32_t* idx) {
  vi_t* a = (vi_t*)malloc(sizeof(vi_t) * (size_t)n);
  for (int j = 0; j < n; ++j) { a[j].v = logits[j]; a[j].i = j; }
  qsort(a, (size_t)n, sizeof(vi_t), cmp_vi);
  for (int r = 0; r < K; ++r) idx[r] = a[r].i;
  qsort(idx, (size_t)K, sizeof(int32_t), cmp_i32);
  free(a);
}

/* Fine attention of ONE query token i over the valid tokens of the selected key cubes.
 * Returns lse; writes of[d]; if p != NULL stores the probabilities in list order
 * (K*Bk entries, 0 for pad keys). */
static real fine_row(const grid_t* g, int d, real scale, const uint8_t* valid, const real* q, const real* k,
                     const real* v, int64_t i, const int32_t* idx, int K, real* of, real* p_out) {
  int64_t nkeys = (int64_t)K * g->Bk;
  real* s = (real*)malloc(sizeof(real) * (size_t)nkeys);
  real m = -INFINITY;
  for (int r = 0; r < K; ++r)
    for (int p = 0; p < g->Bk; ++p) {
      int64_t j = (int64_t)idx[r] * g->Bk + p;
      real acc = -INFINITY;
      if (valid[j]) {
        acc = 0;
        for (int e = 0; e < d; ++e) acc += q[i * d + e] * k[j * d + e];
        acc *= scale;
        if (acc > m) m = acc;
      }
      s[(int64_t)r * g->Bk + p] = acc;
    }
  real l = 0;
  for (int64_t x = 0; x < nkeys; ++x) { s[x] = (s[x] == -INFINITY) ? (real)0 : EXP(s[x] - m); l += s[x]; }
  for (int e = 0; e < d; ++e) of[e] = 0;
  for (int r = 0; r < K; ++r)
    for (int p = 0; p < g->Bk; ++p) {
      int64_t j = (int64_t)idx[r] * g->Bk + p;
      real pj = s[(int64_t)r * g->Bk + p] / l;
      if (p_out) p_out[(int64_t)r * g->Bk + p] = pj;
      if (pj != 0)
        for (int e = 0; e < d; ++e) of[e] += pj * v[j * d + e];
    }
  free(s);
  return m + LOG(l);
}

/* ------------------------------------------------------------------------------------ */
/* Forward                                                                              */
/* ------------------------------------------------------------------------------------ */
/*
 * q,k,v,gate_c,gate_f: [B,H,Np,d] tiled (gate_f may be NULL = ones).
 * cubes/ncubes: optional subset of query cubes to evaluate (NULL = all); with a subset
 *   only those cubes' rows of out/out_fine/lse_fine/block_idx/out_coarse/lse_coarse/sc
 *   are written.
 * indices_given != 0: block_idx [B,H,Nc,topk] is an input (ascending, distinct).
 * sc (optional): coarse logits [B,H,Nc,Nc].
 * Any output pointer may be NULL.  Returns 0, or -1 on a bad argument.
 */
int vsa_oracle_forward(int B, int H, int T, int Hh, int W, int Ct, int Ch, int Cw, int d, int topk, double scale_,
                       int indices_given, const real* q, const real* k, const real* v, const real* gate_c,
                       const real* gate_f, const int32_t* cubes, int ncubes, real* out, int32_t* block_idx,
                       real* out_fine, real* lse_fine, real* out_coarse, real* lse_coarse, real* sc) {
  grid_t g = make_grid(T, Hh, W, Ct, Ch, Cw);
  if (B < 1 || H < 1 || d < 1 || topk < 1 || topk > g.Nc) return -1;
  if (indices_given && !block_idx) return -1;
  real scale = (real)scale_;
  uint8_t* valid = (uint8_t*)malloc((size_t)g.Np);
  int32_t* cnt = (int32_t*)malloc(sizeof(int32_t) * (size_t)g.Nc);
  vsa_oracle_valid(T, Hh, W, Ct, Ch, Cw, valid, cnt);
  int nq = cubes ? ncubes : g.Nc;

  for (int bh = 0; bh < B * H; ++bh) {
    const real* qh = q + (int64_t)bh * g.Np * d;
    const real* kh = k + (int64_t)bh * g.Np * d;
    const real* vh = v + (int64_t)bh * g.Np * d;
    real* Qc = (real*)malloc(sizeof(real) * (size_t)g.Nc * d);
    real* Kc = (real*)malloc(sizeof(real) * (size_t)g.Nc * d);
    real* Vc = (real*)malloc(sizeof(real) * (size_t)g.Nc * d);
    pool_mean(&g, d, valid, cnt, qh, Qc);
    pool_mean(&g, d, valid, cnt, kh, Kc);
    pool_mean(&g, d, valid, cnt, vh, Vc);

#pragma omp parallel for schedule(dynamic, 1)
    for (int ci = 0; ci < nq; ++ci) {
      int c = cubes ? cubes[ci] : ci;
      real* row = (real*)malloc(sizeof(real) * (size_t)g.Nc);
      real* prob = (real*)malloc(sizeof(real) * (size_t)g.Nc);
      real* oc = (real*)malloc(sizeof(real) * (size_t)d);
      real* of = (real*)malloc(sizeof(real) * (size_t)d);
      int32_t* idx = (int32_t*)malloc(sizeof(int32_t) * (size_t)topk);

      /* coarse stage */
      coarse_logits_row(&g, d, scale, Qc, Kc, c, row);
      real lse_c = softmax_row(g.Nc, row, prob);
      for (int e = 0; e < d; ++e) {
        real s = 0;
        for (int j = 0; j < g.Nc; ++j) s += prob[j] * Vc[(int64_t)j * d + e];
        oc[e] = s;
      }
      if (sc) memcpy(sc + ((int64_t)bh * g.Nc + c) * g.Nc, row, sizeof(real) * (size_t)g.Nc);
      if (out_coarse) memcpy(out_coarse + ((int64_t)bh * g.Nc + c) * d, oc, sizeof(real) * (size_t)d);
      if (lse_coarse) lse_coarse[(int64_t)bh * g.Nc + c] = lse_c;

      /* selection */
      if (indices_given) memcpy(idx, block_idx + ((int64_t)bh * g.Nc + c) * topk, sizeof(int32_t) * (size_t)topk);
      else {
        topk_row(g.Nc, row, topk, idx);
        if (block_idx) memcpy(block_idx + ((int64_t)bh * g.Nc + c) * topk, idx, sizeof(int32_t) * (size_t)topk);
      }

      /* fine stage + gated combine, token by token */
      for (int p = 0; p < g.Bk; ++p) {
        int64_t i = (int64_t)c * g.Bk + p;
        int64_t gi = ((int64_t)bh * g.Np + i) * d;
        if (!valid[i]) {
          for (int e = 0; e < d; ++e) {
            if (out) out[gi + e] = 0;
            if (out_fine) out_fine[gi + e] = 0;
          }
          if (lse_fine) lse_fine[(int64_t)bh * g.Np + i] = 0;
          continue;
        }
        real lse = fine_row(&g, d, scale, valid, qh, kh, vh, i, idx, topk, of, NULL);
        if (lse_fine) lse_fine[(int64_t)bh * g.Np + i] = lse;
        for (int e = 0; e < d; ++e) {
          if (out_fine) out_fine[gi + e] = of[e];
          if (out) {
            real gfv = gate_f ? gate_f[gi + e] : (real)1;
            out[gi + e] = oc[e] * gate_c[gi + e] + of[e] * gfv;
          }
        }
      }
      free(row); free(prob); free(oc); free(of); free(idx);
    }
    free(Qc); free(Kc); free(Vc);
  }
  free(valid); free(cnt);
  return 0;
}

/* ------------------------------------------------------------------------------------ */
/* Mismatched granularity [Sec. 3.2, paragraph after the tile-size tables]              */
/* ------------------------------------------------------------------------------------ */
/*
 * The coarse stage pools over (Ct,Ch,Cw) cubes while the fine stage attends in tiles of (1,2,2)
 * cubes, i.e. (Ct,2Ch,2Cw) tokens: the coarse stage's attention map A_c [Nc x Nc] is average-pooled
 * over the 2x2 groups of cubes, on the query and on the key axis, and the top-K is taken on the
 * pooled map [Ns x Ns] (ties to the lower tile index).  Everything else (pooled tensors, O_c, the
 * gated sum) stays at cube granularity.  Needs even numbers of cubes along h and w.
 *
 * Per (b,h):  tile_idx [Ns, topk]      the selected key tiles of every query tile, ascending;
 *             cube_idx [Nc, 4*topk]    the same selection as a list of key cubes for every query
 *                                      cube (all four cubes of each selected tile), ascending: the
 *                                      form vsa_oracle_forward / _backward take as block_idx;
 *             pooled   [Ns, Ns]        the pooled map (may be NULL).
 * Tile (st,sh,sw) has index (st*Nh/2 + sh)*Nw/2 + sw and holds cubes (st, 2sh+a, 2sw+b), a,b in {0,1}.
 */
int vsa_oracle_select_pooled(int B, int H, int T, int Hh, int W, int Ct, int Ch, int Cw, int d, int topk, double scale_,
                             const real* q, const real* k, int32_t* tile_idx, int32_t* cube_idx, real* pooled) {
  grid_t g = make_grid(T, Hh, W, Ct, Ch, Cw);
  if (g.Nh % 2 || g.Nw % 2) return -1;
  const int Nc = g.Nc, Sh = g.Nh / 2, Sw = g.Nw / 2, Ns = g.Nt * Sh * Sw;
  if (B < 1 || H < 1 || d < 1 || topk < 1 || topk > Ns || !tile_idx || !cube_idx) return -1;
  real scale = (real)scale_;
  uint8_t* valid = (uint8_t*)malloc((size_t)g.Np);
  int32_t* cnt = (int32_t*)malloc(sizeof(int32_t) * (size_t)Nc);
  vsa_oracle_valid(T, Hh, W, Ct, Ch, Cw, valid, cnt);
  for (int bh = 0; bh < B * H; ++bh) {
    const real* qh = q + (int64_t)bh * g.Np * d;
    const real* kh = k + (int64_t)bh * g.Np * d;
    real* Qc = (real*)malloc(sizeof(real) * (size_t)Nc * d);
    real* Kc = (real*)malloc(sizeof(real) * (size_t)Nc * d);
    real* Ac = (real*)malloc(sizeof(real) * (size_t)Nc * Nc);
    real* Ps = (real*)calloc((size_t)Ns * Ns, sizeof(real));
    real* row = (real*)malloc(sizeof(real) * (size_t)Nc);
    pool_mean(&g, d, valid, cnt, qh, Qc);
    pool_mean(&g, d, valid, cnt, kh, Kc);
    for (int c = 0; c < Nc; ++c) {
      coarse_logits_row(&g, d, scale, Qc, Kc, c, row);
      softmax_row(Nc, row, Ac + (int64_t)c * Nc);
    }
    /* average over the 2x2 cubes of the query tile and the 2x2 cubes of the key tile */
    for (int c = 0; c < Nc; ++c) {
      int cw = c % g.Nw, ch = (c / g.Nw) % g.Nh, ct = c / (g.Nw * g.Nh);
      int sq = (ct * Sh + ch / 2) * Sw + cw / 2;
      for (int j = 0; j < Nc; ++j) {
        int jw = j % g.Nw, jh = (j / g.Nw) % g.Nh, jt = j / (g.Nw * g.Nh);
        int sk = (jt * Sh + jh / 2) * Sw + jw / 2;
        Ps[(int64_t)sq * Ns + sk] += Ac[(int64_t)c * Nc + j] / (real)16;
      }
    }
    int32_t* tl = tile_idx + (int64_t)bh * Ns * topk;
    for (int s = 0; s < Ns; ++s) topk_row(Ns, Ps + (int64_t)s * Ns, topk, tl + (int64_t)s * topk);
    for (int c = 0; c < Nc; ++c) {
      int cw = c % g.Nw, ch = (c / g.Nw) % g.Nh, ct = c / (g.Nw * g.Nh);
      int sq = (ct * Sh + ch / 2) * Sw + cw / 2;
      int32_t* out = cube_idx + ((int64_t)bh * Nc + c) * 4 * topk;
      for (int r = 0; r < topk; ++r) {
        int s = tl[(int64_t)sq * topk + r];
        int sw = s % Sw, sh = (s / Sw) % Sh, st = s / (Sw * Sh);
        for (int a = 0; a < 2; ++a)
          for (int b = 0; b < 2; ++b) out[4 * r + 2 * a + b] = (st * g.Nh + 2 * sh + a) * g.Nw + 2 * sw + b;
      }
      qsort(out, (size_t)(4 * topk), sizeof(int32_t), cmp_i32);
    }
    if (pooled) memcpy(pooled + (int64_t)bh * Ns * Ns, Ps, sizeof(real) * (size_t)Ns * Ns);
    free(Qc); free(Kc); free(Ac); free(Ps); free(row);
  }
  free(valid); free(cnt);
  return 0;
}

/* ------------------------------------------------------------------------------------ */
/* Selection-quality diagnostic [Sec. 3.5]                                              */
/* ------------------------------------------------------------------------------------ */
/*
 * Sec. 3.5 asks how much of the dense attention a set of key cubes captures: the sum of the dense
 * attention scores that fall inside the cubes, averaged over query tokens.  For ONE (b, h) slice
 * this returns the whole cube-by-cube table
 *   mass[c][j] = (1 / cnt_c) sum_{valid i in cube c} sum_{valid n in cube j} A_in,
 *   A = softmax over all valid keys of q_i . k_n * scale            [Sec. 2.1 attention equation]
 * so that rows sum to 1 and the mass captured by any selection is a sum of K entries of a row.
 * q, k: [Np, d] tiled.  Plain token loops.
 */
int vsa_oracle_block_mass(int T, int Hh, int W, int Ct, int Ch, int Cw, int d, double scale_, const real* q,
                          const real* k, real* mass) {
  grid_t g = make_grid(T, Hh, W, Ct, Ch, Cw);
  if (d < 1 || !q || !k || !mass) return -1;
  real scale = (real)scale_;
  uint8_t* valid = (uint8_t*)malloc((size_t)g.Np);
  int32_t* cnt = (int32_t*)malloc(sizeof(int32_t) * (size_t)g.Nc);
  vsa_oracle_valid(T, Hh, W, Ct, Ch, Cw, valid, cnt);
  const int Nc = g.Nc, Bk = g.Bk;
  for (int64_t x = 0; x < (int64_t)Nc * Nc; ++x) mass[x] = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int c = 0; c < Nc; ++c) {
    real* s = (real*)malloc(sizeof(real) * (size_t)g.Np);
    for (int p = 0; p < Bk; ++p) {
      int64_t i = (int64_t)c * Bk + p;
      if (!valid[i]) continue;
      real m = -INFINITY, l = 0;
      for (int64_t n = 0; n < g.Np; ++n) {
        if (!valid[n]) continue;
        real acc = 0;
        for (int e = 0; e < d; ++e) acc += q[i * d + e] * k[n * d + e];
        s[n] = acc * scale;
        if (s[n] > m) m = s[n];
      }
      for (int64_t n = 0; n < g.Np; ++n)
        if (valid[n]) { s[n] = EXP(s[n] - m); l += s[n]; }
      for (int64_t n = 0; n < g.Np; ++n)
        if (valid[n]) mass[(int64_t)c * Nc + n / Bk] += s[n] / l / (real)cnt[c];
    }
    free(s);
  }
  free(valid); free(cnt);
  return 0;
}

/* ------------------------------------------------------------------------------------ */
/* Backward                                                                             */
/* ------------------------------------------------------------------------------------ */
/*
 * Gradients of L = sum(out * dout) w.r.t. q,k,v,gate_c,gate_f with block_idx held fixed.
 * Everything the forward produced is recomputed here from the inputs; nothing saved by
 * a forward call is trusted.  dgate_f may be NULL (and must be when gate_f is NULL).
 *
 *   dGc_i = dO_i * Oc[c(i)]          dGf_i = dO_i * Of_i
 *   dOc[c] = sum_{i in c} dO_i * Gc_i (a sum, not a mean)       dOf_i = dO_i * Gf_i
 *   fine:   P_ij = exp(S_ij - lse_i), dP_ij = dOf_i . v_j, D_i = dOf_i . Of_i,
 *           dS_ij = P_ij (dP_ij - D_i),
 *           dQ_i = scale sum_j dS_ij k_j, dK_j = scale sum_i dS_ij q_i, dV_j = sum_i P_ij dOf_i
 *   coarse: dVc_j = sum_c Ac[c,j] dOc[c], dAc[c,j] = dOc[c] . Vc[j],
 *           dSc[c,j] = Ac[c,j] (dAc[c,j] - sum_j' Ac[c,j'] dAc[c,j']),
 *           dQc[c] = scale sum_j dSc[c,j] Kc[j], dKc[j] = scale sum_c dSc[c,j] Qc[c]
 *   pooling: every valid token of cube c receives dXc[c] / cnt_c.
 */
int vsa_oracle_backward(int B, int H, int T, int Hh, int W, int Ct, int Ch, int Cw, int d, int topk, double scale_,
                        const real* q, const real* k, const real* v, const real* gate_c, const real* gate_f,
                        const real* dout, const int32_t* block_idx, real* dq, real* dk, real* dv, real* dgate_c,
                        real* dgate_f) {
  grid_t g = make_grid(T, Hh, W, Ct, Ch, Cw);
  if (B < 1 || H < 1 || d < 1 || topk < 1 || topk > g.Nc || !block_idx) return -1;
  real scale = (real)scale_;
  uint8_t* valid = (uint8_t*)malloc((size_t)g.Np);
  int32_t* cnt = (int32_t*)malloc(sizeof(int32_t) * (size_t)g.Nc);
  vsa_oracle_valid(T, Hh, W, Ct, Ch, Cw, valid, cnt);
  const int Nc = g.Nc, Bk = g.Bk;
  const int64_t Np = g.Np;

  for (int bh = 0; bh < B * H; ++bh) {
    const int64_t off = (int64_t)bh * Np * d;
    const real *qh = q + off, *kh = k + off, *vh = v + off, *gch = gate_c + off, *doh = dout + off;
    const real* gfh = gate_f ? gate_f + off : NULL;
    const int32_t* idxh = block_idx + (int64_t)bh * Nc * topk;
    real *dqh = dq + off, *dkh = dk + off, *dvh = dv + off, *dgch = dgate_c + off;
    real* dgfh = dgate_f ? dgate_f + off : NULL;

    real* Qc = (real*)malloc(sizeof(real) * (size_t)Nc * d);
    real* Kc = (real*)malloc(sizeof(real) * (size_t)Nc * d);
    real* Vc = (real*)malloc(sizeof(real) * (size_t)Nc * d);
    real* Ac = (real*)malloc(sizeof(real) * (size_t)Nc * Nc);
    real* Oc = (real*)calloc((size_t)Nc * d, sizeof(real));
    real* Of = (real*)calloc((size_t)Np * d, sizeof(real));
    real* lse = (real*)calloc((size_t)Np, sizeof(real));
    real* dOf = (real*)calloc((size_t)Np * d, sizeof(real));
    real* Dl = (real*)calloc((size_t)Np, sizeof(real));
    real* dOc = (real*)calloc((size_t)Nc * d, sizeof(real));
    real* dSc = (real*)malloc(sizeof(real) * (size_t)Nc * Nc);
    real* dQc = (real*)calloc((size_t)Nc * d, sizeof(real));
    real* dKc = (real*)calloc((size_t)Nc * d, sizeof(real));
    real* dVc = (real*)calloc((size_t)Nc * d, sizeof(real));

    /* recompute the forward */
    pool_mean(&g, d, valid, cnt, qh, Qc);
    pool_mean(&g, d, valid, cnt, kh, Kc);
    pool_mean(&g, d, valid, cnt, vh, Vc);
#pragma omp parallel for schedule(dynamic, 1)
    for (int c = 0; c < Nc; ++c) {
      real* row = (real*)malloc(sizeof(real) * (size_t)Nc);
      coarse_logits_row(&g, d, scale, Qc, Kc, c, row);
      softmax_row(Nc, row, Ac + (int64_t)c * Nc);
      for (int e = 0; e < d; ++e) {
        real s = 0;
        for (int j = 0; j < Nc; ++j) s += Ac[(int64_t)c * Nc + j] * Vc[(int64_t)j * d + e];
        Oc[(int64_t)c * d + e] = s;
      }
      for (int p = 0; p < Bk; ++p) {
        int64_t i = (int64_t)c * Bk + p;
        if (valid[i]) lse[i] = fine_row(&g, d, scale, valid, qh, kh, vh, i, idxh + (int64_t)c * topk, topk, Of + i * d, NULL);
      }
      free(row);
    }

    /* gates, dOf, D, dOc */
    for (int c = 0; c < Nc; ++c)
      for (int p = 0; p < Bk; ++p) {
        int64_t i = (int64_t)c * Bk + p;
        for (int e = 0; e < d; ++e) {
          if (!valid[i]) {
            dgch[i * d + e] = 0;
            if (dgfh) dgfh[i * d + e] = 0;
            continue;
          }
          real go = doh[i * d + e];
          dgch[i * d + e] = go * Oc[(int64_t)c * d + e];
          if (dgfh) dgfh[i * d + e] = go * Of[i * d + e];
          dOc[(int64_t)c * d + e] += go * gch[i * d + e];
          dOf[i * d + e] = go * (gfh ? gfh[i * d + e] : (real)1);
          Dl[i] += dOf[i * d + e] * Of[i * d + e];
        }
      }

    /* fine backward, dQ: one query token at a time */
#pragma omp parallel for schedule(dynamic, 1)
    for (int c = 0; c < Nc; ++c)
      for (int p = 0; p < Bk; ++p) {
        int64_t i = (int64_t)c * Bk + p;
        for (int e = 0; e < d; ++e) dqh[i * d + e] = 0;
        if (!valid[i]) continue;
        for (int r = 0; r < topk; ++r)
          for (int pk = 0; pk < Bk; ++pk) {
            int64_t j = (int64_t)idxh[(int64_t)c * topk + r] * Bk + pk;
            if (!valid[j]) continue;
            real s = 0, dp = 0;
            for (int e = 0; e < d; ++e) { s += qh[i * d + e] * kh[j * d + e]; dp += dOf[i * d + e] * vh[j * d + e]; }
            real P = EXP(s * scale - lse[i]);
            real dS = P * (dp - Dl[i]);
            for (int e = 0; e < d; ++e) dqh[i * d + e] += scale * dS * kh[j * d + e];
          }
      }

    /* fine backward, dK and dV: one key cube at a time, over the query cubes that selected it */
#pragma omp parallel for schedule(dynamic, 1)
    for (int jc = 0; jc < Nc; ++jc) {
      for (int pk = 0; pk < Bk; ++pk)
        for (int e = 0; e < d; ++e) { dkh[((int64_t)jc * Bk + pk) * d + e] = 0; dvh[((int64_t)jc * Bk + pk) * d + e] = 0; }
      for (int c = 0; c < Nc; ++c) {
        int sel = 0;
        for (int r = 0; r < topk; ++r) if (idxh[(int64_t)c * topk + r] == jc) sel = 1;
        if (!sel) continue;
        for (int p = 0; p < Bk; ++p) {
          int64_t i = (int64_t)c * Bk + p;
          if (!valid[i]) continue;
          for (int pk = 0; pk < Bk; ++pk) {
            int64_t j = (int64_t)jc * Bk + pk;
            if (!valid[j]) continue;
            real s = 0, dp = 0;
            for (int e = 0; e < d; ++e) { s += qh[i * d + e] * kh[j * d + e]; dp += dOf[i * d + e] * vh[j * d + e]; }
            real P = EXP(s * scale - lse[i]);
            real dS = P * (dp - Dl[i]);
            for (int e = 0; e < d; ++e) {
              dkh[j * d + e] += scale * dS * qh[i * d + e];
              dvh[j * d + e] += P * dOf[i * d + e];
            }
          }
        }
      }
    }

    /* coarse backward */
    for (int c = 0; c < Nc; ++c) {
      real dot = 0;
      for (int j = 0; j < Nc; ++j) {
        real dA = 0;
        for (int e = 0; e < d; ++e) dA += dOc[(int64_t)c * d + e] * Vc[(int64_t)j * d + e];
        dSc[(int64_t)c * Nc + j] = dA; /* holds dAc for the moment */
        dot += Ac[(int64_t)c * Nc + j] * dA;
      }
      for (int j = 0; j < Nc; ++j) dSc[(int64_t)c * Nc + j] = Ac[(int64_t)c * Nc + j] * (dSc[(int64_t)c * Nc + j] - dot);
    }
    for (int c = 0; c < Nc; ++c)
      for (int j = 0; j < Nc; ++j)
        for (int e = 0; e < d; ++e) {
          dVc[(int64_t)j * d + e] += Ac[(int64_t)c * Nc + j] * dOc[(int64_t)c * d + e];
          dQc[(int64_t)c * d + e] += scale * dSc[(int64_t)c * Nc + j] * Kc[(int64_t)j * d + e];
          dKc[(int64_t)j * d + e] += scale * dSc[(int64_t)c * Nc + j] * Qc[(int64_t)c * d + e];
        }

    /* pooling backward: the mean spreads 1/cnt to each valid token */
    for (int c = 0; c < Nc; ++c)
      for (int p = 0; p < Bk; ++p) {
        int64_t i = (int64_t)c * Bk + p;
        if (!valid[i]) continue;
        for (int e = 0; e < d; ++e) {
          dqh[i * d + e] += dQc[(int64_t)c * d + e] / (real)cnt[c];
          dkh[i * d + e] += dKc[(int64_t)c * d + e] / (real)cnt[c];
          dvh[i * d + e] += dVc[(int64_t)c * d + e] / (real)cnt[c];
        }
      }

    free(Qc); free(Kc); free(Vc); free(Ac); free(Oc); free(Of); free(lse); free(dOf); free(Dl);
    free(dOc); free(dSc); free(dQc); free(dKc); free(dVc);
  }
  free(valid); free(cnt);
  return 0;
}

/* ------------------------------------------------------------------------------------ */
/* Key cubes smaller than query cubes [Sec. 3.2, tile-size tables: the 64 x 16 row]      */
/* ------------------------------------------------------------------------------------ */
/*
 * Reading: queries keep the (Ct,Ch,Cw) cubes and their token order; keys are grouped in smaller
 * (Kt,Kh,Kw) cubes that divide the query cube (B=16: (2,4,2) inside (4,4,4)).  The coarse stage
 * pools Q over query cubes and K, V over key cubes, its map is [Nc x Nk], the top-K of a row
 * names key cubes, and a query token attends to the valid tokens of the key cubes its cube
 * selected.  Key cube numbering: R = (Ct/Kt)(Ch/Kh)(Cw/Kw) key cubes per query cube,
 *   label(t,h,w) = cube(t,h,w) * R + (((t mod Ct)/Kt) (Ch/Kh) + (h mod Ch)/Kh) (Cw/Kw) + (w mod Cw)/Kw.
 * A key cube of a padded grid may hold no valid token at all: it is then DEAD -- its pooled
 * rows are zero, it is left out of the coarse softmax and it is never selected (topk must not
 * exceed the number of live key cubes).
 * With (Kt,Kh,Kw) == (Ct,Ch,Cw) everything here is the ordinary method.
 */
typedef struct {
  grid_t g;
  int R, Nk;
  int32_t* label;  /* [Np] key cube of each tiled slot, -1 for a pad slot */
  int32_t* kcnt;   /* [Nk] valid tokens per key cube */
  int64_t* first;  /* [Nk+1] members of key cube j: member[first[j] .. first[j+1]) */
  int64_t* member; /* tiled slots of the valid tokens, grouped by key cube */
  uint8_t* valid;  /* [Np] */
  int32_t* qcnt;   /* [Nc] valid tokens per query cube */
} kq_t;

static int kq_make(kq_t* x, int T, int Hh, int W, int Ct, int Ch, int Cw, int Kt, int Kh, int Kw) {
  if (Kt < 1 || Kh < 1 || Kw < 1 || Ct % Kt || Ch % Kh || Cw % Kw) return -1;
  x->g = make_grid(T, Hh, W, Ct, Ch, Cw);
  const grid_t* g = &x->g;
  x->R = (Ct / Kt) * (Ch / Kh) * (Cw / Kw);
  x->Nk = g->Nc * x->R;
  x->label = (int32_t*)malloc(sizeof(int32_t) * (size_t)g->Np);
  x->kcnt = (int32_t*)calloc((size_t)x->Nk, sizeof(int32_t));
  x->first = (int64_t*)calloc((size_t)x->Nk + 1, sizeof(int64_t));
  x->member = (int64_t*)malloc(sizeof(int64_t) * (size_t)g->Np);
  x->valid = (uint8_t*)malloc((size_t)g->Np);
  x->qcnt = (int32_t*)malloc(sizeof(int32_t) * (size_t)g->Nc);
  vsa_oracle_valid(T, Hh, W, Ct, Ch, Cw, x->valid, x->qcnt);
  for (int64_t n = 0; n < g->Np; ++n) x->label[n] = -1;
  for (int t = 0; t < T; ++t)
    for (int h = 0; h < Hh; ++h)
      for (int w = 0; w < W; ++w) {
        int64_t n = tiled_index(g, t, h, w);
        int local = (((t % Ct) / Kt) * (Ch / Kh) + (h % Ch) / Kh) * (Cw / Kw) + (w % Cw) / Kw;
        x->label[n] = (int32_t)(n / g->Bk) * x->R + local;
        x->kcnt[x->label[n]] += 1;
      }
  for (int j = 0; j < x->Nk; ++j) x->first[j + 1] = x->first[j] + x->kcnt[j];
  int64_t* fill = (int64_t*)malloc(sizeof(int64_t) * (size_t)x->Nk);
  memcpy(fill, x->first, sizeof(int64_t) * (size_t)x->Nk);
  for (int64_t n = 0; n < g->Np; ++n)
    if (x->label[n] >= 0) x->member[fill[x->label[n]]++] = n;
  free(fill);
  return 0;
}
static void kq_free(kq_t* x) {
  free(x->label); free(x->kcnt); free(x->first); free(x->member); free(x->valid); free(x->qcnt);
}

/* label [Np] (-1 on pad slots) and kcnt [Nk] of the key-cube partition; returns Nk, or -1 */
int vsa_oracle_keycubes(int T, int Hh, int W, int Ct, int Ch, int Cw, int Kt, int Kh, int Kw, int32_t* label,
                        int32_t* kcnt) {
  kq_t x;
  if (kq_make(&x, T, Hh, W, Ct, Ch, Cw, Kt, Kh, Kw)) return -1;
  if (label) memcpy(label, x.label, sizeof(int32_t) * (size_t)x.g.Np);
  if (kcnt) memcpy(kcnt, x.kcnt, sizeof(int32_t) * (size_t)x.Nk);
  int Nk = x.Nk;
  kq_free(&x);
  return Nk;
}

/* mean over the valid tokens of every key cube (zero rows for dead ones).  x: [Np,d] -> xc: [Nk,d] */
static void kq_pool_keys(const kq_t* x, int d, const real* in, real* xc) {
  for (int j = 0; j < x->Nk; ++j)
    for (int e = 0; e < d; ++e) {
      real s = 0;
      for (int64_t m = x->first[j]; m < x->first[j + 1]; ++m) s += in[x->member[m] * d + e];
      xc[(int64_t)j * d + e] = x->kcnt[j] ? s / (real)x->kcnt[j] : (real)0;
    }
}
/* coarse logits of query cube c against every key cube; -inf for dead key cubes */
static void kq_logits_row(const kq_t* x, int d, real scale, const real* Qc, const real* Kc, int c, real* row) {
  for (int j = 0; j < x->Nk; ++j) {
    real s = 0;
    for (int e = 0; e < d; ++e) s += Qc[(int64_t)c * d + e] * Kc[(int64_t)j * d + e];
    row[j] = x->kcnt[j] ? s * scale : -INFINITY;
  }
}
/* softmax over a row that may hold -inf entries (they get probability 0); returns logsumexp */
static real kq_softmax_row(int n, const real* logits, real* prob) {
  real m = -INFINITY;
  for (int j = 0; j < n; ++j) if (logits[j] > m) m = logits[j];
  real l = 0;
  for (int j = 0; j < n; ++j) { prob[j] = (logits[j] == -INFINITY) ? (real)0 : EXP(logits[j] - m); l += prob[j]; }
  for (int j = 0; j < n; ++j) prob[j] /= l;
  return m + LOG(l);
}
/* fine attention of query token i over the valid tokens of the K listed key cubes; returns lse */
static real kq_fine_row(const kq_t* x, int d, real scale, const real* q, const real* k, const real* v, int64_t i,
                        const int32_t* idx, int K, real* of) {
  real m = -INFINITY;
  for (int r = 0; r < K; ++r)
    for (int64_t mm = x->first[idx[r]]; mm < x->first[idx[r] + 1]; ++mm) {
      int64_t j = x->member[mm];
      real acc = 0;
      for (int e = 0; e < d; ++e) acc += q[i * d + e] * k[j * d + e];
      acc *= scale;
      if (acc > m) m = acc;
    }
  real l = 0;
  for (int e = 0; e < d; ++e) of[e] = 0;
  for (int r = 0; r < K; ++r)
    for (int64_t mm = x->first[idx[r]]; mm < x->first[idx[r] + 1]; ++mm) {
      int64_t j = x->member[mm];
      real acc = 0;
      for (int e = 0; e < d; ++e) acc += q[i * d + e] * k[j * d + e];
      real p = EXP(acc * scale - m);
      l += p;
      for (int e = 0; e < d; ++e) of[e] += p * v[j * d + e];
    }
  for (int e = 0; e < d; ++e) of[e] /= l;
  return m + LOG(l);
}

/*
 * Forward with key cubes (Kt,Kh,Kw).  Arguments as vsa_oracle_forward, except: topk counts key
 * cubes (1 .. live key cubes); block_idx is [B,H,Nc,topk] of key cube labels, ascending;
 * out_coarse is [B,H,Nc,d]; sc (optional) is [B,H,Nc,Nk] with -inf for dead key cubes.
 */
int vsa_oracle_forward_kq(int B, int H, int T, int Hh, int W, int Ct, int Ch, int Cw, int Kt, int Kh, int Kw, int d,
                          int topk, double scale_, int indices_given, const real* q, const real* k, const real* v,
                          const real* gate_c, const real* gate_f, const int32_t* cubes, int ncubes, real* out,
                          int32_t* block_idx, real* out_fine, real* lse_fine, real* out_coarse, real* lse_coarse,
                          real* sc) {
  kq_t x;
  if (kq_make(&x, T, Hh, W, Ct, Ch, Cw, Kt, Kh, Kw)) return -1;
  const grid_t g = x.g;
  int live = 0;
  for (int j = 0; j < x.Nk; ++j) live += x.kcnt[j] > 0;
  if (B < 1 || H < 1 || d < 1 || topk < 1 || topk > live || (indices_given && !block_idx)) { kq_free(&x); return -1; }
  real scale = (real)scale_;
  int nq = cubes ? ncubes : g.Nc;
  for (int bh = 0; bh < B * H; ++bh) {
    const real* qh = q + (int64_t)bh * g.Np * d;
    const real* kh = k + (int64_t)bh * g.Np * d;
    const real* vh = v + (int64_t)bh * g.Np * d;
    real* Qc = (real*)malloc(sizeof(real) * (size_t)g.Nc * d);
    real* Kc = (real*)malloc(sizeof(real) * (size_t)x.Nk * d);
    real* Vc = (real*)malloc(sizeof(real) * (size_t)x.Nk * d);
    pool_mean(&g, d, x.valid, x.qcnt, qh, Qc);
    kq_pool_keys(&x, d, kh, Kc);
    kq_pool_keys(&x, d, vh, Vc);
#pragma omp parallel for schedule(dynamic, 1)
    for (int ci = 0; ci < nq; ++ci) {
      int c = cubes ? cubes[ci] : ci;
      real* row = (real*)malloc(sizeof(real) * (size_t)x.Nk);
      real* prob = (real*)malloc(sizeof(real) * (size_t)x.Nk);
      real* oc = (real*)malloc(sizeof(real) * (size_t)d);
      real* of = (real*)malloc(sizeof(real) * (size_t)d);
      int32_t* idx = (int32_t*)malloc(sizeof(int32_t) * (size_t)topk);
      kq_logits_row(&x, d, scale, Qc, Kc, c, row);
      real lse_c = kq_softmax_row(x.Nk, row, prob);
      for (int e = 0; e < d; ++e) {
        real s = 0;
        for (int j = 0; j < x.Nk; ++j) s += prob[j] * Vc[(int64_t)j * d + e];
        oc[e] = s;
      }
      if (sc) memcpy(sc + ((int64_t)bh * g.Nc + c) * x.Nk, row, sizeof(real) * (size_t)x.Nk);
      if (out_coarse) memcpy(out_coarse + ((int64_t)bh * g.Nc + c) * d, oc, sizeof(real) * (size_t)d);
      if (lse_coarse) lse_coarse[(int64_t)bh * g.Nc + c] = lse_c;
      if (indices_given) memcpy(idx, block_idx + ((int64_t)bh * g.Nc + c) * topk, sizeof(int32_t) * (size_t)topk);
      else {
        topk_row(x.Nk, row, topk, idx); /* dead key cubes carry -inf and sort last */
        if (block_idx) memcpy(block_idx + ((int64_t)bh * g.Nc + c) * topk, idx, sizeof(int32_t) * (size_t)topk);
      }
      for (int p = 0; p < g.Bk; ++p) {
        int64_t i = (int64_t)c * g.Bk + p;
        int64_t gi = ((int64_t)bh * g.Np + i) * d;
        if (!x.valid[i]) {
          for (int e = 0; e < d; ++e) {
            if (out) out[gi + e] = 0;
            if (out_fine) out_fine[gi + e] = 0;
          }
          if (lse_fine) lse_fine[(int64_t)bh * g.Np + i] = 0;
          continue;
        }
        real lse = kq_fine_row(&x, d, scale, qh, kh, vh, i, idx, topk, of);
        if (lse_fine) lse_fine[(int64_t)bh * g.Np + i] = lse;
        for (int e = 0; e < d; ++e) {
          if (out_fine) out_fine[gi + e] = of[e];
          if (out) out[gi + e] = oc[e] * gate_c[gi + e] + of[e] * (gate_f ? gate_f[gi + e] : (real)1);
        }
      }
      free(row); free(prob); free(oc); free(of); free(idx);
    }
    free(Qc); free(Kc); free(Vc);
  }
  kq_free(&x);
  return 0;
}

/* Backward with key cubes (Kt,Kh,Kw): the formulas listed at vsa_oracle_backward, with j running
 * over key cubes in the coarse part and the pooled K, V gradients spread over key cubes. */
int vsa_oracle_backward_kq(int B, int H, int T, int Hh, int W, int Ct, int Ch, int Cw, int Kt, int Kh, int Kw, int d,
                           int topk, double scale_, const real* q, const real* k, const real* v, const real* gate_c,
                           const real* gate_f, const real* dout, const int32_t* block_idx, real* dq, real* dk,
                           real* dv, real* dgate_c, real* dgate_f) {
  kq_t x;
  if (kq_make(&x, T, Hh, W, Ct, Ch, Cw, Kt, Kh, Kw)) return -1;
  const grid_t g = x.g;
  if (B < 1 || H < 1 || d < 1 || topk < 1 || topk > x.Nk || !block_idx) { kq_free(&x); return -1; }
  real scale = (real)scale_;
  const int Nc = g.Nc, Nk = x.Nk, Bk = g.Bk;
  const int64_t Np = g.Np;
  for (int bh = 0; bh < B * H; ++bh) {
    const int64_t off = (int64_t)bh * Np * d;
    const real *qh = q + off, *kh = k + off, *vh = v + off, *gch = gate_c + off, *doh = dout + off;
    const real* gfh = gate_f ? gate_f + off : NULL;
    const int32_t* idxh = block_idx + (int64_t)bh * Nc * topk;
    real *dqh = dq + off, *dkh = dk + off, *dvh = dv + off, *dgch = dgate_c + off;
    real* dgfh = dgate_f ? dgate_f + off : NULL;
    real* Qc = (real*)malloc(sizeof(real) * (size_t)Nc * d);
    real* Kc = (real*)malloc(sizeof(real) * (size_t)Nk * d);
    real* Vc = (real*)malloc(sizeof(real) * (size_t)Nk * d);
    real* Ac = (real*)malloc(sizeof(real) * (size_t)Nc * Nk);
    real* Oc = (real*)calloc((size_t)Nc * d, sizeof(real));
    real* Of = (real*)calloc((size_t)Np * d, sizeof(real));
    real* lse = (real*)calloc((size_t)Np, sizeof(real));
    real* dOf = (real*)calloc((size_t)Np * d, sizeof(real));
    real* Dl = (real*)calloc((size_t)Np, sizeof(real));
    real* dOc = (real*)calloc((size_t)Nc * d, sizeof(real));
    real* dSc = (real*)malloc(sizeof(real) * (size_t)Nc * Nk);
    real* dQc = (real*)calloc((size_t)Nc * d, sizeof(real));
    real* dKc = (real*)calloc((size_t)Nk * d, sizeof(real));
    real* dVc = (real*)calloc((size_t)Nk * d, sizeof(real));

    pool_mean(&g, d, x.valid, x.qcnt, qh, Qc);
    kq_pool_keys(&x, d, kh, Kc);
    kq_pool_keys(&x, d, vh, Vc);
#pragma omp parallel for schedule(dynamic, 1)
    for (int c = 0; c < Nc; ++c) {
      real* row = (real*)malloc(sizeof(real) * (size_t)Nk);
      kq_logits_row(&x, d, scale, Qc, Kc, c, row);
      kq_softmax_row(Nk, row, Ac + (int64_t)c * Nk);
      for (int e = 0; e < d; ++e) {
        real s = 0;
        for (int j = 0; j < Nk; ++j) s += Ac[(int64_t)c * Nk + j] * Vc[(int64_t)j * d + e];
        Oc[(int64_t)c * d + e] = s;
      }
      for (int p = 0; p < Bk; ++p) {
        int64_t i = (int64_t)c * Bk + p;
        if (x.valid[i]) lse[i] = kq_fine_row(&x, d, scale, qh, kh, vh, i, idxh + (int64_t)c * topk, topk, Of + i * d);
      }
      free(row);
    }
    for (int c = 0; c < Nc; ++c)
      for (int p = 0; p < Bk; ++p) {
        int64_t i = (int64_t)c * Bk + p;
        for (int e = 0; e < d; ++e) {
          dqh[i * d + e] = 0; dkh[i * d + e] = 0; dvh[i * d + e] = 0;
          if (!x.valid[i]) {
            dgch[i * d + e] = 0;
            if (dgfh) dgfh[i * d + e] = 0;
            continue;
          }
          real go = doh[i * d + e];
          dgch[i * d + e] = go * Oc[(int64_t)c * d + e];
          if (dgfh) dgfh[i * d + e] = go * Of[i * d + e];
          dOc[(int64_t)c * d + e] += go * gch[i * d + e];
          dOf[i * d + e] = go * (gfh ? gfh[i * d + e] : (real)1);
          Dl[i] += dOf[i * d + e] * Of[i * d + e];
        }
      }
    /* fine backward, dQ: one query token at a time */
#pragma omp parallel for schedule(dynamic, 1)
    for (int c = 0; c < Nc; ++c)
      for (int p = 0; p < Bk; ++p) {
        int64_t i = (int64_t)c * Bk + p;
        if (!x.valid[i]) continue;
        for (int r = 0; r < topk; ++r) {
          int jc = idxh[(int64_t)c * topk + r];
          for (int64_t mm = x.first[jc]; mm < x.first[jc + 1]; ++mm) {
            int64_t j = x.member[mm];
            real s = 0, dp = 0;
            for (int e = 0; e < d; ++e) { s += qh[i * d + e] * kh[j * d + e]; dp += dOf[i * d + e] * vh[j * d + e]; }
            real P = EXP(s * scale - lse[i]);
            real dS = P * (dp - Dl[i]);
            for (int e = 0; e < d; ++e) dqh[i * d + e] += scale * dS * kh[j * d + e];
          }
        }
      }
    /* fine backward, dK and dV: one key cube at a time, over the query cubes that selected it */
#pragma omp parallel for schedule(dynamic, 1)
    for (int jc = 0; jc < Nk; ++jc)
      for (int c = 0; c < Nc; ++c) {
        int sel = 0;
        for (int r = 0; r < topk; ++r) if (idxh[(int64_t)c * topk + r] == jc) sel = 1;
        if (!sel) continue;
        for (int p = 0; p < Bk; ++p) {
          int64_t i = (int64_t)c * Bk + p;
          if (!x.valid[i]) continue;
          for (int64_t mm = x.first[jc]; mm < x.first[jc + 1]; ++mm) {
            int64_t j = x.member[mm];
            real s = 0, dp = 0;
            for (int e = 0; e < d; ++e) { s += qh[i * d + e] * kh[j * d + e]; dp += dOf[i * d + e] * vh[j * d + e]; }
            real P = EXP(s * scale - lse[i]);
            real dS = P * (dp - Dl[i]);
            for (int e = 0; e < d; ++e) {
              dkh[j * d + e] += scale * dS * qh[i * d + e];
              dvh[j * d + e] += P * dOf[i * d + e];
            }
          }
        }
      }
    /* coarse backward */
    for (int c = 0; c < Nc; ++c) {
      real dot = 0;
      for (int j = 0; j < Nk; ++j) {
        real dA = 0;
        for (int e = 0; e < d; ++e) dA += dOc[(int64_t)c * d + e] * Vc[(int64_t)j * d + e];
        dSc[(int64_t)c * Nk + j] = dA;
        dot += Ac[(int64_t)c * Nk + j] * dA;
      }
      for (int j = 0; j < Nk; ++j) dSc[(int64_t)c * Nk + j] = Ac[(int64_t)c * Nk + j] * (dSc[(int64_t)c * Nk + j] - dot);
    }
    for (int c = 0; c < Nc; ++c)
      for (int j = 0; j < Nk; ++j)
        for (int e = 0; e < d; ++e) {
          dVc[(int64_t)j * d + e] += Ac[(int64_t)c * Nk + j] * dOc[(int64_t)c * d + e];
          dQc[(int64_t)c * d + e] += scale * dSc[(int64_t)c * Nk + j] * Kc[(int64_t)j * d + e];
          dKc[(int64_t)j * d + e] += scale * dSc[(int64_t)c * Nk + j] * Qc[(int64_t)c * d + e];
        }
    /* pooling backward */
    for (int64_t i = 0; i < Np; ++i) {
      if (!x.valid[i]) continue;
      int c = (int)(i / Bk), j = x.label[i];
      for (int e = 0; e < d; ++e) {
        dqh[i * d + e] += dQc[(int64_t)c * d + e] / (real)x.qcnt[c];
        dkh[i * d + e] += dKc[(int64_t)j * d + e] / (real)x.kcnt[j];
        dvh[i * d + e] += dVc[(int64_t)j * d + e] / (real)x.kcnt[j];
      }
    }
    free(Qc); free(Kc); free(Vc); free(Ac); free(Oc); free(Of); free(lse); free(dOf); free(Dl);
    free(dOc); free(dSc); free(dQc); free(dKc); free(dVc);
  }
  kq_free(&x);
  return 0;
}

/* [App. C.4] attention FLOPs: forward 4 * S * S_kv * d per head; forward+backward 3.5x. */
double vsa_oracle_attention_flops(double n_query_tokens, double n_key_tokens_per_query, double d, double heads,
                                  double batch, int with_backward) {
  double f = 4.0 * n_query_tokens * n_key_tokens_per_query * d * heads * batch;
  return with_backward ? 3.5 * f : f;
}

int vsa_oracle_real_bytes(void) { return (int)sizeof(real); }
