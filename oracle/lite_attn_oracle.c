/*
 * LiteAttention CPU oracle  --  TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, obviously-correct CPU statement of what one call of the
 * skip-aware attention forward computes.  It is independent of the HIP path:
 * it shares no source, header, table or helper with it, and nothing in the
 * product may call it.  Only the tests, the smoke check and the benchmark's
 * cpu_baseline leg load this file.
 *
 * What it follows (paper sections / equations / algorithms):
 *   - tiling of Q, K, V along the sequence and the per-tile recurrences
 *     S_ij, P~_ij, m_ij, O~_ij: Preliminaries, "FlashAttention" (the three
 *     tile equations after eqs. 1-3);
 *   - the local skip predicate max(m_local - m_ij) <= -eps: Preliminaries,
 *     "SpargeAttention", eq. (sparge_cond);
 *   - the loop with the Skip-Mask test before QK^T and the mask update:
 *     Method, Algorithm 2 (QK-Skip);
 *   - deferral of a freshly fired bit to the next timestep (the tile is still
 *     accumulated in the step that marks it): Implementation, "Skip-Mask
 *     Evaluation Mechanism" and "Producer and Skip-List Optimization";
 *   - linear order of the j loop: Experiments, "Settings"; optionally another visiting order given as an
 *     explicit permutation per Q tile (Method, "Skipping Condition": other orders reach the global maximum sooner).
 * The row-sum l and the final division are the textbook online softmax the
 * paper leaves out "for brevity".
 *
 * Arithmetic type: `real` (float by default; -DLA_ORACLE_F64 gives double).
 * Inputs are bf16 bit patterns widened exactly to `real`.
 *
 * Pins (tests/test_oracle_*.py, all CPU): dense softmax attention in float64
 * with the threshold disabled; float64 block-masked dense attention for the
 * output given a live set; an O(N^2) prefix-max formula for every predicate
 * value; a closed-form two-tile case; the bound max P~ <= e^thr on fired
 * tiles; monotone mask, first live tile never fires, pinned tiles never fire,
 * deferred and immediate modes give equal masks; a five-step trajectory
 * (masks and outputs of every step) against the same loop composed from the
 * O(N^2) float64 definitions alone.  The paper prints no worked numeric
 * example, so no pin compares with a value of the paper's: in that sense
 * the multi-step trajectory on the synthetic data stays "parity unpinned"
 * -- it is pinned to the definitions, not to published numbers.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef LA_ORACLE_F64
typedef double real;
#define REAL_EXP exp
#define REAL_SQRT sqrt
#else
typedef float real;
#define REAL_EXP expf
#define REAL_SQRT sqrtf
#endif

typedef struct {
  int32_t batch, heads, seqlen, head_dim;
  int32_t tile_q, tile_k;               /* h_q, h_k of the paper's tiling */
  int64_t stride_b, stride_h, stride_n; /* element strides of q, k, v; head_dim contiguous */
  int32_t protect_start, protect_len;   /* token range whose tiles are never marked */
  int32_t immediate;                    /* 1: Algorithm 2 literally (fired tile dropped at once) */
} la_oracle_shape;

enum { LA_ORACLE_OK = 0, LA_ORACLE_EINVAL = -1, LA_ORACLE_ENOMEM = -2 };

int la_oracle_real_bytes(void) { return (int)sizeof(real); }

static real widen_bf16(uint16_t h) {
  uint32_t u = ((uint32_t)h) << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (real)f;
}

static int intersects(int64_t lo, int64_t hi, int64_t ps, int64_t pl) {
  /* [lo,hi) against [ps,ps+pl) */
  return pl > 0 && lo < ps + pl && ps < hi;
}

/* One Q-tile row (b,h,i): Algorithm 2 with the deferred / immediate reading. */
static int oracle_row(const la_oracle_shape* sh, const uint16_t* q, const uint16_t* k, const uint16_t* v,
                      uint8_t* mask_row, real thr, real* out_bh, real* g_row, int b, int h, int i,
                      const int32_t* visit) {
  const int d = sh->head_dim, hq = sh->tile_q, hk = sh->tile_k, N = sh->seqlen;
  const int Tk = (N + hk - 1) / hk;
  const int r0 = i * hq;
  const int nr = (N - r0 < hq) ? (N - r0) : hq;
  const real inv_sqrt_d = (real)1 / REAL_SQRT((real)d);
  const int64_t base = (int64_t)b * sh->stride_b + (int64_t)h * sh->stride_h;

  real* Qi = (real*)malloc(sizeof(real) * (size_t)nr * d);
  real* Kj = (real*)malloc(sizeof(real) * (size_t)hk * d);
  real* Vj = (real*)malloc(sizeof(real) * (size_t)hk * d);
  real* S = (real*)malloc(sizeof(real) * (size_t)nr * hk);
  real* acc = (real*)calloc((size_t)nr * d, sizeof(real));
  real* m = (real*)malloc(sizeof(real) * nr);
  real* l = (real*)calloc(nr, sizeof(real));
  real* mloc = (real*)malloc(sizeof(real) * nr);
  real* mnew = (real*)malloc(sizeof(real) * nr);
  uint8_t* newmask = (uint8_t*)calloc(Tk, 1);
  if (!Qi || !Kj || !Vj || !S || !acc || !m || !l || !mloc || !mnew || !newmask) {
    free(Qi); free(Kj); free(Vj); free(S); free(acc); free(m); free(l); free(mloc); free(mnew); free(newmask);
    return LA_ORACLE_ENOMEM;
  }
  for (int r = 0; r < nr; ++r) {
    m[r] = -INFINITY; /* m_{i,-1} */
    for (int x = 0; x < d; ++x) Qi[(size_t)r * d + x] = widen_bf16(q[base + (int64_t)(r0 + r) * sh->stride_n + x]);
  }
  const int q_pinned = intersects(r0, r0 + nr, sh->protect_start, sh->protect_len);

  for (int t = 0; t < Tk; ++t) {
    const int j = visit ? visit[t] : t; /* linear order unless a visiting order is given */
    if (mask_row[j]) {                  /* SkipMask(i,j): nothing of tile j is touched */
      if (g_row) g_row[j] = (real)NAN;
      continue;
    }
    const int c0 = j * hk;
    const int nc = (N - c0 < hk) ? (N - c0) : hk;
    for (int c = 0; c < nc; ++c)
      for (int x = 0; x < d; ++x) {
        Kj[(size_t)c * d + x] = widen_bf16(k[base + (int64_t)(c0 + c) * sh->stride_n + x]);
        Vj[(size_t)c * d + x] = widen_bf16(v[base + (int64_t)(c0 + c) * sh->stride_n + x]);
      }
    /* S_ij = Q_i K_j^T / sqrt(d);  m_local = rowmax(S_ij);  m_ij = max(m_{i,j-1}, m_local) */
    real gval = -INFINITY;
    for (int r = 0; r < nr; ++r) {
      real best = -INFINITY;
      for (int c = 0; c < nc; ++c) {
        real s = 0;
        for (int x = 0; x < d; ++x) s += Qi[(size_t)r * d + x] * Kj[(size_t)c * d + x];
        s *= inv_sqrt_d;
        S[(size_t)r * hk + c] = s;
        if (s > best) best = s;
      }
      mloc[r] = best;
      mnew[r] = (m[r] > best) ? m[r] : best;
      real diff = mloc[r] - mnew[r];
      if (diff > gval) gval = diff; /* the max over the tile's rows in the predicate */
    }
    if (g_row) g_row[j] = gval;
    const int pinned = q_pinned || intersects(c0, c0 + nc, sh->protect_start, sh->protect_len);
    const int fire = (gval <= thr) && !pinned;
    if (fire) newmask[j] = 1;
    if (fire && sh->immediate) continue; /* fired => m_local < m on every row, so m_ij = m_{i,j-1} */
    /* P~ = exp(S - m_ij); l and O~ rescaled by exp(m_{i,j-1} - m_ij) */
    for (int r = 0; r < nr; ++r) {
      real a = (m[r] == -INFINITY) ? (real)0 : REAL_EXP(m[r] - mnew[r]);
      real rowsum = 0;
      real* accr = acc + (size_t)r * d;
      for (int x = 0; x < d; ++x) accr[x] *= a;
      for (int c = 0; c < nc; ++c) {
        real p = REAL_EXP(S[(size_t)r * hk + c] - mnew[r]);
        rowsum += p;
        const real* vc = Vj + (size_t)c * d;
        for (int x = 0; x < d; ++x) accr[x] += p * vc[x];
      }
      l[r] = a * l[r] + rowsum;
      m[r] = mnew[r];
    }
  }
  for (int r = 0; r < nr; ++r)
    for (int x = 0; x < d; ++x) out_bh[(size_t)(r0 + r) * d + x] = acc[(size_t)r * d + x] / l[r];
  for (int j = 0; j < Tk; ++j) mask_row[j] |= newmask[j]; /* bits are only ever set */

  free(Qi); free(Kj); free(Vj); free(S); free(acc); free(m); free(l); free(mloc); free(mnew); free(newmask);
  return LA_ORACLE_OK;
}

/*
 * One attention call (one denoising step of one layer).
 *   q,k,v  bf16 bit patterns, element strides from `sh`
 *   mask   [B,H,Tq,Tk] one byte per tile, nonzero = skipped; read on entry, updated in place
 *   thr    signed threshold (= -eps) in natural-log units of S; -INFINITY never fires
 *   out    [B,H,N,d] contiguous `real`; only the rows computed are written
 *   g      [B,H,Tq,Tk] predicate value of every evaluated tile, NaN for tiles skipped on entry; may be NULL
 *   rows   optional list of flattened row ids (b*H+h)*Tq+i to compute; NULL = every row
 *   visit  optional [Tq][Tk] int32: visit[i][t] = K/V tile visited t-th by Q tile i (a permutation of 0..Tk-1,
 *          the same for every batch entry and head); NULL = ascending
 */
int la_oracle_step(const la_oracle_shape* sh, const uint16_t* q, const uint16_t* k, const uint16_t* v,
                   uint8_t* mask, real thr, real* out, real* g, const int64_t* rows, int64_t nrows,
                   const int32_t* visit) {
  if (!sh || !q || !k || !v || !mask || !out) return LA_ORACLE_EINVAL;
  if (sh->batch < 1 || sh->heads < 1 || sh->seqlen < 1 || sh->head_dim < 1 || sh->tile_q < 1 || sh->tile_k < 1)
    return LA_ORACLE_EINVAL;
  if (thr != thr || thr >= 0) return LA_ORACLE_EINVAL; /* eps > 0 */
  const int N = sh->seqlen, H = sh->heads, d = sh->head_dim;
  const int Tq = (N + sh->tile_q - 1) / sh->tile_q, Tk = (N + sh->tile_k - 1) / sh->tile_k;
  const int64_t total = (int64_t)sh->batch * H * Tq;
  const int64_t count = rows ? nrows : total;
  int status = LA_ORACLE_OK;
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t t = 0; t < count; ++t) {
    int64_t row = rows ? rows[t] : t;
    if (row < 0 || row >= total) {
#pragma omp critical
      status = LA_ORACLE_EINVAL;
      continue;
    }
    int i = (int)(row % Tq);
    int h = (int)((row / Tq) % H);
    int b = (int)(row / ((int64_t)Tq * H));
    int rc = oracle_row(sh, q, k, v, mask + row * Tk, thr, out + ((int64_t)b * H + h) * N * d,
                        g ? g + row * Tk : NULL, b, h, i, visit ? visit + (int64_t)i * Tk : NULL);
    if (rc != LA_ORACLE_OK) {
#pragma omp critical
      status = rc;
    }
  }
  return status;
}
