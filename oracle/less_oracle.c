/*
 * CPU oracle for one LESS generation step and for the prompt phase.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * HIP library is checked against.  It shares nothing with the HIP sources and
 * the product never calls it; only tests, the smoke check and the benchmark's
 * CPU-baseline leg load it.
 *
 * Everything is fp64, one (batch, head) unit at a time, loops written in the
 * order of the paper's equations.  OpenMP is used over units only, never
 * inside a unit, so every unit's summation order is fixed.
 *
 * What follows the paper and what is a reading of it:
 *   - feature maps phi, psi ............ Eq. 1, Eq. 2 (GELU per Sec. 3.2,
 *                                        "Inexpensive Training"; exact erf form)
 *   - attention synthesis .............. Eq. 3 (evaluated with a common shift
 *                                        m*, which cancels between numerator
 *                                        and denominator)
 *   - state update ..................... Eq. 4, Eq. 5, in Algorithm 1's order:
 *                                        the output uses H_t, z_t from before
 *                                        this step's eviction
 *   - sparse policy .................... H2O as Sec. 2.1 describes it: the
 *                                        attention probabilities of every step
 *                                        are accumulated per cached token; the
 *                                        budget is split into heavy hitters and
 *                                        most recent tokens (Sec. 4)
 *   second sparse policy ............... Lambda-masking (Sec. 4, "Setup"): the
 *                                        cache holds the first tokens of the
 *                                        sequence and the most recent ones, so
 *                                        the pair that leaves is always the
 *                                        oldest one that is not among the first
 *                                        (flag bit 1; n_heavy then counts the
 *                                        kept first tokens, 4 in the paper)
 *   - in-place replacement ............. Sec. 3.2, "Efficient Generation"
 *   - prompt phase ..................... regular attention (remark after Eq. 3)
 *   several query heads per KV head ..... multi-query / grouped-query attention (Sec. 3.2,
 *                                        "Inexpensive Training"): the G query heads that
 *                                        share a key/value head share its sparse cache and
 *                                        its state H, z (psi acts on keys), each has its own
 *                                        phi and its own Eq. 3, and H2O accumulates the
 *                                        attention probabilities of all of them per token
 *   Readings where the paper is silent (listed in the design notes as well):
 *     which denominator the accumulated probabilities use (flag bit 0),
 *     a new token's own probability starts its score, recency is decided by
 *     original position, ties evict the older token, the prompt is pruned in
 *     one shot from plain causal column sums.
 *
 * Parity pins: tests/test_oracle_*.py (full attention with an unbounded
 * budget, pure H2O with zero feature maps, the closed-form state of Eq. 6,
 * the set-based brute-force twin, Table 1 token counts, GELU spot values).
 * Absolute values of a LESS step are not printed anywhere in the paper, so
 * they rest on those reductions: "parity unpinned" by a worked example.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define LESS_FLAG_SPARSE_DENOM 1u /* accumulate e^s / (sparse-only denominator) */
#define LESS_FLAG_LAMBDA 2u       /* Lambda-masking instead of H2O: keep the first n_heavy
                                     tokens and the n_recent most recent ones              */
#define LESS_FLAG_PROMPT_STEPWISE 4u /* the sparse policy runs from the first prompt token
                                     (the evaluation setting of Sec. 4.1, where the policy
                                     masks query-key pairs throughout the sequence) instead
                                     of once at the end of the prompt                      */

typedef struct less_oracle_state {
  int32_t U, heads, D, n_heavy, n_recent, R, Rp;
  uint32_t flags;
  int32_t G;                                     /* query heads per unit (KV head); >= 1   */
  const int32_t *head;                           /* [U] head index of each unit            */
  const double *Wq1, *Wq2;                       /* phi, per query head: [heads*G,D,Rp] [heads*G,Rp,R] */
  const double *Wk1, *Wk2, *Wk3;                 /* psi, per KV head: [heads,D,Rp] [heads,Rp,R] [heads,R,R] */
  double *Kc, *Vc;                               /* [U,C,D]                                */
  double *acc;                                   /* [U,C]                                  */
  int64_t *pos;                                  /* [U,C], -1 = empty                      */
  double *H, *z;                                 /* [U,R,D], [U,R]                         */
  int64_t *n;                                    /* [U] tokens seen so far                 */
} less_oracle_state;

/* ---- Table 1: tokens kept at a given percentage of the maximum length ---- */
int64_t less_oracle_budget_tokens(double percent, int64_t max_len)
{
  /* rounded down to the nearest even number so heavy/recent split evenly (Sec. 4) */
  double tokens = percent * (double)max_len / 100.0;
  int64_t half = (int64_t)floor(tokens / 2.0 + 1e-9);
  return 2 * half;
}

/* ---- Eq. 1 / Eq. 2 -------------------------------------------------------- */
/* x * Phi(x); written with erfc so that the left tail keeps its relative accuracy */
double less_oracle_gelu(double x) { return 0.5 * x * erfc(-x / sqrt(2.0)); }

/* f = | gelu( gelu(q W1) W2 ) |,  W1 [D,Rp], W2 [Rp,R]   (Eq. 1) */
void less_oracle_phi(const double *q, const double *W1, const double *W2,
                     int D, int Rp, int R, double *f)
{
  double *h = (double *)malloc(sizeof(double) * (size_t)Rp);
  for (int i = 0; i < Rp; ++i) {
    double a = 0.0;
    for (int d = 0; d < D; ++d) a += q[d] * W1[(size_t)d * Rp + i];
    h[i] = less_oracle_gelu(a);
  }
  for (int r = 0; r < R; ++r) {
    double a = 0.0;
    for (int i = 0; i < Rp; ++i) a += h[i] * W2[(size_t)i * R + r];
    f[r] = fabs(less_oracle_gelu(a));
  }
  free(h);
}

/* g = | gelu( gelu(k W1) W2 ) W3 |,  W3 [R,R]   (Eq. 2) */
void less_oracle_psi(const double *k, const double *W1, const double *W2, const double *W3,
                     int D, int Rp, int R, double *g)
{
  double *h = (double *)malloc(sizeof(double) * (size_t)(Rp + R));
  double *h2 = h + Rp;
  for (int i = 0; i < Rp; ++i) {
    double a = 0.0;
    for (int d = 0; d < D; ++d) a += k[d] * W1[(size_t)d * Rp + i];
    h[i] = less_oracle_gelu(a);
  }
  for (int r = 0; r < R; ++r) {
    double a = 0.0;
    for (int i = 0; i < Rp; ++i) a += h[i] * W2[(size_t)i * R + r];
    h2[r] = less_oracle_gelu(a);
  }
  for (int r = 0; r < R; ++r) {
    double a = 0.0;
    for (int i = 0; i < R; ++i) a += h2[i] * W3[(size_t)i * R + r];
    g[r] = fabs(a);
  }
  free(h);
}

/* ---- per-unit views -------------------------------------------------------- */
typedef struct {
  int D, C, Nh, Nr, R, Rp, G;
  uint32_t flags;
  const double *Wq1, *Wq2, *Wk1, *Wk2, *Wk3;
  double *Kc, *Vc, *acc, *H, *z;
  int64_t *pos, *n;
} unit_view;

static unit_view view_of(const less_oracle_state *S, int u)
{
  unit_view v;
  int h = S->head[u];
  v.D = S->D; v.Nh = S->n_heavy; v.Nr = S->n_recent; v.C = v.Nh + v.Nr;
  v.R = S->R; v.Rp = S->Rp; v.flags = S->flags; v.G = S->G < 1 ? 1 : S->G;
  v.Wq1 = S->Wq1 + (size_t)h * v.G * v.D * v.Rp;          /* query head h G + g follows at g */
  v.Wq2 = S->Wq2 + (size_t)h * v.G * v.Rp * v.R;
  v.Wk1 = S->Wk1 + (size_t)h * v.D * v.Rp;
  v.Wk2 = S->Wk2 + (size_t)h * v.Rp * v.R;
  v.Wk3 = S->Wk3 + (size_t)h * v.R * v.R;
  v.Kc = S->Kc + (size_t)u * v.C * v.D;
  v.Vc = S->Vc + (size_t)u * v.C * v.D;
  v.acc = S->acc + (size_t)u * v.C;
  v.pos = S->pos + (size_t)u * v.C;
  v.H = S->H + (size_t)u * v.R * v.D;
  v.z = S->z + (size_t)u * v.R;
  v.n = S->n + u;
  return v;
}

static void reset_unit(unit_view *s)
{
  /* H_0 = 0, z_0 = 0 (Sec. 2.2); empty sparse cache */
  memset(s->H, 0, sizeof(double) * (size_t)s->R * s->D);
  memset(s->z, 0, sizeof(double) * (size_t)s->R);
  memset(s->Kc, 0, sizeof(double) * (size_t)s->C * s->D);
  memset(s->Vc, 0, sizeof(double) * (size_t)s->C * s->D);
  for (int j = 0; j < s->C; ++j) { s->acc[j] = 0.0; s->pos[j] = -1; }
  *s->n = 0;
}

/* H += psi(k)^T v,  z += psi(k)   (Eq. 4, Eq. 5 for one discarded pair) */
static void fold_into_state(unit_view *s, const double *k, const double *v)
{
  double g[64];
  less_oracle_psi(k, s->Wk1, s->Wk2, s->Wk3, s->D, s->Rp, s->R, g);
  for (int r = 0; r < s->R; ++r) {
    for (int d = 0; d < s->D; ++d) s->H[(size_t)r * s->D + d] += g[r] * v[d];
    s->z[r] += g[r];
  }
}

/*
 * One generation step of one unit (Algorithm 1).
 *   force_pos  >= 0 : evict the cached token with this original position
 *                     instead of the policy's own choice (used by the parity
 *                     protocol after an exempt near-tie); < 0: policy decides.
 *   q, out   [G,D]  : the unit's G query heads and their a-hat_t (Eq. 3)
 *   evicted    [1]  : original position of the pair folded into H, z; -1 none
 *   dec        [4]  : smallest and second smallest candidate (score, position);
 *                     position -1 where there is no such candidate.  Under
 *                     Lambda-masking the policy's key is the position alone and
 *                     "score" repeats it.
 *   share      [1]  : low-rank share of the denominator, phi(q) z^T / den
 * returns 0, or -1 if force_pos names no eviction candidate.
 */
static int step_unit(unit_view *s, const double *q, const double *k, const double *v,
                     int64_t force_pos, double *out, int64_t *evicted, double *dec,
                     double *share)
{
  const int D = s->D, C = s->C, R = s->R, G = s->G;
  const int64_t n = *s->n;
  double f[64];
  double *sc = (double *)malloc(sizeof(double) * (size_t)(C + 1));
  double *e = (double *)malloc(sizeof(double) * (size_t)(C + 1));
  double *inc = (double *)calloc((size_t)(C + 1), sizeof(double));   /* this step's probabilities per pair */
  const double sqrtD = sqrt((double)D);
  int rc = 0;
  int live = 0;
  for (int j = 0; j < C; ++j) if (s->pos[j] >= 0) ++live;
  double share_sum = 0.0;

  /* every query head of the unit attends over the same cache and state with its own phi */
  for (int g = 0; g < G; ++g) {
    const double *qg = q + (size_t)g * D;
    double *og = out + (size_t)g * D;
    less_oracle_phi(qg, s->Wq1 + (size_t)g * D * s->Rp, s->Wq2 + (size_t)g * s->Rp * R, D, s->Rp, R, f);   /* Eq. 1 */

    /* scores against the cached keys and the appended key (K' of Eq. 3) */
    for (int j = 0; j < C; ++j) {
      if (s->pos[j] < 0) { sc[j] = -INFINITY; continue; }
      double a = 0.0;
      for (int d = 0; d < D; ++d) a += qg[d] * s->Kc[(size_t)j * D + d];
      sc[j] = a / sqrtD;
    }
    {
      double a = 0.0;
      for (int d = 0; d < D; ++d) a += qg[d] * k[d];
      sc[C] = a / sqrtD;
    }

    /* phi(q) z^T and the common shift m* = max(scores, ln(phi(q) z^T)) */
    double fz = 0.0;
    for (int r = 0; r < R; ++r) fz += f[r] * s->z[r];
    double mstar = sc[C];
    for (int j = 0; j < C; ++j) if (s->pos[j] >= 0 && sc[j] > mstar) mstar = sc[j];
    double lfz = (fz > 0.0) ? log(fz) : -INFINITY;
    if (lfz > mstar) mstar = lfz;

    /* Eq. 3, numerator and denominator both multiplied by e^{-m*} */
    double wl = (fz > 0.0) ? exp(lfz - mstar) : 0.0;       /* phi(q) z^T e^{-m*} */
    double den = wl;
    for (int d = 0; d < D; ++d) og[d] = 0.0;
    if (fz > 0.0) {
      double sh = exp(-mstar);
      for (int d = 0; d < D; ++d) {
        double a = 0.0;
        for (int r = 0; r < R; ++r) a += f[r] * s->H[(size_t)r * D + d];
        og[d] = a * sh;                                    /* phi(q) H e^{-m*} */
      }
    }
    for (int j = 0; j < C; ++j) {
      if (s->pos[j] < 0) { e[j] = 0.0; continue; }
      e[j] = exp(sc[j] - mstar);
      den += e[j];
      for (int d = 0; d < D; ++d) og[d] += e[j] * s->Vc[(size_t)j * D + d];
    }
    e[C] = exp(sc[C] - mstar);
    den += e[C];
    for (int d = 0; d < D; ++d) og[d] += e[C] * v[d];
    for (int d = 0; d < D; ++d) og[d] /= den;
    share_sum += wl / den;

    /* H2O: this head's attention probabilities, added up over the heads of the unit */
    double dacc = (s->flags & LESS_FLAG_SPARSE_DENOM) ? (den - wl) : den;
    for (int j = 0; j < C; ++j)
      if (s->pos[j] >= 0) inc[j] += e[j] / dacc;
    inc[C] += e[C] / dacc;
  }
  if (share) *share = share_sum / G;

  /* H2O: accumulate this step's attention probabilities per cached token */
  for (int j = 0; j < C; ++j)
    if (s->pos[j] >= 0) s->acc[j] += inc[j];
  double acc_new = inc[C];

  /* cache update: append, and if over capacity evict one pair into H, z */
  dec[0] = dec[2] = INFINITY; dec[1] = dec[3] = -1.0;
  *evicted = -1;
  if (live < C) {
    int slot = 0;
    while (s->pos[slot] >= 0) ++slot;                   /* lowest free slot */
    memcpy(s->Kc + (size_t)slot * D, k, sizeof(double) * (size_t)D);
    memcpy(s->Vc + (size_t)slot * D, v, sizeof(double) * (size_t)D);
    s->acc[slot] = acc_new; s->pos[slot] = n;
  } else {
    /* recent = the Nr largest positions, the new token (position n) included */
    const int lambda = (s->flags & LESS_FLAG_LAMBDA) != 0;
    int best = -2, second = -2;                          /* -1 denotes the new token */
    double bacc = INFINITY, sacc = INFINITY; int64_t bpos = -1, spos = -1;
    int forced = -2;
    for (int j = -1; j < C; ++j) {
      double a; int64_t p;
      if (j < 0) { if (s->Nr != 0) continue; a = acc_new; p = n; }
      else { if (s->pos[j] > n - s->Nr) continue; a = s->acc[j]; p = s->pos[j]; }
      if (lambda) {
        /* the first Nh tokens of the sequence stay for good; of the others the oldest leaves */
        if (j >= 0 && p < s->Nh) continue;
        a = (double)p;
      }
      if (p == force_pos) forced = j;
      if (a < bacc || (a == bacc && p < bpos)) {
        second = best; sacc = bacc; spos = bpos;
        best = j; bacc = a; bpos = p;
      } else if (a < sacc || (a == sacc && p < spos)) {
        second = j; sacc = a; spos = p;
      }
    }
    (void)second;
    dec[0] = bacc; dec[1] = (double)bpos; dec[2] = sacc; dec[3] = (double)spos;
    int ev = best;
    if (force_pos >= 0) { if (forced == -2) rc = -1; else ev = forced; }
    if (ev == -2) {
      rc = -1;                                           /* no candidate: C == 0 */
    } else if (ev == -1) {
      fold_into_state(s, k, v);                          /* Eq. 4, Eq. 5 */
      *evicted = n;
    } else {
      fold_into_state(s, s->Kc + (size_t)ev * D, s->Vc + (size_t)ev * D);
      *evicted = s->pos[ev];
      memcpy(s->Kc + (size_t)ev * D, k, sizeof(double) * (size_t)D);   /* in place */
      memcpy(s->Vc + (size_t)ev * D, v, sizeof(double) * (size_t)D);
      s->acc[ev] = acc_new; s->pos[ev] = n;
    }
  }
  *s->n = n + 1;
  free(sc); free(e); free(inc);
  return rc;
}

/* ascending (column sum, position) */
typedef struct { double a; int64_t p; } scored;
static int cmp_scored(const void *x, const void *y)
{
  const scored *a = (const scored *)x, *b = (const scored *)y;
  if (a->a < b->a) return -1;
  if (a->a > b->a) return 1;
  return (a->p < b->p) ? -1 : (a->p > b->p);
}

/*
 * Prompt phase of one unit: regular causal attention (H_0 = z_0 = 0), then the
 * cache is cut to the budget in one shot: the last Nr tokens are kept as
 * recent, the Nh tokens with the largest column sums of the attention matrix
 * as heavy hitters (under Lambda-masking: the first Nh tokens instead), and
 * every other token is folded into H, z (Eq. 6).  The column sums become the
 * kept tokens' accumulated scores under either policy.
 *   out     [P,D] or NULL
 *   colsum  [P]   or NULL : accumulated attention probability of every token
 *   kept    [P]   or NULL : 1 kept, 0 discarded
 *   dec     [4]           : (colsum,pos) of the last discarded and the first
 *                           kept token in ascending order, -1 positions if the
 *                           prompt fits the budget
 */
static void prefill_unit(unit_view *s, const double *Q, const double *K, const double *V,
                         int64_t P, double *out, double *colsum_out, int8_t *kept_out,
                         double *dec)
{
  const int D = s->D, C = s->C;
  const double sqrtD = sqrt((double)D);
  reset_unit(s);
  double *colsum = (double *)calloc((size_t)(P > 0 ? P : 1), sizeof(double));
  double *row = (double *)malloc(sizeof(double) * (size_t)(P > 0 ? P : 1));
  /* Q and out are [G,P,D]: every query head of the unit attends over the same keys and
     values, and a token's score is the attention mass it receives from all of them */
  for (int g = 0; g < s->G; ++g) {
    const double *Qg = Q + (size_t)g * P * D;
    for (int64_t i = 0; i < P; ++i) {
      double m = -INFINITY;
      for (int64_t j = 0; j <= i; ++j) {
        double a = 0.0;
        for (int d = 0; d < D; ++d) a += Qg[i * D + d] * K[j * D + d];
        row[j] = a / sqrtD;
        if (row[j] > m) m = row[j];
      }
      double L = 0.0;
      for (int64_t j = 0; j <= i; ++j) { row[j] = exp(row[j] - m); L += row[j]; }
      for (int64_t j = 0; j <= i; ++j) { row[j] /= L; colsum[j] += row[j]; }
      if (out) {
        for (int d = 0; d < D; ++d) {
          double a = 0.0;
          for (int64_t j = 0; j <= i; ++j) a += row[j] * V[j * D + d];
          out[((size_t)g * P + i) * D + d] = a;
        }
      }
    }
  }
  int8_t *kept = (int8_t *)malloc((size_t)(P > 0 ? P : 1));
  dec[0] = dec[2] = INFINITY; dec[1] = dec[3] = -1.0;
  if (P <= C) {
    for (int64_t j = 0; j < P; ++j) kept[j] = 1;
  } else if (s->flags & LESS_FLAG_LAMBDA) {
    for (int64_t j = 0; j < P; ++j) kept[j] = (j < s->Nh || j >= P - s->Nr) ? 1 : 0;
  } else {
    int64_t ncand = P - s->Nr;                            /* positions < P - Nr */
    scored *c = (scored *)malloc(sizeof(scored) * (size_t)(ncand > 0 ? ncand : 1));
    for (int64_t j = 0; j < ncand; ++j) { c[j].a = colsum[j]; c[j].p = j; }
    qsort(c, (size_t)ncand, sizeof(scored), cmp_scored);
    int64_t nev = ncand - s->Nh;                          /* discarded count */
    for (int64_t j = 0; j < P; ++j) kept[j] = 1;
    for (int64_t r = 0; r < nev; ++r) kept[c[r].p] = 0;
    if (nev > 0) { dec[0] = c[nev - 1].a; dec[1] = (double)c[nev - 1].p; }
    if (nev < ncand) { dec[2] = c[nev].a; dec[3] = (double)c[nev].p; }
    free(c);
  }
  /* slots: kept tokens in ascending position (heavy hitters precede recent ones) */
  int slot = 0;
  for (int64_t j = 0; j < P; ++j) {
    if (kept[j]) {
      memcpy(s->Kc + (size_t)slot * D, K + j * D, sizeof(double) * (size_t)D);
      memcpy(s->Vc + (size_t)slot * D, V + j * D, sizeof(double) * (size_t)D);
      s->acc[slot] = colsum[j]; s->pos[slot] = j;
      ++slot;
    } else {
      fold_into_state(s, K + j * D, V + j * D);           /* Eq. 6 */
    }
  }
  *s->n = P;
  if (colsum_out) memcpy(colsum_out, colsum, sizeof(double) * (size_t)P);
  if (kept_out) memcpy(kept_out, kept, (size_t)P);
  free(kept); free(row); free(colsum);
}

/* ---- exported drivers over units ------------------------------------------ */

void less_oracle_reset(less_oracle_state *S)
{
  for (int u = 0; u < S->U; ++u) { unit_view v = view_of(S, u); reset_unit(&v); }
}

/* q [U,G,D]; k,v [U,D]; force [U] or NULL; out [U,G,D]; evicted [U]; dec [U,4]; share [U] or NULL.
   returns the number of units whose forced position was not a candidate. */
int less_oracle_step(less_oracle_state *S, const double *q, const double *k, const double *v,
                     const int64_t *force, double *out, int64_t *evicted, double *dec,
                     double *share)
{
  int bad = 0;
  const int D = S->D, G = S->G < 1 ? 1 : S->G;
#pragma omp parallel for schedule(static) reduction(+ : bad)
  for (int u = 0; u < S->U; ++u) {
    unit_view s = view_of(S, u);
    int rc = step_unit(&s, q + (size_t)u * G * D, k + (size_t)u * D, v + (size_t)u * D,
                       force ? force[u] : -1, out + (size_t)u * G * D, evicted + u,
                       dec + (size_t)u * 4, share ? share + u : NULL);
    if (rc) ++bad;
  }
  return bad;
}

/*
 * Prompt phase with the policy active from the first token: token t of the prompt is one
 * generation step (Algorithm 1) with its own query, key and value, exactly as if the prompt
 * were generated.  out [P,D] or NULL: Eq. 3's output at every token.
 */
static void prefill_unit_stepwise(unit_view *s, const double *Q, const double *K, const double *V,
                                  int64_t P, double *out)
{
  const int D = s->D, G = s->G;
  double *o = (double *)malloc(sizeof(double) * (size_t)G * D);
  double *qt = (double *)malloc(sizeof(double) * (size_t)G * D);      /* token t's G queries */
  double dec[4];
  int64_t ev;
  reset_unit(s);
  for (int64_t t = 0; t < P; ++t) {
    for (int g = 0; g < G; ++g) memcpy(qt + (size_t)g * D, Q + ((size_t)g * P + t) * D, sizeof(double) * (size_t)D);
    step_unit(s, qt, K + t * D, V + t * D, -1, o, &ev, dec, NULL);
    if (out)
      for (int g = 0; g < G; ++g) memcpy(out + ((size_t)g * P + t) * D, o + (size_t)g * D, sizeof(double) * (size_t)D);
  }
  free(o); free(qt);
}

/* Q [U,G,P,D]; K,V [U,P,D]; out [U,G,P,D] or NULL; colsum [U,P] or NULL; kept [U,P] or NULL; dec [U,4]
   (colsum, kept and dec are left untouched in the stepwise setting) */
void less_oracle_prefill(less_oracle_state *S, const double *Q, const double *K, const double *V,
                         int64_t P, double *out, double *colsum, int8_t *kept, double *dec)
{
  const size_t PD = (size_t)P * S->D, GPD = PD * (size_t)(S->G < 1 ? 1 : S->G);
  if (S->flags & LESS_FLAG_PROMPT_STEPWISE) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < S->U; ++u) {
      unit_view s = view_of(S, u);
      prefill_unit_stepwise(&s, Q + u * GPD, K + u * PD, V + u * PD, P, out ? out + u * GPD : NULL);
    }
    return;
  }
#pragma omp parallel for schedule(dynamic, 1)
  for (int u = 0; u < S->U; ++u) {
    unit_view s = view_of(S, u);
    prefill_unit(&s, Q + u * GPD, K + u * PD, V + u * PD, P, out ? out + u * GPD : NULL,
                 colsum ? colsum + (size_t)u * P : NULL, kept ? kept + (size_t)u * P : NULL,
                 dec + (size_t)u * 4);
  }
}

/* Eq. 7: Hellinger distance between two discrete probability vectors */
double less_oracle_hellinger(const double *p, const double *q, int64_t n)
{
  double a = 0.0;
  for (int64_t i = 0; i < n; ++i) { double d = sqrt(p[i]) - sqrt(q[i]); a += d * d; }
  return sqrt(a) / sqrt(2.0);
}
