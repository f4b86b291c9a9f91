/*
 * BalanceRoute CPU oracle -- TEST INFRASTRUCTURE ONLY (see br_oracle.h).
 *
 * Plain single-threaded C.  No blocking, fusion or reordering beyond what the
 * paper's definitions state.  Build: gcc -O2 -ffp-contract=off -fPIC -shared.
 */
#include "br_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ scores */

/* Sec. 3.1, eq. (br0-Fscore): F = Delta - G * (Delta - m)_+ , exact integers. */
int64_t orc_score_br0(int64_t G, int64_t m, int64_t delta) {
  int64_t over = delta - m;
  if (over < 0) over = 0;
  return delta - G * over;
}

typedef struct {
  int32_t G, H;
  int32_t use_float; /* horizon score in fp32 (H > 0, or forced for the H = 0 reduction check) */
  float d[ORC_MAX_H + 1]; /* discount vector (1, gamma, ..., gamma^H), by repeated product */
  float aD;               /* alpha * (1^T d) */
  float beta;
} scorer;

static void scorer_init(scorer *S, const orc_params *P, int force_float) {
  int h;
  float D = 0.0f;
  S->G = P->G;
  S->H = P->H;
  S->use_float = (P->H > 0) || force_float;
  S->d[0] = 1.0f;
  for (h = 1; h <= P->H; ++h) S->d[h] = S->d[h - 1] * P->gamma;
  for (h = 0; h <= P->H; ++h) D = D + S->d[h];
  S->aD = P->alpha * D;
  S->beta = P->beta;
}

/* Sec. 4.1, eq. (brh-Fscore): alpha (1^T d) Delta - beta ((Delta 1 - m)_+)^T d, fp32,
 * penalty accumulated from h = 0 upwards, one fused multiply-add (a single rounding) per offset. */
static float horizon_score(const scorer *S, const int64_t *m, int64_t delta) {
  float pen = 0.0f;
  int h;
  for (h = 0; h <= S->H; ++h) {
    int64_t over = delta - m[h];
    if (over < 0) over = 0;
    pen = fmaf(S->d[h], (float)over, pen);
  }
  return S->aD * (float)delta - S->beta * pen;
}

float orc_score_brh(int32_t H, float alpha, float beta, float gamma, const int64_t *m, int64_t delta) {
  orc_params P;
  scorer S;
  memset(&P, 0, sizeof P);
  P.H = H;
  P.alpha = alpha;
  P.beta = beta;
  P.gamma = gamma;
  scorer_init(&S, &P, 1);
  return horizon_score(&S, m, delta);
}

/* One score as a double: exact for the integer score (|F| < 2^53) and for fp32,
 * so comparisons on it equal comparisons in the native type. */
static double score(const scorer *S, const int64_t *m, int64_t delta) {
  if (S->use_float) return (double)horizon_score(S, m, delta);
  return (double)orc_score_br0(S->G, m[0], delta);
}

/* ------------------------------------------------- in-window contribution */

/* Appendix "Short-horizon prediction interface": c_hat ~ E[min(r, H)].
 * With per-step hazards p_j = P(r = j | r >= j): survival S_0 = 1, S_j = S_{j-1}(1 - p_j),
 * E[min(r,H)] = sum_{j=0}^{H-1} S_j, which equals the composite of eq. (two-stage)/(composite)
 * with p_fin = 1 - S_H.  Gate (p_fin below the threshold -> conservative anchor H) and
 * floor 1 follow Appendix "Refresh logic"; the clip to [.,H] follows eq. (composite). */
float orc_chat(int32_t H, int32_t pred_mode, float gate_pfin, const float *p) {
  float c;
  float Hf = (float)H;
  if (H == 0) return 0.0f;
  if (pred_mode == 3) { /* the two stages themselves: eq. (composite) on (p_fin, mu_rem), same gate */
    float pfin = p[0], mu = p[1];
    c = (1.0f - pfin) * Hf + pfin * mu;
    if (gate_pfin > 0.0f && pfin < gate_pfin) c = Hf;
  } else if (pred_mode >= 1) {
    c = p[0];
  } else {
    float S = 1.0f, pfin;
    int j;
    c = 0.0f;
    for (j = 1; j <= H; ++j) {
      c = c + S;
      S = S * (1.0f - p[j - 1]);
    }
    pfin = 1.0f - S;
    if (gate_pfin > 0.0f && pfin < gate_pfin) c = Hf;
  }
  if (c < 1.0f) c = 1.0f;
  if (c > Hf) c = Hf;
  return c;
}

/* floats kept per active request / per waiting request */
static int32_t pred_width(const orc_params *P) {
  if (P->H == 0) return 0;
  return P->pred_mode == 2 ? 3 : (P->pred_mode == 3 ? 2 : (P->pred_mode == 1 ? 1 : P->H));
}

static int32_t queue_pred_width(const orc_params *P) { return P->pred_mode == 2 ? 0 : pred_width(P); }

/* number of history entries <= x */
static int64_t hist_rank(const orc_params *P, int64_t x) {
  int64_t lo = 0, hi = P->hist_n;
  while (lo < hi) {
    int64_t mid = (lo + hi) / 2;
    if (P->hist[mid] <= x)
      lo = mid + 1;
    else
      hi = mid;
  }
  return lo;
}

/* Appendix "Estimator realizations", empirical-survival: with F the empirical CDF of the output-length
 * history, p_fin = (F(a+H) - F(a)) / (1 - F(a)) and mu_rem = mean of (o_j - a) over a < o_j <= a+H;
 * composite, gate, floor and clip as in eq. (composite) and "Refresh logic".  A request that has
 * outlived the whole history, or with nothing in the window, gets the conservative anchor H. */
float orc_survival(const orc_params *P, int64_t age) {
  float Hf = (float)P->H, p = 0.0f, mu = 0.0f, c;
  int64_t lo = hist_rank(P, age), hi = hist_rank(P, age + P->H);
  int64_t surv = P->hist_n - lo, cnt = hi - lo;
  if (surv > 0 && cnt > 0) {
    int64_t rem_sum = (P->hist_sum[hi] - P->hist_sum[lo]) - cnt * age;
    p = (float)cnt / (float)surv;
    mu = (float)rem_sum / (float)cnt;
  }
  c = (1.0f - p) * Hf + p * mu;
  if (P->gate_pfin > 0.0f && p < P->gate_pfin) c = Hf;
  if (c < 1.0f) c = 1.0f;
  if (c > Hf) c = Hf;
  return c;
}

/* ------------------------------------------------------------ route state */

typedef struct {
  const orc_params *P;
  scorer S;
  int64_t L[ORC_MAX_G];
  int64_t cap[ORC_MAX_G];
  int64_t Lh[ORC_MAX_G][ORC_MAX_H + 1];
  int64_t Mh[ORC_MAX_H + 1];
  int64_t m[ORC_MAX_G][ORC_MAX_H + 1];
  int64_t minm[ORC_MAX_G];
} rstate;

/* envelope M_h = max_g L_g(k+h) */
static void envelope(rstate *R) {
  int g, h;
  for (h = 0; h <= R->P->H; ++h) {
    int64_t M = R->Lh[0][h];
    for (g = 1; g < R->P->G; ++g)
      if (R->Lh[g][h] > M) M = R->Lh[g][h];
    R->Mh[h] = M;
  }
}

/* margins m_{g,h} = (M_h - L_g(k+h))_+ and their horizon minimum */
static void margins(rstate *R) {
  int g, h;
  for (g = 0; g < R->P->G; ++g) {
    int64_t mn = 0;
    for (h = 0; h <= R->P->H; ++h) {
      int64_t v = R->Mh[h] - R->Lh[g][h];
      if (v < 0) v = 0;
      R->m[g][h] = v;
      if (h == 0 || v < mn) mn = v;
    }
    R->minm[g] = mn;
  }
}

/* Horizon projection: request with current load kv contributes (kv + h) at offset h
 * while h <= c_hat, nothing after (eq. (wprofile-new), offsets counted from the current
 * step so that h = 0 reproduces L_g(k)). */
static void project(rstate *R, const orc_io *io, float *chat_out) {
  const orc_params *P = R->P;
  int32_t pw = pred_width(P);
  int g, h, j;
  for (g = 0; g < P->G; ++g) {
    for (h = 0; h <= P->H; ++h) R->Lh[g][h] = 0;
    for (j = 0; j < io->n[g]; ++j) {
      int64_t kv = io->kv[(int64_t)g * P->B + j];
      float c = 0.0f;
      if (P->H > 0) c = orc_chat(P->H, P->pred_mode, P->gate_pfin, io->pred + ((int64_t)g * P->B + j) * pw);
      if (chat_out) chat_out[(int64_t)g * P->B + j] = c;
      for (h = 0; h <= P->H; ++h)
        if ((float)h <= c) R->Lh[g][h] += kv + h;
    }
  }
}

int32_t orc_project(const orc_params *P, orc_io *io) {
  rstate R;
  int g, h;
  if (P->G < 1 || P->G > ORC_MAX_G || P->H < 0 || P->H > ORC_MAX_H) return -1;
  R.P = P;
  project(&R, io, io->chat);
  envelope(&R);
  margins(&R);
  for (g = 0; g < P->G; ++g) {
    for (h = 0; h <= P->H; ++h) {
      if (io->Lh) io->Lh[g * (P->H + 1) + h] = R.Lh[g][h];
      if (io->mh) io->mh[g * (P->H + 1) + h] = R.m[g][h];
    }
    if (io->minm) io->minm[g] = R.minm[g];
  }
  for (h = 0; h <= P->H; ++h)
    if (io->Mh) io->Mh[h] = R.Mh[h];
  return 0;
}

/* ------------------------------------------------------- Stage-2 subsets */

static int popcount32(uint32_t x) {
  int c = 0;
  while (x) {
    c += (int)(x & 1u);
    x >>= 1;
  }
  return c;
}

/* Exhaustive search over the non-empty subsets of the window (Appendix "Bit-set subset
 * selection": with R_max = 4 the deployed rule enumerates all 2^R_max subsets).  Subsets
 * are scanned in ascending mask order and a later one wins only if strictly better. */
static int32_t best_subset(const orc_params *P, const scorer *S, const int64_t *m_g, int64_t L_g,
                           int64_t cap_g, const int32_t *win_s, int32_t w, double *best_score) {
  int32_t best = 0;
  double bs = 0.0;
  int64_t kmax = cap_g < P->R_max ? cap_g : P->R_max;
  uint32_t mask;
  for (mask = 1; mask < (1u << w); ++mask) {
    int64_t delta = 0;
    int b;
    double f;
    if (popcount32(mask) > kmax) continue;
    for (b = 0; b < w; ++b)
      if (mask & (1u << b)) delta += win_s[b];
    if (P->token_watermark > 0 && L_g + delta > P->token_watermark) continue;
    f = score(S, m_g, delta);
    if (best == 0 || f > bs) {
      best = (int32_t)mask;
      bs = f;
    }
  }
  if (best_score) *best_score = bs;
  return best;
}

int32_t orc_best_subset(const orc_params *P, const int64_t *m_g, int64_t L_g, int32_t cap_g,
                        const int32_t *win_s, int32_t w, double *best_score) {
  scorer S;
  scorer_init(&S, P, P->force_float);
  return best_subset(P, &S, m_g, L_g, cap_g, win_s, w, best_score);
}

/* Appendix "Bit-set subset selection", "Reduction to reachable sums": F_g(Q) depends on Q only through
 * Delta_s(Q), so it suffices to know, for the cardinality limit k, which sums are reachable with at most k
 * requests of the window, to score each of them once and to recover a subset for the best one.  The table is the
 * 0/1-knapsack recurrence over the window in mask-bit order (entry [j][sum] is filled from [j-1][sum - s_b], j
 * descending so that request b is used at most once); instead of a reachable bit an entry holds the lowest mask
 * that attains it: a subset that uses request b has a higher mask than any subset of the requests before b, so an
 * entry, once filled, already holds its lowest mask, and a new entry takes the lowest mask of its predecessor
 * plus bit b.  Equal best scores resolve to the lowest mask, as in the scan over all masks. */
static int32_t best_subset_reach(const orc_params *P, const scorer *S, const int64_t *m_g, int64_t L_g,
                                 int64_t cap_g, const int32_t *win_s, int32_t w, double *best_score) {
  int64_t kmax = cap_g < P->R_max ? cap_g : P->R_max;
  int64_t top = 0, sum, j;
  int64_t *tab; /* [kmax + 1][top + 1]: lowest mask of a subset with at most j requests and that sum, -1 = none */
  int32_t best = 0;
  double bs = 0.0;
  int b;
  if (kmax > w) kmax = w;
  if (kmax < 1) {
    if (best_score) *best_score = 0.0;
    return 0;
  }
  { /* no subset of at most kmax requests sums to more than the kmax longest ones: the table ends there */
    uint8_t used[ORC_MAX_RMAX];
    memset(used, 0, sizeof used);
    for (j = 0; j < kmax; ++j) {
      int pick = -1;
      for (b = 0; b < w; ++b)
        if (!used[b] && (pick < 0 || win_s[b] > win_s[pick])) pick = b;
      used[pick] = 1;
      top += win_s[pick];
    }
  }
  if (top > ORC_DP_MAX_SUM) top = ORC_DP_MAX_SUM;
  tab = (int64_t *)malloc(sizeof(int64_t) * (size_t)(kmax + 1) * (size_t)(top + 1));
  for (j = 0; j <= kmax; ++j) {
    for (sum = 0; sum <= top; ++sum) tab[j * (top + 1) + sum] = -1;
    tab[j * (top + 1)] = 0; /* the empty subset */
  }
  for (b = 0; b < w; ++b) {
    int64_t s = win_s[b];
    for (j = kmax; j >= 1; --j)
      for (sum = top; sum >= s; --sum) {
        int64_t from = tab[(j - 1) * (top + 1) + (sum - s)];
        if (from >= 0 && tab[j * (top + 1) + sum] < 0) tab[j * (top + 1) + sum] = from | ((int64_t)1 << b);
      }
  }
  for (sum = 1; sum <= top; ++sum) {
    int64_t mask = tab[kmax * (top + 1) + sum];
    double f;
    if (mask < 0) continue;
    if (P->token_watermark > 0 && L_g + sum > P->token_watermark) continue;
    f = score(S, m_g, sum);
    if (best == 0 || f > bs || (f == bs && mask < (int64_t)(uint32_t)best)) {
      best = (int32_t)(uint32_t)mask;
      bs = f;
    }
  }
  free(tab);
  if (best_score) *best_score = bs;
  return best;
}

int32_t orc_best_subset_reach(const orc_params *P, const int64_t *m_g, int64_t L_g, int32_t cap_g,
                              const int32_t *win_s, int32_t w, double *best_score) {
  scorer S;
  scorer_init(&S, P, P->force_float);
  return best_subset_reach(P, &S, m_g, L_g, cap_g, win_s, w, best_score);
}

/* ---------------------------------------------------------------- a round */

typedef struct {
  int32_t s;
  int32_t idx; /* position in the arrival-ordered queue */
} qent;

/* waiting set ordered by prefill length, largest first; equal lengths keep arrival order */
static int cmp_qent(const void *a, const void *b) {
  const qent *x = (const qent *)a, *y = (const qent *)b;
  if (x->s != y->s) return x->s > y->s ? -1 : 1;
  return x->idx < y->idx ? -1 : (x->idx > y->idx ? 1 : 0);
}

static int32_t clamp_s(int32_t s) { return s < 1 ? 1 : (s > ORC_MAX_S ? ORC_MAX_S : s); }

typedef struct {
  rstate *R;
  orc_io *io;
  qent *ord;      /* sorted view */
  uint8_t *alive; /* per sorted position */
  int32_t n_sorted, n_alive;
  int64_t S_tot;
  int64_t stage1, pops, guard, wdrop, admitted;
  int32_t n_ev;
} round_t;

/* bind one waiting request (sorted position pos) to worker g: sticky from here on */
static void bind(round_t *T, int pos, int g) {
  const orc_params *P = T->R->P;
  orc_io *io = T->io;
  int32_t pw = queue_pred_width(P);
  int32_t idx = T->ord[pos].idx;
  int64_t slot = (int64_t)g * P->B + io->n[g];
  io->kv[slot] = T->ord[pos].s;
  io->rem[slot] = io->qo[idx];
  if (pw) memcpy(io->pred + slot * pw, io->qpred + (int64_t)idx * pw, sizeof(float) * (size_t)pw);
  if (P->H > 0 && P->pred_mode == 2) { /* first query of the estimator, at age 0 */
    io->pred[slot * 3 + 0] = orc_survival(P, 0);
    io->pred[slot * 3 + 1] = 0.0f;
    io->pred[slot * 3 + 2] = 0.0f;
  }
  io->n[g] += 1;
  T->R->cap[g] -= 1;
  T->S_tot -= 1;
  T->alive[pos] = 0;
  T->n_alive -= 1;
  T->admitted += 1;
  if (io->assign) io->assign[idx] = g;
}

/* load update after binding total length delta to g: the admitted load is added at every
 * horizon offset (constant-s_i approximation of Sec. 4.1), envelope and margins follow */
static void add_load(rstate *R, int g, int64_t delta) {
  int h;
  R->L[g] += delta;
  for (h = 0; h <= R->P->H; ++h) {
    R->Lh[g][h] += delta;
    if (R->Lh[g][h] > R->Mh[h]) R->Mh[h] = R->Lh[g][h];
  }
  margins(R);
}

static int admissible(const rstate *R, int g, int64_t s) {
  return R->P->token_watermark <= 0 || R->L[g] + s <= R->P->token_watermark;
}

/* argmax_i F_g({i}) over the alive, admissible waiting requests; equal scores resolve to
 * the lowest sorted position.  Returns -1 when none is admissible. */
static int best_single(const round_t *T, int g, double *f_out) {
  int pos, best = -1;
  double bf = 0.0;
  for (pos = 0; pos < T->n_sorted; ++pos) {
    double f;
    if (!T->alive[pos] || !admissible(T->R, g, T->ord[pos].s)) continue;
    f = score(&T->R->S, T->R->m[g], T->ord[pos].s);
    if (best < 0 || f > bf) {
      best = pos;
      bf = f;
    }
  }
  if (f_out) *f_out = bf;
  return best;
}

static void log_event(round_t *T, int g, int stage, int n_req, int64_t delta, double f) {
  if (T->io->events) {
    orc_event *e = &T->io->events[T->n_ev];
    e->g = g;
    e->stage = stage;
    e->n_req = n_req;
    e->pad = 0;
    e->delta = delta;
    e->score = f;
  }
  T->n_ev += 1;
}

static void drop_worker(round_t *T, int g) {
  T->S_tot -= T->R->cap[g];
  T->R->cap[g] = 0;
  T->wdrop += 1;
}

static int64_t imbalance(const int64_t *L, int G) {
  int64_t M = L[0], sum = 0;
  int g;
  for (g = 0; g < G; ++g) {
    if (L[g] > M) M = L[g];
    sum += L[g];
  }
  return (int64_t)G * M - sum; /* Sec. 3.1: I = G * M - sum_g L_g */
}

int32_t orc_route_step(const orc_params *P, orc_io *io) {
  rstate R;
  round_t T;
  int32_t pw = queue_pred_width(P);
  int g, i, pos, G = P->G;
  int32_t qlen, space, acc;
  int64_t st[ORC_NSTATS];

  if (G < 1 || G > ORC_MAX_G || P->H < 0 || P->H > ORC_MAX_H || P->R_max < 1 || P->R_max > ORC_MAX_RMAX ||
      P->B < 1 || P->max_wait < 1)
    return -1;
  memset(st, 0, sizeof st);
  memset(&T, 0, sizeof T);
  R.P = P;
  scorer_init(&R.S, P, P->force_float);

  /* arrivals join the waiting queue in arrival order; what does not fit is dropped */
  qlen = *io->qlen;
  space = P->max_wait - qlen;
  acc = io->a_count < space ? io->a_count : space;
  if (acc < 0) acc = 0;
  for (i = 0; i < acc; ++i) {
    io->qs[qlen + i] = clamp_s(io->a_s[i]);
    io->qo[qlen + i] = io->a_o[i] < 1 ? 1 : io->a_o[i];
    io->qid[qlen + i] = io->a_id ? io->a_id[i] : i;
    if (pw) memcpy(io->qpred + (int64_t)(qlen + i) * pw, io->a_pred + (int64_t)i * pw, sizeof(float) * (size_t)pw);
  }
  st[ORC_ST_DROPPED] = (io->a_count > 0 ? io->a_count : 0) - acc;
  qlen += acc;
  st[ORC_ST_QLEN] = qlen;

  for (i = 0; i < P->max_wait; ++i) {
    if (io->assign) io->assign[i] = -1;
    if (io->assign_id) io->assign_id[i] = i < qlen ? io->qid[i] : -1;
    if (io->best_g) io->best_g[i] = -1;
  }

  /* free slots (Alg. BR-0 / BR-H, first line) */
  T.S_tot = 0;
  for (g = 0; g < G; ++g) {
    R.L[g] = io->L[g];
    R.cap[g] = (int64_t)P->B - io->n[g];
    T.S_tot += R.cap[g];
  }
  st[ORC_ST_I_BEFORE] = imbalance(R.L, G);

  /* preparation: projected loads, envelope, margins (for H = 0 this is M and M - L_g) */
  project(&R, io, io->chat);
  envelope(&R);
  margins(&R);
  for (g = 0; g < G; ++g) {
    int h;
    for (h = 0; h <= P->H; ++h) {
      if (io->Lh) io->Lh[g * (P->H + 1) + h] = R.Lh[g][h];
      if (io->mh) io->mh[g * (P->H + 1) + h] = R.m[g][h];
    }
    if (io->minm) io->minm[g] = R.minm[g];
  }
  if (io->Mh) {
    int h;
    for (h = 0; h <= P->H; ++h) io->Mh[h] = R.Mh[h];
  }

  /* snapshot scores of every (waiting request, worker) pair and their two reductions */
  for (g = 0; g < G; ++g)
    if (io->best_i) io->best_i[g] = -1;
  {
    double bi_f[ORC_MAX_G];
    int32_t bi_s[ORC_MAX_G];
    for (i = 0; i < qlen; ++i) {
      int bg = -1;
      double bgf = 0.0;
      for (g = 0; g < G; ++g) {
        double f = score(&R.S, R.m[g], io->qs[i]);
        int ok = R.cap[g] > 0 && admissible(&R, g, io->qs[i]);
        if (io->F_i32 && !R.S.use_float) io->F_i32[(int64_t)i * G + g] = (int32_t)f;
        if (io->F_f32 && R.S.use_float) io->F_f32[(int64_t)i * G + g] = (float)f;
        if (!ok) continue;
        if (bg < 0 || f > bgf) {
          bg = g;
          bgf = f;
        }
        if (io->best_i) {
          int32_t cur = io->best_i[g];
          if (cur < 0 || f > bi_f[g] || (f == bi_f[g] && io->qs[i] > bi_s[g])) {
            io->best_i[g] = i;
            bi_f[g] = f;
            bi_s[g] = io->qs[i];
          }
        }
      }
      if (io->best_g) io->best_g[i] = bg;
    }
  }

  if (T.S_tot > 0 && qlen > 0) {
    T.R = &R;
    T.io = io;
    T.ord = (qent *)malloc(sizeof(qent) * (size_t)qlen);
    T.alive = (uint8_t *)malloc((size_t)qlen);
    T.n_sorted = T.n_alive = qlen;
    for (i = 0; i < qlen; ++i) {
      T.ord[i].s = io->qs[i];
      T.ord[i].idx = i;
      T.alive[i] = 1;
    }
    qsort(T.ord, (size_t)qlen, sizeof(qent), cmp_qent);

    /* Stage 1: greedy fill while free capacity is abundant */
    while (T.S_tot > P->S_greedy && T.n_alive > 0) {
      int bw = -1;
      double f;
      for (g = 0; g < G; ++g) { /* most free slots; then lightest; then lowest index */
        if (R.cap[g] <= 0) continue;
        if (bw < 0 || R.cap[g] > R.cap[bw] || (R.cap[g] == R.cap[bw] && R.L[g] < R.L[bw])) bw = g;
      }
      if (bw < 0) break;
      pos = best_single(&T, bw, &f);
      if (pos < 0) {
        drop_worker(&T, bw);
        continue;
      }
      bind(&T, pos, bw);
      log_event(&T, bw, 1, 1, T.ord[pos].s, f);
      add_load(&R, bw, T.ord[pos].s);
      T.stage1 += 1;
    }

    /* Stage 2: refined allocation over the workers that still have free slots */
    while (T.n_alive > 0) {
      int bw = -1, w = 0, b;
      int32_t win_s[ORC_MAX_RMAX], win_pos[ORC_MAX_RMAX], mask;
      double f = 0.0;
      for (g = 0; g < G; ++g) { /* priority (cap, horizon-min margin), both larger first */
        if (R.cap[g] <= 0) continue;
        if (bw < 0 || R.cap[g] > R.cap[bw] || (R.cap[g] == R.cap[bw] && R.minm[g] > R.minm[bw])) bw = g;
      }
      if (bw < 0) break;
      T.pops += 1;
      for (pos = 0; pos < T.n_sorted && w < P->R_max; ++pos)
        if (T.alive[pos]) {
          win_s[w] = T.ord[pos].s;
          win_pos[w] = pos;
          ++w;
        }
      if (w <= ORC_ENUM_RMAX)
        mask = best_subset(P, &R.S, R.m[bw], R.L[bw], R.cap[bw], win_s, w, &f);
      else
        mask = best_subset_reach(P, &R.S, R.m[bw], R.L[bw], R.cap[bw], win_s, w, &f);
      if (mask == 0 || f <= 0.0) { /* starvation guard: single best request anyway */
        T.guard += 1;
        pos = best_single(&T, bw, &f);
        if (pos < 0) {
          drop_worker(&T, bw);
          continue;
        }
        bind(&T, pos, bw);
        log_event(&T, bw, 3, 1, T.ord[pos].s, f);
        add_load(&R, bw, T.ord[pos].s);
      } else {
        int64_t delta = 0;
        int cnt = 0;
        for (b = 0; b < w; ++b)
          if ((uint32_t)mask & ((uint32_t)1 << b)) {
            bind(&T, win_pos[b], bw);
            delta += win_s[b];
            ++cnt;
          }
        log_event(&T, bw, 2, cnt, delta, f);
        add_load(&R, bw, delta);
      }
    }

    /* the waiting queue keeps the deferred requests in arrival order */
    {
      uint8_t *gone = (uint8_t *)calloc((size_t)qlen, 1);
      int32_t k = 0;
      for (pos = 0; pos < T.n_sorted; ++pos)
        if (!T.alive[pos]) gone[T.ord[pos].idx] = 1;
      for (i = 0; i < qlen; ++i) {
        if (gone[i]) continue;
        if (k != i) {
          io->qs[k] = io->qs[i];
          io->qo[k] = io->qo[i];
          io->qid[k] = io->qid[i];
          if (pw) memmove(io->qpred + (int64_t)k * pw, io->qpred + (int64_t)i * pw, sizeof(float) * (size_t)pw);
        }
        ++k;
      }
      qlen = k;
      free(gone);
    }
    free(T.ord);
    free(T.alive);
  }

  *io->qlen = qlen;
  for (g = 0; g < G; ++g) io->L[g] = R.L[g];

  st[ORC_ST_ADMITTED] = T.admitted;
  st[ORC_ST_DEFERRED] = qlen;
  st[ORC_ST_STAGE1] = T.stage1;
  st[ORC_ST_STAGE2_POPS] = T.pops;
  st[ORC_ST_GUARD] = T.guard;
  st[ORC_ST_WORKERS_DROPPED] = T.wdrop;
  st[ORC_ST_I_AFTER] = imbalance(R.L, G);
  {
    int64_t mx = R.L[0], mn = R.L[0];
    for (g = 0; g < G; ++g) {
      if (R.L[g] > mx) mx = R.L[g];
      if (R.L[g] < mn) mn = R.L[g];
      if (P->token_cap > 0 && R.L[g] > P->token_cap) st[ORC_ST_OVERCAP] += 1;
      if (R.L[g] >= ((int64_t)1 << 25)) st[ORC_ST_LOAD_RANGE] += 1;
    }
    st[ORC_ST_SPREAD] = mx - mn;
  }
  if (io->stats) memcpy(io->stats, st, sizeof st);
  if (io->n_events) *io->n_events = T.n_ev;
  return 0;
}

/* ------------------------------------------------------------- decode step */

/* Sec. 2.2: every active request advances by one decode iteration per step; its load grows
 * by one token (w^(j) = s + j - 1) and it leaves after o_i steps.  Lists stay dense and keep
 * their order. */
int32_t orc_advance(const orc_params *P, orc_io *io, int32_t n_steps) {
  int32_t pw = pred_width(P);
  int t, g, j;
  for (t = 0; t < n_steps; ++t) {
    for (g = 0; g < P->G; ++g) {
      int32_t k = 0;
      int64_t base = (int64_t)g * P->B;
      for (j = 0; j < io->n[g]; ++j) {
        int32_t kv = io->kv[base + j];
        int32_t rem = io->rem[base + j] - 1;
        if (rem <= 0) { /* finished: its whole KV footprint leaves the worker */
          io->L[g] -= kv;
          continue;
        }
        io->kv[base + k] = kv + 1;
        io->rem[base + k] = rem;
        io->L[g] += 1;
        if (pw && k != j)
          memmove(io->pred + (base + k) * pw, io->pred + (base + j) * pw, sizeof(float) * (size_t)pw);
        if (P->H > 0 && P->pred_mode == 2) {
          /* Appendix "Refresh logic": one more token generated; re-query every `refresh` tokens, in
           * between one step less of in-window contribution; falling below the floor re-queries at once */
          float *q = io->pred + (base + k) * 3;
          float age = q[1] + 1.0f, since = q[2] + 1.0f, c = q[0];
          if ((int64_t)since >= P->refresh) {
            c = orc_survival(P, (int64_t)age);
            since = 0.0f;
          } else {
            c = c - 1.0f;
            if (c < 1.0f) {
              c = orc_survival(P, (int64_t)age);
              since = 0.0f;
            }
          }
          q[0] = c;
          q[1] = age;
          q[2] = since;
        }
        ++k;
      }
      io->n[g] = k;
    }
  }
  return 0;
}

/* ------------------------------------------------------------- pool bypass */

/* Appendix "Pool-bypass deployment path for BR-0": every request that finishes prefill is scored
 * at once with the single-step score F_g(s) = s - G (s - m_g)_+ over all decode workers, against
 * the virtual load (everything already dispatched to the worker counts), and forwarded to the best
 * worker; the per-worker inflight cap is the slot limit B.  BR-0 only.  Equal scores resolve to the
 * lowest worker index (the paper is silent).  A request no worker can take joins the waiting queue. */
int32_t orc_route_bypass(const orc_params *P, orc_io *io) {
  int G = P->G, a, g;
  int64_t st[ORC_NSTATS];
  int32_t qlen = *io->qlen;
  int32_t pw = pred_width(P);
  int64_t L0[ORC_MAX_G];
  if (G < 1 || G > ORC_MAX_G || P->H != 0 || pw != 0) return -1;
  memset(st, 0, sizeof st);
  for (g = 0; g < G; ++g) L0[g] = io->L[g];
  st[ORC_ST_I_BEFORE] = imbalance(L0, G);
  st[ORC_ST_QLEN] = io->a_count;
  for (a = 0; a < io->a_count; ++a) {
    int64_t s = clamp_s(io->a_s[a]);
    int64_t M = io->L[0];
    int best = -1;
    int64_t bf = 0;
    for (g = 1; g < G; ++g)
      if (io->L[g] > M) M = io->L[g];
    for (g = 0; g < G; ++g) {
      int64_t f;
      if (io->n[g] >= P->B) continue;
      if (P->token_watermark > 0 && io->L[g] + s > P->token_watermark) continue;
      f = orc_score_br0(G, M - io->L[g], s);
      if (best < 0 || f > bf) {
        best = g;
        bf = f;
      }
    }
    if (best >= 0) {
      int64_t slot = (int64_t)best * P->B + io->n[best];
      io->kv[slot] = (int32_t)s;
      io->rem[slot] = io->a_o[a] < 1 ? 1 : io->a_o[a];
      io->n[best] += 1;
      io->L[best] += s;
      st[ORC_ST_ADMITTED] += 1;
      if (io->assign) io->assign[a] = best;
    } else if (qlen < P->max_wait) {
      io->qs[qlen] = (int32_t)s;
      io->qo[qlen] = io->a_o[a] < 1 ? 1 : io->a_o[a];
      io->qid[qlen] = io->a_id ? io->a_id[a] : a;
      ++qlen;
      if (io->assign) io->assign[a] = -1;
    } else {
      st[ORC_ST_DROPPED] += 1;
      if (io->assign) io->assign[a] = -2;
    }
  }
  *io->qlen = qlen;
  st[ORC_ST_DEFERRED] = qlen;
  for (g = 0; g < G; ++g) L0[g] = io->L[g];
  st[ORC_ST_I_AFTER] = imbalance(L0, G);
  {
    int64_t mx = L0[0], mn = L0[0];
    for (g = 0; g < G; ++g) {
      if (L0[g] > mx) mx = L0[g];
      if (L0[g] < mn) mn = L0[g];
      if (P->token_cap > 0 && L0[g] > P->token_cap) st[ORC_ST_OVERCAP] += 1;
      if (L0[g] >= ((int64_t)1 << 25)) st[ORC_ST_LOAD_RANGE] += 1;
    }
    st[ORC_ST_SPREAD] = mx - mn;
  }
  if (io->stats) memcpy(io->stats, st, sizeof st);
  return 0;
}

/* ------------------------------------------------------ comparison policies */

/* Output c of the SplitMix64 stream started at `key` (published output function and increment). */
uint64_t orc_hash64(uint64_t key, uint64_t c) {
  uint64_t z = key + (c + 1) * 0x9E3779B97F4A7C15ULL;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
  return z ^ (z >> 31);
}

/* the k-th eligible worker (free slot) in ascending index order, k counted from 0; `skip`: a worker left out */
static int kth_eligible(const orc_params *P, const orc_io *io, int k, int skip) {
  int g;
  for (g = 0; g < P->G; ++g) {
    if (io->n[g] >= P->B || g == skip) continue;
    if (k == 0) return g;
    --k;
  }
  return -1;
}

/* Sec. 6.1 "Baselines": Random, Round-Robin, Power-of-Two-Choices, Join-Shortest-Queue; see br_oracle.h for
 * the rules.  Requests leave the waiting queue in arrival order; lengths are never looked at. */
int32_t orc_route_baseline(const orc_params *P, orc_io *io, int32_t policy, uint64_t seed, int32_t cluster,
                           int32_t *pol_state) {
  int G = P->G, g, i;
  int32_t qlen, space, acc, taken = 0;
  int64_t st[ORC_NSTATS], L0[ORC_MAX_G];
  uint64_t key = seed ^ ((uint64_t)(uint32_t)cluster << 32);
  if (G < 1 || G > ORC_MAX_G || P->H != 0 || policy < 0 || policy > 3 || !pol_state) return -1;
  memset(st, 0, sizeof st);

  /* arrivals join the waiting queue in arrival order; what does not fit is dropped */
  qlen = *io->qlen;
  space = P->max_wait - qlen;
  acc = io->a_count < space ? io->a_count : space;
  if (acc < 0) acc = 0;
  for (i = 0; i < acc; ++i) {
    io->qs[qlen + i] = clamp_s(io->a_s[i]);
    io->qo[qlen + i] = io->a_o[i] < 1 ? 1 : io->a_o[i];
    io->qid[qlen + i] = io->a_id ? io->a_id[i] : i;
  }
  st[ORC_ST_DROPPED] = (io->a_count > 0 ? io->a_count : 0) - acc;
  qlen += acc;
  st[ORC_ST_QLEN] = qlen;
  for (i = 0; i < P->max_wait; ++i) {
    if (io->assign) io->assign[i] = -1;
    if (io->assign_id) io->assign_id[i] = i < qlen ? io->qid[i] : -1;
  }
  for (g = 0; g < G; ++g) L0[g] = io->L[g];
  st[ORC_ST_I_BEFORE] = imbalance(L0, G);

  for (i = 0; i < qlen; ++i) {
    int E = 0, pick = -1;
    for (g = 0; g < G; ++g)
      if (io->n[g] < P->B) ++E;
    if (E == 0) break; /* every worker is full: the rest keeps waiting */
    if (policy == ORC_POLICY_RR) {
      int k;
      for (k = 0; k < G; ++k) {
        g = (pol_state[0] + k) % G;
        if (io->n[g] < P->B) {
          pick = g;
          break;
        }
      }
      pol_state[0] = (pick + 1) % G;
    } else if (policy == ORC_POLICY_JSQ) {
      for (g = 0; g < G; ++g)
        if (io->n[g] < P->B && (pick < 0 || io->n[g] < io->n[pick])) pick = g;
    } else {
      uint64_t z = orc_hash64(key, (uint64_t)(uint32_t)pol_state[1]);
      uint32_t lo = (uint32_t)z, hi = (uint32_t)(z >> 32);
      int a = kth_eligible(P, io, (int)(((uint64_t)lo * (uint64_t)E) >> 32), -1);
      pol_state[1] += 1;
      pick = a;
      if (policy == ORC_POLICY_P2C && E > 1) {
        int b = kth_eligible(P, io, (int)(((uint64_t)hi * (uint64_t)(E - 1)) >> 32), a);
        if (io->n[b] < io->n[a]) pick = b;
      }
    }
    {
      int64_t slot = (int64_t)pick * P->B + io->n[pick];
      io->kv[slot] = io->qs[i];
      io->rem[slot] = io->qo[i];
      io->n[pick] += 1;
      io->L[pick] += io->qs[i];
      if (io->assign) io->assign[i] = pick;
      ++taken;
    }
  }
  /* the dispatched requests are a prefix of the queue: the rest moves up */
  for (i = taken; i < qlen; ++i) {
    io->qs[i - taken] = io->qs[i];
    io->qo[i - taken] = io->qo[i];
    io->qid[i - taken] = io->qid[i];
  }
  qlen -= taken;
  *io->qlen = qlen;
  st[ORC_ST_ADMITTED] = taken;
  st[ORC_ST_DEFERRED] = qlen;
  for (g = 0; g < G; ++g) L0[g] = io->L[g];
  st[ORC_ST_I_AFTER] = imbalance(L0, G);
  {
    int64_t mx = L0[0], mn = L0[0];
    for (g = 0; g < G; ++g) {
      if (L0[g] > mx) mx = L0[g];
      if (L0[g] < mn) mn = L0[g];
      if (P->token_cap > 0 && L0[g] > P->token_cap) st[ORC_ST_OVERCAP] += 1;
      if (L0[g] >= ((int64_t)1 << 25)) st[ORC_ST_LOAD_RANGE] += 1;
    }
    st[ORC_ST_SPREAD] = mx - mn;
  }
  if (io->stats) memcpy(io->stats, st, sizeof st);
  return 0;
}
