/*
 * BalanceRoute CPU oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, single-threaded implementation of the per-decode-step routing
 * decision of BalanceRoute (BR-0 and BR-H), written from the paper so that the
 * GPU path can be checked against it.  It shares no code with the GPU library
 * and must never be called from a product path: only tests, the smoke check and
 * the benchmark's CPU-baseline leg may use it.
 *
 * What it follows:
 *   - load model and sticky assignment:        Sec. 2.2 (workload profile, L_g(k))
 *   - BR-0 score:                              Sec. 3.1, eq. (br0-Fscore)
 *   - BR-0 two-stage procedure:                Sec. 3.2 and Appendix, Alg. BR-0
 *   - horizon score:                           Sec. 4.1, eq. (brh-Fscore)
 *   - BR-H two-stage procedure:                Sec. 4.2 and Appendix, Alg. BR-H
 *   - in-window contribution, projected loads: Appendix "Short-horizon prediction
 *     interface", eqs. (two-stage), (composite), (wprofile-new); gate and floor from
 *     Appendix "Refresh logic"
 *   - subset search of Stage 2:                Appendix "Bit-set subset selection" (every mask for windows of up
 *     to 16 requests; the optimum over reachable sums for wider ones)
 *   - pool-bypass dispatch:                    Appendix "Pool-bypass deployment path for BR-0"
 *   - empirical-survival estimator, refresh:   Appendix "Estimator realizations", "Refresh logic"
 *   - comparison policies (Random, RR, P2C, JSQ): Sec. 6.1 "Baselines" names them; their rules are stated below
 *
 * BR-0/BR-H are heuristics without an exactness claim, so the oracle is the
 * algorithm itself, step by step.  Integer quantities are int64; BR-H scores are
 * IEEE fp32 in a fixed evaluation order (compile with -ffp-contract=off).
 *
 * Pins (tests/test_oracle_*.py): closed form of the BR-0 score at its breakpoints;
 * score == drop of the imbalance G*M - sum(L); BR-H at H=0,(alpha,beta)=(1,G) == BR-0;
 * discounted-imbalance identity of the horizon score; survival-sum == two-stage
 * composite; eq. (composite) on a supplied (p_fin, mu_rem) against fp64 and at its corners;
 * subset enumeration == best over reachable sums (for windows of up to 16 requests the sums are
 * built by the shift-OR recurrence of Appendix "Bit-set subset selection"); the reachable-sum search of wide
 * windows == the scan of all masks wherever both apply, == brute force over all masks of 20-request windows; structural invariants
 * of a round (sticky, disjoint, slot limit, load conservation, work conservation,
 * telescoping of the imbalance); brute force over all assignments on tiny instances.
 *
 * Parity unpinned (the paper is silent; fixed here by choice): worker / request / subset tie-breaks, the Stage-1 threshold default,
 * the descending sort of the waiting set, the token-watermark admission filter, the
 * waiting-queue cap with counted drops.
 */
#ifndef BR_ORACLE_H
#define BR_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ORC_MAX_G 64
#define ORC_MAX_H 128
#define ORC_MAX_RMAX 32
#define ORC_ENUM_RMAX 16     /* windows up to here: every subset mask is scanned; beyond: reachable sums */
#define ORC_DP_MAX_SUM 131071 /* windows beyond ORC_ENUM_RMAX: the table of reachable sums ends here */
#define ORC_NSTATS 16
#define ORC_MAX_S 32768

/* stats slots (int64 each) */
enum {
  ORC_ST_ADMITTED = 0,
  ORC_ST_DEFERRED = 1,
  ORC_ST_DROPPED = 2,
  ORC_ST_STAGE1 = 3,
  ORC_ST_STAGE2_POPS = 4,
  ORC_ST_GUARD = 5,
  ORC_ST_OVERCAP = 6,
  ORC_ST_I_BEFORE = 7,
  ORC_ST_I_AFTER = 8,
  ORC_ST_SPREAD = 9,
  ORC_ST_QLEN = 10,
  ORC_ST_WORKERS_DROPPED = 11,
  ORC_ST_LOAD_RANGE = 12 /* workers whose load after the call is 2^25 or more (outside the stated input range) */
};

typedef struct {
  int32_t G, B, max_wait, H;
  int32_t R_max, S_greedy;
  int32_t token_watermark, token_cap;
  int32_t pred_mode; /* 0: per-step hazards p[1..H]; 1: direct c_hat (one float);
                        2: empirical-survival estimator maintained per request (c_hat, age, since-refresh);
                        3: the two-stage pair (p_fin, mu_rem) per request, combined by eq. (composite) */
  int32_t force_float; /* evaluate the horizon score in fp32 even when H == 0 (reduction check) */
  float alpha, beta, gamma, gate_pfin;
  /* pred_mode 2: sorted history of output lengths, its prefix sums (hist_sum[k] = sum of the first k),
   * and the refresh period Delta T in generated tokens */
  const int32_t *hist;
  const int64_t *hist_sum;
  int32_t hist_n;
  int32_t refresh;
} orc_params;

/* One admission event (a single request in Stage 1, a subset in Stage 2). */
typedef struct {
  int32_t g;
  int32_t stage;    /* 1 or 2; 3 = starvation guard inside Stage 2 */
  int32_t n_req;    /* requests bound by this event */
  int32_t pad;
  int64_t delta;    /* sum of their prefill lengths */
  double score;     /* F_g(Q) at the moment of the decision (exact for both score types) */
} orc_event;

/* All arrays of ONE instance; every pointer is caller-owned host memory. */
typedef struct {
  /* active state (in/out) */
  int64_t *L;      /* [G] */
  int32_t *n;      /* [G] */
  int32_t *kv;     /* [G][B] dense lists */
  int32_t *rem;    /* [G][B] */
  float *pred;     /* [G][B][P] or NULL when H == 0 */
  /* waiting queue in arrival order (in/out) */
  int32_t *qlen;   /* [1] */
  int32_t *qs, *qo, *qid; /* [max_wait] */
  float *qpred;    /* [max_wait][P] */
  /* arrivals of this step (in) */
  int32_t a_count;
  int32_t pad0;
  const int32_t *a_s, *a_o, *a_id;
  const float *a_pred;
  /* outputs, each optional (NULL to skip) */
  int32_t *assign;     /* [max_wait] worker per queue entry (order after append), -1 = deferred */
  int32_t *assign_id;  /* [max_wait] id of that queue entry, -1 beyond the queue */
  int64_t *stats;      /* [ORC_NSTATS] */
  int32_t *F_i32;      /* [max_wait][G] snapshot scores, BR-0 */
  float *F_f32;        /* [max_wait][G] snapshot scores, BR-H */
  int32_t *best_g;     /* [max_wait] */
  int32_t *best_i;     /* [G] */
  int64_t *Lh;         /* [G][H+1] projected loads at step start */
  int64_t *Mh;         /* [H+1] envelope */
  int64_t *mh;         /* [G][H+1] margins */
  int64_t *minm;       /* [G] */
  float *chat;         /* [G][B] in-window contribution per active slot */
  orc_event *events;   /* [max_wait] */
  int32_t *n_events;   /* [1] */
} orc_io;

/* scores */
int64_t orc_score_br0(int64_t G, int64_t m, int64_t delta);
float orc_score_brh(int32_t H, float alpha, float beta, float gamma, const int64_t *m, int64_t delta);
/* in-window contribution from the prediction inputs of one request */
float orc_chat(int32_t H, int32_t pred_mode, float gate_pfin, const float *p);
/* empirical-survival estimate of the in-window contribution at age a (pred_mode 2) */
float orc_survival(const orc_params *P, int64_t age);
/* Stage-2 subset search on an explicit window; returns the chosen mask (0 = none feasible) */
int32_t orc_best_subset(const orc_params *P, const int64_t *m_g, int64_t L_g, int32_t cap_g,
                        const int32_t *win_s, int32_t w, double *best_score);
/* The same search by the reduction of Appendix "Bit-set subset selection": the score of a subset depends on its
 * sum only, so the optimum is the best score over the sums reachable with 1..k requests of the window; among the
 * subsets that attain it the lowest mask is returned, as by the scan of all masks.  Subsets whose sum exceeds
 * ORC_DP_MAX_SUM are not candidates (the table of reachable sums is sized by that bound).  Any window size up to
 * ORC_MAX_RMAX; the round uses it for windows beyond ORC_ENUM_RMAX. */
int32_t orc_best_subset_reach(const orc_params *P, const int64_t *m_g, int64_t L_g, int32_t cap_g,
                              const int32_t *win_s, int32_t w, double *best_score);

int32_t orc_project(const orc_params *P, orc_io *io);
int32_t orc_route_step(const orc_params *P, orc_io *io);
int32_t orc_advance(const orc_params *P, orc_io *io, int32_t n_steps);
/* Pool-bypass dispatch (Appendix "Pool-bypass deployment path for BR-0"): arrivals are placed one
 * at a time, in order, on argmax_g F_g(s) over the workers with a free slot; io->assign[a] gets the
 * worker of arrival a, -1 if it had to join the waiting queue, -2 if that was full too. */
int32_t orc_route_bypass(const orc_params *P, orc_io *io);

/* ---- comparison policies (Sec. 6.1 "Baselines": Random, Round-Robin, Power-of-Two-Choices, Join-Shortest-Queue) ----
 * Workload-unaware dispatch: waiting requests are taken in arrival order and each goes to a worker chosen among
 * those with a free slot (eligible workers), without looking at any length:
 *   ORC_POLICY_RANDOM  uniform over the eligible workers;
 *   ORC_POLICY_RR      the first eligible worker at or after a cursor, cyclically; the cursor moves one past it;
 *   ORC_POLICY_P2C     two distinct eligible workers drawn uniformly, the one holding fewer requests (the first
 *                      drawn on equal counts); the only eligible worker if there is one;
 *   ORC_POLICY_JSQ     the eligible worker holding the fewest requests, lowest index on equal counts.
 * Dispatch stops when no worker has a free slot; what is left keeps waiting, in arrival order.
 * Random draws are counter-based: draw number c of cluster i under `seed` is the SplitMix64 output function
 * (Steele, Lea, Flood 2014: z = x; z = (z ^ z >> 30) * 0xBF58476D1CE4E5B9; z = (z ^ z >> 27) * 0x94D049BB133111EB;
 * z ^ z >> 31) applied to x = (seed ^ i << 32) + (c + 1) * 0x9E3779B97F4A7C15, i.e. output c of the SplitMix64
 * stream started at seed ^ i << 32.  A 32-bit half u picks index (u * E) >> 32 among E candidates in ascending
 * worker order; P2C uses the low half for the first pick and the high half for the second (among the other
 * E - 1).  pol_state[0] is the round-robin cursor, pol_state[1] the number of draws made so far; both persist
 * across calls (in/out). */
enum { ORC_POLICY_RANDOM = 0, ORC_POLICY_RR = 1, ORC_POLICY_P2C = 2, ORC_POLICY_JSQ = 3 };
uint64_t orc_hash64(uint64_t key, uint64_t c);
int32_t orc_route_baseline(const orc_params *P, orc_io *io, int32_t policy, uint64_t seed, int32_t cluster,
                           int32_t *pol_state);

#ifdef __cplusplus
}
#endif
#endif
