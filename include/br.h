/*
 * BalanceRoute route-step library for MI355X (gfx950): C ABI.
 *
 * The library keeps, in caller-provided device memory, the cluster snapshot of
 * eq. (cluster-snapshot) (Sec. 5) for `n_inst` independent clusters: per worker g
 * the active set A_g with its load L_g (Sec. 2.2) and, for BR-H, each active request's
 * prediction inputs; plus the waiting set R_wait in arrival order.  One call to
 * br_route_step runs one scheduling round of Alg. BR-0 (H == 0) or Alg. BR-H (H > 0)
 * (Appendix "Algorithm Pseudocode") on every cluster; br_advance_decode applies the
 * decode step of Sec. 2.2 (each active request grows by one token and leaves after its
 * output length).  Call order per decode step k: route, then advance.
 *
 * Conventions
 *  - Every pointer inside br_config / br_init_state / br_arrivals / br_step_out is a
 *    DEVICE pointer unless stated otherwise; the structs themselves are host memory.
 *  - The library allocates and frees no device memory and never synchronises the
 *    stream: all work is enqueued on `stream`; outputs are valid once the caller has
 *    synchronised it.  Buffers passed to a call must stay alive until that work ran.
 *  - The only host allocation the library owns is the opaque br_ctx.
 *  - Every entry point returns BR_OK or a negative error code; nothing is printed,
 *    nothing aborts.  Data-dependent conditions (a full waiting queue, a worker that
 *    can take nothing) are not errors: they are counted in the stats block.
 *  - Limits: G <= 64, B <= 1024, max_wait <= 2048, H <= 128 (H <= 8 with pred_mode 0),
 *    R_max <= 32 (R_max <= 16 when H > 8), prefill length in [1, 32768] (values outside are clamped on arrival),
 *    per-worker load < 2^25.
 */
#ifndef BR_H
#define BR_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BR_MAX_G 64
#define BR_MAX_B 1024
#define BR_MAX_WAIT 2048
#define BR_MAX_H 128
#define BR_MAX_RMAX 32
#define BR_DP_MAX_SUM 131071 /* windows beyond 16 requests: largest total prefill length a Stage-2 subset may have */
#define BR_MAX_S 32768
#define BR_NSTATS 16
#define BR_NKERNELS 7
#define BR_STATIC_MAX_INST 16          /* most clusters br_route_step_static serves */
#define BR_STATIC_SCRATCH_BYTES 1441792 /* device memory the library holds per GPU for it, until the process ends */

enum {
  BR_OK = 0,
  BR_EINVAL = -1, /* null pointer, limit exceeded, inconsistent sizes */
  BR_ENOMEM = -2, /* workspace smaller than br_workspace_bytes() */
  BR_EHIP = -3,   /* a HIP call failed; code kept for br_last_hip_error() */
  BR_ELIMIT = -4  /* br_route_step_static: the context is larger than the fixed scratch array serves */
};

/* Slots of the per-instance stats block (int64 each). */
enum {
  BR_ST_ADMITTED = 0,        /* requests bound to a worker in this round */
  BR_ST_DEFERRED = 1,        /* requests left waiting after the round */
  BR_ST_DROPPED = 2,         /* arrivals that did not fit the waiting-queue cap */
  BR_ST_STAGE1 = 3,          /* admissions made by Stage 1 (greedy fill) */
  BR_ST_STAGE2_POPS = 4,     /* workers popped in Stage 2 */
  BR_ST_GUARD = 5,           /* pops resolved by the starvation guard */
  BR_ST_OVERCAP = 6,         /* workers whose load exceeds token_cap after the round */
  BR_ST_I_BEFORE = 7,        /* imbalance G*max(L) - sum(L) (Sec. 3.1) before the round */
  BR_ST_I_AFTER = 8,         /* ... after the round */
  BR_ST_SPREAD = 9,          /* max(L) - min(L) after the round (Sec. 6.1 "average imbalance") */
  BR_ST_QLEN = 10,           /* waiting requests considered (after the arrivals joined) */
  BR_ST_WORKERS_DROPPED = 11, /* workers set aside because no waiting request was admissible */
  BR_ST_LOAD_RANGE = 12       /* workers whose load after the call is 2^25 or more: outside the input range stated
                                 above.  The kernels order workers by keys that pack a load into 25 bits, so from the
                                 round that reports a non-zero count on the choice of worker may differ from
                                 Alg. BR-0 / BR-H (loads, lists and counters stay consistent); keep B * (longest
                                 KV length) below 2^25 */
};

/* Kernel ids for br_profile_read(). */
enum {
  BR_K_PROJECT = 0, /* projected loads over the horizon (BR-H preparation) */
  BR_K_SCORE = 1,   /* F-score matrix + stage-one reductions */
  BR_K_ASSIGN = 2,  /* sequential two-stage assignment */
  BR_K_ADVANCE = 3, /* decode step */
  BR_K_INIT = 4,
  BR_K_BYPASS = 5,  /* pool-bypass dispatch */
  BR_K_BASELINE = 6 /* comparison policies */
};

/* Comparison policies of br_route_baseline (Sec. 6.1, "Baselines"). */
enum { BR_POLICY_RANDOM = 0, BR_POLICY_RR = 1, BR_POLICY_P2C = 2, BR_POLICY_JSQ = 3 };

typedef struct br_ctx br_ctx; /* opaque; host object owned by the library */

/*
 * Static configuration (Sec. 2.2 for G, B; Alg. BR-0/BR-H inputs for the rest).
 */
typedef struct {
  int32_t n_inst;          /* independent clusters handled per call, >= 1 */
  int32_t G;               /* DP workers per cluster, 1..64 */
  int32_t B;               /* max concurrent requests per worker (slot limit), 1..1024 */
  int32_t max_wait;        /* capacity of the waiting queue per cluster, 1..2048 */
  int32_t H;               /* lookahead horizon, 0..128; 0 selects BR-0 (exact integers); beyond 8 the
                              per-offset state moves from registers to on-chip memory (same results,
                              other kernels) and pred_mode must not be 0 */
  int32_t S_greedy;        /* Stage 1 runs while total free slots > S_greedy; >= 0 */
  int32_t R_max;           /* Stage-2 candidate window and subset size, 1..32 (1..16 when H > 8).  The search is exact:
                              windows of up to 16 requests scan every subset; wider ones (Appendix "Bit-set subset
                              selection") score every sum reachable with the allowed number of requests, up to
                              BR_DP_MAX_SUM tokens (subsets with a larger total are not candidates), and return the
                              same subset the scan would: best score, lowest mask in window order.  R_max > 16 adds
                              16 KB + 144 KB x min(B, R_max) of workspace per cluster (br_workspace_bytes says) */
  int32_t token_watermark; /* 0 = off; else a request is admissible on g only if L_g + s <= watermark */
  int32_t token_cap;       /* 0 = off; reporting only (BR_ST_OVERCAP) */
  int32_t pred_mode;       /* H > 0: 0 = per-step termination hazards p[1..H] per request,
                              1 = one float per request holding c_hat directly,
                              2 = c_hat maintained by the library with the empirical-survival
                                  estimator and the refresh rules of Appendix "Refresh logic"
                                  (arrivals carry no prediction inputs; needs hist below),
                              3 = two floats per request, the two stages (p_fin, mu_rem) of Appendix
                                  "Short-horizon prediction interface": c_hat = (1 - p_fin) H + p_fin mu_rem
                                  (eq. (composite)), gate on p_fin, floor 1, clip H */
  float alpha, beta, gamma; /* horizon score parameters, eq. (brh-Fscore); ignored when H == 0
                               (BR-0 is (1, G)); alpha > 0, beta >= 0, 0 < gamma <= 1 */
  float gate_pfin;          /* confidence gate on p_fin (Appendix "Refresh logic"); <= 0 disables */
  void *stream;             /* hipStream_t, borrowed for the life of the context (NULL = default) */
  void *workspace;          /* device memory, >= br_workspace_bytes() bytes, 256-byte aligned, borrowed */
  uint64_t workspace_bytes;
  /* pred_mode 2 only (Appendix "Estimator realizations", empirical-survival): the output lengths of
   * a training corpus, sorted ascending, and their prefix sums (hist_sum[k] = sum of the first k
   * lengths, hist_n + 1 entries); device memory, borrowed until br_free.  hist_n in [1, 2^20]. */
  const int32_t *hist;
  const int64_t *hist_sum;
  int32_t hist_n;
  int32_t refresh_period;   /* Delta T: generated tokens between two queries of the estimator, >= 1 */
} br_config;

/*
 * Optional active sets at step 0.  Dense lists: slots [0, n[i][g]) of worker g are used.
 * n [n_inst][G]; kv, rem [n_inst][G][B]; pred [n_inst][G][B][P] with P = H (pred_mode 0),
 * 1 (pred_mode 1), 2 (pred_mode 3) or 3 (pred_mode 2: c_hat, tokens generated so far, tokens since the last
 * estimator query), NULL when H == 0.  kv = current KV length (s_i + a_i), rem = decode
 * steps still to run (>= 1).  Copied into the workspace by br_init.
 */
typedef struct {
  const int32_t *n;
  const int32_t *kv;
  const int32_t *rem;
  const float *pred;
} br_init_state;

/*
 * Requests that finished prefill since the previous round (they join R_wait in this order).
 * count [n_inst]; s, o, id [n_inst][arr_cap]; pred [n_inst][arr_cap][Pq] with Pq = H (pred_mode 0),
 * 1 (pred_mode 1), 2 (pred_mode 3) or 0 (pred_mode 2 and BR-0: pred is ignored).
 * s = prefill length s_i; o = output length o_i (never read by the routing decision, only
 * stored for br_advance_decode; values < 1 count as 1); id = caller's request handle
 * (NULL: the position within this batch is used).
 */
typedef struct {
  const int32_t *count;
  const int32_t *s;
  const int32_t *o;
  const int32_t *id;
  const float *pred;
  int32_t arr_cap; /* row stride of s/o/id/pred; count[i] > arr_cap is read as arr_cap */
  int32_t pad;
} br_arrivals;

/*
 * Outputs of one round; every pointer may be NULL to skip that output.
 * Queue positions refer to the waiting queue after this round's arrivals joined it.
 *  assign    [n_inst][max_wait]    worker the entry was bound to, -1 = still waiting / no entry
 *  assign_id [n_inst][max_wait]    id of the entry, -1 = no entry
 *  stats     [n_inst][BR_NSTATS]   int64 counters, see BR_ST_*
 *  F         [n_inst][max_wait][G] score of every (waiting request, worker) pair on the
 *                                  step-start snapshot: int32 when H == 0 (eq. (br0-Fscore)),
 *                                  float when H > 0 (eq. (brh-Fscore)); rows >= qlen untouched
 *  best_g    [n_inst][max_wait]    argmax_g F over workers that have a free slot and can admit
 *                                  the request (lowest g on ties), -1 if none
 *  best_i    [n_inst][G]           queue position of argmax_i F_g({i}) over admissible requests
 *                                  (larger s, then earlier arrival on ties), -1 if none / no slot
 */
typedef struct {
  int32_t *assign;
  int32_t *assign_id;
  int64_t *stats;
  void *F;
  int32_t *best_g;
  int32_t *best_i;
} br_step_out;

/*
 * Where the state lives inside the workspace (byte offsets), for inspection by tests and
 * tools.  All arrays are int32 except pred/qpred (float).
 *  L, n [n_inst][G];  kv, rem [n_inst][G][B_stride];  pred [n_inst][G][B_stride][P]
 *  qlen [n_inst];  qs, qo, qid [n_inst][max_wait];  qpred [n_inst][max_wait][Pq]
 *  Lh, mh [n_inst][G][H+1];  Mh [n_inst][H+1];  minm [n_inst][G]   (written when H > 0)
 */
typedef struct {
  uint64_t L, n, kv, rem, pred, qlen, qs, qo, qid, qpred, Lh, Mh, mh, minm;
  uint64_t total_bytes;
  int32_t B_stride, P, Pq, pad;
} br_layout;

/* Bytes of workspace a configuration needs (0 if the configuration is invalid). Host only. */
uint64_t br_workspace_bytes(const br_config *cfg);

/*
 * Create a context.  Validates cfg, lays the state out in cfg->workspace, enqueues the
 * kernels that clear it and, if `init` is given, load the initial active sets (L_g is
 * computed as the sum of kv).  *out is set only on BR_OK.
 */
int32_t br_init(const br_config *cfg, const br_init_state *init, br_ctx **out);

/*
 * One scheduling round on every cluster (Alg. BR-0 / BR-H): the arrivals join the waiting
 * queue (what exceeds max_wait is dropped and counted), the preparation step projects the
 * loads over the horizon (BR-H), all (request, worker) pairs are scored on the snapshot,
 * Stage 1 and Stage 2 bind requests to workers (sticky: a bound request occupies a slot of
 * that worker until it finishes), and the queue keeps the deferred requests in arrival
 * order.  `in` may be NULL (no arrivals); `out` may be NULL.
 */
int32_t br_route_step(br_ctx *ctx, const br_arrivals *in, const br_step_out *out);

/*
 * n_steps decode steps (Sec. 2.2): every active request's KV length and its worker's load
 * grow by one per step; a request whose remaining steps reach zero leaves and frees its
 * slot.  n_steps >= 0.
 */
int32_t br_advance_decode(br_ctx *ctx, int32_t n_steps);

/*
 * One decode step of the serving loop in a single call: the round of br_route_step followed by
 * n_steps decode steps of br_advance_decode (Sec. 2.2; Alg. BR-0 / Alg. BR-H), with exactly their
 * results: same outputs (written as br_route_step writes them, statistics describe the state
 * right after the round) and same workspace contents afterwards as the two calls in sequence.
 * Where the shape allows, the assignment launch itself applies the decode steps (the wave that has
 * routed a cluster goes on to that cluster's lists, so clusters that finish their round early stream
 * their lists while others are still routing; small BR-0 batches use a second wave per cluster for
 * them); candidate windows beyond 8 requests and long-horizon rounds that several waves share are
 * followed by the decode kernel as a launch of its own on the same stream.
 * Arguments, ownership and errors as for br_route_step; n_steps >= 0 (0: identical to
 * br_route_step), BR_EINVAL otherwise.
 */
int32_t br_route_advance(br_ctx *ctx, const br_arrivals *in, const br_step_out *out, int32_t n_steps);

/*
 * br_route_step for callers that cannot allocate and cannot hand the library scratch space of their own choosing:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, outputs and
 * workspace contents afterwards as br_route_step (inputs and outputs are still the caller's buffers).  The one
 * difference: the partial results of the stage-one reductions for a few clusters with long queues (per-group best
 * worker per request, per-tile best request per worker) go to a fixed device array inside the library
 * (BR_STATIC_SCRATCH_BYTES; every GPU the library runs on holds its own copy until the process ends) instead of the
 * private tail of the workspace.  The call makes no hipMalloc / hipFree, creates no event (launches are not
 * bracketed even while br_profile_enable is on) and allocates no host memory.
 * Limit: contexts of at most BR_STATIC_MAX_INST clusters (any G, max_wait, H within the library's limits);
 * larger ones return BR_ELIMIT and nothing is enqueued.  BR_EHIP if the array's address could not be resolved
 * when the context was created (br_last_hip_error has the code).
 * All contexts on one GPU share the array: calls that may overlap on that GPU (different streams, different
 * threads) race on it and must be serialised by the caller; successive calls on one stream are safe, and nothing
 * needs clearing between them (every entry that is read is written first by the same call).
 */
int32_t br_route_step_static(br_ctx *ctx, const br_arrivals *in, const br_step_out *out);

/*
 * Pool-bypass dispatch for BR-0 (Appendix "Pool-bypass deployment path for BR-0"): instead of
 * waiting in the pool for a scheduling round, each arrival is placed at once, in order, on
 * argmax_g F_g(s) with F_g(s) = s - G (s - m_g)_+ (eq. (br0-Fscore)) over the workers that have a
 * free slot (and pass the token watermark), against the virtual load: everything already
 * dispatched to a worker counts.  The per-worker inflight cap is the slot limit B.  Equal scores
 * go to the lowest worker index.  An arrival no worker can take joins the waiting queue (a later
 * br_route_step serves it); if that is full it is dropped and counted.
 * Requires H == 0 and in->arr_cap <= BR_MAX_WAIT (else BR_EINVAL).
 * out->assign is [n_inst][in->arr_cap], per ARRIVAL: worker, -1 = queued, -2 = dropped; entries
 * at or beyond count[i] are left untouched.  out->stats as in br_route_step (BR_ST_QLEN = arrivals
 * considered; stage counters zero).  Other outputs are ignored.
 */
int32_t br_route_bypass(br_ctx *ctx, const br_arrivals *in, const br_step_out *out);

/*
 * One dispatch round of a comparison policy (Sec. 6.1 "Baselines": Random, Round-Robin, Power-of-Two-Choices,
 * Join-Shortest-Queue, the load-balancing policies BalanceRoute is measured against) on the same cluster
 * state, so that a replay can report the per-step imbalance (BR_ST_SPREAD, the paper's "average imbalance" is its
 * trace mean) of every policy side by side.  The arrivals join the waiting queue as in br_route_step; then the
 * waiting requests are taken in arrival order and each is bound to a worker chosen among those with a free slot,
 * without looking at any length:
 *   BR_POLICY_RANDOM  uniform over the eligible workers;
 *   BR_POLICY_RR      the first eligible worker at or after a per-cluster cursor, cyclically; the cursor then
 *                     stands one past it;
 *   BR_POLICY_P2C     two distinct eligible workers drawn uniformly, the one holding fewer requests (the first
 *                     drawn on equal counts); the only eligible worker if there is just one;
 *   BR_POLICY_JSQ     the eligible worker holding the fewest requests, lowest index on equal counts.
 * Dispatch stops when every worker is full; the rest keeps waiting in arrival order.  The token watermark is
 * not applied (these policies are workload-unaware).  Draws are counter-based and reproducible: draw c of
 * cluster i is SplitMix64 output c of the stream started at seed ^ (i << 32) (output function
 * z ^= z >> 30, z *= 0xBF58476D1CE4E5B9, z ^= z >> 27, z *= 0x94D049BB133111EB, z ^= z >> 31 on
 * state = start + (c + 1) * 0x9E3779B97F4A7C15); a 32-bit half u picks index (u * E) >> 32 among E candidates in
 * ascending worker order, low half first.  Cursor and draw count live in the workspace and persist across calls.
 * Requires H == 0 (BR_EINVAL otherwise, and for an unknown policy).  out->assign / assign_id / stats as in
 * br_route_step (stage counters zero); other outputs are ignored.
 */
int32_t br_route_baseline(br_ctx *ctx, const br_arrivals *in, const br_step_out *out, int32_t policy, uint64_t seed);

/* Destroy the context (host memory only; the workspace stays the caller's). NULL is allowed. */
void br_free(br_ctx *ctx);

/* The hipError_t of the last failed HIP call on this context (0 if none). */
int32_t br_last_hip_error(const br_ctx *ctx);

/* Fill *out with the workspace layout of this context. */
int32_t br_get_layout(const br_ctx *ctx, br_layout *out);

/*
 * Per-kernel timing with HIP events on the context's stream.  br_profile_enable(ctx, 1)
 * brackets every subsequent kernel launch with an event pair; br_profile_read synchronises
 * on the recorded events, adds their durations into ms[BR_NKERNELS] / launches[BR_NKERNELS]
 * (host arrays) and forgets them.  Off by default.
 */
int32_t br_profile_enable(br_ctx *ctx, int32_t on);
int32_t br_profile_read(br_ctx *ctx, double *ms, int64_t *launches);

#ifdef __cplusplus
}
#endif
#endif /* BR_H */
