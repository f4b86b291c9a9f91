// Shared tail of the assignment kernels: writes the admitted requests into their workers'
// lists, emits the per-entry outputs in arrival order, compacts the waiting queue in place and
// stores worker state and statistics.  Everything here is lane-parallel; `adm` (by sorted
// position: worker << 16 | slot, or -1) and the sorted keys in `skey` come from the round.
#pragma once

#include "br_device.h"
#include "br_score_wave.h"

#define BR_STAT(o, inst, k) (o).stats[(int64_t)(inst) * 16 + (k)]

struct BrRoundCounts {
  int admitted, stage1, pops, guard, wdrop;
  long long I_before;
};

// What the tail needs of the kernel arguments.  The assignment kernels take (BrParams, BrArr,
// BrOut) by value; keeping all of that in scalar registers across the admission loops starves
// them, so the tail reads its own copy from the kernel-argument segment when it starts.
struct BrTailArgs {
  int32_t *L, *n, *kv, *rem;
  float *pred;
  int32_t *qlen, *qs, *qo, *qid;
  float *qpred;
  const int32_t *as, *ao, *aid;
  const float *apred;
  int32_t *assign, *assign_id;
  long long *stats;
  int32_t G, B, Bs, Q, P, Pq, C, arr_cap, adv_t;
};

static_assert(sizeof(BrParams) == 256 && sizeof(BrArr) == 48 && sizeof(BrOut) == 48, "kernel argument layout");

__device__ __forceinline__ BrTailArgs br_tail_args() {
  typedef __attribute__((address_space(4))) const char kchar_t;
  typedef __attribute__((address_space(4))) const BrParams kparams_t;
  typedef __attribute__((address_space(4))) const BrArr karr_t;
  typedef __attribute__((address_space(4))) const BrOut kout_t;
  kchar_t *ka = (kchar_t *)__builtin_amdgcn_kernarg_segment_ptr();
  asm volatile("" : "+s"(ka));  // the loads below may not move above this point
  kparams_t *kp = (kparams_t *)ka;
  karr_t *kaa = (karr_t *)(ka + sizeof(BrParams));
  kout_t *ko = (kout_t *)(ka + sizeof(BrParams) + sizeof(BrArr));
  BrTailArgs t;
  t.L = kp->L, t.n = kp->n, t.kv = kp->kv, t.rem = kp->rem, t.pred = kp->pred;
  t.qlen = kp->qlen, t.qs = kp->qs, t.qo = kp->qo, t.qid = kp->qid, t.qpred = kp->qpred;
  t.as = kaa->s, t.ao = kaa->o, t.aid = kaa->id, t.apred = kaa->pred;
  t.assign = ko->assign, t.assign_id = ko->assign_id, t.stats = ko->stats;
  t.G = kp->G, t.B = kp->B, t.Bs = kp->Bs, t.Q = kp->Q, t.P = kp->P, t.Pq = kp->Pq, t.C = kp->C, t.adv_t = kp->adv_t;
  t.arr_cap = kaa->arr_cap;
  return t;
}

// ---- pieces of the epilogue, each over GR blocks of 64 positions starting at block j0 ----

// Commit of the admitted requests at sorted positions [j0*64, (j0+GR)*64) into their workers' dense
// lists: what the group reads from the queue and the arrivals is requested before its first store.
template <int GR>
__device__ __forceinline__ void br_commit_group(const BrTailArgs &t, int inst, int lane, int j0, int q0, int qn,
                                                const int *skey, const int *adm, int *who, float c0) {
  constexpr int IDX_MASK = (1 << BR_IDX_BITS) - 1;
  const int G = t.G;
  const int64_t qrow = (int64_t)inst * t.Q, arow = (int64_t)inst * t.arr_cap;
  int64_t row[GR];
  int idx[GR], kvv[GR], remv[GR];
  float pr[GR][BR_HP];
  bool ok[GR];
#pragma unroll
  for (int u = 0; u < GR; ++u) {
    const int pos = (j0 + u) * BR_WAVE + lane;
    ok[u] = false;
    idx[u] = 0, kvv[u] = 0, remv[u] = 1, row[u] = 0;
    if (pos < qn) {
      const int ad = adm[pos];
      if (ad >= 0) {
        const int key = skey[pos];
        idx[u] = IDX_MASK - (key & IDX_MASK);
        const int g = ad >> 16, slot = ad & 0xffff;
        if (g < G && slot < t.B && idx[u] < qn) {
          ok[u] = true;
          row[u] = ((int64_t)inst * G + g) * t.Bs + slot;
          kvv[u] = key >> BR_IDX_BITS;
          const bool old = idx[u] < q0;
          remv[u] = old ? t.qo[qrow + idx[u]] : max(t.ao[arow + (idx[u] - q0)], 1);
#pragma unroll
          for (int q = 0; q < BR_HP; ++q)
            if (q < t.Pq)
              pr[u][q] = old ? t.qpred[(qrow + idx[u]) * t.Pq + q] : t.apred[(arow + (idx[u] - q0)) * t.Pq + q];
          who[idx[u]] = g;
        }
      }
    }
  }
#pragma unroll
  for (int u = 0; u < GR; ++u) {
    if (ok[u]) {
      t.kv[row[u]] = kvv[u];
      t.rem[row[u]] = remv[u];
#pragma unroll
      for (int q = 0; q < BR_HP; ++q)
        if (q < t.Pq) t.pred[row[u] * t.P + q] = pr[u][q];
      if (t.P == 3 && t.Pq == 0) {  // maintained estimate: first query at age 0, nothing generated yet
        t.pred[row[u] * 3] = c0;
        t.pred[row[u] * 3 + 1] = 0.0f;
        t.pred[row[u] * 3 + 2] = 0.0f;
      }
    }
  }
}

// What the arrival positions [j0*64, (j0+GR)*64) hold and where they went.
template <int GR>
struct BrQueueGroup {
  int wg[GR], id[GR], sq[GR], oq[GR];
  float pr[GR][BR_HP];
  bool keep[GR];
};

template <int GR>
__device__ __forceinline__ void br_queue_load(const BrTailArgs &t, int inst, int lane, int j0, int q0, int qn,
                                              const int *who, BrQueueGroup<GR> &v) {
  const int64_t qrow = (int64_t)inst * t.Q, arow = (int64_t)inst * t.arr_cap;
#pragma unroll
  for (int u = 0; u < GR; ++u) {
    const int i = (j0 + u) * BR_WAVE + lane;
    const bool in = i < qn, old = i < q0;
    v.wg[u] = in ? who[i] : -1;
    v.id[u] = -1;
    if (in) v.id[u] = old ? t.qid[qrow + i] : (t.aid ? t.aid[arow + (i - q0)] : i - q0);
    v.keep[u] = in && v.wg[u] < 0;
    v.sq[u] = 1, v.oq[u] = 1;
    if (v.keep[u]) {
      v.sq[u] = old ? t.qs[qrow + i] : t.as[arow + (i - q0)];
      v.oq[u] = old ? t.qo[qrow + i] : t.ao[arow + (i - q0)];
#pragma unroll
      for (int q = 0; q < BR_HP; ++q)
        if (q < t.Pq) v.pr[u][q] = old ? t.qpred[(qrow + i) * t.Pq + q] : t.apred[(arow + (i - q0)) * t.Pq + q];
    }
  }
}

// Outputs of those positions in arrival order, and their deferred requests to queue positions `kept`
// onwards (order preserved); `kept` moves on by the number stored.
template <int GR>
__device__ __forceinline__ void br_queue_store(const BrTailArgs &t, int inst, int lane, int j0, int q0,
                                               const BrQueueGroup<GR> &v, int &kept) {
  const int64_t qrow = (int64_t)inst * t.Q;
#pragma unroll
  for (int u = 0; u < GR; ++u) {
    const int i = (j0 + u) * BR_WAVE + lane;
    if ((j0 + u) * BR_WAVE < t.Q) {
      if (i < t.Q) {
        if (t.assign) t.assign[qrow + i] = v.wg[u];
        if (t.assign_id) t.assign_id[qrow + i] = v.id[u];
      }
      const unsigned long long bal = br_ballot(v.keep[u]);
      const int ni = kept + br_rank_below(bal);
      if (v.keep[u] && (ni != i || i >= q0)) {
        t.qs[qrow + ni] = min(max(v.sq[u], 1), BR_MAX_S_DEV);
        t.qo[qrow + ni] = max(v.oq[u], 1);
        t.qid[qrow + ni] = v.id[u];
#pragma unroll
        for (int q = 0; q < BR_HP; ++q)
          if (q < t.Pq) t.qpred[(qrow + ni) * t.Pq + q] = v.pr[u][q];
      }
      kept += __builtin_popcountll(bal);
    }
  }
}

// Worker state and the statistics of the round (one wave).
__device__ __forceinline__ void br_write_state(const BrTailArgs &t, int inst, int lane, int q0, int qn, int cnt, int kept,
                                               int Lcur, int nn, const BrRoundCounts &rc, bool store_workers = true) {
  const int G = t.G;
  const bool act = lane < G;
  const int64_t wrow = (int64_t)inst * G + lane;
  if (act && store_workers) {
    t.L[wrow] = Lcur;
    t.n[wrow] = nn;
  }
  const int Lact = Lcur;
  const int Lmax = br_wave_max(Lact);
  const int Lmin = br_wave_min(act ? Lact : INT32_MAX);
  const int over = __builtin_popcountll(br_ballot(act && t.C > 0 && Lact > t.C));
  const int wide = __builtin_popcountll(br_ballot(act && Lact >= (1 << 25)));  // beyond what the packed worker keys order
  long long sumL = 0;
  if (t.stats) {
    const int L0 = act ? Lcur : 0;
    sumL = ((long long)br_wave_sum(L0 >> 16) << 16) + br_wave_sum(L0 & 0xffff);
  }
  if (lane == 0) {
    t.qlen[inst] = kept;
    if (t.stats) {
      BR_STAT(t, inst, 0) = rc.admitted;
      BR_STAT(t, inst, 1) = kept;
      BR_STAT(t, inst, 2) = cnt - (qn - q0);
      BR_STAT(t, inst, 3) = rc.stage1;
      BR_STAT(t, inst, 4) = rc.pops;
      BR_STAT(t, inst, 5) = rc.guard;
      BR_STAT(t, inst, 6) = over;
      BR_STAT(t, inst, 7) = rc.I_before;
      BR_STAT(t, inst, 8) = (long long)G * Lmax - sumL;
      BR_STAT(t, inst, 9) = (long long)Lmax - Lmin;
      BR_STAT(t, inst, 10) = qn;
      BR_STAT(t, inst, 11) = rc.wdrop;
      BR_STAT(t, inst, 12) = wide;
      for (int k = 13; k < 16; ++k) BR_STAT(t, inst, k) = 0;
    }
  }
}

// The epilogue on the wave that ran the round.  Blocks are taken GR at a time so that the loads of a
// group overlap (each block is a round trip to memory otherwise).  The queue is compacted in place: a
// deferred entry moves to a position at or below its own, inside or before its group, and later groups
// read only beyond it.
template <int E>
__device__ __forceinline__ void br_assign_epilogue(int inst, int lane, int q0, int qn, int cnt, const int *skey,
                                                   const int *adm, int *who, int Lcur, int nn,
                                                   const BrRoundCounts &rc, float c0) {
  const BrTailArgs t = br_tail_args();
  constexpr int GR = E < 4 ? E : 4;
  if (rc.admitted > 0) {
#pragma unroll
    for (int j0 = 0; j0 < E; j0 += GR)
      if (j0 * BR_WAVE < qn) br_commit_group<GR>(t, inst, lane, j0, q0, qn, skey, adm, who, c0);
  }
  br_wave_sync();
  int kept = 0;
#pragma unroll
  for (int j0 = 0; j0 < E; j0 += GR) {
    if (j0 * BR_WAVE < t.Q) {
      BrQueueGroup<GR> v;
      br_queue_load<GR>(t, inst, lane, j0, q0, qn, who, v);
      br_queue_store<GR>(t, inst, lane, j0, q0, v, kept);
    }
  }
  br_write_state(t, inst, lane, q0, qn, cnt, kept, Lcur, nn, rc);
}

// The epilogue on the four waves of a block (queues of up to 2048 entries): wave w owns the sorted
// positions and the arrival positions [w*512, (w+1)*512).  Every wave requests all it will read of the
// queue before the barrier that precedes the first store, so the in-place compaction needs no order
// between waves; the counts of deferred requests per wave go through `sh` (4 words of LDS).
// With `share_workers` wave 0's per-worker (load, count) are handed to every wave (for a decode step split
// among the waves) and wave 0 leaves their store to that step.
__device__ __forceinline__ void br_assign_epilogue_block4(int inst, int lane, int w, int q0, int qn, int cnt, int *skey,
                                                          const int *adm, int *who, int *sh, int &Lcur, int &nn,
                                                          const BrRoundCounts &rc, float c0, bool share_workers) {
  const BrTailArgs t = br_tail_args();
  __syncthreads();  // the round is over: adm[] is complete
  br_commit_group<4>(t, inst, lane, w * 8, q0, qn, skey, adm, who, c0);
  br_commit_group<4>(t, inst, lane, w * 8 + 4, q0, qn, skey, adm, who, c0);
  __syncthreads();  // who[] is complete
  BrQueueGroup<4> va, vb;
  br_queue_load<4>(t, inst, lane, w * 8, q0, qn, who, va);
  br_queue_load<4>(t, inst, lane, w * 8 + 4, q0, qn, who, vb);
  int mine = 0;
#pragma unroll
  for (int u = 0; u < 4; ++u) mine += __builtin_popcountll(br_ballot(va.keep[u])) + __builtin_popcountll(br_ballot(vb.keep[u]));
  // the loaded values must have arrived before any wave stores
  asm volatile("" ::"v"(va.sq[0]), "v"(va.sq[1]), "v"(va.sq[2]), "v"(va.sq[3]), "v"(vb.sq[0]), "v"(vb.sq[1]), "v"(vb.sq[2]),
               "v"(vb.sq[3])
               : "memory");
  __builtin_amdgcn_s_waitcnt(0);
  if (lane == 0) sh[w] = mine;
  if (share_workers && w == 0) skey[lane] = Lcur, skey[BR_WAVE + lane] = nn;  // the sorted keys are no longer needed
  __syncthreads();
  if (share_workers) Lcur = skey[lane], nn = skey[BR_WAVE + lane];
  int kept = 0, total = 0;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int c = sh[k];
    kept += k < w ? c : 0;
    total += c;
  }
  br_queue_store<4>(t, inst, lane, w * 8, q0, va, kept);
  br_queue_store<4>(t, inst, lane, w * 8 + 4, q0, vb, kept);
  if (w == 0) br_write_state(t, inst, lane, q0, qn, cnt, total, Lcur, nn, rc, !share_workers);
}

// Late copy of the whole parameter block from the kernel-argument segment (same reason as above).
__device__ __forceinline__ BrParams br_late_params() {
  typedef __attribute__((address_space(4))) const char kchar_t;
  typedef __attribute__((address_space(4))) const BrParams kparams_t;
  kchar_t *ka = (kchar_t *)__builtin_amdgcn_kernarg_segment_ptr();
  asm volatile("" : "+s"(ka));
  BrParams p;
  __builtin_memcpy(&p, (kparams_t *)ka, sizeof(BrParams));
  return p;
}

// Decode advance of one cluster by the wave that has just routed it: br_adv_apply (the arithmetic of
// the stand-alone advance kernel) over the cluster's G lists in (list, 256-slot chunk) units, UB units
// requested before the first is used.  `Lcur`, `nn`: load and list length of worker `lane` after the round.
// STORE = false: loads and counts are not stored; lane g returns its list's load change in `dL_out` and its new
// length in `n_out` instead (the split kernels, where another wave owns the workers' final state).
template <int UB, bool BRH, bool STORE = true>
__device__ __forceinline__ void br_advance_cluster(int inst, int lane, int Lcur, int nn, int g0 = 0, int g1 = 64,
                                                   int *dL_out = nullptr, int *n_out = nullptr) {
  const BrParams p = br_late_params();
  const int t = p.adv_t;
  br_wave_sync();  // the round's own writes into the lists are read back below
  const int G = min(p.G, g1), NC = (p.Bs + 255) >> 8, U = max(G - g0, 0) * NC;  // lists [g0, G) are this wave's
  const int64_t row0 = (int64_t)__builtin_amdgcn_readfirstlane(inst) * p.G;  // scalar: list bases stay in SGPRs
  const int64_t rowa = row0 + g0;
  int dLw = 0, nw = nn;     // lane g: load change and new length of worker g
  int kept = 0, gone = 0;   // running state of the list in progress: survivors, kv that left
  int gl = g0, cl = 0, gp = g0, cp = 0;  // (list, chunk) cursors of the load and the update pass
  const int32_t *kl = p.kv + rowa * p.Bs, *rl = p.rem + rowa * p.Bs;  // list the load pass is at
  int32_t *kw = p.kv + rowa * p.Bs, *rw = p.rem + rowa * p.Bs;        // list the update pass is at
  float *pw = p.pred + rowa * p.Bs * p.P;
  for (int u0 = 0; u0 < U; u0 += UB) {
    int4 kv[UB], rem[UB];
#pragma unroll
    for (int k = 0; k < UB; ++k) {
      kv[k] = make_int4(0, 0, 0, 0), rem[k] = make_int4(0, 0, 0, 0);
      if (gl < G) br_adv_load(kl, rl, cl * 256 + 4 * lane, __builtin_amdgcn_readlane(nn, gl), kv[k], rem[k]);
      if (++cl == NC) cl = 0, ++gl, kl += p.Bs, rl += p.Bs;
    }
#pragma unroll
    for (int k = 0; k < UB; ++k) {
      if (gp < G) {
        const int ng = __builtin_amdgcn_readlane(nn, gp);
        if (cp * 256 < ng) br_adv_apply<BRH>(p, t, cp * 256 + 4 * lane, ng, cp * 256, kv[k], rem[k], kw, rw, pw, kept, gone);
        if (++cp == NC) {
          if (lane == gp) dLw = kept * t - gone, nw = kept;  // survivors gain t tokens each
          kept = 0, gone = 0, cp = 0, ++gp;
          kw += p.Bs, rw += p.Bs, pw += (int64_t)p.Bs * p.P;
        }
      }
    }
  }
  if constexpr (STORE) {
    if (lane >= g0 && lane < G) {
      p.L[row0 + lane] = Lcur + dLw;
      p.n[row0 + lane] = nw;
    }
  } else {
    *dL_out = dLw;
    *n_out = nw;
  }
}

// ---------------------------------------------------------------- split step: round and decode step on two waves
// In the split kernels (BR-0, queues of up to 512) the decode steps of a cluster's lists as they stand at the
// start of the step are applied by a second wave (the helper) while the first runs the round; the wave that ran
// the round then appends its admissions behind the survivors, already advanced.  Same final state as the round
// followed by the decode steps: a list holds its old survivors in order, then the new survivors in admission
// order; L_g = sum of the kv held; a request whose output is used up within the t steps leaves at once.
// LDS area of one cluster: [0] flag (helper done), [4..68) per worker: entries its list lost (old length - kept),
// [68..132) per worker: load change of the old entries.
#define BR_SPLIT_WORDS 132

// The helper's part for one cluster: snapshot reductions if asked for (they read what the round's epilogue will
// overwrite, and the epilogue waits for the flag), the decode steps of the old entries, then the flag.
// UB: (list, chunk) units requested before the first is used
template <int E, int UB>
__device__ __forceinline__ void br_split_helper(const BrParams &p, const BrArr &a, const BrOut &o, int inst, int lane,
                                                int *split) {
  const bool act = lane < p.G;
  int n0;
  if (o.best_g || o.best_i) {
    BrScoreIn<E, false> in;
    br_score_wave_load<E, false>(p, a, inst, lane, in);
    br_score_wave_run<E, false>(p, o, inst, lane, in);
    n0 = in.n;
  } else {
    n0 = act ? p.n[(int64_t)inst * p.G + lane] : p.B;
  }
  n0 = act ? min(max(n0, 0), p.B) : 0;
  int dL = 0, kept = n0;
  br_advance_cluster<UB, false, false>(inst, lane, 0, n0, 0, 64, &dL, &kept);
  split[4 + lane] = n0 - kept;
  split[4 + BR_WAVE + lane] = dL;
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");  // the lists are in place before the flag is seen
  __builtin_amdgcn_wave_barrier();
  if (lane == 0) split[0] = 1;
}

// The epilogue of the wave that ran the round, in a split kernel.  nn0: list lengths at the start of the step.
template <int E>
__device__ __forceinline__ void br_assign_epilogue_split(int inst, int lane, int q0, int qn, int cnt, const int *skey,
                                                         const int *adm, int *who, int Lcur, int nn, int nn0,
                                                         const BrRoundCounts &rc, int *split) {
  const BrTailArgs t = br_tail_args();
  constexpr int IDX_MASK = (1 << BR_IDX_BITS) - 1;
  const int G = t.G, tt = t.adv_t;
  const int64_t qrow = (int64_t)inst * t.Q, arow = (int64_t)inst * t.arr_cap;
  // the helper is done with this cluster's lists (it never waits for anything: the flag always comes)
  while (__atomic_load_n(split, __ATOMIC_RELAXED) == 0) __builtin_amdgcn_s_sleep(4);
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  const int lost = split[4 + lane], dold = split[4 + BR_WAVE + lane];  // lane g: worker g
  const int kept0 = nn0 - lost, a_g = nn - nn0;                        // old survivors, admissions of this round
  int nfin = kept0 + a_g, Lfin = Lcur + dold + a_g * tt;               // if every admitted request outlives the t steps
  bool slow = false;
  if (rc.admitted > 0) {
    // every admitted request of the cluster, E sorted positions per lane: all reads before the first store
    int64_t row[E];
    int kvv[E], remv[E];
    bool ok[E];
    bool short_one = false;
#pragma unroll
    for (int u = 0; u < E; ++u) {
      const int pos = u * BR_WAVE + lane;
      ok[u] = false;
      kvv[u] = 0, remv[u] = 1, row[u] = 0;
      if (pos < qn) {
        const int ad = adm[pos];
        if (ad >= 0) {
          const int key = skey[pos];
          const int idx = IDX_MASK - (key & IDX_MASK);
          const int g = ad >> 16, slot = ad & 0xffff;
          if (g < G && slot < t.B && idx < qn) {
            ok[u] = true;
            row[u] = ((int64_t)inst * G + g) * t.Bs + (slot - split[4 + g]);  // behind the old survivors
            kvv[u] = key >> BR_IDX_BITS;
            remv[u] = idx < q0 ? t.qo[qrow + idx] : max(t.ao[arow + (idx - q0)], 1);
            short_one |= remv[u] <= tt;
            who[idx] = g;
          }
        }
      }
    }
    slow = br_ballot(short_one) != 0ull;  // some admitted request ends within the t steps: lists are compacted below
    const int add = slow ? 0 : tt;
#pragma unroll
    for (int u = 0; u < E; ++u) {
      if (ok[u]) {
        t.kv[row[u]] = kvv[u] + add;
        t.rem[row[u]] = remv[u] - add;
      }
    }
  }
  br_wave_sync();
  int keptq = 0;
  constexpr int GR = E < 4 ? E : 4;
#pragma unroll
  for (int j0 = 0; j0 < E; j0 += GR) {
    if (j0 * BR_WAVE < t.Q) {
      BrQueueGroup<GR> v;
      br_queue_load<GR>(t, inst, lane, j0, q0, qn, who, v);
      br_queue_store<GR>(t, inst, lane, j0, q0, v, keptq);
    }
  }
  br_write_state(t, inst, lane, q0, qn, cnt, keptq, Lcur, nn, rc, false);  // statistics: the state right after the round
  if (slow) {
    // The admissions sit behind the old survivors as admitted (kv = s, rem = o); per worker the decode steps
    // now run over that stretch alone: who outlives them moves up and gains t tokens, the others leave.
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");  // the stores above are read back below
    __builtin_amdgcn_wave_barrier();
    for (int g = 0; g < G; ++g) {
      const int ag = __builtin_amdgcn_readlane(a_g, g);
      if (ag <= 0) continue;
      const int64_t base = ((int64_t)inst * G + g) * t.Bs + __builtin_amdgcn_readlane(kept0, g);
      int keptn = 0, gone = 0;
      for (int c0 = 0; c0 < ag; c0 += BR_WAVE) {
        const int j = c0 + lane;
        const bool in = j < ag;
        const int kv = in ? t.kv[base + j] : 0, rem = in ? t.rem[base + j] : 0;
        const bool stay = in && rem > tt;
        const unsigned long long bal = br_ballot(stay);
        const int dst = keptn + br_rank_below(bal);
        if (stay) {  // at or below its own position; the chunk was read whole before
          t.kv[base + dst] = kv + tt;
          t.rem[base + dst] = rem - tt;
        }
        gone += br_wave_sum((in && !stay) ? kv : 0);
        keptn += (int)__builtin_popcountll(bal);
      }
      if (lane == g) {
        nfin = kept0 + keptn;
        Lfin = Lcur + dold - gone + keptn * tt;
      }
    }
  }
  if (lane < G) {
    const int64_t wrow = (int64_t)inst * G + lane;
    t.L[wrow] = Lfin;
    t.n[wrow] = nfin;
  }
}

