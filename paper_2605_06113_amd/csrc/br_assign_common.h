// Shared tail of the assignment kernels: writes the admitted requests into their workers'
// lists, emits the per-entry outputs in arrival order, compacts the waiting queue in place and
// stores worker state and statistics.  Everything here is lane-parallel; `adm` (by sorted
// position: worker << 16 | slot, or -1) and the sorted keys in `skey` come from the round.
#pragma once

#include "br_device.h"

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
  int32_t G, B, Bs, Q, P, Pq, C, arr_cap;
};

static_assert(sizeof(BrParams) == 240 && sizeof(BrArr) == 48 && sizeof(BrOut) == 48, "kernel argument layout");

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
  t.G = kp->G, t.B = kp->B, t.Bs = kp->Bs, t.Q = kp->Q, t.P = kp->P, t.Pq = kp->Pq, t.C = kp->C;
  t.arr_cap = kaa->arr_cap;
  return t;
}

template <int E>
__device__ __forceinline__ void br_assign_epilogue(int inst, int lane, int q0, int qn, int cnt, const int *skey,
                                                   const int *adm, int *who, int Lcur, int nn,
                                                   const BrRoundCounts &rc, float c0) {
  constexpr int IDX_MASK = (1 << BR_IDX_BITS) - 1;
  const BrTailArgs t = br_tail_args();
  const int G = t.G;
  const bool act = lane < G;
  const int64_t wrow = (int64_t)inst * G + lane;
  const int64_t qrow = (int64_t)inst * t.Q, arow = (int64_t)inst * t.arr_cap;
  const int admitted = rc.admitted;
  // ---- commit the admitted requests into their workers' dense lists, GR blocks of sorted positions
  //      at a time: what a group reads from the queue and the arrivals is requested before its first store
  constexpr int GR = E < 4 ? E : 4;
  if (admitted > 0) {
#pragma unroll
    for (int j0 = 0; j0 < E; j0 += GR) {
      if (j0 * BR_WAVE < qn) {
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
    }
  }
  br_wave_sync();

  // ---- outputs in arrival order; the queue keeps the deferred requests, order preserved.
  // Blocks of 64 entries are taken GR at a time: everything the group reads is requested before its
  // first store, so the loads of a group overlap (a 2048-entry queue is 32 blocks, each a round trip to
  // memory otherwise).  In place: a deferred entry moves to a position at or below its own, inside or
  // before its group, and later groups read only beyond it.
  int kept = 0;
#pragma unroll
  for (int j0 = 0; j0 < E; j0 += GR) {
    if (j0 * BR_WAVE < t.Q) {
      int wg[GR], id[GR], sq[GR], oq[GR];
      float pr[GR][BR_HP];
      bool keep[GR];
#pragma unroll
      for (int u = 0; u < GR; ++u) {
        const int i = (j0 + u) * BR_WAVE + lane;
        const bool in = i < qn, old = i < q0;
        wg[u] = in ? who[i] : -1;
        id[u] = -1;
        if (in) id[u] = old ? t.qid[qrow + i] : (t.aid ? t.aid[arow + (i - q0)] : i - q0);
        keep[u] = in && wg[u] < 0;
        sq[u] = 1, oq[u] = 1;
        if (keep[u]) {
          sq[u] = old ? t.qs[qrow + i] : t.as[arow + (i - q0)];
          oq[u] = old ? t.qo[qrow + i] : t.ao[arow + (i - q0)];
#pragma unroll
          for (int q = 0; q < BR_HP; ++q)
            if (q < t.Pq) pr[u][q] = old ? t.qpred[(qrow + i) * t.Pq + q] : t.apred[(arow + (i - q0)) * t.Pq + q];
        }
      }
#pragma unroll
      for (int u = 0; u < GR; ++u) {
        const int i = (j0 + u) * BR_WAVE + lane;
        if ((j0 + u) * BR_WAVE < t.Q) {
          if (i < t.Q) {
            if (t.assign) t.assign[qrow + i] = wg[u];
            if (t.assign_id) t.assign_id[qrow + i] = id[u];
          }
          const unsigned long long bal = br_ballot(keep[u]);
          const int ni = kept + br_rank_below(bal);
          if (keep[u] && (ni != i || i >= q0)) {
            t.qs[qrow + ni] = min(max(sq[u], 1), BR_MAX_S_DEV);
            t.qo[qrow + ni] = max(oq[u], 1);
            t.qid[qrow + ni] = id[u];
#pragma unroll
            for (int q = 0; q < BR_HP; ++q)
              if (q < t.Pq) t.qpred[(qrow + ni) * t.Pq + q] = pr[u][q];
          }
          kept += __builtin_popcountll(bal);
        }
      }
    }
  }

  // ---- state and statistics
  if (act) {
    t.L[wrow] = Lcur;
    t.n[wrow] = nn;
  }
  const int Lact = Lcur;
  const int Lmax = br_wave_max(Lact);
  const int Lmin = br_wave_min(act ? Lact : INT32_MAX);
  const int over = __builtin_popcountll(br_ballot(act && t.C > 0 && Lact > t.C));
  long long sumL = 0;
  if (t.stats) {
    const int L0 = act ? Lcur : 0;
    sumL = ((long long)br_wave_sum(L0 >> 16) << 16) + br_wave_sum(L0 & 0xffff);
  }
  if (lane == 0) {
    t.qlen[inst] = kept;
    if (t.stats) {
      BR_STAT(t, inst, 0) = admitted;
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
      for (int k = 12; k < 16; ++k) BR_STAT(t, inst, k) = 0;
    }
  }
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
template <int UB, bool BRH>
__device__ __forceinline__ void br_advance_cluster(int inst, int lane, int Lcur, int nn) {
  const BrParams p = br_late_params();
  const int t = p.adv_t;
  br_wave_sync();  // the round's own writes into the lists are read back below
  const int G = p.G, NC = (p.Bs + 255) >> 8, U = G * NC;
  const int64_t row0 = (int64_t)__builtin_amdgcn_readfirstlane(inst) * G;  // scalar: list bases stay in SGPRs
  int dLw = 0, nw = nn;     // lane g: load change and new length of worker g
  int kept = 0, gone = 0;   // running state of the list in progress: survivors, kv that left
  int gl = 0, cl = 0, gp = 0, cp = 0;  // (list, chunk) cursors of the load and the update pass
  const int32_t *kl = p.kv + row0 * p.Bs, *rl = p.rem + row0 * p.Bs;  // list the load pass is at
  int32_t *kw = p.kv + row0 * p.Bs, *rw = p.rem + row0 * p.Bs;        // list the update pass is at
  float *pw = p.pred + row0 * p.Bs * p.P;
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
  if (lane < G) {
    p.L[row0 + lane] = Lcur + dLw;
    p.n[row0 + lane] = nw;
  }
}
