// K2 + K3 for large batches of small clusters: one wavefront per cluster, no LDS and no barrier.
// Lane g holds worker g (margins of eq. (br0-Fscore) / eq. (brh-Fscore)); each lane holds E waiting
// requests in arrival order.  For every worker (margins broadcast by readlane) all requests are
// scored once; the same score feeds the running best worker of each request (ties: lowest g) and
// the best request of this worker (ties: larger s, then earlier arrival), the latter finished by two
// wave reductions.  Results equal br_k_score's; the score matrix itself is not written here.
// Split in two so that a caller can have the inputs of several clusters in registers before it scores.
#pragma once

#include "br_device.h"

template <int E, bool BRH>
struct BrScoreIn {
  static constexpr int NH = BRH ? BR_HP + 1 : 1;
  int qn, q0, cnt, L, cap, n;  // queue length with and without this round's arrivals, arrivals taken; lane g: load,
                               // free slots and request count of worker g as stored
  int m[NH];  // BR-H: margins of the step-start projection; BR-0: filled by br_score_wave_run
  int s[E];
};

template <int E, bool BRH>
__device__ __forceinline__ void br_score_wave_load(const BrParams &p, const BrArr &a, int inst, int lane,
                                                   BrScoreIn<E, BRH> &in) {
  // every load that does not need the queue length is requested before the first result is used, and the waiting
  // set comes in one batch of unconditional loads (addresses chosen by select, an entry beyond the set reads the
  // cluster's first queue word): two memory round trips for the whole cluster
  const int q0_raw = p.qlen[inst];
  const int cnt_raw = a.count ? a.count[inst] : 0;
  const int64_t qrow = (int64_t)inst * p.Q, arow = (int64_t)inst * a.arr_cap;
  const bool act = lane < p.G;
  const int64_t wrow = (int64_t)inst * p.G + lane;
  const int64_t wrow_ld = act ? wrow : (int64_t)inst * p.G;  // lanes without a worker read worker 0's words (unused)
  const int L_raw = p.L[wrow_ld], n_raw = p.n[wrow_ld];
  int m_raw[BrScoreIn<E, BRH>::NH];
  if constexpr (BRH) {
#pragma unroll
    for (int h = 0; h < BrScoreIn<E, BRH>::NH; ++h) m_raw[h] = p.mh[wrow_ld * (p.H + 1) + min(h, p.H)];
  }
  in.L = act ? L_raw : BR_LOW;
  in.n = act ? n_raw : p.B;
  in.cap = act ? p.B - in.n : 0;
  if constexpr (BRH) {
#pragma unroll
    for (int h = 0; h < BrScoreIn<E, BRH>::NH; ++h) in.m[h] = (act && h <= p.H) ? m_raw[h] : 0;
  } else {
    in.m[0] = 0;
  }
  const int q0 = br_uniform(min(max(q0_raw, 0), p.Q));
  const int cnt = br_uniform(min(max(cnt_raw, 0), a.arr_cap));
  in.qn = q0 + min(cnt, p.Q - q0);
  in.q0 = q0;
  in.cnt = cnt;
  int v[E];
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const int i = e * BR_WAVE + lane;
    const bool ina = i >= q0 && i < in.qn;
    const int32_t *src = ina ? a.s + (arow + (i - q0)) : p.qs + (qrow + (i < q0 ? i : 0));
    v[e] = *src;
  }
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const int i = e * BR_WAVE + lane;
    in.s[e] = i < in.qn ? min(max(v[e], 1), BR_MAX_S_DEV) : 1;
  }
}

template <int E, bool BRH>
__device__ __forceinline__ void br_score_wave_run(const BrParams &p, const BrOut &o, int inst, int lane,
                                                  const BrScoreIn<E, BRH> &in) {
  constexpr int NH = BrScoreIn<E, BRH>::NH;
  constexpr int IDX_MASK = (1 << BR_IDX_BITS) - 1;
  const int G = p.G, qn = in.qn;
  const bool act = lane < G;
  const int64_t qrow = (int64_t)inst * p.Q, wrow = (int64_t)inst * G + lane;
  const int L = in.L, cap = in.cap;
  int m[NH];
#pragma unroll
  for (int h = 0; h < NH; ++h) m[h] = in.m[h];
  if constexpr (!BRH) m[0] = br_wave_max(L) - L;  // M(k) = max_g L_g, m_g = M - L_g

  int s[E], sec[E], bk[E], bg[E];
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const int i = e * BR_WAVE + lane;
    s[e] = in.s[e];
    sec[e] = i < qn ? ((s[e] << BR_IDX_BITS) | (IDX_MASK - i)) : -1;  // larger s first, then earlier arrival
    bk[e] = BR_KEY_NONE;
    bg[e] = -1;
  }

  int bi_mine = -1;  // lane g: best request of worker g
  for (int g = 0; g < G; ++g) {
    int mg[BR_HP + 1];
#pragma unroll
    for (int h = 0; h <= BR_HP; ++h) mg[h] = 0;
#pragma unroll
    for (int h = 0; h < NH; ++h) mg[h] = __builtin_amdgcn_readlane(m[h], g);
    const int Lg = __builtin_amdgcn_readlane(L, g);
    const bool free_slot = __builtin_amdgcn_readlane(cap, g) > 0;
    int bi = -1;
    if (free_slot) {
      const int room = p.W > 0 ? p.W - Lg : INT32_MAX;
      int kk[E], lmax = BR_KEY_NONE;
#pragma unroll
      for (int e = 0; e < E; ++e) {  // straight-line selects; lanes without a request carry sec = -1
        if (E > 4 && e * BR_WAVE >= qn) {  // wide layouts: skip the registers beyond the queue
          kk[e] = BR_KEY_NONE;
          continue;
        }
        const int key = br_score_key<BRH>(p, mg, s[e]);
        kk[e] = ((sec[e] >= 0) & (s[e] <= room)) ? key : BR_KEY_NONE;
        const bool newg = kk[e] > bk[e];
        bk[e] = newg ? kk[e] : bk[e];
        bg[e] = newg ? g : bg[e];
        lmax = max(lmax, kk[e]);
      }
      const int km = br_wave_max(lmax);
      if (km != BR_KEY_NONE) {  // among the requests that reach the best score: larger s, then earlier arrival
        int w2 = -1;
#pragma unroll
        for (int e = 0; e < E; ++e) w2 = max(w2, kk[e] == km ? sec[e] : -1);
        bi = IDX_MASK - (br_wave_max(w2) & IDX_MASK);
      }
    }
    bi_mine = lane == g ? bi : bi_mine;
  }

  if (o.best_g) {
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const int i = e * BR_WAVE + lane;
      if (i < p.Q) o.best_g[qrow + i] = i < qn ? bg[e] : -1;
    }
  }
  if (o.best_i && act) o.best_i[wrow] = bi_mine;
}
