// Two-stage assignment of one scheduling round for horizons beyond the offsets the register kernel
// carries (Appendix, Alg. BR-H; H up to 128, the deployed value of Sec. 6 is 80), one wavefront per
// cluster runs the round (others may serve its searches, below).
//
// The round is the loop of Alg. BR-H: Stage 1 gives the worker with the most free slots (then the
// lightest, then the lowest index) its best single request while free capacity exceeds S_greedy (taken a
// level of equal free-slot counts at a time where that is provably the same, see below); Stage 2 pops
// workers by (free slots, horizon-min margin), searches the subsets of the top-R_max window and falls
// back to the single best request when no subset scores above zero.
//
// What differs from the short-horizon kernel is where the per-offset state lives:
//   - the step-start projections L_g(k+h) stay in LDS, sL[h][g] (row stride G | 1 words: odd, so that both
//     "lane = worker" and "lane = offset" reads spread over the banks, and no wider than the cluster needs:
//     with few workers several clusters then share a CU's LDS) and are never rewritten: an
//     admission adds its length at every offset (constant-s approximation of Sec. 4.1), so worker g's
//     current projection is sL[h][g] + add_g with one register add_g per lane;
//   - the envelope M_h and the margins of the worker in hand are LDS arrays maintained with lanes
//     mapped to offsets (lane l also keeps the envelope at offsets l, l + 64, l + 128 and the projections of
//     the worker in hand in registers, so that the update after an admission needs no LDS read);
//   - a score walks the offsets in order with margins and discounts broadcast from LDS, four per load, and
//     skips the groups of offsets whose margins no value in question reaches (exact zeros);
//   - the single best request argmax_i F_g({i}) is found by bracketing, not by scoring the whole waiting set
//     (pick_single: the score is concave in the length, the waiting set is sorted by length);
//   - Stage 2 goes straight to the starvation guard when the window's smallest entry scores clearly below
//     zero (then every subset does).
// Waiting set, sticky binding, epilogue and the optional decode steps are those of the short-horizon
// kernel (br_sort.h, br_assign_common.h).
//
// With fewer clusters than the chip has room for waves (NW = 2 or 4 waves per cluster) the searches, which
// are most of a round at these horizons, are shared: wave 0 runs the round and posts a command in LDS (the
// margins are there already), every wave does its share between two block barriers: of the probes' offset
// groups in a bracketing search (the order of that sum is free), or of the sorted positions in a full scan
// (wave 0 takes the best of the partial results; the share of a later wave holds higher positions, so only a
// strictly better score wins).  The helper waves leave when wave 0 posts the end of the round; decode steps
// then follow as a launch of their own.
#include "br_device.h"
#include "br_launch.h"
#include "br_sort.h"
#include "br_assign_common.h"

#define BR_LSTRIDE(G) ((G) | 1)  // words between offsets in sL (odd; one spare "no worker" column when G is even)

// Best (score key, sorted position) among the alive, admissible requests of NB blocks of 64 sorted positions
// (block jb + j in sv[J0 + j], alive bit J0 + j), lowest position on equal scores.  The longest alive request of
// a block is its first alive one: offsets whose margin it does not reach add nothing for any request of the
// block and are skipped for that block.
template <int NS, int J0, int NB>
__device__ __forceinline__ void br_long_slice_best(const BrParams &p, const float *smg, const float *sd, int HS, int lane,
                                                   int qn, const int (&sv)[NS], unsigned alive, int jb, int room, int &bk,
                                                   int &bp) {
  constexpr int NV = NB >= 4 ? 4 : NB;
  bk = BR_KEY_NONE, bp = INT32_MAX;
#pragma unroll
  for (int c = 0; c < NB; c += NV) {
    if ((jb + c) * BR_WAVE < qn) {
      int top[NV], dv[NV];
      int any = 0;
#pragma unroll
      for (int u = 0; u < NV; ++u) {
        const unsigned long long bal = br_ballot((alive >> (J0 + c + u)) & 1u);
        const int first = __builtin_amdgcn_readlane(sv[J0 + c + u], bal != 0ull ? (int)__builtin_ctzll(bal) : 0);
        top[u] = bal != 0ull ? first : 0;
        dv[u] = sv[J0 + c + u];
        any |= top[u];
      }
      if (any == 0) continue;
      float Fv[NV];
      br_scoreh_long_sel<NV>(p.aD, p.beta, smg, sd, HS, lane, top, dv, Fv);
#pragma unroll
      for (int u = 0; u < NV; ++u) {
        const bool ok = ((alive >> (J0 + c + u)) & 1u) && dv[u] <= room;
        const int key = ok ? br_ord(Fv[u]) : BR_KEY_NONE;
        if (key > bk) {  // positions rise with the block within a lane: the first best stays
          bk = key;
          bp = (jb + c + u) * BR_WAVE + lane;
        }
      }
    }
  }
}

template <int E, bool ADV, int NW>
// (queues of up to 256: four waves per SIMD are asked for, which is what br_long_waves counts on)
__global__ __launch_bounds__(64 * NW, E == 4 ? 4 : 1) void br_k_assign_long(BrParams p, BrArr a, BrOut o) {
  static_assert(NW == 1 || !ADV, "decode steps ride along only with one wave per cluster");
  static_assert(E % NW == 0, "every wave takes whole blocks of 64 sorted positions");
  constexpr int EW = E / NW;  // blocks of 64 sorted positions per wave in a shared search
  // four-offset groups of wave 0 when the probes of a bracketing search are shared: every NW-th, wave w takes the
  // same pattern shifted by w
  constexpr unsigned long long SHARE = NW == 1 ? ~0ull : NW == 2 ? 0x5555555555555555ull : 0x1111111111111111ull;
  extern __shared__ int lds[];
  constexpr int NP = E * BR_WAVE;
  constexpr int IDX_MASK = (1 << BR_IDX_BITS) - 1;
  const int inst = (int)blockIdx.x;
  if (inst >= p.N) return;
  const int H1 = p.H + 1, HS = BR_HS(p.H);
  int *skey = lds;                  // [NP] sorted keys (s << 11 | 2047 - arrival position)
  int *adm = lds + NP;              // [NP] by sorted position: worker << 16 | slot, or -1
  int *who = lds + 2 * NP;          // [NP] by arrival position: worker, or -1
  int *win = lds + 3 * NP;          // [64] Stage-1 level: k-th alive request (s << 11 | sorted position);
                                    //      Stage 2: the candidate window, same packing (16-byte aligned)
  int *pm = win + BR_WAVE;          // [64] partial horizon-min margins (offsets split over the lanes)
  int *sM = pm + BR_WAVE;           // [HS] envelope M_h
  float *smg = (float *)(sM + HS);  // [HS] margins of the worker in hand, as floats
  float *sd = smg + HS;             // [HS] discounts, zero beyond H
  const int LS = BR_LSTRIDE(p.G);
  int *sL = sM + 3 * HS;            // [HS][LS] step-start projections (rows beyond H: "no worker")
  int *hitab = sL + ((HS * LS + 3) & ~3);  // R_max > 8: [1024] sums of window entries 6.. by upper mask bits
  int *mbox = hitab + (p.R_max > 8 ? 1024 : 0);  // NW > 1: [16] search mailbox: command, admissible length; results from word 4
  int *salive = pm;                 // alive words of the lanes of wave 0 during a search (pm is idle then)

  const int lane = br_lane();
  const int G = p.G;
  const int q0 = br_uniform(min(max(p.qlen[inst], 0), p.Q));
  int cnt = a.count ? a.count[inst] : 0;
  cnt = br_uniform(min(max(cnt, 0), a.arr_cap));
  const int qn = q0 + min(cnt, p.Q - q0);
  const int64_t qrow = (int64_t)inst * p.Q, arow = (int64_t)inst * a.arr_cap;

  if constexpr (NW > 1) {
    const int w = (int)(threadIdx.x >> 6);
    if (w != 0) {  // serves wave 0's searches: every wave of the block meets at both barriers of each, wave 0 ends the loop
      __syncthreads();  // the sorted keys and the discounts are in LDS
      int svh[EW];
#pragma unroll
      for (int j = 0; j < EW; ++j) svh[j] = skey[(w * EW + j) * BR_WAVE + lane] >> BR_IDX_BITS;
      const int sprobe = skey[lane * E] >> BR_IDX_BITS;  // the probe of this lane in a bracketing search
      for (;;) {
        __syncthreads();
        const int cmd = mbox[0];
        if (cmd == 0) break;
        if (cmd == 2) {  // this wave's share of the probes' penalty sums
          who[w * BR_WAVE + lane] = __float_as_int(br_long_penalty_part(smg, sd, HS, lane, mbox[2], sprobe, SHARE << w));
        } else {         // this wave's share of a full scan
          const int roomq = mbox[1];
          const unsigned al = (unsigned)salive[lane] >> (w * EW);
          int bk, bp;
          br_long_slice_best<EW, 0, EW>(p, smg, sd, HS, lane, qn, svh, al, w * EW, roomq, bk, bp);
          const int km = br_wave_max(bk);
          const int pmn = km == BR_KEY_NONE ? INT32_MAX : br_wave_min(bk == km ? bp : INT32_MAX);
          if (lane == 0) mbox[4 + 2 * w] = km, mbox[5 + 2 * w] = pmn;
        }
        __syncthreads();
      }
      return;
    }
  }

  float c0 = 0.0f;  // first estimate of a newly admitted request when the library maintains c_hat
  if (p.pred_mode == 2) c0 = br_survival(p, 0);

  // ---- worker state: lane g holds worker g
  const bool act = lane < G;
  const int64_t wrow = (int64_t)inst * G + lane;
  int nn = act ? min(max(p.n[wrow], 0), p.B) : p.B;
  int cap = p.B - nn;
  int Lcur = act ? p.Lh[wrow * H1] : BR_LOW;  // L_g(k) + what this round admits
  int add = 0;                                // tokens admitted to this lane's worker in this round
  // envelope: lane l also keeps the offsets l, l + 64, l + 128 in registers (the LDS copy serves the reads that
  // need other lanes' offsets); Lg: the same offsets of the step-start projection of the worker in hand
  int Mr[3] = {0, 0, 0}, Lg[3] = {0, 0, 0};
#pragma unroll
  for (int u = 0; u < 3; ++u) {
    const int h = u * BR_WAVE + lane;
    if (h < HS) {
      Mr[u] = h < H1 ? p.Mh[(int64_t)inst * H1 + h] : 0;
      sM[h] = Mr[u];
      sd[h] = p.dl[h];
      smg[h] = 0.0f;
    }
  }
  for (int g = 0; g < LS; ++g) {  // a column beyond G and offsets beyond H read as "no worker"
    for (int h0 = 0; h0 < HS; h0 += BR_WAVE) {
      const int h = h0 + lane;
      if (h < HS) sL[h * LS + g] = (g < G && h < H1) ? p.Lh[((int64_t)inst * G + g) * H1 + h] : BR_LOW;
    }
  }
  int S_tot = br_wave_sum(cap);
  long long I_before = 0;
  if (o.stats) {
    const int L0 = act ? Lcur : 0;
    const long long sumL = ((long long)br_wave_sum(L0 >> 16) << 16) + br_wave_sum(L0 & 0xffff);
    I_before = (long long)G * br_wave_max(Lcur) - sumL;
  }

  // ---- waiting set, sorted in registers (largest prefill first, arrival order among equals)
  const bool run = S_tot > 0 && qn > 0;
  unsigned xk[E];
  int s_raw[E];
#pragma unroll
  for (int j = 0; j < E; ++j) {  // one batch of unconditional loads (an entry beyond the set reads the first queue word)
    const int i = j * BR_WAVE + lane;
    const bool ina = i >= q0 && i < qn;
    const int32_t *src = ina ? a.s + (arow + (i - q0)) : p.qs + (qrow + (i < q0 ? i : 0));
    s_raw[j] = *src;
  }
#pragma unroll
  for (int j = 0; j < E; ++j) {
    const int i = j * BR_WAVE + lane;
    unsigned key = 0;
    if (i < qn) {
      const int s = min(max(s_raw[j], 1), BR_MAX_S_DEV);
      key = ((unsigned)s << BR_IDX_BITS) | (unsigned)(IDX_MASK - i);
    }
    xk[j] = key;
    adm[i] = -1;
    who[i] = -1;
  }
  if (run) {
    int N2 = BR_WAVE;
    while (N2 < qn) N2 <<= 1;
    br_sort_desc<E>(xk, lane, N2);
  }
  int sv[E];
  unsigned alive = 0;
#pragma unroll
  for (int j = 0; j < E; ++j) {
    const int pos = j * BR_WAVE + lane;
    skey[pos] = (int)xk[j];
    sv[j] = (int)(xk[j] >> BR_IDX_BITS);
    if (pos < qn) alive |= 1u << j;
  }
  br_wave_sync();
  if constexpr (NW > 1) __syncthreads();  // the helper waves read their share of the sorted keys

  int n_alive = qn;
  int stage1 = 0, pops = 0, guard = 0, wdrop = 0, admitted = 0;

  // margins of worker g against the current envelope, into smg (lanes = offsets)
  auto margins_of = [&](int g) {
    const int ag = __builtin_amdgcn_readlane(add, g);
#pragma unroll
    for (int u = 0; u < 3; ++u) {
      const int h = u * BR_WAVE + lane;
      if (h < H1) {
        Lg[u] = sL[h * LS + g];
        smg[h] = (float)max(Mr[u] - (Lg[u] + ag), 0);
      }
    }
    br_wave_sync();
  };

  // horizon-min margin of the worker each lane holds.  With few workers the offsets are split over the lanes:
  // lane c * GP + g takes every C-th group of four offsets of worker g (GP = workers rounded up to a power of
  // two, C = 64 / GP), the partial minima meet in LDS.  Padded offsets: envelope 0 against "no worker".
  const int GP = G <= 8 ? 8 : G <= 16 ? 16 : G <= 32 ? 32 : 64;
  const int C = BR_WAVE / GP;
  auto lane_minm = [&]() {
    const int g = lane & (GP - 1), c = lane / GP;
    int mn = INT32_MAX;
    const int *row = sL + min(g, LS - 1);  // lanes that stand for no worker read the last column (their result is never used)
    for (int h = 4 * c; h < HS; h += 4 * C) {
      const int4 M4 = *reinterpret_cast<const int4 *>(sM + h);
      const int l0 = row[(h + 0) * LS], l1 = row[(h + 1) * LS];
      const int l2 = row[(h + 2) * LS], l3 = row[(h + 3) * LS];
      mn = min(mn, min(min(M4.x - l0, M4.y - l1), min(M4.z - l2, M4.w - l3)));
    }
    if (C > 1) {
      pm[lane] = mn;
      br_wave_sync();
      for (int cc = 0; cc < C; ++cc) mn = min(mn, pm[cc * GP + g]);
      br_wave_sync();
    }
    return max(mn - add, 0);  // min_h (M_h - sL_h) - add, clamped once: the same as clamping every offset
  };

  // Rounding of one evaluation of eq. (brh-Fscore) in fp32: at most H + 5 roundings, each relative 2^-24 on terms
  // bounded by (alpha D + beta D) Delta, so a computed score differs from the exact one by at most
  // err_unit * Delta (a quarter of slack on top covers the rounding of this bound itself).
  float err_unit;
  {
    float Dsum = 0.0f;
    for (int h = 0; h < HS; h += 4) {
      const float4 q = *reinterpret_cast<const float4 *>(sd + h);
      Dsum += (q.x + q.y) + (q.z + q.w);
    }
    err_unit = 1.25f * (float)(p.H + 5) * 5.9604645e-8f * (p.aD + p.beta * Dsum);
  }

  // argmax_i F_g({i}) over alive, admissible requests against the margins in smg (lowest sorted
  // position on ties); false when no request is admissible.
  //
  // The exact score is concave in the request's length, and the waiting set is sorted by length: the search
  // brackets the maximum instead of scoring every request.  Probes: every E-th sorted position from the first
  // request in question on (up to 64 lanes), waiting or not, scored by the order-free evaluation (br_long_penalty_part, shared out by offset groups when
  // several waves serve the cluster); Fb is the best probe among the requests in question.  With e =
  // err_unit times the longest length (a bound on the distance of either evaluation from the exact score): a probe
  // that is longer than the best one and scores below Fb - 4 e has an exact score below the best probe's, by
  // concavity the exact score cannot rise again beyond it, and every position at or before it computes (in the
  // ordered evaluation) below what the best probe's request computes; likewise for a shorter probe and every
  // position at or after it.  What lies strictly between the nearest such probes on both sides of the best one
  // (at most 64 positions, else the full scan below takes over) is scored in the ordered evaluation, and the best
  // request in question there, lowest position on equal scores, is the argmax over the whole waiting set:
  // everything left out computes strictly below a score that was kept.
  int span_fa = -1, span_la = -1;
  bool span_dirty = true;
  // `sure_pos` >= 0 (Stage 2): the sorted position of the window's smallest entry.  The search then first decides,
  // from the probe at or after that position (a request no longer than that entry), whether the pop is certain to
  // end in the starvation guard: eq. (brh-Fscore) is concave with F(0) = 0, so F(Delta) <= F(s) Delta / s for every
  // Delta >= s; if that probe scores at or below -3 e(s) in the order-free evaluation, its exact score is at or
  // below -2 e(s), every subset of the window (all of them sum to at least s) has an exact score at or below
  // -2 e(Delta) and computes below zero.  If so the search goes on and returns the guard's pick; if not, it stops
  // with *unsure set and the caller enumerates the subsets.
  auto pick_single = [&](int room, int &pos, int &swin, int sure_pos = -1, bool *unsure = nullptr) -> bool {
    int bk, bp, km;
    {
      // first and last sorted position of a request in question: kept from search to search while the alive set
      // loses nothing at either end and no watermark narrows the set
      if (span_dirty || p.W > 0) {
        span_fa = -1, span_la = -1;
#pragma unroll
        for (int j = 0; j < E; ++j) {
          if (j * BR_WAVE < qn) {
            const unsigned long long bal = br_ballot(((alive >> j) & 1u) && sv[j] <= room);
            if (bal != 0ull) {
              if (span_fa < 0) span_fa = j * BR_WAVE + (int)__builtin_ctzll(bal);
              span_la = j * BR_WAVE + 63 - (int)__builtin_clzll(bal);
            }
          }
        }
        span_dirty = false;
      }
      const int fa = span_fa, la = span_la;
      if (fa < 0) return false;  // (no request in question: no subset of the window is admissible either)
      salive[lane] = (int)alive;
      br_wave_sync();
      const int p1 = lane * E;  // probe position
      const int e1 = skey[p1];
      const int s1 = e1 >> BR_IDX_BITS;
      const bool in1 = p1 < qn && p1 >= fa;  // (a probe before the first request in question brackets nothing that one does not)
      const bool q1 = in1 && (((unsigned)salive[p1 & 63] >> (p1 >> 6)) & 1u) && s1 <= room;
      const int top1 = br_uniform(skey[fa] >> BR_IDX_BITS);  // the longest request in question
      float pen1;
      if constexpr (NW > 1) {  // the probes' penalty sums are shared out by offset groups (the order is free here)
        mbox[2] = top1;
        mbox[0] = 2;
        __syncthreads();
        pen1 = br_long_penalty_part(smg, sd, HS, lane, top1, s1, SHARE);
        __syncthreads();
#pragma unroll
        for (int u = 1; u < NW; ++u) pen1 = __fadd_rn(pen1, __int_as_float(who[u * BR_WAVE + lane]));
      } else {
        pen1 = br_long_penalty_part(smg, sd, HS, lane, top1, s1, ~0ull);
      }
      const float F1 = br_scoreh_long_from(p.aD, p.beta, s1, pen1);
      if (sure_pos >= 0) {
        const int lw = (sure_pos + E - 1) / E;  // first probe at or after the window's smallest entry
        bool sure = false;
        if (lw < BR_WAVE && lw * E < qn) {
          const float Fw = __builtin_amdgcn_readlane(F1, lw);
          const int sw = __builtin_amdgcn_readlane(s1, lw);
          sure = Fw <= -3.0f * err_unit * (float)sw;
        }
        if (!sure) {
          *unsure = true;
          br_wave_sync();
          return false;
        }
      }
      const int k1 = q1 ? br_ord(F1) : BR_KEY_NONE;
      const int km1 = br_wave_max(k1);
      if (km1 != BR_KEY_NONE) {
        const int ls = (int)__builtin_ctzll(br_ballot(k1 == km1));
        const float thr = br_unord(km1) - 4.0f * err_unit * (float)top1;
        const unsigned long long ex = br_ballot(in1 && F1 < thr);
        const unsigned long long before = ex & ((1ull << ls) - 1ull);
        const unsigned long long after = ls < 63 ? ex >> (ls + 1) : 0ull;
        const int lo = before != 0ull ? (63 - (int)__builtin_clzll(before)) * E + 1 : fa;
        const int hi = after != 0ull ? min((ls + 1 + (int)__builtin_ctzll(after)) * E - 1, la) : la;
        const int nc = hi - lo + 1;
        if (nc <= BR_WAVE) {
          const int p2 = min(lo + lane, NP - 1);
          const int e2 = skey[p2];
          const int s2[1] = {e2 >> BR_IDX_BITS};
          const bool q2 = lane < nc && (((unsigned)salive[p2 & 63] >> (p2 >> 6)) & 1u) && s2[0] <= room;
          const int top2[1] = {__builtin_amdgcn_readfirstlane(s2[0])};
          float F2[1];
          br_scoreh_long_sel<1>(p.aD, p.beta, smg, sd, HS, lane, top2, s2, F2);
          const int k2 = q2 ? br_ord(F2[0]) : BR_KEY_NONE;
          const int km2 = br_wave_max(k2);
          const int l2 = (int)__builtin_ctzll(br_ballot(k2 == km2));  // positions rise with the lane: lowest first
          pos = lo + l2;
          swin = __builtin_amdgcn_readlane(s2[0], l2);
          br_wave_sync();
          return true;
        }
      }
      br_wave_sync();
    }
    if constexpr (NW > 1) {
      mbox[1] = room;
      salive[lane] = (int)alive;
      mbox[0] = 1;
      __syncthreads();
      br_long_slice_best<E, 0, EW>(p, smg, sd, HS, lane, qn, sv, alive, 0, room, bk, bp);
      km = br_wave_max(bk);
      pos = km == BR_KEY_NONE ? INT32_MAX : br_wave_min(bk == km ? bp : INT32_MAX);
      __syncthreads();
#pragma unroll
      for (int u = 1; u < NW; ++u) {
        const int ku = mbox[4 + 2 * u], pu = mbox[5 + 2 * u];
        if (ku > km) km = ku, pos = pu;  // positions of wave u lie above those of the waves before it
      }
      if (km == BR_KEY_NONE) return false;
    } else {
      if (p.W > 0) {  // under the watermark the longest alive requests may all be out of the question
        int smax = 0;
#pragma unroll
        for (int j = 0; j < E; ++j) smax = max(smax, (((alive >> j) & 1u) && sv[j] <= room) ? sv[j] : 0);
        if (br_wave_max(smax) == 0) return false;
      }
      br_long_slice_best<E, 0, E>(p, smg, sd, HS, lane, qn, sv, alive, 0, room, bk, bp);
      km = br_wave_max(bk);
      if (km == BR_KEY_NONE) return false;
      pos = br_wave_min(bk == km ? bp : INT32_MAX);
    }
    swin = br_uniform(skey[pos] >> BR_IDX_BITS);
    return true;
  };

  // sticky binding of the request at sorted position pos to worker g
  auto bind = [&](int pos, int g, int slot) {
    adm[pos] = (g << 16) | slot;  // every lane stores the same word
    const int jw = pos >> 6, lw = pos & 63;
    alive = (lane == lw) ? (alive & ~(1u << jw)) : alive;
    span_dirty |= pos == span_fa || pos == span_la;
  };

  // load update: the admitted length enters every horizon offset of worker g; the envelope follows.  Worker g is
  // the one whose margins were formed last (margins_of(g)): its projections are still in Lg.
  auto add_load = [&](int g, int delta, int k) {
    add += (lane == g) ? delta : 0;
    Lcur += (lane == g) ? delta : 0;
    const int ag = __builtin_amdgcn_readlane(add, g);
#pragma unroll
    for (int u = 0; u < 3; ++u) {
      const int h = u * BR_WAVE + lane;
      if (h < H1) {
        Mr[u] = max(Mr[u], Lg[u] + ag);
        sM[h] = Mr[u];
      }
    }
    br_wave_sync();
    cap -= (lane == g) ? k : 0;
    nn += (lane == g) ? k : 0;
    S_tot -= k;
    n_alive -= k;
    admitted += k;
  };

  auto drop_worker = [&](int g, int capg) {
    S_tot -= capg;
    cap = (lane == g) ? 0 : cap;
    ++wdrop;
  };

  if (run) {
    const int bound = qn + G + 1;  // every iteration admits a request or sets a worker aside

    // ---- Stage 1: greedy fill while free capacity is abundant.  Taken a level at a time: the workers that
    // share the largest free-slot count are picked once each in order of (load, index) before any other
    // worker can reach that count.  While the largest waiting request fits the next worker's horizon-min
    // margin (and the watermark), every penalty term of eq. (brh-Fscore) is zero for it, its score alpha D s
    // is the largest one, and the envelope does not move: the k-th lightest worker of the level takes the
    // k-th largest waiting request, all in one step.  The rest of the level goes one worker at a time.
    for (int it = 0; it < bound; ++it) {
      if (!(S_tot > p.S_greedy && n_alive > 0)) break;
      const int capmax = br_wave_max(cap);
      if (capmax <= 0) break;
      const bool member = cap == capmax;
      const int wkey = member ? (int)(((unsigned)Lcur << 6) | (unsigned)lane) : INT32_MAX;
      int rank = 0;
      for (int g0 = 0; g0 < G; g0 += 4) {  // lanes beyond G hold INT32_MAX and never count
#pragma unroll
        for (int u = 0; u < 4; ++u) rank += (__builtin_amdgcn_readlane(wkey, g0 + u) < wkey) ? 1 : 0;
      }
      const int level = __builtin_popcountll(br_ballot(member));
      const int kmaxp = min(level, min(S_tot - p.S_greedy, n_alive));
      {  // the first kmaxp alive requests, by rank, through LDS
        int base = 0;
#pragma unroll
        for (int j = 0; j < E; ++j) {
          if (base < kmaxp && j * BR_WAVE < qn) {
            const bool al = (alive >> j) & 1u;
            const unsigned long long bal = br_ballot(al);
            const int ar = base + br_rank_below(bal);
            if (al && ar < kmaxp) win[ar] = (sv[j] << BR_IDX_BITS) | (j * BR_WAVE + lane);
            base += __builtin_popcountll(bal);
          }
        }
      }
      br_wave_sync();
      const bool cand = member && rank < kmaxp;
      const int mine = cand ? win[rank] : 0;
      const int s_k = mine >> BR_IDX_BITS, pos_k = mine & IDX_MASK;
      int lim = lane_minm();
      if (p.W > 0) lim = min(lim, p.W - Lcur);
      const int k0 = br_wave_min((cand && s_k > lim) ? rank : kmaxp);
      if (k0 > 0) {
        const bool take = cand && rank < k0;
        if (take) adm[pos_k] = (lane << 16) | nn;
        add += take ? s_k : 0;
        Lcur += take ? s_k : 0;
        nn += take ? 1 : 0;
        cap -= take ? 1 : 0;
        const int pstar = br_uniform(win[k0 - 1] & IDX_MASK);  // last position taken; everything alive before it went too
        const int jf = pstar >> 6, lf = pstar & 63;
        const unsigned clear = ((1u << jf) - 1u) | ((lane <= lf) ? (1u << jf) : 0u);
        alive &= ~clear;
        span_dirty = true;
        S_tot -= k0;
        n_alive -= k0;
        admitted += k0;
        stage1 += k0;
      }
      br_wave_sync();
      for (int r = k0; r < level; ++r) {
        if (!(S_tot > p.S_greedy && n_alive > 0)) break;
        const int g = (int)__builtin_ctzll(br_ballot(member && rank == r));
        margins_of(g);
        const int room = p.W > 0 ? p.W - __builtin_amdgcn_readlane(Lcur, g) : INT32_MAX;
        int pos = 0, swin = 0;
        if (!pick_single(room, pos, swin)) {
          drop_worker(g, capmax);
          continue;
        }
        bind(pos, g, __builtin_amdgcn_readlane(nn, g));
        add_load(g, swin, 1);
        ++stage1;
      }
    }

    // ---- Stage 2: refined allocation over the workers that still have free slots
    int lbit[6];
#pragma unroll
    for (int b = 0; b < 6; ++b) lbit[b] = (lane >> b) & 1;
    const int lpop = __builtin_popcount(lane);
    for (int it = 0; it < bound; ++it) {
      if (n_alive <= 0) break;
      const int capmax = br_wave_max(cap);
      if (capmax <= 0) break;
      // priority (free slots, horizon-min margin), lowest index on ties
      const bool member = cap == capmax;
      const int mine_m = lane_minm();
      const int mm = br_wave_max(member ? mine_m : -1);
      const int g = (int)__builtin_ctzll(br_ballot(member && mine_m == mm));
      ++pops;
      margins_of(g);
      const int room = p.W > 0 ? p.W - __builtin_amdgcn_readlane(Lcur, g) : INT32_MAX;

      // candidate window: the first min(R_max, |R_wait|) alive requests in sorted order
      const int w = min(p.R_max, n_alive);
      {
        int base = 0;
#pragma unroll
        for (int j = 0; j < E; ++j) {
          if (base < w && j * BR_WAVE < qn) {
            const bool al = (alive >> j) & 1u;
            const unsigned long long bal = br_ballot(al);
            const int ar = base + br_rank_below(bal);
            if (al && ar < w) win[ar] = (sv[j] << BR_IDX_BITS) | (j * BR_WAVE + lane);
            base += __builtin_popcountll(bal);
          }
        }
      }
      br_wave_sync();
      const int kmax = min(capmax, p.R_max);
      const int nmask = 1 << w;
      int bestmask = 0, bestkey = BR_KEY_NONE;
      int wv[8], ws[8];
      // certain guard (decided inside the search from its probes): then `picked` holds the guard's pick already
      int gpos = 0, gswin = 0;
      bool unsure = false;
      const bool picked = pick_single(room, gpos, gswin, br_uniform(win[w - 1] & IDX_MASK), &unsure);
      const bool guard_sure = !unsure;
      if (guard_sure) {
        br_wave_sync();  // the window has been read before a later pop rewrites it
      } else if (p.R_max > 8) {
        // Windows of up to 16 requests: lane l keeps the lower six mask bits, the upper bits run as passes
        // over a table of their partial sums (built here, 64 entries per step), four passes per trip; trips
        // whose upper bits alone exceed the cardinality limit are skipped.  A lane sees its masks in ascending
        // order and keeps the first best; across lanes the lowest mask of the best score wins.
#pragma unroll
        for (int b = 0; b < 8; ++b) wv[b] = 0, ws[b] = 0;
        const int nhi = w > 6 ? 1 << (w - 6) : 1;
        for (int c0 = 0; c0 < nhi; c0 += BR_WAVE) {
          const int c = c0 + lane;
          int sum = 0;
          for (int b = 6; b < w; ++b) sum += ((c >> (b - 6)) & 1) * (win[b] >> BR_IDX_BITS);
          if (c < nhi) hitab[c] = sum;
        }
        int base = 0, top = 0;  // top: the largest sum any admissible subset can have (bound)
        for (int b = 0; b < w; ++b) {
          const int sb = win[b] >> BR_IDX_BITS;
          if (b < 6) base += ((lane >> b) & 1) * sb;
          if (b < kmax) top += sb;
        }
        top = min(top, room);
        br_wave_sync();
        unsigned long long act[3];
        br_long_active(smg, HS, lane, top, act);
        const int klim = kmax - lpop;
        const bool lane_ok = lane < nmask;
        int bk = BR_KEY_NONE, bm = INT32_MAX;
        for (int c0 = 0; c0 < nhi; c0 += 4) {
          if (__builtin_popcount(c0) > kmax) continue;
          const int4 h4 = *reinterpret_cast<const int4 *>(hitab + c0);  // (entries beyond nhi: masks out of range)
          const int hd[4] = {h4.x, h4.y, h4.z, h4.w};
          int dv[4];
          bool okv[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int c = c0 + u;
            const int delta = base + hd[u];
            okv[u] = lane_ok && c < nhi && __builtin_popcount(c) <= klim && delta <= room && (c != 0 || lane != 0);
            dv[u] = okv[u] ? delta : 0;
          }
          float Fv[4];
          br_scoreh_long_act<4>(p.aD, p.beta, smg, sd, act, dv, Fv);
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int key = okv[u] ? br_ord(Fv[u]) : BR_KEY_NONE;
            if (key > bk) {
              bk = key;
              bm = (c0 + u) * BR_WAVE + lane;
            }
          }
        }
        bestkey = br_wave_max(bk);
        bestmask = bestkey == BR_KEY_NONE ? 0 : br_wave_min(bk == bestkey ? bm : INT32_MAX);
        br_wave_sync();
      } else {
      {
        const int4 lo = *reinterpret_cast<const int4 *>(win);
        const int4 hi = *reinterpret_cast<const int4 *>(win + 4);
        wv[0] = lo.x, wv[1] = lo.y, wv[2] = lo.z, wv[3] = lo.w;
        wv[4] = hi.x, wv[5] = hi.y, wv[6] = hi.z, wv[7] = hi.w;
      }
#pragma unroll
      for (int b = 0; b < 8; ++b) ws[b] = b < w ? (wv[b] >> BR_IDX_BITS) : 0;
      br_wave_sync();  // every lane holds the window before a later pop rewrites it

      // exhaustive subset search: lane l of pass c stands for mask c*64 + l (ascending masks, a later
      // one wins only if strictly better)
      int dv[4];
      bool okv[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        int delta = (c & 1) * ws[6] + (c >> 1) * ws[7];
#pragma unroll
        for (int b = 0; b < 6; ++b)
          if (b < w) delta += lbit[b] * ws[b];
        const int mask = c * BR_WAVE + lane;
        dv[c] = delta;
        okv[c] = mask != 0 && mask < nmask && lpop + __builtin_popcount(c) <= kmax && delta <= room;
      }
      float Fv[4] = {0.0f, 0.0f, 0.0f, 0.0f};
      int dmax = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) dmax = max(dmax, okv[c] ? dv[c] : 0);
      dmax = br_wave_max(dmax);
      if (dmax > 0) {  // else no subset is admissible
        unsigned long long act[3];
        br_long_active(smg, HS, lane, dmax, act);
        if (nmask <= BR_WAVE) {
          const int d1[1] = {dv[0]};
          float F1[1];
          br_scoreh_long_act<1>(p.aD, p.beta, smg, sd, act, d1, F1);
          Fv[0] = F1[0];
        } else {
          br_scoreh_long_act<4>(p.aD, p.beta, smg, sd, act, dv, Fv);
        }
      }
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        if (c * BR_WAVE < nmask) {
          const int key = okv[c] ? br_ord(Fv[c]) : BR_KEY_NONE;
          const int km = br_wave_max(key);
          if (km > bestkey) {
            bestkey = km;
            bestmask = c * BR_WAVE + (int)__builtin_ctzll(br_ballot(key == km));
          }
        }
      }

      }

      if (bestmask == 0 || bestkey <= 0) {  // starvation guard: the single best request anyway
        ++guard;
        int pos = gpos, swin = gswin;
        if (!(guard_sure ? picked : pick_single(room, pos, swin))) {
          drop_worker(g, capmax);
          continue;
        }
        bind(pos, g, __builtin_amdgcn_readlane(nn, g));
        add_load(g, swin, 1);
      } else {
        // lane b binds window entry b if chosen; slots follow the order of the window
        const int slot = __builtin_amdgcn_readlane(nn, g);
        int delta = 0;
        if (p.R_max > 8) {
          if (lane < 16 && ((bestmask >> lane) & 1))
            adm[win[lane] & IDX_MASK] = (g << 16) | (slot + __builtin_popcount(bestmask & ((1 << lane) - 1)));
          for (int b = 0; b < w; ++b)
            if ((bestmask >> b) & 1) {
              const int e = win[b];
              const int pb = e & IDX_MASK;
              alive = (lane == (pb & 63)) ? (alive & ~(1u << (pb >> 6))) : alive;
              span_dirty = true;
              delta += e >> BR_IDX_BITS;
            }
          br_wave_sync();  // the window has been read before a later pop rewrites it
        } else {
          const bool mine = lane < 8 && ((bestmask >> lane) & 1);
          if (mine) {
            const int me = lane == 0 ? wv[0] : lane == 1 ? wv[1] : lane == 2 ? wv[2] : lane == 3 ? wv[3]
                         : lane == 4 ? wv[4] : lane == 5 ? wv[5] : lane == 6 ? wv[6] : wv[7];
            adm[me & IDX_MASK] = (g << 16) | (slot + __builtin_popcount(bestmask & ((1 << lane) - 1)));
          }
#pragma unroll
          for (int b = 0; b < 8; ++b)
            if ((bestmask >> b) & 1) {
              const int pb = wv[b] & IDX_MASK;
              alive = (lane == (pb & 63)) ? (alive & ~(1u << (pb >> 6))) : alive;
              span_dirty = true;
              delta += ws[b];
            }
        }
        add_load(g, br_uniform(delta), __builtin_popcount(bestmask));
      }
    }
  }
  br_wave_sync();
  if constexpr (NW > 1) {
    mbox[0] = 0;  // the round is over: the helper waves leave
    __syncthreads();
#pragma unroll
    for (int u = 1; u < NW; ++u) who[u * BR_WAVE + lane] = -1;  // (held the helpers' partial sums)
    br_wave_sync();
  }

  BrRoundCounts rc;
  rc.admitted = admitted;
  rc.stage1 = stage1;
  rc.pops = pops;
  rc.guard = guard;
  rc.wdrop = wdrop;
  rc.I_before = I_before;
  br_assign_epilogue<E>(inst, lane, q0, qn, cnt, skey, adm, who, Lcur, nn, rc, c0);
  if constexpr (ADV) br_advance_cluster<4, true>(inst, lane, Lcur, nn);
}

// Waves per cluster: as many as still leave every cluster of the batch resident at once (registers allow about
// 4 / 3 / 2 / 1 waves per SIMD for queues of up to 256 / 512 / 1024 / 2048 on 1024 SIMDs).
int br_long_waves(const BrParams &p) {
  const long long room = 1024ll * (p.Q <= 256 ? 4 : p.Q <= 512 ? 3 : p.Q <= 1024 ? 2 : 1);
  return (long long)p.N * 4 <= room ? 4 : (long long)p.N * 2 <= room ? 2 : 1;
}

template <int E>
static void br_launch_assign_long_one(const BrParams &p, const BrArr &a, const BrOut &o, hipStream_t st) {
  const int HS = BR_HS(p.H);
  const int nw = br_long_waves(p);
  const size_t lds = ((size_t)3 * E * BR_WAVE + 2 * BR_WAVE + 3 * (size_t)HS + (((size_t)HS * BR_LSTRIDE(p.G) + 3) & ~(size_t)3) +
                      (p.R_max > 8 ? 1024 : 0) + (nw > 1 ? 16 : 0)) * sizeof(int);
  const dim3 grid((unsigned)p.N), block(BR_WAVE * nw);
  if (nw == 4)
    hipLaunchKernelGGL((br_k_assign_long<E, false, 4>), grid, block, lds, st, p, a, o);
  else if (nw == 2)
    hipLaunchKernelGGL((br_k_assign_long<E, false, 2>), grid, block, lds, st, p, a, o);
  else if (p.adv_t > 0)
    hipLaunchKernelGGL((br_k_assign_long<E, true, 1>), grid, block, lds, st, p, a, o);
  else
    hipLaunchKernelGGL((br_k_assign_long<E, false, 1>), grid, block, lds, st, p, a, o);
}

void br_launch_assign_long(const BrParams &p, const BrArr &a, const BrOut &o, hipStream_t st) {
  if (p.Q <= 256)
    br_launch_assign_long_one<4>(p, a, o, st);
  else if (p.Q <= 512)
    br_launch_assign_long_one<8>(p, a, o, st);
  else if (p.Q <= 1024)
    br_launch_assign_long_one<16>(p, a, o, st);
  else
    br_launch_assign_long_one<32>(p, a, o, st);
}
