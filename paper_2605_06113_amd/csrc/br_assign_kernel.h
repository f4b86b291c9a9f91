// Sequential two-stage assignment of one scheduling round (Appendix, Alg. BR-0 / Alg. BR-H),
// one wavefront per cluster.
//
// The round is a dependent chain: every admission changes L_g, possibly the envelope M and
// with it every margin.  The chain therefore stays inside one wave, with no block barrier and
// no HBM access on its critical path:
//   - lane g holds worker g's state (free slots, projected loads L_g(k+h), request count);
//   - the waiting set, ordered by prefill length (largest first, arrival order among equals),
//     lives in registers, E requests per lane, sorted position = j*64 + lane, with a copy of the
//     sorted keys in LDS for uniform look-ups;
//   - "pick a worker" and "pick a request" are DPP reductions on packed int32 keys; Stage-2
//     subsets are enumerated one subset mask per lane.
//
// Stage 1 is taken a whole capacity level at a time where that is provably the same as the
// one-by-one loop: the workers that share the largest free-slot count are picked once each in
// order of load, and as long as the largest waiting request still fits the next worker's
// (horizon-min) margin its score is the largest one (score = const * s in the safe regime of
// eq. (br0-Fscore) / eq. (brh-Fscore)), the envelope does not move, and the k-th lightest worker
// takes the k-th largest waiting request.  The first worker for which this fails falls back to
// the full single-request search.
//
// BR-0 with G > 1 has three more steps of the same kind (the one-step forms only without a token
// watermark), each stated and argued where it is coded: when no waiting request is shorter than a worker's margin the best single request is the
// shortest one (two ballots instead of a scan); from the first Stage-1 worker of a level for which
// that holds, the rest of the level takes the shortest requests in order, in one step; Stage 2 skips
// the subset enumeration when the window's smallest entry alone scores <= 0 (the starvation guard is
// then certain), and takes the consecutive guard pops of one free-slot count in one step while the
// window stays untouched.
//
// Ties: Stage 1 worker (most free slots, then lightest, then lowest index); Stage 2 worker
// (most free slots, then largest horizon-min margin, then lowest index); equal request scores
// resolve to the lowest sorted position; equal subset scores to the lowest mask.
//
// ADV: the wave goes on to apply the decode steps to the lists of the cluster it has routed
// (br_route_advance); a separate instantiation, so that the two kinds of launch carry distinct
// kernel names in profiles.
#pragma once

#include "br_device.h"
#include "br_launch.h"
#include <type_traits>

#include "br_sort.h"
#include "br_assign_common.h"
#include "br_subset_dp.h"
#include "br_score_wave.h"

template <int E>
struct Log2E {
  static constexpr int v = E == 4 ? 2 : E == 8 ? 3 : E == 16 ? 4 : 5;
};

// Subset scan of a window of up to 16 requests (Stage 2, BIGR), this wave's share of it: lane l keeps the lower
// six mask bits, the upper bits c run as passes over the table `hitab` of their partial sums, four passes per
// trip; the wave takes the trips wv, wv + nwv, ... (trips whose upper bits alone exceed the cardinality limit are
// skipped).  A lane sees its masks in ascending order and keeps the first best: returns the lane's best key and
// its lowest mask.
template <bool BRH>
__device__ __forceinline__ void br_bigr_scan(const BrParams &p, const int (&mg)[BR_HP + 1], const int *win, const int *hitab,
                                             int w, int kmax, int room, int lane, int wv, int nwv, int &bk, int &bm) {
  const int nhi = w > 6 ? 1 << (w - 6) : 1;
  const int nmask = 1 << w;
  int base = 0;
  for (int b = 0; b < min(w, 6); ++b) base += ((lane >> b) & 1) * (win[b] >> BR_IDX_BITS);
  const int klim = kmax - __builtin_popcount(lane);  // bits the upper part of a mask may still add on this lane
  const bool lane_ok = lane < nmask;                  // (windows below six requests use the lower lanes only)
  bk = BR_KEY_NONE, bm = INT32_MAX;
  for (int c0 = 4 * wv; c0 < nhi; c0 += 4 * nwv) {  // four passes per trip: one 16-byte table read, independent scores
    if (__builtin_popcount(c0) > kmax) continue;     // c0 + u has at least the bits of c0: too many for every lane
    const int4 h4 = *reinterpret_cast<const int4 *>(hitab + c0);
    const int hd[4] = {h4.x, h4.y, h4.z, h4.w};
    int key[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int c = c0 + u;
      const int delta = base + hd[u];
      bool ok = lane_ok && c < nhi && __builtin_popcount(c) <= klim && delta <= room;
      if (c == 0) ok = ok && lane != 0;  // the empty subset
      const int k = br_score_key<BRH>(p, mg, ok ? delta : 0);
      key[u] = ok ? k : BR_KEY_NONE;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (key[u] > bk) {
        bk = key[u];
        bm = (c0 + u) * BR_WAVE + lane;
      }
  }
}

// One cluster's round on one wave.  `lds`: this wave's 3*E*64 + 72 words.  COOP (queues of up to 2048):
// the block has four waves; all of them sort the waiting set together (br_sort_desc_block4), wave 0 runs
// the round with the sorted keys read back from LDS and hands every full search over the waiting set
// (argmax_i F_g({i})) to all four, 512 sorted positions each; all four share the epilogue and the decode step.
template <int E, bool BRH, bool ADV, bool COOP = false, bool BIGR = false>
// `pre`: what the snapshot reductions of the same wave have already loaded for this cluster (queue lengths,
// prefill lengths in arrival order, worker loads and counts), or null: the round then loads them itself.
// `split`: the cluster's BR_SPLIT_WORDS of LDS in a split kernel (another wave applies the decode steps to the old
// list entries meanwhile), or null.
// `shared` (BIGR without COOP, one cluster per block of four waves): waves 1-3 serve the subset searches of wave 0
// (every fourth trip of a mask scan, every fourth run of 64 words of the rows of reachable sums) through the
// mailbox `svc` and two block barriers per search.
__device__ __forceinline__ void br_assign_body(const BrParams &p, const BrArr &a, const BrOut &o, int *lds, int inst,
                                               int w = 0, const BrScoreIn<E, BRH> *pre = nullptr, int *split = nullptr,
                                               bool shared = false) {
  static_assert(!COOP || E == 32, "the four-wave sort covers 4 x 512 keys");
  constexpr int NP = E * BR_WAVE;
  constexpr int NH = BRH ? BR_HP + 1 : 1;
  constexpr int IDX_MASK = (1 << BR_IDX_BITS) - 1;
  constexpr int PB = 6 + Log2E<E>::v;          // bits of a sorted position
  constexpr bool PACK1 = !BRH && E <= 16;      // (score, position) of one request fits 32 bits
  constexpr int BIAS1 = 1 << 21;               // single request: score in (-2^21, 2^15]
  constexpr int BIAS2 = 1 << 24;               // subset of <= 8 requests: score in (-2^24, 2^18]
  if (inst >= p.N) return;
  int *skey = lds;            // [NP] sort buffer, then the sorted keys (s << 11 | 2047 - arrival position)
  int *adm = lds + NP;        // [NP] by sorted position: worker << 16 | slot, or -1
  int *who = lds + 2 * NP;    // [NP] by arrival position: worker, or -1
  int *slots = lds + 3 * NP;  // [64] k-th alive request of a Stage-1 level: s << 11 | sorted position
  int *win = slots + BR_WAVE; // [8]  Stage-2 candidate window, same packing (16-byte aligned); BIGR: [32]
  int *hitab = win + 32;      // BIGR: [1024] sums of the window entries 6.. selected by the upper mask bits (16-byte aligned)
  // COOP: mailbox of the searches that wave 0 hands to all four waves (one per 512 sorted positions)
  int *svc = win + (BIGR ? 32 + 1024 : 8);  // [16] 0: 1 = search, 0 = round over; 1..9: margins; 10: room
  // BIGR with windows beyond 16 requests: bit rows of the subset search (present when R_max > 16), after the rest
  int *dprows = lds + 3 * NP + BR_WAVE + 32 + 1024 + (COOP ? 96 : (shared ? 32 : 0));
  int *salive = svc + 16;                   // [64] wave 0's alive bits, one word per lane
  int *sres = salive + BR_WAVE;             // [8]  per wave: best key, its lowest sorted position

  const int lane = br_lane();
  if constexpr (BIGR && !COOP) {
    if (shared && w != 0) {  // one pass per scan; every wave of the block meets at both barriers, wave 0 ends the loop
      for (;;) {
        __syncthreads();
        const int cmd = svc[0];
        if (cmd == 0) break;
        if (cmd == 2) {  // this wave's words of the rows of reachable sums
          br_dp_build_helper(p, win, svc, dprows, p.dp + (size_t)inst * br_dp_cluster_words(min(p.B, p.R_max)), lane, w);
        } else {         // this wave's trips of a mask scan
          int mgq[BR_HP + 1];
#pragma unroll
          for (int h = 0; h <= BR_HP; ++h) mgq[h] = svc[1 + h];
          int bk, bm;
          br_bigr_scan<BRH>(p, mgq, win, hitab, svc[3 + BR_HP], svc[4 + BR_HP], svc[2 + BR_HP], lane, w, 4, bk, bm);
          const int km = br_wave_max(bk);
          const int mm = km == BR_KEY_NONE ? INT32_MAX : br_wave_min(bk == km ? bm : INT32_MAX);
          if (lane == 0) svc[16 + 2 * w] = km, svc[17 + 2 * w] = mm;
        }
        __syncthreads();
      }
      return;
    }
  }
  const int G = p.G;
  // Loads: everything that does not need the queue length is requested before the first result is used, and the
  // waiting set then comes in one batch of unconditional loads (below): two memory round trips for the cluster.
  const bool act = lane < G;
  const int64_t wrow = (int64_t)inst * G + lane;
  int q0_raw = 0, cnt_raw = 0, n_raw = p.B, L_raw[NH];
#pragma unroll
  for (int h = 0; h < NH; ++h) L_raw[h] = BR_LOW;
  const int64_t wrow_ld = act ? wrow : (int64_t)inst * G;  // lanes without a worker read worker 0's words (unused)
  if (!pre) {
    q0_raw = p.qlen[inst];
    cnt_raw = a.count ? a.count[inst] : 0;
    n_raw = p.n[wrow_ld];
    if constexpr (!BRH) L_raw[0] = p.L[wrow_ld];
  }
  if constexpr (BRH) {
#pragma unroll
    for (int h = 0; h < NH; ++h) L_raw[h] = p.Lh[wrow_ld * (p.H + 1) + min(h, p.H)];
  }
  if (!act) {
    n_raw = p.B;
#pragma unroll
    for (int h = 0; h < NH; ++h) L_raw[h] = BR_LOW;
  }
  int q0, cnt;
  if (pre) {
    q0 = pre->q0, cnt = pre->cnt;
  } else {
    q0 = br_uniform(min(max(q0_raw, 0), p.Q));
    cnt = br_uniform(min(max(cnt_raw, 0), a.arr_cap));
  }
  const int qn = q0 + min(cnt, p.Q - q0);
  const int64_t qrow = (int64_t)inst * p.Q, arow = (int64_t)inst * a.arr_cap;
  // the waiting set's prefill lengths, unclamped: addresses by select, an entry beyond the set reads the cluster's
  // first queue word (COOP and `pre`: loaded elsewhere)
  int s_raw[E];
  if constexpr (!COOP) {
    if (!pre) {
#pragma unroll
      for (int j = 0; j < E; ++j) {
        const int i = j * BR_WAVE + lane;
        const bool ina = i >= q0 && i < qn;
        const int32_t *src = ina ? a.s + (arow + (i - q0)) : p.qs + (qrow + (i < q0 ? i : 0));
        s_raw[j] = *src;
      }
    }
  }

  // first estimate of a newly admitted request when the library maintains c_hat (age 0)
  float c0 = 0.0f;
  if constexpr (BRH) {
    if (p.pred_mode == 2) c0 = br_survival(p, 0);
  }

  unsigned xk[E];
  if constexpr (COOP) {
    unsigned x8[8];
    int s8[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {  // one batch of unconditional loads (an entry beyond the set reads the first queue word)
      const int i = w * 512 + j * BR_WAVE + lane;
      const bool ina = i >= q0 && i < qn;
      const int32_t *src = ina ? a.s + (arow + (i - q0)) : p.qs + (qrow + (i < q0 ? i : 0));
      s8[j] = *src;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int i = w * 512 + j * BR_WAVE + lane;
      unsigned key = 0;
      if (i < qn) {
        const int s = min(max(s8[j], 1), BR_MAX_S_DEV);
        key = ((unsigned)s << BR_IDX_BITS) | (unsigned)(IDX_MASK - i);
      }
      x8[j] = key;
      adm[i] = -1;
      who[i] = -1;
    }
    if (qn > 512) {  // same for every wave of the block
      br_sort_desc_block4(x8, skey, w, lane);
    } else if (w == 0 && qn > 0) {  // everything is in wave 0's slice
      int N2 = BR_WAVE;
      while (N2 < qn) N2 <<= 1;
      br_sort_desc<8>(x8, lane, N2);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) skey[w * 512 + j * BR_WAVE + lane] = (int)x8[j];
    __syncthreads();
    if (w != 0) {  // waves 1-3 serve wave 0's searches during the round, then take their share of the epilogue and the decode step
      int sv8[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) sv8[j] = (int)(x8[j] >> BR_IDX_BITS);
      for (;;) {  // one pass per search; every wave of the block meets at both barriers, wave 0 ends the loop
        __syncthreads();
        if (svc[0] == 0) break;
        int mgq[BR_HP + 1];
#pragma unroll
        for (int h = 0; h <= BR_HP; ++h) mgq[h] = svc[1 + h];
        const int roomq = svc[2 + BR_HP];
        const unsigned al = (unsigned)salive[lane] >> (8 * w);
        int bk = BR_KEY_NONE, bp = INT32_MAX;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const bool ok = ((al >> j) & 1u) && sv8[j] <= roomq;
          int key = br_score_key<BRH>(p, mgq, sv8[j]);
          key = ok ? key : BR_KEY_NONE;
          if (key > bk) {
            bk = key;
            bp = w * 512 + j * BR_WAVE + lane;
          }
        }
        const int km = br_wave_max(bk);
        const int pm = km == BR_KEY_NONE ? INT32_MAX : br_wave_min(bk == km ? bp : INT32_MAX);
        if (lane == 0) sres[2 * w] = km, sres[2 * w + 1] = pm;
        __syncthreads();
      }
      int Lw = 0, nw = 0;
      BrRoundCounts none = {};
      br_assign_epilogue_block4(inst, lane, w, q0, qn, cnt, skey, adm, who, slots, Lw, nw, none, c0, ADV);
      if constexpr (ADV) {
        const int per = (G + 3) >> 2;
        br_advance_cluster<4, BRH>(inst, lane, Lw, nw, min(w * per, G), min(w * per + per, G));
      }
      return;
    }
#pragma unroll
    for (int j = 0; j < E; ++j) xk[j] = (unsigned)skey[j * BR_WAVE + lane];
  }

  // ---- worker state, one worker per lane
  int nn = act ? min(max(pre ? pre->n : n_raw, 0), p.B) : p.B;
  int cap = p.B - nn;
  const int nn_start = nn;
  int Lh[NH], Mh[NH];
  if constexpr (BRH) {
#pragma unroll
    for (int h = 0; h < NH; ++h) Lh[h] = L_raw[h];
  } else {
    Lh[0] = act ? (pre ? pre->L : L_raw[0]) : BR_LOW;
  }
#pragma unroll
  for (int h = 0; h < NH; ++h) Mh[h] = br_wave_max(Lh[h]);
  int S_tot = br_wave_sum(cap);
  const bool small = G <= 16;  // every worker sits in the first row of 16 lanes: row reductions serve
  // largest free-slot count among the workers: free slots only shrink during a round, so the value is tracked
  // downwards with ballots instead of a reduction per pick
  int capmax_cur = br_wave_max(cap);
  auto cap_max = [&]() -> int {
    while (capmax_cur > 0 && br_ballot(cap == capmax_cur) == 0ull) --capmax_cur;
    return capmax_cur;
  };
  auto workers_max = [&](int x) -> int { return small ? br_row0_max(x) : br_wave_max(x); };
  auto workers_min = [&](int x) -> int { return small ? br_row0_min(x) : br_wave_min(x); };
  // rank of each member among the members by (load, index): lanes that are no members hold INT32_MAX
  auto rank_of = [&](int wkey) -> int {
    if (small) return br_row_rank(wkey);
    int rank = 0;
    for (int g0 = 0; g0 < G; g0 += 4) {  // lanes beyond G hold INT32_MAX and never count
#pragma unroll
      for (int u = 0; u < 4; ++u) rank += (__builtin_amdgcn_readlane(wkey, g0 + u) < wkey) ? 1 : 0;
    }
    return rank;
  };

  // sum of loads in two 16-bit halves (each partial sum fits int32 for loads below 2^25)
  auto sum_loads = [&]() -> long long {
    const int L0 = act ? Lh[0] : 0;
    return ((long long)br_wave_sum(L0 >> 16) << 16) + br_wave_sum(L0 & 0xffff);
  };
  const long long I_before = o.stats ? (long long)G * Mh[0] - sum_loads() : 0;

  // ---- waiting set: keys (s << 11 | 2047 - arrival position) sorted in registers, descending;
  //      a copy goes to LDS for uniform look-ups
  const bool run = S_tot > 0 && qn > 0;
  if constexpr (!COOP) {
#pragma unroll
    for (int j = 0; j < E; ++j) {
      const int i = j * BR_WAVE + lane;
      unsigned key = 0;
      if (i < qn) {
        int s;
        if (pre) {
          s = pre->s[j];  // already clamped
        } else {
          s = min(max(s_raw[j], 1), BR_MAX_S_DEV);
        }
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
  }
  int sv[E];
  unsigned alive = 0;
#pragma unroll
  for (int j = 0; j < E; ++j) {
    const int pos = j * BR_WAVE + lane;
    if constexpr (!COOP) skey[pos] = (int)xk[j];  // (already there after the four-wave sort)
    sv[j] = (int)(xk[j] >> BR_IDX_BITS);
    if (pos < qn) alive |= 1u << j;
  }
  br_wave_sync();

  int n_alive = qn;
  int jhead = 0;  // blocks below jhead hold no alive request any more
  int stage1 = 0, pops = 0, guard = 0, wdrop = 0, admitted = 0;

  auto advance_head = [&]() {
    while (jhead < E - 1 && br_ballot((alive >> jhead) & 1u) == 0ull) ++jhead;
  };

  // lane-constant part of a packed (score, position) key: bias << PB | (NP-1 - position)
  unsigned ckey[E];
#pragma unroll
  for (int j = 0; j < E; ++j) ckey[j] = ((unsigned)BIAS1 << PB) + (unsigned)(NP - 1 - (j * BR_WAVE + lane));

  // argmax_i F_g({i}) over alive, admissible requests (lowest sorted position on ties).
  // Returns false when no request is admissible.
  auto pick_single = [&](const int(&mg)[BR_HP + 1], int room, int &pos, int &swin) -> bool {
    if constexpr (PACK1) {
      unsigned bk = 0;
      const int negG = -(G & 0x7f);
      auto scan = [&](auto wm) {
#pragma unroll
        for (int j = 0; j < E; ++j) {
          if (E <= 8 || (j >= jhead && j * BR_WAVE < qn)) {  // few registers: cheaper to score all than to branch
            const int s = sv[j];
            const int F = s + (max(s - mg[0], 0) & 0xffff) * negG;       // one 24-bit multiply-add
            unsigned key = ((unsigned)F << PB) + ckey[j];
            key &= (unsigned)(((int)(alive << (31 - j))) >> 31);         // all ones if still waiting
            if constexpr (decltype(wm)::value) key = s <= room ? key : 0u;
            bk = max(bk, key);
          }
        }
      };
      if (p.W > 0)
        scan(std::true_type{});
      else
        scan(std::false_type{});
      const unsigned km = br_wave_umax(bk);
      if (km == 0u) return false;
      pos = NP - 1 - (int)(km & (unsigned)(NP - 1));
      if constexpr (E <= 8) {  // the winner's length straight from its register, no LDS round trip
        const int lw = pos & 63, jw = pos >> 6;
        int sw = __builtin_amdgcn_readlane(sv[0], lw);
#pragma unroll
        for (int j = 1; j < E; ++j) {
          const int sj = __builtin_amdgcn_readlane(sv[j], lw);
          sw = jw == j ? sj : sw;
        }
        swin = sw;
        return true;
      }
    } else if constexpr (COOP) {
      // the four waves search 512 sorted positions each: the request goes out through LDS, every wave returns
      // its best (score, lowest position), the best of the four wins (lower position on equal scores)
#pragma unroll
      for (int h = 0; h <= BR_HP; ++h) svc[1 + h] = mg[h];
      svc[2 + BR_HP] = room;
      salive[lane] = (int)alive;
      svc[0] = 1;
      __syncthreads();
      int bk = BR_KEY_NONE, bp = INT32_MAX;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int s = sv[j];
        const bool ok = ((alive >> j) & 1u) && s <= room;
        int key = br_score_key<BRH>(p, mg, s);
        key = ok ? key : BR_KEY_NONE;
        if (key > bk) {
          bk = key;
          bp = j * BR_WAVE + lane;
        }
      }
      int km = br_wave_max(bk);
      pos = km == BR_KEY_NONE ? INT32_MAX : br_wave_min(bk == km ? bp : INT32_MAX);
      __syncthreads();
#pragma unroll
      for (int u = 1; u < 4; ++u) {
        const int ku = sres[2 * u], pu = sres[2 * u + 1];
        if (ku > km) km = ku, pos = pu;  // positions of wave u lie above those of the waves before it
      }
      if (km == BR_KEY_NONE) return false;
    } else {
      int bk = BR_KEY_NONE, bp = INT32_MAX;
#pragma unroll
      for (int j = 0; j < E; ++j) {
        if (j >= jhead && j * BR_WAVE < qn) {
          const int s = sv[j];
          const bool ok = ((alive >> j) & 1u) && s <= room;
          int key = br_score_key<BRH>(p, mg, s);
          key = ok ? key : BR_KEY_NONE;
          if (key > bk) {
            bk = key;
            bp = j * BR_WAVE + lane;
          }
        }
      }
      const int km = br_wave_max(bk);
      if (km == BR_KEY_NONE) return false;
      const unsigned long long tie = br_ballot(bk == km);
      if ((tie & (tie - 1)) == 0ull)
        pos = __builtin_amdgcn_readlane(bp, (int)__builtin_ctzll(tie));
      else
        pos = br_wave_min(bk == km ? bp : INT32_MAX);
    }
    swin = br_uniform(skey[pos] >> BR_IDX_BITS);
    return true;
  };

  // margins of worker g against the current envelope
  auto margins_of = [&](int g, int(&Lg)[NH], int(&mg)[BR_HP + 1]) {
#pragma unroll
    for (int h = 0; h <= BR_HP; ++h) mg[h] = 0;
#pragma unroll
    for (int h = 0; h < NH; ++h) {
      Lg[h] = __builtin_amdgcn_readlane(Lh[h], g);
      mg[h] = max(Mh[h] - Lg[h], 0);
    }
  };

  // horizon-min margin of the worker each lane holds
  auto lane_minm = [&]() {
    int mn = INT32_MAX;
#pragma unroll
    for (int h = 0; h < NH; ++h) mn = min(mn, max(Mh[h] - Lh[h], 0));
    return mn;
  };

  // BR-0 with G > 1: when no waiting request is shorter than the margin,
  // eq. (br0-Fscore) is G m - (G-1) s on the whole waiting set, so argmax_i F_g({i}) is the shortest
  // request (earliest arrival among equals) and no scan is needed.  The shortest waiting request is
  // the last alive position of the sorted set; it is looked up again after it has been taken.
  const bool tail_rule = !BRH && G > 1;
  const bool tail_bulk_ok = p.W <= 0;  // the one-step admissions below are argued without the watermark
  int tail_pos = -1, tail_s = 0;
  bool tail_dirty = true;
  auto ensure_tail = [&]() {
    if (!tail_dirty) return;
    tail_dirty = false;
    tail_pos = -1;
    tail_s = 0;
#pragma unroll
    for (int j = E - 1; j >= 0; --j) {
      if (tail_pos < 0 && j * BR_WAVE < qn) {
        const unsigned long long bal = br_ballot((alive >> j) & 1u);
        if (bal != 0ull) {
          const int l = 63 - (int)__builtin_clzll(bal);
          tail_pos = j * BR_WAVE + l;
          tail_s = __builtin_amdgcn_readlane(sv[j], l);
        }
      }
    }
  };
  // the earliest arrival among the alive requests of the shortest length
  auto pick_tail = [&](int &pos, int &swin) {
    pos = tail_pos;
#pragma unroll
    for (int j = E - 1; j >= 0; --j) {
      if (j * BR_WAVE <= tail_pos) {
        const unsigned long long c = br_ballot(((alive >> j) & 1u) && sv[j] == tail_s);
        if (c != 0ull) pos = j * BR_WAVE + (int)__builtin_ctzll(c);
      }
    }
    swin = tail_s;
  };

  // sticky binding of the request at sorted position pos to worker g
  auto bind = [&](int pos, int g, int slot) {
    adm[pos] = (g << 16) | slot;  // every lane stores the same word: no lane masking needed
    const int jw = pos >> 6, lw = pos & 63;
    alive = (lane == lw) ? (alive & ~(1u << jw)) : alive;
    tail_dirty |= pos == tail_pos;
  };

  // load update: the admitted length enters every horizon offset; envelope follows
  auto add_load = [&](int g, const int(&Lg)[NH], int delta, int k) {
#pragma unroll
    for (int h = 0; h < NH; ++h) {
      Lh[h] += (lane == g) ? delta : 0;
      Mh[h] = max(Mh[h], Lg[h] + delta);
    }
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

  // Admission of the K shortest waiting requests, in order of (length, arrival), to the workers with
  // `member` set and rank r0 .. r0+K-1 (one each; ranks order the members by load, then index).
  // `smax` >= 0 limits K to the requests no longer than smax.  Returns the number admitted, or 0
  // when the order cannot be read off the 64 shortest requests (a run of equal lengths crossing
  // that edge).  Loads, free slots, the envelope and the alive set are updated; counters are the
  // caller's.
  auto tail_bulk = [&](bool member, int rank, int r0, int K, int smax) -> int {
    int base = 0;
#pragma unroll
    for (int j = E - 1; j >= 0; --j) {  // the 64 shortest alive requests, shortest first, through LDS
      if (base < BR_WAVE && j * BR_WAVE < qn) {
        const bool al = (alive >> j) & 1u;
        const unsigned long long bal = br_ballot(al);
        const int cj = __builtin_popcountll(bal);
        const int rr = base + cj - 1 - br_rank_below(bal);
        if (al && rr < BR_WAVE) slots[rr] = (sv[j] << BR_IDX_BITS) | (j * BR_WAVE + lane);
        base += cj;
      }
    }
    br_wave_sync();
    const int nA = min(n_alive, BR_WAVE);
    const bool valid = lane < nA;
    const int e = slots[lane];
    const int eprev = slots[max(lane - 1, 0)], enext = slots[min(lane + 1, BR_WAVE - 1)];
    const int st = e >> BR_IDX_BITS;
    // requests of equal length are contiguous; within such a run the order of admission is by
    // position ascending, the reverse of the order they were gathered in
    const bool gs = valid && (lane == 0 || (eprev >> BR_IDX_BITS) != st);
    const bool ge = valid && (lane == nA - 1 || (enext >> BR_IDX_BITS) != st);
    const unsigned long long sm = br_ballot(gs), em = br_ballot(ge);
    int T = BR_WAVE, ga = BR_WAVE;
    if (valid) {
      ga = 63 - (int)__builtin_clzll(sm & ((2ull << lane) - 1ull));
      const int gb = lane + (int)__builtin_ctzll(em >> lane);
      T = ga + gb - lane;
    }
    if (smax >= 0) K = min(K, (int)__builtin_popcountll(br_ballot(T < K && st <= smax)));  // lengths rise with T
    br_wave_sync();  // every lane holds its entry; the array is refilled in admission order below
    if (K <= 0) return 0;
    // a run cut by the edge of the 64 gathered requests has an unknown order here
    if (n_alive > BR_WAVE && __builtin_amdgcn_readlane(ga, BR_WAVE - 1) < K) return 0;
    if (T < K) slots[T] = e;
    br_wave_sync();
    const bool cand = member && rank >= r0 && rank < r0 + K;
    const int mine = slots[cand ? rank - r0 : 0];
    const int s_k = mine >> BR_IDX_BITS, pos_k = mine & IDX_MASK;
    if (cand) adm[pos_k] = (lane << 16) | nn;
    Lh[0] += cand ? s_k : 0;
    nn += cand ? 1 : 0;
    cap -= cand ? 1 : 0;
    // taken: every alive request shorter than the K-th one, and of its length those up to it
    const int tK = (int)__builtin_ctzll(br_ballot(T == K - 1));
    const int eK = __builtin_amdgcn_readlane(e, tK);
    const int vK = eK >> BR_IDX_BITS, pK = eK & IDX_MASK;
    const int pend = __builtin_amdgcn_readlane(e, __builtin_amdgcn_readlane(ga, tK)) & IDX_MASK;
#pragma unroll
    for (int j = 0; j < E; ++j) {
      const int pp = j * BR_WAVE + lane;
      const bool taken = pp > pend || (sv[j] == vK && pp <= pK);
      alive &= ~((taken ? 1u : 0u) << j);
    }
    Mh[0] = workers_max(Lh[0]);
    S_tot -= K;
    n_alive -= K;
    admitted += K;
    tail_dirty = true;
    br_wave_sync();
    return K;
  };

  if (run) {
    const int bound = qn + G + 1;  // every iteration admits a request or sets a worker aside

    // ---- Stage 1: greedy fill while free capacity is abundant
    for (int it = 0; it < bound; ++it) {
      if (!(S_tot > p.S_greedy && n_alive > 0)) break;
      const int capmax = cap_max();
      if (capmax <= 0) break;
      // the level: workers sharing the largest free-slot count, ranked by (load, index); each is
      // picked exactly once, in rank order, before any other worker can reach this free-slot count
      const bool member = cap == capmax;
      const int wkey = member ? (int)(((unsigned)Lh[0] << 6) | (unsigned)lane) : INT32_MAX;
      const int rank = rank_of(wkey);
      const int level = __builtin_popcountll(br_ballot(member));
      const int kmaxp = min(level, min(S_tot - p.S_greedy, n_alive));
      // the first kmaxp alive requests, by rank, through LDS
      advance_head();
      {
        int base = 0;
#pragma unroll
        for (int j = 0; j < E; ++j) {
          if (j >= jhead && base < kmaxp && j * BR_WAVE < qn) {
            const bool al = (alive >> j) & 1u;
            const unsigned long long bal = br_ballot(al);
            const int ar = base + br_rank_below(bal);
            if (al && ar < kmaxp) slots[ar] = (sv[j] << BR_IDX_BITS) | (j * BR_WAVE + lane);
            base += __builtin_popcountll(bal);
          }
        }
      }
      br_wave_sync();
      const bool cand = member && rank < kmaxp;
      const int mine = cand ? slots[rank] : 0;
      const int s_k = mine >> BR_IDX_BITS, pos_k = mine & IDX_MASK;
      int lim = lane_minm();
      if (p.W > 0) lim = min(lim, p.W - Lh[0]);
      const int k0 = workers_min((cand && s_k > lim) ? rank : kmaxp);
      if (k0 > 0) {  // ranks 0..k0-1 are in the safe regime: k-th lightest worker takes k-th largest request
        const bool take = cand && rank < k0;
        if (take) adm[pos_k] = (lane << 16) | nn;
#pragma unroll
        for (int h = 0; h < NH; ++h) Lh[h] += take ? s_k : 0;
        nn += take ? 1 : 0;
        cap -= take ? 1 : 0;
        // last position taken (everything alive before it went too): the request of the worker ranked k0 - 1
        const int pstar = __builtin_amdgcn_readlane(pos_k, (int)__builtin_ctzll(br_ballot(cand && rank == k0 - 1)));
        const int jf = pstar >> 6, lf = pstar & 63;
        const unsigned clear = ((1u << jf) - 1u) | ((lane <= lf) ? (1u << jf) : 0u);
        alive &= ~clear;
        tail_dirty |= pstar >= tail_pos;
        S_tot -= k0;
        n_alive -= k0;
        admitted += k0;
        stage1 += k0;
      }
      br_wave_sync();
      // the rest of the level one worker at a time, in rank order
      for (int r = k0; r < level; ++r) {
        if (!(S_tot > p.S_greedy && n_alive > 0)) break;
        const int g = (int)__builtin_ctzll(br_ballot(member && rank == r));
        int Lg[NH], mg[BR_HP + 1];
        margins_of(g, Lg, mg);
        const int room = p.W > 0 ? p.W - Lg[0] : INT32_MAX;
        int pos = 0, swin = 0;
        bool found = false;
        if constexpr (!BRH) {
          if (tail_rule) {
            ensure_tail();
            if (tail_s >= mg[0]) {
              // No waiting request is shorter than this worker's margin.  It takes the shortest one and
              // the envelope becomes its new load; the next worker of the level is at least as loaded,
              // so its margin is at most that length and the same holds for it: the rest of the level
              // takes the waiting requests in order of (length, arrival), one each.
              const int K = min(level - r, min(S_tot - p.S_greedy, n_alive));
              if (tail_bulk_ok && K >= 3) {
                const int done = tail_bulk(member, rank, r, K, -1);
                if (done > 0) {
                  stage1 += done;
                  r += done - 1;
                  continue;
                }
              }
              if (tail_s > room) {  // under the watermark even the shortest request is too long: nothing is admissible
                drop_worker(g, capmax);
                continue;
              }
              pick_tail(pos, swin);
              found = true;
            }
          }
        }
        if (!found && !pick_single(mg, room, pos, swin)) {
          drop_worker(g, capmax);
          continue;
        }
        bind(pos, g, __builtin_amdgcn_readlane(nn, g));
        add_load(g, Lg, swin, 1);
        ++stage1;
      }
    }

    // ---- Stage 2: refined allocation over the workers that still have free slots
    // lane-constant pieces of the subset enumeration: lane l of pass c stands for mask c*64 + l
    int lbit[6];
#pragma unroll
    for (int b = 0; b < 6; ++b) lbit[b] = (lane >> b) & 1;
    const int lpop = __builtin_popcount(lane);
    for (int it = 0; it < bound; ++it) {
      if (n_alive <= 0) break;
      const int capmax = cap_max();
      if (capmax <= 0) break;
      // priority (free slots, horizon-min margin), lowest index on ties
      const int kc = (cap == capmax) ? (int)(((unsigned)lane_minm() << 6) | (unsigned)(63 - lane)) : -1;
      const int g = 63 - (workers_max(kc) & 63);
      ++pops;
      int Lg[NH], mg[BR_HP + 1];
      margins_of(g, Lg, mg);
      const int room = p.W > 0 ? p.W - Lg[0] : INT32_MAX;

      // candidate window: the first min(R_max, |R_wait|) alive requests in sorted order, ranked
      // by ballots and passed through LDS so that every lane holds all of them
      const int w = min(p.R_max, n_alive);
      advance_head();
      int s_last = 0;  // smallest length in the window (its w-th entry)
      {
        int base = 0;
#pragma unroll
        for (int j = 0; j < E; ++j) {
          if (j >= jhead && base < w && j * BR_WAVE < qn) {
            const bool al = (alive >> j) & 1u;
            const unsigned long long bal = br_ballot(al);
            const int ar = base + br_rank_below(bal);
            if (al && ar < w) win[ar] = (sv[j] << BR_IDX_BITS) | (j * BR_WAVE + lane);
            const unsigned long long hit = br_ballot(al && ar == w - 1);
            if (hit != 0ull) s_last = __builtin_amdgcn_readlane(sv[j], (int)__builtin_ctzll(hit));
            base += __builtin_popcountll(bal);
          }
        }
      }
      // BR-0: every subset of the window sums to at least its smallest entry, and eq. (br0-Fscore)
      // falls beyond the margin; if that entry alone scores <= 0 (then it exceeds the margin), no
      // subset scores above 0 and the round goes to the starvation guard without the enumeration.
      // BR-H: eq. (brh-Fscore) is concave in Delta with F(0) = 0, so F(Delta) <= F(s) Delta / s for every
      // Delta >= s.  The scores are compared as computed in fp32: each of the at most H + 5 roundings of
      // one evaluation is relative 2^-24 on terms bounded by (alpha D + beta D) Delta, under 8e-7 of that in
      // all.  If the smallest entry's computed score is below -8e-6 (alpha D + beta D) s, its exact score
      // is below -7e-6 of it, every subset's exact score below the same fraction of its own Delta, and
      // every subset's computed score below zero: the guard is certain here too.
      bool guard_sure = false;
      if constexpr (!BRH) {
        guard_sure = br_score0(G, mg[0], s_last) <= 0;
      } else {
        float Dsum = 0.0f;
#pragma unroll
        for (int h = 0; h <= BR_HP; ++h) Dsum += p.d[h];
        guard_sure = br_scoreh(p, mg, s_last) <= -8e-6f * (p.aD + p.beta * Dsum) * (float)s_last;
      }
      if constexpr (!BRH) {
        if (guard_sure && tail_rule && tail_bulk_ok) {
          ensure_tail();
          if (tail_s >= mg[0]) {
            // This worker takes the shortest waiting request through the guard and the envelope becomes
            // its new load.  The next pop goes to the next lightest worker that still has this many free
            // slots; its margin is at most the length just admitted.  While the lengths admitted stay
            // at or below (G-1)/G of the window's smallest entry, the window is untouched, that entry
            // still scores <= 0 for every such margin (so the guard fires again) and no waiting request
            // is below the margin: the pops of this free-slot count follow in one step.
            const bool member = cap == capmax;
            const int level = __builtin_popcountll(br_ballot(member));
            const int K = min(level, n_alive - w);
            if (K >= 3) {
              const int wkey = member ? (int)(((unsigned)Lh[0] << 6) | (unsigned)lane) : INT32_MAX;
              const int rank = rank_of(wkey);
              const int done = tail_bulk(member, rank, 0, K, (G - 1) * s_last / G);
              if (done > 0) {
                pops += done - 1;
                guard += done;
                continue;
              }
            }
          }
        }
      }
      int wv[8], ws[8];
      int bestmask = 0, bestkey = BR_KEY_NONE;
      if constexpr (BIGR) {
        // Windows of up to 16 requests: lane l keeps the lower six mask bits, the upper bits c run over
        // 2^(w-6) passes whose partial sums come from a table built here, 64 entries at a time.  A lane sees
        // its masks in ascending order and keeps the first best; across lanes the lowest mask of the best
        // score wins.
#pragma unroll
        for (int b = 0; b < 8; ++b) wv[b] = 0, ws[b] = 0;
        if (!guard_sure && w > 16) {
          // windows of 17..32 requests: reachable sums instead of masks (br_subset_dp.h)
          br_wave_sync();
          unsigned dm = 0u;
          int *share = nullptr;
          if constexpr (!COOP) share = shared ? svc : nullptr;
          br_subset_dp<BRH>(p, mg, win, w, min(capmax, p.R_max), room, lane, dprows,
                            p.dp + (size_t)inst * br_dp_cluster_words(min(p.B, p.R_max)), dm, bestkey, share);
          bestmask = (int)dm;
        } else if (!guard_sure) {
          br_wave_sync();
          const int nhi = w > 6 ? 1 << (w - 6) : 1;
          for (int c0 = 0; c0 < nhi; c0 += BR_WAVE) {
            const int c = c0 + lane;
            int sum = 0;
            for (int b = 6; b < w; ++b) sum += ((c >> (b - 6)) & 1) * (win[b] >> BR_IDX_BITS);
            if (c < nhi) hitab[c] = sum;
          }
          br_wave_sync();
          const int kmax = min(capmax, p.R_max);
          int bk, bm;
          bool shared_scan = false;
          if constexpr (!COOP) shared_scan = shared && nhi >= 16;  // (a few trips are not worth two barriers)
          if (shared_scan) {
#pragma unroll
            for (int h = 0; h <= BR_HP; ++h) svc[1 + h] = mg[h];
            svc[2 + BR_HP] = room, svc[3 + BR_HP] = w, svc[4 + BR_HP] = kmax;
            svc[0] = 1;
            __syncthreads();
            br_bigr_scan<BRH>(p, mg, win, hitab, w, kmax, room, lane, 0, 4, bk, bm);
          } else {
            br_bigr_scan<BRH>(p, mg, win, hitab, w, kmax, room, lane, 0, 1, bk, bm);
          }
          bestkey = br_wave_max(bk);
          bestmask = bestkey == BR_KEY_NONE ? 0 : br_wave_min(bk == bestkey ? bm : INT32_MAX);
          if (shared_scan) {  // the best of the four shares: lowest mask among equal scores
            __syncthreads();
            int mbest = bestkey == BR_KEY_NONE ? INT32_MAX : bestmask;
#pragma unroll
            for (int u = 1; u < 4; ++u) {
              const int ku = svc[16 + 2 * u], mu = svc[17 + 2 * u];
              if (ku > bestkey || (ku == bestkey && mu < mbest)) bestkey = ku, mbest = mu;
            }
            bestmask = bestkey == BR_KEY_NONE ? 0 : mbest;
          }
        }
      } else if (!guard_sure) {
        br_wave_sync();
        {
          const int4 lo = *reinterpret_cast<const int4 *>(win);
          const int4 hi = *reinterpret_cast<const int4 *>(win + 4);
          wv[0] = lo.x, wv[1] = lo.y, wv[2] = lo.z, wv[3] = lo.w;
          wv[4] = hi.x, wv[5] = hi.y, wv[6] = hi.z, wv[7] = hi.w;
        }
#pragma unroll
        for (int b = 0; b < 8; ++b) ws[b] = b < w ? (wv[b] >> BR_IDX_BITS) : 0;

        // exhaustive subset search, one subset mask per lane (ascending masks, strict improvement)
        const int kmax = min(capmax, p.R_max);
        const int nmask = 1 << w;
        for (int c = 0; c * BR_WAVE < nmask; ++c) {
          int delta = (c & 1) * ws[6] + (c >> 1) * ws[7];
#pragma unroll
          for (int b = 0; b < 6; ++b)
            if (b < w) delta += lbit[b] * ws[b];
          const int mask = c * BR_WAVE + lane;
          const bool ok = mask != 0 && mask < nmask && lpop + __builtin_popcount(c) <= kmax && delta <= room;
          if constexpr (!BRH) {
            const int F = delta - (int)((unsigned)(max(delta - mg[0], 0) & 0x7ffff) * (unsigned)(G & 0x7f));
            const unsigned key = ok ? (((unsigned)(F + BIAS2) << 6) | (unsigned)(63 - lane)) : 0u;
            const unsigned km = br_wave_umax(key);
            if (km != 0u) {
              const int Fm = (int)(km >> 6) - BIAS2;
              if (Fm > bestkey) {
                bestkey = Fm;
                bestmask = c * BR_WAVE + (63 - (int)(km & 63u));
              }
            }
          } else {
            int key = br_score_key<BRH>(p, mg, delta);
            key = ok ? key : BR_KEY_NONE;
            const int km = br_wave_max(key);
            if (km > bestkey) {
              bestkey = km;
              bestmask = c * BR_WAVE + (int)__builtin_ctzll(br_ballot(key == km));
            }
          }
        }
      } else {
#pragma unroll
        for (int b = 0; b < 8; ++b) wv[b] = 0, ws[b] = 0;
      }

      if (bestmask == 0 || bestkey <= 0) {  // starvation guard: the single best request anyway
        ++guard;
        int pos = 0, swin = 0;
        bool found = false;
        if constexpr (!BRH) {
          if (tail_rule) {
            ensure_tail();
            if (tail_s >= mg[0]) {
              if (tail_s > room) {  // nothing is admissible under the watermark
                drop_worker(g, capmax);
                continue;
              }
              pick_tail(pos, swin);
              found = true;
            }
          }
        }
        if (!found && !pick_single(mg, room, pos, swin)) {
          drop_worker(g, capmax);
          continue;
        }
        bind(pos, g, __builtin_amdgcn_readlane(nn, g));
        add_load(g, Lg, swin, 1);
      } else {
        // lane b binds window entry b if chosen; slots follow the order of the window
        const int slot = __builtin_amdgcn_readlane(nn, g);
        int delta = 0;
        if constexpr (BIGR) {
          const unsigned um = (unsigned)bestmask;
          if (lane < 32 && ((um >> lane) & 1u))
            adm[win[lane] & IDX_MASK] = (g << 16) | (slot + __builtin_popcount(um & ((1u << (lane & 31)) - 1u)));
          for (int b = 0; b < w; ++b)
            if ((um >> b) & 1u) {
              const int e = win[b];
              const int pb = e & IDX_MASK;
              alive = (lane == (pb & 63)) ? (alive & ~(1u << (pb >> 6))) : alive;
              tail_dirty |= pb == tail_pos;
              delta += e >> BR_IDX_BITS;
            }
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
              tail_dirty |= pb == tail_pos;
              delta += ws[b];
            }
        }
        add_load(g, Lg, br_uniform(delta), __builtin_popcount(bestmask));
      }
    }
  }
  br_wave_sync();

  BrRoundCounts rc;
  rc.admitted = admitted;
  rc.stage1 = stage1;
  rc.pops = pops;
  rc.guard = guard;
  rc.wdrop = wdrop;
  rc.I_before = I_before;
  if constexpr (BIGR && !COOP) {
    if (shared) {
      svc[0] = 0;  // the round is over: the waves that served the scans leave
      __syncthreads();
    }
  }
  if constexpr (COOP) {
    svc[0] = 0;  // the round is over: the waves that served the searches go on to the epilogue
    __syncthreads();
    int Lw = Lh[0];
    br_assign_epilogue_block4(inst, lane, 0, q0, qn, cnt, skey, adm, who, slots, Lw, nn, rc, c0, ADV);
    if constexpr (ADV) br_advance_cluster<4, BRH>(inst, lane, Lw, nn, 0, min((G + 3) >> 2, G));
  } else {
    bool done = false;
    if constexpr (!BRH && !BIGR && !ADV && E <= 8) {
      if (split != nullptr) {
        br_assign_epilogue_split<E>(inst, lane, q0, qn, cnt, skey, adm, who, Lh[0], nn, nn_start, rc, split);
        done = true;
      }
    }
    if (!done) {
      br_assign_epilogue<E>(inst, lane, q0, qn, cnt, skey, adm, who, Lh[0], nn, rc, c0);
      if constexpr (ADV) br_advance_cluster<(BRH ? 4 : 8), BRH>(inst, lane, Lh[0], nn);  // BR-H units carry the estimator code: fewer unrolled
    }
  }
}

// every wave of the block owns one cluster and its own slice of LDS; waves never meet at a barrier
// The BR-H kernel for queues of up to 512 needs one register more than lets four waves share a SIMD
// (a batch of 4096 clusters is four waves per SIMD): it is asked to fit.
// BIGR: candidate windows of 9..16 requests (R_max > 8); a separate instantiation so that the kernels for
// the deployed window sizes keep their registers and code size.
template <int E, bool BRH, bool ADV, bool BIGR = false>
// `share` (BIGR, queues of up to 1024): one cluster per block, its four waves share the subset scans
__global__ __launch_bounds__(256, (BRH && E == 8 && !BIGR) ? 4 : 1) void br_k_assign(BrParams p, BrArr a, BrOut o, int share) {
  extern __shared__ int lds_all[];
  constexpr int WORDS = 3 * E * BR_WAVE + BR_WAVE + (BIGR ? 32 + 1024 : 8) + (E == 32 ? 96 : 0);  // skey, adm, who, slots, win (+ table, + mailbox) per wave
  const int w = threadIdx.x >> 6;
  if constexpr (E == 32)  // one cluster per block, four waves for the sort
    br_assign_body<E, BRH, ADV, true, BIGR>(p, a, o, lds_all, (int)blockIdx.x, w);
  else if (BIGR && share)
    br_assign_body<E, BRH, ADV, false, BIGR>(p, a, o, lds_all, (int)blockIdx.x, w, nullptr, nullptr, true);
  else
    br_assign_body<E, BRH, ADV, false, BIGR>(p, a, o, lds_all + w * WORDS, (int)(blockIdx.x * (blockDim.x >> 6)) + w);
}

template <int E, bool BRH, bool BIGR = false>
static void br_launch_assign_one(const BrParams &p, const BrArr &a, const BrOut &o, hipStream_t st) {
  // several single-wave clusters share a block so that the chip's per-CU block slots do not cap residency
  const bool dp = BIGR && p.R_max > 16;   // windows beyond 16 requests: one cluster per block, with LDS for the bit rows
  const int wpb = (E <= 8 && !dp) ? 4 : 1;  // clusters per block
  const size_t lds = ((size_t)wpb * (3 * E * BR_WAVE + BR_WAVE + (BIGR ? 32 + 1024 : 8) + (E == 32 ? 96 : 0)) +
                      (dp ? BR_DP_LDS_WORDS : 0)) * sizeof(int);
  const dim3 grid((unsigned)((p.N + wpb - 1) / wpb)), block(E == 32 ? 4 * BR_WAVE : BR_WAVE * wpb);
  if constexpr (BIGR) {  // no fused decode steps for these: the caller launches the decode kernel
    // windows of 9..16 requests on a batch that leaves room on the chip (registers allow about 4 / 3 / 2 waves per
    // SIMD for queues of up to 256 / 512 / 1024, one less for BR-H): a block of four waves per cluster, the scans shared
    const long long room = 1024ll * max(1, (E == 4 ? 4 : E == 8 ? 3 : 2) - (BRH ? 1 : 0));
    if (E <= 16 && (long long)p.N * 4 <= room) {
      const size_t lds1 = ((size_t)3 * E * BR_WAVE + BR_WAVE + 32 + 1024 + 32 + (dp ? BR_DP_LDS_WORDS : 0)) * sizeof(int);
      hipLaunchKernelGGL((br_k_assign<E, BRH, false, true>), dim3((unsigned)p.N), dim3(4 * BR_WAVE), lds1, st, p, a, o, 1);
    } else {
      hipLaunchKernelGGL((br_k_assign<E, BRH, false, true>), grid, block, lds, st, p, a, o, 0);
    }
  } else {
    if (p.adv_t > 0)
      hipLaunchKernelGGL((br_k_assign<E, BRH, true>), grid, block, lds, st, p, a, o, 0);
    else
      hipLaunchKernelGGL((br_k_assign<E, BRH, false>), grid, block, lds, st, p, a, o, 0);
  }
}

template <bool BRH, bool BIGR = false>
static void br_launch_assign_sized(const BrParams &p, const BrArr &a, const BrOut &o, hipStream_t st) {
  if (p.Q <= 256)
    br_launch_assign_one<4, BRH, BIGR>(p, a, o, st);
  else if (p.Q <= 512)
    br_launch_assign_one<8, BRH, BIGR>(p, a, o, st);
  else if (p.Q <= 1024)
    br_launch_assign_one<16, BRH, BIGR>(p, a, o, st);
  else
    br_launch_assign_one<32, BRH, BIGR>(p, a, o, st);
}
