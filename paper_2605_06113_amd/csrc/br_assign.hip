// Sequential two-stage assignment of one scheduling round (Appendix, Alg. BR-0 / Alg. BR-H),
// one wavefront per cluster.
//
// The round is a dependent chain: every admission changes L_g, possibly the envelope M and
// with it every margin.  The chain therefore stays inside one wave, with no barrier and no
// LDS round trip on its critical path:
//   - lane g holds worker g's state (free slots, projected loads L_g(k+h), request count);
//   - the waiting set, ordered by prefill length (largest first, arrival order among equals),
//     lives in registers, E requests per lane, sorted position = j*64 + lane;
//   - "pick a worker" and "pick a request" are DPP reductions on int32 keys; Stage-2 subsets
//     are enumerated one subset mask per lane.
// Ties: Stage 1 worker (most free slots, then lightest, then lowest index); Stage 2 worker
// (most free slots, then largest horizon-min margin, then lowest index); equal request scores
// resolve to the lowest sorted position; equal subset scores to the lowest mask.
#include "br_device.h"
#include "br_launch.h"

#define BR_STAT(o, inst, k) (o).stats[(int64_t)(inst) * 16 + (k)]

template <int E, bool BRH>
__global__ __launch_bounds__(64) void br_k_assign(BrParams p, BrArr a, BrOut o) {
  extern __shared__ int lds[];
  constexpr int NP = E * BR_WAVE;
  constexpr int NH = BRH ? BR_HP + 1 : 1;
  constexpr int IDX_MASK = (1 << BR_IDX_BITS) - 1;
  int *skey = lds;          // [NP] sort buffer, then the sorted keys (s << 11 | 2047 - arrival position)
  int *adm = lds + NP;      // [NP] by sorted position: worker << 16 | slot, or -1
  int *who = lds + 2 * NP;  // [NP] by arrival position: worker, or -1

  const int inst = blockIdx.x, lane = br_lane();
  const int G = p.G;
  const int q0 = br_uniform(min(max(p.qlen[inst], 0), p.Q));
  int cnt = a.count ? a.count[inst] : 0;
  cnt = br_uniform(min(max(cnt, 0), a.arr_cap));
  const int qn = q0 + min(cnt, p.Q - q0);
  const int64_t qrow = (int64_t)inst * p.Q, arow = (int64_t)inst * a.arr_cap;

  // ---- worker state, one worker per lane
  const bool act = lane < G;
  const int64_t wrow = (int64_t)inst * G + lane;
  int nn = act ? min(max(p.n[wrow], 0), p.B) : p.B;
  int cap = p.B - nn;
  int Lh[NH], Mh[NH];
  if constexpr (BRH) {
#pragma unroll
    for (int h = 0; h < NH; ++h) Lh[h] = act ? p.Lh[wrow * (p.H + 1) + min(h, p.H)] : BR_LOW;
  } else {
    Lh[0] = act ? p.L[wrow] : BR_LOW;
  }
#pragma unroll
  for (int h = 0; h < NH; ++h) Mh[h] = br_wave_max(Lh[h]);
  int S_tot = br_wave_sum(cap);

  long long sumL = 0;
  for (int g = 0; g < G; ++g) sumL += __builtin_amdgcn_readlane(Lh[0], g);
  const long long I_before = (long long)G * Mh[0] - sumL;

  // ---- waiting set: keys into LDS, bitonic sort (descending), back into registers
#pragma unroll
  for (int j = 0; j < E; ++j) {
    const int i = j * BR_WAVE + lane;
    int key = 0;
    if (i < qn) {
      int s = i < q0 ? p.qs[qrow + i] : a.s[arow + (i - q0)];
      s = min(max(s, 1), BR_MAX_S_DEV);
      key = (s << BR_IDX_BITS) | (IDX_MASK - i);
    }
    skey[i] = key;
    adm[i] = -1;
    who[i] = -1;
  }
  __syncthreads();
  const bool run = S_tot > 0 && qn > 0;
  if (run) {
    int N2 = BR_WAVE;
    while (N2 < qn) N2 <<= 1;
    for (int k = 2; k <= N2; k <<= 1)
      for (int jj = k >> 1; jj > 0; jj >>= 1) {
        for (int t = lane; t < (N2 >> 1); t += BR_WAVE) {
          const int i = ((t & ~(jj - 1)) << 1) | (t & (jj - 1));
          const int l = i | jj;
          const int x = skey[i], y = skey[l];
          const bool desc = (i & k) == 0;
          if ((x < y) == desc) {
            skey[i] = y;
            skey[l] = x;
          }
        }
        __syncthreads();
      }
  }
  int sv[E];
  unsigned alive = 0;
#pragma unroll
  for (int j = 0; j < E; ++j) {
    const int pos = j * BR_WAVE + lane;
    sv[j] = skey[pos] >> BR_IDX_BITS;
    if (pos < qn) alive |= 1u << j;
  }

  int n_alive = qn;
  int stage1 = 0, pops = 0, guard = 0, wdrop = 0, admitted = 0;

  // argmax_i F_g({i}) over alive, admissible requests (lowest sorted position on ties)
  auto pick_single = [&](const int(&mg)[BR_HP + 1], int room, int &pos, int &swin) -> int {
    int bk = BR_KEY_NONE, bp = INT32_MAX, bs = 0;
#pragma unroll
    for (int j = 0; j < E; ++j) {
      if (j * BR_WAVE < qn) {
        const int s = sv[j];
        const bool ok = ((alive >> j) & 1u) && s <= room;
        int key = br_score_key<BRH>(p, mg, s);
        key = ok ? key : BR_KEY_NONE;
        if (key > bk) {
          bk = key;
          bp = j * BR_WAVE + lane;
          bs = s;
        }
      }
    }
    const int km = br_wave_max(bk);
    if (km == BR_KEY_NONE) return BR_KEY_NONE;
    pos = br_wave_min(bk == km ? bp : INT32_MAX);
    swin = __builtin_amdgcn_readlane(bs, pos & 63);
    return km;
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

  // sticky binding of the request at sorted position pos to worker g
  auto bind = [&](int pos, int g, int slot) {
    if (lane == 0) adm[pos] = (g << 16) | slot;
    const int jw = pos >> 6, lw = pos & 63;
    alive = (lane == lw) ? (alive & ~(1u << jw)) : alive;
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

  if (run) {
    const int bound = qn + G + 1;  // every iteration admits a request or sets a worker aside

    // ---- Stage 1: greedy fill while free capacity is abundant
    for (int it = 0; it < bound; ++it) {
      if (!(S_tot > p.S_greedy && n_alive > 0)) break;
      const int capmax = br_wave_max(cap);
      if (capmax <= 0) break;
      const int Lc = (cap == capmax) ? Lh[0] : INT32_MAX;
      const int Lmin = br_wave_min(Lc);
      const int g = (int)__builtin_ctzll(br_ballot(Lc == Lmin));
      int Lg[NH], mg[BR_HP + 1];
      margins_of(g, Lg, mg);
      const int room = p.W > 0 ? p.W - Lg[0] : INT32_MAX;
      int pos = 0, swin = 0;
      const int key = pick_single(mg, room, pos, swin);
      if (key == BR_KEY_NONE) {
        drop_worker(g, capmax);
        continue;
      }
      bind(pos, g, __builtin_amdgcn_readlane(nn, g));
      add_load(g, Lg, swin, 1);
      ++stage1;
    }

    // ---- Stage 2: refined allocation over the workers that still have free slots
    for (int it = 0; it < bound; ++it) {
      if (n_alive <= 0) break;
      const int capmax = br_wave_max(cap);
      if (capmax <= 0) break;
      int minm = INT32_MAX;
#pragma unroll
      for (int h = 0; h < NH; ++h) minm = min(minm, max(Mh[h] - Lh[h], 0));
      const int kc = (cap == capmax) ? minm : -1;
      const int kmaxm = br_wave_max(kc);
      const int g = (int)__builtin_ctzll(br_ballot(kc == kmaxm));
      ++pops;
      int Lg[NH], mg[BR_HP + 1];
      margins_of(g, Lg, mg);
      const int room = p.W > 0 ? p.W - Lg[0] : INT32_MAX;

      // candidate window: the first min(R_max, |R_wait|) alive requests in sorted order
      const int w = min(p.R_max, n_alive);
      int wpos[8], ws[8];
      unsigned wk = alive;
#pragma unroll
      for (int b = 0; b < 8; ++b) {
        wpos[b] = 0;
        ws[b] = 0;
        if (b < w) {
          const int lp = wk ? (__builtin_ctz(wk) * BR_WAVE + lane) : INT32_MAX;
          const int pb = min(br_wave_min(lp), NP - 1);
          wk = (lane == (pb & 63)) ? (wk & ~(1u << (pb >> 6))) : wk;
          wpos[b] = pb;
          ws[b] = skey[pb] >> BR_IDX_BITS;
        }
      }

      // exhaustive subset search, one subset mask per lane (ascending masks, strict improvement)
      const int kmax = min(capmax, p.R_max);
      const int nmask = 1 << w;
      int bestmask = 0, bestkey = BR_KEY_NONE;
      for (int c = 0; c * BR_WAVE + 1 < nmask; ++c) {
        const int mask = c * BR_WAVE + lane + 1;
        int delta = 0;
#pragma unroll
        for (int b = 0; b < 8; ++b) delta += ((mask >> b) & 1) ? ws[b] : 0;
        const bool ok = mask < nmask && __builtin_popcount(mask) <= kmax && delta <= room;
        int key = br_score_key<BRH>(p, mg, delta);
        key = ok ? key : BR_KEY_NONE;
        const int km = br_wave_max(key);
        if (km > bestkey) {
          bestkey = km;
          bestmask = c * BR_WAVE + (int)__builtin_ctzll(br_ballot(key == km)) + 1;
        }
      }

      if (bestmask == 0 || bestkey <= 0) {  // starvation guard: the single best request anyway
        ++guard;
        int pos = 0, swin = 0;
        const int key = pick_single(mg, room, pos, swin);
        if (key == BR_KEY_NONE) {
          drop_worker(g, capmax);
          continue;
        }
        bind(pos, g, __builtin_amdgcn_readlane(nn, g));
        add_load(g, Lg, swin, 1);
      } else {
        int slot = __builtin_amdgcn_readlane(nn, g);
        int delta = 0, k = 0;
#pragma unroll
        for (int b = 0; b < 8; ++b)
          if ((bestmask >> b) & 1) {
            bind(wpos[b], g, slot + k);
            delta += ws[b];
            ++k;
          }
        add_load(g, Lg, delta, k);
      }
    }
  }
  __syncthreads();

  // ---- commit the admitted requests into their workers' dense lists
  if (admitted > 0) {
#pragma unroll
    for (int j = 0; j < E; ++j) {
      const int pos = j * BR_WAVE + lane;
      if (pos < qn) {
        const int ad = adm[pos];
        if (ad >= 0) {
          const int key = skey[pos];
          const int idx = IDX_MASK - (key & IDX_MASK);
          const int g = ad >> 16, slot = ad & 0xffff;
          if (g < G && slot < p.B && idx < qn) {
            const int64_t row = ((int64_t)inst * G + g) * p.Bs + slot;
            const bool old = idx < q0;
            p.kv[row] = key >> BR_IDX_BITS;
            p.rem[row] = old ? p.qo[qrow + idx] : max(a.o[arow + (idx - q0)], 1);
            for (int q = 0; q < p.P; ++q)
              p.pred[row * p.P + q] = old ? p.qpred[(qrow + idx) * p.P + q] : a.pred[(arow + (idx - q0)) * p.P + q];
            who[idx] = g;
          }
        }
      }
    }
  }
  __syncthreads();

  // ---- outputs in arrival order; the queue keeps the deferred requests, order preserved
  int kept = 0;
#pragma unroll
  for (int j = 0; j < E; ++j) {
    const int i = j * BR_WAVE + lane;
    if (j * BR_WAVE < p.Q) {
      const bool in = i < qn;
      const int wg = in ? who[i] : -1;
      const bool old = i < q0;
      int id = -1;
      if (in) id = old ? p.qid[qrow + i] : (a.id ? a.id[arow + (i - q0)] : i - q0);
      if (i < p.Q) {
        if (o.assign) o.assign[qrow + i] = wg;
        if (o.assign_id) o.assign_id[qrow + i] = id;
      }
      const bool keep = in && wg < 0;
      const unsigned long long bal = br_ballot(keep);
      const int ni = kept + br_rank_below(bal);
      if (keep && (ni != i || !old)) {
        int s = old ? p.qs[qrow + i] : a.s[arow + (i - q0)];
        s = min(max(s, 1), BR_MAX_S_DEV);
        const int oo = old ? p.qo[qrow + i] : max(a.o[arow + (i - q0)], 1);
        float pr[BR_HP];
        for (int q = 0; q < p.P; ++q) pr[q] = old ? p.qpred[(qrow + i) * p.P + q] : a.pred[(arow + (i - q0)) * p.P + q];
        p.qs[qrow + ni] = s;
        p.qo[qrow + ni] = oo;
        p.qid[qrow + ni] = id;
        for (int q = 0; q < p.P; ++q) p.qpred[(qrow + ni) * p.P + q] = pr[q];
      }
      kept += __builtin_popcountll(bal);
    }
  }

  // ---- state and statistics
  if (act) {
    p.L[wrow] = Lh[0];
    p.n[wrow] = nn;
  }
  const int Lact = Lh[0];
  const int Lmax = br_wave_max(Lact);
  const int Lmin = br_wave_min(act ? Lact : INT32_MAX);
  const int over = __builtin_popcountll(br_ballot(act && p.C > 0 && Lact > p.C));
  sumL = 0;
  for (int g = 0; g < G; ++g) sumL += __builtin_amdgcn_readlane(Lact, g);
  if (lane == 0) {
    p.qlen[inst] = kept;
    if (o.stats) {
      BR_STAT(o, inst, 0) = admitted;
      BR_STAT(o, inst, 1) = kept;
      BR_STAT(o, inst, 2) = cnt - (qn - q0);
      BR_STAT(o, inst, 3) = stage1;
      BR_STAT(o, inst, 4) = pops;
      BR_STAT(o, inst, 5) = guard;
      BR_STAT(o, inst, 6) = over;
      BR_STAT(o, inst, 7) = I_before;
      BR_STAT(o, inst, 8) = (long long)G * Lmax - sumL;
      BR_STAT(o, inst, 9) = (long long)Lmax - Lmin;
      BR_STAT(o, inst, 10) = qn;
      BR_STAT(o, inst, 11) = wdrop;
      for (int k = 12; k < 16; ++k) BR_STAT(o, inst, k) = 0;
    }
  }
}

template <bool BRH>
static void launch_e(const BrParams &p, const BrArr &a, const BrOut &o, hipStream_t st) {
  const dim3 grid((unsigned)p.N), block(BR_WAVE);
  if (p.Q <= 256)
    hipLaunchKernelGGL((br_k_assign<4, BRH>), grid, block, 3 * 4 * 64 * 4, st, p, a, o);
  else if (p.Q <= 512)
    hipLaunchKernelGGL((br_k_assign<8, BRH>), grid, block, 3 * 8 * 64 * 4, st, p, a, o);
  else if (p.Q <= 1024)
    hipLaunchKernelGGL((br_k_assign<16, BRH>), grid, block, 3 * 16 * 64 * 4, st, p, a, o);
  else
    hipLaunchKernelGGL((br_k_assign<32, BRH>), grid, block, 3 * 32 * 64 * 4, st, p, a, o);
}

void br_launch_assign(const BrParams &p, const BrArr &a, const BrOut &o, hipStream_t st) {
  if (p.H > 0)
    launch_e<true>(p, a, o, st);
  else
    launch_e<false>(p, a, o, st);
}
