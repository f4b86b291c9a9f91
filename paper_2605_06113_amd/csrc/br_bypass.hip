// Pool-bypass dispatch for BR-0 (Appendix "Pool-bypass deployment path for BR-0"): arrivals are
// placed one at a time, in order, on argmax_g F_g(s) over the workers that can take them, against
// the virtual load (every placement counts at once).  One wavefront per cluster, lane g = worker g;
// each placement is one packed-key DPP reduction ((F + bias) << 6 | 63 - g: best score, lowest
// index on ties).  Decisions are collected in LDS and written out lane-parallel afterwards.
#include "br_device.h"
#include "br_launch.h"

#define BR_STATB(o, inst, k) (o).stats[(int64_t)(inst) * 16 + (k)]

__global__ __launch_bounds__(256) void br_k_bypass(BrParams p, BrArr a, BrOut o, int cap_pad) {
  extern __shared__ int lds_all[];
  constexpr int BIAS1 = 1 << 21;  // single request: score in (-2^21, 2^15]
  const int inst = (int)(blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6));
  if (inst >= p.N) return;
  int *ss = lds_all + (threadIdx.x >> 6) * (2 * cap_pad);  // [cap_pad] prefill lengths of the arrivals
  int *dec = ss + cap_pad;                                  // [cap_pad] worker << 16 | slot, or -1
  const int lane = br_lane();
  const int G = p.G;
  int cnt = a.count[inst];
  cnt = br_uniform(min(max(cnt, 0), a.arr_cap));
  const int64_t arow = (int64_t)inst * a.arr_cap, qrow = (int64_t)inst * p.Q;

  const bool act = lane < G;
  const int64_t wrow = (int64_t)inst * G + lane;
  int nn = act ? min(max(p.n[wrow], 0), p.B) : p.B;
  int cap = p.B - nn;
  int L = act ? p.L[wrow] : BR_LOW;
  int M = br_wave_max(L);
  auto sum_loads = [&]() -> long long {
    const int L0 = act ? L : 0;
    return ((long long)br_wave_sum(L0 >> 16) << 16) + br_wave_sum(L0 & 0xffff);
  };
  const long long I_before = o.stats ? (long long)G * M - sum_loads() : 0;

  for (int i = lane; i < cnt; i += BR_WAVE) ss[i] = min(max(a.s[arow + i], 1), BR_MAX_S_DEV);
  br_wave_sync();

  int admitted = 0;
  for (int i = 0; i < cnt; ++i) {
    const int s = br_uniform(ss[i]);
    const int m = M - L;
    const int F = s - (int)((unsigned)(max(s - m, 0) & 0xffff) * (unsigned)(G & 0x7f));
    const bool ok = act && cap > 0 && (p.W <= 0 || L + s <= p.W);
    const unsigned key = ok ? (((unsigned)(F + BIAS1) << 6) | (unsigned)(63 - lane)) : 0u;
    const unsigned km = br_wave_umax(key);
    int d = -1;
    if (km != 0u) {
      const int g = 63 - (int)(km & 63u);
      const int Lg = __builtin_amdgcn_readlane(L, g);
      d = (g << 16) | __builtin_amdgcn_readlane(nn, g);
      L += (lane == g) ? s : 0;
      cap -= (lane == g) ? 1 : 0;
      nn += (lane == g) ? 1 : 0;
      M = max(M, Lg + s);
      ++admitted;
    }
    if (lane == 0) dec[i] = d;
  }
  br_wave_sync();

  // commit: placed arrivals go to their workers' lists; the rest join the waiting queue in order
  int q = br_uniform(min(max(p.qlen[inst], 0), p.Q));
  int dropped = 0;
  for (int c = 0; c < cnt; c += BR_WAVE) {
    const int i = c + lane;
    const bool in = i < cnt;
    const int d = in ? dec[i] : 0;
    const bool placed = in && d >= 0;
    const bool left = in && d < 0;
    const unsigned long long bal = br_ballot(left);
    const int qpos = q + br_rank_below(bal);
    int res = -2;
    if (placed) {
      const int g = d >> 16, slot = d & 0xffff;
      if (g < G && slot < p.B) {
        const int64_t row = ((int64_t)inst * G + g) * p.Bs + slot;
        p.kv[row] = ss[i];
        p.rem[row] = max(a.o[arow + i], 1);
      }
      res = g;
    } else if (left && qpos < p.Q) {
      p.qs[qrow + qpos] = ss[i];
      p.qo[qrow + qpos] = max(a.o[arow + i], 1);
      p.qid[qrow + qpos] = a.id ? a.id[arow + i] : i;
      res = -1;
    }
    if (in && o.assign) o.assign[arow + i] = res;
    const int nleft = __builtin_popcountll(bal);
    const int fit = min(nleft, p.Q - q);
    dropped += nleft - fit;
    q += fit;
  }

  if (act) {
    p.L[wrow] = L;
    p.n[wrow] = nn;
  }
  const int Lmax = br_wave_max(L);
  const int Lmin = br_wave_min(act ? L : INT32_MAX);
  const int over = __builtin_popcountll(br_ballot(act && p.C > 0 && L > p.C));
  const int wide = __builtin_popcountll(br_ballot(act && L >= (1 << 25)));
  const long long sumL = o.stats ? sum_loads() : 0;
  if (lane == 0) {
    p.qlen[inst] = q;
    if (o.stats) {
      for (int k = 0; k < 16; ++k) BR_STATB(o, inst, k) = 0;
      BR_STATB(o, inst, 0) = admitted;
      BR_STATB(o, inst, 1) = q;
      BR_STATB(o, inst, 2) = dropped;
      BR_STATB(o, inst, 6) = over;
      BR_STATB(o, inst, 7) = I_before;
      BR_STATB(o, inst, 8) = (long long)G * Lmax - sumL;
      BR_STATB(o, inst, 9) = (long long)Lmax - Lmin;
      BR_STATB(o, inst, 10) = cnt;
      BR_STATB(o, inst, 12) = wide;
    }
  }
}

void br_launch_bypass(const BrParams &p, const BrArr &a, const BrOut &o, hipStream_t st) {
  const int cap_pad = (a.arr_cap + 63) & ~63;
  const int wpb = cap_pad <= 512 ? 4 : 1;
  const size_t lds = (size_t)wpb * 2 * cap_pad * sizeof(int);
  hipLaunchKernelGGL(br_k_bypass, dim3((unsigned)((p.N + wpb - 1) / wpb)), dim3(BR_WAVE * wpb), lds, st, p, a, o, cap_pad);
}
