// Comparison policies of Sec. 6.1 ("Baselines": Random, Round-Robin, Power-of-Two-Choices,
// Join-Shortest-Queue) on the library's cluster state, so that a replay can put BalanceRoute's imbalance
// next to theirs.  Workload-unaware dispatch: waiting requests leave the queue in arrival order and each goes
// to a worker chosen among those with a free slot, without looking at any length; dispatch stops when every
// worker is full.  One wavefront per cluster, lane g = worker g; a pick is a ballot, a bit scan and (JSQ, P2C)
// one comparison of request counts.  Decisions are collected in LDS and committed lane-parallel afterwards; the
// dispatched requests are a prefix of the queue, so the rest simply moves up.
//
// Random draws are counter-based (one SplitMix64 output per dispatched request: the published output function
// applied to (seed ^ cluster << 32) + (draw + 1) * 0x9E3779B97F4A7C15); a 32-bit half u picks index
// (u * E) >> 32 among E candidates in ascending worker order.  Round-robin cursor and draw count persist per
// cluster in the workspace.
#include "br_device.h"
#include "br_launch.h"

#define BR_STATP(o, inst, k) (o).stats[(int64_t)(inst) * 16 + (k)]

__device__ __forceinline__ unsigned long long br_splitmix64(unsigned long long key, unsigned c) {
  unsigned long long z = key + ((unsigned long long)c + 1ull) * 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// index of the k-th set bit of m (k below its population count)
__device__ __forceinline__ int br_kth_bit(unsigned long long m, int k) {
  for (int i = 0; i < k; ++i) m &= m - 1ull;
  return (int)__builtin_ctzll(m);
}

__global__ __launch_bounds__(256) void br_k_baseline(BrParams p, BrArr a, BrOut o, int *pol, int policy,
                                                    unsigned long long seed, int q_pad) {
  extern __shared__ int lds_all[];
  const int inst = (int)(blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6));
  if (inst >= p.N) return;
  int *ss = lds_all + (threadIdx.x >> 6) * (2 * q_pad);  // [q_pad] prefill lengths by queue position
  int *dec = ss + q_pad;                                 // [q_pad] worker << 16 | slot of the dispatched prefix
  const int lane = br_lane();
  const int G = p.G;
  const int q0 = br_uniform(min(max(p.qlen[inst], 0), p.Q));
  int cnt = a.count ? a.count[inst] : 0;
  cnt = br_uniform(min(max(cnt, 0), a.arr_cap));
  const int qn = q0 + min(cnt, p.Q - q0);
  const int64_t qrow = (int64_t)inst * p.Q, arow = (int64_t)inst * a.arr_cap;

  const bool act = lane < G;
  const int64_t wrow = (int64_t)inst * G + lane;
  int nn = act ? min(max(p.n[wrow], 0), p.B) : p.B;
  int cap = p.B - nn;
  int L = act ? p.L[wrow] : BR_LOW;
  auto sum_loads = [&]() -> long long {
    const int L0 = act ? L : 0;
    return ((long long)br_wave_sum(L0 >> 16) << 16) + br_wave_sum(L0 & 0xffff);
  };
  const long long I_before = o.stats ? (long long)G * br_wave_max(L) - sum_loads() : 0;

  for (int i = lane; i < qn; i += BR_WAVE) {
    const int s = i < q0 ? p.qs[qrow + i] : a.s[arow + (i - q0)];
    ss[i] = min(max(s, 1), BR_MAX_S_DEV);
  }
  br_wave_sync();

  const int K = min(br_wave_sum(cap), qn);  // while a slot is free somewhere every request finds a worker
  int cursor = br_uniform(pol[2 * inst]);
  unsigned draws = (unsigned)br_uniform(pol[2 * inst + 1]);
  cursor = min(max(cursor, 0), G - 1);
  const unsigned long long key = seed ^ ((unsigned long long)(unsigned)inst << 32);
  for (int i = 0; i < K; ++i) {
    const unsigned long long elig = br_ballot(cap > 0);
    int g;
    if (policy == 1) {  // round-robin: first eligible worker at or after the cursor, cyclically
      const unsigned long long hi = elig & ~((1ull << cursor) - 1ull);
      g = (int)__builtin_ctzll(hi != 0ull ? hi : elig);
      cursor = g + 1 == G ? 0 : g + 1;
    } else if (policy == 3) {  // fewest requests, lowest index on equal counts
      g = br_wave_min(cap > 0 ? ((nn << 6) | lane) : INT32_MAX) & 63;
    } else {
      const int E = (int)__builtin_popcountll(elig);
      const unsigned long long z = br_splitmix64(key, draws);
      ++draws;
      const unsigned lo = (unsigned)z, hi = (unsigned)(z >> 32);
      g = br_kth_bit(elig, (int)(((unsigned long long)lo * (unsigned long long)E) >> 32));
      if (policy == 2 && E > 1) {  // second candidate among the others; it wins only with strictly fewer requests
        const int gb = br_kth_bit(elig & ~(1ull << g), (int)(((unsigned long long)hi * (unsigned long long)(E - 1)) >> 32));
        if (__builtin_amdgcn_readlane(nn, gb) < __builtin_amdgcn_readlane(nn, g)) g = gb;
      }
    }
    const int s = br_uniform(ss[i]);
    if (lane == 0) dec[i] = (g << 16) | __builtin_amdgcn_readlane(nn, g);
    L += (lane == g) ? s : 0;
    nn += (lane == g) ? 1 : 0;
    cap -= (lane == g) ? 1 : 0;
  }
  br_wave_sync();

  // commit: the dispatched prefix goes to the workers' lists; outputs by queue position
  for (int c = 0; c < p.Q; c += BR_WAVE) {
    const int i = c + lane;
    if (i < p.Q) {
      int wg = -1, id = -1;
      if (i < qn) id = i < q0 ? p.qid[qrow + i] : (a.id ? a.id[arow + (i - q0)] : i - q0);
      if (i < K) {
        const int d = dec[i];
        const int g = d >> 16, slot = d & 0xffff;
        wg = g;
        if (g < G && slot < p.B) {
          const int64_t row = ((int64_t)inst * G + g) * p.Bs + slot;
          p.kv[row] = ss[i];
          p.rem[row] = i < q0 ? p.qo[qrow + i] : max(a.o[arow + (i - q0)], 1);
        }
      }
      if (o.assign) o.assign[qrow + i] = wg;
      if (o.assign_id) o.assign_id[qrow + i] = id;
    }
  }
  // the rest of the queue moves up by K, 64 entries at a time in ascending order: a chunk is read whole before
  // it is written, and it is written only to positions at or below the ones it read
  for (int c = K; c < qn; c += BR_WAVE) {
    const int i = c + lane;
    int so = 1, oo = 1, io = -1;
    if (i < qn) {
      so = ss[i];
      oo = i < q0 ? p.qo[qrow + i] : max(a.o[arow + (i - q0)], 1);
      io = i < q0 ? p.qid[qrow + i] : (a.id ? a.id[arow + (i - q0)] : i - q0);
    }
    br_wave_sync();
    if (i < qn && (K > 0 || i >= q0)) {
      p.qs[qrow + i - K] = so;
      p.qo[qrow + i - K] = oo;
      p.qid[qrow + i - K] = io;
    }
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
    p.qlen[inst] = qn - K;
    pol[2 * inst] = cursor;
    pol[2 * inst + 1] = (int)draws;
    if (o.stats) {
      for (int k = 0; k < 16; ++k) BR_STATP(o, inst, k) = 0;
      BR_STATP(o, inst, 0) = K;
      BR_STATP(o, inst, 1) = qn - K;
      BR_STATP(o, inst, 2) = cnt - (qn - q0);
      BR_STATP(o, inst, 6) = over;
      BR_STATP(o, inst, 7) = I_before;
      BR_STATP(o, inst, 8) = (long long)G * Lmax - sumL;
      BR_STATP(o, inst, 9) = (long long)Lmax - Lmin;
      BR_STATP(o, inst, 10) = qn;
      BR_STATP(o, inst, 12) = wide;
    }
  }
}

void br_launch_baseline(const BrParams &p, const BrArr &a, const BrOut &o, int *pol, int policy, unsigned long long seed,
                        hipStream_t st) {
  const int q_pad = (p.Q + 63) & ~63;
  const int wpb = q_pad <= 512 ? 4 : 1;
  const size_t lds = (size_t)wpb * 2 * q_pad * sizeof(int);
  hipLaunchKernelGGL(br_k_baseline, dim3((unsigned)((p.N + wpb - 1) / wpb)), dim3(BR_WAVE * wpb), lds, st, p, a, o, pol,
                     policy, seed, q_pad);
}
