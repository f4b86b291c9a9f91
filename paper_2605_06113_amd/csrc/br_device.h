// Device-side helpers shared by the gfx950 kernels: wave64 reductions on DPP,
// the two score functions, and the parameter block the host passes by value.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#define BR_WAVE 64
#define BR_HP 8          // horizon offsets h = 0..BR_HP are carried in registers
#define BR_HL 128        // longest horizon; beyond BR_HP the per-offset state lives in LDS (the *_long kernels)
#define BR_HS(H) (((H) + 4) & ~3)  // H + 1 offsets padded to whole 16-byte groups
#define BR_LOW (-(1 << 30))  // "minus infinity" load of a lane that holds no worker
#define BR_MAX_G_DEV 64
#define BR_MAX_S_DEV 32768
#define BR_IDX_BITS 11   // queue positions fit 11 bits (max_wait <= 2048)
#define BR_SCORE_TILES_MAX_N 16    // up to this many clusters, long queues are scored a wave per (request tile, worker group)
#define BR_SCORE_WAVE_MIN_N 2048  // from this many clusters on (two waves per SIMD), short queues are scored one wave per cluster

struct BrParams {
  int32_t N, G, B, Bs, Q, H, P, R_max, S_greedy, W, C, pred_mode;
  int32_t Pq, hist_n, refresh, adv_t;  // queue prediction width; survival-estimator history size and period;
                                       // decode steps the assignment kernel applies after the round (0: none)
  float aD, beta, gate;
  float d[BR_HP + 1];  // discount vector, zero beyond H
  // workspace arrays
  int32_t *L, *n, *kv, *rem;
  float *pred;
  int32_t *qlen, *qs, *qo, *qid;
  float *qpred;
  int32_t *Lh, *Mh, *mh, *minm;
  const int32_t *hist;      // sorted output lengths (pred_mode 2)
  const long long *hsum;    // their prefix sums
  const float *dl;          // H > BR_HP: discount vector d[0..H], then zeros up to BR_HS(H) entries
  int32_t *dp;              // R_max > 16: per-cluster areas for the subset search by reachable sums (br_subset_dp.h)
};

struct BrArr {  // arrivals of one round (device pointers, may be null when none)
  const int32_t *count, *s, *o, *id;
  const float *pred;
  int32_t arr_cap;
};

struct BrOut {
  int32_t *assign, *assign_id;
  long long *stats;
  void *F;
  int32_t *best_g, *best_i;
};

// ---------------------------------------------------------------- wave64 reductions
// Cross-lane data movement on the DPP path (no LDS traffic).  Every lane of the wave
// must be active when these run.  Pattern: swap within pairs, within quads, mirror
// within half rows, mirror within rows of 16, then carry lane 15 of each row into the
// next row and lane 31 into the upper half; lane 63 ends up with the full reduction.

// `old` is what a lane keeps when its source is masked off; passing the identity of the
// combining operation lets the compiler fold the move into the ALU instruction itself.
template <int CTRL, int ROW_MASK = 0xF, bool BOUND = false>
__device__ __forceinline__ int br_dpp(int old, int src) {
  return __builtin_amdgcn_update_dpp(old, src, CTRL, ROW_MASK, 0xF, BOUND);
}

__device__ __forceinline__ int br_wave_max(int x) {
  x = max(x, br_dpp<0xB1, 0xF, true>(0, x));          // quad_perm [1,0,3,2]
  x = max(x, br_dpp<0x4E, 0xF, true>(0, x));          // quad_perm [2,3,0,1]
  x = max(x, br_dpp<0x141, 0xF, true>(0, x));         // row_half_mirror
  x = max(x, br_dpp<0x140, 0xF, true>(0, x));         // row_mirror
  x = max(x, br_dpp<0x142, 0xA>(INT32_MIN, x));       // row_bcast:15 into rows 1 and 3
  x = max(x, br_dpp<0x143, 0xC>(INT32_MIN, x));       // row_bcast:31 into rows 2 and 3
  return __builtin_amdgcn_readlane(x, 63);
}

__device__ __forceinline__ unsigned br_wave_umax(unsigned x) {
  x = max(x, (unsigned)br_dpp<0xB1, 0xF, true>(0, (int)x));
  x = max(x, (unsigned)br_dpp<0x4E, 0xF, true>(0, (int)x));
  x = max(x, (unsigned)br_dpp<0x141, 0xF, true>(0, (int)x));
  x = max(x, (unsigned)br_dpp<0x140, 0xF, true>(0, (int)x));
  x = max(x, (unsigned)br_dpp<0x142, 0xA>(0, (int)x));
  x = max(x, (unsigned)br_dpp<0x143, 0xC>(0, (int)x));
  return (unsigned)__builtin_amdgcn_readlane((int)x, 63);
}

__device__ __forceinline__ int br_wave_min(int x) {
  x = min(x, br_dpp<0xB1, 0xF, true>(0, x));
  x = min(x, br_dpp<0x4E, 0xF, true>(0, x));
  x = min(x, br_dpp<0x141, 0xF, true>(0, x));
  x = min(x, br_dpp<0x140, 0xF, true>(0, x));
  x = min(x, br_dpp<0x142, 0xA>(INT32_MAX, x));
  x = min(x, br_dpp<0x143, 0xC>(INT32_MAX, x));
  return __builtin_amdgcn_readlane(x, 63);
}

__device__ __forceinline__ int br_wave_sum(int x) {
  x += br_dpp<0xB1, 0xF, true>(0, x);
  x += br_dpp<0x4E, 0xF, true>(0, x);
  x += br_dpp<0x141, 0xF, true>(0, x);
  x += br_dpp<0x140, 0xF, true>(0, x);
  x += br_dpp<0x142, 0xA>(0, x);
  x += br_dpp<0x143, 0xC>(0, x);
  return __builtin_amdgcn_readlane(x, 63);
}

// Reductions over one row of 16 lanes (lanes 0..15 of the wave: clusters of up to 16 workers keep all of them
// there): four butterfly steps leave the row's result in each of its lanes, two DPP steps and a bubble less than
// the wave-wide forms.  What the other rows hold does not matter.
__device__ __forceinline__ int br_row0_max(int x) {
  x = max(x, br_dpp<0xB1, 0xF, true>(0, x));
  x = max(x, br_dpp<0x4E, 0xF, true>(0, x));
  x = max(x, br_dpp<0x141, 0xF, true>(0, x));
  x = max(x, br_dpp<0x140, 0xF, true>(0, x));
  return __builtin_amdgcn_readlane(x, 0);
}

__device__ __forceinline__ int br_row0_min(int x) {
  x = min(x, br_dpp<0xB1, 0xF, true>(0, x));
  x = min(x, br_dpp<0x4E, 0xF, true>(0, x));
  x = min(x, br_dpp<0x141, 0xF, true>(0, x));
  x = min(x, br_dpp<0x140, 0xF, true>(0, x));
  return __builtin_amdgcn_readlane(x, 0);
}

// Number of lanes of the caller's row of 16 whose key is below the caller's (keys of one row pairwise
// distinct, or INT32_MAX for lanes that do not take part): fifteen row rotations, no scalar traffic.
template <int K>
__device__ __forceinline__ int br_row_rank_step(int key, int acc) {
  const int other = __builtin_amdgcn_update_dpp(0, key, 0x120 + K, 0xF, 0xF, false);  // row_ror:K
  acc += other < key ? 1 : 0;
  if constexpr (K < 15) return br_row_rank_step<K + 1>(key, acc);
  else return acc;
}

__device__ __forceinline__ int br_row_rank(int key) { return br_row_rank_step<1>(key, 0); }

__device__ __forceinline__ unsigned long long br_ballot(bool p) { return __builtin_amdgcn_ballot_w64(p); }

__device__ __forceinline__ int br_lane() { return (int)(threadIdx.x & 63u); }

// number of set bits of m in lanes below the caller
__device__ __forceinline__ int br_rank_below(unsigned long long m) {
  return (int)__builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
}

// Orders this wave's LDS traffic (the waves of a block that each work alone never need more).
__device__ __forceinline__ void br_wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

__device__ __forceinline__ int br_uniform(int x) { return __builtin_amdgcn_readfirstlane(x); }

// ---------------------------------------------------------------- scores
// Scores are compared as int32 keys: the BR-0 score is its own key; an fp32 horizon score
// maps to the integer with the same ordering, so that one set of integer reductions serves
// both.  key <= 0 exactly when the score is <= 0.

__device__ __forceinline__ int br_ord(float f) {
  int b = __float_as_int(f);
  return b ^ ((b >> 31) & 0x7fffffff);
}

__device__ __forceinline__ float br_unord(int k) { return __int_as_float(k ^ ((k >> 31) & 0x7fffffff)); }

#define BR_KEY_NONE INT32_MIN

// Sec. 3.1, eq. (br0-Fscore): F = Delta - G (Delta - m)_+ in exact int32.  Delta <= 16 * 32768 and
// G <= 64, so both factors fit 24 bits; the masks say so and the product becomes one full-rate
// 24-bit multiply-add instead of a quarter-rate 32-bit multiply.
__device__ __forceinline__ int br_score0(int G, int m, int delta) {
  return delta + (max(delta - m, 0) & 0x7fffff) * -(G & 0x7f);
}

// Sec. 4.1, eq. (brh-Fscore): alpha (1^T d) Delta - beta ((Delta 1 - m)_+)^T d, fp32: the penalty is
// accumulated from h = 0 upwards with one fused multiply-add per offset (pen = fma(d_h, (Delta - m_h)_+, pen),
// a single rounding), the two products and the difference of the last line are rounded one by one.  Offsets beyond H carry
// a zero discount and add exactly +0.
__device__ __forceinline__ float br_scoreh(const BrParams &p, const int (&m)[BR_HP + 1], int delta) {
  // The excess (Delta - m)_+ is formed in fp32, one operation less per offset than in integers and the same
  // value: Delta <= 2^19 is an exact float; a margin below Delta is one too and so is the difference; a margin
  // at or above Delta stays so after rounding and the term is zero either way.  (The conversions of the margins
  // do not depend on Delta: where one worker is scored against many requests they are done once.)
  const float fd = (float)delta;
  float pen = 0.0f;
#pragma unroll
  for (int h = 0; h <= BR_HP / 2; ++h)
    pen = __fmaf_rn(p.d[h], fmaxf(__fsub_rn(fd, (float)m[h]), 0.0f), pen);
  if (p.H > BR_HP / 2) {  // short horizons: the remaining terms are +0 and leave the sum as it is
#pragma unroll
    for (int h = BR_HP / 2 + 1; h <= BR_HP; ++h)
      pen = __fmaf_rn(p.d[h], fmaxf(__fsub_rn(fd, (float)m[h]), 0.0f), pen);
  }
  return __fsub_rn(__fmul_rn(p.aD, fd), __fmul_rn(p.beta, pen));
}

// The same score for horizons beyond BR_HP, NV subset sums at a time: margins `m` (as floats) and
// discounts `d` are read from LDS, four offsets per load, the same address on every lane; entries from
// H + 1 up to the padded length carry a zero discount and add exactly +0.  Rounding and order as above.
// The excess (Delta - m)_+ is formed in fp32: Delta <= 2^18 and, wherever Delta > m, m are exact floats and
// so is their difference; where Delta <= m the rounded margin is still >= Delta and the term is zero, as in
// integers.
// The group after the one in use is requested first, so that the LDS latency hides under the arithmetic:
// both arrays are read up to four entries beyond HS (the callers keep other LDS data there; the values are
// not used).
template <int NV>
__device__ __forceinline__ void br_scoreh_long(float aD, float beta, const float *m, const float *d, int HS,
                                               const int (&delta)[NV], float (&F)[NV]) {
  float pen[NV], fd[NV];
#pragma unroll
  for (int v = 0; v < NV; ++v) pen[v] = 0.0f, fd[v] = (float)delta[v];
  float4 m4 = *reinterpret_cast<const float4 *>(m);
  float4 d4 = *reinterpret_cast<const float4 *>(d);
  for (int h = 0; h < HS; h += 4) {
    const float4 mn = *reinterpret_cast<const float4 *>(m + h + 4);
    const float4 dn = *reinterpret_cast<const float4 *>(d + h + 4);
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      pen[v] = __fmaf_rn(d4.x, fmaxf(__fsub_rn(fd[v], m4.x), 0.0f), pen[v]);
      pen[v] = __fmaf_rn(d4.y, fmaxf(__fsub_rn(fd[v], m4.y), 0.0f), pen[v]);
      pen[v] = __fmaf_rn(d4.z, fmaxf(__fsub_rn(fd[v], m4.z), 0.0f), pen[v]);
      pen[v] = __fmaf_rn(d4.w, fmaxf(__fsub_rn(fd[v], m4.w), 0.0f), pen[v]);
    }
    m4 = mn;
    d4 = dn;
  }
#pragma unroll
  for (int v = 0; v < NV; ++v) F[v] = __fsub_rn(__fmul_rn(aD, fd[v]), __fmul_rn(beta, pen[v]));
}

// Offsets whose margin lies below `maxdelta`, as one bit per offset (lanes stand for offsets; every lane of
// the wave must call).  For every Delta <= maxdelta the other offsets contribute exactly +0 to the penalty
// sum, which leaves it as it is: br_scoreh_long_act walks only the four-offset groups that hold a set bit,
// in ascending order, and returns the same bits as the full walk.
__device__ __forceinline__ void br_long_active(const float *m, int HS, int lane, int maxdelta,
                                               unsigned long long (&act)[3]) {
  const float fmx = (float)maxdelta;
#pragma unroll
  for (int c = 0; c < 3; ++c) {
    const int h = c * BR_WAVE + lane;
    act[c] = br_ballot(h < HS && m[h] < fmx);
  }
}

template <int NV>
__device__ __forceinline__ void br_scoreh_long_act(float aD, float beta, const float *m, const float *d,
                                                   const unsigned long long (&act)[3], const int (&delta)[NV],
                                                   float (&F)[NV]) {
  float pen[NV], fd[NV];
#pragma unroll
  for (int v = 0; v < NV; ++v) pen[v] = 0.0f, fd[v] = (float)delta[v];
#pragma unroll
  for (int c = 0; c < 3; ++c) {
    unsigned long long g = act[c];
    g = (g | (g >> 1) | (g >> 2) | (g >> 3)) & 0x1111111111111111ull;  // bit 4k: group k of this chunk is needed
    while (g != 0ull) {
      const int h = c * BR_WAVE + (int)__builtin_ctzll(g);
      g &= g - 1ull;
      const float4 m4 = *reinterpret_cast<const float4 *>(m + h);
      const float4 d4 = *reinterpret_cast<const float4 *>(d + h);
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        pen[v] = __fmaf_rn(d4.x, fmaxf(__fsub_rn(fd[v], m4.x), 0.0f), pen[v]);
        pen[v] = __fmaf_rn(d4.y, fmaxf(__fsub_rn(fd[v], m4.y), 0.0f), pen[v]);
        pen[v] = __fmaf_rn(d4.z, fmaxf(__fsub_rn(fd[v], m4.z), 0.0f), pen[v]);
        pen[v] = __fmaf_rn(d4.w, fmaxf(__fsub_rn(fd[v], m4.w), 0.0f), pen[v]);
      }
    }
  }
#pragma unroll
  for (int v = 0; v < NV; ++v) F[v] = __fsub_rn(__fmul_rn(aD, fd[v]), __fmul_rn(beta, pen[v]));
}

// One stage of a walk over four-offset groups: the next NB groups named by the set bits of `u` (taken off it),
// their margins and discounts requested from LDS.  has[i]: the stage's i-th group exists.
template <int NB>
struct BrGroupStage {
  int k[NB];
  bool has[NB];
  float4 m4[NB], d4[NB];
  __device__ __forceinline__ void fetch(unsigned long long &u, const float *m, const float *d) {
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      has[i] = u != 0ull;
      k[i] = has[i] ? (int)__builtin_ctzll(u) : 0;
      u &= u - 1ull;  // (u == 0 stays 0)
      if (has[i]) {
        m4[i] = *reinterpret_cast<const float4 *>(m + 4 * k[i]);
        d4[i] = *reinterpret_cast<const float4 *>(d + 4 * k[i]);
      }
    }
  }
};

// the four offsets of a group added to one penalty sum in ascending order
__device__ __forceinline__ void br_group_add(const float4 &m4, const float4 &d4, float fd, float &pen) {
  pen = __fmaf_rn(d4.x, fmaxf(__fsub_rn(fd, m4.x), 0.0f), pen);
  pen = __fmaf_rn(d4.y, fmaxf(__fsub_rn(fd, m4.y), 0.0f), pen);
  pen = __fmaf_rn(d4.z, fmaxf(__fsub_rn(fd, m4.z), 0.0f), pen);
  pen = __fmaf_rn(d4.w, fmaxf(__fsub_rn(fd, m4.w), 0.0f), pen);
}

// the same into four separate partial sums
__device__ __forceinline__ void br_group_add4(const float4 &m4, const float4 &d4, float fd, float4 &pen) {
  pen.x = __fmaf_rn(d4.x, fmaxf(__fsub_rn(fd, m4.x), 0.0f), pen.x);
  pen.y = __fmaf_rn(d4.y, fmaxf(__fsub_rn(fd, m4.y), 0.0f), pen.y);
  pen.z = __fmaf_rn(d4.z, fmaxf(__fsub_rn(fd, m4.z), 0.0f), pen.z);
  pen.w = __fmaf_rn(d4.w, fmaxf(__fsub_rn(fd, m4.w), 0.0f), pen.w);
}

// The same walk with a bound per value: value v is known not to exceed bound[v] (0: the value is not in
// question and its result is not used).  A four-offset group whose margins all lie at or above bound[v] adds
// exact zeros to value v's penalty and is skipped for that value alone, so a lane that holds a long and a short
// request pays the long walk only for the long one.  Lanes stand for groups when the masks are formed (one
// 16-byte read each); the groups in use are then walked in ascending order with margins and discounts
// broadcast, reads requested ahead of their use.  Every lane of the wave must call with
// the same bounds.  Results are the bits of the full walk.
template <int NV>
__device__ __forceinline__ void br_scoreh_long_sel(float aD, float beta, const float *m, const float *d, int HS, int lane,
                                                   const int (&bound)[NV], const int (&delta)[NV], float (&F)[NV]) {
  float pen[NV], fd[NV];
  unsigned long long gm[NV], u = 0ull;
  {
    const bool in = lane * 4 < HS;  // HS <= 132: at most 33 groups
    const float4 q = *reinterpret_cast<const float4 *>(m + (in ? lane * 4 : 0));
    const float lo = fminf(fminf(q.x, q.y), fminf(q.z, q.w));
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      pen[v] = 0.0f, fd[v] = (float)delta[v];
      gm[v] = br_ballot(in && lo < (float)bound[v]);
      u |= gm[v];
    }
  }
  if constexpr (NV >= 4) {
    // four values per lane: the arithmetic of a group covers the LDS latency of the next one
    if (u != 0ull) {
      int k = (int)__builtin_ctzll(u);
      u &= u - 1ull;
      float4 m4 = *reinterpret_cast<const float4 *>(m + 4 * k);
      float4 d4 = *reinterpret_cast<const float4 *>(d + 4 * k);
      for (;;) {
        const bool more = u != 0ull;
        const int kn = more ? (int)__builtin_ctzll(u) : k;
        u &= u - 1ull;  // (u == 0 stays 0)
        const float4 mn = *reinterpret_cast<const float4 *>(m + 4 * kn);
        const float4 dn = *reinterpret_cast<const float4 *>(d + 4 * kn);
#pragma unroll
        for (int v = 0; v < NV; ++v) {
          if ((gm[v] >> k) & 1ull) {
            pen[v] = __fmaf_rn(d4.x, fmaxf(__fsub_rn(fd[v], m4.x), 0.0f), pen[v]);
            pen[v] = __fmaf_rn(d4.y, fmaxf(__fsub_rn(fd[v], m4.y), 0.0f), pen[v]);
            pen[v] = __fmaf_rn(d4.z, fmaxf(__fsub_rn(fd[v], m4.z), 0.0f), pen[v]);
            pen[v] = __fmaf_rn(d4.w, fmaxf(__fsub_rn(fd[v], m4.w), 0.0f), pen[v]);
          }
        }
        if (!more) break;
        k = kn;
        m4 = mn;
        d4 = dn;
      }
    }
  } else {
    // one or two values per lane: too little arithmetic per group to cover a read, so the groups are taken in
    // stages of NB, two stages in turn: the reads of one are requested before the other is used
    constexpr int NB = 2 / NV;
    BrGroupStage<NB> A, B;
    A.fetch(u, m, d);
    for (;;) {
      if (!A.has[0]) break;
      B.fetch(u, m, d);
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        if (A.has[i]) {
#pragma unroll
          for (int v = 0; v < NV; ++v)
            if (NV == 1 || ((gm[v] >> A.k[i]) & 1ull)) br_group_add(A.m4[i], A.d4[i], fd[v], pen[v]);
        }
      }
      if (!B.has[0]) break;
      A.fetch(u, m, d);
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        if (B.has[i]) {
#pragma unroll
          for (int v = 0; v < NV; ++v)
            if (NV == 1 || ((gm[v] >> B.k[i]) & 1ull)) br_group_add(B.m4[i], B.d4[i], fd[v], pen[v]);
        }
      }
    }
  }
#pragma unroll
  for (int v = 0; v < NV; ++v) F[v] = __fsub_rn(__fmul_rn(aD, fd[v]), __fmul_rn(beta, pen[v]));
}

// An approximation of the same score for one value per lane, for use where only a bound on the error matters:
// the four offsets of a group feed four separate partial sums (independent chains instead of one), which are
// added at the end, and the groups may be shared out: br_long_penalty_part returns the penalty over the groups
// named in `share` (bit k: offsets 4k .. 4k+3), br_scoreh_long_from the score from the sum of such parts.  Not
// the bits of br_scoreh_long: with the parts of up to four sharers it has at most H / 4 + 12 roundings, each
// relative 2^-24 on terms bounded by (alpha D + beta D) Delta, so it lies within the same distance of the exact
// score as the ordered walk does.  `bound`: no value exceeds it (groups whose margins all lie at or above it are
// skipped).
__device__ __forceinline__ float br_long_penalty_part(const float *m, const float *d, int HS, int lane, int bound, int delta,
                                                      unsigned long long share) {
  const float fd = (float)delta;
  float4 pen = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
  unsigned long long u;
  {
    const bool in = lane * 4 < HS;
    const float4 q = *reinterpret_cast<const float4 *>(m + (in ? lane * 4 : 0));
    u = br_ballot(in && fminf(fminf(q.x, q.y), fminf(q.z, q.w)) < (float)bound) & share;
  }
  BrGroupStage<2> A, B;
  A.fetch(u, m, d);
  for (;;) {
    if (!A.has[0]) break;
    B.fetch(u, m, d);
#pragma unroll
    for (int i = 0; i < 2; ++i)
      if (A.has[i]) br_group_add4(A.m4[i], A.d4[i], fd, pen);
    if (!B.has[0]) break;
    A.fetch(u, m, d);
#pragma unroll
    for (int i = 0; i < 2; ++i)
      if (B.has[i]) br_group_add4(B.m4[i], B.d4[i], fd, pen);
  }
  return __fadd_rn(__fadd_rn(pen.x, pen.y), __fadd_rn(pen.z, pen.w));
}

__device__ __forceinline__ float br_scoreh_long_from(float aD, float beta, int delta, float penalty) {
  return __fsub_rn(__fmul_rn(aD, (float)delta), __fmul_rn(beta, penalty));
}

template <bool BRH>
__device__ __forceinline__ int br_score_key(const BrParams &p, const int (&m)[BR_HP + 1], int delta) {
  if constexpr (BRH) return br_ord(br_scoreh(p, m, delta));
  else return br_score0(p.G, m[0], delta);
}

// Empirical-survival estimate of the in-window contribution at age a (Appendix "Estimator
// realizations"): with F the empirical CDF of the sorted output-length history,
// p_fin = (F(a+H) - F(a)) / (1 - F(a)), mu_rem = mean of (o_j - a) over a < o_j <= a+H, then the
// composite, gate, floor and clip of eq. (composite) / "Refresh logic".  All counts and the sum of
// remainders are exact integers below 2^24, so each quotient is one correctly rounded division.
// Number of history entries <= x[q], NQ look-ups side by side: a fixed number of halving steps (set by the
// history length alone, the same on every lane), each with the NQ loads in flight together, so that the
// latency of a step is paid once for all of them.
template <int NQ>
__device__ __forceinline__ void br_hist_ranks(const BrParams &p, const int (&x)[NQ], int (&r)[NQ]) {
  const int n = p.hist_n;
  int step = 1;
  while (step <= n) step <<= 1;
#pragma unroll
  for (int q = 0; q < NQ; ++q) r[q] = 0;
  for (step >>= 1; step > 0; step >>= 1) {
    int v[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) v[q] = p.hist[min(r[q] + step, n) - 1];
#pragma unroll
    for (int q = 0; q < NQ; ++q) r[q] += (r[q] + step <= n && v[q] <= x[q]) ? step : 0;
  }
}

// the estimate from the two ranks lo = #{o_j <= age}, hi = #{o_j <= age + H} and the prefix sums at both
__device__ __forceinline__ float br_survival_at(const BrParams &p, int age, int lo, int hi, long long sum_lo, long long sum_hi) {
  const float Hf = (float)p.H;
  const int surv = p.hist_n - lo, cnt = hi - lo;
  float pf = 0.0f, mu = 0.0f;
  if (surv > 0 && cnt > 0) {
    const long long rem_sum = (sum_hi - sum_lo) - (long long)cnt * age;
    pf = __fdiv_rn((float)cnt, (float)surv);
    mu = __fdiv_rn((float)(int)rem_sum, (float)cnt);
  }
  float c = __fadd_rn(__fmul_rn(__fsub_rn(1.0f, pf), Hf), __fmul_rn(pf, mu));
  if (p.gate > 0.0f && pf < p.gate) c = Hf;
  c = c < 1.0f ? 1.0f : c;
  c = c > Hf ? Hf : c;
  return c;
}

__device__ __forceinline__ float br_survival(const BrParams &p, int age) {
  const int x[2] = {age, age + p.H};
  int r[2];
  br_hist_ranks<2>(p, x, r);
  return br_survival_at(p, age, r[0], r[1], p.hsum[r[0]], p.hsum[r[1]]);
}

// Appendix "Refresh logic", for the four requests a lane holds (`on`: the request stays active over t more
// generated tokens): per token one step less of in-window contribution; the estimator is queried again every
// `refresh` tokens and whenever c_hat would fall below its floor of one.  The four are taken together token by
// token, so that the look-ups of those that query the estimator run side by side (eight ranks per lane in flight)
// instead of one after the other.  Every lane of the wave must call.
__device__ __forceinline__ void br_refresh_update4(const BrParams &p, int t, const bool (&on)[4], float (&ch)[4],
                                                   float (&age)[4], float (&since)[4]) {
  for (int u = 0; u < t; ++u) {
    bool ask[4];
    int x[8];
    bool any = false;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      ask[k] = false;
      if (on[k]) {
        age[k] = __fadd_rn(age[k], 1.0f);
        since[k] = __fadd_rn(since[k], 1.0f);
        const float dec = __fsub_rn(ch[k], 1.0f);
        ask[k] = (int)since[k] >= p.refresh || dec < 1.0f;
        if (!ask[k]) ch[k] = dec;
      }
      any |= ask[k];
      x[2 * k] = ask[k] ? (int)age[k] : 0;
      x[2 * k + 1] = x[2 * k] + p.H;
    }
    if (br_ballot(any) == 0ull) continue;
    int r[8];
    br_hist_ranks<8>(p, x, r);
    long long hs[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) hs[q] = p.hsum[r[q]];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (ask[k]) {
        ch[k] = br_survival_at(p, x[2 * k], r[2 * k], r[2 * k + 1], hs[2 * k], hs[2 * k + 1]);
        since[k] = 0.0f;
      }
    }
  }
}

// the maintained rows (c_hat, age, since) of four consecutive requests: twelve floats, 16-byte aligned
__device__ __forceinline__ void br_rows3_load(const float *q, float (&ch)[4], float (&age)[4], float (&since)[4]) {
  const float4 a0 = *reinterpret_cast<const float4 *>(q);
  const float4 a1 = *reinterpret_cast<const float4 *>(q + 4);
  const float4 a2 = *reinterpret_cast<const float4 *>(q + 8);
  ch[0] = a0.x, age[0] = a0.y, since[0] = a0.z;
  ch[1] = a0.w, age[1] = a1.x, since[1] = a1.y;
  ch[2] = a1.z, age[2] = a1.w, since[2] = a2.x;
  ch[3] = a2.y, age[3] = a2.z, since[3] = a2.w;
}

// ---------------------------------------------------------------- decode step on one list chunk
// Sec. 2.2 load model applied to 256 consecutive slots of one worker list, four slots per lane
// (16-byte accesses): a request whose remaining output is used up within t steps leaves, the others
// gain t tokens and move up to keep the list dense.  `kept` counts the survivors of the list so far
// (uniform), `gone` the kv that left it.  While no request of the list has left, positions do not
// change and the chunk is updated in place with vector stores; from the first leaver on, survivors are
// ranked (lower lanes first, then the lane's own slots in order) and stored one by one.  Every slot
// the chunk overwrites lies at or below the slot it came from and was read by this call or an earlier
// one, so the compaction is safe in place.
// `lim`: slots to fetch, the list length if it is already known, else the row length (the request then does
// not wait for the length to arrive; what lies beyond the list is ignored by br_adv_apply)
__device__ __forceinline__ void br_adv_load(const int32_t *kl, const int32_t *rl, int e0, int lim, int4 &kv, int4 &rem) {
  kv = make_int4(0, 0, 0, 0);
  rem = make_int4(0, 0, 0, 0);
  if (e0 < lim) {
    kv = *reinterpret_cast<const int4 *>(kl + e0);
    rem = *reinterpret_cast<const int4 *>(rl + e0);
  }
}

template <bool PRED>
__device__ __forceinline__ void br_adv_apply(const BrParams &p, int t, int e0, int ng, int chunk0, const int4 &kv4,
                                             const int4 &rem4, int32_t *kw, int32_t *rw, float *pw, int &kept,
                                             int &gone) {
  const int kv[4] = {kv4.x, kv4.y, kv4.z, kv4.w}, rem[4] = {rem4.x, rem4.y, rem4.z, rem4.w};
  bool stay[4], leave[4];
  unsigned long long bs[4];
  bool any_leave = false;
  int nstay = 0;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const bool used = e0 + k < ng;
    stay[k] = used && rem[k] > t;
    leave[k] = used && !stay[k];
    any_leave |= leave[k];
    bs[k] = br_ballot(stay[k]);
    nstay += __builtin_popcountll(bs[k]);
  }
  // maintained estimates: the rows of the lane's four requests are read and brought up to date before anything
  // is written (every lane goes through the update: its look-ups are taken by the whole wave)
  float ch[4] = {0.0f, 0.0f, 0.0f, 0.0f}, age[4] = {0.0f, 0.0f, 0.0f, 0.0f}, since[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  if constexpr (PRED) {
    if (p.pred_mode == 2) {
      if (e0 < ng) br_rows3_load(pw + (int64_t)e0 * 3, ch, age, since);
      br_refresh_update4(p, t, stay, ch, age, since);
    }
  }
  const bool shifted = kept != chunk0;  // an earlier chunk of this list lost a request
  if (!shifted && br_ballot(any_leave) == 0ull) {
    if (e0 < ng) {  // same positions: 16-byte stores; slots beyond the list keep what they held
      *reinterpret_cast<int4 *>(kw + e0) = make_int4(kv[0] + (stay[0] ? t : 0), kv[1] + (stay[1] ? t : 0),
                                                      kv[2] + (stay[2] ? t : 0), kv[3] + (stay[3] ? t : 0));
      *reinterpret_cast<int4 *>(rw + e0) = make_int4(rem[0] - (stay[0] ? t : 0), rem[1] - (stay[1] ? t : 0),
                                                      rem[2] - (stay[2] ? t : 0), rem[3] - (stay[3] ? t : 0));
    }
    if constexpr (PRED) {
      if (p.pred_mode == 2) {
        float *q = pw + (int64_t)e0 * 3;
        if (e0 < ng) {  // rows beyond the list go back as they came
          *reinterpret_cast<float4 *>(q) = make_float4(ch[0], age[0], since[0], ch[1]);
          *reinterpret_cast<float4 *>(q + 4) = make_float4(age[1], since[1], ch[2], age[2]);
          *reinterpret_cast<float4 *>(q + 8) = make_float4(since[2], ch[3], age[3], since[3]);
        }
      }
    }
  } else {
    int below = 0;  // survivors in lower lanes
#pragma unroll
    for (int k = 0; k < 4; ++k) below += br_rank_below(bs[k]);
    int pos = kept + below;
    if constexpr (PRED) {
      // prediction rows move with their requests: all rows of the lane are read before the first is written
      float pr[4][BR_HP];
      if (p.pred_mode == 2) {
#pragma unroll
        for (int k = 0; k < 4; ++k) pr[k][0] = ch[k], pr[k][1] = age[k], pr[k][2] = since[k];
      } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          if (stay[k]) {
#pragma unroll
            for (int q = 0; q < BR_HP; ++q)
              if (q < p.P) pr[k][q] = pw[(int64_t)(e0 + k) * p.P + q];
          }
        }
      }
      int pp = pos;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        if (stay[k]) {
#pragma unroll
          for (int q = 0; q < BR_HP; ++q)
            if (q < p.P) pw[(int64_t)pp * p.P + q] = pr[k][q];
          ++pp;
        }
      }
    }
    int lost = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (stay[k]) {
        kw[pos] = kv[k] + t;
        rw[pos] = rem[k] - t;
        ++pos;
      }
      lost += leave[k] ? kv[k] : 0;
    }
    gone += br_wave_sum(lost);
  }
  kept += nstay;
}
