// Stage-2 subset search for candidate windows of 17..32 requests by the reduction of Appendix "Bit-set subset
// selection": the score of a subset depends on its sum only, so the search needs the set of sums reachable with
// at most k requests of the window, the score of each, and a subset for the best one.
//
// Reachable sums are bit rows: row j (j = 0..k) has bit b set when some subset of at most j requests sums to b.
// Requests are taken in mask-bit order (the window's order, longest first) and each is one shift-OR per row,
// row[j] |= row[j-1] << s, with j descending so that a request is used at most once.  A wave owns the rows:
// lane l updates the 32-bit words l, l + 64, ... of a row, reading two words of the row below.  The rows live in
// LDS when (k + 1) rows of the needed length fit the wave's slice, otherwise in a per-cluster area of the
// workspace (same code, other pointer).
//
// Which subset: the scan over all masks that serves narrower windows returns the lowest mask among the subsets
// with the best score.  For every bit that appears in a row, the index of the request whose shift-OR set it is
// written to a byte table in the workspace (first[j][b]).  A subset that uses request t has a higher mask than
// any subset of the requests before t; so the lowest mask for (sum b, at most j requests) has first[j][b] as its
// highest request, followed by the lowest mask for (b - s_t, at most j - 1), whose highest request is below t
// because that sum was in row j-1 before request t was taken.  Entries left by earlier searches are never read:
// only bits set by this search are looked up.
//
// Which sums are scored.  Bits beyond `room` (token watermark), beyond the sum of the k longest requests and
// beyond BR_DP_MAX_SUM (the length the rows are sized for; wider sums are not candidates, on both sides of the
// parity tests) do not exist.  Of the rest:
//   - below or at the smallest margin min_h m_h every penalty term is zero and the score is aD * sum, strictly
//     increasing in the sum (distinct integers below 2^24 times a positive float stay distinct and ordered after
//     rounding), so only the largest such reachable sum can win;
//   - BR-0 with G > 1 falls strictly beyond the margin (eq. (br0-Fscore): slope -(G-1) in exact integers), so
//     only the smallest reachable sum above the margin can win there, and the rows need no bit beyond
//     margin + longest request;
//   - every other reachable sum is scored as computed (BR-H in fp32 as the kernels round it: no monotonicity is
//     assumed where roundings could reorder neighbours).
// Equal best scores at several sums (or G = 1, whose score is flat beyond the margin) resolve to the lowest
// mask over all of them, found by building the mask of each tied sum.
#pragma once

#include <type_traits>

#include "br_device.h"

#define BR_DP_MAX_SUM 131071                    // rows hold sums 0..131071
#define BR_DP_ROW_WORDS ((BR_DP_MAX_SUM + 1) / 32)
#define BR_DP_LDS_WORDS 8192                    // LDS slice for the rows of one cluster

// words of workspace per cluster: (KM + 1) bit rows + KM byte rows of first[][]
__host__ __device__ inline size_t br_dp_cluster_words(int KM) {
  return (size_t)(KM + 1) * BR_DP_ROW_WORDS + (size_t)KM * (BR_DP_ROW_WORDS * 8);
}

// highest set bit of row `r` at or below `lim` (-1 if none); nw words are in use
template <class RowPtr>
__device__ __forceinline__ int br_dp_highest_at_or_below(RowPtr r, int nw, int lim, int lane) {
  if (lim < 0) return -1;
  const int wl = min(lim >> 5, nw - 1);
  for (int c = (wl >> 6) << 6; c >= 0; c -= BR_WAVE) {
    const int i = c + lane;
    unsigned v = i <= wl ? (unsigned)r[i] : 0u;
    if (i == (lim >> 5) && (lim & 31) != 31) v &= (2u << (lim & 31)) - 1u;
    const unsigned long long bal = br_ballot(v != 0u);
    if (bal != 0ull) {
      const int l = 63 - (int)__builtin_clzll(bal);
      const unsigned vv = (unsigned)__builtin_amdgcn_readlane((int)v, l);
      return (c + l) * 32 + (31 - (int)__builtin_clz(vv));
    }
  }
  return -1;
}

// lowest set bit of row `r` above `lim` (-1 if none)
template <class RowPtr>
__device__ __forceinline__ int br_dp_lowest_above(RowPtr r, int nw, int lim, int lane) {
  const int from = lim + 1;
  for (int c = ((from >> 5) >> 6) << 6; c < nw; c += BR_WAVE) {
    const int i = c + lane;
    unsigned v = (i < nw && i >= (from >> 5)) ? (unsigned)r[i] : 0u;
    if (i == (from >> 5)) v &= ~((1u << (from & 31)) - 1u);
    const unsigned long long bal = br_ballot(v != 0u);
    if (bal != 0ull) {
      const int l = (int)__builtin_ctzll(bal);
      const unsigned vv = (unsigned)__builtin_amdgcn_readlane((int)v, l);
      return (c + l) * 32 + (int)__builtin_ctz(vv);
    }
  }
  return -1;
}

// The lowest mask among the subsets of at most k window requests that sum to `sum` (uniform; `sum` is a bit of
// row k of the finished table).
__device__ __forceinline__ unsigned br_dp_mask_of(const unsigned char *first, const int *win, int k, int sum) {
  unsigned mask = 0u;
  int j = k;
  while (sum > 0 && j >= 1) {
    const int t = br_uniform((int)first[(size_t)(j - 1) * (BR_DP_ROW_WORDS * 32) + sum]) & 31;
    mask |= 1u << t;
    sum -= win[t] >> BR_IDX_BITS;
    --j;
  }
  return mask;
}

// The rows of reachable sums for the window `win` (w requests), at most kmax per subset, sums up to R (nw words per
// row, `stride` words between rows), and the first-request table.  nwv waves may share the work (LDS rows of one
// block): wave wv takes the words lane + 64 (wv + nwv t) of every row, and `sync` is then a block barrier: row
// j-1 is rewritten only after every wave has read it for row j.  UN words per lane and trip.
template <int UN, class RowPtr, class Sync>
__device__ __forceinline__ void br_dp_build(const int *win, int w, int kmax, int R, int nw, RowPtr rows, int stride,
                                            unsigned char *first, int lane, int wv, int nwv, Sync sync) {
  constexpr int RW = BR_DP_ROW_WORDS;
  const unsigned lastmask = (R & 31) == 31 ? 0xffffffffu : (2u << (R & 31)) - 1u;
  for (int j = 0; j <= kmax; ++j)
    for (int i = lane + BR_WAVE * wv; i < nw; i += BR_WAVE * nwv) rows[j * stride + i] = i == 0 ? 1 : 0;  // the empty subset
  sync();
  for (int b = 0; b < w; ++b) {
    const int s = win[b] >> BR_IDX_BITS;
    if (s > R) continue;  // every subset that holds it lies beyond the rows
    const int q = s >> 5, r = s & 31;
    // every row takes every request: row j then always contains row j-1 ("at most j requests")
    for (int j = kmax; j >= 1; --j) {
      auto src = rows + (j - 1) * stride;
      auto dst = rows + j * stride;
      unsigned char *fj = first + (size_t)(j - 1) * (RW * 32);
      for (int i0 = q + lane + BR_WAVE * wv; i0 < nw; i0 += UN * BR_WAVE * nwv) {
        unsigned lo[UN], hi[UN], old[UN];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
          const int i = i0 + u * BR_WAVE * nwv;
          const bool in = i < nw;
          lo[u] = in ? (unsigned)src[i - q] : 0u;
          hi[u] = (in && i - q >= 1) ? (unsigned)src[i - q - 1] : 0u;
          old[u] = in ? (unsigned)dst[i] : 0u;
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
          const int i = i0 + u * BR_WAVE * nwv;
          unsigned v = r ? (lo[u] << r) | (hi[u] >> (32 - r)) : lo[u];
          if (i == nw - 1) v &= lastmask;
          unsigned fresh = v & ~old[u];
          if (i < nw && fresh != 0u) {
            dst[i] = (int)(old[u] | fresh);
            while (fresh != 0u) {
              const int bit = (int)__builtin_ctz(fresh);
              fresh &= fresh - 1u;
              fj[i * 32 + bit] = (unsigned char)b;
            }
          }
        }
      }
      // row j-1 is rewritten next, after every lane has read it here; row j is read again by the next request
      sync();
    }
  }
}

// Between the rows of a build that a block shares in the workspace: every wave's stores to the row just written are
// visible to the others before any of them goes on.
__device__ __forceinline__ void br_dp_sync_ws() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __syncthreads();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

// A helper wave's part of a shared build: the plan comes from the mailbox `svc` (words 11..15: w, kmax, R, nw,
// 1 = rows in the workspace), as wave 0 posted it in br_subset_dp.
__device__ __forceinline__ void br_dp_build_helper(const BrParams &p, const int *win, const int *svc, int *rows_lds, int *ws,
                                                   int lane, int wv) {
  const int KM = min(p.B, p.R_max);
  unsigned char *first = (unsigned char *)(ws + (size_t)(KM + 1) * BR_DP_ROW_WORDS);
  const int nw = svc[14];
  if (svc[15])
    br_dp_build<4>(win, svc[11], svc[12], svc[13], nw, ws, BR_DP_ROW_WORDS, first, lane, wv, 4, [] { br_dp_sync_ws(); });
  else
    br_dp_build<1>(win, svc[11], svc[12], svc[13], nw, rows_lds, nw, first, lane, wv, 4, [] { __syncthreads(); });
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");  // the first-request bytes are visible to wave 0 after the barrier
}

// `win`: the window in LDS, entry b = s << 11 | sorted position, b < w (17..32); kmax = most requests the subset
// may hold; `room`: largest admissible sum; `rows_lds`: BR_DP_LDS_WORDS words of LDS; `ws`: this cluster's
// br_dp_cluster_words(KM) words of workspace.  Returns the chosen mask (0: no admissible subset) and its score key.
// `svc` (or null): the mailbox of a block whose four waves share LDS builds: wave 0 (the caller) posts the plan,
// the others join through br_dp_build_helper between the block barriers.
template <bool BRH>
__device__ __forceinline__ void br_subset_dp(const BrParams &p, const int (&mg)[BR_HP + 1], const int *win, int w,
                                             int kmax, int room, int lane, int *rows_lds, int *ws, unsigned &bestmask,
                                             int &bestkey, int *svc = nullptr) {
  constexpr int RW = BR_DP_ROW_WORDS;
  bestmask = 0u;
  bestkey = BR_KEY_NONE;
  kmax = min(kmax, w);
  if (kmax < 1) return;
  const int KM = min(p.B, p.R_max);
  unsigned char *first = (unsigned char *)(ws + (size_t)(KM + 1) * RW);
  int top = 0;
  for (int b = 0; b < kmax; ++b) top += win[b] >> BR_IDX_BITS;
  const int s0 = win[0] >> BR_IDX_BITS, slast = win[w - 1] >> BR_IDX_BITS;
  int minm = mg[0];
  if constexpr (BRH) {
#pragma unroll
    for (int h = 1; h <= BR_HP; ++h) minm = h <= p.H ? min(minm, mg[h]) : minm;
  }
  const bool two_probe = !BRH && p.G > 1;
  int R = min(min(top, room), BR_DP_MAX_SUM);
  if (two_probe) R = min(R, mg[0] + s0);  // the smallest reachable sum above the margin lies within one request of it
  if (R < slast) return;                  // not even the shortest request of the window is admissible
  if (R == top && minm >= top) {          // the k longest requests fit every margin: the largest sum wins
    bestmask = kmax >= 32 ? 0xffffffffu : (1u << kmax) - 1u;
    bestkey = br_score_key<BRH>(p, mg, top);
    return;
  }
  const int nw = (R >> 5) + 1;

  // scoring over the finished rows: (kmax + 1) rows of `stride` words, LDS or workspace
  auto run = [&](auto rows, const int stride) {
    auto last = rows + kmax * stride;

    // ---- scoring
    int cand_sum = -1, cand_key = BR_KEY_NONE;   // uniform: best so far
    int ties = 0;                                 // sums that share the best key (> 1: masks are compared)
    auto offer = [&](int sum) {
      if (sum < 1) return;
      const int key = br_score_key<BRH>(p, mg, sum);
      if (key > cand_key) {
        cand_key = key, cand_sum = sum, ties = 1;
      } else if (key == cand_key) {
        ++ties;
      }
    };
    offer(br_dp_highest_at_or_below(last, nw, min(minm, R), lane));
    int hi_from = minm;  // sums above this are scored one by one
    if (two_probe) {
      offer(br_dp_lowest_above(last, nw, mg[0], lane));
      hi_from = R;
    }
    if (hi_from < R) {
      // every reachable sum in (hi_from, R]: lanes take words, each lane keeps its best (key, sum) and how many
      // of its sums share that key
      int bk = BR_KEY_NONE, bsum = -1, bn = 0;
      const int from = hi_from + 1;
      for (int i = (from >> 5) + lane; i < nw; i += BR_WAVE) {
        unsigned v = (unsigned)last[i];
        if (i == (from >> 5)) v &= ~((1u << (from & 31)) - 1u);
        while (v != 0u) {
          const int sum = i * 32 + (int)__builtin_ctz(v);
          v &= v - 1u;
          const int key = br_score_key<BRH>(p, mg, sum);
          if (key > bk) {
            bk = key, bsum = sum, bn = 1;
          } else if (key == bk) {
            ++bn;
          }
        }
      }
      const int km = br_wave_max(bk);
      if (km != BR_KEY_NONE && km >= cand_key) {
        const int n_at = br_wave_sum(bk == km ? bn : 0);
        const int s_at = br_wave_min(bk == km ? bsum : INT32_MAX);
        if (km > cand_key) {
          cand_key = km, cand_sum = s_at, ties = n_at;
        } else {
          ties += n_at;
        }
      }
    }
    if (cand_sum < 0) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");  // first[][] is complete and visible
    __builtin_amdgcn_wave_barrier();
    bestkey = cand_key;
    if (ties <= 1) {
      bestmask = br_dp_mask_of(first, win, kmax, cand_sum);
      return;
    }
    // several sums share the best score: the lowest mask over all of them (one sum at a time, in ascending order)
    unsigned best = 0xffffffffu;
    for (int sum = br_dp_lowest_above(last, nw, 0, lane); sum >= 0; sum = br_dp_lowest_above(last, nw, sum, lane)) {
      if (br_score_key<BRH>(p, mg, sum) == cand_key) best = min(best, br_dp_mask_of(first, win, kmax, sum));
    }
    bestmask = best;
  };

  if ((kmax + 1) * nw <= BR_DP_LDS_WORDS) {
    if (svc != nullptr) {  // the block's four waves build the rows together
      svc[11] = w, svc[12] = kmax, svc[13] = R, svc[14] = nw, svc[15] = 0;
      svc[0] = 2;
      __syncthreads();
      br_dp_build<1>(win, w, kmax, R, nw, rows_lds, nw, first, lane, 0, 4, [] { __syncthreads(); });
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      __syncthreads();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");  // the helpers' first-request bytes
    } else {
      // LDS operations of one wave execute in order: a wave-level fence is all the exchange between lanes needs,
      // and the byte stores to first[][] stay in flight behind it
      br_dp_build<1>(win, w, kmax, R, nw, rows_lds, nw, first, lane, 0, 1, [] { br_wave_sync(); });
    }
    run(rows_lds, nw);
  } else {
    // workspace rows: four words per lane and trip, so that their loads overlap
    if (svc != nullptr) {
      svc[11] = w, svc[12] = kmax, svc[13] = R, svc[14] = nw, svc[15] = 1;
      svc[0] = 2;
      __syncthreads();
      br_dp_build<4>(win, w, kmax, R, nw, ws, RW, first, lane, 0, 4, [] { br_dp_sync_ws(); });
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      __syncthreads();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    } else {
      br_dp_build<4>(win, w, kmax, R, nw, ws, RW, first, lane, 0, 1, [] {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
        __builtin_amdgcn_wave_barrier();
      });
    }
    run(ws, RW);
  }
}
