// In-register bitonic sort of one wavefront's E*64 keys, descending by position
// pos = j*64 + lane (x[j] of lane l holds position j*64 + l).
//
// Compare-exchange partners that differ in a bit >= 64 sit in the same lane (two registers of
// one lane: a min and a max, no data movement).  Partners 1 or 2 lanes apart come through a DPP
// quad permute, 4 or 8 lanes apart through a pair of bank-masked DPP row shifts, 16 apart
// through ds_swizzle and 32 apart through ds_bpermute; none of these touches LDS memory.
#pragma once

#include "br_device.h"

template <int S>
__device__ __forceinline__ unsigned br_xor_lane(unsigned x, int bperm_addr) {
  if constexpr (S == 1) {
    return (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0xB1, 0xF, 0xF, true);  // quad_perm [1,0,3,2]
  } else if constexpr (S == 2) {
    return (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x4E, 0xF, 0xF, true);  // quad_perm [2,3,0,1]
  } else if constexpr (S == 4) {
    // lanes with bit 2 clear (banks 0,2) read lane+4, the others (banks 1,3) read lane-4
    int y = __builtin_amdgcn_update_dpp(0, (int)x, 0x104, 0xF, 0x5, false);  // row_shl:4
    y = __builtin_amdgcn_update_dpp(y, (int)x, 0x114, 0xF, 0xA, false);      // row_shr:4
    return (unsigned)y;
  } else if constexpr (S == 8) {
    int y = __builtin_amdgcn_update_dpp(0, (int)x, 0x108, 0xF, 0x3, false);  // row_shl:8
    y = __builtin_amdgcn_update_dpp(y, (int)x, 0x118, 0xF, 0xC, false);      // row_shr:8
    return (unsigned)y;
  } else if constexpr (S == 16) {
    return (unsigned)__builtin_amdgcn_ds_swizzle((int)x, 0x401F);  // and 0x1f, or 0, xor 0x10
  } else {
    return (unsigned)__builtin_amdgcn_ds_bpermute(bperm_addr, (int)x);
  }
}

// One cross-lane stage (partner distance S < 64) of the merge of blocks of size K.
template <int E, int K, int S>
__device__ __forceinline__ void br_sort_lane_stage(unsigned (&x)[E], int lane, int n2) {
  const int addr32 = (lane ^ 32) << 2;
  const bool lower = (lane & S) == 0;
  bool keep_max_lane = lower;  // K >= 64: direction is a per-register constant
  if constexpr (K < 64) keep_max_lane = ((lane & K) == 0) == lower;
#pragma unroll
  for (int j = 0; j < E; ++j) {
    if (j * 64 < n2) {
      const unsigned y = br_xor_lane<S>(x[j], addr32);
      const unsigned hi = max(x[j], y), lo = min(x[j], y);
      bool keep_max = keep_max_lane;
      if constexpr (K >= 64) keep_max = (((j * 64) & K) == 0) ? lower : !lower;
      x[j] = keep_max ? hi : lo;
    }
  }
}

// One in-lane stage (partner distance S >= 64): registers j and j + S/64 of the same lane.
template <int E, int K, int S>
__device__ __forceinline__ void br_sort_reg_stage(unsigned (&x)[E], int n2) {
  constexpr int JS = S / 64;
#pragma unroll
  for (int j = 0; j < E; ++j) {
    if ((j & JS) == 0 && j + JS < E && (j + JS) * 64 < n2) {
      const bool desc = ((j * 64) & K) == 0;
      const unsigned hi = max(x[j], x[j + JS]), lo = min(x[j], x[j + JS]);
      x[j] = desc ? hi : lo;
      x[j + JS] = desc ? lo : hi;
    }
  }
}

template <int E, int K, int S>
__device__ __forceinline__ void br_sort_merge(unsigned (&x)[E], int lane, int n2) {
  if constexpr (S >= 64)
    br_sort_reg_stage<E, K, S>(x, n2);
  else
    br_sort_lane_stage<E, K, S>(x, lane, n2);
  if constexpr (S > 1) br_sort_merge<E, K, S / 2>(x, lane, n2);
}

template <int E, int K>
__device__ __forceinline__ void br_sort_levels(unsigned (&x)[E], int lane, int n2) {
  if constexpr (K > 2) br_sort_levels<E, K / 2>(x, lane, n2);
  if (K <= n2) br_sort_merge<E, K, K / 2>(x, lane, n2);
}

// Sort the first n2 positions (n2 a power of two, 64 <= n2 <= E*64) in descending order.
// Positions >= n2 must hold keys no larger than any key below n2 (they are left alone).
template <int E>
__device__ __forceinline__ void br_sort_desc(unsigned (&x)[E], int lane, int n2) {
  br_sort_levels<E, E * 64>(x, lane, n2);
}

// Sort of up to 2048 keys by the four waves of a block, 512 per wave (8 registers per lane):
// position = w*512 + j*64 + lane, descending over the whole block.  Each wave sorts its own 512, then
// two merge levels follow.  A level starts by comparing the two sorted halves mirrored (element i of
// the first with element n-1-i of the second, through `buf` in LDS); after that every element of the
// first half is at least every element of the second and each half is bitonic, so halves are finished
// by plain half-cleaners: across waves at distance 512 (same position in the partner wave), inside a
// wave by the register and lane stages above.  Every wave of the block must call this (block barriers).
__device__ __forceinline__ void br_sort_block4_exchange(unsigned (&x)[8], int *buf, int w, int lane, int partner,
                                                        bool mirrored, bool keep_max) {
#pragma unroll
  for (int j = 0; j < 8; ++j) buf[w * 512 + j * 64 + lane] = (int)x[j];
  __syncthreads();
  unsigned y[8];
#pragma unroll
  for (int j = 0; j < 8; ++j)
    y[j] = (unsigned)(mirrored ? buf[partner * 512 + (7 - j) * 64 + (63 - lane)] : buf[partner * 512 + j * 64 + lane]);
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 8; ++j) x[j] = keep_max ? max(x[j], y[j]) : min(x[j], y[j]);
}

__device__ __forceinline__ void br_sort_desc_block4(unsigned (&x)[8], int *buf, int w, int lane) {
  br_sort_desc<8>(x, lane, 512);
  br_sort_block4_exchange(x, buf, w, lane, w ^ 1, true, (w & 1) == 0);   // pairs of waves: 1024 keys each
  br_sort_merge<8, 512, 256>(x, lane, 512);
  br_sort_block4_exchange(x, buf, w, lane, 3 - w, true, w < 2);          // all four: 2048 keys
  br_sort_block4_exchange(x, buf, w, lane, w ^ 1, false, (w & 1) == 0);
  br_sort_merge<8, 512, 256>(x, lane, 512);
}
