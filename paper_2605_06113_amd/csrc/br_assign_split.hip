// Round and decode steps of a BR-0 cluster on two waves (br_route_advance for queues of up to 512 entries,
// windows of up to 8 requests, small batches): a block holds RPB waves that each run the round of one cluster
// (Alg. BR-0) and NH helper waves that, meanwhile, compute the snapshot reductions of those clusters (if asked for) and applies the
// decode steps (Sec. 2.2) to their lists as they stand at the start of the step.  The wave that ran the round
// appends its admissions behind the old survivors, already advanced (br_assign_epilogue_split).  The decode step
// streams the lists from HBM while the rounds, dependent chains that leave the memory system idle, are still
// running: neither waits for the other except at one LDS flag per cluster, which the helper always sets.
#include "br_assign_kernel.h"

template <int E, int RPB, int NH>
__global__ __launch_bounds__((RPB + NH) * BR_WAVE) void br_k_route_split(BrParams p, BrArr a, BrOut o) {
  extern __shared__ int lds_all[];
  constexpr int WORDS = 3 * E * BR_WAVE + BR_WAVE + 8 + BR_SPLIT_WORDS;  // skey, adm, who, slots, win, split area
  constexpr int SPLIT_AT = WORDS - BR_SPLIT_WORDS;
  const int w = threadIdx.x >> 6, lane = br_lane();
  const int first = (int)blockIdx.x * RPB;
  if (w == RPB && lane < RPB) lds_all[lane * WORDS + SPLIT_AT] = 0;  // flags down before any wave looks
  __syncthreads();
  if (w < RPB) {
    const int inst = first + w;
    if (inst >= p.N) return;
    int *lds = lds_all + w * WORDS;
    br_assign_body<E, false, false>(p, a, o, lds, inst, 0, nullptr, lds + SPLIT_AT);
  } else {
    for (int c = w - RPB; c < RPB; c += NH) {  // helper h takes clusters h, h + NH, ...
      const int inst = first + c;
      if (inst >= p.N) break;
      br_split_helper<E, 8>(p, a, o, inst, lane, lds_all + c * WORDS + SPLIT_AT);
    }
  }
}

template <int E, int RPB, int NH>
static void launch_split(const BrParams &p, const BrArr &a, const BrOut &o, hipStream_t st) {
  const size_t lds = (size_t)RPB * (3 * E * BR_WAVE + BR_WAVE + 8 + BR_SPLIT_WORDS) * sizeof(int);
  const dim3 grid((unsigned)((p.N + RPB - 1) / RPB)), block((RPB + NH) * BR_WAVE);
  hipLaunchKernelGGL((br_k_route_split<E, RPB, NH>), grid, block, lds, st, p, a, o);
}

// For batches that leave most SIMDs to a single wave (fewer clusters than two waves per SIMD): one round and one
// helper per block.  Larger batches keep the one-wave kernels: with four or more waves per SIMD the decode step
// already overlaps other clusters' rounds, and a block of four rounds and two helpers (six waves per SIMD) has to
// fit 80 registers, which spills in the round's loops (measured on 4096 clusters of the c4 shape: 153 us against
// 134 us for the one-wave kernel; 163 us with five waves per SIMD and one helper for four clusters, which then
// is the last to finish).
bool br_split_serves(const BrParams &p) {
  return p.adv_t > 0 && p.H == 0 && p.R_max <= 8 && p.Q <= 512 && p.N < BR_SCORE_WAVE_MIN_N;
}

void br_launch_route_split(const BrParams &p, const BrArr &a, const BrOut &o, hipStream_t st) {
  if (p.Q <= 256)
    launch_split<4, 1, 1>(p, a, o, st);
  else
    launch_split<8, 1, 1>(p, a, o, st);
}
