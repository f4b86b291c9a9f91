// BR-H counterpart of br_k_route4: for large batches of clusters with queues of up to 512 entries the wave that
// owns a cluster first computes the snapshot reductions (K2 + K3, on the step-start margins of the projection
// kernels), then runs the two-stage assignment (K4, and the decode step with ADV), in one launch.
#include "br_assign_kernel.h"
#include "br_score_wave.h"

template <int E, bool ADV>
__global__ __launch_bounds__(256, E == 8 ? 4 : 1) void br_k_route_h(BrParams p, BrArr a, BrOut o) {
  extern __shared__ int lds_all[];
  const int w = threadIdx.x >> 6, inst = (int)blockIdx.x * 4 + w;
  if (inst >= p.N) return;
  BrScoreIn<E, true> in;  // queue lengths, prefill lengths and counts are loaded once, for both parts
  br_score_wave_load<E, true>(p, a, inst, br_lane(), in);
  br_score_wave_run<E, true>(p, o, inst, br_lane(), in);
  br_assign_body<E, true, ADV>(p, a, o, lds_all + w * (3 * E * BR_WAVE + BR_WAVE + 8), inst, 0, &in);
}

template <int E>
static void launch_route_h(const BrParams &p, const BrArr &a, const BrOut &o, hipStream_t st) {
  const size_t lds = (size_t)(4 * (3 * E * BR_WAVE + BR_WAVE + 8)) * sizeof(int);
  const dim3 grid((unsigned)((p.N + 3) / 4)), block(256);
  if (p.adv_t > 0)
    hipLaunchKernelGGL((br_k_route_h<E, true>), grid, block, lds, st, p, a, o);
  else
    hipLaunchKernelGGL((br_k_route_h<E, false>), grid, block, lds, st, p, a, o);
}

void br_launch_route_h(const BrParams &p, const BrArr &a, const BrOut &o, hipStream_t st) {
  if (p.Q <= 256)
    launch_route_h<4>(p, a, o, st);
  else
    launch_route_h<8>(p, a, o, st);
}
