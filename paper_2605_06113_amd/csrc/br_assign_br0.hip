// BR-0 instantiations of the assignment kernel (Alg. BR-0); the BR-H ones are a translation unit
// of their own so that the two compile side by side.
#include "br_assign_kernel.h"
#include "br_score_wave.h"

// The whole round of a cluster with a short queue on one wave, in one launch: first the snapshot
// reductions (per-request best worker, per-worker best request: K2 + K3), then the two-stage assignment
// (K4, and the decode step with ADV).  The reductions read the step-start state before the assignment
// changes it, cost the wave about a tenth more instructions, and save a launch of their own.
template <bool ADV>
__global__ __launch_bounds__(256) void br_k_route4(BrParams p, BrArr a, BrOut o) {
  extern __shared__ int lds_all[];
  constexpr int E = 4;
  const int w = threadIdx.x >> 6, inst = (int)blockIdx.x * 4 + w;
  if (inst >= p.N) return;
  BrScoreIn<E, false> in;  // loaded once, used by both parts
  br_score_wave_load<E, false>(p, a, inst, br_lane(), in);
  br_score_wave_run<E, false>(p, o, inst, br_lane(), in);
  br_assign_body<E, false, ADV>(p, a, o, lds_all + w * (3 * E * BR_WAVE + BR_WAVE + 8), inst, 0, &in);
}

void br_launch_route4(const BrParams &p, const BrArr &a, const BrOut &o, hipStream_t st) {
  const size_t lds = (size_t)(4 * (3 * 4 * BR_WAVE + BR_WAVE + 8)) * sizeof(int);
  const dim3 grid((unsigned)((p.N + 3) / 4)), block(256);
  if (p.adv_t > 0)
    hipLaunchKernelGGL(br_k_route4<true>, grid, block, lds, st, p, a, o);
  else
    hipLaunchKernelGGL(br_k_route4<false>, grid, block, lds, st, p, a, o);
}

void br_launch_assign_br0(const BrParams &p, const BrArr &a, const BrOut &o, hipStream_t st) {
  br_launch_assign_sized<false>(p, a, o, st);
}
