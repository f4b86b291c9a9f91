// Host-side launchers of the gfx950 kernels (one per kernel; each only enqueues).
#pragma once

#include <hip/hip_runtime.h>

#include "br_device.h"

// `pol`: per-cluster state of the comparison policies (round-robin cursor, draws made), [N][2]
void br_launch_clear(const BrParams &p, int *pol, hipStream_t st);
void br_launch_load_init(const BrParams &p, const int32_t *n, const int32_t *kv, const int32_t *rem, const float *pred,
                         hipStream_t st);
void br_launch_advance(const BrParams &p, int t, hipStream_t st);
void br_launch_project(const BrParams &p, hipStream_t st);
// horizons beyond BR_HP: fills the discount table p.dl (once per context)
void br_launch_discounts(const BrParams &p, float gamma, hipStream_t st);
// `partials`: br_score_scratch_bytes() of device memory for the partial results of the tiled path, or null
void br_launch_score(const BrParams &p, const BrArr &a, const BrOut &o, int *partials, hipStream_t st);
size_t br_score_scratch_bytes(int N, int Q, int G);
// the library's fixed scratch array (for the entry point that may not use workspace scratch): its size, and its
// device address on the current device
size_t br_static_scratch_bytes();
hipError_t br_static_scratch_resolve(int **out);
void br_launch_assign(const BrParams &p, const BrArr &a, const BrOut &o, hipStream_t st);
// horizons beyond BR_HP: per-offset state in LDS, one wave per cluster
void br_launch_assign_long(const BrParams &p, const BrArr &a, const BrOut &o, hipStream_t st);
// waves per cluster of that kernel (1, 2 or 4); with more than one the decode steps are a launch of their own
int br_long_waves(const BrParams &p);
// candidate windows of 9..16 requests (H <= BR_HP); no fused decode steps
void br_launch_assign_bigr(const BrParams &p, const BrArr &a, const BrOut &o, hipStream_t st);
void br_launch_assign_br0(const BrParams &p, const BrArr &a, const BrOut &o, hipStream_t st);
// BR-0, Q <= 256: snapshot reductions and assignment of four clusters per block in one launch
void br_launch_route4(const BrParams &p, const BrArr &a, const BrOut &o, hipStream_t st);
// BR-H (H <= BR_HP), Q <= 512: the same in one launch per four clusters
void br_launch_route_h(const BrParams &p, const BrArr &a, const BrOut &o, hipStream_t st);
void br_launch_bypass(const BrParams &p, const BrArr &a, const BrOut &o, hipStream_t st);
// comparison policies (Random, RR, P2C, JSQ): FIFO dispatch of the waiting queue, BR-0 contexts
void br_launch_baseline(const BrParams &p, const BrArr &a, const BrOut &o, int *pol, int policy, unsigned long long seed,
                        hipStream_t st);
// BR-0 with decode steps, queues of up to 512, windows of up to 8: round and decode steps on two waves per cluster;
// the snapshot reductions (best_g / best_i, when asked for without the matrix) ride on the helper wave
bool br_split_serves(const BrParams &p);
void br_launch_route_split(const BrParams &p, const BrArr &a, const BrOut &o, hipStream_t st);
