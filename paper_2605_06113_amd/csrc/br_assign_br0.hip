// BR-0 instantiations of the assignment kernel (Alg. BR-0); the BR-H ones are a translation unit
// of their own so that the two compile side by side.
#include "br_assign_kernel.h"

void br_launch_assign_br0(const BrParams &p, const BrArr &a, const BrOut &o, hipStream_t st) {
  br_launch_assign_sized<false>(p, a, o, st);
}
