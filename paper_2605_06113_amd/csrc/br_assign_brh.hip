// BR-H instantiations of the assignment kernel (Alg. BR-H), and the dispatch between the
// integer kernel, the register-horizon kernel and the long-horizon kernel.
#include "br_assign_kernel.h"

void br_launch_assign(const BrParams &p, const BrArr &a, const BrOut &o, hipStream_t st) {
  if (p.H > BR_HP)
    br_launch_assign_long(p, a, o, st);
  else if (p.R_max > 8)
    br_launch_assign_bigr(p, a, o, st);
  else if (p.H > 0)
    br_launch_assign_sized<true>(p, a, o, st);
  else
    br_launch_assign_br0(p, a, o, st);
}
