// Instantiations of the assignment kernel for candidate windows of 9..16 requests (R_max > 8; Appendix
// "Bit-set subset selection" is about exactly this regime).  The subset search stays an exhaustive one:
// 2^16 masks are 1024 per lane, a few integer operations each, where rows of reachable sums would need
// hundreds of kilobytes per worker popped; see br_assign_kernel.h for the search itself.
#include "br_assign_kernel.h"

void br_launch_assign_bigr(const BrParams &p, const BrArr &a, const BrOut &o, hipStream_t st) {
  if (p.H > 0)
    br_launch_assign_sized<true, true>(p, a, o, st);
  else
    br_launch_assign_sized<false, true>(p, a, o, st);
}
