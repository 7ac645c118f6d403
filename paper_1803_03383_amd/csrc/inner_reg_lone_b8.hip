// Instantiations of the register-resident inner loop with one chain wave and helper waves on
// the other SIMDs (8 bits; see inner_reg_lone_impl.hpp).
#include "inner_reg_lone_impl.hpp"

namespace halp {
int launch_inner_reg_lone_b8(const InArgs& a, int upl, int R, bool pair, hipStream_t s) {
  if (upl == 2) return pair ? innerlone::launch_one<2, true>(a, R, s) : innerlone::launch_one<2, false>(a, R, s);
  if (upl == 4) return pair ? innerlone::launch_one<4, true>(a, R, s) : innerlone::launch_one<4, false>(a, R, s);
  if (upl == 8) return innerlone::launch_one<8, false>(a, R, s);
  return HALP_ERR_UNSUPPORTED;
}
}  // namespace halp
