// 8-bit instantiations of the register-resident inner loop with helper waves
// (see inner_reg_helped_impl.hpp).
#include "inner_reg_helped_impl.hpp"

namespace halp {
int launch_inner_reg_helped_b8(const InArgs& a, int nw, int upl, int R, hipStream_t s) {
  return innerhelp::launch_bits<8>(a, nw, upl, R, s);
}
}  // namespace halp
