// 16-bit instantiations of the register-resident inner loop (see inner_reg_impl.hpp).
#include "inner_reg_impl.hpp"

namespace halp {
int launch_inner_reg_b16(const InArgs& a, int nw, int upl, int R, hipStream_t s) {
  return innerreg::launch_bits<16>(a, nw, upl, R, false, s);
}
}  // namespace halp
