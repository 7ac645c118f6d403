// 8-bit instantiations of the register-resident inner loop (see inner_reg_impl.hpp).
#include "inner_reg_impl.hpp"

namespace halp {
int launch_inner_reg_b8(const InArgs& a, int nw, int upl, int R, bool packed, hipStream_t s) {
  return innerreg::launch_bits<8>(a, nw, upl, R, packed, s);
}
}  // namespace halp
