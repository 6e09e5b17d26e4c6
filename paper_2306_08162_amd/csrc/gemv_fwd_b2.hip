// Small-token-count forward kernels for 2-bit codes (see gemv_fwd_impl.hpp).
#include "gemv_fwd_impl.hpp"

namespace qlora {

template bool launch_fwd_small_bits<2>(const FwdMulti &, int, bool, hipStream_t);

}  // namespace qlora
