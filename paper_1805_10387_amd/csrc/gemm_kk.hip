// Instantiations of the contraction kernels: both operands contraction-contiguous (forward products).
#include "gemm_dtl.hpp"

namespace mp {
template int launch_tile<true, true>(int, const GemmArgs&, dim3, hipStream_t);
template int launch_dtl_tile<true, true>(int, const GemmArgs&, int, hipStream_t);
}  // namespace mp
