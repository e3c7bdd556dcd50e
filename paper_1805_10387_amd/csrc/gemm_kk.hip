// Instantiations of the contraction kernels: both operands contraction-contiguous (forward products).
#include "gemm_kernels.hpp"

namespace mp {
template int launch_tile<true, true>(int, const GemmArgs&, dim3, hipStream_t);
}  // namespace mp
