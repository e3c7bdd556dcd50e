// Instantiations of the contraction kernels: first operand contraction-contiguous, second output-contiguous (input-gradient products).
#include "gemm_kernels.hpp"

namespace mp {
template int launch_tile<true, false>(int, const GemmArgs&, dim3, hipStream_t);
}  // namespace mp
