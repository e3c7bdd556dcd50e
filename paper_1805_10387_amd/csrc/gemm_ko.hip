// Instantiations of the contraction kernels: first operand contraction-contiguous, second output-contiguous (input-gradient products).
#include "gemm_dtl.hpp"

namespace mp {
template int launch_tile<true, false>(int, const GemmArgs&, dim3, hipStream_t);
template int launch_dtl_tile<true, false>(int, const GemmArgs&, int, hipStream_t);
}  // namespace mp
