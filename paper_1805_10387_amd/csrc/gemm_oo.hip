// Instantiations of the contraction kernels: both operands output-contiguous (weight-gradient products, single and grouped).
#include "gemm_dtl.hpp"

namespace mp {
template int launch_tile<false, false>(int, const GemmArgs&, dim3, hipStream_t);
template int launch_dtl_tile<false, false>(int, const GemmArgs&, int, hipStream_t);
template int launch_grouped<256, 256>(const GroupArgs&, int, hipStream_t);
template int launch_grouped<128, 128>(const GroupArgs&, int, hipStream_t);
template int launch_dtl_grouped<256, 256>(const GroupArgs&, int, hipStream_t);
template int launch_dtl_grouped<128, 128>(const GroupArgs&, int, hipStream_t);
}  // namespace mp
