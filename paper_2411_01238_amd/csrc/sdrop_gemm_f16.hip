// The GEMM kernels and their launch code for fp16 operands (design notes: sdrop_gemm.hip).
#include "gemm_launch.h"

namespace sdrop {
template int dispatch_typed<F16>(int, bool, GemmParams &, hipStream_t);
template int fwd_seeded_typed<F16>(bool, const GemmParams &, hipStream_t);
template int bwd_fused_typed<F16>(int, int, bool, bool, const GemmParams &, const GemmParams &, int, hipStream_t);
}  // namespace sdrop
