// The GEMM kernels and their launch code for bf16 operands (design notes: sdrop_gemm.hip).
#include "gemm_launch.h"

namespace sdrop {
template int dispatch_typed<BF16>(int, bool, GemmParams &, hipStream_t);
template int fwd_seeded_typed<BF16>(bool, const GemmParams &, hipStream_t);
template int bwd_fused_typed<BF16>(int, int, bool, bool, const GemmParams &, const GemmParams &, int, hipStream_t);
}  // namespace sdrop
