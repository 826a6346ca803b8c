// The transposed-operand matmuls of Section 4.6.1 (A^T B and A B^T): instantiations of the GEMM
// kernel whose A (resp. B) slice is staged in the other LDS kind; see gemm_kernel.hpp.
#include "gemm_kernel.hpp"

namespace lg {

void launch_tn(const GemmArgs& a, const Plan& pl, bool vec, hipStream_t s) { launch_planned<false, true, false>(a, pl, vec, s); }
void launch_nt(const GemmArgs& a, const Plan& pl, bool vec, hipStream_t s) { launch_planned<false, false, true>(a, pl, vec, s); }

}  // namespace lg
