// The two products in one launch, operand kinds 2 (g_x product) and 1 (g_w product): see gemm_pair_impl.hpp.
#include "gemm_pair_impl.hpp"

namespace hlq {

hipError_t launch_pair_21(const GemmDev &ga, const GemmDev &gb, const GemmDev &gbt, bool bigA, bool f32, bool bigB, int outB,
                          bool b_first, hipStream_t st)
{
    return launch_pair_kinds<2, 1>(ga, gb, gbt, bigA, f32, bigB, outB, b_first, st);
}

}  // namespace hlq
