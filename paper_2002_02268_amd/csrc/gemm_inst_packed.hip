// Kernels of the product for one operand layout (B_PACKED, A_MK), all tile shapes.
#include "gemm_launch.hpp"

namespace gemmf32_host {
template int launch_tile<B_PACKED, A_MK>(int, const KArgs &);
}
