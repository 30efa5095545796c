// Instantiation of the ping-pong bf16 GEMM for the TN operand layout (see rtp_gemm_pp.h).
#include "rtp_gemm_pp.h"

namespace rtp {
hipError_t launch_gemm_bf16_pp_tn(const PpGroup &g, unsigned blocks, hipStream_t s)
{
    return launch_gemm_bf16_pp_layout<LAY_TN>(g, blocks, s);
}
} // namespace rtp
