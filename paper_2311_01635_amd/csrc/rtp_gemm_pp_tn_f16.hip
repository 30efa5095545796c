// Instantiation of the ping-pong GEMM for fp16 inputs, TN operand layout (see rtp_gemm_pp.h).
#include "rtp_gemm_pp.h"

namespace rtp {
hipError_t launch_gemm_pp_tn_f16(const PpGroup &g, unsigned blocks, hipStream_t s, hipEvent_t done)
{
    return launch_gemm_pp_layout<LAY_TN, _Float16>(g, blocks, s, done);
}
} // namespace rtp
