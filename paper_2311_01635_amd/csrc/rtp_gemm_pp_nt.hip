// Instantiation of the ping-pong GEMM for bf16 inputs, NT operand layout (see rtp_gemm_pp.h).
#include "rtp_gemm_pp.h"

namespace rtp {
hipError_t launch_gemm_pp_nt_bf16(const PpGroup &g, unsigned blocks, hipStream_t s, hipEvent_t done)
{
    return launch_gemm_pp_layout<LAY_NT, __bf16>(g, blocks, s, done);
}
} // namespace rtp
