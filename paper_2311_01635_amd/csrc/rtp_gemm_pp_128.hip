// Instantiation of the ping-pong bf16 GEMM for tile height 128 (see rtp_gemm_pp.h).
#include "rtp_gemm_pp.h"

namespace rtp {
hipError_t launch_gemm_bf16_pp_128(int layout, const GemmArgs &a, int tiles_n, hipStream_t s)
{
    return launch_gemm_bf16_pp_bm<128>(layout, a, tiles_n, s);
}
} // namespace rtp
