// Launcher of the ping-pong bf16 GEMM: shape rules and the choice of tile height.
#include "rtp_kernels.h"

#include <algorithm>

namespace rtp {

hipError_t launch_gemm_bf16_pp_256(int layout, const GemmArgs &a, int tiles_n, hipStream_t s);
hipError_t launch_gemm_bf16_pp_192(int layout, const GemmArgs &a, int tiles_n, hipStream_t s);
hipError_t launch_gemm_bf16_pp_128(int layout, const GemmArgs &a, int tiles_n, hipStream_t s);

bool gemm_bf16_pp_supported(int layout, const GemmArgs &a)
{
    if (a.K < 32 || (a.K & 31)) return false;
    if (layout == LAY_TN && a.M < 8) return false;
    if (layout != LAY_NT && a.N < 8) return false;
    return true;
}

static int compute_units()
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            cus = n;
        else
            cus = 256;
    }
    return cus;
}

// Tile height with the shortest estimated run: (rounds of workgroups over the compute units) x
// (work per tile), with a small handicap for the shorter tiles, which move more operand bytes
// per flop.  bm_override != 0 forces a height (kernel tests).
int gemm_bf16_pp_pick_bm(const GemmArgs &a, int bm_override)
{
    if (bm_override == 256 || bm_override == 192 || bm_override == 128) return bm_override;
    const int ncols = a.epi == EPI_SWIGLU_FWD ? a.half : a.N;
    const int bn = a.epi == EPI_SWIGLU_FWD ? 128 : 256;
    const long tiles_n = (ncols + bn - 1) / bn;
    const int cus = std::max(1, compute_units() / std::max(1, a.cu_share));
    const int heights[3] = {256, 192, 128};
    const double handicap[3] = {1.0, 1.04, 1.12};
    int best = 256;
    double best_cost = 1e300;
    for (int i = 0; i < 3; ++i) {
        const long tiles = (long)((a.M + heights[i] - 1) / heights[i]) * tiles_n;
        const long rounds = (tiles + cus - 1) / cus;
        const double cost = (double)rounds * heights[i] * handicap[i];
        if (cost < best_cost - 1e-9) {
            best_cost = cost;
            best = heights[i];
        }
    }
    return best;
}

hipError_t launch_gemm_bf16_pp(int layout, const GemmArgs &a, int bm_override, hipStream_t s)
{
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    if (!gemm_bf16_pp_supported(layout, a)) return hipErrorInvalidValue;
    const int ncols = a.epi == EPI_SWIGLU_FWD ? a.half : a.N;
    const int bn = a.epi == EPI_SWIGLU_FWD ? 128 : 256;
    const int tiles_n = (ncols + bn - 1) / bn;
    switch (gemm_bf16_pp_pick_bm(a, bm_override)) {
    case 256: return launch_gemm_bf16_pp_256(layout, a, tiles_n, s);
    case 192: return launch_gemm_bf16_pp_192(layout, a, tiles_n, s);
    default: return launch_gemm_bf16_pp_128(layout, a, tiles_n, s);
    }
}

} // namespace rtp
