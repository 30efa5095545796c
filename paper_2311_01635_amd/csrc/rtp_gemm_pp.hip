// Launcher of the ping-pong bf16 GEMM: shape rules, the choice of tile heights for a
// launch (one GEMM or a group of independent ones) and the order of the group's problems.
#include "rtp_gemm_pp.h"

#include <string.h>

#include <algorithm>
#include <functional>
#include <queue>
#include <vector>

namespace rtp {

hipError_t launch_gemm_pp_nt_bf16(const PpGroup &g, unsigned blocks, hipStream_t s);
hipError_t launch_gemm_pp_nn_bf16(const PpGroup &g, unsigned blocks, hipStream_t s);
hipError_t launch_gemm_pp_tn_bf16(const PpGroup &g, unsigned blocks, hipStream_t s);
hipError_t launch_gemm_pp_nt_f16(const PpGroup &g, unsigned blocks, hipStream_t s);
hipError_t launch_gemm_pp_nn_f16(const PpGroup &g, unsigned blocks, hipStream_t s);
hipError_t launch_gemm_pp_tn_f16(const PpGroup &g, unsigned blocks, hipStream_t s);

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

static int tiles_n_of(const GemmArgs &a)
{
    const int ncols = a.epi == EPI_SWIGLU_FWD ? a.half : a.N;
    const int bn = a.epi == EPI_SWIGLU_FWD ? 128 : 256;
    return (ncols + bn - 1) / bn;
}

// ---- run-time estimate of a launch ------------------------------------------------------
// Unit: one K sub-tile (32) of a 256 x 256 tile.  A tile costs its K loop plus its epilogue,
// scaled by its height; the shorter tiles carry a small handicap because they move more
// operand bytes per flop.  The epilogue terms stand for the HBM traffic of the tile's results
// (fp32 read-modify-write of an accumulator is the heaviest) in units of main-loop steps.
static double epilogue_steps(int epi, int c_is_f32)
{
    switch (epi) {
    case EPI_ACC_ADD: return 30.0;
    case EPI_ACC_FIRST: return 16.0;
    case EPI_ACC_LAST: return 22.0;
    case EPI_SWIGLU_FWD: return 14.0;
    case EPI_GELU_ERF_FWD:
    case EPI_GELU_TANH_FWD: return 16.0;
    case EPI_SWIGLU_BWD: return 20.0;
    case EPI_GELU_ERF_BWD:
    case EPI_GELU_TANH_BWD: return 14.0;
    default: return c_is_f32 ? 16.0 : 8.0;
    }
}

static double tile_cost(const GemmArgs &a, int bm)
{
    const double handicap = bm == 256 ? 1.0 : bm == 192 ? 1.04 : 1.12;
    return handicap * (bm / 256.0) * (a.K / 32 + epilogue_steps(a.epi, a.c_is_f32));
}

// Greedy list schedule of one XCD's share (an eighth of each problem, rounded up) over its
// compute units, problems in the order given: the finishing time of the last tile.
static double makespan(const GemmArgs *a, const int *bm, const int *order, int count, int cus_per_xcd)
{
    std::priority_queue<double, std::vector<double>, std::greater<double>> free_at;
    for (int i = 0; i < cus_per_xcd; ++i) free_at.push(0.0);
    double end = 0.0;
    for (int i = 0; i < count; ++i) {
        const int q = order[i];
        const long tiles = (long)((a[q].M + bm[q] - 1) / bm[q]) * tiles_n_of(a[q]);
        const long mine = (tiles + 7) / 8;
        const double c = tile_cost(a[q], bm[q]);
        for (long t = 0; t < mine; ++t) {
            const double start = free_at.top();
            free_at.pop();
            free_at.push(start + c);
            end = std::max(end, start + c);
        }
    }
    return end;
}

// Heights and launch order (longest tiles first) of a group.  Every combination of heights
// is tried (at most 3^4); the estimate above picks.
static void plan_group(const GemmArgs *a, int count, const int *bm_override, int cu_share, int *bm_out, int *order_out)
{
    const int heights[3] = {256, 192, 128};
    const int cus_per_xcd = std::max(1, compute_units() / std::max(1, cu_share) / 8);
    int combos = 1;
    for (int q = 0; q < count; ++q) combos *= 3;
    double best = 1e300;
    int bm[PP_MAX_GROUP], order[PP_MAX_GROUP];
    for (int c = 0; c < combos; ++c) {
        int x = c;
        bool ok = true;
        for (int q = 0; q < count; ++q, x /= 3) {
            bm[q] = heights[x % 3];
            const int forced = bm_override ? bm_override[q] : 0;
            if ((forced == 256 || forced == 192 || forced == 128) && forced != bm[q]) ok = false;
        }
        if (!ok) continue;
        for (int q = 0; q < count; ++q) order[q] = q;
        std::stable_sort(order, order + count, [&](int i, int j) { return tile_cost(a[i], bm[i]) > tile_cost(a[j], bm[j]); });
        const double t = makespan(a, bm, order, count, cus_per_xcd);
        if (t < best - 1e-9) {
            best = t;
            for (int q = 0; q < count; ++q) {
                bm_out[q] = bm[q];
                order_out[q] = order[q];
            }
        }
    }
}

void gemm_bf16_pp_plan(int layout, const GemmArgs *a, int count, const int *bm_override, int *bm_out)
{
    (void)layout;
    int order[PP_MAX_GROUP];
    if (count < 1 || count > PP_MAX_GROUP) return;
    plan_group(a, count, bm_override, count == 1 ? a[0].cu_share : 1, bm_out, order);
}

hipError_t launch_gemm_bf16_pp_group(int layout, const GemmArgs *a_in, int count_in, const int *bm_override, hipStream_t s)
{
    if (count_in < 0 || count_in > PP_MAX_GROUP) return hipErrorInvalidValue;
    GemmArgs a[PP_MAX_GROUP];
    int forced[PP_MAX_GROUP];
    int count = 0;
    for (int q = 0; q < count_in; ++q) {
        if (a_in[q].M <= 0 || a_in[q].N <= 0) continue; // nothing to compute
        if (!gemm_bf16_args_ok(layout, a_in[q]) || !gemm_bf16_pp_supported(layout, a_in[q])) return hipErrorInvalidValue;
        if (count > 0 && a_in[q].elem != a[0].elem) return hipErrorInvalidValue; // one element type per launch
        forced[count] = bm_override ? bm_override[q] : 0;
        a[count++] = a_in[q];
    }
    if (count == 0) return hipSuccess;
    int bm[PP_MAX_GROUP], order[PP_MAX_GROUP];
    plan_group(a, count, forced, count == 1 ? a[0].cu_share : 1, bm, order);

    PpGroup g;
    memset(&g, 0, sizeof g);
    g.count = count;
    unsigned per_xcd = 0;
    for (int i = 0; i < count; ++i) {
        const int q = order[i];
        PpProblem &p = g.p[i];
        p.a = a[q];
        p.bm = bm[q];
        p.tiles_m = (a[q].M + bm[q] - 1) / bm[q];
        p.tiles_n = tiles_n_of(a[q]);
        p.vec_epilogue = gemm_epilogue_vec_ok(a[q]) ? 1 : 0;
        per_xcd += (unsigned)(((long)p.tiles_m * p.tiles_n + 7) / 8);
    }
    const unsigned blocks = per_xcd * 8;
    const bool f16 = a[0].elem == ELEM_F16;
    switch (layout) {
    case LAY_NT: return f16 ? launch_gemm_pp_nt_f16(g, blocks, s) : launch_gemm_pp_nt_bf16(g, blocks, s);
    case LAY_NN: return f16 ? launch_gemm_pp_nn_f16(g, blocks, s) : launch_gemm_pp_nn_bf16(g, blocks, s);
    case LAY_TN: return f16 ? launch_gemm_pp_tn_f16(g, blocks, s) : launch_gemm_pp_tn_bf16(g, blocks, s);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_gemm_bf16_pp(int layout, const GemmArgs &a, int bm_override, hipStream_t s)
{
    return launch_gemm_bf16_pp_group(layout, &a, 1, &bm_override, s);
}

} // namespace rtp
