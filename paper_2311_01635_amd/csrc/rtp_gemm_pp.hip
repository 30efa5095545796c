// Launcher of the ping-pong bf16 GEMM: shape rules, the choice of tile heights for a
// launch (one GEMM or a group of independent ones) and the order of the group's problems.
#include "rtp_gemm_pp.h"

#include <string.h>

#include <algorithm>
#include <functional>
#include <map>
#include <mutex>
#include <queue>
#include <vector>

namespace rtp {

hipError_t launch_gemm_pp_nt_bf16(const PpGroup &g, unsigned blocks, hipStream_t s, hipEvent_t done);
hipError_t launch_gemm_pp_nn_bf16(const PpGroup &g, unsigned blocks, hipStream_t s, hipEvent_t done);
hipError_t launch_gemm_pp_tn_bf16(const PpGroup &g, unsigned blocks, hipStream_t s, hipEvent_t done);
hipError_t launch_gemm_pp_nt_f16(const PpGroup &g, unsigned blocks, hipStream_t s, hipEvent_t done);
hipError_t launch_gemm_pp_nn_f16(const PpGroup &g, unsigned blocks, hipStream_t s, hipEvent_t done);
hipError_t launch_gemm_pp_tn_f16(const PpGroup &g, unsigned blocks, hipStream_t s, hipEvent_t done);

bool gemm_bf16_pp_supported(int layout, const GemmArgs &a)
{
    if (a.K < 32 || (a.K & 31)) return false;
    if (layout == LAY_TN && a.M < 8) return false;
    if (layout != LAY_NT && a.N < 8) return false;
    // the kernel addresses each operand through a buffer descriptor with 32-bit byte offsets
    const bool a_kc = layout != LAY_TN, b_kc = layout == LAY_NT;
    const int64_t a_elems = (int64_t)((a_kc ? a.M : a.K) - 1) * a.lda + (a_kc ? a.K : a.M);
    const int64_t b_elems = (int64_t)((b_kc ? a.N : a.K) - 1) * a.ldb + (b_kc ? a.K : a.N);
    if (a_elems * 2 >= (int64_t)1 << 31 || b_elems * 2 >= (int64_t)1 << 31) return false;
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

int gemm_bf16_pp_tiles_n(const GemmArgs &a) { return tiles_n_of(a); }

// ---- run-time estimate of a launch ------------------------------------------------------
// Unit: one K sub-tile (32) of a 256 x 256 tile.  A tile costs its K loop plus its epilogue,
// scaled by its height; the shorter tiles carry a small handicap because they move more
// operand bytes per flop.  The epilogue terms stand for the HBM traffic of the tile's results
// (fp32 read-modify-write of an accumulator is the heaviest) in units of main-loop steps.
static double epilogue_steps(int epi, int c_is_f32)
{
    switch (epi) {
    case EPI_ACC_ADD: return 30.0;
    case EPI_ACC_ATOMIC: return 40.0;
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

// frac: the share of the K loop's MFMA time an edge tile still needs (1 for an interior tile), area: the share
// of the tile that exists (scales the epilogue's traffic)
static double tile_cost(const GemmArgs &a, int bm, int ksplit, double frac = 1.0, double area = 1.0)
{
    const double handicap = bm == 256 ? 1.0 : bm == 192 ? 1.04 : 1.12;
    const int kt = a.K / 32, each = (kt + ksplit - 1) / ksplit;
    // (an edge tile still fetches whole sub-tiles and passes every barrier: a floor under its loop time)
    const double loop = each * std::max(frac, 0.35);
    return handicap * (bm / 256.0) * (loop + area * epilogue_steps(ksplit > 1 ? EPI_ACC_ATOMIC : a.epi, a.c_is_f32));
}

// The kernel skips the fragments of an edge tile that lie wholly outside the matrix; the tile then runs as long
// as its busiest wave.  Waves split the tile's rows in two halves (BM / 64 fragment rows each) and hold two
// fragment columns 128 apart (gate / up halves of the paired epilogue: always both or none).
static void edge_shares(const GemmArgs &a, int bm, double *frac_m, double *area_m, double *frac_n, double *area_n)
{
    const int tm = (a.M + bm - 1) / bm, vr = a.M - (tm - 1) * bm; // valid rows of the last tile row
    const int fm = bm / 64;
    *frac_m = vr >= bm / 2 ? 1.0 : (double)((vr + 31) / 32) / fm;
    *area_m = (double)vr / bm;
    const bool paired = a.epi == EPI_SWIGLU_FWD;
    const int ncols = paired ? a.half : a.N, bn = paired ? 128 : 256;
    const int tn = (ncols + bn - 1) / bn, vc = ncols - (tn - 1) * bn;
    *frac_n = paired || vc > 128 ? 1.0 : 0.5;
    *area_n = (double)vc / bn;
}

// A problem may have its K loop cut into chunks when its result is an fp32 sum onto an accumulator
// (the chunks' partial sums are added atomically) and it is short of tiles: the weight-gradient
// GEMM of a narrow shard contracts over all T tokens into an output of a few tiles.
static bool may_split_k(const GemmArgs &a)
{
    if (a.sync) return false; // the counters count whole tiles
    return a.epi == EPI_ACC_ADD && a.c_is_f32 && a.C == (void *)a.ws && a.ldc == a.ldws;
}

// Greedy list schedule of one XCD's share (an eighth of each problem, rounded up) over its
// compute units, problems in the order given: the finishing time of the last tile.
static double makespan(const GemmArgs *a, const int *bm, const int *ks, const int *order, int count, int cus_per_xcd)
{
    std::priority_queue<double, std::vector<double>, std::greater<double>> free_at;
    for (int i = 0; i < cus_per_xcd; ++i) free_at.push(0.0);
    double end = 0.0;
    for (int i = 0; i < count; ++i) {
        const int q = order[i];
        const int kt = a[q].K / 32, each = (kt + ks[q] - 1) / ks[q], chunks = (kt + each - 1) / each;
        const long tm = (a[q].M + bm[q] - 1) / bm[q], tn = tiles_n_of(a[q]);
        const long tiles = tm * tn * chunks;
        const long mine = (tiles + 7) / 8;
        // interior tiles, then the last tile column, the last tile row and the corner, each with its own cost
        double fm, am, fn, an;
        edge_shares(a[q], bm[q], &fm, &am, &fn, &an);
        const double cost[4] = {tile_cost(a[q], bm[q], ks[q]), tile_cost(a[q], bm[q], ks[q], fn, an),
                                tile_cost(a[q], bm[q], ks[q], fm, am), tile_cost(a[q], bm[q], ks[q], fm * fn, am * an)};
        const long cls[4] = {(tm - 1) * (tn - 1) * chunks, (tm - 1) * chunks, (tn - 1) * chunks, (long)chunks};
        // this XCD's share of each class: the edge classes rounded up, the interior takes the rest
        long cnt[4] = {0, 0, 0, 0}, left = mine;
        for (int c = 3; c >= 1; --c) {
            cnt[c] = std::min(left, (cls[c] * mine + tiles - 1) / tiles);
            left -= cnt[c];
        }
        cnt[0] = left;
        // cheap tiles first: the grid hands tiles out in index order, not longest first, so the tile that starts a
        // further round is as likely a full one as not; an estimate that kept the cheap ones for last favoured plans
        // whose last round never comes out that short (a K split that spilled 8 tiles into a second round)
        for (int c = 3; c >= 0; --c)
            for (long t = 0; t < cnt[c]; ++t) {
                const double start = free_at.top();
                free_at.pop();
                free_at.push(start + cost[c]);
                end = std::max(end, start + cost[c]);
            }
    }
    return end;
}

// Heights, K splits and launch order (longest tiles first) of a group.  Every combination is tried
// (3 heights, and up to 6 split factors for a problem that may be split and is short of tiles);
// the estimate above picks.  Plans are remembered per shape.
struct PlanKey {
    int layout, count, cu_share;
    int dims[PP_MAX_GROUP][6]; // M, N, K, epi, forced height, may split
    bool operator<(const PlanKey &o) const { return memcmp(this, &o, sizeof *this) < 0; }
};
struct Plan {
    int bm[PP_MAX_GROUP], ks[PP_MAX_GROUP], order[PP_MAX_GROUP];
};

static Plan plan_group(int layout, const GemmArgs *a, int count, const int *bm_override, int cu_share)
{
    static std::map<PlanKey, Plan> cache;
    static std::mutex lock;
    PlanKey key;
    memset(&key, 0, sizeof key);
    key.layout = layout; key.count = count; key.cu_share = cu_share;
    for (int q = 0; q < count; ++q) {
        const int forced = bm_override ? bm_override[q] : 0;
        const int d[6] = {a[q].M, a[q].N, a[q].K, a[q].epi + (a[q].sync ? 64 : 0), forced, may_split_k(a[q]) ? 1 : 0};
        memcpy(key.dims[q], d, sizeof d);
    }
    {
        std::lock_guard<std::mutex> g(lock);
        auto it = cache.find(key);
        if (it != cache.end()) return it->second;
    }
    const int heights[3] = {256, 192, 128};
    const int splits[6] = {1, 2, 4, 8, 16, 32};
    const int cus = std::max(8, compute_units() / std::max(1, cu_share));
    const int cus_per_xcd = std::max(1, cus / 8);
    // options per problem
    int nopt[PP_MAX_GROUP], obm[PP_MAX_GROUP][18], oks[PP_MAX_GROUP][18];
    for (int q = 0; q < count; ++q) {
        nopt[q] = 0;
        const int forced = bm_override ? bm_override[q] : 0;
        const long tiles128 = (long)((a[q].M + 127) / 128) * tiles_n_of(a[q]);
        const bool split_ok = may_split_k(a[q]) && tiles128 < cus;
        for (int h = 0; h < 3; ++h) {
            if ((forced == 256 || forced == 192 || forced == 128) && forced != heights[h]) continue;
            for (int k = 0; k < (split_ok ? 6 : 1); ++k) {
                if (splits[k] > 1 && a[q].K / 32 / splits[k] < 4) break; // keep at least four sub-tiles per chunk
                obm[q][nopt[q]] = heights[h];
                oks[q][nopt[q]] = splits[k];
                ++nopt[q];
            }
        }
    }
    Plan best_plan;
    memset(&best_plan, 0, sizeof best_plan);
    double best = 1e300;
    int idx[PP_MAX_GROUP] = {0, 0, 0, 0};
    for (;;) {
        int bm[PP_MAX_GROUP], ks[PP_MAX_GROUP], order[PP_MAX_GROUP];
        for (int q = 0; q < count; ++q) {
            bm[q] = obm[q][idx[q]];
            ks[q] = oks[q][idx[q]];
            order[q] = q;
        }
        bool ordered = false; // a producer / consumer pair keeps the order it was given in
        for (int q = 0; q < count; ++q) ordered = ordered || a[q].sync != nullptr;
        if (!ordered)
            std::stable_sort(order, order + count,
                             [&](int i, int j) { return tile_cost(a[i], bm[i], ks[i]) > tile_cost(a[j], bm[j], ks[j]); });
        // A launch that shares the machine (cu_share > 1) seldom gets exactly its share: its partner on the other
        // stream may be a GEMM of a hundred tiles, or done already.  The estimate is the mean of the two ends, its
        // share of the compute units and all of them, which is what the in-situ sweeps of the tile heights favour
        // (a 96-tile GEMM planned for half the machine kept its 256-high tiles and left compute units idle).
        double t = makespan(a, bm, ks, order, count, cus_per_xcd);
        if (cu_share > 1) t = 0.5 * (t + makespan(a, bm, ks, order, count, std::max(1, compute_units() / 8)));
        if (t < best - 1e-9) {
            best = t;
            for (int q = 0; q < count; ++q) {
                best_plan.bm[q] = bm[q];
                best_plan.ks[q] = ks[q];
                best_plan.order[q] = order[q];
            }
        }
        int q = 0;
        while (q < count && ++idx[q] == nopt[q]) idx[q++] = 0;
        if (q == count) break;
    }
    std::lock_guard<std::mutex> g(lock);
    cache[key] = best_plan;
    return best_plan;
}

void gemm_bf16_pp_plan(int layout, const GemmArgs *a, int count, const int *bm_override, int *bm_out, int *ksplit_out)
{
    if (count < 1 || count > PP_MAX_GROUP) return;
    const Plan pl = plan_group(layout, a, count, bm_override, count == 1 ? a[0].cu_share : 1);
    for (int q = 0; q < count; ++q) {
        if (bm_out) bm_out[q] = pl.bm[q];
        if (ksplit_out) ksplit_out[q] = pl.ks[q];
    }
}

hipError_t launch_gemm_bf16_pp_group(int layout, const GemmArgs *a_in, int count_in, const int *bm_override, hipStream_t s,
                                     hipEvent_t done)
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
    if (count == 0) return done ? hipEventRecord(done, s) : hipSuccess; // nothing to launch: the event still marks this point
    const Plan pl = plan_group(layout, a, count, forced, count == 1 ? a[0].cu_share : 1);
    const int *bm = pl.bm, *order = pl.order;

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
        // as many chunks as are not empty
        const int kt = a[q].K / 32, each = (kt + pl.ks[q] - 1) / pl.ks[q];
        p.ksplit = (kt + each - 1) / each;
        if (p.ksplit > 1) p.a.epi = EPI_ACC_ATOMIC;
        per_xcd += (unsigned)(((long)p.tiles_m * p.tiles_n * p.ksplit + 7) / 8);
    }
    const unsigned blocks = per_xcd * 8;
    const bool f16 = a[0].elem == ELEM_F16;
    switch (layout) {
    case LAY_NT: return f16 ? launch_gemm_pp_nt_f16(g, blocks, s, done) : launch_gemm_pp_nt_bf16(g, blocks, s, done);
    case LAY_NN: return f16 ? launch_gemm_pp_nn_f16(g, blocks, s, done) : launch_gemm_pp_nn_bf16(g, blocks, s, done);
    case LAY_TN: return f16 ? launch_gemm_pp_tn_f16(g, blocks, s, done) : launch_gemm_pp_tn_bf16(g, blocks, s, done);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_gemm_bf16_pp(int layout, const GemmArgs &a, int bm_override, hipStream_t s)
{
    return launch_gemm_bf16_pp_group(layout, &a, 1, &bm_override, s, nullptr);
}

} // namespace rtp
