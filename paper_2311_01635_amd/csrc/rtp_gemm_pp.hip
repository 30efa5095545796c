// bf16 partition GEMM for gfx950, "ping-pong" form: the kernel the rotated
// linear layer uses whenever the contraction length is a multiple of 32.
//
// One workgroup of 8 waves owns a 256 x 256 tile of C (wave tile 128 x 64,
// 32x32x16 bf16 MFMA, fp32 accumulators in registers).  K advances in
// sub-tiles of 32 through a ring of four 32 KB LDS stages.
//
//  * HBM -> LDS goes through the direct load (global_load_lds_dwordx4): no
//    staging registers and no ds_write; three sub-tiles are always in flight,
//    which is what hides the L2/HBM latency.
//  * The two waves that share a SIMD run half an iteration apart.  Every
//    iteration of a wave is a "memory" slot (read the 12 MFMA fragments of
//    the sub-tile out of LDS, issue the loads three sub-tiles ahead) and a
//    "compute" slot (16 MFMAs back to back), and a workgroup barrier ends
//    each slot.  Because one group of four waves starts one slot late, one
//    wave of every SIMD is always in its compute slot while the other is in
//    its memory slot, so the LDS pipeline and the MFMA pipeline stay busy at
//    the same time instead of taking turns.
//  * LDS layouts are chosen so that every fragment read is bank-conflict
//    free on the 64-bank LDS: operands contiguous along K are stored as
//    64-byte rows with the 16-byte chunk index xor-ed with (row/4)%4;
//    operands contiguous along M or N are stored as 512-byte K-rows with the
//    chunk index xor-ed with 4*(k%4) and read back with the transposing
//    ds_read_b64_tr_b16.  The direct load writes 64 lanes x 16 bytes to
//    consecutive LDS addresses, so the permutation is applied on the global
//    address each lane fetches.
//
// Layouts and epilogues are those of rtp_gemm_bf16.hip; ragged M and N are
// handled by clamping the fetched row/column (the clamped results are never
// stored), K must be a multiple of 32.
#include "rtp_gemm_epilogue.h"

namespace rtp {

namespace pp {
#ifndef PP_STAGES
#define PP_STAGES 4
#endif
#ifndef PP_PF
#define PP_PF 3
#endif
constexpr int BM = 256, BN = 256, BK = 32, STAGES = PP_STAGES, PF = PP_PF;
static_assert(PF >= 2 && PF < STAGES, "a stage is refilled only after both groups have read it");
constexpr int WM = 2, WN = 4, NTHR = 512;
constexpr int FM = BM / (WM * 32), FN = BN / (WN * 32); // 4 x 2 fragments per wave
constexpr int OPND = BM * BK * 2;                       // 16 KB per operand and stage
constexpr int STAGE = 2 * OPND;
typedef __attribute__((address_space(3))) void *lds_vp;
typedef __attribute__((address_space(1))) const void *glb_vp;
} // namespace pp

template <int LAY>
__global__ __launch_bounds__(pp::NTHR) void gemm_bf16_pp_kernel(const GemmArgs p, const int tiles_m, const int tiles_n,
                                                                 const int vec_epilogue)
{
    using namespace pp;
    constexpr bool A_KC = (LAY != LAY_TN), B_KC = (LAY == LAY_NT);
    __shared__ __attribute__((aligned(1024))) char smem[STAGES * STAGE];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int group = wave >> 2; // waves 0-3 and 4-7 sit on SIMDs 0-3 respectively

    // ---- which tile: neighbouring tiles share one XCD's L2 -----------------------
    int pid = blockIdx.x;
    {
        const int total = gridDim.x;
        const int per = (total + 7) >> 3;
        int tall = total & 7;
        if (tall == 0) tall = 8;
        const int xcd = pid & 7, local = pid >> 3;
        pid = xcd < tall ? xcd * per + local : tall * per + (xcd - tall) * (per - 1) + local;
    }
    constexpr int GROUP_M = 4;
    const int group_sz = GROUP_M * tiles_n;
    const int grp = pid / group_sz;
    const int first_m = grp * GROUP_M;
    const int gm = min(tiles_m - first_m, GROUP_M);
    const int tm = first_m + (pid % group_sz) % gm;
    const int tn = (pid % group_sz) / gm;

    const bool paired = (p.epi == EPI_SWIGLU_FWD);
    const int m0 = tm * BM;
    const int n0 = paired ? tn * (BN / 2) : tn * BN;
    const int M = p.M, N = p.N, K = p.K;
    const int half = p.half;

    // ---- direct-load addresses: two 1 KB pieces of each operand per wave -----------
    // piece j of a K-contiguous operand holds rows 16j..16j+15 (64 bytes each);
    // piece j of an M/N-contiguous operand holds K-rows 2j, 2j+1 (512 bytes each).
    auto a_row = [&](int r) { return min(m0 + r, M - 1); };
    auto a_col = [&](int c) { return min(m0 + c, M - 8); };
    auto b_row = [&](int r) {
        if (paired) return r < BN / 2 ? min(n0 + r, half - 1) : half + min(n0 + r - BN / 2, half - 1);
        return min(n0 + r, N - 1);
    };
    auto b_col = [&](int c) { return min(n0 + c, N - 8); };

    const char *ga[2], *gb[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int j = 2 * wave + i;
        if (A_KC) {
            const int row = 16 * j + (lane >> 2), pc = lane & 3, c = pc ^ ((row >> 2) & 3);
            ga[i] = (const char *)p.A + ((int64_t)a_row(row) * p.lda + c * 8) * 2;
        } else {
            const int kr = 2 * j + (lane >> 5), pc = lane & 31, c = pc ^ (4 * (kr & 3));
            ga[i] = (const char *)p.A + ((int64_t)kr * p.lda + a_col(c * 8)) * 2;
        }
        if (B_KC) {
            const int row = 16 * j + (lane >> 2), pc = lane & 3, c = pc ^ ((row >> 2) & 3);
            gb[i] = (const char *)p.B + ((int64_t)b_row(row) * p.ldb + c * 8) * 2;
        } else {
            const int kr = 2 * j + (lane >> 5), pc = lane & 31, c = pc ^ (4 * (kr & 3));
            gb[i] = (const char *)p.B + ((int64_t)kr * p.ldb + b_col(c * 8)) * 2;
        }
    }
    const int64_t stepA = A_KC ? (int64_t)BK * 2 : (int64_t)BK * p.lda * 2;
    const int64_t stepB = B_KC ? (int64_t)BK * 2 : (int64_t)BK * p.ldb * 2;
    const int KT = K / BK;

    auto issue = [&](int kt) {
        const int kk = min(kt, KT - 1); // past the end: refetch the last sub-tile into a stage nobody reads
        char *st = smem + (kt % STAGES) * STAGE + 2 * wave * 1024;
#pragma unroll
        for (int i = 0; i < 2; ++i)
            __builtin_amdgcn_global_load_lds((glb_vp)(ga[i] + kk * stepA), (lds_vp)(st + i * 1024), 16, 0, 0);
#pragma unroll
        for (int i = 0; i < 2; ++i)
            __builtin_amdgcn_global_load_lds((glb_vp)(gb[i] + kk * stepB), (lds_vp)(st + OPND + i * 1024), 16, 0, 0);
    };

    // ---- fragment addresses -----------------------------------------------------------
    int a_off[FM], b_off[FN];
    {
        const int q = lane >> 4, i16 = lane & 15;
#pragma unroll
        for (int f = 0; f < FM; ++f) {
            const int rb = wm * (BM / WM) + f * 32;
            if (A_KC) {
                const int row = rb + (lane & 31);
                a_off[f] = row * 64 + (((lane >> 5) ^ ((row >> 2) & 3)) << 4);
            } else {
                const int col = rb + (q & 1) * 16 + (i16 & 3) * 4;
                const int kr = (q >> 1) * 8 + (i16 >> 2);
                a_off[f] = kr * 512 + (((col >> 3) ^ (4 * (i16 >> 2))) << 4) + (col & 7) * 2;
            }
        }
#pragma unroll
        for (int f = 0; f < FN; ++f) {
            const int rb = f * (WN * 32) + wn * 32;
            if (B_KC) {
                const int row = rb + (lane & 31);
                b_off[f] = row * 64 + (((lane >> 5) ^ ((row >> 2) & 3)) << 4);
            } else {
                const int col = rb + (q & 1) * 16 + (i16 & 3) * 4;
                const int kr = (q >> 1) * 8 + (i16 >> 2);
                b_off[f] = kr * 512 + (((col >> 3) ^ (4 * (i16 >> 2))) << 4) + (col & 7) * 2;
            }
        }
    }
    // 8 consecutive k of one row (K-contiguous stage) ...
    auto frag_kc = [](const char *opnd, int off, int ks) { return *(const bf16x8 *)(opnd + (off ^ (ks << 5))); };
    // ... or the same 8 k of one column through two transposing reads of 4 K-rows x 16 columns
    auto frag_mc = [](const char *opnd, int off, int ks) {
        typedef s16x4 __attribute__((address_space(3))) * lp;
        const char *q = opnd + off + ks * 16 * 512;
        union {
            s16x4 h[2];
            bf16x8 v;
        } u;
        u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lp)(q));
        u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lp)(q + 4 * 512));
        return u.v;
    };

    // at most 4*(PF-1) direct loads stay in flight past this point
    auto wait_loads_and_barrier = [](bool lds_too) {
        static_assert(PF == 2 || PF == 3 || PF == 4, "vmcnt immediates below");
#ifdef PP_NO_GLOBAL
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
#else
        if (PF == 2) asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        if (PF == 3) asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        if (PF == 4) asm volatile("s_waitcnt vmcnt(12) lgkmcnt(0)\n\ts_barrier" ::: "memory");
#endif
        (void)lds_too;
    };

    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                acc[i][j][v] = 0.0f;

    // ---- prologue: three sub-tiles in flight, the first one landed -------------------
#pragma unroll
    for (int i = 0; i < PF; ++i) issue(i);
    wait_loads_and_barrier(false);
    if (group == 1) asm volatile("s_barrier" ::: "memory"); // start one slot late

    bf16x8 af[2][FM], bf[2][FN];
    for (int kt = 0; kt < KT; ++kt) {
        // ---- memory slot ---------------------------------------------------------------
        const char *sa = smem + (kt % STAGES) * STAGE;
        const char *sb = sa + OPND;
#ifdef PP_NO_LDSREAD
        if (kt == 0)
#endif
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
            for (int f = 0; f < FM; ++f) af[ks][f] = A_KC ? frag_kc(sa, a_off[f], ks) : frag_mc(sa, a_off[f], ks);
#pragma unroll
            for (int f = 0; f < FN; ++f) bf[ks][f] = B_KC ? frag_kc(sb, b_off[f], ks) : frag_mc(sb, b_off[f], ks);
        }
#ifndef PP_NO_GLOBAL
        issue(kt + PF);
#endif
        // own loads of sub-tile kt+1 have landed (the 4*(PF-1) newer ones may still fly), fragments are in registers
        wait_loads_and_barrier(true);
        __builtin_amdgcn_sched_barrier(0); // nothing may drift across a slot boundary
        // ---- compute slot ----------------------------------------------------------------
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks][i], bf[ks][j], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_s_setprio(0);
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_barrier" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
    }
    if (group == 0) asm volatile("s_barrier" ::: "memory"); // every wave passes the same number of barriers
    // the refetches past the end may still be landing in LDS: drain everybody's before LDS is reused
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");

    if (vec_epilogue)
        gemm_epilogue_staged<FM, FN, WN * 32>(p, acc, (float *)(smem + wave * EPI_LDS_BYTES_PER_WAVE),
                                              m0 + wm * (BM / WM), n0, wn * 32, lane);
    else
        gemm_epilogue<FM, FN, WN * 32>(p, acc, m0 + wm * (BM / WM) + 4 * (lane >> 5), n0, wn * 32 + (lane & 31));
}

bool gemm_bf16_pp_supported(int layout, const GemmArgs &a)
{
    if (a.K < 32 || (a.K & 31)) return false;
    if (layout == LAY_TN && a.M < 8) return false;
    if (layout != LAY_NT && a.N < 8) return false;
    return true;
}

hipError_t launch_gemm_bf16_pp(int layout, const GemmArgs &a, hipStream_t s)
{
    using namespace pp;
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    if (!gemm_bf16_pp_supported(layout, a)) return hipErrorInvalidValue;
    const int ncols = a.epi == EPI_SWIGLU_FWD ? a.half : a.N;
    const int bn = a.epi == EPI_SWIGLU_FWD ? BN / 2 : BN;
    const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (ncols + bn - 1) / bn;
    const dim3 grid((unsigned)(tiles_m * tiles_n)), block(NTHR);
    const int vec = gemm_epilogue_vec_ok(a) ? 1 : 0;
    switch (layout) {
    case LAY_NT: hipLaunchKernelGGL(gemm_bf16_pp_kernel<LAY_NT>, grid, block, 0, s, a, tiles_m, tiles_n, vec); break;
    case LAY_NN: hipLaunchKernelGGL(gemm_bf16_pp_kernel<LAY_NN>, grid, block, 0, s, a, tiles_m, tiles_n, vec); break;
    case LAY_TN: hipLaunchKernelGGL(gemm_bf16_pp_kernel<LAY_TN>, grid, block, 0, s, a, tiles_m, tiles_n, vec); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

} // namespace rtp
