// bf16 GEMM tiles for gfx950 (MI355X): the partition GEMM that an RTP worker
// runs N times per pass (Analysis section, computational-efficiency equation:
// N x Kernel(B/N, I, O/N)), in the three operand layouts the forward, the
// input gradient and the weight gradient need.
//
//   NT  C[M,N] = A[M,K] B[N,K]^T     forward            Y_k  = X W_k^T
//   NN  C[M,N] = A[M,K] B[K,N]       input gradient     dX  += dY_k W_k
//   TN  C[M,N] = A[K,M]^T B[K,N]     weight gradient    G_k += dY_k^T X
//
// One workgroup owns a BM x BN tile of C.  Operand tiles of BK = 64 are
// brought HBM -> registers -> LDS with 16-byte accesses, double buffered in
// LDS; waves read MFMA fragments back with ds_read_b128 when the operand is
// contiguous along K, and with the transposing ds_read_b64_tr_b16 when it is
// contiguous along M or N, so no operand is ever transposed in HBM.  The
// accumulators stay in registers (v_mfma_f32_32x32x16_bf16, fp32) and the
// epilogue writes straight into the column slice / accumulator the step
// targets, which is how the paper's concat and add layers disappear.
#include "rtp_gemm_epilogue.h"

namespace rtp {

constexpr int BK = 64;      // K extent of one LDS stage
constexpr int MC_PAD = 32;  // elements of padding per K-row of an M/N-contiguous tile:
                            // 64 bytes, so that the 4 K-rows x 2 column groups one
                            // transposing read touches cover all 64 banks once
                            // (row length mod 256 bytes must be 64 or 192)

// ---- tile geometry ----------------------------------------------------------
template <int BM, int BN, int WM, int WN, int LAY>
struct Cfg {
    static constexpr int NTHR = WM * WN * 64;
    static constexpr bool A_KC = (LAY != LAY_TN); // A contiguous along K
    static constexpr bool B_KC = (LAY == LAY_NT);
    static constexpr int A_LD = BM + MC_PAD;      // row length of an M-contiguous A stage
    static constexpr int B_LD = BN + MC_PAD;
    static constexpr int A_BYTES = A_KC ? BM * BK * 2 : BK * A_LD * 2;
    static constexpr int B_BYTES = B_KC ? BN * BK * 2 : BK * B_LD * 2;
    static constexpr int STAGE = A_BYTES + B_BYTES;
    static constexpr int FM = BM / (WM * 32);     // 32x32 fragments per wave
    static constexpr int FN = BN / (WN * 32);
    static constexpr int A_CH = (BM * BK / 8) / NTHR; // 16-byte chunks per thread and stage
    static constexpr int B_CH = (BN * BK / 8) / NTHR;
    static_assert(FM >= 1 && FN >= 1 && A_CH >= 1 && B_CH >= 1, "tile too small for the wave grid");
    static_assert(FN % 2 == 0 || LAY != LAY_NT, "paired epilogue needs an even fragment count");
    static_assert(2 * STAGE <= 160 * 1024, "two stages must fit the 160 KB LDS");
    static_assert((A_LD * 2) % 128 == 64 && (B_LD * 2) % 128 == 64, "padded rows must shift by half the bank space");
};

// One operand's HBM -> LDS path for a stage.  R = rows (K-contiguous) or
// columns (M/N-contiguous) of the tile, CH chunks per thread.
template <int R, int CH, int NTHR, bool KC>
struct Loader {
    const char *gp[CH]; // byte address of this thread's chunk in K-tile 0
    int lds_off[CH];
    int kpos[CH];       // K index of the chunk inside a K-tile (for the tail predicate)
    int64_t kstep;      // bytes to advance per K-tile
    u32x4 reg[CH];

    // rowmap(local) -> global row/col index, already clamped into range
    template <class RowMap>
    __device__ __forceinline__ void init(const void *base, int64_t ld, int tid, RowMap rowmap)
    {
        constexpr int LD_MC = R + MC_PAD;
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int c = tid + NTHR * i;
            if (KC) {
                const int row = c >> 3, kc = c & 7;
                gp[i] = (const char *)base + ((int64_t)rowmap(row) * ld + kc * 8) * 2;
                lds_off[i] = row * 128 + ((kc ^ ((row >> 1) & 7)) << 4);
                kpos[i] = kc * 8;
            } else {
                constexpr int CPR = R / 8; // chunks per K-row
                const int k = c / CPR, mc = c % CPR;
                // a chunk is 8 consecutive rows/cols; rowmap clamps its first one
                gp[i] = (const char *)base + ((int64_t)k * ld + rowmap(mc * 8)) * 2;
                lds_off[i] = (k * LD_MC + mc * 8) * 2;
                kpos[i] = k;
            }
        }
        kstep = KC ? (int64_t)BK * 2 : (int64_t)BK * ld * 2;
    }

    __device__ __forceinline__ void load(int kt)
    {
#pragma unroll
        for (int i = 0; i < CH; ++i)
            reg[i] = *(const u32x4 *)(gp[i] + kt * kstep);
    }
    // last K-tile: chunks past K read as zero
    __device__ __forceinline__ void load_tail(int kt, int K)
    {
        const int k0 = kt * BK;
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            u32x4 z = {0u, 0u, 0u, 0u};
            if (k0 + kpos[i] < K)
                z = *(const u32x4 *)(gp[i] + kt * kstep);
            reg[i] = z;
        }
    }
    __device__ __forceinline__ void store(char *stage)
    {
#pragma unroll
        for (int i = 0; i < CH; ++i)
            *(u32x4 *)(stage + lds_off[i]) = reg[i];
    }
};

// Fragment of a K-contiguous stage: 8 consecutive k of one row per lane.  A
// row is 128 bytes (8 chunks of 16); chunk c of row r sits at chunk slot
// c ^ ((r >> 1) & 7), which spreads the 32 rows one ds_read_b128 touches over
// all 64 banks.  base_off already holds the slot of K-step 0; K-step ks
// flips chunk bits 1..2.
__device__ __forceinline__ bf16x8 frag_kc(const char *stage, int base_off, int ks)
{
    return *(const bf16x8 *)(stage + (base_off ^ (ks << 5)));
}

// Fragment of an M/N-contiguous stage through the transposing LDS read.
// Within a group of 16 lanes the read takes 4 K-rows x 16 columns (each lane
// supplies the address of 4 consecutive columns of one K-row) and hands lane
// i the 4 K values of column i.
__device__ __forceinline__ bf16x8 frag_mc(const char *stage, int addr_lo, int ld_bytes, int ks)
{
    typedef s16x4 __attribute__((address_space(3))) * lds_p;
    const char *p = stage + addr_lo + ks * 16 * ld_bytes;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(p + 4 * ld_bytes));
    union {
        s16x4 h[2];
        bf16x8 v;
    } u;
    u.h[0] = lo;
    u.h[1] = hi;
    return u.v;
}

template <int BM, int BN, int WM, int WN, int LAY>
__global__ __launch_bounds__(WM *WN * 64) void gemm_bf16_kernel(const GemmArgs p, const int tiles_m,
                                                                 const int tiles_n)
{
    using C = Cfg<BM, BN, WM, WN, LAY>;
    __shared__ __attribute__((aligned(16))) char smem[2 * C::STAGE];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    // ---- which tile: spread neighbouring tiles over one XCD's L2 -----------
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
    const int group = pid / group_sz;
    const int first_m = group * GROUP_M;
    const int gm = min(tiles_m - first_m, GROUP_M);
    const int tm = first_m + (pid % group_sz) % gm;
    const int tn = (pid % group_sz) / gm;

    const bool paired = (p.epi == EPI_SWIGLU_FWD);
    const int m0 = tm * BM;
    const int n0 = paired ? tn * (BN / 2) : tn * BN;
    const int M = p.M, N = p.N, K = p.K;

    // ---- loaders --------------------------------------------------------------
    Loader<BM, C::A_CH, C::NTHR, C::A_KC> la;
    Loader<BN, C::B_CH, C::NTHR, C::B_KC> lb;
    if (C::A_KC)
        la.init(p.A, p.lda, tid, [&](int r) { return min(m0 + r, M - 1); });
    else
        la.init(p.A, p.lda, tid, [&](int c) { return min(m0 + c, M - 8); });
    if (C::B_KC) {
        if (paired) {
            const int half = p.half;
            lb.init(p.B, p.ldb, tid, [&](int r) {
                return r < BN / 2 ? min(n0 + r, half - 1) : half + min(n0 + r - BN / 2, half - 1);
            });
        } else {
            lb.init(p.B, p.ldb, tid, [&](int r) { return min(n0 + r, N - 1); });
        }
    } else {
        lb.init(p.B, p.ldb, tid, [&](int c) { return min(n0 + c, N - 8); });
    }

    // ---- fragment addresses -----------------------------------------------------
    int a_off[C::FM], b_off[C::FN];
#pragma unroll
    for (int f = 0; f < C::FM; ++f) {
        const int rb = wm * (BM / WM) + f * 32;
        if (C::A_KC) {
            const int row = rb + (lane & 31);
            a_off[f] = row * 128 + ((((lane >> 5)) ^ ((row >> 1) & 7)) << 4);
        } else {
            const int q = lane >> 4, i = lane & 15;
            const int col = rb + (q & 1) * 16 + (i & 3) * 4;
            const int krow = (q >> 1) * 8 + (i >> 2);
            a_off[f] = (krow * C::A_LD + col) * 2;
        }
    }
#pragma unroll
    for (int f = 0; f < C::FN; ++f) {
        const int rb = f * (WN * 32) + wn * 32;
        if (C::B_KC) {
            const int row = rb + (lane & 31);
            b_off[f] = row * 128 + ((((lane >> 5)) ^ ((row >> 1) & 7)) << 4);
        } else {
            const int q = lane >> 4, i = lane & 15;
            const int col = rb + (q & 1) * 16 + (i & 3) * 4;
            const int krow = (q >> 1) * 8 + (i >> 2);
            b_off[f] = (krow * C::B_LD + col) * 2;
        }
    }

    f32x16 acc[C::FM][C::FN];
#pragma unroll
    for (int i = 0; i < C::FM; ++i)
#pragma unroll
        for (int j = 0; j < C::FN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                acc[i][j][v] = 0.0f;

    const int KT = (K + BK - 1) / BK;

    // ---- prologue ---------------------------------------------------------------
    if (KT == 1) {
        la.load_tail(0, K);
        lb.load_tail(0, K);
    } else {
        la.load(0);
        lb.load(0);
    }
    la.store(smem);
    lb.store(smem + C::A_BYTES);
    __syncthreads();

    // ---- main loop ----------------------------------------------------------------
    for (int kt = 0; kt < KT; ++kt) {
        char *cur = smem + (kt & 1) * C::STAGE;
        char *nxt = smem + ((kt & 1) ^ 1) * C::STAGE;
        const bool more = kt + 1 < KT;
        if (more) {
            if (kt + 2 == KT) {
                la.load_tail(kt + 1, K);
                lb.load_tail(kt + 1, K);
            } else {
                la.load(kt + 1);
                lb.load(kt + 1);
            }
        }
        const char *sa = cur;
        const char *sb = cur + C::A_BYTES;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 af[C::FM], bf[C::FN];
#pragma unroll
            for (int f = 0; f < C::FM; ++f)
                af[f] = C::A_KC ? frag_kc(sa, a_off[f], ks) : frag_mc(sa, a_off[f], C::A_LD * 2, ks);
#pragma unroll
            for (int f = 0; f < C::FN; ++f)
                bf[f] = C::B_KC ? frag_kc(sb, b_off[f], ks) : frag_mc(sb, b_off[f], C::B_LD * 2, ks);
#pragma unroll
            for (int i = 0; i < C::FM; ++i)
#pragma unroll
                for (int j = 0; j < C::FN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
        if (more) {
            la.store(nxt);
            lb.store(nxt + C::A_BYTES);
        }
        __syncthreads();
    }

    // ---- epilogue -------------------------------------------------------------------
    gemm_epilogue<__bf16, C::FM, C::FN, WN * 32>(p, acc, m0 + wm * (BM / WM) + 4 * (lane >> 5), n0, wn * 32 + (lane & 31));
}

// ---- host side ------------------------------------------------------------------------

struct Variant {
    int bm, bn, wm, wn;
    const char *name[3];
};

// variant 1: 256x256 tile, 8 waves (2 per SIMD); variant 2: 128x128 tile, 4 waves.
static const Variant kVariants[] = {
    {0, 0, 0, 0, {"", "", ""}},
    {256, 256, 2, 4, {"gemm_bf16_256x256_nt", "gemm_bf16_256x256_nn", "gemm_bf16_256x256_tn"}},
    {128, 128, 2, 2, {"gemm_bf16_128x128_nt", "gemm_bf16_128x128_nn", "gemm_bf16_128x128_tn"}},
    {256, 256, 2, 2, {"gemm_bf16_256x256w4_nt", "gemm_bf16_256x256w4_nn", "gemm_bf16_256x256w4_tn"}},
    {256, 256, 2, 4, {"gemm_pp_kernel<0, __bf16>", "gemm_pp_kernel<1, __bf16>", "gemm_pp_kernel<2, __bf16>"}},
    {256, 256, 2, 4, {"gemm_pp_kernel<0, __bf16>", "gemm_pp_kernel<1, __bf16>", "gemm_pp_kernel<2, __bf16>"}},
    {192, 256, 2, 4, {"gemm_pp_kernel<0, __bf16>", "gemm_pp_kernel<1, __bf16>", "gemm_pp_kernel<2, __bf16>"}},
    {128, 256, 2, 4, {"gemm_pp_kernel<0, __bf16>", "gemm_pp_kernel<1, __bf16>", "gemm_pp_kernel<2, __bf16>"}},
};
constexpr int kNumVariants = 7;

const char *gemm_bf16_kernel_name(int layout, int variant)
{
    if (layout < 0 || layout > 2 || variant < 1 || variant > kNumVariants) return "";
    return kVariants[variant].name[layout];
}

static int pick_variant(int layout, const GemmArgs &a)
{
    if (a.elem != ELEM_BF16) return 4; // fp16 inputs: only the tiled kernel is built
    // the ping-pong kernel whenever its shape rules hold and there is at least a tile's worth of work
    if (gemm_bf16_pp_supported(layout, a) && a.M >= 64 && a.N >= 64) return 4;
    // the large tile when it yields at least ~one workgroup per CU, else the small one
    const int ncols = a.epi == EPI_SWIGLU_FWD ? a.half : a.N;
    const int bn = a.epi == EPI_SWIGLU_FWD ? 128 : 256;
    const long big = (long)((a.M + 255) / 256) * ((ncols + bn - 1) / bn);
    return big >= 160 ? 1 : 2;
}

template <int BM, int BN, int WM, int WN>
static hipError_t launch_cfg(int layout, const GemmArgs &a, hipStream_t s)
{
    const int ncols = a.epi == EPI_SWIGLU_FWD ? a.half : a.N;
    const int bn = a.epi == EPI_SWIGLU_FWD ? BN / 2 : BN;
    const int tiles_m = (a.M + BM - 1) / BM;
    const int tiles_n = (ncols + bn - 1) / bn;
    const dim3 grid((unsigned)(tiles_m * tiles_n)), block(WM * WN * 64);
    if (tiles_m <= 0 || tiles_n <= 0) return hipSuccess;
    switch (layout) {
    case LAY_NT:
        hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, LAY_NT>), grid, block, 0, s, a, tiles_m, tiles_n);
        break;
    case LAY_NN:
        hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, LAY_NN>), grid, block, 0, s, a, tiles_m, tiles_n);
        break;
    case LAY_TN:
        hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, LAY_TN>), grid, block, 0, s, a, tiles_m, tiles_n);
        break;
    default:
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// what the kernels' clamped, 16-byte loads assume
bool gemm_bf16_args_ok(int layout, const GemmArgs &a)
{
    if (layout < LAY_NT || layout > LAY_TN) return false;
    if (a.K <= 0 || (a.lda & 7) || (a.ldb & 7) || ((uintptr_t)a.A & 15) || ((uintptr_t)a.B & 15)) return false;
    if (layout != LAY_TN && (a.K & 7)) return false; // A rows are read in 8-element chunks of K
    if (layout == LAY_TN && ((a.M & 7) || a.M < 8)) return false;
    if (layout != LAY_NT && ((a.N & 7) || a.N < 8)) return false;
    if (a.epi == EPI_SWIGLU_FWD && (layout != LAY_NT || a.half * 2 != a.N)) return false;
    return true;
}

hipError_t launch_gemm_bf16(int layout, const GemmArgs &a, int variant, hipStream_t s)
{
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    if (!gemm_bf16_args_ok(layout, a)) return hipErrorInvalidValue;
    if (variant == 0) variant = pick_variant(layout, a);
    if (a.elem != ELEM_BF16 && (variant < 4 || variant > 7)) return hipErrorInvalidValue; // fp16: tiled kernel only
    if (variant >= 4 && variant <= 7) {
        if (!gemm_bf16_pp_supported(layout, a)) return hipErrorInvalidValue;
        const int bm[4] = {0, 256, 192, 128};
        return launch_gemm_bf16_pp(layout, a, bm[variant - 4], s);
    }
    switch (variant) {
    case 1:
        return launch_cfg<256, 256, 2, 4>(layout, a, s);
    case 2:
        return launch_cfg<128, 128, 2, 2>(layout, a, s);
    case 3:
        return launch_cfg<256, 256, 2, 2>(layout, a, s);
    default:
        return hipErrorInvalidValue;
    }
}

} // namespace rtp
