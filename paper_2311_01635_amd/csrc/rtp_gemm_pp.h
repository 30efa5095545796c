// bf16 / fp16 partition GEMM for gfx950, "ping-pong" form: the kernel the rotated
// linear layer uses whenever the contraction length is a multiple of 32.
// (Template; instantiated per operand layout in rtp_gemm_pp_<layout>.hip.)
//
// One workgroup of 8 waves owns a BM x 256 tile of C, BM = 256, 192 or 128
// (wave tile BM/2 x 64, 32x32x16 bf16 MFMA, fp32 accumulators in registers).
// K advances in sub-tiles of 32 through a ring of four LDS stages
// (96 to 128 KB of the 160 KB LDS).
//
//  * HBM -> LDS goes through the direct load (buffer_load_dwordx4 ... lds): no
//    staging registers and no ds_write; three sub-tiles are always in flight.
//    Buffer addressing (descriptor + 32-bit lane offset + scalar K offset)
//    keeps vector address arithmetic out of the loop.
//  * The two waves that share a SIMD run half an iteration apart.  Every
//    iteration of a wave is a "memory" slot (read the MFMA fragments of the
//    sub-tile out of LDS, issue the loads for the far end of the ring) and a
//    "compute" slot (the MFMAs, back to back), and a workgroup barrier ends
//    each slot.  Because one group of four waves starts one slot late, one
//    wave of every SIMD is always in its compute slot while the other is in
//    its memory slot, so the LDS pipeline and the MFMA pipeline stay busy at
//    the same time instead of taking turns.
//  * LDS layouts are chosen so that every fragment read is bank-conflict
//    free on the 64-bank LDS: operands contiguous along K are stored as
//    64-byte rows with the 16-byte chunk index xor-ed with (row/4)%4;
//    operands contiguous along M or N are stored as K-rows of the tile's
//    width with the chunk index xor-ed with (or, for 384-byte rows, rotated
//    by) 4*(k%4) and read back with the transposing ds_read_b64_tr_b16.  The
//    direct load writes 64 lanes x 16 bytes to consecutive LDS addresses, so
//    the permutation is applied on the global address each lane fetches.
//  * Why three tile heights: a shard GEMM rarely yields a multiple of 256
//    tiles at 256 x 256 (176 or 96 on the Llama-shaped unit), which would
//    leave a third to two thirds of the compute units idle -- the occupancy
//    loss the paper's Analysis section predicts for N small kernels.  A
//    shorter tile that fills the machine in one round wins; the launcher
//    picks the height with the smallest (rounds x height) product.
//    (Splitting tiles along K over all compute units, "stream-K", was built
//    and measured slower: workgroups at different K offsets stop sharing
//    operand panels in L2, the hit rate fell from 86 % to 43 %.)
//
//  * One launch can carry up to four GEMMs of the same operand layout (a
//    "group"): the tiles of all of them form one grid, longest tiles first,
//    each XCD owning an eighth of every problem.  GEMMs of a rotation step
//    that do not depend on each other can be launched this way, so a problem
//    with few tiles fills the compute units another one leaves idle and the
//    epilogue of one tile overlaps the main loop of another.
//
// Layouts and epilogues are those of rtp_gemm_bf16.hip; ragged M and N are
// handled by clamping the fetched row/column (the clamped results are never
// stored), K must be a multiple of 32.
#pragma once
#include "rtp_gemm_epilogue.h"
#include <type_traits>
#include <hip/hip_ext.h>

namespace rtp {

namespace pp {
constexpr int BN = 256, BK = 32;
constexpr int WM = 2, WN = 4, NTHR = 512;
constexpr int FN = BN / (WN * 32);   // 2 fragments of 32 columns per wave
constexpr int B_BYTES = BN * BK * 2; // 16 KB of B per stage
constexpr int STAGES = 4; // deeper rings (5 or 6 stages fit the 160 KB LDS) measured no faster
constexpr int RING_BYTES = STAGES * (256 * BK * 2 + B_BYTES); // the tallest tile's ring: 128 KB
// the epilogue reuses the ring: per wave, one parked fragment row and the landing area of its fp32 reads (136 KB)
constexpr int EPI_BYTES = NTHR / 64 * (EPI_LDS_BYTES_PER_WAVE + EPI_LAND_BYTES_PER_WAVE);
constexpr int SMEM_BYTES = RING_BYTES > EPI_BYTES ? RING_BYTES : EPI_BYTES;
static_assert(SMEM_BYTES <= 160 * 1024, "one workgroup per compute unit: 160 KB of LDS");
typedef __attribute__((address_space(3))) void *lds_vp;
// fourth word of a raw buffer descriptor on gfx9-family parts: 32-bit data format, no swizzle, no stride
constexpr int BUFFER_RSRC_FLAGS = 0x00020000;
} // namespace pp

// One GEMM of a group launch and the whole group (a kernel argument, passed by value).
struct PpProblem {
    GemmArgs a;
    int bm;               // tile height: 256, 192 or 128
    int tiles_m, tiles_n;
    int vec_epilogue;
    int ksplit;           // > 1: the K loop is cut into this many chunks, one workgroup each, whose partial
                          // sums meet in the fp32 accumulator through atomic adds (a.epi == EPI_ACC_ATOMIC)
};
struct PpGroup {
    int count;
    PpProblem p[PP_MAX_GROUP];
};

// The transposing fragment read, issued as an instruction of our own.  Through the builtin the compiler puts a
// wait for ALL outstanding direct loads in front of these reads (it cannot tell that the LDS stage being read is
// not the one a load in flight is writing), which empties the ring of sub-tiles in flight at every slot; the slot
// ends with an explicit wait for the stage that is read next, and that wait is the one that is needed.
// addr: LDS byte address; OFF: immediate byte offset.
template <int OFF> __device__ __forceinline__ s16x4 ds_read_tr16_b64(unsigned addr)
{
    s16x4 v;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}
// 8 consecutive k (sub-tile half KS) of one column of an M- or N-contiguous stage with K-rows of ROWB bytes:
// two transposing reads of 4 K-rows x 16 columns (K-rows 16*KS + 8*(lane/32) + 0..3 and + 4..7)
template <typename V8, int KS, int ROWB> __device__ __forceinline__ V8 frag_mc_read(unsigned addr)
{
    union {
        s16x4 h[2];
        V8 v;
    } u;
    u.h[0] = ds_read_tr16_b64<KS * 16 * ROWB>(addr);
    u.h[1] = ds_read_tr16_b64<KS * 16 * ROWB + 4 * ROWB>(addr);
    return u.v;
}

// One BM x 256 tile over the K sub-tiles [kt_begin, kt_begin + kt_count): `pid` is the tile's index inside its
// problem, `smem` the workgroup's LDS.
template <int LAY, int BM, typename E>
__device__ __forceinline__ void pp_tile(const GemmArgs &p, const int tiles_m, const int tiles_n, const int vec_epilogue,
                                        const int pid, const int kt_begin, const int kt_count, char *smem)
{
    using namespace pp;
    typedef typename ElemVec<E>::v8 frag8; // eight K-consecutive elements of an operand: one lane's share of an MFMA input
    static_assert(BM == 256 || BM == 192 || BM == 128, "tile heights built");
    constexpr bool A_KC = (LAY != LAY_TN), B_KC = (LAY == LAY_NT);
    constexpr int FM = BM / (WM * 32);       // 4, 3 or 2 fragments of 32 rows per wave
    constexpr int A_BYTES = BM * BK * 2;     // 16, 12 or 8 KB of A per stage
    constexpr int STAGE = A_BYTES + B_BYTES;
    constexpr int PF = STAGES - 1;               // sub-tiles in flight
    constexpr int A_PIECES = A_BYTES / 1024; // 1 KB direct-load pieces of A per stage: 16, 12, 8
    constexpr int A_PW = (A_PIECES + 7) / 8; // ... per wave (the second one only on waves 0-3 when BM = 192)
    constexpr int A_CPR = BM / 8;            // 16-byte chunks per K-row of an M-contiguous A stage
    constexpr int A_ROWB = BM * 2;           // bytes per K-row of an M-contiguous A stage
    static_assert(STAGES * STAGE <= SMEM_BYTES, "ring fits the workgroup's LDS");

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    // the wave index as a scalar: everything derived from it (LDS destinations of the direct loads, hence the
    // M0 values; which pieces a wave fetches) then stays in scalar registers instead of costing vector
    // instructions and readfirstlanes in the loop
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int group = wave >> 2; // waves 0-3 and 4-7 sit on SIMDs 0-3 respectively

    // ---- which tile: consecutive tile indices walk 4-tall column strips, so an XCD's contiguous
    // run of indices is a compact block of tiles that share operand panels in its L2
    constexpr int GROUP_M = 4;
    const int group_sz = GROUP_M * tiles_n;
    const int grp = pid / group_sz;
    const int first_m = grp * GROUP_M;
    const int gm = min(tiles_m - first_m, GROUP_M);
    const int tm = first_m + (pid % group_sz) % gm;
    const int tn = (pid % group_sz) / gm;

    const bool paired = (p.epi == EPI_SWIGLU_FWD);
    const int m0 = tm * BM;
    const int sync_b0 = m0 / SYNC_ROWS, sync_b1 = (min(m0 + BM, p.M) + SYNC_ROWS - 1) / SYNC_ROWS; // row blocks of this tile

    // ---- consumer of another problem of this launch: wait until its producer tiles are done.  The producer's
    // workgroups precede this one in dispatch order, so they are running or finished; the wait is bounded all
    // the same, and a tile that gives up says so in the error word instead of hanging the launch.
    if (p.sync_wait > 0) {
        if (tid == 0) {
            const int blocks_total = (p.M + SYNC_ROWS - 1) / SYNC_ROWS;
            for (int b = sync_b0; b < sync_b1; ++b) {
                int spins = 0;
                while (__hip_atomic_load(p.sync + b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < p.sync_wait) {
                    __builtin_amdgcn_s_sleep(8);
                    if (++spins > (1 << 21)) {
                        __hip_atomic_store(p.sync + blocks_total, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        break;
                    }
                }
            }
        }
        __syncthreads();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent"); // what the producers stored is read from memory, not from a stale line
    }
    const int n0 = paired ? tn * (BN / 2) : tn * BN;
    const int M = p.M, N = p.N, K = p.K;
    const int half = p.half;

    // chunk permutation of an M-contiguous A stage: slot of logical chunk c in K-row kr
    auto a_slot = [](int c, int kr) { return BM == 192 ? (c + 4 * (kr & 3)) % A_CPR : c ^ (4 * (kr & 3)); };
    auto a_unslot = [](int pc, int kr) { return BM == 192 ? (pc + A_CPR - 4 * (kr & 3)) % A_CPR : pc ^ (4 * (kr & 3)); };

    // ---- direct-load addresses --------------------------------------------------------
    // A: piece j (1 KB) of a K-contiguous stage holds rows 16j..16j+15 (64 bytes each); of an
    //    M-contiguous stage it holds chunks 64j..64j+63 of the K-rows laid end to end.  Wave w
    //    fetches pieces w and w + 8.
    // B: pieces 2w and 2w + 1, rows 16j.. or K-rows 2j, 2j+1 (512 bytes each).
    auto a_row = [&](int r) { return min(m0 + r, M - 1); };
    auto a_col = [&](int c) { return min(m0 + c, M - 8); };
    auto b_row = [&](int r) {
        if (paired) return r < BN / 2 ? min(n0 + r, half - 1) : half + min(n0 + r - BN / 2, half - 1);
        return min(n0 + r, N - 1);
    };
    auto b_col = [&](int c) { return min(n0 + c, N - 8); };

    // Each operand is read through a buffer descriptor (base + byte range) with a 32-bit offset per lane and
    // the K advance in a scalar offset: the loop then holds no vector address arithmetic at all.  (With 64-bit
    // global addresses every load cost two vector adds in the memory slot, and vector instructions of one wave
    // take issue slots from the MFMAs of the other wave on the same SIMD: the same kernel ran 20-25 % slower.)
    unsigned oa[A_PW], ob[2];
    const int a_pieces_mine = (A_PIECES - wave + 7) / 8; // 2, or 1 on waves 4-7 when BM = 192, or 1 when BM = 128
#pragma unroll
    for (int i = 0; i < A_PW; ++i) {
        const int j = min(wave + 8 * i, A_PIECES - 1);
        if (A_KC) {
            const int row = 16 * j + (lane >> 2), pc = lane & 3, c = pc ^ ((row >> 2) & 3);
            oa[i] = (unsigned)(((int64_t)a_row(row) * p.lda + c * 8) * 2);
        } else {
            const int L = 64 * j + lane, kr = L / A_CPR, c = a_unslot(L % A_CPR, kr);
            oa[i] = (unsigned)(((int64_t)kr * p.lda + a_col(c * 8)) * 2);
        }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int j = 2 * wave + i;
        if (B_KC) {
            const int row = 16 * j + (lane >> 2), pc = lane & 3, c = pc ^ ((row >> 2) & 3);
            ob[i] = (unsigned)(((int64_t)b_row(row) * p.ldb + c * 8) * 2);
        } else {
            const int kr = 2 * j + (lane >> 5), pc = lane & 31, c = pc ^ (4 * (kr & 3));
            ob[i] = (unsigned)(((int64_t)kr * p.ldb + b_col(c * 8)) * 2);
        }
    }
    // byte ranges of the operands (the launcher has checked that they stay below 2^31: 32-bit scalar arithmetic,
    // so that the descriptors live in scalar registers; a 64-bit product would be computed on the vector unit and
    // every load would then run inside a loop that re-reads the descriptor lane by lane)
    const unsigned a_bytes = __builtin_amdgcn_readfirstlane(((unsigned)((A_KC ? M : K) - 1) * (unsigned)p.lda + (unsigned)(A_KC ? K : M)) * 2u);
    const unsigned b_bytes = __builtin_amdgcn_readfirstlane(((unsigned)((B_KC ? N : K) - 1) * (unsigned)p.ldb + (unsigned)(B_KC ? K : N)) * 2u);
    const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc((void *)p.A, 0, a_bytes, BUFFER_RSRC_FLAGS);
    const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc((void *)p.B, 0, b_bytes, BUFFER_RSRC_FLAGS);
    const int stepA = A_KC ? BK * 2 : (int)(BK * p.lda * 2);
    const int stepB = B_KC ? BK * 2 : (int)(BK * p.ldb * 2);
    const int KT = kt_count;

    auto issue = [&](int kt) {
        const int kk = kt_begin + min(kt, KT - 1); // past the end: refetch the last sub-tile into a stage nobody reads
        char *st = smem + (kt % STAGES) * STAGE;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, (lds_vp)(st + wave * 1024), 16, oa[0], kk * stepA, 0, 0);
        if (A_PW == 2 && a_pieces_mine == 2)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, (lds_vp)(st + (wave + 8) * 1024), 16, oa[A_PW - 1], kk * stepA, 0, 0);
#pragma unroll
        for (int i = 0; i < 2; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, (lds_vp)(st + A_BYTES + (2 * wave + i) * 1024), 16, ob[i], kk * stepB, 0, 0);
    };
    // ends a slot: all but this wave's PF-1 newest sub-tiles of direct loads have landed, its LDS
    // reads have returned, and everybody is here
    auto end_slot_after_loads = [&]() {
        if (a_pieces_mine == 2)
            asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"((PF - 1) * 4) : "memory"); // 4 loads per sub-tile
        else
            asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"((PF - 1) * 3) : "memory"); // 3 loads per sub-tile
    };
    static_assert(PF >= 2 && (PF - 1) * 4 < 64, "vmcnt is a 6-bit counter");

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
                a_off[f] = kr * A_ROWB + (a_slot(col >> 3, kr) << 4) + (col & 7) * 2;
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
    auto frag_kc = [](const char *opnd, int off, int ks) { return *(const frag8 *)(opnd + (off ^ (ks << 5))); };
    // ... or the same 8 k of one column through two transposing reads (frag_mc_read): the row index changes by
    // multiples of 4 between them, so the chunk permutation of the lane's row stays the one a_off / b_off were built with
    auto lds_addr = [](const char *q) { return (unsigned)(uintptr_t)(__attribute__((address_space(3))) const char *)q; };
    const unsigned smem_lds = lds_addr(smem); // the ring's LDS address, folded into the transposing reads' lane addresses once
    unsigned a_tr[FM], b_tr[FN];
#pragma unroll
    for (int f = 0; f < FM; ++f) a_tr[f] = smem_lds + (unsigned)a_off[f];
#pragma unroll
    for (int f = 0; f < FN; ++f) b_tr[f] = smem_lds + (unsigned)(A_BYTES + b_off[f]);

    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                acc[i][j][v] = 0.0f;

    // ---- prologue: PF sub-tiles in flight, the first one landed -------------------------
#pragma unroll
    for (int i = 0; i < PF; ++i) issue(i);
    end_slot_after_loads();
    if (group == 1) asm volatile("s_barrier" ::: "memory"); // start one slot late

    // ---- which of this wave's fragments hold anything: a tile on the matrix edge (N = 1376 is 5.4 tile columns)
    // has fragment rows / columns that lie wholly outside; their MFMAs and LDS reads are skipped.  On a part whose
    // clock follows the switching activity that is energy for the other tiles, and the edge tile itself ends sooner.
    // All of it is wave-uniform scalar state; interior waves run the loop without a single test.
    const int iv = max(0, min(FM, (M - (m0 + wm * (BM / WM)) + 31) / 32)); // valid fragment rows: 0 .. iv-1
    bool jv[FN];
#pragma unroll
    for (int j = 0; j < FN; ++j)
        jv[j] = paired ? (n0 + wn * 32 < half) : (n0 + j * (WN * 32) + wn * 32 < N);
    const bool interior = iv == FM && jv[0] && jv[FN - 1];

    frag8 af[2][FM], bf[2][FN];
    auto k_loop = [&](auto full_tag) {
        constexpr bool FULL = decltype(full_tag)::value;
        if (!FULL) {
            // fragments that are never read must still be defined where the compiler sees them used
#pragma unroll
            for (int f = 0; f < FM; ++f) af[0][f] = af[1][f] = frag8{};
#pragma unroll
            for (int f = 0; f < FN; ++f) bf[0][f] = bf[1][f] = frag8{};
        }
        for (int kt = 0; kt < KT; ++kt) {
            // ---- memory slot ------------------------------------------------------------------
            const unsigned stage_off = (unsigned)((kt % STAGES) * STAGE);
            const char *sa = smem + stage_off;
            const char *sb = sa + A_BYTES;
#pragma unroll
            for (int f = 0; f < FM; ++f) {
                if (!FULL && f >= iv) continue;
                if (A_KC) {
                    af[0][f] = frag_kc(sa, a_off[f], 0);
                    af[1][f] = frag_kc(sa, a_off[f], 1);
                } else {
                    af[0][f] = frag_mc_read<frag8, 0, A_ROWB>(a_tr[f] + stage_off);
                    af[1][f] = frag_mc_read<frag8, 1, A_ROWB>(a_tr[f] + stage_off);
                }
            }
#pragma unroll
            for (int f = 0; f < FN; ++f) {
                if (!FULL && !jv[f]) continue;
                if (B_KC) {
                    bf[0][f] = frag_kc(sb, b_off[f], 0);
                    bf[1][f] = frag_kc(sb, b_off[f], 1);
                } else {
                    bf[0][f] = frag_mc_read<frag8, 0, 512>(b_tr[f] + stage_off);
                    bf[1][f] = frag_mc_read<frag8, 1, 512>(b_tr[f] + stage_off);
                }
            }
            issue(kt + PF);
            // own loads of sub-tile kt+1 have landed, fragments are in registers
            end_slot_after_loads();
            __builtin_amdgcn_sched_barrier(0); // nothing may drift across a slot boundary
            // ---- compute slot -------------------------------------------------------------------
            __builtin_amdgcn_s_setprio(1);
            if (FULL) {
#pragma unroll
                for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                    for (int i = 0; i < FM; ++i)
#pragma unroll
                        for (int j = 0; j < FN; ++j)
                            acc[i][j] = mfma_32x32x16(af[ks][i], bf[ks][j], acc[i][j]);
            } else {
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    if (jv[j]) {
#pragma unroll
                        for (int i = 0; i < FM; ++i)
                            if (i < iv) {
                                acc[i][j] = mfma_32x32x16(af[0][i], bf[0][j], acc[i][j]);
                                acc[i][j] = mfma_32x32x16(af[1][i], bf[1][j], acc[i][j]);
                            }
                    }
            }
            __builtin_amdgcn_s_setprio(0);
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_barrier" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    if (interior)
        k_loop(std::true_type{});
    else
        k_loop(std::false_type{});
    if (group == 0) asm volatile("s_barrier" ::: "memory"); // every wave passes the same number of barriers
    // the refetches past the end may still be landing in LDS: drain everybody's before LDS is reused
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");

    if (vec_epilogue)
        gemm_epilogue_staged<E, FM, FN, WN * 32>(p, acc, (float *)(smem + wave * EPI_LDS_BYTES_PER_WAVE),
                                              m0 + wm * (BM / WM), n0, wn * 32, lane,
                                              smem + (pp::NTHR / 64) * EPI_LDS_BYTES_PER_WAVE + wave * EPI_LAND_BYTES_PER_WAVE);
    else
        gemm_epilogue<E, FM, FN, WN * 32>(p, acc, m0 + wm * (BM / WM) + 4 * (lane >> 5), n0, wn * 32 + (lane & 31));

    // ---- producer: the tile's results are visible device-wide before the counters say so
    if (p.sync_signal) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        __syncthreads();
        if (tid == 0)
            for (int b = sync_b0; b < sync_b1; ++b) __hip_atomic_fetch_add(p.sync + b, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// Workgroup ids are dealt round-robin to the 8 XCDs.  XCD x works through its own list: its
// contiguous eighth of problem 0's tiles, then of problem 1's, ...; workgroup 8 l + x takes entry l
// of that list (the host sizes the grid for the longest list; surplus workgroups leave at once).
template <int LAY, typename E>
__global__ __launch_bounds__(pp::NTHR) void gemm_pp_kernel(const PpGroup g)
{
    __shared__ __attribute__((aligned(1024))) char smem[pp::SMEM_BYTES];
    const int xcd = blockIdx.x & 7;
    int l = blockIdx.x >> 3;
    int q = 0, pid = -1;
    for (; q < g.count; ++q) {
        const int tiles = g.p[q].tiles_m * g.p[q].tiles_n * g.p[q].ksplit;
        const int base = tiles >> 3, rem = tiles & 7;
        const int mine = base + (xcd < rem ? 1 : 0);
        if (l < mine) {
            pid = xcd * base + min(xcd, rem) + l;
            break;
        }
        l -= mine;
    }
    if (pid < 0) return;
    const PpProblem &P = g.p[q];
    // K chunk of this workgroup: consecutive ids are different tiles of the same chunk, so they share panels
    const int per_chunk = P.tiles_m * P.tiles_n;
    const int chunk = pid / per_chunk;
    pid -= chunk * per_chunk;
    const int kt_total = P.a.K / pp::BK;
    const int kt_each = (kt_total + P.ksplit - 1) / P.ksplit;
    const int kt_begin = chunk * kt_each;
    const int kt_count = min(kt_each, kt_total - kt_begin);
    if (kt_count <= 0) return;
    switch (P.bm) {
    case 256: pp_tile<LAY, 256, E>(P.a, P.tiles_m, P.tiles_n, P.vec_epilogue, pid, kt_begin, kt_count, smem); break;
    case 192: pp_tile<LAY, 192, E>(P.a, P.tiles_m, P.tiles_n, P.vec_epilogue, pid, kt_begin, kt_count, smem); break;
    default: pp_tile<LAY, 128, E>(P.a, P.tiles_m, P.tiles_n, P.vec_epilogue, pid, kt_begin, kt_count, smem); break;
    }
}

// done: an event that completes with the kernel (its completion signal is the event's: no packet of its own in
// the queue, which a separate record costs ~4 us of queue time between two dependent launches), or null.
template <int LAY, typename E>
static hipError_t launch_gemm_pp_layout(const PpGroup &g, unsigned blocks, hipStream_t s, hipEvent_t done)
{
    if (done)
        hipExtLaunchKernelGGL((gemm_pp_kernel<LAY, E>), dim3(blocks), dim3(pp::NTHR), 0, s, nullptr, done, 0, g);
    else
        hipLaunchKernelGGL((gemm_pp_kernel<LAY, E>), dim3(blocks), dim3(pp::NTHR), 0, s, g);
    return hipGetLastError();
}

} // namespace rtp
