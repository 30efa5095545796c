// Shared by the bf16 GEMM kernels: vector types, the fused activations and the
// epilogue that writes an accumulator tile to its destination.
#pragma once
#include "rtp_kernels.h"

namespace rtp {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
// E is the 16-bit input/output element type of a kernel: __bf16 or _Float16
template <typename E> struct ElemVec;
template <> struct ElemVec<__bf16> {
    typedef __attribute__((ext_vector_type(4))) __bf16 v4;
    typedef bf16x8 v8;
};
template <> struct ElemVec<_Float16> {
    typedef __attribute__((ext_vector_type(4))) _Float16 v4;
    typedef f16x8 v8;
};
__device__ __forceinline__ f32x16 mfma_32x32x16(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x16 mfma_32x32x16(f16x8 a, f16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

// ---- activations (fp32) ---------------------------------------------------
__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_erf_grad(float x)
{
    const float Phi = 0.5f * (1.0f + erff(x * 0.70710678118654752f));
    const float phi = 0.3989422804014327f * __expf(-0.5f * x * x);
    return Phi + x * phi;
}
__device__ __forceinline__ float gelu_tanh(float x)
{
    const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
    return 0.5f * x * (1.0f + tanhf(u));
}
__device__ __forceinline__ float gelu_tanh_grad(float x)
{
    const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
    const float th = tanhf(u);
    const float du = 0.7978845608028654f * (1.0f + 3.0f * 0.044715f * x * x);
    return 0.5f * (1.0f + th) + 0.5f * x * (1.0f - th * th) * du;
}
__device__ __forceinline__ float sigmoidf_(float x) { return 1.0f / (1.0f + __expf(-x)); }
__device__ __forceinline__ float silu(float x) { return x * sigmoidf_(x); }
__device__ __forceinline__ float silu_grad(float x)
{
    const float s = sigmoidf_(x);
    return s * (1.0f + x * (1.0f - s));
}

template <typename E> __device__ __forceinline__ float bf2f(E v) { return (float)v; }


// The bias joins the product before a store or a forward activation sees it.  A lane's accumulators of
// fragment column j all belong to one output column (col0 + j * NSTRIDE), so it needs one value per j
// (zero when there is no bias or the epilogue takes none), added where the accumulators are read;
// for the gated form fragment j < FN/2 is a gate column and fragment j + FN/2 the up column with the
// same index, whose bias entries sit `half` further on.
template <typename E, int FN, int NSTRIDE>
__device__ __forceinline__ void gemm_epilogue_bias(const GemmArgs &p, int col0, float (&bj)[FN])
{
    const E *bias = (const E *)p.bias;
    const bool gated = p.epi == EPI_SWIGLU_FWD;
    const bool on = bias && (gated || p.epi == EPI_STORE || p.epi == EPI_GELU_ERF_FWD || p.epi == EPI_GELU_TANH_FWD);
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        int idx;
        bool lim;
        if (gated) {
            const int col = col0 + (j % (FN / 2)) * NSTRIDE;
            lim = col < p.half;
            idx = col + (j >= FN / 2 ? p.half : 0);
        } else {
            idx = col0 + j * NSTRIDE;
            lim = idx < p.N;
        }
        bj[j] = 0.0f;
        if (on && lim) bj[j] = (float)bias[idx];
    }
}

// Writes a wave's FM x FN grid of 32x32 accumulator fragments.
// acc[i][j][v] is C[row, col] with
//   row = rbase + i*32 + 8*(v/4) + v%4        (rbase already holds 4*(lane/32))
//   col = n0 + j*NSTRIDE + cl                 (tile-local for the paired form)
// The N fragments of a wave are NSTRIDE columns apart so that, for the gated
// (gate, up) form, fragment j and fragment j + FN/2 of the same wave hold the
// two halves of a pair in the same lanes.
template <typename E, int FM, int FN, int NSTRIDE>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs &p, f32x16 (&acc)[FM][FN], int rbase, int n0, int cl)
{
    const int M = p.M, N = p.N;
    E *Cb = (E *)p.C;
    float *Cf = (float *)p.C;
    const E *auxr = (const E *)p.aux;
    E *auxw = (E *)p.aux;
    const int64_t ldc = p.ldc, ldws = p.ldws, ldaux = p.ldaux;
    float *ws = p.ws;
    float bj[FN];
    gemm_epilogue_bias<E, FN, NSTRIDE>(p, n0 + cl, bj);

    if (p.epi == EPI_SWIGLU_FWD) {
        const int half = p.half;
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN / 2; ++j) {
                const int col = n0 + j * NSTRIDE + cl;
                if (col >= half) continue;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = rbase + i * 32 + 8 * (v >> 2) + (v & 3);
                    if (row >= M) continue;
                    const float a = acc[i][j][v] + bj[j], b = acc[i][j + FN / 2][v] + bj[j + FN / 2];
                    auxw[(int64_t)row * ldaux + col] = (E)a;
                    auxw[(int64_t)row * ldaux + half + col] = (E)b;
                    Cb[(int64_t)row * ldc + col] = (E)(silu(a) * b);
                }
            }
        return;
    }

    // visit every valid element of the tile; the branch on the epilogue kind
    // stays outside the unrolled loops
    auto each = [&](auto fn) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                const int col = n0 + j * NSTRIDE + cl;
                if (col >= N) continue;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = rbase + i * 32 + 8 * (v >> 2) + (v & 3);
                    if (row < M) fn(row, col, acc[i][j][v] + bj[j]);
                }
            }
    };
    switch (p.epi) {
    case EPI_STORE:
        if (p.c_is_f32)
            each([&](int row, int col, float x) { Cf[(int64_t)row * ldc + col] = x; });
        else
            each([&](int row, int col, float x) { Cb[(int64_t)row * ldc + col] = (E)x; });
        break;
    case EPI_ACC_FIRST:
        each([&](int row, int col, float x) { ws[(int64_t)row * ldws + col] = x; });
        break;
    case EPI_ACC_ADD:
        each([&](int row, int col, float x) { ws[(int64_t)row * ldws + col] += x; });
        break;
    case EPI_ACC_ATOMIC:
        each([&](int row, int col, float x) { unsafeAtomicAdd(ws + (int64_t)row * ldws + col, x); });
        break;
    case EPI_ACC_LAST:
        if (p.c_is_f32)
            each([&](int row, int col, float x) { Cf[(int64_t)row * ldc + col] = ws[(int64_t)row * ldws + col] + x; });
        else
            each([&](int row, int col, float x) {
                Cb[(int64_t)row * ldc + col] = (E)(ws[(int64_t)row * ldws + col] + x);
            });
        break;
    case EPI_GELU_ERF_FWD:
        each([&](int row, int col, float x) {
            auxw[(int64_t)row * ldaux + col] = (E)x;
            Cb[(int64_t)row * ldc + col] = (E)gelu_erf(x);
        });
        break;
    case EPI_GELU_TANH_FWD:
        each([&](int row, int col, float x) {
            auxw[(int64_t)row * ldaux + col] = (E)x;
            Cb[(int64_t)row * ldc + col] = (E)gelu_tanh(x);
        });
        break;
    case EPI_GELU_ERF_BWD:
        each([&](int row, int col, float x) {
            Cb[(int64_t)row * ldc + col] = (E)(x * gelu_erf_grad(bf2f(auxr[(int64_t)row * ldaux + col])));
        });
        break;
    case EPI_GELU_TANH_BWD:
        each([&](int row, int col, float x) {
            Cb[(int64_t)row * ldc + col] = (E)(x * gelu_tanh_grad(bf2f(auxr[(int64_t)row * ldaux + col])));
        });
        break;
    case EPI_SWIGLU_BWD: {
        const int half = p.half;
        each([&](int row, int col, float x) {
            const float a = bf2f(auxr[(int64_t)row * ldaux + col]);
            const float b = bf2f(auxr[(int64_t)row * ldaux + half + col]);
            Cb[(int64_t)row * ldc + col] = (E)(x * b * silu_grad(a));
            Cb[(int64_t)row * ldc + half + col] = (E)(x * silu(a));
        });
        break;
    }
    default:
        break;
    }
}


// ---- the same epilogue with 16-byte global accesses -----------------------------------
// The accumulator layout gives a lane one column and 16 scattered rows, which
// turns every fp32 read-modify-write or bf16 store into 2- or 4-byte accesses.
// Here a wave first parks one 32-row fragment row of its tile in its own LDS
// region (row pitch 288 bytes, so that the two half-waves of a ds_write_b32
// fall into different banks), then reads it back four consecutive columns per
// lane and touches global memory with float4 / 4 x bf16 accesses: whole 128-byte
// lines per row segment.  Needs every leading dimension to be a multiple of 4
// elements and 16-byte aligned bases; callers fall back to gemm_epilogue()
// otherwise.  No workgroup barrier: a wave only reads what it wrote.
constexpr int EPI_LDS_PITCH = 72;                       // floats per staged row (64 columns + pad)
constexpr int EPI_LDS_BYTES_PER_WAVE = 32 * EPI_LDS_PITCH * 4;
constexpr int EPI_LAND_ROUNDS = 8;                                   // reads of an fp32 sum in flight per wave ...
constexpr int EPI_LAND_BYTES_PER_WAVE = EPI_LAND_ROUNDS * 64 * 16;   // ... landing in LDS, 16 bytes per lane each

typedef __attribute__((ext_vector_type(4))) float f32x4;

template <typename E>
__device__ __forceinline__ typename ElemVec<E>::v4 to_elem4(f32x4 x)
{
    typename ElemVec<E>::v4 r;
    r.x = (E)x.x; r.y = (E)x.y; r.z = (E)x.z; r.w = (E)x.w;
    return r;
}
template <typename E>
__device__ __forceinline__ f32x4 from_elem4(typename ElemVec<E>::v4 x)
{
    f32x4 r;
    r.x = (float)x.x; r.y = (float)x.y; r.z = (float)x.z; r.w = (float)x.w;
    return r;
}
template <class F>
__device__ __forceinline__ f32x4 map4(f32x4 x, F f)
{
    f32x4 r;
    r.x = f(x.x); r.y = f(x.y); r.z = f(x.z); r.w = f(x.w);
    return r;
}

__host__ __device__ inline bool gemm_epilogue_vec_ok(const GemmArgs &p)
{
    auto al = [](const void *q, int a) { return ((uintptr_t)q & (uintptr_t)(a - 1)) == 0; };
    bool ok = (p.ldc & 3) == 0 && al(p.C, 16);
    if (p.epi == EPI_ACC_FIRST || p.epi == EPI_ACC_ADD || p.epi == EPI_ACC_LAST || p.epi == EPI_ACC_ATOMIC) ok = ok && (p.ldws & 3) == 0 && al(p.ws, 16);
    if (p.epi >= EPI_GELU_ERF_FWD && p.epi <= EPI_SWIGLU_BWD) ok = ok && (p.ldaux & 3) == 0 && al(p.aux, 8) && (p.half & 3) == 0;
    return ok && (p.N & 3) == 0;
}

template <typename E, int FM, int FN, int NSTRIDE>
__device__ __forceinline__ void gemm_epilogue_staged(const GemmArgs &p, f32x16 (&acc)[FM][FN], float *wlds,
                                                     int rbase_wave, int n0, int wn32, int lane, char *land = nullptr)
{
    typedef typename ElemVec<E>::v4 out4; // four consecutive elements of the 16-bit output type
    static_assert(FN == 2, "staging layout is written for two 32-column fragments per wave");
    const int M = p.M, N = p.N;
    const int64_t ldc = p.ldc, ldws = p.ldws, ldaux = p.ldaux;
    const int half = p.half;
    E *Cb = (E *)p.C;
    float *Cf = (float *)p.C;
    E *aux = (E *)p.aux;
    float *ws = p.ws;
    const int wrow = 4 * (lane >> 5), wcol = lane & 31;
    float bj[FN];
    gemm_epilogue_bias<E, FN, NSTRIDE>(p, n0 + wn32 + wcol, bj);

    // park fragment row i: rows 8*(v/4) + 4*(lane/32) + v%4, columns j*32 + lane%32
    auto park = [&](int i) {
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                wlds[(8 * (v >> 2) + wrow + (v & 3)) * EPI_LDS_PITCH + j * 32 + wcol] = acc[i][j][v] + bj[j];
        __builtin_amdgcn_s_waitcnt(0xc07f); // lgkmcnt(0): the wave's own writes have landed
        __builtin_amdgcn_wave_barrier();
    };

    if (p.epi == EPI_SWIGLU_FWD) {
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            park(i);
            // a lane takes the gate and the up value of the same 4 columns
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = 8 * r + (lane >> 3), c = (lane & 7) * 4;
                const f32x4 a = *(const f32x4 *)(wlds + row * EPI_LDS_PITCH + c);
                const f32x4 b = *(const f32x4 *)(wlds + row * EPI_LDS_PITCH + 32 + c);
                const int grow = rbase_wave + i * 32 + row, col = n0 + wn32 + c;
                if (grow < M && col < half) {
                    *(out4 *)(aux + (int64_t)grow * ldaux + col) = to_elem4<E>(a);
                    *(out4 *)(aux + (int64_t)grow * ldaux + half + col) = to_elem4<E>(b);
                    f32x4 h;
                    h.x = silu(a.x) * b.x; h.y = silu(a.y) * b.y; h.z = silu(a.z) * b.z; h.w = silu(a.w) * b.w;
                    *(out4 *)(Cb + (int64_t)grow * ldc + col) = to_elem4<E>(h);
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
        return;
    }

    // every valid group of 4 consecutive columns; the branch on the kind stays outside the loops
    auto each = [&](auto op) {
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            park(i);
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const int row = 4 * r + (lane >> 4), c4 = lane & 15;
                const f32x4 x = *(const f32x4 *)(wlds + row * EPI_LDS_PITCH + c4 * 4);
                const int grow = rbase_wave + i * 32 + row;
                const int col = n0 + (c4 >> 3) * NSTRIDE + wn32 + (c4 & 7) * 4;
                if (grow < M && col < N) op(grow, col, x);
            }
            __builtin_amdgcn_wave_barrier();
        }
    };
    // The same for an epilogue that READS global memory (an fp32 sum it adds onto, saved pre-activations): the reads
    // of a fragment row are issued four at a time before the first of their results is stored.  Written load -
    // compute - store group by group, each read waits behind the previous group's store (the compiler cannot tell
    // the addresses apart), i.e. 8 x FM memory round trips in a row per tile instead of 2 x FM.  The reads use clamped
    // coordinates, so that they are legal and unconditional (a vector epilogue has M >= 1 and N >= 4); what they
    // fetch for a group outside the matrix is not used.
    auto each_rw = [&](auto load, auto op) {
        constexpr int DEPTH = 4; // reads in flight per lane: 16 registers (eight at once push the kernel past the
                                 // register count at which the staging copies' waves still fit beside its own)
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            park(i);
#pragma unroll
            for (int r0 = 0; r0 < 8; r0 += DEPTH) {
                decltype(load(0, 0)) in[DEPTH];
#pragma unroll
                for (int r = r0; r < r0 + DEPTH; ++r) {
                    const int c4 = lane & 15;
                    const int grow = rbase_wave + i * 32 + 4 * r + (lane >> 4);
                    const int col = n0 + (c4 >> 3) * NSTRIDE + wn32 + (c4 & 7) * 4;
                    in[r - r0] = load(min(grow, M - 1), min(col, N - 4));
                }
#pragma unroll
                for (int r = r0; r < r0 + DEPTH; ++r) {
                    const int row = 4 * r + (lane >> 4), c4 = lane & 15;
                    const f32x4 x = *(const f32x4 *)(wlds + row * EPI_LDS_PITCH + c4 * 4);
                    const int grow = rbase_wave + i * 32 + row;
                    const int col = n0 + (c4 >> 3) * NSTRIDE + wn32 + (c4 & 7) * 4;
                    if (grow < M && col < N) op(grow, col, x, in[r - r0]);
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    };
    // The same for the fp32 sum `ws`, read straight into LDS (`land`: EPI_LAND_BYTES_PER_WAVE of the wave's own) instead
    // of into registers: the eight reads of a fragment row are in flight at once at no register cost, and the reads
    // of the next fragment row are on their way while this one's accumulators are parked.  Each lane's 16 bytes land
    // at land + 1024 * round + 16 * lane.  Byte offsets into `ws` are 32-bit: the caller checks the range.
    auto each_rw_landed = [&](auto op) {
        typedef __attribute__((address_space(3))) void *lds_vp;
        const unsigned ws_bytes = __builtin_amdgcn_readfirstlane((unsigned)(((int64_t)(M - 1) * ldws + N) * 4));
        const __amdgpu_buffer_rsrc_t rws = __builtin_amdgcn_make_buffer_rsrc((void *)ws, 0, ws_bytes, 0x00020000);
        auto fetch = [&](int i) {
#pragma unroll
            for (int r = 0; r < EPI_LAND_ROUNDS; ++r) {
                const int c4 = lane & 15;
                const int grow = rbase_wave + i * 32 + 4 * r + (lane >> 4);
                const int col = n0 + (c4 >> 3) * NSTRIDE + wn32 + (c4 & 7) * 4;
                const unsigned off = ((unsigned)min(grow, M - 1) * (unsigned)ldws + (unsigned)min(col, N - 4)) * 4u;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rws, (lds_vp)(land + r * 1024), 16, off, 0, 0, 0);
            }
        };
        fetch(0);
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            park(i);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); // this fragment row's reads have landed
#pragma unroll
            for (int r = 0; r < EPI_LAND_ROUNDS; ++r) {
                const int row = 4 * r + (lane >> 4), c4 = lane & 15;
                const f32x4 x = *(const f32x4 *)(wlds + row * EPI_LDS_PITCH + c4 * 4);
                const f32x4 old = *(const f32x4 *)(land + r * 1024 + lane * 16);
                const int grow = rbase_wave + i * 32 + row;
                const int col = n0 + (c4 >> 3) * NSTRIDE + wn32 + (c4 & 7) * 4;
                if (grow < M && col < N) op(grow, col, x, old);
            }
            __builtin_amdgcn_s_waitcnt(0xc07f); // lgkmcnt(0): the landing area has been read ...
            __builtin_amdgcn_wave_barrier();
            if (i + 1 < FM) fetch(i + 1);       // ... before the next reads are sent into it
        }
    };
    const bool landed = land != nullptr && ((int64_t)(M - 1) * ldws + N) * 4 < ((int64_t)1 << 32);
    switch (p.epi) {
    case EPI_STORE:
        if (p.c_is_f32)
            each([&](int r, int c, f32x4 x) { *(f32x4 *)(Cf + (int64_t)r * ldc + c) = x; });
        else
            each([&](int r, int c, f32x4 x) { *(out4 *)(Cb + (int64_t)r * ldc + c) = to_elem4<E>(x); });
        break;
    case EPI_ACC_FIRST:
        each([&](int r, int c, f32x4 x) { *(f32x4 *)(ws + (int64_t)r * ldws + c) = x; });
        break;
    case EPI_ACC_ADD:
        if (landed)
            each_rw_landed([&](int r, int c, f32x4 x, f32x4 old) { *(f32x4 *)(ws + (int64_t)r * ldws + c) = old + x; });
        else
            each_rw([&](int r, int c) { return *(const f32x4 *)(ws + (int64_t)r * ldws + c); },
                    [&](int r, int c, f32x4 x, f32x4 old) { *(f32x4 *)(ws + (int64_t)r * ldws + c) = old + x; });
        break;
    case EPI_ACC_ATOMIC:
        // one float per lane, 32 consecutive lanes on 32 consecutive columns: an atomic instruction
        // then covers two whole 128-byte lines (one row of each fragment) instead of a quarter of eight
#pragma unroll
        for (int i = 0; i < FM; ++i) {
            park(i);
            const int j = lane >> 5, c = lane & 31;
            const int col = n0 + j * NSTRIDE + wn32 + c;
#pragma unroll 8
            for (int row = 0; row < 32; ++row) {
                const float x = wlds[row * EPI_LDS_PITCH + j * 32 + c];
                const int grow = rbase_wave + i * 32 + row;
                if (grow < M && col < N) unsafeAtomicAdd(ws + (int64_t)grow * ldws + col, x);
            }
            __builtin_amdgcn_wave_barrier();
        }
        break;
    case EPI_ACC_LAST:
        if (landed && p.c_is_f32)
            each_rw_landed([&](int r, int c, f32x4 x, f32x4 old) { *(f32x4 *)(Cf + (int64_t)r * ldc + c) = old + x; });
        else if (landed)
            each_rw_landed([&](int r, int c, f32x4 x, f32x4 old) { *(out4 *)(Cb + (int64_t)r * ldc + c) = to_elem4<E>(old + x); });
        else if (p.c_is_f32)
            each_rw([&](int r, int c) { return *(const f32x4 *)(ws + (int64_t)r * ldws + c); },
                    [&](int r, int c, f32x4 x, f32x4 old) { *(f32x4 *)(Cf + (int64_t)r * ldc + c) = old + x; });
        else
            each_rw([&](int r, int c) { return *(const f32x4 *)(ws + (int64_t)r * ldws + c); },
                    [&](int r, int c, f32x4 x, f32x4 old) { *(out4 *)(Cb + (int64_t)r * ldc + c) = to_elem4<E>(old + x); });
        break;
    case EPI_GELU_ERF_FWD:
        each([&](int r, int c, f32x4 x) {
            *(out4 *)(aux + (int64_t)r * ldaux + c) = to_elem4<E>(x);
            *(out4 *)(Cb + (int64_t)r * ldc + c) = to_elem4<E>(map4(x, [](float t) { return gelu_erf(t); }));
        });
        break;
    case EPI_GELU_TANH_FWD:
        each([&](int r, int c, f32x4 x) {
            *(out4 *)(aux + (int64_t)r * ldaux + c) = to_elem4<E>(x);
            *(out4 *)(Cb + (int64_t)r * ldc + c) = to_elem4<E>(map4(x, [](float t) { return gelu_tanh(t); }));
        });
        break;
    case EPI_GELU_ERF_BWD:
        each_rw([&](int r, int c) { return *(const out4 *)(aux + (int64_t)r * ldaux + c); },
                [&](int r, int c, f32x4 x, out4 zz) {
                    const f32x4 z = from_elem4<E>(zz);
                    *(out4 *)(Cb + (int64_t)r * ldc + c) = to_elem4<E>(x * map4(z, [](float t) { return gelu_erf_grad(t); }));
                });
        break;
    case EPI_GELU_TANH_BWD:
        each_rw([&](int r, int c) { return *(const out4 *)(aux + (int64_t)r * ldaux + c); },
                [&](int r, int c, f32x4 x, out4 zz) {
                    const f32x4 z = from_elem4<E>(zz);
                    *(out4 *)(Cb + (int64_t)r * ldc + c) = to_elem4<E>(x * map4(z, [](float t) { return gelu_tanh_grad(t); }));
                });
        break;
    case EPI_SWIGLU_BWD: {
        struct GateUp {
            out4 a, b;
        };
        each_rw([&](int r, int c) {
                    return GateUp{*(const out4 *)(aux + (int64_t)r * ldaux + c), *(const out4 *)(aux + (int64_t)r * ldaux + half + c)};
                },
                [&](int r, int c, f32x4 x, GateUp g) {
                    const f32x4 a = from_elem4<E>(g.a), b = from_elem4<E>(g.b);
                    *(out4 *)(Cb + (int64_t)r * ldc + c) = to_elem4<E>(x * b * map4(a, [](float t) { return silu_grad(t); }));
                    *(out4 *)(Cb + (int64_t)r * ldc + half + c) = to_elem4<E>(x * map4(a, [](float t) { return silu(t); }));
                });
        break;
    }
    default:
        break;
    }
}

} // namespace rtp
