// Shared by the bf16 GEMM kernels: vector types, the fused activations and the
// epilogue that writes an accumulator tile to its destination.
#pragma once
#include "rtp_kernels.h"

namespace rtp {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
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

__device__ __forceinline__ float bf2f(__bf16 v) { return (float)v; }


// Writes a wave's FM x FN grid of 32x32 accumulator fragments.
// acc[i][j][v] is C[row, col] with
//   row = rbase + i*32 + 8*(v/4) + v%4        (rbase already holds 4*(lane/32))
//   col = n0 + j*NSTRIDE + cl                 (tile-local for the paired form)
// The N fragments of a wave are NSTRIDE columns apart so that, for the gated
// (gate, up) form, fragment j and fragment j + FN/2 of the same wave hold the
// two halves of a pair in the same lanes.
template <int FM, int FN, int NSTRIDE>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs &p, f32x16 (&acc)[FM][FN], int rbase, int n0, int cl)
{
    const int M = p.M, N = p.N;
    __bf16 *Cb = (__bf16 *)p.C;
    float *Cf = (float *)p.C;
    const __bf16 *auxr = (const __bf16 *)p.aux;
    __bf16 *auxw = (__bf16 *)p.aux;
    const int64_t ldc = p.ldc, ldws = p.ldws, ldaux = p.ldaux;
    float *ws = p.ws;

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
                    const float a = acc[i][j][v], b = acc[i][j + FN / 2][v];
                    auxw[(int64_t)row * ldaux + col] = (__bf16)a;
                    auxw[(int64_t)row * ldaux + half + col] = (__bf16)b;
                    Cb[(int64_t)row * ldc + col] = (__bf16)(silu(a) * b);
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
                    if (row < M) fn(row, col, acc[i][j][v]);
                }
            }
    };
    switch (p.epi) {
    case EPI_STORE:
        if (p.c_is_f32)
            each([&](int row, int col, float x) { Cf[(int64_t)row * ldc + col] = x; });
        else
            each([&](int row, int col, float x) { Cb[(int64_t)row * ldc + col] = (__bf16)x; });
        break;
    case EPI_ACC_FIRST:
        each([&](int row, int col, float x) { ws[(int64_t)row * ldws + col] = x; });
        break;
    case EPI_ACC_ADD:
        each([&](int row, int col, float x) { ws[(int64_t)row * ldws + col] += x; });
        break;
    case EPI_ACC_LAST:
        if (p.c_is_f32)
            each([&](int row, int col, float x) { Cf[(int64_t)row * ldc + col] = ws[(int64_t)row * ldws + col] + x; });
        else
            each([&](int row, int col, float x) {
                Cb[(int64_t)row * ldc + col] = (__bf16)(ws[(int64_t)row * ldws + col] + x);
            });
        break;
    case EPI_GELU_ERF_FWD:
        each([&](int row, int col, float x) {
            auxw[(int64_t)row * ldaux + col] = (__bf16)x;
            Cb[(int64_t)row * ldc + col] = (__bf16)gelu_erf(x);
        });
        break;
    case EPI_GELU_TANH_FWD:
        each([&](int row, int col, float x) {
            auxw[(int64_t)row * ldaux + col] = (__bf16)x;
            Cb[(int64_t)row * ldc + col] = (__bf16)gelu_tanh(x);
        });
        break;
    case EPI_GELU_ERF_BWD:
        each([&](int row, int col, float x) {
            Cb[(int64_t)row * ldc + col] = (__bf16)(x * gelu_erf_grad(bf2f(auxr[(int64_t)row * ldaux + col])));
        });
        break;
    case EPI_GELU_TANH_BWD:
        each([&](int row, int col, float x) {
            Cb[(int64_t)row * ldc + col] = (__bf16)(x * gelu_tanh_grad(bf2f(auxr[(int64_t)row * ldaux + col])));
        });
        break;
    case EPI_SWIGLU_BWD: {
        const int half = p.half;
        each([&](int row, int col, float x) {
            const float a = bf2f(auxr[(int64_t)row * ldaux + col]);
            const float b = bf2f(auxr[(int64_t)row * ldaux + half + col]);
            Cb[(int64_t)row * ldc + col] = (__bf16)(x * b * silu_grad(a));
            Cb[(int64_t)row * ldc + half + col] = (__bf16)(x * silu(a));
        });
        break;
    }
    default:
        break;
    }
}

} // namespace rtp
