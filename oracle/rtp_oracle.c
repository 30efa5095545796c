/*
 * rtp_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, fp64 CPU statement of what the rotated-shard linear layer of
 * Rotated Tensor Parallelism (arXiv 2311.01635) computes.  It exists so that
 * the GPU path can be checked against something that can be read against the
 * paper by eye.  It shares no code, header, table or helper with the HIP
 * library and must never be linked into, imported by, or called from the
 * product path.
 *
 * What is here:
 *   - the rotation schedule (Design section, workflow paragraph: every worker
 *     sends its held shard to the next worker and receives from the previous
 *     one, N-1 times per pass; the backward pass mirrors it),
 *   - the three contractions of a linear layer, written as triple loops with
 *     no blocking, no BLAS and no reordering of the sum over the contracted
 *     index (RTP Transformers section, the block equation of the
 *     output-partitioned linear),
 *   - the elementwise activations and their derivatives that the MLP block
 *     places between its two GEMMs,
 *   - the closed forms of the parameter-memory table (Table 1).
 *
 * Every matrix is row-major with an explicit leading dimension so that a
 * shard can be addressed as a slice of the full matrix without a copy.
 * OpenMP threads split the OUTPUT rows only; each output element is always
 * one sequential sum over the contracted index in increasing order, so a
 * result does not depend on the thread count.
 */
#define _GNU_SOURCE
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- schedule: Design section, workflow paragraph ---------------------- */

/* Shard held by worker `rank` at forward step `step` (0-based).  Each
 * rotation hands the held shard to rank+1 and takes the one from rank-1, so
 * after `step` rotations the worker holds what rank-step started with. */
int orc_fwd_shard(int rank, int step, int n)
{
    int k = (rank - step) % n;
    return k < 0 ? k + n : k;
}

/* Backward mirrors forward: it starts on the shard the forward pass ended
 * on, (rank+1) mod n, and every rotation moves the other way, so the last
 * step (n-1) is back on the worker's own shard. */
int orc_bwd_shard(int rank, int step, int n)
{
    return (rank + 1 + step) % n;
}

/* Rotations per pass: compute runs n times, rotation n-1 times
 * (Memory Arrangement paragraph). */
int orc_rotations_per_pass(int n) { return n - 1; }

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- contractions ------------------------------------------------------ */

/* C[m,n] (+)= sum_k A[m,k] * B[n,k]      (forward:  Y = X W^T) */
void orc_gemm_nt(const double *A, int64_t lda, const double *B, int64_t ldb,
                 double *C, int64_t ldc, int64_t M, int64_t N, int64_t K,
                 int accumulate)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            double s = 0.0;
            for (int64_t k = 0; k < K; ++k)
                s += A[m * lda + k] * B[n * ldb + k];
            if (accumulate)
                C[m * ldc + n] += s;
            else
                C[m * ldc + n] = s;
        }
    }
}

/* C[m,n] (+)= sum_k A[m,k] * B[k,n]      (input gradient: dX = dY W) */
void orc_gemm_nn(const double *A, int64_t lda, const double *B, int64_t ldb,
                 double *C, int64_t ldc, int64_t M, int64_t N, int64_t K,
                 int accumulate)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        double *c = C + m * ldc;
        if (!accumulate)
            for (int64_t n = 0; n < N; ++n)
                c[n] = 0.0;
        /* k outermost of the two inner loops so that B is walked along its
         * rows; each c[n] still receives its terms in increasing k. */
        for (int64_t k = 0; k < K; ++k) {
            const double a = A[m * lda + k];
            const double *b = B + k * ldb;
            for (int64_t n = 0; n < N; ++n)
                c[n] += a * b[n];
        }
    }
}

/* C[m,n] (+)= sum_k A[k,m] * B[k,n]      (weight gradient: dW = dY^T X) */
void orc_gemm_tn(const double *A, int64_t lda, const double *B, int64_t ldb,
                 double *C, int64_t ldc, int64_t M, int64_t N, int64_t K,
                 int accumulate)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        double *c = C + m * ldc;
        if (!accumulate)
            for (int64_t n = 0; n < N; ++n)
                c[n] = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            const double a = A[k * lda + m];
            const double *b = B + k * ldb;
            for (int64_t n = 0; n < N; ++n)
                c[n] += a * b[n];
        }
    }
}

/* ---- activations of the MLP block -------------------------------------- */

/* GELU in its exact (erf) form: x * Phi(x). */
double orc_gelu(double x) { return 0.5 * x * (1.0 + erf(x * M_SQRT1_2)); }

/* d/dx [x Phi(x)] = Phi(x) + x phi(x). */
double orc_gelu_grad(double x)
{
    const double Phi = 0.5 * (1.0 + erf(x * M_SQRT1_2));
    const double phi = exp(-0.5 * x * x) / sqrt(2.0 * M_PI);
    return Phi + x * phi;
}

/* GELU in its tanh form and derivative. */
double orc_gelu_tanh(double x)
{
    const double c = sqrt(2.0 / M_PI);
    return 0.5 * x * (1.0 + tanh(c * (x + 0.044715 * x * x * x)));
}

double orc_gelu_tanh_grad(double x)
{
    const double c = sqrt(2.0 / M_PI);
    const double u = c * (x + 0.044715 * x * x * x);
    const double th = tanh(u);
    const double du = c * (1.0 + 3.0 * 0.044715 * x * x);
    return 0.5 * (1.0 + th) + 0.5 * x * (1.0 - th * th) * du;
}

static double sigmoid(double x) { return 1.0 / (1.0 + exp(-x)); }

/* silu(x) = x sigma(x);  silu'(x) = sigma(x) (1 + x (1 - sigma(x))). */
double orc_silu(double x) { return x * sigmoid(x); }

double orc_silu_grad(double x)
{
    const double s = sigmoid(x);
    return s * (1.0 + x * (1.0 - s));
}

/* Vector forms so that the Python side does no arithmetic of its own.
 * kind: 0 gelu(erf), 1 gelu(tanh), 2 silu. */
void orc_act(const double *x, double *y, int64_t n, int kind)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        y[i] = kind == 0 ? orc_gelu(x[i]) : kind == 1 ? orc_gelu_tanh(x[i]) : orc_silu(x[i]);
}

void orc_act_grad(const double *x, double *y, int64_t n, int kind)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        y[i] = kind == 0 ? orc_gelu_grad(x[i]) : kind == 1 ? orc_gelu_tanh_grad(x[i]) : orc_silu_grad(x[i]);
}

/* ---- parameter memory, Table 1 ----------------------------------------- */

/* System-wide parameter bytes for weight bytes W and gradient bytes G over
 * n workers.  technique: 0 none, 1 tensor parallel, 2 data parallel,
 * 3 pipeline parallel, 4 FSDP, 5 RTP (out of place), 6 RTP in place. */
int64_t orc_param_bytes(int technique, int64_t W, int64_t G, int64_t n)
{
    const int64_t mx = W > G ? W : G;
    switch (technique) {
    case 0: return W + G;
    case 1: return W + G;
    case 2: return (W + G) * n;
    case 3: return W + G;
    case 4: return W + G + mx * (n - 1);
    case 5: return W + G + mx;
    case 6: return W + G;
    default: return -1;
    }
}

/* The duplicated part of the same row of Table 1. */
int64_t orc_param_duplication(int technique, int64_t W, int64_t G, int64_t n)
{
    return orc_param_bytes(technique, W, G, n) - (W + G);
}
