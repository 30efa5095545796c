// Internal launch interface between the host scheduler and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rtp {

enum : int { LAY_NT = 0, LAY_NN = 1, LAY_TN = 2 };
enum : int { ELEM_BF16 = 0, ELEM_F16 = 1 }; // 16-bit element type of a GEMM's inputs and non-fp32 outputs

// What happens to the fp32 accumulator tile when the K loop is done.
enum : int {
    EPI_STORE = 0,        // C = acc                         (C in the output dtype)
    EPI_ACC_FIRST = 1,    // ws = acc                        (fp32 workspace)
    EPI_ACC_ADD = 2,      // ws += acc
    EPI_ACC_LAST = 3,     // C = ws + acc                    (rounded once)
    EPI_GELU_ERF_FWD = 4, // aux = acc ; C = gelu(acc)
    EPI_GELU_TANH_FWD = 5,
    EPI_SWIGLU_FWD = 6,   // B is [gate rows | up rows]; aux = (a | b); C = silu(a) * b
    EPI_GELU_ERF_BWD = 7, // C = acc * gelu'(aux)
    EPI_GELU_TANH_BWD = 8,
    EPI_SWIGLU_BWD = 9,   // C[:, n] = acc * b * silu'(a) ; C[:, half + n] = acc * silu(a)
    EPI_ACC_ATOMIC = 10   // ws += acc with fp32 atomic adds (set by the launcher when it splits K; not for callers)
};

struct GemmArgs {
    const void *A;
    const void *B;
    int64_t lda, ldb;   // elements
    int M, N, K;        // N counts both halves for EPI_SWIGLU_FWD
    int epi;
    void *C;            // output-dtype result
    int64_t ldc;
    float *ws;          // fp32 accumulator (EPI_ACC_*)
    int64_t ldws;
    void *aux;          // pre-activations, in the input dtype
    int64_t ldaux;
    const void *bias;   // optional, input dtype, one per column of B's rows (N of them, the (gate | up) order for
                        // EPI_SWIGLU_FWD): added to the product before EPI_STORE / EPI_*_FWD act on it
    int half;           // EPI_SWIGLU_FWD: N/2 ; EPI_SWIGLU_BWD: N
    int c_is_f32;       // EPI_STORE / EPI_ACC_LAST write fp32 instead of the input dtype
    int elem;           // ELEM_BF16 or ELEM_F16 (the ping-pong kernel only; the register-staged one is bf16)
    int cu_share;       // > 1: this launch runs beside cu_share - 1 others of similar size, so the
                        // tile height is picked for 1/cu_share of the compute units (0, 1: all)
    // Producer / consumer GEMMs inside one group launch of the tiled kernel (a rotation step as one launch):
    // `sync` points at one int32 counter per SYNC_ROWS rows of M, followed by one error word.  A tile of a
    // problem with sync_signal != 0 adds 1 to the counter of every row block it covers once its results are
    // visible device-wide; a tile of a problem with sync_wait > 0 starts only when the counter of every row
    // block it covers has reached sync_wait (a bounded wait: on giving up it raises the error word and
    // goes on).  The consumer must follow its producer in the group (the launcher keeps the given order).
    int *sync;
    int sync_signal, sync_wait;
};
constexpr int SYNC_ROWS = 64;

// bf16 inputs, fp32 MFMA accumulation.  variant: 0 = pick by shape; 1, 2, 3 = register-staged
// tiles (256x256/8 waves, 128x128/4 waves, 256x256/4 waves); 4 = the ping-pong kernel with the
// tile height picked by shape; 5, 6, 7 = the ping-pong kernel with tile height 256, 192, 128.
hipError_t launch_gemm_bf16(int layout, const GemmArgs &a, int variant, hipStream_t s);
// alignment and minimum sizes every bf16 kernel needs (M, N > 0 assumed)
bool gemm_bf16_args_ok(int layout, const GemmArgs &a);
// the ping-pong kernel (rtp_gemm_pp.h): needs K % 32 == 0; bm_override 0 = pick the tile height
bool gemm_bf16_pp_supported(int layout, const GemmArgs &a);
hipError_t launch_gemm_bf16_pp(int layout, const GemmArgs &a, int bm_override, hipStream_t s);
// up to PP_MAX_GROUP independent GEMMs of one layout in a single launch; tile heights, and for an
// fp32 `ws += ...` problem short of tiles a split of its K loop (partial sums meet through atomic
// adds, so the order of that sum is not fixed), are picked for the group as a whole (bm_override: null, or one forced height per problem, 0 = pick).
// hipErrorInvalidValue if a problem does not meet gemm_bf16_pp_supported.
constexpr int PP_MAX_GROUP = 4;
// done (may be null): an event that completes when the launch does, as if recorded right after it
hipError_t launch_gemm_bf16_pp_group(int layout, const GemmArgs *a, int count, const int *bm_override, hipStream_t s,
                                     hipEvent_t done = nullptr);
// the tile heights and K splits that launch would use (either output may be null)
void gemm_bf16_pp_plan(int layout, const GemmArgs *a, int count, const int *bm_override, int *bm_out, int *ksplit_out);
// column tiles the tiled kernel cuts a problem into (what a producer problem adds to each row block's counter)
int gemm_bf16_pp_tiles_n(const GemmArgs &a);
const char *gemm_bf16_kernel_name(int layout, int variant);

// fp32 inputs and outputs (epi: EPI_STORE, EPI_ACC_ADD with ws == C).
hipError_t launch_gemm_f32(int layout, const GemmArgs &a, hipStream_t s);

// elementwise pieces of the fp32 path (the bf16 path fuses them into the GEMMs)
// kind: EPI_GELU_ERF_FWD / EPI_GELU_TANH_FWD / EPI_SWIGLU_FWD / *_BWD
hipError_t launch_act_f32(int kind, const float *pre, int64_t ldpre, const float *in, int64_t ldin,
                          float *out, int64_t ldout, int rows, int cols, int half, hipStream_t s);

// device-to-device staging copy with a bounded number of workgroups
hipError_t launch_copy(void *dst, const void *src, size_t bytes, hipStream_t s, hipEvent_t done = nullptr);
// up to COPY_MAX_SEGS copies that do not overlap one another, as one launch (no order among them)
constexpr int COPY_MAX_SEGS = 4;
hipError_t launch_copy_multi(void *const *dst, const void *const *src, const size_t *bytes, int count, hipStream_t s,
                             hipEvent_t done = nullptr);
hipError_t launch_fill_zero(void *dst, size_t bytes, hipStream_t s);
// shard layout (pack: W -> slots, unpack: slots -> W): slot k's part at home + k * slot_bytes + off holds rows
// [k w, (k+1) w) of W[O, I] as [w, I] (cols == 0) or columns [k w, (k+1) w) as [O, w] (cols != 0); elements past
// the matrix are zero (pack) / skipped (unpack).  elem_bytes 2 or 4.
hipError_t launch_shard_layout(void *home, size_t slot_bytes, size_t off, int n, int cols, void *W, int64_t O, int64_t I,
                               int64_t w, int elem_bytes, int unpack, hipStream_t s);
// bias gradient: out[c] = in[c] + sum over rows of Y[r, c], c < cols (fp32 in/out, which may be the same);
// elem: -1 fp32, ELEM_BF16, ELEM_F16
hipError_t launch_colsum(int elem, const void *Y, int64_t ld, int rows, int cols, const float *in, float *out, hipStream_t s);

// ---- expert partition: tokens grouped by the expert they are routed to -----------------------
// Stable grouping of T tokens by route[t] in [0, n): group e starts at a multiple of `align` rows,
// perm[p] = the token in grouped row p or -1 (padding), p < cap.  counts[e] = tokens of expert e,
// counts[n] = tokens whose id is out of range (they are left out).  One workgroup; n <= MOE_MAX_EXPERTS;
// cap >= align * (T / align + n) is the caller's to guarantee.
constexpr int MOE_MAX_EXPERTS = 64;
hipError_t launch_moe_dispatch(const int *route, int T, int n, int align, int cap, int *counts, int *perm, hipStream_t s);
// out[p, :] = in[perm[p], :], zero where perm[p] < 0 (rows of row_bytes, a multiple of 16)
hipError_t launch_gather_rows(void *out, const void *in, const int *perm, int rows, size_t row_bytes, hipStream_t s);
// out[perm[p], :] = in[p, :] where perm[p] >= 0
hipError_t launch_scatter_rows(void *out, const void *in, const int *perm, int rows, size_t row_bytes, hipStream_t s);

// dst[r, c] += bias[c] for r < rows, c < cols (dst fp32 with leading dimension ld; bias in the
// element type: -1 fp32, ELEM_BF16, ELEM_F16)
hipError_t launch_bias_add(int elem, float *dst, int64_t ld, int rows, int cols, const void *bias, hipStream_t s);

// out[0] = wall-clock ticks, out[1] = shader cycles over a spin of wall_ticks
hipError_t launch_clock_probe(long long *out, long long wall_ticks, hipStream_t s);

} // namespace rtp
