// Host scheduler behind the C ABI of include/rtp.h: shard index arithmetic,
// the ring's buffer/state machine, the event graph between the compute and
// the stage stream, and the per-step kernel launches.  No device memory is
// allocated here; the only HIP objects owned are events.
#include "../../include/rtp.h"
#include "rtp_kernels.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

using namespace rtp;

// ---------------------------------------------------------------------------
// errors
// ---------------------------------------------------------------------------
static thread_local char g_err[512] = "";

static rtp_status fail(rtp_status s, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return s;
}

#define HIP_TRY(expr)                                                                                       \
    do {                                                                                                    \
        hipError_t e_ = (expr);                                                                             \
        if (e_ != hipSuccess) return fail(RTP_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_));             \
    } while (0)

#define RTP_TRY(expr)                       \
    do {                                    \
        rtp_status s_ = (expr);             \
        if (s_ != RTP_OK) return s_;        \
    } while (0)

extern "C" const char *rtp_last_error(void) { return g_err; }

extern "C" const char *rtp_status_str(rtp_status s)
{
    switch (s) {
    case RTP_OK: return "RTP_OK";
    case RTP_ERR_INVALID: return "RTP_ERR_INVALID";
    case RTP_ERR_SHAPE: return "RTP_ERR_SHAPE";
    case RTP_ERR_STATE: return "RTP_ERR_STATE";
    case RTP_ERR_UNSUPPORTED: return "RTP_ERR_UNSUPPORTED";
    case RTP_ERR_HIP: return "RTP_ERR_HIP";
    }
    return "RTP_ERR_?";
}

// ---------------------------------------------------------------------------
// per-launch timing of the GEMM kernels (opt-in, for the roofline figures)
// ---------------------------------------------------------------------------
struct ProfRec {
    int layout;
    double flops;
    hipEvent_t start, stop;
};
static bool g_prof_on = false, g_prof_alone = false;
static std::vector<ProfRec> g_prof;

extern "C" rtp_status rtp_prof_begin_alone(int alone)
{
    if (g_prof_on) return fail(RTP_ERR_STATE, "rtp_prof_begin: already collecting");
    g_prof.clear();
    g_prof_on = true;
    g_prof_alone = alone != 0;
    return RTP_OK;
}

extern "C" rtp_status rtp_prof_begin(void) { return rtp_prof_begin_alone(0); }

extern "C" rtp_status rtp_prof_end(rtp_prof_result out[3])
{
    if (!g_prof_on) return fail(RTP_ERR_STATE, "rtp_prof_end: not collecting");
    g_prof_on = false;
    if (out) memset(out, 0, 3 * sizeof(rtp_prof_result));
    rtp_status st = RTP_OK;
    for (ProfRec &r : g_prof) {
        float ms = 0.f;
        hipError_t e = hipEventSynchronize(r.stop);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.start, r.stop);
        if (e != hipSuccess && st == RTP_OK) st = fail(RTP_ERR_HIP, "rtp_prof_end: %s", hipGetErrorString(e));
        if (out && e == hipSuccess) {
            out[r.layout].launches += 1;
            out[r.layout].total_ms += ms;
            out[r.layout].total_flops += r.flops;
        }
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
    }
    g_prof.clear();
    return st;
}

// brackets one launch with events on its own stream when collecting
template <class F>
static hipError_t timed_launch(int layout, double flops, hipStream_t s, F launch)
{
    if (!g_prof_on) return launch();
    ProfRec r{layout, flops, nullptr, nullptr};
    hipError_t e = hipEventCreate(&r.start);
    if (e != hipSuccess) return e;
    e = hipEventCreate(&r.stop);
    if (e != hipSuccess) {
        (void)hipEventDestroy(r.start);
        return e;
    }
    // "alone": the device is idle when the launch starts and nothing else is enqueued until it has
    // ended, so its duration is that of the kernel with the machine to itself
    e = g_prof_alone ? hipDeviceSynchronize() : hipSuccess;
    if (e == hipSuccess) e = hipEventRecord(r.start, s);
    if (e == hipSuccess) e = launch();
    if (e == hipSuccess) e = hipEventRecord(r.stop, s);
    if (e == hipSuccess && g_prof_alone) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
        return e;
    }
    g_prof.push_back(r);
    return hipSuccess;
}

// ---------------------------------------------------------------------------
// schedule (Design section, workflow paragraph)
// ---------------------------------------------------------------------------
extern "C" int rtp_fwd_shard(int rank, int step, int n)
{
    if (n <= 0 || rank < 0 || rank >= n || step < 0 || step >= n) return -1;
    // each clockwise rotation brings in what the previous worker held
    return (rank - step + n) % n;
}

extern "C" int rtp_bwd_shard(int rank, int step, int n)
{
    if (n <= 0 || rank < 0 || rank >= n || step < 0 || step >= n) return -1;
    // starts where the forward pass ended and walks back to the worker's own shard
    return (rank + 1 + step) % n;
}

extern "C" int64_t rtp_shard_begin(int k, int64_t dim, int n)
{
    if (n <= 0 || k < 0 || k >= n || dim < 0 || dim % n != 0) return -1;
    return (int64_t)k * (dim / n);
}

static int64_t width_align(rtp_dtype t) { return t == RTP_F32 ? 1 : t == RTP_F16 ? 32 : 8; }

extern "C" int64_t rtp_shard_width(int64_t dim, int n, rtp_dtype dtype)
{
    if (n <= 0 || dim <= 0) return -1;
    if (dim % n == 0) return dim / n;
    // FlatParameter-style padding: equal shards of the smallest aligned width that covers dim;
    // the last one is only partly filled, and must not be empty
    const int64_t al = width_align(dtype);
    const int64_t o = ((dim + n - 1) / n + al - 1) / al * al;
    if ((int64_t)(n - 1) * o >= dim) return -1;
    return o;
}

extern "C" size_t rtp_worker_bytes(rtp_mode mode, size_t w, size_t g)
{
    switch (mode) {
    case RTP_DOUBLE_BUFFER: return 2 * (w + g);
    case RTP_INPLACE_STAGED: return 2 * w + g;
    case RTP_INPLACE_BLOCKING: return w + g;
    }
    return 0;
}

extern "C" size_t rtp_table1_worker_bytes(int inplace, size_t w, size_t g)
{
    // Table 1, rows "RTP" and "RTP Inplace", divided evenly over the workers
    return inplace ? w + g : w + g + std::max(w, g);
}

// ---------------------------------------------------------------------------
// shard layout (Partition Strategies section; FlatParameter paragraph)
// ---------------------------------------------------------------------------
static rtp_status shard_layout(const char *who, void *home, size_t slot_bytes, size_t offset, int n, rtp_split split,
                               void *W, int64_t O, int64_t I, int64_t width, rtp_dtype dtype, void *stream, int unpack)
{
    if (!home || !W) return fail(RTP_ERR_INVALID, "%s: null pointer", who);
    if (split != RTP_SPLIT_OUT && split != RTP_SPLIT_IN) return fail(RTP_ERR_INVALID, "%s: bad split", who);
    if (dtype != RTP_F32 && dtype != RTP_BF16 && dtype != RTP_F16) return fail(RTP_ERR_INVALID, "%s: bad dtype", who);
    if (n < 1 || O <= 0 || I <= 0 || width <= 0) return fail(RTP_ERR_SHAPE, "%s: n, O, I and the shard width must be positive", who);
    const int64_t part = split == RTP_SPLIT_OUT ? O : I, other = split == RTP_SPLIT_OUT ? I : O;
    if ((int64_t)n * width < part)
        return fail(RTP_ERR_SHAPE, "%s: %d shards of width %lld do not cover a dimension of %lld", who, n, (long long)width,
                    (long long)part);
    const size_t es = dtype == RTP_F32 ? 4 : 2;
    if (offset % es || ((uintptr_t)home % es) || slot_bytes % es || ((uintptr_t)W % es))
        return fail(RTP_ERR_SHAPE, "%s: pointers, the slot size and the offset must be multiples of the element size", who);
    if (offset + (size_t)width * (size_t)other * es > slot_bytes)
        return fail(RTP_ERR_SHAPE, "%s: the shard part does not fit the slot", who);
    HIP_TRY(launch_shard_layout(home, slot_bytes, offset, n, split == RTP_SPLIT_IN, W, O, I, width, (int)es, unpack,
                                (hipStream_t)stream));
    return RTP_OK;
}

extern "C" rtp_status rtp_pack_shards(void *home, size_t slot_bytes, size_t offset, int n, rtp_split split, const void *W,
                                      int64_t O, int64_t I, int64_t width, rtp_dtype dtype, void *stream)
{
    return shard_layout("rtp_pack_shards", home, slot_bytes, offset, n, split, (void *)W, O, I, width, dtype, stream, 0);
}

extern "C" rtp_status rtp_unpack_shards(void *W, const void *home, size_t slot_bytes, size_t offset, int n, rtp_split split,
                                        int64_t O, int64_t I, int64_t width, rtp_dtype dtype, void *stream)
{
    return shard_layout("rtp_unpack_shards", (void *)home, slot_bytes, offset, n, split, W, O, I, width, dtype, stream, 1);
}

// ---------------------------------------------------------------------------
// ring
// ---------------------------------------------------------------------------
enum { TR_FWD = 1, TR_BWD = 2, TR_W_IN = 3, TR_W_OUT = 4, TR_G_IN = 5, TR_G_OUT = 6 };

struct rtp_linear;

struct rtp_ring {
    rtp_ring_desc d;
    bool dry = false;
    bool events_ready = false;
    bool abl_rotate = true, abl_compute = true;
    rtp_pass pass = RTP_PASS_IDLE;
    int resident = -1;   // shard whose weights are in buf_w[res_idx]
    int res_idx = 0;
    bool joined = false;      // nothing has been enqueued on the stage / auxiliary stream since rtp_ring_end joined them
    bool pass_uses_as = true; // the open pass enqueues on the auxiliary stream (a schedule that does not says so)
    bool w_held = false; // buf_w[res_idx] really holds shard `resident` as the store has it (not after a flush,
                         // an abort, or a pass run with the rotation switched off)
    int res_g = -1;      // shard whose gradients are in buf_g[res_g_idx]
    int res_g_idx = 0;
    int base_idx = 0;    // weight buffer index at step 0 of the open pass
    int rotations = 0;   // rotate_step calls in the open pass
    int executed = 0;    // blocking mode: rotations already carried out
    // test aid: a bounded spin kernel ahead of every transfer on the stage stream / every GEMM on the
    // auxiliary stream stretches the windows in which a missing cross-stream wait would show
    long long delay_stage_ticks = 0, delay_aux_ticks = 0, delay_compute_ticks = 0;
    long long *delay_out = nullptr, *delay_compute_out = nullptr;
    std::vector<rtp_linear *> linears;
    std::vector<rtp_trace_rec> trace;
    hipEvent_t ev_free = nullptr, ev_free2 = nullptr, ev_join = nullptr, ev_aux = nullptr;
    hipEvent_t ev_w[2] = {nullptr, nullptr};
    // the pipelined schedule of the MLP unit moves the two linears' shard parts separately
    hipEvent_t ev_w2[2] = {nullptr, nullptr}, ev_g2[2] = {nullptr, nullptr}, ev_k[2] = {nullptr, nullptr};
    hipEvent_t ev_g[2] = {nullptr, nullptr};
    hipEvent_t ev_g0 = nullptr; // the gradient shard a backward pass starts on has landed

    hipStream_t cs() const { return (hipStream_t)d.compute_stream; }
    hipStream_t ss() const { return d.mode == RTP_INPLACE_BLOCKING ? cs() : (hipStream_t)d.stage_stream; }
    // second compute stream (weight-gradient kernels); the compute stream itself when none was given
    hipStream_t as() const { return d.aux_stream ? (hipStream_t)d.aux_stream : cs(); }
    char *home_w(int k) const { return (char *)d.home_w_dev + (size_t)k * d.w_bytes; }
    char *home_g(int k) const { return (char *)d.home_g_dev + (size_t)k * d.g_bytes; }
    int w_idx(int step) const { return d.mode == RTP_INPLACE_BLOCKING ? 0 : (base_idx + step) & 1; }
    int g_idx(int step) const { return d.mode == RTP_DOUBLE_BUFFER ? (step & 1) : 0; }
    int shard_at(int step) const
    {
        return pass == RTP_PASS_BWD ? rtp_bwd_shard(d.rank, step, d.n) : rtp_fwd_shard(d.rank, step, d.n);
    }
    void rec(int kind, int step, int shard, int buffer)
    {
        trace.push_back(rtp_trace_rec{kind, (int)pass, step, shard, buffer});
    }
};

struct rtp_linear {
    rtp_ring *ring;
    rtp_linear_desc d;
    int64_t o;        // shard width along the partitioned dimension
    size_t w_shard_bytes, g_shard_bytes;
    int next_step = 0;
    hipEvent_t ev_dw = nullptr, ev_g_in = nullptr;
};

static rtp_status ensure_events(rtp_ring *r)
{
    if (r->dry || r->events_ready) return RTP_OK;
    hipEvent_t *all[] = {&r->ev_free, &r->ev_free2, &r->ev_join, &r->ev_aux, &r->ev_w[0], &r->ev_w[1], &r->ev_g[0], &r->ev_g[1],
                         &r->ev_w2[0], &r->ev_w2[1], &r->ev_g2[0], &r->ev_g2[1], &r->ev_k[0], &r->ev_k[1], &r->ev_g0};
    for (hipEvent_t *e : all)
        HIP_TRY(hipEventCreateWithFlags(e, hipEventDisableTiming));
    for (rtp_linear *l : r->linears) {
        if (!l->ev_dw) HIP_TRY(hipEventCreateWithFlags(&l->ev_dw, hipEventDisableTiming));
        if (!l->ev_g_in) HIP_TRY(hipEventCreateWithFlags(&l->ev_g_in, hipEventDisableTiming));
    }
    r->events_ready = true;
    return RTP_OK;
}

// done: an event recorded on `s` behind the transfer; a copy kernel carries it as its completion signal (one host
// call and one packet in the queue less than a record of its own).  A dry ring has no events.
static rtp_status copy_async(rtp_ring *r, void *dst, const void *src, size_t bytes, hipStream_t s, hipEvent_t done = nullptr)
{
    if (r->dry) return RTP_OK;
    if (bytes == 0) {
        if (done) HIP_TRY(hipEventRecord(done, s));
        return RTP_OK;
    }
    if (r->delay_stage_ticks > 0 && s == r->ss() && r->ss() != r->cs())
        HIP_TRY(launch_clock_probe(r->delay_out, r->delay_stage_ticks, s));
    if (r->d.flags & RTP_FLAG_STAGE_MEMCPY) {
        HIP_TRY(hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToDevice, s));
        if (done) HIP_TRY(hipEventRecord(done, s));
    } else {
        HIP_TRY(launch_copy(dst, src, bytes, s, done));
    }
    return RTP_OK;
}

// Transfers that do not depend on one another, gathered so that they go out as ONE launch: the host pays for
// every launch (and every cross-stream wait) of a pass, and the narrow-shard units are bound by exactly that.
// The workgroups of the launch are dealt segment by segment, so the copies still pass through the machine one
// after the other.  (A kernel in which every thread served both directions of a rotation at once was measured
// 40 % slower than two plain copies: four interleaved address streams use HBM worse than two.)
constexpr size_t COPY_BATCH_MAX_BYTES = (size_t)16 << 20;
struct CopyBatch {
    int n = 0;
    void *dst[COPY_MAX_SEGS];
    const void *src[COPY_MAX_SEGS];
    size_t bytes[COPY_MAX_SEGS];
};

static rtp_status copy_batch_flush(rtp_ring *r, CopyBatch &b, hipStream_t s, hipEvent_t done = nullptr)
{
    if (r->dry) {
        b.n = 0;
        return RTP_OK;
    }
    if (b.n == 0) {
        if (done) HIP_TRY(hipEventRecord(done, s));
        return RTP_OK;
    }
    const int n = b.n;
    b.n = 0;
    // Large transfers go out one by one, in the order they were added (callers add the transfer a kernel waits for
    // first): beside a GEMM that fills the machine, copies that follow one another disturb it less than the same
    // bytes all at once (Llama-shaped unit: 4.31 against 4.39 ms per pass, expert unit 16.9 against 17.2; the
    // large unit with its few tokens per shard is the exception, 9.1 against 8.9), and a launch is nothing beside them.
    size_t total = 0;
    for (int i = 0; i < n; ++i) total += b.bytes[i];
    if (n == 1 || (r->d.flags & RTP_FLAG_STAGE_MEMCPY) || total >= COPY_BATCH_MAX_BYTES) {
        for (int i = 0; i < n; ++i) RTP_TRY(copy_async(r, b.dst[i], b.src[i], b.bytes[i], s, i == n - 1 ? done : nullptr));
        return RTP_OK;
    }
    if (r->delay_stage_ticks > 0 && s == r->ss() && r->ss() != r->cs())
        HIP_TRY(launch_clock_probe(r->delay_out, r->delay_stage_ticks, s));
    HIP_TRY(launch_copy_multi(b.dst, b.src, b.bytes, n, s, done));
    return RTP_OK;
}

// adds a transfer to the batch; the caller guarantees that it overlaps none of those already in it
static rtp_status copy_batch_add(rtp_ring *r, CopyBatch &b, void *dst, const void *src, size_t bytes, hipStream_t s)
{
    if (bytes == 0) return RTP_OK;
    if (b.n == COPY_MAX_SEGS) RTP_TRY(copy_batch_flush(r, b, s));
    b.dst[b.n] = dst; b.src[b.n] = src; b.bytes[b.n] = bytes;
    b.n++;
    return RTP_OK;
}

// One rotation of a shard part: the held part goes out and the next one comes in.  held_next may be the
// buffer the held part just left (the in-place exchange): then stream order keeps the two copies apart;
// otherwise they are one launch.
static rtp_status rotate_async(rtp_ring *r, void *out, const void *held, void *held_next, const void *in, size_t bytes,
                               hipStream_t s, hipEvent_t done = nullptr)
{
    if (held_next == held || out == in) {
        RTP_TRY(copy_async(r, out, held, bytes, s));
        RTP_TRY(copy_async(r, held_next, in, bytes, s, done));
        return RTP_OK;
    }
    CopyBatch b;
    RTP_TRY(copy_batch_add(r, b, held_next, in, bytes, s)); // the incoming part first: a kernel waits for it
    RTP_TRY(copy_batch_add(r, b, out, held, bytes, s));
    return copy_batch_flush(r, b, s, done);
}

// make each stream wait for everything enqueued so far on the other
static rtp_status cross_join(rtp_ring *r)
{
    if (r->dry) return RTP_OK;
    if (r->as() != r->cs()) {
        HIP_TRY(hipEventRecord(r->ev_join, r->as()));
        HIP_TRY(hipStreamWaitEvent(r->cs(), r->ev_join, 0));
    }
    if (r->ss() != r->cs()) {
        HIP_TRY(hipEventRecord(r->ev_join, r->ss()));
        HIP_TRY(hipStreamWaitEvent(r->cs(), r->ev_join, 0));
    }
    HIP_TRY(hipEventRecord(r->ev_join, r->cs()));
    if (r->ss() != r->cs()) HIP_TRY(hipStreamWaitEvent(r->ss(), r->ev_join, 0));
    if (r->as() != r->cs()) HIP_TRY(hipStreamWaitEvent(r->as(), r->ev_join, 0));
    return RTP_OK;
}

// Start of a pass: the stage and auxiliary streams wait for everything the compute stream holds (the caller's
// inputs were produced there); the other direction only if they may hold work the compute stream has not yet
// waited for (rtp_ring_end joins them, and only passes enqueue on them).
static rtp_status begin_join(rtp_ring *r)
{
    if (r->dry) return RTP_OK;
    if (!r->joined) return cross_join(r);
    r->joined = false;
    HIP_TRY(hipEventRecord(r->ev_join, r->cs()));
    if (r->ss() != r->cs()) HIP_TRY(hipStreamWaitEvent(r->ss(), r->ev_join, 0));
    if (r->as() != r->cs()) HIP_TRY(hipStreamWaitEvent(r->as(), r->ev_join, 0));
    return RTP_OK;
}

// A pass cannot be recorded into a HIP graph (the calls decide on the host what they enqueue, on
// three streams): refuse, before anything is enqueued, when one of the ring's streams is capturing.
static rtp_status refuse_capture(const rtp_ring *r, const char *who)
{
    if (r->dry) return RTP_OK;
    hipStream_t all[3] = {r->cs(), r->ss(), r->as()};
    for (int i = 0; i < 3; ++i) {
        if (i > 0 && all[i] == all[0]) continue;
        hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
        HIP_TRY(hipStreamIsCapturing(all[i], &st));
        if (st != hipStreamCaptureStatusNone)
            return fail(RTP_ERR_UNSUPPORTED, "%s: a stream of the ring is being captured into a graph; "
                                             "passes cannot be captured", who);
    }
    return RTP_OK;
}

extern "C" rtp_status rtp_ring_create(rtp_ring **out, const rtp_ring_desc *d)
{
    if (!out || !d) return fail(RTP_ERR_INVALID, "rtp_ring_create: null argument");
    *out = nullptr;
    if (d->n < 1 || d->rank < 0 || d->rank >= d->n)
        return fail(RTP_ERR_SHAPE, "rtp_ring_create: need n >= 1 and 0 <= rank < n (n=%d rank=%d)", d->n, d->rank);
    if ((d->w_bytes & 15) || (d->g_bytes & 15) || d->w_bytes == 0)
        return fail(RTP_ERR_SHAPE, "rtp_ring_create: slot sizes must be positive multiples of 16 bytes");
    if (d->mode != RTP_DOUBLE_BUFFER && d->mode != RTP_INPLACE_STAGED && d->mode != RTP_INPLACE_BLOCKING)
        return fail(RTP_ERR_INVALID, "rtp_ring_create: bad mode %d", (int)d->mode);
    const bool dry = (d->flags & RTP_FLAG_DRY_RUN) != 0;
    if (!dry) {
        if (!d->home_w_dev || !d->buf_w_dev[0]) return fail(RTP_ERR_INVALID, "rtp_ring_create: null weight buffer");
        if (d->mode != RTP_INPLACE_BLOCKING && !d->buf_w_dev[1])
            return fail(RTP_ERR_INVALID, "rtp_ring_create: the staging weight buffer is missing");
        if (d->g_bytes && (!d->home_g_dev || !d->buf_g_dev[0]))
            return fail(RTP_ERR_INVALID, "rtp_ring_create: null gradient buffer");
        if (d->g_bytes && d->mode == RTP_DOUBLE_BUFFER && !d->buf_g_dev[1])
            return fail(RTP_ERR_INVALID, "rtp_ring_create: double buffering needs two gradient buffers");
        if (d->buf_w_dev[0] == d->buf_w_dev[1] || (d->g_bytes && d->buf_g_dev[1] && d->buf_g_dev[0] == d->buf_g_dev[1]))
            return fail(RTP_ERR_INVALID, "rtp_ring_create: resident and staging buffers alias");
        if (d->mode != RTP_INPLACE_BLOCKING && d->compute_stream == d->stage_stream)
            return fail(RTP_ERR_INVALID, "rtp_ring_create: the stage stream must differ from the compute stream");
        if (d->aux_stream && (d->aux_stream == d->compute_stream || d->aux_stream == d->stage_stream))
            return fail(RTP_ERR_INVALID, "rtp_ring_create: the auxiliary stream must differ from the other two");
    }
    rtp_ring *r = new (std::nothrow) rtp_ring;
    if (!r) return fail(RTP_ERR_INVALID, "rtp_ring_create: out of host memory");
    r->d = *d;
    r->dry = dry;
    *out = r;
    return RTP_OK;
}

extern "C" rtp_status rtp_ring_destroy(rtp_ring *r)
{
    if (!r) return RTP_OK;
    if (!r->linears.empty()) return fail(RTP_ERR_STATE, "rtp_ring_destroy: destroy the ring's linears first");
    if (r->events_ready) {
        hipEvent_t all[] = {r->ev_free, r->ev_free2, r->ev_join, r->ev_aux, r->ev_w[0], r->ev_w[1], r->ev_g[0], r->ev_g[1],
                            r->ev_w2[0], r->ev_w2[1], r->ev_g2[0], r->ev_g2[1], r->ev_k[0], r->ev_k[1]};
        for (hipEvent_t e : all)
            if (e) (void)hipEventDestroy(e);
    }
    delete r;
    return RTP_OK;
}

extern "C" int rtp_ring_resident(const rtp_ring *r) { return r ? r->resident : -1; }
extern "C" int rtp_ring_resident_grad(const rtp_ring *r) { return r && r->d.g_bytes ? r->res_g : -1; }

extern "C" int64_t rtp_ring_trace(rtp_ring *r, rtp_trace_rec *out, int64_t cap, int clear)
{
    if (!r) return -1;
    const int64_t total = (int64_t)r->trace.size();
    if (out)
        for (int64_t i = 0; i < std::min(total, cap); ++i) out[i] = r->trace[(size_t)i];
    if (clear) r->trace.clear();
    return total;
}

static rtp_status set_ablation(rtp_ring *r, int rotate, int compute)
{
    if (r->pass != RTP_PASS_IDLE) return fail(RTP_ERR_STATE, "ablation can only change between passes");
    r->abl_rotate = rotate != 0;
    r->abl_compute = compute != 0;
    r->w_held = false;
    return RTP_OK;
}

extern "C" rtp_status rtp_ring_set_test_delay(rtp_ring *r, void *scratch32_dev, int64_t stage_us, int64_t aux_us)
{
    if (!r) return fail(RTP_ERR_INVALID, "rtp_ring_set_test_delay: null ring");
    if (r->pass != RTP_PASS_IDLE) return fail(RTP_ERR_STATE, "rtp_ring_set_test_delay: a pass is open");
    if (stage_us < 0 || aux_us < 0 || stage_us > 5000 || aux_us > 5000)
        return fail(RTP_ERR_INVALID, "rtp_ring_set_test_delay: delays are 0 to 5000 microseconds");
    r->delay_stage_ticks = r->delay_aux_ticks = 0;
    r->delay_out = nullptr;
    if (r->dry || (stage_us == 0 && aux_us == 0)) return RTP_OK;
    if (!scratch32_dev || ((uintptr_t)scratch32_dev & 7))
        return fail(RTP_ERR_INVALID, "rtp_ring_set_test_delay: the spin kernels need 32 bytes of 8-byte aligned device memory");
    int dev = 0, khz = 0;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev));
    if (khz <= 0) return fail(RTP_ERR_UNSUPPORTED, "rtp_ring_set_test_delay: the device reports no wall clock rate");
    r->delay_out = (long long *)scratch32_dev;
    r->delay_stage_ticks = stage_us * (int64_t)khz / 1000;
    r->delay_aux_ticks = aux_us * (int64_t)khz / 1000;
    return RTP_OK;
}

extern "C" rtp_status rtp_ring_set_test_delay_compute(rtp_ring *r, void *scratch16_dev, int64_t compute_us)
{
    if (!r) return fail(RTP_ERR_INVALID, "rtp_ring_set_test_delay_compute: null ring");
    if (r->pass != RTP_PASS_IDLE) return fail(RTP_ERR_STATE, "rtp_ring_set_test_delay_compute: a pass is open");
    if (compute_us < 0 || compute_us > 5000)
        return fail(RTP_ERR_INVALID, "rtp_ring_set_test_delay_compute: the delay is 0 to 5000 microseconds");
    r->delay_compute_ticks = 0;
    r->delay_compute_out = nullptr;
    if (r->dry || compute_us == 0) return RTP_OK;
    if (!scratch16_dev || ((uintptr_t)scratch16_dev & 7))
        return fail(RTP_ERR_INVALID, "rtp_ring_set_test_delay_compute: the spin kernels need 16 bytes of 8-byte aligned device memory");
    int dev = 0, khz = 0;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev));
    if (khz <= 0) return fail(RTP_ERR_UNSUPPORTED, "rtp_ring_set_test_delay_compute: the device reports no wall clock rate");
    r->delay_compute_out = (long long *)scratch16_dev;
    r->delay_compute_ticks = compute_us * (int64_t)khz / 1000;
    return RTP_OK;
}

extern "C" rtp_status rtp_ring_set_ablation(rtp_ring *r, int rotate, int compute)
{
    if (!r) return fail(RTP_ERR_INVALID, "rtp_ring_set_ablation: null ring");
    return set_ablation(r, rotate, compute);
}

extern "C" rtp_status rtp_ring_begin(rtp_ring *r, rtp_pass pass)
{
    if (!r) return fail(RTP_ERR_INVALID, "rtp_ring_begin: null ring");
    if (pass != RTP_PASS_FWD && pass != RTP_PASS_BWD) return fail(RTP_ERR_INVALID, "rtp_ring_begin: bad pass");
    if (r->pass != RTP_PASS_IDLE) return fail(RTP_ERR_STATE, "rtp_ring_begin: a pass is already open");
    const int n = r->d.n, rank = r->d.rank;
    if (pass == RTP_PASS_BWD && r->resident != (rank + 1) % n)
        return fail(RTP_ERR_STATE, "rtp_ring_begin: backward needs shard %d resident (forward pass first), have %d",
                    (rank + 1) % n, r->resident);
    RTP_TRY(refuse_capture(r, "rtp_ring_begin"));
    RTP_TRY(ensure_events(r));
    RTP_TRY(begin_join(r));
    r->joined = false;
    r->pass = pass;
    r->rotations = 0;
    r->executed = 0;
    for (rtp_linear *l : r->linears) l->next_step = 0;
    if (pass == RTP_PASS_FWD) {
        // the worker starts on its own shard: the one a backward pass ended on, if it is still in its buffer
        // (Design section, workflow paragraph: the backward rotation ends on the worker's own shard)
        if (r->w_held && r->resident == rank && r->abl_rotate) {
            r->base_idx = r->res_idx;
        } else {
            r->res_idx = 0;
            r->base_idx = 0;
            r->resident = rank;
            RTP_TRY(copy_async(r, r->d.buf_w_dev[0], r->home_w(rank), r->d.w_bytes, r->cs()));
            r->rec(TR_W_IN, -1, rank, 0);
            r->w_held = r->abl_rotate;
        }
    } else {
        // gradient shards come into being where the weights ended the forward pass
        r->base_idx = r->res_idx;
        // The gradient transfers of the pass's start run on the stage stream: only the weight-gradient kernels
        // (auxiliary stream, or the compute stream when there is none) wait for them, the first input-gradient
        // kernels do not.  cross_join above has ordered the stage stream after everything enqueued so far.
        hipStream_t gs = r->ss();
        if (r->d.g_bytes && r->res_g >= 0) {
            // the gradient shard the previous backward pass ended on (the worker's own) is still in the
            // buffer: it goes back to its slot before the buffer takes the shard this pass starts with
            RTP_TRY(copy_async(r, r->home_g(r->res_g), r->d.buf_g_dev[r->res_g_idx], r->d.g_bytes, gs));
            r->rec(TR_G_OUT, -1, r->res_g, r->res_g_idx);
        }
        r->res_g_idx = 0;
        r->res_g = r->resident;
        if (r->d.g_bytes) {
            RTP_TRY(copy_async(r, r->d.buf_g_dev[0], r->home_g(r->resident), r->d.g_bytes, gs));
            r->rec(TR_G_IN, -1, r->resident, 0);
            if (!r->dry && gs != r->cs()) {
                HIP_TRY(hipEventRecord(r->ev_g0, gs));
                HIP_TRY(hipStreamWaitEvent(r->as(), r->ev_g0, 0));
            }
        }
    }
    return RTP_OK;
}

extern "C" rtp_status rtp_ring_seek_bwd_start(rtp_ring *r)
{
    if (!r) return fail(RTP_ERR_INVALID, "null ring");
    if (r->pass != RTP_PASS_IDLE) return fail(RTP_ERR_STATE, "rtp_ring_seek_bwd_start: a pass is open");
    RTP_TRY(refuse_capture(r, "rtp_ring_seek_bwd_start"));
    RTP_TRY(ensure_events(r));
    RTP_TRY(cross_join(r));
    const int k = (r->d.rank + 1) % r->d.n;
    r->res_idx = 0;
    r->resident = k;
    RTP_TRY(copy_async(r, r->d.buf_w_dev[0], r->home_w(k), r->d.w_bytes, r->cs()));
    r->rec(TR_W_IN, -1, k, 0);
    r->w_held = r->abl_rotate;
    return RTP_OK;
}

// The transfers of one rotation.  Staged modes call this from rtp_rotate_step
// on the stage stream; the blocking mode calls it on the compute stream when
// the next step's first kernel is about to be enqueued.
static rtp_status do_rotation(rtp_ring *r, int step)
{
    const bool bwd = r->pass == RTP_PASS_BWD;
    const int k = r->shard_at(step), kin = r->shard_at(step + 1);
    const int src = r->w_idx(step), dst = r->w_idx(step + 1);
    hipStream_t s = r->ss();
    const bool blocking = r->d.mode == RTP_INPLACE_BLOCKING;
    if (!r->dry && !blocking) {
        // the staging buffer was resident one step ago: wait for its readers
        HIP_TRY(hipEventRecord(r->ev_free, r->cs()));
        HIP_TRY(hipStreamWaitEvent(s, r->ev_free, 0));
        if (r->as() != r->cs()) {
            // ... on the auxiliary stream too (the input-partitioned forward GEMM runs there)
            HIP_TRY(hipEventRecord(r->ev_free2, r->as()));
            HIP_TRY(hipStreamWaitEvent(s, r->ev_free2, 0));
        }
    }
    if (!r->dry && blocking && r->as() != r->cs()) {
        // the exchange runs on the compute stream: the weight-gradient kernels of the step that
        // just ended (auxiliary stream) must be done with the gradient shard first
        HIP_TRY(hipEventRecord(r->ev_join, r->as()));
        HIP_TRY(hipStreamWaitEvent(r->cs(), r->ev_join, 0));
    }
    // send the held weights to their next holder, receive the next shard; with two gradient buffers the next
    // gradient shard comes in with them (one launch for the three transfers)
    if (bwd && r->d.g_bytes && r->d.mode == RTP_DOUBLE_BUFFER && src != dst) {
        const int gdst = r->g_idx(step + 1);
        CopyBatch b;
        RTP_TRY(copy_batch_add(r, b, r->d.buf_w_dev[dst], r->home_w(kin), r->d.w_bytes, s));
        RTP_TRY(copy_batch_add(r, b, r->d.buf_g_dev[gdst], r->home_g(kin), r->d.g_bytes, s));
        RTP_TRY(copy_batch_add(r, b, r->home_w(k), r->d.buf_w_dev[src], r->d.w_bytes, s));
        RTP_TRY(copy_batch_flush(r, b, s, r->ev_w[(step + 1) & 1]));
        r->rec(TR_W_OUT, step, k, src);
        r->rec(TR_W_IN, step, kin, dst);
        r->rec(TR_G_IN, step, kin, gdst);
        if (!r->dry) HIP_TRY(hipEventRecord(r->ev_g[(step + 1) & 1], s));
        return RTP_OK;
    }
    RTP_TRY(rotate_async(r, r->home_w(k), r->d.buf_w_dev[src], r->d.buf_w_dev[dst], r->home_w(kin), r->d.w_bytes, s,
                         blocking ? nullptr : r->ev_w[(step + 1) & 1]));
    r->rec(TR_W_OUT, step, k, src);
    r->rec(TR_W_IN, step, kin, dst);
    if (bwd && r->d.g_bytes) {
        if (r->d.mode == RTP_DOUBLE_BUFFER) {
            const int gdst = r->g_idx(step + 1);
            RTP_TRY(copy_async(r, r->d.buf_g_dev[gdst], r->home_g(kin), r->d.g_bytes, s, r->ev_g[(step + 1) & 1]));
            r->rec(TR_G_IN, step, kin, gdst);
        } else if (blocking) {
            RTP_TRY(rotate_async(r, r->home_g(k), r->d.buf_g_dev[0], r->d.buf_g_dev[0], r->home_g(kin), r->d.g_bytes, s));
            r->rec(TR_G_OUT, step, k, 0);
            r->rec(TR_G_IN, step, kin, 0);
        }
        // RTP_INPLACE_STAGED: each linear exchanges its part right after its dW kernel
    }
    return RTP_OK;
}

extern "C" rtp_status rtp_rotate_step(rtp_ring *r, int direction, int step)
{
    if (!r) return fail(RTP_ERR_INVALID, "rtp_rotate_step: null ring");
    if (r->pass == RTP_PASS_IDLE) return fail(RTP_ERR_STATE, "rtp_rotate_step: no pass is open");
    const int want = r->pass == RTP_PASS_FWD ? RTP_CW : RTP_CCW;
    if (direction != want)
        return fail(RTP_ERR_STATE, "rtp_rotate_step: direction %d does not match the open pass", direction);
    if (step != r->rotations)
        return fail(RTP_ERR_STATE, "rtp_rotate_step: step %d out of order (next is %d)", step, r->rotations);
    if (step >= r->d.n - 1)
        return fail(RTP_ERR_STATE, "rtp_rotate_step: a pass of n=%d steps rotates n-1 times; step %d is past the last",
                    r->d.n, step);
    for (rtp_linear *l : r->linears)
        if (l->next_step < step)
            return fail(RTP_ERR_STATE, "rtp_rotate_step: a linear has not been issued for step %d yet", step - 1);
        else if (l->next_step > step)
            return fail(RTP_ERR_STATE, "rtp_rotate_step: must precede the linear calls of step %d", step);
    if (r->abl_rotate && r->d.mode != RTP_INPLACE_BLOCKING) RTP_TRY(do_rotation(r, step));
    r->rotations = step + 1;
    return RTP_OK;
}

// Called by every linear (or unit) before it enqueues kernels for `step`; next_step is the caller's own count.
static rtp_status enter_step(rtp_ring *r, int next_step, int step, rtp_pass pass, const char *who)
{
    if (r->pass != pass) return fail(RTP_ERR_STATE, "%s: the matching pass is not open", who);
    if (step != next_step)
        return fail(RTP_ERR_STATE, "%s: step %d out of order (next is %d)", who, step, next_step);
    if (step >= r->d.n) return fail(RTP_ERR_STATE, "%s: step %d past the last (n=%d)", who, step, r->d.n);
    if (step > 0 && r->rotations < step)
        return fail(RTP_ERR_STATE, "%s: the shard of step %d has not been staged (rtp_rotate_step(%d) missing)", who,
                    step, step - 1);
    if (step < r->d.n - 1 && r->rotations <= step)
        return fail(RTP_ERR_STATE, "%s: call rtp_rotate_step(%d) before the step's linears", who, step);
    if (r->abl_rotate) {
        if (r->d.mode == RTP_INPLACE_BLOCKING) {
            while (r->executed < step) {
                RTP_TRY(do_rotation(r, r->executed));
                r->executed++;
            }
        } else if (step > 0 && !r->dry) {
            HIP_TRY(hipStreamWaitEvent(r->cs(), r->ev_w[step & 1], 0));
        }
        r->resident = r->shard_at(step);
        r->res_idx = r->w_idx(step);
        if (pass == RTP_PASS_BWD) {
            r->res_g = r->resident;
            r->res_g_idx = r->g_idx(step);
        }
    }
    return RTP_OK;
}

extern "C" rtp_status rtp_ring_end(rtp_ring *r)
{
    if (!r) return fail(RTP_ERR_INVALID, "rtp_ring_end: null ring");
    if (r->pass == RTP_PASS_IDLE) return fail(RTP_ERR_STATE, "rtp_ring_end: no pass is open");
    for (rtp_linear *l : r->linears)
        if (l->next_step != r->d.n) return fail(RTP_ERR_STATE, "rtp_ring_end: steps remain");
    if (r->linears.empty() && r->rotations != r->d.n - 1) return fail(RTP_ERR_STATE, "rtp_ring_end: rotations remain");
    if (r->linears.empty() && r->abl_rotate) {
        // a bare ring (no linears): finish the bookkeeping the linears would have done
        if (r->d.mode == RTP_INPLACE_BLOCKING)
            while (r->executed < r->d.n - 1) {
                RTP_TRY(do_rotation(r, r->executed));
                r->executed++;
            }
        r->resident = r->shard_at(r->d.n - 1);
        r->res_idx = r->w_idx(r->d.n - 1);
    }
    if (!r->abl_rotate) {
        // keep the shard ids consistent even though nothing moved
        r->resident = r->shard_at(r->d.n - 1);
        r->w_held = false;
    }
    r->pass = RTP_PASS_IDLE;
    // the pass is complete on the compute stream only once the stage stream's last transfers are:
    // a caller that waits on (or captures) the compute stream alone then sees the whole pass
    if (!r->dry && r->events_ready) {
        if (r->cs() != r->ss()) {
            HIP_TRY(hipEventRecord(r->ev_join, r->ss()));
            HIP_TRY(hipStreamWaitEvent(r->cs(), r->ev_join, 0));
        }
        if (r->cs() != r->as() && r->pass_uses_as) {
            HIP_TRY(hipEventRecord(r->ev_join, r->as()));
            HIP_TRY(hipStreamWaitEvent(r->cs(), r->ev_join, 0));
        }
        r->joined = true;
    }
    r->pass_uses_as = true;
    return RTP_OK;
}

extern "C" rtp_status rtp_ring_abort(rtp_ring *r)
{
    if (!r) return fail(RTP_ERR_INVALID, "rtp_ring_abort: null ring");
    if (r->pass == RTP_PASS_IDLE) return RTP_OK;
    // whatever the streams still hold runs to its end before anybody reuses the buffers
    rtp_status st = (r->dry || !r->events_ready) ? RTP_OK : cross_join(r);
    r->pass = RTP_PASS_IDLE;
    r->joined = false;
    r->pass_uses_as = true;
    r->resident = -1;
    r->w_held = false;
    r->res_g = -1;
    r->rotations = 0;
    r->executed = 0;
    for (rtp_linear *l : r->linears) l->next_step = 0;
    return st;
}

// error path of the calls that run a whole pass: leave the ring usable, keep the first error's text
static rtp_status close_failed_pass(rtp_ring *r, rtp_status s)
{
    if (s == RTP_OK || r->pass == RTP_PASS_IDLE) return s;
    char keep[sizeof g_err];
    memcpy(keep, g_err, sizeof keep);
    (void)rtp_ring_abort(r);
    memcpy(g_err, keep, sizeof keep);
    return s;
}

extern "C" rtp_status rtp_ring_flush(rtp_ring *r)
{
    if (!r) return fail(RTP_ERR_INVALID, "rtp_ring_flush: null ring");
    if (r->pass != RTP_PASS_IDLE) return fail(RTP_ERR_STATE, "rtp_ring_flush: a pass is open");
    if (r->resident < 0) return RTP_OK;
    RTP_TRY(refuse_capture(r, "rtp_ring_flush"));
    RTP_TRY(ensure_events(r));
    RTP_TRY(cross_join(r));
    RTP_TRY(copy_async(r, r->home_w(r->resident), r->d.buf_w_dev[r->res_idx], r->d.w_bytes, r->cs()));
    r->rec(TR_W_OUT, -1, r->resident, r->res_idx);
    r->w_held = false; // the store may be written from here on (an optimizer step): the next forward pass loads anew
    if (r->d.g_bytes && r->res_g >= 0) {
        RTP_TRY(copy_async(r, r->home_g(r->res_g), r->d.buf_g_dev[r->res_g_idx], r->d.g_bytes, r->cs()));
        r->rec(TR_G_OUT, -1, r->res_g, r->res_g_idx);
        r->res_g = -1; // the slot is current: the next backward pass has nothing to write back
    }
    return RTP_OK;
}

extern "C" rtp_status rtp_ring_zero_grads(rtp_ring *r)
{
    if (!r) return fail(RTP_ERR_INVALID, "rtp_ring_zero_grads: null ring");
    if (r->pass != RTP_PASS_IDLE) return fail(RTP_ERR_STATE, "rtp_ring_zero_grads: a pass is open");
    RTP_TRY(refuse_capture(r, "rtp_ring_zero_grads"));
    RTP_TRY(ensure_events(r));
    RTP_TRY(cross_join(r));
    if (!r->dry && r->d.g_bytes) HIP_TRY(launch_fill_zero(r->d.home_g_dev, (size_t)r->d.n * r->d.g_bytes, r->cs()));
    r->res_g = -1; // the copy in the worker's buffer is dropped with the rest
    return RTP_OK;
}

extern "C" rtp_status rtp_ring_sync(rtp_ring *r)
{
    if (!r) return fail(RTP_ERR_INVALID, "rtp_ring_sync: null ring");
    if (r->dry) return RTP_OK;
    HIP_TRY(hipStreamSynchronize(r->cs()));
    if (r->ss() != r->cs()) HIP_TRY(hipStreamSynchronize(r->ss()));
    if (r->as() != r->cs()) HIP_TRY(hipStreamSynchronize(r->as()));
    HIP_TRY(hipGetLastError());
    return RTP_OK;
}

// ---------------------------------------------------------------------------
// linear
// ---------------------------------------------------------------------------
static size_t esize(rtp_dtype t) { return t == RTP_F32 ? 4 : 2; }

// Entries of the bias piece an input-partitioned layer's shard carries: ceil(O / n), rounded up so
// that the piece is a whole number of 16-byte units in the parameter's and the gradient's type.
extern "C" int64_t rtp_bias_piece_width(int64_t O, int n, rtp_dtype dtype)
{
    if (O <= 0 || n < 1) return -1;
    const int64_t p = (O + n - 1) / n, al = dtype == RTP_F32 ? 4 : 8;
    return (p + al - 1) / al * al;
}

static size_t shard_bytes(const rtp_linear_desc *d, int n, size_t es)
{
    if (!d || n <= 0 || d->I <= 0 || d->O <= 0) return 0;
    const int64_t o = rtp_shard_width(d->split == RTP_SPLIT_OUT ? d->O : d->I, n, d->dtype);
    if (o <= 0) return 0;
    const size_t other = (size_t)(d->split == RTP_SPLIT_OUT ? d->I : d->O);
    const size_t bias = !d->has_bias ? 0 : d->split == RTP_SPLIT_OUT ? (size_t)o : (size_t)rtp_bias_piece_width(d->O, n, d->dtype);
    const size_t elems = (size_t)o * other + bias;
    return (elems * es + 15) & ~(size_t)15;
}

extern "C" size_t rtp_linear_shard_w_bytes(const rtp_linear_desc *d, int n) { return d ? shard_bytes(d, n, esize(d->dtype)) : 0; }
extern "C" size_t rtp_linear_shard_g_bytes(const rtp_linear_desc *d, int n) { return d ? shard_bytes(d, n, 4) : 0; }

extern "C" rtp_status rtp_linear_create(rtp_linear **out, rtp_ring *ring, const rtp_linear_desc *d)
{
    if (!out || !ring || !d) return fail(RTP_ERR_INVALID, "rtp_linear_create: null argument");
    *out = nullptr;
    if (ring->pass != RTP_PASS_IDLE) return fail(RTP_ERR_STATE, "rtp_linear_create: a pass is open");
    if (d->T < 0 || d->I <= 0 || d->O <= 0) return fail(RTP_ERR_SHAPE, "rtp_linear_create: T >= 0, I > 0, O > 0 needed");
    if (d->T > 0x7fffffff || d->I > 0x7fffffff || d->O > 0x7fffffff)
        return fail(RTP_ERR_SHAPE, "rtp_linear_create: a dimension exceeds 2^31-1");
    if (d->split != RTP_SPLIT_OUT && d->split != RTP_SPLIT_IN) return fail(RTP_ERR_INVALID, "bad split");
    if (d->dtype != RTP_F32 && d->dtype != RTP_BF16 && d->dtype != RTP_F16) return fail(RTP_ERR_INVALID, "bad dtype");
    if (d->grad_dtype != RTP_F32)
        return fail(RTP_ERR_UNSUPPORTED, "rtp_linear_create: gradient shards are kept in fp32");
    if (d->act < RTP_ACT_NONE || d->act > RTP_ACT_SWIGLU) return fail(RTP_ERR_INVALID, "bad activation");
    const int n = ring->d.n;
    const int64_t part = d->split == RTP_SPLIT_OUT ? d->O : d->I;
    if (part % n != 0 && d->act == RTP_ACT_SWIGLU)
        return fail(RTP_ERR_SHAPE, "rtp_linear_create: n=%d does not divide the partitioned dimension %lld of a gated layer "
                                   "(the MLP unit pads its hidden width itself: rtp_mlp_hidden_width)", n, (long long)part);
    const int64_t o = rtp_shard_width(part, n, d->dtype);
    if (o <= 0)
        return fail(RTP_ERR_SHAPE, "rtp_linear_create: dimension %lld cannot be split into n=%d non-empty aligned shards",
                    (long long)part, n);
    if (d->act == RTP_ACT_SWIGLU && d->split == RTP_SPLIT_OUT && (o & 1))
        return fail(RTP_ERR_SHAPE, "rtp_linear_create: a (gate, up) shard needs an even width");
    if (d->dtype != RTP_F32) {
        const int64_t half = (d->act == RTP_ACT_SWIGLU && d->split == RTP_SPLIT_OUT) ? o / 2 : o;
        if ((d->I & 7) || (d->O & 7) || (o & 7) || (half & 7))
            return fail(RTP_ERR_SHAPE, "rtp_linear_create: 16-bit kernels need I, O and the shard width to be multiples of 8");
    }
    if (d->dtype == RTP_F16) {
        // fp16 runs on the tiled kernel only: every contraction length (the batch, the shard width and
        // the dimension that is not partitioned) must be a multiple of 32
        const int64_t other = d->split == RTP_SPLIT_OUT ? d->I : d->O;
        if ((d->T & 31) || (o & 31) || (other & 31) || (part & 31))
            return fail(RTP_ERR_UNSUPPORTED, "rtp_linear_create: fp16 inputs need T, the shard width and the other "
                                             "matrix dimension to be multiples of 32");
    }
    const size_t wsz = rtp_linear_shard_w_bytes(d, n);   // a padded shard is stored at its full width
    const size_t gsz = rtp_linear_shard_g_bytes(d, n);
    if ((d->w_offset & 15) || (d->g_offset & 15)) return fail(RTP_ERR_SHAPE, "rtp_linear_create: offsets must be multiples of 16");
    if (d->w_offset + wsz > ring->d.w_bytes || d->g_offset + gsz > ring->d.g_bytes)
        return fail(RTP_ERR_SHAPE, "rtp_linear_create: the shard does not fit the ring's slot");
    if (!ring->dry && d->T > 0) {
        if (d->act != RTP_ACT_NONE && !d->preact_dev)
            return fail(RTP_ERR_INVALID, "rtp_linear_create: an activation needs the pre-activation buffer");
    }
    rtp_linear *l = new (std::nothrow) rtp_linear;
    if (!l) return fail(RTP_ERR_INVALID, "out of host memory");
    l->ring = ring;
    l->d = *d;
    l->o = o;
    l->w_shard_bytes = wsz;
    l->g_shard_bytes = gsz;
    if (ring->events_ready) {
        if (hipEventCreateWithFlags(&l->ev_dw, hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&l->ev_g_in, hipEventDisableTiming) != hipSuccess) {
            delete l;
            return fail(RTP_ERR_HIP, "rtp_linear_create: hipEventCreate failed");
        }
    }
    ring->linears.push_back(l);
    *out = l;
    return RTP_OK;
}

extern "C" rtp_status rtp_linear_destroy(rtp_linear *l)
{
    if (!l) return RTP_OK;
    rtp_ring *r = l->ring;
    if (r->pass != RTP_PASS_IDLE) return fail(RTP_ERR_STATE, "rtp_linear_destroy: a pass is open");
    r->linears.erase(std::remove(r->linears.begin(), r->linears.end(), l), r->linears.end());
    if (l->ev_dw) (void)hipEventDestroy(l->ev_dw);
    if (l->ev_g_in) (void)hipEventDestroy(l->ev_g_in);
    delete l;
    return RTP_OK;
}

static int fwd_act_epi(rtp_act a)
{
    return a == RTP_ACT_GELU_ERF ? EPI_GELU_ERF_FWD : a == RTP_ACT_GELU_TANH ? EPI_GELU_TANH_FWD : EPI_SWIGLU_FWD;
}
static int bwd_act_epi(rtp_act a)
{
    return a == RTP_ACT_GELU_ERF ? EPI_GELU_ERF_BWD : a == RTP_ACT_GELU_TANH ? EPI_GELU_TANH_BWD : EPI_SWIGLU_BWD;
}

// epilogue of a result that is summed over the n steps
static int acc_epi(int step, int n) { return n == 1 ? EPI_STORE : step == 0 ? EPI_ACC_FIRST : step == n - 1 ? EPI_ACC_LAST : EPI_ACC_ADD; }

// test aid (rtp_ring_set_test_delay, rtp_ring_set_test_delay_compute): hold the auxiliary or the compute stream
// back ahead of a GEMM it is about to run
static rtp_status aux_delay(rtp_ring *r, hipStream_t st)
{
    if (r->delay_aux_ticks > 0 && st == r->as() && r->as() != r->cs())
        HIP_TRY(launch_clock_probe(r->delay_out + 2, r->delay_aux_ticks, st));
    if (r->delay_compute_ticks > 0 && st == r->cs())
        HIP_TRY(launch_clock_probe(r->delay_compute_out, r->delay_compute_ticks, st));
    return RTP_OK;
}

static rtp_status gemm(rtp_linear *l, int layout, GemmArgs &a, hipStream_t st)
{
    rtp_ring *r = l->ring;
    if (r->dry || !r->abl_compute) return RTP_OK;
    RTP_TRY(aux_delay(r, st));
    if (l->d.dtype != RTP_F32) {
        a.elem = l->d.dtype == RTP_F16 ? ELEM_F16 : ELEM_BF16;
        HIP_TRY(timed_launch(layout, 2.0 * a.M * a.N * a.K, st, [&] { return launch_gemm_bf16(layout, a, 0, st); }));
    } else {
        HIP_TRY(timed_launch(layout, 2.0 * a.M * a.N * a.K, st, [&] { return launch_gemm_f32(layout, a, st); }));
    }
    return RTP_OK;
}

// whether the layer's steps meet in an fp32 accumulator (16-bit layer, more than one step)
static bool needs_acc(const rtp_linear *l) { return l->d.dtype != RTP_F32 && l->ring->d.n > 1 && l->d.T > 0 && !l->ring->dry; }

// `acc`: the fp32 cross-step accumulator of an input-partitioned layer (null where none is needed)
static rtp_status linear_fwd_step(rtp_linear *l, int step, const void *X, void *Y, float *acc, const char *who)
{
    rtp_ring *r = l->ring;
    if (!r->dry && l->d.T > 0 && (!X || !Y)) return fail(RTP_ERR_INVALID, "%s: null tensor", who);
    if (l->d.split == RTP_SPLIT_IN && needs_acc(l) && !acc)
        return fail(RTP_ERR_INVALID, "%s: the layer was created without its fp32 cross-step accumulator", who);
    RTP_TRY(enter_step(r, l->next_step, step, RTP_PASS_FWD, who));
    const rtp_linear_desc &d = l->d;
    const int n = r->d.n;
    const int k = r->abl_rotate ? r->resident : rtp_fwd_shard(r->d.rank, step, n);
    const size_t es = esize(d.dtype);
    const char *Wk = (const char *)r->d.buf_w_dev[r->res_idx] + d.w_offset;
    const int64_t o = l->o;
    // columns of this shard that exist (the last shard of a padded partition is narrower)
    const int64_t ov = std::min<int64_t>(o, (d.split == RTP_SPLIT_OUT ? d.O : d.I) - (int64_t)k * o);
    const bool f32 = d.dtype == RTP_F32;
    r->rec(TR_FWD, step, k, r->res_idx);
    GemmArgs a;
    memset(&a, 0, sizeof a);
    a.c_is_f32 = f32;
    // with an auxiliary stream and a second linear on the ring, two forward GEMMs share the machine
    const int fwd_share = (r->as() != r->cs() && r->linears.size() > 1) ? 2 : 1;
    a.cu_share = fwd_share;
    if (d.split == RTP_SPLIT_OUT) {
        a.A = X; a.lda = d.I;
        a.B = Wk; a.ldb = d.I;
        a.M = (int)d.T; a.N = (int)o; a.K = (int)d.I;
        if (d.has_bias) a.bias = Wk + (size_t)o * d.I * es; // the shard's bias entries follow its rows
        if (d.act == RTP_ACT_NONE) {
            a.N = (int)ov;
            a.epi = EPI_STORE;
            a.C = (char *)Y + (size_t)k * o * es; a.ldc = d.O;
            RTP_TRY(gemm(l, LAY_NT, a, r->cs()));
        } else {
            const bool gated = d.act == RTP_ACT_SWIGLU;
            const int64_t ow = gated ? o / 2 : ov, Ow = gated ? d.O / 2 : d.O;   // (a gated layer is never padded)
            char *pre = (char *)d.preact_dev + (size_t)k * o * es;
            char *Yk = (char *)Y + (size_t)k * (gated ? o / 2 : o) * es;
            a.N = (int)ov;
            if (!f32) {
                a.epi = fwd_act_epi(d.act);
                a.half = (int)(o / 2);
                a.aux = pre; a.ldaux = d.O;
                a.C = Yk; a.ldc = Ow;
                RTP_TRY(gemm(l, LAY_NT, a, r->cs()));
            } else {
                a.epi = EPI_STORE;
                a.C = pre; a.ldc = d.O;
                RTP_TRY(gemm(l, LAY_NT, a, r->cs()));
                if (!r->dry && r->abl_compute)
                    HIP_TRY(launch_act_f32(fwd_act_epi(d.act), (const float *)pre, d.O, nullptr, 0, (float *)Yk, Ow,
                                           (int)d.T, (int)ow, (int)(o / 2), r->cs()));
            }
        }
    } else {
        a.A = (const char *)X + (size_t)k * o * es; a.lda = d.I;
        a.B = Wk; a.ldb = o;
        a.M = (int)d.T; a.N = (int)d.O; a.K = (int)ov;
        a.C = Y; a.ldc = d.O;
        if (f32) {
            a.epi = step == 0 ? EPI_STORE : EPI_ACC_ADD;
        } else {
            a.epi = acc_epi(step, n);
            a.ws = acc; a.ldws = d.O;
        }
        // The partial products of the N steps only meet in the accumulator, so this GEMM can run
        // on the auxiliary stream beside the next step's output-partitioned GEMM.  It starts after
        // everything enqueued so far on the compute stream (its input may just have been produced
        // there) and after this step's shard has been staged.
        hipStream_t fs = r->as();
        if (!r->dry && fs != r->cs()) {
            HIP_TRY(hipEventRecord(r->ev_aux, r->cs()));
            HIP_TRY(hipStreamWaitEvent(fs, r->ev_aux, 0));
            if (r->abl_rotate && step > 0 && r->d.mode != RTP_INPLACE_BLOCKING)
                HIP_TRY(hipStreamWaitEvent(fs, r->ev_w[step & 1], 0));
        }
        // The bias of this layer is spread over the shards in pieces; shard k's piece, which follows
        // its matrix in the slot, is added to its entries of every output row at shard k's step:
        // onto the fp32 sum (after the kernel that starts it, before the kernel that rounds it),
        // or inside the kernel when there is only one step.
        const int64_t pb = d.has_bias ? rtp_bias_piece_width(d.O, n, d.dtype) : 0;
        const int64_t pv = d.has_bias ? std::max<int64_t>(0, std::min<int64_t>(pb, d.O - (int64_t)k * pb)) : 0;
        const char *bk = Wk + (size_t)d.O * o * es;
        const int belem = f32 ? -1 : d.dtype == RTP_F16 ? ELEM_F16 : ELEM_BF16;
        const bool live = pv > 0 && !r->dry && r->abl_compute && d.T > 0;
        float *bdst = (f32 ? (float *)Y : acc) + (size_t)k * pb;
        bool after = false;
        if (live) {
            if (f32 || (n > 1 && step == 0)) after = true;
            else if (n == 1) a.bias = bk;
            else HIP_TRY(launch_bias_add(belem, bdst, d.O, (int)d.T, (int)pv, bk, fs));
        }
        RTP_TRY(gemm(l, LAY_NT, a, fs));
        if (after) HIP_TRY(launch_bias_add(belem, bdst, d.O, (int)d.T, (int)pv, bk, fs));
    }
    l->next_step = step + 1;
    return RTP_OK;
}

extern "C" rtp_status rtp_linear_fwd(rtp_linear *l, int step, const void *X, void *Y)
{
    if (!l) return fail(RTP_ERR_INVALID, "rtp_linear_fwd: null linear");
    return linear_fwd_step(l, step, X, Y, l->d.acc_ws_dev, "rtp_linear_fwd");
}

// ---- the forward step for callers that cannot allocate --------------------------------------
// The fp32 cross-step accumulator of an input-partitioned layer is device memory beyond the
// layer's inputs and outputs.  rtp_linear_fwd takes it from the caller (acc_ws_dev); this variant
// takes it from a fixed array in the library's device image, so a caller that cannot call hipMalloc
// (graph capture around its own allocation-free code, a tight serving loop, a harness that forbids
// allocation) still gets the layer.  The array's name is a host-side stand-in for the symbol: only
// the address hipGetSymbolAddress returns, looked up once per device with that device current, is a
// device pointer, and only that address is ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[RTP_NOALLOC_ACC_BYTES];

constexpr int NOALLOC_MAX_DEVICES = 64;
static void *g_scratch_ptr[NOALLOC_MAX_DEVICES];
static std::mutex g_scratch_lock;

// device address of `scratch` on the current device
static rtp_status noalloc_scratch(float **out)
{
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= NOALLOC_MAX_DEVICES)
        return fail(RTP_ERR_UNSUPPORTED, "rtp_linear_fwd_noalloc: device ordinal %d is beyond the %d this entry point keeps a pointer for",
                    dev, NOALLOC_MAX_DEVICES);
    std::lock_guard<std::mutex> g(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(RTP_ERR_HIP, "rtp_linear_fwd_noalloc: hipGetSymbolAddress returned a null address");
        g_scratch_ptr[dev] = p;
    }
    *out = (float *)g_scratch_ptr[dev];
    return RTP_OK;
}

extern "C" rtp_status rtp_linear_fwd_noalloc(rtp_linear *l, int step, const void *X, void *Y)
{
    if (!l) return fail(RTP_ERR_INVALID, "rtp_linear_fwd_noalloc: null linear");
    const rtp_linear_desc &d = l->d;
    if (d.split != RTP_SPLIT_IN || d.dtype == RTP_F32)
        return fail(RTP_ERR_UNSUPPORTED, "rtp_linear_fwd_noalloc: for input-partitioned 16-bit layers (the ones whose steps "
                                         "meet in an fp32 accumulator); use rtp_linear_fwd for the others");
    const size_t need = (size_t)d.T * (size_t)d.O * sizeof(float);
    if (need > RTP_NOALLOC_ACC_BYTES)
        return fail(RTP_ERR_SHAPE, "rtp_linear_fwd_noalloc: the fp32 accumulator [T=%lld, O=%lld] takes %zu bytes, the "
                                   "library's fixed array holds %zu", (long long)d.T, (long long)d.O, need,
                    (size_t)RTP_NOALLOC_ACC_BYTES);
    float *acc = nullptr;
    if (needs_acc(l)) RTP_TRY(noalloc_scratch(&acc));
    // step 0 stores into the accumulator (EPI_ACC_FIRST), so nothing of the previous call's content
    // has to be cleared; steps 1 .. n-1 add onto what step 0 .. of the same pass left there
    return linear_fwd_step(l, step, X, Y, acc, "rtp_linear_fwd_noalloc");
}

extern "C" rtp_status rtp_linear_bwd(rtp_linear *l, int step, const void *X, const void *dY, void *dX)
{
    if (!l) return fail(RTP_ERR_INVALID, "rtp_linear_bwd: null linear");
    rtp_ring *r = l->ring;
    if (!r->dry && l->d.T > 0 && (!X || !dY)) return fail(RTP_ERR_INVALID, "rtp_linear_bwd: null tensor");
    if (l->d.split == RTP_SPLIT_OUT && dX && needs_acc(l) && !l->d.acc_ws_dev)
        return fail(RTP_ERR_INVALID, "rtp_linear_bwd: the layer was created without its fp32 cross-step accumulator");
    RTP_TRY(enter_step(r, l->next_step, step, RTP_PASS_BWD, "rtp_linear_bwd"));
    const rtp_linear_desc &d = l->d;
    const int n = r->d.n;
    const int k = r->abl_rotate ? r->resident : rtp_bwd_shard(r->d.rank, step, n);
    const size_t es = esize(d.dtype);
    const int64_t o = l->o;
    const int64_t ov = std::min<int64_t>(o, (d.split == RTP_SPLIT_OUT ? d.O : d.I) - (int64_t)k * o);
    const bool f32 = d.dtype == RTP_F32;
    const bool rotating = r->abl_rotate && step < n - 1;
    const bool staged_g = r->d.mode == RTP_INPLACE_STAGED;
    const int gi = r->res_g_idx;
    const char *Wk = (const char *)r->d.buf_w_dev[r->res_idx] + d.w_offset;
    float *Gk = (float *)((char *)r->d.buf_g_dev[gi] + d.g_offset);
    r->rec(TR_BWD, step, k, r->res_idx);

    // The weight-gradient kernel runs on the auxiliary stream when there is one, beside the
    // input-gradient kernels: shard GEMMs seldom fill the machine alone.  It starts after
    // everything enqueued so far on the compute stream (its dY may just have been produced there).
    hipStream_t ws = r->as();
    const bool split = ws != r->cs();
    if (!r->dry && split) {
        HIP_TRY(hipEventRecord(r->ev_aux, r->cs()));
        HIP_TRY(hipStreamWaitEvent(ws, r->ev_aux, 0));
    }
    // the gradient shard this step adds onto must have arrived
    if (!r->dry && r->abl_rotate && step > 0) {
        if (r->d.mode == RTP_DOUBLE_BUFFER)
            HIP_TRY(hipStreamWaitEvent(ws, r->ev_g[step & 1], 0));
        else if (staged_g)
            HIP_TRY(hipStreamWaitEvent(ws, l->ev_g_in, 0));
    }

    GemmArgs a;
    // ---- weight gradient, fused into the travelling gradient shard -----------
    memset(&a, 0, sizeof a);
    a.c_is_f32 = 1;
    a.epi = EPI_ACC_ADD;
    a.K = (int)d.T;
    if (d.split == RTP_SPLIT_OUT) {
        a.A = (const char *)dY + (size_t)k * o * es; a.lda = d.O;
        a.B = X; a.ldb = d.I;
        a.M = (int)ov; a.N = (int)d.I;
        a.ws = Gk; a.ldws = d.I;
    } else {
        a.A = dY; a.lda = d.O;
        a.B = (const char *)X + (size_t)k * o * es; a.ldb = d.I;
        a.M = (int)d.O; a.N = (int)ov;
        a.ws = Gk; a.ldws = o;
    }
    a.C = a.ws; a.ldc = a.ldws;
    a.cu_share = split ? 2 : 1;
    // The send of the gradient part is fused into the kernel that completes it: when the shard
    // moves on after this step, the sum (arriving content + this worker's contribution) is written
    // straight to where it travels to, instead of back into the buffer and copied from there.
    const bool moves_on = rotating && r->d.g_bytes && r->d.mode != RTP_INPLACE_BLOCKING;
    bool fused_send = moves_on && !f32 && !r->dry && r->abl_compute && d.T > 0;
    if (fused_send && gemm_bf16_pp_supported(LAY_TN, a)) {
        // not when the launcher would cut this GEMM's K loop into chunks (few output tiles, long
        // contraction): their partial sums need the plain `+=` form
        int ks = 1;
        gemm_bf16_pp_plan(LAY_TN, &a, 1, nullptr, nullptr, &ks);
        if (ks > 1) fused_send = false;
    }
    if (fused_send) {
        a.epi = EPI_ACC_LAST;
        a.C = r->home_g(k) + d.g_offset;
    }
    if (d.T > 0) RTP_TRY(gemm(l, LAY_TN, a, ws));
    if (d.has_bias && !r->dry && r->abl_compute) {
        // bias gradient: column sums of this shard's slice of dY, onto the entries that follow the
        // matrix gradient in the travelling shard (and out to where it travels, like the matrix part)
        // (input-partitioned layer: the shard carries a piece of the bias, the columns of dY that piece covers)
        const bool out_split = d.split == RTP_SPLIT_OUT;
        const int64_t pb = out_split ? o : rtp_bias_piece_width(d.O, n, d.dtype);
        const int64_t pv = out_split ? ov : std::max<int64_t>(0, std::min<int64_t>(pb, d.O - (int64_t)k * pb));
        const size_t boff = (out_split ? (size_t)o * d.I : (size_t)d.O * o) * 4;
        const float *gb_in = (const float *)((const char *)Gk + boff);
        float *gb_out = fused_send ? (float *)(r->home_g(k) + d.g_offset + boff) : (float *)((char *)Gk + boff);
        const int elem = f32 ? -1 : d.dtype == RTP_F16 ? ELEM_F16 : ELEM_BF16;
        HIP_TRY(launch_colsum(elem, (const char *)dY + (size_t)k * pb * es, d.O, (int)d.T, (int)pv, gb_in, gb_out, ws));
        // (padding entries of a partly filled shard are zero in the buffer and in the slot alike, and nobody
        // writes them)
    }

    // ---- hand the gradient part to the stage stream ---------------------------
    if (moves_on) {
        const int kin = rtp_bwd_shard(r->d.rank, step + 1, n);
        if (!r->dry) {
            HIP_TRY(hipEventRecord(l->ev_dw, ws));
            HIP_TRY(hipStreamWaitEvent(r->ss(), l->ev_dw, 0));
        }
        char *part = (char *)r->d.buf_g_dev[gi] + d.g_offset;
        if (!fused_send) RTP_TRY(copy_async(r, r->home_g(k) + d.g_offset, part, l->g_shard_bytes, r->ss()));
        r->rec(TR_G_OUT, step, k, gi);
        if (staged_g) {
            // in place: the next shard's part comes into the buffer the kernel has just finished with
            RTP_TRY(copy_async(r, part, r->home_g(kin) + d.g_offset, l->g_shard_bytes, r->ss(), l->ev_g_in));
            r->rec(TR_G_IN, step, kin, gi);
        }
    }

    // ---- input gradient ----------------------------------------------------------
    if ((dX && d.T > 0) || r->dry) {
        memset(&a, 0, sizeof a);
        a.c_is_f32 = f32;
        a.cu_share = split ? 2 : 1;
        if (d.split == RTP_SPLIT_OUT) {
            a.A = (const char *)dY + (size_t)k * o * es; a.lda = d.O;
            a.B = Wk; a.ldb = d.I;
            a.M = (int)d.T; a.N = (int)d.I; a.K = (int)ov;
            a.C = dX; a.ldc = d.I;
            if (f32) {
                a.epi = step == 0 ? EPI_STORE : EPI_ACC_ADD;
            } else {
                a.epi = acc_epi(step, n);
                a.ws = d.acc_ws_dev; a.ldws = d.I;
            }
            RTP_TRY(gemm(l, LAY_NN, a, r->cs()));
        } else {
            a.A = dY; a.lda = d.O;
            a.B = Wk; a.ldb = o;
            a.M = (int)d.T; a.N = (int)o; a.K = (int)d.O;
            if (d.act == RTP_ACT_NONE) {
                a.N = (int)ov;
                a.epi = EPI_STORE;
                a.C = (char *)dX + (size_t)k * o * es; a.ldc = d.I;
                RTP_TRY(gemm(l, LAY_NN, a, r->cs()));
            } else {
                const bool gated = d.act == RTP_ACT_SWIGLU;
                const int64_t P = gated ? 2 * d.I : d.I, po = gated ? 2 * o : o;
                char *out = (char *)dX + (size_t)k * po * es;
                const char *pre = (const char *)d.preact_dev + (size_t)k * po * es;
                a.N = (int)ov;                                                   // (a gated layer is never padded)
                if (!f32) {
                    a.epi = bwd_act_epi(d.act);
                    a.half = (int)o;
                    a.aux = (void *)pre; a.ldaux = P;
                    a.C = out; a.ldc = P;
                    RTP_TRY(gemm(l, LAY_NN, a, r->cs()));
                } else {
                    // the plain product lands in the last o columns of the slice, then the
                    // activation's derivative is applied elementwise, in place
                    float *tmp = (float *)out + (gated ? o : 0);
                    a.epi = EPI_STORE;
                    a.C = tmp; a.ldc = P;
                    RTP_TRY(gemm(l, LAY_NN, a, r->cs()));
                    if (!r->dry && r->abl_compute)
                        HIP_TRY(launch_act_f32(bwd_act_epi(d.act), (const float *)pre, P, tmp, P, (float *)out, P,
                                               (int)d.T, (int)ov, (int)o, r->cs()));
                }
            }
        }
    }
    l->next_step = step + 1;
    return RTP_OK;
}

// ---------------------------------------------------------------------------
// MLP unit
// ---------------------------------------------------------------------------
struct rtp_mlp {
    rtp_mlp_desc d;
    rtp_ring *ring = nullptr;
    rtp_linear *l1 = nullptr, *l2 = nullptr;
};

static bool mlp_gated(const rtp_mlp_desc *d) { return d->act == RTP_ACT_SWIGLU; }

// the unit's two linears: the first output-partitioned with the activation, the second input-partitioned
// The hidden width the unit computes on: O when n divides it, else n shards of the smallest aligned
// width that covers it (FlatParameter padding).  The padding units have zero weights and biases, so
// their pre-activations are 0, their activations act(0) = 0 (also silu(0) * 0 for the gated form),
// they add nothing to the second GEMM, and every gradient that belongs to them is an exact zero:
// the unit simply runs on an evenly divided hidden dimension of this width.
extern "C" int64_t rtp_mlp_hidden_width(const rtp_mlp_desc *d)
{
    if (!d || d->n < 1 || d->O <= 0) return -1;
    const int64_t o = rtp_shard_width(d->O, d->n, d->dtype);
    return o <= 0 ? -1 : o * d->n;
}

static void mlp_linear_descs(const rtp_mlp_desc *d, rtp_linear_desc *l1, rtp_linear_desc *l2)
{
    const int64_t p = mlp_gated(d) ? 2 : 1;
    const int64_t hw = rtp_mlp_hidden_width(d);
    memset(l1, 0, sizeof *l1);
    l1->T = d->T; l1->I = d->I; l1->O = p * hw;
    l1->split = RTP_SPLIT_OUT; l1->dtype = d->dtype; l1->grad_dtype = RTP_F32; l1->act = d->act;
    l1->preact_dev = d->preact_dev; l1->acc_ws_dev = d->acc_dx_dev;
    l1->has_bias = d->has_bias;
    memset(l2, 0, sizeof *l2);
    l2->T = d->T; l2->I = hw; l2->O = d->O2;
    l2->split = RTP_SPLIT_IN; l2->dtype = d->dtype; l2->grad_dtype = RTP_F32; l2->act = d->act;
    l2->preact_dev = d->preact_dev; l2->acc_ws_dev = d->acc_y_dev;
    l2->has_bias = d->has_bias;
    l2->w_offset = rtp_linear_shard_w_bytes(l1, d->n);
    l2->g_offset = rtp_linear_shard_g_bytes(l1, d->n);
}

extern "C" size_t rtp_mlp_slot_w_bytes(const rtp_mlp_desc *d)
{
    if (!d || d->n < 1 || d->O <= 0 || d->I <= 0 || d->O2 <= 0 || rtp_mlp_hidden_width(d) <= 0) return 0;
    rtp_linear_desc l1, l2;
    mlp_linear_descs(d, &l1, &l2);
    return l2.w_offset + rtp_linear_shard_w_bytes(&l2, d->n);
}

extern "C" size_t rtp_mlp_slot_g_bytes(const rtp_mlp_desc *d)
{
    if (!d || d->n < 1 || d->O <= 0 || d->I <= 0 || d->O2 <= 0 || rtp_mlp_hidden_width(d) <= 0) return 0;
    rtp_linear_desc l1, l2;
    mlp_linear_descs(d, &l1, &l2);
    return l2.g_offset + rtp_linear_shard_g_bytes(&l2, d->n);
}

extern "C" rtp_status rtp_mlp_create(rtp_mlp **out, const rtp_mlp_desc *d)
{
    if (!out || !d) return fail(RTP_ERR_INVALID, "rtp_mlp_create: null argument");
    *out = nullptr;
    if (d->act == RTP_ACT_NONE) return fail(RTP_ERR_INVALID, "rtp_mlp_create: an MLP block has an activation");
    if (d->n < 1 || d->O <= 0 || d->I <= 0 || d->O2 <= 0)
        return fail(RTP_ERR_SHAPE, "rtp_mlp_create: n >= 1 and positive sizes needed");
    if (rtp_mlp_hidden_width(d) <= 0)
        return fail(RTP_ERR_SHAPE, "rtp_mlp_create: a hidden width of %lld cannot be split into n=%d non-empty aligned shards",
                    (long long)d->O, d->n);
    rtp_ring_desc rd;
    memset(&rd, 0, sizeof rd);
    rd.n = d->n; rd.rank = d->rank; rd.mode = d->mode; rd.flags = d->flags;
    rd.w_bytes = rtp_mlp_slot_w_bytes(d);
    rd.g_bytes = rtp_mlp_slot_g_bytes(d);
    rd.home_w_dev = d->home_w_dev; rd.home_g_dev = d->home_g_dev;
    rd.buf_w_dev[0] = d->buf_w_dev[0]; rd.buf_w_dev[1] = d->buf_w_dev[1];
    rd.buf_g_dev[0] = d->buf_g_dev[0]; rd.buf_g_dev[1] = d->buf_g_dev[1];
    rd.compute_stream = d->compute_stream; rd.stage_stream = d->stage_stream; rd.aux_stream = d->aux_stream;
    rtp_mlp *m = new (std::nothrow) rtp_mlp;
    if (!m) return fail(RTP_ERR_INVALID, "out of host memory");
    m->d = *d;
    rtp_status s = rtp_ring_create(&m->ring, &rd);
    if (s != RTP_OK) { delete m; return s; }
    rtp_linear_desc l1, l2;
    mlp_linear_descs(d, &l1, &l2);
    s = rtp_linear_create(&m->l1, m->ring, &l1);
    if (s == RTP_OK) s = rtp_linear_create(&m->l2, m->ring, &l2);
    if (s == RTP_OK && !(d->flags & RTP_FLAG_DRY_RUN) && (!d->hidden_dev || !d->dpre_dev))
        s = fail(RTP_ERR_INVALID, "rtp_mlp_create: hidden/dpre buffers are missing");
    if (s != RTP_OK) {
        rtp_linear_destroy(m->l2);
        rtp_linear_destroy(m->l1);
        rtp_ring_destroy(m->ring);
        delete m;
        return s;
    }
    *out = m;
    return RTP_OK;
}

extern "C" rtp_status rtp_mlp_destroy(rtp_mlp *m)
{
    if (!m) return RTP_OK;
    RTP_TRY(rtp_linear_destroy(m->l2));
    RTP_TRY(rtp_linear_destroy(m->l1));
    RTP_TRY(rtp_ring_destroy(m->ring));
    delete m;
    return RTP_OK;
}

extern "C" rtp_ring *rtp_mlp_ring(rtp_mlp *m) { return m ? m->ring : nullptr; }

extern "C" rtp_status rtp_mlp_set_ablation(rtp_mlp *m, int rotate, int compute)
{
    if (!m) return fail(RTP_ERR_INVALID, "null mlp");
    return set_ablation(m->ring, rotate, compute);
}

// ---- grouped schedule of the MLP unit ---------------------------------------------------
// One rotation step of the unit holds GEMMs that do not depend on each other once the second
// linear lags the first by one step: forward, Z_t = X W1_t^T needs nothing from
// down_{t-1} = H_{t-1} W2_{t-1}^T; backward, dH_s = dY W2_s needs nothing from
// dX_{s-1} += dPre_{s-1} W1_{s-1}, and the two weight gradients of a step are independent.
// Each such pair has one operand layout and goes out as one group launch, whose tiles fill the
// machine where a shard GEMM alone leaves compute units idle.  The shard parts travel
// accordingly: the weights of the lagging linear stay one step longer, so a staging buffer is
// reused one launch later than in the step-by-step schedule; the buffers themselves (two
// weight slots, one or two gradient slots) and the bytes moved per step are the same.

struct MlpShapes {
    int64_t T, I, O2, P1, o1, o2, Ohid;
    size_t es, w_off2, g_off2;
    bool gated, has_bias;
    int n, belem;
    int64_t pb2;          // entries of the piece of the second linear's bias a shard carries
    // valid entries of piece k (the last pieces may be short or empty)
    int64_t pv2(int k) const { return std::max<int64_t>(0, std::min<int64_t>(pb2, O2 - (int64_t)k * pb2)); }
    // byte offsets inside a weight slot / a gradient slot of the two bias parts
    size_t wb1() const { return (size_t)o1 * I * es; }
    size_t wb2() const { return w_off2 + (size_t)O2 * o2 * es; }
    size_t gb1() const { return (size_t)o1 * I * 4; }
    size_t gb2() const { return g_off2 + (size_t)O2 * o2 * 4; }
};

static MlpShapes mlp_shapes(const rtp_mlp *m)
{
    MlpShapes h;
    h.gated = mlp_gated(&m->d);
    h.T = m->d.T; h.I = m->d.I; h.O2 = m->d.O2; h.Ohid = rtp_mlp_hidden_width(&m->d);
    h.P1 = (h.gated ? 2 : 1) * h.Ohid;
    h.o1 = h.P1 / m->d.n;
    h.o2 = h.Ohid / m->d.n;
    h.has_bias = m->d.has_bias != 0;
    h.n = m->d.n;
    h.belem = m->d.dtype == RTP_F16 ? ELEM_F16 : ELEM_BF16;
    h.pb2 = h.has_bias ? rtp_bias_piece_width(m->d.O2, m->d.n, m->d.dtype) : 0;
    h.es = esize(m->d.dtype);
    h.w_off2 = m->l2->d.w_offset;
    h.g_off2 = m->l2->d.g_offset;
    return h;
}

// Z_k = X W1_k^T with the activation fused (pre-activations kept for the backward pass)
static GemmArgs mlp_args_z(const rtp_mlp *m, const MlpShapes &h, int k, const void *X, const char *Wslot)
{
    GemmArgs a;
    memset(&a, 0, sizeof a);
    a.elem = m->d.dtype == RTP_F16 ? ELEM_F16 : ELEM_BF16;
    const int64_t ow = h.gated ? h.o1 / 2 : h.o1;
    a.A = X; a.lda = h.I;
    a.B = Wslot; a.ldb = h.I;
    a.M = (int)h.T; a.N = (int)h.o1; a.K = (int)h.I;
    a.epi = fwd_act_epi(m->d.act);
    a.half = (int)(h.o1 / 2);
    a.aux = (char *)m->d.preact_dev + (size_t)k * h.o1 * h.es; a.ldaux = h.P1;
    a.C = (char *)m->d.hidden_dev + (size_t)k * ow * h.es; a.ldc = h.Ohid;
    if (h.has_bias) a.bias = Wslot + h.wb1(); // the shard's bias entries follow its rows ((gate | up) order)
    return a;
}

// Y (+)= H_k W2_k^T, summed over the steps in fp32
static GemmArgs mlp_args_down(const rtp_mlp *m, const MlpShapes &h, int k, int step, const char *Wslot, void *Y)
{
    GemmArgs a;
    memset(&a, 0, sizeof a);
    a.elem = m->d.dtype == RTP_F16 ? ELEM_F16 : ELEM_BF16;
    a.A = (const char *)m->d.hidden_dev + (size_t)k * h.o2 * h.es; a.lda = h.Ohid;
    a.B = Wslot + h.w_off2; a.ldb = h.o2;
    a.M = (int)h.T; a.N = (int)h.O2; a.K = (int)h.o2;
    a.C = Y; a.ldc = h.O2;
    a.epi = acc_epi(step, m->d.n);
    a.ws = m->d.acc_y_dev; a.ldws = h.O2;
    if (h.has_bias && h.n == 1) a.bias = Wslot + h.wb2(); // one step: the whole bias, inside the kernel
    return a;
}

// Piece k of the second linear's bias onto the fp32 sum of the unit's output (n > 1): its place in the
// stream is after the launch that starts the sum (step 0) and before the launch of any later step.
static rtp_status mlp_bias2_add(rtp_mlp *m, const MlpShapes &h, int k, const char *Wslot, hipStream_t st)
{
    rtp_ring *r = m->ring;
    if (!h.has_bias || h.n == 1 || h.pv2(k) <= 0 || r->dry || !r->abl_compute || h.T <= 0) return RTP_OK;
    HIP_TRY(launch_bias_add(h.belem, m->d.acc_y_dev + (size_t)k * h.pb2, h.O2, (int)h.T, (int)h.pv2(k), Wslot + h.wb2(), st));
    return RTP_OK;
}

// The two bias gradients of step s (shard k) onto the travelling gradient shard in `Gslot`: column sums of
// dPre_k (first linear) and of the columns of dY that piece k of the second bias covers.  When the shard's
// gradient parts are sent by the kernels that complete them, the sums go straight to `home` as well.
static rtp_status mlp_bias_grads(rtp_mlp *m, const MlpShapes &h, int k, char *Gslot, char *home, const void *dY,
                                 bool first, bool second, hipStream_t st)
{
    rtp_ring *r = m->ring;
    if (!h.has_bias || r->dry || !r->abl_compute || h.T <= 0) return RTP_OK;
    char *dst = home ? home : Gslot;
    if (first)
        HIP_TRY(launch_colsum(h.belem, (const char *)m->d.dpre_dev + (size_t)k * h.o1 * h.es, h.P1, (int)h.T, (int)h.o1,
                              (const float *)(Gslot + h.gb1()), (float *)(dst + h.gb1()), st));
    if (second && h.pv2(k) > 0)
        HIP_TRY(launch_colsum(h.belem, (const char *)dY + (size_t)k * h.pb2 * h.es, h.O2, (int)h.T, (int)h.pv2(k),
                              (const float *)(Gslot + h.gb2()), (float *)(dst + h.gb2()), st));
    return RTP_OK;
}

// dPre_k = (dY W2_k) * act'(pre_k)
static GemmArgs mlp_args_dh(const rtp_mlp *m, const MlpShapes &h, int k, const char *Wslot, const void *dY)
{
    GemmArgs a;
    memset(&a, 0, sizeof a);
    a.elem = m->d.dtype == RTP_F16 ? ELEM_F16 : ELEM_BF16;
    a.A = dY; a.lda = h.O2;
    a.B = Wslot + h.w_off2; a.ldb = h.o2;
    a.M = (int)h.T; a.N = (int)h.o2; a.K = (int)h.O2;
    a.epi = bwd_act_epi(m->d.act);
    a.half = (int)h.o2;
    a.aux = (char *)m->d.preact_dev + (size_t)k * h.o1 * h.es; a.ldaux = h.P1;
    a.C = (char *)m->d.dpre_dev + (size_t)k * h.o1 * h.es; a.ldc = h.P1;
    return a;
}

// G2_k += dY^T H_k
static GemmArgs mlp_args_dw2(const rtp_mlp *m, const MlpShapes &h, int k, char *Gslot, const void *dY)
{
    GemmArgs a;
    memset(&a, 0, sizeof a);
    a.elem = m->d.dtype == RTP_F16 ? ELEM_F16 : ELEM_BF16;
    a.A = dY; a.lda = h.O2;
    a.B = (const char *)m->d.hidden_dev + (size_t)k * h.o2 * h.es; a.ldb = h.Ohid;
    a.M = (int)h.O2; a.N = (int)h.o2; a.K = (int)h.T;
    a.epi = EPI_ACC_ADD; a.c_is_f32 = 1;
    a.ws = (float *)(Gslot + h.g_off2); a.ldws = h.o2;
    a.C = a.ws; a.ldc = a.ldws;
    return a;
}

// G1_k += dPre_k^T X
static GemmArgs mlp_args_dw1(const rtp_mlp *m, const MlpShapes &h, int k, char *Gslot, const void *X)
{
    GemmArgs a;
    memset(&a, 0, sizeof a);
    a.elem = m->d.dtype == RTP_F16 ? ELEM_F16 : ELEM_BF16;
    a.A = (const char *)m->d.dpre_dev + (size_t)k * h.o1 * h.es; a.lda = h.P1;
    a.B = X; a.ldb = h.I;
    a.M = (int)h.o1; a.N = (int)h.I; a.K = (int)h.T;
    a.epi = EPI_ACC_ADD; a.c_is_f32 = 1;
    a.ws = (float *)Gslot; a.ldws = h.I;
    a.C = a.ws; a.ldc = a.ldws;
    return a;
}

// dX (+)= dPre_k W1_k, summed over the steps in fp32
static GemmArgs mlp_args_dx(const rtp_mlp *m, const MlpShapes &h, int k, int step, const char *Wslot, void *dX)
{
    GemmArgs a;
    memset(&a, 0, sizeof a);
    a.elem = m->d.dtype == RTP_F16 ? ELEM_F16 : ELEM_BF16;
    a.A = (const char *)m->d.dpre_dev + (size_t)k * h.o1 * h.es; a.lda = h.P1;
    a.B = Wslot; a.ldb = h.I;
    a.M = (int)h.T; a.N = (int)h.I; a.K = (int)h.o1;
    a.C = dX; a.ldc = h.I;
    a.epi = acc_epi(step, m->d.n);
    a.ws = m->d.acc_dx_dev; a.ldws = h.I;
    return a;
}

// whether the unit can run the grouped schedule: bf16, staged transfers, and all six GEMM
// shapes within what the ping-pong kernel takes
static bool mlp_grouped_ok(const rtp_mlp *m, const void *X, const void *Y, const void *dY, const void *dX)
{
    const rtp_ring *r = m->ring;
    if (r->dry || (m->d.flags & RTP_FLAG_STEPWISE) || m->d.dtype == RTP_F32 || m->d.T <= 0) return false;
    if (r->d.mode == RTP_INPLACE_BLOCKING) return false;
    const MlpShapes h = mlp_shapes(m);
    const char *W = (const char *)r->d.buf_w_dev[0];
    char *G = (char *)r->d.buf_g_dev[0];
    // dummy non-null tensors where a pass does not use one: only shapes and alignment matter here
    const void *x = X ? X : m->d.hidden_dev, *dy = dY ? dY : m->d.hidden_dev;
    void *y = Y ? (void *)Y : m->d.hidden_dev, *dx = dX ? (void *)dX : m->d.hidden_dev;
    const GemmArgs nt[2] = {mlp_args_z(m, h, 0, x, W), mlp_args_down(m, h, 0, 0, W, y)};
    const GemmArgs nn[2] = {mlp_args_dh(m, h, 0, W, dy), mlp_args_dx(m, h, 0, 0, W, dx)};
    const GemmArgs tn[2] = {mlp_args_dw1(m, h, 0, G, x), mlp_args_dw2(m, h, 0, G, dy)};
    for (int i = 0; i < 2; ++i) {
        if (!gemm_bf16_args_ok(LAY_NT, nt[i]) || !gemm_bf16_pp_supported(LAY_NT, nt[i])) return false;
        if (!gemm_bf16_args_ok(LAY_NN, nn[i]) || !gemm_bf16_pp_supported(LAY_NN, nn[i])) return false;
        if (!gemm_bf16_args_ok(LAY_TN, tn[i]) || !gemm_bf16_pp_supported(LAY_TN, tn[i])) return false;
    }
    return true;
}

// done (may be null): an event that marks the end of this launch on its stream, as a record right after the
// launch would, but carried by the kernel's own completion signal when there is a kernel
static rtp_status gemm_group(rtp_ring *r, int layout, const GemmArgs *a, int count, hipStream_t st, hipEvent_t done = nullptr)
{
    if (r->dry) return RTP_OK;
    if (!r->abl_compute || count == 0) {
        if (done) HIP_TRY(hipEventRecord(done, st));
        return RTP_OK;
    }
    RTP_TRY(aux_delay(r, st));
    double flops = 0.0;
    for (int i = 0; i < count; ++i) flops += 2.0 * a[i].M * a[i].N * a[i].K;
    if (g_prof_on) { // the timing events bracket the launch; the caller's event follows them
        HIP_TRY(timed_launch(layout, flops, st, [&] { return launch_gemm_bf16_pp_group(layout, a, count, nullptr, st); }));
        if (done) HIP_TRY(hipEventRecord(done, st));
        return RTP_OK;
    }
    HIP_TRY(launch_gemm_bf16_pp_group(layout, a, count, nullptr, st, done));
    return RTP_OK;
}

static rtp_status stream_after(hipEvent_t ev, hipStream_t later, hipStream_t earlier)
{
    HIP_TRY(hipEventRecord(ev, earlier));
    HIP_TRY(hipStreamWaitEvent(later, ev, 0));
    return RTP_OK;
}

// stage stream: wait for everything enqueued so far on the compute stream
static rtp_status stage_after_compute(rtp_ring *r)
{
    HIP_TRY(hipEventRecord(r->ev_free, r->cs()));
    HIP_TRY(hipStreamWaitEvent(r->ss(), r->ev_free, 0));
    return RTP_OK;
}

// one part [off, off + bytes) of the weight slot: send shard k's from buffer `src`, receive
// shard kin's into buffer `dst`
static rtp_status rotate_w_part(rtp_ring *r, int step, int k, int kin, int src, int dst, size_t off, size_t bytes)
{
    RTP_TRY(rotate_async(r, r->home_w(k) + off, (char *)r->d.buf_w_dev[src] + off, (char *)r->d.buf_w_dev[dst] + off,
                         r->home_w(kin) + off, bytes, r->ss()));
    r->rec(TR_W_OUT, step, k, src);
    r->rec(TR_W_IN, step, kin, dst);
    return RTP_OK;
}

// the same into a batch (src != dst: the staged modes)
static rtp_status rotate_w_part(rtp_ring *r, CopyBatch &b, int step, int k, int kin, int src, int dst, size_t off, size_t bytes)
{
    RTP_TRY(copy_batch_add(r, b, (char *)r->d.buf_w_dev[dst] + off, r->home_w(kin) + off, bytes, r->ss()));
    RTP_TRY(copy_batch_add(r, b, r->home_w(k) + off, (char *)r->d.buf_w_dev[src] + off, bytes, r->ss()));
    r->rec(TR_W_OUT, step, k, src);
    r->rec(TR_W_IN, step, kin, dst);
    return RTP_OK;
}

static void mlp_close_pass(rtp_mlp *m)
{
    rtp_ring *r = m->ring;
    const int n = r->d.n;
    r->rotations = n - 1;
    m->l1->next_step = m->l2->next_step = n;
    if (r->abl_rotate) {
        r->resident = r->shard_at(n - 1);
        r->res_idx = r->w_idx(n - 1);
        if (r->pass == RTP_PASS_BWD) {
            r->res_g = r->resident;
            r->res_g_idx = r->g_idx(n - 1);
        }
    }
}

static rtp_status mlp_fwd_grouped(rtp_mlp *m, const void *X, void *Y)
{
    rtp_ring *r = m->ring;
    const int n = r->d.n;
    const MlpShapes h = mlp_shapes(m);
    RTP_TRY(rtp_ring_begin(r, RTP_PASS_FWD));
    r->pass_uses_as = false; // everything below runs on the compute and the stage stream
    const bool rot = r->abl_rotate && n > 1;
    const size_t w1_bytes = h.w_off2, w2_bytes = r->d.w_bytes - h.w_off2;
    auto buf = [&](int step) { return (const char *)r->d.buf_w_dev[rot ? r->w_idx(step) : r->res_idx]; };
    // launch t = {Z_t, down_{t-1}}
    for (int t = 0; t <= n; ++t) {
        // transfers that may start once launch t-1 is done and must end before launch t+1:
        // the lagging linear's part of shard t (its buffer was last read by down_{t-2}) and the
        // leading linear's part of shard t+1 (last reader of its buffer: Z_{t-1})
        const bool move_w2 = rot && t >= 1 && t <= n - 1, move_w1 = rot && t <= n - 2;
        if (rot && t >= 1) HIP_TRY(hipStreamWaitEvent(r->cs(), r->ev_w[t & 1], 0));
        if (move_w1 || move_w2) {
            // after launch t-1, which carries ev_free (t = 0: after the load of the own shard, if there was one)
            if (t >= 1)
                HIP_TRY(hipStreamWaitEvent(r->ss(), r->ev_free, 0));
            else
                RTP_TRY(stage_after_compute(r));
            CopyBatch b; // four transfers, no two on the same bytes: one launch
            if (move_w2)
                RTP_TRY(rotate_w_part(r, b, t - 1, r->shard_at(t - 1), r->shard_at(t), r->w_idx(t - 1), r->w_idx(t), h.w_off2, w2_bytes));
            if (move_w1)
                RTP_TRY(rotate_w_part(r, b, t, r->shard_at(t), r->shard_at(t + 1), r->w_idx(t), r->w_idx(t + 1), 0, w1_bytes));
            RTP_TRY(copy_batch_flush(r, b, r->ss(), r->ev_w[(t + 1) & 1]));
        }
        GemmArgs g[2];
        int cnt = 0;
        if (t < n) {
            r->rec(TR_FWD, t, r->shard_at(t), rot ? r->w_idx(t) : r->res_idx);
            g[cnt++] = mlp_args_z(m, h, r->shard_at(t), X, buf(t));
        }
        if (t >= 1) g[cnt++] = mlp_args_down(m, h, r->shard_at(t - 1), t - 1, buf(t - 1), Y);
        if (t >= 2) RTP_TRY(mlp_bias2_add(m, h, r->shard_at(t - 1), buf(t - 1), r->cs()));
        const bool bias_after = t == 1 && h.has_bias && h.n > 1;
        RTP_TRY(gemm_group(r, LAY_NT, g, cnt, r->cs(), rot && !bias_after ? r->ev_free : nullptr));
        if (t == 1) RTP_TRY(mlp_bias2_add(m, h, r->shard_at(0), buf(0), r->cs())); // the sum exists from here on
        if (rot && bias_after) HIP_TRY(hipEventRecord(r->ev_free, r->cs()));
    }
    mlp_close_pass(m);
    return rtp_ring_end(r);
}

static rtp_status mlp_bwd_grouped(rtp_mlp *m, const void *X, const void *dY, void *dX)
{
    rtp_ring *r = m->ring;
    const int n = r->d.n;
    const MlpShapes h = mlp_shapes(m);
    RTP_TRY(rtp_ring_begin(r, RTP_PASS_BWD));
    const bool rot = r->abl_rotate && n > 1;
    const bool move_g = rot && r->d.g_bytes != 0;
    auto wbuf = [&](int step) { return (const char *)r->d.buf_w_dev[rot ? r->w_idx(step) : r->res_idx]; };
    auto gbuf = [&](int step) { return (char *)r->d.buf_g_dev[rot ? r->g_idx(step) : r->res_g_idx]; };
    for (int s = 0; s <= n; ++s) {
        // ---- input-gradient launch s = {dX_{s-1}, dPre_s} -------------------------------
        if (rot && s >= 1 && s < n) HIP_TRY(hipStreamWaitEvent(r->cs(), r->ev_w[s & 1], 0));
        GemmArgs g[2];
        int cnt = 0;
        if (s >= 1) g[cnt++] = mlp_args_dx(m, h, r->shard_at(s - 1), s - 1, wbuf(s - 1), dX);
        if (s < n) {
            r->rec(TR_BWD, s, r->shard_at(s), rot ? r->w_idx(s) : r->res_idx);
            g[cnt++] = mlp_args_dh(m, h, r->shard_at(s), wbuf(s), dY);
        }
        RTP_TRY(gemm_group(r, LAY_NN, g, cnt, r->cs()));
        if (s == n) break;
        // ---- weights of shard s+1: their buffer was last read by dX_{s-1}, just enqueued ----
        if (rot && s <= n - 2) {
            RTP_TRY(stage_after_compute(r));
            CopyBatch b;
            RTP_TRY(rotate_w_part(r, b, s, r->shard_at(s), r->shard_at(s + 1), r->w_idx(s), r->w_idx(s + 1), 0, r->d.w_bytes));
            RTP_TRY(copy_batch_flush(r, b, r->ss(), r->ev_w[(s + 1) & 1]));
        }
        // ---- weight-gradient launch s = {G1_s, G2_s}, onto the travelling gradient shard ----
        // (on the auxiliary stream when there is one: it only has to follow dPre_s, so it runs
        // beside the next input-gradient launch and the two fill each other's idle tails)
        hipStream_t ws = r->as();
        if (ws != r->cs()) {
            HIP_TRY(hipEventRecord(r->ev_aux, r->cs()));
            HIP_TRY(hipStreamWaitEvent(ws, r->ev_aux, 0));
        }
        if (move_g && s >= 1) HIP_TRY(hipStreamWaitEvent(ws, r->ev_g[s & 1], 0));
        g[0] = mlp_args_dw1(m, h, r->shard_at(s), gbuf(s), X);
        g[1] = mlp_args_dw2(m, h, r->shard_at(s), gbuf(s), dY);
        // the send of the finished gradient shard is fused into the kernels (as in rtp_linear_bwd)
        bool fused_send = move_g && s <= n - 2 && r->abl_compute;
        if (fused_send) {
            int ks[2] = {1, 1};
            gemm_bf16_pp_plan(LAY_TN, g, 2, nullptr, nullptr, ks);
            if (ks[0] > 1 || ks[1] > 1) fused_send = false; // K-split partial sums need the plain `+=` form
        }
        if (fused_send) {
            char *home = r->home_g(r->shard_at(s));
            g[0].epi = g[1].epi = EPI_ACC_LAST;
            g[0].C = home;
            g[1].C = home + h.g_off2;
        }
        RTP_TRY(gemm_group(r, LAY_TN, g, 2, ws));
        RTP_TRY(mlp_bias_grads(m, h, r->shard_at(s), gbuf(s), fused_send ? r->home_g(r->shard_at(s)) : nullptr, dY, true, true, ws));
        // ---- the gradient shard moves on as soon as both parts are complete; the next
        // input-gradient launch runs meanwhile
        if (move_g && s <= n - 2) {
            const int k = r->shard_at(s), kin = r->shard_at(s + 1);
            HIP_TRY(hipEventRecord(r->ev_free2, ws));
            HIP_TRY(hipStreamWaitEvent(r->ss(), r->ev_free2, 0));
            if (r->g_idx(s) != r->g_idx(s + 1)) {
                // two buffers: the next shard comes into the other one, the two transfers are one launch
                CopyBatch b;
                RTP_TRY(copy_batch_add(r, b, r->d.buf_g_dev[r->g_idx(s + 1)], r->home_g(kin), r->d.g_bytes, r->ss()));
                if (!fused_send) RTP_TRY(copy_batch_add(r, b, r->home_g(k), r->d.buf_g_dev[r->g_idx(s)], r->d.g_bytes, r->ss()));
                RTP_TRY(copy_batch_flush(r, b, r->ss(), r->ev_g[(s + 1) & 1]));
            } else {
                if (!fused_send) RTP_TRY(copy_async(r, r->home_g(k), r->d.buf_g_dev[r->g_idx(s)], r->d.g_bytes, r->ss()));
                RTP_TRY(copy_async(r, r->d.buf_g_dev[r->g_idx(s + 1)], r->home_g(kin), r->d.g_bytes, r->ss(), r->ev_g[(s + 1) & 1]));
            }
            r->rec(TR_G_OUT, s, k, r->g_idx(s));
            r->rec(TR_G_IN, s, kin, r->g_idx(s + 1));
        }
    }
    mlp_close_pass(m);
    return rtp_ring_end(r);
}

// The default backward pass beside an auxiliary stream: one launch per GEMM, the input gradients (dPre_s, dX_s)
// on the compute stream and the weight gradients (dW2_s, dW1_s) on the auxiliary stream, exactly the kernels and
// the order of the step-by-step calls, but with the cross-stream waits and transfer launches of a step cut to what
// the data flow needs (the host pays ~5 us for each of them, and units with narrow shards are bound by the host):
//   stage stream   waits for the compute stream's last readers of the staging weight buffer, then moves
//                  shard s out and shard s+1 in as one launch; waits for the weight-gradient kernel(s) that
//                  complete a gradient part, then exchanges that part (two buffers: the whole shard at once
//                  into the other buffer; one buffer: part by part, in place);
//   compute stream waits for the weights of step s;
//   auxiliary      waits for the gradient part it adds onto, and dW1_s for dPre_s.
static rtp_status mlp_bwd_two_stream(rtp_mlp *m, const void *X, const void *dY, void *dX)
{
    rtp_ring *r = m->ring;
    const int n = r->d.n;
    const MlpShapes h = mlp_shapes(m);
    RTP_TRY(rtp_ring_begin(r, RTP_PASS_BWD));
    const bool rot = r->abl_rotate && n > 1;
    const bool move_g = rot && r->d.g_bytes != 0;
    const bool two_g = r->d.mode == RTP_DOUBLE_BUFFER;
    hipStream_t cs = r->cs(), as = r->as(), ss = r->ss();
    const size_t g1_bytes = h.g_off2, g2_bytes = r->d.g_bytes - h.g_off2;
    auto wbuf = [&](int step) { return (const char *)r->d.buf_w_dev[rot ? r->w_idx(step) : r->res_idx]; };
    auto gidx = [&](int step) { return rot ? r->g_idx(step) : r->res_g_idx; };
    auto gbuf = [&](int step) { return (char *)r->d.buf_g_dev[gidx(step)]; };

    // The shard of the last step is the worker's own and goes nowhere (Design section, workflow paragraph): its two
    // kernels store `arrived + own` straight into the shard's slot, and nothing is left in the buffer for the next
    // backward pass (or a flush) to write back.  Both parts or neither: a write-back of the whole buffer would
    // overwrite a part that is current in the slot only.
    bool own_to_slot = false;
    if (move_g && r->abl_compute && !r->dry) {
        const int k = r->shard_at(n - 1);
        GemmArgs a2 = mlp_args_dw2(m, h, k, gbuf(n - 1), dY), a1 = mlp_args_dw1(m, h, k, gbuf(n - 1), X);
        a1.cu_share = a2.cu_share = 2;
        int ks1 = 1, ks2 = 1;
        gemm_bf16_pp_plan(LAY_TN, &a2, 1, nullptr, nullptr, &ks2);
        gemm_bf16_pp_plan(LAY_TN, &a1, 1, nullptr, nullptr, &ks1);
        own_to_slot = ks1 == 1 && ks2 == 1;
    }
    // a weight-gradient kernel; the send of its part of the gradient shard is fused into it when the shard moves on
    // (mark: ev_free2 completes with the kernel, or with the bias sums that follow it, when a transfer waits for it)
    auto emit_dw = [&](int s, GemmArgs a, size_t off, bool first, bool *fused, bool mark) -> rtp_status {
        const bool moves_on = move_g && s <= n - 2;
        bool fused_send = (moves_on && r->abl_compute) || (own_to_slot && s == n - 1);
        a.cu_share = 2; // (before the plan is asked for: the launcher plans with it)
        if (fused_send && moves_on) {
            int ks = 1;
            gemm_bf16_pp_plan(LAY_TN, &a, 1, nullptr, nullptr, &ks);
            if (ks > 1) fused_send = false; // K-split partial sums need the plain `+=` form
        }
        if (fused_send) {
            a.epi = EPI_ACC_LAST;
            a.C = r->home_g(r->shard_at(s)) + off;
        }
        RTP_TRY(gemm_group(r, LAY_TN, &a, 1, as, mark && !h.has_bias ? r->ev_free2 : nullptr));
        RTP_TRY(mlp_bias_grads(m, h, r->shard_at(s), gbuf(s), fused_send ? r->home_g(r->shard_at(s)) : nullptr, dY, first, !first, as));
        if (mark && h.has_bias && !r->dry) HIP_TRY(hipEventRecord(r->ev_free2, as));
        *fused = fused_send;
        return RTP_OK;
    };
    // stage stream, after the weight-gradient kernel that carries ev_free2: part [off, off + bytes) of gradient shard s goes
    // out (unless its kernel has sent it) and the same part of shard s+1 comes into buffer gidx(s+1)
    auto exchange_g = [&](int s, size_t off, size_t bytes, bool out_by_copy, hipEvent_t landed, bool whole) -> rtp_status {
        const int k = r->shard_at(s), kin = r->shard_at(s + 1);
        HIP_TRY(hipStreamWaitEvent(ss, r->ev_free2, 0));
        CopyBatch b;
        if (two_g) {
            RTP_TRY(copy_batch_add(r, b, gbuf(s + 1) + off, r->home_g(kin) + off, bytes, ss));
            if (out_by_copy) RTP_TRY(copy_batch_add(r, b, r->home_g(k) + off, gbuf(s) + off, bytes, ss));
        } else {
            // in place: the part comes into the buffer it just left
            if (out_by_copy) RTP_TRY(copy_async(r, r->home_g(k) + off, gbuf(s) + off, bytes, ss));
            RTP_TRY(copy_batch_add(r, b, gbuf(s + 1) + off, r->home_g(kin) + off, bytes, ss));
        }
        RTP_TRY(copy_batch_flush(r, b, ss, landed));
        if (whole || off != 0) r->rec(TR_G_OUT, s, k, gidx(s));
        if (whole || off != 0) r->rec(TR_G_IN, s, kin, gidx(s + 1));
        return RTP_OK;
    };

    for (int s = 0; s < n; ++s) {
        const int k = r->shard_at(s);
        // ---- weights of step s+1: their buffer was last read by dPre_{s-1} and dX_{s-1}
        if (rot && s <= n - 2) {
            if (s >= 1) HIP_TRY(hipStreamWaitEvent(ss, r->ev_free, 0)); // dX_{s-1} carries ev_free (step 0: rtp_ring_begin has ordered the streams)
            CopyBatch b;
            RTP_TRY(rotate_w_part(r, b, s, k, r->shard_at(s + 1), r->w_idx(s), r->w_idx(s + 1), 0, r->d.w_bytes));
            RTP_TRY(copy_batch_flush(r, b, ss, r->ev_w[(s + 1) & 1]));
        }
        // ---- input gradients
        if (rot && s >= 1) HIP_TRY(hipStreamWaitEvent(cs, r->ev_w[s & 1], 0));
        r->rec(TR_BWD, s, k, rot ? r->w_idx(s) : r->res_idx);
        GemmArgs a = mlp_args_dh(m, h, k, wbuf(s), dY);
        a.cu_share = 2;
        RTP_TRY(gemm_group(r, LAY_NN, &a, 1, cs, r->ev_k[s & 1]));
        a = mlp_args_dx(m, h, k, s, wbuf(s), dX);
        a.cu_share = 2;
        RTP_TRY(gemm_group(r, LAY_NN, &a, 1, cs, rot && s <= n - 2 ? r->ev_free : nullptr));
        // ---- weight gradients, onto the travelling gradient shard
        const bool moves_on = move_g && s <= n - 2;
        bool sent2 = false, sent1 = false;
        if (move_g && s >= 1) HIP_TRY(hipStreamWaitEvent(as, (two_g ? r->ev_g : r->ev_g2)[s & 1], 0));
        RTP_TRY(emit_dw(s, mlp_args_dw2(m, h, k, gbuf(s), dY), h.g_off2, false, &sent2, moves_on && !two_g));
        if (moves_on && !two_g) RTP_TRY(exchange_g(s, h.g_off2, g2_bytes, !sent2, r->ev_g2[(s + 1) & 1], false));
        HIP_TRY(hipStreamWaitEvent(as, r->ev_k[s & 1], 0));
        if (move_g && s >= 1 && !two_g) HIP_TRY(hipStreamWaitEvent(as, r->ev_g[s & 1], 0));
        RTP_TRY(emit_dw(s, mlp_args_dw1(m, h, k, gbuf(s), X), 0, true, &sent1, moves_on));
        if (moves_on && !two_g) RTP_TRY(exchange_g(s, 0, g1_bytes, !sent1, r->ev_g[(s + 1) & 1], false));
        if (moves_on && two_g) {
            // two buffers: the whole shard at once (a part its kernel did not send goes out by copy)
            if (sent1 == sent2) {
                RTP_TRY(exchange_g(s, 0, r->d.g_bytes, !sent1, r->ev_g[(s + 1) & 1], true));
            } else {
                const int kk = r->shard_at(s), kin = r->shard_at(s + 1);
                HIP_TRY(hipStreamWaitEvent(ss, r->ev_free2, 0));
                CopyBatch b;
                RTP_TRY(copy_batch_add(r, b, gbuf(s + 1), r->home_g(kin), r->d.g_bytes, ss));
                if (!sent1) RTP_TRY(copy_batch_add(r, b, r->home_g(kk), gbuf(s), g1_bytes, ss));
                if (!sent2) RTP_TRY(copy_batch_add(r, b, r->home_g(kk) + h.g_off2, gbuf(s) + h.g_off2, g2_bytes, ss));
                RTP_TRY(copy_batch_flush(r, b, ss, r->ev_g[(s + 1) & 1]));
                r->rec(TR_G_OUT, s, kk, gidx(s));
                r->rec(TR_G_IN, s, kin, gidx(s + 1));
            }
        }
    }
    mlp_close_pass(m);
    if (own_to_slot) r->res_g = -1; // the slot is current
    return rtp_ring_end(r);
}

// ---- fused step: the unit's dependent GEMMs of a rotation step as ONE launch ---------------------
// Forward, Z_t = act(X W1_t^T) and down_t = H_t W2_t^T of the SAME step go out as one launch of the
// tiled kernel: the tiles of down_t follow those of Z_t in the grid and each starts as soon as the Z
// tiles of its rows are done (a counter per 64 rows in device memory), so the hidden activations
// are read back while they are still in the cache they were written through, and a step is one
// kernel.  (They are still stored: the backward pass needs them.  Keeping them in LDS instead
// would need a workgroup to own all `o` columns of its rows: 64-row tiles at most, a quarter of the
// operand reuse of the 256-row tile.)  Backward the same holds for dPre_s -> dX_s; the weight
// gradients stay two launches on the auxiliary stream.  Rotation, buffers, events: the step-by-step
// schedule's, in all three modes.
static size_t mlp_sync_words(const rtp_mlp_desc *d)
{
    const size_t blocks = ((size_t)std::max<int64_t>(d->T, 0) + SYNC_ROWS - 1) / SYNC_ROWS;
    return (blocks + 1 + 3) / 4 * 4; // one counter per row block, the error word, whole 16-byte units
}

extern "C" size_t rtp_mlp_step_sync_bytes(const rtp_mlp_desc *d) { return d ? mlp_sync_words(d) * sizeof(int) : 0; }

static bool mlp_fused_ok(const rtp_mlp *m, const void *X, const void *Y, const void *dY, const void *dX)
{
    if (!(m->d.flags & RTP_FLAG_FUSED_STEP) || !m->d.step_sync_dev) return false;
    // same shape rules as the grouped launches (16-bit inputs, every GEMM within the tiled kernel's reach);
    // the blocking mode is fine here: the rotation is the step-by-step schedule's
    const rtp_ring *r = m->ring;
    if (r->dry || m->d.dtype == RTP_F32 || m->d.T <= 0) return false;
    const MlpShapes h = mlp_shapes(m);
    const char *W = (const char *)r->d.buf_w_dev[0];
    const void *x = X ? X : m->d.hidden_dev, *dy = dY ? dY : m->d.hidden_dev;
    void *y = Y ? (void *)Y : m->d.hidden_dev, *dx = dX ? (void *)dX : m->d.hidden_dev;
    const GemmArgs nt[2] = {mlp_args_z(m, h, 0, x, W), mlp_args_down(m, h, 0, 0, W, y)};
    const GemmArgs nn[2] = {mlp_args_dh(m, h, 0, W, dy), mlp_args_dx(m, h, 0, 0, W, dx)};
    for (int i = 0; i < 2; ++i) {
        if (!gemm_bf16_args_ok(LAY_NT, nt[i]) || !gemm_bf16_pp_supported(LAY_NT, nt[i])) return false;
        if (!gemm_bf16_args_ok(LAY_NN, nn[i]) || !gemm_bf16_pp_supported(LAY_NN, nn[i])) return false;
    }
    return true;
}

static rtp_status mlp_sync_reset(rtp_mlp *m)
{
    rtp_ring *r = m->ring;
    if (r->dry || !r->abl_compute) return RTP_OK;
    HIP_TRY(launch_fill_zero(m->d.step_sync_dev, mlp_sync_words(&m->d) * sizeof(int), r->cs()));
    return RTP_OK;
}

static rtp_status mlp_fwd_fused(rtp_mlp *m, const void *X, void *Y)
{
    rtp_ring *r = m->ring;
    const int n = r->d.n;
    const MlpShapes h = mlp_shapes(m);
    RTP_TRY(rtp_ring_begin(r, RTP_PASS_FWD));
    RTP_TRY(mlp_sync_reset(m));
    for (int t = 0; t < n; ++t) {
        if (t < n - 1) RTP_TRY(rtp_rotate_step(r, RTP_CW, t));
        RTP_TRY(enter_step(r, t, t, RTP_PASS_FWD, "rtp_mlp_fwd"));
        const int k = r->abl_rotate ? r->resident : rtp_fwd_shard(r->d.rank, t, n);
        const char *W = (const char *)r->d.buf_w_dev[r->res_idx];
        r->rec(TR_FWD, t, k, r->res_idx);
        GemmArgs g[2] = {mlp_args_z(m, h, k, X, W), mlp_args_down(m, h, k, t, W, Y)};
        g[0].sync = g[1].sync = (int *)m->d.step_sync_dev;
        g[0].sync_signal = 1;
        g[1].sync_wait = (t + 1) * gemm_bf16_pp_tiles_n(g[0]); // every Z tile of the rows, of this and the earlier steps
        if (t >= 1) RTP_TRY(mlp_bias2_add(m, h, k, W, r->cs()));
        RTP_TRY(gemm_group(r, LAY_NT, g, 2, r->cs()));
        if (t == 0) RTP_TRY(mlp_bias2_add(m, h, k, W, r->cs()));
        m->l1->next_step = m->l2->next_step = t + 1;
    }
    return rtp_ring_end(r);
}

static rtp_status mlp_bwd_fused(rtp_mlp *m, const void *X, const void *dY, void *dX)
{
    rtp_ring *r = m->ring;
    const int n = r->d.n;
    const MlpShapes h = mlp_shapes(m);
    RTP_TRY(rtp_ring_begin(r, RTP_PASS_BWD));
    RTP_TRY(mlp_sync_reset(m));
    for (int s = 0; s < n; ++s) {
        if (s < n - 1) RTP_TRY(rtp_rotate_step(r, RTP_CCW, s));
        // the second linear's weight gradient (auxiliary stream, gradient part handed on), no input gradient yet
        RTP_TRY(rtp_linear_bwd(m->l2, s, m->d.hidden_dev, dY, nullptr));
        // dPre_s and dX_s as one launch: the tiles of dX_s wait for the dPre tiles of their rows
        const int k = r->abl_rotate ? r->resident : rtp_bwd_shard(r->d.rank, s, n);
        const char *W = (const char *)r->d.buf_w_dev[r->res_idx];
        GemmArgs g[2] = {mlp_args_dh(m, h, k, W, dY), mlp_args_dx(m, h, k, s, W, dX)};
        g[0].sync = g[1].sync = (int *)m->d.step_sync_dev;
        g[0].sync_signal = 1;
        g[1].sync_wait = (s + 1) * gemm_bf16_pp_tiles_n(g[0]);
        g[0].cu_share = g[1].cu_share = r->as() != r->cs() ? 2 : 1;
        RTP_TRY(gemm_group(r, LAY_NN, g, 2, r->cs()));
        // the first linear's weight gradient needs dPre_s: ordered after the launch above
        RTP_TRY(rtp_linear_bwd(m->l1, s, X, m->d.dpre_dev, nullptr));
    }
    return rtp_ring_end(r);
}

// ---- pipelined schedule of the MLP unit (two compute streams) ---------------------------
// The unit's GEMMs form two chains that only touch through data: forward, Z_t = act(X W1_t^T) on
// the compute stream and down_t = H_t W2_t^T on the auxiliary stream (down_t needs Z_t, nothing
// needs down_t but the fp32 sum it adds to); backward, {dPre_s, dX_s} on the compute stream and
// {dW2_s, dW1_s} on the auxiliary stream, where dPre_{s+1} = (dY W2_{s+1}) act'(.) needs nothing of
// step s and is therefore issued BEFORE dX_s.  Each chain's next kernel then has its inputs ready
// long before its predecessor ends, so a kernel that leaves compute units idle (a shard GEMM of 96
// tiles on 256 units) runs beside the other chain's kernel instead of beside nothing, and no chain
// waits for a transfer.  The shard parts move per buffer part: as soon as the last kernel that
// reads a part of a weight buffer (W1 part: Z_t / dX_s; W2 part: down_t / dPre_s) or that adds onto
// a part of a gradient buffer is enqueued, that part of the shard is sent on and the part of the
// next shard that uses the same buffer (two steps on for the weights, `ng` steps on for the
// gradients, ng = number of gradient buffers) is received into it.  Same buffers, same bytes and the
// same N-1 sends and receives per part and pass as in the step-by-step schedule; same kernels.


// send shard k's part [off, off + bytes) of weight buffer `src` home (rotation `step`)
static rtp_status w_part_out(rtp_ring *r, int step, int k, int src, size_t off, size_t bytes)
{
    RTP_TRY(copy_async(r, r->home_w(k) + off, (const char *)r->d.buf_w_dev[src] + off, bytes, r->ss()));
    r->rec(TR_W_OUT, step, k, src);
    return RTP_OK;
}

// receive shard kin's part into weight buffer `dst` (rotation `step`)
static rtp_status w_part_in(rtp_ring *r, int step, int kin, int dst, size_t off, size_t bytes)
{
    RTP_TRY(copy_async(r, (char *)r->d.buf_w_dev[dst] + off, r->home_w(kin) + off, bytes, r->ss()));
    r->rec(TR_W_IN, step, kin, dst);
    return RTP_OK;
}

// After the last reader (step t) of part [off, off + bytes) of its weight buffer has been enqueued
// on `reader`: that part of shard t goes home and the part of shard t+2 comes into the buffer.
static rtp_status w_part_turnover(rtp_ring *r, int t, hipEvent_t scratch_ev, hipStream_t reader, size_t off, size_t bytes,
                                  hipEvent_t landed)
{
    const int n = r->d.n;
    if (t > n - 2 || bytes == 0) return RTP_OK; // the last shard of a pass stays
    RTP_TRY(stream_after(scratch_ev, r->ss(), reader));
    RTP_TRY(w_part_out(r, t, r->shard_at(t), r->w_idx(t), off, bytes));
    if (t + 2 <= n - 1) {
        RTP_TRY(w_part_in(r, t + 1, r->shard_at(t + 2), r->w_idx(t + 2), off, bytes));
        HIP_TRY(hipEventRecord(landed, r->ss()));
    }
    return RTP_OK;
}

static rtp_status mlp_fwd_pipelined(rtp_mlp *m, const void *X, void *Y)
{
    rtp_ring *r = m->ring;
    const int n = r->d.n;
    const MlpShapes h = mlp_shapes(m);
    RTP_TRY(rtp_ring_begin(r, RTP_PASS_FWD));
    const bool rot = r->abl_rotate && n > 1;
    hipStream_t cs = r->cs(), as = r->as();
    const size_t w1_bytes = h.w_off2, w2_bytes = r->d.w_bytes - h.w_off2;
    auto buf = [&](int step) { return (const char *)r->d.buf_w_dev[rot ? r->w_idx(step) : r->res_idx]; };
    if (rot) {
        // shard 1 comes into the free buffer at once (its readers belong to earlier passes, which
        // rtp_ring_begin has ordered before everything enqueued from here on)
        RTP_TRY(w_part_in(r, 0, r->shard_at(1), r->w_idx(1), 0, w1_bytes));
        HIP_TRY(hipEventRecord(r->ev_w[1], r->ss()));
        RTP_TRY(w_part_in(r, 0, r->shard_at(1), r->w_idx(1), h.w_off2, w2_bytes));
        HIP_TRY(hipEventRecord(r->ev_w2[1], r->ss()));
    }
    for (int t = 0; t < n; ++t) {
        const int k = r->shard_at(t);
        // ---- Z_t on the compute stream
        if (rot && t >= 1) HIP_TRY(hipStreamWaitEvent(cs, r->ev_w[t & 1], 0));
        r->rec(TR_FWD, t, k, rot ? r->w_idx(t) : r->res_idx);
        GemmArgs a = mlp_args_z(m, h, k, X, buf(t));
        a.cu_share = 2;
        RTP_TRY(gemm_group(r, LAY_NT, &a, 1, cs));
        HIP_TRY(hipEventRecord(r->ev_k[t & 1], cs));
        if (rot) RTP_TRY(w_part_turnover(r, t, r->ev_free, cs, 0, w1_bytes, r->ev_w[t & 1]));
        // ---- down_t on the auxiliary stream (the own shard's initial load is ordered before Z_0)
        HIP_TRY(hipStreamWaitEvent(as, r->ev_k[t & 1], 0));
        if (rot && t >= 1) HIP_TRY(hipStreamWaitEvent(as, r->ev_w2[t & 1], 0));
        a = mlp_args_down(m, h, k, t, buf(t), Y);
        a.cu_share = 2;
        if (t >= 1) RTP_TRY(mlp_bias2_add(m, h, k, buf(t), as));
        RTP_TRY(gemm_group(r, LAY_NT, &a, 1, as));
        if (t == 0) RTP_TRY(mlp_bias2_add(m, h, k, buf(t), as)); // the sum exists from here on
        if (rot) RTP_TRY(w_part_turnover(r, t, r->ev_free2, as, h.w_off2, w2_bytes, r->ev_w2[t & 1]));
    }
    mlp_close_pass(m);
    return rtp_ring_end(r);
}

static rtp_status mlp_bwd_pipelined(rtp_mlp *m, const void *X, const void *dY, void *dX)
{
    rtp_ring *r = m->ring;
    const int n = r->d.n;
    const MlpShapes h = mlp_shapes(m);
    RTP_TRY(rtp_ring_begin(r, RTP_PASS_BWD));
    const bool rot = r->abl_rotate && n > 1;
    const bool move_g = rot && r->d.g_bytes != 0;
    const int ng = r->d.mode == RTP_DOUBLE_BUFFER ? 2 : 1;
    hipStream_t cs = r->cs(), as = r->as(), ss = r->ss();
    const size_t w1_bytes = h.w_off2, w2_bytes = r->d.w_bytes - h.w_off2;
    const size_t g1_bytes = h.g_off2, g2_bytes = r->d.g_bytes - h.g_off2;
    auto wbuf = [&](int step) { return (const char *)r->d.buf_w_dev[rot ? r->w_idx(step) : r->res_idx]; };
    auto gidx = [&](int step) { return rot ? r->g_idx(step) : r->res_g_idx; };
    auto gbuf = [&](int step) { return (char *)r->d.buf_g_dev[gidx(step)]; };

    // receive the gradient part [off, off + bytes) of the shard step `c` adds onto, into its buffer
    auto g_part_in = [&](int c, size_t off, size_t bytes, hipEvent_t landed) -> rtp_status {
        const int kin = r->shard_at(c);
        RTP_TRY(copy_async(r, gbuf(c) + off, r->home_g(kin) + off, bytes, ss));
        r->rec(TR_G_IN, c - 1, kin, gidx(c));
        HIP_TRY(hipEventRecord(landed, ss));
        return RTP_OK;
    };
    // dPre_s on the compute stream, and the turnover of the W2 part it is the last reader of
    auto emit_dpre = [&](int s) -> rtp_status {
        if (rot && s >= 1) HIP_TRY(hipStreamWaitEvent(cs, r->ev_w2[s & 1], 0));
        r->rec(TR_BWD, s, r->shard_at(s), rot ? r->w_idx(s) : r->res_idx);
        GemmArgs a = mlp_args_dh(m, h, r->shard_at(s), wbuf(s), dY);
        a.cu_share = 2;
        RTP_TRY(gemm_group(r, LAY_NN, &a, 1, cs));
        HIP_TRY(hipEventRecord(r->ev_k[s & 1], cs));
        if (rot) RTP_TRY(w_part_turnover(r, s, r->ev_free, cs, h.w_off2, w2_bytes, r->ev_w2[s & 1]));
        return RTP_OK;
    };
    // one weight-gradient kernel on the auxiliary stream, fused with the send of its part of the
    // travelling gradient shard when the shard moves on, then the turnover of that part's buffer
    auto emit_dw = [&](int s, GemmArgs a, size_t off, size_t bytes, hipEvent_t *landed, bool first) -> rtp_status {
        if (move_g && s >= 1) HIP_TRY(hipStreamWaitEvent(as, landed[s & 1], 0));
        const bool moves_on = move_g && s <= n - 2;
        bool fused_send = moves_on && r->abl_compute;
        if (fused_send) {
            int ks = 1;
            gemm_bf16_pp_plan(LAY_TN, &a, 1, nullptr, nullptr, &ks);
            if (ks > 1) fused_send = false; // K-split partial sums need the plain `+=` form
        }
        if (fused_send) {
            a.epi = EPI_ACC_LAST;
            a.C = r->home_g(r->shard_at(s)) + off;
        }
        RTP_TRY(gemm_group(r, LAY_TN, &a, 1, as));
        // this linear's bias gradient belongs to the same part of the gradient shard
        RTP_TRY(mlp_bias_grads(m, h, r->shard_at(s), gbuf(s), fused_send ? r->home_g(r->shard_at(s)) : nullptr, dY, first, !first, as));
        if (!move_g) return RTP_OK;
        if (moves_on || s + ng <= n - 1) RTP_TRY(stream_after(r->ev_free2, ss, as));
        if (moves_on) {
            if (!fused_send) RTP_TRY(copy_async(r, r->home_g(r->shard_at(s)) + off, gbuf(s) + off, bytes, ss));
            r->rec(TR_G_OUT, s, r->shard_at(s), gidx(s));
        }
        if (s + ng <= n - 1) RTP_TRY(g_part_in(s + ng, off, bytes, landed[(s + ng) & 1]));
        return RTP_OK;
    };

    if (rot) {
        // stage stream: after rtp_ring_begin's copies on the compute stream (the second gradient
        // buffer may be the source of its write-back); then shard 1 comes into the free buffers
        RTP_TRY(stream_after(r->ev_free, ss, cs));
        RTP_TRY(w_part_in(r, 0, r->shard_at(1), r->w_idx(1), h.w_off2, w2_bytes));
        HIP_TRY(hipEventRecord(r->ev_w2[1], ss));
        RTP_TRY(w_part_in(r, 0, r->shard_at(1), r->w_idx(1), 0, w1_bytes));
        HIP_TRY(hipEventRecord(r->ev_w[1], ss));
        if (move_g && ng == 2) {
            RTP_TRY(g_part_in(1, h.g_off2, g2_bytes, r->ev_g2[1]));
            RTP_TRY(g_part_in(1, 0, g1_bytes, r->ev_g[1]));
        }
    }
    // the auxiliary stream starts after rtp_ring_begin's load of the first gradient shard
    RTP_TRY(stream_after(r->ev_aux, as, cs));
    RTP_TRY(emit_dpre(0));
    for (int s = 0; s < n; ++s) {
        const int k = r->shard_at(s);
        if (s + 1 < n) RTP_TRY(emit_dpre(s + 1));
        // ---- dX_s (last reader of its buffer's W1 part)
        if (rot && s >= 1) HIP_TRY(hipStreamWaitEvent(cs, r->ev_w[s & 1], 0));
        GemmArgs a = mlp_args_dx(m, h, k, s, wbuf(s), dX);
        a.cu_share = 2;
        RTP_TRY(gemm_group(r, LAY_NN, &a, 1, cs));
        if (rot) RTP_TRY(w_part_turnover(r, s, r->ev_free, cs, 0, w1_bytes, r->ev_w[s & 1]));
        // ---- dW2_s, then dW1_s (needs dPre_s)
        a = mlp_args_dw2(m, h, k, gbuf(s), dY);
        a.cu_share = 2;
        RTP_TRY(emit_dw(s, a, h.g_off2, g2_bytes, r->ev_g2, false));
        HIP_TRY(hipStreamWaitEvent(as, r->ev_k[s & 1], 0));
        a = mlp_args_dw1(m, h, k, gbuf(s), X);
        a.cu_share = 2;
        RTP_TRY(emit_dw(s, a, 0, g1_bytes, r->ev_g, true));
    }
    mlp_close_pass(m);
    return rtp_ring_end(r);
}

static rtp_status mlp_fwd_pass(rtp_mlp *m, const void *X, void *Y)
{
    const bool have_aux = m->ring->as() != m->ring->cs();
    if (mlp_fused_ok(m, X, Y, nullptr, nullptr)) return mlp_fwd_fused(m, X, Y);
    if (mlp_grouped_ok(m, X, Y, nullptr, nullptr))
        return have_aux && (m->d.flags & RTP_FLAG_PIPELINED) ? mlp_fwd_pipelined(m, X, Y) : mlp_fwd_grouped(m, X, Y);
    const int n = m->d.n;
    RTP_TRY(rtp_ring_begin(m->ring, RTP_PASS_FWD));
    for (int t = 0; t < n; ++t) {
        if (t < n - 1) RTP_TRY(rtp_rotate_step(m->ring, RTP_CW, t));
        RTP_TRY(rtp_linear_fwd(m->l1, t, X, m->d.hidden_dev));
        RTP_TRY(rtp_linear_fwd(m->l2, t, m->d.hidden_dev, Y));
    }
    return rtp_ring_end(m->ring);
}

static rtp_status mlp_bwd_pass(rtp_mlp *m, const void *X, const void *dY, void *dX)
{
    // Measured on the Llama-shaped unit (ms per backward pass, same box): with an auxiliary stream, one launch
    // per GEMM with the weight gradients on that stream 3.15, the pipelined schedule 3.2-3.4, the two grouped
    // launches per step 3.4-3.5; without one the grouped launches win (3.5 against 3.7).  Whatever the schedule,
    // the kernels of a pass need the same time of a machine that is busy throughout.
    const bool have_aux = m->ring->as() != m->ring->cs();
    if (dX && mlp_fused_ok(m, X, nullptr, dY, dX)) return mlp_bwd_fused(m, X, dY, dX);
    if (dX && mlp_grouped_ok(m, X, nullptr, dY, dX)) {
        if (have_aux && (m->d.flags & RTP_FLAG_PIPELINED)) return mlp_bwd_pipelined(m, X, dY, dX);
        if (!have_aux || (m->d.flags & RTP_FLAG_GROUPED)) return mlp_bwd_grouped(m, X, dY, dX);
        return mlp_bwd_two_stream(m, X, dY, dX);
    }
    const int n = m->d.n;
    RTP_TRY(rtp_ring_begin(m->ring, RTP_PASS_BWD));
    for (int s = 0; s < n; ++s) {
        if (s < n - 1) RTP_TRY(rtp_rotate_step(m->ring, RTP_CCW, s));
        RTP_TRY(rtp_linear_bwd(m->l2, s, m->d.hidden_dev, dY, m->d.dpre_dev));
        RTP_TRY(rtp_linear_bwd(m->l1, s, X, m->d.dpre_dev, dX));
    }
    return rtp_ring_end(m->ring);
}

// A failure half-way through a pass leaves the ring idle again (rtp_ring_abort), not wedged.
extern "C" rtp_status rtp_mlp_fwd(rtp_mlp *m, const void *X, void *Y)
{
    if (!m) return fail(RTP_ERR_INVALID, "rtp_mlp_fwd: null mlp");
    if (!m->ring->dry && m->d.T > 0 && (!X || !Y)) return fail(RTP_ERR_INVALID, "rtp_mlp_fwd: null tensor");
    if (m->ring->pass != RTP_PASS_IDLE) return fail(RTP_ERR_STATE, "rtp_mlp_fwd: a pass is already open");
    return close_failed_pass(m->ring, mlp_fwd_pass(m, X, Y));
}

extern "C" rtp_status rtp_mlp_bwd(rtp_mlp *m, const void *X, const void *dY, void *dX)
{
    if (!m) return fail(RTP_ERR_INVALID, "rtp_mlp_bwd: null mlp");
    if (!m->ring->dry && m->d.T > 0 && (!X || !dY)) return fail(RTP_ERR_INVALID, "rtp_mlp_bwd: null tensor");
    if (m->ring->pass != RTP_PASS_IDLE) return fail(RTP_ERR_STATE, "rtp_mlp_bwd: a pass is already open");
    return close_failed_pass(m->ring, mlp_bwd_pass(m, X, dY, dX));
}

extern "C" rtp_status rtp_mlp_flush(rtp_mlp *m) { return m ? rtp_ring_flush(m->ring) : fail(RTP_ERR_INVALID, "null mlp"); }
extern "C" rtp_status rtp_mlp_sync(rtp_mlp *m)
{
    if (!m) return fail(RTP_ERR_INVALID, "null mlp");
    RTP_TRY(rtp_ring_sync(m->ring));
    if ((m->d.flags & RTP_FLAG_FUSED_STEP) && m->d.step_sync_dev && !m->ring->dry) {
        // a consumer tile that gave up waiting for its producers has raised the word after the counters
        const size_t blocks = ((size_t)m->d.T + SYNC_ROWS - 1) / SYNC_ROWS;
        int flag = 0;
        HIP_TRY(hipMemcpy(&flag, (const int *)m->d.step_sync_dev + blocks, sizeof flag, hipMemcpyDeviceToHost));
        if (flag) return fail(RTP_ERR_HIP, "rtp_mlp_sync: a tile of a fused step gave up waiting for the tiles it depends on; "
                                            "the results of that pass are not valid");
    }
    return RTP_OK;
}

// ---------------------------------------------------------------------------
// expert partition: the ring's shard is one whole expert
// ---------------------------------------------------------------------------
// The worker's tokens are grouped by the expert they are routed to (a stable grouping, each group
// padded with zero rows to a multiple of MOE_ROW_ALIGN so that the token count is a legal
// contraction length for the tiled kernels); at rotation step t the worker runs the expert it
// holds on that expert's group, and the outputs go back to token order at the end.  Padding rows
// are zero through the whole unit (act(0) = 0 for every activation here), so they add nothing.
constexpr int MOE_ROW_ALIGN = 32;

struct rtp_moe {
    rtp_moe_desc d;
    rtp_ring *ring = nullptr;
    int next_step = 0;
    bool routed = false;                 // a forward pass has left a routing and saved activations
    std::vector<int> counts;             // [n + 1], as the dispatch kernel wrote them
    std::vector<int64_t> begin;          // [n + 1] first grouped row of each expert
    hipEvent_t ev_dw = nullptr, ev_g_in = nullptr, ev_dpre = nullptr;
};

static bool moe_gated(const rtp_moe_desc *d) { return d->act == RTP_ACT_SWIGLU; }

extern "C" int64_t rtp_moe_padded_rows(int64_t T, int n)
{
    if (T < 0 || n < 1) return -1;
    return (int64_t)MOE_ROW_ALIGN * (T / MOE_ROW_ALIGN + n);
}

extern "C" size_t rtp_moe_slot_w_bytes(const rtp_moe_desc *d)
{
    if (!d || d->I <= 0 || d->O <= 0 || d->O2 <= 0) return 0;
    const size_t p = moe_gated(d) ? 2 : 1;
    return (p * (size_t)d->O * d->I + (size_t)d->O2 * d->O) * esize(d->dtype);
}

extern "C" size_t rtp_moe_slot_g_bytes(const rtp_moe_desc *d)
{
    if (!d || d->I <= 0 || d->O <= 0 || d->O2 <= 0) return 0;
    const size_t p = moe_gated(d) ? 2 : 1;
    return (p * (size_t)d->O * d->I + (size_t)d->O2 * d->O) * 4;
}

extern "C" rtp_status rtp_moe_create(rtp_moe **out, const rtp_moe_desc *d)
{
    if (!out || !d) return fail(RTP_ERR_INVALID, "rtp_moe_create: null argument");
    *out = nullptr;
    if (d->flags & RTP_FLAG_DRY_RUN) return fail(RTP_ERR_UNSUPPORTED, "rtp_moe_create: no dry run (the routing is read on the device)");
    if (d->act <= RTP_ACT_NONE || d->act > RTP_ACT_SWIGLU) return fail(RTP_ERR_INVALID, "rtp_moe_create: an expert has an activation");
    if (d->dtype != RTP_BF16 && d->dtype != RTP_F16) return fail(RTP_ERR_UNSUPPORTED, "rtp_moe_create: 16-bit inputs only");
    if (d->n < 1 || d->n > MOE_MAX_EXPERTS) return fail(RTP_ERR_SHAPE, "rtp_moe_create: 1 to %d experts", MOE_MAX_EXPERTS);
    if (d->T < 0 || d->I <= 0 || d->O <= 0 || d->O2 <= 0 || d->T > 0x3fffffff || d->I > 0x3fffffff || d->O > 0x3fffffff ||
        d->O2 > 0x3fffffff)
        return fail(RTP_ERR_SHAPE, "rtp_moe_create: bad sizes");
    const int64_t mult = d->dtype == RTP_F16 ? 32 : 8;
    if ((d->I % mult) || (d->O % mult) || (d->O2 % mult))
        return fail(d->dtype == RTP_F16 ? RTP_ERR_UNSUPPORTED : RTP_ERR_SHAPE,
                    "rtp_moe_create: I, O and O2 must be multiples of %d for this input type", (int)mult);
    if (!d->xp_dev || !d->preact_dev || !d->hidden_dev || !d->yp_dev || !d->dpre_dev || !d->dxp_dev || !d->perm_dev ||
        !d->counts_dev)
        return fail(RTP_ERR_INVALID, "rtp_moe_create: a workspace buffer is missing");
    rtp_ring_desc rd;
    memset(&rd, 0, sizeof rd);
    rd.n = d->n; rd.rank = d->rank; rd.mode = d->mode; rd.flags = d->flags;
    rd.w_bytes = rtp_moe_slot_w_bytes(d);
    rd.g_bytes = rtp_moe_slot_g_bytes(d);
    rd.home_w_dev = d->home_w_dev; rd.home_g_dev = d->home_g_dev;
    rd.buf_w_dev[0] = d->buf_w_dev[0]; rd.buf_w_dev[1] = d->buf_w_dev[1];
    rd.buf_g_dev[0] = d->buf_g_dev[0]; rd.buf_g_dev[1] = d->buf_g_dev[1];
    rd.compute_stream = d->compute_stream; rd.stage_stream = d->stage_stream; rd.aux_stream = d->aux_stream;
    rtp_moe *m = new (std::nothrow) rtp_moe;
    if (!m) return fail(RTP_ERR_INVALID, "out of host memory");
    m->d = *d;
    m->counts.assign((size_t)d->n + 1, 0);
    m->begin.assign((size_t)d->n + 1, 0);
    rtp_status s = rtp_ring_create(&m->ring, &rd);
    if (s != RTP_OK) { delete m; return s; }
    *out = m;
    return RTP_OK;
}

extern "C" rtp_status rtp_moe_destroy(rtp_moe *m)
{
    if (!m) return RTP_OK;
    if (m->ring->pass != RTP_PASS_IDLE) return fail(RTP_ERR_STATE, "rtp_moe_destroy: a pass is open");
    for (hipEvent_t e : {m->ev_dw, m->ev_g_in, m->ev_dpre})
        if (e) (void)hipEventDestroy(e);
    RTP_TRY(rtp_ring_destroy(m->ring));
    delete m;
    return RTP_OK;
}

extern "C" rtp_ring *rtp_moe_ring(rtp_moe *m) { return m ? m->ring : nullptr; }
extern "C" rtp_status rtp_moe_flush(rtp_moe *m) { return m ? rtp_ring_flush(m->ring) : fail(RTP_ERR_INVALID, "null moe"); }
extern "C" rtp_status rtp_moe_sync(rtp_moe *m) { return m ? rtp_ring_sync(m->ring) : fail(RTP_ERR_INVALID, "null moe"); }

extern "C" rtp_status rtp_moe_set_ablation(rtp_moe *m, int rotate, int compute)
{
    if (!m) return fail(RTP_ERR_INVALID, "null moe");
    return set_ablation(m->ring, rotate, compute);
}

extern "C" rtp_status rtp_moe_routing(const rtp_moe *m, int32_t *counts_out, int64_t *begin_out)
{
    if (!m) return fail(RTP_ERR_INVALID, "null moe");
    if (!m->routed) return fail(RTP_ERR_STATE, "rtp_moe_routing: no forward pass has run");
    for (int e = 0; e < m->d.n; ++e)
        if (counts_out) counts_out[e] = m->counts[(size_t)e];
    for (int e = 0; e <= m->d.n; ++e)
        if (begin_out) begin_out[e] = m->begin[(size_t)e];
    return RTP_OK;
}

static rtp_status moe_gemm(rtp_moe *m, int layout, GemmArgs &a, hipStream_t st)
{
    rtp_ring *r = m->ring;
    if (!r->abl_compute || a.M <= 0 || a.N <= 0 || a.K <= 0) return RTP_OK;
    RTP_TRY(aux_delay(r, st));
    a.elem = m->d.dtype == RTP_F16 ? ELEM_F16 : ELEM_BF16;
    HIP_TRY(timed_launch(layout, 2.0 * a.M * a.N * a.K, st, [&] { return launch_gemm_bf16(layout, a, 0, st); }));
    return RTP_OK;
}

static rtp_status moe_events(rtp_moe *m)
{
    for (hipEvent_t *e : {&m->ev_dw, &m->ev_g_in, &m->ev_dpre})
        if (!*e) HIP_TRY(hipEventCreateWithFlags(e, hipEventDisableTiming));
    return RTP_OK;
}

static rtp_status moe_fwd_pass(rtp_moe *m, const void *X, const int32_t *route, void *Y)
{
    rtp_ring *r = m->ring;
    const rtp_moe_desc &d = m->d;
    if (d.T > 0 && (!X || !route || !Y)) return fail(RTP_ERR_INVALID, "rtp_moe_fwd: null tensor");
    if (r->pass != RTP_PASS_IDLE) return fail(RTP_ERR_STATE, "rtp_moe_fwd: a pass is open");
    RTP_TRY(refuse_capture(r, "rtp_moe_fwd"));
    RTP_TRY(moe_events(m));
    const int n = d.n;
    const size_t es = esize(d.dtype);
    const int64_t P = moe_gated(&d) ? 2 : 1, PO = P * d.O;
    const int64_t cap = rtp_moe_padded_rows(d.T, n);
    hipStream_t cs = r->cs();
    m->routed = false;
    // ---- group the tokens; the host needs the group sizes to shape the GEMMs: the one wait of the pass
    HIP_TRY(launch_moe_dispatch(route, (int)d.T, n, MOE_ROW_ALIGN, (int)cap, d.counts_dev, d.perm_dev, cs));
    HIP_TRY(hipMemcpyAsync(m->counts.data(), d.counts_dev, ((size_t)n + 1) * sizeof(int), hipMemcpyDeviceToHost, cs));
    HIP_TRY(hipStreamSynchronize(cs));
    if (m->counts[(size_t)n] != 0)
        return fail(RTP_ERR_INVALID, "rtp_moe_fwd: %d tokens are routed to an expert outside [0, %d)", m->counts[(size_t)n], n);
    m->begin[0] = 0;
    for (int e = 0; e < n; ++e)
        m->begin[(size_t)e + 1] = m->begin[(size_t)e] + (m->counts[(size_t)e] + MOE_ROW_ALIGN - 1) / MOE_ROW_ALIGN * MOE_ROW_ALIGN;
    const int64_t rows = m->begin[(size_t)n];
    if (rows > cap) return fail(RTP_ERR_STATE, "rtp_moe_fwd: grouped rows exceed the workspace");
    HIP_TRY(launch_gather_rows(d.xp_dev, X, d.perm_dev, (int)rows, (size_t)d.I * es, cs));

    RTP_TRY(rtp_ring_begin(r, RTP_PASS_FWD));
    m->next_step = 0;
    for (int t = 0; t < n; ++t) {
        if (t < n - 1) RTP_TRY(rtp_rotate_step(r, RTP_CW, t));
        RTP_TRY(enter_step(r, m->next_step, t, RTP_PASS_FWD, "rtp_moe_fwd"));
        const int e = r->abl_rotate ? r->resident : rtp_fwd_shard(d.rank, t, n);
        r->rec(TR_FWD, t, e, r->res_idx);
        const int64_t b = m->begin[(size_t)e], rows_e = m->begin[(size_t)e + 1] - b;
        const char *W1 = (const char *)r->d.buf_w_dev[r->res_idx];
        const char *W2 = W1 + (size_t)PO * d.I * es;
        GemmArgs a;
        memset(&a, 0, sizeof a);
        a.A = (const char *)d.xp_dev + (size_t)b * d.I * es; a.lda = d.I;
        a.B = W1; a.ldb = d.I;
        a.M = (int)rows_e; a.N = (int)PO; a.K = (int)d.I;
        a.epi = fwd_act_epi(d.act);
        a.half = (int)d.O;
        a.aux = (char *)d.preact_dev + (size_t)b * PO * es; a.ldaux = PO;
        a.C = (char *)d.hidden_dev + (size_t)b * d.O * es; a.ldc = d.O;
        RTP_TRY(moe_gemm(m, LAY_NT, a, cs));
        memset(&a, 0, sizeof a);
        a.A = (const char *)d.hidden_dev + (size_t)b * d.O * es; a.lda = d.O;
        a.B = W2; a.ldb = d.O;
        a.M = (int)rows_e; a.N = (int)d.O2; a.K = (int)d.O;
        a.epi = EPI_STORE;
        a.C = (char *)d.yp_dev + (size_t)b * d.O2 * es; a.ldc = d.O2;
        RTP_TRY(moe_gemm(m, LAY_NT, a, cs));
        m->next_step = t + 1;
    }
    RTP_TRY(rtp_ring_end(r));
    // "concatenation": the outputs of the N steps back in token order
    if (r->abl_compute) HIP_TRY(launch_scatter_rows(Y, d.yp_dev, d.perm_dev, (int)rows, (size_t)d.O2 * es, cs));
    m->routed = true;
    return RTP_OK;
}

extern "C" rtp_status rtp_moe_fwd(rtp_moe *m, const void *X, const int32_t *route, void *Y)
{
    if (!m) return fail(RTP_ERR_INVALID, "rtp_moe_fwd: null moe");
    if (m->ring->pass != RTP_PASS_IDLE) return fail(RTP_ERR_STATE, "rtp_moe_fwd: a pass is open");
    return close_failed_pass(m->ring, moe_fwd_pass(m, X, route, Y));
}

static rtp_status moe_bwd_pass(rtp_moe *m, const void *dY, void *dX)
{
    rtp_ring *r = m->ring;
    const rtp_moe_desc &d = m->d;
    if (d.T > 0 && (!dY || !dX)) return fail(RTP_ERR_INVALID, "rtp_moe_bwd: null tensor");
    if (r->pass != RTP_PASS_IDLE) return fail(RTP_ERR_STATE, "rtp_moe_bwd: a pass is open");
    if (!m->routed) return fail(RTP_ERR_STATE, "rtp_moe_bwd: needs the routing and activations of a forward pass");
    RTP_TRY(refuse_capture(r, "rtp_moe_bwd"));
    const int n = d.n;
    const size_t es = esize(d.dtype);
    const int64_t P = moe_gated(&d) ? 2 : 1, PO = P * d.O;
    const int64_t rows = m->begin[(size_t)n];
    hipStream_t cs = r->cs(), ws = r->as();
    const bool split = ws != cs;
    // the gradient of the output, grouped like the tokens (into the buffer the expert outputs used)
    HIP_TRY(launch_gather_rows(d.yp_dev, dY, d.perm_dev, (int)rows, (size_t)d.O2 * es, cs));

    RTP_TRY(rtp_ring_begin(r, RTP_PASS_BWD));
    m->next_step = 0;
    bool own_to_slot = false;
    for (int s = 0; s < n; ++s) {
        if (s < n - 1) RTP_TRY(rtp_rotate_step(r, RTP_CCW, s));
        RTP_TRY(enter_step(r, m->next_step, s, RTP_PASS_BWD, "rtp_moe_bwd"));
        const int e = r->abl_rotate ? r->resident : rtp_bwd_shard(d.rank, s, n);
        r->rec(TR_BWD, s, e, r->res_idx);
        const int gi = r->res_g_idx;
        const int64_t b = m->begin[(size_t)e], rows_e = m->begin[(size_t)e + 1] - b;
        const char *W1 = (const char *)r->d.buf_w_dev[r->res_idx];
        const char *W2 = W1 + (size_t)PO * d.I * es;
        float *G1 = (float *)r->d.buf_g_dev[gi];
        float *G2 = G1 + (size_t)PO * d.I;
        const char *dYe = (const char *)d.yp_dev + (size_t)b * d.O2 * es;
        const char *He = (const char *)d.hidden_dev + (size_t)b * d.O * es;
        const char *Xe = (const char *)d.xp_dev + (size_t)b * d.I * es;
        char *dPe = (char *)d.dpre_dev + (size_t)b * PO * es;
        const bool rotating = r->abl_rotate && s < n - 1;
        const bool staged_g = r->d.mode == RTP_INPLACE_STAGED;

        // the weight-gradient kernels run on the auxiliary stream when there is one
        if (split) {
            HIP_TRY(hipEventRecord(r->ev_aux, cs));
            HIP_TRY(hipStreamWaitEvent(ws, r->ev_aux, 0));
        }
        // the gradient shard this step adds onto must have arrived
        if (r->abl_rotate && s > 0) {
            if (r->d.mode == RTP_DOUBLE_BUFFER) HIP_TRY(hipStreamWaitEvent(ws, r->ev_g[s & 1], 0));
            else if (staged_g) HIP_TRY(hipStreamWaitEvent(ws, m->ev_g_in, 0));
        }
        // When the expert moves on after this step, a weight-gradient kernel writes its sum (arriving
        // content + this worker's contribution) straight to where the gradients travel to instead of
        // back into the buffer; not for a group without tokens (no kernel runs) or when the launcher
        // would cut the contraction into chunks (their partial sums need the plain `+=` form).
        const bool moves_on = rotating && r->d.g_bytes && r->d.mode != RTP_INPLACE_BLOCKING;
        auto whole_k = [&](const GemmArgs &g) {
            int ks = 1;
            if (gemm_bf16_pp_supported(LAY_TN, g)) gemm_bf16_pp_plan(LAY_TN, &g, 1, nullptr, nullptr, &ks);
            return ks == 1;
        };
        const size_t g1_bytes = (size_t)PO * d.I * 4, g2_bytes = (size_t)d.O2 * d.O * 4;
        // G2_e += dY_e^T H_e and G1_e += dPre_e^T X_e
        GemmArgs a2, a1;
        memset(&a2, 0, sizeof a2);
        a2.A = dYe; a2.lda = d.O2;
        a2.B = He; a2.ldb = d.O;
        a2.M = (int)d.O2; a2.N = (int)d.O; a2.K = (int)rows_e;
        a2.epi = EPI_ACC_ADD; a2.c_is_f32 = 1;
        a2.ws = G2; a2.ldws = d.O; a2.C = G2; a2.ldc = d.O;
        a2.cu_share = split ? 2 : 1;
        memset(&a1, 0, sizeof a1);
        a1.A = dPe; a1.lda = PO;
        a1.B = Xe; a1.ldb = d.I;
        a1.M = (int)PO; a1.N = (int)d.I; a1.K = (int)rows_e;
        a1.epi = EPI_ACC_ADD; a1.c_is_f32 = 1;
        a1.ws = G1; a1.ldws = d.I; a1.C = G1; a1.ldc = d.I;
        a1.cu_share = split ? 2 : 1;
        // The expert of the last step is the worker's own and goes nowhere (Design section, workflow paragraph): its
        // kernels store the sum straight into the own slot and nothing stays behind in the buffer.  Both matrices or
        // neither: a write-back of the whole buffer would overwrite the one that is current in the slot only.
        const bool stays = s == n - 1 && r->abl_rotate && n > 1 && r->d.g_bytes && r->d.mode != RTP_INPLACE_BLOCKING &&
                           r->abl_compute && rows_e > 0 && whole_k(a2) && whole_k(a1);
        own_to_slot = stays;
        auto send_fused = [&](GemmArgs &g, size_t g_off) {
            if (!stays && (!moves_on || !r->abl_compute || rows_e <= 0 || !whole_k(g))) return false;
            g.epi = EPI_ACC_LAST;
            g.C = r->home_g(e) + g_off;
            return true;
        };
        GemmArgs a;
        const bool sent2 = send_fused(a2, g1_bytes);
        RTP_TRY(moe_gemm(m, LAY_TN, a2, ws));
        // dPre_e = (dY_e W2_e) * act'(pre_e)
        memset(&a, 0, sizeof a);
        a.A = dYe; a.lda = d.O2;
        a.B = W2; a.ldb = d.O;
        a.M = (int)rows_e; a.N = (int)d.O; a.K = (int)d.O2;
        a.epi = bwd_act_epi(d.act);
        a.half = (int)d.O;
        a.aux = (char *)d.preact_dev + (size_t)b * PO * es; a.ldaux = PO;
        a.C = dPe; a.ldc = PO;
        a.cu_share = split ? 2 : 1;
        RTP_TRY(moe_gemm(m, LAY_NN, a, cs));
        if (split) {
            HIP_TRY(hipEventRecord(m->ev_dpre, cs));
            HIP_TRY(hipStreamWaitEvent(ws, m->ev_dpre, 0));
        }
        const bool sent1 = send_fused(a1, 0);
        RTP_TRY(moe_gemm(m, LAY_TN, a1, ws));
        // the expert's gradients move on with it: handed to the stage stream once both kernels are done
        if (moves_on) {
            const int ein = rtp_bwd_shard(d.rank, s + 1, n);
            HIP_TRY(hipEventRecord(m->ev_dw, ws));
            HIP_TRY(hipStreamWaitEvent(r->ss(), m->ev_dw, 0));
            char *buf = (char *)r->d.buf_g_dev[gi];
            if (!sent1) RTP_TRY(copy_async(r, r->home_g(e), buf, g1_bytes, r->ss()));
            if (!sent2) RTP_TRY(copy_async(r, r->home_g(e) + g1_bytes, buf + g1_bytes, g2_bytes, r->ss()));
            r->rec(TR_G_OUT, s, e, gi);
            if (staged_g) {
                RTP_TRY(copy_async(r, r->d.buf_g_dev[gi], r->home_g(ein), r->d.g_bytes, r->ss(), m->ev_g_in));
                r->rec(TR_G_IN, s, ein, gi);
            }
        }
        // dX_e = dPre_e W1_e
        memset(&a, 0, sizeof a);
        a.A = dPe; a.lda = PO;
        a.B = W1; a.ldb = d.I;
        a.M = (int)rows_e; a.N = (int)d.I; a.K = (int)PO;
        a.epi = EPI_STORE;
        a.C = (char *)d.dxp_dev + (size_t)b * d.I * es; a.ldc = d.I;
        a.cu_share = split ? 2 : 1;
        RTP_TRY(moe_gemm(m, LAY_NN, a, cs));
        m->next_step = s + 1;
    }
    if (own_to_slot) r->res_g = -1; // the slot is current
    RTP_TRY(rtp_ring_end(r));
    if (r->abl_compute) HIP_TRY(launch_scatter_rows(dX, d.dxp_dev, d.perm_dev, (int)rows, (size_t)d.I * es, cs));
    return RTP_OK;
}

extern "C" rtp_status rtp_moe_bwd(rtp_moe *m, const void *dY, void *dX)
{
    if (!m) return fail(RTP_ERR_INVALID, "rtp_moe_bwd: null moe");
    if (m->ring->pass != RTP_PASS_IDLE) return fail(RTP_ERR_STATE, "rtp_moe_bwd: a pass is open");
    return close_failed_pass(m->ring, moe_bwd_pass(m, dY, dX));
}

// ---------------------------------------------------------------------------
// single GEMM launch
// ---------------------------------------------------------------------------
extern "C" rtp_status rtp_gemm(int layout, rtp_dtype in_dtype, rtp_dtype out_dtype, int accumulate, const void *A,
                               int64_t lda, const void *B, int64_t ldb, void *C, int64_t ldc, int64_t M, int64_t N,
                               int64_t K, int variant, void *stream)
{
    if (!A || !B || !C) return fail(RTP_ERR_INVALID, "rtp_gemm: null pointer");
    if (layout < 0 || layout > 2) return fail(RTP_ERR_INVALID, "rtp_gemm: bad layout");
    if (M < 0 || N < 0 || K <= 0 || M > 0x7fffffff || N > 0x7fffffff || K > 0x7fffffff)
        return fail(RTP_ERR_SHAPE, "rtp_gemm: bad sizes");
    if (accumulate && out_dtype != RTP_F32) return fail(RTP_ERR_UNSUPPORTED, "rtp_gemm: accumulation is fp32 only");
    GemmArgs a;
    memset(&a, 0, sizeof a);
    a.A = A; a.lda = lda; a.B = B; a.ldb = ldb;
    a.M = (int)M; a.N = (int)N; a.K = (int)K;
    a.C = C; a.ldc = ldc; a.ws = (float *)C; a.ldws = ldc;
    a.epi = accumulate ? EPI_ACC_ADD : EPI_STORE;
    a.c_is_f32 = out_dtype == RTP_F32;
    if (in_dtype == RTP_BF16 || in_dtype == RTP_F16) {
        if (out_dtype != RTP_F32 && out_dtype != in_dtype) return fail(RTP_ERR_UNSUPPORTED, "rtp_gemm: bad output type");
        a.elem = in_dtype == RTP_F16 ? ELEM_F16 : ELEM_BF16;
        hipError_t e = timed_launch(layout, 2.0 * a.M * a.N * a.K, (hipStream_t)stream,
                                    [&] { return launch_gemm_bf16(layout, a, variant, (hipStream_t)stream); });
        if (e == hipErrorInvalidValue) return fail(RTP_ERR_SHAPE, "rtp_gemm: sizes/alignment the bf16 kernels need are not met");
        HIP_TRY(e);
    } else if (in_dtype == RTP_F32) {
        if (out_dtype != RTP_F32) return fail(RTP_ERR_UNSUPPORTED, "rtp_gemm: fp32 inputs give fp32 outputs");
        HIP_TRY(launch_gemm_f32(layout, a, (hipStream_t)stream));
    } else {
        return fail(RTP_ERR_UNSUPPORTED, "rtp_gemm: input type not built");
    }
    return RTP_OK;
}

extern "C" rtp_status rtp_clock_probe(void *stream, void *out_dev, int64_t wall_us, int *wall_khz)
{
    if (!out_dev || ((uintptr_t)out_dev & 7)) return fail(RTP_ERR_INVALID, "rtp_clock_probe: null or misaligned output");
    if (wall_us < 0) return fail(RTP_ERR_INVALID, "rtp_clock_probe: negative duration");
    int dev = 0, khz = 0;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev));
    if (khz <= 0) return fail(RTP_ERR_UNSUPPORTED, "rtp_clock_probe: the device reports no wall clock rate");
    if (wall_khz) *wall_khz = khz;
    const int64_t us = std::min<int64_t>(wall_us, 1000000);
    HIP_TRY(launch_clock_probe((long long *)out_dev, us * (int64_t)khz / 1000, (hipStream_t)stream));
    return RTP_OK;
}

extern "C" const char *rtp_gemm_kernel_name(int layout, int variant) { return gemm_bf16_kernel_name(layout, variant); }
