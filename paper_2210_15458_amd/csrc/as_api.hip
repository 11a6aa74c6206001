// extern "C" entry points: argument checks on the host, then kernel launches on
// the context's stream.  No entry point synchronises the device except
// as_ctx_destroy and as_model_create_bigram / as_model_destroy.
#include <math.h>
#include <stdlib.h>

#include <mutex>
#include <new>

#include "as_common.hpp"

// Workspace of as_step_static, the entry point for callers that cannot allocate: the per-row keep thresholds
// that the threshold kernel hands to the sampling kernel.  Every GPU the library runs on holds its own copy
// (256 KiB) until the process ends.  In host code this name is only a handle for hipGetSymbolAddress; the
// address the kernels are given is looked up once per device (static_scratch below).
constexpr int64_t kStaticMaxRows = AS_STATIC_MAX_ROWS;
static __device__ __align__(256) float scratch[kStaticMaxRows];

namespace as {

static thread_local std::string g_err;

as_status fail(as_ctx *ctx, as_status code, const std::string &msg)
{
    if (ctx) ctx->err = msg;
    else g_err = msg;
    return code;
}

as_status hip_fail(as_ctx *ctx, hipError_t e, const char *what)
{
    return fail(ctx, AS_ERR_DEVICE, std::string(what) + ": " + hipGetErrorString(e));
}

bool profile_acquire(as_ctx *ctx, int kid, hipEvent_t *start, hipEvent_t *stop)
{
    Profile &p = ctx->prof;
    if (p.used[kid] >= kProfileCapacity) {
        ++p.dropped[kid];
        return false;
    }
    if (p.used[kid] == p.slots[kid].size()) {
        ProfileSlot s;
        if (hipEventCreate(&s.start) != hipSuccess || hipEventCreate(&s.stop) != hipSuccess) {
            (void)hipGetLastError();
            ++p.dropped[kid];
            return false;
        }
        p.slots[kid].push_back(s);
    }
    *start = p.slots[kid][p.used[kid]].start;
    *stop = p.slots[kid][p.used[kid]].stop;
    ++p.used[kid];
    return true;
}

static as_status grow(as_ctx *ctx, DeviceBuf &b, size_t bytes)
{
    if (b.bytes >= bytes) return AS_OK;
    if (b.ptr) {
        AS_HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
        AS_HIP_TRY(ctx, hipFree(b.ptr));
        b.ptr = nullptr;
        b.bytes = 0;
    }
    if (hipMalloc(&b.ptr, bytes) != hipSuccess) {
        b.ptr = nullptr;
        (void)hipGetLastError();
        return fail(ctx, AS_ERR_ALLOC, "device allocation of the decode workspace failed");
    }
    b.bytes = bytes;
    return AS_OK;
}

// Row indices handed in by the caller, as the kernels use them: a copy in the context's workspace with every
// index brought into [0, logits_rows) (an index outside is a caller's error that no call can report, since
// none reads device data back; it must not send a kernel outside the logits).
__global__ void row_ids_in_range_kernel(const int32_t *in, int32_t *out, int64_t n, int64_t logits_rows)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int64_t v = in[i];
    out[i] = (int32_t)(v < 0 ? 0 : (v > logits_rows - 1 ? logits_rows - 1 : v));
}

static as_status row_ids_in_range(as_ctx *ctx, const int32_t *&row_ids, int64_t rows, int64_t logits_rows)
{
    if (!row_ids) return AS_OK;
    const int64_t top = logits_rows < 0x7fffffffLL ? logits_rows : 0x7fffffffLL;
    hipLaunchKernelGGL(row_ids_in_range_kernel, dim3((unsigned)((rows + 255) / 256)), dim3(256), 0, ctx->stream,
                       row_ids, ctx->rid, rows, top);
    AS_HIP_TRY(ctx, hipGetLastError());
    row_ids = ctx->rid;
    return AS_OK;
}

// Device address of `scratch` on the current device, looked up on the first call made with that device current.
constexpr int kMaxDevices = 64;
static std::mutex g_static_mu;
static float *g_static_ptr[kMaxDevices] = {};

static as_status static_scratch(int *device_out, float **ptr_out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(nullptr, e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(nullptr, AS_ERR_UNSUPPORTED, "device ordinal beyond 63");
    std::lock_guard<std::mutex> lock(g_static_mu);
    if (!g_static_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            (void)hipGetLastError();
            return hip_fail(nullptr, e, "hipGetSymbolAddress(scratch)");
        }
        g_static_ptr[dev] = static_cast<float *>(p);
    }
    *device_out = dev;
    *ptr_out = g_static_ptr[dev];
    return AS_OK;
}

static bool truncation_on(int32_t V, int32_t top_k, float top_p)
{
    return (top_k > 0 && top_k < V) || (top_p > 0.f && top_p < 1.f);
}

static as_status check_step(as_ctx *ctx, const void *logits, int64_t rows, int64_t ld, const float *codes,
                            float temp, const int32_t *tokens_out, const float *codes_out)
{
    if (!ctx) return fail(nullptr, AS_ERR_INVALID_ARG, "ctx is NULL");
    if (rows < 0 || rows > ctx->max_rows) return fail(ctx, AS_ERR_INVALID_ARG, "rows outside [0, max_rows]");
    if (rows == 0) return AS_OK;
    if (!logits || !codes || !tokens_out || !codes_out)
        return fail(ctx, AS_ERR_INVALID_ARG, "logits, codes, tokens_out and codes_out must not be NULL");
    if (ld < ctx->V) return fail(ctx, AS_ERR_INVALID_ARG, "ld is smaller than the vocabulary");
    if (!(temp > 0.f) || !isfinite(temp)) return fail(ctx, AS_ERR_INVALID_ARG, "temp must be finite and > 0");
    const size_t esz = ctx->dtype == AS_BF16 ? 2 : 4;
    if (reinterpret_cast<uintptr_t>(logits) % esz != 0)
        return fail(ctx, AS_ERR_INVALID_ARG, "logits pointer is not aligned to its element type");
    return AS_OK;
}

}  // namespace as

using namespace as;

extern "C" {

as_status as_ctx_create(as_ctx **out, int64_t max_rows, int32_t V, as_dtype logits_dtype, void *hip_stream)
{
    if (!out) return fail(nullptr, AS_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (max_rows < 1 || max_rows > 0x7fffffffLL) return fail(nullptr, AS_ERR_INVALID_ARG, "max_rows outside [1, 2^31)");
    if (V < 1 || V > AS_MAX_VOCAB) return fail(nullptr, AS_ERR_INVALID_ARG, "V outside [1, AS_MAX_VOCAB]");
    if (logits_dtype != AS_F32 && logits_dtype != AS_BF16)
        return fail(nullptr, AS_ERR_INVALID_ARG, "unknown logits dtype");
    as_ctx *c = new (std::nothrow) as_ctx();
    if (!c) return fail(nullptr, AS_ERR_ALLOC, "host allocation failed");
    hipError_t e = hipGetDevice(&c->device);
    if (e != hipSuccess) {
        delete c;
        return hip_fail(nullptr, e, "hipGetDevice");
    }
    c->stream = static_cast<hipStream_t>(hip_stream);
    c->max_rows = max_rows;
    c->V = V;
    c->dtype = logits_dtype;
    e = hipDeviceGetAttribute(&c->num_cus, hipDeviceAttributeMultiprocessorCount, c->device);
    if (e != hipSuccess) {
        delete c;
        return hip_fail(nullptr, e, "hipDeviceGetAttribute");
    }
    e = hipMalloc(reinterpret_cast<void **>(&c->thr), (size_t)max_rows * sizeof(float));
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&c->rid), (size_t)max_rows * sizeof(int32_t));
    if (e != hipSuccess) {
        (void)hipGetLastError();
        if (c->thr) (void)hipFree(c->thr);
        delete c;
        return fail(nullptr, AS_ERR_ALLOC, "device allocation of the context workspace failed");
    }
    *out = c;
    return AS_OK;
}

as_status as_ctx_destroy(as_ctx *ctx)
{
    if (!ctx) return AS_OK;
    (void)hipStreamSynchronize(ctx->stream);
    if (ctx->thr) (void)hipFree(ctx->thr);
    if (ctx->rid) (void)hipFree(ctx->rid);
    if (ctx->logits.ptr) (void)hipFree(ctx->logits.ptr);
    if (ctx->state.ptr) (void)hipFree(ctx->state.ptr);
    for (auto &v : ctx->prof.slots)
        for (auto &s : v) {
            (void)hipEventDestroy(s.start);
            (void)hipEventDestroy(s.stop);
        }
    delete ctx;
    return AS_OK;
}

const char *as_last_error(const as_ctx *ctx) { return ctx ? ctx->err.c_str() : g_err.c_str(); }

as_status as_ctx_set_tuning(as_ctx *ctx, as_tuning knob, int32_t value)
{
    if (!ctx) return fail(nullptr, AS_ERR_INVALID_ARG, "ctx is NULL");
    if (value < 0) return fail(ctx, AS_ERR_INVALID_ARG, "a tuning value is >= 0");
    switch (knob) {
    case AS_TUNE_STEP_SHAPE: ctx->step_shape = value; return AS_OK;
    case AS_TUNE_GEMM_SHAPE: ctx->gemm_shape = value; return AS_OK;
    case AS_TUNE_THR_PATH: ctx->thr_path = value; return AS_OK;
    case AS_TUNE_GEMM_GM: ctx->gemm_gm = value; return AS_OK;
    }
    return fail(ctx, AS_ERR_INVALID_ARG, "unknown tuning knob");
}

as_status as_ctx_profile(as_ctx *ctx, int enable)
{
    if (!ctx) return fail(nullptr, AS_ERR_INVALID_ARG, "ctx is NULL");
    ctx->prof.on = enable != 0;
    return AS_OK;
}

as_status as_ctx_profile_read(as_ctx *ctx, int kernel, double *total_ms, int64_t *launches, int64_t *untimed)
{
    if (!ctx) return fail(nullptr, AS_ERR_INVALID_ARG, "ctx is NULL");
    if (kernel < 0 || kernel >= kKernelCount) return fail(ctx, AS_ERR_INVALID_ARG, "unknown kernel id");
    AS_HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    Profile &p = ctx->prof;
    double ms = 0.0;
    for (size_t i = 0; i < p.used[kernel]; ++i) {
        float t = 0.f;
        AS_HIP_TRY(ctx, hipEventElapsedTime(&t, p.slots[kernel][i].start, p.slots[kernel][i].stop));
        ms += t;
    }
    if (total_ms) *total_ms = ms;
    if (launches) *launches = (int64_t)p.used[kernel];
    if (untimed) *untimed = (int64_t)p.dropped[kernel];
    p.used[kernel] = 0;
    p.dropped[kernel] = 0;
    return AS_OK;
}

as_status as_ctx_profile_samples(as_ctx *ctx, int kernel, float *ms_out, int64_t capacity, int64_t *count)
{
    if (!ctx) return fail(nullptr, AS_ERR_INVALID_ARG, "ctx is NULL");
    if (kernel < 0 || kernel >= kKernelCount) return fail(ctx, AS_ERR_INVALID_ARG, "unknown kernel id");
    if (capacity < 0 || (capacity > 0 && !ms_out)) return fail(ctx, AS_ERR_INVALID_ARG, "ms_out is NULL");
    AS_HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    Profile &p = ctx->prof;
    const int64_t n = (int64_t)p.used[kernel] < capacity ? (int64_t)p.used[kernel] : capacity;
    for (int64_t i = 0; i < n; ++i)
        AS_HIP_TRY(ctx, hipEventElapsedTime(&ms_out[i], p.slots[kernel][i].start, p.slots[kernel][i].stop));
    if (count) *count = (int64_t)p.used[kernel];
    return AS_OK;
}

as_status as_step_ex(as_ctx *ctx, const void *logits, int64_t rows, int64_t ld, const float *codes, float temp,
                     int32_t top_k, float top_p, int32_t *tokens_out, float *codes_out,
                     const uint8_t *finished_in, int32_t eos_id, uint8_t *finished_out, float *prob_out,
                     float *flo_out, const int32_t *row_ids, int64_t logits_rows)
{
    as_status st = check_step(ctx, logits, rows, ld, codes, temp, tokens_out, codes_out);
    if (st != AS_OK || rows == 0) return st;
    if (row_ids && logits_rows < 1) return fail(ctx, AS_ERR_INVALID_ARG, "row_ids given but logits_rows < 1");
    if (finished_in && eos_id < 0)
        return fail(ctx, AS_ERR_INVALID_ARG, "finished_in given without an eos_id to emit");
    if (eos_id >= ctx->V) return fail(ctx, AS_ERR_INVALID_ARG, "eos_id outside the vocabulary");
    if (isnan(top_p)) return fail(ctx, AS_ERR_INVALID_ARG, "top_p is NaN");
    st = row_ids_in_range(ctx, row_ids, rows, logits_rows);
    if (st != AS_OK) return st;

    StepArgs a{};
    a.logits = logits; a.rows = rows; a.ld = ld; a.V = ctx->V; a.dtype = ctx->dtype;
    a.codes = codes; a.temp = temp; a.k = 1.44269504088896340736f / temp; a.thr = nullptr;
    a.tokens_out = tokens_out; a.tok_stride = 1; a.codes_out = codes_out;
    a.finished_in = finished_in; a.eos_id = eos_id; a.finished_out = finished_out;
    a.prob_out = prob_out; a.flo_out = flo_out; a.row_ids = row_ids; a.prev_out = nullptr;
    if (truncation_on(ctx->V, top_k, top_p)) {
        // top-k rows that fit the resident kernel are finished there; otherwise threshold, then step
        if (launch_topk_step(ctx, a, top_k, top_p, &st)) return st;
        st = launch_threshold(ctx, logits, rows, ld, finished_in, row_ids, temp, top_k, top_p, ctx->thr);
        if (st != AS_OK) return st;
        a.thr = ctx->thr;
    }
    return launch_step(ctx, a);
}

as_status as_step(as_ctx *ctx, const void *logits, int64_t rows, int64_t ld, const float *codes, float temp,
                  int32_t top_k, float top_p, int32_t *tokens_out, float *codes_out)
{
    return as_step_ex(ctx, logits, rows, ld, codes, temp, top_k, top_p, tokens_out, codes_out, nullptr, -1,
                      nullptr, nullptr, nullptr, nullptr, 0);
}

as_status as_step_static(const void *logits, as_dtype logits_dtype, int64_t rows, int64_t ld, int32_t V,
                         const float *codes, float temp, int32_t top_k, float top_p, int32_t *tokens_out,
                         float *codes_out, void *hip_stream)
{
    if (V < 1 || V > AS_MAX_VOCAB) return fail(nullptr, AS_ERR_INVALID_ARG, "V outside [1, AS_MAX_VOCAB]");
    if (logits_dtype != AS_F32 && logits_dtype != AS_BF16)
        return fail(nullptr, AS_ERR_INVALID_ARG, "unknown logits dtype");
    if (rows < 0) return fail(nullptr, AS_ERR_INVALID_ARG, "rows is negative");
    if (rows > kStaticMaxRows)
        return fail(nullptr, AS_ERR_INVALID_ARG,
                    "rows exceeds AS_STATIC_MAX_ROWS (65536), the size of the static workspace of as_step_static");
    if (isnan(top_p)) return fail(nullptr, AS_ERR_INVALID_ARG, "top_p is NaN");
    // a context that lives for this call only and owns nothing: its threshold workspace is the static array
    as_ctx c;
    as_status st = static_scratch(&c.device, &c.thr);
    if (st != AS_OK) return st;
    c.stream = static_cast<hipStream_t>(hip_stream);
    c.max_rows = kStaticMaxRows;
    c.V = V;
    c.dtype = logits_dtype;
    st = check_step(&c, logits, rows, ld, codes, temp, tokens_out, codes_out);
    if (st == AS_OK && rows > 0) {
        StepArgs a{};
        a.logits = logits; a.rows = rows; a.ld = ld; a.V = V; a.dtype = logits_dtype;
        a.codes = codes; a.temp = temp; a.k = 1.44269504088896340736f / temp; a.thr = nullptr;
        a.tokens_out = tokens_out; a.tok_stride = 1; a.codes_out = codes_out;
        a.finished_in = nullptr; a.eos_id = -1; a.finished_out = nullptr;
        a.prob_out = nullptr; a.flo_out = nullptr; a.row_ids = nullptr; a.prev_out = nullptr;
        bool done = false;
        if (truncation_on(V, top_k, top_p)) {
            done = launch_topk_step(&c, a, top_k, top_p, &st);
            if (!done) {
                st = launch_threshold(&c, logits, rows, ld, nullptr, nullptr, temp, top_k, top_p, c.thr);
                a.thr = c.thr;
            }
        }
        if (!done && st == AS_OK) st = launch_step(&c, a);
    }
    if (st != AS_OK) g_err = c.err;
    return st;
}

as_status as_lattice(as_ctx *ctx, const float *u, int32_t B, int32_t N, float *codes_out)
{
    if (!ctx) return fail(nullptr, AS_ERR_INVALID_ARG, "ctx is NULL");
    if (B < 0 || N < 1) return fail(ctx, AS_ERR_INVALID_ARG, "B must be >= 0 and N >= 1");
    if ((int64_t)B * N > ctx->max_rows) return fail(ctx, AS_ERR_INVALID_ARG, "B*N exceeds max_rows");
    if (B == 0) return AS_OK;
    if (!u || !codes_out) return fail(ctx, AS_ERR_INVALID_ARG, "u and codes_out must not be NULL");
    return launch_lattice(ctx, u, B, N, codes_out, nullptr, nullptr, nullptr);
}

as_status as_model_create_bigram(as_model **out, const void *E, const void *U, int32_t V, int32_t d, float scale,
                                 as_dtype wdtype)
{
    if (!out) return fail(nullptr, AS_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (!E || !U) return fail(nullptr, AS_ERR_INVALID_ARG, "E and U must not be NULL");
    if (V < 1 || V > AS_MAX_VOCAB || d < 1) return fail(nullptr, AS_ERR_INVALID_ARG, "V or d out of range");
    if (wdtype != AS_F32 && wdtype != AS_BF16) return fail(nullptr, AS_ERR_INVALID_ARG, "unknown weight dtype");
    if (!isfinite(scale)) return fail(nullptr, AS_ERR_INVALID_ARG, "scale must be finite");
    as_model *m = new (std::nothrow) as_model();
    if (!m) return fail(nullptr, AS_ERR_ALLOC, "host allocation failed");
    (void)hipGetDevice(&m->device);
    m->V = V; m->d = d; m->scale = scale; m->wdtype = wdtype; m->E = E;
    const size_t esz = wdtype == AS_BF16 ? 2 : 4;
    // rows of Ut are padded with zeros to a whole number of the logits kernel's 256-column tiles, so that its
    // loader needs no bounds on the rows it requests
    const size_t vpad = ((size_t)V + 255) / 256 * 256;
    if (hipMalloc(&m->Ut, vpad * d * esz) != hipSuccess) {
        (void)hipGetLastError();
        delete m;
        return fail(nullptr, AS_ERR_ALLOC, "device allocation of the transposed weights failed");
    }
    as_status st = AS_OK;
    if (vpad > (size_t)V &&
        hipMemset(static_cast<unsigned char *>(m->Ut) + (size_t)V * d * esz, 0, (vpad - V) * d * esz) != hipSuccess) {
        (void)hipGetLastError();
        st = fail(nullptr, AS_ERR_DEVICE, "clearing the padding of the transposed weights failed");
    }
    if (st == AS_OK) st = launch_transpose(U, m->Ut, d, V, wdtype);
    if (st != AS_OK) {
        (void)hipFree(m->Ut);
        delete m;
        return st;
    }
    *out = m;
    return AS_OK;
}

as_status as_model_destroy(as_model *model)
{
    if (!model) return AS_OK;
    (void)hipDeviceSynchronize();
    if (model->Ut) (void)hipFree(model->Ut);
    delete model;
    return AS_OK;
}

as_status as_bigram_logits(as_ctx *ctx, const as_model *model, const int32_t *prev, int64_t rows,
                           void *logits_out, int64_t ld)
{
    if (!ctx) return fail(nullptr, AS_ERR_INVALID_ARG, "ctx is NULL");
    if (!model) return fail(ctx, AS_ERR_INVALID_ARG, "model is NULL");
    if (model->V != ctx->V) return fail(ctx, AS_ERR_INVALID_ARG, "model and context disagree on V");
    if (rows < 0 || rows > ctx->max_rows) return fail(ctx, AS_ERR_INVALID_ARG, "rows outside [0, max_rows]");
    if (rows == 0) return AS_OK;
    if (!prev || !logits_out) return fail(ctx, AS_ERR_INVALID_ARG, "prev and logits_out must not be NULL");
    if (ld < ctx->V) return fail(ctx, AS_ERR_INVALID_ARG, "ld is smaller than the vocabulary");
    return launch_bigram_logits(ctx, model, prev, rows, logits_out, ld);
}

// as_decode and as_decode_ancestral: with `uniforms` the code of row r at step t is uniforms[t*R + r] and
// the rescaled code is dropped, otherwise codes start on the lattice of u and are carried from step to step.
static as_status decode_impl(as_ctx *ctx, const as_model *model, const int32_t *prompts, int32_t B, int32_t N,
                             int32_t T, const float *u, const float *uniforms, float temp, int32_t top_k,
                             float top_p, int32_t eos_id, int32_t *tokens_out, float *codes_out)
{
    if (!ctx) return fail(nullptr, AS_ERR_INVALID_ARG, "ctx is NULL");
    if (!model) return fail(ctx, AS_ERR_INVALID_ARG, "model is NULL");
    if (model->V != ctx->V) return fail(ctx, AS_ERR_INVALID_ARG, "model and context disagree on V");
    if (B < 0 || N < 1 || T < 0) return fail(ctx, AS_ERR_INVALID_ARG, "B, T must be >= 0 and N >= 1");
    const int64_t R = (int64_t)B * N;
    if (R > ctx->max_rows) return fail(ctx, AS_ERR_INVALID_ARG, "B*N exceeds max_rows");
    if (R == 0) return AS_OK;
    if (!prompts || (!u && !uniforms)) return fail(ctx, AS_ERR_INVALID_ARG, "prompts and u must not be NULL");
    if (T > 0 && !tokens_out) return fail(ctx, AS_ERR_INVALID_ARG, "tokens_out must not be NULL");
    if (!(temp > 0.f) || !isfinite(temp)) return fail(ctx, AS_ERR_INVALID_ARG, "temp must be finite and > 0");
    if (eos_id >= ctx->V) return fail(ctx, AS_ERR_INVALID_ARG, "eos_id outside the vocabulary");
    if (isnan(top_p)) return fail(ctx, AS_ERR_INVALID_ARG, "top_p is NaN");

    const size_t esz = ctx->dtype == AS_BF16 ? 2 : 4;
    const int64_t ldw = ((int64_t)ctx->V + 7) / 8 * 8;        // rows start 16-byte aligned
    as_status st = grow(ctx, ctx->logits, (size_t)R * ldw * esz);
    if (st != AS_OK) return st;
    st = grow(ctx, ctx->state, (size_t)R * 9);
    if (st != AS_OK) return st;
    float *codes = static_cast<float *>(ctx->state.ptr);
    int32_t *prev = reinterpret_cast<int32_t *>(codes + R);
    uint8_t *fin = reinterpret_cast<uint8_t *>(prev + R);

    st = launch_lattice(ctx, u, B, N, uniforms ? nullptr : codes, prompts, prev, fin);
    if (st != AS_OK) return st;
    const bool trunc = truncation_on(ctx->V, top_k, top_p);
    for (int32_t t = 0; t < T; ++t) {
        st = launch_bigram_logits(ctx, model, prev, R, ctx->logits.ptr, ldw);
        if (st != AS_OK) return st;
        StepArgs a{};
        a.logits = ctx->logits.ptr; a.rows = R; a.ld = ldw; a.V = ctx->V; a.dtype = ctx->dtype;
        a.codes = uniforms ? uniforms + (int64_t)t * R : codes; a.temp = temp; a.k = 1.44269504088896340736f / temp; a.thr = nullptr;
        a.tokens_out = tokens_out + t; a.tok_stride = T; a.codes_out = codes;
        a.finished_in = eos_id >= 0 ? fin : nullptr; a.eos_id = eos_id;
        a.finished_out = eos_id >= 0 ? fin : nullptr;
        a.prob_out = nullptr; a.flo_out = nullptr; a.row_ids = nullptr; a.prev_out = prev;
        if (trunc) {
            if (launch_topk_step(ctx, a, top_k, top_p, &st)) {
                if (st != AS_OK) return st;
                continue;
            }
            st = launch_threshold(ctx, ctx->logits.ptr, R, ldw, eos_id >= 0 ? fin : nullptr, nullptr, temp,
                                  top_k, top_p, ctx->thr);
            if (st != AS_OK) return st;
            a.thr = ctx->thr;
        }
        st = launch_step(ctx, a);
        if (st != AS_OK) return st;
    }
    if (codes_out)
        AS_HIP_TRY(ctx, hipMemcpyAsync(codes_out, codes, (size_t)R * sizeof(float), hipMemcpyDeviceToDevice,
                                       ctx->stream));
    return AS_OK;
}

as_status as_decode(as_ctx *ctx, const as_model *model, const int32_t *prompts, int32_t B, int32_t N, int32_t T,
                    const float *u, float temp, int32_t top_k, float top_p, int32_t eos_id, int32_t *tokens_out,
                    float *codes_out)
{
    if (ctx && !u) return fail(ctx, AS_ERR_INVALID_ARG, "prompts and u must not be NULL");
    return decode_impl(ctx, model, prompts, B, N, T, u, nullptr, temp, top_k, top_p, eos_id, tokens_out, codes_out);
}

as_status as_decode_ancestral(as_ctx *ctx, const as_model *model, const int32_t *prompts, int32_t B, int32_t N,
                              int32_t T, const float *uniforms, float temp, int32_t top_k, float top_p,
                              int32_t eos_id, int32_t *tokens_out)
{
    if (ctx && !uniforms && (int64_t)B * N * T > 0)
        return fail(ctx, AS_ERR_INVALID_ARG, "uniforms must not be NULL");
    return decode_impl(ctx, model, prompts, B, N, T, nullptr, uniforms, temp, top_k, top_p, eos_id, tokens_out,
                       nullptr);
}

as_status as_bigram_group_mass(as_ctx *ctx, const as_model *model, const int32_t *prev, int64_t rows, float temp,
                               float *mass_out, int64_t ldp)
{
    if (!ctx) return fail(nullptr, AS_ERR_INVALID_ARG, "ctx is NULL");
    if (!model) return fail(ctx, AS_ERR_INVALID_ARG, "model is NULL");
    if (model->V != ctx->V) return fail(ctx, AS_ERR_INVALID_ARG, "model and context disagree on V");
    if (rows < 0 || rows > ctx->max_rows) return fail(ctx, AS_ERR_INVALID_ARG, "rows outside [0, max_rows]");
    if (rows == 0) return AS_OK;
    if (!prev || !mass_out) return fail(ctx, AS_ERR_INVALID_ARG, "prev and mass_out must not be NULL");
    if (!(temp > 0.f) || !isfinite(temp)) return fail(ctx, AS_ERR_INVALID_ARG, "temp must be finite and > 0");
    const int64_t ngroups = ((int64_t)ctx->V + 31) / 32;
    if (ldp < ngroups || ldp % 16 != 0 || reinterpret_cast<uintptr_t>(mass_out) % 16 != 0)
        return fail(ctx, AS_ERR_INVALID_ARG, "ldp must be a multiple of 16 covering ceil(V/32) groups, mass_out 16-byte aligned");
    if (!fused_path_applies(ctx, model))
        return fail(ctx, AS_ERR_UNSUPPORTED,
                    "group masses need bf16 weights, a rank that is a multiple of 64 and at least 128, "
                    "and operands below 4 GB");
    return launch_bigram_partials(ctx, model, prev, rows, temp, reinterpret_cast<float2 *>(mass_out), ldp);
}

as_status as_step_fused(as_ctx *ctx, const as_model *model, const float *mass, int64_t ldp, const int32_t *prev,
                        int64_t rows, const float *codes, float temp, int32_t *tokens_out, float *codes_out,
                        const uint8_t *finished_in, int32_t eos_id, uint8_t *finished_out)
{
    if (!ctx) return fail(nullptr, AS_ERR_INVALID_ARG, "ctx is NULL");
    if (!model) return fail(ctx, AS_ERR_INVALID_ARG, "model is NULL");
    if (model->V != ctx->V) return fail(ctx, AS_ERR_INVALID_ARG, "model and context disagree on V");
    if (rows < 0 || rows > ctx->max_rows) return fail(ctx, AS_ERR_INVALID_ARG, "rows outside [0, max_rows]");
    if (rows == 0) return AS_OK;
    if (!mass || !prev || !codes || !tokens_out || !codes_out)
        return fail(ctx, AS_ERR_INVALID_ARG, "mass, prev, codes, tokens_out and codes_out must not be NULL");
    if (!(temp > 0.f) || !isfinite(temp)) return fail(ctx, AS_ERR_INVALID_ARG, "temp must be finite and > 0");
    if (finished_in && eos_id < 0) return fail(ctx, AS_ERR_INVALID_ARG, "finished_in given without an eos_id to emit");
    if (eos_id >= ctx->V) return fail(ctx, AS_ERR_INVALID_ARG, "eos_id outside the vocabulary");
    const int64_t ngroups = ((int64_t)ctx->V + 31) / 32;
    if (ldp < ngroups || ldp % 16 != 0 || ldp > 65536 || reinterpret_cast<uintptr_t>(mass) % 16 != 0)
        return fail(ctx, AS_ERR_INVALID_ARG,
                    "ldp must be a multiple of 16, at most 65536, covering ceil(V/32) groups; mass 16-byte aligned");
    if (!fused_path_applies(ctx, model))
        return fail(ctx, AS_ERR_UNSUPPORTED, "the fused step needs bf16 weights and a rank that is a multiple of 64");
    FusedArgs a{};
    a.part = reinterpret_cast<const float2 *>(mass); a.ldp = ldp; a.ngroups = (int32_t)ngroups; a.rows = rows;
    a.V = ctx->V; a.d = model->d;
    a.E = static_cast<const uint16_t *>(model->E); a.Ut = static_cast<const uint16_t *>(model->Ut);
    a.alpha = (float)((double)model->scale / sqrt((double)model->d) * 1.44269504088896340736 / (double)temp);
    a.codes = codes; a.codes_out = codes_out; a.tokens_out = tokens_out; a.tok_stride = 1;
    a.finished_in = finished_in; a.eos_id = eos_id; a.finished_out = finished_out; a.prev = prev; a.prev_out = nullptr;
    return launch_fused_sample(ctx, a);
}

as_status as_decode_fused(as_ctx *ctx, const as_model *model, const int32_t *prompts, int32_t B, int32_t N, int32_t T,
                          const float *u, float temp, int32_t eos_id, int32_t *tokens_out, float *codes_out)
{
    if (!ctx) return fail(nullptr, AS_ERR_INVALID_ARG, "ctx is NULL");
    if (!model) return fail(ctx, AS_ERR_INVALID_ARG, "model is NULL");
    if (model->V != ctx->V) return fail(ctx, AS_ERR_INVALID_ARG, "model and context disagree on V");
    if (B < 0 || N < 1 || T < 0) return fail(ctx, AS_ERR_INVALID_ARG, "B, T must be >= 0 and N >= 1");
    const int64_t R = (int64_t)B * N;
    if (R > ctx->max_rows) return fail(ctx, AS_ERR_INVALID_ARG, "B*N exceeds max_rows");
    if (R == 0) return AS_OK;
    if (!prompts || !u) return fail(ctx, AS_ERR_INVALID_ARG, "prompts and u must not be NULL");
    if (T > 0 && !tokens_out) return fail(ctx, AS_ERR_INVALID_ARG, "tokens_out must not be NULL");
    if (!(temp > 0.f) || !isfinite(temp)) return fail(ctx, AS_ERR_INVALID_ARG, "temp must be finite and > 0");
    if (eos_id >= ctx->V) return fail(ctx, AS_ERR_INVALID_ARG, "eos_id outside the vocabulary");
    if (!fused_path_applies(ctx, model))
        return fail(ctx, AS_ERR_UNSUPPORTED,
                    "the fused decode needs bf16 weights, a rank that is a multiple of 64 and at least 128, "
                    "and operands below 4 GB");

    const int32_t ngroups = (ctx->V + 31) / 32;
    const int64_t ldp = ((int64_t)ngroups + 15) / 16 * 16;
    as_status st = grow(ctx, ctx->logits, (size_t)R * ldp * sizeof(float2));
    if (st != AS_OK) return st;
    st = grow(ctx, ctx->state, (size_t)R * 9);
    if (st != AS_OK) return st;
    float *codes = static_cast<float *>(ctx->state.ptr);
    int32_t *prev = reinterpret_cast<int32_t *>(codes + R);
    uint8_t *fin = reinterpret_cast<uint8_t *>(prev + R);
    float2 *part = static_cast<float2 *>(ctx->logits.ptr);

    st = launch_lattice(ctx, u, B, N, codes, prompts, prev, fin);
    if (st != AS_OK) return st;
    for (int32_t t = 0; t < T; ++t) {
        st = launch_bigram_partials(ctx, model, prev, R, temp, part, ldp);
        if (st != AS_OK) return st;
        FusedArgs a{};
        a.part = part; a.ldp = ldp; a.ngroups = ngroups; a.rows = R; a.V = ctx->V; a.d = model->d;
        a.E = static_cast<const uint16_t *>(model->E); a.Ut = static_cast<const uint16_t *>(model->Ut);
        a.alpha = (float)((double)model->scale / sqrt((double)model->d) * 1.44269504088896340736 / (double)temp);
        a.codes = codes; a.codes_out = codes; a.tokens_out = tokens_out + t; a.tok_stride = T;
        a.finished_in = eos_id >= 0 ? fin : nullptr; a.eos_id = eos_id;
        a.finished_out = eos_id >= 0 ? fin : nullptr; a.prev = prev; a.prev_out = prev;
        st = launch_fused_sample(ctx, a);
        if (st != AS_OK) return st;
    }
    if (codes_out)
        AS_HIP_TRY(ctx, hipMemcpyAsync(codes_out, codes, (size_t)R * sizeof(float), hipMemcpyDeviceToDevice,
                                       ctx->stream));
    return AS_OK;
}

as_status as_estimate_mean(as_ctx *ctx, const int32_t *tokens, int32_t B, int32_t N, int32_t T, const float *score,
                           int32_t eos_id, double *est_out)
{
    if (!ctx) return fail(nullptr, AS_ERR_INVALID_ARG, "ctx is NULL");
    if (B < 0 || N < 1 || T < 0) return fail(ctx, AS_ERR_INVALID_ARG, "B, T must be >= 0 and N >= 1");
    if (B == 0) return AS_OK;
    if (!score || !est_out || (T > 0 && !tokens))
        return fail(ctx, AS_ERR_INVALID_ARG, "tokens, score and est_out must not be NULL");
    if (eos_id >= ctx->V) return fail(ctx, AS_ERR_INVALID_ARG, "eos_id outside the vocabulary");
    return launch_estimate(ctx, tokens, B, N, T, score, eos_id, est_out);
}

as_status as_interval_step(as_ctx *ctx, const void *logits, int64_t rows, int64_t ld, const int32_t *tokens,
                           float temp, int32_t top_k, float top_p, double *lo, double *width,
                           const uint8_t *finished_in, int32_t eos_id, uint8_t *finished_out,
                           const int32_t *row_ids, int64_t logits_rows)
{
    if (!ctx) return fail(nullptr, AS_ERR_INVALID_ARG, "ctx is NULL");
    if (rows < 0 || rows > ctx->max_rows) return fail(ctx, AS_ERR_INVALID_ARG, "rows outside [0, max_rows]");
    if (rows == 0) return AS_OK;
    if (!logits || !tokens || !lo || !width)
        return fail(ctx, AS_ERR_INVALID_ARG, "logits, tokens, lo and width must not be NULL");
    if (ld < ctx->V) return fail(ctx, AS_ERR_INVALID_ARG, "ld is smaller than the vocabulary");
    if (!(temp > 0.f) || !isfinite(temp)) return fail(ctx, AS_ERR_INVALID_ARG, "temp must be finite and > 0");
    if (row_ids && logits_rows < 1) return fail(ctx, AS_ERR_INVALID_ARG, "row_ids given but logits_rows < 1");
    if (finished_in && eos_id < 0)
        return fail(ctx, AS_ERR_INVALID_ARG, "finished_in given without an eos_id");
    if (eos_id >= ctx->V) return fail(ctx, AS_ERR_INVALID_ARG, "eos_id outside the vocabulary");
    if (isnan(top_p)) return fail(ctx, AS_ERR_INVALID_ARG, "top_p is NaN");
    if (as_status st = row_ids_in_range(ctx, row_ids, rows, logits_rows); st != AS_OK) return st;

    const float *thr = nullptr;
    if (truncation_on(ctx->V, top_k, top_p)) {
        as_status st = launch_threshold(ctx, logits, rows, ld, finished_in, row_ids, temp, top_k, top_p, ctx->thr);
        if (st != AS_OK) return st;
        thr = ctx->thr;
    }
    IntervalArgs a{};
    a.logits = logits; a.rows = rows; a.ld = ld; a.V = ctx->V; a.dtype = ctx->dtype;
    a.tokens = tokens; a.tok_stride = 1; a.k = 1.44269504088896340736f / temp; a.thr = thr;
    a.finished_in = finished_in; a.eos_id = eos_id; a.finished_out = finished_out;
    a.lo = lo; a.width = width; a.row_ids = row_ids; a.prev_out = nullptr;
    return launch_interval(ctx, a);
}

as_status as_encode(as_ctx *ctx, const as_model *model, const int32_t *prompts, int32_t B, int32_t N, int32_t T,
                    const int32_t *tokens, float temp, int32_t top_k, float top_p, int32_t eos_id,
                    double *lo_out, double *width_out)
{
    if (!ctx) return fail(nullptr, AS_ERR_INVALID_ARG, "ctx is NULL");
    if (!model) return fail(ctx, AS_ERR_INVALID_ARG, "model is NULL");
    if (model->V != ctx->V) return fail(ctx, AS_ERR_INVALID_ARG, "model and context disagree on V");
    if (B < 0 || N < 1 || T < 0) return fail(ctx, AS_ERR_INVALID_ARG, "B, T must be >= 0 and N >= 1");
    const int64_t R = (int64_t)B * N;
    if (R > ctx->max_rows) return fail(ctx, AS_ERR_INVALID_ARG, "B*N exceeds max_rows");
    if (R == 0) return AS_OK;
    if (!prompts || !lo_out || !width_out)
        return fail(ctx, AS_ERR_INVALID_ARG, "prompts, lo_out and width_out must not be NULL");
    if (T > 0 && !tokens) return fail(ctx, AS_ERR_INVALID_ARG, "tokens must not be NULL");
    if (!(temp > 0.f) || !isfinite(temp)) return fail(ctx, AS_ERR_INVALID_ARG, "temp must be finite and > 0");
    if (eos_id >= ctx->V) return fail(ctx, AS_ERR_INVALID_ARG, "eos_id outside the vocabulary");
    if (isnan(top_p)) return fail(ctx, AS_ERR_INVALID_ARG, "top_p is NaN");

    const size_t esz = ctx->dtype == AS_BF16 ? 2 : 4;
    const int64_t ldw = ((int64_t)ctx->V + 7) / 8 * 8;        // rows start 16-byte aligned
    as_status st = grow(ctx, ctx->logits, (size_t)R * ldw * esz);
    if (st != AS_OK) return st;
    st = grow(ctx, ctx->state, (size_t)R * 9);
    if (st != AS_OK) return st;
    float *codes = static_cast<float *>(ctx->state.ptr);      // (unused here; same layout as as_decode)
    int32_t *prev = reinterpret_cast<int32_t *>(codes + R);
    uint8_t *fin = reinterpret_cast<uint8_t *>(prev + R);

    st = launch_interval_init(ctx, B, N, prompts, lo_out, width_out, prev, fin);
    if (st != AS_OK) return st;
    const bool trunc = truncation_on(ctx->V, top_k, top_p);
    for (int32_t t = 0; t < T; ++t) {
        st = launch_bigram_logits(ctx, model, prev, R, ctx->logits.ptr, ldw);
        if (st != AS_OK) return st;
        if (trunc) {
            st = launch_threshold(ctx, ctx->logits.ptr, R, ldw, eos_id >= 0 ? fin : nullptr, nullptr, temp,
                                  top_k, top_p, ctx->thr);
            if (st != AS_OK) return st;
        }
        IntervalArgs a{};
        a.logits = ctx->logits.ptr; a.rows = R; a.ld = ldw; a.V = ctx->V; a.dtype = ctx->dtype;
        a.tokens = tokens + t; a.tok_stride = T; a.k = 1.44269504088896340736f / temp;
        a.thr = trunc ? ctx->thr : nullptr;
        a.finished_in = eos_id >= 0 ? fin : nullptr; a.eos_id = eos_id;
        a.finished_out = eos_id >= 0 ? fin : nullptr;
        a.lo = lo_out; a.width = width_out; a.row_ids = nullptr; a.prev_out = prev;
        st = launch_interval(ctx, a);
        if (st != AS_OK) return st;
    }
    return AS_OK;
}

}  // extern "C"
