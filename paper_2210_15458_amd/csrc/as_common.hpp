// Shared declarations of the HIP library: context, model, error plumbing and
// the wave-level primitives (DPP scans/reductions for 64-wide wavefronts).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "../../include/arith_sampling.h"

namespace as {

constexpr int kWave = 64;

// ---------------------------------------------------------------- host state

struct DeviceBuf {
    void *ptr = nullptr;
    size_t bytes = 0;
};

// Optional per-kernel timing: when switched on, every launch of a profiled
// kernel carries its own start/stop events (taken from the dispatch itself,
// not from separate stream markers), read back by as_ctx_profile_read.
enum KernelId { kKernelStep = 0, kKernelLogits = 1, kKernelThreshold = 2, kKernelInterval = 3, kKernelCount = 4 };
constexpr size_t kProfileCapacity = 16384;      // timed launches per kernel between reads

struct ProfileSlot {
    hipEvent_t start = nullptr, stop = nullptr;
};
struct Profile {
    bool on = false;
    std::vector<ProfileSlot> slots[kKernelCount];   // created on demand, reused after a read
    size_t used[kKernelCount] = {};
    size_t dropped[kKernelCount] = {};
};

}  // namespace as

struct as_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    int64_t max_rows = 0;
    int32_t V = 0;
    as_dtype dtype = AS_BF16;
    // fixed workspace (allocated at creation): per-row truncation thresholds
    float *thr = nullptr;          // [max_rows]
    int32_t *rid = nullptr;        // [max_rows] the caller's row_ids brought into range
    // decode workspace (grown on demand by as_decode)
    as::DeviceBuf logits;          // [rows, ld]
    as::DeviceBuf state;           // codes f32[rows] | prev i32[rows] | finished u8[rows]
    as::Profile prof;
    int step_shape = 0;            // work-group shape of the sampling kernel (tuning knob, 0 = default)
    int gemm_shape = 0;            // logits kernel choice (tuning knob: 0 = persistent where it applies, 1 = tile kernel)
    int thr_path = 0;              // keep-threshold kernel choice (tuning knob: 0 = resident where it applies, 1 = radix)
    int gemm_gm = 0;               // logits kernel, many row tiles: workers of an XCD along the rows (tuning knob: 0 = default)
    int num_cus = 0;               // compute units of the device (the persistent logits kernel runs one block on each)
    std::string err;
};

struct as_model {
    int device = 0;
    int32_t V = 0;
    int32_t d = 0;
    float scale = 0.f;
    as_dtype wdtype = AS_BF16;
    const void *E = nullptr;       // borrowed [V, d]
    void *Ut = nullptr;            // owned    [V, d]  (U transposed: K contiguous)
};

namespace as {

as_status fail(as_ctx *ctx, as_status code, const std::string &msg);
as_status hip_fail(as_ctx *ctx, hipError_t e, const char *what);

#define AS_HIP_TRY(ctx, expr)                                        \
    do {                                                             \
        hipError_t _e = (expr);                                      \
        if (_e != hipSuccess) return ::as::hip_fail((ctx), _e, #expr); \
    } while (0)

// Launch on the context's stream; with profiling on, attach dispatch events.
bool profile_acquire(as_ctx *ctx, int kid, hipEvent_t *start, hipEvent_t *stop);

template <class K, class... A>
inline void launch(as_ctx *ctx, int kid, K kernel, dim3 grid, dim3 block, size_t lds, A... args)
{
    hipEvent_t s = nullptr, e = nullptr;
    if (ctx->prof.on && profile_acquire(ctx, kid, &s, &e))
        hipExtLaunchKernelGGL(kernel, grid, block, (unsigned)lds, ctx->stream, s, e, 0, args...);
    else
        hipLaunchKernelGGL(kernel, grid, block, (unsigned)lds, ctx->stream, args...);
}

// -------------------------------------------------------------- launch entry
// (implemented in as_step.hip / as_model.hip; called only from as_api.hip)

// How the one-tile kernels load a row.  Logits that the logits kernel has just written are partly still in the
// caches when the whole tensor fits them: ordinary loads then (0.5 us of 13.4 per launch at 1024 x 32128 bf16
// inside a decode).  A tensor beyond the caches is streamed with the non-temporal hint (65536 rows: 651 us
// against 718 with ordinary loads).
inline bool stream_rows(int64_t rows, int64_t ld, size_t esz)
{
    return (double)rows * (double)ld * (double)esz > 128.0 * 1024.0 * 1024.0;
}

struct StepArgs {
    const void *logits;
    int64_t rows;
    int64_t ld;
    int32_t V;
    as_dtype dtype;
    const float *codes;
    float temp;
    float k;                     // log2(e)/temp, computed once on the host
    const float *thr;            // per-row keep threshold on raw logits, or null
    int32_t *tokens_out;
    int64_t tok_stride;          // tokens_out[r * tok_stride]
    float *codes_out;
    const uint8_t *finished_in;
    int32_t eos_id;
    uint8_t *finished_out;
    float *prob_out;
    float *flo_out;
    const int32_t *row_ids;
    int32_t *prev_out;           // decode state: next step's conditioning token, or null
};

struct IntervalArgs {
    const void *logits;
    int64_t rows;
    int64_t ld;
    int32_t V;
    as_dtype dtype;
    const int32_t *tokens;
    int64_t tok_stride;          // token of row r at tokens[r * tok_stride]
    float k;                     // log2(e)/temp
    const float *thr;            // per-row keep threshold on raw logits, or null
    const uint8_t *finished_in;
    int32_t eos_id;
    uint8_t *finished_out;
    double *lo;                  // [rows] in/out
    double *width;               // [rows] in/out
    const int32_t *row_ids;
    int32_t *prev_out;           // encode state: next step's conditioning token, or null
};

struct FusedArgs {
    const float2 *part;          // [rows, ldp]: (sum, reference) per group of 32 logits
    int64_t ldp;                 // multiple of 16
    int32_t ngroups;             // ceil(V / 32)
    int64_t rows;
    int32_t V;
    int32_t d;
    const uint16_t *E;           // [V, d] bf16
    const uint16_t *Ut;          // [V, d] bf16
    float alpha;                 // scale/sqrt(d) * log2(e)/temp
    const float *codes;
    float *codes_out;
    int32_t *tokens_out;
    int64_t tok_stride;
    const uint8_t *finished_in;
    int32_t eos_id;
    uint8_t *finished_out;
    const int32_t *prev;         // conditioning token of each row (may alias prev_out)
    int32_t *prev_out;
};

as_status launch_step(as_ctx *ctx, const StepArgs &a);
as_status launch_fused_sample(as_ctx *ctx, const FusedArgs &a);
as_status launch_bigram_partials(as_ctx *ctx, const as_model *m, const int32_t *prev, int64_t rows, float temp,
                                 float2 *part, int64_t ldp);
bool fused_path_applies(const as_ctx *ctx, const as_model *m);
as_status launch_interval(as_ctx *ctx, const IntervalArgs &a);
as_status launch_interval_init(as_ctx *ctx, int32_t B, int32_t N, const int32_t *prompts, double *lo,
                               double *width, int32_t *prev, uint8_t *finished);
bool launch_topk_step(as_ctx *ctx, const StepArgs &a, int32_t top_k, float top_p, as_status *st);
as_status launch_threshold(as_ctx *ctx, const void *logits, int64_t rows, int64_t ld,
                           const uint8_t *finished_in, const int32_t *row_ids,
                           float temp, int32_t top_k, float top_p, float *thr_out);
as_status launch_lattice(as_ctx *ctx, const float *u, int32_t B, int32_t N, float *codes_out,
                         const int32_t *prompts, int32_t *prev_out, uint8_t *finished_out);
as_status launch_estimate(as_ctx *ctx, const int32_t *tokens, int32_t B, int32_t N, int32_t T, const float *score,
                          int32_t eos_id, double *est_out);
as_status launch_transpose(const void *U, void *Ut, int32_t d, int32_t V, as_dtype wdtype);
as_status launch_bigram_logits(as_ctx *ctx, const as_model *m, const int32_t *prev,
                               int64_t rows, void *logits_out, int64_t ld);

// ------------------------------------------------------------ wave primitives
// Data-parallel-primitive (DPP) cross-lane moves.  bound_ctrl is off, so a lane
// whose source is outside its row (or that is masked out) receives `old`.

constexpr int kRowShr1 = 0x111, kRowShr2 = 0x112, kRowShr4 = 0x114, kRowShr8 = 0x118;
constexpr int kRowBcast15 = 0x142, kRowBcast31 = 0x143;

// A conditioning token as a row index of the embedding: tokens the library emits are in [0, V); one handed in
// from outside that is not (a prompt) is clamped rather than followed out of the table.
__device__ __forceinline__ int32_t clamp_token(int32_t t, int32_t V) { return t < 0 ? 0 : (t > V - 1 ? V - 1 : t); }

template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ int dpp_i32(int old, int src)
{
    return __builtin_amdgcn_update_dpp(old, src, CTRL, ROW_MASK, 0xf, false);
}
template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ float dpp_f32(float old, float src)
{
    return __builtin_bit_cast(
        float, dpp_i32<CTRL, ROW_MASK>(__builtin_bit_cast(int, old), __builtin_bit_cast(int, src)));
}
template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ double dpp_f64(double old, double src)
{
    long long o = __builtin_bit_cast(long long, old), s = __builtin_bit_cast(long long, src);
    int lo = dpp_i32<CTRL, ROW_MASK>((int)o, (int)s);
    int hi = dpp_i32<CTRL, ROW_MASK>((int)(o >> 32), (int)(s >> 32));
    long long r = ((long long)hi << 32) | (unsigned int)lo;
    return __builtin_bit_cast(double, r);
}

// Inclusive prefix sum over the 64 lanes of a wave, lane order.
__device__ __forceinline__ float wave_scan_add(float x)
{
    x += dpp_f32<kRowShr1>(0.f, x);
    x += dpp_f32<kRowShr2>(0.f, x);
    x += dpp_f32<kRowShr4>(0.f, x);
    x += dpp_f32<kRowShr8>(0.f, x);
    x += dpp_f32<kRowBcast15, 0xa>(0.f, x);
    x += dpp_f32<kRowBcast31, 0xc>(0.f, x);
    return x;
}
__device__ __forceinline__ double wave_scan_add(double x)
{
    x += dpp_f64<kRowShr1>(0.0, x);
    x += dpp_f64<kRowShr2>(0.0, x);
    x += dpp_f64<kRowShr4>(0.0, x);
    x += dpp_f64<kRowShr8>(0.0, x);
    x += dpp_f64<kRowBcast15, 0xa>(0.0, x);
    x += dpp_f64<kRowBcast31, 0xc>(0.0, x);
    return x;
}

__device__ __forceinline__ float read_lane(float x, int lane)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), lane));
}
__device__ __forceinline__ double read_lane(double x, int lane)
{
    long long v = __builtin_bit_cast(long long, x);
    int lo = __builtin_amdgcn_readlane((int)v, lane);
    int hi = __builtin_amdgcn_readlane((int)(v >> 32), lane);
    long long r = ((long long)hi << 32) | (unsigned int)lo;
    return __builtin_bit_cast(double, r);
}

// Sum / max over the wave, result in every lane (wave-uniform).
// Written as six fused DPP instructions: destination and both sources are the
// same register, so a lane without a valid source (or masked off by row_mask)
// simply keeps its value, which is the identity for both operations.  A VALU
// write needs two wait states before a DPP read of the same register.
__device__ __forceinline__ float wave_sum(float x)
{
    asm volatile(
        "s_nop 1\n\t"
        "v_add_f32_dpp %0, %0, %0 row_shr:1 row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_add_f32_dpp %0, %0, %0 row_shr:2 row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_add_f32_dpp %0, %0, %0 row_shr:4 row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_add_f32_dpp %0, %0, %0 row_shr:8 row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_add_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_add_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
        "s_nop 0"
        : "+v"(x));
    return read_lane(x, 63);
}
__device__ __forceinline__ double wave_sum(double x) { return read_lane(wave_scan_add(x), 63); }

__device__ __forceinline__ float wave_max(float x)
{
    asm volatile(
        "s_nop 1\n\t"
        "v_max_f32_dpp %0, %0, %0 row_shr:1 row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_max_f32_dpp %0, %0, %0 row_shr:2 row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_max_f32_dpp %0, %0, %0 row_shr:4 row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_max_f32_dpp %0, %0, %0 row_shr:8 row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_max_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_max_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
        "s_nop 0"
        : "+v"(x));
    return read_lane(x, 63);
}

__device__ __forceinline__ int lane_id() { return (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)); }

}  // namespace as
