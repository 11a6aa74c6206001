// What a sampling step writes per row, and the plain three-pass form of the step (Sec. 4.1, Algorithm 1 loop
// body: vocabulary-order cumulative sums, first bucket above the code, rescale), shared by the kernels that
// finish a row.
#ifndef AS_ROW_HPP
#define AS_ROW_HPP

#include "as_common.hpp"

namespace as {

constexpr float kRefFloor = -100000.f;  // reference when only -inf has been seen

// exp2 straight on the hardware instruction (no denormal fix-up: results below
// 2^-126 may flush to zero, which is far below anything that can matter here)
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float widen_stored(float h) { return h; }
__device__ __forceinline__ float widen_stored(uint16_t h) { return __builtin_bit_cast(float, (uint32_t)h << 16); }

struct RowOut {
    int32_t token;
    float c_next, prob, f_lo;
};

__device__ __forceinline__ void write_row(const StepArgs &a, int64_t r, const RowOut &o)
{
    a.tokens_out[r * a.tok_stride] = o.token;
    a.codes_out[r] = o.c_next;
    if (a.finished_out) a.finished_out[r] = (a.eos_id >= 0 && o.token == a.eos_id) ? 1 : 0;
    if (a.prob_out) a.prob_out[r] = o.prob;
    if (a.flo_out) a.flo_out[r] = o.f_lo;
    if (a.prev_out) a.prev_out[r] = o.token;
}

// finished sequence: padding after EOS (Sec. 3.3); the code stops moving
__device__ __forceinline__ void write_finished(const StepArgs &a, int64_t r)
{
    a.tokens_out[r * a.tok_stride] = a.eos_id;
    a.codes_out[r] = a.codes[r];
    if (a.finished_out) a.finished_out[r] = 1;
    if (a.prob_out) a.prob_out[r] = 1.f;
    if (a.flo_out) a.flo_out[r] = 0.f;
    if (a.prev_out) a.prev_out[r] = a.eos_id;
}

// c' = (c*S - before)/e_v: the difference is taken in fp64, the quotient is an fp32 result anyway
__device__ __forceinline__ float rescale_code(double tau, double before, double ev)
{
    float cnf = (float)(tau - before) / (float)ev;
    cnf = fminf(cnf, 0x1.fffffep-1f);        // 1 - 2^-24
    if (!(cnf >= 0.f)) cnf = 0.f;
    return cnf;
}

struct GenericScratch {
    float red[4];
    double tot[256];
    int hit;
    double run;
};

// One row by a block of 256 threads, any alignment, any V: three plain passes (max, sums, search), each
// thread owning one contiguous run of elements so that thread order is vocabulary order.  Every thread of
// the block must call it; keeps x >= thr.
template <class T>
__device__ __forceinline__ void generic_step_row(const StepArgs &a, int64_t r, float thr, GenericScratch &sh)
{
    const int tid = threadIdx.x;
    const int64_t src = a.row_ids ? (int64_t)a.row_ids[r] : r;
    const T *row = reinterpret_cast<const T *>(a.logits) + src * a.ld;
    const int32_t V = a.V;
    const float k = a.k;
    const int32_t len = (V + 255) / 256;
    const int32_t lo = tid * len, hi = (lo + len < V) ? lo + len : V;

    float m = -__builtin_inff();
    for (int32_t v = lo; v < hi; ++v) {
        const float x = widen_stored(row[v]);
        if (x >= thr) m = fmaxf(m, x);
    }
    m = wave_max(m);
    if ((tid & 63) == 0) sh.red[tid >> 6] = m;
    __syncthreads();
    m = fmaxf(fmaxf(sh.red[0], sh.red[1]), fmaxf(sh.red[2], sh.red[3]));
    const float ref = fmaxf(ceilf(m * k), kRefFloor);

    double tot = 0.0;
    for (int32_t v = lo; v < hi; ++v) {
        const float x = widen_stored(row[v]);
        if (x >= thr) tot += (double)fast_exp2(fmaf(x, k, -ref));
    }
    sh.tot[tid] = tot;
    __syncthreads();
    if (tid == 0) {
        double S = 0.0;
        for (int i = 0; i < 256; ++i) S += sh.tot[i];
        const double tau = (double)a.codes[r] * S;
        double run = 0.0, run_last = 0.0;
        int hit = -1, last_nz = 0;
        for (int i = 0; i < 256; ++i) {
            if (sh.tot[i] > 0.0) { last_nz = i; run_last = run; }
            if (run + sh.tot[i] > tau) { hit = i; break; }
            run += sh.tot[i];
        }
        if (hit < 0) { hit = last_nz; run = run_last; }
        sh.hit = hit;
        sh.run = run;
        sh.tot[0] = S;                     // thread 0's own total is not needed any more
    }
    __syncthreads();
    if (tid != sh.hit) return;
    const double S = sh.tot[0];
    const double tau = (double)a.codes[r] * S;
    double acc = sh.run, before = sh.run, before_last = sh.run, ev = 0.0, ev_last = 0.0;
    int32_t tok = -1, tok_last = lo < V ? lo : V - 1;
    for (int32_t v = lo; v < hi; ++v) {
        const float x = widen_stored(row[v]);
        const double e = (x >= thr) ? (double)fast_exp2(fmaf(x, k, -ref)) : 0.0;
        if (e > 0.0) { tok_last = v; before_last = acc; ev_last = e; }
        if (tok < 0 && acc + e > tau) { tok = v; before = acc; ev = e; }
        acc += e;
    }
    if (tok < 0) { tok = tok_last; before = before_last; ev = ev_last; }
    RowOut o;
    o.token = tok;
    o.c_next = rescale_code(tau, before, ev);
    o.prob = (float)(ev / S);
    o.f_lo = (float)(before / S);
    write_row(a, r, o);
}

}  // namespace as
#endif
