// Pieces shared by the kernels that keep a whole row in the registers of one workgroup ("one tile": four waves,
// sixteen 1-KiB chunks each, a 16-byte vector per lane and chunk): unpacking, the lane and chunk sums of the
// softmax weights against an integer reference per wave, and the search for the code's bucket over those sums
// (Sec. 4.1, one loop body of Algorithm 1).
#ifndef AS_TILE_HPP
#define AS_TILE_HPP
#include <type_traits>
#include <utility>

#include "as_common.hpp"
#include "as_row.hpp"

namespace as {
namespace {

constexpr float kMinShift = -300.f;     // 2^-300 is 0 in fp32: clamp before float->int

template <int DT> struct Elem;
template <> struct Elem<AS_F32> {
    using T = float;
    static constexpr int kPerVec = 4;
};
template <> struct Elem<AS_BF16> {
    using T = uint16_t;
    static constexpr int kPerVec = 8;
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bits_f32(uint32_t b) { return __builtin_bit_cast(float, b); }

template <int DT>
__device__ __forceinline__ void unpack(const u32x4 &v, float *x)
{
    if constexpr (DT == AS_BF16) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[2 * i] = bits_f32(v[i] << 16);
            x[2 * i + 1] = bits_f32(v[i] & 0xffff0000u);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) x[i] = bits_f32(v[i]);
    }
}

template <int DT> __device__ __forceinline__ float widen(typename Elem<DT>::T h)
{
    if constexpr (DT == AS_BF16) return bits_f32((uint32_t)h << 16);
    else return h;
}

// Three-operand maximum as one instruction.  (fmaxf on values that come from
// bit casts makes the compiler quiet possible signalling NaNs first, one extra
// instruction per operand; NaN logits are outside the contract anyway.)
__device__ __forceinline__ float max3(float a, float b, float c)
{
    float d;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    return d;
}

template <int EPV> __device__ __forceinline__ float vec_max(const float *x)
{
    if constexpr (EPV == 8) return max3(max3(max3(x[0], x[1], x[2]), x[3], x[4]), max3(x[5], x[6], x[7]), x[5]);
    else return max3(max3(x[0], x[1], x[2]), x[3], x[3]);
}
template <int EPV> __device__ __forceinline__ float vec_sum(const float *e)
{
    if constexpr (EPV == 8) return ((e[0] + e[1]) + (e[2] + e[3])) + ((e[4] + e[5]) + (e[6] + e[7]));
    else return (e[0] + e[1]) + (e[2] + e[3]);
}

__device__ __forceinline__ int shift_of(float r, float R) { return (int)fmaxf(r - R, kMinShift); }

// calls f(integral_constant<i>) for i == idx (wave-uniform) through a tree of scalar branches
template <int LO, int HI, class F>
__device__ __forceinline__ void with_uniform_index(int idx, F &&f)
{
    if constexpr (HI - LO == 1) {
        f(std::integral_constant<int, LO>{});
    } else {
        constexpr int MID = (LO + HI) / 2;
        if (idx < MID) with_uniform_index<LO, MID>(idx, f);
        else with_uniform_index<MID, HI>(idx, f);
    }
}

// Four independent wave sums at once: the DPP steps of the four interleave, which hides their latency and makes
// the wait states between dependent DPP instructions free.  The totals are left in lane 63.
__device__ __forceinline__ void wave_sum4_in_lane63(float &a, float &b, float &c, float &d)
{
#define AS_DPP4(ctrl)                                                 \
    "v_add_f32_dpp %0, %0, %0 " ctrl " bank_mask:0xf\n\t"           \
    "v_add_f32_dpp %1, %1, %1 " ctrl " bank_mask:0xf\n\t"           \
    "v_add_f32_dpp %2, %2, %2 " ctrl " bank_mask:0xf\n\t"           \
    "v_add_f32_dpp %3, %3, %3 " ctrl " bank_mask:0xf\n\t"
    asm volatile("s_nop 1\n\t"
                 AS_DPP4("row_shr:1 row_mask:0xf")
                 AS_DPP4("row_shr:2 row_mask:0xf")
                 AS_DPP4("row_shr:4 row_mask:0xf")
                 AS_DPP4("row_shr:8 row_mask:0xf")
                 AS_DPP4("row_bcast:15 row_mask:0xa")
                 AS_DPP4("row_bcast:31 row_mask:0xc")
                 "s_nop 0"
                 : "+v"(a), "+v"(b), "+v"(c), "+v"(d));
#undef AS_DPP4
}


// ---------------------------------------------------------------------------
// a row of whole, aligned vectors in one tile
constexpr int kTileWaves = 4, kTileIters = 16, kTileGroup = 4;
// The kernels that take a wave's reference from its share's first chunk lose a row to their slow path when a
// logit lies more than 127/k above that chunk's largest (weights beyond fp32).  The host keeps them for
// k = log2(e)/temp up to this: a logit 30 above the first chunk's largest still fits.  Lower temperatures take
// the kernels that follow the running maximum.
constexpr float kTileMaxScale = 4.f;
typedef float f32x4 __attribute__((ext_vector_type(4)));

struct TileSums {
    __attribute__((aligned(16))) float chunk_sum[kTileWaves * kTileIters];   // sum of every chunk of the row, vocabulary order
    __attribute__((aligned(16))) float share_ref[kTileWaves];                // the integer reference its share's sums are relative to
};

// the lane's sum over one chunk, relative to the reference -nr
template <int DT, bool HAS_THR>
__device__ __forceinline__ float tile_lane_sum(const u32x4 &v, float k, float nr, float thr)
{
    constexpr int EPV = Elem<DT>::kPerVec;
    float x[EPV], e[EPV];
    unpack<DT>(v, x);
#pragma unroll
    for (int i = 0; i < EPV; ++i) {
        e[i] = fast_exp2(fmaf(x[i], k, nr));
        if constexpr (HAS_THR) e[i] = (x[i] >= thr) ? e[i] : 0.f;
    }
    return vec_sum<EPV>(e);
}

// the wave's reference: from the first chunk's largest kept logit and, with a threshold, the threshold itself
// (every kept logit is at or above it).  mych: chunks of the share in which this lane is inside the row.
template <int DT, bool HAS_THR, bool RAGGED>
__device__ __forceinline__ float tile_reference(const u32x4 &first, float k, float thr, int32_t mych)
{
    constexpr int EPV = Elem<DT>::kPerVec;
    float x[EPV];
    unpack<DT>(first, x);
    if constexpr (HAS_THR) {
#pragma unroll
        for (int i = 0; i < EPV; ++i) x[i] = (x[i] >= thr) ? x[i] : -__builtin_inff();
    }
    float m = vec_max<EPV>(x);
    if constexpr (RAGGED) m = mych > 0 ? m : -__builtin_inff();
    m = wave_max(m);
    if constexpr (HAS_THR) m = fmaxf(m, thr);
    return fmaxf(ceilf(m * k), kRefFloor);
}

// the sums of the share's sixteen chunks over the wave, relative to rw, to my_sums (LDS, four at a time, by the
// lane that ends up with them); chunks are taken as they land
template <int DT, bool HAS_THR, bool RAGGED>
__device__ __forceinline__ void tile_chunk_sums(const u32x4 (&raw)[kTileIters], float k, float rw, float thr,
                                                int32_t mych, int lane, f32x4 *my_sums)
{
    constexpr int G = kTileGroup;
    const float nr = -rw;
#pragma unroll
    for (int g = 0; g < kTileIters / G; ++g) {
        float t[G];
#pragma unroll
        for (int jj = 0; jj < G; ++jj) {
            const int j = g * G + jj;
            t[jj] = tile_lane_sum<DT, HAS_THR>(raw[j], k, nr, thr);
            if constexpr (RAGGED) t[jj] = j < mych ? t[jj] : 0.f;
        }
        wave_sum4_in_lane63(t[0], t[1], t[2], t[3]);
        if (lane == 63) my_sums[g] = f32x4{t[0], t[1], t[2], t[3]};
    }
}

// After the barrier that follows the chunk sums: every wave scans the row's 64 chunk sums (fp64) for the total,
// the target c*S and the chunk that holds it; the wave that owns that chunk finds the lane, that lane the
// element, and writes the row's results.  Every thread of the block calls it.  rw is the calling wave's own
// reference (also in ts.share_ref), v0 the first vector of its share.
template <int DT, bool HAS_THR>
__device__ __forceinline__ void tile_select(const StepArgs &a, int64_t r, float code, float thr,
                                            const u32x4 (&raw)[kTileIters], float rw, int32_t mych, bool ragged,
                                            int32_t v0, int lane, int wave, const TileSums &ts, GenericScratch &gen)
{
    using T = typename Elem<DT>::T;
    constexpr int EPV = Elem<DT>::kPerVec;
    constexpr int NW = kTileWaves, ITERS = kTileIters;
    const float k = a.k;
    float R = ts.share_ref[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) R = fmaxf(R, ts.share_ref[w]);
    const float my_ref = ts.share_ref[lane / ITERS];
    const double cv = (double)ldexpf(ts.chunk_sum[lane], shift_of(my_ref, R));
    const double cincl = wave_scan_add(cv);
    const double S = read_lane(cincl, 63);
    if (!(S < (double)__builtin_inff())) {
        // weights beyond fp32 against a first-chunk reference, or NaN in the data: the plain routine
        generic_step_row<T>(a, r, thr, gen);
        return;
    }
    const double tau = (double)code * S;
    const unsigned long long chit = __ballot(cincl > tau);
    const unsigned long long cnz = __ballot(cv > 0.0);
    // the first chunk whose running sum passes c*S; past the end by rounding: the last chunk that holds weight
    const int ch = chit ? (__ffsll((long long)chit) - 1) : (cnz ? (63 - __clzll((long long)cnz)) : 0);
    if (wave != ch / ITERS) return;
    const double run = read_lane(cincl - cv, ch);

    // ---------------- owning wave: lane, then element.  Everything it holds is relative to rw.
    const int shf = shift_of(rw, R);
    const int cj = ch % ITERS;
    u32x4 hv;
    with_uniform_index<0, ITERS>(cj, [&](auto c_c) __attribute__((always_inline)) {
        uint32_t w0 = raw[decltype(c_c)::value][0], w1 = raw[decltype(c_c)::value][1],
                 w2 = raw[decltype(c_c)::value][2], w3 = raw[decltype(c_c)::value][3];
        // opaque to the optimiser: keeps this a tree of branches over registers instead of an indexed read
        // that would force the array into memory
        asm volatile("" : "+v"(w0), "+v"(w1), "+v"(w2), "+v"(w3));
        hv = u32x4{w0, w1, w2, w3};
    });
    // the lane sums of that chunk once more (sixteen sums per lane kept for this would cost the registers
    // that let a row have eight waves)
    float cl = tile_lane_sum<DT, HAS_THR>(hv, k, -rw, thr);
    if (ragged) cl = cj < mych ? cl : 0.f;
    const double lv = (double)ldexpf(cl, shf);
    const double incl2 = wave_scan_add(lv) + run;
    const unsigned long long hit2 = __ballot(incl2 > tau);
    const unsigned long long nz2 = __ballot(lv > 0.0);
    const int l2 = hit2 ? (__ffsll((long long)hit2) - 1) : (nz2 ? (63 - __clzll((long long)nz2)) : 0);
    if (lane != l2) return;

    float x[EPV];
    unpack<DT>(hv, x);
    double ed[EPV];
#pragma unroll
    for (int i = 0; i < EPV; ++i) {
        float e = fast_exp2(fmaf(x[i], k, -rw));
        if constexpr (HAS_THR) e = (x[i] >= thr) ? e : 0.f;
        ed[i] = (double)ldexpf(e, shf);
    }
    double acc = incl2 - lv;
    int ih = -1, ilast = 0;
    double before = acc, before_last = acc, ev = 0.0, ev_last = 0.0;
#pragma unroll
    for (int i = 0; i < EPV; ++i) {
        if (ed[i] > 0.0) { ilast = i; before_last = acc; ev_last = ed[i]; }
        if (ih < 0 && acc + ed[i] > tau) { ih = i; before = acc; ev = ed[i]; }
        acc += ed[i];
    }
    if (ih < 0) { ih = ilast; before = before_last; ev = ev_last; }

    int64_t tok64 = ((int64_t)v0 + (int64_t)cj * 64 + lane) * EPV + ih;
    if (tok64 > a.V - 1) tok64 = a.V - 1;
    RowOut o;
    o.token = (int32_t)tok64;
    o.c_next = rescale_code(tau, before, ev);
    o.prob = 0.f;
    o.f_lo = 0.f;
    if (a.prob_out || a.flo_out) {          // records for tests and callers that ask: fp32 quotients of fp64 sums
        const float Sf = (float)S;
        o.prob = (float)ev / Sf;
        o.f_lo = (float)before / Sf;
    }
    write_row(a, r, o);
}

}  // namespace
}  // namespace as
#endif
