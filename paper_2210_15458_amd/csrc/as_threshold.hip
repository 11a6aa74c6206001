// Keep thresholds for the logit modifiers of Sec. 2 (top-k, nucleus): one value
// per row such that the kept set is { v : logit_v >= thr }.  Everything outside
// gets probability zero before the vocabulary-order cumulative sums are formed
// (Sec. 5, top-k paragraph).
//
// Both selections are radix selects over an order-preserving integer key of the
// stored logit, most significant digit first, with an LDS histogram per digit:
//   top-k    histogram of counts; descend into the digit that holds the k-th
//            largest key.  Ties at the k-th value all stay (threshold rule).
//   nucleus  histogram of probability mass; descend into the first digit (from
//            the top) at which the running mass reaches top_p of the total.
//            The group of equal logits that closes the nucleus stays whole.
// Mass is accumulated in fixed point (integer atomics) so that the result does
// not depend on the order in which lanes reach the histogram.
#include "as_common.hpp"

namespace as {
namespace {

constexpr int kThreads = 256;
constexpr int kMaxBins = 4096;

template <int DT> struct Key;
template <> struct Key<AS_BF16> {
    using T = uint16_t;
    static constexpr int kBits = 16;
    static constexpr int kPasses = 2;
    static __device__ __forceinline__ int width(int p) { return p == 0 ? 12 : 4; }
    static __device__ __forceinline__ uint32_t key(uint16_t h) { return (uint32_t)(h ^ ((h & 0x8000u) ? 0xffffu : 0x8000u)); }
    static __device__ __forceinline__ float value(uint16_t h) { return __builtin_bit_cast(float, (uint32_t)h << 16); }
    static __device__ __forceinline__ float from_key(uint32_t k)
    {
        const uint32_t h = (k & 0x8000u) ? (k ^ 0x8000u) : (k ^ 0xffffu);
        return __builtin_bit_cast(float, (h & 0xffffu) << 16);
    }
};
template <> struct Key<AS_F32> {
    using T = float;
    static constexpr int kBits = 32;
    static constexpr int kPasses = 3;
    static __device__ __forceinline__ int width(int p) { return p == 2 ? 8 : 12; }
    static __device__ __forceinline__ uint32_t key(float f)
    {
        const uint32_t b = __builtin_bit_cast(uint32_t, f);
        return b ^ ((b & 0x80000000u) ? 0xffffffffu : 0x80000000u);
    }
    static __device__ __forceinline__ float value(float f) { return f; }
    static __device__ __forceinline__ float from_key(uint32_t k)
    {
        const uint32_t b = (k & 0x80000000u) ? (k ^ 0x80000000u) : ~k;
        return __builtin_bit_cast(float, b);
    }
};

struct Shared {
    unsigned long long hist[kMaxBins];
    unsigned long long part[kThreads];
    unsigned long long wave_tot[kThreads / 64];
    unsigned long long above;      // mass / count strictly above the chosen digit
    unsigned long long total;
    int digit;
    float red[kThreads / 64];
};

// Exclusive prefix of one value per thread, thread order, plus the block total.
__device__ __forceinline__ unsigned long long block_excl_scan(unsigned long long x, Shared &sh,
                                                              unsigned long long &total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned long long incl = x;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const unsigned long long y = __shfl_up(incl, d, 64);
        if (lane >= d) incl += y;
    }
    if (lane == 63) sh.wave_tot[wave] = incl;
    __syncthreads();
    unsigned long long base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) {
        const unsigned long long t = sh.wave_tot[w];
        if (w < wave) base += t;
        tot += t;
    }
    __syncthreads();
    total = tot;
    return base + incl - x;
}

// Scan hist[0..nb) from the top bin down and pick the first bin D at which
// before + (sum of bins >= D) satisfies `reached`.  Leaves sh.digit = D and
// sh.above = before + (sum of bins > D); sh.total = sum of all bins.
template <class Reached>
__device__ __forceinline__ void pick_digit(Shared &sh, int nb, unsigned long long before, Reached reached)
{
    const int per = (nb + kThreads - 1) / kThreads;
    // thread t owns the `per` bins nb-1-t*per, nb-2-t*per, ... (descending)
    unsigned long long local = 0;
    for (int i = 0; i < per; ++i) {
        const int bin = nb - 1 - ((int)threadIdx.x * per + i);
        if (bin >= 0) local += sh.hist[bin];
    }
    if (threadIdx.x == 0) sh.digit = -1;
    unsigned long long total;
    const unsigned long long excl = block_excl_scan(local, sh, total);
    // exactly one thread sees the predicate flip inside its bins
    if (!reached(before + excl) && reached(before + excl + local)) {
        unsigned long long acc = before + excl;
        for (int i = 0; i < per; ++i) {
            const int bin = nb - 1 - ((int)threadIdx.x * per + i);
            if (bin < 0) break;
            const unsigned long long h = sh.hist[bin];
            if (reached(acc + h)) {
                sh.digit = bin;
                sh.above = acc;
                break;
            }
            acc += h;
        }
    }
    if (threadIdx.x == 0) sh.total = total;
    __syncthreads();
    if (sh.digit < 0) {                 // target beyond everything present: keep all
        __syncthreads();
        if (threadIdx.x == 0) {
            int lowest = 0;
            for (int b = 0; b < nb; ++b)
                if (sh.hist[b]) { lowest = b; break; }
            sh.digit = lowest;
            sh.above = before + total - sh.hist[lowest];
        }
        __syncthreads();
    }
}

template <int DT>
__global__ __launch_bounds__(kThreads) void threshold_kernel(const void *logits, int64_t ld, int32_t V,
                                                             const uint8_t *finished_in,
                                                             const int32_t *row_ids, float temp,
                                                             int32_t top_k, float top_p, float *thr_out)
{
    using K = Key<DT>;
    using T = typename K::T;
    __shared__ Shared sh;

    const int64_t r = blockIdx.x;
    if (finished_in != nullptr && finished_in[r] != 0) return;
    const int64_t src = row_ids ? (int64_t)row_ids[r] : r;
    const T *row = reinterpret_cast<const T *>(logits) + src * ld;

    uint32_t thr_key = 0;               // keep key >= thr_key

    // ---------------- top-k: k-th largest key, counted with multiplicity
    if (top_k > 0 && top_k < V) {
        uint32_t prefix = 0;
        int done = 0;
        unsigned long long krem = (unsigned long long)top_k;
        for (int p = 0; p < K::kPasses; ++p) {
            const int w = K::width(p), nb = 1 << w, shift = K::kBits - done - w;
            for (int b = threadIdx.x; b < nb; b += kThreads) sh.hist[b] = 0;
            __syncthreads();
            for (int32_t v = threadIdx.x; v < V; v += kThreads) {
                const uint32_t key = K::key(row[v]);
                if (done == 0 || (key >> (shift + w)) == prefix)
                    atomicAdd(&sh.hist[(key >> shift) & (uint32_t)(nb - 1)], 1ull);
            }
            __syncthreads();
            pick_digit(sh, nb, 0ull, [&](unsigned long long c) { return c >= krem; });
            krem -= sh.above;
            prefix = (prefix << w) | (uint32_t)sh.digit;
            done += w;
            __syncthreads();
        }
        thr_key = prefix;
    }

    // ---------------- nucleus over the survivors
    if (top_p > 0.f && top_p < 1.f) {
        const float k = 1.44269504088896340736f / temp;
        float m = -__builtin_inff();
        for (int32_t v = threadIdx.x; v < V; v += kThreads) {
            const T h = row[v];
            if (K::key(h) >= thr_key) m = fmaxf(m, K::value(h));
        }
        m = wave_max(m);
        if ((threadIdx.x & 63) == 0) sh.red[threadIdx.x >> 6] = m;
        __syncthreads();
        m = sh.red[0];
#pragma unroll
        for (int w = 1; w < kThreads / 64; ++w) m = fmaxf(m, sh.red[w]);
        const float nr = -fmaxf(ceilf(m * k), -100000.f);
        __syncthreads();

        uint32_t prefix = 0;
        int done = 0;
        unsigned long long before = 0;       // mass of groups above the current prefix
        double need = 0.0;
        for (int p = 0; p < K::kPasses; ++p) {
            const int w = K::width(p), nb = 1 << w, shift = K::kBits - done - w;
            for (int b = threadIdx.x; b < nb; b += kThreads) sh.hist[b] = 0;
            __syncthreads();
            for (int32_t v = threadIdx.x; v < V; v += kThreads) {
                const T h = row[v];
                const uint32_t key = K::key(h);
                if (key >= thr_key && (done == 0 || (key >> (shift + w)) == prefix)) {
                    // fixed point, 31 fractional bits relative to 2^ceil(max*k)
                    const float e = __builtin_amdgcn_exp2f(fmaf(K::value(h), k, nr));
                    const unsigned long long q = (unsigned long long)(uint32_t)(e * 2147483648.f + 0.5f);
                    if (q) atomicAdd(&sh.hist[(key >> shift) & (uint32_t)(nb - 1)], q);
                }
            }
            __syncthreads();
            if (p == 0) {
                // total mass = sum of the first histogram
                unsigned long long local = 0, total;
                for (int b = threadIdx.x; b < nb; b += kThreads) local += sh.hist[b];
                block_excl_scan(local, sh, total);
                need = (double)top_p * (double)total;
            }
            pick_digit(sh, nb, before, [&](unsigned long long c) { return (double)c >= need; });
            before = sh.above;
            prefix = (prefix << w) | (uint32_t)sh.digit;
            done += w;
            __syncthreads();
        }
        if (prefix > thr_key) thr_key = prefix;
    }

    if (threadIdx.x == 0) thr_out[r] = K::from_key(thr_key);
}

}  // namespace

as_status launch_threshold(as_ctx *ctx, const void *logits, int64_t rows, int64_t ld,
                           const uint8_t *finished_in, const int32_t *row_ids, float temp,
                           int32_t top_k, float top_p, float *thr_out)
{
    if (rows == 0) return AS_OK;
    if (ctx->dtype == AS_BF16)
        launch(ctx, kKernelThreshold, threshold_kernel<AS_BF16>, dim3((unsigned)rows), dim3(kThreads), 0,
               logits, ld, ctx->V, finished_in, row_ids, temp, top_k, top_p, thr_out);
    else
        launch(ctx, kKernelThreshold, threshold_kernel<AS_F32>, dim3((unsigned)rows), dim3(kThreads), 0,
               logits, ld, ctx->V, finished_in, row_ids, temp, top_k, top_p, thr_out);
    AS_HIP_TRY(ctx, hipGetLastError());
    return AS_OK;
}

}  // namespace as
