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
//
// The radix select reads the row once per digit and its histograms are hot in a
// few bins (the leading digit of a bell-shaped row is mostly sign and exponent),
// so it is the general path only.  Rows of up to 32768 logits that can be read in
// 16-byte pieces take the resident path further down: the row is loaded once into
// registers, a coarse histogram with evenly filled bins finds the neighbourhood of
// the answer, and the few logits in that neighbourhood are ranked exactly.  Longer
// rows take the same method with passes over memory instead (the streamed path at
// the end).  All paths use the same keys and the same fixed-point masses, so they
// return the same threshold.
#include <type_traits>

#include "as_common.hpp"
#include "as_row.hpp"
#include "as_tile.hpp"

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
    // (-0 and +0 are one value: one key)
    static __device__ __forceinline__ uint32_t key(uint16_t h)
    {
        h = (h & 0x7fffu) ? h : (uint16_t)0;
        return (uint32_t)(h ^ ((h & 0x8000u) ? 0xffffu : 0x8000u));
    }
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
        uint32_t b = __builtin_bit_cast(uint32_t, f);
        b = (b << 1) ? b : 0u;                   // (-0 and +0 are one value: one key)
        return b ^ ((b & 0x80000000u) ? 0xffffffffu : 0x80000000u);
    }
    static __device__ __forceinline__ float value(float f) { return f; }
    static __device__ __forceinline__ float from_key(uint32_t k)
    {
        const uint32_t b = (k & 0x80000000u) ? (k ^ 0x80000000u) : ~k;
        return __builtin_bit_cast(float, b);
    }
};

// Probability mass of a logit in fixed point: 31 fractional bits relative to 2^ceil(max*k), nr = -ceil(max*k).
__device__ __forceinline__ unsigned long long mass_q(float x, float k, float nr)
{
    const float e = __builtin_amdgcn_exp2f(fmaf(x, k, nr));
    return (unsigned long long)(uint32_t)(e * 2147483648.f + 0.5f);
}

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
__device__ __forceinline__ unsigned long long block_excl_scan(unsigned long long x, unsigned long long *wave_tot,
                                                              unsigned long long &total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned long long incl = x;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const unsigned long long y = __shfl_up(incl, d, 64);
        if (lane >= d) incl += y;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    unsigned long long base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) {
        const unsigned long long t = wave_tot[w];
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
    const unsigned long long excl = block_excl_scan(local, sh.wave_tot, total);
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

// Radix select over one row; every thread of the block returns the threshold key.
template <int DT>
__device__ __forceinline__ uint32_t radix_threshold(Shared &sh, const typename Key<DT>::T *row, int32_t V, float temp,
                                                    int32_t top_k, float top_p)
{
    using K = Key<DT>;
    using T = typename K::T;
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
                    const unsigned long long q = mass_q(K::value(h), k, nr);
                    if (q) atomicAdd(&sh.hist[(key >> shift) & (uint32_t)(nb - 1)], q);
                }
            }
            __syncthreads();
            if (p == 0) {
                // total mass = sum of the first histogram
                unsigned long long local = 0, total;
                for (int b = threadIdx.x; b < nb; b += kThreads) local += sh.hist[b];
                block_excl_scan(local, sh.wave_tot, total);
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
    return thr_key;
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
    const uint32_t thr_key = radix_threshold<DT>(sh, row, V, temp, top_k, top_p);
    if (threadIdx.x == 0) thr_out[r] = K::from_key(thr_key);
}

// ------------------------------------------------------------ resident path

constexpr int kCoarseBins = 2048;        // mass histogram: 64 bins per factor of two below the row's reference
constexpr int kCandCap = 1024;           // logits ranked exactly

struct Resident {
    unsigned long long hist[kCoarseBins];
    uint32_t ckey[kCandCap];
    uint32_t cq[kCandCap];
    uint32_t cidx[kCandCap];             // vocabulary index of each candidate (fused step)
    uint32_t mcount[kThreads];           // thread maxima per coarse bin (top-k)
    unsigned long long wave_tot[kThreads / 64];
    uint32_t ncand;
    uint32_t pick;                       // coarse bin / key handed from the thread that found it
    uint32_t lkey;
    int fallback;
};

union Scratch {
    Shared radix;
    Resident res;
    GenericScratch gen;
};

__device__ __forceinline__ uint32_t wave_reduce_umax(uint32_t x)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const uint32_t y = (uint32_t)__shfl_xor((int)x, d, 64);
        x = x > y ? x : y;
    }
    return x;
}
__device__ __forceinline__ uint32_t wave_reduce_umin(uint32_t x)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const uint32_t y = (uint32_t)__shfl_xor((int)x, d, 64);
        x = x < y ? x : y;
    }
    return x;
}

// Coarse bin of a logit from its exponent argument y (base 2, relative to the row's reference): -64*y rounded
// to the nearest integer (adding 2^23 leaves it in the low mantissa bits) and clamped to the table; monotone
// in y.  The second form is for y <= 0, which is every logit of the row itself, and agrees with the first there.
__device__ __forceinline__ int coarse_bin(float y)
{
    float t = fmaf(y, -64.f, 8388608.f);
    t = fminf(fmaxf(t, 8388608.f), 8388608.f + (float)(kCoarseBins - 1));
    return (int)(__builtin_bit_cast(uint32_t, t) - 0x4B000000u);
}
__device__ __forceinline__ int coarse_bin_nonpositive(float y)
{
    const float t = fminf(fmaf(y, -64.f, 8388608.f), 8388608.f + (float)(kCoarseBins - 1));
    return (int)(__builtin_bit_cast(uint32_t, t) - 0x4B000000u);
}

// ---- stages that work on the block's LDS tables only; every thread of the block calls them

// Top-k with k at most half the thread count, first half: each thread brings the largest key it holds; the k-th
// largest of those bounds the k-th largest logit from below.  Returns a key at or below it: the lowest thread
// maximum among the bins (256, even over the range of the maxima, from the top) that hold the first k of them.
// Also empties the candidate table.
__device__ __forceinline__ uint32_t bound_from_thread_maxima(Resident &sh, uint32_t tmax, int32_t top_k)
{
    const int tid = threadIdx.x;
    sh.mcount[tid] = 0;
    if (tid == 0) sh.ncand = 0;
    uint32_t hi = wave_reduce_umax(tmax), lo = wave_reduce_umin(tmax);
    uint32_t *red = reinterpret_cast<uint32_t *>(sh.hist);
    if ((tid & 63) == 0) { red[tid >> 6] = hi; red[4 + (tid >> 6)] = lo; }
    __syncthreads();
    hi = red[0]; lo = red[4];
#pragma unroll
    for (int w = 1; w < kThreads / 64; ++w) { hi = red[w] > hi ? red[w] : hi; lo = red[4 + w] < lo ? red[4 + w] : lo; }
    const float scale = 256.f / ((float)(hi - lo) + 1.f);
    int mb = (int)((float)(hi - tmax) * scale);
    mb = mb > kThreads - 1 ? kThreads - 1 : mb;
    atomicAdd(&sh.mcount[mb], 1u);
    __syncthreads();
    // first bin (from the top) at which k maxima have been seen
    unsigned long long total;
    const unsigned long long mine = sh.mcount[tid];
    const unsigned long long excl = block_excl_scan(mine, sh.wave_tot, total);
    if (excl < (unsigned long long)top_k && excl + mine >= (unsigned long long)top_k) sh.pick = (uint32_t)tid;
    if (tid == 0) sh.lkey = 0xffffffffu;
    __syncthreads();
    uint32_t l = mb <= (int)sh.pick ? tmax : 0xffffffffu;
    l = wave_reduce_umin(l);
    if ((tid & 63) == 0) atomicMin(&sh.lkey, l);
    __syncthreads();
    return sh.lkey;
}

// ... second half: the table holds every logit at or above that bound (ncand of them, no more than the table
// takes); the one with exactly k-1 ahead of it is the k-th largest logit.
__device__ __forceinline__ uint32_t kth_of_candidates(Resident &sh, uint32_t ncand, int32_t top_k)
{
    for (uint32_t c = threadIdx.x; c < ncand; c += kThreads) {
        const uint32_t my = sh.ckey[c];
        uint32_t ahead = 0;
        for (uint32_t j = 0; j < ncand; ++j) {
            const uint32_t o = sh.ckey[j];
            ahead += (o > my || (o == my && j < c)) ? 1u : 0u;
        }
        if (ahead == (uint32_t)top_k - 1u) sh.pick = my;
    }
    __syncthreads();
    const uint32_t key = sh.pick;
    __syncthreads();
    return key;
}

// Exact end of a selection by weight: candidates c < ncand with key ckey[c] and integer weight cq[c] (0: not in
// the running), `before` the weight of everything above all of them.  The group of equal keys at which the
// running weight, from the largest key down, reaches `need` is the one that closes the selection; returns its
// key (or thr_key if that is larger).
__device__ __forceinline__ uint32_t closing_group(Resident &sh, uint32_t ncand, unsigned long long before, double need,
                                                  uint32_t thr_key)
{
    for (uint32_t c = threadIdx.x; c < ncand; c += kThreads) {
        const uint32_t my = sh.ckey[c];
        if (sh.cq[c] == 0) continue;
        unsigned long long above = before, group = 0;
        for (uint32_t j = 0; j < ncand; ++j) {
            const uint32_t o = sh.ckey[j];
            const unsigned long long q = sh.cq[j];
            above += o > my ? q : 0ull;
            group += o == my ? q : 0ull;
        }
        if (!((double)above >= need) && (double)(above + group) >= need) sh.pick = my;
    }
    __syncthreads();
    const uint32_t pkey = sh.pick;
    __syncthreads();
    return pkey > thr_key ? pkey : thr_key;
}

// The nucleus over the survivors of top-k, all of which are in the candidate table: their masses against the
// reference of the largest of them, then the closing group.
template <class K>
__device__ __forceinline__ uint32_t nucleus_on_candidates(Resident &sh, uint32_t ncand, uint32_t thr_key, float k,
                                                          float top_p)
{
    const int tid = threadIdx.x;
    float m = -__builtin_inff();
    for (uint32_t c = tid; c < ncand; c += kThreads)
        if (sh.ckey[c] >= thr_key) m = fmaxf(m, K::from_key(sh.ckey[c]));
    m = wave_max(m);
    float *fred = reinterpret_cast<float *>(sh.hist);
    if ((tid & 63) == 0) fred[tid >> 6] = m;
    __syncthreads();
    m = fred[0];
#pragma unroll
    for (int w = 1; w < kThreads / 64; ++w) m = fmaxf(m, fred[w]);
    const float nr = -fmaxf(ceilf(m * k), -100000.f);
    unsigned long long local = 0, total;
    for (uint32_t c = tid; c < ncand; c += kThreads) {
        const uint32_t key = sh.ckey[c];
        const unsigned long long q = key >= thr_key ? mass_q(K::from_key(key), k, nr) : 0ull;
        sh.cq[c] = (uint32_t)q;                 // 0 also takes the candidates below the threshold out
        local += q;
    }
    block_excl_scan(local, sh.wave_tot, total);
    __syncthreads();
    return closing_group(sh, ncand, 0ull, (double)top_p * (double)total, thr_key);
}

// After the masses (or counts) of a whole row have gone into the coarse bins: the first bin, from the top, at
// which the running weight reaches goal(total).  Leaves that bin in sh.pick (if any bin gets there) and
// returns the weight above it and, through `need`, the goal.
template <class Goal>
__device__ __forceinline__ unsigned long long bin_that_reaches(Resident &sh, Goal goal, double &need)
{
    const int tid = threadIdx.x;
    constexpr int kPer = kCoarseBins / kThreads;
    unsigned long long local = 0, total;
#pragma unroll
    for (int i = 0; i < kPer; ++i) local += sh.hist[tid * kPer + i];
    const unsigned long long excl = block_excl_scan(local, sh.wave_tot, total);
    need = goal(total);
    if (!((double)excl >= need) && (double)(excl + local) >= need) {
        unsigned long long acc = excl;
        for (int i = 0; i < kPer; ++i) {
            const unsigned long long h = sh.hist[tid * kPer + i];
            if ((double)(acc + h) >= need) {
                sh.pick = (uint32_t)(tid * kPer + i);
                // weight above the bin, split over two words of the (still free) candidate key table
                sh.ckey[kCandCap - 2] = (uint32_t)acc;
                sh.ckey[kCandCap - 1] = (uint32_t)(acc >> 32);
                break;
            }
            acc += h;
        }
    }
    __syncthreads();
    const unsigned long long before =
        (unsigned long long)sh.ckey[kCandCap - 2] | ((unsigned long long)sh.ckey[kCandCap - 1] << 32);
    __syncthreads();
    return before;
}

// STEP: go on and finish the sampling step for the row, which is then not read a second time.  With HAS_K from
// the candidate table (after top-k every kept logit is in it); with the nucleus alone, where most of the row
// can be kept, from the registers (bf16 rows: their 4096 sums of 8 logits take the histogram's place in LDS).
// sa then carries the step's arguments.
template <int DT, bool HAS_K, bool HAS_P, bool STEP = false>
__global__ __launch_bounds__(kThreads) void threshold_resident_kernel(const void *logits, int64_t ld, int32_t V,
                                                                      const uint8_t *finished_in,
                                                                      const int32_t *row_ids, float temp,
                                                                      int32_t top_k, float top_p, float *thr_out,
                                                                      StepArgs sa)
{
    static_assert(!STEP || HAS_K || (HAS_P && DT == AS_BF16),
                  "the fused step works on the top-k candidate table, or for a bf16 row on its registers");
    using K = Key<DT>;
    using T = typename K::T;
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    constexpr bool kHalf = sizeof(T) == 2;               // two logits per register
    constexpr int EPP = 16 / (int)sizeof(T);             // logits per 16-byte piece
    constexpr int NP = 32768 / (EPP * kThreads);         // pieces per thread: 16 (bf16) or 32 (fp32)
    __shared__ Scratch sc;
    Resident &sh = sc.res;

    const int tid = threadIdx.x;
    const int64_t r = blockIdx.x;
    if (finished_in != nullptr && finished_in[r] != 0) {
        if constexpr (STEP) {
            if (tid == 0) write_finished(sa, r);
        }
        return;
    }
    const int64_t src = row_ids ? (int64_t)row_ids[r] : r;
    const T *row = reinterpret_cast<const T *>(logits) + src * ld;

    // The row, resident: piece p of this thread holds logits (p*256 + tid)*EPP ... + EPP-1.  With top-k the
    // registers hold the order-preserving keys (0 = "no logit here", below every real key), otherwise the
    // stored values with the positions past V set to -inf.
    u32x4 pc[NP];
    const int32_t npieces = (V + EPP - 1) / EPP;
    constexpr uint32_t kNegInf = kHalf ? 0xff80ff80u : 0xff800000u;
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int32_t piece = p * kThreads + tid;
        if (piece < npieces) pc[p] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(row) + piece);
        else pc[p] = u32x4{kNegInf, kNegInf, kNegInf, kNegInf};
    }
    if (V % EPP != 0) {
        // the one piece that straddles V
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int32_t piece = p * kThreads + tid;
            if (piece == npieces - 1) {
                const int live = V - piece * EPP;            // 1 .. EPP-1
#pragma unroll
                for (int e = 0; e < EPP; ++e) {
                    if (e < live) continue;
                    if constexpr (kHalf) pc[p][e >> 1] = (e & 1) ? ((pc[p][e >> 1] & 0xffffu) | 0xff800000u)
                                                                  : ((pc[p][e >> 1] & 0xffff0000u) | 0xff80u);
                    else pc[p][e] = kNegInf;
                }
            }
        }
    }
    if (HAS_K) {
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const bool live = p * kThreads + tid < npieces;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                uint32_t w = pc[p][i];
                if constexpr (kHalf) {
                    const uint32_t neg = ((w >> 15) & 0x00010001u) * 0xffffu;     // 0xffff in each negative half
                    w ^= neg | 0x80008000u;
                } else {
                    w ^= (uint32_t)((int32_t)w >> 31) | 0x80000000u;
                }
                pc[p][i] = live ? w : 0u;
            }
        }
        if (V % EPP != 0) {
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                const int32_t piece = p * kThreads + tid;
                if (piece == npieces - 1) {
                    const int live = V - piece * EPP;
#pragma unroll
                    for (int e = 0; e < EPP; ++e) {
                        if (e < live) continue;
                        if constexpr (kHalf) pc[p][e >> 1] &= (e & 1) ? 0x0000ffffu : 0xffff0000u;
                        else pc[p][e] = 0u;
                    }
                }
            }
        }
    }

    // Between passes over the resident row: make the compiler forget what it derived from the registers, or
    // it keeps every unpacked value of one pass alive for the next and the kernel no longer fits.
    auto forget_row = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < NP; ++p) asm volatile("" : "+v"(pc[p]));
    };

    uint32_t thr_key = 0;
    bool fall = false;
    uint32_t ncand = 0;

    // ---------------- top-k.  The k-th largest of the 256 thread maxima bounds the k-th largest logit from
    // below, and for anything but adversarial rows only a few more than k logits reach it.
    if (HAS_K) {
        uint32_t tmax;
        if constexpr (kHalf) {
            uint32_t mh = 0, ml = 0;
#pragma unroll
            for (int p = 0; p < NP; ++p)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t w = pc[p][i];
                    mh = w > mh ? w : mh;
                    const uint32_t l = w << 16;
                    ml = l > ml ? l : ml;
                }
            mh >>= 16; ml >>= 16;
            tmax = mh > ml ? mh : ml;
        } else {
            tmax = 0;
#pragma unroll
            for (int p = 0; p < NP; ++p)
#pragma unroll
                for (int i = 0; i < 4; ++i) tmax = pc[p][i] > tmax ? pc[p][i] : tmax;
        }
        const uint32_t lkey = bound_from_thread_maxima(sh, tmax, top_k);
        forget_row();
        auto candidate = [&](uint32_t key, int32_t v) __attribute__((always_inline)) {
            const uint32_t i = atomicAdd(&sh.ncand, 1u);
            if (i < (uint32_t)kCandCap) {
                sh.ckey[i] = key;
                if constexpr (STEP) sh.cidx[i] = (uint32_t)v;
            }
        };
        // Branch-free over the registers: which of this thread's pieces hold a key at or above the bound (the
        // compares as wave-wide lane masks, their or is scalar work); those few pieces are then read once more
        // from memory, in one loop, since a loop over set bits cannot index registers.
        {
            const int lane_no = tid & 63;
            const uint32_t t = kHalf ? lkey << 16 : lkey;
            uint32_t hot = 0;
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                uint64_t lanes = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t w = pc[p][i];
                    lanes |= __builtin_amdgcn_uicmp(w, t, 35 /* unsigned >= */);
                    if constexpr (kHalf) lanes |= __builtin_amdgcn_uicmp(w << 16, t, 35);
                }
                hot |= ((lanes >> lane_no) & 1u) ? 1u << p : 0u;
            }
            while (hot) {
                const int p = __builtin_ctz(hot);
                hot &= hot - 1;
                const int32_t piece = p * kThreads + tid;
                const u32x4 again = reinterpret_cast<const u32x4 *>(row)[piece];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t w = again[i];
                    if constexpr (kHalf) {
                        const int32_t v = piece * EPP + 2 * i;
                        const uint32_t k0 = K::key((T)(w & 0xffffu)), k1 = K::key((T)(w >> 16));
                        if (v < V && k0 >= lkey) candidate(k0, v);
                        if (v + 1 < V && k1 >= lkey) candidate(k1, v + 1);
                    } else {
                        const int32_t v = piece * EPP + i;
                        const uint32_t k0 = K::key(__builtin_bit_cast(float, w));
                        if (v < V && k0 >= lkey) candidate(k0, v);
                    }
                }
            }
        }
        __syncthreads();
        ncand = sh.ncand;
        if (ncand > (uint32_t)kCandCap) fall = true;
        else thr_key = kth_of_candidates(sh, ncand, top_k);
        __syncthreads();
    }

    // ---------------- nucleus over the survivors
    float nr_row = 0.f;                  // minus the row's integer reference, as the nucleus pass took it
    if (HAS_P && !fall) {
        const float k = 1.44269504088896340736f / temp;
        double need;
        unsigned long long before = 0;
        if (HAS_K) {
            // every survivor of top-k is in the candidate table: work on that
            thr_key = nucleus_on_candidates<K>(sh, ncand, thr_key, k, top_p);
        } else {
            float m = -__builtin_inff();
#pragma unroll
            for (int p = 0; p < NP; ++p)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t w = pc[p][i];
                    if constexpr (kHalf) {
                        m = fmaxf(m, __builtin_bit_cast(float, w << 16));
                        m = fmaxf(m, __builtin_bit_cast(float, w & 0xffff0000u));
                    } else {
                        m = fmaxf(m, __builtin_bit_cast(float, w));
                    }
                }
            m = wave_max(m);
            float *fred = reinterpret_cast<float *>(sh.ckey);
            if ((tid & 63) == 0) fred[tid >> 6] = m;
            for (int b = tid; b < kCoarseBins; b += kThreads) sh.hist[b] = 0;
            if (tid == 0) sh.ncand = 0;
            __syncthreads();
            m = fred[0];
#pragma unroll
            for (int w = 1; w < kThreads / 64; ++w) m = fmaxf(m, fred[w]);
            const float nr = -fmaxf(ceilf(m * k), -100000.f);
            nr_row = nr;
            __syncthreads();
            // mass per coarse bin, in the fixed point of the radix path
            forget_row();
            // A logit whose mass rounds to zero adds it to a slot of the lane's own instead of a bin: no
            // branch per logit, and the many zeros of a peaked row do not pile onto the last bin.
            typedef __attribute__((address_space(3))) unsigned long long lds_u64;
            lds_u64 *const bins = (lds_u64 *)sh.hist;
            lds_u64 *const sink = (lds_u64 *)sh.mcount + (tid & 63);
            auto add_mass = [&](float x) __attribute__((always_inline)) {
                const float y = fmaf(x, k, nr);
                const float e = __builtin_amdgcn_exp2f(y);
                const uint32_t q = (uint32_t)(e * 2147483648.f + 0.5f);
                lds_u64 *const dst = q ? bins + coarse_bin_nonpositive(y) : sink;
                __hip_atomic_fetch_add(dst, (unsigned long long)q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            };
#pragma unroll
            for (int p = 0; p < NP; ++p)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t w = pc[p][i];
                    if constexpr (kHalf) {
                        add_mass(__builtin_bit_cast(float, w << 16));
                        add_mass(__builtin_bit_cast(float, w & 0xffff0000u));
                    } else {
                        add_mass(__builtin_bit_cast(float, w));
                    }
                }
            __syncthreads();
            // total, then the first bin (from the top) at which top_p of it is reached
            before = bin_that_reaches(sh, [&](unsigned long long total) { return (double)top_p * (double)total; }, need);
            // the logits of that bin go to the candidate table
            // (second pass over the row: keep the compiler from holding every exponent of the first pass in a
            // register until here)
            float nr2 = nr;
            asm volatile("" : "+v"(nr2));
            forget_row();
            // The coarse bin is monotone in the logit, so the logits of one bin are one interval of values:
            // its ends by bisection over the keys between -inf and +inf (the same few steps in every thread),
            // and the pass over the row is two compares per logit.
            const int pick_bin = (int)(sh.pick < (uint32_t)kCoarseBins ? sh.pick : (uint32_t)(kCoarseBins - 1));   // (a row without mass picks nothing)
            auto first_key_with_bin_at_most = [&](int b) __attribute__((always_inline)) {
                // 64 keys at a time, one per lane: each round cuts the interval to a 63rd (3 rounds for
                // bf16 keys, 6 for fp32 ones, against 16 and 32 dependent steps of a plain bisection)
                uint32_t lo = kHalf ? 0x007fu : 0x007fffffu, hi = kHalf ? 0xff80u : 0xff800000u;
                const uint32_t lane_no = (uint32_t)(tid & 63);
                while (lo < hi) {                      // bin(hi) = 0 <= b always holds
                    const uint32_t step = (hi - lo + 62u) / 63u;            // lane 63 then probes hi (or beyond: clamped)
                    const uint64_t probe64 = (uint64_t)lo + (uint64_t)lane_no * step;
                    const uint32_t probe = probe64 < hi ? (uint32_t)probe64 : hi;
                    const bool at_most = coarse_bin(fmaf(K::from_key(probe), k, nr2)) <= b;
                    const unsigned long long yes = __ballot(at_most);       // lane 63 probes hi or beyond
                    const uint32_t first = (uint32_t)__builtin_ctzll(yes);
                    const uint64_t top = (uint64_t)lo + (uint64_t)first * step;
                    const uint32_t new_hi = top < hi ? (uint32_t)top : hi;
                    if (first > 0) lo = lo + (first - 1u) * step + 1u;      // the lane before said no
                    hi = new_hi;
                }
                return lo;
            };
            const float xlo = K::from_key(first_key_with_bin_at_most(pick_bin));
            const float xhi = pick_bin > 0 ? K::from_key(first_key_with_bin_at_most(pick_bin - 1)) : __builtin_inff();
            auto in_bin = [&](uint32_t bits) __attribute__((always_inline)) {
                const float x = __builtin_bit_cast(float, bits);
                return (x >= xlo) & (x < xhi);
            };
            auto candidate = [&](uint32_t bits) __attribute__((always_inline)) {
                const float x = __builtin_bit_cast(float, bits);
                const unsigned long long q = mass_q(x, k, nr2);
                if (q) {
                    const uint32_t i = atomicAdd(&sh.ncand, 1u);
                    if (i < (uint32_t)kCandCap) {
                        sh.ckey[i] = kHalf ? K::key((T)(bits >> 16)) : K::key(__builtin_bit_cast(T, (typename std::conditional<kHalf, uint16_t, uint32_t>::type)bits));
                        sh.cq[i] = (uint32_t)q;
                    }
                }
            };
            // branch-free over the registers: which of this thread's pieces hold a logit of the bin
            // (compares as wave-wide lane masks: two vector compares per logit, the and/or of the masks is
            // scalar work)
            auto bin_lanes = [&](uint32_t bits) __attribute__((always_inline)) {
                const float x = __builtin_bit_cast(float, bits);
                return __builtin_amdgcn_fcmpf(x, xlo, 3 /* ordered >= */) &
                       __builtin_amdgcn_fcmpf(x, xhi, 4 /* ordered <  */);
            };
            const int lane_no = tid & 63;
            uint32_t hot = 0;
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                uint64_t lanes = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t w = pc[p][i];
                    if constexpr (kHalf) lanes |= bin_lanes(w << 16) | bin_lanes(w & 0xffff0000u);
                    else lanes |= bin_lanes(w);
                }
                hot |= ((lanes >> lane_no) & 1u) ? 1u << p : 0u;
            }
            // those few pieces once more from memory (a loop over set bits cannot index registers), one body
            // of code for all of them
            while (hot) {
                const int p = __builtin_ctz(hot);
                hot &= hot - 1;
                const int32_t piece = p * kThreads + tid;
                const u32x4 again = reinterpret_cast<const u32x4 *>(row)[piece];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t w = again[i];
                    if constexpr (kHalf) {
                        const int32_t v = piece * EPP + 2 * i;
                        if (v < V && in_bin(w << 16)) candidate(w << 16);
                        if (v + 1 < V && in_bin(w & 0xffff0000u)) candidate(w & 0xffff0000u);
                    } else {
                        if (piece * EPP + i < V && in_bin(w)) candidate(w);
                    }
                }
            }
            __syncthreads();
            ncand = sh.ncand;
            if (ncand > (uint32_t)kCandCap) fall = true;
        }
        // rank exactly: the nucleus closes with a whole group of equal logits
        if (!HAS_K && !fall) thr_key = closing_group(sh, ncand, before, need, thr_key);
    }

    if (fall) {            // uniform over the block: every thread saw the same counters
        __syncthreads();
        thr_key = radix_threshold<DT>(sc.radix, row, V, temp, top_k, top_p);
    }
    if (tid == 0 && thr_out != nullptr) thr_out[r] = K::from_key(thr_key);

    if constexpr (STEP) {
        __syncthreads();
        if (fall) {
            generic_step_row<T>(sa, r, K::from_key(thr_key), sc.gen);
            return;
        }
        if constexpr (!HAS_K) {
            // ---- the sampling step from the registers (Sec. 4.1 loop body).  Weights exp2(x*k - ref) of the
            // kept logits against the reference of the nucleus pass; per piece of 8 an fp32 sum in vocabulary
            // order; fp64 from there on.  The bucket is the last piece, then the last logit in it, that has
            // weight and whose mass before it does not exceed c*S: with c*S inside the row that is the one
            // it falls into, and past the end by rounding it is the last kept token.
            const float k = sa.k;
            const float thr = K::from_key(thr_key);
            float nr3 = nr_row;
            asm volatile("" : "+v"(nr3));
            forget_row();
            float *psum = reinterpret_cast<float *>(sh.hist);            // NP * kThreads = 4096 entries
            double *dred = reinterpret_cast<double *>(sh.ckey);
            uint32_t *ured = sh.mcount;
            auto weight = [&](uint32_t bits) __attribute__((always_inline)) {
                const float x = __builtin_bit_cast(float, bits);
                return x >= thr ? fast_exp2(fmaf(x, k, nr3)) : 0.f;
            };
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                float sum = 0.f;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t w = pc[p][i];
                    sum += weight(w << 16);
                    sum += weight(w & 0xffff0000u);
                }
                psum[p * kThreads + tid] = sum;
            }
            __syncthreads();
            float ent[NP];
            double local = 0.0;
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                ent[i] = psum[tid * NP + i];
                local += (double)ent[i];
            }
            const double incl = wave_scan_add(local);
            if ((tid & 63) == 63) dred[tid >> 6] = incl;
            __syncthreads();
            double base = 0.0, S = 0.0;
#pragma unroll
            for (int w = 0; w < kThreads / 64; ++w) {
                const double t = dred[w];
                if (w < (tid >> 6)) base += t;
                S += t;
            }
            const double tau = (double)sa.codes[r] * S;
            uint32_t best = 0;                                           // piece index + 1
            double best_before = 0.0, acc = base + incl - local;
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                if (ent[i] > 0.f && acc <= tau) {
                    best = (uint32_t)(tid * NP + i) + 1u;
                    best_before = acc;
                }
                acc += (double)ent[i];
            }
            const uint32_t wbest = wave_reduce_umax(best);
            if ((tid & 63) == 0) ured[tid >> 6] = wbest;
            __syncthreads();
            uint32_t gbest = ured[0];
#pragma unroll
            for (int w = 1; w < kThreads / 64; ++w) gbest = gbest > ured[w] ? gbest : ured[w];
            if (best == gbest && gbest != 0u) dred[4] = best_before;
            __syncthreads();
            if (tid == 0) {
                int32_t piece = gbest ? (int32_t)gbest - 1 : 0;
                if (piece > npieces - 1) piece = npieces - 1;
                const u32x4 again = reinterpret_cast<const u32x4 *>(row)[piece];
                double before = gbest ? dred[4] : 0.0, lo = before;
                float ev = 0.f;
                int32_t token = piece * EPP;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t w = again[i];
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const int32_t v = piece * EPP + 2 * i + h;
                        const float e = v < V ? weight(h ? (w & 0xffff0000u) : (w << 16)) : 0.f;
                        if (e > 0.f && before <= tau) {
                            token = v;
                            lo = before;
                            ev = e;
                        }
                        before += (double)e;
                    }
                }
                RowOut o;
                o.token = token;
                o.c_next = rescale_code(tau, lo, (double)ev);
                o.prob = (float)((double)ev / S);
                o.f_lo = (float)(lo / S);
                write_row(sa, r, o);
            }
            return;
        }
        // ---- the sampling step on the kept candidates (Sec. 4.1 loop body): weights against an integer
        // reference, cumulative sums in vocabulary order, first bucket above the code, rescale
        const float k = sa.k;
        float m = -__builtin_inff();
        for (uint32_t c = tid; c < ncand; c += kThreads)
            if (sh.ckey[c] >= thr_key) m = fmaxf(m, K::from_key(sh.ckey[c]));
        m = wave_max(m);
        float *fred = reinterpret_cast<float *>(sh.hist);
        double *dred = reinterpret_cast<double *>(sh.hist) + 8;
        if ((tid & 63) == 0) fred[tid >> 6] = m;
        if (tid == 0) sh.pick = 0xffffffffu;
        __syncthreads();
        m = fmaxf(fmaxf(fred[0], fred[1]), fmaxf(fred[2], fred[3]));
        const float ref = fmaxf(ceilf(m * k), kRefFloor);
        double part = 0.0;
        for (uint32_t c = tid; c < ncand; c += kThreads) {
            const uint32_t key = sh.ckey[c];
            const float e = key >= thr_key ? fast_exp2(fmaf(K::from_key(key), k, -ref)) : 0.f;
            sh.cq[c] = __builtin_bit_cast(uint32_t, e);
            if (!(e > 0.f)) sh.cidx[c] = 0xffffffffu;       // not kept (or no weight): behind every real index
            part += (double)e;
        }
        if (ncand <= (uint32_t)kThreads) {
            // The usual case, one candidate per thread: its rank among the kept ones by vocabulary index (the
            // indices are distinct) is an integer loop; the weights go to their ranks, one fp64 scan gives
            // every kept token the mass before it, and the bucket is the last one whose mass before it does
            // not exceed c*S (past the end by rounding: the last kept token).
            double *se = reinterpret_cast<double *>(sh.hist) + 16;           // [kThreads] weights by rank
            uint32_t *sc = reinterpret_cast<uint32_t *>(se + kThreads);      // [kThreads] candidate at that rank
            uint32_t *ured = sh.mcount;
            __syncthreads();
            const bool have = (uint32_t)tid < ncand;
            const float e_mine = have ? __builtin_bit_cast(float, sh.cq[tid]) : 0.f;
            const uint32_t idx = have ? sh.cidx[tid] : 0xffffffffu;
            uint32_t rank = 0, nk = 0;
            for (uint32_t j = 0; j < ncand; ++j) {
                const uint32_t o = sh.cidx[j];
                rank += o < idx ? 1u : 0u;
                nk += o != 0xffffffffu ? 1u : 0u;
            }
            if (idx != 0xffffffffu) {
                se[rank] = (double)e_mine;
                sc[rank] = (uint32_t)tid;
            }
            __syncthreads();
            const double v = (uint32_t)tid < nk ? se[tid] : 0.0;
            const double incl = wave_scan_add(v);
            if ((tid & 63) == 63) dred[tid >> 6] = incl;
            __syncthreads();
            double base = 0.0, S = 0.0;
#pragma unroll
            for (int w = 0; w < kThreads / 64; ++w) {
                const double t = dred[w];
                if (w < (tid >> 6)) base += t;
                S += t;
            }
            const double tau = (double)sa.codes[r] * S;
            const double lo = base + incl - v;
            const uint32_t best = ((uint32_t)tid < nk && lo <= tau) ? (uint32_t)tid + 1u : 0u;
            const uint32_t wbest = wave_reduce_umax(best);
            if ((tid & 63) == 0) ured[tid >> 6] = wbest;
            __syncthreads();
            uint32_t gbest = ured[0];
#pragma unroll
            for (int w = 1; w < kThreads / 64; ++w) gbest = gbest > ured[w] ? gbest : ured[w];
            if (best == gbest && gbest != 0u) {
                RowOut o;
                o.token = (int32_t)sh.cidx[sc[tid]];
                o.c_next = rescale_code(tau, lo, v);
                o.prob = (float)(v / S);
                o.f_lo = (float)(lo / S);
                write_row(sa, r, o);
            } else if (gbest == 0u && tid == 0) {
                // no kept candidate with weight: cannot happen for finite logits; leave a valid row behind
                RowOut o;
                o.token = 0;
                o.c_next = rescale_code(0.0, 0.0, 1.0);
                o.prob = 0.f;
                o.f_lo = 0.f;
                write_row(sa, r, o);
            }
            return;
        }
        part = wave_sum(part);
        if ((tid & 63) == 0) dred[tid >> 6] = part;
        __syncthreads();
        const double S = (dred[0] + dred[1]) + (dred[2] + dred[3]);
        const double tau = (double)sa.codes[r] * S;
        for (uint32_t c = tid; c < ncand; c += kThreads) {
            const float e = __builtin_bit_cast(float, sh.cq[c]);
            if (!(e > 0.f)) continue;
            const uint32_t my = sh.cidx[c];
            double lo = 0.0;
            for (uint32_t j = 0; j < ncand; ++j)
                lo += sh.cidx[j] < my ? (double)__builtin_bit_cast(float, sh.cq[j]) : 0.0;
            if (lo <= tau && tau < lo + (double)e) {
                sh.pick = c;
                dred[4] = lo;
            }
        }
        __syncthreads();
        if (tid == 0) {
            uint32_t win = sh.pick;
            double lo = dred[4];
            if (win == 0xffffffffu) {
                // code at the very top by rounding: the last kept token of the vocabulary
                uint32_t best = 0;
                win = 0;
                for (uint32_t j = 0; j < ncand; ++j)
                    if (__builtin_bit_cast(float, sh.cq[j]) > 0.f && sh.cidx[j] >= best) { best = sh.cidx[j]; win = j; }
                lo = 0.0;
                for (uint32_t j = 0; j < ncand; ++j)
                    lo += sh.cidx[j] < best ? (double)__builtin_bit_cast(float, sh.cq[j]) : 0.0;
            }
            const double ev = (double)__builtin_bit_cast(float, sh.cq[win]);
            RowOut o;
            o.token = (int32_t)sh.cidx[win];
            o.c_next = rescale_code(tau, lo, ev);
            o.prob = (float)(ev / S);
            o.f_lo = (float)(lo / S);
            if (sh.cidx[win] == 0xffffffffu) {
                // no kept candidate with weight: cannot happen for finite logits; leave a valid row behind
                o.token = 0;
                o.c_next = rescale_code(0.0, 0.0, 1.0);
                o.prob = 0.f;
                o.f_lo = 0.f;
            }
            write_row(sa, r, o);
        }
    }
}


// ------------------------------------------------------------ streamed path
//
// Rows too long for the registers (more than 32768 logits) or not laid out in whole 16-byte pieces, k at most
// half the thread count: the method of the resident kernel with every visit of the row a pass over memory, four pieces
// per thread in flight.  Top-k with k up to 128 takes two passes (thread maxima, then the logits at or above
// the bound they give), any larger k three (maximum, count per coarse bin, the logits of the bin that holds
// the k-th), the nucleus alone three (maximum, mass per coarse bin, the logits of the bin where the nucleus
// closes); the nucleus after top-k works on the candidate table.  Same keys, same fixed-point masses, same
// fall-back as the other two kernels, so the same threshold.
// KMODE 0: no top-k; 1: bound from the thread maxima (k at most half the thread count); 2: any k, by counts per
// coarse bin, the way the nucleus goes by mass per coarse bin.
template <int DT, int KMODE, bool HAS_P>
__global__ __launch_bounds__(kThreads) void threshold_stream_kernel(const void *logits, int64_t ld, int32_t V,
                                                                    const uint8_t *finished_in,
                                                                    const int32_t *row_ids, float temp,
                                                                    int32_t top_k, float top_p, float *thr_out)
{
    using K = Key<DT>;
    using T = typename K::T;
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    constexpr bool kHalf = sizeof(T) == 2;
    constexpr int EPP = 16 / (int)sizeof(T);
    __shared__ Scratch sc;
    Resident &sh = sc.res;
    const int tid = threadIdx.x;
    const int64_t r = blockIdx.x;
    if (finished_in != nullptr && finished_in[r] != 0) return;
    const int64_t src = row_ids ? (int64_t)row_ids[r] : r;
    const T *row = reinterpret_cast<const T *>(logits) + src * ld;
    // the row as the whole 16-byte pieces it touches: `shift` elements of the first one lie before it
    const int32_t shift = (int32_t)((reinterpret_cast<uintptr_t>(row) & 15u) / sizeof(T));
    const u32x4 *const pieces = reinterpret_cast<const u32x4 *>(row - shift);
    const int32_t vend = V + shift;
    const int32_t npieces = (vend + EPP - 1) / EPP;

    // f(key, value) for every logit of the row (value: the stored logit widened to fp32), each once
    auto sweep = [&](auto f) __attribute__((always_inline)) {
        for (int32_t base = tid; base < npieces; base += 4 * kThreads) {
            u32x4 w[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int32_t piece = base + u * kThreads;
                w[u] = piece < npieces ? pieces[piece] : u32x4{0, 0, 0, 0};
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int32_t piece = base + u * kThreads;
                if (piece >= npieces) break;
                // elements [first, live) of this piece are the row's (all of them except at the row's two ends)
                const int32_t first = piece == 0 ? shift : 0, live = vend - piece * EPP;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t d = w[u][i];
                    if constexpr (kHalf) {
                        if (2 * i >= first && 2 * i < live) f(K::key((T)(d & 0xffffu)), __builtin_bit_cast(float, d << 16));
                        if (2 * i + 1 >= first && 2 * i + 1 < live)
                            f(K::key((T)(d >> 16)), __builtin_bit_cast(float, d & 0xffff0000u));
                    } else {
                        if (i >= first && i < live) f(K::key(__builtin_bit_cast(float, d)), __builtin_bit_cast(float, d));
                    }
                }
            }
        }
    };
    auto umax = [](uint32_t a, uint32_t b) { return a > b ? a : b; };

    uint32_t thr_key = 0;
    bool fall = false;
    uint32_t ncand = 0;

    constexpr bool HAS_K = KMODE == 1;
    if (HAS_K) {
        // the k-th largest of the thread maxima bounds the k-th largest logit from below
        uint32_t tmax = 0;
        sweep([&](uint32_t key, float) __attribute__((always_inline)) { tmax = umax(tmax, key); });
        const uint32_t lkey = bound_from_thread_maxima(sh, tmax, top_k);
        sweep([&](uint32_t key, float) __attribute__((always_inline)) {
            if (key >= lkey) {
                const uint32_t i = atomicAdd(&sh.ncand, 1u);
                if (i < (uint32_t)kCandCap) sh.ckey[i] = key;
            }
        });
        __syncthreads();
        ncand = sh.ncand;
        if (ncand > (uint32_t)kCandCap) fall = true;
        else thr_key = kth_of_candidates(sh, ncand, top_k);
        __syncthreads();
    }

    const float k = 1.44269504088896340736f / temp;

    // The row's integer reference (for the bins and the masses), by one pass.
    auto row_reference = [&]() __attribute__((always_inline)) {
        float m = -__builtin_inff();
        sweep([&](uint32_t, float x) __attribute__((always_inline)) { m = fmaxf(m, x); });
        m = wave_max(m);
        float *fred = reinterpret_cast<float *>(sh.ckey);
        __syncthreads();
        if ((tid & 63) == 0) fred[tid >> 6] = m;
        __syncthreads();
        m = fred[0];
#pragma unroll
        for (int w = 1; w < kThreads / 64; ++w) m = fmaxf(m, fred[w]);
        __syncthreads();
        return -fmaxf(ceilf(m * k), -100000.f);
    };

    // One selection over the whole row by coarse bins.  weigh(key, x) is a logit's integer weight: 1 to count
    // it, its fixed-point mass for the nucleus, 0 to leave it out; goal(total) is what the running weight,
    // from the largest logit down, has to reach.  Two passes: weight per bin, then the logits of the bin in
    // which the goal is reached, ranked exactly; the group of equal logits that reaches it stays whole and
    // its key becomes the threshold.
    auto select = [&](float nr, auto weigh, auto goal) __attribute__((always_inline)) {
        for (int b = tid; b < kCoarseBins; b += kThreads) sh.hist[b] = 0;
        if (tid == 0) sh.ncand = 0;
        __syncthreads();
        typedef __attribute__((address_space(3))) unsigned long long lds_u64;
        lds_u64 *const bins = (lds_u64 *)sh.hist;
        lds_u64 *const sink = (lds_u64 *)sh.mcount + (tid & 63);      // where a weight of zero is "added"
        sweep([&](uint32_t key, float x) __attribute__((always_inline)) {
            const unsigned long long q = weigh(key, x);
            lds_u64 *const dst = q ? bins + coarse_bin_nonpositive(fmaf(x, k, nr)) : sink;
            __hip_atomic_fetch_add(dst, q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        });
        __syncthreads();
        double need;
        const unsigned long long before = bin_that_reaches(sh, goal, need);
        const int pick_bin = (int)(sh.pick < (uint32_t)kCoarseBins ? sh.pick : (uint32_t)(kCoarseBins - 1));
        sweep([&](uint32_t key, float x) __attribute__((always_inline)) {
            if (coarse_bin(fmaf(x, k, nr)) == pick_bin) {
                const unsigned long long q = weigh(key, x);
                if (q) {
                    const uint32_t i = atomicAdd(&sh.ncand, 1u);
                    if (i < (uint32_t)kCandCap) {
                        sh.ckey[i] = key;
                        sh.cq[i] = (uint32_t)q;
                    }
                }
            }
        });
        __syncthreads();
        ncand = sh.ncand;
        if (ncand > (uint32_t)kCandCap) {
            fall = true;
            return;
        }
        thr_key = closing_group(sh, ncand, before, need, thr_key);
    };

    if (KMODE == 2) {
        // top-k for any k: count the logits per coarse bin from the top until k are reached
        const float nr = row_reference();
        select(nr, [](uint32_t, float) { return 1ull; }, [&](unsigned long long) { return (double)top_k; });
        if (HAS_P && !fall) {
            const uint32_t floor_key = thr_key;
            select(nr, [&](uint32_t key, float x) { return key >= floor_key ? mass_q(x, k, nr) : 0ull; },
                   [&](unsigned long long total) { return (double)top_p * (double)total; });
        }
    } else if (HAS_P && !fall) {
        if (HAS_K) {
            // every survivor of top-k is in the candidate table
            thr_key = nucleus_on_candidates<K>(sh, ncand, thr_key, k, top_p);
        } else {
            const float nr = row_reference();
            select(nr, [&](uint32_t, float x) { return mass_q(x, k, nr); },
                   [&](unsigned long long total) { return (double)top_p * (double)total; });
        }
    }

    if (fall) {
        __syncthreads();
        thr_key = radix_threshold<DT>(sc.radix, row, V, temp, top_k, top_p);
    }
    if (tid == 0) thr_out[r] = K::from_key(thr_key);
}

}  // namespace

// ------------------------------------------------------------ top-k step, single tile
//
// Top-k (k up to kTileTopK, optionally followed by the nucleus) and the sampling step for bf16 rows of whole,
// aligned 16-byte pieces that fit one tile of 64 KiB: four waves of 16 KiB each, the loads and the early look at
// the finished flag as in the single-tile sampling kernel.  Nothing per logit but integer work, and after the
// row has landed nothing that waits for memory:
//   * a stored bf16 becomes an order-preserving signed 16-bit key, two to a register (three packed
//     instructions per register); a lane keeps the packed maximum of each of its 16 pieces and of all of them.
//   * the k-th largest of the block's 256 lane maxima, found by every wave by bisection between the smallest
//     and the largest of them (four ballot counts per round), is at or below the k-th largest logit, and for
//     anything but adversarial rows only a few more than k logits reach it.
//   * a piece whose packed maximum reaches that bound (a wave-uniform test per piece, mostly not taken) goes to
//     LDS whole, 16 bytes and its position, into a table of the wave's own (no atomics: slots come from the
//     wave's ballot).
//   * one wave finishes the step with no further barrier: a lane per hot piece takes it apart and the logits
//     that reach the bound become the candidates, at most 64, a candidate per lane; two passes over the table
//     (every lane reads every candidate, broadcast reads) give each candidate the number and the weight of the
//     keys above its own (top-k with ties, nucleus with whole groups) and then the mass before it in
//     vocabulary order; the bucket of the code and the rescaling follow (Sec. 4.1 loop body).  fp64 sums.
// A table that overflows (heavy ties, flat rows) sends the block to the radix select and the plain three-pass
// step, as in the resident kernel.
constexpr int kTileTopK = 48;
constexpr int kTileCand = 64;

typedef short i16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pk_max_i16(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(i16x2, a), __builtin_bit_cast(i16x2, b)));
}
// two stored bf16 -> two signed 16-bit keys in the same order as the values (negative values have their
// magnitude bits flipped); its own inverse
__device__ __forceinline__ uint32_t pk_key_bf16(uint32_t w)
{
    const i16x2 v = __builtin_bit_cast(i16x2, w);
    const uint32_t neg = __builtin_bit_cast(uint32_t, v >> 15);      // 0xffff in each negative half
    return w ^ (neg & 0x7fff7fffu);
}
__device__ __forceinline__ float key_to_float(int32_t key)
{
    const uint32_t k16 = (uint32_t)key & 0xffffu;
    const uint32_t bits = (k16 & 0x8000u) ? (k16 ^ 0x7fffu) : k16;
    return __builtin_bit_cast(float, bits << 16);
}
// lanes below this one among those set in `mask`
__device__ __forceinline__ uint32_t rank_in(unsigned long long mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

struct TileTopK {
    int32_t lane_max[kThreads];                          // key of the largest logit of every lane
    uint32_t hot_vec[kThreads / 64][kTileCand][4];       // pieces that hold a logit at or above the bound, per wave
    int32_t hot_pos[kThreads / 64][kTileCand];           // vocabulary index of their first logit
    int32_t hot_n[kThreads / 64];
    // the candidates: key, vocabulary index, weight (sentinels behind the last: lowest key, largest index, no weight)
    __attribute__((aligned(16))) int32_t ckey[kTileCand];
    __attribute__((aligned(16))) int32_t cidx[kTileCand];
    __attribute__((aligned(16))) double cw[kTileCand];
};

template <bool HAS_P, bool NT>
__global__ __launch_bounds__(kThreads, 4) void topk_tile_kernel(StepArgs a, int32_t top_k, float top_p)
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    constexpr int NW = 4, ITERS = 16, G = 4, NG = ITERS / G, EPV = 8;
    constexpr int kShare = ITERS * 64;
    constexpr uint32_t kLowest = 0x80008000u;            // below the key of every stored value, twice: never a candidate
    // the tables of this kernel and the scratch of the general path it falls back to are never live together
    __shared__ union Shared {
        Scratch sc;
        TileTopK tk;
        __device__ Shared() {}
    } sh;
    Scratch &sc = sh.sc;
    TileTopK &tk = sh.tk;

    const int64_t r = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    uint32_t fin_word = 0u, fin_at = 0u;
    if (a.finished_in != nullptr) {
        const uint8_t *q = a.finished_in + r;
        fin_at = (uint32_t)(reinterpret_cast<uintptr_t>(q) & 3u);
        fin_word = *reinterpret_cast<const uint32_t *>(q - fin_at);
    }
    const float code = a.codes[r];
    const int64_t src = a.row_ids ? (int64_t)a.row_ids[r] : r;
    const uint16_t *row = reinterpret_cast<const uint16_t *>(a.logits) + src * a.ld;
    const unsigned char *rowb = reinterpret_cast<const unsigned char *>(row);
    const int32_t V = a.V;
    const int32_t nvec = V / EPV;
    const int32_t v0 = wave * kShare;
    u32x4 raw[ITERS];
    int32_t mych = (nvec - v0 - lane + 63) >> 6;
    mych = mych < 0 ? 0 : (mych > ITERS ? ITERS : mych);
    const bool live = v0 < nvec;
    const bool ragged = v0 + kShare > nvec;
    const unsigned char *base = rowb + (size_t)(live ? v0 : 0) * 16u;
    const uint32_t off0 = (uint32_t)lane * 16u;
    const uint32_t off_last = mych > 0 ? off0 + (uint32_t)(mych - 1) * 1024u : 0u;
    auto request_group = [&](int g) __attribute__((always_inline)) {
        // (ordinary loads where the tensor fits the caches, the non-temporal hint where it is streamed from HBM;
        // each load behind the two vector instructions of its own offset either way)
        if constexpr (NT) {
#pragma unroll
            for (int jj = 0; jj < G; ++jj) {
                uint32_t off = off0 + (uint32_t)(g * G + jj) * 1024u;
                off = off < off_last ? off : off_last;
                raw[g * G + jj] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(base + off));
            }
        } else {
#pragma unroll
            for (int jj = 0; jj < G; ++jj) {
                uint32_t off = off0 + (uint32_t)(g * G + jj) * 1024u;
                off = off < off_last ? off : off_last;
                raw[g * G + jj] = *reinterpret_cast<const u32x4 *>(base + off);
            }
        }
    };
    if (live) request_group(0);
    __builtin_amdgcn_sched_barrier(0);
    if (((fin_word >> (8u * fin_at)) & 0xffu) != 0u) {
        if (threadIdx.x == 0) write_finished(a, r);
        return;
    }
    uint32_t vm[ITERS];                    // packed maximum of each piece
    uint32_t lm = kLowest;
    if (live) {
#pragma unroll
        for (int g = 1; g < NG; ++g) request_group(g);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < ITERS; ++j) {
#pragma unroll
            for (int i = 0; i < 4; ++i) raw[j][i] = pk_key_bf16(raw[j][i]);
            if (ragged) {
                // a lane past the row's end has re-read one of its earlier pieces: no logit there
#pragma unroll
                for (int i = 0; i < 4; ++i) raw[j][i] = j < mych ? raw[j][i] : kLowest;
            }
            vm[j] = pk_max_i16(pk_max_i16(raw[j][0], raw[j][1]), pk_max_i16(raw[j][2], raw[j][3]));
            lm = pk_max_i16(lm, vm[j]);
        }
    } else {
#pragma unroll
        for (int j = 0; j < ITERS; ++j) {
            raw[j] = u32x4{kLowest, kLowest, kLowest, kLowest};
            vm[j] = kLowest;
        }
    }
    {
        const int32_t hi = (int32_t)lm >> 16, lo = (int32_t)(lm << 16) >> 16;
        tk.lane_max[threadIdx.x] = hi > lo ? hi : lo;
    }
    __syncthreads();

    // ---------------- every wave: the k-th largest of the 256 lane maxima (four per lane), by bisection between
    // the smallest and the largest of them (keys as unsigned: + 32768); a round is four ballot counts
    int32_t bound;
    {
        uint32_t m4[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) m4[i] = (uint32_t)(tk.lane_max[i * 64 + lane] + 32768);
        const uint32_t mx = max(max(m4[0], m4[1]), max(m4[2], m4[3]));
        const uint32_t mn = min(min(m4[0], m4[1]), min(m4[2], m4[3]));
        // (16-bit integers are exact as floats)
        uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)wave_max((float)mx));
        uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)-wave_max(-(float)mn));
        // at least k of the maxima are >= lo (k <= 256), fewer than k are > hi
        while (lo < hi) {
            const uint32_t mid = (lo + hi + 1u) >> 1;
            int cnt = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) cnt += __builtin_popcountll(__ballot(m4[i] >= mid));
            if (cnt >= top_k) lo = mid;
            else hi = mid - 1u;
        }
        bound = (int32_t)lo - 32768;       // the largest value that at least k lane maxima reach
        // -0 (key -1) and +0 (key 0) are one value: a bound at +0 takes the -0s in as well, and as candidates
        // both carry the key 0
        bound = bound == 0 ? -1 : bound;
    }
    // pieces that hold a logit at or above the bound go to the wave's table; `below` is bound - 1 in both halves
    const bool no_bound = bound <= -32768;  // fewer than k lanes hold anything: no bound this way
    int32_t wc = 0;                         // pieces in the wave's table so far (wave-uniform)
    if (!no_bound) {
        const uint32_t b16 = (uint32_t)(bound - 1) & 0xffffu;
        const uint32_t below = b16 | (b16 << 16);
#pragma unroll
        for (int j = 0; j < ITERS; ++j) {
            const bool hot = pk_max_i16(vm[j], below) != below;
            const unsigned long long hm = __ballot(hot);
            if (hm != 0ull) {
                const uint32_t slot = (uint32_t)wc + rank_in(hm);
                if (hot && slot < (uint32_t)kTileCand) {
                    *reinterpret_cast<u32x4 *>(tk.hot_vec[wave][slot]) = raw[j];
                    tk.hot_pos[wave][slot] = (v0 + j * 64 + lane) * EPV;
                }
                wc += __builtin_popcountll(hm);
            }
        }
    }
    if (lane == 0) tk.hot_n[wave] = no_bound ? kTileCand + 1 : wc;
    __syncthreads();

    // ---------------- every wave: a lane per hot piece takes it apart; how many logits reach the bound
    int32_t nh[NW], nhot = 0;
    bool fall = false;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        nh[w] = tk.hot_n[w];
        fall = fall || nh[w] > kTileCand;
        nhot += nh[w];
    }
    fall = fall || nhot > kTileCand;
    int32_t pkey[EPV];
    int32_t ppos = 0;
    int ncand = 0;
    if (!fall) {
        int w = 0, sl = lane;
#pragma unroll
        for (int q = 0; q < NW - 1; ++q) {
            if (w == q && sl >= nh[q]) { sl -= nh[q]; w = q + 1; }
        }
        const bool have = lane < nhot;
        u32x4 pv = u32x4{kLowest, kLowest, kLowest, kLowest};
        if (have) {
            pv = *reinterpret_cast<const u32x4 *>(tk.hot_vec[w][sl]);
            ppos = tk.hot_pos[w][sl];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            pkey[2 * i] = (int32_t)(pv[i] << 16) >> 16;
            pkey[2 * i + 1] = (int32_t)pv[i] >> 16;
        }
#pragma unroll
        for (int e = 0; e < EPV; ++e) ncand += __builtin_popcountll(__ballot(have && pkey[e] >= bound));
        fall = ncand > kTileCand;
    }
    if (fall) {
        // ties or a flat row: the general selection, then the plain step (every thread of the block)
        __syncthreads();                   // the tables give way to the general path's scratch
        const uint32_t thr_key = radix_threshold<AS_BF16>(sc.radix, row, V, a.temp, top_k, HAS_P ? top_p : 1.f);
        __syncthreads();
        generic_step_row<uint16_t>(a, r, Key<AS_BF16>::from_key(thr_key), sc.gen);
        return;
    }
    if (wave != 0) return;

    // ---------------- one wave: the candidates, one per lane
    {
        int32_t at = 0;
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
            const bool hit = lane < nhot && pkey[e] >= bound;
            const unsigned long long m = __ballot(hit);
            if (hit) {
                const uint32_t slot = (uint32_t)at + rank_in(m);
                tk.ckey[slot] = pkey[e] == -1 ? 0 : pkey[e];
                tk.cidx[slot] = ppos + e;
            }
            at += __builtin_popcountll(m);
        }
        if (lane >= ncand) {
            tk.ckey[lane] = -32768;
            tk.cidx[lane] = 0x7fffffff;
        }
    }
    const bool valid = lane < ncand;
    const int32_t key = tk.ckey[lane];
    const int32_t idx = tk.cidx[lane];
    const float x = key_to_float(key);
    const float ks = a.k;
    const float ref = fmaxf(ceilf(wave_max(valid ? x * ks : -__builtin_inff())), kRefFloor);
    const float w0 = valid ? fast_exp2(fmaf(x, ks, -ref)) : 0.f;
    tk.cw[lane] = (double)w0;
    // pass over the table by key: how many candidates, and how much weight, lie above this one's key.  Every
    // logit at or above the bound is in the table, so ranks in the table are ranks in the row: a candidate is
    // among the k highest (ties at the k-th all stay) if fewer than k keys are above its own; the nucleus keeps
    // it if the weight above its key has not reached top_p of the survivors' total (the group of equal keys
    // that closes the nucleus stays whole).  Groups of four behind the last candidate are skipped.
    typedef double f64x2 __attribute__((ext_vector_type(2)));
    int32_t ngt = 0;
    double above[2] = {0.0, 0.0};
    auto by_key = [&](int g0, int g1) __attribute__((always_inline)) {
#pragma unroll
        for (int g = g0; g < g1; ++g) {
            const i32x4 kj = *reinterpret_cast<const i32x4 *>(&tk.ckey[4 * g]);
            f64x2 wj[2];
            if constexpr (HAS_P) {
                wj[0] = *reinterpret_cast<const f64x2 *>(&tk.cw[4 * g]);
                wj[1] = *reinterpret_cast<const f64x2 *>(&tk.cw[4 * g + 2]);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const bool gt = kj[i] > key;
                ngt += gt ? 1 : 0;
                if constexpr (HAS_P) above[i & 1] = fma(gt ? 1.0 : 0.0, wj[i >> 1][i & 1], above[i & 1]);
            }
        }
    };
    constexpr int kMostGroups = (kTileTopK + 3) / 4;     // what a row without ties at the bound needs
    by_key(0, kMostGroups);
    if (ncand > 4 * kMostGroups) by_key(kMostGroups, kTileCand / 4);
    bool kept = valid && ngt < top_k;
    if constexpr (HAS_P) {
        const double total = wave_sum((double)(kept ? w0 : 0.f));
        kept = kept && !(above[0] + above[1] >= (double)top_p * total);
    }
    const float w = kept ? w0 : 0.f;
    tk.cw[lane] = (double)w;
    const double S = wave_sum((double)w);
    // pass by vocabulary index: the mass before every candidate
    double before[2] = {0.0, 0.0};
    auto by_index = [&](int g0, int g1) __attribute__((always_inline)) {
#pragma unroll
        for (int g = g0; g < g1; ++g) {
            const i32x4 ij = *reinterpret_cast<const i32x4 *>(&tk.cidx[4 * g]);
            const f64x2 wa = *reinterpret_cast<const f64x2 *>(&tk.cw[4 * g]);
            const f64x2 wb = *reinterpret_cast<const f64x2 *>(&tk.cw[4 * g + 2]);
            before[0] = fma(ij[0] < idx ? 1.0 : 0.0, wa[0], before[0]);
            before[1] = fma(ij[1] < idx ? 1.0 : 0.0, wa[1], before[1]);
            before[0] = fma(ij[2] < idx ? 1.0 : 0.0, wb[0], before[0]);
            before[1] = fma(ij[3] < idx ? 1.0 : 0.0, wb[1], before[1]);
        }
    };
    by_index(0, kMostGroups);
    if (ncand > 4 * kMostGroups) by_index(kMostGroups, kTileCand / 4);
    const double bef = before[0] + before[1];
    const double tau = (double)code * S;
    const bool has_weight = kept && w > 0.f;
    unsigned long long sel = __ballot(has_weight && bef <= tau && tau < bef + (double)w);
    if (sel == 0ull) {
        // the code at the very top by rounding: the last kept token of the vocabulary
        int32_t best = has_weight ? idx : -1;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            const int32_t o = __shfl_xor(best, d, 64);
            best = o > best ? o : best;
        }
        sel = __ballot(has_weight && idx == best);
    }
    if (sel == 0ull) {
        // no kept candidate with weight: cannot happen for finite logits; leave a valid row behind
        if (lane == 0) {
            RowOut o;
            o.token = 0;
            o.c_next = rescale_code(0.0, 0.0, 1.0);
            o.prob = 0.f;
            o.f_lo = 0.f;
            write_row(a, r, o);
        }
        return;
    }
    if (lane == (int)__builtin_ctzll(sel)) {
        RowOut o;
        o.token = idx;
        o.c_next = rescale_code(tau, bef, (double)w);
        o.prob = (float)((double)w / S);
        o.f_lo = (float)(bef / S);
        write_row(a, r, o);
    }
}

// ------------------------------------------------------------ nucleus step, single tile
//
// The nucleus alone (no top-k) and the sampling step for bf16 rows of whole, aligned 16-byte pieces that fit one
// tile.  A bf16 logit has one of 65536 values and its weight depends on nothing else, so the mass of a group of
// equal logits is a count times one weight: the kernel counts, it does not add weights per logit.
//   * while the row lands (loads and the look at the finished flag as in the single-tile sampling kernel) every
//     logit goes into a table of counters in LDS, one per stored value in a window of kNucBins values that ends
//     kNucMargin values (six factors of two: a confident row's one large logit is still inside) above the
//     largest logit of the row's first chunks; values of the other sign or below the window go to a counter per
//     lane that nobody reads.  Alongside, the sums of all weights per chunk, against one integer reference per
//     wave, as in the sampling kernel (for the total).
//   * after the barrier: 8 counters per thread become masses (count x weight of that value), a scan over the
//     block finds the first value, from the top, at which the running mass reaches top_p of the total: the keep
//     threshold; the group of equal logits that closes the nucleus stays whole (its counter is one group).
//   * the counters give way to a table of weights, one per kept value: the chunk sums of the kept logits are
//     look-ups and additions, and the search for the code's bucket over them is the sampling kernel's.
// The row stays in registers throughout.  A logit above the window, a nucleus that does not close inside it (it
// would have to reach down by a factor of 2^10 below the first chunks' largest logit, or across zero), sums beyond fp32: the block takes the general
// selection and the plain three-pass step instead.
constexpr int kNucBins = 2048;
#ifndef AS_NUC_AHEAD
#define AS_NUC_AHEAD 4
#endif
constexpr int kNucAhead = AS_NUC_AHEAD;  // groups of four loads requested ahead of the group being counted
constexpr int kNucMargin = 768;

struct TileNucleus {
    __attribute__((aligned(16))) uint32_t hist[kNucBins + 64];
    TileSums sums;
    double wave_tot[kThreads / 64];
    int32_t anchor[kThreads / 64];
    int32_t over[kThreads / 64];
    int32_t pick[kThreads / 64];
};

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pk_min_u16(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b)));
}
__device__ __forceinline__ uint32_t pk_sub_u16(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, (u16x2)(__builtin_bit_cast(u16x2, a) - __builtin_bit_cast(u16x2, b)));
}

template <bool NT>
__global__ __launch_bounds__(kThreads, 4) void nucleus_tile_kernel(StepArgs a, float top_p)
{
    constexpr int DT = AS_BF16;
    constexpr int NW = kTileWaves, ITERS = kTileIters, G = kTileGroup, NG = ITERS / G, EPV = 8;
    constexpr int kShare = ITERS * 64;
    __shared__ union Shared {
        Scratch sc;
        TileNucleus tn;
        __device__ Shared() {}
    } sh;
    Scratch &sc = sh.sc;
    TileNucleus &tn = sh.tn;

    const int64_t r = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    uint32_t fin_word = 0u, fin_at = 0u;
    if (a.finished_in != nullptr) {
        const uint8_t *q = a.finished_in + r;
        fin_at = (uint32_t)(reinterpret_cast<uintptr_t>(q) & 3u);
        fin_word = *reinterpret_cast<const uint32_t *>(q - fin_at);
    }
    const float code = a.codes[r];
    const int64_t src = a.row_ids ? (int64_t)a.row_ids[r] : r;
    const uint16_t *row = reinterpret_cast<const uint16_t *>(a.logits) + src * a.ld;
    const unsigned char *rowb = reinterpret_cast<const unsigned char *>(row);
    const int32_t V = a.V;
    const int32_t nvec = V / EPV;
    const float k = a.k;
    const int32_t v0 = wave * kShare;
    u32x4 raw[ITERS];
    int32_t mych = (nvec - v0 - lane + 63) >> 6;
    mych = mych < 0 ? 0 : (mych > ITERS ? ITERS : mych);
    const bool live = v0 < nvec;
    const bool ragged = v0 + kShare > nvec;
    const unsigned char *base = rowb + (size_t)(live ? v0 : 0) * 16u;
    const uint32_t off0 = (uint32_t)lane * 16u;
    const uint32_t off_last = mych > 0 ? off0 + (uint32_t)(mych - 1) * 1024u : 0u;
    auto request_group = [&](int g) __attribute__((always_inline)) {
        // (ordinary loads where the tensor fits the caches, the non-temporal hint where it is streamed from HBM;
        // each load behind the two vector instructions of its own offset either way)
        if constexpr (NT) {
#pragma unroll
            for (int jj = 0; jj < G; ++jj) {
                uint32_t off = off0 + (uint32_t)(g * G + jj) * 1024u;
                off = off < off_last ? off : off_last;
                raw[g * G + jj] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(base + off));
            }
        } else {
#pragma unroll
            for (int jj = 0; jj < G; ++jj) {
                uint32_t off = off0 + (uint32_t)(g * G + jj) * 1024u;
                off = off < off_last ? off : off_last;
                raw[g * G + jj] = *reinterpret_cast<const u32x4 *>(base + off);
            }
        }
    };
    // the counters start at zero (before anything is loaded: the registers of the row are not free later)
    for (int i = threadIdx.x; i < (kNucBins + 64) / 4; i += kThreads)
        reinterpret_cast<u32x4 *>(tn.hist)[i] = u32x4{0u, 0u, 0u, 0u};
    __builtin_amdgcn_sched_barrier(0);
    // From here to the end of the counting there is one path for every wave, with no branch between the loads
    // and the code that takes them in (the compiler's wait counters are exact only then).  A share past the
    // row's end (mych = 0 in every lane) re-reads the row's first piece and counts it for nothing.
    request_group(0);
    __builtin_amdgcn_sched_barrier(0);
    if (((fin_word >> (8u * fin_at)) & 0xffu) != 0u) {
        if (threadIdx.x == 0) write_finished(a, r);
        return;
    }
#pragma unroll
    for (int g = 1; g < kNucAhead; ++g) request_group(g);
    __builtin_amdgcn_sched_barrier(0);
    f32x4 *const my_sums = reinterpret_cast<f32x4 *>(tn.sums.chunk_sum + wave * ITERS);

    // ---------------- where the window goes: the largest logit of the four waves' first chunks (as a key that
    // orders like the values), and a margin above it
    {
        const uint32_t m2 = pk_max_i16(pk_max_i16(pk_key_bf16(raw[0][0]), pk_key_bf16(raw[0][1])),
                                       pk_max_i16(pk_key_bf16(raw[0][2]), pk_key_bf16(raw[0][3])));
        const int32_t hi = (int32_t)m2 >> 16, lo = (int32_t)(m2 << 16) >> 16;
        const int32_t km = mych > 0 ? (hi > lo ? hi : lo) : -32768;
        const float fm = wave_max((float)(km + 32768));      // (16-bit integers are exact as floats)
        if (lane == 0) tn.anchor[wave] = (int32_t)fm;
    }
    __syncthreads();
    int32_t kb = tn.anchor[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) kb = tn.anchor[w] > kb ? tn.anchor[w] : kb;
    kb = __builtin_amdgcn_readfirstlane(kb) - 32768;
    // A stored value v is counted at e - C, where e = v ^ X falls as the logit rises (X flips the magnitude bits
    // of positive values; negative ones already run that way) and C is e of the window's top.  Values of the
    // other sign give an e - C beyond the window either way.
    const bool positive = kb >= 0;
    int32_t top_raw = kb + kNucMargin;
    top_raw = top_raw > 0x7f7f ? 0x7f7f : top_raw;           // the largest finite value
    int32_t top_mag = (-1 - kb) - kNucMargin;
    top_mag = top_mag < 0 ? 0 : top_mag;
    const uint32_t X = positive ? 0x7fffu : 0u;
    const uint32_t C = positive ? 0x7fffu - (uint32_t)top_raw : (0x8000u | (uint32_t)top_mag);
    bool fall = positive && top_raw < kNucBins - 1;         // a window that would cross zero
    float rw;
    uint32_t emin = 0xffffffffu;
    {
        const uint32_t X2 = X | (X << 16), C2 = C | (C << 16);
        const uint32_t NBL = (uint32_t)(kNucBins + lane) * 0x10001u;
        rw = tile_reference<DT, false, true>(raw[0], k, 0.f, mych);
        const float nr = -rw;
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            if (g + kNucAhead < NG) {
                request_group(g + kNucAhead);
                __builtin_amdgcn_sched_barrier(0);
            }
            float t[G];
#pragma unroll
            for (int jj = 0; jj < G; ++jj) {
                const int j = g * G + jj;
                t[jj] = tile_lane_sum<DT, false>(raw[j], k, nr, 0.f);
                t[jj] = j < mych ? t[jj] : 0.f;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t e = raw[j][i] ^ X2;
                    emin = pk_min_u16(emin, e);
                    uint32_t d = pk_min_u16(pk_sub_u16(e, C2), NBL);
                    d = j < mych ? d : NBL;
                    __hip_atomic_fetch_add(&tn.hist[d & 0xffffu], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    __hip_atomic_fetch_add(&tn.hist[d >> 16], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                }
                // (a piece at a time, the running minimum in this order: work of several pieces interleaved, or
                // a minimum taken as a tree at the end, does not fit the registers)
                asm volatile("" : "+v"(emin));
                __builtin_amdgcn_sched_barrier(0);
            }
            wave_sum4_in_lane63(t[0], t[1], t[2], t[3]);
            if (lane == 63) my_sums[g] = f32x4{t[0], t[1], t[2], t[3]};
        }
    }
    {
        const uint32_t em = min(emin & 0xffffu, emin >> 16);
        const bool above = em < C;                           // a logit above the window's top (or of the other sign)
        const unsigned long long any = __ballot(above);
        if (lane == 0) {
            tn.over[wave] = any != 0ull;
            tn.sums.share_ref[wave] = rw;
        }
    }
    __syncthreads();

    // ---------------- every wave: the total of all weights; masses of the counters; where the nucleus closes
    float R = tn.sums.share_ref[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) {
        R = fmaxf(R, tn.sums.share_ref[w]);
        fall = fall || tn.over[w] != 0;
    }
    fall = fall || tn.over[0] != 0;
    double need = 0.0;
    {
        const float my_ref = tn.sums.share_ref[lane / ITERS];
        const double cv = (double)ldexpf(tn.sums.chunk_sum[lane], shift_of(my_ref, R));
        const double S_all = wave_sum(cv);
        fall = fall || !(S_all < (double)__builtin_inff());
        need = (double)top_p * S_all;
    }
    constexpr int kPer = kNucBins / kThreads;
    double m[kPer], local = 0.0;
    float wv[kPer];
    uint32_t cnt[kPer];
    {
        const u32x4 c0 = reinterpret_cast<const u32x4 *>(tn.hist)[threadIdx.x * 2];
        const u32x4 c1 = reinterpret_cast<const u32x4 *>(tn.hist)[threadIdx.x * 2 + 1];
#pragma unroll
        for (int i = 0; i < 4; ++i) { cnt[i] = c0[i]; cnt[4 + i] = c1[i]; }
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const uint32_t v = ((C + (uint32_t)(threadIdx.x * kPer + i)) ^ X) & 0xffffu;    // the stored value of this counter
            const float w = fast_exp2(fmaf(bits_f32(v << 16), k, -R));
            wv[i] = w;
            m[i] = cnt[i] ? (double)((float)cnt[i] * w) : 0.0;
            local += m[i];
        }
    }
    const double incl = wave_scan_add(local);
    if (lane == 63) tn.wave_tot[wave] = incl;
    __syncthreads();
    double cum = incl;
#pragma unroll
    for (int w = 0; w < NW - 1; ++w) cum += w < wave ? tn.wave_tot[w] : 0.0;
    {
        // the first thread, in the order of the values, whose running mass reaches the goal names the counter
        const unsigned long long hit = __ballot(cum >= need);
        int32_t mine = -1;
        if (hit != 0ull && lane == (int)__builtin_ctzll(hit)) {
            double acc = cum - local;
            int32_t last = -1;
#pragma unroll
            for (int i = 0; i < kPer; ++i) {
                acc += m[i];
                if (cnt[i]) last = threadIdx.x * kPer + i;
                if (mine < 0 && cnt[i] && acc >= need) mine = threadIdx.x * kPer + i;
            }
            if (mine < 0) mine = last;                       // (the two orders of summation differ in the last place)
            tn.pick[wave] = mine;
        }
        if (hit == 0ull && lane == 0) tn.pick[wave] = -1;
    }
    __syncthreads();
    int32_t pick = -1;
#pragma unroll
    for (int w = NW - 1; w >= 0; --w) pick = tn.pick[w] >= 0 ? tn.pick[w] : pick;
    fall = fall || pick < 0;
    if (fall) {
        // the general selection, then the plain step (every thread of the block)
        __syncthreads();
        const uint32_t thr_key = radix_threshold<AS_BF16>(sc.radix, row, V, a.temp, 0, top_p);
        __syncthreads();
        generic_step_row<uint16_t>(a, r, Key<AS_BF16>::from_key(thr_key), sc.gen);
        return;
    }
    const float thr = bits_f32((((C + (uint32_t)pick) ^ X) & 0xffffu) << 16);

    // ---------------- the chunk sums of the kept logits, and the bucket of the code.  The counters give way to
    // the weights of their values against the block's reference R (nothing for the values below the threshold
    // and for the counters outside the window): a kept logit's weight is then a look-up, not an exponential.
    {
        float *const wtab = reinterpret_cast<float *>(tn.hist);
        f32x4 w0, w1;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            w0[i] = threadIdx.x * kPer + i <= pick ? wv[i] : 0.f;
            w1[i] = threadIdx.x * kPer + 4 + i <= pick ? wv[4 + i] : 0.f;
        }
        reinterpret_cast<f32x4 *>(wtab)[threadIdx.x * 2] = w0;
        reinterpret_cast<f32x4 *>(wtab)[threadIdx.x * 2 + 1] = w1;
        if (threadIdx.x < 16) reinterpret_cast<f32x4 *>(wtab + kNucBins)[threadIdx.x] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (lane == 0) tn.sums.share_ref[wave] = R;          // the sums that follow are relative to R in every wave
        __syncthreads();
        const uint32_t X2 = X | (X << 16), C2 = C | (C << 16);
        // everything below the threshold reads one of the 64 zeros that follow it in the table, each lane its
        // own: consecutive words, no bank conflicts (most of the row is below the threshold)
        const uint32_t NBL = (uint32_t)(pick + 1 + lane) * 0x10001u;
        // (the row's registers made opaque: otherwise every counter index of the first pass is kept, in memory,
        // for this one)
#pragma unroll
        for (int j = 0; j < ITERS; ++j)
            asm volatile("" : "+v"(raw[j][0]), "+v"(raw[j][1]), "+v"(raw[j][2]), "+v"(raw[j][3]));
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            float t[G];
#pragma unroll
            for (int jj = 0; jj < G; ++jj) {
                const int j = g * G + jj;
                float w[EPV];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    uint32_t d = pk_min_u16(pk_sub_u16(raw[j][i] ^ X2, C2), NBL);
                    d = j < mych ? d : NBL;
                    w[2 * i] = wtab[d & 0xffffu];
                    w[2 * i + 1] = wtab[d >> 16];
                }
                t[jj] = vec_sum<EPV>(w);
            }
            wave_sum4_in_lane63(t[0], t[1], t[2], t[3]);
            if (lane == 63) my_sums[g] = f32x4{t[0], t[1], t[2], t[3]};
        }
    }
    __syncthreads();
    tile_select<DT, true>(a, r, code, thr, raw, R, mych, ragged, v0, lane, wave, tn.sums, sc.gen);
}

template <int DT>
void launch_resident(as_ctx *ctx, const void *logits, int64_t rows, int64_t ld, const uint8_t *finished_in,
                     const int32_t *row_ids, float temp, int32_t top_k, float top_p, float *thr_out, bool has_k,
                     bool has_p)
{
    const dim3 grid((unsigned)rows), block(kThreads);
    if (has_k && has_p)
        launch(ctx, kKernelThreshold, threshold_resident_kernel<DT, true, true>, grid, block, 0, logits, ld, ctx->V,
               finished_in, row_ids, temp, top_k, top_p, thr_out, StepArgs{});
    else if (has_k)
        launch(ctx, kKernelThreshold, threshold_resident_kernel<DT, true, false>, grid, block, 0, logits, ld, ctx->V,
               finished_in, row_ids, temp, top_k, top_p, thr_out, StepArgs{});
    else
        launch(ctx, kKernelThreshold, threshold_resident_kernel<DT, false, true>, grid, block, 0, logits, ld, ctx->V,
               finished_in, row_ids, temp, top_k, top_p, thr_out, StepArgs{});
}

// top-k (optionally followed by the nucleus), or the nucleus alone on bf16 rows, and the sampling step in one
// launch; false if the shape does not qualify (then the caller runs the threshold kernel and the step kernel one after the other)
bool launch_topk_step(as_ctx *ctx, const StepArgs &args, int32_t top_k, float top_p, as_status *st)
{
    const size_t esz = ctx->dtype == AS_BF16 ? 2 : 4;
    const StepArgs &a = args;
    const bool nt = stream_rows(a.rows, a.ld, esz);
    const bool has_k = top_k > 0 && top_k < ctx->V, has_p = top_p > 0.f && top_p < 1.f;
    const bool nucleus_only = !has_k && has_p && ctx->dtype == AS_BF16;
    if ((ctx->thr_path != 0 && ctx->thr_path != 2) || !(has_k || nucleus_only) || top_k > kThreads / 2 || ctx->V > 32768 ||
        reinterpret_cast<uintptr_t>(a.logits) % 16 != 0 || (a.ld * esz) % 16 != 0)
        return false;
    *st = AS_OK;
    if (a.rows == 0) return true;
    const dim3 grid((unsigned)a.rows), block(kThreads);
    if (has_k && top_k <= kTileTopK && ctx->dtype == AS_BF16 && ctx->V % 8 == 0 && ctx->thr_path != 2) {
        if (has_p && nt) launch(ctx, kKernelStep, topk_tile_kernel<true, true>, grid, block, 0, a, top_k, top_p);
        else if (has_p) launch(ctx, kKernelStep, topk_tile_kernel<true, false>, grid, block, 0, a, top_k, top_p);
        else if (nt) launch(ctx, kKernelStep, topk_tile_kernel<false, true>, grid, block, 0, a, top_k, top_p);
        else launch(ctx, kKernelStep, topk_tile_kernel<false, false>, grid, block, 0, a, top_k, top_p);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) *st = hip_fail(ctx, e, "top-k step launch");
        return true;
    }
    if (nucleus_only && ctx->V % 8 == 0 && ctx->thr_path != 2 && a.k <= kTileMaxScale) {
        if (nt) launch(ctx, kKernelStep, nucleus_tile_kernel<true>, grid, block, 0, a, top_p);
        else launch(ctx, kKernelStep, nucleus_tile_kernel<false>, grid, block, 0, a, top_p);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) *st = hip_fail(ctx, e, "nucleus step launch");
        return true;
    }
    if (nucleus_only) {
        launch(ctx, kKernelStep, threshold_resident_kernel<AS_BF16, false, true, true>, grid, block, 0, a.logits, a.ld,
               ctx->V, a.finished_in, a.row_ids, a.temp, top_k, top_p, (float *)nullptr, a);
    } else if (ctx->dtype == AS_BF16) {
        if (has_p)
            launch(ctx, kKernelStep, threshold_resident_kernel<AS_BF16, true, true, true>, grid, block, 0, a.logits, a.ld,
                   ctx->V, a.finished_in, a.row_ids, a.temp, top_k, top_p, (float *)nullptr, a);
        else
            launch(ctx, kKernelStep, threshold_resident_kernel<AS_BF16, true, false, true>, grid, block, 0, a.logits, a.ld,
                   ctx->V, a.finished_in, a.row_ids, a.temp, top_k, top_p, (float *)nullptr, a);
    } else {
        if (has_p)
            launch(ctx, kKernelStep, threshold_resident_kernel<AS_F32, true, true, true>, grid, block, 0, a.logits, a.ld,
                   ctx->V, a.finished_in, a.row_ids, a.temp, top_k, top_p, (float *)nullptr, a);
        else
            launch(ctx, kKernelStep, threshold_resident_kernel<AS_F32, true, false, true>, grid, block, 0, a.logits, a.ld,
                   ctx->V, a.finished_in, a.row_ids, a.temp, top_k, top_p, (float *)nullptr, a);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) *st = hip_fail(ctx, e, "fused top-k step launch");
    return true;
}

as_status launch_threshold(as_ctx *ctx, const void *logits, int64_t rows, int64_t ld,
                           const uint8_t *finished_in, const int32_t *row_ids, float temp,
                           int32_t top_k, float top_p, float *thr_out)
{
    if (rows == 0) return AS_OK;
    const size_t esz = ctx->dtype == AS_BF16 ? 2 : 4;
    const bool has_k = top_k > 0 && top_k < ctx->V, has_p = top_p > 0.f && top_p < 1.f;
    // resident path: the row fits the block's registers, is read in 16-byte pieces, k at most half the thread
    // count (the k-th largest thread maximum must leave only a few hundred logits above it)
    const bool resident = ctx->thr_path != 1 && (has_k || has_p) && ctx->V <= 32768 &&
                          reinterpret_cast<uintptr_t>(logits) % 16 == 0 && (ld * esz) % 16 == 0 &&
                          (!has_k || top_k <= kThreads / 2);
    // what the resident kernel does not take goes to the streamed one (any row length and stride, any k)
    const bool streamed = !resident && ctx->thr_path != 1 && (has_k || has_p) &&
                          reinterpret_cast<uintptr_t>(logits) % esz == 0;
    if (streamed) {
        const dim3 grid((unsigned)rows), block(kThreads);
        const int kmode = !has_k ? 0 : top_k <= kThreads / 2 ? 1 : 2;
#define AS_STREAM_LAUNCH1(DT_, KM_, HP_)                                                                        \
    launch(ctx, kKernelThreshold, threshold_stream_kernel<DT_, KM_, HP_>, grid, block, 0, logits, ld, ctx->V,   \
           finished_in, row_ids, temp, top_k, top_p, thr_out)
#define AS_STREAM_LAUNCH(DT_)                                                                                    \
    do {                                                                                                         \
        if (kmode == 0) AS_STREAM_LAUNCH1(DT_, 0, true);                                                         \
        else if (kmode == 1 && has_p) AS_STREAM_LAUNCH1(DT_, 1, true);                                           \
        else if (kmode == 1) AS_STREAM_LAUNCH1(DT_, 1, false);                                                   \
        else if (has_p) AS_STREAM_LAUNCH1(DT_, 2, true);                                                         \
        else AS_STREAM_LAUNCH1(DT_, 2, false);                                                                   \
    } while (0)
        if (ctx->dtype == AS_BF16) AS_STREAM_LAUNCH(AS_BF16);
        else AS_STREAM_LAUNCH(AS_F32);
#undef AS_STREAM_LAUNCH1
#undef AS_STREAM_LAUNCH
    } else if (resident) {
        if (ctx->dtype == AS_BF16)
            launch_resident<AS_BF16>(ctx, logits, rows, ld, finished_in, row_ids, temp, top_k, top_p, thr_out, has_k,
                                     has_p);
        else
            launch_resident<AS_F32>(ctx, logits, rows, ld, finished_in, row_ids, temp, top_k, top_p, thr_out, has_k,
                                    has_p);
    } else if (ctx->dtype == AS_BF16) {
        launch(ctx, kKernelThreshold, threshold_kernel<AS_BF16>, dim3((unsigned)rows), dim3(kThreads), 0,
               logits, ld, ctx->V, finished_in, row_ids, temp, top_k, top_p, thr_out);
    } else {
        launch(ctx, kKernelThreshold, threshold_kernel<AS_F32>, dim3((unsigned)rows), dim3(kThreads), 0,
               logits, ld, ctx->V, finished_in, row_ids, temp, top_k, top_p, thr_out);
    }
    AS_HIP_TRY(ctx, hipGetLastError());
    return AS_OK;
}

}  // namespace as
