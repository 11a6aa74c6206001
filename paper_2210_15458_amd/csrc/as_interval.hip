// Encode direction: the interval of a given token sequence (Sec. 4.1, the
// codebook recursion; Sec. 3.1 for one token's sub-interval).  Per step and row,
// with the row's kept, tempered softmax in vocabulary order,
//     lo    += width * F(token - 1)      (mass of the tokens before it)
//     width *= P(token)
// so that after the last step the codes in [lo, lo + width) are exactly the ones
// that decode to the sequence.  The per-row pass is the one of the sampling step
// with the search replaced by a lookup: weights exp2(x*k - ref) in fp32 against an
// integer reference ref >= max x*k, sums in fp64.  lo and width are fp64 state.
#include <type_traits>

#include "as_common.hpp"
#include "as_row.hpp"
#include "as_tile.hpp"

namespace as {
namespace {

constexpr int kThreads = 256;


// g(v0, x, first, n) over the row's logits in runs: elements first..n-1 of x are logits v0+first..v0+n-1 of the
// row, each logit of the row exactly once per thread block.  The row is read as the whole 16-byte pieces it
// touches, four in flight per thread; only the pieces at the row's two ends have first > 0 or n < 8 (4).
template <class T, class G>
__device__ __forceinline__ void for_row(const T *row, int32_t V, G g)
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    constexpr int EPP = 16 / (int)sizeof(T);
    const int32_t shift = (int32_t)((reinterpret_cast<uintptr_t>(row) & 15u) / sizeof(T));
    const u32x4 *const pieces = reinterpret_cast<const u32x4 *>(row - shift);
    const int32_t vend = V + shift;
    const int32_t npieces = (vend + EPP - 1) / EPP;
    for (int32_t base = threadIdx.x; base < npieces; base += 4 * kThreads) {
        u32x4 w[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int32_t piece = base + u * kThreads;
            w[u] = piece < npieces ? __builtin_nontemporal_load(pieces + piece) : u32x4{0, 0, 0, 0};
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int32_t piece = base + u * kThreads;
            if (piece >= npieces) break;
            float x[EPP];
#pragma unroll
            for (int e = 0; e < EPP; ++e) {
                if constexpr (sizeof(T) == 2) {
                    const uint32_t word = w[u][e >> 1];
                    x[e] = __builtin_bit_cast(float, (e & 1) ? (word & 0xffff0000u) : (word << 16));
                } else {
                    const uint32_t word = w[u][e];
                    x[e] = __builtin_bit_cast(float, word);
                }
            }
            const int32_t left = vend - piece * EPP;
            g(piece * EPP - shift, x, piece == 0 ? shift : 0, left < EPP ? left : EPP,
              std::integral_constant<int, EPP>{});
        }
    }
}

// three block-wide sums at once, each in a fixed order: lanes by the wave scan, then the waves in index order
__device__ __forceinline__ void block_sum3(double &a, double &b, double &c, double *scratch)
{
    a = wave_sum(a);
    b = wave_sum(b);
    c = wave_sum(c);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) {
        scratch[wave] = a;
        scratch[kThreads / 64 + wave] = b;
        scratch[2 * (kThreads / 64) + wave] = c;
    }
    __syncthreads();
    a = b = c = 0.0;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) {
        a += scratch[w];
        b += scratch[kThreads / 64 + w];
        c += scratch[2 * (kThreads / 64) + w];
    }
}

// what a row's sums do to its interval (one thread)
__device__ __forceinline__ void narrow_interval(const IntervalArgs &a, int64_t r, int32_t tok, double all, double before,
                                                double at)
{
    // a token outside the vocabulary or outside the kept set has probability zero
    const double f_lo = all > 0.0 ? before / all : 0.0;
    const double p = (all > 0.0 && tok >= 0 && tok < a.V) ? at / all : 0.0;
    const double w = a.width[r];
    a.lo[r] += w * f_lo;
    a.width[r] = w * p;
    if (a.finished_out) a.finished_out[r] = (a.eos_id >= 0 && tok == a.eos_id) ? 1 : 0;
    if (a.prev_out) a.prev_out[r] = (tok >= 0 && tok < a.V) ? tok : 0;
}

// One row by a block of 256 threads, any alignment, any V, one pass over memory: every thread keeps an integer
// reference that follows the largest logit it has seen (see below).  Every thread of the block must call it.
template <class T>
__device__ __forceinline__ void interval_row(const IntervalArgs &a, int64_t r, int32_t tok, double *scratch,
                                             float *fscratch)
{
    const int64_t src = a.row_ids ? (int64_t)a.row_ids[r] : r;
    const T *row = reinterpret_cast<const T *>(a.logits) + src * a.ld;
    const float thr = a.thr ? a.thr[r] : -__builtin_inff();
    const float k = a.k;

    auto each_run = [&](auto g) __attribute__((always_inline)) { for_row<T>(row, a.V, g); };

    // a run as the sums see it: what is cut off by the threshold or lies outside the row counts as -inf
    // (weight exactly 0); whole runs of an untruncated row, nearly all of them, pass through untouched
    const bool cut = a.thr != nullptr;
    auto kept = [&](const float *x, int first, int n, auto cap, float *y) __attribute__((always_inline)) {
        constexpr int E = decltype(cap)::value;
        if (!cut && first == 0 && n == E) {
#pragma unroll
            for (int e = 0; e < E; ++e) y[e] = x[e];
        } else {
#pragma unroll
            for (int e = 0; e < E; ++e) y[e] = (e >= first && e < n && x[e] >= thr) ? x[e] : -__builtin_inff();
        }
    };

    // per run: fp32 sum of its (at most 8) weights in order, then one fp64 add per total; only the one run
    // that holds the token looks at single weights
    double all = 0.0, before = 0.0, at = 0.0;
    auto add_run = [&](int32_t v0, const float *y, float nref, auto cap) __attribute__((always_inline)) {
        constexpr int E = decltype(cap)::value;
        float w[E];
        float s_all = 0.f;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            w[e] = __builtin_amdgcn_exp2f(fmaf(y[e], k, nref));
            s_all += w[e];
        }
        const double d = (double)s_all;
        all += d;
        if (v0 + E <= tok) {
            before += d;
        } else if (v0 <= tok) {
            float s_before = 0.f;
#pragma unroll
            for (int e = 0; e < E; ++e) {
                s_before += v0 + e < tok ? w[e] : 0.f;
                if (v0 + e == tok) at = (double)w[e];
            }
            before += (double)s_before;
        }
    };
    {
        // One pass over memory: every thread keeps an integer reference that follows the largest logit it has
        // seen; when it rises, what the thread has summed so far shrinks by an exact power of two.  At the end
        // the threads are brought to the block's reference the same way.
        float ref = -100000.f;
        auto rescale = [&](float to) __attribute__((always_inline)) {
            const int down = (int)fmaxf(ref - to, -2000.f);
            all = ldexp(all, down);
            before = ldexp(before, down);
            at = ldexp(at, down);
            ref = to;
        };
        each_run([&](int32_t v0, const float *x, int first, int n, auto cap) __attribute__((always_inline)) {
            constexpr int E = decltype(cap)::value;
            float y[E];
            kept(x, first, n, cap, y);
            float pm = y[0];
#pragma unroll
            for (int e = 1; e < E; ++e) pm = fmaxf(pm, y[e]);
            const float want = fmaxf(ceilf(pm * k), ref);
            if (want > ref) rescale(want);
            add_run(v0, y, -ref, cap);
        });
        float top = wave_max(ref);
        if ((threadIdx.x & 63) == 0) fscratch[threadIdx.x >> 6] = top;
        __syncthreads();
        top = fscratch[0];
#pragma unroll
        for (int w = 1; w < kThreads / 64; ++w) top = fmaxf(top, fscratch[w]);
        rescale(top);
    }
    block_sum3(all, before, at, scratch);
    if (threadIdx.x == 0) narrow_interval(a, r, tok, all, before, at);
}

template <class T>
__global__ __launch_bounds__(kThreads) void interval_kernel(IntervalArgs a)
{
    __shared__ double scratch[3 * (kThreads / 64)];
    __shared__ float fscratch[kThreads / 64];
    const int64_t r = blockIdx.x;
    const int32_t tok = a.tokens[r * a.tok_stride];
    if (a.finished_in != nullptr && a.finished_in[r] != 0) {
        // past its EOS: the position is padding and does not narrow the interval
        if (threadIdx.x == 0) {
            if (a.finished_out) a.finished_out[r] = 1;
            if (a.prev_out) a.prev_out[r] = a.eos_id;
        }
        return;
    }
    interval_row<T>(a, r, tok, scratch, fscratch);
}

// Rows of whole, aligned vectors that fit one tile (the headline shape): the single-tile sampling kernel with
// the search replaced by a look-up.  Same loads, same chunk sums against one integer reference per wave, one
// barrier; then every wave scans the 64 chunk sums (fp64) for the total and the mass before the token's chunk,
// and the wave that holds the token's chunk adds the lanes before it and the elements before it.  Sums that
// leave fp32 against a first-chunk reference send the block to the one-pass routine above.
template <int DT, bool HAS_THR, bool NT>
__global__ __launch_bounds__(kThreads, 4) void interval_tile_kernel(IntervalArgs a)
{
    using T = typename Elem<DT>::T;
    constexpr int EPV = Elem<DT>::kPerVec;
    constexpr int NW = kTileWaves, ITERS = kTileIters, G = kTileGroup, NG = ITERS / G;
    constexpr int kShare = ITERS * 64;
    __shared__ TileSums ts;
    __shared__ double scratch[3 * (kThreads / 64)];
    __shared__ float fscratch[kThreads / 64];

    const int64_t r = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint32_t fin_word = 0u, fin_at = 0u;
    if (a.finished_in != nullptr) {
        const uint8_t *q = a.finished_in + r;
        fin_at = (uint32_t)(reinterpret_cast<uintptr_t>(q) & 3u);
        fin_word = *reinterpret_cast<const uint32_t *>(q - fin_at);
    }
    const int32_t tok = a.tokens[r * a.tok_stride];
    float thr = -__builtin_inff();
    if constexpr (HAS_THR) thr = a.thr[r];
    const int64_t src = a.row_ids ? (int64_t)a.row_ids[r] : r;
    const unsigned char *rowb =
        reinterpret_cast<const unsigned char *>(reinterpret_cast<const T *>(a.logits) + src * a.ld);
    const int32_t nvec = a.V / EPV;
    const float k = a.k;
    const int32_t v0 = wave * kShare;
    u32x4 raw[ITERS];
    float rw = kRefFloor;
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
        // past its EOS: the position is padding and does not narrow the interval
        if (threadIdx.x == 0) {
            if (a.finished_out) a.finished_out[r] = 1;
            if (a.prev_out) a.prev_out[r] = a.eos_id;
        }
        return;
    }
    f32x4 *const my_sums = reinterpret_cast<f32x4 *>(ts.chunk_sum + wave * ITERS);
    auto stream = [&](auto ragged_c) __attribute__((always_inline)) {
        constexpr bool RAGGED = decltype(ragged_c)::value;
#pragma unroll
        for (int g = 1; g < NG; ++g) request_group(g);
        __builtin_amdgcn_sched_barrier(0);
        rw = tile_reference<DT, HAS_THR, RAGGED>(raw[0], k, thr, mych);
        tile_chunk_sums<DT, HAS_THR, RAGGED>(raw, k, rw, thr, mych, lane, my_sums);
    };
    if (live) {
        if (!ragged) stream(std::false_type{});
        else stream(std::true_type{});
    } else {
#pragma unroll
        for (int j = 0; j < ITERS; ++j) raw[j] = u32x4{0u, 0u, 0u, 0u};
        if (lane < NG) my_sums[lane] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    if (lane == 0) ts.share_ref[wave] = rw;
    __syncthreads();

    float R = ts.share_ref[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) R = fmaxf(R, ts.share_ref[w]);
    const float my_ref = ts.share_ref[lane / ITERS];
    const double cv = (double)ldexpf(ts.chunk_sum[lane], shift_of(my_ref, R));
    const double cincl = wave_scan_add(cv);
    const double S = read_lane(cincl, 63);
    if (!(S < (double)__builtin_inff())) {
        interval_row<T>(a, r, tok, scratch, fscratch);
        return;
    }
    if (tok < 0 || tok >= a.V) {
        // outside the vocabulary: probability zero, everything (or nothing) before it
        if (threadIdx.x == 0) narrow_interval(a, r, tok, S, tok < 0 ? 0.0 : S, 0.0);
        return;
    }
    const int32_t vi = tok / EPV, el = tok % EPV;
    const int ch = vi >> 6, ln = vi & 63;
    if (wave != ch / ITERS) return;
    const double run = read_lane(cincl - cv, ch);
    const int shf = shift_of(rw, R);
    const int cj = ch % ITERS;
    u32x4 hv;
    with_uniform_index<0, ITERS>(cj, [&](auto c_c) __attribute__((always_inline)) {
        uint32_t w0 = raw[decltype(c_c)::value][0], w1 = raw[decltype(c_c)::value][1],
                 w2 = raw[decltype(c_c)::value][2], w3 = raw[decltype(c_c)::value][3];
        asm volatile("" : "+v"(w0), "+v"(w1), "+v"(w2), "+v"(w3));
        hv = u32x4{w0, w1, w2, w3};
    });
    float cl = tile_lane_sum<DT, HAS_THR>(hv, k, -rw, thr);
    if (ragged) cl = cj < mych ? cl : 0.f;
    const double lv = (double)ldexpf(cl, shf);
    const double scan2 = wave_scan_add(lv);
    const double before_lane = read_lane(scan2 - lv, ln) + run;
    // The total with this chunk and this lane taken the way `before` takes them (fp64 sums of the lane sums
    // and of the weights, where S has an fp32 wave sum and an fp32 lane sum): the mass before the token plus
    // its own can then not exceed the total by rounding, and nested intervals stay nested.
    const double S_rest = (S - read_lane(cv, ch)) + (read_lane(scan2, 63) - lv);
    if (lane != ln) return;
    float x[EPV];
    unpack<DT>(hv, x);
    double before = before_lane, at = 0.0, mine = 0.0;
#pragma unroll
    for (int i = 0; i < EPV; ++i) {
        float e = fast_exp2(fmaf(x[i], k, -rw));
        if constexpr (HAS_THR) e = (x[i] >= thr) ? e : 0.f;
        const double ed = (double)ldexpf(e, shf);
        mine += ed;
        before += i < el ? ed : 0.0;
        at = i == el ? ed : at;
    }
    narrow_interval(a, r, tok, S_rest + mine, before, at);
}

__global__ void interval_init_kernel(int32_t B, int32_t N, const int32_t *prompts, double *lo, double *width,
                                     int32_t *prev, uint8_t *finished)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)B * N) return;
    lo[idx] = 0.0;
    width[idx] = 1.0;
    prev[idx] = prompts[idx / N];
    finished[idx] = 0;
}

}  // namespace

as_status launch_interval(as_ctx *ctx, const IntervalArgs &args)
{
    if (args.rows == 0) return AS_OK;
    const IntervalArgs &a = args;
    const dim3 grid((unsigned)a.rows), block(kThreads);
    const size_t esz = a.dtype == AS_BF16 ? 2 : 4;
    const bool nt = stream_rows(a.rows, a.ld, esz);
    const int epv = (int)(16 / esz);
    const bool tile = a.V % epv == 0 && a.V / epv <= kTileWaves * kTileIters * 64 &&
                      reinterpret_cast<uintptr_t>(a.logits) % 16 == 0 && (a.ld * (int64_t)esz) % 16 == 0 &&
                      ctx->step_shape == 0 && a.k <= kTileMaxScale;
    if (tile) {
#define AS_INTERVAL_TILE(DT_)                                                                                   \
    do {                                                                                                        \
        if (a.thr && nt) launch(ctx, kKernelInterval, interval_tile_kernel<DT_, true, true>, grid, block, 0, a);   \
        else if (a.thr) launch(ctx, kKernelInterval, interval_tile_kernel<DT_, true, false>, grid, block, 0, a);   \
        else if (nt) launch(ctx, kKernelInterval, interval_tile_kernel<DT_, false, true>, grid, block, 0, a);      \
        else launch(ctx, kKernelInterval, interval_tile_kernel<DT_, false, false>, grid, block, 0, a);             \
    } while (0)
        if (a.dtype == AS_BF16) AS_INTERVAL_TILE(AS_BF16);
        else AS_INTERVAL_TILE(AS_F32);
#undef AS_INTERVAL_TILE
    } else if (a.dtype == AS_BF16) {
        launch(ctx, kKernelInterval, interval_kernel<uint16_t>, grid, block, 0, a);
    } else {
        launch(ctx, kKernelInterval, interval_kernel<float>, grid, block, 0, a);
    }
    AS_HIP_TRY(ctx, hipGetLastError());
    return AS_OK;
}

as_status launch_interval_init(as_ctx *ctx, int32_t B, int32_t N, const int32_t *prompts, double *lo,
                               double *width, int32_t *prev, uint8_t *finished)
{
    const int64_t n = (int64_t)B * N;
    if (n == 0) return AS_OK;
    hipLaunchKernelGGL(interval_init_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, ctx->stream, B, N,
                       prompts, lo, width, prev, finished);
    AS_HIP_TRY(ctx, hipGetLastError());
    return AS_OK;
}

}  // namespace as
