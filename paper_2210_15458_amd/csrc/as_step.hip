// Fused arithmetic-sampling step for gfx950: temperature, optional keep
// threshold, softmax, vocabulary-order cumulative sums, interval search and code
// rescale (Algorithm 1 of Sec. 4.1, one loop body) in ONE pass over each logits
// row.  Nothing but the row itself is read from HBM and only O(1) values per
// row are written.
//
// Shape of the computation (one workgroup per row, NW waves):
//   * A row is cut into 16-byte vectors.  A "tile" is NW*ITERS*64 vectors; wave
//     w of the block owns ITERS consecutive 1-KiB chunks of it, lane l one
//     vector of each chunk, so every wave load is one contiguous KiB and the
//     vocabulary order is tile > wave > chunk > lane > element.
//   * Each lane turns a vector into  s = sum_i exp2(x_i*k - r)  as soon as that
//     vector lands, with k = log2(e)/temp and r an INTEGER >= max_i x_i*k chosen
//     per lane and chunk.  Integer references make every later rescale an exact
//     multiplication by a power of two (ldexp), so partial sums taken against
//     different references combine without rounding and without a second exp.
//   * Per chunk the wave adds its 64 lane sums (DPP scan) into a segment sum and
//     leaves it in LDS; after one barrier every wave scans the segment table in
//     fp64, finds the segment whose running sum crosses c*S, and the wave that
//     owns it finishes: lane sums -> lane, element sums -> token.  Its vectors
//     are still in registers when the row is a single tile; otherwise the one
//     hit vector per lane is read again (16 B per lane, normally an L2 hit).
#include <type_traits>
#include <utility>

#include "as_common.hpp"

#ifndef AS_STEP_DEPTH
#define AS_STEP_DEPTH 6
#endif
#ifndef AS_WAVE_PD
#define AS_WAVE_PD 4
#endif

namespace as {
namespace {

constexpr float kRefFloor = -100000.f;  // reference of a chunk that holds only -inf
constexpr float kMinShift = -300.f;     // 2^-300 is 0 in fp32: clamp before float->int

template <int DT> struct Elem;
template <> struct Elem<AS_F32> {
    using T = float;
    static constexpr int kPerVec = 4;
    static constexpr uint32_t kNegInfWord = 0xff800000u;
};
template <> struct Elem<AS_BF16> {
    using T = uint16_t;
    static constexpr int kPerVec = 8;
    static constexpr uint32_t kNegInfWord = 0xff80ff80u;
};

struct Vec {
    uint32_t w[4];
};

__device__ __forceinline__ float bits_f32(uint32_t b) { return __builtin_bit_cast(float, b); }

template <int DT>
__device__ __forceinline__ void unpack(const Vec &v, float *x)
{
    if constexpr (DT == AS_BF16) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[2 * i] = bits_f32(v.w[i] << 16);
            x[2 * i + 1] = bits_f32(v.w[i] & 0xffff0000u);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) x[i] = bits_f32(v.w[i]);
    }
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Vector `vi` of a row, element by element.  Elements at or beyond V read as
// -inf (probability 0).  Used for rows that do not start on 16 bytes and for
// the ragged end of a row.
template <int DT>
__device__ __noinline__ Vec load_vec_slow(const typename Elem<DT>::T *row, int64_t vi, int32_t V)
{
    const int64_t base = vi * Elem<DT>::kPerVec;
    Vec v;
#pragma unroll
    for (int i = 0; i < 4; ++i) v.w[i] = Elem<DT>::kNegInfWord;
    if (base < V) {
        if constexpr (DT == AS_BF16) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (base + i < V) {
                    const uint32_t h = row[base + i];
                    const int sh = (i & 1) * 16;
                    v.w[i >> 1] = (v.w[i >> 1] & ~(0xffffu << sh)) | (h << sh);
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (base + i < V) v.w[i] = __builtin_bit_cast(uint32_t, row[base + i]);
        }
    }
    return v;
}

// One whole, 16-byte aligned vector (no bounds check: the caller has shown it is inside the row).
template <int DT>
__device__ __forceinline__ Vec load_vec_full(const typename Elem<DT>::T *p)
{
    // streamed once: non-temporal, so the row does not push other data out of L2
    const u32x4 q = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
    Vec v;
    v.w[0] = q[0]; v.w[1] = q[1]; v.w[2] = q[2]; v.w[3] = q[3];
    return v;
}

// Any vector index: whole vectors below nfull (the number of whole, aligned
// vectors of the row; 0 for a row that does not start on 16 bytes) as one load,
// the rest element by element.
template <int DT>
__device__ __forceinline__ Vec load_vec_any(const typename Elem<DT>::T *row, int64_t vi, int32_t V, int64_t nfull)
{
    if (vi < nfull) return load_vec_full<DT>(row + vi * Elem<DT>::kPerVec);
    return load_vec_slow<DT>(row, vi, V);
}

// exp2 straight on the hardware instruction (no denormal fix-up: results below
// 2^-126 may flush to zero, which is far below anything that can matter here)
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Three-operand maximum as one instruction.  (fmaxf on values that come from
// bit casts makes the compiler quiet possible signalling NaNs first, one extra
// instruction per operand; NaN logits are outside the contract anyway.)
__device__ __forceinline__ float max3(float a, float b, float c)
{
    float d;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    return d;
}

// One vector -> its EPV weights e_i = exp2(x_i*k - r) and their integer reference r.
template <int DT, bool HAS_THR>
__device__ __forceinline__ float chunk_weights(const Vec &v, float k, float thr, float *e)
{
    constexpr int EPV = Elem<DT>::kPerVec;
    float x[EPV];
    unpack<DT>(v, x);
    if constexpr (HAS_THR) {
#pragma unroll
        for (int i = 0; i < EPV; ++i) x[i] = (x[i] >= thr) ? x[i] : -__builtin_inff();
    }
    float m;
    if constexpr (EPV == 8) m = max3(max3(max3(x[0], x[1], x[2]), x[3], x[4]), max3(x[5], x[6], x[7]), x[5]);
    else m = max3(max3(x[0], x[1], x[2]), x[3], x[3]);
    const float r = fmaxf(ceilf(m * k), kRefFloor);
    const float nr = -r;
#pragma unroll
    for (int i = 0; i < EPV; ++i) e[i] = fast_exp2(fmaf(x[i], k, nr));
    return r;
}

template <int DT, bool HAS_THR>
__device__ __forceinline__ float chunk_sum(const Vec &v, float k, float thr, float &r)
{
    constexpr int EPV = Elem<DT>::kPerVec;
    float e[EPV];
    r = chunk_weights<DT, HAS_THR>(v, k, thr, e);
    if constexpr (EPV == 8)
        return ((e[0] + e[1]) + (e[2] + e[3])) + ((e[4] + e[5]) + (e[6] + e[7]));
    else
        return (e[0] + e[1]) + (e[2] + e[3]);
}

__device__ __forceinline__ int shift_of(float r, float R) { return (int)fmaxf(r - R, kMinShift); }

constexpr int kGroup = 4;               // chunks of a lane that share one reference
constexpr int kDepth = AS_STEP_DEPTH;   // loads per lane kept in flight

template <int DT, int NW, int ITERS, int OCC, bool ALIGNED, bool HAS_THR>
__global__ __launch_bounds__(NW * 64, OCC) void step_kernel(StepArgs a, int ntiles)
{
    using T = typename Elem<DT>::T;
    constexpr int EPV = Elem<DT>::kPerVec;
    constexpr int64_t kTileVecs = (int64_t)NW * ITERS * 64;
    constexpr int G = ITERS < kGroup ? ITERS : kGroup;
    constexpr int NG = ITERS / G;
    static_assert(ITERS % G == 0 && ITERS <= 64, "chunks per wave must split into whole groups");

    extern __shared__ float smem[];
    const int nent = ntiles * NW;          // (tile, wave) shares of the row, in vocabulary order
    float *ent_sum = smem;                 // [nent]  sum of a share, relative to its reference
    float *ent_ref = smem + nent;          // [nent]  integer reference of the share

    const int64_t r = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    if (a.finished_in != nullptr && a.finished_in[r] != 0) {
        // finished sequence: padding after EOS (Sec. 3.3); the code stops moving
        if (threadIdx.x == 0) {
            a.tokens_out[r * a.tok_stride] = a.eos_id;
            a.codes_out[r] = a.codes[r];
            if (a.finished_out) a.finished_out[r] = 1;
            if (a.prob_out) a.prob_out[r] = 1.f;
            if (a.flo_out) a.flo_out[r] = 0.f;
            if (a.prev_out) a.prev_out[r] = a.eos_id;
        }
        return;
    }

    const int64_t src = a.row_ids ? (int64_t)a.row_ids[r] : r;
    const T *row = reinterpret_cast<const T *>(a.logits) + src * a.ld;
    const int32_t V = a.V;
    const int64_t nfull = ALIGNED ? (int64_t)(V / EPV) : 0;
    const bool whole_vectors = ALIGNED && (V % EPV == 0) && nfull > 0;
    const float k = 1.44269504088896340736f / a.temp;
    float thr = 0.f;
    if constexpr (HAS_THR) thr = a.thr[r];

    // ---------------- streaming pass
    // A wave's share of tile t is ITERS chunks of 64 vectors.  Its loads are
    // issued up front, in vocabulary order, in one basic block with the code that
    // consumes them, so each chunk is worked on as soon as it lands while the
    // later ones are still in flight.  Everything in this phase is lane-local:
    //   cs[j]   sum of the lane's vector of chunk j, relative to its group's reference
    //   rlg[g]  integer reference shared by the G chunks of group g
    //   TL, RL  the lane's total over the share and its reference
    // One wave reduction per share then leaves (sum, reference) in LDS.
    Vec raw[ITERS];
    float cs[ITERS], rlg[NG];
    const int64_t wave_vec0 = (int64_t)wave * ITERS * 64;

    // How a share reaches the registers:
    //   kFull     every vector of the share is a whole vector inside the row
    //   kMasked   aligned row, share runs past the row end: lanes past the end read
    //             the row's last vector (a valid address) and are blanked when used
    //   kChecked  anything else (row not 16-byte aligned, partial last vector):
    //             per-lane checked loads, all done before the arithmetic starts
    // kFull and kMasked keep at most DEPTH loads per lane in flight: the first
    // DEPTH are issued up front and chunk j+DEPTH is requested right after chunk j
    // has been consumed.  A wave can only use its chunks in order, so a short
    // request queue (served nearly first-in first-out by the memory system) lets
    // arithmetic start early and overlap the rest of the row's transfer, where
    // thousands of requests posted at once would be served in arbitrary order.
    constexpr int kFull = 0, kMasked = 1, kChecked = 2;
    constexpr int DEPTH = ITERS < 4 ? ITERS : (ITERS < kDepth ? ITERS : kDepth);

    auto consume = [&](auto mode_c, const T *p0, int64_t last_off, int lim) {
        constexpr int MODE = decltype(mode_c)::value;
        auto issue = [&](int j) {
            if constexpr (MODE == kFull) {
                raw[j] = load_vec_full<DT>(p0 + (int64_t)j * 64 * EPV);
            } else if constexpr (MODE == kMasked) {
                int64_t off = (int64_t)j * 64 * EPV;       // element offset from p0, clamped to the last vector
                off = off < last_off ? off : last_off;
                raw[j] = load_vec_full<DT>(p0 + off);
            }
            // keep the request order and keep the loads from sinking below arithmetic
            __builtin_amdgcn_sched_barrier(0);
        };
        if constexpr (MODE != kChecked) {
#pragma unroll
            for (int j = 0; j < DEPTH; ++j) issue(j);
        }
        float TL = 0.f, RL = kRefFloor;
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            float s[G], ref[G];
#pragma unroll
            for (int jj = 0; jj < G; ++jj) {
                const int j = g * G + jj;
                if constexpr (MODE == kMasked) {
                    if (j * 64 >= lim) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) raw[j].w[i] = Elem<DT>::kNegInfWord;
                    }
                }
                s[jj] = chunk_sum<DT, HAS_THR>(raw[j], k, thr, ref[jj]);
                if constexpr (MODE != kChecked) {
                    if (j + DEPTH < ITERS) issue(j + DEPTH);
                }
            }
            float rl = ref[0];
#pragma unroll
            for (int jj = 1; jj < G; ++jj) rl = fmaxf(rl, ref[jj]);
            float gs = 0.f;
#pragma unroll
            for (int jj = 0; jj < G; ++jj) {
                cs[g * G + jj] = ldexpf(s[jj], shift_of(ref[jj], rl));
                gs += cs[g * G + jj];
            }
            rlg[g] = rl;
            const float RLn = fmaxf(RL, rl);
            TL = ldexpf(TL, shift_of(RL, RLn)) + ldexpf(gs, shift_of(rl, RLn));
            RL = RLn;
        }
        const float rW = wave_max(RL);
        const float W = wave_sum(ldexpf(TL, shift_of(RL, rW)));
        return std::pair<float, float>(W, rW);
    };

    auto load_and_consume = [&](int t) {
        const int64_t v0 = (int64_t)t * kTileVecs + wave_vec0;
        if (v0 + (int64_t)ITERS * 64 <= nfull) {
            return consume(std::integral_constant<int, kFull>{}, row + (v0 + lane) * EPV, 0, 0);
        }
        if (whole_vectors) {
            const int64_t lim64 = nfull - v0 - lane;          // vectors from this lane's first one to the row end
            const int lim = lim64 < 0 ? 0 : (lim64 > (1 << 20) ? (1 << 20) : (int)lim64);
            // a lane that starts past the row end reads the row's last vector and blanks everything
            const bool any = lim64 >= 1;
            const T *p0 = any ? row + (v0 + lane) * EPV : row + (nfull - 1) * EPV;
            const int64_t last_off = any ? (lim64 - 1) / 64 * 64 * EPV : 0;
            return consume(std::integral_constant<int, kMasked>{}, p0, last_off, lim);
        }
#pragma unroll
        for (int j = 0; j < ITERS; ++j) raw[j] = load_vec_any<DT>(row, v0 + lane + j * 64, V, nfull);
        return consume(std::integral_constant<int, kChecked>{}, row, 0, 0);
    };

    // Pass 0 streams every tile and, after one barrier, finds the share that holds
    // c.  Only the wave that owns that share goes on; if its registers hold a later
    // tile it runs the loop once more (pass 1) over just that share.  Written as
    // one loop so that the share code exists once.
    float R = 0.f;
    double S = 0.0, tau = 0.0, run = 0.0;
    int ts = 0, ws = 0;
    int t_begin = 0, t_end = ntiles;
    for (int pass = 0;; ++pass) {
        for (int t = t_begin; t < t_end; ++t) {
            const std::pair<float, float> wr = load_and_consume(t);
            if (pass == 0 && lane == 0) {
                ent_sum[t * NW + wave] = wr.first;
                ent_ref[t * NW + wave] = wr.second;
            }
        }
        if (pass == 1) break;
        __syncthreads();

        // ---------------- every wave: locate the share that holds c (fp64 carries)
        float Rl = -__builtin_inff();
        for (int i = lane; i < nent; i += 64) Rl = fmaxf(Rl, ent_ref[i]);
        R = wave_max(Rl);
        auto ent_val = [&](int idx) -> double {
            return (double)ldexpf(ent_sum[idx], shift_of(ent_ref[idx], R));
        };
        const int P = (nent + 63) >> 6;    // shares per lane, contiguous
        double lane_tot = 0.0;
        for (int q = 0; q < P; ++q) {
            const int idx = lane * P + q;
            if (idx < nent) lane_tot += ent_val(idx);
        }
        const double incl = wave_scan_add(lane_tot);
        S = read_lane(incl, 63);
        tau = (double)a.codes[r] * S;

        const unsigned long long hit = __ballot(incl > tau);
        const unsigned long long nz = __ballot(lane_tot > 0.0);
        const int Lh = hit ? (__ffsll((long long)hit) - 1) : (nz ? (63 - __clzll((long long)nz)) : 0);
        run = read_lane(incl - lane_tot, Lh);
        int sh = -1, last_nz = -1;
        double run_last = run;
        for (int q = 0; q < P; ++q) {
            const int idx = Lh * P + q;
            if (idx >= nent) break;
            const double v = ent_val(idx);
            if (v > 0.0) { last_nz = idx; run_last = run; }
            if (run + v > tau) { sh = idx; break; }
            run += v;
        }
        if (sh < 0) {                      // only by rounding: take the last non-empty share
            sh = last_nz >= 0 ? last_nz : 0;
            run = run_last;
        }
        ts = sh / NW;
        ws = sh % NW;
        if (wave != ws) return;
        if (ts == ntiles - 1) break;       // the share is still in registers
        t_begin = ts;
        t_end = ts + 1;
    }

    // ---------------- owning wave: chunk, lane, element
    // chunk totals: lane j ends up with the sum of chunk j over the wave
    float ctot = 0.f;
#pragma unroll
    for (int j = 0; j < ITERS; ++j) {
        const float tot = wave_sum(ldexpf(cs[j], shift_of(rlg[j / G], R)));
        if (lane == j) ctot = tot;
    }
    int js;
    {
        const double cv = (double)ctot;
        const double ci = wave_scan_add(cv) + run;
        const unsigned long long hit = __ballot(ci > tau);
        const unsigned long long nz = __ballot(cv > 0.0);
        js = hit ? (__ffsll((long long)hit) - 1) : (nz ? (63 - __clzll((long long)nz)) : 0);
        run = read_lane(ci - cv, js);
    }

    Vec hv = raw[0];
#pragma unroll
    for (int j = 1; j < ITERS; ++j)
        if (j == js) hv = raw[j];
    float e[EPV];
    const float rl = chunk_weights<DT, HAS_THR>(hv, k, thr, e);
    const int shf = shift_of(rl, R);
    double ed[EPV];
    double ls = 0.0;
#pragma unroll
    for (int i = 0; i < EPV; ++i) {
        ed[i] = (double)ldexpf(e[i], shf);
        ls += ed[i];
    }
    const double incl2 = wave_scan_add(ls) + run;
    const unsigned long long hit2 = __ballot(incl2 > tau);
    const unsigned long long nz2 = __ballot(ls > 0.0);
    const int l2 = hit2 ? (__ffsll((long long)hit2) - 1) : (nz2 ? (63 - __clzll((long long)nz2)) : 0);
    if (lane != l2) return;

    double acc = incl2 - ls;
    int ih = -1, ilast = 0;
    double before = acc, before_last = acc, ev = 0.0, ev_last = 0.0;
#pragma unroll
    for (int i = 0; i < EPV; ++i) {
        if (ed[i] > 0.0) { ilast = i; before_last = acc; ev_last = ed[i]; }
        if (ih < 0 && acc + ed[i] > tau) { ih = i; before = acc; ev = ed[i]; }
        acc += ed[i];
    }
    if (ih < 0) { ih = ilast; before = before_last; ev = ev_last; }

    const int64_t vec_idx = (int64_t)ts * kTileVecs + ((int64_t)ws * ITERS + js) * 64 + lane;
    int64_t tok64 = vec_idx * EPV + ih;
    if (tok64 > V - 1) tok64 = V - 1;
    if (tok64 < 0) tok64 = 0;
    const int32_t token = (int32_t)tok64;

    // c' = (c*S - before)/e_v: the difference is taken in fp64, the quotient is an fp32 result anyway
    float cnf = (float)(tau - before) / (float)ev;
    cnf = fminf(cnf, 0x1.fffffep-1f);        // 1 - 2^-24
    if (!(cnf >= 0.f)) cnf = 0.f;

    a.tokens_out[r * a.tok_stride] = token;
    a.codes_out[r] = cnf;
    if (a.finished_out) a.finished_out[r] = (a.eos_id >= 0 && token == a.eos_id) ? 1 : 0;
    if (a.prob_out) a.prob_out[r] = (float)(ev / S);
    if (a.flo_out) a.flo_out[r] = (float)(before / S);
    if (a.prev_out) a.prev_out[r] = token;
}

// ===========================================================================
// Row-per-wave kernel (the fast path): one 64-lane wave owns one row.
//
// On this chip a wave64 vector instruction occupies its SIMD for 4 cycles, so a
// row costs (instructions per element) x V / 64 x 4 cycles of one SIMD whatever
// the memory system does; with ~1000 rows over 1024 SIMDs the arithmetic of one
// row (a few microseconds) has to hide under that row's own transfer.  Giving a
// row to ONE wave removes everything that is paid per wave rather than per
// element (row set-up, LDS hand-off, barrier, redundant search) and lets the
// wave keep a whole 64-KiB row in its registers, so the final search needs no
// second read.
//
//   chunk  = 64 vectors (1 KiB), lane l holds vector l
//   group  = 4 chunks; all lanes share ONE integer reference per group
//            (ceil of the group's maximum scaled logit, a wave max), so the
//            group's lane sums add up without rescaling
//   table  = per group (total, reference) in LDS
//
// The row is walked in rounds of SLOTS groups, group i of a round living in
// register slot i.  A round is straight-line code with no branch between a
// request and its use: the compiler's wait counters stay exact only then, and
// an over-cautious wait serialises transfer and arithmetic.  Loads run PD
// groups ahead.  A row is padded, logically, to whole rounds: vectors past its
// end are read from the row's last vector (a valid address) and their lane sums
// are zeroed.  When the group count is a multiple of SLOTS only the last slot
// can be ragged and only it pays for the clamping and zeroing (MASK_ALL false).
// Rows of one round stay in registers; for longer rows (STREAM) the registers
// are reused round after round and the one group that holds the code is read
// again at the end.
// Requirements (checked by the launcher): rows start on 16 bytes and V is a
// multiple of the vector length.
// ===========================================================================

template <class F, int... Is>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, Is...>)
{
    (f(std::integral_constant<int, Is>{}), ...);
}
// f(integral_constant<0>), ..., f(integral_constant<N-1>), in order
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

template <int LO, int HI, class F>
__device__ __forceinline__ void with_uniform_index(int idx, F &&f)
{
    // calls f(integral_constant<i>) for i == idx through a tree of scalar branches
    if constexpr (HI - LO == 1) {
        f(std::integral_constant<int, LO>{});
    } else {
        constexpr int MID = (LO + HI) / 2;
        if (idx < MID) with_uniform_index<LO, MID>(idx, f);
        else with_uniform_index<MID, HI>(idx, f);
    }
}

template <int DT, bool HAS_THR, int SLOTS, int PD, bool MASK_ALL, bool STREAM>
__global__ __launch_bounds__(64) void step_wave_kernel(StepArgs a, int ngroups)
{
    using T = typename Elem<DT>::T;
    constexpr int EPV = Elem<DT>::kPerVec;
    constexpr int NCH = SLOTS * 4;         // chunk slots in registers
    static_assert(PD >= 1 && PD <= SLOTS, "prefetch distance");

    extern __shared__ float smem[];
    const int nrounds = (ngroups + SLOTS - 1) / SLOTS;
    const int npad = nrounds * SLOTS;      // groups after padding to whole rounds
    float *g_sum = smem;                   // [npad] total of a group, relative to its reference
    float *g_ref = smem + npad;            // [npad] integer reference of the group

    const int64_t r = blockIdx.x;
    const int lane = threadIdx.x;

    if (a.finished_in != nullptr && a.finished_in[r] != 0) {
        // finished sequence: padding after EOS (Sec. 3.3); the code stops moving
        if (lane == 0) {
            a.tokens_out[r * a.tok_stride] = a.eos_id;
            a.codes_out[r] = a.codes[r];
            if (a.finished_out) a.finished_out[r] = 1;
            if (a.prob_out) a.prob_out[r] = 1.f;
            if (a.flo_out) a.flo_out[r] = 0.f;
            if (a.prev_out) a.prev_out[r] = a.eos_id;
        }
        return;
    }

    const int64_t src = a.row_ids ? (int64_t)a.row_ids[r] : r;
    const unsigned char *row = reinterpret_cast<const unsigned char *>(reinterpret_cast<const T *>(a.logits) + src * a.ld);
    const int32_t nvec = a.V / EPV;                       // whole vectors in the row (>= 1)
    const int32_t my_chunks = (nvec - lane + 63) / 64;    // chunks in which this lane holds a real vector (may be <= 0)
    // byte offset of this lane's vector in chunk 0, and of the last vector it may read
    const uint32_t off0 = (uint32_t)lane * 16u;
    const uint32_t off_last = my_chunks > 0 ? off0 + (uint32_t)(my_chunks - 1) * 1024u : (uint32_t)(nvec - 1) * 16u;
    const float k = 1.44269504088896340736f / a.temp;
    float thr = 0.f;
    if constexpr (HAS_THR) thr = a.thr[r];

    Vec raw[NCH];
    float cs[NCH];                          // lane sum of each resident chunk, relative to its group's reference

    // request the 4 chunks of group g into register slot SLOT
    auto issue = [&](auto slot_c, int g) __attribute__((always_inline)) {
        constexpr int SLOT = decltype(slot_c)::value;
        constexpr bool CLAMP = MASK_ALL || SLOT == SLOTS - 1;
        const unsigned char *gp = row + (size_t)g * 4096u;          // uniform
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            uint32_t off = off0 + (uint32_t)jj * 1024u;
            if constexpr (CLAMP) {
                // compare offsets from the row start; lanes past the end fall back to their last real vector
                const uint32_t want = (uint32_t)g * 4096u + off;
                raw[SLOT * 4 + jj] = load_vec_full<DT>(reinterpret_cast<const T *>(row + (want < off_last ? want : off_last)));
            } else {
                raw[SLOT * 4 + jj] = load_vec_full<DT>(reinterpret_cast<const T *>(gp + off));
            }
        }
        __builtin_amdgcn_sched_barrier(0);      // requests stay in order, ahead of later arithmetic
    };

    // arithmetic of the group held in slot SLOT: reference, lane sums, total
    auto consume = [&](auto slot_c, int g, float &ref_out) __attribute__((always_inline)) -> float {
        constexpr int SLOT = decltype(slot_c)::value;
        constexpr bool MASK = MASK_ALL || SLOT == SLOTS - 1;
        float x[4][EPV];
        float m[4];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            unpack<DT>(raw[SLOT * 4 + jj], x[jj]);
            if constexpr (HAS_THR) {
#pragma unroll
                for (int i = 0; i < EPV; ++i) x[jj][i] = (x[jj][i] >= thr) ? x[jj][i] : -__builtin_inff();
            }
            if constexpr (EPV == 8)
                m[jj] = max3(max3(max3(x[jj][0], x[jj][1], x[jj][2]), x[jj][3], x[jj][4]),
                             max3(x[jj][5], x[jj][6], x[jj][7]), x[jj][5]);
            else
                m[jj] = max3(max3(x[jj][0], x[jj][1], x[jj][2]), x[jj][3], x[jj][3]);
        }
        const float ml = max3(max3(m[0], m[1], m[2]), m[3], m[3]);
        const float ref = fmaxf(ceilf(wave_max(ml) * k), kRefFloor);
        const float nr = -ref;
        float gs = 0.f;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            float e[EPV];
#pragma unroll
            for (int i = 0; i < EPV; ++i) e[i] = fast_exp2(fmaf(x[jj][i], k, nr));
            float s;
            if constexpr (EPV == 8) s = ((e[0] + e[1]) + (e[2] + e[3])) + ((e[4] + e[5]) + (e[6] + e[7]));
            else s = (e[0] + e[1]) + (e[2] + e[3]);
            if constexpr (MASK) s = (g * 4 + jj < my_chunks) ? s : 0.f;   // past the row end: a copy of another vector
            cs[SLOT * 4 + jj] = s;
            gs += s;
        }
        ref_out = ref;
        return wave_sum(gs);
    };

    // ---------------- streaming pass: whole rounds, no branch inside a round
    static_for<PD>([&](auto i_c) __attribute__((always_inline)) { issue(i_c, decltype(i_c)::value); });

    int gb = 0;
    for (int rnd = 0; rnd < nrounds; ++rnd, gb += SLOTS) {
        static_for<SLOTS>([&](auto i_c) __attribute__((always_inline)) {
            constexpr int I = decltype(i_c)::value;
            // next requests: same round, or (long rows only) the start of the next round.  Past the last
            // round these read the row's last vectors once more; nothing uses them.
            if constexpr (I + PD < SLOTS) issue(std::integral_constant<int, I + PD>{}, gb + I + PD);
            else if constexpr (STREAM) issue(std::integral_constant<int, I + PD - SLOTS>{}, gb + I + PD);
            float ref;
            const float tot = consume(i_c, gb + I, ref);
            if (lane == 0) {
                g_sum[gb + I] = tot;
                g_ref[gb + I] = ref;
            }
        });
    }
    const int round0 = gb - SLOTS;           // first group of the round whose data the registers hold
    __builtin_amdgcn_s_waitcnt(0xc07f);      // lgkmcnt(0): the table written above is read back below (same wave)

    // ---------------- locate the group (fp64 carries)
    float Rl = -__builtin_inff();
    for (int i = lane; i < npad; i += 64) Rl = fmaxf(Rl, g_ref[i]);
    const float R = wave_max(Rl);
    auto g_val = [&](int idx) __attribute__((always_inline)) -> double {
        return (double)ldexpf(g_sum[idx], shift_of(g_ref[idx], R));
    };

    const int P = (npad + 63) >> 6;          // groups per lane, contiguous
    double lane_tot = 0.0;
    for (int q = 0; q < P; ++q) {
        const int idx = lane * P + q;
        if (idx < npad) lane_tot += g_val(idx);
    }
    const double incl = wave_scan_add(lane_tot);
    const double S = read_lane(incl, 63);
    const double tau = (double)a.codes[r] * S;

    int gh;                                  // group that holds the code
    double run;                              // sum of everything before it
    {
        const unsigned long long hit = __ballot(incl > tau);
        const unsigned long long nz = __ballot(lane_tot > 0.0);
        const int Lh = hit ? (__ffsll((long long)hit) - 1) : (nz ? (63 - __clzll((long long)nz)) : 0);
        run = read_lane(incl - lane_tot, Lh);
        gh = -1;
        int last_nz = -1;
        double run_last = run;
        for (int q = 0; q < P; ++q) {
            const int idx = Lh * P + q;
            if (idx >= npad) break;
            const double v = g_val(idx);
            if (v > 0.0) { last_nz = idx; run_last = run; }
            if (run + v > tau) { gh = idx; break; }
            run += v;
        }
        if (gh < 0) {                        // only by rounding: take the last non-empty group
            gh = last_nz >= 0 ? last_nz : 0;
            run = run_last;
        }
    }
    gh = __builtin_amdgcn_readfirstlane(gh);

    // ---------------- chunk, lane, element inside that group
    int slot = gh - round0;                  // register slot that holds group gh
    if constexpr (STREAM) {
        // overwritten by a later round, or by the requests the last round posted
        // past the end of the row (they land in its first PD slots): read the group again
        if (gh < round0 + PD) {
            issue(std::integral_constant<int, SLOTS - 1>{}, gh);
            float ref;
            (void)consume(std::integral_constant<int, SLOTS - 1>{}, gh, ref);
            slot = SLOTS - 1;
        }
    }
    const float refh = g_ref[gh];
    const int shf = shift_of(refh, R);

    float c4[4] = {0.f, 0.f, 0.f, 0.f};
    with_uniform_index<0, SLOTS>(slot, [&](auto s_c) __attribute__((always_inline)) {
        constexpr int SL = decltype(s_c)::value;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) c4[jj] = cs[SL * 4 + jj];
        // opaque to the optimiser: keeps this a tree of branches over registers
        // instead of an indexed read that would force the arrays into memory
        asm volatile("" : "+v"(c4[0]), "+v"(c4[1]), "+v"(c4[2]), "+v"(c4[3]));
    });
    int jh = 3;
    {
        double t[4];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) t[jj] = (double)ldexpf(wave_sum(c4[jj]), shf);
        // first chunk whose running sum passes tau; else the last non-empty one
        int last_nz = -1, found = -1;
        double acc = run, acc_found = run, acc_last = run;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            if (t[jj] > 0.0) { last_nz = jj; acc_last = acc; }
            if (found < 0 && acc + t[jj] > tau) { found = jj; acc_found = acc; }
            acc += t[jj];
        }
        if (found >= 0) { jh = found; run = acc_found; }
        else { jh = last_nz >= 0 ? last_nz : 0; run = acc_last; }
    }
    jh = __builtin_amdgcn_readfirstlane(jh);
    float cl = c4[0];
#pragma unroll
    for (int jj = 1; jj < 4; ++jj)
        if (jj == jh) cl = c4[jj];

    const double lv = (double)ldexpf(cl, shf);
    const double incl2 = wave_scan_add(lv) + run;
    const unsigned long long hit2 = __ballot(incl2 > tau);
    const unsigned long long nz2 = __ballot(lv > 0.0);
    const int l2 = hit2 ? (__ffsll((long long)hit2) - 1) : (nz2 ? (63 - __clzll((long long)nz2)) : 0);

    Vec hv;
    const int cslot = __builtin_amdgcn_readfirstlane(slot * 4 + jh);
    with_uniform_index<0, NCH>(cslot, [&](auto c_c) __attribute__((always_inline)) {
        hv = raw[decltype(c_c)::value];
        asm volatile("" : "+v"(hv.w[0]), "+v"(hv.w[1]), "+v"(hv.w[2]), "+v"(hv.w[3]));
    });
    if (lane != l2) return;

    float x[EPV];
    unpack<DT>(hv, x);
    double ed[EPV];
#pragma unroll
    for (int i = 0; i < EPV; ++i) {
        float e = fast_exp2(fmaf(x[i], k, -refh));
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

    int64_t tok64 = ((int64_t)(gh * 4 + jh) * 64 + lane) * EPV + ih;
    if (tok64 > a.V - 1) tok64 = a.V - 1;
    if (tok64 < 0) tok64 = 0;
    const int32_t token = (int32_t)tok64;

    // c' = (c*S - before)/e_v: the difference is taken in fp64, the quotient is an fp32 result anyway
    float cnf = (float)(tau - before) / (float)ev;
    cnf = fminf(cnf, 0x1.fffffep-1f);        // 1 - 2^-24
    if (!(cnf >= 0.f)) cnf = 0.f;

    a.tokens_out[r * a.tok_stride] = token;
    a.codes_out[r] = cnf;
    if (a.finished_out) a.finished_out[r] = (a.eos_id >= 0 && token == a.eos_id) ? 1 : 0;
    if (a.prob_out) a.prob_out[r] = (float)(ev / S);
    if (a.flo_out) a.flo_out[r] = (float)(before / S);
    if (a.prev_out) a.prev_out[r] = token;
}

template <int DT, bool HAS_THR, int SLOTS, int PD, bool MASK_ALL, bool STREAM>
as_status launch_wave_cfg(as_ctx *ctx, const StepArgs &a, int ngroups)
{
    const int npad = (ngroups + SLOTS - 1) / SLOTS * SLOTS;
    const size_t lds = (size_t)npad * 2 * sizeof(float);
    if (lds > 60 * 1024) return fail(ctx, AS_ERR_UNSUPPORTED, "vocabulary too large for the group table");
    launch(ctx, kKernelStep, step_wave_kernel<DT, HAS_THR, SLOTS, PD, MASK_ALL, STREAM>, dim3((unsigned)a.rows),
           dim3(64), lds, a, ngroups);
    AS_HIP_TRY(ctx, hipGetLastError());
    return AS_OK;
}

template <int DT, bool HAS_THR>
as_status launch_wave(as_ctx *ctx, const StepArgs &a)
{
    constexpr int EPV = Elem<DT>::kPerVec;
    constexpr int PD = AS_WAVE_PD;
    const int nvec = a.V / EPV;
    const int ngroups = (nvec + 255) / 256;
    if (ngroups > 16) return launch_wave_cfg<DT, HAS_THR, 16, PD, true, true>(ctx, a, ngroups);
    if (ngroups == 16) return launch_wave_cfg<DT, HAS_THR, 16, PD, false, false>(ctx, a, ngroups);
    if (ngroups > 8) return launch_wave_cfg<DT, HAS_THR, 16, PD, true, false>(ctx, a, ngroups);
    if (ngroups > 4) return launch_wave_cfg<DT, HAS_THR, 8, PD, true, false>(ctx, a, ngroups);
    return launch_wave_cfg<DT, HAS_THR, 4, PD, true, false>(ctx, a, ngroups);
}

template <int DT, int NW, int ITERS, int OCC, bool ALIGNED, bool HAS_THR>
as_status launch_shape(as_ctx *ctx, const StepArgs &a)
{
    constexpr int EPV = Elem<DT>::kPerVec;
    const int64_t nvec = ((int64_t)a.V + EPV - 1) / EPV;
    const int64_t tile = (int64_t)NW * ITERS * 64;
    const int ntiles = (int)((nvec + tile - 1) / tile);
    const size_t lds = (size_t)ntiles * NW * 2 * sizeof(float);
    if (lds > 60 * 1024) return fail(ctx, AS_ERR_UNSUPPORTED, "vocabulary too large for the share table");
    launch(ctx, kKernelStep, step_kernel<DT, NW, ITERS, OCC, ALIGNED, HAS_THR>, dim3((unsigned)a.rows),
           dim3(NW * 64), lds, a, ntiles);
    AS_HIP_TRY(ctx, hipGetLastError());
    return AS_OK;
}

template <int DT, bool ALIGNED, bool HAS_THR>
as_status launch_cfg(as_ctx *ctx, const StepArgs &a)
{
    switch (ctx->step_shape) {
    case 1: return launch_shape<DT, 8, 8, 8, ALIGNED, HAS_THR>(ctx, a);
    case 2: return launch_shape<DT, 16, 4, 8, ALIGNED, HAS_THR>(ctx, a);
    case 3: return launch_shape<DT, 4, 8, 6, ALIGNED, HAS_THR>(ctx, a);
    case 4: return launch_shape<DT, 2, 16, 4, ALIGNED, HAS_THR>(ctx, a);
    case 5: return launch_shape<DT, 4, 16, 3, ALIGNED, HAS_THR>(ctx, a);
    default: return launch_shape<DT, 4, 16, 4, ALIGNED, HAS_THR>(ctx, a);
    }
}

template <int DT>
as_status launch_dt(as_ctx *ctx, const StepArgs &a)
{
    const size_t esz = (DT == AS_BF16) ? 2 : 4;
    const bool aligned = (reinterpret_cast<uintptr_t>(a.logits) % 16 == 0) && ((a.ld * esz) % 16 == 0);
    constexpr int EPV = Elem<DT>::kPerVec;
    if (aligned && a.V % EPV == 0 && ctx->step_shape != 9)
        return a.thr ? launch_wave<DT, true>(ctx, a) : launch_wave<DT, false>(ctx, a);
    if (aligned) {
        return a.thr ? launch_cfg<DT, true, true>(ctx, a) : launch_cfg<DT, true, false>(ctx, a);
    }
    return a.thr ? launch_cfg<DT, false, true>(ctx, a) : launch_cfg<DT, false, false>(ctx, a);
}

}  // namespace

as_status launch_step(as_ctx *ctx, const StepArgs &a)
{
    if (a.rows == 0) return AS_OK;
    return a.dtype == AS_BF16 ? launch_dt<AS_BF16>(ctx, a) : launch_dt<AS_F32>(ctx, a);
}

}  // namespace as
