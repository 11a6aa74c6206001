// Fused arithmetic-sampling step for gfx950: temperature, optional keep
// threshold, softmax, vocabulary-order cumulative sums, interval search and code
// rescale (Algorithm 1 of Sec. 4.1, one loop body) in ONE pass over each logits
// row.  Nothing but the row itself is read from HBM and only O(1) values per
// row are written.
//
// Cost model the design follows (measured on MI355X): a wave64 vector
// instruction holds its SIMD for 4 cycles and a wave issues at most one
// instruction of any kind per 4 cycles, so a row costs
//     (instructions per element) x V / 64 x 4 cycles
// of SIMD time whatever the memory system does.  At V = 32128 a budget of about
// 50 issue slots per 512-element chunk keeps that below the row's HBM transfer;
// everything that is paid per wave or per row (set-up, hand-off, search) has to
// be a few hundred instructions at most, and several waves must share a SIMD so
// that scalar and memory instructions of one overlap vector work of another.
//
// Shape (one workgroup of NW waves per row):
//   * A row is cut into 16-byte vectors.  A tile is NW*ITERS*64 vectors; wave w
//     owns ITERS consecutive 1-KiB chunks of it (its "share"), lane l one vector
//     of each chunk, so every wave load is one contiguous KiB and the vocabulary
//     order is tile > wave > chunk > lane > element.
//   * The loads of a share are issued up front, in order, in the same basic
//     block as the code that consumes them (no branch in between: the compiler's
//     wait counters are exact only then), and chunks are worked on as they land.
//   * The streaming phase is lane-local.  Chunks are taken four at a time; a
//     lane scales the group's logits by k = log2(e)/temp, takes an INTEGER
//     reference r >= every scaled logit it has seen so far, and adds
//     exp2(x*k - r).  Integer references make every later change of reference an
//     exact multiplication by a power of two (ldexp), so sums taken against
//     different references combine without a second exp and without rounding.
//     Kept per lane: the sum of each chunk, the reference of each group, and a
//     running (total, reference).
//   * One wave reduction per share leaves (sum, reference) in LDS; after one
//     barrier each wave adds up the few shares, and the wave whose share holds
//     c*S walks down inside it: 4-chunk groups, chunks, lanes, elements - a
//     handful of wave reductions instead of one per chunk.  Its vectors are
//     still in registers when the row is a single tile; otherwise the share is
//     read again.
//   * Rows that do not start on 16 bytes or whose length is not a whole number
//     of vectors take the same kernel in a form that masks the row's two ends
//     (PARTIAL); rows of whole vectors that fit one tile take step_tile_kernel
//     further down.  The plain three-pass kernel (step_generic_kernel) is left
//     behind its knob.
#include <type_traits>
#include <utility>

#include "as_common.hpp"
#include "as_row.hpp"
#include "as_tile.hpp"

#ifndef AS_STEP_AHEAD
#define AS_STEP_AHEAD 4
#endif
#ifndef AS_STEP_GROUP
#define AS_STEP_GROUP 4
#endif

namespace as {
namespace {

// first index i in [0, N) with run + t[0..i] > tau, else the last i with t[i] > 0 (else 0);
// `run` becomes the sum before the chosen index.  All wave-uniform.
template <int N>
__device__ __forceinline__ int pick_first(const double *t, double tau, double &run)
{
    int found = -1, last_nz = -1;
    double acc = run, acc_found = run, acc_last = run;
#pragma unroll
    for (int i = 0; i < N; ++i) {
        if (t[i] > 0.0) { last_nz = i; acc_last = acc; }
        if (found < 0 && acc + t[i] > tau) { found = i; acc_found = acc; }
        acc += t[i];
    }
    if (found >= 0) { run = acc_found; return found; }
    run = acc_last;
    return last_nz >= 0 ? last_nz : 0;
}

struct SumRef {
    float sum, ref;      // a sum of weights and the integer reference it is relative to
};

// ===========================================================================
// fast kernel: rows start on 16 bytes and are padded to whole vectors (the last vector of a row may be partial)
// ===========================================================================
// PARTIAL: the row's length is not a whole number of vectors (its last vector is padded out by the row stride)
template <int DT, int NW, int ITERS, int OCC, bool HAS_THR, bool PARTIAL>
__global__ __launch_bounds__(NW * 64, OCC) void step_kernel(StepArgs a, int ntiles)
{
    using T = typename Elem<DT>::T;
    constexpr int EPV = Elem<DT>::kPerVec;
    constexpr int G = AS_STEP_GROUP;                  // chunks per group
    constexpr int NG = ITERS / G;
    constexpr int kShare = ITERS * 64;                // vectors per share
    constexpr int kTile = NW * kShare;                // vectors per tile
    static_assert(ITERS % G == 0, "a share is a whole number of groups");

    // LDS: per lane the sums of the chunks of the share in registers (group-major,
    // so a group is one 16- or 8-byte access), then the table of shares
    extern __shared__ float smem[];
    constexpr int kCsFloats = NW * ITERS * 64;
    const int nent = ntiles * NW;          // shares of the row, in vocabulary order
    float *ent_sum = smem + kCsFloats;     // [nent]  sum of a share, relative to its reference
    float *ent_ref = ent_sum + nent;       // [nent]  integer reference of the share

    const int64_t r = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    if (a.finished_in != nullptr && a.finished_in[r] != 0) {
        if (threadIdx.x == 0) write_finished(a, r);
        return;
    }
    const float code = a.codes[r];         // requested early, used after the barrier

    const int64_t src = a.row_ids ? (int64_t)a.row_ids[r] : r;
    const unsigned char *rowb =
        reinterpret_cast<const unsigned char *>(reinterpret_cast<const T *>(a.logits) + src * a.ld);
    // PARTIAL: the row is read as the whole 16-byte vectors it touches; `shift` elements of the first one lie
    // before the row and (with `rem` != 0) the last one holds only `rem` elements of it
    int32_t shift = 0;
    if constexpr (PARTIAL) {
        const uint32_t mis = (uint32_t)(reinterpret_cast<uintptr_t>(rowb) & 15u);
        rowb -= mis;
        shift = (int32_t)(mis / sizeof(T));
    }
    const int32_t vlen = a.V + shift;              // the row's end, counted from the first vector's first element
    const int32_t nvec = (vlen + EPV - 1) / EPV;
    const int32_t rem = PARTIAL ? vlen % EPV : 0;
    const float k = a.k;
    float thr = 0.f;
    if constexpr (HAS_THR) thr = a.thr[r];
    const uint32_t off0 = (uint32_t)lane * 16u;

    typedef float csvec __attribute__((ext_vector_type(G)));
    u32x4 raw[ITERS];        // the share, as loaded
    float rgl[NG];           // lane reference of each group (non-decreasing over the share)
    // lane sums of the chunks of group g, relative to rgl[g]: cs_lds[g * 64 + lane]
    csvec *cs_lds = reinterpret_cast<csvec *>(smem) + (wave * NG) * 64 + lane;

    // Loads and lane-local sums of the share that starts at vector v0 (uniform).
    // RAGGED: the share runs past the row end; a lane then re-reads its last real
    // vector (or the share's first vector, which exists) and zeroes those sums.
    // Returns the share's (sum, reference) after one wave reduction.
    auto stream = [&](int32_t v0, auto ragged_c) __attribute__((always_inline)) {
        constexpr bool RAGGED = decltype(ragged_c)::value;
        const unsigned char *base = rowb + (size_t)v0 * 16u;
        int32_t mych = ITERS;                                   // chunks of the share in which this lane is inside the row
        uint32_t off_last = 0;
        uint32_t tail_off = 0;                                  // where the row's partial last vector sits in the share
        if constexpr (RAGGED) {
            mych = (nvec - v0 - lane + 63) >> 6;
            mych = mych < 0 ? 0 : (mych > ITERS ? ITERS : mych);
            off_last = mych > 0 ? off0 + (uint32_t)(mych - 1) * 1024u : 0u;
            if constexpr (PARTIAL) tail_off = (uint32_t)(nvec - 1 - v0) * 16u;
        }
        // A wave issues in order: while a load waits for room in the memory pipeline the wave
        // cannot start on data it already has.  So only AHEAD groups are requested up front
        // and group g+AHEAD is requested right after group g has been consumed.
        constexpr int AHEAD = AS_STEP_AHEAD < NG ? AS_STEP_AHEAD : NG;
        auto request = [&](int g) __attribute__((always_inline)) {
#pragma unroll
            for (int jj = 0; jj < G; ++jj) {
                const int j = g * G + jj;
                uint32_t off = off0 + (uint32_t)j * 1024u;
                if constexpr (RAGGED) off = off < off_last ? off : off_last;
                // ordinary loads, not non-temporal ones: the row has just been written by the logits kernel and
            // part of it is still in the caches (0.45 us per launch inside a decode; 0.35 us the other way
            // on rows that come from HBM)
                raw[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(base + off));
            }
            // keep the requests in vocabulary order and where they are written: the consumer
            // waits for them one by one, in this order
            __builtin_amdgcn_sched_barrier(0);
        };
#pragma unroll
        for (int g = 0; g < AHEAD; ++g) request(g);
        float TL = 0.f, RL = kRefFloor;
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            float x[G][EPV];
            float m[G];
#pragma unroll
            for (int jj = 0; jj < G; ++jj) {
                unpack<DT>(raw[g * G + jj], x[jj]);
                if constexpr (HAS_THR) {
#pragma unroll
                    for (int i = 0; i < EPV; ++i) x[jj][i] = (x[jj][i] >= thr) ? x[jj][i] : -__builtin_inff();
                }
                if constexpr (PARTIAL) {
                    // What lies before the row in its first vector and after it in its last one is no logit.
                    // A lane past the row's end has re-read one of its earlier vectors, or the share's first.
                    uint32_t off = off0 + (uint32_t)(g * G + jj) * 1024u;
                    if constexpr (RAGGED) off = off < off_last ? off : off_last;
                    const bool head = shift != 0 && v0 == 0 && off == 0u;
                    const bool tail = RAGGED && rem != 0 && off == tail_off;
                    if (shift != 0 || rem != 0) {
#pragma unroll
                        for (int i = 0; i < EPV; ++i)
                            x[jj][i] = ((head && i < shift) || (tail && i >= rem)) ? -__builtin_inff() : x[jj][i];
                    }
                }
                m[jj] = vec_max<EPV>(x[jj]);
            }
            float gm = m[0];
#pragma unroll
            for (int jj = 1; jj < G; ++jj) gm = max3(gm, m[jj], m[jj]);
            const float RLn = fmaxf(ceilf(gm * k), RL);          // RL starts at the floor
            const float nr = -RLn;
            float gs = 0.f;
            csvec cv;
#pragma unroll
            for (int jj = 0; jj < G; ++jj) {
                float e[EPV];
#pragma unroll
                for (int i = 0; i < EPV; ++i) e[i] = fast_exp2(fmaf(x[jj][i], k, nr));
                float s = vec_sum<EPV>(e);
                if constexpr (RAGGED) s = (g * G + jj < mych) ? s : 0.f;
                cv[jj] = s;
                gs += s;
            }
            cs_lds[g * 64] = cv;
            rgl[g] = RLn;
            TL = ldexpf(TL, shift_of(RL, RLn)) + gs;
            RL = RLn;
            if (g + AHEAD < NG) {
                __builtin_amdgcn_sched_barrier(0);
                request(g + AHEAD);
            }
        }
        const float rW = wave_max(RL);
        const float W = wave_sum(ldexpf(TL, shift_of(RL, rW)));
        return SumRef{W, rW};
    };

    // Pass 0 streams every tile and, after one barrier, finds the share that holds
    // c*S.  Only the wave that owns it goes on; if its registers hold a later tile
    // it runs the loop once more (pass 1) over just that share.  One loop, so the
    // share code exists once per flavour.
    float R = 0.f;
    double S = 0.0, tau = 0.0, run = 0.0;
    int ts = 0;
    int t_begin = 0, t_end = ntiles;
    for (int pass = 0;; ++pass) {
        for (int t = t_begin; t < t_end; ++t) {
            const int32_t v0 = t * kTile + wave * kShare;
            SumRef wr{0.f, kRefFloor};
            // (a share that ends exactly with the row still takes the ragged form if the row's last vector is partial)
            if (v0 + kShare < nvec || (v0 + kShare == nvec && rem == 0)) wr = stream(v0, std::false_type{});
            else if (v0 < nvec) wr = stream(v0, std::true_type{});
            else {
                // a share wholly past the row end.  (The vectors are overwritten too so that the
                // previous tile's registers are dead here and need not be kept alive around the loop.)
#pragma unroll
                for (int j = 0; j < ITERS; ++j) raw[j] = u32x4{0u, 0u, 0u, 0u};
                csvec zero;
#pragma unroll
                for (int jj = 0; jj < G; ++jj) zero[jj] = 0.f;
#pragma unroll
                for (int g = 0; g < NG; ++g) {
                    cs_lds[g * 64] = zero;
                    rgl[g] = kRefFloor;
                }
            }
            if (pass == 0 && lane == 0) {
                ent_sum[t * NW + wave] = wr.sum;
                ent_ref[t * NW + wave] = wr.ref;
            }
        }
        if (pass == 1) break;
        __syncthreads();

        // ---------------- every wave: total, target, owning share (fp64 carries)
        if (ntiles == 1) {
            // the common case: NW shares, read by every lane, handled without cross-lane traffic
            float es[NW], er[NW];
#pragma unroll
            for (int i = 0; i < NW; ++i) { es[i] = ent_sum[i]; er[i] = ent_ref[i]; }
            R = er[0];
#pragma unroll
            for (int i = 1; i < NW; ++i) R = fmaxf(R, er[i]);
            double t[NW];
            S = 0.0;
#pragma unroll
            for (int i = 0; i < NW; ++i) {
                t[i] = (double)ldexpf(es[i], shift_of(er[i], R));
                S += t[i];
            }
            tau = (double)code * S;
            run = 0.0;
            const int sh = pick_first<NW>(t, tau, run);
            ts = 0;
            if (wave != sh) return;
            break;
        }
        const int P = (nent + 63) >> 6;    // shares per lane, contiguous
        float Rl = -__builtin_inff();
        for (int q = 0; q < P; ++q) {
            const int idx = lane * P + q;
            if (idx < nent) Rl = fmaxf(Rl, ent_ref[idx]);
        }
        R = wave_max(Rl);
        double lane_tot = 0.0;
        for (int q = 0; q < P; ++q) {
            const int idx = lane * P + q;
            if (idx < nent) lane_tot += (double)ldexpf(ent_sum[idx], shift_of(ent_ref[idx], R));
        }
        const double incl = wave_scan_add(lane_tot);
        S = read_lane(incl, 63);
        tau = (double)code * S;

        const unsigned long long hit = __ballot(incl > tau);
        const unsigned long long nz = __ballot(lane_tot > 0.0);
        const int Lh = hit ? (__ffsll((long long)hit) - 1) : (nz ? (63 - __clzll((long long)nz)) : 0);
        run = read_lane(incl - lane_tot, Lh);
        int sh = Lh;                       // P == 1: the lane is the share
        if (P > 1) {
            sh = -1;
            int last_nz = -1;
            double run_last = run;
            for (int q = 0; q < P; ++q) {
                const int idx = Lh * P + q;
                if (idx >= nent) break;
                const double v = (double)ldexpf(ent_sum[idx], shift_of(ent_ref[idx], R));
                if (v > 0.0) { last_nz = idx; run_last = run; }
                if (run + v > tau) { sh = idx; break; }
                run += v;
            }
            if (sh < 0) {                  // only by rounding: take the last non-empty share
                sh = last_nz >= 0 ? last_nz : 0;
                run = run_last;
            }
        }
        if (sh >= nent) sh = nent - 1;
        ts = sh / NW;
        if (wave != sh % NW) return;
        if (ts == ntiles - 1) break;       // the share is still in registers
        t_begin = ts;
        t_end = ts + 1;
    }

    // ---------------- owning wave: group, chunk, lane, element
    // group totals, then the group that holds tau (a lane reads back only its own sums)
    int gh;
    {
        double t[NG];
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            const csvec cv = cs_lds[g * 64];
            float gs = cv[0];
#pragma unroll
            for (int jj = 1; jj < G; ++jj) gs += cv[jj];
            t[g] = (double)wave_sum(ldexpf(gs, shift_of(rgl[g], R)));
        }
        gh = pick_first<NG>(t, tau, run);
    }
    gh = __builtin_amdgcn_readfirstlane(gh);

    const csvec ch = cs_lds[gh * 64];
    float c4[G];
#pragma unroll
    for (int jj = 0; jj < G; ++jj) c4[jj] = ch[jj];
    float rh = kRefFloor;
    with_uniform_index<0, NG>(gh, [&](auto g_c) __attribute__((always_inline)) {
        rh = rgl[decltype(g_c)::value];
        // opaque to the optimiser: keeps this a tree of branches over registers
        // instead of an indexed read that would force the array into memory
        asm volatile("" : "+v"(rh));
    });
    const int shf = shift_of(rh, R);       // per lane: this lane's reference for the group
    int jh;
    {
        double t[G];
#pragma unroll
        for (int jj = 0; jj < G; ++jj) t[jj] = (double)wave_sum(ldexpf(c4[jj], shf));
        jh = pick_first<G>(t, tau, run);
    }
    jh = __builtin_amdgcn_readfirstlane(jh);
    float cl = c4[0];
#pragma unroll
    for (int jj = 1; jj < G; ++jj)
        if (jj == jh) cl = c4[jj];

    const double lv = (double)ldexpf(cl, shf);
    const double incl2 = wave_scan_add(lv) + run;
    const unsigned long long hit2 = __ballot(incl2 > tau);
    const unsigned long long nz2 = __ballot(lv > 0.0);
    const int l2 = hit2 ? (__ffsll((long long)hit2) - 1) : (nz2 ? (63 - __clzll((long long)nz2)) : 0);

    u32x4 hv;
    const int cj = __builtin_amdgcn_readfirstlane(gh * G + jh);
    with_uniform_index<0, ITERS>(cj, [&](auto c_c) __attribute__((always_inline)) {
        uint32_t w0 = raw[decltype(c_c)::value][0], w1 = raw[decltype(c_c)::value][1],
                 w2 = raw[decltype(c_c)::value][2], w3 = raw[decltype(c_c)::value][3];
        asm volatile("" : "+v"(w0), "+v"(w1), "+v"(w2), "+v"(w3));
        hv = u32x4{w0, w1, w2, w3};
    });
    if (lane != l2) return;

    float x[EPV];
    unpack<DT>(hv, x);
    double ed[EPV];
    const int64_t vec_no = (int64_t)ts * kTile + (int64_t)wave * kShare + (int64_t)cj * 64 + lane;
    const bool last_partial = PARTIAL && rem != 0 && vec_no == nvec - 1;
    const bool first_partial = PARTIAL && shift != 0 && vec_no == 0;
#pragma unroll
    for (int i = 0; i < EPV; ++i) {
        float e = fast_exp2(fmaf(x[i], k, -rh));
        if constexpr (HAS_THR) e = (x[i] >= thr) ? e : 0.f;
        if (last_partial && i >= rem) e = 0.f;
        if (first_partial && i < shift) e = 0.f;
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

    int64_t tok64 = vec_no * EPV + ih - shift;
    if (tok64 > a.V - 1) tok64 = a.V - 1;
    if (tok64 < 0) tok64 = 0;
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

// ===========================================================================
// single-tile kernel: a row of whole, aligned vectors that fits one tile (4 waves x 16 KiB: 32768 bf16 or
// 16384 fp32 logits), the shape of the headline workload.  Same sums in the same vocabulary order as
// step_kernel, with what a one-tile row allows.
//
// What the clock says about this shape (1024 rows, every block resident at once): a CU's memory pipeline takes
// the 256 loads of its 16 waves at the rate the data comes back, so a wave spends most of its life waiting to
// issue its loads, cannot work on anything meanwhile, and has its data almost as soon as its last load is
// accepted.  The launch therefore takes the time of a read-only kernel of the same shape plus whatever a wave
// still has to do after its last chunk has landed, and the design minimises that remainder:
//   * one integer reference per WAVE, taken from the share's first chunk (or from the keep threshold): every
//     later chunk is unpack, fma, exp2, add and nothing else, worked on as it lands, with no maximum and no
//     change of reference.  Weights may exceed 1 (the reference is not the share's maximum); a share whose
//     weights overflow fp32 (a logit more than 127/k above the first chunk's largest) makes the sums non-finite,
//     which the block sees after its barrier and answers with the plain three-pass routine.
//   * the sums of the 64 chunks of the row (one wave reduction per chunk, four at a time, done while later
//     chunks are still on their way) go to LDS; after the one barrier a single fp64 scan over those 64 values
//     gives the total, the target c*S and the chunk that holds it - share, group and chunk in one step.
//   * the wave that owns that chunk has the lane sums of its chunks in registers: one more scan finds the lane,
//     and that lane the element.
// ===========================================================================
template <int DT, bool HAS_THR, bool NT>
__global__ __launch_bounds__(256, 4) void step_tile_kernel(StepArgs a)
{
    using T = typename Elem<DT>::T;
    constexpr int EPV = Elem<DT>::kPerVec;
    // (eight waves of 8 KiB per row, which this code also fits in 64 registers, measured the same)
    constexpr int NW = kTileWaves, ITERS = kTileIters, G = kTileGroup, NG = ITERS / G;
    constexpr int kShare = ITERS * 64;                // vectors per share

    __shared__ TileSums ts;
    __shared__ GenericScratch gen;

    const int64_t r = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    // What is known per row sits at wave-uniform addresses: scalar loads, requested before anything else and
    // looked at only after the first vector loads are on their way.  The finished flag, one byte, comes as the
    // aligned 32-bit word that holds it (there are no scalar byte loads).
    uint32_t fin_word = 0u, fin_at = 0u;
    if (a.finished_in != nullptr) {
        const uint8_t *q = a.finished_in + r;
        fin_at = (uint32_t)(reinterpret_cast<uintptr_t>(q) & 3u);
        fin_word = *reinterpret_cast<const uint32_t *>(q - fin_at);
    }
    const float code = a.codes[r];
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
    // chunks of the share in which this lane is inside the row (a lane past the row's end re-reads its last
    // real vector, or the share's first one, and its sums are zeroed)
    int32_t mych = (nvec - v0 - lane + 63) >> 6;
    mych = mych < 0 ? 0 : (mych > ITERS ? ITERS : mych);
    const bool live = v0 < nvec;                         // wave-uniform: the share holds some of the row
    const bool ragged = v0 + kShare > nvec;              // wave-uniform: ... and not all of its chunks are whole
    const unsigned char *base = rowb + (size_t)(live ? v0 : 0) * 16u;
    const uint32_t off0 = (uint32_t)lane * 16u;
    const uint32_t off_last = mych > 0 ? off0 + (uint32_t)(mych - 1) * 1024u : 0u;
    // Every offset is clamped to the lane's last vector inside the row (only the one share of a row that runs
    // past its end needs it).  The two vector instructions this puts between consecutive loads are not a cost:
    // with addresses that need none (a scalar base per group and immediates) the launch is 0.8 us slower; a wave
    // that issues its loads back to back takes the CU's memory pipeline for itself, the four waves of a row
    // drift apart and wait for each other at the barrier.
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
    // The first group is requested before the row's finished flag is looked at: the flag is a memory round trip
    // of its own, and the row's first bytes need not wait behind it.  (A finished row thus costs a few KiB
    // of its logits; an unfinished one starts earlier.)
    if (live) request_group(0);
    __builtin_amdgcn_sched_barrier(0);
    if (((fin_word >> (8u * fin_at)) & 0xffu) != 0u) {
        if (threadIdx.x == 0) write_finished(a, r);
        return;
    }
    f32x4 *const my_sums = reinterpret_cast<f32x4 *>(ts.chunk_sum + wave * ITERS);
    auto stream = [&](auto ragged_c) __attribute__((always_inline)) {
        constexpr bool RAGGED = decltype(ragged_c)::value;
#pragma unroll
        for (int g = 1; g < NG; ++g) request_group(g);
        // keep the requests in vocabulary order and where they are written: the consumer waits for them one
        // by one, in this order
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
    tile_select<DT, HAS_THR>(a, r, code, thr, raw, rw, mych, ragged, v0, lane, wave, ts, gen);
}

// ===========================================================================
// generic kernel: any alignment, any V.  Three plain passes over the row (max,
// sums, search), each thread owning one contiguous run of elements so that
// thread order is vocabulary order.  Slow; meant for odd shapes only.
// ===========================================================================
template <int DT, bool HAS_THR>
__global__ __launch_bounds__(256) void step_generic_kernel(StepArgs a)
{
    using T = typename Elem<DT>::T;
    __shared__ GenericScratch sh;
    const int64_t r = blockIdx.x;
    if (a.finished_in != nullptr && a.finished_in[r] != 0) {
        if (threadIdx.x == 0) write_finished(a, r);
        return;
    }
    float thr = -__builtin_inff();
    if constexpr (HAS_THR) thr = a.thr[r];
    generic_step_row<T>(a, r, thr, sh);
}

// ---------------------------------------------------------------------------

template <int DT, int NW, int ITERS, int OCC, bool HAS_THR>
as_status launch_shape(as_ctx *ctx, const StepArgs &a)
{
    constexpr int EPV = Elem<DT>::kPerVec;
    const bool whole = a.V % EPV == 0 && reinterpret_cast<uintptr_t>(a.logits) % 16 == 0 &&
                       (a.ld * (int64_t)sizeof(typename Elem<DT>::T)) % 16 == 0;
    // a row that does not start on 16 bytes can touch one vector more
    const int64_t nvec = ((int64_t)a.V + (whole ? 0 : EPV - 1) + EPV - 1) / EPV;
    const int64_t tile = (int64_t)NW * ITERS * 64;
    const int ntiles = (int)((nvec + tile - 1) / tile);
    const size_t lds = ((size_t)NW * ITERS * 64 + (size_t)ntiles * NW * 2) * sizeof(float);
    if (lds > 60 * 1024) return fail(ctx, AS_ERR_UNSUPPORTED, "vocabulary too large for the share table");
    if (whole && ntiles == 1 && NW == 4 && ITERS == 16 && ctx->step_shape == 0 && a.k <= kTileMaxScale)
    {
        if (stream_rows(a.rows, a.ld, sizeof(typename Elem<DT>::T)))
            launch(ctx, kKernelStep, step_tile_kernel<DT, HAS_THR, true>, dim3((unsigned)a.rows), dim3(256), 0, a);
        else
            launch(ctx, kKernelStep, step_tile_kernel<DT, HAS_THR, false>, dim3((unsigned)a.rows), dim3(256), 0, a);
    }
    else if (!whole)
        launch(ctx, kKernelStep, step_kernel<DT, NW, ITERS, OCC, HAS_THR, true>, dim3((unsigned)a.rows), dim3(NW * 64),
               lds, a, ntiles);
    else
        launch(ctx, kKernelStep, step_kernel<DT, NW, ITERS, OCC, HAS_THR, false>, dim3((unsigned)a.rows), dim3(NW * 64),
               lds, a, ntiles);
    AS_HIP_TRY(ctx, hipGetLastError());
    return AS_OK;
}

template <int DT, bool HAS_THR>
as_status launch_fast(as_ctx *ctx, const StepArgs &a)
{
    switch (ctx->step_shape) {
    case 1: return launch_shape<DT, 2, 32, 2, HAS_THR>(ctx, a);
    case 2: return launch_shape<DT, 8, 8, 8, HAS_THR>(ctx, a);
    case 3: return launch_shape<DT, 4, 8, 6, HAS_THR>(ctx, a);
    case 4: return launch_shape<DT, 2, 16, 4, HAS_THR>(ctx, a);
    case 5: return launch_shape<DT, 1, 32, 2, HAS_THR>(ctx, a);
    case 6: return launch_shape<DT, 4, 16, 4, HAS_THR>(ctx, a);    // the default shape without the single-tile kernel
    default: return launch_shape<DT, 4, 16, 4, HAS_THR>(ctx, a);
    }
}

template <int DT>
as_status launch_dt(as_ctx *ctx, const StepArgs &a)
{
    const size_t esz = (DT == AS_BF16) ? 2 : 4;
    // the fast kernel reads whole 16-byte vectors; all it needs of the rows is that they start on an element
    if (reinterpret_cast<uintptr_t>(a.logits) % esz == 0 && ctx->step_shape != 9)
        return a.thr ? launch_fast<DT, true>(ctx, a) : launch_fast<DT, false>(ctx, a);
    if (a.thr) launch(ctx, kKernelStep, step_generic_kernel<DT, true>, dim3((unsigned)a.rows), dim3(256), 0, a);
    else launch(ctx, kKernelStep, step_generic_kernel<DT, false>, dim3((unsigned)a.rows), dim3(256), 0, a);
    AS_HIP_TRY(ctx, hipGetLastError());
    return AS_OK;
}

}  // namespace

as_status launch_step(as_ctx *ctx, const StepArgs &a)
{
    if (a.rows == 0) return AS_OK;
    return a.dtype == AS_BF16 ? launch_dt<AS_BF16>(ctx, a) : launch_dt<AS_F32>(ctx, a);
}

}  // namespace as
