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
#include "as_common.hpp"

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

// Vector `vi` of a row.  Elements at or beyond V read as -inf (probability 0).
template <int DT, bool ALIGNED>
__device__ __forceinline__ Vec load_vec(const typename Elem<DT>::T *row, int64_t vi, int32_t V)
{
    constexpr int EPV = Elem<DT>::kPerVec;
    const int64_t base = vi * EPV;
    Vec v;
    if (ALIGNED && base + EPV <= V) {
        const uint4 q = *reinterpret_cast<const uint4 *>(row + base);
        v.w[0] = q.x; v.w[1] = q.y; v.w[2] = q.z; v.w[3] = q.w;
        return v;
    }
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

// exp2 straight on the hardware instruction (no denormal fix-up: results below
// 2^-126 may flush to zero, which is far below anything that can matter here)
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

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
    float m = x[0];
#pragma unroll
    for (int i = 1; i < EPV; ++i) m = fmaxf(m, x[i]);
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

template <int DT, int NW, int ITERS, bool ALIGNED, bool HAS_THR>
__global__ __launch_bounds__(NW * 64) void step_kernel(StepArgs a, int ntiles)
{
    using T = typename Elem<DT>::T;
    constexpr int EPV = Elem<DT>::kPerVec;
    constexpr int64_t kTileVecs = (int64_t)NW * ITERS * 64;

    extern __shared__ float smem[];
    const int nent = ntiles * NW;          // (tile, wave) pairs
    const int nseg = nent * ITERS;         // 1-KiB segments of the row
    float *seg_sum = smem;                 // [nseg]  sum of a segment, relative to its pair's reference
    float *seg_ref = smem + nseg;          // [nent]  integer reference of the pair

    const int64_t r = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;

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
    const float k = 1.44269504088896340736f / a.temp;
    float thr = 0.f;
    if constexpr (HAS_THR) thr = a.thr[r];

    // ---------------- streaming pass: segment sums into LDS
    Vec raw[ITERS];
    const int64_t wave_vec0 = (int64_t)wave * ITERS * 64 + lane;
#pragma unroll
    for (int j = 0; j < ITERS; ++j) raw[j] = load_vec<DT, ALIGNED>(row, wave_vec0 + j * 64, V);

    for (int t = 0; t < ntiles; ++t) {
        float s[ITERS], ref[ITERS];
        const bool more = (t + 1 < ntiles);
        const int64_t next0 = (int64_t)(t + 1) * kTileVecs + wave_vec0;
#pragma unroll
        for (int j = 0; j < ITERS; ++j) {
            s[j] = chunk_sum<DT, HAS_THR>(raw[j], k, thr, ref[j]);
            if (more) raw[j] = load_vec<DT, ALIGNED>(row, next0 + j * 64, V);
        }
        float rl = ref[0];
#pragma unroll
        for (int j = 1; j < ITERS; ++j) rl = fmaxf(rl, ref[j]);
        const float rW = wave_max(rl);
        float segv = 0.f;
#pragma unroll
        for (int j = 0; j < ITERS; ++j) {
            const float tot = wave_sum(ldexpf(s[j], shift_of(ref[j], rW)));
            if (lane == j) segv = tot;
        }
        const int ent = t * NW + wave;
        if (lane < ITERS) seg_sum[ent * ITERS + lane] = segv;
        if (lane == 0) seg_ref[ent] = rW;
    }
    __syncthreads();

    // ---------------- every wave: locate the segment that holds c (fp64 carries)
    float Rl = -__builtin_inff();
    for (int i = lane; i < nent; i += 64) Rl = fmaxf(Rl, seg_ref[i]);
    const float R = wave_max(Rl);

    auto seg_val = [&](int idx) -> double {
        return (double)ldexpf(seg_sum[idx], shift_of(seg_ref[idx / ITERS], R));
    };

    const int P = (nseg + 63) >> 6;        // segments per lane, contiguous
    double lane_tot = 0.0;
    for (int q = 0; q < P; ++q) {
        const int idx = lane * P + q;
        if (idx < nseg) lane_tot += seg_val(idx);
    }
    const double incl = wave_scan_add(lane_tot);
    const double S = read_lane(incl, 63);
    const double tau = (double)a.codes[r] * S;

    const unsigned long long hit = __ballot(incl > tau);
    const unsigned long long nz = __ballot(lane_tot > 0.0);
    const int Lh = hit ? (__ffsll((long long)hit) - 1) : (nz ? (63 - __clzll((long long)nz)) : 0);
    double run = read_lane(incl - lane_tot, Lh);

    int sh = -1, last_nz = -1;
    double run_last = run;
    for (int q = 0; q < P; ++q) {
        const int idx = Lh * P + q;
        if (idx >= nseg) break;
        const double v = seg_val(idx);
        if (v > 0.0) { last_nz = idx; run_last = run; }
        if (run + v > tau) { sh = idx; break; }
        run += v;
    }
    if (sh < 0) {                       // only by rounding: take the last non-empty segment
        sh = last_nz >= 0 ? last_nz : 0;
        run = run_last;
    }
    const int ts = sh / (NW * ITERS);
    const int ws = (sh / ITERS) % NW;
    const int js = sh % ITERS;
    if (wave != ws) return;

    // ---------------- owning wave: lane, then element
    Vec hv;
    const int64_t vec_idx = (int64_t)ts * kTileVecs + ((int64_t)ws * ITERS + js) * 64 + lane;
    if (ts == ntiles - 1) {
        hv = raw[0];
#pragma unroll
        for (int j = 1; j < ITERS; ++j)
            if (j == js) hv = raw[j];
    } else {
        hv = load_vec<DT, ALIGNED>(row, vec_idx, V);
    }
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

    int64_t tok64 = vec_idx * EPV + ih;
    if (tok64 > V - 1) tok64 = V - 1;
    if (tok64 < 0) tok64 = 0;
    const int32_t token = (int32_t)tok64;

    double cn = (tau - before) / ev;
    cn = fmax(cn, 0.0);
    float cnf = (float)cn;
    cnf = fminf(cnf, 0x1.fffffep-1f);        // 1 - 2^-24
    if (!(cnf >= 0.f)) cnf = 0.f;

    a.tokens_out[r * a.tok_stride] = token;
    a.codes_out[r] = cnf;
    if (a.finished_out) a.finished_out[r] = (a.eos_id >= 0 && token == a.eos_id) ? 1 : 0;
    if (a.prob_out) a.prob_out[r] = (float)(ev / S);
    if (a.flo_out) a.flo_out[r] = (float)(before / S);
    if (a.prev_out) a.prev_out[r] = token;
}

template <int DT, bool ALIGNED, bool HAS_THR>
as_status launch_cfg(as_ctx *ctx, const StepArgs &a)
{
    constexpr int NW = 4, ITERS = 16;
    constexpr int EPV = Elem<DT>::kPerVec;
    const int64_t nvec = ((int64_t)a.V + EPV - 1) / EPV;
    const int64_t tile = (int64_t)NW * ITERS * 64;
    const int ntiles = (int)((nvec + tile - 1) / tile);
    const size_t lds = ((size_t)ntiles * NW * ITERS + (size_t)ntiles * NW) * sizeof(float);
    if (lds > 48 * 1024) return fail(ctx, AS_ERR_UNSUPPORTED, "vocabulary too large for the segment table");
    launch(ctx, kKernelStep, step_kernel<DT, NW, ITERS, ALIGNED, HAS_THR>, dim3((unsigned)a.rows), dim3(NW * 64),
           lds, a, ntiles);
    AS_HIP_TRY(ctx, hipGetLastError());
    return AS_OK;
}

template <int DT>
as_status launch_dt(as_ctx *ctx, const StepArgs &a)
{
    const size_t esz = (DT == AS_BF16) ? 2 : 4;
    const bool aligned = (reinterpret_cast<uintptr_t>(a.logits) % 16 == 0) && ((a.ld * esz) % 16 == 0);
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
