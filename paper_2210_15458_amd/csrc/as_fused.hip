// Sampling step without the logits round trip: the logits kernel leaves, per row and per group of 32
// consecutive logits, (sum of exp2(y - ref), ref) with y = logit*log2(e)/temp and an integer ref; this
// kernel finds the group a row's code falls into from those 8 bytes per group (Sec. 3.1: the bucket search
// over the vocabulary-order cumulative sums, here first over group totals), recomputes the 32 logits of that
// one group from the model, and finishes the search and the rescaling (Algorithm 1, Sec. 4.1) inside it.
// One wave per row.  Sums and the search are fp64 against integer references, weights fp32, as in the
// stand-alone step.
#include "as_common.hpp"

namespace as {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int kGroupsPerLane = 16;

__device__ __forceinline__ int first_lane(unsigned long long mask) { return __builtin_ctzll(mask); }
__device__ __forceinline__ int last_lane(unsigned long long mask) { return 63 - __builtin_clzll(mask); }

// One 256-thread block per row.  Wave 0 walks the row's table (read as whole lines, regrouped through LDS so
// that a lane holds 16 consecutive groups); then all four waves recompute the hit group's 32 logits, a wave
// reading one whole row of U^T per instruction (8 rows per wave) against the embedding piece it fetched at
// the start; wave 0 finishes.
constexpr int kMaxPiecesPerLane = 8;          // rank up to 64 * 8 * 8 = 4096

__global__ __launch_bounds__(256) void fused_sample_kernel(FusedArgs a)
{
    __shared__ __attribute__((aligned(16))) float2 table[64 * kGroupsPerLane];     // 8 KB
    __shared__ float dots[32];
    __shared__ int32_t hit_group;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t r = blockIdx.x;
    // the row of the table first (it depends on nothing but the row number), whole lines at a time
    float4 tw[kGroupsPerLane / 2];
    const int nvec = (int)(a.ldp / 2);                            // float4 = two groups
    if (wave == 0) {
        const float4 *prow4 = reinterpret_cast<const float4 *>(a.part + r * a.ldp);
#pragma unroll
        for (int t = 0; t < kGroupsPerLane / 2; ++t) {
            const int i = t * 64 + lane;
            tw[t] = i < nvec ? prow4[i] : float4{0.f, 0.f, 0.f, 0.f};
        }
    }
    const float c = a.codes[r];
    const int32_t prev = clamp_token(a.prev[r], a.V);
    if (a.finished_in != nullptr && a.finished_in[r] != 0) {
        if (threadIdx.x == 0) {
            a.tokens_out[r * a.tok_stride] = a.eos_id;
            a.codes_out[r] = c;
            if (a.finished_out) a.finished_out[r] = 1;
            if (a.prev_out) a.prev_out[r] = a.eos_id;
        }
        return;
    }
    // pieces lane, lane+64, ... of the conditioning token's embedding: not needed before the dot products
    const int npieces = a.d / 8;
    u32x4 ew[kMaxPiecesPerLane];
    const u32x4 *ep = reinterpret_cast<const u32x4 *>(a.E + (int64_t)prev * a.d);
#pragma unroll
    for (int i = 0; i < kMaxPiecesPerLane; ++i)
        ew[i] = lane + 64 * i < npieces ? ep[lane + 64 * i] : u32x4{0, 0, 0, 0};

    float rw = 0.f;
    double tau2 = 0.0;
    if (wave == 0) {
        // regroup through LDS so that a lane holds 16 consecutive groups
#pragma unroll
        for (int t = 0; t < kGroupsPerLane / 2; ++t) reinterpret_cast<float4 *>(table)[t * 64 + lane] = tw[t];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        float2 pr[kGroupsPerLane];
        const int g0 = lane * kGroupsPerLane;
#pragma unroll
        for (int t = 0; t < kGroupsPerLane; t += 2) {
            const float4 w = reinterpret_cast<const float4 *>(table)[(g0 + t) / 2];
            pr[t] = float2{w.x, w.y};
            pr[t + 1] = float2{w.z, w.w};
        }
        float rl = -200000.f;
#pragma unroll
        for (int t = 0; t < kGroupsPerLane; ++t) {
            if (g0 + t >= a.ngroups) pr[t] = float2{0.f, -200000.f};      // padding of the table
            rl = fmaxf(rl, pr[t].y);
        }
        rw = wave_max(rl);
        double gm[kGroupsPerLane];
        double sl = 0.0;
#pragma unroll
        for (int t = 0; t < kGroupsPerLane; ++t) {
            gm[t] = (double)__builtin_amdgcn_ldexpf(pr[t].x, (int)fmaxf(pr[t].y - rw, -300.f));   // exact
            sl += gm[t];
        }
        const double incl = wave_scan_add(sl);
        const double S = read_lane(incl, 63);
        const double tau = (double)c * S;
        const unsigned long long hit = __ballot(incl > tau);
        const unsigned long long live = __ballot(sl > 0.0);
        const int lstar = hit ? first_lane(hit) : (live ? last_lane(live) : 0);
        const double tau1 = tau - (read_lane(incl, lstar) - read_lane(sl, lstar));
        // the 16 groups of that lane: walk them (wave-uniform after the lane read)
        int gstar = 0, glast = 0;
        double before = 0.0, run = 0.0;
        bool found = false;
#pragma unroll
        for (int t = 0; t < kGroupsPerLane; ++t) {
            const double g = read_lane(gm[t], lstar);
            if (g > 0.0) glast = t;
            if (!found && run + g > tau1) { found = true; gstar = t; before = run; }
            run += g;
        }
        if (!found) {                       // code at the very top by rounding: last group that has any mass
            gstar = glast;
            before = 0.0;
#pragma unroll
            for (int t = 0; t < kGroupsPerLane; ++t)
                if (t < glast) before += read_lane(gm[t], lstar);
        }
        tau2 = tau1 - before;
        if (lane == 0) hit_group = lstar * kGroupsPerLane + gstar;
    }
    __syncthreads();
    const int32_t grp = hit_group;

    // ---- the 32 logits of that group again: wave w takes columns 8w .. 8w+7, eight row loads in flight
    const u32x4 *up[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int32_t col = grp * 32 + wave * 8 + j;
        const int32_t colc = col < a.V ? col : a.V - 1;
        up[j] = reinterpret_cast<const u32x4 *>(a.Ut + (int64_t)colc * a.d);
    }
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < kMaxPiecesPerLane; ++i) {
        if (64 * i >= npieces) break;                           // uniform
        const bool in = lane + 64 * i < npieces;
        u32x4 uw[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) uw[j] = in ? up[j][lane + 64 * i] : u32x4{0, 0, 0, 0};
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t e = ew[i][q], u = uw[j][q];
                acc[j] = fmaf(__builtin_bit_cast(float, e << 16), __builtin_bit_cast(float, u << 16), acc[j]);
                acc[j] = fmaf(__builtin_bit_cast(float, e & 0xffff0000u), __builtin_bit_cast(float, u & 0xffff0000u),
                              acc[j]);
            }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float t = wave_sum(acc[j]);
        if (lane == 0) dots[wave * 8 + j] = t;
    }
    __syncthreads();
    if (wave != 0) return;
    const int32_t col = grp * 32 + (lane & 31);
    const float y = col < a.V ? dots[lane & 31] * a.alpha : -__builtin_inff();
    const float w = lane < 32 ? __builtin_amdgcn_exp2f(y - rw) : 0.f;
    const double wincl = wave_scan_add((double)w);
    const unsigned long long whit = __ballot(wincl > tau2) & 0xffffffffull;
    const unsigned long long wlive = __ballot(w > 0.f) & 0xffffffffull;
    const int cstar = whit ? first_lane(whit) : (wlive ? last_lane(wlive) : 0);
    const float wt = read_lane(w, cstar);
    const double lo = read_lane(wincl, cstar) - (double)wt;

    if (lane == 0) {
        int32_t token = grp * 32 + cstar;
        token = token < a.V ? token : a.V - 1;
        const float num = (float)fmax(tau2 - lo, 0.0);
        float cn = wt > 0.f ? num / wt : 0.f;
        cn = fminf(fmaxf(cn, 0.f), 0x1.fffffep-1f);
        a.tokens_out[r * a.tok_stride] = token;
        a.codes_out[r] = cn;
        if (a.finished_out) a.finished_out[r] = (a.eos_id >= 0 && token == a.eos_id) ? 1 : 0;
        if (a.prev_out) a.prev_out[r] = token;
    }
}

}  // namespace

as_status launch_fused_sample(as_ctx *ctx, const FusedArgs &a)
{
    if (a.rows == 0) return AS_OK;
    if (a.d > 64 * 8 * kMaxPiecesPerLane) return fail(ctx, AS_ERR_UNSUPPORTED, "the fused step takes ranks up to 4096");
    launch(ctx, kKernelStep, fused_sample_kernel, dim3((unsigned)a.rows), dim3(256), 0, a);
    AS_HIP_TRY(ctx, hipGetLastError());
    return AS_OK;
}

}  // namespace as
