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

// One 256-thread block per row.  A tile is 1024 groups (a lane of one wave holds 16 consecutive ones, read as
// whole lines and regrouped through LDS).  Rows of one tile (vocabularies up to 32768): wave 0 walks the row's
// table.  Longer rows (MULTI): the four waves take the tiles in turn and leave (sum, reference) per tile; wave 0
// scans those (up to 64: vocabularies up to 2^21), finds the tile of the row's code and walks that one tile
// again.  Then all four waves recompute the hit group's 32 logits, a wave reading one whole row of U^T per
// instruction (8 rows per wave) against the embedding piece it fetched at the start; wave 0 finishes.
constexpr int kMaxPiecesPerLane = 8;          // rank up to 64 * 8 * 8 = 4096
constexpr int kTileGroups = 64 * kGroupsPerLane;
constexpr int kMaxTiles = 64;

template <bool MULTI>
__global__ __launch_bounds__(256) void fused_sample_kernel(FusedArgs a)
{
    __shared__ __attribute__((aligned(16))) float2 table[(MULTI ? 4 : 1) * kTileGroups];     // 8 KB per wave that walks
    __shared__ double tile_sum[MULTI ? kMaxTiles : 1];
    __shared__ float tile_ref[MULTI ? kMaxTiles : 1];
    __shared__ float dots[32];
    __shared__ int32_t hit_group;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t r = blockIdx.x;
    const int nvec = (int)(a.ldp / 2);                            // float4 = two groups
    const int ntiles = MULTI ? (int)((a.ldp + kTileGroups - 1) / kTileGroups) : 1;
    const float4 *prow4 = reinterpret_cast<const float4 *>(a.part + r * a.ldp);
    float4 tw[kGroupsPerLane / 2];
    // a tile of the row's table, whole lines at a time
    auto load_tile = [&](int tile) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < kGroupsPerLane / 2; ++t) {
            const int i = tile * (kTileGroups / 2) + t * 64 + lane;
            tw[t] = i < nvec ? prow4[i] : float4{0.f, 0.f, 0.f, 0.f};
        }
    };
    // the first tile first (it depends on nothing but the row number)
    if (MULTI ? wave < ntiles : wave == 0) load_tile(MULTI ? wave : 0);
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
    float2 *const tb = table + (MULTI ? wave * kTileGroups : 0);
    double gm[kGroupsPerLane];
    double sl = 0.0;
    // the tile in tw: regrouped through LDS so that a lane holds 16 consecutive groups; gm = their masses
    // relative to the tile's reference rw (the largest of its groups' references), sl = the lane's sum
    auto tile_masses = [&](int tile) __attribute__((always_inline)) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");       // (earlier reads of this wave's buffer are done)
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int t = 0; t < kGroupsPerLane / 2; ++t) reinterpret_cast<float4 *>(tb)[t * 64 + lane] = tw[t];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        float2 pr[kGroupsPerLane];
        const int g0 = lane * kGroupsPerLane;
#pragma unroll
        for (int t = 0; t < kGroupsPerLane; t += 2) {
            const float4 w = reinterpret_cast<const float4 *>(tb)[(g0 + t) / 2];
            pr[t] = float2{w.x, w.y};
            pr[t + 1] = float2{w.z, w.w};
        }
        float rl = -200000.f;
#pragma unroll
        for (int t = 0; t < kGroupsPerLane; ++t) {
            if (tile * kTileGroups + g0 + t >= a.ngroups) pr[t] = float2{0.f, -200000.f};      // padding of the table
            rl = fmaxf(rl, pr[t].y);
        }
        rw = wave_max(rl);
        sl = 0.0;
#pragma unroll
        for (int t = 0; t < kGroupsPerLane; ++t) {
            gm[t] = (double)__builtin_amdgcn_ldexpf(pr[t].x, (int)fmaxf(pr[t].y - rw, -300.f));   // exact
            sl += gm[t];
        }
    };
    // the group of the tile in which tau (in the units of the tile's masses) falls; leaves tau2, the rest of
    // tau inside that group, and returns the group's number within the tile
    auto group_in_tile = [&](double tau, double incl) __attribute__((always_inline)) {
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
        return lstar * kGroupsPerLane + gstar;
    };
    if constexpr (!MULTI) {
        if (wave == 0) {
            tile_masses(0);
            const double incl = wave_scan_add(sl);
            const double S = read_lane(incl, 63);
            const int g = group_in_tile((double)c * S, incl);
            if (lane == 0) hit_group = g;
        }
    } else {
        // every wave: its tiles' totals
        for (int tile = wave; tile < ntiles; tile += 4) {
            if (tile != wave) load_tile(tile);
            tile_masses(tile);
            const double St = wave_sum(sl);
            if (lane == 0) {
                tile_sum[tile] = St;
                tile_ref[tile] = rw;
            }
        }
        __syncthreads();
        if (wave == 0) {
            // a lane per tile: totals brought to the row's reference (exact: powers of two), scanned
            const float rt = lane < ntiles ? tile_ref[lane] : -200000.f;
            const float Rg = wave_max(rt);
            const float down = __builtin_amdgcn_ldexpf(1.f, (int)fmaxf(rt - Rg, -126.f));     // 2^(rt - Rg), 0 below 2^-126
            const double st = lane < ntiles && rt - Rg >= -126.f ? tile_sum[lane] * (double)down : 0.0;
            const double tincl = wave_scan_add(st);
            const double S = read_lane(tincl, 63);
            const double tau = (double)c * S;
            const unsigned long long thit = __ballot(tincl > tau);
            const unsigned long long tlive = __ballot(st > 0.0);
            const int tstar = thit ? first_lane(thit) : (tlive ? last_lane(tlive) : 0);
            // the rest of tau inside that tile, in the tile's own units
            const double rest = tau - (read_lane(tincl, tstar) - read_lane(st, tstar));
            const float up = __builtin_amdgcn_ldexpf(1.f, (int)fminf(Rg - read_lane(rt, tstar), 126.f));
            load_tile(tstar);
            tile_masses(tstar);
            const double incl = wave_scan_add(sl);
            const int g = group_in_tile(rest * (double)up, incl);
            if (lane == 0) hit_group = tstar * kTileGroups + g;
        }
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
    if (a.ldp > (int64_t)kTileGroups * kMaxTiles) return fail(ctx, AS_ERR_UNSUPPORTED, "the fused step takes vocabularies up to 2^21");
    if (a.ldp <= kTileGroups) launch(ctx, kKernelStep, fused_sample_kernel<false>, dim3((unsigned)a.rows), dim3(256), 0, a);
    else launch(ctx, kKernelStep, fused_sample_kernel<true>, dim3((unsigned)a.rows), dim3(256), 0, a);
    AS_HIP_TRY(ctx, hipGetLastError());
    return AS_OK;
}

}  // namespace as
