// Lattice initialisation (Sec. 4.2, Definition "Arithmetic sampling") and the
// synthetic low-rank bigram model that stands in for P(X_t | X_<t) (Sec. 3.3):
// logits[r, v] = (scale/sqrt(d)) * sum_k E[prev[r], k] * U[k, v].
//
// The model keeps U transposed (Ut[V, d], K contiguous) so that both MFMA
// operands are read as 16-byte K-runs; the logits GEMM is then an "NT" product
// C[R, V] = gather(E, prev)[R, d] * Ut[V, d]^T on v_mfma_f32_32x32x16_bf16 with
// fp32 accumulation.  It is the only dense contraction on the path.
#include <type_traits>

#include "as_common.hpp"

namespace as {
namespace {

// ------------------------------------------------------------------ lattice

__global__ void lattice_kernel(const float *u, int32_t B, int32_t N, float *codes,
                               const int32_t *prompts, int32_t *prev, uint8_t *finished)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)B * N) return;
    const int32_t b = (int32_t)(idx / N), i = (int32_t)(idx % N);
    // c_i = (i + u)/N: spacing exactly 1/N around the circle, one shift per prompt
    const double c = codes ? ((double)i + (double)u[b]) / (double)N : 0.0;
    if (codes) codes[idx] = fminf((float)c, 0x1.fffffep-1f);
    if (prev) prev[idx] = prompts[b];
    if (finished) finished[idx] = 0;
}

// ---------------------------------------------------------------- transpose

template <class T>
__global__ __launch_bounds__(256) void transpose_kernel(const T *U, T *Ut, int32_t d, int32_t V)
{
    __shared__ T tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;      // 32 x 8
    const int64_t v0 = (int64_t)blockIdx.x * 32, k0 = (int64_t)blockIdx.y * 32;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t k = k0 + ty + i * 8, v = v0 + tx;
        if (k < d && v < V) tile[ty + i * 8][tx] = U[k * V + v];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t v = v0 + ty + i * 8, k = k0 + tx;
        if (k < d && v < V) Ut[v * d + k] = tile[tx][ty + i * 8];
    }
}

// -------------------------------------------------------------- logits GEMM

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void glb_void;

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t b = __builtin_bit_cast(uint32_t, f);
    b += 0x7fffu + ((b >> 16) & 1u);
    return (uint16_t)(b >> 16);
}

template <class OutT> __device__ __forceinline__ OutT to_out(float f);
template <> __device__ __forceinline__ float to_out<float>(float f) { return f; }
template <> __device__ __forceinline__ uint16_t to_out<uint16_t>(float f) { return f32_to_bf16_rne(f); }

// Two fp32 values to one packed pair of bf16 (round to nearest even), low half first.
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    uint32_t r;
    asm("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(r) : "v"(lo), "v"(hi));
    return r;
}

// ---- persistent kernel --------------------------------------------------------
//
// Block tile 256 x 256, K step 64, 512 threads = 8 waves as 4 (M) x 2 (N), each wave 64 x 128 = 2 x 4 MFMA
// tiles of 32 x 32 (128 accumulator registers per lane).  One block per CU walks its tiles.
//
// Operands go global -> LDS directly (global_load_lds_dwordx4: lane l's 16 bytes land at base + 16*l), as whole
// 128-byte lines per tile row, into a ring of two 64 KB stages.  The load stream runs on across tile
// boundaries: the next tile's first two stages are requested before this tile's epilogue, and because a wave's
// vector-memory operations complete in issue order, those loads land before the epilogue's stores do.
// Fragment reads are hand-placed ds_read_b128, one between every two MFMAs, a K slice of 16 ahead.
// LDS rows are 128 B; 16-byte piece c of row r sits at piece c ^ ((r >> 1) & 7), which makes both the
// 16-row fragment reads and the contiguous loader writes bank-conflict free.
//
// The accumulators are kept transposed (vocabulary along the MFMA's rows): register v of lane l is
// vocabulary 8*(v/4) + 4*(l/32) + v%4 of the tile, batch row l%32, so a lane holds runs of 4 consecutive
// logits of one row.  The epilogue stages them through a private 4 KB of LDS per wave and writes whole
// 128-byte row pieces.
constexpr int PM = 256, PN = 256, PK = 64;
constexpr int kRingA = PM * PK * 2;                    // 32 KB of A rows per stage
constexpr int kRing = (PM + PN) * PK * 2;              // 64 KB per stage
constexpr int kWaveStage = 4096;                       // epilogue staging per wave: 32 rows x 128 B
constexpr int kPersistLds = 2 * kRing + 8 * kWaveStage;   // 160 KB: all of a CU's LDS

__device__ __forceinline__ bf16x8 lds_read16(uint32_t addr)
{
    bf16x8 r;
    asm volatile("ds_read_b128 %0, %1" : "=v"(r) : "v"(addr));
    return r;
}

// FUSED: instead of the logits, write per row and per group of 32 consecutive logits the pair
// (sum of exp2(y - ref), ref) with y = logit * log2(e)/temp and ref = ceil(max y) -- what the sampling
// step needs to find the group its code falls into (the logits never reach memory).  C then is that table,
// float2 [R, ldc], and alpha carries the extra factor log2(e)/temp.
template <class OutT, bool FUSED = false>
__global__ __launch_bounds__(512, 1) void bigram_gemm_persistent(const uint16_t *__restrict__ E,
                                                                 const uint16_t *__restrict__ Ut,
                                                                 const int32_t *__restrict__ prev, int64_t R,
                                                                 int32_t V, int32_t d, float alpha,
                                                                 OutT *__restrict__ C, int64_t ldc, int vec_store,
                                                                 int gm)
{
    __shared__ __attribute__((aligned(1024))) unsigned char smem[kPersistLds];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);       // uniform: LDS targets stay scalar
    const int wm = wave >> 1, wn = wave & 1;

    // Work-groups are handed to the 8 XCDs round-robin, so block b runs on XCD b & 7 and is worker b >> 3 of
    // the W workers there.  XCD x owns column tiles x, x+8, ...  A worker keeps one row tile as long as it can
    // (its gathered A rows stay the same from tile to tile) and the workers of an XCD sit on the same few
    // column tiles at the same time, so a Ut tile is fetched into that XCD's L2 once.  With more row tiles
    // than workers, the W workers of an XCD stand gm x W/gm over row and column tiles: what they have open
    // at one time, gm A tiles and W/gm Ut tiles, has to fit that XCD's L2 or every tile refetches both.
    const int64_t m_blocks = (R + PM - 1) / PM;
    const int64_t n_blocks = ((int64_t)V + PN - 1) / PN;
    const int W = (int)(gridDim.x >> 3);
    const int xcd = blockIdx.x & 7, q = blockIdx.x >> 3;
    const int64_t nbx = n_blocks > xcd ? (n_blocks - xcd + 7) / 8 : 0;
    const int64_t cg = m_blocks < W ? W / m_blocks : 0;
    auto item = [&](int64_t j, int64_t &bm, int64_t &bn) __attribute__((always_inline)) -> bool {
        if (nbx <= 0) return false;
        if (m_blocks >= W || (m_blocks >= gm && m_blocks % gm == 0)) {
            const int gn = W / gm, qm = q % gm, qn = q / gm;        // host: gm divides W
            if (nbx <= qn) return false;
            const int64_t mine = (nbx - qn + gn - 1) / gn;         // column tiles of this XCD that are this worker's
            bm = qm + gm * (j / mine);
            bn = xcd + 8 * (qn + gn * (j % mine));
            return bm < m_blocks;
        }
        if (q >= cg * m_blocks) return false;
        bm = q % m_blocks;
        const int64_t bnx = q / m_blocks + cg * j;
        bn = xcd + 8 * bnx;
        return bnx < nbx;
    };
    int64_t j = 0, bm, bn, bm_next = 0, bn_next = 0;
    if (!item(j, bm, bn)) return;

    // Loader: a stage is 64 chunks of 1 KB (8 tile rows x 128 B); chunk it*8 + wave, it 0..3, is A rows
    // it*64 + rowb, it 4..7 is B rows (it-4)*64 + rowb; a lane always moves logical piece pc of its row.
    // Every address is a uniform base plus a 32-bit offset per lane: the B offsets never change (Ut is padded
    // to whole column tiles, so no row needs a bound), the A offsets change with the row tile.
    const uint32_t rowbytes = (uint32_t)d * 2;
    const unsigned char *Eb = reinterpret_cast<const unsigned char *>(E);
    const unsigned char *Ub = reinterpret_cast<const unsigned char *>(Ut);
    const int rowb = wave * 8 + (lane >> 3);
    const uint32_t pcoff = (uint32_t)(((lane & 7) ^ ((rowb >> 1) & 7)) << 4);
    uint32_t aoff[4], boff[4];
#pragma unroll
    for (int it = 0; it < 4; ++it) boff[it] = (uint32_t)(it * 64 + rowb) * rowbytes + pcoff;
    auto load_aoff = [&](int64_t m0) __attribute__((always_inline)) {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            int64_t m = m0 + it * 64 + rowb;
            if (m > R - 1) m = R - 1;
            aoff[it] = (uint32_t)clamp_token(prev[m], V) * rowbytes + pcoff;
        }
    };
    // request chunk `it` of K stage `st` of the tile whose columns start at n0_ into ring slot buf_
    auto issue1 = [&](int64_t n0_, int st, int buf_, auto it_c) __attribute__((always_inline)) {
        constexpr int it = decltype(it_c)::value;
        unsigned char *dst = smem + buf_ * kRing + (it * 8 + wave) * 1024;
        if constexpr (it < 4) {
            __builtin_amdgcn_global_load_lds((glb_void *)(Eb + (int64_t)st * (PK * 2) + aoff[it]), (lds_void *)dst,
                                             16, 0, 0);
        } else {
            const unsigned char *base = Ub + n0_ * (int64_t)rowbytes + (int64_t)st * (PK * 2);
            __builtin_amdgcn_global_load_lds((glb_void *)(base + boff[it - 4]), (lds_void *)dst, 16, 0, 0);
        }
    };

    f32x16 acc[2][4];
    const int frow = lane & 31, fc = lane >> 5;
    uint32_t fa_addr[2], fb_addr[4];
    const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_void *)smem;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int row = wm * 64 + i * 32 + frow;
        fa_addr[i] = lds_base + row * 128 + ((fc ^ ((row >> 1) & 7)) << 4);
    }
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
        const int row = wn * 128 + jj * 32 + frow;
        fb_addr[jj] = lds_base + kRingA + row * 128 + ((fc ^ ((row >> 1) & 7)) << 4);
    }

    // The schedule below is spelled out instruction by instruction; the scheduling barriers keep it that way.
#define AS_SB() __builtin_amdgcn_sched_barrier(0)
#define AS_GL(n0_, st_, buf_, n_)                                                                            \
    do {                                                                                                     \
        issue1(n0_, st_, buf_, std::integral_constant<int, n_>{});                                           \
        AS_SB();                                                                                             \
    } while (0)
    // fragment of K slice kk (0..3) of the stage at ring offset so_: the slice is an XOR on the piece index
#define AS_RD_A(fr_, i_, so_, kk_)                                                                           \
    do {                                                                                                     \
        fr_[i_] = lds_read16((fa_addr[i_] + (so_)) ^ ((kk_) << 5));                                          \
        AS_SB();                                                                                             \
    } while (0)
#define AS_RD_B(fr_, j_, so_, kk_)                                                                           \
    do {                                                                                                     \
        fr_[j_] = lds_read16((fb_addr[j_] + (so_)) ^ ((kk_) << 5));                                          \
        AS_SB();                                                                                             \
    } while (0)
#define AS_MM(fa_, fb_, i_, j_)                                                                              \
    do {                                                                                                     \
        acc[i_][j_] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb_[j_], fa_[i_], acc[i_][j_], 0, 0, 0);      \
        AS_SB();                                                                                             \
    } while (0)
    // the fragments are outputs of hand-written reads: tie the wait to them so no MFMA moves above it
#define AS_WAIT_FR(fa_, fb_)                                                                                 \
    do {                                                                                                     \
        asm volatile("s_waitcnt lgkmcnt(0)"                                                                  \
                     : "+v"(fa_[0]), "+v"(fa_[1]), "+v"(fb_[0]), "+v"(fb_[1]), "+v"(fb_[2]), "+v"(fb_[3]));  \
        AS_SB();                                                                                             \
    } while (0)
    // multiply the slice held in (ca, cb) while reading slice kk_ into (na, nb_)
#define AS_SLICE(ca, cb, na, nb_, so_, kk_)                                                                  \
    do {                                                                                                     \
        AS_RD_A(na, 0, so_, kk_); AS_MM(ca, cb, 0, 0); AS_RD_B(nb_, 0, so_, kk_); AS_MM(ca, cb, 0, 1);       \
        AS_RD_B(nb_, 1, so_, kk_); AS_MM(ca, cb, 0, 2); AS_RD_A(na, 1, so_, kk_); AS_MM(ca, cb, 0, 3);       \
        AS_RD_B(nb_, 2, so_, kk_); AS_MM(ca, cb, 1, 0); AS_RD_B(nb_, 3, so_, kk_); AS_MM(ca, cb, 1, 1);      \
        AS_MM(ca, cb, 1, 2); AS_MM(ca, cb, 1, 3);                                                            \
    } while (0)

    const int nstages = d / PK;                  // host guarantees nstages >= 2
    bf16x8 xa[2], xb[4], ya[2], yb[4];
    int gs = 0;                                  // running stage count: stage gs lives in ring slot gs & 1
    bool fresh = true;                           // this tile's first stages are not on their way yet
    int stores_behind = 0;                       // stores of the previous tile issued after this tile's stage 1
    for (;;) {
        const int64_t m0 = bm * PM, n0 = bn * PN;
        const bool has_next = item(j + 1, bm_next, bn_next);
        const bool carry = has_next && bm_next == bm;      // the next tile's loads may run ahead of this epilogue
        const int64_t n0n = bn_next * PN;
        if (fresh) {
            load_aoff(m0);
            const int b0 = gs & 1, b1 = b0 ^ 1;
            AS_GL(n0, 0, b0, 0); AS_GL(n0, 0, b0, 1); AS_GL(n0, 0, b0, 2); AS_GL(n0, 0, b0, 3);
            AS_GL(n0, 0, b0, 4); AS_GL(n0, 0, b0, 5); AS_GL(n0, 0, b0, 6); AS_GL(n0, 0, b0, 7);
            AS_GL(n0, 1, b1, 0); AS_GL(n0, 1, b1, 1); AS_GL(n0, 1, b1, 2); AS_GL(n0, 1, b1, 3);
            AS_GL(n0, 1, b1, 4); AS_GL(n0, 1, b1, 5); AS_GL(n0, 1, b1, 6); AS_GL(n0, 1, b1, 7);
            asm volatile("s_waitcnt vmcnt(8)" ::: "memory");      // stage 0 has landed, stage 1 may still fly
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            const uint32_t so0 = b0 * kRing;
            AS_RD_A(xa, 0, so0, 0); AS_RD_A(xa, 1, so0, 0);
            AS_RD_B(xb, 0, so0, 0); AS_RD_B(xb, 1, so0, 0); AS_RD_B(xb, 2, so0, 0); AS_RD_B(xb, 3, so0, 0);
            stores_behind = 0;
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][jj][v] = 0.f;
        for (int s = 0; s < nstages; ++s, ++gs) {
            const int cur = gs & 1, nb = cur ^ 1;
            const uint32_t so = cur * kRing, son = nb * kRing;
            // Stage s+2 is requested whole during the last slice of stage s, into the ring slot that stage s
            // has just left; past the end of this tile it is stage 0 or 1 of the next one.
            const bool in2 = s + 2 < nstages;
            const bool ld2 = in2 || carry;
            const int st2 = in2 ? s + 2 : s + 2 - nstages;
            const int64_t nn2 = in2 ? n0 : n0n;
            AS_WAIT_FR(xa, xb);
            AS_SLICE(xa, xb, ya, yb, so, 1);
            AS_WAIT_FR(ya, yb);
            AS_SLICE(ya, yb, xa, xb, so, 2);
            AS_WAIT_FR(xa, xb);
            AS_SLICE(xa, xb, ya, yb, so, 3);
            AS_WAIT_FR(ya, yb);
            // Every wave has read all of this stage and the next stage has landed.  Behind the next stage's
            // loads there may be the previous tile's stores: let those drain on (vmcnt counts in issue order).
            if (s == 0 && stores_behind == 16) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
            else if (s == 0 && stores_behind == 32) asm volatile("s_waitcnt vmcnt(32)" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            AS_SB();
            // last slice, with the first fragments of the next stage (read for nothing after the last stage
            // of the last tile) and, where there is a stage to request, its eight chunks; the MFMAs stay
            // outside the conditions (a second copy of them costs the accumulators a second set of registers)
            AS_RD_A(xa, 0, son, 0); AS_MM(ya, yb, 0, 0);
            AS_RD_B(xb, 0, son, 0); AS_MM(ya, yb, 0, 1);
            if (ld2) AS_GL(nn2, st2, cur, 0);
            AS_RD_B(xb, 1, son, 0); AS_MM(ya, yb, 0, 2);
            if (ld2) AS_GL(nn2, st2, cur, 1);
            AS_RD_A(xa, 1, son, 0); AS_MM(ya, yb, 0, 3);
            if (ld2) AS_GL(nn2, st2, cur, 2);
            AS_RD_B(xb, 2, son, 0); AS_MM(ya, yb, 1, 0);
            if (ld2) AS_GL(nn2, st2, cur, 3);
            AS_RD_B(xb, 3, son, 0); AS_MM(ya, yb, 1, 1);
            if (ld2) { AS_GL(nn2, st2, cur, 4); AS_GL(nn2, st2, cur, 5); }
            AS_MM(ya, yb, 1, 2);
            if (ld2) { AS_GL(nn2, st2, cur, 6); AS_GL(nn2, st2, cur, 7); }
            AS_MM(ya, yb, 1, 3);
        }

        // ---- epilogue: scale, round once to the storage type, transpose through this wave's 32 x 128 B of
        // staging (16-byte pieces permuted by the row's bits 1..3), write 128-byte row pieces.  The LDS
        // accesses are written by hand so that the compiler does not tie them to the loads in flight.
        if constexpr (FUSED) {
            // Lane l holds, for each 32-row group i and each 32-column MFMA tile j, 16 logits of batch row
            // l%32: columns 8q + 4*(l/32) + 0..3, q = 0..3; the other 16 of that row and tile sit in lane l^32.
            const int b = lane & 31, h = lane >> 5;
            float2 *P = reinterpret_cast<float2 *>(C);
            if (n0 + PN > V) {                    // last column tile: columns past V carry no mass
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int jx = 0; jx < 4; ++jx)
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int64_t n = n0 + wn * 128 + jx * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
                            if (n >= V) acc[i][jx][v] = -__builtin_inff();
                        }
            }
            // references of the 8 groups first (alpha > 0: the maximum commutes with the scaling), then the sums
            float ref[2][4];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int jx = 0; jx < 4; ++jx) {
                    float mx = acc[i][jx][0];
#pragma unroll
                    for (int v = 1; v < 16; ++v) mx = fmaxf(mx, acc[i][jx][v]);
                    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
                    ref[i][jx] = fmaxf(ceilf(mx * alpha), -100000.f);
                }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int jx = 0; jx < 4; ++jx) {
                    float sum = 0.f;
#pragma unroll
                    for (int v = 0; v < 16; ++v) sum += __builtin_amdgcn_exp2f(fmaf(acc[i][jx][v], alpha, -ref[i][jx]));
                    sum += __shfl_xor(sum, 32, 64);
                    const int64_t ncol = n0 + wn * 128 + jx * 32;
                    const int64_t m = m0 + wm * 64 + i * 32 + b;
                    if (h == 0 && m < R && ncol < V) P[m * ldc + (ncol >> 5)] = float2{sum, ref[i][jx]};
                }
            stores_behind = -1;      // few small stores: the next tile's first barrier simply waits for them
        } else {
            constexpr int kPerPiece = 16 / (int)sizeof(OutT);     // outputs per 16-byte piece
            constexpr int kCols = 8 * kPerPiece;                  // tile columns per pass: 64 (bf16) or 32 (fp32)
            constexpr int kPasses = 128 / kCols;                  // per 32-row group of the wave tile
            const uint32_t stg = lds_base + 2 * kRing + wave * kWaveStage;
            const int b = lane & 31, h = lane >> 5;
            const bool interior = vec_store && m0 + PM <= R && n0 + PN <= V;
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int ps = 0; ps < kPasses; ++ps) {
                    if constexpr (sizeof(OutT) == 2) {
#pragma unroll
                        for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                            for (int qq = 0; qq < 4; ++qq) {
                                const int jx = ps * 2 + jj;
                                u32x2 w;
                                w[0] = pack_bf16(acc[i][jx][4 * qq + 0] * alpha, acc[i][jx][4 * qq + 1] * alpha);
                                w[1] = pack_bf16(acc[i][jx][4 * qq + 2] * alpha, acc[i][jx][4 * qq + 3] * alpha);
                                const int piece = (jj * 4 + qq) ^ ((b >> 1) & 7);
                                asm volatile("ds_write_b64 %0, %1" ::"v"(stg + b * 128 + piece * 16 + h * 8), "v"(w)
                                             : "memory");
                            }
                    } else {
#pragma unroll
                        for (int qq = 0; qq < 4; ++qq) {
                            u32x4 w;
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                w[e] = __builtin_bit_cast(uint32_t, acc[i][ps][4 * qq + e] * alpha);
                            const int piece = (qq * 2 + h) ^ ((b >> 1) & 7);
                            asm volatile("ds_write_b128 %0, %1" ::"v"(stg + b * 128 + piece * 16), "v"(w) : "memory");
                        }
                    }
                    u32x4 val[4];
#pragma unroll
                    for (int p = 0; p < 4; ++p) {
                        const int idx = p * 64 + lane;
                        const int row = idx >> 3, piece = idx & 7;
                        asm volatile("ds_read_b128 %0, %1"
                                     : "=v"(val[p])
                                     : "v"(stg + row * 128 + ((piece ^ ((row >> 1) & 7)) << 4))
                                     : "memory");
                    }
                    asm volatile("s_waitcnt lgkmcnt(0)"
                                 : "+v"(val[0]), "+v"(val[1]), "+v"(val[2]), "+v"(val[3])
                                 :
                                 : "memory");
#pragma unroll
                    for (int p = 0; p < 4; ++p) {
                        const int idx = p * 64 + lane;
                        const int row = idx >> 3, piece = idx & 7;
                        const int64_t m = m0 + wm * 64 + i * 32 + row;
                        const int64_t n = n0 + wn * 128 + ps * kCols + piece * kPerPiece;
                        OutT *gp = C + m * ldc + n;
                        if (interior) {
                            *reinterpret_cast<u32x4 *>(gp) = val[p];
                        } else if (m < R && n < V) {
                            if (vec_store && n + kPerPiece <= V) {
                                *reinterpret_cast<u32x4 *>(gp) = val[p];
                            } else {
#pragma unroll
                                for (int e = 0; e < kPerPiece; ++e) {
                                    if (n + e >= V) continue;
                                    // (copy the lane out first: a bit cast applied to a vector element
                                    // designator reads the vector's first element)
                                    const uint32_t bits = val[p][sizeof(OutT) == 2 ? e >> 1 : e];
                                    if constexpr (sizeof(OutT) == 2)
                                        gp[e] = (OutT)(bits >> ((e & 1) * 16));
                                    else
                                        gp[e] = __builtin_bit_cast(OutT, bits);
                                }
                            }
                        }
                    }
                }
            stores_behind = interior ? 8 * kPasses : -1;
        }
        if (!has_next) break;
        fresh = !carry;
        if (fresh) {
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
        }
        ++j;
        bm = bm_next;
        bn = bn_next;
    }
#undef AS_SB
#undef AS_GL
#undef AS_RD_A
#undef AS_RD_B
#undef AS_MM
#undef AS_WAIT_FR
#undef AS_SLICE
}

// ---- tile kernel: any rank d that is a multiple of 64, any size ----------------------
//
// Block tile 128 x 256, K step 64; 4 waves as 2 (M) x 2 (N), each wave 64 x 128.  Operands are staged
// global -> registers -> LDS one K step ahead.  Used where the persistent kernel does not apply.
constexpr int BM = 128, BN = 256, BK = 64;
constexpr int kPieces = BK / 8;                       // 16-byte pieces per tile row
constexpr int kStageRows = 32;                        // C rows staged per epilogue pass

// Byte offset of 16-byte piece c of tile row `row`: pieces of a row are permuted by the row's bits 1..3 so
// that the 16 lanes served together by a fragment read touch all LDS banks once.
__device__ __forceinline__ int swz(int row, int c) { return row * (BK * 2) + ((c ^ ((row >> 1) & 7)) << 4); }

template <class OutT>
__global__ __launch_bounds__(256, 2) void bigram_gemm_bf16(const uint16_t *__restrict__ E,
                                                           const uint16_t *__restrict__ Ut,
                                                           const int32_t *__restrict__ prev, int64_t R,
                                                           int32_t V, int32_t d, float alpha,
                                                           OutT *__restrict__ C, int64_t ldc, int vec_store)
{
    constexpr int WNT = 4;
    constexpr int kBPieces = BN / 32;                  // 16-byte pieces of B per thread and K step
    constexpr int kABytes = BM * BK * 2, kBBytes = BN * BK * 2;
    constexpr int kStageStride = BN * (int)sizeof(OutT) + 16;          // bytes per staged C row
    constexpr int kStageBytes = kStageRows * kStageStride;
    constexpr int kLds = (kABytes + kBBytes) > kStageBytes ? (kABytes + kBBytes) : kStageBytes;
    __shared__ __attribute__((aligned(16))) unsigned char smem[kLds];
    unsigned char *sA = smem, *sB = smem + kABytes;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // Work-groups are handed to the 8 XCDs round-robin.  Give each XCD whole
    // column tiles and let it walk the row tiles of one column tile back to
    // back, so the Ut tile they share is fetched into that XCD's L2 once.
    const int64_t m_blocks = (R + BM - 1) / BM;
    const int64_t n_blocks = ((int64_t)V + BN - 1) / BN;
    const int64_t xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int64_t bn = xcd + 8 * (slot / m_blocks), bm = slot % m_blocks;
    if (bn >= n_blocks) return;
    const int64_t m0 = bm * BM, n0 = bn * BN;

    // global -> register -> LDS: 4 pieces of A and 8 of B per thread and K step
    const int prow = tid >> 3, pc = tid & 7;
    const uint16_t *gA[4], *gB[kBPieces];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int64_t m = m0 + prow + i * 32;
        if (m > R - 1) m = R - 1;
        gA[i] = E + (int64_t)clamp_token(prev[m], V) * d + pc * 8;
    }
#pragma unroll
    for (int i = 0; i < kBPieces; ++i) {
        int64_t n = n0 + prow + i * 32;
        if (n > V - 1) n = V - 1;
        gB[i] = Ut + n * d + pc * 8;
    }

    f32x16 acc[2][WNT];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < WNT; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    u32x4 ra[4], rb[kBPieces];
#pragma unroll
    for (int i = 0; i < 4; ++i) ra[i] = *reinterpret_cast<const u32x4 *>(gA[i]);
#pragma unroll
    for (int i = 0; i < kBPieces; ++i) rb[i] = *reinterpret_cast<const u32x4 *>(gB[i]);

    const int frow = lane & 31, fc = lane >> 5;
    for (int k0 = 0; k0 < d; k0 += BK) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4 *>(sA + swz(prow + i * 32, pc)) = ra[i];
#pragma unroll
        for (int i = 0; i < kBPieces; ++i) *reinterpret_cast<u32x4 *>(sB + swz(prow + i * 32, pc)) = rb[i];
        __syncthreads();
        if (k0 + BK < d) {
#pragma unroll
            for (int i = 0; i < 4; ++i) ra[i] = *reinterpret_cast<const u32x4 *>(gA[i] + k0 + BK);
#pragma unroll
            for (int i = 0; i < kBPieces; ++i) rb[i] = *reinterpret_cast<const u32x4 *>(gB[i] + k0 + BK);
        }
#pragma unroll
        for (int kk = 0; kk < kPieces; kk += 2) {
            bf16x8 fa[2], fb[WNT];
#pragma unroll
            for (int i = 0; i < 2; ++i)
                fa[i] = *reinterpret_cast<const bf16x8 *>(sA + swz(wm * 64 + i * 32 + frow, kk + fc));
#pragma unroll
            for (int j = 0; j < WNT; ++j)
                fb[j] = *reinterpret_cast<const bf16x8 *>(sB + swz(wn * (WNT * 32) + j * 32 + frow, kk + fc));
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < WNT; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    }

    // Epilogue: scale, round once to the storage type, stage 32 rows at a time in
    // LDS and write them out as whole 16-byte pieces along the row.
    // D layout of the 32x32 MFMA: register v of lane l is row 8*(v/4) + 4*(l/32) + v%4, column l%32.
    constexpr int kOutPerPiece = 16 / (int)sizeof(OutT);
    constexpr int kPiecesPerRow = BN / kOutPerPiece;
    auto do_pass = [&](auto pass_c) {
        constexpr int pass = decltype(pass_c)::value;
        constexpr int i = pass & 1;
        __syncthreads();
        if (wm == pass / 2) {
#pragma unroll
            for (int j = 0; j < WNT; ++j) {
                const int col = wn * (WNT * 32) + j * 32 + (lane & 31);
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                    *reinterpret_cast<OutT *>(smem + row * kStageStride + col * (int)sizeof(OutT)) =
                        to_out<OutT>(acc[i][j][v] * alpha);
                }
            }
        }
        __syncthreads();
        for (int p = tid; p < kStageRows * kPiecesPerRow; p += 256) {
            const int row = p / kPiecesPerRow, pcol = p % kPiecesPerRow;
            const int64_t m = m0 + pass * kStageRows + row;
            const int64_t n = n0 + (int64_t)pcol * kOutPerPiece;
            if (m >= R || n >= V) continue;
            const unsigned char *sp = smem + row * kStageStride + pcol * 16;
            OutT *gp = C + m * ldc + n;
            if (vec_store && n + kOutPerPiece <= V) {
                *reinterpret_cast<u32x4 *>(gp) = *reinterpret_cast<const u32x4 *>(sp);
            } else {
                const OutT *se = reinterpret_cast<const OutT *>(sp);
                for (int e = 0; e < kOutPerPiece; ++e)
                    if (n + e < V) gp[e] = se[e];
            }
        }
    };
    static_assert(BM / kStageRows == 4, "epilogue passes are spelled out");
    do_pass(std::integral_constant<int, 0>{});
    do_pass(std::integral_constant<int, 1>{});
    do_pass(std::integral_constant<int, 2>{});
    do_pass(std::integral_constant<int, 3>{});
}

// Plain dot products for what the MFMA kernel does not take: fp32 weights, or a
// rank d that is not a multiple of its K step (small models only).
__device__ __forceinline__ float widen(float x) { return x; }
__device__ __forceinline__ float widen(uint16_t h) { return __builtin_bit_cast(float, (uint32_t)h << 16); }

template <class WT, class OutT>
__global__ __launch_bounds__(256) void bigram_dot(const WT *__restrict__ E, const WT *__restrict__ Ut,
                                                  const int32_t *__restrict__ prev, int64_t R, int32_t V,
                                                  int32_t d, float alpha, OutT *__restrict__ C, int64_t ldc)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= R * V) return;
    const int64_t r = idx / V, v = idx % V;
    const WT *a = E + (int64_t)clamp_token(prev[r], V) * d, *b = Ut + v * d;
    float acc = 0.f;
    for (int k = 0; k < d; ++k) acc = fmaf(widen(a[k]), widen(b[k]), acc);
    C[r * ldc + v] = to_out<OutT>(acc * alpha);
}

template <class WT, class OutT>
void launch_dot(as_ctx *ctx, const as_model *m, const int32_t *prev, int64_t rows, void *out, int64_t ld,
                float alpha)
{
    const int64_t n = rows * (int64_t)m->V;
    launch(ctx, kKernelLogits, bigram_dot<WT, OutT>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0,
           (const WT *)m->E, (const WT *)m->Ut, prev, rows, m->V, m->d, alpha, (OutT *)out, ld);
}

// ------------------------------------------------------------------ estimator

// (1/N) sum_i s(x_i) per prompt (Sec. 4.2) for additive per-token scores: s(x) = sum of score[x_t] up to
// and including the first EOS.  One block per prompt; fp64 sums in a fixed order.
__global__ __launch_bounds__(256) void estimate_kernel(const int32_t *tokens, int32_t N, int32_t T, int32_t V,
                                                       const float *score, int32_t eos_id, double *est)
{
    __shared__ double part[4];
    const int64_t b = blockIdx.x;
    double acc = 0.0;
    for (int32_t i = threadIdx.x; i < N; i += 256) {
        const int32_t *seq = tokens + (b * N + i) * T;
        double s = 0.0;
        for (int32_t t = 0; t < T; ++t) {
            const int32_t tok = seq[t];
            if (tok >= 0 && tok < V) s += (double)score[tok];
            if (eos_id >= 0 && tok == eos_id) break;
        }
        acc += s;
    }
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) est[b] = (part[0] + part[1] + part[2] + part[3]) / (double)N;
}

}  // namespace

as_status launch_lattice(as_ctx *ctx, const float *u, int32_t B, int32_t N, float *codes_out,
                         const int32_t *prompts, int32_t *prev_out, uint8_t *finished_out)
{
    const int64_t n = (int64_t)B * N;
    if (n == 0) return AS_OK;
    hipLaunchKernelGGL(lattice_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, ctx->stream, u, B, N,
                       codes_out, prompts, prev_out, finished_out);
    AS_HIP_TRY(ctx, hipGetLastError());
    return AS_OK;
}

as_status launch_estimate(as_ctx *ctx, const int32_t *tokens, int32_t B, int32_t N, int32_t T, const float *score,
                          int32_t eos_id, double *est_out)
{
    if (B == 0) return AS_OK;
    hipLaunchKernelGGL(estimate_kernel, dim3((unsigned)B), dim3(256), 0, ctx->stream, tokens, N, T, ctx->V, score,
                       eos_id, est_out);
    AS_HIP_TRY(ctx, hipGetLastError());
    return AS_OK;
}

as_status launch_transpose(const void *U, void *Ut, int32_t d, int32_t V, as_dtype wdtype)
{
    const dim3 grid((unsigned)((V + 31) / 32), (unsigned)((d + 31) / 32));
    if (wdtype == AS_BF16)
        hipLaunchKernelGGL((transpose_kernel<uint16_t>), grid, dim3(256), 0, nullptr,
                           (const uint16_t *)U, (uint16_t *)Ut, d, V);
    else
        hipLaunchKernelGGL((transpose_kernel<float>), grid, dim3(256), 0, nullptr, (const float *)U,
                           (float *)Ut, d, V);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(nullptr, e, "transpose launch");
    e = hipStreamSynchronize(nullptr);
    if (e != hipSuccess) return hip_fail(nullptr, e, "transpose sync");
    return AS_OK;
}

// Workers of an XCD along the row tiles when there are more row tiles than workers (a divisor of their number)
static int persistent_gm(const as_ctx *ctx)
{
    const int W = ctx->num_cus / 8;
    if (ctx->gemm_gm > 0 && W % ctx->gemm_gm == 0) return ctx->gemm_gm;
    // 8 x W/8: with 256 KB per operand tile (d = 512) that is 2 MB of A and 1 MB of Ut open in a 4 MB L2;
    // measured at 65536 x 32128 x 512: 768 TFLOP/s with all workers along the rows, 992 with 8, 938 with 4
    return W % 8 == 0 ? 8 : W;
}

as_status launch_bigram_logits(as_ctx *ctx, const as_model *m, const int32_t *prev, int64_t rows,
                               void *logits_out, int64_t ld)
{
    if (rows == 0) return AS_OK;
    const float alpha = (float)((double)m->scale / sqrt((double)m->d));
    const bool mfma = m->wdtype == AS_BF16 && m->d % BK == 0 &&
                      reinterpret_cast<uintptr_t>(m->E) % 16 == 0 && reinterpret_cast<uintptr_t>(m->Ut) % 16 == 0;
    if (mfma) {
        const size_t osz = ctx->dtype == AS_BF16 ? 2 : 4;
        const int vec_store = (reinterpret_cast<uintptr_t>(logits_out) % 16 == 0) && ((ld * osz) % 16 == 0);
        const uint16_t *Ep = (const uint16_t *)m->E, *Up = (const uint16_t *)m->Ut;
        // the persistent kernel addresses operand rows with 32-bit byte offsets and wants two K stages
        const bool persistent = ctx->gemm_shape != 1 && m->d >= 2 * PK && (int64_t)m->V * m->d * 2 < (1LL << 32) &&
                                ctx->num_cus >= 8;
        if (persistent) {
            const dim3 grid((unsigned)(8 * (ctx->num_cus / 8))), block(512);
            if (ctx->dtype == AS_BF16)
                launch(ctx, kKernelLogits, bigram_gemm_persistent<uint16_t>, grid, block, 0, Ep, Up, prev, rows,
                       m->V, m->d, alpha, (uint16_t *)logits_out, ld, vec_store, persistent_gm(ctx));
            else
                launch(ctx, kKernelLogits, bigram_gemm_persistent<float>, grid, block, 0, Ep, Up, prev, rows, m->V,
                       m->d, alpha, (float *)logits_out, ld, vec_store, persistent_gm(ctx));
        } else {
            // grid: 8 XCD lanes x ceil(column tiles / 8) x row tiles (see the kernel's tile mapping)
            const int64_t m_blocks = (rows + BM - 1) / BM, n_blocks = ((int64_t)m->V + BN - 1) / BN;
            const int64_t blocks = 8 * ((n_blocks + 7) / 8) * m_blocks;
            if (blocks > 0x7fffffffLL) return fail(ctx, AS_ERR_UNSUPPORTED, "logits GEMM grid too large");
            const dim3 grid((unsigned)blocks), block(256);
            if (ctx->dtype == AS_BF16)
                launch(ctx, kKernelLogits, bigram_gemm_bf16<uint16_t>, grid, block, 0, Ep, Up, prev, rows, m->V,
                       m->d, alpha, (uint16_t *)logits_out, ld, vec_store);
            else
                launch(ctx, kKernelLogits, bigram_gemm_bf16<float>, grid, block, 0, Ep, Up, prev, rows, m->V, m->d,
                       alpha, (float *)logits_out, ld, vec_store);
        }
    } else {
        if ((rows * (int64_t)m->V + 255) / 256 > 0x7fffffffLL)
            return fail(ctx, AS_ERR_UNSUPPORTED, "logits grid too large");
        if (m->wdtype == AS_BF16) {
            if (ctx->dtype == AS_BF16) launch_dot<uint16_t, uint16_t>(ctx, m, prev, rows, logits_out, ld, alpha);
            else launch_dot<uint16_t, float>(ctx, m, prev, rows, logits_out, ld, alpha);
        } else {
            if (ctx->dtype == AS_BF16) launch_dot<float, uint16_t>(ctx, m, prev, rows, logits_out, ld, alpha);
            else launch_dot<float, float>(ctx, m, prev, rows, logits_out, ld, alpha);
        }
    }
    AS_HIP_TRY(ctx, hipGetLastError());
    return AS_OK;
}

// The fused decode needs the persistent kernel (bf16 weights, rank a multiple of 64 and at least 128,
// operands within 4 GB, 16-byte aligned).
bool fused_path_applies(const as_ctx *ctx, const as_model *m)
{
    return m->wdtype == AS_BF16 && m->d % PK == 0 && m->d >= 2 * PK && (int64_t)m->V * m->d * 2 < (1LL << 32) &&
           reinterpret_cast<uintptr_t>(m->E) % 16 == 0 && reinterpret_cast<uintptr_t>(m->Ut) % 16 == 0 &&
           ctx->num_cus >= 8;
}

as_status launch_bigram_partials(as_ctx *ctx, const as_model *m, const int32_t *prev, int64_t rows, float temp,
                                 float2 *part, int64_t ldp)
{
    if (rows == 0) return AS_OK;
    const float alpha = (float)((double)m->scale / sqrt((double)m->d) * 1.44269504088896340736 / (double)temp);
    const dim3 grid((unsigned)(8 * (ctx->num_cus / 8))), block(512);
    launch(ctx, kKernelLogits, bigram_gemm_persistent<float, true>, grid, block, 0, (const uint16_t *)m->E,
           (const uint16_t *)m->Ut, prev, rows, m->V, m->d, alpha, reinterpret_cast<float *>(part), ldp, 0,
           persistent_gm(ctx));
    AS_HIP_TRY(ctx, hipGetLastError());
    return AS_OK;
}

}  // namespace as
