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
    const double c = ((double)i + (double)u[b]) / (double)N;
    codes[idx] = fminf((float)c, 0x1.fffffep-1f);
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

// Block tile BM x BN, K step BK; 4 waves as 2 (M) x 2 (N), each wave 64 x 128 =
// 2 x 4 MFMA tiles of 32 x 32 (128 accumulator registers per lane).
constexpr int BM = 128, BK = 64;
constexpr int kPieces = BK / 8;                       // 16-byte pieces per tile row
constexpr int kStageRows = 32;                        // C rows staged per epilogue pass

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t b = __builtin_bit_cast(uint32_t, f);
    b += 0x7fffu + ((b >> 16) & 1u);
    return (uint16_t)(b >> 16);
}

template <class OutT> __device__ __forceinline__ OutT to_out(float f);
template <> __device__ __forceinline__ float to_out<float>(float f) { return f; }
template <> __device__ __forceinline__ uint16_t to_out<uint16_t>(float f) { return f32_to_bf16_rne(f); }

// Byte offset of 16-byte piece c of tile row `row`: pieces of a row are permuted
// by the row's low bits so that 8 lanes reading the same piece index of 8
// consecutive rows (an MFMA fragment read) touch all LDS banks once.
#ifndef AS_GEMM_SWZ
#define AS_GEMM_SWZ 1
#endif
__device__ __forceinline__ int swz(int row, int c)
{
#if AS_GEMM_SWZ == 0
    return row * (BK * 2) + ((c ^ (row & 7)) << 4);
#elif AS_GEMM_SWZ == 1
    return row * (BK * 2) + ((c ^ ((row >> 1) & 7)) << 4);
#else
    return row * (BK * 2 + 16) + (c << 4);
#endif
}

template <class OutT, int WNT, int OCC>
__global__ __launch_bounds__(256, OCC) void bigram_gemm_bf16(const uint16_t *__restrict__ E,
                                                           const uint16_t *__restrict__ Ut,
                                                           const int32_t *__restrict__ prev, int64_t R,
                                                           int32_t V, int32_t d, float alpha,
                                                           OutT *__restrict__ C, int64_t ldc, int vec_store)
{
    constexpr int BN = 2 * WNT * 32;                   // 2 waves along N, WNT MFMA tiles each
    constexpr int kBPieces = BN / 32;                  // 16-byte pieces of B per thread and K step
    constexpr int kRowBytes = (AS_GEMM_SWZ == 2) ? BK * 2 + 16 : BK * 2;
    constexpr int kABytes = BM * kRowBytes, kBBytes = BN * kRowBytes;
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
        gA[i] = E + (int64_t)prev[m] * d + pc * 8;
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
    const WT *a = E + (int64_t)prev[r] * d, *b = Ut + v * d;
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

as_status launch_bigram_logits(as_ctx *ctx, const as_model *m, const int32_t *prev, int64_t rows,
                               void *logits_out, int64_t ld)
{
    if (rows == 0) return AS_OK;
    const float alpha = (float)((double)m->scale / sqrt((double)m->d));
    const bool mfma = m->wdtype == AS_BF16 && m->d % BK == 0 &&
                      reinterpret_cast<uintptr_t>(m->E) % 16 == 0 && reinterpret_cast<uintptr_t>(m->Ut) % 16 == 0;
    if (mfma) {
        // grid: 8 XCD lanes x ceil(column tiles / 8) x row tiles (see the kernel's tile mapping)
        const int shape = ctx->gemm_shape;
        const int BN = shape == 1 ? 128 : 256;
        const int64_t m_blocks = (rows + BM - 1) / BM, n_blocks = ((int64_t)m->V + BN - 1) / BN;
        const int64_t blocks = 8 * ((n_blocks + 7) / 8) * m_blocks;
        if (blocks > 0x7fffffffLL) return fail(ctx, AS_ERR_UNSUPPORTED, "logits GEMM grid too large");
        const size_t osz = ctx->dtype == AS_BF16 ? 2 : 4;
        const int vec_store = (reinterpret_cast<uintptr_t>(logits_out) % 16 == 0) && ((ld * osz) % 16 == 0);
        const dim3 grid((unsigned)blocks), block(256);
        const uint16_t *Ep = (const uint16_t *)m->E, *Up = (const uint16_t *)m->Ut;
        if (ctx->dtype == AS_BF16) {
            if (shape == 1)
                launch(ctx, kKernelLogits, bigram_gemm_bf16<uint16_t, 2, 4>, grid, block, 0, Ep, Up, prev, rows, m->V,
                       m->d, alpha, (uint16_t *)logits_out, ld, vec_store);
            else
                launch(ctx, kKernelLogits, bigram_gemm_bf16<uint16_t, 4, 2>, grid, block, 0, Ep, Up, prev, rows, m->V,
                       m->d, alpha, (uint16_t *)logits_out, ld, vec_store);
        } else {
            if (shape == 1)
                launch(ctx, kKernelLogits, bigram_gemm_bf16<float, 2, 4>, grid, block, 0, Ep, Up, prev, rows, m->V,
                       m->d, alpha, (float *)logits_out, ld, vec_store);
            else
                launch(ctx, kKernelLogits, bigram_gemm_bf16<float, 4, 2>, grid, block, 0, Ep, Up, prev, rows, m->V,
                       m->d, alpha, (float *)logits_out, ld, vec_store);
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

}  // namespace as
