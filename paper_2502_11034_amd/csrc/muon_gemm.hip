// bf16 matrix-core GEMM for the Newton-Schulz iteration of Muon (the optimizer the paper pairs AdaGC with in
// "Optimizer Compatibility: Muon and Lion", Sec. 5.4), for gfx950.
//
//   C[i][j] = bf16( alpha * sum_k P[i][k] * Q[j][k]  +  beta * D[i][j] )            ("NT": both operands K-contiguous)
//
// P is M x K, Q is N x K, both row-major bf16 with K contiguous, which is the layout the matrix-core
// instruction wants for both operands: every lane's fragment is 16 contiguous bytes.  All three products
// of one Newton-Schulz step have this form when X is kept together with its transpose Y:
//   A  = X X^T                P = Q = X                       (alpha 1, beta 0)
//   B  = b A + c A A          P = Q = A (A is symmetric)      (alpha c, beta b, D = A)
//   X' = a X + B X            P = B, Q = Y = X^T              (alpha 1, beta a, D = X)
// The result is written row-major (C), transposed (Ct, N x M), or both; D is read through its transpose
// Dt (N x M): in the accumulator layout a lane holds 4 consecutive rows of one column, which are 4
// consecutive elements of a transposed array, so those accesses are 8-byte vectors.
//
// All dimensions are multiples of the 128 x 128 x 64 block tile: the caller (muon.hip) keeps every matrix
// in zero-padded workspace buffers, and zero rows and columns stay zero through the iteration.
//
// Tiling: 256 lanes = 4 waves in a 2 x 2 grid, each wave a 64 x 64 tile = 2 x 2 accumulators of
// v_mfma_f32_32x32x16_bf16 (fp32 accumulation).  Operand tiles go global -> registers -> LDS (rows padded
// by 16 bytes against bank conflicts), double-buffered: the loads of tile k+1 are in flight while tile k
// is multiplied.  Workgroups are dealt to the 8 XCDs in turn, so block ids are remapped to give each XCD
// (one L2 each) a contiguous band of output tiles.

#include "adagc_internal.h"

namespace adagc {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2v __attribute__((ext_vector_type(2)));

constexpr int kBM = 128, kBN = 128, kBK = 64;
constexpr int kLdsRow = kBK + 8;                       // bf16 elements per LDS row (16 bytes of padding)
constexpr int kGemmThreads = 256;
constexpr int kVecPerRow = kBK / 8;                    // 16-byte vectors per tile row
constexpr int kLoadsP = kBM * kVecPerRow / kGemmThreads;   // 16-byte loads per lane per P tile (4)
constexpr int kLoadsQ = kBN * kVecPerRow / kGemmThreads;

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    uint32_t rounded = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    return ((u & 0x7FFFFFFFu) > 0x7F800000u) ? ((u >> 16) | 0x40u) : rounded;
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

__global__ __launch_bounds__(kGemmThreads) void gemm_nt_bf16_kernel(
    const uint16_t* __restrict__ P, int ldp, const uint16_t* __restrict__ Q, int ldq, int M, int N, int K,
    float alpha, float beta, const uint16_t* __restrict__ Dt, int lddt, uint16_t* __restrict__ C, int ldc,
    uint16_t* __restrict__ Ct, int ldct)
{
    __shared__ __attribute__((aligned(16))) uint16_t lds_p[2][kBM * kLdsRow];
    __shared__ __attribute__((aligned(16))) uint16_t lds_q[2][kBN * kLdsRow];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // XCD-aware tile order: block b runs on XCD b mod 8; give XCD x the x-th contiguous eighth of the tiles.
    const int tiles_n = N / kBN;
    const int n_tiles = (M / kBM) * tiles_n;
    int b = blockIdx.x;
    if (n_tiles % 8 == 0) b = (b % 8) * (n_tiles / 8) + b / 8;
    const int tile_m = b / tiles_n, tile_n = b % tiles_n;
    const uint16_t* Pt = P + (size_t)tile_m * kBM * ldp;
    const uint16_t* Qt = Q + (size_t)tile_n * kBN * ldq;

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    u32x4 stage_p[kLoadsP], stage_q[kLoadsQ];
    auto load_tile = [&](int kt) {
#pragma unroll
        for (int u = 0; u < kLoadsP; ++u) {
            const int v = u * kGemmThreads + tid;
            const int row = v / kVecPerRow, kv = v % kVecPerRow;
            stage_p[u] = *reinterpret_cast<const u32x4*>(Pt + (size_t)row * ldp + kt * kBK + kv * 8);
        }
#pragma unroll
        for (int u = 0; u < kLoadsQ; ++u) {
            const int v = u * kGemmThreads + tid;
            const int row = v / kVecPerRow, kv = v % kVecPerRow;
            stage_q[u] = *reinterpret_cast<const u32x4*>(Qt + (size_t)row * ldq + kt * kBK + kv * 8);
        }
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int u = 0; u < kLoadsP; ++u) {
            const int v = u * kGemmThreads + tid;
            const int row = v / kVecPerRow, kv = v % kVecPerRow;
            *reinterpret_cast<u32x4*>(&lds_p[buf][row * kLdsRow + kv * 8]) = stage_p[u];
        }
#pragma unroll
        for (int u = 0; u < kLoadsQ; ++u) {
            const int v = u * kGemmThreads + tid;
            const int row = v / kVecPerRow, kv = v % kVecPerRow;
            *reinterpret_cast<u32x4*>(&lds_q[buf][row * kLdsRow + kv * 8]) = stage_q[u];
        }
    };

    const int k_tiles = K / kBK;
    load_tile(0);
    store_tile(0);
    __syncthreads();

    // fragment addressing: lane l holds row (l % 32), k offset (l / 32) * 8 of a 32 x 16 operand block
    const int frag_row = lane & 31;
    const int frag_k = (lane >> 5) * 8;
    for (int kt = 0; kt < k_tiles; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < k_tiles) load_tile(kt + 1);
#pragma unroll
        for (int kk = 0; kk < kBK / 16; ++kk) {
            bf16x8 fa[2], fb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i)
                fa[i] = *reinterpret_cast<const bf16x8*>(&lds_p[buf][(wm * 64 + i * 32 + frag_row) * kLdsRow + kk * 16 + frag_k]);
#pragma unroll
            for (int j = 0; j < 2; ++j)
                fb[j] = *reinterpret_cast<const bf16x8*>(&lds_q[buf][(wn * 64 + j * 32 + frag_row) * kLdsRow + kk * 16 + frag_k]);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < k_tiles) store_tile(buf ^ 1);
        __syncthreads();
    }

    // Epilogue.  Accumulator register r of lane l is element (row (r/4)*8 + (l/32)*4 + r%4, column l%32) of its
    // 32 x 32 block: four consecutive registers are four consecutive rows of one column.
    const int col_in = lane & 31;
    const int row_in = (lane >> 5) * 4;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = tile_n * kBN + wn * 64 + j * 32 + col_in;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int row0 = tile_m * kBM + wm * 64 + i * 32 + q * 8 + row_in;
                float v[4] = {alpha * acc[i][j][q * 4 + 0], alpha * acc[i][j][q * 4 + 1], alpha * acc[i][j][q * 4 + 2],
                              alpha * acc[i][j][q * 4 + 3]};
                if (Dt) {
                    const u32x2v d = *reinterpret_cast<const u32x2v*>(Dt + (size_t)col * lddt + row0);
                    v[0] = fmaf(beta, bf16_lo(d.x), v[0]);
                    v[1] = fmaf(beta, bf16_hi(d.x), v[1]);
                    v[2] = fmaf(beta, bf16_lo(d.y), v[2]);
                    v[3] = fmaf(beta, bf16_hi(d.y), v[3]);
                }
                const uint32_t h0 = f32_to_bf16_rne(v[0]), h1 = f32_to_bf16_rne(v[1]);
                const uint32_t h2 = f32_to_bf16_rne(v[2]), h3 = f32_to_bf16_rne(v[3]);
                if (Ct) {
                    u32x2v o;
                    o.x = h0 | (h1 << 16);
                    o.y = h2 | (h3 << 16);
                    *reinterpret_cast<u32x2v*>(Ct + (size_t)col * ldct + row0) = o;
                }
                if (C) {
                    C[(size_t)(row0 + 0) * ldc + col] = (uint16_t)h0;
                    C[(size_t)(row0 + 1) * ldc + col] = (uint16_t)h1;
                    C[(size_t)(row0 + 2) * ldc + col] = (uint16_t)h2;
                    C[(size_t)(row0 + 3) * ldc + col] = (uint16_t)h3;
                }
            }
        }
}

}  // namespace

// Shapes must be multiples of the block tile and every leading dimension a multiple of 8 elements (16-byte rows).
hipError_t launch_gemm_nt_bf16(const void* P, int ldp, const void* Q, int ldq, int M, int N, int K, float alpha,
                               float beta, const void* Dt, int lddt, void* C, int ldc, void* Ct, int ldct,
                               hipStream_t stream)
{
    if (M <= 0 || N <= 0 || K <= 0 || M % kBM || N % kBN || K % kBK || ldp % 8 || ldq % 8 || (Dt && lddt % 8) ||
        (Ct && ldct % 8) || (!C && !Ct))
        return hipErrorInvalidValue;
    const int blocks = (M / kBM) * (N / kBN);
    gemm_nt_bf16_kernel<<<dim3(blocks), dim3(kGemmThreads), 0, stream>>>(
        static_cast<const uint16_t*>(P), ldp, static_cast<const uint16_t*>(Q), ldq, M, N, K, alpha, beta,
        static_cast<const uint16_t*>(Dt), lddt, static_cast<uint16_t*>(C), ldc, static_cast<uint16_t*>(Ct), ldct);
    return hipGetLastError();
}

}  // namespace adagc

// Test hook of the matrix-core GEMM through the C ABI (see include/adagc.h).
extern "C" int adagc_muon_gemm_nt(const void* P, int64_t ldp, const void* Q, int64_t ldq, int64_t M, int64_t N, int64_t K,
                                  float alpha, float beta, const void* Dt, int64_t lddt, void* C, int64_t ldc, void* Ct,
                                  int64_t ldct, void* stream)
{
    if (!P || !Q) return ADAGC_ERR_INVALID_ARG;
    if (M > INT32_MAX || N > INT32_MAX || K > INT32_MAX || ldp > INT32_MAX || ldq > INT32_MAX || lddt > INT32_MAX ||
        ldc > INT32_MAX || ldct > INT32_MAX)
        return ADAGC_ERR_TOO_LARGE;
    if (ldp < K || ldq < K || (Dt && lddt < M) || (C && ldc < N) || (Ct && ldct < M)) return ADAGC_ERR_INVALID_ARG;
    const hipError_t e = adagc::launch_gemm_nt_bf16(P, (int)ldp, Q, (int)ldq, (int)M, (int)N, (int)K, alpha, beta, Dt, (int)lddt,
                                                    C, (int)ldc, Ct, (int)ldct, static_cast<hipStream_t>(stream));
    if (e == hipErrorInvalidValue) return ADAGC_ERR_INVALID_ARG;
    return e == hipSuccess ? ADAGC_OK : ADAGC_ERR_HIP;
}
