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
// A = X X^T and A A are symmetric: for those only the tiles on and below the diagonal are computed and each is
// written twice, to its place and to its mirror image, which saves a third of a step's multiplications.
//
// M and N are multiples of the 128 x 128 block tile and K of 128 (two 64-deep tiles): the caller (muon.hip) keeps every matrix
// in zero-padded workspace buffers, and zero rows and columns stay zero through the iteration.
//
// Tiling: 128 x 128 block tile with 4 waves in a 2 x 2 grid (each wave 64 x 64 = 2 x 2 accumulators of
// v_mfma_f32_32x32x16_bf16, fp32 accumulation); where the launch has enough of them to fill the compute units,
// 256 x 256 tiles with 8 waves in a 4 x 2 grid (each 64 x 128).  One launch can cover a batch of equal-shaped products.  Operand tiles, 64 deep, go global -> registers -> LDS (rows padded by
// 16 bytes against bank conflicts), double-buffered in LDS, with the global loads issued two tiles ahead.
// Workgroups are dealt to the 8 XCDs in turn, so block ids are remapped to give each XCD (one L2 each) a
// contiguous band of output tiles.

#include "adagc_internal.h"

namespace adagc {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2v __attribute__((ext_vector_type(2)));

// Distance in elements from one matrix of a batch to the next, per array (0 for a single product).
struct GemmBatch {
    int64_t stride_p, stride_q, stride_dt, stride_c, stride_ct;
};

#ifndef ADAGC_GEMM_GROUP_M
#define ADAGC_GEMM_GROUP_M 8
#endif
#ifndef ADAGC_GEMM_BIG_THREADS
#define ADAGC_GEMM_BIG_THREADS 512      // lanes of a 256 x 256 workgroup: 8 waves (512) measured 5-7 % faster than 4 (256)
#endif
constexpr int kBK = 64;
constexpr int kLdsRow = kBK + 8;                       // bf16 elements per LDS row (16 bytes of padding)
constexpr int kVecPerRow = kBK / 8;                    // 16-byte vectors per tile row

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    uint32_t rounded = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    return ((u & 0x7FFFFFFFu) > 0x7F800000u) ? ((u >> 16) | 0x40u) : rounded;
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// BT x BT block tile (128 or 256).  SYM: the result is symmetric (P = Q, D symmetric) and C = Ct is one array: only
// the tiles on and below the diagonal are computed, each written to its own place and to its mirror image.
template <int BT, bool SYM, int kGemmThreads>
__global__ __launch_bounds__(kGemmThreads) void gemm_nt_bf16_kernel(
    const uint16_t* __restrict__ P, int ldp, const uint16_t* __restrict__ Q, int ldq, int M, int N, int K,
    float alpha, float beta, const uint16_t* __restrict__ Dt, int lddt, uint16_t* __restrict__ C, int ldc,
    uint16_t* __restrict__ Ct, int ldct, GemmBatch bt)
{
    constexpr int kBM = BT, kBN = BT;
    constexpr int kWM = kGemmThreads / 128;                // waves in a kWM x 2 grid
    constexpr int kTM = kBM / kWM, kTN = kBN / 2;          // wave tile
    constexpr int kMI = kTM / 32, kNI = kTN / 32;          // 32 x 32 accumulators per wave
    constexpr int kLoadsP = kBM * kVecPerRow / kGemmThreads;   // 16-byte loads per lane per P tile
    constexpr int kLoadsQ = kBN * kVecPerRow / kGemmThreads;
    __shared__ __attribute__((aligned(16))) uint16_t lds_p[2][kBM * kLdsRow];
    __shared__ __attribute__((aligned(16))) uint16_t lds_q[2][kBN * kLdsRow];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;               // wm in [0, kWM)

    // XCD-aware tile order: block b runs on XCD b mod 8; give XCD x the x-th contiguous eighth of the tiles of the
    // whole batch (with 8 or more matrices in the batch an XCD then stays on its own matrices).
    const int tiles_n = N / kBN;
    const int n_tiles = SYM ? tiles_n * (tiles_n + 1) / 2 : (M / kBM) * tiles_n;     // per matrix
    const int all_tiles = (int)gridDim.x;                                             // n_tiles x matrices
    int b = blockIdx.x;
    if (all_tiles % 8 == 0) b = (b % 8) * (all_tiles / 8) + b / 8;
    const int z = b / n_tiles;                             // matrix of the batch
    b -= z * n_tiles;
    P += (size_t)z * bt.stride_p;
    Q += (size_t)z * bt.stride_q;
    if (Dt) Dt += (size_t)z * bt.stride_dt;
    if (C) C += (size_t)z * bt.stride_c;
    if (Ct) Ct += (size_t)z * bt.stride_ct;
    int tile_m, tile_n;
    if constexpr (SYM) {
        // b-th tile of the lower triangle, row by row: row r starts at r (r + 1) / 2
        int r = (int)((sqrtf(8.0f * (float)b + 1.0f) - 1.0f) * 0.5f);
        while (r * (r + 1) / 2 > b) --r;
        while ((r + 1) * (r + 2) / 2 <= b) ++r;
        tile_m = r;
        tile_n = b - r * (r + 1) / 2;
    } else {
        // walk the tiles in panels of kGroupM tile rows, down the rows of a panel first: the workgroups that run at
        // the same time on an XCD then form a patch a few tiles high and wide and share both operands in its L2
        constexpr int kGroupM = ADAGC_GEMM_GROUP_M;
        const int tiles_m = M / kBM;
        const int per_group = kGroupM * tiles_n;
        const int group = b / per_group;
        const int first_m = group * kGroupM;
        const int rows_here = (tiles_m - first_m) < kGroupM ? (tiles_m - first_m) : kGroupM;
        const int in_group = b - group * per_group;
        tile_m = first_m + in_group % rows_here;
        tile_n = in_group / rows_here;
    }
    const uint16_t* Pt = P + (size_t)tile_m * kBM * ldp;
    const uint16_t* Qt = Q + (size_t)tile_n * kBN * ldq;

    f32x16 acc[kMI][kNI];
#pragma unroll
    for (int i = 0; i < kMI; ++i)
#pragma unroll
        for (int j = 0; j < kNI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // Two register sets for operand tiles in flight: the loads of tile k+2 are issued before tile k is multiplied
    // and are written to LDS one tile later, so a load has two tiles' worth of matrix-core work to arrive.
    u32x4 stage_p[2][kLoadsP], stage_q[2][kLoadsQ];
    auto load_tile = [&](int kt, u32x4 (&sp)[kLoadsP], u32x4 (&sq)[kLoadsQ]) {
#pragma unroll
        for (int u = 0; u < kLoadsP; ++u) {
            const int v = u * kGemmThreads + tid;
            const int row = v / kVecPerRow, kv = v % kVecPerRow;
            sp[u] = *reinterpret_cast<const u32x4*>(Pt + (size_t)row * ldp + kt * kBK + kv * 8);
        }
#pragma unroll
        for (int u = 0; u < kLoadsQ; ++u) {
            const int v = u * kGemmThreads + tid;
            const int row = v / kVecPerRow, kv = v % kVecPerRow;
            sq[u] = *reinterpret_cast<const u32x4*>(Qt + (size_t)row * ldq + kt * kBK + kv * 8);
        }
    };
    auto store_tile = [&](int buf, const u32x4 (&sp)[kLoadsP], const u32x4 (&sq)[kLoadsQ]) {
#pragma unroll
        for (int u = 0; u < kLoadsP; ++u) {
            const int v = u * kGemmThreads + tid;
            const int row = v / kVecPerRow, kv = v % kVecPerRow;
            *reinterpret_cast<u32x4*>(&lds_p[buf][row * kLdsRow + kv * 8]) = sp[u];
        }
#pragma unroll
        for (int u = 0; u < kLoadsQ; ++u) {
            const int v = u * kGemmThreads + tid;
            const int row = v / kVecPerRow, kv = v % kVecPerRow;
            *reinterpret_cast<u32x4*>(&lds_q[buf][row * kLdsRow + kv * 8]) = sq[u];
        }
    };
    // fragment addressing: lane l holds row (l % 32), k offset (l / 32) * 8 of a 32 x 16 operand block
    const int frag_row = lane & 31;
    const int frag_k = (lane >> 5) * 8;
    auto multiply_tile = [&](int buf) {
#pragma unroll
        for (int kk = 0; kk < kBK / 16; ++kk) {
            bf16x8 fa[kMI], fb[kNI];
#pragma unroll
            for (int i = 0; i < kMI; ++i)
                fa[i] = *reinterpret_cast<const bf16x8*>(&lds_p[buf][(wm * kTM + i * 32 + frag_row) * kLdsRow + kk * 16 + frag_k]);
#pragma unroll
            for (int j = 0; j < kNI; ++j)
                fb[j] = *reinterpret_cast<const bf16x8*>(&lds_q[buf][(wn * kTN + j * 32 + frag_row) * kLdsRow + kk * 16 + frag_k]);
#pragma unroll
            for (int i = 0; i < kMI; ++i)
#pragma unroll
                for (int j = 0; j < kNI; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    };

    const int k_tiles = K / kBK;          // even: K is a multiple of 128
    load_tile(0, stage_p[0], stage_q[0]);
    load_tile(1, stage_p[1], stage_q[1]);
    store_tile(0, stage_p[0], stage_q[0]);
    __syncthreads();
    for (int kt = 0; kt < k_tiles; kt += 2) {
        // tile kt is in LDS buffer 0, tile kt+1 in register set 1
        if (kt + 2 < k_tiles) load_tile(kt + 2, stage_p[0], stage_q[0]);
        multiply_tile(0);
        store_tile(1, stage_p[1], stage_q[1]);
        __syncthreads();
        // tile kt+1 is in LDS buffer 1, tile kt+2 in register set 0
        if (kt + 3 < k_tiles) load_tile(kt + 3, stage_p[1], stage_q[1]);
        multiply_tile(1);
        if (kt + 2 < k_tiles) store_tile(0, stage_p[0], stage_q[0]);
        __syncthreads();
    }

    // Epilogue.  Accumulator register r of lane l is element (row (r/4)*8 + (l/32)*4 + r%4, column l%32) of its
    // 32 x 32 block: four consecutive registers are four consecutive rows of one column.
    const int col_in = lane & 31;
    const int row_in = (lane >> 5) * 4;
#pragma unroll
    for (int i = 0; i < kMI; ++i)
#pragma unroll
        for (int j = 0; j < kNI; ++j) {
            const int col = tile_n * kBN + wn * kTN + j * 32 + col_in;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int row0 = tile_m * kBM + wm * kTM + i * 32 + q * 8 + row_in;
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
                if (SYM ? (tile_m != tile_n) : (C != nullptr)) {      // SYM: the mirror image, C is the same array as Ct
                    C[(size_t)(row0 + 0) * ldc + col] = (uint16_t)h0;
                    C[(size_t)(row0 + 1) * ldc + col] = (uint16_t)h1;
                    C[(size_t)(row0 + 2) * ldc + col] = (uint16_t)h2;
                    C[(size_t)(row0 + 3) * ldc + col] = (uint16_t)h3;
                }
            }
        }
}

}  // namespace

// M, N, K must be multiples of 128 and every leading dimension a multiple of 8 elements (16-byte rows).
// symmetric: P = Q (and D symmetric), so the result is symmetric: C and Ct are then the same array (pass it as Ct)
// and only the lower triangle of tiles is computed.
// batch > 1: that many products of the same shape in one launch, matrix z of every array at its base + z * stride
// (elements).  One launch over many matrices keeps all compute units busy where one matrix has too few tiles, and
// spreads the partly filled last round of workgroups over the whole batch instead of paying it per matrix.
hipError_t launch_gemm_nt_bf16(const void* P, int ldp, const void* Q, int ldq, int M, int N, int K, float alpha,
                               float beta, const void* Dt, int lddt, void* C, int ldc, void* Ct, int ldct,
                               hipStream_t stream, bool symmetric, int batch, int64_t stride_p, int64_t stride_q,
                               int64_t stride_dt, int64_t stride_c, int64_t stride_ct)
{
    if (M <= 0 || N <= 0 || K <= 0 || M % 128 || N % 128 || K % 128 || ldp % 8 || ldq % 8 || (Dt && lddt % 8) ||
        (Ct && ldct % 8) || (!C && !Ct) || batch < 1)
        return hipErrorInvalidValue;
    if ((stride_p | stride_q | stride_dt | stride_c | stride_ct) % 8 || stride_p < 0 || stride_q < 0 || stride_dt < 0 ||
        stride_c < 0 || stride_ct < 0)
        return hipErrorInvalidValue;
    if (symmetric && (M != N || P != Q || stride_p != stride_q || !Ct || (C && (C != Ct || stride_c != stride_ct))))
        return hipErrorInvalidValue;
    const uint16_t *p = static_cast<const uint16_t*>(P), *q = static_cast<const uint16_t*>(Q), *dt = static_cast<const uint16_t*>(Dt);
    uint16_t *c = static_cast<uint16_t*>(C), *ct = static_cast<uint16_t*>(Ct);
    // Tile choice.  A compute unit holds one 256 x 256 workgroup or two 128 x 128 ones, and multiplies about a quarter
    // faster on the large tile (fewer LDS reads per matrix-core instruction); a launch costs whole rounds of workgroups.
    // Compare the two in units of "one 128-tile on a shared compute unit": a round of large tiles is 4 / 1.25 of them.
    const int64_t t128 = symmetric ? (int64_t)(M / 128) * (M / 128 + 1) / 2 : (int64_t)(M / 128) * (N / 128);
    const int64_t t256 = symmetric ? (int64_t)(M / 256) * (M / 256 + 1) / 2 : (int64_t)(M / 256) * (N / 256);
    const int64_t n128 = t128 * batch, n256 = t256 * batch;
    const double cost128 = 2.0 * (double)((n128 + 511) / 512);
    const double cost256 = 3.2 * (double)((n256 + 255) / 256);
    const bool big = (M % 256 == 0) && (N % 256 == 0) && cost256 < cost128;
    const int64_t blocks = big ? n256 : n128;
    if (blocks > INT32_MAX) return hipErrorInvalidValue;
    const GemmBatch bt{stride_p, stride_q, stride_dt, symmetric ? stride_ct : stride_c, stride_ct};
    if (symmetric) {
        c = ct;
        ldc = ldct;
        if (big)
            gemm_nt_bf16_kernel<256, true, ADAGC_GEMM_BIG_THREADS><<<dim3((uint32_t)blocks), dim3(ADAGC_GEMM_BIG_THREADS), 0, stream>>>(p, ldp, q, ldq, M, N, K, alpha, beta, dt, lddt, c, ldc, ct, ldct, bt);
        else
            gemm_nt_bf16_kernel<128, true, 256><<<dim3((uint32_t)blocks), dim3(256), 0, stream>>>(p, ldp, q, ldq, M, N, K, alpha, beta, dt, lddt, c, ldc, ct, ldct, bt);
    } else if (big) {
        gemm_nt_bf16_kernel<256, false, ADAGC_GEMM_BIG_THREADS><<<dim3((uint32_t)blocks), dim3(ADAGC_GEMM_BIG_THREADS), 0, stream>>>(p, ldp, q, ldq, M, N, K, alpha, beta, dt, lddt, c, ldc, ct, ldct, bt);
    } else {
        gemm_nt_bf16_kernel<128, false, 256><<<dim3((uint32_t)blocks), dim3(256), 0, stream>>>(p, ldp, q, ldq, M, N, K, alpha, beta, dt, lddt, c, ldc, ct, ldct, bt);
    }
    return hipGetLastError();
}

}  // namespace adagc

// The matrix-core GEMM through the C ABI, single and batched (see include/adagc.h).
extern "C" int adagc_muon_gemm_nt_batched(const void* P, int64_t ldp, const void* Q, int64_t ldq, int64_t M, int64_t N, int64_t K,
                                          float alpha, float beta, const void* Dt, int64_t lddt, void* C, int64_t ldc, void* Ct,
                                          int64_t ldct, int32_t symmetric, int64_t batch, const int64_t* strides, void* stream)
{
    if (!P || !Q || batch < 1 || (batch > 1 && !strides)) return ADAGC_ERR_INVALID_ARG;
    if (M > INT32_MAX || N > INT32_MAX || K > INT32_MAX || ldp > INT32_MAX || ldq > INT32_MAX || lddt > INT32_MAX ||
        ldc > INT32_MAX || ldct > INT32_MAX || batch > INT32_MAX)
        return ADAGC_ERR_TOO_LARGE;
    if (ldp < K || ldq < K || (Dt && lddt < M) || (C && ldc < N) || (Ct && ldct < M)) return ADAGC_ERR_INVALID_ARG;
    int64_t st[5] = {0, 0, 0, 0, 0};
    if (strides) {
        st[0] = strides[0];
        st[1] = strides[1];
        st[2] = Dt ? strides[2] : 0;
        st[3] = C ? strides[3] : 0;
        st[4] = Ct ? strides[4] : 0;
        if (symmetric && C == nullptr) st[3] = st[4];
    }
    const hipError_t e = adagc::launch_gemm_nt_bf16(P, (int)ldp, Q, (int)ldq, (int)M, (int)N, (int)K, alpha, beta, Dt, (int)lddt,
                                                    C, (int)ldc, Ct, (int)ldct, static_cast<hipStream_t>(stream), symmetric != 0,
                                                    (int)batch, st[0], st[1], st[2], st[3], st[4]);
    if (e == hipErrorInvalidValue) return ADAGC_ERR_INVALID_ARG;
    return e == hipSuccess ? ADAGC_OK : ADAGC_ERR_HIP;
}

extern "C" int adagc_muon_gemm_nt(const void* P, int64_t ldp, const void* Q, int64_t ldq, int64_t M, int64_t N, int64_t K,
                                  float alpha, float beta, const void* Dt, int64_t lddt, void* C, int64_t ldc, void* Ct,
                                  int64_t ldct, int32_t symmetric, void* stream)
{
    return adagc_muon_gemm_nt_batched(P, ldp, Q, ldq, M, N, K, alpha, beta, Dt, lddt, C, ldc, Ct, ldct, symmetric, 1, nullptr, stream);
}
