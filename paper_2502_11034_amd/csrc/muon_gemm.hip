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
// Dt (N x M).  The epilogue goes through LDS, so that all of these are 16-byte accesses along rows (store_result).
//
// A = X X^T and A A are symmetric: for those only the tiles on and below the diagonal are computed and each is
// written twice, to its place and to its mirror image, which saves about a quarter of a step's multiplications.
//
// M and N are multiples of the 128 x 128 block tile and K of 128 (two 64-deep tiles): the caller (muon.hip) keeps every matrix
// in zero-padded workspace buffers, and zero rows and columns stay zero through the iteration.
//
// Tiling: 128 x 128 block tile with 4 waves in a 2 x 2 grid (each wave 64 x 64 = 2 x 2 accumulators of
// v_mfma_f32_32x32x16_bf16, fp32 accumulation); where the launch has enough of them to fill the compute units,
// 256 x 256 tiles with 8 waves in a 4 x 2 grid (each 64 x 128).  One launch can cover a batch of equal-shaped
// products.  Operand tiles, 64 deep, are loaded from global memory straight into LDS (global_load_lds_dwordx4, no
// staging registers), swizzled against bank conflicts, double-buffered; the fragment reads of the next 16-deep
// slice overlap the current slice's multiplications.  Workgroups are dealt to the 8 XCDs in turn, so block ids are
// remapped to give each XCD (one L2 each) a contiguous band of output tiles.

#include "muon_internal.h"

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
#define ADAGC_GEMM_BIG_THREADS 512      // lanes of a 256 x 256 workgroup: 8 waves; 4 waves (256) measured no better overall
#endif
constexpr int kBK = 64;
constexpr int kVecPerRow = kBK / 8;                    // 16-byte vectors per tile row

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    uint32_t rounded = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    return ((u & 0x7FFFFFFFu) > 0x7F800000u) ? ((u >> 16) | 0x40u) : rounded;
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// Which output tile a workgroup computes, and the batch's matrix it belongs to.
struct TilePlace {
    int tile_m, tile_n, z;
};

// XCD-aware tile order: block b runs on XCD b mod 8; XCD x gets the x-th contiguous eighth of the tiles of the whole
// batch (with 8 or more matrices in the batch an XCD then stays on its own matrices).  Within a matrix: SYM walks the
// lower triangle row by row; otherwise the tiles are walked in panels of kGroupM tile rows, down the rows of a panel
// first: the workgroups that run at the same time on an XCD then form a patch a few tiles high and wide and share
// both operands in its L2.
template <int BT, bool SYM>
__device__ __forceinline__ TilePlace place_tile(int b, int all_tiles, int M, int N)
{
    const int tiles_n = N / BT;
    const int n_tiles = SYM ? tiles_n * (tiles_n + 1) / 2 : (M / BT) * tiles_n;     // per matrix
    if (all_tiles % 8 == 0) b = (b % 8) * (all_tiles / 8) + b / 8;
    TilePlace t;
    t.z = b / n_tiles;
    b -= t.z * n_tiles;
    if constexpr (SYM) {
        // b-th tile of the lower triangle: row r starts at r (r + 1) / 2
        int r = (int)((sqrtf(8.0f * (float)b + 1.0f) - 1.0f) * 0.5f);
        while (r * (r + 1) / 2 > b) --r;
        while ((r + 1) * (r + 2) / 2 <= b) ++r;
        t.tile_m = r;
        t.tile_n = b - r * (r + 1) / 2;
    } else {
        constexpr int kGroupM = ADAGC_GEMM_GROUP_M;
        const int tiles_m = M / BT;
        const int per_group = kGroupM * tiles_n;
        const int group = b / per_group;
        const int first_m = group * kGroupM;
        const int rows_here = (tiles_m - first_m) < kGroupM ? (tiles_m - first_m) : kGroupM;
        const int in_group = b - group * per_group;
        t.tile_m = first_m + in_group % rows_here;
        t.tile_n = in_group / rows_here;
    }
    return t;
}

// s_waitcnt for "at most n vector-memory operations of this wave still outstanding", nothing else waited for
#define ADAGC_WAIT_VMEM(n) __builtin_amdgcn_s_waitcnt(((n) & 0xF) | (((n) >> 4) << 14) | (7 << 4) | (0xF << 8))
// nothing is moved across this point by the compiler's instruction scheduler
#define ADAGC_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

// 16 bytes per lane from global memory straight into LDS: lane i's data lands at lds_dst + 16 i (lds_dst: the same in
// all lanes).  The instruction takes the LDS byte address from M0, and wants one wait state after M0 is written; M0 is
// put back afterwards, so the compiler's own uses of it are not disturbed.
// Written as inline assembly rather than through the compiler's builtin so that the compiler does not track these
// loads: it would count each as outstanding in both of its memory counters ("flat" access) and, while one is, turn
// every wait for an LDS read into a wait for all LDS reads, which serialises the fragment reads with the
// multiplications.  The waits for these loads are explicit (ADAGC_WAIT_VMEM) wherever their data is needed.
__device__ __forceinline__ void load_to_lds_16(const void* src, const uint16_t* lds_dst)
{
    const uint32_t lds_addr = (uint32_t)reinterpret_cast<uintptr_t>(lds_dst);      // low half of the flat address = LDS offset
    uint32_t saved_m0;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\ts_mov_b32 m0, %0"
                 : "=&s"(saved_m0)
                 : "s"(lds_addr), "v"(src)
                 : "memory");
}

// Epilogue of a workgroup: bf16(alpha acc + beta D) to Ct and C, staged through LDS so that every global access is a
// 16-byte vector per lane along a row of the array it touches.  (In the accumulator layout a lane holds 4 consecutive
// rows of one column and 32 lanes hold 32 columns: stored directly, that is 8 bytes per lane for Ct and D, each in a
// different cache line, and 2 bytes per lane for C.)
//
// The staging tile T holds the BT x BT result transposed, T[c][r] = result(r, c), as Ct and Dt do: row c of T is BT
// contiguous elements of global row tile_n BT + c of Ct.  Within a row the 16-byte chunks are permuted: chunk g sits
// at position g ^ f(c), f(c) = (c ^ (c / chunks)) mod chunks, which spreads over the LDS banks both the accumulator-
// layout accesses (32 lanes = 32 consecutive c, one r) and the reads of the C pass (8 consecutive c at a time).
//   1. Dt's tile is loaded into T (global_load_lds, the permutation applied on the global side);
//   2. every lane reads the D values of its accumulator elements from T, and writes the rounded results back to the
//      same places;
//   3. T is written out row by row to Ct, and, gathered by columns, row by row to C.
// Accumulator register r of lane l is element (row (r/4)*8 + (l/32)*4 + r%4, column l%32) of its 32 x 32 block.
// On entry no wave reads LDS any more (all are past the main loop's last barrier).
template <int BT, int kMI, int kNI, bool SYM, int kWaves>
__device__ __forceinline__ void store_result(uint16_t* T, const f32x16 (&acc)[kMI][kNI], int lane, int wave, int wave_row, int wave_col,
                                             int tile_m, int tile_n, float alpha, float beta, const uint16_t* __restrict__ Dt,
                                             int lddt, uint16_t* __restrict__ C, int ldc, uint16_t* __restrict__ Ct, int ldct)
{
    constexpr int kChunks = BT / 8;                         // 16-byte chunks per row of T
    constexpr int kChunkBits = BT == 256 ? 5 : 4;
    static_assert((1 << kChunkBits) == kChunks, "BT is 128 or 256");
    constexpr int kRowsPerInst = 64 / kChunks;              // rows of T one wave-wide 16-byte access covers: 2 or 4
    constexpr int kInsts = BT / kRowsPerInst / kWaves;      // such accesses per wave for the whole tile
    auto f = [](int c) { return (c ^ (c >> kChunkBits)) & (kChunks - 1); };
    const size_t row0_g = (size_t)tile_m * BT, col0_g = (size_t)tile_n * BT;

    // lane i of a row-wise access: row c = first + i / kChunks of T, position i % kChunks, i.e. chunk (i % kChunks) ^ f(c)
    const int rw_row = lane / kChunks;
    const int rw_pos = lane % kChunks;
    if (Dt) {
#pragma unroll
        for (int u = 0; u < kInsts; ++u) {
            const int first = (u * kWaves + wave) * kRowsPerInst;
            const int c = first + rw_row;
            const int g = rw_pos ^ f(c);
            load_to_lds_16(Dt + (col0_g + c) * lddt + row0_g + g * 8, T + first * BT);
        }
        ADAGC_WAIT_VMEM(0);
        __syncthreads();
    }
    const int col_in = lane & 31;
    const int row_in = (lane >> 5) * 4;
#pragma unroll
    for (int i = 0; i < kMI; ++i)
#pragma unroll
        for (int j = 0; j < kNI; ++j) {
            const int c = wave_col + j * 32 + col_in;
            const int fc = f(c);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int r = wave_row + i * 32 + q * 8 + row_in;
                u32x2v* slot = reinterpret_cast<u32x2v*>(T + c * BT + (((r >> 3) ^ fc) << 3) + (r & 7));
                float v[4] = {alpha * acc[i][j][q * 4 + 0], alpha * acc[i][j][q * 4 + 1], alpha * acc[i][j][q * 4 + 2],
                              alpha * acc[i][j][q * 4 + 3]};
                if (Dt) {
                    const u32x2v d = *slot;
                    v[0] = fmaf(beta, bf16_lo(d.x), v[0]);
                    v[1] = fmaf(beta, bf16_hi(d.x), v[1]);
                    v[2] = fmaf(beta, bf16_lo(d.y), v[2]);
                    v[3] = fmaf(beta, bf16_hi(d.y), v[3]);
                }
                u32x2v o;
                o.x = f32_to_bf16_rne(v[0]) | (f32_to_bf16_rne(v[1]) << 16);
                o.y = f32_to_bf16_rne(v[2]) | (f32_to_bf16_rne(v[3]) << 16);
                *slot = o;
            }
        }
    __syncthreads();
    if (Ct) {
#pragma unroll
        for (int u = 0; u < kInsts; ++u) {
            const int c = (u * kWaves + wave) * kRowsPerInst + rw_row;
            const int g = rw_pos ^ f(c);
            const u32x4 v = *reinterpret_cast<const u32x4*>(T + c * BT + rw_pos * 8);
            *reinterpret_cast<u32x4*>(Ct + (col0_g + c) * ldct + row0_g + g * 8) = v;
        }
    }
    if (SYM ? (tile_m != tile_n) : (C != nullptr)) {        // SYM: the mirror image, C is the same array as Ct
        // one access: 8 rows r of the result, 8 chunks (64 columns) of each; lane i takes row i / 8, chunk i % 8
        constexpr int kColGroups = BT / 64;
        constexpr int kCInsts = (BT / 8) * kColGroups / kWaves;
        const int cr = lane >> 3, cc = lane & 7;
#pragma unroll 4
        for (int u = 0; u < kCInsts; ++u) {
            const int n = u * kWaves + wave;
            const int r = (n / kColGroups) * 8 + cr;
            const int c0 = (n % kColGroups) * 64 + cc * 8;
            uint32_t w[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int ca = c0 + 2 * e, cb = ca + 1;
                const uint32_t lo = T[ca * BT + (((r >> 3) ^ f(ca)) << 3) + (r & 7)];
                const uint32_t hi = T[cb * BT + (((r >> 3) ^ f(cb)) << 3) + (r & 7)];
                w[e] = lo | (hi << 16);
            }
            u32x4 v;
            v.x = w[0];
            v.y = w[1];
            v.z = w[2];
            v.w = w[3];
            *reinterpret_cast<u32x4*>(C + (row0_g + r) * ldc + col0_g + c0) = v;
        }
    }
}

// BT x BT block tile (128 or 256), operand tiles loaded from global memory straight into LDS.
// One global_load_lds_dwordx4 of a wave writes 1024 contiguous LDS bytes, lane i the i-th 16: that is 8 rows of a
// 64-deep tile stored without padding.  Bank conflicts of the fragment reads (16 lanes = 16 consecutive rows per
// clock over 64 banks) are avoided by a swizzle instead: the 16-byte vector v of tile row r sits at position
// v ^ ((r / 2) mod 8) of its LDS row, which the loading lane applies on the global side.
template <int BT, bool SYM, int kGemmThreads>
__global__ __launch_bounds__(kGemmThreads) void gemm_nt_bf16_kernel(
    const uint16_t* __restrict__ P, int ldp, const uint16_t* __restrict__ Q, int ldq, int M, int N, int K,
    float alpha, float beta, const uint16_t* __restrict__ Dt, int lddt, uint16_t* __restrict__ C, int ldc,
    uint16_t* __restrict__ Ct, int ldct, GemmBatch bt)
{
    constexpr int kWaves = kGemmThreads / 64;
    constexpr int kWM = kGemmThreads / 128;                // waves in a kWM x 2 grid
    constexpr int kTM = BT / kWM, kTN = BT / 2;            // wave tile
    constexpr int kMI = kTM / 32, kNI = kTN / 32;          // 32 x 32 accumulators per wave
    constexpr int kRowsPerLoad = 64 / kVecPerRow;          // tile rows one wave-wide load covers: 8
    constexpr int kLoads = BT / kRowsPerLoad / kWaves;     // loads per wave per operand tile
    static_assert(kWaves % 2 == 0, "the swizzle of a load is taken from the wave's parity");
    // two buffers of a P and a Q tile each; the epilogue reuses all of it as one BT x BT staging tile (or half of it)
    __shared__ __attribute__((aligned(16))) uint16_t lds[4 * BT * kBK];
    uint16_t* const lds_p0 = lds;
    uint16_t* const lds_q0 = lds + BT * kBK;
    uint16_t* const lds_p1 = lds + 2 * BT * kBK;
    uint16_t* const lds_q1 = lds + 3 * BT * kBK;
    static_assert(4 * BT * kBK >= BT * BT, "the staging tile of the epilogue must fit");

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // the same in all lanes: kept in a scalar register
    const int wm = wave >> 1, wn = wave & 1;

    const TilePlace tp = place_tile<BT, SYM>((int)blockIdx.x, (int)gridDim.x, M, N);
    const int tile_m = tp.tile_m, tile_n = tp.tile_n;
    P += (size_t)tp.z * bt.stride_p;
    Q += (size_t)tp.z * bt.stride_q;
    if (Dt) Dt += (size_t)tp.z * bt.stride_dt;
    if (C) C += (size_t)tp.z * bt.stride_c;
    if (Ct) Ct += (size_t)tp.z * bt.stride_ct;
    const uint16_t* Pt = P + (size_t)tile_m * BT * ldp;
    const uint16_t* Qt = Q + (size_t)tile_n * BT * ldq;

    f32x16 acc[kMI][kNI];
#pragma unroll
    for (int i = 0; i < kMI; ++i)
#pragma unroll
        for (int j = 0; j < kNI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // Load u of this wave covers tile rows first .. first + 7, first = (u kWaves + wave) 8; lane i writes LDS row
    // first + i / 8, position i mod 8, so it fetches vector (i mod 8) ^ ((row / 2) mod 8) of that row, and
    // (row / 2) mod 8 = (4 (wave mod 2) + i / 16) mod 8 because kWaves is even.
    // The address is split into a part common to the wave (scalar registers) and one 32-bit offset per lane.
    const int load_row = lane >> 3;
    const int load_vec = (lane & 7) ^ ((((wave & 1) << 2) + (lane >> 4)) & 7);
    const uint32_t lane_off_p = (uint32_t)(load_row * ldp + load_vec * 8) * 2u;      // bytes
    const uint32_t lane_off_q = (uint32_t)(load_row * ldq + load_vec * 8) * 2u;
    auto load_tile = [&](int kt, uint16_t* bp, uint16_t* bq) {
#pragma unroll
        for (int u = 0; u < kLoads; ++u) {
            const int first = (u * kWaves + wave) * kRowsPerLoad;
            const char* row0 = reinterpret_cast<const char*>(Pt + (size_t)first * ldp + kt * kBK);
            load_to_lds_16(row0 + lane_off_p, bp + first * kBK);
        }
#pragma unroll
        for (int u = 0; u < kLoads; ++u) {
            const int first = (u * kWaves + wave) * kRowsPerLoad;
            const char* row0 = reinterpret_cast<const char*>(Qt + (size_t)first * ldq + kt * kBK);
            load_to_lds_16(row0 + lane_off_q, bq + first * kBK);
        }
    };
    // Fragment addressing: lane l holds row l mod 32 of its 32-row block and the 16-byte vector 2 kk + l / 32 of that
    // row; a block's first row is a multiple of 32, so (row / 2) mod 8 = (l / 2) mod 8.
    const int frag_row = lane & 31;
    const int frag_hi = lane >> 5;
    const int frag_x = (lane >> 1) & 7;
    auto read_frags = [&](const uint16_t* bp, const uint16_t* bq, int kk, bf16x8 (&fa)[kMI], bf16x8 (&fb)[kNI]) {
        const int pos = ((kk * 2 + frag_hi) ^ frag_x) * 8;
#pragma unroll
        for (int i = 0; i < kMI; ++i) fa[i] = *reinterpret_cast<const bf16x8*>(bp + (wm * kTM + i * 32 + frag_row) * kBK + pos);
#pragma unroll
        for (int j = 0; j < kNI; ++j) fb[j] = *reinterpret_cast<const bf16x8*>(bq + (wn * kTN + j * 32 + frag_row) * kBK + pos);
    };
    auto multiply = [&](const bf16x8 (&fa)[kMI], const bf16x8 (&fb)[kNI]) {
#pragma unroll
        for (int i = 0; i < kMI; ++i)
#pragma unroll
            for (int j = 0; j < kNI; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    };

    // Software pipeline.  A 64-deep tile is four 16-deep slices; the fragments of slice s+1 are read from LDS while
    // slice s is multiplied (two fragment register sets).  Before the last slice of tile k is multiplied, every wave
    // has read all of tile k: after the barrier there the tile's buffer is free for the loads of tile k+2, which then
    // have until the same point of tile k+1 to arrive, and the first slice of tile k+1 is read during the last
    // multiplications of tile k.
    bf16x8 fa0[kMI], fb0[kNI], fa1[kMI], fb1[kNI];
    const int k_tiles = K / kBK;          // even: K is a multiple of 128
    // slices 0 to 2 of the tile in (cur_p, cur_q); on entry set 0 holds slice 0, on exit set 1 holds slice 3, this
    // wave's loads have arrived and all waves are past the barrier
    auto first_three_slices = [&](const uint16_t* cur_p, const uint16_t* cur_q) {
        read_frags(cur_p, cur_q, 1, fa1, fb1);
        ADAGC_SCHED_FENCE();
        multiply(fa0, fb0);
        ADAGC_SCHED_FENCE();
        read_frags(cur_p, cur_q, 2, fa0, fb0);
        ADAGC_SCHED_FENCE();
        multiply(fa1, fb1);
        ADAGC_SCHED_FENCE();
        read_frags(cur_p, cur_q, 3, fa1, fb1);
        ADAGC_SCHED_FENCE();
        multiply(fa0, fb0);
        ADAGC_SCHED_FENCE();
        ADAGC_WAIT_VMEM(0);
        __syncthreads();
    };
    load_tile(0, lds_p0, lds_q0);
    ADAGC_WAIT_VMEM(0);
    __syncthreads();
    load_tile(1, lds_p1, lds_q1);
    read_frags(lds_p0, lds_q0, 0, fa0, fb0);
    ADAGC_SCHED_FENCE();
    first_three_slices(lds_p0, lds_q0);
    for (int kt = 0; kt + 2 < k_tiles; kt += 2) {
        // tile kt (buffer 0): slice 3 left; tile kt+1 is in buffer 1
        load_tile(kt + 2, lds_p0, lds_q0);
        read_frags(lds_p1, lds_q1, 0, fa0, fb0);
        ADAGC_SCHED_FENCE();
        multiply(fa1, fb1);
        ADAGC_SCHED_FENCE();
        first_three_slices(lds_p1, lds_q1);
        // tile kt+1 (buffer 1): slice 3 left; tile kt+2 is in buffer 0
        load_tile(kt + 3, lds_p1, lds_q1);
        read_frags(lds_p0, lds_q0, 0, fa0, fb0);
        ADAGC_SCHED_FENCE();
        multiply(fa1, fb1);
        ADAGC_SCHED_FENCE();
        first_three_slices(lds_p0, lds_q0);
    }
    // the last two tiles: k_tiles - 2 (buffer 0, slice 3 left) and k_tiles - 1 (buffer 1)
    read_frags(lds_p1, lds_q1, 0, fa0, fb0);
    ADAGC_SCHED_FENCE();
    multiply(fa1, fb1);
    ADAGC_SCHED_FENCE();
    first_three_slices(lds_p1, lds_q1);
    multiply(fa1, fb1);
    store_result<BT, kMI, kNI, SYM, kWaves>(lds, acc, lane, wave, wm * kTM, wn * kTN, tile_m, tile_n, alpha, beta, Dt, lddt, C, ldc, Ct,
                                            ldct);
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
    auto misaligned = [](const void* a) { return (reinterpret_cast<uintptr_t>(a) & 15u) != 0; };      // 16-byte vector accesses
    if (misaligned(P) || misaligned(Q) || misaligned(Dt) || misaligned(C) || misaligned(Ct)) return hipErrorInvalidValue;
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
