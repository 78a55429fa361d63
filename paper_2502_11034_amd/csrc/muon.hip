// Elementwise kernels of the Muon step with AdaGC's clipped gradient (Muon is the optimizer the paper pairs
// AdaGC with in "Optimizer Compatibility: Muon and Lion", Sec. 5.4; its rule is the published one, the paper
// prints none):
//
//   muon_momentum_kernel    per chunk:  M <- mu M + h g;  partial sum of squares of U
//                                       (U = h g + mu M in the Nesterov form, U = M otherwise)
//   muon_normalise_kernel   per matrix: X0 = bf16(U / (||U||_F + 1e-7)) into the zero-padded workspace, row-major
//                                       and transposed (the matrix-core products want both, see muon_gemm.hip)
//   muon_apply_kernel       per matrix: theta <- theta - lr (wd theta + scale O), optional bf16 copy
//
// The clip coefficient h of every tensor comes from the same norm and rule kernels as for AdamW and Lion
// (kernels.hip); the Newton-Schulz products run in muon_gemm.hip.  Arithmetic is double with one rounding per
// stored value, as in the other update kernels; reductions are in fixed order.

#include "muon_internal.h"

namespace adagc {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    uint32_t rounded = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    return ((u & 0x7FFFFFFFu) > 0x7F800000u) ? ((u >> 16) | 0x40u) : rounded;
}

template <bool BF16>
__device__ __forceinline__ float grad_at(const void* g, int64_t j)
{
    if constexpr (BF16) return __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(g)[j] << 16);
    else return reinterpret_cast<const float*>(g)[j];
}

// M' and U of one element.  The momentum is stored as fp32; U uses the stored value.
__device__ __forceinline__ double momentum_elem(double h, double mu, int nesterov, float g, float m_prev, float* m_new)
{
    const double gh = h * (double)g;
    const float m = (float)(mu * (double)m_prev + gh);
    *m_new = m;
    return nesterov ? gh + mu * (double)m : (double)m;
}

__device__ __forceinline__ double wave_sum(double x)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);    // a fixed butterfly: same value in every lane
    return x;
}

// One workgroup per chunk (positions b, b+grid, ... of the list): momentum update and the chunk's sum of U^2.
// Tensors whose pointers allow it are walked in 128-bit vectors (4 elements per lane and access, streaming loads
// and stores: every element is touched once per kernel); the others, and the last len mod 4 elements, one by one.
template <bool BF16>
__global__ __launch_bounds__(kBlock) void muon_momentum_kernel(DeviceTables t, double mu, int nesterov)
{
    __shared__ double wave_sums[kWavesPerBlock];
    const int tid = threadIdx.x;
    for (uint32_t k = blockIdx.x; k < t.n_chunks; k += gridDim.x) {
        const uint32_t c = t.schedule ? t.schedule[k] : k;     // the visiting order of the norm kernel (XCD-aware)
        const ChunkRef ck = t.chunks[c];
        const TensorArgs& ta = t.targs[ck.tensor];
        const int64_t first = (int64_t)ck.index * kChunkElems;
        const int64_t rest = ta.numel - first;
        const int len = rest < (int64_t)kChunkElems ? (int)rest : kChunkElems;
        const double h = t.coef64[ck.tensor];
        float* m = reinterpret_cast<float*>(ta.exp_avg) + first;
        double acc = 0.0;
        int done = 0;
        if (ta.vec_ok) {
            const int groups = len / 4;
            f32x4* m4 = reinterpret_cast<f32x4*>(m);
            auto load_g = [&](int j, float (&g)[4]) {
                if constexpr (BF16) {
                    const u32x2 w = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(reinterpret_cast<const uint16_t*>(ta.grad) + first) + j);
                    g[0] = __uint_as_float(w.x << 16);
                    g[1] = __uint_as_float(w.x & 0xFFFF0000u);
                    g[2] = __uint_as_float(w.y << 16);
                    g[3] = __uint_as_float(w.y & 0xFFFF0000u);
                } else {
                    const f32x4 w = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(ta.grad) + first) + j);
                    g[0] = w.x; g[1] = w.y; g[2] = w.z; g[3] = w.w;
                }
            };
            auto update4 = [&](int j, const float (&g)[4], const f32x4 mp) {
                f32x4 mn;
                float e;
                double u = momentum_elem(h, mu, nesterov, g[0], mp.x, &e); mn.x = e; acc = fma(u, u, acc);
                u = momentum_elem(h, mu, nesterov, g[1], mp.y, &e); mn.y = e; acc = fma(u, u, acc);
                u = momentum_elem(h, mu, nesterov, g[2], mp.z, &e); mn.z = e; acc = fma(u, u, acc);
                u = momentum_elem(h, mu, nesterov, g[3], mp.w, &e); mn.w = e; acc = fma(u, u, acc);
                __builtin_nontemporal_store(mn, m4 + j);
            };
            if (len == kChunkElems) {
                // a full chunk is 16 vectors per lane: 8 of each array in flight at a time
                constexpr int kPerLane = kChunkElems / 4 / kBlock, kFlight = 8;
                static_assert(kPerLane % kFlight == 0, "chunk size and block size");
#pragma unroll
                for (int base = 0; base < kPerLane; base += kFlight) {
                    float g[kFlight][4];
                    f32x4 mp[kFlight];
#pragma unroll
                    for (int v = 0; v < kFlight; ++v) {
                        load_g((base + v) * kBlock + tid, g[v]);
                        mp[v] = __builtin_nontemporal_load(m4 + (base + v) * kBlock + tid);
                    }
#pragma unroll
                    for (int v = 0; v < kFlight; ++v) update4((base + v) * kBlock + tid, g[v], mp[v]);
                }
            } else {
                for (int j = tid; j < groups; j += kBlock) {
                    float g[4];
                    load_g(j, g);
                    update4(j, g, __builtin_nontemporal_load(m4 + j));
                }
            }
            done = groups * 4;
        }
        for (int j = done + tid; j < len; j += kBlock) {
            float m_new;
            const double u = momentum_elem(h, mu, nesterov, grad_at<BF16>(ta.grad, first + j), m[j], &m_new);
            m[j] = m_new;
            acc = fma(u, u, acc);
        }
        const double s = wave_sum(acc);
        if ((tid & 63) == 0) wave_sums[tid >> 6] = s;
        __syncthreads();
        if (tid == 0) {
            double b = wave_sums[0];
#pragma unroll
            for (int w = 1; w < kWavesPerBlock; ++w) b += wave_sums[w];
            t.partials[c] = b;
        }
        __syncthreads();
    }
}

// X0 of one matrix.  The source U (rows x cols, recomputed from g and the updated momentum) is walked in 64 x 64
// tiles of its extent padded to (rows_p, cols_p); every element of the padded extent is written: zeros outside
// the matrix.  same[r][c] (leading dimension ld_same) receives the tile as is, trans[c][r] (ld_trans) its
// transpose, through LDS so that both are written along their rows.
// VEC (cols a multiple of 4, g and m 16-byte aligned; bf16 g 8-byte): a lane handles 4 consecutive elements of a
// row on the way in and 4 consecutive elements of a transposed row on the way out: 16-byte loads, 8-byte stores.
template <bool BF16, bool VEC>
__global__ __launch_bounds__(256) void muon_normalise_kernel(const void* g, const float* m, int64_t rows, int64_t cols,
                                                              int64_t rows_p, int64_t cols_p, const double* coef,
                                                              const double* sumsq, double mu, int nesterov,
                                                              uint16_t* same, int64_t ld_same, uint16_t* trans, int64_t ld_trans)
{
    constexpr int kTileLd = VEC ? 68 : 66;                 // u16 per LDS row (VEC: rows stay 8-byte aligned)
    __shared__ __attribute__((aligned(8))) uint16_t tile[64 * kTileLd];
    const int64_t r0 = (int64_t)blockIdx.y * 64, c0 = (int64_t)blockIdx.x * 64;
    const double h = *coef;
    const double denom = sqrt(*sumsq) + 1e-7;
    auto x0_bits = [&](float gv, float mv) {
        const double gh = h * (double)gv;
        const double u = nesterov ? gh + mu * (double)mv : (double)mv;         // m already holds this step's momentum
        return f32_to_bf16_bits((float)(u / denom));
    };
    if constexpr (VEC) {
        const int q = (threadIdx.x & 15) * 4, p = threadIdx.x >> 4;            // 16 lanes per row, 16 rows per pass
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int tr = p + 16 * k;
            const int64_t r = r0 + tr, c = c0 + q;
            u32x2 bits = {0u, 0u};
            if (r < rows && c < cols) {
                const int64_t j = r * cols + c;
                float gv[4];
                if constexpr (BF16) {
                    const u32x2 w = *reinterpret_cast<const u32x2*>(reinterpret_cast<const uint16_t*>(g) + j);
                    gv[0] = __uint_as_float(w.x << 16);
                    gv[1] = __uint_as_float(w.x & 0xFFFF0000u);
                    gv[2] = __uint_as_float(w.y << 16);
                    gv[3] = __uint_as_float(w.y & 0xFFFF0000u);
                } else {
                    const f32x4 w = *reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(g) + j);
                    gv[0] = w.x; gv[1] = w.y; gv[2] = w.z; gv[3] = w.w;
                }
                const f32x4 mv = *reinterpret_cast<const f32x4*>(m + j);
                bits.x = x0_bits(gv[0], mv.x) | (x0_bits(gv[1], mv.y) << 16);
                bits.y = x0_bits(gv[2], mv.z) | (x0_bits(gv[3], mv.w) << 16);
            }
            *reinterpret_cast<u32x2*>(&tile[tr * kTileLd + q]) = bits;
            if (r < rows_p && c < cols_p) *reinterpret_cast<u32x2*>(same + r * ld_same + c) = bits;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int tc = p + 16 * k;                                         // column of the tile = row of the transpose
            const int64_t c = c0 + tc, r = r0 + q;
            if (r < rows_p && c < cols_p) {
                u32x2 bits;
                bits.x = (uint32_t)tile[(q + 0) * kTileLd + tc] | ((uint32_t)tile[(q + 1) * kTileLd + tc] << 16);
                bits.y = (uint32_t)tile[(q + 2) * kTileLd + tc] | ((uint32_t)tile[(q + 3) * kTileLd + tc] << 16);
                *reinterpret_cast<u32x2*>(trans + c * ld_trans + r) = bits;
            }
        }
    } else {
        const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
#pragma unroll 4
        for (int k = 0; k < 16; ++k) {
            const int64_t r = r0 + ty + 4 * k, c = c0 + tx;
            uint16_t bits = 0;
            if (r < rows && c < cols) {
                const int64_t j = r * cols + c;
                bits = (uint16_t)x0_bits(grad_at<BF16>(g, j), m[j]);
            }
            tile[(ty + 4 * k) * kTileLd + tx] = bits;
            if (r < rows_p && c < cols_p) same[r * ld_same + c] = bits;
        }
        __syncthreads();
#pragma unroll 4
        for (int k = 0; k < 16; ++k) {
            const int64_t c = c0 + ty + 4 * k, r = r0 + tx;
            if (r < rows_p && c < cols_p) trans[c * ld_trans + r] = tile[tx * kTileLd + ty + 4 * k];
        }
    }
}

// theta <- theta - lr (wd theta + scale O) on one matrix; O is bf16 with leading dimension ld_o.
// VEC: cols is a multiple of 4 and theta (and the copy) are 16-byte (8-byte) aligned: 4 elements per lane and access.
template <bool COPY, bool VEC>
__global__ __launch_bounds__(256) void muon_apply_kernel(float* theta, const uint16_t* o, int64_t ld_o, int64_t rows, int64_t cols,
                                                          double lr, double wd, double scale, uint16_t* copy)
{
    const int64_t r = blockIdx.x;
    auto one = [&](float th_f, uint32_t o_bits) {
        const double th = (double)th_f;
        const double ov = (double)__uint_as_float(o_bits << 16);
        return (float)(th - lr * (wd * th + scale * ov));
    };
    if constexpr (VEC) {
        const int64_t groups = cols / 4;
        for (int64_t q = (int64_t)blockIdx.y * 256 + threadIdx.x; q < groups; q += (int64_t)gridDim.y * 256) {
            const int64_t j = r * cols + q * 4;
            const f32x4 th = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(theta + j));
            const u32x2 ow = *reinterpret_cast<const u32x2*>(o + r * ld_o + q * 4);
            f32x4 out;
            out.x = one(th.x, ow.x & 0xFFFFu);
            out.y = one(th.y, ow.x >> 16);
            out.z = one(th.z, ow.y & 0xFFFFu);
            out.w = one(th.w, ow.y >> 16);
            __builtin_nontemporal_store(out, reinterpret_cast<f32x4*>(theta + j));
            if constexpr (COPY) {
                u32x2 cw;
                cw.x = f32_to_bf16_bits(out.x) | (f32_to_bf16_bits(out.y) << 16);
                cw.y = f32_to_bf16_bits(out.z) | (f32_to_bf16_bits(out.w) << 16);
                __builtin_nontemporal_store(cw, reinterpret_cast<u32x2*>(copy + j));
            }
        }
    } else {
        for (int64_t c = (int64_t)blockIdx.y * 256 + threadIdx.x; c < cols; c += (int64_t)gridDim.y * 256) {
            const int64_t j = r * cols + c;
            const float out = one(theta[j], o[r * ld_o + c]);
            theta[j] = out;
            if constexpr (COPY) copy[j] = (uint16_t)f32_to_bf16_bits(out);
        }
    }
}

}  // namespace

hipError_t launch_muon_momentum(const DeviceTables& t, double mu, int nesterov, int grad_bf16, int grid, hipStream_t stream)
{
    if (grad_bf16) muon_momentum_kernel<true><<<dim3(grid), dim3(kBlock), 0, stream>>>(t, mu, nesterov);
    else muon_momentum_kernel<false><<<dim3(grid), dim3(kBlock), 0, stream>>>(t, mu, nesterov);
    return hipGetLastError();
}

hipError_t launch_muon_normalise(const void* g, const void* m, int64_t rows, int64_t cols, int64_t rows_p, int64_t cols_p,
                                 const double* coef, const double* sumsq, double mu, int nesterov, int grad_bf16,
                                 void* same, int64_t ld_same, void* trans, int64_t ld_trans, hipStream_t stream)
{
    const dim3 grid((uint32_t)(cols_p / 64), (uint32_t)(rows_p / 64));
    if (grid.y > 65535u) return hipErrorInvalidValue;
    auto misaligned = [](const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; };
    // the padded extents are multiples of 64 and the workspace rows of 128 elements, so only the caller's arrays decide
    const bool vec = cols % 4 == 0 && !misaligned(g, grad_bf16 ? 8 : 16) && !misaligned(m, 16) && !misaligned(same, 8) &&
                     !misaligned(trans, 8) && ld_same % 4 == 0 && ld_trans % 4 == 0;
    const float* mf = static_cast<const float*>(m);
    uint16_t *sp = static_cast<uint16_t*>(same), *tp = static_cast<uint16_t*>(trans);
#define ADAGC_NORMALISE(B, V) \
    muon_normalise_kernel<B, V><<<grid, dim3(256), 0, stream>>>(g, mf, rows, cols, rows_p, cols_p, coef, sumsq, mu, nesterov, sp, ld_same, tp, ld_trans)
    if (grad_bf16 && vec) ADAGC_NORMALISE(true, true);
    else if (grad_bf16) ADAGC_NORMALISE(true, false);
    else if (vec) ADAGC_NORMALISE(false, true);
    else ADAGC_NORMALISE(false, false);
#undef ADAGC_NORMALISE
    return hipGetLastError();
}

hipError_t launch_muon_apply(void* theta, const void* o, int64_t ld_o, int64_t rows, int64_t cols, double lr, double wd,
                             double scale, void* copy, hipStream_t stream)
{
    auto misaligned = [](const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; };
    const bool vec = cols % 4 == 0 && !misaligned(theta, 16) && !misaligned(o, 8) && ld_o % 4 == 0 && !(copy && misaligned(copy, 8));
    const int64_t per_row = vec ? cols / 4 : cols;
    int64_t col_blocks = (per_row + 255) / 256;
    if (col_blocks > 64) col_blocks = 64;
    const dim3 grid((uint32_t)rows, (uint32_t)col_blocks);
    float* th = static_cast<float*>(theta);
    const uint16_t* ob = static_cast<const uint16_t*>(o);
    uint16_t* cp = static_cast<uint16_t*>(copy);
    if (copy && vec) muon_apply_kernel<true, true><<<grid, dim3(256), 0, stream>>>(th, ob, ld_o, rows, cols, lr, wd, scale, cp);
    else if (copy) muon_apply_kernel<true, false><<<grid, dim3(256), 0, stream>>>(th, ob, ld_o, rows, cols, lr, wd, scale, cp);
    else if (vec) muon_apply_kernel<false, true><<<grid, dim3(256), 0, stream>>>(th, ob, ld_o, rows, cols, lr, wd, scale, nullptr);
    else muon_apply_kernel<false, false><<<grid, dim3(256), 0, stream>>>(th, ob, ld_o, rows, cols, lr, wd, scale, nullptr);
    return hipGetLastError();
}

}  // namespace adagc
