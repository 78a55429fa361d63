// HIP kernels of libadagc for gfx950 (wave64).
//
//   sumsq_partials_kernel   per chunk:   sum of g^2 in fp64              (l2 norm of Sec. 4.1, for Eq. 3)
//   finalize_adagc_kernel   per tensor:  norm, h_i, clip flag, EMA update          (Eq. 3, Alg. 1)
//   tensor_sumsq_kernel / global_rule_kernel / finalize_global_kernel
//                           one coefficient for the whole model: warm-up branch of Alg. 1
//                           (GlobalGC + running minimum), GlobalGC on every step (Eq. 2),
//                           Global AdaGC (Eq. 3 on the model's norm; "Ablation Study", Sec. 5.6)
//   update_kernel           per quarter chunk: clipped gradient into AdamW / Lion  (Alg. 1)
//   direction_stats_kernel / finalize_update_clip_kernel
//                           update clipping (AGC and Clippy rows of Table 2): norms of theta and of the
//                           optimizer's direction per tensor, and the coefficient that scales the direction
//   prepare_step_kernel / global_rule_device_kernel / finalize_device_kernel
//                           the same rules with the step's scalars read from device memory, for a
//                           launch sequence that is recorded once and replayed for later steps
//
// Nothing here is a dense contraction, so there is no MFMA: the streaming kernels
// are bound by HBM and are built around 128-bit coalesced accesses with many
// independent loads in flight per lane.  Reductions are deterministic: a lane
// accumulates its elements in index order, lanes are combined with a fixed DPP
// tree, waves through LDS in wave order, chunks by a second kernel in slot order.
// No floating-point atomics anywhere.

#include "adagc_internal.h"

namespace adagc {
namespace {

// Native clang vectors (the nontemporal builtins do not take HIP's struct vector types).
typedef float    f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// ---------------------------------------------------------------------------------------------
// wave64 reduction in double: rotate-and-add inside each row of 16 lanes with DPP, then read the
// four row totals with readlane and add them in row order.

template <int DPP_CTRL>
__device__ __forceinline__ double dpp_mov(double x)
{
    int lo = __double2loint(x);
    int hi = __double2hiint(x);
    lo = __builtin_amdgcn_update_dpp(0, lo, DPP_CTRL, 0xF, 0xF, false);
    hi = __builtin_amdgcn_update_dpp(0, hi, DPP_CTRL, 0xF, 0xF, false);
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ double readlane_f64(double x, int lane)
{
    int lo = __builtin_amdgcn_readlane(__double2loint(x), lane);
    int hi = __builtin_amdgcn_readlane(__double2hiint(x), lane);
    return __hiloint2double(hi, lo);
}

// All 64 lanes must be active.  Returns the same value in every lane.
__device__ __forceinline__ double wave_sum_f64(double x)
{
    x += dpp_mov<0x128>(x);  // row_ror:8
    x += dpp_mov<0x124>(x);  // row_ror:4
    x += dpp_mov<0x122>(x);  // row_ror:2
    x += dpp_mov<0x121>(x);  // row_ror:1
    double r0 = readlane_f64(x, 0);
    double r1 = readlane_f64(x, 16);
    double r2 = readlane_f64(x, 32);
    double r3 = readlane_f64(x, 48);
    return ((r0 + r1) + r2) + r3;
}

// ---------------------------------------------------------------------------------------------
// loads / stores

template <bool NT, typename T>
__device__ __forceinline__ T ld(const T* p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}

template <bool NT, typename T>
__device__ __forceinline__ void st(T* p, T v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// Four consecutive gradient elements, widened to fp32.  `vec` counts groups of four from `base`.
template <bool BF16, bool NT>
__device__ __forceinline__ f32x4 load_grad4(const void* base, int vec)
{
    if constexpr (BF16) {
        u32x2 r = ld<NT>(reinterpret_cast<const u32x2*>(base) + vec);
        f32x4 o;
        o.x = __uint_as_float(r.x << 16);
        o.y = __uint_as_float(r.x & 0xFFFF0000u);
        o.z = __uint_as_float(r.y << 16);
        o.w = __uint_as_float(r.y & 0xFFFF0000u);
        return o;
    } else {
        return ld<NT>(reinterpret_cast<const f32x4*>(base) + vec);
    }
}

template <bool BF16>
__device__ __forceinline__ float load_grad1(const void* base, int j)
{
    if constexpr (BF16) return bf16_bits_to_float(reinterpret_cast<const uint16_t*>(base)[j]);
    else return reinterpret_cast<const float*>(base)[j];
}

template <bool BF16>
__device__ __forceinline__ const void* grad_chunk_ptr(const void* grad, int64_t first)
{
    if constexpr (BF16) return reinterpret_cast<const uint16_t*>(grad) + first;
    else return reinterpret_cast<const float*>(grad) + first;
}

// fp32 -> bf16, round to nearest even (add half an ulp of the kept part, plus the parity bit).
__device__ __forceinline__ uint32_t float_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    uint32_t rounded = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    uint32_t quiet_nan = (u >> 16) | 0x40u;
    return ((u & 0x7FFFFFFFu) > 0x7F800000u) ? quiet_nan : rounded;
}

__device__ __forceinline__ u32x2 pack_bf16x4(f32x4 v)
{
    u32x2 o;
    o.x = float_to_bf16_bits(v.x) | (float_to_bf16_bits(v.y) << 16);
    o.y = float_to_bf16_bits(v.z) | (float_to_bf16_bits(v.w) << 16);
    return o;
}

struct ChunkView {
    uint32_t tensor;
    int64_t  first;   // first element of the chunk inside its tensor
    int      len;     // 1..kChunkElems
};

__device__ __forceinline__ ChunkView chunk_view(const DeviceTables& t, uint32_t c)
{
    ChunkRef ck = t.chunks[c];
    ChunkView v;
    v.tensor = ck.tensor;
    v.first = (int64_t)ck.index * kChunkElems;
    int64_t rest = t.targs[ck.tensor].numel - v.first;
    v.len = rest < (int64_t)kChunkElems ? (int)rest : kChunkElems;
    return v;
}

// ---------------------------------------------------------------------------------------------
// K1: one fp64 partial sum of squares per chunk.  Workgroup b takes positions b, b+grid, b+2*grid, ...
// of the visiting order (by default the grid has one workgroup per chunk).

__device__ __forceinline__ void acc4(double (&acc)[4], f32x4 g)
{
    double x = (double)g.x, y = (double)g.y, z = (double)g.z, w = (double)g.w;
    acc[0] = fma(x, x, acc[0]);
    acc[1] = fma(y, y, acc[1]);
    acc[2] = fma(z, z, acc[2]);
    acc[3] = fma(w, w, acc[3]);
}

template <bool BF16, bool NTL>
__global__ __launch_bounds__(kBlock) void sumsq_partials_kernel(DeviceTables t)
{
    __shared__ double wave_sums[kWavesPerBlock];
    const int tid = threadIdx.x;

    for (uint32_t k = blockIdx.x; k < t.n_chunks; k += gridDim.x) {
        const uint32_t c = t.schedule ? t.schedule[k] : k;     // no visiting order given: list order
        const ChunkView cv = chunk_view(t, c);
        const TensorArgs& ta = t.targs[cv.tensor];
        const void* g = grad_chunk_ptr<BF16>(ta.grad, cv.first);
        double acc[4] = {0.0, 0.0, 0.0, 0.0};

        if (ta.vec_ok) {
            if (cv.len == kChunkElems) {
                f32x4 r[kVecPerLane];
#pragma unroll
                for (int u = 0; u < kVecPerLane; ++u) r[u] = load_grad4<BF16, NTL>(g, u * kBlock + tid);
#pragma unroll
                for (int u = 0; u < kVecPerLane; ++u) acc4(acc, r[u]);
            } else {
                const int nvec = cv.len >> 2;
                for (int v = tid; v < nvec; v += kBlock) acc4(acc, load_grad4<BF16, NTL>(g, v));
                const int j = (nvec << 2) + tid;
                if (j < cv.len) {
                    double x = (double)load_grad1<BF16>(g, j);
                    acc[0] = fma(x, x, acc[0]);
                }
            }
        } else {
            for (int j = tid; j < cv.len; j += kBlock) {
                double x = (double)load_grad1<BF16>(g, j);
                acc[0] = fma(x, x, acc[0]);
            }
        }

        double s = wave_sum_f64((acc[0] + acc[1]) + (acc[2] + acc[3]));
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

// ---------------------------------------------------------------------------------------------
// K2: per-tensor scalars.  One workgroup per tensor sums that tensor's partial slots in a fixed
// order that depends only on the slot count: lane l owns slots l, l+256, l+512, ... and keeps four
// accumulators (slot row mod 4) so that four loads are in flight; lanes are combined by the
// wave tree, waves through LDS in wave order.

__device__ __forceinline__ double tensor_slot_sum(const DeviceTables& t, const double* slots, uint32_t i,
                                                  double* wave_sums, uint32_t slots_per_chunk = 1)
{
    const uint32_t count = t.targs[i].chunk_count * slots_per_chunk;
    const double* p = slots + (size_t)t.targs[i].chunk_begin * slots_per_chunk;
    double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
    uint32_t k = threadIdx.x;
    for (; k + 3 * kBlock < count; k += 4 * kBlock) {
        const double x0 = p[k], x1 = p[k + kBlock], x2 = p[k + 2 * kBlock], x3 = p[k + 3 * kBlock];
        a0 += x0; a1 += x1; a2 += x2; a3 += x3;
    }
    if (k < count) a0 += p[k];
    if (k + kBlock < count) a1 += p[k + kBlock];
    if (k + 2 * kBlock < count) a2 += p[k + 2 * kBlock];
    const double s = wave_sum_f64((a0 + a1) + (a2 + a3));
    if ((threadIdx.x & 63) == 0) wave_sums[threadIdx.x >> 6] = s;
    __syncthreads();
    double total = wave_sums[0];
#pragma unroll
    for (int w = 1; w < kWavesPerBlock; ++w) total += wave_sums[w];
    return total;
}

// AdaGC branch of Alg. 1 / Eq. 3 for tensor i with sum of squares s, in double, with separately rounded
// operations.  One lane.
__device__ __forceinline__ void adagc_rule(const DeviceTables& t, float* ema, const RuleArgs& r, uint32_t i, double s)
{
    const double norm = sqrt(s);
    const double gamma_prev = (double)ema[i];
    const double threshold = __dmul_rn(r.lambda_rel, gamma_prev);
    const bool active = norm > threshold;                 // strict; false if either side is NaN
    const double h = active ? __ddiv_rn(threshold, norm) : 1.0;
    const double clipped_norm = active ? threshold : norm;
    const double gamma_new = __dadd_rn(__dmul_rn(r.ema_beta, gamma_prev),
                                       __dmul_rn(__dsub_rn(1.0, r.ema_beta), clipped_norm));
    t.sumsq[i] = s;
    t.norm[i] = (float)norm;
    t.coef[i] = (float)h;
    t.coef64[i] = h;
    t.flag[i] = active ? 1 : 0;
    ema[i] = (float)gamma_new;
}

__global__ __launch_bounds__(kBlock) void finalize_adagc_kernel(DeviceTables t, float* ema, RuleArgs r)
{
    __shared__ double wave_sums[kWavesPerBlock];
    const uint32_t i = blockIdx.x;
    const double s = tensor_slot_sum(t, t.partials, i, wave_sums);
    if (threadIdx.x == 0) adagc_rule(t, ema, r, i, s);
}

// Global stage 1: per-tensor sum of squares only.
__global__ __launch_bounds__(kBlock) void tensor_sumsq_kernel(DeviceTables t)
{
    __shared__ double wave_sums[kWavesPerBlock];
    const uint32_t i = blockIdx.x;
    const double s = tensor_slot_sum(t, t.partials, i, wave_sums);
    if (threadIdx.x == 0) t.sumsq[i] = s;
}

// Global stage 2: the model's norm over all tensors (fixed order) and one coefficient for the
// whole model.  Warm-up steps and the GlobalGC mode use Eq. 2; the Global AdaGC mode applies Eq. 3
// (and, during warm-up, the running minimum of Alg. 1) to the model's norm with the single gamma
// kept in ema[0]; the ZClip mode applies Table 2's z-score rule with its mean in ema[0] and its
// variance in ema[1].
__device__ __forceinline__ void global_rule(const DeviceTables& t, float* ema, const RuleArgs& r, double* wave_sums)
{
    const int tid = threadIdx.x;
    double acc = 0.0;
    for (uint32_t i = tid; i < t.n_tensors; i += kBlock) acc += t.sumsq[i];
    double s = wave_sum_f64(acc);
    if ((tid & 63) == 0) wave_sums[tid >> 6] = s;
    __syncthreads();
    if (tid != 0) return;
    double total = wave_sums[0];
#pragma unroll
    for (int w = 1; w < kWavesPerBlock; ++w) total += wave_sums[w];
    const double gnorm = sqrt(total);
    double h;
    bool active, clipped;
    if (r.mode == ADAGC_MODE_GLOBAL_ADAGC && !r.warmup) {
        const double gamma_prev = (double)ema[0];
        const double threshold = __dmul_rn(r.lambda_rel, gamma_prev);
        active = gnorm > threshold;
        h = active ? __ddiv_rn(threshold, gnorm) : 1.0;
        const double clipped_norm = active ? threshold : gnorm;
        ema[0] = (float)__dadd_rn(__dmul_rn(r.ema_beta, gamma_prev),
                                  __dmul_rn(__dsub_rn(1.0, r.ema_beta), clipped_norm));
        clipped = active;
    } else if (r.mode == ADAGC_MODE_ZCLIP && !r.warmup) {
        // Table 2's ZClip row on the model's norm: z-score against the moving mean and deviation,
        // threshold mu + (z_thres^2 / z) sigma, statistics fed the clipped norm.
        const double mu_prev = (double)ema[0], var_prev = (double)ema[1];
        const double sigma = sqrt(var_prev);
        const double z = __ddiv_rn(__dsub_rn(gnorm, mu_prev), sigma);
        active = z > r.z_thres;                                   // false for NaN (sigma = 0 and norm = mu)
        const double xi = __ddiv_rn(__dmul_rn(r.z_thres, r.z_thres), z);
        const double tau = __dadd_rn(mu_prev, __dmul_rn(xi, sigma));
        h = active ? __ddiv_rn(tau, gnorm) : 1.0;
        const double clipped_norm = active ? tau : gnorm;
        const double mu = __dadd_rn(__dmul_rn(r.ema_beta, mu_prev), __dmul_rn(__dsub_rn(1.0, r.ema_beta), clipped_norm));
        const double dev = __dsub_rn(clipped_norm, mu);
        ema[0] = (float)mu;
        ema[1] = (float)__dadd_rn(__dmul_rn(r.ema_beta, var_prev),
                                  __dmul_rn(__dmul_rn(__dsub_rn(1.0, r.ema_beta), dev), dev));
        clipped = active;
    } else {
        active = gnorm > r.lambda_abs;
        h = active ? __ddiv_rn(r.lambda_abs, gnorm) : 1.0;
        clipped = h < 1.0;
        if (r.mode == ADAGC_MODE_GLOBAL_ADAGC) {
            const double clipped_norm = __dmul_rn(h, gnorm);
            const double gamma_prev = (double)ema[0];
            double gamma_new = clipped_norm;
            if (!r.first_step) gamma_new = clipped_norm < gamma_prev ? clipped_norm : gamma_prev;
            ema[0] = (float)gamma_new;
        }
        if (r.mode == ADAGC_MODE_ZCLIP) {
            // steps that only gather the statistics: set on the first step, moving averages afterwards
            const double clipped_norm = __dmul_rn(h, gnorm);
            double mu = clipped_norm, var = 0.0;
            if (!r.first_step) {
                const double mu_prev = (double)ema[0], var_prev = (double)ema[1];
                mu = __dadd_rn(__dmul_rn(r.ema_beta, mu_prev), __dmul_rn(__dsub_rn(1.0, r.ema_beta), clipped_norm));
                const double dev = __dsub_rn(clipped_norm, mu);
                var = __dadd_rn(__dmul_rn(r.ema_beta, var_prev), __dmul_rn(__dmul_rn(__dsub_rn(1.0, r.ema_beta), dev), dev));
            }
            ema[0] = (float)mu;
            ema[1] = (float)var;
        }
    }
    t.global[0] = total;
    t.global[1] = h;
    t.global[2] = clipped ? 1.0 : 0.0;
}

__global__ __launch_bounds__(kBlock) void global_rule_kernel(DeviceTables t, float* ema, RuleArgs r)
{
    __shared__ double wave_sums[kWavesPerBlock];
    global_rule(t, ema, r, wave_sums);
}

// Global stage 3 for tensor i: it takes the model's coefficient.  In the AdaGC mode (warm-up branch of
// Alg. 1) gamma_i = min{gamma_i, h*n_i}, or h*n_i on the first step; the global modes keep no per-tensor
// state.
__device__ __forceinline__ void take_global_coefficient(const DeviceTables& t, float* ema, const RuleArgs& r, uint32_t i)
{
    const double h = t.global[1];
    const double norm = sqrt(t.sumsq[i]);
    t.norm[i] = (float)norm;
    t.coef[i] = (float)h;
    t.coef64[i] = h;
    t.flag[i] = (t.global[2] != 0.0) ? 1 : 0;
    if (r.mode == ADAGC_MODE_ADAGC) {
        const double clipped_norm = __dmul_rn(h, norm);
        const double gamma_prev = (double)ema[i];
        double gamma_new = clipped_norm;
        if (!r.first_step) gamma_new = clipped_norm < gamma_prev ? clipped_norm : gamma_prev;
        ema[i] = (float)gamma_new;
    }
}

__global__ __launch_bounds__(kBlock) void finalize_global_kernel(DeviceTables t, float* ema, RuleArgs r)
{
    const uint32_t i = blockIdx.x * kBlock + threadIdx.x;
    if (i < t.n_tensors) take_global_coefficient(t, ema, r, i);
}

// ---------------------------------------------------------------------------------------------
// The same rules with the step's scalars taken from device memory (adagc_step_graph): the step number
// and the hyper-parameters are read when the kernels run, so a recorded launch sequence stays valid
// for other steps.  Which branch of Alg. 1 applies is therefore decided on the device as well.

// One lane: validate the caller's step parameters and derive the scalars of both stages from them.
__global__ void prepare_step_kernel(DeviceTables t, const adagc_step_params* params, int optimizer)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    const adagc_hyper hp = params->hp;
    const int64_t step = params->step;
    auto unit = [](float b) { return b >= 0.0f && b < 1.0f; };   // false for NaN
    auto finite = [](float x) { return fabsf(x) <= 3.402823466e+38f; };
    bool ok = step >= 1 && finite(hp.lr) && finite(hp.weight_decay) && unit(hp.beta1) && unit(hp.beta2) &&
              unit(hp.ema_beta) && hp.lambda_rel >= 0.0f && hp.lambda_abs > 0.0f && hp.t_start >= 0 &&
              hp.clip_mode >= ADAGC_MODE_ADAGC && hp.clip_mode <= ADAGC_MODE_ZCLIP &&
              (hp.clip_mode != ADAGC_MODE_ZCLIP || hp.z_thres > 0.0f);
    if (optimizer == ADAGC_OPT_ADAMW) ok = ok && hp.eps >= 0.0f && finite(hp.eps);
    StepScalars sc;
    const double lr = hp.lr, b1 = hp.beta1, b2 = hp.beta2, wd = hp.weight_decay, tt = (double)step;
    sc.r.lambda_rel = (double)hp.lambda_rel;
    sc.r.ema_beta = (double)hp.ema_beta;
    sc.r.lambda_abs = (double)hp.lambda_abs;
    sc.r.z_thres = (double)hp.z_thres;
    sc.r.pad = 0;
    sc.r.first_step = (step == 1) ? 1 : 0;
    sc.r.warmup = ((step - 1) < (int64_t)hp.t_start) ? 1 : 0;
    sc.r.mode = hp.clip_mode;
    sc.u.beta1 = b1;
    sc.u.one_minus_beta1 = 1.0 - b1;
    sc.u.beta2 = b2;
    sc.u.one_minus_beta2 = 1.0 - b2;
    sc.u.inv_bias2 = 1.0 / (1.0 - pow(b2, tt));
    sc.u.step_size = lr / (1.0 - pow(b1, tt));
    sc.u.lr_wd = lr * wd;
    sc.u.eps = (double)hp.eps;
    sc.u.lr = lr;
    sc.u.weight_decay = wd;
    sc.u.inv_bias1 = 1.0 / (1.0 - pow(b1, tt));
    sc.u.update_clip = 0;                       // the update-clipping modes are rejected above
    sc.u.pad = 0;
    sc.r.lr = lr;
    sc.status = ok ? 0 : 1;
    sc.pad = 0;
    *t.scalars = sc;
}

__global__ __launch_bounds__(kBlock) void global_rule_device_kernel(DeviceTables t, float* ema)
{
    __shared__ double wave_sums[kWavesPerBlock];
    const RuleArgs r = t.scalars->r;
    if (t.scalars->status != 0 || !(r.warmup || r.mode != ADAGC_MODE_ADAGC)) return;   // uniform
    global_rule(t, ema, r, wave_sums);
}

__global__ __launch_bounds__(kBlock) void finalize_device_kernel(DeviceTables t, float* ema)
{
    const uint32_t i = blockIdx.x * kBlock + threadIdx.x;
    if (i >= t.n_tensors || t.scalars->status != 0) return;
    const RuleArgs r = t.scalars->r;
    if (r.warmup || r.mode != ADAGC_MODE_ADAGC) take_global_coefficient(t, ema, r, i);
    else adagc_rule(t, ema, r, i, t.sumsq[i]);
}

// ---------------------------------------------------------------------------------------------
// K3: clipped gradient into the optimizer, element by element.

struct ElemState {
    float p, m, v;
};

// The elementwise update is evaluated in double and each stored value is rounded to fp32 once.
// The kernel waits on HBM (hardware counters on Llama-3-8B shapes: memory interface busy 99 %,
// vector ALU active 15 % of the time), so double arithmetic costs no time (measured: 37.9 ms with
// either precision) and makes the result the correctly rounded value of Alg. 1's statements, not
// an accumulation of fp32 roundings.

// AdamW statements of Alg. 1 on the clipped gradient h*g; the bias corrections are folded into two
// host-computed scalars (step_size = lr / (1 - beta1^t), inv_bias2 = 1 / (1 - beta2^t)).
// uc scales the direction m_hat/(sqrt(v_hat)+eps) (update clipping); it is exactly 1.0 in every other mode.
__device__ __forceinline__ void adamw_elem(const UpdateArgs& a, double h, double uc, float g, ElemState& s)
{
    const double gh = h * (double)g;
    const double m = a.beta1 * (double)s.m + a.one_minus_beta1 * gh;
    const double v = a.beta2 * (double)s.v + a.one_minus_beta2 * gh * gh;
    const double denom = sqrt(v * a.inv_bias2) + a.eps;
    const double th = (double)s.p;
    s.p = (float)(th - a.lr_wd * th - uc * (a.step_size * m / denom));
    s.m = (float)m;
    s.v = (float)v;
}

// Lion (rule of Chen et al.; the paper only cites it).  The sign is a discrete decision: the
// interpolation c is evaluated with separately rounded operations, the sequence a plain C
// implementation without contraction produces.
__device__ __forceinline__ double lion_sign(const UpdateArgs& a, double gh, float m)
{
    const double c = __dadd_rn(__dmul_rn(a.beta1, (double)m), __dmul_rn(a.one_minus_beta1, gh));
    return (c > 0.0) ? 1.0 : ((c < 0.0) ? -1.0 : 0.0);
}

__device__ __forceinline__ void lion_elem(const UpdateArgs& a, double h, double uc, float g, ElemState& s)
{
    const double gh = __dmul_rn(h, (double)g);
    const double sgn = lion_sign(a, gh, s.m);
    const double th = (double)s.p;
    s.p = (float)(th - a.lr * (uc * sgn + a.weight_decay * th));
    s.m = (float)(a.beta2 * (double)s.m + a.one_minus_beta2 * gh);
}

template <int OPT>
__device__ __forceinline__ void apply_elem(const UpdateArgs& a, double h, double uc, float g, ElemState& s)
{
    if constexpr (OPT == ADAGC_OPT_ADAMW) adamw_elem(a, h, uc, g, s);
    else lion_elem(a, h, uc, g, s);
}

template <int OPT>
__device__ __forceinline__ void apply_vec(const UpdateArgs& a, double h, double uc, f32x4 g, f32x4& p, f32x4& m, f32x4& v)
{
    ElemState s;
    s = {p.x, m.x, v.x}; apply_elem<OPT>(a, h, uc, g.x, s); p.x = s.p; m.x = s.m; v.x = s.v;
    s = {p.y, m.y, v.y}; apply_elem<OPT>(a, h, uc, g.y, s); p.y = s.p; m.y = s.m; v.y = s.v;
    s = {p.z, m.z, v.z}; apply_elem<OPT>(a, h, uc, g.z, s); p.z = s.p; m.z = s.m; v.z = s.v;
    s = {p.w, m.w, v.w}; apply_elem<OPT>(a, h, uc, g.w, s); p.w = s.p; m.w = s.m; v.w = s.v;
}

// Telemetry: per-lane fp64 sums of m^2, v^2 and (theta_new - theta_old)^2 over the lane's elements,
// in element order; they become one slot per chunk and per quantity, reduced per tensor afterwards.
template <bool HAS_V>
__device__ __forceinline__ void tele_elem(double (&acc)[3], float p_old, float p_new, float m, float v)
{
    const double dm = (double)m;
    acc[0] = fma(dm, dm, acc[0]);
    if constexpr (HAS_V) {
        const double dv = (double)v;
        acc[1] = fma(dv, dv, acc[1]);
    }
    const double du = (double)p_new - (double)p_old;
    acc[2] = fma(du, du, acc[2]);
}

template <bool HAS_V>
__device__ __forceinline__ void tele_vec(double (&acc)[3], f32x4 p_old, f32x4 p_new, f32x4 m, f32x4 v)
{
    tele_elem<HAS_V>(acc, p_old.x, p_new.x, m.x, v.x);
    tele_elem<HAS_V>(acc, p_old.y, p_new.y, m.y, v.y);
    tele_elem<HAS_V>(acc, p_old.z, p_new.z, m.z, v.z);
    tele_elem<HAS_V>(acc, p_old.w, p_new.w, m.w, v.w);
}

// A tile is U*kBlock consecutive 128-bit vectors (U*1024 elements) of one chunk, handled with U vectors per
// lane and per array in flight; a chunk has kVecPerLane/U tiles.  A workgroup's work item is 1/items_per_chunk
// of a chunk: a run of consecutive tiles (the whole chunk when items_per_chunk is 1).  Small items shorten
// the tail of the launch and give short lists more workgroups; whole chunks cost the fewest dispatches.
// Workgroups are dealt to the XCDs in turn (workgroup b to XCD b mod 8), so items are numbered such that
// eight consecutive workgroups work on eight consecutive positions of the visiting order (one from each of
// its parts) and the items of one chunk all go to the same XCD:
//   item T  ->  position 8*(T / (8*I)) + T % 8,  item (T / 8) % I of that chunk      (I = items_per_chunk).
template <int OPT, bool BF16G, bool COPY, int U, bool NT, bool TELE>
__global__ __launch_bounds__(kBlock) void update_kernel(DeviceTables t, UpdateArgs a, uint32_t items_per_chunk,
                                                        const StepScalars* device_scalars)
{
    static_assert(kVecPerLane % U == 0, "a chunk is a whole number of tiles");
    if (device_scalars) {                      // adagc_step_graph: this step's scalars live in device memory
        if (device_scalars->status != 0) return;
        a = device_scalars->u;
    }
    constexpr bool NTL = NT, NTS = NT;    // non-temporal loads and stores
    constexpr bool kHasV = (OPT == ADAGC_OPT_ADAMW);
    constexpr int kTiles = kVecPerLane / U;
    constexpr int kTileVecs = U * kBlock;
    constexpr int kTileElems = kTileVecs * 4;
    const int tid = threadIdx.x;
    __shared__ double tele_sums[3][kWavesPerBlock];

    const uint32_t group = 8u * items_per_chunk;
    const int tiles_per_item = kTiles / (int)items_per_chunk;
    const uint64_t n_items = (((uint64_t)t.n_chunks + 7u) & ~(uint64_t)7u) * items_per_chunk;
    for (uint64_t item = blockIdx.x; item < n_items; item += gridDim.x) {
        const uint32_t r = (uint32_t)(item % group);
        const uint32_t k = (uint32_t)(item / group) * 8u + (r & 7u);
        const int isub = (int)(r >> 3);
        if (k >= t.n_chunks) continue;
        const uint32_t c = t.schedule ? t.schedule[k] : k;     // no visiting order given: list order
        const ChunkView cv = chunk_view(t, c);
        const TensorArgs& ta = t.targs[cv.tensor];
        const double h = t.coef64[cv.tensor];     // the tensor's coefficient as computed, in double
        const double uc = a.update_clip ? t.ucoef64[cv.tensor] : 1.0;   // update clipping: scales the direction
        const void* g = grad_chunk_ptr<BF16G>(ta.grad, cv.first);
        float* p = reinterpret_cast<float*>(ta.param) + cv.first;
        float* m = reinterpret_cast<float*>(ta.exp_avg) + cv.first;
        float* v = kHasV ? reinterpret_cast<float*>(ta.exp_avg_sq) + cv.first : nullptr;
        uint16_t* pc = COPY ? reinterpret_cast<uint16_t*>(ta.param_copy) + cv.first : nullptr;
        double tele[3] = {0.0, 0.0, 0.0};

#pragma unroll 1
        for (int tt = 0; tt < tiles_per_item; ++tt) {
            const int sub = isub * tiles_per_item + tt;
            const int e0 = sub * kTileElems;                                   // the tile's elements inside the chunk:
            const int e1 = cv.len < e0 + kTileElems ? cv.len : e0 + kTileElems; // [e0, e1), empty past a ragged end
            if (e0 >= e1) break;
            if (ta.vec_ok) {
                f32x4* p4 = reinterpret_cast<f32x4*>(p);
                f32x4* m4 = reinterpret_cast<f32x4*>(m);
                f32x4* v4 = reinterpret_cast<f32x4*>(v);
                u32x2* c4 = reinterpret_cast<u32x2*>(pc);
                const int v0 = sub * kTileVecs;

                if (e1 - e0 == kTileElems) {
                    f32x4 gg[U], pp[U], mm[U], vv[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int idx = v0 + u * kBlock + tid;
                        gg[u] = load_grad4<BF16G, NTL>(g, idx);
                        pp[u] = ld<NTL>(p4 + idx);
                        mm[u] = ld<NTL>(m4 + idx);
                        if constexpr (kHasV) vv[u] = ld<NTL>(v4 + idx);
                        else vv[u] = f32x4{0.f, 0.f, 0.f, 0.f};
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int idx = v0 + u * kBlock + tid;
                        const f32x4 p_old = pp[u];
                        apply_vec<OPT>(a, h, uc, gg[u], pp[u], mm[u], vv[u]);
                        if constexpr (TELE) tele_vec<kHasV>(tele, p_old, pp[u], mm[u], vv[u]);
                        st<NTS>(p4 + idx, pp[u]);
                        st<NTS>(m4 + idx, mm[u]);
                        if constexpr (kHasV) st<NTS>(v4 + idx, vv[u]);
                        if constexpr (COPY) st<NTS>(c4 + idx, pack_bf16x4(pp[u]));
                    }
                } else {
                    // the last tile of a ragged chunk: its whole vectors, then up to three single elements
                    const int nvec = cv.len >> 2;
                    for (int idx = v0 + tid; idx < nvec; idx += kBlock) {
                        f32x4 gg = load_grad4<BF16G, NTL>(g, idx);
                        f32x4 pp = ld<NTL>(p4 + idx);
                        f32x4 mm = ld<NTL>(m4 + idx);
                        f32x4 vv = f32x4{0.f, 0.f, 0.f, 0.f};
                        if constexpr (kHasV) vv = ld<NTL>(v4 + idx);
                        const f32x4 p_old = pp;
                        apply_vec<OPT>(a, h, uc, gg, pp, mm, vv);
                        if constexpr (TELE) tele_vec<kHasV>(tele, p_old, pp, mm, vv);
                        st<NTS>(p4 + idx, pp);
                        st<NTS>(m4 + idx, mm);
                        if constexpr (kHasV) st<NTS>(v4 + idx, vv);
                        if constexpr (COPY) st<NTS>(c4 + idx, pack_bf16x4(pp));
                    }
                    const int j = (nvec << 2) + tid;
                    if (j < cv.len) {
                        ElemState s = {p[j], m[j], kHasV ? v[j] : 0.f};
                        const float p_old = s.p;
                        apply_elem<OPT>(a, h, uc, load_grad1<BF16G>(g, j), s);
                        if constexpr (TELE) tele_elem<kHasV>(tele, p_old, s.p, s.m, s.v);
                        p[j] = s.p;
                        m[j] = s.m;
                        if constexpr (kHasV) v[j] = s.v;
                        if constexpr (COPY) pc[j] = (uint16_t)float_to_bf16_bits(s.p);
                    }
                }
            } else {
                for (int j = e0 + tid; j < e1; j += kBlock) {
                    ElemState s = {p[j], m[j], kHasV ? v[j] : 0.f};
                    const float p_old = s.p;
                    apply_elem<OPT>(a, h, uc, load_grad1<BF16G>(g, j), s);
                    if constexpr (TELE) tele_elem<kHasV>(tele, p_old, s.p, s.m, s.v);
                    p[j] = s.p;
                    m[j] = s.m;
                    if constexpr (kHasV) v[j] = s.v;
                    if constexpr (COPY) pc[j] = (uint16_t)float_to_bf16_bits(s.p);
                }
            }
        }

        if constexpr (TELE) {
            // every item of every chunk writes its slots, an empty item writes zeros
#pragma unroll
            for (int q = 0; q < 3; ++q) {
                const double w = wave_sum_f64(tele[q]);
                if ((tid & 63) == 0) tele_sums[q][tid >> 6] = w;
            }
            __syncthreads();
            if (tid < 3) {
                double b = tele_sums[tid][0];
#pragma unroll
                for (int w = 1; w < kWavesPerBlock; ++w) b += tele_sums[tid][w];
                t.tele_partials[((size_t)tid * t.n_chunks + c) * items_per_chunk + isub] = b;
            }
            __syncthreads();
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Update clipping (AGC and Clippy rows of Table 2).  The coefficient of a tensor's update needs the norms
// of theta and of the whole tensor's direction Delta, so the direction is evaluated twice: here for its
// norms (nothing is written but two partial results per work item), then by update_kernel, which scales it.
// Work items are those of update_kernel.  LINF selects maxima of |.| (Clippy) instead of sums of squares (AGC).

// All 64 lanes must be active.  Returns the same value in every lane.  Maxima are exact in any order.
__device__ __forceinline__ double wave_max_f64(double x)
{
    x = fmax(x, dpp_mov<0x128>(x));  // row_ror:8
    x = fmax(x, dpp_mov<0x124>(x));  // row_ror:4
    x = fmax(x, dpp_mov<0x122>(x));  // row_ror:2
    x = fmax(x, dpp_mov<0x121>(x));  // row_ror:1
    return fmax(fmax(readlane_f64(x, 0), readlane_f64(x, 16)), fmax(readlane_f64(x, 32), readlane_f64(x, 48)));
}

// The direction of one element for the unclipped gradient: AdamW m_hat/(sqrt(v_hat)+eps) from this step's
// moments, Lion the sign of the interpolation.
template <int OPT>
__device__ __forceinline__ double direction_elem(const UpdateArgs& a, float g, float m_prev, float v_prev)
{
    const double gd = (double)g;
    if constexpr (OPT == ADAGC_OPT_ADAMW) {
        const double m = a.beta1 * (double)m_prev + a.one_minus_beta1 * gd;
        const double v = a.beta2 * (double)v_prev + a.one_minus_beta2 * gd * gd;
        return (m * a.inv_bias1) / (sqrt(v * a.inv_bias2) + a.eps);
    } else {
        return lion_sign(a, gd, m_prev);
    }
}

template <bool LINF>
__device__ __forceinline__ void stat_acc(double (&acc)[2], float theta, double delta)
{
    const double th = (double)theta;
    if constexpr (LINF) {
        acc[0] = fmax(acc[0], fabs(th));       // a NaN never becomes the maximum
        acc[1] = fmax(acc[1], fabs(delta));
    } else {
        acc[0] = fma(th, th, acc[0]);
        acc[1] = fma(delta, delta, acc[1]);
    }
}

template <int OPT, bool BF16G, bool LINF, bool NT>
__global__ __launch_bounds__(kBlock) void direction_stats_kernel(DeviceTables t, UpdateArgs a, uint32_t items_per_chunk)
{
    constexpr int U = 4;
    constexpr bool kHasV = (OPT == ADAGC_OPT_ADAMW);
    constexpr int kTiles = kVecPerLane / U;
    constexpr int kTileVecs = U * kBlock;
    constexpr int kTileElems = kTileVecs * 4;
    const int tid = threadIdx.x;
    __shared__ double wave_part[2][kWavesPerBlock];

    const uint32_t group = 8u * items_per_chunk;
    const int tiles_per_item = kTiles / (int)items_per_chunk;
    const uint64_t n_items = (((uint64_t)t.n_chunks + 7u) & ~(uint64_t)7u) * items_per_chunk;
    for (uint64_t item = blockIdx.x; item < n_items; item += gridDim.x) {
        const uint32_t r = (uint32_t)(item % group);
        const uint32_t k = (uint32_t)(item / group) * 8u + (r & 7u);
        const int isub = (int)(r >> 3);
        if (k >= t.n_chunks) continue;
        const uint32_t c = t.schedule ? t.schedule[k] : k;
        const ChunkView cv = chunk_view(t, c);
        const TensorArgs& ta = t.targs[cv.tensor];
        const void* g = grad_chunk_ptr<BF16G>(ta.grad, cv.first);
        const float* p = reinterpret_cast<const float*>(ta.param) + cv.first;
        const float* m = reinterpret_cast<const float*>(ta.exp_avg) + cv.first;
        const float* v = kHasV ? reinterpret_cast<const float*>(ta.exp_avg_sq) + cv.first : nullptr;
        double acc[2] = {0.0, 0.0};

#pragma unroll 1
        for (int tt = 0; tt < tiles_per_item; ++tt) {
            const int sub = isub * tiles_per_item + tt;
            const int e0 = sub * kTileElems;
            const int e1 = cv.len < e0 + kTileElems ? cv.len : e0 + kTileElems;
            if (e0 >= e1) break;
            if (ta.vec_ok) {
                const f32x4* p4 = reinterpret_cast<const f32x4*>(p);
                const f32x4* m4 = reinterpret_cast<const f32x4*>(m);
                const f32x4* v4 = reinterpret_cast<const f32x4*>(v);
                const int v0 = sub * kTileVecs;
                const int vend = (e1 - e0 == kTileElems) ? v0 + kTileVecs : (cv.len >> 2);
                if (e1 - e0 == kTileElems) {
                    f32x4 gg[U], pp[U], mm[U], vv[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int idx = v0 + u * kBlock + tid;
                        gg[u] = load_grad4<BF16G, NT>(g, idx);
                        pp[u] = ld<NT>(p4 + idx);
                        mm[u] = ld<NT>(m4 + idx);
                        if constexpr (kHasV) vv[u] = ld<NT>(v4 + idx);
                        else vv[u] = f32x4{0.f, 0.f, 0.f, 0.f};
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        stat_acc<LINF>(acc, pp[u].x, direction_elem<OPT>(a, gg[u].x, mm[u].x, vv[u].x));
                        stat_acc<LINF>(acc, pp[u].y, direction_elem<OPT>(a, gg[u].y, mm[u].y, vv[u].y));
                        stat_acc<LINF>(acc, pp[u].z, direction_elem<OPT>(a, gg[u].z, mm[u].z, vv[u].z));
                        stat_acc<LINF>(acc, pp[u].w, direction_elem<OPT>(a, gg[u].w, mm[u].w, vv[u].w));
                    }
                } else {
                    for (int idx = v0 + tid; idx < vend; idx += kBlock) {
                        const f32x4 gg = load_grad4<BF16G, NT>(g, idx);
                        const f32x4 pp = ld<NT>(p4 + idx);
                        const f32x4 mm = ld<NT>(m4 + idx);
                        f32x4 vv = f32x4{0.f, 0.f, 0.f, 0.f};
                        if constexpr (kHasV) vv = ld<NT>(v4 + idx);
                        stat_acc<LINF>(acc, pp.x, direction_elem<OPT>(a, gg.x, mm.x, vv.x));
                        stat_acc<LINF>(acc, pp.y, direction_elem<OPT>(a, gg.y, mm.y, vv.y));
                        stat_acc<LINF>(acc, pp.z, direction_elem<OPT>(a, gg.z, mm.z, vv.z));
                        stat_acc<LINF>(acc, pp.w, direction_elem<OPT>(a, gg.w, mm.w, vv.w));
                    }
                    const int j = ((cv.len >> 2) << 2) + tid;      // up to three single elements at the ragged end
                    if (j < cv.len)
                        stat_acc<LINF>(acc, p[j], direction_elem<OPT>(a, load_grad1<BF16G>(g, j), m[j], kHasV ? v[j] : 0.f));
                }
            } else {
                for (int j = e0 + tid; j < e1; j += kBlock)
                    stat_acc<LINF>(acc, p[j], direction_elem<OPT>(a, load_grad1<BF16G>(g, j), m[j], kHasV ? v[j] : 0.f));
            }
        }

        // every item of every chunk writes its two slots, an empty item writes zeros
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const double w = LINF ? wave_max_f64(acc[q]) : wave_sum_f64(acc[q]);
            if ((tid & 63) == 0) wave_part[q][tid >> 6] = w;
        }
        __syncthreads();
        if (tid < 2) {
            double b = wave_part[tid][0];
#pragma unroll
            for (int w = 1; w < kWavesPerBlock; ++w) b = LINF ? fmax(b, wave_part[tid][w]) : b + wave_part[tid][w];
            t.ustat_partials[((size_t)tid * t.n_chunks + c) * items_per_chunk + isub] = b;
        }
        __syncthreads();
    }
}

// The maximum of a tensor's slots (any order gives the same value).
__device__ __forceinline__ double tensor_slot_max(const DeviceTables& t, const double* slots, uint32_t i, double* wave_part,
                                                  uint32_t slots_per_chunk)
{
    const uint32_t count = t.targs[i].chunk_count * slots_per_chunk;
    const double* p = slots + (size_t)t.targs[i].chunk_begin * slots_per_chunk;
    double a0 = 0.0;
    for (uint32_t k = threadIdx.x; k < count; k += kBlock) a0 = fmax(a0, p[k]);
    const double s = wave_max_f64(a0);
    if ((threadIdx.x & 63) == 0) wave_part[threadIdx.x >> 6] = s;
    __syncthreads();
    double total = wave_part[0];
#pragma unroll
    for (int w = 1; w < kWavesPerBlock; ++w) total = fmax(total, wave_part[w]);
    return total;
}

// One workgroup per tensor: the two norms from the item slots, then Table 2's AGC or Clippy coefficient.
// The gradient's own coefficient is 1 in these modes.  Reported to the caller: the direction's norm,
// the update coefficient, and whether it is below 1.
__global__ __launch_bounds__(kBlock) void finalize_update_clip_kernel(DeviceTables t, RuleArgs r, uint32_t items_per_chunk)
{
    __shared__ double wave_part[kWavesPerBlock];
    const uint32_t i = blockIdx.x;
    const bool linf = r.mode == ADAGC_MODE_CLIPPY;
    double stat[2];
    for (int q = 0; q < 2; ++q) {
        const double* slots = t.ustat_partials + (size_t)q * t.n_chunks * items_per_chunk;
        stat[q] = linf ? tensor_slot_max(t, slots, i, wave_part, items_per_chunk)
                       : tensor_slot_sum(t, slots, i, wave_part, items_per_chunk);
        __syncthreads();
    }
    if (threadIdx.x != 0) return;
    double ratio, delta_norm;
    if (linf) {
        delta_norm = stat[1];
        ratio = __ddiv_rn(__dadd_rn(__dmul_rn(r.lambda_rel, stat[0]), r.lambda_abs), __dmul_rn(r.lr, delta_norm));
    } else {
        delta_norm = sqrt(stat[1]);
        ratio = __ddiv_rn(__dmul_rn(r.lambda_rel, sqrt(stat[0])), delta_norm);
    }
    const bool active = ratio < 1.0;              // false for NaN (0/0): the update is left alone
    const double c = active ? ratio : 1.0;
    t.norm[i] = (float)delta_norm;
    t.coef[i] = (float)c;
    t.ucoef64[i] = c;
    t.coef64[i] = 1.0;
    t.flag[i] = active ? 1 : 0;
}

// Telemetry finalize: per tensor, the three norms from the item slots (same fixed order as K2).
__global__ __launch_bounds__(kBlock) void finalize_telemetry_kernel(DeviceTables t, uint32_t items_per_chunk)
{
    __shared__ double wave_sums[kWavesPerBlock];
    const uint32_t i = blockIdx.x;
    for (int q = 0; q < 3; ++q) {
        const double s = tensor_slot_sum(t, t.tele_partials + (size_t)q * t.n_chunks * items_per_chunk, i, wave_sums,
                                         items_per_chunk);
        if (threadIdx.x == 0) t.tele_norm[(size_t)q * t.n_tensors + i] = (float)sqrt(s);
        __syncthreads();
    }
}

using UpdateFn = void (*)(DeviceTables, UpdateArgs, uint32_t, const StepScalars*);
using SumsqFn = void (*)(DeviceTables);

template <int OPT, bool BF16G, bool COPY, int U>
UpdateFn select_update_flags(int nt, int tele)
{
    if (nt) return tele ? update_kernel<OPT, BF16G, COPY, U, true, true> : update_kernel<OPT, BF16G, COPY, U, true, false>;
    return tele ? update_kernel<OPT, BF16G, COPY, U, false, true> : update_kernel<OPT, BF16G, COPY, U, false, false>;
}

template <int OPT, bool BF16G, bool COPY>
UpdateFn select_update_variant(int unroll, int nt, int tele)
{
    if (unroll == 4) return select_update_flags<OPT, BF16G, COPY, 4>(nt, tele);
    if (unroll == 2) return select_update_flags<OPT, BF16G, COPY, 2>(nt, tele);
    return select_update_flags<OPT, BF16G, COPY, 1>(nt, tele);
}

UpdateFn select_update(int optimizer, int grad_bf16, int with_copy, int unroll, int nt, int tele)
{
    const int key = (optimizer == ADAGC_OPT_LION ? 4 : 0) | (grad_bf16 ? 2 : 0) | (with_copy ? 1 : 0);
    switch (key) {
    case 0: return select_update_variant<ADAGC_OPT_ADAMW, false, false>(unroll, nt, tele);
    case 1: return select_update_variant<ADAGC_OPT_ADAMW, false, true>(unroll, nt, tele);
    case 2: return select_update_variant<ADAGC_OPT_ADAMW, true, false>(unroll, nt, tele);
    case 3: return select_update_variant<ADAGC_OPT_ADAMW, true, true>(unroll, nt, tele);
    case 4: return select_update_variant<ADAGC_OPT_LION, false, false>(unroll, nt, tele);
    case 5: return select_update_variant<ADAGC_OPT_LION, false, true>(unroll, nt, tele);
    case 6: return select_update_variant<ADAGC_OPT_LION, true, false>(unroll, nt, tele);
    default: return select_update_variant<ADAGC_OPT_LION, true, true>(unroll, nt, tele);
    }
}

SumsqFn select_sumsq(int grad_bf16, int nt)
{
    if (nt) return grad_bf16 ? sumsq_partials_kernel<true, true> : sumsq_partials_kernel<false, true>;
    return grad_bf16 ? sumsq_partials_kernel<true, false> : sumsq_partials_kernel<false, false>;
}

}  // namespace

hipError_t launch_sumsq_partials(const DeviceTables& t, int grad_bf16, int nt, int grid, hipStream_t stream)
{
    select_sumsq(grad_bf16, nt)<<<dim3(grid), dim3(kBlock), 0, stream>>>(t);
    return hipGetLastError();
}

hipError_t launch_finalize_adagc(const DeviceTables& t, float* ema, const RuleArgs& r, hipStream_t stream)
{
    finalize_adagc_kernel<<<dim3(t.n_tensors), dim3(kBlock), 0, stream>>>(t, ema, r);
    return hipGetLastError();
}

hipError_t launch_tensor_sumsq(const DeviceTables& t, hipStream_t stream)
{
    tensor_sumsq_kernel<<<dim3(t.n_tensors), dim3(kBlock), 0, stream>>>(t);
    return hipGetLastError();
}

hipError_t launch_finalize_global(const DeviceTables& t, float* ema, const RuleArgs& r, hipStream_t stream)
{
    tensor_sumsq_kernel<<<dim3(t.n_tensors), dim3(kBlock), 0, stream>>>(t);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    global_rule_kernel<<<dim3(1), dim3(kBlock), 0, stream>>>(t, ema, r);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    const uint32_t blocks = (t.n_tensors + kBlock - 1) / kBlock;
    finalize_global_kernel<<<dim3(blocks), dim3(kBlock), 0, stream>>>(t, ema, r);
    return hipGetLastError();
}

using StatsFn = void (*)(DeviceTables, UpdateArgs, uint32_t);

template <int OPT, bool BF16G>
static StatsFn select_stats_flags(bool linf, int nt)
{
    if (linf) return nt ? direction_stats_kernel<OPT, BF16G, true, true> : direction_stats_kernel<OPT, BF16G, true, false>;
    return nt ? direction_stats_kernel<OPT, BF16G, false, true> : direction_stats_kernel<OPT, BF16G, false, false>;
}

hipError_t launch_update_clip_rule(const DeviceTables& t, const UpdateArgs& u, const RuleArgs& r, int optimizer,
                                   int grad_bf16, int items_per_chunk, int nt, int grid, hipStream_t stream)
{
    const bool linf = r.mode == ADAGC_MODE_CLIPPY;
    StatsFn fn;
    if (optimizer == ADAGC_OPT_LION) fn = grad_bf16 ? select_stats_flags<ADAGC_OPT_LION, true>(linf, nt) : select_stats_flags<ADAGC_OPT_LION, false>(linf, nt);
    else fn = grad_bf16 ? select_stats_flags<ADAGC_OPT_ADAMW, true>(linf, nt) : select_stats_flags<ADAGC_OPT_ADAMW, false>(linf, nt);
    fn<<<dim3(grid), dim3(kBlock), 0, stream>>>(t, u, (uint32_t)items_per_chunk);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    finalize_update_clip_kernel<<<dim3(t.n_tensors), dim3(kBlock), 0, stream>>>(t, r, (uint32_t)items_per_chunk);
    return hipGetLastError();
}

hipError_t launch_rules_from_device(const DeviceTables& t, float* ema, const adagc_step_params* params,
                                    int optimizer, hipStream_t stream)
{
    prepare_step_kernel<<<dim3(1), dim3(64), 0, stream>>>(t, params, optimizer);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    tensor_sumsq_kernel<<<dim3(t.n_tensors), dim3(kBlock), 0, stream>>>(t);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    global_rule_device_kernel<<<dim3(1), dim3(kBlock), 0, stream>>>(t, ema);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    const uint32_t blocks = (t.n_tensors + kBlock - 1) / kBlock;
    finalize_device_kernel<<<dim3(blocks), dim3(kBlock), 0, stream>>>(t, ema);
    return hipGetLastError();
}

hipError_t launch_update(const DeviceTables& t, const UpdateArgs& a, int optimizer, int grad_bf16,
                         int with_copy, int unroll, int items_per_chunk, int nt, int tele, int grid,
                         hipStream_t stream, bool device_scalars)
{
    select_update(optimizer, grad_bf16, with_copy, unroll, nt, tele)<<<dim3(grid), dim3(kBlock), 0, stream>>>(
        t, a, (uint32_t)items_per_chunk, device_scalars ? t.scalars : nullptr);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || !tele) return e;
    finalize_telemetry_kernel<<<dim3(t.n_tensors), dim3(kBlock), 0, stream>>>(t, (uint32_t)items_per_chunk);
    return hipGetLastError();
}

}  // namespace adagc
