// Shared between the host API and the HIP kernels of libadagc.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cmath>

#include "adagc.h"

namespace adagc {

// Elements per chunk.  Every tensor is cut at multiples of this counted from its
// own first element, so a tensor's reduction tree depends only on its own size.
// 16384 fp32 = 64 KiB per stream per chunk: one workgroup of 256 lanes covers a
// full chunk with 16 independent 128-bit loads per lane per stream.
#ifndef ADAGC_CHUNK_ELEMS
#define ADAGC_CHUNK_ELEMS 16384
#endif
constexpr int kChunkElems = ADAGC_CHUNK_ELEMS;
constexpr int kBlock = 256;              // lanes per workgroup (4 wave64)
constexpr int kWavesPerBlock = kBlock / 64;
constexpr int kVecPerLane = kChunkElems / 4 / kBlock;   // 128-bit vectors per lane in a full chunk

// Device-resident per-tensor record: everything a workgroup needs about the
// tensor that owns its chunk, fetched with one scalar load burst.
struct TensorArgs {
    void*       param;       // fp32, in/out
    const void* grad;        // fp32 or bf16, in
    void*       exp_avg;     // fp32, in/out
    void*       exp_avg_sq;  // fp32, in/out (unused by Lion)
    void*       param_copy;  // bf16, out (optional)
    int64_t     numel;
    uint32_t    chunk_begin; // index of this tensor's first chunk / partial slot
    uint32_t    chunk_count;
    uint32_t    vec_ok;      // 1: all of this tensor's pointers allow 128-bit (64-bit for bf16) access
    uint32_t    pad;
};
static_assert(sizeof(TensorArgs) == 64, "TensorArgs is one 64-byte record");

struct ChunkRef {
    uint32_t tensor;  // owning tensor
    uint32_t index;   // position inside the tensor: first element = index * kChunkElems
};

// Scalars of the per-tensor rule (Eq. 3 / warm-up branch of Alg. 1), all widened from the
// caller's fp32 hyper-parameters so that decisions are taken in double.
struct RuleArgs {
    double lambda_rel;
    double ema_beta;
    double lambda_abs;
    double z_thres;      // ZClip
    double lr;           // Clippy's ratio divides by the learning rate
    int    first_step;   // step == 1: gamma is set, not min-ed
    int    warmup;       // step <= t_start
    int    mode;         // ADAGC_MODE_*
    int    pad;
};

// Scalars of the elementwise update, precomputed on the host in double from the caller's fp32
// hyper-parameters.
struct UpdateArgs {
    double beta1, one_minus_beta1;
    double beta2, one_minus_beta2;
    double inv_bias2;      // 1 / (1 - beta2^t)
    double step_size;      // lr / (1 - beta1^t)
    double lr_wd;          // lr * weight_decay
    double eps;
    double lr;             // Lion
    double weight_decay;   // Lion
    double inv_bias1;      // 1 / (1 - beta1^t) (the direction's norms of the update-clipping modes)
    int    update_clip;    // 1: the direction is scaled by the tensor's update coefficient
    int    pad;
};

// Scalars of one step kept in device memory: written by a small kernel from the caller's
// device-resident adagc_step_params, read by the rule kernels and the update kernel.  This is what
// lets a step be recorded into a HIP graph once and replayed for other step numbers.
struct StepScalars {
    RuleArgs   r;
    UpdateArgs u;
    int32_t    status;   // 0 = valid; otherwise the step leaves all state untouched
    int32_t    pad;
};

struct DeviceTables {
    const ChunkRef*   chunks;     // canonical order: tensor by tensor; slot c of `partials` belongs to chunk c
    const uint32_t*   schedule;   // order in which the streaming kernels visit the chunks (null: list order)
    const TensorArgs* targs;
    double*           partials;   // one per chunk
    double*           sumsq;      // one per tensor
    double*           global;     // [0] = model's sum of squares, [1] = its coefficient, [2] = 1 if clipped
    float*            norm;       // per tensor, pre-clip
    float*            coef;       // per tensor, fp32 (reported to the caller)
    double*           coef64;     // per tensor, as computed (what the update kernel multiplies by)
    uint8_t*          flag;       // per tensor, 1 = clip active
    double*           tele_partials;  // telemetry: [3][n_chunks][items per chunk] sums of m^2, v^2, (dtheta)^2 (or null)
    float*            tele_norm;      // telemetry: [3][n_tensors] norms
    StepScalars*      scalars;        // used by adagc_step_graph only
    double*           ustat_partials; // update clipping: [2][n_chunks][items per chunk] partial norms of theta and of
                                      // the direction (sums of squares for AGC, maxima for Clippy), or null
    double*           ucoef64;        // update clipping: per-tensor coefficient of the direction, or null
    uint32_t          n_chunks;
    uint32_t          n_tensors;
};

// What every step entry point accepts as hyper-parameters.
inline bool hyper_ok(const adagc_hyper& h, int optimizer)
{
    auto unit = [](float b) { return b >= 0.0f && b < 1.0f; };   // false for NaN
    if (!std::isfinite(h.lr) || !std::isfinite(h.weight_decay)) return false;
    if (!unit(h.beta1) || !unit(h.beta2) || !unit(h.ema_beta)) return false;
    if (optimizer == ADAGC_OPT_ADAMW && !(h.eps >= 0.0f && std::isfinite(h.eps))) return false;
    if (!(h.lambda_rel >= 0.0f)) return false;    // +inf allowed, NaN not
    if (!(h.lambda_abs > 0.0f)) return false;     // +inf allowed, NaN not
    if (h.t_start < 0) return false;
    if (h.clip_mode < ADAGC_MODE_ADAGC || h.clip_mode > ADAGC_MODE_CLIPPY) return false;
    if (h.clip_mode == ADAGC_MODE_ZCLIP && !(h.z_thres > 0.0f)) return false;   // +inf allowed, NaN not
    return true;
}

// Scalars of one step, in double from the caller's fp32 values (host side).
inline void host_step_scalars(const adagc_hyper& hp, int64_t step, RuleArgs& r, UpdateArgs& u)
{
    const double lr = hp.lr, b1 = hp.beta1, b2 = hp.beta2, wd = hp.weight_decay;
    const double t = (double)step;
    r.lambda_rel = (double)hp.lambda_rel;
    r.ema_beta = (double)hp.ema_beta;
    r.lambda_abs = (double)hp.lambda_abs;
    r.z_thres = (double)hp.z_thres;
    r.lr = lr;
    r.pad = 0;
    r.first_step = (step == 1) ? 1 : 0;
    r.warmup = ((step - 1) < (int64_t)hp.t_start) ? 1 : 0;   // steps 1..t_start
    r.mode = hp.clip_mode;
    u.beta1 = b1;
    u.one_minus_beta1 = 1.0 - b1;
    u.beta2 = b2;
    u.one_minus_beta2 = 1.0 - b2;
    u.inv_bias2 = 1.0 / (1.0 - std::pow(b2, t));
    u.step_size = lr / (1.0 - std::pow(b1, t));
    u.lr_wd = lr * wd;
    u.eps = (double)hp.eps;
    u.lr = lr;
    u.weight_decay = wd;
    u.inv_bias1 = 1.0 / (1.0 - std::pow(b1, t));
    u.update_clip = (hp.clip_mode == ADAGC_MODE_AGC || hp.clip_mode == ADAGC_MODE_CLIPPY) ? 1 : 0;
    u.pad = 0;
}

// Launchers (kernels.hip).  Each only enqueues on `stream`.
hipError_t launch_sumsq_partials(const DeviceTables& t, int grad_bf16, int nt, int grid, hipStream_t stream);
hipError_t launch_finalize_adagc(const DeviceTables& t, float* ema, const RuleArgs& r, hipStream_t stream);
hipError_t launch_finalize_global(const DeviceTables& t, float* ema, const RuleArgs& r, hipStream_t stream);
hipError_t launch_update(const DeviceTables& t, const UpdateArgs& u, int optimizer, int grad_bf16,
                         int with_copy, int unroll, int items_per_chunk, int nt, int tele, int grid,
                         hipStream_t stream, bool device_scalars = false);
// Update-clipping modes (AGC, Clippy): norms of theta and of the direction per work item, then one workgroup
// per tensor turns them into the tensor's update coefficient.
hipError_t launch_update_clip_rule(const DeviceTables& t, const UpdateArgs& u, const RuleArgs& r, int optimizer,
                                   int grad_bf16, int items_per_chunk, int nt, int grid, hipStream_t stream);
// Per-tensor sums of the per-chunk partials into t.sumsq (K2's fixed order); used by the Muon path for ||U||^2.
hipError_t launch_tensor_sumsq(const DeviceTables& t, hipStream_t stream);
// Rule stage of adagc_step_graph: scalars from device-resident step parameters, then the per-tensor
// sums, the model-wide rule (a no-op outside warm-up and the global modes) and the per-tensor rule.
hipError_t launch_rules_from_device(const DeviceTables& t, float* ema, const adagc_step_params* params,
                                    int optimizer, hipStream_t stream);

}  // namespace adagc
