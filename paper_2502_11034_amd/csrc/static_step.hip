// adagc_step_static: the step of adagc_step for callers that cannot allocate (code under HIP graph
// capture, tight serving loops, harnesses that forbid hipMalloc).  No context: the segment table,
// the per-chunk partial sums and the per-tensor results live in a fixed array in device memory that
// is part of this library's code object, one copy per GPU, held until the process ends.  The tensor
// records reach the GPU as kernel arguments, so there is no copy, no memset and no event either.
//
// The norm, rule and update kernels are the ones adagc_step launches (kernels.hip), given pointers
// into that array; the chunks are visited in list order.

#include <mutex>

#include "adagc_internal.h"

namespace adagc {
namespace {

constexpr size_t align256(size_t x) { return (x + 255) / 256 * 256; }

// Layout of the scratch array (byte offsets, each a multiple of 256).
constexpr size_t kMaxT = ADAGC_STATIC_MAX_TENSORS;
constexpr size_t kMaxC = ADAGC_STATIC_MAX_CHUNKS;
constexpr size_t kOffTargs = 0;
constexpr size_t kOffChunks = kOffTargs + align256(kMaxT * sizeof(TensorArgs));
constexpr size_t kOffPartials = kOffChunks + align256(kMaxC * sizeof(ChunkRef));
constexpr size_t kOffSumsq = kOffPartials + align256(kMaxC * sizeof(double));
constexpr size_t kOffCoef64 = kOffSumsq + align256(kMaxT * sizeof(double));
constexpr size_t kOffGlobal = kOffCoef64 + align256(kMaxT * sizeof(double));
constexpr size_t kOffNorm = kOffGlobal + align256(4 * sizeof(double));
constexpr size_t kOffCoef = kOffNorm + align256(kMaxT * sizeof(float));
constexpr size_t kOffFlag = kOffCoef + align256(kMaxT * sizeof(float));
constexpr size_t kScratchBytes = kOffFlag + align256(kMaxT);

// In host code this name is only a handle for hipGetSymbolAddress, never an address to hand to a kernel.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
void*      g_scratch_ptr[kMaxDevices];    // device address of `scratch` on each GPU, once looked up
bool       g_scratch_known[kMaxDevices];
std::mutex g_scratch_mutex;

// Device address of this GPU's copy of the array (`device` must be the current device).
hipError_t scratch_address(int device, unsigned char** out)
{
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_known[device]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = p;
        g_scratch_known[device] = true;
    }
    *out = static_cast<unsigned char*>(g_scratch_ptr[device]);
    return hipSuccess;
}

// Tensor records travel as kernel arguments, a batch per launch (the argument block is limited to 4 KiB).
constexpr int kBatch = 56;
struct TensorBatch {
    TensorArgs t[kBatch];
    uint32_t   first;    // list index of t[0]
    uint32_t   count;
};
static_assert(sizeof(TensorBatch) + 2 * sizeof(void*) <= 4096, "a batch fits the kernel-argument block");

// Workgroup b stores the record of tensor first+b and writes that tensor's rows of the chunk table.
__global__ __launch_bounds__(kBlock) void store_tensor_batch_kernel(TensorBatch batch, TensorArgs* targs, ChunkRef* chunks)
{
    const uint32_t b = blockIdx.x;
    if (b >= batch.count) return;
    const TensorArgs a = batch.t[b];
    const uint32_t i = batch.first + b;
    if (threadIdx.x == 0) targs[i] = a;
    for (uint32_t k = threadIdx.x; k < a.chunk_count; k += kBlock) chunks[a.chunk_begin + k] = ChunkRef{i, k};
}

inline bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

}  // namespace
}  // namespace adagc

using namespace adagc;

extern "C" int adagc_step_static(const adagc_tensor_desc* descs, int64_t n_tensors, const adagc_config* cfg,
                                 void* const* params, const void* const* grads, void* const* exp_avg,
                                 void* const* exp_avg_sq, void* const* params_bf16, float* ema_norms,
                                 const adagc_hyper* hp, int64_t step, float* out_norms, float* out_coefs,
                                 uint8_t* out_clipped, void* stream_v)
{
    if (!descs || !cfg || !params || !grads || !exp_avg || !ema_norms || !hp || n_tensors <= 0 || step < 1)
        return ADAGC_ERR_INVALID_ARG;
    if (cfg->optimizer != ADAGC_OPT_ADAMW && cfg->optimizer != ADAGC_OPT_LION) return ADAGC_ERR_INVALID_ARG;
    if (cfg->grad_dtype != ADAGC_GRAD_F32 && cfg->grad_dtype != ADAGC_GRAD_BF16) return ADAGC_ERR_INVALID_ARG;
    if (cfg->has_bf16_param_copy != 0 && cfg->has_bf16_param_copy != 1) return ADAGC_ERR_INVALID_ARG;
    // no telemetry and no launch tuning here: the defaults, chunks in list order
    if (cfg->telemetry != 0 || cfg->grid_blocks != 0 || cfg->unroll != 0 || cfg->nontemporal != 0 ||
        cfg->schedule != 0 || cfg->update_split != 0 || cfg->schedule_run != 0 || cfg->update_clipping != 0)
        return ADAGC_ERR_INVALID_ARG;
    const bool adamw = cfg->optimizer == ADAGC_OPT_ADAMW;
    const bool bf16g = cfg->grad_dtype == ADAGC_GRAD_BF16;
    const bool copy = cfg->has_bf16_param_copy != 0;
    if (adamw && !exp_avg_sq) return ADAGC_ERR_INVALID_ARG;
    if (copy && !params_bf16) return ADAGC_ERR_INVALID_ARG;
    if (!hyper_ok(*hp, cfg->optimizer) || hp->clip_mode > ADAGC_MODE_ZCLIP) return ADAGC_ERR_INVALID_ARG;
    if (n_tensors > (int64_t)kMaxT) return ADAGC_ERR_TOO_LARGE;

    // Everything is validated before anything is enqueued: one pass over the list.
    uint64_t n_chunks = 0;
    for (int64_t i = 0; i < n_tensors; ++i) {
        if (descs[i].numel <= 0 || descs[i].flags != 0 || descs[i].reserved != 0) return ADAGC_ERR_INVALID_ARG;
        if (!params[i] || !grads[i] || !exp_avg[i] || (adamw && !exp_avg_sq[i]) || (copy && !params_bf16[i]))
            return ADAGC_ERR_INVALID_ARG;
        n_chunks += (uint64_t)((descs[i].numel + kChunkElems - 1) / kChunkElems);
        if (n_chunks > (uint64_t)kMaxC) return ADAGC_ERR_TOO_LARGE;
    }

    int device = -1;
    if (hipGetDevice(&device) != hipSuccess) return ADAGC_ERR_HIP;
    if (device < 0 || device >= kMaxDevices) return ADAGC_ERR_HIP;
    unsigned char* base = nullptr;
    if (scratch_address(device, &base) != hipSuccess) return ADAGC_ERR_HIP;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);

    DeviceTables t{};
    TensorArgs* d_targs = reinterpret_cast<TensorArgs*>(base + kOffTargs);
    ChunkRef* d_chunks = reinterpret_cast<ChunkRef*>(base + kOffChunks);
    t.chunks = d_chunks;
    t.schedule = nullptr;                         // list order
    t.targs = d_targs;
    t.partials = reinterpret_cast<double*>(base + kOffPartials);
    t.sumsq = reinterpret_cast<double*>(base + kOffSumsq);
    t.coef64 = reinterpret_cast<double*>(base + kOffCoef64);
    t.global = reinterpret_cast<double*>(base + kOffGlobal);
    t.norm = out_norms ? out_norms : reinterpret_cast<float*>(base + kOffNorm);
    t.coef = out_coefs ? out_coefs : reinterpret_cast<float*>(base + kOffCoef);
    t.flag = out_clipped ? out_clipped : reinterpret_cast<uint8_t*>(base + kOffFlag);
    t.tele_partials = nullptr;
    t.tele_norm = nullptr;
    t.scalars = nullptr;
    t.n_chunks = (uint32_t)n_chunks;
    t.n_tensors = (uint32_t)n_tensors;

    // Tensor records and chunk table, a batch of tensors per launch.
    const uintptr_t grad_align = bf16g ? 8 : 16;
    uint32_t chunk_begin = 0;
    TensorBatch batch;
    for (int64_t first = 0; first < n_tensors; first += kBatch) {
        const int64_t count = (n_tensors - first) < kBatch ? (n_tensors - first) : kBatch;
        for (int64_t b = 0; b < count; ++b) {
            const int64_t i = first + b;
            TensorArgs& a = batch.t[b];
            a.param = params[i];
            a.grad = grads[i];
            a.exp_avg = exp_avg[i];
            a.exp_avg_sq = adamw ? exp_avg_sq[i] : nullptr;
            a.param_copy = copy ? params_bf16[i] : nullptr;
            a.numel = descs[i].numel;
            a.chunk_begin = chunk_begin;
            a.chunk_count = (uint32_t)((descs[i].numel + kChunkElems - 1) / kChunkElems);
            a.vec_ok = (aligned(a.param, 16) && aligned(a.exp_avg, 16) && aligned(a.grad, grad_align) &&
                        (!adamw || aligned(a.exp_avg_sq, 16)) && (!copy || aligned(a.param_copy, 8)))
                           ? 1u : 0u;
            a.pad = 0;
            chunk_begin += a.chunk_count;
        }
        for (int64_t b = count; b < kBatch; ++b) batch.t[b] = TensorArgs{};
        batch.first = (uint32_t)first;
        batch.count = (uint32_t)count;
        store_tensor_batch_kernel<<<dim3((uint32_t)count), dim3(kBlock), 0, stream>>>(batch, d_targs, d_chunks);
        if (hipGetLastError() != hipSuccess) return ADAGC_ERR_HIP;
    }

    RuleArgs r;
    UpdateArgs u;
    host_step_scalars(*hp, step, r, u);
    const bool global_rule = r.warmup || hp->clip_mode != ADAGC_MODE_ADAGC;
    const int items_per_chunk = kChunkElems >= 4096 ? kChunkElems / 4096 : 1;
    const int64_t items = (((int64_t)n_chunks + 7) / 8 * 8) * items_per_chunk;
    const int64_t max_grid = (int64_t)(0xFFFFFFFFu / (uint32_t)kBlock);
    const int grid_norm = (int)((int64_t)n_chunks > max_grid ? max_grid : (int64_t)n_chunks);
    const int grid_update = (int)(items > max_grid ? max_grid : items);

    if (launch_sumsq_partials(t, bf16g, 1, grid_norm, stream) != hipSuccess) return ADAGC_ERR_HIP;
    const hipError_t e = global_rule ? launch_finalize_global(t, ema_norms, r, stream)
                                     : launch_finalize_adagc(t, ema_norms, r, stream);
    if (e != hipSuccess) return ADAGC_ERR_HIP;
    if (launch_update(t, u, cfg->optimizer, bf16g, copy, 4, items_per_chunk, 1, 0, grid_update, stream) != hipSuccess)
        return ADAGC_ERR_HIP;
    return ADAGC_OK;
}
