// Host side of libadagc: context, argument validation, per-step scalar preparation and
// kernel sequencing.  See include/adagc.h for the contract of every entry point.

#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "adagc_internal.h"
#include "muon_internal.h"

using namespace adagc;

struct adagc_ctx {
    int          device = 0;
    int64_t      n_tensors = 0;
    int64_t      n_chunks = 0;
    adagc_config cfg{};
    int          grid_norm = 0;     // workgroups of the norm kernel
    int          grid_update = 0;   // workgroups of the update kernel
    int          unroll = 0;
    int          nontemporal = 0;
    int          items_per_chunk = 1;   // work items of the update kernel per chunk

    std::vector<int64_t>    numel;
    std::vector<int64_t>    chunk_begin;      // n_tensors + 1
    std::vector<void*>      param_copies;     // device pointers, empty until set
    std::vector<TensorArgs> cached_args;      // what the device table currently holds
    std::vector<TensorArgs> scratch_args;     // rebuilt on every step, then compared
    bool                    args_uploaded = false;

    void*        slab = nullptr;              // single device allocation, carved below
    DeviceTables tables{};
    TensorArgs*  d_targs = nullptr;
    // Pinned host mirrors for the asynchronous upload of the pointer table: a ring, so that a caller
    // who alternates between pointer sets (two gradient buffers, say) does not have to wait for the
    // previous upload before the next one can be staged.
    static constexpr int kStagingSlots = 4;
    TensorArgs*  staging = nullptr;           // kStagingSlots consecutive tables
    hipEvent_t   upload_done[kStagingSlots] = {nullptr, nullptr, nullptr, nullptr};
    bool         upload_pending[kStagingSlots] = {false, false, false, false};
    uint64_t     uploads = 0;                 // tables uploaded so far; slot = uploads % kStagingSlots
    bool         device_scalars_used = false;   // adagc_step_graph was called: its status word is meaningful

    // Muon (adagc_muon_attach): shapes, the batches the Newton-Schulz iteration runs in (matrices of one padded
    // shape, iterated together by batched launches) and the workspace one batch at a time is carved out of
    struct MuonBatch {
        int mp = 0, np = 0;                  // padded extent of the wide orientation
        std::vector<int64_t> members;        // tensor indices
    };
    std::vector<adagc_matrix_shape> shapes;
    std::vector<MuonBatch> muon_batches;
    void*  muon_ws = nullptr;
    size_t muon_ws_bytes = 0;

    std::vector<hipEvent_t> prof_events;      // 4 per step while profiling
    int32_t                 prof_capacity = 0;
    int32_t                 prof_steps = 0;
};

namespace {

struct DeviceGuard {
    int  prev = -1;
    bool ok = true;
    explicit DeviceGuard(int dev)
    {
        if (hipGetDevice(&prev) != hipSuccess) { ok = false; return; }
        if (prev != dev && hipSetDevice(dev) != hipSuccess) ok = false;
    }
    ~DeviceGuard()
    {
        int cur = -1;
        if (ok && hipGetDevice(&cur) == hipSuccess && cur != prev) (void)hipSetDevice(prev);
    }
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Largest grid this library launches: the runtime wants workgroups x lanes below 2^32.
constexpr int64_t kMaxGridBlocks = (int64_t)(0xFFFFFFFFu / (uint32_t)kBlock);

inline bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

void free_ctx(adagc_ctx* c)
{
    if (!c) return;
    for (hipEvent_t e : c->prof_events) (void)hipEventDestroy(e);
    for (hipEvent_t e : c->upload_done)
        if (e) (void)hipEventDestroy(e);
    if (c->muon_ws) (void)hipFree(c->muon_ws);
    if (c->staging) (void)hipHostFree(c->staging);
    if (c->slab) (void)hipFree(c->slab);
    delete c;
}

}  // namespace

extern "C" int64_t adagc_chunk_elems(void) { return kChunkElems; }

extern "C" const char* adagc_strerror(int code)
{
    switch (code) {
    case ADAGC_OK: return "ok";
    case ADAGC_ERR_INVALID_ARG: return "invalid argument";
    case ADAGC_ERR_OOM: return "out of memory";
    case ADAGC_ERR_HIP: return "HIP runtime error";
    case ADAGC_ERR_TOO_LARGE: return "tensor list too large (too many chunks or tensors)";
    case ADAGC_ERR_STATE: return "call made in the wrong state";
    default: return "unknown error code";
    }
}

extern "C" int adagc_create(adagc_ctx** out, const adagc_tensor_desc* descs, int64_t n_tensors,
                            const adagc_config* cfg)
{
    if (!out || !descs || !cfg || n_tensors <= 0) return ADAGC_ERR_INVALID_ARG;
    if (cfg->optimizer != ADAGC_OPT_ADAMW && cfg->optimizer != ADAGC_OPT_LION && cfg->optimizer != ADAGC_OPT_MUON)
        return ADAGC_ERR_INVALID_ARG;
    if (cfg->optimizer == ADAGC_OPT_MUON && (cfg->telemetry || cfg->update_clipping)) return ADAGC_ERR_INVALID_ARG;
    if (cfg->grad_dtype != ADAGC_GRAD_F32 && cfg->grad_dtype != ADAGC_GRAD_BF16) return ADAGC_ERR_INVALID_ARG;
    if (cfg->has_bf16_param_copy != 0 && cfg->has_bf16_param_copy != 1) return ADAGC_ERR_INVALID_ARG;
    if (cfg->grid_blocks < 0 || cfg->nontemporal < 0 || cfg->nontemporal > 2 || cfg->schedule < 0 ||
        cfg->schedule_run < 0 || cfg->telemetry < 0 || cfg->telemetry > 1 || cfg->update_clipping < 0 ||
        cfg->update_clipping > 1)
        return ADAGC_ERR_INVALID_ARG;
    if (cfg->unroll != 0 && cfg->unroll != 1 && cfg->unroll != 2 && cfg->unroll != 4) return ADAGC_ERR_INVALID_ARG;
    {
        const int tiles = kVecPerLane / (cfg->unroll ? cfg->unroll : 4);       // unroll*1024-element tiles per chunk
        const int sp = cfg->update_split;
        if (sp < 0 || sp > tiles || (sp & (sp - 1)) != 0) return ADAGC_ERR_INVALID_ARG;
    }
    if (n_tensors > kMaxGridBlocks) return ADAGC_ERR_TOO_LARGE;   // the per-tensor kernels run one workgroup per tensor

    adagc_ctx* c = new (std::nothrow) adagc_ctx;
    if (!c) return ADAGC_ERR_OOM;
    int rc = ADAGC_OK;
    std::vector<uint32_t> chunk_tensor, chunk_index;
    try {
        c->chunk_begin.resize((size_t)n_tensors + 1);
        int64_t n_chunks = 0;
        rc = adagc_build_segment_table(descs, n_tensors, kChunkElems, c->chunk_begin.data(), nullptr,
                                       nullptr, 0, &n_chunks);
        if (rc != ADAGC_OK) { free_ctx(c); return rc; }
        chunk_tensor.resize((size_t)n_chunks);
        chunk_index.resize((size_t)n_chunks);
        rc = adagc_build_segment_table(descs, n_tensors, kChunkElems, c->chunk_begin.data(),
                                       chunk_tensor.data(), chunk_index.data(), n_chunks, &n_chunks);
        if (rc != ADAGC_OK) { free_ctx(c); return rc; }
        c->n_tensors = n_tensors;
        c->n_chunks = n_chunks;
        c->cfg = *cfg;
        c->numel.resize((size_t)n_tensors);
        for (int64_t i = 0; i < n_tensors; ++i) c->numel[(size_t)i] = descs[i].numel;
        c->cached_args.assign((size_t)n_tensors, TensorArgs{});
        c->scratch_args.assign((size_t)n_tensors, TensorArgs{});
    } catch (const std::bad_alloc&) {
        free_ctx(c);
        return ADAGC_ERR_OOM;
    }

    if (hipGetDevice(&c->device) != hipSuccess) {
        free_ctx(c);
        return ADAGC_ERR_HIP;
    }
    // Launch defaults, each chosen by measurement on Llama-3-8B shapes (see the profiles):
    //  - one work item (a chunk in the norm kernel, a tile in the update kernel) per workgroup,
    //    dispatched by the hardware, beat a static persistent grid by 1.5-2 % (a CU that falls
    //    behind simply receives fewer); grid_blocks > 0 selects a persistent grid of that many
    //    workgroups, each walking items b, b+grid, ...
    //  - non-temporal loads/stores in the update kernel: +4.5 %
    //  - visiting order: the list cut into 2 halves, the 4 XCDs that share a half (workgroup b goes
    //    to XCD b mod 8) taking runs of 8 chunks (512 KiB of each fp32 array) in turn.  Against
    //    list order: norm kernel -5 %, update -3.5 %; against 8 parts (one per XCD): update
    //    -1.9 % (AdamW, 8 B parameters), -0.4 % (Lion), -1.2 % (20 001 ragged tensors).  Fewer
    //    address fronts per array mean fewer DRAM rows open at once; runs keep each XCD on
    //    its own pages.
    c->unroll = cfg->unroll ? cfg->unroll : 4;
    c->nontemporal = cfg->nontemporal == 2 ? 0 : 1;
    //  - work items of the update kernel: 4096 elements, a quarter of a chunk.  Against whole
    //    chunks: AdamW on Llama-3-8B shapes -0.1 %, Lion -3.1 %, a 20 001-tensor ragged list
    //    +0.2 %, 0.1-0.5 B-parameter lists -1.5...-3.7 % (shorter tail of the launch), a list of
    //    50 chunks -25 % (more workgroups to spread over the CUs).  Halves are 0.9 % slower than
    //    either on the 8 B list, and 1024-element items 16 % slower.
    // Both streaming kernels walk their work items b, b+grid, ..., so any grid size is valid.
    c->items_per_chunk = cfg->update_split ? cfg->update_split : (kChunkElems >= 4096 ? kChunkElems / 4096 : 1);
    const int64_t tiles = ((c->n_chunks + 7) / 8 * 8) * c->items_per_chunk;
    auto grid_for = [cfg](int64_t items) {
        int64_t want = cfg->grid_blocks > 0 ? (int64_t)cfg->grid_blocks : items;
        if (want > items) want = items;
        return (int)(want > kMaxGridBlocks ? kMaxGridBlocks : want);
    };
    c->grid_norm = grid_for(c->n_chunks);
    c->grid_update = grid_for(tiles);

    // One slab, carved into 256-byte aligned arrays.
    const size_t nt = (size_t)n_tensors, nc = (size_t)c->n_chunks;
    size_t off = 0;
    auto carve = [&off](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    const size_t o_chunks = carve(nc * sizeof(ChunkRef));
    const size_t o_schedule = carve(nc * sizeof(uint32_t));
    const size_t o_targs = carve(nt * sizeof(TensorArgs));
    const size_t o_partials = carve(nc * sizeof(double));
    const size_t o_sumsq = carve(nt * sizeof(double));
    const size_t o_global = carve(4 * sizeof(double));
    const size_t o_scalars = carve(sizeof(StepScalars));
    const size_t o_coef64 = carve(nt * sizeof(double));
    const size_t o_norm = carve(nt * sizeof(float));
    const size_t o_coef = carve(nt * sizeof(float));
    const size_t o_flag = carve(nt);
    const size_t tiles_per_chunk = (size_t)c->items_per_chunk;
    const size_t o_tele_partials = carve(cfg->telemetry ? 3 * nc * tiles_per_chunk * sizeof(double) : 0);
    const size_t o_tele_norm = carve(cfg->telemetry ? 3 * nt * sizeof(float) : 0);
    const size_t o_ustat = carve(cfg->update_clipping ? 2 * nc * tiles_per_chunk * sizeof(double) : 0);
    const size_t o_ucoef64 = carve(cfg->update_clipping ? nt * sizeof(double) : 0);
    const size_t slab_bytes = off;

    hipError_t e = hipMalloc(&c->slab, slab_bytes);
    if (e != hipSuccess) { free_ctx(c); return e == hipErrorOutOfMemory ? ADAGC_ERR_OOM : ADAGC_ERR_HIP; }
    char* base = static_cast<char*>(c->slab);
    if (hipMemset(c->slab, 0, slab_bytes) != hipSuccess) { free_ctx(c); return ADAGC_ERR_HIP; }

    std::vector<ChunkRef> refs;
    try {
        refs.resize(nc);
    } catch (const std::bad_alloc&) { free_ctx(c); return ADAGC_ERR_OOM; }
    for (size_t k = 0; k < nc; ++k) refs[k] = ChunkRef{chunk_tensor[k], chunk_index[k]};
    if (hipMemcpy(base + o_chunks, refs.data(), nc * sizeof(ChunkRef), hipMemcpyHostToDevice) != hipSuccess) {
        free_ctx(c);
        return ADAGC_ERR_HIP;
    }
    // Visiting order of the streaming kernels (see adagc_build_visiting_order).
    {
        std::vector<uint32_t> order;
        try {
            order.resize(nc);
        } catch (const std::bad_alloc&) { free_ctx(c); return ADAGC_ERR_OOM; }
        rc = adagc_build_visiting_order(c->n_chunks, cfg->schedule ? cfg->schedule : 2,
                                        cfg->schedule_run ? cfg->schedule_run : 8, order.data());
        if (rc != ADAGC_OK) { free_ctx(c); return rc; }
        if (hipMemcpy(base + o_schedule, order.data(), nc * sizeof(uint32_t), hipMemcpyHostToDevice) != hipSuccess) {
            free_ctx(c);
            return ADAGC_ERR_HIP;
        }
    }
    if (hipHostMalloc(reinterpret_cast<void**>(&c->staging), adagc_ctx::kStagingSlots * nt * sizeof(TensorArgs),
                      hipHostMallocDefault) != hipSuccess) {
        free_ctx(c);
        return ADAGC_ERR_HIP;
    }
    for (hipEvent_t& ev : c->upload_done)
        if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) {
            free_ctx(c);
            return ADAGC_ERR_HIP;
        }

    c->d_targs = reinterpret_cast<TensorArgs*>(base + o_targs);
    DeviceTables& t = c->tables;
    t.chunks = reinterpret_cast<const ChunkRef*>(base + o_chunks);
    t.schedule = reinterpret_cast<const uint32_t*>(base + o_schedule);
    t.targs = c->d_targs;
    t.partials = reinterpret_cast<double*>(base + o_partials);
    t.sumsq = reinterpret_cast<double*>(base + o_sumsq);
    t.global = reinterpret_cast<double*>(base + o_global);
    t.scalars = reinterpret_cast<StepScalars*>(base + o_scalars);
    t.coef64 = reinterpret_cast<double*>(base + o_coef64);
    t.norm = reinterpret_cast<float*>(base + o_norm);
    t.coef = reinterpret_cast<float*>(base + o_coef);
    t.flag = reinterpret_cast<uint8_t*>(base + o_flag);
    t.tele_partials = cfg->telemetry ? reinterpret_cast<double*>(base + o_tele_partials) : nullptr;
    t.tele_norm = cfg->telemetry ? reinterpret_cast<float*>(base + o_tele_norm) : nullptr;
    t.ustat_partials = cfg->update_clipping ? reinterpret_cast<double*>(base + o_ustat) : nullptr;
    t.ucoef64 = cfg->update_clipping ? reinterpret_cast<double*>(base + o_ucoef64) : nullptr;
    t.n_chunks = (uint32_t)c->n_chunks;
    t.n_tensors = (uint32_t)c->n_tensors;

    *out = c;
    return ADAGC_OK;
}

extern "C" void adagc_destroy(adagc_ctx* ctx)
{
    if (!ctx) return;
    DeviceGuard guard(ctx->device);
    free_ctx(ctx);
}

extern "C" int64_t adagc_num_tensors(const adagc_ctx* ctx) { return ctx ? ctx->n_tensors : ADAGC_ERR_INVALID_ARG; }
extern "C" int64_t adagc_num_chunks(const adagc_ctx* ctx) { return ctx ? ctx->n_chunks : ADAGC_ERR_INVALID_ARG; }

extern "C" int adagc_set_param_copies(adagc_ctx* ctx, void* const* params_bf16)
{
    if (!ctx || !params_bf16) return ADAGC_ERR_INVALID_ARG;
    if (!ctx->cfg.has_bf16_param_copy) return ADAGC_ERR_STATE;
    for (int64_t i = 0; i < ctx->n_tensors; ++i)
        if (!params_bf16[i]) return ADAGC_ERR_INVALID_ARG;
    try {
        ctx->param_copies.assign(params_bf16, params_bf16 + ctx->n_tensors);
    } catch (const std::bad_alloc&) { return ADAGC_ERR_OOM; }
    return ADAGC_OK;
}

namespace {

// Shared front half of the two step entry points: argument checks, per-tensor records, upload of the
// pointer table when it changed.  `capturing` forbids everything but kernel launches.
int prepare_tables(adagc_ctx* ctx, void* const* params, const void* const* grads, void* const* exp_avg,
                   void* const* exp_avg_sq, hipStream_t stream, bool capturing)
{
    const bool adamw = ctx->cfg.optimizer == ADAGC_OPT_ADAMW;
    const bool bf16g = ctx->cfg.grad_dtype == ADAGC_GRAD_BF16;
    const bool copy = ctx->cfg.has_bf16_param_copy != 0;
    if (adamw && !exp_avg_sq) return ADAGC_ERR_INVALID_ARG;
    if (copy && ctx->param_copies.size() != (size_t)ctx->n_tensors) return ADAGC_ERR_STATE;

    // Rebuild the per-tensor records from the caller's pointer arrays.
    const uintptr_t grad_align = bf16g ? 8 : 16;
    for (int64_t i = 0; i < ctx->n_tensors; ++i) {
        TensorArgs& a = ctx->scratch_args[(size_t)i];
        a.param = params[i];
        a.grad = grads[i];
        a.exp_avg = exp_avg[i];
        a.exp_avg_sq = adamw ? exp_avg_sq[i] : nullptr;
        a.param_copy = copy ? ctx->param_copies[(size_t)i] : nullptr;
        if (!a.param || !a.grad || !a.exp_avg || (adamw && !a.exp_avg_sq)) return ADAGC_ERR_INVALID_ARG;
        a.numel = ctx->numel[(size_t)i];
        a.chunk_begin = (uint32_t)ctx->chunk_begin[(size_t)i];
        a.chunk_count = (uint32_t)(ctx->chunk_begin[(size_t)i + 1] - ctx->chunk_begin[(size_t)i]);
        a.vec_ok = (aligned(a.param, 16) && aligned(a.exp_avg, 16) && aligned(a.grad, grad_align) &&
                    (!adamw || aligned(a.exp_avg_sq, 16)) && (!copy || aligned(a.param_copy, 8)))
                       ? 1u : 0u;
        a.pad = 0;
    }

    const size_t args_bytes = (size_t)ctx->n_tensors * sizeof(TensorArgs);
    if (!ctx->args_uploaded ||
        std::memcmp(ctx->scratch_args.data(), ctx->cached_args.data(), args_bytes) != 0) {
        if (capturing) return ADAGC_ERR_STATE;   // a recorded copy would re-read the staging buffer on every replay
        // Next slot of the staging ring.  It may still be the source of the upload made kStagingSlots
        // table changes ago; only then (the host that far ahead of the GPU) does this call wait.
        const int slot = (int)(ctx->uploads % adagc_ctx::kStagingSlots);
        if (ctx->upload_pending[slot] && hipEventSynchronize(ctx->upload_done[slot]) != hipSuccess) return ADAGC_ERR_HIP;
        TensorArgs* stage = ctx->staging + (size_t)slot * (size_t)ctx->n_tensors;
        std::memcpy(stage, ctx->scratch_args.data(), args_bytes);
        if (hipMemcpyAsync(ctx->d_targs, stage, args_bytes, hipMemcpyHostToDevice, stream) != hipSuccess ||
            hipEventRecord(ctx->upload_done[slot], stream) != hipSuccess)
            return ADAGC_ERR_HIP;
        ctx->upload_pending[slot] = true;
        ctx->uploads++;
        ctx->cached_args.swap(ctx->scratch_args);
        ctx->args_uploaded = true;
    }
    return ADAGC_OK;
}

}  // namespace

extern "C" int adagc_step(adagc_ctx* ctx, void* const* params, const void* const* grads,
                          void* const* exp_avg, void* const* exp_avg_sq, float* ema_norms,
                          const adagc_hyper* hp, int64_t step, void* stream_v)
{
    if (!ctx || !params || !grads || !exp_avg || !ema_norms || !hp || step < 1) return ADAGC_ERR_INVALID_ARG;
    if (ctx->cfg.optimizer == ADAGC_OPT_MUON) return ADAGC_ERR_STATE;      // stepped with adagc_muon_step
    if (!hyper_ok(*hp, ctx->cfg.optimizer)) return ADAGC_ERR_INVALID_ARG;
    const bool update_clip = hp->clip_mode == ADAGC_MODE_AGC || hp->clip_mode == ADAGC_MODE_CLIPPY;
    if (update_clip && !ctx->cfg.update_clipping) return ADAGC_ERR_STATE;
    const bool bf16g = ctx->cfg.grad_dtype == ADAGC_GRAD_BF16;
    const bool copy = ctx->cfg.has_bf16_param_copy != 0;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return ADAGC_ERR_HIP;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    const int rc = prepare_tables(ctx, params, grads, exp_avg, exp_avg_sq, stream, false);
    if (rc != ADAGC_OK) return rc;

    RuleArgs r;
    UpdateArgs u;
    host_step_scalars(*hp, step, r, u);
    const bool global_rule = r.warmup || hp->clip_mode != ADAGC_MODE_ADAGC;
    ctx->device_scalars_used = false;
    const bool prof = ctx->prof_steps < ctx->prof_capacity;
    hipEvent_t* ev = prof ? &ctx->prof_events[(size_t)ctx->prof_steps * 4] : nullptr;

    if (prof && hipEventRecord(ev[0], stream) != hipSuccess) return ADAGC_ERR_HIP;
    if (update_clip) {
        // AGC / Clippy: no gradient norms; the direction's norms (timed in the norm slot together with their
        // per-tensor rule), then the update scales the direction
        if (launch_update_clip_rule(ctx->tables, u, r, ctx->cfg.optimizer, bf16g, ctx->items_per_chunk, ctx->nontemporal,
                                    ctx->grid_update, stream) != hipSuccess)
            return ADAGC_ERR_HIP;
        if (prof && (hipEventRecord(ev[1], stream) != hipSuccess || hipEventRecord(ev[2], stream) != hipSuccess))
            return ADAGC_ERR_HIP;
    } else {
        if (launch_sumsq_partials(ctx->tables, bf16g, ctx->nontemporal, ctx->grid_norm, stream) != hipSuccess) return ADAGC_ERR_HIP;
        if (prof && hipEventRecord(ev[1], stream) != hipSuccess) return ADAGC_ERR_HIP;
        const hipError_t e = global_rule ? launch_finalize_global(ctx->tables, ema_norms, r, stream)
                                         : launch_finalize_adagc(ctx->tables, ema_norms, r, stream);
        if (e != hipSuccess) return ADAGC_ERR_HIP;
        if (prof && hipEventRecord(ev[2], stream) != hipSuccess) return ADAGC_ERR_HIP;
    }
    if (launch_update(ctx->tables, u, ctx->cfg.optimizer, bf16g, copy, ctx->unroll, ctx->items_per_chunk,
                      ctx->nontemporal, ctx->cfg.telemetry, ctx->grid_update, stream) != hipSuccess)
        return ADAGC_ERR_HIP;
    if (prof) {
        if (hipEventRecord(ev[3], stream) != hipSuccess) return ADAGC_ERR_HIP;
        ctx->prof_steps++;
    }
    return ADAGC_OK;
}

extern "C" int adagc_step_graph(adagc_ctx* ctx, void* const* params, const void* const* grads,
                                void* const* exp_avg, void* const* exp_avg_sq, float* ema_norms,
                                const adagc_step_params* step_params, void* stream_v)
{
    if (!ctx || !params || !grads || !exp_avg || !ema_norms || !step_params) return ADAGC_ERR_INVALID_ARG;
    if (ctx->cfg.optimizer == ADAGC_OPT_MUON) return ADAGC_ERR_STATE;
    const bool bf16g = ctx->cfg.grad_dtype == ADAGC_GRAD_BF16;
    const bool copy = ctx->cfg.has_bf16_param_copy != 0;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return ADAGC_ERR_HIP;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &cap) != hipSuccess) return ADAGC_ERR_HIP;
    const bool capturing = cap != hipStreamCaptureStatusNone;
    if (capturing && ctx->prof_capacity > 0) return ADAGC_ERR_STATE;     // event records do not belong in a graph
    const int rc = prepare_tables(ctx, params, grads, exp_avg, exp_avg_sq, stream, capturing);
    if (rc != ADAGC_OK) return rc;

    const bool prof = !capturing && ctx->prof_steps < ctx->prof_capacity;
    hipEvent_t* ev = prof ? &ctx->prof_events[(size_t)ctx->prof_steps * 4] : nullptr;
    ctx->device_scalars_used = true;
    if (prof && hipEventRecord(ev[0], stream) != hipSuccess) return ADAGC_ERR_HIP;
    if (launch_sumsq_partials(ctx->tables, bf16g, ctx->nontemporal, ctx->grid_norm, stream) != hipSuccess) return ADAGC_ERR_HIP;
    if (prof && hipEventRecord(ev[1], stream) != hipSuccess) return ADAGC_ERR_HIP;
    if (launch_rules_from_device(ctx->tables, ema_norms, step_params, ctx->cfg.optimizer, stream) != hipSuccess)
        return ADAGC_ERR_HIP;
    if (prof && hipEventRecord(ev[2], stream) != hipSuccess) return ADAGC_ERR_HIP;
    if (launch_update(ctx->tables, UpdateArgs{}, ctx->cfg.optimizer, bf16g, copy, ctx->unroll, ctx->items_per_chunk,
                      ctx->nontemporal, ctx->cfg.telemetry, ctx->grid_update, stream, true) != hipSuccess)
        return ADAGC_ERR_HIP;
    if (prof) {
        if (hipEventRecord(ev[3], stream) != hipSuccess) return ADAGC_ERR_HIP;
        ctx->prof_steps++;
    }
    return ADAGC_OK;
}

// ---------------------------------------------------------------------------------------------
// Muon

namespace {
constexpr int64_t kMuonTile = 128;     // the matrix-core kernel's block tile: workspace matrices are padded to it
// Matrices of one padded shape are iterated together, up to this many per batched launch and as many as fit this much
// workspace (32 matrices of 4096 x 14336 take 17.2 GB).  32 is where the symmetric products of 4096-row matrices fill
// whole rounds of workgroups: 32 x 136 tiles of 256 x 256 = 17 x 256 compute units.
constexpr int64_t kMuonMaxBatch = 32;
constexpr int64_t kMuonWorkspaceBudget = (int64_t)24 << 30;
inline int64_t pad_to_tile(int64_t x) { return (x + kMuonTile - 1) / kMuonTile * kMuonTile; }
// bf16 elements of workspace per matrix: X and Y = X^T twice (a step reads one pair and writes the other), A and B
inline int64_t muon_ws_elems(int64_t mp, int64_t np) { return 4 * mp * np + 2 * mp * mp; }
}  // namespace

extern "C" int adagc_muon_attach(adagc_ctx* ctx, const adagc_matrix_shape* shapes)
{
    if (!ctx || !shapes) return ADAGC_ERR_INVALID_ARG;
    if (ctx->cfg.optimizer != ADAGC_OPT_MUON || ctx->muon_ws) return ADAGC_ERR_STATE;
    std::vector<adagc_ctx::MuonBatch> groups, batches;
    try {
        for (int64_t i = 0; i < ctx->n_tensors; ++i) {
            const int64_t r = shapes[i].rows, c = shapes[i].cols;
            if (r <= 0 || c <= 0 || r > INT32_MAX || c > INT32_MAX || r * c != ctx->numel[(size_t)i]) return ADAGC_ERR_INVALID_ARG;
            const int64_t mp = pad_to_tile(r < c ? r : c), np = pad_to_tile(r < c ? c : r);
            if (np > INT32_MAX || np / 64 > 65535) return ADAGC_ERR_TOO_LARGE;
            size_t g = 0;
            while (g < groups.size() && (groups[g].mp != mp || groups[g].np != np)) ++g;
            if (g == groups.size()) {
                groups.emplace_back();
                groups[g].mp = (int)mp;
                groups[g].np = (int)np;
            }
            groups[g].members.push_back(i);
        }
        ctx->shapes.assign(shapes, shapes + ctx->n_tensors);
    } catch (const std::bad_alloc&) { return ADAGC_ERR_OOM; }
    DeviceGuard guard(ctx->device);
    if (!guard.ok) {
        ctx->shapes.clear();
        return ADAGC_ERR_HIP;
    }
    // Cut every group into batches of equal size (to one matrix), as large as the limits allow, and allocate the
    // workspace for the largest batch.  If the device cannot give that much, try again with half the batch limit.
    for (int64_t limit = kMuonMaxBatch;; limit /= 2) {
        int64_t ws_elems = 0;
        try {
            batches.clear();
            for (const adagc_ctx::MuonBatch& grp : groups) {
                const int64_t per_matrix = muon_ws_elems(grp.mp, grp.np) * (int64_t)sizeof(uint16_t);
                int64_t cap = kMuonWorkspaceBudget / per_matrix;
                if (cap > limit) cap = limit;
                if (cap < 1) cap = 1;
                const int64_t count = (int64_t)grp.members.size();
                const int64_t n_batches = (count + cap - 1) / cap;
                const int64_t size = (count + n_batches - 1) / n_batches;
                for (int64_t first = 0; first < count; first += size) {
                    const int64_t n = count - first < size ? count - first : size;
                    batches.emplace_back();
                    batches.back().mp = grp.mp;
                    batches.back().np = grp.np;
                    batches.back().members.assign(grp.members.begin() + first, grp.members.begin() + first + n);
                    const int64_t need = n * muon_ws_elems(grp.mp, grp.np);
                    if (need > ws_elems) ws_elems = need;
                }
            }
        } catch (const std::bad_alloc&) {
            ctx->shapes.clear();
            return ADAGC_ERR_OOM;
        }
        const size_t bytes = (size_t)ws_elems * sizeof(uint16_t);
        const hipError_t e = hipMalloc(&ctx->muon_ws, bytes);
        if (e == hipSuccess) {
            ctx->muon_ws_bytes = bytes;
            break;
        }
        ctx->muon_ws = nullptr;
        (void)hipGetLastError();          // the failed allocation is handled here: do not leave its error for the next call
        if (e != hipErrorOutOfMemory || limit == 1) {
            ctx->shapes.clear();
            return e == hipErrorOutOfMemory ? ADAGC_ERR_OOM : ADAGC_ERR_HIP;
        }
    }
    ctx->muon_batches.swap(batches);
    return ADAGC_OK;
}

extern "C" int64_t adagc_muon_workspace_bytes(const adagc_ctx* ctx) { return ctx && ctx->muon_ws ? (int64_t)ctx->muon_ws_bytes : 0; }

extern "C" int adagc_muon_step(adagc_ctx* ctx, void* const* params, const void* const* grads, void* const* momentum,
                               float* ema_norms, const adagc_hyper* hp, const adagc_muon_hyper* mh, int64_t step,
                               void* stream_v)
{
    if (!ctx || !params || !grads || !momentum || !ema_norms || !hp || !mh || step < 1) return ADAGC_ERR_INVALID_ARG;
    if (ctx->cfg.optimizer != ADAGC_OPT_MUON || !ctx->muon_ws) return ADAGC_ERR_STATE;
    adagc_hyper h = *hp;
    h.beta1 = 0.0f;     // Adam's rates and epsilon play no part here; neutral values pass the shared check
    h.beta2 = 0.0f;
    h.eps = 0.0f;
    if (!hyper_ok(h, ADAGC_OPT_LION) || h.clip_mode > ADAGC_MODE_ZCLIP) return ADAGC_ERR_INVALID_ARG;
    if (!(mh->momentum >= 0.0f && mh->momentum < 1.0f) || (mh->nesterov != 0 && mh->nesterov != 1) || mh->ns_steps < 0 ||
        mh->ns_steps > 16 || mh->reserved != 0)
        return ADAGC_ERR_INVALID_ARG;
    const bool bf16g = ctx->cfg.grad_dtype == ADAGC_GRAD_BF16;
    const bool copy = ctx->cfg.has_bf16_param_copy != 0;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return ADAGC_ERR_HIP;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    const int rc = prepare_tables(ctx, params, grads, momentum, nullptr, stream, false);
    if (rc != ADAGC_OK) return rc;

    RuleArgs r;
    UpdateArgs u;
    host_step_scalars(h, step, r, u);
    const bool global_rule = r.warmup || h.clip_mode != ADAGC_MODE_ADAGC;
    ctx->device_scalars_used = false;
    const bool prof = ctx->prof_steps < ctx->prof_capacity;
    hipEvent_t* ev = prof ? &ctx->prof_events[(size_t)ctx->prof_steps * 4] : nullptr;
    const DeviceTables& t = ctx->tables;

    // gradient norms and clip coefficients: the kernels of adagc_step
    if (prof && hipEventRecord(ev[0], stream) != hipSuccess) return ADAGC_ERR_HIP;
    if (launch_sumsq_partials(t, bf16g, ctx->nontemporal, ctx->grid_norm, stream) != hipSuccess) return ADAGC_ERR_HIP;
    if (prof && hipEventRecord(ev[1], stream) != hipSuccess) return ADAGC_ERR_HIP;
    const hipError_t e = global_rule ? launch_finalize_global(t, ema_norms, r, stream) : launch_finalize_adagc(t, ema_norms, r, stream);
    if (e != hipSuccess) return ADAGC_ERR_HIP;
    if (prof && hipEventRecord(ev[2], stream) != hipSuccess) return ADAGC_ERR_HIP;

    // momentum with the clipped gradient, and ||U||_F^2 of every tensor
    const double mu = (double)mh->momentum;
    if (launch_muon_momentum(t, mu, mh->nesterov, bf16g, ctx->grid_norm, stream) != hipSuccess) return ADAGC_ERR_HIP;
    if (launch_tensor_sumsq(t, stream) != hipSuccess) return ADAGC_ERR_HIP;

    // Newton-Schulz and the update, batch by batch.  Matrix z of a batch has slot z of each workspace array:
    // X is mp x np (leading dimension np), Y = X^T is np x mp (leading dimension mp), A and B are mp x mp.
    const float ns_a = 3.4445f, ns_b = -4.7750f, ns_c = 2.0315f;
    for (const adagc_ctx::MuonBatch& bt : ctx->muon_batches) {
        const int mp = bt.mp, np = bt.np;
        const int count = (int)bt.members.size();
        const int64_t mn = (int64_t)mp * np, mm = (int64_t)mp * mp;
        uint16_t* base = static_cast<uint16_t*>(ctx->muon_ws);
        uint16_t *x = base, *x2 = base + count * mn, *y = base + 2 * count * mn, *y2 = base + 3 * count * mn;
        uint16_t *wa = base + 4 * count * mn, *wb = wa + count * mm;
        for (int z = 0; z < count; ++z) {
            const int64_t i = bt.members[(size_t)z];
            const int64_t rows = ctx->shapes[(size_t)i].rows, cols = ctx->shapes[(size_t)i].cols;
            const bool flip = rows > cols;                  // the iteration runs on the wide orientation
            const hipError_t g =
                flip ? launch_muon_normalise(grads[i], momentum[i], rows, cols, np, mp, t.coef64 + i, t.sumsq + i, mu, mh->nesterov,
                                             bf16g, y + z * mn, mp, x + z * mn, np, stream)
                     : launch_muon_normalise(grads[i], momentum[i], rows, cols, mp, np, t.coef64 + i, t.sumsq + i, mu, mh->nesterov,
                                             bf16g, x + z * mn, np, y + z * mn, mp, stream);
            if (g != hipSuccess) return ADAGC_ERR_HIP;
        }
        bool any_tall = false, any_wide = false;
        for (int64_t i : bt.members) {
            if (ctx->shapes[(size_t)i].rows > ctx->shapes[(size_t)i].cols) any_tall = true;
            else any_wide = true;
        }
        for (int k = 0; k < mh->ns_steps; ++k) {
            // A = X X^T (symmetric: its transposed store is itself)
            if (launch_gemm_nt_bf16(x, np, x, np, mp, mp, np, 1.0f, 0.0f, nullptr, 0, nullptr, 0, wa, mp, stream, true, count, mn, mn,
                                    0, mm, mm) != hipSuccess)
                return ADAGC_ERR_HIP;
            // B = b A + c A A
            if (launch_gemm_nt_bf16(wa, mp, wa, mp, mp, mp, mp, ns_c, ns_b, wa, mp, nullptr, 0, wb, mp, stream, true, count, mm, mm, mm,
                                    mm, mm) != hipSuccess)
                return ADAGC_ERR_HIP;
            // X' = a X + B X, written as X' and as Y' = X'^T; (B X)[i][j] = sum_k B[i][k] Y[j][k].  After the last step
            // only the orientation the update reads is needed: X' for wide matrices, Y' for tall ones.
            const bool last = k + 1 == mh->ns_steps;
            uint16_t* out_x = (last && !any_wide) ? nullptr : x2;
            uint16_t* out_y = (last && !any_tall) ? nullptr : y2;
            if (launch_gemm_nt_bf16(wb, mp, y, mp, mp, np, mp, 1.0f, ns_a, y, mp, out_x, np, out_y, mp, stream, false, count, mm, mn, mn,
                                    mn, mn) != hipSuccess)
                return ADAGC_ERR_HIP;
            uint16_t* s = x; x = x2; x2 = s;
            s = y; y = y2; y2 = s;
        }
        for (int z = 0; z < count; ++z) {
            const int64_t i = bt.members[(size_t)z];
            const int64_t rows = ctx->shapes[(size_t)i].rows, cols = ctx->shapes[(size_t)i].cols;
            const bool flip = rows > cols;
            const double scale = std::sqrt(flip ? (double)rows / (double)cols : 1.0);
            const hipError_t g = launch_muon_apply(params[i], (flip ? y : x) + z * mn, flip ? mp : np, rows, cols, (double)h.lr,
                                                   (double)h.weight_decay, scale, copy ? ctx->param_copies[(size_t)i] : nullptr, stream);
            if (g != hipSuccess) return ADAGC_ERR_HIP;
        }
    }
    if (prof) {
        if (hipEventRecord(ev[3], stream) != hipSuccess) return ADAGC_ERR_HIP;
        ctx->prof_steps++;
    }
    return ADAGC_OK;
}

namespace {

// Wait for the copies; after adagc_step_graph also fetch the status word the device wrote for that step.
int finish_readback(adagc_ctx* ctx, hipStream_t stream)
{
    int32_t status = 0;
    if (ctx->device_scalars_used &&
        hipMemcpyAsync(&status, &ctx->tables.scalars->status, sizeof(status), hipMemcpyDeviceToHost, stream) != hipSuccess)
        return ADAGC_ERR_HIP;
    if (hipStreamSynchronize(stream) != hipSuccess) return ADAGC_ERR_HIP;
    return status == 0 ? ADAGC_OK : ADAGC_ERR_INVALID_ARG;
}

}  // namespace

extern "C" int adagc_get_norms(adagc_ctx* ctx, float* host_norms, float* host_coefs, uint8_t* host_clipped,
                               int64_t n_tensors, void* stream_v)
{
    if (!ctx || n_tensors != ctx->n_tensors) return ADAGC_ERR_INVALID_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return ADAGC_ERR_HIP;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    const size_t n = (size_t)n_tensors;
    const DeviceTables& t = ctx->tables;
    if (host_norms && hipMemcpyAsync(host_norms, t.norm, n * sizeof(float), hipMemcpyDeviceToHost, stream) != hipSuccess)
        return ADAGC_ERR_HIP;
    if (host_coefs && hipMemcpyAsync(host_coefs, t.coef, n * sizeof(float), hipMemcpyDeviceToHost, stream) != hipSuccess)
        return ADAGC_ERR_HIP;
    if (host_clipped && hipMemcpyAsync(host_clipped, t.flag, n, hipMemcpyDeviceToHost, stream) != hipSuccess)
        return ADAGC_ERR_HIP;
    return finish_readback(ctx, stream);
}

extern "C" int adagc_get_state_norms(adagc_ctx* ctx, float* host_m_norms, float* host_v_norms,
                                     float* host_update_norms, int64_t n_tensors, void* stream_v)
{
    if (!ctx || n_tensors != ctx->n_tensors) return ADAGC_ERR_INVALID_ARG;
    if (!ctx->cfg.telemetry) return ADAGC_ERR_STATE;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return ADAGC_ERR_HIP;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    const size_t n = (size_t)n_tensors;
    float* out[3] = {host_m_norms, host_v_norms, host_update_norms};
    for (int q = 0; q < 3; ++q)
        if (out[q] && hipMemcpyAsync(out[q], ctx->tables.tele_norm + q * n, n * sizeof(float),
                                     hipMemcpyDeviceToHost, stream) != hipSuccess)
            return ADAGC_ERR_HIP;
    return finish_readback(ctx, stream);
}

extern "C" int adagc_get_segment_table(adagc_ctx* ctx, int64_t* chunk_begin, uint32_t* chunk_tensor,
                                       uint32_t* chunk_index)
{
    if (!ctx) return ADAGC_ERR_INVALID_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return ADAGC_ERR_HIP;
    if (chunk_begin) std::memcpy(chunk_begin, ctx->chunk_begin.data(), ((size_t)ctx->n_tensors + 1) * sizeof(int64_t));
    if (chunk_tensor || chunk_index) {
        std::vector<ChunkRef> refs;
        try {
            refs.resize((size_t)ctx->n_chunks);
        } catch (const std::bad_alloc&) { return ADAGC_ERR_OOM; }
        if (hipMemcpy(refs.data(), ctx->tables.chunks, refs.size() * sizeof(ChunkRef), hipMemcpyDeviceToHost) !=
            hipSuccess)
            return ADAGC_ERR_HIP;
        for (size_t k = 0; k < refs.size(); ++k) {
            if (chunk_tensor) chunk_tensor[k] = refs[k].tensor;
            if (chunk_index) chunk_index[k] = refs[k].index;
        }
    }
    return ADAGC_OK;
}

extern "C" int adagc_profile_begin(adagc_ctx* ctx, int32_t max_steps)
{
    if (!ctx || max_steps <= 0 || max_steps > 4096) return ADAGC_ERR_INVALID_ARG;
    if (!ctx->prof_events.empty()) return ADAGC_ERR_STATE;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return ADAGC_ERR_HIP;
    try {
        ctx->prof_events.reserve((size_t)max_steps * 4);
    } catch (const std::bad_alloc&) { return ADAGC_ERR_OOM; }
    for (int32_t k = 0; k < max_steps * 4; ++k) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) {
            for (hipEvent_t x : ctx->prof_events) (void)hipEventDestroy(x);
            ctx->prof_events.clear();
            return ADAGC_ERR_HIP;
        }
        ctx->prof_events.push_back(e);
    }
    ctx->prof_capacity = max_steps;
    ctx->prof_steps = 0;
    return ADAGC_OK;
}

extern "C" int adagc_profile_end(adagc_ctx* ctx, float* ms, int32_t* n_steps)
{
    if (!ctx || !ms || !n_steps) return ADAGC_ERR_INVALID_ARG;
    if (ctx->prof_events.empty()) return ADAGC_ERR_STATE;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return ADAGC_ERR_HIP;
    int rc = ADAGC_OK;
    const int32_t n = ctx->prof_steps;
    if (n > 0 && hipEventSynchronize(ctx->prof_events[(size_t)n * 4 - 1]) != hipSuccess) rc = ADAGC_ERR_HIP;
    for (int32_t s = 0; s < n && rc == ADAGC_OK; ++s)
        for (int k = 0; k < 3; ++k)
            if (hipEventElapsedTime(&ms[s * 3 + k], ctx->prof_events[(size_t)s * 4 + k],
                                    ctx->prof_events[(size_t)s * 4 + k + 1]) != hipSuccess)
                rc = ADAGC_ERR_HIP;
    for (hipEvent_t e : ctx->prof_events) (void)hipEventDestroy(e);
    ctx->prof_events.clear();
    ctx->prof_capacity = 0;
    ctx->prof_steps = 0;
    *n_steps = n;
    return rc;
}
