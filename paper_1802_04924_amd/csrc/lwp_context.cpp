// Context life cycle, its buffers, launch timing (C ABI: lwp_create ... lwp_profile_read).
#include "lwp_context.h"

#include <new>

namespace lwp {

lwp_status fail(lwp_ctx* ctx, lwp_status s, const std::string& why) {
    if (ctx) ctx->err = why;
    return s;
}

lwp_status check_ctx(lwp_ctx* ctx) {
    if (!ctx) return LWP_E_INVAL;
    ctx->err.clear();
    hipError_t e = hipSetDevice(ctx->device);
    if (e != hipSuccess) return fail(ctx, LWP_E_HIP, std::string("hipSetDevice: ") + hipGetErrorString(e));
    return LWP_OK;
}

lwp_status ensure_workspace(lwp_ctx* ctx, size_t bytes) {
    if (bytes <= ctx->ws_bytes) return LWP_OK;
    LWP_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (ctx->ws) { LWP_HIP(ctx, hipFree(ctx->ws)); ctx->ws = nullptr; ctx->ws_bytes = 0; }
    void* p = nullptr;
    hipError_t e = hipMalloc(&p, bytes);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(ctx, LWP_E_NOMEM, "device workspace of " + std::to_string(bytes) + " bytes: " + hipGetErrorString(e));
    }
    ctx->ws = static_cast<char*>(p);
    ctx->ws_bytes = bytes;
    return LWP_OK;
}

lwp_status ensure_pinned(lwp_ctx* ctx, size_t bytes) {
    if (bytes <= ctx->pin_bytes) return LWP_OK;
    LWP_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (ctx->pin) { LWP_HIP(ctx, hipHostFree(ctx->pin)); ctx->pin = nullptr; ctx->pin_bytes = 0; }
    void* p = nullptr;
    bytes = align_up(bytes, 1 << 16);
    hipError_t e = hipHostMalloc(&p, bytes, hipHostMallocDefault);
    if (e != hipSuccess) { (void)hipGetLastError(); return fail(ctx, LWP_E_NOMEM, std::string("pinned host buffer: ") + hipGetErrorString(e)); }
    ctx->pin = static_cast<char*>(p);
    ctx->pin_bytes = bytes;
    return LWP_OK;
}

lwp_status ensure_split_buffers(lwp_ctx* ctx) {
    if (ctx->split) return LWP_OK;
    const size_t ints = (size_t)kSplitMaxWorkgroups * kSplitScratchIntsPerPart + kSplitMaxTiles;
    void* p = nullptr;
    hipError_t e = hipMalloc(&p, ints * sizeof(int32_t));
    if (e != hipSuccess) { (void)hipGetLastError(); return fail(ctx, LWP_E_NOMEM, std::string("split-tile scratch: ") + hipGetErrorString(e)); }
    ctx->split = static_cast<int32_t*>(p);
    // the counters start at zero and every launch leaves them at zero
    LWP_HIP(ctx, hipMemsetAsync(ctx->split + (size_t)kSplitMaxWorkgroups * kSplitScratchIntsPerPart, 0,
                                kSplitMaxTiles * sizeof(int32_t), ctx->stream));
    return LWP_OK;
}

lwp_status ensure_state(lwp_ctx* ctx) {
    if (ctx->dstate && ctx->hstate) return LWP_OK;
    if (!ctx->hstate) {
        void* h = nullptr;
        hipError_t e = hipHostMalloc(&h, 64, hipHostMallocDefault);
        if (e != hipSuccess) { (void)hipGetLastError(); return fail(ctx, LWP_E_NOMEM, std::string("pinned state word: ") + hipGetErrorString(e)); }
        ctx->hstate = static_cast<int32_t*>(h);
    }
    if (!ctx->dstate) {
        void* p = nullptr;
        hipError_t e = hipMalloc(&p, 256);
        if (e != hipSuccess) { (void)hipGetLastError(); return fail(ctx, LWP_E_NOMEM, std::string("device state words: ") + hipGetErrorString(e)); }
        ctx->dstate = static_cast<int32_t*>(p);
        LWP_HIP(ctx, hipMemsetAsync(p, 0, 256, ctx->stream));
    }
    return LWP_OK;
}

void set_split(lwp_ctx* ctx, NodeArgs& a, Split split) {
    const int kparts = split.kparts;
    a.kparts = kparts;
    a.n_whole = (int32_t)split.n_whole;
    a.scratch = kparts > 1 ? ctx->split : nullptr;
    a.counters = kparts > 1 ? ctx->split + (size_t)kSplitMaxWorkgroups * kSplitScratchIntsPerPart : nullptr;
}

ScopedTimer::ScopedTimer(lwp_ctx* c, int kind, int64_t work, bool keyed) : ctx(c) {
    if (!c->profiling) return;
    lwp_ctx::Timed t{nullptr, nullptr, kind, work, keyed};
    if (hipEventCreate(&t.a) != hipSuccess || hipEventCreate(&t.b) != hipSuccess) return;
    (void)hipEventRecord(t.a, c->stream);
    c->timed.push_back(t);
    idx = c->timed.size() - 1;
}
ScopedTimer::~ScopedTimer() { if (idx != (size_t)-1) (void)hipEventRecord(ctx->timed[idx].b, ctx->stream); }

lwp_status drain_profile(lwp_ctx* ctx) {
    LWP_HIP(ctx, hipStreamSynchronize(ctx->stream));
    for (auto& t : ctx->timed) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, t.a, t.b) == hipSuccess) {
            if (t.kind == 0) {
                ctx->prof.node_launches++; ctx->prof.node_cell_updates += t.work; ctx->prof.node_ms += ms;
                if (t.keyed) ctx->prof.keyed_launches++;
            } else {
                ctx->prof.edge_launches++; ctx->prof.edge_cells += t.work; ctx->prof.edge_ms += ms;
            }
        }
        (void)hipEventDestroy(t.a); (void)hipEventDestroy(t.b);
    }
    ctx->timed.clear();
    return LWP_OK;
}

}  // namespace lwp

using namespace lwp;

extern "C" {

const char* lwp_status_string(lwp_status s) {
    switch (s) {
        case LWP_OK: return "ok";
        case LWP_E_INVAL: return "invalid argument";
        case LWP_E_GRAPH: return "invalid graph";
        case LWP_E_NOT_REDUCIBLE: return "graph not reducible";
        case LWP_E_OVERFLOW: return "int32 overflow possible";
        case LWP_E_NOMEM: return "out of memory";
        case LWP_E_HIP: return "HIP error";
        case LWP_E_TOO_LARGE: return "size beyond the fixed capacity of an entry point that does not allocate";
    }
    return "unknown status";
}

lwp_status lwp_create(lwp_ctx** out, int device, void* hip_stream) {
    if (!out) return LWP_E_INVAL;
    *out = nullptr;
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || device < 0 || device >= n) return LWP_E_HIP;
    if (hipSetDevice(device) != hipSuccess) return LWP_E_HIP;
    lwp_ctx* c = new (std::nothrow) lwp_ctx();
    if (!c) return LWP_E_NOMEM;
    c->device = device;
    c->stream = static_cast<hipStream_t>(hip_stream);
    (void)prepare_noalloc_scratch(device);     // set-up for lwp_eliminate_node_noalloc; it retries if this failed
    (void)hipGetLastError();
    *out = c;
    return LWP_OK;
}

void lwp_destroy(lwp_ctx* ctx) {
    if (!ctx) return;
    (void)hipSetDevice(ctx->device);
    (void)hipStreamSynchronize(ctx->stream);
    for (auto& t : ctx->timed) { (void)hipEventDestroy(t.a); (void)hipEventDestroy(t.b); }
    if (ctx->ws) (void)hipFree(ctx->ws);
    if (ctx->pin) (void)hipHostFree(ctx->pin);
    if (ctx->split) (void)hipFree(ctx->split);
    if (ctx->dstate) (void)hipFree(ctx->dstate);
    if (ctx->hstate) (void)hipHostFree(ctx->hstate);
    delete ctx;
}

const char* lwp_last_error(const lwp_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }

lwp_status lwp_set_option(lwp_ctx* ctx, int32_t option, int32_t value) {
    if (lwp_status s = check_ctx(ctx)) return s;
    if (option == LWP_OPT_SINGLE_LAUNCH) ctx->single_launch = value != 0;
    else if (option == LWP_OPT_SMALL_PRODUCT_KERNEL) ctx->wave_kernel = value != 0;
    else return fail(ctx, LWP_E_INVAL, "unknown option");
    return LWP_OK;
}

lwp_status lwp_synchronize(lwp_ctx* ctx) {
    if (lwp_status s = check_ctx(ctx)) return s;
    if (!ctx->dstate || !ctx->hstate) {
        LWP_HIP(ctx, hipStreamSynchronize(ctx->stream));
        return LWP_OK;
    }
    // what the kernels of lwp_eliminate_node / _edge found since the last call: the word is copied
    // behind them on the stream into pinned memory, so one wait covers both
    int32_t* bits_p = ctx->hstate;
    LWP_HIP(ctx, hipMemcpyAsync(bits_p, ctx->dstate, sizeof(int32_t), hipMemcpyDeviceToHost, ctx->stream));
    LWP_HIP(ctx, hipStreamSynchronize(ctx->stream));
    const int32_t bits = *bits_p;
    if (!bits) return LWP_OK;
    LWP_HIP(ctx, hipMemsetAsync(ctx->dstate, 0, sizeof(int32_t), ctx->stream));
    LWP_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (bits & 2) return fail(ctx, LWP_E_INVAL, "an elimination met values outside the ranges its caller promised; its results are invalid");
    return fail(ctx, LWP_E_OVERFLOW, "a sum of an elimination enqueued since the last lwp_synchronize may leave int32; its results are invalid");
}

lwp_status lwp_measure_valu_rate(lwp_ctx* ctx, double* lane_ops_per_s, double* cell_updates_per_s) {
    if (lwp_status s = check_ctx(ctx)) return s;
    if (!lane_ops_per_s || !cell_updates_per_s) return fail(ctx, LWP_E_INVAL, "null output");
    if (lwp_status s = ensure_workspace(ctx, 4096)) return s;
    hipDeviceProp_t prop;
    LWP_HIP(ctx, hipGetDeviceProperties(&prop, ctx->device));
    const int blocks = prop.multiProcessorCount * 8;        // 8 wavefronts per SIMD
    const int iters = 4000;
    uint32_t* d_out = reinterpret_cast<uint32_t*>(ctx->ws);
    hipEvent_t a = nullptr, b = nullptr;
    LWP_HIP(ctx, hipEventCreate(&a));
    hipError_t e = hipEventCreate(&b);
    if (e != hipSuccess) { (void)hipEventDestroy(a); return fail(ctx, LWP_E_HIP, std::string("hipEventCreate: ") + hipGetErrorString(e)); }
    float best_ms = 0.f;
    hipError_t err = hipSuccess;
    for (int rep = 0; rep < 3 && err == hipSuccess; ++rep) {     // first pass warms up; keep the fastest
        err = hipEventRecord(a, ctx->stream);
        if (err == hipSuccess) err = launch_alu_probe(d_out, blocks, iters, ctx->stream);
        if (err == hipSuccess) err = hipEventRecord(b, ctx->stream);
        if (err == hipSuccess) err = hipEventSynchronize(b);
        float ms = 0.f;
        if (err == hipSuccess) err = hipEventElapsedTime(&ms, a, b);
        if (err == hipSuccess && rep > 0 && (best_ms == 0.f || ms < best_ms)) best_ms = ms;
    }
    (void)hipEventDestroy(a); (void)hipEventDestroy(b);
    if (err != hipSuccess) { (void)hipGetLastError(); return fail(ctx, LWP_E_HIP, std::string("VALU probe: ") + hipGetErrorString(err)); }
    const double threads = (double)blocks * kNodeThreads, sec = best_ms * 1e-3;
    *lane_ops_per_s = threads * iters * alu_probe_instr_per_iter() / sec;
    *cell_updates_per_s = threads * iters * alu_probe_updates_per_iter() / sec;
    return LWP_OK;
}

lwp_status lwp_profile_enable(lwp_ctx* ctx, int32_t on) {
    if (lwp_status s = check_ctx(ctx)) return s;
    ctx->profiling = on != 0;
    return LWP_OK;
}

lwp_status lwp_profile_reset(lwp_ctx* ctx) {
    if (lwp_status s = check_ctx(ctx)) return s;
    if (lwp_status s = drain_profile(ctx)) return s;
    ctx->prof = lwp_profile{};
    if (ctx->dstate) {
        LWP_HIP(ctx, hipMemsetAsync(ctx->dstate + 1, 0, (kStateInts - 1) * sizeof(int32_t), ctx->stream));
        LWP_HIP(ctx, hipStreamSynchronize(ctx->stream));
    }
    return LWP_OK;
}

lwp_status lwp_profile_read(lwp_ctx* ctx, lwp_profile* out) {
    if (lwp_status s = check_ctx(ctx)) return s;
    if (!out) return fail(ctx, LWP_E_INVAL, "null output");
    if (lwp_status s = drain_profile(ctx)) return s;
    *out = ctx->prof;
    if (ctx->dstate) {
        int32_t st[kStateInts] = {};
        LWP_HIP(ctx, hipMemcpyAsync(st, ctx->dstate, sizeof(st), hipMemcpyDeviceToHost, ctx->stream));
        LWP_HIP(ctx, hipStreamSynchronize(ctx->stream));
        out->products_keyed = st[1 + kModeKeyed];
        out->products_plain = st[1 + kModePlain];
        out->products_value = st[1 + kModeValue];
        out->products_keyed_row = st[1 + kModeKeyedRow];
    }
    return LWP_OK;
}

}  // extern "C"
