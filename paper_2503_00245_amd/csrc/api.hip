// extern "C" entry points of moe.h: argument checks on the host, workspace carving, and
// the order in which the stage kernels are enqueued.  No kernel lives here.
#include "common.h"

namespace moe {

bool decode_supported(const moe_shape& s);  // expert_gemv.hip

int validate_shape(const moe_shape* s) {
    if (!s) return MOE_ERR_INVALID;
    if (s->n_tokens < 0 || s->top_k < 1 || s->n_experts < 1 || s->top_k > s->n_experts ||
        s->d_model < 1 || s->d_ff < 1 || s->rank < 0)
        return MOE_ERR_INVALID;
    if ((s->flags & MOE_FLAG_SHARED_BASE) && s->rank == 0) return MOE_ERR_INVALID;
    if (s->flags & ~(MOE_FLAG_SHARED_BASE | MOE_FLAG_RESIDUAL)) return MOE_ERR_INVALID;
    if (s->act_dtype != MOE_F32 && s->act_dtype != MOE_BF16) return MOE_ERR_UNSUPPORTED;
    if (s->n_experts > kMaxExperts) return MOE_ERR_UNSUPPORTED;
    if (s->d_model % 8 || s->d_ff % 8 || s->rank % 8) return MOE_ERR_UNSUPPORTED;
    if ((long long)s->n_tokens * s->top_k >= (1ll << 24)) return MOE_ERR_UNSUPPORTED;
    return MOE_OK;
}

static int validate_weights(const moe_shape& s, const moe_weights* w, bool need_router) {
    if (!w) return MOE_ERR_INVALID;
    if (need_router && (!w->router_w || !aligned16(w->router_w))) return MOE_ERR_INVALID;
    const bool base = s.rank == 0 || (s.flags & MOE_FLAG_SHARED_BASE);
    const void* dense[3] = {w->w_gate, w->w_up, w->w_down};
    const void* fac[6] = {w->rg, w->ru, w->rd, w->lg, w->lu, w->ld};
    for (const void* p : dense) {
        if (base && (!p || !aligned16(p))) return MOE_ERR_INVALID;
        if (!base && p) return MOE_ERR_INVALID;  // a dense block without the shared-base flag
    }
    if (s.rank > 0)
        for (const void* p : fac)
            if (!p || !aligned16(p)) return MOE_ERR_INVALID;
    return MOE_OK;
}

// Workspace carving; every region starts 256-byte aligned.
struct Workspace {
    size_t topk_idx, topk_gate, offsets, perm, inv_perm, sort_scratch, y_perm, y_base, ffn_scratch,
        decode_scratch, stack_tmp, total;
};

static Workspace carve(const moe_shape& s) {
    Workspace ws{};
    const size_t P = (size_t)s.n_tokens * s.top_k;
    size_t cur = 0;
    auto take = [&](size_t bytes) {
        const size_t at = cur;
        cur += round_up(bytes ? bytes : 1, 256);
        return at;
    };
    ws.topk_idx = take(P * sizeof(int32_t));
    ws.topk_gate = take(P * sizeof(float));
    ws.offsets = take((size_t)(s.n_experts + 1) * sizeof(int32_t));
    ws.perm = take(P * sizeof(int32_t));
    ws.inv_perm = take(P * sizeof(int32_t));
    ws.sort_scratch = take(permute_scratch_bytes((int)P, s.n_experts));
    ws.y_perm = take(P * s.d_model * elt_size(s.act_dtype) * down_parts_capacity(s));  // room for partial outputs
    ws.y_base = take(token_base_supported(s) ? (size_t)s.n_tokens * s.d_model * elt_size(s.act_dtype) : 0);
    ws.ffn_scratch = take(ffn_scratch_bytes(s));
    ws.decode_scratch = take(decode_scratch_bytes(s));
    ws.stack_tmp = take((size_t)s.n_tokens * s.d_model * elt_size(s.act_dtype));
    ws.total = cur;
    return ws;
}

static int forward_impl(const moe_shape& s, const moe_weights& w, const void* x, void* y,
                        int32_t* topk_idx, float* topk_gate, char* wsp, hipStream_t st,
                        StageTimer* timer = nullptr) {
    const Workspace ws = carve(s);
    int32_t* idx = topk_idx ? topk_idx : reinterpret_cast<int32_t*>(wsp + ws.topk_idx);
    float* gate = topk_gate ? topk_gate : reinterpret_cast<float*>(wsp + ws.topk_gate);
    int rc = launch_route(s, x, w.router_w, w.router_b, idx, gate, nullptr, st);
    if (rc != MOE_OK) return rc;
    stage_mark(timer, "route");
    if (decode_supported(s))
        return launch_decode_ffn(s, w, x, idx, gate, y, wsp + ws.decode_scratch, st, timer);
    const int P = s.n_tokens * s.top_k;
    int32_t* offsets = reinterpret_cast<int32_t*>(wsp + ws.offsets);
    int32_t* perm = reinterpret_cast<int32_t*>(wsp + ws.perm);
    int32_t* inv_perm = reinterpret_cast<int32_t*>(wsp + ws.inv_perm);
    rc = launch_permute(P, s.n_experts, idx, offsets, perm, inv_perm, wsp + ws.sort_scratch, st);
    if (rc != MOE_OK) return rc;
    stage_mark(timer, "permute");
    // the gather of token rows into expert order is fused into the first GEMM's A loads
    const void* residual = (s.flags & MOE_FLAG_RESIDUAL) ? x : nullptr;
    if (token_base_supported(s)) {  // shared base: its products run once per token
        rc = launch_expert_ffn_token_base(s, w, x, perm, inv_perm, gate, offsets, wsp + ws.y_perm,
                                          wsp + ws.y_base, wsp + ws.ffn_scratch, st, timer);
        if (rc != MOE_OK) return rc;
        rc = launch_combine(s, wsp + ws.y_perm, inv_perm, gate, residual, y, st, wsp + ws.y_base);
        stage_mark(timer, "combine");
        return rc;
    }
    int y_parts = down_parts_capacity(s);  // the down projection may leave partial outputs for the combine to add
    rc = launch_expert_ffn(s, w, x, perm, s.top_k, offsets, wsp + ws.y_perm, wsp + ws.ffn_scratch, st,
                           timer, &y_parts);
    if (rc != MOE_OK) return rc;
    rc = launch_combine(s, wsp + ws.y_perm, inv_perm, gate, residual, y, st, nullptr, y_parts);
    stage_mark(timer, "combine");
    return rc;
}

// ---- scratch of the allocation-free entry point ------------------------------------------------
// A file-scope device array stands in for the caller's workspace.  Every GPU the library runs on
// holds its own copy at its own address until the process ends; in host code the array's name is
// only a handle for the runtime, so the device address is looked up once per device (with that
// device current) and kept, and only that pointer is ever handed to kernels.
static __device__ __align__(256) unsigned char scratch[MOE_STATIC_WORKSPACE_BYTES];
constexpr int kMaxDevices = 64;
static std::atomic<void*> scratch_ptr[kMaxDevices];

static int static_scratch(char** out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return MOE_ERR_LAUNCH;
    if (dev < 0 || dev >= kMaxDevices) return MOE_ERR_UNSUPPORTED;
    void* p = scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {  // first call on this device (a race merely repeats the lookup)
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return MOE_ERR_LAUNCH;
        scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = static_cast<char*>(p);
    return MOE_OK;
}

}  // namespace moe

using namespace moe;

extern "C" {

size_t moe_workspace_bytes(const moe_shape* shape) {
    if (validate_shape(shape) != MOE_OK) return 0;
    return carve(*shape).total;
}

const char* moe_status_string(int status) {
    switch (status) {
        case MOE_OK: return "ok";
        case MOE_ERR_INVALID: return "invalid argument";
        case MOE_ERR_UNSUPPORTED: return "unsupported shape or dtype";
        case MOE_ERR_WORKSPACE: return "workspace too small";
        case MOE_ERR_LAUNCH: return "kernel launch failed";
        default: return "unknown status";
    }
}

int moe_route(const moe_shape* shape, const void* x, const float* router_w, const float* router_b,
              int32_t* topk_idx, float* topk_gate, float* probs, void* stream) {
    int rc = validate_shape(shape);
    if (rc != MOE_OK) return rc;
    if (shape->n_tokens == 0) return MOE_OK;
    if (!x || !router_w || !topk_idx || !topk_gate) return MOE_ERR_INVALID;
    if (!aligned16(x) || !aligned16(router_w)) return MOE_ERR_INVALID;
    return launch_route(*shape, x, router_w, router_b, topk_idx, topk_gate, probs, as_stream(stream));
}

int moe_permute(const moe_shape* shape, const int32_t* topk_idx, int32_t* expert_offsets,
                int32_t* perm, int32_t* inv_perm, const void* x, void* x_perm, void* workspace,
                size_t workspace_bytes, void* stream) {
    int rc = validate_shape(shape);
    if (rc != MOE_OK) return rc;
    if (!expert_offsets) return MOE_ERR_INVALID;
    const int P = shape->n_tokens * shape->top_k;
    if (P > 0 && (!topk_idx || !perm || !inv_perm)) return MOE_ERR_INVALID;
    if ((x == nullptr) != (x_perm == nullptr)) return MOE_ERR_INVALID;
    if (x && (!aligned16(x) || !aligned16(x_perm))) return MOE_ERR_INVALID;
    const size_t need = permute_scratch_bytes(P, shape->n_experts);
    if (need > 0 && (!workspace || workspace_bytes < need)) return MOE_ERR_WORKSPACE;
    hipStream_t st = as_stream(stream);
    rc = launch_permute(P, shape->n_experts, topk_idx, expert_offsets, perm, inv_perm, workspace, st);
    if (rc != MOE_OK || !x) return rc;
    return launch_gather_rows(*shape, perm, x, x_perm, st);
}

int moe_expert_ffn(const moe_shape* shape, const moe_weights* weights, const void* x_perm,
                   const int32_t* expert_offsets, void* y_perm, void* workspace,
                   size_t workspace_bytes, void* stream) {
    int rc = validate_shape(shape);
    if (rc != MOE_OK) return rc;
    if ((rc = validate_weights(*shape, weights, false)) != MOE_OK) return rc;
    if (shape->n_tokens == 0) return MOE_OK;
    if (!x_perm || !expert_offsets || !y_perm || !aligned16(x_perm) || !aligned16(y_perm))
        return MOE_ERR_INVALID;
    if (!workspace || !aligned16(workspace)) return MOE_ERR_WORKSPACE;
    if (workspace_bytes < ffn_scratch_bytes(*shape)) return MOE_ERR_WORKSPACE;
    return launch_expert_ffn(*shape, *weights, x_perm, nullptr, 1, expert_offsets, y_perm, workspace,
                             as_stream(stream));
}

int moe_combine(const moe_shape* shape, const void* y_perm, const int32_t* inv_perm,
                const float* topk_gate, const void* residual, void* y, void* stream) {
    int rc = validate_shape(shape);
    if (rc != MOE_OK) return rc;
    if (shape->n_tokens == 0) return MOE_OK;
    if (!y_perm || !inv_perm || !topk_gate || !y) return MOE_ERR_INVALID;
    if (!aligned16(y_perm) || !aligned16(y) || (residual && !aligned16(residual)))
        return MOE_ERR_INVALID;
    return launch_combine(*shape, y_perm, inv_perm, topk_gate, residual, y, as_stream(stream));
}

int moe_forward(const moe_shape* shape, const moe_weights* weights, const void* x, void* y,
                int32_t* topk_idx, float* topk_gate, void* workspace, size_t workspace_bytes,
                void* stream) {
    int rc = validate_shape(shape);
    if (rc != MOE_OK) return rc;
    if ((rc = validate_weights(*shape, weights, true)) != MOE_OK) return rc;
    if (shape->n_tokens == 0) return MOE_OK;
    if (!x || !y || x == y || !aligned16(x) || !aligned16(y)) return MOE_ERR_INVALID;
    if (!workspace || !aligned16(workspace) || workspace_bytes < carve(*shape).total)
        return MOE_ERR_WORKSPACE;
    return forward_impl(*shape, *weights, x, y, topk_idx, topk_gate, static_cast<char*>(workspace),
                        as_stream(stream));
}

int moe_forward_static(const moe_shape* shape, const moe_weights* weights, const void* x, void* y,
                       int32_t* topk_idx, float* topk_gate, void* stream) {
    int rc = validate_shape(shape);
    if (rc != MOE_OK) return rc;
    if ((rc = validate_weights(*shape, weights, true)) != MOE_OK) return rc;
    if (shape->n_tokens == 0) return MOE_OK;
    if (!x || !y || x == y || !aligned16(x) || !aligned16(y)) return MOE_ERR_INVALID;
    if (carve(*shape).total > (size_t)MOE_STATIC_WORKSPACE_BYTES) return MOE_ERR_WORKSPACE;
    char* wsp = nullptr;
    if ((rc = static_scratch(&wsp)) != MOE_OK) return rc;
    // nothing in the workspace has to start at zero: every stage writes what the next one reads
    return forward_impl(*shape, *weights, x, y, topk_idx, topk_gate, wsp, as_stream(stream));
}

int moe_forward_timed(const moe_shape* shape, const moe_weights* weights, const void* x, void* y,
                      void* workspace, size_t workspace_bytes, void* stream, float* stage_ms,
                      const char** stage_names, int32_t* n_stages) {
    if (!stage_ms || !n_stages) return MOE_ERR_INVALID;
    *n_stages = 0;
    int rc = validate_shape(shape);
    if (rc != MOE_OK) return rc;
    if ((rc = validate_weights(*shape, weights, true)) != MOE_OK) return rc;
    if (shape->n_tokens == 0) return MOE_OK;
    if (!x || !y || x == y || !aligned16(x) || !aligned16(y)) return MOE_ERR_INVALID;
    if (!workspace || !aligned16(workspace) || workspace_bytes < carve(*shape).total)
        return MOE_ERR_WORKSPACE;
    StageTimer timer{};
    timer.st = as_stream(stream);
    for (auto& e : timer.ev)
        if (hipEventCreate(&e) != hipSuccess) return MOE_ERR_LAUNCH;
    (void)hipEventRecord(timer.ev[0], timer.st);
    rc = forward_impl(*shape, *weights, x, y, nullptr, nullptr, static_cast<char*>(workspace),
                      timer.st, &timer);
    if (hipStreamSynchronize(timer.st) != hipSuccess && rc == MOE_OK) rc = MOE_ERR_LAUNCH;
    if (rc == MOE_OK) {
        for (int i = 0; i < timer.n; ++i) {
            if (hipEventElapsedTime(&stage_ms[i], timer.ev[i], timer.ev[i + 1]) != hipSuccess)
                rc = MOE_ERR_LAUNCH;
            if (stage_names) stage_names[i] = timer.name[i];
        }
        *n_stages = timer.n;
    }
    for (auto& e : timer.ev) (void)hipEventDestroy(e);
    return rc;
}

int moe_stack_forward(const moe_shape* shape, const moe_weights* layers, int32_t n_layers,
                      const void* x, void* y, int32_t* topk_trace, void* workspace,
                      size_t workspace_bytes, void* stream) {
    int rc = validate_shape(shape);
    if (rc != MOE_OK) return rc;
    if (n_layers < 1 || !layers) return MOE_ERR_INVALID;
    for (int l = 0; l < n_layers; ++l)
        if ((rc = validate_weights(*shape, &layers[l], true)) != MOE_OK) return rc;
    if (shape->n_tokens == 0) return MOE_OK;
    if (!x || !y || x == y || !aligned16(x) || !aligned16(y)) return MOE_ERR_INVALID;
    moe_shape s = *shape;
    s.flags |= MOE_FLAG_RESIDUAL;
    const Workspace ws = carve(s);
    if (!workspace || !aligned16(workspace) || workspace_bytes < ws.total) return MOE_ERR_WORKSPACE;
    char* wsp = static_cast<char*>(workspace);
    void* tmp = wsp + ws.stack_tmp;
    const size_t Pk = (size_t)s.n_tokens * s.top_k;
    const void* cur = x;
    for (int l = 0; l < n_layers; ++l) {
        // ping-pong so that the last layer writes y and no layer reads what it writes
        void* out = ((n_layers - l) & 1) ? y : tmp;
        rc = forward_impl(s, layers[l], cur, out, topk_trace ? topk_trace + (size_t)l * Pk : nullptr,
                          nullptr, wsp, as_stream(stream));
        if (rc != MOE_OK) return rc;
        cur = out;
    }
    return MOE_OK;
}

}  // extern "C"
