// Fused router: logits, softmax (Sec. 2.3 Eq. 2, temperature 1), top-k (Eq. 3) with
// lowest-index tie-break and gates renormalised over the k chosen.
//
// One workgroup per kRouteTok tokens.  Wave w accumulates the logits of experts w, w+W, ...
// for all of the group's tokens at once (each router row chunk is read once and reused),
// with 16-byte loads striding the rows and 64-lane butterflies; then wave w takes tokens
// w, w+W, ..., holds one logit per lane and runs k rounds of a (value, index) arg-max
// butterfly.  Everything stays in registers / LDS; only the k indices, k gates and
// (optionally) the E probabilities are written.
#include "router.h"

namespace moe {

constexpr int kRouteWaves = 8;
constexpr int kRouteTok = 2;  // tokens per workgroup

template <typename T>
__global__ __launch_bounds__(kRouteWaves* kWave) void route_kernel(
    const T* __restrict__ x, const float* __restrict__ rw, const float* __restrict__ rb,
    int32_t* __restrict__ topk_idx, float* __restrict__ topk_gate, float* __restrict__ probs,
    int T_, int d, int E, int k) {
    typedef Store<T> S;
    constexpr int VEC = S::VEC;
    __shared__ float s_logit[kRouteTok][kMaxExperts];

    const int t0 = blockIdx.x * kRouteTok;
    const int ntok = min(kRouteTok, T_ - t0);
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;

    auto load_x = [&](int t, int i, float* out) {
        const typename S::vec_t xv =
            *reinterpret_cast<const typename S::vec_t*>(x + (size_t)(t0 + t) * d + i);
#pragma unroll
        for (int q = 0; q < VEC; ++q) out[q] = S::get(xv, q);
    };
    for (int e = wave; e < E; e += kRouteWaves) {
        float acc[kRouteTok];
        router_logits<VEC, kRouteTok>(load_x, rw + (size_t)e * d, d, lane, ntok, acc);
        if (lane == 0) {
            const float b = rb ? rb[e] : 0.f;
#pragma unroll
            for (int t = 0; t < kRouteTok; ++t) s_logit[t][e] = acc[t] + b;
        }
    }
    __syncthreads();

    for (int tt = wave; tt < ntok; tt += kRouteWaves) {
        const int t = t0 + tt;
        const RouterPick r = router_select(lane, E, k, lane < E ? s_logit[tt][lane] : 0.f);
        if (probs && lane < E) probs[(size_t)t * E + lane] = r.p / r.den;
        if (r.slot >= 0) {
            topk_idx[(size_t)t * k + r.slot] = lane;
            // (p/den) / (sum_sel p/den) with the common 1/den cancelled
            topk_gate[(size_t)t * k + r.slot] = r.p / r.sel_sum;
        }
    }
}

int launch_route(const moe_shape& s, const void* x, const float* rw, const float* rb,
                 int32_t* topk_idx, float* topk_gate, float* probs, hipStream_t st) {
    if (s.n_tokens == 0) return MOE_OK;
    dim3 grid((s.n_tokens + kRouteTok - 1) / kRouteTok), block(kRouteWaves * kWave);
    if (s.act_dtype == MOE_F32)
        hipLaunchKernelGGL(route_kernel<float>, grid, block, 0, st, (const float*)x, rw, rb,
                           topk_idx, topk_gate, probs, s.n_tokens, s.d_model, s.n_experts, s.top_k);
    else
        hipLaunchKernelGGL(route_kernel<bf16_t>, grid, block, 0, st, (const bf16_t*)x, rw, rb,
                           topk_idx, topk_gate, probs, s.n_tokens, s.d_model, s.n_experts, s.top_k);
    return launch_status();
}

}  // namespace moe
