// Fused router: logits, softmax (Sec. 2.3 Eq. 2, temperature 1), top-k (Eq. 3) with
// lowest-index tie-break and gates renormalised over the k chosen.
//
// One workgroup per token.  Wave w accumulates the logits of experts w, w+W, ... with
// 16-byte loads striding the token row, lane-partial sums are folded with a 64-lane
// butterfly, and wave 0 then holds one logit per lane and runs k rounds of a
// (value, index) arg-max butterfly.  Everything stays in registers / LDS; only the k
// indices, k gates and (optionally) the E probabilities are written.
#include "router.h"

namespace moe {

constexpr int kRouteWaves = 8;

template <typename T>
__global__ __launch_bounds__(kRouteWaves* kWave) void route_kernel(
    const T* __restrict__ x, const float* __restrict__ rw, const float* __restrict__ rb,
    int32_t* __restrict__ topk_idx, float* __restrict__ topk_gate, float* __restrict__ probs,
    int d, int E, int k) {
    typedef Store<T> S;
    constexpr int VEC = S::VEC;
    __shared__ float s_logit[kMaxExperts];

    const int t = blockIdx.x;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const T* xt = x + (size_t)t * d;

    auto load_x = [&](int i, float* out) {
        const typename S::vec_t xv = *reinterpret_cast<const typename S::vec_t*>(xt + i);
#pragma unroll
        for (int q = 0; q < VEC; ++q) out[q] = S::get(xv, q);
    };
    for (int e = wave; e < E; e += kRouteWaves) {
        const float acc = router_logit<VEC>(load_x, rw + (size_t)e * d, d, lane);
        if (lane == 0) s_logit[e] = acc + (rb ? rb[e] : 0.f);
    }
    __syncthreads();
    if (wave != 0) return;

    const RouterPick r = router_select(lane, E, k, lane < E ? s_logit[lane] : 0.f);
    if (probs && lane < E) probs[(size_t)t * E + lane] = r.p / r.den;
    if (r.slot >= 0) {
        topk_idx[(size_t)t * k + r.slot] = lane;
        // (p/den) / (sum_sel p/den) with the common 1/den cancelled
        topk_gate[(size_t)t * k + r.slot] = r.p / r.sel_sum;
    }
}

int launch_route(const moe_shape& s, const void* x, const float* rw, const float* rb,
                 int32_t* topk_idx, float* topk_gate, float* probs, hipStream_t st) {
    if (s.n_tokens == 0) return MOE_OK;
    dim3 grid(s.n_tokens), block(kRouteWaves * kWave);
    if (s.act_dtype == MOE_F32)
        hipLaunchKernelGGL(route_kernel<float>, grid, block, 0, st, (const float*)x, rw, rb,
                           topk_idx, topk_gate, probs, s.d_model, s.n_experts, s.top_k);
    else
        hipLaunchKernelGGL(route_kernel<bf16_t>, grid, block, 0, st, (const bf16_t*)x, rw, rb,
                           topk_idx, topk_gate, probs, s.d_model, s.n_experts, s.top_k);
    return launch_status();
}

}  // namespace moe
