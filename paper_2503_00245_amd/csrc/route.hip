// Fused router: logits, softmax (Sec. 2.3 Eq. 2, temperature 1), top-k (Eq. 3) with
// lowest-index tie-break and gates renormalised over the k chosen.
//
// One workgroup per token.  Wave w accumulates the logits of experts w, w+W, ... with
// 16-byte loads striding the token row, lane-partial sums are folded with a 64-lane
// butterfly, and wave 0 then holds one logit per lane and runs k rounds of a
// (value, index) arg-max butterfly.  Everything stays in registers / LDS; only the k
// indices, k gates and (optionally) the E probabilities are written.
#include "common.h"

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

    for (int e = wave; e < E; e += kRouteWaves) {
        const float* we = rw + (size_t)e * d;
        float acc = 0.f;
        for (int i = lane * VEC; i < d; i += kWave * VEC) {
            typename S::vec_t xv = *reinterpret_cast<const typename S::vec_t*>(xt + i);
#pragma unroll
            for (int q = 0; q < VEC; q += 4) {
                f32x4 wv = *reinterpret_cast<const f32x4*>(we + i + q);
                acc = fmaf(S::get(xv, q + 0), wv[0], acc);
                acc = fmaf(S::get(xv, q + 1), wv[1], acc);
                acc = fmaf(S::get(xv, q + 2), wv[2], acc);
                acc = fmaf(S::get(xv, q + 3), wv[3], acc);
            }
        }
        acc = wave_sum(acc);
        if (lane == 0) s_logit[e] = acc + (rb ? rb[e] : 0.f);
    }
    __syncthreads();
    if (wave != 0) return;

    // lane e owns expert e; lanes >= E carry -inf and an index that never wins a tie
    const bool valid = lane < E;
    const float logit = valid ? s_logit[lane] : -INFINITY;
    float cand = logit;  // -inf once taken
    float vmax = 0.f;
    float p_sel_sum = 0.f;
    float my_p = 0.f;
    int my_slot = -1;  // selection round in which this lane's expert was taken
    for (int j = 0; j < k; ++j) {
        float bv = cand;
        int bi = lane;
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) {
            float ov = __shfl_xor(bv, m, kWave);
            int oi = __shfl_xor(bi, m, kWave);
            if (ov > bv || (ov == bv && oi < bi)) {
                bv = ov;
                bi = oi;
            }
        }
        if (j == 0) vmax = bv;  // the first pick is the row maximum
        if (lane == bi) {
            cand = -INFINITY;
            my_slot = j;
        }
    }
    my_p = valid ? __expf(logit - vmax) : 0.f;
    const float den = wave_sum(my_p);
    p_sel_sum = wave_sum(my_slot >= 0 ? my_p : 0.f);
    if (probs && valid) probs[(size_t)t * E + lane] = my_p / den;
    if (my_slot >= 0) {
        topk_idx[(size_t)t * k + my_slot] = lane;
        // (p/den) / (sum_sel p/den) with the common 1/den cancelled
        topk_gate[(size_t)t * k + my_slot] = my_p / p_sel_sum;
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
