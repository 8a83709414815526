// Gate-weighted combine back to token order:
//   y[t,:] = sum_{j<k} gate[t,j] * y_perm[inv_perm[t*k+j], :]  (+ residual[t,:]) (+ addend[t,:])
// y_perm may come as several partial outputs (a down projection whose k-steps were cut into parts):
// then y_perm[s,:] stands for the sum of the parts' rows s, added here in part order.
// (Sec. 1 / Sec. 2.1: the gate sets each selected expert's contribution.)  One workgroup
// per token, 16-byte loads, fp32 accumulation in ascending j, one rounding at the store.
#include "common.h"

namespace moe {

template <typename T>
__global__ __launch_bounds__(256) void combine_kernel(const T* __restrict__ y_perm,
                                                      const int32_t* __restrict__ inv_perm,
                                                      const float* __restrict__ gate,
                                                      const T* __restrict__ residual,
                                                      const T* __restrict__ addend,
                                                      T* __restrict__ y, int d, int k, int P, int parts) {
    typedef Store<T> S;
    constexpr int VEC = S::VEC;
    typedef typename S::vec_t vec_t;
    const int t = blockIdx.x;
    for (int i = threadIdx.x * VEC; i < d; i += blockDim.x * VEC) {
        float acc[VEC];
#pragma unroll
        for (int q = 0; q < VEC; ++q) acc[q] = 0.f;
        for (int j = 0; j < k; ++j) {
            const int s = min(max(inv_perm[(size_t)t * k + j], 0), P - 1);
            const float g = gate[(size_t)t * k + j];
            for (int part = 0; part < parts; ++part) {
                const vec_t v = *reinterpret_cast<const vec_t*>(y_perm + ((size_t)part * P + s) * d + i);
#pragma unroll
                for (int q = 0; q < VEC; ++q) acc[q] = fmaf(g, S::get(v, q), acc[q]);
            }
        }
        if (residual) {
            const vec_t r = *reinterpret_cast<const vec_t*>(residual + (size_t)t * d + i);
#pragma unroll
            for (int q = 0; q < VEC; ++q) acc[q] += S::get(r, q);
        }
        if (addend) {
            const vec_t r = *reinterpret_cast<const vec_t*>(addend + (size_t)t * d + i);
#pragma unroll
            for (int q = 0; q < VEC; ++q) acc[q] += S::get(r, q);
        }
        vec_t o;
#pragma unroll
        for (int q = 0; q < VEC; ++q) o[q] = S::from_f32(acc[q]);
        *reinterpret_cast<vec_t*>(y + (size_t)t * d + i) = o;
    }
}

int launch_combine(const moe_shape& s, const void* y_perm, const int32_t* inv_perm,
                   const float* topk_gate, const void* residual, void* y, hipStream_t st,
                   const void* addend, int y_parts) {
    if (s.n_tokens == 0) return MOE_OK;
    const int P = s.n_tokens * s.top_k;
    dim3 grid(s.n_tokens), block(256);
    if (s.act_dtype == MOE_F32)
        hipLaunchKernelGGL(combine_kernel<float>, grid, block, 0, st, (const float*)y_perm, inv_perm,
                           topk_gate, (const float*)residual, (const float*)addend, (float*)y, s.d_model,
                           s.top_k, P, y_parts);
    else
        hipLaunchKernelGGL(combine_kernel<bf16_t>, grid, block, 0, st, (const bf16_t*)y_perm,
                           inv_perm, topk_gate, (const bf16_t*)residual, (const bf16_t*)addend, (bf16_t*)y,
                           s.d_model, s.top_k, P, y_parts);
    return launch_status();
}

}  // namespace moe
