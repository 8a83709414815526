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
constexpr int kRouteTok = 2;       // tokens per workgroup
constexpr int kRouteTokLarge = 4;  // ... from kRouteLargeFrom tokens on
constexpr int kRouteLargeFrom = 1024;

#ifndef MOE_ROUTE_NB_LARGE
#define MOE_ROUTE_NB_LARGE 2
#endif
// NB: router-row chunks a wave requests at once (4 for small batches, where the kernel is a chain
// of memory round trips; fewer for large ones, where registers per wave decide how many
// workgroups a CU holds)
// TOK: tokens per workgroup.  Every workgroup reads the whole router (E x d fp32) once, and with
// many tokens that re-read, not the token rows, is most of what the CUs pull in: at 2048 tokens of
// the 2048-wide, 8-expert router 11.1 us with four tokens per workgroup against 13.5 with two (and
// 11.2-12.1 with eight); at 512 tokens two are the faster (128 workgroups do not fill the chip).
template <typename T, int NB, int TOK>
__global__ __launch_bounds__(kRouteWaves* kWave) void route_kernel(
    const T* __restrict__ x, const float* __restrict__ rw, const float* __restrict__ rb,
    int32_t* __restrict__ topk_idx, float* __restrict__ topk_gate, float* __restrict__ probs,
    int T_, int d, int E, int k) {
    typedef Store<T> S;
    constexpr int VEC = S::VEC;
    __shared__ float s_logit[TOK][kMaxExperts];

    const int t0 = blockIdx.x * TOK;
    const int ntok = min(TOK, T_ - t0);
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;

    auto load_x = [&](int t, int i, float* out) {
        const typename S::vec_t xv =
            *reinterpret_cast<const typename S::vec_t*>(x + (size_t)(t0 + t) * d + i);
#pragma unroll
        for (int q = 0; q < VEC; ++q) out[q] = S::get(xv, q);
    };
    for (int e = wave; e < E; e += kRouteWaves) {
        float acc[TOK];
        // (the bias is requested before the row is streamed: at a single token, with a cold router,
        // a load issued only after the reduction is a second full memory round trip)
        const float b = rb ? rb[e] : 0.f;
        router_logits<VEC, TOK, NB>(load_x, rw + (size_t)e * d, d, lane, ntok, acc);
        if (lane == 0) {
#pragma unroll
            for (int t = 0; t < TOK; ++t) s_logit[t][e] = acc[t] + b;
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

// Large batches: the whole router (E x d fp32) is staged in LDS once per workgroup and a wave
// owns a token: it reads the token's row once, takes the E router rows from LDS and ends with
// one butterfly per expert, so lane e holds logit e and the selection follows in the same wave
// with no further exchange.  The multiply-adds of a logit run in the same order as in
// router_logits (lane l: elements [l*VEC, l*VEC+VEC) of every 64*VEC-wide chunk, ascending), so
// both kernels give bit-identical logits.  For E <= kRouteLdsMaxE and E * d * 4 bytes of LDS.
constexpr int kRouteLdsMaxE = 16;
constexpr int kRouteLdsBytes = 128 * 1024;

template <typename T>
__global__ __launch_bounds__(kRouteWaves* kWave) void route_lds_kernel(
    const T* __restrict__ x, const float* __restrict__ rw, const float* __restrict__ rb,
    int32_t* __restrict__ topk_idx, float* __restrict__ topk_gate, float* __restrict__ probs,
    int T_, int d, int E, int k, int tokens_per_wave) {
    typedef Store<T> S;
    constexpr int VEC = S::VEC;
    constexpr int CH = kWave * VEC;
    extern __shared__ __align__(16) float s_rw[];  // [E][d]
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    for (int i = threadIdx.x; i < E * d / 4; i += kRouteWaves * kWave)
        reinterpret_cast<f32x4*>(s_rw)[i] = reinterpret_cast<const f32x4*>(rw)[i];
    __syncthreads();

    const int t_first = (blockIdx.x * kRouteWaves + wave) * tokens_per_wave;
    const int nfull = d / CH;
    for (int t = t_first; t < min(T_, t_first + tokens_per_wave); ++t) {
        float acc[kRouteLdsMaxE];
#pragma unroll
        for (int e = 0; e < kRouteLdsMaxE; ++e) acc[e] = 0.f;
        auto chunk = [&](int i) {
            const typename S::vec_t xv = *reinterpret_cast<const typename S::vec_t*>(x + (size_t)t * d + i);
#pragma unroll
            for (int e = 0; e < kRouteLdsMaxE; ++e) {
                if (e < E) {  // wave-uniform
                    const float* w = s_rw + e * d + i;
#pragma unroll
                    for (int q = 0; q < VEC; q += 4) {
                        const f32x4 wv = *reinterpret_cast<const f32x4*>(w + q);
                        acc[e] = fmaf(S::get(xv, q + 0), wv[0], acc[e]);
                        acc[e] = fmaf(S::get(xv, q + 1), wv[1], acc[e]);
                        acc[e] = fmaf(S::get(xv, q + 2), wv[2], acc[e]);
                        acc[e] = fmaf(S::get(xv, q + 3), wv[3], acc[e]);
                    }
                }
            }
        };
        for (int c = 0; c < nfull; ++c) chunk(c * CH + lane * VEC);
        if (nfull * CH + lane * VEC < d) chunk(nfull * CH + lane * VEC);
        float logit = 0.f;
#pragma unroll
        for (int e = 0; e < kRouteLdsMaxE; ++e) {
            if (e < E) {
                const float sum = wave_sum(acc[e]);
                if (lane == e) logit = sum + (rb ? rb[e] : 0.f);
            }
        }
        const RouterPick r = router_select(lane, E, k, lane < E ? logit : 0.f);
        if (probs && lane < E) probs[(size_t)t * E + lane] = r.p / r.den;
        if (r.slot >= 0) {
            topk_idx[(size_t)t * k + r.slot] = lane;
            topk_gate[(size_t)t * k + r.slot] = r.p / r.sel_sum;
        }
    }
}

template <typename T>
static int launch_route_lds(const moe_shape& s, const T* x, const float* rw, const float* rb,
                            int32_t* topk_idx, float* topk_gate, float* probs, hipStream_t st) {
    const size_t lds = (size_t)s.n_experts * s.d_model * sizeof(float);
    static std::atomic<uint64_t> lds_allowed;
    if (allow_dynamic_lds(reinterpret_cast<const void*>(route_lds_kernel<T>), kRouteLdsBytes, lds_allowed) != MOE_OK)
        return MOE_ERR_LAUNCH;
    // up to two workgroups per CU, every wave with the same number of tokens
    const int waves = 2 * 256 * kRouteWaves;
    const int tokens_per_wave = (s.n_tokens + waves - 1) / waves;
    const int per_block = tokens_per_wave * kRouteWaves;
    dim3 grid((s.n_tokens + per_block - 1) / per_block), block(kRouteWaves * kWave);
    hipLaunchKernelGGL(route_lds_kernel<T>, grid, block, lds, st, x, rw, rb, topk_idx, topk_gate, probs,
                       s.n_tokens, s.d_model, s.n_experts, s.top_k, tokens_per_wave);
    return launch_status();
}

int launch_route(const moe_shape& s, const void* x, const float* rw, const float* rb,
                 int32_t* topk_idx, float* topk_gate, float* probs, hipStream_t st) {
    if (s.n_tokens == 0) return MOE_OK;
    // (measured on the 2048-wide, 8-expert router: 15.6 us against 12.7 at 2048 tokens, 41 against
    // 64 at 16384; the two cross near 4096)
    if (s.n_tokens >= 8192 && s.n_experts <= kRouteLdsMaxE &&
        (size_t)s.n_experts * s.d_model * sizeof(float) <= (size_t)kRouteLdsBytes) {
        if (s.act_dtype == MOE_F32)
            return launch_route_lds<float>(s, (const float*)x, rw, rb, topk_idx, topk_gate, probs, st);
        return launch_route_lds<bf16_t>(s, (const bf16_t*)x, rw, rb, topk_idx, topk_gate, probs, st);
    }
    const bool small = s.n_tokens <= 256, large = s.n_tokens >= kRouteLargeFrom;
    const int tok = large ? kRouteTokLarge : kRouteTok;
    dim3 grid((s.n_tokens + tok - 1) / tok), block(kRouteWaves * kWave);
    auto launch = [&](auto kern, auto* xp) {
        hipLaunchKernelGGL(kern, grid, block, 0, st, xp, rw, rb, topk_idx, topk_gate, probs, s.n_tokens,
                           s.d_model, s.n_experts, s.top_k);
    };
    if (s.act_dtype == MOE_F32) {
        if (small) launch(route_kernel<float, 4, kRouteTok>, (const float*)x);
        else if (!large) launch(route_kernel<float, MOE_ROUTE_NB_LARGE, kRouteTok>, (const float*)x);
        else launch(route_kernel<float, MOE_ROUTE_NB_LARGE, kRouteTokLarge>, (const float*)x);
    } else {
        if (small) launch(route_kernel<bf16_t, 4, kRouteTok>, (const bf16_t*)x);
        else if (!large) launch(route_kernel<bf16_t, MOE_ROUTE_NB_LARGE, kRouteTok>, (const bf16_t*)x);
        else launch(route_kernel<bf16_t, MOE_ROUTE_NB_LARGE, kRouteTokLarge>, (const bf16_t*)x);
    }
    return launch_status();
}

}  // namespace moe
