// Router arithmetic (Sec. 2.3: Eq. 2 softmax at temperature 1, Eq. 3 top-k; lowest index
// wins ties; gates renormalised over the k chosen), kept apart from the kernel that drives
// it so that every caller produces bit-identical logits, indices and gates.
#pragma once

#include <type_traits>

#include "common.h"

namespace moe {

// One wave, TOK tokens at once: logits <x_t, we> (the caller adds the bias).  Lane l takes
// elements [l*VEC, l*VEC+VEC) of every 64*VEC-wide chunk; per token the fused multiply-adds
// run in ascending index order and end in a 64-lane butterfly, so a token's logit does not
// depend on TOK.  load_x(t, i, out) must yield x_t[i .. i+VEC) as floats; only tokens
// t < ntok are ever asked for (the slots beyond re-read the last valid token and are ignored).  The router row is read once per chunk and reused for all TOK tokens.
template <int VEC, int TOK, int NBATCH = 4, typename LoadX>
__device__ __forceinline__ void router_logits(LoadX load_x, const float* __restrict__ we, int d,
                                              int lane, int ntok, float (&out)[TOK]) {
    float acc[TOK];
#pragma unroll
    for (int t = 0; t < TOK; ++t) acc[t] = 0.f;
    // NB chunks at once (NBATCH of them while that many are left): every load of the batch (router row and all TOK token rows; a token
    // beyond ntok re-reads the last valid one, so no load is conditional) is issued before the
    // first multiply-add.  Chunk by chunk, with a wait after each load, a single cold token paid
    // eight dependent memory round trips for 12 KB.
    auto batch = [&](int i0, auto nb) {
        constexpr int NB = decltype(nb)::value;
        constexpr int CHB = kWave * VEC;
        f32x4 wv[NB][VEC / 4];
        float xv[NB][TOK][VEC];
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int q = 0; q < VEC; q += 4) wv[b][q / 4] = *reinterpret_cast<const f32x4*>(we + i0 + b * CHB + q);
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int t = 0; t < TOK; ++t) load_x(min(t, ntok - 1), i0 + b * CHB, xv[b][t]);
#if defined(__HIP_DEVICE_COMPILE__)
        __builtin_amdgcn_sched_group_barrier(0x020, NB * (VEC / 4) + NB * TOK * (VEC == 8 ? 1 : VEC / 4), 0);
#endif
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int t = 0; t < TOK; ++t)
#pragma unroll
                for (int q = 0; q < VEC; q += 4) {
                    acc[t] = fmaf(xv[b][t][q + 0], wv[b][q / 4][0], acc[t]);
                    acc[t] = fmaf(xv[b][t][q + 1], wv[b][q / 4][1], acc[t]);
                    acc[t] = fmaf(xv[b][t][q + 2], wv[b][q / 4][2], acc[t]);
                    acc[t] = fmaf(xv[b][t][q + 3], wv[b][q / 4][3], acc[t]);
                }
    };
    constexpr int CH = kWave * VEC;
    const int nfull = d / CH;
    int c = 0;
    for (; c + NBATCH <= nfull; c += NBATCH) batch(c * CH + lane * VEC, std::integral_constant<int, NBATCH>{});
    for (; c < nfull; ++c) batch(c * CH + lane * VEC, std::integral_constant<int, 1>{});
    if (nfull * CH + lane * VEC < d) batch(nfull * CH + lane * VEC, std::integral_constant<int, 1>{});
#pragma unroll
    for (int t = 0; t < TOK; ++t) out[t] = wave_sum(acc[t]);
}

struct RouterPick {
    int slot;        // selection round in which this lane's expert was taken, or -1
    float p;         // exp(logit - max) of this lane's expert (0 for lanes >= E)
    float den;       // sum of p over all experts
    float sel_sum;   // sum of p over the k selected experts
};

// One wave, lane e owning expert e (lanes >= E idle): k rounds of a (value, index) arg-max
// butterfly on the logits; equal logits go to the lower index.
__device__ __forceinline__ RouterPick router_select(int lane, int E, int k, float logit_of_lane) {
    const bool valid = lane < E;
    const float logit = valid ? logit_of_lane : -INFINITY;
    float cand = logit;  // -inf once taken
    float vmax = 0.f;
    RouterPick r;
    r.slot = -1;
    for (int j = 0; j < k; ++j) {
        float bv = cand;
        int bi = lane;
        auto take = [&](float ov, int oi) {
            if (ov > bv || (ov == bv && oi < bi)) {
                bv = ov;
                bi = oi;
            }
        };
        // (value, index) arg-max all-reduce; every pairing is symmetric, so all lanes agree
        take(dpp_f32<kDppSwap1>(bv), dpp_i32<kDppSwap1>(bi));
        take(dpp_f32<kDppSwap2>(bv), dpp_i32<kDppSwap2>(bi));
        take(dpp_f32<kDppHalfMirror>(bv), dpp_i32<kDppHalfMirror>(bi));
        take(dpp_f32<kDppMirror>(bv), dpp_i32<kDppMirror>(bi));
        take(__shfl_xor(bv, 16, kWave), __shfl_xor(bi, 16, kWave));
        take(__shfl_xor(bv, 32, kWave), __shfl_xor(bi, 32, kWave));
        if (j == 0) vmax = bv;  // the first pick is the row maximum
        if (lane == bi) {
            cand = -INFINITY;
            r.slot = j;
        }
    }
    r.p = valid ? __expf(logit - vmax) : 0.f;
    r.den = wave_sum(r.p);
    r.sel_sum = wave_sum(r.slot >= 0 ? r.p : 0.f);
    return r;
}

}  // namespace moe
