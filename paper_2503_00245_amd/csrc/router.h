// Router arithmetic shared by the stand-alone route kernel and the single-token expert
// kernel that recomputes the routing in its prologue (Sec. 2.3: Eq. 2 softmax at
// temperature 1, Eq. 3 top-k; lowest index wins ties; gates renormalised over the k
// chosen).  Both callers go through these functions with the same lane layout, so their
// logits, indices and gates are bit-identical.
#pragma once

#include "common.h"

namespace moe {

// One wave: logit <x, we> (+ nothing: the caller adds the bias).  Lane l takes elements
// [l*VEC, l*VEC+VEC) of every 64*VEC-wide chunk, fused multiply-adds in ascending index
// order, then a 64-lane butterfly.  load_x(i, out) must yield x[i .. i+VEC) as floats.
template <int VEC, typename LoadX>
__device__ __forceinline__ float router_logit(LoadX load_x, const float* __restrict__ we, int d,
                                              int lane) {
    float acc = 0.f;
    for (int i = lane * VEC; i < d; i += kWave * VEC) {
        float xv[VEC];
        load_x(i, xv);
#pragma unroll
        for (int q = 0; q < VEC; q += 4) {
            const f32x4 wv = *reinterpret_cast<const f32x4*>(we + i + q);
            acc = fmaf(xv[q + 0], wv[0], acc);
            acc = fmaf(xv[q + 1], wv[1], acc);
            acc = fmaf(xv[q + 2], wv[2], acc);
            acc = fmaf(xv[q + 3], wv[3], acc);
        }
    }
    return wave_sum(acc);
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
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) {
            const float ov = __shfl_xor(bv, m, kWave);
            const int oi = __shfl_xor(bi, m, kWave);
            if (ov > bv || (ov == bv && oi < bi)) {
                bv = ov;
                bi = oi;
            }
        }
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
