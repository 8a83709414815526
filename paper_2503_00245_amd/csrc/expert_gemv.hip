// Single-token (decode) expert path: only the k selected experts' matrices are streamed
// from HBM, once, as wave-per-row matrix-vector products (the paper's observation that
// generation time scales with the active and not the total experts, Sec. 3.4.3, is this
// bandwidth bound).  The expert ids are read on the device from topk_idx; the host never
// sees them.
//
// One generic kernel covers every stage of a dense or weight-decomposed (Sec. 2.2, Eq. 1)
// SwiGLU expert.  A stage is: for every output row, for every selected pair j,
//     acc_j = sum over up to two "segments" of  <W_seg[expert_j][row,:], v_seg,j>
// followed by a mode-specific epilogue:
//     PLAIN    out0[j][row] = acc_j                                   (rank-r intermediates)
//     DUAL     two independent PLAIN products (gate and up factors)  in one pass
//     SWIGLU   out0[j][row] = silu(acc0_j) * acc1_j                   (hidden vector)
//     COMBINE  y[row] = sum_j gate_j * acc_j (+ residual[row])        (down proj. + combine)
// A segment whose matrix is shared by all experts (the shared dense base) is read once
// per row, not once per pair: with a shared input vector its product is reused for every
// pair; in COMBINE the pairs' inputs are pre-mixed with the gates (linearity).
// A wave reads a matrix row with 16-byte loads, 1 KB per instruction, takes the matching slice
// of the input vector straight from L1/L2, and reduces with a 64-lane butterfly.  Nothing is
// staged in LDS, so the weight stream starts at once.
//
// Two kernels.  gemv_pairs_kernel serves the stages with one segment and a matrix of its own per
// expert (every stage of a dense or purely decomposed expert): it walks the row chunk by chunk
// with the pairs inside, so a wave has the chunks of two experts (and of both matrices of a
// gate/up product) in flight at once -- eight 1 KB loads -- and reads a shared input vector once
// per chunk.  A wave's share of a row is a few KB, so what the stage costs is the number of
// dependent load round trips per wave, not the bytes: pair by pair and matrix by matrix the
// gate/up stage took eight round trips and the down stage six; chunk-major they take two.
// gemv_kernel is the general form (two segments, segments shared by all experts).
#include <type_traits>

#include "common.h"

namespace moe {

enum { GEMV_PLAIN = 0, GEMV_DUAL = 1, GEMV_SWIGLU = 2, GEMV_COMBINE = 3 };
constexpr int kGemvThreads = 512;
constexpr int kGemvWaves = kGemvThreads / kWave;
// Chunk loads a wave issues before consuming the first.  Measured on MI355X: 2 beats 1, 4
// and 8 -- many resident waves (about 60 VGPRs, 8 per SIMD) with few loads each stream
// faster than few waves with many loads each.
constexpr int kBatch = 2;

struct GemvSeg {
    const void* W0;      // [Eb, rows, n]
    const void* W1;      // second matrix (DUAL / SWIGLU), same shape
    long long stride;    // elements between experts; 0 = one matrix shared by all experts
    const void* v0;      // input vector(s): [n] if vstride == 0, else [k][n]
    const void* v1;      // input of the second product (may equal v0)
    int v_is_f32;        // 1: fp32 scratch vector; 0: stored in the activation type
    int vstride;         // elements between pairs' vectors; 0 = same vector for every pair
    int n;               // row length
    int vdiv;            // consecutive pairs that share one vector (a token's pairs share its row); 0 or 1: none
};

struct GemvArgs {
    GemvSeg seg[2];
    int nseg;
    int rows;
    int k;
    int rows_per_wave;
    int slices;           // waves per row: 1, 2, 4 or 8
    int E;
    const int32_t* idx;   // [k] selected experts
    const float* gate;    // [k]
    float* out0;          // [k][rows]
    void* out0_act;       // SWIGLU: [k][rows] in the activation type, written instead of out0 (or NULL)
    float* out1;          // [k][rows] (DUAL)
    void* y;              // [tokens][rows] activation type (COMBINE)
    const void* residual; // [tokens][rows] or NULL (COMBINE)
    int kk;               // pairs per token: the k pairs are k / kk tokens' (chunk-major kernel; 0 = one token)
};

// Where a stage's input vector comes from.  Vectors are read straight from global memory
// with the same 16-byte lane layout as the matrix row (they are a few KB, so they sit in
// L1/L2): no LDS staging, no barrier, and the weight stream starts with the first
// instruction of every wave.
struct VecSrc {
    const void* p;       // first element of this pair's vector
    int is_f32;          // 1: fp32 scratch vector, 0: activation type
    int nmix;            // 0: plain vector; else the gate-weighted mix of nmix vectors
    int mix_stride;      // elements between the mixed vectors
    const float* mix_w;  // [nmix] weights (the gates)
};

template <typename T>
__device__ __forceinline__ void load_vec_raw(const void* p, int is_f32, int off,
                                             float (&out)[Store<T>::VEC]) {
    typedef Store<T> S;
    if (is_f32) {
#pragma unroll
        for (int q = 0; q < S::VEC; q += 4) {
            const f32x4 t = *reinterpret_cast<const f32x4*>(static_cast<const float*>(p) + off + q);
            out[q] = t[0]; out[q + 1] = t[1]; out[q + 2] = t[2]; out[q + 3] = t[3];
        }
    } else {
        const typename S::vec_t t = *reinterpret_cast<const typename S::vec_t*>(static_cast<const T*>(p) + off);
#pragma unroll
        for (int q = 0; q < S::VEC; ++q) out[q] = S::get(t, q);
    }
}

// activation-typed / fp32 scratch / gate-mixed fp32 / gate-mixed activation-typed
enum { VK_ACT = 0, VK_F32 = 1, VK_MIX = 2, VK_MIX_ACT = 3 };

template <typename T, int VK>
__device__ __forceinline__ void load_vec(const VecSrc& v, int off, float (&out)[Store<T>::VEC]) {
    constexpr int VEC = Store<T>::VEC;
    if (VK == VK_ACT || VK == VK_F32) {
        load_vec_raw<T>(v.p, VK == VK_F32, off, out);
        return;
    }
#pragma unroll
    for (int q = 0; q < VEC; ++q) out[q] = 0.f;
    for (int j = 0; j < v.nmix; ++j) {
        float t[VEC];
        load_vec_raw<T>(v.p, VK == VK_MIX, j * v.mix_stride + off, t);
        const float g = v.mix_w[j];
#pragma unroll
        for (int q = 0; q < VEC; ++q) out[q] = fmaf(g, t[q], out[q]);
    }
}

// Lane-partial dot of one matrix row with a vector.  The row is cut into 1 KB chunks
// (64 lanes x 16 bytes); with `slices` > 1 this wave takes chunks slice, slice + slices, ...
// kBatch chunk loads (and their vector loads) are issued back to back before any is consumed.
template <typename T, int VK>
__device__ __forceinline__ float row_dot_k(const T* __restrict__ wrow, const VecSrc& v, int n,
                                           int lane, int slice, int slices) {
    typedef Store<T> S;
    typedef typename S::vec_t vec_t;
    constexpr int VEC = S::VEC;
    constexpr int CH = kWave * VEC;
    const int nfull = n / CH;
    const int lo = lane * VEC;
    float acc = 0.f;
    auto fma_chunk = [&](const vec_t& w, const float (&x)[VEC]) {
#pragma unroll
        for (int q = 0; q < VEC; ++q) acc = fmaf(S::get(w, q), x[q], acc);
    };
    auto load_chunk = [&](int c) {
        return __builtin_nontemporal_load(reinterpret_cast<const vec_t*>(wrow + c * CH + lo));
    };
    int c = slice;
    for (; c + (kBatch - 1) * slices < nfull; c += kBatch * slices) {
        vec_t w[kBatch];
        float x[kBatch][VEC];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) w[u] = load_chunk(c + u * slices);
#pragma unroll
        for (int u = 0; u < kBatch; ++u) load_vec<T, VK>(v, (c + u * slices) * CH + lo, x[u]);
#pragma unroll
        for (int u = 0; u < kBatch; ++u) fma_chunk(w[u], x[u]);
    }
    for (; c < nfull; c += slices) {
        const vec_t w0 = load_chunk(c);
        float x0[VEC];
        load_vec<T, VK>(v, c * CH + lo, x0);
        fma_chunk(w0, x0);
    }
    // ragged tail chunk (n is a multiple of VEC, so a lane is entirely in or out of it)
    if (c == nfull && nfull * CH + lo < n) {
        const vec_t w0 = load_chunk(nfull);
        float x0[VEC];
        load_vec<T, VK>(v, nfull * CH + lo, x0);
        fma_chunk(w0, x0);
    }
    return acc;
}

// MIX: the caller may pass gate-mixed vectors (only the down + combine stage does)
template <typename T, bool MIX>
__device__ __forceinline__ float row_dot(const T* __restrict__ wrow, const VecSrc& v, int n,
                                         int lane, int slice, int slices) {
    // wave-uniform dispatch on the vector kind, outside the streaming loop
    if (MIX && v.nmix)
        return v.is_f32 ? row_dot_k<T, VK_MIX>(wrow, v, n, lane, slice, slices)
                        : row_dot_k<T, VK_MIX_ACT>(wrow, v, n, lane, slice, slices);
    if (v.is_f32) return row_dot_k<T, VK_F32>(wrow, v, n, lane, slice, slices);
    return row_dot_k<T, VK_ACT>(wrow, v, n, lane, slice, slices);
}

template <typename T>
__device__ __forceinline__ void store_hidden(const GemvArgs& a, size_t at, float h) {
    if (a.out0_act)
        static_cast<T*>(a.out0_act)[at] = Store<T>::from_f32(h);
    else
        a.out0[at] = h;
}

// Workgroup = 8 waves = (8 / slices) rows x `slices` waves per row.  Short stages (few rows)
// use several waves per row so that every CU still has tens of waves with loads in flight;
// the per-slice sums meet in LDS and are added in slice order (deterministic).
template <typename T, int MODE>
__global__ __launch_bounds__(kGemvThreads) void gemv_kernel(const GemvArgs a) {
    __shared__ float s_part[kGemvWaves][2 * kMaxExperts + 2];
    constexpr bool DUAL = (MODE == GEMV_DUAL || MODE == GEMV_SWIGLU);
    const int lane = threadIdx.x & (kWave - 1);
    // (wave-uniform by construction; saying so keeps the row, the slice and the chunk loops in
    // scalar registers: 32.2 us per phone-shaped token instead of 33.6)
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int k = a.k;
    const int slices = a.slices;
    const int slice = wave % slices;
    const int local_row = wave / slices;

    bool once[2];  // segment evaluated once per row (shared matrix and one effective vector)
    bool premix[2];
    for (int s = 0; s < a.nseg; ++s) {
        const GemvSeg& g = a.seg[s];
        premix[s] = (MODE == GEMV_COMBINE) && g.stride == 0 && g.vstride != 0;
        once[s] = g.stride == 0 && (g.vstride == 0 || premix[s]);
    }
    auto vec_of = [&](const GemvSeg& g, const void* base, int j, bool mix) {
        VecSrc v;
        const size_t es = g.v_is_f32 ? 4 : sizeof(T);
        v.p = static_cast<const char*>(base) + (size_t)j * g.vstride * es;
        v.is_f32 = g.v_is_f32;
        v.nmix = mix ? k : 0;
        v.mix_stride = g.vstride;
        v.mix_w = a.gate;
        return v;
    };

    const int rows_per_block = kGemvWaves / slices;
    const int row0 = (blockIdx.x * rows_per_block + local_row) * a.rows_per_wave;
    // rows_per_wave is 1 whenever slices > 1, so the barrier below is reached once by all
    for (int ri = 0; ri < a.rows_per_wave; ++ri) {
        const int row = row0 + ri;
        const bool active = row < a.rows;
        float* part = s_part[wave];
        // per-slice sums of this row: [0],[1] segments read once per row; [2+2j],[3+2j] pair j
        float sh0 = 0.f, sh1 = 0.f;
        if (active) {
            for (int s = 0; s < a.nseg; ++s) {
                if (!once[s]) continue;
                const GemvSeg& g = a.seg[s];
                sh0 += row_dot<T, MODE == GEMV_COMBINE>(static_cast<const T*>(g.W0) + (size_t)row * g.n,
                                  vec_of(g, g.v0, 0, premix[s]), g.n, lane, slice, slices);
                if (DUAL)
                    sh1 += row_dot<T, MODE == GEMV_COMBINE>(static_cast<const T*>(g.W1) + (size_t)row * g.n,
                                      vec_of(g, g.v1, 0, premix[s]), g.n, lane, slice, slices);
            }
        }
        sh0 = wave_sum(sh0);
        if (DUAL) sh1 = wave_sum(sh1);
        float total = sh0;  // COMBINE, single slice
        for (int j = 0; j < k; ++j) {
            float acc0 = 0.f, acc1 = 0.f;
            if (active) {
                const int e = min(max(a.idx[j], 0), a.E - 1);
                for (int s = 0; s < a.nseg; ++s) {
                    if (once[s]) continue;
                    const GemvSeg& g = a.seg[s];
                    const size_t woff = (size_t)e * g.stride + (size_t)row * g.n;
                    acc0 += row_dot<T, MODE == GEMV_COMBINE>(static_cast<const T*>(g.W0) + woff, vec_of(g, g.v0, j, false),
                                       g.n, lane, slice, slices);
                    if (DUAL)
                        acc1 += row_dot<T, MODE == GEMV_COMBINE>(static_cast<const T*>(g.W1) + woff,
                                           vec_of(g, g.v1, j, false), g.n, lane, slice, slices);
                }
            }
            acc0 = wave_sum(acc0);
            if (DUAL) acc1 = wave_sum(acc1);
            if (slices > 1) {
                if (lane == 0) {
                    part[2 + 2 * j] = acc0;
                    part[3 + 2 * j] = acc1;
                }
            } else if (MODE == GEMV_COMBINE) {
                total = fmaf(a.gate[j], acc0, total);
            } else if (lane == 0 && active) {
                if (MODE == GEMV_SWIGLU) {
                    store_hidden<T>(a, (size_t)j * a.rows + row, silu_f32(sh0 + acc0) * (sh1 + acc1));
                } else {
                    a.out0[(size_t)j * a.rows + row] = sh0 + acc0;
                    if (MODE == GEMV_DUAL) a.out1[(size_t)j * a.rows + row] = sh1 + acc1;
                }
            }
        }
        if (slices > 1) {
            if (lane == 0) {
                part[0] = sh0;
                part[1] = sh1;
            }
            __syncthreads();
            if (slice == 0 && active) {
                // lane q sums value q (and q + 64) over the row's slices, in slice order
                float sum_lo = 0.f, sum_hi = 0.f;
                for (int sl = 0; sl < slices; ++sl) {
                    if (lane < 2 + 2 * k) sum_lo += s_part[wave + sl][lane];
                    if (lane + kWave < 2 + 2 * k) sum_hi += s_part[wave + sl][lane + kWave];
                }
                auto value = [&](int q) {
                    return q < kWave ? __shfl(sum_lo, q, kWave) : __shfl(sum_hi, q - kWave, kWave);
                };
                const float t0 = value(0), t1 = value(1);
                if (MODE == GEMV_COMBINE) {
                    float tot = t0;
                    for (int j = 0; j < k; ++j) tot = fmaf(a.gate[j], value(2 + 2 * j), tot);
                    total = tot;
                } else {
                    for (int j = 0; j < k; ++j) {
                        const float a0 = t0 + value(2 + 2 * j);
                        const float a1 = t1 + value(3 + 2 * j);
                        if (lane == 0) {
                            if (MODE == GEMV_SWIGLU) {
                                store_hidden<T>(a, (size_t)j * a.rows + row, silu_f32(a0) * a1);
                            } else {
                                a.out0[(size_t)j * a.rows + row] = a0;
                                if (MODE == GEMV_DUAL) a.out1[(size_t)j * a.rows + row] = a1;
                            }
                        }
                    }
                }
            }
        }
        if (MODE == GEMV_COMBINE && lane == 0 && active && slice == 0) {
            if (a.residual) total += Store<T>::to_f32(static_cast<const T*>(a.residual)[row]);
            static_cast<T*>(a.y)[row] = Store<T>::from_f32(total);
        }
    }
}


// ---- one segment, one matrix per expert: chunk-major over pairs -------------------------------
enum { VS_SHARED = 0, VS_PAIR_ACT = 1, VS_PAIR_F32 = 2 };  // one activation-typed vector for all pairs / one per pair

// Row results of one wave -> outputs.  Shared by the single-slice paths of both kernels' callers.
template <typename T, int MODE>
__device__ __forceinline__ void store_pair(const GemvArgs& a, int j, int row, float a0, float a1) {
    if (MODE == GEMV_SWIGLU) {
        store_hidden<T>(a, (size_t)j * a.rows + row, silu_f32(a0) * a1);
    } else {
        a.out0[(size_t)j * a.rows + row] = a0;
        if (MODE == GEMV_DUAL) a.out1[(size_t)j * a.rows + row] = a1;
    }
}

// SEVERAL: the k pairs belong to k / kk tokens (a separate instantiation: the single token's
// kernel carries none of the per-token bookkeeping, which cost its down + combine stage 4-7 %)
template <typename T, int MODE, int VS, bool SEVERAL>
__global__ __launch_bounds__(kGemvThreads) __attribute__((amdgpu_waves_per_eu(4, 4))) void gemv_pairs_kernel(const GemvArgs a) {
    typedef Store<T> S;
    typedef typename S::vec_t vec_t;
    constexpr int VEC = S::VEC;
    constexpr int CH = kWave * VEC;
    constexpr bool DUAL = (MODE == GEMV_DUAL || MODE == GEMV_SWIGLU);
    // chunks of one pair group in flight: 8 weight loads per wave either way (fp32 vectors, twice
    // the registers per chunk, take half)
    constexpr int UB = (DUAL || VS == VS_PAIR_F32) ? 2 : 4;
    __shared__ float s_part[kGemvWaves][2 * kMaxExperts + 2];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int k = a.k;
    const int slices = a.slices;
    const int slice = wave % slices;
    const int local_row = wave / slices;
    const GemvSeg& g = a.seg[0];
    const int n = g.n;
    const int nfull = n / CH;
    const int lo = lane * VEC;
    const bool tail_lane = nfull * CH + lo < n;  // n is a multiple of VEC: a lane is wholly in or out
    const bool two_vecs = DUAL && g.v1 != g.v0;
    const int vdiv = SEVERAL && g.vdiv > 1 ? g.vdiv : 1;
    const int kk = SEVERAL && a.kk > 0 ? a.kk : k;  // pairs per token; COMBINE writes one output row per token
    // COMBINE: token t's output element of this row, from the gate-weighted sum of its pairs
    auto store_token = [&](int t, int row, float total) {
        if (a.residual) total += Store<T>::to_f32(static_cast<const T*>(a.residual)[(size_t)t * a.rows + row]);
        static_cast<T*>(a.y)[(size_t)t * a.rows + row] = Store<T>::from_f32(total);
    };

    const int rows_per_block = kGemvWaves / slices;
    const int row0 = (blockIdx.x * rows_per_block + local_row) * a.rows_per_wave;
    for (int ri = 0; ri < a.rows_per_wave; ++ri) {
        const int row = row0 + ri;
        const bool active = row < a.rows;
        float* part = s_part[wave];
        float total = 0.f;  // COMBINE, single slice: the running sum of the current token's pairs
        // One token: the residual element this wave will add is requested now, ahead of the weight
        // stream (asked for at the end, its latency would be the wave's last wait).
        float res0 = 0.f;
        if constexpr (MODE == GEMV_COMBINE && !SEVERAL) {
            if (a.residual && lane == 0 && active && slice == 0)
                res0 = Store<T>::to_f32(static_cast<const T*>(a.residual)[row]);
        }
        // KJ pairs at a time: their chunk loads are issued together
        auto group = [&](int j0, auto kj) {
            constexpr int KJ = decltype(kj)::value;
            const T* w0[KJ];
            const T* w1[KJ];
            const void* v0[KJ];
            const void* v1[KJ];
#pragma unroll
            for (int q = 0; q < KJ; ++q) {
                const int e = min(max(a.idx[j0 + q], 0), a.E - 1);
                const size_t woff = (size_t)e * g.stride + (size_t)row * n;
                w0[q] = static_cast<const T*>(g.W0) + woff;
                w1[q] = DUAL ? static_cast<const T*>(g.W1) + woff : w0[q];
                const size_t voff = (size_t)(SEVERAL ? (j0 + q) / vdiv : j0 + q) * g.vstride * (VS == VS_PAIR_F32 ? 4 : sizeof(T));
                v0[q] = static_cast<const char*>(g.v0) + voff;
                v1[q] = DUAL ? static_cast<const char*>(g.v1) + voff : v0[q];
            }
            float acc0[KJ], acc1[KJ], gq[KJ];
#pragma unroll
            for (int q = 0; q < KJ; ++q) {
                acc0[q] = acc1[q] = 0.f;
                gq[q] = MODE == GEMV_COMBINE ? a.gate[j0 + q] : 0.f;  // with the expert ids, not after the stream
            }
            // nu chunks c, c + slices, ...: every load of the batch is issued before the first sum
            // (the scheduling barrier keeps the compiler from sinking each load to its use, which
            // would leave one load in flight per wave)
            auto chunks = [&](int c, auto nu) {
                constexpr int NU = decltype(nu)::value;
                constexpr int NV = VS == VS_SHARED ? 1 : KJ;          // vectors per chunk and product
                constexpr int VL = VS == VS_PAIR_F32 ? VEC / 4 : 1;   // load instructions per vector chunk
                typedef typename std::conditional<VS == VS_PAIR_F32, f32x4, vec_t>::type xv_t;
                vec_t wa[NU][KJ], wb[DUAL ? NU : 1][DUAL ? KJ : 1];
                xv_t xa[NU][NV][VL], xb[DUAL ? NU : 1][DUAL ? NV : 1][VL];
#pragma unroll
                for (int u = 0; u < NU; ++u)
#pragma unroll
                    for (int q = 0; q < KJ; ++q) {
                        const int at = (c + u * slices) * CH + lo;
                        wa[u][q] = __builtin_nontemporal_load(reinterpret_cast<const vec_t*>(w0[q] + at));
                        if (DUAL) wb[u][q] = __builtin_nontemporal_load(reinterpret_cast<const vec_t*>(w1[q] + at));
                    }
#pragma unroll
                for (int u = 0; u < NU; ++u)
#pragma unroll
                    for (int q = 0; q < NV; ++q) {
                        const int at = (c + u * slices) * CH + lo;
#pragma unroll
                        for (int l = 0; l < VL; ++l) {
                            if (VS == VS_PAIR_F32) {
                                xa[u][q][l] = *reinterpret_cast<const xv_t*>(static_cast<const float*>(v0[q]) + at + 4 * l);
                                if (DUAL) xb[u][q][l] = *reinterpret_cast<const xv_t*>(static_cast<const float*>(v1[q]) + at + 4 * l);
                            } else {
                                xa[u][q][l] = *reinterpret_cast<const xv_t*>(static_cast<const T*>(v0[q]) + at);
                                if (DUAL) xb[u][q][l] = two_vecs ? *reinterpret_cast<const xv_t*>(static_cast<const T*>(v1[q]) + at) : xa[u][q][l];
                            }
                        }
                    }
#if defined(__HIP_DEVICE_COMPILE__)
                __builtin_amdgcn_sched_group_barrier(0x020, NU * KJ * (DUAL ? 2 : 1) + NU * NV * VL * (DUAL ? 2 : 1), 0);
#endif
#pragma unroll
                for (int u = 0; u < NU; ++u)
#pragma unroll
                    for (int q = 0; q < KJ; ++q) {
                        const int qv = VS == VS_SHARED ? 0 : q;
#pragma unroll
                        for (int i = 0; i < VEC; ++i) {
                            float x0, x1;
                            if (VS == VS_PAIR_F32) {
                                x0 = xa[u][qv][i / 4][i % 4];
                                x1 = DUAL ? xb[u][qv][i / 4][i % 4] : 0.f;
                            } else {
                                x0 = S::to_f32(xa[u][qv][0][i]);
                                x1 = DUAL ? S::to_f32(xb[u][qv][0][i]) : 0.f;
                            }
                            acc0[q] = fmaf(S::get(wa[u][q], i), x0, acc0[q]);
                            if (DUAL) acc1[q] = fmaf(S::get(wb[u][q], i), x1, acc1[q]);
                        }
                    }
            };
            if (active) {
                int c = slice;
                for (; c + (UB - 1) * slices < nfull; c += UB * slices) chunks(c, std::integral_constant<int, UB>{});
                for (; c < nfull; c += slices) chunks(c, std::integral_constant<int, 1>{});
                if (c == nfull && tail_lane) chunks(nfull, std::integral_constant<int, 1>{});
            }
#pragma unroll
            for (int q = 0; q < KJ; ++q) {
                const int j = j0 + q;
                const float s0 = wave_sum(acc0[q]);
                const float s1 = DUAL ? wave_sum(acc1[q]) : 0.f;
                if (slices > 1) {
                    if (lane == 0) {
                        part[2 + 2 * j] = s0;
                        part[3 + 2 * j] = s1;
                    }
                } else if (MODE == GEMV_COMBINE) {
                    total = fmaf(gq[q], s0, total);
                    if constexpr (SEVERAL) {
                        if ((j + 1) % kk == 0) {  // the token's last pair
                            if (lane == 0 && active) store_token(j / kk, row, total);
                            total = 0.f;
                        }
                    }
                } else if (lane == 0 && active) {
                    store_pair<T, MODE>(a, j, row, s0, s1);
                }
            }
        };
        int j0 = 0;
        for (; j0 + 2 <= k; j0 += 2) group(j0, std::integral_constant<int, 2>{});
        if (j0 < k) group(j0, std::integral_constant<int, 1>{});

        if (slices > 1) {  // rows_per_wave is 1 here: the barrier is reached once, by every wave
            __syncthreads();
            if (slice == 0 && active) {
                // lane q sums value q (and q + 64) over the row's slices, in slice order
                float sum_lo = 0.f, sum_hi = 0.f;
                for (int sl = 0; sl < slices; ++sl) {
                    if (lane >= 2 && lane < 2 + 2 * k) sum_lo += s_part[wave + sl][lane];
                    if (lane + kWave < 2 + 2 * k) sum_hi += s_part[wave + sl][lane + kWave];
                }
                auto value = [&](int q) {
                    return q < kWave ? __shfl(sum_lo, q, kWave) : __shfl(sum_hi, q - kWave, kWave);
                };
                if (MODE == GEMV_COMBINE) {
                    if constexpr (SEVERAL) {
                        for (int t = 0; t < k / kk; ++t) {
                            float tot = 0.f;
                            for (int j = t * kk; j < (t + 1) * kk; ++j) tot = fmaf(a.gate[j], value(2 + 2 * j), tot);
                            if (lane == 0) store_token(t, row, tot);
                        }
                    } else {
                        float tot = 0.f;
                        for (int j = 0; j < k; ++j) tot = fmaf(a.gate[j], value(2 + 2 * j), tot);
                        total = tot;
                    }
                } else {
                    for (int j = 0; j < k; ++j) {
                        const float a0 = value(2 + 2 * j), a1 = value(3 + 2 * j);
                        if (lane == 0) store_pair<T, MODE>(a, j, row, a0, a1);
                    }
                }
            }
        }
        if constexpr (!SEVERAL) {
            if (MODE == GEMV_COMBINE && lane == 0 && active && slice == 0)
                static_cast<T*>(a.y)[row] = Store<T>::from_f32(total + res0);
        }
    }
}

template <typename T>
static int launch_gemv(GemvArgs& a, int mode, hipStream_t st) {
    const size_t lds = 0;
    const GemvSeg& g = a.seg[0];
    const bool dual = mode == GEMV_DUAL || mode == GEMV_SWIGLU;
    // One segment with a matrix per expert: the chunk-major kernel, unless the stage is a large
    // two-matrix one.  Measured per stage (events; old / chunk-major): 2048 x 5632 gate/up, 92 MB:
    // 20.0 / 21.4 us (there the stage runs at the rate of a plain read, and the older kernel's
    // eight waves per SIMD all fit the chip at once where the wider kernel's four do not);
    // 1024 x 2816 gate/up, 23 MB: 12.2 / 10.9; rank-1024 factors of a 2048 x 5632 expert: 12.3 /
    // 10.2, 15.0 / 15.2, 11.7 / 10.3, 9.6 / 7.5; 2048 x 5632 down + combine, 46 MB: 13.9 / 13.4.
    const size_t stage_bytes = (size_t)a.k * a.rows * g.n * (dual ? 2 : 1) * sizeof(T);
    const bool several = a.kk > 0 && a.kk < a.k;  // several tokens: only the chunk-major kernel knows them
    const bool pairs = a.nseg == 1 && g.stride != 0 && (g.vstride != 0 || !g.v_is_f32) &&
                       (several || !(dual && stage_bytes > ((size_t)64 << 20)));
    if (several && !pairs) return MOE_ERR_UNSUPPORTED;
    // enough waves that every CU holds many of them: split rows over several waves when the
    // stage has few rows, give a wave several rows when it has very many.  A wave of the
    // chunk-major kernel keeps eight weight loads in flight, so half as many waves do.
    const int want_waves = pairs ? 256 * 8 : 256 * 16;
    a.slices = 1;
    while (a.k < 63 && a.slices < kGemvWaves && a.rows * a.slices * 2 <= want_waves) a.slices *= 2;
    a.rows_per_wave = a.slices > 1 ? 1 : max(1, min(8, a.rows / (4 * want_waves)));
    const int rows_per_block = (kGemvWaves / a.slices) * a.rows_per_wave;
    dim3 grid((a.rows + rows_per_block - 1) / rows_per_block), block(kGemvThreads);
    if (pairs) {
        const int vs = g.vstride == 0 ? VS_SHARED : (g.v_is_f32 ? VS_PAIR_F32 : VS_PAIR_ACT);
#define MOE_GEMV_PAIRS(M, V, SEV)                                                                   \
    if (mode == M && vs == V && several == SEV) {                                                  \
        hipLaunchKernelGGL((gemv_pairs_kernel<T, M, V, SEV>), grid, block, lds, st, a);            \
        return launch_status();                                                                    \
    }
        // one token: its row is every pair's input (shared); several: a row per kk pairs
        MOE_GEMV_PAIRS(GEMV_DUAL, VS_SHARED, false)
        MOE_GEMV_PAIRS(GEMV_DUAL, VS_PAIR_ACT, true)
        MOE_GEMV_PAIRS(GEMV_SWIGLU, VS_SHARED, false)
        MOE_GEMV_PAIRS(GEMV_SWIGLU, VS_PAIR_ACT, true)
        MOE_GEMV_PAIRS(GEMV_SWIGLU, VS_PAIR_F32, false)
        MOE_GEMV_PAIRS(GEMV_SWIGLU, VS_PAIR_F32, true)
        MOE_GEMV_PAIRS(GEMV_PLAIN, VS_PAIR_ACT, false)
        MOE_GEMV_PAIRS(GEMV_PLAIN, VS_PAIR_ACT, true)
        MOE_GEMV_PAIRS(GEMV_PLAIN, VS_PAIR_F32, false)
        MOE_GEMV_PAIRS(GEMV_PLAIN, VS_PAIR_F32, true)
        MOE_GEMV_PAIRS(GEMV_COMBINE, VS_PAIR_ACT, false)
        MOE_GEMV_PAIRS(GEMV_COMBINE, VS_PAIR_ACT, true)
        MOE_GEMV_PAIRS(GEMV_COMBINE, VS_PAIR_F32, false)
        MOE_GEMV_PAIRS(GEMV_COMBINE, VS_PAIR_F32, true)
#undef MOE_GEMV_PAIRS
        return MOE_ERR_LAUNCH;  // unreachable: every (mode, vector kind) the stages use is listed
    }
    switch (mode) {
        case GEMV_PLAIN:
            hipLaunchKernelGGL((gemv_kernel<T, GEMV_PLAIN>), grid, block, lds, st, a);
            break;
        case GEMV_DUAL:
            hipLaunchKernelGGL((gemv_kernel<T, GEMV_DUAL>), grid, block, lds, st, a);
            break;
        case GEMV_SWIGLU:
            hipLaunchKernelGGL((gemv_kernel<T, GEMV_SWIGLU>), grid, block, lds, st, a);
            break;
        default:
            hipLaunchKernelGGL((gemv_kernel<T, GEMV_COMBINE>), grid, block, lds, st, a);
            break;
    }
    return launch_status();
}

// Two tokens take the matrix-vector path too: their 2 k pairs are walked like one token's k, with
// one output row per token (the kernel takes any number of tokens up to 64 pairs).  Every pair
// streams its expert's rows from memory -- the weight loads are non-temporal, and pairs of different
// tokens that chose the same expert are not neighbours -- so the step costs about 22 us per token
// on the 2048 / 5632 layer: 60 us at two tokens against 69 for the grouped GEMM, which streams
// each selected expert once, but 82 against 72 at three and 193 against 98 at eight.  Layers with
// a shared base (whose per-row products serve one token) keep the grouped GEMM.
constexpr int kMaxDecodeTokens = 2;
bool decode_supported(const moe_shape& s) {
    if (s.n_tokens == 1) return true;
    return s.n_tokens <= kMaxDecodeTokens && (long long)s.n_tokens * s.top_k <= kMaxExperts &&
           !(s.flags & MOE_FLAG_SHARED_BASE);
}

// scratch: h [P][F] fp32 (in the activation type once P F floats outgrow the L1), then (rank > 0) tg, tu, td [P][r] fp32
size_t decode_scratch_bytes(const moe_shape& s) {
    const size_t P = decode_supported(s) ? (size_t)s.n_tokens * s.top_k : (size_t)s.top_k;
    return round_up(sizeof(float) * P * ((size_t)s.d_ff + 3 * (size_t)s.rank), 256);
}

template <typename T>
static int decode_ffn_t(const moe_shape& s, const moe_weights& w, const void* x,
                        const int32_t* idx, const float* gate, void* y, void* scratch,
                        hipStream_t st, StageTimer* timer) {
    // k: all (token, slot) pairs of the step; kk of them per token.  One token: its input vector is
    // shared by every pair (vstride 0); several: pair p reads token p / kk's row (vdiv).
    const int d = s.d_model, F = s.d_ff, r = s.rank, kk = s.top_k, k = s.n_tokens * s.top_k;
    const int xs = s.n_tokens > 1 ? d : 0, xdiv = s.n_tokens > 1 ? kk : 0;
    const bool base = (r == 0) || (s.flags & MOE_FLAG_SHARED_BASE);
    const long long base_stride_gu = (r == 0) ? (long long)F * d : 0;  // shared base: stride 0
    float* h = static_cast<float*>(scratch);
    // The k hidden vectors are read by every wave of the down stage.  In fp32 they are twice the
    // bytes of the bf16 weight rows they meet, and once they outgrow the 32 KB of a CU's L1 every
    // one of those reads goes to L2; from that size on they are kept in the activation type
    // (the prefill path rounds h the same way).  Measured on the 2048 / 5632 layer: down stage
    // 13.9 us instead of 15.4; below that size the fp32 form is the faster one.
    const bool h_act = sizeof(T) == 2 && (size_t)k * F * sizeof(float) > 32 * 1024;
    float* tg = h + (size_t)k * F;
    float* tu = tg + (size_t)k * r;
    float* td = tu + (size_t)k * r;
    int rc;
    GemvArgs a;

    if (r > 0) {  // rank-r inputs of the gate and up factors: tg = R_g x, tu = R_u x
        a = GemvArgs{};
        a.nseg = 1;
        a.seg[0] = GemvSeg{w.rg, w.ru, (long long)r * d, x, x, 0, xs, d, xdiv};
        a.rows = r; a.k = k; a.kk = kk; a.E = s.n_experts; a.idx = idx; a.gate = gate; a.out0 = tg; a.out1 = tu;
        if ((rc = launch_gemv<T>(a, GEMV_DUAL, st)) != MOE_OK) return rc;
        stage_mark(timer, "gemv_rank_gate_up");
    }
    {  // hidden vector h_j = silu(M_gate x) * (M_up x)
        a = GemvArgs{};
        int ns = 0;
        if (base) a.seg[ns++] = GemvSeg{w.w_gate, w.w_up, base_stride_gu, x, x, 0, xs, d, xdiv};
        if (r > 0) a.seg[ns++] = GemvSeg{w.lg, w.lu, (long long)F * r, tg, tu, 1, r, r};
        a.nseg = ns;
        a.rows = F; a.k = k; a.kk = kk; a.E = s.n_experts; a.idx = idx; a.gate = gate; a.out0 = h;
        if (h_act) a.out0_act = h;
        if ((rc = launch_gemv<T>(a, GEMV_SWIGLU, st)) != MOE_OK) return rc;
        stage_mark(timer, "gemv_gate_up_swiglu");
    }
    if (r > 0) {  // td_j = R_d h_j
        a = GemvArgs{};
        a.nseg = 1;
        a.seg[0] = GemvSeg{w.rd, nullptr, (long long)r * F, h, h, h_act ? 0 : 1, F, F};
        a.rows = r; a.k = k; a.kk = kk; a.E = s.n_experts; a.idx = idx; a.gate = gate; a.out0 = td;
        if ((rc = launch_gemv<T>(a, GEMV_PLAIN, st)) != MOE_OK) return rc;
        stage_mark(timer, "gemv_rank_down");
    }
    {  // y = sum_j gate_j M_down h_j (+ x)
        a = GemvArgs{};
        int ns = 0;
        if (base) a.seg[ns++] = GemvSeg{w.w_down, nullptr, (r == 0) ? (long long)d * F : 0, h, h, h_act ? 0 : 1, F, F};
        if (r > 0) a.seg[ns++] = GemvSeg{w.ld, nullptr, (long long)d * r, td, td, 1, r, r};
        a.nseg = ns;
        a.rows = d; a.k = k; a.kk = kk; a.E = s.n_experts; a.idx = idx; a.gate = gate; a.y = y;
        a.residual = (s.flags & MOE_FLAG_RESIDUAL) ? x : nullptr;
        if ((rc = launch_gemv<T>(a, GEMV_COMBINE, st)) != MOE_OK) return rc;
        stage_mark(timer, "gemv_down_combine");
    }
    return MOE_OK;
}

int launch_decode_ffn(const moe_shape& s, const moe_weights& w, const void* x,
                      const int32_t* topk_idx, const float* topk_gate, void* y, void* scratch,
                      hipStream_t st, StageTimer* timer) {
    if (s.act_dtype == MOE_F32)
        return decode_ffn_t<float>(s, w, x, topk_idx, topk_gate, y, scratch, st, timer);
    return decode_ffn_t<bf16_t>(s, w, x, topk_idx, topk_gate, y, scratch, st, timer);
}

}  // namespace moe
