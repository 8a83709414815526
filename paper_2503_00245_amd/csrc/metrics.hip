// Routing-trace statistics the paper defines on the router's outputs:
//   - hard expert replacements H_e, H (Sec. 2.3, Eq. 4) and floor(H/2) of Eq. 5;
//   - the forward value of the block-wise expert selection loss (Eq. 4-7);
//   - set changes and expert loads under the offloading rule of Sec. 3.4.2;
//   - "Delta Uniform" (Sec. 3.2 metric list, Table 3, Fig. 6): per-layer divergence of the
//     realised expert balance from the uniform one, and its mean over layers.
// All integer work uses integer atomics (order-independent, hence deterministic); the one
// floating-point reduction (Eq. 6) sums fixed-size blocks in a fixed tree order and adds the
// block sums in index order in fp64.
#include "common.h"

namespace moe {

constexpr int kMetricThreads = 256;

// 64-bit mask of the experts selected for one token; entries outside [0, E) are dropped.
__device__ __forceinline__ unsigned long long expert_mask(const int32_t* __restrict__ s, int K,
                                                          int E) {
    unsigned long long m = 0;
    for (int j = 0; j < K; ++j) {
        const int e = s[j];
        if ((unsigned)e < (unsigned)E) m |= 1ull << e;
    }
    return m;
}

__global__ void zero_u64_kernel(unsigned long long* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// one thread per adjacent token pair (b, t), t < T-1; H_e += [e in S(b,t+1)] xor [e in S(b,t)]
__global__ __launch_bounds__(kMetricThreads) void replacements_kernel(
    const int32_t* __restrict__ S, int B, int T, int K, int E, unsigned long long* __restrict__ He) {
    __shared__ int s_cnt[kMaxExperts];
    if (threadIdx.x < kMaxExperts) s_cnt[threadIdx.x] = 0;
    __syncthreads();
    const long long npairs = (long long)B * (T - 1);
    const long long i = (long long)blockIdx.x * kMetricThreads + threadIdx.x;
    if (i < npairs) {
        const long long b = i / (T - 1), t = i % (T - 1);
        const int32_t* s0 = S + (b * T + t) * K;
        unsigned long long diff = expert_mask(s0, K, E) ^ expert_mask(s0 + K, K, E);
        while (diff) {
            const int e = __ffsll((long long)diff) - 1;
            atomicAdd(&s_cnt[e], 1);
            diff &= diff - 1;
        }
    }
    __syncthreads();
    if (threadIdx.x < E && s_cnt[threadIdx.x])
        atomicAdd(&He[threadIdx.x], (unsigned long long)s_cnt[threadIdx.x]);
}

__global__ void sum_replacements_kernel(const unsigned long long* __restrict__ He, int E,
                                        unsigned long long* __restrict__ H) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        unsigned long long h = 0;
        for (int e = 0; e < E; ++e) h += He[e];
        *H = h;
    }
}

// block partial sums of |W[b,t+1,e] - W[b,t,e]| over the flattened (b, t < T-1, e) index
__global__ __launch_bounds__(kMetricThreads) void soft_partial_kernel(
    const float* __restrict__ W, int B, int T, int E, float* __restrict__ partial) {
    __shared__ float s_sum[kMetricThreads];
    const long long n = (long long)B * (T - 1) * E;
    const long long i = (long long)blockIdx.x * kMetricThreads + threadIdx.x;
    float v = 0.f;
    if (i < n) {
        const long long row = i / E;  // (b, t) with t < T-1
        const int e = (int)(i % E);
        const long long b = row / (T - 1), t = row % (T - 1);
        const float* w0 = W + (b * T + t) * E + e;
        v = fabsf(w0[E] - w0[0]);
    }
    s_sum[threadIdx.x] = v;
    __syncthreads();
    for (int off = kMetricThreads / 2; off > 0; off >>= 1) {
        if (threadIdx.x < off) s_sum[threadIdx.x] += s_sum[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[blockIdx.x] = s_sum[0];
}

// out = {H, H_norm, L, L_norm, loss} (Eq. 5, 6, 7)
__global__ void bles_finalize_kernel(const float* __restrict__ partial, int nblocks,
                                     const unsigned long long* __restrict__ H, int B, int T, int K,
                                     double* __restrict__ out) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    double L = 0.0;
    for (int i = 0; i < nblocks; ++i) L += (double)partial[i];
    const double h = (double)*H;
    const double Hn = T > 1 ? (double)(*H / 2) / ((double)B * K * (T - 1)) : 0.0;
    const double Ln = L / ((double)B * T);
    out[0] = h;
    out[1] = Hn;
    out[2] = L;
    out[3] = Ln;
    out[4] = Hn * Ln;
}

// one workgroup per layer: adjacent-token set comparisons (the resident set after token t is
// always S_t, so the rule's state is just the previous token's selection)
__global__ __launch_bounds__(kMetricThreads) void offload_kernel(
    const int32_t* __restrict__ trace, int T, int K, int E, unsigned long long* __restrict__ changes,
    unsigned long long* __restrict__ loads) {
    __shared__ int s_ch, s_ld;
    if (threadIdx.x == 0) {
        s_ch = 0;
        s_ld = 0;
    }
    __syncthreads();
    const int32_t* tr = trace + (size_t)blockIdx.x * T * K;
    int ch = 0, ld = 0;
    for (int t = threadIdx.x; t < T; t += kMetricThreads) {
        const unsigned long long cur = expert_mask(tr + (size_t)t * K, K, E);
        const unsigned long long prev = t > 0 ? expert_mask(tr + (size_t)(t - 1) * K, K, E) : 0ull;
        if (cur != prev) {
            ch += 1;
            ld += __popcll(cur & ~prev);
        }
    }
    atomicAdd(&s_ch, ch);
    atomicAdd(&s_ld, ld);
    __syncthreads();
    if (threadIdx.x == 0) {
        changes[blockIdx.x] = (unsigned long long)s_ch;
        loads[blockIdx.x] = (unsigned long long)s_ld;
    }
}

// counts[l][e] += pairs of layer l that chose expert e (grid: x = token chunks, y = layers)
__global__ __launch_bounds__(kMetricThreads) void balance_count_kernel(
    const int32_t* __restrict__ trace, int TK, int E, unsigned long long* __restrict__ counts) {
    __shared__ int s_cnt[kMaxExperts];
    if (threadIdx.x < kMaxExperts) s_cnt[threadIdx.x] = 0;
    __syncthreads();
    const int32_t* tr = trace + (size_t)blockIdx.y * TK;
    const int stride = gridDim.x * kMetricThreads;
    for (int i = blockIdx.x * kMetricThreads + threadIdx.x; i < TK; i += stride) {
        const int e = tr[i];
        if ((unsigned)e < (unsigned)E) atomicAdd(&s_cnt[e], 1);
    }
    __syncthreads();
    if (threadIdx.x < E && s_cnt[threadIdx.x])
        atomicAdd(&counts[(size_t)blockIdx.y * E + threadIdx.x], (unsigned long long)s_cnt[threadIdx.x]);
}

// delta[l] = sum_e | counts[l][e] / (T K) - 1/E |, summed in ascending e; mean = (sum_l delta[l]) / L
// in ascending l.  One thread: L E terms of fp64.
__global__ void balance_finalize_kernel(const unsigned long long* __restrict__ counts, int L, int TK,
                                        int E, double* __restrict__ delta, double* __restrict__ mean) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    double total = 0.0;
    for (int l = 0; l < L; ++l) {
        double dl = 0.0;
        for (int e = 0; e < E; ++e) {
            const double dev = (double)counts[(size_t)l * E + e] / (double)TK - 1.0 / (double)E;
            dl += dev < 0 ? -dev : dev;
        }
        if (delta) delta[l] = dl;
        total += dl;
    }
    *mean = total / (double)L;
}

static int launch_replacements(const int32_t* S, int B, int T, int K, int E, unsigned long long* He,
                               unsigned long long* H, hipStream_t st) {
    hipLaunchKernelGGL(zero_u64_kernel, dim3(1), dim3(kMaxExperts), 0, st, He, E);
    const long long npairs = (long long)B * (T - 1);
    if (npairs > 0) {
        const int grid = (int)((npairs + kMetricThreads - 1) / kMetricThreads);
        hipLaunchKernelGGL(replacements_kernel, dim3(grid), dim3(kMetricThreads), 0, st, S, B, T, K, E,
                           He);
    }
    hipLaunchKernelGGL(sum_replacements_kernel, dim3(1), dim3(64), 0, st, He, E, H);
    return launch_status();
}

}  // namespace moe

using namespace moe;

static int check_trace_shape(int B, int T, int K, int E) {
    if (B < 1 || T < 1 || K < 1 || E < 1 || K > E) return MOE_ERR_INVALID;
    if (E > kMaxExperts) return MOE_ERR_UNSUPPORTED;
    if ((long long)B * T * (long long)(E > K ? E : K) >= (1ll << 31)) return MOE_ERR_UNSUPPORTED;
    return MOE_OK;
}

extern "C" {

int moe_expert_replacements(const int32_t* S, int32_t B, int32_t T, int32_t K, int32_t E,
                            int64_t* H_e, int64_t* H, void* stream) {
    int rc = check_trace_shape(B, T, K, E);
    if (rc != MOE_OK) return rc;
    if (!S || !H_e || !H) return MOE_ERR_INVALID;
    return launch_replacements(S, B, T, K, E, reinterpret_cast<unsigned long long*>(H_e),
                               reinterpret_cast<unsigned long long*>(H), as_stream(stream));
}

size_t moe_bles_workspace_bytes(int32_t B, int32_t T, int32_t E) {
    if (check_trace_shape(B, T, 1, E) != MOE_OK) return 0;
    const long long n = (long long)B * (T > 1 ? T - 1 : 0) * E;
    const size_t nblocks = (size_t)((n + kMetricThreads - 1) / kMetricThreads);
    // [E+1] u64 replacement counters, then one float per block
    return round_up(sizeof(unsigned long long) * (kMaxExperts + 1), 256) +
           round_up(sizeof(float) * (nblocks ? nblocks : 1), 256);
}

int moe_bles_loss(const float* probs, const int32_t* S, int32_t B, int32_t T, int32_t K, int32_t E,
                  double* out, void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_trace_shape(B, T, K, E);
    if (rc != MOE_OK) return rc;
    if (!probs || !S || !out) return MOE_ERR_INVALID;
    if (!workspace || workspace_bytes < moe_bles_workspace_bytes(B, T, E)) return MOE_ERR_WORKSPACE;
    hipStream_t st = as_stream(stream);
    unsigned long long* He = static_cast<unsigned long long*>(workspace);
    unsigned long long* H = He + kMaxExperts;
    float* partial = reinterpret_cast<float*>(static_cast<char*>(workspace) +
                                              round_up(sizeof(unsigned long long) * (kMaxExperts + 1), 256));
    rc = launch_replacements(S, B, T, K, E, He, H, st);
    if (rc != MOE_OK) return rc;
    const long long n = (long long)B * (T - 1) * E;
    const int nblocks = (int)((n + kMetricThreads - 1) / kMetricThreads);
    if (nblocks > 0)
        hipLaunchKernelGGL(soft_partial_kernel, dim3(nblocks), dim3(kMetricThreads), 0, st, probs, B, T,
                           E, partial);
    hipLaunchKernelGGL(bles_finalize_kernel, dim3(1), dim3(64), 0, st, partial, nblocks, H, B, T, K,
                       out);
    return launch_status();
}

int moe_offload_counters(const int32_t* trace, int32_t L, int32_t T, int32_t K, int32_t E,
                         int64_t* changes, int64_t* loads, void* stream) {
    int rc = check_trace_shape(L, T, K, E);
    if (rc != MOE_OK) return rc;
    if (!trace || !changes || !loads) return MOE_ERR_INVALID;
    hipLaunchKernelGGL(offload_kernel, dim3(L), dim3(kMetricThreads), 0, as_stream(stream), trace, T,
                       K, E, reinterpret_cast<unsigned long long*>(changes),
                       reinterpret_cast<unsigned long long*>(loads));
    return launch_status();
}

int moe_delta_uniform(const int32_t* trace, int32_t L, int32_t T, int32_t K, int32_t E,
                      int64_t* counts, double* delta, double* mean, void* stream) {
    int rc = check_trace_shape(L, T, K, E);
    if (rc != MOE_OK) return rc;
    if (!trace || !counts || !mean) return MOE_ERR_INVALID;
    if ((long long)L * E >= (1ll << 31)) return MOE_ERR_UNSUPPORTED;
    hipStream_t st = as_stream(stream);
    unsigned long long* cnt = reinterpret_cast<unsigned long long*>(counts);
    const int n = L * E;
    hipLaunchKernelGGL(zero_u64_kernel, dim3((n + kMetricThreads - 1) / kMetricThreads), dim3(kMetricThreads), 0,
                       st, cnt, n);
    const int TK = T * K;  // < 2^31 by check_trace_shape
    const int chunks = min(64, (TK + 4 * kMetricThreads - 1) / (4 * kMetricThreads));
    hipLaunchKernelGGL(balance_count_kernel, dim3(chunks, L), dim3(kMetricThreads), 0, st, trace, TK, E, cnt);
    hipLaunchKernelGGL(balance_finalize_kernel, dim3(1), dim3(64), 0, st, cnt, L, TK, E, delta, mean);
    return launch_status();
}

}  // extern "C"
