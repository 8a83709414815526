// Dispatch of (token, slot) pairs into per-expert groups: an LDS-staged, stable counting
// sort by expert index (token-choice routing, Sec. 2.1 / Fig. 2: every token goes to its
// own k experts, so each expert ends up with a contiguous, order-preserving group).
//
// Pairs are cut into chunks of kChunk consecutive p.  Chunk c, expert e:
//   count[e][c] (histogram)  ->  base[e][c] = exclusive scan in (e major, c minor) order
//   slot(p) = base[key][chunk] + #{p' < p in the chunk with the same key}
// The in-chunk rank comes from wave ballots (lanes below me with my key) plus per-wave
// counts held in LDS, so equal keys keep ascending p: the sort is stable by construction.
// Small problems (one chunk) run all three phases in a single workgroup.
#include "common.h"

namespace moe {

constexpr int kSortThreads = 1024;
constexpr int kSortWaves = kSortThreads / kWave;
constexpr int kChunk = 8192;  // pairs per workgroup in the multi-block path

// In-wave stable rank: returns #lanes below this one holding the same key, and adds the
// wave's per-key totals to s_wcount[wave][key].  Inactive lanes pass key = -1.
__device__ __forceinline__ int wave_rank(int key, int lane, int* wcount_row) {
    int rank = 0;
    unsigned long long pending = __ballot(key >= 0);
    while (pending) {
        const int leader = __ffsll((long long)pending) - 1;
        const int lk = __shfl(key, leader, kWave);
        const unsigned long long same = __ballot(key == lk);
        if (key == lk) rank = __popcll(same & ((1ull << lane) - 1ull));
        if (lane == leader) wcount_row[lk] = __popcll(same);
        pending &= ~same;
    }
    return rank;
}

// Key of pair p, or -1 for p outside [0, n) and for values outside [0, E) (which the
// contract forbids; dropping them keeps every LDS and global index in range).
__device__ __forceinline__ int load_key(const int32_t* __restrict__ keys, int p, int n, int E) {
    if (p >= n) return -1;
    const int key = keys[p];
    return (unsigned)key < (unsigned)E ? key : -1;
}

// Adds this wave's per-key totals to hist (LDS): one atomic per distinct key per wave.
__device__ __forceinline__ void wave_hist(int key, int lane, int* hist) {
    unsigned long long pending = __ballot(key >= 0);
    while (pending) {
        const int leader = __ffsll((long long)pending) - 1;
        const int lk = __shfl(key, leader, kWave);
        const unsigned long long same = __ballot(key == lk);
        if (lane == leader) atomicAdd(&hist[lk], __popcll(same));
        pending &= ~same;
    }
}

// Scatter one chunk [p0, p1) given running per-expert bases in s_run (LDS, updated in place).
__device__ void scatter_chunk(const int32_t* __restrict__ keys, int p0, int p1, int E,
                              int* s_run, int (*s_wcount)[kMaxExperts],
                              int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    for (int q0 = p0; q0 < p1; q0 += kSortThreads) {
        for (int i = threadIdx.x; i < kSortWaves * kMaxExperts; i += kSortThreads)
            (&s_wcount[0][0])[i] = 0;
        __syncthreads();
        const int p = q0 + threadIdx.x;
        const int key = load_key(keys, p, p1, E);
        const int rank = wave_rank(key, lane, s_wcount[wave]);
        __syncthreads();
        if (key >= 0) {
            int before = 0;
            for (int w = 0; w < wave; ++w) before += s_wcount[w][key];
            const int slot = s_run[key] + before + rank;
            perm[slot] = p;
            inv_perm[p] = slot;
        }
        __syncthreads();
        if (threadIdx.x < E) {
            int tot = 0;
            for (int w = 0; w < kSortWaves; ++w) tot += s_wcount[w][threadIdx.x];
            s_run[threadIdx.x] += tot;
        }
        __syncthreads();
    }
}

// ---- single-workgroup path (P <= kChunk): keys stay in registers ---------------------------
// Pass q covers pairs [q*1024, (q+1)*1024).  One sweep gives every pair its in-wave rank and
// every (pass, wave, expert) its count; a wave-level scan per expert over the 128 (pass, wave)
// cells turns counts into bases, a 64-lane scan of the expert totals gives the offsets, and
// slot = offset[e] + base[pass][wave][e] + rank.  Three barriers in all.
constexpr int kSmallPasses = kChunk / kSortThreads;

__device__ __forceinline__ int wave_inclusive_scan(int v, int lane) {
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int o = __shfl_up(v, d, kWave);
        if (lane >= d) v += o;
    }
    return v;
}

__global__ __launch_bounds__(kSortThreads) void permute_small_kernel(
    const int32_t* __restrict__ keys, int P, int E, int32_t* __restrict__ offsets,
    int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm) {
    __shared__ int s_cnt[kSmallPasses * kSortWaves][kMaxExperts];  // [pass*16 + wave][expert]
    __shared__ int s_total[kMaxExperts];
    __shared__ int s_off[kMaxExperts];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int npass = (P + kSortThreads - 1) / kSortThreads;
    constexpr int kCells = kSmallPasses * kSortWaves;  // 128 = two per lane

    for (int i = threadIdx.x; i < kCells * kMaxExperts; i += kSortThreads) (&s_cnt[0][0])[i] = 0;
    __syncthreads();
    int key[kSmallPasses], rank[kSmallPasses];
#pragma unroll
    for (int q = 0; q < kSmallPasses; ++q) {
        key[q] = -1;
        rank[q] = 0;
        if (q < npass) {
            key[q] = load_key(keys, q * kSortThreads + threadIdx.x, P, E);
            rank[q] = wave_rank(key[q], lane, s_cnt[q * kSortWaves + wave]);
        }
    }
    __syncthreads();
    for (int e = wave; e < E; e += kSortWaves) {
        const int v0 = s_cnt[lane][e], v1 = s_cnt[lane + kWave][e];
        const int i0 = wave_inclusive_scan(v0, lane);
        const int t0 = __shfl(i0, kWave - 1, kWave);
        const int i1 = wave_inclusive_scan(v1, lane) + t0;
        s_cnt[lane][e] = i0 - v0;
        s_cnt[lane + kWave][e] = i1 - v1;
        if (lane == kWave - 1) s_total[e] = i1;
    }
    __syncthreads();
    if (wave == 0) {
        const int tot = lane < E ? s_total[lane] : 0;
        const int excl = wave_inclusive_scan(tot, lane) - tot;
        if (lane < E) {
            s_off[lane] = excl;
            offsets[lane] = excl;
        }
        if (lane == E - 1) offsets[E] = excl + tot;
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < kSmallPasses; ++q) {
        if (key[q] >= 0) {
            const int p = q * kSortThreads + threadIdx.x;
            const int slot = s_off[key[q]] + s_cnt[q * kSortWaves + wave][key[q]] + rank[q];
            perm[slot] = p;
            inv_perm[p] = slot;
        }
    }
}

// ---- multi-workgroup path ---------------------------------------------------------------------
__global__ __launch_bounds__(kSortThreads) void permute_hist_kernel(
    const int32_t* __restrict__ keys, int P, int E, int n_chunks, int32_t* __restrict__ counts) {
    __shared__ int s_hist[kMaxExperts];
    if (threadIdx.x < kMaxExperts) s_hist[threadIdx.x] = 0;
    __syncthreads();
    const int p0 = blockIdx.x * kChunk;
    const int p1 = min(P, p0 + kChunk);
    for (int q = p0; q < p1; q += kSortThreads)
        wave_hist(load_key(keys, q + threadIdx.x, p1, E), threadIdx.x & (kWave - 1), s_hist);
    __syncthreads();
    if (threadIdx.x < E) counts[(size_t)threadIdx.x * n_chunks + blockIdx.x] = s_hist[threadIdx.x];
}

// exclusive scan of counts[e][c] in row-major order, in place; also the expert offsets
__global__ __launch_bounds__(kSortThreads) void permute_scan_kernel(
    int32_t* __restrict__ counts, int n, int E, int n_chunks, int P,
    int32_t* __restrict__ offsets) {
    __shared__ int s_part[kSortThreads];
    const int per = (n + kSortThreads - 1) / kSortThreads;
    const int i0 = min(n, (int)threadIdx.x * per);
    const int i1 = min(n, i0 + per);
    int sum = 0;
    for (int i = i0; i < i1; ++i) sum += counts[i];
    s_part[threadIdx.x] = sum;
    __syncthreads();
    // Hillis-Steele inclusive scan over the per-thread partials
    for (int off = 1; off < kSortThreads; off <<= 1) {
        int v = threadIdx.x >= off ? s_part[threadIdx.x - off] : 0;
        __syncthreads();
        s_part[threadIdx.x] += v;
        __syncthreads();
    }
    int run = s_part[threadIdx.x] - sum;
    for (int i = i0; i < i1; ++i) {
        const int c = counts[i];
        counts[i] = run;
        if (i % n_chunks == 0) offsets[i / n_chunks] = run;
        run += c;
    }
    if (threadIdx.x == 0) offsets[E] = P;
}

__global__ __launch_bounds__(kSortThreads) void permute_scatter_kernel(
    const int32_t* __restrict__ keys, int P, int E, int n_chunks,
    const int32_t* __restrict__ base, int32_t* __restrict__ perm,
    int32_t* __restrict__ inv_perm) {
    __shared__ int s_run[kMaxExperts];
    __shared__ int s_wcount[kSortWaves][kMaxExperts];
    if (threadIdx.x < E) s_run[threadIdx.x] = base[(size_t)threadIdx.x * n_chunks + blockIdx.x];
    __syncthreads();
    const int p0 = blockIdx.x * kChunk;
    scatter_chunk(keys, p0, min(P, p0 + kChunk), E, s_run, s_wcount, perm, inv_perm);
}

size_t permute_scratch_bytes(int P, int E) {
    const size_t n_chunks = ((size_t)P + kChunk - 1) / kChunk;
    return round_up(sizeof(int32_t) * n_chunks * (size_t)E, 256);
}

int launch_permute(int P, int E, const int32_t* topk_idx, int32_t* offsets, int32_t* perm,
                   int32_t* inv_perm, void* scratch, hipStream_t st) {
    if (P <= kChunk) {
        hipLaunchKernelGGL(permute_small_kernel, dim3(1), dim3(kSortThreads), 0, st, topk_idx, P, E,
                           offsets, perm, inv_perm);
        return launch_status();
    }
    const int n_chunks = (P + kChunk - 1) / kChunk;
    int32_t* counts = static_cast<int32_t*>(scratch);
    hipLaunchKernelGGL(permute_hist_kernel, dim3(n_chunks), dim3(kSortThreads), 0, st, topk_idx, P,
                       E, n_chunks, counts);
    hipLaunchKernelGGL(permute_scan_kernel, dim3(1), dim3(kSortThreads), 0, st, counts,
                       E * n_chunks, E, n_chunks, P, offsets);
    hipLaunchKernelGGL(permute_scatter_kernel, dim3(n_chunks), dim3(kSortThreads), 0, st, topk_idx,
                       P, E, n_chunks, counts, perm, inv_perm);
    return launch_status();
}

// x_perm[s,:] = x[perm[s] / k, :]   (16-byte copies; one workgroup per sorted row)
__global__ __launch_bounds__(256) void gather_rows_kernel(const uint4* __restrict__ x,
                                                          const int32_t* __restrict__ perm,
                                                          uint4* __restrict__ x_perm, int k,
                                                          int row_vec, int P) {
    const int s = blockIdx.x;
    const int p = min(max(perm[s], 0), P - 1);  // stays in range even on a malformed perm
    const size_t src = (size_t)(p / k) * row_vec;
    for (int i = threadIdx.x; i < row_vec; i += blockDim.x)
        x_perm[(size_t)s * row_vec + i] = x[src + i];
}

int launch_gather_rows(const moe_shape& s, const int32_t* perm, const void* x, void* x_perm,
                       hipStream_t st) {
    const int P = s.n_tokens * s.top_k;
    if (P == 0) return MOE_OK;
    const int row_vec = (int)((size_t)s.d_model * elt_size(s.act_dtype) / 16);
    hipLaunchKernelGGL(gather_rows_kernel, dim3(P), dim3(256), 0, st, (const uint4*)x, perm,
                       (uint4*)x_perm, s.top_k, row_vec, P);
    return launch_status();
}

}  // namespace moe
