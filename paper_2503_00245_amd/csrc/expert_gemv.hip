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
// Input vectors are staged once per workgroup in LDS as fp32; a wave reads a matrix row
// with 16-byte loads, 1 KB per instruction, and reduces with a 64-lane butterfly.
#include "common.h"

namespace moe {

enum { GEMV_PLAIN = 0, GEMV_DUAL = 1, GEMV_SWIGLU = 2, GEMV_COMBINE = 3 };
constexpr int kGemvThreads = 512;
constexpr int kGemvWaves = kGemvThreads / kWave;
constexpr size_t kGemvMaxLds = 64 * 1024;

struct GemvSeg {
    const void* W0;      // [Eb, rows, n]
    const void* W1;      // second matrix (DUAL / SWIGLU), same shape
    long long stride;    // elements between experts; 0 = one matrix shared by all experts
    const void* v0;      // input vector(s): [n] if vstride == 0, else [k][n]
    const void* v1;      // input of the second product (may equal v0)
    int v_is_f32;        // 1: fp32 scratch vector; 0: stored in the activation type
    int vstride;         // elements between pairs' vectors; 0 = same vector for every pair
    int n;               // row length
};

struct GemvArgs {
    GemvSeg seg[2];
    int nseg;
    int rows;
    int k;
    int rows_per_wave;
    int E;
    const int32_t* idx;   // [k] selected experts
    const float* gate;    // [k]
    float* out0;          // [k][rows]
    float* out1;          // [k][rows] (DUAL)
    void* y;              // [rows] activation type (COMBINE)
    const void* residual; // [rows] or NULL (COMBINE)
};

template <typename T>
__device__ __forceinline__ float row_dot(const T* __restrict__ wrow, const float* v, int n,
                                         int lane) {
    typedef Store<T> S;
    constexpr int VEC = S::VEC;
    float acc = 0.f;
#pragma unroll 4
    for (int c = lane * VEC; c < n; c += kWave * VEC) {
        const typename S::vec_t w =
            __builtin_nontemporal_load(reinterpret_cast<const typename S::vec_t*>(wrow + c));
#pragma unroll
        for (int q = 0; q < VEC; q += 4) {
            const f32x4 vv = *reinterpret_cast<const f32x4*>(v + c + q);
            acc = fmaf(S::get(w, q + 0), vv[0], acc);
            acc = fmaf(S::get(w, q + 1), vv[1], acc);
            acc = fmaf(S::get(w, q + 2), vv[2], acc);
            acc = fmaf(S::get(w, q + 3), vv[3], acc);
        }
    }
    return acc;
}

template <typename T>
__device__ __forceinline__ float load_vec_elem(const void* v, int is_f32, size_t i) {
    return is_f32 ? static_cast<const float*>(v)[i] : Store<T>::to_f32(static_cast<const T*>(v)[i]);
}

template <typename T, int MODE>
__global__ __launch_bounds__(kGemvThreads) void gemv_kernel(const GemvArgs a) {
    extern __shared__ __align__(16) float lds[];
    constexpr bool DUAL = (MODE == GEMV_DUAL || MODE == GEMV_SWIGLU);
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int k = a.k;

    // ---- stage the input vectors ------------------------------------------------------------
    const float* sv0[2];
    const float* sv1[2];
    bool once[2];  // segment evaluated once per row (shared matrix and one effective vector)
    {
        float* cur = lds;
        for (int s = 0; s < a.nseg; ++s) {
            const GemvSeg& g = a.seg[s];
            const bool premix = (MODE == GEMV_COMBINE) && g.stride == 0 && g.vstride != 0;
            once[s] = g.stride == 0 && (g.vstride == 0 || premix);
            const int nv = (g.vstride == 0 || premix) ? 1 : k;
            sv0[s] = cur;
            if (premix) {
                for (int i = threadIdx.x; i < g.n; i += kGemvThreads) {
                    float m = 0.f;
                    for (int j = 0; j < k; ++j)
                        m = fmaf(a.gate[j], load_vec_elem<T>(g.v0, g.v_is_f32, (size_t)j * g.vstride + i), m);
                    cur[i] = m;
                }
            } else {
                for (int i = threadIdx.x; i < nv * g.n; i += kGemvThreads) {
                    const int j = i / g.n;
                    cur[i] = load_vec_elem<T>(g.v0, g.v_is_f32, (size_t)j * g.vstride + (i - j * g.n));
                }
            }
            cur += nv * g.n;
            sv1[s] = sv0[s];
            if (DUAL && g.v1 != g.v0) {
                sv1[s] = cur;
                for (int i = threadIdx.x; i < nv * g.n; i += kGemvThreads) {
                    const int j = i / g.n;
                    cur[i] = load_vec_elem<T>(g.v1, g.v_is_f32, (size_t)j * g.vstride + (i - j * g.n));
                }
                cur += nv * g.n;
            }
        }
    }
    __syncthreads();

    const int gw = blockIdx.x * kGemvWaves + wave;
    const int row_end = min(a.rows, (gw + 1) * a.rows_per_wave);
    for (int row = gw * a.rows_per_wave; row < row_end; ++row) {
        // segments read once per row
        float sh0 = 0.f, sh1 = 0.f;
        for (int s = 0; s < a.nseg; ++s) {
            if (!once[s]) continue;
            const GemvSeg& g = a.seg[s];
            sh0 += row_dot<T>(static_cast<const T*>(g.W0) + (size_t)row * g.n, sv0[s], g.n, lane);
            if (DUAL)
                sh1 += row_dot<T>(static_cast<const T*>(g.W1) + (size_t)row * g.n, sv1[s], g.n, lane);
        }
        float total = (MODE == GEMV_COMBINE) ? wave_sum(sh0) : 0.f;
        for (int j = 0; j < k; ++j) {
            const int e = min(max(a.idx[j], 0), a.E - 1);
            float acc0 = (MODE == GEMV_COMBINE) ? 0.f : sh0;
            float acc1 = sh1;
            for (int s = 0; s < a.nseg; ++s) {
                if (once[s]) continue;
                const GemvSeg& g = a.seg[s];
                const size_t woff = (size_t)e * g.stride + (size_t)row * g.n;
                const int voff = g.vstride ? j * g.n : 0;
                acc0 += row_dot<T>(static_cast<const T*>(g.W0) + woff, sv0[s] + voff, g.n, lane);
                if (DUAL)
                    acc1 += row_dot<T>(static_cast<const T*>(g.W1) + woff, sv1[s] + voff, g.n, lane);
            }
            acc0 = wave_sum(acc0);
            if (DUAL) acc1 = wave_sum(acc1);
            if (MODE == GEMV_COMBINE) {
                total = fmaf(a.gate[j], acc0, total);
            } else if (lane == 0) {
                if (MODE == GEMV_SWIGLU) {
                    a.out0[(size_t)j * a.rows + row] = silu_f32(acc0) * acc1;
                } else {
                    a.out0[(size_t)j * a.rows + row] = acc0;
                    if (MODE == GEMV_DUAL) a.out1[(size_t)j * a.rows + row] = acc1;
                }
            }
        }
        if (MODE == GEMV_COMBINE && lane == 0) {
            if (a.residual) total += Store<T>::to_f32(static_cast<const T*>(a.residual)[row]);
            static_cast<T*>(a.y)[row] = Store<T>::from_f32(total);
        }
    }
}

static size_t gemv_lds_bytes(const GemvArgs& a, int mode) {
    size_t fl = 0;
    for (int s = 0; s < a.nseg; ++s) {
        const GemvSeg& g = a.seg[s];
        const bool premix = mode == GEMV_COMBINE && g.stride == 0 && g.vstride != 0;
        const size_t nv = (g.vstride == 0 || premix) ? 1 : (size_t)a.k;
        const bool dual = (mode == GEMV_DUAL || mode == GEMV_SWIGLU) && g.v1 != g.v0;
        fl += nv * (size_t)g.n * (dual ? 2 : 1);
    }
    return fl * sizeof(float);
}

template <typename T>
static int launch_gemv(GemvArgs& a, int mode, hipStream_t st) {
    const size_t lds = gemv_lds_bytes(a, mode);
    if (lds > kGemvMaxLds) return MOE_ERR_UNSUPPORTED;
    // about four workgroups per CU of work, at least one row per wave
    const int target_waves = 4 * 256 * kGemvWaves;
    a.rows_per_wave = max(1, min(8, (a.rows + target_waves - 1) / target_waves));
    const int waves = (a.rows + a.rows_per_wave - 1) / a.rows_per_wave;
    dim3 grid((waves + kGemvWaves - 1) / kGemvWaves), block(kGemvThreads);
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

// scratch: h [k][F] fp32, then (rank > 0) tg, tu, td [k][r] fp32
size_t decode_scratch_bytes(const moe_shape& s) {
    const size_t k = s.top_k;
    return round_up(sizeof(float) * k * ((size_t)s.d_ff + 3 * (size_t)s.rank), 256);
}

bool decode_supported(const moe_shape& s) {
    if (s.n_tokens != 1) return false;
    // the largest LDS stage: COMBINE holds k hidden vectors (+ k rank vectors)
    const size_t k = s.top_k;
    size_t worst = k * ((size_t)s.d_ff + s.rank);
    const size_t swiglu = (size_t)s.d_model + 2 * k * (size_t)s.rank;
    if (swiglu > worst) worst = swiglu;
    return worst * sizeof(float) <= kGemvMaxLds;
}

template <typename T>
static int decode_ffn_t(const moe_shape& s, const moe_weights& w, const void* x,
                        const int32_t* idx, const float* gate, void* y, void* scratch,
                        hipStream_t st, StageTimer* timer) {
    const int d = s.d_model, F = s.d_ff, r = s.rank, k = s.top_k;
    const bool base = (r == 0) || (s.flags & MOE_FLAG_SHARED_BASE);
    const long long base_stride_gu = (r == 0) ? (long long)F * d : 0;  // shared base: stride 0
    float* h = static_cast<float*>(scratch);
    float* tg = h + (size_t)k * F;
    float* tu = tg + (size_t)k * r;
    float* td = tu + (size_t)k * r;
    int rc;
    GemvArgs a;

    if (r > 0) {  // rank-r inputs of the gate and up factors: tg = R_g x, tu = R_u x
        a = GemvArgs{};
        a.nseg = 1;
        a.seg[0] = GemvSeg{w.rg, w.ru, (long long)r * d, x, x, 0, 0, d};
        a.rows = r; a.k = k; a.E = s.n_experts; a.idx = idx; a.gate = gate; a.out0 = tg; a.out1 = tu;
        if ((rc = launch_gemv<T>(a, GEMV_DUAL, st)) != MOE_OK) return rc;
        stage_mark(timer, "gemv_rank_gate_up");
    }
    {  // hidden vector h_j = silu(M_gate x) * (M_up x)
        a = GemvArgs{};
        int ns = 0;
        if (base) a.seg[ns++] = GemvSeg{w.w_gate, w.w_up, base_stride_gu, x, x, 0, 0, d};
        if (r > 0) a.seg[ns++] = GemvSeg{w.lg, w.lu, (long long)F * r, tg, tu, 1, r, r};
        a.nseg = ns;
        a.rows = F; a.k = k; a.E = s.n_experts; a.idx = idx; a.gate = gate; a.out0 = h;
        if ((rc = launch_gemv<T>(a, GEMV_SWIGLU, st)) != MOE_OK) return rc;
        stage_mark(timer, "gemv_gate_up_swiglu");
    }
    if (r > 0) {  // td_j = R_d h_j
        a = GemvArgs{};
        a.nseg = 1;
        a.seg[0] = GemvSeg{w.rd, nullptr, (long long)r * F, h, h, 1, F, F};
        a.rows = r; a.k = k; a.E = s.n_experts; a.idx = idx; a.gate = gate; a.out0 = td;
        if ((rc = launch_gemv<T>(a, GEMV_PLAIN, st)) != MOE_OK) return rc;
        stage_mark(timer, "gemv_rank_down");
    }
    {  // y = sum_j gate_j M_down h_j (+ x)
        a = GemvArgs{};
        int ns = 0;
        if (base) a.seg[ns++] = GemvSeg{w.w_down, nullptr, (r == 0) ? (long long)d * F : 0, h, h, 1, F, F};
        if (r > 0) a.seg[ns++] = GemvSeg{w.ld, nullptr, (long long)d * r, td, td, 1, r, r};
        a.nseg = ns;
        a.rows = d; a.k = k; a.E = s.n_experts; a.idx = idx; a.gate = gate; a.y = y;
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
