// Shared device/host helpers of the gfx950 MoE library (internal; not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "moe.h"

namespace moe {

constexpr int kWave = 64;        // CDNA wavefront width
constexpr int kMaxExperts = 64;  // one lane per expert in the router's selection step

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// ---- storage-type traits: VEC elements per 16-byte load -------------------------------
template <typename T>
struct Store;
template <>
struct Store<float> {
    static constexpr int VEC = 4;
    typedef f32x4 vec_t;
    static __device__ __forceinline__ float get(const vec_t& v, int i) { return v[i]; }
    static __device__ __forceinline__ float to_f32(float v) { return v; }
    static __device__ __forceinline__ float from_f32(float v) { return v; }
};
template <>
struct Store<bf16_t> {
    static constexpr int VEC = 8;
    typedef bf16x8 vec_t;
    static __device__ __forceinline__ float get(const vec_t& v, int i) { return (float)v[i]; }
    static __device__ __forceinline__ float to_f32(bf16_t v) { return (float)v; }
    static __device__ __forceinline__ bf16_t from_f32(float v) { return (bf16_t)v; }  // RNE
};

// ---- wavefront reductions: every lane gets the result --------------------------------------
// Within a row of 16 lanes the exchange is done with DPP modifiers (register-to-register,
// no LDS round trip): swap neighbours, swap pairs, mirror within 8, mirror within 16.  After
// those four steps every lane of a row holds the row's result; the four rows are then
// combined with two cross-lane permutes (xor 16, xor 32).
constexpr int kDppSwap1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppSwap2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;  // lane i <-> 7 - i within 8
constexpr int kDppMirror = 0x140;      // lane i <-> 15 - i within 16

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
template <int CTRL>
__device__ __forceinline__ int dpp_i32(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, false);
}

__device__ __forceinline__ float wave_sum(float v) {
    v += dpp_f32<kDppSwap1>(v);
    v += dpp_f32<kDppSwap2>(v);
    v += dpp_f32<kDppHalfMirror>(v);
    v += dpp_f32<kDppMirror>(v);
    v += __shfl_xor(v, 16, kWave);
    v += __shfl_xor(v, 32, kWave);
    return v;
}

// silu(z) = z / (1 + e^-z) with the hardware reciprocal (1 ulp) in place of an IEEE division:
// the epilogue of a 256 x 256 SwiGLU tile evaluates it 64 times per lane.
__device__ __forceinline__ float silu_f32(float z) {
#if defined(__HIP_DEVICE_COMPILE__)
    return z * __builtin_amdgcn_rcpf(1.0f + __expf(-z));
#else
    return z / (1.0f + __expf(-z));
#endif
}

// ---- host side ---------------------------------------------------------------------------
inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

inline int launch_status() { return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_LAUNCH; }

// Kernels that use more than the default 64 KB of dynamic LDS need the limit raised once per
// device.  `done` is a per-kernel bit mask of the devices already set up (the only state the
// library keeps; a race merely repeats the call).
inline int allow_dynamic_lds(const void* kernel, size_t bytes, std::atomic<uint64_t>& done) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return MOE_ERR_LAUNCH;
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return MOE_OK;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess)
        return MOE_ERR_LAUNCH;
    done.fetch_or(bit, std::memory_order_release);
    return MOE_OK;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline size_t elt_size(int act_dtype) { return act_dtype == MOE_F32 ? 4 : 2; }

inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Optional per-stage timing (moe_forward_timed): an event before the first stage and after
// every stage kernel, all on the launch stream.  A null timer costs nothing.
struct StageTimer {
    hipStream_t st;
    hipEvent_t ev[MOE_MAX_STAGES + 1];
    const char* name[MOE_MAX_STAGES];
    int n;
};
inline void stage_mark(StageTimer* t, const char* name) {
    if (!t || t->n >= MOE_MAX_STAGES) return;
    t->name[t->n] = name;
    (void)hipEventRecord(t->ev[t->n + 1], t->st);
    t->n += 1;
}

// Shape check shared by every entry point: MOE_OK, MOE_ERR_INVALID or MOE_ERR_UNSUPPORTED.
int validate_shape(const moe_shape* s);

// ---- per-stage launchers (each file owns its kernels) ---------------------------------------
int launch_route(const moe_shape& s, const void* x, const float* rw, const float* rb,
                 int32_t* topk_idx, float* topk_gate, float* probs, hipStream_t st);

size_t permute_scratch_bytes(int P, int E);
int launch_permute(int P, int E, const int32_t* topk_idx, int32_t* offsets, int32_t* perm,
                   int32_t* inv_perm, void* scratch, hipStream_t st);
int launch_gather_rows(const moe_shape& s, const int32_t* perm, const void* x, void* x_perm,
                       hipStream_t st);

// addend: optional second per-token term [T, d] in the activation type (beside the residual).
// y_parts > 1: y_perm holds that many partial outputs [P, d], one after the other, to be added.
int launch_combine(const moe_shape& s, const void* y_perm, const int32_t* inv_perm,
                   const float* topk_gate, const void* residual, void* y, hipStream_t st,
                   const void* addend = nullptr, int y_parts = 1);

// Grouped expert FFN on P sorted rows.  a_row_map/a_row_div: optional gather of the input
// rows (row of sorted slot s is x[a_row_map[s] / a_row_div]); NULL = x is already grouped.
// y_parts: NULL = y_perm is one output [P, d].  Otherwise *y_parts says how many outputs [P, d]
// y_perm has room for (down_parts_capacity) and receives how many partial outputs, to be added
// by the consumer, were written: the last product may cut its k-steps into parts to fill the chip.
constexpr int kMaxDownParts = 4;
int down_parts_capacity(const moe_shape& s);
size_t ffn_scratch_bytes(const moe_shape& s);
int launch_expert_ffn(const moe_shape& s, const moe_weights& w, const void* x,
                      const int32_t* a_row_map, int a_row_div, const int32_t* offsets,
                      void* y_perm, void* scratch, hipStream_t st, StageTimer* timer = nullptr,
                      int* y_parts = nullptr);

// Shared-base experts M_e = M0 + L_e R_e (Sec. 2.2, Eq. 1 with a base shared by all experts), prefill,
// with the token of every sorted slot known: the base products run once per token instead
// of once per (token, expert) pair.  y_perm [P, d] receives only the low-rank part of the down
// projection and y_base [T, d] the shared part, to be added in the combine.
bool token_base_supported(const moe_shape& s);
int launch_expert_ffn_token_base(const moe_shape& s, const moe_weights& w, const void* x,
                                 const int32_t* perm, const int32_t* inv_perm, const float* topk_gate,
                                 const int32_t* offsets, void* y_perm, void* y_base, void* scratch,
                                 hipStream_t st, StageTimer* timer = nullptr);

// Single-token layer: experts chosen on the device from topk_idx, weights streamed once.
size_t decode_scratch_bytes(const moe_shape& s);
int launch_decode_ffn(const moe_shape& s, const moe_weights& w, const void* x,
                      const int32_t* topk_idx, const float* topk_gate, void* y, void* scratch,
                      hipStream_t st, StageTimer* timer = nullptr);

}  // namespace moe
