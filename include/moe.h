/*
 * moe.h - C ABI of the MI355X (gfx950) sparse Mixture-of-Experts feed-forward layer.
 *
 * The layer is the one CoSMoEs (arXiv 2503.00245) builds on: the dense
 * feed-forward block of a Llama-style decoder is replaced by a router and E
 * experts with token-choice routing, k experts active per token (Sec. 2.1,
 * Fig. 2; Sec. 3.1: E = 8, k = 2).  Router probabilities and the selection are
 * Eq. 2 and Eq. 3 of Sec. 2.3 (softmax over all E logits, then top-k); an
 * expert is a bias-free SwiGLU block whose three matrices are either stored
 * whole or weight-decomposed, M (n x m) = L (n x r) . R (r x m), Sec. 2.2 Eq. 1.
 *
 * Conventions shared by every entry point
 *   - Every pointer named below is a DEVICE pointer into memory the caller
 *     owns (the structs themselves are host memory).  The library allocates,
 *     frees and retains nothing; scratch comes from a caller workspace sized
 *     by moe_workspace_bytes().
 *   - `stream` is a hipStream_t passed as void*.  Calls enqueue kernels on it
 *     and return without synchronising; nothing is read back to the host.
 *   - Tensors are row-major with the innermost dimension contiguous and
 *     16-byte-aligned base pointers.  Activations and expert weights share one
 *     storage type, shape.act_dtype (fp32 or bf16); the router, logits,
 *     probabilities and gates are always fp32; indices are int32.
 *   - Return value: MOE_OK, or a negative status found on the host before any
 *     kernel is launched (bad argument, unsupported shape, short workspace) or
 *     MOE_ERR_LAUNCH if the runtime refused a launch.  There is no device-side
 *     error reporting; non-finite inputs give unspecified outputs.
 *   - No global state (beyond raising, once per device, the LDS limit of the
 *     kernels that need it); calls on distinct streams with distinct workspaces
 *     and outputs may run concurrently, from any host thread.  Results are deterministic (no floating
 *     point atomics): the same call on the same inputs returns the same bits.
 *   - Limits: 1 <= k <= E <= 64; d_model, d_ff, rank multiples of 8;
 *     n_tokens * k < 2^24 (n_tokens = 0 is a valid no-op).
 */
#ifndef MOE_H_
#define MOE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* exported from the shared library (which is built with hidden default visibility) */
#define MOE_API __attribute__((visibility("default")))

enum { MOE_F32 = 0, MOE_BF16 = 1 };

enum {
    MOE_FLAG_SHARED_BASE = 1, /* w_gate/w_up/w_down hold ONE dense block shared by all experts */
    MOE_FLAG_RESIDUAL = 2     /* moe_forward adds its input: y = x + layer(x) */
};

enum {
    MOE_OK = 0,
    MOE_ERR_INVALID = -1,     /* null / misaligned pointer, k < 1, k > E, negative size */
    MOE_ERR_UNSUPPORTED = -2, /* shape or dtype outside the limits above */
    MOE_ERR_WORKSPACE = -3,   /* workspace_bytes < moe_workspace_bytes(shape) */
    MOE_ERR_LAUNCH = -4       /* hipGetLastError() after a launch was not hipSuccess */
};

/* Problem shape.  T tokens of width d; E experts of inner width F; k active. */
typedef struct moe_shape {
    int32_t n_tokens;  /* T (batch folded into the token dimension)            */
    int32_t d_model;   /* d                                                     */
    int32_t d_ff;      /* F, per expert                                         */
    int32_t n_experts; /* E                                                     */
    int32_t top_k;     /* k                                                     */
    int32_t rank;      /* r of Eq. 1; 0 = experts stored as whole matrices      */
    int32_t act_dtype; /* MOE_F32 or MOE_BF16                                   */
    int32_t flags;     /* MOE_FLAG_*                                            */
} moe_shape;

/*
 * Weights of one layer ([expert, out, in] = the linear-layer convention y = M v).
 *   router_w [E, d] fp32; router_b [E] fp32 or NULL (the paper has no router
 *   bias; it exists to impose skewed expert loads on synthetic inputs).
 *   rank == 0:            w_gate, w_up [E, F, d], w_down [E, d, F]; factor pointers ignored.
 *   rank  > 0, no base:   w_* NULL; every product M v is L_M (R_M v)  (Eq. 1):
 *                         rg, ru [E, r, d]; lg, lu [E, F, r]; rd [E, r, F]; ld [E, d, r].
 *   rank  > 0 and MOE_FLAG_SHARED_BASE: w_gate, w_up [1, F, d], w_down [1, d, F]
 *                         shared by all experts; M_e v = M0 v + L_{M,e} (R_{M,e} v).
 */
typedef struct moe_weights {
    const float* router_w;
    const float* router_b;
    const void* w_gate;
    const void* w_up;
    const void* w_down;
    const void* rg;
    const void* ru;
    const void* rd;
    const void* lg;
    const void* lu;
    const void* ld;
} moe_weights;

/*
 * Router: logits R[t,e] = <x[t,:], router_w[e,:]> (+ router_b[e]), probabilities
 * W = softmax(R) over the E experts (Sec. 2.3, Eq. 2 with temperature 1), and the
 * selection S = top_k(W, k) (Eq. 3).  The k experts of a token are ordered by
 * descending logit; equal logits are ordered by ascending expert index (the
 * comparison is made on logits, which softmax preserves).  Gates are the selected
 * probabilities renormalised to sum to one: g[t,j] = W[t,S[t,j]] / sum_j' W[t,S[t,j']].
 *   x          [T, d]  act_dtype      in
 *   topk_idx   [T, k]  int32          out
 *   topk_gate  [T, k]  fp32           out
 *   probs      [T, E]  fp32 or NULL   out (full softmax, for routing statistics)
 */
MOE_API int moe_route(const moe_shape* shape, const void* x, const float* router_w,
              const float* router_b, int32_t* topk_idx, float* topk_gate, float* probs,
              void* stream);

/*
 * Dispatch: stable counting sort of the P = T*k (token, slot) pairs p = t*k + j by
 * their expert topk_idx[p], so each expert's rows become one contiguous group
 * (Sec. 2.1: every token is sent to its own subset of experts).
 *   expert_offsets [E+1] int32 out: group e is sorted slots [offsets[e], offsets[e+1])
 *   perm           [P]   int32 out: perm[s] = p, the pair held by sorted slot s
 *   inv_perm       [P]   int32 out: inv_perm[p] = s
 *   x / x_perm     optional gather: x_perm[s,:] = x[perm[s] / k, :]  ([P, d], act_dtype);
 *                  pass both NULL to skip it.
 * Every topk_idx value must lie in [0, E).  workspace: moe_workspace_bytes(shape).
 */
MOE_API int moe_permute(const moe_shape* shape, const int32_t* topk_idx, int32_t* expert_offsets,
                int32_t* perm, int32_t* inv_perm, const void* x, void* x_perm,
                void* workspace, size_t workspace_bytes, void* stream);

/*
 * Expert feed-forward on grouped rows: for every expert e and every row s of its
 * group,  y_perm[s,:] = W_down,e ( silu(W_gate,e v) * (W_up,e v) ),  v = x_perm[s,:],
 * silu(z) = z / (1 + exp(-z)), no biases (Sec. 3.1: Llama-style blocks).  With
 * rank > 0 each matrix-vector product is the factored one of Sec. 2.2, Eq. 1 (see
 * moe_weights).  Accumulation is fp32; with bf16 storage the inner activations
 * (the F-wide hidden vector and the rank-r intermediates) are rounded to bf16.
 *   x_perm [P, d] in, y_perm [P, d] out (act_dtype); expert_offsets [E+1] as above.
 */
MOE_API int moe_expert_ffn(const moe_shape* shape, const moe_weights* weights, const void* x_perm,
                   const int32_t* expert_offsets, void* y_perm, void* workspace,
                   size_t workspace_bytes, void* stream);

/*
 * Combine: y[t,:] = sum_{j<k} topk_gate[t,j] * y_perm[inv_perm[t*k+j], :]  (+ residual[t,:]),
 * summed in fp32 in ascending j (Sec. 1: the gate sets each expert's contribution).
 *   residual [T, d] act_dtype or NULL; y [T, d] act_dtype out.
 */
MOE_API int moe_combine(const moe_shape* shape, const void* y_perm, const int32_t* inv_perm,
                const float* topk_gate, const void* residual, void* y, void* stream);

/*
 * Whole layer: route -> dispatch -> expert FFN -> combine in one call, free to fuse
 * stages (a decode step of one or two tokens streams only the selected experts'
 * weights as a bandwidth-bound matrix-vector product; larger T runs a grouped MFMA GEMM).
 * With a shared base (Sec. 2.2, M_e = M0 + L_e R_e) and k > 1 the shared matrices are
 * applied once per token, not once per (token, expert) pair: M0 x_t serves all of the
 * token's experts, and sum_j g_j M0 h_j = M0 (sum_j g_j h_j); the result equals the staged
 * calls' within the bf16 tolerance, not bit for bit.
 * topk_idx / topk_gate ([T,k]) are optional outputs (NULL to skip) and equal what
 * moe_route returns.  With MOE_FLAG_RESIDUAL, y = x + layer(x); y must not alias x.
 */
MOE_API int moe_forward(const moe_shape* shape, const moe_weights* weights, const void* x, void* y,
                int32_t* topk_idx, float* topk_gate, void* workspace, size_t workspace_bytes,
                void* stream);

/*
 * moe_forward for callers that cannot allocate or pass a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the same
 * results as moe_forward, bit for bit; the scratch is an array inside the library, held by every
 * GPU the library runs on until the process ends (its device address is looked up on the first
 * call on a device).  The call allocates and frees nothing.
 *   - shapes whose moe_workspace_bytes() exceeds MOE_STATIC_WORKSPACE_BYTES are refused with
 *     MOE_ERR_WORKSPACE before any launch (single-token steps of every size fit; a 2048 / 5632
 *     layer up to about 140 tokens);
 *   - every call on one GPU uses that GPU's one array: calls that overlap in time on the same GPU
 *     (two streams, two threads) race; calls on one stream, or otherwise ordered, are fine.
 *     Nothing in the array has to be cleared between calls.
 */
#define MOE_STATIC_WORKSPACE_BYTES (8u << 20)
MOE_API int moe_forward_static(const moe_shape* shape, const moe_weights* weights, const void* x,
                               void* y, int32_t* topk_idx, float* topk_gate, void* stream);

/*
 * Residual stack of n_layers layers of one shape: x_{l+1} = x_l + layer_l(x_l), no
 * normalisation, activations between layers stored in act_dtype.  `layers` is a
 * host array of n_layers weight structs.  y [T, d] receives x_{n_layers}.
 * topk_trace ([n_layers, T, k] int32) is optional.  shape.flags' residual bit is
 * implied.  workspace: moe_workspace_bytes(shape).
 */
MOE_API int moe_stack_forward(const moe_shape* shape, const moe_weights* layers, int32_t n_layers,
                      const void* x, void* y, int32_t* topk_trace, void* workspace,
                      size_t workspace_bytes, void* stream);

/*
 * Measurement aid (not an operation of the paper): does exactly what moe_forward does, with
 * a hipEventRecord on `stream` before the first and after every stage kernel, then
 * SYNCHRONISES the stream and reports each stage's elapsed time.  Unlike the other entry
 * points it creates and destroys events and blocks the host.
 *   stage_ms    [MOE_MAX_STAGES] host floats, out: milliseconds per stage
 *   stage_names [MOE_MAX_STAGES] host, out or NULL: static strings naming each stage
 *   n_stages    host, out: how many stages ran
 */
#define MOE_MAX_STAGES 12
MOE_API int moe_forward_timed(const moe_shape* shape, const moe_weights* weights, const void* x,
                              void* y, void* workspace, size_t workspace_bytes, void* stream,
                              float* stage_ms, const char** stage_names, int32_t* n_stages);

/*
 * Hard expert replacements of a routing trace (Sec. 2.3, Eq. 4): S [B,T,K] int32 holds the
 * experts selected for token t of sequence b (for example topk_idx of moe_route, or the
 * topk_trace of moe_stack_forward with B = layers).
 *   H_e[e] = sum_b sum_{t<T-1} | [e in S[b,t+1]] - [e in S[b,t]] |,   H = sum_e H_e.
 * Every replacement is counted twice; Eq. 5 uses floor(H/2).  H_e [E] and H [1] are int64
 * device outputs.  1 <= K <= E <= 64.
 */
MOE_API int moe_expert_replacements(const int32_t* S, int32_t B, int32_t T, int32_t K, int32_t E,
                                    int64_t* H_e, int64_t* H, void* stream);

/*
 * Forward value of the block-wise expert selection loss (Sec. 2.3, Eq. 4-7) from the routing
 * probabilities probs [B,T,E] fp32 (the optional output of moe_route) and the selection S [B,T,K]:
 *   H_norm = floor(H/2) / (B K (T-1)),  L = sum |W[b,t+1,e] - W[b,t,e]|,  L_norm = L / (B T),
 *   loss = H_norm * L_norm.
 * out [5] fp64 device: H, H_norm, L, L_norm, loss.  The backward pass is not provided.
 * workspace: moe_bles_workspace_bytes(B, T, E) device bytes.
 */
MOE_API size_t moe_bles_workspace_bytes(int32_t B, int32_t T, int32_t E);
MOE_API int moe_bles_loss(const float* probs, const int32_t* S, int32_t B, int32_t T, int32_t K,
                          int32_t E, double* out, void* workspace, size_t workspace_bytes,
                          void* stream);

/*
 * Counters of the expert-offloading rule (Sec. 3.4.2): for each layer l of trace [L,T,K], whenever
 * the selected set differs from the previous token's, the non-selected experts leave the GPU
 * and the selected ones are brought in.  changes[l] = number of tokens whose set differs from
 * the previous one (the first token differs from the empty set); loads[l] = experts brought
 * in = sum_t |S_t \ S_{t-1}|.  Multiply loads by the bytes of one expert for the traffic the
 * rule would cause.  changes, loads: [L] int64 device outputs.
 */
MOE_API int moe_offload_counters(const int32_t* trace, int32_t L, int32_t T, int32_t K, int32_t E,
                                 int64_t* changes, int64_t* loads, void* stream);

/*
 * "Delta Uniform" of a routing trace [L,T,K] (Sec. 3.2: the average per-layer delta between the
 * uniform distribution and the realised expert balance; the third column of Table 3, per group of
 * layers in Fig. 6).  The paper prints no formula for a layer's delta; this library takes the L1
 * distance between the layer's realised shares and the uniform share,
 *   counts[l,e] = #{(t,j) : trace[l,t,j] = e},   share = counts / (T K),
 *   delta[l] = sum_e | share[l,e] - 1/E |   (= the mean over experts of |share - 1/E| relative to 1/E),
 *   mean = (1/L) sum_l delta[l],
 * as fractions (the paper prints percent): 0 for a balanced layer, 2 (1 - K/E) when every token
 * uses the same K experts.  That the reported figure is the plain mean over layers is the paper's
 * (Fig. 6's values average to Table 3's); the per-layer formula is this library's reading.
 * counts [L,E] int64, mean [1] fp64, delta [L] fp64 or NULL: device outputs.  Entries of the trace
 * outside [0,E) are ignored.
 */
MOE_API int moe_delta_uniform(const int32_t* trace, int32_t L, int32_t T, int32_t K, int32_t E,
                              int64_t* counts, double* delta, double* mean, void* stream);

/* Bytes of workspace that any entry point above needs for this shape (0 if invalid). */
MOE_API size_t moe_workspace_bytes(const moe_shape* shape);

/* Static, NUL-terminated description of a status code. */
MOE_API const char* moe_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* MOE_H_ */
