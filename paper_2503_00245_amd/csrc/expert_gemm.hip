// Grouped expert GEMMs for prefill: every expert multiplies its own contiguous group of
// sorted rows by its own matrices (Sec. 2.1), with the SwiGLU activation fused into the
// gate/up product's epilogue and weight-decomposed experts (Sec. 2.2, Eq. 1) expressed
// as extra K-segments accumulated into the same output tile.
//
// One generic problem:   C[s, n] = epi( sum_seg  A_seg[row(s), :] . B_seg[e(s)][n, :] )
//   PLAIN   one accumulator, C = acc
//   SWIGLU  two accumulators over (A0,B0) and (A1,B1); C = silu(acc0) * acc1
// A and B are both K-contiguous ("NT" GEMM), the natural layout of activations [rows, in]
// and linear-layer weights [out, in], and exactly what an MFMA lane wants: 8 consecutive
// k of one row per 16-byte read.
//
// bf16 kernels: block tile BM x BN x BK on (BM / WM) * (BN / WN) waves, wave tile WM x WN built
// from v_mfma_f32_32x32x16_bf16, fp32 accumulators in registers.  Global -> registers -> LDS
// with two LDS stages and two register sets, so that three tiles are in flight; a K that is
// not a multiple of BK (any multiple of 8) ends in a partly zero-filled step.  LDS rows are BK bf16 wide with the 16-byte chunk index XOR-ed by a
// function of the row, which spreads both the row-wise fills and the column-of-rows MFMA
// operand reads over all banks.  Tiles are enumerated expert-major, then n-tile, then the
// expert's m-tiles, and the workgroup id is remapped so that each XCD walks a contiguous
// eighth of that order (consecutive tiles share a weight tile and hit in that XCD's L2).
// run_gemm picks the tile shape from the pair count and the output width.
//
// fp32 problems (correctness-only configuration) use a plain LDS-tiled FMA kernel.
#include <type_traits>
#include <utility>

#include "common.h"

namespace moe {

template <int... I, typename F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F&& f) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    static_for_impl(std::make_integer_sequence<int, N>{}, static_cast<F&&>(f));
}

// Products whose activation operand is the F-wide hidden tensor (down, rank-down): that operand is
// as large as an expert's weights, so tiles are ordered in blocks of this many n-tiles with the
// expert's m-tiles inside a block -- the workgroups in flight on an XCD then share a few A tiles
// and a few B tiles instead of one B tile and every A tile (measured on the phone shape with
// Zipf loads: down product 145 us with blocks of 8 or 16, 148 with 4, 153-157 with n-tile outer).
constexpr int kHiddenOperandBlock = 8;

struct GemmSeg {
    const void* A0;     // [*, K]
    const void* A1;     // A of the second accumulator (SWIGLU); may equal A0
    const void* B0;     // [Eb, N, K]
    const void* B1;
    long long strideB;  // elements between experts; 0 = shared by all experts
    int K;
    int gather;         // 1: the A row of sorted slot s is row_map[s] / row_div
};

struct GemmArgs {
    GemmSeg seg[2];
    int nseg;
    void* C;            // [P, N]
    void* C1;           // PLAIN only, deep kernel: second product (A1 . B1) of the same shape, or NULL
    int N;
    const int32_t* offsets;  // [E+1]
    const int32_t* row_map;  // [P] or NULL
    int row_div;
    int E;
    int P;
    int m_tiles_max;
    int n_tiles;        // n-tiles of the launch (twice those of one product when C1 is set)
    // SWIGLU, deep kernel: per-token rows added to the two accumulators before the activation
    // (the token of sorted slot s is row_map[s] / row_div), [*, N] in the activation type, or NULL
    const void* add0;
    const void* add1;
    int n_inner;        // tile order inside an expert: blocks of this many n-tiles (0 or 1: n-tile outer, m-tiles inner)
    int split_slots;    // workgroups one XCD runs at a time; > 0: the tiles of its last, partial round are cut
                        // into upper and lower halves when both halves still fit in one round (set by the launcher)
    // PLAIN, one segment: the k-steps of every tile are cut into k_parts consecutive ranges, each
    // computed by a workgroup of its own and stored to its own output [P, N] (part q at
    // C + q * part_stride elements); whoever consumes C adds the parts.  In: the most parts the
    // caller's output can take (0 or 1: none).  Out (set by run_gemm): the parts used.
    int k_parts;
    long long part_stride;
};

// Group e's row range; offsets == NULL means one group holding all P rows (a plain product).
__device__ __forceinline__ int group_begin(const int32_t* __restrict__ offsets, int e) {
    return offsets ? offsets[e] : 0;
}
__device__ __forceinline__ int group_end(const int32_t* __restrict__ offsets, int e, int P) {
    return offsets ? offsets[e + 1] : P;
}

// Workgroup -> output tile.  Tiles are ordered expert-major, then n-tile, then the expert's
// own m-tiles, so neighbouring tiles share the expert's activation rows (and, for equal
// n-tile, its weight tile).  Workgroups are handed to the 8 XCDs round-robin by id; XCD x
// takes the x-th contiguous eighth of that order, which keeps each XCD's L2 working set to
// about one expert's rows plus the weight tiles it is streaming.  The grid is an upper
// bound (group sizes live on the device); surplus workgroups return false.
//
// Tail split: an XCD runs split_slots workgroups at a time, so its tiles take
// ceil(tiles / split_slots) rounds and the last round may be nearly empty.  When there is at
// least one full round and the last one holds at most split_slots / 2 tiles, each of those is
// cut into an upper and a lower half (BM / 2 rows) handled by two workgroups: the halves still
// fit in one round and each is shorter than a whole tile (it fills half the activation rows
// and multiplies half the blocks).
__device__ __forceinline__ bool find_tile(const int32_t* __restrict__ offsets, int E, int P, int BM,
                                          int n_tiles, int& e_out, int& row0, int& row_end,
                                          int& nt_out, int n_inner = 0, int split_slots = 0) {
#if defined(__HIP_DEVICE_COMPILE__)
    // Lane e of every wave fetches group e's bounds with ONE vector load (E <= 64); the sums below
    // then run on scalar registers through readlane.  (A loop of dependent scalar loads over the
    // offsets cost 2.6-3.3 us per tile here, a twentieth of a tile's whole duration.)
    const int lane = threadIdx.x & (kWave - 1);
    int lo = 0, hi = 0;
    if (lane < E) {
        lo = group_begin(offsets, lane);
        hi = group_end(offsets, lane, P);
    }
    const int cnt = (hi - lo + BM - 1) / BM;  // m-tiles of group `lane` (0 beyond E)
    int total = 0;
    for (int e = 0; e < E; ++e) total += __builtin_amdgcn_readlane(cnt, e);
    total *= n_tiles;
#else
    int total = 0;
    for (int e = 0; e < E; ++e)
        total += (group_end(offsets, e, P) - group_begin(offsets, e) + BM - 1) / BM;
    total *= n_tiles;
#endif
    const int per_xcd = (total + 7) / 8;
    const int slot = blockIdx.x >> 3;
    const int first = (blockIdx.x & 7) * per_xcd;               // this XCD's first tile
    const int mine = max(0, min(per_xcd, total - first));       // and how many it has
    int local_tile = slot, half = -1;
    if (split_slots > 0) {
        const int whole = (mine / split_slots) * split_slots;   // tiles in full rounds
        const int rem = mine - whole;
        if (whole > 0 && rem > 0 && 2 * rem <= split_slots && slot >= whole) {
            const int idx = slot - whole;
            local_tile = whole + idx / 2;
            half = idx & 1;
        }
    }
    if (local_tile >= mine) return false;
    const int L = first + local_tile;
    int before = 0;
    for (int e = 0; e < E; ++e) {
#if defined(__HIP_DEVICE_COMPILE__)
        const int mtiles = __builtin_amdgcn_readlane(cnt, e);
#else
        const int mtiles = (group_end(offsets, e, P) - group_begin(offsets, e) + BM - 1) / BM;
#endif
        const int here = mtiles * n_tiles;
        if (L < before + here) {
#if defined(__HIP_DEVICE_COMPILE__)
            const int prev = __builtin_amdgcn_readlane(lo, e), next = __builtin_amdgcn_readlane(hi, e);
#else
            const int prev = group_begin(offsets, e), next = group_end(offsets, e, P);
#endif
            const int local = L - before;
            e_out = e;
            // blocks of n_inner n-tiles: block outer, the expert's m-tiles in the middle, the
            // block's n-tiles inner (n_inner = 1: n-tile outer, m-tiles inner)
            const int nb = max(n_inner, 1);
            const int full = (n_tiles / nb) * nb * mtiles;  // tiles in whole blocks
            int mt, nt;
            if (local < full) {
                const int rem = local % (mtiles * nb);
                mt = rem / nb;
                nt = (local / (mtiles * nb)) * nb + rem % nb;
            } else {
                const int nb_tail = n_tiles % nb;
                const int rem = local - full;
                mt = rem / nb_tail;
                nt = (n_tiles / nb) * nb + rem % nb_tail;
            }
            nt_out = nt;
            row0 = prev + mt * BM;
            row_end = next;
            if (half >= 0) {
                row0 += half * (BM / 2);
                row_end = min(next, row0 + BM / 2);
                if (row0 >= row_end) return false;  // the tile had no rows in its lower half
            }
            return true;
        }
        before += here;
    }
    return false;
}

// m-tile index (over all experts, in expert order) -> expert and row range
__device__ __forceinline__ bool find_m_tile(const int32_t* __restrict__ offsets, int E, int P, int BM,
                                            int mt, int& e_out, int& row0, int& row_end) {
    int acc = 0;
    int prev = group_begin(offsets, 0);
    for (int e = 0; e < E; ++e) {
        const int next = group_end(offsets, e, P);
        const int tiles = (next - prev + BM - 1) / BM;
        if (mt < acc + tiles) {
            e_out = e;
            row0 = prev + (mt - acc) * BM;
            row_end = next;
            return true;
        }
        acc += tiles;
        prev = next;
    }
    return false;
}

__device__ __forceinline__ int src_row(const GemmArgs& g, const GemmSeg& sg, int s) {
    if (!sg.gather) return s;
    const int p = min(max(g.row_map[s], 0), g.P - 1);
    return p / g.row_div;
}

// ============================================================================= bf16 MFMA
// LDS tile rows hold BK bf16 (BK/8 chunks of 16 bytes).  The chunk index is XOR-ed with a
// function of the row chosen so that 16 consecutive rows read at one chunk index (an MFMA
// operand read) touch 16 distinct 16-byte bank groups, as do the row-wise fills.
template <int BK>
__device__ __forceinline__ int lds_off(int row, int chunk) {
    constexpr int CPR = BK / 8;  // chunks per row
    return row * (BK * 2) + ((chunk ^ ((row / (16 / CPR)) % CPR)) << 4);
}

// ============================================================================= bf16 MFMA, deep pipeline
// K a multiple of 8 (rows are read in 16-byte chunks).  Two register sets and two LDS stages, so
// three tiles are in flight: tile kt is multiplied out of LDS while tile kt+1 waits in registers to be
// written to the other LDS stage at the end of the step and tile kt+2 is being fetched.
// That puts two full steps of MFMA work between issuing a global load and first needing
// its data.  Loads are unconditional (rows past the end of a group / matrix are clamped to
// its last row and only feed outputs the epilogue never stores), so the loop has no
// divergent control flow.  (Direct global->LDS loads were measured here and rejected:
// on this chip they stall co-issued MFMAs far more than register loads do.)
//
// KG > 1: the workgroup holds KG groups of (BM / WM) * (BN / WN) waves.  Every group runs
// the whole pipeline on its own 1/KG of the k-steps, with its own LDS stages, and the
// groups' accumulators meet in LDS at the end, added in group order.  This is for products
// with fewer tiles than CUs and a long K, where the serial chain of k-steps of a single
// tile, not the chip's throughput, sets the time.  Needs K % (KG * BK) == 0.
// TAIL: K need not be a multiple of BK (a separate instantiation, so that the loop of the common
// case carries none of the tail's bookkeeping: with it the down product of a 2048 x 5632 layer
// measured 3.5 % slower).
// HF ("half fills"): the LDS stages hold k-steps of BK = 64 -- a row's share of a step is one whole
// 128-byte line, where a step of 32 asks for every line twice, half each time -- but a step is
// filled in two halves by rows (the upper and the lower half of the A and of the B tile), half a
// step apart, each through its own small register set.  Registers per thread are those of the
// BK = 32 pipeline (two full BK = 64 sets do not fit beside a 64 x 128 wave tile's accumulators),
// the barriers per k are halved, and every load instruction covers 8 rows x 128 bytes.
template <int BM, int BN, int BK, int WM, int WN, bool SWIGLU, bool DUAL_A, int NS, int KG, bool ADD = false,
          bool TAIL = false, bool HF = false>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64 * KG) void gemm_bf16_deep_kernel(const GemmArgs g) {
    static_assert(!ADD || SWIGLU, "per-token addends belong to the SwiGLU epilogue");
    static_assert(!TAIL || KG == 1, "a K tail only without k-groups");
    static_assert(!HF || (KG == 1 && NS == 2 && BK == 64), "half fills: 64-wide steps, two half sets, no k-groups");
    constexpr int WAVES_N = BN / WN;
    constexpr int NTHR = (BM / WM) * WAVES_N * 64;  // threads of one k-group
    constexpr int MT = WM / 32, NT = WN / 32;
    static_assert(!SWIGLU || NT % 2 == 0, "gate and up fragments pair up");
    constexpr int CPR = BK / 8;
    constexpr int RPP = NTHR / CPR;
    static_assert(BM % RPP == 0 && BN % RPP == 0 && (BN / 2) % RPP == 0, "fill passes");
    constexpr int AI = BM / RPP, BI = BN / RPP;
    constexpr int NA = DUAL_A ? 2 : 1;
    constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
    constexpr int STAGE = A_BYTES * NA + B_BYTES;
    extern __shared__ __align__(16) char smem[];

    int e, row0, row_end, nt;
    if (!find_tile(g.offsets, g.E, g.P, BM, g.n_tiles, e, row0, row_end, nt, g.n_inner, g.split_slots)) return;
    constexpr int BN_OUT = SWIGLU ? BN / 2 : BN;
    // two plain products in one launch: the upper half of the n-tiles belongs to (A1, B1, C1)
    const bool second = !SWIGLU && g.C1 != nullptr && nt >= g.n_tiles / 2;
    if (second) nt -= g.n_tiles / 2;
    // k-parts ride on the n-tile index: n-tiles [q * n_base, (q + 1) * n_base) are part q
    int part = 0;
    if (!SWIGLU && KG == 1 && g.k_parts > 1) {
        const int n_base = g.n_tiles / g.k_parts;
        part = nt / n_base;
        nt -= part * n_base;
    }
    const int n0 = nt * BN_OUT;

    const int kg = threadIdx.x / NTHR;   // k-group of this wave
    const int tid = threadIdx.x % NTHR;  // thread within the group
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int ld_row = tid / CPR, ld_chunk = tid % CPR;
    char* const gmem = smem + kg * (2 * STAGE);  // this group's two stages

    f32x16 acc[MT][NT];
    if constexpr (ADD) {
        // Per-token addends: the accumulators start from the token's rows of add0 / add1 instead
        // of zero.  The gathers are issued here, ahead of the first tile loads and with every
        // register still free, so their latency hides behind the pipeline's own start-up.
        static_assert(KG == 1, "addends are added once");
        const bf16_t* add0 = static_cast<const bf16_t*>(g.add0);
        const bf16_t* add1 = static_cast<const bf16_t*>(g.add1);
#pragma unroll
        for (int mi = 0; mi < MT; ++mi) {
            int tok[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int row = min(row0 + wm * WM + mi * 32 + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3), row_end - 1);
                tok[i] = min(max(g.row_map[row], 0), g.P - 1) / g.row_div;
            }
#pragma unroll
            for (int ni = 0; ni < NT / 2; ++ni) {
                const int col = min(n0 + wn * (WN / 2) + ni * 32 + (lane & 31), g.N - 1);
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const size_t at = (size_t)tok[i] * g.N + col;
                    acc[mi][ni][i] = (float)add0[at];
                    acc[mi][ni + NT / 2][i] = (float)add1[at];
                }
            }
        }
    } else {
#pragma unroll
        for (int mi = 0; mi < MT; ++mi)
#pragma unroll
            for (int ni = 0; ni < NT; ++ni)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.f;
    }

    // passes (of RPP rows) one register set covers: all of a tile, or (HF) one half of it
    constexpr int AP = HF ? AI / 2 : AI, BP = HF ? BI / 2 : BI;
    static_assert(!HF || (AI % 2 == 0 && BI % 2 == 0), "half fills cut the fill passes in two");
    struct Regs {
        bf16x8 a[AP], a1[DUAL_A ? AP : 1], b[BP];
    };

    for (int sidx = 0; sidx < g.nseg; ++sidx) {
        const GemmSeg& sg = g.seg[sidx];
        const int K = sg.K;
        const bool dual = DUAL_A && sg.A1 != sg.A0;
        const bf16_t* B0 = static_cast<const bf16_t*>(second ? sg.B1 : sg.B0) + (size_t)e * sg.strideB;
        const bf16_t* B1 = SWIGLU ? static_cast<const bf16_t*>(sg.B1) + (size_t)e * sg.strideB : B0;
        int nk = (K + BK * KG - 1) / (BK * KG);  // k-steps of this group (the same for every group)
        int k_begin = kg * nk * BK;
        if (!SWIGLU && KG == 1 && g.k_parts > 1) {  // this workgroup's share of the k-steps
            const int s0 = nk * part / g.k_parts, s1 = nk * (part + 1) / g.k_parts;
            k_begin = s0 * BK;
            nk = s1 - s0;
        }
        const int k_last = (nk - 1) * BK;    // relative to k_begin
        // K tail (TAIL: K % BK != 0, a multiple of 8): in the last k-step a thread whose 16-byte
        // chunk lies at or beyond K reads an earlier chunk of its row instead (in bounds) and zeroes
        // its registers before they go to LDS.  Which threads those are never changes (a thread
        // always loads the same chunk of a tile), so the loop pays one vector min per step.
        const int tail_kt = (TAIL && K % BK != 0) ? nk - 1 : -1;               // wave-uniform
        const bool tail_dead = TAIL && k_begin + k_last + ld_chunk * 8 >= K;    // per thread (never in a k-part before the last)
        const int k_last_t = tail_dead ? max(k_last - BK, -(ld_chunk * 8)) : k_last;

        // Where a thread's rows start.  HF keeps 32-bit byte offsets from wave-uniform bases (the
        // load then takes a scalar base and one vector register; its launcher checks that every
        // operand stays below 4 GB): eight 64-bit pointers are registers this kernel does not have.
        typedef typename std::conditional<HF, unsigned, const bf16_t*>::type rowref_t;
        rowref_t pa[AI];
        rowref_t pa1[DUAL_A ? AI : 1];
        rowref_t pb[BI];
        const char* const a0_base = static_cast<const char*>(second ? sg.A1 : sg.A0);
        const char* const a1_base = static_cast<const char*>(sg.A1);
        // (the row-map lookups of all of a thread's rows are issued together: one latency, not AI)
        int arow[AI];
#pragma unroll
        for (int i = 0; i < AI; ++i) arow[i] = min(row0 + ld_row + RPP * i, row_end - 1);
        if (sg.gather) {
#pragma unroll
            for (int i = 0; i < AI; ++i) arow[i] = g.row_map[arow[i]];
#pragma unroll
            for (int i = 0; i < AI; ++i) arow[i] = min(max(arow[i], 0), g.P - 1) / g.row_div;
        }
#pragma unroll
        for (int i = 0; i < AI; ++i) {
            const size_t off = (size_t)arow[i] * K + k_begin + ld_chunk * 8;
            if constexpr (HF) {
                pa[i] = (unsigned)(off * 2);
                if (DUAL_A) pa1[i] = (unsigned)(off * 2);
            } else {
                pa[i] = static_cast<const bf16_t*>(second ? sg.A1 : sg.A0) + off;
                if (DUAL_A) pa1[i] = static_cast<const bf16_t*>(sg.A1) + off;
            }
        }
#pragma unroll
        for (int i = 0; i < BI; ++i) {
            const int j = ld_row + RPP * i;
            const int n = min(SWIGLU ? n0 + (j % (BN / 2)) : n0 + j, g.N - 1);
            const size_t off = (size_t)n * K + k_begin + ld_chunk * 8;
            if constexpr (HF)
                pb[i] = (unsigned)(off * 2);
            else
                pb[i] = ((SWIGLU && i >= BI / 2) ? B1 : B0) + off;
        }
        // one 16-byte chunk at k offset k0 (elements) of the row a reference stands for
        auto ld16 = [&](const char* base, rowref_t ref, int k0) {
            if constexpr (HF)
                return *reinterpret_cast<const bf16x8*>(base + (size_t)k0 * 2 + ref);
            else
                return *reinterpret_cast<const bf16x8*>(ref + k0);
        };

        // half: which half of the tile's fill passes the set covers (HF; 0 otherwise)
        auto gload = [&](Regs& r, int k0, int half = 0) {
#pragma unroll
            for (int i = 0; i < AP; ++i) {
                r.a[i] = ld16(a0_base, pa[half * AP + i], k0);
                if (DUAL_A && dual) r.a1[i] = ld16(a1_base, pa1[half * AP + i], k0);
            }
#pragma unroll
            for (int i = 0; i < BP; ++i) {
                const int pass = half * BP + i;
                r.b[i] = ld16(reinterpret_cast<const char*>((SWIGLU && pass >= BI / 2) ? B1 : B0), pb[pass], k0);
            }
        };
        auto zero_dead = [&](Regs& r) {
            if (tail_dead) {
#pragma unroll
                for (int i = 0; i < AP; ++i) {
                    r.a[i] = bf16x8{};
                    if (DUAL_A) r.a1[i] = bf16x8{};
                }
#pragma unroll
                for (int i = 0; i < BP; ++i) r.b[i] = bf16x8{};
            }
        };
        auto lstore = [&](int stage, const Regs& r, int half = 0) {
            char* base = gmem + stage * STAGE;
#pragma unroll
            for (int i = 0; i < AP; ++i) {
                const int row = ld_row + RPP * (half * AP + i);
                *reinterpret_cast<bf16x8*>(base + lds_off<BK>(row, ld_chunk)) = r.a[i];
                if (DUAL_A && dual)
                    *reinterpret_cast<bf16x8*>(base + A_BYTES + lds_off<BK>(row, ld_chunk)) = r.a1[i];
            }
            char* bb = base + A_BYTES * NA;
#pragma unroll
            for (int i = 0; i < BP; ++i)
                *reinterpret_cast<bf16x8*>(bb + lds_off<BK>(ld_row + RPP * (half * BP + i), ld_chunk)) = r.b[i];
        };
        // MA = how many of the wave's MT 32-row blocks hold rows of the group (the rest are skipped)
        auto compute = [&](int stage, auto ma, int ks_begin = 0, int ks_end = BK / 16) {
            constexpr int MA = decltype(ma)::value;
            const char* base = gmem + stage * STAGE;
            const char* a0b = base;
            const char* a1b = (DUAL_A && dual) ? base + A_BYTES : base;
            const char* bb = base + A_BYTES * NA;
#pragma unroll
            for (int ks = ks_begin; ks < ks_end; ++ks) {
                const int chunk = ks * 2 + (lane >> 5);
                bf16x8 fa[MA], fa1[DUAL_A ? MA : 1], fb[NT];
#pragma unroll
                for (int mi = 0; mi < MA; ++mi) {
                    const int r = wm * WM + mi * 32 + (lane & 31);
                    fa[mi] = *reinterpret_cast<const bf16x8*>(a0b + lds_off<BK>(r, chunk));
                    if (DUAL_A) fa1[mi] = *reinterpret_cast<const bf16x8*>(a1b + lds_off<BK>(r, chunk));
                }
#pragma unroll
                for (int ni = 0; ni < NT; ++ni) {
                    int r;
                    if constexpr (SWIGLU)
                        r = (ni < NT / 2 ? 0 : BN / 2) + wn * (WN / 2) + (ni % (NT / 2)) * 32 + (lane & 31);
                    else
                        r = wn * WN + ni * 32 + (lane & 31);
                    fb[ni] = *reinterpret_cast<const bf16x8*>(bb + lds_off<BK>(r, chunk));
                }
#pragma unroll
                for (int mi = 0; mi < MA; ++mi)
#pragma unroll
                    for (int ni = 0; ni < NT; ++ni) {
                        const bf16x8 av = (DUAL_A && SWIGLU && ni >= NT / 2) ? fa1[mi] : fa[mi];
                        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, fb[ni], acc[mi][ni], 0, 0, 0);
                    }
            }
        };

        // NS register sets: tile kt is multiplied out of LDS while tile kt+1 waits in registers to
        // be written to the other LDS stage at the end of the step and tiles kt+2 .. kt+NS are in
        // flight from memory.  Every load and LDS write below is unconditional (k offsets are
        // clamped to the last tile, whose re-fetch near the end is harmless): the
        // outstanding-load count at each wait is then a compile-time constant and a wait for
        // tile kt+1 never also waits for the younger loads behind it.
        constexpr int UNR = (NS % 2 == 0) ? NS : 2 * NS;  // steps until (set, stage) repeat
        Regs r[NS];
        if constexpr (HF) {
            // r[0] / r[1] carry the upper / lower half of a tile: tile 0 goes to stage 0 through
            // them, then they hold tile 1
            gload(r[0], 0, 0);
            gload(r[1], 0, 1);
            if constexpr (TAIL) {
                if (tail_kt == 0) {
                    zero_dead(r[0]);
                    zero_dead(r[1]);
                }
            }
            __syncthreads();  // the previous segment's readers are done with both stages
            lstore(0, r[0], 0);
            gload(r[0], min(BK, k_last_t), 0);
            lstore(0, r[1], 1);
            gload(r[1], min(BK, k_last_t), 1);
        } else {
#pragma unroll
            for (int q = 0; q < NS; ++q) gload(r[q], min(q * BK, k_last_t));
            if constexpr (TAIL) {
                if (tail_kt == 0) zero_dead(r[0]);
            }
            __syncthreads();  // the previous segment's readers are done with both stages
            lstore(0, r[0]);
        }
        __syncthreads();
        // Issue order inside a step: the step's global loads and LDS writes are spread through
        // the MFMA sequence (one memory instruction in the shadow of each MFMA) instead of
        // running as separate phases, so a wave's MFMA stream has no load/store-only gaps.
        auto interleave = [&](auto ma) {
#if defined(__HIP_DEVICE_COMPILE__)
            constexpr int MA = decltype(ma)::value;
            constexpr int NM = MA * NT * (BK / 16);           // MFMAs per step
            constexpr int NR = (MA * NA + NT) * (BK / 16);    // LDS fragment reads per step
            constexpr int NL = AI * NA + BI;                  // global loads = LDS writes per step
            constexpr int RPM = (NR + NM - 1) / NM;
            constexpr int LPM = (2 * NL + NM - 1) / NM;
            __builtin_amdgcn_sched_group_barrier(0x100, MA * NA + NT, 0);  // first fragments
#pragma unroll
            for (int i = 0; i < NM; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);    // one MFMA
                __builtin_amdgcn_sched_group_barrier(0x100, RPM, 0);  // next fragments
                if (i < NM / 2)
                    __builtin_amdgcn_sched_group_barrier(0x020, LPM, 0);  // global loads, tile kt+2
                else
                    __builtin_amdgcn_sched_group_barrier(0x200, LPM, 0);  // LDS writes, tile kt+1
            }
#endif
        };
        // HF: a step writes the two halves of tile kt+1 to the other stage, the upper half at its
        // start and the lower half in its middle, and refills each half's registers with tile
        // kt+2 right after; memory instructions are spread one per two MFMAs in that order
        auto interleave_hf = [&](auto ma) {
#if defined(__HIP_DEVICE_COMPILE__)
            constexpr int MA = decltype(ma)::value;
            constexpr int NM = MA * NT * (BK / 16);           // MFMAs per step
            constexpr int NR = (MA * NA + NT) * (BK / 16);    // LDS fragment reads per step
            constexpr int NH = AP * NA + BP;                  // loads = LDS writes per half
            constexpr int RPM = (NR + NM - 1) / NM;
            constexpr int GAP = NM / (4 * NH) > 0 ? NM / (4 * NH) : 1;  // MFMAs per memory instruction
            __builtin_amdgcn_sched_group_barrier(0x100, MA * NA + NT, 0);  // first fragments
#pragma unroll
            for (int i = 0; i < NM; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);    // one MFMA
                __builtin_amdgcn_sched_group_barrier(0x100, RPM, 0);  // next fragments
                if (i % GAP == 0) {
                    const int op = i / GAP;  // 0 .. 4 NH - 1: writes of half 0, loads, writes of half 1, loads
                    if (op < NH || (op >= 2 * NH && op < 3 * NH))
                        __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
                    else if (op < 4 * NH)
                        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                }
            }
#endif
        };
        // The wave multiplies only those of its 32-row blocks that hold rows of the group.  A wave
        // with none keeps filling LDS and meeting the barriers but issues no fragment reads or
        // MFMAs, which leaves its SIMD and the LDS read port to the waves that do have rows.
        auto k_loop = [&](auto ma) {
            constexpr int MA = decltype(ma)::value;
            // step S of the unrolled body: multiply tile kt (stage S & 1), refill set S % NS (its
            // tile went to LDS at the end of the previous step) with tile kt + NS, write tile
            // kt + 1 (set (S + 1) % NS) to the other stage
            auto step = [&](auto sc, int kt) {
                constexpr int S = decltype(sc)::value;
                if constexpr (HF) {
                    if constexpr (TAIL) {
                        if (kt + 1 == tail_kt) {  // both halves of the tile this step writes to LDS
                            zero_dead(r[0]);
                            zero_dead(r[1]);
                        }
                    }
                    const int k_next = min((kt + 2) * BK, k_last_t);
                    lstore((S & 1) ^ 1, r[0], 0);
                    gload(r[0], k_next, 0);
                    if constexpr (MA > 0) compute(S & 1, ma, 0, BK / 32);
                    lstore((S & 1) ^ 1, r[1], 1);
                    gload(r[1], k_next, 1);
                    if constexpr (MA > 0) compute(S & 1, ma, BK / 32, BK / 16);
                    if constexpr (MA > 0) interleave_hf(ma);
                    __syncthreads();
                    return;
                }
                if constexpr (TAIL) {
                    if (kt + 1 == tail_kt) zero_dead(r[(S + 1) % NS]);  // the tile this step writes to LDS
                }
                gload(r[S % NS], min((kt + NS) * BK, k_last_t));
                if constexpr (MA > 0) compute(S & 1, ma);
                lstore((S & 1) ^ 1, r[(S + 1) % NS]);
                if constexpr (MA > 0) interleave(ma);
                __syncthreads();
            };
            for (int kt = 0; kt < nk; kt += UNR) {
                bool more = true;
                static_for<UNR>([&](auto sc) {
                    constexpr int S = decltype(sc)::value;
                    if (more) {
                        step(sc, kt + S);
                        more = kt + S + 1 < nk;
                    }
                });
                if (!more) break;
            }
        };
        const int live = min(MT, max(0, (row_end - row0 - wm * WM + 31) / 32));  // wave-uniform
        static_assert(MT <= 4, "one k_loop instance per count of live 32-row blocks");
        if (live == MT) k_loop(std::integral_constant<int, MT>{});
        else if (live == 0) k_loop(std::integral_constant<int, 0>{});
        else if (live == 1) k_loop(std::integral_constant<int, 1>{});
        else if (live == 2) k_loop(std::integral_constant<int, (MT > 2 ? 2 : 1)>{});
        else k_loop(std::integral_constant<int, (MT > 3 ? 3 : 1)>{});
    }

    // ---- k-groups 1 .. KG-1 hand their sums to group 0 through LDS (every stage is idle now) ------
    if constexpr (KG > 1) {
        constexpr int NACC = MT * NT * 16;
        static_assert(NACC * NTHR * 4 <= 2 * STAGE, "a group's accumulators fit in its own stages");
        float* mine = reinterpret_cast<float*>(gmem) + tid;
        if (kg > 0) {
#pragma unroll
            for (int mi = 0; mi < MT; ++mi)
#pragma unroll
                for (int ni = 0; ni < NT; ++ni)
#pragma unroll
                    for (int i = 0; i < 16; ++i) mine[((mi * NT + ni) * 16 + i) * NTHR] = acc[mi][ni][i];
        }
        __syncthreads();
        if (kg > 0) return;
        for (int q = 1; q < KG; ++q) {
            const float* src = reinterpret_cast<const float*>(smem + q * (2 * STAGE)) + tid;
#pragma unroll
            for (int mi = 0; mi < MT; ++mi)
#pragma unroll
                for (int ni = 0; ni < NT; ++ni)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[mi][ni][i] += src[((mi * NT + ni) * 16 + i) * NTHR];
        }
    }

    // ---- epilogue: accumulator element i of a 32x32 block sits at row (i/4)*8 + (lane/32)*4 + i%4,
    //      column lane%32 -------------------------------------------------------------------------
    // A block with no rows of the group is skipped.
    bf16_t* const Ct = static_cast<bf16_t*>(second ? g.C1 : g.C) + (size_t)part * g.part_stride +
                       (size_t)row0 * g.N + n0;  // wave-uniform
    const unsigned ldc = (unsigned)g.N;
    if constexpr (KG == 1) {
        // Through LDS, so that the tile leaves in 16-byte stores (8 per wave and 32 x 64 block)
        // instead of one bf16 per lane and instruction (64 of them).  Each wave stages 32 rows x up
        // to 64 columns at a time in a region of its own (every wave is past the k-loop's last
        // barrier, so the tile stages are free; a wave's LDS operations complete in order, so no
        // further barrier is needed): neighbouring lanes first swap half of their values so that
        // a lane holds two adjacent columns of two rows, written as 32-bit words; then the rows
        // are read back 16 bytes per lane.  Worth 0.5-1 % of a prefill step on the shapes measured.
        constexpr int OC = SWIGLU ? WN / 2 : WN;   // output columns of a wave
        constexpr int PW = OC < 64 ? OC : 64;      // columns staged per pass
        constexpr int NB = PW / 32;
        constexpr int PITCH = PW * 2 + 32;         // bytes per staged row (keeps the four lane groups of a write on distinct banks)
        constexpr int REGION = 32 * PITCH;
        static_assert(REGION * (NTHR / 64) <= 2 * STAGE, "the staging regions fit in the tile stages");
        constexpr int LPR = PW / 8, RPI = 64 / LPR;  // lanes per staged row, rows per read instruction
        char* const region = smem + wave * REGION;
        const bool odd = lane & 1;
        const int wr_row = (lane >> 5) * 4 + (odd ? 2 : 0);
        const int wr_col = (lane & 30) * 2;        // byte offset of the column pair in a 32-column block
        const int rd_row = lane / LPR, rd_chunk = lane % LPR;
#pragma unroll
        for (int mi = 0; mi < MT; ++mi) {
            const int rb = wm * WM + mi * 32;           // the block's first row within the tile
            const int rows_here = row_end - row0 - rb;  // rows of the group from there on (wave-uniform)
            if (rows_here <= 0) continue;
#pragma unroll
            for (int cg = 0; cg < OC / PW; ++cg) {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const int ni = cg * NB + nb;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        float o[4];
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            o[j] = acc[mi][ni][q * 4 + j];
                            if (SWIGLU) o[j] = silu_f32(o[j]) * acc[mi][ni + NT / 2][q * 4 + j];
                        }
                        const bf16x2 t01 = {(bf16_t)o[0], (bf16_t)o[1]}, t23 = {(bf16_t)o[2], (bf16_t)o[3]};
                        const unsigned p01 = __builtin_bit_cast(unsigned, t01);  // rows +0, +1 of my column
                        const unsigned p23 = __builtin_bit_cast(unsigned, t23);  // rows +2, +3
                        // even lanes keep rows +0, +1 and get them of the next column; odd lanes keep
                        // rows +2, +3 and get them of the previous column
                        const unsigned keep = odd ? p23 : p01;
                        const unsigned recv = (unsigned)dpp_i32<kDppSwap1>((int)(odd ? p01 : p23));
                        const unsigned lo = odd ? recv : keep, hi = odd ? keep : recv;  // even / odd column
                        char* at = region + (q * 8 + wr_row) * PITCH + nb * 64 + wr_col;
                        *reinterpret_cast<unsigned*>(at) = (lo & 0xffffu) | (hi << 16);
                        *reinterpret_cast<unsigned*>(at + PITCH) = (lo >> 16) | (hi & 0xffff0000u);
                    }
                }
                const int c0 = wn * OC + cg * PW + rd_chunk * 8;  // first of this lane's 8 columns within the tile
#pragma unroll
                for (int it = 0; it < 32 / RPI; ++it) {
                    const int r = it * RPI + rd_row;
                    const uint4 v = *reinterpret_cast<const uint4*>(region + r * PITCH + rd_chunk * 16);
                    if (r < rows_here && n0 + c0 < g.N)
                        *reinterpret_cast<uint4*>(Ct + (unsigned)(rb + r) * ldc + (unsigned)c0) = v;
                }
            }
        }
        return;
    }
    // Kernels with k-groups (small products) store straight from the accumulator layout.  Offsets
    // are 32-bit, relative to the tile's first output (a 64-bit multiply per element costs as much
    // as the SiLU), and a 32-row block that lies wholly inside the group and the matrix stores
    // without per-element predicates.
    const unsigned lane_off = (unsigned)((lane >> 5) * 4) * ldc + (unsigned)(lane & 31);
    const bool cols_inside = n0 + BN_OUT <= g.N;
#pragma unroll
    for (int mi = 0; mi < MT; ++mi) {
        const int rb = wm * WM + mi * 32;             // the block's first row within the tile
        const int rows_here = row_end - row0 - rb;    // rows of the group from there on (wave-uniform)
        if (rows_here <= 0) continue;
#pragma unroll
        for (int ni = 0; ni < (SWIGLU ? NT / 2 : NT); ++ni) {
            const int cb = wn * (SWIGLU ? WN / 2 : WN) + ni * 32;
            const unsigned base = lane_off + (unsigned)rb * ldc + (unsigned)cb;
            if (rows_here >= 32 && cols_inside) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    float v = acc[mi][ni][i];
                    if (SWIGLU) v = silu_f32(v) * acc[mi][ni + NT / 2][i];
                    Ct[base + (unsigned)((i >> 2) * 8 + (i & 3)) * ldc] = (bf16_t)v;
                }
            } else {
                const bool col_ok = n0 + cb + (lane & 31) < g.N;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int rr = (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3);
                    if (rr < rows_here && col_ok) {
                        float v = acc[mi][ni][i];
                        if (SWIGLU) v = silu_f32(v) * acc[mi][ni + NT / 2][i];
                        Ct[base + (unsigned)((i >> 2) * 8 + (i & 3)) * ldc] = (bf16_t)v;
                    }
                }
            }
        }
    }
}

// ============================================================================= generic tiled FMA
// 64 x 64 output tile, 256 threads, 4 x 4 outputs each, K stepped by 16 through LDS.
template <typename T, bool SWIGLU>
__global__ __launch_bounds__(256) void gemm_simple_kernel(const GemmArgs g) {
    constexpr int TM = 64, TN = 64, TK = 16;
    __shared__ float sA0[TK][TM + 1], sA1[TK][TM + 1], sB0[TK][TN + 1], sB1[TK][TN + 1];
    const int mt = blockIdx.x % g.m_tiles_max;
    const int nt = blockIdx.x / g.m_tiles_max;
    int e, row0, row_end;
    if (!find_m_tile(g.offsets, g.E, g.P, TM, mt, e, row0, row_end)) return;
    const int n0 = nt * TN;
    const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
    float acc0[4][4] = {}, acc1[4][4] = {};
    for (int sidx = 0; sidx < g.nseg; ++sidx) {
        const GemmSeg& sg = g.seg[sidx];
        const T* A0 = static_cast<const T*>(sg.A0);
        const T* A1 = static_cast<const T*>(sg.A1);
        const T* B0 = static_cast<const T*>(sg.B0) + (size_t)e * sg.strideB;
        const T* B1 = SWIGLU ? static_cast<const T*>(sg.B1) + (size_t)e * sg.strideB : B0;
        for (int k0 = 0; k0 < sg.K; k0 += TK) {
            __syncthreads();
            for (int i = threadIdx.x; i < TM * TK; i += 256) {
                const int r = i / TK, kk = i % TK;
                const int s = row0 + r;
                const bool ok = s < row_end && k0 + kk < sg.K;
                const size_t off = ok ? (size_t)src_row(g, sg, s) * sg.K + k0 + kk : 0;
                sA0[kk][r] = ok ? Store<T>::to_f32(A0[off]) : 0.f;
                if (SWIGLU) sA1[kk][r] = ok ? Store<T>::to_f32(A1[off]) : 0.f;
                const int n = n0 + r;
                const bool okb = n < g.N && k0 + kk < sg.K;
                const size_t boff = okb ? (size_t)n * sg.K + k0 + kk : 0;
                sB0[kk][r] = okb ? Store<T>::to_f32(B0[boff]) : 0.f;
                if (SWIGLU) sB1[kk][r] = okb ? Store<T>::to_f32(B1[boff]) : 0.f;
            }
            __syncthreads();
#pragma unroll
            for (int kk = 0; kk < TK; ++kk) {
#pragma unroll
                for (int a = 0; a < 4; ++a)
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        acc0[a][b] = fmaf(sA0[kk][ty * 4 + a], sB0[kk][tx * 4 + b], acc0[a][b]);
                        if (SWIGLU)
                            acc1[a][b] = fmaf(sA1[kk][ty * 4 + a], sB1[kk][tx * 4 + b], acc1[a][b]);
                    }
            }
        }
    }
    T* C = static_cast<T*>(g.C);
    for (int a = 0; a < 4; ++a)
        for (int b = 0; b < 4; ++b) {
            const int row = row0 + ty * 4 + a, col = n0 + tx * 4 + b;
            if (row < row_end && col < g.N) {
                const float v = SWIGLU ? silu_f32(acc0[a][b]) * acc1[a][b] : acc0[a][b];
                C[(size_t)row * g.N + col] = Store<T>::from_f32(v);
            }
        }
}

// ============================================================================= host side
template <int BM, int BN, int BK, int WM, int WN, bool SWIGLU, bool DUAL_A, int NS = 2, int KG = 1, bool ADD = false,
          bool HF = false>
static int launch_bf16_deep(GemmArgs& g, hipStream_t st) {
    if ((g.add0 != nullptr) != ADD) return MOE_ERR_INVALID;
    if constexpr (HF) {
        // the half-fill kernel addresses rows by 32-bit byte offsets from the operand's base:
        // an operand of 4 GB or more goes to the 32-wide pipeline with its 64-bit pointers
        for (int i = 0; i < g.nseg; ++i) {
            const GemmSeg& sg = g.seg[i];
            const long long a_rows = sg.gather ? (g.P - 1) / (g.row_div > 0 ? g.row_div : 1) + 1 : g.P;
            if (a_rows * sg.K * 2 >= (1ll << 32) || (long long)g.N * sg.K * 2 >= (1ll << 32))
                return launch_bf16_deep<BM, BN, 32, WM, WN, SWIGLU, DUAL_A, NS, KG, ADD, false>(g, st);
        }
    }
    constexpr int BN_OUT = SWIGLU ? BN / 2 : BN;
    constexpr int NTHR = (BM / WM) * (BN / WN) * 64 * KG;
    static_assert(NTHR <= 1024, "workgroup size");
    g.m_tiles_max = g.P / BM + g.E;
    g.n_tiles = (g.N + BN_OUT - 1) / BN_OUT * ((!SWIGLU && g.C1) ? 2 : 1) * (g.k_parts > 1 ? g.k_parts : 1);
    const int total = g.m_tiles_max * g.n_tiles;
    constexpr size_t lds = KG * 2 * ((size_t)BM * BK * 2 * (DUAL_A ? 2 : 1) + (size_t)BN * BK * 2);
    static_assert(lds <= 160 * 1024, "LDS stages exceed the CU's 160 KB");
    // workgroups of this kernel that one XCD (32 CUs) holds at a time: bounded by LDS and, for
    // these tiles (64 or more accumulator registers per lane), by two waves per SIMD; halves of
    // BM / 2 rows only make sense when each wave's rows fall in one half
    constexpr int kWavesPerSimd = (WM * WN / 64 >= 64) ? 2 : 3;  // by accumulator registers per lane
    constexpr int kByLds = (int)((160 * 1024) / lds), kByWaves = kWavesPerSimd * 256 / NTHR;
    constexpr int kPerCU = kByLds < kByWaves ? kByLds : kByWaves;
    // (for kernels that run one or two workgroups per CU.  It needs a full round before the thin
    // one: with less than one round of tiles in all, halves -- which each still stream the whole
    // weight tile -- measured slower, down product at 512 tokens 94 us instead of 73.  Cutting the
    // halves once more along the columns, one wave of four left with work, was slower too:
    // down product at 2048 tokens 152 us against 144.)
    g.split_slots = (BM / 2) % WM == 0 && KG == 1 && kPerCU <= 2 ? 32 * kPerCU : 0;
    const int grid = ((total + 7) / 8 + g.split_slots / 2) * 8;
    bool tail = false;
    for (int i = 0; i < g.nseg; ++i) {
        const int K = g.seg[i].K;  // rows are read in 16-byte chunks; a K tail only without k-groups
        if (K < 8 || K % 8 != 0 || (KG > 1 && K % (BK * KG) != 0)) return MOE_ERR_UNSUPPORTED;
        tail |= K % BK != 0;
    }
    static std::atomic<uint64_t> lds_allowed[2];
    auto launch = [&](auto kern, int which) {
        if (lds > 32 * 1024 &&
            allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds, lds_allowed[which]) != MOE_OK)
            return (int)MOE_ERR_LAUNCH;
        hipLaunchKernelGGL(kern, dim3(grid), dim3(NTHR), lds, st, g);
        return launch_status();
    };
    if constexpr (KG == 1) {
        if (tail) return launch(gemm_bf16_deep_kernel<BM, BN, BK, WM, WN, SWIGLU, DUAL_A, NS, KG, ADD, true, HF>, 1);
    }
    return launch(gemm_bf16_deep_kernel<BM, BN, BK, WM, WN, SWIGLU, DUAL_A, NS, KG, ADD, false, HF>, 0);
}

template <typename T, bool SWIGLU>
static int launch_simple(GemmArgs& g, hipStream_t st) {
    g.m_tiles_max = g.P / 64 + g.E;
    g.n_tiles = (g.N + 63) / 64;
    hipLaunchKernelGGL((gemm_simple_kernel<T, SWIGLU>), dim3(g.m_tiles_max * g.n_tiles), dim3(256),
                       0, st, g);
    return launch_status();
}

static int run_gemm(const moe_shape& s, GemmArgs& g, bool swiglu, hipStream_t st) {
    if (g.P == 0) return MOE_OK;
    if (g.add0 && (!g.add1 || !g.row_map || !swiglu || s.act_dtype != MOE_BF16)) return MOE_ERR_INVALID;
    for (int i = 0; g.add0 && i < g.nseg; ++i)
        if (g.seg[i].K % 8 != 0) return MOE_ERR_UNSUPPORTED;  // addends exist only in the deep kernels
    const int n_eff = g.N * (g.C1 ? 2 : 1);  // output columns of the launch
    bool dual = false, fast = s.act_dtype != MOE_F32;
    for (int i = 0; i < g.nseg; ++i) {
        dual |= swiglu && g.seg[i].A1 != g.seg[i].A0;
        fast &= g.seg[i].K >= 8 && g.seg[i].K % 8 == 0;  // the deep pipeline reads 16-byte chunks
    }
    if (g.C1 && !fast) {  // only the deep kernel takes two products per launch: run them one by one
        GemmArgs second = g;
        second.C = g.C1;
        second.C1 = nullptr;
        for (int i = 0; i < g.nseg; ++i) {
            second.seg[i].A0 = g.seg[i].A1;
            second.seg[i].B0 = g.seg[i].B1;
        }
        g.C1 = nullptr;
        const int rc = run_gemm(s, g, swiglu, st);
        return rc != MOE_OK ? rc : run_gemm(s, second, swiglu, st);
    }
    if (s.act_dtype == MOE_F32)
        return swiglu ? launch_simple<float, true>(g, st) : launch_simple<float, false>(g, st);
    if (fast) {
        // Tile choice, measured on the 2048 / 5632 and 1024 / 2816 shapes with uniform and Zipf-skewed
        // groups, from 16 to 2048 tokens.  Enough 256 x 256 tiles to fill 256 CUs: those, on 8 waves
        // (64 x 128 per wave, two waves per SIMD), with 64-wide k-steps filled in halves where the
        // kernel has one activation operand.  Below that the products are bound by streaming the
        // weights, and what counts is enough workgroups to pull them with every CU: 128 x 128 x 64
        // tiles (two workgroups per CU), 64-row tiles once the groups hold about 128 rows or
        // fewer, and for a plain product with few tiles and a long K two k-groups per workgroup
        // (on 64 x 64 tiles while the groups average 64 rows or less).
        const int n256 = (n_eff + (swiglu ? 127 : 255)) / (swiglu ? 128 : 256);
        const long long big_tiles = (long long)(g.P / 256 + (g.E + 1) / 2) * n256;
        // A plain product with a narrow output has too few 256 x 256 tiles for 256 CUs (the
        // 2048-wide down projection of 4096 rows: 160), and smaller tiles move two to four times
        // the operand bytes into the CUs.  If the consumer can add partial outputs, the k-steps
        // of every tile are cut into 2-4 parts, each a workgroup's: the count that minimises
        // rounds x (k-steps per part + about 12 k-steps of fixed cost per workgroup).  Worth it
        // from about 24 rows per expert on, when four parts of every tile (one per expert at
        // least) make some 220 workgroups: the 2048-wide down projection from 128 tokens on (45 us
        // against 53, 79 against 111 at 1024 tokens, 116 against 142 at 2048), the 1024-wide one
        // from 1024 tokens on.
        const int max_parts = g.k_parts;
        g.k_parts = 0;
        if (!swiglu && !g.C1 && !g.add0 && g.nseg == 1 && max_parts >= 2 && g.P > 24 * g.E && big_tiles < 400 &&
            g.seg[0].K % 32 == 0 && g.seg[0].K >= 32 * 64 && (long long)(g.P / 256 + g.E) * n256 * 4 >= 224) {
            const int steps = g.seg[0].K / 32;
            long long best = 0;
            for (int q = 2; q <= (max_parts < 4 ? max_parts : 4); ++q) {
                const long long rounds = (big_tiles * q + 255) / 256;
                const long long cost = rounds * (steps / q + 12);
                if (g.k_parts == 0 || cost < best) {
                    best = cost;
                    g.k_parts = q;
                }
            }
            return launch_bf16_deep<256, 256, 64, 64, 128, false, false, 2, 1, false, true>(g, st);
        }
        if (swiglu && !dual && !g.add0 && g.P >= 128 * g.E && big_tiles >= 320)
            return launch_bf16_deep<256, 256, 64, 64, 128, true, false, 2, 1, false, true>(g, st);
        if (g.P >= 384 * g.E && big_tiles >= 400) {  // enough 256 x 256 tiles to fill 256 CUs
            if (swiglu && g.add0) return launch_bf16_deep<256, 256, 32, 64, 128, true, true, 2, 1, true>(g, st);
            if (swiglu) return launch_bf16_deep<256, 256, 32, 64, 128, true, true>(g, st);  // two activation operands
            return launch_bf16_deep<256, 256, 64, 64, 128, false, false, 2, 1, false, true>(g, st);
        }
        const bool small_groups = g.P <= 128 * g.E;
        if (swiglu && g.add0)
            return small_groups ? launch_bf16_deep<64, 128, 64, 32, 64, true, true, 2, 1, true>(g, st)
                                : launch_bf16_deep<128, 128, 64, 64, 64, true, true, 2, 1, true>(g, st);
        if (swiglu) {
            if (small_groups)
                return dual ? launch_bf16_deep<64, 128, 64, 32, 64, true, true>(g, st)
                            : launch_bf16_deep<64, 128, 64, 32, 64, true, false>(g, st);
            return dual ? launch_bf16_deep<128, 128, 64, 64, 64, true, true>(g, st)
                        : launch_bf16_deep<128, 128, 64, 64, 64, true, false>(g, st);
        }
        const long long tiles128 = (long long)(g.P / 128 + (g.E + 1) / 2) * ((n_eff + 127) / 128);
        bool k_pairs = true;
        for (int i = 0; i < g.nseg; ++i) k_pairs &= g.seg[i].K % 128 == 0;
        if (tiles128 < 160 && k_pairs) {
            // (64 x 64: the 1024-wide down projection at 16 rows per expert 16.4 us against 20.1 with
            // 64 x 128, at 32 rows 17.2 against 21.1, at 64 rows 18.1 against 21.8, at 128 rows 24.6
            // against 22.3)
            if (g.P <= 64 * g.E) return launch_bf16_deep<64, 64, 64, 32, 32, false, false, 2, 2>(g, st);
            return launch_bf16_deep<64, 128, 64, 32, 64, false, false, 2, 2>(g, st);
        }
        return launch_bf16_deep<128, 128, 64, 64, 64, false, false>(g, st);
    }
    return MOE_ERR_UNSUPPORTED;  // bf16 rows that are not whole 16-byte chunks (the entry points reject them)
}

// Partial outputs the final down projection of this shape may leave (room the caller provides):
// only tall groups are ever cut along K (see run_gemm).
int down_parts_capacity(const moe_shape& s) {
    const long long P = (long long)s.n_tokens * s.top_k;
    return (s.act_dtype == MOE_BF16 && P > 24ll * s.n_experts) ? kMaxDownParts : 1;
}

// The per-token treatment of a shared base needs the deep bf16 kernels (every K a multiple of 8,
// which the shape check of the entry points already demands) and pays only when a token has more
// than one expert.
bool token_base_supported(const moe_shape& s) {
    return (s.flags & MOE_FLAG_SHARED_BASE) && s.rank > 0 && s.top_k > 1 && s.act_dtype == MOE_BF16 &&
           s.d_model % 8 == 0 && s.d_ff % 8 == 0 && s.rank % 8 == 0;
}

// scratch: h [P,F], then (rank > 0) tg, tu, td [P,r]; with a per-token shared base also the base
// gate and up products and the gate-mixed h [T,F] each; all in the activation type
size_t ffn_scratch_bytes(const moe_shape& s) {
    const size_t P = (size_t)s.n_tokens * s.top_k, es = elt_size(s.act_dtype);
    size_t n = round_up(P * s.d_ff * es, 256) + 3 * round_up(P * s.rank * es, 256);
    if (token_base_supported(s)) n += 3 * round_up((size_t)s.n_tokens * s.d_ff * es, 256);
    return n;
}

int launch_expert_ffn(const moe_shape& s, const moe_weights& w, const void* x,
                      const int32_t* a_row_map, int a_row_div, const int32_t* offsets,
                      void* y_perm, void* scratch, hipStream_t st, StageTimer* timer, int* y_parts) {
    const int d = s.d_model, F = s.d_ff, r = s.rank, E = s.n_experts;
    const int P = s.n_tokens * s.top_k;
    if (P == 0) return MOE_OK;
    const size_t es = elt_size(s.act_dtype);
    char* sc = static_cast<char*>(scratch);
    void* h = sc;
    sc += round_up((size_t)P * F * es, 256);
    void* tg = sc;
    sc += round_up((size_t)P * r * es, 256);
    void* tu = sc;
    sc += round_up((size_t)P * r * es, 256);
    void* td = sc;
    const bool base = (r == 0) || (s.flags & MOE_FLAG_SHARED_BASE);
    const int gather = a_row_map ? 1 : 0;
    int rc;
    auto fresh = [&]() {
        GemmArgs g{};
        g.offsets = offsets; g.row_map = a_row_map; g.row_div = a_row_div > 0 ? a_row_div : 1;
        g.E = E; g.P = P;
        return g;
    };
    if (r > 0) {  // tg = x R_g^T, tu = x R_u^T   [P, r], both in one launch
        GemmArgs g = fresh();
        g.nseg = 1; g.N = r; g.C = tg; g.C1 = tu;
        g.seg[0] = GemmSeg{x, x, w.rg, w.ru, (long long)r * d, d, gather};
        if ((rc = run_gemm(s, g, false, st)) != MOE_OK) return rc;
        stage_mark(timer, "gemm_rank_gate_up");
    }
    {  // h = silu(M_gate x) * (M_up x)   [P, F]
        GemmArgs g = fresh();
        int ns = 0;
        if (base) g.seg[ns++] = GemmSeg{x, x, w.w_gate, w.w_up, r == 0 ? (long long)F * d : 0, d, gather};
        if (r > 0) g.seg[ns++] = GemmSeg{tg, tu, w.lg, w.lu, (long long)F * r, r, 0};
        g.nseg = ns; g.N = F; g.C = h;
        if ((rc = run_gemm(s, g, true, st)) != MOE_OK) return rc;
        stage_mark(timer, "gemm_gate_up_swiglu");
    }
    if (r > 0) {  // td = h R_d^T   [P, r]
        GemmArgs g = fresh();
        g.nseg = 1; g.N = r; g.C = td; g.n_inner = kHiddenOperandBlock;
        g.seg[0] = GemmSeg{h, h, w.rd, w.rd, (long long)r * F, F, 0};
        if ((rc = run_gemm(s, g, false, st)) != MOE_OK) return rc;
        stage_mark(timer, "gemm_rank_down");
    }
    {  // y_perm = M_down h   [P, d]
        GemmArgs g = fresh();
        int ns = 0;
        if (base) g.seg[ns++] = GemmSeg{h, h, w.w_down, w.w_down, r == 0 ? (long long)d * F : 0, F, 0};
        if (r > 0) g.seg[ns++] = GemmSeg{td, td, w.ld, w.ld, (long long)d * r, r, 0};
        g.nseg = ns; g.N = d; g.C = y_perm; g.n_inner = kHiddenOperandBlock;
        // *y_parts in: how many outputs [P, d] the caller's y_perm has room for
        if (y_parts) {
            g.k_parts = *y_parts;
            g.part_stride = (long long)P * d;
        }
        if ((rc = run_gemm(s, g, false, st)) != MOE_OK) return rc;
        if (y_parts) *y_parts = g.k_parts > 1 ? g.k_parts : 1;
        stage_mark(timer, "gemm_down");
    }
    return MOE_OK;
}

// M_e = M0 + L_e R_e with M0 shared by all experts.  Per token t with experts e_j and gates g_j:
//   gate/up:  M0 x_t is the same for every j, so it is computed once per token (a plain product
//             over T rows) and added, per pair, to the low-rank term in the SwiGLU epilogue;
//   down:     sum_j g_j M0 h_tj = M0 (sum_j g_j h_tj): the shared matrix meets the gate-mixed
//             hidden vector once per token; the low-rank terms stay per pair and are mixed by
//             the combine, which also adds the shared part.
// This halves the base work at k = 2 (6 T d F flops instead of 6 P d F).
int launch_expert_ffn_token_base(const moe_shape& s, const moe_weights& w, const void* x,
                                 const int32_t* perm, const int32_t* inv_perm, const float* topk_gate,
                                 const int32_t* offsets, void* y_perm, void* y_base, void* scratch,
                                 hipStream_t st, StageTimer* timer) {
    const int d = s.d_model, F = s.d_ff, r = s.rank, E = s.n_experts, T = s.n_tokens;
    const int P = T * s.top_k;
    if (P == 0) return MOE_OK;
    const size_t es = elt_size(s.act_dtype);
    char* sc = static_cast<char*>(scratch);
    auto take = [&](size_t bytes) {
        void* at = sc;
        sc += round_up(bytes, 256);
        return at;
    };
    void* h = take((size_t)P * F * es);
    void* tg = take((size_t)P * r * es);
    void* tu = take((size_t)P * r * es);
    void* td = take((size_t)P * r * es);
    void* bg = take((size_t)T * F * es);
    void* bu = take((size_t)T * F * es);
    void* z = take((size_t)T * F * es);
    int rc;
    auto grouped = [&]() {  // rows = pairs in expert order
        GemmArgs g{};
        g.offsets = offsets; g.row_map = perm; g.row_div = s.top_k; g.E = E; g.P = P;
        return g;
    };
    auto per_token = [&]() {  // rows = tokens, one group, one matrix
        GemmArgs g{};
        g.offsets = nullptr; g.row_map = nullptr; g.row_div = 1; g.E = 1; g.P = T;
        return g;
    };
    {  // tg = x R_g^T, tu = x R_u^T   [P, r]
        GemmArgs g = grouped();
        g.nseg = 1; g.N = r; g.C = tg; g.C1 = tu;
        g.seg[0] = GemmSeg{x, x, w.rg, w.ru, (long long)r * d, d, 1};
        if ((rc = run_gemm(s, g, false, st)) != MOE_OK) return rc;
        stage_mark(timer, "gemm_rank_gate_up");
    }
    {  // bg = x M0_gate^T, bu = x M0_up^T   [T, F]
        GemmArgs g = per_token();
        g.nseg = 1; g.N = F; g.C = bg; g.C1 = bu;
        g.seg[0] = GemmSeg{x, x, w.w_gate, w.w_up, 0, d, 0};
        if ((rc = run_gemm(s, g, false, st)) != MOE_OK) return rc;
        stage_mark(timer, "gemm_base_gate_up");
    }
    {  // h = silu(bg[t] + tg L_g^T) * (bu[t] + tu L_u^T)   [P, F]
        GemmArgs g = grouped();
        g.nseg = 1; g.N = F; g.C = h; g.add0 = bg; g.add1 = bu;
        g.seg[0] = GemmSeg{tg, tu, w.lg, w.lu, (long long)F * r, r, 0};
        if ((rc = run_gemm(s, g, true, st)) != MOE_OK) return rc;
        stage_mark(timer, "gemm_gate_up_swiglu");
    }
    {  // td = h R_d^T   [P, r]
        GemmArgs g = grouped();
        g.nseg = 1; g.N = r; g.C = td; g.n_inner = kHiddenOperandBlock;
        g.seg[0] = GemmSeg{h, h, w.rd, w.rd, (long long)r * F, F, 0};
        if ((rc = run_gemm(s, g, false, st)) != MOE_OK) return rc;
        stage_mark(timer, "gemm_rank_down");
    }
    {  // z[t] = sum_j g_tj h[slot(t, j)]   [T, F]
        moe_shape sm = s;
        sm.d_model = F;
        if ((rc = launch_combine(sm, h, inv_perm, topk_gate, nullptr, z, st)) != MOE_OK) return rc;
        stage_mark(timer, "mix_hidden");
    }
    {  // y_base = z M0_down^T   [T, d]
        GemmArgs g = per_token();
        g.nseg = 1; g.N = d; g.C = y_base; g.n_inner = kHiddenOperandBlock;
        g.seg[0] = GemmSeg{z, z, w.w_down, w.w_down, 0, F, 0};
        if ((rc = run_gemm(s, g, false, st)) != MOE_OK) return rc;
        stage_mark(timer, "gemm_base_down");
    }
    {  // y_perm = td L_d^T   [P, d]
        GemmArgs g = grouped();
        g.nseg = 1; g.N = d; g.C = y_perm;
        g.seg[0] = GemmSeg{td, td, w.ld, w.ld, (long long)d * r, r, 0};
        if ((rc = run_gemm(s, g, false, st)) != MOE_OK) return rc;
        stage_mark(timer, "gemm_down");
    }
    return MOE_OK;
}

}  // namespace moe
