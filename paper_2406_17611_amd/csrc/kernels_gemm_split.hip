// Dense feature transform of eq. (2) and its gradients for fp32-stored activations, computed on the bf16
// matrix cores from exact bf16 expansions of the fp32 operands:
//     x = x0 + x1 + x2,   x0 = bf16(x), x1 = bf16(x - x0), x2 = bf16(x - x0 - x1)
// (each difference is exact in fp32, and three 8-bit significands cover the 24 bits of x), so
//     a * b = a0 b0 + (a0 b1 + a1 b0) + (a1 b1 + a0 b2 + a2 b0) + terms below 2^-24 |a b|.
// The six kept products are exact in the fp32 accumulators of v_mfma_f32_32x32x16_bf16, which leaves the
// result with the accuracy of an fp32 product-sum; six bf16 instructions cost 6/16 of the fp32 matrix
// instructions that cover the same reduction steps. TERMS = 2 keeps x0 + x1 and three products (relative
// error about 2^-16 per product); the library does not use it by default.
//
// A workgroup of four wavefronts computes a 128 x 128 tile of C (128 x 64 for outputs at most 64 columns wide), a
// wavefront 64 x 64 (32 x 64); two workgroups are resident per compute unit (see the kernel). A stage of 32
// reduction steps is fetched into registers one step ahead, then expanded and written to LDS as TERMS planes of
// bf16 rows (one output index per row, reduction index contiguous, 80-byte pitch).
//   "NT" products (transform, input gradient): A has the reduction index contiguous and is expanded here;
//        B is the library's own expanded copy of the weights (varco_launch_prep_weight_split), zero-padded
//        to whole tiles and copied as is.
//   "TN" products (weight gradient, reduction over nodes): both operands have the node index as the slow
//        one; a thread loads an 8 (nodes) x 4 (columns) block with eight 16-byte loads and expands the values of
//        two consecutive nodes of a column together, which yields the transposed (node index contiguous) words
//        directly; it writes four 16-byte LDS rows per plane. Half the threads serve A, half B.
// The ReLU mask of the backward pass is applied before the expansion, the activation in the epilogue.
#include <type_traits>

#include "elem.h"
#include "varco_internal.h"

namespace {

constexpr int BK = 32;
constexpr int kThreads = 256;
constexpr int kPitch = BK + 8;   // bf16 elements per LDS row (80 bytes)
constexpr int kPrepRows = 128;   // expanded weight copies are padded to this many rows (the widest B tile) and to BK columns

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct SplitOperand {
    const void* ptr;      // fp32 matrix, or the expanded bf16 copy of a weight matrix
    const float* gate;
    int64_t ld;
    int64_t plane;        // elements between the planes of an expanded copy
};

struct SplitGemm {
    int32_t m, n, k, k2;
    SplitOperand a, b, a2, b2;
    float* c;
    int64_t ldc;
    int32_t accumulate, relu;
    int32_t split_k, tiles_per_split;
    float* partial;
    int32_t tiles_m, tiles_n;
    int32_t inner, outer;            // tiles along the fast and the slow direction of the workgroup order
};


typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

// Two fp32 values rounded to bf16 (nearest even) by one packed conversion; `lo` in the low half.
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    const floatx2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// Expansion of two fp32 values: w[p] holds term p of both (x0 in the low half).
template <int TERMS>
__device__ __forceinline__ void expand_pair(float x0, float x1, uint32_t (&w)[TERMS]) {
#pragma unroll
    for (int p = 0; p < TERMS; ++p) {
        w[p] = pack_bf16(x0, x1);
        if (p + 1 < TERMS) {
            x0 -= __uint_as_float(w[p] << 16);
            x1 -= __uint_as_float(w[p] & 0xFFFF0000u);
        }
    }
}

__device__ __forceinline__ float4 gate4(float4 x, float4 y) {
    x.x = y.x > 0.f ? x.x : 0.f, x.y = y.y > 0.f ? x.y : 0.f;
    x.z = y.z > 0.f ? x.z : 0.f, x.w = y.w > 0.f ? x.w : 0.f;
    return x;
}

// Consecutive groups of lanes write consecutive tile rows; with an 80-byte pitch rows r and r + 1 overlap in
// four LDS banks while rows r and r + 4 tile all of them, so the q-th row group of a wavefront goes to row
// (q with its low three bits rotated): 0 4 1 5 2 6 3 7.
__device__ __forceinline__ int tile_row(int q) { return (q & ~7) | ((q & 1) << 2) | ((q >> 1) & 3); }

template <typename T>
__device__ __forceinline__ T load_at(const void* base, uint32_t byte_offset) {
    return *reinterpret_cast<const T*>(static_cast<const char*>(base) + byte_offset);
}

// ---- fp32 operand with the reduction index contiguous: chunks of CH floats ----
// Addresses are a per-tile base (uniform) plus a 32-bit offset per chunk that does not change along the
// reduction. Rows beyond the matrix are clamped to its last row (their results are never stored); chunks
// beyond the reduction length re-read the tile's first chunk of the same row, and meet zeros in B.
template <int ROWS, int CH, bool GATE>
struct RowRegs {
    static constexpr int PER_ROW = BK / CH;
    static constexpr int N = ROWS * PER_ROW / kThreads;
    float4 v[N][CH / 4];
    float4 g[GATE ? N : 1][CH / 4];
};

template <int ROWS, int CH>
struct RowPlan {
    static constexpr int PER_ROW = BK / CH;
    static constexpr int N = ROWS * PER_ROW / kThreads;
    uint32_t off[N];     // bytes from the tile base
    __device__ __forceinline__ void init(int tid, int32_t i0, int32_t extent, int64_t ld) {
#pragma unroll
        for (int h = 0; h < N; ++h) {
            const int c = tid + h * kThreads;
            const int32_t r = min(tile_row(c / PER_ROW), extent - 1 - i0);
            off[h] = uint32_t(r * ld + (c % PER_ROW) * CH) * 4u;
        }
    }
};

template <int ROWS, int CH, bool GATE>
__device__ __forceinline__ void load_rows(int tid, const float* base, const float* gate, const RowPlan<ROWS, CH>& plan,
                                          int32_t k_left, RowRegs<ROWS, CH, GATE>& r) {
    using R = RowRegs<ROWS, CH, GATE>;
#pragma unroll
    for (int h = 0; h < R::N; ++h) {
        const int kc = ((tid + h * kThreads) % R::PER_ROW) * CH;
        const uint32_t off = kc < k_left ? plan.off[h] : plan.off[h] - uint32_t(kc) * 4u;   // k_left is a multiple of CH
#pragma unroll
        for (int u = 0; u < CH / 4; ++u) {
            r.v[h][u] = load_at<float4>(base, off + 16u * u);
            if (GATE) r.g[h][u] = load_at<float4>(gate, off + 16u * u);
        }
    }
}

template <int TERMS, int ROWS, int CH, bool GATE>
__device__ __forceinline__ void store_rows(int tid, const RowRegs<ROWS, CH, GATE>& r, uint16_t* s) {
    using R = RowRegs<ROWS, CH, GATE>;
#pragma unroll
    for (int h = 0; h < R::N; ++h) {
        const int c = tid + h * kThreads;
        uint32_t w[CH / 2][TERMS];
#pragma unroll
        for (int u = 0; u < CH / 4; ++u) {
            float4 x = r.v[h][u];
            if (GATE) x = gate4(x, r.g[h][u]);
            expand_pair<TERMS>(x.x, x.y, w[2 * u]);
            expand_pair<TERMS>(x.z, x.w, w[2 * u + 1]);
        }
        uint16_t* dst = s + tile_row(c / R::PER_ROW) * kPitch + (c % R::PER_ROW) * CH;
#pragma unroll
        for (int p = 0; p < TERMS; ++p) {
            if constexpr (CH == 8)
                *reinterpret_cast<uint4*>(dst + p * ROWS * kPitch) = make_uint4(w[0][p], w[1][p], w[2][p], w[3][p]);
            else
                *reinterpret_cast<uint2*>(dst + p * ROWS * kPitch) = make_uint2(w[0][p], w[1][p]);
        }
    }
}

// ---- expanded bf16 weight copy: chunks of 8 elements, copied unchanged ----
// The copy is stored by tile and stage, [row tile][stage of BK reduction steps][term][row in tile][BK], so that what
// a workgroup fetches per step is one contiguous block (whole cache lines, one 1 KB run per wavefront load), and it
// is zero-padded to whole tiles and stages, so no chunk needs a bounds check.
template <int TERMS, int ROWS>
struct PrepRegs {
    static constexpr int PER_ROW = BK / 8;
    static constexpr int N = TERMS * ROWS * PER_ROW / kThreads;
    uint4 v[N];
};

template <int TERMS, int ROWS>
struct PrepPlan {
    static constexpr int PER_ROW = BK / 8;
    static constexpr int N = TERMS * ROWS * PER_ROW / kThreads;
    uint32_t off[N];     // bytes from the block's base
    __device__ __forceinline__ void init(int tid) {
#pragma unroll
        for (int h = 0; h < N; ++h) {
            const int c = tid + h * kThreads;
            const int p = c / (ROWS * PER_ROW), rc = c % (ROWS * PER_ROW);
            off[h] = uint32_t((p * ROWS + tile_row(rc / PER_ROW)) * BK + (rc % PER_ROW) * 8) * 2u;
        }
    }
};

template <int TERMS, int ROWS>
__device__ __forceinline__ void load_prep(const uint16_t* base, const PrepPlan<TERMS, ROWS>& plan, PrepRegs<TERMS, ROWS>& r) {
#pragma unroll
    for (int h = 0; h < PrepRegs<TERMS, ROWS>::N; ++h) r.v[h] = load_at<uint4>(base, plan.off[h]);
}

template <int TERMS, int ROWS>
__device__ __forceinline__ void store_prep(int tid, const PrepRegs<TERMS, ROWS>& r, uint16_t* s) {
    using R = PrepRegs<TERMS, ROWS>;
#pragma unroll
    for (int h = 0; h < R::N; ++h) {
        const int c = tid + h * kThreads;
        const int p = c / (ROWS * R::PER_ROW), rc = c % (ROWS * R::PER_ROW);
        *reinterpret_cast<uint4*>(s + p * ROWS * kPitch + tile_row(rc / R::PER_ROW) * kPitch + (rc % R::PER_ROW) * 8) = r.v[h];
    }
}

// ---- fp32 operand with the output index contiguous: one 8 (reduction) x 4 (output) block per thread ----
// Block b of an operand's tile covers reduction steps 8 * (b % 4) .. + 7 and output indices 4 * (b / 4) .. + 3:
// eight consecutive lanes then write two LDS rows that are four rows apart, all four 16-byte chunks of each,
// which touches every LDS bank once. Output indices beyond the matrix are clamped (their results are never
// stored). In the last, partial tile of the reduction the node index is clamped and A is zeroed beyond it.
template <bool GATE>
struct ColRegs {
    float4 v[8];
    float4 g[GATE ? 8 : 1];
};

__device__ __forceinline__ uint32_t col_offset(int b, int32_t i0, int32_t extent) {
    return uint32_t(min(i0 + (b >> 2) * 4, extent - 4) - i0) * 4u;      // bytes; extent is a multiple of 4
}

template <bool GATE, bool TAIL, bool ZERO>
__device__ __forceinline__ void load_cols(const float* base, const float* gate, int b, uint32_t col_off, uint32_t ld_bytes,
                                          int32_t k_left, ColRegs<GATE>& r) {
    const int kb = (b & 3) * 8;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
        const int node = TAIL ? min(kb + kk, k_left - 1) : kb + kk;
        const uint32_t off = uint32_t(node) * ld_bytes + col_off;
        r.v[kk] = load_at<float4>(base, off);
        if (GATE) r.g[kk] = load_at<float4>(gate, off);
        if (TAIL && ZERO && kb + kk >= k_left) r.v[kk] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
}

// The same block of an operand whose rows are not 16-byte aligned or whose width is not a multiple of 4 (the 47
// class columns of the last layer): element loads; columns beyond the matrix repeat its last one (their products
// are never stored), nodes beyond the reduction repeat the last one (the other operand is zero there).
__device__ __forceinline__ void load_cols_ragged(const float* base, int b, int32_t i0, int32_t extent, uint32_t ld_bytes,
                                                 int32_t k_left, ColRegs<false>& r) {
    const int kb = (b & 3) * 8;
    uint32_t off[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) off[e] = uint32_t(min(i0 + (b >> 2) * 4 + e, extent - 1) - i0) * 4u;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
        const uint32_t row = uint32_t(min(kb + kk, k_left - 1)) * ld_bytes;
        r.v[kk] = make_float4(load_at<float>(base, row + off[0]), load_at<float>(base, row + off[1]),
                              load_at<float>(base, row + off[2]), load_at<float>(base, row + off[3]));
    }
}

template <int TERMS, int ROWS, bool GATE>
__device__ __forceinline__ void store_cols(const ColRegs<GATE>& r, int b, uint16_t* s) {
    // An LDS row holds one output index with its 8 reduction steps contiguous, two steps per 32-bit word: the two
    // values expanded together are steps 2 q and 2 q + 1 of one output index, which is the transposition itself.
    float x[8][4];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
        float4 v = r.v[kk];
        if constexpr (GATE) v = gate4(v, r.g[kk]);
        x[kk][0] = v.x, x[kk][1] = v.y, x[kk][2] = v.z, x[kk][3] = v.w;
    }
    uint16_t* base = s + (b >> 2) * 4 * kPitch + (b & 3) * 8;
#pragma unroll
    for (int ii = 0; ii < 4; ++ii) {                          // output index i + ii: its 8 reduction steps
        uint32_t o[4][TERMS];
#pragma unroll
        for (int q = 0; q < 4; ++q) expand_pair<TERMS>(x[2 * q][ii], x[2 * q + 1][ii], o[q]);
#pragma unroll
        for (int p = 0; p < TERMS; ++p)
            *reinterpret_cast<uint4*>(base + p * ROWS * kPitch + ii * kPitch) = make_uint4(o[0][p], o[1][p], o[2][p], o[3][p]);
    }
}

__device__ __forceinline__ bf16x8 fragment(const uint16_t* s, int row, int koff) {
    return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(s + row * kPitch + koff));
}

template <int TMB, int TNB, int PA, int PB>
__device__ __forceinline__ void multiply(const bf16x8 (&fa)[3][TMB], const bf16x8 (&fb)[3][TNB], floatx16 (&acc)[TMB][TNB]) {
#pragma unroll
    for (int i = 0; i < TMB; ++i)
#pragma unroll
        for (int j = 0; j < TNB; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[PA][i], fb[PB][j], acc[i][j], 0, 0, 0);
}

// All wavefronts of the workgroup meet here (same fences as __syncthreads); the two halves of a workgroup call
// it from different places, always the same number of times.
__device__ __forceinline__ void workgroup_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

// TN: both operands stored with the output index contiguous (weight gradient), else A with the reduction
// index contiguous and B an expanded weight copy. WM x WN wavefronts per tile, each TMB x TNB blocks of
// 32 x 32. A_CH: floats per chunk of A (NT); in a TN product A_CH = 1 says that B is read element by element
// (unaligned rows, never masked). GATE masks A (NT) or B (TN).
//
// A workgroup is four wavefronts with one tile and one LDS stage (60 KB), so that two workgroups are resident
// on a compute unit and each SIMD holds one wavefront of either. On this device the vector ALU and the matrix
// unit of a SIMD do not run side by side (hardware counters: their busy times add up), so nothing is gained by
// steering one wavefront's conversions under the other's products; what matters is that the SIMD always has a
// wavefront that can issue, and that as few vector instructions as possible accompany the matrix instructions.
// Two independent workgroups give the first: while one waits at a barrier, for its global loads, or stores its
// tile, the other multiplies. (Two groups in lock step inside one 512-thread workgroup, the previous form, left
// a tile's first fetch and epilogue uncovered and tied both groups to the slower one.)
template <int TERMS, bool TN, int WM, int WN, int TMB, int TNB, int A_CH, bool GATE>
__global__ __launch_bounds__(kThreads, 2) void gemm_split_kernel(SplitGemm g) {
    static_assert(TERMS == 2 || TERMS == 3, "two or three bf16 terms per operand");
    constexpr int BM = 32 * TMB * WM, BN = 32 * TNB * WN;
    static_assert(BM + BN <= kThreads, "one 8 x 4 block per thread in the TN layout");
    static_assert(!(TN && A_CH == 1 && GATE), "an operand read element by element is never masked");
    __shared__ __attribute__((aligned(16))) uint16_t smem[TERMS * (BM + BN) * kPitch];
    const int tid = threadIdx.x;
    uint16_t* const sa = smem;
    uint16_t* const sb = smem + TERMS * BM * kPitch;

    // workgroup -> tile: tiles that share streamed data go to one XCD (workgroups are dealt to the 8 XCDs
    // round-robin), so that the streamed operand is fetched into a single L2
    const int32_t xcd = blockIdx.x & 7, within = blockIdx.x >> 3;
    const int32_t in = within % g.inner, out = (within / g.inner) * 8 + xcd;
    if (out >= g.outer) return;                // whole workgroup leaves together: no barrier is skipped
    const int32_t tiles1 = (g.k + BK - 1) / BK;
    const int32_t tiles2 = (g.k2 + BK - 1) / BK;
    int32_t t_begin = 0, t_end = tiles1 + tiles2;
    int32_t tm, tn, z;
    if (g.split_k > 1) {
        t_begin = out * g.tiles_per_split;
        t_end = min(t_end, t_begin + g.tiles_per_split);
        z = out, tm = in / g.tiles_n, tn = in % g.tiles_n;
    } else {
        z = 0, tm = out, tn = in;
    }
    const int32_t steps = max(t_end - t_begin, 0);
    const int32_t m0 = tm * BM, n0 = tn * BN;

    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // uniform: addresses built from it stay scalar
    const int wm = (wave / WN) * (32 * TMB), wn = (wave % WN) * (32 * TNB);
    const int lrow = lane & 31, lk = lane >> 5;

    floatx16 acc[TMB][TNB];
#pragma unroll
    for (int i = 0; i < TMB; ++i)
#pragma unroll
        for (int j = 0; j < TNB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // staging registers and per-thread offsets of the two layouts (only one set is used per instantiation)
    RowRegs<BM, A_CH, GATE && !TN> ra;
    PrepRegs<TERMS, BN> rb;
    RowPlan<BM, A_CH> plan_a;
    PrepPlan<TERMS, BN> plan_b;
    if constexpr (!TN) {
        plan_a.init(tid, m0, g.m, g.a.ld);        // a chained second product has the same leading dimensions
        plan_b.init(tid);
    }

    auto fetch = [&](int32_t t) {                 // NT
        const bool first = t < tiles1;
        const int32_t k0 = (first ? t : t - tiles1) * BK, k_left = (first ? g.k : g.k2) - k0;
        const float* abase = static_cast<const float*>(first ? g.a.ptr : g.a2.ptr) + int64_t(m0) * g.a.ld + k0;
        const float* gbase = GATE ? g.a.gate + int64_t(m0) * g.a.ld + k0 : nullptr;   // never with a second product
        const uint16_t* bbase = static_cast<const uint16_t*>(first ? g.b.ptr : g.b2.ptr) +
                                (int64_t(tn) * (g.b.ld / BK) + k0 / BK) * (TERMS * BN * BK);      // g.b.ld: padded reduction length
        if constexpr (!TN) {
            load_rows<BM, A_CH, GATE>(tid, abase, gbase, plan_a, k_left, ra);
            load_prep<TERMS, BN>(bbase, plan_b, rb);
        }
    };
    auto stash = [&]() {                          // NT
        if constexpr (!TN) {
            store_rows<TERMS, BM, A_CH, GATE>(tid, ra, sa);
            store_prep<TERMS, BN>(tid, rb, sb);
        }
    };
    auto compute = [&]() {
#pragma unroll
        for (int s = 0; s < BK / 16; ++s) {
            const int koff = s * 16 + lk * 8;
            bf16x8 fa[3][TMB], fb[3][TNB];
#pragma unroll
            for (int p = 0; p < TERMS; ++p) {
#pragma unroll
                for (int i = 0; i < TMB; ++i) fa[p][i] = fragment(sa + p * BM * kPitch, wm + i * 32 + lrow, koff);
#pragma unroll
                for (int j = 0; j < TNB; ++j) fb[p][j] = fragment(sb + p * BN * kPitch, wn + j * 32 + lrow, koff);
            }
            multiply<TMB, TNB, 0, 0>(fa, fb, acc);
            multiply<TMB, TNB, 0, 1>(fa, fb, acc);
            multiply<TMB, TNB, 1, 0>(fa, fb, acc);
            if constexpr (TERMS == 3) {
                multiply<TMB, TNB, 1, 1>(fa, fb, acc);
                multiply<TMB, TNB, 0, 2>(fa, fb, acc);
                multiply<TMB, TNB, 2, 0>(fa, fb, acc);
            }
        }
    };

    // One LDS stage: a step's operands are fetched into registers while the previous step is multiplied, then
    // expanded and written once its fragments have been read. (A second register set, fetching two steps ahead,
    // was measured and changes nothing.)
    auto pipeline = [&](auto&& fetch_fn, auto&& stash_fn) {
        if (steps > 0) fetch_fn(t_begin);
        for (int32_t it = 0; it < steps; ++it) {
            stash_fn();
            if (it + 1 < steps) fetch_fn(t_begin + it + 1);
            workgroup_barrier();
            compute();
            workgroup_barrier();   // the stage's fragments have been read: the next one may overwrite them
        }
    };
    if constexpr (TN) {
        // Every wavefront serves 8 x 4 blocks of one operand only (BM and BN are multiples of 64), so the role is
        // a scalar and each role gets a loop of its own: one shared loop with per-thread role tests made the
        // compiler copy the 32 staging registers between the paths every step.
        const int role = __builtin_amdgcn_readfirstlane(tid < BM ? 0 : (tid < BM + BN ? 1 : 2));
        auto run = [&](auto is_a) {
            constexpr bool A = decltype(is_a)::value;
            constexpr bool G = GATE && !A;
            ColRegs<G> cr;
            const int b = A ? tid : tid - BM;
            constexpr bool RAGGED = !A && A_CH == 1;
            const uint32_t col_off = RAGGED ? 0u : (A ? col_offset(b, m0, g.m) : col_offset(b, n0, g.n));
            const SplitOperand& op = A ? g.a : g.b;
            const uint32_t ld_bytes = uint32_t(op.ld) * 4u;
            auto fetch_cols = [&](int32_t t) {
                const int32_t k0 = t * BK, k_left = g.k - k0;
                const float* base = static_cast<const float*>(op.ptr) + int64_t(k0) * op.ld + (A ? m0 : n0);
                const float* gbase = G ? op.gate + int64_t(k0) * op.ld + n0 : nullptr;
                if constexpr (RAGGED)
                    load_cols_ragged(base, b, n0, g.n, ld_bytes, k_left, cr);
                else if (k_left >= BK)
                    load_cols<G, false, A>(base, gbase, b, col_off, ld_bytes, k_left, cr);
                else
                    load_cols<G, true, A>(base, gbase, b, col_off, ld_bytes, k_left, cr);
            };
            pipeline(fetch_cols, [&]() { store_cols<TERMS, A ? BM : BN, G>(cr, b, A ? sa : sb); });
        };
        if (role == 0)
            run(std::true_type{});
        else if (role == 1)
            run(std::false_type{});
        else
            pipeline([](int32_t) {}, []() {});
    } else {
        pipeline(fetch, stash);
    }
    if (steps == 0) return;

    // epilogue: accumulator register v of a lane is element (8 * (v / 4) + 4 * (lane / 32) + v % 4, lane % 32).
    // A tile that lies wholly inside C (all but the last row and column of tiles) is stored through one scalar
    // base per output row plus one 32-bit lane offset (4 lk rows + lrow columns), so that the address arithmetic
    // runs on the scalar unit and the vector unit only sees the loads, adds and stores; the edge tiles take the
    // path with per-element tests and clamped addresses. When C is added to, the old values of a block are fetched
    // by loads that are all issued before the first one is used, not one round trip per element.
    const bool to_partial = g.split_k > 1;
    const int64_t pitch = to_partial ? int64_t(g.n) : g.ldc;
    float* const base = to_partial ? g.partial + int64_t(z) * g.m * g.n : g.c;
    const bool add_old = !to_partial && g.accumulate, relu = !to_partial && g.relu;
    if (m0 + BM <= g.m && n0 + BN <= g.n) {
        float* const tile = base + int64_t(m0 + wm) * pitch + (n0 + wn);               // scalar
        const uint32_t lane_off = uint32_t(4 * lk) * uint32_t(pitch) + uint32_t(lrow);  // a tile spans < 2^32 elements
#pragma unroll
        for (int i = 0; i < TMB; ++i) {
#pragma unroll
            for (int j = 0; j < TNB; ++j) {
                float old[16];
#pragma unroll
                for (int v = 0; v < 16; ++v) old[v] = 0.f;
                if (add_old) {
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        old[v] = (tile + int64_t(i * 32 + 8 * (v >> 2) + (v & 3)) * pitch + j * 32)[lane_off];
                }
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    float x = acc[i][j][v] + old[v];
                    if (relu) x = fmaxf(x, 0.f);
                    (tile + int64_t(i * 32 + 8 * (v >> 2) + (v & 3)) * pitch + j * 32)[lane_off] = x;
                }
            }
        }
        return;
    }
    const int32_t col_base = n0 + wn + lrow;
#pragma unroll
    for (int i = 0; i < TMB; ++i) {
#pragma unroll
        for (int j = 0; j < TNB; ++j) {
            float* ptr[16];
            bool ok[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int32_t row = m0 + wm + i * 32 + 4 * lk + 8 * (v >> 2) + (v & 3), col = col_base + j * 32;
                ok[v] = row < g.m && col < g.n;
                ptr[v] = base + int64_t(min(row, g.m - 1)) * pitch + min(col, g.n - 1);
            }
            float old[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) old[v] = 0.f;
            if (add_old) {
#pragma unroll
                for (int v = 0; v < 16; ++v) old[v] = *ptr[v];
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float x = acc[i][j][v] + old[v];
                if (relu) x = fmaxf(x, 0.f);
                if (ok[v]) *ptr[v] = x;
            }
        }
    }
}


// ---------------------------------------------------------------------------------------------------------
// Short reductions on the bf16 matrix units: C (+)= A B^T with at most 64 reduction steps and densely stored
// rows of A (the input gradient of the last layer: the reduction runs over the classes). Rows of, say, 47
// elements are not 16-byte aligned, so a workgroup copies its 128 rows of A, one contiguous range of memory,
// into LDS with 16-byte loads (masked and widened to fp32 on the way; the row pitch stays k). Each wavefront
// owns 64 columns of C: their weights, expanded into TERMS bf16 terms, sit in registers as matrix operands for
// the whole kernel; for each block of 32 rows the wavefront reads its 8 values per 16 reduction steps from LDS,
// expands them in registers and issues the products. With fp32 matrix instructions (the previous form of this
// kernel, still used when the context asks for them) the same product took 2.7 times the matrix-unit time and
// was bound by it; this form is bound by writing C. TERMS = 1: bf16 storage (the values are bf16 already; the
// weights are rounded to bf16 as for the other products of that storage type).
constexpr int kShortRows = 128;
constexpr int kEpiPitch = 68;      // floats per row of the epilogue's LDS block (64 + 4: rows start on different banks)

template <typename T>
__device__ __forceinline__ void load_chunk16(const T* p, float (&x)[16 / sizeof(T)]) {
    if constexpr (sizeof(T) == 4) {
        const float4 v = *reinterpret_cast<const float4*>(p);
        x[0] = v.x, x[1] = v.y, x[2] = v.z, x[3] = v.w;
    } else {
        const uint4 v = *reinterpret_cast<const uint4*>(p);
        const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) x[2 * i] = __uint_as_float(u[i] << 16), x[2 * i + 1] = __uint_as_float(u[i] & 0xFFFF0000u);
    }
}

// Eight consecutive values as TERMS bf16 fragments.
template <int TERMS>
__device__ __forceinline__ void expand8(const float (&x)[8], bf16x8 (&f)[3]) {
    uint32_t w[4][TERMS];
#pragma unroll
    for (int q = 0; q < 4; ++q) expand_pair<TERMS>(x[2 * q], x[2 * q + 1], w[q]);
#pragma unroll
    for (int p = 0; p < TERMS; ++p) f[p] = __builtin_bit_cast(bf16x8, make_uint4(w[0][p], w[1][p], w[2][p], w[3][p]));
}
template <>
__device__ __forceinline__ void expand8<1>(const float (&x)[8], bf16x8 (&f)[3]) {
    f[0] = __builtin_bit_cast(bf16x8, make_uint4(pack_bf16(x[0], x[1]), pack_bf16(x[2], x[3]), pack_bf16(x[4], x[5]), pack_bf16(x[6], x[7])));
}

template <typename T, int KS, bool GATE, int TERMS>
__global__ __launch_bounds__(kThreads, 2) void gemm_short_k_kernel(const T* __restrict__ a, const T* __restrict__ gate,
                                                                   const float* __restrict__ b, int64_t ldb, T* __restrict__ c,
                                                                   int64_t ldc, int32_t m, int32_t n, int32_t k,
                                                                   int32_t accumulate) {
    constexpr int VE = 16 / int(sizeof(T));                       // elements per 16-byte load
    __shared__ __attribute__((aligned(16))) float tile[kShortRows * 16 * KS + 64];
    __shared__ __attribute__((aligned(16))) float epi[4 * 32 * kEpiPitch];      // a 32 x 64 block per wavefront
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lcol = lane & 31, lk = lane >> 5;
    const int32_t r0 = blockIdx.x * kShortRows, rows = min(kShortRows, m - r0);
    const int32_t c0 = blockIdx.y * 256 + wave * 64;
    // rows of C can be written 4 elements at a time: whole vectors inside the matrix, aligned
    const bool vec_out = n % 4 == 0 && ldc % 4 == 0 && (reinterpret_cast<uintptr_t>(c) & (4 * sizeof(T) - 1)) == 0;

    // weights of this wavefront's two column blocks: lane holds B[column][16 s + 8 lk .. + 7], expanded
    bf16x8 w[2][KS][3];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const int32_t col = c0 + cb * 32 + lcol;
#pragma unroll
        for (int s2 = 0; s2 < KS; ++s2) {
            float x[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int kk = 16 * s2 + 8 * lk + e;
                x[e] = col < n && kk < k ? b[int64_t(col) * ldb + kk] : 0.f;
            }
            expand8<TERMS>(x, w[cb][s2]);
        }
    }

    // the rows of this tile as one contiguous range, read in 16-byte chunks on 16-byte boundaries (the range
    // may start `skew` elements into a chunk; A and its mask have the same skew, checked by the launcher)
    const int32_t n_el = rows * k;
    const T* src = a + int64_t(r0) * k;
    const T* gsrc = GATE ? gate + int64_t(r0) * k : nullptr;
    const int32_t skew = int32_t((reinterpret_cast<uintptr_t>(src) & 15u) / sizeof(T));
    for (int32_t e0 = threadIdx.x * VE - skew; e0 < n_el; e0 += kThreads * VE) {
        float x[VE], y[VE];
        if (e0 >= 0 && e0 + VE <= n_el) {
            load_chunk16<T>(src + e0, x);
            if (GATE) load_chunk16<T>(gsrc + e0, y);
        } else {
#pragma unroll
            for (int i = 0; i < VE; ++i) {
                const bool in = e0 + i >= 0 && e0 + i < n_el;
                x[i] = in ? Elem<T>::load(src + e0 + i) : 0.f;
                if (GATE) y[i] = in ? Elem<T>::load(gsrc + e0 + i) : 0.f;
            }
        }
#pragma unroll
        for (int i = 0; i < VE; ++i) {
            if (GATE) x[i] = y[i] > 0.f ? x[i] : 0.f;
            if (e0 + i >= 0 && e0 + i < n_el) tile[e0 + i] = x[i];
        }
    }
    __syncthreads();
    if (c0 >= n) return;               // no barrier follows

    for (int rb = 0; rb * 32 < rows; ++rb) {
        const int32_t lrow = min(rb * 32 + lcol, rows - 1);          // rows past the end repeat the last one; never stored
        floatx16 acc[2];
#pragma unroll
        for (int cb = 0; cb < 2; ++cb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[cb][v] = 0.f;
#pragma unroll
        for (int s2 = 0; s2 < KS; ++s2) {
            float x[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int kk = 16 * s2 + 8 * lk + e;
                const float v = tile[lrow * k + kk];                 // in bounds: the tile has 64 spare floats
                x[e] = kk < k ? v : 0.f;
            }
            bf16x8 fa[3];
            expand8<TERMS>(x, fa);
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) {
                auto mul = [&](int pa, int pb) {
                    acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[pa], w[cb][s2][pb], acc[cb], 0, 0, 0);
                };
                mul(0, 0);
                if constexpr (TERMS >= 2) {
                    mul(0, 1);
                    mul(1, 0);
                }
                if constexpr (TERMS == 3) {
                    mul(1, 1);
                    mul(0, 2);
                    mul(2, 0);
                }
            }
        }
        // accumulator register v of a lane is element (8 * (v / 4) + 4 * (lane / 32) + v % 4, lane % 32): a lane holds
        // one column. Stored that way a wavefront needs 32 store instructions of 256 bytes each per block of rows,
        // and the kernel is bound by issuing them; so the block goes through LDS once and leaves as 4-element
        // vectors along the rows (8 stores of 1 KB; the old values of C, when added to, come in the same way).
        if (vec_out) {
            float* ep = epi + wave * (32 * kEpiPitch);
#pragma unroll
            for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                for (int v = 0; v < 16; ++v) ep[(8 * (v >> 2) + 4 * lk + (v & 3)) * kEpiPitch + cb * 32 + lcol] = acc[cb][v];
            // same wavefront writes and reads: no barrier, the LDS operations of a wavefront complete in order
            const int er = lane >> 4, ec = (lane & 15) * 4;
            float4 old[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) old[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (accumulate) {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int32_t row = min(rb * 32 + er + 4 * i, rows - 1);
                    if (c0 + ec < n) old[i] = Elem<T>::load4(c + int64_t(r0 + row) * ldc + c0 + ec);
                }
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int32_t row = rb * 32 + er + 4 * i;
                float4 x = *reinterpret_cast<const float4*>(ep + (er + 4 * i) * kEpiPitch + ec);
                x.x += old[i].x, x.y += old[i].y, x.z += old[i].z, x.w += old[i].w;
                if (row < rows && c0 + ec < n) Elem<T>::store4(c + int64_t(r0 + row) * ldc + c0 + ec, x);
            }
            continue;
        }
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
            const int32_t col = c0 + cb * 32 + lcol;
            const int32_t row0 = rb * 32 + 4 * lk;
            float old[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) old[v] = 0.f;
            if (accumulate) {   // all loads issued before the first use, from clamped (always valid) addresses
                const T* cbase = c + min(col, n - 1);
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    old[v] = Elem<T>::load(cbase + int64_t(r0 + min(row0 + 8 * (v >> 2) + (v & 3), rows - 1)) * ldc);
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int32_t row = row0 + 8 * (v >> 2) + (v & 3);
                if (row < rows && col < n) Elem<T>::store(c + int64_t(r0 + row) * ldc + col, acc[cb][v] + old[v]);
            }
        }
    }
}

// Expanded copy of (transpose ? h[c][r] : h[r][c]), r < rows, c < cols, zero beyond, in the tiled layout the product
// kernel fetches: element (term p, row r, column c) sits at
//   (((r / bn) * (pitch / BK) + c / BK) * TERMS + p) * bn * BK + (r % bn) * BK + c % BK,
// bn = rows of a B tile (64 for at most 64 rows, else 128), rows padded to `rows_padded`, columns to `pitch`.
template <int TERMS>
__global__ __launch_bounds__(kThreads) void prep_weight_split_kernel(const float* __restrict__ h, int64_t ld, int32_t rows,
                                                                     int32_t cols, int32_t rows_padded, int32_t pitch,
                                                                     int32_t bn, int32_t transpose, uint16_t* __restrict__ out) {
    const int64_t idx = int64_t(blockIdx.x) * kThreads + threadIdx.x;
    if (idx >= int64_t(rows_padded) * pitch) return;
    const int32_t r = int32_t(idx / pitch), c = int32_t(idx % pitch);
    float x = 0.f;
    if (r < rows && c < cols) x = transpose ? h[int64_t(c) * ld + r] : h[int64_t(r) * ld + c];
    const int64_t block = (int64_t(r / bn) * (pitch / BK) + c / BK) * TERMS;
    const int32_t inside = (r % bn) * BK + c % BK;
#pragma unroll
    for (int p = 0; p < TERMS; ++p) {
        const uint16_t t = float_to_bf16(x);
        out[(block + p) * bn * BK + inside] = t;
        x -= __uint_as_float(uint32_t(t) << 16);
    }
}

bool aligned_to(const void* p, uintptr_t bytes) { return (reinterpret_cast<uintptr_t>(p) & (bytes - 1)) == 0; }

template <class F>
void with_flag(bool b, F&& f) {
    if (b)
        f(std::true_type{});
    else
        f(std::false_type{});
}

}  // namespace

hipError_t varco_launch_prep_weight_split(int terms, const float* h, int64_t ld, int32_t rows, int32_t cols,
                                          int32_t rows_padded, int32_t pitch, bool transpose, void* out, hipStream_t stream) {
    const int64_t total = int64_t(rows_padded) * pitch;
    if (total == 0) return hipSuccess;
    if (terms != 2 && terms != 3) return hipErrorInvalidValue;
    if (rows_padded < rows || rows_padded % kPrepRows != 0 || pitch < cols || pitch % BK != 0) return hipErrorInvalidValue;
    const dim3 grid(unsigned((total + kThreads - 1) / kThreads));
    const int32_t bn = rows <= 64 ? 64 : 128;      // the product kernel's B tile for this many output columns
    if (terms == 3)
        hipLaunchKernelGGL(prep_weight_split_kernel<3>, grid, dim3(kThreads), 0, stream, h, ld, rows, cols, rows_padded,
                           pitch, bn, transpose ? 1 : 0, static_cast<uint16_t*>(out));
    else
        hipLaunchKernelGGL(prep_weight_split_kernel<2>, grid, dim3(kThreads), 0, stream, h, ld, rows, cols, rows_padded,
                           pitch, bn, transpose ? 1 : 0, static_cast<uint16_t*>(out));
    return hipGetLastError();
}

namespace {
template <typename U>
struct TypeTag {
    using type = U;
};
}  // namespace

// Short reductions (see gemm_short_k_kernel): terms = 1 for bf16 storage, 2 or 3 for fp32 storage.
hipError_t varco_launch_gemm_short_k(const GemmArgs& ga, int terms, hipStream_t stream) {
    const dim3 grid(unsigned((ga.m + kShortRows - 1) / kShortRows), unsigned((ga.n + 255) / 256));
    const int ks = (ga.k + 15) / 16;
    if (ks < 1 || ks > 4) return hipErrorInvalidValue;
    auto go = [&](auto type, auto ksc, auto gt, auto tc) {
        using T = typename decltype(type)::type;
        hipLaunchKernelGGL((gemm_short_k_kernel<T, decltype(ksc)::value, decltype(gt)::value, decltype(tc)::value>), grid,
                           dim3(kThreads), 0, stream, static_cast<const T*>(ga.a.ptr), static_cast<const T*>(ga.a.gate),
                           static_cast<const float*>(ga.b.ptr), ga.b.ld, static_cast<T*>(ga.c), ga.ldc, ga.m, ga.n, ga.k,
                           ga.accumulate ? 1 : 0);
    };
    auto with_ks = [&](auto type, auto gt, auto tc) {
        switch (ks) {
            case 1: go(type, std::integral_constant<int, 1>{}, gt, tc); break;
            case 2: go(type, std::integral_constant<int, 2>{}, gt, tc); break;
            case 3: go(type, std::integral_constant<int, 3>{}, gt, tc); break;
            default: go(type, std::integral_constant<int, 4>{}, gt, tc); break;
        }
    };
    auto with_gate = [&](auto type, auto tc) {
        if (ga.a.gate)
            with_ks(type, std::true_type{}, tc);
        else
            with_ks(type, std::false_type{}, tc);
    };
    if (ga.a.dtype == VARCO_BF16)
        with_gate(TypeTag<bf16_t>{}, std::integral_constant<int, 1>{});
    else if (terms == 3)
        with_gate(TypeTag<float>{}, std::integral_constant<int, 3>{});
    else
        with_gate(TypeTag<float>{}, std::integral_constant<int, 2>{});
    return hipGetLastError();
}

namespace {
// TN: B can be read four columns at a time.
bool b_vector_ok(const GemmArgs& ga) {
    return aligned_to(ga.b.ptr, 16) && aligned_to(ga.b.gate, 16) && ga.b.ld % 4 == 0 && ga.n % 4 == 0;
}
}  // namespace

bool varco_gemm_split_usable(const GemmArgs& ga) {
    if (ga.f32_terms != 2 && ga.f32_terms != 3) return false;
    if (ga.m <= 0 || ga.n <= 0) return false;
    if (ga.a.dtype != VARCO_F32 || ga.c_dtype != VARCO_F32) return false;
    auto ok16 = [](const GemmOperand& o) { return aligned_to(o.ptr, 16) && aligned_to(o.gate, 16) && o.ld % 4 == 0; };
    if (!ga.a.transposed) {   // NT: needs the library's expanded weight copy [term][rows][pitch], padded to whole tiles
        auto prep_ok = [&](const void* p, int64_t ld, int64_t plane, int32_t k) {
            return p && aligned_to(p, 16) && ld % BK == 0 && ld >= k && plane == (int64_t(ga.n) + kPrepRows - 1) / kPrepRows * kPrepRows * ld;
        };
        if (!prep_ok(ga.b_prep, ga.b_prep_ld, ga.b_prep_plane, ga.k)) return false;
        if (ga.b.gate || ga.k % 4 != 0 || !ok16(ga.a)) return false;
        if (ga.k2 > 0) {   // a chained product shares the first one's leading dimensions and is never masked
            if (!prep_ok(ga.b2_prep, ga.b2_prep_ld, ga.b2_prep_plane, ga.k2) || ga.b2_prep_ld != ga.b_prep_ld) return false;
            if (ga.k2 % 4 != 0 || !ok16(ga.a2) || ga.a2.ld != ga.a.ld || ga.a.gate || ga.a2.gate || ga.a2.dtype != VARCO_F32 ||
                ga.a2.transposed)
                return false;
        }
        return true;
    }
    // TN: weight gradient
    if (ga.b.transposed || ga.b.dtype != VARCO_F32 || ga.k2 > 0 || ga.a.gate) return false;
    if (!ok16(ga.a) || ga.m % 4 != 0) return false;
    return b_vector_ok(ga) || (ga.n <= 64 && !ga.b.gate && aligned_to(ga.b.ptr, 4));   // else B element by element
}

hipError_t varco_launch_gemm_split(const GemmArgs& ga, hipStream_t stream, const LaunchTag& tag, int32_t* split_used) {
    const bool tn = ga.a.transposed;
    const bool narrow = ga.n <= 64;
    const int bm = 128, bn = narrow ? 64 : 128;
    const bool a8 = !tn && ga.k % 8 == 0 && (ga.k2 == 0 || ga.k2 % 8 == 0);
    const bool gate = tn ? ga.b.gate != nullptr : ga.a.gate != nullptr;

    SplitGemm g;
    g.m = ga.m, g.n = ga.n, g.k = ga.k, g.k2 = ga.k2;
    auto f32 = [](const void* p) { return static_cast<const float*>(p); };
    g.a = {ga.a.ptr, f32(ga.a.gate), ga.a.ld, 0};
    g.a2 = {ga.a2.ptr, f32(ga.a2.gate), ga.a2.ld, 0};
    if (tn) {
        g.b = {ga.b.ptr, f32(ga.b.gate), ga.b.ld, 0};
        g.b2 = {nullptr, nullptr, 0, 0};
    } else {
        g.b = {ga.b_prep, nullptr, ga.b_prep_ld, ga.b_prep_plane};
        g.b2 = {ga.b2_prep, nullptr, ga.b2_prep_ld, ga.b2_prep_plane};
    }
    g.c = static_cast<float*>(ga.c);
    g.ldc = ga.ldc;
    g.accumulate = ga.accumulate ? 1 : 0;
    g.relu = ga.relu ? 1 : 0;
    g.tiles_m = (ga.m + bm - 1) / bm;
    g.tiles_n = (ga.n + bn - 1) / bn;
    const int32_t k_tiles = (ga.k + BK - 1) / BK + (ga.k2 + BK - 1) / BK;
    int32_t split = ga.split_k < 1 ? 1 : ga.split_k;
    if (split > k_tiles) split = k_tiles < 1 ? 1 : k_tiles;
    g.tiles_per_split = (k_tiles + split - 1) / split;
    split = g.tiles_per_split > 0 ? (k_tiles + g.tiles_per_split - 1) / g.tiles_per_split : 1;
    if (split < 1) split = 1;
    g.split_k = split;
    g.partial = ga.partial;
    if (split > 1 && !ga.partial) return hipErrorInvalidValue;
    if (split > 1) {
        g.inner = g.tiles_m * g.tiles_n;
        g.outer = split;
    } else {
        g.inner = g.tiles_n;
        g.outer = g.tiles_m;
    }
    const int64_t blocks = int64_t((g.outer + 7) / 8 * 8) * g.inner;
    if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    const dim3 grid{unsigned(blocks)};
    *split_used = split;

    tag.begin(stream);
    with_flag(ga.f32_terms == 3, [&](auto t3) {
        with_flag(narrow, [&](auto nr) {
            with_flag(gate, [&](auto gt) {
                constexpr int T = decltype(t3)::value ? 3 : 2;
                constexpr bool NR = decltype(nr)::value, GT = decltype(gt)::value;
                constexpr int WM = NR ? 4 : 2, WN = NR ? 1 : 2, TMB = NR ? 1 : 2, TNB = 2;
                if (tn && !b_vector_ok(ga)) {
                    if constexpr (NR && !GT)
                        hipLaunchKernelGGL((gemm_split_kernel<T, true, WM, WN, TMB, TNB, 1, false>), grid, dim3(kThreads), 0, stream, g);
                } else if (tn) {
                    hipLaunchKernelGGL((gemm_split_kernel<T, true, WM, WN, TMB, TNB, 4, GT>), grid, dim3(kThreads), 0, stream, g);
                } else if (a8) {
                    hipLaunchKernelGGL((gemm_split_kernel<T, false, WM, WN, TMB, TNB, 8, GT>), grid, dim3(kThreads), 0, stream, g);
                } else {
                    hipLaunchKernelGGL((gemm_split_kernel<T, false, WM, WN, TMB, TNB, 4, GT>), grid, dim3(kThreads), 0, stream, g);
                }
            });
        });
    });
    tag.end(stream);
    return hipGetLastError();
}
