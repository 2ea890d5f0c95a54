// Dense feature transform of eq. (2) and its gradients for bf16-stored activations, on the bf16 matrix
// cores with fp32 accumulation (v_mfma_f32_32x32x16_bf16): X_out = act(M H1 + X H0), dM = dZ H1^T,
// dH += M^T dZ. Weights are kept in fp32 by the caller; the library hands this kernel a bf16 copy laid out
// [output index][reduction index] (see varco_launch_prep_weight), and weight gradients leave in fp32.
//
// One 256-thread workgroup (4 wavefronts) computes a 256 x 128 tile of C (256 x 64 for outputs at most 64
// columns wide). A wavefront owns 128 x 64 (or 64 x 64) of it as 32 x 32 blocks: at bf16 rates a wavefront
// tile smaller than that is limited by LDS reads of its fragments, not by the matrix cores. Operand tiles of
// 32 reduction steps are staged through LDS as rows of one output index with the reduction index contiguous
// (80-byte row pitch: 16-byte fragment reads without bank conflicts), double-buffered against the global
// loads of the next tile.
//   "NT" products (transform, input gradient): both operands already have the reduction index contiguous
//        in memory, so the global -> LDS copy moves 8 (or 4) elements at a time unchanged;
//   "TN" products (weight gradient, reduction over nodes): both operands have the node index as the slow
//        one. A thread loads an 8 (nodes) x 4 (columns) block with eight 8-byte loads, transposes it in
//        registers and writes four 16-byte LDS rows.
// The ReLU mask of the backward pass is applied when a tile is written to LDS, the activation in the
// epilogue. Reductions over nodes are split over workgroups into an fp32 partial buffer and summed by the
// caller's reduction kernel in a fixed order.
#include <type_traits>

#include "elem.h"
#include "varco_internal.h"

namespace {

constexpr int BK = 32;
constexpr int kThreads = 256;
constexpr int kPitch = BK + 8;   // bf16 elements per LDS row (80 bytes)

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct OperandDev {
    const uint16_t* ptr;
    const uint16_t* gate;
    int64_t ld;
};

struct GemmDev {
    int32_t m, n, k, k2;
    OperandDev a, b, a2, b2;
    void* c;
    int64_t ldc;
    int32_t accumulate, relu;
    int32_t split_k, tiles_per_split;
    float* partial;
    int32_t tiles_m, tiles_n;
    int32_t inner, outer;
};

// Two bf16 values packed in a word: keep each where the packed gate value is > 0.
__device__ __forceinline__ uint32_t gate_pair(uint32_t v, uint32_t g) {
    const uint32_t lo = __uint_as_float(g << 16) > 0.f ? 0x0000FFFFu : 0u;
    const uint32_t hi = __uint_as_float(g & 0xFFFF0000u) > 0.f ? 0xFFFF0000u : 0u;
    return v & (lo | hi);
}

// ---- operand with the reduction index contiguous in memory: chunks of CH elements, copied unchanged ----
template <int ROWS, int CH, bool GATE>
struct RowRegs {
    static constexpr int PER_ROW = BK / CH;
    static constexpr int N = ROWS * PER_ROW / kThreads;
    uint32_t v[N][CH / 2];
    uint32_t g[GATE ? N : 1][CH / 2];
    uint32_t inside;
};

template <int ROWS, int CH, bool GATE>
__device__ __forceinline__ void load_rows(const OperandDev& op, int32_t i0, int32_t extent, int32_t k0, int32_t kmax,
                                          RowRegs<ROWS, CH, GATE>& r) {
    using R = RowRegs<ROWS, CH, GATE>;
    using W = std::conditional_t<CH == 8, uint4, uint2>;
    r.inside = 0u;
#pragma unroll
    for (int h = 0; h < R::N; ++h) {
        const int c = threadIdx.x + h * kThreads;
        const int32_t i = i0 + c / R::PER_ROW;
        const int32_t kk = k0 + (c % R::PER_ROW) * CH;
        const bool in = i < extent && kk < kmax;          // kmax is a multiple of CH: a chunk is wholly in or out
        const int64_t off = in ? int64_t(i) * op.ld + kk : 0;
        const W x = *reinterpret_cast<const W*>(op.ptr + off);
        r.v[h][0] = x.x, r.v[h][1] = x.y;
        if constexpr (CH == 8) r.v[h][2] = x.z, r.v[h][3] = x.w;
        if (GATE) {
            const W y = *reinterpret_cast<const W*>(op.gate + off);
            r.g[h][0] = y.x, r.g[h][1] = y.y;
            if constexpr (CH == 8) r.g[h][2] = y.z, r.g[h][3] = y.w;
        }
        r.inside |= in ? (1u << h) : 0u;
    }
}

template <int ROWS, int CH, bool GATE>
__device__ __forceinline__ void store_rows(const RowRegs<ROWS, CH, GATE>& r, uint16_t* s) {
    using R = RowRegs<ROWS, CH, GATE>;
#pragma unroll
    for (int h = 0; h < R::N; ++h) {
        const int c = threadIdx.x + h * kThreads;
        const bool in = (r.inside >> h) & 1u;
        uint32_t x[CH / 2];
#pragma unroll
        for (int u = 0; u < CH / 2; ++u) {
            x[u] = in ? r.v[h][u] : 0u;
            if (GATE) x[u] = gate_pair(x[u], r.g[h][u]);
        }
        uint16_t* dst = s + (c / R::PER_ROW) * kPitch + (c % R::PER_ROW) * CH;
        if constexpr (CH == 8)
            *reinterpret_cast<uint4*>(dst) = make_uint4(x[0], x[1], x[2], x[3]);
        else
            *reinterpret_cast<uint2*>(dst) = make_uint2(x[0], x[1]);
    }
}

// ---- operand with the output index contiguous in memory: 8 (reduction) x 4 (output) blocks, transposed ----
template <int ROWS, bool GATE>
struct ColRegs {
    static constexpr int BLOCKS = ROWS;                       // (ROWS / 4) * (BK / 8)
    static constexpr int N = (BLOCKS + kThreads - 1) / kThreads;
    uint2 v[N][8];
    uint2 g[GATE ? N : 1][8];
    uint32_t inside;                                          // bit h * 8 + kk
};

template <int ROWS, bool GATE>
__device__ __forceinline__ void load_cols(const OperandDev& op, int32_t i0, int32_t extent, int32_t k0, int32_t kmax,
                                          ColRegs<ROWS, GATE>& r) {
    using R = ColRegs<ROWS, GATE>;
    r.inside = 0u;
#pragma unroll
    for (int h = 0; h < R::N; ++h) {
        const int b = threadIdx.x + h * kThreads;
        const bool active = b < R::BLOCKS;
        const int32_t i = i0 + (b % (ROWS / 4)) * 4;          // extent is a multiple of 4: a group is wholly in or out
        const int32_t kb = k0 + (b / (ROWS / 4)) * 8;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            const bool in = active && i < extent && kb + kk < kmax;
            const int64_t off = in ? int64_t(kb + kk) * op.ld + i : 0;
            r.v[h][kk] = *reinterpret_cast<const uint2*>(op.ptr + off);
            if (GATE) r.g[h][kk] = *reinterpret_cast<const uint2*>(op.gate + off);
            r.inside |= in ? (1u << (h * 8 + kk)) : 0u;
        }
    }
}

// The same block for an operand whose rows are not 8-byte aligned or whose width is not a multiple of 4 (the
// 47 class columns of the last layer): element loads; columns beyond the matrix repeat its last one, and their
// products are never stored.
template <int ROWS>
__device__ __forceinline__ void load_cols_ragged(const OperandDev& op, int32_t i0, int32_t extent, int32_t k0, int32_t kmax,
                                                 ColRegs<ROWS, false>& r) {
    using R = ColRegs<ROWS, false>;
    r.inside = 0u;
#pragma unroll
    for (int h = 0; h < R::N; ++h) {
        const int b = threadIdx.x + h * kThreads;
        const bool active = b < R::BLOCKS;
        const int32_t i = i0 + (b % (ROWS / 4)) * 4;
        const int32_t kb = k0 + (b / (ROWS / 4)) * 8;
        int32_t col[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) col[e] = min(i + e, extent - 1);
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            const bool in = active && kb + kk < kmax;
            const uint16_t* row = op.ptr + (in ? int64_t(kb + kk) * op.ld : 0);
            const uint32_t x0 = row[col[0]], x1 = row[col[1]], x2 = row[col[2]], x3 = row[col[3]];
            r.v[h][kk] = make_uint2(x0 | (x1 << 16), x2 | (x3 << 16));
            r.inside |= in ? (1u << (h * 8 + kk)) : 0u;
        }
    }
}

template <int ROWS, bool GATE>
__device__ __forceinline__ void store_cols(const ColRegs<ROWS, GATE>& r, uint16_t* s) {
    using R = ColRegs<ROWS, GATE>;
#pragma unroll
    for (int h = 0; h < R::N; ++h) {
        const int b = threadIdx.x + h * kThreads;
        if (b >= R::BLOCKS) continue;                         // uniform per wavefront (BLOCKS is a multiple of 64)
        uint32_t w[8][2];
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            const bool in = (r.inside >> (h * 8 + kk)) & 1u;
            w[kk][0] = in ? r.v[h][kk].x : 0u;
            w[kk][1] = in ? r.v[h][kk].y : 0u;
            if (GATE) {
                w[kk][0] = gate_pair(w[kk][0], r.g[h][kk].x);
                w[kk][1] = gate_pair(w[kk][1], r.g[h][kk].y);
            }
        }
        uint16_t* base = s + (b % (ROWS / 4)) * 4 * kPitch + (b / (ROWS / 4)) * 8;
#pragma unroll
        for (int ii = 0; ii < 4; ++ii) {                      // output index i + ii: its 8 reduction steps
            uint32_t o[4];
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const uint32_t e0 = w[2 * p][ii >> 1], e1 = w[2 * p + 1][ii >> 1];
                o[p] = (ii & 1) ? ((e0 >> 16) | (e1 & 0xFFFF0000u)) : ((e0 & 0xFFFFu) | (e1 << 16));
            }
            *reinterpret_cast<uint4*>(base + ii * kPitch) = make_uint4(o[0], o[1], o[2], o[3]);
        }
    }
}

template <bool TN, int ROWS, int CH, bool GATE>
struct Stage {
    using Regs = std::conditional_t<TN, ColRegs<ROWS, GATE>, RowRegs<ROWS, CH, GATE>>;
    static __device__ __forceinline__ void load(const OperandDev& op, int32_t i0, int32_t extent, int32_t k0, int32_t kmax,
                                                Regs& r) {
        if constexpr (TN && CH == 1)
            load_cols_ragged<ROWS>(op, i0, extent, k0, kmax, r);
        else if constexpr (TN)
            load_cols<ROWS, GATE>(op, i0, extent, k0, kmax, r);
        else
            load_rows<ROWS, CH, GATE>(op, i0, extent, k0, kmax, r);
    }
    static __device__ __forceinline__ void store(const Regs& r, uint16_t* s) {
        if constexpr (TN)
            store_cols<ROWS, GATE>(r, s);
        else
            store_rows<ROWS, CH, GATE>(r, s);
    }
};

__device__ __forceinline__ bf16x8 fragment(const uint16_t* s, int row, int koff) {
    return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(s + row * kPitch + koff));
}

// TN: both operands stored with the output index contiguous (weight gradient), else both with the reduction
// index contiguous. WM x WN wavefronts, each TMB x TNB blocks of 32 x 32. A_CH: elements per global load of
// A (NT; B is the library's own padded weight copy, always 8); in a TN product A_CH = 1 says that B is read
// element by element (unaligned rows, never masked). GATE masks A (NT) or B (TN).
// TC: bf16_t (activations) or float (weight gradients).
template <typename TC, bool TN, int WM, int WN, int TMB, int TNB, int A_CH, bool GATE>
__global__ __launch_bounds__(kThreads, 2) void gemm_bf16_kernel(GemmDev g) {
    constexpr int BM = 32 * TMB * WM, BN = 32 * TNB * WN;
    constexpr bool A_GATE = GATE && !TN, B_GATE = GATE && TN;
    static_assert(!(TN && A_CH == 1 && GATE), "an operand read element by element is never masked");
    using StageA = Stage<TN, BM, TN ? 8 : A_CH, A_GATE>;
    using StageB = Stage<TN, BN, TN ? A_CH : 8, B_GATE>;
    __shared__ __attribute__((aligned(16))) uint16_t sa[2][BM * kPitch];
    __shared__ __attribute__((aligned(16))) uint16_t sb[2][BN * kPitch];

    // workgroup -> tile: tiles that share streamed data go to one XCD (workgroups are dealt to the 8 XCDs
    // round-robin), so that the streamed operand is fetched into a single L2
    const int32_t xcd = blockIdx.x & 7, within = blockIdx.x >> 3;
    const int32_t in = within % g.inner, out = (within / g.inner) * 8 + xcd;
    if (out >= g.outer) return;        // whole workgroup leaves together: no barrier is skipped
    int32_t tm, tn, z;
    if (g.split_k > 1) {
        z = out, tm = in / g.tiles_n, tn = in % g.tiles_n;
    } else {
        z = 0, tm = out, tn = in;
    }
    const int32_t m0 = tm * BM, n0 = tn * BN;

    const int32_t tiles1 = (g.k + BK - 1) / BK;
    const int32_t tiles2 = (g.k2 + BK - 1) / BK;
    int32_t t_begin = 0, t_end = tiles1 + tiles2;
    if (g.split_k > 1) {
        t_begin = z * g.tiles_per_split;
        t_end = min(t_end, t_begin + g.tiles_per_split);
    }

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int wm = (wave / WN) * (32 * TMB), wn = (wave % WN) * (32 * TNB);
    const int lrow = lane & 31, lk = lane >> 5;

    floatx16 acc[TMB][TNB];
#pragma unroll
    for (int i = 0; i < TMB; ++i)
#pragma unroll
        for (int j = 0; j < TNB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    typename StageA::Regs ra;
    typename StageB::Regs rb;
    // operands of tile t are picked with selects, not branches, so that the loads stay straight-line code
    auto fetch = [&](int32_t t) {
        const bool first = t < tiles1;
        OperandDev oa, ob;
        oa.ptr = first ? g.a.ptr : g.a2.ptr, oa.gate = first ? g.a.gate : g.a2.gate, oa.ld = first ? g.a.ld : g.a2.ld;
        ob.ptr = first ? g.b.ptr : g.b2.ptr, ob.gate = first ? g.b.gate : g.b2.gate, ob.ld = first ? g.b.ld : g.b2.ld;
        const int32_t k0 = (first ? t : t - tiles1) * BK, kmax = first ? g.k : g.k2;
        StageA::load(oa, m0, g.m, k0, kmax, ra);
        StageB::load(ob, n0, g.n, k0, kmax, rb);
    };
    auto stash = [&](int buf) {
        StageA::store(ra, sa[buf]);
        StageB::store(rb, sb[buf]);
    };

    if (t_begin < t_end) {
        fetch(t_begin);
        stash(0);
    }
    __syncthreads();
    for (int32_t t = t_begin; t < t_end; ++t) {
        const int buf = (t - t_begin) & 1;
        if (t + 1 < t_end) fetch(t + 1);
#pragma unroll
        for (int s = 0; s < BK / 16; ++s) {
            const int koff = s * 16 + lk * 8;
            bf16x8 fa[TMB], fb[TNB];
#pragma unroll
            for (int i = 0; i < TMB; ++i) fa[i] = fragment(sa[buf], wm + i * 32 + lrow, koff);
#pragma unroll
            for (int j = 0; j < TNB; ++j) fb[j] = fragment(sb[buf], wn + j * 32 + lrow, koff);
#pragma unroll
            for (int i = 0; i < TMB; ++i)
#pragma unroll
                for (int j = 0; j < TNB; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (t + 1 < t_end) stash(buf ^ 1);
        __syncthreads();
    }

    // epilogue: accumulator register v of a lane is element (8 * (v / 4) + 4 * (lane / 32) + v % 4, lane % 32).
    // A tile that lies wholly inside C takes a path without per-element tests, with addresses formed from one
    // 64-bit base per lane plus 32-bit multiples of the row pitch. When C is added to, the old values of a
    // block are fetched by loads that are all issued before the first one is used (from clamped, always valid
    // addresses), not one round trip per element.
    const int32_t col_base = n0 + wn + lrow;
    if (g.split_k > 1) {
        float* pout = g.partial + int64_t(z) * g.m * g.n;
#pragma unroll
        for (int i = 0; i < TMB; ++i)
#pragma unroll
            for (int j = 0; j < TNB; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int32_t row = m0 + wm + i * 32 + 4 * lk + 8 * (v >> 2) + (v & 3), col = col_base + j * 32;
                    if (row < g.m && col < g.n) pout[int64_t(row) * g.n + col] = acc[i][j][v];
                }
        return;
    }
    TC* const base = static_cast<TC*>(g.c);
    const bool add_old = g.accumulate, relu = g.relu;
    auto finish = [&](auto guard) {
        constexpr bool GUARD = decltype(guard)::value;
        TC* const out0 = base + int64_t(m0 + wm) * g.ldc + col_base;          // interior tiles only
#pragma unroll
        for (int i = 0; i < TMB; ++i) {
#pragma unroll
            for (int j = 0; j < TNB; ++j) {
                TC* ptr[16];
                bool ok[16];
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int32_t r = i * 32 + 4 * lk + 8 * (v >> 2) + (v & 3);        // row inside the wavefront's part
                    if constexpr (GUARD) {
                        const int32_t row = m0 + wm + r, col = col_base + j * 32;
                        ok[v] = row < g.m && col < g.n;
                        ptr[v] = base + int64_t(min(row, g.m - 1)) * g.ldc + min(col, g.n - 1);
                    } else {
                        ok[v] = true;
                        ptr[v] = out0 + j * 32 + uint32_t(r) * uint32_t(g.ldc);        // a tile spans < 2^32 elements
                    }
                }
                float old[16];
#pragma unroll
                for (int v = 0; v < 16; ++v) old[v] = 0.f;
                if (add_old) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) old[v] = Elem<TC>::load(ptr[v]);
                }
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    float x = acc[i][j][v] + old[v];
                    if (relu) x = fmaxf(x, 0.f);
                    if (ok[v]) Elem<TC>::store(ptr[v], x);
                }
            }
        }
    };
    if (m0 + BM <= g.m && n0 + BN <= g.n)
        finish(std::false_type{});
    else
        finish(std::true_type{});
}

// out[r][c] (bf16, pitch `pitch` >= cols, zero beyond cols) = transpose ? h[c][r] : h[r][c], h fp32 with
// leading dimension ld.
__global__ __launch_bounds__(kThreads) void prep_weight_kernel(const float* __restrict__ h, int64_t ld, int32_t rows,
                                                               int32_t cols, int32_t pitch, int32_t transpose,
                                                               bf16_t* __restrict__ out) {
    const int64_t idx = int64_t(blockIdx.x) * kThreads + threadIdx.x;
    if (idx >= int64_t(rows) * pitch) return;
    const int32_t r = int32_t(idx / pitch), c = int32_t(idx % pitch);
    float x = 0.f;
    if (c < cols) x = transpose ? h[int64_t(c) * ld + r] : h[int64_t(r) * ld + c];
    Elem<bf16_t>::store(out + idx, x);
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

hipError_t varco_launch_prep_weight(const float* h, int64_t ld, int32_t rows, int32_t cols, int32_t pitch, bool transpose,
                                    void* out, hipStream_t stream) {
    const int64_t total = int64_t(rows) * pitch;
    if (total == 0) return hipSuccess;
    hipLaunchKernelGGL(prep_weight_kernel, dim3(unsigned((total + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream, h,
                       ld, rows, cols, pitch, transpose ? 1 : 0, static_cast<bf16_t*>(out));
    return hipGetLastError();
}

namespace {
// TN: B can be read four columns at a time.
bool b_vector_ok(const GemmArgs& ga) {
    return aligned_to(ga.b.ptr, 8) && aligned_to(ga.b.gate, 8) && ga.b.ld % 4 == 0 && ga.n % 4 == 0;
}
}  // namespace

bool varco_gemm_bf16_usable(const GemmArgs& ga) {
    if (ga.m <= 0 || ga.n <= 0) return false;
    const bool a_kc = !ga.a.transposed, b_kc = ga.b.transposed;
    if (ga.a.dtype != VARCO_BF16) return false;
    auto ok8 = [](const GemmOperand& o) { return aligned_to(o.ptr, 8) && aligned_to(o.gate, 8) && o.ld % 4 == 0; };
    if (a_kc) {   // NT: needs the library's bf16 weight copy [n][pitch], pitch a multiple of 8
        if (ga.c_dtype != VARCO_BF16 || !ga.b_prep || ga.b_prep_ld % 8 != 0 || !aligned_to(ga.b_prep, 16)) return false;
        if (ga.b.gate || ga.k % 4 != 0 || !ok8(ga.a)) return false;
        if (ga.k2 > 0 && (!ga.b2_prep || ga.b2_prep_ld % 8 != 0 || !aligned_to(ga.b2_prep, 16) || ga.k2 % 4 != 0 ||
                          !ok8(ga.a2) || ga.a2.gate || ga.a2.dtype != VARCO_BF16 || ga.a2.transposed))
            return false;
        return true;
    }
    // TN: weight gradient
    if (b_kc || ga.b.dtype != VARCO_BF16 || ga.c_dtype != VARCO_F32 || ga.k2 > 0 || ga.a.gate) return false;
    if (!ok8(ga.a) || ga.m % 4 != 0) return false;
    return b_vector_ok(ga) || (ga.n <= 64 && !ga.b.gate && aligned_to(ga.b.ptr, 2));   // else B element by element
}

hipError_t varco_launch_gemm_bf16(const GemmArgs& ga, hipStream_t stream, const LaunchTag& tag, int32_t* split_used) {
    const bool tn = ga.a.transposed;
    const bool narrow = ga.n <= 64;
    const int bm = 256, bn = narrow ? 64 : 128;
    auto chunk8 = [](const GemmOperand& o, int32_t k) {
        return !o.ptr || (aligned_to(o.ptr, 16) && aligned_to(o.gate, 16) && o.ld % 8 == 0 && k % 8 == 0);
    };
    const bool a8 = !tn && chunk8(ga.a, ga.k) && (ga.k2 == 0 || chunk8(ga.a2, ga.k2));
    const bool gate = tn ? ga.b.gate != nullptr : ga.a.gate != nullptr;

    GemmDev g;
    g.m = ga.m, g.n = ga.n, g.k = ga.k, g.k2 = ga.k2;
    auto u16 = [](const void* p) { return static_cast<const uint16_t*>(p); };
    g.a = {u16(ga.a.ptr), u16(ga.a.gate), ga.a.ld};
    g.a2 = {u16(ga.a2.ptr), u16(ga.a2.gate), ga.a2.ld};
    if (tn) {
        g.b = {u16(ga.b.ptr), u16(ga.b.gate), ga.b.ld};
        g.b2 = {nullptr, nullptr, 0};
    } else {
        g.b = {u16(ga.b_prep), nullptr, ga.b_prep_ld};
        g.b2 = {u16(ga.b2_prep), nullptr, ga.b2_prep_ld};
    }
    g.c = ga.c;
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
    with_flag(narrow, [&](auto nr) {
        with_flag(gate, [&](auto gt) {
            constexpr bool NR = decltype(nr)::value, GT = decltype(gt)::value;
            constexpr int WM = NR ? 4 : 2, WN = NR ? 1 : 2, TMB = NR ? 2 : 4, TNB = 2;
            if (tn && !b_vector_ok(ga)) {
                if constexpr (NR && !GT)
                    hipLaunchKernelGGL((gemm_bf16_kernel<float, true, WM, WN, TMB, TNB, 1, false>), grid, dim3(kThreads), 0, stream, g);
            } else if (tn) {
                hipLaunchKernelGGL((gemm_bf16_kernel<float, true, WM, WN, TMB, TNB, 8, GT>), grid, dim3(kThreads), 0, stream, g);
            } else if (a8) {
                hipLaunchKernelGGL((gemm_bf16_kernel<bf16_t, false, WM, WN, TMB, TNB, 8, GT>), grid, dim3(kThreads), 0, stream, g);
            } else {
                hipLaunchKernelGGL((gemm_bf16_kernel<bf16_t, false, WM, WN, TMB, TNB, 4, GT>), grid, dim3(kThreads), 0, stream, g);
            }
        });
    });
    tag.end(stream);
    return hipGetLastError();
}
