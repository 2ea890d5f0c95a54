// Dense feature transform of eq. (2) and its gradients on the CDNA matrix cores, in true fp32
// (v_mfma_f32_32x32x2_f32): X_out = act(M H1 + X H0), dM = dZ H1^T, dH += M^T dZ. Operands and results
// stored as bf16 are widened when a tile is fetched and rounded (to nearest even) in the epilogue.
//
// One 256-thread workgroup (4 wavefronts) computes a tile of C; each wavefront owns a 64 x 64 sub-tile as
// 2 x 2 MFMA blocks of 32 x 32 (64 accumulator registers per lane). The wavefronts are laid out 2 x 2
// (128 x 128 tile) or, for outputs at most 64 columns wide (the class logits), 4 x 1 (256 x 64 tile), so that
// a narrow output does not waste most of a 128-wide tile. Operand tiles of 16 reduction steps are staged
// through LDS (layout per operand: see store_tile) and double-buffered against the global loads of the next
// tile. The ReLU mask of the backward pass is applied when an operand tile is written to LDS ("gate"), the
// activation in the epilogue. A second (A2, B2) product can be chained into the same accumulators (the two
// taps of a SAGE layer). Reductions over the node dimension (weight gradients) are split over workgroups
// into a partial buffer and summed by a second kernel in a fixed order.
#include <type_traits>

#include "elem.h"
#include "varco_internal.h"

namespace {

constexpr int BK = 16;
constexpr int kThreads = 256;

typedef float floatx16 __attribute__((ext_vector_type(16)));

struct OperandDev {
    const void* ptr;     // elements of the kernel's operand type (TA or TB)
    const void* gate;
    int64_t ld;
};

struct GemmDev {
    int32_t m, n, k, k2;
    OperandDev a, b, a2, b2;
    void* c;             // elements of type TC
    int64_t ldc;
    int32_t accumulate, relu;
    int32_t split_k, tiles_per_split;   // reduction tiles (of BK) handled by one split
    float* partial;
    int32_t tiles_m, tiles_n;
    int32_t inner, outer;               // see the workgroup -> tile mapping in the kernel
};

// Registers holding this thread's share (ROWS / 64 groups of 4 floats) of one ROWS x BK operand tile, and
// of its gate when the operand is masked. Loads only fill these registers; nothing consumes them before the
// tile is written to LDS, so the global-memory latency of tile t+1 hides behind the matrix instructions
// of tile t.
template <int ROWS, bool GATE>
struct TileRegs {
    static constexpr int H = ROWS / 64;
    float v[H][4];
    float g[GATE ? H : 1][4];
    uint32_t inside;   // bit h * 4 + u: element (h, u) lies inside the matrix (scalar path only)
};

// Loads the thread's share of a (ROWS x BK) operand tile whose row index starts at i0 (M or N side).
// KC: the reduction index is contiguous in memory.
//   VEC: a group of 4 elements is wholly inside or wholly outside the matrix (the host checks alignment and
//        divisibility) and is fetched by one predicated load of 4 elements;
//   otherwise every element is loaded on its own, unconditionally (an out-of-range element reads element
//        0 of the matrix instead and is zeroed at the LDS write), so that the loads stay straight-line code.
template <typename T, int ROWS, bool KC, bool GATE, bool VEC>
__device__ __forceinline__ void load_tile(const OperandDev& op, int32_t i0, int32_t extent, int32_t k0, int32_t kmax,
                                          TileRegs<ROWS, GATE>& r) {
    constexpr int H = ROWS / 64;
    constexpr int Q = ROWS / 4;   // groups of 4 rows per reduction index (layout with rows contiguous)
    const int tid = threadIdx.x;
    const T* ptr = static_cast<const T*>(op.ptr);
    const T* gate = static_cast<const T*>(op.gate);
    r.inside = 0u;
#pragma unroll
    for (int h = 0; h < H; ++h) {
        const int f = tid + h * kThreads;   // index of a group of 4 floats in the tile
        const int32_t i = KC ? i0 + (f >> 2) : i0 + ((f % Q) << 2);
        const int32_t kk = KC ? k0 + ((f & 3) << 2) : k0 + f / Q;
        const int64_t off = KC ? int64_t(i) * op.ld + kk : int64_t(kk) * op.ld + i;
        if (VEC) {
            float4 x = make_float4(0.f, 0.f, 0.f, 0.f), gt = x;
            if (i < extent && kk < kmax) {
                x = load_vec<T, 4>(ptr + off);
                if (GATE) gt = load_vec<T, 4>(gate + off);
            }
            r.v[h][0] = x.x, r.v[h][1] = x.y, r.v[h][2] = x.z, r.v[h][3] = x.w;
            if (GATE) r.g[h][0] = gt.x, r.g[h][1] = gt.y, r.g[h][2] = gt.z, r.g[h][3] = gt.w;
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const bool in = KC ? (i < extent && kk + u < kmax) : (kk < kmax && i + u < extent);
                const int64_t o = in ? off + u : 0;
                r.v[h][u] = Elem<T>::load(ptr + o);
                if (GATE) r.g[h][u] = Elem<T>::load(gate + o);
                r.inside |= in ? (1u << (4 * h + u)) : 0u;
            }
        }
    }
}

// LDS layout of an operand tile (ROWS rows x BK reduction steps), chosen so that the global -> LDS copy is a
// 16-byte store whichever way the operand lies in memory:
//   KC  (reduction index contiguous in memory): row-major, s[row * kRowStride + k]; a lane then fetches the
//        8 reduction steps it feeds to the matrix cores with two 16-byte reads;
//   !KC (row index contiguous in memory): k-major, s[k * (ROWS + 4) + row]; fragments are scalar reads.
// Matrix-core step t of a tile multiplies reduction indices t (lanes 0-31) and 8 + t (lanes 32-63); any
// pairing is valid as long as both operands use the same one.
constexpr int kRowStride = BK + 4;    // 20 floats: 16-byte aligned rows, conflict-free 16-byte reads
template <int ROWS>
constexpr int tile_floats() {
    return ROWS * kRowStride > BK * (ROWS + 4) ? ROWS * kRowStride : BK * (ROWS + 4);
}

// Writes the registers into the LDS tile, applying bounds and the gate (ReLU mask).
template <int ROWS, bool KC, bool GATE, bool VEC>
__device__ __forceinline__ void store_tile(const TileRegs<ROWS, GATE>& r, float* s) {
    constexpr int H = ROWS / 64;
    constexpr int Q = ROWS / 4;
    const int tid = threadIdx.x;
#pragma unroll
    for (int h = 0; h < H; ++h) {
        const int f = tid + h * kThreads;
        float x[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const bool keep = (VEC || ((r.inside >> (4 * h + u)) & 1u)) && (!GATE || r.g[h][u] > 0.f);
            x[u] = keep ? r.v[h][u] : 0.f;
        }
        const int off = KC ? (f >> 2) * kRowStride + ((f & 3) << 2) : (f / Q) * (ROWS + 4) + ((f % Q) << 2);
        *reinterpret_cast<float4*>(s + off) = make_float4(x[0], x[1], x[2], x[3]);
    }
}

// The 8 values a lane feeds to the matrix cores for tile row `row` during one tile: reduction indices
// lk * 8 .. lk * 8 + 7.
template <int ROWS, bool KC>
__device__ __forceinline__ void load_fragment(const float* s, int row, int lk, float (&out)[8]) {
    if (KC) {
        const float4 lo = *reinterpret_cast<const float4*>(s + row * kRowStride + lk * 8);
        const float4 hi = *reinterpret_cast<const float4*>(s + row * kRowStride + lk * 8 + 4);
        out[0] = lo.x, out[1] = lo.y, out[2] = lo.z, out[3] = lo.w;
        out[4] = hi.x, out[5] = hi.y, out[6] = hi.z, out[7] = hi.w;
    } else {
#pragma unroll
        for (int t = 0; t < 8; ++t) out[t] = s[(lk * 8 + t) * (ROWS + 4) + row];
    }
}

// TA / TB / TC: storage types of the operands and of the result; WM x WN: layout of the four wavefronts
// over the tile (2 x 2 or 4 x 1); A_KC / B_KC: operand stored with the reduction index contiguous;
// A_GATE / B_GATE: operand is masked; A_VEC / B_VEC: operand may be fetched four elements at a time.
template <typename TA, typename TB, typename TC, int WM, int WN, bool A_KC, bool B_KC, bool A_GATE, bool B_GATE, bool A_VEC,
          bool B_VEC>
__global__ __launch_bounds__(kThreads, 4) void gemm_kernel(GemmDev g) {
    constexpr int BM = 64 * WM, BN = 64 * WN;
    __shared__ __attribute__((aligned(16))) float sa[2][tile_floats<BM>()];
    __shared__ __attribute__((aligned(16))) float sb[2][tile_floats<BN>()];

    // Workgroups are dealt to the 8 XCDs round-robin. The tiles that share streamed data (the column tiles
    // of one row tile; or, for a split reduction, all output tiles of one slab of the reduction range) are
    // given to one XCD, so that the streamed operand is fetched into a single L2.
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
    const int wm = (wave / WN) * 64, wn = (wave % WN) * 64;
    const int lrow = lane & 31, lk = lane >> 5;

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    TileRegs<BM, A_GATE> ra;
    TileRegs<BN, B_GATE> rb;
    // Tile t of the chained reduction: tiles [0, tiles1) come from the first product, the rest from the second.
    // The operands are picked with selects, not branches: a branch around the loads would make the compiler
    // wait for every load in flight where the two paths meet.
    auto fetch = [&](int32_t t) {
        const bool first = t < tiles1;
        OperandDev oa, ob;
        oa.ptr = first ? g.a.ptr : g.a2.ptr, oa.gate = first ? g.a.gate : g.a2.gate, oa.ld = first ? g.a.ld : g.a2.ld;
        ob.ptr = first ? g.b.ptr : g.b2.ptr, ob.gate = first ? g.b.gate : g.b2.gate, ob.ld = first ? g.b.ld : g.b2.ld;
        const int32_t k0 = (first ? t : t - tiles1) * BK, kmax = first ? g.k : g.k2;
        load_tile<TA, BM, A_KC, A_GATE, A_VEC>(oa, m0, g.m, k0, kmax, ra);
        load_tile<TB, BN, B_KC, B_GATE, B_VEC>(ob, n0, g.n, k0, kmax, rb);
    };
    auto stash = [&](int buf) {
        store_tile<BM, A_KC, A_GATE, A_VEC>(ra, sa[buf]);
        store_tile<BN, B_KC, B_GATE, B_VEC>(rb, sb[buf]);
    };

    if (t_begin < t_end) {
        fetch(t_begin);
        stash(0);
    }
    __syncthreads();
    for (int32_t t = t_begin; t < t_end; ++t) {
        const int buf = (t - t_begin) & 1;
        if (t + 1 < t_end) fetch(t + 1);
        float fa[2][8], fb[2][8];
        load_fragment<BM, A_KC>(sa[buf], wm + lrow, lk, fa[0]);
        load_fragment<BM, A_KC>(sa[buf], wm + 32 + lrow, lk, fa[1]);
        load_fragment<BN, B_KC>(sb[buf], wn + lrow, lk, fb[0]);
        load_fragment<BN, B_KC>(sb[buf], wn + 32 + lrow, lk, fb[1]);
#pragma unroll
        for (int s8 = 0; s8 < 8; ++s8) {
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[0][s8], fb[0][s8], acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[0][s8], fb[1][s8], acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[1][s8], fb[0][s8], acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[1][s8], fb[1][s8], acc[1][1], 0, 0, 0);
        }
        if (t + 1 < t_end) stash(buf ^ 1);
        __syncthreads();
    }

    // epilogue: accumulator register v of a lane is element (8 * (v / 4) + 4 * (lane / 32) + v % 4, lane % 32).
    // When C is added to, the old values of a block are fetched by loads that are all issued before the first
    // one is used (from clamped, always valid addresses), not one round trip per element.
    const bool to_partial = g.split_k > 1;
    TC* cout = static_cast<TC*>(g.c);
    float* pout = g.partial + int64_t(z) * g.m * g.n;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int32_t col = n0 + wn + j * 32 + lrow;
            const int32_t row0 = m0 + wm + i * 32 + 4 * lk;
            const bool col_ok = col < g.n;
            if (to_partial) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int32_t row = row0 + 8 * (v >> 2) + (v & 3);
                    if (col_ok && row < g.m) pout[int64_t(row) * g.n + col] = acc[i][j][v];
                }
                continue;
            }
            float old[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) old[v] = 0.f;
            if (g.accumulate) {
                const TC* cbase = cout + min(col, g.n - 1);
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    old[v] = Elem<TC>::load(cbase + int64_t(min(row0 + 8 * (v >> 2) + (v & 3), g.m - 1)) * g.ldc);
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int32_t row = row0 + 8 * (v >> 2) + (v & 3);
                float x = acc[i][j][v] + old[v];
                if (g.relu) x = fmaxf(x, 0.f);
                if (col_ok && row < g.m) Elem<TC>::store(cout + int64_t(row) * g.ldc + col, x);
            }
        }
    }
}

// C (+)= sum over splits of partial[s]. 64 consecutive output elements per workgroup; the four wavefronts
// sum interleaved quarters of the splits (several loads in flight each) and the quarters are added in a
// fixed order, so the result does not depend on scheduling.
template <typename TC>
__global__ __launch_bounds__(kThreads) void gemm_reduce_kernel(const float* partial, int32_t splits, int64_t mn,
                                                               int32_t n, TC* c, int64_t ldc, int32_t accumulate,
                                                               int32_t relu) {
    __shared__ float part[4][64];
    const int e = threadIdx.x & 63, quarter = threadIdx.x >> 6;
    const int64_t i = int64_t(blockIdx.x) * 64 + e;
    float x = 0.f;
    if (i < mn) {
        int32_t s = quarter;
        for (; s + 12 < splits; s += 16) {
            const float x0 = partial[int64_t(s) * mn + i], x1 = partial[int64_t(s + 4) * mn + i];
            const float x2 = partial[int64_t(s + 8) * mn + i], x3 = partial[int64_t(s + 12) * mn + i];
            x += x0, x += x1, x += x2, x += x3;
        }
        for (; s < splits; s += 4) x += partial[int64_t(s) * mn + i];
    }
    part[quarter][e] = x;
    __syncthreads();
    if (quarter == 0 && i < mn) {
        x = ((part[0][e] + part[1][e]) + part[2][e]) + part[3][e];
        TC* dst = c + (i / n) * ldc + (i % n);
        if (accumulate) x += Elem<TC>::load(dst);
        if (relu) x = fmaxf(x, 0.f);
        Elem<TC>::store(dst, x);
    }
}

// Loads of 4 elements are legal for an operand when its base (and gate) are aligned to them, its leading
// dimension is a multiple of 4 and groups of 4 consecutive elements never straddle the matrix edge. `rows`
// is the extent of the non-reduction index (M for A, N for B), `red` the reduction length.
// ---- short reductions: C (+)= A B^T with at most 64 reduction steps and densely stored rows of A (the input
// gradient of the last layer, whose output width is the number of classes) ----
// The general kernel would spend its time in prologue and epilogue here, and rows of, say, 47 elements are
// not 16-byte aligned; the product itself is bound by writing C. A workgroup copies its 128 rows of A, which
// are one contiguous range of memory, into LDS with 16-byte loads (masked and widened to fp32 on the way;
// the row pitch stays k, which is odd-friendly: a column of 32 rows touches 32 different banks). Each
// wavefront owns 64 columns of C: their weights sit in registers as MFMA operands for the whole kernel, and
// for each block of 32 rows the wavefront reads its A operands from LDS and issues the fp32 matrix
// instructions of the whole reduction.
constexpr int kSmallRows = 128;

template <typename T>
__device__ __forceinline__ void load_chunk(const T* p, float (&x)[16 / sizeof(T)]) {
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

template <typename T, int KSTEPS, bool GATE>
__global__ __launch_bounds__(kThreads, 2) void gemm_small_k_kernel(const T* __restrict__ a, const T* __restrict__ gate,
                                                                   const float* __restrict__ b, int64_t ldb, T* __restrict__ c,
                                                                   int64_t ldc, int32_t m, int32_t n, int32_t k,
                                                                   int32_t accumulate) {
    constexpr int VE = 16 / int(sizeof(T));                       // elements per 16-byte load
    __shared__ __attribute__((aligned(16))) float tile[kSmallRows * 2 * KSTEPS + 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lcol = lane & 31, lk = lane >> 5;
    const int32_t r0 = blockIdx.x * kSmallRows, rows = min(kSmallRows, m - r0);
    const int32_t c0 = blockIdx.y * 256 + wave * 64;

    // weights of this wavefront's two column blocks: lane holds B[2 s + lane / 32][column]
    float w[2][KSTEPS];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        const int32_t col = c0 + cb * 32 + lcol;
#pragma unroll
        for (int s2 = 0; s2 < KSTEPS; ++s2) {
            const int kk = 2 * s2 + lk;
            w[cb][s2] = col < n && kk < k ? b[int64_t(col) * ldb + kk] : 0.f;
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
            load_chunk<T>(src + e0, x);
            if (GATE) load_chunk<T>(gsrc + e0, y);
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
        float af[KSTEPS];
#pragma unroll
        for (int s2 = 0; s2 < KSTEPS; ++s2) {
            const int kk = 2 * s2 + lk;
            const float x = tile[lrow * k + kk];                     // in bounds: the tile has 64 spare floats
            af[s2] = kk < k ? x : 0.f;
        }
#pragma unroll
        for (int s2 = 0; s2 < KSTEPS; ++s2)
#pragma unroll
            for (int cb = 0; cb < 2; ++cb) acc[cb] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[s2], w[cb][s2], acc[cb], 0, 0, 0);
        // accumulator register v of a lane is element (8 * (v / 4) + 4 * (lane / 32) + v % 4, lane % 32)
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

// A [m x k] with k contiguous and rows densely stored, B = fp32 weights stored [n x k], no chained product,
// no split, no activation.
bool small_k_usable(const GemmArgs& ga) {
    const uintptr_t pa = reinterpret_cast<uintptr_t>(ga.a.ptr), pg = reinterpret_cast<uintptr_t>(ga.a.gate);
    const uintptr_t es = ga.a.dtype == VARCO_BF16 ? 2 : 4;
    const bool same_skew = !ga.a.gate || (pa & 15u) == (pg & 15u);     // A and its mask are read with the same chunking
    return !ga.a.transposed && ga.b.transposed && ga.k >= 1 && ga.k <= 64 && ga.a.ld == ga.k && ga.k2 == 0 && !ga.b.gate &&
           !ga.relu && ga.b.dtype == VARCO_F32 && ga.a.dtype == ga.c_dtype && ga.split_k <= 1 && pa % es == 0 && same_skew;
}

template <typename T>
void launch_small_k(const GemmArgs& ga, hipStream_t stream) {
    const dim3 grid(unsigned((ga.m + kSmallRows - 1) / kSmallRows), unsigned((ga.n + 255) / 256));
    const int steps = (ga.k + 15) / 16 * 8;       // reduction steps of two, in units the kernel is instantiated for
    auto go = [&](auto sc, auto gt) {
        hipLaunchKernelGGL((gemm_small_k_kernel<T, decltype(sc)::value, decltype(gt)::value>), grid, dim3(kThreads), 0, stream,
                           static_cast<const T*>(ga.a.ptr), static_cast<const T*>(ga.a.gate), static_cast<const float*>(ga.b.ptr),
                           ga.b.ld, static_cast<T*>(ga.c), ga.ldc, ga.m, ga.n, ga.k, ga.accumulate ? 1 : 0);
    };
    auto with_gate = [&](auto sc) {
        if (ga.a.gate)
            go(sc, std::true_type{});
        else
            go(sc, std::false_type{});
    };
    if (steps == 8)
        with_gate(std::integral_constant<int, 8>{});
    else if (steps == 16)
        with_gate(std::integral_constant<int, 16>{});
    else if (steps == 24)
        with_gate(std::integral_constant<int, 24>{});
    else
        with_gate(std::integral_constant<int, 32>{});
}

bool vector_ok(const GemmOperand& o, bool k_contig, int32_t rows, int32_t red) {
    if (!o.ptr) return true;
    const uintptr_t mask = (o.dtype == VARCO_BF16 ? 8u : 16u) - 1u;
    const bool al = (reinterpret_cast<uintptr_t>(o.ptr) & mask) == 0 && (reinterpret_cast<uintptr_t>(o.gate) & mask) == 0;
    const bool whole = k_contig ? red % 4 == 0 : rows % 4 == 0;
    return al && o.ld % 4 == 0 && whole;
}

template <class F>
void with_flag(bool b, F&& f) {
    if (b)
        f(std::true_type{});
    else
        f(std::false_type{});
}

template <typename TA, typename TB, typename TC, bool A_KC, bool B_KC, bool A_GATE, bool B_GATE>
void launch_layout(bool narrow, bool a_vec, bool b_vec, dim3 grid, hipStream_t stream, const GemmDev& g) {
    with_flag(narrow, [&](auto nr) {
        with_flag(a_vec, [&](auto av) {
            with_flag(b_vec, [&](auto bv) {
                constexpr int WM = decltype(nr)::value ? 4 : 2, WN = decltype(nr)::value ? 1 : 2;
                hipLaunchKernelGGL((gemm_kernel<TA, TB, TC, WM, WN, A_KC, B_KC, A_GATE, B_GATE, decltype(av)::value,
                                                decltype(bv)::value>),
                                   grid, dim3(kThreads), 0, stream, g);
            });
        });
    });
}

}  // namespace

namespace {

hipError_t launch_reduce(const GemmArgs& ga, int32_t split, hipStream_t stream, const LaunchTag& tag) {
    const int64_t mn = int64_t(ga.m) * ga.n;
    const int32_t acc = ga.accumulate ? 1 : 0, relu = ga.relu ? 1 : 0;
    // reads the partial products and, when adding, the old result; writes the result once
    tag.begin_as(VARCO_K_REDUCE, stream, double(mn) * (4.0 * split + (acc ? 2.0 : 1.0) * (ga.c_dtype == VARCO_BF16 ? 2.0 : 4.0)));
    if (ga.c_dtype == VARCO_BF16)
        hipLaunchKernelGGL(gemm_reduce_kernel<bf16_t>, dim3(unsigned((mn + 63) / 64)), dim3(kThreads), 0, stream, ga.partial,
                           split, mn, ga.n, static_cast<bf16_t*>(ga.c), ga.ldc, acc, relu);
    else
        hipLaunchKernelGGL(gemm_reduce_kernel<float>, dim3(unsigned((mn + 63) / 64)), dim3(kThreads), 0, stream, ga.partial,
                           split, mn, ga.n, static_cast<float*>(ga.c), ga.ldc, acc, relu);
    tag.end(stream);
    return hipGetLastError();
}

}  // namespace

hipError_t varco_launch_gemm_reduce(const float* partial, int32_t slabs, int32_t m, int32_t n, float* c, int64_t ldc,
                                    bool accumulate, hipStream_t stream, const LaunchTag& tag) {
    if (slabs <= 0 || m <= 0 || n <= 0) return hipSuccess;
    GemmArgs ga;
    ga.m = m, ga.n = n;
    ga.partial = const_cast<float*>(partial);
    ga.c = c, ga.ldc = ldc, ga.c_dtype = VARCO_F32;
    ga.accumulate = accumulate;
    return launch_reduce(ga, slabs, stream, tag);
}

hipError_t varco_launch_gemm(const GemmArgs& ga, hipStream_t stream, const LaunchTag& tag) {
    if (ga.m == 0 || ga.n == 0) return hipSuccess;
    if (small_k_usable(ga)) {
        tag.begin(stream);
        hipError_t e = hipSuccess;
        if (ga.a.dtype == VARCO_BF16)
            e = varco_launch_gemm_short_k(ga, 1, stream);               // bf16 matrix instructions
        else if (ga.f32_terms == 2 || ga.f32_terms == 3)
            e = varco_launch_gemm_short_k(ga, ga.f32_terms, stream);    // fp32 products from bf16 terms
        else
            launch_small_k<float>(ga, stream);                          // fp32 matrix instructions
        tag.end(stream);
        return e != hipSuccess ? e : hipGetLastError();
    }
    if (varco_gemm_bf16_usable(ga)) {
        int32_t split = 1;
        const hipError_t e = varco_launch_gemm_bf16(ga, stream, tag, &split);
        if (e != hipSuccess || split <= 1) return e;
        return launch_reduce(ga, split, stream, tag);
    }
    if (varco_gemm_split_usable(ga)) {
        int32_t split = 1;
        const hipError_t e = varco_launch_gemm_split(ga, stream, tag, &split);
        if (e != hipSuccess || split <= 1) return e;
        return launch_reduce(ga, split, stream, tag);
    }
    // A is M x K: k-contiguous as stored unless transposed. B is K x N: k-contiguous only when transposed.
    const bool a_kc = !ga.a.transposed, b_kc = ga.b.transposed;
    const bool a_gate = ga.a.gate != nullptr, b_gate = ga.b.gate != nullptr;
    if (ga.k2 > 0 && (ga.a2.transposed != ga.a.transposed || ga.b2.transposed != ga.b.transposed || ga.a2.gate || ga.b2.gate))
        return hipErrorInvalidValue;   // the chained product must share the first one's layout and is never masked
    const bool a_vec = vector_ok(ga.a, a_kc, ga.m, ga.k) && (ga.k2 == 0 || vector_ok(ga.a2, a_kc, ga.m, ga.k2));
    const bool b_vec = vector_ok(ga.b, b_kc, ga.n, ga.k) && (ga.k2 == 0 || vector_ok(ga.b2, b_kc, ga.n, ga.k2));
    const bool narrow = ga.n <= 64;
    const int bm = narrow ? 256 : 128, bn = narrow ? 64 : 128;

    GemmDev g;
    g.m = ga.m, g.n = ga.n, g.k = ga.k, g.k2 = ga.k2;
    g.a = {ga.a.ptr, ga.a.gate, ga.a.ld};
    g.b = {ga.b.ptr, ga.b.gate, ga.b.ld};
    g.a2 = {ga.a2.ptr, ga.a2.gate, ga.a2.ld};
    g.b2 = {ga.b2.ptr, ga.b2.gate, ga.b2.ld};
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

    const bool known = (a_kc && !b_kc && !a_gate && !b_gate) || (a_kc && b_kc && !b_gate) || (!a_kc && !b_kc && !a_gate);
    if (!known) return hipErrorInvalidValue;
    // storage types: all fp32; or bf16 activations with fp32 weights: (A, B, C) = (bf16, f32, bf16) for the
    // transform and the input gradient, (bf16, bf16, f32) for the weight gradient
    const int ta = ga.a.dtype, tb = ga.b.dtype, tc = ga.c_dtype;
    if (ga.k2 > 0 && (ga.a2.dtype != ta || ga.b2.dtype != tb)) return hipErrorInvalidValue;
    const bool all_f32 = ta == VARCO_F32 && tb == VARCO_F32 && tc == VARCO_F32;
    const bool act_out = ta == VARCO_BF16 && tb == VARCO_F32 && tc == VARCO_BF16 && a_kc;
    const bool weight_out = ta == VARCO_BF16 && tb == VARCO_BF16 && tc == VARCO_F32 && !a_kc;
    if (!all_f32 && !act_out && !weight_out) return hipErrorInvalidValue;
    tag.begin(stream);
    if (all_f32) {
        if (a_kc && !b_kc)                                   // act(M H)
            launch_layout<float, float, float, true, false, false, false>(narrow, a_vec, b_vec, grid, stream, g);
        else if (a_kc && b_kc && a_gate)                     // dZ H^T, masked
            launch_layout<float, float, float, true, true, true, false>(narrow, a_vec, b_vec, grid, stream, g);
        else if (a_kc && b_kc)                               // dZ H^T
            launch_layout<float, float, float, true, true, false, false>(narrow, a_vec, b_vec, grid, stream, g);
        else if (b_gate)                                     // M^T dZ, masked
            launch_layout<float, float, float, false, false, false, true>(narrow, a_vec, b_vec, grid, stream, g);
        else                                                 // M^T dZ
            launch_layout<float, float, float, false, false, false, false>(narrow, a_vec, b_vec, grid, stream, g);
    } else if (act_out) {
        if (!b_kc)
            launch_layout<bf16_t, float, bf16_t, true, false, false, false>(narrow, a_vec, b_vec, grid, stream, g);
        else if (a_gate)
            launch_layout<bf16_t, float, bf16_t, true, true, true, false>(narrow, a_vec, b_vec, grid, stream, g);
        else
            launch_layout<bf16_t, float, bf16_t, true, true, false, false>(narrow, a_vec, b_vec, grid, stream, g);
    } else {
        if (b_gate)
            launch_layout<bf16_t, bf16_t, float, false, false, false, true>(narrow, a_vec, b_vec, grid, stream, g);
        else
            launch_layout<bf16_t, bf16_t, float, false, false, false, false>(narrow, a_vec, b_vec, grid, stream, g);
    }
    tag.end(stream);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    if (split > 1) err = launch_reduce(ga, split, stream, tag);
    return err;
}
