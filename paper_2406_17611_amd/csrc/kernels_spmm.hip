// Graph-convolution aggregation M = S_q [X_loc ; X~_halo] (eq. (1)-(2) of the paper; Algorithm 1: local
// rows uncompressed, remote rows in compressed form) and its transpose for the backward pass.
//
// HBM-bound gather kernels. One wavefront (64 lanes) takes one work item = a run of consecutive CSR entries
// of one row, as long as the host's work list makes it (at most 128 entries in the forward block, 32 in the
// transposed ones); longer rows are split and their partial sums reduced in a second pass, so power-law hubs
// do not serialise on one wavefront and no floating-point atomics reach memory. The kernels are latency
// bound unless many loads are in flight, and a wavefront waits for the slowest load of a batch, so every
// gather loop first issues a block of independent loads and only then consumes them.
//
//   dense source rows (local rows; halo rows when k == width): a power-of-two group of lanes covers one
//     row with 16-byte loads, the groups of a wavefront take different edges and are summed at the end
//     with cross-lane shuffles (wavefront-level segmented reduction);
//   compressed halo rows (k < width): never decompressed to memory. The stored elements of several edges
//     are loaded side by side (lane = (edge, j)), their positions pi_v(j) are recomputed from the key,
//     and they are accumulated into a per-wavefront row in LDS.
//
// The forward kernel reads a per-entry record {source row, node id} that the library derives once from
// the caller's column indices, so that a halo entry needs no dependent index lookups before its data load.
#include <algorithm>

#include <type_traits>

#include "elem.h"
#include "mask_device.h"

namespace {

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / 64;
// Threads per workgroup of spmm_kernel. With compressed rows a wavefront is a workgroup of its own: runs differ in
// length, and a workgroup keeps its LDS and wavefront slots until its last wavefront is done (bf16 configuration,
// forward aggregation 23.7 -> 22.8 ms per step). The dense-only kernels use no LDS and run faster four to a
// workgroup (large fp32 configuration, transposed local block 4.5 against 4.8 ms).
constexpr int agg_block(int mode) { return mode == 0 /* dense rows only */ ? kBlock : 64; }
// Independent row loads issued back to back by the kernels that also take compressed rows (dense rows here,
// compressed rows see sparse_phase): their register budget is the 64 of eight wavefronts per SIMD, or the 72 of
// seven; resident wavefronts, each a chain of dependent round trips, are what their rate is made of.
constexpr int kXcdRun = 32;       // consecutive workgroups of the work list that one XCD takes (see spmm_kernel)
constexpr int kUnroll = 3;
constexpr int kUnrollDense = 4;   // dense-only kernels have registers to spare

template <int VEC>
using Vec = FloatVec<VEC>;

__device__ __forceinline__ void fma_vec(float4& acc, float w, const float4& v) {
    acc.x += w * v.x;
    acc.y += w * v.y;
    acc.z += w * v.z;
    acc.w += w * v.w;
}
__device__ __forceinline__ void fma_vec(float& acc, float w, const float& v) { acc += w * v; }
__device__ __forceinline__ void add_vec(float4& a, const float4& b) {
    a.x += b.x;
    a.y += b.y;
    a.z += b.z;
    a.w += b.w;
}
__device__ __forceinline__ void add_vec(float& a, const float& b) { a += b; }
__device__ __forceinline__ void add_vec(float2& a, const float2& b) {
    a.x += b.x;
    a.y += b.y;
}
__device__ __forceinline__ float4 shfl_xor_vec(const float4& v, int mask) {
    return make_float4(__shfl_xor(v.x, mask), __shfl_xor(v.y, mask), __shfl_xor(v.z, mask), __shfl_xor(v.w, mask));
}
__device__ __forceinline__ float shfl_xor_vec(const float& v, int mask) { return __shfl_xor(v, mask); }
__device__ __forceinline__ void zero_vec(float4& v) { v = make_float4(0.f, 0.f, 0.f, 0.f); }
__device__ __forceinline__ void zero_vec(float& v) { v = 0.f; }
__device__ __forceinline__ void zero_vec(float2& v) { v = make_float2(0.f, 0.f); }
__device__ __forceinline__ float elem(const float2& v, int i) { return i == 0 ? v.x : v.y; }
__device__ __forceinline__ float elem(const float4& v, int i) { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }
__device__ __forceinline__ float elem(const float& v, int) { return v; }

template <typename T>
struct SpmmArgs {
    const SpmmItem* items;
    int32_t n_items;
    const VarcoEdge* edge;    // HALO kernels: one record per CSR entry
    const int32_t* colidx;    // dense-only kernels: column = source row
    const float* vals;
    const T* dense;
    const T* z;
    MaskRule rule;
    T* out;
    int32_t row_base;
    float* partial;           // partial sums of split rows stay in fp32
    int32_t lpr_log2;         // lanes per dense row = 1 << lpr_log2
    int32_t ev;               // stored elements of a compressed row per lane and load: 4, 2 or 1
    int32_t ku;               // loads per compressed row = k / ev
    int32_t lpe_log2;         // lanes that share one compressed row = 1 << lpe_log2 (>= min(ku, 64))
    int32_t epi;              // compressed rows handled per instruction = private LDS rows per wavefront
    int32_t swizzle;          // private rows hold position q at q ^ ((q >> 5) & 3) (see sparse_phase)
};

// N consecutive stored elements as they come from memory (bf16 stays packed until it is used).
template <typename T, int N>
struct Stored {
    using type = typename FloatVec<N>::type;
    static __device__ __forceinline__ float get(const type& v, int i) { return elem(v, i); }
};
template <>
struct Stored<bf16_t, 4> {
    using type = uint2;
    static __device__ __forceinline__ float get(const uint2& v, int i) {
        const uint32_t u = i < 2 ? v.x : v.y;
        return __uint_as_float((i & 1) ? (u & 0xFFFF0000u) : (u << 16));
    }
};
template <>
struct Stored<bf16_t, 2> {
    using type = uint32_t;
    static __device__ __forceinline__ float get(const uint32_t& v, int i) {
        return __uint_as_float(i ? (v & 0xFFFF0000u) : (v << 16));
    }
};
template <>
struct Stored<bf16_t, 1> {
    using type = uint16_t;
    static __device__ __forceinline__ float get(const uint16_t& v, int) { return bf16_to_float(v); }
};

// Scatter-accumulate the compressed rows of the wavefront's current batch: lanes [nd, nd + ns) hold one
// halo entry each (row in z, weight, packed (a, b)). A group of `lpe` lanes takes one entry (lane = group
// of EV stored elements), `epi` entries are handled per instruction, and each of those lane groups adds
// into a private LDS row of its own: the positions of one entry are distinct, so plain read-add-write is
// race-free and no LDS atomics (which run at a small fraction of the plain LDS rate) are needed.
// Z32: every element of the compressed buffer lies below 2^32 bytes, so a row's address is the (uniform) base
// plus a 32-bit offset: one address register per gather in flight instead of two, which is what decides how
// many wavefronts fit a SIMD here. `srow` then holds the row's element offset (row * k), not the row.
// SWZ: the lanes of one entry step through its stored elements EV at a time, so at one instruction their positions
// differ by multiples of EV * a: with 16 or more lanes per entry, lanes 8 (EV = 4) apart meet in one LDS bank at
// different addresses, a 4-way conflict on every access of a 512-wide row. Their positions differ by odd multiples
// of 32, so folding bits 5-6 of the position into bits 0-1 of the address (which the lanes of an instruction share)
// separates them; the row is read back through the same map.
// POW2: the width is a power of two, so positions wrap with a mask instead of a division by multiplication and
// conditional subtractions (the kernel is bound by its vector instructions once the conflicts are gone).
template <typename T, int EV, bool Z32, bool SWZ, bool POW2 = false>
__device__ __forceinline__ void sparse_phase(const SpmmArgs<T>& p, int lane, int nd, int ns, int32_t srow, float w,
                                             uint32_t mab, float* lpriv) {
    using S = typename Stored<T, EV>::type;
    // Gathers in flight per lane: six of at most 8 bytes (four bf16 or two fp32 elements), three of 16 bytes:
    // about the same registers either way. A wavefront waits for the slowest of its gathers, so fewer, larger
    // batches win even at the price of one resident wavefront (bf16 rows of 512 elements: 7 per SIMD, forward
    // aggregation 30.6 -> 24.8 ms per step; the fp32 kernel keeps 8: 13.8 -> 13.5 ms). Eight gathers, or four
    // of 16 bytes, cost more wavefronts than they gain (27.6 ms and 14.5 ms).
    constexpr int G = EV * sizeof(T) <= 8 ? 2 * kUnroll : kUnroll;
    const int32_t k = int32_t(p.rule.k);
    const uint32_t width = p.rule.width;
    const int sub = lane >> p.lpe_log2;
    const int jl = lane & ((1 << p.lpe_log2) - 1);
    const bool lane_ok = sub < p.epi && jl < p.ku;
    float* row = lpriv + sub * int32_t(width);
    for (int j0 = 0; j0 < p.ku; j0 += 64) {          // more than one pass only when an entry needs > 64 lanes
        const int ju = j0 + jl;
        const bool j_ok = lane_ok && ju < p.ku;
        const int j = ju * EV;
        for (int r0 = 0; r0 < ns; r0 += p.epi * G) {
            // Issue all gathers first; only the loaded values stay in registers across the wait. Everything
            // else about an entry (weight, multiplier, offset, positions) is fetched from its lane and
            // computed after the wait, so that more gathers fit the registers of a wavefront.
            S v[G];
#pragma unroll
            for (int u = 0; u < G; ++u) {
                const int es = r0 + u * p.epi + sub;
                const bool act = j_ok && es < ns;
                const int32_t r = __shfl(srow, act ? nd + es : 0);
                // lanes without an entry re-read the start of the buffer (never used, but no branch around the load)
                if constexpr (Z32)
                    v[u] = *reinterpret_cast<const S*>(p.z + (act ? uint32_t(r) + uint32_t(j) : 0u));
                else
                    v[u] = *reinterpret_cast<const S*>(p.z + (act ? int64_t(r) * k + j : int64_t(0)));
            }
            __builtin_amdgcn_sched_barrier(0);       // keep the work below behind the loads
#pragma unroll
            for (int u = 0; u < G; ++u) {
                const int es = r0 + u * p.epi + sub;
                const bool act = j_ok && es < ns;
                const int src_lane = act ? nd + es : 0;
                const float wi = __shfl(w, src_lane);
                const uint32_t ab = __shfl(mab, src_lane);
                const uint32_t a = ab & 0xFFFFu;
                if (act) {
                    uint32_t q[EV];
                    float cur[EV];
                    if constexpr (POW2) {
                        q[0] = (__umul24(a, uint32_t(j)) + (ab >> 16)) & (width - 1u);
#pragma unroll
                        for (int i = 1; i < EV; ++i) q[i] = (q[i - 1] + a) & (width - 1u);
                    } else {
                        q[0] = varco_mod_width(__umul24(a, uint32_t(j)) + (ab >> 16), width, p.rule.width_magic);
#pragma unroll
                        for (int i = 1; i < EV; ++i) {
                            q[i] = q[i - 1] + a;
                            if (q[i] >= width) q[i] -= width;
                        }
                    }
                    if constexpr (SWZ) {
#pragma unroll
                        for (int i = 0; i < EV; ++i) q[i] ^= (q[i] >> 5) & 3u;
                    }
#pragma unroll
                    for (int i = 0; i < EV; ++i) cur[i] = row[q[i]];          // distinct positions of one entry
#pragma unroll
                    for (int i = 0; i < EV; ++i) row[q[i]] = cur[i] + wi * Stored<T, EV>::get(v[u], i);
                }
            }
        }
    }
}

// T: storage type of the dense rows, the compressed rows and the output (sums are kept in fp32);
// VEC: elements per lane per load of a dense row (4 needs width % 4 == 0 and bases aligned to 4 elements);
// NV: such loads per lane per row, so that width <= VEC * NV * lanes-per-row;
// MODE: kDenseOnly: all rows are dense; kHalo / kHaloZ32: entries may refer to compressed halo rows (forward
// aggregation), the latter with 32-bit offsets into the compressed buffer (see sparse_phase).
constexpr int kDenseOnly = 0, kHalo = 1, kHaloZ32 = 2;
template <typename T, int VEC, int NV, int MODE>
__global__ __launch_bounds__(agg_block(MODE)) void spmm_kernel(SpmmArgs<T> p) {
    using V = typename Vec<VEC>::type;
    constexpr bool HALO = MODE != kDenseOnly, Z32 = MODE == kHaloZ32;
    constexpr int kAggBlock = agg_block(MODE), kAggWaves = kAggBlock / 64;
    constexpr int U = NV >= 4 ? 1 : (NV == 2 ? 2 : (HALO ? kUnroll : kUnrollDense));
    extern __shared__ float lds[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int32_t width = int32_t(p.rule.width);
    const bool full = p.rule.k == p.rule.width;
    const bool sparse = HALO && !full;
    float* lpriv = lds + wave * p.epi * width;   // this wavefront's private rows of compressed-row sums
    uint16_t* lunits = reinterpret_cast<uint16_t*>(lds + kAggWaves * p.epi * width);

    // The wavefront's item and the records of its first batch are requested before the table is staged and the
    // workgroup meets at the barrier: three round trips in a row become little more than one.
    // Workgroups are dealt to the 8 XCDs round-robin; an XCD takes the work list in runs of kXcdRun consecutive
    // workgroups (the grid is a multiple of 8 runs), so that rows next to each other - which on a graph with any
    // locality share source rows - are aggregated through the same L2 at about the same time, while every XCD still
    // sees the same mix of long and short rows (contiguous eighths put all split rows on one XCD: twice as slow).
    const int32_t xcd = int32_t(blockIdx.x & 7u), seq = int32_t(blockIdx.x >> 3);
    const int32_t block = ((seq / kXcdRun) * 8 + xcd) * kXcdRun + seq % kXcdRun;
    const int32_t idx = block * kAggWaves + __builtin_amdgcn_readfirstlane(wave);   // uniform: the item sits in scalar registers
    const bool has_item = idx < p.n_items;
    SpmmItem it{};                      // empty range for a wavefront without an item
    if (has_item) it = p.items[idx];
    VarcoEdge ed{0, -1};                // the current batch's records: one entry per lane
    int32_t col = 0;
    float w = 0.f;
    auto load_records = [&](int32_t base) {
        ed = VarcoEdge{0, -1}, col = 0, w = 0.f;
        if (base + lane < it.e1) {
            if (HALO)
                ed = p.edge[base + lane];
            else
                col = p.colidx[base + lane];
            w = p.vals[base + lane];
        }
    };
    load_records(it.e0);
    if (sparse) {   // the multiplier table is looked up once per halo entry: keep it in LDS
        for (uint32_t i = threadIdx.x; i < p.rule.n_units; i += kAggBlock) lunits[i] = p.rule.units[i];
        for (int c = lane; c < p.epi * width; c += 64) lpriv[c] = 0.f;
        __syncthreads();
    }
    if (!has_item) return;              // no block-wide barrier below: wavefronts are independent

    const int lpr = 1 << p.lpr_log2;
    const int t = lane & (lpr - 1);     // position inside the group
    const int g = lane >> p.lpr_log2;   // group index: which edge of a step this lane works on
    const int ng = 64 >> p.lpr_log2;

    V acc[NV];
#pragma unroll
    for (int m = 0; m < NV; ++m) zero_vec(acc[m]);
    bool any_sparse = false;

    for (int32_t base = it.e0; base < it.e1; base += 64) {
        if (base != it.e0) load_records(base);
        int32_t srow = 0;
        bool is_halo = false;
        uint32_t mab = 0;
        if (HALO) {
            srow = ed.src;
            is_halo = ed.gid >= 0;
            if (Z32 && sparse && is_halo) srow = int32_t(uint32_t(ed.src) * p.rule.k);   // one multiply per entry, not per gather
            if (sparse && is_halo) {
                const uint32_t h1 = varco_mix32(uint32_t(ed.gid) ^ varco_key0(p.rule));
                const uint32_t h2 = varco_mix32(h1 ^ varco_key1(p.rule));
                mab = uint32_t(lunits[__umulhi(h2, p.rule.n_units)]) | (__umulhi(h1, p.rule.width) << 16);
            }
        } else {
            srow = col;
        }
        const uint64_t hmask = HALO ? __ballot(is_halo) : 0ull;
        const int cnt = min(64, it.e1 - base);
        const int ns = sparse ? __popcll(hmask) : 0;
        const int nd = cnt - ns;        // columns ascend within a row, so dense entries sit in lanes [0, nd)

        // dense rows: group g takes entries g, g + ng, ...; U row loads are issued before they are used
        for (int i0 = 0; i0 < nd; i0 += ng * U) {
            V v[U][NV];
            float wi[U];
            bool ok[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = i0 + u * ng + g;
                ok[u] = i < nd;
                const int src_lane = ok[u] ? i : 0;
                const int32_t r = __shfl(srow, src_lane);
                wi[u] = __shfl(w, src_lane);
                const bool h = HALO && ((hmask >> src_lane) & 1);
                const T* src = (h ? p.z : p.dense) + int64_t(r) * width;
#pragma unroll
                for (int m = 0; m < NV; ++m) {
                    const int col = VEC * (t + lpr * m);
                    zero_vec(v[u][m]);
                    if (ok[u] && col < width) v[u][m] = load_vec<T, VEC>(src + col);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int m = 0; m < NV; ++m) fma_vec(acc[m], ok[u] ? wi[u] : 0.f, v[u][m]);
        }

        if (ns > 0) {
            any_sparse = true;
            if (p.ev == 4 && p.swizzle && (width & (width - 1)) == 0)
                sparse_phase<T, 4, Z32, true, true>(p, lane, nd, ns, srow, w, mab, lpriv);
            else if (p.ev == 4 && p.swizzle)
                sparse_phase<T, 4, Z32, true>(p, lane, nd, ns, srow, w, mab, lpriv);
            else if (p.ev == 4)
                sparse_phase<T, 4, Z32, false>(p, lane, nd, ns, srow, w, mab, lpriv);
            else if (p.ev == 2)
                sparse_phase<T, 2, Z32, false>(p, lane, nd, ns, srow, w, mab, lpriv);
            else
                sparse_phase<T, 1, Z32, false>(p, lane, nd, ns, srow, w, mab, lpriv);
        }
    }

    // sum the groups' partial rows
    for (int off = lpr; off < 64; off <<= 1) {
#pragma unroll
        for (int m = 0; m < NV; ++m) add_vec(acc[m], shfl_xor_vec(acc[m], off));
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    if (g == 0) {
#pragma unroll
        for (int m = 0; m < NV; ++m) {
            const int col = VEC * (t + lpr * m);
            if (col < width) {
                V v = acc[m];
                if (any_sparse) {
                    for (int sub = 0; sub < p.epi; ++sub) {
                        V x = *reinterpret_cast<const V*>(lpriv + sub * width + col);
                        if constexpr (VEC == 4) {
                            if (p.swizzle) {        // element i of the group of 4 sits at i ^ s
                                const int sw = (col >> 5) & 3;
                                const float e[4] = {x.x, x.y, x.z, x.w};
                                x = make_float4(e[sw], e[1 ^ sw], e[2 ^ sw], e[3 ^ sw]);
                            }
                        }
                        add_vec(v, x);
                    }
                }
                if (it.dst < 0)
                    store_vec<T, VEC>(p.out + int64_t(it.row - p.row_base) * width + col, v);
                else
                    *reinterpret_cast<V*>(p.partial + int64_t(it.dst) * width + col) = v;
            }
        }
    }
}

// Dense-only blocks whose rows are very short (the transposed local block of a finely partitioned graph has
// one or two entries per row): a wavefront per row would leave the device waiting on each wavefront's chain of
// dependent loads (row extent -> entry records -> source row), with nothing else in flight in that wavefront.
// Here a wavefront takes four consecutive rows and walks them in step: the extents, then the entry records,
// then the i-th source row of all four are each fetched by loads issued together. Rows longer than `max_len`
// are left to spmm_kernel (whose work list then holds only those).
template <typename T>
struct ShortRowArgs {
    const int32_t* rowptr;    // CSR row pointer of the block's matrix (absolute entry offsets)
    const int32_t* colidx;
    const float* vals;
    const T* dense;
    T* out;
    int32_t r0, n_rows;       // rows r0 .. r0 + n_rows - 1
    int32_t row_base;         // out row = row - row_base
    int32_t max_len;          // at most 64
    int32_t width;
};

template <typename T, int VEC, int NV>
__global__ __launch_bounds__(kBlock) void spmm_short_rows_kernel(ShortRowArgs<T> p) {
    using V = typename Vec<VEC>::type;
    constexpr int R = 4;
    const int lane = threadIdx.x & 63;
    const int32_t first = p.r0 + (blockIdx.x * kWaves + (threadIdx.x >> 6)) * R;
    const int32_t n_here = min(R, p.r0 + p.n_rows - first);
    if (n_here <= 0) return;           // wavefronts are independent: no barrier below

    const int32_t ptr = lane <= n_here ? p.rowptr[first + lane] : 0;
    int32_t e0[R], len[R];
    bool mine[R];
    int32_t longest = 0;
#pragma unroll
    for (int q = 0; q < R; ++q) {
        e0[q] = __shfl(ptr, q);
        const int32_t l = __shfl(ptr, q + 1) - e0[q];
        mine[q] = q < n_here && l <= p.max_len;
        len[q] = mine[q] ? l : 0;
        longest = max(longest, len[q]);
    }
    int32_t col[R];
    float wt[R];
#pragma unroll
    for (int q = 0; q < R; ++q) {      // lane j holds entry j of every row
        const bool has = lane < len[q];
        col[q] = has ? p.colidx[e0[q] + lane] : 0;
        wt[q] = has ? p.vals[e0[q] + lane] : 0.f;
    }
    V acc[R][NV];
#pragma unroll
    for (int q = 0; q < R; ++q)
#pragma unroll
        for (int m = 0; m < NV; ++m) zero_vec(acc[q][m]);
    for (int32_t i = 0; i < longest; ++i) {
        V v[R][NV];
        float wi[R];
#pragma unroll
        for (int q = 0; q < R; ++q) {
            const bool on = i < len[q];
            const int32_t r = __shfl(col[q], i);
            wi[q] = on ? __shfl(wt[q], i) : 0.f;
            const T* src = p.dense + int64_t(r) * p.width;
#pragma unroll
            for (int m = 0; m < NV; ++m) {
                const int c = VEC * (lane + 64 * m);
                zero_vec(v[q][m]);
                if (on && c < p.width) v[q][m] = load_vec<T, VEC>(src + c);
            }
        }
#pragma unroll
        for (int q = 0; q < R; ++q)
#pragma unroll
            for (int m = 0; m < NV; ++m) fma_vec(acc[q][m], wi[q], v[q][m]);
    }
#pragma unroll
    for (int q = 0; q < R; ++q) {
        if (!mine[q]) continue;
        T* dst = p.out + int64_t(first + q - p.row_base) * p.width;
#pragma unroll
        for (int m = 0; m < NV; ++m) {
            const int c = VEC * (lane + 64 * m);
            if (c < p.width) store_vec<T, VEC>(dst + c, acc[q][m]);
        }
    }
}

// out[row] = sum of the partial rows of a split row, in slot order (fixed order: reproducible bits).
template <typename T>
__global__ __launch_bounds__(kBlock) void spmm_fixup_kernel(const SpmmSplit* splits, int32_t n_splits,
                                                            const float* partial, T* out, int32_t row_base,
                                                            int32_t width) {
    const int32_t s = blockIdx.x;
    if (s >= n_splits) return;
    const SpmmSplit sp = splits[s];
    for (int c = threadIdx.x; c < width; c += kBlock) {
        const float* src = partial + int64_t(sp.first) * width + c;
        float acc = 0.f;
        int i = 0;
        for (; i + 8 <= sp.count; i += 8) {      // eight loads in flight; the additions keep slot order
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = src[int64_t(i + u) * width];
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += v[u];
        }
        for (; i < sp.count; ++i) acc += src[int64_t(i) * width];
        Elem<T>::store(out + int64_t(sp.row - row_base) * width + c, acc);
    }
}

// The same for rows whose width is a multiple of 4: a launch ends with its longest split row (a hub's hundreds of
// partial rows, one dependent chain per thread above), so here the four wavefronts of the workgroup each sum a
// contiguous quarter of the slots, 4 columns per lane and 8 loads in flight, and the quarters are added in wavefront
// order: a fixed order as well, with a chain a quarter as long.
template <typename T>
__global__ __launch_bounds__(kBlock) void spmm_fixup4_kernel(const SpmmSplit* splits, int32_t n_splits,
                                                             const float* partial, T* out, int32_t row_base,
                                                             int32_t width) {
    __shared__ float4 part[kWaves][64];
    const int32_t s = blockIdx.x;
    if (s >= n_splits) return;          // whole workgroup
    const SpmmSplit sp = splits[s];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int32_t per = (sp.count + kWaves - 1) / kWaves;
    const int32_t i0 = min(wave * per, sp.count), i1 = min(i0 + per, sp.count);
    for (int32_t c0 = 0; c0 < width; c0 += 256) {
        const int32_t c = c0 + 4 * lane;
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        if (c < width) {
            const float* src = partial + int64_t(sp.first) * width + c;
            int32_t i = i0;
            for (; i + 8 <= i1; i += 8) {
                float4 v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const float4*>(src + int64_t(i + u) * width);
#pragma unroll
                for (int u = 0; u < 8; ++u) add_vec(acc, v[u]);
            }
            for (; i < i1; ++i) add_vec(acc, *reinterpret_cast<const float4*>(src + int64_t(i) * width));
        }
        part[wave][lane] = acc;
        __syncthreads();
        if (wave == 0 && c < width) {
            float4 x = part[0][lane];
#pragma unroll
            for (int w = 1; w < kWaves; ++w) add_vec(x, part[w][lane]);
            store_vec<T, 4>(out + int64_t(sp.row - row_base) * width + c, x);
        }
        __syncthreads();                // the next column group reuses the block
    }
}

// ---------------------------------------------------------------------------------------------------------
// Transposed aggregation for halo rows, produced directly in compressed form:
//     dz_halo[s, j] = sum over local rows i of S[i, halo s] * dM[i, pi_v(j)],  j < k,  v = node of slot s.
// Gathering the k scattered columns of every dM row an entry refers to would pull whole cache lines for
// 4 useful bytes each, once per entry. Instead the work is done in two streaming passes:
//   1. row order: a wavefront stages dM[i, :] in LDS once, and for each halo entry of row i writes the k
//      products w * dM[i, pi_v(j)] as one contiguous row of a product buffer (elements of the storage type),
//      at the entry's position in the transposed order (prow, derived once at registration);
//   2. transposed order: the products of one halo slot are now consecutive rows; they are summed in entry
//      order (fixed order: reproducible bits) into dz_halo.
// ---------------------------------------------------------------------------------------------------------
template <typename T>
struct ProductArgs {
    const SpmmItem* items;      // work list of the forward row block
    int32_t n_items;
    const VarcoEdge* edge;
    const float* vals;
    const int32_t* prow;        // per entry: row of the product buffer (halo entries only)
    const T* dm;                // n_local x width
    MaskRule rule;
    T* prod;                    // (halo entries) x k, in the storage type
    int32_t ev;                 // floats per lane and store: 4, 2 or 1
    int32_t ku;                 // stores per entry = k / ev
    int32_t lpe_log2;           // lanes per entry
};

template <typename T, int EV>
__device__ __forceinline__ void product_phase(const ProductArgs<T>& p, int lane, int first, int ns, int32_t pr, float w,
                                              uint32_t mab, const float* lrow) {
    using V = typename Vec<EV>::type;
    const int64_t k = p.rule.k;
    const uint32_t width = p.rule.width;
    const int epi = 64 >> p.lpe_log2;
    const int sub = lane >> p.lpe_log2;
    const int jl = lane & ((1 << p.lpe_log2) - 1);
    for (int j0 = 0; j0 < p.ku; j0 += 64) {
        const int ju = j0 + jl;
        const bool j_ok = ju < p.ku;
        const int j = ju * EV;
        for (int r0 = 0; r0 < ns; r0 += epi) {
            const int es = r0 + sub;
            const bool act = j_ok && es < ns;
            const int src_lane = act ? first + es : 0;
            const int32_t row = __shfl(pr, src_lane);
            const float wi = __shfl(w, src_lane);
            const uint32_t ab = __shfl(mab, src_lane);
            if (act) {
                const uint32_t a = ab & 0xFFFFu;
                uint32_t q = varco_mod_width(a * uint32_t(j) + (ab >> 16), width, p.rule.width_magic);
                float out[EV];
#pragma unroll
                for (int i = 0; i < EV; ++i) {
                    out[i] = wi * lrow[q];
                    q += a;
                    if (q >= width) q -= width;
                }
                T* dst = p.prod + int64_t(row) * k + j;
                if constexpr (EV == 4)
                    store_vec<T, 4>(dst, make_float4(out[0], out[1], out[2], out[3]));
                else if constexpr (EV == 2)
                    store_vec<T, 2>(dst, make_float2(out[0], out[1]));
                else
                    store_vec<T, 1>(dst, out[0]);
            }
        }
    }
}

template <typename T>
__global__ __launch_bounds__(kBlock) void halo_products_kernel(ProductArgs<T> p) {
    extern __shared__ float lds[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int32_t width = int32_t(p.rule.width);
    float* lrow = lds + wave * width;
    uint16_t* lunits = reinterpret_cast<uint16_t*>(lds + kWaves * width);
    const int32_t idx = blockIdx.x * kWaves + __builtin_amdgcn_readfirstlane(wave);   // uniform: the item sits in scalar registers
    const bool has_item = idx < p.n_items;
    SpmmItem it{};                      // empty range for a wavefront without an item
    if (has_item) it = p.items[idx];

    // The records of a batch (entry, weight, product row) are loaded together and for every entry, halo or
    // not, so that one memory round trip serves all three; the first batch's loads are in flight while the
    // row of dM is staged in LDS, and all of that is requested before the workgroup stages the multiplier
    // table and meets at the barrier.
    VarcoEdge ed{0, -1};
    float w = 0.f;
    int32_t pr = 0;
    auto load_batch = [&](int32_t base) {
        const int32_t e = base + lane;
        ed = VarcoEdge{0, -1}, w = 0.f, pr = 0;
        if (e < it.e1) ed = p.edge[e], w = p.vals[e], pr = p.prow[e];
    };
    load_batch(it.e0);
    if (it.e0 < it.e1) {
        const T* src = p.dm + int64_t(it.row) * width;
        for (int c = lane; c < width; c += 64) lrow[c] = Elem<T>::load(src + c);
    }
    for (uint32_t i = threadIdx.x; i < p.rule.n_units; i += kBlock) lunits[i] = p.rule.units[i];
    __syncthreads();                    // also orders the wavefront's own row behind its writes
    if (it.e0 >= it.e1) return;         // no block-wide barrier below
    for (int32_t base = it.e0; base < it.e1; base += 64) {
        const bool is_halo = ed.gid >= 0;
        const uint64_t hmask = __ballot(is_halo);
        uint32_t mab = 0;
        if (is_halo) {
            const uint32_t h1 = varco_mix32(uint32_t(ed.gid) ^ varco_key0(p.rule));
            const uint32_t h2 = varco_mix32(h1 ^ varco_key1(p.rule));
            mab = uint32_t(lunits[__umulhi(h2, p.rule.n_units)]) | (__umulhi(h1, p.rule.width) << 16);
        }
        const int cnt = min(64, it.e1 - base);
        const int ns = __popcll(hmask);
        const int first = cnt - ns;     // columns ascend within a row: halo entries sit in the last lanes
        const float wb = w;
        const int32_t prb = pr;
        if (base + 64 < it.e1) load_batch(base + 64);
        if (ns > 0) {
            if (p.ev == 4)
                product_phase<T, 4>(p, lane, first, ns, prb, wb, mab, lrow);
            else if (p.ev == 2)
                product_phase<T, 2>(p, lane, first, ns, prb, wb, mab, lrow);
            else
                product_phase<T, 1>(p, lane, first, ns, prb, wb, mab, lrow);
        }
    }
}

template <typename T>
struct SegsumArgs {
    const SpmmItem* items;      // work list of the transposed halo rows (entry ranges in transposed order)
    int32_t n_items;
    const T* prod;
    int32_t prod_base;          // transposed position of the first halo entry (= product row 0)
    int32_t k;
    T* out;
    int32_t row_base;
    float* partial;
    int32_t ev, ku, lpe_log2;
};

template <typename T, int EV>
__device__ __forceinline__ void segsum_body(const SegsumArgs<T>& p, const SpmmItem& it, int jl, int lpe) {
    using V = typename Vec<EV>::type;
    for (int ju = jl; ju < p.ku; ju += lpe) {
        const T* src = p.prod + int64_t(it.e0 - p.prod_base) * p.k + ju * EV;
        V acc;
        zero_vec(acc);
        int32_t n = it.e1 - it.e0;
        for (; n >= 4; n -= 4) {
            const V v0 = load_vec<T, EV>(src), v1 = load_vec<T, EV>(src + p.k);
            const V v2 = load_vec<T, EV>(src + 2 * int64_t(p.k));
            const V v3 = load_vec<T, EV>(src + 3 * int64_t(p.k));
            add_vec(acc, v0), add_vec(acc, v1), add_vec(acc, v2), add_vec(acc, v3);
            src += 4 * int64_t(p.k);
        }
        if (n > 0) {   // up to three rows left: fetched together (rows past the end re-read the first), added in order
            const V v0 = load_vec<T, EV>(src), v1 = load_vec<T, EV>(src + (n > 1 ? p.k : 0));
            const V v2 = load_vec<T, EV>(src + (n > 2 ? 2 * int64_t(p.k) : 0));
            add_vec(acc, v0);
            if (n > 1) add_vec(acc, v1);
            if (n > 2) add_vec(acc, v2);
        }
        if (it.dst < 0)
            store_vec<T, EV>(p.out + int64_t(it.row - p.row_base) * p.k + ju * EV, acc);
        else
            *reinterpret_cast<V*>(p.partial + int64_t(it.dst) * p.k + ju * EV) = acc;
    }
}

// bf16 rows, 8 elements (16 bytes) per lane and load: half as many, twice as wide loads as the 4-element form.
struct Float8 {
    float4 lo, hi;
};
__device__ __forceinline__ Float8 load8(const bf16_t* p) {
    const uint4 u = *reinterpret_cast<const uint4*>(p);
    Float8 v;
    v.lo = make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xFFFF0000u), __uint_as_float(u.y << 16),
                       __uint_as_float(u.y & 0xFFFF0000u));
    v.hi = make_float4(__uint_as_float(u.z << 16), __uint_as_float(u.z & 0xFFFF0000u), __uint_as_float(u.w << 16),
                       __uint_as_float(u.w & 0xFFFF0000u));
    return v;
}
__device__ __forceinline__ void add8(Float8& a, const Float8& b) {
    add_vec(a.lo, b.lo);
    add_vec(a.hi, b.hi);
}
__device__ __forceinline__ void segsum_body8(const SegsumArgs<bf16_t>& p, const SpmmItem& it, int jl, int lpe) {
    for (int ju = jl; ju < p.ku; ju += lpe) {
        const bf16_t* src = p.prod + int64_t(it.e0 - p.prod_base) * p.k + ju * 8;
        Float8 acc;
        zero_vec(acc.lo), zero_vec(acc.hi);
        int32_t n = it.e1 - it.e0;
        for (; n >= 4; n -= 4) {
            const Float8 v0 = load8(src), v1 = load8(src + p.k), v2 = load8(src + 2 * int64_t(p.k)), v3 = load8(src + 3 * int64_t(p.k));
            add8(acc, v0), add8(acc, v1), add8(acc, v2), add8(acc, v3);
            src += 4 * int64_t(p.k);
        }
        if (n > 0) {   // up to three rows left: fetched together (rows past the end re-read the first), added in order
            const Float8 v0 = load8(src), v1 = load8(src + (n > 1 ? p.k : 0)), v2 = load8(src + (n > 2 ? 2 * int64_t(p.k) : 0));
            add8(acc, v0);
            if (n > 1) add8(acc, v1);
            if (n > 2) add8(acc, v2);
        }
        if (it.dst < 0) {
            bf16_t* dst = p.out + int64_t(it.row - p.row_base) * p.k + ju * 8;
            Elem<bf16_t>::store4(dst, acc.lo);
            Elem<bf16_t>::store4(dst + 4, acc.hi);
        } else {
            float* dst = p.partial + int64_t(it.dst) * p.k + ju * 8;
            *reinterpret_cast<float4*>(dst) = acc.lo;
            *reinterpret_cast<float4*>(dst + 4) = acc.hi;
        }
    }
}

template <typename T>
__global__ __launch_bounds__(kBlock) void halo_segsum_kernel(SegsumArgs<T> p) {
    const int lpe = 1 << p.lpe_log2;
    const int64_t gidx = (int64_t(blockIdx.x) * kBlock + threadIdx.x) >> p.lpe_log2;
    if (gidx >= p.n_items) return;
    const SpmmItem it = p.items[gidx];
    const int jl = threadIdx.x & (lpe - 1);
    if constexpr (std::is_same_v<T, bf16_t>) {
        if (p.ev == 8) {
            segsum_body8(p, it, jl, lpe);
            return;
        }
    }
    if (p.ev == 4)
        segsum_body<T, 4>(p, it, jl, lpe);
    else if (p.ev == 2)
        segsum_body<T, 2>(p, it, jl, lpe);
    else
        segsum_body<T, 1>(p, it, jl, lpe);
}

// prow[e] of a halo entry e = (local row i, halo column c): its position among the halo entries in the
// transposed order, found by searching i in the ascending row list of transposed row c. One thread per row.
__global__ __launch_bounds__(kBlock) void build_prow_kernel(const int32_t* rowptr, const int32_t* colidx, int32_t n_local,
                                                            const int32_t* t_rowptr, const int32_t* t_colidx,
                                                            int32_t* prow) {
    const int32_t i = blockIdx.x * kBlock + threadIdx.x;
    if (i >= n_local) return;
    const int32_t base = t_rowptr[n_local];
    for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
        const int32_t c = colidx[e];
        int32_t pos = -1;
        if (c >= n_local) {
            int32_t lo = t_rowptr[c], hi = t_rowptr[c + 1] - 1;
            while (lo < hi) {
                const int32_t mid = (lo + hi) >> 1;
                if (t_colidx[mid] < i) lo = mid + 1; else hi = mid;
            }
            pos = lo - base;
        }
        prow[e] = pos;
    }
}

// Per-entry records of a partition's row block: local column -> {row, -1}; halo column -> {row of the
// node in the concatenated compressed buffer, node id}.
__global__ __launch_bounds__(kBlock) void build_edges_kernel(const int32_t* colidx, int64_t nnz, int32_t n_local,
                                                             const int32_t* halo_zrow, const int32_t* halo_gid,
                                                             VarcoEdge* edge) {
    const int64_t e = int64_t(blockIdx.x) * kBlock + threadIdx.x;
    if (e >= nnz) return;
    const int32_t c = colidx[e];
    VarcoEdge ed;
    if (c < n_local) {
        ed.src = c, ed.gid = -1;
    } else {
        ed.src = halo_zrow[c - n_local], ed.gid = halo_gid[c - n_local];
    }
    edge[e] = ed;
}

// Checks of a partition's index arrays at registration, so that no later kernel can be led out of bounds or to
// silently wrong sums by a malformed descriptor. Every failed check sets a bit of *flags.
//   rows:  columns of each row strictly ascending and inside [0, n_local + n_halo)
//   trows: row indices of each transposed row strictly ascending and inside [0, n_local), and every transposed
//          entry (c, i, v) present in forward row i with the same value (with equal entry counts and distinct
//          entries on both sides: the two structures hold the same triplets)
// One thread per (transposed) row; row pointers were checked on the host.
__global__ __launch_bounds__(kBlock) void validate_rows_kernel(const int32_t* rowptr, const int32_t* colidx, int32_t n_local,
                                                               int32_t n_cols, int32_t* flags) {
    const int32_t i = blockIdx.x * kBlock + threadIdx.x;
    if (i >= n_local) return;
    int32_t prev = -1, bad = 0;
    for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
        const int32_t c = colidx[e];
        if (c < 0 || c >= n_cols) bad |= VARCO_BAD_COLUMN_RANGE;
        if (c <= prev) bad |= VARCO_BAD_COLUMN_ORDER;
        prev = c;
    }
    if (bad) atomicOr(flags, bad);
}
__global__ __launch_bounds__(kBlock) void validate_trows_kernel(const int32_t* rowptr, const int32_t* colidx, const float* vals,
                                                                int32_t n_local, int32_t n_cols, const int32_t* t_rowptr,
                                                                const int32_t* t_colidx, const float* t_vals, int32_t* flags) {
    const int32_t c = blockIdx.x * kBlock + threadIdx.x;
    if (c >= n_cols) return;
    int32_t prev = -1, bad = 0;
    for (int32_t pos = t_rowptr[c]; pos < t_rowptr[c + 1]; ++pos) {
        const int32_t i = t_colidx[pos];
        if (i < 0 || i >= n_local) {
            bad |= VARCO_BAD_TROW_RANGE;
            continue;
        }
        if (i <= prev) bad |= VARCO_BAD_TROW_ORDER;
        prev = i;
        int32_t lo = rowptr[i], hi = rowptr[i + 1];     // first entry of row i with column >= c (rows may be unsorted
        while (lo < hi) {                               // if the other kernel flags them: the search stays in bounds)
            const int32_t mid = lo + ((hi - lo) >> 1);
            if (colidx[mid] < c) lo = mid + 1; else hi = mid;
        }
        if (lo >= rowptr[i + 1] || colidx[lo] != c || __float_as_uint(vals[lo]) != __float_as_uint(t_vals[pos]))
            bad |= VARCO_BAD_TRANSPOSE;
    }
    if (bad) atomicOr(flags, bad);
}
// Non-negative ids (a: n values), strictly ascending rows inside [0, limit) when ascending != 0.
__global__ __launch_bounds__(kBlock) void validate_ids_kernel(const int32_t* a, int64_t n, int32_t limit, int ascending,
                                                              int32_t bit, int32_t* flags) {
    const int64_t i = int64_t(blockIdx.x) * kBlock + threadIdx.x;
    if (i >= n) return;
    const int32_t v = a[i];
    bool bad = v < 0 || (limit > 0 && v >= limit);
    if (ascending && i > 0 && a[i - 1] >= v) bad = true;
    if (bad) atomicOr(flags, bit);
}

template <typename T, int VEC, int MODE>
hipError_t launch_spmm_vec(int nv, const SpmmArgs<T>& a, dim3 grid, size_t lds_bytes, hipStream_t stream) {
    switch (nv) {
        case 1: hipLaunchKernelGGL((spmm_kernel<T, VEC, 1, MODE>), grid, dim3(agg_block(MODE)), lds_bytes, stream, a); break;
        case 2: hipLaunchKernelGGL((spmm_kernel<T, VEC, 2, MODE>), grid, dim3(agg_block(MODE)), lds_bytes, stream, a); break;
        case 4: hipLaunchKernelGGL((spmm_kernel<T, VEC, 4, MODE>), grid, dim3(agg_block(MODE)), lds_bytes, stream, a); break;
        case 8: hipLaunchKernelGGL((spmm_kernel<T, VEC, 8, MODE>), grid, dim3(agg_block(MODE)), lds_bytes, stream, a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

bool aligned_to(const void* p, size_t bytes) { return (reinterpret_cast<uintptr_t>(p) & (bytes - 1)) == 0; }

template <typename T>
hipError_t spmm_t(const SpmmPlan& plan, const VarcoEdge* edge, const int32_t* colidx, const float* vals, const void* dense_v,
                  const void* z_v, int64_t z_rows, const MaskRule& rule, void* out_v, int32_t row_base, float* partial,
                  hipStream_t stream, const LaunchTag& tag) {
    const T* dense = static_cast<const T*>(dense_v);
    const T* z = static_cast<const T*>(z_v);
    T* out = static_cast<T*>(out_v);
    const int32_t width = int32_t(rule.width);
    const bool full = rule.k == rule.width;
    const bool halo = edge != nullptr;
    const bool vec4 = width % 4 == 0 && aligned_to(dense, 4 * sizeof(T)) && aligned_to(out, 4 * sizeof(T)) &&
                      aligned_to(partial, 16) && (!(halo && full) || aligned_to(z, 4 * sizeof(T)));
    const int vec = vec4 ? 4 : 1;
    const int per_row = (width + vec - 1) / vec;   // loads of VEC elements that cover a row
    int lpr_log2 = 0;
    while ((1 << lpr_log2) < per_row && lpr_log2 < 6) ++lpr_log2;
    int nv = 1;
    while (nv * (1 << lpr_log2) < per_row) nv <<= 1;
    if (nv > 8) return hipErrorInvalidValue;

    SpmmArgs<T> a;
    a.items = plan.items;
    a.n_items = plan.n_items;
    a.edge = edge;
    a.colidx = colidx;
    a.vals = vals;
    a.dense = dense;
    a.z = z;
    a.rule = rule;
    a.out = out;
    a.row_base = row_base;
    a.partial = partial;
    a.lpr_log2 = lpr_log2;
    // Compressed rows: `ev` stored elements per lane and load, lpe = pow2 >= k / ev lanes per row, epi = 64 / lpe
    // rows per instruction, each with a private LDS row. Prefer wide loads, but keep the private rows of
    // a wavefront within 4 KB so that LDS does not limit the number of resident wavefronts.
    const int epi_cap = std::max(1, 1024 / width);
    a.ev = 1;
    for (int ev : {4, 2}) {
        if (rule.k % ev != 0 || !aligned_to(z, ev * sizeof(T))) continue;
        int lg = 0;
        while ((1 << lg) < int(rule.k) / ev && lg < 6) ++lg;
        if ((64 >> lg) <= epi_cap) {
            a.ev = ev;
            break;
        }
    }
    a.ku = int32_t(rule.k) / a.ev;
    a.lpe_log2 = 0;
    while ((1 << a.lpe_log2) < a.ku && a.lpe_log2 < 6) ++a.lpe_log2;
    a.epi = std::max(1, std::min(64 >> a.lpe_log2, epi_cap));
    // 16 or more lanes per compressed row, 4 elements each, rows of whole 128-position blocks read back 4 at a time
    a.swizzle = halo && !full && a.ev == 4 && a.lpe_log2 >= 4 && vec4 && width % 128 == 0 ? 1 : 0;
    const int agg_waves = agg_block(halo ? kHalo : kDenseOnly) / 64;
    const int32_t per_round = 8 * kXcdRun;                                         // see the kernel's XCD mapping
    const dim3 grid(((plan.n_items + agg_waves - 1) / agg_waves + per_round - 1) / per_round * per_round);
    size_t lds_bytes = 0;
    if (halo && !full)
        lds_bytes = size_t(agg_waves) * a.epi * width * sizeof(float) + size_t(rule.n_units) * sizeof(uint16_t);
    tag.begin(stream);
    hipError_t err;
    // compressed buffer below 4 GiB: 32-bit row offsets (z_rows = 0: size unknown)
    const bool z32 = halo && !full && z_rows > 0 && z_rows * int64_t(rule.k) * int64_t(sizeof(T)) < (int64_t(1) << 32);
    if (halo && z32)
        err = vec4 ? launch_spmm_vec<T, 4, kHaloZ32>(nv, a, grid, lds_bytes, stream)
                   : launch_spmm_vec<T, 1, kHaloZ32>(nv, a, grid, lds_bytes, stream);
    else if (halo)
        err = vec4 ? launch_spmm_vec<T, 4, kHalo>(nv, a, grid, lds_bytes, stream)
                   : launch_spmm_vec<T, 1, kHalo>(nv, a, grid, lds_bytes, stream);
    else
        err = vec4 ? launch_spmm_vec<T, 4, kDenseOnly>(nv, a, grid, lds_bytes, stream)
                   : launch_spmm_vec<T, 1, kDenseOnly>(nv, a, grid, lds_bytes, stream);
    tag.end(stream);
    if (err != hipSuccess) return err;
    if (plan.n_splits > 0) {
        // the split records, every fp32 partial row once, every split row written once
        tag.begin_as(VARCO_K_REDUCE, stream, 16.0 * plan.n_splits + 4.0 * double(plan.n_partials) * width +
                                                 double(sizeof(T)) * plan.n_splits * width);
        if (vec4)
            hipLaunchKernelGGL(spmm_fixup4_kernel<T>, dim3(plan.n_splits), dim3(kBlock), 0, stream, plan.splits, plan.n_splits,
                               partial, out, row_base, width);
        else
            hipLaunchKernelGGL(spmm_fixup_kernel<T>, dim3(plan.n_splits), dim3(kBlock), 0, stream, plan.splits, plan.n_splits,
                               partial, out, row_base, width);
        tag.end(stream);
        err = hipGetLastError();
    }
    return err;
}

// The short rows of a dense-only block (see spmm_short_rows_kernel); the block's other rows are on plan.items.
template <typename T>
hipError_t spmm_short_t(const SpmmPlan& plan, const int32_t* colidx, const float* vals, const void* dense_v, void* out_v,
                        int32_t width, int32_t row_base, hipStream_t stream, const LaunchTag& tag) {
    ShortRowArgs<T> a;
    a.rowptr = plan.short_rowptr;
    a.colidx = colidx;
    a.vals = vals;
    a.dense = static_cast<const T*>(dense_v);
    a.out = static_cast<T*>(out_v);
    a.r0 = plan.short_r0, a.n_rows = plan.short_rows, a.row_base = row_base;
    a.max_len = plan.short_max_len;
    a.width = width;
    const bool vec4 = width % 4 == 0 && aligned_to(a.dense, 4 * sizeof(T)) && aligned_to(a.out, 4 * sizeof(T));
    const int per_row = vec4 ? width / 4 : width;
    int nv = 1;
    while (nv * 64 < per_row) nv <<= 1;
    if (nv > 8) return hipErrorInvalidValue;
    const int32_t n_waves = (plan.short_rows + 3) / 4;
    const dim3 grid((n_waves + kWaves - 1) / kWaves), block(kBlock);
    tag.begin(stream);
    auto go = [&](auto vec, auto nvc) {
        hipLaunchKernelGGL((spmm_short_rows_kernel<T, decltype(vec)::value, decltype(nvc)::value>), grid, block, 0, stream, a);
    };
    auto with_nv = [&](auto vec) {
        switch (nv) {
            case 1: go(vec, std::integral_constant<int, 1>{}); break;
            case 2: go(vec, std::integral_constant<int, 2>{}); break;
            case 4: go(vec, std::integral_constant<int, 4>{}); break;
            default: go(vec, std::integral_constant<int, 8>{}); break;
        }
    };
    if (vec4)
        with_nv(std::integral_constant<int, 4>{});
    else
        with_nv(std::integral_constant<int, 1>{});
    tag.end(stream);
    return hipGetLastError();
}

template <typename T>
hipError_t halo_grad_t(const SpmmPlan& fwd_plan, const SpmmPlan& t_halo_plan, const VarcoEdge* edge, const float* vals,
                       const int32_t* prow, int32_t prod_base, const void* dm, const MaskRule& rule, void* prod_v,
                       void* out_v, int32_t row_base, float* partial, hipStream_t stream, const LaunchTag& tag,
                       const LaunchTag& sum_tag) {
    T* out = static_cast<T*>(out_v);
    T* prod = static_cast<T*>(prod_v);
    const int32_t width = int32_t(rule.width);
    int ev = 1;
    for (int c : {4, 2})
        if (rule.k % c == 0 && aligned_to(prod, c * sizeof(T)) && aligned_to(out, c * sizeof(T)) && aligned_to(partial, 4 * c)) {
            ev = c;
            break;
        }
    const int ku = int(rule.k) / ev;
    int lpe_log2 = 0;
    while ((1 << lpe_log2) < ku && lpe_log2 < 6) ++lpe_log2;

    ProductArgs<T> a;
    a.items = fwd_plan.items;
    a.n_items = fwd_plan.n_items;
    a.edge = edge;
    a.vals = vals;
    a.prow = prow;
    a.dm = static_cast<const T*>(dm);
    a.rule = rule;
    a.prod = prod;
    a.ev = ev, a.ku = ku, a.lpe_log2 = lpe_log2;
    const size_t lds_bytes = size_t(kWaves) * width * sizeof(float) + size_t(rule.n_units) * sizeof(uint16_t);
    tag.begin(stream);
    hipLaunchKernelGGL(halo_products_kernel<T>, dim3((fwd_plan.n_items + kWaves - 1) / kWaves), dim3(kBlock), lds_bytes,
                       stream, a);
    tag.end(stream);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    SegsumArgs<T> b;
    b.items = t_halo_plan.items;
    b.n_items = t_halo_plan.n_items;
    b.prod = prod;
    b.prod_base = prod_base;
    b.k = int32_t(rule.k);
    b.out = out;
    b.row_base = row_base;
    b.partial = partial;
    b.ev = ev, b.ku = ku, b.lpe_log2 = lpe_log2;
    if (std::is_same_v<T, bf16_t> && rule.k % 8 == 0 && aligned_to(prod, 16) && aligned_to(out, 16) && aligned_to(partial, 16)) {
        b.ev = 8, b.ku = int(rule.k) / 8;      // the sums read 16 bytes per lane (the products above are written 4 elements at a time)
        b.lpe_log2 = 0;
        while ((1 << b.lpe_log2) < b.ku && b.lpe_log2 < 6) ++b.lpe_log2;
    }
    const int64_t threads = int64_t(t_halo_plan.n_items) << b.lpe_log2;
    sum_tag.begin(stream);
    hipLaunchKernelGGL(halo_segsum_kernel<T>, dim3(unsigned((threads + kBlock - 1) / kBlock)), dim3(kBlock), 0, stream, b);
    sum_tag.end(stream);
    err = hipGetLastError();
    if (err != hipSuccess) return err;
    if (t_halo_plan.n_splits > 0) {
        tag.begin_as(VARCO_K_REDUCE, stream, 16.0 * t_halo_plan.n_splits + 4.0 * double(t_halo_plan.n_partials) * rule.k +
                                                 double(sizeof(T)) * t_halo_plan.n_splits * rule.k);
        if (ev == 4)
            hipLaunchKernelGGL(spmm_fixup4_kernel<T>, dim3(t_halo_plan.n_splits), dim3(kBlock), 0, stream, t_halo_plan.splits,
                               t_halo_plan.n_splits, partial, out, row_base, int32_t(rule.k));
        else
            hipLaunchKernelGGL(spmm_fixup_kernel<T>, dim3(t_halo_plan.n_splits), dim3(kBlock), 0, stream, t_halo_plan.splits,
                               t_halo_plan.n_splits, partial, out, row_base, int32_t(rule.k));
        tag.end(stream);
        err = hipGetLastError();
    }
    return err;
}

}  // namespace

hipError_t varco_launch_build_edges(const int32_t* colidx, int64_t nnz, int32_t n_local, const int32_t* halo_zrow,
                                    const int32_t* halo_gid, VarcoEdge* edge, hipStream_t stream) {
    if (nnz == 0) return hipSuccess;
    hipLaunchKernelGGL(build_edges_kernel, dim3(unsigned((nnz + kBlock - 1) / kBlock)), dim3(kBlock), 0, stream, colidx,
                       nnz, n_local, halo_zrow, halo_gid, edge);
    return hipGetLastError();
}

hipError_t varco_launch_validate_partition(const varco_partition_desc& d, int32_t* flags, hipStream_t stream) {
    const int32_t n_cols = d.n_local + d.n_halo;
    auto blocks = [](int64_t n) { return dim3(unsigned((n + kBlock - 1) / kBlock)); };
    if (d.n_local > 0 && d.nnz > 0)
        hipLaunchKernelGGL(validate_rows_kernel, blocks(d.n_local), dim3(kBlock), 0, stream, d.rowptr, d.colidx, d.n_local,
                           n_cols, flags);
    if (n_cols > 0 && d.nnz > 0)
        hipLaunchKernelGGL(validate_trows_kernel, blocks(n_cols), dim3(kBlock), 0, stream, d.rowptr, d.colidx, d.vals,
                           d.n_local, n_cols, d.t_rowptr, d.t_colidx, d.t_vals, flags);
    struct Ids { const int32_t* a; int64_t n; int32_t limit; int ascending; int32_t bit; };
    const Ids lists[] = {{d.local_gid, d.n_local, 0, 0, VARCO_BAD_ID}, {d.halo_gid, d.n_halo, 0, 0, VARCO_BAD_ID},
                         {d.halo_zrow, d.n_halo, 0, 0, VARCO_BAD_ID}, {d.halo_src_row, d.n_halo, 0, 0, VARCO_BAD_ID},
                         {d.boundary_rows, d.n_boundary, d.n_local, 1, VARCO_BAD_BOUNDARY},
                         {d.ret_src, d.ret_src ? d.n_returned : 0, 0, 0, VARCO_BAD_RETURN_MAP}};
    for (const Ids& l : lists)
        if (l.n > 0 && l.a)
            hipLaunchKernelGGL(validate_ids_kernel, blocks(l.n), dim3(kBlock), 0, stream, l.a, l.n, l.limit, l.ascending, l.bit, flags);
    return hipGetLastError();
}

hipError_t varco_launch_spmm(int dtype, const SpmmPlan& plan, const VarcoEdge* edge, const int32_t* colidx,
                             const float* vals, const void* dense, const void* z, int64_t z_rows, const MaskRule& rule,
                             void* out, int32_t row_base, float* partial, hipStream_t stream, const LaunchTag& tag) {
    hipError_t err = hipSuccess;
    if (plan.n_items > 0)
        err = dtype == VARCO_BF16
                  ? spmm_t<bf16_t>(plan, edge, colidx, vals, dense, z, z_rows, rule, out, row_base, partial, stream, tag)
                  : spmm_t<float>(plan, edge, colidx, vals, dense, z, z_rows, rule, out, row_base, partial, stream, tag);
    if (err != hipSuccess || plan.short_rows == 0) return err;
    if (edge) return hipErrorInvalidValue;     // short-row plans are built for dense-only blocks
    LaunchTag rest = tag;                      // the block's bytes are booked once
    if (plan.n_items > 0) rest.bytes = 0, rest.flops = 0;
    return dtype == VARCO_BF16
               ? spmm_short_t<bf16_t>(plan, colidx, vals, dense, out, int32_t(rule.width), row_base, stream, rest)
               : spmm_short_t<float>(plan, colidx, vals, dense, out, int32_t(rule.width), row_base, stream, rest);
}

hipError_t varco_launch_build_prow(const int32_t* rowptr, const int32_t* colidx, int32_t n_local,
                                   const int32_t* t_rowptr, const int32_t* t_colidx, int32_t* prow, hipStream_t stream) {
    if (n_local == 0) return hipSuccess;
    hipLaunchKernelGGL(build_prow_kernel, dim3(unsigned((n_local + kBlock - 1) / kBlock)), dim3(kBlock), 0, stream, rowptr,
                       colidx, n_local, t_rowptr, t_colidx, prow);
    return hipGetLastError();
}

hipError_t varco_launch_halo_grad(int dtype, const SpmmPlan& fwd_plan, const SpmmPlan& t_halo_plan, const VarcoEdge* edge,
                                  const float* vals, const int32_t* prow, int32_t prod_base, const void* dm,
                                  const MaskRule& rule, void* prod, void* out, int32_t row_base, float* partial,
                                  hipStream_t stream, const LaunchTag& tag, const LaunchTag& sum_tag) {
    if (t_halo_plan.n_items == 0 || fwd_plan.n_items == 0) return hipSuccess;
    return dtype == VARCO_BF16 ? halo_grad_t<bf16_t>(fwd_plan, t_halo_plan, edge, vals, prow, prod_base, dm, rule, prod, out,
                                                     row_base, partial, stream, tag, sum_tag)
                               : halo_grad_t<float>(fwd_plan, t_halo_plan, edge, vals, prow, prod_base, dm, rule, prod, out,
                                                    row_base, partial, stream, tag, sum_tag);
}
