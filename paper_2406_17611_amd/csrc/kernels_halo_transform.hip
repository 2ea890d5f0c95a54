// The halo block of a layer that applies its weights before the aggregation (eq. (2) read as S (X H)): the halo
// rows exist only in compressed form, k received elements each, and are transformed from those (bf16 storage).
//
//   forward   Y[s, :]      = sum_j z[s, j] H[pi_s(j), :]                    (halo rows x width[l+1])
//   weights   dH[pi_s(j), :] += z[s, j] dY[s, :]   summed over the halo rows
//   errors    dz[s, j]     = sum_c dY[s, c] H[pi_s(j), c]                   (handed back in compressed form)
//
// Every row has a position rule of its own, so none of these is a plain dense product; but a row's rule is a
// permutation of the positions, and a tile of rows, written out densely with zeros at the positions that were not
// kept, is an operand the bf16 matrix units take. A workgroup therefore reads the compressed rows of its tile with
// contiguous 16-byte loads, scatters (forward, weights) or gathers (errors) their elements through a dense tile in
// LDS, 2 bytes at a time - LDS takes 64 scattered accesses in a few cycles, whereas 64 scattered 2-byte accesses
// to memory cost the vector memory unit about a cycle each (a first version that read the kept elements of a
// dense-looking operand straight from memory ran five times slower than this one) - and multiplies from LDS.
// The dense tile is never zeroed between tiles: the positions a tile wrote are cleared again after use, k writes per
// row instead of width. Workgroups are persistent over the tiles, so that the weights are fetched once.
#include <algorithm>

#include "elem.h"
#include "varco_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kMaxWidth = 512;              // positions of a row: 4 wavefronts x 4 blocks of 32
constexpr int kPitch = kMaxWidth + 8;       // elements per dense row in LDS (rows start 4 banks apart)
constexpr int kTile = 64;                   // halo rows per tile (forward, errors)
constexpr int kTileT = 32;                  // halo rows per tile of the transposed layout (weights)
constexpr int kPitchT = kTileT + 8;         // elements per position in the transposed layout
constexpr int kPitchC = 64 + 8;             // elements per row of a tile of dY (at most 64 columns)

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct HaloRows {
    const uint16_t* z;      // compressed rows, k elements each
    const uint2* rec;       // per halo row: {(a << 16) | b, row of z}: element j sits at position (a j + b) mod width
    int32_t n;              // halo rows
    uint32_t width, k, magic;
    int32_t fo;             // columns of the transformed rows
};

__device__ __forceinline__ uint32_t position(const HaloRows& p, uint32_t ab, uint32_t j) {
    const uint32_t x = (ab >> 16) * j + (ab & 0xFFFFu);
    const uint32_t r = x - __umulhi(x, p.magic) * p.width;
    return r >= p.width ? r - p.width : r;
}

__device__ __forceinline__ bf16x8 zero_fragment() { return __builtin_bit_cast(bf16x8, make_uint4(0u, 0u, 0u, 0u)); }
__device__ __forceinline__ bf16x8 fragment(const uint16_t* p) { return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(p)); }

enum { kScatter = 0, kClear = 1, kGather = 2 };

// Element (position, row) of the transposed tile. The lanes that scatter one row write positions that differ by
// multiples of 8, i.e. by multiples of 160 words with the 80-byte pitch: all in one LDS bank. So the four groups of
// 8 rows of a position are stored in an order that depends on the position (bits 3-4), which spreads those writes
// over four banks; a fragment (8 consecutive rows of one position) stays one aligned 16-byte read.
__device__ __forceinline__ int transposed_cell(int pos, int r) {
    return pos * kPitchT + ((((r >> 3) ^ (pos >> 3)) & 3) << 3) + (r & 7);
}

// What a thread needs of the first kAhead chunks it walks in a tile (chunks of 8 elements): the rows' rules and, for
// a scatter, the compressed elements. Fetched one tile ahead, so that the loads are in flight while the previous tile
// is multiplied, stored and cleared; a tile of 64 rows of up to 128 kept elements is covered entirely.
constexpr int kAhead = 4;
struct Ahead {
    uint4 data[kAhead];
    uint32_t ab[kAhead];
};

template <bool WITH_DATA>
__device__ __forceinline__ void fetch_ahead(const HaloRows& p, int32_t row0, int32_t rows, Ahead& f) {
    const int32_t per_row = int32_t(p.k) / 8;
    const int32_t total = rows * per_row;
#pragma unroll
    for (int i = 0; i < kAhead; ++i) {
        const int32_t idx = threadIdx.x + i * kThreads;
        f.ab[i] = 0u;
        f.data[i] = make_uint4(0u, 0u, 0u, 0u);
        if (idx < total) {
            const int32_t r = idx / per_row;
            const uint2 rec = p.rec[row0 + r];
            f.ab[i] = rec.x;
            if constexpr (WITH_DATA)
                f.data[i] = *reinterpret_cast<const uint4*>(p.z + int64_t(rec.y) * p.k + uint32_t(idx - r * per_row) * 8u);
        }
    }
}

// Walks the kept elements of rows [row0, row0 + rows) in chunks of VEC (8 when k is a multiple of 8 and the buffers
// are 16-byte aligned, else 1): kScatter writes them into the dense tile, kClear writes zeros to the same places,
// kGather reads the tile at those places and stores the compressed rows to `out`. TRANSPOSED: the tile is
// [position][row] instead of [row][position]. ahead (VEC = 8 only): what fetch_ahead brought for this tile; the
// chunks it covers need no loads here.
template <int VEC, int MODE, bool TRANSPOSED>
__device__ __forceinline__ void walk_rows(const HaloRows& p, int32_t row0, int32_t rows, uint16_t* tile, uint16_t* out,
                                          const Ahead* ahead = nullptr) {
    const int32_t per_row = int32_t(p.k) / VEC;
    const int32_t total = rows * per_row;
    auto chunk = [&](int32_t idx, bool have, uint32_t ab_have, const uint4& data_have) {
        const int32_t r = idx / per_row;
        const uint32_t j0 = uint32_t(idx - r * per_row) * VEC;
        uint32_t ab = ab_have;
        int64_t zrow = 0;
        if (!have) {
            const uint2 rec = p.rec[row0 + r];
            ab = rec.x, zrow = rec.y;
        }
        const uint32_t a = ab >> 16;
        uint32_t pos = position(p, ab, j0);
        if constexpr (VEC == 8 && !TRANSPOSED) {
            if (p.k == p.width) {   // every element kept: position j holds element j, a chunk is 16 contiguous bytes on both sides
                uint4* cell = reinterpret_cast<uint4*>(tile + r * kPitch + int32_t(j0));
                if constexpr (MODE == kScatter)
                    *cell = have ? data_have : *reinterpret_cast<const uint4*>(p.z + zrow * p.k + j0);
                else if constexpr (MODE == kClear)
                    *cell = make_uint4(0u, 0u, 0u, 0u);
                else
                    *reinterpret_cast<uint4*>(out + int64_t(row0 + r) * p.k + j0) = *cell;
                return;
            }
        }
        uint16_t v[VEC];
        if constexpr (MODE == kScatter) {
            if constexpr (VEC == 8) {
                const uint4 u = have ? data_have : *reinterpret_cast<const uint4*>(p.z + zrow * p.k + j0);
                const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = uint16_t(w[e >> 1] >> (16 * (e & 1)));
            } else {
                v[0] = p.z[zrow * p.k + j0];
            }
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            uint16_t* cell = tile + (TRANSPOSED ? transposed_cell(int32_t(pos), r) : r * kPitch + int32_t(pos));
            if constexpr (MODE == kScatter)
                *cell = v[e];
            else if constexpr (MODE == kClear)
                *cell = 0;
            else
                v[e] = *cell;
            pos += a;
            if (pos >= p.width) pos -= p.width;
        }
        if constexpr (MODE == kGather) {
            uint16_t* dst = out + int64_t(row0 + r) * p.k + j0;
            if constexpr (VEC == 8) {
                uint32_t w[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) w[q] = uint32_t(v[2 * q]) | (uint32_t(v[2 * q + 1]) << 16);
                *reinterpret_cast<uint4*>(dst) = make_uint4(w[0], w[1], w[2], w[3]);
            } else {
                dst[0] = v[0];
            }
        }
    };
    int32_t idx = threadIdx.x;
    if constexpr (VEC == 8) {
        if (ahead) {
#pragma unroll
            for (int i = 0; i < kAhead; ++i) {
                if (idx < total) chunk(idx, true, ahead->ab[i], ahead->data[i]);
                idx += kThreads;
            }
        }
    }
    const uint4 none = make_uint4(0u, 0u, 0u, 0u);
    for (; idx < total; idx += kThreads) chunk(idx, false, 0u, none);
}

// The elements of a tile of dY that a thread copies into LDS (the tile's rows are one contiguous range of `count`
// elements), fetched one tile ahead; N covers the largest tile (rows x 64 columns).
template <int N>
__device__ __forceinline__ void fetch_dy(const uint16_t* __restrict__ src, int32_t count, uint16_t (&v)[N]) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const int32_t e = threadIdx.x + i * kThreads;
        v[i] = e < count ? src[e] : uint16_t(0);
    }
}

__device__ __forceinline__ void zero_lds(uint16_t* s, int32_t elems) {     // elems: a multiple of 8
    for (int32_t i = threadIdx.x * 8; i < elems; i += kThreads * 8) *reinterpret_cast<uint4*>(s + i) = make_uint4(0u, 0u, 0u, 0u);
}

// ---- forward: Y = X~ H, H given as its bf16 copy [column][position] (pitch wpitch >= width, a multiple of 8) ----
// Wavefront w multiplies rows 32 (w / 2) .. + 31 of the tile by columns 32 (w % 2) .. + 31; its columns' weights
// stay in registers for the whole kernel (one fragment per 16 positions).
template <int VEC>
__global__ __launch_bounds__(kThreads, 2) void halo_transform_fwd_kernel(HaloRows p, const uint16_t* __restrict__ wt,
                                                                        int32_t wpitch, uint16_t* __restrict__ y) {
    __shared__ __attribute__((aligned(16))) uint16_t tile[kTile * kPitch];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lrow = lane & 31, lk = lane >> 5;
    const int rb = wave >> 1, col = (wave & 1) * 32 + lrow;
    const int steps = int(p.width) / 16;          // width is a multiple of 16
    bf16x8 wf[kMaxWidth / 16];
#pragma unroll
    for (int s = 0; s < kMaxWidth / 16; ++s) {
        wf[s] = zero_fragment();
        if (s < steps && col < p.fo) wf[s] = fragment(wt + int64_t(col) * wpitch + 16 * s + 8 * lk);
    }
    zero_lds(tile, kTile * kPitch);
    __syncthreads();
    const int32_t n_tiles = (p.n + kTile - 1) / kTile;
    Ahead next, cur;
    if (VEC == 8 && int32_t(blockIdx.x) < n_tiles) fetch_ahead<true>(p, blockIdx.x * kTile, min(kTile, p.n - int32_t(blockIdx.x) * kTile), next);
    for (int32_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        const int32_t row0 = t * kTile, rows = min(kTile, p.n - row0);
        cur = next;
        walk_rows<VEC, kScatter, false>(p, row0, rows, tile, nullptr, VEC == 8 ? &cur : nullptr);
        __syncthreads();
        const int32_t tn = t + int32_t(gridDim.x);
        if (VEC == 8 && tn < n_tiles) fetch_ahead<true>(p, tn * kTile, min(kTile, p.n - tn * kTile), next);
        floatx16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.f;
        const uint16_t* arow = tile + (rb * 32 + lrow) * kPitch + 8 * lk;
#pragma unroll
        for (int s = 0; s < kMaxWidth / 16; ++s)
            if (s < steps) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fragment(arow + 16 * s), wf[s], acc, 0, 0, 0);
        // accumulator register v of a lane is element (8 * (v / 4) + 4 * (lane / 32) + v % 4, lane % 32)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int32_t r = rb * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
            if (r < rows && col < p.fo) y[int64_t(row0 + r) * p.fo + col] = float_to_bf16(acc[v]);
        }
        __syncthreads();                           // every fragment has been read
        walk_rows<VEC, kClear, false>(p, row0, rows, tile, nullptr, VEC == 8 ? &cur : nullptr);
        __syncthreads();
    }
}

// ---- errors handed back: dz[s, j] = (dY[s, :] H^T)[pi_s(j)], H given as its bf16 copy [position][column] (pitch
// cpitch, a multiple of 8, zero beyond the columns) ----
// Wavefront w produces positions 128 w .. + 127 of all 64 rows of the tile; the dense rows go to LDS as bf16 and the
// kept elements are gathered from there.
template <int VEC>
__global__ __launch_bounds__(kThreads, 2) void halo_transform_bwd_kernel(HaloRows p, const uint16_t* __restrict__ dy,
                                                                        const uint16_t* __restrict__ wr, int32_t cpitch,
                                                                        uint16_t* __restrict__ dz) {
    __shared__ __attribute__((aligned(16))) uint16_t tile[kTile * kPitch];
    __shared__ __attribute__((aligned(16))) uint16_t dtile[kTile * kPitchC];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lrow = lane & 31, lk = lane >> 5;
    const int ksteps = (p.fo + 15) / 16;          // at most 4
    bf16x8 wf[4][4];                              // [block of 32 positions][16 columns]
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const int32_t pos = wave * 128 + b * 32 + lrow;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            wf[b][s] = zero_fragment();
            const int32_t c0 = 16 * s + 8 * lk;    // a chunk of 8 columns lies wholly inside the pitch or outside
            if (s < ksteps && pos < int32_t(p.width) && c0 + 8 <= cpitch) wf[b][s] = fragment(wr + int64_t(pos) * cpitch + c0);
        }
    }
    zero_lds(dtile, kTile * kPitchC);
    __syncthreads();
    const int32_t n_tiles = (p.n + kTile - 1) / kTile;
    constexpr int kDy = kTile * 64 / kThreads;     // elements of a tile of dY per thread
    uint16_t dnext[kDy];
    Ahead next, cur;
    auto fetch_tile = [&](int32_t t) {
        const int32_t row0 = t * kTile, rows = min(kTile, p.n - row0);
        fetch_dy<kDy>(dy + int64_t(row0) * p.fo, rows * p.fo, dnext);
        if (VEC == 8) fetch_ahead<false>(p, row0, rows, next);
    };
    if (int32_t(blockIdx.x) < n_tiles) fetch_tile(blockIdx.x);
    for (int32_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        const int32_t row0 = t * kTile, rows = min(kTile, p.n - row0);
        // the tile's rows of dY are one contiguous range (columns beyond fo stay zero; rows beyond the tile keep an
        // older tile's values, and their results are never read)
#pragma unroll
        for (int i = 0; i < kDy; ++i) {
            const int32_t e = threadIdx.x + i * kThreads;
            if (e < rows * p.fo) {
                const int32_t r = e / p.fo;
                dtile[r * kPitchC + (e - r * p.fo)] = dnext[i];
            }
        }
        cur = next;
        __syncthreads();
        if (t + int32_t(gridDim.x) < n_tiles) fetch_tile(t + gridDim.x);
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            bf16x8 fa[4];
#pragma unroll
            for (int s = 0; s < 4; ++s) fa[s] = s < ksteps ? fragment(dtile + (rb * 32 + lrow) * kPitchC + 16 * s + 8 * lk) : zero_fragment();
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                floatx16 acc;
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
                for (int s = 0; s < 4; ++s)
                    if (s < ksteps) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[s], wf[b][s], acc, 0, 0, 0);
                const int32_t pos = wave * 128 + b * 32 + lrow;
                if (pos < int32_t(p.width)) {
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        tile[(rb * 32 + 8 * (v >> 2) + 4 * lk + (v & 3)) * kPitch + pos] = float_to_bf16(acc[v]);
                }
            }
        }
        __syncthreads();
        walk_rows<VEC, kGather, false>(p, row0, rows, tile, dz, VEC == 8 ? &cur : nullptr);
        __syncthreads();                           // the next tile overwrites both LDS blocks
    }
}

// ---- weight gradient: partial[g][position][column] = sum over workgroup g's tiles of X~^T dY ----
// The dense tile is kept transposed, [position][row], so that the positions are the rows of the matrix product.
// Wavefront w accumulates positions 128 w .. + 127 x 64 columns in registers over all of its workgroup's tiles.
template <int VEC>
__global__ __launch_bounds__(kThreads, 2) void halo_transform_wgrad_kernel(HaloRows p, const uint16_t* __restrict__ dy,
                                                                          float* __restrict__ partial) {
    __shared__ __attribute__((aligned(16))) uint16_t tile[kMaxWidth * kPitchT];
    __shared__ __attribute__((aligned(16))) uint16_t dtile[64 * kPitchT];      // [column][row]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lrow = lane & 31, lk = lane >> 5;
    floatx16 acc[4][2];
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[b][c][v] = 0.f;
    zero_lds(tile, kMaxWidth * kPitchT);
    zero_lds(dtile, 64 * kPitchT);
    __syncthreads();
    const int32_t n_tiles = (p.n + kTileT - 1) / kTileT;
    constexpr int kDy = kTileT * 64 / kThreads;    // elements of a tile of dY per thread
    uint16_t dnext[kDy];
    Ahead next, cur;
    auto fetch_tile = [&](int32_t t) {
        const int32_t row0 = t * kTileT, rows = min(kTileT, p.n - row0);
        fetch_dy<kDy>(dy + int64_t(row0) * p.fo, rows * p.fo, dnext);      // rows beyond the tile: zeros
        if (VEC == 8) fetch_ahead<true>(p, row0, rows, next);
    };
    if (int32_t(blockIdx.x) < n_tiles) fetch_tile(blockIdx.x);
    for (int32_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        const int32_t row0 = t * kTileT, rows = min(kTileT, p.n - row0);
        cur = next;
        walk_rows<VEC, kScatter, true>(p, row0, rows, tile, nullptr, VEC == 8 ? &cur : nullptr);
#pragma unroll
        for (int i = 0; i < kDy; ++i) {
            const int32_t e = threadIdx.x + i * kThreads;
            if (e < kTileT * p.fo) {
                const int32_t r = e / p.fo;
                dtile[(e - r * p.fo) * kPitchT + r] = dnext[i];
            }
        }
        __syncthreads();
        if (t + int32_t(gridDim.x) < n_tiles) fetch_tile(t + gridDim.x);
#pragma unroll
        for (int s = 0; s < kTileT / 16; ++s) {
            bf16x8 fb[2];
#pragma unroll
            for (int c = 0; c < 2; ++c) fb[c] = fragment(dtile + (c * 32 + lrow) * kPitchT + 16 * s + 8 * lk);
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const bf16x8 fa = fragment(tile + transposed_cell(wave * 128 + b * 32 + lrow, 16 * s + 8 * lk));
#pragma unroll
                for (int c = 0; c < 2; ++c) acc[b][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb[c], acc[b][c], 0, 0, 0);
            }
        }
        __syncthreads();
        walk_rows<VEC, kClear, true>(p, row0, rows, tile, nullptr, VEC == 8 ? &cur : nullptr);
        __syncthreads();
    }
    float* out = partial + int64_t(blockIdx.x) * p.width * p.fo;
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int32_t pos = wave * 128 + b * 32 + 8 * (v >> 2) + 4 * lk + (v & 3), col = c * 32 + lrow;
                if (pos < int32_t(p.width) && col < p.fo) out[int64_t(pos) * p.fo + col] = acc[b][c][v];
            }
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool shape_ok(const HaloTransform& h) {
    return h.width >= 16 && h.width <= uint32_t(kMaxWidth) && h.width % 16 == 0 && h.k <= h.width && h.fo >= 1 && h.fo <= 64 &&
           h.rec && (h.z || h.k == 0);
}

HaloRows device_args(const HaloTransform& h) {
    HaloRows p;
    p.z = static_cast<const uint16_t*>(h.z);
    p.rec = h.rec;
    p.n = h.n;
    p.width = h.width, p.k = h.k, p.magic = h.width_magic;
    p.fo = h.fo;
    return p;
}

unsigned grid_for(int32_t n, int tile_rows, int64_t cap) {
    const int64_t tiles = (int64_t(n) + tile_rows - 1) / tile_rows;
    return unsigned(std::max<int64_t>(1, std::min<int64_t>(tiles, cap)));
}

}  // namespace

hipError_t varco_launch_halo_transform_fwd(const HaloTransform& h, const void* wt, int32_t wpitch, void* y, hipStream_t stream) {
    if (h.n <= 0) return hipSuccess;
    if (!shape_ok(h) || !wt || !y || wpitch < int32_t(h.width) || wpitch % 8 != 0 || !aligned16(wt)) return hipErrorInvalidValue;
    const HaloRows p = device_args(h);
    const dim3 grid(grid_for(h.n, kTile, 512)), block(kThreads);
    if (h.k % 8 == 0 && aligned16(h.z))
        hipLaunchKernelGGL(halo_transform_fwd_kernel<8>, grid, block, 0, stream, p, static_cast<const uint16_t*>(wt), wpitch,
                           static_cast<uint16_t*>(y));
    else
        hipLaunchKernelGGL(halo_transform_fwd_kernel<1>, grid, block, 0, stream, p, static_cast<const uint16_t*>(wt), wpitch,
                           static_cast<uint16_t*>(y));
    return hipGetLastError();
}

hipError_t varco_launch_halo_transform_bwd(const HaloTransform& h, const void* dy, const void* wr, int32_t cpitch, void* dz,
                                           hipStream_t stream) {
    if (h.n <= 0 || h.k == 0) return hipSuccess;
    if (!shape_ok(h) || !dy || !wr || !dz || cpitch < h.fo || cpitch % 8 != 0 || !aligned16(wr)) return hipErrorInvalidValue;
    const HaloRows p = device_args(h);
    const dim3 grid(grid_for(h.n, kTile, 512)), block(kThreads);
    if (h.k % 8 == 0 && aligned16(dz))
        hipLaunchKernelGGL(halo_transform_bwd_kernel<8>, grid, block, 0, stream, p, static_cast<const uint16_t*>(dy),
                           static_cast<const uint16_t*>(wr), cpitch, static_cast<uint16_t*>(dz));
    else
        hipLaunchKernelGGL(halo_transform_bwd_kernel<1>, grid, block, 0, stream, p, static_cast<const uint16_t*>(dy),
                           static_cast<const uint16_t*>(wr), cpitch, static_cast<uint16_t*>(dz));
    return hipGetLastError();
}

hipError_t varco_launch_halo_transform_wgrad(const HaloTransform& h, const void* dy, float* partial, int64_t partial_elems,
                                             int32_t* slabs, hipStream_t stream) {
    *slabs = 0;
    if (h.n <= 0 || h.k == 0) return hipSuccess;
    if (!shape_ok(h) || !dy || !partial) return hipErrorInvalidValue;
    const int64_t fit = partial_elems / (int64_t(h.width) * h.fo);
    if (fit < 1) return hipErrorInvalidValue;
    const HaloRows p = device_args(h);
    const dim3 grid(grid_for(h.n, kTileT, std::min<int64_t>(512, fit))), block(kThreads);
    *slabs = int32_t(grid.x);
    if (h.k % 8 == 0 && aligned16(h.z))
        hipLaunchKernelGGL(halo_transform_wgrad_kernel<8>, grid, block, 0, stream, p, static_cast<const uint16_t*>(dy), partial);
    else
        hipLaunchKernelGGL(halo_transform_wgrad_kernel<1>, grid, block, 0, stream, p, static_cast<const uint16_t*>(dy), partial);
    return hipGetLastError();
}
