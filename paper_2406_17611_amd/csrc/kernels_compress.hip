// Encoder and decoder of Definition 1 / Appendix "Compression Mechanism": keep k keyed-random elements of
// each node vector; decode by writing them in place and zero elsewhere (no rescale). Pure data movement:
// HBM-bound, no index bytes are stored or read. A power-of-two group of lanes serves one row, so that
// narrow messages (k of 4..32) still fill the 64-wide wavefront with several rows.
#include <algorithm>

#include "elem.h"
#include "mask_device.h"

namespace {

constexpr int kBlock = 256;

__device__ __forceinline__ float vec_elem(const float4& v, int i) { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }
__device__ __forceinline__ float vec_elem(const float2& v, int i) { return i == 0 ? v.x : v.y; }
__device__ __forceinline__ float vec_elem(const float& v, int) { return v; }

__device__ __forceinline__ int64_t group_row(int g_log2) {
    return (int64_t(blockIdx.x) * kBlock + threadIdx.x) >> g_log2;
}

template <typename T>
__global__ __launch_bounds__(kBlock) void compress_kernel(MaskRule rule, const int32_t* __restrict__ gids,
                                                          const int32_t* __restrict__ rows, int64_t n_rows,
                                                          const T* __restrict__ x, int64_t ldx,
                                                          T* __restrict__ z, int g_log2) {
    const uint32_t g = 1u << g_log2;
    const uint32_t gl = threadIdx.x & (g - 1);
    const int64_t stride = (int64_t(gridDim.x) * kBlock) >> g_log2;
    for (int64_t row = group_row(g_log2); row < n_rows; row += stride) {
        const int64_t src = rows ? int64_t(rows[row]) : row;
        const T* xr = x + src * ldx;
        T* zr = z + row * int64_t(rule.k);
        if (rule.k == rule.width) {
            for (uint32_t j = gl; j < rule.k; j += g) zr[j] = xr[j];
        } else {
            const MaskAffine m = varco_affine(rule, uint32_t(gids[row]));
            for (uint32_t j = gl; j < rule.k; j += g) zr[j] = xr[varco_position(rule, m, j)];
        }
    }
}

// bf16 rows: picking the kept elements straight from memory is 64 scattered 2-byte loads per instruction, which the
// vector memory unit takes about one per cycle. Here a wavefront copies the row into LDS with 16-byte loads (a
// 512-wide row is one instruction), picks from there, two elements per lane, and writes 4 bytes per lane.
// Needs width % 8 == 0, width <= kStagedWidth, k even, 16-byte aligned rows of x and 4-byte aligned rows of z.
constexpr int kStagedWidth = 2048;
__global__ __launch_bounds__(kBlock) void compress_staged_kernel(MaskRule rule, const int32_t* __restrict__ gids,
                                                                 const int32_t* __restrict__ rows, int64_t n_rows,
                                                                 const uint16_t* __restrict__ x, int64_t ldx,
                                                                 uint16_t* __restrict__ z) {
    __shared__ __attribute__((aligned(16))) uint16_t staged[kBlock / 64][kStagedWidth];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint16_t* row_lds = staged[wave];
    const int64_t stride = int64_t(gridDim.x) * (kBlock / 64);
    for (int64_t row = int64_t(blockIdx.x) * (kBlock / 64) + wave; row < n_rows; row += stride) {
        const uint16_t* xr = x + (rows ? int64_t(rows[row]) : row) * ldx;
        for (uint32_t c = lane * 8; c < rule.width; c += 512) *reinterpret_cast<uint4*>(row_lds + c) = *reinterpret_cast<const uint4*>(xr + c);
        const MaskAffine m = varco_affine(rule, uint32_t(gids[row]));
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");     // the wavefront's own LDS writes, then its reads
        uint16_t* zr = z + row * int64_t(rule.k);
        for (uint32_t j = 2 * lane; j < rule.k; j += 128) {
            const uint32_t p0 = varco_position(rule, m, j);
            uint32_t p1 = p0 + m.a;
            if (p1 >= rule.width) p1 -= rule.width;
            *reinterpret_cast<uint32_t*>(zr + j) = uint32_t(row_lds[p0]) | (uint32_t(row_lds[p1]) << 16);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");     // reads done before the next row overwrites the buffer
    }
}

// Full rows are written in one coalesced pass: column c holds z[j] when its inverse position j is kept.
template <typename T>
__global__ __launch_bounds__(kBlock) void decompress_kernel(MaskRule rule, const int32_t* __restrict__ gids,
                                                            const int32_t* __restrict__ rows, int64_t n_rows,
                                                            const T* __restrict__ z, T* __restrict__ x,
                                                            int64_t ldx, int g_log2) {
    const uint32_t g = 1u << g_log2;
    const uint32_t gl = threadIdx.x & (g - 1);
    const int64_t stride = (int64_t(gridDim.x) * kBlock) >> g_log2;
    for (int64_t row = group_row(g_log2); row < n_rows; row += stride) {
        const int64_t dst = rows ? int64_t(rows[row]) : row;
        T* xr = x + dst * ldx;
        const T* zr = z + row * int64_t(rule.k);
        if (rule.k == rule.width) {
            for (uint32_t c = gl; c < rule.width; c += g) xr[c] = zr[c];
        } else {
            const MaskAffine m = varco_affine(rule, uint32_t(gids[row]));
            for (uint32_t c = gl; c < rule.width; c += g) {
                const uint32_t j = varco_inverse_position(rule, m, c);
                xr[c] = j < rule.k ? zr[j] : T{};
            }
        }
    }
}

// Owner-side sum of returned errors: rows are distinct within a call and positions are distinct within a
// row, so plain read-modify-write is race-free and the result does not depend on scheduling.
template <typename T>
__global__ __launch_bounds__(kBlock) void decompress_add_kernel(MaskRule rule, const int32_t* __restrict__ gids,
                                                                const int32_t* __restrict__ rows, int64_t n_rows,
                                                                const T* __restrict__ z, T* __restrict__ x,
                                                                int64_t ldx, int g_log2) {
    const uint32_t g = 1u << g_log2;
    const uint32_t gl = threadIdx.x & (g - 1);
    const int64_t stride = (int64_t(gridDim.x) * kBlock) >> g_log2;
    for (int64_t row = group_row(g_log2); row < n_rows; row += stride) {
        const int64_t dst = rows ? int64_t(rows[row]) : row;
        T* xr = x + dst * ldx;
        const T* zr = z + row * int64_t(rule.k);
        MaskAffine m{1, 0, 1};
        if (rule.k != rule.width) m = varco_affine(rule, uint32_t(gids[row]));
        for (uint32_t j = gl; j < rule.k; j += g) {
            T* dstp = xr + (rule.k == rule.width ? j : varco_position(rule, m, j));
            Elem<T>::store(dstp, Elem<T>::load(dstp) + Elem<T>::load(zr + j));
        }
    }
}

// Owner-side sum over all consumers: a group of lanes (one per EV stored elements) owns one boundary row,
// adds up the rows returned for it (coalesced reads of k consecutive values each, four in flight), and
// touches the wide gradient row once.
template <typename T, int EV>
__global__ __launch_bounds__(kBlock) void accumulate_returned_kernel(MaskRule rule, const int32_t* __restrict__ gids,
                                                                     const int32_t* __restrict__ rows, int64_t n_rows,
                                                                     const int32_t* __restrict__ ptr,
                                                                     const int32_t* __restrict__ src,
                                                                     const T* __restrict__ returned,
                                                                     T* __restrict__ x, int64_t ldx, int g_log2) {
    using V = typename FloatVec<EV>::type;
    const uint32_t g = 1u << g_log2;
    const uint32_t gl = threadIdx.x & (g - 1);
    const int64_t stride = (int64_t(gridDim.x) * kBlock) >> g_log2;
    const int64_t k = rule.k;
    const uint32_t ku = rule.k / EV;
    for (int64_t b = group_row(g_log2); b < n_rows; b += stride) {
        const int32_t e0 = ptr[b], e1 = ptr[b + 1];
        if (e0 == e1) continue;
        T* xr = x + int64_t(rows[b]) * ldx;
        MaskAffine m{1, 0, 1};
        if (rule.k != rule.width) m = varco_affine(rule, uint32_t(gids[b]));
        for (uint32_t ju = gl; ju < ku; ju += g) {
            const uint32_t j = ju * EV;
            float acc[EV];
#pragma unroll
            for (int i = 0; i < EV; ++i) acc[i] = 0.f;
            for (int32_t e = e0; e < e1; e += 4) {          // rows past the end re-read row e0 and are dropped
                V v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) v[u] = load_vec<T, EV>(returned + int64_t(src[e + u < e1 ? e + u : e0]) * k + j);
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (e + u < e1) {
#pragma unroll
                        for (int i = 0; i < EV; ++i) acc[i] += vec_elem(v[u], i);
                    }
            }
            uint32_t pos = rule.k == rule.width ? j : varco_position(rule, m, j);
#pragma unroll
            for (int i = 0; i < EV; ++i) {
                Elem<T>::store(xr + pos, Elem<T>::load(xr + pos) + acc[i]);
                pos += rule.k == rule.width ? 1u : m.a;
                if (pos >= rule.width) pos -= rule.width;
            }
        }
    }
}

__global__ __launch_bounds__(kBlock) void calibration_copy_kernel(const float4* __restrict__ src,
                                                                  float4* __restrict__ dst, int64_t n) {
    const int64_t stride = int64_t(gridDim.x) * kBlock;
    for (int64_t i = int64_t(blockIdx.x) * kBlock + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

__global__ __launch_bounds__(kBlock) void sum_gradients_kernel(float* __restrict__ dst, const float* __restrict__ src,
                                                               int64_t n) {
    const int64_t stride = int64_t(gridDim.x) * kBlock;
    for (int64_t i = int64_t(blockIdx.x) * kBlock + threadIdx.x; i < n; i += stride) dst[i] += src[i];
}

__device__ __forceinline__ uint64_t mix64_device(uint64_t x) {   // splitmix64 output function
    x ^= x >> 30;
    x *= 0xBF58476D1CE4E5B9ull;
    x ^= x >> 27;
    x *= 0x94D049BB133111EBull;
    x ^= x >> 31;
    return x;
}

// One workgroup of 256 threads, thread t = tap address t.
__global__ __launch_bounds__(kBlock) void step_table_kernel(uint64_t* d_step, uint32_t* table, uint64_t key, int set,
                                                            uint64_t value) {
    const uint64_t step = set ? value : *d_step + 1;
    __syncthreads();                       // every thread has read the old step before it is replaced
    if (threadIdx.x == 0) *d_step = step;
    const uint64_t inner = mix64_device(step + 0x9E3779B97F4A7C15ull * uint64_t(threadIdx.x + 1));
    const uint64_t s = mix64_device(key ^ inner);
    table[2 * threadIdx.x] = uint32_t(s & 0xFFFFFFFFull);
    table[2 * threadIdx.x + 1] = uint32_t(s >> 32);
}

int group_log2(uint32_t elems) {
    int l = 0;
    while ((1u << l) < elems && l < 6) ++l;
    return l;
}

unsigned grid_for(int64_t n_rows, int g_log2) {
    const int64_t threads = n_rows << g_log2;
    int64_t blocks = (threads + kBlock - 1) / kBlock;
    const int64_t cap = 256 * 16;  // 16 resident blocks on each of the 256 compute units, grid-stride beyond
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    return unsigned(blocks);
}

// Per halo row: its position rule (element j sits at position (a j + b) mod width) and its row in the compressed
// buffer, for the kernels that transform halo rows from their received elements.
__global__ __launch_bounds__(kBlock) void halo_rows_kernel(MaskRule rule, const int32_t* __restrict__ gids,
                                                           const int32_t* __restrict__ zrow, int32_t n,
                                                           uint2* __restrict__ out) {
    const int32_t s = blockIdx.x * kBlock + threadIdx.x;
    if (s >= n) return;
    uint32_t ab = 1u << 16;                       // every element kept: position c holds element c
    if (rule.k < rule.width) {
        const MaskAffine m = varco_affine(rule, uint32_t(gids[s]));
        ab = (m.a << 16) | m.b;
    }
    out[s] = make_uint2(ab, uint32_t(zrow[s]));
}

template <typename T>
hipError_t launch_compress_t(const MaskRule& rule, const int32_t* gids, const int32_t* rows, int64_t n_rows, const void* x,
                             int64_t ldx, void* z, hipStream_t stream) {
    if (sizeof(T) == 2 && rule.k < rule.width && rule.k % 2 == 0 && rule.width % 8 == 0 && rule.width <= uint32_t(kStagedWidth) &&
        ldx % 8 == 0 && (reinterpret_cast<uintptr_t>(x) & 15u) == 0 && (reinterpret_cast<uintptr_t>(z) & 3u) == 0) {
        const int64_t blocks = std::min<int64_t>((n_rows + kBlock / 64 - 1) / (kBlock / 64), 256 * 8);
        hipLaunchKernelGGL(compress_staged_kernel, dim3(unsigned(blocks)), dim3(kBlock), 0, stream, rule, gids, rows, n_rows,
                           static_cast<const uint16_t*>(x), ldx, static_cast<uint16_t*>(z));
        return hipGetLastError();
    }
    const int gl = group_log2(rule.k);
    hipLaunchKernelGGL(compress_kernel<T>, dim3(grid_for(n_rows, gl)), dim3(kBlock), 0, stream, rule, gids, rows, n_rows,
                       static_cast<const T*>(x), ldx, static_cast<T*>(z), gl);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_decompress_t(const MaskRule& rule, const int32_t* gids, const int32_t* rows, int64_t n_rows,
                               const void* z, void* x, int64_t ldx, int accumulate, hipStream_t stream) {
    if (accumulate) {
        const int gl = group_log2(rule.k);
        hipLaunchKernelGGL(decompress_add_kernel<T>, dim3(grid_for(n_rows, gl)), dim3(kBlock), 0, stream, rule, gids,
                           rows, n_rows, static_cast<const T*>(z), static_cast<T*>(x), ldx, gl);
    } else {
        const int gl = group_log2(rule.width);
        hipLaunchKernelGGL(decompress_kernel<T>, dim3(grid_for(n_rows, gl)), dim3(kBlock), 0, stream, rule, gids, rows,
                           n_rows, static_cast<const T*>(z), static_cast<T*>(x), ldx, gl);
    }
    return hipGetLastError();
}

template <typename T>
hipError_t launch_accumulate_t(const MaskRule& rule, const int32_t* gids, const int32_t* rows, int64_t n_rows,
                               const int32_t* ptr, const int32_t* src, const void* returned, void* x, int64_t ldx,
                               hipStream_t stream) {
    // wide loads only while at least 32 lanes still share a row: fewer lanes per row means more rows per
    // wavefront, whose differing numbers of returned rows then serialise
    int ev = 1;
    for (int c : {4, 2})
        if (rule.k % c == 0 && rule.k / c >= 32 && (reinterpret_cast<uintptr_t>(returned) & (c * sizeof(T) - 1)) == 0) {
            ev = c;
            break;
        }
    const int gl = group_log2(rule.k / ev);
    const dim3 grid(grid_for(n_rows, gl)), block(kBlock);
    const T* ret = static_cast<const T*>(returned);
    T* xt = static_cast<T*>(x);
    if (ev == 4)
        hipLaunchKernelGGL((accumulate_returned_kernel<T, 4>), grid, block, 0, stream, rule, gids, rows, n_rows, ptr, src, ret,
                           xt, ldx, gl);
    else if (ev == 2)
        hipLaunchKernelGGL((accumulate_returned_kernel<T, 2>), grid, block, 0, stream, rule, gids, rows, n_rows, ptr, src, ret,
                           xt, ldx, gl);
    else
        hipLaunchKernelGGL((accumulate_returned_kernel<T, 1>), grid, block, 0, stream, rule, gids, rows, n_rows, ptr, src, ret,
                           xt, ldx, gl);
    return hipGetLastError();
}

}  // namespace

hipError_t varco_launch_compress(int dtype, const MaskRule& rule, const int32_t* gids, const int32_t* rows, int64_t n_rows,
                                 const void* x, int64_t ldx, void* z, hipStream_t stream, const LaunchTag& tag) {
    if (n_rows == 0) return hipSuccess;
    tag.begin(stream);
    const hipError_t e = dtype == VARCO_BF16 ? launch_compress_t<bf16_t>(rule, gids, rows, n_rows, x, ldx, z, stream)
                                             : launch_compress_t<float>(rule, gids, rows, n_rows, x, ldx, z, stream);
    tag.end(stream);
    return e;
}

hipError_t varco_launch_decompress(int dtype, const MaskRule& rule, const int32_t* gids, const int32_t* rows,
                                   int64_t n_rows, const void* z, void* x, int64_t ldx, int accumulate,
                                   hipStream_t stream, const LaunchTag& tag) {
    if (n_rows == 0) return hipSuccess;
    tag.begin(stream);
    const hipError_t e = dtype == VARCO_BF16
                             ? launch_decompress_t<bf16_t>(rule, gids, rows, n_rows, z, x, ldx, accumulate, stream)
                             : launch_decompress_t<float>(rule, gids, rows, n_rows, z, x, ldx, accumulate, stream);
    tag.end(stream);
    return e;
}

hipError_t varco_launch_accumulate_returned(int dtype, const MaskRule& rule, const int32_t* gids, const int32_t* rows,
                                            int64_t n_rows, const int32_t* ptr, const int32_t* src, const void* returned,
                                            void* x, int64_t ldx, hipStream_t stream, const LaunchTag& tag) {
    if (n_rows == 0) return hipSuccess;
    tag.begin(stream);
    const hipError_t e = dtype == VARCO_BF16
                             ? launch_accumulate_t<bf16_t>(rule, gids, rows, n_rows, ptr, src, returned, x, ldx, stream)
                             : launch_accumulate_t<float>(rule, gids, rows, n_rows, ptr, src, returned, x, ldx, stream);
    tag.end(stream);
    return e;
}

hipError_t varco_launch_halo_rows(const MaskRule& rule, const int32_t* gids, const int32_t* zrow, int32_t n, uint2* out,
                                  hipStream_t stream) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(halo_rows_kernel, dim3(unsigned((n + kBlock - 1) / kBlock)), dim3(kBlock), 0, stream, rule, gids, zrow,
                       n, out);
    return hipGetLastError();
}

hipError_t varco_launch_calibration_copy(void* dst, const void* src, int64_t bytes, hipStream_t stream) {
    if (bytes == 0) return hipSuccess;
    hipLaunchKernelGGL(calibration_copy_kernel, dim3(256 * 32), dim3(kBlock), 0, stream, static_cast<const float4*>(src),
                       static_cast<float4*>(dst), bytes / 16);
    return hipGetLastError();
}

hipError_t varco_launch_sum_gradients(float* dst, const float* src, int64_t n, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    const int64_t want = (n + kBlock - 1) / kBlock;
    hipLaunchKernelGGL(sum_gradients_kernel, dim3(unsigned(want < 256 * 16 ? want : 256 * 16)), dim3(kBlock), 0, stream, dst,
                       src, n);
    return hipGetLastError();
}

hipError_t varco_launch_step_table(uint64_t* d_step, uint32_t* table, uint64_t key, int set, uint64_t value,
                                   hipStream_t stream) {
    hipLaunchKernelGGL(step_table_kernel, dim3(1), dim3(kBlock), 0, stream, d_step, table, key, set, value);
    return hipGetLastError();
}
