// Graph-convolution aggregation M = S_q [X_loc ; X~_halo] (eq. (1)-(2) of the paper; Algorithm 1: local
// rows uncompressed, remote rows in compressed form) and its transpose for the backward pass.
//
// HBM-bound streaming kernels, one wavefront (64 lanes) per work item = a run of at most kSpmmChunk CSR
// entries of one row; rows longer than that are split and their partial sums reduced in a second pass,
// so the power-law hubs do not serialise on one wavefront and no floating-point atomics reach memory.
//
//   dense source rows (local rows; halo rows when k == width): a power-of-two group of lanes covers one
//     row with 16-byte loads, the groups of a wavefront take different edges and are summed at the end
//     with cross-lane shuffles (wavefront-level segmented reduction);
//   compressed halo rows (k < width): never decompressed to memory. The k stored elements of several
//     edges are loaded side by side (lane = (edge, j)), their positions pi_v(j) are recomputed from the
//     key, and they are accumulated into a per-wavefront row in LDS.
#include "mask_device.h"

namespace {

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / 64;

template <int VEC>
struct Vec;
template <>
struct Vec<4> {
    using type = float4;
};
template <>
struct Vec<1> {
    using type = float;
};

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
__device__ __forceinline__ float4 shfl_xor_vec(const float4& v, int mask) {
    return make_float4(__shfl_xor(v.x, mask), __shfl_xor(v.y, mask), __shfl_xor(v.z, mask), __shfl_xor(v.w, mask));
}
__device__ __forceinline__ float shfl_xor_vec(const float& v, int mask) { return __shfl_xor(v, mask); }
__device__ __forceinline__ void zero_vec(float4& v) { v = make_float4(0.f, 0.f, 0.f, 0.f); }
__device__ __forceinline__ void zero_vec(float& v) { v = 0.f; }

struct SpmmArgs {
    const SpmmItem* items;
    int32_t n_items;
    const int32_t* colidx;
    const float* vals;
    int32_t n_dense_cols;
    const float* dense;
    const HaloDesc* desc;
    const float* z;
    MaskRule rule;
    float* out;
    int32_t row_base;
    float* partial;
    int32_t lpr_log2;   // lanes per dense row = 1 << lpr_log2
    uint32_t k_magic;   // floor(2^32 / k) + 1 for k > 1
};

// VEC: floats per lane per load of a dense row (4 needs width % 4 == 0 and 16-byte aligned bases);
// NV: such loads per lane per row, so that width <= VEC * NV * lanes-per-row.
template <int VEC, int NV>
__global__ __launch_bounds__(kBlock) void spmm_kernel(SpmmArgs p) {
    using V = typename Vec<VEC>::type;
    extern __shared__ float lds[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int32_t width = int32_t(p.rule.width);
    const int32_t k = int32_t(p.rule.k);
    const bool full = k == width;
    float* lacc = lds + wave * width;   // this wavefront's row of sparse contributions

    const int32_t idx = blockIdx.x * kWaves + wave;
    if (idx >= p.n_items) return;       // no block-wide barrier below: wavefronts are independent
    const SpmmItem it = p.items[idx];

    for (int c = lane; c < width; c += 64) lacc[c] = 0.f;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");

    const int lpr = 1 << p.lpr_log2;
    const int t = lane & (lpr - 1);     // position inside the group
    const int g = lane >> p.lpr_log2;   // group index: which edge of a step this lane works on
    const int ng = 64 >> p.lpr_log2;

    V acc[NV];
#pragma unroll
    for (int m = 0; m < NV; ++m) zero_vec(acc[m]);
    bool any_sparse = false;

    for (int32_t base = it.e0; base < it.e1; base += 64) {
        const int32_t e = base + lane;
        const bool valid = e < it.e1;
        const int32_t c = valid ? p.colidx[e] : 0;
        const float w = valid ? p.vals[e] : 0.f;
        const bool is_halo = valid && c >= p.n_dense_cols;
        int32_t srow = c;
        uint32_t ma = 0, mb = 0;
        if (is_halo) {
            const HaloDesc d = p.desc[c - p.n_dense_cols];
            srow = d.zrow;
            if (!full) {
                const MaskAffine m = varco_affine(p.rule, uint32_t(d.gid));
                ma = m.a;
                mb = m.b;
            }
        }
        const uint64_t hmask = __ballot(is_halo);
        const int cnt = min(64, it.e1 - base);
        const int ns = full ? 0 : __popcll(hmask);
        const int nd = cnt - ns;        // columns ascend within a row, so dense edges sit in lanes [0, nd)

        // dense rows: group g takes edges g, g + ng, ...
        for (int i0 = 0; i0 < nd; i0 += ng) {
            const int i = i0 + g;
            const int src_lane = i < nd ? i : 0;
            const int32_t r = __shfl(srow, src_lane);
            const float wi = __shfl(w, src_lane);
            if (i < nd) {
                const bool h = (hmask >> i) & 1;
                const float* src = (h ? p.z : p.dense) + int64_t(r) * width;
#pragma unroll
                for (int m = 0; m < NV; ++m) {
                    const int col = VEC * (t + lpr * m);
                    if (col < width) {
                        const V v = *reinterpret_cast<const V*>(src + col);
                        fma_vec(acc[m], wi, v);
                    }
                }
            }
        }

        // compressed rows: lane = (edge, j), 64 stored elements per step whatever k is
        if (ns > 0) {
            any_sparse = true;
            const int total = ns * k;
            for (int t0 = 0; t0 < total; t0 += 64) {
                const int tt = t0 + lane;
                const bool act = tt < total;
                const int es = k == 1 ? tt : int(__umulhi(uint32_t(tt), p.k_magic));
                const int j = tt - es * k;
                const int src_lane = act ? nd + es : 0;
                const int32_t r = __shfl(srow, src_lane);
                const float wi = __shfl(w, src_lane);
                const uint32_t a = __shfl(ma, src_lane);
                const uint32_t b = __shfl(mb, src_lane);
                if (act) {
                    const float v = p.z[int64_t(r) * k + j];
                    const uint32_t pos = varco_mod_width(a * uint32_t(j) + b, p.rule.width, p.rule.width_magic);
                    __hip_atomic_fetch_add(&lacc[pos], wi * v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
                }
            }
        }
    }

    // sum the groups' partial rows
    for (int off = lpr; off < 64; off <<= 1) {
#pragma unroll
        for (int m = 0; m < NV; ++m) add_vec(acc[m], shfl_xor_vec(acc[m], off));
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    if (g == 0) {
        float* dst = it.dst < 0 ? p.out + int64_t(it.row - p.row_base) * width : p.partial + int64_t(it.dst) * width;
#pragma unroll
        for (int m = 0; m < NV; ++m) {
            const int col = VEC * (t + lpr * m);
            if (col < width) {
                V v = acc[m];
                if (any_sparse) add_vec(v, *reinterpret_cast<const V*>(lacc + col));
                *reinterpret_cast<V*>(dst + col) = v;
            }
        }
    }
}

// out[row] = sum of the partial rows of a split row, in slot order (fixed order: reproducible bits).
__global__ __launch_bounds__(kBlock) void spmm_fixup_kernel(const SpmmSplit* splits, int32_t n_splits,
                                                            const float* partial, float* out, int32_t row_base,
                                                            int32_t width) {
    const int32_t s = blockIdx.x;
    if (s >= n_splits) return;
    const SpmmSplit sp = splits[s];
    for (int c = threadIdx.x; c < width; c += kBlock) {
        float acc = 0.f;
        for (int i = 0; i < sp.count; ++i) acc += partial[int64_t(sp.first + i) * width + c];
        out[int64_t(sp.row - row_base) * width + c] = acc;
    }
}

struct KeptArgs {
    const SpmmItem* items;
    int32_t n_items;
    const int32_t* colidx;
    const float* vals;
    const float* src;
    const int32_t* gids;
    MaskRule rule;
    float* out;
    int32_t row_base;
    float* partial;
    int32_t g_log2;   // lanes per edge = 1 << g_log2 >= min(k, 64)
};

// Transposed aggregation for halo rows, produced directly in compressed form: only the k kept columns
// of each gathered row of `src` are read. Lane = (edge sub-group, j).
__global__ __launch_bounds__(kBlock) void spmm_kept_kernel(KeptArgs p) {
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int32_t idx = blockIdx.x * kWaves + wave;
    if (idx >= p.n_items) return;
    const SpmmItem it = p.items[idx];
    const int32_t width = int32_t(p.rule.width);
    const int32_t k = int32_t(p.rule.k);
    const int gsz = 1 << p.g_log2;
    const int jl = lane & (gsz - 1);
    const int sg = lane >> p.g_log2;
    const int nsg = 64 >> p.g_log2;
    const MaskAffine m = varco_affine(p.rule, uint32_t(p.gids[it.row - p.row_base]));
    float* dst = it.dst < 0 ? p.out + int64_t(it.row - p.row_base) * k : p.partial + int64_t(it.dst) * k;

    for (int jbase = 0; jbase < k; jbase += gsz) {
        const int j = jbase + jl;
        const bool jact = j < k;
        const uint32_t pos = jact ? varco_position(p.rule, m, uint32_t(j)) : 0u;
        float acc = 0.f;
        for (int32_t base = it.e0; base < it.e1; base += 64) {
            const int32_t e = base + lane;
            const bool valid = e < it.e1;
            const int32_t c = valid ? p.colidx[e] : 0;
            const float w = valid ? p.vals[e] : 0.f;
            const int cnt = min(64, it.e1 - base);
            for (int i0 = 0; i0 < cnt; i0 += nsg) {
                const int i = i0 + sg;
                const int src_lane = i < cnt ? i : 0;
                const int32_t r = __shfl(c, src_lane);
                const float wi = __shfl(w, src_lane);
                if (i < cnt && jact) acc += wi * p.src[int64_t(r) * width + pos];
            }
        }
        for (int off = gsz; off < 64; off <<= 1) acc += __shfl_xor(acc, off);
        if (sg == 0 && jact) dst[j] = acc;
    }
}

template <int VEC>
hipError_t launch_spmm_vec(int nv, const SpmmArgs& a, dim3 grid, size_t lds_bytes, hipStream_t stream) {
    switch (nv) {
        case 1: hipLaunchKernelGGL((spmm_kernel<VEC, 1>), grid, dim3(kBlock), lds_bytes, stream, a); break;
        case 2: hipLaunchKernelGGL((spmm_kernel<VEC, 2>), grid, dim3(kBlock), lds_bytes, stream, a); break;
        case 4: hipLaunchKernelGGL((spmm_kernel<VEC, 4>), grid, dim3(kBlock), lds_bytes, stream, a); break;
        case 8: hipLaunchKernelGGL((spmm_kernel<VEC, 8>), grid, dim3(kBlock), lds_bytes, stream, a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

hipError_t varco_launch_spmm(const SpmmPlan& plan, const int32_t* colidx, const float* vals, int32_t n_dense_cols,
                             const float* dense, const HaloDesc* desc, const float* z, const MaskRule& rule,
                             float* out, int32_t row_base, float* partial, hipStream_t stream, const LaunchTag& tag) {
    if (plan.n_items == 0) return hipSuccess;
    const int32_t width = int32_t(rule.width);
    const bool full = rule.k == rule.width;
    const bool vec4 = width % 4 == 0 && aligned16(dense) && aligned16(out) && aligned16(partial) &&
                      (!full || aligned16(z));
    const int vec = vec4 ? 4 : 1;
    const int per_row = (width + vec - 1) / vec;   // loads of VEC floats that cover a row
    int lpr_log2 = 0;
    while ((1 << lpr_log2) < per_row && lpr_log2 < 6) ++lpr_log2;
    int nv = 1;
    while (nv * (1 << lpr_log2) < per_row) nv <<= 1;
    if (nv > 8) return hipErrorInvalidValue;

    SpmmArgs a;
    a.items = plan.items;
    a.n_items = plan.n_items;
    a.colidx = colidx;
    a.vals = vals;
    a.n_dense_cols = n_dense_cols;
    a.dense = dense;
    a.desc = desc;
    a.z = z;
    a.rule = rule;
    a.out = out;
    a.row_base = row_base;
    a.partial = partial;
    a.lpr_log2 = lpr_log2;
    a.k_magic = rule.k > 1 ? uint32_t((uint64_t(1) << 32) / rule.k) + 1u : 0u;
    const dim3 grid((plan.n_items + kWaves - 1) / kWaves);
    const size_t lds_bytes = size_t(kWaves) * width * sizeof(float);
    tag.begin(stream);
    hipError_t err = vec4 ? launch_spmm_vec<4>(nv, a, grid, lds_bytes, stream)
                          : launch_spmm_vec<1>(nv, a, grid, lds_bytes, stream);
    tag.end(stream);
    if (err != hipSuccess) return err;
    if (plan.n_splits > 0) {
        tag.begin_as(VARCO_K_REDUCE, stream);
        hipLaunchKernelGGL(spmm_fixup_kernel, dim3(plan.n_splits), dim3(kBlock), 0, stream, plan.splits, plan.n_splits,
                           partial, out, row_base, width);
        tag.end(stream);
        err = hipGetLastError();
    }
    return err;
}

hipError_t varco_launch_spmm_kept(const SpmmPlan& plan, const int32_t* colidx, const float* vals, const float* src,
                                  const int32_t* gids, const MaskRule& rule, float* out, int32_t row_base,
                                  float* partial, hipStream_t stream, const LaunchTag& tag) {
    if (plan.n_items == 0) return hipSuccess;
    KeptArgs a;
    a.items = plan.items;
    a.n_items = plan.n_items;
    a.colidx = colidx;
    a.vals = vals;
    a.src = src;
    a.gids = gids;
    a.rule = rule;
    a.out = out;
    a.row_base = row_base;
    a.partial = partial;
    int g_log2 = 0;
    while ((1u << g_log2) < rule.k && g_log2 < 6) ++g_log2;
    a.g_log2 = g_log2;
    const dim3 grid((plan.n_items + kWaves - 1) / kWaves);
    tag.begin(stream);
    hipLaunchKernelGGL(spmm_kept_kernel, grid, dim3(kBlock), 0, stream, a);
    tag.end(stream);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    if (plan.n_splits > 0) {
        tag.begin_as(VARCO_K_REDUCE, stream);
        hipLaunchKernelGGL(spmm_fixup_kernel, dim3(plan.n_splits), dim3(kBlock), 0, stream, plan.splits, plan.n_splits,
                           partial, out, row_base, int32_t(rule.k));
        tag.end(stream);
        err = hipGetLastError();
    }
    return err;
}
