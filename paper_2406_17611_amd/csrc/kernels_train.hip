// The rest of Algorithm 1's iteration around the layer calls: the cross-entropy loss of Section II on a
// partition's labelled rows with its gradient with respect to the logits, fixed-order sums of the per-row
// results, and the gradient step (SGD). Memory-bound elementwise / row-wise kernels.
#include "elem.h"
#include "varco_internal.h"

namespace {

constexpr int kBlock = 256;
constexpr int kWaves = kBlock / 64;

__device__ __forceinline__ float wave_max(float v) {
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

// One wavefront per row: loss_i = logsumexp(z_i) - z_i[y_i], dz_i = scale * (softmax(z_i) - onehot(y_i)),
// correct_i = [argmax z_i == y_i] (lowest index on ties); rows whose y_i is not a class (negative: not a training
// node; n_classes or above: never read as an index) give 0 everywhere.
template <typename T>
__global__ __launch_bounds__(kBlock) void softmax_xent_kernel(const T* __restrict__ logits, int64_t ld,
                                                              const int32_t* __restrict__ labels, int64_t n_rows,
                                                              int32_t n_classes, float scale, T* __restrict__ dlogits,
                                                              int64_t ldd, float* __restrict__ row_loss,
                                                              int32_t* __restrict__ row_correct) {
    const int lane = threadIdx.x & 63;
    const int64_t row = int64_t(blockIdx.x) * kWaves + (threadIdx.x >> 6);
    if (row >= n_rows) return;
    const int32_t y = labels[row];
    const T* z = logits + row * ld;
    float vmax = -INFINITY;
    int32_t imax = 0x7FFFFFFF;
    for (int c = lane; c < n_classes; c += 64) {
        const float v = Elem<T>::load(z + c);
        if (v > vmax) vmax = v, imax = c;      // ascending c within a lane: the first maximum is kept
    }
    const float gmax = wave_max(vmax);
    int32_t cand = vmax == gmax ? imax : 0x7FFFFFFF;
    for (int off = 32; off > 0; off >>= 1) cand = min(cand, __shfl_xor(cand, off));
    float se = 0.f;
    for (int c = lane; c < n_classes; c += 64) se += expf(Elem<T>::load(z + c) - gmax);
    se = wave_sum(se);
    const bool on = y >= 0 && y < n_classes;
    if (dlogits) {
        T* d = dlogits + row * ldd;
        const float inv = scale / se;
        for (int c = lane; c < n_classes; c += 64) {
            float g = 0.f;
            if (on) g = expf(Elem<T>::load(z + c) - gmax) * inv - (c == y ? scale : 0.f);
            Elem<T>::store(d + c, g);
        }
    }
    if (lane == 0) {
        row_loss[row] = on ? gmax + logf(se) - Elem<T>::load(z + y) : 0.f;
        row_correct[row] = on && cand == y ? 1 : 0;
    }
}

// totals[0] += scale * sum(row_loss), totals[1] += count of correct rows; one workgroup, fixed order.
__global__ __launch_bounds__(1024) void sum_rows_kernel(const float* __restrict__ row_loss,
                                                        const int32_t* __restrict__ row_correct, int64_t n, float scale,
                                                        float* __restrict__ totals) {
    __shared__ float sl[1024];
    __shared__ float sc[1024];
    float l = 0.f, c = 0.f;
    for (int64_t i = threadIdx.x; i < n; i += 1024) l += row_loss[i], c += float(row_correct[i]);
    sl[threadIdx.x] = l, sc[threadIdx.x] = c;
    __syncthreads();
    for (int s = 512; s > 0; s >>= 1) {
        if (int(threadIdx.x) < s) sl[threadIdx.x] += sl[threadIdx.x + s], sc[threadIdx.x] += sc[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) totals[0] += scale * sl[0], totals[1] += sc[0];
}

__global__ __launch_bounds__(kBlock) void sgd_kernel(float* __restrict__ w, const float* __restrict__ dw, int64_t n,
                                                     float lr) {
    const int64_t stride = int64_t(gridDim.x) * kBlock;
    for (int64_t i = int64_t(blockIdx.x) * kBlock + threadIdx.x; i < n; i += stride) w[i] -= lr * dw[i];
}

}  // namespace

hipError_t varco_launch_softmax_xent(int dtype, const void* logits, int64_t ld, const int32_t* labels, int64_t n_rows,
                                     int32_t n_classes, float scale, void* dlogits, int64_t ldd, float* row_loss,
                                     int32_t* row_correct, float* totals, hipStream_t stream) {
    if (n_rows == 0) return hipSuccess;
    const dim3 grid(unsigned((n_rows + kWaves - 1) / kWaves));
    if (dtype == VARCO_BF16)
        hipLaunchKernelGGL(softmax_xent_kernel<bf16_t>, grid, dim3(kBlock), 0, stream, static_cast<const bf16_t*>(logits), ld,
                           labels, n_rows, n_classes, scale, static_cast<bf16_t*>(dlogits), ldd, row_loss, row_correct);
    else
        hipLaunchKernelGGL(softmax_xent_kernel<float>, grid, dim3(kBlock), 0, stream, static_cast<const float*>(logits), ld,
                           labels, n_rows, n_classes, scale, static_cast<float*>(dlogits), ldd, row_loss, row_correct);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || !totals) return e;
    hipLaunchKernelGGL(sum_rows_kernel, dim3(1), dim3(1024), 0, stream, row_loss, row_correct, n_rows, scale, totals);
    return hipGetLastError();
}

hipError_t varco_launch_sgd(float* w, const float* dw, int64_t n, float lr, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    const int64_t want = (n + kBlock - 1) / kBlock;
    hipLaunchKernelGGL(sgd_kernel, dim3(unsigned(want < 256 * 16 ? want : 256 * 16)), dim3(kBlock), 0, stream, w, dw, n, lr);
    return hipGetLastError();
}
