// What a quantization did to the vectors it was given, per worker: the number of nonzero coordinates of
// Q(v) (Lemma 2: (1 - p_0) d in expectation), the realised squared error ||Q(v) - v||^2 (eq. (var) in
// expectation, at most epsilon_Q ||v||^2 by Theorem 1) and ||v||^2.  A diagnostic beside the hot path: it
// reads the vectors and their decoded images once; sums in binary64 in a fixed order.
#include "qgx_device.h"

namespace qgx {

__global__ __launch_bounds__(256) void k_metrics_partial(const float* __restrict__ V, const float* __restrict__ Vhat,
                                                         uint64_t d, double* __restrict__ partial)
{
    __shared__ double s_red[3][256];
    const uint32_t k = blockIdx.y;
    const float* __restrict__ v = V + (size_t)k * d;
    const float* __restrict__ q = Vhat + (size_t)k * d;
    const uint64_t per = (d + kMetricBlocks - 1) / kMetricBlocks;
    const uint64_t lo = (uint64_t)blockIdx.x * per, hi = lo + per < d ? lo + per : d;
    double nnz = 0.0, err = 0.0, nrm = 0.0;
    for (uint64_t i = lo + threadIdx.x; i < hi; i += 256u) {
        const double x = (double)v[i], y = (double)q[i];
        nnz += y != 0.0 ? 1.0 : 0.0;          // counts below 2^53 are exact in binary64
        err = fma(y - x, y - x, err);
        nrm = fma(x, x, nrm);
    }
    s_red[0][threadIdx.x] = nnz; s_red[1][threadIdx.x] = err; s_red[2][threadIdx.x] = nrm;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off)
            for (int m = 0; m < 3; ++m) s_red[m][threadIdx.x] += s_red[m][threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x < 3) partial[((size_t)k * 3 + threadIdx.x) * kMetricBlocks + blockIdx.x] = s_red[threadIdx.x][0];
}

// result[k][m], m = 0 nonzeros, 1 squared error, 2 squared norm
__global__ __launch_bounds__(256) void k_metrics_finish(const double* __restrict__ partial, double* __restrict__ result)
{
    __shared__ double s_red[256];
    const double* p = partial + (size_t)blockIdx.x * kMetricBlocks;
    double acc = 0.0;
    for (uint32_t i = threadIdx.x; i < kMetricBlocks; i += 256u) acc += p[i];
    s_red[threadIdx.x] = acc;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) s_red[threadIdx.x] += s_red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) result[blockIdx.x] = s_red[0];
}

hipError_t launch_metrics(const float* V, const float* Vhat, uint64_t d, uint32_t K, double* partial, double* result,
                          hipStream_t st)
{
    hipLaunchKernelGGL(k_metrics_partial, dim3(kMetricBlocks, K), dim3(256), 0, st, V, Vhat, d, partial);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_metrics_finish, dim3(K * 3u), dim3(256), 0, st, partial, result);
    return hipGetLastError();
}

}  // namespace qgx
