// The caller's side of an iteration, for the large quadratic game, as kernels of the library so that an
// iteration can stay on the device (Section 2: stochastic oracle g(z; omega) = A(z) + U(z; omega); the
// residual ||A(x)|| that the convergence theorems are read against): the operator F(z) = M z + b, the K
// workers' dual vectors F(z) + sigma N with reproducible noise, and a 2-norm.  The coding kernel has a
// mode of its own that forms the same dual vectors on the fly instead of reading them (qgx_encode.hip).
#include "qgx_device.h"

namespace qgx {

__global__ __launch_bounds__(256) void k_game_operator(GameArgs G, uint32_t d, float* __restrict__ F)
{
    for (uint32_t i0 = (blockIdx.x * 256u + threadIdx.x) * 4u; i0 < d; i0 += gridDim.x * 1024u)
        *reinterpret_cast<float4*>(F + i0) = game_operator_row(G, i0);
}

hipError_t launch_game_operator(const GameArgs& g, uint32_t d, float* F_out, hipStream_t st)
{
    const uint32_t grid = min((d / 4u + 255u) / 256u, 8192u);
    hipLaunchKernelGGL(k_game_operator, dim3(grid), dim3(256), 0, st, g, d, F_out);
    return hipGetLastError();
}

// The worker is the fast index of the grid, so that the K blocks that need the same piece of z, a and b run
// together and share it through the cache (the pieces would otherwise be streamed from memory K times).  The
// call number may come from the iteration counter on the device, as in the coding kernel, so that a replayed
// graph draws fresh noise.
__global__ __launch_bounds__(256) void k_game_dual_vectors(GameArgs G, uint32_t d, uint32_t K, uint32_t call_id,
                                                           uint32_t call_mode, const Scalars* sc, float* __restrict__ V)
{
    const uint32_t k = blockIdx.x % K, piece = blockIdx.x / K, pieces = gridDim.x / K;
    const uint32_t call = call_mode ? 2u * (uint32_t)(sc->t - 1ull) + (call_mode - 1u) : call_id;
    float* __restrict__ Vk = V + (size_t)k * d;
    for (uint32_t i0 = (piece * 256u + threadIdx.x) * 4u; i0 < d; i0 += pieces * 1024u)
        *reinterpret_cast<float4*>(Vk + i0) = game_dual_row(G, i0, k, call);
}

hipError_t launch_game_dual_vectors(const GameArgs& g, uint32_t d, uint32_t K, uint32_t call_id, uint32_t call_mode,
                                    const Scalars* sc, float* V_out, hipStream_t st)
{
    const uint32_t pieces = min((d / 4u + 255u) / 256u, 16384u);
    hipLaunchKernelGGL(k_game_dual_vectors, dim3(pieces * K), dim3(256), 0, st, g, d, K, call_id, call_mode, sc, V_out);
    return hipGetLastError();
}

// ||x||_2: squares summed in binary64, every block a fixed run of the vector, the blocks' sums added in
// block order, so that the result repeats bit for bit.  partial[kNormBlocks] receives the norm.
__global__ __launch_bounds__(256) void k_norm2_partial(const float* __restrict__ x, uint64_t n, double* __restrict__ partial)
{
    __shared__ double s_red[256];
    const uint64_t per = (n + kNormBlocks - 1) / kNormBlocks;
    const uint64_t lo = (uint64_t)blockIdx.x * per, hi = lo + per < n ? lo + per : n;
    double acc = 0.0;
    for (uint64_t i = lo + threadIdx.x; i < hi; i += 256u) acc = fma((double)x[i], (double)x[i], acc);
    s_red[threadIdx.x] = acc;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) s_red[threadIdx.x] += s_red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[blockIdx.x] = s_red[0];
}

__global__ __launch_bounds__(256) void k_norm2_finish(double* __restrict__ partial)
{
    __shared__ double s_red[256];
    double acc = 0.0;
    for (uint32_t i = threadIdx.x; i < kNormBlocks; i += 256u) acc += partial[i];
    s_red[threadIdx.x] = acc;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) s_red[threadIdx.x] += s_red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[kNormBlocks] = sqrt(s_red[0]);
}

hipError_t launch_norm2(const float* x, uint64_t n, double* partial, hipStream_t st)
{
    hipLaunchKernelGGL(k_norm2_partial, dim3(kNormBlocks), dim3(256), 0, st, x, n, partial);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_norm2_finish, dim3(1), dim3(256), 0, st, partial);
    return hipGetLastError();
}

// Restricted gap (eq. (Gap), Section 2) of F over the closed ball of radius R around `centre` (NULL: the
// origin): sup_x <F(x), xhat - x>.  <M x, x> = mu ||x||^2 (the coupling is skew), so the objective is a concave
// quadratic of the same curvature in every direction and its maximiser over the ball is the point of the ball
// nearest to the free maximiser x0 = (M^T xhat - b) / (2 mu).  Two passes over the blocks in binary64, each
// with the fixed-order sums of the norm above: the distance of x0 from the centre, then the objective at the
// maximiser.  G.z holds xhat.
__device__ __forceinline__ void gap_free_maximiser(const GameArgs& G, const float* __restrict__ centre, uint64_t j,
                                                   double& x0, double& x1, double& c0, double& c1)
{
    const double h0 = (double)G.z[j], h1 = (double)G.z[j + 1], a = (double)G.a[j >> 1], mu = (double)G.mu;
    x0 = (mu * h0 - a * h1 - (double)G.b[j]) / (2.0 * mu);
    x1 = (a * h0 + mu * h1 - (double)G.b[j + 1]) / (2.0 * mu);
    c0 = centre ? (double)centre[j] : 0.0;
    c1 = centre ? (double)centre[j + 1] : 0.0;
}

__device__ __forceinline__ void block_sum_to(double acc, double* __restrict__ out)
{
    __shared__ double s_red[256];
    s_red[threadIdx.x] = acc;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) s_red[threadIdx.x] += s_red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) *out = s_red[0];
}

// PASS 0: partial[block] = sum of ||x0 - c||^2 over the block's run of 2x2 blocks.
// PASS 1: with shrink = partial[kNormBlocks] (1 inside the ball, R / distance outside), the objective's sum.
template <int PASS>
__global__ __launch_bounds__(256) void k_gap_partial(GameArgs G, const float* __restrict__ centre, uint64_t d,
                                                     double* __restrict__ partial)
{
    const uint64_t pairs = d / 2, per = (pairs + kNormBlocks - 1) / kNormBlocks;
    const uint64_t lo = (uint64_t)blockIdx.x * per, hi = lo + per < pairs ? lo + per : pairs;
    const double shrink = PASS == 1 ? partial[kNormBlocks] : 1.0;
    double* out = partial + (PASS == 1 ? kNormBlocks + 1 : 0) + blockIdx.x;
    double acc = 0.0;
    for (uint64_t p = lo + threadIdx.x; p < hi; p += 256u) {
        double x0, x1, c0, c1;
        gap_free_maximiser(G, centre, 2 * p, x0, x1, c0, c1);
        if (PASS == 0) {
            acc += (x0 - c0) * (x0 - c0) + (x1 - c1) * (x1 - c1);
        } else {
            x0 = c0 + shrink * (x0 - c0);
            x1 = c1 + shrink * (x1 - c1);
            const double a = (double)G.a[p], mu = (double)G.mu;
            const double F0 = mu * x0 + a * x1 + (double)G.b[2 * p], F1 = -a * x0 + mu * x1 + (double)G.b[2 * p + 1];
            acc += F0 * ((double)G.z[2 * p] - x0) + F1 * ((double)G.z[2 * p + 1] - x1);
        }
    }
    block_sum_to(acc, out);
}

// PASS 0: partial[kNormBlocks] = the factor that brings x0 into the ball; PASS 1: partial[2 kNormBlocks + 1] = the gap.
template <int PASS>
__global__ __launch_bounds__(256) void k_gap_finish(double* __restrict__ partial, double R)
{
    const double* in = partial + (PASS == 1 ? kNormBlocks + 1 : 0);
    double acc = 0.0;
    for (uint32_t i = threadIdx.x; i < kNormBlocks; i += 256u) acc += in[i];
    __shared__ double s_total;
    block_sum_to(acc, &s_total);
    __syncthreads();
    if (threadIdx.x == 0) {
        if (PASS == 0) {
            const double dist = sqrt(s_total);
            partial[kNormBlocks] = dist > R ? R / dist : 1.0;
        } else {
            partial[2 * kNormBlocks + 1] = s_total;
        }
    }
}

hipError_t launch_game_gap(const GameArgs& g, const float* centre, double R, uint64_t d, double* partial, hipStream_t st)
{
    hipLaunchKernelGGL(k_gap_partial<0>, dim3(kNormBlocks), dim3(256), 0, st, g, centre, d, partial);
    hipLaunchKernelGGL(k_gap_finish<0>, dim3(1), dim3(256), 0, st, partial, R);
    hipLaunchKernelGGL(k_gap_partial<1>, dim3(kNormBlocks), dim3(256), 0, st, g, centre, d, partial);
    hipLaunchKernelGGL(k_gap_finish<1>, dim3(1), dim3(256), 0, st, partial, R);
    return hipGetLastError();
}

}  // namespace qgx
