// Adaptive levels (Section 3.3): the weighted empirical CDF of eq. (QAda) as a histogram of the
// normalised coordinates, and the one-level-at-a-time solver on it.
//
// Histogram: persistent workgroups walk the (worker, bucket) pairs with a fixed stride; per bucket the
// data is read once into registers (same row layout as the encoder), the norm is reduced, every
// coordinate bumps an integer LDS counter of its bin, and the counters are folded into per-workgroup
// binary64 sums weighted by the squared norm.  Workgroup sums go to scratch and are added in a fixed
// order, so the histogram is reproducible bit for bit.
//
// Bins follow the binary32 grid: 64 equal-width bins per octave over n_bins/64 octaves below 1 (bin 0
// also takes everything smaller, u = 1 goes to the last bin), so the bin of u is an integer function
// of its bits and the resolution follows the heavy concentration of u near zero.
#include "qgx_device.h"

namespace qgx {

__device__ __forceinline__ uint32_t bin_of(float u, uint32_t n_bins)
{
    const int key = (int)(__float_as_uint(u) >> 17) - (127 * 64 - (int)n_bins);
    return (uint32_t)min(max(key, 0), (int)n_bins - 1);
}

__device__ __forceinline__ double bin_edge(uint32_t b, uint32_t n_bins)
{
    if (b == 0) return 0.0;
    if (b >= n_bins) return 1.0;
    return (double)__uint_as_float((uint32_t)((int)b + (127 * 64 - (int)n_bins)) << 17);
}

// A workgroup walks its buckets one after the other, each in three phases divided by barriers (norm, count,
// fold), and a compute unit holds only two or three such workgroups (LDS): nothing hides a phase's
// latency but the next bucket's rows, so with buckets of at most four chunks those are loaded into a
// second set of registers before the current bucket is worked on.
template <int MAXW>
__global__ __launch_bounds__(MAXW * kWave) void k_histogram(Layout lay, const float* __restrict__ V, int norm_kind,
                                                            uint32_t n_bins, double* __restrict__ partial, Scalars* sc)
{
    constexpr bool kAhead = MAXW <= 4;                                   // registers for a second bucket's rows
    extern __shared__ __align__(16) unsigned char s_raw[];
    double* s_acc = reinterpret_cast<double*>(s_raw);                    // [n_bins]
    uint32_t* s_cnt = reinterpret_cast<uint32_t*>(s_acc + n_bins);       // [n_bins]
    __shared__ double s_red[kMaxWaves];
    __shared__ uint32_t s_bad[kMaxWaves];

    const int tid = (int)threadIdx.x, lane = lane_id(), w = wave_id();
    const int nwaves = (int)(blockDim.x >> 6);
    for (uint32_t i = (uint32_t)tid; i < n_bins; i += blockDim.x) { s_acc[i] = 0.0; s_cnt[i] = 0; }
    __syncthreads();

    const uint32_t n_work = lay.K * lay.NB;
    // the rows of this wave's chunk of unit t (bucket t / K of worker t % K), zeros past the bucket's end
    auto load_rows = [&](uint32_t t, float4 (&v)[kRows]) {
        const uint32_t b = t / lay.K, k = t - b * lay.K;
        const uint32_t lo = lay.bucket_start[b], hi = lay.bucket_start[b + 1];
        const uint32_t clo = lo + (uint32_t)w * kChunk;
        const uint32_t cend = clo < hi ? clo + min((uint32_t)kChunk, hi - clo) : clo;
        const size_t kbase = (size_t)k * lay.d;
        const bool vec_ok = (kbase & 3u) == 0;
        const float* __restrict__ Vk = V + kbase;
#pragma unroll
        for (int r = 0; r < kRows; ++r) {
            const uint32_t i0 = clo + (uint32_t)r * 256u + (uint32_t)lane * 4u;
            float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
            if (i0 + 4u <= cend) {
                if (vec_ok) x = nt_load4(Vk + i0);                // (read once)
                else x = make_float4(Vk[i0], Vk[i0 + 1], Vk[i0 + 2], Vk[i0 + 3]);
            } else if (i0 < cend) {
                x.x = Vk[i0];
                if (i0 + 1 < cend) x.y = Vk[i0 + 1];
                if (i0 + 2 < cend) x.z = Vk[i0 + 2];
            }
            v[r] = x;
        }
    };
    float4 v[kRows], v_next[kAhead ? kRows : 1];
    if constexpr (kAhead) {
        if (blockIdx.x < n_work) load_rows(blockIdx.x, v);
    }
    for (uint32_t t = blockIdx.x; t < n_work; t += gridDim.x) {
        const uint32_t b = t / lay.K, k = t - b * lay.K;
        const uint32_t lo = lay.bucket_start[b], hi = lay.bucket_start[b + 1];
        const uint32_t clo = lo + (uint32_t)w * kChunk;
        const uint32_t clen = clo < hi ? min((uint32_t)kChunk, hi - clo) : 0u;
        const uint32_t cend = clo + clen;
        const size_t kbase = (size_t)k * lay.d;
        const float* __restrict__ Vk = V + kbase;
        if constexpr (kAhead) {
            if (t + gridDim.x < n_work) load_rows(t + gridDim.x, v_next);
        } else {
            load_rows(t, v);
        }
        double acc = 0.0;
        float mx = 0.0f;
        uint32_t bad = 0;
#pragma unroll
        for (int r = 0; r < kRows; ++r) {
            const float e[4] = {v[r].x, v[r].y, v[r].z, v[r].w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float ax = fabsf(e[q]);
                bad |= !(ax <= 3.402823466e+38f);
                if (norm_kind == QGX_NORM_L2) acc = fma((double)e[q], (double)e[q], acc);
                else mx = fmaxf(mx, ax);
            }
        }
        if (norm_kind == QGX_NORM_L2) acc = wave_sum(acc);
        else acc = (double)wave_max(mx);
        bad = wave_or(bad);
        if (lane == 0) { s_red[w] = acc; s_bad[w] = bad; }
        __syncthreads();
        double tot = 0.0;
        uint32_t anybad = 0;
        for (int i = 0; i < nwaves; ++i) {
            if (norm_kind == QGX_NORM_L2) tot += s_red[i];
            else tot = fmax(tot, s_red[i]);
            anybad |= s_bad[i];
        }
        float n = (norm_kind == QGX_NORM_L2) ? (float)sqrt(tot) : (float)tot;
        if (norm_kind != QGX_NORM_L2 && norm_kind != QGX_NORM_LINF && anybad == 0 && tot > 0.0) {
            // general q: (sum |v_i|^q)^(1/q) relative to the largest magnitude, as in the encoder
            const double inv_m = 1.0 / tot;
            double sum = 0.0;
#pragma unroll 1
            for (uint32_t i = clo + (uint32_t)lane; i < cend; i += kWave) {      // rolled, from memory
                sum += pow_int(fabs((double)Vk[i]) * inv_m, (uint32_t)norm_kind);
            }
            sum = wave_sum(sum);
            __syncthreads();                         // everyone has read the first set of partial results
            if (lane == 0) s_red[w] = sum;
            __syncthreads();
            double all = 0.0;
            for (int i = 0; i < nwaves; ++i) all += s_red[i];
            n = (float)(tot * root_int(all, (uint32_t)norm_kind));
        }
        const bool usable = (anybad == 0) && (n > 0.0f) && (n <= 3.402823466e+38f);
        if (anybad != 0 && tid == 0) raise_error(sc, QGX_EBIT_NONFINITE);
        if (usable) {
            const float rinv = 1.0f / n;
            if (clen == (uint32_t)kChunk) {
                // a whole chunk: no coordinate to leave out, and u above 1 (by a rounding) ends in the last bin
                // with the clamp of the bin number alone
#pragma unroll
                for (int r = 0; r < kRows; ++r) {
                    const float e[4] = {v[r].x, v[r].y, v[r].z, v[r].w};
#pragma unroll
                    for (int q = 0; q < 4; ++q) atomicAdd(&s_cnt[bin_of(fabsf(e[q]) * rinv, n_bins)], 1u);
                }
            } else {
#pragma unroll
                for (int r = 0; r < kRows; ++r) {
                    const uint32_t i0 = clo + (uint32_t)r * 256u + (uint32_t)lane * 4u;
                    const float e[4] = {v[r].x, v[r].y, v[r].z, v[r].w};
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        if (i0 + (uint32_t)q < cend) {
                            const float u = fminf(fabsf(e[q]) * rinv, 1.0f);
                            atomicAdd(&s_cnt[bin_of(u, n_bins)], 1u);
                        }
                    }
                }
            }
        }
        __syncthreads();
        if (usable) {
            const double wgt = (double)n * (double)n;           // lambda of Section 3.3, unnormalised
            for (uint32_t i = (uint32_t)tid; i < n_bins; i += blockDim.x) {
                const uint32_t cnt = s_cnt[i];
                if (cnt) { s_acc[i] += (double)cnt * wgt; s_cnt[i] = 0; }
            }
        }
        __syncthreads();
        if constexpr (kAhead) {
#pragma unroll
            for (int r = 0; r < kRows; ++r) v[r] = v_next[r];
        }
    }
    for (uint32_t i = (uint32_t)tid; i < n_bins; i += blockDim.x)
        partial[(size_t)blockIdx.x * n_bins + i] = s_acc[i];
}

// Buckets of 256..2048 coordinates (one to eight rows of 256): a workgroup of one wave per bucket
// would leave the chip nearly empty and spend its time folding 4096 counters per bucket.  Here a
// workgroup is four waves with a bucket each.  A wave counts into 16-bit counters of its own (two to
// a word; a count is at most 2048), and the lane that takes a counter from zero remembers it: after
// the count exactly those lanes fold their counters into the workgroup's binary64 sums, weighted by
// the squared norm, and clear them, so a fold costs what the bucket touched, not the whole table.
// The waves fold one after the other, in wave order, so every sum still receives its terms in a
// fixed order and the histogram is reproducible bit for bit.
template <int RPB>
__global__ __launch_bounds__(256) void k_histogram_small(Layout lay, const float* __restrict__ V, int norm_kind,
                                                         uint32_t n_bins, double* __restrict__ partial, Scalars* sc)
{
    extern __shared__ __align__(16) unsigned char s_raw[];
    constexpr int kW = 4;
    const int tid = (int)threadIdx.x, lane = lane_id(), w = wave_id();
    double* s_acc = reinterpret_cast<double*>(s_raw);                                   // [n_bins]
    uint32_t* s_cnt = reinterpret_cast<uint32_t*>(s_acc + n_bins) + (size_t)w * (n_bins / 2);   // [n_bins / 2] per wave
    for (uint32_t i = (uint32_t)tid; i < n_bins; i += kW * kWave) s_acc[i] = 0.0;
    for (uint32_t i = (uint32_t)lane; i < n_bins / 2; i += kWave) s_cnt[i] = 0u;
    __syncthreads();

    const uint32_t n_work = lay.K * lay.NB;
    for (uint32_t t0 = (uint32_t)blockIdx.x * kW; t0 < n_work; t0 += gridDim.x * kW) {
        const uint32_t t = t0 + (uint32_t)w;
        const bool have = t < n_work;                     // wave-uniform
        const uint32_t b = have ? t / lay.K : 0u, k = have ? t - b * lay.K : 0u;
        const uint32_t lo = lay.bucket_start[b], hi = have ? lay.bucket_start[b + 1] : lo;
        const size_t kbase = (size_t)k * lay.d;
        const bool vec_ok = (kbase & 3u) == 0;
        const float* __restrict__ Vk = V + kbase;
        float4 v[RPB];
#pragma unroll
        for (int r = 0; r < RPB; ++r) {
            const uint32_t i0 = lo + (uint32_t)r * 256u + (uint32_t)lane * 4u;
            float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
            if (i0 + 4u <= hi) {
                if (vec_ok) x = nt_load4(Vk + i0);                // (read once)
                else x = make_float4(Vk[i0], Vk[i0 + 1], Vk[i0 + 2], Vk[i0 + 3]);
            } else if (i0 < hi) {
                x.x = Vk[i0];
                if (i0 + 1 < hi) x.y = Vk[i0 + 1];
                if (i0 + 2 < hi) x.z = Vk[i0 + 2];
            }
            v[r] = x;
        }
        // the norm, with the arithmetic of k_histogram for a bucket of one wave
        double acc = 0.0;
        float mx = 0.0f;
        uint32_t bad = 0;
#pragma unroll
        for (int r = 0; r < RPB; ++r) {
            const float e[4] = {v[r].x, v[r].y, v[r].z, v[r].w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float ax = fabsf(e[q]);
                bad |= !(ax <= 3.402823466e+38f);
                if (norm_kind == QGX_NORM_L2) acc = fma((double)e[q], (double)e[q], acc);
                else mx = fmaxf(mx, ax);
            }
        }
        double tot = (norm_kind == QGX_NORM_L2) ? wave_sum(acc) : (double)wave_max(mx);
        bad = wave_or(bad);
        float n = (norm_kind == QGX_NORM_L2) ? (float)sqrt(tot) : (float)tot;
        if (norm_kind != QGX_NORM_L2 && norm_kind != QGX_NORM_LINF && bad == 0 && tot > 0.0) {
            const double inv_m = 1.0 / tot;
            double sum = 0.0;
#pragma unroll 1
            for (uint32_t i = lo + (uint32_t)lane; i < hi; i += kWave)
                sum += pow_int(fabs((double)Vk[i]) * inv_m, (uint32_t)norm_kind);
            n = (float)(tot * root_int(wave_sum(sum), (uint32_t)norm_kind));
        }
        const bool usable = have && (bad == 0) && (n > 0.0f) && (n <= 3.402823466e+38f);
        if (have && bad != 0 && lane == 0) raise_error(sc, QGX_EBIT_NONFINITE);

        uint32_t bins[4 * RPB];
        uint32_t mine = 0;                                // slots whose counter this lane took from zero
        if (usable) {
            const float rinv = 1.0f / n;
#pragma unroll
            for (int r = 0; r < RPB; ++r) {
                const uint32_t i0 = lo + (uint32_t)r * 256u + (uint32_t)lane * 4u;
                const float e[4] = {v[r].x, v[r].y, v[r].z, v[r].w};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    bins[4 * r + q] = 0;
                    if (i0 + (uint32_t)q < hi) {
                        const float u = fminf(fabsf(e[q]) * rinv, 1.0f);
                        const uint32_t bin = bin_of(u, n_bins), sh = (bin & 1u) * 16u;
                        bins[4 * r + q] = bin;
                        const uint32_t old = atomicAdd(&s_cnt[bin >> 1], 1u << sh);
                        if (((old >> sh) & 0xFFFFu) == 0u) mine |= 1u << (4 * r + q);
                    }
                }
            }
        }
        const double wgt = (double)n * (double)n;         // lambda of Section 3.3, unnormalised
        wave_lds_fence();                                 // the counts a lane folds hold other lanes' additions
        for (int turn = 0; turn < kW; ++turn) {
            if (turn == w && usable) {
#pragma unroll
                for (int s = 0; s < 4 * RPB; ++s) {
                    if (mine & (1u << s)) {
                        const uint32_t bin = bins[s], sh = (bin & 1u) * 16u;
                        const uint32_t cnt = (s_cnt[bin >> 1] >> sh) & 0xFFFFu;
                        s_acc[bin] += (double)cnt * wgt;
                        atomicAnd(&s_cnt[bin >> 1], ~(0xFFFFu << sh));
                    }
                }
            }
            __syncthreads();
        }
    }
    for (uint32_t i = (uint32_t)tid; i < n_bins; i += kW * kWave)
        partial[(size_t)blockIdx.x * n_bins + i] = s_acc[i];
}

// Workgroup sums -> histogram, in an order that does not depend on timing: the workgroups' values of a
// bin are cut into kRedSegs runs of consecutive workgroups, a thread adds one run, then the runs of a bin
// are added in order.  16 bins to a workgroup: 256 workgroups for the largest histogram, a row of 16 lanes
// reads 128 consecutive bytes of one workgroup's sums.
constexpr uint32_t kRedBins = 16;
constexpr uint32_t kRedSegs = 16;

__global__ __launch_bounds__(kRedBins * kRedSegs) void k_hist_reduce(uint32_t n_bins, uint32_t n_partial,
                                                                     const double* __restrict__ partial,
                                                                     double* __restrict__ hist)
{
    __shared__ double s_run[kRedSegs][kRedBins];
    const uint32_t bl = threadIdx.x & (kRedBins - 1u), seg = threadIdx.x / kRedBins;
    const uint32_t i = blockIdx.x * kRedBins + bl;
    const uint32_t run = (n_partial + kRedSegs - 1u) / kRedSegs;
    const uint32_t lo = min(seg * run, n_partial), hi = min(lo + run, n_partial);
    double acc = 0.0;
    if (i < n_bins) {
        uint32_t g = lo;
        for (; g + 4u <= hi; g += 4u) {                   // four loads on their way, added in order
            const double v0 = partial[(size_t)g * n_bins + i], v1 = partial[(size_t)(g + 1u) * n_bins + i];
            const double v2 = partial[(size_t)(g + 2u) * n_bins + i], v3 = partial[(size_t)(g + 3u) * n_bins + i];
            acc += v0; acc += v1; acc += v2; acc += v3;
        }
        for (; g < hi; ++g) acc += partial[(size_t)g * n_bins + i];
    }
    s_run[seg][bl] = acc;
    __syncthreads();
    if (seg == 0 && i < n_bins) {
        double tot = 0.0;
        for (uint32_t q = 0; q < kRedSegs; ++q) tot += s_run[q][bl];
        hist[i] = tot;
    }
}

uint32_t histogram_groups(const Layout& lay)
{
    // two workgroups per compute unit; three (what its LDS holds with 4096 bins) where a workgroup is a single wave
    const uint32_t n_work = lay.K * lay.NB;
    const uint32_t groups = (!lay.shared_chunks && lay.waves_per_bucket == 1u) ? 768u : 512u;
    return n_work < groups ? n_work : groups;
}

hipError_t launch_histogram(const Layout& lay, const float* V, int norm_kind, uint32_t n_bins, double* partial,
                            uint32_t n_partial, double* hist, Scalars* sc, hipStream_t st)
{
    if (lay.shared_chunks) {                              // buckets of 256 << s coordinates, s = 0..3
        const size_t lds = (size_t)n_bins * (sizeof(double) + 4 * sizeof(uint16_t));
        switch (lay.bucket_shift) {
            case 8: hipLaunchKernelGGL(k_histogram_small<1>, dim3(n_partial), dim3(256), lds, st, lay, V, norm_kind, n_bins, partial, sc); break;
            case 9: hipLaunchKernelGGL(k_histogram_small<2>, dim3(n_partial), dim3(256), lds, st, lay, V, norm_kind, n_bins, partial, sc); break;
            case 10: hipLaunchKernelGGL(k_histogram_small<4>, dim3(n_partial), dim3(256), lds, st, lay, V, norm_kind, n_bins, partial, sc); break;
            default: hipLaunchKernelGGL(k_histogram_small<8>, dim3(n_partial), dim3(256), lds, st, lay, V, norm_kind, n_bins, partial, sc); break;
        }
    } else {
        const size_t lds = (size_t)n_bins * (sizeof(double) + sizeof(uint32_t));
        if (lay.waves_per_bucket <= 4u)
            hipLaunchKernelGGL(k_histogram<4>, dim3(n_partial), dim3(lay.waves_per_bucket * kWave), lds, st, lay, V, norm_kind,
                               n_bins, partial, sc);
        else
            hipLaunchKernelGGL(k_histogram<kMaxWaves>, dim3(n_partial), dim3(lay.waves_per_bucket * kWave), lds, st, lay, V,
                               norm_kind, n_bins, partial, sc);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_hist_reduce, dim3((n_bins + kRedBins - 1u) / kRedBins), dim3(kRedBins * kRedSegs), 0, st, n_bins, n_partial,
                       partial, hist);
    return hipGetLastError();
}

// ---- solver ---------------------------------------------------------------------------------------
// With F~ piecewise uniform inside bins, the stationarity condition of (QAda) in l_j = x between its
// neighbours a = l_{j-1}, c = l_{j+1},
//     G(x) = int_a^x (u - a) dF~ - int_x^c (c - u) dF~ = 0 ,
// has dG/dx = (c - a) * density(x), so G(x) = (c - a) * mass(a, x) - int_a^c (c - u) dF~: the level goes
// where the mass between a and x reaches  t = int_a^c (c - u) dF~ / (c - a).  Where that holds on a
// whole interval (no mass there) the smallest such x is taken; with no mass at all between the
// neighbours that is a.  Levels stay in binary64 between the sweeps and are rounded to the table's
// binary32 once, at the end.
//
// Everything is summed from a onwards, non-negative terms only (a difference of cumulative sums taken
// from 0 would lose a sliver of mass next to a level against the total).  A two-level tree over the bins
// keeps that short: nodes of 16 and 256 bins hold their mass and their moment about their own right
// edge, rho = sum H_b (edge - mid_b), so that int (c - u) dF~ over a node is (c - edge) * mass + rho.
// The whole bins between a and c are then at most five runs of at most 16 items: bins up to a multiple
// of 16, nodes of 16 up to a multiple of 256, nodes of 256, and down again.  One update is the work of a
// row of 16 lanes, a lane per item of a run: the integral is one sum across the row, and the place where
// the mass reaches t is found with a prefix sum across the row per run, then inside the node that holds
// it, a level of the tree at a time.

struct Tree {
    const double* H;      // LDS [n_bins]
    const double* m1;     // [n_bins / 16] mass of a node of 16 bins
    const double* r1;     // its moment about its right edge
    const double* m2;     // [n_bins / 256] the same for the nodes of 256 bins
    const double* r2;
    uint32_t n_bins;
};

constexpr uint32_t kRow = 16;     // lanes per update

// The bin whose half-open interval [edge, next edge) holds x >= 0: the bins are 64 to an octave, so the bin
// number is the exponent and the top six fraction bits, which a binary64 number shows as its bits 46 and up.
__device__ __forceinline__ uint32_t bin_containing(uint32_t n_bins, double x)
{
    const int key = (int)((unsigned long long)__double_as_longlong(x) >> 46) - (1023 * 64 - (int)n_bins);
    return (uint32_t)min(max(key, 0), (int)n_bins - 1);
}

// x of another lane of the row, by a DPP control word; lanes without a source read 0
template <int CTRL>
__device__ __forceinline__ double row_dpp(double x)
{
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(x), CTRL, 0xf, 0xf, true);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(x), CTRL, 0xf, 0xf, true);
    return __hiloint2double(hi, lo);
}

// The sum over the row, the same bits in all its lanes: mirror, mirror within eight, swap pairs, swap
// neighbours; at every step the two lanes of a pair add the same two numbers.
__device__ __forceinline__ double row_sum(double x)
{
    x += row_dpp<0x140>(x);      // row_mirror
    x += row_dpp<0x141>(x);      // row_half_mirror
    x += row_dpp<0x4E>(x);       // quad_perm [2,3,0,1]
    x += row_dpp<0xB1>(x);       // quad_perm [1,0,3,2]
    return x;
}

// inclusive prefix sum over the lanes of the row (row_shr by 1, 2, 4, 8; nothing is shifted in from outside)
__device__ __forceinline__ double row_scan(double x, uint32_t)
{
    x += row_dpp<0x111>(x);
    x += row_dpp<0x112>(x);
    x += row_dpp<0x114>(x);
    x += row_dpp<0x118>(x);
    return x;
}

// first lane of this row with the predicate set, kRow if none
__device__ __forceinline__ uint32_t row_first(bool pred)
{
    const unsigned long long b = __ballot(pred);
    const uint32_t mine = (uint32_t)(b >> (threadIdx.x & 48u)) & 0xFFFFu;
    return mine ? (uint32_t)__ffs((int)mine) - 1u : kRow;
}

// mass of item idx of a level of the tree (0: a bin, 1: 16 bins, 2: 256 bins)
__device__ __forceinline__ double item_mass(const Tree& T, uint32_t lvl, uint32_t idx)
{
    return lvl == 2u ? T.m2[idx] : lvl == 1u ? T.m1[idx] : T.H[idx];
}

// Right edge of the last bin with mass in [first, last_plus_1), or `fallback` if none has any.
__device__ double last_mass_edge(const Tree& T, uint32_t first, uint32_t last_plus_1, double fallback)
{
    for (uint32_t b = last_plus_1; b > first; --b)
        if (T.H[b - 1u] > 0.0) return bin_edge(b, T.n_bins);
    return fallback;
}

// All 16 lanes of a row call this with the same a and c and get the same x.
__device__ double stationary_point(const Tree& T, double a, double c)
{
    if (!(c > a)) return a;
    const uint32_t nb = T.n_bins, li = threadIdx.x & (kRow - 1u);
    const uint32_t ba = bin_containing(nb, a), bc = bin_containing(nb, c);
    // the pieces of the bins that hold a and c, and the whole bins P .. Q - 1 between them
    const double a_e0 = bin_edge(ba, nb), a_e1 = bin_edge(ba + 1u, nb);
    const double a_hi = c < a_e1 ? c : a_e1;
    const double m_a = T.H[ba] * (a_hi - a) / (a_e1 - a_e0);
    double m_c = 0.0, c_e0 = c;
    if (bc > ba) {
        c_e0 = bin_edge(bc, nb);
        m_c = T.H[bc] * (c - c_e0) / (bin_edge(bc + 1u, nb) - c_e0);
    }
    const uint32_t P = ba + 1u, Q = bc > P ? bc : P;
    // runs: bins [P, P1), nodes of 16 [p1, p2), nodes of 256 [p2 / 16, q2 / 16), nodes of 16 [q2, q1), bins [Q1, Q)
    const uint32_t up = (P + 15u) & ~15u;
    const uint32_t P1 = Q < up ? Q : up;
    const uint32_t dn = Q & ~15u;
    const uint32_t Q1 = dn > P1 ? dn : P1;
    const uint32_t p1 = P1 >> 4, q1 = Q1 >> 4;                 // equal when no whole node of 16 lies between
    const uint32_t up1 = (p1 + 15u) & ~15u;
    const uint32_t p2 = q1 < up1 ? q1 : up1;
    const uint32_t dn1 = q1 & ~15u;
    const uint32_t q2 = dn1 > p2 ? dn1 : p2;
    const uint32_t lo[5] = {P, p1, p2 >> 4, q2, Q1}, hi[5] = {P1, p2, p2 < q2 ? q2 >> 4 : p2 >> 4, q1, Q};
    const uint32_t lvl[5] = {0u, 1u, 2u, 1u, 0u};
    double m[5], rho = 0.0;
#pragma unroll
    for (int s = 0; s < 5; ++s) {
        const uint32_t idx = lo[s] + li;
        m[s] = 0.0;
        if (idx < hi[s]) {
            m[s] = item_mass(T, lvl[s], idx);
            if (lvl[s] == 0u) rho += m[s] * (c - 0.5 * (bin_edge(idx, nb) + bin_edge(idx + 1u, nb)));
            else if (lvl[s] == 1u) rho += (c - bin_edge(16u * idx + 16u, nb)) * m[s] + T.r1[idx];
            else rho += (c - bin_edge(256u * idx + 256u, nb)) * m[s] + T.r2[idx];
        }
    }
    // int_a^c (c - u) dF~
    const double right_all = m_a * (c - 0.5 * (a + a_hi)) + row_sum(rho) + m_c * (c - 0.5 * (c_e0 + c));
    if (!(right_all > 0.0)) return a;                                  // no mass between the neighbours
    const double t = right_all / (c - a);
    // the smallest x with mass(a, x) >= t
    if (m_a >= t) return fmin(fmax(a + t / m_a * (a_hi - a), a), c);
    // the runs' prefix sums side by side, then each run's mass on top of the runs before it
    double cum[5], base[6], tot[5];
#pragma unroll
    for (int s = 0; s < 5; ++s) { cum[s] = row_scan(m[s], li); tot[s] = row_sum(m[s]); }
    base[0] = m_a;
#pragma unroll
    for (int s = 0; s < 5; ++s) {
        cum[s] += base[s];
        base[s + 1] = base[s] + tot[s];
    }
    double acc = base[5], prev = 0.0;
    uint32_t at_lvl = 0u, at_idx = 0u;
    bool found = false;
#pragma unroll
    for (int s = 0; s < 5; ++s) {
        const uint32_t first = row_first(lo[s] + li < hi[s] && cum[s] >= t);
        if (!found && first < kRow) {
            found = true;
            at_lvl = lvl[s];
            at_idx = lo[s] + first;
            const double before = __shfl(cum[s], (int)(first > 0u ? first - 1u : 0u), (int)kRow);
            prev = first > 0u ? before : base[s];
        }
    }
    double x;
    if (!found) {
        // the mass reaches t in the piece of c's bin, or t is a rounding above all the mass: then the answer
        // is where the mass ends
        x = m_c > 0.0 ? c_e0 + (t - acc) / m_c * (c - c_e0) : last_mass_edge(T, P, Q, m_a > 0.0 ? a_hi : a);
    } else {
        const uint32_t node_end = at_lvl == 2u ? 256u * at_idx + 256u : at_lvl == 1u ? 16u * at_idx + 16u : at_idx + 1u;
        bool lost = false;
        while (at_lvl > 0u && !lost) {                                 // into the node that holds it
            const uint32_t child = 16u * at_idx + li;
            const double cum = prev + row_scan(item_mass(T, at_lvl - 1u, child), li);
            const uint32_t first = row_first(cum >= t);
            if (first < kRow) {
                const double before = __shfl(cum, (int)(first > 0u ? first - 1u : 0u), (int)kRow);
                prev = first > 0u ? before : prev;
                at_idx = 16u * at_idx + first;
                at_lvl -= 1u;
            } else {
                lost = true;       // the node's mass reached t and the sum of its parts, rounded otherwise, did not
            }
        }
        if (lost) {
            x = last_mass_edge(T, P, node_end, m_a > 0.0 ? a_hi : a);
        } else {
            const double e0 = bin_edge(at_idx, nb);
            x = e0 + (t - prev) / T.H[at_idx] * (bin_edge(at_idx + 1u, nb) - e0);
            x = fmax(x, e0);
        }
    }
    return fmin(fmax(x, a), c);
}

// The sweeps update level j from the new l_{j-1} and the old l_{j+1}, one level after the other.
// Update (sweep s, level j) therefore only waits for (s, j-1) and (s-1, j+1), and all updates with
// the same 2s + j can run together: row s of the workgroup's 16 rows of 16 lanes carries sweep s, two
// levels behind row s-1, and takes its upper neighbour from what that row left in LDS one step ago.
// Same updates in the same order as the plain double loop, in 2 sweeps + n_sym steps instead of
// sweeps * n_sym.
__global__ __launch_bounds__(256) void k_fit(Tables* tab, const double* __restrict__ hist, uint32_t n_bins,
                                             uint32_t sweeps)
{
    extern __shared__ __align__(16) unsigned char s_raw[];
    double* H = reinterpret_cast<double*>(s_raw);                // [n_bins]
    __shared__ double s_m1[QGX_MAX_BINS / 16], s_r1[QGX_MAX_BINS / 16];
    __shared__ double s_m2[QGX_MAX_BINS / 256], s_r2[QGX_MAX_BINS / 256];
    __shared__ double s_lev[kSymMax + 1];                         // the table between passes
    __shared__ double s_moved[2][kRow];                           // what each row moved in the last two steps

    const uint32_t tid = threadIdx.x;
    for (uint32_t b = tid; b < n_bins; b += 256u) H[b] = hist[b];
    __syncthreads();
    const uint32_t n1 = n_bins >> 4, n2 = n_bins >> 8;            // n_bins is a multiple of 64
    if (tid < n1) {
        const double edge = bin_edge(16u * tid + 16u, n_bins);
        double m = 0.0, r = 0.0;
        for (uint32_t b = 16u * tid; b < 16u * tid + 16u; ++b) {
            m += H[b];
            r += H[b] * (edge - 0.5 * (bin_edge(b, n_bins) + bin_edge(b + 1u, n_bins)));
        }
        s_m1[tid] = m; s_r1[tid] = r;
    }
    __syncthreads();
    // the last node of 256 is short when n_bins is not a multiple of 256: nothing reads it then (a run of
    // nodes of 256 only holds whole ones), but its slot is written all the same
    if (tid < (n_bins + 255u) >> 8) {
        const uint32_t last = min(16u * tid + 16u, n1);
        const double edge = bin_edge(16u * last, n_bins);
        double m = 0.0, r = 0.0;
        for (uint32_t i = 16u * tid; i < last; ++i) {
            m += s_m1[i];
            r += (edge - bin_edge(16u * i + 16u, n_bins)) * s_m1[i] + s_r1[i];
        }
        s_m2[tid] = m; s_r2[tid] = r;
    }
    const uint32_t n_sym = tab->n_sym;
    if (tid < n_sym) s_lev[tid] = (double)tab->levels[tid];
    __syncthreads();
    // is there any mass at all?  (terms that are not negative: the order of the sum does not matter to that)
    double total = 0.0;
    for (uint32_t i = 0; i < (n_bins + 255u) >> 8; ++i) total += s_m2[i];
    (void)n2;

    const Tree T = {H, s_m1, s_r1, s_m2, s_r2, n_bins};
    const uint32_t row = tid >> 4, top = n_sym - 1u;
    if (total > 0.0 && n_sym > 2u) {
        for (uint32_t first = 0; first < sweeps; first += kRow) {
            const uint32_t ns = min(kRow, sweeps - first);               // sweeps of this pass, one per row
            double mine = 0.0;                      // the level this row moved in its last step
            const uint32_t steps = 2u * (ns - 1u) + (top - 1u);
            for (uint32_t t = 1; t <= steps; ++t) {
                const int j = (int)t - 2 * (int)row;
                const bool active = row < ns && j >= 1 && j < (int)top;
                if (active) {
                    // the row below moved level j + 1 one step ago; the first row reads the table of the last pass
                    double above = row == 0u ? s_lev[j + 1] : s_moved[(t - 1u) & 1u][row - 1u];
                    if (j + 1 == (int)top) above = 1.0;
                    const double below = j == 1 ? 0.0 : mine;
                    mine = stationary_point(T, below, above);
                    if ((tid & (kRow - 1u)) == 0u) {
                        s_moved[t & 1u][row] = mine;
                        if (row == ns - 1u) s_lev[j] = mine;
                    }
                }
                __syncthreads();
            }
        }
    }
    // strictly increasing with gaps of at least 2^-24: up from l_0 = 0, then down from l_s = 1; one
    // lane, the table is short
    if (tid == 0) {
        float* lv = tab->levels;
        lv[0] = 0.0f; lv[top] = 1.0f;
        for (uint32_t j = 1; j < top; ++j) {
            const float x = (float)s_lev[j];
            const float floor_ = lv[j - 1] + 0x1p-24f;
            lv[j] = x < floor_ ? floor_ : x;
        }
        for (uint32_t j = top - 1u; j >= 1u; --j) {
            const float ceil_ = lv[j + 1] - 0x1p-24f;
            if (lv[j] > ceil_) lv[j] = ceil_;
        }
    }
}

hipError_t launch_fit(Tables* tab, const double* hist, uint32_t n_bins, uint32_t sweeps, hipStream_t st)
{
    const size_t lds = (size_t)n_bins * sizeof(double);
    hipLaunchKernelGGL(k_fit, dim3(1), dim3(256), lds, st, tab, hist, n_bins, sweeps);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_build_tables(tab, st);
}

// ---- Psi from estimated symbol probabilities (Proposition 1; Appendix J, Huffman coding) ---------------
// p_j: the mass F~ sends to level j through the random rounding.  Thread j walks the bins under the
// gap below its level (rising part of its hat function) and then the gap above (falling part); a
// piece of a bin contributes its mass times the rounding probability at its midpoint, which is exact
// for the piecewise-uniform density.
//
// The code: optimal prefix code for the weights round(p 2^32) (at least 1) with no word longer than
// max_len, by package-merge (Larmore and Hirschberg 1990); with a slack limit that is Huffman's code.
// Every level offers each symbol one coin at the symbol's weight; from the deepest level up, the
// sorted list of a level is paired into packages that are merged into the next level's coins; the
// cheapest 2 (n - 1) entries of the top list are bought, a package standing for its two entries one
// level down.  A symbol's length is the number of its coins bought.  Equal weights: coin before
// package, lower index first.  Words are numbered canonically by (length, index), first bit first.
__global__ __launch_bounds__(256) void k_fit_code(Tables* tab, const double* __restrict__ hist, uint32_t n_bins,
                                                  uint32_t max_len, double* __restrict__ p_out)
{
    extern __shared__ __align__(16) unsigned char s_raw[];
    double* H = reinterpret_cast<double*>(s_raw);                      // [n_bins]
    __shared__ double s_part[256];
    __shared__ double s_lev[kSymMax];
    __shared__ unsigned long long s_w[kSymMax], s_sw[kSymMax], s_cur[2 * kSymMax], s_nxt[2 * kSymMax];
    __shared__ uint8_t s_pkg[kMaxCode][2 * kSymMax];
    __shared__ uint32_t s_count[kMaxCode];
    __shared__ uint8_t s_order[kSymMax], s_len[kSymMax];

    const uint32_t tid = threadIdx.x, n = tab->n_sym;
    double part = 0.0;
    for (uint32_t b = tid; b < n_bins; b += 256u) { const double h = hist[b]; H[b] = h; part += h; }
    s_part[tid] = part;
    if (tid < n) s_lev[tid] = (double)tab->levels[tid];
    __syncthreads();
    for (uint32_t off = 128; off > 0; off >>= 1) {
        if (tid < off) s_part[tid] += s_part[tid + off];
        __syncthreads();
    }
    const double total = s_part[0];

    // p_j: a row of 16 lanes per level, every lane each 16th bin under the two gaps next to the level
    for (uint32_t j = tid >> 4; j < ((n + 15u) & ~15u); j += 16u) {        // whole rows walk together
        const uint32_t li = tid & 15u;
        double acc = 0.0;
        if (j < n && total > 0.0) {
            for (int side = 0; side < 2; ++side) {                         // 0: gap below (rising), 1: gap above (falling)
                if ((side == 0 && j == 0) || (side == 1 && j + 1 >= n)) continue;
                const double a = side == 0 ? s_lev[j - 1] : s_lev[j], c = side == 0 ? s_lev[j] : s_lev[j + 1];
                uint32_t b = bin_of((float)a, n_bins);
                while (b > 0 && bin_edge(b, n_bins) > a) --b;
                for (b += li; b < n_bins; b += 16u) {
                    const double e0 = bin_edge(b, n_bins), e1 = bin_edge(b + 1, n_bins);
                    if (e0 >= c) break;
                    const double lo = a > e0 ? a : e0, hi = c < e1 ? c : e1;
                    if (!(hi > lo) || H[b] == 0.0) continue;
                    const double mass = H[b] * (hi - lo) / (e1 - e0);
                    const double up = (0.5 * (lo + hi) - a) / (c - a);
                    acc += side == 0 ? mass * up : mass * (1.0 - up);
                }
            }
        }
        acc = row_sum(acc);
        if (j < n && li == 0u) {
            if (total > 0.0) acc /= total;
            p_out[j] = acc;
            const double x = floor(acc * 4294967296.0 + 0.5);
            s_w[j] = x >= 1.0 ? (unsigned long long)x : 1ull;
        }
    }
    __syncthreads();

    // Symbols by weight, then index: a symbol's place is the number of symbols that come before it.
    if (tid < n) {
        const unsigned long long wi = s_w[tid];
        uint32_t rank = 0;
        for (uint32_t k = 0; k < n; ++k) {
            const unsigned long long wk = s_w[k];
            rank += (wk < wi || (wk == wi && k < tid)) ? 1u : 0u;
        }
        s_order[rank] = (uint8_t)tid;
    }
    __syncthreads();
    if (tid < n) s_sw[tid] = s_w[s_order[tid]];
    __syncthreads();
    // Package-merge, a level per round: the list of a level is the merge of the n single symbols with the
    // packages (pairs, in order) of the level above; at equal weight the single comes first.  Both lists are
    // sorted, so an item's place is its own index plus the number of items of the other list before it
    // (a binary search): a thread per item.
    unsigned long long* cur = s_cur;
    unsigned long long* nxt = s_nxt;
    uint32_t m = n;
    if (tid < n) { cur[tid] = s_sw[tid]; s_pkg[max_len - 1][tid] = 0; }
    if (tid == 0) s_count[max_len - 1] = m;
    __syncthreads();
    for (int l = (int)max_len - 2; l >= 0; --l) {
        const uint32_t n_pk = m >> 1;
        if (tid < n) {                                   // single tid: after the packages that weigh less
            const unsigned long long wa = s_sw[tid];
            uint32_t lo = 0, hi = n_pk;                  // first package with weight >= wa
            while (lo < hi) {
                const uint32_t mid = (lo + hi) >> 1;
                if (cur[2 * mid] + cur[2 * mid + 1] < wa) lo = mid + 1; else hi = mid;
            }
            nxt[tid + lo] = wa;
            s_pkg[l][tid + lo] = 0;
        } else if (tid - n < n_pk) {                     // package tid - n: after the singles that weigh no more
            const uint32_t ib = tid - n;
            const unsigned long long wb = cur[2 * ib] + cur[2 * ib + 1];
            uint32_t lo = 0, hi = n;                     // first single with weight > wb
            while (lo < hi) {
                const uint32_t mid = (lo + hi) >> 1;
                if (s_sw[mid] <= wb) lo = mid + 1; else hi = mid;
            }
            nxt[ib + lo] = wb;
            s_pkg[l][ib + lo] = 1;
        }
        m = n + n_pk;
        if (tid == 0) s_count[l] = m;
        __syncthreads();
        unsigned long long* t = cur; cur = nxt; nxt = t;
    }
    // The 2 (n - 1) lightest items of the lowest level are taken; every single among the items taken at a
    // level adds a bit to its symbol (the singles are the lightest symbols in order), every package sends
    // its two parts of the level above.
    if (tid < n) s_len[tid] = 0;
    __syncthreads();
    uint32_t take = 2u * (n - 1u);
    for (uint32_t l = 0; l < max_len; ++l) {                           // (take falls to 0 and stays there)
        take = min(take, s_count[l]);
        const uint32_t packages = (uint32_t)__syncthreads_count(tid < take && s_pkg[l][tid] != 0);
        const uint32_t singles = take - packages;
        if (tid < singles) s_len[s_order[tid]] += 1;
        take = 2u * packages;
    }
    __syncthreads();
    // canonical words: the symbols in the order (length, index), each word the count of the words before it at
    // its own length's scale; the table wants the first-written bit in bit 0
    if (tid < n) {
        const uint32_t L = s_len[tid];
        uint32_t code = 0;
        for (uint32_t k = 0; k < n; ++k) {
            const uint32_t lk = s_len[k];
            if (lk < L || (lk == L && k < tid)) code += 1u << (L - lk);
        }
        tab->code[tid] = (__brev(code) >> (32u - L)) | (L << 16);
    }
}

hipError_t launch_fit_code(Tables* tab, const double* hist, uint32_t n_bins, uint32_t max_len, double* p_out,
                           hipStream_t st)
{
    hipLaunchKernelGGL(k_fit_code, dim3(1), dim3(256), (size_t)n_bins * sizeof(double), st, tab, hist, n_bins, max_len, p_out);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_build_tables(tab, st);
}

}  // namespace qgx
