// CODE o Q in one pass: per-bucket norm, normalise, level lookup, stochastic rounding, code lookup,
// bit packing through LDS, ordered placement of the chunks in the payload.
// (Definition 1; Section 3.2; Appendix J "Encoding".)
//
// Work decomposition for 64-wide wavefronts: one workgroup per (worker, bucket); one wave per chunk of
// 4096 coordinates.  A wave holds its chunk in registers as 16 rows of 256 coordinates, lane L owning
// the four consecutive coordinates 4L..4L+3 of every row, so that (a) every global load is a fully
// coalesced 16-byte-per-lane access, (b) the bucket is read from HBM once and stays in registers
// between the norm reduction and the rounding pass, (c) one Philox4x32 block (four words) serves
// exactly the four coordinates of a lane and row.
//
// The stream keeps coordinate order: per row the lanes' code lengths are prefix-summed across the wave
// and every lane ORs its (at most 56) bits into the wave's LDS staging buffer.  Chunks are placed in
// the payload in chunk order, so a workgroup needs the total length of all earlier buckets of its
// worker: a decoupled look-back over per-bucket (flag, length) words gives it without a second pass
// over V.  Workgroups take their (bucket, worker) from an atomic ticket, so every workgroup a waiting
// one depends on is already running; the wait is bounded all the same.
#include "qgx_device.h"

namespace qgx {

constexpr int kStageWords = kChunkWordsMax + 4;   // per-wave LDS staging, 16-byte multiple
constexpr unsigned kSpinLimit = 1u << 22;

struct Sym4 {                // the four symbols of one lane and row
    uint32_t idx[4];
    uint32_t neg[4];
};

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t x)
{
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) x += (uint32_t)__shfl_xor((int)x, off, kWave);
    return x;
}

// Exclusive prefix of `agg` over buckets 0..b-1 of one worker (decoupled look-back, one wave).
// state[] entries: high word = epoch << 2 | status (1 = aggregate, 2 = inclusive prefix), low word = value.
__device__ uint32_t lookback_exclusive(unsigned long long* state, uint32_t b, uint32_t agg, uint32_t epoch,
                                       Scalars* sc)
{
    const int lane = lane_id();
    const unsigned long long tag_agg = (unsigned long long)((epoch << 2) | 1u) << 32;
    const unsigned long long tag_pre = (unsigned long long)((epoch << 2) | 2u) << 32;
    if (b == 0) {
        if (lane == 0) __hip_atomic_store(&state[0], tag_pre | agg, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return 0;
    }
    if (lane == 0) __hip_atomic_store(&state[b], tag_agg | agg, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    uint32_t excl = 0;
    int pos = (int)b - 1;
    unsigned spins = 0;
    for (;;) {
        const int i = pos - lane;
        unsigned long long s = 0;
        bool ready = true;
        for (;;) {
            if (i >= 0) {
                s = __hip_atomic_load(&state[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const uint32_t flag = (uint32_t)(s >> 32);
                ready = ((flag >> 2) == epoch) && ((flag & 3u) != 0u);
            }
            if (__all(ready)) break;
            if (++spins > kSpinLimit) {           // never expected: every predecessor is already running
                if (lane == 0) raise_error(sc, QGX_EBIT_STATE);
                if (!ready) s = 0;
                break;
            }
            __builtin_amdgcn_s_sleep(8);
        }
        const bool have = (i >= 0) && ready;
        const uint32_t val = have ? (uint32_t)s : 0u;
        const bool is_pre = have && (((uint32_t)(s >> 32) & 3u) == 2u);
        const unsigned long long m = __ballot(is_pre);
        if (m != 0ull) {
            const int first = __ffsll((long long)m) - 1;      // nearest predecessor with a full prefix
            excl += wave_sum_u32(lane <= first ? val : 0u);
            break;
        }
        excl += wave_sum_u32(val);
        if (pos < kWave) break;
        pos -= kWave;
    }
    if (lane == 0)
        __hip_atomic_store(&state[b], tag_pre | (unsigned long long)(excl + agg), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    return excl;
}

template <EncMode MODE>
__global__ __launch_bounds__(1024) void k_encode(Layout lay, const Tables* __restrict__ tab, Scalars* sc,
                                                 EncodeArgs a)
{
    extern __shared__ __align__(16) uint32_t s_stage[];          // [waves][kStageWords]
    __shared__ float4 s_lev[kSymMax];
    __shared__ uint32_t s_code[kSymMax];
    __shared__ __align__(4) uint8_t s_cell[kCellsPad];
    __shared__ double s_red[kMaxWaves];
    __shared__ uint32_t s_bad[kMaxWaves];
    __shared__ uint32_t s_words[kMaxWaves];
    __shared__ __align__(4) uint16_t s_sub[kMaxWaves][kSubs];
    __shared__ uint32_t s_misc[2];

    const int tid = (int)threadIdx.x, lane = lane_id(), w = wave_id();
    const int nwaves = (int)(blockDim.x >> 6);
    const uint32_t n_sym = tab->n_sym;

    if (MODE != EncMode::QuantOnly) {
        if (tid == 0) s_misc[0] = atomicAdd(&sc->ticket, 1u) - a.ticket_base;
    }
    for (int i = tid; i < kSymMax; i += (int)blockDim.x) {
        s_lev[i] = tab->lev[i];
        s_code[i] = tab->code[i];
    }
    for (int i = tid; i < kCellsPad / 4; i += (int)blockDim.x)
        reinterpret_cast<uint32_t*>(s_cell)[i] = reinterpret_cast<const uint32_t*>(tab->cell)[i];
    uint32_t* stage = s_stage + (size_t)w * kStageWords;
    if (MODE != EncMode::QuantOnly) {
        for (int q = lane; q < kStageWords / 4; q += kWave) reinterpret_cast<uint4*>(stage)[q] = make_uint4(0, 0, 0, 0);
    }
    __syncthreads();

    const uint32_t ticket = (MODE != EncMode::QuantOnly) ? s_misc[0] : (uint32_t)blockIdx.x;
    const uint32_t b = ticket / lay.K;                 // bucket-major: the K scans advance together
    const uint32_t k = ticket - b * lay.K;
    const uint32_t lo = lay.bucket_start[b], hi = lay.bucket_start[b + 1];
    const uint32_t c = lay.bucket_chunk0[b] + (uint32_t)w;
    const uint32_t clo = lo + (uint32_t)w * kChunk;
    const uint32_t clen = clo < hi ? min((uint32_t)kChunk, hi - clo) : 0u;
    const uint32_t cend = clo + clen;
    const int nrows = (int)((clen + 255u) >> 8);
    const size_t kbase = (size_t)k * lay.d;
    const bool vec_ok = (kbase & 3u) == 0;             // 16-byte aligned rows for this worker

    // ---- read the chunk once; norm of the bucket ------------------------------------------------
    float4 v[kRows];
    float n = 0.0f;
    bool bucket_bad = false;
    if (MODE != EncMode::EncodeOnly) {
        const float* __restrict__ Vk = a.V + kbase;
#pragma unroll
        for (int r = 0; r < kRows; ++r) {
            const uint32_t i0 = clo + (uint32_t)r * 256u + (uint32_t)lane * 4u;
            float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
            if (i0 + 4u <= cend) {
                if (vec_ok) x = *reinterpret_cast<const float4*>(Vk + i0);
                else x = make_float4(Vk[i0], Vk[i0 + 1], Vk[i0 + 2], Vk[i0 + 3]);
            } else if (i0 < cend) {
                x.x = Vk[i0];
                if (i0 + 1 < cend) x.y = Vk[i0 + 1];
                if (i0 + 2 < cend) x.z = Vk[i0 + 2];
            }
            v[r] = x;
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
                if (a.norm_kind == QGX_NORM_L2) acc = fma((double)e[q], (double)e[q], acc);
                else mx = fmaxf(mx, ax);
            }
        }
        if (a.norm_kind == QGX_NORM_L2) acc = wave_sum(acc);
        else acc = (double)wave_max(mx);
        bad = wave_or(bad);
        if (lane == 0) { s_red[w] = acc; s_bad[w] = bad; }
        __syncthreads();
        double tot = 0.0;
        uint32_t anybad = 0;
        for (int i = 0; i < nwaves; ++i) {
            if (a.norm_kind == QGX_NORM_L2) tot += s_red[i];
            else tot = fmax(tot, s_red[i]);
            anybad |= s_bad[i];
        }
        n = (a.norm_kind == QGX_NORM_L2) ? (float)sqrt(tot) : (float)tot;
        if (a.norms_in) n = a.norms_in[(size_t)k * lay.NB + b];
        bucket_bad = (anybad != 0) || !(fabsf(n) <= 3.402823466e+38f);
        if (bucket_bad) n = 0.0f;
        if (tid == 0) {
            if (bucket_bad) raise_error(sc, QGX_EBIT_NONFINITE);
            if (a.norms_out) a.norms_out[(size_t)k * lay.NB + b] = n;
        }
    }
    const float rinv = 1.0f / n;                       // one IEEE division per bucket
    const bool live = n > 0.0f;

    // ---- per row: quantise, code, pack ----------------------------------------------------------
    uint32_t row_base = 0;                             // bits of this chunk written so far (wave-uniform)
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        if (r < nrows) {
            const uint32_t i0 = clo + (uint32_t)r * 256u + (uint32_t)lane * 4u;
            Sym4 s;
            if (MODE == EncMode::EncodeOnly) {
                const uint8_t* __restrict__ Sk = a.sym_in + kbase;
                uint32_t pk = 0;
                if (i0 + 4u <= cend && vec_ok) pk = *reinterpret_cast<const uint32_t*>(Sk + i0);
                else {
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        if (i0 + (uint32_t)q < cend) pk |= (uint32_t)Sk[i0 + q] << (8 * q);
                }
                bool unknown = false;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t by = (pk >> (8 * q)) & 0xFFu;
                    s.idx[q] = by & 0x7Fu;
                    s.neg[q] = by >> 7;
                    if (s.idx[q] >= n_sym) { s.idx[q] = 0; unknown = true; }
                }
                if (__any(unknown) && lane == 0) raise_error(sc, QGX_EBIT_STREAM);
            } else {
                uint32_t rnd[4];
                philox4x32_10(i0 >> 2, 0u, k, a.call_id, a.seed_lo, a.seed_hi, rnd);
                const float e[4] = {v[r].x, v[r].y, v[r].z, v[r].w};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float x = e[q];
                    uint32_t sym = 0;
                    if (live) {
                        // u = min(|v| / ||v||, 1); tau(u) from the cell table, then at most a few steps up
                        const float u = fminf(fabsf(x) * rinv, 1.0f);
                        int key = (int)(__float_as_uint(u) >> (23 - kCellMant)) - kCellKey0;
                        key = key < 0 ? 0 : key;
                        uint32_t j = s_cell[key];
                        float4 t = s_lev[j];
                        while (t.z <= u) { ++j; t = s_lev[j]; }
                        // up with probability xi = (u - l_j) / (l_{j+1} - l_j):  r * gap < u - l_j
                        const float rr = (float)(rnd[q] >> 8);           // r * 2^24, exact
                        sym = j + ((rr * t.y < u - t.x) ? 1u : 0u);     // t.y = gap * 2^-24, exact scaling
                    }
                    s.idx[q] = sym;
                    s.neg[q] = __float_as_uint(x) >> 31;
                }
            }
            if (MODE == EncMode::QuantOnly) {
                uint8_t* __restrict__ Sk = a.sym_out + kbase;
                uint32_t pk = 0;
#pragma unroll
                for (int q = 0; q < 4; ++q) pk |= (s.idx[q] | (s.neg[q] << 7)) << (8 * q);
                if (i0 + 4u <= cend && vec_ok) *reinterpret_cast<uint32_t*>(Sk + i0) = pk;
                else {
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        if (i0 + (uint32_t)q < cend) Sk[i0 + q] = (uint8_t)(pk >> (8 * q));
                }
            } else {
                // Psi(idx) then the sign bit of a non-zero symbol; four symbols -> at most 56 bits
                uint64_t bits = 0;
                uint32_t len = 0;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if (i0 + (uint32_t)q < cend) {
                        const uint32_t cw = s_code[s.idx[q]];
                        uint32_t cb = cw & 0xFFFFu, cl = cw >> 16;
                        if (s.idx[q] != 0) { cb |= s.neg[q] << cl; cl += 1; }
                        bits |= (uint64_t)cb << len;
                        len += cl;
                    }
                }
                const uint32_t incl = wave_incl_scan(len);
                const uint32_t pos = row_base + incl - len;
                if (len != 0) {
                    const uint32_t wi = pos >> 5, sh = pos & 31u;
                    const uint64_t lo64 = (uint64_t)(uint32_t)bits << sh;
                    const uint64_t hi64 = (uint64_t)(uint32_t)(bits >> 32) << sh;
                    const uint32_t x0 = (uint32_t)lo64;
                    const uint32_t x1 = (uint32_t)(lo64 >> 32) | (uint32_t)hi64;
                    const uint32_t x2 = (uint32_t)(hi64 >> 32);
                    __hip_atomic_fetch_or(&stage[wi], x0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    if (x1) __hip_atomic_fetch_or(&stage[wi + 1], x1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    if (x2) __hip_atomic_fetch_or(&stage[wi + 2], x2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                }
                if ((lane & 15) == 15) s_sub[w][4 * r + (lane >> 4)] = (uint16_t)(row_base + incl);
                row_base += bcast_lane(incl, kWave - 1);
            }
        }
    }
    if (MODE == EncMode::QuantOnly) return;

    // ---- sizes, ordered offsets, flush ----------------------------------------------------------
    const uint32_t total_bits = row_base;
    uint32_t words = (total_bits + 31u) >> 5;
    words = (words + (kAlignWords - 1)) & ~(uint32_t)(kAlignWords - 1);
    if (lane >= 4 * nrows) s_sub[w][lane] = (uint16_t)total_bits;
    if (lane == 0) s_words[w] = words;
    __syncthreads();
    uint32_t bucket_words = 0, wave_excl = 0;
    for (int i = 0; i < nwaves; ++i) {
        if (i == w) wave_excl = bucket_words;
        bucket_words += s_words[i];
    }
    if (w == 0) {
        const uint32_t excl = lookback_exclusive(a.scan_state + (size_t)k * lay.NB, b, bucket_words, a.epoch, sc);
        if (lane == 0) s_misc[1] = excl;
    }
    __syncthreads();
    if (clen == 0) return;
    const uint32_t off = s_misc[1] + wave_excl;
    if (lane == 0) {
        a.chunk_off[(size_t)k * (lay.NC + 1) + c] = off;
        if (c + 1 == lay.NC) a.chunk_off[(size_t)k * (lay.NC + 1) + lay.NC] = off + words;
    }
    if (lane < 32)
        reinterpret_cast<uint32_t*>(a.sub_end + ((size_t)k * lay.NC + c) * kSubs)[lane] =
            reinterpret_cast<const uint32_t*>(s_sub[w])[lane];
    if ((uint64_t)off + words > a.cap_words) {
        if (lane == 0) raise_error(sc, QGX_EBIT_CAPACITY);
        return;
    }
    uint4* __restrict__ dst = reinterpret_cast<uint4*>(a.payload + (size_t)k * a.cap_words + off);
    const uint4* src = reinterpret_cast<const uint4*>(stage);
    for (uint32_t q = (uint32_t)lane; q < (words >> 2); q += kWave) dst[q] = src[q];
}

template <EncMode MODE>
static hipError_t launch_mode(const Layout& lay, const Tables* tab, Scalars* sc, const EncodeArgs& a, hipStream_t st)
{
    const int waves = (int)lay.waves_per_bucket;
    const size_t lds = (MODE == EncMode::QuantOnly) ? 16 : (size_t)waves * kStageWords * sizeof(uint32_t);
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_encode<MODE>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           kMaxWaves * kStageWords * (int)sizeof(uint32_t));
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    hipLaunchKernelGGL(k_encode<MODE>, dim3(lay.K * lay.NB), dim3(waves * kWave), lds, st, lay, tab, sc, a);
    return hipGetLastError();
}

hipError_t launch_encode(EncMode mode, const Layout& lay, const Tables* tab, Scalars* sc, const EncodeArgs& a,
                         hipStream_t st)
{
    switch (mode) {
        case EncMode::Fused: return launch_mode<EncMode::Fused>(lay, tab, sc, a, st);
        case EncMode::QuantOnly: return launch_mode<EncMode::QuantOnly>(lay, tab, sc, a, st);
        default: return launch_mode<EncMode::EncodeOnly>(lay, tab, sc, a, st);
    }
}

}  // namespace qgx
