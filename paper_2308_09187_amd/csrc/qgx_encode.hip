// CODE o Q in one pass: per-bucket norm, normalise, level lookup, stochastic rounding, code lookup,
// bit packing through LDS, ordered placement of the chunks in the payload.
// (Definition 1; Section 3.2; Appendix J "Encoding".)
//
// Work decomposition for 64-wide wavefronts: one workgroup per (worker, bucket), or several per
// bucket when it is longer than four chunks (see exchange_parts); one wave per chunk of
// 4096 coordinates.  A wave holds its chunk in registers as 16 rows of 256 coordinates, lane L owning
// the four consecutive coordinates 4L..4L+3 of every row, so that (a) every global load is a fully
// coalesced 16-byte-per-lane access, (b) the bucket is read from HBM once and stays in registers
// between the norm reduction and the rounding pass, (c) one Philox4x32 block (four words) serves
// exactly the four coordinates of a lane and row.
//
// The kernel runs close to what the memory system gives (about 93 % of a plain copy of its input) and
// at about two thirds of what the vector ALUs could issue, so the per-coordinate path is kept to a straight
// line: u -> cell (1/16, 1/32 or 1/64 of an octave, by the table's size) -> (boundary level, address of the lower candidate table row) -> one
// 16-byte LDS row holding the level, the scaled gap and the two candidate code words with the sign
// already appended -> compare against the Philox draw -> select.  Chunks that are not full, buckets
// with a zero norm and level tables too fine for the cell table take a general path.
//
// The stream keeps coordinate order: per row the lanes' code lengths are prefix-summed across the wave
// (DPP) and every lane ORs its (at most 56) bits into the wave's LDS staging buffer.
// Placement of the chunks in the payload.  Slotted: chunk c goes to c * slot_words; no workgroup waits
// for another.  Compact: chunks in chunk order without gaps, so a workgroup needs the total length of
// all earlier buckets of its worker: a decoupled look-back over per-bucket (flag, length) words gives
// it without a second pass over V.  There a workgroup's worker is fixed by its block index and its
// buckets come from that worker's atomic ticket, so every bucket a waiting workgroup depends on is
// held by a running workgroup that needs nothing from later tickets; the wait is bounded all the same.
#include "qgx_device.h"

namespace qgx {

constexpr unsigned kSpinLimit = 1u << 22;

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

// Buckets longer than four chunks are shared by several workgroups of four waves (parts), which a
// compute unit holds five of at different points of their life, where one workgroup of sixteen waves
// would have the unit to itself and leave the memory system idle while it computes and the ALUs idle
// while it loads.  What the parts must agree on is the bucket's norm: every part publishes its
// partial sum (or maximum) and reads the others'.  A published value is two words, each tagged with
// the launch's epoch, so a reader knows a word is this launch's without any ordering between
// stores.  The wait cannot deadlock: parts take their (bucket, part) from the worker's ticket
// counter, so at most the bucket of the newest tickets is incomplete, and every other waiting
// workgroup has all its partners running; the wait is bounded all the same.
// Called by one whole wave; returns the parts' values combined in part order in every lane.
__device__ double exchange_parts(unsigned long long* words /* [parts][2 phases][2] of this bucket */, uint32_t parts,
                                 uint32_t part, uint32_t phase, double mine, bool take_max, uint32_t epoch, Scalars* sc)
{
    const int lane = lane_id();
    const unsigned long long tag = (unsigned long long)epoch << 32;
    const unsigned long long bits = (unsigned long long)__double_as_longlong(mine);
    if (lane < 2)
        __hip_atomic_store(&words[(part * 2u + phase) * 2u + (uint32_t)lane],
                           tag | (lane ? (bits >> 32) : (bits & 0xFFFFFFFFull)), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const bool reader = (uint32_t)lane < 2u * parts;
    const uint32_t at = (((uint32_t)lane >> 1) * 2u + phase) * 2u + ((uint32_t)lane & 1u);
    unsigned long long s = 0;
    unsigned spins = 0;
    for (;;) {
        bool ready = true;
        if (reader) {
            s = __hip_atomic_load(&words[at], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            ready = (uint32_t)(s >> 32) == epoch;
        }
        if (__all(ready)) break;
        if (++spins > kSpinLimit) {               // never expected: see above
            if (lane == 0) raise_error(sc, QGX_EBIT_STATE);
            if (!ready) s = 0;
            break;
        }
        __builtin_amdgcn_s_sleep(8);
    }
    double tot = 0.0;
    for (uint32_t p = 0; p < parts; ++p) {
        const uint32_t lo = (uint32_t)__shfl((int)(uint32_t)s, (int)(2u * p), kWave);
        const uint32_t hi = (uint32_t)__shfl((int)(uint32_t)s, (int)(2u * p + 1u), kWave);
        const double x = __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
        if (take_max) tot = (x > tot || x != x) ? x : tot;
        else tot += x;
    }
    return tot;
}

struct LdsPlan {                 // where things live in the workgroup's LDS
    const float2* cell;          // cell table; an entry's second word is the LDS address of a level row
    const unsigned char* lev;    // level rows, two sign halves, lev_stride bytes apart
    uint32_t lev_addr;           // LDS byte address of the level rows (the cell table sits at address 0)
    uint32_t lev_stride, sign_shift;
    uint32_t cell_shift;         // bits of u >> cell_shift = cell number + cell_key0
    uint32_t cell_key0;          // key of the first cell (everything below goes there too)
};

// tau(u) by the general route: start at the cell's lower level and walk up; returns the byte offset
// of row j in the level table.
__device__ __forceinline__ uint32_t level_row_general(const LdsPlan& L, float u, uint32_t n_sym)
{
    const float um = fminf(fmaxf(u, __uint_as_float(L.cell_key0 << L.cell_shift)), 1.0f);
    const float2 c = L.cell[(__float_as_uint(um) >> L.cell_shift) - L.cell_key0];
    uint32_t j = (__float_as_uint(c.y) - L.lev_addr) >> 4;
    while (j + 2 < n_sym && reinterpret_cast<const float4*>(L.lev)[j + 1].x <= u) ++j;
    return j << 4;
}

// One coordinate: the packed code entry E(idx, sign) = bits | length << 16 of q_l(u) with sign.
// FAST: straight-line cell route, valid when u <= 1 up to rounding (so the clamp of u to 1 can be
// left out: at u >= 1 the coordinate rounds up whatever the draw) and no cell holds two levels.
// CM: the cell size as a compile-time constant (mantissa bits per octave), 0 = whatever L says.
template <bool FAST, int CM = 0>
__device__ __forceinline__ uint32_t quantize_one(float x, float rinv, uint32_t rnd, const LdsPlan& L, uint32_t n_sym,
                                                 uint32_t& idx_out)
{
    float u = fabsf(x) * rinv;                          // |v| / ||v||
    // the sign selects the table half (by constants where the cell size is one)
    const uint32_t sg = CM != 0 ? (__float_as_uint(x) >> lev_sign_shift_of(CM)) & lev_stride_of(CM)
                                : (__float_as_uint(x) >> L.sign_shift) & L.lev_stride;
    float4 t;
    uint32_t row;                                       // byte offset of the level row in its half
    if (FAST) {
        // cell number times eight; a saturating subtraction sends everything below the first cell there
        uint32_t key8;
        if constexpr (CM != 0) {
            constexpr uint32_t shift = 23u - CM, key0 = (uint32_t)(127 - kCellOct) << CM;
            key8 = (__builtin_elementwise_sub_sat(__float_as_uint(u), key0 << shift) >> (shift - 3u)) & 0xFFF8u;
            static_assert(((uint32_t)((kCellOct << CM) + 1) * 8u) <= 0x10000u, "cell numbers times eight fit 16 bits");
        } else {
            key8 = (__builtin_elementwise_sub_sat(__float_as_uint(u), L.cell_key0 << L.cell_shift) >> (L.cell_shift - 3u)) & ~7u;
        }
        const uint2 c = lds_load_u2(key8);          // the cell table starts at LDS address 0 (checked at entry)
        // the cell's lower row, or the next one from the boundary level on (one level per cell at most)
        const uint32_t at = sg + c.y + (u >= __uint_as_float(c.x) ? 16u : 0u);
        t = lds_load_f4(at);
        row = (at - L.lev_addr) & ((CM != 0 ? lev_stride_of(CM) : L.lev_stride) - 1u);
    } else {
        u = fminf(u, 1.0f);
        row = level_row_general(L, u, n_sym);
        t = *reinterpret_cast<const float4*>(L.lev + (row | sg));
    }
    // up with probability xi = (u - l_j) / (l_{j+1} - l_j):  r * gap < u - l_j, r = top 24 bits * 2^-24
    const float rr = (float)(rnd >> 8);                 // exact
    const bool up = rr * t.y < u - t.x;                 // t.y = gap * 2^-24 (exact scaling)
    idx_out = (row >> 4) + (up ? 1u : 0u);
    return up ? __float_as_uint(t.w) : __float_as_uint(t.z);
}

// Appends one row (four entries per lane) to the wave's staging buffer; returns the row's bit count.
// sub_mine: where the lane's run of this row ends in the sub-chunk table, written by the run's last
// lane (ends_run); both are the caller's so that they are worked out once per chunk, not per row.
__device__ __forceinline__ uint32_t pack_row(uint32_t* stage, uint16_t* sub_mine, bool ends_run, uint32_t row_base,
                                             const uint32_t (&e)[4])
{
    const uint32_t l0 = e[0] >> 16, l1 = e[1] >> 16, l2 = e[2] >> 16, l3 = e[3] >> 16;
    const uint32_t c01 = (e[0] & 0xFFFFu) | ((e[1] & 0xFFFFu) << l0);     // <= 28 bits
    const uint32_t c23 = (e[2] & 0xFFFFu) | ((e[3] & 0xFFFFu) << l2);
    const uint32_t l01 = l0 + l1, len = l01 + l2 + l3;
    const uint64_t bits = (uint64_t)c01 | ((uint64_t)c23 << l01);         // <= 56 bits
    const uint32_t incl = wave_incl_scan(len);
    const uint32_t pos = row_base + incl - len;
    const uint32_t wi = pos >> 5, sh = pos & 31u;
    const uint64_t lo64 = (uint64_t)(uint32_t)bits << sh;
    const uint64_t hi64 = (uint64_t)(uint32_t)(bits >> 32) << sh;
    __hip_atomic_fetch_or(&stage[wi], (uint32_t)lo64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    __hip_atomic_fetch_or(&stage[wi + 1], (uint32_t)(lo64 >> 32) | (uint32_t)hi64, __ATOMIC_RELAXED,
                          __HIP_MEMORY_SCOPE_WORKGROUP);
    __hip_atomic_fetch_or(&stage[wi + 2], (uint32_t)(hi64 >> 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    if (ends_run) *sub_mine = (uint16_t)(row_base + incl);                      // a sub-chunk is eight lanes of a row
    return (uint32_t)__builtin_amdgcn_readlane((int)incl, kWave - 1);
}

struct ChunkGeom {            // one wave's share of a bucket
    uint32_t c;               // chunk number
    uint32_t clo, clen, cend; // first coordinate, length, one past the last
    int nrows;                // rows of 256 coordinates that hold data
    bool full;                // all 4096 coordinates present
    uint32_t bparts;          // workgroups that share the bucket (groups of four chunks that hold data)
};

__device__ __forceinline__ ChunkGeom chunk_geom(const Layout& lay, uint32_t b, int w)
{
    uint32_t lo, hi, c0;
    if (lay.uniform_bucket) {                      // one segment: no table look-ups on the critical path
        lo = b * lay.uniform_bucket;
        hi = min(lo + lay.uniform_bucket, lay.d);
        c0 = b * lay.waves_per_bucket;
    } else {
        lo = lay.bucket_start[b]; hi = lay.bucket_start[b + 1]; c0 = lay.bucket_chunk0[b];
    }
    ChunkGeom g;
    g.c = c0 + (uint32_t)w;
    g.clo = lo + (uint32_t)w * kChunk;
    g.clen = g.clo < hi ? min((uint32_t)kChunk, hi - g.clo) : 0u;
    g.cend = g.clo + g.clen;
    g.nrows = (int)((g.clen + 255u) >> 8);
    g.full = g.clen == (uint32_t)kChunk;
    g.bparts = ((hi - lo + (uint32_t)kChunk - 1u) / (uint32_t)kChunk + 3u) >> 2;
    return g;
}

// Issues the loads of one chunk into registers (16 rows x 4 coordinates per lane).
__device__ __forceinline__ void load_chunk(float4 (&v)[kRows], const float* __restrict__ Vk, const ChunkGeom& g,
                                           bool vec_ok, int lane)
{
    if (g.full && vec_ok) {
#pragma unroll
        for (int r = 0; r < kRows; ++r)
            v[r] = nt_load4(Vk + g.clo + (uint32_t)r * 256u + (uint32_t)lane * 4u);
    } else {
#pragma unroll
        for (int r = 0; r < kRows; ++r) {
            const uint32_t i0 = g.clo + (uint32_t)r * 256u + (uint32_t)lane * 4u;
            float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
            if (i0 < g.cend) x.x = Vk[i0];
            if (i0 + 1 < g.cend) x.y = Vk[i0 + 1];
            if (i0 + 2 < g.cend) x.z = Vk[i0 + 2];
            if (i0 + 3 < g.cend) x.w = Vk[i0 + 3];
            v[r] = x;
        }
    }
}

// Shared chunks (buckets of 256..2048 coordinates): a wave's chunk holds up to 16 buckets, each a run
// of whole rows, so the wave works out their norms by itself, one wave reduction at the last row of
// every bucket, and leaves 1 / norm (0 for a bucket that is all zero or rejected) in LDS for the
// rounding pass.  Returns whether the straight-line rounding path applies to the whole chunk: every
// bucket live and no coordinate above its norm.
template <EncMode MODE>
__device__ __forceinline__ bool shared_chunk_norms(const float4 (&v)[kRows], const float* __restrict__ Vk,
                                                   const ChunkGeom& g, const Layout& lay, const EncodeArgs& a,
                                                   Scalars* sc, uint32_t k, uint32_t bucket0, float* rinv_out, int lane)
{
    const uint32_t bshift = lay.bucket_shift, rshift = bshift - 8u;
    const uint32_t rows_mask = (1u << rshift) - 1u;
    const bool l2 = a.norm_kind == QGX_NORM_L2;
    bool plain = true;
    float p0 = 0.0f, p1 = 0.0f, p2 = 0.0f, p3 = 0.0f;
    uint32_t mx = 0;
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        if (l2) {
            p0 = fmaf(v[r].x, v[r].x, p0);
            p1 = fmaf(v[r].y, v[r].y, p1);
            p2 = fmaf(v[r].z, v[r].z, p2);
            p3 = fmaf(v[r].w, v[r].w, p3);
        } else {
            mx = max(mx, __float_as_uint(v[r].x) & 0x7FFFFFFFu);
            mx = max(mx, __float_as_uint(v[r].y) & 0x7FFFFFFFu);
            mx = max(mx, __float_as_uint(v[r].z) & 0x7FFFFFFFu);
            mx = max(mx, __float_as_uint(v[r].w) & 0x7FFFFFFFu);
        }
        if ((((uint32_t)r + 1u) & rows_mask) != 0u) continue;             // wave-uniform: the bucket goes on
        const uint32_t gb = (uint32_t)r >> rshift;
        const uint32_t lo = g.clo + (gb << bshift);
        if (lo < g.cend) {
            const uint32_t hi = min(lo + (1u << bshift), g.cend);
            double tot;
            if (l2) {
                tot = wave_sum(((double)p0 + (double)p1) + ((double)p2 + (double)p3));
                if (!(tot >= 0x1p-60 && tot <= 0x1p100)) {                // as in the kernel: redo in binary64
                    double acc = 0.0;
#pragma unroll 1
                    for (uint32_t i = lo + (uint32_t)lane; i < hi; i += kWave) acc = fma((double)Vk[i], (double)Vk[i], acc);
                    tot = wave_sum(acc);
                }
            } else {
                uint32_t m = mx;
#pragma unroll
                for (int off = kWave / 2; off > 0; off >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, off, kWave));
                tot = (double)__uint_as_float(m);
            }
            float n = l2 ? (float)sqrt(tot) : (float)tot;
            if (!l2 && a.norm_kind != QGX_NORM_LINF && tot > 0.0 && tot <= 3.402823466e+38) {
                const double inv_m = 1.0 / tot;
                double acc = 0.0;
#pragma unroll 1
                for (uint32_t i = lo + (uint32_t)lane; i < hi; i += kWave)
                    acc += pow_int(fabs((double)Vk[i]) * inv_m, (uint32_t)a.norm_kind);
                n = (float)(tot * root_int(wave_sum(acc), (uint32_t)a.norm_kind));
            }
            bool u_le_1 = true;
            if (a.norms_in) {
                const float forced = a.norms_in[(size_t)k * lay.NB + bucket0 + gb];
                u_le_1 = forced >= n;
                n = (n == n && fabsf(n) <= 3.402823466e+38f) ? forced : n;
            }
            const bool bucket_bad = !(fabsf(n) <= 3.402823466e+38f);
            if (bucket_bad) n = 0.0f;
            const bool live = n > 0.0f;
            if (lane == 0) {
                if (bucket_bad) raise_error(sc, QGX_EBIT_NONFINITE);
                if (a.norms_out) a.norms_out[(size_t)k * lay.NB + bucket0 + gb] = n;
                rinv_out[gb] = live ? 1.0f / n : 0.0f;                    // one IEEE division per bucket
            }
            plain = plain && live && u_le_1;
        }
        p0 = p1 = p2 = p3 = 0.0f;
        mx = 0;
    }
    return plain;
}

// One workgroup per (worker, bucket).  Workgroups are short-lived on purpose: with five of them per
// compute unit at different points of their life, the load, ticket and look-back latencies of one
// overlap the arithmetic of the others (a persistent, lock-stepped variant measured slower).
// GROUPED: the layout has shared chunks; a workgroup is four waves with a chunk each, and every wave
// finds the norms of its chunk's buckets by itself.
// CM: cell_mant of the level table, so that the rounding pass has the cell size as a constant.
template <EncMode MODE, bool GROUPED, int CM>
__global__ __launch_bounds__(GROUPED ? 256 : 1024) __attribute__((amdgpu_waves_per_eu(5)))
void k_encode(Layout lay, const Tables* __restrict__ tab, Scalars* sc, EncodeArgs a)
{
    extern __shared__ __align__(16) unsigned char s_all[];
    const int tid = (int)threadIdx.x, lane = lane_id(), w = wave_id();
    const int nwaves = (int)(blockDim.x >> 6);
    const uint32_t n_sym = tab->n_sym;
    const uint32_t k = (uint32_t)blockIdx.x % lay.K;    // worker fixed by the block, buckets by ticket

    // LDS plan: [cell][lev + / lev -][reduction scratch][one staging buffer per wave]
    float2* s_cell = reinterpret_cast<float2*>(s_all);
    const int n_cells = cell_count((int)a.cell_mant);
    unsigned char* s_lev = s_all + cell_count_padded((int)a.cell_mant) * sizeof(float2);
    double* s_red = reinterpret_cast<double*>(s_lev + a.lev_bytes);
    double* s_tot = s_red + 2 * nwaves;                                       // second set: the general-q sum
    uint32_t* s_words = reinterpret_cast<uint32_t*>(s_tot + 2);               // bucket totals of a split bucket
    uint32_t* s_misc = s_words + (nwaves + 3) / 4 * 4;
    float* s_rinv = reinterpret_cast<float*>(reinterpret_cast<unsigned char*>(s_misc) + 32);      // GROUPED: [waves][16]
    uint32_t* stage = reinterpret_cast<uint32_t*>(reinterpret_cast<unsigned char*>(s_misc) + 32 +
                                                  (GROUPED ? (size_t)nwaves * 64 : 0) + (size_t)w * a.stage_bytes);
    LdsPlan L;
    L.cell = s_cell; L.lev = s_lev; L.lev_stride = a.lev_stride; L.sign_shift = a.sign_shift;
    L.lev_addr = lds_address(s_lev);
    L.cell_shift = 23u - a.cell_mant;
    L.cell_key0 = (uint32_t)(127 - kCellOct) << a.cell_mant;
    // The straight-line lookup addresses the cell table by number: the kernel has no static LDS, so
    // the dynamic array (and with it the table) starts at address 0.
    if (lds_address(s_all) != 0u) {
        if (tid == 0) raise_error(sc, QGX_EBIT_STATE);
        return;
    }

    // Compact placement: buckets by ticket (the ticket first: the table loads overlap its latency).
    // Slotted placement and plain quantisation have no order to keep: the bucket is the block's own.
    // Split buckets: (bucket, part) by ticket as well, whatever the placement (see exchange_parts).
    const bool ordered = MODE != EncMode::QuantOnly && a.slot_words == 0u;
    const bool ticketed = ordered || a.parts > 1u;
    // A worker's counter only ever grows, and every launch of a context that takes tickets takes the
    // same number from it, so a ticket tells both the unit inside this launch and the number of the
    // launch, which tags what the workgroups publish to each other (30 bits, never 0: untouched
    // words hold 0).  Nothing about it comes from the host: a captured graph can be replayed.
    if (ticketed) {
        if (tid == 0) {
            const unsigned long long per_launch = GROUPED ? (lay.NC + 3u) / 4u : (unsigned long long)lay.NB * a.parts;
            const unsigned long long raw = atomicAdd(a.tickets + k * kTicketStride, 1ull);
            const unsigned long long launch = raw / per_launch;
            s_misc[2] = (uint32_t)(raw - launch * per_launch);
            s_misc[3] = (uint32_t)(launch % 0x3FFFFFFFull) + 1u;
        }
    }
    for (int i = tid; i < (int)n_sym; i += (int)blockDim.x) {
        reinterpret_cast<float4*>(s_lev)[i] = tab->lev2[0][i];
        reinterpret_cast<float4*>(s_lev + a.lev_stride)[i] = tab->lev2[1][i];
    }
    for (int i = tid; i < n_cells; i += (int)blockDim.x) {
        float2 c = tab->cell[i];                       // row offset -> LDS address of the row
        c.y = __uint_as_float((__float_as_uint(c.y) & 0xFFFFu) + L.lev_addr);
        s_cell[i] = c;
    }
    if (MODE != EncMode::QuantOnly) {
        for (uint32_t q = (uint32_t)lane; q < a.stage_bytes / 16; q += kWave)
            reinterpret_cast<uint4*>(stage)[q] = make_uint4(0, 0, 0, 0);
    }
    // (the table builder and the host take the cell size from the table's length by the same rule)
    const uint32_t cell_exact = (tab->cell_exact != 0u && (uint32_t)cell_mant(n_sym) == a.cell_mant) ? 1u : 0u;
    __syncthreads();

    const size_t kbase = (size_t)k * lay.d;
    const bool vec_ok = MODE == EncMode::Generate || (kbase & 3u) == 0;    // 16-byte aligned rows for this worker
    // the number of this quantisation call: given, or taken from the iteration counter (replayed graphs)
    const uint32_t call_id = a.call_mode ? 2u * (uint32_t)(sc->t - 1ull) + (a.call_mode - 1u) : a.call_id;
    const float* __restrict__ Vk = (MODE == EncMode::Fused || MODE == EncMode::QuantOnly) ? a.V + kbase : nullptr;
    // one coordinate of the worker's vector again, for the rolled paths: from memory, or (Generate) formed again
    auto value_at = [&](uint32_t i) -> float {
        if constexpr (MODE == EncMode::Generate) {
            const float4 row = game_dual_row(a.game, i & ~3u, k, call_id);
            const uint32_t q = i & 3u;
            return q == 0u ? row.x : q == 1u ? row.y : q == 2u ? row.z : row.w;
        } else {
            return Vk[i];
        }
    };
    const uint32_t unit = ticketed ? s_misc[2] : (uint32_t)blockIdx.x / lay.K;
    const uint32_t epoch = ticketed ? s_misc[3] : 0u;
    uint32_t b = a.parts > 1u ? unit / a.parts : unit;  // the bucket; with shared chunks the first of the wave's chunk
    const uint32_t part = GROUPED ? 0u : unit - b * a.parts;
    ChunkGeom g;
    if constexpr (GROUPED) {
        if (unit * 4u >= lay.NC) return;               // cannot happen: one workgroup per four chunks and worker
        g.c = unit * 4u + (uint32_t)w;
        const bool there = g.c < lay.NC;
        g.clo = there ? lay.chunk_start[g.c] : 0u;
        g.clen = there ? lay.chunk_start[g.c + 1] - g.clo : 0u;
        g.cend = g.clo + g.clen;
        g.nrows = (int)((g.clen + 255u) >> 8);
        g.full = g.clen == (uint32_t)kChunk;
        g.bparts = 1u;
        b = there ? lay.chunk_bucket[g.c] : 0u;
    } else {
        if (b >= lay.NB) return;                       // cannot happen: one workgroup per unit and worker
        g = chunk_geom(lay, b, (int)part * 4 + w);
    }
    if (part >= g.bparts) {
        // a short bucket has nothing for this part; no partner waits for it, but in compact placement
        // the units after it look back over its (empty) aggregate
        if (ordered && tid == 0)
            __hip_atomic_store(a.scan_state + (size_t)k * lay.NB * a.parts + unit,
                               (unsigned long long)((epoch << 2) | 1u) << 32, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return;
    }
    const bool split = a.parts > 1u && g.bparts > 1u;
    unsigned long long* xch = a.xch + ((size_t)k * lay.NB + b) * a.parts * 4u;
    // The sub-chunk ends go straight to the table in global memory (eight lanes of a row write one
    // 16-byte piece): staging them in LDS would cost the fifth workgroup of a compute unit.
    uint16_t* __restrict__ sub_g =
        MODE != EncMode::QuantOnly ? a.sub_end + ((size_t)k * lay.NC + g.c) * kSubs : nullptr;
    uint16_t* __restrict__ sub_mine = sub_g + (lane >> 3);
    const bool ends_run = (lane & 7) == 7;
    float4 v[kRows];
    if constexpr (MODE == EncMode::Generate) {
        // the dual vector is formed here instead of read: operator and noise for four coordinates per lane and row
        // (every bucket and vector length is a multiple of four in this mode)
#pragma unroll
        for (int r = 0; r < kRows; ++r) {
            const uint32_t i0 = g.clo + (uint32_t)r * 256u + (uint32_t)lane * 4u;
            float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
            if (i0 < g.cend) {
                x = game_dual_row(a.game, i0, k, call_id);
                if (a.game.V_out) *reinterpret_cast<float4*>(a.game.V_out + kbase + i0) = x;
            }
            v[r] = x;
        }
    } else if (MODE != EncMode::EncodeOnly) {
        load_chunk(v, Vk, g, vec_ok, lane);
    }
    {

        // ---- norm of the bucket from the rows in registers ---------------------------------------
        float n = 0.0f;
        bool u_le_1 = true;
        bool plain = true;                             // GROUPED: every bucket of the chunk live, no u above 1
        if constexpr (GROUPED) {
            if (MODE != EncMode::EncodeOnly && g.clen != 0u)
                plain = shared_chunk_norms<MODE>(v, Vk, g, lay, a, sc, k, b, s_rinv + w * 16, lane);
            wave_lds_fence();                              // lane 0 left the buckets' 1 / norm for all lanes
        } else if (MODE != EncMode::EncodeOnly) {
            // A non-finite coordinate shows in the reduced value itself (a sum of squares with a NaN
            // or an infinity in it, a maximum taken on magnitude bits).
            double red;
            if (a.norm_kind == QGX_NORM_L2) {
                // four binary32 runs of 16 fused multiply-adds per lane (error of a run at most
                // 15 roundings, 1e-6 relative, half of that on the norm), everything after in
                // binary64; sums outside the range where binary32 squares are safe are redone below
                float p0 = 0.0f, p1 = 0.0f, p2 = 0.0f, p3 = 0.0f;
#pragma unroll
                for (int r = 0; r < kRows; ++r) {
                    p0 = fmaf(v[r].x, v[r].x, p0);
                    p1 = fmaf(v[r].y, v[r].y, p1);
                    p2 = fmaf(v[r].z, v[r].z, p2);
                    p3 = fmaf(v[r].w, v[r].w, p3);
                }
                red = wave_sum(((double)p0 + (double)p1) + ((double)p2 + (double)p3));
            } else {
                uint32_t mx = 0;
#pragma unroll
                for (int r = 0; r < kRows; ++r) {
                    mx = max(mx, __float_as_uint(v[r].x) & 0x7FFFFFFFu);
                    mx = max(mx, __float_as_uint(v[r].y) & 0x7FFFFFFFu);
                    mx = max(mx, __float_as_uint(v[r].z) & 0x7FFFFFFFu);
                    mx = max(mx, __float_as_uint(v[r].w) & 0x7FFFFFFFu);
                }
#pragma unroll
                for (int off = kWave / 2; off > 0; off >>= 1) mx = max(mx, (uint32_t)__shfl_xor((int)mx, off, kWave));
                red = (double)__uint_as_float(mx);      // inf or NaN bits survive the conversion
            }
            if (lane == 0) s_red[w] = red;
            __syncthreads();
            double tot = 0.0;
            for (int i = 0; i < nwaves; ++i) {
                if (a.norm_kind == QGX_NORM_L2) tot += s_red[i];
                else tot = (s_red[i] > tot || s_red[i] != s_red[i]) ? s_red[i] : tot;
            }
            if (split) {
                if (w == 0) {
                    const double t = exchange_parts(xch, g.bparts, part, 0u, tot, a.norm_kind != QGX_NORM_L2, epoch, sc);
                    if (lane == 0) s_tot[0] = t;
                }
                __syncthreads();
                tot = s_tot[0];
            }
            if (a.norm_kind == QGX_NORM_L2 && !(tot >= 0x1p-60 && tot <= 0x1p100)) {
                // squares that overflow or go subnormal in binary32 (or a non-finite input): the sum
                // again in binary64, from memory (the rolled loop keeps the register copy intact)
                double acc = 0.0;
#pragma unroll 1
                for (uint32_t i = g.clo + (uint32_t)lane; i < g.cend; i += kWave) { const double x = (double)value_at(i); acc = fma(x, x, acc); }
                acc = wave_sum(acc);
                if (lane == 0) s_red[nwaves + w] = acc;
                __syncthreads();
                tot = 0.0;
                for (int i = 0; i < nwaves; ++i) tot += s_red[nwaves + i];
                if (split) {
                    if (w == 0) {
                        const double t = exchange_parts(xch, g.bparts, part, 1u, tot, false, epoch, sc);
                        if (lane == 0) s_tot[1] = t;
                    }
                    __syncthreads();
                    tot = s_tot[1];
                }
            }
            n = (a.norm_kind == QGX_NORM_L2) ? (float)sqrt(tot) : (float)tot;
            if (a.norm_kind != QGX_NORM_L2 && a.norm_kind != QGX_NORM_LINF && tot > 0.0 && tot <= 3.402823466e+38) {
                // any other q of Definition 1: (sum |v_i|^q)^(1/q), relative to the largest magnitude
                // found above so that no power leaves the range of binary64
                const double inv_m = 1.0 / tot;
                const uint32_t q = (uint32_t)a.norm_kind;
                double acc = 0.0;
                // (a rolled loop over memory: indexing the register copy by a run-time row would
                // push it out of registers for the common norms as well)
#pragma unroll 1
                for (uint32_t i = g.clo + (uint32_t)lane; i < g.cend; i += kWave)
                    acc += pow_int(fabs((double)value_at(i)) * inv_m, q);
                acc = wave_sum(acc);
                if (lane == 0) s_red[nwaves + w] = acc;
                __syncthreads();
                double sum = 0.0;
                for (int i = 0; i < nwaves; ++i) sum += s_red[nwaves + i];
                if (split) {
                    if (w == 0) {
                        const double t = exchange_parts(xch, g.bparts, part, 1u, sum, false, epoch, sc);
                        if (lane == 0) s_tot[1] = t;
                    }
                    __syncthreads();
                    sum = s_tot[1];
                }
                n = (float)(tot * root_int(sum, q));
            }
            if (a.norms_in) {
                const float forced = a.norms_in[(size_t)k * lay.NB + b];
                u_le_1 = forced >= n;                                        // else |v| / norm may exceed 1
                n = (n == n && fabsf(n) <= 3.402823466e+38f) ? forced : n;   // a poisoned bucket stays rejected
            }
            const bool bucket_bad = !(fabsf(n) <= 3.402823466e+38f);
            if (bucket_bad) n = 0.0f;
            if (tid == 0) {
                if (bucket_bad) raise_error(sc, QGX_EBIT_NONFINITE);
                if (a.norms_out && part == 0u) a.norms_out[(size_t)k * lay.NB + b] = n;
            }
        }
        const float rinv = GROUPED ? 0.0f : 1.0f / n;  // one IEEE division per bucket
        const bool live = GROUPED ? plain : n > 0.0f;
        const bool fast = g.full && live && vec_ok && u_le_1 && (cell_exact != 0u) && MODE != EncMode::EncodeOnly;
        const uint32_t rshift = GROUPED ? lay.bucket_shift - 8u : 0u;         // rows per bucket, as a shift

        // ---- per row: quantise, code, pack -------------------------------------------------------
        uint32_t row_base = 0;                         // bits of this chunk written so far (wave-uniform)
        if (fast) {
#pragma unroll
            for (int r = 0; r < kRows; ++r) {
                const uint32_t i0 = g.clo + (uint32_t)r * 256u + (uint32_t)lane * 4u;
                uint32_t rnd[4], e[4], idx[4];
                philox4x32_10(i0 >> 2, 0u, k, call_id, a.seed_lo, a.seed_hi, rnd);
                const float rinv_r = GROUPED ? s_rinv[w * 16 + (int)((uint32_t)r >> rshift)] : rinv;
                e[0] = quantize_one<true, CM>(v[r].x, rinv_r, rnd[0], L, n_sym, idx[0]);
                e[1] = quantize_one<true, CM>(v[r].y, rinv_r, rnd[1], L, n_sym, idx[1]);
                e[2] = quantize_one<true, CM>(v[r].z, rinv_r, rnd[2], L, n_sym, idx[2]);
                e[3] = quantize_one<true, CM>(v[r].w, rinv_r, rnd[3], L, n_sym, idx[3]);
                if (MODE == EncMode::QuantOnly) {
                    uint32_t pk = 0;
                    const float xs[4] = {v[r].x, v[r].y, v[r].z, v[r].w};
#pragma unroll
                    for (int q = 0; q < 4; ++q) pk |= (idx[q] | ((__float_as_uint(xs[q]) >> 31) << 7)) << (8 * q);
                    *reinterpret_cast<uint32_t*>(a.sym_out + kbase + i0) = pk;
                } else {
                    row_base += pack_row(stage, sub_mine + 8 * r, ends_run, row_base, e);
                }
            }
        } else {
#pragma unroll 1
            for (int r = 0; r < g.nrows; ++r) {
                const uint32_t i0 = g.clo + (uint32_t)r * 256u + (uint32_t)lane * 4u;
                uint32_t e[4], idx[4], neg[4];
                if (MODE == EncMode::EncodeOnly) {
                    const uint8_t* __restrict__ Sk = a.sym_in + kbase;
                    bool unknown = false;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const uint32_t by = (i0 + (uint32_t)q < g.cend) ? (uint32_t)Sk[i0 + q] : 0u;
                        idx[q] = by & 0x7Fu;
                        neg[q] = by >> 7;
                        if (idx[q] >= n_sym) { idx[q] = 0; unknown = true; }
                    }
                    if (__any(unknown) && lane == 0) raise_error(sc, QGX_EBIT_STREAM);
                } else {
                    uint32_t rnd[4];
                    philox4x32_10(i0 >> 2, 0u, k, call_id, a.seed_lo, a.seed_hi, rnd);
                    // the register copy is indexed by compile-time row numbers only: this path reads the row again
                    float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
                    if constexpr (MODE == EncMode::Generate) {
                        if (i0 < g.cend) x = game_dual_row(a.game, i0, k, call_id);
                    } else {
                        if (i0 < g.cend) x.x = Vk[i0];
                        if (i0 + 1 < g.cend) x.y = Vk[i0 + 1];
                        if (i0 + 2 < g.cend) x.z = Vk[i0 + 2];
                        if (i0 + 3 < g.cend) x.w = Vk[i0 + 3];
                    }
                    const float xs[4] = {x.x, x.y, x.z, x.w};
                    const float rinv_r = GROUPED ? s_rinv[w * 16 + (int)((uint32_t)r >> rshift)] : rinv;
                    const bool live_r = GROUPED ? rinv_r != 0.0f : live;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        idx[q] = 0;
                        neg[q] = __float_as_uint(xs[q]) >> 31;
                        if (live_r) (void)quantize_one<false>(xs[q], rinv_r, rnd[q], L, n_sym, idx[q]);
                    }
                }
                if (MODE == EncMode::QuantOnly) {
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        if (i0 + (uint32_t)q < g.cend) a.sym_out[kbase + i0 + q] = (uint8_t)(idx[q] | (neg[q] << 7));
                } else {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        // E(idx, sign) from the table row of idx (its third word), nothing for a padded slot
                        const float4 t = *reinterpret_cast<const float4*>(s_lev + idx[q] * 16u + neg[q] * a.lev_stride);
                        e[q] = (i0 + (uint32_t)q < g.cend) ? __float_as_uint(t.z) : 0u;
                    }
                    row_base += pack_row(stage, sub_mine + 8 * r, ends_run, row_base, e);
                }
            }
        }

        // ---- sizes, ordered offsets, flush ---------------------------------------------------------
        const uint32_t total_bits = row_base;
        uint32_t words = (total_bits + 31u) >> 5;
        words = (words + (kAlignWords - 1)) & ~(uint32_t)(kAlignWords - 1);
        if (MODE != EncMode::QuantOnly) {
            if (g.clen != 0) {
                for (int j = lane; j < kSubs; j += kWave)
                    if (j >= 8 * g.nrows) sub_g[j] = (uint16_t)total_bits;
            }
            if (lane == 0 && ordered) s_words[w] = words;
        }
        if (MODE != EncMode::QuantOnly) {
            uint32_t off;
            if (ordered) {
                __syncthreads();
                uint32_t bucket_words = 0, wave_excl = 0;
                for (int i = 0; i < nwaves; ++i) {
                    if (i == w) wave_excl = bucket_words;
                    bucket_words += s_words[i];
                }
                if (w == 0) {
                    const uint32_t excl = lookback_exclusive(a.scan_state + (size_t)k * lay.NB * a.parts, unit, bucket_words, epoch, sc);
                    if (lane == 0) s_misc[1] = excl;
                }
                __syncthreads();
                off = s_misc[1] + wave_excl;
            } else {
                off = g.c * a.slot_words;
            }
            if (g.clen != 0) {
                if (lane == 0) {
                    a.chunk_off[(size_t)k * (lay.NC + 1) + g.c] = off;
                    if (g.c + 1 == lay.NC) a.chunk_off[(size_t)k * (lay.NC + 1) + lay.NC] = off + (ordered ? words : a.slot_words);
                }
                if ((uint64_t)off + words > a.cap_words) {
                    if (lane == 0) raise_error(sc, QGX_EBIT_CAPACITY);
                } else {
                    uint4* __restrict__ dst = reinterpret_cast<uint4*>(a.payload + (size_t)k * a.cap_words + off);
                    uint4* src = reinterpret_cast<uint4*>(stage);
                    wave_lds_fence();                          // a lane stores words that all lanes' codes went into
                    for (uint32_t q = (uint32_t)lane; q < (words >> 2); q += kWave) dst[q] = src[q];
                }
            }
        }
    }
}

static size_t encode_lds_bytes(int waves, const EncodeArgs& a, bool with_stage, bool grouped)
{
    size_t n = cell_count_padded((int)a.cell_mant) * sizeof(float2) + (size_t)a.lev_bytes + (grouped ? (size_t)waves * 64 : 0) +
               (2 * (size_t)waves + 2) * sizeof(double) + (size_t)(waves + 3) / 4 * 4 * sizeof(uint32_t) + 32;
    if (with_stage) n += (size_t)waves * a.stage_bytes;
    return n;
}

template <EncMode MODE, bool GROUPED, int CM>
static hipError_t launch_mode(const Layout& lay, const Tables* tab, Scalars* sc, const EncodeArgs& a, hipStream_t st)
{
    const int waves = (GROUPED || a.parts > 1u) ? 4 : (int)lay.waves_per_bucket;
    const size_t lds = encode_lds_bytes(waves, a, MODE != EncMode::QuantOnly, GROUPED);
    static LdsLimit limit;
    hipError_t e = limit.ensure(reinterpret_cast<const void*>(&k_encode<MODE, GROUPED, CM>), 160 * 1024);
    if (e != hipSuccess) return e;
    // one workgroup per bucket, per part of a bucket, or (shared chunks) per four chunks; in compact
    // placement and with split buckets each takes one ticket of its worker (the kernel's per_launch)
    const uint32_t units = GROUPED ? (lay.NC + 3u) / 4u : lay.NB * a.parts;
    hipLaunchKernelGGL((k_encode<MODE, GROUPED, CM>), dim3(lay.K * units), dim3(waves * kWave), lds, st, lay, tab, sc, a);
    return hipGetLastError();
}

template <EncMode MODE>
static hipError_t launch_kind(const Layout& lay, const Tables* tab, Scalars* sc, const EncodeArgs& a, hipStream_t st)
{
    switch (a.cell_mant) {
        case 4: return lay.shared_chunks ? launch_mode<MODE, true, 4>(lay, tab, sc, a, st)
                                         : launch_mode<MODE, false, 4>(lay, tab, sc, a, st);
        case 5: return lay.shared_chunks ? launch_mode<MODE, true, 5>(lay, tab, sc, a, st)
                                         : launch_mode<MODE, false, 5>(lay, tab, sc, a, st);
        default: return lay.shared_chunks ? launch_mode<MODE, true, 6>(lay, tab, sc, a, st)
                                          : launch_mode<MODE, false, 6>(lay, tab, sc, a, st);
    }
}

hipError_t launch_encode(EncMode mode, const Layout& lay, const Tables* tab, Scalars* sc, const EncodeArgs& a,
                         hipStream_t st)
{
    switch (mode) {
        case EncMode::Fused: return launch_kind<EncMode::Fused>(lay, tab, sc, a, st);
        case EncMode::Generate:
            if (lay.shared_chunks) return hipErrorInvalidValue;          // (the host side has refused this layout)
            switch (a.cell_mant) {
                case 4: return launch_mode<EncMode::Generate, false, 4>(lay, tab, sc, a, st);
                case 5: return launch_mode<EncMode::Generate, false, 5>(lay, tab, sc, a, st);
                default: return launch_mode<EncMode::Generate, false, 6>(lay, tab, sc, a, st);
            }
        case EncMode::QuantOnly: return launch_kind<EncMode::QuantOnly>(lay, tab, sc, a, st);
        default: return launch_kind<EncMode::EncodeOnly>(lay, tab, sc, a, st);
    }
}

}  // namespace qgx
