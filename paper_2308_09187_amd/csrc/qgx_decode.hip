// DEQ o CODE and everything fused onto it: plain decode, the mean over K workers, and the two
// extra-gradient half-steps with the step-size accumulator.
// (Section 3.2 / Appendix J for the decoding; Algorithm 1 and eq. (Q-GenX) for the updates;
// Theorem 3 for gamma_t.)
//
// One wave per chunk position.  The wave copies a worker's chunk from the payload into LDS with
// coalesced 16-byte loads, then every lane parses its own 64 coordinates, that is two sub-chunks of
// 32, each starting at the bit offset the sub-chunk table gives: a 64-bit window from three LDS words
// per three symbols, one table look-up by the next 13 (or 11) stream bits for each symbol's length and
// level, the sign bit, one multiply by the bucket norm.  A symbol's length decides where the next one
// starts, so a parse is one long dependent chain of LDS look-ups; what a lane can do about that is to
// follow several chains at once: its two sub-chunks, of one stream or (second half-step) of both.
// The K decoded values of a coordinate are summed in registers, so decoded vectors never go to HBM in
// the fused modes.  Chunk positions with fewer than 4096 coordinates are few and have a body of their
// own (decode_ragged_body), which spreads a position's workers over the waves of a workgroup; it runs
// in the same launch as the full positions' body when a layout has both.
#include "qgx_device.h"

namespace qgx {

constexpr int kPre = kChunkWordsMax / (kWave * 4);   // 7 x uint4 per lane cover a worst-case chunk
constexpr int kDecWaves = 8;                          // waves per workgroup: they share the decode table

// Staged chunk layout in LDS.  Lane j parses the j-th run of 64 coordinates, whose bits start roughly
// 64 * (bits per coordinate) / 32 words after lane j-1's: a power-of-two stride that would put all
// lanes on a few banks.  So two pad words are inserted after every 32 words (word i lives at
// i + 2 (i / 32)), and the pad slots repeat the two words that follow them, so that a lane always
// finds the three words of its 64-bit window next to each other.
__device__ __forceinline__ uint32_t staged(uint32_t i) { return i + ((i >> 5) << 1); }

struct ChunkRef {            // where one worker's chunk lives and how long it is
    const uint4* src;
    uint32_t words;          // multiple of 4, 0 when the tables are inconsistent
};

// A chunk's size comes from its bit length (last sub-chunk entry), so compact and slotted
// placements read alike; its start comes from the offset table.
__device__ __forceinline__ ChunkRef chunk_ref(const uint32_t* payload, uint64_t cap, const uint32_t* chunk_off,
                                              const uint16_t* sub_end, uint32_t k, uint32_t c, uint32_t NC,
                                              uint32_t max_words, Scalars* sc)
{
    const uint32_t off = chunk_off[(size_t)k * (NC + 1) + c];
    const uint32_t bits = sub_end[((size_t)k * NC + c) * kSubs + (kSubs - 1)];
    ChunkRef r;
    r.src = reinterpret_cast<const uint4*>(payload + (size_t)k * cap + off);
    r.words = (((bits + 31u) >> 5) + 3u) & ~3u;
    if (r.words > max_words || (off & 3u) || (uint64_t)off + r.words > cap) {
        if (lane_id() == 0) raise_error(sc, QGX_EBIT_STREAM);
        r.words = 0;
    }
    return r;
}

__device__ __forceinline__ void prefetch_chunk(const ChunkRef& cr, uint4 (&pre)[kPre])
{
    const uint32_t lane = (uint32_t)lane_id();
#pragma unroll
    for (int q = 0; q < kPre; ++q) {
        const uint32_t i = lane + (uint32_t)q * kWave;
        pre[q] = (i < (cr.words >> 2)) ? nt_load4u(cr.src + i) : make_uint4(0, 0, 0, 0);
    }
}

__device__ __forceinline__ void commit_chunk(uint32_t* stage, const uint4 (&pre)[kPre], uint32_t stage_words)
{
    const uint32_t lane = (uint32_t)lane_id();
#pragma unroll
    for (int q = 0; q < kPre; ++q) {
        const uint32_t i0 = (lane + (uint32_t)q * kWave) * 4u;
        if (i0 < stage_words) {
            uint2* at = reinterpret_cast<uint2*>(stage + staged(i0));          // even slot: 8-byte aligned
            at[0] = make_uint2(pre[q].x, pre[q].y);
            at[1] = make_uint2(pre[q].z, pre[q].w);
            if ((i0 & 31u) == 0u && i0 != 0u) at[-1] = make_uint2(pre[q].x, pre[q].y);   // pads repeat their successors
        }
    }
}

// The chunk back to front, for the parse of the full positions: stream bit t goes to bit
// 32 (kTail + stage_words) - 1 - t of the buffer (word w to place kTail + stage_words - 1 - w, its bits
// turned round), so that a plain funnel shift of buffer words gives a window with the FIRST stream bit on
// top, which is how the decode tables are indexed, and no window has to be turned round when it is read:
// a word is turned once here instead of twice per three symbols there.  kTail zero words lie below the
// chunk's end (the windows of its last symbols reach there), and the buffer's slack above its first word
// stays zero as well (a cursor may point one bit before the chunk).  The pads are as in the forward layout.
// `words`: the chunk's own size; pieces of 256 words that lie beyond it are left as they are (a valid
// stream's symbols never depend on what follows its last bit).
constexpr int kTail = 4;
__device__ __forceinline__ void commit_chunk_reversed(uint32_t* stage, const uint4 (&pre)[kPre], uint32_t stage_words,
                                                      uint32_t words)
{
    static_assert(kTail % 4 == 0 && kChunkWordsMax % 4 == 0, "16-byte pieces stay aligned");
    const uint32_t lane = (uint32_t)lane_id();
#pragma unroll
    for (int q = 0; q < kPre; ++q) {
        if ((uint32_t)q * (kWave * 4u) >= words) break;                       // (wave-uniform)
        const uint32_t i0 = (lane + (uint32_t)q * kWave) * 4u;
        if (i0 < stage_words) {
            const uint32_t j0 = (uint32_t)kTail + stage_words - 4u - i0;      // place of the piece's LAST word
            uint2* at = reinterpret_cast<uint2*>(stage + staged(j0));
            const uint2 low = make_uint2(__brev(pre[q].w), __brev(pre[q].z));
            at[0] = low;
            at[1] = make_uint2(__brev(pre[q].y), __brev(pre[q].x));
            if ((j0 & 31u) == 0u) at[-1] = low;                               // (j0 >= kTail: never the buffer's first word)
        }
    }
}

// LDS tables of the decoder in one array: level values first, then the decode table, so that the
// level index of a reject entry (flag bit set) still lands inside the array.
constexpr int kTabLvalBytes = kSymMax * 4;
constexpr int kTabBytes = kTabLvalBytes + kDlut * 2;

// Symbols are parsed in groups of up to three from one 64-bit window (three LDS words): a symbol
// takes at most 15 bits with its sign, so the third one still starts inside the first word.  A table
// entry is a bit count | 4 idx << 4 with bits 4 and 5 clear (the 13-bit table counts the symbol's bits
// incl. sign less one, the 8-byte table all of them), so sums of entries carry the consumed bits in
// their low six bits and an entry can be used as a shift count as it is.
// The three steps are separate so that the caller can issue the next group's window reads before
// it turns the current group's entries into values.
struct Window { uint32_t w0, w1, w2; };

__device__ __forceinline__ Window read_window(const uint32_t* stage, uint32_t p)
{
    const uint32_t* wp = stage + (p >> 5) + ((p >> 10) << 1);
    return Window{wp[0], wp[1], wp[2]};
}

// The dependent chain: window i needs the lengths of the symbols before it.  Advances the cursor.
// The 64 bits are turned so that the first stream bit is on top: a window is then a funnel shift
// away, its top 13 bits index the table, and a symbol's last bit (the sign) reaches bit 31 by a left
// shift of (symbol bits - 1), which is what the entry's low bits hold.  `neg` counts the used bits
// downwards (adding ~e takes off the entry's count plus one); only its low six bits mean anything.
template <int N>
__device__ __forceinline__ void parse_group(const Window& w, const unsigned char* tab, uint32_t& p,
                                            uint32_t (&win)[3], uint32_t (&e)[3])
{
    const uint32_t top = __brev(__builtin_amdgcn_alignbit(w.w1, w.w0, p));    // shifts use p mod 32
    const uint32_t nxt = __brev(__builtin_amdgcn_alignbit(w.w2, w.w1, p));
    uint32_t neg = 0;
#pragma unroll
    for (int i = 0; i < N; ++i) {
        win[i] = i == 0 ? top : __builtin_amdgcn_alignbit(top, nxt, neg);     // (top:nxt) << used, upper word
        e[i] = *reinterpret_cast<const uint16_t*>(tab + kTabLvalBytes + ((win[i] >> 18) & 0x3FFEu));
        neg += ~e[i];
    }
    p -= neg | 0xFFFFFFC0u;                                                   // minus (minus the bits used)
}

// The same chain for the kernel of the full positions, which stages its chunks back to front
// (commit_chunk_reversed): the cursor r is a bit position in the buffer and moves DOWN, the three words
// from it give the 64 bits with the first stream bit on top by two funnel shifts and nothing else.
// The windows are taken one bit early: r + 63 is the buffer bit of the stream bit BEFORE the next symbol,
// so bit 31 of a symbol's window is the last bit of the symbol before it, which is that symbol's sign
// if it has one.  The sign of a symbol is thus read off the window of the next one with a single
// AND-OR, no shift by its length: W[i + 1] for symbol i, the next group's W[0] for a group's last
// symbol, and for the last group of a run (LAST, two symbols) the window after its second symbol, W[2].
// The table index sits one bit lower (bits 30..20 resp. 30..18).
// `seen` gathers the AND of the groups' (negative) bit counts: a reject entry leaves a zero among bits
// 15..31, valid entries never do, so no per-symbol flag is kept.
// WIDE: the 8-byte table's entries are the negative counts themselves and only need adding up.
template <int N, bool WIDE, bool LAST>
__device__ __forceinline__ void parse_group_early(const Window& w, const unsigned char* tab, uint32_t& r,
                                                  uint32_t (&W)[4], uint32_t (&e)[3], float (&lv)[3], uint32_t& seen)
{
    static_assert(!LAST || N == 2, "a run of 32 symbols ends with a group of two");
    const uint32_t top = __builtin_amdgcn_alignbit(w.w2, w.w1, r);            // shifts use r mod 32
    const uint32_t nxt = __builtin_amdgcn_alignbit(w.w1, w.w0, r);
    uint32_t neg = 0;
#pragma unroll
    for (int i = 0; i < N; ++i) {
        W[i] = i == 0 ? top : __builtin_amdgcn_alignbit(top, nxt, neg);       // (top:nxt) << used, upper word
        if constexpr (WIDE) {
            const uint2 t = *reinterpret_cast<const uint2*>(tab + kTabLvalBytes + ((W[i] >> 17) & 0x3FF8u));
            e[i] = t.x;
            lv[i] = __uint_as_float(t.y);
            neg = i == 0 ? t.x : neg + t.x;
        } else {
            e[i] = *reinterpret_cast<const uint16_t*>(tab + kTabLvalBytes + ((W[i] >> 17) & 0x3FFEu));
            neg += ~e[i];
        }
    }
    if constexpr (LAST) W[N] = __builtin_amdgcn_alignbit(top, nxt, neg);     // at least two bits used: never a shift by 0
    seen &= neg;
    r += neg | 0xFFFFFFC0u;                                                   // down by the bits used
}

// norm with the sign of the symbol whose last bit is bit 31 of `w_next` (norms are not negative)
__device__ __forceinline__ float signed_norm(uint32_t w_next, float n)
{
    return __uint_as_float((w_next & 0x80000000u) | __float_as_uint(n));
}

// +-(norm * level), one binary32 product, sign from the window of the next symbol
// EXACT_ZERO: +0 for the zero symbol, whose sign bit is not in the stream (the level 0 is the only one
// that is zero)
template <bool EXACT_ZERO>
__device__ __forceinline__ float value_early(uint32_t w_next, float lv, float n)
{
    const float val = __uint_as_float((w_next & 0x80000000u) | __float_as_uint(n * lv));
    if (EXACT_ZERO) return lv == 0.0f ? 0.0f : val;
    return val;
}

__device__ __forceinline__ float level_of(const unsigned char* tab, uint32_t e)
{
    return *reinterpret_cast<const float*>(tab + (e >> 4));                  // the entry holds 4 * idx
}

// Signed value norm * l_idx of one parsed symbol, lv = level_of(entry).
// EXACT_ZERO: give +0 for the zero symbol (whose sign bit is not in the stream); the accumulating
// modes leave the stray sign on the zero, which adds nothing.
template <bool EXACT_ZERO>
__device__ __forceinline__ float symbol_value(float lv, uint32_t win, uint32_t e, float n)
{
    const uint32_t sg = win << (e & 31u);                                      // last bit of the symbol -> bit 31
    // norm and level are not negative: the sign goes in with one OR
    const float val = __uint_as_float((sg & 0x80000000u) | __float_as_uint(n * lv));
    if (EXACT_ZERO) return (e >> 4) == 0u ? 0.0f : val;
    return val;
}

struct SubMeta {             // what a lane needs to parse its run of one worker's chunk
    uint32_t p0, p_end;      // bit cursor at the start and expected at the end
    uint32_t p_mid;          // where the lane's second sub-chunk starts
    float n;                 // norm of the bucket
};

__device__ __forceinline__ SubMeta load_meta(const uint16_t* sub_end, const float* norms, uint32_t k, uint32_t c,
                                             uint32_t bkt, const Layout& lay, int lane)
{
    const uint16_t* se = sub_end + ((size_t)k * lay.NC + c) * kSubs;
    SubMeta m;
    m.p_end = se[2 * lane + 1];
    m.p_mid = se[2 * lane];
    m.p0 = lane ? (uint32_t)se[2 * lane - 1] : 0u;
    // the lane's 64 coordinates lie in one bucket: the chunk's own, or with shared chunks one further on
    // (a lane past the end of a short chunk has nothing to decode: its index is kept inside the table)
    m.n = norms[(size_t)k * lay.NB + min(bkt + (((uint32_t)lane * (uint32_t)kLaneCoords) >> lay.bucket_shift), lay.NB - 1u)];
    return m;
}

// Level values and decode table of one Tables object into the decoder's LDS array (WIDE: the table of
// 8-byte entries, which has the same size).
template <bool WIDE = false>
__device__ __forceinline__ void load_tables(unsigned char* s_tab, const Tables* __restrict__ tab, int tid, int nthreads)
{
    static_assert(kWide * sizeof(uint2) == kDlut * sizeof(uint16_t), "the two decode tables share one LDS area");
    for (int i = tid; i < kSymMax; i += nthreads) reinterpret_cast<float*>(s_tab)[i] = tab->lval[i];
    const uint32_t* src = WIDE ? reinterpret_cast<const uint32_t*>(tab->dlutw) : reinterpret_cast<const uint32_t*>(tab->dlut);
    for (int i = tid; i < kDlut / 2; i += nthreads) reinterpret_cast<uint32_t*>(s_tab + kTabLvalBytes)[i] = src[i];
}

// First coordinate, length and bucket of chunk position c.
__device__ __forceinline__ void chunk_geometry(const Layout& lay, uint32_t c, uint32_t& clo, uint32_t& clen, uint32_t& bkt)
{
    if (lay.uniform_bucket) {                             // one segment: chunk geometry is arithmetic
        bkt = c / lay.waves_per_bucket;
        const uint32_t lo = bkt * lay.uniform_bucket, hi = min(lo + lay.uniform_bucket, lay.d);
        clo = lo + (c - bkt * lay.waves_per_bucket) * (uint32_t)kChunk;
        clen = min((uint32_t)kChunk, hi - clo);
    } else {
        clo = lay.chunk_start[c];
        clen = lay.chunk_start[c + 1] - clo;
        bkt = lay.chunk_bucket[c];
    }
}

// Covers the chunk positions that hold 4096 coordinates (straight-line parse, output turned through
// LDS); the others are k_decode_ragged's.
// PREV (Half1): the previous half-step's streams are there; without them the vectors count as zero.
// TWO: those were coded with another level table and code (a.tab_p) than the current ones.
// WIDE: the first kWideBits bits of a code word always tell which one it is, so the 8-byte decode table
// is there (of both codes, with TWO).
// KSPLIT = 2 or 4: that many neighbouring waves share a position, each takes a run of the workers (as
// equal as K allows, the longer runs first), and they add their sums through LDS before the update
// (for layouts with too few positions to fill the GPU's wave slots).
// The kernel's body, for workgroup `block` of the full positions' grid; the LDS arrays are the caller's:
// s_dyn [waves][1 or 2][stage_stride], s_tab and (TWO) s_tab2 of kTabBytes, s_sd [kDecWaves] (KSPLIT > 1).
template <DecMode MODE, bool PREV, bool TWO, bool WIDE, int KSPLIT>
__device__ __forceinline__ void decode_full_body(const Layout& lay, const Tables* __restrict__ tab, Scalars* sc,
                                                 const DecodeArgs& a, uint32_t block, uint32_t* s_dyn,
                                                 unsigned char* s_tab, unsigned char* s_tab2, double* s_sd)
{
    static_assert(!PREV || MODE == DecMode::Half1, "only the second half-step reads two streams");
    static_assert(!TWO || PREV, "a second table only comes with a second stream");
    static_assert(KSPLIT == 1 || KSPLIT == 2 || KSPLIT == 4, "the waves of a workgroup in groups of 1, 2 or 4");
    static_assert(KSPLIT == 1 || MODE != DecMode::Decode, "plain decoding has nothing to add up");
    const unsigned char* s_tab_p = TWO ? s_tab2 : s_tab;

    const int tid = (int)threadIdx.x, lane = lane_id(), w = wave_id();
    const int part = w & (KSPLIT - 1);                   // this wave's place in its group
    constexpr int kBufs = PREV ? 2 : 1;
    const uint32_t stage_words = a.stage_words;          // words a chunk of this code can take
    const uint32_t stage_stride = a.stage_stride;        // padded size of one staging buffer, words
    uint32_t* stage = s_dyn + (size_t)w * kBufs * stage_stride;
    uint32_t* stage_p = stage + stage_stride;

    if constexpr (WIDE) {
        bool ok = tab->wide_ok != 0u;
        if constexpr (TWO) ok = ok && a.tab_p->wide_ok != 0u;
        if (!ok) {                                        // the host chose this variant for another code
            if (tid == 0) raise_error(sc, QGX_EBIT_STATE);
            return;
        }
    }
    load_tables<WIDE>(s_tab, tab, tid, kDecWaves * kWave);
    if constexpr (TWO) load_tables<WIDE>(s_tab2, a.tab_p, tid, kDecWaves * kWave);
    // words past a chunk's end are read by the window of its last symbols: keep them defined
    for (uint32_t q = (uint32_t)lane; q < kBufs * stage_stride; q += kWave) stage[q] = 0;
    __syncthreads();

    const uint32_t g = block * (uint32_t)kDecWaves + (uint32_t)w;                // global wave number
    const uint32_t n_pos = lay.NC;
    uint32_t c, k_first, k_count;
    bool mine;                                           // wave-uniform: a full position that this launch covers
    if (MODE == DecMode::Decode) {
        mine = g < lay.K * n_pos;
        k_first = g / n_pos; c = g - k_first * n_pos; k_count = 1;
    } else if (KSPLIT > 1) {
        const uint32_t each = lay.K / KSPLIT, more = lay.K % KSPLIT;   // `more` runs of each + 1, then runs of each
        c = g / KSPLIT;
        mine = c < n_pos;
        k_first = (uint32_t)part * each + min((uint32_t)part, more);
        k_count = each + ((uint32_t)part < more ? 1u : 0u);
    } else {
        mine = g < n_pos;
        c = g; k_first = 0; k_count = lay.K;
    }
    uint32_t clo = 0, clen = 0, bkt = 0;
    if (mine) chunk_geometry(lay, c, clo, clen, bkt);
    mine = mine && clen == (uint32_t)kChunk;             // the ragged launch takes the other positions
    if constexpr (KSPLIT == 1) {
        if (!mine) return;
    } else {
        // the waves of a group meet at workgroup barriers below, so every wave of the workgroup
        // goes there, the ones without a position with nothing to do on the way
        if (!mine) k_count = 0;
    }
    // A cursor from a corrupt table is pulled back so that a chain of 32 symbols from it stays inside
    // the buffer.  No valid cursor is beyond that: the last chain of a chunk starts after 4064 symbols
    // of at most sym_bits each, and the buffer holds 4096 of them.
    const uint32_t p_limit = stage_words * 32u - 32u * a.sym_bits;

    float acc[kLaneCoords];
#pragma unroll
    for (int s = 0; s < kLaneCoords; ++s) acc[s] = 0.0f;
    double sdiff = 0.0;
    uint32_t seen = 0xFFFFFFFFu;
    bool malformed = false;

    // Two streams: the next worker's chunks are already in flight in registers while these are parsed.
    // One stream: the registers go to the second parse chain instead; the load of a chunk is covered
    // by the other waves of the SIMD.  The lane's cursors and the norm travel ahead either way.
    constexpr bool kAhead = PREV;
    uint4 pre[kPre];
    uint4 pre_p[PREV ? kPre : 1];
    ChunkRef cr{nullptr, 0u}, cp{nullptr, 0u};
    SubMeta nxt{0u, 0u, 0u, 0.0f}, nxt_p{0u, 0u, 0u, 0.0f};
    if (k_count != 0u) {                                  // (always, unless KSPLIT left this wave without work)
        cr = chunk_ref(a.payload, a.cap_words, a.chunk_off, a.sub_end, k_first, c, lay.NC, stage_words, sc);
        if constexpr (kAhead) prefetch_chunk(cr, pre);
        nxt = load_meta(a.sub_end, a.norms, k_first, c, bkt, lay, lane);
        if constexpr (PREV) {
            cp = chunk_ref(a.payload_p, a.cap_words_p, a.chunk_off_p, a.sub_end_p, k_first, c, lay.NC, stage_words, sc);
            prefetch_chunk(cp, pre_p);
            nxt_p = load_meta(a.sub_end_p, a.norms_p, k_first, c, bkt, lay, lane);
        }
    }

    for (uint32_t kk = 0; kk < k_count; ++kk) {
        const uint32_t k = k_first + kk;
        const SubMeta cur = nxt, prv = nxt_p;
        if constexpr (!kAhead) prefetch_chunk(cr, pre);
        wave_lds_fence();                                     // the last worker's windows have been read
        commit_chunk_reversed(stage, pre, stage_words, (uint32_t)__builtin_amdgcn_readfirstlane((int)cr.words));
        if constexpr (PREV)
            commit_chunk_reversed(stage_p, pre_p, stage_words, (uint32_t)__builtin_amdgcn_readfirstlane((int)cp.words));
        wave_lds_fence();                                     // a lane parses words that other lanes stored
        if (kk + 1 < k_count) {
            cr = chunk_ref(a.payload, a.cap_words, a.chunk_off, a.sub_end, k + 1, c, lay.NC, stage_words, sc);
            nxt = load_meta(a.sub_end, a.norms, k + 1, c, bkt, lay, lane);
            if constexpr (kAhead) prefetch_chunk(cr, pre);
            if constexpr (PREV) {
                cp = chunk_ref(a.payload_p, a.cap_words_p, a.chunk_off_p, a.sub_end_p, k + 1, c, lay.NC, stage_words, sc);
                nxt_p = load_meta(a.sub_end_p, a.norms_p, k + 1, c, bkt, lay, lane);
                prefetch_chunk(cp, pre_p);
            }
        }
        uint32_t p = cur.p0, pp = prv.p0;
        if (p > p_limit) { p = p_limit; malformed = true; }
        if (pp > p_limit) { pp = p_limit; malformed = true; }
        const float n = cur.n, np = prv.n;
        float* vout = nullptr;
        if constexpr (MODE == DecMode::Decode) vout = a.out + (size_t)k * lay.d + clo + 64u * (uint32_t)lane;
        // From stream bit p to the buffer bit r with the bit before p on top of the 64 bits from r:
        // r = r_base - p (the chunk lies back to front).
        const uint32_t r_base = 32u * ((uint32_t)kTail + stage_words) - 63u;
        constexpr int kHalf = kLaneCoords / 2;
        if constexpr (!PREV) {
            // the lane's two sub-chunks side by side: ten groups of three symbols and one of two each;
            // a group's last symbol is finished when the next group's first window (its sign on top) is there
            uint32_t pb = cur.p_mid;
            if (pb > p_limit) { pb = p_limit; malformed = true; }
            uint32_t q = r_base - p, qb = r_base - pb;
            uint32_t W[4], e[3], W_b[4], e_b[3];
            float lv_held = 0.0f, lv_held_b = 0.0f;
            Window wn = read_window(stage, q), wn_b = read_window(stage, qb);
            auto emit = [&](int at, uint32_t w_next, float lv) {
                if constexpr (MODE == DecMode::Decode) {
                    vout[at] = value_early<true>(w_next, lv, n);
                } else if constexpr (MODE == DecMode::Half1) {           // no previous streams: the vectors of t count as zero
                    const float val = value_early<false>(w_next, lv, n);
                    acc[at] += val;
                    sdiff = fma((double)val, (double)val, sdiff);
                } else {
                    acc[at] = fmaf(signed_norm(w_next, n), lv, acc[at]);    // (a stray sign on a zero adds nothing)
                }
            };
#pragma unroll
            for (int s = 0; s < kHalf; s += 3) {
                float lv[3], lv_b[3];
                if (s + 3 <= kHalf) {
                    parse_group_early<3, WIDE, false>(wn, s_tab, q, W, e, lv, seen);
                    wn = read_window(stage, q);
                    parse_group_early<3, WIDE, false>(wn_b, s_tab, qb, W_b, e_b, lv_b, seen);
                    wn_b = read_window(stage, qb);
                } else {
                    parse_group_early<2, WIDE, true>(wn, s_tab, q, W, e, lv, seen);
                    parse_group_early<2, WIDE, true>(wn_b, s_tab, qb, W_b, e_b, lv_b, seen);
                }
                const int cnt = s + 3 <= kHalf ? 3 : 2;
                if constexpr (!WIDE) {
#pragma unroll
                    for (int i = 0; i < 3; ++i) {
                        if (i < cnt) { lv[i] = level_of(s_tab, e[i]); lv_b[i] = level_of(s_tab, e_b[i]); }
                    }
                }
                if (s > 0) { emit(s - 1, W[0], lv_held); emit(kHalf + s - 1, W_b[0], lv_held_b); }
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    if (i + 1 < cnt || cnt == 2) { emit(s + i, W[i + 1], lv[i]); emit(kHalf + s + i, W_b[i + 1], lv_b[i]); }
                }
                if (cnt == 3) { lv_held = lv[2]; lv_held_b = lv_b[2]; }
            }
            if (r_base - q != cur.p_mid) malformed = true;
            p = r_base - qb;
        } else {
            // two streams, two sub-chunks each: four chains, ten groups of three symbols and one of two
            uint32_t pb = cur.p_mid, ppb = prv.p_mid;
            if (pb > p_limit) { pb = p_limit; malformed = true; }
            if (ppb > p_limit) { ppb = p_limit; malformed = true; }
            uint32_t q = r_base - p, qb = r_base - pb, qp = r_base - pp, qpb = r_base - ppb;
            uint32_t W[4], e[3], W_b[4], e_b[3], W_p[4], e_p[3], W_pb[4], e_pb[3];
            float lv_held = 0.0f, lv_held_b = 0.0f, lv_held_p = 0.0f, lv_held_pb = 0.0f;
            Window wn = read_window(stage, q), wn_b = read_window(stage, qb);
            Window wn_p = read_window(stage_p, qp), wn_pb = read_window(stage_p, qpb);
            // Squared differences: six at a time in binary32 (at most six roundings on a sum of
            // non-negative terms), the groups in binary64.  The differences are scaled by a power of two
            // taken from the larger of the lane's two norms, so that no square leaves the range of
            // binary32 whatever the scale of the vectors; the sum is scaled back in binary64.
            const uint32_t ex = min((__float_as_uint(fmaxf(n, np)) >> 23) & 0xFFu, 253u);   // (254 - ex = 0 would be no power of two)
            const float down = __uint_as_float((254u - ex) << 23);                       // 2^(127 - ex)
            const double up2 = __longlong_as_double((long long)(2 * (int)ex - 254 + 1023) << 52);   // 2^(2 ex - 254)
            float sd32 = 0.0f;
            double sw = 0.0;
            auto emit2 = [&](int at, uint32_t w_next, float lv, uint32_t w_next_p, float lv_p) {
                const float val = value_early<false>(w_next, lv, n);
                acc[at] += val;
                const float df = (value_early<false>(w_next_p, lv_p, np) - val) * down;   // (a stray sign on a zero does not show in a difference)
                sd32 = fmaf(df, df, sd32);
            };
#pragma unroll
            for (int s = 0; s < kHalf; s += 3) {
                float lv[3], lv_p[3], lv_b[3], lv_pb[3];
                if (s + 3 <= kHalf) {
                    parse_group_early<3, WIDE, false>(wn, s_tab, q, W, e, lv, seen);
                    wn = read_window(stage, q);
                    parse_group_early<3, WIDE, false>(wn_p, s_tab_p, qp, W_p, e_p, lv_p, seen);
                    wn_p = read_window(stage_p, qp);
                    parse_group_early<3, WIDE, false>(wn_b, s_tab, qb, W_b, e_b, lv_b, seen);
                    wn_b = read_window(stage, qb);
                    parse_group_early<3, WIDE, false>(wn_pb, s_tab_p, qpb, W_pb, e_pb, lv_pb, seen);
                    wn_pb = read_window(stage_p, qpb);
                } else {
                    parse_group_early<2, WIDE, true>(wn, s_tab, q, W, e, lv, seen);
                    parse_group_early<2, WIDE, true>(wn_p, s_tab_p, qp, W_p, e_p, lv_p, seen);
                    parse_group_early<2, WIDE, true>(wn_b, s_tab, qb, W_b, e_b, lv_b, seen);
                    parse_group_early<2, WIDE, true>(wn_pb, s_tab_p, qpb, W_pb, e_pb, lv_pb, seen);
                }
                const int cnt = s + 3 <= kHalf ? 3 : 2;
                if constexpr (!WIDE) {
#pragma unroll
                    for (int i = 0; i < 3; ++i) {
                        if (i < cnt) {
                            lv[i] = level_of(s_tab, e[i]);
                            lv_p[i] = level_of(s_tab_p, e_p[i]);
                            lv_b[i] = level_of(s_tab, e_b[i]);
                            lv_pb[i] = level_of(s_tab_p, e_pb[i]);
                        }
                    }
                }
                if (s > 0) {
                    emit2(s - 1, W[0], lv_held, W_p[0], lv_held_p);
                    emit2(kHalf + s - 1, W_b[0], lv_held_b, W_pb[0], lv_held_pb);
                }
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    if (i + 1 < cnt || cnt == 2) {
                        emit2(s + i, W[i + 1], lv[i], W_p[i + 1], lv_p[i]);
                        emit2(kHalf + s + i, W_b[i + 1], lv_b[i], W_pb[i + 1], lv_pb[i]);
                    }
                }
                if (cnt == 3) { lv_held = lv[2]; lv_held_b = lv_b[2]; lv_held_p = lv_p[2]; lv_held_pb = lv_pb[2]; }
                sw += (double)sd32;
                sd32 = 0.0f;
            }
            sdiff = fma(sw, up2, sdiff);
            if (r_base - q != cur.p_mid || r_base - qp != prv.p_mid) malformed = true;
            p = r_base - qb;
            pp = r_base - qpb;
        }
        if (p != cur.p_end) malformed = true;
        if constexpr (PREV) {
            if (pp != prv.p_end) malformed = true;
        }
    }
    // a reject entry leaves a zero among bits 15..31 of its group's negative bit count
    malformed = malformed || (seen >> 15) != 0x1FFFFu;
    if (__any(malformed) && lane == 0) raise_error(sc, QGX_EBIT_STREAM);
    if (MODE == DecMode::Decode) return;

    // ---- aggregate and update ---------------------------------------------------------------------
    const float invK = 1.0f / (float)lay.K;
    const float gam = sc->gamma_f;
    if constexpr (MODE == DecMode::Half1) {
        sdiff = wave_sum(sdiff);
        if constexpr (KSPLIT > 1) {
            if (lane == 0) s_sd[w] = sdiff;               // joined below, after the first barrier
        } else {
            if (lane == 0) a.s_partial[c] = sdiff;
        }
    }
    // Lane L holds coordinates 64L..64L+63 of the chunk.  Through LDS the wave turns them, a quarter of them
    // at a time, so that neighbouring lanes own consecutive floats and global accesses touch whole pieces
    // of kPiece floats instead of 16 bytes per 256.  Where the output is another array than the one read
    // (the first half-step, the plain average) a piece is a whole 128-byte line, from the 32 lanes of one
    // half of the wave and 32 of their symbols: with pieces of 64 bytes the cache fetched the other half of
    // every output line that it did not hold, a sixth more traffic for the launch.  The second half-step
    // updates Y in place, the line is there when it is written, and pieces of 64 bytes from all 64 lanes
    // and 16 of their symbols are the quicker turn.
    // KSPLIT: all waves of the group put their sums there, and after a barrier each of them adds them
    // up (in the order of the workers' runs) for its share of the rows and does the update for those.
    constexpr int kPiece = MODE == DecMode::Half1 ? 16 : 32;   // floats of a row per pass
    constexpr int kPitch = kPiece + 4;                          // 64 rows of 20 floats or 32 rows of 36: at most 5120 bytes
    constexpr int kRowLanes = kPiece / 4;                       // lanes that read a row, a float4 each
    constexpr int kRowsPerRead = kWave / kRowLanes;
    float* tr = reinterpret_cast<float*>(stage);
    const float* tr0 = KSPLIT > 1 ? reinterpret_cast<const float*>(s_dyn + (size_t)(w - part) * kBufs * stage_stride) : tr;
    const size_t tr_step = (size_t)kBufs * stage_stride;  // from one wave's buffer to the next, in words
    const float scale = KSPLIT > 1 ? 1.0f : invK;         // KSPLIT: the division comes after the group's sum
    // Where this lane's i-th float4 of pass q lies in the vectors.
    auto place = [&](int q, int i) -> uint32_t {
        const int first_lane = kPiece == 32 ? 32 * (q >> 1) : 0, first_sym = kPiece == 32 ? 32 * (q & 1) : 16 * q;
        const int row = lane / kRowLanes + kRowsPerRead * i, col = lane % kRowLanes;
        return clo + 64u * (uint32_t)(first_lane + row) + (uint32_t)first_sym + 4u * (uint32_t)col;
    };
    // A piece of Y is asked for as soon as the piece before it in the same registers has been used, a pass
    // ahead of its own use: every wave of the launch reaches this stage at about the same time, and a load
    // issued where it is used would be waited for in full, four times over.
    constexpr bool kReadsY = MODE == DecMode::Half0 || MODE == DecMode::Half1;
    float4 y_ahead[4];
    auto load_y = [&](int q, int i) {
        y_ahead[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (KSPLIT > 1 && i * KSPLIT / 4 != part) return;
        if (mine) y_ahead[i] = *reinterpret_cast<const float4*>(a.Y + place(q, i));
    };
    if constexpr (kReadsY) {
#pragma unroll
        for (int i = 0; i < 4; ++i) load_y(0, i);
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int first_lane = kPiece == 32 ? 32 * (q >> 1) : 0;    // the lanes whose symbols this pass turns
        const int first_sym = kPiece == 32 ? 32 * (q & 1) : 16 * q;  // ... and which of their symbols
        if (mine && (kPiece == 16 || (lane >> 5) == (q >> 1))) {
#pragma unroll
            for (int j = 0; j < kRowLanes; ++j)
                *reinterpret_cast<float4*>(tr + (lane - first_lane) * kPitch + 4 * j) =
                    make_float4(acc[first_sym + 4 * j] * scale, acc[first_sym + 4 * j + 1] * scale,
                                acc[first_sym + 4 * j + 2] * scale, acc[first_sym + 4 * j + 3] * scale);
        }
        wave_lds_fence();                                     // the rows are read by other lanes than wrote them
        if constexpr (KSPLIT > 1) {
            __syncthreads();
            if (MODE == DecMode::Half1 && q == 0 && mine && part == 0 && lane == 0) {
                double sd = s_sd[w];
                for (int j = 1; j < KSPLIT; ++j) sd += s_sd[w + j];
                a.s_partial[c] = sd;
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (KSPLIT > 1 && i * KSPLIT / 4 != part) continue;   // a share of the rows for each wave of the group
            if (!mine) continue;
            const int row = lane / kRowLanes + kRowsPerRead * i, col = lane % kRowLanes;
            float4 m = *reinterpret_cast<const float4*>(tr0 + row * kPitch + 4 * col);
            if constexpr (KSPLIT > 1) {
#pragma unroll
                for (int j = 1; j < KSPLIT; ++j) {
                    const float4 h4 = *reinterpret_cast<const float4*>(tr0 + j * tr_step + row * kPitch + 4 * col);
                    m.x += h4.x; m.y += h4.y; m.z += h4.z; m.w += h4.w;
                }
                m.x *= invK; m.y *= invK; m.z *= invK; m.w *= invK;
            }
            const uint32_t at = place(q, i);
            if (MODE == DecMode::Average) {
                *reinterpret_cast<float4*>(a.out + at) = m;
            } else if (MODE == DecMode::Half0) {
                const float4 y = y_ahead[i];
                float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
                if (a.anchor) x = *reinterpret_cast<const float4*>(a.anchor + at);
                x.x = (x.x + gam * y.x) - gam * m.x;
                x.y = (x.y + gam * y.y) - gam * m.y;
                x.z = (x.z + gam * y.z) - gam * m.z;
                x.w = (x.w + gam * y.w) - gam * m.w;
                *reinterpret_cast<float4*>(a.out + at) = x;
                if (q < 3) load_y(q + 1, i);
                if (a.x_sum) {                                   // ergodic average: sum of the half-step iterates
                    double2* xs = reinterpret_cast<double2*>(a.x_sum + at);
                    double2 s0 = xs[0], s1 = xs[1];
                    s0.x += (double)x.x; s0.y += (double)x.y; s1.x += (double)x.z; s1.y += (double)x.w;
                    xs[0] = s0; xs[1] = s1;
                }
            } else {
                float4 y = y_ahead[i];
                y.x -= m.x; y.y -= m.y; y.z -= m.z; y.w -= m.w;
                *reinterpret_cast<float4*>(a.Y + at) = y;
                if (q < 3) load_y(q + 1, i);
            }
        }
        wave_lds_fence();                                     // ... and written again in the next pass
        if constexpr (KSPLIT > 1) {
            if (q < 3) __syncthreads();                       // the partners have read this quarter
        }
    }
}

template <DecMode MODE, bool PREV, bool TWO, bool WIDE, int KSPLIT = 1>
__global__ __launch_bounds__(kDecWaves * kWave) __attribute__((amdgpu_waves_per_eu(MODE == DecMode::Half1 ? 2 : 4)))
void k_decode(Layout lay, const Tables* __restrict__ tab, Scalars* sc, DecodeArgs a)
{
    __shared__ double s_sd[KSPLIT > 1 ? kDecWaves : 1];
    extern __shared__ __align__(16) uint32_t s_dyn[];    // [waves][1 or 2][stage_stride]
    __shared__ __align__(16) unsigned char s_tab[kTabBytes];
    __shared__ __align__(16) unsigned char s_tab2[TWO ? kTabBytes : 16];
    decode_full_body<MODE, PREV, TWO, WIDE, KSPLIT>(lay, tab, sc, a, blockIdx.x, s_dyn, s_tab, s_tab2, s_sd);
}

// ---- chunk positions with fewer than 4096 coordinates --------------------------------------------
// They are the tails of buckets and tensors: few, but a wave that walked all K workers of one, symbol
// by symbol, would take as long as the whole launch of the full positions.  So a position gets a
// workgroup of its own and its workers are spread over the waves: wave w stages and parses the chunk
// of worker k0 + w (every lane its two sub-chunks side by side, as far as they go), then the waves
// add their values to accumulators in LDS one after the other, so that a coordinate's K values are
// summed in worker order like everywhere else.  The update itself is done by all threads, coalesced.
constexpr int kAccPitch = 65;                         // s_acc[s][lane], padded: both access patterns spread over the banks

template <bool PREV>
constexpr int ragged_waves() { return PREV ? 4 : 8; } // two staging buffers per wave with two streams

// The body, for ragged position `index` (of lay.ragged_chunk) and the first ragged_waves() waves of the workgroup
// (further waves leave at once, before any barrier); the LDS arrays are the caller's: s_dyn [waves][1 or 2]
// [rag_stride], s_tab and (TWO) s_tab2 of kTabBytes, s_acc [kLaneCoords * kAccPitch], s_sd [ragged_waves()].
template <DecMode MODE, bool PREV, bool TWO>
__device__ __forceinline__ void decode_ragged_body(const Layout& lay, const Tables* __restrict__ tab, Scalars* sc,
                                                   const DecodeArgs& a, uint32_t index, uint32_t* s_dyn,
                                                   unsigned char* s_tab, unsigned char* s_tab2, float* s_acc, double* s_sd)
{
    static_assert(!PREV || MODE == DecMode::Half1, "only the second half-step reads two streams");
    static_assert(!TWO || PREV, "a second table only comes with a second stream");
    constexpr int W = ragged_waves<PREV>();
    constexpr int kBufs = PREV ? 2 : 1;
    constexpr bool kExact = MODE == DecMode::Decode;
    constexpr int kHalf = kLaneCoords / 2;
    const unsigned char* s_tab_p = TWO ? s_tab2 : s_tab;

    const int tid = (int)threadIdx.x, lane = lane_id(), w = wave_id();
    if (w >= W) return;
    const uint32_t stage_words = a.rag_words, stage_stride = a.rag_stride;
    uint32_t* stage = s_dyn + (size_t)w * kBufs * stage_stride;
    uint32_t* stage_p = stage + stage_stride;

    load_tables(s_tab, tab, tid, W * kWave);
    if constexpr (TWO) load_tables(s_tab2, a.tab_p, tid, W * kWave);
    for (int i = tid; i < kLaneCoords * kAccPitch; i += W * kWave) s_acc[i] = 0.0f;
    for (uint32_t q = (uint32_t)lane; q < kBufs * stage_stride; q += kWave) stage[q] = 0;
    __syncthreads();

    const uint32_t c = lay.ragged_chunk[index];
    uint32_t clo, clen, bkt;
    chunk_geometry(lay, c, clo, clen, bkt);
    const int cnt = (int)min(64u, clen > 64u * (uint32_t)lane ? clen - 64u * (uint32_t)lane : 0u);
    const int cnt_a = min(cnt, kHalf), cnt_b = cnt - cnt_a;       // symbols of the lane's two sub-chunks
    // Every chain parses 32 symbols whatever its count, so the buffer has room for that beyond the
    // longest chunk (rag_words); a cursor from a corrupt table is pulled back to where that room starts.
    const uint32_t p_limit = stage_words * 32u - (uint32_t)kHalf * a.sym_bits - 64u;

    double sdiff = 0.0;
    uint32_t flags = 0;
    bool malformed = false;

    for (uint32_t k0 = 0; k0 < lay.K; k0 += W) {
        const uint32_t k = k0 + (uint32_t)w;
        const bool active = k < lay.K;                    // wave-uniform
        float val[kLaneCoords];
#pragma unroll
        for (int s = 0; s < kLaneCoords; ++s) val[s] = 0.0f;
        if (active) {
            uint4 pre[kPre];
            const ChunkRef cr = chunk_ref(a.payload, a.cap_words, a.chunk_off, a.sub_end, k, c, lay.NC, stage_words, sc);
            prefetch_chunk(cr, pre);
            const SubMeta cur = load_meta(a.sub_end, a.norms, k, c, bkt, lay, lane);
            SubMeta prv{0u, 0u, 0u, 0.0f};
            commit_chunk(stage, pre, stage_words);
            if constexpr (PREV) {
                const ChunkRef cp = chunk_ref(a.payload_p, a.cap_words_p, a.chunk_off_p, a.sub_end_p, k, c, lay.NC, stage_words, sc);
                prefetch_chunk(cp, pre);
                prv = load_meta(a.sub_end_p, a.norms_p, k, c, bkt, lay, lane);
                commit_chunk(stage_p, pre, stage_words);
            }
            wave_lds_fence();                                 // a lane parses words that other lanes stored
            uint32_t p = cur.p0, pb = cur.p_mid, pp = prv.p0, ppb = prv.p_mid;
            if (p > p_limit) { p = p_limit; malformed = true; }
            if (pb > p_limit) { pb = p_limit; malformed = true; }
            if (pp > p_limit) { pp = p_limit; malformed = true; }
            if (ppb > p_limit) { ppb = p_limit; malformed = true; }
            const float n = cur.n, np = prv.n;
            // Every lane parses 32 symbols per chain whatever its count (from a cursor below p_limit they
            // stay inside the buffer, and any window finds a table entry), and what lies past its count
            // is masked out: without branches the chains of a lane advance side by side, in groups of
            // three symbols per window as in the kernel for the full positions.
            float* vout = nullptr;
            if constexpr (MODE == DecMode::Decode) vout = a.out + (size_t)k * lay.d + clo + 64u * (uint32_t)lane;
            const uint32_t start_a = p, start_b = pb, start_pa = pp, start_pb = ppb;
            uint32_t used_a = 0, used_b = 0, used_pa = 0, used_pb = 0;     // bits of the symbols that count
            uint32_t win[3], e[3], win_b[3], e_b[3];
            uint32_t win_p[3] = {0u, 0u, 0u}, e_p[3] = {0u, 0u, 0u}, win_pb[3] = {0u, 0u, 0u}, e_pb[3] = {0u, 0u, 0u};
            Window wn = read_window(stage, p), wn_b = read_window(stage, pb);
            Window wn_p{0u, 0u, 0u}, wn_pb{0u, 0u, 0u};
            if constexpr (PREV) { wn_p = read_window(stage_p, pp); wn_pb = read_window(stage_p, ppb); }
#pragma unroll
            for (int s = 0; s < kHalf; s += 3) {
                if (s + 3 <= kHalf) { parse_group<3>(wn, s_tab, p, win, e); parse_group<3>(wn_b, s_tab, pb, win_b, e_b); }
                else { parse_group<2>(wn, s_tab, p, win, e); parse_group<2>(wn_b, s_tab, pb, win_b, e_b); }
                if (s + 3 < kHalf) { wn = read_window(stage, p); wn_b = read_window(stage, pb); }
                if constexpr (PREV) {
                    if (s + 3 <= kHalf) { parse_group<3>(wn_p, s_tab_p, pp, win_p, e_p); parse_group<3>(wn_pb, s_tab_p, ppb, win_pb, e_pb); }
                    else { parse_group<2>(wn_p, s_tab_p, pp, win_p, e_p); parse_group<2>(wn_pb, s_tab_p, ppb, win_pb, e_pb); }
                    if (s + 3 < kHalf) { wn_p = read_window(stage_p, pp); wn_pb = read_window(stage_p, ppb); }
                }
#pragma unroll
                for (int i = 0; i < 3; ++i) {
                    if (s + i < kHalf) {
                        const bool ok_a = s + i < cnt_a, ok_b = s + i < cnt_b;
                        const float v = symbol_value<kExact>(level_of(s_tab, e[i]), win[i], e[i], n);
                        const float v_b = symbol_value<kExact>(level_of(s_tab, e_b[i]), win_b[i], e_b[i], n);
                        if constexpr (MODE == DecMode::Decode) {
                            if (ok_a) vout[s + i] = v;
                            if (ok_b) vout[kHalf + s + i] = v_b;
                        } else {
                            val[s + i] = ok_a ? v : 0.0f;
                            val[kHalf + s + i] = ok_b ? v_b : 0.0f;
                        }
                        flags |= (ok_a ? e[i] : 0u) | (ok_b ? e_b[i] : 0u);
                        used_a += ok_a ? (e[i] & 15u) + 1u : 0u;
                        used_b += ok_b ? (e_b[i] & 15u) + 1u : 0u;
                        if constexpr (MODE == DecMode::Half1) {
                            float pv = 0.0f, pv_b = 0.0f;
                            if constexpr (PREV) {
                                pv = symbol_value<true>(level_of(s_tab_p, e_p[i]), win_p[i], e_p[i], np);
                                pv_b = symbol_value<true>(level_of(s_tab_p, e_pb[i]), win_pb[i], e_pb[i], np);
                                flags |= (ok_a ? e_p[i] : 0u) | (ok_b ? e_pb[i] : 0u);
                                used_pa += ok_a ? (e_p[i] & 15u) + 1u : 0u;
                                used_pb += ok_b ? (e_pb[i] & 15u) + 1u : 0u;
                            }
                            const double df = ok_a ? (double)pv - (double)v : 0.0;
                            const double df_b = ok_b ? (double)pv_b - (double)v_b : 0.0;
                            sdiff = fma(df, df, sdiff);
                            sdiff = fma(df_b, df_b, sdiff);
                        }
                    }
                }
            }
            if (cnt > 0 && (start_a + used_a != cur.p_mid || start_b + used_b != cur.p_end)) malformed = true;
            if constexpr (PREV) {
                if (cnt > 0 && (start_pa + used_pa != prv.p_mid || start_pb + used_pb != prv.p_end)) malformed = true;
            }
        }
        if constexpr (MODE != DecMode::Decode) {
            for (int turn = 0; turn < W; ++turn) {        // worker order: k0, k0 + 1, ...
                if (turn == w && active) {
#pragma unroll
                    for (int s = 0; s < kLaneCoords; ++s)
                        if (s < cnt) s_acc[s * kAccPitch + lane] += val[s];
                }
                __syncthreads();
            }
        }
    }
    malformed = malformed || (flags & 0x8000u) != 0u;
    if (__any(malformed) && lane == 0) raise_error(sc, QGX_EBIT_STREAM);
    if (MODE == DecMode::Decode) return;

    if constexpr (MODE == DecMode::Half1) {
        sdiff = wave_sum(sdiff);
        if (lane == 0) s_sd[w] = sdiff;
        __syncthreads();
        if (tid == 0) {
            double t = 0.0;
            for (int i = 0; i < W; ++i) t += s_sd[i];
            a.s_partial[c] = t;
        }
    }
    const float invK = 1.0f / (float)lay.K;
    const float gam = sc->gamma_f;
    for (uint32_t i = (uint32_t)tid; i < clen; i += W * kWave) {
        const float m = s_acc[(i & 63u) * kAccPitch + (i >> 6)] * invK;
        const uint32_t at = clo + i;
        if (MODE == DecMode::Average) a.out[at] = m;
        else if (MODE == DecMode::Half0) {
            const float x = a.anchor ? a.anchor[at] : 0.0f;
            const float xh = (x + gam * a.Y[at]) - gam * m;
            a.out[at] = xh;
            if (a.x_sum) a.x_sum[at] += (double)xh;
        } else a.Y[at] -= m;
    }
}

template <DecMode MODE, bool PREV, bool TWO>
__global__ __launch_bounds__(ragged_waves<PREV>() * kWave)
void k_decode_ragged(Layout lay, const Tables* __restrict__ tab, Scalars* sc, DecodeArgs a)
{
    extern __shared__ __align__(16) uint32_t s_dyn[];    // [waves][1 or 2][rag_stride]
    __shared__ __align__(16) unsigned char s_tab[kTabBytes];
    __shared__ __align__(16) unsigned char s_tab2[TWO ? kTabBytes : 16];
    __shared__ float s_acc[kLaneCoords * kAccPitch];
    __shared__ double s_sd[ragged_waves<PREV>()];
    decode_ragged_body<MODE, PREV, TWO>(lay, tab, sc, a, blockIdx.x, s_dyn, s_tab, s_tab2, s_acc, s_sd);
}

// Layouts with both kinds of positions: one launch, a workgroup per ragged position first and the workgroups
// of the full positions after them, so that the few, slow ragged ones (a cold instruction cache and the
// tables' load for a single position each) start at once and run beside the full ones, not before or after
// them.  The ragged workgroups take their sums' array from the dynamic LDS, behind their staging buffers.
template <DecMode MODE, bool PREV, bool TWO, bool WIDE, int KSPLIT>
__global__ __launch_bounds__(kDecWaves * kWave) __attribute__((amdgpu_waves_per_eu(MODE == DecMode::Half1 ? 2 : 4)))
void k_decode_both(Layout lay, const Tables* __restrict__ tab, Scalars* sc, DecodeArgs a)
{
    __shared__ double s_sd[kDecWaves];
    extern __shared__ __align__(16) uint32_t s_dyn[];
    __shared__ __align__(16) unsigned char s_tab[kTabBytes];
    __shared__ __align__(16) unsigned char s_tab2[TWO ? kTabBytes : 16];
    if (blockIdx.x >= lay.n_ragged) {
        decode_full_body<MODE, PREV, TWO, WIDE, KSPLIT>(lay, tab, sc, a, blockIdx.x - lay.n_ragged, s_dyn, s_tab, s_tab2, s_sd);
    } else {
        float* s_acc = reinterpret_cast<float*>(s_dyn + (size_t)ragged_waves<PREV>() * (PREV ? 2 : 1) * a.rag_stride);
        decode_ragged_body<MODE, PREV, TWO>(lay, tab, sc, a, blockIdx.x, s_dyn, s_tab, s_tab2, s_acc, s_sd);
    }
}

template <DecMode MODE, bool PREV, bool TWO, bool WIDE, int KSPLIT>
static hipError_t launch_full_as(const Layout& lay, const Tables* tab, Scalars* sc, const DecodeArgs& a, hipStream_t st)
{
    if (lay.n_ragged == lay.NC) return hipSuccess;
    const size_t lds = (size_t)kDecWaves * (PREV ? 2 : 1) * a.stage_stride * sizeof(uint32_t);
    static LdsLimit limit;
    hipError_t e = limit.ensure(reinterpret_cast<const void*>(&k_decode<MODE, PREV, TWO, WIDE, KSPLIT>), lds);
    if (e != hipSuccess) return e;
    const uint64_t nwork = (MODE == DecMode::Decode) ? (uint64_t)lay.K * lay.NC : (uint64_t)lay.NC * (uint32_t)KSPLIT;
    const uint32_t grid = (uint32_t)((nwork + kDecWaves - 1) / kDecWaves);
    hipLaunchKernelGGL((k_decode<MODE, PREV, TWO, WIDE, KSPLIT>), dim3(grid), dim3(kDecWaves * kWave), lds, st, lay, tab, sc, a);
    return hipGetLastError();
}

template <DecMode MODE, bool PREV, bool TWO>
static hipError_t launch_full(const Layout& lay, const Tables* tab, Scalars* sc, const DecodeArgs& a, hipStream_t st)
{
    if constexpr (MODE != DecMode::Decode) {
        if (a.ksplit == 2u) {
            if (a.wide) return launch_full_as<MODE, PREV, TWO, true, 2>(lay, tab, sc, a, st);
            return launch_full_as<MODE, PREV, TWO, false, 2>(lay, tab, sc, a, st);
        }
        if (a.ksplit == 4u) {
            if (a.wide) return launch_full_as<MODE, PREV, TWO, true, 4>(lay, tab, sc, a, st);
            return launch_full_as<MODE, PREV, TWO, false, 4>(lay, tab, sc, a, st);
        }
    }
    if (a.wide) return launch_full_as<MODE, PREV, TWO, true, 1>(lay, tab, sc, a, st);
    return launch_full_as<MODE, PREV, TWO, false, 1>(lay, tab, sc, a, st);
}

template <DecMode MODE, bool PREV, bool TWO>
static hipError_t launch_ragged(const Layout& lay, const Tables* tab, Scalars* sc, const DecodeArgs& a, hipStream_t st)
{
    if (lay.n_ragged == 0) return hipSuccess;
    constexpr int W = ragged_waves<PREV>();
    const size_t lds = (size_t)W * (PREV ? 2 : 1) * a.rag_stride * sizeof(uint32_t);
    static LdsLimit limit;
    hipError_t e = limit.ensure(reinterpret_cast<const void*>(&k_decode_ragged<MODE, PREV, TWO>), lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((k_decode_ragged<MODE, PREV, TWO>), dim3(lay.n_ragged), dim3(W * kWave), lds, st, lay, tab, sc, a);
    return hipGetLastError();
}

// Both kinds of positions in one launch (k_decode_both).
template <DecMode MODE, bool PREV, bool TWO, bool WIDE, int KSPLIT>
static hipError_t launch_both_as(const Layout& lay, const Tables* tab, Scalars* sc, const DecodeArgs& a, hipStream_t st)
{
    constexpr int W = ragged_waves<PREV>();
    constexpr size_t bufs = PREV ? 2 : 1;
    const size_t lds_full = (size_t)kDecWaves * bufs * a.stage_stride * sizeof(uint32_t);
    const size_t lds_ragged = (size_t)W * bufs * a.rag_stride * sizeof(uint32_t) + (size_t)kLaneCoords * kAccPitch * sizeof(float);
    const size_t lds = lds_full > lds_ragged ? lds_full : lds_ragged;
    static LdsLimit limit;
    hipError_t e = limit.ensure(reinterpret_cast<const void*>(&k_decode_both<MODE, PREV, TWO, WIDE, KSPLIT>), lds);
    if (e != hipSuccess) return e;
    const uint64_t nwork = (MODE == DecMode::Decode) ? (uint64_t)lay.K * lay.NC : (uint64_t)lay.NC * (uint32_t)KSPLIT;
    const uint32_t full_blocks = (uint32_t)((nwork + kDecWaves - 1) / kDecWaves);
    hipLaunchKernelGGL((k_decode_both<MODE, PREV, TWO, WIDE, KSPLIT>), dim3(lay.n_ragged + full_blocks), dim3(kDecWaves * kWave),
                       lds, st, lay, tab, sc, a);
    return hipGetLastError();
}

template <DecMode MODE, bool PREV, bool TWO>
static hipError_t launch_both(const Layout& lay, const Tables* tab, Scalars* sc, const DecodeArgs& a, hipStream_t st)
{
    if constexpr (MODE != DecMode::Decode) {
        if (a.ksplit == 2u) {
            if (a.wide) return launch_both_as<MODE, PREV, TWO, true, 2>(lay, tab, sc, a, st);
            return launch_both_as<MODE, PREV, TWO, false, 2>(lay, tab, sc, a, st);
        }
        if (a.ksplit == 4u) {
            if (a.wide) return launch_both_as<MODE, PREV, TWO, true, 4>(lay, tab, sc, a, st);
            return launch_both_as<MODE, PREV, TWO, false, 4>(lay, tab, sc, a, st);
        }
    }
    if (a.wide) return launch_both_as<MODE, PREV, TWO, true, 1>(lay, tab, sc, a, st);
    return launch_both_as<MODE, PREV, TWO, false, 1>(lay, tab, sc, a, st);
}

// A layout's full positions go to k_decode, its ragged ones to k_decode_ragged; a layout that has both
// takes one launch of the kernel that holds both bodies.
template <DecMode MODE, bool PREV, bool TWO = false>
static hipError_t launch_mode(const Layout& lay, const Tables* tab, Scalars* sc, const DecodeArgs& a, hipStream_t st)
{
    if (lay.n_ragged != 0 && lay.n_ragged != lay.NC) return launch_both<MODE, PREV, TWO>(lay, tab, sc, a, st);
    hipError_t e = launch_ragged<MODE, PREV, TWO>(lay, tab, sc, a, st);
    if (e != hipSuccess) return e;
    return launch_full<MODE, PREV, TWO>(lay, tab, sc, a, st);
}

hipError_t launch_decode(DecMode mode, const Layout& lay, const Tables* tab, Scalars* sc, const DecodeArgs& a,
                         hipStream_t st)
{
    switch (mode) {
        case DecMode::Decode: return launch_mode<DecMode::Decode, false>(lay, tab, sc, a, st);
        case DecMode::Average: return launch_mode<DecMode::Average, false>(lay, tab, sc, a, st);
        case DecMode::Half0: return launch_mode<DecMode::Half0, false>(lay, tab, sc, a, st);
        default:
            if (a.payload_p == nullptr) return launch_mode<DecMode::Half1, false>(lay, tab, sc, a, st);
            return a.tab_p ? launch_mode<DecMode::Half1, true, true>(lay, tab, sc, a, st)
                           : launch_mode<DecMode::Half1, true>(lay, tab, sc, a, st);
    }
}

// ---- the scalar end of the second half-step: S, gamma_{t+1}, t; then X_{t+1} on request -----------
__global__ __launch_bounds__(256) void k_finish_half1(uint32_t NC, uint32_t K, Scalars* sc, const double* s_partial)
{
    __shared__ double s_red[256];
    double acc = 0.0;
    for (uint32_t i = threadIdx.x; i < NC; i += 256) acc += s_partial[i];     // fixed order: reproducible
    s_red[threadIdx.x] = acc;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) s_red[threadIdx.x] += s_red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const double S = sc->S + s_red[0];
        const double gamma = (double)K / sqrt(1.0 + S);       // Theorem 3: gamma_t = K (1 + sum ...)^(-1/2)
        sc->S = S;
        sc->gamma = gamma;
        sc->gamma_f = (float)gamma;
        sc->t += 1ull;
    }
}

__global__ __launch_bounds__(256) void k_x_from_y(uint32_t d, const Scalars* sc, const float* __restrict__ Y,
                                                  const float* __restrict__ anchor, float* __restrict__ X)
{
    const float gam = sc->gamma_f;
    for (uint32_t i = blockIdx.x * 256u + threadIdx.x; i < d; i += gridDim.x * 256u)
        X[i] = (anchor ? anchor[i] : 0.0f) + gam * Y[i];
}

hipError_t launch_finish_half1(const Layout& lay, Scalars* sc, const double* s_partial, const float* Y,
                               const float* anchor, float* X_out, hipStream_t st)
{
    hipLaunchKernelGGL(k_finish_half1, dim3(1), dim3(256), 0, st, lay.NC, lay.K, sc, s_partial);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || X_out == nullptr) return e;
    const uint32_t grid = min((lay.d + 255u) / 256u, 4096u);
    hipLaunchKernelGGL(k_x_from_y, dim3(grid), dim3(256), 0, st, lay.d, sc, Y, anchor, X_out);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void k_state_init(uint32_t d, uint32_t K, Scalars* sc, float* Y, float* anchor,
                                                    const float* X1)
{
    for (uint32_t i = blockIdx.x * 256u + threadIdx.x; i < d; i += gridDim.x * 256u) {
        Y[i] = 0.0f;
        anchor[i] = X1 ? X1[i] : 0.0f;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        sc->S = 0.0; sc->gamma = (double)K; sc->gamma_f = (float)K; sc->t = 1ull;
    }
}

hipError_t launch_state_init(const Layout& lay, Scalars* sc, float* Y, float* anchor, const float* X1, hipStream_t st)
{
    const uint32_t grid = min((lay.d + 255u) / 256u, 4096u);
    hipLaunchKernelGGL(k_state_init, dim3(grid), dim3(256), 0, st, lay.d, lay.K, sc, Y, anchor, X1);
    return hipGetLastError();
}

// Ergodic average of the half-step iterates: out = x_sum / count, the count kept on the device (so
// that the half-steps of a replayed graph are counted too); clearing the sum; counting a half-step.
__global__ __launch_bounds__(256) void k_average(uint32_t d, const double* __restrict__ x_sum, const Scalars* sc,
                                                 float* __restrict__ out)
{
    const double count = (double)sc->avg_count;
    for (uint32_t i = blockIdx.x * 256u + threadIdx.x; i < d; i += gridDim.x * 256u) out[i] = (float)(x_sum[i] / count);
}

hipError_t launch_average(uint32_t d, const double* x_sum, const Scalars* sc, float* out, hipStream_t st)
{
    const uint32_t grid = min((d + 255u) / 256u, 4096u);
    hipLaunchKernelGGL(k_average, dim3(grid), dim3(256), 0, st, d, x_sum, sc, out);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void k_average_reset(uint32_t d, double* __restrict__ x_sum, Scalars* sc)
{
    for (uint32_t i = blockIdx.x * 256u + threadIdx.x; i < d; i += gridDim.x * 256u) x_sum[i] = 0.0;
    if (blockIdx.x == 0 && threadIdx.x == 0) sc->avg_count = 0ull;
}

hipError_t launch_average_reset(uint32_t d, double* x_sum, Scalars* sc, hipStream_t st)
{
    const uint32_t grid = min((d + 255u) / 256u, 4096u);
    hipLaunchKernelGGL(k_average_reset, dim3(grid), dim3(256), 0, st, d, x_sum, sc);
    return hipGetLastError();
}

__global__ void k_average_count(Scalars* sc) { sc->avg_count += 1ull; }

hipError_t launch_average_count(Scalars* sc, hipStream_t st)
{
    hipLaunchKernelGGL(k_average_count, dim3(1), dim3(1), 0, st, sc);
    return hipGetLastError();
}

__global__ void k_state_set(Scalars* sc, double S, unsigned long long t, uint32_t K)
{
    const double gamma = (double)K / sqrt(1.0 + S);
    sc->S = S; sc->gamma = gamma; sc->gamma_f = (float)gamma; sc->t = t;
}

hipError_t launch_state_set(Scalars* sc, double S, unsigned long long t, uint32_t K, hipStream_t st)
{
    hipLaunchKernelGGL(k_state_set, dim3(1), dim3(1), 0, st, sc, S, t, K);
    return hipGetLastError();
}

// Bits of the last coded streams, without padding: the last sub-chunk entry of every chunk.
__global__ __launch_bounds__(256) void k_sum_bits(uint64_t n_chunks, const uint16_t* sub_end, Scalars* sc)
{
    __shared__ unsigned long long s_red[256];
    unsigned long long acc = 0;
    for (uint64_t i = threadIdx.x; i < n_chunks; i += 256) acc += sub_end[i * kSubs + (kSubs - 1)];
    s_red[threadIdx.x] = acc;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) s_red[threadIdx.x] += s_red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) sc->total_bits = s_red[0];
}

hipError_t launch_sum_bits(const Layout& lay, const uint16_t* sub_end, Scalars* sc, hipStream_t st)
{
    hipLaunchKernelGGL(k_sum_bits, dim3(1), dim3(256), 0, st, (uint64_t)lay.K * lay.NC, sub_end, sc);
    return hipGetLastError();
}

// ---- slotted -> compact ---------------------------------------------------------------------------
// One workgroup per worker scans the chunk sizes (from the bit lengths) into exclusive offsets; then
// one wave per chunk copies its words.
__device__ __forceinline__ uint32_t chunk_words_of(const uint16_t* __restrict__ sub_end, size_t chunk)
{
    const uint32_t bits = sub_end[chunk * kSubs + (kSubs - 1)];
    return (((bits + 31u) >> 5) + 3u) & ~3u;
}

__global__ __launch_bounds__(1024) void k_compact_offsets(uint32_t NC, const uint16_t* __restrict__ sub_end,
                                                          uint32_t* __restrict__ out_off, uint64_t out_cap, Scalars* sc)
{
    __shared__ uint32_t s_wave[16];
    const uint32_t k = blockIdx.x, tid = threadIdx.x;
    const int lane = lane_id(), w = wave_id();
    // a thread's chunks are consecutive, so its own running sum is all it carries between the two passes
    const uint32_t per = (NC + 1023u) / 1024u;
    const uint32_t c0 = min(tid * per, NC), c1 = min(c0 + per, NC);
    uint32_t sum = 0;
    for (uint32_t c = c0; c < c1; ++c) sum += chunk_words_of(sub_end, (size_t)k * NC + c);
    const uint32_t incl = wave_incl_scan(sum);
    if (lane == kWave - 1) s_wave[w] = incl;
    __syncthreads();
    uint32_t before = 0, total = 0;
    for (int i = 0; i < 16; ++i) {
        if (i == w) before = total;
        total += s_wave[i];
    }
    if (tid == 0) {
        out_off[(size_t)k * (NC + 1) + NC] = total;
        if ((uint64_t)total > out_cap) raise_error(sc, QGX_EBIT_CAPACITY);
    }
    uint32_t run = before + incl - sum;
    for (uint32_t c = c0; c < c1; ++c) {
        out_off[(size_t)k * (NC + 1) + c] = run;
        run += chunk_words_of(sub_end, (size_t)k * NC + c);
    }
}

__global__ __launch_bounds__(256) void k_compact_copy(uint32_t NC, uint32_t K, const uint16_t* __restrict__ sub_end,
                                                      const uint32_t* __restrict__ in_off, const uint32_t* __restrict__ in_payload,
                                                      uint64_t in_cap, const uint32_t* __restrict__ out_off,
                                                      uint32_t* __restrict__ out_payload, uint64_t out_cap, Scalars* sc)
{
    const uint32_t g = blockIdx.x * (blockDim.x >> 6) + (uint32_t)wave_id();
    if (g >= K * NC) return;
    const uint32_t k = g / NC, c = g - k * NC, lane = (uint32_t)lane_id();
    const uint32_t words = chunk_words_of(sub_end, (size_t)k * NC + c);
    const uint32_t src = in_off[(size_t)k * (NC + 1) + c], dst = out_off[(size_t)k * (NC + 1) + c];
    if ((src & 3u) || (uint64_t)src + words > in_cap || (uint64_t)dst + words > out_cap) {
        if (lane == 0) raise_error(sc, (uint64_t)dst + words > out_cap ? QGX_EBIT_CAPACITY : QGX_EBIT_STREAM);
        return;
    }
    const uint4* s = reinterpret_cast<const uint4*>(in_payload + (size_t)k * in_cap + src);
    uint4* d = reinterpret_cast<uint4*>(out_payload + (size_t)k * out_cap + dst);
    // a chunk of the largest size is kPre pieces per lane: all of a lane's loads are on their way before
    // its first store (a chunk of some other origin may be longer: the loop goes on)
    for (uint32_t q0 = 0; q0 < (words >> 2); q0 += (uint32_t)(kPre * kWave)) {
        uint4 held[kPre];
#pragma unroll
        for (int j = 0; j < kPre; ++j) {
            const uint32_t q = q0 + lane + (uint32_t)j * kWave;
            held[j] = q < (words >> 2) ? nt_load4u(s + q) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < kPre; ++j) {
            const uint32_t q = q0 + lane + (uint32_t)j * kWave;
            if (q < (words >> 2)) d[q] = held[j];
        }
    }
}

hipError_t launch_compact(const Layout& lay, const uint16_t* sub_end, const uint32_t* in_off, const uint32_t* in_payload,
                          uint64_t in_cap, uint32_t* out_off, uint32_t* out_payload, uint64_t out_cap, Scalars* sc,
                          hipStream_t st)
{
    hipLaunchKernelGGL(k_compact_offsets, dim3(lay.K), dim3(1024), 0, st, lay.NC, sub_end, out_off, out_cap, sc);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const uint32_t grid = (lay.K * lay.NC + 3u) / 4u;
    hipLaunchKernelGGL(k_compact_copy, dim3(grid), dim3(256), 0, st, lay.NC, lay.K, sub_end, in_off, in_payload, in_cap,
                       out_off, out_payload, out_cap, sc);
    return hipGetLastError();
}

}  // namespace qgx
