// Internal declarations shared by the host side of the library and its gfx950 kernels.
// Nothing here is part of the C ABI (include/qgx.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <mutex>

#include "../../include/qgx.h"

namespace qgx {

constexpr int kWave = 64;                 // CDNA wavefront
constexpr int kChunk = QGX_CHUNK;         // coordinates per chunk = one wave's share
constexpr int kRows = 16;                 // rows of 256 coordinates per chunk (4 per lane and row)
constexpr int kSub = QGX_SUB;
constexpr int kSubs = QGX_SUBS;           // sub-chunk table entries per chunk
constexpr int kLaneCoords = 64;           // coordinates one decoder lane parses: two sub-chunks
constexpr int kMaxCode = QGX_MAX_CODE_BITS;             // longest code word
constexpr int kMaxSymBits = kMaxCode + 1;               // plus the sign bit
constexpr int kChunkWordsMax = kChunk * kMaxSymBits / 32;  // 1792
constexpr int kAlignWords = 4;
constexpr int kMaxWaves = QGX_MAX_BUCKET / kChunk;      // 16 waves = 1024 threads per bucket
constexpr int kTicketStride = 16;           // one 128-byte line per worker's (64-bit) counter
constexpr int kSymMax = 128;              // table storage (QGX_MAX_SYM = 127 entries used at most)

// tau lookup: one cell per 1/16, 1/32 or 1/64 octave (by the size of the level table: a cell must not
// hold two levels) over 24 octaves below 1, plus the cell of u = 1.
constexpr int kCellOct = 24;
constexpr int kCellMantMax = 6;
constexpr int kCellsMax = (kCellOct << kCellMantMax) + 1;    // 1537
constexpr int kCellsPadMax = 1540;
inline __host__ __device__ int cell_mant(uint32_t n_sym) { return n_sym <= 33u ? 4 : n_sym <= 65u ? 5 : 6; }
// Bytes between the two sign halves of the encoder's level rows in LDS, by cell size (that is, by the
// largest table of the class): a power of two that the kernel knows at compile time, so that the sign of
// a coordinate picks its half with a shift and a mask by constants.
inline __host__ __device__ constexpr uint32_t lev_stride_of(int mant) { return mant == 4 ? 1024u : 2048u; }
inline __host__ __device__ constexpr uint32_t lev_sign_shift_of(int mant) { return mant == 4 ? 21u : 20u; }
inline __host__ __device__ int cell_count(int mant) { return (kCellOct << mant) + 1; }
inline __host__ __device__ int cell_count_padded(int mant) { return (cell_count(mant) + 3) / 4 * 4; }
constexpr int kLevRegion = kSymMax * 16;                // bytes between the two sign halves of lev2

constexpr int kDlutBits = kMaxCode;       // decode window
constexpr int kDlut = 1 << kDlutBits;     // 8192 entries

// The decode table is indexed by the next 13 stream bits read as a number with the FIRST bit on top,
// so the windows that start with one code word are neighbours: lanes that parse the same symbol read
// the same or adjacent entries, whatever follows the word in their streams.
constexpr uint32_t kDlutReject = 0x8000u; // no code word starts this window: flag, one bit long, symbol 0
// When the first kWideBits bits of a code word always tell which word it is (every word at most that
// long, or longer ones that differ from each other earlier: Elias' code up to 63 symbols), a second
// table indexed by the next kWideBits stream bits (first bit on top as well) holds the level value
// beside the bit count, so that one 8-byte look-up per symbol replaces the entry look-up and the level
// look-up (same footprint: 2^11 entries of 8 bytes).  Its counts are MINUS the symbol's bits, sign
// included, as a 32-bit number and nothing else: the parse counts downwards, and sums of these entries
// are its shift counts as they are.  Its reject entry is minus one bit with bit 15 cleared.
constexpr int kWideBits = 11;
constexpr int kWide = 1 << kWideBits;
constexpr uint32_t kWideReject = 0xFFFF7FFFu;

// Device-resident tables: rebuilt on the device whenever the level table or the code changes.
struct Tables {
    // lev2[sg][j] = {l_j, (l_{j+1}-l_j)*2^-24, E(j, sg), E(j+1, sg)}: everything the rounding of a
    // coordinate with sign sg between levels j and j+1 needs.  E(idx, sg) = code word of idx with the
    // sign bit appended (idx != 0), first-written bit in bit 0, total length << 16.
    float4 lev2[2][kSymMax];
    // cell[c] = {B, a0 | a1 << 16} for the c-th cell of u (cell_mant(n_sym) mantissa bits per octave): a0 = byte offset in lev2 of the row of
    // the last level <= the cell's lower edge; B = the level inside the cell (+inf if none), a1 = the
    // row to use when u >= B.  Exact only if no cell holds two levels (cell_exact).
    float2 cell[kCellsPadMax];
    float lval[kSymMax];        // l_j
    float levels[kSymMax];      // the table as set or fitted (source of the ones above)
    uint32_t code[kSymMax];     // code word (first-written bit in bit 0) | length << 16, no sign
    uint32_t n_sym;
    uint32_t code_kind;
    uint32_t cell_exact;
    uint32_t pad_;
    // dlut[next 13 stream bits, first bit on top] = (bits of the symbol incl. sign - 1) | (4 * idx) << 4,
    // or kDlutReject
    uint16_t dlut[kDlut];
    // dlutw[next 11 stream bits, first bit on top] = {-(bits of the symbol incl. sign), bits of l_idx}, or
    // {kWideReject, 0}; wide_ok tells whether 11 bits identify every code word
    uint2 dlutw[kWide];
    uint32_t wide_ok;
    uint32_t pad2_[3];
};

// Scalars of the iteration; lives in device memory, read by kernels, copied out on request.
struct Scalars {
    double S;                   // sum of squared half-step differences (Theorem 3)
    double gamma;               // K / sqrt(1 + S)
    unsigned long long t;       // iteration counter, starts at 1
    unsigned long long total_bits;
    float gamma_f;              // gamma rounded to binary32, what the update kernels multiply by
    unsigned int err;           // QGX_EBIT_*
    unsigned int pad_[2];
    unsigned long long avg_count;   // first half-steps added to the running sum since its reset
};

struct Layout {                 // device pointers into one allocation
    const uint32_t* bucket_start;   // [NB+1]
    const uint32_t* bucket_chunk0;  // [NB+1] first chunk of each bucket
    const uint32_t* chunk_start;    // [NC+1]
    const uint32_t* chunk_bucket;   // [NC] bucket of the chunk's first coordinate
    const uint32_t* ragged_chunk;   // [n_ragged] chunk positions with fewer than kChunk coordinates, ascending
    uint32_t NB, NC, K, d;
    uint32_t n_ragged;
    uint32_t max_ragged;            // coordinates of the longest of them
    uint32_t waves_per_bucket;      // ceil(bucket / kChunk)
    uint32_t uniform_bucket;        // bucket size if there is one segment (offsets are then arithmetic), else 0
    // Buckets of 256, 512, 1024 or 2048 coordinates share chunks: a segment is cut into runs of kChunk
    // coordinates that hold whole buckets.  bucket_shift = log2(bucket) there and 31 otherwise, so that
    // coordinate i of chunk c lies in bucket chunk_bucket[c] + (i >> bucket_shift) with either kind.
    uint32_t shared_chunks;
    uint32_t bucket_shift;
};

inline bool shares_chunks(uint32_t bucket) { return bucket == 256u || bucket == 512u || bucket == 1024u || bucket == 2048u; }

// Fused: V from memory; Generate: V formed on the fly from the game's operator and noise (GameArgs)
enum class EncMode { Fused, QuantOnly, EncodeOnly, Generate };
enum class DecMode { Decode, Average, Half0, Half1 };

// The synthetic stochastic oracle of the large quadratic game (Section 2: g(z; omega) = A(z) + U(z; omega)):
// F(z) = M z + b, M block diagonal with 2x2 blocks [[mu, a_j], [-a_j, mu]] on the pairs (2j, 2j+1), plus
// sigma times standard normal noise drawn per (worker, call, coordinate).
struct GameArgs {
    const float* z;             // [d]
    const float* a;             // [d / 2]
    const float* b;             // [d]
    float mu, sigma;
    uint32_t seed_lo, seed_hi;  // key of the noise draws
    float* V_out;               // [K][d] or null: the dual vectors as the fused coding kernel formed them (for tests)
};

struct EncodeArgs {
    const float* V;             // [K][d]           (Fused, QuantOnly)
    const float* norms_in;      // [K][NB] or null
    float* norms_out;           // [K][NB] or null
    uint8_t* sym_out;           // [K][d]           (QuantOnly)
    const uint8_t* sym_in;      // [K][d]           (EncodeOnly)
    uint32_t* chunk_off;        // [K][NC+1]
    uint16_t* sub_end;          // [K][NC][kSubs]
    uint32_t* payload;          // [K][cap]
    uint64_t cap_words;
    unsigned long long* scan_state;  // [K][NB * parts] look-back words
    unsigned long long* xch;         // [K][NB][parts][2][2] partial norms of split buckets, epoch-tagged
    uint32_t parts;             // workgroups per bucket: 1, or ceil(waves_per_bucket / 4) when that exceeds 4
    unsigned long long* tickets;   // [K] ever-increasing tickets, kTicketStride counters apart
    uint32_t seed_lo, seed_hi, call_id;
    uint32_t call_mode;         // 0: call_id as given; 1, 2: 2(t-1), 2(t-1)+1 from the iteration counter on the device
    int norm_kind;
    // LDS plan of the launch (bytes): [cell][lev: two sign halves lev_stride apart][misc][stage x waves]
    uint32_t cell_mant;         // cell_mant(n_sym) of the table in use
    uint32_t lev_stride;        // lev_stride_of(cell_mant): a power of two >= 16 * n_sym
    uint32_t lev_bytes;         // lev_stride + 16 * n_sym: the second half ends with its last row
    uint32_t sign_shift;        // (bits of v) >> sign_shift puts the sign bit on lev_stride
    uint32_t stage_bytes;       // per wave, multiple of 16, covers 4096 symbols of the longest code + sign
    uint32_t slot_words;        // 0: compact placement (ordered scan); else chunk c goes to c * slot_words
    GameArgs game;              // EncMode::Generate
};

struct DecodeArgs {
    const float* norms;  const uint32_t* chunk_off;  const uint16_t* sub_end;  const uint32_t* payload;
    uint64_t cap_words;
    // previous half-step's streams (Half1 only; payload_p null => all-zero vectors)
    const float* norms_p;  const uint32_t* chunk_off_p;  const uint16_t* sub_end_p;  const uint32_t* payload_p;
    uint64_t cap_words_p;
    const Tables* tab_p;        // tables the previous streams were coded with, null when they are the current ones
    float* out;                 // Decode: Vhat [K][d]; Average: mean [d]; Half0: X_{t+1/2} [d]
    float* Y;                   // [d] dual state (Half0 reads, Half1 updates)
    const float* anchor;        // [d] or null
    double* s_partial;          // [NC] per-chunk partial of S (Half1)
    double* x_sum;              // [d] running sum of the X_{t+1/2} or null (Half0 adds its output)
    uint32_t stage_words;       // most words a chunk can take with the code in use (multiple of 4)
    uint32_t stage_stride;      // words of one LDS staging buffer (padded layout plus slack)
    uint32_t sym_bits;          // most bits a symbol can take with the codes in use (longest word + sign)
    uint32_t rag_words;         // the same two for the layout's longest chunk of fewer than 4096 coordinates,
                                // plus room for 32 symbols and a window past its end
    uint32_t rag_stride;
    uint32_t wide;              // the 8-byte decode table of the current streams' code is valid (Tables::wide_ok)
    uint32_t ksplit;            // fused modes: 1, 2 or 4 waves per full position, a run of the workers each
};

// The dynamic LDS a kernel may be launched with is an attribute of the kernel on a device, raised with
// hipFuncSetAttribute.  One object per kernel (a function-local static of its launcher) remembers, per
// device, what was last granted, and asks again only when a launch needs more; contexts on several
// threads and devices share it, hence the lock.
struct LdsLimit {
    static constexpr int kDevices = 64;
    std::atomic<size_t> granted[kDevices];
    std::mutex lock;
    hipError_t ensure(const void* kernel, size_t bytes)
    {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev < 0 || dev >= kDevices) return hipErrorInvalidDevice;
        if (bytes <= granted[dev].load(std::memory_order_acquire)) return hipSuccess;
        std::lock_guard<std::mutex> hold(lock);
        if (bytes <= granted[dev].load(std::memory_order_relaxed)) return hipSuccess;
        e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
        if (e == hipSuccess) granted[dev].store(bytes, std::memory_order_release);
        return e;
    }
};

hipError_t launch_build_tables(Tables* tab, hipStream_t st);
hipError_t launch_encode(EncMode mode, const Layout& lay, const Tables* tab, Scalars* sc, const EncodeArgs& a,
                         hipStream_t st);
hipError_t launch_decode(DecMode mode, const Layout& lay, const Tables* tab, Scalars* sc, const DecodeArgs& a,
                         hipStream_t st);
hipError_t launch_finish_half1(const Layout& lay, Scalars* sc, const double* s_partial, const float* Y,
                               const float* anchor, float* X_out, hipStream_t st);
hipError_t launch_state_init(const Layout& lay, Scalars* sc, float* Y, float* anchor, const float* X1,
                             hipStream_t st);
hipError_t launch_average(uint32_t d, const double* x_sum, const Scalars* sc, float* out, hipStream_t st);
hipError_t launch_average_reset(uint32_t d, double* x_sum, Scalars* sc, hipStream_t st);
hipError_t launch_average_count(Scalars* sc, hipStream_t st);
hipError_t launch_state_set(Scalars* sc, double S, unsigned long long t, uint32_t K, hipStream_t st);
hipError_t launch_sum_bits(const Layout& lay, const uint16_t* sub_end, Scalars* sc, hipStream_t st);
hipError_t launch_histogram(const Layout& lay, const float* V, int norm_kind, uint32_t n_bins, double* partial,
                            uint32_t n_partial, double* hist, Scalars* sc, hipStream_t st);
hipError_t launch_compact(const Layout& lay, const uint16_t* sub_end, const uint32_t* in_off, const uint32_t* in_payload,
                          uint64_t in_cap, uint32_t* out_off, uint32_t* out_payload, uint64_t out_cap, Scalars* sc,
                          hipStream_t st);
hipError_t launch_fit(Tables* tab, const double* hist, uint32_t n_bins, uint32_t sweeps, hipStream_t st);
hipError_t launch_fit_code(Tables* tab, const double* hist, uint32_t n_bins, uint32_t max_len, double* p_out,
                           hipStream_t st);
uint32_t histogram_groups(const Layout& lay);
hipError_t launch_game_operator(const GameArgs& g, uint32_t d, float* F_out, hipStream_t st);
hipError_t launch_game_dual_vectors(const GameArgs& g, uint32_t d, uint32_t K, uint32_t call_id, uint32_t call_mode,
                                    const Scalars* sc, float* V_out, hipStream_t st);
constexpr uint32_t kNormBlocks = 1024;     // partial sums of qgx_norm2
hipError_t launch_norm2(const float* x, uint64_t n, double* partial /*[kNormBlocks + 1]*/, hipStream_t st);
hipError_t launch_game_gap(const GameArgs& g, const float* centre, double R, uint64_t d,
                           double* partial /*[2 kNormBlocks + 2]: the result in the last*/, hipStream_t st);
constexpr uint32_t kMetricBlocks = 256;    // partial sums per worker and figure of qgx_quantization_metrics
hipError_t launch_metrics(const float* V, const float* Vhat, uint64_t d, uint32_t K, double* partial /*[K][3][kMetricBlocks]*/,
                          double* result /*[K][3]*/, hipStream_t st);

}  // namespace qgx
