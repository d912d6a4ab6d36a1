/*
 * qgx.h -- C ABI of the MI355X (gfx950) Q-GenX hot-path library.
 *
 * The calls follow the paper's own statement of the method (arXiv 2308.09187):
 *   Q_l(v), random quantisation of normalised coordinates     Definition 1
 *   CODE o Q / DEQ o CODE, norm + sign + integer code Psi       Section 3.2, Appendix J (Encoding)
 *   adaptive levels from the weighted empirical CDF             Section 3.3, eq. (QAda)
 *   aggregate and the two extra-gradient half-steps             Algorithm 1, eq. (Q-GenX)
 *   adaptive step size gamma_t                                  Theorem 3 / Theorem 4
 *
 * Conventions
 *   - No C++ types, no exceptions.  Every function returns a qgx_status (negative = error); after
 *     an error the context stays usable and outputs are unspecified but never written out of bounds.
 *   - Pointers marked DEVICE are caller-owned HIP device memory on the device that was current in
 *     qgx_create; pointers marked HOST are ordinary host memory.  Device buffers must be 16-byte
 *     aligned.  The library allocates only inside qgx_create (tables, state, scratch) and frees in
 *     qgx_destroy.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue work on
 *     it and return; only the calls documented as synchronising wait for it.
 *   - The K workers of the paper are a batch: V is [K][d] worker-major, contiguous, binary32.
 *   - Errors found on the device (non-finite bucket, stream capacity, malformed stream) set bits in
 *     a device error word that qgx_poll_error returns and clears.
 *   - Determinism: the same (config, levels, V, call_id) gives a byte-identical qgx_stream.
 *   - A context serves one caller at a time: its calls are issued from one thread, in order.
 *   - HIP graphs: the coding, decoding and half-step calls may be captured and the graph replayed:
 *     their kernels take everything that changes between iterations (Y, S, gamma, t, the running
 *     sum and its count, the tags and ticket counters that order workgroups, and with
 *     QGX_CALL_FIRST_HALF / QGX_CALL_SECOND_HALF the call number) from device memory.  Run them once
 *     before capturing (the first launch of a kernel sets its attributes).  Every call works on
 *     `stream` alone.
 *
 * Stream container (the paper fixes only the bit string {0,1}*; the container is this library's):
 *   Coordinates of one worker are cut into segments (tensors), segments into buckets of at most
 *   `bucket` coordinates (own norm each; the last bucket of a segment may be short), buckets into
 *   chunks of at most QGX_CHUNK coordinates; buckets of 256, 512, 1024 or 2048 coordinates share
 *   chunks instead (a segment is cut into runs of QGX_CHUNK coordinates, each holding whole buckets),
 *   so that a chunk's tables and the kernels' lanes are not left mostly empty.  A chunk's bits are: for every coordinate in index
 *   order the code word Psi(idx), first-written bit first, then one sign bit (1 = negative) iff
 *   idx != 0.  Stream bit p of a chunk lives in 32-bit word p>>5, bit p&31.  Every chunk starts at
 *   a multiple of 4 words; pad bits are 0.
 *     norms     [K][NB]       binary32 norm of every bucket (C_b = 32 bits), 0 for a rejected bucket
 *     chunk_off [K][NC+1]     word offset of chunk c inside worker k's payload; entry NC = words used
 *     sub_end   [K][NC][128]  bit offset, from the chunk start, one past the last bit of the j-th run
 *                             of QGX_SUB coordinates (entries past the chunk's last run repeat the
 *                             chunk's bit length); makes the decode parallel
 *     payload   [K][payload_words_per_worker]
 *   Psi is Elias' recursive (omega) code of idx+1 (QGX_CODE_ELIAS_OMEGA), or a caller-supplied
 *   prefix code table (QGX_CODE_TABLE).
 *   Two placements of the chunks inside a worker's payload:
 *     compact (slot_words = 0): chunk_off is the exclusive scan of the chunk sizes in chunk order, the
 *       payload has no gaps and chunk_off[k][NC] is the number of words used: the form to ship;
 *     slotted (slot_words > 0): chunk c starts at c * slot_words, slot_words = what qgx_slot_words
 *       reports; no workgroup waits for another's output, so coding is faster; the bits of every
 *       chunk are the same as in the compact form, and qgx_compact turns one into the other.
 *   Buckets of more than 16384 coordinates are coded by several workgroups that exchange their
 *   partial norms (for K <= 64; one large workgroup per bucket beyond that).
 *   A chunk's size in words is always ceil(sub_end[k][c][127] / 32) rounded up to a multiple of 4.
 */
#ifndef QGX_H
#define QGX_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define QGX_CHUNK 4096u      /* coordinates per chunk */
#define QGX_SUB 32u          /* coordinates per sub-chunk table entry */
#define QGX_SUBS 128u        /* sub-chunk table entries per chunk */
#define QGX_MAX_BUCKET 65536u
#define QGX_MAX_SYM 127u     /* largest level table (l_0 .. l_{s+1}) */
#define QGX_MAX_BINS 4096u
#define QGX_MAX_CODE_BITS 13u
#define QGX_FIT_CODE_BITS 11u  /* longest word of a code made by qgx_fit_code */
#define QGX_TABLES 2         /* level tables (each with its code) a context holds */
#define QGX_STATIC_MAX_CHUNKS 65536u  /* most chunks per worker qgx_eg_step_static takes (2^28 coordinates) */

typedef struct qgx_ctx qgx_ctx;

typedef enum {
    QGX_OK = 0,
    QGX_ERR_ARG = -1,        /* null pointer, zero size, misaligned or out-of-range argument */
    QGX_ERR_LEVELS = -2,     /* level table not 0 = l_0 < l_1 < ... < l_last = 1 */
    QGX_ERR_CAPACITY = -3,   /* a worker's stream does not fit payload_words_per_worker */
    QGX_ERR_STREAM = -4,     /* malformed stream: unknown code word, overrun, table mismatch */
    QGX_ERR_NONFINITE = -5,  /* a bucket held a non-finite value; it was coded as all-zero */
    QGX_ERR_HIP = -6,        /* a HIP runtime call failed */
    QGX_ERR_STATE = -7       /* call order (levels not set, state not initialised) or internal wait expired */
} qgx_status;

/* bits of the device error word returned by qgx_poll_error */
#define QGX_EBIT_CAPACITY 1u
#define QGX_EBIT_STREAM 2u
#define QGX_EBIT_NONFINITE 4u
#define QGX_EBIT_STATE 8u

/* q of ||v||_q (Definition 1: q in Z_+): 0 stands for the q -> infinity limit, 2 has a route of its
 * own, any other q in 1..QGX_MAX_NORM_Q is (sum |v_i|^q)^(1/q) accumulated in binary64. */
typedef enum { QGX_NORM_LINF = 0, QGX_NORM_L2 = 2 } qgx_norm;
#define QGX_MAX_NORM_Q 64
typedef enum { QGX_CODE_ELIAS_OMEGA = 0, QGX_CODE_TABLE = 1 } qgx_code; /* Psi, Appendix J */
/* call_id values that stand for "from the iteration counter on the device" (see qgx_quantize) */
#define QGX_CALL_FIRST_HALF 0xFFFFFFFEu
#define QGX_CALL_SECOND_HALF 0xFFFFFFFFu

typedef struct {
    uint64_t d;                   /* coordinates per worker, 1 <= d < 2^31 */
    uint32_t K;                   /* workers, 1 <= K <= 65535; K * buckets and K * chunks per worker below 2^31 */
    uint32_t bucket;              /* coordinates per bucket, multiple of 4, <= QGX_MAX_BUCKET */
    uint32_t n_segments;          /* 0 or 1 => one segment of length d */
    const uint64_t* segment_len;  /* HOST, n_segments lengths summing to d; all but the last multiples of 4 */
    int32_t norm;                 /* qgx_norm, or another q in 1..QGX_MAX_NORM_Q */
    int32_t code;                 /* qgx_code */
    uint64_t seed;                /* key of the counter-based generator */
} qgx_config;

/* One CODE o Q result for all K workers.  All pointers DEVICE, caller-owned. */
typedef struct {
    float* norms;                       /* [K][NB] */
    uint32_t* chunk_off;                /* [K][NC+1] */
    uint16_t* sub_end;                  /* [K][NC][QGX_SUBS] */
    uint32_t* payload;                  /* [K][payload_words_per_worker] */
    uint64_t payload_words_per_worker;  /* multiple of 4 */
    uint64_t slot_words;                /* 0 = compact placement; else the fixed chunk slot (see above) */
} qgx_stream;

/* Creates a context on the current device: validates the configuration, builds the bucket and chunk
 * tables, allocates state (Y, anchor), tables and scratch.  Synchronises the device. */
qgx_status qgx_create(qgx_ctx** out, const qgx_config* cfg);
void qgx_destroy(qgx_ctx* ctx);

/* Sizes a caller needs to allocate a qgx_stream: buckets and chunks per worker and the payload
 * words per worker that can never overflow (14 bits per coordinate plus chunk padding). */
qgx_status qgx_stream_sizes(const qgx_ctx* ctx, uint64_t* n_buckets, uint64_t* n_chunks,
                            uint64_t* worst_case_payload_words);

/* The chunk slot of the slotted placement for the level table and code in use: the words a full chunk
 * can take at most.  A slotted stream needs payload_words_per_worker >= n_chunks * slot_words. */
qgx_status qgx_slot_words(const qgx_ctx* ctx, uint64_t* slot_words);

/* Rewrites a slotted stream as a compact one (same bits per chunk, exclusive-scan offsets).
 * `out` must be compact (slot_words = 0) and may not alias `in`. */
qgx_status qgx_compact(qgx_ctx* ctx, const qgx_stream* in, qgx_stream* out, void* stream);

/* A context holds QGX_TABLES level tables, each with its own code: Section 3.3 notes that the dual
 * vectors of the two half-steps, V_t and V_{t+1/2}, may be given level sequences of their own.
 * `table` names the one that every call from here on sets, fits, reads, codes with and decodes with;
 * `prev_table` the one the `prev` streams of qgx_eg_step(half = 1) were coded with.  Both are 0
 * until this is called.  Slot sizes (qgx_slot_words) cover the longest code of the tables set, so
 * streams of either table can share their buffers' geometry.  Host-side only; nothing is launched. */
qgx_status qgx_select_table(qgx_ctx* ctx, uint32_t table, uint32_t prev_table);

/* Level table l of Definition 1: levels_host HOST [n_sym], 2 <= n_sym <= QGX_MAX_SYM,
 * 0 = l[0] < ... < l[n_sym-1] = 1 (QGX_ERR_LEVELS otherwise).  Synchronises `stream`. */
qgx_status qgx_set_levels(qgx_ctx* ctx, const float* levels_host, uint32_t n_sym, void* stream);
/* Reads the current table back (after qgx_fit_levels).  levels_host HOST [QGX_MAX_SYM]. Synchronises. */
qgx_status qgx_get_levels(qgx_ctx* ctx, float* levels_host, uint32_t* n_sym, void* stream);

/* Psi as a prefix code table (Appendix J: Huffman or any other prefix code), only with
 * QGX_CODE_TABLE: code_len HOST [n_sym] in 1..QGX_MAX_CODE_BITS, code_bits HOST [n_sym] with the
 * first-written bit in bit 0.  Must be prefix-free (QGX_ERR_ARG otherwise) and cover the level
 * table in use.  Synchronises `stream`. */
qgx_status qgx_set_code_table(qgx_ctx* ctx, const uint8_t* code_len, const uint32_t* code_bits,
                              uint32_t n_sym, void* stream);

/* Q_l(v) of Definition 1, bucket by bucket (norm, normalise, level below, stochastic rounding).
 *   V         DEVICE [K][d] binary32
 *   call_id   distinguishes quantisation calls under one seed (e.g. 2t + half): coordinate i of
 *             worker k draws word (i mod 4) of Philox4x32-10(key = seed, counter = (i/4, 0, k, call_id)),
 *             top 24 bits as r in [0,1); rounds up iff r * (l_{j+1}-l_j) < u - l_j.
 *             QGX_CALL_FIRST_HALF / QGX_CALL_SECOND_HALF instead of a number: the kernel takes
 *             2(t-1) resp. 2(t-1)+1 (mod 2^32) with t the iteration counter of the context's state
 *             as it is on the device when the kernel runs (1 after qgx_state_init, advanced by every
 *             second half-step), so that a captured HIP graph of an iteration draws fresh numbers
 *             at every replay.
 *   norms_in  DEVICE [K][NB] or NULL: non-negative norms to use instead of computing them (a common
 *             scale for several workers, say); coordinates that exceed it are clamped to u = 1
 *   norms_out DEVICE [K][NB]: the norm used (0 for a rejected bucket)
 *   sym       DEVICE [K][d] bytes: level index in bits 0..6, sign bit of v in bit 7 */
qgx_status qgx_quantize(qgx_ctx* ctx, const float* V, uint32_t call_id, const float* norms_in,
                        float* norms_out, uint8_t* sym, void* stream);

/* CODE of Section 3.2 / Appendix J applied to symbols from qgx_quantize.  `norms` DEVICE [K][NB] is
 * copied into out->norms unless it is the same pointer. */
qgx_status qgx_encode(qgx_ctx* ctx, const float* norms, const uint8_t* sym, qgx_stream* out, void* stream);

/* CODE o Q in one pass over V (the fast path): V crosses HBM once, symbols never leave registers.
 * norms_in as in qgx_quantize (NULL = compute). */
qgx_status qgx_quantize_encode(qgx_ctx* ctx, const float* V, uint32_t call_id, const float* norms_in,
                               qgx_stream* out, void* stream);

/* DEQ o CODE: Vhat DEVICE [K][d], vhat_i = +-(norm * l_idx). */
qgx_status qgx_decode(qgx_ctx* ctx, const qgx_stream* in, float* Vhat, void* stream);

/* Aggregate of Algorithm 1: mean DEVICE [d] = (1/K) sum_k DEQ(CODE_k), decoded on the fly.
 * The K values of a coordinate are added in binary32, in worker order; on layouts with too few
 * chunks to fill the GPU the workers are split in two or four runs (as equal as K allows, the
 * longer ones first), each added in order, and the runs' sums added in order (the same in
 * qgx_eg_step).  The number of runs follows from the layout, K and the device, so results repeat bit
 * for bit (qgx_debug_set_waves_per_position overrides the choice, for tests and timing). */
qgx_status qgx_decode_average(qgx_ctx* ctx, const qgx_stream* in, float* mean, void* stream);

/* Adaptive levels, eq. (QAda): weighted histogram of the normalised coordinates of V (each bucket
 * weighted by its squared norm) over n_bins bins on the binary32 grid (64 bins per octave, n_bins a
 * multiple of 64, <= QGX_MAX_BINS), then `sweeps` passes that move one interior level at a time to
 * the stationary point between its neighbours (the smallest one where the condition holds on a whole
 * interval, i.e. where the histogram has no mass; the lower neighbour itself when there is none between
 * the two), starting from the current table; levels stay in binary64 between the passes and are rounded
 * to binary32, gaps at least 2^-24, at the end.  n_sym must equal the current table's length.  The new table replaces the context's.  hist_out DEVICE [n_bins]
 * doubles or NULL. */
qgx_status qgx_fit_levels(qgx_ctx* ctx, const float* V, uint32_t n_sym, uint32_t n_bins, uint32_t sweeps,
                          double* hist_out, void* stream);

/* Psi from estimated symbol probabilities (Appendix J: Huffman coding when the distribution of the
 * symbols can be estimated), only with QGX_CODE_TABLE.  p_j of Proposition 1 is taken from the
 * histogram of the last qgx_fit_levels call (with sweeps = 0 that call only measures: a table whose
 * gaps are at least 2^-24 stays as it is) and the current level table; the code is the optimal prefix code for the weights
 * round(p_j 2^32), at least 1, with no word longer than QGX_FIT_CODE_BITS (Huffman's code whenever
 * that limit is slack; 11 bits and not the 13 a caller's table may have, so that the decoders can
 * always take their one-look-up table), words numbered canonically by (length, index).  It replaces the context's
 * code table; the slot size of slotted streams follows its longest word (qgx_slot_words).
 * p_host HOST [n_sym] doubles, code_len_host HOST [n_sym], code_bits_host HOST [n_sym] (layout as in
 * qgx_set_code_table), each may be NULL.  Synchronises `stream`.
 * QGX_ERR_STATE without a histogram, a level table, or QGX_CODE_TABLE. */
qgx_status qgx_fit_code(qgx_ctx* ctx, double* p_host, uint8_t* code_len_host, uint32_t* code_bits_host, void* stream);

/* The caller's side of an iteration for the large quadratic game, as calls of the library, so that a whole
 * iteration can stay on the device (Section 2: the stochastic oracle g(z; omega) = A(z) + U(z; omega) with
 * E U = 0 and bounded variance; the residual ||A(x)|| the convergence theorems are read against).
 * The operator is F(z) = M z + b, M block diagonal with 2x2 blocks [[mu, a_j], [-a_j, mu]] on the coordinate
 * pairs (2j, 2j+1): strongly monotone with modulus mu.  Worker k's dual vector in call `call_id` is
 * F(z) + sigma N with N standard normal, independent over workers, calls and coordinates: coordinates
 * 4g..4g+3 take Philox4x32-10(key = noise_seed, counter = (g, 1, k, call_id)), words (w0, w1) and (w2, w3)
 * each give two draws by Box-Muller with u1 = (2 (w >> 9) + 1) 2^-24, u2 = (w' >> 8) 2^-24.  All pointers
 * DEVICE; z and b 16-byte aligned, a 8-byte aligned; d a multiple of 4. */
typedef struct {
    const float* z;       /* [d] the point */
    const float* a;       /* [d / 2] couplings of the 2x2 blocks */
    const float* b;       /* [d] */
    float mu;             /* modulus of strong monotonicity (diagonal of every block) */
    float sigma;          /* standard deviation of the noise, >= 0 */
    uint64_t noise_seed;  /* key of the noise draws */
} qgx_game;

/* F_out DEVICE [d] = F(z). */
qgx_status qgx_game_operator(qgx_ctx* ctx, const qgx_game* game, float* F_out, void* stream);
/* V_out DEVICE [K][d]: the K workers' dual vectors.  call_id as in qgx_quantize (the two special values too). */
qgx_status qgx_game_dual_vectors(qgx_ctx* ctx, const qgx_game* game, uint32_t call_id, float* V_out, void* stream);
/* CODE o Q of those same dual vectors without writing them to memory and reading them back: the coding
 * kernel forms each coordinate where qgx_quantize_encode would load it (the rounding draws use the context's
 * seed and the same call_id; the noise draws differ from them in key and counter).  The stream equals, bit
 * for bit, that of qgx_quantize_encode on the output of qgx_game_dual_vectors.  V_out DEVICE [K][d] or NULL:
 * the dual vectors as formed, for checking.  One segment, buckets that do not share chunks, L2 or
 * L-infinity norm (QGX_ERR_ARG otherwise). */
qgx_status qgx_quantize_encode_game(qgx_ctx* ctx, const qgx_game* game, uint32_t call_id, qgx_stream* out,
                                    float* V_out, void* stream);
/* result_host HOST <- ||x||_2 of x DEVICE [n], squares summed in binary64 in a fixed order (the residual
 * ||F(x)|| once F(x) has been formed with qgx_game_operator, say at the ergodic average).  Synchronises. */
qgx_status qgx_norm2(qgx_ctx* ctx, const float* x, uint64_t n, double* result_host, void* stream);

/* result_host HOST <- the restricted gap of eq. (Gap), Section 2, for the game's operator and the candidate
 * game->z over the closed ball of `radius` around centre (DEVICE [d], or NULL = the origin):
 * sup_{x in ball} <F(x), z - x>, the quantity the convergence theorems bound at the ergodic average.  For this
 * operator the supremum has a closed form (a concave quadratic of equal curvature mu in all directions: the
 * maximiser is the point of the ball nearest to (M^T z - b) / (2 mu)); binary64 sums in a fixed order.
 * mu > 0 (QGX_ERR_ARG otherwise); sigma and noise_seed are not used.  Synchronises. */
qgx_status qgx_game_gap(qgx_ctx* ctx, const qgx_game* game, const float* centre, double radius, double* result_host,
                        void* stream);

/* What one call of Q did, per worker (Section 3.1; a diagnostic beside the hot path).  V DEVICE [K][d] the vectors
 * given to qgx_quantize / qgx_quantize_encode, Vhat DEVICE [K][d] their decoded images (qgx_decode).  HOST
 * arrays of K, each optional (NULL): nonzeros = ||Q(v_k)||_0, whose expectation is (1 - p_0) d (Lemma 2);
 * sq_error = ||Q(v_k) - v_k||^2, whose expectation is eq. (var) and which Theorem 1 bounds by
 * epsilon_Q ||v_k||^2 on average; sq_norm = ||v_k||^2.  Sums in binary64 in a fixed order.  Synchronises. */
qgx_status qgx_quantization_metrics(qgx_ctx* ctx, const float* V, const float* Vhat, uint64_t* nonzeros_host,
                                    double* sq_error_host, double* sq_norm_host, void* stream);

/* State of eq. (Q-GenX): Y_1 = 0, S = 0, t = 1, gamma_1 = K, anchor = X1 (DEVICE [d] or NULL = 0).
 * The paper's X_{t+1} = gamma_{t+1} Y_{t+1} is the X1 = 0 case of X_{t+1} = X1 + gamma_{t+1} Y_{t+1}. */
qgx_status qgx_state_init(qgx_ctx* ctx, const float* X1, void* stream);

/* One half-step of eq. (Q-GenX), decoding the K streams on the fly.
 *   half = 0: X_out DEVICE [d] <- X_t - (gamma_t/K) sum_k Vhat_{k,t},  X_t = X1 + gamma_t Y_t.
 *             `cur` holds CODE(Q(V_{k,t})); prev must be NULL.
 *   half = 1: Y <- Y - (1/K) sum_k Vhat_{k,t+1/2};  S += sum_k ||Vhat_{k,t} - Vhat_{k,t+1/2}||^2;
 *             gamma_{t+1} = K / sqrt(1 + S);  t += 1;  X_out (may be NULL) <- X1 + gamma_{t+1} Y.
 *             `cur` holds the t+1/2 streams, `prev` the t streams (NULL: Vhat_{k,t} = 0, the
 *             dual-averaging case).  `cur` must have been coded with the selected table as it is
 *             now, `prev` with the table qgx_select_table names for it. */
qgx_status qgx_eg_step(qgx_ctx* ctx, int half, const qgx_stream* cur, const qgx_stream* prev,
                       float* X_out, void* stream);

/* qgx_eg_step for callers that may not allocate device memory and want the guarantee in the interface:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same kernels, same results bit for bit as qgx_eg_step; the one difference is where the second
 * half-step keeps its scratch, the per-chunk partial sums of S: not in memory that qgx_create allocated
 * but in a fixed array inside the library's device image (8 * QGX_STATIC_MAX_CHUNKS = 512 KiB per GPU,
 * held until the process ends; its address on a device is looked up once, in the first qgx_create on
 * that device).  The call itself allocates and frees nothing.
 *   - QGX_ERR_CAPACITY if the layout has more than QGX_STATIC_MAX_CHUNKS chunks per worker (qgx_eg_step
 *     has no such limit); QGX_ERR_STATE if the context's device is not the current one.
 *   - All contexts on one GPU share the array: every call overwrites the entries 0 .. n_chunks - 1 it
 *     then reads and relies on nothing a previous call left, but two such calls that overlap on one
 *     GPU (different streams or threads) race on it.  Calls on one stream, or ordered by events, do not. */
qgx_status qgx_eg_step_static(qgx_ctx* ctx, int half, const qgx_stream* cur, const qgx_stream* prev,
                              float* X_out, void* stream);

/* Scalars of the iteration.  Any pointer may be NULL.  Synchronises `stream`. */
qgx_status qgx_get_scalars(qgx_ctx* ctx, double* S, double* gamma, uint64_t* t, void* stream);

/* Bits of a coded stream over all workers: code words and signs, without padding and without the
 * 32 bits per bucket for the norm (the quantity Theorem 2 bounds, less C_b per bucket).  Synchronises. */
qgx_status qgx_stream_bits(qgx_ctx* ctx, const qgx_stream* coded, uint64_t* total_bits, void* stream);

/* Test and timing hook: the number of waves that share a full chunk position in the decoding calls
 * (1, 2 or 4; ignored when above K), or 0 to go back to the library's own rule.  Host-side only. */
qgx_status qgx_debug_set_waves_per_position(qgx_ctx* ctx, int waves);

/* Copies the dual state out (checkpoint) or in (resume).  Y, anchor DEVICE [d]; NULL skips. */
qgx_status qgx_state_export(qgx_ctx* ctx, float* Y, float* anchor, void* stream);
qgx_status qgx_state_import(qgx_ctx* ctx, const float* Y, const float* anchor, double S, uint64_t t,
                            void* stream);

/* Ergodic average of the half-step iterates, X_bar = (1/T) sum_t X_{t+1/2} (the point the
 * convergence theorems bound; Section 2, Theorems 3 and 4).  qgx_average_reset(on = 1) clears a
 * binary64 running sum in the context (allocated at the first such call; this is the one call
 * besides qgx_create that allocates) and makes every later qgx_eg_step(half = 0) add its output to
 * it, at 16 more bytes of traffic per coordinate; on = 0 switches that off.
 * qgx_average_export: X_bar DEVICE [d] (or NULL) = sum / count, count = half-steps since the reset
 * (kept on the device, so that the half-steps of a replayed graph count; the call reads it back and
 * so synchronises `stream`). */
qgx_status qgx_average_reset(qgx_ctx* ctx, int on, void* stream);
qgx_status qgx_average_export(qgx_ctx* ctx, float* X_bar, uint64_t* count, void* stream);

/* Returns and clears the device error word (QGX_EBIT_*).  Synchronises `stream`. */
uint32_t qgx_poll_error(qgx_ctx* ctx, void* stream);

/* Human-readable text of the last host-side error of this context (never NULL). */
const char* qgx_last_error(const qgx_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* QGX_H */
