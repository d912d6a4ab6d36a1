/*
 * qgx_oracle.c -- TEST INFRASTRUCTURE, not the product.
 *
 * A plain, slow, scalar CPU statement of what the Q-GenX data-parallel hot
 * path computes, written from the paper (arXiv 2308.09187) one step at a time:
 *
 *   normalise + random quantisation Q_l(v)      Definition 1, Section 3.2
 *   CODE o Q  (norm, sign of non-zeros, Psi)    Section 3.2, Appendix J (Encoding)
 *   DEQ o CODE                                  Section 3.2, Appendix J
 *   mean over K workers + the two half-steps    Algorithm 1, eq. (Q-GenX)
 *   adaptive step size gamma_t                  Theorem 3 / Theorem 4
 *   adaptive levels from an empirical CDF       Section 3.3, eq. (QAda)
 *   symbol probabilities p_j                    Proposition 1
 *   Psi as an optimal prefix code on the p_j    Appendix J (Huffman), with a
 *                                               limit on the word length
 *
 * Only tests, the smoke check and the cpu_baseline leg of the benchmark may
 * call this file.  It shares no source, header, table or helper with the HIP
 * library; the random draws use a counter-based generator (Philox4x32-10,
 * Salmon et al., SC'11) that each side implements on its own.
 *
 * Pins (see tests/test_oracle_*.py): Philox known answers, exhaustive
 * enumeration of rounding outcomes for d <= 8, the closed-form variance of
 * eq. (var), the variance bound of Theorem 1, Lemma 2 (expected non-zeros),
 * exact expected code length, decode(encode(x)) == x, gamma_1 = K and
 * monotone gamma, the dual-averaging special case, the fine-level limit against
 * a textbook extra-gradient run, uniform-density => uniform levels for (QAda),
 * closed-form p_j on a uniform density and p_j against emitted symbol counts,
 * the optimal code against a textbook Huffman merge (cost and H <= E[L] <= H+1)
 * and, with the length limit active, against brute force over all lengths.
 *
 * parity unpinned: the container around the paper's bit string (chunk offset
 * table, sub-chunk table, 128-bit chunk alignment) is this project's own
 * format; the paper fixes only the symbol stream.  It is pinned by round trip
 * and by the strip-the-padding invariant only.
 *
 * Arithmetic: every decision that produces an integer (level index, rounding
 * up or down, histogram bin) is taken in IEEE binary32 with separately rounded
 * operations, because that is the precision the method's inputs live in and
 * both sides must take the same decision.  Everything that is a real number
 * (norm accumulation, mean, iterates, step size, level fitting) is binary64.
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_CH 4096u        /* coordinates per chunk                       */
#define ORC_SUB 32u         /* coordinates per sub-chunk                   */
#define ORC_SUBS 128u       /* sub-chunk table entries per chunk           */
#define ORC_ALIGN_WORDS 4u  /* chunk start alignment in 32-bit words       */

enum { ORC_NORM_LINF = 0, ORC_NORM_L2 = 2 };

/* ------------------------------------------------------------------------ */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as   */
/* easy as 1, 2, 3", SC'11).  Ten rounds; the key is bumped between rounds.  */
/* ------------------------------------------------------------------------ */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The uniform draw that decides the rounding of coordinate i of worker k in
 * quantisation call call_id.  Four consecutive coordinates share one Philox
 * block; coordinate i takes word i mod 4; the top 24 bits become r in [0,1). */
float orc_uniform24(uint64_t seed, uint32_t k, uint32_t call_id, uint64_t i)
{
    uint32_t ctr[4], key[2], out[4];
    uint64_t blk = i >> 2;
    ctr[0] = (uint32_t)blk; ctr[1] = (uint32_t)(blk >> 32); ctr[2] = k; ctr[3] = call_id;
    key[0] = (uint32_t)seed; key[1] = (uint32_t)(seed >> 32);
    orc_philox4x32_10(ctr, key, out);
    return (float)(out[i & 3] >> 8) * 0x1p-24f;
}

/* ------------------------------------------------------------------------ */
/* Layout: segments (tensors) are cut into buckets of at most `bucket`       */
/* coordinates (the last bucket of a segment may be short).  Chunks, the     */
/* container's unit, hold at most ORC_CH coordinates: every bucket is cut    */
/* into chunks of its own, except that buckets of 256, 512, 1024 or 2048     */
/* coordinates share chunks: there a segment is cut into runs of ORC_CH      */
/* coordinates, each holding whole buckets (the paper's experiment uses      */
/* buckets of 1024; a chunk per bucket would leave three quarters of every   */
/* chunk's tables empty).  chunk_bucket[c] is the bucket of the chunk's      */
/* first coordinate.                                                         */
/* ------------------------------------------------------------------------ */
static int orc_shared_chunks(uint32_t bucket)
{
    return bucket == 256 || bucket == 512 || bucket == 1024 || bucket == 2048;
}

void orc_layout_counts(uint64_t d, uint32_t bucket, uint32_t n_seg, const uint64_t* seg_len,
                       uint64_t* n_buckets, uint64_t* n_chunks)
{
    uint64_t one = d, nb = 0, nc = 0;
    if (seg_len == NULL) { seg_len = &one; n_seg = 1; }
    for (uint32_t s = 0; s < n_seg; ++s) {
        uint64_t left = seg_len[s];
        if (orc_shared_chunks(bucket)) nc += (left + ORC_CH - 1) / ORC_CH;
        while (left > 0) {
            uint64_t len = left < bucket ? left : bucket;
            nb += 1;
            if (!orc_shared_chunks(bucket)) nc += (len + ORC_CH - 1) / ORC_CH;
            left -= len;
        }
    }
    *n_buckets = nb; *n_chunks = nc;
}

/* bucket_start has NB+1 entries, chunk_start NC+1, chunk_bucket NC. */
void orc_layout_fill(uint64_t d, uint32_t bucket, uint32_t n_seg, const uint64_t* seg_len,
                     uint64_t* bucket_start, uint64_t* chunk_start, uint64_t* chunk_bucket)
{
    uint64_t one = d, nb = 0, nc = 0, pos = 0;
    if (seg_len == NULL) { seg_len = &one; n_seg = 1; }
    for (uint32_t s = 0; s < n_seg; ++s) {
        uint64_t left = seg_len[s];
        if (orc_shared_chunks(bucket)) {
            for (uint64_t o = 0; o < left; o += ORC_CH) {
                chunk_start[nc] = pos + o;
                chunk_bucket[nc] = nb + o / bucket;
                nc += 1;
            }
        }
        while (left > 0) {
            uint64_t len = left < bucket ? left : bucket;
            bucket_start[nb] = pos;
            if (!orc_shared_chunks(bucket)) {
                for (uint64_t o = 0; o < len; o += ORC_CH) {
                    chunk_start[nc] = pos + o;
                    chunk_bucket[nc] = nb;
                    nc += 1;
                }
            }
            nb += 1;
            pos += len;
            left -= len;
        }
    }
    bucket_start[nb] = pos;
    chunk_start[nc] = pos;
}

/* ------------------------------------------------------------------------ */
/* Norm of one bucket (Section 3.2: the tuple (||v||_q, s, u)); norm_kind is   */
/* q in Z_+ (Definition 1), or 0 for the q -> infinity limit.  Returns the binary32 value that is stored/sent      */
/* (C_b = 32 bits).  *finite is 0 when the bucket holds a non-finite value   */
/* or the norm does not fit binary32.                                        */
/* ------------------------------------------------------------------------ */
float orc_bucket_norm(const float* v, uint64_t len, int norm_kind, int* finite)
{
    int ok = 1;
    float n;
    if (norm_kind == ORC_NORM_L2) {
        double acc = 0.0;
        for (uint64_t i = 0; i < len; ++i) {
            if (!isfinite(v[i])) ok = 0;
            acc += (double)v[i] * (double)v[i];
        }
        n = (float)sqrt(acc);
    } else if (norm_kind != ORC_NORM_LINF) {
        /* any other q in Z_+: (sum |v_i|^q)^(1/q), taken relative to the largest magnitude so    */
        /* that no power leaves the range of binary64 */
        const double q = (double)norm_kind;
        double m = 0.0, acc = 0.0;
        for (uint64_t i = 0; i < len; ++i) {
            if (!isfinite(v[i])) ok = 0;
            if (fabs((double)v[i]) > m) m = fabs((double)v[i]);
        }
        if (ok && m > 0.0) {
            for (uint64_t i = 0; i < len; ++i) acc += pow(fabs((double)v[i]) / m, q);
            n = (float)(m * pow(acc, 1.0 / q));
        } else {
            n = (float)m;
        }
    } else {
        n = 0.0f;
        for (uint64_t i = 0; i < len; ++i) {
            float a = fabsf(v[i]);
            if (!isfinite(v[i])) ok = 0;
            if (a > n) n = a;
        }
    }
    if (!isfinite(n)) ok = 0;
    *finite = ok;
    return n;
}

/* tau(u): the largest j <= n_sym-2 with l_j <= u (Definition 1; at u = 1 the
 * definition has no solution, so the index is capped and xi becomes 1). */
static uint32_t level_below(const float* levels, uint32_t n_sym, float u)
{
    uint32_t j = 0;
    while (j + 2 < n_sym && levels[j + 1] <= u) ++j;
    return j;
}

/* ------------------------------------------------------------------------ */
/* Q_l(v) of Definition 1 applied bucket by bucket, for K workers.           */
/* V is [K][d]; norms_in (may be NULL) overrides the computed norms;         */
/* norms_out [K][NB]; idx [K][d] level index of q_l(u_i); neg [K][d] sign    */
/* bit of v_i.  Returns the number of non-finite buckets (all their symbols  */
/* are 0 and the stored norm is 0).  k0 and i0 shift the worker and          */
/* coordinate numbers the draws are keyed by, so that a slice of a larger    */
/* problem can be checked on its own (0 for a whole problem).                */
/* ------------------------------------------------------------------------ */
uint64_t orc_quantize(const float* V, uint32_t K, uint64_t d,
                      const uint64_t* bucket_start, uint64_t NB, int norm_kind,
                      const float* levels, uint32_t n_sym,
                      uint64_t seed, uint32_t call_id,
                      const float* norms_in, float* norms_out,
                      uint8_t* idx, uint8_t* neg,
                      uint32_t k0, uint64_t i0)
{
    uint64_t bad = 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(+ : bad)
    for (uint32_t k = 0; k < K; ++k) {
        for (uint64_t b = 0; b < NB; ++b) {
            const uint64_t lo = bucket_start[b], hi = bucket_start[b + 1];
            const float* v = V + (uint64_t)k * d;
            int finite = 1;
            float n = orc_bucket_norm(v + lo, hi - lo, norm_kind, &finite);
            if (norms_in) { n = norms_in[(uint64_t)k * NB + b]; if (!isfinite(n)) finite = 0; }
            if (!finite) { n = 0.0f; bad += 1; }
            norms_out[(uint64_t)k * NB + b] = n;
            const float rinv = 1.0f / n;          /* one IEEE division per bucket */
            for (uint64_t i = lo; i < hi; ++i) {
                const float x = v[i];
                uint32_t sym = 0;
                if (n > 0.0f) {
                    const float a = fabsf(x);
                    const float u = fminf(a * rinv, 1.0f);
                    const uint32_t j = level_below(levels, n_sym, u);
                    const float t = u - levels[j];
                    const float g = levels[j + 1] - levels[j];
                    const float r = orc_uniform24(seed, k0 + k, call_id, i0 + i);
                    /* up with probability xi = t / g, written without a division */
                    sym = j + ((r * g < t) ? 1u : 0u);
                }
                idx[(uint64_t)k * d + i] = (uint8_t)sym;
                neg[(uint64_t)k * d + i] = (uint8_t)(signbit(x) ? 1 : 0);
            }
        }
    }
    return bad;
}

/* ------------------------------------------------------------------------ */
/* Psi: Elias' recursive ("omega") integer code of N >= 1, most significant   */
/* bit of every group first.  bits[i] is the i-th bit written.  Returns the   */
/* length.  (Appendix J: a universal code that gives smaller values shorter   */
/* words; symbol index j is coded as the integer j+1.)                        */
/* ------------------------------------------------------------------------ */
uint32_t orc_elias_omega(uint32_t N, uint8_t bits[64])
{
    uint8_t tmp[64];
    uint32_t len = 0;
    tmp[len++] = 0;                       /* the terminating 0, written last   */
    while (N > 1) {
        uint32_t nb = 0;
        for (uint32_t x = N; x; x >>= 1) ++nb;
        /* prepend binary(N): store reversed, reverse everything at the end */
        for (uint32_t i = 0; i < nb; ++i) tmp[len++] = (uint8_t)((N >> i) & 1u);
        N = nb - 1;
    }
    for (uint32_t i = 0; i < len; ++i) bits[i] = tmp[len - 1 - i];
    return len;
}

static void put_bit(uint32_t* words, uint64_t pos, uint32_t bit)
{
    if (bit) words[pos >> 5] |= (uint32_t)1u << (pos & 31);
}
static uint32_t get_bit(const uint32_t* words, uint64_t pos)
{
    return (words[pos >> 5] >> (pos & 31)) & 1u;
}

/* ------------------------------------------------------------------------ */
/* CODE: for every coordinate in index order emit Psi(idx), then one sign    */
/* bit iff idx != 0 (proof of Theorem 2: one bit per non-zero entry).  The   */
/* norm is carried as raw binary32 in the norms array (C_b = 32).            */
/* Container (this project's own): stream bit p lives in word p>>5, bit p&31;*/
/* each chunk starts on a multiple of ORC_ALIGN_WORDS words, pad bits are 0; */
/* chunk_off[k][c] word offset of chunk c (exclusive scan, entry NC = total);*/
/* sub_end[k][c][j] = bit offset, from the chunk start, one past the last    */
/* bit of sub-chunk j (entries past the chunk's last sub-chunk repeat the    */
/* chunk's bit length).                                                      */
/* code_len/code_bits (may be NULL => Elias omega of idx+1): a prefix code   */
/* table, code_bits[j] holds the word with the first-written bit in bit 0.   */
/* payload is [K][cap_words] and must be zeroed by the caller.               */
/* Returns 0, or -3 if a worker's stream does not fit cap_words.             */
/* total_bits[k]: bits without padding (symbols and signs only).             */
/* ------------------------------------------------------------------------ */
int orc_encode(const uint8_t* idx, const uint8_t* neg, uint32_t K, uint64_t d,
               const uint64_t* chunk_start, uint64_t NC,
               const uint8_t* code_len, const uint32_t* code_bits,
               uint32_t* payload, uint64_t cap_words,
               uint32_t* chunk_off, uint16_t* sub_end, uint64_t* total_bits)
{
    int rc = 0;
#pragma omp parallel for schedule(static)
    for (uint32_t k = 0; k < K; ++k) {
        uint32_t* words = payload + (uint64_t)k * cap_words;
        uint64_t word_pos = 0, nbits_total = 0;
        int overflow = 0;
        for (uint64_t c = 0; c < NC && !overflow; ++c) {
            const uint64_t lo = chunk_start[c], hi = chunk_start[c + 1];
            uint64_t p = 0;                               /* bit position inside the chunk */
            uint16_t* se = sub_end + ((uint64_t)k * NC + c) * ORC_SUBS;
            chunk_off[(uint64_t)k * (NC + 1) + c] = (uint32_t)word_pos;
            {   /* exact size of this chunk first, so that nothing is written past cap_words */
                uint64_t need = 0;
                for (uint64_t i = lo; i < hi; ++i) {
                    const uint32_t sym = idx[(uint64_t)k * d + i];
                    uint8_t bits[64];
                    need += code_len ? code_len[sym] : orc_elias_omega(sym + 1u, bits);
                    need += sym != 0 ? 1u : 0u;
                }
                need = (need + 31) / 32;
                need = (need + ORC_ALIGN_WORDS - 1) / ORC_ALIGN_WORDS * ORC_ALIGN_WORDS;
                if (word_pos + need > cap_words) { overflow = 1; break; }
            }
            for (uint64_t i = lo; i < hi; ++i) {
                const uint32_t sym = idx[(uint64_t)k * d + i];
                if (code_len) {
                    for (uint32_t t = 0; t < code_len[sym]; ++t)
                        put_bit(words, word_pos * 32 + p++, (code_bits[sym] >> t) & 1u);
                } else {
                    uint8_t bits[64];
                    uint32_t len = orc_elias_omega(sym + 1u, bits);
                    for (uint32_t t = 0; t < len; ++t) put_bit(words, word_pos * 32 + p++, bits[t]);
                }
                if (sym != 0) put_bit(words, word_pos * 32 + p++, neg[(uint64_t)k * d + i]);
                if (((i - lo) % ORC_SUB) == ORC_SUB - 1 || i + 1 == hi)
                    se[(i - lo) / ORC_SUB] = (uint16_t)p;
            }
            for (uint64_t j = (hi - lo + ORC_SUB - 1) / ORC_SUB; j < ORC_SUBS; ++j) se[j] = (uint16_t)p;
            nbits_total += p;
            {
                uint64_t w = (p + 31) / 32;
                w = (w + ORC_ALIGN_WORDS - 1) / ORC_ALIGN_WORDS * ORC_ALIGN_WORDS;
                word_pos += w;
            }
        }
        if (overflow) {
#pragma omp critical
            rc = -3;
        }
        chunk_off[(uint64_t)k * (NC + 1) + NC] = (uint32_t)word_pos;
        total_bits[k] = nbits_total;
    }
    return rc;
}

/* Psi^{-1} read bit by bit.  With a table (code_len != NULL) the decoder walks
 * the bits until the word read so far equals a code word. */
static int read_symbol(const uint32_t* words, uint64_t* pos, uint64_t end,
                       const uint8_t* code_len, const uint32_t* code_bits, uint32_t n_sym,
                       uint32_t* sym)
{
    if (code_len) {
        uint32_t acc = 0, len = 0;
        while (len < 32) {
            if (*pos >= end) return -4;
            acc |= get_bit(words, (*pos)++) << len;
            ++len;
            for (uint32_t j = 0; j < n_sym; ++j)
                if (code_len[j] == len && code_bits[j] == acc) { *sym = j; return 0; }
        }
        return -4;
    }
    uint32_t N = 1;
    for (;;) {
        if (*pos >= end) return -4;
        if (get_bit(words, (*pos)++) == 0) break;
        if (N > 31) return -4;
        uint32_t val = 1;
        for (uint32_t t = 0; t < N; ++t) {
            if (*pos >= end) return -4;
            val = (val << 1) | get_bit(words, (*pos)++);
        }
        N = val;
    }
    if (N - 1 >= n_sym) return -4;
    *sym = N - 1;
    return 0;
}

/* ------------------------------------------------------------------------ */
/* DEQ o CODE (Section 3.2, Appendix J): read the norm, then for every       */
/* coordinate Psi^{-1} and, for a non-zero symbol, the sign bit;             */
/* vhat_i = +-(norm * l_idx), one binary32 multiplication.  Also returns the */
/* symbols (idx_out/neg_out may be NULL).  Returns 0 or -4 (malformed).      */
/* The sub-chunk table is checked against the parse as it goes.             */
/* ------------------------------------------------------------------------ */
int orc_decode(const uint32_t* payload, uint64_t cap_words, const uint32_t* chunk_off,
               const uint16_t* sub_end, const float* norms,
               uint32_t K, uint64_t d, const uint64_t* chunk_start, const uint64_t* chunk_bucket,
               const uint64_t* bucket_start, uint64_t NC, uint64_t NB, const float* levels, uint32_t n_sym,
               const uint8_t* code_len, const uint32_t* code_bits,
               float* Vhat, uint8_t* idx_out, uint8_t* neg_out)
{
    int rc = 0;
#pragma omp parallel for collapse(2) schedule(static)
    for (uint32_t k = 0; k < K; ++k) {
        for (uint64_t c = 0; c < NC; ++c) {
            const uint32_t* words = payload + (uint64_t)k * cap_words;
            const uint64_t lo = chunk_start[c], hi = chunk_start[c + 1];
            const uint64_t base = (uint64_t)chunk_off[(uint64_t)k * (NC + 1) + c] * 32;
            const uint64_t end = (uint64_t)chunk_off[(uint64_t)k * (NC + 1) + c + 1] * 32;
            const uint16_t* se = sub_end + ((uint64_t)k * NC + c) * ORC_SUBS;
            uint64_t b = chunk_bucket[c];                 /* bucket of coordinate i: a chunk may hold several */
            uint64_t pos = base;
            int bad = 0;
            for (uint64_t i = lo; i < hi && !bad; ++i) {
                uint32_t sym = 0, sg = 0;
                while (i >= bucket_start[b + 1]) ++b;
                const float n = norms[(uint64_t)k * NB + b];
                if (read_symbol(words, &pos, end, code_len, code_bits, n_sym, &sym)) { bad = 1; break; }
                if (sym != 0) {
                    if (pos >= end) { bad = 1; break; }
                    sg = get_bit(words, pos++);
                }
                {
                    const float mag = n * levels[sym];
                    Vhat[(uint64_t)k * d + i] = sg ? -mag : mag;
                }
                if (idx_out) idx_out[(uint64_t)k * d + i] = (uint8_t)sym;
                if (neg_out) neg_out[(uint64_t)k * d + i] = (uint8_t)sg;
                if (((i - lo) % ORC_SUB) == ORC_SUB - 1 || i + 1 == hi)
                    if (se[(i - lo) / ORC_SUB] != (uint16_t)(pos - base)) bad = 1;
            }
            if (bad) {
#pragma omp critical
                rc = -4;
            }
        }
    }
    return rc;
}

/* ------------------------------------------------------------------------ */
/* Aggregate: mean of the K decoded vectors (Algorithm 1, "Aggregate").      */
/* ------------------------------------------------------------------------ */
void orc_mean(const float* Vhat, uint32_t K, uint64_t d, double* mean)
{
#pragma omp parallel for schedule(static)
    for (uint64_t i = 0; i < d; ++i) {
        double acc = 0.0;
        for (uint32_t k = 0; k < K; ++k) acc += (double)Vhat[(uint64_t)k * d + i];
        mean[i] = acc / (double)K;
    }
}

/* ------------------------------------------------------------------------ */
/* The iteration state of eq. (Q-GenX): Y_t, the anchor X_1 (the paper sets  */
/* X_1 = 0 for notational ease; X_{t+1} = X_1 + gamma_{t+1} Y_{t+1} is the    */
/* relaxed form), S = sum over past iterations and workers of               */
/* ||Vhat_{k,i} - Vhat_{k,i+1/2}||^2, gamma_t = K / sqrt(1 + S).             */
/* ------------------------------------------------------------------------ */

/* First half-step: X_{t+1/2} = X_t - (gamma_t / K) sum_k Vhat_{k,t}, with
 * X_t = anchor + gamma_t * Y_t.  anchor may be NULL (zero). */
void orc_eg_half0(const float* Vhat, uint32_t K, uint64_t d, const double* Y, const double* anchor,
                  double gamma, double* X_half)
{
#pragma omp parallel for schedule(static)
    for (uint64_t i = 0; i < d; ++i) {
        double acc = 0.0;
        for (uint32_t k = 0; k < K; ++k) acc += (double)Vhat[(uint64_t)k * d + i];
        const double x_t = (anchor ? anchor[i] : 0.0) + gamma * Y[i];
        X_half[i] = x_t - gamma * (acc / (double)K);
    }
}

/* Second half-step: Y_{t+1} = Y_t - (1/K) sum_k Vhat_{k,t+1/2};
 * S += sum_k ||Vhat_{k,t} - Vhat_{k,t+1/2}||^2 (Vhat_prev NULL means Vhat_{k,t} = 0,
 * the dual-averaging case); gamma_{t+1} = K / sqrt(1 + S);
 * X_{t+1} = anchor + gamma_{t+1} Y_{t+1} (X_next may be NULL). */
void orc_eg_half1(const float* Vhat_cur, const float* Vhat_prev, uint32_t K, uint64_t d,
                  double* Y, const double* anchor, double* S, double* gamma, double* X_next)
{
    double s_add = 0.0;
#pragma omp parallel for schedule(static) reduction(+ : s_add)
    for (uint64_t i = 0; i < d; ++i) {
        double acc = 0.0;
        for (uint32_t k = 0; k < K; ++k) {
            const double cur = (double)Vhat_cur[(uint64_t)k * d + i];
            const double prev = Vhat_prev ? (double)Vhat_prev[(uint64_t)k * d + i] : 0.0;
            acc += cur;
            s_add += (prev - cur) * (prev - cur);
        }
        Y[i] = Y[i] - acc / (double)K;
    }
    *S += s_add;
    *gamma = (double)K / sqrt(1.0 + *S);
    if (X_next) {
#pragma omp parallel for schedule(static)
        for (uint64_t i = 0; i < d; ++i) X_next[i] = (anchor ? anchor[i] : 0.0) + (*gamma) * Y[i];
    }
}

/* ------------------------------------------------------------------------ */
/* Empirical weighted CDF F~ of eq. (QAda) as a histogram of the normalised   */
/* coordinates u, each bucket weighted by its squared norm (lambda_j of       */
/* Section 3.3, before normalisation).                                        */
/* Bins follow the binary32 grid: 64 equal-width bins per octave, n_bins/64   */
/* octaves below 1; bin 0 also takes everything smaller; u = 1 goes to the    */
/* last bin.  The bin index is an integer function of the bits of u.          */
/* ------------------------------------------------------------------------ */
uint32_t orc_bin_of(float u, uint32_t n_bins)
{
    uint32_t bits;
    memcpy(&bits, &u, 4);
    const int64_t key = (int64_t)(bits >> 17) - ((int64_t)127 * 64 - (int64_t)n_bins);
    if (key < 0) return 0;
    if (key >= (int64_t)n_bins) return n_bins - 1;
    return (uint32_t)key;
}

/* Lower edge of bin b (edge 0 is 0, edge n_bins is 1). */
double orc_bin_edge(uint32_t b, uint32_t n_bins)
{
    if (b == 0) return 0.0;
    if (b >= n_bins) return 1.0;
    uint32_t bits = (uint32_t)((int64_t)b + ((int64_t)127 * 64 - (int64_t)n_bins)) << 17;
    float e;
    memcpy(&e, &bits, 4);
    return (double)e;
}

void orc_histogram(const float* V, uint32_t K, uint64_t d,
                   const uint64_t* bucket_start, uint64_t NB, int norm_kind,
                   const float* norms_in, uint32_t n_bins, double* H)
{
    for (uint32_t b = 0; b < n_bins; ++b) H[b] = 0.0;
    for (uint32_t k = 0; k < K; ++k) {
        for (uint64_t b = 0; b < NB; ++b) {
            const uint64_t lo = bucket_start[b], hi = bucket_start[b + 1];
            const float* v = V + (uint64_t)k * d;
            int finite = 1;
            float n = orc_bucket_norm(v + lo, hi - lo, norm_kind, &finite);
            if (norms_in) { n = norms_in[(uint64_t)k * NB + b]; if (!isfinite(n)) finite = 0; }
            if (!finite || !(n > 0.0f)) continue;
            const float rinv = 1.0f / n;
            const double w = (double)n * (double)n;
            for (uint64_t i = lo; i < hi; ++i) {
                const float u = fminf(fabsf(v[i]) * rinv, 1.0f);
                H[orc_bin_of(u, n_bins)] += w;
            }
        }
    }
}

/* The bin with edge(b) <= x < edge(b+1) (the last bin for x = 1): start from the bin of x rounded to
 * binary32, then walk to the exact answer for the binary64 x. */
static uint32_t bin_containing(uint32_t n_bins, double x)
{
    uint32_t b = orc_bin_of((float)x, n_bins);
    while (b + 1 < n_bins && orc_bin_edge(b + 1, n_bins) <= x) ++b;
    while (b > 0 && orc_bin_edge(b, n_bins) > x) --b;
    return b;
}

/* ------------------------------------------------------------------------ */
/* (QAda) by updating one level at a time (Section 3.3, last sentence):      */
/* each interior level moves to the root of the stationarity condition       */
/* between its neighbours a = l_{j-1} and c = l_{j+1}, in index order,        */
/* `sweeps` times.  The condition: the derivative in l_j = x of the two terms */
/* of (QAda) that contain l_j,                                               */
/*     G(x) = int_a^x (u - a) dF~(u) - int_x^c (c - u) dF~(u) ,               */
/* vanishes.  On the piecewise-uniform density of the histogram G is          */
/* continuous, non-decreasing and linear on every piece (a piece is the part  */
/* of one bin inside [a, c]; dG/dx = (c - a) * density), with G(a) <= 0 <=    */
/* G(c).  It is zero on a whole interval where that interval holds no mass    */
/* (every point of it minimises the update; the paper leaves the choice       */
/* open): the level goes to the smallest root, inf{x in [a,c] : G(x) >= 0};   */
/* with no mass at all between the neighbours that is a itself.               */
/* G at the piece ends comes from two running sums of non-negative terms,     */
/* the left integral summed upwards from a and the right one downwards from   */
/* c (the integral of a linear weight over a piece is the piece's mass times  */
/* the weight at its midpoint), so that a sliver of mass next to a neighbour  */
/* is not lost against the total mass, as it would be in a difference of      */
/* cumulative sums taken from 0.  The root is read off the first piece at     */
/* whose upper end G is no longer negative.                                   */
/* levels[n_sym] in/out (binary32 table); work in binary64; finally round to */
/* binary32 and keep the table strictly increasing with gaps >= 2^-24.       */
/* ------------------------------------------------------------------------ */
static double smallest_stationary_point(const double* H, uint32_t n_bins, double a, double c,
                                        double* lo, double* hi, double* mass, double* left, double* right)
{
    /* the pieces of [a, c] */
    uint32_t n = 0;
    if (!(c > a)) return a;
    for (uint32_t b = bin_containing(n_bins, a); b < n_bins; ++b) {
        const double e0 = orc_bin_edge(b, n_bins), e1 = orc_bin_edge(b + 1, n_bins);
        if (e0 >= c) break;
        lo[n] = a > e0 ? a : e0;
        hi[n] = c < e1 ? c : e1;
        if (!(hi[n] > lo[n])) continue;
        mass[n] = H[b] * (hi[n] - lo[n]) / (e1 - e0);
        n += 1;
    }
    /* left[p] = int_a^{lo_p} (u - a) dF~,  right[p] = int_{lo_p}^c (c - u) dF~ ; entry n stands for x = c */
    left[0] = 0.0;
    for (uint32_t p = 0; p < n; ++p) {
        const double piece_mid = 0.5 * (lo[p] + hi[p]);
        left[p + 1] = left[p] + mass[p] * (piece_mid - a);
    }
    right[n] = 0.0;
    for (uint32_t p = n; p > 0; --p) {
        const double piece_mid = 0.5 * (lo[p - 1] + hi[p - 1]);
        right[p - 1] = right[p] + mass[p - 1] * (c - piece_mid);
    }
    if (!(right[0] > 0.0)) return a;                      /* no mass between the neighbours */
    for (uint32_t p = 0; p < n; ++p) {
        const double G_lo = left[p] - right[p], G_hi = left[p + 1] - right[p + 1];
        if (G_lo < 0.0 && G_hi >= 0.0) {
            const double slope = (c - a) * mass[p] / (hi[p] - lo[p]);
            double x = lo[p] - G_lo / slope;
            if (x > hi[p]) x = hi[p];
            return x;
        }
    }
    return c;                                             /* not reached: G(c) >= 0 */
}

/* One update on its own (for the pins): the smallest root for the neighbours a < c. */
double orc_stationary_point(const double* H, uint32_t n_bins, double a, double c)
{
    double* work = (double*)malloc(sizeof(double) * 5 * ((size_t)n_bins + 2));
    const size_t m = (size_t)n_bins + 2;
    const double x = smallest_stationary_point(H, n_bins, a, c, work, work + m, work + 2 * m, work + 3 * m, work + 4 * m);
    free(work);
    return x;
}

void orc_fit_levels(const double* H, uint32_t n_bins, float* levels, uint32_t n_sym, uint32_t sweeps)
{
    double* l = (double*)malloc(sizeof(double) * n_sym);
    double* work = (double*)malloc(sizeof(double) * 5 * ((size_t)n_bins + 2));
    double* lo = work, *hi = lo + n_bins + 2, *mass = hi + n_bins + 2, *left = mass + n_bins + 2, *right = left + n_bins + 2;
    double total = 0.0;
    for (uint32_t b = 0; b < n_bins; ++b) total += H[b];
    for (uint32_t j = 0; j < n_sym; ++j) l[j] = (double)levels[j];
    if (total > 0.0) {
        for (uint32_t s = 0; s < sweeps; ++s)
            for (uint32_t j = 1; j + 1 < n_sym; ++j)
                l[j] = smallest_stationary_point(H, n_bins, l[j - 1], l[j + 1], lo, hi, mass, left, right);
    }
    levels[0] = 0.0f; levels[n_sym - 1] = 1.0f;
    for (uint32_t j = 1; j + 1 < n_sym; ++j) {
        float x = (float)l[j];
        const float floor_ = levels[j - 1] + 0x1p-24f;
        if (x < floor_) x = floor_;
        levels[j] = x;
    }
    for (uint32_t j = n_sym - 2; j >= 1; --j) {
        const float ceil_ = levels[j + 1] - 0x1p-24f;
        if (levels[j] > ceil_) levels[j] = ceil_;
    }
    free(l); free(work);
}

/* The objective of (QAda) for a level table, on the same piecewise-uniform
 * density: sum_j int_{l_j}^{l_{j+1}} (l_{j+1}-u)(u-l_j) dF~(u).  Evaluated bin by
 * bin with the exact integral of the quadratic over each (bin x level-gap) piece. */
double orc_qada_objective(const double* H, uint32_t n_bins, const float* levels, uint32_t n_sym)
{
    double total = 0.0;
    for (uint32_t j = 0; j + 1 < n_sym; ++j) {
        const double a = (double)levels[j], c = (double)levels[j + 1];
        for (uint32_t b = 0; b < n_bins; ++b) {
            const double e0 = orc_bin_edge(b, n_bins), e1 = orc_bin_edge(b + 1, n_bins);
            const double lo = a > e0 ? a : e0, hi = c < e1 ? c : e1;
            if (!(hi > lo) || H[b] == 0.0) continue;
            /* int_lo^hi (c-u)(u-a) du = [-(u^3)/3 + (a+c)u^2/2 - a c u] */
            const double P_hi = -hi * hi * hi / 3.0 + (a + c) * hi * hi / 2.0 - a * c * hi;
            const double P_lo = -lo * lo * lo / 3.0 + (a + c) * lo * lo / 2.0 - a * c * lo;
            total += H[b] / (e1 - e0) * (P_hi - P_lo);
        }
    }
    return total;
}

/* ------------------------------------------------------------------------ */
/* Symbol probabilities of Proposition 1: p_j is the mass F~ puts on l_j      */
/* through the random rounding, i.e. the integral of the "hat" function that  */
/* rises linearly from l_{j-1} to l_j and falls linearly to l_{j+1} (only the */
/* falling half for l_0 = 0, read as (l_1 - u)/l_1 so that it is a            */
/* probability; only the rising half for the last level), normalised by the   */
/* total mass.  Evaluated bin by bin on the same piecewise-uniform density as */
/* the fit: over a piece [lo, hi] of a bin the integral of a linear function  */
/* is its value at the midpoint times the mass of the piece.                  */
/* ------------------------------------------------------------------------ */
void orc_symbol_probabilities(const double* H, uint32_t n_bins, const float* levels, uint32_t n_sym, double* p)
{
    double total = 0.0;
    for (uint32_t b = 0; b < n_bins; ++b) total += H[b];
    for (uint32_t j = 0; j < n_sym; ++j) p[j] = 0.0;
    if (!(total > 0.0)) return;
    for (uint32_t j = 0; j + 1 < n_sym; ++j) {          /* gap [a, c] feeds l_j (falling) and l_{j+1} (rising) */
        const double a = (double)levels[j], c = (double)levels[j + 1];
        for (uint32_t b = 0; b < n_bins; ++b) {
            const double e0 = orc_bin_edge(b, n_bins), e1 = orc_bin_edge(b + 1, n_bins);
            const double lo = a > e0 ? a : e0, hi = c < e1 ? c : e1;
            if (!(hi > lo) || H[b] == 0.0) continue;
            const double mass = H[b] * (hi - lo) / (e1 - e0);
            const double mid = 0.5 * (lo + hi);
            const double up = (mid - a) / (c - a);      /* probability of rounding up at the midpoint */
            p[j] += mass * (1.0 - up);
            p[j + 1] += mass * up;
        }
    }
    for (uint32_t j = 0; j < n_sym; ++j) p[j] /= total;
}

/* ------------------------------------------------------------------------ */
/* Psi as an optimal prefix code for given symbol weights (Appendix J: Huffman*/
/* coding when the symbol distribution is known or estimated), with no word   */
/* longer than max_len bits, straight from the definition of optimality:      */
/*     minimise  sum_i w_i len_i   over  1 <= len_i <= max_len                */
/*     subject to Kraft's inequality  sum_i 2^-len_i <= 1                     */
/* (a prefix code with these lengths exists exactly when it holds).  Without  */
/* the limit being active the minimum is the cost of Huffman's code.          */
/* Exhaustive dynamic programme over (symbol, code space left): in units of   */
/* 2^-max_len the whole code space is B = 2^max_len and a word of len bits    */
/* takes 2^(max_len - len); best[i][k] is the least cost of words for the     */
/* symbols i .. n-1 out of k units.  Among optimal assignments the one whose  */
/* length vector is smallest in dictionary order is returned.  Weights are    */
/* integers (exact sums).  n >= 2, max_len <= 16.                             */
/* Returns 0, or -1 if no such code exists (2^max_len < n) or max_len > 16.   */
/* ------------------------------------------------------------------------ */
int orc_limited_prefix_lengths(const uint64_t* w, uint32_t n, uint32_t max_len, uint8_t* len)
{
    if (n < 2 || max_len < 1 || max_len > 16 || (1u << max_len) < n) return -1;
    const uint64_t none = UINT64_MAX;
    const uint32_t B = 1u << max_len;
    uint64_t* best = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)(n + 1) * (B + 1));
    if (!best) return -1;
#define BEST(i, k) best[(size_t)(i) * (B + 1) + (k)]
    for (uint32_t k = 0; k <= B; ++k) BEST(n, k) = 0;              /* nothing left to code */
    for (uint32_t i = n; i-- > 0;) {
        for (uint32_t k = 0; k <= B; ++k) {
            uint64_t least = none;
            for (uint32_t l = 1; l <= max_len; ++l) {
                const uint32_t space = 1u << (max_len - l);
                if (space > k || BEST(i + 1, k - space) == none) continue;
                const uint64_t cost = w[i] * l + BEST(i + 1, k - space);
                if (cost < least) least = cost;
            }
            BEST(i, k) = least;
        }
    }
    int rc = BEST(0, B) == none ? -1 : 0;
    uint32_t k = B;
    for (uint32_t i = 0; i < n && rc == 0; ++i) {                    /* read one optimal assignment back */
        len[i] = 0;
        for (uint32_t l = 1; l <= max_len; ++l) {
            const uint32_t space = 1u << (max_len - l);
            if (space > k || BEST(i + 1, k - space) == none) continue;
            if (w[i] * l + BEST(i + 1, k - space) == BEST(i, k)) { len[i] = (uint8_t)l; k -= space; break; }
        }
        if (len[i] == 0) rc = -1;
    }
#undef BEST
    free(best);
    return rc;
}

/* Integer weights for the code construction from probabilities: p * 2^32 rounded to the nearest  */
/* integer, at least 1 so that a symbol never seen in the fitted sample still gets a word.          */
void orc_code_weights(const double* p, uint32_t n, uint64_t* w)
{
    for (uint32_t i = 0; i < n; ++i) {
        const long long x = llround(ldexp(p[i], 32));
        w[i] = x >= 1 ? (uint64_t)x : 1ull;
    }
}

/* Canonical words for given lengths: list the symbols by (length, index); the first takes the word  */
/* of all zeros, every next one the previous word plus one, extended by zeros on the right to its   */
/* own length (words read most significant bit first).  bits[i] holds word i with its first bit in  */
/* bit 0 (the container's bit order).  Returns 0, or -1 if the lengths overfill the code space.     */
typedef struct { uint32_t len, index; } orc_word_order;
static int by_length_then_index(const void* x, const void* y)
{
    const orc_word_order* a = (const orc_word_order*)x;
    const orc_word_order* b = (const orc_word_order*)y;
    if (a->len != b->len) return a->len < b->len ? -1 : 1;
    return a->index < b->index ? -1 : (a->index > b->index ? 1 : 0);
}

int orc_canonical_code(const uint8_t* len, uint32_t n, uint32_t* bits)
{
    orc_word_order* order = (orc_word_order*)malloc(sizeof(orc_word_order) * n);
    long double kraft = 0.0L;
    for (uint32_t i = 0; i < n; ++i) {
        order[i].len = len[i]; order[i].index = i;
        if (len[i] < 1 || len[i] > 32) { free(order); return -1; }
        kraft += ldexpl(1.0L, -(int)len[i]);
    }
    if (kraft > 1.0L) { free(order); return -1; }
    qsort(order, n, sizeof(orc_word_order), by_length_then_index);
    uint64_t word = 0;                                      /* value of the word, most significant bit first */
    for (uint32_t r = 0; r < n; ++r) {
        if (r > 0) word = (word + 1) << (order[r].len - order[r - 1].len);
        uint32_t first_bit_low = 0;                         /* the same word with its first bit in bit 0 */
        for (uint32_t q = 0; q < order[r].len; ++q)
            if ((word >> (order[r].len - 1 - q)) & 1u) first_bit_low |= 1u << q;
        bits[order[r].index] = first_bit_low;
    }
    free(order);
    return 0;
}

/* ------------------------------------------------------------------------ */
/* The synthetic stochastic oracle of the large quadratic game (Section 2:    */
/* a dual vector is g(z; omega) = A(z) + U(z; omega) with E U = 0 and bounded */
/* variance, the absolute-noise model).  The operator is strongly monotone:   */
/* F(z) = M z + b with M block diagonal, 2x2 blocks [[mu, a_j], [-a_j, mu]]   */
/* acting on the coordinate pairs (2j, 2j+1).  Worker k's dual vector in      */
/* quantisation call `call_id` is F(z) + sigma * N, N standard normal and     */
/* independent over workers, calls and coordinates.  The draws are this       */
/* project's own choice, made reproducible like the rounding draws: the four  */
/* coordinates 4g..4g+3 take the Philox4x32-10 block with key noise_seed and  */
/* counter (g, 1, k, call_id) (the rounding draws have 0 in the second word), */
/* words (w0, w1) give coordinates 4g, 4g+1 and (w2, w3) give 4g+2, 4g+3 by   */
/* the Box-Muller transform: u1 = (2 (w >> 9) + 1) 2^-24 in (0, 1),           */
/* u2 = (w' >> 8) 2^-24 in [0, 1), r = sqrt(-2 ln u1),                        */
/* n = r cos(2 pi u2), n' = r sin(2 pi u2).  Binary64 throughout; the dual    */
/* vector is rounded to binary32 once.                                       */
/* ------------------------------------------------------------------------ */
void orc_game_operator(const float* z, const float* a, const float* b, double mu, uint64_t d, double* F)
{
    for (uint64_t j = 0; j + 1 < d; j += 2) {
        const double z0 = z[j], z1 = z[j + 1], aj = a[j / 2];
        F[j] = mu * z0 + aj * z1 + (double)b[j];
        F[j + 1] = -aj * z0 + mu * z1 + (double)b[j + 1];
    }
}

double orc_normal(uint64_t noise_seed, uint32_t k, uint32_t call_id, uint64_t i)
{
    const double two_pi = 6.283185307179586476925286766559;
    uint32_t ctr[4], key[2], out[4];
    const uint64_t g = i >> 2;
    ctr[0] = (uint32_t)g; ctr[1] = 1u; ctr[2] = k; ctr[3] = call_id;
    key[0] = (uint32_t)noise_seed; key[1] = (uint32_t)(noise_seed >> 32);
    orc_philox4x32_10(ctr, key, out);
    const uint32_t wr = out[(i & 2)], wt = out[(i & 2) + 1];       /* the pair this coordinate belongs to */
    const double u1 = (2.0 * (double)(wr >> 9) + 1.0) * 0x1p-24;
    const double u2 = (double)(wt >> 8) * 0x1p-24;
    const double r = sqrt(-2.0 * log(u1));
    return (i & 1) ? r * sin(two_pi * u2) : r * cos(two_pi * u2);
}

/* V [K][d]: worker k's dual vector F(z) + sigma N_k, rounded to binary32. */
void orc_game_dual_vectors(const float* z, const float* a, const float* b, double mu, double sigma,
                           uint64_t noise_seed, uint32_t call_id, uint32_t K, uint64_t d, float* V)
{
    double* F = (double*)malloc(sizeof(double) * d);
    orc_game_operator(z, a, b, mu, d, F);
#pragma omp parallel for schedule(static)
    for (uint32_t k = 0; k < K; ++k)
        for (uint64_t i = 0; i < d; ++i)
            V[(uint64_t)k * d + i] = (float)(F[i] + sigma * orc_normal(noise_seed, k, call_id, i));
    free(F);
}

/* ||x||_2 in binary64 (the residual ||F(x)|| of Section 2 once x = F(.) has been formed). */
double orc_norm2(const float* x, uint64_t n)
{
    double acc = 0.0;
    for (uint64_t i = 0; i < n; ++i) acc += (double)x[i] * (double)x[i];
    return sqrt(acc);
}

/* ------------------------------------------------------------------------ */
/* Restricted gap (eq. (Gap), Section 2) of the game's operator over the      */
/* closed ball C of radius R around `center` (NULL = the origin):             */
/*   Gap_C(xhat) = sup_{x in C} <A(x), xhat - x>,  A(x) = M x + b.            */
/* M is mu I plus a skew part, so <M x, x> = mu ||x||^2 and                   */
/*   <A(x), xhat - x> = -mu ||x||^2 + <M^T xhat - b, x> + <b, xhat>,          */
/* a concave quadratic with the same curvature in every direction (mu > 0):   */
/* its maximiser over the ball is the point of the ball nearest to the free   */
/* maximiser x0 = (M^T xhat - b) / (2 mu).  The supremum is then taken from   */
/* the definition at that point.  Binary64.                                   */
/* ------------------------------------------------------------------------ */
double orc_game_gap(const float* xhat, const float* a, const float* b, double mu, const float* center, double R,
                    uint64_t d, double* maximiser /* [d] or NULL */)
{
    double* x = (double*)malloc(sizeof(double) * d);
    double dist2 = 0.0;
    for (uint64_t j = 0; j + 1 < d; j += 2) {
        const double h0 = xhat[j], h1 = xhat[j + 1], aj = a[j / 2];
        /* M^T = [[mu, -a], [a, mu]] on the block */
        x[j] = (mu * h0 - aj * h1 - (double)b[j]) / (2.0 * mu);
        x[j + 1] = (aj * h0 + mu * h1 - (double)b[j + 1]) / (2.0 * mu);
        for (int q = 0; q < 2; ++q) {
            const double c = center ? (double)center[j + q] : 0.0;
            dist2 += (x[j + q] - c) * (x[j + q] - c);
        }
    }
    const double dist = sqrt(dist2);
    if (dist > R) {
        for (uint64_t i = 0; i < d; ++i) {
            const double c = center ? (double)center[i] : 0.0;
            x[i] = c + (R / dist) * (x[i] - c);
        }
    }
    double gap = 0.0;
    for (uint64_t j = 0; j + 1 < d; j += 2) {
        const double x0 = x[j], x1 = x[j + 1], aj = a[j / 2];
        const double A0 = mu * x0 + aj * x1 + (double)b[j], A1 = -aj * x0 + mu * x1 + (double)b[j + 1];
        gap += A0 * ((double)xhat[j] - x0) + A1 * ((double)xhat[j + 1] - x1);
    }
    if (maximiser) memcpy(maximiser, x, sizeof(double) * d);
    free(x);
    return gap;
}

uint32_t orc_chunk_coords(void) { return ORC_CH; }
uint32_t orc_sub_coords(void) { return ORC_SUB; }
uint32_t orc_align_words(void) { return ORC_ALIGN_WORDS; }
