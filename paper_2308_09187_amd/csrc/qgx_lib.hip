// Host side of the C ABI: context, validation, layout tables, launches.  No arithmetic of the
// method happens here; every step runs in the gfx950 kernels.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "qgx_internal.h"

using namespace qgx;

// Scratch of qgx_eg_step_static, the variant of qgx_eg_step for callers that may not allocate: the
// per-chunk partial sums of the step-size accumulator S, which qgx_eg_step keeps in memory that
// qgx_create allocated.  Every GPU the library runs on holds its own copy of the array, at its own
// address, until the process ends.  The name below is a host-side stand-in for it, not a device
// address: host code uses the address hipGetSymbolAddress gave for the device (static_scratch_of).
static __device__ __align__(256) double scratch[QGX_STATIC_MAX_CHUNKS];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
double* g_scratch_ptr[kMaxDevices] = {nullptr};

// Address of `scratch` on `device`, which must be the current device; asked for once per device.
hipError_t static_scratch_of(int device, double** out)
{
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = static_cast<double*>(p);
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}
}  // namespace

// What the host knows of one of the context's level tables (the table itself lives on the device).
struct TableState {
    uint32_t n_sym = 0;
    uint32_t max_code_len = 0;      // longest code word of the code in use (without the sign bit)
    bool levels_set = false, code_set = false;
    bool wide = false;              // 11 bits identify every code word: the decoders may use the 8-byte table
};

struct qgx_ctx {
    qgx_config cfg{};
    std::vector<uint64_t> seg;
    int device = 0;
    uint32_t n_simd = 1024;          // SIMDs of the device (four per compute unit)
    int ksplit_forced = -1;          // qgx_debug_set_waves_per_position: 1, 2 or 4, else -1: by the rule
    Layout lay{};
    uint32_t* d_layout = nullptr;
    Tables* d_tabs = nullptr;        // [QGX_TABLES]
    TableState ts[QGX_TABLES];
    uint32_t sel = 0, sel_prev = 0;  // qgx_select_table
    Scalars* d_sc = nullptr;
    float* d_Y = nullptr;
    float* d_anchor = nullptr;
    unsigned long long* d_scan = nullptr;
    unsigned long long* d_xch = nullptr;   // partial norms of buckets shared by several workgroups
    uint32_t parts = 1;                    // workgroups per bucket in the encoder
    unsigned long long* d_tickets = nullptr;
    double* d_spartial = nullptr;
    double* d_static_scratch = nullptr;   // this device's copy of the file-scope scratch array (not owned)
    double* d_hpartial = nullptr;
    double* d_hist = nullptr;
    double* d_prob = nullptr;       // [kSymMax] symbol probabilities of the last qgx_fit_code
    double* d_norm = nullptr;       // [2 kNormBlocks + 2] partial sums and results of qgx_norm2 and qgx_game_gap
    double* d_metrics = nullptr;    // [K][3][kMetricBlocks] partial sums, then [K][3] results of qgx_quantization_metrics
    double* d_xsum = nullptr;       // [d] sum of the X_{t+1/2} since qgx_average_reset (allocated there)
    bool xsum_on = false;
    uint32_t hist_bins = 0;         // bins of the histogram d_hist holds (0: none yet)
    uint32_t h_groups = 0;
    bool state_ready = false, has_anchor = false;
    uint64_t worst_words = 0;
    char err[256] = "";
};

namespace {

qgx_status fail(qgx_ctx* ctx, qgx_status st, const char* fmt, ...)
{
    if (ctx) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
        va_end(ap);
    }
    return st;
}

#define QGX_HIP(ctx, call)                                                                             \
    do {                                                                                               \
        hipError_t e_ = (call);                                                                        \
        if (e_ != hipSuccess) return fail((ctx), QGX_ERR_HIP, "%s: %s", #call, hipGetErrorString(e_)); \
    } while (0)

// The same after an asynchronous copy into a local variable has been queued on `st`: the function may
// not return, and so end the variable's life, before the queue has drained.
#define QGX_HIP_DRAIN(ctx, st, call)                                                                   \
    do {                                                                                               \
        hipError_t e_ = (call);                                                                        \
        if (e_ != hipSuccess) {                                                                        \
            (void)hipStreamSynchronize(st);                                                            \
            return fail((ctx), QGX_ERR_HIP, "%s: %s", #call, hipGetErrorString(e_));                   \
        }                                                                                              \
    } while (0)

// Length of Elias' recursive (omega) code of N >= 1: one terminating bit plus every prefixed group.
uint32_t omega_length(uint32_t N)
{
    uint32_t len = 1;
    while (N > 1) {
        uint32_t nb = 0;
        for (uint32_t x = N; x; x >>= 1) ++nb;
        len += nb;
        N = nb - 1;
    }
    return len;
}

TableState& T(qgx_ctx* ctx) { return ctx->ts[ctx->sel]; }
const TableState& T(const qgx_ctx* ctx) { return ctx->ts[ctx->sel]; }
Tables* tab_of(const qgx_ctx* ctx) { return ctx->d_tabs + ctx->sel; }

// Do the first kWideBits bits of a code word always tell which one it is?  packed[j] = bits | length << 16,
// first-written bit in bit 0.  In a prefix-free code only two words that are both longer can agree there.
bool wide_table_ok(const uint32_t* packed, uint32_t n_sym)
{
    const uint32_t mask = (1u << kWideBits) - 1u;
    for (uint32_t i = 0; i < n_sym; ++i)
        for (uint32_t j = i + 1; j < n_sym; ++j)
            if ((packed[i] >> 16) > (uint32_t)kWideBits && (packed[j] >> 16) > (uint32_t)kWideBits &&
                ((packed[i] ^ packed[j]) & mask) == 0u)
                return false;
    return true;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

qgx_status check_stream(qgx_ctx* ctx, const qgx_stream* s, const char* what)
{
    if (!s || !s->norms || !s->chunk_off || !s->sub_end || !s->payload)
        return fail(ctx, QGX_ERR_ARG, "%s: null stream pointer", what);
    if (!aligned16(s->norms) || !aligned16(s->chunk_off) || !aligned16(s->sub_end) || !aligned16(s->payload))
        return fail(ctx, QGX_ERR_ARG, "%s: stream buffers must be 16-byte aligned", what);
    if (s->payload_words_per_worker == 0 || (s->payload_words_per_worker & 3u) ||
        s->payload_words_per_worker > 0xFFFFFFFFull)
        return fail(ctx, QGX_ERR_ARG, "%s: payload_words_per_worker must be a non-zero multiple of 4 below 2^32", what);
    if (s->slot_words & 3u) return fail(ctx, QGX_ERR_ARG, "%s: slot_words must be a multiple of 4", what);
    return QGX_OK;
}

// longest code word over the context's tables, so that streams of either share a slot size
uint32_t longest_code(const qgx_ctx* ctx)
{
    uint32_t m = 0;
    for (const TableState& t : ctx->ts) m = t.levels_set && t.max_code_len > m ? t.max_code_len : m;
    return m;
}

// most words a full chunk can take with the codes in use, multiple of 4
uint32_t chunk_slot_words(const qgx_ctx* ctx)
{
    const uint32_t words = (kChunk * (longest_code(ctx) + 1) + 31) / 32;
    return (words + 3) / 4 * 4;
}

qgx_status need_levels(qgx_ctx* ctx, uint32_t which)
{
    const TableState& t = ctx->ts[which];
    if (!t.levels_set) return fail(ctx, QGX_ERR_STATE, "level table %u not set", which);
    if (ctx->cfg.code == QGX_CODE_TABLE && !t.code_set) return fail(ctx, QGX_ERR_STATE, "code table %u not set", which);
    return QGX_OK;
}

qgx_status need_levels(qgx_ctx* ctx) { return need_levels(ctx, ctx->sel); }

void free_all(qgx_ctx* c)
{
    void* all[] = {c->d_layout, c->d_tabs, c->d_sc, c->d_Y, c->d_anchor, c->d_scan, c->d_xch, c->d_tickets, c->d_spartial, c->d_hpartial, c->d_hist, c->d_prob, c->d_norm, c->d_metrics, c->d_xsum};
    for (void* p : all) (void)hipFree(p);
}

}  // namespace

extern "C" {

qgx_status qgx_create(qgx_ctx** out, const qgx_config* cfg)
{
    if (!out || !cfg) return QGX_ERR_ARG;
    *out = nullptr;
    if (cfg->d == 0 || cfg->d >= (1ull << 31) || cfg->K == 0 || cfg->K > 65535u) return QGX_ERR_ARG;
    if (cfg->bucket == 0 || (cfg->bucket & 3u) || cfg->bucket > QGX_MAX_BUCKET) return QGX_ERR_ARG;
    if (cfg->norm < 0 || cfg->norm > QGX_MAX_NORM_Q) return QGX_ERR_ARG;
    if (cfg->code != QGX_CODE_ELIAS_OMEGA && cfg->code != QGX_CODE_TABLE) return QGX_ERR_ARG;
    qgx_ctx* c = new (std::nothrow) qgx_ctx;
    if (!c) return QGX_ERR_ARG;
    c->cfg = *cfg;
    if (cfg->n_segments > 1) {
        if (!cfg->segment_len) { delete c; return QGX_ERR_ARG; }
        c->seg.assign(cfg->segment_len, cfg->segment_len + cfg->n_segments);
    } else {
        c->seg.assign(1, cfg->n_segments == 1 && cfg->segment_len ? cfg->segment_len[0] : cfg->d);
    }
    c->cfg.segment_len = nullptr;
    uint64_t sum = 0;
    for (size_t s = 0; s < c->seg.size(); ++s) {
        if (c->seg[s] == 0 || (s + 1 < c->seg.size() && (c->seg[s] & 3u))) { delete c; return QGX_ERR_ARG; }
        sum += c->seg[s];
    }
    if (sum != cfg->d) { delete c; return QGX_ERR_ARG; }

    // buckets and chunks of one worker
    std::vector<uint32_t> bstart, bchunk0, cstart, cbucket, ragged;
    uint64_t pos = 0, worst = 0;
    uint32_t max_ragged = 0;
    const bool shared = shares_chunks(cfg->bucket);
    auto add_chunk = [&](uint64_t start, uint64_t cl, uint32_t first_bucket) {
        if (cl < (uint64_t)kChunk) {
            ragged.push_back((uint32_t)cstart.size());
            if (cl > max_ragged) max_ragged = (uint32_t)cl;
        }
        cstart.push_back((uint32_t)start);
        cbucket.push_back(first_bucket);
        const uint64_t wds = (cl * kMaxSymBits + 31) / 32;
        worst += (wds + kAlignWords - 1) / kAlignWords * kAlignWords;
    };
    for (uint64_t len_s : c->seg) {
        uint64_t left = len_s;
        if (shared) {                                   // chunks are runs of the segment, each holding whole buckets
            for (uint64_t o = 0; o < len_s; o += kChunk)
                add_chunk(pos + o, (len_s - o) < (uint64_t)kChunk ? (len_s - o) : (uint64_t)kChunk,
                          (uint32_t)(bstart.size() + o / cfg->bucket));
        }
        while (left) {
            const uint64_t len = left < cfg->bucket ? left : cfg->bucket;
            bstart.push_back((uint32_t)pos);
            bchunk0.push_back((uint32_t)cstart.size());     // (not meaningful with shared chunks)
            if (!shared) {
                for (uint64_t o = 0; o < len; o += kChunk)
                    add_chunk(pos + o, (len - o) < (uint64_t)kChunk ? (len - o) : (uint64_t)kChunk,
                              (uint32_t)(bstart.size() - 1));
            }
            pos += len;
            left -= len;
        }
    }
    bstart.push_back((uint32_t)pos);
    bchunk0.push_back((uint32_t)cstart.size());
    cstart.push_back((uint32_t)pos);
    const uint32_t NB = (uint32_t)bstart.size() - 1, NC = (uint32_t)cbucket.size();
    if ((uint64_t)NB * cfg->K >= (1ull << 31) || (uint64_t)NC * cfg->K >= (1ull << 31)) { delete c; return QGX_ERR_ARG; }
    c->worst_words = worst;

    if (hipGetDevice(&c->device) != hipSuccess) { delete c; return QGX_ERR_HIP; }
    if (static_scratch_of(c->device, &c->d_static_scratch) != hipSuccess) { delete c; return QGX_ERR_HIP; }
    {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, c->device) == hipSuccess && cus > 0)
            c->n_simd = 4u * (uint32_t)cus;
    }
    const size_t n_lay = (size_t)(NB + 1) * 2 + (NC + 1) + NC + ragged.size() + 1;
    std::vector<uint32_t> flat;
    flat.reserve(n_lay);
    flat.insert(flat.end(), bstart.begin(), bstart.end());
    flat.insert(flat.end(), bchunk0.begin(), bchunk0.end());
    flat.insert(flat.end(), cstart.begin(), cstart.end());
    flat.insert(flat.end(), cbucket.begin(), cbucket.end());
    flat.insert(flat.end(), ragged.begin(), ragged.end());
    flat.push_back(0u);

    c->lay.NB = NB; c->lay.NC = NC; c->lay.K = cfg->K; c->lay.d = (uint32_t)cfg->d;
    c->lay.n_ragged = (uint32_t)ragged.size();
    c->lay.max_ragged = max_ragged;
    uint32_t max_len = 0;
    for (uint32_t b = 0; b < NB; ++b) max_len = bstart[b + 1] - bstart[b] > max_len ? bstart[b + 1] - bstart[b] : max_len;
    c->lay.waves_per_bucket = (max_len + kChunk - 1) / kChunk;
    c->lay.uniform_bucket = (c->seg.size() == 1 && !shared) ? cfg->bucket : 0u;
    c->lay.shared_chunks = shared ? 1u : 0u;
    c->lay.bucket_shift = 31u;
    if (shared)
        for (c->lay.bucket_shift = 0; (1u << c->lay.bucket_shift) < cfg->bucket;) ++c->lay.bucket_shift;
    c->h_groups = histogram_groups(c->lay);

    bool ok = true;
    ok = ok && hipMalloc(&c->d_layout, n_lay * sizeof(uint32_t)) == hipSuccess;
    ok = ok && hipMalloc(&c->d_tabs, QGX_TABLES * sizeof(Tables)) == hipSuccess;
    ok = ok && hipMalloc(&c->d_sc, sizeof(Scalars)) == hipSuccess;
    ok = ok && hipMalloc(&c->d_Y, cfg->d * sizeof(float)) == hipSuccess;
    ok = ok && hipMalloc(&c->d_anchor, cfg->d * sizeof(float)) == hipSuccess;
    // A bucket of more than four chunks is shared by workgroups of four waves.  Per worker, the parts
    // of one bucket (the newest tickets) can be waiting for partners that have not started yet: up
    // to 3 K workgroups, which must stay below what the GPU holds at once, so only for K <= 64.
    c->parts = (c->lay.waves_per_bucket > 4u && cfg->K <= 64u) ? (c->lay.waves_per_bucket + 3u) / 4u : 1u;
    const size_t n_units = (size_t)cfg->K * NB * c->parts;
    ok = ok && hipMalloc(&c->d_scan, n_units * sizeof(unsigned long long)) == hipSuccess;
    if (c->parts > 1u) {
        ok = ok && hipMalloc(&c->d_xch, n_units * 4 * sizeof(unsigned long long)) == hipSuccess;
        ok = ok && hipMemset(c->d_xch, 0, n_units * 4 * sizeof(unsigned long long)) == hipSuccess;
    }
    ok = ok && hipMalloc(&c->d_tickets, (size_t)cfg->K * kTicketStride * sizeof(unsigned long long)) == hipSuccess;
    ok = ok && hipMalloc(&c->d_spartial, (size_t)NC * sizeof(double)) == hipSuccess;
    ok = ok && hipMalloc(&c->d_hpartial, (size_t)c->h_groups * QGX_MAX_BINS * sizeof(double)) == hipSuccess;
    ok = ok && hipMalloc(&c->d_hist, QGX_MAX_BINS * sizeof(double)) == hipSuccess;
    ok = ok && hipMalloc(&c->d_prob, kSymMax * sizeof(double)) == hipSuccess;
    ok = ok && hipMalloc(&c->d_norm, (2 * kNormBlocks + 2) * sizeof(double)) == hipSuccess;
    ok = ok && hipMalloc(&c->d_metrics, (size_t)cfg->K * 3 * (kMetricBlocks + 1) * sizeof(double)) == hipSuccess;
    ok = ok && hipMemcpy(c->d_layout, flat.data(), n_lay * sizeof(uint32_t), hipMemcpyHostToDevice) == hipSuccess;
    ok = ok && hipMemset(c->d_tabs, 0, QGX_TABLES * sizeof(Tables)) == hipSuccess;
    ok = ok && hipMemset(c->d_sc, 0, sizeof(Scalars)) == hipSuccess;
    ok = ok && hipMemset(c->d_scan, 0, n_units * sizeof(unsigned long long)) == hipSuccess;
    ok = ok && hipMemset(c->d_tickets, 0, (size_t)cfg->K * kTicketStride * sizeof(unsigned long long)) == hipSuccess;
    if (ok) {
        const uint32_t kind = (uint32_t)cfg->code;
        for (int t = 0; ok && t < QGX_TABLES; ++t)
            ok = hipMemcpy(&c->d_tabs[t].code_kind, &kind, sizeof(kind), hipMemcpyHostToDevice) == hipSuccess;
    }
    ok = ok && hipDeviceSynchronize() == hipSuccess;
    if (!ok) { free_all(c); delete c; return QGX_ERR_HIP; }
    c->lay.bucket_start = c->d_layout;
    c->lay.bucket_chunk0 = c->d_layout + (NB + 1);
    c->lay.chunk_start = c->d_layout + 2 * (size_t)(NB + 1);
    c->lay.chunk_bucket = c->lay.chunk_start + (NC + 1);
    c->lay.ragged_chunk = c->lay.chunk_bucket + NC;
    *out = c;
    return QGX_OK;
}

void qgx_destroy(qgx_ctx* ctx)
{
    if (!ctx) return;
    (void)hipDeviceSynchronize();
    free_all(ctx);
    delete ctx;
}

qgx_status qgx_stream_sizes(const qgx_ctx* ctx, uint64_t* n_buckets, uint64_t* n_chunks,
                            uint64_t* worst_case_payload_words)
{
    if (!ctx) return QGX_ERR_ARG;
    if (n_buckets) *n_buckets = ctx->lay.NB;
    if (n_chunks) *n_chunks = ctx->lay.NC;
    if (worst_case_payload_words) *worst_case_payload_words = ctx->worst_words;
    return QGX_OK;
}

qgx_status qgx_slot_words(const qgx_ctx* ctx, uint64_t* slot_words)
{
    if (!ctx || !slot_words) return QGX_ERR_ARG;
    if (!T(ctx).levels_set || (ctx->cfg.code == QGX_CODE_TABLE && !T(ctx).code_set))
        return fail(const_cast<qgx_ctx*>(ctx), QGX_ERR_STATE,
                    "qgx_slot_words: the slot follows the longest code word: set the level table (and the code table) first");
    *slot_words = chunk_slot_words(ctx);
    return QGX_OK;
}

qgx_status qgx_compact(qgx_ctx* ctx, const qgx_stream* in, qgx_stream* out, void* stream)
{
    if (!ctx) return QGX_ERR_ARG;
    qgx_status s = check_stream(ctx, in, "qgx_compact(in)");
    if (s == QGX_OK) s = check_stream(ctx, out, "qgx_compact(out)");
    if (s != QGX_OK) return s;
    if (out->slot_words != 0) return fail(ctx, QGX_ERR_ARG, "qgx_compact: out must be a compact stream");
    if (in->payload == out->payload || in->chunk_off == out->chunk_off)
        return fail(ctx, QGX_ERR_ARG, "qgx_compact: in and out must not alias");
    hipStream_t st = (hipStream_t)stream;
    const Layout& lay = ctx->lay;
    if (in->norms != out->norms)
        QGX_HIP(ctx, hipMemcpyAsync(out->norms, in->norms, (size_t)lay.K * lay.NB * sizeof(float), hipMemcpyDeviceToDevice, st));
    if (in->sub_end != out->sub_end)
        QGX_HIP(ctx, hipMemcpyAsync(out->sub_end, in->sub_end, (size_t)lay.K * lay.NC * kSubs * sizeof(uint16_t),
                                    hipMemcpyDeviceToDevice, st));
    QGX_HIP(ctx, launch_compact(lay, in->sub_end, in->chunk_off, in->payload, in->payload_words_per_worker,
                                out->chunk_off, out->payload, out->payload_words_per_worker, ctx->d_sc, st));
    return QGX_OK;
}

qgx_status qgx_select_table(qgx_ctx* ctx, uint32_t table, uint32_t prev_table)
{
    if (!ctx) return QGX_ERR_ARG;
    if (table >= QGX_TABLES || prev_table >= QGX_TABLES)
        return fail(ctx, QGX_ERR_ARG, "qgx_select_table: a context has tables 0..%d", QGX_TABLES - 1);
    ctx->sel = table;
    ctx->sel_prev = prev_table;
    return QGX_OK;
}

qgx_status qgx_set_levels(qgx_ctx* ctx, const float* levels_host, uint32_t n_sym, void* stream)
{
    if (!ctx || !levels_host) return fail(ctx, QGX_ERR_ARG, "qgx_set_levels: null argument");
    if (n_sym < 2 || n_sym > QGX_MAX_SYM) return fail(ctx, QGX_ERR_ARG, "qgx_set_levels: n_sym out of range");
    if (levels_host[0] != 0.0f || levels_host[n_sym - 1] != 1.0f)
        return fail(ctx, QGX_ERR_LEVELS, "level table must start at 0 and end at 1");
    for (uint32_t j = 0; j + 1 < n_sym; ++j)
        if (!(levels_host[j] < levels_host[j + 1]))
            return fail(ctx, QGX_ERR_LEVELS, "level table not strictly increasing at %u", j);
    hipStream_t st = (hipStream_t)stream;
    if (ctx->cfg.code == QGX_CODE_TABLE && T(ctx).code_set && n_sym != T(ctx).n_sym) T(ctx).code_set = false;
    QGX_HIP(ctx, hipMemcpyAsync(tab_of(ctx)->levels, levels_host, n_sym * sizeof(float), hipMemcpyHostToDevice, st));
    QGX_HIP(ctx, hipMemcpyAsync(&tab_of(ctx)->n_sym, &n_sym, sizeof(n_sym), hipMemcpyHostToDevice, st));
    QGX_HIP(ctx, launch_build_tables(tab_of(ctx), st));
    QGX_HIP(ctx, hipStreamSynchronize(st));
    T(ctx).n_sym = n_sym;
    T(ctx).levels_set = true;
    if (ctx->cfg.code == QGX_CODE_ELIAS_OMEGA) {
        T(ctx).max_code_len = omega_length(n_sym);
        T(ctx).wide = n_sym <= 63u;     // the words of 1..63 differ within their first 11 bits, those of 64 and 65 do not
    }
    return QGX_OK;
}

qgx_status qgx_get_levels(qgx_ctx* ctx, float* levels_host, uint32_t* n_sym, void* stream)
{
    if (!ctx || !levels_host || !n_sym) return fail(ctx, QGX_ERR_ARG, "qgx_get_levels: null argument");
    if (!T(ctx).levels_set) return fail(ctx, QGX_ERR_STATE, "level table not set");
    hipStream_t st = (hipStream_t)stream;
    QGX_HIP(ctx, hipMemcpyAsync(levels_host, tab_of(ctx)->levels, T(ctx).n_sym * sizeof(float), hipMemcpyDeviceToHost, st));
    QGX_HIP(ctx, hipStreamSynchronize(st));
    *n_sym = T(ctx).n_sym;
    return QGX_OK;
}

qgx_status qgx_set_code_table(qgx_ctx* ctx, const uint8_t* code_len, const uint32_t* code_bits, uint32_t n_sym,
                              void* stream)
{
    if (!ctx || !code_len || !code_bits) return fail(ctx, QGX_ERR_ARG, "qgx_set_code_table: null argument");
    if (ctx->cfg.code != QGX_CODE_TABLE) return fail(ctx, QGX_ERR_STATE, "context was not created with QGX_CODE_TABLE");
    if (!T(ctx).levels_set || n_sym != T(ctx).n_sym)
        return fail(ctx, QGX_ERR_STATE, "set the level table first; the code table must have as many entries");
    double kraft = 0.0;
    for (uint32_t j = 0; j < n_sym; ++j) {
        if (code_len[j] < 1 || code_len[j] > QGX_MAX_CODE_BITS || (code_bits[j] >> code_len[j]))
            return fail(ctx, QGX_ERR_ARG, "code word %u: length must be 1..13 and bits must fit it", j);
        kraft += std::ldexp(1.0, -(int)code_len[j]);
        for (uint32_t i = 0; i < j; ++i) {
            const uint32_t m = code_len[i] < code_len[j] ? code_len[i] : code_len[j];
            if (((code_bits[i] ^ code_bits[j]) & ((1u << m) - 1u)) == 0)
                return fail(ctx, QGX_ERR_ARG, "code words %u and %u: one is a prefix of the other", i, j);
        }
    }
    if (kraft > 1.0) return fail(ctx, QGX_ERR_ARG, "code table violates the Kraft inequality");
    uint32_t packed[kSymMax] = {0};
    for (uint32_t j = 0; j < n_sym; ++j) packed[j] = code_bits[j] | ((uint32_t)code_len[j] << 16);
    hipStream_t st = (hipStream_t)stream;
    QGX_HIP(ctx, hipMemcpyAsync(tab_of(ctx)->code, packed, sizeof(packed), hipMemcpyHostToDevice, st));
    QGX_HIP(ctx, launch_build_tables(tab_of(ctx), st));
    QGX_HIP(ctx, hipStreamSynchronize(st));
    T(ctx).code_set = true;
    T(ctx).max_code_len = 0;
    for (uint32_t j = 0; j < n_sym; ++j) T(ctx).max_code_len = code_len[j] > T(ctx).max_code_len ? code_len[j] : T(ctx).max_code_len;
    T(ctx).wide = wide_table_ok(packed, n_sym);
    return QGX_OK;
}

static qgx_status run_encode(qgx_ctx* ctx, EncMode mode, const float* V, uint32_t call_id, const float* norms_in,
                             float* norms_out, uint8_t* sym_out, const uint8_t* sym_in, qgx_stream* out, void* stream,
                             const GameArgs* game = nullptr)
{
    qgx_status s = need_levels(ctx);
    if (s != QGX_OK) return s;
    EncodeArgs a{};
    a.V = V; a.norms_in = norms_in; a.norms_out = norms_out; a.sym_out = sym_out; a.sym_in = sym_in;
    a.seed_lo = (uint32_t)ctx->cfg.seed; a.seed_hi = (uint32_t)(ctx->cfg.seed >> 32); a.call_id = call_id;
    a.call_mode = call_id == QGX_CALL_FIRST_HALF ? 1u : call_id == QGX_CALL_SECOND_HALF ? 2u : 0u;
    a.norm_kind = ctx->cfg.norm;
    a.cell_mant = (uint32_t)cell_mant(T(ctx).n_sym);
    a.lev_stride = lev_stride_of((int)a.cell_mant);
    a.lev_bytes = a.lev_stride + 16u * T(ctx).n_sym;
    a.sign_shift = lev_sign_shift_of((int)a.cell_mant);
    {
        const uint32_t words = (kChunk * (T(ctx).max_code_len + 1) + 31) / 32 + 4;
        a.stage_bytes = (words + 3) / 4 * 16;
    }
    if (mode != EncMode::QuantOnly) {
        if (out->slot_words) {
            if (out->slot_words < chunk_slot_words(ctx))
                return fail(ctx, QGX_ERR_ARG, "slot_words %llu is below the %u words a chunk can take",
                            (unsigned long long)out->slot_words, chunk_slot_words(ctx));
            if (out->slot_words * ctx->lay.NC > out->payload_words_per_worker)
                return fail(ctx, QGX_ERR_CAPACITY, "slotted stream needs n_chunks * slot_words payload words per worker");
            a.slot_words = (uint32_t)out->slot_words;
        }
        a.chunk_off = out->chunk_off; a.sub_end = out->sub_end; a.payload = out->payload;
        a.cap_words = out->payload_words_per_worker;
        a.scan_state = ctx->d_scan;
    }
    if (game) a.game = *game;
    a.parts = ctx->parts;
    a.xch = ctx->d_xch;
    a.tickets = ctx->d_tickets;
    hipError_t le = launch_encode(mode, ctx->lay, tab_of(ctx), ctx->d_sc, a, (hipStream_t)stream);
    if (le != hipSuccess) return fail(ctx, QGX_ERR_HIP, "encode launch: %s", hipGetErrorString(le));
    return QGX_OK;
}

qgx_status qgx_quantize(qgx_ctx* ctx, const float* V, uint32_t call_id, const float* norms_in, float* norms_out,
                        uint8_t* sym, void* stream)
{
    if (!ctx || !V || !norms_out || !sym) return fail(ctx, QGX_ERR_ARG, "qgx_quantize: null argument");
    if (!aligned16(V) || !aligned16(sym) || !aligned16(norms_out) || !aligned16(norms_in))
        return fail(ctx, QGX_ERR_ARG, "qgx_quantize: buffers must be 16-byte aligned");
    return run_encode(ctx, EncMode::QuantOnly, V, call_id, norms_in, norms_out, sym, nullptr, nullptr, stream);
}

qgx_status qgx_encode(qgx_ctx* ctx, const float* norms, const uint8_t* sym, qgx_stream* out, void* stream)
{
    if (!ctx || !norms || !sym) return fail(ctx, QGX_ERR_ARG, "qgx_encode: null argument");
    qgx_status s = check_stream(ctx, out, "qgx_encode");
    if (s != QGX_OK) return s;
    if (!aligned16(sym)) return fail(ctx, QGX_ERR_ARG, "qgx_encode: sym must be 16-byte aligned");
    if (norms != out->norms)
        QGX_HIP(ctx, hipMemcpyAsync(out->norms, norms, (size_t)ctx->lay.K * ctx->lay.NB * sizeof(float),
                                    hipMemcpyDeviceToDevice, (hipStream_t)stream));
    return run_encode(ctx, EncMode::EncodeOnly, nullptr, 0, nullptr, nullptr, nullptr, sym, out, stream);
}

qgx_status qgx_quantize_encode(qgx_ctx* ctx, const float* V, uint32_t call_id, const float* norms_in, qgx_stream* out,
                               void* stream)
{
    if (!ctx || !V) return fail(ctx, QGX_ERR_ARG, "qgx_quantize_encode: null argument");
    qgx_status s = check_stream(ctx, out, "qgx_quantize_encode");
    if (s != QGX_OK) return s;
    if (!aligned16(V) || !aligned16(norms_in)) return fail(ctx, QGX_ERR_ARG, "qgx_quantize_encode: V must be 16-byte aligned");
    return run_encode(ctx, EncMode::Fused, V, call_id, norms_in, out->norms, nullptr, nullptr, out, stream);
}

// qgx_game -> kernel arguments, with the checks the kernels rely on (four coordinates at a time)
static qgx_status game_args(qgx_ctx* ctx, const qgx_game* game, GameArgs& g, const char* what)
{
    if (!game || !game->z || !game->a || !game->b) return fail(ctx, QGX_ERR_ARG, "%s: null game pointer", what);
    if (!aligned16(game->z) || !aligned16(game->b) || (reinterpret_cast<uintptr_t>(game->a) & 7u))
        return fail(ctx, QGX_ERR_ARG, "%s: z and b must be 16-byte aligned, a 8-byte aligned", what);
    if (ctx->cfg.d & 3u) return fail(ctx, QGX_ERR_ARG, "%s: the vector length must be a multiple of 4", what);
    if (!(game->sigma >= 0.0f) || !(std::fabs(game->mu) <= 3.402823466e+38f))
        return fail(ctx, QGX_ERR_ARG, "%s: sigma must be >= 0 and mu finite", what);
    g.z = game->z; g.a = game->a; g.b = game->b; g.mu = game->mu; g.sigma = game->sigma;
    g.seed_lo = (uint32_t)game->noise_seed; g.seed_hi = (uint32_t)(game->noise_seed >> 32);
    g.V_out = nullptr;
    return QGX_OK;
}

qgx_status qgx_game_operator(qgx_ctx* ctx, const qgx_game* game, float* F_out, void* stream)
{
    if (!ctx || !F_out || !aligned16(F_out)) return fail(ctx, QGX_ERR_ARG, "qgx_game_operator: F_out null or misaligned");
    GameArgs g{};
    qgx_status s = game_args(ctx, game, g, "qgx_game_operator");
    if (s != QGX_OK) return s;
    QGX_HIP(ctx, launch_game_operator(g, ctx->lay.d, F_out, (hipStream_t)stream));
    return QGX_OK;
}

qgx_status qgx_game_dual_vectors(qgx_ctx* ctx, const qgx_game* game, uint32_t call_id, float* V_out, void* stream)
{
    if (!ctx || !V_out || !aligned16(V_out)) return fail(ctx, QGX_ERR_ARG, "qgx_game_dual_vectors: V_out null or misaligned");
    GameArgs g{};
    qgx_status s = game_args(ctx, game, g, "qgx_game_dual_vectors");
    if (s != QGX_OK) return s;
    const uint32_t mode = call_id == QGX_CALL_FIRST_HALF ? 1u : call_id == QGX_CALL_SECOND_HALF ? 2u : 0u;
    QGX_HIP(ctx, launch_game_dual_vectors(g, ctx->lay.d, ctx->lay.K, call_id, mode, ctx->d_sc, V_out, (hipStream_t)stream));
    return QGX_OK;
}

qgx_status qgx_quantize_encode_game(qgx_ctx* ctx, const qgx_game* game, uint32_t call_id, qgx_stream* out, float* V_out,
                                    void* stream)
{
    if (!ctx) return QGX_ERR_ARG;
    qgx_status s = check_stream(ctx, out, "qgx_quantize_encode_game");
    if (s != QGX_OK) return s;
    GameArgs g{};
    s = game_args(ctx, game, g, "qgx_quantize_encode_game");
    if (s != QGX_OK) return s;
    if (!aligned16(V_out)) return fail(ctx, QGX_ERR_ARG, "qgx_quantize_encode_game: V_out misaligned");
    if (ctx->lay.shared_chunks || ctx->seg.size() != 1)
        return fail(ctx, QGX_ERR_ARG, "qgx_quantize_encode_game: one segment, and buckets that do not share chunks (not 256..2048)");
    if (ctx->cfg.norm != QGX_NORM_L2 && ctx->cfg.norm != QGX_NORM_LINF)
        return fail(ctx, QGX_ERR_ARG, "qgx_quantize_encode_game: L2 or L-infinity norm");
    g.V_out = V_out;
    return run_encode(ctx, EncMode::Generate, nullptr, call_id, nullptr, out->norms, nullptr, nullptr, out, stream, &g);
}

qgx_status qgx_norm2(qgx_ctx* ctx, const float* x, uint64_t n, double* result_host, void* stream)
{
    if (!ctx || !x || !result_host || n == 0) return fail(ctx, QGX_ERR_ARG, "qgx_norm2: null argument or empty vector");
    hipStream_t st = (hipStream_t)stream;
    QGX_HIP(ctx, launch_norm2(x, n, ctx->d_norm, st));
    QGX_HIP(ctx, hipMemcpyAsync(result_host, ctx->d_norm + kNormBlocks, sizeof(double), hipMemcpyDeviceToHost, st));
    QGX_HIP(ctx, hipStreamSynchronize(st));
    return QGX_OK;
}

qgx_status qgx_game_gap(qgx_ctx* ctx, const qgx_game* game, const float* centre, double radius, double* result_host,
                        void* stream)
{
    if (!ctx || !result_host) return fail(ctx, QGX_ERR_ARG, "qgx_game_gap: null argument");
    GameArgs g;
    qgx_status s = game_args(ctx, game, g, "qgx_game_gap");
    if (s != QGX_OK) return s;
    if (!(game->mu > 0.0f) || !(radius >= 0.0) || !(radius <= 1.7976931348623157e308))
        return fail(ctx, QGX_ERR_ARG, "qgx_game_gap: mu must be positive and the radius finite and >= 0");
    hipStream_t st = (hipStream_t)stream;
    QGX_HIP(ctx, launch_game_gap(g, centre, radius, ctx->lay.d, ctx->d_norm, st));
    QGX_HIP(ctx, hipMemcpyAsync(result_host, ctx->d_norm + 2 * kNormBlocks + 1, sizeof(double), hipMemcpyDeviceToHost, st));
    QGX_HIP(ctx, hipStreamSynchronize(st));
    return QGX_OK;
}

qgx_status qgx_quantization_metrics(qgx_ctx* ctx, const float* V, const float* Vhat, uint64_t* nonzeros_host,
                                    double* sq_error_host, double* sq_norm_host, void* stream)
{
    if (!ctx || !V || !Vhat) return fail(ctx, QGX_ERR_ARG, "qgx_quantization_metrics: null argument");
    hipStream_t st = (hipStream_t)stream;
    const uint32_t K = ctx->lay.K;
    double* result = ctx->d_metrics + (size_t)K * 3 * kMetricBlocks;
    QGX_HIP(ctx, launch_metrics(V, Vhat, ctx->lay.d, K, ctx->d_metrics, result, st));
    std::vector<double> h((size_t)K * 3);
    QGX_HIP_DRAIN(ctx, st, hipMemcpyAsync(h.data(), result, h.size() * sizeof(double), hipMemcpyDeviceToHost, st));
    QGX_HIP(ctx, hipStreamSynchronize(st));
    for (uint32_t k = 0; k < K; ++k) {
        if (nonzeros_host) nonzeros_host[k] = (uint64_t)h[(size_t)k * 3];
        if (sq_error_host) sq_error_host[k] = h[(size_t)k * 3 + 1];
        if (sq_norm_host) sq_norm_host[k] = h[(size_t)k * 3 + 2];
    }
    return QGX_OK;
}

static void fill_decode_args(const qgx_ctx* ctx, DecodeArgs& a, const qgx_stream* cur, const qgx_stream* prev)
{
    a.stage_words = chunk_slot_words(ctx);
    a.stage_stride = (a.stage_words + a.stage_words / 16 + 20 + 3) / 4 * 4;   // padded layout, four zero words below the chunk's end, zero words above its first
    if (a.stage_stride < 1280u) a.stage_stride = 1280u;   // the buffer also turns the output (32 rows of 36 floats)
    a.sym_bits = longest_code(ctx) + 1;
    a.rag_words = ((ctx->lay.max_ragged * a.sym_bits + 31) / 32 + a.sym_bits + 2 + 3) / 4 * 4;
    a.rag_stride = (a.rag_words + a.rag_words / 16 + 12 + 3) / 4 * 4;
    a.wide = (T(ctx).wide && (!prev || ctx->ts[ctx->sel_prev].wide)) ? 1u : 0u;   // one kernel variant reads both streams
    // Full positions against the wave slots the kernel can hold (4 per SIMD with one stream, 2 with two):
    // a launch takes about as long as its rounds of waves, counted whole; with a position given to f
    // waves, a run of the workers each, the rounds are 1/f as long and the last one is rounded up to
    // 1/f of one.  Taken (f = 2 or 4) when that saves more than the joining costs.
    a.ksplit = 1u;
    {
        const double r = (double)(ctx->lay.NC - ctx->lay.n_ragged) / ((double)ctx->n_simd * (prev ? 2.0 : 4.0));
        double best = std::ceil(r);
        for (uint32_t f = 2; f <= 4u && f <= ctx->lay.K; f *= 2) {
            const double cost = std::ceil(f * r) / f * (f == 2 ? 1.05 : 1.10);
            if (cost < best) { best = cost; a.ksplit = f; }
        }
        if (ctx->ksplit_forced >= 0 && (uint32_t)ctx->ksplit_forced <= ctx->lay.K) a.ksplit = (uint32_t)ctx->ksplit_forced;
    }
    a.norms = cur->norms; a.chunk_off = cur->chunk_off; a.sub_end = cur->sub_end; a.payload = cur->payload;
    a.cap_words = cur->payload_words_per_worker;
    if (prev) {
        a.norms_p = prev->norms; a.chunk_off_p = prev->chunk_off; a.sub_end_p = prev->sub_end;
        a.payload_p = prev->payload; a.cap_words_p = prev->payload_words_per_worker;
        a.tab_p = ctx->sel_prev != ctx->sel ? ctx->d_tabs + ctx->sel_prev : nullptr;
    }
}

qgx_status qgx_decode(qgx_ctx* ctx, const qgx_stream* in, float* Vhat, void* stream)
{
    if (!ctx || !Vhat) return fail(ctx, QGX_ERR_ARG, "qgx_decode: null argument");
    qgx_status s = check_stream(ctx, in, "qgx_decode");
    if (s == QGX_OK) s = need_levels(ctx);
    if (s != QGX_OK) return s;
    DecodeArgs a{};
    fill_decode_args(ctx, a, in, nullptr);
    a.out = Vhat;
    QGX_HIP(ctx, launch_decode(DecMode::Decode, ctx->lay, tab_of(ctx), ctx->d_sc, a, (hipStream_t)stream));
    return QGX_OK;
}

qgx_status qgx_decode_average(qgx_ctx* ctx, const qgx_stream* in, float* mean, void* stream)
{
    if (!ctx || !mean || !aligned16(mean)) return fail(ctx, QGX_ERR_ARG, "qgx_decode_average: mean null or misaligned");
    qgx_status s = check_stream(ctx, in, "qgx_decode_average");
    if (s == QGX_OK) s = need_levels(ctx);
    if (s != QGX_OK) return s;
    DecodeArgs a{};
    fill_decode_args(ctx, a, in, nullptr);
    a.out = mean;
    QGX_HIP(ctx, launch_decode(DecMode::Average, ctx->lay, tab_of(ctx), ctx->d_sc, a, (hipStream_t)stream));
    return QGX_OK;
}

qgx_status qgx_fit_levels(qgx_ctx* ctx, const float* V, uint32_t n_sym, uint32_t n_bins, uint32_t sweeps,
                          double* hist_out, void* stream)
{
    if (!ctx || !V || !aligned16(V)) return fail(ctx, QGX_ERR_ARG, "qgx_fit_levels: V null or misaligned");
    if (!T(ctx).levels_set) return fail(ctx, QGX_ERR_STATE, "qgx_fit_levels starts from the current table: set one first");
    if (n_sym != T(ctx).n_sym) return fail(ctx, QGX_ERR_ARG, "qgx_fit_levels: n_sym differs from the current table");
    if (n_bins == 0 || (n_bins & 63u) || n_bins > QGX_MAX_BINS)
        return fail(ctx, QGX_ERR_ARG, "qgx_fit_levels: n_bins must be a multiple of 64, at most 4096");
    hipStream_t st = (hipStream_t)stream;
    QGX_HIP(ctx, launch_histogram(ctx->lay, V, ctx->cfg.norm, n_bins, ctx->d_hpartial, ctx->h_groups, ctx->d_hist,
                                  ctx->d_sc, st));
    if (hist_out)
        QGX_HIP(ctx, hipMemcpyAsync(hist_out, ctx->d_hist, n_bins * sizeof(double), hipMemcpyDeviceToDevice, st));
    QGX_HIP(ctx, launch_fit(tab_of(ctx), ctx->d_hist, n_bins, sweeps, st));
    ctx->hist_bins = n_bins;
    return QGX_OK;
}

qgx_status qgx_fit_code(qgx_ctx* ctx, double* p_host, uint8_t* code_len_host, uint32_t* code_bits_host, void* stream)
{
    if (!ctx) return QGX_ERR_ARG;
    if (ctx->cfg.code != QGX_CODE_TABLE) return fail(ctx, QGX_ERR_STATE, "context was not created with QGX_CODE_TABLE");
    if (!T(ctx).levels_set || ctx->hist_bins == 0)
        return fail(ctx, QGX_ERR_STATE, "qgx_fit_code needs the histogram of a qgx_fit_levels call (sweeps = 0 leaves the table as it is)");
    uint32_t need = 1;
    while ((1u << need) < T(ctx).n_sym) ++need;
    if (need > QGX_FIT_CODE_BITS) return fail(ctx, QGX_ERR_ARG, "too many symbols for the longest code word");
    hipStream_t st = (hipStream_t)stream;
    QGX_HIP(ctx, launch_fit_code(tab_of(ctx), ctx->d_hist, ctx->hist_bins, QGX_FIT_CODE_BITS, ctx->d_prob, st));
    uint32_t packed[kSymMax];
    QGX_HIP(ctx, hipMemcpyAsync(packed, tab_of(ctx)->code, sizeof(packed), hipMemcpyDeviceToHost, st));
    if (p_host) QGX_HIP_DRAIN(ctx, st, hipMemcpyAsync(p_host, ctx->d_prob, T(ctx).n_sym * sizeof(double), hipMemcpyDeviceToHost, st));
    QGX_HIP(ctx, hipStreamSynchronize(st));
    T(ctx).max_code_len = 0;
    for (uint32_t j = 0; j < T(ctx).n_sym; ++j) {
        const uint32_t len = packed[j] >> 16;
        T(ctx).max_code_len = len > T(ctx).max_code_len ? len : T(ctx).max_code_len;
        if (code_len_host) code_len_host[j] = (uint8_t)len;
        if (code_bits_host) code_bits_host[j] = packed[j] & 0xFFFFu;
    }
    T(ctx).code_set = true;
    T(ctx).wide = wide_table_ok(packed, T(ctx).n_sym);
    return QGX_OK;
}

qgx_status qgx_state_init(qgx_ctx* ctx, const float* X1, void* stream)
{
    if (!ctx || !aligned16(X1)) return fail(ctx, QGX_ERR_ARG, "qgx_state_init: null context or misaligned X1");
    QGX_HIP(ctx, launch_state_init(ctx->lay, ctx->d_sc, ctx->d_Y, ctx->d_anchor, X1, (hipStream_t)stream));
    ctx->has_anchor = X1 != nullptr;
    ctx->state_ready = true;
    return QGX_OK;
}

static qgx_status eg_step_with(qgx_ctx* ctx, int half, const qgx_stream* cur, const qgx_stream* prev, float* X_out,
                               void* stream, double* s_partial)
{
    if (!ctx || (half != 0 && half != 1)) return fail(ctx, QGX_ERR_ARG, "qgx_eg_step: half must be 0 or 1");
    if (!ctx->state_ready) return fail(ctx, QGX_ERR_STATE, "qgx_eg_step before qgx_state_init");
    qgx_status s = check_stream(ctx, cur, "qgx_eg_step(cur)");
    if (s == QGX_OK && prev) s = check_stream(ctx, prev, "qgx_eg_step(prev)");
    if (s == QGX_OK) s = need_levels(ctx);
    if (s == QGX_OK && prev) s = need_levels(ctx, ctx->sel_prev);
    if (s != QGX_OK) return s;
    if (!aligned16(X_out)) return fail(ctx, QGX_ERR_ARG, "qgx_eg_step: X_out misaligned");
    hipStream_t st = (hipStream_t)stream;
    DecodeArgs a{};
    a.Y = ctx->d_Y;
    a.anchor = ctx->has_anchor ? ctx->d_anchor : nullptr;
    if (half == 0) {
        if (prev) return fail(ctx, QGX_ERR_ARG, "qgx_eg_step: prev must be NULL for half = 0");
        if (!X_out) return fail(ctx, QGX_ERR_ARG, "qgx_eg_step: X_out is required for half = 0");
        fill_decode_args(ctx, a, cur, nullptr);
        a.out = X_out;
        a.x_sum = ctx->xsum_on ? ctx->d_xsum : nullptr;
        QGX_HIP(ctx, launch_decode(DecMode::Half0, ctx->lay, tab_of(ctx), ctx->d_sc, a, st));
        if (ctx->xsum_on) QGX_HIP(ctx, launch_average_count(ctx->d_sc, st));
        return QGX_OK;
    }
    fill_decode_args(ctx, a, cur, prev);
    a.s_partial = s_partial;
    QGX_HIP(ctx, launch_decode(DecMode::Half1, ctx->lay, tab_of(ctx), ctx->d_sc, a, st));
    QGX_HIP(ctx, launch_finish_half1(ctx->lay, ctx->d_sc, s_partial, ctx->d_Y, a.anchor, X_out, st));
    return QGX_OK;
}

qgx_status qgx_eg_step(qgx_ctx* ctx, int half, const qgx_stream* cur, const qgx_stream* prev, float* X_out,
                       void* stream)
{
    return eg_step_with(ctx, half, cur, prev, X_out, stream, ctx ? ctx->d_spartial : nullptr);
}

qgx_status qgx_eg_step_static(qgx_ctx* ctx, int half, const qgx_stream* cur, const qgx_stream* prev, float* X_out,
                              void* stream)
{
    if (!ctx) return QGX_ERR_ARG;
    if (ctx->lay.NC > QGX_STATIC_MAX_CHUNKS)
        return fail(ctx, QGX_ERR_CAPACITY, "qgx_eg_step_static: %u chunks per worker exceed the %u the static scratch holds; use qgx_eg_step",
                    ctx->lay.NC, (unsigned)QGX_STATIC_MAX_CHUNKS);
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != ctx->device)
        return fail(ctx, QGX_ERR_STATE, "qgx_eg_step_static: the context's device must be current");
    return eg_step_with(ctx, half, cur, prev, X_out, stream, ctx->d_static_scratch);
}

qgx_status qgx_average_reset(qgx_ctx* ctx, int on, void* stream)
{
    if (!ctx) return QGX_ERR_ARG;
    ctx->xsum_on = on != 0;
    if (!ctx->xsum_on) return QGX_OK;
    if (!ctx->d_xsum && hipMalloc(&ctx->d_xsum, ctx->cfg.d * sizeof(double)) != hipSuccess)
        return fail(ctx, QGX_ERR_HIP, "qgx_average_reset: no memory for the running sum");
    QGX_HIP(ctx, launch_average_reset(ctx->lay.d, ctx->d_xsum, ctx->d_sc, (hipStream_t)stream));
    return QGX_OK;
}

qgx_status qgx_average_export(qgx_ctx* ctx, float* X_bar, uint64_t* count, void* stream)
{
    if (!ctx || !aligned16(X_bar)) return fail(ctx, QGX_ERR_ARG, "qgx_average_export: null context or misaligned X_bar");
    if (!ctx->xsum_on) return fail(ctx, QGX_ERR_STATE, "qgx_average_export: averaging is off (qgx_average_reset)");
    unsigned long long n = 0;                               // the count lives on the device: replayed graphs add to it too
    QGX_HIP(ctx, hipMemcpyAsync(&n, &ctx->d_sc->avg_count, sizeof(n), hipMemcpyDeviceToHost, (hipStream_t)stream));
    QGX_HIP(ctx, hipStreamSynchronize((hipStream_t)stream));
    if (count) *count = n;
    if (X_bar) {
        if (n == 0) return fail(ctx, QGX_ERR_STATE, "qgx_average_export: no half-step since the reset");
        QGX_HIP(ctx, launch_average(ctx->lay.d, ctx->d_xsum, ctx->d_sc, X_bar, (hipStream_t)stream));
    }
    return QGX_OK;
}

qgx_status qgx_get_scalars(qgx_ctx* ctx, double* S, double* gamma, uint64_t* t, void* stream)
{
    if (!ctx) return QGX_ERR_ARG;
    hipStream_t st = (hipStream_t)stream;
    Scalars h;
    QGX_HIP(ctx, hipMemcpyAsync(&h, ctx->d_sc, sizeof(h), hipMemcpyDeviceToHost, st));
    QGX_HIP(ctx, hipStreamSynchronize(st));
    if (S) *S = h.S;
    if (gamma) *gamma = h.gamma;
    if (t) *t = h.t;
    return QGX_OK;
}

qgx_status qgx_stream_bits(qgx_ctx* ctx, const qgx_stream* coded, uint64_t* total_bits, void* stream)
{
    if (!ctx || !total_bits) return fail(ctx, QGX_ERR_ARG, "qgx_stream_bits: null argument");
    qgx_status s = check_stream(ctx, coded, "qgx_stream_bits");
    if (s != QGX_OK) return s;
    hipStream_t st = (hipStream_t)stream;
    QGX_HIP(ctx, launch_sum_bits(ctx->lay, coded->sub_end, ctx->d_sc, st));
    unsigned long long bits = 0;
    QGX_HIP(ctx, hipMemcpyAsync(&bits, &ctx->d_sc->total_bits, sizeof(bits), hipMemcpyDeviceToHost, st));
    QGX_HIP(ctx, hipStreamSynchronize(st));
    *total_bits = bits;
    return QGX_OK;
}

qgx_status qgx_debug_set_waves_per_position(qgx_ctx* ctx, int waves)
{
    if (!ctx) return QGX_ERR_ARG;
    if (waves != 0 && waves != 1 && waves != 2 && waves != 4)
        return fail(ctx, QGX_ERR_ARG, "qgx_debug_set_waves_per_position: 0 (by the rule), 1, 2 or 4");
    ctx->ksplit_forced = waves == 0 ? -1 : waves;
    return QGX_OK;
}

qgx_status qgx_state_export(qgx_ctx* ctx, float* Y, float* anchor, void* stream)
{
    if (!ctx) return QGX_ERR_ARG;
    if (!ctx->state_ready) return fail(ctx, QGX_ERR_STATE, "state not initialised");
    hipStream_t st = (hipStream_t)stream;
    const size_t bytes = (size_t)ctx->lay.d * sizeof(float);
    if (Y) QGX_HIP(ctx, hipMemcpyAsync(Y, ctx->d_Y, bytes, hipMemcpyDeviceToDevice, st));
    if (anchor) QGX_HIP(ctx, hipMemcpyAsync(anchor, ctx->d_anchor, bytes, hipMemcpyDeviceToDevice, st));
    return QGX_OK;
}

qgx_status qgx_state_import(qgx_ctx* ctx, const float* Y, const float* anchor, double S, uint64_t t, void* stream)
{
    if (!ctx) return QGX_ERR_ARG;
    if (!(S >= 0.0) || t == 0) return fail(ctx, QGX_ERR_ARG, "qgx_state_import: S must be >= 0 and t >= 1");
    hipStream_t st = (hipStream_t)stream;
    const size_t bytes = (size_t)ctx->lay.d * sizeof(float);
    if (!ctx->state_ready) {
        QGX_HIP(ctx, launch_state_init(ctx->lay, ctx->d_sc, ctx->d_Y, ctx->d_anchor, nullptr, st));
        ctx->state_ready = true;
    }
    if (Y) QGX_HIP(ctx, hipMemcpyAsync(ctx->d_Y, Y, bytes, hipMemcpyDeviceToDevice, st));
    if (anchor) {
        QGX_HIP(ctx, hipMemcpyAsync(ctx->d_anchor, anchor, bytes, hipMemcpyDeviceToDevice, st));
        ctx->has_anchor = true;
    }
    QGX_HIP(ctx, launch_state_set(ctx->d_sc, S, t, ctx->lay.K, st));
    return QGX_OK;
}

uint32_t qgx_poll_error(qgx_ctx* ctx, void* stream)
{
    if (!ctx) return 0;
    hipStream_t st = (hipStream_t)stream;
    uint32_t e = 0;
    const uint32_t zero = 0;
    if (hipMemcpyAsync(&e, &ctx->d_sc->err, sizeof(e), hipMemcpyDeviceToHost, st) != hipSuccess) return QGX_EBIT_STATE;
    if (hipStreamSynchronize(st) != hipSuccess) return QGX_EBIT_STATE;
    if (e) {
        (void)hipMemcpyAsync(&ctx->d_sc->err, &zero, sizeof(zero), hipMemcpyHostToDevice, st);
        (void)hipStreamSynchronize(st);
    }
    return e;
}

const char* qgx_last_error(const qgx_ctx* ctx) { return ctx ? ctx->err : "null context"; }

}  // extern "C"
