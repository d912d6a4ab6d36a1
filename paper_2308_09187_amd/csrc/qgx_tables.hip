// Derived device tables: level pairs for the rounding step, the tau lookup cells, the code words of
// Psi and the decode tables.  Rebuilt on the device whenever the level table or the code
// changes, so that a refit never goes through the host.
#include "qgx_device.h"

namespace qgx {

// Elias' recursive (omega) code of N >= 1 (Appendix J, "Elias recursive coding"), returned with the
// first-written bit in bit 0: write "0", then while N > 1 prepend binary(N) and continue with the
// number of bits of N minus one.
__device__ inline uint32_t elias_omega(uint32_t N, uint32_t* len_out)
{
    uint32_t bits = 0, len = 1;
    while (N > 1) {
        const uint32_t nb = 32u - (uint32_t)__clz((int)N);
        const uint32_t rev = __brev(N) >> (32u - nb);   // most significant bit of the group first
        bits = rev | (bits << nb);
        len += nb;
        N = nb - 1;
    }
    *len_out = len;
    return bits;
}

// E(idx, sg): code word of idx with the sign bit appended when idx != 0, total length << 16.
__device__ inline uint32_t coded_entry(uint32_t cw, uint32_t idx, uint32_t sg)
{
    uint32_t bits = cw & 0xFFFFu, len = cw >> 16;
    if (idx != 0) { bits |= sg << len; len += 1; }
    return bits | (len << 16);
}

static __device__ void build_tables_block(Tables* tab)
{
    // the levels and the code words are read over and over below: a copy in LDS
    __shared__ float lv[kSymMax];
    __shared__ uint32_t code[kSymMax];
    const uint32_t n_sym = tab->n_sym;
    const int tid = (int)threadIdx.x, nt = (int)blockDim.x;
    const float inf = __uint_as_float(0x7f800000u);

    const bool omega = tab->code_kind == QGX_CODE_ELIAS_OMEGA;
    for (int j = tid; j < kSymMax; j += nt) {
        lv[j] = tab->levels[j];
        uint32_t cw = tab->code[j];
        if (omega) {
            uint32_t len = 0, bits = 0;
            if ((uint32_t)j < n_sym) bits = elias_omega((uint32_t)j + 1u, &len);
            cw = bits | (len << 16);
            tab->code[j] = cw;
        }
        code[j] = cw;
    }
    for (int i = tid; i < kDlut; i += nt) tab->dlut[i] = (uint16_t)kDlutReject;
    for (int i = tid; i < kWide; i += nt) tab->dlutw[i] = make_uint2(kWideReject, 0u);
    __syncthreads();

    for (int j = tid; j < kSymMax; j += nt) {
        float l = 1.0f, g = 0.0f;
        if ((uint32_t)j < n_sym) l = lv[j];
        if ((uint32_t)j + 1 < n_sym) g = (lv[j + 1] - lv[j]) * 0x1p-24f;
        for (uint32_t sg = 0; sg < 2; ++sg) {
            float4 e = make_float4(l, g, 0.0f, 0.0f);
            if ((uint32_t)j < n_sym) e.z = __uint_as_float(coded_entry(code[j], (uint32_t)j, sg));
            if ((uint32_t)j + 1 < n_sym) e.w = __uint_as_float(coded_entry(code[j + 1], (uint32_t)j + 1, sg));
            tab->lev2[sg][j] = e;
        }
        tab->lval[j] = l;
    }
    // cells: lower level, the level inside (if any), and whether a second one makes the cell inexact
    if (tid == 0) { tab->cell_exact = 1u; tab->wide_ok = 1u; }
    __syncthreads();
    const int mant = cell_mant(n_sym), cells = cell_count(mant), cell_shift = 23 - mant;
    const int key0 = (127 - kCellOct) << mant;
    for (int c = tid; c < cell_count_padded(mant); c += nt) {
        uint32_t j = 0;
        float B = inf;
        uint32_t a1 = 0;
        bool crowded = false;
        if (c < cells) {
            const float edge = c == 0 ? 0.0f : __uint_as_float((uint32_t)(c + key0) << cell_shift);
            const float next = c + 1 < cells ? __uint_as_float((uint32_t)(c + 1 + key0) << cell_shift) : inf;
            // the last level, short of the top one, that is not above the edge (l_0 = 0 never is)
            uint32_t hi = n_sym - 2u;
            while (j < hi) {
                const uint32_t mid = (j + hi + 1u) >> 1;
                if (lv[mid] <= edge) j = mid; else hi = mid - 1u;
            }
            a1 = j;
            if (j + 2 < n_sym && lv[j + 1] < next) {      // a level strictly inside the cell
                B = lv[j + 1];
                a1 = j + 1;
                if (j + 3 < n_sym && lv[j + 2] < next) crowded = true;
            }
        }
        tab->cell[c] = make_float2(B, __uint_as_float((j << 4) | (a1 << 20)));
        if (crowded) tab->cell_exact = 0u;
    }
    // every 13-bit window that starts with code word j decodes to j: with the first stream bit on
    // top these windows are one run of 2^(13 - len) entries.  A wave per word (the words' runs do not meet:
    // the code is prefix-free), its lanes along the run.
    const uint32_t n_waves = (uint32_t)nt / kWave, lane = (uint32_t)tid % kWave;
    for (uint32_t j = (uint32_t)tid / kWave; j < n_sym; j += n_waves) {
        const uint32_t cw = code[j];
        const uint32_t len = cw >> 16, bits = cw & 0xFFFFu;
        if (len == 0 || len > (uint32_t)kMaxCode) continue;
        const uint32_t first = (__brev(bits) >> (32u - len)) << (kDlutBits - len);   // the word, first bit on top
        const uint32_t reps = 1u << (kDlutBits - len);
        const uint32_t entry = (j << 6) | (len - (j != 0u ? 0u : 1u));               // symbol bits - 1: sign for j != 0
        for (uint32_t s = lane; s < reps; s += kWave) tab->dlut[first + s] = (uint16_t)entry;
        // the same run in the 11-bit table, with minus the symbol's bits (sign included) and the level; a
        // longer word takes the one slot of its first 11 bits (no shorter word's run reaches it: the code is
        // prefix-free)
        const uint32_t first_w = first >> (kDlutBits - kWideBits);
        const uint32_t reps_w = len <= (uint32_t)kWideBits ? 1u << (kWideBits - len) : 1u;
        const uint32_t entry_w = 0u - (len + (j != 0u ? 1u : 0u));
        for (uint32_t s = lane; s < reps_w; s += kWave)
            tab->dlutw[first_w + s] = make_uint2(entry_w, __float_as_uint(lv[j]));
    }
    __syncthreads();
    // the 11-bit table is no use if two of the longer words begin with the same 11 bits: they would meet in
    // one slot, and one of them would no longer find itself
    for (uint32_t j = (uint32_t)tid; j < n_sym; j += (uint32_t)nt) {
        const uint32_t cw = code[j];
        const uint32_t len = cw >> 16;
        if (len <= (uint32_t)kWideBits || len > (uint32_t)kMaxCode) continue;
        const uint32_t head = cw & ((1u << kWideBits) - 1u);                  // (the first-written bit is bit 0)
        for (uint32_t i = 0; i < n_sym; ++i) {
            const uint32_t ci = code[i];
            if (i != j && (ci >> 16) > (uint32_t)kWideBits && (ci & ((1u << kWideBits) - 1u)) == head) tab->wide_ok = 0u;
        }
    }
    __syncthreads();
}

__global__ __launch_bounds__(256) void k_build_tables(Tables* tab) { build_tables_block(tab); }

hipError_t launch_build_tables(Tables* tab, hipStream_t st)
{
    hipLaunchKernelGGL(k_build_tables, dim3(1), dim3(256), 0, st, tab);
    return hipGetLastError();
}

}  // namespace qgx
