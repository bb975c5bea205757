// Host-only part of the library: error reporting and the template -> mask
// metadata (ancestor bit sets, slot starts, levels, dense expansion).
// No GPU call in this file.
#include "fdc_internal.hpp"

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <vector>

namespace fdc {

static thread_local char g_err[512] = "";

int32_t fail(int32_t code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

// Validates the template and computes strict-ancestor bit sets by one sweep in
// field order: every edge goes from a lower to a higher field index, so when
// field f is reached the sets of all its parents are final and
// anc[f] = union over parents p of (anc[p] | {p})   (Eq. 1: paths of >= 1 edge).
int32_t build_plan(int32_t F, const int32_t* slot_len, int32_t E, const int32_t* src,
                   const int32_t* dst, int32_t prefix_len, uint64_t* anc, int32_t* slot_start,
                   int32_t* level, int32_t* total_len) {
    if (F < 1) return fail(FDC_EINVAL, "n_fields must be >= 1 (got %d)", F);
    if (!slot_len || !anc || !slot_start || !total_len)
        return fail(FDC_EINVAL, "null pointer argument");
    if (E < 0 || (E > 0 && (!src || !dst))) return fail(FDC_EINVAL, "bad edge list");
    if (prefix_len < 0) return fail(FDC_EINVAL, "prefix_len must be >= 0");
    for (int f = 0; f < F; ++f)
        if (slot_len[f] < 1) return fail(FDC_EINVAL, "slot_len[%d] = %d must be >= 1", f, slot_len[f]);
    for (int e = 0; e < E; ++e)
        if (src[e] < 0 || src[e] >= F || dst[e] < 0 || dst[e] >= F)
            return fail(FDC_ERANGE, "edge %d (%d -> %d) names a field outside 0..%d", e, src[e], dst[e], F - 1);

    // acyclicity first (so a cycle is reported as such, not as an order error):
    // repeatedly remove fields without incoming edges
    {
        std::vector<int> indeg(F, 0);
        for (int e = 0; e < E; ++e) indeg[dst[e]]++;
        std::vector<int> stack;
        for (int f = 0; f < F; ++f) if (indeg[f] == 0) stack.push_back(f);
        int removed = 0;
        while (!stack.empty()) {
            int u = stack.back(); stack.pop_back(); ++removed;
            for (int e = 0; e < E; ++e)
                if (src[e] == u && --indeg[dst[e]] == 0) stack.push_back(dst[e]);
        }
        if (removed != F) return fail(FDC_ECYCLE, "dependency graph has a cycle");
    }
    for (int e = 0; e < E; ++e)
        if (src[e] >= dst[e])
            return fail(FDC_EORDER, "edge %d (%d -> %d): fields must be listed in a topological order", e, src[e], dst[e]);

    const int W = (F + 63) / 64;
    std::memset(anc, 0, sizeof(uint64_t) * (size_t)F * W);
    if (level) std::memset(level, 0, sizeof(int32_t) * F);
    for (int f = 0; f < F; ++f) {
        for (int e = 0; e < E; ++e) {
            if (dst[e] != f) continue;
            const int p = src[e];
            for (int w = 0; w < W; ++w) anc[(size_t)f * W + w] |= anc[(size_t)p * W + w];
            anc[(size_t)f * W + p / 64] |= 1ull << (p % 64);
            if (level && level[p] + 1 > level[f]) level[f] = level[p] + 1;
        }
    }
    int64_t at = prefix_len;
    for (int f = 0; f < F; ++f) {
        slot_start[f] = (int32_t)at;
        at += slot_len[f];
        if (at > 0x7fffff00) return fail(FDC_ECAP, "sequence too long");
    }
    *total_len = (int32_t)at;
    return FDC_OK;
}

}  // namespace fdc

extern "C" {

const char* fdc_strerror(int32_t code) {
    switch (code) {
        case FDC_OK: return "ok";
        case FDC_EINVAL: return "invalid argument";
        case FDC_ECYCLE: return "dependency graph is not acyclic";
        case FDC_EORDER: return "template order is not a topological order";
        case FDC_ERANGE: return "index out of range";
        case FDC_ECAP: return "size above the library's limits";
        case FDC_EHIP: return "HIP runtime error";
        case FDC_ESTATE: return "context is missing weights, cache or workspace";
        default: return "unknown error";
    }
}

const char* fdc_last_error(void) { return fdc::g_err; }

int32_t fdc_version(void) { return 100; }

int32_t fdc_build_mask(int32_t n_fields, const int32_t* slot_len, int32_t n_edges,
                       const int32_t* edge_src, const int32_t* edge_dst, int32_t prefix_len,
                       uint64_t* anc_words, int32_t* slot_start, int32_t* level,
                       int32_t* total_len) {
    return fdc::build_plan(n_fields, slot_len, n_edges, edge_src, edge_dst, prefix_len, anc_words,
                           slot_start, level, total_len);
}

int32_t fdc_dense_mask(int32_t F, const int32_t* slot_len, const int32_t* slot_start,
                       const uint64_t* anc, int32_t prefix_len, const int32_t* valid_len,
                       int32_t n_rows, const int32_t* row_field, const int32_t* row_off,
                       uint8_t* mask, int32_t* pos) {
    if (F < 1 || n_rows < 0 || prefix_len < 0) return fdc::fail(FDC_EINVAL, "bad size");
    if (!slot_len || !slot_start || !anc || !valid_len || (n_rows && (!row_field || !row_off || !mask || !pos)))
        return fdc::fail(FDC_EINVAL, "null pointer argument");
    const int W = (F + 63) / 64;
    const int64_t N = (int64_t)slot_start[F - 1] + slot_len[F - 1];
    for (int g = 0; g < F; ++g)
        if (valid_len[g] < 0 || valid_len[g] > slot_len[g])
            return fdc::fail(FDC_ERANGE, "valid_len[%d] = %d outside 0..%d", g, valid_len[g], slot_len[g]);
    for (int r = 0; r < n_rows; ++r) {
        const int f = row_field[r], t = row_off[r];
        if (f < 0 || f >= F) return fdc::fail(FDC_ERANGE, "row %d: field %d outside 0..%d", r, f, F - 1);
        if (t < 0 || t >= slot_len[f]) return fdc::fail(FDC_ERANGE, "row %d: offset %d outside slot of %d", r, t, slot_len[f]);
        uint8_t* m = mask + (size_t)r * N;
        std::memset(m, 0, (size_t)N);
        std::memset(m, 1, (size_t)prefix_len);
        for (int g = 0; g < F; ++g) {
            int n = 0;                                   // visible tokens of slot g
            if (g == f) n = t + 1;
            else if (anc[(size_t)f * W + g / 64] >> (g % 64) & 1) n = valid_len[g];
            std::memset(m + slot_start[g], 1, (size_t)n);
        }
        pos[r] = slot_start[f] + t;
    }
    return FDC_OK;
}

}  // extern "C"
