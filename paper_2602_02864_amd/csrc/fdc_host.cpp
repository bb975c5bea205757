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

// Algorithm 1 as a host object: in-degree counters, the ready set, and one
// token per ready field per pass.
struct fdc_sched {
    int F = 0;
    std::vector<int32_t> indeg, done, content_len;
    std::vector<std::vector<int32_t>> succ;
    std::vector<char> ready, finished;
    int64_t passes = 0, tokens = 0;
};

extern "C" {

int32_t fdc_sched_create(int32_t F, int32_t E, const int32_t* src, const int32_t* dst,
                         const int32_t* content_len, fdc_sched** out) {
    if (!out) return fdc::fail(FDC_EINVAL, "null pointer argument");
    *out = nullptr;
    if (F < 1) return fdc::fail(FDC_EINVAL, "bad field list");
    std::vector<int32_t> ones(F, 1), start(F);
    std::vector<uint64_t> anc((size_t)F * ((F + 63) / 64));
    int32_t total = 0;
    int32_t rc = fdc::build_plan(F, ones.data(), E, src, dst, 0, anc.data(), start.data(), nullptr, &total);
    if (rc != FDC_OK) return rc;
    if (content_len)
        for (int f = 0; f < F; ++f)
            if (content_len[f] < 1) return fdc::fail(FDC_EINVAL, "content_len[%d] = %d must be >= 1", f, content_len[f]);
    fdc_sched* s = new fdc_sched;
    s->F = F;
    s->indeg.assign(F, 0);
    s->done.assign(F, 0);
    if (content_len) s->content_len.assign(content_len, content_len + F);
    s->succ.resize(F);
    s->ready.assign(F, 0);
    s->finished.assign(F, 0);
    // duplicate edges count once
    std::vector<char> seen((size_t)F * F, 0);
    for (int e = 0; e < E; ++e) {
        if (seen[(size_t)src[e] * F + dst[e]]) continue;
        seen[(size_t)src[e] * F + dst[e]] = 1;
        s->indeg[dst[e]]++;
        s->succ[src[e]].push_back(dst[e]);
    }
    for (int f = 0; f < F; ++f) s->ready[f] = s->indeg[f] == 0;
    *out = s;
    return FDC_OK;
}

void fdc_sched_destroy(fdc_sched* s) { delete s; }

namespace {
// a finished field leaves the ready set and signals its successors
void retire(fdc_sched* s, int f) {
    s->ready[f] = 0;
    s->finished[f] = 1;
    for (int u : s->succ[f])
        if (--s->indeg[u] == 0) s->ready[u] = 1;
}
}  // namespace

int32_t fdc_sched_peek(fdc_sched* s, int32_t max_branches, int32_t* branch_field,
                       int32_t* branch_off, int32_t* n_active) {
    if (!s || !branch_field || !branch_off || !n_active) return fdc::fail(FDC_EINVAL, "null pointer argument");
    int n = 0;
    for (int f = 0; f < s->F; ++f) n += s->ready[f] ? 1 : 0;
    if (n > max_branches) return fdc::fail(FDC_ECAP, "%d fields are ready, room for %d", n, max_branches);
    int i = 0;
    for (int f = 0; f < s->F; ++f)
        if (s->ready[f]) {
            branch_field[i] = f;
            branch_off[i] = s->done[f];
            ++i;
        }
    for (int j = i; j < max_branches; ++j) {
        branch_field[j] = -1;
        branch_off[j] = 0;
    }
    *n_active = n;
    return FDC_OK;
}

int32_t fdc_sched_advance(fdc_sched* s, int32_t n, const int32_t* field_finished) {
    if (!s || (n > 0 && !field_finished)) return fdc::fail(FDC_EINVAL, "null pointer argument");
    std::vector<int32_t> act;
    for (int f = 0; f < s->F; ++f)
        if (s->ready[f]) act.push_back(f);
    if (n != (int)act.size()) return fdc::fail(FDC_EINVAL, "%d flags for %d ready fields", n, (int)act.size());
    if (n == 0) return FDC_OK;
    s->passes++;
    s->tokens += n;
    // every ready field has decoded one token; finished ones release their successors
    for (int i = 0; i < n; ++i) s->done[act[i]]++;
    for (int i = 0; i < n; ++i)
        if (field_finished[i]) retire(s, act[i]);
    return FDC_OK;
}

int32_t fdc_sched_complete(fdc_sched* s, int32_t field, int32_t n_tokens) {
    if (!s) return fdc::fail(FDC_EINVAL, "null pointer argument");
    if (field < 0 || field >= s->F) return fdc::fail(FDC_ERANGE, "field %d outside 0..%d", field, s->F - 1);
    if (n_tokens < 0) return fdc::fail(FDC_EINVAL, "negative token count");
    if (!s->ready[field] || s->done[field] != 0)
        return fdc::fail(FDC_EINVAL, "field %d is not an untouched ready field (its prerequisites must be complete)", field);
    s->done[field] = n_tokens;
    retire(s, field);
    return FDC_OK;
}

int32_t fdc_sched_next(fdc_sched* s, int32_t max_branches, int32_t* branch_field,
                       int32_t* branch_off, int32_t* n_active) {
    if (s && s->content_len.empty()) return fdc::fail(FDC_EINVAL, "scheduler was created without content lengths");
    int32_t rc = fdc_sched_peek(s, max_branches, branch_field, branch_off, n_active);
    if (rc != FDC_OK || *n_active == 0) return rc;
    std::vector<int32_t> fin(*n_active);
    for (int i = 0; i < *n_active; ++i)
        fin[i] = s->done[branch_field[i]] + 1 >= s->content_len[branch_field[i]];
    return fdc_sched_advance(s, *n_active, fin.data());
}

int32_t fdc_sched_stats(const fdc_sched* s, int64_t* passes, int64_t* tokens, int32_t* n_unfinished) {
    if (!s) return fdc::fail(FDC_EINVAL, "null pointer argument");
    if (passes) *passes = s->passes;
    if (tokens) *tokens = s->tokens;
    if (n_unfinished) {
        *n_unfinished = 0;
        for (int f = 0; f < s->F; ++f) *n_unfinished += s->finished[f] ? 0 : 1;
    }
    return FDC_OK;
}

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
    // the layout must be the one fdc_build_mask produces: slots back to back after the prefix
    for (int g = 0; g < F; ++g) {
        if (slot_len[g] < 1) return fdc::fail(FDC_EINVAL, "slot_len[%d] = %d must be >= 1", g, slot_len[g]);
        const int64_t want = g == 0 ? (int64_t)prefix_len : (int64_t)slot_start[g - 1] + slot_len[g - 1];
        if (slot_start[g] != want) return fdc::fail(FDC_EINVAL, "slot_start[%d] = %d, expected %lld", g, slot_start[g], (long long)want);
    }
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
