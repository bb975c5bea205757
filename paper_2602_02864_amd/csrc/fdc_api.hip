// C ABI of the library: context, buffers, and the orchestration of one
// parallel decoding step (Sec. 3.3) out of the gfx950 kernels.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "fdc_internal.hpp"
#include "fdc_launch.hpp"

using namespace fdc;

#define FDC_HIP(call)                                                                         \
    do {                                                                                      \
        hipError_t e_ = (call);                                                               \
        if (e_ != hipSuccess)                                                                 \
            return fail(FDC_EHIP, "%s failed: %s", #call, hipGetErrorString(e_));             \
    } while (0)

namespace {
inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }
}  // namespace

struct fdc_ctx {
    fdc_model_desc m{};
    int F = 0, P = 0, N = 0, Npad = 0, NB = 0, B = 0, Rmax = 0, Tmax = 0, Mmax = 0;
    std::vector<int32_t> slot_len, slot_start, level, valid_len;
    std::vector<uint64_t> anc;
    std::vector<int32_t> edge_src, edge_dst;
    std::vector<fdc_layer_weights> lw;
    std::vector<char> lw_set;
    std::vector<fdc_layer_weights_f16> lw16;     // optional fp16 copies for steps of more than 16 rows
    std::vector<char> lw16_set;
    const uint16_t* lm16 = nullptr;
    int f16_mask = 0;                    // which projections may take the fp16 path: 1 QKV, 2 O, 4 gate/up, 8 down, 16 LM head
    const uint16_t* emb = nullptr;
    const float* gf = nullptr;
    const uint16_t* lm = nullptr;
    uint16_t* kc = nullptr;
    uint16_t* vc = nullptr;
    size_t kv_layer_elems = 0;

    GemmPlan p_qkv, p_o, p_gu, p_down, p_lm;
    int Mp = kMaxRowsDense;              // rows the workspace is laid out for (multiple of 16)

    // attention launch shape for the largest step
    int attn_nrt = 1, attn_rg_max = 1, attn_cb = 4, attn_chunks = 1, attn_variant = 0, attn_wq = 16;
    int step_cb = 0, step_wq = 0, step_chunks = 0;   // this step's chunk cut (many-row kernel); 0: the context's

    // workspace
    char* ws = nullptr;
    size_t ws_bytes = 0;
    struct Off {
        size_t anc, slot_start, mask_words, row_pos, inv_freq, rope_tab, meta, x, a_hi, a_lo, o_hi, o_lo, h_hi, h_lo,
            q, part, logits, attn_o, attn_ml, tok_tmp, end;
    } off{};
    size_t meta_ints = 0;

    // pinned staging ring for the per-step tables
    int32_t* stage[kStageSlots] = {};
    hipEvent_t stage_ev[kStageSlots] = {};
    bool stage_used[kStageSlots] = {};
    int stage_next = 0;
    std::vector<int32_t> meta_last;      // the tables the device holds (branch_field, branch_off, valid_len)
    int meta_last_T = 0;                 // ... their T (0: none valid) and the stream they were enqueued on
    hipStream_t meta_last_stream = nullptr;
    int32_t* drv_host = nullptr;         // pinned: token inputs [Mmax], token outputs [Mmax] of the CoT driver

    // optional per-kernel timing with HIP events (benchmarks only)
    bool prof_on = false;
    struct ProfRec { int kind; hipEvent_t e0, e1; };
    std::vector<ProfRec> prof_recs;      // recorded since the last read
    std::vector<ProfRec> prof_pool;      // idle event pairs

    template <class T>
    T* at(size_t o) const { return reinterpret_cast<T*>(ws + o); }
};

namespace {
// brackets one kernel launch with two events when profiling is on
struct ProfScope {
    fdc_ctx* c;
    hipStream_t st;
    fdc_ctx::ProfRec r{};
    bool live = false;
    ProfScope(fdc_ctx* c_, int kind, hipStream_t st_) : c(c_), st(st_) {
        if (!c->prof_on) return;
        if (!c->prof_pool.empty()) {
            r = c->prof_pool.back();
            c->prof_pool.pop_back();
        } else if (hipEventCreate(&r.e0) != hipSuccess || hipEventCreate(&r.e1) != hipSuccess) {
            return;
        }
        r.kind = kind;
        live = hipEventRecord(r.e0, st) == hipSuccess;
    }
    ~ProfScope() {
        if (!live) return;
        (void)hipEventRecord(r.e1, st);
        c->prof_recs.push_back(r);
    }
};
enum { PK_NORM = 0, PK_QKV, PK_ROPE, PK_ATTN, PK_O, PK_GATEUP, PK_DOWN, PK_LMHEAD, PK_ARGMAX, PK_COUNT };
static_assert(PK_COUNT == FDC_PROF_KINDS, "profile kinds");
}  // namespace

namespace {

void plan_attention(fdc_ctx* c) {
    const int G = c->m.n_q_heads / c->m.n_kv_heads;
    const int rows = c->Rmax * c->Tmax * G;
    int forced = -1;
    if (const char* e = std::getenv("FDC_ATTN_VARIANT")) forced = std::atoi(e);
    const long t0 = c->P / 32, masked_total = c->NB - t0;
    // More than 64 rows per KV head (several tokens per branch, many branches): one
    // workgroup of 4 or 8 wavefronts takes up to 128 / 256 rows of a KV head, so a
    // K/V tile is fetched once for all of them and shared through LDS.
    if (forced == 2 || (forced < 0 && rows > 64)) {
        c->attn_variant = 2;
        c->attn_nrt = rows > 128 ? 8 : 4;
        const int NR = c->attn_nrt * 32;
        c->attn_rg_max = (rows + NR - 1) / NR;
        // tiles past the prefix carry masks and measure about 1.5 plain tiles each:
        // chunks are cut equal in weighted tiles, or the chunk with the slots would
        // finish long after the others
        c->attn_wq = 24;
        const long total = t0 + (masked_total * c->attn_wq + 15) / 16;
        const long zr = (long)c->B * c->m.n_kv_heads * c->attn_rg_max;
        long want_wgs = c->attn_nrt == 8 ? 256 : 512;      // four-wavefront workgroups run two to a compute unit
        if (const char* e = std::getenv("FDC_ATTN_WGS")) want_wgs = std::max(1L, std::atol(e));
        const long chunks = std::max(1L, (want_wgs + zr / 2) / zr);
        long cb = (total + chunks - 1) / chunks;
        cb = std::min(std::max(4L, cb), (long)kMaxChunkTilesWide);
        if (masked_total > kMaxMaskedTiles) cb = std::min(cb, (long)kMaxMaskedTiles);
        c->attn_cb = (int)cb;
        c->attn_chunks = (int)((total + cb - 1) / cb);
        return;
    }
    c->attn_nrt = rows > 32 ? 2 : 1;
    const int NR = c->attn_nrt * 32;
    c->attn_rg_max = (rows + NR - 1) / NR;
    // A layer's K/V of tens of megabytes and more is a bandwidth problem: one
    // workgroup per compute unit (two at head_dim 64), tiles fetched straight
    // into registers.  Below that the call is a chain of latencies and fewer,
    // longer chunks (a shorter merge) with LDS-shared tiles measure faster.
    const long zr = (long)c->B * c->m.n_kv_heads * c->attn_rg_max;
    const double layer_kv_bytes = 4.0 * c->B * c->m.n_kv_heads * (double)c->Npad * c->m.head_dim;
    const bool large = layer_kv_bytes >= 64e6;
    c->attn_variant = large ? 1 : 0;
    long want_wgs = (large ? 256L : 128L) * (c->m.head_dim == 128 ? 1 : 2);
    if (const char* e = std::getenv("FDC_ATTN_WGS")) want_wgs = std::max(1L, std::atol(e));
    if (forced == 0 || forced == 1) c->attn_variant = forced;
    long cb, total = c->NB;
    if (c->attn_variant == 1 && !std::getenv("FDC_ATTN_WGS")) {
        // Tiles past the prefix carry masks and measure about 1.5 plain tiles
        // each (table set-up included): chunks are cut equal in weighted tiles.
        // Whole rounds of workgroups over the compute units: the cheapest of
        // (rounds) x (weighted tiles per chunk + a fixed set-up and merge cost).
        c->attn_wq = 24;
        total = t0 + (masked_total * c->attn_wq + 15) / 16;
        long best = 0, best_cost = 0;
        for (long ch = 1; ch <= std::max(1L, total / 8); ++ch) {
            const long t = (total + ch - 1) / ch;
            if (t > kMaxChunkTilesReg) continue;
            const long cost = ((zr * ch + 255) / 256) * (t + 6);
            if (best == 0 || cost < best_cost) {
                best = ch;
                best_cost = cost;
            }
        }
        cb = best ? (total + best - 1) / best : kMaxChunkTilesReg;
    } else {
        const long chunks = std::max(1L, (want_wgs + zr / 2) / zr);
        cb = (c->NB + chunks - 1) / chunks;
        cb = std::max(4L, (cb + 1) / 2 * 2);
        cb = std::min(cb, (long)(c->attn_variant == 1 ? kMaxChunkTilesReg : kMaxChunkTiles));
    }
    if (masked_total > kMaxMaskedTiles) cb = std::min(cb, (long)kMaxMaskedTiles);
    c->attn_cb = (int)cb;
    c->attn_chunks = (int)((total + cb - 1) / cb);
}

size_t carve(fdc_ctx* c) {
    const fdc_model_desc& m = c->m;
    size_t o = 0;
    auto take = [&](size_t bytes) {
        size_t at = o;
        o = align_up(o + bytes);
        return at;
    };
    const int Mp = c->Mp = std::max(kMaxRowsDense, (c->Mmax + 15) / 16 * 16);
    const size_t HqD = (size_t)m.n_q_heads * m.head_dim;
    const size_t Nqkv = (size_t)(m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim;
    c->off.anc = take(sizeof(uint64_t) * c->F);
    c->off.slot_start = take(sizeof(int32_t) * c->F);
    c->off.mask_words = take(sizeof(uint32_t) * (size_t)c->Mmax * std::max(1, c->NB - c->P / 32));
    c->off.row_pos = take(sizeof(int32_t) * (size_t)c->Mmax);
    c->off.inv_freq = take(sizeof(double) * (m.head_dim / 2));
    c->off.rope_tab = take(sizeof(float2) * (size_t)c->Npad * (m.head_dim / 2));
    c->meta_ints = (size_t)2 * c->B * c->Rmax + (size_t)c->B * c->F;
    c->off.meta = take(sizeof(int32_t) * c->meta_ints);
    c->off.x = take(sizeof(float) * Mp * m.d_model);
    c->off.a_hi = take(2 * (size_t)Mp * m.d_model);
    c->off.a_lo = take(2 * (size_t)Mp * m.d_model);
    c->off.o_hi = take(2 * (size_t)Mp * HqD);
    c->off.o_lo = take(2 * (size_t)Mp * HqD);
    c->off.h_hi = take(2 * (size_t)Mp * m.d_mlp);
    c->off.h_lo = take(2 * (size_t)Mp * m.d_mlp);
    c->off.q = take(sizeof(float) * (size_t)Mp * HqD);
    // split-K partials: the streaming kernels' splits for up to 16 rows, the
    // tiled kernels' for every larger step shape this context admits
    size_t part = 0;
    part = std::max(part, (size_t)c->p_qkv.S * kMaxRowsDense * Nqkv);
    part = std::max(part, (size_t)c->p_o.S * kMaxRowsDense * m.d_model);
    part = std::max(part, (size_t)c->p_down.S * kMaxRowsDense * m.d_model);
    for (int R = 1; R <= c->Rmax; ++R)
        for (int T = 1; T <= c->Tmax; ++T) {
            const int M = c->B * R * T;
            if (M <= kMaxRowsDense) continue;
            part = std::max(part, (size_t)plan_tiled(M, Nqkv, m.d_model, false).S * M * Nqkv);
            part = std::max(part, (size_t)plan_tiled(M, m.d_model, HqD, false).S * M * m.d_model);
            part = std::max(part, (size_t)plan_tiled(M, m.d_model, m.d_mlp, false).S * M * m.d_model);
        }
    c->off.part = take(sizeof(float) * part);
    c->off.logits = take(sizeof(float) * Mp * m.vocab);
    const size_t zr = (size_t)c->B * m.n_kv_heads * c->attn_rg_max;
    const size_t NR = (size_t)c->attn_nrt * 32;
    c->off.attn_o = take(sizeof(float) * zr * c->attn_chunks * NR * m.head_dim);
    c->off.attn_ml = take(sizeof(float) * zr * c->attn_chunks * NR * 2);
    c->off.tok_tmp = take(sizeof(int32_t) * 2 * c->Mmax);   // the CoT driver's token inputs, outputs
    c->off.end = o;
    return o;
}

// `appending`: the rows are new tokens (the decode step).  Slots fill from the
// front (Sec. 3.3), so the first new offset must not lie beyond what is written:
// a gap would be read by the row itself and by every descendant as if it held
// tokens.  A field may appear once per scene.
int32_t check_step(const fdc_ctx* c, int R, int T, const int32_t* bf, const int32_t* bo, bool appending) {
    if (!bf || !bo) return fail(FDC_EINVAL, "branch_field / branch_off is null");
    if (R < 1 || R > c->Rmax) return fail(FDC_ECAP, "n_branches %d outside 1..%d", R, c->Rmax);
    if (T < 1 || T > c->Tmax) return fail(FDC_ECAP, "T %d outside 1..%d", T, c->Tmax);
    for (int b = 0; b < c->B; ++b) {
        uint64_t seen = 0;
        for (int r = 0; r < R; ++r) {
            const int i = b * R + r, f = bf[i];
            if (f == -1) continue;
            if (f < 0 || f >= c->F) return fail(FDC_ERANGE, "branch %d: field %d outside 0..%d", i, f, c->F - 1);
            if (bo[i] < 0 || bo[i] + T > c->slot_len[f])
                return fail(FDC_ERANGE, "branch %d: offsets %d..%d do not fit slot %d of length %d", i,
                            bo[i], bo[i] + T - 1, f, c->slot_len[f]);
            if ((seen >> f) & 1ull) return fail(FDC_EINVAL, "scene %d: field %d is listed twice", b, f);
            seen |= 1ull << f;
            if (appending && bo[i] > c->valid_len[(size_t)b * c->F + f])
                return fail(FDC_ERANGE, "branch %d: offset %d would leave a gap after the %d tokens of field %d", i,
                            bo[i], c->valid_len[(size_t)b * c->F + f], f);
        }
    }
    return FDC_OK;
}

// pinned staging for the per-step tables and the CoT driver's tokens: allocated
// when the workspace is set (a context can be created and its plan inspected
// without a GPU)
int32_t ensure_staging(fdc_ctx* c) {
    // whole pages: sub-page pinned allocations share pages with other host data
    const size_t stage_bytes = align_up(sizeof(int32_t) * c->meta_ints, 4096);
    for (int i = 0; i < kStageSlots; ++i) {
        if (!c->stage[i]) FDC_HIP(hipHostMalloc((void**)&c->stage[i], stage_bytes, hipHostMallocDefault));
        if (!c->stage_ev[i]) FDC_HIP(hipEventCreateWithFlags(&c->stage_ev[i], hipEventDisableTiming));
    }
    if (!c->drv_host)
        FDC_HIP(hipHostMalloc((void**)&c->drv_host, align_up(sizeof(int32_t) * 2 * c->Mmax, 4096), hipHostMallocDefault));
    return FDC_OK;
}

// Brings branch tables + valid_len to the device through the pinned ring (a
// one-workgroup kernel reads them from host memory) and builds the step's
// visibility words and position table from them.  A call with the tables the
// device already holds (the attention of another layer in the same state, on the
// same stream) reuses both.
int32_t upload_meta(fdc_ctx* c, int R, const int32_t* bf, const int32_t* bo, hipStream_t st,
                    StepMeta* sm, int T) {
    const size_t nbr = (size_t)c->B * R;
    const size_t n = 2 * nbr + (size_t)c->B * c->F;
    int32_t* d = c->at<int32_t>(c->off.meta);
    sm->branch_field = d;
    sm->branch_off = d + nbr;
    sm->valid_len = d + 2 * nbr;
    sm->slot_start = c->at<int32_t>(c->off.slot_start);
    sm->row_pos = c->at<int32_t>(c->off.row_pos);
    sm->B = c->B;
    sm->R = R;
    sm->T = T;
    sm->F = c->F;
    std::vector<int32_t>& last = c->meta_last;
    if (c->meta_last_T == T && c->meta_last_stream == st && last.size() == n &&
        std::equal(bf, bf + nbr, last.begin()) && std::equal(bo, bo + nbr, last.begin() + nbr) &&
        std::equal(c->valid_len.begin(), c->valid_len.end(), last.begin() + 2 * nbr))
        return FDC_OK;
    c->meta_last_T = 0;                                  // nothing valid until all of it is enqueued
    const int slot = c->stage_next;
    c->stage_next = (slot + 1) % kStageSlots;
    if (c->stage_used[slot]) FDC_HIP(hipEventSynchronize(c->stage_ev[slot]));
    int32_t* h = c->stage[slot];
    std::memcpy(h, bf, sizeof(int32_t) * nbr);
    std::memcpy(h + nbr, bo, sizeof(int32_t) * nbr);
    std::memcpy(h + 2 * nbr, c->valid_len.data(), sizeof(int32_t) * c->B * c->F);
    launch_tables_copy(h, d, (int)n, st);              // the device reads the pinned tables itself
    FDC_HIP(hipEventRecord(c->stage_ev[slot], st));
    c->stage_used[slot] = true;
    launch_mask_words(*sm, c->at<uint64_t>(c->off.anc), c->P, c->NB - c->P / 32,
                      c->at<uint32_t>(c->off.mask_words), st);
    FDC_HIP(hipGetLastError());
    last.assign(h, h + n);
    c->meta_last_T = T;
    c->meta_last_stream = st;
    return FDC_OK;
}

// The many-row kernel skips slot tiles that no row of the step sees, so what a
// slot tile costs on average depends on the step: a pass of root fields touches one
// tile per branch, a pass of late fields nearly all of them.  The chunk cut weights
// a slot tile by wq / 16 plain tiles (attn_chunk_start); here wq is set from the
// step's own count of visible slot tiles (largest over the scenes; a visible one
// measures 1.2 plain tiles, plus about one tile's time of table set-up in the
// chunk that has them), with the chunk count the workspace was carved for.  A cut that would
// overflow a workgroup's tile list or mask table keeps the context's.
void balance_chunks(fdc_ctx* c, int R, int T, const int32_t* bf, const int32_t* bo) {
    c->step_cb = c->step_wq = c->step_chunks = 0;
    if (c->attn_variant != 2) return;
    const int t0 = c->P / 32, masked_total = c->NB - t0;
    if (masked_total <= 0) return;
    std::vector<uint8_t> seen((size_t)masked_total);
    int most = 0;
    for (int b = 0; b < c->B; ++b) {
        std::fill(seen.begin(), seen.end(), 0);
        auto mark = [&](int g, int len) {
            if (len <= 0) return;
            const int p0 = c->slot_start[g], p1 = p0 + len - 1;
            for (int t = p0 / 32; t <= p1 / 32; ++t) seen[t - t0] = 1;
        };
        for (int r = 0; r < R; ++r) {
            const int f = bf[b * R + r];
            if (f < 0) continue;
            mark(f, bo[b * R + r] + T);
            for (int g = 0; g < c->F; ++g)
                if (c->anc[f] >> g & 1) mark(g, c->valid_len[(size_t)b * c->F + g]);
        }
        int n = 0;
        for (uint8_t v : seen) n += v;
        most = std::max(most, n);
    }
    const double weight = 1.2 * most + 1.0;
    const int wq = (int)std::min(32.0, std::max(2.0, std::floor(16.0 * weight / masked_total + 0.5)));
    const long total = t0 + ((long)masked_total * wq + 15) / 16;
    long cb = (total + c->attn_chunks - 1) / c->attn_chunks;
    cb = std::max(4L, cb);
    const int chunks = (int)((total + cb - 1) / cb);
    if (chunks > c->attn_chunks) return;
    for (int ch = 0; ch < chunks; ++ch) {
        const int a0 = attn_chunk_start(c->P, c->NB, (int)cb, wq, ch);
        const int a1 = std::min(c->NB, attn_chunk_start(c->P, c->NB, (int)cb, wq, ch + 1));
        if (a1 - a0 > kMaxChunkTilesWide || a1 - std::max(a0, t0) > kMaxMaskedTiles) return;
    }
    if (attn_chunk_start(c->P, c->NB, (int)cb, wq, chunks) < c->NB) return;
    c->step_cb = (int)cb;
    c->step_wq = wq;
    c->step_chunks = chunks;
}

void fill_attn(const fdc_ctx* c, int layer, int R, int T, AttnArgs* a) {
    const fdc_model_desc& m = c->m;
    const int G = m.n_q_heads / m.n_kv_heads;
    const int rows = R * T * G;
    std::memset(a, 0, sizeof(*a));
    a->kc = c->kc + (size_t)layer * c->kv_layer_elems;
    a->vc = c->vc + (size_t)layer * c->kv_layer_elems;
    a->part_o = c->at<float>(c->off.attn_o);
    a->part_ml = c->at<float>(c->off.attn_ml);
    a->mask_words = c->at<uint32_t>(c->off.mask_words);
    a->mw_tiles = c->NB - c->P / 32;
    a->Hq = m.n_q_heads;
    a->Hkv = m.n_kv_heads;
    a->G = G;
    a->D = m.head_dim;
    a->P = c->P;
    a->NB = c->NB;
    a->CB = c->step_cb ? c->step_cb : c->attn_cb;
    a->wq = c->step_cb ? c->step_wq : c->attn_wq;
    a->n_chunks = c->step_cb ? c->step_chunks : c->attn_chunks;
    a->nrt = c->attn_nrt;
    a->variant = c->attn_variant;
    const int NR = a->nrt * 32;
    a->n_rg = (rows + NR - 1) / NR;
    a->scale_log2 = (float)(1.4426950408889634 / std::sqrt((double)m.head_dim));
}

bool aligned(const void* p, size_t a = 16) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

}  // namespace

namespace fdc {

GemmPlan plan_gemm(int64_t n_out, int64_t k_in, bool swiglu) {
    GemmPlan p;
    p.KT = (int)(k_in / 32);
    p.n_tiles = (int)((n_out + 15) / 16);
    p.nt = swiglu ? 2 : 1;
    p.n_tasks = p.n_tiles / p.nt;
    const int cap = 8 * 16;                          // k tiles one workgroup keeps in registers
    int S = 1;
    if (!swiglu) {
        const int s_min = (p.KT + cap - 1) / cap;
        const int s_want = (768 + p.n_tasks - 1) / std::max(1, p.n_tasks);
        S = std::max(s_min, std::min(s_want, std::max(1, p.KT / 4)));
        // a long K is cut so that a wavefront holds at most 8 k tiles: two
        // workgroups then fit a compute unit and cover each other's reduction
        // bubbles (measured on the 7B down projection: 28.8 -> 22.8 us)
        S = std::max(S, (p.KT + 63) / 64);
        S = std::max(s_min, std::min(S, 16));
    }
    p.kt_split = (p.KT + S - 1) / S;
    p.S = (p.KT + p.kt_split - 1) / p.kt_split;
    p.nw = p.kt_split >= 32 ? 8 : p.kt_split >= 16 ? 4 : p.kt_split >= 8 ? 2 : 1;
    const int per = (p.kt_split + p.nw - 1) / p.nw;
    static const int buckets[] = {2, 4, 6, 8, 10, 12, 14, 16, 20};
    p.ktw = 0;
    for (int b : buckets)
        if (b >= per) {
            p.ktw = b;
            break;
        }
    const int waves_per_cu = p.ktw <= 8 ? 16 : 8;
    const int wgs = std::max(1, 256 * std::max(1, waves_per_cu / p.nw) / p.S);
    p.grid = p.S * std::min(p.n_tasks, wgs);
    return p;
}

TiledPlan plan_tiled(int M, int64_t n_out, int64_t k_in, bool swiglu, int max_splits) {
    TiledPlan best;
    double best_cost = 0.0;
    const int KT = (int)(k_in / 32), n_tiles = (int)((n_out + 15) / 16), m_tiles = (M + 15) / 16;
    const int m_blocks = (m_tiles + 7) / 8;
    static const int widths[] = {4, 8, 10};
    for (int ntw : widths)
        for (int S = 1; S <= (swiglu ? 1 : max_splits); ++S) {
            const int kts = (KT + S - 1) / S;
            if (S > 1 && kts < 8) break;
            const int Seff = (KT + kts - 1) / kts;
            const int n_groups = (n_tiles + 2 * ntw - 1) / (2 * ntw);
            const long tasks = (long)n_groups * m_blocks * Seff;
            const long rounds = (tasks + 255) / 256;
            // Clocks of one workgroup, fitted to measurements of the 7B-class projections
            // at 256 and 1024 rows (the kernels are bound by the requests a compute unit
            // keeps in flight, not by the matrix pipe): a fixed part (launch, ramp,
            // epilogue) plus a cost per k tile - 1080 for the 128-wide tile; 2040 (up to
            // 256 rows) or 1820 for the 256-wide one, whose weight fragments go to two
            // wavefronts each; 2290 for the 320-wide one.  Every split writes its partial
            // and the consumer reads it: 3e-3 clocks per element and split, measured.
            const double fixed = ntw == 4 ? 19000.0 : 15000.0;
            const double per_kt = ntw == 4 ? 1080.0 : ntw == 8 ? (m_blocks <= 2 ? 2040.0 : 1820.0) : 2290.0;
            const double partials = Seff > 1 ? 3.0e-3 * Seff * M * (double)n_out : 0.0;
            const double cost = rounds * (kts * per_kt + fixed) + partials;
            if (best.grid == 0 || cost < best_cost) {
                best_cost = cost;
                best.KT = KT;
                best.n_tiles = n_tiles;
                best.m_tiles = m_tiles;
                best.S = Seff;
                best.kt_split = kts;
                best.ntw = ntw;
                best.n_groups = n_groups;
                best.m_blocks = m_blocks;
                best.grid = (int)((tasks + 7) / 8 * 8);
            }
        }
    return best;
}

}  // namespace fdc

extern "C" {

size_t fdc_packed_weight_bytes(int64_t n_out, int64_t k_in) {
    if (n_out <= 0 || k_in <= 0) return 0;
    return (size_t)((n_out + 15) / 16 * 16) * (size_t)k_in * 2;
}

int32_t fdc_pack_weight(const void* src, void* dst, int64_t n_out, int64_t k_in, int32_t mode,
                        void* stream) {
    if (!src || !dst) return fail(FDC_EINVAL, "null pointer argument");
    if (n_out <= 0 || k_in <= 0 || k_in % 32)
        return fail(FDC_EINVAL, "n_out (%lld) must be positive and k_in (%lld) a multiple of 32",
                    (long long)n_out, (long long)k_in);
    if (mode < 0 || mode > (FDC_PACK_GATE_UP | FDC_PACK_F16)) return fail(FDC_EINVAL, "unknown pack mode %d", mode);
    if ((mode & 1) == FDC_PACK_GATE_UP && n_out % 32) return fail(FDC_EINVAL, "gate/up packing needs n_out %% 32 == 0");
    if (!aligned(src) || !aligned(dst)) return fail(FDC_EINVAL, "pointers must be 16-byte aligned");
    launch_pack_weight((const uint16_t*)src, (uint16_t*)dst, n_out, k_in, mode, (hipStream_t)stream);
    FDC_HIP(hipGetLastError());
    return FDC_OK;
}

int32_t fdc_create(const fdc_model_desc* model, int32_t n_fields, const int32_t* slot_len,
                   int32_t n_edges, const int32_t* edge_src, const int32_t* edge_dst,
                   int32_t prefix_len, int32_t n_scenes, int32_t max_branches, int32_t max_tokens,
                   fdc_ctx** out) {
    if (!model || !out) return fail(FDC_EINVAL, "null pointer argument");
    *out = nullptr;
    const fdc_model_desc& m = *model;
    if (m.n_layers < 1 || m.d_model < 32 || m.n_q_heads < 1 || m.n_kv_heads < 1 || m.d_mlp < 32 ||
        m.vocab < 2 || !(m.rope_base > 1.0f) || !(m.norm_eps >= 0.0f))
        return fail(FDC_EINVAL, "bad model description");
    if (m.head_dim != 64 && m.head_dim != 128) return fail(FDC_ECAP, "head_dim %d: only 64 and 128 are built", m.head_dim);
    if (m.n_q_heads % m.n_kv_heads) return fail(FDC_EINVAL, "n_kv_heads must divide n_q_heads");
    if (m.d_model % 32 || m.d_mlp % 32 || m.vocab % 4)
        return fail(FDC_ECAP, "d_model and d_mlp must be multiples of 32, vocab of 4");
    if (n_fields > kMaxFields) return fail(FDC_ECAP, "n_fields %d above %d", n_fields, kMaxFields);
    if (n_scenes < 1 || max_branches < 1 || max_tokens < 1) return fail(FDC_EINVAL, "bad batch shape");
    if ((int64_t)n_scenes * max_branches * max_tokens > kMaxRowsStep)
        return fail(FDC_ECAP, "%lld rows per step above %d", (long long)n_scenes * max_branches * max_tokens, kMaxRowsStep);
    if (m.d_model > 8 * 20 * 32) return fail(FDC_ECAP, "d_model above %d", 8 * 20 * 32);

    fdc_ctx* c = new (std::nothrow) fdc_ctx;
    if (!c) return fail(FDC_EINVAL, "out of host memory");
    c->m = m;
    c->F = n_fields > 0 ? n_fields : 0;
    c->anc.resize(std::max(1, n_fields));
    c->slot_start.resize(std::max(1, n_fields));
    c->level.resize(std::max(1, n_fields));
    int32_t N = 0;
    int32_t rc = build_plan(n_fields, slot_len, n_edges, edge_src, edge_dst, prefix_len,
                            c->anc.data(), c->slot_start.data(), c->level.data(), &N);
    if (rc != FDC_OK) {
        delete c;
        return rc;
    }
    c->slot_len.assign(slot_len, slot_len + n_fields);
    if (n_edges > 0) {
        c->edge_src.assign(edge_src, edge_src + n_edges);
        c->edge_dst.assign(edge_dst, edge_dst + n_edges);
    }
    c->P = prefix_len;
    c->N = N;
    c->Npad = (N + 31) / 32 * 32;
    c->NB = c->Npad / 32;
    c->B = n_scenes;
    c->Rmax = max_branches;
    c->Tmax = max_tokens;
    c->Mmax = n_scenes * max_branches * max_tokens;
    c->valid_len.assign((size_t)n_scenes * n_fields, 0);
    c->lw.resize(m.n_layers);
    c->lw_set.assign(m.n_layers, 0);
    c->lw16.resize(m.n_layers);
    c->lw16_set.assign(m.n_layers, 0);
    c->kv_layer_elems = (size_t)n_scenes * m.n_kv_heads * c->Npad * m.head_dim;
    const int64_t HqD = (int64_t)m.n_q_heads * m.head_dim;
    c->p_qkv = plan_gemm(HqD + 2 * (int64_t)m.n_kv_heads * m.head_dim, m.d_model, false);
    c->p_o = plan_gemm(m.d_model, HqD, false);
    c->p_gu = plan_gemm(2 * (int64_t)m.d_mlp, m.d_model, true);
    c->p_down = plan_gemm(m.d_model, m.d_mlp, false);
    c->p_lm = plan_gemm(m.vocab, m.d_model, false);
    c->p_lm.S = 1;     // logits are written in place: one split
    c->p_lm.kt_split = c->p_lm.KT;
    {
        GemmPlan& p = c->p_lm;
        p.nw = 8;
        const int per = (p.kt_split + p.nw - 1) / p.nw;
        p.ktw = per <= 2 ? 2 : per <= 4 ? 4 : per <= 6 ? 6 : per <= 8 ? 8 : per <= 10 ? 10 : per <= 12 ? 12
              : per <= 14 ? 14 : per <= 16 ? 16 : 20;
        p.grid = std::min(p.n_tasks, 256 * (p.ktw <= 8 ? 2 : 1));
    }
    for (const GemmPlan* p : {&c->p_qkv, &c->p_o, &c->p_gu, &c->p_down, &c->p_lm})
        if (p->ktw == 0) {
            delete c;
            return fail(FDC_ECAP, "projection with K = %d does not fit the streaming kernel", p->KT * 32);
        }
    if (c->NB > 65535) {               // the attention kernels keep tile numbers in 16 bits
        delete c;
        return fail(FDC_ECAP, "%d cache positions: more than 65535 tiles of 32 keys", N);
    }
    c->f16_mask = kF16Default;
    if (const char* e = std::getenv("FDC_F16_MASK")) c->f16_mask = std::atoi(e) & 31;
    plan_attention(c);
    carve(c);
    *out = c;
    return FDC_OK;
}

void fdc_destroy(fdc_ctx* c) {
    if (!c) return;
    if (c->drv_host) (void)hipHostFree(c->drv_host);
    for (auto* v : {&c->prof_recs, &c->prof_pool})
        for (auto& r : *v) {
            (void)hipEventDestroy(r.e0);
            (void)hipEventDestroy(r.e1);
        }
    for (int i = 0; i < kStageSlots; ++i) {
        if (c->stage_ev[i]) {
            (void)hipEventSynchronize(c->stage_ev[i]);
            (void)hipEventDestroy(c->stage_ev[i]);
        }
        if (c->stage[i]) (void)hipHostFree(c->stage[i]);
    }
    delete c;
}

size_t fdc_kv_cache_bytes(const fdc_ctx* c) {
    return c ? sizeof(uint16_t) * c->kv_layer_elems * c->m.n_layers : 0;
}

size_t fdc_workspace_bytes(const fdc_ctx* c) { return c ? c->off.end : 0; }

int32_t fdc_set_kv_cache(fdc_ctx* c, void* k, void* v) {
    if (!c || !k || !v) return fail(FDC_EINVAL, "null pointer argument");
    if (!aligned(k, 256) || !aligned(v, 256)) return fail(FDC_EINVAL, "cache pointers must be 256-byte aligned");
    c->kc = (uint16_t*)k;
    c->vc = (uint16_t*)v;
    return FDC_OK;
}

int32_t fdc_set_workspace(fdc_ctx* c, void* ws, size_t bytes, void* stream) {
    if (!c || !ws) return fail(FDC_EINVAL, "null pointer argument");
    if (!aligned(ws, 256)) return fail(FDC_EINVAL, "workspace must be 256-byte aligned");
    if (bytes < c->off.end) return fail(FDC_EINVAL, "workspace of %zu bytes, %zu needed", bytes, c->off.end);
    hipStream_t st = (hipStream_t)stream;
    int32_t rc_st = ensure_staging(c);
    if (rc_st != FDC_OK) return rc_st;
    c->ws = (char*)ws;
    c->meta_last_T = 0;
    c->ws_bytes = bytes;
    // template tables (pageable host memory: the copies complete before return)
    std::vector<double> inv(c->m.head_dim / 2);
    for (int i = 0; i < c->m.head_dim / 2; ++i)
        inv[i] = std::pow((double)c->m.rope_base, -2.0 * i / c->m.head_dim);
    FDC_HIP(hipMemsetAsync(ws, 0, c->off.end, st));
    FDC_HIP(hipMemcpyAsync(c->at<void>(c->off.anc), c->anc.data(), sizeof(uint64_t) * c->F, hipMemcpyHostToDevice, st));
    FDC_HIP(hipMemcpyAsync(c->at<void>(c->off.slot_start), c->slot_start.data(), sizeof(int32_t) * c->F, hipMemcpyHostToDevice, st));
    FDC_HIP(hipMemcpyAsync(c->at<void>(c->off.inv_freq), inv.data(), sizeof(double) * inv.size(), hipMemcpyHostToDevice, st));
    launch_rope_table(c->at<double>(c->off.inv_freq), c->at<float2>(c->off.rope_tab), c->Npad, c->m.head_dim / 2, st);
    FDC_HIP(hipGetLastError());
    FDC_HIP(hipStreamSynchronize(st));
    return FDC_OK;
}

int32_t fdc_set_layer_weights(fdc_ctx* c, int32_t layer, const fdc_layer_weights* w) {
    if (!c || !w) return fail(FDC_EINVAL, "null pointer argument");
    if (layer < 0 || layer >= c->m.n_layers) return fail(FDC_ERANGE, "layer %d outside 0..%d", layer, c->m.n_layers - 1);
    if (!w->g1 || !w->wqkv || !w->wo || !w->g2 || !w->wgu || !w->wd) return fail(FDC_EINVAL, "null weight pointer");
    for (const void* p : {(const void*)w->g1, w->wqkv, w->wo, (const void*)w->g2, w->wgu, w->wd})
        if (!aligned(p)) return fail(FDC_EINVAL, "weight pointers must be 16-byte aligned");
    c->lw[layer] = *w;
    c->lw_set[layer] = 1;
    return FDC_OK;
}

int32_t fdc_set_head_weights(fdc_ctx* c, const void* emb, const float* gf, const void* lm) {
    if (!c || !emb || !gf || !lm) return fail(FDC_EINVAL, "null pointer argument");
    if (!aligned(emb) || !aligned(gf) || !aligned(lm)) return fail(FDC_EINVAL, "weight pointers must be 16-byte aligned");
    c->emb = (const uint16_t*)emb;
    c->gf = gf;
    c->lm = (const uint16_t*)lm;
    return FDC_OK;
}

int32_t fdc_set_layer_weights_f16(fdc_ctx* c, int32_t layer, const fdc_layer_weights_f16* w) {
    if (!c || !w) return fail(FDC_EINVAL, "null pointer argument");
    if (layer < 0 || layer >= c->m.n_layers) return fail(FDC_ERANGE, "layer %d outside 0..%d", layer, c->m.n_layers - 1);
    if (!w->wqkv || !w->wo || !w->wgu || !w->wd) return fail(FDC_EINVAL, "null weight pointer");
    for (const void* p : {w->wqkv, w->wo, w->wgu, w->wd})
        if (!aligned(p)) return fail(FDC_EINVAL, "weight pointers must be 16-byte aligned");
    c->lw16[layer] = *w;
    c->lw16_set[layer] = 1;
    return FDC_OK;
}

int32_t fdc_set_f16_projections(fdc_ctx* c, int32_t mask) {
    if (!c) return fail(FDC_EINVAL, "null context");
    if (mask < 0 || mask > 31) return fail(FDC_EINVAL, "projection mask %d outside 0..31", mask);
    c->f16_mask = mask;
    return FDC_OK;
}

int32_t fdc_set_head_weights_f16(fdc_ctx* c, const void* lm_f16) {
    if (!c || !lm_f16) return fail(FDC_EINVAL, "null pointer argument");
    if (!aligned(lm_f16)) return fail(FDC_EINVAL, "weight pointers must be 16-byte aligned");
    c->lm16 = (const uint16_t*)lm_f16;
    return FDC_OK;
}

int32_t fdc_reset(fdc_ctx* c) {
    if (!c) return fail(FDC_EINVAL, "null context");
    std::fill(c->valid_len.begin(), c->valid_len.end(), 0);
    return FDC_OK;
}

int32_t fdc_set_valid_len(fdc_ctx* c, const int32_t* v) {
    if (!c || !v) return fail(FDC_EINVAL, "null pointer argument");
    for (int b = 0; b < c->B; ++b)
        for (int g = 0; g < c->F; ++g)
            if (v[b * c->F + g] < 0 || v[b * c->F + g] > c->slot_len[g])
                return fail(FDC_ERANGE, "valid_len[%d][%d] = %d outside 0..%d", b, g, v[b * c->F + g], c->slot_len[g]);
    c->valid_len.assign(v, v + (size_t)c->B * c->F);
    return FDC_OK;
}

int32_t fdc_get_valid_len(const fdc_ctx* c, int32_t* v) {
    if (!c || !v) return fail(FDC_EINVAL, "null pointer argument");
    std::memcpy(v, c->valid_len.data(), sizeof(int32_t) * c->valid_len.size());
    return FDC_OK;
}

int32_t fdc_kv_append(fdc_ctx* c, int32_t layer, const void* k_new, const void* v_new,
                      const int32_t* row_scene, const int32_t* row_pos, int32_t n_rows, void* stream) {
    if (!c) return fail(FDC_EINVAL, "null context");
    if (!c->kc || !c->vc) return fail(FDC_ESTATE, "KV cache not set");
    if (layer < 0 || layer >= c->m.n_layers) return fail(FDC_ERANGE, "layer %d outside 0..%d", layer, c->m.n_layers - 1);
    if (n_rows < 0) return fail(FDC_EINVAL, "n_rows < 0");
    if (n_rows == 0) return FDC_OK;
    if (!k_new || !v_new || !row_scene || !row_pos) return fail(FDC_EINVAL, "null pointer argument");
    launch_kv_scatter((const uint16_t*)k_new, (const uint16_t*)v_new, row_scene, row_pos, n_rows,
                      c->kc + (size_t)layer * c->kv_layer_elems, c->vc + (size_t)layer * c->kv_layer_elems,
                      c->B, c->m.n_kv_heads, c->m.head_dim, c->NB, c->N, (hipStream_t)stream);
    FDC_HIP(hipGetLastError());
    return FDC_OK;
}

int32_t fdc_attention_plan(const fdc_ctx* c, int32_t* info, int32_t* chunk_first_tile) {
    if (!c || !info) return fail(FDC_EINVAL, "null pointer argument");
    info[0] = c->attn_variant;
    info[1] = c->attn_nrt;
    info[2] = c->attn_rg_max;
    info[3] = c->attn_chunks;
    info[4] = c->attn_cb;
    info[5] = c->attn_wq;
    info[6] = c->NB;
    info[7] = c->P / 32;
    info[8] = c->attn_variant == 2 ? kMaxChunkTilesWide : c->attn_variant == 1 ? kMaxChunkTilesReg : kMaxChunkTiles;
    info[9] = kMaxMaskedTiles;
    if (chunk_first_tile)
        for (int ch = 0; ch <= c->attn_chunks; ++ch)
            chunk_first_tile[ch] = attn_chunk_start(c->P, c->NB, c->attn_cb, c->attn_wq, ch);
    return FDC_OK;
}

int32_t fdc_attention_plan_step(fdc_ctx* c, int32_t R, int32_t T, const int32_t* bf, const int32_t* bo,
                                int32_t* info, int32_t* chunk_first_tile) {
    if (!c || !info) return fail(FDC_EINVAL, "null pointer argument");
    int32_t rc = check_step(c, R, T, bf, bo, false);
    if (rc != FDC_OK) return rc;
    rc = fdc_attention_plan(c, info, nullptr);
    if (rc != FDC_OK) return rc;
    balance_chunks(c, R, T, bf, bo);
    if (c->step_cb) {
        info[3] = c->step_chunks;
        info[4] = c->step_cb;
        info[5] = c->step_wq;
    }
    if (chunk_first_tile)
        for (int ch = 0; ch <= info[3]; ++ch)
            chunk_first_tile[ch] = attn_chunk_start(c->P, c->NB, info[4], info[5], ch);
    return FDC_OK;
}

int32_t fdc_step_tables_dense(fdc_ctx* c, int32_t R, int32_t T, const int32_t* bf, const int32_t* bo,
                              uint8_t* mask, int32_t* pos, void* stream) {
    if (!c || !mask || !pos) return fail(FDC_EINVAL, "null pointer argument");
    if (!c->ws) return fail(FDC_ESTATE, "workspace not set");
    hipStream_t st = (hipStream_t)stream;
    if (bf || bo) {
        int32_t rc = check_step(c, R, T, bf, bo, false);
        if (rc != FDC_OK) return rc;
        for (int i = 0; i < c->B * R; ++i)
            if (bf[i] >= 0 && c->valid_len[(size_t)(i / R) * c->F + bf[i]] < bo[i] + T)
                return fail(FDC_ERANGE, "branch %d: valid_len does not cover the rows' own tokens", i);
        StepMeta sm;
        rc = upload_meta(c, R, bf, bo, st, &sm, T);
        if (rc != FDC_OK) return rc;
    } else {
        // the tables of the last step or attention call, as they sit on the device
        const size_t fixed = (size_t)c->B * c->F;
        if (c->meta_last_T != T || T < 1 || R < 1 || c->meta_last.size() != 2 * (size_t)c->B * R + fixed)
            return fail(FDC_ESTATE, "the device holds no tables of a step with R = %d, T = %d", R, T);
    }
    const int RT = R * T, mw = c->NB - c->P / 32, t0 = c->P / 32;
    const size_t rows = (size_t)c->B * RT;
    std::vector<uint32_t> words((size_t)c->B * mw * RT);
    std::vector<int32_t> dpos(rows);
    FDC_HIP(hipMemcpyAsync(words.data(), c->at<void>(c->off.mask_words), sizeof(uint32_t) * words.size(),
                           hipMemcpyDeviceToHost, st));
    FDC_HIP(hipMemcpyAsync(dpos.data(), c->at<void>(c->off.row_pos), sizeof(int32_t) * rows, hipMemcpyDeviceToHost, st));
    FDC_HIP(hipStreamSynchronize(st));
    // What the attention kernels do with the tables: tiles that end inside the
    // prefix are visible to every active row without a word, every other tile
    // bit by bit; rows of inactive entries (position -1) see nothing.
    for (size_t m = 0; m < rows; ++m) {
        const int b = (int)(m / RT), j = (int)(m % RT);
        uint8_t* row = mask + m * (size_t)c->N;
        pos[m] = dpos[m];
        for (int key = 0; key < c->N; ++key) {
            const int t = key >> 5;
            if (dpos[m] < 0) row[key] = 0;
            else if (t < t0) row[key] = 1;
            else row[key] = (uint8_t)((words[((size_t)b * mw + (t - t0)) * RT + j] >> (key & 31)) & 1u);
        }
    }
    return FDC_OK;
}

int32_t fdc_masked_attention(fdc_ctx* c, int32_t layer, const void* q, int32_t R, int32_t T,
                             const int32_t* bf, const int32_t* bo, float* out, void* stream) {
    if (!c || !q || !out) return fail(FDC_EINVAL, "null pointer argument");
    if (!c->kc || !c->vc || !c->ws) return fail(FDC_ESTATE, "KV cache or workspace not set");
    if (layer < 0 || layer >= c->m.n_layers) return fail(FDC_ERANGE, "layer %d outside 0..%d", layer, c->m.n_layers - 1);
    int32_t rc = check_step(c, R, T, bf, bo, false);
    if (rc != FDC_OK) return rc;
    for (int i = 0; i < c->B * R; ++i)
        if (bf[i] >= 0 && c->valid_len[(size_t)(i / R) * c->F + bf[i]] < bo[i] + T)
            return fail(FDC_ERANGE, "branch %d: valid_len does not cover the rows' own tokens", i);
    if (!aligned(q) || !aligned(out)) return fail(FDC_EINVAL, "pointers must be 16-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    StepMeta sm;
    rc = upload_meta(c, R, bf, bo, st, &sm, T);
    if (rc != FDC_OK) return rc;
    AttnArgs a;
    balance_chunks(c, R, T, bf, bo);
    fill_attn(c, layer, R, T, &a);
    a.q_bf16 = (const uint16_t*)q;
    a.out_f32 = out;
    {
        ProfScope ps_(c, PK_ATTN, st);
        launch_attention(a, sm, st);
    }
    FDC_HIP(hipGetLastError());
    return FDC_OK;
}

int32_t fdc_parallel_decode_step(fdc_ctx* c, int32_t R, int32_t T, const int32_t* bf,
                                 const int32_t* bo, const int32_t* tok_in, const void* emb_in,
                                 int32_t* tok_out, float* gap_out, float* logits_out,
                                 float* hidden_out, void* stream) {
    if (!c) return fail(FDC_EINVAL, "null context");
    if (!c->kc || !c->vc || !c->ws || !c->emb || !c->gf || !c->lm) return fail(FDC_ESTATE, "cache, workspace or head weights not set");
    for (int l = 0; l < c->m.n_layers; ++l)
        if (!c->lw_set[l]) return fail(FDC_ESTATE, "weights of layer %d not set", l);
    if (!tok_out && (gap_out || logits_out))
        return fail(FDC_EINVAL, "tok_out is null although logits or gaps are asked for");
    if ((tok_in == nullptr) == (emb_in == nullptr)) return fail(FDC_EINVAL, "give exactly one of tok_in and emb_in");
    int32_t rc = check_step(c, R, T, bf, bo, true);
    if (rc != FDC_OK) return rc;
    const fdc_model_desc& m = c->m;
    const int M = c->B * R * T;
    if (M > c->Mp) return fail(FDC_ECAP, "%d rows in one step; this context was created for %d", M, c->Mp);
    if ((emb_in && !aligned(emb_in)) || (logits_out && !aligned(logits_out)) || (hidden_out && !aligned(hidden_out)))
        return fail(FDC_EINVAL, "pointers must be 16-byte aligned");
    hipStream_t st = (hipStream_t)stream;

    // append-then-attend: the step's own tokens count as written
    std::vector<int32_t> saved = c->valid_len;
    for (int i = 0; i < c->B * R; ++i)
        if (bf[i] >= 0) {
            int32_t& v = c->valid_len[(size_t)(i / R) * c->F + bf[i]];
            v = std::max(v, bo[i] + T);
        }
    StepMeta sm;
    rc = upload_meta(c, R, bf, bo, st, &sm, T);
    if (rc != FDC_OK) {
        c->valid_len = saved;
        return rc;
    }
    balance_chunks(c, R, T, bf, bo);

    const int d = m.d_model, HqD = m.n_q_heads * m.head_dim;
    const int Nqkv = HqD + 2 * m.n_kv_heads * m.head_dim;
    float* x = c->at<float>(c->off.x);
    float* part = c->at<float>(c->off.part);
    uint16_t *a_hi = c->at<uint16_t>(c->off.a_hi), *a_lo = c->at<uint16_t>(c->off.a_lo);
    uint16_t *o_hi = c->at<uint16_t>(c->off.o_hi), *o_lo = c->at<uint16_t>(c->off.o_lo);
    uint16_t *h_hi = c->at<uint16_t>(c->off.h_hi), *h_lo = c->at<uint16_t>(c->off.h_lo);
    float* q = c->at<float>(c->off.q);
    float* logits = logits_out ? logits_out : c->at<float>(c->off.logits);
    const size_t hstride = (size_t)M * d;

    // up to 16 rows the projections stream their weights once (bandwidth-bound);
    // above, they are tiled matrix products; either way `S` partials come back
    const bool tiled = M > kMaxRowsDense;
    // the single-pass fp16 projections: only in tiled steps, only those the mask
    // names, and only where the fp16 copies exist (layers: all or none)
    bool f16_layers = tiled;
    for (int l = 0; f16_layers && l < m.n_layers; ++l) f16_layers = c->lw16_set[l] != 0;
    const bool f16_head = tiled && c->lm16 != nullptr;
    const int fm = (f16_layers ? c->f16_mask & 15 : 0) | (f16_head ? c->f16_mask & 16 : 0);
    bool launched = true;              // false: a projection had no kernel for its plan
    auto project = [&](const GemmPlan& skinny, int64_t n_out, int64_t k_in, int epi, const GemmArgs& ga,
                       bool one_split) -> int {
        if (!tiled) {
            launched = launch_gemm(skinny, epi, ga, st) && launched;
            return skinny.S;
        }
        const TiledPlan tp = plan_tiled(M, n_out, k_in, epi == EPI_SWIGLU, one_split ? 1 : 16);
        launched = launch_gemm_tiled(tp, epi, ga, st) && launched;
        return tp.S;
    };

    NormArgs na{};
    na.x = x;
    na.eps = m.norm_eps;
    na.a_hi = a_hi;
    na.a_lo = a_lo;
    na.M = M;
    na.d = d;
    na.vocab = m.vocab;
    na.f16 = false;

    int s_down = c->p_down.S;
    for (int l = 0; l < m.n_layers; ++l) {
        const fdc_layer_weights& w = c->lw[l];
        // residual (embedding, or + MLP output of the previous layer) and attention norm
        NormArgs n1 = na;
        if (l == 0) {
            n1.tok = tok_in;
            n1.emb = c->emb;
            n1.emb_rows = (const uint16_t*)emb_in;
        } else {
            n1.part = part;
            n1.S = s_down;
        }
        n1.gain = w.g1;
        n1.f16 = (fm & 1) != 0;
        n1.hidden_x = hidden_out ? hidden_out + (size_t)l * hstride : nullptr;
        { ProfScope ps_(c, PK_NORM, st); launch_resid_norm(n1, sm, st); }

        GemmArgs g{};
        g.f16 = (fm & 1) != 0;
        g.out_scale = 1.0f / 256.0f;
        const fdc_layer_weights_f16& w16 = c->lw16[l];
        g.w = (const uint16_t*)(g.f16 ? w16.wqkv : w.wqkv);
        g.act_hi = a_hi;
        g.act_lo = a_lo;
        g.out = part;
        g.M = M;
        g.N = Nqkv;
        g.n_valid = Nqkv;
        int s_qkv;
        { ProfScope ps_(c, PK_QKV, st); s_qkv = project(c->p_qkv, Nqkv, d, EPI_PARTIAL, g, false); }

        RopeArgs ra{};
        ra.part = part;
        ra.S = s_qkv;
        ra.q = q;
        ra.kc = c->kc + (size_t)l * c->kv_layer_elems;
        ra.vc = c->vc + (size_t)l * c->kv_layer_elems;
        ra.tab = c->at<float2>(c->off.rope_tab);
        ra.M = M;
        ra.Hq = m.n_q_heads;
        ra.Hkv = m.n_kv_heads;
        ra.D = m.head_dim;
        ra.NB = c->NB;
        { ProfScope ps_(c, PK_ROPE, st); launch_rope_append(ra, sm, st); }

        AttnArgs aa;
        fill_attn(c, l, R, T, &aa);
        aa.q_f32 = q;
        aa.out_hi = o_hi;
        aa.out_lo = o_lo;
        aa.out_f16 = (fm & 2) != 0;
        { ProfScope ps_(c, PK_ATTN, st); launch_attention(aa, sm, st); }

        g.f16 = (fm & 2) != 0;
        g.w = (const uint16_t*)(g.f16 ? w16.wo : w.wo);
        g.act_hi = o_hi;
        g.act_lo = o_lo;
        g.N = d;
        g.n_valid = d;
        int s_o;
        { ProfScope ps_(c, PK_O, st); s_o = project(c->p_o, d, HqD, EPI_PARTIAL, g, false); }

        NormArgs n2 = na;
        n2.part = part;
        n2.S = s_o;
        n2.gain = w.g2;
        n2.f16 = (fm & 4) != 0;
        { ProfScope ps_(c, PK_NORM, st); launch_resid_norm(n2, sm, st); }

        GemmArgs gu{};
        gu.f16 = (fm & 4) != 0;
        gu.out_f16 = (fm & 8) != 0;
        gu.out_scale = 1.0f / 256.0f;
        gu.w = (const uint16_t*)(gu.f16 ? w16.wgu : w.wgu);
        gu.act_hi = a_hi;
        gu.act_lo = a_lo;
        gu.out_hi = h_hi;
        gu.out_lo = h_lo;
        gu.out_KT = m.d_mlp / 32;
        gu.M = M;
        { ProfScope ps_(c, PK_GATEUP, st); project(c->p_gu, 2 * (int64_t)m.d_mlp, d, EPI_SWIGLU, gu, true); }

        g.f16 = (fm & 8) != 0;
        g.w = (const uint16_t*)(g.f16 ? w16.wd : w.wd);
        g.act_hi = h_hi;
        g.act_lo = h_lo;
        g.N = d;
        g.n_valid = d;
        { ProfScope ps_(c, PK_DOWN, st); s_down = project(c->p_down, d, m.d_mlp, EPI_PARTIAL, g, false); }
    }
    NormArgs nf = na;
    nf.part = part;
    nf.S = s_down;
    nf.gain = c->gf;
    nf.f16 = (fm & 16) != 0;
    nf.hidden_x = hidden_out ? hidden_out + (size_t)m.n_layers * hstride : nullptr;
    nf.hidden_n = hidden_out ? hidden_out + (size_t)(m.n_layers + 1) * hstride : nullptr;
    { ProfScope ps_(c, PK_NORM, st); launch_resid_norm(nf, sm, st); }

    GemmArgs gl{};
    gl.f16 = (fm & 16) != 0;
    gl.out_scale = 1.0f / 256.0f;
    gl.w = gl.f16 ? c->lm16 : c->lm;
    gl.act_hi = a_hi;
    gl.act_lo = a_lo;
    gl.out = logits;
    gl.M = M;
    gl.N = m.vocab;
    gl.n_valid = m.vocab;
    // no tokens wanted (a prefill pass: the rows only fill the cache): no head
    if (tok_out) {
        { ProfScope ps_(c, PK_LMHEAD, st); project(c->p_lm, m.vocab, d, EPI_PARTIAL, gl, true); }
        { ProfScope ps_(c, PK_ARGMAX, st); launch_argmax(logits, M, m.vocab, m.vocab, tok_out, gap_out, sm.branch_field, T, st); }
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || !launched) {
        c->valid_len = saved;
        c->meta_last_T = 0;
        if (e != hipSuccess) return fail(FDC_EHIP, "kernel launch failed: %s", hipGetErrorString(e));
        return fail(FDC_ECAP, "a projection of this step has no kernel for its plan");
    }
    return FDC_OK;
}

// Algorithm 1 end to end: one scheduler per scene, one forward pass per
// iteration for the union of the ready sets, finishing decided on the host from
// the tokens the pass produced.
int32_t fdc_cot_decode(fdc_ctx* c, const int32_t* start_token, const int32_t* fixed_len,
                       const int32_t* fixed_tok, const int32_t* eos_ids, int32_t n_eos,
                       int32_t max_passes, int32_t* out_tok, int32_t* out_len, int32_t* out_passes,
                       void* stream) {
    if (!c) return fail(FDC_EINVAL, "null context");
    if (!start_token || !out_tok || !out_len) return fail(FDC_EINVAL, "null pointer argument");
    if (n_eos < 0 || (n_eos > 0 && !eos_ids)) return fail(FDC_EINVAL, "bad end-of-field token list");
    if (!c->ws) return fail(FDC_ESTATE, "cache, workspace or head weights not set");
    const int F = c->F, B = c->B, V = c->m.vocab;
    const int Smax = *std::max_element(c->slot_len.begin(), c->slot_len.end());
    std::vector<int32_t> fixed_at(F, 0);
    {
        int32_t at = 0;
        for (int f = 0; f < F; ++f) {
            const int n = fixed_len ? fixed_len[f] : 0;
            if (n < 0 || n > c->slot_len[f]) return fail(FDC_ERANGE, "fixed_len[%d] = %d outside 0..%d", f, n, c->slot_len[f]);
            if (n > 0 && !fixed_tok) return fail(FDC_EINVAL, "fixed_tok is null");
            fixed_at[f] = at;
            for (int i = 0; i < n; ++i)
                if (fixed_tok[at + i] < 0 || fixed_tok[at + i] >= V)
                    return fail(FDC_ERANGE, "token %d of fixed field %d outside the vocabulary", i, f);
            if (n == 0 && (start_token[f] < 0 || start_token[f] >= V))
                return fail(FDC_ERANGE, "start_token[%d] outside the vocabulary", f);
            at += n;
        }
    }
    hipStream_t st = (hipStream_t)stream;
    struct Scheds {
        std::vector<fdc_sched*> s;
        ~Scheds() { for (fdc_sched* p : s) fdc_sched_destroy(p); }
    } sch;
    sch.s.assign(B, nullptr);
    for (int b = 0; b < B; ++b) {
        int32_t rc = fdc_sched_create(F, (int32_t)c->edge_src.size(), c->edge_src.data(), c->edge_dst.data(),
                                      nullptr, &sch.s[b]);
        if (rc != FDC_OK) return rc;
    }
    std::fill(out_tok, out_tok + (size_t)B * F * Smax, -1);
    std::fill(out_len, out_len + (size_t)B * F, 0);
    std::fill(c->valid_len.begin(), c->valid_len.end(), 0);      // every slot starts empty

    int32_t* h_in = c->drv_host;
    int32_t* h_out = c->drv_host + c->Mmax;
    int32_t* d_in = c->at<int32_t>(c->off.tok_tmp);
    int32_t* d_out = d_in + c->Mmax;
    std::vector<int32_t> bf((size_t)B * c->Rmax), bo((size_t)B * c->Rmax);

    // fixed template text: known from the start, so each such field is filled by
    // multi-token passes (all scenes at once) before Algorithm 1 begins
    int32_t fixed_passes = 0;
    for (int f = 0; f < F; ++f) {
        const int n = fixed_len ? fixed_len[f] : 0;
        if (n == 0) continue;
        for (int b = 0; b < B; ++b) {
            int32_t rc = fdc_sched_complete(sch.s[b], f, n);
            if (rc != FDC_OK) return fail(FDC_EINVAL, "fixed field %d depends on a field that is not fixed", f);
        }
        for (int t0 = 0; t0 < n; t0 += c->Tmax) {
            const int T = std::min(c->Tmax, n - t0);
            for (int b = 0; b < B; ++b) {
                bf[b] = f;
                bo[b] = t0;
                for (int t = 0; t < T; ++t) h_in[b * T + t] = fixed_tok[fixed_at[f] + t0 + t];
            }
            launch_tables_copy(h_in, d_in, B * T, st);
            int32_t rc = fdc_parallel_decode_step(c, 1, T, bf.data(), bo.data(), d_in, nullptr, d_out, nullptr,
                                                  nullptr, nullptr, stream);
            if (rc != FDC_OK) return rc;
            FDC_HIP(hipStreamSynchronize(st));                   // h_in is reused
            ++fixed_passes;
        }
        for (int b = 0; b < B; ++b) {
            out_len[(size_t)b * F + f] = n;
            std::copy(fixed_tok + fixed_at[f], fixed_tok + fixed_at[f] + n, out_tok + ((size_t)b * F + f) * Smax);
        }
    }

    std::vector<int32_t> last((size_t)B * F);
    for (int b = 0; b < B; ++b) std::copy(start_token, start_token + F, last.begin() + (size_t)b * F);
    std::vector<int32_t> pf((size_t)B * c->Rmax), po((size_t)B * c->Rmax), nact(B), fin(c->Rmax);
    int32_t passes = 0;
    for (;;) {
        int R = 0;
        for (int b = 0; b < B; ++b) {
            int32_t rc = fdc_sched_peek(sch.s[b], c->Rmax, &pf[(size_t)b * c->Rmax], &po[(size_t)b * c->Rmax], &nact[b]);
            if (rc != FDC_OK) return rc;
            R = std::max(R, nact[b]);
        }
        if (R == 0) break;
        if (max_passes > 0 && passes >= max_passes)
            return fail(FDC_ECAP, "template not complete after %d passes", max_passes);
        for (int b = 0; b < B; ++b)
            for (int i = 0; i < R; ++i) {
                const bool on = i < nact[b];
                const int f = on ? pf[(size_t)b * c->Rmax + i] : -1;
                bf[(size_t)b * R + i] = f;
                bo[(size_t)b * R + i] = on ? po[(size_t)b * c->Rmax + i] : 0;
                h_in[(size_t)b * R + i] = on ? last[(size_t)b * F + f] : 0;
            }
        launch_tables_copy(h_in, d_in, B * R, st);
        int32_t rc = fdc_parallel_decode_step(c, R, 1, bf.data(), bo.data(), d_in, nullptr, d_out, nullptr, nullptr,
                                              nullptr, stream);
        if (rc != FDC_OK) return rc;
        launch_tables_copy(d_out, h_out, B * R, st);         // the device writes the pinned result buffer
        FDC_HIP(hipStreamSynchronize(st));
        // when a field counts as finished (Algorithm 1's test): the model ended
        // the line, or the slot is full (truncation to the fixed length)
        for (int b = 0; b < B; ++b) {
            for (int i = 0; i < nact[b]; ++i) {
                const int f = bf[(size_t)b * R + i], off = bo[(size_t)b * R + i];
                const int32_t t = h_out[(size_t)b * R + i];
                if (t < 0 || t >= V) return fail(FDC_EHIP, "pass %d produced token %d outside the vocabulary", passes, t);
                out_tok[((size_t)b * F + f) * Smax + off] = t;
                out_len[(size_t)b * F + f] = off + 1;
                last[(size_t)b * F + f] = t;
                fin[i] = off + 1 >= c->slot_len[f] || std::find(eos_ids, eos_ids + n_eos, t) != eos_ids + n_eos;
            }
            rc = fdc_sched_advance(sch.s[b], nact[b], fin.data());
            if (rc != FDC_OK) return rc;
        }
        ++passes;
    }
    if (out_passes) {
        out_passes[0] = passes;
        out_passes[1] = fixed_passes;
    }
    return FDC_OK;
}

int32_t fdc_profile_enable(fdc_ctx* c, int32_t on) {
    if (!c) return fail(FDC_EINVAL, "null context");
    c->prof_on = on != 0;
    return FDC_OK;
}

const char* fdc_profile_kind_name(int32_t kind) {
    static const char* names[PK_COUNT] = {"resid_norm", "qkv_proj", "rope_append", "masked_attention",
                                          "o_proj", "gate_up_swiglu", "down_proj", "lm_head", "argmax"};
    return kind >= 0 && kind < PK_COUNT ? names[kind] : nullptr;
}

int32_t fdc_profile_read(fdc_ctx* c, float* ms_sum, int32_t* launches) {
    if (!c || !ms_sum || !launches) return fail(FDC_EINVAL, "null pointer argument");
    for (int k = 0; k < FDC_PROF_KINDS; ++k) {
        ms_sum[k] = 0.f;
        launches[k] = 0;
    }
    for (auto& r : c->prof_recs) {
        FDC_HIP(hipEventSynchronize(r.e1));
        float ms = 0.f;
        FDC_HIP(hipEventElapsedTime(&ms, r.e0, r.e1));
        if (r.kind >= 0 && r.kind < FDC_PROF_KINDS) {
            ms_sum[r.kind] += ms;
            launches[r.kind] += 1;
        }
        c->prof_pool.push_back(r);
    }
    c->prof_recs.clear();
    return FDC_OK;
}

int32_t fdc_profile_calibrate(int32_t rounds, void* scratch, size_t scratch_bytes, float* overhead_us,
                              float* null_us, void* stream) {
    if (!overhead_us || rounds < 1 || rounds > 10000) return fail(FDC_EINVAL, "bad calibration arguments");
    if (scratch && (!aligned(scratch, 256) || scratch_bytes < 512)) return fail(FDC_EINVAL, "bad calibration scratch");
    const size_t half = scratch ? scratch_bytes / 2 / 256 * 256 : 0;
    auto launch_one = [&](hipStream_t s) {
        if (half) launch_stream_copy(scratch, (char*)scratch + half, half, s);
        else launch_null(s);
    };
    hipStream_t st = (hipStream_t)stream;
    hipEvent_t e[2] = {nullptr, nullptr};
    FDC_HIP(hipEventCreate(&e[0]));
    if (hipEventCreate(&e[1]) != hipSuccess) {
        (void)hipEventDestroy(e[0]);
        return fail(FDC_EHIP, "event creation failed");
    }
    // one launch between two events against two launches between two events:
    // the difference is one launch, the rest of the first is the pair's cost
    double sum1 = 0.0, sum2 = 0.0;
    hipError_t err = hipSuccess;
    for (int n = 1; n <= 2 && err == hipSuccess; ++n)
        for (int r = 0; r < rounds + 3 && err == hipSuccess; ++r) {
            err = hipEventRecord(e[0], st);
            for (int i = 0; i < n; ++i) launch_one(st);
            if (err == hipSuccess) err = hipEventRecord(e[1], st);
            if (err == hipSuccess) err = hipEventSynchronize(e[1]);
            float ms = 0.f;
            if (err == hipSuccess) err = hipEventElapsedTime(&ms, e[0], e[1]);
            if (r >= 3) (n == 1 ? sum1 : sum2) += ms;
        }
    (void)hipEventDestroy(e[0]);
    (void)hipEventDestroy(e[1]);
    if (err != hipSuccess) return fail(FDC_EHIP, "calibration: %s", hipGetErrorString(err));
    const double t1 = 1e3 * sum1 / rounds, t2 = 1e3 * sum2 / rounds;
    const double one = std::max(0.0, t2 - t1);
    *overhead_us = (float)std::max(0.0, t1 - one);
    if (null_us) *null_us = (float)one;
    return FDC_OK;
}

int32_t fdc_stream_copy(void* dst, const void* src, size_t bytes, void* stream) {
    if (!dst || !src) return fail(FDC_EINVAL, "null pointer argument");
    if (!aligned(dst) || !aligned(src) || bytes % 16) return fail(FDC_EINVAL, "copy needs 16-byte alignment and size");
    if (bytes == 0) return FDC_OK;
    launch_stream_copy(src, dst, bytes, (hipStream_t)stream);
    FDC_HIP(hipGetLastError());
    return FDC_OK;
}

int32_t fdc_argmax(const float* logits, int32_t M, int32_t V, int64_t ld, int32_t* idx_out,
                   float* gap, void* stream) {
    if (!logits || !idx_out) return fail(FDC_EINVAL, "null pointer argument");
    if (M < 0 || V < 1 || ld < V) return fail(FDC_EINVAL, "bad shape M=%d V=%d ld=%lld", M, V, (long long)ld);
    launch_argmax(logits, M, V, ld, idx_out, gap, nullptr, 1, (hipStream_t)stream);
    FDC_HIP(hipGetLastError());
    return FDC_OK;
}

size_t fdc_linear_scratch_bytes(int32_t M, int64_t n_out, int64_t k_in) {
    if (M < 1 || M > kMaxRowsStep || n_out < 16 || k_in < 32) return 0;
    const int Mp = (M + 15) / 16 * 16;
    const int S = M <= kMaxRowsDense ? plan_gemm(n_out, k_in, false).S : plan_tiled(M, n_out, k_in, false).S;
    return align_up(2 * (size_t)Mp * k_in) * 2 + align_up(sizeof(float) * S * M * n_out);
}

}  // extern "C"

namespace {

// the launches of one projection; `buf` holds the activation fragments
// (bf16 heads, then tails) and behind them the split-K partials
int32_t linear_enqueue(const float* x, const void* w, float* y, int32_t M, int64_t n_out, int64_t k_in,
                       void* buf, hipStream_t st) {
    char* s = (char*)buf;
    const int Mp = (M + 15) / 16 * 16;
    const size_t fb = align_up(2 * (size_t)Mp * k_in);
    uint16_t *hi = (uint16_t*)s, *lo = (uint16_t*)(s + fb);
    float* part = (float*)(s + 2 * fb);
    GemmArgs g{};
    g.w = (const uint16_t*)w;
    g.act_hi = hi;
    g.act_lo = lo;
    g.M = M;
    g.N = (int)n_out;
    g.n_valid = (int)n_out;
    int S;
    if (M <= kMaxRowsDense) {
        const GemmPlan p = plan_gemm(n_out, k_in, false);
        if (p.ktw == 0) return fail(FDC_ECAP, "k_in = %lld does not fit the streaming kernel", (long long)k_in);
        launch_to_frag(x, hi, lo, M, (int)k_in, st);
        S = p.S;
        g.out = S == 1 ? y : part;
        if (!launch_gemm(p, EPI_PARTIAL, g, st)) return fail(FDC_ECAP, "no streaming kernel for this shape");
    } else {
        const TiledPlan p = plan_tiled(M, n_out, k_in, false);
        launch_to_frag(x, hi, lo, M, (int)k_in, st);
        S = p.S;
        g.out = S == 1 ? y : part;
        if (!launch_gemm_tiled(p, EPI_PARTIAL, g, st)) return fail(FDC_ECAP, "no tiled kernel for this shape");
    }
    if (S > 1) launch_sum_partials(part, y, S, M, n_out, st);
    FDC_HIP(hipGetLastError());
    return FDC_OK;
}

int32_t check_linear(const float* x, const void* w, const float* y, int32_t M, int64_t n_out, int64_t k_in) {
    if (!x || !w || !y) return fail(FDC_EINVAL, "null pointer argument");
    if (M < 1 || M > kMaxRowsStep) return fail(FDC_ECAP, "M = %d outside 1..%d", M, kMaxRowsStep);
    if (n_out <= 0 || k_in <= 0 || n_out % 4 || k_in % 32) return fail(FDC_EINVAL, "n_out must be a multiple of 4, k_in of 32");
    if (!aligned(w) || !aligned(y)) return fail(FDC_EINVAL, "misaligned pointer");
    return FDC_OK;
}

// ---- scratch memory that nobody allocates -----------------------------------
// Every GPU the library runs on holds its own copy of this array, at its own
// address, until the process ends.  In host code the array's name is only a
// handle for hipGetSymbolAddress: what kernels, copies and fills get is the
// address that call returns for the current device, looked up once per device.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

int32_t static_scratch(void** out) {
    int dev = -1;
    FDC_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(FDC_ECAP, "device ordinal %d outside 0..%d", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        FDC_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || !aligned(p, 256)) return fail(FDC_EHIP, "device %d: no usable address for the static scratch array", dev);
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return FDC_OK;
}

}  // namespace

extern "C" {

int32_t fdc_linear(const float* x, const void* w, float* y, int32_t M, int64_t n_out, int64_t k_in,
                   void* scratch_dev, void* stream) {
    int32_t rc = check_linear(x, w, y, M, n_out, k_in);
    if (rc != FDC_OK) return rc;
    if (!scratch_dev) return fail(FDC_EINVAL, "null pointer argument");
    if (!aligned(scratch_dev, 256)) return fail(FDC_EINVAL, "misaligned pointer");
    return linear_enqueue(x, w, y, M, n_out, k_in, scratch_dev, (hipStream_t)stream);
}

int32_t fdc_linear_static(const float* x, const void* w, float* y, int32_t M, int64_t n_out, int64_t k_in,
                          void* stream) {
    int32_t rc = check_linear(x, w, y, M, n_out, k_in);
    if (rc != FDC_OK) return rc;
    const size_t need = fdc_linear_scratch_bytes(M, n_out, k_in);
    if (need == 0) return fail(FDC_ECAP, "shape M=%d n_out=%lld k_in=%lld not supported", M, (long long)n_out, (long long)k_in);
    if (need > kStaticScratchBytes)
        return fail(FDC_ECAP, "projection needs %zu bytes of scratch, the static buffer holds %zu", need,
                    kStaticScratchBytes);
    void* s = nullptr;
    rc = static_scratch(&s);
    if (rc != FDC_OK) return rc;
    return linear_enqueue(x, w, y, M, n_out, k_in, s, (hipStream_t)stream);
}

}  // extern "C"
