// DAG-masked GQA decode attention over the field-slot KV cache (Sec. 3.3).
//
// All query rows that share a KV head - every active branch of a scene, its T
// new tokens and the G query heads of the group - form one row group of up to
// 64 rows, so the shared prefix and every visible slot are streamed from HBM
// once for all of them (Sec. 3.3: one kernel serves every query token that
// reads the shared cache).  The key dimension is cut into
// chunks (split-K); one workgroup takes one chunk of one (scene, kv head, row
// group) and emits one partial softmax state; a second kernel merges the
// chunks' partials in a fixed order (no atomics: results are bit-reproducible).
//
// Inside a workgroup two independent tile streams run side by side (even / odd
// active tiles of the chunk).  A stream is NRT wavefronts, one per 32-row tile;
// they share each 32-key K/V tile through LDS.  Tiles are copied HBM -> LDS
// with the direct-to-LDS load (no registers involved) into a four-stage ring,
// so three tiles per stream are in flight while a fourth is consumed.  The
// cache stores tiles in matrix-operand order, so one load instruction moves a
// contiguous 1 KiB and the LDS image is read back conflict-free.
//
// The mask is never materialised in memory.  A row of field f at slot offset t
// sees the prefix, the first valid_len[g] keys of each strict ancestor slot g
// and the first t+1 keys of its own slot - a *count* of visible keys per slot.
// At start-up the workgroup turns those counts into one 32-bit visibility word
// per (row, tile) for the few tiles that reach into the slots; tiles no row can
// see are never fetched, prefix tiles run without any masking.
//
// Matrix-core mapping (v_mfma_f32_32x32x16_bf16): S^T = K * Q^T puts one query
// row in each lane (column = lane % 32), so the running max / sum are in-lane
// plus one exchange with lane ^ 32; the score registers are, unchanged, the
// P^T operand of O^T = V^T * P^T because the V tiles are stored in that key
// order.  Softmax weights (and fp32 queries) enter the matrix cores as a bf16
// head plus a bf16 tail, so the only bf16 rounding left is that of the cache.
#include <type_traits>

#include "kernels_common.hpp"
#include "fdc_launch.hpp"

namespace fdc {

namespace {

constexpr float kNegBig = -1.0e30f;     // score of a masked key
// The running maximum (log2 domain) never drops below this, so a masked score's
// exponent stays hugely negative and its weight is exactly 0 without a second
// masking pass, also for a row that has seen no visible key yet.
constexpr float kMaxFloor = -1.0e20f;
constexpr float kLazy = 8.0f;

// score or kNegBig by visibility bit k of `bits`, without a compare
__device__ __forceinline__ float keep_if(float x, uint32_t bits, int k) {
    const uint32_t keep = (uint32_t)((int32_t)(bits << (31 - k)) >> 31);
    return __uint_as_float((__float_as_uint(x) & keep) | (__float_as_uint(kNegBig) & ~keep));
}
constexpr int kStages = 4;
constexpr int kStreams = 2;

__device__ __forceinline__ int chunk_start(const AttnArgs& a, int c) {
    return attn_chunk_start(a.P, a.NB, a.CB, a.wq, c);
}

struct RowInfo {
    int m;       // global row of the step, or -1 if the row does not exist / is inactive
    int head;    // query head
    int field;
    int off;     // slot offset of this row's token
};

__device__ __forceinline__ RowInfo row_info(int gr, int b, int kvh, int G, const StepMeta& sm) {
    RowInfo ri{-1, 0, -1, 0};
    const int jr = gr / G, ridx = jr / sm.T, tt = jr % sm.T;
    if (ridx < sm.R) {
        const int f = sm.branch_field[b * sm.R + ridx];
        if (f >= 0) {
            ri.m = (b * sm.R + ridx) * sm.T + tt;
            ri.head = kvh * G + gr % G;
            ri.field = f;
            ri.off = sm.branch_off[b * sm.R + ridx] + tt;
        }
    }
    return ri;
}

union Frag {
    bf16x8 v;
    uint32_t u[4];
};

// two floats -> packed bf16 heads and packed bf16 tails (head + tail ~ value to 2^-17)
__device__ __forceinline__ void split2(float x, float y, uint32_t& hi, uint32_t& lo) {
    f32x2 v = {x, y};
    hi = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
    f32x2 r = {x - __uint_as_float(hi << 16), y - __uint_as_float(hi & 0xffff0000u)};
    lo = __builtin_bit_cast(uint32_t, __builtin_convertvector(r, bf16x2));
}

// bits of a 32-key visibility word that belong to this lane's 16 score registers:
// register i <-> key 8*(i/4) + 4*hh + i%4
__device__ __forceinline__ uint32_t lane_bits(uint32_t word, int hh) {
    const uint32_t x = word >> (4 * hh);
    return (x & 0xfu) | ((x >> 4) & 0xf0u) | ((x >> 8) & 0xf00u) | ((x >> 12) & 0xf000u);
}

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void glb_void;

// LDS accesses of the main loop are written out by hand.  The tile copies are
// asynchronous (direct-to-LDS loads counted by vmcnt) and stay in flight across
// iterations; letting the compiler see LDS reads there would make it wait for
// *all* outstanding copies before each of them.  So the loop uses raw LDS
// offsets, its own s_waitcnt and a bare s_barrier.
__device__ __forceinline__ uint32_t lds_off(const void* p) {
    return (uint32_t)(uintptr_t)(lds_void*)p;
}
__device__ __forceinline__ void lds_read128(Frag& f, uint32_t off) {
    asm volatile("ds_read_b128 %0, %1" : "=v"(f.v) : "v"(off));
}
template <int OFF>
__device__ __forceinline__ void lds_read128_at(Frag& f, uint32_t base) {   // OFF: immediate byte offset
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f.v) : "v"(base), "n"(OFF));
}
// the DJ 1 KiB fragments of one K or V tile, one address register for all of them
template <int DJ>
__device__ __forceinline__ void read_frags(Frag (&fr)[DJ], uint32_t base) {
    static_assert(DJ == 8 || DJ == 4, "head sizes 128 and 64");
    lds_read128_at<0>(fr[0], base);
    lds_read128_at<1024>(fr[1], base);
    lds_read128_at<2048>(fr[2], base);
    lds_read128_at<3072>(fr[3], base);
    if (DJ == 8) {
        lds_read128_at<4096>(fr[4 % DJ], base);
        lds_read128_at<5120>(fr[5 % DJ], base);
        lds_read128_at<6144>(fr[6 % DJ], base);
        lds_read128_at<7168>(fr[7 % DJ], base);
    }
}
__device__ __forceinline__ uint32_t lds_read32(uint32_t off) {
    uint32_t v;
    asm volatile("ds_read_b32 %0, %1" : "=v"(v) : "v"(off));
    return v;
}
// value of the lane 32 away (v_permlane32_swap exchanges the upper half of its
// first operand with the lower half of its second)
__device__ __forceinline__ float other_half(float x, int hh) {
    const uint32_t u = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float(hh ? r[0] : r[1]);
}

// Visibility words and position ids of one step.  Words: for every scene b,
// every 32-key tile t that reaches past the prefix and every branch-token row j
// (branch r, token tt: j = r * T + tt) the 32 bits "key k of the tile is visible
// to that row".  A row of field f at slot offset o sees what is left of the
// prefix in the tile, the first valid_len[g] keys of each strict ancestor slot g
// and the first o+1 keys of its own slot (Sec. 3.3; Eq. 1).  Positions: row
// m = (b * R + r) * T + tt sits at slot_start[f] + o, which is also its cache
// index (Sec. 3.3: the fixed slot lengths fix every position id); -1 marks the
// rows of inactive branch entries.  Both depend on the step only, not on the
// layer or the head: they are built once per step; every attention workgroup of
// every layer fetches the few words it needs, the rotary kernel the positions.
__global__ __launch_bounds__(256) void mask_words_kernel(StepMeta sm, const uint64_t* __restrict__ anc, int P,
                                                         int n_tiles, uint32_t* __restrict__ words,
                                                         int32_t* __restrict__ row_pos) {
    const int RT = sm.R * sm.T;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx < sm.B * RT) {
        const int br = idx / sm.T;
        const int f = sm.branch_field[br];
        row_pos[idx] = f >= 0 ? sm.slot_start[f] + sm.branch_off[br] + idx % sm.T : -1;
    }
    if (idx >= sm.B * n_tiles * RT) return;
    const int j = idx % RT, t = (idx / RT) % n_tiles, b = idx / (RT * n_tiles);
    const int r = j / sm.T, tt = j % sm.T;
    const int f = sm.branch_field[b * sm.R + r];
    uint32_t bits = 0;
    if (f >= 0) {
        const int off = sm.branch_off[b * sm.R + r] + tt;
        const int key0 = ((P >> 5) + t) * 32;
        if (key0 < P) {
            const int nb = min(P - key0, 32);
            bits = nb >= 32 ? 0xffffffffu : ((1u << nb) - 1u);
        }
        const unsigned long long av = anc[f];
        for (int g = 0; g < sm.F; ++g) {             // slots are laid out in field order
            const int s0 = sm.slot_start[g];
            if (s0 >= key0 + 32) break;
            // keys of slot g this row sees: its own up to its token, an ancestor's all written
            const int n = g == f ? off + 1 : ((av >> g) & 1ull) ? sm.valid_len[b * sm.F + g] : 0;
            const int lo = max(s0, key0), hi = min(s0 + n, key0 + 32);
            if (hi > lo) {
                const int nb = hi - lo;
                bits |= (nb >= 32 ? 0xffffffffu : ((1u << nb) - 1u)) << (lo - key0);
            }
        }
    }
    words[idx] = bits;
}

// QF32: the queries come in fp32 (inside the decode step) and are used as bf16
// head + tail; otherwise they are bf16 data and have no tail.
// Start-up tables of a workgroup: its rows, and for the tiles of its chunk that
// reach past the prefix one 32-key visibility word per (tile, row) plus their
// OR per tile.  Everything read from memory (branch tables, the step's
// visibility words) is fetched in one round trip; the words exist once per
// branch-token row (the G query heads of a branch token share them) and are
// copied to the rows.  Ends with a barrier.
template <int NR, int NT>
__device__ __forceinline__ void build_tables(const AttnArgs& a, const StepMeta& sm, int b, int kvh, int rg, int mt0,
                                             int nmt, int* row_m, int* row_head,
                                             uint32_t (*bmask)[NR], uint32_t (*rowmask)[NR], uint32_t* tile_any) {
    const int tid = threadIdx.x;
    // branch-token rows of this row group: jr = (rg * NR + r) / G
    const int RT = sm.R * sm.T;
    const int jr0 = (rg * NR) / a.G, nbr = (rg * NR + NR - 1) / a.G - jr0 + 1;
    const uint32_t* __restrict__ words = a.mask_words + ((size_t)b * a.mw_tiles + (mt0 - (a.P >> 5))) * RT;
    for (int idx = tid; idx < nmt * nbr; idx += NT) {
        const int t = idx / nbr, j = idx % nbr;
        bmask[t][j] = jr0 + j < RT ? words[(size_t)t * RT + jr0 + j] : 0u;
    }
    for (int r = tid; r < NR; r += NT) {
        const RowInfo ri = row_info(rg * NR + r, b, kvh, a.G, sm);
        row_m[r] = ri.m;
        row_head[r] = ri.head;
    }
    for (int t = tid; t < nmt; t += NT) tile_any[t] = 0u;
    __syncthreads();
    if (nmt > 0) {
        for (int idx = tid; idx < nmt * NR; idx += NT) {
            const int t = idx / NR, r = idx % NR;
            const uint32_t bits = row_m[r] >= 0 ? bmask[t][(rg * NR + r) / a.G - jr0] : 0u;
            rowmask[t][r] = bits;
            if (bits) atomicOr(&tile_any[t], bits);
        }
    }
    __syncthreads();
}

// The same tables without the per-branch staging array: every (tile, row) entry
// fetches its word itself (rows of one branch token read the same address).
template <int NR, int NT>
__device__ __forceinline__ void build_tables_direct(const AttnArgs& a, const StepMeta& sm, int b, int kvh, int rg,
                                                    int mt0, int nmt, int* row_m, int* row_head,
                                                    uint32_t (*rowmask)[NR], uint32_t* tile_any) {
    const int tid = threadIdx.x;
    const int RT = sm.R * sm.T;
    const uint32_t* __restrict__ words = a.mask_words + ((size_t)b * a.mw_tiles + (mt0 - (a.P >> 5))) * RT;
    for (int t = tid; t < nmt; t += NT) tile_any[t] = 0u;
    for (int r = tid; r < NR; r += NT) {
        const RowInfo ri = row_info(rg * NR + r, b, kvh, a.G, sm);
        row_m[r] = ri.m;
        row_head[r] = ri.head;
    }
    __syncthreads();
    // one row per thread, NT / NR threads to a row, every TS-th tile each: all words
    // of a thread are requested before the first is used (one memory latency, not
    // one per tile)
    static_assert(NT % NR == 0 && NR % 64 == 0, "whole threads per row, whole wavefronts per tile");
    constexpr int TS = NT / NR, PER = (kMaxMaskedTiles + TS - 1) / TS;
    const int r = tid % NR, tq = tid / NR;
    const int jr = (rg * NR + r) / a.G;
    const bool row_ok = row_m[r] >= 0 && jr < RT;
    uint32_t bits[PER];
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const int t = tq + k * TS;
        bits[k] = (row_ok && t < nmt) ? words[(size_t)t * RT + jr] : 0u;
    }
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const int t = tq + k * TS;
        if (t < nmt) {                                      // the same tile for the whole wavefront
            rowmask[t][r] = bits[k];
            // one atomic per wavefront: 64 lanes on one LDS word would take turns
            uint32_t v = bits[k];
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) v |= (uint32_t)__shfl_xor((int)v, o);
            if ((tid & 63) == 0 && v) atomicOr(&tile_any[t], v);
        }
    }
    __syncthreads();
}

template <int D, int NRT, bool QF32>
__global__ __launch_bounds__(kStreams* NRT * 64) void attn_partial_kernel(AttnArgs a, StepMeta sm) {
    constexpr int DJ = D / 16, DT = D / 32, NR = NRT * 32, NT = kStreams * NRT * 64;
    constexpr int TILE = 32 * D;                    // bf16 elements of one K (or V) tile
    constexpr int LPT = 2 * DJ;                     // 1 KiB load instructions per K+V tile
    constexpr int LPW = LPT / NRT;                  // ... issued by each wavefront of a stream
    __shared__ __attribute__((aligned(16))) uint16_t stage[kStreams][kStages][2 * TILE];
    __shared__ uint32_t bmask[kMaxMaskedTiles][NR];
    __shared__ uint32_t rowmask[kMaxMaskedTiles][NR];
    __shared__ uint32_t tile_any[kMaxMaskedTiles];
    __shared__ int row_m[NR], row_head[NR];
    __shared__ uint16_t act_list[kStreams][kMaxChunkTiles / kStreams];
    __shared__ int n_act[kStreams];
    __shared__ float xm[NR], xl[NR];

    const int chunk = blockIdx.x, rg = blockIdx.y, z = blockIdx.z;
    const int b = z / a.Hkv, kvh = z % a.Hkv;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int strm = wave / NRT, rt = wave % NRT;
    const int r32 = lane & 31, hh = lane >> 5;
    const int cb0 = chunk_start(a, chunk), blk_end = min(a.NB, chunk_start(a, chunk + 1));
    const int mt0 = max(cb0, a.P >> 5);             // first tile of the chunk that reaches past the prefix
    const int nmt = max(0, blk_end - mt0);

    // The query rows are requested first: where a row of the group lives (step
    // row m, head) follows from the launch shape alone; whether its branch is
    // active is known only after the tables and decides below if it is used.
    // row rt*32 + lane%32, d = 16*j + 8*(lane/32) + 0..7
    f32x4 qraw[QF32 ? DJ : 1][2];
    bf16x8 qb[QF32 ? 1 : DJ];
    {
        const int gr = rg * NR + rt * 32 + r32;
        const int jr = gr / a.G, ridx = jr / sm.T;
        const bool exists = ridx < sm.R;
        const int m = exists ? (b * sm.R + ridx) * sm.T + jr % sm.T : 0;
        const size_t qo = ((size_t)m * a.Hq + kvh * a.G + gr % a.G) * D + 8 * hh;
#pragma unroll
        for (int j = 0; j < DJ; ++j) {
            if (QF32) {
                qraw[j][0] = qraw[j][1] = f32x4{0.f, 0.f, 0.f, 0.f};
                if (exists) {
                    qraw[j][0] = *reinterpret_cast<const f32x4*>(a.q_f32 + qo + 16 * j);
                    qraw[j][1] = *reinterpret_cast<const f32x4*>(a.q_f32 + qo + 16 * j + 4);
                }
            } else {
                qb[j] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
                if (exists) qb[j] = *reinterpret_cast<const bf16x8*>(a.q_bf16 + qo + 16 * j);
            }
        }
    }

    // ---- start-up: rows, visibility words, tile lists ---
    build_tables<NR, NT>(a, sm, b, kvh, rg, mt0, nmt, row_m, row_head, bmask, rowmask, tile_any);
    if (wave < kStreams) {
        // candidates of stream w: tiles cb0 + w, cb0 + w + 2, ...; keep the visible ones
        const int blk = cb0 + wave + kStreams * lane;
        bool actv = blk < blk_end;
        if (actv && blk >= mt0) actv = tile_any[blk - mt0] != 0u;
        const unsigned long long mask = __ballot(actv);
        if (actv) act_list[wave][__popcll(mask & ((1ull << lane) - 1ull))] = (uint16_t)blk;
        if (lane == 0) n_act[wave] = __popcll(mask);
    }
    __syncthreads();
    const int n_mine = n_act[strm];
    const int n_iter = max(n_act[0], n_act[1]);
    // lane j keeps the j-th active tile of this stream (read back with readlane)
    const int my_tiles = lane < n_mine ? (int)act_list[strm][lane] : 0;

    // query operand in registers (zero for rows of inactive branches)
    Frag qh[DJ], ql[QF32 ? DJ : 1];
    {
        const bool act = row_m[rt * 32 + r32] >= 0;
#pragma unroll
        for (int j = 0; j < DJ; ++j) {
            if (QF32) {
                const f32x4 z = {0.f, 0.f, 0.f, 0.f};
                const f32x4 q0 = act ? qraw[j][0] : z, q1 = act ? qraw[j][1] : z;
                split2(q0[0], q0[1], qh[j].u[0], ql[j].u[0]);
                split2(q0[2], q0[3], qh[j].u[1], ql[j].u[1]);
                split2(q1[0], q1[1], qh[j].u[2], ql[j].u[2]);
                split2(q1[2], q1[3], qh[j].u[3], ql[j].u[3]);
            } else {
                qh[j].v = act ? qb[j] : bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
            }
        }
    }
    // the query loads above must not be counted among the tile loads below
    __builtin_amdgcn_s_waitcnt(0);

    f32x16 o[DT];
    float m_run = kMaxFloor, l_run = 0.f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[dt][i] = 0.f;

    const size_t tile_base = ((size_t)b * a.Hkv + kvh) * a.NB;
    // Tile i of this stream -> stage i % kStages.  The K half and the V half are LPT
    // pieces of 1 KiB; wavefront rt of the stream copies pieces rt*LPW .. +LPW.
    const uint32_t stage_off = lds_off(&stage[strm][0][0]);
    const uint32_t rowmask_off = lds_off(&rowmask[0][rt * 32 + r32]);
    const uint32_t any_off = lds_off(&tile_any[0]);
    auto issue = [&](int i, int stg) {
        if (i >= n_mine) return;
        const int blk = __builtin_amdgcn_readlane(my_tiles, i);
#pragma unroll
        for (int p = 0; p < LPW; ++p) {
            const int piece = rt * LPW + p;                 // < DJ: K, else V
            const uint16_t* src = (piece < DJ ? a.kc : a.vc) + (tile_base + blk) * TILE +
                                  (piece % DJ) * 512 + lane * 8;
            uint16_t* dst = &stage[strm][stg][piece * 512];
            __builtin_amdgcn_global_load_lds((glb_void*)src, (lds_void*)dst, 16, 0, 2 /* nt: streamed once */);
        }
    };
    // one 32-key tile against this wavefront's 32 rows; MASKED tiles reach into
    // the slots and carry a visibility word per row
    auto tile = [&](auto masked_tag, int stg, int blk) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        const uint32_t ks = stage_off + stg * (4 * TILE) + lane * 16;      // bytes
        const uint32_t vs = ks + 2 * TILE;
        uint32_t vbits = 0xffffu, anyb = 0xffffu;
        if (MASKED) {
            uint32_t w0 = lds_read32(rowmask_off + (blk - mt0) * (NR * 4));
            uint32_t w1 = lds_read32(any_off + (blk - mt0) * 4);
            // the registers are operands of the wait so that nothing that uses
            // them can be scheduled ahead of it
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(w0), "+v"(w1)::"memory");
            vbits = lane_bits(w0, hh);
            anyb = lane_bits(w1, hh);
        }
        Frag kf[DJ];
#pragma unroll
        for (int j = 0; j < DJ; ++j) lds_read128(kf[j], ks + j * 1024);
        f32x16 sc;
#pragma unroll
        for (int k = 0; k < 16; ++k) sc[k] = 0.f;
        // scalar loads share the counter and may return out of order, so only
        // a full drain is a safe wait
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int j = 0; j < DJ; ++j) {
            // tie the register to the wait so that the matrix instruction
            // cannot be scheduled before it
            asm volatile("" : "+v"(kf[j].v));
            sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[j].v, qh[j].v, sc, 0, 0, 0);
            if (QF32) sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[j].v, ql[j].v, sc, 0, 0, 0);
        }
        // V fragments: requested now, consumed after the softmax
        Frag vf[DT][2];
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int s = 0; s < 2; ++s) lds_read128(vf[dt][s], vs + (dt * 2 + s) * 1024);
        // running max and sum are kept in the exponent's (log2, scaled) domain
        float mx = kNegBig;
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            if (MASKED) sc[k] = keep_if(sc[k], vbits, k);
            mx = fmaxf(mx, sc[k]);
        }
        mx = fmaxf(mx, other_half(mx, hh));
        const float m_new = fmaxf(m_run, mx * a.scale_log2);
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        float psum = 0.f;
        float p[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            p[k] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[k], a.scale_log2, -m_new));
            psum += p[k];
        }
        l_run = l_run * alpha + psum;
        Frag ph[2], pl[2];
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int k = 0; k < 4; ++k)
                split2(p[8 * s + 2 * k], p[8 * s + 2 * k + 1], ph[s].u[k], pl[s].u[k]);
        if (__any(alpha != 1.0f)) {
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int k = 0; k < 16; ++k) o[dt][k] *= alpha;
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int s = 0; s < 2; ++s) asm volatile("" : "+v"(vf[dt][s].v));
        if (MASKED) {
            // keys nobody sees may be padding or not yet written: whatever the
            // cache holds there is zeroed so that 0 * garbage stays 0
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const uint32_t wm = ((anyb >> (8 * s + 2 * k) & 1u) ? 0x0000ffffu : 0u) |
                                        ((anyb >> (8 * s + 2 * k + 1) & 1u) ? 0xffff0000u : 0u);
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt) vf[dt][s].u[k] &= wm;
                }
        }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[dt][s].v, ph[s].v, o[dt], 0, 0, 0);
                o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[dt][s].v, pl[s].v, o[dt], 0, 0, 0);
            }
    };

#pragma unroll
    for (int i = 0; i < kStages - 1; ++i) issue(i, i);

    int stg = 0;
    for (int i = 0; i < n_iter; ++i) {
        // my copies of tile i have landed; up to kStages - 2 later tiles stay in flight
        const int ahead = min(n_mine - 1 - i, kStages - 2);
        if (ahead >= 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * LPW) : "memory");
        else if (ahead == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LPW) : "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        // everyone's copies of tile i landed; everyone is done with tile i-1
        asm volatile("s_barrier" ::: "memory");
        issue(i + kStages - 1, stg == 0 ? kStages - 1 : stg - 1);
        if (i < n_mine) {
            const int blk = __builtin_amdgcn_readlane(my_tiles, i);
            if (blk >= mt0) tile(std::true_type{}, stg, blk);
            else tile(std::false_type{}, stg, blk);
        }
        stg = stg == kStages - 1 ? 0 : stg + 1;
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");

    // ---- fold stream 1 into stream 0 through LDS, emit the chunk's partial ---------
    l_run += other_half(l_run, hh);
    __syncthreads();                                   // all tiles consumed: the ring is free
    f32x4* xo = reinterpret_cast<f32x4*>(&stage[0][0][0]);   // NRT * DT * 4 * 64 vectors
    if (strm == 1) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4)
                xo[((rt * DT + dt) * 4 + i4) * 64 + lane] =
                    f32x4{o[dt][4 * i4], o[dt][4 * i4 + 1], o[dt][4 * i4 + 2], o[dt][4 * i4 + 3]};
        if (hh == 0) {
            xm[rt * 32 + r32] = m_run;
            xl[rt * 32 + r32] = l_run;
        }
    }
    __syncthreads();
    if (strm == 0) {
        const int r = rt * 32 + r32;
        const float m1 = xm[r], l1 = xl[r];
        const float mg = fmaxf(m_run, m1);
        const float e0 = __builtin_amdgcn_exp2f(m_run - mg), e1 = __builtin_amdgcn_exp2f(m1 - mg);
        const size_t pidx = ((size_t)z * a.n_rg + rg) * a.n_chunks + chunk;
        f32x4* po = reinterpret_cast<f32x4*>(a.part_o) + pidx * (NRT * DT * 4 * 64);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const int idx = ((rt * DT + dt) * 4 + i4) * 64 + lane;
                const f32x4 mine = {o[dt][4 * i4], o[dt][4 * i4 + 1], o[dt][4 * i4 + 2], o[dt][4 * i4 + 3]};
                po[idx] = mine * e0 + xo[idx] * e1;
            }
        if (hh == 0) {
            float* ml = a.part_ml + (pidx * NR + r) * 2;
            ml[0] = mg;
            ml[1] = l_run * e0 + l1 * e1;
        }
    }
}

// ---------------------------------------------------------------------------
// Wide variant, for steps with many rows per KV head (several scenes' worth of
// branches x tokens x group heads: up to NRT * 32 = 256 rows).  One workgroup of
// NRT wavefronts - two per SIMD at NRT = 8 - takes ALL row tiles of one (scene,
// KV head, key chunk): every K/V tile is fetched from memory once (direct-to-LDS
// ring, as above) and read from LDS by all wavefronts, one row tile each.  With
// two wavefronts on a SIMD the matrix instructions of one run under the softmax
// arithmetic of the other.  A wavefront keeps 32 rows: queries (bf16 head + tail)
// and the output accumulators in registers, K and V fragments pass through one
// set of registers (K first, V re-uses them).  One tile stream per workgroup; a
// chunk holds at most 64 tiles (one per lane of the tile list).
template <int D, int NRT, bool QF32>
__global__ __launch_bounds__(NRT * 64, 2) void attn_partial_wide_kernel(AttnArgs a, StepMeta sm) {
    constexpr int DJ = D / 16, DT = D / 32, NR = NRT * 32, NT = NRT * 64;
    // TPI tiles are consumed between two barriers (with eight wavefronts two: half
    // as many barriers, and between them the wavefronts drift apart, so that on a
    // SIMD the matrix instructions of one run under the softmax arithmetic of the
    // other and the LDS reads spread out).  Ring: the TPI tiles being consumed plus
    // kDist tiles requested ahead.  Four wavefronts: three stages, so that two
    // workgroups share a compute unit's LDS.
    constexpr int TPI = NRT >= 8 ? 2 : 1;
    constexpr int kDist = NRT >= 8 ? 4 : 2;         // tiles in flight while a group is consumed (multiple of TPI)
    constexpr int kWideStages = TPI + kDist;
    constexpr int TILE = 32 * D;
    constexpr int LPT = 2 * DJ;                     // 1 KiB load instructions per K+V tile
    static_assert(LPT % NRT == 0 || NRT > LPT, "tile pieces must divide over the wavefronts");
    constexpr int LPW = LPT >= NRT ? LPT / NRT : 1; // pieces issued by each (issuing) wavefront
    constexpr int NISS = LPT >= NRT ? NRT : LPT;    // wavefronts that issue copies
    __shared__ __attribute__((aligned(16))) uint16_t stage[kWideStages][2 * TILE];
    __shared__ uint32_t rowmask[kMaxMaskedTiles][NR];
    __shared__ uint32_t tile_any[kMaxMaskedTiles];
    __shared__ int row_m[NR], row_head[NR];
    __shared__ uint16_t act_list[kMaxChunkTilesWide];
    __shared__ int n_act_sh;

    // Row groups of one (scene, KV head, chunk) read the same tiles: consecutive
    // ids on one compute die (launch ids go round the eight dies)
    const int n_wg = gridDim.x * gridDim.y * gridDim.z;
    int lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
    if ((n_wg & 7) == 0) lin = (lin & 7) * (n_wg >> 3) + (lin >> 3);
    const int rg = lin % a.n_rg, chunk = (lin / a.n_rg) % a.n_chunks, z = lin / (a.n_rg * a.n_chunks);
    const int b = z / a.Hkv, kvh = z % a.Hkv;
    // the wavefront's index as a scalar: tile piece numbers and copy addresses then
    // live in scalar registers
    const int tid = threadIdx.x, rt = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int r32 = lane & 31, hh = lane >> 5;
    const int cb0 = chunk_start(a, chunk), blk_end = min(a.NB, chunk_start(a, chunk + 1));
    const int mt0 = max(cb0, a.P >> 5);
    const int nmt = max(0, blk_end - mt0);

    // The query rows are requested first: where a row of the group lives (step row
    // m, head) follows from the launch shape alone; whether its branch is active is
    // known only after the tables and decides below if it is used.
    f32x4 qraw[QF32 ? DJ : 1][2];
    bf16x8 qb[QF32 ? 1 : DJ];
    {
        const int gr = rg * NR + rt * 32 + r32;
        const int jr = gr / a.G, ridx = jr / sm.T;
        const bool exists = ridx < sm.R;
        const int m = exists ? (b * sm.R + ridx) * sm.T + jr % sm.T : 0;
        const size_t qo = ((size_t)m * a.Hq + kvh * a.G + gr % a.G) * D + 8 * hh;
#pragma unroll
        for (int j = 0; j < DJ; ++j) {
            if (QF32) {
                qraw[j][0] = qraw[j][1] = f32x4{0.f, 0.f, 0.f, 0.f};
                if (exists) {
                    qraw[j][0] = *reinterpret_cast<const f32x4*>(a.q_f32 + qo + 16 * j);
                    qraw[j][1] = *reinterpret_cast<const f32x4*>(a.q_f32 + qo + 16 * j + 4);
                }
            } else {
                qb[j] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
                if (exists) qb[j] = *reinterpret_cast<const bf16x8*>(a.q_bf16 + qo + 16 * j);
            }
        }
    }

    // Tiles of the prefix are visible to every row: when the chunk starts with kDist
    // of them their copies leave now, under the table set-up, not after it.
    const size_t tile_base = ((size_t)b * a.Hkv + kvh) * a.NB;
    const uint32_t lane_off = (uint32_t)lane * 8;           // bf16 elements
    auto issue_tile = [&](int blk, int stg) {               // blk, stg: scalar
        const size_t toff = (tile_base + blk) * TILE;
#pragma unroll
        for (int p = 0; p < LPW; ++p) {
            const int piece = rt * LPW + p;                 // < DJ: K, else V (scalar)
            const uint16_t* base = (piece < DJ ? a.kc : a.vc) + toff + (piece % DJ) * 512;
            uint16_t* dst = &stage[stg][piece * 512];
            __builtin_amdgcn_global_load_lds((glb_void*)(base + lane_off), (lds_void*)dst, 16, 0, 2 /* nt: streamed once */);
        }
    };
    const bool early = cb0 + kDist <= min(mt0, blk_end);
    if (early && rt < NISS) {
#pragma unroll
        for (int i = 0; i < kDist; ++i) issue_tile(cb0 + i, i);
    }

    build_tables_direct<NR, NT>(a, sm, b, kvh, rg, mt0, nmt, row_m, row_head, rowmask, tile_any);
    if (rt == 0) {
        const int blk = cb0 + lane;                         // at most 64 tiles per chunk
        bool actv = blk < blk_end;
        if (actv && blk >= mt0) actv = tile_any[blk - mt0] != 0u;
        const unsigned long long mask = __ballot(actv);
        if (actv) act_list[__popcll(mask & ((1ull << lane) - 1ull))] = (uint16_t)blk;
        if (lane == 0) n_act_sh = __popcll(mask);
    }
    __syncthreads();
    const int n_act = n_act_sh;
    const int my_tiles = lane < n_act ? (int)act_list[lane] : 0;

    // query operand (bf16 head + tail), zero for rows of inactive branches; the
    // loads have landed while the tables were built
    Frag qh[DJ], ql[QF32 ? DJ : 1];
    const bool row_act = row_m[rt * 32 + r32] >= 0;
    // a wavefront none of whose rows is active still copies its share of the tiles
    // and meets the barriers, but does no arithmetic
    const bool wave_act = __any(row_act);
#pragma unroll
    for (int j = 0; j < DJ; ++j) {
        if (QF32) {
            const f32x4 zz = {0.f, 0.f, 0.f, 0.f};
            const f32x4 q0 = row_act ? qraw[j][0] : zz, q1 = row_act ? qraw[j][1] : zz;
            split2(q0[0], q0[1], qh[j].u[0], ql[j].u[0]);
            split2(q0[2], q0[3], qh[j].u[1], ql[j].u[1]);
            split2(q1[0], q1[1], qh[j].u[2], ql[j].u[2]);
            split2(q1[2], q1[3], qh[j].u[3], ql[j].u[3]);
        } else {
            qh[j].v = row_act ? qb[j] : bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
        }
    }
    // no load of the set-up may be counted among the tile copies below (copies that
    // left early have landed by then, which the loop's waits allow for)
    __builtin_amdgcn_s_waitcnt(0);

    auto issue = [&](int i, int stg) {
        if (i >= n_act || rt >= NISS) return;
        issue_tile(__builtin_amdgcn_readlane(my_tiles, i), stg);
    };
    if (!early) {
#pragma unroll
        for (int i = 0; i < kDist; ++i) issue(i, i);
    }

    f32x16 o[DT];
    float m_run = kMaxFloor, l_run = 0.f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[dt][i] = 0.f;

    const uint32_t stage_off = lds_off(&stage[0][0]) + lane * 16;
    const uint32_t rowmask_off = lds_off(&rowmask[0][rt * 32 + r32]);
    const uint32_t any_off = lds_off(&tile_any[0]);
    // One 32-key tile against this wavefront's 32 rows, in two phases: scores
    // (S^T = K * Q^T into `sc`), then softmax and O^T += V^T * P^T.  The eight
    // fragments of K and then the eight of V pass through the same registers.
    // Query heads and tails accumulate into the same registers: the other wavefront
    // of the SIMD fills the gaps between dependent matrix instructions.
    f32x16 sc;
    auto scores = [&](int stg) {
        const uint32_t ks = stage_off + stg * (4 * TILE);   // bytes
        Frag fr[DJ];
        read_frags<DJ>(fr, ks);
#pragma unroll
        for (int k = 0; k < 16; ++k) sc[k] = 0.f;
        constexpr int HJ = DJ / 2;
        asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(HJ) : "memory");
#pragma unroll
        for (int j = 0; j < HJ; ++j) {
            asm volatile("" : "+v"(fr[j].v));
            sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j].v, qh[j].v, sc, 0, 0, 0);
            if (QF32) sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j].v, ql[j].v, sc, 0, 0, 0);
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int j = HJ; j < DJ; ++j) {
            asm volatile("" : "+v"(fr[j].v));
            sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j].v, qh[j].v, sc, 0, 0, 0);
            if (QF32) sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j].v, ql[j].v, sc, 0, 0, 0);
        }
    };
    auto softmax_pv = [&](int stg, int blk) {
        const bool masked = blk >= mt0;                     // the tile reaches into the slots
        const uint32_t vs = stage_off + stg * (4 * TILE) + 2 * TILE;
        uint32_t vbits = 0xffffu, anyb = 0xffffu;
        bool holes = false;                                 // some key of the tile is seen by no row
        // the V fragments are requested now and consumed after the softmax:
        // fragment dt*2 + s2 of the V half of the stage
        Frag fr[DJ];
        read_frags<DJ>(fr, vs);
        if (masked) {
            uint32_t w0 = lds_read32(rowmask_off + (blk - mt0) * (NR * 4));
            uint32_t w1 = lds_read32(any_off + (blk - mt0) * 4);
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(w0), "+v"(w1)::"memory");
            vbits = lane_bits(w0, hh);
            anyb = lane_bits(w1, hh);
            holes = __builtin_amdgcn_readfirstlane(w1) != 0xffffffffu;
#pragma unroll
            for (int k = 0; k < 16; ++k) sc[k] = keep_if(sc[k], vbits, k);
        }
        float mx = kNegBig;
#pragma unroll
        for (int k = 0; k < 16; ++k) mx = fmaxf(mx, sc[k]);
        mx = fmaxf(mx, other_half(mx, hh));
        float m_new = fmaxf(m_run, mx * a.scale_log2);
        // the reference point of the exponentials moves only when a score exceeds it by
        // more than 2^kLazy: weights then stay below 2^kLazy (no loss in fp32 or in the
        // head + tail pair), and the rescaling of the 64 accumulator registers is skipped
        // for almost every tile after a chunk's first
        if (m_new - m_run <= kLazy) m_new = m_run;
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        float psum = 0.f;
        Frag ph[2], pl[2];
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[8 * s2 + 2 * k], a.scale_log2, -m_new));
                const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[8 * s2 + 2 * k + 1], a.scale_log2, -m_new));
                psum += p0 + p1;
                split2(p0, p1, ph[s2].u[k], pl[s2].u[k]);
            }
        l_run = l_run * alpha + psum;
        if (__any(alpha != 1.0f)) {
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int k = 0; k < 16; ++k) o[dt][k] *= alpha;
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int j = 0; j < DJ; ++j) asm volatile("" : "+v"(fr[j].v));
        if (holes) {
            // keys nobody sees may be padding or not yet written: zeroed so that 0 * garbage stays 0
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const uint32_t wm = ((anyb >> (8 * s2 + 2 * k) & 1u) ? 0x0000ffffu : 0u) |
                                        ((anyb >> (8 * s2 + 2 * k + 1) & 1u) ? 0xffff0000u : 0u);
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt) fr[dt * 2 + s2].u[k] &= wm;
                }
        }
        // round the four output blocks: consecutive matrix instructions are independent
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
                o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[dt * 2 + s2].v, ph[s2].v, o[dt], 0, 0, 0);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
                o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[dt * 2 + s2].v, pl[s2].v, o[dt], 0, 0, 0);
        }
    };

    // Main loop: groups of TPI tiles.  Barrier g: every copy of the tiles of group g
    // has landed, and nobody reads the tiles of group g - 1 any more; their stages
    // take the copies of the group kDist tiles ahead.
    int stg = 0;
    for (int i0 = 0; i0 < n_act; i0 += TPI) {
        if (rt < NISS) {
            // my copies of the group have landed; later groups stay in flight
            const int later = min(n_act - (i0 + TPI), kDist - TPI);
            if (later >= 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * LPW) : "memory");
            else if (later == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LPW) : "memory");
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        asm volatile("s_barrier" ::: "memory");
#pragma unroll
        for (int t = 0; t < TPI; ++t) {
            int into = stg + t + kDist;
            if (into >= kWideStages) into -= kWideStages;
            issue(i0 + t + kDist, into);
        }
#pragma unroll
        for (int t = 0; t < TPI; ++t) {
            if (i0 + t < n_act && wave_act) {
                int st = stg + t;
                if (st >= kWideStages) st -= kWideStages;
                scores(st);
                softmax_pv(st, __builtin_amdgcn_readlane(my_tiles, i0 + t));
            }
        }
        stg += TPI;
        if (stg >= kWideStages) stg -= kWideStages;
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");

    // ---- emit the chunk's partial: every wavefront its own row tile ---------------
    l_run += other_half(l_run, hh);
    const size_t pidx = ((size_t)z * a.n_rg + rg) * a.n_chunks + chunk;
    f32x4* po = reinterpret_cast<f32x4*>(a.part_o) + pidx * (NRT * DT * 4 * 64);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4)
            po[((rt * DT + dt) * 4 + i4) * 64 + lane] =
                f32x4{o[dt][4 * i4], o[dt][4 * i4 + 1], o[dt][4 * i4 + 2], o[dt][4 * i4 + 3]};
    if (hh == 0) {
        float* ml = a.part_ml + (pidx * NR + rt * 32 + r32) * 2;
        ml[0] = m_run;
        ml[1] = l_run;
    }
}

// ---------------------------------------------------------------------------
// Register variant.  Four independent wavefronts per workgroup; each takes every
// fourth active tile of the chunk, handles ALL row tiles of the row group for
// it, and fetches its tiles straight into registers (one tile ahead), so there
// is no LDS traffic for K/V and no barrier in the loop.  The four softmax
// states meet in LDS at the end (fixed order).
template <int D, int NRT, bool QF32>
__global__ __launch_bounds__(256) void attn_partial_reg_kernel(AttnArgs a, StepMeta sm) {
    constexpr int DJ = D / 16, DT = D / 32, NR = NRT * 32, NT = 256;
    constexpr int TILE = 32 * D;
    __shared__ uint32_t bmask[kMaxMaskedTiles][NR];
    __shared__ uint32_t rowmask[kMaxMaskedTiles][NR];
    __shared__ uint32_t tile_any[kMaxMaskedTiles];
    __shared__ int row_m[NR], row_head[NR];
    __shared__ uint16_t act_list[kMaxChunkTilesReg];
    __shared__ int n_act_sh;
    __shared__ float red_m[4][NR], red_l[4][NR];
    __shared__ f32x4 red_o[2 * NRT * DT * 4 * 64];
    __shared__ bf16x8 qlo[QF32 ? NRT * DJ * 64 : 1];

    // Row groups of the same (scene, KV head, chunk) read the same tiles: they
    // get consecutive ids on one compute die (launch ids go round the eight
    // dies), so that one fetch from memory serves them all through that die's L2.
    const int n_wg = gridDim.x * gridDim.y * gridDim.z;
    int lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
    if ((n_wg & 7) == 0) lin = (lin & 7) * (n_wg >> 3) + (lin >> 3);
    const int rg = lin % a.n_rg, chunk = (lin / a.n_rg) % a.n_chunks, z = lin / (a.n_rg * a.n_chunks);
    const int b = z / a.Hkv, kvh = z % a.Hkv;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int r32 = lane & 31, hh = lane >> 5;
    const int cb0 = chunk_start(a, chunk), blk_end = min(a.NB, chunk_start(a, chunk + 1));
    const int mt0 = max(cb0, a.P >> 5);
    const int nmt = max(0, blk_end - mt0);

    build_tables<NR, NT>(a, sm, b, kvh, rg, mt0, nmt, row_m, row_head, bmask, rowmask, tile_any);
    if (wave == 0) {
        int base = 0;
        for (int c0 = 0; c0 < a.CB; c0 += 64) {               // CB <= kMaxChunkTilesReg
            const int blk = cb0 + c0 + lane;
            bool actv = blk < blk_end;
            if (actv && blk >= mt0) actv = tile_any[blk - mt0] != 0u;
            const unsigned long long mask = __ballot(actv);
            if (actv) act_list[base + __popcll(mask & ((1ull << lane) - 1ull))] = (uint16_t)blk;
            base += __popcll(mask);
        }
        if (lane == 0) n_act_sh = base;
    }
    // query operand: head (bf16) in registers, tail in LDS (filled below, after the
    // first tile is on its way)
    Frag qh[NRT][DJ];
    __syncthreads();
    const int n_act = n_act_sh;

    f32x16 o[NRT][DT];
    float m_run[NRT], l_run[NRT];
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) {
        m_run[rt] = kMaxFloor;
        l_run[rt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[rt][dt][i] = 0.f;
    }
    const size_t tile_base = ((size_t)b * a.Hkv + kvh) * a.NB;
    auto load_tile = [&](int blk, Frag (&kf)[DJ], Frag (&vf)[DT][2]) {
        const uint16_t* kt = a.kc + (tile_base + blk) * TILE + lane * 8;
        const uint16_t* vt = a.vc + (tile_base + blk) * TILE + lane * 8;
#pragma unroll
        for (int j = 0; j < DJ; ++j)
            kf[j].v = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(kt + j * 512));
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int s = 0; s < 2; ++s)
                vf[dt][s].v = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(vt + (dt * 2 + s) * 512));
    };
    auto tile = [&](auto masked_tag, int blk, Frag (&kf)[DJ], Frag (&vf)[DT][2]) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        uint32_t anyb = 0xffffu;
        if (MASKED) {
            anyb = lane_bits(tile_any[blk - mt0], hh);
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const uint32_t wm = ((anyb >> (8 * s + 2 * k) & 1u) ? 0x0000ffffu : 0u) |
                                        ((anyb >> (8 * s + 2 * k + 1) & 1u) ? 0xffff0000u : 0u);
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt) vf[dt][s].u[k] &= wm;
                }
        }
        // scores of every row tile first: the matrix pipe then has work queued
        // while the vector ALUs run the softmax of the first row tile
        f32x16 sc[NRT];
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt) {
#pragma unroll
            for (int k = 0; k < 16; ++k) sc[rt][k] = 0.f;
#pragma unroll
            for (int j = 0; j < DJ; ++j) {
                sc[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[j].v, qh[rt][j].v, sc[rt], 0, 0, 0);
                if (QF32)
                    sc[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[j].v, qlo[(rt * DJ + j) * 64 + lane], sc[rt], 0, 0, 0);
            }
        }
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt) {
            uint32_t vbits = 0xffffu;
            if (MASKED) vbits = lane_bits(rowmask[blk - mt0][rt * 32 + r32], hh);
            float mx = kNegBig;
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                if (MASKED) sc[rt][k] = keep_if(sc[rt][k], vbits, k);
                mx = fmaxf(mx, sc[rt][k]);
            }
            mx = fmaxf(mx, other_half(mx, hh));
            const float m_new = fmaxf(m_run[rt], mx * a.scale_log2);
            const float alpha = __builtin_amdgcn_exp2f(m_run[rt] - m_new);
            m_run[rt] = m_new;
            float psum = 0.f;
            float p[16];
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                p[k] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[rt][k], a.scale_log2, -m_new));
                psum += p[k];
            }
            l_run[rt] = l_run[rt] * alpha + psum;
            Frag ph[2], pl[2];
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    split2(p[8 * s + 2 * k], p[8 * s + 2 * k + 1], ph[s].u[k], pl[s].u[k]);
            // unconditional: a branch here would cut the tile into scheduling regions
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int k = 0; k < 16; ++k) o[rt][dt][k] *= alpha;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    o[rt][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[dt][s].v, ph[s].v, o[rt][dt], 0, 0, 0);
                    o[rt][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[dt][s].v, pl[s].v, o[rt][dt], 0, 0, 0);
                }
        }
    };

    Frag kn[DJ], vn[DT][2];
    int i = wave;
    if (i < n_act) load_tile(act_list[i], kn, vn);
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) {
        const int r = rt * 32 + r32;
        const int m = row_m[r];
#pragma unroll
        for (int j = 0; j < DJ; ++j) {
            Frag lo;
#pragma unroll
            for (int k = 0; k < 4; ++k) qh[rt][j].u[k] = lo.u[k] = 0;
            if (m >= 0) {
                const size_t qo = ((size_t)m * a.Hq + row_head[r]) * D + 16 * j + 8 * hh;
                if (QF32) {
                    const f32x4 q0 = *reinterpret_cast<const f32x4*>(a.q_f32 + qo);
                    const f32x4 q1 = *reinterpret_cast<const f32x4*>(a.q_f32 + qo + 4);
                    split2(q0[0], q0[1], qh[rt][j].u[0], lo.u[0]);
                    split2(q0[2], q0[3], qh[rt][j].u[1], lo.u[1]);
                    split2(q1[0], q1[1], qh[rt][j].u[2], lo.u[2]);
                    split2(q1[2], q1[3], qh[rt][j].u[3], lo.u[3]);
                } else {
                    qh[rt][j].v = *reinterpret_cast<const bf16x8*>(a.q_bf16 + qo);
                }
            }
            if (QF32 && wave == 0) qlo[(rt * DJ + j) * 64 + lane] = lo.v;
        }
    }
    if (QF32) __syncthreads();                       // the query tails are in LDS
    while (i < n_act) {
        // keeps the query tail in LDS (re-read per tile) instead of in registers
        if (QF32) asm volatile("" ::: "memory");
        Frag kf[DJ], vf[DT][2];
#pragma unroll
        for (int j = 0; j < DJ; ++j) kf[j] = kn[j];
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            vf[dt][0] = vn[dt][0];
            vf[dt][1] = vn[dt][1];
        }
        const int blk = act_list[i];
        const int nxt = i + 4;
        if (nxt < n_act) load_tile(act_list[nxt], kn, vn);      // in flight during this tile's math
        if (blk >= mt0) tile(std::true_type{}, blk, kf, vf);
        else tile(std::false_type{}, blk, kf, vf);
        i = nxt;
    }

    // ---- merge the four wavefronts (fixed order), emit one partial ---------------
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) {
        l_run[rt] += other_half(l_run[rt], hh);
        if (hh == 0) red_m[wave][rt * 32 + r32] = m_run[rt];
    }
    __syncthreads();
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) {
        const int r = rt * 32 + r32;
        const float mg = fmaxf(fmaxf(red_m[0][r], red_m[1][r]), fmaxf(red_m[2][r], red_m[3][r]));
        const float e = __builtin_amdgcn_exp2f(m_run[rt] - mg);
        if (hh == 0) red_l[wave][r] = l_run[rt] * e;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int k = 0; k < 16; ++k) o[rt][dt][k] *= e;
    }
    // two rounds instead of four: wavefronts 0 and 1 store into a buffer each,
    // wavefronts 2 and 3 add into them, the store to memory adds the two:
    // (w0 + w2) + (w1 + w3), the same order every time
    constexpr int Q = NRT * DT * 4 * 64;
    for (int round = 0; round < 2; ++round) {
        if ((wave >> 1) == round) {
            f32x4* dst = red_o + (wave & 1) * Q;
#pragma unroll
            for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int i4 = 0; i4 < 4; ++i4) {
                        const f32x4 v = {o[rt][dt][4 * i4], o[rt][dt][4 * i4 + 1], o[rt][dt][4 * i4 + 2],
                                         o[rt][dt][4 * i4 + 3]};
                        const int idx = ((rt * DT + dt) * 4 + i4) * 64 + lane;
                        if (round == 0) dst[idx] = v;
                        else dst[idx] += v;
                    }
        }
        __syncthreads();
    }
    const size_t pidx = ((size_t)z * a.n_rg + rg) * a.n_chunks + chunk;
    f32x4* po = reinterpret_cast<f32x4*>(a.part_o) + pidx * Q;
    for (int q = tid; q < Q; q += 256) po[q] = red_o[q] + red_o[Q + q];
    if (tid < NR) {
        float* ml = a.part_ml + (pidx * NR + tid) * 2;
        ml[0] = fmaxf(fmaxf(red_m[0][tid], red_m[1][tid]), fmaxf(red_m[2][tid], red_m[3][tid]));
        ml[1] = red_l[0][tid] + red_l[1][tid] + red_l[2][tid] + red_l[3][tid];
    }
}

// Merge the chunks' partials of one (scene, kv head, row group) in chunk order.
// One thread per accumulator quad (4 consecutive head-dim elements of one row) in
// the partial's own order, so reads are contiguous; chunks are fetched four at a
// time (CB independent loads per thread) and folded with a running maximum.
template <int D, int NRT, int CB>
__global__ __launch_bounds__(256) void attn_merge_kernel(AttnArgs a, StepMeta sm) {
    constexpr int DT = D / 32, NR = NRT * 32, Q4 = NRT * DT * 4 * 64;
    const int q4 = blockIdx.x * blockDim.x + threadIdx.x;
    if (q4 >= Q4) return;
    const int zr = blockIdx.y, z = zr / a.n_rg, rg = zr % a.n_rg;
    const int b = z / a.Hkv, kvh = z % a.Hkv;
    const int lane = q4 & 63, i4 = (q4 >> 6) & 3, dt = (q4 >> 8) % DT, rt = (q4 >> 8) / DT;
    const int r = rt * 32 + (lane & 31);
    const int d0 = 32 * dt + 8 * i4 + 4 * (lane >> 5);
    // The partials are requested before the branch tables are looked at (their
    // addresses do not depend on them); rows of inactive branches read theirs
    // for nothing.
    const size_t p0 = (size_t)zr * a.n_chunks;
    const f32x4* __restrict__ po = reinterpret_cast<const f32x4*>(a.part_o) + p0 * Q4 + q4;
    const float2* __restrict__ pml = reinterpret_cast<const float2*>(a.part_ml) + p0 * NR + r;
    float mg = kNegBig, L = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    RowInfo ri{-1, 0, -1, 0};
    for (int c0 = 0; c0 < a.n_chunks; c0 += CB) {
        float2 ml[CB];
        f32x4 o[CB];
#pragma unroll
        for (int j = 0; j < CB; ++j) {
            const int c = min(c0 + j, a.n_chunks - 1);
            ml[j] = pml[(size_t)c * NR];
            o[j] = po[(size_t)c * Q4];
        }
        if (c0 == 0) ri = row_info(rg * NR + r, b, kvh, a.G, sm);
        // all loads above are in flight together; entries past the last chunk
        // (repeats of it) get weight 0 instead of a branch, which would push the
        // arrays out of registers and serialise the loads
#pragma unroll
        for (int j = 0; j < CB; ++j) {
            if (c0 + j >= a.n_chunks) ml[j] = make_float2(kNegBig, 0.f);
            const float mn = fmaxf(mg, ml[j].x);
            const float e_old = __builtin_amdgcn_exp2f(mg - mn), e_new = __builtin_amdgcn_exp2f(ml[j].x - mn);
            L = L * e_old + ml[j].y * e_new;
            acc = acc * e_old + o[j] * e_new;
            mg = mn;
        }
    }
    if (ri.m < 0) {
        // rows of inactive branches: zero in the fp32 output, nothing for fragments
        const int gr = rg * NR + r, jr = gr / a.G, ridx = jr / sm.T;
        if (a.out_f32 && ridx < sm.R) {
            const int m = (b * sm.R + ridx) * sm.T + jr % sm.T;
            const int head = kvh * a.G + gr % a.G;
            *reinterpret_cast<f32x4*>(a.out_f32 + ((size_t)m * a.Hq + head) * D + d0) =
                f32x4{0.f, 0.f, 0.f, 0.f};
        }
        return;
    }
    acc *= L > 0.f ? 1.0f / L : 0.f;
    if (a.out_f32) {
        *reinterpret_cast<f32x4*>(a.out_f32 + ((size_t)ri.m * a.Hq + ri.head) * D + d0) = acc;
    } else {
        const size_t o = act_frag_index(ri.m, ri.head * D + d0, a.Hq * D / 32);
        if (a.out_f16) {
            *reinterpret_cast<uint2*>(a.out_hi + o) =
                make_uint2(f2h(acc[0]) | (uint32_t)f2h(acc[1]) << 16, f2h(acc[2]) | (uint32_t)f2h(acc[3]) << 16);
        } else {
            uint32_t hi[2], lo[2];
            split2(acc[0], acc[1], hi[0], lo[0]);
            split2(acc[2], acc[3], hi[1], lo[1]);
            *reinterpret_cast<uint2*>(a.out_hi + o) = make_uint2(hi[0], hi[1]);
            *reinterpret_cast<uint2*>(a.out_lo + o) = make_uint2(lo[0], lo[1]);
        }
    }
}

template <int D, int NRT>
void launch_t(const AttnArgs& a, const StepMeta& sm, hipStream_t st) {
    const int z = sm.B * a.Hkv;
    const dim3 grid(a.n_chunks, a.n_rg, z);
    if constexpr (NRT >= 4) {
        // only the wide kernel has that many row tiles per workgroup
        if (a.q_f32) hipLaunchKernelGGL((attn_partial_wide_kernel<D, NRT, true>), grid, dim3(NRT * 64), 0, st, a, sm);
        else hipLaunchKernelGGL((attn_partial_wide_kernel<D, NRT, false>), grid, dim3(NRT * 64), 0, st, a, sm);
    } else {
        const dim3 block(kStreams * NRT * 64);
        if (a.variant == 1) {
            if (a.q_f32) hipLaunchKernelGGL((attn_partial_reg_kernel<D, NRT, true>), grid, dim3(256), 0, st, a, sm);
            else hipLaunchKernelGGL((attn_partial_reg_kernel<D, NRT, false>), grid, dim3(256), 0, st, a, sm);
        } else {
            if (a.q_f32) hipLaunchKernelGGL((attn_partial_kernel<D, NRT, true>), grid, block, 0, st, a, sm);
            else hipLaunchKernelGGL((attn_partial_kernel<D, NRT, false>), grid, block, 0, st, a, sm);
        }
    }
    constexpr int Q4 = NRT * (D / 32) * 4 * 64;
    // one wavefront per workgroup: the partials of a row group come in through as
    // many compute units as possible (each takes in only so many bytes per clock)
    constexpr int mb = 64;
    const dim3 mgrid((Q4 + mb - 1) / mb, z * a.n_rg);
    if (a.n_chunks <= 4) hipLaunchKernelGGL((attn_merge_kernel<D, NRT, 4>), mgrid, dim3(mb), 0, st, a, sm);
    else hipLaunchKernelGGL((attn_merge_kernel<D, NRT, 16>), mgrid, dim3(mb), 0, st, a, sm);
}

}  // namespace

void launch_mask_words(const StepMeta& sm, const uint64_t* anc, int P, int n_tiles, uint32_t* words,
                       hipStream_t st) {
    const long rows = (long)sm.B * sm.R * sm.T;
    const long n = rows * (n_tiles > 1 ? n_tiles : 1);          // at least one thread per row (positions)
    if (n <= 0) return;
    hipLaunchKernelGGL(mask_words_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, sm, anc, P, n_tiles,
                       words, const_cast<int32_t*>(sm.row_pos));
}

void launch_attention(const AttnArgs& a, const StepMeta& sm, hipStream_t st) {
    if (a.D == 128) {
        if (a.nrt == 8) launch_t<128, 8>(a, sm, st);
        else if (a.nrt == 4) launch_t<128, 4>(a, sm, st);
        else if (a.nrt == 2) launch_t<128, 2>(a, sm, st);
        else launch_t<128, 1>(a, sm, st);
    } else {
        if (a.nrt == 8) launch_t<64, 8>(a, sm, st);
        else if (a.nrt == 4) launch_t<64, 4>(a, sm, st);
        else if (a.nrt == 2) launch_t<64, 2>(a, sm, st);
        else launch_t<64, 1>(a, sm, st);
    }
}

}  // namespace fdc
