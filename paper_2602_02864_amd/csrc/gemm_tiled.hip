// Dense projections of the decode step for many rows (M > 16: several scenes,
// several tokens per branch): y[M][N] = x[M][K] * W^T on the bf16 matrix cores.
// Here the contraction itself is the bound, so the kernel is a tiled GEMM:
//   * both operands already sit in memory as 16 x 32 fragments of 1 KiB in
//     matrix-instruction operand order (weights: fdc_pack_weight; activations:
//     the fragments the row kernels write): one 16-byte-per-lane load each, so
//     staging them through LDS needs no swizzle and has no bank conflicts;
//   * a workgroup of 2 x 2 wavefronts owns 128 rows x (32 * NTW) features; each
//     wavefront keeps a 64 x (16 * NTW) block of accumulators and feeds it from
//     LDS (4 row fragments as bf16 head + tail, NTW weight fragments per k tile);
//   * fragments go from memory through registers into a three-stage LDS ring,
//     requested three k tiles ahead; one LDS-only barrier per k tile,
//     across which the global loads stay in flight;
//   * the activations keep their bf16 tail: two matrix instructions per weight
//     fragment, fp32-accurate inputs;
//   * K may be split over workgroups (partials summed by the consumer), and
//     the SwiGLU epilogue pairs the interleaved gate / up tiles in registers;
//   * F16 variants: where the caller has packed a second copy of the weights as
//     fp16 (the bf16 values times 2^8: exact, fdc_pack_weight), the activations come
//     as single fp16 fragments (11 significant bits) instead of a bf16 head + tail:
//     one matrix instruction per weight fragment instead of two and half the row
//     traffic; the epilogue takes the 2^8 out again.  The eight-wavefront F16 kernels
//     bring the weights through LDS too (asynchronous copies straight into a
//     four-stage ring, operands of the next k tile read during the matrix work of
//     this one).
#include "kernels_common.hpp"
#include "fdc_launch.hpp"

namespace fdc {

namespace {

constexpr int kWgMTiles = 8;     // 16-row fragments per workgroup (2 wavefronts x 4)
constexpr int kStages = 3;       // k tiles resident in LDS

// Workgroup barrier that orders LDS traffic only: the global loads of the k
// tile after next stay in flight across it.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

template <bool F16>
__device__ __forceinline__ f32x16 mma32(const uint4& w, const uint4& x, const f32x16& c) {
    if constexpr (F16) return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, w), __builtin_bit_cast(f16x8, x), c, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w), __builtin_bit_cast(bf16x8, x), c, 0, 0, 0);
}
template <bool F16>
__device__ __forceinline__ f32x4 mma16(const f32x4& w, const uint4& x, const f32x4& c) {
    if constexpr (F16) return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, w), __builtin_bit_cast(f16x8, x), c, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w), __builtin_bit_cast(bf16x8, x), c, 0, 0, 0);
}

// silu(gate) * up as the activation fragment element(s) of the next projection
__device__ __forceinline__ void store_h4(const GemmArgs& a, size_t o, const float (&h)[4]) {
    if (a.out_f16) {
        uint16_t v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = f2h(h[e]);
        *reinterpret_cast<uint2*>(a.out_hi + o) = make_uint2(v[0] | (uint32_t)v[1] << 16, v[2] | (uint32_t)v[3] << 16);
    } else {
        uint16_t hi[4], lo[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) split_bf16(h[e], hi[e], lo[e]);
        *reinterpret_cast<uint2*>(a.out_hi + o) = make_uint2(hi[0] | (uint32_t)hi[1] << 16, hi[2] | (uint32_t)hi[3] << 16);
        *reinterpret_cast<uint2*>(a.out_lo + o) = make_uint2(lo[0] | (uint32_t)lo[1] << 16, lo[2] | (uint32_t)lo[3] << 16);
    }
}

template <int NTW, int EPI, bool F16>
__global__ __launch_bounds__(256) void gemm_tiled_kernel(GemmArgs a, TiledPlan p) {
    constexpr int NA = F16 ? kWgMTiles : 2 * kWgMTiles; // row fragments per k tile: heads (, tails)
    constexpr int NF = NA + 2 * NTW;                   // fragments per k tile: rows, weights
    constexpr int NLD = NF / 4;                        // ... fetched per wavefront
    static_assert(NF % 4 == 0, "fragments must divide over four wavefronts");
    __shared__ uint4 lds[kStages][NF][64];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wm = wave >> 1, wn = wave & 1;

    // workgroups that share a compute die (consecutive ids go round the eight
    // dies) take neighbouring tasks: the same weight columns for every row block
    const int per_die = gridDim.x >> 3;
    const int task = (blockIdx.x & 7) * per_die + (blockIdx.x >> 3);
    if (task >= p.n_groups * p.m_blocks * p.S) return;
    const int mb = task % p.m_blocks;
    const int ng = (task / p.m_blocks) % p.n_groups;
    const int s = task / (p.m_blocks * p.n_groups);
    const int kt0 = s * p.kt_split;
    const int nkt = min(p.KT, kt0 + p.kt_split) - kt0;

    // The fragments this wavefront fetches each k tile; in LDS: the bf16 heads of
    // the eight row fragments, their tails, then the weight fragments.  Fragments
    // past the last row or feature tile re-read the last one: what they produce
    // is never stored.
    const uint16_t* src[NLD];
#pragma unroll
    for (int j = 0; j < NLD; ++j) {
        const int f = wave + 4 * j;
        if (f < NA) {
            const int mt = min(mb * kWgMTiles + (f & 7), p.m_tiles - 1);
            src[j] = ((f >> 3) ? a.act_lo : a.act_hi) + (((size_t)mt * p.KT + kt0) * 64 + lane) * 8;
        } else {
            const int tile = min(ng * 2 * NTW + (f - NA), p.n_tiles - 1);
            src[j] = a.w + (((size_t)tile * p.KT + kt0) * 64 + lane) * 8;
        }
    }
    // The contraction uses v_mfma_f32_32x32x16_bf16 (a single wavefront per SIMD
    // keeps the matrix pipe full with it, which it does not with the 16x16x32
    // form).  Its operand for 32 rows and one half of the k tile takes, from two
    // neighbouring 16-row fragments, the 16-byte pieces
    //   fragment (l % 32) / 16, piece l % 16 + 16 * (2 * half + l / 32)
    // so the fragments stay as they are in memory and in LDS; only the LDS read
    // address of a lane differs (16 consecutive lanes still read 256 contiguous
    // bytes: no bank conflicts).
    const int pair_off = ((lane & 31) >> 4) * 64 + (lane & 15) + 16 * (lane >> 5);   // in 16-byte units
    constexpr int NB = NTW / 2;                         // 32-feature blocks per wavefront
    f32x16 acc[2][NB];
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[q][nb][e] = 0.f;

    // k tile i: memory -> registers -> ring stage.  Past the last tile the last
    // one is fetched and parked again (into a stage nobody reads any more), so
    // that every iteration is the same straight-line code.
    f32x4 g0[NLD], g1[NLD], g2[NLD];
#define FDC_FETCH(g, i)                                                                    \
    _Pragma("unroll") for (int j = 0; j < NLD; ++j)                                        \
        g[j] = *reinterpret_cast<const f32x4*>(src[j] + (size_t)min((i), nkt - 1) * 512)
#define FDC_PARK(g, stg)                                                                   \
    _Pragma("unroll") for (int j = 0; j < NLD; ++j)                                        \
        *reinterpret_cast<f32x4*>(&lds[stg][wave + 4 * j][lane]) = g[j]
    // the matrix work of one k tile out of ring stage `stg`
#define FDC_MMA(stg)                                                                                  \
    {                                                                                                 \
        const uint4* st = &lds[stg][0][0] + pair_off;                                                 \
        uint4 ah[2][2], al[2][2]; /* [32-row block][k half] */                                        \
        _Pragma("unroll") for (int q = 0; q < 2; ++q)                                                 \
        _Pragma("unroll") for (int h = 0; h < 2; ++h) {                                               \
            ah[q][h] = st[(4 * wm + 2 * q) * 64 + 32 * h];                                            \
            if (!F16) al[q][h] = st[(8 + 4 * wm + 2 * q) * 64 + 32 * h];                              \
        }                                                                                             \
        _Pragma("unroll") for (int nb = 0; nb < NB; ++nb) {                                           \
            uint4 wv[2];                                                                              \
            _Pragma("unroll") for (int h = 0; h < 2; ++h)                                             \
                wv[h] = st[(NA + wn * NTW + 2 * nb) * 64 + 32 * h];                                   \
            _Pragma("unroll") for (int h = 0; h < 2; ++h)                                             \
            _Pragma("unroll") for (int q = 0; q < 2; ++q)                                             \
                acc[q][nb] = mma32<F16>(wv[h], ah[q][h], acc[q][nb]);                                 \
            if (!F16) {                                                                               \
                _Pragma("unroll") for (int h = 0; h < 2; ++h)                                         \
                _Pragma("unroll") for (int q = 0; q < 2; ++q)                                         \
                    acc[q][nb] = mma32<F16>(wv[h], al[q][h], acc[q][nb]);                             \
            }                                                                                         \
        }                                                                                             \
    }
    // One iteration.  Tile i+2 (requested three iterations ago into `g`) goes
    // into the ring stage tile i-1 occupied, tile i+5 is requested into `g`,
    // and the matrix cores work on k tile i (stage i % 3); the LDS writes and the
    // global loads run under the matrix instructions.  One LDS-only barrier.
#define FDC_ITER(g, i)                                                                     \
    {                                                                                      \
        const int into = stg == 0 ? 2 : stg - 1; /* (i + 2) % 3 */                         \
        FDC_PARK(g, into);                                                                 \
        FDC_FETCH(g, (i) + 5);                                                             \
        FDC_MMA(stg);                                                                      \
        lds_barrier();                                                                     \
        stg = stg == 2 ? 0 : stg + 1;                                                      \
    }
    if (nkt > 0) {
        FDC_FETCH(g0, 0);
        FDC_FETCH(g1, 1);
        FDC_FETCH(g2, 2);
        FDC_PARK(g0, 0);
        FDC_FETCH(g0, 3);
        FDC_PARK(g1, 1);
        FDC_FETCH(g1, 4);
        lds_barrier();
        int stg = 0, i = 0;
        for (; i + 2 < nkt; i += 3) {          // tile t travels in set t % 3
            FDC_ITER(g2, i);
            FDC_ITER(g0, i + 1);
            FDC_ITER(g1, i + 2);
        }
        if (i < nkt) {
            FDC_ITER(g2, i);
            ++i;
        }
        if (i < nkt) FDC_MMA(stg);
    }
#undef FDC_ITER
#undef FDC_MMA
#undef FDC_FETCH
#undef FDC_PARK

    // accumulator register e of lane l in block (q, nb):
    //   y[m = 32 * (row block) + l % 32][n = 32 * (feature block) + 8 * (e / 4) + 4 * (l / 32) + e % 4]
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int m = (mb * kWgMTiles + wm * 4 + 2 * q) * 16 + (lane & 31);
        if (m >= a.M) continue;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int tile0 = ng * 2 * NTW + wn * NTW + 2 * nb;      // first of the block's two 16-feature tiles
            if (EPI == EPI_PARTIAL) {
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4) {
                    const int n = tile0 * 16 + 8 * e4 + 4 * (lane >> 5);
                    if (n < a.n_valid) {
                        f32x4 v = {acc[q][nb][4 * e4], acc[q][nb][4 * e4 + 1], acc[q][nb][4 * e4 + 2],
                                   acc[q][nb][4 * e4 + 3]};
                        if (F16) v *= a.out_scale;
                        *reinterpret_cast<f32x4*>(a.out + ((size_t)s * a.M + m) * a.N + n) = v;
                    }
                }
            } else {   // the block's first tile holds the gate rows, its second the up rows of 16 features
                if (tile0 + 1 >= p.n_tiles) continue;
                const int ftile = tile0 >> 1;
#pragma unroll
                for (int e4 = 0; e4 < 2; ++e4) {
                    float h[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float gt = acc[q][nb][4 * e4 + e], up = acc[q][nb][8 + 4 * e4 + e];
                        if (F16) {
                            gt *= a.out_scale;
                            up *= a.out_scale;
                        }
                        h[e] = gt / (1.0f + __expf(-gt)) * up;
                    }
                    store_h4(a, act_frag_index(m, ftile * 16 + 8 * e4 + 4 * (lane >> 5), a.out_KT), h);
                }
            }
        }
    }
}

// Eight wavefronts, two per SIMD, for the wide tiles.  How fast a compute unit
// takes data in from L2 is set by the number of wavefronts that issue loads
// (about 5 bytes per clock each), and four of them cannot feed the matrix pipe;
// with two wavefronts per SIMD the 16x16x32 instruction keeps the pipe full too
// (measured: 90-98 % of peak, against 55-62 % with one).  The workgroup still
// owns 128 rows x (32 * NTW) features; the wavefronts form a WM x (8 / WM) grid
// (2 x 4 as launched: 64 rows x 5 feature tiles each at NTW = 10).  Row
// fragments (bf16 head + tail) go through the three-stage LDS ring as above, two
// fetched per wavefront and k tile; the weight fragments go straight from memory
// into matrix-instruction operands (the wavefronts with the same feature tiles
// ask for the same lines at the same time and the L1 serves them), and the
// registers of a weight fragment are refilled, right after its last use, with
// the fragment four k tiles ahead.  A wavefront fits 256 registers.  With an odd
// number of feature tiles per wavefront a gate tile and its up tile can end up
// in neighbouring wavefronts: the SwiGLU epilogue passes that one tile through
// LDS.  (A 4 x 2 grid needs no such exchange but asks the L1 for every weight
// line four times and measured slower than the four-wavefront kernel.)
// waits until at most n LDS reads of this wavefront are outstanding (n is a constant
// after unrolling)
__device__ __forceinline__ void wait_lds_reads(int n) {
    switch (n) {
        case 0: asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); break;
        case 1: asm volatile("s_waitcnt lgkmcnt(1)" ::: "memory"); break;
        case 2: asm volatile("s_waitcnt lgkmcnt(2)" ::: "memory"); break;
        case 3: asm volatile("s_waitcnt lgkmcnt(3)" ::: "memory"); break;
        case 4: asm volatile("s_waitcnt lgkmcnt(4)" ::: "memory"); break;
        case 5: asm volatile("s_waitcnt lgkmcnt(5)" ::: "memory"); break;
        default: asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); break;
    }
}

typedef __attribute__((address_space(3))) void lds_void_t;
typedef const __attribute__((address_space(1))) void glb_void_t;

// LW: the weight fragments go through the LDS ring as well (asynchronous copies
// straight into LDS, four stages), so that each is fetched once per workgroup and
// not once by each of the WM wavefronts that use it.
template <int NTW, int EPI, int WM, bool F16, bool LW = false>
__global__ __launch_bounds__(512) void gemm_tiled8_kernel(GemmArgs a, TiledPlan p) {
    constexpr int NFA = F16 ? kWgMTiles : 2 * kWgMTiles;   // row fragments per k tile: heads (, tails)
    constexpr int NSRC = F16 ? 1 : 2;
    constexpr int WN = 8 / WM;                         // wavefronts along the features
    constexpr int MF = kWgMTiles / WM;                 // 16-row fragments per wavefront
    constexpr int TW = 2 * NTW / WN;                   // 16-feature tiles per wavefront
    static_assert(2 * NTW % WN == 0, "feature tiles must divide over the wavefronts");
    constexpr int NPC = NFA + 2 * NTW;                 // LW: 1 KiB pieces per k tile (rows, then weights)
    constexpr int kRing = LW ? 4 : kStages;
    __shared__ uint4 lds[kRing][LW ? NPC : NFA][64];

    // the wavefront's index as a scalar: what follows from it (tile numbers, base
    // addresses) then lives in scalar registers, and the loads take a scalar base
    // plus the lane's 16-byte offset
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int wm = wave / WN, wn = wave % WN;

    const int per_die = gridDim.x >> 3;
    const int task = (blockIdx.x & 7) * per_die + (blockIdx.x >> 3);
    if (task >= p.n_groups * p.m_blocks * p.S) return;
    const int mb = task % p.m_blocks;
    const int ng = (task / p.m_blocks) % p.n_groups;
    const int s = task / (p.m_blocks * p.n_groups);
    const int kt0 = s * p.kt_split;
    const int nkt = min(p.KT, kt0 + p.kt_split) - kt0;

    // the two row fragments this wavefront stages each k tile: fragment `wave`
    // as head and as tail
    const uint16_t* src[2];
    {
        const int mt = min(mb * kWgMTiles + wave, p.m_tiles - 1);
        const size_t off = ((size_t)mt * p.KT + kt0) * 512;
        src[0] = a.act_hi + off;
        src[1] = F16 ? src[0] : a.act_lo + off;
    }
    // its weight fragments; past the last feature tile the last one is re-read
    // (what it produces is never stored)
    const int tile_first = ng * 2 * NTW + wn * TW;
    const uint16_t* wsrc[TW];
#pragma unroll
    for (int t = 0; t < TW; ++t) {
        const int tile = min(tile_first + t, p.n_tiles - 1);
        wsrc[t] = a.w + ((size_t)tile * p.KT + kt0) * 512;
    }

    f32x4 acc[MF][TW];
#pragma unroll
    for (int mf = 0; mf < MF; ++mf)
#pragma unroll
        for (int t = 0; t < TW; ++t) acc[mf][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    // weight fragments of k tile t travel in register set t % NBS: four sets where a
    // wavefront has few tiles (the refill then runs four k tiles ahead), two otherwise
    constexpr int NBS = TW <= 5 ? 4 : 2;
    f32x4 g0[2], g1[2];
    f32x4 b0[TW], b1[TW], b2[NBS == 4 ? TW : 1], b3[NBS == 4 ? TW : 1];
#define FDC_FETCH(g, i)                                                                    \
    _Pragma("unroll") for (int j = 0; j < NSRC; ++j)                                       \
        g[j] = *reinterpret_cast<const f32x4*>(src[j] + (size_t)min((i), nkt - 1) * 512 + lane * 8)
#define FDC_FETCHW1(b, t, i)                                                               \
    b[t] = *reinterpret_cast<const f32x4*>(wsrc[t] + (size_t)min((i), nkt - 1) * 512 + lane * 8)
#define FDC_PARK(g, stg)                                                                   \
    _Pragma("unroll") for (int j = 0; j < NSRC; ++j)                                       \
        *reinterpret_cast<f32x4*>(&lds[stg][wave + 8 * j][lane]) = g[j]
    // k tile i: rows out of ring stage i % 3, weights out of `b`.  `g` holds the
    // rows of tile i+2 (requested two iterations ago): they go into the stage
    // tile i-1 occupied, and the rows of tile i+4 are requested into `g`.
    // (Reading the row operands of the next tile half way through an iteration, so
    // that none starts with a wait for LDS, measured 4 % slower.)
    uint4 ah[MF], al[MF];
#define FDC_ROWS(dh, dl, stg_)                                                             \
    _Pragma("unroll") for (int mf = 0; mf < MF; ++mf) {                                    \
        dh[mf] = lds[stg_][MF * wm + mf][lane];                                            \
        if (!F16) dl[mf] = lds[stg_][(NFA / 2) + MF * wm + mf][lane];                      \
    }
#define FDC_ITER(g, b, i)                                                                  \
    {                                                                                      \
        const int into = stg == 0 ? 2 : stg - 1; /* (i + 2) % 3 */                         \
        FDC_PARK(g, into);                                                                 \
        FDC_FETCH(g, (i) + 4);                                                             \
        FDC_ROWS(ah, al, stg);                                                             \
        _Pragma("unroll") for (int t = 0; t < TW; ++t) {                                   \
            _Pragma("unroll") for (int mf = 0; mf < MF; ++mf) {                            \
                acc[mf][t] = mma16<F16>(b[t], ah[mf], acc[mf][t]);                         \
                if (!F16) acc[mf][t] = mma16<F16>(b[t], al[mf], acc[mf][t]);               \
            }                                                                              \
            FDC_FETCHW1(b, t, (i) + NBS);                                                  \
        }                                                                                  \
        lds_barrier();                                                                     \
        stg = stg == 2 ? 0 : stg + 1;                                                      \
    }
    if constexpr (LW) {
        // piece q of a k tile: q < NFA a row fragment (heads, then tails), else weight
        // tile q - NFA of the group; wavefront w copies pieces w, w + 8, ...
        constexpr int NPJ = (NPC + 7) / 8;
        const uint16_t* psrc[NPJ];
#pragma unroll
        for (int j = 0; j < NPJ; ++j) {
            const int q = wave + 8 * j;
            if (q < NFA) {
                const int mt = min(mb * kWgMTiles + (q % kWgMTiles), p.m_tiles - 1);
                psrc[j] = ((q >= kWgMTiles) ? a.act_lo : a.act_hi) + ((size_t)mt * p.KT + kt0) * 512;
            } else {
                const int tile = min(ng * 2 * NTW + (q - NFA), p.n_tiles - 1);
                psrc[j] = a.w + ((size_t)tile * p.KT + kt0) * 512;
            }
        }
        const bool full = wave + 8 * (NPJ - 1) < NPC;      // this wavefront copies NPJ pieces, else NPJ - 1
        auto issue = [&](int i, int stg) {
            if (i >= nkt) return;
#pragma unroll
            for (int j = 0; j < NPJ; ++j) {
                const int q = wave + 8 * j;
                if (q < NPC)
                    __builtin_amdgcn_global_load_lds((glb_void_t*)(psrc[j] + (size_t)i * 512 + lane * 8),
                                                     (lds_void_t*)&lds[stg][q][0], 16, 0, 0);
            }
        };
        const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_void_t*)&lds[0][0][0] + lane * 16;
        auto rd = [&](f32x4& d, uint32_t off) { asm volatile("ds_read_b128 %0, %1" : "=v"(d) : "v"(off)); };
        // Operands of k tile i are read from LDS during the matrix work of tile i - 1
        // (two register sets), so that no tile starts with a wait for LDS.
        f32x4 rh[2][MF], rl[2][F16 ? 1 : MF], wb[2][TW];
        auto fetch_ops = [&](int set, int stg) {
            const uint32_t base = lds0 + stg * (NPC * 1024);
#pragma unroll
            for (int mf = 0; mf < MF; ++mf) rd(rh[set][mf], base + (MF * wm + mf) * 1024);
            if (!F16) {
#pragma unroll
                for (int mf = 0; mf < MF; ++mf) rd(rl[set][mf], base + (NFA / 2 + MF * wm + mf) * 1024);
            }
#pragma unroll
            for (int t = 0; t < TW; ++t) rd(wb[set][t], base + (NFA + wn * TW + t) * 1024);
        };
        auto wait_mine = [&](int ahead) {            // my copies: all but those of the `ahead` youngest tiles have landed
            if (full) {
                if (ahead >= 3) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(3 * NPJ) : "memory");
                else if (ahead == 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * NPJ) : "memory");
                else if (ahead == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NPJ) : "memory");
                else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            } else {
                if (ahead >= 3) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(3 * (NPJ - 1)) : "memory");
                else if (ahead == 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * (NPJ - 1)) : "memory");
                else if (ahead == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NPJ - 1) : "memory");
                else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            }
        };
        auto mma_tile = [&](int set) {
#pragma unroll
            for (int mf = 0; mf < MF; ++mf) {
                asm volatile("" : "+v"(rh[set][mf]));
                if (!F16) asm volatile("" : "+v"(rl[set][mf]));
            }
#pragma unroll
            for (int t = 0; t < TW; ++t) {
                asm volatile("" : "+v"(wb[set][t]));
#pragma unroll
                for (int mf = 0; mf < MF; ++mf) {
                    acc[mf][t] = mma16<F16>(wb[set][t], __builtin_bit_cast(uint4, rh[set][mf]), acc[mf][t]);
                    if (!F16) acc[mf][t] = mma16<F16>(wb[set][t], __builtin_bit_cast(uint4, rl[set][mf]), acc[mf][t]);
                }
            }
        };
        if (nkt > 0) {
            issue(0, 0);
            issue(1, 1);
            issue(2, 2);
            issue(3, 3);
            // tile 0 into the first operand set
            wait_mine(min(nkt - 1, 3));
            asm volatile("s_barrier" ::: "memory");
            fetch_ops(0, 0);
            // iteration i: tile i's operands are (being) read into set i % 2; tiles i + 1 .. i + 3 in flight
            auto iter = [&](int i, int set) {
                // tile i's operands are in registers (for every wavefront once it passes the barrier)
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                if (i + 1 < nkt) {
                    wait_mine(min(nkt - 2 - i, 2));              // my copies of tile i + 1 have landed
                    asm volatile("s_barrier" ::: "memory");     // everyone's have; stage i % 4 is free
                    issue(i + 4, i & 3);
                    fetch_ops(set ^ 1, (i + 1) & 3);
                }
                mma_tile(set);
            };
            int i = 0;
            for (; i + 1 < nkt; i += 2) {
                iter(i, 0);
                iter(i + 1, 1);
            }
            if (i < nkt) iter(i, 0);
            asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        }
        asm volatile("s_barrier" ::: "memory");          // the ring is free (the epilogue may use it)
    } else if (nkt > 0) {
        FDC_FETCH(g0, 0);
        FDC_FETCH(g1, 1);
        _Pragma("unroll") for (int t = 0; t < TW; ++t) FDC_FETCHW1(b0, t, 0);
        _Pragma("unroll") for (int t = 0; t < TW; ++t) FDC_FETCHW1(b1, t, 1);
        if (NBS == 4) {
            _Pragma("unroll") for (int t = 0; t < TW; ++t) FDC_FETCHW1(b2, t, 2);
            _Pragma("unroll") for (int t = 0; t < TW; ++t) FDC_FETCHW1(b3, t, 3);
        }
        FDC_PARK(g0, 0);
        FDC_FETCH(g0, 2);
        FDC_PARK(g1, 1);
        FDC_FETCH(g1, 3);
        lds_barrier();
        int stg = 0, i = 0;
        if (NBS == 4) {
            for (; i + 3 < nkt; i += 4) {
                FDC_ITER(g0, b0, i);
                FDC_ITER(g1, b1, i + 1);
                FDC_ITER(g0, b2, i + 2);
                FDC_ITER(g1, b3, i + 3);
            }
            if (i < nkt) FDC_ITER(g0, b0, i);
            if (i + 1 < nkt) FDC_ITER(g1, b1, i + 1);
            if (i + 2 < nkt) FDC_ITER(g0, b2, i + 2);
        } else {
            for (; i + 1 < nkt; i += 2) {
                FDC_ITER(g0, b0, i);
                FDC_ITER(g1, b1, i + 1);
            }
            if (i < nkt) FDC_ITER(g0, b0, i);
        }
    }
#undef FDC_ITER
#undef FDC_ROWS
#undef FDC_FETCH
#undef FDC_FETCHW1
#undef FDC_PARK

    // accumulator register e of lane l in block (mf, t):
    //   y[m = 16 * (row fragment) + l % 16][n = 16 * tile + 4 * (l / 16) + e]
    if (EPI == EPI_PARTIAL) {
#pragma unroll
        for (int mf = 0; mf < MF; ++mf) {
            const int m = (mb * kWgMTiles + MF * wm + mf) * 16 + (lane & 15);
            if (m >= a.M) continue;
#pragma unroll
            for (int t = 0; t < TW; ++t) {
                const int n = (tile_first + t) * 16 + 4 * (lane >> 4);
                if (n < a.n_valid)
                    *reinterpret_cast<f32x4*>(a.out + ((size_t)s * a.M + m) * a.N + n) =
                        F16 ? acc[mf][t] * a.out_scale : acc[mf][t];
            }
        }
    } else {
        // Tile 2u holds the gate rows, tile 2u + 1 the up rows of 16 features.  With an
        // odd number of tiles per wavefront the pair at the seam is split: the
        // wavefront with the odd index hands its first tile (an up tile) to its left
        // neighbour through LDS (the ring is free by now).
        constexpr bool SEAM = (TW % 2) != 0;
        f32x4 seam_up[MF];
        if (SEAM) {
            f32x4* xb = reinterpret_cast<f32x4*>(&lds[0][0][0]);      // [wm][wn / 2][mf][lane]
            if (wn & 1) {
#pragma unroll
                for (int mf = 0; mf < MF; ++mf) xb[((wm * (WN / 2) + (wn >> 1)) * MF + mf) * 64 + lane] = acc[mf][0];
            }
            __syncthreads();
            if (!(wn & 1)) {
#pragma unroll
                for (int mf = 0; mf < MF; ++mf) seam_up[mf] = xb[((wm * (WN / 2) + (wn >> 1)) * MF + mf) * 64 + lane];
            }
        }
        auto emit = [&](int m, int tile0, const f32x4& gate, const f32x4& upv) {
            if (tile0 + 1 >= p.n_tiles) return;
            float h[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float gt = F16 ? gate[e] * a.out_scale : gate[e], up = F16 ? upv[e] * a.out_scale : upv[e];
                h[e] = gt / (1.0f + __expf(-gt)) * up;
            }
            store_h4(a, act_frag_index(m, (tile0 >> 1) * 16 + 4 * (lane >> 4), a.out_KT), h);
        };
        // pairs of a wavefront with an even index: (0,1), (2,3), ... and, at a seam,
        // (TW-1, the neighbour's 0); with an odd index at a seam: (1,2), (3,4), ...
        // (two static copies, so that the accumulators keep static indices)
#pragma unroll
        for (int mf = 0; mf < MF; ++mf) {
            const int m = (mb * kWgMTiles + MF * wm + mf) * 16 + (lane & 15);
            if (m >= a.M) continue;
            if (!SEAM || !(wn & 1)) {
#pragma unroll
                for (int tg = 0; tg + 1 < TW; tg += 2) emit(m, tile_first + tg, acc[mf][tg], acc[mf][tg + 1]);
                if (SEAM) emit(m, tile_first + TW - 1, acc[mf][TW - 1], seam_up[mf]);
            } else {
#pragma unroll
                for (int tg = 1; tg + 1 < TW; tg += 2) emit(m, tile_first + tg, acc[mf][tg], acc[mf][tg + 1]);
            }
        }
    }
}

// The narrow tile (ntw 4: QKV, O, down at a few hundred rows) measures faster with
// four wavefronts and 32x32x16 instructions; the wide ones (gate/up, LM head) with
// eight wavefronts (9-10 %).
template <int NTW, bool F16>
void launch_ntw(const TiledPlan& p, int epilogue, const GemmArgs& a, hipStream_t st) {
    const dim3 grid(p.grid);
    if (NTW >= 8) {
        // Single-pass fp16 kernels take the weights through LDS (measured: LM head 88 ->
        // 72 us, gate/up 97 -> 84 us at 256 rows): they are bound by what a compute unit
        // can fetch, and each weight fragment is then fetched once per workgroup.  The
        // two-pass kernels read twice as many row fragments from LDS per k tile and
        // measured 3 % slower that way, so they keep the weights in registers.
        if (epilogue == EPI_SWIGLU)
            hipLaunchKernelGGL((gemm_tiled8_kernel<NTW, EPI_SWIGLU, 2, F16, F16>), grid, dim3(512), 0, st, a, p);
        else
            hipLaunchKernelGGL((gemm_tiled8_kernel<NTW, EPI_PARTIAL, 2, F16, F16>), grid, dim3(512), 0, st, a, p);
    } else {
        if (epilogue == EPI_SWIGLU)
            hipLaunchKernelGGL((gemm_tiled_kernel<NTW, EPI_SWIGLU, F16>), grid, dim3(256), 0, st, a, p);
        else
            hipLaunchKernelGGL((gemm_tiled_kernel<NTW, EPI_PARTIAL, F16>), grid, dim3(256), 0, st, a, p);
    }
}

}  // namespace

bool launch_gemm_tiled(const TiledPlan& p, int epilogue, const GemmArgs& a, hipStream_t st) {
    switch (p.ntw * 2 + (a.f16 ? 1 : 0)) {
        case 8: launch_ntw<4, false>(p, epilogue, a, st); break;
        case 9: launch_ntw<4, true>(p, epilogue, a, st); break;
        case 16: launch_ntw<8, false>(p, epilogue, a, st); break;
        case 17: launch_ntw<8, true>(p, epilogue, a, st); break;
        case 20: launch_ntw<10, false>(p, epilogue, a, st); break;
        case 21: launch_ntw<10, true>(p, epilogue, a, st); break;
        default: return false;   // no kernel for this width: nothing was launched
    }
    return true;
}

}  // namespace fdc
