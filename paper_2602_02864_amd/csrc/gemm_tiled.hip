// Dense projections of the decode step for many rows (M > 16: several scenes,
// several tokens per branch): y[M][N] = x[M][K] * W^T on the bf16 matrix cores.
// Here the contraction itself is the bound, so the kernel is a tiled GEMM:
//   * both operands already sit in memory in the operand order of
//     v_mfma_f32_16x16x32_bf16 (weights: fdc_pack_weight; activations: the
//     fragments the row kernels write), one 16 x 32 fragment = 1 KiB = one
//     16-byte-per-lane load, so staging them through LDS needs no swizzle and
//     has no bank conflicts;
//   * a workgroup of 2 x 2 wavefronts owns 128 rows x (32 * NTW) features; each
//     wavefront keeps a 64 x (16 * NTW) block of accumulators and feeds it from
//     LDS (4 row fragments as bf16 head + tail, NTW weight fragments per k tile);
//   * the activations keep their bf16 tail: two matrix instructions per weight
//     fragment, fp32-accurate inputs;
//   * K may be split over workgroups (partials summed by the consumer), and
//     the SwiGLU epilogue pairs the interleaved gate / up tiles in registers.
#include "kernels_common.hpp"
#include "fdc_launch.hpp"

namespace fdc {

namespace {

constexpr int kWgMTiles = 8;     // 16-row fragments per workgroup (2 wavefronts x 4)

template <int NTW, int EPI>
__global__ __launch_bounds__(256) void gemm_tiled_kernel(GemmArgs a, TiledPlan p) {
    constexpr int NF = 2 * kWgMTiles + 2 * NTW;        // fragments per k tile: rows (head, tail), weights
    constexpr int NLD = NF / 4;                        // ... fetched per wavefront
    static_assert(NF % 4 == 0, "fragments must divide over four wavefronts");
    __shared__ uint4 lds[2][NF][64];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wm = wave >> 1, wn = wave & 1;

    // workgroups that share a compute die (consecutive ids go round the eight
    // dies) take neighbouring tasks: the same weight columns for every row block
    const int per_die = (gridDim.x + 7) / 8;
    const int task = (blockIdx.x & 7) * per_die + (blockIdx.x >> 3);
    if (task >= p.n_groups * p.m_blocks * p.S) return;
    const int mb = task % p.m_blocks;
    const int ng = (task / p.m_blocks) % p.n_groups;
    const int s = task / (p.m_blocks * p.n_groups);
    const int kt0 = s * p.kt_split;
    const int nkt = min(p.KT, kt0 + p.kt_split) - kt0;

    // the fragments this wavefront fetches each k tile
    const uint16_t* src[NLD];
#pragma unroll
    for (int j = 0; j < NLD; ++j) {
        const int f = wave + 4 * j;
        src[j] = nullptr;
        if (f < 2 * kWgMTiles) {
            const int mt = mb * kWgMTiles + (f >> 1);
            const uint16_t* base = (f & 1) ? a.act_lo : a.act_hi;
            if (mt < p.m_tiles && base) src[j] = base + (((size_t)mt * p.KT + kt0) * 64 + lane) * 8;
        } else {
            const int tile = ng * 2 * NTW + (f - 2 * kWgMTiles);
            if (tile < p.n_tiles) src[j] = a.w + (((size_t)tile * p.KT + kt0) * 64 + lane) * 8;
        }
    }

    f32x4 acc[4][NTW];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < NTW; ++ni) acc[mi][ni] = f32x4{0.f, 0.f, 0.f, 0.f};

    uint4 stage[NLD];
    auto fetch = [&](int i) {
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            stage[j] = make_uint4(0, 0, 0, 0);
            if (src[j]) stage[j] = *reinterpret_cast<const uint4*>(src[j] + (size_t)i * 512);
        }
    };
    auto park = [&](int buf) {
#pragma unroll
        for (int j = 0; j < NLD; ++j) lds[buf][wave + 4 * j][lane] = stage[j];
    };

    if (nkt > 0) {
        fetch(0);
        park(0);
    }
    __syncthreads();
    for (int i = 0; i < nkt; ++i) {
        const int buf = i & 1;
        if (i + 1 < nkt) fetch(i + 1);
        bf16x8 ah[4], al[4];
#pragma unroll
        for (int mi = 0; mi < 4; ++mi) {
            ah[mi] = __builtin_bit_cast(bf16x8, lds[buf][2 * (wm * 4 + mi)][lane]);
            al[mi] = __builtin_bit_cast(bf16x8, lds[buf][2 * (wm * 4 + mi) + 1][lane]);
        }
#pragma unroll
        for (int ni = 0; ni < NTW; ++ni) {
            const bf16x8 wv = __builtin_bit_cast(bf16x8, lds[buf][2 * kWgMTiles + wn * NTW + ni][lane]);
#pragma unroll
            for (int mi = 0; mi < 4; ++mi) {
                acc[mi][ni] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv, ah[mi], acc[mi][ni], 0, 0, 0);
                acc[mi][ni] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv, al[mi], acc[mi][ni], 0, 0, 0);
            }
        }
        if (i + 1 < nkt) park(buf ^ 1);
        __syncthreads();
    }

    // accumulator register i of lane l: y[m = 16*mt + l%16][n = 16*tile + 4*(l/16) + i]
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
        const int m = (mb * kWgMTiles + wm * 4 + mi) * 16 + (lane & 15);
        if (m >= a.M) continue;
        if (EPI == EPI_PARTIAL) {
#pragma unroll
            for (int ni = 0; ni < NTW; ++ni) {
                const int n = (ng * 2 * NTW + wn * NTW + ni) * 16 + 4 * (lane >> 4);
                if (n < a.n_valid)
                    *reinterpret_cast<f32x4*>(a.out + ((size_t)s * a.M + m) * a.N + n) = acc[mi][ni];
            }
        } else {   // tiles alternate: gate rows, up rows of the same 16 features
#pragma unroll
            for (int ni = 0; ni < NTW; ni += 2) {
                const int ftile = (ng * 2 * NTW + wn * NTW + ni) >> 1;
                if (2 * ftile + 1 >= p.n_tiles) continue;
                const f32x4 g = acc[mi][ni], u = acc[mi][ni + 1];
                uint16_t hi[4], lo[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float h = g[e] / (1.0f + __expf(-g[e])) * u[e];
                    split_bf16(h, hi[e], lo[e]);
                }
                const size_t o = act_frag_index(m, ftile * 16 + 4 * (lane >> 4), a.out_KT);
                *reinterpret_cast<uint2*>(a.out_hi + o) =
                    make_uint2(hi[0] | (uint32_t)hi[1] << 16, hi[2] | (uint32_t)hi[3] << 16);
                *reinterpret_cast<uint2*>(a.out_lo + o) =
                    make_uint2(lo[0] | (uint32_t)lo[1] << 16, lo[2] | (uint32_t)lo[3] << 16);
            }
        }
    }
}

template <int NTW>
void launch_ntw(const TiledPlan& p, int epilogue, const GemmArgs& a, hipStream_t st) {
    dim3 grid(p.grid), block(256);
    if (epilogue == EPI_SWIGLU)
        hipLaunchKernelGGL((gemm_tiled_kernel<NTW, EPI_SWIGLU>), grid, block, 0, st, a, p);
    else
        hipLaunchKernelGGL((gemm_tiled_kernel<NTW, EPI_PARTIAL>), grid, block, 0, st, a, p);
}

}  // namespace

void launch_gemm_tiled(const TiledPlan& p, int epilogue, const GemmArgs& a, hipStream_t st) {
    switch (p.ntw) {
        case 4: launch_ntw<4>(p, epilogue, a, st); break;
        case 8: launch_ntw<8>(p, epilogue, a, st); break;
        case 10: launch_ntw<10>(p, epilogue, a, st); break;
        default: break;   // plan_tiled never produces another width
    }
}

}  // namespace fdc
