// Dense projections of the decode step for a handful of rows (M <= 16):
// y[M][N] = x[M][K] * W^T.  The contraction runs on the bf16 matrix cores, but
// with so few rows the kernel is bound by streaming W from HBM exactly once, so
// everything is arranged around that stream:
//   * W is stored pre-tiled (fdc_pack_weight): one 16(n) x 32(k) tile is the
//     1 KiB a wavefront fetches with a single 16-byte-per-lane load, already in
//     the operand order of v_mfma_f32_16x16x32_bf16;
//   * the (tiny) activations stay in registers for the life of a workgroup,
//     as a bf16 head plus a bf16 tail, so rounding x to bf16 costs no accuracy
//     (two matrix instructions per weight tile; the matrix cores idle anyway);
//   * the wavefronts of a workgroup split K, partial tiles meet in LDS;
//   * workgroups are persistent and walk the 16-row output tiles.
#include "kernels_common.hpp"
#include "fdc_launch.hpp"

namespace fdc {

namespace {

constexpr int kMaxWaves = 8;

template <int KTW, int NT, int EPI>
__global__ __launch_bounds__(512) void gemm_skinny_kernel(GemmArgs a, int KT, int S, int kt_split,
                                                          int n_tasks, int nw) {
    __shared__ f32x4 red[2][kMaxWaves][NT][64];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int s = blockIdx.x % S, wg = blockIdx.x / S, wgs = gridDim.x / S;
    const int kb = s * kt_split;
    const int ke = min(KT, kb + kt_split);
    const int len = ke - kb;
    const int w0 = kb + (len * wave) / nw;
    const int nkt = kb + (len * (wave + 1)) / nw - w0;     // k tiles of this wavefront

    // activations of this wavefront's K slice: registers, zero beyond its share
    bf16x8 ah[KTW], al[KTW];
    const bool row_ok = (lane & 15) < a.M;
    const bool has_lo = a.act_lo != nullptr;
#pragma unroll
    for (int i = 0; i < KTW; ++i) {
        bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
        ah[i] = z;
        al[i] = z;
        if (i < nkt && row_ok) {
            const size_t off = ((size_t)(w0 + i) * 64 + lane) * 8;
            ah[i] = *reinterpret_cast<const bf16x8*>(a.act_hi + off);
            if (has_lo) al[i] = *reinterpret_cast<const bf16x8*>(a.act_lo + off);
        }
    }
    const int last = nkt > 0 ? nkt - 1 : 0;

    int buf = 0;
    for (int task = wg; task < n_tasks; task += wgs) {
        f32x4 acc[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
            const size_t tile = (size_t)task * NT + t;
            const uint16_t* wp = a.w + ((tile * KT + w0) * 64 + lane) * 8;
            bf16x8 wv[KTW];
            // tiles past this wavefront's share re-read its last tile (their
            // activations are zero), which keeps the loop free of branches
#pragma unroll
            for (int i = 0; i < KTW; ++i)
                wv[i] = __builtin_nontemporal_load(
                    reinterpret_cast<const bf16x8*>(wp + (size_t)(i < last ? i : last) * 512));
#pragma unroll
            for (int i = 0; i < KTW; ++i) {
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv[i], ah[i], acc[t], 0, 0, 0);
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv[i], al[i], acc[t], 0, 0, 0);
            }
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) red[buf][wave][t][lane] = acc[t];
        __syncthreads();
        // accumulator register i of lane l is y[m = l % 16][n = 16*tile + 4*(l/16) + i]
        if (EPI == EPI_PARTIAL) {
            if (tid < NT * 64) {
                const int t = tid >> 6, l = tid & 63;
                f32x4 sum = red[buf][0][t][l];
                for (int w = 1; w < nw; ++w) sum += red[buf][w][t][l];
                const int m = l & 15;
                const size_t n = ((size_t)task * NT + t) * 16 + 4 * (l >> 4);
                if (m < a.M && n < (size_t)a.n_valid) {
                    *reinterpret_cast<f32x4*>(a.out + ((size_t)s * a.M + m) * a.N + n) = sum;
                }
            }
        } else {  // EPI_SWIGLU: tile 0 = gate rows, tile 1 = up rows of the same 16 features
            if (tid < 64) {
                const int l = tid;
                f32x4 g = red[buf][0][0][l], u = red[buf][0][NT - 1][l];
                for (int w = 1; w < nw; ++w) {
                    g += red[buf][w][0][l];
                    u += red[buf][w][NT - 1][l];
                }
                const int m = l & 15;
                if (m < a.M) {
                    const int k0 = task * 16 + 4 * (l >> 4);     // feature index = k of the consumer
                    uint16_t hi[4], lo[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float h = g[i] / (1.0f + __expf(-g[i])) * u[i];
                        split_bf16(h, hi[i], lo[i]);
                    }
                    const size_t o = act_frag_index(m, k0, a.out_KT);
                    *reinterpret_cast<uint2*>(a.out_hi + o) =
                        make_uint2(hi[0] | (uint32_t)hi[1] << 16, hi[2] | (uint32_t)hi[3] << 16);
                    *reinterpret_cast<uint2*>(a.out_lo + o) =
                        make_uint2(lo[0] | (uint32_t)lo[1] << 16, lo[2] | (uint32_t)lo[3] << 16);
                }
            }
        }
        buf ^= 1;
    }
}

template <int NT, int EPI>
bool launch_ktw(const GemmPlan& p, const GemmArgs& a, hipStream_t st) {
    dim3 grid(p.grid), block(p.nw * 64);
#define FDC_CASE(K)                                                                             \
    case K:                                                                                     \
        hipLaunchKernelGGL((gemm_skinny_kernel<K, NT, EPI>), grid, block, 0, st, a, p.KT, p.S,  \
                           p.kt_split, p.n_tasks, p.nw);                                        \
        break;
    switch (p.ktw) {
        FDC_CASE(2) FDC_CASE(4) FDC_CASE(6) FDC_CASE(8) FDC_CASE(10) FDC_CASE(12) FDC_CASE(14)
        FDC_CASE(16) FDC_CASE(20)
        default: return false;   // no kernel for this bound: nothing was launched
    }
#undef FDC_CASE
    return true;
}

// row-major [n_out][k_in] -> [tile][kt][64 lanes][8]; lane = row%16 + 16*((k%32)/8)
// rows >= n_out of the last tile are stored as zeros
__global__ void pack_weight_kernel(const uint16_t* __restrict__ src, uint16_t* __restrict__ dst,
                                   int64_t n_out, int64_t k_in, int mode) {
    const int64_t KT = k_in / 32, n_tiles = (n_out + 15) / 16;
    const int64_t chunk = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;   // one 16-byte chunk
    if (chunk >= n_tiles * KT * 64) return;
    const int lane = (int)(chunk & 63);
    const int64_t kt = (chunk >> 6) % KT, tile = (chunk >> 6) / KT;
    int64_t src_tile = tile;
    if ((mode & 1) == FDC_PACK_GATE_UP) src_tile = (tile & 1) ? n_tiles / 2 + tile / 2 : tile / 2;
    const int64_t row = src_tile * 16 + (lane & 15), k = kt * 32 + 8 * (lane >> 4);
    uint4 v = make_uint4(0, 0, 0, 0);
    if (row < n_out) v = *reinterpret_cast<const uint4*>(src + row * k_in + k);
    if (mode & FDC_PACK_F16) {
        // bf16 value x 2^8 as fp16: exact for 2^-22 <= |w| < 256 (11 >= 8 significant
        // bits), rounded to nearest below (absolute error under 2^-33), saturated above
        uint32_t* u = reinterpret_cast<uint32_t*>(&v);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float lo = __uint_as_float(u[i] << 16) * 256.0f, hi = __uint_as_float(u[i] & 0xffff0000u) * 256.0f;
            u[i] = f2h(lo) | (uint32_t)f2h(hi) << 16;
        }
    }
    *reinterpret_cast<uint4*>(dst + chunk * 8) = v;
}

__global__ void to_frag_kernel(const float* __restrict__ x, uint16_t* __restrict__ hi,
                               uint16_t* __restrict__ lo, int M, int K) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= M * K) return;
    const int m = idx / K, k = idx % K;
    uint16_t h, l;
    split_bf16(x[idx], h, l);
    const size_t o = act_frag_index(m, k, K / 32);
    hi[o] = h;
    lo[o] = l;
}

__global__ void sum_partials_kernel(const float* __restrict__ part, float* __restrict__ y, int S,
                                    int64_t MN) {
    const int64_t idx = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (idx >= MN) return;
    float s = 0.f;
    for (int i = 0; i < S; ++i) s += part[(int64_t)i * MN + idx];
    y[idx] = s;
}

}  // namespace

bool launch_gemm(const GemmPlan& p, int epilogue, const GemmArgs& a, hipStream_t st) {
    if (epilogue == EPI_SWIGLU) return launch_ktw<2, EPI_SWIGLU>(p, a, st);
    return launch_ktw<1, EPI_PARTIAL>(p, a, st);
}

void launch_pack_weight(const uint16_t* src, uint16_t* dst, int64_t n_out, int64_t k_in, int mode,
                        hipStream_t st) {
    const int64_t chunks = (n_out + 15) / 16 * 16 * k_in / 8;
    hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, st,
                       src, dst, n_out, k_in, mode);
}

void launch_to_frag(const float* x, uint16_t* hi, uint16_t* lo, int M, int K, hipStream_t st) {
    hipLaunchKernelGGL(to_frag_kernel, dim3((M * K + 255) / 256), dim3(256), 0, st, x, hi, lo, M, K);
}

void launch_sum_partials(const float* part, float* y, int S, int M, int64_t N, hipStream_t st) {
    const int64_t MN = (int64_t)M * N;
    hipLaunchKernelGGL(sum_partials_kernel, dim3((unsigned)((MN + 255) / 256)), dim3(256), 0, st,
                       part, y, S, MN);
}

}  // namespace fdc
