// Per-row kernels of the decode step: residual add + RMSNorm (also the
// embedding gather), rotary embedding + KV append at the row's fixed position
// id, bulk KV scatter, and per-row greedy argmax.  All are bandwidth-trivial;
// each consumes the split-K partials of the projection before it so that no
// separate reduction pass exists.
#include "kernels_common.hpp"
#include "fdc_launch.hpp"

namespace fdc {

namespace {

__device__ __forceinline__ float block_sum(float v, float* sh) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    const int wave = threadIdx.x >> 6, nwv = blockDim.x >> 6;
    if ((threadIdx.x & 63) == 0) sh[wave] = v;
    __syncthreads();
    float t = 0.f;
    for (int w = 0; w < nwv; ++w) t += sh[w];
    __syncthreads();
    return t;
}

// One workgroup per row.  x <- (embedding | x + sum of partials); a <- rmsnorm(x) * gain.
// Every thread owns VEC groups of four consecutive columns (one at d_model <=
// 4096: NT = 1024 threads) and issues the loads of up to eight split-K
// partials before it adds any of them (in split order): the kernel is one or two
// round trips to memory, one block reduction and one round of stores.
template <int NT, int VEC>
__global__ __launch_bounds__(NT) void resid_norm_kernel(NormArgs a, StepMeta sm) {
    __shared__ float sh[NT / 64];
    const int m = blockIdx.x;
    // whether the row is active is looked at only after its data has been
    // requested: rows of inactive branches exist in every buffer, are read for
    // nothing and come out as zeros
    const int field = sm.branch_field ? sm.branch_field[m / sm.T] : 0;
    const int nvec = a.d >> 2;
    f32x4 v[VEC];
    const float* __restrict__ xin = a.x + (size_t)m * a.d;
    const float* __restrict__ part = a.part;
    const uint16_t* __restrict__ erow = nullptr;
    if (a.tok) {
        int t = a.tok[m];
        t = t < 0 ? 0 : (t >= a.vocab ? a.vocab - 1 : t);
        erow = a.emb + (size_t)t * a.d;
    } else if (a.emb_rows) {
        erow = a.emb_rows + (size_t)m * a.d;
    }
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        const int q = threadIdx.x + i * NT;
        v[i] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (q < nvec) {
            if (erow) {
                const uint2 e = *reinterpret_cast<const uint2*>(erow + 4 * q);
                v[i] = f32x4{__uint_as_float(e.x << 16), __uint_as_float(e.x & 0xffff0000u),
                             __uint_as_float(e.y << 16), __uint_as_float(e.y & 0xffff0000u)};
            } else {
                v[i] = *reinterpret_cast<const f32x4*>(xin + 4 * q);
            }
        }
    }
    if (!erow) {
        // eight partials in flight per thread: the row's partials arrive at the rate
        // one compute unit can take them in, more in flight does not help
        constexpr int PB = 8;
        for (int s0 = 0; s0 < a.S; s0 += PB) {
            f32x4 p[PB][VEC];
#pragma unroll
            for (int j = 0; j < PB; ++j) {
                const int s = min(s0 + j, a.S - 1);            // past the end: a repeat, not added
#pragma unroll
                for (int i = 0; i < VEC; ++i) {
                    const int q = threadIdx.x + i * NT;
                    p[j][i] = f32x4{0.f, 0.f, 0.f, 0.f};
                    if (q < nvec) p[j][i] = *reinterpret_cast<const f32x4*>(part + ((size_t)s * a.M + m) * a.d + 4 * q);
                }
            }
#pragma unroll
            for (int j = 0; j < PB; ++j)
                if (s0 + j < a.S)
#pragma unroll
                    for (int i = 0; i < VEC; ++i) v[i] += p[j][i];
        }
    }
    // the gains are requested before the reduction, not after it
    f32x4 gain[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        const int q = threadIdx.x + i * NT;
        gain[i] = q < nvec ? *reinterpret_cast<const f32x4*>(a.gain + 4 * q) : f32x4{0.f, 0.f, 0.f, 0.f};
    }
    if (field < 0)
#pragma unroll
        for (int i = 0; i < VEC; ++i) v[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < VEC; ++i) ss += v[i][0] * v[i][0] + v[i][1] * v[i][1] + v[i][2] * v[i][2] + v[i][3] * v[i][3];
    const float tot = block_sum(ss, sh);
    const float rstd = rsqrtf(tot / (float)a.d + a.eps);
    const int KT = a.d >> 5;
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        const int q = threadIdx.x + i * NT;
        if (q >= nvec) continue;
        const int k = 4 * q;
        *reinterpret_cast<f32x4*>(a.x + (size_t)m * a.d + k) = v[i];
        if (a.hidden_x) *reinterpret_cast<f32x4*>(a.hidden_x + (size_t)m * a.d + k) = v[i];
        const f32x4 n = v[i] * rstd * gain[i];
        const size_t o = act_frag_index(m, k, KT);           // 4 consecutive k share a fragment lane
        if (a.f16) {                                         // one fp16 fragment for the fp16 tiled projections
            uint16_t h[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) h[j] = f2h(n[j]);
            *reinterpret_cast<uint2*>(a.a_hi + o) =
                make_uint2(h[0] | (uint32_t)h[1] << 16, h[2] | (uint32_t)h[3] << 16);
        } else {
            uint16_t hi[4], lo[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) split_bf16(n[j], hi[j], lo[j]);
            *reinterpret_cast<uint2*>(a.a_hi + o) =
                make_uint2(hi[0] | (uint32_t)hi[1] << 16, hi[2] | (uint32_t)hi[3] << 16);
            *reinterpret_cast<uint2*>(a.a_lo + o) =
                make_uint2(lo[0] | (uint32_t)lo[1] << 16, lo[2] | (uint32_t)lo[3] << 16);
        }
        if (a.hidden_n) *reinterpret_cast<f32x4*>(a.hidden_n + (size_t)m * a.d + k) = n;
    }
}

template <int D>
__device__ __forceinline__ void cache_store(uint16_t* kc, uint16_t* vc, int scene, int kvh, int Hkv,
                                            int NB, int pos, int d, bool is_k, uint16_t val) {
    const size_t tile = ((size_t)scene * Hkv + kvh) * NB + (pos >> 5);
    if (is_k) kc[tile * (32 * D) + k_tile_index<D>(pos & 31, d)] = val;
    else vc[tile * (32 * D) + v_tile_index<D>(pos & 31, d)] = val;
}

// cos / sin of pos * base^(-2i/D) for every cache position, computed once in
// double precision (the positions are fixed by the template, Sec. 3.3)
__global__ void rope_table_kernel(const double* __restrict__ inv_freq, float2* __restrict__ tab,
                                  int n_pos, int half) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n_pos * half) return;
    double sn, cs;
    sincos((double)(idx / half) * inv_freq[idx % half], &sn, &cs);
    tab[idx] = make_float2((float)cs, (float)sn);
}

// Workgroups of 256 threads, several per row: sum the QKV partials, rotate q and
// k by the row's position id (slot_start[field] + offset: fixed by the template,
// Sec. 3.3; taken from the step's position table), store q (fp32) and append
// k, v (bf16) to the cache at index = position id.  A thread handles one rotation pair (or two V elements); its loads
// are independent of each other.
template <int D>
__global__ __launch_bounds__(256) void rope_append_kernel(RopeArgs a, StepMeta sm) {
    const int m = blockIdx.y;
    const int pos = sm.row_pos[m];              // slot_start[field] + offset + t, or -1: one look-up
    const int Nqkv = (a.Hq + 2 * a.Hkv) * D;
    constexpr int half = D / 2;
    const int n_pairs = (a.Hq + a.Hkv) * half;
    const int n_v2 = a.Hkv * D / 2;
    const int item = blockIdx.x * 256 + threadIdx.x;
    if (item >= n_pairs + n_v2) return;
    const bool rot = item < n_pairs;
    // The two elements this thread owns: a rotary pair (i, i + D/2) of a Q or K
    // head, or two neighbouring V elements.  Their split-K partials do not
    // depend on the branch tables, so they are requested before the (dependent)
    // look-ups of field, slot start and rotation, and inactive rows read theirs
    // for nothing (the rows exist in the workspace).
    const int hd = item / half, i = item % half;
    const int e = 2 * (item - n_pairs);
    const int c1 = rot ? hd * D + i : (a.Hq + a.Hkv) * D + e;
    const int c2 = rot ? c1 + half : c1 + 1;
    const float* __restrict__ part = a.part + (size_t)m * Nqkv;
    const size_t sstride = (size_t)a.M * Nqkv;
    float x1 = 0.f, x2 = 0.f;
#pragma unroll 4
    for (int s = 0; s < a.S; ++s) {
        x1 += part[s * sstride + c1];
        x2 += part[s * sstride + c2];
    }
    if (pos < 0) return;
    const int scene = m / (sm.R * sm.T);
    if (rot) {
        const float2 cssn = a.tab[(size_t)pos * half + i];
        const float y1 = x1 * cssn.x - x2 * cssn.y, y2 = x2 * cssn.x + x1 * cssn.y;
        if (hd < a.Hq) {
            float* q = a.q + ((size_t)m * a.Hq + hd) * D;
            q[i] = y1;
            q[i + half] = y2;
        } else {
            const int kvh = hd - a.Hq;
            cache_store<D>(a.kc, a.vc, scene, kvh, a.Hkv, a.NB, pos, i, true, f2bf(y1));
            cache_store<D>(a.kc, a.vc, scene, kvh, a.Hkv, a.NB, pos, i + half, true, f2bf(y2));
        }
    } else {
        cache_store<D>(a.kc, a.vc, scene, e / D, a.Hkv, a.NB, pos, e % D, false, f2bf(x1));
        cache_store<D>(a.kc, a.vc, scene, e / D, a.Hkv, a.NB, pos, e % D + 1, false, f2bf(x2));
    }
}

template <int D>
__global__ __launch_bounds__(256) void kv_scatter_kernel(const uint16_t* __restrict__ k_new,
                                                         const uint16_t* __restrict__ v_new,
                                                         const int32_t* __restrict__ row_scene,
                                                         const int32_t* __restrict__ row_pos,
                                                         int n_rows, uint16_t* kc, uint16_t* vc,
                                                         int B, int Hkv, int NB, int N) {
    const int r = blockIdx.x;
    const int scene = row_scene[r], pos = row_pos[r];
    if (scene < 0 || scene >= B || pos < 0 || pos >= N) return;
    for (int e = threadIdx.x; e < Hkv * D; e += blockDim.x) {
        const size_t src = (size_t)r * Hkv * D + e;
        cache_store<D>(kc, vc, scene, e / D, Hkv, NB, pos, e % D, true, k_new[src]);
        cache_store<D>(kc, vc, scene, e / D, Hkv, NB, pos, e % D, false, v_new[src]);
    }
}

struct Top2 {
    float m1, m2;
    int i1;
};
__device__ __forceinline__ Top2 top2_merge(Top2 a, Top2 b) {
    if (b.m1 > a.m1 || (b.m1 == a.m1 && b.i1 < a.i1)) {
        Top2 t = a;
        a = b;
        b = t;
    }
    a.m2 = fmaxf(a.m2, b.m1);
    return a;
}

// One workgroup per row.  Lowest index among equal maxima; gap = best - runner-up.
__global__ __launch_bounds__(1024) void argmax_kernel(const float* __restrict__ logits, int V,
                                                      int64_t ld, int32_t* idx, float* gap,
                                                      const int32_t* branch_field, int T) {
    __shared__ Top2 sh[16];
    const int m = blockIdx.x;
    if (branch_field && branch_field[m / T] < 0) {
        if (threadIdx.x == 0) {
            idx[m] = -1;
            if (gap) gap[m] = 0.f;
        }
        return;
    }
    const float* row = logits + (size_t)m * ld;
    Top2 t{-INFINITY, -INFINITY, 0x7fffffff};
    auto push = [&](float x, int v) {
        if (x > t.m1) {
            t.m2 = t.m1;
            t.m1 = x;
            t.i1 = v;
        } else if (x > t.m2) {
            t.m2 = x;
        }
    };
    if ((reinterpret_cast<uintptr_t>(row) & 15) == 0) {
        // 16-byte loads, eight per thread in flight: the row comes in about one
        // round trip instead of one per element
        const int V4 = V >> 2;
        constexpr int U = 8;
        for (int v0 = threadIdx.x; v0 < V4; v0 += U * blockDim.x) {
            float4 x[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int v4 = v0 + u * blockDim.x;
                x[u] = v4 < V4 ? reinterpret_cast<const float4*>(row)[v4] : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int v = 4 * (v0 + u * blockDim.x);
                push(x[u].x, v);
                push(x[u].y, v + 1);
                push(x[u].z, v + 2);
                push(x[u].w, v + 3);
            }
        }
        for (int v = 4 * V4 + threadIdx.x; v < V; v += blockDim.x) push(row[v], v);
    } else {
        for (int v = threadIdx.x; v < V; v += blockDim.x) push(row[v], v);
    }
    for (int o = 32; o > 0; o >>= 1) {
        Top2 u{__shfl_xor(t.m1, o), __shfl_xor(t.m2, o), __shfl_xor(t.i1, o)};
        t = top2_merge(t, u);
    }
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = t;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < (int)(blockDim.x >> 6); ++w) t = top2_merge(t, sh[w]);
        idx[m] = t.i1;
        if (gap) gap[m] = t.m1 - t.m2;
    }
}

// The step's small tables (branch fields, offsets, valid lengths) come from pinned
// host memory, which the device reads directly: one workgroup copies them into
// the workspace, where every later kernel of the step finds them.
__global__ __launch_bounds__(256) void tables_copy_kernel(const int32_t* __restrict__ host_tables,
                                                          int32_t* __restrict__ dev_tables, int n) {
    for (int i = threadIdx.x; i < n; i += 256) dev_tables[i] = host_tables[i];
}

// measurement helpers: an empty kernel (what an event pair costs around a
// launch) and a streaming copy (what the device's HBM sustains, and the
// reference the traffic counters are scaled by)
__global__ void null_kernel() {}

typedef unsigned int copy_u32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void stream_copy_kernel(const copy_u32x4* __restrict__ src,
                                                          copy_u32x4* __restrict__ dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride)
        __builtin_nontemporal_store(__builtin_nontemporal_load(&src[i]), &dst[i]);
}

}  // namespace

void launch_null(hipStream_t st) { null_kernel<<<1, 64, 0, st>>>(); }

void launch_tables_copy(const int32_t* host_tables, int32_t* dev_tables, int n, hipStream_t st) {
    if (n > 0) tables_copy_kernel<<<1, 256, 0, st>>>(host_tables, dev_tables, n);
}

void launch_stream_copy(const void* src, void* dst, size_t bytes, hipStream_t st) {
    const size_t n16 = bytes / 16;
    const size_t want = (n16 + 256 * 8 - 1) / (256 * 8);
    const unsigned grid = (unsigned)std::min<size_t>(std::max<size_t>(want, 1), 256 * 16);
    stream_copy_kernel<<<grid, 256, 0, st>>>((const copy_u32x4*)src, (copy_u32x4*)dst, n16);
}

void launch_resid_norm(const NormArgs& a, const StepMeta& sm, hipStream_t st) {
    const int nvec = a.d / 4;                       // d_model <= 8192
    if (nvec <= 256) hipLaunchKernelGGL((resid_norm_kernel<256, 1>), dim3(a.M), dim3(256), 0, st, a, sm);
    else if (nvec <= 1024) hipLaunchKernelGGL((resid_norm_kernel<1024, 1>), dim3(a.M), dim3(1024), 0, st, a, sm);
    else hipLaunchKernelGGL((resid_norm_kernel<1024, 2>), dim3(a.M), dim3(1024), 0, st, a, sm);
}

void launch_rope_table(const double* inv_freq, float2* tab, int n_pos, int half, hipStream_t st) {
    const int n = n_pos * half;
    hipLaunchKernelGGL(rope_table_kernel, dim3((n + 255) / 256), dim3(256), 0, st, inv_freq, tab, n_pos, half);
}

void launch_rope_append(const RopeArgs& a, const StepMeta& sm, hipStream_t st) {
    const int items = (a.Hq + a.Hkv) * a.D / 2 + a.Hkv * a.D / 2;
    const dim3 grid((items + 255) / 256, a.M);
    if (a.D == 128) hipLaunchKernelGGL(rope_append_kernel<128>, grid, dim3(256), 0, st, a, sm);
    else hipLaunchKernelGGL(rope_append_kernel<64>, grid, dim3(256), 0, st, a, sm);
}

void launch_kv_scatter(const uint16_t* k_new, const uint16_t* v_new, const int32_t* row_scene,
                       const int32_t* row_pos, int n_rows, uint16_t* kc, uint16_t* vc, int B,
                       int Hkv, int D, int NB, int N, hipStream_t st) {
    if (n_rows <= 0) return;
    if (D == 128)
        hipLaunchKernelGGL(kv_scatter_kernel<128>, dim3(n_rows), dim3(256), 0, st, k_new, v_new,
                           row_scene, row_pos, n_rows, kc, vc, B, Hkv, NB, N);
    else
        hipLaunchKernelGGL(kv_scatter_kernel<64>, dim3(n_rows), dim3(256), 0, st, k_new, v_new,
                           row_scene, row_pos, n_rows, kc, vc, B, Hkv, NB, N);
}

void launch_argmax(const float* logits, int M, int V, int64_t ld, int32_t* idx, float* gap,
                   const int32_t* branch_field, int T, hipStream_t st) {
    if (M <= 0) return;
    hipLaunchKernelGGL(argmax_kernel, dim3(M), dim3(1024), 0, st, logits, V, ld, idx, gap,
                       branch_field, T);
}

}  // namespace fdc
