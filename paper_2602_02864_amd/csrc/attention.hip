// DAG-masked GQA decode attention over the field-slot KV cache (Sec. 3.3).
//
// All query rows that share a KV head - every active branch of a scene, its T
// new tokens and the G query heads of the group - form one row tile, so the
// shared prefix and every visible slot are streamed from HBM once for all of
// them (the paper's "shared KV cache accessed by multiple query tokens within a
// single attention kernel").  The key dimension is cut into chunks (split-K);
// a workgroup of four wavefronts takes one chunk of one (scene, kv head, row
// group), its wavefronts take the chunk's 32-key tiles round-robin, merge
// their softmax states through LDS in a fixed order and emit one partial.  A
// second kernel merges the chunks' partials in chunk order (no atomics: results
// are bit-reproducible).
//
// The mask is never materialised.  A row of field f at slot offset t sees
//   the prefix, the first valid_len[g] keys of each strict ancestor slot g, and
//   the first t+1 keys of its own slot;
// i.e. a *count* of visible keys per slot.  The kernel builds that count table
// in LDS from the ancestor bit words, skips every 32-key tile no row of the
// tile can see, runs prefix tiles without any masking, and masks slot tiles
// per key with one table lookup.
//
// Matrix-core mapping (v_mfma_f32_32x32x16_bf16): S^T = K * Q^T puts one query
// row in each lane (column = lane % 32), so the running max / sum are in-lane
// plus one exchange with lane ^ 32; the score registers are, unchanged, the
// P^T operand of O^T = V^T * P^T because the V tiles are stored in that key
// order.  K and V tiles are contiguous 1 KiB pieces per load instruction.
#include "kernels_common.hpp"
#include "fdc_launch.hpp"

namespace fdc {

namespace {

constexpr float kNegBig = -1.0e30f;

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

// two floats -> packed bf16 heads and packed bf16 tails (head + tail ~ value to 2^-17)
__device__ __forceinline__ void split2(float x, float y, uint32_t& hi, uint32_t& lo) {
    f32x2 v = {x, y};
    hi = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
    f32x2 r = {x - __uint_as_float(hi << 16), y - __uint_as_float(hi & 0xffff0000u)};
    lo = __builtin_bit_cast(uint32_t, __builtin_convertvector(r, bf16x2));
}

union Frag {
    bf16x8 v;
    uint32_t u[4];
};

// QF32: the queries come in fp32 (inside the decode step) and are used as bf16
// head + tail; otherwise they are bf16 data and have no tail.  The softmax
// weights are always used as head + tail, so the only bf16 rounding left in the
// attention is the one the bf16 KV cache itself implies.
template <int D, int NRT, bool QF32>
__global__ __launch_bounds__(256) void attn_partial_kernel(AttnArgs a, StepMeta sm) {
    constexpr int DJ = D / 16, DT = D / 32, NR = NRT * 32, QP = QF32 ? 2 : 1;
    __shared__ uint16_t vis[NR][kMaxFields + 2];
    __shared__ uint16_t maxvis[kMaxFields];
    __shared__ int row_field[NR], row_off[NR], row_m[NR], row_head[NR];
    __shared__ float red_m[4][NR], red_l[4][NR];
    __shared__ f32x4 red_o[NRT * DT * 4 * 64];
    __shared__ bf16x8 qs[NRT][DJ][QP][64];

    const int chunk = blockIdx.x, rg = blockIdx.y, z = blockIdx.z;
    const int b = z / a.Hkv, kvh = z % a.Hkv;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int r32 = lane & 31, hh = lane >> 5;
    const int F = sm.F;

    for (int r = tid; r < NR; r += 256) {
        const RowInfo ri = row_info(rg * NR + r, b, kvh, a.G, sm);
        row_m[r] = ri.m;
        row_head[r] = ri.head;
        row_field[r] = ri.field;
        row_off[r] = ri.off;
    }
    __syncthreads();
    // visible-key count of every (row, slot)
    for (int idx = tid; idx < NR * F; idx += 256) {
        const int r = idx / F, g = idx % F;
        const int f = row_field[r];
        int n = 0;
        if (f >= 0) {
            if (g == f) n = row_off[r] + 1;
            else if ((a.anc[f] >> g) & 1ull) n = sm.valid_len[b * F + g];
        }
        vis[r][g] = (uint16_t)n;
    }
    // query operand in LDS: fragment (rt, j) holds, per lane, row rt*32 + lane%32,
    // d = 16*j + 8*(lane/32) + 0..7
    for (int idx = wave; idx < NRT * DJ; idx += 4) {
        const int rt = idx / DJ, j = idx % DJ;
        const int r = rt * 32 + r32;
        const int m = row_m[r];
        Frag fh, fl;
#pragma unroll
        for (int k = 0; k < 4; ++k) fh.u[k] = fl.u[k] = 0;
        if (m >= 0) {
            const size_t qo = ((size_t)m * a.Hq + row_head[r]) * D + 16 * j + 8 * hh;
            if (QF32) {
                const f32x4 q0 = *reinterpret_cast<const f32x4*>(a.q_f32 + qo);
                const f32x4 q1 = *reinterpret_cast<const f32x4*>(a.q_f32 + qo + 4);
                split2(q0[0], q0[1], fh.u[0], fl.u[0]);
                split2(q0[2], q0[3], fh.u[1], fl.u[1]);
                split2(q1[0], q1[1], fh.u[2], fl.u[2]);
                split2(q1[2], q1[3], fh.u[3], fl.u[3]);
            } else {
                fh.v = *reinterpret_cast<const bf16x8*>(a.q_bf16 + qo);
            }
        }
        qs[rt][j][0][lane] = fh.v;
        if (QF32) qs[rt][j][QP - 1][lane] = fl.v;
    }
    __syncthreads();
    if (tid < F) {
        int mx = 0;
        for (int r = 0; r < NR; ++r) mx = max(mx, (int)vis[r][tid]);
        maxvis[tid] = (uint16_t)mx;
    }
    __syncthreads();

    f32x16 o[NRT][DT];
    float m_run[NRT], l_run[NRT];
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) {
        m_run[rt] = kNegBig;
        l_run[rt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[rt][dt][i] = 0.f;
    }

    const int blk_end = min(a.NB, (chunk + 1) * a.CB);
    const size_t tile_base = ((size_t)b * a.Hkv + kvh) * a.NB;

    // a tile that reaches into the slots is fetched only if some row of the row
    // tile can see one of its keys (wave-uniform answer)
    auto tile_active = [&](int blk) -> bool {
        const int key0 = blk * 32;
        if (key0 + 32 <= a.P) return true;
        bool mine = false;
        if (lane < 32) {
            const int key = key0 + lane;
            if (key < a.P) mine = true;
            else {
                const uint32_t tab = a.slot_tab[key - a.P];
                mine = tab != 0xffffffffu && (tab >> 8) < maxvis[tab & 0xff];
            }
        }
        return __any(mine);
    };
    auto load_tile = [&](int blk, bf16x8 (&kf)[DJ], bf16x8 (&vf)[DT][2]) {
        const uint16_t* kt = a.kc + (tile_base + blk) * (32 * D);
        const uint16_t* vt = a.vc + (tile_base + blk) * (32 * D);
#pragma unroll
        for (int j = 0; j < DJ; ++j)
            kf[j] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(kt + (j * 64 + lane) * 8));
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int s = 0; s < 2; ++s)
                vf[dt][s] = __builtin_nontemporal_load(
                    reinterpret_cast<const bf16x8*>(vt + ((dt * 2 + s) * 64 + lane) * 8));
    };

    int blk = chunk * a.CB + wave;
    while (blk < blk_end && !tile_active(blk)) blk += 4;
    bf16x8 kn[DJ], vn[DT][2];
    if (blk < blk_end) load_tile(blk, kn, vn);

    while (blk < blk_end) {
        // keeps the query fragments in LDS (re-read per tile) instead of letting
        // the compiler hoist them into 64-128 registers for the whole loop
        asm volatile("" ::: "memory");
        bf16x8 kf[DJ], vf[DT][2];
#pragma unroll
        for (int j = 0; j < DJ; ++j) kf[j] = kn[j];
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            vf[dt][0] = vn[dt][0];
            vf[dt][1] = vn[dt][1];
        }
        // next tile of this wavefront: issue its loads before computing on this one
        int nxt = blk + 4;
        while (nxt < blk_end && !tile_active(nxt)) nxt += 4;
        if (nxt < blk_end) load_tile(nxt, kn, vn);

        const int key0 = blk * 32;
        const bool masked = key0 + 32 > a.P;          // tile reaches into the slots
        // register i of this lane belongs to key0 + 8*(i/4) + 4*hh + i%4.  For a
        // tile that reaches into the slots look the keys up once: tabs[i] =
        // field | offset << 8, anybits = keys some row of the tile can see.  Keys
        // nobody sees may be padding or not yet written: they may hold anything.
        uint32_t tabs[16];
        uint32_t anybits = 0xffffu;
        if (masked) {
            anybits = 0;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int key = key0 + 8 * (i >> 2) + 4 * hh + (i & 3);
                bool v;
                if (key < a.P) {
                    tabs[i] = 0xfffffffeu;            // prefix key
                    v = true;
                } else {
                    tabs[i] = a.slot_tab[key - a.P];
                    v = tabs[i] != 0xffffffffu && (tabs[i] >> 8) < maxvis[tabs[i] & 0xff];
                }
                anybits |= (v ? 1u : 0u) << i;
            }
            if (anybits != 0xffffu) {
                // zero the V columns of keys nobody sees (0 * garbage must stay 0)
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    uint32_t wm[4];
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        wm[k] = ((anybits >> (8 * s + 2 * k) & 1u) ? 0x0000ffffu : 0u) |
                                ((anybits >> (8 * s + 2 * k + 1) & 1u) ? 0xffff0000u : 0u);
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt) {
                        Frag cv;
                        cv.v = vf[dt][s];
#pragma unroll
                        for (int k = 0; k < 4; ++k) cv.u[k] &= wm[k];
                        vf[dt][s] = cv.v;
                    }
                }
            }
        }
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt) {
            f32x16 sc;
#pragma unroll
            for (int i = 0; i < 16; ++i) sc[i] = 0.f;
#pragma unroll
            for (int j = 0; j < DJ; ++j) {
                sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[j], qs[rt][j][0][lane], sc, 0, 0, 0);
                if (QF32)
                    sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[j], qs[rt][j][QP - 1][lane], sc, 0, 0, 0);
            }
            uint32_t vbits = 0xffffu;
            if (masked) {
                vbits = 0;
                const int r = rt * 32 + r32;
                const bool act = row_m[r] >= 0;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const uint32_t tab = tabs[i];
                    const bool v = tab == 0xfffffffeu ? act
                                 : (tab != 0xffffffffu && (tab >> 8) < vis[r][tab & 0xff]);
                    vbits |= (v ? 1u : 0u) << i;
                }
            }
            float mx = kNegBig;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                sc[i] = (vbits >> i & 1u) ? sc[i] * a.scale_log2 : kNegBig;
                mx = fmaxf(mx, sc[i]);
            }
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run[rt], mx);
            const float alpha = exp2f(m_run[rt] - m_new);
            m_run[rt] = m_new;
            float psum = 0.f;
            float p[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                p[i] = (vbits >> i & 1u) ? exp2f(sc[i] - m_new) : 0.f;
                psum += p[i];
            }
            l_run[rt] = l_run[rt] * alpha + psum;
            Frag ph[2], pl[2];
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    split2(p[8 * s + 2 * k], p[8 * s + 2 * k + 1], ph[s].u[k], pl[s].u[k]);
            const bool rescale = __any(alpha != 1.0f);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                if (rescale) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) o[rt][dt][i] *= alpha;
                }
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    o[rt][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[dt][s], ph[s].v, o[rt][dt], 0, 0, 0);
                    o[rt][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[dt][s], pl[s].v, o[rt][dt], 0, 0, 0);
                }
            }
        }
        blk = nxt;
    }

    // ---- merge the four wavefronts (fixed order), emit one partial ---------------
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) {
        l_run[rt] += __shfl_xor(l_run[rt], 32);
        if (hh == 0) red_m[wave][rt * 32 + r32] = m_run[rt];
    }
    __syncthreads();
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) {
        const int r = rt * 32 + r32;
        const float mg = fmaxf(fmaxf(red_m[0][r], red_m[1][r]), fmaxf(red_m[2][r], red_m[3][r]));
        const float sc = exp2f(m_run[rt] - mg);
        if (hh == 0) red_l[wave][r] = l_run[rt] * sc;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[rt][dt][i] *= sc;
    }
    for (int w = 0; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int i4 = 0; i4 < 4; ++i4) {
                        f32x4 v = {o[rt][dt][4 * i4], o[rt][dt][4 * i4 + 1], o[rt][dt][4 * i4 + 2],
                                   o[rt][dt][4 * i4 + 3]};
                        const int idx = ((rt * DT + dt) * 4 + i4) * 64 + lane;
                        if (w == 0) red_o[idx] = v;
                        else red_o[idx] += v;
                    }
        }
        __syncthreads();
    }
    const size_t pidx = ((size_t)z * a.n_rg + rg) * a.n_chunks + chunk;
    f32x4* po = reinterpret_cast<f32x4*>(a.part_o) + pidx * (NRT * DT * 4 * 64);
    for (int i = tid; i < NRT * DT * 4 * 64; i += 256) po[i] = red_o[i];
    if (tid < NR) {
        float* ml = a.part_ml + (pidx * NR + tid) * 2;
        ml[0] = fmaxf(fmaxf(red_m[0][tid], red_m[1][tid]), fmaxf(red_m[2][tid], red_m[3][tid]));
        ml[1] = red_l[0][tid] + red_l[1][tid] + red_l[2][tid] + red_l[3][tid];
    }
}

// Merge the chunks' partials of one (scene, kv head, row group) in chunk order.
// One thread per 4 consecutive head-dim elements of one row.
template <int D, int NRT>
__global__ __launch_bounds__(256) void attn_merge_kernel(AttnArgs a, StepMeta sm) {
    constexpr int DT = D / 32, NR = NRT * 32, Q4 = NRT * DT * 4 * 64;
    const int q4 = blockIdx.x * 256 + threadIdx.x;
    if (q4 >= Q4) return;
    const int zr = blockIdx.y, z = zr / a.n_rg, rg = zr % a.n_rg;
    const int b = z / a.Hkv, kvh = z % a.Hkv;
    const int lane = q4 & 63, i4 = (q4 >> 6) & 3, dt = (q4 >> 8) % DT, rt = (q4 >> 8) / DT;
    const int r = rt * 32 + (lane & 31);
    const int d0 = 32 * dt + 8 * i4 + 4 * (lane >> 5);
    const RowInfo ri = row_info(rg * NR + r, b, kvh, a.G, sm);
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
    const size_t p0 = (size_t)zr * a.n_chunks;
    float mg = kNegBig;
    for (int c = 0; c < a.n_chunks; ++c) mg = fmaxf(mg, a.part_ml[((p0 + c) * NR + r) * 2]);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    float L = 0.f;
    for (int c = 0; c < a.n_chunks; ++c) {
        const float* ml = a.part_ml + ((p0 + c) * NR + r) * 2;
        const float l = ml[1];
        if (l > 0.f) {
            const float w = exp2f(ml[0] - mg);
            L += w * l;
            acc += w * reinterpret_cast<const f32x4*>(a.part_o)[(p0 + c) * Q4 + q4];
        }
    }
    const float inv = L > 0.f ? 1.0f / L : 0.f;
    acc *= inv;
    if (a.out_f32) {
        *reinterpret_cast<f32x4*>(a.out_f32 + ((size_t)ri.m * a.Hq + ri.head) * D + d0) = acc;
    } else {
        uint16_t hi[4], lo[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) split_bf16(acc[i], hi[i], lo[i]);
        const size_t o = act_frag_index(ri.m, ri.head * D + d0, a.Hq * D / 32);
        *reinterpret_cast<uint2*>(a.out_hi + o) =
            make_uint2(hi[0] | (uint32_t)hi[1] << 16, hi[2] | (uint32_t)hi[3] << 16);
        *reinterpret_cast<uint2*>(a.out_lo + o) =
            make_uint2(lo[0] | (uint32_t)lo[1] << 16, lo[2] | (uint32_t)lo[3] << 16);
    }
}

template <int D, int NRT>
void launch_t(const AttnArgs& a, const StepMeta& sm, hipStream_t st) {
    const int z = sm.B * a.Hkv;
    if (a.q_f32)
        hipLaunchKernelGGL((attn_partial_kernel<D, NRT, true>), dim3(a.n_chunks, a.n_rg, z), dim3(256),
                           0, st, a, sm);
    else
        hipLaunchKernelGGL((attn_partial_kernel<D, NRT, false>), dim3(a.n_chunks, a.n_rg, z), dim3(256),
                           0, st, a, sm);
    constexpr int Q4 = NRT * (D / 32) * 4 * 64;
    hipLaunchKernelGGL((attn_merge_kernel<D, NRT>), dim3((Q4 + 255) / 256, z * a.n_rg), dim3(256), 0,
                       st, a, sm);
}

}  // namespace

void launch_attention(const AttnArgs& a, const StepMeta& sm, hipStream_t st) {
    if (a.D == 128) {
        if (a.nrt == 2) launch_t<128, 2>(a, sm, st);
        else launch_t<128, 1>(a, sm, st);
    } else {
        if (a.nrt == 2) launch_t<64, 2>(a, sm, st);
        else launch_t<64, 1>(a, sm, st);
    }
}

}  // namespace fdc
