// Host-callable launchers of the gfx950 kernels.  Every launcher only enqueues
// work on `st`; none allocates or synchronises.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

#include "fdc_internal.hpp"

namespace fdc {

// ---- projections (gemm_skinny.hip) -----------------------------------------
enum GemmEpilogue { EPI_PARTIAL = 0, EPI_SWIGLU = 1 };

struct GemmArgs {
    const uint16_t* w;        // packed weights
    const uint16_t* act_hi;   // activation fragments, bf16 head
    const uint16_t* act_lo;   // bf16 tail, or nullptr
    float* out;               // EPI_PARTIAL: [S][M][N] fp32
    uint16_t* out_hi;         // EPI_SWIGLU: fragments of silu(g)*u for the next projection
    uint16_t* out_lo;
    int M;                    // valid rows
    int N;                    // row stride of `out`
    int n_valid;              // output features actually stored (multiple of 4)
    int out_KT;               // EPI_SWIGLU: k tiles of the consumer (= d_mlp / 32)
    // tiled kernels only: `w` is the fp16 copy of the weights (values times 2^8) and
    // act_hi holds single fp16 fragments (no tail); results are multiplied by
    // out_scale (2^-8)
    bool f16;
    float out_scale;
    bool out_f16;             // EPI_SWIGLU writes single fp16 fragments to out_hi (the consumer runs fp16)
};
// both return false (and launch nothing) for a plan no kernel was built for
bool launch_gemm(const GemmPlan& p, int epilogue, const GemmArgs& a, hipStream_t st);
bool launch_gemm_tiled(const TiledPlan& p, int epilogue, const GemmArgs& a, hipStream_t st);
void launch_pack_weight(const uint16_t* src, uint16_t* dst, int64_t n_out, int64_t k_in, int mode,
                        hipStream_t st);
// x fp32 [M][K] -> hi/lo fragments (no normalisation); y = sum of S partials
void launch_to_frag(const float* x, uint16_t* hi, uint16_t* lo, int M, int K, hipStream_t st);
void launch_sum_partials(const float* part, float* y, int S, int M, int64_t N, hipStream_t st);

// ---- row operations (rowops.hip) ---------------------------------------------
struct StepMeta {             // device copies of the step's small tables
    const int32_t* branch_field;   // [B*R]
    const int32_t* branch_off;     // [B*R]
    const int32_t* valid_len;      // [B*F]
    const int32_t* slot_start;     // [F]
    const int32_t* row_pos;        // [B*R*T] position id (= cache index) of every row, -1 for inactive
                                   // rows; written by launch_mask_words for the step
    int B, R, T, F;
};

struct NormArgs {
    float* x;                 // residual stream [M][d], updated in place
    const float* part;        // partial sums to add, [S][M][d], or nullptr
    int S;
    const int32_t* tok;       // first layer: token ids [M] ...
    const uint16_t* emb;      // ... gathered from this [V][d] bf16 table
    const uint16_t* emb_rows; // or input rows [M][d] bf16
    const float* gain;
    float eps;
    uint16_t* a_hi;           // normalised row, fragments for the next projection
    uint16_t* a_lo;
    float* hidden_x;          // optional copy of the updated residual [M][d]
    float* hidden_n;          // optional copy of the normalised row [M][d]
    int M, d, vocab;
    bool f16;                 // a_hi gets single fp16 fragments (a_lo untouched)
};
void launch_resid_norm(const NormArgs& a, const StepMeta& sm, hipStream_t st);

struct RopeArgs {
    const float* part;        // QKV partials [S][M][Nqkv]
    int S;
    float* q;                 // fp32 [M][Hq][D] rotated queries
    uint16_t* kc;             // layer base of the K cache
    uint16_t* vc;
    const float2* tab;        // [N][D/2] (cos, sin) of pos * base^(-2i/D)
    int M, Hq, Hkv, D, NB;    // NB = 32-key tiles per (scene, kv head)
};
void launch_rope_append(const RopeArgs& a, const StepMeta& sm, hipStream_t st);
void launch_rope_table(const double* inv_freq, float2* tab, int n_pos, int half, hipStream_t st);

void launch_kv_scatter(const uint16_t* k_new, const uint16_t* v_new, const int32_t* row_scene,
                       const int32_t* row_pos, int n_rows, uint16_t* kc, uint16_t* vc, int B,
                       int Hkv, int D, int NB, int N, hipStream_t st);

void launch_argmax(const float* logits, int M, int V, int64_t ld, int32_t* idx, float* gap,
                   const int32_t* branch_field, int T, hipStream_t st);

// host_tables: pinned host memory (device-readable); n ints into the workspace
void launch_tables_copy(const int32_t* host_tables, int32_t* dev_tables, int n, hipStream_t st);
void launch_null(hipStream_t st);
void launch_stream_copy(const void* src, void* dst, size_t bytes, hipStream_t st);

// ---- attention (attention.hip) -------------------------------------------------
struct AttnArgs {
    const uint16_t* q_bf16;   // queries [M][Hq][D]: bf16 data ...
    const float* q_f32;       // ... or fp32 (used as bf16 head + tail)
    const uint16_t* kc;       // layer base
    const uint16_t* vc;
    float* part_o;            // [z*n_rg][n_chunks][NR*D]
    float* part_ml;           // [z*n_rg][n_chunks][NR][2]
    const uint32_t* mask_words; // the step's visibility words [B][mw_tiles][R*T] (launch_mask_words)
    int mw_tiles;             // tiles that reach past the prefix: NB - P / 32
    float* out_f32;           // merge output: fp32 [M][Hq*D] ...
    uint16_t* out_hi;         // ... or fragments with K = Hq*D: bf16 head + tail,
    uint16_t* out_lo;         //     or (out_f16) single fp16 fragments in out_hi
    bool out_f16;
    int Hq, Hkv, G, D, P, NB, CB, n_chunks, n_rg, nrt;   // CB: weighted tiles per chunk
    int wq;                   // weight of a tile past the prefix, in sixteenths of a prefix tile
    int variant;              // 0: LDS-shared tiles (direct-to-LDS ring), 1: tiles in registers
    float scale_log2;         // log2(e) / sqrt(D)
};
void launch_attention(const AttnArgs& a, const StepMeta& sm, hipStream_t st);
// once per step, after the step's tables are on the device and before its first
// kernel: the visibility words and the rows' position ids (sm.row_pos is written)
void launch_mask_words(const StepMeta& sm, const uint64_t* anc, int P, int n_tiles, uint32_t* words,
                       hipStream_t st);

// First 32-key tile of key chunk c of an attention launch.  Tiles that reach past
// the prefix carry masks and cost more (measured: about 1.5 plain tiles each,
// their table set-up included), so chunks are equal in weighted tiles: a tile
// past the prefix counts wq / 16.  P: prefix length, NB: tiles in all, CB:
// weighted tiles per chunk.
__host__ __device__ inline int attn_chunk_start(int P, int NB, int CB, int wq, int c) {
    const int t0 = P >> 5;
    const long x = (long)c * CB;
    if (x <= t0) return (int)x;
    const long t = t0 + (16 * (x - t0) + wq - 1) / wq;
    return (int)(t < NB ? t : NB);
}

}  // namespace fdc
