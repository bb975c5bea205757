/*
 * fdc - parallel decoding step for template-structured chain-of-thought on one
 * AMD MI355X (gfx950).  C ABI: plain pointers and sizes only.
 *
 * The library implements the forward pass in which every ready field of a CoT
 * template decodes together (Sec. 3.3 of the FastDriveCoT paper): the new
 * tokens of all ready fields are packed along the sequence dimension of one
 * sequence, attend through a mask derived from the template's dependency graph
 * (Eq. 1) to the shared prefix, to the written tokens of their ancestor fields
 * and to their own earlier tokens, use position ids fixed by the per-field
 * slot lengths, and share one KV cache in which padding is never written or
 * read.  Which fields are ready is decided by the caller (Algorithm 1).
 *
 * Conventions
 *  - every function returns 0 (FDC_OK) or a negative FDC_E* code; a message for
 *    the last failure of the calling thread is available from fdc_last_error().
 *  - "host" pointers are ordinary CPU memory, read or written before the call
 *    returns.  "device" pointers are GPU memory owned by the caller; the
 *    library allocates no device memory (the caller sizes buffers with the
 *    *_bytes queries).  Device work is enqueued on the given hipStream_t
 *    (passed as void*) and the call returns without synchronising.
 *  - matrices handed in are bf16, row-major, [out_features][in_features];
 *    a projection is y = x * W^T.  fdc_pack_weight() converts them once into
 *    the tile order the kernels stream.
 *  - rows of a step are ordered m = (scene * R + branch) * T + t.
 *  - limits: n_fields <= 64 for a context; head_dim in {64, 128};
 *    d_model, n_q_heads*head_dim and d_mlp multiples of 32, vocab of 4;
 *    d_model <= 5120; B*R*T <= 1024 rows per step; at most 65535 * 32 cache
 *    positions per scene (FDC_ECAP otherwise).  Up to
 *    16 rows the projections stream the weights once (HBM-bound kernels), above
 *    that they run as tiled matrix-core products (single-pass on an fp16 copy of
 *    the weights where the caller provides one).
 */
#ifndef FDC_H
#define FDC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FDC_OK       0
#define FDC_EINVAL  (-1)  /* null pointer, bad size, misaligned pointer          */
#define FDC_ECYCLE  (-2)  /* dependency graph is not acyclic                      */
#define FDC_EORDER  (-3)  /* an edge points from a later field to an earlier one */
#define FDC_ERANGE  (-4)  /* field id, slot offset or position out of range       */
#define FDC_ECAP    (-5)  /* a size exceeds what the kernels are built for        */
#define FDC_EHIP    (-6)  /* a HIP runtime call failed                            */
#define FDC_ESTATE  (-7)  /* weights, cache or workspace not set                  */

typedef struct fdc_ctx fdc_ctx;

typedef struct fdc_model_desc {
    int32_t n_layers;
    int32_t d_model;
    int32_t n_q_heads;
    int32_t n_kv_heads;   /* divides n_q_heads (grouped-query attention) */
    int32_t head_dim;     /* 64 or 128 */
    int32_t d_mlp;        /* SwiGLU inner width */
    int32_t vocab;
    float   rope_base;    /* rotary base; pair (i, i + head_dim/2) turns by pos * base^(-2i/head_dim) */
    float   norm_eps;     /* RMSNorm epsilon */
} fdc_model_desc;

/* device pointers to one decoder layer's parameters */
typedef struct fdc_layer_weights {
    const float* g1;      /* [d_model] fp32 gain of the attention RMSNorm               */
    const void*  wqkv;    /* packed [(Hq+2Hkv)*D][d_model]; rows: Q heads, K heads, V heads */
    const void*  wo;      /* packed [d_model][Hq*D]                                      */
    const float* g2;      /* [d_model] fp32 gain of the MLP RMSNorm                      */
    const void*  wgu;     /* packed with mode FDC_PACK_GATE_UP from [2*d_mlp][d_model], gate rows first */
    const void*  wd;      /* packed [d_model][d_mlp]                                     */
} fdc_layer_weights;

const char* fdc_strerror(int32_t code);
const char* fdc_last_error(void);
int32_t     fdc_version(void);

/* ---------------------------------------------------------------------------
 * Template -> mask metadata (host only; no GPU needed).  Sec. 3.3, Eq. 1:
 * a token of field B may attend to tokens of field A iff a path of >= 1 edge
 * leads from A to B.  Fixed slot lengths fix every position id.
 *
 *  slot_len [F]        host in   fixed length of each field's slot (>= 1)
 *  edge_src/dst [E]    host in   direct dependencies src -> dst
 *  anc_words [F*W]     host out  strict ancestors, bit (g%64) of word g/64 of
 *                                row f, W = (F+63)/64
 *  slot_start [F]      host out  prefix_len + sum of earlier slot lengths
 *  level [F]           host out  longest-path depth, roots 0 (may be NULL)
 *  total_len           host out  N = prefix_len + sum of slots
 * Errors: FDC_EINVAL (null, F < 1, slot < 1, prefix < 0), FDC_ERANGE (edge names
 * a field outside 0..F-1), FDC_ECYCLE, FDC_EORDER (src >= dst: the template order
 * must be a topological order so that visible keys precede the query).
 */
int32_t fdc_build_mask(int32_t n_fields, const int32_t* slot_len,
                       int32_t n_edges, const int32_t* edge_src, const int32_t* edge_dst,
                       int32_t prefix_len,
                       uint64_t* anc_words, int32_t* slot_start, int32_t* level,
                       int32_t* total_len);

/* Dense expansion of the template metadata (slot starts, ancestor words) under
 * a given cache state, for one scene, computed on the host (host only; test
 * helper: it checks fdc_build_mask's outputs, not the device's tables - for
 * those see fdc_step_tables_dense).  Row r is the token at offset
 * row_off[r] of field row_field[r]; valid_len[g] is the number of tokens of
 * field g in the cache after the step's appends.  mask[r*N + j] = 1 iff j is
 * in the prefix, or a written token of a strict ancestor, or an own token at
 * offset <= row_off[r] (Sec. 3.3: padding is invisible to everyone).
 * pos[r] = slot_start[row_field[r]] + row_off[r].
 */
int32_t fdc_dense_mask(int32_t n_fields, const int32_t* slot_len, const int32_t* slot_start,
                       const uint64_t* anc_words, int32_t prefix_len,
                       const int32_t* valid_len,
                       int32_t n_rows, const int32_t* row_field, const int32_t* row_off,
                       uint8_t* mask, int32_t* pos);

/* ---------------------------------------------------------------------------
 * Algorithm 1 (host only): in-degree counters and the ready set.
 *
 * fdc_sched_peek returns the ready fields in field order with their next slot
 * offset and pads the arrays [max_branches] with field -1; *n_active == 0 means
 * every field is complete.  fdc_sched_advance then accounts one decoded token
 * per ready field; field_finished[i] != 0 says that the i-th field peek
 * returned is finished (the model ended its line, or its slot is full): it
 * leaves the set and releases the successors whose last prerequisite it was.
 * fdc_sched_complete marks a field whose tokens are known beforehand (fixed
 * template text, Sec. 3.3) as finished with n_tokens tokens without a pass; its
 * prerequisites must be complete already.
 *
 * fdc_sched_next is peek + advance with "finished" := content_len[f] tokens
 * decoded (the caller's stand-in for the model ending the line; needs a
 * scheduler created with content_len != NULL, each >= 1).  With it the number
 * of non-empty passes equals the critical-path length of the template.
 * fdc_sched_stats: passes and tokens accounted so far, fields not finished yet
 * (each pointer may be NULL).
 * Errors: as fdc_build_mask for the graph; FDC_ECAP if more than max_branches
 * fields are ready; FDC_EINVAL if n differs from the size of the ready set.
 */
typedef struct fdc_sched fdc_sched;
int32_t fdc_sched_create(int32_t n_fields, int32_t n_edges, const int32_t* edge_src,
                         const int32_t* edge_dst, const int32_t* content_len /* or NULL */,
                         fdc_sched** out);
int32_t fdc_sched_peek(fdc_sched* s, int32_t max_branches, int32_t* branch_field,
                       int32_t* branch_off, int32_t* n_active);
int32_t fdc_sched_advance(fdc_sched* s, int32_t n, const int32_t* field_finished);
int32_t fdc_sched_complete(fdc_sched* s, int32_t field, int32_t n_tokens);
int32_t fdc_sched_next(fdc_sched* s, int32_t max_branches, int32_t* branch_field,
                       int32_t* branch_off, int32_t* n_active);
int32_t fdc_sched_stats(const fdc_sched* s, int64_t* passes, int64_t* tokens, int32_t* n_unfinished);
void    fdc_sched_destroy(fdc_sched* s);

/* ---------------------------------------------------------------------------
 * Weight packing.  Streams a row-major bf16 matrix [n_out][k_in] (device) into
 * the 16x32-element tile order the projection kernels read with one contiguous
 * 1 KiB load per wavefront.  k_in multiple of 32; n_out is padded with zero
 * rows to a multiple of 16 in dst.
 * FDC_PACK_GATE_UP interleaves the 16-row tiles of the gate half and the up
 * half of a [2*d_mlp][d_model] matrix (n_out multiple of 32) so SwiGLU can be
 * applied in the projection's epilogue.  dst needs
 * fdc_packed_weight_bytes(n_out, k_in) bytes and must not overlap src.
 */
#define FDC_PACK_PLAIN   0
#define FDC_PACK_GATE_UP 1
/* flag, or-ed to either mode: dst holds fp16 instead of bf16, each weight times
 * 2^8 (exact for 2^-22 <= |w| < 256; smaller ones are rounded to the nearest
 * fp16 subnormal, absolute error below 2^-33; larger ones saturate).  The fp16
 * copy feeds the single-pass projections of steps with more than 16 rows, see
 * fdc_set_layer_weights_f16. */
#define FDC_PACK_F16     2
size_t  fdc_packed_weight_bytes(int64_t n_out, int64_t k_in);
int32_t fdc_pack_weight(const void* src_dev, void* dst_dev, int64_t n_out, int64_t k_in,
                        int32_t mode, void* stream);

/* ---------------------------------------------------------------------------
 * Context: model shape + template + batch shape.  Validates the template like
 * fdc_build_mask.  n_scenes = B; max_branches = largest R and max_tokens =
 * largest T a step will use.
 * Tuning and test hooks read from the environment at creation: FDC_ATTN_VARIANT
 * (0 / 1 / 2: attention kernel with K/V tiles shared through LDS by the two row
 * tiles of a KV head / kept in registers / shared through LDS by up to eight
 * row tiles; default: 2 when a step can have more than 64 rows per KV head,
 * else by cache size) and FDC_ATTN_WGS (workgroups the key chunks of one
 * attention launch are cut for).  Results do not depend on them beyond the
 * order of floating-point sums.
 */
int32_t fdc_create(const fdc_model_desc* model,
                   int32_t n_fields, const int32_t* slot_len,
                   int32_t n_edges, const int32_t* edge_src, const int32_t* edge_dst,
                   int32_t prefix_len,
                   int32_t n_scenes, int32_t max_branches, int32_t max_tokens,
                   fdc_ctx** out);
void    fdc_destroy(fdc_ctx* ctx);

/* Bytes of the K cache (the V cache has the same size): all layers, all
 * scenes, position-indexed (cache index == position id), N rounded up to a
 * multiple of 32, bf16, stored in 32-key tiles in the operand order of the
 * attention kernel's matrix instructions. */
size_t  fdc_kv_cache_bytes(const fdc_ctx* ctx);
size_t  fdc_workspace_bytes(const fdc_ctx* ctx);
/* device buffers, 256-byte aligned; kept (not copied) until fdc_destroy */
int32_t fdc_set_kv_cache(fdc_ctx* ctx, void* k_cache_dev, void* v_cache_dev);
/* also uploads the template tables into the workspace on `stream` */
int32_t fdc_set_workspace(fdc_ctx* ctx, void* workspace_dev, size_t bytes, void* stream);
int32_t fdc_set_layer_weights(fdc_ctx* ctx, int32_t layer, const fdc_layer_weights* w);
/* emb: device bf16 row-major [vocab][d_model] (gathered, not packed);
 * gf: device fp32 [d_model] final-norm gain; lm: packed [vocab][d_model] */
int32_t fdc_set_head_weights(fdc_ctx* ctx, const void* emb, const float* gf, const void* lm);

/* Optional second copy of the projection weights as fp16 (packed with
 * FDC_PACK_F16), used by steps of more than 16 rows, where the projections are
 * bound by the matrix cores and not by streaming the weights: with it the
 * activations enter the matrix cores as one fp16 value (11 significant bits)
 * instead of a bf16 head + tail (16 bits), i.e. one matrix instruction per
 * weight fragment instead of two.  Costs the copied weights' size in memory
 * again.  A layer projection takes the fp16 path only when every layer has its
 * copy, the LM head when it has its own; steps of up to 16 rows never do.
 * Activations beyond +-65504 saturate on that path.
 *
 * Which projections take the fp16 path is a mask (fdc_set_f16_projections; bits:
 * 1 QKV, 2 O, 4 gate/up, 8 down, 16 LM head; environment FDC_F16_MASK at creation
 * overrides the default).  The default is 16, the LM head alone: measured on the
 * 7B-class model at 32 rows per step, every other projection run single-pass
 * adds about 3e-4 of the residual stream's scale per layer it is used in, and
 * all of them together reach 2.9e-3 after 28 layers, beyond the 2e-3 this
 * library holds against the fp64 definition; the LM head's rounding does not
 * feed back.  The full mask is for callers who trade that accuracy for about a
 * sixth of the step time at 256 rows. */
typedef struct fdc_layer_weights_f16 {
    const void* wqkv;     /* as fdc_layer_weights, packed with mode | FDC_PACK_F16 */
    const void* wo;
    const void* wgu;
    const void* wd;
} fdc_layer_weights_f16;
int32_t fdc_set_layer_weights_f16(fdc_ctx* ctx, int32_t layer, const fdc_layer_weights_f16* w);
int32_t fdc_set_head_weights_f16(fdc_ctx* ctx, const void* lm_f16);
int32_t fdc_set_f16_projections(fdc_ctx* ctx, int32_t mask);

/* valid_len[b*F + g] = number of tokens of field g of scene b in the cache.
 * host arrays. fdc_reset zeroes them. */
int32_t fdc_reset(fdc_ctx* ctx);
int32_t fdc_set_valid_len(fdc_ctx* ctx, const int32_t* valid_len);
int32_t fdc_get_valid_len(const fdc_ctx* ctx, int32_t* valid_len);

/* ---------------------------------------------------------------------------
 * The one KV cache all branches share (Sec. 3.3): write rows of K (already
 * rotated) and V into layer `layer` of the cache at (scene, position).  Used in
 * bulk to install prefix K/V and slot history; the decode step appends its own
 * rows itself.  Does not change valid_len.
 *  k_new, v_new   device bf16 [n_rows][Hkv][D]
 *  row_scene/pos  device int32 [n_rows]; rows with scene < 0 are skipped.
 *                 Out-of-range scene or position: the row is skipped and the
 *                 call still returns FDC_OK (indices live on the device).
 */
int32_t fdc_kv_append(fdc_ctx* ctx, int32_t layer, const void* k_new, const void* v_new,
                      const int32_t* row_scene, const int32_t* row_pos, int32_t n_rows,
                      void* stream);

/* ---------------------------------------------------------------------------
 * One forward pass in which every listed branch decodes T tokens (Sec. 3.3;
 * the loop body of Algorithm 1).  For each scene b and branch r:
 * field = branch_field[b*R + r] (-1 = inactive entry), first new slot offset =
 * branch_off[b*R + r].  All new K/V are appended (cache index = position id =
 * slot_start[field] + offset) and valid_len is advanced before any row attends;
 * inside a branch the T rows are causal.
 *  branch_field/off host int32 [B*R]
 *  tok_in      device int32 [B*R*T] input token ids, or NULL when emb_in given
 *  emb_in      device bf16 [B*R*T][d_model] input rows, or NULL
 *  tok_out     device int32 [B*R*T] greedy next token (lowest index among
 *              maxima), -1 for inactive rows; or NULL (gap_out and logits_out
 *              NULL too): the rows only fill the cache, the LM head and the
 *              argmax are not run (a prefill pass)
 *  gap_out     device fp32 [B*R*T] top-1 minus top-2 logit, or NULL
 *  logits_out  device fp32 [B*R*T][vocab], or NULL
 *  hidden_out  device fp32 [(L+2)][B*R*T][d_model], or NULL: residual stream
 *              after the embedding (0) and after each layer (1..L), then the
 *              final normalised hidden state (L+1)
 * Errors: FDC_ESTATE, FDC_ECAP (R, T or rows above limits), FDC_ERANGE (field id,
 * offset + T beyond the slot, or an offset beyond the tokens the slot holds:
 * slots fill from the front, a gap would be attended to as if written),
 * FDC_EINVAL (also: a field listed twice for one scene), FDC_EHIP.  On error
 * nothing is enqueued and valid_len is unchanged.
 */
int32_t fdc_parallel_decode_step(fdc_ctx* ctx, int32_t n_branches, int32_t T,
                                 const int32_t* branch_field, const int32_t* branch_off,
                                 const int32_t* tok_in, const void* emb_in,
                                 int32_t* tok_out, float* gap_out,
                                 float* logits_out, float* hidden_out, void* stream);

/* ---------------------------------------------------------------------------
 * Algorithm 1 end to end (Sec. 3.2), with the finishing rules of Sec. 3.3: the
 * template of every scene is decoded greedily from empty slots until every
 * field is finished.  Each iteration runs one fdc_parallel_decode_step for the
 * union of the scenes' ready sets (scenes whose sets differ share the pass;
 * R = the largest set), reads the produced tokens back and decides on the host
 * which fields are finished: a field is finished when the token it just
 * produced is one of eos_ids (the model ended the line) or when its slot is
 * full (truncation to the fixed length).  A field's first input is
 * start_token[f] at slot offset 0; afterwards its previous output.  The
 * finishing token is recorded but not fed back, so valid_len[f] afterwards is
 * the number of tokens recorded for f.
 *
 * Fixed template text (field names, Sec. 3.3: written beforehand and seen by
 * whatever comes after it): a field with fixed_len[f] > 0 holds known tokens.  Such fields are
 * written first, in field order, by multi-token passes of up to max_tokens
 * tokens for all scenes at once, and count as finished from the start; the
 * template's edges say who sees them (a header that every later field depends
 * on is visible to all of them).  Every prerequisite of a fixed field must be
 * fixed too.
 *
 *  start_token  host [F]     ignored for fixed fields
 *  fixed_len    host [F] or NULL (no fixed fields)
 *  fixed_tok    host, the fixed fields' tokens one after the other in field order
 *  eos_ids      host [n_eos] (n_eos may be 0: every field runs to its slot length)
 *  max_passes   > 0: FDC_ECAP if Algorithm 1 needs more passes; <= 0: no limit
 *               (truncation bounds the loop by the longest chain of slots)
 *  out_tok      host [B][F][Smax], Smax = the longest slot: recorded tokens
 *               (for fixed fields their own tokens), -1 beyond out_len
 *  out_len      host [B][F]
 *  out_passes   host [2] or NULL: passes of Algorithm 1, passes spent on fixed fields
 * Needs what fdc_parallel_decode_step needs, with the prefix K/V in the cache.
 * Synchronises `stream` once per pass.  Errors: those of the step and of the
 * scheduler (FDC_ECAP when a ready set exceeds max_branches); after an error
 * the slots hold what was decoded so far.
 */
int32_t fdc_cot_decode(fdc_ctx* ctx, const int32_t* start_token, const int32_t* fixed_len,
                       const int32_t* fixed_tok, const int32_t* eos_ids, int32_t n_eos,
                       int32_t max_passes, int32_t* out_tok, int32_t* out_len, int32_t* out_passes,
                       void* stream);

/* The step's attention alone (Sec. 3.3 mask; one kernel serves all query
 * tokens that read the shared cache): DAG-masked GQA
 * decode attention of the given rotated queries against layer `layer` of the
 * cache under the current valid_len (which must already include the rows'
 * own tokens; not advanced here).
 *  q    device bf16 [B*R*T][Hq][D]
 *  out  device fp32 [B*R*T][Hq*D]; rows of inactive branches are zero
 * The branch tables go to the device and a small kernel derives the step's
 * visibility words from them (one 32-key word per tile past the prefix and
 * branch-token row; every layer's attention reads them).  A call that brings the
 * tables of the previous call on the same stream (another layer in the same
 * state) reuses both.
 */
int32_t fdc_masked_attention(fdc_ctx* ctx, int32_t layer, const void* q,
                             int32_t n_branches, int32_t T,
                             const int32_t* branch_field, const int32_t* branch_off,
                             float* out, void* stream);

/* Test helper for the mask and the position ids the DEVICE uses (Sec. 3.3, Eq. 1;
 * they must equal the definition bit for bit).  Every step builds two tables on
 * the GPU from the branch tables and valid_len: one 32-key visibility word per
 * (scene, tile past the prefix, branch-token row), which is all the attention
 * kernels know about the mask, and one position id per row, which the rotary /
 * append kernel uses as rotation angle index and as cache index.  This call
 * copies both tables back and expands them the way the kernels read them:
 * mask[m*N + j] = 1 iff row m attends to cache position j (tiles that end inside
 * the prefix: every active row; other tiles: bit j%32 of the row's word);
 * pos[m] = the row's position id, -1 for rows of inactive entries (their mask
 * rows are zero).  m = (scene*R + branch)*T + t, N = total_len.
 *  branch_field/off  host [B*R]: the tables are built for this call under the
 *                    current valid_len (which must cover the rows' own tokens,
 *                    as for fdc_masked_attention); or both NULL: the tables the
 *                    last fdc_parallel_decode_step / fdc_masked_attention with
 *                    this R and T left on the device are read (FDC_ESTATE if none)
 *  mask, pos         host out [B*R*T][N] and [B*R*T]
 * Synchronises `stream`. */
int32_t fdc_step_tables_dense(fdc_ctx* ctx, int32_t n_branches, int32_t T,
                              const int32_t* branch_field, const int32_t* branch_off,
                              uint8_t* mask, int32_t* pos, void* stream);

/* How a context cuts its attention launches (host only, works without a GPU;
 * for tests of the launch arithmetic).  info[10]: kernel variant, 32-row tiles
 * per row group, row groups at the largest step, key chunks, weighted tiles per
 * chunk, weight of a tile past the prefix in sixteenths, 32-key tiles in all,
 * tiles that end inside the prefix, the kernel's limit of tiles per chunk, its
 * limit of tiles past the prefix per chunk.  chunk_first_tile [chunks + 1] or
 * NULL: first tile of every chunk, then the end. */
int32_t fdc_attention_plan(const fdc_ctx* ctx, int32_t* info, int32_t* chunk_first_tile);

/* The same for one step (host only): with many rows per KV head the key chunks
 * are cut per step, by how many slot tiles the step's rows see at the current
 * valid_len (tiles nobody sees are skipped by the kernel, so a pass of root
 * fields and a pass of late fields want different cuts).  Arguments as
 * fdc_masked_attention's tables; info and chunk_first_tile as above, with the
 * step's chunk count, weighted tiles per chunk and weight (never more chunks
 * than the context's plan: chunk_first_tile holds that many + 1 entries).
 * Contexts whose plan is not cut per step report the context's plan. */
int32_t fdc_attention_plan_step(fdc_ctx* ctx, int32_t n_branches, int32_t T,
                                const int32_t* branch_field, const int32_t* branch_off,
                                int32_t* info, int32_t* chunk_first_tile);

/* Per-row greedy argmax over fp32 logits (final logits are fp32, Sec. 4.1).
 * logits device [M][ld] (ld >= V); idx_out device int32 [M]: lowest index of
 * the maximum; top2_gap_out device fp32 [M] or NULL. */
int32_t fdc_argmax(const float* logits, int32_t M, int32_t V, int64_t ld,
                   int32_t* idx_out, float* top2_gap_out, void* stream);

/* One dense projection y[M][n_out] = x[M][k_in] * W^T with W packed, x and y
 * device fp32 row-major, M <= 1024; `scratch` device, fdc_linear_scratch_bytes().
 * Exposes the projection kernels of the step for tests and measurements: up to
 * 16 rows the weight-streaming kernel, above it the tiled matrix-core kernel. */
size_t  fdc_linear_scratch_bytes(int32_t M, int64_t n_out, int64_t k_in);
int32_t fdc_linear(const float* x, const void* w_packed, float* y,
                   int32_t M, int64_t n_out, int64_t k_in, void* scratch, void* stream);

/* fdc_linear for callers that cannot allocate device memory or bring a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same kernels and bit-identical results,
 * but the activation fragments and split-K partials live in an 8 MiB array
 * that is part of the library's device image (every GPU the library runs on
 * holds its own copy until the process ends); the call allocates and frees
 * nothing.  FDC_ECAP when fdc_linear_scratch_bytes(M, n_out, k_in) exceeds
 * 8 MiB (8388608 bytes; every M <= 16 projection of the 7B-class shapes fits,
 * large-M products do not): use fdc_linear then.  Nothing in the array needs
 * to start at zero, and it keeps the previous call's contents.  All calls on one
 * GPU share the one array: calls that overlap on a GPU (two streams, two
 * threads) race; calls enqueued on one stream are ordered and safe. */
int32_t fdc_linear_static(const float* x, const void* w_packed, float* y,
                          int32_t M, int64_t n_out, int64_t k_in, void* stream);

/* ---------------------------------------------------------------------------
 * Optional per-kernel timing for benchmarks (the paper times with device events,
 * Sec. 4.1).  While enabled, every kernel launch of fdc_parallel_decode_step and
 * fdc_masked_attention is bracketed by two HIP events on the caller's stream.
 * fdc_profile_read waits for the recorded events, returns per kind the summed
 * milliseconds and the number of launches since the last read, and clears them.
 * masked_attention covers both of its kernels (partial + merge).
 */
#define FDC_PROF_KINDS 9
int32_t     fdc_profile_enable(fdc_ctx* ctx, int32_t on);
int32_t     fdc_profile_read(fdc_ctx* ctx, float* ms_sum /* host [FDC_PROF_KINDS] */,
                             int32_t* launches /* host [FDC_PROF_KINDS] */);
const char* fdc_profile_kind_name(int32_t kind);   /* NULL outside 0..FDC_PROF_KINDS-1 */

/* What an event pair adds to the launch it brackets: `rounds` times a kernel is
 * timed once and twice between two events on `stream`; the difference is one
 * launch (*null_us, may be NULL), the remainder of the single-launch time is the
 * cost of the pair (*overhead_us), which a benchmark subtracts from its
 * per-kernel event times.  The kernel is a copy of one half of `scratch` (device,
 * 256-byte aligned, caller-owned, contents destroyed) onto the other, or an
 * empty kernel when scratch is NULL.  Synchronises the stream.  Host pointers
 * for the results. */
int32_t fdc_profile_calibrate(int32_t rounds, void* scratch, size_t scratch_bytes, float* overhead_us,
                              float* null_us, void* stream);

/* Plain streaming copy of `bytes` (multiple of 16) between two device buffers
 * (16-byte aligned, not overlapping): the sustained-bandwidth reference of the
 * device, and the known-size kernel that hardware traffic counters are scaled by. */
int32_t fdc_stream_copy(void* dst, const void* src, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FDC_H */
