/* cascade_moe.h — C ABI of the MI355X (gfx950) MoE verification path and of the host-side
 * utility-driven choice of the speculation length K.
 *
 * What the device calls compute (paper: Section 1, Section 2.1, Section 2.2, Section 2.4):
 * one decode iteration of speculative decoding pushes T = K+1 tokens (one accepted, K drafted)
 * through every MoE layer; each token independently selects top_k of E experts, the layer has to
 * fetch the UNION of the selected experts, and the cost of the step is the HBM traffic for those
 * unique experts' weights.  Each call below is one step of that path.  The operator itself is the
 * usual one: bias-free linear router, top-k on the logits, gates = softmax over the selected
 * logits, expert = w2 . (silu(w1 x) * (w3 x)), optional always-on shared experts with gate 1.
 *
 * What the host calls compute (paper: Section 4, Definition of speculation utility, Eq. 3 and
 * Theorem 1; Section 5.3 test-and-set; 5.4 disabling speculation; 5.5 adaptive back-off; 5.6
 * hill-climbing search; Section 6 hyper-parameters).
 *
 * Conventions
 *  - C11, no C++ types, no exceptions; every call returns a moe_status (or a plain value).
 *  - "DEVICE" pointers are HIP device pointers owned by the caller; "HOST" pointers are ordinary
 *    host memory.  bf16 tensors are passed as uint16_t bit patterns (FP8 tensors as bytes),
 *    row-major and dense unless a call says otherwise.
 *  - Device calls only ENQUEUE work on `stream` (a hipStream_t passed as void*, NULL = the default
 *    stream).  They never synchronise, never copy to the host and never allocate; outputs are
 *    valid once the caller has synchronised the stream.  Argument validation is synchronous.
 *  - A moe_ctx owns the device workspace for one layer geometry.  It is not thread-safe: use one
 *    ctx per stream, and do not overlap calls on the same ctx from different streams.
 *  - The library never falls back to the CPU: without a usable GPU every device call fails with
 *    MOE_ERR_HIP.
 *  - The library reads no environment variable.  Two families of calls are aids and not part of the
 *    path, and are the only exceptions to the rules above: moe_ctx_tune changes the launch plan of one
 *    context (tuning and tests; the plan moe_plan_query reports is the automatic one), and while
 *    moe_ctx_profile is switched on every layer-step creates HIP event objects (host-side allocations)
 *    and records them between its kernels, which moe_ctx_profile_read waits for and frees.
 */
#ifndef CASCADE_MOE_H
#define CASCADE_MOE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MOE_OK = 0,
  MOE_ERR_INVALID_ARG = -1,       /* NULL required pointer, T out of range, bad enum, ...        */
  MOE_ERR_UNSUPPORTED_SHAPE = -2, /* geometry outside what the kernels are built for             */
  MOE_ERR_WORKSPACE = -3,         /* device workspace could not be allocated                     */
  MOE_ERR_HIP = -4,               /* a HIP runtime call or kernel launch failed                  */
  MOE_ERR_UNIMPLEMENTED = -5      /* kept for ABI stability: no call returns it at present         */
} moe_status;

/* Static description of a status code; never freed. */
const char* moe_strerror(moe_status s);
int moe_abi_version(void);

/* Geometry of one MoE layer (paper: Table 1 lists the shapes the method was evaluated on).
 * Supported: d % 32 == 0, ffn % 32 == 0, 1 <= top_k <= min(n_experts, 16), n_experts <= 256,
 * 0 <= n_shared <= 8, 1 <= max_tokens <= 16 (T = K+1 tokens in flight, K <= 15); attention stub either absent
 * (n_heads = n_kv_heads = head_dim = 0) or n_heads % n_kv_heads == 0, head_dim in {32, 64, 96, 128}. */
typedef struct {
  int32_t d;          /* hidden size                                   */
  int32_t ffn;        /* expert intermediate size                      */
  int32_t n_experts;  /* E, routed experts                             */
  int32_t top_k;      /* experts selected per token                    */
  int32_t n_shared;   /* always-on shared experts (same ffn), may be 0 */
  int32_t max_tokens; /* largest T that will be passed                 */
  int32_t gate_mode;  /* MOE_GATE_*: how the picked experts are weighted */
  int32_t n_heads;    /* attention stub (moe_decoder_stack only): query heads, 0 = no attention workspace */
  int32_t n_kv_heads; /*   key/value heads, divides n_heads                                              */
  int32_t head_dim;   /*   multiple of 32, <= 128                                                        */
} moe_shape;

/* Weighting of a token's top_k picks (the selection itself — top_k largest logits, ties to the lower
 * index — is the same).  The paper's Table 1 families differ in this and the paper does not say:
 * MOE_GATE_RENORM_TOPK: softmax over the top_k selected logits (gates sum to 1);
 * MOE_GATE_SOFTMAX_ALL: softmax over all E logits, the picks' probabilities used as they are
 *                       (gates sum to less than 1). */
enum { MOE_GATE_RENORM_TOPK = 0, MOE_GATE_SOFTMAX_ALL = 1 };

typedef struct moe_ctx moe_ctx; /* opaque: shape + device workspace */

/* Create / destroy a context on the CURRENT HIP device.  The only calls that allocate or free
 * device memory.  *out is set to NULL on failure. */
moe_status moe_ctx_create(const moe_shape* shape, moe_ctx** out);
moe_status moe_ctx_destroy(moe_ctx* ctx);
/* Bytes of device workspace held by the context. */
int64_t moe_ctx_workspace_bytes(const moe_ctx* ctx);

/* Tuning aid: override parts of the launch plan of THIS context for all later calls (what moe_plan_query
 * describes; the kernels and their results per element are the same, only the split of the work changes).
 *   gu_tiles, dn_tiles  0 = automatic, or 1, 2, 4 (gu_tiles is honoured for row-major bf16 weights and, as
 *                       1 or 2 tile pairs per wavefront, for tiled FP8 weights with T <= 8; the other gate/up
 *                       kernels have one fixed shape)
 *   dn_split_k          0 = automatic, or a power of two <= 16; clamped to what the shape allows and to the
 *                       largest split the workspace was sized for at creation
 *   fused_down          -1 = automatic (few tokens in flight), 0 = never fuse the down projection with the
 *                       combine, 1 = always (tiled weights)
 * Host only, no device work.  MOE_ERR_INVALID_ARG for any other value. */
moe_status moe_ctx_tune(moe_ctx* ctx, int32_t gu_tiles, int32_t dn_tiles, int32_t dn_split_k, int32_t fused_down);

/* Step 1 — router logits, top-k, gates, and the union of activated experts (Section 2.1: a small
 * gating network selects a few experts per token; Section 1 / 2.2: the in-flight tokens together
 * activate a larger set of experts).
 *   logit[t,e] = sum_j hidden[t,j] * router_w[e,j], accumulated in fp64 (products are exact there)
 *   ids[t,0..top_k)   the top_k largest logits of token t in descending order; equal -> lower e
 *   gates[t,i]        softmax over the selected logits (fp32), sums to 1 per token; or, with
 *                     MOE_GATE_SOFTMAX_ALL, softmax over all E logits read at the picks
 *   unique_experts[E] ascending distinct ids in the first *n_unique entries, -1 after them
 * hidden [T,d] fp32, router_w [E,d] bf16: DEVICE, read-only.  ids [T,top_k] int32, gates
 * [T,top_k] fp32, unique_experts [E] int32, n_unique [1] int32: DEVICE outputs; any of the four
 * may be NULL if not wanted.  1 <= T <= shape.max_tokens. */
moe_status moe_route(moe_ctx* ctx, const float* hidden, const uint16_t* router_w, int32_t T,
                     int32_t* ids, float* gates, int32_t* unique_experts, int32_t* n_unique, void* stream);

/* Step 2 — per-expert token lists for a given routing (Section 2.2 / 2.4: the set of unique
 * experts is what must be fetched; tokens are grouped so each unique expert is visited once).
 *   expert_count[e]   number of (token, slot) pairs routed to e
 *   expert_offset[e]  exclusive prefix sum of expert_count, expert_offset[E] = T*top_k
 *   assign[..]        flat pair indices a = t*top_k + i grouped by expert (ascending e), ascending
 *                     a inside each group
 * ids [T,top_k]: DEVICE input, every id in [0,E) and the top_k ids of one token distinct (as
 * moe_route produces them; a repeated id inside a token is counted once).  unique_experts [E],
 * n_unique [1], expert_count [E], expert_offset [E+1], assign [T*top_k]: DEVICE int32 outputs, each
 * may be NULL. */
moe_status moe_group(moe_ctx* ctx, const int32_t* ids, int32_t T, int32_t* unique_experts, int32_t* n_unique,
                     int32_t* expert_count, int32_t* expert_offset, int32_t* assign, void* stream);

/* Storage order of the expert matrices (the router is always row-major).
 * MOE_LAYOUT_ROW_MAJOR: dense row-major as listed below.
 * MOE_LAYOUT_TILED:     same bytes, re-ordered once by moe_pack_weights so that the block of 16 rows
 *                       a wavefront consumes per step is 1 KB of contiguous memory.
 *                       bf16: block (i, s) = rows 16i..16i+15, columns 32s..32s+31 at block index
 *                       i*(K/32)+s; inside a block, 16-byte unit l = r + 16*g holds row 16i+r, columns
 *                       32s+8g..32s+8g+7.
 *                       FP8: block (i, p) = rows 16i..16i+15, columns 64p..64p+63 at block index
 *                       i*(K/64)+p; unit l = r + 16*g holds row 16i+r, columns 64p+8g..64p+8g+7
 *                       followed by columns 64p+32+8g..64p+32+8g+7.
 *                       Per-matrix and per-expert sizes are unchanged. */
enum { MOE_LAYOUT_ROW_MAJOR = 0, MOE_LAYOUT_TILED = 1 };

/* Element type of the expert matrices (Table 1 of the paper lists bf16/fp16 and FP8 checkpoints;
 * Section 6.1: quantised models).  The paper does not define the FP8 scheme; the one built here:
 * MOE_WEIGHT_FP8_E4M3: one byte per weight, E4M3 (1 sign, 4 exponent bits biased by 7, 3 mantissa
 *                      bits, no infinities, S.1111.111 = NaN, largest finite value 448), and one fp32
 *                      scale per OUTPUT channel (matrix row): weight = scale[row] * value(code).
 *                      Activations, accumulation and the router are as for bf16.  d and ffn must be
 *                      multiples of 64.  Both layouts are accepted; the TILED one is the one that
 *                      streams at speed (row-major FP8 is read in 8-byte row pieces: pack first). */
enum { MOE_WEIGHT_BF16 = 0, MOE_WEIGHT_FP8_E4M3 = 1 };

/* One layer's weights: DEVICE pointers, caller-owned, alive until the stream drains.
 * sw1/sw3/sw2 (and their scales) are required iff shape.n_shared > 0.  The scale pointers are read
 * only for MOE_WEIGHT_FP8_E4M3 and are always plain row-major fp32.  Every pointer must be 16-byte
 * aligned. */
typedef struct {
  const uint16_t* router_w; /* [E, d] bf16                               */
  const void* w1;           /* [E, ffn, d]  gate   bf16 or FP8 codes      */
  const void* w3;           /* [E, ffn, d]  up                            */
  const void* w2;           /* [E, d, ffn]  down                          */
  const void* sw1;          /* [n_shared, ffn, d]                         */
  const void* sw3;          /* [n_shared, ffn, d]                         */
  const void* sw2;          /* [n_shared, d, ffn]                         */
  int32_t layout;           /* MOE_LAYOUT_* of w1, w3, w2, sw1, sw3, sw2  */
  int32_t dtype;            /* MOE_WEIGHT_* of w1, w3, w2, sw1, sw3, sw2  */
  const float* w1_scale;    /* [E, ffn]        FP8 only                   */
  const float* w3_scale;    /* [E, ffn]                                   */
  const float* w2_scale;    /* [E, d]                                     */
  const float* sw1_scale;   /* [n_shared, ffn]                            */
  const float* sw3_scale;   /* [n_shared, ffn]                            */
  const float* sw2_scale;   /* [n_shared, d]                              */
} moe_layer_weights;

/* One-off static re-layout of a layer's expert weights for streaming (weights do not change while
 * serving, so this runs once at load time, outside the path the paper's Section 2.4 cost is about).
 * src: row-major weights.  dst: HOST struct whose DEVICE pointers the caller has set to buffers of
 * the same sizes as src's (dst->router_w may equal src->router_w; otherwise the router is copied).
 * On success dst->layout is set to MOE_LAYOUT_TILED, dst->dtype to src->dtype and the scale
 * pointers of dst to those of src (scales are not re-ordered).  Enqueues on `stream`; src and dst
 * buffers must not overlap. */
moe_status moe_pack_weights(moe_ctx* ctx, const moe_layer_weights* src, moe_layer_weights* dst, void* stream);

/* Steps 1-5 — the whole verification step of one MoE layer (Section 2.2: the target model
 * verifies all K+1 tokens in one step; Section 2.4: expert-layer latency follows the number of
 * unique experts).  Route, group, then for every UNIQUE expert stream w1/w3/w2 from HBM once and
 * apply it to the tokens routed to it, and combine:
 *   out[t] = sum_i gates[t,i] * FFN_{ids[t,i]}(hidden[t])  +  sum_s FFN_shared_s(hidden[t])
 * with fp32 accumulation.  Row t of `out` equals what a T = 1 call on hidden[t] alone gives
 * (verification is iso-accuracy) up to fp32 summation order.
 * hidden [T,d] fp32 DEVICE in; out [T,d] fp32 DEVICE out.  ids_opt [T,top_k], gates_opt
 * [T,top_k], unique_opt [E], n_unique_opt [1]: optional DEVICE outputs (NULL = not wanted). */
moe_status moe_verify_layer(moe_ctx* ctx, const moe_layer_weights* w, const float* hidden, int32_t T, float* out,
                            int32_t* ids_opt, float* gates_opt, int32_t* unique_opt, int32_t* n_unique_opt,
                            void* stream);

/* moe_verify_layer for callers that cannot allocate device memory and cannot hold a moe_ctx that did: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same computation, same kernels and
 * launch plan, same results as moe_verify_layer on a fresh context of `shape`, but the workspace is a fixed
 * 32 MiB array inside the library's device code (every GPU the library runs on holds it until the process ends),
 * and the call itself allocates nothing: no hipMalloc / hipFree, no event objects, no allocating library routine.
 *   - The geometry's workspace (that of a context of `shape`, less the extra copies of the routing tables that
 *     only moe_verify_stack uses; 12 MiB for the Mixtral-8x7B-shaped layer at max_tokens 9, under 23 MiB for every
 *     Table 1 shape at max_tokens 16) must fit the array; a geometry that needs more returns MOE_ERR_WORKSPACE and
 *     launches nothing.
 *   - All calls on one GPU share that GPU's array, which keeps the last call's contents; each call first clears
 *     the part a layer-step reads before writing (a small fill kernel on `stream`).  Calls that overlap on one GPU
 *     — from different streams or threads — race: serialise them.  The array's device address is looked up on the
 *     first call on each device, which must therefore not happen inside a stream capture.
 * shape: HOST; every other argument as for moe_verify_layer.  moe_ctx_tune / moe_ctx_profile do not apply. */
moe_status moe_verify_layer_noalloc(const moe_shape* shape, const moe_layer_weights* w, const float* hidden, int32_t T,
                                    float* out, int32_t* ids_opt, float* gates_opt, int32_t* unique_opt,
                                    int32_t* n_unique_opt, void* stream);

/* L layers back to back on one stream without host synchronisation: layer l reads hidden[l] and
 * writes out[l] (independent per-layer inputs; the method's cost model — Section 2.4: the bytes of the unique
 * experts of every layer — needs no chaining).  Because no layer's input depends on another layer's output, the
 * call routes up to 16 layers ahead in one pair of launches and lets the slab sum of one layer ride in the next
 * layer's gate/up launch: two launches per layer-step.  The results are those of L moe_verify_layer calls, bit for
 * bit wherever both pick the same down-projection plan (a slab sum that costs no launch moves the point where the
 * fused down + combine kernel stops paying, so a step may differ in the order of that sum).
 * A decoder cannot be run this way (its layer l + 1 reads what layer l wrote): see moe_chained_stack and
 * moe_decoder_stack, which pay the router's launch in every layer.
 * layers: HOST array of L structs (copied during the call).  hidden, out: DEVICE [L,T,d].
 * n_unique_per_layer_opt: DEVICE [L] int32 or NULL. */
moe_status moe_verify_stack(moe_ctx* ctx, const moe_layer_weights* layers, int32_t L, const float* hidden,
                            int32_t T, float* out, int32_t* n_unique_per_layer_opt, void* stream);

/* L pre-norm residual MoE blocks back to back on one stream, each feeding the next (the alternative to
 * independent per-layer inputs; Table 1's model families are built from such blocks, and Section 2.2's
 * verification step runs all of them for the K+1 tokens):
 *   x_{l+1} = x_l + MoE_l( RMSNorm(x_l) * gamma_l ),   RMSNorm(x)_j = x_j / sqrt( mean_j x_j^2 + eps )
 * with the MoE layer exactly as in moe_verify_layer.  The sum over a token's picks, the residual add and
 * the next block's normalisation run in one kernel; the residual stream stays fp32.
 * layers: HOST array of L structs (copied during the call).  gammas: HOST array of L DEVICE pointers to
 * bf16 [d], 16-byte aligned.  x_in, x_out: DEVICE [T,d] fp32 (x_out = x_L; may equal x_in).
 * trace_opt: DEVICE [L,T,d] fp32 or NULL; receives x_l, the stream entering block l (trace[0] = x_in).
 * n_unique_per_layer_opt: DEVICE [L] int32 or NULL.  L = 1 is a single block.  Needs d <= 16384. */
moe_status moe_chained_stack(moe_ctx* ctx, const moe_layer_weights* layers, const uint16_t* const* gammas, int32_t L,
                             const float* x_in, int32_t T, float eps, float* x_out, float* trace_opt,
                             int32_t* n_unique_per_layer_opt, void* stream);

/* Attention stub of a decoder block (moe_decoder_stack).  The paper needs attention only as the share of an
 * iteration that does not grow with K (Section 2.4); the stub streams the attention block's weights and does
 * the smallest thing that is still attention: causal grouped-query self-attention among the T in-flight
 * tokens (no cache of earlier context, no rotation, no biases).  DEVICE pointers, bf16, 16-byte aligned;
 * wqkv and wo in the TILED layout (moe_pack_matrix); geometry as in the moe_shape of the context. */
typedef struct {
  const uint16_t* wqkv;       /* [(H + 2 Hkv) dh, d]: rows of the query heads, then key heads, then value heads */
  const uint16_t* wo;         /* [d, H dh]                                                                       */
  const uint16_t* gamma_attn; /* [d] RMSNorm weight in front of the attention half                               */
  const uint16_t* gamma_moe;  /* [d] RMSNorm weight in front of the MoE half                                     */
} moe_attn_weights;

/* Re-order one row-major [rows, K] matrix (rows % 16 == 0; K % 32 == 0 for bf16, % 64 for FP8) into the TILED
 * layout described at MOE_LAYOUT_TILED.  src, dst: DEVICE, same size, not overlapping.  dtype: MOE_WEIGHT_*. */
moe_status moe_pack_matrix(moe_ctx* ctx, const void* src, void* dst, int64_t rows, int32_t K, int32_t dtype,
                           void* stream);

/* L decoder blocks back to back, each feeding the next:
 *   h       = x_l + Wo . Attn( Wqkv . (RMSNorm(x_l) * gamma_attn) )         attention stub, see moe_attn_weights
 *   x_{l+1} = h   + MoE_l( RMSNorm(h) * gamma_moe )                          as in moe_chained_stack
 * Arguments as for moe_chained_stack, with attn: HOST array of L structs.  The context must have been created
 * with the attention geometry in its moe_shape (n_heads > 0). */
moe_status moe_decoder_stack(moe_ctx* ctx, const moe_layer_weights* layers, const moe_attn_weights* attn, int32_t L,
                             const float* x_in, int32_t T, float eps, float* x_out, float* trace_opt,
                             int32_t* n_unique_per_layer_opt, void* stream);

/* Measurement aid: per-kernel timing.  While enabled, every layer of moe_verify_layer /
 * moe_verify_stack (and the MoE half of every block of the chained calls, whose slab sum is then
 * counted with the next block and reads as zero here) records HIP events on its stream around each
 * of its four stages (route with the expert-union step, gate/up, down, combine); this adds event
 * packets between the kernels, so whole-step latency is measured with profiling OFF.
 * moe_ctx_profile_read waits for the recorded events, adds the elapsed times into ms_sum[0..3]
 * (HOST, milliseconds, same stage order), stores the number of layer-steps in *steps (HOST) and
 * forgets the events.  Both calls may allocate/free event objects. */
moe_status moe_ctx_profile(moe_ctx* ctx, int32_t enable);
moe_status moe_ctx_profile_read(moe_ctx* ctx, double* ms_sum, int64_t* steps);

/* Measurement aid: read `bytes` (multiple of 16) of DEVICE memory at `src` once with contiguous
 * non-temporal 128-bit loads (each wavefront streams its own chunk, the wavefronts starting at staggered
 * offsets of their chunks and wrapping around) and fold them into `sink` (DEVICE,
 * >= 4096 words).  Used only to report the box's achievable read-stream bandwidth next to the
 * published HBM peak. */
moe_status moe_stream_read_probe(const void* src, int64_t bytes, float* sink, void* stream);

/* Measurement aid: the weight loads of the tiled bf16 gate/up kernel and nothing else — the same grid (`tiles` x
 * `slots` wavefronts), each streaming the tile row of matrix a and the tile row of matrix b (`steps` contiguous
 * 1 KB blocks each, `slot_stride` bytes from one slot's matrix to the next) with the same non-temporal 128-bit
 * loads at the same software-pipeline depth, folding the words into `sink` (DEVICE, >= 4096 words) instead of
 * feeding matrix-core instructions.  What it takes is the cost of the bytes alone on this access pattern: the
 * difference to the real kernel bounds what any other arithmetic formulation of the step (wavefront dot products
 * instead of matrix cores) could gain.  a, b: DEVICE, 16-byte aligned, each at least slots*slot_stride bytes. */
moe_status moe_weight_load_twin(const void* a, const void* b, int32_t slots, int32_t tiles, int32_t steps,
                                int64_t slot_stride, float* sink, void* stream);

/* The launch plan moe_verify_layer would use for T tokens in flight on a layer of this shape, layout
 * (MOE_LAYOUT_*) and weight type (MOE_WEIGHT_*).  Pure host arithmetic (no device, no context): the plan
 * depends only on its arguments, because the union of experts the T tokens form (Section 2.4) is known on
 * the device only and the grids are sized for the largest union they could form.
 *   routed_slots     expert slots the grids cover besides the shared experts: min(n_experts, T*top_k)
 *   expected_slots   live slots expected under uniform routing, shared experts included (balls into bins)
 *   wide_router      1: logits over (token, 16 experts) workgroups + one top-k/grouping workgroup; 0: one workgroup
 *                    per token (+ a grouping launch when T > 1)
 *   packed_fragments 1: T <= 8, the bf16 hi and lo halves of the activations share one MFMA operand
 *   gu_tiles         16-row tile pairs of w1/w3 per wavefront in the gate/up kernel
 *   dn_tiles         16-row tiles of w2 per wavefront in the down kernel
 *   dn_split_k       k-chunks of the down projection across workgroups (slabs per slot)
 *   dn_fused_chunks  > 0: down projection and combine run as one launch with this many k-chunks per slot
 *                    (few tokens in flight); dn_tiles / dn_split_k are then unused
 *   launches         kernel launches of one moe_verify_layer call
 * Errors: MOE_ERR_INVALID_ARG for NULL pointers, T outside 1..max_tokens or unknown layout / dtype;
 * MOE_ERR_UNSUPPORTED_SHAPE as moe_ctx_create, and for FP8 when d or ffn is not a multiple of 64. */
typedef struct {
  int32_t routed_slots, wide_router, packed_fragments, gu_tiles, dn_tiles, dn_split_k, dn_fused_chunks, launches;
  double expected_slots;
} moe_plan_info;
moe_status moe_plan_query(const moe_shape* shape, int32_t T, int32_t layout, int32_t dtype, moe_plan_info* out);

/* ----------------------------------------------------------------------------------------
 * Host side — pure C, no device.
 * -------------------------------------------------------------------------------------- */

/* Speculation utility (Section 4, Definition and Eq. 3): benefit / cost with benefit = tokens
 * emitted per iteration (ETR, counts the always-emitted token, so 1 without speculation) and
 * cost = t_verify / t_base.  By Theorem 1, time per output token = t_base / utility.
 * Returns NaN if t_verify <= 0 or t_base <= 0 (or either is NaN). */
double cascade_utility(double tokens_per_iter, double t_verify, double t_base);

/* Hyper-parameters of the test-and-set policy (Section 5.3 and Section 6: t = 4, up to M = 4
 * trials, S = 16; Section 7.4: K_start = 3; Section 5.3: baseline from the first 4 iterations,
 * refreshed about every 100).  cascade_default_params fills the paper's values. */
typedef struct {
  int32_t t_trial;      /* iterations per trial                                  (4)   */
  int32_t max_trials;   /* M, trials per test phase                              (4)   */
  int32_t s_set;        /* S, set-phase length                                   (16)  */
  int32_t k_max;        /* largest K ever proposed                               (8)   */
  int32_t k_start;      /* K of a request's first trial                          (3)   */
  int32_t base_iters;   /* no-speculation iterations that measure t_base         (4)   */
  int32_t base_refresh; /* re-measure t_base after about this many iterations    (100) */
  int32_t s_max;        /* cap on the backed-off set length, 0 = uncapped        (0)   */
  double converge_frac; /* early exit when successive utilities differ by less   (0.10)*/
  int32_t backoff;      /* adaptive back-off (Section 5.5): 0 off; 1 the first disabled set phase keeps S and every
                           further consecutive one doubles (utility "persistently" below 1, as the section's
                           figure puts it); 2 every drop to K = 0 doubles S, the first included (the section's
                           sentence taken literally)                             (1)   */
  int32_t hillclimb;    /* 1 = hill-climbing search (Section 5.6) on             (1)   */
} cascade_params;
void cascade_default_params(cascade_params* p);

typedef struct cascade_ctrl cascade_ctrl; /* per-request controller state, HOST */
cascade_ctrl* cascade_ctrl_create(const cascade_params* p); /* NULL on bad parameters; p == NULL -> defaults */
void cascade_ctrl_destroy(cascade_ctrl* c);

/* K to use for the coming iteration, 0 (speculation off) .. k_max.  Does not change state. */
int32_t cascade_next_k(const cascade_ctrl* c);
/* Report one finished iteration: the K that was used (must equal cascade_next_k), the tokens it
 * emitted (1 .. k_used+1, Section 2.2) and its duration (> 0, any unit, consistent across calls).
 * MOE_ERR_INVALID_ARG leaves the state unchanged. */
moe_status cascade_observe(cascade_ctrl* c, int32_t k_used, int32_t tokens_emitted, double t_iter);

/* Read-only view of the controller for logging. */
typedef struct {
  int32_t phase;         /* 0 baseline measurement, 1 test, 2 set */
  int32_t cur_k;         /* same as cascade_next_k                */
  int32_t s_cur;         /* current (backed-off) set-phase length */
  int32_t trials_done;   /* trials finished in the current test phase */
  int64_t iters;         /* iterations observed so far            */
  int64_t trial_iters;   /* of which inside test phases           */
  double t_base;         /* current no-speculation iteration time (NaN before it is known) */
  double last_utility;   /* utility of the last finished trial or speculative set phase (NaN if none) */
} cascade_state;
void cascade_get_state(const cascade_ctrl* c, cascade_state* out);

#ifdef __cplusplus
}
#endif
#endif /* CASCADE_MOE_H */
