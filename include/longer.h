/*
 * longer.h -- C ABI of the MI355X (gfx950) LONGER forward / KV-cache serving library.
 *
 * The library computes the data-parallel forward pass of the LONGER long-sequence
 * stack (arXiv 2505.04421): token merge with an InnerTrans block (Section 3.4), the
 * hybrid attention of Section 3.5 (one cross-causal layer whose queries are the global
 * tokens plus the k most recent merged tokens, Eq. 5-8, followed by N self-causal layers,
 * Eq. 9-10) and the two-stage KV-cache serving path of Section 3.6.3.
 *
 * Conventions (all entry points)
 *   - every tensor pointer is a DEVICE pointer owned by the caller, 16-byte aligned for the
 *     activations (H, G, M, X, Y, G_cand, Yg); the config and weight structs themselves live in
 *     HOST memory and hold device pointers;
 *   - tensors are dense row-major; weights are stored [in, out] so that y = x W + b, the
 *     way Eq. 6 writes Q = O W_Q; element type is `dtype` of the config (fp32 or bf16)
 *     for every activation, weight, bias and LayerNorm vector; logits are always fp32;
 *     arithmetic: fp32 accumulation, residual stream, LayerNorm and softmax in both modes; in
 *     bf16 mode the matrix-core operands are bf16, except in the second FFN GEMM, whose
 *     activated hidden values and weights are fp16 (W2 is converted when it is packed; exact
 *     for 1.6e-5 <= |w| < 16376), and GELU is a polynomial evaluated in fp16;
 *   - `lens` is int32 [B] raw (un-merged) valid lengths, or NULL for "all L"; sequences are
 *     stored oldest-first and right-padded; padded values are never read into the result
 *     (they may hold NaN);
 *   - `ws` is caller-supplied device scratch of at least longer_workspace_bytes()
 *     (256-byte aligned); the library allocates nothing, enqueues all work on `stream`
 *     (a hipStream_t passed as void*, NULL = the default stream) and does not synchronise;
 *     calls that share a workspace must be ordered on one stream;
 *   - return value: 0 on success; LONGER_ERR_ARG for a null pointer / unsupported shape /
 *     bad enum; LONGER_ERR_WS when the workspace is too small; LONGER_ERR_HIP when a HIP
 *     call failed.  Nothing throws.  longer_last_error() gives a thread-local message.
 *   - rows of invalid tokens (padded raw tokens, merged tokens past T_u = ceil(len/K),
 *     recent-query slots with a negative merged index) are written as exact zeros.
 *
 * Supported shapes, as (width, head width = width / heads): bf16 (32, 16), (64, 16), (64, 32),
 * (128, 16), (128, 32), (256, 16), (256, 32); fp32 (32, 16), (64, 16), (128, 16) (the last as a check of the headline
 * width without bf16 rounding: one workgroup per compute unit, the reduced stack one launch pair per layer).  The pair is checked for the main stack (d, d / heads) and
 * for the InnerTrans blocks (their width, that width / inner_heads) separately; with
 * LONGER_MERGE_CONCAT the InnerTrans width is d / K.  K and m must divide 32 (K for the merge,
 * m for candidate scoring); the FFN hidden width is ffn_mult * width with (9 + ffn_mult) * width
 * fp32 values fitting one 32-row weight segment (ffn_mult <= 7 in bf16, <= 23 in fp32).
 * Anything else returns LONGER_ERR_ARG, and so does a call with B * ceil(L / K) * K >= 2^31 - 256
 * raw token slots (the merge kernel indexes them in 32 bits; split the batch).
 *
 * Mask (Eq. 8, applied by token type on chronologically stored data): a sequence query
 * sees sequence keys that are not newer than itself and never a global key; a global
 * query sees every valid sequence key and, for LONGER_GMASK_FULL, every global key of
 * its own set, for LONGER_GMASK_CAUSAL (Eq. 8 read literally) only globals with an
 * index >= its own.
 */
#ifndef LONGER_H_
#define LONGER_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LONGER_OK        0
#define LONGER_ERR_ARG  -1
#define LONGER_ERR_WS   -2
#define LONGER_ERR_HIP  -3

typedef enum { LONGER_F32 = 0, LONGER_BF16 = 1 } longer_dtype;
typedef enum { LONGER_GMASK_FULL = 0, LONGER_GMASK_CAUSAL = 1 } longer_gmask;
typedef enum { LONGER_ACT_GELU_ERF = 0, LONGER_ACT_RELU = 1 } longer_act;
/* How the K InnerTrans outputs of a group become one merged token (Section 3.4):
 *   LONGER_MERGE_MEAN    raw tokens, InnerTrans blocks and the main stack all have width d;
 *                        the merged token is the mean over the group's valid tokens;
 *   LONGER_MERGE_CONCAT  the paper's concatenation (merged width K d_raw, the width Eq. 4
 *                        counts): raw tokens H and the InnerTrans blocks have width d / K,
 *                        the merged token is the group's K outputs side by side, oldest
 *                        first, zeros in the slots of padded tokens; the main stack runs
 *                        at width d.  Needs d / K to be a supported width. */
typedef enum { LONGER_MERGE_MEAN = 0, LONGER_MERGE_CONCAT = 1 } longer_merge;

/* Model shape.  Names follow the paper: d width, m global tokens (Section 3.3), K merge
 * group size (Section 3.4), k_recent sampled recent queries (Eq. 5), n_self = N stacked
 * self-attention layers (Eq. 10). */
typedef struct {
  int32_t d, heads, ffn_mult;
  int32_t m, K, k_recent, n_self;
  int32_t inner_layers, inner_heads;
  int32_t act;      /* longer_act   */
  int32_t gmask;    /* longer_gmask */
  float   ln_eps;
  int32_t dtype;    /* longer_dtype */
  int32_t merge;    /* longer_merge */
  int32_t k_uniform; /* query sampling (Section 3.5.1): 0 = the k_recent most recent merged tokens (Eq. 5
                        as evaluated); k_uniform > 0: the first k_uniform query slots hold uniformly
                        sampled older tokens (slot i the newest token of the i-th of k_uniform equal
                        shares of the tokens before the recent part), the other k_recent - k_uniform
                        slots the most recent ones; k_uniform = k_recent samples all slots uniformly.
                        A user with no more than k_recent merged tokens gets all of them either way. */
  const void* q_learn; /* learnable query tokens (Section 3.5.1, the third query strategy of the ablation):
                        NULL = the query slots are sampled from the sequence as above; else a DEVICE
                        pointer to [k_recent, d] values of `dtype`, 16-byte aligned, the same for every
                        user, that take the place of the sampled tokens in O (needs k_uniform = 0).  A
                        learnable slot is not a sequence position: in the first layer it sees every
                        valid merged token of the user (and, like all sequence-side rows, no global
                        token); in the self-causal layers slot i sees slots 0..i.  A user without any
                        token has no valid slot.  Every entry point that takes this config must be
                        given the same pointer (the serving calls and longer_self_attn_layer use it
                        only to tell which slots are valid). */
} longer_config;

/* One pre-LayerNorm transformer block: 12 d^2 + 13 d scalars for ffn_mult = 4 (Eq. 3).
 * ln*_g/ln*_b [d]; wq,wk,wv,wo [d,d]; bq,bk,bv,bo [d]; w1 [d, f]; b1 [f]; w2 [f, d];
 * b2 [d] with f = ffn_mult*d. */
typedef struct {
  const void *ln1_g, *ln1_b, *wq, *bq, *wk, *bk, *wv, *bv, *wo, *bo,
             *ln2_g, *ln2_b, *w1, *b1, *w2, *b2;
} longer_block;

typedef struct {
  const longer_block* inner;   /* host array [inner_layers] */
  const longer_block* cross;   /* host pointer to 1 block    */
  const longer_block* self;    /* host array [n_self]        */
  const void* head_w;          /* device [m*d], may be NULL when no logits are asked for */
  const void* head_b;          /* device [1]  */
  const void* packed;          /* NULL: every call re-packs the parameters it streams into its workspace (one
                                  small launch); else a DEVICE buffer that longer_pack_weights filled for the
                                  same config: the calls stream from it, launch no packing and read none of the
                                  other members */
} longer_weights;

/* Scratch needed by any entry point for a batch of B users (serving: U = B users, any
 * number of candidates) of padded raw length L. */
size_t longer_workspace_bytes(const longer_config* cfg, int B, int L);

/* Size of the opaque per-batch KV cache written by longer_kv_cache_build. */
size_t longer_kv_cache_bytes(const longer_config* cfg, int U, int L);

/* InnerTrans (Section 3.4, InnerTrans equation): cfg->inner_layers blocks applied inside
 * each group of K adjacent raw tokens, attention bidirectional inside the group, keys
 * masked by validity.  H [B, L, d] -> Z_out [B, T, K, d] with T = ceil(L / K)
 * (LONGER_MERGE_CONCAT: H [B, L, d / K] -> Z_out [B, T, K, d / K], inner blocks of width d / K). */
int longer_inner_transformer(const longer_config* cfg, const longer_block* inner, const void* H,
                             const int32_t* lens, int B, int L, void* Z_out,
                             void* ws, size_t ws_bytes, void* stream);

/* Token merge (Section 3.4): InnerTrans fused with the group gather and a mean over each
 * group's valid tokens.  H [B, L, d] -> M_out [B, T, d].
 * LONGER_MERGE_CONCAT: H [B, L, d / K] -> M_out [B, T, d], the group's outputs side by side. */
int longer_token_merge(const longer_config* cfg, const longer_block* inner, const void* H,
                       const int32_t* lens, int B, int L, void* M_out,
                       void* ws, size_t ws_bytes, void* stream);

/* First layer, cross-causal attention (Section 3.5.1-3.5.2, Eq. 5-8): queries
 * O = [G; M[T_u-k .. T_u-1]] over keys/values R = [G; M], then the FFN.
 * G [B, m, d], M [B, T, d], lens = raw lengths -> X_out [B, m+k, d] (globals first, then
 * the k recent slots, right-aligned). L is the padded raw length M was merged from. */
int longer_hybrid_cross_attn(const longer_config* cfg, const longer_block* cross, const void* G,
                             const void* M, const int32_t* lens, int B, int L, void* X_out,
                             void* ws, size_t ws_bytes, void* stream);

/* One self-causal layer over the reduced set (Section 3.5.3, Eq. 9).
 * X_in [B, m+k, d] -> X_out [B, m+k, d] (may not alias). */
int longer_self_attn_layer(const longer_config* cfg, const longer_block* blk, const void* X_in,
                           const int32_t* lens, int B, int L, void* X_out,
                           void* ws, size_t ws_bytes, void* stream);

/* The whole stack CrossAttn(O, R) -> SelfAttn x N (Eq. 10) after the token merge.
 * H [B, L, d] (LONGER_MERGE_CONCAT: [B, L, d / K]), G [B, m, d] -> Y_out [B, m+k, d]; logits_out [B] fp32 (or NULL):
 * logit = <head_w, flatten(Y[0:m])> + head_b. */
int longer_forward(const longer_config* cfg, const longer_weights* w, const void* H, const void* G,
                   const int32_t* lens, int B, int L, void* Y_out, float* logits_out,
                   void* ws, size_t ws_bytes, void* stream);

/* Serving stage 1 (Section 3.6.3): everything that depends on the user sequence only --
 * token merge, the sequence rows of every layer and their per-layer K/V -- written to
 * `cache` (longer_kv_cache_bytes, opaque layout, 256-byte aligned).  H [U, L, d]
 * (LONGER_MERGE_CONCAT: [U, L, d / K]). */
int longer_kv_cache_build(const longer_config* cfg, const longer_weights* w, const void* H,
                          const int32_t* lens, int U, int L, void* cache,
                          void* ws, size_t ws_bytes, void* stream);

/* Serving stage 2 (Section 3.6.3): every candidate's m global tokens run through the
 * 1 + N layers attending to their own globals and the cached sequence K/V.
 * G_cand [U, C, m, d] -> Yg_out [U, C, m, d] (or NULL) and logits_out [U, C] fp32.
 * `lens`, U and L must be those the cache was built with. */
int longer_score_candidates(const longer_config* cfg, const longer_weights* w, const void* cache,
                            const int32_t* lens, int U, int L, const void* G_cand, int C,
                            void* Yg_out, float* logits_out,
                            void* ws, size_t ws_bytes, void* stream);

/* Input generation (Section 3.5.1, "Input Generation"): the sequence-token representations
 * H = MLP([item embedding + learnable absolute positional embedding ; time-difference side
 * information]).  The paper fixes neither the widths nor the MLP; here the item and positional
 * embeddings have width d_e (a multiple of 32, 0 < d_e < d), the side information d - d_e, and
 * the MLP is d -> ffn_mult*d -> d with the config's activation:
 * E [B, L, d_e], pos [L, d_e] (indexed by position), tdiff [B, L, d - d_e]
 * -> H_out [B, L, d] = act([E + pos ; tdiff] w1 + b1) w2 + b2, w1 [d, f], w2 [f, d], f = ffn_mult*d.
 * Rows of padded tokens are written as zeros.  H_out is what longer_token_merge / longer_forward
 * take as H (merge mode LONGER_MERGE_MEAN). */
typedef struct { const void *pos, *w1, *b1, *w2, *b2; } longer_input_weights;
int longer_input_generation(const longer_config* cfg, const longer_input_weights* w, const void* E,
                            const void* tdiff, const int32_t* lens, int B, int L, int d_e,
                            void* H_out, void* ws, size_t ws_bytes, void* stream);

/* longer_forward on the raw inputs of the input-generation stage (Section 3.5.1 in front of
 * Section 3.4): H = MLP([E + pos ; tdiff]) is formed inside the token-merge kernel, in front of
 * the InnerTrans blocks, and never written to memory (it stays in fp32, where the two-call
 * sequence longer_input_generation + longer_forward rounds it to `dtype` in between).
 * Arguments as in longer_input_generation and longer_forward; merge mode LONGER_MERGE_MEAN only. */
int longer_forward_from_inputs(const longer_config* cfg, const longer_weights* w, const longer_input_weights* iw,
                               const void* E, const void* tdiff, int d_e, const void* G, const int32_t* lens,
                               int B, int L, void* Y_out, float* logits_out,
                               void* ws, size_t ws_bytes, void* stream);

/* longer_kv_cache_build on the raw inputs, in the same way (serving stage 1 of Section 3.6.3 with
 * the input generation of Section 3.5.1 inside its token-merge kernel). */
int longer_kv_cache_build_from_inputs(const longer_config* cfg, const longer_weights* w, const longer_input_weights* iw,
                                      const void* E, const void* tdiff, int d_e, const int32_t* lens, int U, int L,
                                      void* cache, void* ws, size_t ws_bytes, void* stream);

/* Packing once.  The kernels stream every block's parameters as matrix-core operand fragments in the
 * order they consume them (with the value bias folded into the output bias; in bf16 mode W1 and
 * b1 scaled by 1/4 and W2 by 4 in fp16).  By default each call derives that form from the raw
 * weights again, one launch of about 10 microseconds.  longer_pack_weights writes it once, for
 * every entry point that takes a longer_weights (forward, cache build, scoring; `iw` non-NULL adds
 * the input-generation MLP for the *_from_inputs calls, head_w / head_b non-NULL add the head),
 * into caller-owned device memory of longer_packed_weights_bytes(cfg) bytes, 256-byte aligned; a
 * longer_weights whose `packed` member points there then skips the packing launch.  The buffer
 * depends on the config (not on B, L or C) and must be re-packed when a weight changes.  The
 * library cannot check that a buffer it is handed was packed for the same config, with the head
 * or the input MLP a call needs: that is the caller's contract.  (An optimisation of the call
 * sequence, not an operation of the paper.) */
size_t longer_packed_weights_bytes(const longer_config* cfg);
int longer_pack_weights(const longer_config* cfg, const longer_weights* w, const longer_input_weights* iw,
                        void* packed_out, size_t bytes, void* stream);

/* longer_score_candidates for callers that cannot allocate or carry a workspace (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments without
 * `ws`, same results.  The packed parameters of the scoring launch go to a file-scope device
 * array of LONGER_STATIC_SCRATCH_BYTES inside the library (each GPU the library runs on holds its
 * own copy until the process ends; its address is looked up on the first call on a device, with
 * that device current, and the call must be made with the stream's device current).  A model
 * whose packed cross + self blocks and head exceed that size (d = 256 with ffn_mult = 4: more
 * than 1 + 4 layers) is rejected with LONGER_ERR_WS.  The call allocates nothing and calls no
 * allocating routine.  Every call on a GPU shares that GPU's array and overwrites it: calls that
 * overlap on one GPU (two streams, two threads) race; order them on one stream. */
#define LONGER_STATIC_SCRATCH_BYTES (8u << 20)
int longer_score_candidates_static(const longer_config* cfg, const longer_weights* w, const void* cache,
                                   const int32_t* lens, int U, int L, const void* G_cand, int C,
                                   void* Yg_out, float* logits_out, void* stream);

/* Thread-local text of the last error returned on this thread ("" if none). */
const char* longer_last_error(void);

/* Backward pass of the token merge (Section 3.4) under the training set-up of Section 3.6.2:
 * activation recomputation (nothing is kept from a forward call: the pass reads the raw tokens,
 * recomputes the chain of InnerTrans block inputs, then, block by block from the last to the
 * first, the block's intermediates) and mixed precision (bf16 matrix-core operands and stored
 * activations, fp32 accumulation, residual stream, LayerNorm / softmax statistics and parameter
 * gradients).  The function differentiated is longer_token_merge with exact-erf GELU (or ReLU); the
 * pass evaluates GELU and its derivative to 1.3e-3 absolute, below the bf16 step of the values it stores.
 *   H [B, L, w] raw tokens and the InnerTrans blocks `inner` as for longer_token_merge, in bf16
 *     (cfg->dtype must be LONGER_BF16); w = d, or d / K for LONGER_MERGE_CONCAT;
 *   dM [B, T, d] fp32: gradient of the loss (Eq. 2) with respect to the merged tokens; entries of
 *     merged tokens past T_u, and of the slots of padded tokens in a concatenated token, are ignored;
 *   dH_out [B, L, w] fp32: gradient with respect to the raw tokens, exact zeros for padded tokens;
 *   grads_out fp32 [inner_layers][longer_block_grad_floats(cfg)]: gradient of every parameter of every
 *     InnerTrans block, dense, in the order and with the shapes of the longer_block members
 *     (ln1_g [w], ln1_b [w], wq [w, w], bq [w], wk, bk, wv, bv, wo, bo, ln2_g, ln2_b, w1 [w, f], b1 [f],
 *     w2 [f, w], b2 [w], f = ffn_mult * w), summed over all users of the batch; overwritten, not
 *     accumulated into.
 * ws: device scratch of at least longer_backward_workspace_bytes(cfg, B, L), 256-byte aligned; all
 * pointers (parameters included) 16-byte aligned.  Supports head width 16 or 32, w one
 * of 32, 64, 128 or 256, f <= 2048.  A parameter gradient is a sum over the batch: slices of the
 * tokens are summed in a fixed order, the last step adds up to 64 such partial sums with fp32 atomics,
 * so the last bits may differ between two calls.  Same stream, error and ownership rules as the forward
 * entry points; both size queries return 0 for an unsupported configuration. */
size_t longer_backward_workspace_bytes(const longer_config* cfg, int B, int L);
size_t longer_block_grad_floats(const longer_config* cfg);
int longer_token_merge_backward(const longer_config* cfg, const longer_block* inner, const void* H,
                                const int32_t* lens, int B, int L, const float* dM,
                                float* dH_out, float* grads_out,
                                void* ws, size_t ws_bytes, void* stream);

/* Loss and gradients of the whole model (Section 3.6.2 applied to the forward pass of longer_forward):
 * token merge, cross-causal layer, N self-causal layers, the linear head on the global rows (Eq. 1) and
 * the binary cross-entropy of Eq. 2, mean over the B users of the batch.  Recomputation and precision
 * as for longer_token_merge_backward, applied selectively: the token merge (nine tenths of the
 * activations) keeps nothing and is recomputed, block by block, when its gradients are taken; the reduced
 * stack (B (m + k) query rows, B (m + T) key rows) keeps its layers' intermediates.
 *   H, G, lens, B, L as for longer_forward (bf16 only);
 *   labels [B] fp32 (0 or 1);
 *   loss_out [1] fp32; logits_out [B] fp32 or NULL;
 *   dH_out [B, L, w] fp32, dG_out [B, m, d] fp32: gradients of the loss with respect to the inputs;
 *   grads_out fp32 [longer_model_grad_floats(cfg)]: parameter gradients, dense, in this order: the
 *     InnerTrans blocks, the cross block, the self blocks (each block as for
 *     longer_token_merge_backward, at its own width), head_w [m d], head_b [1] (+ padding to a multiple
 *     of 4 floats), and, when cfg->q_learn is set, the learnable query tokens [k_recent, d].
 * ws: at least longer_forward_backward_workspace_bytes(cfg, B, L). */
size_t longer_model_grad_floats(const longer_config* cfg);
size_t longer_forward_backward_workspace_bytes(const longer_config* cfg, int B, int L);
int longer_forward_backward(const longer_config* cfg, const longer_weights* w, const void* H, const void* G,
                            const int32_t* lens, int B, int L, const float* labels,
                            float* loss_out, float* logits_out, float* dH_out, float* dG_out, float* grads_out,
                            void* ws, size_t ws_bytes, void* stream);

/* Gradients of the input-generation stage (Section 3.5.1, Input Generation, under the mixed
 * precision training of Section 3.6.2): for H = act([E + pos ; tdiff] w1 + b1) w2 + b2 on the valid
 * tokens and an upstream gradient dH [B, L, d] (fp32, device; what longer_forward_backward
 * writes to dH_out), the call writes dE_out [B, L, d_e], dtdiff_out [B, L, d - d_e] (fp32, exact
 * zeros at padded tokens) and grads_out, longer_input_grad_floats(cfg, L, d_e) fp32 values in the
 * order pos [L, d_e] | w1 [d, f] | b1 [f] | w2 [f, d] | b2 [d] (f = ffn_mult d; overwritten, not
 * accumulated; the positional embedding's row p sums over the users whose sequence reaches p).
 * The hidden layer is recomputed from E and tdiff (bf16 operands, fp32 accumulation, as in the
 * forward call; GELU and its derivative to 1.3e-3 absolute, as in longer_token_merge_backward); padded tokens are neither read nor written beyond those zeros.
 * cfg: dtype LONGER_BF16, merge LONGER_MERGE_MEAN, d a multiple of 32 (at most 512), f at most
 * 2048, d_e a multiple of 32 below d.  E, tdiff, w: device, bf16, as for longer_input_generation;
 * lens: device int32 [B] or NULL.  ws: device, 256-byte aligned, at least
 * longer_input_backward_workspace_bytes(cfg, B, L, d_e) bytes (0 = unsupported configuration).
 * Nothing is allocated; every launch goes to `stream`; parameter gradients add their last partial
 * sums with fp32 atomics as in longer_token_merge_backward (last-bit differences from run to run).
 * Errors: LONGER_ERR_ARG (shape, alignment, NULL), LONGER_ERR_WS, LONGER_ERR_HIP. */
size_t longer_input_backward_workspace_bytes(const longer_config* cfg, int B, int L, int d_e);
size_t longer_input_grad_floats(const longer_config* cfg, int L, int d_e);
int longer_input_generation_backward(const longer_config* cfg, const longer_input_weights* w, const void* E,
                                     const void* tdiff, const int32_t* lens, int B, int L, int d_e, const float* dH,
                                     float* dE_out, float* dtdiff_out, float* grads_out,
                                     void* ws, size_t ws_bytes, void* stream);

/* Measurement aid: when enabled, every kernel launch group of the entry points is bracketed
 * by a pair of HIP events recorded on the caller's stream (at most 4096 pairs between two
 * reads; later launches go unrecorded).  enable = 0: off; 1: every stage; any other value:
 * bit (s + 1) selects stage s (an event pair costs a few microseconds of launch time, so a
 * caller that wants one kernel's duration inside a timed loop selects that stage alone).  longer_stage_timing_read waits for the recorded
 * events, adds up the elapsed milliseconds and the number of launch groups per stage into
 * HOST arrays of LONGER_NUM_STAGES entries (0 parameter packing, 1 token merge, 2 K/V
 * projection, 3 attention + FFN, 4 candidate scoring) and clears the record.  The aid is the one
 * place where the library creates HIP objects: event pairs, made on first use (hipEventCreate)
 * and kept in fixed storage until the process ends; with timing off no entry point creates
 * anything.  Not thread-safe; do not enable under graph capture. */
#define LONGER_NUM_STAGES 5
int longer_stage_timing(int enable);
int longer_stage_timing_read(double* ms_out, int32_t* launches_out);

/* In-bounds probe of the matrix-core register layout the kernels rely on: runs one
 * 32x32 MFMA per element type on index-coded operands and writes, for every lane and
 * accumulator register, the (row, column) it holds as row*32+column into out[2][64][16]
 * (int32, device; [0] = bf16 32x32x16, [1] = fp32 32x32x2). */
int longer_probe_mfma_layout(int32_t* out, void* stream);

/* In-bounds instruction-rate probe (measurement aid): `workgroups` workgroups of 512 threads (two
 * waves per SIMD) run `iters` iterations; per iteration a wave issues 16 bf16 32x32x16 MFMAs
 * (16 x 32768 FLOP) and / or 128 fp32 FMAs, arranged by `mode`:
 *   0 MFMAs in all 8 waves (the rate the matrix pipe sustains: the attainable peak a kernel is
 *     priced against beside the vendor figure)   1 FMAs in all 8 waves
 *   2 MFMAs then FMAs in every wave               3 waves 0-3 MFMAs, waves 4-7 FMAs
 *   4 as 3, idle cycles after each MFMA           5 every MFMA followed by 4 FMAs
 *   6 every MFMA followed by 8 FMAs               7 MFMAs in waves 0-3 only (one wave per SIMD)
 *   8 as 0 with the idle cycles of 4              9 as 3 with the MFMA waves at raised priority
 *   10 / 12 every MFMA followed by 4 / 2 packed fp16 FMAs       11 packed fp16 FMAs alone (128)
 *   13 every MFMA followed by 2 v_exp_f32         14 v_exp_f32 alone (128)
 *   15 every MFMA followed by one 16-byte LDS read per lane
 *   16 every MFMA followed by 4 fp32 -> bf16 pair conversions    17 every MFMA followed by 6 FMAs
 *   18-21 (128 instructions alone) packed fp16 FMA with a scalar-register constant / with the clamp
 *   modifier / packed fp16 multiply / fp32 -> fp16 pair conversion toward zero
 * The caller times the launch (events on `stream`).  out: device, workgroups * 512 floats
 * (a sink that keeps the work alive). */
int longer_probe_rate(int mode, int iters, int workgroups, float* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LONGER_H_ */
