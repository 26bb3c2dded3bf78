/* fllayer.h - C ABI of the layer glue around the pool's hot path: what a decoder layer of the
 * models the paper serves (Llama-7B/13B/34B, arXiv 2505.03756 section 6.1) computes besides the
 * calls of flpool.h, and one call that runs a whole layer step.  The paper leaves the model to the
 * serving engine; the operations are those of the published Llama architecture (pre-norm decoder,
 * root-mean-square norm, rotary embedding in the rotate-half pairing, gated SiLU MLP, no biases).
 *
 * Every tensor is a device pointer in the element type `dtype` (FLP_F32 / FLP_F16 / FLP_BF16),
 * row-major and dense unless a leading dimension is given.  Arithmetic is fp32 (angles of the
 * rotary embedding fp64); every output tensor is rounded once, to nearest even, where it is stored.
 * All calls enqueue on `hip_stream` and return; the caller owns every buffer until that work is
 * done.  Errors: FLP_EINVAL (null / misaligned pointer, non-positive size), FLP_ENOTSUP (a width that
 * is not a multiple of 16 bytes, head_dim other than 64 / 128 for the rotary embedding), FLP_EHIP;
 * text via flp_last_error().  Pointers must be 16-byte aligned.
 */
#ifndef FLLAYER_H_
#define FLLAYER_H_

#include "flpool.h"

#ifdef __cplusplus
extern "C" {
#endif

/* y[t, :] = x[t, :] / sqrt(mean(x[t, :]^2) + eps) * w   for t < n_tokens; x, y [n_tokens, hidden], w [hidden].
 * y may be x. */
flp_status fll_rmsnorm(int32_t dtype, const void* x, const void* w, void* y, int32_t n_tokens, int32_t hidden,
                       float eps, void* hip_stream);

/* The residual update and the norm that follows it in one pass over the row:
 * resid[t, :] = round(resid[t, :] + delta[t, :]); y[t, :] = rmsnorm of the rounded row (as fll_rmsnorm would
 * compute from the stored resid).  y == NULL: only the residual update. */
flp_status fll_add_rmsnorm(int32_t dtype, void* resid, const void* delta, const void* w, void* y, int32_t n_tokens,
                           int32_t hidden, float eps, void* hip_stream);

/* Rotary position embedding, in place, on q [n_tokens, n_q_heads, head_dim] and k [n_tokens, n_kv_heads,
 * head_dim] (either may be NULL): in every head, channel i < head_dim / 2 and channel i + head_dim / 2 form a
 * pair (a, b) that becomes (a cos - b sin, b cos + a sin) with the angle positions[t] * theta^(-2 i / head_dim).
 * positions: device int32[n_tokens], the absolute position of each token in its sequence. */
flp_status fll_rope(int32_t dtype, void* q, void* k, const int32_t* positions, int32_t n_tokens, int32_t n_q_heads,
                    int32_t n_kv_heads, int32_t head_dim, float theta, void* hip_stream);

/* out = gate * sigmoid(gate) * up, element-wise over [n_tokens, width]; ld_* = elements between rows
 * (gate and up may be the two halves of one [n_tokens, 2 * width] tensor).  out may be gate. */
flp_status fll_silu_mul(int32_t dtype, const void* gate, int64_t ld_gate, const void* up, int64_t ld_up, void* out,
                        int64_t ld_out, int32_t n_tokens, int32_t width, void* hip_stream);

typedef struct {
  int32_t hidden, n_q_heads, mlp_dim;   /* kv heads, head_dim, element type come from the pool               */
  float   rms_eps;                       /* <= 0: 1e-5                                                         */
  float   rope_theta;                    /* <= 0: 10000                                                        */
  int32_t reserved;
} fll_layer_config;

/* Dense weights of one layer, device pointers in the pool's element type.  The matrices are stored
 * [d_out, d_in] row-major (one row per output feature, the layout of a linear layer's weight). */
typedef struct {
  const void* in_norm;    /* [hidden]                                   */
  const void* post_norm;  /* [hidden]                                   */
  const void* wq;         /* [n_q_heads * head_dim, hidden]             */
  const void* wk;         /* [n_kv_heads * head_dim, hidden]            */
  const void* wv;         /* [n_kv_heads * head_dim, hidden]            */
  const void* wo;         /* [hidden, n_q_heads * head_dim]             */
  const void* w_gate;     /* [mlp_dim, hidden]                          */
  const void* w_up;       /* [mlp_dim, hidden]                          */
  const void* w_down;     /* [hidden, mlp_dim]                          */
} fll_layer_weights;

/* Where one projection's LoRA matrices sit in the adapters' block tables (as in flp_lora_proj). */
typedef struct {
  const int32_t* a_tab_off;
  const int32_t* a_row_base;
  const int32_t* b_tab_off;
  const int32_t* b_row_base;
} fll_lora_place;

/* One batch of a layer step: the arguments of flp_lora_apply_paged and flp_paged_prefix_attention that
 * do not change from projection to projection.  lora[] is indexed q, k, v, o, gate, up, down; a
 * projection whose four pointers are NULL has no LoRA branch. */
typedef struct {
  int32_t n_tokens, n_seqs;
  int32_t n_adapters, max_rank;
  int32_t max_blocks_per_seq, reserved;
  const int32_t* cu_new;          /* HOST   int32[n_seqs + 1]                                       */
  const int32_t* prefix_len;      /* HOST   int32[n_seqs]                                           */
  const int32_t* positions;       /* device int32[n_tokens]: prefix_len[i] + j for token j of seq i  */
  const int32_t* kv_tables;       /* device int32[n_seqs, max_blocks_per_seq]                       */
  const int32_t* token_adapter;   /* device int32[n_tokens], -1 = no adapter                        */
  const int32_t* rank;            /* device int32[n_adapters]                                       */
  const float*   scale;           /* device float[n_adapters]                                       */
  const int32_t* lora_tables;     /* device int32[]                                                 */
  fll_lora_place lora[7];
} fll_layer_batch;

/* Bytes of device scratch that fll_layer_forward needs for n_tokens tokens (activations between the
 * steps; the LoRA intermediates live in the pool's own workspace). */
int64_t fll_layer_scratch_bytes(const flp_pool* pool, const fll_layer_config* cfg, int32_t n_tokens);

/* One decoder layer over the batch, on the pool that holds this layer's KV blocks and LoRA pages:
 *   n1 = rmsnorm(h, in_norm);  q, k, v = n1 . W^T + LoRA (one rounding of base + branch);  rope(q, k)
 *   K, V appended to the sequences' blocks;  a = paged prefix attention(q)
 *   h = h + (a . Wo^T + LoRA);  n2 = rmsnorm(h, post_norm)
 *   g, u = n2 . W^T + LoRA;  h = h + ((g * sigmoid(g) * u) . Wdown^T + LoRA)
 * h: device [n_tokens, hidden], in/out (the residual stream).  scratch: device memory of at least
 * fll_layer_scratch_bytes(), 256-byte aligned, contents undefined afterwards.  Blocks that the batch
 * needs must be resident (swap-ins ordered before this call by the caller's events). */
flp_status fll_layer_forward(flp_pool* pool, const fll_layer_config* cfg, const fll_layer_weights* w,
                             const fll_layer_batch* batch, void* h, void* scratch, int64_t scratch_bytes,
                             void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif  /* FLLAYER_H_ */
