/*
 * flpool - C ABI of the MI355X paged multi-LoRA layer step.
 *
 * One pool of equal-size blocks in device memory (plus a host tier of the same
 * block size) holds both LoRA adapter weights and prefix KV caches, as in the
 * unified caching pool of the paper (section 4.3, "Unified Caching Pool for
 * LoRAs and KVs").  The calls below are what a cache manager needs once it has
 * matched a query: hand out / recycle blocks, move listed blocks between the
 * tiers, then run the batched multi-LoRA projection and the attention of the
 * new tokens over whatever is resident.
 *
 * Conventions
 *   - Every function returns 0 (FLP_OK) or a negative flp_status; none throws.
 *     Text for the last failure on the calling thread: flp_last_error().
 *   - "host" pointers are dereferenced by the CPU inside the call and may be
 *     freed once it returns.  "device" pointers are borrowed until the work
 *     enqueued on the given stream has completed; the caller owns them.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Calls on one stream run in order; ordering between streams is the
 *     caller's business (events).
 *   - On an error that the host can detect nothing is enqueued and no state
 *     changes.  Faults raised asynchronously by the GPU surface as FLP_EHIP on
 *     a later call.
 *   - dtype: 0 = fp32, 1 = fp16, 2 = bf16.  16-bit types accumulate in fp32.
 *
 * Block layout (the paper fixes only that all blocks have one size)
 *   BLOCK_ELEMS = 2 * block_tokens * n_kv_heads * head_dim.
 *   KV block:   K of (kv head g, slot s, channel c) at ((g*bt + s)*d + c),
 *               V of the same at n_kv*bt*d + ((g*d + c)*bt + s)   (V transposed,
 *               so the bt positions of one channel are contiguous; the kernels work
 *               on groups of 16 positions, one or two per block).
 *   LoRA block: page-rows of `row_len` elements packed from the start of the
 *               block, floor(BLOCK_ELEMS / row_len) rows per block, never
 *               straddling blocks (partition along the rank dimension, section
 *               4.3).  Page-row i of a table lives in block table[i / rows_per_block]
 *               at element (i % rows_per_block) * row_len.  A page-row of A is the
 *               d_in coefficients of one rank index; a page-row of B its d_out
 *               coefficients.
 */
#ifndef FLPOOL_H
#define FLPOOL_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct flp_pool flp_pool;   /* opaque; created and destroyed by the library */
typedef int32_t flp_status;

#define FLP_OK        0
#define FLP_EINVAL   (-1)   /* null pointer, negative count, inconsistent sizes            */
#define FLP_ENOSPC   (-2)   /* not enough free blocks; nothing was allocated               */
#define FLP_ERANGE   (-3)   /* block id or length out of range                             */
#define FLP_EDUP     (-4)   /* duplicate destination in a swap list / double free          */
#define FLP_EHIP     (-5)   /* HIP runtime error                                           */
#define FLP_ENOTSUP  (-6)   /* dtype / head_dim / block_tokens not supported by the kernels */

#define FLP_F32  0
#define FLP_F16  1
#define FLP_BF16 2

#define FLP_TIER_DEVICE 0
#define FLP_TIER_HOST   1

typedef struct {
  int32_t dtype;            /* FLP_F32 / FLP_F16 / FLP_BF16                                   */
  int32_t block_tokens;     /* token positions per KV block (kernels support 16 and 32)       */
  int32_t n_kv_heads;
  int32_t head_dim;         /* kernels support 64 and 128                                     */
  int64_t n_dev_blocks;
  int64_t n_host_blocks;
  void*   dev_base;         /* device memory of n_dev_blocks*BLOCK_BYTES bytes owned by the
                               caller (256-byte aligned), or NULL: the library allocates     */
  void*   host_base;        /* memory of n_host_blocks*BLOCK_BYTES bytes that the GPU can
                               address (pinned host memory; 256-byte aligned), or NULL: the
                               library allocates pinned memory                               */
} flp_pool_config;

/* Pool life cycle (section 4.3: both tiers are cut into blocks of one size at
 * initialisation).  The current HIP device at creation is the pool's device. */
flp_status flp_pool_create(const flp_pool_config* cfg, flp_pool** out);
flp_status flp_pool_destroy(flp_pool* pool);
int64_t    flp_pool_block_bytes(const flp_pool* pool);
int64_t    flp_pool_num_free(const flp_pool* pool, int32_t tier);
void*      flp_pool_base(const flp_pool* pool, int32_t tier);

/* Block allocation (section 4.3: freed blocks are recycled for later
 * allocations; LoRA pages and KV blocks come from the same list).  The free
 * list is a LIFO stack: a fresh pool hands out 0,1,2,...; blocks are reused in
 * the reverse order of their release.  `out_ids` / `ids` are host arrays.
 * alloc is all-or-nothing (FLP_ENOSPC leaves the pool unchanged); free rejects
 * ids out of range (FLP_ERANGE) and ids that are already free or repeated
 * (FLP_EDUP) without releasing anything. */
flp_status flp_pool_alloc(flp_pool* pool, int32_t tier, int32_t n, int32_t* out_ids);
flp_status flp_pool_free(flp_pool* pool, int32_t tier, int32_t n, const int32_t* ids);

/* Block moves between the tiers (sections 3.2 and 5.3: the swapper's decision
 * list is executed as block moves; section 4.3: asynchronously on a stream).
 * swap_in:  device block dev_ids[k]  <- host block host_ids[k], k = 0..n-1.
 * swap_out: host block host_ids[k]   <- device block dev_ids[k].
 * Whole blocks, byte for byte; every other block is left untouched; allocation
 * state does not change.  The id arrays are host arrays and are consumed
 * before the call returns.  n = 0 succeeds and enqueues nothing.  Ids out of
 * range give FLP_ERANGE, a destination listed twice FLP_EDUP (sources may
 * repeat). */
flp_status flp_pool_swap_in(flp_pool* pool, int32_t n, const int32_t* host_ids, const int32_t* dev_ids,
                            void* hip_stream);
flp_status flp_pool_swap_out(flp_pool* pool, int32_t n, const int32_t* dev_ids, const int32_t* host_ids,
                             void* hip_stream);

/* ---------------------------------------------------------------------------
 * Paged prefix attention (sections 2.1 and 4.2: a query reuses the stored KV of
 * its matched prefix and attends over it together with the KV of its own new
 * tokens; section 4.3: new KV stays in the pool where it is produced).
 *
 * Sequence i has prefix_len[i] reusable positions already in the pool and
 * n_i = cu_new[i+1]-cu_new[i] >= 0 new tokens (rows cu_new[i].. of q/out).
 * Position p of sequence i lives in block block_tables[i][p / bt], slot p % bt.
 * New token j (position p = prefix_len[i] + j), query head h, kv head
 * g = h / (n_q_heads / n_kv_heads):
 *     out[t,h,:] = sum_{k<=p} softmax_k( sm_scale * q[t,h,:].K_i[k,g,:] ) * V_i[k,g,:]
 * Slots beyond a sequence's length are never read into the result, whatever
 * bits they hold. */
typedef struct {
  int32_t n_seqs;
  int32_t n_q_heads;
  int32_t max_blocks_per_seq;     /* row stride of block_tables                               */
  float   sm_scale;               /* <= 0: 1/sqrt(head_dim)                                   */
  const void*    q;               /* device [T, n_q_heads, head_dim], pool dtype              */
  const void*    k_new;           /* device [T, n_kv_heads, head_dim] or NULL                 */
  const void*    v_new;           /* device [T, n_kv_heads, head_dim] or NULL                 */
  void*          out;             /* device [T, n_q_heads, head_dim], pool dtype              */
  const int32_t* cu_new;          /* HOST   int32[n_seqs+1], cu_new[0] = 0, non-decreasing    */
  const int32_t* prefix_len;      /* HOST   int32[n_seqs]                                     */
  const int32_t* block_tables;    /* device int32[n_seqs, max_blocks_per_seq]                 */
} flp_attn_batch;

/* Store the new tokens' K and V rows into their slots (bit for bit).  Uses
 * k_new, v_new, cu_new, prefix_len, block_tables of the batch; q/out ignored.
 * FLP_ERANGE if prefix_len[i] + n_i exceeds max_blocks_per_seq * bt. */
flp_status flp_kv_append(flp_pool* pool, const flp_attn_batch* batch, void* hip_stream);

/* Attention of the new tokens.  If k_new and v_new are non-NULL the append
 * above is enqueued first; if both are NULL the fresh K/V must already be in
 * the pool. */
flp_status flp_paged_prefix_attention(flp_pool* pool, const flp_attn_batch* batch, void* hip_stream);

/* ---------------------------------------------------------------------------
 * Batched heterogeneous LoRA (Eq. 1 and Eq. 2 in row-vector form; section 2.1:
 * queries with different adapters run in one batch).  Token t carries adapter
 * a = token_adapter[t]; for every projection p of the batch
 *     y_p[t,:] = base_p[t,:] + scale[a] * ( x[t,:] . A_{p,a}^T ) . B_{p,a}
 * where base_p is what y_p holds on entry (w_base == NULL) or x.W_base, A_{p,a}
 * is rank[a] page-rows of length d_in starting at page-row a_row_base[a] of the
 * table block_tables + a_tab_off[a], and B_{p,a} is rank[a] page-rows of length
 * d_out located the same way through b_tab_off / b_row_base.  a = -1 leaves the
 * base term.  A token whose adapter has rank 0 (not resident) is a caller
 * error; its row is left at the base term.  The projections of one batch share
 * x (q, k and v read it once).  The call keeps its intermediates (segment lists,
 * fp32 x.A^T) in a workspace owned by the pool: LoRA calls on one pool must be
 * ordered with respect to each other (same stream, or events between them).
 * Limits, checked on the host before anything is enqueued: n_adapters <= 2048
 * and 1 <= max_rank <= 64 (FLP_ERANGE otherwise).  rank[] lives in device memory
 * and is not read by the host: rank[a] > max_rank is a caller error, and every
 * kernel then uses the first max_rank page-rows of that adapter's A and B
 * (the same result whatever the batch size). */
#define FLP_MAX_PROJ 4

typedef struct {
  int32_t d_out;
  int32_t w_base_layout;          /* 0: w_base is [d_in, d_out]; 1: w_base is [d_out, d_in] (one row per
                                     output feature, a linear layer's weight: no transposition pass)  */
  int64_t ld_y;                   /* elements between rows of y (>= d_out)                    */
  void*          y;               /* device [T, ld_y], pool dtype, in/out                     */
  const void*    w_base;          /* device, row-major in the layout above, pool dtype, or NULL (y
                                     already holds the base); 16-bit pools need d_in % 64 == 0   */
  const int32_t* a_tab_off;       /* device int32[n_adapters]                                 */
  const int32_t* a_row_base;      /* device int32[n_adapters]                                 */
  const int32_t* b_tab_off;       /* device int32[n_adapters]                                 */
  const int32_t* b_row_base;      /* device int32[n_adapters]                                 */
} flp_lora_proj;

typedef struct {
  int32_t n_tokens;
  int32_t d_in;
  int64_t ld_x;                   /* elements between rows of x (>= d_in)                     */
  int32_t n_adapters;             /* <= 2048                                                  */
  int32_t max_rank;               /* upper bound of rank[], 1..64                             */
  int32_t n_proj;                 /* 1..FLP_MAX_PROJ                                          */
  int32_t reserved;
  const void*    x;               /* device [T, ld_x], pool dtype                             */
  const int32_t* token_adapter;   /* device int32[T], -1 = no adapter                         */
  const int32_t* rank;            /* device int32[n_adapters], 0 = not resident               */
  const float*   scale;           /* device float[n_adapters]                                 */
  const int32_t* block_tables;    /* device int32[], all adapter tables back to back          */
  flp_lora_proj  proj[FLP_MAX_PROJ];
} flp_lora_batch;

flp_status flp_lora_apply_paged(flp_pool* pool, const flp_lora_batch* batch, void* hip_stream);

/* The same call for callers that cannot allocate device memory (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): same
 * arguments, same kernels, same results bit for bit, but the intermediates live
 * in a fixed array of flp_static_scratch_bytes() bytes (64 MiB) that every GPU
 * using the library holds from the moment the library's code is loaded there
 * until the process ends.  The call allocates and frees nothing (no hipMalloc /
 * hipFree, no pinned memory, no growth).  A batch whose intermediates do not fit
 * (roughly 4 * n_tokens * n_proj * max_rank bytes rounded up to whole 16-rank
 * tiles and doubled or quadrupled when the contraction is split, plus 12 bytes
 * per token; a dense base adds its transposed copy and, outside the large-batch
 * path, 4 * n_tokens * d_out bytes per projection) is refused with FLP_ENOSPC
 * before anything is enqueued; the five benchmark workloads' calls without a
 * dense base need 1-44 MiB.  The pool's device must be the current device
 * (FLP_EINVAL otherwise).  All calls on one GPU, from whatever pool or thread,
 * share that GPU's one array, which keeps the previous call's contents (every
 * kernel writes what it later reads, nothing needs to start at zero): calls
 * whose work overlaps in time on one GPU race with each other, so keep them on
 * one stream or order them with events.  The array's address is looked up when
 * a pool is created on the device (again here if that failed). */
flp_status flp_lora_apply_paged_static(flp_pool* pool, const flp_lora_batch* batch, void* hip_stream);
int64_t    flp_static_scratch_bytes(void);

/* Adapter segmentation used by the call above, exposed for inspection: a stable
 * grouping of token indices by adapter id (section 2.1 names the batched kernel
 * "segmented gather"; the grouping itself is this build's).  Device outputs:
 * n_seg[1]; seg_adapter[n_adapters] (increasing ids of the non-empty adapters);
 * seg_start[n_adapters+1] (offsets into perm; seg_start[n_seg] = number of
 * tokens with an adapter); perm[n_tokens] (token indices grouped by adapter,
 * original order kept inside a group).  Entries past the counts are
 * unspecified.  n_adapters <= 2048 (FLP_ERANGE otherwise). */
flp_status flp_lora_segment(flp_pool* pool, int32_t n_tokens, const int32_t* token_adapter, int32_t n_adapters,
                            int32_t* n_seg, int32_t* seg_adapter, int32_t* seg_start, int32_t* perm,
                            void* hip_stream);

const char* flp_last_error(void);   /* thread-local; valid until the next call on this thread */
const char* flp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FLPOOL_H */
