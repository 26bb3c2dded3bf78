/* flcache.h - C ABI of the host logic that produces the block lists of flpool.h: the
 * dependency-aware cache manager and the performance-driven cache swapper of the paper
 * (arXiv 2505.03756, sections 4 and 5).  Everything here runs on the host; the lists it
 * returns are what flp_pool_swap_out / flp_pool_swap_in take.
 *
 * Model (sections 4.1-4.3).  One tree: a virtual root, the LoRA nodes on the second layer
 * (label: LoRA id), below each LoRA node the KV caches computed with that LoRA (label: the
 * token sequence).  A KV node is one pool block, i.e. `block_tokens` consecutive tokens; only
 * full blocks become nodes.  A LoRA node owns the blocks that hold the adapter's pages.
 * Every node records its tier (0 = HBM, 1 = host), its block ids on that tier, how often it
 * was visited and when it was used last.  The manager allocates and frees block ids through
 * the flp_pool it was created on; it never touches block contents.
 *
 * Dependencies (section 4.2).  A query first matches its LoRA node, then the KV nodes that
 * spell its tokens, top down.  Swap-out only takes nodes that have no child in HBM, swap-in
 * only nodes whose parent is in HBM, so an HBM-resident node never has a non-resident
 * ancestor ("all KV caches that reside in the HBM are valid ones").
 *
 * Cost model (section 5; `now` and last-use times are seconds on the caller's clock):
 *   Eq. 3  Low_lora      = sum over LoRAs of 1 - (1 - prob_i)^BS
 *   Eq. 4  LoRA_Eval     = max(1, Low_lora / Now_LoRA)          (LoRA nodes; 1 for KV nodes)
 *   Eq. 5  Retain_Eval_i = cost_i * prob_i * (1 - sigmoid(t_i))
 *   Eq. 6  Eval_i        = LoRA_Eval_i * Retain_Eval_i
 * with prob_i = visits_i / number of matched queries, cost_i = node bytes / pcie_bytes_per_s,
 * t_i = (now - last use) / time_scale_s, Now_LoRA = LoRAs in HBM (at least 1), Low_lora and
 * Now_LoRA sampled once per tick, ties broken in favour of the older node.
 *
 * Swapper (section 5.3).  flc_tick is one monitor interval: with HBM usage (1 - free / total
 * blocks of the pool's HBM tier) above `upper` it swaps out candidates in increasing order of
 * Eval until usage <= upper; with usage below `lower` it swaps in candidates in decreasing
 * order until usage >= lower (never past `upper`); in between it does nothing.
 *
 * Errors: FLP_EINVAL (null pointer, unknown LoRA or query, bad argument), FLP_ENOSPC (the
 * tier has too few free blocks; nothing changed), FLP_ERANGE (an output array is too small;
 * nothing changed), FLP_EDUP (LoRA id already present).  Text via flp_last_error().
 * All calls on one flc_cache are serialised by an internal lock.
 */
#ifndef FLCACHE_H_
#define FLCACHE_H_

#include "flpool.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct flc_cache flc_cache;

typedef struct {
  int32_t block_tokens;        /* tokens per KV node = block_tokens of the pool (> 0)                   */
  int32_t use_lru;             /* ablation (section 6.7): Eval_i = time of last use                     */
  int32_t ignore_dependencies; /* ablation (section 6.6): every unused node is a candidate              */
  int32_t no_lora_reward;      /* ablation (section 6.8): LoRA_Eval = 1                                 */
  double upper, lower;         /* HBM usage thresholds of section 5.3 (the paper uses 0.95 and 0.70)    */
  double pcie_bytes_per_s;     /* host link bandwidth behind cost_i of Eq. 5                            */
  double time_scale_s;         /* seconds per unit of t_i in Eq. 5 (the paper gives no unit)            */
} flc_config;

typedef struct {
  int64_t n_nodes, n_lora_nodes, n_kv_nodes;   /* without the virtual root                              */
  int64_t n_lora_hbm;                          /* Now_LoRA                                              */
  int64_t n_queries;                           /* matched queries so far                                */
  int64_t n_running;                           /* queries matched and not yet released                  */
  int64_t hbm_blocks_held, host_blocks_held;   /* blocks owned by nodes, per tier                       */
  int64_t invalid_kv_blocks;                   /* HBM KV blocks below a non-resident ancestor           */
  double usage;                                /* 1 - free / total of the pool's HBM tier               */
} flc_stats;

/* One row per node for inspection and tests, in increasing id order. */
typedef struct {
  int32_t id, kind /* 0 LoRA, 1 KV */, parent /* 0 = virtual root */, tier;
  int32_t first_block, n_blocks, pins, pad;
  int64_t visits;
  double last_use;
} flc_node_info;

/* The cache works on `pool` (kept by pointer; destroy the cache first).  flc_destroy returns the blocks that the
 * nodes still hold to the pool (blocks of not_taken lists and of forgotten queries were the caller's already).
 * Section 4.3. */
flp_status flc_create(flp_pool* pool, const flc_config* cfg, flc_cache** out);
flp_status flc_destroy(flc_cache* c);

/* A LoRA enters the pool on `tier`: n_blocks ids are allocated there and returned in out_ids
 * (host array of n_blocks; the caller fills the pages).  Sections 4.1, 4.3. */
flp_status flc_add_lora(flc_cache* c, int32_t lora_id, int32_t n_blocks, int32_t tier, double now, int32_t* out_ids);

/* Section 4.2, matching: the LoRA node, then the KV nodes spelling tokens[0 .. n_tokens), whole
 * blocks only.  Visit counts and last-use times of the matched nodes are updated.  Matched nodes
 * on the host tier are moved to HBM top down as far as free HBM blocks allow (pairs returned in
 * swap_host / swap_dev, n_swap of them, in the order to copy them: pass them to
 * flp_pool_swap_in before the query runs); the match ends at the first node that cannot be
 * brought in.  The usable nodes are pinned until flc_release(*query).
 * n_lora_blocks = -1 and n_kv_blocks = 0 when not even the LoRA fits (the query waits).
 * Capacities: lora_cap >= blocks of the LoRA, kv_cap >= n_tokens / block_tokens,
 * swap_cap >= lora blocks + n_tokens / block_tokens, else FLP_ERANGE.  All arrays are host. */
flp_status flc_match(flc_cache* c, int32_t lora_id, const int32_t* tokens, int32_t n_tokens, double now,
                     int64_t* query, int32_t* lora_blocks, int32_t lora_cap, int32_t* n_lora_blocks,
                     int32_t* kv_blocks, int32_t kv_cap, int32_t* n_kv_blocks, int32_t* swap_host,
                     int32_t* swap_dev, int32_t swap_cap, int32_t* n_swap);

/* Section 4.2, updating: the n_new HBM blocks the query filled (full blocks of `tokens` right
 * after the blocks it already holds; tokens must cover them) become KV nodes below the last
 * node of the query and are pinned by it.  Ids that are not taken over, because a node with the
 * same tokens exists already, come back in not_taken (host array of n_new) for the caller to free. */
flp_status flc_insert(flc_cache* c, int64_t query, const int32_t* tokens, int32_t n_tokens,
                      const int32_t* new_blocks, int32_t n_new, double now, int32_t* not_taken,
                      int32_t* n_not_taken);

/* The query is done: its nodes are no longer pinned. */
flp_status flc_release(flc_cache* c, int64_t query);

/* Section 5.3, one monitor interval with the recent batch size BS of Eq. 3.  At most out_cap /
 * in_cap block moves are decided per call (the rest waits for the next interval).  Swap-out pairs
 * go to flp_pool_swap_out(n_out, out_dev, out_host), swap-in pairs to
 * flp_pool_swap_in(n_in, in_host, in_dev), in this order, on one stream.  When the host tier is
 * full a swap-out victim is forgotten instead (with everything below it); the ids of forgotten
 * nodes are returned in `dropped` (up to drop_cap of them; n_dropped counts all). */
flp_status flc_tick(flc_cache* c, double now, int32_t batch_size, int32_t* out_dev, int32_t* out_host,
                    int32_t out_cap, int32_t* n_out, int32_t* in_host, int32_t* in_dev, int32_t in_cap,
                    int32_t* n_in, int32_t* dropped, int32_t drop_cap, int32_t* n_dropped);

/* Eq. 3 for the current visit statistics, and Eq. 6 for one node (as flc_tick would compute them now). */
flp_status flc_low_lora(flc_cache* c, int32_t batch_size, double* out);
flp_status flc_eval(flc_cache* c, int32_t node_id, double now, int32_t batch_size, double* out);

flp_status flc_get_stats(flc_cache* c, flc_stats* out);
/* Up to cap rows, in increasing id order; *n_nodes is the number of nodes whatever cap is. */
flp_status flc_snapshot(flc_cache* c, flc_node_info* rows, int64_t cap, int64_t* n_nodes);

#ifdef __cplusplus
}
#endif
#endif  /* FLCACHE_H_ */
