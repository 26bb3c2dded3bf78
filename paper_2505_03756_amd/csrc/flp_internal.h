// Internal declarations shared by the host logic (pool.cpp, dispatch.cpp) and the
// kernel translation units.  Not part of the ABI.
#pragma once

#include <hip/hip_runtime_api.h>

#include <cstdint>
#include <mutex>
#include <vector>

#include "flpool.h"

void flp_set_error(const char* fmt, ...) __attribute__((format(printf, 1, 2)));

#define FLP_TRY_HIP(expr)                                                                        \
  do {                                                                                           \
    hipError_t e_ = (expr);                                                                      \
    if (e_ != hipSuccess) {                                                                      \
      flp_set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__);  \
      return FLP_EHIP;                                                                           \
    }                                                                                            \
  } while (0)

#define FLP_TRY(expr)            \
  do {                           \
    flp_status s_ = (expr);      \
    if (s_ != FLP_OK) return s_; \
  } while (0)

// LIFO free list of one tier.
struct FlpFreeList {
  int64_t n = 0;
  std::vector<int32_t> stack;     // stack.back() is handed out next
  std::vector<uint8_t> is_free;
  std::vector<uint32_t> stamp;    // scratch for duplicate detection
  uint32_t gen = 0;
};

// One slot of the ring that carries small host arrays (id lists, work lists) to the
// device: pinned host buffer + device mirror + the event that marks the slot's last use.
struct FlpStageSlot {
  void* host = nullptr;
  void* dev = nullptr;
  size_t cap = 0;
  hipEvent_t ev = nullptr;
  bool in_flight = false;
};

constexpr int kStageSlots = 16;

struct flp_pool {
  flp_pool_config cfg{};
  int elem_bytes = 0;
  int64_t block_elems = 0;
  int64_t block_bytes = 0;
  int device = 0;
  uint8_t* dev_base = nullptr;
  uint8_t* host_base = nullptr;
  bool own_dev = false, own_host = false;
  bool host_tier_in_hbm = false;  // the caller placed the "host" tier in device memory
  FlpFreeList tier[2];
  FlpStageSlot stage[kStageSlots];
  int stage_next = 0;
  void* work = nullptr;           // device workspace (LoRA intermediates), grown on demand
  size_t work_cap = 0;
  void* attn_work = nullptr;      // device workspace of the attention call (split-KV partial results)
  size_t attn_work_cap = 0;
  std::vector<void*> retired;     // outgrown workspace buffers, freed with the pool
  mutable std::mutex mu;          // guards the free lists, the staging slots and the workspace
};

// Staging: acquire a slot with room for `bytes` (waits for the slot's previous use),
// fill slot->host, then flp_stage_upload() copies to slot->dev on the stream; after the
// consuming kernels are enqueued call flp_stage_release().
flp_status flp_stage_acquire(flp_pool* pool, size_t bytes, FlpStageSlot** slot);
flp_status flp_stage_upload(FlpStageSlot* slot, size_t bytes, hipStream_t stream);
flp_status flp_stage_release(FlpStageSlot* slot, hipStream_t stream);
flp_status flp_workspace(flp_pool* pool, size_t bytes, void** out);
// the host-side checks of flp_pool_swap_in (src_tier 1) / flp_pool_swap_out (src_tier 0) without enqueuing anything
flp_status flp_swap_check(flp_pool* pool, int32_t n, const int32_t* src_ids, const int32_t* dst_ids, int src_tier,
                          const char* who);

// A workspace of fixed size that the caller of the LoRA path brings along instead of the pool's growing one:
// `resolve` returns its device address for the pool's device (called only after the size check has passed).
struct FlpFixedWorkspace {
  size_t cap;
  flp_status (*resolve)(flp_pool* pool, void** out);
  const char* who;
};
// flp_lora_apply_paged with its intermediates in `ws` (no allocation, no growth)
flp_status flp_lora_apply_fixed(flp_pool* pool, const flp_lora_batch* batch, void* hip_stream, const FlpFixedWorkspace& ws);
// set-up of the file-scope scratch array for the current device (looks its device address up once per device);
// called when a pool is created, and again by the entry point that uses the array if that first attempt failed
flp_status flp_static_scratch_setup(int device, void** out);

// ---- kernel launchers (defined in the .hip files) ---------------------------------------
flp_status flp_launch_copy_blocks(const uint8_t* src_base, uint8_t* dst_base, const int32_t* src_ids_dev,
                                  const int32_t* dst_ids_dev, int32_t n, int64_t block_bytes,
                                  int host_link, hipStream_t stream);
// host_link: which side of the copy is the pinned host tier, and how wide the caller wants the launch
enum { FLP_LINK_NONE = 0, FLP_LINK_IN = 1, FLP_LINK_OUT = 2, FLP_LINK_IN_DUPLEX = 3, FLP_LINK_OUT_DUPLEX = 4,
       FLP_LINK_IN_NARROW = 5, FLP_LINK_OUT_NARROW = 6 };
// flp_pool_swap_in / flp_pool_swap_out (src_tier 1 / 0) for a caller that knows what runs beside the move: one
// direction alone, both directions together, or moves that need not hurry
enum { FLP_WIDTH_SINGLE = 0, FLP_WIDTH_DUPLEX = 1, FLP_WIDTH_NARROW = 2 };
flp_status flp_swap_width(flp_pool* p, int32_t n, const int32_t* src_ids, const int32_t* dst_ids, int src_tier,
                           void* hip_stream, int width);

flp_status flp_launch_stage_copy(const void* src_pinned, void* dst_dev, size_t bytes, hipStream_t stream);

// Kernels work on groups of 16 token positions; a block of 32 positions is two such groups (group index
// gi = position / 16 lives in block gi / (bt / 16), at slots 16 * (gi % (bt / 16)) ...).
struct FlpAppendUnit {   // the slots [s0, s1) of the 16-position group `blk_idx` of sequence `seq`
  int32_t seq, blk_idx, s0, s1, t_first, pad0, pad1, pad2;
};
struct FlpAttnUnit {     // new tokens [j0, j0+n_tok) of sequence `seq`
  int32_t seq, j0, n_tok;
  // split-KV (few long sequences): with n_split > 1 the unit is ONE token and covers only the 16-position groups
  // [g_lo, g_hi) of its context; its unnormalised result goes to row part_row of the partials buffer, piece `split`
  int32_t n_split, split, g_lo, g_hi, part_row;
};

struct FlpMfmaItem {     // query rows [r0, r0+n_rows) of (sequence, kv head g); n_rows == 0: padding
  int32_t seq, g, r0, n_rows;
};

struct FlpAttnArgs {
  uint8_t* pool;
  int64_t block_elems;
  const int32_t* tables;
  int32_t max_blocks;
  int32_t n_h, n_kv;
  int32_t bt;                  // token positions per block: 16 or 32
  const void* q;
  void* out;
  const void* k_new;
  const void* v_new;
  const int32_t* cu_new;       // device copies
  const int32_t* prefix_len;
  float scale_log2e;
  float* partials;             // split-KV: [part_row][n_h][max_split][head_dim + 2] fp32 (running max, sum, channels)
  int32_t max_split;
};

flp_status flp_launch_kv_append(int dtype, int head_dim, const FlpAttnArgs& a, const FlpAppendUnit* units_dev,
                                int32_t n_units, hipStream_t stream);
flp_status flp_launch_attn_rows(int dtype, int head_dim, const FlpAttnArgs& a, const FlpAttnUnit* units_dev,
                                int32_t n_units, hipStream_t stream);
// split-KV: one merged row per (partials row, head): token t = merge_tok[row], n_split[row] pieces combined in
// piece order (so the result does not depend on which piece finished first)
flp_status flp_launch_attn_merge(int dtype, int head_dim, const FlpAttnArgs& a, const int32_t* merge_tok_dev,
                                 const int32_t* merge_nsplit_dev, int32_t n_rows, hipStream_t stream);
flp_status flp_attn_workspace(flp_pool* pool, size_t bytes, void** out);

flp_status flp_launch_attn_mfma(int dtype, const FlpAttnArgs& a, const FlpMfmaItem* items_dev, int32_t n_items,
                                hipStream_t stream);
constexpr int kMfmaRowsPerItem = 256;
constexpr int kMfmaMaxBlocks = 4096;       // longest context of the matrix-core kernel: 65536 positions

struct FlpLoraArgs {
  const uint8_t* pool;
  int64_t block_elems;
  int32_t T, d_in, n_adapters, max_rank, n_proj;
  int64_t ld_x;
  const void* x;
  const int32_t* token_adapter;
  const int32_t* rank;
  const float* scale;
  const int32_t* tables;
  flp_lora_proj proj[FLP_MAX_PROJ];
  // unrounded base term x.W_base [T, d_out] of a projection whose w_base was given (16-bit pools), else null:
  // the expand kernels then take the base from here instead of y and round base + delta once
  const float* base32[FLP_MAX_PROJ];
  // workspace
  float* v;                    // [T, n_proj, max_rank] fp32
  int32_t* n_seg;
  int32_t* seg_adapter;
  int32_t* seg_start;
  int32_t* perm;
  int32_t* tile_start;         // [n_seg + 1] first tile of each segment (matrix-core kernels)
  int32_t* group_start;        // [n_seg + 1] first tile group of each segment (expand kernel)
};

struct FlpLoraMfma {
  int32_t mt;                  // 16-token tiles per work item (1 or 2)
  int32_t k_splits, k_per_split;
  int32_t v_rows;              // rows of one split's partial v buffer (= tiles_bound * 16 * mt)
  int32_t cols_per_slab;
  int32_t tiles_bound;         // host-side upper bound of the number of tiles (sizes the v buffer)
  int32_t tiles_grid;          // tiles the shrink launch covers in one pass (multiple of 8); more are looped over
  int32_t group_tokens;        // tokens per tile group of the expand kernel (multiple of 16*mt)
  int32_t groups_bound;
  int32_t groups_grid;         // tile groups the expand launch covers in one pass (multiple of 8)
  int32_t slabs;               // column slabs per projection (set by the launcher)
  int32_t shrink_only;         // 1: stop after the shrink step (the expand step runs inside the dense product)
};

// What the large-batch dense product needs to add one projection's LoRA branch to its accumulators before it
// rounds (the expand step as an epilogue: y = round(x . W + s (x A^T) B), no fp32 copy of the product, no second
// pass over y).  v is the shrink step's output, rows in segment order: token t of adapter a sits in row
// vrow_base[a] + inv_perm[t] (both written by the segmentation kernel).
struct FlpGemmLora {
  const int32_t* token_adapter;
  const int32_t* rank;
  const float* scale;
  const int32_t* tables;
  const int32_t* b_tab_off;    // this projection's
  const int32_t* b_row_base;
  const void* pool;
  int64_t block_elems;
  const float* v;              // [k_splits][v_rows][n_proj][rp] fp32
  int32_t v_rows, k_splits, n_proj, p, rp;
  int32_t n_adapters, max_rank;
  const int32_t* inv_perm;     // [T] token -> position in segment order
  const int32_t* vrow_base;    // [n_adapters]
};

flp_status flp_launch_lora_segment(int32_t T, const int32_t* token_adapter, int32_t n_adapters, int32_t* n_seg,
                                   int32_t* seg_adapter, int32_t* seg_start, int32_t* perm, int32_t tm,
                                   int32_t* tile_start, int32_t tg, int32_t* group_start, hipStream_t stream,
                                   int32_t* inv_perm = nullptr, int32_t* vrow_base = nullptr);
flp_status flp_launch_lora_mfma(int dtype, const FlpLoraArgs& a, const FlpLoraMfma& c, hipStream_t stream);
flp_status flp_launch_lora_simple(int dtype, const FlpLoraArgs& a, hipStream_t stream);
flp_status flp_launch_base_gemm(int dtype, const void* x, int64_t ld_x, const void* w, int w_layout, void* y,
                                int64_t ld_y, int M, int N, int K, void* wt_scratch, float* y32, float* splitk_scratch,
                                size_t splitk_bytes, hipStream_t stream, const FlpGemmLora* lora = nullptr);
// true when flp_launch_base_gemm runs the large-batch kernel for this shape (the one that can take the LoRA branch
// as an epilogue)
bool flp_gemm_is_large(int dtype, int M, int N, int K, int64_t ld_x);
// silu(x . Wg^T) * (x . Wu^T) in one pass (16-bit types, weights [N, K]); FLP_ENOTSUP, nothing launched, for shapes
// that the large-batch kernel does not take
flp_status flp_launch_gated_gemm(int dtype, const void* x, int64_t ld_x, const void* w_gate, const void* w_up,
                                 void* out, int64_t ld_out, int M, int N, int K, hipStream_t stream,
                                 const FlpGemmLora* lora_gate = nullptr, const FlpGemmLora* lora_up = nullptr);
// true when flp_launch_gated_gemm takes this shape
bool flp_gemm_gated_fits(int dtype, int M, int N, int K, int64_t ld_x);
// flp_lora_apply_paged for exactly two projections with dense bases stored [d_out, d_in] and equal widths (gate and
// up of an MLP), whose results are not stored: out = silu(y0) * y1 in one pass of the large-batch GEMM, each product
// with its LoRA branch added before it is rounded.  FLP_ENOTSUP, nothing launched, when the batch is not one that
// this path takes; the caller then runs flp_lora_apply_paged and the element-wise step.
flp_status flp_lora_apply_gated(flp_pool* pool, const flp_lora_batch* batch, void* out, int64_t ld_out, void* hip_stream);
// bytes of split-K scratch worth offering for an [M, N] product (0 for large batches, which are not split)
inline size_t flp_gemm_splitk_bytes(int M, int N) { return M <= 1024 ? (size_t)8 * M * N * 4 : 0; }
