// Host-side dispatch of the compute entry points: argument checks, the work lists built
// from the host-resident sequence lengths, and the launches.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <numeric>

#include "flp_internal.h"

namespace {

bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

flp_status check_attn_batch(const flp_pool* p, const flp_attn_batch* b, bool need_qo, bool need_kv, const char* who) {
  if (!p || !b) {
    flp_set_error("%s: null pool or batch", who);
    return FLP_EINVAL;
  }
  if (b->n_seqs < 0 || b->max_blocks_per_seq < 0 || (b->n_seqs > 0 && (!b->cu_new || !b->prefix_len || !b->block_tables))) {
    flp_set_error("%s: bad sequence arrays", who);
    return FLP_EINVAL;
  }
  if ((p->cfg.block_tokens != 16 && p->cfg.block_tokens != 32) || (p->cfg.head_dim != 64 && p->cfg.head_dim != 128)) {
    flp_set_error("%s: kernels support block_tokens 16 or 32 and head_dim 64/128 (pool has %d / %d)", who,
                  p->cfg.block_tokens, p->cfg.head_dim);
    return FLP_ENOTSUP;
  }
  if (need_qo) {
    if (b->n_q_heads <= 0 || b->n_q_heads % p->cfg.n_kv_heads) {
      flp_set_error("%s: n_q_heads %d is not a multiple of n_kv_heads %d", who, b->n_q_heads, p->cfg.n_kv_heads);
      return FLP_EINVAL;
    }
  }
  if (b->n_seqs > 0 && b->cu_new[0] != 0) {
    flp_set_error("%s: cu_new[0] must be 0", who);
    return FLP_EINVAL;
  }
  const int64_t cap = (int64_t)b->max_blocks_per_seq * p->cfg.block_tokens;
  for (int32_t i = 0; i < b->n_seqs; ++i) {
    int64_t n = (int64_t)b->cu_new[i + 1] - b->cu_new[i];
    if (n < 0 || b->prefix_len[i] < 0) {
      flp_set_error("%s: sequence %d has negative length", who, i);
      return FLP_EINVAL;
    }
    if (b->prefix_len[i] + n > cap) {
      flp_set_error("%s: sequence %d needs %lld positions, its block table covers %lld", who, i,
                    (long long)(b->prefix_len[i] + n), (long long)cap);
      return FLP_ERANGE;
    }
  }
  const int32_t T = b->n_seqs > 0 ? b->cu_new[b->n_seqs] : 0;
  if (T > 0) {
    if (need_qo && (!b->q || !b->out || !aligned16(b->q) || !aligned16(b->out))) {
      flp_set_error("%s: q/out must be non-null and 16-byte aligned", who);
      return FLP_EINVAL;
    }
    if (need_kv && (!b->k_new || !b->v_new || !aligned16(b->k_new) || !aligned16(b->v_new))) {
      flp_set_error("%s: k_new/v_new must be non-null and 16-byte aligned", who);
      return FLP_EINVAL;
    }
  }
  return FLP_OK;
}

// device copies of cu_new / prefix_len plus a unit list, in one staging slot
struct StagedSeqs {
  FlpStageSlot* slot = nullptr;
  const int32_t* cu_new = nullptr;
  const int32_t* prefix_len = nullptr;
  const void* units = nullptr;
};

flp_status stage_seqs(flp_pool* p, const flp_attn_batch* b, const void* units, size_t unit_bytes, hipStream_t stream,
                      StagedSeqs* out) {
  const size_t S = (size_t)b->n_seqs;
  const size_t off_pl = (S + 1) * 4, off_units = ((off_pl + S * 4 + 31) / 32) * 32;
  const size_t bytes = off_units + unit_bytes;
  FLP_TRY(flp_stage_acquire(p, bytes, &out->slot));
  uint8_t* h = (uint8_t*)out->slot->host;
  memcpy(h, b->cu_new, (S + 1) * 4);
  memcpy(h + off_pl, b->prefix_len, S * 4);
  if (unit_bytes) memcpy(h + off_units, units, unit_bytes);
  FLP_TRY(flp_stage_upload(out->slot, bytes, stream));
  const uint8_t* d = (const uint8_t*)out->slot->dev;
  out->cu_new = (const int32_t*)d;
  out->prefix_len = (const int32_t*)(d + off_pl);
  out->units = d + off_units;
  return FLP_OK;
}

FlpAttnArgs make_args(const flp_pool* p, const flp_attn_batch* b, const StagedSeqs& st) {
  FlpAttnArgs a{};
  a.pool = p->dev_base;
  a.block_elems = p->block_elems;
  a.tables = b->block_tables;
  a.max_blocks = b->max_blocks_per_seq;
  a.n_h = b->n_q_heads;
  a.n_kv = p->cfg.n_kv_heads;
  a.bt = p->cfg.block_tokens;
  a.q = b->q;
  a.out = b->out;
  a.k_new = b->k_new;
  a.v_new = b->v_new;
  a.cu_new = st.cu_new;
  a.prefix_len = st.prefix_len;
  float sc = b->sm_scale > 0.f ? b->sm_scale : 1.0f / std::sqrt((float)p->cfg.head_dim);
  a.scale_log2e = sc * 1.4426950408889634f;
  return a;
}

flp_status append_locked(flp_pool* p, const flp_attn_batch* b, hipStream_t stream) {
  const int bt = 16;                                 // the kernel's unit is a group of 16 positions, whatever the block size
  std::vector<FlpAppendUnit> units;
  for (int32_t i = 0; i < b->n_seqs; ++i) {
    const int32_t P = b->prefix_len[i], n = b->cu_new[i + 1] - b->cu_new[i];
    int32_t pos = P;
    while (pos < P + n) {
      FlpAppendUnit u{};
      u.seq = i;
      u.blk_idx = pos / bt;
      u.s0 = pos % bt;
      u.s1 = std::min<int32_t>(bt, u.s0 + (P + n - pos));
      u.t_first = b->cu_new[i] + (pos - P);
      units.push_back(u);
      pos += u.s1 - u.s0;
    }
  }
  if (units.empty()) return FLP_OK;
  StagedSeqs st;
  FLP_TRY(stage_seqs(p, b, units.data(), units.size() * sizeof(FlpAppendUnit), stream, &st));
  FlpAttnArgs a = make_args(p, b, st);
  flp_status s1 = flp_launch_kv_append(p->cfg.dtype, p->cfg.head_dim, a, (const FlpAppendUnit*)st.units,
                                       (int32_t)units.size(), stream);
  flp_status s2 = flp_stage_release(st.slot, stream);
  return s1 != FLP_OK ? s1 : s2;
}

}  // namespace

extern "C" flp_status flp_kv_append(flp_pool* p, const flp_attn_batch* b, void* hip_stream) {
  FLP_TRY(check_attn_batch(p, b, false, true, "flp_kv_append"));
  std::lock_guard<std::mutex> lk(p->mu);
  return append_locked(p, b, (hipStream_t)hip_stream);
}

extern "C" flp_status flp_paged_prefix_attention(flp_pool* p, const flp_attn_batch* b, void* hip_stream) {
  const bool with_append = b && (b->k_new || b->v_new);
  FLP_TRY(check_attn_batch(p, b, true, with_append, "flp_paged_prefix_attention"));
  std::lock_guard<std::mutex> lk(p->mu);
  hipStream_t stream = (hipStream_t)hip_stream;
  if (with_append) FLP_TRY(append_locked(p, b, stream));

  // Two kinds of work.  Sequences with at least 8 query rows per kv head (prefill, or decode
  // under grouped-query attention) on a 16-bit pool with head_dim 128 go to the matrix-core
  // kernel in tiles of 256 rows; everything else (fp32, head_dim 64, single-row decode) goes to
  // the row-streaming kernel in runs of up to 4 tokens.  Both lists are ordered heaviest first.
  const bool mfma_ok = p->cfg.dtype != FLP_F32 && p->cfg.head_dim == 128;
  const int G = b->n_q_heads / p->cfg.n_kv_heads;
  const int n_kv = p->cfg.n_kv_heads;
  std::vector<int32_t> seq_order(b->n_seqs);
  std::iota(seq_order.begin(), seq_order.end(), 0);
  auto seq_cost = [&](int32_t i) {
    int64_t n = b->cu_new[i + 1] - b->cu_new[i];
    return n * (2 * (int64_t)b->prefix_len[i] + n);
  };
  std::stable_sort(seq_order.begin(), seq_order.end(), [&](int32_t x, int32_t y) { return seq_cost(x) > seq_cost(y); });

  std::vector<FlpAttnUnit> units;
  std::vector<int64_t> cost;
  constexpr int kTokPerUnit = 4;
  // A launch of a handful of matrix-core items (a few decode sequences under grouped-query attention) would leave
  // most of the chip idle: such sequences go to the row-streaming kernel instead, where their long contexts are
  // split over many waves (below).
  int64_t mfma_items_est = 0;
  if (mfma_ok)
    for (int32_t i = 0; i < b->n_seqs; ++i) {
      const int64_t n = b->cu_new[i + 1] - b->cu_new[i];
      if (G * n >= 8) mfma_items_est += (int64_t)n_kv * ((G * n + kMfmaRowsPerItem - 1) / kMfmaRowsPerItem);
    }
  const bool small_launch = mfma_items_est < 128;
  // matrix-core items: the row tiles of one (sequence, kv head) are dealt to ONE of 8 queues and
  // the queues are interleaved, so that under round-robin dispatch of workgroups over the 8
  // XCDs the tiles that re-read the same K/V run on the same XCD and share its L2.
  std::vector<FlpMfmaItem> queue[8];
  int next_q = 0;
  std::vector<int32_t> row_seqs;                      // sequences of the row-streaming kernel, heaviest first
  int64_t row_tokens = 0;
  for (int32_t i : seq_order) {
    const int32_t n = b->cu_new[i + 1] - b->cu_new[i];
    if (n <= 0) continue;
    const int64_t blocks_i = ((int64_t)b->prefix_len[i] + n + p->cfg.block_tokens - 1) / p->cfg.block_tokens;
    if (mfma_ok && (int64_t)G * n >= 8 && blocks_i <= kMfmaMaxBlocks && !(small_launch && n <= kTokPerUnit)) {
      const int32_t R = G * n;
      for (int g = 0; g < n_kv; ++g) {
        for (int32_t r0 = 0; r0 < R; r0 += kMfmaRowsPerItem)
          queue[next_q].push_back(FlpMfmaItem{i, g, r0, std::min<int32_t>(kMfmaRowsPerItem, R - r0)});
        next_q = (next_q + 1) & 7;
      }
    } else {
      row_seqs.push_back(i);
      row_tokens += n;
    }
  }
  // Split-KV.  The row kernel runs one wave per (token, head); with few rows and long contexts (a handful of decode
  // sequences at 16 k tokens) that is far fewer waves than the chip holds.  Below kSplitBelow waves every token
  // becomes a unit of its own and its context is cut into pieces of at least kMinGroups groups of 16 positions, each
  // piece a wave; a second kernel merges the pieces of a row in piece order.
  constexpr int64_t kSplitBelow = 2048, kSplitTarget = 8192;
  constexpr int kMinGroups = 16, kMaxSplit = 64;
  const int64_t row_waves = row_tokens * b->n_q_heads;
  const int want_split = row_waves > 0 && row_waves < kSplitBelow
                             ? (int)std::min<int64_t>(kMaxSplit, (kSplitTarget + row_waves - 1) / row_waves) : 1;
  std::vector<int32_t> merge_tok, merge_nsplit;
  int max_split = 1;
  for (int32_t i : row_seqs) {
    const int32_t n = b->cu_new[i + 1] - b->cu_new[i];
    if (want_split > 1) {
      for (int32_t j = 0; j < n; ++j) {
        const int32_t groups = (b->prefix_len[i] + j + 1 + 15) / 16;
        const int ns = std::max(1, std::min(want_split, groups / kMinGroups));
        if (ns == 1) {
          units.push_back(FlpAttnUnit{i, j, 1, 1, 0, 0, 0, 0});
          cost.push_back(groups);
          continue;
        }
        const int32_t row = (int32_t)merge_tok.size();
        merge_tok.push_back(b->cu_new[i] + j);
        merge_nsplit.push_back(ns);
        max_split = std::max(max_split, ns);
        for (int sidx = 0; sidx < ns; ++sidx) {
          const int32_t lo = (int32_t)((int64_t)groups * sidx / ns), hi = (int32_t)((int64_t)groups * (sidx + 1) / ns);
          units.push_back(FlpAttnUnit{i, j, 1, ns, sidx, lo, hi, row});
          cost.push_back(hi - lo);
        }
      }
    } else {
      for (int32_t j0 = 0; j0 < n; j0 += kTokPerUnit) {
        FlpAttnUnit u{i, j0, std::min(kTokPerUnit, n - j0), 1, 0, 0, 0, 0};
        units.push_back(u);
        cost.push_back((int64_t)u.n_tok * (b->prefix_len[i] + j0 + u.n_tok));
      }
    }
  }
  std::vector<int32_t> order(units.size());
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) { return cost[x] > cost[y]; });
  size_t qmax = 0;
  for (auto& q : queue) qmax = std::max(qmax, q.size());
  const size_t n_items = qmax * 8;
  if (units.empty() && n_items == 0) return FLP_OK;

  const size_t units_bytes = units.size() * sizeof(FlpAttnUnit), items_bytes = n_items * sizeof(FlpMfmaItem);
  const size_t n_merge = merge_tok.size();
  std::vector<uint8_t> blob(units_bytes + items_bytes + 2 * n_merge * sizeof(int32_t));
  FlpAttnUnit* hu = (FlpAttnUnit*)blob.data();
  for (size_t k = 0; k < order.size(); ++k) hu[k] = units[order[k]];
  FlpMfmaItem* hi = (FlpMfmaItem*)(blob.data() + units_bytes);
  for (size_t s = 0; s < qmax; ++s)
    for (int x = 0; x < 8; ++x) hi[8 * s + x] = s < queue[x].size() ? queue[x][s] : FlpMfmaItem{0, 0, 0, 0};
  if (n_merge) {
    int32_t* hm = (int32_t*)(blob.data() + units_bytes + items_bytes);
    memcpy(hm, merge_tok.data(), n_merge * sizeof(int32_t));
    memcpy(hm + n_merge, merge_nsplit.data(), n_merge * sizeof(int32_t));
  }
  void* partials = nullptr;
  if (n_merge)
    FLP_TRY(flp_attn_workspace(p, n_merge * (size_t)b->n_q_heads * max_split * (p->cfg.head_dim + 2) * sizeof(float),
                               &partials));

  StagedSeqs st;
  FLP_TRY(stage_seqs(p, b, blob.data(), blob.size(), stream, &st));
  FlpAttnArgs a = make_args(p, b, st);
  a.partials = (float*)partials;
  a.max_split = max_split;
  const FlpAttnUnit* du = (const FlpAttnUnit*)st.units;
  const FlpMfmaItem* di = (const FlpMfmaItem*)((const uint8_t*)st.units + units_bytes);
  const int32_t* dm = (const int32_t*)((const uint8_t*)st.units + units_bytes + items_bytes);
  flp_status s0 = flp_launch_attn_mfma(p->cfg.dtype, a, di, (int32_t)n_items, stream);
  flp_status s1 = flp_launch_attn_rows(p->cfg.dtype, p->cfg.head_dim, a, du, (int32_t)units.size(), stream);
  flp_status s3 = s1 == FLP_OK ? flp_launch_attn_merge(p->cfg.dtype, p->cfg.head_dim, a, dm, dm + n_merge,
                                                        (int32_t)n_merge, stream) : FLP_OK;
  flp_status s2 = flp_stage_release(st.slot, stream);
  return s0 != FLP_OK ? s0 : (s1 != FLP_OK ? s1 : (s3 != FLP_OK ? s3 : s2));
}

// ------------------------------------------------------------------------------- LoRA
extern "C" flp_status flp_lora_segment(flp_pool* p, int32_t n_tokens, const int32_t* token_adapter,
                                       int32_t n_adapters, int32_t* n_seg, int32_t* seg_adapter, int32_t* seg_start,
                                       int32_t* perm, void* hip_stream) {
  if (!p || n_tokens < 0 || n_adapters < 0 || !n_seg || !seg_adapter || !seg_start || (n_tokens > 0 && (!token_adapter || !perm))) {
    flp_set_error("flp_lora_segment: invalid argument");
    return FLP_EINVAL;
  }
  if (n_adapters > 2048) {
    flp_set_error("flp_lora_segment: %d adapters, at most 2048 supported", n_adapters);
    return FLP_ERANGE;
  }
  return flp_launch_lora_segment(n_tokens, token_adapter, n_adapters, n_seg, seg_adapter, seg_start, perm, 0, nullptr, 0,
                                 nullptr, (hipStream_t)hip_stream);
}

namespace {
flp_status lora_apply_impl(flp_pool* p, const flp_lora_batch* b, void* hip_stream, void* gated_out, int64_t ld_gated,
                           const FlpFixedWorkspace* fixed = nullptr);
}

extern "C" flp_status flp_lora_apply_paged(flp_pool* p, const flp_lora_batch* b, void* hip_stream) {
  return lora_apply_impl(p, b, hip_stream, nullptr, 0);
}

flp_status flp_lora_apply_fixed(flp_pool* p, const flp_lora_batch* b, void* hip_stream, const FlpFixedWorkspace& ws) {
  return lora_apply_impl(p, b, hip_stream, nullptr, 0, &ws);
}

flp_status flp_lora_apply_gated(flp_pool* p, const flp_lora_batch* b, void* out, int64_t ld_out, void* hip_stream) {
  if (!out || ((uintptr_t)out & 15)) {
    flp_set_error("flp_lora_apply_gated: out is null or misaligned");
    return FLP_EINVAL;
  }
  return lora_apply_impl(p, b, hip_stream, out, ld_out);
}

namespace {
// gated_out != nullptr: two projections (gate, up) whose results are not stored; gated_out = silu(y0) * y1
// fixed != nullptr: the intermediates go into the caller-provided buffer and nothing is allocated; a batch that
// needs more than the buffer holds is refused before anything is enqueued
flp_status lora_apply_impl(flp_pool* p, const flp_lora_batch* b, void* hip_stream, void* gated_out, int64_t ld_gated,
                           const FlpFixedWorkspace* fixed) {
  if (!p || !b) {
    flp_set_error("flp_lora_apply_paged: null pool or batch");
    return FLP_EINVAL;
  }
  if (b->n_tokens < 0 || b->n_proj < 1 || b->n_proj > FLP_MAX_PROJ || b->n_adapters < 0 || b->d_in <= 0 ||
      b->ld_x < b->d_in) {
    flp_set_error("flp_lora_apply_paged: bad sizes (n_tokens=%d n_proj=%d n_adapters=%d d_in=%d ld_x=%lld)",
                  b->n_tokens, b->n_proj, b->n_adapters, b->d_in, (long long)b->ld_x);
    return FLP_EINVAL;
  }
  if (b->n_tokens == 0) return FLP_OK;
  if (b->max_rank < 1 || b->max_rank > 64) {
    flp_set_error("flp_lora_apply_paged: max_rank %d outside 1..64", b->max_rank);
    return FLP_ERANGE;
  }
  if (b->n_adapters > 2048) {
    flp_set_error("flp_lora_apply_paged: %d adapters, at most 2048 supported", b->n_adapters);
    return FLP_ERANGE;
  }
  const int epl = 16 / p->elem_bytes;
  if (!b->x || !b->token_adapter || !b->rank || !b->scale || !b->block_tables || !aligned16(b->x) ||
      b->d_in % epl || b->ld_x % epl || b->d_in > p->block_elems) {
    flp_set_error("flp_lora_apply_paged: x/metadata null or misaligned, or d_in %d not a multiple of %d / larger than a block",
                  b->d_in, epl);
    return FLP_EINVAL;
  }
  for (int q = 0; q < b->n_proj; ++q) {
    const flp_lora_proj& pr = b->proj[q];
    if (pr.w_base_layout != 0 && pr.w_base_layout != 1) {
      flp_set_error("flp_lora_apply_paged: projection %d: w_base_layout %d is neither 0 nor 1", q, pr.w_base_layout);
      return FLP_EINVAL;
    }
    if (pr.d_out <= 0 || pr.ld_y < pr.d_out || pr.d_out % epl || pr.ld_y % epl || pr.d_out > p->block_elems || !pr.y ||
        !aligned16(pr.y) || !pr.a_tab_off || !pr.a_row_base || !pr.b_tab_off || !pr.b_row_base) {
      flp_set_error("flp_lora_apply_paged: projection %d has bad sizes or null/misaligned pointers", q);
      return FLP_EINVAL;
    }
    if (pr.w_base && (!aligned16(pr.w_base) || (p->elem_bytes == 2 && b->d_in % 64))) {
      flp_set_error("flp_lora_apply_paged: projection %d: w_base misaligned, or d_in %d not a multiple of 64", q,
                    b->d_in);
      return pr.w_base && aligned16(pr.w_base) ? FLP_ENOTSUP : FLP_EINVAL;
    }
  }
  std::lock_guard<std::mutex> lk(p->mu);
  hipStream_t stream = (hipStream_t)hip_stream;
  const size_t T = (size_t)b->n_tokens;

  // Matrix-core path for 16-bit pools when every width is a multiple of the tile widths (32 in, 64 out) and
  // the batch is large enough for token tiles to fill (prefill); otherwise the vector-ALU
  // kernels: fp32 pools, odd widths, and small decode batches, where a segment is a handful of
  // tokens and the per-token kernels (measured on 256 tokens over 92 adapters: 0.11 ms against
  // 0.20 ms for q/k/v) win because they need fewer dependent round trips per wave.
  bool mfma_ok = p->cfg.dtype != FLP_F32 && b->d_in % 32 == 0 && b->n_tokens >= 1024;
  int max_dout = 0;
  for (int q = 0; q < b->n_proj; ++q) {
    mfma_ok = mfma_ok && b->proj[q].d_out % 64 == 0;
    max_dout = std::max(max_dout, b->proj[q].d_out);
  }
  FlpLoraMfma c{};
  size_t v_elems = T * b->n_proj * b->max_rank;
  if (mfma_ok) {
    c.mt = b->n_tokens >= 2048 ? 2 : 1;
    const int tm = 16 * c.mt;
    // The number of segments is only known on the device.  The bounds (every adapter present, each adding a
    // partly filled tile) size the buffers; the launches cover the tiles of up to 64 present adapters in one
    // pass and loop for the rest, so that a pool of thousands of adapters does not launch thousands of
    // workgroups that find nothing to do.
    const int32_t seg_bound = (int32_t)std::min<size_t>((size_t)b->n_adapters, T);
    c.tiles_bound = (int32_t)((T + tm - 1) / tm) + seg_bound;
    c.tiles_grid = (std::min(c.tiles_bound, (int32_t)((T + tm - 1) / tm) + 64) + 7) / 8 * 8;
    // split K until enough workgroups are in flight, in pieces of 128 coefficients: about 2048 for the kernel
    // that reads its operands from global memory (it lives on loads in flight), about 1024 for the LDS-staged
    // ones (they keep three chunks in flight themselves; fewer partial sums for the expand kernel to add)
    const int wg_target = (c.mt == 2 && b->d_in % 64 == 0) ? 1024 : 2048;
    int ks = 1;
    while (ks < 8 && c.tiles_grid * ks < wg_target && b->d_in / (ks * 2) >= 256) ks *= 2;
    c.k_splits = ks;
    c.k_per_split = ((b->d_in + ks - 1) / ks + 127) / 128 * 128;
    c.v_rows = c.tiles_bound * tm;
    const int nt = (b->max_rank + 15) / 16 <= 2 ? (b->max_rank + 15) / 16 : 4;
    // long segments: wide slabs amortise the gathered B fragments over many tokens; short ones
    // (decode): narrow slabs, i.e. more waves, each gathering one piece
    c.cols_per_slab = c.mt == 2 ? 256 : 256 / nt;
    c.group_tokens = tm * (c.mt == 2 ? 8 : 1);
    c.groups_bound = (int32_t)((T + c.group_tokens - 1) / c.group_tokens) + seg_bound;
    c.groups_grid = (std::min(c.groups_bound, (int32_t)((T + c.group_tokens - 1) / c.group_tokens) + 64) + 7) / 8 * 8;
    const int rp = 16 * nt;
    v_elems = (size_t)ks * c.v_rows * b->n_proj * rp;
  }
  // Dense base on every projection, and every product large enough for the large-batch GEMM: the expand step runs
  // as that kernel's epilogue (segment, shrink, then one GEMM per projection that adds the LoRA branch to its
  // accumulators before it rounds): no fp32 copy of the product, no second pass over y.
  // (Batches of 2048 tokens and more only: the epilogue walks the adapters present among a wave's 128 tokens, which
  // are one or two when tokens come in sequences and up to 128 in a large pure-decode batch.)
  bool fused = mfma_ok && b->n_tokens >= 2048;
  for (int q = 0; q < b->n_proj; ++q)
    fused = fused && b->proj[q].w_base &&
            flp_gemm_is_large(p->cfg.dtype, b->n_tokens, b->proj[q].d_out, b->d_in, b->ld_x);
  if (gated_out) {
    const bool ok = fused && b->n_proj == 2 && b->proj[0].d_out == b->proj[1].d_out && b->proj[0].w_base_layout == 1 &&
                    b->proj[1].w_base_layout == 1 && ld_gated >= b->proj[0].d_out && ld_gated % epl == 0 &&
                    flp_gemm_gated_fits(p->cfg.dtype, b->n_tokens, b->proj[0].d_out, b->d_in, b->ld_x);
    if (!ok) return FLP_ENOTSUP;                // nothing launched: the caller takes the separate products
  }
  size_t wt_bytes = 0;                         // transposed copy of the widest dense base matrix
  if (p->elem_bytes == 2)
    for (int q = 0; q < b->n_proj; ++q)
      if (b->proj[q].w_base && b->proj[q].w_base_layout == 0)
        wt_bytes = std::max(wt_bytes, (size_t)b->d_in * b->proj[q].d_out * 2);
  wt_bytes = (wt_bytes + 255) & ~(size_t)255;
  size_t base_bytes[FLP_MAX_PROJ] = {0, 0, 0, 0}, base_total = 0;   // unrounded base terms (16-bit pools)
  if (p->elem_bytes == 2 && !fused)
    for (int q = 0; q < b->n_proj; ++q)
      if (b->proj[q].w_base) {
        base_bytes[q] = (T * b->proj[q].d_out * 4 + 255) & ~(size_t)255;
        base_total += base_bytes[q];
      }
  size_t splitk_bytes = 0;                     // slices of the dense product of a small batch
  for (int q = 0; q < b->n_proj; ++q)
    if (b->proj[q].w_base && p->elem_bytes == 2)
      splitk_bytes = std::max(splitk_bytes, flp_gemm_splitk_bytes(b->n_tokens, b->proj[q].d_out));
  splitk_bytes = (splitk_bytes + 255) & ~(size_t)255;
  const size_t v_bytes = (v_elems * 4 + 255) & ~(size_t)255;
  const size_t seg_bytes = ((size_t)(4 * b->n_adapters + 5) * 4 + 255) & ~(size_t)255;
  const size_t perm_bytes = (T * 4 + 255) & ~(size_t)255;
  // token -> position in segment order, adapter -> first row of its tokens in the shrink output
  const size_t inv_bytes = fused ? perm_bytes + (((size_t)b->n_adapters * 4 + 255) & ~(size_t)255) : 0;
  void* ws = nullptr;
  const size_t ws_bytes = v_bytes + seg_bytes + perm_bytes + wt_bytes + base_total + splitk_bytes + inv_bytes;
  if (fixed) {
    if (ws_bytes > fixed->cap) {
      flp_set_error("%s: the batch needs %zu bytes of intermediates, the fixed buffer holds %zu (fewer tokens, a lower "
                    "max_rank or no dense base make it fit)", fixed->who, ws_bytes, fixed->cap);
      return FLP_ENOSPC;
    }
    FLP_TRY(fixed->resolve(p, &ws));
  } else {
    FLP_TRY(flp_workspace(p, ws_bytes, &ws));
  }
  FlpLoraArgs a{};
  a.pool = p->dev_base;
  a.block_elems = p->block_elems;
  a.T = b->n_tokens;
  a.d_in = b->d_in;
  a.n_adapters = b->n_adapters;
  a.max_rank = b->max_rank;
  a.n_proj = b->n_proj;
  a.ld_x = b->ld_x;
  a.x = b->x;
  a.token_adapter = b->token_adapter;
  a.rank = b->rank;
  a.scale = b->scale;
  a.tables = b->block_tables;
  for (int q = 0; q < b->n_proj; ++q) a.proj[q] = b->proj[q];
  uint8_t* w = (uint8_t*)ws;
  a.v = (float*)w;
  a.n_seg = (int32_t*)(w + v_bytes);
  a.seg_adapter = a.n_seg + 1;
  a.seg_start = a.seg_adapter + b->n_adapters;
  a.tile_start = a.seg_start + b->n_adapters + 1;
  a.group_start = a.tile_start + b->n_adapters + 1;
  a.perm = (int32_t*)(w + v_bytes + seg_bytes);
  if (fused) {
    int32_t* inv_perm = (int32_t*)(w + v_bytes + seg_bytes + perm_bytes + wt_bytes + base_total + splitk_bytes);
    uint8_t* wt = w + v_bytes + seg_bytes + perm_bytes;
    int32_t* vrow_base = (int32_t*)((uint8_t*)inv_perm + perm_bytes);
    FLP_TRY(flp_launch_lora_segment(a.T, a.token_adapter, a.n_adapters, a.n_seg, a.seg_adapter, a.seg_start, a.perm,
                                    16 * c.mt, a.tile_start, c.group_tokens, a.group_start, stream, inv_perm, vrow_base));
    c.shrink_only = 1;
    FLP_TRY(flp_launch_lora_mfma(p->cfg.dtype, a, c, stream));
    const int nt = (b->max_rank + 15) / 16 <= 2 ? (b->max_rank + 15) / 16 : 4;
    auto branch = [&](int q) {
      FlpGemmLora lp{};
      lp.token_adapter = a.token_adapter;
      lp.rank = a.rank;
      lp.scale = a.scale;
      lp.tables = a.tables;
      lp.b_tab_off = b->proj[q].b_tab_off;
      lp.b_row_base = b->proj[q].b_row_base;
      lp.pool = a.pool;
      lp.block_elems = a.block_elems;
      lp.v = a.v;
      lp.v_rows = c.v_rows;
      lp.k_splits = c.k_splits;
      lp.n_proj = b->n_proj;
      lp.p = q;
      lp.rp = 16 * nt;
      lp.n_adapters = b->n_adapters;
      lp.max_rank = b->max_rank < 16 * nt ? b->max_rank : 16 * nt;
      lp.inv_perm = inv_perm;
      lp.vrow_base = vrow_base;
      return lp;
    };
    if (gated_out) {
      const FlpGemmLora lg = branch(0), lu = branch(1);
      return flp_launch_gated_gemm(p->cfg.dtype, b->x, b->ld_x, b->proj[0].w_base, b->proj[1].w_base, gated_out, ld_gated,
                                   b->n_tokens, b->proj[0].d_out, b->d_in, stream, &lg, &lu);
    }
    for (int q = 0; q < b->n_proj; ++q) {
      const FlpGemmLora lp = branch(q);
      FLP_TRY(flp_launch_base_gemm(p->cfg.dtype, b->x, b->ld_x, b->proj[q].w_base, b->proj[q].w_base_layout,
                                   b->proj[q].y, b->proj[q].ld_y, b->n_tokens, b->proj[q].d_out, b->d_in, wt, nullptr,
                                   nullptr, 0, stream, &lp));
    }
    return FLP_OK;
  }
  // base term first where the caller asked for it (x . W_base), then the adapters' deltas on top.
  // 16-bit pools also keep the product unrounded in the workspace so that base + delta is rounded
  // once; tokens without an adapter keep the rounded value that the GEMM wrote into y.
  {
    uint8_t* wt = w + v_bytes + seg_bytes + perm_bytes;
    uint8_t* basep = wt + wt_bytes;
    float* splitk = splitk_bytes ? (float*)(basep + base_total) : nullptr;
    for (int q = 0; q < b->n_proj; ++q) {
      if (!b->proj[q].w_base) continue;
      float* y32 = p->elem_bytes == 2 ? (float*)basep : nullptr;
      FLP_TRY(flp_launch_base_gemm(p->cfg.dtype, b->x, b->ld_x, b->proj[q].w_base, b->proj[q].w_base_layout,
                                   b->proj[q].y, b->proj[q].ld_y, b->n_tokens, b->proj[q].d_out, b->d_in, wt, y32,
                                   splitk, splitk_bytes, stream));
      a.base32[q] = y32;
      basep += base_bytes[q];
    }
  }
  if (!mfma_ok) return flp_launch_lora_simple(p->cfg.dtype, a, stream);
  FLP_TRY(flp_launch_lora_segment(a.T, a.token_adapter, a.n_adapters, a.n_seg, a.seg_adapter, a.seg_start, a.perm,
                                  16 * c.mt, a.tile_start, c.group_tokens, a.group_start, stream));
  return flp_launch_lora_mfma(p->cfg.dtype, a, c, stream);
}
}  // namespace
