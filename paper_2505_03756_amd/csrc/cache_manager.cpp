// Host logic behind flcache.h: the usage-dependency tree of the cache manager (paper sections
// 4.1-4.3) and the cost-model swapper (sections 5.1-5.3, Eq. 3-6), with the paper's ablation
// switches (sections 6.6-6.8).  No device work: the block lists decided here are executed by
// flp_pool_swap_in / flp_pool_swap_out.
//
// Nodes live in a deque indexed by their id (ids are creation order and never reused, so ties in
// the cost model can go to the older node).  Children are found through one hash table keyed by
// (parent id, hash of the child's label), labels compared in full on a hit.  Each node counts its
// children per tier, which makes "has no child in HBM" (the leaf rule of swap-out) and "parent is
// in HBM" (the root rule of swap-in) O(1); a tick scans the nodes once for the initial candidates
// and then works from a heap, adding the parent (swap-out) or the host children (swap-in) of every
// node it moves.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <deque>
#include <mutex>
#include <queue>
#include <unordered_map>
#include <vector>

#include "flcache.h"
#include "flp_internal.h"

namespace {

enum : int32_t { kHbm = 0, kHost = 1 };
enum : int32_t { kLora = 0, kKv = 1 };

struct Node {
  int32_t id = 0, kind = kLora, parent = 0, tier = kHbm;
  int32_t lora_id = 0;                   // label of a LoRA node
  std::vector<int32_t> tokens;           // label of a KV node (block_tokens ids)
  std::vector<int32_t> blocks;           // ids on `tier`
  std::vector<int32_t> children;         // node ids, in creation order
  int32_t n_child_tier[2] = {0, 0};
  int32_t pins = 0;
  int64_t visits = 0;
  double last_use = 0.0;
  bool alive = true;
  uint64_t key = 0;                      // hash-table key under which the node is filed
};

uint64_t mix(uint64_t h, uint64_t v) {
  h ^= v + 0x9e3779b97f4a7c15ull + (h << 6) + (h >> 2);
  h *= 0xff51afd7ed558ccdull;
  return h ^ (h >> 33);
}

}  // namespace

struct flc_cache {
  flp_pool* pool = nullptr;
  flc_config cfg{};
  int64_t n_dev = 0;
  std::deque<Node> nodes;                // nodes[0] is the virtual root
  std::unordered_map<uint64_t, std::vector<int32_t>> index;   // key -> node ids filed under it
  int64_t n_queries = 0, next_query = 1;
  std::unordered_map<int64_t, std::vector<int32_t>> running;  // query -> pinned path
  std::mutex mu;

  uint64_t lora_key(int32_t lora_id) const { return mix(0x1234567ull, (uint64_t)(uint32_t)lora_id); }
  uint64_t kv_key(int32_t parent, const int32_t* tok) const {
    uint64_t h = mix(0xabcdefull, (uint64_t)parent);
    for (int i = 0; i < cfg.block_tokens; ++i) h = mix(h, (uint64_t)(uint32_t)tok[i]);
    return h;
  }
  int32_t find_lora(int32_t lora_id) const {
    auto it = index.find(lora_key(lora_id));
    if (it == index.end()) return -1;
    for (int32_t id : it->second)
      if (nodes[id].kind == kLora && nodes[id].lora_id == lora_id) return id;
    return -1;
  }
  int32_t find_kv(int32_t parent, const int32_t* tok) const {
    auto it = index.find(kv_key(parent, tok));
    if (it == index.end()) return -1;
    for (int32_t id : it->second) {
      const Node& n = nodes[id];
      if (n.kind == kKv && n.parent == parent &&
          std::memcmp(n.tokens.data(), tok, sizeof(int32_t) * (size_t)cfg.block_tokens) == 0)
        return id;
    }
    return -1;
  }
  Node& new_node(int32_t kind, int32_t parent, int32_t tier, double now, uint64_t key) {
    nodes.emplace_back();
    Node& n = nodes.back();
    n.id = (int32_t)nodes.size() - 1;
    n.kind = kind;
    n.parent = parent;
    n.tier = tier;
    n.last_use = now;
    n.key = key;
    index[key].push_back(n.id);
    nodes[parent].children.push_back(n.id);
    nodes[parent].n_child_tier[tier]++;
    return n;
  }
  void set_tier(Node& n, int32_t tier) {
    nodes[n.parent].n_child_tier[n.tier]--;
    n.tier = tier;
    nodes[n.parent].n_child_tier[tier]++;
  }
  double usage() const { return 1.0 - (double)flp_pool_num_free(pool, kHbm) / (double)n_dev; }

  // ---- cost model (section 5)
  double prob(const Node& n) const { return n_queries ? (double)n.visits / (double)n_queries : 0.0; }
  double low_lora(int32_t batch_size) const {        // Eq. 3 (LoRA nodes in id order)
    double s = 0.0;
    for (int32_t id : nodes[0].children) s += 1.0 - std::pow(1.0 - prob(nodes[id]), (double)batch_size);
    return s;
  }
  int64_t now_lora() const { return nodes[0].n_child_tier[kHbm]; }
  static double lora_eval(double low, int64_t now_lora) {   // Eq. 4
    const double r = low / (double)(now_lora > 1 ? now_lora : 1);
    return r > 1.0 ? r : 1.0;
  }
  double retain_eval(const Node& n, double now) const {     // Eq. 5
    const double cost = (double)n.blocks.size() * (double)pool->block_bytes / cfg.pcie_bytes_per_s;
    const double t = (now - n.last_use) / cfg.time_scale_s;
    return cost * prob(n) * (1.0 - 1.0 / (1.0 + std::exp(-t)));
  }
  double eval(const Node& n, double now, double low, int64_t n_lora) const {   // Eq. 6
    if (cfg.use_lru) return n.last_use;
    const double reward = (n.kind == kLora && !cfg.no_lora_reward) ? lora_eval(low, n_lora) : 1.0;
    return reward * retain_eval(n, now);
  }

  bool out_candidate(const Node& n) const {
    return n.alive && n.id != 0 && n.tier == kHbm && n.pins == 0 && (cfg.ignore_dependencies || n.n_child_tier[kHbm] == 0);
  }
  bool in_candidate(const Node& n) const {
    return n.alive && n.id != 0 && n.tier == kHost &&
           (cfg.ignore_dependencies || n.parent == 0 || nodes[n.parent].tier == kHbm);
  }

  // Forget n and everything below it.  n's own blocks must already be back in the free list;
  // the descendants' blocks are returned here, in pre-order by id.
  void drop(int32_t top, std::vector<int32_t>* gone) {
    std::vector<int32_t> stack{top};
    bool first = true;
    while (!stack.empty()) {
      const int32_t id = stack.back();
      stack.pop_back();
      Node& m = nodes[id];
      std::vector<int32_t> ch = m.children;
      std::sort(ch.begin(), ch.end(), [](int32_t a, int32_t b) { return a > b; });
      for (int32_t c : ch) stack.push_back(c);
      if (!first && !m.blocks.empty()) (void)flp_pool_free(pool, m.tier, (int32_t)m.blocks.size(), m.blocks.data());
      first = false;
      gone->push_back(id);
      auto& bucket = index[m.key];
      bucket.erase(std::remove(bucket.begin(), bucket.end(), id), bucket.end());
      if (bucket.empty()) index.erase(m.key);
      m.alive = false;
      m.children.clear();
      m.blocks.clear();
      m.tokens.clear();
    }
    Node& n = nodes[top];
    Node& par = nodes[n.parent];
    par.children.erase(std::remove(par.children.begin(), par.children.end(), top), par.children.end());
    par.n_child_tier[n.tier]--;
  }
};

#define FLC_CHECK(cond, code, ...)   \
  do {                               \
    if (!(cond)) {                   \
      flp_set_error(__VA_ARGS__);    \
      return code;                   \
    }                                \
  } while (0)

extern "C" flp_status flc_create(flp_pool* pool, const flc_config* cfg, flc_cache** out) {
  FLC_CHECK(pool && cfg && out, FLP_EINVAL, "flc_create: null argument");
  FLC_CHECK(cfg->block_tokens > 0 && cfg->pcie_bytes_per_s > 0 && cfg->time_scale_s > 0 && cfg->lower <= cfg->upper,
            FLP_EINVAL, "flc_create: block_tokens, bandwidth and time scale must be positive, lower <= upper");
  FLC_CHECK(cfg->block_tokens == pool->cfg.block_tokens, FLP_EINVAL, "flc_create: block_tokens %d differs from the pool's %d",
            cfg->block_tokens, pool->cfg.block_tokens);
  FLC_CHECK(pool->cfg.n_dev_blocks > 0, FLP_EINVAL, "flc_create: the pool has no HBM tier");
  flc_cache* c = new flc_cache();
  c->pool = pool;
  c->cfg = *cfg;
  c->n_dev = pool->cfg.n_dev_blocks;
  c->nodes.emplace_back();               // virtual root
  *out = c;
  return FLP_OK;
}

extern "C" flp_status flc_destroy(flc_cache* c) {
  if (!c) return FLP_OK;
  // the blocks that the nodes still hold go back to the pool, which outlives the cache
  for (const Node& n : c->nodes)
    if (n.alive && !n.blocks.empty()) (void)flp_pool_free(c->pool, n.tier, (int32_t)n.blocks.size(), n.blocks.data());
  delete c;
  return FLP_OK;
}

extern "C" flp_status flc_add_lora(flc_cache* c, int32_t lora_id, int32_t n_blocks, int32_t tier, double now,
                                   int32_t* out_ids) {
  FLC_CHECK(c && out_ids && n_blocks > 0 && (tier == kHbm || tier == kHost), FLP_EINVAL, "flc_add_lora: invalid argument");
  std::lock_guard<std::mutex> lk(c->mu);
  FLC_CHECK(c->find_lora(lora_id) < 0, FLP_EDUP, "flc_add_lora: LoRA %d is already in the tree", lora_id);
  FLP_TRY(flp_pool_alloc(c->pool, tier, n_blocks, out_ids));
  Node& n = c->new_node(kLora, 0, tier, now, c->lora_key(lora_id));
  n.lora_id = lora_id;
  n.blocks.assign(out_ids, out_ids + n_blocks);
  return FLP_OK;
}

extern "C" flp_status flc_match(flc_cache* c, int32_t lora_id, const int32_t* tokens, int32_t n_tokens, double now,
                                int64_t* query, int32_t* lora_blocks, int32_t lora_cap, int32_t* n_lora_blocks,
                                int32_t* kv_blocks, int32_t kv_cap, int32_t* n_kv_blocks, int32_t* swap_host,
                                int32_t* swap_dev, int32_t swap_cap, int32_t* n_swap) {
  FLC_CHECK(c && query && n_lora_blocks && n_kv_blocks && n_swap && n_tokens >= 0 && (n_tokens == 0 || tokens) &&
                lora_cap >= 0 && kv_cap >= 0 && swap_cap >= 0 && (lora_cap == 0 || lora_blocks) &&
                (kv_cap == 0 || kv_blocks) && (swap_cap == 0 || (swap_host && swap_dev)),
            FLP_EINVAL, "flc_match: invalid argument");
  std::lock_guard<std::mutex> lk(c->mu);
  const int32_t lora = c->find_lora(lora_id);
  FLC_CHECK(lora >= 0, FLP_EINVAL, "flc_match: LoRA %d is not in the tree (flc_add_lora first)", lora_id);
  const int bt = c->cfg.block_tokens;
  const int32_t n_blk = n_tokens / bt;
  const int64_t lora_n = (int64_t)c->nodes[lora].blocks.size();
  FLC_CHECK(lora_cap >= lora_n && kv_cap >= n_blk && swap_cap >= lora_n + n_blk, FLP_ERANGE,
            "flc_match: output arrays too small (%lld LoRA blocks, up to %d KV blocks)", (long long)lora_n, n_blk);
  std::vector<int32_t> path{lora};
  for (int32_t b = 0, node = lora; b < n_blk; ++b) {
    const int32_t child = c->find_kv(node, tokens + (size_t)b * bt);
    if (child < 0) break;
    path.push_back(child);
    node = child;
  }
  c->n_queries++;
  for (int32_t id : path) {
    c->nodes[id].visits++;
    c->nodes[id].last_use = now;
  }
  std::vector<int32_t> usable;
  int32_t ns = 0;
  std::vector<int32_t> ids;
  for (int32_t id : path) {
    Node& n = c->nodes[id];
    if (n.tier == kHost) {
      ids.resize(n.blocks.size());
      if (flp_pool_alloc(c->pool, kHbm, (int32_t)ids.size(), ids.data()) != FLP_OK) break;
      for (size_t k = 0; k < ids.size(); ++k) {
        swap_host[ns] = n.blocks[k];
        swap_dev[ns] = ids[k];
        ++ns;
      }
      (void)flp_pool_free(c->pool, kHost, (int32_t)n.blocks.size(), n.blocks.data());
      c->set_tier(n, kHbm);
      n.blocks = ids;
    }
    usable.push_back(id);
  }
  for (int32_t id : usable) c->nodes[id].pins++;
  *n_swap = ns;
  if (usable.empty()) {
    *n_lora_blocks = -1;
    *n_kv_blocks = 0;
  } else {
    const Node& l = c->nodes[lora];
    std::copy(l.blocks.begin(), l.blocks.end(), lora_blocks);
    *n_lora_blocks = (int32_t)l.blocks.size();
    for (size_t k = 1; k < usable.size(); ++k) kv_blocks[k - 1] = c->nodes[usable[k]].blocks[0];
    *n_kv_blocks = (int32_t)usable.size() - 1;
  }
  *query = c->next_query++;
  c->running[*query] = std::move(usable);
  return FLP_OK;
}

extern "C" flp_status flc_insert(flc_cache* c, int64_t query, const int32_t* tokens, int32_t n_tokens,
                                 const int32_t* new_blocks, int32_t n_new, double now, int32_t* not_taken,
                                 int32_t* n_not_taken) {
  FLC_CHECK(c && n_not_taken && n_new >= 0 && n_tokens >= 0 && (n_new == 0 || (new_blocks && not_taken && tokens)),
            FLP_EINVAL, "flc_insert: invalid argument");
  std::lock_guard<std::mutex> lk(c->mu);
  auto it = c->running.find(query);
  FLC_CHECK(it != c->running.end(), FLP_EINVAL, "flc_insert: unknown query %lld", (long long)query);
  std::vector<int32_t>& path = it->second;
  const int bt = c->cfg.block_tokens;
  int32_t nt = 0;
  if (path.empty()) {                    // the query holds nothing (its LoRA is not resident)
    for (int32_t j = 0; j < n_new; ++j) not_taken[nt++] = new_blocks[j];
    *n_not_taken = nt;
    return FLP_OK;
  }
  const int32_t first = (int32_t)path.size() - 1;
  FLC_CHECK((int64_t)(first + n_new) * bt <= n_tokens, FLP_EINVAL,
            "flc_insert: %d tokens do not cover %d held + %d new blocks of %d", n_tokens, first, n_new, bt);
  for (int32_t j = 0; j < n_new; ++j) {
    const int32_t blk = new_blocks[j];
    FLC_CHECK(blk >= 0 && blk < c->n_dev, FLP_ERANGE, "flc_insert: block id %d out of range", blk);
  }
  int32_t node = path.back();
  for (int32_t j = 0; j < n_new; ++j) {
    const int32_t* tok = tokens + (size_t)(first + j) * bt;
    int32_t child = c->find_kv(node, tok);
    if (child < 0) {
      Node& n = c->new_node(kKv, node, kHbm, now, c->kv_key(node, tok));
      n.tokens.assign(tok, tok + bt);
      n.blocks.assign(1, new_blocks[j]);
      n.visits = 1;
      child = n.id;
    } else if (c->nodes[child].tier == kHbm) {
      not_taken[nt++] = new_blocks[j];   // somebody else inserted the same continuation first
      c->nodes[child].visits++;
      c->nodes[child].last_use = now;
    } else {
      // the same continuation exists on the host tier: a resident chain cannot go on below it
      for (int32_t k = j; k < n_new; ++k) not_taken[nt++] = new_blocks[k];
      break;
    }
    c->nodes[child].pins++;
    path.push_back(child);
    node = child;
  }
  *n_not_taken = nt;
  return FLP_OK;
}

extern "C" flp_status flc_release(flc_cache* c, int64_t query) {
  FLC_CHECK(c, FLP_EINVAL, "flc_release: null cache");
  std::lock_guard<std::mutex> lk(c->mu);
  auto it = c->running.find(query);
  FLC_CHECK(it != c->running.end(), FLP_EINVAL, "flc_release: unknown query %lld", (long long)query);
  for (int32_t id : it->second) c->nodes[id].pins--;
  c->running.erase(it);
  return FLP_OK;
}

extern "C" flp_status flc_tick(flc_cache* c, double now, int32_t batch_size, int32_t* out_dev, int32_t* out_host,
                               int32_t out_cap, int32_t* n_out, int32_t* in_host, int32_t* in_dev, int32_t in_cap,
                               int32_t* n_in, int32_t* dropped, int32_t drop_cap, int32_t* n_dropped) {
  FLC_CHECK(c && n_out && n_in && n_dropped && batch_size >= 0 && out_cap >= 0 && in_cap >= 0 && drop_cap >= 0 &&
                (out_cap == 0 || (out_dev && out_host)) && (in_cap == 0 || (in_host && in_dev)) &&
                (drop_cap == 0 || dropped),
            FLP_EINVAL, "flc_tick: invalid argument");
  std::lock_guard<std::mutex> lk(c->mu);
  *n_out = *n_in = *n_dropped = 0;
  const double low = c->low_lora(batch_size);
  const int64_t n_lora = c->now_lora();
  typedef std::pair<double, int32_t> Item;       // (Eval or its negative, id): smallest first, older node on ties
  std::priority_queue<Item, std::vector<Item>, std::greater<Item>> heap;
  std::vector<int32_t> ids, gone;
  if (c->usage() > c->cfg.upper) {
    for (const Node& n : c->nodes)
      if (c->out_candidate(n)) heap.push(Item(c->eval(n, now, low, n_lora), n.id));
    while (c->usage() > c->cfg.upper && !heap.empty()) {
      const int32_t id = heap.top().second;
      heap.pop();
      Node& n = c->nodes[id];
      if (!c->out_candidate(n)) continue;        // moved or forgotten since it was queued
      const int32_t nb = (int32_t)n.blocks.size();
      if (*n_out + nb > out_cap) break;
      ids.resize((size_t)nb);
      const bool host_ok = flp_pool_alloc(c->pool, kHost, nb, ids.data()) == FLP_OK;
      (void)flp_pool_free(c->pool, kHbm, nb, n.blocks.data());
      const int32_t parent = n.parent;
      if (!host_ok) {
        gone.clear();
        c->drop(id, &gone);
        for (int32_t g : gone) {
          if (*n_dropped < drop_cap) dropped[*n_dropped] = g;
          ++*n_dropped;
        }
      } else {
        for (int32_t k = 0; k < nb; ++k) {
          out_dev[*n_out] = n.blocks[(size_t)k];
          out_host[*n_out] = ids[(size_t)k];
          ++*n_out;
        }
        c->set_tier(n, kHost);
        n.blocks = ids;
      }
      // the parent may have become a leaf among the HBM nodes
      if (!c->cfg.ignore_dependencies && parent != 0 && c->out_candidate(c->nodes[parent]))
        heap.push(Item(c->eval(c->nodes[parent], now, low, n_lora), parent));
    }
  } else if (c->usage() < c->cfg.lower) {
    for (const Node& n : c->nodes)
      if (c->in_candidate(n)) heap.push(Item(-c->eval(n, now, low, n_lora), n.id));
    while (c->usage() < c->cfg.lower && !heap.empty()) {
      const int32_t id = heap.top().second;
      Node& n = c->nodes[id];
      if (!c->in_candidate(n)) {
        heap.pop();
        continue;
      }
      const int32_t nb = (int32_t)n.blocks.size();
      const int64_t free_after = flp_pool_num_free(c->pool, kHbm) - nb;
      if (1.0 - (double)free_after / (double)c->n_dev > c->cfg.upper) break;
      if (*n_in + nb > in_cap) break;
      ids.resize((size_t)nb);
      if (flp_pool_alloc(c->pool, kHbm, nb, ids.data()) != FLP_OK) break;
      heap.pop();
      for (int32_t k = 0; k < nb; ++k) {
        in_host[*n_in] = n.blocks[(size_t)k];
        in_dev[*n_in] = ids[(size_t)k];
        ++*n_in;
      }
      (void)flp_pool_free(c->pool, kHost, nb, n.blocks.data());
      c->set_tier(n, kHbm);
      n.blocks = ids;
      // its children on the host tier are now roots of host sub-trees
      if (!c->cfg.ignore_dependencies)
        for (int32_t ch : n.children)
          if (c->in_candidate(c->nodes[ch])) heap.push(Item(-c->eval(c->nodes[ch], now, low, n_lora), ch));
    }
  }
  return FLP_OK;
}

extern "C" flp_status flc_low_lora(flc_cache* c, int32_t batch_size, double* out) {
  FLC_CHECK(c && out && batch_size >= 0, FLP_EINVAL, "flc_low_lora: invalid argument");
  std::lock_guard<std::mutex> lk(c->mu);
  *out = c->low_lora(batch_size);
  return FLP_OK;
}

extern "C" flp_status flc_eval(flc_cache* c, int32_t node_id, double now, int32_t batch_size, double* out) {
  FLC_CHECK(c && out && batch_size >= 0, FLP_EINVAL, "flc_eval: invalid argument");
  std::lock_guard<std::mutex> lk(c->mu);
  FLC_CHECK(node_id > 0 && node_id < (int32_t)c->nodes.size() && c->nodes[node_id].alive, FLP_EINVAL,
            "flc_eval: no node %d", node_id);
  *out = c->eval(c->nodes[node_id], now, c->low_lora(batch_size), c->now_lora());
  return FLP_OK;
}

extern "C" flp_status flc_get_stats(flc_cache* c, flc_stats* out) {
  FLC_CHECK(c && out, FLP_EINVAL, "flc_get_stats: null argument");
  std::lock_guard<std::mutex> lk(c->mu);
  flc_stats s{};
  for (const Node& n : c->nodes) {
    if (!n.alive || n.id == 0) continue;
    s.n_nodes++;
    (n.kind == kLora ? s.n_lora_nodes : s.n_kv_nodes)++;
    (n.tier == kHbm ? s.hbm_blocks_held : s.host_blocks_held) += (int64_t)n.blocks.size();
    if (n.kind == kKv && n.tier == kHbm) {
      int32_t p = n.parent;
      while (p != 0 && c->nodes[p].tier == kHbm) p = c->nodes[p].parent;
      if (p != 0) s.invalid_kv_blocks += (int64_t)n.blocks.size();
    }
  }
  s.n_lora_hbm = c->now_lora();
  s.n_queries = c->n_queries;
  s.n_running = (int64_t)c->running.size();
  s.usage = c->usage();
  *out = s;
  return FLP_OK;
}

extern "C" flp_status flc_snapshot(flc_cache* c, flc_node_info* rows, int64_t cap, int64_t* n_nodes) {
  FLC_CHECK(c && n_nodes && cap >= 0 && (cap == 0 || rows), FLP_EINVAL, "flc_snapshot: invalid argument");
  std::lock_guard<std::mutex> lk(c->mu);
  int64_t k = 0;
  for (const Node& n : c->nodes) {
    if (!n.alive || n.id == 0) continue;
    if (k < cap) {
      flc_node_info r{};
      r.id = n.id;
      r.kind = n.kind;
      r.parent = n.parent;
      r.tier = n.tier;
      r.first_block = n.blocks.empty() ? -1 : n.blocks[0];
      r.n_blocks = (int32_t)n.blocks.size();
      r.pins = n.pins;
      r.visits = n.visits;
      r.last_use = n.last_use;
      rows[k] = r;
    }
    ++k;
  }
  *n_nodes = k;
  return FLP_OK;
}
