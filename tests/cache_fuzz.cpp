// Random walk over the host-side C ABI (include/flcache.h on top of include/flpool.h), meant to be built with
// AddressSanitizer and UndefinedBehaviorSanitizer and run on the CPU (tests/test_cache_manager.py builds and runs
// it).  It checks no results against a model (the Python tests do that against the oracle); it drives every entry
// point through many states, legal and illegal arguments included, so that the sanitizers see the code paths, and
// it checks the accounting that must hold after every call: every block of a tier is either free or held by
// exactly one node or by a running query's fresh blocks.  A second walk drives the pool's own alloc / free / swap
// calls against a set of held ids and through every argument check.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <map>
#include <random>
#include <set>
#include <vector>

#include "flcache.h"
#include "flp_internal.h"

// The pool's source file refers to the two copy launchers of the GPU build; the walk never swaps block
// contents, so here they only have to exist.
flp_status flp_launch_copy_blocks(const uint8_t*, uint8_t*, const int32_t*, const int32_t*, int32_t, int64_t, int,
                                  hipStream_t) {
  std::fprintf(stderr, "cache_fuzz: a copy was launched\n");
  std::abort();
}
flp_status flp_launch_stage_copy(const void*, void*, size_t, hipStream_t) {
  std::fprintf(stderr, "cache_fuzz: a copy was launched\n");
  std::abort();
}
// the fixed scratch array belongs to the GPU build; pool creation tolerates that its set-up fails
flp_status flp_static_scratch_setup(int, void**) { return FLP_EHIP; }

#define REQUIRE(cond)                                                                     \
  do {                                                                                    \
    if (!(cond)) {                                                                        \
      std::fprintf(stderr, "cache_fuzz: line %d: %s (last error: %s)\n", __LINE__, #cond, \
                   flp_last_error());                                                     \
      std::exit(1);                                                                       \
    }                                                                                     \
  } while (0)

namespace {

// how often the walk reached the states it is meant to reach (printed at the end, checked to be non-zero)
struct Seen {
  long out = 0, in = 0, dropped = 0, waiting = 0, match_swaps = 0, given_back = 0, matched_blocks = 0;
} seen;

struct Running {
  int64_t query;
  int32_t lora;
  std::vector<int32_t> tokens;   // the conversation so far
  int32_t held_blocks;           // KV blocks the query holds (matched + inserted)
  bool waiting;
};

void run(uint64_t seed, int n_ops, const flc_config& cfg, int64_t n_dev, int64_t n_host) {
  std::mt19937_64 rng(seed);
  auto uni = [&](int lo, int hi) { return (int)(lo + rng() % (uint64_t)(hi - lo + 1)); };
  const int bt = cfg.block_tokens;
  flp_pool_config pc{};
  pc.dtype = FLP_F16;
  pc.block_tokens = bt;
  pc.n_kv_heads = 1;
  pc.head_dim = 64;
  pc.n_dev_blocks = n_dev;
  pc.n_host_blocks = n_host;
  // the manager never touches block contents: any aligned address range of the right size will do
  const size_t block_bytes = (size_t)2 * bt * 1 * 64 * 2;
  void* dev = std::aligned_alloc(256, block_bytes * (size_t)n_dev);
  void* host = std::aligned_alloc(256, block_bytes * (size_t)n_host);
  REQUIRE(dev && host);
  pc.dev_base = dev;
  pc.host_base = host;
  flp_pool* pool = nullptr;
  REQUIRE(flp_pool_create(&pc, &pool) == FLP_OK);
  REQUIRE((size_t)flp_pool_block_bytes(pool) == block_bytes);
  flc_cache* c = nullptr;
  REQUIRE(flc_create(pool, &cfg, &c) == FLP_OK);

  std::map<int32_t, int32_t> loras;          // id -> blocks
  std::vector<Running> running;
  double now = 0.0;
  bool any_dropped = false;                  // a monitor interval forgot nodes: LoRAs may have left the tree
  const int max_tokens = 12 * bt;
  std::vector<int32_t> lora_blocks(64), kv_blocks(max_tokens / bt + 1), swap_host(64 + max_tokens / bt + 1),
      swap_dev(64 + max_tokens / bt + 1);

  auto check_accounting = [&]() {
    flc_stats st{};
    REQUIRE(flc_get_stats(c, &st) == FLP_OK);
    int64_t n = 0;
    REQUIRE(flc_snapshot(c, nullptr, 0, &n) == FLP_OK);
    REQUIRE(n == st.n_nodes);
    std::vector<flc_node_info> rows((size_t)n + 1);
    int64_t n2 = 0;
    REQUIRE(flc_snapshot(c, rows.data(), n, &n2) == FLP_OK && n2 == n);
    int64_t held[2] = {0, 0}, n_lora = 0, n_kv = 0, lora_hbm = 0;
    for (int64_t i = 0; i < n; ++i) {
      const flc_node_info& r = rows[(size_t)i];
      REQUIRE(r.tier == 0 || r.tier == 1);
      REQUIRE(r.kind == 0 || r.kind == 1);
      REQUIRE(r.n_blocks >= 0 && r.pins >= 0 && r.visits >= 0);
      REQUIRE(i == 0 || rows[(size_t)i - 1].id < r.id);
      held[r.tier] += r.n_blocks;
      n_lora += r.kind == 0;
      n_kv += r.kind == 1;
      lora_hbm += r.kind == 0 && r.tier == 0;
      if (r.kind == 0) REQUIRE(r.parent == 0);
      if (r.kind == 1) REQUIRE(r.n_blocks == 1);
    }
    REQUIRE(n_lora == st.n_lora_nodes && n_kv == st.n_kv_nodes && lora_hbm == st.n_lora_hbm);
    REQUIRE(held[0] == st.hbm_blocks_held && held[1] == st.host_blocks_held);
    REQUIRE(st.n_running == (int64_t)running.size());
    // every block of a tier is free or held by a node (the walk frees what it allocates itself at once)
    REQUIRE(flp_pool_num_free(pool, 0) + held[0] == n_dev);
    REQUIRE(flp_pool_num_free(pool, 1) + held[1] == n_host);
    if (!cfg.ignore_dependencies) REQUIRE(st.invalid_kv_blocks == 0);
  };

  for (int op = 0; op < n_ops; ++op) {
    now += 0.001 * uni(0, 200);
    const int what = uni(0, 99);
    if (what < 8) {                                            // a LoRA enters (sometimes one that is there)
      const int32_t id = uni(0, 11), nb = uni(1, 5), tier = uni(0, 1);
      std::vector<int32_t> ids((size_t)nb);
      const flp_status s = flc_add_lora(c, id, nb, tier, now, ids.data());
      if (loras.count(id) && !(any_dropped && s != FLP_EDUP)) {
        REQUIRE(s == FLP_EDUP);
      } else if (s == FLP_OK) {                                 // new, or forgotten by a monitor interval and back
        loras[id] = nb;
        std::set<int32_t> distinct(ids.begin(), ids.end());
        REQUIRE((int)distinct.size() == nb);
      } else {
        REQUIRE(s == FLP_ENOSPC);
      }
    } else if (what < 45) {                                    // a query arrives
      const int32_t id = uni(0, 13);                           // 12, 13 are never added
      Running r;
      r.lora = id;
      // conversations share prefixes: tokens are drawn from a tiny alphabet, block by block
      const int n_tok = uni(0, max_tokens);
      r.tokens.resize((size_t)n_tok);
      for (int i = 0; i < n_tok; ++i) r.tokens[(size_t)i] = (i / bt) < 3 ? (id + i / bt) % 3 : uni(0, 2);
      int32_t n_l = 0, n_k = 0, n_s = 0;
      const bool small_cap = uni(0, 19) == 0;
      const flp_status s = flc_match(c, id, r.tokens.data(), n_tok, now, &r.query, lora_blocks.data(),
                                     small_cap ? 0 : (int32_t)lora_blocks.size(), &n_l, kv_blocks.data(),
                                     (int32_t)kv_blocks.size(), &n_k, swap_host.data(), swap_dev.data(),
                                     (int32_t)swap_host.size(), &n_s);
      if (!loras.count(id)) {
        REQUIRE(s == FLP_EINVAL);
      } else if (any_dropped && s == FLP_EINVAL) {
        loras.erase(id);                                       // a monitor interval forgot this LoRA
      } else if (small_cap) {
        REQUIRE(s == FLP_ERANGE);
      } else {
        REQUIRE(s == FLP_OK);
        REQUIRE(n_k >= 0 && n_k <= n_tok / bt && n_s >= 0 && n_s <= (int)swap_host.size());
        r.waiting = n_l < 0;
        seen.waiting += r.waiting;
        seen.match_swaps += n_s;
        seen.matched_blocks += n_k;
        if (!r.waiting) REQUIRE(n_l == loras[id]);
        r.held_blocks = n_k;
        running.push_back(r);
      }
    } else if (what < 70 && !running.empty()) {                // a running query stores fresh KV blocks
      Running& r = running[(size_t)uni(0, (int)running.size() - 1)];
      const int full = (int)r.tokens.size() / bt;
      int n_new = uni(0, 3);
      if (r.held_blocks + n_new > full) n_new = full - r.held_blocks;
      if (n_new < 0) n_new = 0;
      std::vector<int32_t> fresh((size_t)n_new + 1), back((size_t)n_new + 1);
      if (flp_pool_alloc(pool, 0, n_new, fresh.data()) == FLP_OK) {
        int32_t n_back = -1;
        const flp_status s = flc_insert(c, r.query, r.tokens.data(), (int32_t)r.tokens.size(), fresh.data(), n_new,
                                        now, back.data(), &n_back);
        if (r.waiting) {                                       // holds nothing: every block comes back
          REQUIRE(s == FLP_OK && n_back == n_new);
          REQUIRE(flp_pool_free(pool, 0, n_back, back.data()) == FLP_OK);
        } else {
          REQUIRE(s == FLP_OK && n_back >= 0 && n_back <= n_new);
          seen.given_back += n_back;
          REQUIRE(flp_pool_free(pool, 0, n_back, back.data()) == FLP_OK);
          r.held_blocks += n_new;
        }
      }
    } else if (what < 85 && !running.empty()) {                // a query ends
      const size_t k = (size_t)uni(0, (int)running.size() - 1);
      REQUIRE(flc_release(c, running[k].query) == FLP_OK);
      REQUIRE(flc_release(c, running[k].query) == FLP_EINVAL);  // a second time: unknown query
      running.erase(running.begin() + (long)k);
    } else if (what < 97) {                                    // a monitor interval
      const int cap = uni(0, 1) ? 64 : uni(0, 3);
      std::vector<int32_t> od((size_t)cap + 1), oh((size_t)cap + 1), ih((size_t)cap + 1), id((size_t)cap + 1),
          dr((size_t)cap + 1);
      int32_t n_out = -1, n_in = -1, n_drop = -1;
      REQUIRE(flc_tick(c, now, uni(1, 64), od.data(), oh.data(), cap, &n_out, ih.data(), id.data(), cap, &n_in,
                       dr.data(), cap, &n_drop) == FLP_OK);
      REQUIRE(n_out >= 0 && n_out <= cap && n_in >= 0 && n_in <= cap && n_drop >= 0);
      any_dropped = any_dropped || n_drop > 0;
      seen.out += n_out;
      seen.in += n_in;
      seen.dropped += n_drop;
      for (int i = 0; i < n_out; ++i) REQUIRE(od[(size_t)i] >= 0 && od[(size_t)i] < n_dev && oh[(size_t)i] >= 0 && oh[(size_t)i] < n_host);
      for (int i = 0; i < n_in; ++i) REQUIRE(id[(size_t)i] >= 0 && id[(size_t)i] < n_dev && ih[(size_t)i] >= 0 && ih[(size_t)i] < n_host);
    } else {                                                   // the inspection calls, bad arguments included
      double v = 0.0;
      REQUIRE(flc_low_lora(c, uni(1, 64), &v) == FLP_OK && v >= 0.0);
      int64_t n = 0;
      REQUIRE(flc_snapshot(c, nullptr, 0, &n) == FLP_OK);
      const flp_status s = flc_eval(c, uni(-2, (int)n + 2), now, uni(1, 64), &v);
      REQUIRE(s == FLP_OK || s == FLP_EINVAL);
      REQUIRE(flc_get_stats(c, nullptr) == FLP_EINVAL);
      REQUIRE(flc_release(c, -5) == FLP_EINVAL);
    }
    check_accounting();
  }
  for (const Running& r : running) REQUIRE(flc_release(c, r.query) == FLP_OK);
  running.clear();
  check_accounting();
  REQUIRE(flc_destroy(c) == FLP_OK);
  REQUIRE(flp_pool_num_free(pool, 0) == n_dev && flp_pool_num_free(pool, 1) == n_host);
  REQUIRE(flp_pool_destroy(pool) == FLP_OK);
  std::free(dev);
  std::free(host);
}

// The pool alone: seeded allocations and frees against a set of held ids, and every argument check of the
// alloc / free / swap calls (the swap calls must refuse bad lists before they launch anything).
void run_pool(uint64_t seed, int n_ops) {
  std::mt19937_64 rng(seed);
  auto uni = [&](int lo, int hi) { return (int)(lo + rng() % (uint64_t)(hi - lo + 1)); };
  const int64_t n_blocks[2] = {40, 24};
  flp_pool_config pc{};
  pc.dtype = FLP_BF16;
  pc.block_tokens = 16;
  pc.n_kv_heads = 1;
  pc.head_dim = 64;
  pc.n_dev_blocks = n_blocks[0];
  pc.n_host_blocks = n_blocks[1];
  const size_t block_bytes = (size_t)2 * 16 * 64 * 2;
  void* dev = std::aligned_alloc(256, block_bytes * (size_t)n_blocks[0]);
  void* host = std::aligned_alloc(256, block_bytes * (size_t)n_blocks[1]);
  REQUIRE(dev && host);
  pc.dev_base = dev;
  pc.host_base = host;
  flp_pool* pool = nullptr;
  REQUIRE(flp_pool_create(nullptr, &pool) == FLP_EINVAL && flp_pool_create(&pc, nullptr) == FLP_EINVAL);
  pc.dev_base = (char*)dev + 8;
  REQUIRE(flp_pool_create(&pc, &pool) == FLP_EINVAL);            // misaligned base
  pc.dev_base = dev;
  REQUIRE(flp_pool_create(&pc, &pool) == FLP_OK);
  std::set<int32_t> held[2];
  for (int op = 0; op < n_ops; ++op) {
    const int tier = uni(0, 1), what = uni(0, 9);
    if (what < 5) {
      const int n = uni(0, 12);
      std::vector<int32_t> ids((size_t)n + 1, -7);
      const flp_status s = flp_pool_alloc(pool, tier, n, ids.data());
      if (n > n_blocks[tier] - (int64_t)held[tier].size()) {
        REQUIRE(s == FLP_ENOSPC && (n == 0 || ids[0] == -7));      // all or nothing
      } else {
        REQUIRE(s == FLP_OK);
        for (int i = 0; i < n; ++i) {
          REQUIRE(ids[(size_t)i] >= 0 && ids[(size_t)i] < n_blocks[tier]);
          REQUIRE(held[tier].insert(ids[(size_t)i]).second);       // never an id that is held
        }
      }
    } else if (what < 8 && !held[tier].empty()) {
      std::vector<int32_t> ids;
      for (int32_t id : held[tier])
        if (uni(0, 2) == 0) ids.push_back(id);
      REQUIRE(flp_pool_free(pool, tier, (int32_t)ids.size(), ids.data()) == FLP_OK);
      for (int32_t id : ids) held[tier].erase(id);
      if (!ids.empty()) REQUIRE(flp_pool_free(pool, tier, 1, ids.data()) == FLP_EDUP);   // free twice
    } else {
      int32_t bad[3] = {-1, (int32_t)n_blocks[tier], 0};
      REQUIRE(flp_pool_free(pool, tier, 1, &bad[0]) == FLP_ERANGE && flp_pool_free(pool, tier, 1, &bad[1]) == FLP_ERANGE);
      REQUIRE(flp_pool_free(pool, tier, -1, bad) == FLP_EINVAL && flp_pool_free(pool, 2, 1, bad) == FLP_EINVAL);
      REQUIRE(flp_pool_alloc(pool, tier, -1, bad) == FLP_EINVAL && flp_pool_alloc(pool, tier, 1, nullptr) == FLP_EINVAL);
      if (held[tier].size() >= 2) {                             // one id twice in a list: nothing is freed
        int32_t twice[2] = {*held[tier].begin(), *held[tier].begin()};
        REQUIRE(flp_pool_free(pool, tier, 2, twice) == FLP_EDUP);
      }
      // swap lists that must be refused before anything is launched
      int32_t src[2] = {0, 1}, dup[2] = {3, 3}, far[2] = {0, (int32_t)n_blocks[0]};
      REQUIRE(flp_pool_swap_in(pool, 2, src, dup, nullptr) == FLP_EDUP);
      REQUIRE(flp_pool_swap_out(pool, 2, src, dup, nullptr) == FLP_EDUP);
      REQUIRE(flp_pool_swap_in(pool, 2, src, far, nullptr) == FLP_ERANGE);
      REQUIRE(flp_pool_swap_out(pool, 2, far, src, nullptr) == FLP_ERANGE);
      REQUIRE(flp_pool_swap_in(pool, -1, src, src, nullptr) == FLP_EINVAL);
      REQUIRE(flp_pool_swap_in(pool, 1, nullptr, src, nullptr) == FLP_EINVAL);
      REQUIRE(flp_pool_swap_in(pool, 0, nullptr, nullptr, nullptr) == FLP_OK);
    }
    for (int t = 0; t < 2; ++t) REQUIRE(flp_pool_num_free(pool, t) + (int64_t)held[t].size() == n_blocks[t]);
  }
  REQUIRE(flp_pool_destroy(pool) == FLP_OK);
  std::free(dev);
  std::free(host);
}

}  // namespace

int main(int argc, char** argv) {
  const int n_ops = argc > 1 ? std::atoi(argv[1]) : 4000;
  int runs = 0;
  for (int variant = 0; variant < 4; ++variant)
    for (uint64_t seed = 1; seed <= 3; ++seed) {
      flc_config cfg{};
      cfg.block_tokens = 4;
      cfg.use_lru = variant == 1;
      cfg.ignore_dependencies = variant == 2;
      cfg.no_lora_reward = variant == 3;
      cfg.upper = 0.9;
      cfg.lower = 0.6;
      cfg.pcie_bytes_per_s = 5e10;
      cfg.time_scale_s = 1.0;
      // a roomy pool, a tight HBM tier, and a tight host tier (swap-out victims get forgotten)
      const int64_t n_dev = seed == 2 ? 24 : 64, n_host = seed == 3 ? 8 : 96;
      run(seed * 7919 + (uint64_t)variant, n_ops, cfg, n_dev, n_host);
      ++runs;
    }
  for (uint64_t seed = 1; seed <= 3; ++seed) run_pool(seed, n_ops);
  std::printf("cache_fuzz: %d runs of %d calls, accounting held after every call; swapped out %ld, in %ld (by "
              "matches %ld), forgotten %ld, waiting queries %ld, matched blocks %ld, blocks given back %ld\n",
              runs, n_ops, seen.out, seen.in, seen.match_swaps, seen.dropped, seen.waiting, seen.matched_blocks,
              seen.given_back);
  if (n_ops >= 1000)
    REQUIRE(seen.out && seen.in && seen.match_swaps && seen.dropped && seen.waiting && seen.matched_blocks &&
            seen.given_back);
  return 0;
}
