// Four threads on one pool and one cache (include/flcache.h says that the calls on a cache are serialised by an
// internal lock, include/flpool.h the same of a pool), meant to be built with ThreadSanitizer and run on the CPU
// (tests/test_cache_manager.py builds and runs it).  Each thread serves its own LoRAs and conversations, one of
// them also runs the monitor intervals; at the end every block is either free or held by a node.
#include <atomic>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <thread>
#include <vector>

#include "flcache.h"
#include "flp_internal.h"

// The pool's source file refers to the two copy launchers of the GPU build; nothing here swaps block contents.
flp_status flp_launch_copy_blocks(const uint8_t*, uint8_t*, const int32_t*, const int32_t*, int32_t, int64_t, int,
                                  hipStream_t) {
  std::abort();
}
flp_status flp_launch_stage_copy(const void*, void*, size_t, hipStream_t) { std::abort(); }
// the fixed scratch array belongs to the GPU build; pool creation tolerates that its set-up fails
flp_status flp_static_scratch_setup(int, void**) { return FLP_EHIP; }

#define REQUIRE(cond)                                                                       \
  do {                                                                                      \
    if (!(cond)) {                                                                          \
      std::fprintf(stderr, "cache_threads: line %d: %s (last error: %s)\n", __LINE__, #cond, \
                   flp_last_error());                                                       \
      std::exit(1);                                                                         \
    }                                                                                       \
  } while (0)

namespace {

constexpr int kThreads = 4, kBt = 4, kMaxBlocks = 10;
std::atomic<long> n_calls{0};

void worker(int me, flp_pool* pool, flc_cache* c, int n_ops) {
  std::mt19937_64 rng(1000 + (uint64_t)me);
  auto uni = [&](int lo, int hi) { return (int)(lo + rng() % (uint64_t)(hi - lo + 1)); };
  std::vector<int32_t> lora_blocks(8), kv(kMaxBlocks + 1), sh(8 + kMaxBlocks + 1), sd(8 + kMaxBlocks + 1);
  for (int a = 0; a < 3; ++a) {
    int32_t ids[4];
    const flp_status s = flc_add_lora(c, 10 * me + a, uni(1, 4), uni(0, 1), 0.0, ids);
    REQUIRE(s == FLP_OK || s == FLP_ENOSPC);
  }
  for (int op = 0; op < n_ops; ++op) {
    const double now = 0.001 * op;
    const int32_t lora = 10 * me + uni(0, 2);
    const int n_tok = kBt * uni(0, kMaxBlocks);
    std::vector<int32_t> tokens((size_t)n_tok);
    for (int i = 0; i < n_tok; ++i) tokens[(size_t)i] = (i / kBt) < 4 ? (i / kBt) % 2 : uni(0, 1);
    int64_t q = 0;
    int32_t n_l = 0, n_k = 0, n_s = 0;
    const flp_status s = flc_match(c, lora, tokens.data(), n_tok, now, &q, lora_blocks.data(), 8, &n_l, kv.data(),
                                   kMaxBlocks + 1, &n_k, sh.data(), sd.data(), 8 + kMaxBlocks + 1, &n_s);
    if (s == FLP_EINVAL) continue;                    // this LoRA never fitted, or a monitor interval forgot it
    REQUIRE(s == FLP_OK);
    const int n_new = n_l < 0 ? 0 : n_tok / kBt - n_k;
    std::vector<int32_t> fresh((size_t)n_new + 1), back((size_t)n_new + 1);
    if (n_new > 0 && flp_pool_alloc(pool, 0, n_new, fresh.data()) == FLP_OK) {
      int32_t n_back = 0;
      REQUIRE(flc_insert(c, q, tokens.data(), n_tok, fresh.data(), n_new, now, back.data(), &n_back) == FLP_OK);
      REQUIRE(flp_pool_free(pool, 0, n_back, back.data()) == FLP_OK);
    }
    REQUIRE(flc_release(c, q) == FLP_OK);
    if (me == 0 && op % 8 == 0) {                     // the monitor thread
      int32_t od[32], oh[32], ih[32], id[32], dr[32], n_out = 0, n_in = 0, n_drop = 0;
      REQUIRE(flc_tick(c, now, 16, od, oh, 32, &n_out, ih, id, 32, &n_in, dr, 32, &n_drop) == FLP_OK);
    }
    if (op % 16 == 0) {
      flc_stats st{};
      REQUIRE(flc_get_stats(c, &st) == FLP_OK);
    }
    n_calls += 3;
  }
}

}  // namespace

int main(int argc, char** argv) {
  const int n_ops = argc > 1 ? std::atoi(argv[1]) : 2000;
  const int64_t n_dev = 96, n_host = 64;
  flp_pool_config pc{};
  pc.dtype = FLP_F16;
  pc.block_tokens = kBt;
  pc.n_kv_heads = 1;
  pc.head_dim = 64;
  pc.n_dev_blocks = n_dev;
  pc.n_host_blocks = n_host;
  const size_t block_bytes = (size_t)2 * kBt * 64 * 2;
  void* dev = std::aligned_alloc(256, block_bytes * (size_t)n_dev);
  void* host = std::aligned_alloc(256, block_bytes * (size_t)n_host);
  pc.dev_base = dev;
  pc.host_base = host;
  flp_pool* pool = nullptr;
  REQUIRE(flp_pool_create(&pc, &pool) == FLP_OK);
  flc_config cfg{};
  cfg.block_tokens = kBt;
  cfg.upper = 0.9;
  cfg.lower = 0.6;
  cfg.pcie_bytes_per_s = 5e10;
  cfg.time_scale_s = 1.0;
  flc_cache* c = nullptr;
  REQUIRE(flc_create(pool, &cfg, &c) == FLP_OK);
  std::vector<std::thread> threads;
  for (int t = 0; t < kThreads; ++t) threads.emplace_back(worker, t, pool, c, n_ops);
  for (std::thread& t : threads) t.join();
  flc_stats st{};
  REQUIRE(flc_get_stats(c, &st) == FLP_OK);
  REQUIRE(st.n_running == 0);
  REQUIRE(flp_pool_num_free(pool, 0) + st.hbm_blocks_held == n_dev);
  REQUIRE(flp_pool_num_free(pool, 1) + st.host_blocks_held == n_host);
  REQUIRE(st.invalid_kv_blocks == 0);
  REQUIRE(flc_destroy(c) == FLP_OK);
  REQUIRE(flp_pool_num_free(pool, 0) == n_dev && flp_pool_num_free(pool, 1) == n_host);
  REQUIRE(flp_pool_destroy(pool) == FLP_OK);
  std::free(dev);
  std::free(host);
  std::printf("cache_threads: %d threads, %ld calls, accounting intact\n", kThreads, n_calls.load());
  return 0;
}
