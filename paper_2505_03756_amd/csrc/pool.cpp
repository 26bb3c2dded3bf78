// Host side of the unified caching pool: the two tiers' free lists, swap-list
// validation, and the staging ring that carries small host arrays to the device.
// (Paper section 4.3: device and host memory are both cut into blocks of one size at
// initialisation; blocks released by a swap-out are recycled for later allocations.)
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>

#include "flp_internal.h"

static thread_local std::string g_last_error;

void flp_set_error(const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof(buf), fmt, ap);
  va_end(ap);
  g_last_error = buf;
}

extern "C" const char* flp_last_error(void) { return g_last_error.c_str(); }
extern "C" const char* flp_version(void) { return "flpool 0.1 (gfx950)"; }

static void freelist_init(FlpFreeList& f, int64_t n) {
  f.n = n;
  f.stack.resize((size_t)n);
  for (int64_t i = 0; i < n; ++i) f.stack[(size_t)i] = (int32_t)(n - 1 - i);   // first pops: 0,1,2,...
  f.is_free.assign((size_t)n, 1);
  f.stamp.assign((size_t)n, 0);
  f.gen = 0;
}

static uint32_t next_gen(FlpFreeList& f) {
  if (++f.gen == 0) {   // wrapped: clear the stamps once
    std::fill(f.stamp.begin(), f.stamp.end(), 0u);
    f.gen = 1;
  }
  return f.gen;
}

extern "C" flp_status flp_pool_create(const flp_pool_config* cfg, flp_pool** out) {
  if (!cfg || !out) {
    flp_set_error("flp_pool_create: null argument");
    return FLP_EINVAL;
  }
  *out = nullptr;
  if (cfg->dtype < FLP_F32 || cfg->dtype > FLP_BF16) {
    flp_set_error("flp_pool_create: dtype %d not supported", cfg->dtype);
    return FLP_ENOTSUP;
  }
  if (cfg->block_tokens <= 0 || cfg->n_kv_heads <= 0 || cfg->head_dim <= 0 || cfg->n_dev_blocks < 0 ||
      cfg->n_host_blocks < 0 || cfg->n_dev_blocks > INT32_MAX || cfg->n_host_blocks > INT32_MAX) {
    flp_set_error("flp_pool_create: bad geometry (block_tokens=%d n_kv_heads=%d head_dim=%d dev=%lld host=%lld)",
                  cfg->block_tokens, cfg->n_kv_heads, cfg->head_dim, (long long)cfg->n_dev_blocks,
                  (long long)cfg->n_host_blocks);
    return FLP_EINVAL;
  }
  flp_pool* p = new (std::nothrow) flp_pool();
  if (!p) {
    flp_set_error("flp_pool_create: out of host memory");
    return FLP_ENOSPC;
  }
  p->cfg = *cfg;
  p->elem_bytes = cfg->dtype == FLP_F32 ? 4 : 2;
  p->block_elems = 2LL * cfg->block_tokens * cfg->n_kv_heads * cfg->head_dim;
  p->block_bytes = p->block_elems * p->elem_bytes;
  if (((uintptr_t)cfg->dev_base | (uintptr_t)cfg->host_base) & 255) {
    flp_set_error("flp_pool_create: pool bases must be 256-byte aligned");
    delete p;
    return FLP_EINVAL;
  }
  const bool must_alloc = (!cfg->dev_base && cfg->n_dev_blocks > 0) || (!cfg->host_base && cfg->n_host_blocks > 0);
  hipError_t e = hipGetDevice(&p->device);
  if (e != hipSuccess) {
    // Without a usable GPU the pool can still do its host-side bookkeeping (free lists,
    // list validation) over caller-owned regions; every launch will report FLP_EHIP.
    (void)hipGetLastError();
    p->device = -1;
    if (must_alloc) {
      flp_set_error("flp_pool_create: hipGetDevice failed: %s (is the HIP runtime / a GPU present?)",
                    hipGetErrorString(e));
      delete p;
      return FLP_EHIP;
    }
  }
  p->dev_base = (uint8_t*)cfg->dev_base;
  p->host_base = (uint8_t*)cfg->host_base;
  if (!p->dev_base && cfg->n_dev_blocks > 0) {
    e = hipMalloc((void**)&p->dev_base, (size_t)(cfg->n_dev_blocks * p->block_bytes));
    if (e != hipSuccess) {
      flp_set_error("flp_pool_create: hipMalloc of %lld bytes failed: %s",
                    (long long)(cfg->n_dev_blocks * p->block_bytes), hipGetErrorString(e));
      delete p;
      return FLP_EHIP;
    }
    p->own_dev = true;
  }
  if (!p->host_base && cfg->n_host_blocks > 0) {
    e = hipHostMalloc((void**)&p->host_base, (size_t)(cfg->n_host_blocks * p->block_bytes), hipHostMallocDefault);
    if (e != hipSuccess) {
      flp_set_error("flp_pool_create: hipHostMalloc of %lld bytes failed: %s",
                    (long long)(cfg->n_host_blocks * p->block_bytes), hipGetErrorString(e));
      if (p->own_dev) (void)hipFree(p->dev_base);
      delete p;
      return FLP_EHIP;
    }
    p->own_host = true;
  }
  if (p->host_base && !p->own_host && p->device >= 0) {
    hipPointerAttribute_t attr{};
    if (hipPointerGetAttributes(&attr, p->host_base) == hipSuccess)
      p->host_tier_in_hbm = attr.type == hipMemoryTypeDevice;
    else
      (void)hipGetLastError();
  }
  freelist_init(p->tier[0], cfg->n_dev_blocks);
  freelist_init(p->tier[1], cfg->n_host_blocks);
  // set-up for the entry point that may not allocate: find this device's copy of its scratch array now, while
  // allocation is still allowed (a failure is not this call's; that entry point tries again and reports it)
  if (p->device >= 0 && flp_static_scratch_setup(p->device, nullptr) != FLP_OK) (void)hipGetLastError();
  *out = p;
  return FLP_OK;
}

extern "C" flp_status flp_pool_destroy(flp_pool* p) {
  if (!p) return FLP_OK;
  if (p->device >= 0) (void)hipDeviceSynchronize();
  for (auto& s : p->stage) {
    if (s.ev) (void)hipEventDestroy(s.ev);
    if (s.host) (void)hipHostFree(s.host);
    if (s.dev) (void)hipFree(s.dev);
  }
  if (p->work) (void)hipFree(p->work);
  if (p->attn_work) (void)hipFree(p->attn_work);
  for (void* old : p->retired) (void)hipFree(old);
  if (p->own_dev && p->dev_base) (void)hipFree(p->dev_base);
  if (p->own_host && p->host_base) (void)hipHostFree(p->host_base);
  delete p;
  return FLP_OK;
}

extern "C" int64_t flp_pool_block_bytes(const flp_pool* p) { return p ? p->block_bytes : 0; }
extern "C" int64_t flp_pool_num_free(const flp_pool* p, int32_t tier) {
  if (!p || tier < 0 || tier > 1) return -1;
  std::lock_guard<std::mutex> lk(p->mu);               // another thread may be allocating
  return (int64_t)p->tier[tier].stack.size();
}
extern "C" void* flp_pool_base(const flp_pool* p, int32_t tier) {
  if (!p || tier < 0 || tier > 1) return nullptr;
  return tier == 0 ? (void*)p->dev_base : (void*)p->host_base;
}

extern "C" flp_status flp_pool_alloc(flp_pool* p, int32_t tier, int32_t n, int32_t* out_ids) {
  if (!p || tier < 0 || tier > 1 || n < 0 || (n > 0 && !out_ids)) {
    flp_set_error("flp_pool_alloc: invalid argument");
    return FLP_EINVAL;
  }
  std::lock_guard<std::mutex> lk(p->mu);
  FlpFreeList& f = p->tier[tier];
  if ((size_t)n > f.stack.size()) {
    flp_set_error("flp_pool_alloc: %d blocks asked, %zu free in tier %d", n, f.stack.size(), tier);
    return FLP_ENOSPC;
  }
  for (int32_t k = 0; k < n; ++k) {
    int32_t id = f.stack.back();
    f.stack.pop_back();
    f.is_free[(size_t)id] = 0;
    out_ids[k] = id;
  }
  return FLP_OK;
}

extern "C" flp_status flp_pool_free(flp_pool* p, int32_t tier, int32_t n, const int32_t* ids) {
  if (!p || tier < 0 || tier > 1 || n < 0 || (n > 0 && !ids)) {
    flp_set_error("flp_pool_free: invalid argument");
    return FLP_EINVAL;
  }
  std::lock_guard<std::mutex> lk(p->mu);
  FlpFreeList& f = p->tier[tier];
  uint32_t gen = next_gen(f);
  for (int32_t k = 0; k < n; ++k) {
    int32_t id = ids[k];
    if (id < 0 || id >= f.n) {
      flp_set_error("flp_pool_free: id %d out of range [0,%lld)", id, (long long)f.n);
      return FLP_ERANGE;
    }
    if (f.is_free[(size_t)id] || f.stamp[(size_t)id] == gen) {
      flp_set_error("flp_pool_free: block %d is already free or listed twice", id);
      return FLP_EDUP;
    }
    f.stamp[(size_t)id] = gen;
  }
  for (int32_t k = 0; k < n; ++k) {
    f.is_free[(size_t)ids[k]] = 1;
    f.stack.push_back(ids[k]);
  }
  return FLP_OK;
}

// ------------------------------------------------------------------------- staging
flp_status flp_stage_acquire(flp_pool* p, size_t bytes, FlpStageSlot** out) {
  FlpStageSlot& s = p->stage[p->stage_next];
  p->stage_next = (p->stage_next + 1) % kStageSlots;
  if (!s.ev) FLP_TRY_HIP(hipEventCreateWithFlags(&s.ev, hipEventDisableTiming));
  if (s.in_flight) {
    // normally the slot's last use finished long ago: poll first, block only if it has not
    hipError_t q = hipEventQuery(s.ev);
    if (q == hipErrorNotReady) {
      FLP_TRY_HIP(hipEventSynchronize(s.ev));
    } else if (q != hipSuccess) {
      flp_set_error("hipEventQuery failed: %s", hipGetErrorString(q));
      return FLP_EHIP;
    }
    s.in_flight = false;
  }
  if (s.cap < bytes) {
    // freeing device or pinned memory waits for the whole device, so a slot starts large
    // enough (1 MiB) that ordinary id lists and work lists never make it grow
    size_t cap = 1 << 20;
    while (cap < bytes) cap <<= 1;
    if (s.host) FLP_TRY_HIP(hipHostFree(s.host));
    if (s.dev) FLP_TRY_HIP(hipFree(s.dev));
    s.host = s.dev = nullptr;
    s.cap = 0;
    FLP_TRY_HIP(hipHostMalloc(&s.host, cap, hipHostMallocDefault));
    FLP_TRY_HIP(hipMalloc(&s.dev, cap));
    s.cap = cap;
  }
  *out = &s;
  return FLP_OK;
}

flp_status flp_stage_upload(FlpStageSlot* s, size_t bytes, hipStream_t stream) {
  return flp_launch_stage_copy(s->host, s->dev, bytes, stream);   // capacities are multiples of 16
}

flp_status flp_stage_release(FlpStageSlot* s, hipStream_t stream) {
  FLP_TRY_HIP(hipEventRecord(s->ev, stream));
  s->in_flight = true;
  return FLP_OK;
}

// Both workspaces only grow, and a buffer that has become too small is not freed before the pool is destroyed:
// launches enqueued earlier may still read it, and freeing device memory (or waiting for the device) inside a
// compute call would stall every stream.  Capacities double, so the retired buffers together stay below the live one.
static flp_status grow(flp_pool* p, void** buf, size_t* cap_now, size_t bytes) {
  if (*cap_now < bytes) {
    size_t cap = *cap_now ? *cap_now : ((size_t)1 << 20);
    while (cap < bytes) cap <<= 1;
    void* fresh = nullptr;
    FLP_TRY_HIP(hipMalloc(&fresh, cap));
    if (*buf) p->retired.push_back(*buf);
    *buf = fresh;
    *cap_now = cap;
  }
  return FLP_OK;
}

flp_status flp_workspace(flp_pool* p, size_t bytes, void** out) {
  FLP_TRY(grow(p, &p->work, &p->work_cap, bytes));
  *out = p->work;
  return FLP_OK;
}

flp_status flp_attn_workspace(flp_pool* p, size_t bytes, void** out) {
  FLP_TRY(grow(p, &p->attn_work, &p->attn_work_cap, bytes));
  *out = p->attn_work;
  return FLP_OK;
}

// ------------------------------------------------------------------------- swap
// (Paper sections 3.2 / 5.3: the swapper's ordered decisions are carried out as block
// moves, swap-out before swap-in when the device tier is full; section 4.3: on a stream,
// asynchronously to the compute of the requests that are ready.)
// argument and list checks of a swap call (with the pool's lock held)
static flp_status swap_check_locked(flp_pool* p, int32_t n, const int32_t* src_ids, const int32_t* dst_ids, int src_tier,
                                    const char* who) {
  const int dst_tier = 1 - src_tier;
  FlpFreeList& fs = p->tier[src_tier];
  FlpFreeList& fd = p->tier[dst_tier];
  uint32_t gen = next_gen(fd);
  for (int32_t k = 0; k < n; ++k) {
    if (src_ids[k] < 0 || src_ids[k] >= fs.n || dst_ids[k] < 0 || dst_ids[k] >= fd.n) {
      flp_set_error("%s: entry %d (src %d, dst %d) out of range", who, k, src_ids[k], dst_ids[k]);
      return FLP_ERANGE;
    }
    if (fd.stamp[(size_t)dst_ids[k]] == gen) {
      flp_set_error("%s: destination block %d listed twice", who, dst_ids[k]);
      return FLP_EDUP;
    }
    fd.stamp[(size_t)dst_ids[k]] = gen;
  }
  return FLP_OK;
}

flp_status flp_swap_check(flp_pool* p, int32_t n, const int32_t* src_ids, const int32_t* dst_ids, int src_tier,
                          const char* who) {
  if (!p || n < 0 || (n > 0 && (!src_ids || !dst_ids))) {
    flp_set_error("%s: invalid argument", who);
    return FLP_EINVAL;
  }
  std::lock_guard<std::mutex> lk(p->mu);
  return swap_check_locked(p, n, src_ids, dst_ids, src_tier, who);
}

static flp_status swap_common(flp_pool* p, int32_t n, const int32_t* src_ids, const int32_t* dst_ids,
                              int src_tier, void* hip_stream, const char* who, int width = FLP_WIDTH_SINGLE) {
  if (!p || n < 0 || (n > 0 && (!src_ids || !dst_ids))) {
    flp_set_error("%s: invalid argument", who);
    return FLP_EINVAL;
  }
  if (n == 0) return FLP_OK;
  std::lock_guard<std::mutex> lk(p->mu);
  const int dst_tier = 1 - src_tier;
  FLP_TRY(swap_check_locked(p, n, src_ids, dst_ids, src_tier, who));
  hipStream_t stream = (hipStream_t)hip_stream;
  FlpStageSlot* slot = nullptr;
  size_t bytes = sizeof(int32_t) * 2 * (size_t)n;
  FLP_TRY(flp_stage_acquire(p, bytes, &slot));
  int32_t* h = (int32_t*)slot->host;
  memcpy(h, src_ids, sizeof(int32_t) * (size_t)n);
  memcpy(h + n, dst_ids, sizeof(int32_t) * (size_t)n);
  FLP_TRY(flp_stage_upload(slot, bytes, stream));
  const uint8_t* src_base = src_tier == 0 ? p->dev_base : p->host_base;
  uint8_t* dst_base = dst_tier == 0 ? p->dev_base : p->host_base;
  const int32_t* d = (const int32_t*)slot->dev;
  flp_status st = flp_launch_copy_blocks(src_base, dst_base, d, d + n, n, p->block_bytes,
                                         p->host_tier_in_hbm ? FLP_LINK_NONE
                                         : src_tier == 1   ? (width == FLP_WIDTH_DUPLEX   ? FLP_LINK_IN_DUPLEX
                                                              : width == FLP_WIDTH_NARROW ? FLP_LINK_IN_NARROW
                                                                                          : FLP_LINK_IN)
                                                           : (width == FLP_WIDTH_DUPLEX   ? FLP_LINK_OUT_DUPLEX
                                                              : width == FLP_WIDTH_NARROW ? FLP_LINK_OUT_NARROW
                                                                                          : FLP_LINK_OUT),
                                         stream);
  flp_status st2 = flp_stage_release(slot, stream);
  return st != FLP_OK ? st : st2;
}

flp_status flp_swap_width(flp_pool* p, int32_t n, const int32_t* src_ids, const int32_t* dst_ids, int src_tier,
                           void* hip_stream, int width) {
  return swap_common(p, n, src_ids, dst_ids, src_tier, hip_stream, src_tier == 1 ? "fetch" : "write-back", width);
}

extern "C" flp_status flp_pool_swap_in(flp_pool* p, int32_t n, const int32_t* host_ids, const int32_t* dev_ids,
                                       void* hip_stream) {
  return swap_common(p, n, host_ids, dev_ids, 1, hip_stream, "flp_pool_swap_in");
}

extern "C" flp_status flp_pool_swap_out(flp_pool* p, int32_t n, const int32_t* dev_ids, const int32_t* host_ids,
                                        void* hip_stream) {
  return swap_common(p, n, dev_ids, host_ids, 0, hip_stream, "flp_pool_swap_out");
}
