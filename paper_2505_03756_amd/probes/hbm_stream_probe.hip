// What plain streaming kernels reach on this GPU's HBM: the practical ceilings that the memory-bound
// kernels of the library (decode attention: read only; KV append and block copy: read + write to another
// place; LoRA expand: read-modify-write in place) are compared with, beside the published 8 TB/s.
//
// Each kernel moves 16 bytes per lane per access, grid-stride, with U independent accesses in flight per
// lane; buffers are far larger than the 256 MiB of last-level cache.  Times are HIP events around 10
// launches after 3 warm-up launches, best of 3.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>

#define CHECK(x)                                                                       \
  do {                                                                                 \
    hipError_t e_ = (x);                                                               \
    if (e_ != hipSuccess) {                                                            \
      std::fprintf(stderr, "%s:%d %s\n", __FILE__, __LINE__, hipGetErrorString(e_));   \
      std::exit(1);                                                                    \
    }                                                                                  \
  } while (0)

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int U>
__global__ __launch_bounds__(256) void read_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ sink, size_t n) {
  const size_t stride = (size_t)gridDim.x * 256;
  u32x4 acc = {0u, 0u, 0u, 0u};
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + (U - 1) * stride < n; i += U * stride) {
    u32x4 r[U];
#pragma unroll
    for (int u = 0; u < U; ++u) r[u] = src[i + u * stride];
#pragma unroll
    for (int u = 0; u < U; ++u) acc ^= r[u];
  }
  for (; i < n; i += stride) acc ^= src[i];
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[threadIdx.x] = acc;   // keeps the loads alive
}

template <int U>
__global__ __launch_bounds__(256) void copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n) {
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + (U - 1) * stride < n; i += U * stride) {
    u32x4 r[U];
#pragma unroll
    for (int u = 0; u < U; ++u) r[u] = src[i + u * stride];
#pragma unroll
    for (int u = 0; u < U; ++u) dst[i + u * stride] = r[u];
  }
  for (; i < n; i += stride) dst[i] = src[i];
}

// the same copy with non-temporal loads and stores (streaming hints: the lines are not kept in cache)
template <int U>
__global__ __launch_bounds__(256) void copy_nt_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n) {
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + (U - 1) * stride < n; i += U * stride) {
    u32x4 r[U];
#pragma unroll
    for (int u = 0; u < U; ++u) r[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
    for (int u = 0; u < U; ++u) __builtin_nontemporal_store(r[u], dst + i + u * stride);
  }
  for (; i < n; i += stride) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// a workgroup owns a contiguous chunk instead of a grid-strided comb
template <int U>
__global__ __launch_bounds__(256) void copy_chunk_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n) {
  const size_t per = (n + gridDim.x - 1) / gridDim.x;
  const size_t beg = (size_t)blockIdx.x * per, end = beg + per < n ? beg + per : n;
  size_t i = beg + threadIdx.x;
  for (; i + (U - 1) * 256 < end; i += U * 256) {
    u32x4 r[U];
#pragma unroll
    for (int u = 0; u < U; ++u) r[u] = src[i + u * 256];
#pragma unroll
    for (int u = 0; u < U; ++u) dst[i + u * 256] = r[u];
  }
  for (; i < end; i += 256) dst[i] = src[i];
}

template <int U>
__global__ __launch_bounds__(256) void copy_chunk_nt_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n) {
  const size_t per = (n + gridDim.x - 1) / gridDim.x;
  const size_t beg = (size_t)blockIdx.x * per, end = beg + per < n ? beg + per : n;
  size_t i = beg + threadIdx.x;
  for (; i + (U - 1) * 256 < end; i += U * 256) {
    u32x4 r[U];
#pragma unroll
    for (int u = 0; u < U; ++u) r[u] = __builtin_nontemporal_load(src + i + u * 256);
#pragma unroll
    for (int u = 0; u < U; ++u) __builtin_nontemporal_store(r[u], dst + i + u * 256);
  }
  for (; i < end; i += 256) dst[i] = src[i];
}

// update in place, a workgroup owning a contiguous chunk, plain or non-temporal accesses
template <int U, bool NT>
__global__ __launch_bounds__(256) void rmw_chunk_kernel(u32x4* __restrict__ buf, size_t n) {
  const size_t per = (n + gridDim.x - 1) / gridDim.x;
  const size_t beg = (size_t)blockIdx.x * per, end = beg + per < n ? beg + per : n;
  size_t i = beg + threadIdx.x;
  for (; i + (U - 1) * 256 < end; i += U * 256) {
    u32x4 r[U];
#pragma unroll
    for (int u = 0; u < U; ++u) r[u] = NT ? __builtin_nontemporal_load(buf + i + u * 256) : buf[i + u * 256];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (NT) __builtin_nontemporal_store(r[u] + 1u, buf + i + u * 256); else buf[i + u * 256] = r[u] + 1u;
    }
  }
  for (; i < end; i += 256) buf[i] = buf[i] + 1u;
}

template <int U>
__global__ __launch_bounds__(256) void rmw_kernel(u32x4* __restrict__ buf, size_t n) {
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + (U - 1) * stride < n; i += U * stride) {
    u32x4 r[U];
#pragma unroll
    for (int u = 0; u < U; ++u) r[u] = buf[i + u * stride];
#pragma unroll
    for (int u = 0; u < U; ++u) buf[i + u * stride] = r[u] + 1u;
  }
  for (; i < n; i += stride) buf[i] = buf[i] + 1u;
}

// Update in place of a [rows][4096] matrix of 16-bit elements (8 KiB rows) by one-wave workgroups in the
// lane layout of the LoRA expand kernel: 16 rows x 256 columns per step, a lane holding 16 consecutive
// columns of one row (two 16-byte accesses), the four lanes of a row covering a 128-byte line, four such
// 64-column chunks per step.  MODE 0: a wave keeps its 256-column slab and walks down 256 rows in 16 steps
// (what the expand kernel does: the B fragments of the slab stay in registers).  MODE 1: a wave keeps its
// 16 rows and walks along them through the 16 slabs (each row is touched as one contiguous 8 KiB run).
template <int MODE, bool NT>
__global__ __launch_bounds__(64) void rmw_tile_kernel(uint16_t* __restrict__ y, int n_rows) {
  const int lane = threadIdx.x, n = lane & 15, kg = lane >> 4;
  for (int step = 0; step < 16; ++step) {
    int row, slab;
    if (MODE == 0) {
      row = (blockIdx.x >> 4) * 256 + step * 16 + n;
      slab = blockIdx.x & 15;
    } else {
      row = blockIdx.x * 16 + n;
      slab = step;
    }
    if (row >= n_rows) return;
    u32x4* p = reinterpret_cast<u32x4*>(y + (size_t)row * 4096 + 256 * slab + 16 * kg);
    u32x4 r[4][2];
#pragma unroll
    for (int ch = 0; ch < 4; ++ch) {
      r[ch][0] = NT ? __builtin_nontemporal_load(p + 8 * ch) : p[8 * ch];
      r[ch][1] = NT ? __builtin_nontemporal_load(p + 8 * ch + 1) : p[8 * ch + 1];
    }
#pragma unroll
    for (int ch = 0; ch < 4; ++ch) {
      if (NT) {
        __builtin_nontemporal_store(r[ch][0] + 1u, p + 8 * ch);
        __builtin_nontemporal_store(r[ch][1] + 1u, p + 8 * ch + 1);
      } else {
        p[8 * ch] = r[ch][0] + 1u;
        p[8 * ch + 1] = r[ch][1] + 1u;
      }
    }
  }
}

// The same 16 rows x 256 columns per step, but in a row-contiguous lane layout: an access instruction covers
// 4 rows x 256 bytes (lane l: row 4q + l / 16, 16 bytes at column 8 (l % 16) of the 128-column half h), so
// every group of 16 lanes touches two whole lines instead of sixteen partial ones.
template <bool NT>
__global__ __launch_bounds__(64) void rmw_tile_rows_kernel(uint16_t* __restrict__ y, int n_rows) {
  const int lane = threadIdx.x;
  for (int step = 0; step < 16; ++step) {
    const int row0 = (blockIdx.x >> 4) * 256 + step * 16, slab = blockIdx.x & 15;
    if (row0 >= n_rows) return;
    u32x4* p[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int row = row0 + 4 * q + (lane >> 4) < n_rows ? row0 + 4 * q + (lane >> 4) : n_rows - 1;
      p[q] = reinterpret_cast<u32x4*>(y + (size_t)row * 4096 + 256 * slab + 8 * (lane & 15));
    }
    u32x4 r[2][4];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int q = 0; q < 4; ++q) r[h][q] = NT ? __builtin_nontemporal_load(p[q] + 16 * h) : p[q][16 * h];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (NT)
          __builtin_nontemporal_store(r[h][q] + 1u, p[q] + 16 * h);
        else
          p[q][16 * h] = r[h][q] + 1u;
      }
  }
}

template <typename F>
float best_ms(F launch) {
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  for (int i = 0; i < 3; ++i) launch();
  CHECK(hipDeviceSynchronize());
  float best = 1e30f;
  for (int rep = 0; rep < 3; ++rep) {
    CHECK(hipEventRecord(e0, 0));
    for (int i = 0; i < 10; ++i) launch();
    CHECK(hipEventRecord(e1, 0));
    CHECK(hipEventSynchronize(e1));
    float ms;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    best = ms / 10 < best ? ms / 10 : best;
  }
  CHECK(hipGetLastError());
  return best;
}

int main() {
  const size_t bytes = (size_t)2 << 30;            // 2 GiB per buffer
  const size_t n = bytes / 16;
  u32x4 *a, *b;
  CHECK(hipMalloc(&a, bytes));
  CHECK(hipMalloc(&b, bytes));
  CHECK(hipMemset(a, 1, bytes));
  CHECK(hipMemset(b, 2, bytes));
  std::printf("%-28s %8s %10s %12s\n", "kernel", "grid", "ms", "TB/s moved");
  const int grids[] = {1024, 2048, 8192, 32768};
  for (int g : grids) {
    float t = best_ms([&] { hipLaunchKernelGGL(read_kernel<4>, dim3(g), dim3(256), 0, 0, a, b, n); });
    std::printf("%-28s %8d %10.3f %12.2f\n", "read, 4 x 16 B in flight", g, t, bytes / t / 1e9);
    t = best_ms([&] { hipLaunchKernelGGL(read_kernel<8>, dim3(g), dim3(256), 0, 0, a, b, n); });
    std::printf("%-28s %8d %10.3f %12.2f\n", "read, 8 x 16 B in flight", g, t, bytes / t / 1e9);
    t = best_ms([&] { hipLaunchKernelGGL(copy_kernel<4>, dim3(g), dim3(256), 0, 0, a, b, n); });
    std::printf("%-28s %8d %10.3f %12.2f\n", "copy, 4 x 16 B in flight", g, t, 2.0 * bytes / t / 1e9);
    t = best_ms([&] { hipLaunchKernelGGL(copy_kernel<8>, dim3(g), dim3(256), 0, 0, a, b, n); });
    std::printf("%-28s %8d %10.3f %12.2f\n", "copy, 8 x 16 B in flight", g, t, 2.0 * bytes / t / 1e9);
    t = best_ms([&] { hipLaunchKernelGGL(copy_nt_kernel<4>, dim3(g), dim3(256), 0, 0, a, b, n); });
    std::printf("%-28s %8d %10.3f %12.2f\n", "copy, non-temporal, 4 x 16 B", g, t, 2.0 * bytes / t / 1e9);
    t = best_ms([&] { hipLaunchKernelGGL(copy_chunk_kernel<4>, dim3(g), dim3(256), 0, 0, a, b, n); });
    std::printf("%-28s %8d %10.3f %12.2f\n", "copy, chunk per WG, 4 x 16 B", g, t, 2.0 * bytes / t / 1e9);
    t = best_ms([&] { hipLaunchKernelGGL(copy_chunk_nt_kernel<4>, dim3(g), dim3(256), 0, 0, a, b, n); });
    std::printf("%-28s %8d %10.3f %12.2f\n", "copy, chunk + non-temporal", g, t, 2.0 * bytes / t / 1e9);
    t = best_ms([&] { hipLaunchKernelGGL((rmw_chunk_kernel<4, false>), dim3(g), dim3(256), 0, 0, a, n); });
    std::printf("%-28s %8d %10.3f %12.2f\n", "update in place, chunk", g, t, 2.0 * bytes / t / 1e9);
    t = best_ms([&] { hipLaunchKernelGGL((rmw_chunk_kernel<4, true>), dim3(g), dim3(256), 0, 0, a, n); });
    std::printf("%-28s %8d %10.3f %12.2f\n", "update in place, chunk + nt", g, t, 2.0 * bytes / t / 1e9);
    t = best_ms([&] { hipLaunchKernelGGL(rmw_kernel<4>, dim3(g), dim3(256), 0, 0, a, n); });
    std::printf("%-28s %8d %10.3f %12.2f\n", "update in place, 4 x 16 B", g, t, 2.0 * bytes / t / 1e9);
    t = best_ms([&] { hipLaunchKernelGGL(rmw_kernel<8>, dim3(g), dim3(256), 0, 0, a, n); });
    std::printf("%-28s %8d %10.3f %12.2f\n", "update in place, 8 x 16 B", g, t, 2.0 * bytes / t / 1e9);
    std::fflush(stdout);
  }
  // the LoRA expand pattern: 3 x 18944 rows of 8 KiB (what the q,k,v call of the 7b_prefill batch updates)
  {
    const int n_rows = 3 * 18944;
    const double moved = 2.0 * n_rows * 8192.0;
    uint16_t* y = reinterpret_cast<uint16_t*>(a);
    const int g0 = n_rows / 256 * 16, g1 = n_rows / 16;
    float t = best_ms([&] { hipLaunchKernelGGL((rmw_tile_kernel<0, false>), dim3(g0), dim3(64), 0, 0, y, n_rows); });
    std::printf("%-44s %8d %10.3f %12.2f\n", "tile update, wave keeps its 256 columns", g0, t, moved / t / 1e9);
    t = best_ms([&] { hipLaunchKernelGGL((rmw_tile_kernel<0, true>), dim3(g0), dim3(64), 0, 0, y, n_rows); });
    std::printf("%-44s %8d %10.3f %12.2f\n", "  same, non-temporal", g0, t, moved / t / 1e9);
    t = best_ms([&] { hipLaunchKernelGGL((rmw_tile_kernel<1, false>), dim3(g1), dim3(64), 0, 0, y, n_rows); });
    std::printf("%-44s %8d %10.3f %12.2f\n", "tile update, wave keeps its 16 rows", g1, t, moved / t / 1e9);
    t = best_ms([&] { hipLaunchKernelGGL((rmw_tile_kernel<1, true>), dim3(g1), dim3(64), 0, 0, y, n_rows); });
    std::printf("%-44s %8d %10.3f %12.2f\n", "  same, non-temporal", g1, t, moved / t / 1e9);
    t = best_ms([&] { hipLaunchKernelGGL((rmw_tile_rows_kernel<false>), dim3(g0), dim3(64), 0, 0, y, n_rows); });
    std::printf("%-44s %8d %10.3f %12.2f\n", "tile update, 256 columns, row-contiguous lanes", g0, t, moved / t / 1e9);
    t = best_ms([&] { hipLaunchKernelGGL((rmw_tile_rows_kernel<true>), dim3(g0), dim3(64), 0, 0, y, n_rows); });
    std::printf("%-44s %8d %10.3f %12.2f\n", "  same, non-temporal", g0, t, moved / t / 1e9);
  }
  CHECK(hipFree(a));
  CHECK(hipFree(b));
  return 0;
}
