// Block gather/scatter copy behind swap-in and swap-out (paper sections 3.2, 4.3, 5.3:
// the swapper's decisions are executed as moves of whole pool blocks between the host
// tier and the device tier).  One launch moves the whole list: workgroups walk a
// (block, chunk) grid and copy 16 bytes per lane with several loads in flight, reading or
// writing the pinned host tier directly over the host link, so the cost per block is the
// transfer itself rather than one copy-engine submission per block.
#include <hip/hip_runtime.h>

#include <cstdlib>

#include "flp_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 4;

// A fixed number of workgroups walks the (block, chunk) grid with a stride: the host link
// needs only a few hundred KiB in flight to stay busy, so a small resident grid reaches the
// same rate as one workgroup per chunk and leaves the rest of the chip to the compute
// kernels that run beside the swap on another stream.
template <typename V>
__global__ __launch_bounds__(kThreads) void copy_blocks_kernel(const uint8_t* __restrict__ src_base,
                                                               uint8_t* __restrict__ dst_base,
                                                               const int32_t* __restrict__ src_ids,
                                                               const int32_t* __restrict__ dst_ids,
                                                               int64_t block_bytes, int32_t chunks_per_block,
                                                               int64_t vec_per_chunk, int64_t total_chunks) {
  const int64_t nvec = block_bytes / (int64_t)sizeof(V);
  for (int64_t w = blockIdx.x; w < total_chunks; w += gridDim.x) {
    const int32_t blk = (int32_t)(w / chunks_per_block);
    const int32_t chunk = (int32_t)(w - (int64_t)blk * chunks_per_block);
    const V* __restrict__ s = reinterpret_cast<const V*>(src_base + (int64_t)src_ids[blk] * block_bytes);
    V* __restrict__ d = reinterpret_cast<V*>(dst_base + (int64_t)dst_ids[blk] * block_bytes);
    const int64_t lo = (int64_t)chunk * vec_per_chunk;
    const int64_t hi = lo + vec_per_chunk < nvec ? lo + vec_per_chunk : nvec;
    for (int64_t i = lo + threadIdx.x; i < hi; i += kThreads * kUnroll) {
      V r[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        int64_t j = i + (int64_t)u * kThreads;
        if (j < hi) r[u] = __builtin_nontemporal_load(s + j);
      }
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        int64_t j = i + (int64_t)u * kThreads;
        if (j < hi) __builtin_nontemporal_store(r[u], d + j);
      }
    }
  }
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Small host-to-device copy of staged id / work lists, as a kernel on the caller's stream:
// it stays in order with the kernels that consume the lists without a hand-off to a copy
// engine and back.
__global__ __launch_bounds__(kThreads) void stage_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                                              int64_t n_vec) {
  int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i < n_vec) dst[i] = src[i];
}

}  // namespace

flp_status flp_launch_stage_copy(const void* src_pinned, void* dst_dev, size_t bytes, hipStream_t stream) {
  const int64_t n_vec = (int64_t)((bytes + 15) / 16);
  if (n_vec == 0) return FLP_OK;
  hipLaunchKernelGGL(stage_copy_kernel, dim3((unsigned)((n_vec + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream,
                     (const u32x4*)src_pinned, (u32x4*)dst_dev, n_vec);
  FLP_TRY_HIP(hipGetLastError());
  return FLP_OK;
}

flp_status flp_launch_copy_blocks(const uint8_t* src_base, uint8_t* dst_base, const int32_t* src_ids_dev,
                                  const int32_t* dst_ids_dev, int32_t n, int64_t block_bytes, int host_link,
                                  hipStream_t stream) {
  if (n <= 0) return FLP_OK;
  const int64_t chunk_bytes = 16384;
  const int64_t chunks = (block_bytes + chunk_bytes - 1) / chunk_bytes;
  const int64_t total = (int64_t)n * chunks;
  // Measured on MI355X.  One direction alone: 16 resident workgroups saturate the host link (57 GB/s in,
  // 55 GB/s out), and every further workgroup that waits on host-link reads slows the HBM traffic of the
  // kernels running beside the move (96 workgroups: a streaming copy on another stream runs 4x slower;
  // 16: 1.1x).  Both directions at once share the link unevenly at equal widths (16 and 16: 40 GB/s in,
  // 47 out, and the write-backs are what slows the kernels beside them most); the fetch is what the next
  // compute step waits for, so a caller that runs both directions together (the planner, for a request
  // with both lists) asks for three workgroups per XCD in and one out: 46 and 45 GB/s (a step of 1.44 GB
  // each way: 36.7 ms at 16 and 16, 33.7 ms at 24 and 8; widths that do not divide by the 8 XCDs load
  // them unevenly and do worse).  A tier that lives in device memory wants the whole chip.
  // Moves that need not hurry (a small request beside a whole compute step) run on 12 and 4 workgroups: about two
  // thirds of the rate, and the matrix-bound attention kernel beside them is not slowed at all (12.7 -> 13.0 ms
  // instead of -> 17.9 ms beside the wide pair).
  const int64_t max_wgs = host_link == FLP_LINK_NONE         ? 2048
                          : host_link == FLP_LINK_IN_DUPLEX  ? 24
                          : host_link == FLP_LINK_OUT_DUPLEX ? 8
                          : host_link == FLP_LINK_IN_NARROW  ? 12
                          : host_link == FLP_LINK_OUT_NARROW ? 4
                                                             : 16;
  dim3 grid((unsigned)(total < max_wgs ? total : max_wgs));
  if (block_bytes % 16 == 0) {
    hipLaunchKernelGGL(copy_blocks_kernel<u32x4>, grid, dim3(kThreads), 0, stream, src_base, dst_base, src_ids_dev,
                       dst_ids_dev, block_bytes, (int32_t)chunks, chunk_bytes / 16, total);
  } else if (block_bytes % 4 == 0) {
    hipLaunchKernelGGL(copy_blocks_kernel<uint32_t>, grid, dim3(kThreads), 0, stream, src_base, dst_base,
                       src_ids_dev, dst_ids_dev, block_bytes, (int32_t)chunks, chunk_bytes / 4, total);
  } else {
    hipLaunchKernelGGL(copy_blocks_kernel<uint16_t>, grid, dim3(kThreads), 0, stream, src_base, dst_base,
                       src_ids_dev, dst_ids_dev, block_bytes, (int32_t)chunks, chunk_bytes / 2, total);
  }
  FLP_TRY_HIP(hipGetLastError());
  return FLP_OK;
}
