// Batched heterogeneous LoRA over paged adapters (paper Eq. 1 / Eq. 2 in row-vector form:
// y = base + s (x A^T) B, section 2.1: queries with different adapters share one batch;
// section 4.3: adapters are split along the rank dimension into pool blocks).
//
// This file holds the adapter segmentation (stable counting sort of token indices by
// adapter id) and the vector-ALU shrink / expand kernels that serve fp32 pools.
#include <hip/hip_runtime.h>

#include "flp_internal.h"
#include "flp_types.h"

namespace {

// ----------------------------------------------------------------------------- segmentation
// One workgroup of 16 waves.  Wave w owns a contiguous range of tokens; per-wave
// histograms give every wave the first output position of each adapter inside its range,
// so the waves can place their tokens independently and still keep the original order
// inside each adapter (a stable counting sort, bit-exact against a sequential one).
constexpr int kSegWaves = 16;

__global__ __launch_bounds__(1024) void lora_segment_kernel(int32_t T, const int32_t* __restrict__ token_adapter,
                                                            int32_t n_ad, int32_t* __restrict__ n_seg,
                                                            int32_t* __restrict__ seg_adapter,
                                                            int32_t* __restrict__ seg_start,
                                                            int32_t* __restrict__ perm, int32_t tm,
                                                            int32_t* __restrict__ tile_start, int32_t tg,
                                                            int32_t* __restrict__ group_start) {
  extern __shared__ int32_t sm[];
  int32_t* whist = sm;                         // [kSegWaves][n_ad]: counts, then running cursors
  int32_t* tot = sm + kSegWaves * n_ad;        // [n_ad] tokens per adapter
  int32_t* seg_off = tot + n_ad;               // [n_ad] first output position of the adapter
  int32_t* wsum = seg_off + n_ad;              // [4*kSegWaves + 4] scan scratch
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;

  for (int i = tid; i < kSegWaves * n_ad; i += 1024) whist[i] = 0;
  __syncthreads();

  const int chunk = (((T + kSegWaves - 1) / kSegWaves) + 63) & ~63;
  const int lo = wave * chunk < T ? wave * chunk : T;
  const int hi = lo + chunk < T ? lo + chunk : T;
  // counting: the lanes that hold the same adapter are matched with ballots and their leader
  // adds the group's size (tokens of one sequence share an adapter, so a wave usually sees
  // one or two distinct ids per 64 tokens; no atomics, each wave owns its row of counters)
  {
    volatile int32_t* cnt_row = whist + wave * n_ad;
    for (int tb = lo; tb < hi; tb += 64 * 8) {        // 8 loads in flight per lane, then their 8 ballot rounds
      int a8[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const int t = tb + 64 * k + lane;
        a8[k] = t < hi ? token_adapter[t] : -1;
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const int a = a8[k];
        const bool valid = a >= 0 && a < n_ad;
        uint64_t remaining = __ballot(valid);
        while (remaining) {
          const int leader = __ffsll((long long)remaining) - 1;
          const int v = __shfl(a, leader);
          const uint64_t same = __ballot(valid && a == v);
          if (lane == leader) cnt_row[v] = cnt_row[v] + __popcll(same);
          __builtin_amdgcn_wave_barrier();
          remaining &= ~same;
        }
      }
    }
  }
  __syncthreads();

  // per adapter: total, and per-wave exclusive offsets
  for (int a = tid; a < n_ad; a += 1024) {
    int run = 0;
    for (int w = 0; w < kSegWaves; ++w) {
      int c = whist[w * n_ad + a];
      whist[w * n_ad + a] = run;
      run += c;
    }
    tot[a] = run;
  }
  __syncthreads();

  // exclusive scan over adapters of (count, non-empty flag); thread i owns a run of adapters
  const int per = (n_ad + 1023) / 1024;
  // (two more quantities ride along for the matrix-core kernels: the number of tm-token tiles
  // and the number of tg-token tile groups)
  int cnt = 0, flg = 0, til = 0, grp = 0;
  for (int k = 0; k < per; ++k) {
    int a = tid * per + k;
    if (a < n_ad) {
      cnt += tot[a];
      flg += tot[a] > 0;
      if (tm > 0) til += (tot[a] + tm - 1) / tm;
      if (tg > 0) grp += (tot[a] + tg - 1) / tg;
    }
  }
  int icnt = cnt, iflg = flg, itil = til, igrp = grp;      // inclusive wave scan
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    int c = __shfl_up(icnt, off), f = __shfl_up(iflg, off), t = __shfl_up(itil, off), gq = __shfl_up(igrp, off);
    if (lane >= off) {
      icnt += c;
      iflg += f;
      itil += t;
      igrp += gq;
    }
  }
  if (lane == 63) {
    wsum[wave] = icnt;
    wsum[kSegWaves + wave] = iflg;
    wsum[2 * kSegWaves + wave] = itil;
    wsum[3 * kSegWaves + wave] = igrp;
  }
  __syncthreads();
  if (tid == 0) {
    int rc = 0, rf = 0, rt = 0, rg = 0;
    for (int w = 0; w < kSegWaves; ++w) {
      int c = wsum[w], f = wsum[kSegWaves + w], t = wsum[2 * kSegWaves + w], gq = wsum[3 * kSegWaves + w];
      wsum[w] = rc;
      wsum[kSegWaves + w] = rf;
      wsum[2 * kSegWaves + w] = rt;
      wsum[3 * kSegWaves + w] = rg;
      rc += c;
      rf += f;
      rt += t;
      rg += gq;
    }
    wsum[4 * kSegWaves] = rc;
    wsum[4 * kSegWaves + 1] = rf;
    wsum[4 * kSegWaves + 2] = rt;
    wsum[4 * kSegWaves + 3] = rg;
  }
  __syncthreads();
  {
    int pos = wsum[wave] + icnt - cnt;         // tokens before this thread's first adapter
    int seg = wsum[kSegWaves + wave] + iflg - flg;
    int tl = wsum[2 * kSegWaves + wave] + itil - til;
    int gr = wsum[3 * kSegWaves + wave] + igrp - grp;
    for (int k = 0; k < per; ++k) {
      int a = tid * per + k;
      if (a < n_ad) {
        seg_off[a] = pos;
        if (tot[a] > 0) {
          seg_adapter[seg] = a;
          seg_start[seg] = pos;
          if (tile_start) tile_start[seg] = tl;
          if (group_start) group_start[seg] = gr;
          ++seg;
        }
        pos += tot[a];
        if (tm > 0) tl += (tot[a] + tm - 1) / tm;
        if (tg > 0) gr += (tot[a] + tg - 1) / tg;
      }
    }
    if (tid == 0) {
      *n_seg = wsum[4 * kSegWaves + 1];
      seg_start[wsum[4 * kSegWaves + 1]] = wsum[4 * kSegWaves];
      if (tile_start) tile_start[wsum[4 * kSegWaves + 1]] = wsum[4 * kSegWaves + 2];
      if (group_start) group_start[wsum[4 * kSegWaves + 1]] = wsum[4 * kSegWaves + 3];
    }
  }
  __syncthreads();

  // placement: each wave walks its range in order, 64 tokens at a time
  volatile int32_t* cur = whist + wave * n_ad;
  for (int tb = lo; tb < hi; tb += 64 * 8) {
    int a8[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int t = tb + 64 * k + lane;
      a8[k] = t < hi ? token_adapter[t] : -1;
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int t = tb + 64 * k + lane;
      const int a = a8[k];
      const bool valid = a >= 0 && a < n_ad;
      uint64_t remaining = __ballot(valid);
      while (remaining) {
        const int leader = __ffsll((long long)remaining) - 1;
        const int v = __shfl(a, leader);
        const uint64_t same = __ballot(valid && a == v);
        const int before = cur[v];
        if (valid && a == v) perm[seg_off[v] + before + __popcll(same & ((1ull << lane) - 1))] = t;
        __builtin_amdgcn_wave_barrier();
        if (lane == leader) cur[v] = before + __popcll(same);
        __builtin_amdgcn_wave_barrier();
        remaining &= ~same;
      }
    }
  }
}

// ----------------------------------------------------------------------------- vector-ALU LoRA
// shrink: one wave per (token, projection); v[t,p,rho] = sum_c x[t,c] A[rho,c], fp32.
template <typename S>
__global__ __launch_bounds__(256) void lora_shrink_rows_kernel(FlpLoraArgs a) {
  typedef typename S::storage ST;
  constexpr int EPL = 16 / (int)sizeof(ST);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + wave;
  const int p = blockIdx.y;
  if (t >= a.T) return;
  const int ad = a.token_adapter[t];
  if (ad < 0 || ad >= a.n_adapters) return;
  const int r = a.rank[ad] < a.max_rank ? a.rank[ad] : a.max_rank;
  if (r <= 0) return;
  const ST* __restrict__ pool = reinterpret_cast<const ST*>(a.pool);
  const ST* __restrict__ xrow = reinterpret_cast<const ST*>(a.x) + (int64_t)t * a.ld_x;
  const int32_t* __restrict__ table = a.tables + a.proj[p].a_tab_off[ad];
  const int row0 = a.proj[p].a_row_base[ad];
  const int rpb = (int)(a.block_elems / a.d_in);
  float* __restrict__ vout = a.v + ((int64_t)t * a.n_proj + p) * a.max_rank;
  for (int r0 = 0; r0 < r; r0 += 8) {
    const ST* rows[8];
    float acc[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      int row = row0 + (r0 + k < r ? r0 + k : r0);
      rows[k] = pool + (int64_t)table[row / rpb] * a.block_elems + (int64_t)(row % rpb) * a.d_in;
      acc[k] = 0.f;
    }
    for (int c0 = lane * EPL; c0 < a.d_in; c0 += 64 * EPL) {
      ST xs[EPL];
      u32x4 raw = *reinterpret_cast<const u32x4*>(xrow + c0);
      __builtin_memcpy(xs, &raw, 16);
      float xf[EPL];
#pragma unroll
      for (int e = 0; e < EPL; ++e) xf[e] = S::to_float(xs[e]);
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        ST as[EPL];
        u32x4 ra = *reinterpret_cast<const u32x4*>(rows[k] + c0);
        __builtin_memcpy(as, &ra, 16);
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[k] = fmaf(xf[e], S::to_float(as[e]), acc[k]);
      }
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      float s = acc[k];
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
      if (lane == 0 && r0 + k < r) vout[r0 + k] = s;
    }
  }
}

// expand: one thread per 16 bytes of a y row; y[t,o] += s * sum_rho v[t,p,rho] B[rho,o].
template <typename S>
__global__ __launch_bounds__(256) void lora_expand_rows_kernel(FlpLoraArgs a) {
  typedef typename S::storage ST;
  constexpr int EPL = 16 / (int)sizeof(ST);
  const int t = blockIdx.x;
  const int p = blockIdx.z;
  const flp_lora_proj& pr = a.proj[p];
  const int col0 = (blockIdx.y * 256 + threadIdx.x) * EPL;
  if (col0 >= pr.d_out) return;
  const int ad = a.token_adapter[t];
  if (ad < 0 || ad >= a.n_adapters) return;
  const int r = a.rank[ad] < a.max_rank ? a.rank[ad] : a.max_rank;
  if (r <= 0) return;
  const float sc = a.scale[ad];
  const ST* __restrict__ pool = reinterpret_cast<const ST*>(a.pool);
  const int32_t* __restrict__ table = a.tables + pr.b_tab_off[ad];
  const int row0 = pr.b_row_base[ad];
  const int rpb = (int)(a.block_elems / pr.d_out);
  const float* __restrict__ v = a.v + ((int64_t)t * a.n_proj + p) * a.max_rank;
  float acc[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
  for (int rho = 0; rho < r; ++rho) {
    const int row = row0 + rho;
    const ST* brow = pool + (int64_t)table[row / rpb] * a.block_elems + (int64_t)(row % rpb) * pr.d_out + col0;
    ST bs[EPL];
    u32x4 raw = *reinterpret_cast<const u32x4*>(brow);
    __builtin_memcpy(bs, &raw, 16);
    const float vv = v[rho];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = fmaf(vv, S::to_float(bs[e]), acc[e]);
  }
  ST* yp = reinterpret_cast<ST*>(pr.y) + (int64_t)t * pr.ld_y + col0;
  ST ys[EPL];
  u32x4 raw;
  if (a.base32[p]) {                               // unrounded base from the dense projection
    const float* bp = a.base32[p] + (int64_t)t * pr.d_out + col0;
#pragma unroll
    for (int e = 0; e < EPL; ++e) ys[e] = S::from_float(fmaf(sc, acc[e], bp[e]));
  } else {
    raw = *reinterpret_cast<const u32x4*>(yp);
    __builtin_memcpy(ys, &raw, 16);
#pragma unroll
    for (int e = 0; e < EPL; ++e) ys[e] = S::from_float(fmaf(sc, acc[e], S::to_float(ys[e])));
  }
  __builtin_memcpy(&raw, ys, 16);
  *reinterpret_cast<u32x4*>(yp) = raw;
}

}  // namespace

flp_status flp_launch_lora_segment(int32_t T, const int32_t* token_adapter, int32_t n_adapters, int32_t* n_seg,
                                   int32_t* seg_adapter, int32_t* seg_start, int32_t* perm, int32_t tm,
                                   int32_t* tile_start, int32_t tg, int32_t* group_start, hipStream_t stream) {
  const size_t smem = ((size_t)(kSegWaves + 2) * (size_t)(n_adapters > 0 ? n_adapters : 1) + 4 * kSegWaves + 4) * 4;
  static bool attr_set = false;
  if (!attr_set) {
    FLP_TRY_HIP(hipFuncSetAttribute((const void*)lora_segment_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    160 * 1024));
    attr_set = true;
  }
  hipLaunchKernelGGL(lora_segment_kernel, dim3(1), dim3(1024), smem, stream, T, token_adapter, n_adapters, n_seg,
                     seg_adapter, seg_start, perm, tm, tile_start, tg, group_start);
  FLP_TRY_HIP(hipGetLastError());
  return FLP_OK;
}

flp_status flp_launch_lora_simple(int dtype, const FlpLoraArgs& a, hipStream_t stream) {
  if (a.T <= 0) return FLP_OK;
  const int epl = dtype == FLP_F32 ? 4 : 8;
  int max_dout = 0;
  for (int p = 0; p < a.n_proj; ++p) max_dout = a.proj[p].d_out > max_dout ? a.proj[p].d_out : max_dout;
  dim3 gs((unsigned)((a.T + 3) / 4), (unsigned)a.n_proj);
  dim3 ge((unsigned)a.T, (unsigned)((max_dout + 256 * epl - 1) / (256 * epl)), (unsigned)a.n_proj);
  if (dtype == FLP_F32) {
    hipLaunchKernelGGL(lora_shrink_rows_kernel<F32>, gs, dim3(256), 0, stream, a);
    hipLaunchKernelGGL(lora_expand_rows_kernel<F32>, ge, dim3(256), 0, stream, a);
  } else if (dtype == FLP_F16) {
    hipLaunchKernelGGL(lora_shrink_rows_kernel<F16>, gs, dim3(256), 0, stream, a);
    hipLaunchKernelGGL(lora_expand_rows_kernel<F16>, ge, dim3(256), 0, stream, a);
  } else {
    hipLaunchKernelGGL(lora_shrink_rows_kernel<BF16>, gs, dim3(256), 0, stream, a);
    hipLaunchKernelGGL(lora_expand_rows_kernel<BF16>, ge, dim3(256), 0, stream, a);
  }
  FLP_TRY_HIP(hipGetLastError());
  return FLP_OK;
}
