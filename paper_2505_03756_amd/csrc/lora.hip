// Batched heterogeneous LoRA over paged adapters (paper Eq. 1 / Eq. 2 in row-vector form:
// y = base + s (x A^T) B, section 2.1: queries with different adapters share one batch;
// section 4.3: adapters are split along the rank dimension into pool blocks).
//
// This file holds the adapter segmentation (stable counting sort of token indices by
// adapter id) and the vector-ALU shrink / expand kernels that serve fp32 pools.
#include <atomic>
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
                                                            int32_t* __restrict__ group_start,
                                                            int32_t* __restrict__ inv_perm,
                                                            int32_t* __restrict__ vrow_base) {
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
        // row of the shrink output that holds the adapter's first token, minus that token's position: a token at
        // position pos sits in row vrow_base[a] + pos
        if (vrow_base) vrow_base[a] = tl * tm - pos;
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
        if (valid && a == v) {
          const int pos = seg_off[v] + before + __popcll(same & ((1ull << lane) - 1));
          perm[pos] = t;
          if (inv_perm) inv_perm[t] = pos;
        }
        __builtin_amdgcn_wave_barrier();
        if (lane == leader) cur[v] = before + __popcll(same);
        __builtin_amdgcn_wave_barrier();
        remaining &= ~same;
      }
    }
  }
}

// ----------------------------------------------------------------------------- vector-ALU LoRA
// The per-token kernels below serve fp32 pools, widths the matrix-core tiles do not divide, and small
// (decode) batches.  In a decode batch a few tokens share each adapter, and the adapters' pages, not the
// activations, are the traffic: the tokens of one adapter are therefore taken four at a time by one
// workgroup, which reads the pages once for all four.  Who belongs together is found by every workgroup
// itself from the batch's adapter ids (a bit mask of the tokens with the same id, built with ballots);
// that scan is only done for batches of up to kShareMaxT tokens, larger ones take every token alone.
constexpr int kShareTokens = 4;
constexpr int kShareMaxT = 1024;

// The batch's adapter ids, kShareMaxT / 256 per thread: requested early, so that they arrive while the
// workgroup looks up its adapter's rank and pages.
__device__ __forceinline__ void mates_prefetch(const int32_t* __restrict__ token_adapter, int T, int ids[kShareMaxT / 256]) {
#pragma unroll
  for (int j = 0; j < kShareMaxT / 256; ++j) {
    const int i = 256 * j + (int)threadIdx.x;
    ids[j] = i < T ? token_adapter[i] : -1;
  }
}

// For token t of adapter ad (>= 0): the tokens with the same adapter, in token order, are taken in fours and
// the first of each four works for all of them.  Returns how many tokens this workgroup handles (0: t is
// not a first) and their indices in tok[] (unused entries repeat t).  All 256 threads call it; mask is
// LDS, kShareMaxT / 64 words.
__device__ __forceinline__ int adapter_mates(const int ids[kShareMaxT / 256], int T, int t, int ad, uint64_t* mask,
                                             int tok[kShareTokens]) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int j = 0; j < kShareMaxT / 256; ++j) {
    const uint64_t b = __ballot(ids[j] == ad);
    if ((tid & 63) == 0) mask[4 * j + (tid >> 6)] = b;
  }
  __syncthreads();
  const int nw = (T + 63) >> 6;
  int w = t >> 6, before = 0;
  for (int k = 0; k < w; ++k) before += __popcll(mask[k]);
  before += __popcll(mask[w] & ((1ull << (t & 63)) - 1));
  if (before % kShareTokens) return 0;
  uint64_t cur = mask[w] & ~((1ull << (t & 63)) - 1);     // bit t itself is set: tok[0] == t
  int n = 0;
#pragma unroll
  for (int k = 0; k < kShareTokens; ++k) {
    while (!cur && w + 1 < nw) cur = mask[++w];
    if (cur) {
      tok[k] = __builtin_amdgcn_readfirstlane(64 * w + __ffsll((long long)cur) - 1);
      cur &= cur - 1;
      n = k + 1;
    } else {
      tok[k] = t;
    }
  }
  return __builtin_amdgcn_readfirstlane(n);
}

// shrink: one workgroup per (token four, projection, block of 8 ranks); v[t,p,rho] = sum_c x[t,c] A[rho,c],
// fp32.  The four waves split the row's columns between them, eight ranks and two column pieces (16 loads
// of 16 bytes) in flight per lane; the waves' partial sums meet in LDS.
template <typename S>
__global__ __launch_bounds__(256) void lora_shrink_rows_kernel(FlpLoraArgs a) {
  typedef typename S::storage ST;
  constexpr int EPL = 16 / (int)sizeof(ST);
  constexpr int NTK = kShareTokens;
  __shared__ float part[4][NTK][8];
  __shared__ uint64_t mask[kShareMaxT / 64];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int t = blockIdx.x, p = blockIdx.y, r0 = 8 * blockIdx.z;
  const bool share = a.T <= kShareMaxT;
  int ids[kShareMaxT / 256];
  if (share) mates_prefetch(a.token_adapter, a.T, ids);
  const int ad = a.token_adapter[t];
  if (ad < 0 || ad >= a.n_adapters) return;           // every exit up to the barrier is uniform over the workgroup
  const int r = a.rank[ad] < a.max_rank ? a.rank[ad] : a.max_rank;
  if (r0 >= r) return;
  const ST* __restrict__ pool = reinterpret_cast<const ST*>(a.pool);
  const int32_t* __restrict__ table = a.tables + a.proj[p].a_tab_off[ad];
  const int row0 = a.proj[p].a_row_base[ad];
  const int rpb = (int)(a.block_elems / a.d_in);
  constexpr int kStep = 256 * EPL;                     // columns the workgroup covers per piece
  const ST* rows[8];
  float acc[NTK][8];
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const int row = row0 + (r0 + k < r ? r0 + k : r0);
    rows[k] = pool + (int64_t)table[row / rpb] * a.block_elems + (int64_t)(row % rpb) * a.d_in;
#pragma unroll
    for (int j = 0; j < NTK; ++j) acc[j][k] = 0.f;
  }
  int tok[NTK] = {t, t, t, t};
  int n_tok = 1;
  if (share) {
    n_tok = adapter_mates(ids, a.T, t, ad, mask, tok);
    if (n_tok == 0) return;
  }
  for (int c0 = tid * EPL; c0 < a.d_in; c0 += 2 * kStep) {
    const bool two = c0 + kStep < a.d_in;
    const int c1 = two ? c0 + kStep : c0;               // a second piece past the row repeats the first, weight zero
    u32x4 ra0[8], ra1[8], rx0[NTK], rx1[NTK];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      ra0[k] = *reinterpret_cast<const u32x4*>(rows[k] + c0);
      ra1[k] = *reinterpret_cast<const u32x4*>(rows[k] + c1);
    }
#pragma unroll
    for (int j = 0; j < NTK; ++j) {
      const ST* xrow = reinterpret_cast<const ST*>(a.x) + (int64_t)tok[j] * a.ld_x;
      rx0[j] = *reinterpret_cast<const u32x4*>(xrow + c0);
      rx1[j] = *reinterpret_cast<const u32x4*>(xrow + c1);
    }
    if (!two) {
#pragma unroll
      for (int j = 0; j < NTK; ++j) rx1[j] = u32x4{0u, 0u, 0u, 0u};
    }
    // element by element, so that only the eight ranks' current values are live as floats
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      float a0[8], a1[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        ST as0[EPL], as1[EPL];
        __builtin_memcpy(as0, &ra0[k], 16);
        __builtin_memcpy(as1, &ra1[k], 16);
        a0[k] = S::to_float(as0[e]);
        a1[k] = S::to_float(as1[e]);
      }
#pragma unroll
      for (int j = 0; j < NTK; ++j) {
        if (j < n_tok) {
          ST xs0[EPL], xs1[EPL];
          __builtin_memcpy(xs0, &rx0[j], 16);
          __builtin_memcpy(xs1, &rx1[j], 16);
          const float x0 = S::to_float(xs0[e]), x1 = S::to_float(xs1[e]);
#pragma unroll
          for (int k = 0; k < 8; ++k) acc[j][k] = fmaf(x1, a1[k], fmaf(x0, a0[k], acc[j][k]));
        }
      }
    }
  }
#pragma unroll
  for (int j = 0; j < NTK; ++j) {
    if (j < n_tok) {
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        float s = acc[j][k];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
        if (lane == 0) part[wave][j][k] = s;
      }
    }
  }
  __syncthreads();
  if (tid < 8 * NTK) {
    const int j = tid >> 3, k = tid & 7;
    if (j < n_tok && r0 + k < r) {
      int tj = tok[0];
#pragma unroll
      for (int q = 1; q < NTK; ++q) tj = j == q ? tok[q] : tj;
      a.v[((int64_t)tj * a.n_proj + p) * a.max_rank + r0 + k] =
          (part[0][j][k] + part[1][j][k]) + (part[2][j][k] + part[3][j][k]);
    }
  }
}

// expand: one workgroup per (token four, 64 x 16-byte column slab, projection); y[t,o] += s * sum_rho
// v[t,p,rho] B[rho,o].  Wave w takes the ranks 8w..8w+7 and 32+8w..32+8w+7 (eight pieces of B in flight
// per lane), the partial sums of the four waves meet in LDS, and wave j adds them into token j's row.
template <typename S>
__global__ __launch_bounds__(256) void lora_expand_rows_kernel(FlpLoraArgs a) {
  typedef typename S::storage ST;
  constexpr int EPL = 16 / (int)sizeof(ST);
  constexpr int NTK = kShareTokens;
  __shared__ float red[4][NTK][EPL][64];               // [wave][token][element][lane]: conflict-free both ways
  __shared__ uint64_t mask[kShareMaxT / 64];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int t = blockIdx.x;
  const int p = blockIdx.z;
  const flp_lora_proj& pr = a.proj[p];
  const int slab0 = blockIdx.y * 64 * EPL;
  if (slab0 >= pr.d_out) return;                        // every exit up to the barriers is uniform over the workgroup
  const bool share = a.T <= kShareMaxT;
  int ids[kShareMaxT / 256];
  if (share) mates_prefetch(a.token_adapter, a.T, ids);
  const int ad = a.token_adapter[t];
  if (ad < 0 || ad >= a.n_adapters) return;
  const int r = a.rank[ad] < a.max_rank ? a.rank[ad] : a.max_rank;
  if (r <= 0) return;
  const int col0 = slab0 + lane * EPL;
  const bool cvalid = col0 < pr.d_out;
  const int colc = cvalid ? col0 : slab0;
  const float sc = a.scale[ad];
  const ST* __restrict__ pool = reinterpret_cast<const ST*>(a.pool);
  const int32_t* __restrict__ table = a.tables + pr.b_tab_off[ad];
  const int row0 = pr.b_row_base[ad];
  const int rpb = (int)(a.block_elems / pr.d_out);
  int tok[NTK] = {t, t, t, t};
  int n_tok = 1;
  if (share) {
    n_tok = adapter_mates(ids, a.T, t, ad, mask, tok);
    if (n_tok == 0) return;
  }
  // this wave's token for the last step: its y piece is on its way while B streams
  int tw = tok[0];
#pragma unroll
  for (int q = 1; q < NTK; ++q) tw = wave == q ? tok[q] : tw;
  ST* yp = reinterpret_cast<ST*>(pr.y) + (int64_t)tw * pr.ld_y + colc;
  u32x4 yraw{};
  if (wave < n_tok && !a.base32[p]) yraw = *reinterpret_cast<const u32x4*>(yp);
  float acc[NTK][EPL];
#pragma unroll
  for (int j = 0; j < NTK; ++j)
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[j][e] = 0.f;
  for (int rho0 = 8 * wave; rho0 < r; rho0 += 32) {
    u32x4 raw8[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int row = row0 + (rho0 + k < r ? rho0 + k : r - 1);      // ranks past r repeat the last one, weight zero
      raw8[k] = *reinterpret_cast<const u32x4*>(pool + (int64_t)table[row / rpb] * a.block_elems +
                                                (int64_t)(row % rpb) * pr.d_out + colc);
    }
    float vv[NTK][8];
#pragma unroll
    for (int j = 0; j < NTK; ++j) {
      const float* __restrict__ v = a.v + ((int64_t)tok[j] * a.n_proj + p) * a.max_rank;
#pragma unroll
      for (int k = 0; k < 8; ++k) vv[j][k] = (j < n_tok && rho0 + k < r) ? v[rho0 + k < r ? rho0 + k : r - 1] : 0.f;
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      ST bs[EPL];
      __builtin_memcpy(bs, &raw8[k], 16);
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        const float bf = S::to_float(bs[e]);
#pragma unroll
        for (int j = 0; j < NTK; ++j) acc[j][e] = fmaf(vv[j][k], bf, acc[j][e]);
      }
    }
  }
#pragma unroll
  for (int j = 0; j < NTK; ++j)
#pragma unroll
    for (int e = 0; e < EPL; ++e) red[wave][j][e][lane] = acc[j][e];
  __syncthreads();
  if (wave < n_tok && cvalid) {
    float d[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e)
      d[e] = (red[0][wave][e][lane] + red[1][wave][e][lane]) + (red[2][wave][e][lane] + red[3][wave][e][lane]);
    ST ys[EPL];
    if (a.base32[p]) {                               // unrounded base from the dense projection
      const float* bp = a.base32[p] + (int64_t)tw * pr.d_out + col0;
#pragma unroll
      for (int e = 0; e < EPL; ++e) ys[e] = S::from_float(fmaf(sc, d[e], bp[e]));
    } else {
      __builtin_memcpy(ys, &yraw, 16);
#pragma unroll
      for (int e = 0; e < EPL; ++e) ys[e] = S::from_float(fmaf(sc, d[e], S::to_float(ys[e])));
    }
    u32x4 raw;
    __builtin_memcpy(&raw, ys, 16);
    *reinterpret_cast<u32x4*>(yp) = raw;
  }
}

}  // namespace

flp_status flp_launch_lora_segment(int32_t T, const int32_t* token_adapter, int32_t n_adapters, int32_t* n_seg,
                                   int32_t* seg_adapter, int32_t* seg_start, int32_t* perm, int32_t tm,
                                   int32_t* tile_start, int32_t tg, int32_t* group_start, hipStream_t stream,
                                   int32_t* inv_perm, int32_t* vrow_base) {
  const size_t smem = ((size_t)(kSegWaves + 2) * (size_t)(n_adapters > 0 ? n_adapters : 1) + 4 * kSegWaves + 4) * 4;
  static std::atomic<bool> attr_set{false};   // pools on different threads share it
  if (!attr_set.load(std::memory_order_acquire)) {
    FLP_TRY_HIP(hipFuncSetAttribute((const void*)lora_segment_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    160 * 1024));
    attr_set.store(true, std::memory_order_release);
  }
  hipLaunchKernelGGL(lora_segment_kernel, dim3(1), dim3(1024), smem, stream, T, token_adapter, n_adapters, n_seg,
                     seg_adapter, seg_start, perm, tm, tile_start, tg, group_start, inv_perm, vrow_base);
  FLP_TRY_HIP(hipGetLastError());
  return FLP_OK;
}

flp_status flp_launch_lora_simple(int dtype, const FlpLoraArgs& a, hipStream_t stream) {
  if (a.T <= 0) return FLP_OK;
  const int epl = dtype == FLP_F32 ? 4 : 8;
  int max_dout = 0;
  for (int p = 0; p < a.n_proj; ++p) max_dout = a.proj[p].d_out > max_dout ? a.proj[p].d_out : max_dout;
  dim3 gs((unsigned)a.T, (unsigned)a.n_proj, (unsigned)((a.max_rank + 7) / 8));
  dim3 ge((unsigned)a.T, (unsigned)((max_dout + 64 * epl - 1) / (64 * epl)), (unsigned)a.n_proj);
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
