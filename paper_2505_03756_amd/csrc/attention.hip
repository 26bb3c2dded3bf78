// KV append and the row-streaming paged prefix attention kernel.
//
// What is computed (paper sections 2.1 and 4.2: a query reuses the KV of its matched
// prefix and attends over it together with the KV of its own new tokens; section 4.3: new
// KV stays in the pool): for new token j of sequence i (position p = prefix_len + j) and
// query head h, softmax over positions 0..p of sm_scale * q.K, times V, with K and V read
// through the sequence's block table.
//
// Block layout used here, bt = 16 or 32 positions per block: K of (kv head g, slot s, channel c) at
// ((g*bt + s)*D + c); V of the same at n_kv*bt*D + ((g*D + c)*bt + s).  V is stored transposed so that the 16
// positions of one channel are one contiguous run: a lane that owns a channel reads them
// with one or two 16-byte loads and accumulates P.V without any cross-lane traffic.
#include <hip/hip_runtime.h>

#include "flp_internal.h"
#include "flp_types.h"

namespace {

constexpr int BT = 16;   // token positions per group: a block holds one (block size 16) or two (32) groups

// ------------------------------------------------------------------------------- append
// One workgroup per (sequence, block, 256 vector-columns) unit.  A thread owns 16 bytes of a
// token row (8 channels of one head, or 4 for fp32): it copies them into the K rows of the
// unit's slots and, for V, gathers the unit's slots into registers and turns them into the
// 16-slot runs of its channels.  A thread's runs are 256 contiguous bytes of the block and the
// workgroup's 64 KiB, so the runs pass through LDS once and leave as 1 KiB-contiguous
// non-temporal stores (whole lines) instead of 16-byte pieces 256 bytes apart.  A unit that
// covers only part of its block (the first and the last block of a sequence's new tokens)
// merges its slots into the runs already there: a partly filled block belongs to one sequence,
// and this workgroup is the only writer of these columns of it.
template <typename S, int D>
__global__ __launch_bounds__(256, 2) void kv_append_kernel(FlpAttnArgs a, const FlpAppendUnit* __restrict__ units) {
  constexpr int EPV = 16 / (int)sizeof(S);          // elements per 16-byte vector
  constexpr int VPR = BT / EPV;                     // vectors per 16-slot V run
  constexpr int UPT = EPV * VPR;                    // 16-byte pieces of V a thread produces (16)
  static_assert(UPT == 16, "a thread's V runs are 256 bytes");
  __shared__ u32x4 tr[256 * UPT];                   // 64 KiB: [thread][piece], pieces swizzled by thread
  const FlpAppendUnit u = units[blockIdx.x];
  const int row = a.n_kv * D;                       // elements per token in k_new / v_new
  const int tid = threadIdx.x;
  const int e0 = (blockIdx.y * 256 + tid) * EPV;
  const bool valid = e0 < row;
  const int ns = u.s1 - u.s0;
  const bool full = ns == BT;
  const int bt = a.bt, hpb = bt / BT, half = u.blk_idx % hpb;       // the unit is group `half` of its block
  const int64_t blk = a.tables[(int64_t)u.seq * a.max_blocks + u.blk_idx / hpb];
  S* __restrict__ base = reinterpret_cast<S*>(a.pool) + blk * a.block_elems;
  // 16-byte piece p = 16 t + VPR c + v of the unit's V: thread t (of this grid row), its channel c, vector v of
  // the channel's 16-slot run.  With 16-position blocks the 4096 pieces are 64 KiB contiguous (thread t owns
  // bytes 256 t ...); with 32-position blocks a run is one half of a 32-slot row.
  S* __restrict__ vbase = base + (int64_t)a.n_kv * bt * D + (int64_t)blockIdx.y * 256 * EPV * bt + BT * half;
  auto vpiece = [&](int piece) {
    return reinterpret_cast<u32x4*>(vbase + (int64_t)(piece / VPR) * bt + (piece % VPR) * EPV);
  };
  if (valid) {
    const S* __restrict__ kn = reinterpret_cast<const S*>(a.k_new) + (int64_t)u.t_first * row + e0;
    const S* __restrict__ vn = reinterpret_cast<const S*>(a.v_new) + (int64_t)u.t_first * row + e0;
    const int g = e0 / D, c0 = e0 - g * D;
    S* __restrict__ kdst = base + ((int64_t)g * bt + BT * half + u.s0) * D + c0;
    u32x4 vv[BT];
    if (full) {
#pragma unroll
      for (int s = 0; s < BT; ++s) vv[s] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vn + (int64_t)s * row));
#pragma unroll
      for (int h = 0; h < 2; ++h) {                 // K in two halves to keep the register count down
        u32x4 kv[BT / 2];
#pragma unroll
        for (int s = 0; s < BT / 2; ++s)
          kv[s] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kn + (int64_t)(h * (BT / 2) + s) * row));
#pragma unroll
        for (int s = 0; s < BT / 2; ++s)
          __builtin_nontemporal_store(kv[s], reinterpret_cast<u32x4*>(kdst + (h * (BT / 2) + s) * D));
      }
    } else {
      // slot s of the block holds row s - s0 of the unit; slots outside the unit read row 0 and are masked out below
#pragma unroll
      for (int s = 0; s < BT; ++s) {
        const int r_ = (s >= u.s0 && s < u.s1) ? s - u.s0 : 0;
        vv[s] = *reinterpret_cast<const u32x4*>(vn + (int64_t)r_ * row);
      }
      for (int s = 0; s < ns; ++s)
        *reinterpret_cast<u32x4*>(kdst + s * D) = *reinterpret_cast<const u32x4*>(kn + (int64_t)s * row);
    }
    S vals[BT][EPV];
    __builtin_memcpy(vals, vv, sizeof(vals));
#pragma unroll
    for (int c = 0; c < EPV; ++c) {
      S run[BT];
#pragma unroll
      for (int s = 0; s < BT; ++s) run[s] = vals[s][c];
      u32x4 packed[VPR];
      __builtin_memcpy(packed, run, sizeof(run));
      if (!full) {
        // the slots outside the unit keep what the block holds: word w of a run covers slots
        // [w * SPW, (w + 1) * SPW), merged under a bit mask that is the same for every thread
        constexpr int SPW = 4 / (int)sizeof(S);
#pragma unroll
        for (int v = 0; v < VPR; ++v) {
          const u32x4 old = *vpiece(tid * UPT + c * VPR + v);
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            uint32_t mask = 0;
#pragma unroll
            for (int e = 0; e < SPW; ++e) {
              const int sl = (4 * v + w) * SPW + e;
              if (sl >= u.s0 && sl < u.s1) mask |= (SPW == 1 ? 0xffffffffu : 0xffffu << (16 * e));
            }
            packed[v][w] = (packed[v][w] & mask) | (old[w] & ~mask);
          }
        }
      }
#pragma unroll
      for (int v = 0; v < VPR; ++v) tr[tid * UPT + ((c * VPR + v) ^ (tid & 15))] = packed[v];
    }
  }
  __syncthreads();
  // store j of a thread writes piece (256 j + tid), which thread (16 j + tid / 16) produced
#pragma unroll
  for (int j = 0; j < UPT; ++j) {
    const int owner = 16 * j + (tid >> 4), piece = tid & 15;
    if ((blockIdx.y * 256 + owner) * EPV < row) {
      const u32x4 val = tr[owner * UPT + (piece ^ (owner & 15))];
      if (hpb == 1)
        __builtin_nontemporal_store(val, vpiece(256 * j + tid));   // whole lines: streaming stores pay
      else
        *vpiece(256 * j + tid) = val;                              // half lines of 32-slot rows: plain stores
    }
  }
}

// --------------------------------------------------------------------- row-streaming attention
// One wave per (token, query head) row; a workgroup is four heads of one unit's tokens.
// Per block of 16 positions: K rows are read 16 bytes per lane (LPK lanes cover one key),
// scores are reduced inside each LPK-lane group, the online-softmax statistics are kept
// wave-uniform, and each lane accumulates its D/64 channels from the transposed V rows.
// HBM-bound for decode (one row per sequence and head); also the generic path for fp32.
template <typename S, int D>
struct RowCfg {
  static constexpr int EPL = 16 / (int)sizeof(typename S::storage);   // elements per 16-byte load
  static constexpr int LPK = D / EPL;                                 // lanes per key row
  static constexpr int KPL = 64 / LPK;                                // keys per wave-wide load
  static constexpr int NLD = BT / KPL;                                // loads per 16-key block
  static constexpr int CPL = D / 64;                                  // channels per lane
  static constexpr int VLD = BT * (int)sizeof(typename S::storage) / 16;   // 16-byte loads per V row
};

template <typename S, int D>
__global__ __launch_bounds__(256) void attn_rows_kernel(FlpAttnArgs a, const FlpAttnUnit* __restrict__ units) {
  typedef typename S::storage ST;
  typedef RowCfg<S, D> C;
  const FlpAttnUnit u = units[blockIdx.x];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int h = blockIdx.y * 4 + wave;
  if (h >= a.n_h) return;
  const int g = h / (a.n_h / a.n_kv);
  const int P = a.prefix_len[u.seq];
  const int t0 = a.cu_new[u.seq];
  const int32_t* __restrict__ table = a.tables + (int64_t)u.seq * a.max_blocks;
  const ST* __restrict__ pool = reinterpret_cast<const ST*>(a.pool);
  const int ck = lane % C::LPK;     // which 16-byte chunk of a key row this lane reads
  const int kg = lane / C::LPK;     // which key of a wave-wide load this lane works on
  const int bt = a.bt, hpb = bt / BT;
  const int64_t v_region = (int64_t)a.n_kv * bt * D;

  for (int jj = 0; jj < u.n_tok; ++jj) {
    const int j = u.j0 + jj;
    const int t = t0 + j;
    const int ctx = P + j + 1;      // positions 0..P+j are visible
    float qf[C::EPL];
    {
      const ST* qp = reinterpret_cast<const ST*>(a.q) + ((int64_t)t * a.n_h + h) * D + ck * C::EPL;
      u32x4 raw = *reinterpret_cast<const u32x4*>(qp);
      ST tmp[C::EPL];
      __builtin_memcpy(tmp, &raw, 16);
#pragma unroll
      for (int e = 0; e < C::EPL; ++e) qf[e] = S::to_float(tmp[e]) * a.scale_log2e;
    }
    float m = -INFINITY, l = 0.f;
    float acc[C::CPL];
#pragma unroll
    for (int c = 0; c < C::CPL; ++c) acc[c] = 0.f;

    const int nblk = (ctx + BT - 1) / BT;
    const bool split = u.n_split > 1;                   // this unit covers only the groups [g_lo, g_hi) of the context
    const int b_lo = split ? u.g_lo : 0, b_hi = split ? (u.g_hi < nblk ? u.g_hi : nblk) : nblk;
    for (int b = b_lo; b < b_hi; ++b) {
      // group b of 16 positions: group b % hpb of block b / hpb
      const ST* __restrict__ base = pool + (int64_t)table[b / hpb] * a.block_elems + BT * (b % hpb) * D;
      const ST* __restrict__ vbase = pool + (int64_t)table[b / hpb] * a.block_elems + v_region + BT * (b % hpb);
      // ---- scores of the group's 16 keys
      float s[C::NLD];
#pragma unroll
      for (int i = 0; i < C::NLD; ++i) {
        const int key = i * C::KPL + kg;
        u32x4 raw = *reinterpret_cast<const u32x4*>(base + ((int64_t)g * bt + key) * D + ck * C::EPL);
        ST tmp[C::EPL];
        __builtin_memcpy(tmp, &raw, 16);
        float d = 0.f;
#pragma unroll
        for (int e = 0; e < C::EPL; ++e) d = fmaf(qf[e], S::to_float(tmp[e]), d);
#pragma unroll
        for (int off = 1; off < C::LPK; off <<= 1) d += __shfl_xor(d, off);
        s[i] = (b * BT + key < ctx) ? d : -INFINITY;
      }
      float bm = s[0];
#pragma unroll
      for (int i = 1; i < C::NLD; ++i) bm = fmaxf(bm, s[i]);
#pragma unroll
      for (int off = C::LPK; off < 64; off <<= 1) bm = fmaxf(bm, __shfl_xor(bm, off));
      const float m_new = fmaxf(m, bm);          // finite: the block holds at least one visible key
      const float alpha = exp2f(m - m_new);      // 0 on the first block (m = -inf)
      float psum = 0.f;
#pragma unroll
      for (int i = 0; i < C::NLD; ++i) {
        s[i] = exp2f(s[i] - m_new);              // masked keys: exp2(-inf) = 0
        psum += s[i];
      }
#pragma unroll
      for (int off = C::LPK; off < 64; off <<= 1) psum += __shfl_xor(psum, off);
      l = l * alpha + psum;
      m = m_new;
      // ---- weights of the 16 keys, wave-uniform
      float w[BT];
#pragma unroll
      for (int k = 0; k < BT; ++k)
        w[k] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(s[k / C::KPL]), (k % C::KPL) * C::LPK));
      // ---- P.V: this lane's channels, 16 positions each
#pragma unroll
      for (int c = 0; c < C::CPL; ++c) {
        const ST* vp = vbase + ((int64_t)g * D + (lane + 64 * c)) * bt;
        ST vv[BT];
        u32x4 raw[C::VLD];
#pragma unroll
        for (int v = 0; v < C::VLD; ++v) raw[v] = reinterpret_cast<const u32x4*>(vp)[v];
        __builtin_memcpy(vv, raw, sizeof(vv));
        float part = 0.f;
#pragma unroll
        for (int k = 0; k < BT; ++k) {
          // slots past the sequence's length hold arbitrary bits: select, never multiply
          float x = (b * BT + k < ctx) ? S::to_float(vv[k]) : 0.f;
          part = fmaf(w[k], x, part);
        }
        acc[c] = acc[c] * alpha + part;
      }
    }
    if (split) {
      // unnormalised piece: running maximum (in the exponent's units), sum of weights, channels
      float* pp = a.partials + (((int64_t)u.part_row * a.n_h + h) * a.max_split + u.split) * (D + 2);
      if (lane == 0) {
        pp[0] = m;
        pp[1] = l;
      }
#pragma unroll
      for (int c = 0; c < C::CPL; ++c) pp[2 + lane + 64 * c] = acc[c];
      continue;
    }
    const float inv = 1.f / l;
    ST* op = reinterpret_cast<ST*>(a.out) + ((int64_t)t * a.n_h + h) * D;
#pragma unroll
    for (int c = 0; c < C::CPL; ++c) op[lane + 64 * c] = S::from_float(acc[c] * inv);
  }
}

// Merge of the split-KV pieces of one (token, head) row: out = sum_i acc_i 2^(m_i - M) / sum_i l_i 2^(m_i - M)
// with M = max_i m_i, the pieces taken in piece order.  One wave per row, four heads per workgroup.
template <typename S, int D>
__global__ __launch_bounds__(256) void attn_merge_kernel(FlpAttnArgs a, const int32_t* __restrict__ merge_tok,
                                                         const int32_t* __restrict__ merge_nsplit) {
  typedef typename S::storage ST;
  constexpr int CPL = D / 64;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int row = blockIdx.x, h = blockIdx.y * 4 + wave;
  if (h >= a.n_h) return;
  const int t = merge_tok[row], ns = merge_nsplit[row];
  const float* pp = a.partials + ((int64_t)row * a.n_h + h) * a.max_split * (D + 2);
  float M = -INFINITY;
  for (int i = 0; i < ns; ++i) M = fmaxf(M, pp[(int64_t)i * (D + 2)]);
  float l = 0.f, acc[CPL];
#pragma unroll
  for (int c = 0; c < CPL; ++c) acc[c] = 0.f;
  for (int i = 0; i < ns; ++i) {
    const float* q = pp + (int64_t)i * (D + 2);
    const float w = exp2f(q[0] - M);                    // a piece without visible keys has m = -inf, l = 0: weight 0
    l = fmaf(q[1], w, l);
#pragma unroll
    for (int c = 0; c < CPL; ++c) acc[c] = fmaf(q[2 + lane + 64 * c], w, acc[c]);
  }
  const float inv = 1.f / l;
  ST* op = reinterpret_cast<ST*>(a.out) + ((int64_t)t * a.n_h + h) * D;
#pragma unroll
  for (int c = 0; c < CPL; ++c) op[lane + 64 * c] = S::from_float(acc[c] * inv);
}

}  // namespace

#define FLP_DISPATCH(KERNEL, dtype, head_dim, grid, block, stream, ...)                                      \
  do {                                                                                                       \
    if (dtype == FLP_F32 && head_dim == 64)                                                                  \
      hipLaunchKernelGGL((KERNEL<F32, 64>), grid, block, 0, stream, __VA_ARGS__);                            \
    else if (dtype == FLP_F32 && head_dim == 128)                                                            \
      hipLaunchKernelGGL((KERNEL<F32, 128>), grid, block, 0, stream, __VA_ARGS__);                           \
    else if (dtype == FLP_F16 && head_dim == 64)                                                             \
      hipLaunchKernelGGL((KERNEL<F16, 64>), grid, block, 0, stream, __VA_ARGS__);                            \
    else if (dtype == FLP_F16 && head_dim == 128)                                                            \
      hipLaunchKernelGGL((KERNEL<F16, 128>), grid, block, 0, stream, __VA_ARGS__);                           \
    else if (dtype == FLP_BF16 && head_dim == 64)                                                            \
      hipLaunchKernelGGL((KERNEL<BF16, 64>), grid, block, 0, stream, __VA_ARGS__);                           \
    else if (dtype == FLP_BF16 && head_dim == 128)                                                           \
      hipLaunchKernelGGL((KERNEL<BF16, 128>), grid, block, 0, stream, __VA_ARGS__);                          \
    else {                                                                                                   \
      flp_set_error("attention: dtype %d / head_dim %d not supported", dtype, head_dim);                     \
      return FLP_ENOTSUP;                                                                                    \
    }                                                                                                        \
  } while (0)

flp_status flp_launch_kv_append(int dtype, int head_dim, const FlpAttnArgs& a, const FlpAppendUnit* units_dev,
                                int32_t n_units, hipStream_t stream) {
  if (n_units <= 0) return FLP_OK;
  // the append kernel only moves storage words: fp16 and bf16 share the 16-bit instance
  const int epv = dtype == FLP_F32 ? 4 : 8;
  dim3 grid((unsigned)n_units, (unsigned)((a.n_kv * head_dim + 256 * epv - 1) / (256 * epv)));
  if (dtype == FLP_F32 && head_dim == 64)
    hipLaunchKernelGGL((kv_append_kernel<float, 64>), grid, dim3(256), 0, stream, a, units_dev);
  else if (dtype == FLP_F32 && head_dim == 128)
    hipLaunchKernelGGL((kv_append_kernel<float, 128>), grid, dim3(256), 0, stream, a, units_dev);
  else if (dtype != FLP_F32 && head_dim == 64)
    hipLaunchKernelGGL((kv_append_kernel<uint16_t, 64>), grid, dim3(256), 0, stream, a, units_dev);
  else if (dtype != FLP_F32 && head_dim == 128)
    hipLaunchKernelGGL((kv_append_kernel<uint16_t, 128>), grid, dim3(256), 0, stream, a, units_dev);
  else {
    flp_set_error("kv_append: head_dim %d not supported", head_dim);
    return FLP_ENOTSUP;
  }
  FLP_TRY_HIP(hipGetLastError());
  return FLP_OK;
}

flp_status flp_launch_attn_rows(int dtype, int head_dim, const FlpAttnArgs& a, const FlpAttnUnit* units_dev,
                                int32_t n_units, hipStream_t stream) {
  if (n_units <= 0) return FLP_OK;
  dim3 grid((unsigned)n_units, (unsigned)((a.n_h + 3) / 4));
  FLP_DISPATCH(attn_rows_kernel, dtype, head_dim, grid, dim3(256), stream, a, units_dev);
  FLP_TRY_HIP(hipGetLastError());
  return FLP_OK;
}

flp_status flp_launch_attn_merge(int dtype, int head_dim, const FlpAttnArgs& a, const int32_t* merge_tok_dev,
                                 const int32_t* merge_nsplit_dev, int32_t n_rows, hipStream_t stream) {
  if (n_rows <= 0) return FLP_OK;
  dim3 grid((unsigned)n_rows, (unsigned)((a.n_h + 3) / 4));
  FLP_DISPATCH(attn_merge_kernel, dtype, head_dim, grid, dim3(256), stream, a, merge_tok_dev, merge_nsplit_dev);
  FLP_TRY_HIP(hipGetLastError());
  return FLP_OK;
}
