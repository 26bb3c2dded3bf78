// Paged prefix attention on the matrix cores, for 16-bit pools with head_dim 128.
//
// Same definition as the row-streaming kernel (paper sections 2.1 / 4.2: the new tokens of
// a query attend over the reused prefix KV and their own fresh KV, read through the block
// table), organised as a tiled online-softmax so that K and V are read once per tile of
// query rows instead of once per row.
//
// One workgroup (8 waves, one per CU) owns up to 256 query rows of one (sequence, kv head); row r
// is (new token r / G, query head g*G + r % G), so the G query heads that share a kv head
// sit in the same tile and K/V are read once for all of them.  It walks the context in
// tiles of 64 positions (4 pool blocks).
//
// The products are computed transposed, S^T = K Q^T and O^T = V^T P^T, with
// mfma_f32_32x32x16: the accumulator layout then gives every lane ONE query row (column
// l%32) and 16 keys of a 32-key sub-tile, so the softmax statistics are per-lane scalars
// and P^T is already in B-operand layout for the second product.  The A operand of that
// product needs, per lane, 8 consecutive positions of one channel: exactly what the
// transposed V layout of the pool block provides as one 16-byte run.  The order in which
// keys are fed to the first product is permuted (bits 2 and 3 of the key index swapped)
// so that the 8 keys a lane ends up holding are consecutive positions.
//
// K/V tiles travel from the pool to LDS with the direct global-to-LDS loads of gfx950
// (16 bytes per lane, landing at LDS base + 16 * lane): no registers and no LDS stores are
// spent on staging, and a ring of three tiles keeps two tiles in flight behind the one being
// multiplied.  The XOR swizzle of the LDS layout is applied on the global side: a lane
// fetches the 16-byte chunk that belongs at its fixed LDS slot.  A wave issues one
// instruction about every 4.5 cycles whatever its kind, and LDS reads take a few hundred
// cycles under load, so the loops below keep the instruction count per tile low and read the
// operand fragments two steps ahead of the products that use them.
#include <hip/hip_runtime.h>

#include "flp_internal.h"
#include "flp_types.h"

namespace {

constexpr int D = 128;
constexpr int BT = 16;
constexpr int BN = 64;                 // keys per tile
constexpr int kTile = BN * D * 2;      // bytes of one K (or V) tile: 16 KiB
constexpr int kStage = 2 * kTile;      // K tile followed by V tile
constexpr int kStages = 3;         // tiles in the LDS ring: one being multiplied, kStages - 1 in flight

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 h16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 b16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 h16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 b16x2 __attribute__((ext_vector_type(2)));

struct MF16 {
  typedef h16x8 vec;
  static __device__ __forceinline__ f32x16 mfma(vec a, vec b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
  }
  // 8 weights -> 16 bit; returns their sum as seen after rounding
  static __device__ __forceinline__ vec pack(const float* p, float& sum) {
    vec v;
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = (_Float16)p[j];
    const h16x2 one = {(_Float16)1.f, (_Float16)1.f};
#pragma unroll
    for (int j = 0; j < 4; ++j) sum = __builtin_amdgcn_fdot2(h16x2{v[2 * j], v[2 * j + 1]}, one, sum, false);
    return v;
  }
  static __device__ __forceinline__ uint16_t out(float f) { return F16::from_float(f); }
};
struct MBF16 {
  typedef b16x8 vec;
  static __device__ __forceinline__ f32x16 mfma(vec a, vec b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ vec pack(const float* p, float& sum) {
    vec v;
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = (__bf16)p[j];
    const b16x2 one = {(__bf16)1.f, (__bf16)1.f};
#pragma unroll
    for (int j = 0; j < 4; ++j) sum = __builtin_amdgcn_fdot2_f32_bf16(b16x2{v[2 * j], v[2 * j + 1]}, one, sum, false);
    return v;
  }
  static __device__ __forceinline__ uint16_t out(float f) { return BF16::from_float(f); }
};

template <typename V>
__device__ __forceinline__ V as_vec(u32x4 r) {
  V v;
  __builtin_memcpy(&v, &r, 16);
  return v;
}

// m (row of the first product's A operand) -> position inside the 32-key sub-tile
__device__ __forceinline__ int key_of_row(int m) { return (m & 0x13) | ((m & 4) << 1) | ((m & 8) >> 1); }
// XOR term of the K row swizzle (= row of the A operand & 15) and of the V^T run swizzle
__device__ __forceinline__ int k_swz(int key) { return ((key & 4) << 1) | ((key & 8) >> 1) | (key & 3); }
__device__ __forceinline__ int v_swz(int d) { return ((d >> 2) & 1) ^ ((d >> 3) & 1); }

// s_waitcnt immediates (gfx9 encoding: vmcnt[3:0] + [15:14], expcnt[6:4], lgkmcnt[11:8]), other counters untouched
constexpr int kWaitTile = (4 * (kStages - 2)) | (7 << 4) | (15 << 8);   // all but the newest kStages - 2 tiles (4 loads each) have landed
constexpr int kWaitVm0 = 0 | (7 << 4) | (15 << 8);

// One direct global-to-LDS load: every lane fetches 16 bytes from base + voff and the wave's 64
// pieces land at LDS byte address lds .. lds + 1023 in lane order (base and lds wave-uniform).
// Written as inline assembly on purpose: the compiler does not see these loads, so it neither
// counts them in its own memory-counter waits nor makes every later LDS read wait for all of
// them; the kernel orders them against the LDS reads itself (s_waitcnt vmcnt + barrier).
// M0 is named as clobbered so that no pass keeps a value of its own alive in it across the statement; the
// compiler notes that it reserves the register, which is the point.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void load_to_lds16(const void* base, uint32_t voff, uint32_t lds) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(base), "s"(lds)
               : "memory", "m0");
}
#pragma clang diagnostic pop
typedef __attribute__((address_space(3))) uint8_t lds_u8;
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

template <typename M>
__global__ __launch_bounds__(512, 2) void attn_mfma_kernel(FlpAttnArgs a, const FlpMfmaItem* __restrict__ items) {
  typedef typename M::vec vec;
  __shared__ __attribute__((aligned(16))) uint8_t smem[kStages * kStage];
  __shared__ int32_t tab_lds[kMfmaMaxBlocks];          // this sequence's block table

  const FlpMfmaItem it = items[blockIdx.x];
  if (it.n_rows <= 0) return;
  const int tid = threadIdx.x, lane = tid & 63, lr = lane & 31, hf = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int G = a.n_h / a.n_kv, g = it.g;
  const int P = a.prefix_len[it.seq];
  const int t0 = a.cu_new[it.seq];
  const int N = a.cu_new[it.seq + 1] - t0;
  const int L = P + N;
  const int bt = a.bt, hpb = bt / BT;                 // a block holds one or two groups of 16 positions
  const int ngrp_valid = (L + BT - 1) / BT;           // groups of 16 positions that hold keys of this sequence
  const int nblk_valid = (L + bt - 1) / bt;
  const int32_t* __restrict__ table = a.tables + (int64_t)it.seq * a.max_blocks;
  const uint16_t* __restrict__ pool = reinterpret_cast<const uint16_t*>(a.pool);
  const float c = a.scale_log2e;

  // ---- this wave's 32 query rows
  const int row_end = it.r0 + it.n_rows;             // one past the tile's last valid row
  const int wrow0 = it.r0 + wave * 32;
  const bool wave_active = wrow0 < row_end;
  const int wrow_last = (wrow0 + 31 < row_end - 1) ? wrow0 + 31 : row_end - 1;
  const int wave_min_pos = P + wrow0 / G;
  const int n_tiles = (P + (row_end - 1) / G) / BN + 1;
  const int kt_last = wave_active ? (P + wrow_last / G) / BN : -1;   // last tile this wave has keys in

  const int row = wrow0 + lr;
  const bool rvalid = row < row_end;
  const int rc = rvalid ? row : row_end - 1;
  const int prow = P + rc / G;                        // position of this lane's row
  const int64_t rowoff = ((int64_t)(t0 + rc / G) * a.n_h + (g * G + rc % G)) * D;
  vec qf[8];
  {
    const uint16_t* qp = reinterpret_cast<const uint16_t*>(a.q) + rowoff + 8 * hf;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) qf[kk] = as_vec<vec>(*reinterpret_cast<const u32x4*>(qp + 16 * kk));
  }

  f32x16 O[4];
  float mrow = -INFINITY, lsum = 0.f;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int i = 0; i < 16; ++i) O[dt][i] = 0.f;

  // ---- staging: wave w moves pool block w/2 of every tile, quarters 2(w%2) and 2(w%2)+1 of its K rows
  //      and of its V^T runs (1 KiB per instruction).  LDS chunk ci (16 bytes) of a block's K part
  //      holds key ci/16, logical chunk (ci%16) ^ swizzle(key); chunk ci of its V part holds channel
  //      ci/2, positions 8*((ci%2) ^ swizzle(channel)) .. +7.
  const int sblk = wave >> 1;
  uint32_t kg[2], vg[2];                             // this lane's byte offsets inside a block
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int ci = (2 * (wave & 1) + j) * 64 + lane;
    const int key = ci >> 4;
    kg[j] = (uint32_t)(2 * (key * D + 8 * ((ci & 15) ^ k_swz(key))));
    const int vd = ci >> 1;
    vg[j] = (uint32_t)(2 * (vd * bt + 8 * ((ci & 1) ^ v_swz(vd))));     // channel vd's run of 16 slots inside its bt-slot row
  }
  const int64_t k_region = (int64_t)g * bt * D;
  const int64_t v_region = (int64_t)a.n_kv * bt * D + (int64_t)g * D * bt;
  const uint32_t lds_wave = (uint32_t)(uintptr_t)(lds_u8*)smem + sblk * 4096 + 2 * (wave & 1) * 1024;   // LDS address of this wave's first quarter in stage 0

  for (int i = tid; i < nblk_valid; i += 512) tab_lds[i] = table[i];
  __builtin_amdgcn_s_waitcnt(kWaitVm0);                // the query fragments are in: from here on only tile loads are in flight
  __syncthreads();
  // this wave's 16-position group of tile t (clamped: always valid), as block id * 2 + group inside the block
  auto block_id = [&](int t) {
    int gi = 4 * t + sblk;
    gi = gi < ngrp_valid ? gi : ngrp_valid - 1;
    return __builtin_amdgcn_readfirstlane(tab_lds[gi / hpb] * 2 + gi % hpb);
  };
  auto issue_tile = [&](int t, int32_t id) {         // 4 direct loads: tile t -> stage t % kStages
    const int half = id & 1;
    const uint16_t* blk = pool + (int64_t)(id >> 1) * a.block_elems;
    const uint32_t dst = lds_wave + (t % kStages) * kStage;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      load_to_lds16(blk + k_region + BT * half * D, kg[j], dst + j * 1024);
      load_to_lds16(blk + v_region + BT * half, vg[j], dst + kTile + j * 1024);
    }
  };

#pragma unroll
  for (int t = 0; t < kStages - 1; ++t) issue_tile(t, block_id(t));
  int32_t id_next = block_id(kStages - 1);

  const int krow = key_of_row(lr);                    // this lane's key inside a 32-key sub-tile
  const int a_swz = lr & 15;
  int voff[4];                                        // V^T fragment of channel tile dt (block b adds b * 4096)
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) {
    const int d = 32 * dt + lr;
    voff[dt] = kTile + ((2 * d + (hf ^ v_swz(d))) << 4);
  }

  for (int kt = 0; kt < n_tiles; ++kt) {
    // tile kt has landed (this wave's part: all but the 4 loads of tile kt + 1 are complete), and after
    // the barrier so has everybody's; everybody is also done with tile kt - 1, whose stage is refilled next
    __builtin_amdgcn_s_waitcnt(kWaitTile);
    __syncthreads();
    uint8_t* buf = smem + (kt % kStages) * kStage;
    if (BN * kt + BN > L) {
      // slots at or past the sequence's length hold arbitrary bits: zero them so that a zero weight
      // times such a value cannot turn into NaN (only the last tile of a sequence gets here)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int ci = tid + 512 * j;
        const int u = ci >> 8, vd = (ci & 255) >> 1, vh = (ci & 1) ^ v_swz(vd);
        const int pos0 = BN * kt + BT * u + 8 * vh;
        if (pos0 + 8 > L) {
          u32x4* slot = reinterpret_cast<u32x4*>(buf + kTile + ci * 16);
          u32x4 v = *slot;
          uint16_t e[8];
          __builtin_memcpy(e, &v, 16);
#pragma unroll
          for (int s = 0; s < 8; ++s)
            if (pos0 + s >= L) e[s] = 0;
          __builtin_memcpy(&v, e, 16);
          *slot = v;
        }
      }
      __syncthreads();
    }
    issue_tile(kt + kStages - 1, id_next);
    id_next = block_id(kt + kStages);

    if (kt <= kt_last) {
      // ---- S^T = K Q^T for the tile's two 32-key sub-tiles; K fragments are read two steps ahead
      f32x16 S[2];
#pragma unroll
      for (int i = 0; i < 16; ++i) S[0][i] = S[1][i] = 0.f;
      const uint8_t* krowp = buf + krow * 256;
      vec kf[3][2];
      auto load_k = [&](int kk) {
        const int coff = ((2 * kk + hf) ^ a_swz) << 4;
        kf[kk % 3][0] = as_vec<vec>(*reinterpret_cast<const u32x4*>(krowp + coff));
        kf[kk % 3][1] = as_vec<vec>(*reinterpret_cast<const u32x4*>(krowp + 32 * 256 + coff));
      };
      load_k(0);
      load_k(1);
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        if (kk + 2 < 8) load_k(kk + 2);
        S[0] = M::mfma(kf[kk % 3][0], qf[kk], S[0]);
        S[1] = M::mfma(kf[kk % 3][1], qf[kk], S[1]);
      }
      __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
      for (int kk = 0; kk < 6; ++kk) {
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
      __builtin_amdgcn_sched_barrier(0);
      // ---- first V^T fragments: on their way while the weights are computed
      vec vf[3][2];
      auto load_v = [&](int s) {                       // step s: block s/2, channel tiles 2(s%2), 2(s%2)+1
        const int b = s >> 1, d0 = 2 * (s & 1);
        vf[s % 3][0] = as_vec<vec>(*reinterpret_cast<const u32x4*>(buf + b * 4096 + voff[d0]));
        vf[s % 3][1] = as_vec<vec>(*reinterpret_cast<const u32x4*>(buf + b * 4096 + voff[d0 + 1]));
      };
      load_v(0);
      load_v(1);
      __builtin_amdgcn_sched_barrier(0);
      // ---- causal mask on the tiles that reach past the first row's position
      if (BN * kt + BN - 1 > wave_min_pos) {
#pragma unroll
        for (int st = 0; st < 2; ++st) {
          const int thr = prow - (BN * kt + 32 * st + 8 * hf);
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int off = 16 * (i / 8) + 4 * ((i / 4) % 2) + (i % 4);
            S[st][i] = off <= thr ? S[st][i] : -INFINITY;
          }
        }
      }
      // ---- online softmax, one row per lane (both lane halves hold the same row)
      float tmax = S[0][0];
#pragma unroll
      for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int i = 0; i < 16; ++i) tmax = fmaxf(tmax, S[st][i]);
      {
        // exchange between the lane halves: after the swap one register holds the lower half's value
        // in both halves, the other the upper half's
        const u32x2 sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(tmax), __float_as_uint(tmax), false, false);
        tmax = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
      }
      // The running maximum is only raised when some row of the wave has outgrown it by more
      // than 2^8: until then the weights are taken relative to the old maximum (they stay below
      // 256, exact in fp32 and well inside the 16-bit range), which spares the rescaling of the
      // 64 accumulator registers on almost every tile.
      if (__builtin_amdgcn_ballot_w64((tmax - mrow) * c > 8.f)) {
        const float m_new = fmaxf(mrow, tmax);
        const float alpha = __builtin_amdgcn_exp2f((mrow - m_new) * c);
        mrow = m_new;
        lsum *= alpha;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
          for (int i = 0; i < 16; ++i) O[dt][i] *= alpha;
      }
      const float mc = mrow * c;
      vec pb[2][2];
#pragma unroll
      for (int st = 0; st < 2; ++st) {
        float p[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) p[i] = __builtin_amdgcn_exp2f(fmaf(S[st][i], c, -mc));
        // the row sum is taken over the rounded weights, the ones the second product uses
        pb[st][0] = M::pack(p, lsum);
        pb[st][1] = M::pack(p + 8, lsum);
      }
      // ---- O^T += V^T P^T, one pool block (16 keys) per instruction, V^T fragments two steps ahead
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        if (s + 2 < 8) load_v(s + 2);
        const int b = s >> 1, d0 = 2 * (s & 1);
        O[d0] = M::mfma(vf[s % 3][0], pb[b >> 1][b & 1], O[d0]);
        O[d0 + 1] = M::mfma(vf[s % 3][1], pb[b >> 1][b & 1], O[d0 + 1]);
      }
    }
  }
  __builtin_amdgcn_s_waitcnt(kWaitVm0);                // the look-ahead loads past the last tile must land before the LDS is released

  // ---- normalise and store: lane (row, half) holds channels 32dt + 8q + 4hf + (0..3)
  if (wave_active) {
    const u32x2 sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(lsum), __float_as_uint(lsum), false, false);
    const float inv = 1.f / (__uint_as_float(sw[0]) + __uint_as_float(sw[1]));
    if (rvalid) {
      uint16_t* op = reinterpret_cast<uint16_t*>(a.out) + rowoff;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          uint16_t o4[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) o4[r] = M::out(O[dt][4 * q + r] * inv);
          uint2 w;
          __builtin_memcpy(&w, o4, 8);
          *reinterpret_cast<uint2*>(op + 32 * dt + 8 * q + 4 * hf) = w;
        }
    }
  }
}

}  // namespace

flp_status flp_launch_attn_mfma(int dtype, const FlpAttnArgs& a, const FlpMfmaItem* items_dev, int32_t n_items,
                                hipStream_t stream) {
  if (n_items <= 0) return FLP_OK;
  if (dtype == FLP_F16)
    hipLaunchKernelGGL((attn_mfma_kernel<MF16>), dim3(n_items), dim3(512), 0, stream, a, items_dev);
  else if (dtype == FLP_BF16)
    hipLaunchKernelGGL((attn_mfma_kernel<MBF16>), dim3(n_items), dim3(512), 0, stream, a, items_dev);
  else {
    flp_set_error("attention (matrix-core path): dtype %d not supported", dtype);
    return FLP_ENOTSUP;
  }
  FLP_TRY_HIP(hipGetLastError());
  return FLP_OK;
}
