// Paged prefix attention on the matrix cores, for 16-bit pools with head_dim 128.
//
// Same definition as the row-streaming kernel (paper sections 2.1 / 4.2: the new tokens of
// a query attend over the reused prefix KV and their own fresh KV, read through the block
// table), organised as a tiled online-softmax so that K and V are read once per tile of
// query rows instead of once per row.
//
// One workgroup (8 waves, one per CU) owns up to 8*32*NRT query rows of one (sequence, kv head); row r
// is (new token r / G, query head g*G + r % G), so the G query heads that share a kv head
// sit in the same tile and K/V are read once for all of them.  It walks the context in
// tiles of 64 positions (4 pool blocks), staged through LDS and double-buffered.
//
// The products are computed transposed, S^T = K Q^T and O^T = V^T P^T, with
// mfma_f32_32x32x16: the accumulator layout then gives every lane ONE query row (column
// l%32) and 16 keys of a 32-key sub-tile, so the softmax statistics are per-lane scalars
// and P^T is already in B-operand layout for the second product.  The A operand of that
// product needs, per lane, 8 consecutive positions of one channel: exactly what the
// transposed V layout of the pool block provides as one 16-byte run.  The order in which
// keys are fed to the first product is permuted (bits 2 and 3 of the key index swapped)
// so that the 8 keys a lane ends up holding are consecutive positions.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "flp_internal.h"
#include "flp_types.h"

namespace {

constexpr int D = 128;
constexpr int BT = 16;
constexpr int BN = 64;                 // keys per tile
constexpr int kKBytes = BN * D * 2;    // 16 KiB
constexpr int kTileBytes = 2 * kKBytes;

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 h16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 b16x8 __attribute__((ext_vector_type(8)));

struct MF16 {
  typedef h16x8 vec;
  static __device__ __forceinline__ f32x16 mfma(vec a, vec b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ vec pack(const float* p) {
    vec v;
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = (_Float16)p[j];
    return v;
  }
  static __device__ __forceinline__ uint16_t out(float f) { return F16::from_float(f); }
};
struct MBF16 {
  typedef b16x8 vec;
  static __device__ __forceinline__ f32x16 mfma(vec a, vec b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ vec pack(const float* p) {
    vec v;
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = (__bf16)p[j];
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

template <typename M, int NRT>
__global__ __launch_bounds__(NRT == 1 ? 512 : 256, NRT == 1 ? 2 : 1) void attn_mfma_kernel(FlpAttnArgs a, const FlpMfmaItem* __restrict__ items) {
  typedef typename M::vec vec;
  __shared__ __attribute__((aligned(16))) uint8_t smem[2 * kTileBytes];
  __shared__ int32_t tab_lds[kMfmaMaxBlocks];          // this sequence's block table

  const FlpMfmaItem it = items[blockIdx.x];
  if (it.n_rows <= 0) return;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lr = lane & 31, hf = lane >> 5;
  const int G = a.n_h / a.n_kv, g = it.g;
  const int P = a.prefix_len[it.seq];
  const int t0 = a.cu_new[it.seq];
  const int N = a.cu_new[it.seq + 1] - t0;
  const int L = P + N;
  const int nblk_valid = (L + BT - 1) / BT;
  const int32_t* __restrict__ table = a.tables + (int64_t)it.seq * a.max_blocks;
  const uint16_t* __restrict__ pool = reinterpret_cast<const uint16_t*>(a.pool);
  const int64_t v_region = (int64_t)a.n_kv * BT * D + (int64_t)g * D * BT;
  const float c = a.scale_log2e;

  // ---- this wave's query rows
  constexpr int RW = 32 * NRT;
  const int row_end = it.r0 + it.n_rows;             // one past the tile's last valid row
  const int wrow0 = it.r0 + wave * RW;
  const bool wave_active = wrow0 < row_end;
  const int wrow_last = (wrow0 + RW - 1 < row_end - 1) ? wrow0 + RW - 1 : row_end - 1;
  const int wave_max_pos = P + wrow_last / G;
  const int wave_min_pos = P + wrow0 / G;
  const int n_tiles = (P + (row_end - 1) / G) / BN + 1;

  int prow[NRT];                                      // position of this lane's row
  bool rvalid[NRT];
  int64_t rowoff[NRT];                                // element offset of the row in q / out
  vec qf[NRT][8];
#pragma unroll
  for (int nt = 0; nt < NRT; ++nt) {
    int row = wrow0 + 32 * nt + lr;
    rvalid[nt] = row < row_end;
    int rc = rvalid[nt] ? row : row_end - 1;
    int j = rc / G;
    prow[nt] = P + j;
    rowoff[nt] = ((int64_t)(t0 + j) * a.n_h + (g * G + rc % G)) * D;
    const uint16_t* qp = reinterpret_cast<const uint16_t*>(a.q) + rowoff[nt] + 8 * hf;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) qf[nt][kk] = as_vec<vec>(*reinterpret_cast<const u32x4*>(qp + 16 * kk));
  }

  f32x16 O[NRT][4];
  float mrow[NRT], lrow[NRT];
#pragma unroll
  for (int nt = 0; nt < NRT; ++nt) {
    mrow[nt] = -INFINITY;
    lrow[nt] = 0.f;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) O[nt][dt][i] = 0.f;
  }

  // ---- tile staging: the tile's 4 pool blocks are split over the two halves of the workgroup;
  //      a thread moves one K chunk and one V chunk (16 bytes each) of each of its 2 blocks
  constexpr int NTHR = NRT == 1 ? 512 : 256;          // 8 waves x 32 rows or 4 waves x 64 rows
  constexpr int BPT = 1024 / NTHR;                    // pool blocks of a tile staged per thread
  const int sthalf = __builtin_amdgcn_readfirstlane(tid >> 8);   // wave-uniform: table lookups stay scalar
  const int st8 = tid & 255;
  const int kkey = st8 >> 4, kchunk = st8 & 15;      // K: key inside the block, 16-byte chunk of its row
  const int vd = st8 >> 1, vhalf = st8 & 1;          // V: channel, which 8 of the 16 slots
  const int kswz = ((kkey & 4) << 1) | ((kkey & 8) >> 1) | (kkey & 3);   // = row of the A operand & 15
  const int k_lds = kkey * 256 + ((kchunk ^ kswz) << 4);
  const int v_lds = kKBytes + ((2 * vd + (vhalf ^ ((vd >> 2) & 1) ^ ((vd >> 3) & 1))) << 4);
  // two register sets: while tile kt is being multiplied, tile kt+1 waits in registers for its
  // LDS buffer and tile kt+2 is in flight from HBM/L2 (one tile of compute is shorter than the
  // memory latency, so a single tile of look-ahead leaves the loop latency-bound)
  u32x4 kreg[2][BPT], vreg[2][BPT];
  const uint32_t k_goff = (uint32_t)(kkey * D + 8 * kchunk), v_goff = (uint32_t)(8 * st8);   // per-lane element offsets

  // The sequence's block table is copied into LDS once; the per-tile lookups then cost an LDS
  // read instead of a scalar load from memory (whose latency every later LDS wait would inherit,
  // because scalar loads and LDS reads share one completion counter).
  for (int i = tid; i < nblk_valid; i += NTHR) tab_lds[i] = table[i];
  int32_t ids_next[BPT];
  auto fetch_ids = [&](int kt) {
#pragma unroll
    for (int uu = 0; uu < BPT; ++uu) {
      int bi = 4 * kt + BPT * sthalf + uu;
      bi = bi < nblk_valid ? bi : nblk_valid - 1;
      ids_next[uu] = __builtin_amdgcn_readfirstlane(tab_lds[bi]);
    }
  };
  auto load_tile = [&](int set) {                      // loads the tile whose ids are in ids_next
#pragma unroll
    for (int uu = 0; uu < BPT; ++uu) {
      const uint16_t* kbase = pool + (int64_t)ids_next[uu] * a.block_elems + (int64_t)g * BT * D;   // uniform
      const uint16_t* vbase = pool + (int64_t)ids_next[uu] * a.block_elems + v_region;               // uniform
      kreg[set][uu] = *reinterpret_cast<const u32x4*>(kbase + k_goff);
      vreg[set][uu] = *reinterpret_cast<const u32x4*>(vbase + v_goff);
    }
  };
  auto store_tile = [&](int kt, uint8_t* buf, int set) {
#pragma unroll
    for (int uu = 0; uu < BPT; ++uu) {
      const int u = BPT * sthalf + uu;
      *reinterpret_cast<u32x4*>(buf + u * 4096 + k_lds) = kreg[set][uu];
      // slots at or past the sequence's length hold arbitrary bits: zero them so that a
      // zero weight times such a value cannot turn into NaN
      const int pos0 = BN * kt + BT * u + 8 * vhalf;
      u32x4 v = vreg[set][uu];
      if (pos0 + 8 > L) {
        uint16_t e[8];
        __builtin_memcpy(e, &v, 16);
#pragma unroll
        for (int s = 0; s < 8; ++s)
          if (pos0 + s >= L) e[s] = 0;
        __builtin_memcpy(&v, e, 16);
      }
      *reinterpret_cast<u32x4*>(buf + u * 4096 + v_lds) = v;
    }
  };

  __syncthreads();
  fetch_ids(0);
  load_tile(0);
  fetch_ids(1);                                        // (clamped to the last valid block when there is no tile 1)
  store_tile(0, smem, 0);
  if (n_tiles > 1) load_tile(1);
  fetch_ids(2);
  __syncthreads();

  const int krow = key_of_row(lr);                    // this lane's key inside a 32-key sub-tile
  const int a_swz = lr & 15;

  // one tile step; J (compile-time) is the register set that held tile kt
  auto tile_step = [&](auto J, const int kt) {
    constexpr int j = decltype(J)::value;
    uint8_t* buf = smem + (kt & 1) * kTileBytes;
    if (kt + 2 < n_tiles) load_tile(j);                // tile kt+2 into set j (it held tile kt, already in LDS)
    fetch_ids(kt + 3);

    if (wave_active && BN * kt <= wave_max_pos) {
      // ---- S^T = K Q^T for the tile's two 32-key sub-tiles
      f32x16 S[2][NRT];
#pragma unroll
      for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int nt = 0; nt < NRT; ++nt)
#pragma unroll
          for (int i = 0; i < 16; ++i) S[st][nt][i] = 0.f;
      const uint8_t* krowp = buf + krow * 256;
      // K fragments are fetched from LDS one contraction step ahead of the MFMAs that use
      // them, so the LDS latency hides behind the previous step's two instructions
      vec ka[2][2];
      ka[0][0] = as_vec<vec>(*reinterpret_cast<const u32x4*>(krowp + ((hf ^ a_swz) << 4)));
      ka[0][1] = as_vec<vec>(*reinterpret_cast<const u32x4*>(krowp + 32 * 256 + ((hf ^ a_swz) << 4)));
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        if (kk + 1 < 8) {
          const int coff = ((2 * (kk + 1) + hf) ^ a_swz) << 4;
          ka[(kk + 1) & 1][0] = as_vec<vec>(*reinterpret_cast<const u32x4*>(krowp + coff));
          ka[(kk + 1) & 1][1] = as_vec<vec>(*reinterpret_cast<const u32x4*>(krowp + 32 * 256 + coff));
        }
        // the two sub-tiles are independent accumulation chains: alternate them
#pragma unroll
        for (int nt = 0; nt < NRT; ++nt) {
          S[0][nt] = M::mfma(ka[kk & 1][0], qf[nt][kk], S[0][nt]);
          S[1][nt] = M::mfma(ka[kk & 1][1], qf[nt][kk], S[1][nt]);
        }
      }
      // pin that order for the instruction scheduler: 4 LDS reads, then (2 MFMA, 2 LDS reads) x 7, 2 MFMA
      __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
      for (int kk = 0; kk < 7; ++kk) {
        __builtin_amdgcn_sched_group_barrier(0x008, 2 * NRT, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 2 * NRT, 0);
      // ---- causal mask on the tiles that reach past the first row's position
      if (BN * kt + BN - 1 > wave_min_pos) {
#pragma unroll
        for (int st = 0; st < 2; ++st)
#pragma unroll
          for (int nt = 0; nt < NRT; ++nt) {
            const int thr = prow[nt] - (BN * kt + 32 * st + 8 * hf);
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const int off = 16 * (i / 8) + 4 * ((i / 4) % 2) + (i % 4);
              S[st][nt][i] = off <= thr ? S[st][nt][i] : -INFINITY;
            }
          }
      }
      // ---- online softmax, one row per lane (both lane halves hold the same row)
      vec pb[2][NRT][2];
#pragma unroll
      for (int nt = 0; nt < NRT; ++nt) {
        float tmax = S[0][nt][0];
#pragma unroll
        for (int st = 0; st < 2; ++st)
#pragma unroll
          for (int i = 0; i < 16; ++i) tmax = fmaxf(tmax, S[st][nt][i]);
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        // The running maximum is only raised when some row of the wave has outgrown it by
        // more than 2^8: until then the weights are taken relative to the old maximum (they
        // stay below 256, exact in fp32 and well inside the 16-bit range), which spares the
        // rescaling of the 64 accumulator registers on almost every tile.
        if (__builtin_amdgcn_ballot_w64((tmax - mrow[nt]) * c > 8.f)) {
          const float m_new = fmaxf(mrow[nt], tmax);
          const float alpha = __builtin_amdgcn_exp2f((mrow[nt] - m_new) * c);
          mrow[nt] = m_new;
          lrow[nt] *= alpha;
#pragma unroll
          for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int i = 0; i < 16; ++i) O[nt][dt][i] *= alpha;
        }
        const float mc = mrow[nt] * c;
        float psum = 0.f;
#pragma unroll
        for (int st = 0; st < 2; ++st) {
          float p[16];
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            p[i] = __builtin_amdgcn_exp2f(fmaf(S[st][nt][i], c, -mc));
            psum += p[i];
          }
          pb[st][nt][0] = M::pack(p);
          pb[st][nt][1] = M::pack(p + 8);
        }
        lrow[nt] += psum;
      }
      // ---- O^T += V^T P^T, one pool block (16 keys) per instruction
#pragma unroll
      for (int b = 0; b < 4; ++b) {
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          const int d = 32 * dt + lr;
          const int off = kKBytes + b * 4096 + ((2 * d + (hf ^ ((d >> 2) & 1) ^ ((d >> 3) & 1))) << 4);
          vec va = as_vec<vec>(*reinterpret_cast<const u32x4*>(buf + off));
#pragma unroll
          for (int nt = 0; nt < NRT; ++nt) O[nt][dt] = M::mfma(va, pb[b >> 1][nt][b & 1], O[nt][dt]);
        }
      }
    }

    if (kt + 1 < n_tiles) store_tile(kt + 1, smem + ((kt + 1) & 1) * kTileBytes, (j + 1) % 2);
    __syncthreads();
  };
  for (int kt0 = 0; kt0 < n_tiles; kt0 += 2) {
    tile_step(std::integral_constant<int, 0>{}, kt0);
    if (kt0 + 1 < n_tiles) tile_step(std::integral_constant<int, 1>{}, kt0 + 1);
  }

  // ---- normalise and store: lane (row, half) holds channels 32dt + 8q + 4hf + (0..3)
  if (wave_active) {
#pragma unroll
    for (int nt = 0; nt < NRT; ++nt) {
      const float ltot = lrow[nt] + __shfl_xor(lrow[nt], 32);
      const float inv = 1.f / ltot;
      if (rvalid[nt]) {
        uint16_t* op = reinterpret_cast<uint16_t*>(a.out) + rowoff[nt];
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            uint16_t o4[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) o4[r] = M::out(O[nt][dt][4 * q + r] * inv);
            uint2 w;
            __builtin_memcpy(&w, o4, 8);
            *reinterpret_cast<uint2*>(op + 32 * dt + 8 * q + 4 * hf) = w;
          }
      }
    }
  }
}

}  // namespace

flp_status flp_launch_attn_mfma(int dtype, const FlpAttnArgs& a, const FlpMfmaItem* items_dev, int32_t n_items,
                                hipStream_t stream) {
  if (n_items <= 0) return FLP_OK;
  if (dtype == FLP_F16)
    hipLaunchKernelGGL((attn_mfma_kernel<MF16, 1>), dim3(n_items), dim3(512), 0, stream, a, items_dev);
  else if (dtype == FLP_BF16)
    hipLaunchKernelGGL((attn_mfma_kernel<MBF16, 1>), dim3(n_items), dim3(512), 0, stream, a, items_dev);
  else {
    flp_set_error("attention (matrix-core path): dtype %d not supported", dtype);
    return FLP_ENOTSUP;
  }
  FLP_TRY_HIP(hipGetLastError());
  return FLP_OK;
}
