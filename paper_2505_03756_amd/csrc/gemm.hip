// Dense products of the layer step: the base projection y = x . W_base of flp_lora_apply_paged when the caller
// passes w_base (paper Eq. 1: W' = W + A B; this is the W term.  The paper keeps the base model outside the pool,
// and so does this library: w_base is an ordinary dense matrix, [d_in, d_out] or [d_out, d_in]), and the dense
// projections of fll_layer_forward.
//
// 16-bit pools: both operands are read along the contraction (a W given as [d_in, d_out] is first transposed into
// the pool's workspace).  Two tiled MFMA kernels, both computing the product transposed (A operand = rows of W^T,
// B operand = token rows) with the rows of W^T fed in a permuted order, so that a lane ends up with 16 consecutive
// output columns of one token and y is written in 32-byte pieces:
//   gemm_nt_kernel      128 x 128 tile, 4 waves x (64 x 64), k tiles of 64 through LDS with the next tile prefetched
//                       through registers; small batches, with the contraction split over grid z when tiles are few;
//   gemm_nt256_kernel   256 x 256 tile, 4 waves x (128 x 128), operands streamed by direct global-to-LDS loads; large
//                       batches.  Two epilogue variants: GATED (gate and up of an MLP in one pass, silu(g) * u stored)
//                       and LORA (the expand step of the projection's LoRA branch added to the accumulators).
// fp32 pools: a plain one-thread-per-output kernel (the fp32 workload is tiny).
#include <atomic>
#include <hip/hip_runtime.h>

#include <type_traits>

#include "flp_internal.h"
#include "flp_types.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4g __attribute__((ext_vector_type(4)));
typedef _Float16 h16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 b16x8 __attribute__((ext_vector_type(8)));

struct GF16 {
  typedef h16x8 vec;
  typedef _Float16 elem;
  static __device__ __forceinline__ f32x16 mfma(vec a, vec b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint16_t out(float f) { return F16::from_float(f); }
  static __device__ __forceinline__ float in(uint16_t b) { return F16::to_float(b); }
};
struct GBF16 {
  typedef b16x8 vec;
  typedef __bf16 elem;
  static __device__ __forceinline__ f32x16 mfma(vec a, vec b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint16_t out(float f) { return BF16::from_float(f); }
  static __device__ __forceinline__ float in(uint16_t b) { return BF16::to_float(b); }
};

// ---- W [K, N] -> Wt [N, K], 16-bit elements, 64 x 64 tiles through LDS
__global__ __launch_bounds__(256) void transpose16_kernel(const uint16_t* __restrict__ w, uint16_t* __restrict__ wt,
                                                          int K, int N) {
  __shared__ uint16_t tile[64][66];
  const int k0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  for (int i = threadIdx.x; i < 64 * 64; i += 256) {
    const int r = i >> 6, c = i & 63;
    tile[r][c] = (k0 + r < K && n0 + c < N) ? w[(int64_t)(k0 + r) * N + n0 + c] : (uint16_t)0;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < 64 * 64; i += 256) {
    const int r = i >> 6, c = i & 63;      // r: n within tile, c: k within tile
    if (n0 + r < N && k0 + c < K) wt[(int64_t)(n0 + r) * K + k0 + c] = tile[c][r];
  }
}

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int kTile = 128 * BK * 2;        // bytes of one operand tile (16 KiB)

// byte offset of 16-byte chunk c (0..7) of row r (0..127) inside an operand tile: two rows share
// a 256-byte line and the 16 chunk slots of the line are XOR-swizzled with the line index, so the
// 16 lanes that read one logical chunk of 16 consecutive rows hit 16 different bank groups
__device__ __forceinline__ int tile_off(int r, int c) { return (r >> 1) * 256 + (((((r & 1) << 3) | c) ^ ((r >> 1) & 15)) << 4); }

// The product is stored rounded into y and, when y32 is given, also unrounded as fp32 ([M, N]
// dense): the LoRA expand kernel adds the adapter's delta to the unrounded value and rounds once;
// rows of tokens without an adapter keep the rounded value.
// With gridDim.z > 1 the contraction is split: slice z covers K / gridDim.z coefficients and writes its
// unrounded partial product to part + z * M * N (dense fp32); gemm_splitk_reduce_kernel adds the slices in
// order and rounds.  Small batches (decode) have too few 128 x 128 tiles to occupy the chip otherwise.
template <typename G>
__global__ __launch_bounds__(256, 2) void gemm_nt_kernel(const uint16_t* __restrict__ x, int64_t ld_x,
                                                         const uint16_t* __restrict__ wt, uint16_t* __restrict__ y,
                                                         int64_t ld_y, float* __restrict__ y32, int M, int N, int K,
                                                         float* __restrict__ part) {
  typedef typename G::vec vec;
  __shared__ __attribute__((aligned(16))) uint8_t smem[2][2 * kTile];      // [buffer][Wt tile | x tile]
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lr = lane & 31, hf = lane >> 5;
  const int n0 = blockIdx.x * BN, m0 = blockIdx.y * BM;
  const int wn = (wave & 1) * 64, wm = (wave >> 1) * 64;                   // this wave's 64 x 64 corner

  // staging: thread -> chunk (tid & 7) of rows (tid >> 3) + 32*i, i = 0..3, for both operands
  const int sc = tid & 7, sr = tid >> 3;
  u32x4 areg[4], breg[4];
  auto load_tiles = [&](int k0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = sr + 32 * i;
      const int n = n0 + r < N ? n0 + r : N - 1;                            // clamped rows are never stored
      const int m = m0 + r < M ? m0 + r : M - 1;
      areg[i] = *reinterpret_cast<const u32x4*>(wt + (int64_t)n * K + k0 + 8 * sc);
      breg[i] = *reinterpret_cast<const u32x4*>(x + (int64_t)m * ld_x + k0 + 8 * sc);
    }
  };
  auto store_tiles = [&](uint8_t* buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = sr + 32 * i;
      *reinterpret_cast<u32x4*>(buf + tile_off(r, sc)) = areg[i];
      *reinterpret_cast<u32x4*>(buf + kTile + tile_off(r, sc)) = breg[i];
    }
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // A-operand row a of a 32-row tile is output column 16*((a>>2)&1) + 4*(a>>3) + (a&3) of that tile
  const int acol = (((lr >> 2) & 1) << 4) | ((lr >> 3) << 2) | (lr & 3);

  const int nk = K / BK / (int)gridDim.z, kt0 = (int)blockIdx.z * nk;    // this slice's k tiles
  if (gridDim.z > 1) {
    y = nullptr;
    y32 = part + (int64_t)blockIdx.z * M * N;
  }
  load_tiles(kt0 * BK);
  store_tiles(smem[0]);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const uint8_t* buf = smem[kt & 1];
    if (kt + 1 < nk) load_tiles((kt0 + kt + 1) * BK);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      vec af[2], bf[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        af[i] = *reinterpret_cast<const vec*>(buf + tile_off(wn + 32 * i + acol, 2 * kk + hf));
        bf[i] = *reinterpret_cast<const vec*>(buf + kTile + tile_off(wm + 32 * i + lr, 2 * kk + hf));
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = G::mfma(af[i], bf[j], acc[i][j]);
    }
    if (kt + 1 < nk) store_tiles(smem[(kt + 1) & 1]);
    __syncthreads();
  }

  // lane (token lr of tile j, half hf) holds columns 16*hf .. 16*hf+15 of column tile i:
  // register 4*q + r of the accumulator is column 16*hf + 4*q + r
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int m = m0 + wm + 32 * j + lr;
    if (m >= M) continue;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int n = n0 + wn + 32 * i + 16 * hf;
      if (y32) {                                     // 64 contiguous bytes per lane where the row allows it
        float* yp32 = y32 + (int64_t)m * N + n;
        if (n + 16 <= N && (N & 3) == 0) {
#pragma unroll
          for (int e4 = 0; e4 < 4; ++e4) {
            f32x4g v4 = {acc[i][j][4 * e4], acc[i][j][4 * e4 + 1], acc[i][j][4 * e4 + 2], acc[i][j][4 * e4 + 3]};
            reinterpret_cast<f32x4g*>(yp32)[e4] = v4;
          }
        } else {
          for (int e = 0; e < 16; ++e)
            if (n + e < N) yp32[e] = acc[i][j][e];
        }
      }
      if (!y) continue;                              // a slice of a split contraction writes only its partial
      uint16_t o[16];
#pragma unroll
      for (int e = 0; e < 16; ++e) o[e] = G::out(acc[i][j][e]);
      uint16_t* yp = y + (int64_t)m * ld_y + n;
      if (n + 16 <= N) {
        u32x4 raw[2];
        __builtin_memcpy(raw, o, 32);
        reinterpret_cast<u32x4*>(yp)[0] = raw[0];
        reinterpret_cast<u32x4*>(yp)[1] = raw[1];
      } else {
        for (int e = 0; e < 16; ++e)
          if (n + e < N) yp[e] = o[e];
      }
    }
  }
}

// ---- large batches: 256 x 256 output tile per workgroup, operands streamed by direct global-to-LDS loads
//
// Four waves, each a 128 x 128 corner (4 x 4 accumulators of mfma_f32_32x32x16: 256 accumulator registers,
// one wave per SIMD), so that a k step of 16 costs 8 fragment reads for 16 MFMAs: LDS traffic per flop is
// half that of a 64 x 64 corner, and the operand tiles are fetched from L2 half as often as with 128 x 128
// workgroup tiles.  Operand tiles are 256 rows x 64 coefficients (32 KiB each, 64 KiB per stage, two stages):
// a row's 64 coefficients are one whole 128-byte line, and a global_load_lds_dwordx4 instruction (no registers,
// no LDS store instructions; inline assembly with its own s_waitcnt vmcnt) moves 8 whole lines.  Requests of
// half a line (tiles of 32 coefficients in a ring of four) made every line cross from L2 twice and were 4-8 %
// slower.  One barrier per stage, before its last k step: by then the wave has waited for its loads of the next
// stage and has read the last fragments of this one, so after the barrier the next stage is complete for
// everybody (its first fragments are read during the last step) and this stage's buffer is free for the stage
// after next.  LDS layout: row r at r * 128, its 16-byte chunk c in slot c ^ gswz(r), which spreads the 16 lanes
// that read one chunk of their (permuted) 16 rows over the 16 slots of a 256-byte bank window; the swizzle is
// applied on the global side (a lane fetches the chunk that belongs at its fixed LDS slot).  Workgroups of one
// XCD (ids congruent modulo 8) cover 4 x 8 blocks of tiles, so the 32 that run together fetch 12 operand panels
// instead of 64.
constexpr int GT = 256, GK = 64, kGOperand = GT * GK * 2, kGStage = 2 * kGOperand, kGStages = 2;   // 64 KiB per stage
// s_waitcnt immediate (gfx9 encoding: vmcnt[3:0] + [15:14], expcnt[6:4], lgkmcnt[11:8]): vmcnt only
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

// M0 is named as clobbered so that no pass keeps a value of its own alive in it across the statement; the
// compiler notes that it reserves the register, which is the point.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void gload_lds16(const void* base, uint32_t voff, uint32_t lds) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(base), "s"(lds)
               : "memory", "m0");
}
#pragma clang diagnostic pop
typedef __attribute__((address_space(3))) uint8_t g_lds_u8;

// swizzle of row r: the 16-byte chunk c of the row sits in slot c ^ gswz(r) of the row's 128 bytes
__device__ __forceinline__ int gswz(int r) { return ((r >> 1) & 3) | (((r >> 4) & 1) << 2); }
// byte offset of 16-byte chunk c (0..7) of row r (0..255) inside a 256 x 64 operand tile
__device__ __forceinline__ int gtile_off(int r, int c) { return r * 128 + ((c ^ gswz(r)) << 4); }

//
// GATED: the gated-SiLU pair of an MLP in one pass.  The 256 feature rows of a tile are 128 rows of the gate
// matrix (wt) and the same 128 rows of the up matrix (wt2): the waves with wi = 0 multiply the gate rows, those
// with wi = 1 the up rows of the same features and tokens.  After the loop the up waves hand their accumulators
// over through LDS (lane to lane: both layouts are the same) and the gate waves store silu(g) * u, with g and u rounded to the element type first, as the two separate products and
// the element-wise kernel would have stored and re-read them.  Neither product is written.
//
// LORA: the expand step of one projection's LoRA branch as an epilogue.  After the loop a wave holds the dense product
// of its 128 tokens x 128 features; for every adapter among those tokens (tokens of a sequence are neighbours, so one
// or two) it adds B^T (features x ranks, gathered from the adapter's pages in the A-operand layout of the same
// permuted feature rows) times the tokens' scaled v (ranks x tokens, zero for tokens of other adapters; split into a
// 16-bit high part and remainder, two MFMAs, so that v keeps its fp32 precision), 16 ranks per step, straight into
// the accumulators.  The sum is rounded once; there is no fp32 copy of the product and no second pass over y.
template <typename G, bool GATED, bool LORA>
__global__ __launch_bounds__(256, 1) void gemm_nt256_kernel(const uint16_t* __restrict__ x, int64_t ld_x,
                                                            const uint16_t* __restrict__ wt,
                                                            const uint16_t* __restrict__ wt2, uint16_t* __restrict__ y,
                                                            int64_t ld_y, float* __restrict__ y32, int M, int N, int K,
                                                            int tiles_n, int tiles_m, int groups_n, FlpGemmLora lpa,
                                                            FlpGemmLora lp2) {
  constexpr int GTN = GATED ? GT / 2 : GT;              // output features per tile
  typedef typename G::vec vec;
  extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
  const int tid = threadIdx.x, lane = tid & 63, lr = lane & 31, hf = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wi = wave & 1, wj = wave >> 1;

  // workgroup -> tile: 32 consecutive workgroups of one XCD form a block of 4 feature tiles x 8 token tiles
  const int xcd = blockIdx.x & 7, l = blockIdx.x >> 3;
  const int gid = (l >> 5) * 8 + xcd, within = l & 31;
  const int tn = (gid % groups_n) * 4 + (within & 3), tm = (gid / groups_n) * 8 + (within >> 2);
  if (tn >= tiles_n || tm >= tiles_m) return;
  const int n0 = tn * GTN, m0 = tm * GT;
  const uint16_t* __restrict__ wsrc = GATED && wave >= 2 ? wt2 : wt;   // feature rows 128 .. 255 of a gated tile: the up matrix

  // ---- staging: wave w moves rows 64w .. 64w+63 of both tiles, 8 rows (8 whole 128-byte lines) per instruction;
  //      lane l fills slot l % 8 of row l / 8 of the instruction's 1 KiB of LDS, i.e. fetches chunk slot ^ gswz(row)
  uint32_t va[8], vb[8];
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const int r = 64 * wave + 8 * q + (lane >> 3);
    const int ch = (lane & 7) ^ gswz(r);
    const int rf = GATED ? (r & (GTN - 1)) : r;
    const int n = n0 + rf < N ? n0 + rf : N - 1;              // clamped rows are never stored
    const int m = m0 + r < M ? m0 + r : M - 1;
    va[q] = (uint32_t)(((int64_t)n * K + 8 * ch) * 2);
    vb[q] = (uint32_t)(((int64_t)m * ld_x + 8 * ch) * 2);
  }
  const uint32_t lds_wave = (uint32_t)(uintptr_t)(g_lds_u8*)smem + 8192u * (uint32_t)wave;
  const int nk = K / GK;
  // one of the 16 direct loads of stage t: q = 0..7 the W^T tile, q = 8..15 the token tile
  auto issue_load = [&](int t, int q) {
    const int tk = t < nk ? t : nk - 1;                       // past the end: the last tile again, into a free stage
    const uint32_t dst = lds_wave + (uint32_t)(t & 1) * kGStage;
    if (q < 8)
      gload_lds16(wsrc + (int64_t)tk * GK, va[q], dst + 1024 * q);
    else
      gload_lds16(x + (int64_t)tk * GK, vb[q - 8], dst + kGOperand + 1024 * (q - 8));
  };

  // ---- fragments: both operands take their 32 rows in the permuted order that gives a lane 16 consecutive output
  //      columns (row a of a 32-row tile is column 16*((a>>2)&1) + 4*(a>>3) + (a&3)); for the token tile the
  //      permutation only decides which token a lane ends up holding
  const int acol = (((lr >> 2) & 1) << 4) | ((lr >> 3) << 2) | (lr & 3);
  int offa[4], offb[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    offa[i] = gtile_off(128 * wi + 32 * i + acol, hf);
    offb[i] = kGOperand + gtile_off(128 * wj + 32 * i + acol, hf);
  }
  // chunk 2*kk + hf of the row: bits 1, 2 of the slot, bits 5, 6 of the offset
  auto frag = [&](int t, int kk, int off) {
    return *reinterpret_cast<const vec*>(smem + (t & 1) * kGStage + (off ^ (kk << 5)));
  };

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  vec a0[4], b0[4], a1[4], b1[4];
  // One k step of 16: four groups of {two direct loads or none, the two fragment reads that the step after this
  // one needs, four MFMAs}, fenced so that they stay in this order (a burst of loads holds the wave's in-order
  // instruction stream, and with it the matrix pipe, for as long as the memory pipeline takes to accept them;
  // measured: two loads per group over two steps; all sixteen in one step costs 5 %, waiting a stage later for
  // them changes nothing - the stream's rate, not its latency, is what the loop feels).
  auto kstep = [&](vec(&ca)[4], vec(&cb)[4], vec(&na)[4], vec(&nb)[4], int t_next, int kk_next, int t_load, int q0) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      if (q0 >= 0) {
#pragma unroll
        for (int u = 0; u < 2; ++u) issue_load(t_load, q0 + 2 * g + u);
      }
      if (g < 2) {                                            // all token fragments first: the next step's first group needs them
        nb[2 * g] = frag(t_next, kk_next, offb[2 * g]);
        nb[2 * g + 1] = frag(t_next, kk_next, offb[2 * g + 1]);
      } else {
        na[2 * g - 4] = frag(t_next, kk_next, offa[2 * g - 4]);
        na[2 * g - 3] = frag(t_next, kk_next, offa[2 * g - 3]);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[g][j] = G::mfma(ca[g], cb[j], acc[g][j]);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // ---- prologue: stage 0 complete, the first half of stage 1 requested
#pragma unroll
  for (int q = 0; q < 16; ++q) issue_load(0, q);
  __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
  __syncthreads();
#pragma unroll
  for (int q = 0; q < 8; ++q) issue_load(1, q);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a0[i] = frag(0, 0, offa[i]);
    b0[i] = frag(0, 0, offb[i]);
  }
  for (int kt = 0; kt < nk; ++kt) {
    // Stage kt is multiplied in four k steps.  The second half of stage kt + 1 is requested during the first step;
    // before the last step the wave waits for its loads of stage kt + 1, and after the barrier everybody's have
    // landed and everybody has read the last fragments of stage kt: the last step reads the first fragments of
    // stage kt + 1 and requests the first half of stage kt + 2 into the buffer that stage kt leaves.
    kstep(a0, b0, a1, b1, kt, 1, kt + 1, 8);
    kstep(a1, b1, a0, b0, kt, 2, 0, -1);
    kstep(a0, b0, a1, b1, kt, 3, 0, -1);
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    __syncthreads();
    kstep(a1, b1, a0, b0, kt + 1, 0, kt + 2, 0);
  }
  __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));               // the look-ahead loads must land before the LDS is released

  if constexpr (LORA) {
    typedef typename G::elem elem;
    // a gated tile's up waves add the up projection's branch (lp2), everybody else the projection's own (lpa)
    const FlpGemmLora& lp = GATED && wi == 1 ? lp2 : lpa;
    const int fbase = GATED ? n0 : n0 + 128 * wi;         // the wave's first feature
    const uint16_t* __restrict__ pool = reinterpret_cast<const uint16_t*>(lp.pool);
    const int rpb = (int)(lp.block_elems / N);
    int adj[4], posj[4];                                  // adapter and segment-order position of the lane's four tokens
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + 128 * wj + 32 * j + acol;
      int ad = m < M ? lp.token_adapter[m] : -1;
      if (ad >= lp.n_adapters) ad = -1;
      adj[j] = ad;
      posj[j] = ad >= 0 ? lp.inv_perm[m] : 0;
    }
    for (;;) {
      int cand = -1;
#pragma unroll
      for (int j = 3; j >= 0; --j) cand = adj[j] >= 0 ? adj[j] : cand;
      const uint64_t todo = __ballot(cand >= 0);
      if (!todo) break;
      const int ad = __builtin_amdgcn_readlane(cand, __ffsll((long long)todo) - 1);      // wave-uniform
      const int r = lp.rank[ad] < lp.max_rank ? lp.rank[ad] : lp.max_rank;
      if (r > 0) {
        const float sc = lp.scale[ad];
        const int64_t vrow0 = lp.vrow_base[ad];
        const int32_t* __restrict__ tab = lp.tables + lp.b_tab_off[ad];
        const int brow0 = lp.b_row_base[ad];
        for (int nt = 0; 16 * nt < r; ++nt) {
          // A operand: B[rho, feature] for the lane's 8 ranks and its feature row of each of the four feature tiles
          const uint16_t* rowp[8];
#pragma unroll
          for (int q = 0; q < 8; ++q) {
            const int rho = 16 * nt + 8 * hf + q;
            const int row = brow0 + (rho < r ? rho : 0);
            rowp[q] = pool + (int64_t)tab[row / rpb] * lp.block_elems + (int64_t)(row % rpb) * N;
          }
          vec af[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int f = fbase + 32 * i + acol;
            const int fc = f < N ? f : N - 1;
            uint16_t g8[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) g8[q] = rowp[q][fc];
#pragma unroll
            for (int q = 0; q < 8; ++q)
              if (!(16 * nt + 8 * hf + q < r && f < N)) g8[q] = 0;
            __builtin_memcpy(&af[i], g8, 16);
          }
          // B operand: the tokens' scaled v for those 8 ranks, zero for tokens of other adapters
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            float v8[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) v8[q] = 0.f;
            if (adj[j] == ad) {
              for (int ks = 0; ks < lp.k_splits; ++ks) {
                const float* vp = lp.v + (((int64_t)ks * lp.v_rows + vrow0 + posj[j]) * lp.n_proj + lp.p) * lp.rp +
                                  16 * nt + 8 * hf;
                const f32x4g x0 = *reinterpret_cast<const f32x4g*>(vp), x1 = *reinterpret_cast<const f32x4g*>(vp + 4);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                  v8[q] += x0[q];
                  v8[4 + q] += x1[q];
                }
              }
            }
            vec bh, bl;
#pragma unroll
            for (int q = 0; q < 8; ++q) {
              const float vs = v8[q] * sc;
              const elem h = (elem)vs;
              bh[q] = h;
              bl[q] = (elem)(vs - (float)h);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              acc[i][j] = G::mfma(af[i], bh, acc[i][j]);
              acc[i][j] = G::mfma(af[i], bl, acc[i][j]);
            }
          }
        }
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) adj[j] = adj[j] == ad ? -1 : adj[j];
    }
  }

  if constexpr (GATED) {
    // The gate wave and the up wave of a token half split the gating between them: the gate wave hands over its
    // feature tiles 2, 3 and finishes tiles 0, 1, the up wave the other way round (128 accumulator values per lane
    // each way, [wave][value][lane] in the 128 KiB the stages leave), so all four waves share the element-wise work.
    float* const xbase = reinterpret_cast<float*>(smem) + lane;
    float* const xown = xbase + (wave * 128) * 64;
    const float* const xother = xbase + ((wave ^ 1) * 128) * 64;
    __syncthreads();                                       // everybody's loads have landed, nobody reads fragments any more
    auto send = [&](auto i0) {                             // feature tiles i0, i0 + 1 of this wave
      constexpr int I0 = decltype(i0)::value;
#pragma unroll
      for (int ii = 0; ii < 2; ++ii)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int e = 0; e < 16; ++e) xown[((ii * 4 + j) * 16 + e) * 64] = acc[I0 + ii][j][e];
    };
    auto finish = [&](auto i0, auto own_is_gate) {         // feature tiles i0, i0 + 1: own values and the partner's
      constexpr int I0 = decltype(i0)::value;
      constexpr bool OWN_GATE = decltype(own_is_gate)::value;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int m = m0 + 128 * wj + 32 * j + acol;
#pragma unroll
        for (int ii = 0; ii < 2; ++ii) {
          const int n = n0 + 32 * (I0 + ii) + 16 * hf;
          uint16_t o[16];
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const float own = G::in(G::out(acc[I0 + ii][j][e]));
            const float oth = G::in(G::out(xother[((ii * 4 + j) * 16 + e) * 64]));
            const float g = OWN_GATE ? own : oth, u = OWN_GATE ? oth : own;
            o[e] = G::out(g / (1.0f + expf(-g)) * u);
          }
          if (m >= M || n >= N) continue;
          uint16_t* yp = y + (int64_t)m * ld_y + n;
          if (n + 16 <= N) {
            u32x4 raw[2];
            __builtin_memcpy(raw, o, 32);
            reinterpret_cast<u32x4*>(yp)[0] = raw[0];
            reinterpret_cast<u32x4*>(yp)[1] = raw[1];
          } else {
            for (int e = 0; e < 16; ++e)
              if (n + e < N) yp[e] = o[e];
          }
        }
      }
    };
    using I0c = std::integral_constant<int, 0>;
    using I2c = std::integral_constant<int, 2>;
    if (wi == 0) send(I2c{}); else send(I0c{});
    __syncthreads();
    if (wi == 0) finish(I0c{}, std::true_type{}); else finish(I2c{}, std::false_type{});
    return;
  }

  // lane (token acol of tile j, half hf) holds columns 16*hf .. 16*hf+15 of feature tile i
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int m = m0 + 128 * wj + 32 * j + acol;
    if (m >= M) continue;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int n = n0 + 128 * wi + 32 * i + 16 * hf;
      if (n >= N) continue;
      if (y32) {
        float* yp32 = y32 + (int64_t)m * N + n;
        if (n + 16 <= N && (N & 3) == 0) {
#pragma unroll
          for (int e4 = 0; e4 < 4; ++e4) {
            f32x4g v4 = {acc[i][j][4 * e4], acc[i][j][4 * e4 + 1], acc[i][j][4 * e4 + 2], acc[i][j][4 * e4 + 3]};
            reinterpret_cast<f32x4g*>(yp32)[e4] = v4;
          }
        } else {
          for (int e = 0; e < 16; ++e)
            if (n + e < N) yp32[e] = acc[i][j][e];
        }
      }
      uint16_t o[16];
#pragma unroll
      for (int e = 0; e < 16; ++e) o[e] = G::out(acc[i][j][e]);
      uint16_t* yp = y + (int64_t)m * ld_y + n;
      if (n + 16 <= N) {
        u32x4 raw[2];
        __builtin_memcpy(raw, o, 32);
        reinterpret_cast<u32x4*>(yp)[0] = raw[0];
        reinterpret_cast<u32x4*>(yp)[1] = raw[1];
      } else {
        for (int e = 0; e < 16; ++e)
          if (n + e < N) yp[e] = o[e];
      }
    }
  }
}

// y[m, n] = round(sum over the slices, in slice order); y32 (optional) gets the unrounded sum
template <typename G>
__global__ __launch_bounds__(256) void gemm_splitk_reduce_kernel(const float* __restrict__ part, int slices, int M, int N,
                                                                 uint16_t* __restrict__ y, int64_t ld_y,
                                                                 float* __restrict__ y32) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x, total = (int64_t)M * N;
  if (i >= total) return;
  float sum = part[i];
  for (int z = 1; z < slices; ++z) sum += part[(int64_t)z * total + i];
  const int64_t m = i / N;
  const int n = (int)(i - m * N);
  y[m * ld_y + n] = G::out(sum);
  if (y32) y32[i] = sum;
}

__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ x, int64_t ld_x,
                                                       const float* __restrict__ w, int64_t w_k_stride,
                                                       int64_t w_n_stride, float* __restrict__ y, int64_t ld_y, int M,
                                                       int N, int K) {
  const int n = blockIdx.x * 256 + threadIdx.x, m = blockIdx.y;
  if (n >= N) return;
  float acc = 0.f;
  for (int k = 0; k < K; ++k) acc = fmaf(x[(int64_t)m * ld_x + k], w[k * w_k_stride + n * w_n_stride], acc);
  y[(int64_t)m * ld_y + n] = acc;
}

flp_status gemm256_attrs() {
  const void* fns[8] = {(const void*)gemm_nt256_kernel<GF16, false, false>, (const void*)gemm_nt256_kernel<GBF16, false, false>,
                        (const void*)gemm_nt256_kernel<GF16, true, false>, (const void*)gemm_nt256_kernel<GBF16, true, false>,
                        (const void*)gemm_nt256_kernel<GF16, false, true>, (const void*)gemm_nt256_kernel<GBF16, false, true>,
                        (const void*)gemm_nt256_kernel<GF16, true, true>, (const void*)gemm_nt256_kernel<GBF16, true, true>};
  for (const void* f : fns)
    FLP_TRY_HIP(hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, kGStages * kGStage));
  return FLP_OK;
}

// the shapes the 256 x 256 kernel takes: 32-bit byte offsets inside the operands, whole 64-coefficient stages
bool gemm256_fits(int64_t M, int64_t n_rows_w, int64_t K, int64_t ld_x) {
  return M >= 1024 && M * ld_x * 2 < ((int64_t)1 << 32) && n_rows_w * K * 2 < ((int64_t)1 << 32) && ld_x % 8 == 0 &&
         K % GK == 0 && K / GK >= kGStages;
}

}  // namespace

// out[M, N] = silu(x . Wg^T) * (x . Wu^T) with both matrices stored [N, K], 16-bit element types, in one pass of
// the large-batch kernel (the two products are rounded to the element type before the gate is applied, as if
// they had been stored).  Returns FLP_ENOTSUP without launching when the shape is one that the kernel does not
// take (small batches, few tiles, offsets beyond 32 bits): the caller then runs the two products and the
// element-wise step.
flp_status flp_launch_gated_gemm(int dtype, const void* x, int64_t ld_x, const void* w_gate, const void* w_up,
                                 void* out, int64_t ld_out, int M, int N, int K, hipStream_t stream,
                                 const FlpGemmLora* lora_gate, const FlpGemmLora* lora_up) {
  if (dtype != FLP_F16 && dtype != FLP_BF16) return FLP_ENOTSUP;
  const int tiles_n = (N + GT / 2 - 1) / (GT / 2), tiles_m = (M + GT - 1) / GT;
  if (M <= 0 || N < 128 || K <= 0 || !gemm256_fits(M, N, K, ld_x) || (int64_t)tiles_n * tiles_m < 96) return FLP_ENOTSUP;
  if ((lora_gate != nullptr) != (lora_up != nullptr)) return FLP_ENOTSUP;
  static std::atomic<bool> attr_set{false};   // pools on different threads share it
  if (!attr_set.load(std::memory_order_acquire)) {
    FLP_TRY(gemm256_attrs());
    attr_set.store(true, std::memory_order_release);
  }
  const int groups_n = (tiles_n + 3) / 4, groups_m = (tiles_m + 7) / 8;
  const int n_groups = (groups_n * groups_m + 7) / 8 * 8;
  dim3 grid((unsigned)(n_groups * 32));
  const uint16_t *xs = (const uint16_t*)x, *wg = (const uint16_t*)w_gate, *wu = (const uint16_t*)w_up;
  float* no32 = nullptr;
  const size_t lds = kGStages * kGStage;
  if (lora_gate && dtype == FLP_F16)
    hipLaunchKernelGGL((gemm_nt256_kernel<GF16, true, true>), grid, dim3(256), lds, stream, xs, ld_x, wg, wu, (uint16_t*)out,
                       ld_out, no32, M, N, K, tiles_n, tiles_m, groups_n, *lora_gate, *lora_up);
  else if (lora_gate)
    hipLaunchKernelGGL((gemm_nt256_kernel<GBF16, true, true>), grid, dim3(256), lds, stream, xs, ld_x, wg, wu, (uint16_t*)out,
                       ld_out, no32, M, N, K, tiles_n, tiles_m, groups_n, *lora_gate, *lora_up);
  else if (dtype == FLP_F16)
    hipLaunchKernelGGL((gemm_nt256_kernel<GF16, true, false>), grid, dim3(256), lds, stream, xs, ld_x, wg, wu, (uint16_t*)out,
                       ld_out, no32, M, N, K, tiles_n, tiles_m, groups_n, FlpGemmLora{}, FlpGemmLora{});
  else
    hipLaunchKernelGGL((gemm_nt256_kernel<GBF16, true, false>), grid, dim3(256), lds, stream, xs, ld_x, wg, wu,
                       (uint16_t*)out, ld_out, no32, M, N, K, tiles_n, tiles_m, groups_n, FlpGemmLora{}, FlpGemmLora{});
  FLP_TRY_HIP(hipGetLastError());
  return FLP_OK;
}

bool flp_gemm_gated_fits(int dtype, int M, int N, int K, int64_t ld_x) {
  return (dtype == FLP_F16 || dtype == FLP_BF16) && M > 0 && N >= 128 && K > 0 && gemm256_fits(M, N, K, ld_x) &&
         (int64_t)((N + GT / 2 - 1) / (GT / 2)) * ((M + GT - 1) / GT) >= 96;
}

bool flp_gemm_is_large(int dtype, int M, int N, int K, int64_t ld_x) {
  return (dtype == FLP_F16 || dtype == FLP_BF16) && N >= 256 &&
         (int64_t)((M + GT - 1) / GT) * ((N + GT - 1) / GT) >= 96 && gemm256_fits(M, N, K, ld_x);
}

// y[M, N] = x[M, K] . W with w stored [K, N] (w_layout 0) or [N, K] (w_layout 1).  `wt_scratch` (16-bit
// types with layout 0 only) must hold N*K elements; `y32` (16-bit types, optional) receives the
// unrounded product as dense fp32 [M, N].
flp_status flp_launch_base_gemm(int dtype, const void* x, int64_t ld_x, const void* w, int w_layout, void* y,
                                int64_t ld_y, int M, int N, int K, void* wt_scratch, float* y32, float* splitk_scratch,
                                size_t splitk_bytes, hipStream_t stream, const FlpGemmLora* lora) {
  if (M <= 0 || N <= 0 || K <= 0) return FLP_OK;
  if (lora && !flp_gemm_is_large(dtype, M, N, K, ld_x)) {
    flp_set_error("base GEMM: the LoRA epilogue needs the large-batch kernel (M=%d N=%d K=%d)", M, N, K);
    return FLP_ENOTSUP;
  }
  if (dtype == FLP_F32) {
    hipLaunchKernelGGL(gemm_f32_kernel, dim3((N + 255) / 256, M), dim3(256), 0, stream, (const float*)x, ld_x,
                       (const float*)w, w_layout ? (int64_t)1 : (int64_t)N, w_layout ? (int64_t)K : (int64_t)1, (float*)y,
                       ld_y, M, N, K);
    FLP_TRY_HIP(hipGetLastError());
    return FLP_OK;
  }
  if (K % BK != 0) {
    flp_set_error("base GEMM: d_in %d is not a multiple of %d", K, BK);
    return FLP_ENOTSUP;
  }
  if (w_layout == 0)
    hipLaunchKernelGGL(transpose16_kernel, dim3((N + 63) / 64, (K + 63) / 64), dim3(256), 0, stream, (const uint16_t*)w,
                       (uint16_t*)wt_scratch, K, N);
  const uint16_t* xs = (const uint16_t*)x;
  const uint16_t* ws = w_layout == 0 ? (const uint16_t*)wt_scratch : (const uint16_t*)w;
  // 32-bit byte offsets inside the operands and enough 256 x 256 tiles to occupy the chip (measured: with 64
  // tiles the 128 x 128 kernel is ahead, from 172 tiles on this one): the 256 x 256 kernel
  if (flp_gemm_is_large(dtype, M, N, K, ld_x)) {
    const int tiles_n = (N + GT - 1) / GT, tiles_m = (M + GT - 1) / GT;
    const int groups_n = (tiles_n + 3) / 4, groups_m = (tiles_m + 7) / 8;
    const int n_groups = (groups_n * groups_m + 7) / 8 * 8;
    dim3 grid256((unsigned)(n_groups * 32));
    static std::atomic<bool> attr_set{false};   // pools on different threads share it
    if (!attr_set.load(std::memory_order_acquire)) {
      FLP_TRY(gemm256_attrs());
      attr_set.store(true, std::memory_order_release);
    }
    const uint16_t* none = nullptr;
    if (lora && dtype == FLP_F16)
      hipLaunchKernelGGL((gemm_nt256_kernel<GF16, false, true>), grid256, dim3(256), kGStages * kGStage, stream, xs, ld_x,
                         ws, none, (uint16_t*)y, ld_y, y32, M, N, K, tiles_n, tiles_m, groups_n, *lora, FlpGemmLora{});
    else if (lora)
      hipLaunchKernelGGL((gemm_nt256_kernel<GBF16, false, true>), grid256, dim3(256), kGStages * kGStage, stream, xs, ld_x,
                         ws, none, (uint16_t*)y, ld_y, y32, M, N, K, tiles_n, tiles_m, groups_n, *lora, FlpGemmLora{});
    else if (dtype == FLP_F16)
      hipLaunchKernelGGL((gemm_nt256_kernel<GF16, false, false>), grid256, dim3(256), kGStages * kGStage, stream, xs, ld_x,
                         ws, none, (uint16_t*)y, ld_y, y32, M, N, K, tiles_n, tiles_m, groups_n, FlpGemmLora{}, FlpGemmLora{});
    else
      hipLaunchKernelGGL((gemm_nt256_kernel<GBF16, false, false>), grid256, dim3(256), kGStages * kGStage, stream, xs,
                         ld_x, ws, none, (uint16_t*)y, ld_y, y32, M, N, K, tiles_n, tiles_m, groups_n, FlpGemmLora{}, FlpGemmLora{});
    FLP_TRY_HIP(hipGetLastError());
    return FLP_OK;
  }
  // few tiles (decode batches): split the contraction over up to 8 slices until about 256 workgroups run
  const int tiles = ((N + BN - 1) / BN) * ((M + BM - 1) / BM);
  int slices = 1;
  while (slices < 8 && tiles * slices < 192 && (K / BK) % (slices * 2) == 0 && K / (slices * 2) >= 512 &&
         splitk_scratch && (size_t)slices * 2 * M * N * 4 <= splitk_bytes)
    slices *= 2;
  dim3 grid((N + BN - 1) / BN, (M + BM - 1) / BM, slices);
  if (dtype == FLP_F16)
    hipLaunchKernelGGL(gemm_nt_kernel<GF16>, grid, dim3(256), 0, stream, xs, ld_x, ws, (uint16_t*)y, ld_y, y32, M, N, K,
                       splitk_scratch);
  else
    hipLaunchKernelGGL(gemm_nt_kernel<GBF16>, grid, dim3(256), 0, stream, xs, ld_x, ws, (uint16_t*)y, ld_y, y32, M, N,
                       K, splitk_scratch);
  FLP_TRY_HIP(hipGetLastError());
  if (slices > 1) {
    const unsigned nb = (unsigned)(((int64_t)M * N + 255) / 256);
    if (dtype == FLP_F16)
      hipLaunchKernelGGL(gemm_splitk_reduce_kernel<GF16>, dim3(nb), dim3(256), 0, stream, splitk_scratch, slices, M, N,
                         (uint16_t*)y, ld_y, y32);
    else
      hipLaunchKernelGGL(gemm_splitk_reduce_kernel<GBF16>, dim3(nb), dim3(256), 0, stream, splitk_scratch, slices, M, N,
                         (uint16_t*)y, ld_y, y32);
    FLP_TRY_HIP(hipGetLastError());
  }
  return FLP_OK;
}
