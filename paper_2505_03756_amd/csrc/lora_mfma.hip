// Batched heterogeneous LoRA on the matrix cores, for 16-bit pools (paper Eq. 1 / Eq. 2 in
// row-vector form, y = base + s (x A^T) B; section 2.1: tokens of different adapters share
// one batch; section 4.3: adapters live in pool blocks as rank rows).
//
// Tokens are first grouped by adapter (lora.hip); a tile is up to 16*MT consecutive tokens
// of one adapter.  Both kernels read their operands straight from global memory in MFMA
// operand layout: the rank-major page rows make 8 consecutive coefficients of one rank one
// 16-byte run, which is exactly a lane's share of a 16x16x32 operand, so nothing is staged
// or transposed in LDS and every page byte is fetched once per tile.
//
//   shrink  v[t, rho] = sum_c x[t,c] A[rho,c]     M = tokens, N = ranks, K = d_in.  K is
//           split over the 4 waves of a workgroup (summed in LDS in a fixed order) and over
//           KS workgroups (partial sums in global memory, added in order by the expand
//           kernel), so that enough waves are in flight to stream x at HBM rate.
//   expand  y[t, o] += s sum_rho v[t,rho] B[rho,o]   computed transposed, M = columns,
//           N = tokens, K = ranks.  v stays fp32: it is split into a 16-bit high part and
//           a 16-bit remainder that occupy the two halves of the K = 32 contraction (the
//           B coefficients are fed to both halves).  Two column tiles are interleaved so
//           that a lane ends up with 8 consecutive columns of one token: y is read and
//           written in 16-byte pieces.
#include <atomic>
#include <hip/hip_runtime.h>

#include "flp_internal.h"
#include "flp_types.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 h16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 b16x8 __attribute__((ext_vector_type(8)));

struct LF16 {
  typedef h16x8 vec;
  typedef F16 S;
  static __device__ __forceinline__ f32x4 mfma(vec a, vec b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ void split(float v, _Float16* hi, _Float16* lo) {
    *hi = (_Float16)v;
    *lo = (_Float16)(v - (float)*hi);
  }
  typedef _Float16 elem;
};
struct LBF16 {
  typedef b16x8 vec;
  typedef BF16 S;
  static __device__ __forceinline__ f32x4 mfma(vec a, vec b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ void split(float v, __bf16* hi, __bf16* lo) {
    *hi = (__bf16)v;
    *lo = (__bf16)(v - (float)*hi);
  }
  typedef __bf16 elem;
};

template <typename V>
__device__ __forceinline__ V vec_from(u32x4 r) {
  V v;
  __builtin_memcpy(&v, &r, 16);
  return v;
}

// tile -> segment: largest s with tile_start[s] <= tile (tile < tile_start[n_seg])
__device__ __forceinline__ int find_segment(const int32_t* __restrict__ tile_start, int n_seg, int tile) {
  int lo = 0, hi = n_seg;   // invariant: tile_start[lo] <= tile < tile_start[hi]
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (tile_start[mid] <= tile) lo = mid; else hi = mid;
  }
  return lo;
}

// ------------------------------------------------------------------------------- shrink
// ONEP: a workgroup takes ONE projection of its tile (the grid grows by the number of projections): with
// rank tiles NT >= 2 the accumulators and operand fragments of three projections at once leave one
// wave per SIMD, and the kernel, which lives on loads in flight, then runs at a fraction of HBM rate; x is
// re-read per projection, from L2.
template <typename L, int MT, int NT, bool ONEP>
__global__ __launch_bounds__(256) void lora_shrink_mfma_kernel(FlpLoraArgs a, FlpLoraMfma c) {
  typedef typename L::vec vec;
  constexpr int NPJ = ONEP ? 1 : FLP_MAX_PROJ;         // projections held by this workgroup
  extern __shared__ float red[];                       // [4 waves][n_acc][64 lanes]
  // Each XCD (workgroups are placed on the 8 XCDs round-robin by their linear id) takes a contiguous
  // eighth of the tiles with all their k splits: tiles of one adapter are neighbours, so its A pages
  // are fetched into one L2 instead of eight.  The launch covers gridDim.x / (8 k_splits) tiles per XCD
  // in one pass; with more segments than the host allowed for, a workgroup takes several tiles in turn.
  const int n_seg = *a.n_seg;
  const int n_tiles = a.tile_start[n_seg];
  const int per_xcd = (n_tiles + 7) / 8;
  const int per_tile = c.k_splits * (ONEP ? a.n_proj : 1);          // workgroups per tile
  const int ks = ((blockIdx.x >> 3) % per_tile) / (ONEP ? a.n_proj : 1);
  const int p_first = ONEP ? ((blockIdx.x >> 3) % per_tile) % a.n_proj : 0;   // local projection q is p_first + q
  const int n_pl = ONEP ? 1 : a.n_proj;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, row = lane & 15, kg = lane >> 4;
  const uint16_t* __restrict__ pool = reinterpret_cast<const uint16_t*>(a.pool);
  const int rpb = (int)(a.block_elems / a.d_in);
  for (int lt = (blockIdx.x >> 3) / per_tile; lt < per_xcd; lt += (gridDim.x >> 3) / per_tile) {
  const int tile = (blockIdx.x & 7) * per_xcd + lt;
  if (tile >= n_tiles) break;
  const int s = find_segment(a.tile_start, n_seg, tile);
  const int ad = a.seg_adapter[s];
  const int r = a.rank[ad] < a.max_rank ? a.rank[ad] : a.max_rank;
  const int TM = 16 * MT;
  const int pos0 = a.seg_start[s] + (tile - a.tile_start[s]) * TM;
  const int pos_end = a.seg_start[s + 1];

  const uint16_t* xp[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    int pos = pos0 + 16 * mt + row;
    pos = pos < pos_end ? pos : pos_end - 1;           // padding rows repeat the last token
    xp[mt] = reinterpret_cast<const uint16_t*>(a.x) + (int64_t)a.perm[pos] * a.ld_x + 8 * kg;
  }
  const uint16_t* ap[NPJ][NT];
  bool avalid[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) avalid[nt] = 16 * nt + row < r;
#pragma unroll
  for (int p = 0; p < NPJ; ++p)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      ap[p][nt] = pool;
      if (p < n_pl && r > 0) {
        const flp_lora_proj& pr = a.proj[p_first + p];
        const int i = pr.a_row_base[ad] + (avalid[nt] ? 16 * nt + row : 0);
        ap[p][nt] = pool + (int64_t)a.tables[pr.a_tab_off[ad] + i / rpb] * a.block_elems +
                    (int64_t)(i % rpb) * a.d_in + 8 * kg;
      }
    }

  f32x4 acc[MT][NPJ][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int p = 0; p < NPJ; ++p)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) acc[mt][p][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int kbeg = ks * c.k_per_split;
  const int kend = kbeg + c.k_per_split < a.d_in ? kbeg + c.k_per_split : a.d_in;
  const u32x4 zero4 = {0u, 0u, 0u, 0u};
  for (int c0 = kbeg + 32 * wave; c0 < kend; c0 += 128) {
    vec xf[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) xf[mt] = vec_from<vec>(*reinterpret_cast<const u32x4*>(xp[mt] + c0));
#pragma unroll
    for (int p = 0; p < NPJ; ++p) {
      if (p < n_pl) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          if (16 * nt < r) {
            u32x4 raw = avalid[nt] ? *reinterpret_cast<const u32x4*>(ap[p][nt] + c0) : zero4;
            vec af = vec_from<vec>(raw);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[mt][p][nt] = L::mfma(xf[mt], af, acc[mt][p][nt]);
          }
        }
      }
    }
  }

  // ---- sum the four waves' partial tiles in a fixed order, then store
  const int n_acc = MT * n_pl * NT * 4;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int p = 0; p < NPJ; ++p)
      if (p < n_pl)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int i = 0; i < 4; ++i)
            red[(wave * n_acc + ((mt * n_pl + p) * NT + nt) * 4 + i) * 64 + lane] = acc[mt][p][nt][i];
  __syncthreads();
  const int RP = 16 * NT;
  float* __restrict__ vout = a.v + ((int64_t)ks * c.v_rows + (int64_t)tile * TM) * a.n_proj * RP;
  for (int e = tid; e < n_acc * 64; e += 256) {
    const float sum = ((red[e] + red[n_acc * 64 + e]) + red[2 * n_acc * 64 + e]) + red[3 * n_acc * 64 + e];
    const int ln = e & 63, q = e >> 6;
    const int i = q & 3, nt = (q >> 2) % NT, p = ((q >> 2) / NT) % n_pl, mt = (q >> 2) / (NT * n_pl);
    const int trow = 16 * mt + (ln >> 4) * 4 + i, rho = 16 * nt + (ln & 15);
    vout[((int64_t)trow * a.n_proj + p_first + p) * RP + rho] = sum;
  }
  __syncthreads();                                     // the next tile reuses the reduction buffer
  }
}

// ------------------------------------------------------------------------------- shrink, ranks above 16
// The kernel above reads its operands straight from global memory in MFMA layout: 64-byte pieces of 16 rows
// per instruction.  With 2 or 4 rank tiles per token tile that is mostly A traffic from L2 in 64-byte
// requests, and the kernel runs far below the rate of the x stream.  Here a workgroup of four waves owns one
// (32-token tile, projection, k split) and walks its k range in chunks of 64 coefficients: the chunk's x
// rows (32 x 128 bytes) and A rows (16 NT x 128 bytes) travel as whole 128-byte lines into a ring of four LDS
// stages with direct global-to-LDS loads (inline assembly, own s_waitcnt vmcnt; three chunks ahead), slots
// XOR-swizzled by the row on the global side, and the waves split the (token tile, rank tile) pairs, so
// no reduction across waves is needed.  Ranks past the adapter's rank read the adapter's first row: their v
// entries are finite and meet zero coefficients in the expand kernel.
typedef __attribute__((address_space(3))) uint8_t l_lds_u8;
// M0 is named as clobbered so that no pass keeps a value of its own alive in it across the statement; the
// compiler notes that it reserves the register, which is the point.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void lload_lds16(uint64_t addr, uint32_t lds) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(addr), "s"(lds) : "memory", "m0");
}
#pragma clang diagnostic pop
constexpr int lvmcnt(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }   // s_waitcnt vmcnt(n) only

template <typename L, int NT, int NPJ>
__global__ __launch_bounds__(256) void lora_shrink_lds_kernel(FlpLoraArgs a, FlpLoraMfma c) {
  typedef typename L::vec vec;
  // From rank 33 on a workgroup takes TWO neighbouring 32-token tiles of a segment (the first of each pair does
  // the work, the second exits): the adapter's A rows, which at rank 64 are twice the bytes of a 32-token x tile,
  // are then fetched once per 64 tokens (34B shapes: q,k,v call 1.47 -> 1.25 ms; at rank 32 it does not pay).
  // NPJ = 2, 3 (used with two rank tiles): the projections of the call are fused (their A rows sit behind each
  // other in a stage, x is fetched once for all of them); NPJ = 1: one projection per workgroup, taken from the
  // grid.
  constexpr int XT = NT >= 4 ? 4 : 2;                  // 16-token tiles per workgroup
  constexpr int kS = 4;                                // ring stages
  constexpr int kXB = 2048 * XT;                       // bytes of the x rows of a stage
  constexpr int kAB = 2048 * NT;                       // bytes of one projection's A rows
  constexpr int kStageB = kXB + NPJ * kAB;             // x rows, then A rows, 128 bytes each
  constexpr int NINS = 2 * XT + 2 * NT * NPJ;          // 1 KiB load instructions per chunk (8 rows each)
  static_assert(NINS % 4 == 0, "the waves share the load instructions of a chunk evenly");
  constexpr int NPER = NINS / 4;                       // of which each wave issues this many
  constexpr int NP = XT * NT * NPJ / 4;                // (projection, 16-token tile, rank tile) triples per wave
  static_assert(kS * kStageB <= 65536, "the ring fits the LDS of a static array");
  __shared__ __attribute__((aligned(1024))) uint8_t smem[kS * kStageB];
  const int n_seg = *a.n_seg;
  const int n_tiles = a.tile_start[n_seg];
  const int per_xcd = (n_tiles + 7) / 8;
  const int per_tile = c.k_splits * (NPJ == 1 ? a.n_proj : 1);
  const int ks = NPJ == 1 ? ((blockIdx.x >> 3) % per_tile) / a.n_proj : (blockIdx.x >> 3) % per_tile;
  const int p0 = NPJ == 1 ? ((blockIdx.x >> 3) % per_tile) % a.n_proj : 0;       // first (only) projection of this workgroup
  const int tid = threadIdx.x, lane = tid & 63, row16 = lane & 15, kg = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint16_t* __restrict__ pool = reinterpret_cast<const uint16_t*>(a.pool);
  const int rpb = (int)(a.block_elems / a.d_in);
  const uint32_t lds0 = (uint32_t)(uintptr_t)(l_lds_u8*)smem;
  for (int lt = (blockIdx.x >> 3) / per_tile; lt < per_xcd; lt += (gridDim.x >> 3) / per_tile) {
    const int tile = (blockIdx.x & 7) * per_xcd + lt;
    if (tile >= n_tiles) break;
    const int s = find_segment(a.tile_start, n_seg, tile);
    if (XT == 4 && ((tile - a.tile_start[s]) & 1)) continue;     // the second tile of a pair: its neighbour does it
    const bool second = XT == 4 && tile + 1 < a.tile_start[s + 1];  // the pair is complete
    const int ad = a.seg_adapter[s];
    const int r = a.rank[ad] < a.max_rank ? a.rank[ad] : a.max_rank;
    const int pos0 = a.seg_start[s] + (tile - a.tile_start[s]) * 32;
    const int pos_end = a.seg_start[s + 1];
    const int kbeg = ks * c.k_per_split;
    const int kend = kbeg + c.k_per_split < a.d_in ? kbeg + c.k_per_split : a.d_in;
    const int n_chunks = r > 0 ? (kend - kbeg) / 64 : 0;

    // ---- this lane's rows of the load instructions it issues: instruction j = wave + 4 i covers rows
    //      8 j .. 8 j + 7 of the x rows (j < 2 XT) or, for jj = j - 2 XT, rows 8 (jj % 2 NT) .. of the A tile of
    //      projection jj / 2 NT; lane l holds row l / 8, LDS slot l % 8, i.e. the row's logical 16-byte piece
    //      (l % 8) ^ (row % 8)
    uint64_t gaddr[NPER];
    uint32_t ldst[NPER];
#pragma unroll
    for (int i = 0; i < NPER; ++i) {
      const int j = wave + 4 * i, rl = lane >> 3;
      const uint16_t* rowp;
      int rowi;
      if (j < 2 * XT) {
        rowi = 8 * j + rl;
        int pos = pos0 + rowi;
        pos = pos < pos_end ? pos : pos_end - 1;       // padding rows repeat the last token
        rowp = reinterpret_cast<const uint16_t*>(a.x) + (int64_t)a.perm[pos] * a.ld_x;
        ldst[i] = 1024u * j;
      } else {
        const int jj = j - 2 * XT, pj = jj / (2 * NT), jr = jj % (2 * NT);
        const flp_lora_proj& pr = a.proj[p0 + pj];
        rowi = 8 * jr + rl;
        rowp = pool;
        if (r > 0) {
          const int ii = pr.a_row_base[ad] + (rowi < r ? rowi : 0);
          rowp = pool + (int64_t)a.tables[pr.a_tab_off[ad] + ii / rpb] * a.block_elems + (int64_t)(ii % rpb) * a.d_in;
        }
        ldst[i] = (uint32_t)(kXB + pj * kAB) + 1024u * jr;
      }
      gaddr[i] = (uint64_t)(uintptr_t)(rowp + kbeg + 8 * ((lane & 7) ^ (rowi & 7)));
    }
    auto issue_chunk = [&](int t) {
      const int tc = t < n_chunks ? t : n_chunks - 1;   // past the end: the last chunk again, into a free stage
      const uint32_t dst = lds0 + (uint32_t)(t & (kS - 1)) * kStageB;
#pragma unroll
      for (int i = 0; i < NPER; ++i) lload_lds16(gaddr[i] + (uint64_t)tc * 128, dst + ldst[i]);
    };

    f32x4 acc[NP];
    int offx[NP], offa[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
      const int pi = wave + 4 * i, pj = pi / (XT * NT), mt = (pi % (XT * NT)) / NT, nt = pi % NT;
      const int xr = 16 * mt + row16, ar = 16 * nt + row16;
      offx[i] = xr * 128 + ((kg ^ (xr & 7)) << 4);                 // k step 0; step 1 is slot + 4: offset ^ 64
      offa[i] = kXB + pj * kAB + ar * 128 + ((kg ^ (ar & 7)) << 4);
    }

    __builtin_amdgcn_s_waitcnt(lvmcnt(0));             // the loads above are in: only chunk loads are in flight below
    __syncthreads();                                   // the previous item's stages are no longer read
    if (n_chunks > 0) {
#pragma unroll
      for (int t = 0; t < kS - 1; ++t) issue_chunk(t);
    }
    for (int kt = 0; kt < n_chunks; ++kt) {
      __builtin_amdgcn_s_waitcnt(lvmcnt(2 * NPER));    // chunk kt has landed (kt + 1 and kt + 2 may be in flight)
      __syncthreads();
      issue_chunk(kt + kS - 1);
      const uint8_t* buf = smem + (kt & (kS - 1)) * kStageB;
#pragma unroll
      for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
        for (int i = 0; i < NP; ++i) {
          const vec xf = *reinterpret_cast<const vec*>(buf + (offx[i] ^ (k2 << 6)));
          const vec af = *reinterpret_cast<const vec*>(buf + (offa[i] ^ (k2 << 6)));
          acc[i] = L::mfma(xf, af, acc[i]);
        }
    }
    __builtin_amdgcn_s_waitcnt(lvmcnt(0));             // look-ahead loads past the last chunk must land before the ring is reused

    // lane (rank column n = lane % 16, token rows 4 kg .. 4 kg + 3) of each triple; the rows of the pair's second
    // tile follow the first one's in v
    const int RP = 16 * NT;
    float* __restrict__ vout = a.v + ((int64_t)ks * c.v_rows + (int64_t)tile * 32) * a.n_proj * RP;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const int pi = wave + 4 * i, pj = pi / (XT * NT), mt = (pi % (XT * NT)) / NT, nt = pi % NT;
      if (mt >= 2 && !second) continue;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        vout[((int64_t)(16 * mt + 4 * kg + e) * a.n_proj + p0 + pj) * RP + 16 * nt + row16] = acc[i][e];
    }
  }
}

// The same staging for ranks up to 16, where the projections of a call are fused: the A rows of all NPJ
// projections (16 rank rows each) sit behind the 32 x rows of a chunk, x is fetched once for all of them,
// and the waves split the (token tile, projection) pairs.  When the load instructions of a chunk do not
// divide by four, a wave repeats one of its own loads, so that every wave has the same number in flight.
template <typename L, int NPJ>
__global__ __launch_bounds__(256) void lora_shrink_lds16_kernel(FlpLoraArgs a, FlpLoraMfma c) {
  typedef typename L::vec vec;
  constexpr int kS = 4;
  constexpr int kStageB = 4096 + 2048 * NPJ;
  constexpr int NINS = 4 + 2 * NPJ;
  constexpr int NPER = (NINS + 3) / 4;
  constexpr int NP = (2 * NPJ + 3) / 4;
  __shared__ __attribute__((aligned(1024))) uint8_t smem[kS * kStageB];
  const int n_seg = *a.n_seg;
  const int n_tiles = a.tile_start[n_seg];
  const int per_xcd = (n_tiles + 7) / 8;
  const int ks = (blockIdx.x >> 3) % c.k_splits;
  const int tid = threadIdx.x, lane = tid & 63, row16 = lane & 15, kg = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint16_t* __restrict__ pool = reinterpret_cast<const uint16_t*>(a.pool);
  const int rpb = (int)(a.block_elems / a.d_in);
  const uint32_t lds0 = (uint32_t)(uintptr_t)(l_lds_u8*)smem;
  for (int lt = (blockIdx.x >> 3) / c.k_splits; lt < per_xcd; lt += (gridDim.x >> 3) / c.k_splits) {
    const int tile = (blockIdx.x & 7) * per_xcd + lt;
    if (tile >= n_tiles) break;
    const int s = find_segment(a.tile_start, n_seg, tile);
    const int ad = a.seg_adapter[s];
    const int r = a.rank[ad] < a.max_rank ? a.rank[ad] : a.max_rank;
    const int pos0 = a.seg_start[s] + (tile - a.tile_start[s]) * 32;
    const int pos_end = a.seg_start[s + 1];
    const int kbeg = ks * c.k_per_split;
    const int kend = kbeg + c.k_per_split < a.d_in ? kbeg + c.k_per_split : a.d_in;
    const int n_chunks = r > 0 ? (kend - kbeg) / 64 : 0;

    uint64_t gaddr[NPER];
    uint32_t ldst[NPER];
#pragma unroll
    for (int i = 0; i < NPER; ++i) {
      int j = wave + 4 * i;
      if (j >= NINS) j -= 4;                           // no such instruction: this wave's previous one again
      const int rl = lane >> 3;
      const uint16_t* rowp;
      int rowi;
      if (j < 4) {
        rowi = 8 * j + rl;
        int pos = pos0 + rowi;
        pos = pos < pos_end ? pos : pos_end - 1;       // padding rows repeat the last token
        rowp = reinterpret_cast<const uint16_t*>(a.x) + (int64_t)a.perm[pos] * a.ld_x;
        ldst[i] = 1024u * j;
      } else {
        const int pj = (j - 4) >> 1;                   // projection whose A rows this instruction moves
        rowi = 8 * ((j - 4) & 1) + rl;                 // rank row
        rowp = pool;
        if (r > 0) {
          const flp_lora_proj& pr = a.proj[pj];
          const int ii = pr.a_row_base[ad] + (rowi < r ? rowi : 0);
          rowp = pool + (int64_t)a.tables[pr.a_tab_off[ad] + ii / rpb] * a.block_elems + (int64_t)(ii % rpb) * a.d_in;
        }
        ldst[i] = 4096u + 1024u * (j - 4);
      }
      gaddr[i] = (uint64_t)(uintptr_t)(rowp + kbeg + 8 * ((lane & 7) ^ (rowi & 7)));
    }
    auto issue_chunk = [&](int t) {
      const int tc = t < n_chunks ? t : n_chunks - 1;
      const uint32_t dst = lds0 + (uint32_t)(t & (kS - 1)) * kStageB;
#pragma unroll
      for (int i = 0; i < NPER; ++i) lload_lds16(gaddr[i] + (uint64_t)tc * 128, dst + ldst[i]);
    };

    f32x4 acc[NP];
    int offx[NP], offa[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
      int pi = wave + 4 * i;
      pi = pi < 2 * NPJ ? pi : 0;                      // no such pair: pair 0 again, not stored
      const int mt = pi / NPJ, pj = pi % NPJ;
      const int xr = 16 * mt + row16, ar = 16 * pj + row16;
      offx[i] = xr * 128 + ((kg ^ (xr & 7)) << 4);
      offa[i] = 4096 + ar * 128 + ((kg ^ (ar & 7)) << 4);
    }

    __builtin_amdgcn_s_waitcnt(lvmcnt(0));
    __syncthreads();
    if (n_chunks > 0) {
#pragma unroll
      for (int t = 0; t < kS - 1; ++t) issue_chunk(t);
    }
    for (int kt = 0; kt < n_chunks; ++kt) {
      __builtin_amdgcn_s_waitcnt(lvmcnt(2 * NPER));
      __syncthreads();
      issue_chunk(kt + kS - 1);
      const uint8_t* buf = smem + (kt & (kS - 1)) * kStageB;
#pragma unroll
      for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
        for (int i = 0; i < NP; ++i) {
          const vec xf = *reinterpret_cast<const vec*>(buf + (offx[i] ^ (k2 << 6)));
          const vec af = *reinterpret_cast<const vec*>(buf + (offa[i] ^ (k2 << 6)));
          acc[i] = L::mfma(xf, af, acc[i]);
        }
    }
    __builtin_amdgcn_s_waitcnt(lvmcnt(0));

    float* __restrict__ vout = a.v + ((int64_t)ks * c.v_rows + (int64_t)tile * 32) * a.n_proj * 16;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const int pi = wave + 4 * i;
      if (pi < 2 * NPJ) {
        const int mt = pi / NPJ, pj = pi % NPJ;
#pragma unroll
        for (int e = 0; e < 4; ++e) vout[((int64_t)(16 * mt + 4 * kg + e) * a.n_proj + pj) * 16 + row16] = acc[i][e];
      }
    }
  }
}

// ------------------------------------------------------------------------------- expand
// One wave per (tile group, column slab, projection).  The slab's B coefficients are gathered
// once into MFMA A-operand fragments that stay in registers (64 VGPRs) while the wave walks
// the group's 16-token sub-tiles, so the 2-byte gathers are amortised over up to 256 tokens
// and the inner loop is the y stream: 16-byte read, two MFMAs per rank tile, 16-byte write.
template <typename L, int NT>
__global__ __launch_bounds__(64) void lora_expand_mfma_kernel(FlpLoraArgs a, FlpLoraMfma c) {
  typedef typename L::vec vec;
  typedef typename L::elem elem;
  typedef typename L::S S;
  constexpr int CH = 8 / NT;                          // 32-column chunks per resident piece
  // All column slabs and projections of one tile group run on one XCD (workgroups are placed on the
  // 8 XCDs round-robin by their linear id): they re-read the same rows of v and the same B pages,
  // which then stay in that XCD's L2.
  const int per_group = c.slabs * a.n_proj;
  const int n_seg = *a.n_seg;
  const int n_groups = a.group_start[n_seg];
  const int q_total = (n_groups + 7) / 8 * per_group;
  const int xcd = blockIdx.x & 7;
  const int lane = threadIdx.x, n = lane & 15, kg = lane >> 4, kq = kg & 1, lo_half = kg >> 1, m = lane & 15;
  const uint16_t* __restrict__ pool = reinterpret_cast<const uint16_t*>(a.pool);
  // the launch covers gridDim.x / 8 (group, slab, projection) items per XCD in one pass; with more segments
  // than the host allowed for, a wave takes several items in turn
  for (int q = blockIdx.x >> 3; q < q_total; q += gridDim.x >> 3) {
  const int group = (q / per_group) * 8 + xcd, slab = (q % per_group) / a.n_proj, p = (q % per_group) % a.n_proj;
  if (group >= n_groups) continue;
  const flp_lora_proj& pr = a.proj[p];
  const int slab_begin = slab * c.cols_per_slab;
  if (slab_begin >= pr.d_out) continue;
  const int s = find_segment(a.group_start, n_seg, group);
  const int ad = a.seg_adapter[s];
  const int r = a.rank[ad] < a.max_rank ? a.rank[ad] : a.max_rank;
  if (r <= 0) continue;
  const float sc = a.scale[ad];
  const int RP = 16 * NT, TM = 16 * c.mt;
  const int off0 = (group - a.group_start[s]) * c.group_tokens;       // first token of the group inside its segment
  const int pos0 = a.seg_start[s] + off0;
  const int pos_end = a.seg_start[s + 1];
  const int pos_stop = pos0 + c.group_tokens < pos_end ? pos0 + c.group_tokens : pos_end;
  const int64_t vrow0 = (int64_t)a.tile_start[s] * TM + off0;         // the segment's rows of v are contiguous
  const int rpb = (int)(a.block_elems / pr.d_out);

  // page rows of B for this lane's 8 ranks of every rank tile
  const uint16_t* rowp[NT][8];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int rho = 16 * nt + 8 * kq + j;
      const int i = pr.b_row_base[ad] + (rho < r ? rho : 0);
      rowp[nt][j] = pool + (int64_t)a.tables[pr.b_tab_off[ad] + i / rpb] * a.block_elems + (int64_t)(i % rpb) * pr.d_out;
    }

  // the slab's columns in pieces of 64*C64, so that the resident fragments stay at 64 registers
  constexpr int C64 = CH / 2;                         // 64-column chunks per piece
  for (int col_begin = slab_begin; col_begin < slab_begin + c.cols_per_slab && col_begin < pr.d_out;
       col_begin += 64 * C64) {
    // ---- A operand: B[rho, col].  Four column tiles of a 64-column chunk are interleaved: row m of
    //      tile tau is column 16*(m/4) + 4*tau + m%4, so a lane's 16 results are 16 consecutive columns
    //      (32 bytes) and the four lanes of a token row cover one full 128-byte line of y.
    vec bf[C64][4][NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int ch = 0; ch < C64; ++ch)
#pragma unroll
        for (int tau = 0; tau < 4; ++tau) {
          const int col = col_begin + 64 * ch + 16 * (m >> 2) + 4 * tau + (m & 3);
          const int colc = col < pr.d_out ? col : pr.d_out - 1;
          uint16_t g8[8];
          // unconditional loads (padding ranks point at a real row), zeroed afterwards: no
          // divergent branch around each 2-byte gather
#pragma unroll
          for (int j = 0; j < 8; ++j) g8[j] = rowp[nt][j][colc];
#pragma unroll
          for (int j = 0; j < 8; ++j)
            if (!(16 * nt + 8 * kq + j < r && col < pr.d_out)) g8[j] = 0;
          __builtin_memcpy(&bf[ch][tau][nt], g8, 16);
        }

    int tok = a.perm[pos0 + n < pos_stop ? pos0 + n : pos_stop - 1];
    for (int pos_t = pos0; pos_t < pos_stop; pos_t += 16) {
      const int pos = pos_t + n;
      const bool tvalid = pos < pos_stop;
      uint16_t* yrow = reinterpret_cast<uint16_t*>(pr.y) + (int64_t)tok * pr.ld_y + col_begin + 16 * kg;
      const float* brow = a.base32[p] ? a.base32[p] + (int64_t)tok * pr.d_out + col_begin + 16 * kg : nullptr;
      // the y pieces are requested first so that their latency overlaps the preparation of v;
      // the next sub-tile's token index is fetched now as well
      u32x4 yraw[C64][2];
#pragma unroll
      for (int ch = 0; ch < C64; ++ch)
        if (col_begin + 64 * ch < pr.d_out && !brow) {
          yraw[ch][0] = *reinterpret_cast<const u32x4*>(yrow + 64 * ch);
          yraw[ch][1] = *reinterpret_cast<const u32x4*>(yrow + 64 * ch + 8);
        }
      const int pos_n = pos + 16;
      const int tok_next = a.perm[pos_n < pos_stop ? pos_n : pos_stop - 1];
      // ---- B operand: this token's scaled v, high part in k-slots 0..15, remainder in 16..31
      vec vb[NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        float v8[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v8[j] = 0.f;
        if (16 * nt < r) {
          for (int ks = 0; ks < c.k_splits; ++ks) {
            const float* vp =
                a.v + (((int64_t)ks * c.v_rows + vrow0 + (pos - pos0)) * a.n_proj + p) * RP + 16 * nt + 8 * kq;
            const f32x4 x0 = *reinterpret_cast<const f32x4*>(vp), x1 = *reinterpret_cast<const f32x4*>(vp + 4);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              v8[j] += x0[j];
              v8[4 + j] += x1[j];
            }
          }
        }
        vec out;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          elem hi, lo;
          L::split(v8[j] * sc, &hi, &lo);
          out[j] = lo_half ? lo : hi;
        }
        vb[nt] = out;
      }
#pragma unroll
      for (int ch = 0; ch < C64; ++ch) {
        if (col_begin + 64 * ch < pr.d_out) {
          f32x4 acc[4];
#pragma unroll
          for (int tau = 0; tau < 4; ++tau) acc[tau] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            if (16 * nt < r) {
#pragma unroll
              for (int tau = 0; tau < 4; ++tau) acc[tau] = L::mfma(bf[ch][tau][nt], vb[nt], acc[tau]);
            }
          }
          if (tvalid) {
            uint16_t ys[16];
            if (brow) {                          // unrounded base from the dense projection
#pragma unroll
              for (int tau = 0; tau < 4; ++tau) {
                const f32x4 b4 = *reinterpret_cast<const f32x4*>(brow + 64 * ch + 4 * tau);
#pragma unroll
                for (int i = 0; i < 4; ++i) ys[4 * tau + i] = S::from_float(b4[i] + acc[tau][i]);
              }
            } else {
              __builtin_memcpy(ys, &yraw[ch][0], 32);
#pragma unroll
              for (int tau = 0; tau < 4; ++tau)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                  ys[4 * tau + i] = S::from_float(S::to_float(ys[4 * tau + i]) + acc[tau][i]);
            }
            u32x4 raw[2];
            __builtin_memcpy(raw, ys, 32);
            *reinterpret_cast<u32x4*>(yrow + 64 * ch) = raw[0];
            *reinterpret_cast<u32x4*>(yrow + 64 * ch + 8) = raw[1];
          }
        }
      }
      tok = tok_next;
    }
  }
  }
}

// ------------------------------------------------------------------------------- expand, ranks above 16
// With 2 or 4 rank tiles the register-resident fragments of the kernel above cover only 64-128 columns
// per gather, and every such piece re-reads the tokens' v rows (which grow with the rank as well): at rank
// 64 it runs at a seventh of the y stream's rate.  Here a workgroup of four waves owns one (tile group,
// 256-column slab, projection): the slab's B coefficients (up to 64 ranks x 256 columns) are read once,
// coalesced, and laid out in LDS transposed - [column][rank], 128 bytes per column - so that a lane's
// A-operand fragment (8 consecutive ranks of one column) is one 16-byte LDS read; each wave then takes
// every fourth 16-token sub-tile: v is loaded and split once per sub-tile for all 256 columns, and per
// 64-column chunk the wave reads y, 4 x NT fragments from LDS, multiplies and writes y back.
// LDS slot s (16 bytes: rank tile s / 2, half s % 2) of column c sits at c * 128 + ((s ^ f(c)) * 16) with
// f(c) = (c & 3) | ((c >> 4) & 1) << 2: the 8 lanes that read one slot of 8 different columns (the
// interleaved column order of the product) hit 8 different 16-byte bank groups.
template <typename L, int NT>
__global__ __launch_bounds__(256) void lora_expand_lds_kernel(FlpLoraArgs a, FlpLoraMfma c) {
  typedef typename L::vec vec;
  typedef typename L::elem elem;
  typedef typename L::S S;
  __shared__ __attribute__((aligned(16))) uint8_t bt_lds[256 * 128];
  const int per_group = c.slabs * a.n_proj;
  const int n_seg = *a.n_seg;
  const int n_groups = a.group_start[n_seg];
  const int q_total = (n_groups + 7) / 8 * per_group;
  const int xcd = blockIdx.x & 7;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int n = lane & 15, kg = lane >> 4, kq = kg & 1, lo_half = kg >> 1, m = lane & 15;
  const uint16_t* __restrict__ pool = reinterpret_cast<const uint16_t*>(a.pool);
  auto col_hash = [](int col) { return (col & 3) | (((col >> 4) & 1) << 2); };
  for (int q = blockIdx.x >> 3; q < q_total; q += gridDim.x >> 3) {
    const int group = (q / per_group) * 8 + xcd, slab = (q % per_group) / a.n_proj, p = (q % per_group) % a.n_proj;
    if (group >= n_groups) continue;
    const flp_lora_proj& pr = a.proj[p];
    const int slab_begin = slab * 256;
    if (slab_begin >= pr.d_out) continue;
    const int s = find_segment(a.group_start, n_seg, group);
    const int ad = a.seg_adapter[s];
    const int r = a.rank[ad] < a.max_rank ? a.rank[ad] : a.max_rank;
    if (r <= 0) continue;
    const float sc = a.scale[ad];
    const int RP = 16 * NT, TM = 16 * c.mt;
    const int off0 = (group - a.group_start[s]) * c.group_tokens;
    const int pos0 = a.seg_start[s] + off0;
    const int pos_end = a.seg_start[s + 1];
    const int pos_stop = pos0 + c.group_tokens < pos_end ? pos0 + c.group_tokens : pos_end;
    const int64_t vrow0 = (int64_t)a.tile_start[s] * TM + off0;
    const int rpb = (int)(a.block_elems / pr.d_out);

    // ---- stage the slab's B coefficients: thread -> (rank, 8 consecutive columns), 16-byte loads along the
    //      page rows, 2-byte stores into the transposed tile; ranks past r and columns past d_out hold zeros
    __syncthreads();                                   // the previous item's fragments are no longer read
    for (int it = tid; it < RP * 32; it += 256) {
      const int rho = it >> 5, c8 = (it & 31) * 8;     // 32 column octets per rank
      u32x4 raw = {0u, 0u, 0u, 0u};
      if (rho < r && slab_begin + c8 < pr.d_out) {
        const int i = pr.b_row_base[ad] + rho;
        raw = *reinterpret_cast<const u32x4*>(pool + (int64_t)a.tables[pr.b_tab_off[ad] + i / rpb] * a.block_elems +
                                              (int64_t)(i % rpb) * pr.d_out + slab_begin + c8);
      }
      uint16_t e8[8];
      __builtin_memcpy(e8, &raw, 16);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int col = c8 + j;
        *reinterpret_cast<uint16_t*>(bt_lds + col * 128 + (((rho >> 3) ^ col_hash(col)) << 4) + (rho & 7) * 2) = e8[j];
      }
    }
    __syncthreads();

    for (int pos_t = pos0 + 16 * wave; pos_t < pos_stop; pos_t += 64) {
      const int pos = pos_t + n;
      const bool tvalid = pos < pos_stop;
      const int tok = a.perm[tvalid ? pos : pos_stop - 1];
      uint16_t* yrow = reinterpret_cast<uint16_t*>(pr.y) + (int64_t)tok * pr.ld_y + slab_begin + 16 * kg;
      const float* brow = a.base32[p] ? a.base32[p] + (int64_t)tok * pr.d_out + slab_begin + 16 * kg : nullptr;
      // the y pieces of all four chunks are requested first, so that their latency overlaps the preparation of v
      // and four chunks per wave are in flight instead of one
      u32x4 yall[4][2];
      if (!brow) {
#pragma unroll
        for (int ch = 0; ch < 4; ++ch)
          if (slab_begin + 64 * ch < pr.d_out) {
            yall[ch][0] = *reinterpret_cast<const u32x4*>(yrow + 64 * ch);
            yall[ch][1] = *reinterpret_cast<const u32x4*>(yrow + 64 * ch + 8);
          }
      }
      // ---- B operand: this token's scaled v for all rank tiles, high part in k-slots 0..15, remainder in 16..31
      vec vb[NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        float v8[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v8[j] = 0.f;
        if (16 * nt < r) {
          for (int ks = 0; ks < c.k_splits; ++ks) {
            const float* vp =
                a.v + (((int64_t)ks * c.v_rows + vrow0 + (pos - pos0)) * a.n_proj + p) * RP + 16 * nt + 8 * kq;
            const f32x4 x0 = *reinterpret_cast<const f32x4*>(vp), x1 = *reinterpret_cast<const f32x4*>(vp + 4);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              v8[j] += x0[j];
              v8[4 + j] += x1[j];
            }
          }
        }
        vec out;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          elem hi, lo;
          L::split(v8[j] * sc, &hi, &lo);
          out[j] = lo_half ? lo : hi;
        }
        vb[nt] = out;
      }
#pragma unroll
      for (int ch = 0; ch < 4; ++ch) {
        if (slab_begin + 64 * ch >= pr.d_out) continue;
        f32x4 acc[4];
#pragma unroll
        for (int tau = 0; tau < 4; ++tau) {
          acc[tau] = f32x4{0.f, 0.f, 0.f, 0.f};
          // row m of column tile tau is column 16*(m/4) + 4*tau + m%4 of the chunk: a lane's 16 results are 16
          // consecutive columns and the four lanes of a token row cover one 128-byte line of y
          const int col = 64 * ch + 16 * (m >> 2) + 4 * tau + (m & 3);
          const uint8_t* frow = bt_lds + col * 128;
          const int hsh = col_hash(col);
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
            if (16 * nt < r)
              acc[tau] = L::mfma(*reinterpret_cast<const vec*>(frow + (((2 * nt + kq) ^ hsh) << 4)), vb[nt], acc[tau]);
        }
        if (tvalid) {
          uint16_t ys[16];
          if (brow) {                            // unrounded base from the dense projection
#pragma unroll
            for (int tau = 0; tau < 4; ++tau) {
              const f32x4 b4 = *reinterpret_cast<const f32x4*>(brow + 64 * ch + 4 * tau);
#pragma unroll
              for (int i = 0; i < 4; ++i) ys[4 * tau + i] = S::from_float(b4[i] + acc[tau][i]);
            }
          } else {
            __builtin_memcpy(ys, &yall[ch][0], 32);
#pragma unroll
            for (int tau = 0; tau < 4; ++tau)
#pragma unroll
              for (int i = 0; i < 4; ++i) ys[4 * tau + i] = S::from_float(S::to_float(ys[4 * tau + i]) + acc[tau][i]);
          }
          u32x4 raw2[2];
          __builtin_memcpy(raw2, ys, 32);
          *reinterpret_cast<u32x4*>(yrow + 64 * ch) = raw2[0];
          *reinterpret_cast<u32x4*>(yrow + 64 * ch + 8) = raw2[1];
        }
      }
    }
  }
}

template <typename L, int MT, int NT>
flp_status launch_pair(const FlpLoraArgs& a, const FlpLoraMfma& c, hipStream_t stream) {
  constexpr bool ONEP = NT >= 2;                       // one projection per workgroup from rank 17 on
  const int n_pl = ONEP ? 1 : a.n_proj;
  const size_t smem = (size_t)4 * MT * n_pl * NT * 4 * 64 * sizeof(float);
  static std::atomic<bool> attr_set{false};   // pools on different threads share it
  if (!attr_set.load(std::memory_order_acquire)) {
    FLP_TRY_HIP(hipFuncSetAttribute((const void*)lora_shrink_mfma_kernel<L, MT, NT, ONEP>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
    attr_set.store(true, std::memory_order_release);
  }
  bool staged = false;
  if constexpr (NT >= 2 && MT == 2) {
    if (a.d_in % 64 == 0) {
      // two rank tiles: the projections of a call with two or three of them are fused (13B shapes, q,k,v call:
      // 0.89 -> 0.86 ms); with four rank tiles the fused stages leave one workgroup per CU and the call takes
      // twice as long (34B shapes: 1.25 -> 2.35 ms; the same with a ring of four stages in 128 KiB of dynamic LDS: 1.35 ->
      // 2.38 ms), so there a workgroup keeps to one projection
      constexpr int NPJ2 = NT == 2 ? 2 : 1, NPJ3 = NT == 2 ? 3 : 1;
      const dim3 gf((unsigned)(c.tiles_grid * c.k_splits));
      if (NT == 2 && a.n_proj == 2)
        hipLaunchKernelGGL((lora_shrink_lds_kernel<L, NT, NPJ2>), gf, dim3(256), 0, stream, a, c);
      else if (NT == 2 && a.n_proj == 3)
        hipLaunchKernelGGL((lora_shrink_lds_kernel<L, NT, NPJ3>), gf, dim3(256), 0, stream, a, c);
      else
        hipLaunchKernelGGL((lora_shrink_lds_kernel<L, NT, 1>), dim3((unsigned)(c.tiles_grid * c.k_splits * a.n_proj)),
                           dim3(256), 0, stream, a, c);
      staged = true;
    }
  }
  if constexpr (NT == 1 && MT == 2) {
    if (a.d_in % 64 == 0) {
      const dim3 g16((unsigned)(c.tiles_grid * c.k_splits));
      switch (a.n_proj) {
        case 1: hipLaunchKernelGGL((lora_shrink_lds16_kernel<L, 1>), g16, dim3(256), 0, stream, a, c); break;
        case 2: hipLaunchKernelGGL((lora_shrink_lds16_kernel<L, 2>), g16, dim3(256), 0, stream, a, c); break;
        case 3: hipLaunchKernelGGL((lora_shrink_lds16_kernel<L, 3>), g16, dim3(256), 0, stream, a, c); break;
        default: hipLaunchKernelGGL((lora_shrink_lds16_kernel<L, 4>), g16, dim3(256), 0, stream, a, c); break;
      }
      staged = true;
    }
  }
  if (!staged)
    hipLaunchKernelGGL((lora_shrink_mfma_kernel<L, MT, NT, ONEP>),
                       dim3((unsigned)(c.tiles_grid * c.k_splits * (ONEP ? a.n_proj : 1))), dim3(256), smem, stream, a, c);
  FLP_TRY_HIP(hipGetLastError());
  if (c.shrink_only) return FLP_OK;                     // the expand step is the dense product's epilogue
  int max_dout = 0;
  for (int p = 0; p < a.n_proj; ++p) max_dout = a.proj[p].d_out > max_dout ? a.proj[p].d_out : max_dout;
  FlpLoraMfma ce = c;
  ce.slabs = (max_dout + c.cols_per_slab - 1) / c.cols_per_slab;
  const int64_t n_wg = (int64_t)c.groups_grid * ce.slabs * a.n_proj;
  if (n_wg > INT32_MAX) {
    flp_set_error("LoRA (matrix-core path): %lld workgroups, too many for one launch", (long long)n_wg);
    return FLP_ENOTSUP;
  }
  if (NT >= 2 && c.cols_per_slab == 256)
    hipLaunchKernelGGL((lora_expand_lds_kernel<L, NT>), dim3((unsigned)n_wg), dim3(256), 0, stream, a, ce);
  else
    hipLaunchKernelGGL((lora_expand_mfma_kernel<L, NT>), dim3((unsigned)n_wg), dim3(64), 0, stream, a, ce);
  FLP_TRY_HIP(hipGetLastError());
  return FLP_OK;
}

template <typename L>
flp_status launch_dtype(const FlpLoraArgs& a, const FlpLoraMfma& c, hipStream_t stream) {
  const int nt = (a.max_rank + 15) / 16;
  if (c.mt == 2) {
    if (nt <= 1) return launch_pair<L, 2, 1>(a, c, stream);
    if (nt == 2) return launch_pair<L, 2, 2>(a, c, stream);
    return launch_pair<L, 2, 4>(a, c, stream);
  }
  if (nt <= 1) return launch_pair<L, 1, 1>(a, c, stream);
  if (nt == 2) return launch_pair<L, 1, 2>(a, c, stream);
  return launch_pair<L, 1, 4>(a, c, stream);
}

}  // namespace

flp_status flp_launch_lora_mfma(int dtype, const FlpLoraArgs& a, const FlpLoraMfma& c, hipStream_t stream) {
  if (dtype == FLP_F16) return launch_dtype<LF16>(a, c, stream);
  if (dtype == FLP_BF16) return launch_dtype<LBF16>(a, c, stream);
  flp_set_error("LoRA (matrix-core path): dtype %d not supported", dtype);
  return FLP_ENOTSUP;
}
