// Stand-alone probe of what bounds the matrix-core attention kernel on gfx950 (no memory traffic
// inside the timed loops, every access in bounds):
//   1. the per-wave instruction issue rate and how it scales with the waves per SIMD,
//   2. the attention tile loop (32 MFMA 32x32x16, 32 exp2, the softmax arithmetic of a 32-row x
//      64-key tile per wave, 8 waves per CU) held entirely in registers, on 32 and on 256 CUs,
//      with constant and with random operands: the difference is the clock the chip sustains,
//   3. where the 16-byte and 4-byte direct global-to-LDS loads put each lane's data (the
//      attention kernel's staging relies on: LDS base + size * lane, instruction offset 0).
// Build and run:  python -m paper_2505_03756_amd.probes
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <vector>

#define CHECK(x)                                                        \
  do {                                                                  \
    hipError_t e_ = (x);                                                \
    if (e_ != hipSuccess) {                                             \
      printf("%s failed: %s\n", #x, hipGetErrorString(e_));             \
      exit(1);                                                          \
    }                                                                   \
  } while (0)

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 h16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 h16x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) unsigned lds_u32;

// ---- 1. issue rate: 64 dependent-free fused multiply-adds (or exp2) per iteration and wave
template <int OP>
__global__ void issue_kernel(float* out, unsigned long long* clk, int iters) {
  const unsigned long long c0 = __builtin_readcyclecounter();
  float x[16];
  for (int j = 0; j < 16; ++j) x[j] = -0.001f * (threadIdx.x + j);
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int j = 0; j < 16; ++j) x[j] = OP == 0 ? fmaf(x[j], 0.999f, 0.5f) : __builtin_amdgcn_exp2f(x[j]);
  }
  float s = 0;
  for (int j = 0; j < 16; ++j) s += x[j];
  if (s == 123.456f) out[threadIdx.x] = s;
  if (threadIdx.x == 0 && blockIdx.x == 0) clk[0] = __builtin_readcyclecounter() - c0;
}

// ---- 2. the attention tile loop in registers
template <int RND>
__global__ void tile_loop_kernel(float* out, unsigned long long* clk, int iters, float c) {
  const unsigned long long c0 = __builtin_readcyclecounter();
  f32x16 S[2], O[4];
  h16x8 qa, qb;
  unsigned hsh = (threadIdx.x * 2654435761u) ^ (blockIdx.x * 40503u + 12345u);
  for (int j = 0; j < 8; ++j) {
    hsh = hsh * 1664525u + 1013904223u;
    qa[j] = RND ? (_Float16)(((int)(hsh >> 20) - 2048) * (1.0f / 2048.0f)) : (_Float16)(0.05f * j);
    hsh = hsh * 1664525u + 1013904223u;
    qb[j] = RND ? (_Float16)(((int)(hsh >> 20) - 2048) * (1.0f / 2048.0f)) : (_Float16)(0.02f * j);
  }
  for (int d = 0; d < 4; ++d)
    for (int i = 0; i < 16; ++i) O[d][i] = 0.f;
  float mrow = 0.5f, lsum = 0.f;
  h16x8 pb[2][2];
  for (int st = 0; st < 2; ++st)
    for (int h = 0; h < 2; ++h)
      for (int j = 0; j < 8; ++j) pb[st][h][j] = (_Float16)0.5f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      S[0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(qa, qb, kk == 0 ? f32x16{0} : S[0], 0, 0, 0);
      S[1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(qb, qa, kk == 0 ? f32x16{0} : S[1], 0, 0, 0);
    }
    float tmax = S[0][0];
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
      for (int i = 0; i < 16; ++i) tmax = fmaxf(tmax, S[st][i]);
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
    if (__builtin_amdgcn_ballot_w64((tmax - mrow) * c > 8.f)) {
      mrow = fmaxf(mrow, tmax);
      lsum *= 0.5f;
#pragma unroll
      for (int d = 0; d < 4; ++d)
#pragma unroll
        for (int i = 0; i < 16; ++i) O[d][i] *= 0.5f;
    }
    const float mc = mrow * c;
#pragma unroll
    for (int st = 0; st < 2; ++st) {
      float p[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) p[i] = __builtin_amdgcn_exp2f(fmaf(S[st][i], c, -mc));
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        h16x8 v;
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = (_Float16)p[8 * h + j];
        const h16x2 one = {(_Float16)1.f, (_Float16)1.f};
#pragma unroll
        for (int j = 0; j < 4; ++j) lsum = __builtin_amdgcn_fdot2(h16x2{v[2 * j], v[2 * j + 1]}, one, lsum, false);
        pb[st][h] = v;
      }
    }
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int d = 0; d < 4; ++d) O[d] = __builtin_amdgcn_mfma_f32_32x32x16_f16(qa, pb[b >> 1][b & 1], O[d], 0, 0, 0);
  }
  float s = lsum + mrow;
  for (int d = 0; d < 4; ++d) s += O[d][0] + O[d][9];
  if (s == 123.456f) out[threadIdx.x] = s;
  if (threadIdx.x == 0 && blockIdx.x == 0) clk[0] = __builtin_readcyclecounter() - c0;
}

// ---- 3. lane placement of the direct global-to-LDS loads
template <int BYTES>
__global__ void lds_dma_kernel(const unsigned* __restrict__ src, unsigned* __restrict__ out) {
  __shared__ __attribute__((aligned(16))) unsigned lds[2048];
  for (int i = threadIdx.x; i < 2048; i += blockDim.x) lds[i] = 0xdeadbeefu;
  __syncthreads();
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const unsigned base = (unsigned)(unsigned long long)(lds_u32*)lds + 1024u + (unsigned)(wave * 64 * BYTES);
  const unsigned voff = (unsigned)(BYTES * ((7 * (64 * wave + lane) + 3) % 256));   // a permutation of the 256 pieces
  if (BYTES == 16)
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(src), "s"(base) : "memory");
  else
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" ::"v"(voff), "s"(src), "s"(base) : "memory");
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  for (int i = threadIdx.x; i < 2048; i += blockDim.x) out[i] = lds[i];
}

template <int BYTES>
static int check_lds_dma(unsigned* src, unsigned* out) {
  const int words = BYTES / 4;
  std::vector<unsigned> h(256 * words);
  for (int i = 0; i < 256 * words; ++i) h[i] = 0x1000u * (i / words) + (i % words);
  CHECK(hipMemcpy(src, h.data(), h.size() * 4, hipMemcpyHostToDevice));
  hipLaunchKernelGGL(lds_dma_kernel<BYTES>, dim3(1), dim3(256), 0, 0, src, out);
  CHECK(hipDeviceSynchronize());
  std::vector<unsigned> o(2048);
  CHECK(hipMemcpy(o.data(), out, 8192, hipMemcpyDeviceToHost));
  int bad = 0;
  for (int t = 0; t < 256; ++t)
    for (int k = 0; k < words; ++k)
      if (o[256 + t * words + k] != 0x1000u * ((7 * t + 3) % 256) + k) ++bad;
  printf("direct global-to-LDS load, %2d bytes per lane: lane l of wave w lands at base + %d * (64 w + l): %s\n", BYTES,
         BYTES, bad ? "NO" : "yes");
  return bad;
}

int main() {
  float* out;
  unsigned long long* clk;
  unsigned *src, *dma_out;
  CHECK(hipMalloc(&out, 1 << 20));
  CHECK(hipMalloc(&clk, 64));
  CHECK(hipMalloc(&src, 4096));
  CHECK(hipMalloc(&dma_out, 8192));
  unsigned long long h;

  int bad = check_lds_dma<16>(src, dma_out) + check_lds_dma<4>(src, dma_out);

  printf("\ninstruction issue (counter ticks of s_memtime per instruction; 256 workgroups)\n");
  for (int op = 0; op < 2; ++op)
    for (int thr : {256, 512, 1024}) {
      const int iters = 4000;
      for (int rep = 0; rep < 2; ++rep) {
        if (op == 0) hipLaunchKernelGGL(issue_kernel<0>, dim3(256), dim3(thr), 0, 0, out, clk, iters);
        else hipLaunchKernelGGL(issue_kernel<1>, dim3(256), dim3(thr), 0, 0, out, clk, iters);
        CHECK(hipDeviceSynchronize());
      }
      CHECK(hipMemcpy(&h, clk, 8, hipMemcpyDeviceToHost));
      printf("  %-5s %d wave(s) per SIMD: %.2f per wave, %.2f per SIMD\n", op ? "exp2" : "fma", thr / 256,
             (double)h / iters / 64, (double)h / iters / 64 / (thr / 256.0));
    }

  printf("\nattention tile loop in registers, 8 waves per workgroup, one workgroup per CU\n");
  const int iters = 100000;
  for (int rnd = 0; rnd < 2; ++rnd)
    for (int wgs : {32, 256}) {
      hipEvent_t a, b;
      CHECK(hipEventCreate(&a));
      CHECK(hipEventCreate(&b));
      float ms = 0;
      for (int rep = 0; rep < 2; ++rep) {
        CHECK(hipEventRecord(a));
        if (rnd) hipLaunchKernelGGL(tile_loop_kernel<1>, dim3(wgs), dim3(512), 0, 0, out, clk, iters, 0.1275f);
        else hipLaunchKernelGGL(tile_loop_kernel<0>, dim3(wgs), dim3(512), 0, 0, out, clk, iters, 0.1275f);
        CHECK(hipEventRecord(b));
        CHECK(hipDeviceSynchronize());
        CHECK(hipEventElapsedTime(&ms, a, b));
      }
      CHECK(hipMemcpy(&h, clk, 8, hipMemcpyDeviceToHost));
      printf("  %-8s operands, %3d CUs: %.3f us per tile, %.0f counter ticks per tile\n", rnd ? "random" : "constant", wgs,
             ms * 1e3 / iters, (double)h / iters);
    }
  return bad ? 1 : 0;
}
