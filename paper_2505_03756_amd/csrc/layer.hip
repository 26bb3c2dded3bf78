// Layer glue (include/fllayer.h): root-mean-square norm (optionally fused with the residual update
// before it), rotary position embedding, gated SiLU, and the call that strings them together with the
// pool's projections (base GEMM + paged LoRA), KV append and paged prefix attention into one decoder
// layer of the models the paper serves (section 6.1).  The element-wise kernels are plain HBM streams:
// 16 bytes per lane per access, fp32 arithmetic, one rounding at the store.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <mutex>

#include "fllayer.h"
#include "flp_internal.h"
#include "flp_types.h"

namespace {

template <typename S>
struct Vec {
  static constexpr int N = 16 / (int)sizeof(typename S::storage);
  typename S::storage e[N];
};

template <typename S>
__device__ __forceinline__ Vec<S> ldv(const void* p) {
  Vec<S> v;
  const u32x4 raw = *reinterpret_cast<const u32x4*>(p);
  __builtin_memcpy(&v, &raw, 16);
  return v;
}
template <typename S>
__device__ __forceinline__ void stv(void* p, const Vec<S>& v) {
  u32x4 raw;
  __builtin_memcpy(&raw, &v, 16);
  *reinterpret_cast<u32x4*>(p) = raw;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// One wave per token row, four rows per workgroup.  Pass 1 accumulates the sum of squares (and, with
// a delta, stores the rounded residual it is taken over); pass 2 re-reads the row (each lane the bytes
// it touched in pass 1: L1/L2 hits) and writes the normalised row.
template <typename S>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const typename S::storage* x_in, typename S::storage* resid,
                                                      const typename S::storage* __restrict__ delta,
                                                      const typename S::storage* __restrict__ w,
                                                      typename S::storage* y, int T, int H, float eps) {
  typedef typename S::storage ST;
  constexpr int N = Vec<S>::N;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= T) return;
  const ST* xr = (delta ? resid : x_in) + (int64_t)row * H;
  float ss = 0.f;
  for (int c = lane * N; c < H; c += 64 * N) {
    Vec<S> a = ldv<S>(xr + c);
    if (delta) {
      const Vec<S> d = ldv<S>(delta + (int64_t)row * H + c);
#pragma unroll
      for (int j = 0; j < N; ++j) a.e[j] = S::from_float(S::to_float(a.e[j]) + S::to_float(d.e[j]));
      stv<S>(resid + (int64_t)row * H + c, a);
    }
#pragma unroll
    for (int j = 0; j < N; ++j) {
      const float f = S::to_float(a.e[j]);
      ss = fmaf(f, f, ss);
    }
  }
  if (!y) return;
  ss = wave_sum(ss);
  const float inv = 1.0f / sqrtf(ss / (float)H + eps);
  for (int c = lane * N; c < H; c += 64 * N) {
    const Vec<S> a = ldv<S>(xr + c), g = ldv<S>(w + c);
    Vec<S> o;
#pragma unroll
    for (int j = 0; j < N; ++j) o.e[j] = S::from_float(S::to_float(a.e[j]) * inv * S::to_float(g.e[j]));
    stv<S>(y + (int64_t)row * H + c, o);
  }
}

// One workgroup per token.  The d/2 angles of the token are computed once in fp64 (position times
// theta^(-2i/d) reaches thousands of radians: fp32 would lose the fraction that matters), their sine and
// cosine kept in LDS as fp32, then every head's pairs are rotated, 16 bytes of each half per thread.
template <typename S, int D>
__global__ __launch_bounds__(256) void rope_kernel(typename S::storage* __restrict__ q, typename S::storage* __restrict__ k,
                                                   const int32_t* __restrict__ positions, int n_h, int n_kv,
                                                   double log2_theta) {
  typedef typename S::storage ST;
  constexpr int N = Vec<S>::N, HALF = D / 2, VPH = HALF / N;    // 16-byte vectors per half head
  __shared__ float cs[HALF], sn[HALF];
  const int t = blockIdx.x;
  if (threadIdx.x < HALF) {
    const double ang = (double)positions[t] * exp2(-2.0 * (double)threadIdx.x / (double)D * log2_theta);
    double s, c;
    sincos(ang, &s, &c);
    cs[threadIdx.x] = (float)c;
    sn[threadIdx.x] = (float)s;
  }
  __syncthreads();
  const int n_q_items = q ? n_h * VPH : 0, n_items = n_q_items + (k ? n_kv * VPH : 0);
  for (int it = threadIdx.x; it < n_items; it += 256) {
    const bool is_q = it < n_q_items;
    const int local = is_q ? it : it - n_q_items;
    const int head = local / VPH, i0 = (local % VPH) * N;
    ST* base = is_q ? q + ((int64_t)t * n_h + head) * D : k + ((int64_t)t * n_kv + head) * D;
    const Vec<S> a = ldv<S>(base + i0), b = ldv<S>(base + HALF + i0);
    Vec<S> oa, ob;
#pragma unroll
    for (int j = 0; j < N; ++j) {
      const float af = S::to_float(a.e[j]), bf = S::to_float(b.e[j]), c = cs[i0 + j], s = sn[i0 + j];
      oa.e[j] = S::from_float(af * c - bf * s);
      ob.e[j] = S::from_float(bf * c + af * s);
    }
    stv<S>(base + i0, oa);
    stv<S>(base + HALF + i0, ob);
  }
}

template <typename S>
__global__ __launch_bounds__(256) void silu_mul_kernel(const typename S::storage* __restrict__ gate, int64_t ld_g,
                                                       const typename S::storage* __restrict__ up, int64_t ld_u,
                                                       typename S::storage* __restrict__ out, int64_t ld_o, int64_t n_vec,
                                                       int vec_per_row) {
  constexpr int N = Vec<S>::N;
  const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (v >= n_vec) return;
  const int64_t row = v / vec_per_row;
  const int c = (int)(v - row * vec_per_row) * N;
  const Vec<S> g = ldv<S>(gate + row * ld_g + c), u = ldv<S>(up + row * ld_u + c);
  Vec<S> o;
#pragma unroll
  for (int j = 0; j < N; ++j) {
    const float gf = S::to_float(g.e[j]);
    o.e[j] = S::from_float(gf / (1.0f + expf(-gf)) * S::to_float(u.e[j]));
  }
  stv<S>(out + row * ld_o + c, o);
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }
int elem_bytes(int dtype) { return dtype == FLP_F32 ? 4 : 2; }

#define FLL_BY_DTYPE(dtype, CALL)          \
  do {                                     \
    if (dtype == FLP_F32) {                \
      typedef F32 S_;                      \
      CALL;                                \
    } else if (dtype == FLP_F16) {         \
      typedef F16 S_;                      \
      CALL;                                \
    } else {                               \
      typedef BF16 S_;                     \
      CALL;                                \
    }                                      \
  } while (0)

flp_status norm_common(int32_t dtype, const void* x, void* resid, const void* delta, const void* w, void* y, int32_t T,
                       int32_t H, float eps, void* hip_stream, const char* who) {
  if (dtype < FLP_F32 || dtype > FLP_BF16 || T < 0 || H <= 0 || (y && !w) || !aligned16(x) || !aligned16(resid) ||
      !aligned16(delta) || !aligned16(w) || !aligned16(y)) {
    flp_set_error("%s: bad dtype / sizes or null / misaligned pointer", who);
    return FLP_EINVAL;
  }
  if ((int64_t)H * elem_bytes(dtype) % 16) {
    flp_set_error("%s: a row of %d elements is not a multiple of 16 bytes", who, H);
    return FLP_ENOTSUP;
  }
  if (T == 0) return FLP_OK;
  hipStream_t st = (hipStream_t)hip_stream;
  FLL_BY_DTYPE(dtype, hipLaunchKernelGGL(rmsnorm_kernel<S_>, dim3((T + 3) / 4), dim3(256), 0, st,
                                         (const S_::storage*)x, (S_::storage*)resid, (const S_::storage*)delta,
                                         (const S_::storage*)w, (S_::storage*)y, T, H, eps));
  FLP_TRY_HIP(hipGetLastError());
  return FLP_OK;
}

}  // namespace

extern "C" flp_status fll_rmsnorm(int32_t dtype, const void* x, const void* w, void* y, int32_t n_tokens, int32_t hidden,
                                  float eps, void* hip_stream) {
  if (!x || !w || !y) {
    flp_set_error("fll_rmsnorm: null pointer");
    return FLP_EINVAL;
  }
  return norm_common(dtype, x, nullptr, nullptr, w, y, n_tokens, hidden, eps, hip_stream, "fll_rmsnorm");
}

extern "C" flp_status fll_add_rmsnorm(int32_t dtype, void* resid, const void* delta, const void* w, void* y,
                                      int32_t n_tokens, int32_t hidden, float eps, void* hip_stream) {
  if (!resid || !delta) {
    flp_set_error("fll_add_rmsnorm: null pointer");
    return FLP_EINVAL;
  }
  return norm_common(dtype, nullptr, resid, delta, w, y, n_tokens, hidden, eps, hip_stream, "fll_add_rmsnorm");
}

extern "C" flp_status fll_rope(int32_t dtype, void* q, void* k, const int32_t* positions, int32_t n_tokens,
                               int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, float theta, void* hip_stream) {
  if (dtype < FLP_F32 || dtype > FLP_BF16 || n_tokens < 0 || !positions || (q && n_q_heads <= 0) ||
      (k && n_kv_heads <= 0) || !(theta > 0) || !aligned16(q) || !aligned16(k)) {
    flp_set_error("fll_rope: bad dtype / sizes / theta or null / misaligned pointer");
    return FLP_EINVAL;
  }
  if (head_dim != 64 && head_dim != 128) {
    flp_set_error("fll_rope: head_dim %d not supported (64 or 128)", head_dim);
    return FLP_ENOTSUP;
  }
  if (n_tokens == 0 || (!q && !k)) return FLP_OK;
  hipStream_t st = (hipStream_t)hip_stream;
  const double l2t = std::log2((double)theta);
  if (head_dim == 64)
    FLL_BY_DTYPE(dtype, hipLaunchKernelGGL((rope_kernel<S_, 64>), dim3(n_tokens), dim3(256), 0, st, (S_::storage*)q,
                                           (S_::storage*)k, positions, n_q_heads, n_kv_heads, l2t));
  else
    FLL_BY_DTYPE(dtype, hipLaunchKernelGGL((rope_kernel<S_, 128>), dim3(n_tokens), dim3(256), 0, st, (S_::storage*)q,
                                           (S_::storage*)k, positions, n_q_heads, n_kv_heads, l2t));
  FLP_TRY_HIP(hipGetLastError());
  return FLP_OK;
}

extern "C" flp_status fll_silu_mul(int32_t dtype, const void* gate, int64_t ld_gate, const void* up, int64_t ld_up,
                                   void* out, int64_t ld_out, int32_t n_tokens, int32_t width, void* hip_stream) {
  if (dtype < FLP_F32 || dtype > FLP_BF16 || n_tokens < 0 || width <= 0 || !gate || !up || !out || ld_gate < width ||
      ld_up < width || ld_out < width || !aligned16(gate) || !aligned16(up) || !aligned16(out)) {
    flp_set_error("fll_silu_mul: bad dtype / sizes or null / misaligned pointer");
    return FLP_EINVAL;
  }
  const int eb = elem_bytes(dtype);
  if ((int64_t)width * eb % 16 || ld_gate * eb % 16 || ld_up * eb % 16 || ld_out * eb % 16) {
    flp_set_error("fll_silu_mul: width and leading dimensions must be multiples of 16 bytes");
    return FLP_ENOTSUP;
  }
  if (n_tokens == 0) return FLP_OK;
  const int vpr = width * eb / 16;
  const int64_t n_vec = (int64_t)n_tokens * vpr;
  hipStream_t st = (hipStream_t)hip_stream;
  FLL_BY_DTYPE(dtype, hipLaunchKernelGGL(silu_mul_kernel<S_>, dim3((unsigned)((n_vec + 255) / 256)), dim3(256), 0, st,
                                         (const S_::storage*)gate, ld_gate, (const S_::storage*)up, ld_up,
                                         (S_::storage*)out, ld_out, n_vec, vpr));
  FLP_TRY_HIP(hipGetLastError());
  return FLP_OK;
}

// ------------------------------------------------------------------------------- the layer
namespace {
struct Scratch {
  size_t n, q, k, v, attn, proj, gate, up, total;
};
Scratch layout(const flp_pool* p, const fll_layer_config* c, int64_t T) {
  const int64_t eb = p->elem_bytes, d = p->cfg.head_dim;
  auto al = [](int64_t b) { return (size_t)((b + 255) & ~(int64_t)255); };
  Scratch s{};
  size_t off = 0;
  auto take = [&](int64_t bytes) {
    const size_t o = off;
    off += al(bytes);
    return o;
  };
  s.n = take(T * c->hidden * eb);
  s.q = take(T * c->n_q_heads * d * eb);
  s.k = take(T * p->cfg.n_kv_heads * d * eb);
  s.v = take(T * p->cfg.n_kv_heads * d * eb);
  s.attn = take(T * c->n_q_heads * d * eb);
  s.proj = take(T * c->hidden * eb);
  s.gate = take(T * c->mlp_dim * eb);
  s.up = take(T * c->mlp_dim * eb);
  s.total = off;
  return s;
}
bool cfg_ok(const flp_pool* p, const fll_layer_config* c) {
  return p && c && c->hidden > 0 && c->n_q_heads > 0 && c->mlp_dim > 0 && c->n_q_heads % p->cfg.n_kv_heads == 0;
}
}  // namespace

extern "C" int64_t fll_layer_scratch_bytes(const flp_pool* pool, const fll_layer_config* cfg, int32_t n_tokens) {
  if (!cfg_ok(pool, cfg) || n_tokens < 0) return -1;
  return (int64_t)layout(pool, cfg, n_tokens).total;
}

extern "C" flp_status fll_layer_forward(flp_pool* p, const fll_layer_config* c, const fll_layer_weights* w,
                                        const fll_layer_batch* b, void* h, void* scratch, int64_t scratch_bytes,
                                        void* hip_stream) {
  if (!cfg_ok(p, c) || !w || !b || !h || !scratch || b->n_tokens < 0 || b->n_seqs < 0) {
    flp_set_error("fll_layer_forward: null argument or bad layer shape");
    return FLP_EINVAL;
  }
  if (!w->in_norm || !w->post_norm || !w->wq || !w->wk || !w->wv || !w->wo || !w->w_gate || !w->w_up || !w->w_down) {
    flp_set_error("fll_layer_forward: a weight pointer is null");
    return FLP_EINVAL;
  }
  const int32_t T = b->n_tokens;
  if (T == 0) return FLP_OK;
  const Scratch s = layout(p, c, T);
  if (((uintptr_t)scratch & 255) || scratch_bytes < (int64_t)s.total) {
    flp_set_error("fll_layer_forward: scratch misaligned or smaller than %lld bytes", (long long)s.total);
    return FLP_EINVAL;
  }
  const int dtype = p->cfg.dtype, d = p->cfg.head_dim, n_kv = p->cfg.n_kv_heads;
  const int Hq = c->n_q_heads * d, Hkv = n_kv * d, H = c->hidden, M = c->mlp_dim;
  const float eps = c->rms_eps > 0 ? c->rms_eps : 1e-5f, theta = c->rope_theta > 0 ? c->rope_theta : 10000.0f;
  uint8_t* sb = (uint8_t*)scratch;
  void *n = sb + s.n, *q = sb + s.q, *k = sb + s.k, *v = sb + s.v, *attn = sb + s.attn, *proj = sb + s.proj,
       *gate = sb + s.gate, *up = sb + s.up;

  // base GEMM + LoRA branch of up to three projections that share their input
  auto project = [&](const void* x, int d_in, int n_proj, const int* which, void* const* ys, const int* d_outs,
                     const void* const* ws, void* gated_out = nullptr) -> flp_status {
    flp_lora_batch lb{};
    lb.n_tokens = T;
    lb.d_in = d_in;
    lb.ld_x = d_in;
    lb.n_adapters = b->n_adapters;
    lb.max_rank = b->max_rank;
    lb.n_proj = n_proj;
    lb.x = x;
    lb.token_adapter = b->token_adapter;
    lb.rank = b->rank;
    lb.scale = b->scale;
    lb.block_tables = b->lora_tables;
    int n_lora = 0;
    for (int i = 0; i < n_proj; ++i) {
      const fll_lora_place& pl = b->lora[which[i]];
      const int n_set = (pl.a_tab_off != nullptr) + (pl.a_row_base != nullptr) + (pl.b_tab_off != nullptr) +
                        (pl.b_row_base != nullptr);
      if (n_set == 0) {                               // no LoRA branch on this projection: the dense product alone
        if (p->elem_bytes == 2 && d_in % 64) {
          flp_set_error("fll_layer_forward: projection %d: d_in %d is not a multiple of 64", which[i], d_in);
          return FLP_ENOTSUP;
        }
        // split-K slices of a small batch live in the pool's workspace (stream order keeps them apart from the
        // LoRA intermediates of the calls before and after)
        const size_t sk_bytes = p->elem_bytes == 2 ? flp_gemm_splitk_bytes(T, d_outs[i]) : 0;
        void* sk = nullptr;
        if (sk_bytes) {
          std::lock_guard<std::mutex> lk(p->mu);
          FLP_TRY(flp_workspace(p, sk_bytes, &sk));
        }
        FLP_TRY(flp_launch_base_gemm(dtype, x, d_in, ws[i], 1, ys[i], d_outs[i], T, d_outs[i], d_in, nullptr, nullptr,
                                     (float*)sk, sk_bytes, (hipStream_t)hip_stream));
        continue;
      }
      if (n_set != 4) {
        flp_set_error("fll_layer_forward: projection %d has an incomplete LoRA placement", which[i]);
        return FLP_EINVAL;
      }
      flp_lora_proj& pr = lb.proj[n_lora++];
      pr.d_out = d_outs[i];
      pr.w_base_layout = 1;
      pr.ld_y = d_outs[i];
      pr.y = ys[i];
      pr.w_base = ws[i];
      pr.a_tab_off = pl.a_tab_off;
      pr.a_row_base = pl.a_row_base;
      pr.b_tab_off = pl.b_tab_off;
      pr.b_row_base = pl.b_row_base;
    }
    if (n_lora == 0) return FLP_OK;
    lb.n_proj = n_lora;
    if (gated_out) return flp_lora_apply_gated(p, &lb, gated_out, d_outs[0], hip_stream);
    return flp_lora_apply_paged(p, &lb, hip_stream);
  };

  FLP_TRY(fll_rmsnorm(dtype, h, w->in_norm, n, T, H, eps, hip_stream));
  {
    const int which[3] = {0, 1, 2}, d_outs[3] = {Hq, Hkv, Hkv};
    void* const ys[3] = {q, k, v};
    const void* const ws[3] = {w->wq, w->wk, w->wv};
    FLP_TRY(project(n, H, 3, which, ys, d_outs, ws));
  }
  FLP_TRY(fll_rope(dtype, q, k, b->positions, T, c->n_q_heads, n_kv, d, theta, hip_stream));
  {
    flp_attn_batch ab{};
    ab.n_seqs = b->n_seqs;
    ab.n_q_heads = c->n_q_heads;
    ab.max_blocks_per_seq = b->max_blocks_per_seq;
    ab.sm_scale = 0.f;
    ab.q = q;
    ab.k_new = k;
    ab.v_new = v;
    ab.out = attn;
    ab.cu_new = b->cu_new;
    ab.prefix_len = b->prefix_len;
    ab.block_tables = b->kv_tables;
    FLP_TRY(flp_paged_prefix_attention(p, &ab, hip_stream));
  }
  {
    const int which[1] = {3}, d_outs[1] = {H};
    void* const ys[1] = {proj};
    const void* const ws[1] = {w->wo};
    FLP_TRY(project(attn, Hq, 1, which, ys, d_outs, ws));
  }
  FLP_TRY(fll_add_rmsnorm(dtype, h, proj, w->post_norm, n, T, H, eps, hip_stream));
  {
    // without LoRA branches on gate and up, and for a batch that the large-batch GEMM takes, the two products
    // and the gate are one kernel that writes only silu(g) * u; otherwise two products and the element-wise step
    const auto no_lora = [&](int i) {
      const fll_lora_place& pl = b->lora[i];
      return !pl.a_tab_off && !pl.a_row_base && !pl.b_tab_off && !pl.b_row_base;
    };
    const auto full_lora = [&](int i) {
      const fll_lora_place& pl = b->lora[i];
      return pl.a_tab_off && pl.a_row_base && pl.b_tab_off && pl.b_row_base;
    };
    const int which[2] = {4, 5}, d_outs[2] = {M, M};
    void* const ys[2] = {gate, up};
    const void* const ws[2] = {w->w_gate, w->w_up};
    flp_status fused = FLP_ENOTSUP;
    if (no_lora(4) && no_lora(5))
      fused = flp_launch_gated_gemm(dtype, n, H, w->w_gate, w->w_up, gate, M, T, M, H, (hipStream_t)hip_stream);
    else if (full_lora(4) && full_lora(5))          // both with a LoRA branch: the branches are added inside the same pass
      fused = project(n, H, 2, which, ys, d_outs, ws, gate);
    if (fused == FLP_ENOTSUP) {
      FLP_TRY(project(n, H, 2, which, ys, d_outs, ws));
      FLP_TRY(fll_silu_mul(dtype, gate, M, up, M, gate, M, T, M, hip_stream));
    } else if (fused != FLP_OK) {
      return fused;
    }
  }
  {
    const int which[1] = {6}, d_outs[1] = {H};
    void* const ys[1] = {proj};
    const void* const ws[1] = {w->w_down};
    FLP_TRY(project(gate, M, 1, which, ys, d_outs, ws));
  }
  return fll_add_rmsnorm(dtype, h, proj, nullptr, nullptr, T, H, eps, hip_stream);
}
