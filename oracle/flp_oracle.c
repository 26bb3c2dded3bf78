/*
 * CPU oracle for the paged multi-LoRA layer step.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain C, double precision, one loop per index of each definition; nothing is
 * tiled, fused or reordered.  It is called from the tests, from the smoke
 * check and from the benchmark's cpu_baseline leg, never from the product
 * path, and shares no source with the HIP library (the layout rules below are
 * written out a second time here on purpose).
 *
 * What it follows in the paper:
 *   - unified caching pool (section 4.3, "Unified Caching Pool for LoRAs and
 *     KVs"): device and host memory are cut into blocks of one size; a block
 *     holds either LoRA page-rows or the K/V of `bt` token positions; freed
 *     blocks are recycled.
 *   - LoRA is partitioned block-wise along the rank dimension (same
 *     paragraph): a LoRA matrix is a list of rank rows; rows never straddle a
 *     block.
 *   - Eq. 1 (W' = W + A B) and Eq. 2 (K/V of a query under adapter t are the
 *     base projection plus the adapter's low-rank branch), evaluated in the
 *     row-vector convention y = x W + s (x A) B.
 *   - prefix reuse (section 2.1, "KV Caches for Multi-LoRAs", and section 4.2):
 *     a new token attends to the stored K/V of every earlier position of its
 *     own sequence, reused prefix and fresh positions alike; fresh K/V stays in
 *     the pool where it is produced (section 4.3).
 *
 * Readings where the paper is silent (each also listed in the design notes):
 *   block = [K: n_kv x bt x d][V: n_kv x d x bt] elements, V stored transposed;
 *   free list is a LIFO stack; duplicate destinations in a swap list are an
 *   error; softmax scale 1/sqrt(d) unless given; causal over prefix + new.
 *
 * dtype codes: 0 = fp32, 1 = fp16 (IEEE binary16 bits), 2 = bf16 bits.
 * All pointers are host pointers.  Functions return 0 or a negative code:
 * -1 invalid argument, -2 no space, -3 out of range, -4 duplicate.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* Type of the running sums of the LoRA and attention products.  double in the parity build (the only one the
 * tests use); the benchmark's cpu_baseline leg also times a second build with -DORC_ACC_T=float (fp32
 * accumulation, what a production CPU kernel would do), which no parity check ever loads. */
#ifndef ORC_ACC_T
#define ORC_ACC_T double
#endif
typedef ORC_ACC_T acc_t;

/* ------------------------------------------------------------------ formats */
static double half_to_double(uint16_t h) {
  int sign = (h >> 15) & 1;
  int e = (h >> 10) & 0x1F;
  int m = h & 0x3FF;
  double v;
  if (e == 0) v = ldexp((double)m, -24);                 /* zero / subnormal */
  else if (e == 31) v = m ? NAN : INFINITY;
  else v = ldexp((double)(m | 0x400), e - 25);
  return sign ? -v : v;
}
static double bf16_to_double(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, 4);
  return (double)f;
}
static double load_elem(const void* base, int dtype, int64_t i) {
  if (dtype == 0) return (double)((const float*)base)[i];
  uint16_t h = ((const uint16_t*)base)[i];
  return dtype == 1 ? half_to_double(h) : bf16_to_double(h);
}
static int elem_bytes(int dtype) { return dtype == 0 ? 4 : 2; }

/* nearest-even rounding of a double to the storage format, returned as the
 * value it represents (used only by the whole-step chain, where the method
 * stores q/k/v in the pool's element type between stages). */
static double round_to_dtype(double v, int dtype) {
  if (dtype == 0) return (double)(float)v;
  if (!isfinite(v) || v == 0.0) return v;
  int mant_bits = dtype == 1 ? 10 : 7;
  int min_exp = dtype == 1 ? -14 : -126;
  int e;
  double f = frexp(fabs(v), &e);       /* |v| = f * 2^e, f in [0.5,1) */
  int ex = e - 1;                      /* |v| = (2f) * 2^ex, 2f in [1,2) */
  if (ex < min_exp) ex = min_exp;      /* subnormal: fixed quantum */
  double q = ldexp(1.0, ex - mant_bits);
  double r = nearbyint(fabs(v) / q) * q; /* default rounding mode = nearest even */
  double maxv = dtype == 1 ? 65504.0 : 3.3895313892515355e38;
  if (r > maxv) r = INFINITY;
  (void)f;
  return v < 0 ? -r : r;
}
double orc_round_to_dtype(double v, int dtype) { return round_to_dtype(v, dtype); }

/* ------------------------------------------------------------------ layout  */
/* K of (kv head g, slot s, channel c) and V of the same, inside one block. */
static int64_t k_off(int bt, int d, int g, int s, int c) { return ((int64_t)g * bt + s) * d + c; }
static int64_t v_off(int bt, int n_kv, int d, int g, int s, int c) {
  return (int64_t)n_kv * bt * d + ((int64_t)g * d + c) * bt + s;
}
/* element index (in the whole pool) of element c of page-row `row` of a table */
static int64_t lora_elem(const int32_t* table, int64_t block_elems, int row_len, int64_t row, int c) {
  int64_t rpb = block_elems / row_len;
  int64_t blk = table[row / rpb];
  return blk * block_elems + (row % rpb) * row_len + c;
}

/* ------------------------------------------------------------------ O1 pool */
typedef struct {
  int64_t n;
  int64_t top;        /* number of free ids on the stack */
  int32_t* stack;     /* stack[top-1] is handed out next */
  uint8_t* is_free;
} orc_alloc;

orc_alloc* orc_alloc_create(int64_t n) {
  orc_alloc* a = (orc_alloc*)malloc(sizeof(orc_alloc));
  a->n = n;
  a->top = n;
  a->stack = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
  a->is_free = (uint8_t*)malloc((size_t)(n > 0 ? n : 1));
  for (int64_t i = 0; i < n; ++i) {
    a->stack[i] = (int32_t)(n - 1 - i);   /* so the first pops give 0,1,2,... */
    a->is_free[i] = 1;
  }
  return a;
}
void orc_alloc_destroy(orc_alloc* a) {
  if (!a) return;
  free(a->stack);
  free(a->is_free);
  free(a);
}
int64_t orc_alloc_num_free(const orc_alloc* a) { return a->top; }
int orc_alloc_alloc(orc_alloc* a, int32_t n, int32_t* out) {
  if (n < 0) return -1;
  if (n > a->top) return -2;            /* all or nothing */
  for (int32_t k = 0; k < n; ++k) {
    int32_t id = a->stack[--a->top];
    a->is_free[id] = 0;
    out[k] = id;
  }
  return 0;
}
int orc_alloc_free(orc_alloc* a, int32_t n, const int32_t* ids) {
  if (n < 0) return -1;
  for (int32_t k = 0; k < n; ++k) {
    if (ids[k] < 0 || ids[k] >= a->n) return -3;
    if (a->is_free[ids[k]]) return -4;
    for (int32_t j = 0; j < k; ++j)
      if (ids[j] == ids[k]) return -4;
  }
  for (int32_t k = 0; k < n; ++k) {
    a->is_free[ids[k]] = 1;
    a->stack[a->top++] = ids[k];
  }
  return 0;
}

/* ------------------------------------------------------------------ O2 swap */
/* dst[dst_ids[k]] <- src[src_ids[k]] for k in order, whole blocks of raw bytes. */
int orc_swap(uint8_t* dst, int64_t n_dst_blocks, const uint8_t* src, int64_t n_src_blocks,
             int64_t block_bytes, int32_t n, const int32_t* src_ids, const int32_t* dst_ids) {
  if (n < 0) return -1;
  for (int32_t k = 0; k < n; ++k) {
    if (src_ids[k] < 0 || src_ids[k] >= n_src_blocks) return -3;
    if (dst_ids[k] < 0 || dst_ids[k] >= n_dst_blocks) return -3;
    for (int32_t j = 0; j < k; ++j)
      if (dst_ids[j] == dst_ids[k]) return -4;
  }
  for (int32_t k = 0; k < n; ++k)
    memcpy(dst + (int64_t)dst_ids[k] * block_bytes, src + (int64_t)src_ids[k] * block_bytes,
           (size_t)block_bytes);
  return 0;
}

/* -------------------------------------------------------- adapter segmentation */
/* Stable grouping of token indices by adapter id (ids < 0 belong to no segment).
 * seg_adapter/seg_start list the non-empty adapters in increasing id order. */
int orc_segment(int32_t T, const int32_t* token_adapter, int32_t n_adapters,
                int32_t* n_seg_out, int32_t* seg_adapter, int32_t* seg_start, int32_t* perm) {
  int32_t n_seg = 0, pos = 0;
  for (int32_t t = 0; t < T; ++t)
    if (token_adapter[t] >= n_adapters) return -3;
  for (int32_t a = 0; a < n_adapters; ++a) {
    int32_t first = pos;
    for (int32_t t = 0; t < T; ++t)
      if (token_adapter[t] == a) perm[pos++] = t;
    if (pos > first) {
      seg_adapter[n_seg] = a;
      seg_start[n_seg] = first;
      ++n_seg;
    }
  }
  seg_start[n_seg] = pos;
  *n_seg_out = n_seg;
  return 0;
}

/* ------------------------------------------------------------------ O3 LoRA */
/* For each selected token t (sel == NULL: all tokens, n_sel = T):
 *   base[o] = y_in[t,o]                      if w_base == NULL
 *           = sum_c x[t,c] W[c,o]            otherwise      (W is [d_in, d_out])
 *   y[t,o]  = base[o] + s_a * sum_rho ( sum_c x[t,c] A_a[rho,c] ) * B_a[rho,o]
 * with a = token_adapter[t]; a < 0 gives y = base.  A_a[rho,:] is page-row
 * a_row_base[a]+rho of the table at a_tab_off[a] (row length d_in), B_a[rho,:]
 * page-row b_row_base[a]+rho of the table at b_tab_off[a] (row length d_out).
 * out is double [n_sel, d_out]. */
int orc_lora_apply(const void* pool, int dtype, int64_t block_elems,
                   int32_t T, int32_t d_in, int32_t d_out,
                   const void* x, int64_t ld_x, const void* y_in, int64_t ld_y,
                   const void* w_base, const int32_t* token_adapter, int32_t n_adapters,
                   const int32_t* rank, const float* scale,
                   const int32_t* a_tab_off, const int32_t* a_row_base,
                   const int32_t* b_tab_off, const int32_t* b_row_base,
                   const int32_t* block_tables,
                   int32_t n_sel, const int32_t* sel, double* out) {
  if (!pool || !x || !out || (!y_in && !w_base)) return -1;
  for (int32_t i = 0; i < n_sel; ++i) {
    int32_t t = sel ? sel[i] : i;
    if (t < 0 || t >= T) return -3;
    int32_t a = token_adapter[t];
    if (a >= n_adapters) return -3;
    if (a >= 0 && rank[a] <= 0) return -1;   /* token references an adapter that is not resident */
  }
  int status = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int32_t i = 0; i < n_sel; ++i) {
    int32_t t = sel ? sel[i] : i;
    int32_t a = token_adapter[t];
    double* y = out + (int64_t)i * d_out;
    for (int32_t o = 0; o < d_out; ++o) {
      if (w_base) {
        acc_t acc = 0.0;
        for (int32_t c = 0; c < d_in; ++c)
          acc += load_elem(x, dtype, t * ld_x + c) * load_elem(w_base, dtype, (int64_t)c * d_out + o);
        y[o] = acc;
      } else {
        y[o] = load_elem(y_in, dtype, t * ld_y + o);
      }
    }
    if (a < 0) continue;
    int32_t r = rank[a];
    double* v = (double*)malloc(sizeof(double) * (size_t)r);
    if (!v) { status = -2; continue; }
    const int32_t* ta = block_tables + a_tab_off[a];
    const int32_t* tb = block_tables + b_tab_off[a];
    for (int32_t rho = 0; rho < r; ++rho) {
      acc_t acc = 0.0;
      for (int32_t c = 0; c < d_in; ++c)
        acc += load_elem(x, dtype, t * ld_x + c) *
               load_elem(pool, dtype, lora_elem(ta, block_elems, d_in, (int64_t)a_row_base[a] + rho, c));
      v[rho] = acc;
    }
    for (int32_t o = 0; o < d_out; ++o) {
      acc_t acc = 0.0;
      for (int32_t rho = 0; rho < r; ++rho)
        acc += v[rho] * load_elem(pool, dtype, lora_elem(tb, block_elems, d_out, (int64_t)b_row_base[a] + rho, o));
      y[o] += (double)scale[a] * acc;
    }
    free(v);
  }
  return status;
}

/* Dense form of Eq. 1 for one adapter: dW[c,o] = sum_rho A[rho,c] B[rho,o]
 * (double, [d_in, d_out]); lets a test compare the factored result with x.dW. */
int orc_lora_dense_delta(const void* pool, int dtype, int64_t block_elems, int32_t d_in, int32_t d_out,
                         int32_t r, const int32_t* table_a, int32_t a_row_base,
                         const int32_t* table_b, int32_t b_row_base, double* dW) {
  for (int32_t c = 0; c < d_in; ++c)
    for (int32_t o = 0; o < d_out; ++o) {
      double acc = 0.0;
      for (int32_t rho = 0; rho < r; ++rho)
        acc += load_elem(pool, dtype, lora_elem(table_a, block_elems, d_in, (int64_t)a_row_base + rho, c)) *
               load_elem(pool, dtype, lora_elem(table_b, block_elems, d_out, (int64_t)b_row_base + rho, o));
      dW[(int64_t)c * d_out + o] = acc;
    }
  return 0;
}

/* Write / read one page-row through a table (raw elements); test helpers for
 * building structured adapters and for reading A/B back. */
int orc_lora_write_row(void* pool, int dtype, int64_t block_elems, const int32_t* table, int32_t row_len,
                       int64_t row, const void* src) {
  int eb = elem_bytes(dtype);
  memcpy((uint8_t*)pool + lora_elem(table, block_elems, row_len, row, 0) * eb, src, (size_t)row_len * eb);
  return 0;
}
int orc_lora_read_row(const void* pool, int dtype, int64_t block_elems, const int32_t* table, int32_t row_len,
                      int64_t row, double* dst) {
  for (int32_t c = 0; c < row_len; ++c)
    dst[c] = load_elem(pool, dtype, lora_elem(table, block_elems, row_len, row, c));
  return 0;
}

/* ------------------------------------------------------------------ O4 append */
/* Position p of sequence i lives in block tables[i][p / bt], slot p % bt.  The K
 * and V rows of the step's new tokens (k_new, v_new: [T, n_kv, d], pool dtype)
 * are stored there bit for bit. */
int orc_kv_append(void* pool, int dtype, int32_t bt, int32_t n_kv, int32_t d,
                  int32_t S, const int32_t* cu_new, const int32_t* prefix_len,
                  const int32_t* tables, int32_t max_blocks,
                  const void* k_new, const void* v_new) {
  int eb = elem_bytes(dtype);
  int64_t block_elems = 2LL * bt * n_kv * d;
  for (int32_t i = 0; i < S; ++i) {
    int32_t n = cu_new[i + 1] - cu_new[i];
    if (n < 0 || prefix_len[i] < 0) return -1;
    if ((int64_t)prefix_len[i] + n > (int64_t)max_blocks * bt) return -3;
  }
  for (int32_t i = 0; i < S; ++i)
    for (int32_t t = cu_new[i]; t < cu_new[i + 1]; ++t) {
      int32_t p = prefix_len[i] + (t - cu_new[i]);
      int64_t blk = tables[(int64_t)i * max_blocks + p / bt];
      int32_t s = p % bt;
      for (int32_t g = 0; g < n_kv; ++g)
        for (int32_t c = 0; c < d; ++c) {
          int64_t src = ((int64_t)t * n_kv + g) * d + c;
          memcpy((uint8_t*)pool + (blk * block_elems + k_off(bt, d, g, s, c)) * eb,
                 (const uint8_t*)k_new + src * eb, (size_t)eb);
          memcpy((uint8_t*)pool + (blk * block_elems + v_off(bt, n_kv, d, g, s, c)) * eb,
                 (const uint8_t*)v_new + src * eb, (size_t)eb);
        }
    }
  return 0;
}

/* Read positions 0..L-1 of one sequence back through its table as doubles:
 * K, V are [L, n_kv, d]. */
int orc_kv_gather(const void* pool, int dtype, int32_t bt, int32_t n_kv, int32_t d,
                  const int32_t* table, int32_t L, double* K, double* V) {
  int64_t block_elems = 2LL * bt * n_kv * d;
  for (int32_t p = 0; p < L; ++p) {
    int64_t blk = table[p / bt];
    int32_t s = p % bt;
    for (int32_t g = 0; g < n_kv; ++g)
      for (int32_t c = 0; c < d; ++c) {
        K[((int64_t)p * n_kv + g) * d + c] = load_elem(pool, dtype, blk * block_elems + k_off(bt, d, g, s, c));
        V[((int64_t)p * n_kv + g) * d + c] = load_elem(pool, dtype, blk * block_elems + v_off(bt, n_kv, d, g, s, c));
      }
  }
  return 0;
}

/* ------------------------------------------------------------------ O5 attention */
/* For selected token t of sequence i (j = t - cu_new[i], absolute position
 * p = prefix_len[i] + j), query head h, kv head g = h / (n_h / n_kv):
 *   s_k = sm_scale * sum_c q[t,h,c] K_i[k,g,c]        k = 0..p
 *   w   = softmax(s)  (max subtracted, double)
 *   out[t,h,:] = sum_k w_k V_i[k,g,:]
 * q is [T, n_h, d] in the pool dtype; out is double [n_sel, n_h, d]; wsum (may be
 * NULL) receives sum_k w_k per (selected token, head). sm_scale <= 0 means 1/sqrt(d). */
int orc_paged_attention(const void* pool, int dtype, int32_t bt, int32_t n_kv, int32_t d,
                        int32_t S, int32_t n_h, const int32_t* cu_new, const int32_t* prefix_len,
                        const int32_t* tables, int32_t max_blocks, const void* q, double sm_scale,
                        int32_t n_sel, const int32_t* sel, double* out, double* wsum) {
  if (!pool || !q || !out || n_kv <= 0 || n_h % n_kv) return -1;
  int32_t T = cu_new[S];
  int64_t block_elems = 2LL * bt * n_kv * d;
  int32_t group = n_h / n_kv;
  if (sm_scale <= 0) sm_scale = 1.0 / sqrt((double)d);
  for (int32_t i = 0; i < S; ++i)
    if ((int64_t)prefix_len[i] + (cu_new[i + 1] - cu_new[i]) > (int64_t)max_blocks * bt) return -3;
  for (int32_t i = 0; i < n_sel; ++i) {
    int32_t t = sel ? sel[i] : i;
    if (t < 0 || t >= T) return -3;
  }
  int status = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int32_t idx = 0; idx < n_sel; ++idx) {
    int32_t t = sel ? sel[idx] : idx;
    int32_t i = 0;
    while (!(cu_new[i] <= t && t < cu_new[i + 1])) ++i;
    int32_t p = prefix_len[i] + (t - cu_new[i]);
    const int32_t* table = tables + (int64_t)i * max_blocks;
    double* w = (double*)malloc(sizeof(double) * (size_t)(p + 1));
    if (!w) { status = -2; continue; }
    for (int32_t h = 0; h < n_h; ++h) {
      int32_t g = h / group;
      double m = -INFINITY;
      for (int32_t k = 0; k <= p; ++k) {
        int64_t base = (int64_t)table[k / bt] * block_elems;
        acc_t acc = 0.0;
        for (int32_t c = 0; c < d; ++c)
          acc += load_elem(q, dtype, ((int64_t)t * n_h + h) * d + c) *
                 load_elem(pool, dtype, base + k_off(bt, d, g, k % bt, c));
        w[k] = sm_scale * acc;
        if (w[k] > m) m = w[k];
      }
      double den = 0.0;
      for (int32_t k = 0; k <= p; ++k) {
        w[k] = exp(w[k] - m);
        den += w[k];
      }
      double tot = 0.0;
      for (int32_t k = 0; k <= p; ++k) {
        w[k] /= den;
        tot += w[k];
      }
      if (wsum) wsum[(int64_t)idx * n_h + h] = tot;
      double* o = out + ((int64_t)idx * n_h + h) * d;
      for (int32_t c = 0; c < d; ++c) {
        acc_t acc = 0.0;
        for (int32_t k = 0; k <= p; ++k) {
          int64_t base = (int64_t)table[k / bt] * block_elems;
          acc += w[k] * load_elem(pool, dtype, base + v_off(bt, n_kv, d, g, k % bt, c));
        }
        o[c] = acc;
      }
    }
    free(w);
  }
  return status;
}

/* The same definition on contiguous K, V (no pool, no tables): one sequence with
 * P prefix positions and N new tokens; K, V are double [P+N, n_kv, d], q is double
 * [N, n_h, d], out double [N, n_h, d]. */
int orc_contig_attention(const double* K, const double* V, const double* q, int32_t P, int32_t N,
                         int32_t n_h, int32_t n_kv, int32_t d, double sm_scale, double* out) {
  if (n_kv <= 0 || n_h % n_kv) return -1;
  int32_t group = n_h / n_kv;
  if (sm_scale <= 0) sm_scale = 1.0 / sqrt((double)d);
  double* w = (double*)malloc(sizeof(double) * (size_t)(P + N));
  for (int32_t j = 0; j < N; ++j)
    for (int32_t h = 0; h < n_h; ++h) {
      int32_t g = h / group, p = P + j;
      double m = -INFINITY, den = 0.0;
      for (int32_t k = 0; k <= p; ++k) {
        double acc = 0.0;
        for (int32_t c = 0; c < d; ++c)
          acc += q[((int64_t)j * n_h + h) * d + c] * K[((int64_t)k * n_kv + g) * d + c];
        w[k] = sm_scale * acc;
        if (w[k] > m) m = w[k];
      }
      for (int32_t k = 0; k <= p; ++k) { w[k] = exp(w[k] - m); den += w[k]; }
      for (int32_t c = 0; c < d; ++c) {
        double acc = 0.0;
        for (int32_t k = 0; k <= p; ++k) acc += (w[k] / den) * V[((int64_t)k * n_kv + g) * d + c];
        out[((int64_t)j * n_h + h) * d + c] = acc;
      }
    }
  free(w);
  return 0;
}

int orc_num_threads(void) {
#ifdef _OPENMP
  extern int omp_get_max_threads(void);
  return omp_get_max_threads();
#else
  return 1;
#endif
}
