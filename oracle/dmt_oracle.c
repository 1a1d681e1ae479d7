/*
 * CPU oracle for the DMT tower hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, double-precision loops that state what the path computes, for
 * the parity tests and for the benchmark's CPU-baseline leg.  Nothing in the
 * product library includes, links or calls this file, and this file shares no
 * code with the HIP kernels.
 *
 * What each function follows (paper = "Disaggregated Multi-Tower", arXiv
 * 2403.00877):
 *   lookup          Sec. 2.1 (a feature's id tuple becomes one dense vector),
 *                   Sec. 2.2 step b (parallel row queries + pooling); sum
 *                   pooling and multiset semantics are this build's reading.
 *   towered layout  Sec. 3.1.1 steps c-e and Sec. 4 ("embs" of shape
 *                   (B, |F|, N) per tower = what step e leaves on a GPU).
 *   tower modules   Sec. 3.2 and Sec. 4 (Listings 1 and 2, and the pairwise
 *                   dot-product routine); the cross layer is the full-rank
 *                   DCN-v2 form the paper cites.
 *   backward        Sec. 2.2 (gradients go to the activated rows only); the
 *                   rowwise Adagrad rule is this build's reading, the paper
 *                   names no sparse optimizer.
 *
 * Pins (tests/test_oracle_*.py): hand-computed bags, identity-table histogram,
 * length-1 gather, torch embedding_bag, tower-concatenation invariant, Gram
 * symmetry / orthonormal rows, cross-layer closed forms, numpy stable argsort
 * and unique, gradient-sum conservation, finite differences, textbook Adagrad
 * at D = 1.  Unpinned conventions (not derivable from the paper): eps outside
 * the square root and mean (not sum) of squares in the Adagrad state; dots
 * placed before the flattened features in the dot-TM input.
 *
 * All floating point is accumulated in double; the caller rounds once to the
 * output type.  Element types: 0 = float32, 1 = IEEE half, 2 = bfloat16.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_F32 = 0, ORC_F16 = 1, ORC_BF16 = 2 };

int oracle_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void oracle_set_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

static double half_to_double(uint16_t h) {
  int sign = (h >> 15) & 1, ex = (h >> 10) & 0x1f, man = h & 0x3ff;
  double v;
  if (ex == 0) v = ldexp((double)man, -24);                 /* subnormal / zero */
  else if (ex == 31) v = man ? NAN : INFINITY;
  else v = ldexp((double)(man | 0x400), ex - 25);
  return sign ? -v : v;
}

static double bf16_to_double(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, 4);
  return (double)f;
}

static double elt(const void* base, int dtype, int64_t i) {
  switch (dtype) {
    case ORC_F32: return (double)((const float*)base)[i];
    case ORC_F16: return half_to_double(((const uint16_t*)base)[i]);
    default:      return bf16_to_double(((const uint16_t*)base)[i]);
  }
}

/* Decode n stored elements to double (exact). */
void oracle_decode(const void* src, int dtype, int64_t n, double* dst) {
  for (int64_t i = 0; i < n; ++i) dst[i] = elt(src, dtype, i);
}

/* ---------------------------------------------------------------- lookup -- */

/* Untowered lookup: V[b][f][:] = sum over the ids of bag (f, b) of the rows of
 * table f.  Output is [B][sum_f D_f], features in table order.  A repeated id
 * is added each time it occurs; an empty bag gives zeros. */
void oracle_lookup_global(int32_t F, const int32_t* dims, int dtype,
                          const void* const* tables, const int32_t* indices,
                          const int64_t* offsets, int64_t B, double* out) {
  int64_t width = 0;
  for (int32_t f = 0; f < F; ++f) width += dims[f];
#pragma omp parallel for schedule(static)
  for (int64_t b = 0; b < B; ++b) {
    int64_t col = 0;
    for (int32_t f = 0; f < F; ++f) {
      int32_t D = dims[f];
      double* o = out + b * width + col;
      for (int32_t d = 0; d < D; ++d) o[d] = 0.0;
      for (int64_t j = offsets[(int64_t)f * B + b]; j < offsets[(int64_t)f * B + b + 1]; ++j)
        for (int32_t d = 0; d < D; ++d)
          o[d] += elt(tables[f], dtype, (int64_t)indices[j] * D + d);
      col += D;
    }
  }
}

/* Towered lookup: tower t owns the tables with table_to_tower[f] == t, in
 * ascending table id (= slot order).  For every sample the tower's pooled
 * vectors are concatenated, and towers are laid out one after another:
 * out = [T][B][W_t], W_t = sum of the tower's dims. */
void oracle_lookup_towered(int32_t F, const int32_t* dims, int dtype,
                           const void* const* tables, int32_t T,
                           const int32_t* table_to_tower, const int32_t* indices,
                           const int64_t* offsets, int64_t B, double* out) {
  int64_t base = 0;
  for (int32_t t = 0; t < T; ++t) {
    int64_t Wt = 0;
    for (int32_t f = 0; f < F; ++f)
      if (table_to_tower[f] == t) Wt += dims[f];
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b) {
      int64_t col = 0;
      for (int32_t f = 0; f < F; ++f) {
        if (table_to_tower[f] != t) continue;
        int32_t D = dims[f];
        double* o = out + base + b * Wt + col;
        for (int32_t d = 0; d < D; ++d) {
          double s = 0.0;
          for (int64_t j = offsets[(int64_t)f * B + b]; j < offsets[(int64_t)f * B + b + 1]; ++j)
            s += elt(tables[f], dtype, (int64_t)indices[j] * D + d);
          o[d] = s;
        }
        col += D;
      }
    }
    base += B * Wt;
  }
}

/* ---------------------------------------------------------- tower modules -- */

/* y[b][o] = bias[o] + sum_i W[o][i] x[b][i]; optional ReLU. */
void oracle_tm_linear(int64_t B, int32_t in, int32_t out, const double* x,
                      const double* W, const double* bias, int relu, double* y) {
#pragma omp parallel for schedule(static)
  for (int64_t b = 0; b < B; ++b)
    for (int32_t o = 0; o < out; ++o) {
      double s = bias[o];
      for (int32_t i = 0; i < in; ++i) s += W[(int64_t)o * in + i] * x[b * in + i];
      y[b * out + o] = (relu && s < 0.0) ? 0.0 : s;
    }
}

/* Dot-product tower module.  x[b] is read as nf features of n values; the
 * nf(nf-1)/2 dot products of distinct features (i < j, row-major in (i, j))
 * are placed in front of the flattened features, and that vector z goes
 * through a linear layer.  z (width nf(nf-1)/2 + nf*n) is also returned. */
void oracle_tm_dot_linear(int64_t B, int32_t nf, int32_t n, int32_t out,
                          const double* x, const double* W, const double* bias,
                          double* z, double* y) {
  int32_t np = nf * (nf - 1) / 2, kin = np + nf * n;
#pragma omp parallel for schedule(static)
  for (int64_t b = 0; b < B; ++b) {
    const double* xb = x + b * (int64_t)nf * n;
    double* zb = z + b * (int64_t)kin;
    int32_t p = 0;
    for (int32_t i = 0; i < nf; ++i)
      for (int32_t j = i + 1; j < nf; ++j) {
        double s = 0.0;
        for (int32_t k = 0; k < n; ++k) s += xb[i * n + k] * xb[j * n + k];
        zb[p++] = s;
      }
    for (int32_t k = 0; k < nf * n; ++k) zb[np + k] = xb[k];
    for (int32_t o = 0; o < out; ++o) {
      double s = bias[o];
      for (int32_t i = 0; i < kin; ++i) s += W[(int64_t)o * kin + i] * zb[i];
      y[b * out + o] = s;
    }
  }
}

/* One cross layer: xn = x0 (.) (W x + bias) + x, all vectors of width d. */
void oracle_cross_layer(int64_t B, int32_t d, const double* x0, const double* x,
                        const double* W, const double* bias, double* xn) {
#pragma omp parallel for schedule(static)
  for (int64_t b = 0; b < B; ++b)
    for (int32_t o = 0; o < d; ++o) {
      double s = bias[o];
      for (int32_t i = 0; i < d; ++i) s += W[(int64_t)o * d + i] * x[b * d + i];
      xn[b * d + o] = x0[b * d + o] * s + x[b * d + o];
    }
}

/* ---------------------------------------------------------------- backward -- */

typedef struct { int64_t key; int64_t pos; } kp_t;

static void merge_sort(kp_t* a, kp_t* tmp, int64_t n) {
  if (n < 2) return;
  int64_t h = n / 2;
  merge_sort(a, tmp, h);
  merge_sort(a + h, tmp, n - h);
  int64_t i = 0, j = h, k = 0;
  while (i < h && j < n) tmp[k++] = (a[j].key < a[i].key) ? a[j++] : a[i++];  /* left wins ties */
  while (i < h) tmp[k++] = a[i++];
  while (j < n) tmp[k++] = a[j++];
  memcpy(a, tmp, (size_t)n * sizeof(kp_t));
}

/* Keys of all lookups: position j in bag (f, b) has key (f, indices[j]).
 * Stable ascending sort by (table, row); equal keys keep position order. */
int oracle_sort_keys(int32_t F, int64_t B, const int32_t* indices,
                     const int64_t* offsets, int64_t* sorted_table,
                     int64_t* sorted_row, int64_t* sorted_pos) {
  int64_t nnz = offsets[(int64_t)F * B];
  kp_t* a = (kp_t*)malloc((size_t)(nnz + 1) * sizeof(kp_t));
  kp_t* tmp = (kp_t*)malloc((size_t)(nnz + 1) * sizeof(kp_t));
  if (!a || !tmp) { free(a); free(tmp); return 1; }
  for (int32_t f = 0; f < F; ++f)
    for (int64_t j = offsets[(int64_t)f * B]; j < offsets[(int64_t)(f + 1) * B]; ++j) {
      a[j].key = ((int64_t)f << 32) | (uint32_t)indices[j];
      a[j].pos = j;
    }
  merge_sort(a, tmp, nnz);
  for (int64_t i = 0; i < nnz; ++i) {
    sorted_table[i] = a[i].key >> 32;
    sorted_row[i] = a[i].key & 0xffffffffLL;
    sorted_pos[i] = a[i].pos;
  }
  free(a); free(tmp);
  return 0;
}

/* Run-length scan of sorted keys: distinct (table, row) pairs, the start of
 * each run (seg_off has U + 1 entries), returns U. */
int64_t oracle_unique(int64_t nnz, const int64_t* sorted_table, const int64_t* sorted_row,
                      int64_t* uniq_table, int64_t* uniq_row, int64_t* seg_off) {
  int64_t U = 0;
  for (int64_t i = 0; i < nnz; ++i)
    if (i == 0 || sorted_table[i] != sorted_table[i - 1] || sorted_row[i] != sorted_row[i - 1]) {
      uniq_table[U] = sorted_table[i];
      uniq_row[U] = sorted_row[i];
      seg_off[U++] = i;
    }
  seg_off[U] = nnz;
  return U;
}

/* Dictionary-accumulated row gradients.  grad is the gradient w.r.t. the
 * towered lookup output (float32, same [T][B][W_t] layout).  Every lookup of
 * row r of table f in bag (f, b) adds that bag's gradient slice to the entry
 * of (f, r).  Entries are created in first-touch order; keys_out/G_out return
 * them (G_out is [n][Dmax], zero-padded past D_f).  Returns the number of
 * entries, or -1 when out of memory. */
int64_t oracle_bwd_accumulate(int32_t F, const int32_t* dims, int32_t T,
                              const int32_t* table_to_tower, const int32_t* indices,
                              const int64_t* offsets, int64_t B, const float* grad,
                              int32_t Dmax, int64_t* key_table, int64_t* key_row,
                              double* G_out) {
  int64_t nnz = offsets[(int64_t)F * B];
  int64_t cap = 16;
  while (cap < 2 * nnz + 2) cap <<= 1;
  int64_t* hkey = (int64_t*)malloc((size_t)cap * sizeof(int64_t));
  int64_t* hval = (int64_t*)malloc((size_t)cap * sizeof(int64_t));
  int64_t* tower_base = (int64_t*)malloc((size_t)(T + 1) * sizeof(int64_t));
  int64_t* Wt = (int64_t*)calloc((size_t)T, sizeof(int64_t));
  int64_t* col = (int64_t*)malloc((size_t)F * sizeof(int64_t));
  if (!hkey || !hval || !tower_base || !Wt || !col) return -1;
  for (int64_t i = 0; i < cap; ++i) hkey[i] = -1;
  for (int32_t f = 0; f < F; ++f) { col[f] = Wt[table_to_tower[f]]; Wt[table_to_tower[f]] += dims[f]; }
  tower_base[0] = 0;
  for (int32_t t = 0; t < T; ++t) tower_base[t + 1] = tower_base[t] + B * Wt[t];

  int64_t n = 0;
  for (int32_t f = 0; f < F; ++f) {
    int32_t t = table_to_tower[f], D = dims[f];
    for (int64_t b = 0; b < B; ++b) {
      const float* g = grad + tower_base[t] + b * Wt[t] + col[f];
      for (int64_t j = offsets[(int64_t)f * B + b]; j < offsets[(int64_t)f * B + b + 1]; ++j) {
        int64_t key = ((int64_t)f << 32) | (uint32_t)indices[j];
        uint64_t h = (uint64_t)key * 0x9E3779B97F4A7C15ULL;
        int64_t s = (int64_t)(h >> 20) & (cap - 1);
        while (hkey[s] != -1 && hkey[s] != key) s = (s + 1) & (cap - 1);
        if (hkey[s] == -1) {
          hkey[s] = key; hval[s] = n;
          key_table[n] = f; key_row[n] = indices[j];
          for (int32_t d = 0; d < Dmax; ++d) G_out[n * Dmax + d] = 0.0;
          ++n;
        }
        double* acc = G_out + hval[s] * Dmax;
        for (int32_t d = 0; d < D; ++d) acc[d] += (double)g[d];
      }
    }
  }
  free(hkey); free(hval); free(tower_base); free(Wt); free(col);
  return n;
}

/* Rowwise Adagrad on n touched rows.  For row i with summed gradient G[i][0:D]:
 *   state += (1/D) sum_d G[d]^2 ;  w[d] -= lr * G[d] / (sqrt(state) + eps)
 * using the updated state.  w_io [n][Dmax] and state_io [n] are doubles,
 * updated in place; D_of[i] is the row's width. */
void oracle_rowwise_adagrad(int64_t n, int32_t Dmax, const int32_t* D_of,
                            const double* G, double lr, double eps,
                            double* w_io, double* state_io) {
  for (int64_t i = 0; i < n; ++i) {
    int32_t D = D_of[i];
    double ss = 0.0;
    for (int32_t d = 0; d < D; ++d) ss += G[i * Dmax + d] * G[i * Dmax + d];
    state_io[i] += ss / (double)D;
    double denom = sqrt(state_io[i]) + eps;
    for (int32_t d = 0; d < D; ++d) w_io[i * Dmax + d] -= lr * G[i * Dmax + d] / denom;
  }
}
