// Tower Partitioner (paper Sec. 3.3): from a batch of pooled embeddings to a balanced
// feature -> tower map.
//
//   dmt_tp_interaction  device: I = | mean_b Rn_b Rn_b^T |, Rn the per-(sample, feature)
//                       normalised embeddings.  One fused kernel reads the pooled tensor once:
//                       it normalises a 64-feature tile of one sample on the way into LDS (as
//                       float16: the values are at most 1 in magnitude) and feeds the tile to
//                       MFMA, accumulating the 64 x 64 Gram tile over its slice of the batch in
//                       registers; a second kernel sums the slices in a fixed order, divides by
//                       B and takes the absolute value.  At F = 64 the contraction is 64 FLOP
//                       per byte read, so the kernel is bound by reading the pooled tensor.
//   dmt_tp_embed        host, float64: D = f(I), then Adam on the pairwise-distance objective.
//   dmt_tp_kmeans       host, float64: constrained K-means; the assignment step is solved
//                       exactly as a square assignment problem over (group, slot) pairs.
//
// The host steps work on |F| x |F| and |F| x n numbers (|F| a few hundred at most); only the
// interaction matrix touches batch-sized data.
#include <math.h>

#include <algorithm>
#include <limits>
#include <vector>

#include "dmt_internal.h"
#include "dmt_device_utils.h"

namespace {

constexpr int kBlock = 256;
constexpr int kTile = 64;                    // features per Gram tile side
constexpr int kTargetBlocks = 1024;          // blocks per launch the batch is sliced for

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));

__host__ __device__ inline int tp_pair_index(int ti, int tj, int nt) {   // ti <= tj
  return ti * nt - ti * (ti - 1) / 2 + (tj - ti);
}

// 8 consecutive elements of a row as float32.
template <int DT>
__device__ __forceinline__ void load8(const void* base, int64_t off, float (&x)[8]) {
  if constexpr (DT == DMT_F32) {
    const float4 a = dmt::gload((const float4*)((const float*)base + off));
    const float4 b = dmt::gload((const float4*)((const float*)base + off) + 1);
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
    x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
  } else {
    dmt::decode_chunk<DT>(x, dmt::gload((const uint4*)((const uint16_t*)base + off)));
  }
}

// Gram tiles of the normalised embeddings.  Block (pair, slice): features [64 ti, 64 ti + 64)
// against [64 tj, 64 tj + 64), ti <= tj, over samples [slice * per, (slice + 1) * per).
// Thread layout of the staging step: LPR = 4 NP lanes per feature row, 8 elements per lane,
// 256 / LPR rows per pass, NP passes per tile.  LDS rows hold Npad = N rounded up to 16 halfs
// (zeros past N) plus 8 halfs of padding.
template <int DT, int NP>
__global__ __launch_bounds__(kBlock) void tp_gram(const DmtTableMeta* __restrict__ meta,
                                                  const void* __restrict__ pooled, int64_t B,
                                                  int F, int N, int nt, int npairs, int64_t per,
                                                  float* __restrict__ partial) {
  constexpr int LPR = 4 * NP, RP = kBlock / LPR;
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
  __shared__ int64_t s_base[2 * kTile];
  __shared__ int32_t s_pitch[2 * kTile];
  const int pair = blockIdx.x % npairs;
  const int64_t slice = blockIdx.x / npairs;
  int ti = 0;
  while (tp_pair_index(ti + 1, ti + 1, nt) <= pair && ti + 1 < nt) ++ti;
  const int tj = ti + (pair - tp_pair_index(ti, ti, nt));
  const bool diag = ti == tj;
  const int npad = (N + 15) & ~15, ldx = npad + 8;
  uint16_t* Xi = lds;
  uint16_t* Xj = diag ? lds : lds + kTile * ldx;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid < 2 * kTile) {
    const int f = (tid < kTile ? ti : tj) * kTile + (tid & (kTile - 1));
    int64_t base = 0;
    int32_t pitch = 0;
    if (f < F) {
      const DmtTableMeta m = meta[f];
      base = m.out_prefix * B + m.col_off;
      pitch = m.tower_width;
    }
    s_base[tid] = base;
    s_pitch[tid] = pitch;
  }
  __syncthreads();

  const int chunk = tid % LPR, row0 = tid / LPR;
  const bool cin = chunk * 8 < N;
  floatx16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  const int wi = wave >> 1, wj = wave & 1;
  const uint16_t* pa = Xi + (32 * wi + (lane & 31)) * ldx + (lane >> 5) * 8;
  const uint16_t* pb = Xj + (32 * wj + (lane & 31)) * ldx + (lane >> 5) * 8;

  auto stage = [&](int which, int64_t b, uint16_t* Xs) __attribute__((always_inline)) {
    float x[NP][8];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      const int row = p * RP + row0;
      const int f = (which ? tj : ti) * kTile + row;
      if (cin && f < F) {
        load8<DT>(pooled, s_base[which * kTile + row] + b * s_pitch[which * kTile + row] + chunk * 8,
                  x[p]);
      } else {
#pragma unroll
        for (int q = 0; q < 8; ++q) x[p][q] = 0.f;
      }
    }
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      float ss = 0.f;
#pragma unroll
      for (int q = 0; q < 8; ++q) ss += x[p][q] * x[p][q];
#pragma unroll
      for (int o = 1; o < LPR; o <<= 1) ss += __shfl_xor(ss, o);
      const float inv = ss > 0.f ? 1.0f / sqrtf(ss) : 0.f;
      if (chunk * 8 < npad) {
        const int row = p * RP + row0;
        *(uint4*)(Xs + row * ldx + chunk * 8) =
            make_uint4(dmt::pack2<DMT_F16>(x[p][0] * inv, x[p][1] * inv),
                       dmt::pack2<DMT_F16>(x[p][2] * inv, x[p][3] * inv),
                       dmt::pack2<DMT_F16>(x[p][4] * inv, x[p][5] * inv),
                       dmt::pack2<DMT_F16>(x[p][6] * inv, x[p][7] * inv));
      }
    }
  };

  const int64_t b_begin = slice * per, b_end = b_begin + per < B ? b_begin + per : B;
  for (int64_t b = b_begin; b < b_end; ++b) {
    __syncthreads();                         // the previous sample's tile has been consumed
    stage(0, b, Xi);
    if (!diag) stage(1, b, Xj);
    __syncthreads();
    for (int k = 0; k < npad; k += 16) {
      const uint4 a = *(const uint4*)(pa + k);
      const uint4 c = *(const uint4*)(pb + k);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(halfx8, a),
                                                   __builtin_bit_cast(halfx8, c), acc, 0, 0, 0);
    }
  }

  // lane holds column lane % 32 of rows (v / 4) * 8 + (lane / 32) * 4 + v % 4 of its 32 x 32 tile
  float* out = partial + ((int64_t)slice * npairs + pair) * (kTile * kTile);
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int r = 32 * wi + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
    out[r * kTile + 32 * wj + (lane & 31)] = acc[v];
  }
}

// I[i][j] = | sum over the batch slices of the Gram entry | / B.  Entry (i, j) and (j, i) are
// both read from the tile element (min, max), so the result is exactly symmetric.
__global__ __launch_bounds__(kBlock) void tp_finish(const float* __restrict__ partial, int F,
                                                    int nt, int npairs, int64_t nslices,
                                                    float inv_b, float* __restrict__ I) {
  const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (e >= (int64_t)F * F) return;
  const int i = (int)(e / F), j = (int)(e % F);
  const int a = i < j ? i : j, c = i < j ? j : i;
  const float* p = partial + (int64_t)tp_pair_index(a / kTile, c / kTile, nt) * (kTile * kTile) +
                   (a % kTile) * kTile + (c % kTile);
  float s = 0.f;
  for (int64_t q = 0; q < nslices; ++q) s += p[q * npairs * (kTile * kTile)];
  I[e] = fabsf(s * inv_b);
}

struct TpShape {
  int N, nt, npairs;
  int64_t per, nslices;
  size_t bytes;
};

// Every table must have the same embedding dim (the cosine kernel pairs any two features), a
// multiple of 8 up to 512, so that rows split into aligned 8-element chunks.
dmt_status tp_shape(const dmt_plan* p, int64_t B, TpShape& s) {
  if (p->classes.size() != 1) return DMT_ENOTSUP;
  s.N = p->classes[0].D;
  if (s.N % 8 != 0 || s.N > 512) return DMT_ENOTSUP;
  for (const DmtTableMeta& m : p->meta)
    if (m.col_off % 8 != 0 || m.tower_width % 8 != 0) return DMT_ENOTSUP;
  s.nt = (p->F + kTile - 1) / kTile;
  s.npairs = s.nt * (s.nt + 1) / 2;
  const int64_t want = std::max<int64_t>(1, kTargetBlocks / s.npairs);
  s.per = (B + want - 1) / want;
  s.nslices = (B + s.per - 1) / s.per;
  s.bytes = sizeof(float) * (size_t)s.nslices * s.npairs * kTile * kTile;
  return DMT_OK;
}

template <int DT, int NP>
void launch_gram(const dmt_plan* p, const void* pooled, int64_t B, const TpShape& sh,
                 float* partial, hipStream_t s) {
  const int npad = (sh.N + 15) & ~15;
  const size_t lds = sizeof(uint16_t) * 2 * kTile * (npad + 8);
  static bool configured = false;           // wide rows need more than the default LDS limit
  if (!configured) {
    (void)hipFuncSetAttribute((const void*)tp_gram<DT, NP>,
                              hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)(sizeof(uint16_t) * 2 * kTile * (NP * 32 + 8)));
    configured = true;
  }
  hipLaunchKernelGGL((tp_gram<DT, NP>), dim3((unsigned)(sh.nslices * sh.npairs)), dim3(kBlock), lds,
                     s, p->d_meta, pooled, B, p->F, sh.N, sh.nt, sh.npairs, sh.per, partial);
}

template <int DT>
void launch_gram_dt(const dmt_plan* p, const void* pooled, int64_t B, const TpShape& sh,
                    float* partial, hipStream_t s) {
  if (sh.N <= 32) launch_gram<DT, 1>(p, pooled, B, sh, partial, s);
  else if (sh.N <= 64) launch_gram<DT, 2>(p, pooled, B, sh, partial, s);
  else if (sh.N <= 128) launch_gram<DT, 4>(p, pooled, B, sh, partial, s);
  else if (sh.N <= 256) launch_gram<DT, 8>(p, pooled, B, sh, partial, s);
  else launch_gram<DT, 16>(p, pooled, B, sh, partial, s);
}

// ------------------------------------------------------------------ host: assignment

// Minimum-cost perfect matching of an n x n cost matrix (rows to columns) by shortest
// augmenting paths with row / column potentials, O(n^3).  col_of_row[r] = column of row r.
void assign_square(const std::vector<double>& cost, int n, std::vector<int>& col_of_row) {
  const double inf = std::numeric_limits<double>::infinity();
  std::vector<double> u(n + 1, 0.0), v(n + 1, 0.0), minv(n + 1);
  std::vector<int> row_of_col(n + 1, 0), prev(n + 1, 0);
  std::vector<char> used(n + 1);
  for (int r = 1; r <= n; ++r) {
    row_of_col[0] = r;
    int c0 = 0;
    std::fill(minv.begin(), minv.end(), inf);
    std::fill(used.begin(), used.end(), 0);
    do {
      used[c0] = 1;
      const int r0 = row_of_col[c0];
      double delta = inf;
      int c1 = 0;
      for (int c = 1; c <= n; ++c) {
        if (used[c]) continue;
        const double red = cost[(size_t)(r0 - 1) * n + (c - 1)] - u[r0] - v[c];
        if (red < minv[c]) { minv[c] = red; prev[c] = c0; }
        if (minv[c] < delta) { delta = minv[c]; c1 = c; }
      }
      for (int c = 0; c <= n; ++c) {
        if (used[c]) { u[row_of_col[c]] += delta; v[c] -= delta; }
        else minv[c] -= delta;
      }
      c0 = c1;
    } while (row_of_col[c0] != 0);
    do {
      const int c1 = prev[c0];
      row_of_col[c0] = row_of_col[c1];
      c0 = c1;
    } while (c0 != 0);
  }
  col_of_row.assign(n, 0);
  for (int c = 1; c <= n; ++c) col_of_row[row_of_col[c] - 1] = c - 1;
}

void size_bounds(int F, int T, double R, int& smin, int& smax) {
  smin = std::min((int)ceil((double)F / ((double)(T - 1) + R) - 1e-12), F / T);
  smax = std::max((int)floor(R * smin + 1e-12), (F + T - 1) / T);
}

}  // namespace

extern "C" size_t dmt_tp_workspace_bytes(const dmt_plan* plan, int64_t B) {
  TpShape sh;
  if (!plan || B <= 0 || tp_shape(plan, B, sh) != DMT_OK) return 0;
  return sh.bytes;
}

extern "C" dmt_status dmt_tp_interaction(const dmt_plan* plan, const void* pooled, int64_t B,
                                         dmt_dtype pooled_dtype, float* interaction,
                                         void* workspace, size_t workspace_bytes, void* stream) {
  if (!plan || !pooled || !interaction || !workspace) return DMT_EINVAL;
  if (B <= 0 || B > plan->max_batch || !plan->bound) return DMT_EINVAL;
  if (pooled_dtype != DMT_F32 && pooled_dtype != DMT_F16 && pooled_dtype != DMT_BF16)
    return DMT_EINVAL;
  if (((uintptr_t)pooled & 15) || ((uintptr_t)workspace & 15) || ((uintptr_t)interaction & 3))
    return DMT_EINVAL;
  TpShape sh;
  const dmt_status st = tp_shape(plan, B, sh);
  if (st != DMT_OK) return st;
  if (workspace_bytes < sh.bytes) return DMT_ENOMEM;
  hipStream_t s = (hipStream_t)stream;
  float* partial = (float*)workspace;
  {
    DmtScope scope(plan, DMT_K_TP_GRAM, s);
    if (pooled_dtype == DMT_F32) launch_gram_dt<DMT_F32>(plan, pooled, B, sh, partial, s);
    else if (pooled_dtype == DMT_F16) launch_gram_dt<DMT_F16>(plan, pooled, B, sh, partial, s);
    else launch_gram_dt<DMT_BF16>(plan, pooled, B, sh, partial, s);
  }
  {
    DmtScope scope(plan, DMT_K_TP_FINISH, s);
    const int64_t n = (int64_t)plan->F * plan->F;
    hipLaunchKernelGGL(tp_finish, dim3((unsigned)((n + kBlock - 1) / kBlock)), dim3(kBlock), 0, s,
                       partial, plan->F, sh.nt, sh.npairs, sh.nslices, (float)(1.0 / (double)B),
                       interaction);
  }
  return hipGetLastError() == hipSuccess ? DMT_OK : DMT_EHIP;
}

extern "C" dmt_status dmt_tp_embed(const float* interaction, int32_t F, dmt_tp_strategy strategy,
                                   int32_t n, int32_t steps, double lr, const double* x0,
                                   double* x, double* stress) {
  if (!interaction || !x0 || !x || F <= 0 || n <= 0 || steps < 0 || !(lr > 0.0)) return DMT_EINVAL;
  if (strategy != DMT_TP_DIVERSE && strategy != DMT_TP_COHERENT) return DMT_EINVAL;
  const double beta1 = 0.9, beta2 = 0.999, eps = 1e-8;
  // target distance of the pair (i, j), j < i, from the entry below the diagonal
  auto target = [&](int i, int j) {
    const double v = (double)interaction[(size_t)i * F + j];
    return strategy == DMT_TP_DIVERSE ? v : 1.0 - v;
  };
  const size_t len = (size_t)F * n;
  std::vector<double> g(len), m(len, 0.0), v(len, 0.0);
  for (size_t e = 0; e < len; ++e) x[e] = x0[e];
  double b1t = 1.0, b2t = 1.0;
  for (int t = 1; t <= steps; ++t) {
    std::fill(g.begin(), g.end(), 0.0);
    for (int i = 0; i < F; ++i) {
      for (int j = 0; j < i; ++j) {
        double d2 = 0.0;
        for (int k = 0; k < n; ++k) {
          const double df = x[(size_t)i * n + k] - x[(size_t)j * n + k];
          d2 += df * df;
        }
        const double d = sqrt(d2);
        if (!(d > 0.0)) continue;
        const double c = 2.0 * (d - target(i, j)) / d;
        for (int k = 0; k < n; ++k) {
          const double df = x[(size_t)i * n + k] - x[(size_t)j * n + k];
          g[(size_t)i * n + k] += c * df;
          g[(size_t)j * n + k] -= c * df;
        }
      }
    }
    b1t *= beta1;
    b2t *= beta2;
    for (size_t e = 0; e < len; ++e) {
      m[e] = beta1 * m[e] + (1.0 - beta1) * g[e];
      v[e] = beta2 * v[e] + (1.0 - beta2) * g[e] * g[e];
      const double mh = m[e] / (1.0 - b1t), vh = v[e] / (1.0 - b2t);
      x[e] -= lr * mh / (sqrt(vh) + eps);
    }
  }
  if (stress) {
    double s = 0.0;
    for (int i = 0; i < F; ++i)
      for (int j = 0; j < i; ++j) {
        double d2 = 0.0;
        for (int k = 0; k < n; ++k) {
          const double df = x[(size_t)i * n + k] - x[(size_t)j * n + k];
          d2 += df * df;
        }
        const double e = sqrt(d2) - target(i, j);
        s += e * e;
      }
    *stress = s;
  }
  return DMT_OK;
}

extern "C" dmt_status dmt_tp_kmeans(const double* x, int32_t F, int32_t n, int32_t T,
                                    double ratio, const double* centres0, int32_t max_iter,
                                    int32_t* table_to_tower, double* centres,
                                    int32_t* iterations) {
  if (!x || !centres0 || !table_to_tower || F <= 0 || n <= 0 || T <= 0 || T > F) return DMT_EINVAL;
  if (!(ratio >= 1.0) || max_iter <= 0) return DMT_EINVAL;
  int smin, smax;
  size_bounds(F, T, ratio, smin, smax);
  const int ns = T * smax;                  // slots = rows of the square problem
  if ((int64_t)ns * ns > ((int64_t)1 << 26)) return DMT_ENOTSUP;
  std::vector<double> C(centres0, centres0 + (size_t)T * n), d2((size_t)F * T), cost((size_t)ns * ns);
  std::vector<int> col, labels(F, -1), now(F), count(T);
  int it = 0;
  while (it < max_iter) {
    double total = 0.0;
    for (int i = 0; i < F; ++i)
      for (int h = 0; h < T; ++h) {
        double s = 0.0;
        for (int k = 0; k < n; ++k) {
          const double df = x[(size_t)i * n + k] - C[(size_t)h * n + k];
          s += df * df;
        }
        d2[(size_t)i * T + h] = s;
        total += s;
      }
    // slot c belongs to group c / smax and must be taken if c % smax < smin; rows past F are
    // dummies: free in an optional slot, dearer than any assignment of the real points in a
    // mandatory one
    const double big = 1.0 + total;
    for (int r = 0; r < ns; ++r)
      for (int c = 0; c < ns; ++c)
        cost[(size_t)r * ns + c] = r < F ? d2[(size_t)r * T + c / smax] : (c % smax < smin ? big : 0.0);
    assign_square(cost, ns, col);
    for (int i = 0; i < F; ++i) now[i] = col[i] / smax;
    ++it;
    if (now == labels) break;
    labels = now;
    std::fill(count.begin(), count.end(), 0);
    std::vector<double> sum((size_t)T * n, 0.0);
    for (int i = 0; i < F; ++i) {
      ++count[labels[i]];
      for (int k = 0; k < n; ++k) sum[(size_t)labels[i] * n + k] += x[(size_t)i * n + k];
    }
    for (int h = 0; h < T; ++h)
      if (count[h] > 0)
        for (int k = 0; k < n; ++k) C[(size_t)h * n + k] = sum[(size_t)h * n + k] / count[h];
  }
  for (int i = 0; i < F; ++i) table_to_tower[i] = labels[i];
  if (centres) std::copy(C.begin(), C.end(), centres);
  if (iterations) *iterations = it;
  return DMT_OK;
}
