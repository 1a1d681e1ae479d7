// Tower Partitioner (paper Sec. 3.3): from a batch of pooled embeddings to a balanced
// feature -> tower map.
//
//   dmt_tp_interaction  device: I = | mean_b Rn_b Rn_b^T |, Rn the per-(sample, feature)
//                       normalised embeddings.  One fused kernel reads the pooled tensor once:
//                       it stages a 64-feature tile of one sample in LDS, computing the row
//                       norms on the way, multiplies the tile on MFMA and adds the products,
//                       scaled by the two inverse norms, to the 64 x 64 Gram tile it keeps in
//                       registers over its slice of the batch; a second kernel sums the slices
//                       in a fixed order, divides by B and takes the absolute value.  At
//                       F = 64 the contraction is 64 FLOP per byte read, so the kernel is bound
//                       by reading the pooled tensor.  With 65 ... 256 features a 16-wave block
//                       stages all of them, so that the tensor is still read only once
//                       (tp_gram_wide); beyond that, pairs of 64-feature tiles.
//   dmt_tp_embed        host, float64: D = f(I), then Adam on the pairwise-distance objective.
//   dmt_tp_kmeans       host, float64: constrained K-means; the assignment step is solved
//                       exactly as a square assignment problem over (group, slot) pairs.
//
// The host steps work on |F| x |F| and |F| x n numbers (|F| a few hundred at most); only the
// interaction matrix touches batch-sized data.
#include <math.h>

#include <algorithm>
#include <limits>
#include <new>
#include <type_traits>
#include <vector>

#include "dmt_internal.h"
#include "dmt_device_utils.h"

namespace {

constexpr int kBlock = 256;
constexpr int kTile = 64;                    // features per Gram tile side
constexpr int kWideBlocks = 256;             // tp_gram_wide: one block per CU
constexpr int kTargetBlocks = 1024;          // resident blocks: 4 per CU (LDS 34 KB each at N = 128)

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
typedef _Float16 halfx2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

__host__ __device__ inline int tp_pair_index(int ti, int tj, int nt) {   // ti <= tj
  return ti * nt - ti * (ti - 1) / 2 + (tj - ti);
}

// One lane's 8 consecutive elements of a row, as loaded: one 16-byte chunk of 16-bit elements,
// two of float32.
template <int DT> struct Raw8 { uint4 v[DT == DMT_F32 ? 2 : 1]; };

// NT: the tensor is larger than the caches and read once (nontemporal loads keep it from
// sweeping them); a tensor the lookup has just written is better taken from the caches.
template <int DT, bool NT>
__device__ __forceinline__ Raw8<DT> fetch8(const void* base, int64_t off) {
  Raw8<DT> r;
  auto ld = [](const uint4* p) __attribute__((always_inline)) {
    if constexpr (NT) return dmt::nt_load(p);
    else return dmt::gload(p);
  };
  if constexpr (DT == DMT_F32) {
    r.v[0] = ld((const uint4*)((const float*)base + off));
    r.v[1] = ld((const uint4*)((const float*)base + off) + 1);
  } else {
    r.v[0] = ld((const uint4*)((const uint16_t*)base + off));
  }
  return r;
}

template <int DT>
__device__ __forceinline__ void decode8(const Raw8<DT>& r, float (&x)[8]) {
  if constexpr (DT == DMT_F32) {
    x[0] = __uint_as_float(r.v[0].x); x[1] = __uint_as_float(r.v[0].y);
    x[2] = __uint_as_float(r.v[0].z); x[3] = __uint_as_float(r.v[0].w);
    x[4] = __uint_as_float(r.v[1].x); x[5] = __uint_as_float(r.v[1].y);
    x[6] = __uint_as_float(r.v[1].z); x[7] = __uint_as_float(r.v[1].w);
  } else {
    dmt::decode_chunk<DT>(x, r.v[0]);
  }
}

// Sum of `v` over the LPR consecutive lanes (LPR = 4 ... 64, aligned) that hold one row.
template <int LPR>
__device__ __forceinline__ float row_group_sum(float v) {
  auto dpp = [](float x, auto ctrl) __attribute__((always_inline)) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), decltype(ctrl)::value,
                                                      0xf, 0xf, true));
  };
  v += dpp(v, std::integral_constant<int, 0xB1>{});                      // lane ^ 1
  v += dpp(v, std::integral_constant<int, 0x4E>{});                      // lane ^ 2
  if constexpr (LPR >= 8) v += dpp(v, std::integral_constant<int, 0x141>{});   // mirror in 8
  if constexpr (LPR >= 16) v += dpp(v, std::integral_constant<int, 0x140>{});  // mirror in 16
  if constexpr (LPR >= 32) v += __shfl_xor(v, 16);
  if constexpr (LPR >= 64) v += __shfl_xor(v, 32);
  return v;
}

// Sum of squares of the 8 elements of a 16-byte chunk of 16-bit elements.
template <int DT>
__device__ __forceinline__ float sumsq8(uint4 r) {
  float s = 0.f;
  const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    if constexpr (DT == DMT_F16) {
      const halfx2 h = __builtin_bit_cast(halfx2, w[q]);
      s = __builtin_amdgcn_fdot2(h, h, s, false);
    } else {
      const bf16x2 h = __builtin_bit_cast(bf16x2, w[q]);
      s = __builtin_amdgcn_fdot2_f32_bf16(h, h, s, false);
    }
  }
  return s;
}

// Gram tiles of the normalised embeddings.  Block (pair, slice): features [TF ti, TF ti + TF)
// against [TF tj, TF tj + TF), ti <= tj, over samples [slice * per, (slice + 1) * per); TF is
// 64 (one tile covers up to 64 features) or 128 (more features: fewer, larger tiles re-read
// the pooled rows less often).
//
// Per sample the block stages its two feature tiles in LDS, multiplies them on MFMA
// (4 waves, TF / 64 squared 32 x 32 sub-tiles each) and adds  product * inv_norm(row) * inv_norm(column)  to
// its running sum.  16-bit rows go to LDS and into the matrix cores exactly as they were
// loaded (their products are exact in float32); only their norms are computed on the way.
// float32 rows are normalised first and stored as float16, with scales of one.
// Thread layout of the staging step: LPR = 4 NP lanes per feature row, 8 elements per lane,
// 256 / LPR rows per pass.  LDS rows hold Npad = N rounded up to 16
// elements (zeros past N) plus 8 of padding.  The next sample's rows are loaded into
// registers while the current one is multiplied, so global loads stay in flight across the
// barriers.  Consecutive block ids run on different XCDs: the blocks of one batch slice (one
// per tile pair, all reading the same samples) get ids that are equal mod 8, so that they
// share one XCD's L2.
template <int DT, int NP, int TF>
__global__ __launch_bounds__(kBlock) void tp_gram(const DmtTableMeta* __restrict__ meta,
                                                  const void* __restrict__ pooled, int64_t B,
                                                  int F, int N, int nt, int npairs, int64_t per,
                                                  int64_t nslices, float* __restrict__ partial) {
  constexpr int LPR = 4 * NP, RP = kBlock / LPR, PT = TF / RP;   // PT staging passes per tile
  constexpr int SW = TF / 64;                // 32 x 32 sub-tiles per wave and direction
  constexpr bool kRaw = DT != DMT_F32;
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
  __shared__ int64_t s_base[2 * TF];
  __shared__ int32_t s_pitch[2 * TF];
  __shared__ __attribute__((aligned(16))) float s_inv[2][TF];
  const int64_t rest = blockIdx.x >> 3;
  const int pair = (int)(rest % npairs);
  const int64_t slice = (rest / npairs) * 8 + (blockIdx.x & 7);
  if (slice >= nslices) return;
  int ti = 0;
  while (ti + 1 < nt && tp_pair_index(ti + 1, ti + 1, nt) <= pair) ++ti;
  const int tj = ti + (pair - tp_pair_index(ti, ti, nt));
  const bool diag = ti == tj;
  const int npad = (N + 15) & ~15, ldx = npad + 8;
  uint16_t* Xi = lds;
  uint16_t* Xj = diag ? lds : lds + TF * ldx;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid < 2 * TF) {
    const int f = (tid < TF ? ti : tj) * TF + (tid & (TF - 1));
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
  floatx16 total[SW][SW];
#pragma unroll
  for (int i = 0; i < SW; ++i)
#pragma unroll
    for (int j = 0; j < SW; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) total[i][j][v] = 0.f;
  // the wave's SW x SW sub-tiles cover rows [32 SW wi, +32 SW) x columns [32 SW wj, +32 SW)
  const int wi = wave >> 1, wj = wave & 1;
  const uint16_t* pa = Xi + (32 * SW * wi + (lane & 31)) * ldx + (lane >> 5) * 8;
  const uint16_t* pb = Xj + (32 * SW * wj + (lane & 31)) * ldx + (lane >> 5) * 8;
  const float* inv_col = &s_inv[diag ? 0 : 1][32 * SW * wj + (lane & 31)];
  const float* inv_row = &s_inv[0][32 * SW * wi + (lane >> 5) * 4];

  Raw8<DT> raw[2][PT];
  auto fetch = [&](int which, int64_t b) __attribute__((always_inline)) {
#pragma unroll
    for (int p = 0; p < PT; ++p) {
      const int row = p * RP + row0;
      const int f = (which ? tj : ti) * TF + row;
      if (cin && f < F) {
        raw[which][p] = fetch8<DT, false>(
            pooled, s_base[which * TF + row] + b * s_pitch[which * TF + row] + chunk * 8);
      } else {
#pragma unroll
        for (int q = 0; q < (DT == DMT_F32 ? 2 : 1); ++q) raw[which][p].v[q] = make_uint4(0, 0, 0, 0);
      }
    }
  };
  auto commit = [&](int which, uint16_t* Xs) __attribute__((always_inline)) {
#pragma unroll
    for (int p = 0; p < PT; ++p) {
      const int row = p * RP + row0;
      if constexpr (kRaw) {
        const uint4 r = raw[which][p].v[0];
        const float ss = row_group_sum<LPR>(sumsq8<DT>(r));
        if (chunk * 8 < npad) *(uint4*)(Xs + row * ldx + chunk * 8) = r;
        if (chunk == 0) s_inv[which][row] = ss > 0.f ? __builtin_amdgcn_rsqf(ss) : 0.f;
      } else {
        float x[8];
        decode8<DT>(raw[which][p], x);
        float ss = 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q) ss += x[q] * x[q];
        ss = row_group_sum<LPR>(ss);
        const float inv = ss > 0.f ? __builtin_amdgcn_rsqf(ss) : 0.f;
        if (chunk * 8 < npad) {
          *(uint4*)(Xs + row * ldx + chunk * 8) =
              make_uint4(dmt::pack2<DMT_F16>(x[0] * inv, x[1] * inv),
                         dmt::pack2<DMT_F16>(x[2] * inv, x[3] * inv),
                         dmt::pack2<DMT_F16>(x[4] * inv, x[5] * inv),
                         dmt::pack2<DMT_F16>(x[6] * inv, x[7] * inv));
        }
        if (chunk == 0) s_inv[which][row] = 1.0f;
      }
    }
  };

  const int64_t b_begin = slice * per, b_end = b_begin + per < B ? b_begin + per : B;
  if (b_begin < b_end) {
    fetch(0, b_begin);
    if (!diag) fetch(1, b_begin);
  }
  for (int64_t b = b_begin; b < b_end; ++b) {
    __syncthreads();                         // the previous sample's tile has been consumed
    commit(0, Xi);
    if (!diag) commit(1, Xj);
    __syncthreads();
    if (b + 1 < b_end) {
      fetch(0, b + 1);
      if (!diag) fetch(1, b + 1);
    }
    floatx16 acc[SW][SW];
#pragma unroll
    for (int i = 0; i < SW; ++i)
#pragma unroll
      for (int j = 0; j < SW; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    for (int k = 0; k < npad; k += 16) {
      uint4 a[SW], c[SW];
#pragma unroll
      for (int i = 0; i < SW; ++i) {
        a[i] = *(const uint4*)(pa + i * 32 * ldx + k);
        c[i] = *(const uint4*)(pb + i * 32 * ldx + k);
      }
#pragma unroll
      for (int i = 0; i < SW; ++i)
#pragma unroll
        for (int j = 0; j < SW; ++j) {
          if constexpr (DT == DMT_BF16)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                __builtin_bit_cast(bf16x8, a[i]), __builtin_bit_cast(bf16x8, c[j]), acc[i][j], 0, 0, 0);
          else
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
                __builtin_bit_cast(halfx8, a[i]), __builtin_bit_cast(halfx8, c[j]), acc[i][j], 0, 0, 0);
        }
    }
    // lane holds column lane % 32 of rows (v / 4) * 8 + (lane / 32) * 4 + v % 4 of a sub-tile
#pragma unroll
    for (int j = 0; j < SW; ++j) {
      const float ic = inv_col[32 * j];
#pragma unroll
      for (int i = 0; i < SW; ++i) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const float4 ir = *(const float4*)(inv_row + 32 * i + q * 8);
          total[i][j][4 * q + 0] += acc[i][j][4 * q + 0] * (ir.x * ic);
          total[i][j][4 * q + 1] += acc[i][j][4 * q + 1] * (ir.y * ic);
          total[i][j][4 * q + 2] += acc[i][j][4 * q + 2] * (ir.z * ic);
          total[i][j][4 * q + 3] += acc[i][j][4 * q + 3] * (ir.w * ic);
        }
      }
    }
  }

  float* out = partial + ((int64_t)slice * npairs + pair) * (TF * TF);
#pragma unroll
  for (int i = 0; i < SW; ++i)
#pragma unroll
    for (int j = 0; j < SW; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int r = 32 * (SW * wi + i) + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
        out[r * TF + 32 * (SW * wj + j) + (lane & 31)] = total[i][j][v];
      }
}

// The same contraction for 65 ... 256 features of dim N <= 128: one block of 16 waves stages ALL
// features of a sample (up to 256 rows, 68 KB of LDS at N = 128), so the pooled tensor is read
// exactly once, and its waves share out the 32 x 32 sub-tiles of the upper triangle of the
// Gram matrix (at most 36, three per wave).  A sub-tile (r, c), r <= c, is stored like a tile
// pair of 32-feature tiles, which is what tp_finish reads.  One block per CU; block = batch slice.
constexpr int kWideThreads = 1024, kWideRows = 256, kWideSub = 3;
template <int DT, int NP>
__global__ __launch_bounds__(kWideThreads) void tp_gram_wide(
    const DmtTableMeta* __restrict__ meta, const void* __restrict__ pooled, int64_t B, int F, int N,
    int gt, int nsub, int64_t per, float* __restrict__ partial) {
  constexpr int LPR = 4 * NP, RP = kWideThreads / LPR;     // NP passes cover the 256 rows
  constexpr bool kRaw = DT != DMT_F32;
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
  __shared__ int64_t s_base[kWideRows];
  __shared__ int32_t s_pitch[kWideRows];
  __shared__ __attribute__((aligned(16))) float s_inv[kWideRows];
  __shared__ uint8_t s_r[36], s_c[36];
  const int npad = (N + 15) & ~15, ldx = npad + 8;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid < kWideRows) {
    int64_t base = 0;
    int32_t pitch = 0;
    if (tid < F) {
      const DmtTableMeta m = meta[tid];
      base = m.out_prefix * B + m.col_off;
      pitch = m.tower_width;
    }
    s_base[tid] = base;
    s_pitch[tid] = pitch;
  }
  if (tid < nsub) {
    int r = 0;
    while (r + 1 < gt && tp_pair_index(r + 1, r + 1, gt) <= tid) ++r;
    s_r[tid] = (uint8_t)r;
    s_c[tid] = (uint8_t)(r + (tid - tp_pair_index(r, r, gt)));
  }
  __syncthreads();

  const int chunk = tid % LPR, row0 = tid / LPR;
  const bool cin = chunk * 8 < N;
  floatx16 total[kWideSub];
  int oa[kWideSub], ob[kWideSub], ir_off[kWideSub], ic_off[kWideSub];   // LDS element offsets
#pragma unroll
  for (int q = 0; q < kWideSub; ++q) {
    const int sub = wave + 16 * q;
    const int r = sub < nsub ? s_r[sub] : 0, c = sub < nsub ? s_c[sub] : 0;
    oa[q] = (32 * r + (lane & 31)) * ldx + (lane >> 5) * 8;
    ob[q] = (32 * c + (lane & 31)) * ldx + (lane >> 5) * 8;
    ir_off[q] = 32 * r + (lane >> 5) * 4;
    ic_off[q] = 32 * c + (lane & 31);
#pragma unroll
    for (int v = 0; v < 16; ++v) total[q][v] = 0.f;
  }

  Raw8<DT> raw[NP];
  auto fetch = [&](int64_t b) __attribute__((always_inline)) {
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      const int row = p * RP + row0;
      if (cin && row < F) {
        raw[p] = fetch8<DT, true>(pooled, s_base[row] + b * s_pitch[row] + chunk * 8);
      } else {
#pragma unroll
        for (int q = 0; q < (DT == DMT_F32 ? 2 : 1); ++q) raw[p].v[q] = make_uint4(0, 0, 0, 0);
      }
    }
  };
  auto commit = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      const int row = p * RP + row0;
      if constexpr (kRaw) {
        const uint4 r = raw[p].v[0];
        const float ss = row_group_sum<LPR>(sumsq8<DT>(r));
        if (chunk * 8 < npad) *(uint4*)(lds + row * ldx + chunk * 8) = r;
        if (chunk == 0) s_inv[row] = ss > 0.f ? __builtin_amdgcn_rsqf(ss) : 0.f;
      } else {
        float x[8];
        decode8<DT>(raw[p], x);
        float ss = 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q) ss += x[q] * x[q];
        ss = row_group_sum<LPR>(ss);
        const float inv = ss > 0.f ? __builtin_amdgcn_rsqf(ss) : 0.f;
        if (chunk * 8 < npad) {
          *(uint4*)(lds + row * ldx + chunk * 8) =
              make_uint4(dmt::pack2<DMT_F16>(x[0] * inv, x[1] * inv),
                         dmt::pack2<DMT_F16>(x[2] * inv, x[3] * inv),
                         dmt::pack2<DMT_F16>(x[4] * inv, x[5] * inv),
                         dmt::pack2<DMT_F16>(x[6] * inv, x[7] * inv));
        }
        if (chunk == 0) s_inv[row] = 1.0f;
      }
    }
  };

  const int64_t b_begin = blockIdx.x * per, b_end = b_begin + per < B ? b_begin + per : B;
  if (b_begin < b_end) fetch(b_begin);
  for (int64_t b = b_begin; b < b_end; ++b) {
    __syncthreads();                         // the previous sample's rows have been consumed
    commit();
    __syncthreads();
    if (b + 1 < b_end) fetch(b + 1);
#pragma unroll
    for (int q = 0; q < kWideSub; ++q) {
      if (wave + 16 * q < nsub) {            // uniform over the wave
        floatx16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.f;
        for (int k = 0; k < npad; k += 16) {
          const uint4 a = *(const uint4*)(lds + oa[q] + k);
          const uint4 c = *(const uint4*)(lds + ob[q] + k);
          if constexpr (DT == DMT_BF16)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                          __builtin_bit_cast(bf16x8, c), acc, 0, 0, 0);
          else
            acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(halfx8, a),
                                                         __builtin_bit_cast(halfx8, c), acc, 0, 0, 0);
        }
        const float ic = s_inv[ic_off[q]];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float4 ir = *(const float4*)(s_inv + ir_off[q] + j * 8);
          total[q][4 * j + 0] += acc[4 * j + 0] * (ir.x * ic);
          total[q][4 * j + 1] += acc[4 * j + 1] * (ir.y * ic);
          total[q][4 * j + 2] += acc[4 * j + 2] * (ir.z * ic);
          total[q][4 * j + 3] += acc[4 * j + 3] * (ir.w * ic);
        }
      }
    }
  }

#pragma unroll
  for (int q = 0; q < kWideSub; ++q) {
    const int sub = wave + 16 * q;
    if (sub < nsub) {
      float* out = partial + ((int64_t)blockIdx.x * nsub + sub) * (32 * 32);
#pragma unroll
      for (int v = 0; v < 16; ++v)
        out[((v >> 2) * 8 + (lane >> 5) * 4 + (v & 3)) * 32 + (lane & 31)] = total[q][v];
    }
  }
}

// I[i][j] = | sum over the batch slices of the Gram entry | / B.  Entry (i, j) and (j, i) are
// both read from the tile element (min, max), so the result is exactly symmetric.  A block
// takes 16 consecutive entries; its 16 thread groups each add up every 16th slice, then the
// group sums are added in group order: a fixed order whatever the launch.
constexpr int kFinElems = 16, kFinGroups = kBlock / kFinElems;
__global__ __launch_bounds__(kBlock) void tp_finish(const float* __restrict__ partial, int F,
                                                    int tile, int nt, int npairs,
                                                    int64_t nslices, float inv_b,
                                                    float* __restrict__ I) {
  __shared__ float s_sum[kFinGroups][kFinElems];
  const int le = threadIdx.x % kFinElems, g = threadIdx.x / kFinElems;
  const int64_t e = (int64_t)blockIdx.x * kFinElems + le;
  float s = 0.f;
  if (e < (int64_t)F * F) {
    const int i = (int)(e / F), j = (int)(e % F);
    const int a = i < j ? i : j, c = i < j ? j : i;
    const float* p = partial + (int64_t)tp_pair_index(a / tile, c / tile, nt) * (tile * tile) +
                     (a % tile) * tile + (c % tile);
    const int64_t stride = (int64_t)npairs * (tile * tile);
#pragma unroll 8
    for (int64_t q = g; q < nslices; q += kFinGroups) s += p[q * stride];
  }
  s_sum[g][le] = s;
  __syncthreads();
  if (g == 0 && e < (int64_t)F * F) {
    float t = 0.f;
#pragma unroll
    for (int q = 0; q < kFinGroups; ++q) t += s_sum[q][le];
    I[e] = fabsf(t * inv_b);
  }
}

struct TpShape {
  int N, np, tile, nt, npairs;             // np: staging passes per 64 rows (4 np lanes per row)
  bool wide;                               // tp_gram_wide: all features in one block
  int64_t per, nslices;
  size_t bytes;
};

// Every table must have the same embedding dim (the cosine kernel pairs any two features), a
// multiple of 8 up to 512, so that rows split into aligned 8-element chunks.  `rows16`: the
// pooled tensor holds 16-bit elements (float32 rows take the tile-pair kernel: staged, they
// need more registers than a 16-wave block has).
dmt_status tp_shape(const dmt_plan* p, int64_t B, bool rows16, TpShape& s) {
  if (p->classes.size() != 1) return DMT_ENOTSUP;
  s.N = p->classes[0].D;
  if (s.N % 8 != 0 || s.N > 512) return DMT_ENOTSUP;
  for (const DmtTableMeta& m : p->meta)
    if (m.col_off % 8 != 0 || m.tower_width % 8 != 0) return DMT_ENOTSUP;
  s.np = s.N <= 32 ? 1 : s.N <= 64 ? 2 : s.N <= 128 ? 4 : s.N <= 256 ? 8 : 16;
  if (rows16 && p->F > kTile && p->F <= kWideRows && s.np <= 4) {
    // one block per CU stages all features of a sample; "tiles" are its 32 x 32 sub-tiles
    s.wide = true;
    s.tile = 32;
    s.nt = (p->F + 31) / 32;
    s.npairs = s.nt * (s.nt + 1) / 2;
    s.per = (B + kWideBlocks - 1) / kWideBlocks;
    s.nslices = (B + s.per - 1) / s.per;
  } else {
    // tile pairs of 64 features.  (tp_gram also runs with TF = 128, which re-reads the pooled
    // rows less, but measured slower on MI355X: its larger register and LDS footprint halves
    // the resident blocks, and the loads in flight with them.)
    s.wide = false;
    s.tile = kTile;
    s.nt = (p->F + s.tile - 1) / s.tile;
    s.npairs = s.nt * (s.nt + 1) / 2;
    // one round of resident blocks for a single pair; two when diagonal pairs (one tile to
    // stage) and off-diagonal pairs (two) share the launch, so that the uneven blocks even out
    const int64_t want = std::max<int64_t>(1, (s.npairs > 1 ? 2 : 1) * kTargetBlocks / s.npairs);
    s.per = (B + want - 1) / want;
    s.nslices = (B + s.per - 1) / s.per;
  }
  s.bytes = sizeof(float) * (size_t)s.nslices * s.npairs * s.tile * s.tile;
  return DMT_OK;
}

template <int DT, int NP, int TF>
void launch_gram(const dmt_plan* p, const void* pooled, int64_t B, const TpShape& sh,
                 float* partial, hipStream_t s) {
  const int npad = (sh.N + 15) & ~15;
  const size_t lds = sizeof(uint16_t) * 2 * TF * (npad + 8);
  static bool configured = false;           // wide rows need more than the default LDS limit
  if (!configured) {
    (void)hipFuncSetAttribute((const void*)tp_gram<DT, NP, TF>,
                              hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)(sizeof(uint16_t) * 2 * TF * (NP * 32 + 8)));
    configured = true;
  }
  const int64_t blocks = (sh.nslices + 7) / 8 * 8 * sh.npairs;
  hipLaunchKernelGGL((tp_gram<DT, NP, TF>), dim3((unsigned)blocks), dim3(kBlock), lds, s, p->d_meta,
                     pooled, B, p->F, sh.N, sh.nt, sh.npairs, sh.per, sh.nslices, partial);
}

template <int DT, int NP>
void launch_gram_wide(const dmt_plan* p, const void* pooled, int64_t B, const TpShape& sh,
                      float* partial, hipStream_t s) {
  const int npad = (sh.N + 15) & ~15;
  const size_t lds = sizeof(uint16_t) * kWideRows * (npad + 8);
  static bool configured = false;
  if (!configured) {
    (void)hipFuncSetAttribute((const void*)tp_gram_wide<DT, NP>,
                              hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)(sizeof(uint16_t) * kWideRows * (NP * 32 + 8)));
    configured = true;
  }
  hipLaunchKernelGGL((tp_gram_wide<DT, NP>), dim3((unsigned)sh.nslices), dim3(kWideThreads), lds, s,
                     p->d_meta, pooled, B, p->F, sh.N, sh.nt, sh.npairs, sh.per, partial);
}

template <int DT>
void launch_gram_dt(const dmt_plan* p, const void* pooled, int64_t B, const TpShape& sh,
                    float* partial, hipStream_t s) {
  if constexpr (DT != DMT_F32) {
    if (sh.wide) {
      if (sh.np == 1) launch_gram_wide<DT, 1>(p, pooled, B, sh, partial, s);
      else if (sh.np == 2) launch_gram_wide<DT, 2>(p, pooled, B, sh, partial, s);
      else launch_gram_wide<DT, 4>(p, pooled, B, sh, partial, s);
      return;
    }
  }
  if (sh.np == 1) launch_gram<DT, 1, kTile>(p, pooled, B, sh, partial, s);
  else if (sh.np == 2) launch_gram<DT, 2, kTile>(p, pooled, B, sh, partial, s);
  else if (sh.np == 4) launch_gram<DT, 4, kTile>(p, pooled, B, sh, partial, s);
  else if (sh.np == 8) launch_gram<DT, 8, kTile>(p, pooled, B, sh, partial, s);
  else launch_gram<DT, 16, kTile>(p, pooled, B, sh, partial, s);
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
  TpShape a, b;                             // enough for a pooled tensor of any dtype
  if (!plan || B <= 0 || tp_shape(plan, B, true, a) != DMT_OK || tp_shape(plan, B, false, b) != DMT_OK)
    return 0;
  return std::max(a.bytes, b.bytes);
}

extern "C" dmt_status dmt_tp_interaction(const dmt_plan* plan, const void* pooled, int64_t B,
                                         int32_t pooled_dtype, float* interaction,
                                         void* workspace, size_t workspace_bytes, void* stream) {
  if (!plan || !pooled || !interaction || !workspace) return DMT_EINVAL;
  if (B <= 0 || B > plan->max_batch || !plan->bound) return DMT_EINVAL;
  if (pooled_dtype != DMT_F32 && pooled_dtype != DMT_F16 && pooled_dtype != DMT_BF16)
    return DMT_EINVAL;
  if (((uintptr_t)pooled & 15) || ((uintptr_t)workspace & 15) || ((uintptr_t)interaction & 3))
    return DMT_EINVAL;
  TpShape sh;
  const dmt_status st = tp_shape(plan, B, pooled_dtype != DMT_F32, sh);
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
    hipLaunchKernelGGL(tp_finish, dim3((unsigned)((n + kFinElems - 1) / kFinElems)), dim3(kBlock), 0, s,
                       partial, plan->F, sh.tile, sh.nt, sh.npairs, sh.nslices, (float)(1.0 / (double)B),
                       interaction);
  }
  return hipGetLastError() == hipSuccess ? DMT_OK : DMT_EHIP;
}

static dmt_status tp_embed(const float* interaction, int32_t F, int32_t strategy,
                           int32_t n, int32_t steps, double lr, const double* x0, double* x,
                           double* stress) {
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

// No exception crosses the C boundary: a failed host allocation is reported as DMT_ENOMEM.
extern "C" dmt_status dmt_tp_embed(const float* interaction, int32_t F, int32_t strategy,
                                   int32_t n, int32_t steps, double lr, const double* x0,
                                   double* x, double* stress) {
  try {
    return tp_embed(interaction, F, strategy, n, steps, lr, x0, x, stress);
  } catch (const std::bad_alloc&) {
    return DMT_ENOMEM;
  }
}

static dmt_status tp_kmeans(const double* x, int32_t F, int32_t n, int32_t T, double ratio,
                            const double* centres0, int32_t max_iter, int32_t* table_to_tower,
                            double* centres, int32_t* iterations) {
  if (!x || !centres0 || !table_to_tower || F <= 0 || n <= 0 || T <= 0 || T > F) return DMT_EINVAL;
  if (!(ratio >= 1.0) || max_iter <= 0) return DMT_EINVAL;
  int smin, smax;
  size_bounds(F, T, ratio, smin, smax);
  const int ns = T * smax;                  // slots = rows of the square problem
  if (ns > 4096) return DMT_ENOTSUP;         // the O(ns^3) assignment is meant for |F| in the hundreds
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

extern "C" dmt_status dmt_tp_kmeans(const double* x, int32_t F, int32_t n, int32_t T,
                                    double ratio, const double* centres0, int32_t max_iter,
                                    int32_t* table_to_tower, double* centres,
                                    int32_t* iterations) {
  try {
    return tp_kmeans(x, F, n, T, ratio, centres0, max_iter, table_to_tower, centres, iterations);
  } catch (const std::bad_alloc&) {
    return DMT_ENOMEM;
  }
}
