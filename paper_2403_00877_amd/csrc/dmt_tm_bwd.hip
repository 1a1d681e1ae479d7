// dmt_tower_module_bwd: the chain rule through the Tower Module forms (paper
// Sec. 3.2, Sec. 4, Listings 1 and 2), from dL/d(tm_out) to dL/d(pooled) and the
// parameter gradients.
//
// Every contraction of the backward is brought into the forward's shape
// C[M][N] = A[M][K] . W[N][K]^T (both operands K-contiguous), so the grouped MFMA
// kernels of the forward serve it unchanged with a float32-output epilogue:
//   data gradient    dX[B][Kin]  = dz[B][O]   . (W^T)[Kin][O]^T
//   weight gradient  dW[O][Kin]  = (dz^T)[O][B] . (x^T)[Kin][B]^T
// The operands that exist only in the other orientation (W^T, dz^T, x^T) are
// written by an LDS-tiled transpose into 16-byte-aligned, zero-padded rows.
// Towers are grouped into one launch per stage like the forward's.  The
// forward's intermediates are recomputed (dot terms; u_l = W_l x_l + b_l and x_l of
// the cross layers unless the caller hands over what a training forward kept).
// A weight gradient has few output tiles and a long K (the batch): K is cut into
// slices that are contractions of their own and summed in slice order.
// Bias gradients are fixed-order row sums of the transposed gradient operand.
// The DLRM module's shared per-feature layer is the same machinery on rows
// (sample, feature) of the pooled block.
#define DMT_TM_TAG 1          // this file's instances of the shared GEMM kernels
#include "dmt_tm_gemm.h"

namespace {

constexpr int kTile = 32;        // scalar transposes (float32 path, gradient preparation)
constexpr int kVTile = 64;       // 16-bit transpose: 64 x 64 tiles, 8-byte accesses
constexpr int kMaxItems = 32;

template <int DT> struct EltOf { using type = uint16_t; };
template <> struct EltOf<DMT_F32> { using type = float; };

// One tower's share of a grouped launch of the small kernels below: block id ->
// (item, block within the item), like the grouped GEMM.  The meaning of the fields is
// each kernel's own.
struct TmbItem {
  const void* a;
  const void* b;
  const void* c;
  void* o0;
  void* o1;
  void* o2;
  int64_t n0, n1, n2;
  int32_t i0, i1, i2, i3, i4;
  int32_t nbx;               // blocks along the first dimension (2-D kernels) or blocks of the item
};

struct TmbLaunch {
  int32_t n;
  int32_t block_start[kMaxItems + 1];
  TmbItem it[kMaxItems];
};

__device__ __forceinline__ int tmb_find(const TmbLaunch& L) {
  int i = 0;
  while (i + 1 < L.n && (int)blockIdx.x >= L.block_start[i + 1]) ++i;
  return i;
}

// ---------------------------------------------------------------- small kernels

// dz[b][o] = dy[b][o] (zero where ReLU was off: y[b][o] <= 0), rounded to DT, with
// zero columns O .. Op-1; dzT[o][b] the same values transposed, zero for b in [B, Bp).
// Row b of dy (and y) starts at element b * ldy, or, with rdiv > 0, at
// (b / rdiv) * ldy + (b % rdiv) * ld2: rdiv rows of the gradient operand lie side by side in
// one row of the output gradient (a per-feature layer).
// a = dy, b = y, o0 = dz, o1 = dzT, n0 = B, n1 = Bp, n2 = ldy, i0 = O, i1 = Op, i2 = relu,
// i3 = rdiv, i4 = ld2.
template <int DT>
__global__ __launch_bounds__(kBlock) void tmb_prep_dy(const TmbLaunch L) {
  __shared__ float tile[kTile][kTile + 1];
  const int gi = tmb_find(L);
  const TmbItem& G = L.it[gi];
  const int lb = blockIdx.x - L.block_start[gi];
  const float* __restrict__ dy = (const float*)G.a;
  const int64_t B = G.n0, Bp = G.n1;
  const int O = G.i0, Op = G.i1, relu = G.i2;
  const int64_t b0 = (int64_t)(lb % G.nbx) * kTile;
  const int o0 = (lb / G.nbx) * kTile;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  for (int r = ty; r < kTile; r += kBlock / kTile) {
    const int64_t b = b0 + r;
    const int o = o0 + tx;
    float v = 0.f;
    if (b < B && o < O) {
      const int64_t at = (G.i3 > 0 ? (b / G.i3) * G.n2 + (b % G.i3) * G.i4 : b * G.n2) + o;
      v = dy[at];
      if (relu && !(load_elt<DT>(G.b, at) > 0.f)) v = 0.f;
    }
    if (b < B && o < Op) store_elt<DT>(G.o0, b * Op + o, v);
    tile[r][tx] = v;
  }
  __syncthreads();
  for (int r = ty; r < kTile; r += kBlock / kTile) {
    const int o = o0 + r;
    const int64_t b = b0 + tx;
    if (o < O && b < Bp) store_elt<DT>(G.o1, (int64_t)o * Bp + b, tile[tx][r]);
  }
}

// The same for the 16-bit types when O, ldy (and ld2) are multiples of 4 and dy is 16-byte
// aligned: 64 x 64 tiles, 16-byte reads of the gradient, 8-byte writes of both outputs.
template <int DT>
__global__ __launch_bounds__(kBlock) void tmb_prep_dy16(const TmbLaunch L) {
  __shared__ __attribute__((aligned(8))) uint16_t tile[kVTile][kVTile + 4];
  const int gi = tmb_find(L);
  const TmbItem& G = L.it[gi];
  const int lb = blockIdx.x - L.block_start[gi];
  const float* __restrict__ dy = (const float*)G.a;
  const uint16_t* __restrict__ y = (const uint16_t*)G.b;
  uint16_t* __restrict__ dz = (uint16_t*)G.o0;
  uint16_t* __restrict__ dzT = (uint16_t*)G.o1;
  const int64_t B = G.n0, Bp = G.n1;
  const int O = G.i0, Op = G.i1, relu = G.i2;
  const int64_t b0 = (int64_t)(lb % G.nbx) * kVTile;
  const int o0 = (lb / G.nbx) * kVTile;
  const int q = threadIdx.x >> 4, v = (threadIdx.x & 15) * 4;
#pragma unroll
  for (int pass = 0; pass < 4; ++pass) {
    const int i = pass * 16 + q;
    const int64_t b = b0 + i;
    const int o = o0 + v;
    float g[4] = {0.f, 0.f, 0.f, 0.f};
    if (b < B && o < O) {
      const int64_t at = (G.i3 > 0 ? (b / G.i3) * G.n2 + (b % G.i3) * G.i4 : b * G.n2) + o;
      const float4 t = *(const float4*)(dy + at);
      g[0] = t.x; g[1] = t.y; g[2] = t.z; g[3] = t.w;
      if (relu) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (!(load_elt<DT>(y, at + e) > 0.f)) g[e] = 0.f;
      }
    }
    const uint2 packed = make_uint2(dmt::pack2<DT>(g[0], g[1]), dmt::pack2<DT>(g[2], g[3]));
    if (b < B && o < Op) *(uint2*)(dz + b * Op + o) = packed;
    *(uint2*)&tile[i][v] = packed;
  }
  __syncthreads();
#pragma unroll
  for (int pass = 0; pass < 4; ++pass) {
    const int i = pass * 16 + q;                   // output column of the tile
    const int o = o0 + i;
    const int64_t b = b0 + v;
    if (o < O && b < Bp) {
      const uint32_t lo = tile[v][i] | ((uint32_t)tile[v + 1][i] << 16);
      const uint32_t hi = tile[v + 2][i] | ((uint32_t)tile[v + 3][i] << 16);
      *(uint2*)(dzT + (int64_t)o * Bp + b) = make_uint2(lo, hi);
    }
  }
}

// dst[c][r] = src[r][c] for r < R, 0 for R <= r < fill; c < C.  src rows are lds
// elements apart, dst rows ldd; fill = i1, or ldd when that is 0 (a narrower fill writes
// one column block of a wider matrix).
// a = src, o0 = dst, n0 = R, n1 = lds, n2 = ldd, i0 = C, i1 = fill.
// Any element type and alignment: one element per access.
template <typename E>
__global__ __launch_bounds__(kBlock) void tmb_transpose(const TmbLaunch L) {
  __shared__ E tile[kTile][kTile + 1];
  const int gi = tmb_find(L);
  const TmbItem& G = L.it[gi];
  const int lb = blockIdx.x - L.block_start[gi];
  const E* __restrict__ src = (const E*)G.a;
  E* __restrict__ dst = (E*)G.o0;
  const int64_t R = G.n0, lds = G.n1, ldd = G.n2, fill = G.i1 > 0 ? G.i1 : G.n2;
  const int C = G.i0;
  const int64_t r0 = (int64_t)(lb % G.nbx) * kTile;
  const int c0 = (lb / G.nbx) * kTile;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  for (int i = ty; i < kTile; i += kBlock / kTile) {
    const int64_t r = r0 + i;
    const int c = c0 + tx;
    tile[i][tx] = (r < R && c < C) ? src[r * lds + c] : (E)0;
  }
  __syncthreads();
  for (int i = ty; i < kTile; i += kBlock / kTile) {
    const int c = c0 + i;
    const int64_t r = r0 + tx;
    if (c < C && r < fill) dst[(int64_t)c * ldd + r] = tile[tx][i];
  }
}

// The same for 16-bit elements with C, lds and ldd multiples of 4 and 8-byte aligned
// bases: 64 x 64 tiles, four (or, alignment permitting, eight) elements per global access.
__global__ __launch_bounds__(kBlock) void tmb_transpose16(const TmbLaunch L) {
  __shared__ __attribute__((aligned(16))) uint16_t tile[kVTile][kVTile + 8];
  const int gi = tmb_find(L);
  const TmbItem& G = L.it[gi];
  const int lb = blockIdx.x - L.block_start[gi];
  const uint16_t* __restrict__ src = (const uint16_t*)G.a;
  uint16_t* __restrict__ dst = (uint16_t*)G.o0;
  const int64_t R = G.n0, lds = G.n1, ldd = G.n2, fill = G.i1 > 0 ? G.i1 : G.n2;
  const int C = G.i0;
  const int64_t r0 = (int64_t)(lb % G.nbx) * kVTile;
  const int c0 = (lb / G.nbx) * kVTile;
  // 16-byte global accesses where every row of both matrices splits into aligned 8-element
  // chunks (the same for the whole item, so the branch is uniform)
  const bool wide = C % 8 == 0 && lds % 8 == 0 && ldd % 8 == 0 && fill % 8 == 0 &&
                    (((uintptr_t)src | (uintptr_t)dst) & 15) == 0;
  if (wide) {
    const int q = threadIdx.x >> 3, v = (threadIdx.x & 7) * 8;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
      const int i = pass * 32 + q;
      const int64_t r = r0 + i;
      const int c = c0 + v;
      uint4 x = make_uint4(0, 0, 0, 0);
      if (r < R && c < C) x = *(const uint4*)(src + r * lds + c);
      // chunk j of row i sits in slot j ^ (i / 8) % 8: the eight rows 8 apart that one read
      // instruction below touches then fall on eight different 16-byte bank groups
      *(uint4*)&tile[i][v ^ (i & 56)] = x;
    }
    __syncthreads();
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
      const int i = pass * 32 + q;                 // column of the source tile
      const int c = c0 + i;
      const int64_t r = r0 + v;
      if (c < C && r < fill) {
        uint32_t w[4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
          w[k] = tile[v + 2 * k][i ^ v] | ((uint32_t)tile[v + 2 * k + 1][i ^ v] << 16);
        *(uint4*)(dst + (int64_t)c * ldd + r) = make_uint4(w[0], w[1], w[2], w[3]);
      }
    }
    return;
  }
  const int q = threadIdx.x >> 4, v = (threadIdx.x & 15) * 4;
#pragma unroll
  for (int pass = 0; pass < 4; ++pass) {
    const int i = pass * 16 + q;
    const int64_t r = r0 + i;
    const int c = c0 + v;
    uint2 x = make_uint2(0, 0);
    if (r < R && c < C) x = *(const uint2*)(src + r * lds + c);
    *(uint2*)&tile[i][v] = x;
  }
  __syncthreads();
#pragma unroll
  for (int pass = 0; pass < 4; ++pass) {
    const int i = pass * 16 + q;                   // column of the source tile
    const int c = c0 + i;
    const int64_t r = r0 + v;
    if (c < C && r < fill) {
      const uint32_t lo = tile[v][i] | ((uint32_t)tile[v + 1][i] << 16);
      const uint32_t hi = tile[v + 2][i] | ((uint32_t)tile[v + 3][i] << 16);
      *(uint2*)(dst + (int64_t)c * ldd + r) = make_uint2(lo, hi);
    }
  }
}

// out[r] = sum over c < ncols of src[r][c], float32, in a fixed order: thread t of
// the row's block adds columns t, t + 256, ... (16-bit types: the 8-column chunks t,
// t + 256, ..., over the whole padded row, whose padding is zero) and the 256 partial
// sums are folded by halves.  One block per row.  a = src, o0 = out, n0 = ld (a multiple
// of 8 for the 16-bit types), n1 = ncols.
template <int DT>
__global__ __launch_bounds__(kBlock) void tmb_rowsum(const TmbLaunch L) {
  __shared__ float part[kBlock];
  const int gi = tmb_find(L);
  const TmbItem& G = L.it[gi];
  const int64_t row = blockIdx.x - L.block_start[gi];
  const int64_t ld = G.n0, ncols = G.n1;
  float s = 0.f;
  if constexpr (DT == DMT_F32) {
    for (int64_t c = threadIdx.x; c < ncols; c += kBlock) s += load_elt<DT>(G.a, row * ld + c);
  } else {
    for (int64_t c = (int64_t)threadIdx.x * 8; c < ld; c += kBlock * 8) {
      float x[8];
      dmt::decode_chunk<DT>(x, *(const uint4*)((const uint16_t*)G.a + row * ld + c));
#pragma unroll
      for (int q = 0; q < 8; ++q) s += x[q];
    }
  }
  part[threadIdx.x] = s;
  __syncthreads();
  for (int h = kBlock / 2; h > 0; h >>= 1) {
    if ((int)threadIdx.x < h) part[threadIdx.x] += part[threadIdx.x + h];
    __syncthreads();
  }
  if (threadIdx.x == 0) ((float*)G.o0)[row] = part[0];
}

// Elementwise kernels over `count` = n0 elements: 8 per thread step for the 16-bit types
// (count is then a multiple of 8), 1 for float32.  nbx = blocks of the item.
template <int DT> struct Ew { static constexpr int V = DT == DMT_F32 ? 1 : 8; };

template <int DT>
__device__ __forceinline__ void ew_load(const void* p, int64_t e, float (&x)[Ew<DT>::V]) {
  if constexpr (DT == DMT_F32) x[0] = ((const float*)p)[e];
  else dmt::decode_chunk<DT>(x, *(const uint4*)((const uint16_t*)p + e));
}
template <int DT>
__device__ __forceinline__ void ew_store(void* p, int64_t e, const float (&x)[Ew<DT>::V]) {
  if constexpr (DT == DMT_F32) ((float*)p)[e] = x[0];
  else dmt::store_chunk<DT, 8>(p, e, x);
}
template <int V>
__device__ __forceinline__ void ew_load_f32(const float* p, int64_t e, float (&x)[V]) {
  if constexpr (V == 1) x[0] = p[e];
  else {
    const float4 a = *(const float4*)(p + e), b = *(const float4*)(p + e + 4);
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
  }
}
template <int V>
__device__ __forceinline__ void ew_store_f32(float* p, int64_t e, const float (&x)[V]) {
  if constexpr (V == 1) p[e] = x[0];
  else {
    *(float4*)(p + e) = make_float4(x[0], x[1], x[2], x[3]);
    *(float4*)(p + e + 4) = make_float4(x[4], x[5], x[6], x[7]);
  }
}

// Dot-product tower: dx[b][i][c] = dZ[b][np_pad + i n + c]
//                                  + sum over j != i (ascending j) of dZ[b][p(i,j)] x[b][j][c]
// with p the row-major index of the pair {i, j}.  One thread per element of dx.
// a = x, b = dZ, o0 = dx, n0 = B, i0 = nf, i1 = n, i2 = np_pad, i3 = ldz.
template <int DT>
__global__ __launch_bounds__(kBlock) void tmb_dot_bwd(const TmbLaunch L) {
  const int gi = tmb_find(L);
  const TmbItem& G = L.it[gi];
  const int nf = G.i0, n = G.i1, np_pad = G.i2, ldz = G.i3;
  const int wt = nf * n;
  const int64_t e = (int64_t)(blockIdx.x - L.block_start[gi]) * kBlock + threadIdx.x;
  if (e >= G.n0 * wt) return;
  const int64_t b = e / wt;
  const int r = (int)(e % wt), i = r / n, c = r % n;
  const float* __restrict__ z = (const float*)G.b + b * ldz;
  float acc = z[np_pad + r];
  for (int j = 0; j < nf; ++j) {
    if (j == i) continue;
    const int lo = j < i ? j : i, hi = j < i ? i : j;
    acc += z[lo * (2 * nf - lo - 1) / 2 + (hi - lo - 1)] * load_elt<DT>(G.a, b * wt + j * n + c);
  }
  ((float*)G.o0)[e] = acc;
}

// The same for the 16-bit types with n a multiple of 8: one thread per 8 consecutive columns
// of one feature, 16-byte accesses.
template <int DT>
__global__ __launch_bounds__(kBlock) void tmb_dot_bwd8(const TmbLaunch L) {
  const int gi = tmb_find(L);
  const TmbItem& G = L.it[gi];
  const int nf = G.i0, n = G.i1, np_pad = G.i2, ldz = G.i3;
  const int wt = nf * n, w8 = wt / 8;
  const int64_t e = (int64_t)(blockIdx.x - L.block_start[gi]) * kBlock + threadIdx.x;
  if (e >= G.n0 * w8) return;
  const int64_t b = e / w8;
  const int r = (int)(e % w8) * 8, i = r / n, c = r % n;
  const float* __restrict__ z = (const float*)G.b + b * ldz;
  const uint16_t* __restrict__ x = (const uint16_t*)G.a + b * wt + c;
  float acc[8];
  ew_load_f32<8>(z, np_pad + r, acc);
  for (int j = 0; j < nf; ++j) {
    if (j == i) continue;
    const int lo = j < i ? j : i, hi = j < i ? i : j;
    const float g = z[lo * (2 * nf - lo - 1) / 2 + (hi - lo - 1)];
    float xv[8];
    dmt::decode_chunk<DT>(xv, *(const uint4*)(x + j * n));
#pragma unroll
    for (int q = 0; q < 8; ++q) acc[q] += g * xv[q];
  }
  ew_store_f32<8>((float*)G.o0, b * wt + r, acc);
}

// dw[o][k] = sum over slices s (ascending) of part[s][o][k'], where k' = k for k < np and
// k - np + np_pad after: adds up a split contraction's slices and drops the padding columns
// between the dot terms and the flat part (np = np_pad = 0: plain rows).
// a = part, o0 = dw, n0 = slice stride in floats, i0 = O, i1 = np, i2 = np_pad, i3 = wt,
// i4 = slices.
__global__ __launch_bounds__(kBlock) void tmb_sum_slices(const TmbLaunch L) {
  const int gi = tmb_find(L);
  const TmbItem& G = L.it[gi];
  const int O = G.i0, np = G.i1, np_pad = G.i2, wt = G.i3, ns = G.i4;
  const int64_t e = (int64_t)(blockIdx.x - L.block_start[gi]) * kBlock + threadIdx.x;
  const int kin = np + wt;
  if (e >= (int64_t)O * kin) return;
  const int o = (int)(e / kin), k = (int)(e % kin);
  const float* __restrict__ p = (const float*)G.a + (int64_t)o * (np_pad + wt) + (k < np ? k : k - np + np_pad);
  float s = 0.f;
  for (int q = 0; q < ns; ++q) s += p[q * G.n0];
  ((float*)G.o0)[e] = s;
}

// Cross layer backward, elementwise part: du = dxn * x0 (rounded to DT);
// dx0 = (first ? 0 : dx0) + dxn * u (+ dxn when `last`: the layer's data-gradient contraction
// then accumulates du W_l on top, which completes dx_0 + dx0 in place).
// a = dxn, b = x0, c = u, o0 = du, o1 = dx0, i0 = first, i1 = last.
template <int DT>
__global__ __launch_bounds__(kBlock) void tmb_cross_prep(const TmbLaunch L) {
  constexpr int V = Ew<DT>::V;
  const int gi = tmb_find(L);
  const TmbItem& G = L.it[gi];
  const int first = G.i0;
  const float keep = G.i1 ? 1.f : 0.f;
  const int64_t stride = (int64_t)G.nbx * kBlock * V;
  for (int64_t e = ((int64_t)(blockIdx.x - L.block_start[gi]) * kBlock + threadIdx.x) * V; e < G.n0;
       e += stride) {
    float g[V], x0[V], u[V], acc[V];
    ew_load_f32<V>((const float*)G.a, e, g);
    ew_load<DT>(G.b, e, x0);
    ew_load<DT>(G.c, e, u);
    if (first) {
#pragma unroll
      for (int q = 0; q < V; ++q) acc[q] = 0.f;
    } else {
      ew_load_f32<V>((const float*)G.o1, e, acc);
    }
#pragma unroll
    for (int q = 0; q < V; ++q) {
      acc[q] += g[q] * u[q] + keep * g[q];
      x0[q] *= g[q];
    }
    ew_store<DT>(G.o0, e, x0);
    ew_store_f32<V>((float*)G.o1, e, acc);
  }
}

// The same for the 16-bit types, writing du^T as well (the weight gradient's operand), so that du
// is not read back by a transpose: 64 x 64 tiles of the [B][W] tensors, 16-byte reads of dxn and
// dx0, 8-byte accesses of the 16-bit tensors.  W is a multiple of 8.
// a = dxn, b = x0, c = u, o0 = du, o1 = dx0, o2 = du^T [W][Bp], n0 = B, n1 = Bp, i0 = first,
// i1 = last, i2 = W; nbx = tiles along the batch.
template <int DT>
__global__ __launch_bounds__(kBlock) void tmb_cross_prep_t(const TmbLaunch L) {
  __shared__ __attribute__((aligned(8))) uint16_t tile[kVTile][kVTile + 4];
  const int gi = tmb_find(L);
  const TmbItem& G = L.it[gi];
  const int lb = blockIdx.x - L.block_start[gi];
  const float* __restrict__ dxn = (const float*)G.a;
  const uint16_t* __restrict__ x0 = (const uint16_t*)G.b;
  const uint16_t* __restrict__ u = (const uint16_t*)G.c;
  uint16_t* __restrict__ du = (uint16_t*)G.o0;
  float* __restrict__ dx0 = (float*)G.o1;
  uint16_t* __restrict__ duT = (uint16_t*)G.o2;
  const int64_t B = G.n0, Bp = G.n1;
  const int W = G.i2, first = G.i0;
  const float keep = G.i1 ? 1.f : 0.f;
  const int64_t b0 = (int64_t)(lb % G.nbx) * kVTile;
  const int c0 = (lb / G.nbx) * kVTile;
  const int q = threadIdx.x >> 4, v = (threadIdx.x & 15) * 4;
#pragma unroll
  for (int pass = 0; pass < 4; ++pass) {
    const int i = pass * 16 + q;
    const int64_t b = b0 + i;
    const int c = c0 + v;
    uint2 packed = make_uint2(0, 0);
    if (b < B && c < W) {
      const int64_t at = b * W + c;
      const float4 g = *(const float4*)(dxn + at);
      const uint2 xr = *(const uint2*)(x0 + at), ur = *(const uint2*)(u + at);
      float xa, xb, xc, xd, ua, ub, uc, ud;
      dmt::unpack2<DT>(xr.x, xa, xb); dmt::unpack2<DT>(xr.y, xc, xd);
      dmt::unpack2<DT>(ur.x, ua, ub); dmt::unpack2<DT>(ur.y, uc, ud);
      float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
      if (!first) acc = *(const float4*)(dx0 + at);
      acc.x += g.x * ua + keep * g.x; acc.y += g.y * ub + keep * g.y;
      acc.z += g.z * uc + keep * g.z; acc.w += g.w * ud + keep * g.w;
      *(float4*)(dx0 + at) = acc;
      packed = make_uint2(dmt::pack2<DT>(g.x * xa, g.y * xb), dmt::pack2<DT>(g.z * xc, g.w * xd));
      *(uint2*)(du + at) = packed;
    }
    *(uint2*)&tile[i][v] = packed;
  }
  __syncthreads();
#pragma unroll
  for (int pass = 0; pass < 4; ++pass) {
    const int i = pass * 16 + q;                   // column of the tile
    const int c = c0 + i;
    const int64_t b = b0 + v;
    if (c < W && b < Bp) {
      const uint32_t lo = tile[v][i] | ((uint32_t)tile[v + 1][i] << 16);
      const uint32_t hi = tile[v + 2][i] | ((uint32_t)tile[v + 3][i] << 16);
      *(uint2*)(duT + (int64_t)c * Bp + b) = make_uint2(lo, hi);
    }
  }
}

// ----------------------------------------------------------------- host side

inline int64_t up8(int64_t v) { return (v + 7) / 8 * 8; }

inline bool is_cross(const dmt_tm_params& q) {
  return q.kind == DMT_TM_CROSS_LINEAR || q.kind == DMT_TM_CROSS_LOWRANK_LINEAR;
}

// Row length (elements of eb bytes) of a transposed operand whose rows hold `count` batch
// entries: a multiple of 8, and never a multiple of 1 KB in bytes.  With a power-of-two
// row pitch the 256 rows a GEMM block reads in one K step all fall on the same memory channels;
// 128 bytes of (zero) padding spread them.
inline int64_t ld_batch(int64_t count, int eb) {
  int64_t ld = up8(count);
  if ((ld * eb) % 1024 == 0) ld += 128 / eb;
  return ld;
}

// Slices a weight-gradient contraction (M x N outputs, K = batch) is cut into so that a
// launch of `tiles_all` output tiles (all towers) fills the 256 CUs once, as nearly as it can
// without a second, mostly empty round of blocks: each slice at least 1024 long, a multiple
// of 64.
inline void choose_split(const dmt_plan* p, int64_t tiles_all, int64_t K, int* ksplit, int* klen) {
  int ks = (int)std::max<int64_t>(1, std::min<int64_t>(16, 256 / std::max<int64_t>(tiles_all, 1)));
  while (ks > 1 && K / ks < 1024) --ks;
  // A long batch with few tiles (narrow outputs: the contraction is bound by memory latency,
  // one block per CU) measured faster in slices of about 4096 spread over several rounds
  // (Imbalanced: 0.54 against 0.73 ms) than in one round of very long slices.
  if (tiles_all < 256 && K / ks > 4096) ks = (int)std::min<int64_t>(16, (K + 4095) / 4096);
  const int forced = p->sw.tmb_ksplit;
  if (forced > 0 && K / forced >= 128) ks = forced;
  int len = (int)((K + ks - 1) / ks);
  len = (len + 63) / 64 * 64;
  *ksplit = (int)((K + len - 1) / len);
  *klen = len;
}

struct TowerBwdWs {
  int np = 0, np_pad = 0;
  int kin = 0;                 // row length of the projection's GEMM operand (np_pad + wt for dots)
  int64_t Op = 0;
  size_t dz = 0, dzT = 0, wT = 0, zT = 0;
  size_t p = 0, wp = 0, dZ = 0;                                 // dot towers
  size_t xl[DMT_MAX_CROSS_LAYERS] = {}, u[DMT_MAX_CROSS_LAYERS] = {};   // cross towers
  size_t dxn = 0, du = 0, duT = 0, wlT = 0;
  // low-rank cross towers: t_l = V_l x_l per layer; per-layer scratch t^T, U_l^T, V_l^T,
  // dt (float32), dt rounded and its transpose; rp = rank padded to 8
  size_t tl[DMT_MAX_CROSS_LAYERS] = {};
  size_t tT = 0, uT = 0, vT = 0, dtf = 0, dtq = 0, dtT = 0;
  int rp = 0;
  // DLRM towers: the shared per-feature layer's operands (rows = (sample, feature))
  int64_t Fp = 0;              // feat_out padded to 8
  size_t dz2 = 0, dz2T = 0, wcomb = 0, x2T = 0, part2 = 0;
  int ksplit2 = 1, klen2 = 0;
  size_t part = 0;             // weight-gradient slices (split K) / padded dW of a dot tower
  int ksplit = 1, klen = 0;    // of the projection's weight gradient
  int ksplit_c = 1, klen_c = 0;   // of the cross layers' weight gradients
};

dmt_status plan_tm_bwd(const dmt_plan* p, const dmt_tm_params* tp, int64_t B, int eb,
                       bool have_kept, std::vector<TowerBwdWs>* ws, size_t* bytes) {
  size_t off = 0;
  auto take = [&](size_t b) { size_t o = off; off = dmt_align_up(off + b, 256); return o; };
  const int64_t Bp = ld_batch(B, eb);
  ws->assign(p->T, TowerBwdWs());
  // output tiles of the weight-gradient launches (all towers together), 128 x 128 units
  int64_t tiles_proj = 0, tiles_cross = 0;
  for (int32_t t = 0; t < p->T; ++t) {
    const dmt_tm_params& q = tp[t];
    const int64_t wt = p->tower_width[t];
    if (q.out_dim <= 0) return DMT_EINVAL;
    int64_t kin = wt;                                 // columns of the projection's weight gradient
    if (q.kind == DMT_TM_DOT_LINEAR) {
      const int64_t nf = p->tower_ntab[t];
      kin += (nf * (nf - 1) / 2 + 7) / 8 * 8;
    }
    tiles_proj += ((q.out_dim + 255) / 256) * ((kin + 255) / 256);
    if (q.kind == DMT_TM_CROSS_LINEAR) tiles_cross += ((wt + 255) / 256) * ((wt + 255) / 256);
    if (q.kind == DMT_TM_CROSS_LOWRANK_LINEAR) tiles_cross += ((wt + 255) / 256) * ((q.feat_out + 255) / 256);
  }
  for (int32_t t = 0; t < p->T; ++t) {
    const dmt_tm_params& q = tp[t];
    const int64_t wt = p->tower_width[t];
    if (!q.w_proj || !q.b_proj) return DMT_EINVAL;
    if (((uintptr_t)q.w_proj & 15) && q.kind != DMT_TM_DOT_LINEAR) return DMT_EINVAL;
    TowerBwdWs& w = (*ws)[t];
    w.Op = up8(q.out_dim);
    w.kin = (int)wt;
    if (eb == 2) {
      choose_split(p, tiles_proj, Bp, &w.ksplit, &w.klen);
      choose_split(p, std::max<int64_t>(tiles_cross, 1), Bp, &w.ksplit_c, &w.klen_c);
    }
    switch (q.kind) {
      case DMT_TM_LINEAR:
      case DMT_TM_LINEAR_RELU:
        break;
      case DMT_TM_DOT_LINEAR: {
        const int nf = p->tower_ntab[t];
        if (p->tower_uniform_dim[t] == 0) return DMT_ENOTSUP;
        w.np = nf * (nf - 1) / 2;
        w.np_pad = (w.np + 7) / 8 * 8;
        w.kin = w.np_pad + (int)wt;
        w.p = take((size_t)B * w.np_pad * eb);
        w.wp = take((size_t)q.out_dim * w.kin * eb);
        w.dZ = take((size_t)B * w.kin * 4);
        break;
      }
      case DMT_TM_CROSS_LINEAR:
        if (q.num_cross_layers < 1 || q.num_cross_layers > DMT_MAX_CROSS_LAYERS) return DMT_EINVAL;
        for (int l = 0; l < q.num_cross_layers; ++l) {
          if (!q.w_cross[l] || !q.b_cross[l] || ((uintptr_t)q.w_cross[l] & 15)) return DMT_EINVAL;
          if (have_kept) continue;                  // the forward kept them
          w.xl[l] = take((size_t)B * wt * eb);      // x_{l+1}
          w.u[l] = take((size_t)B * wt * eb);
        }
        w.dxn = take((size_t)B * wt * 4);
        w.du = take((size_t)B * wt * eb);
        w.duT = take((size_t)wt * Bp * eb);
        w.wlT = take((size_t)wt * wt * eb);
        break;
      case DMT_TM_CROSS_LOWRANK_LINEAR: {
        const int L = q.num_cross_layers, r = q.feat_out;
        if (L < 1 || 2 * L > DMT_MAX_CROSS_LAYERS || r < 1) return DMT_EINVAL;
        if (eb == 2 && r % 8 != 0) return DMT_ENOTSUP;
        for (int l = 0; l < L; ++l)
          if (!q.w_cross[2 * l] || !q.w_cross[2 * l + 1] || !q.b_cross[l] ||
              (((uintptr_t)q.w_cross[2 * l] | (uintptr_t)q.w_cross[2 * l + 1]) & 15))
            return DMT_EINVAL;
        w.rp = (int)up8(r);
        for (int l = 0; l < L; ++l) {
          w.tl[l] = take((size_t)B * r * eb);
          if (have_kept) continue;
          w.xl[l] = take((size_t)B * wt * eb);
          w.u[l] = take((size_t)B * wt * eb);
        }
        w.dxn = take((size_t)B * wt * 4);
        w.du = take((size_t)B * wt * eb);
        w.duT = take((size_t)wt * Bp * eb);
        w.tT = take((size_t)r * Bp * eb);
        w.uT = take((size_t)r * wt * eb);
        w.vT = take((size_t)wt * w.rp * eb);
        w.dtf = take((size_t)B * r * 4);
        w.dtq = take((size_t)B * w.rp * eb);
        w.dtT = take((size_t)r * Bp * eb);
        break;
      }
      case DMT_TM_DLRM: {
        const int nf = p->tower_ntab[t], n = p->tower_uniform_dim[t];
        if (n == 0) return DMT_ENOTSUP;
        if (q.feat_out < 1 || (int64_t)q.out_dim - (int64_t)nf * q.feat_out < 1) return DMT_EINVAL;
        if (!q.w_cross[0] || !q.b_cross[0] || ((uintptr_t)q.w_cross[0] & 15)) return DMT_EINVAL;
        if (B * nf >= (1LL << 31) - 128) return DMT_ENOTSUP;
        const int64_t BFp = ld_batch(B * nf, eb);
        w.Fp = up8(q.feat_out);
        w.dz2 = take((size_t)B * nf * w.Fp * eb);
        w.dz2T = take((size_t)q.feat_out * BFp * eb);
        // row f n + c: column f n + c of the flat layer's weights, then column c of the shared
        // layer's: what the data gradient of feature f's slice of the pooled block contracts with
        w.wcomb = take((size_t)wt * (up8(q.out_dim - nf * q.feat_out) + w.Fp) * eb);
        w.x2T = take((size_t)n * BFp * eb);
        if (eb == 2) choose_split(p, p->T, BFp, &w.ksplit2, &w.klen2);
        if (w.ksplit2 > 1) w.part2 = take((size_t)w.ksplit2 * q.feat_out * n * 4);
        break;
      }
      default:
        return DMT_EINVAL;
    }
    // rows of the projection's gradient operand: all outputs, or a DLRM tower's flat outputs
    const int64_t O1 = q.kind == DMT_TM_DLRM ? q.out_dim - p->tower_ntab[t] * q.feat_out : q.out_dim;
    w.Op = up8(O1);
    w.dz = take((size_t)B * w.Op * eb);
    w.dzT = take((size_t)O1 * Bp * eb);
    w.wT = take((size_t)w.kin * w.Op * eb);
    w.zT = take((size_t)w.kin * Bp * eb);
    size_t part = 0;
    if (w.ksplit > 1 || q.kind == DMT_TM_DOT_LINEAR)
      part = (size_t)w.ksplit * O1 * w.kin * 4;
    if (q.kind == DMT_TM_CROSS_LINEAR && w.ksplit_c > 1)
      part = std::max(part, (size_t)w.ksplit_c * wt * wt * 4);
    if (q.kind == DMT_TM_CROSS_LOWRANK_LINEAR && w.ksplit_c > 1)
      part = std::max(part, (size_t)w.ksplit_c * wt * q.feat_out * 4);
    if (part) w.part = take(part);
  }
  *bytes = off;
  return DMT_OK;
}

// Items of one grouped launch of a small kernel, with each item's block count.
struct TmbBatch {
  std::vector<TmbItem> items;
  std::vector<int64_t> blocks;
  void add(const TmbItem& it, int64_t nblocks) {
    if (nblocks <= 0) return;
    items.push_back(it);
    blocks.push_back(nblocks);
  }
};

// False when an item alone exceeds the grid limit (nothing of it is launched).
template <typename Kernel>
bool launch_items(const dmt_plan* p, TmbBatch& batch, Kernel kernel, hipStream_t s) {
  bool ok = true;
  for (size_t first = 0; first < batch.items.size();) {
    TmbLaunch L;
    L.n = 0;
    int64_t blocks = 0;
    while (first < batch.items.size() && L.n < kMaxItems &&
           blocks + batch.blocks[first] < (1LL << 30)) {
      L.it[L.n] = batch.items[first];
      L.block_start[L.n] = (int32_t)blocks;
      blocks += batch.blocks[first];
      ++L.n;
      ++first;
    }
    if (L.n == 0) { ok = false; break; }
    L.block_start[L.n] = (int32_t)blocks;
    DmtScope sc_(p, DMT_K_TM_BWD_AUX, s);
    hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(kBlock), 0, s, L);
  }
  batch.items.clear();
  batch.blocks.clear();
  return ok;
}

inline int64_t ew_blocks(int64_t count, int vec) {
  return std::min<int64_t>((count / vec + kBlock - 1) / kBlock, 256 * 8);
}

template <int DT>
void add_transpose(TmbBatch& b, const void* src, int64_t R, int C, int64_t lds, void* dst, int64_t ldd,
                   int fill = 0) {
  constexpr int tile = DT == DMT_F32 ? kTile : kVTile;
  TmbItem it{};
  it.a = src; it.o0 = dst; it.n0 = R; it.n1 = lds; it.n2 = ldd; it.i0 = C; it.i1 = fill;
  it.nbx = (int32_t)(((fill > 0 ? fill : ldd) + tile - 1) / tile);
  b.add(it, (int64_t)it.nbx * ((C + tile - 1) / tile));
}

// Queues a gradient-preparation item (all fields but nbx set) on the 16-byte kernel when its
// shape and alignment allow, else on the one-element kernel.
template <int DT>
void add_prep(TmbBatch& scalar, TmbBatch& vec, TmbItem it) {
  const bool v = DT != DMT_F32 && it.i0 % 4 == 0 && it.n2 % 4 == 0 && (it.i3 == 0 || it.i4 % 4 == 0) &&
                 ((uintptr_t)it.a & 15) == 0;
  const int tile = v ? kVTile : kTile;
  it.nbx = (int32_t)((it.n1 + tile - 1) / tile);
  (v ? vec : scalar).add(it, (int64_t)it.nbx * ((it.i1 + tile - 1) / tile));
}

template <int DT>
bool launch_transposes(const dmt_plan* p, TmbBatch& b, hipStream_t s) {
  if constexpr (DT == DMT_F32) return launch_items(p, b, tmb_transpose<float>, s);
  else return launch_items(p, b, tmb_transpose16, s);
}

template <int DT>
dmt_status run_tm_bwd(const dmt_plan* p, const dmt_tm_params* tp, const std::vector<TowerBwdWs>& ws,
                      const void* pooled, const void* tm_out, int64_t B, const float* dy_all,
                      float* dx_all, const dmt_tm_grads* gr, const char* keptp, char* wsp,
                      hipStream_t s) {
  constexpr int eb = DT == DMT_F32 ? 4 : 2;
  constexpr int V = Ew<DT>::V;
  const char* x_all = (const char*)pooled;
  const int64_t Bp = ld_batch(B, eb);
  std::vector<int64_t> out_prefix(p->T + 1, 0);
  for (int32_t t = 0; t < p->T; ++t) out_prefix[t + 1] = out_prefix[t] + tp[t].out_dim;
  auto x_of = [&](int t) { return (const void*)(x_all + (size_t)B * p->width_prefix[t] * eb); };
  auto dx_of = [&](int t) { return dx_all + (size_t)B * p->width_prefix[t]; };
  // x_l and u_l of a cross tower (x_0 is the pooled block itself): kept by the forward, or
  // recomputed below into the workspace
  std::vector<TmKept> kept;
  if (keptp) plan_tm_kept(p, tp, B, eb, &kept);
  auto xl_of = [&](int t, int l) -> const void* {
    if (l == 0) return x_of(t);
    return keptp ? (const void*)(keptp + kept[t].x[l - 1]) : (const void*)(wsp + ws[t].xl[l - 1]);
  };
  auto u_of = [&](int t, int l) -> const void* {
    return keptp ? (const void*)(keptp + kept[t].u[l]) : (const void*)(wsp + ws[t].u[l]);
  };
  int max_layers = 0;
  TmbBatch batch, batch2, batch3, prep16;
  bool ok = true;

  auto z_of = [&](int t) -> const char* {           // dot terms: kept by the forward, or recomputed
    return keptp && kept[t].has_z ? keptp + kept[t].z : (const char*)(wsp + ws[t].p);
  };
  auto wp_of = [&](int t) -> const char* {          // ... and the repacked projection weights
    return keptp && kept[t].has_z ? keptp + kept[t].wp : (const char*)(wsp + ws[t].wp);
  };
  // ---- recompute what the forward did not keep: dot terms (and the repacked weights)
  std::vector<TmAuxItem> dots_mfma, dots_simple, packs;
  std::vector<int64_t> nb_mfma, nb_simple, nb_pack;
  for (int32_t t = 0; t < p->T; ++t) {
    const dmt_tm_params& q = tp[t];
    if (is_cross(q)) max_layers = std::max(max_layers, q.num_cross_layers);
    if (q.kind != DMT_TM_DOT_LINEAR) continue;
    const TowerBwdWs& w = ws[t];
    TmAuxItem it{};
    it.nf = p->tower_ntab[t]; it.n = p->tower_uniform_dim[t]; it.np = w.np; it.np_pad = w.np_pad;
    it.O = q.out_dim; it.wt = p->tower_width[t];
    it.src = x_of(t);
    it.dst = wsp + w.p;
    if (w.np_pad > 0 && !(keptp && kept[t].has_z)) {
      if (DT != DMT_F32 && 32 % it.nf == 0 && it.n % 16 == 0) {
        dots_mfma.push_back(it);
        nb_mfma.push_back(((B * it.nf + 31) / 32 + 3) / 4);
      } else {
        dots_simple.push_back(it);
        nb_simple.push_back((B * w.np_pad + kBlock - 1) / kBlock);
      }
    }
    if (keptp && kept[t].has_z) continue;
    it.src = q.w_proj;
    it.dst = wsp + w.wp;
    packs.push_back(it);
    nb_pack.push_back(((int64_t)q.out_dim * w.kin + kBlock - 1) / kBlock);
  }
  launch_aux<DT>(p, B, dots_mfma, nb_mfma, 0, s);
  launch_aux<DT>(p, B, dots_simple, nb_simple, 1, s);
  launch_aux<DT>(p, B, packs, nb_pack, 2, s);

  // ---- ... and the cross layers' u_l = x_l W_l^T + b_l, x_{l+1} = x0 * u_l + x_l, both from one
  // contraction as in the training forward (low-rank layers: t_l = x_l V_l^T first, which the
  // backward needs whether or not the rest was kept, then u_l = t_l U_l^T + b_l)
  std::vector<TmGroup> groups, groups_t;
  for (int l = 0; l < max_layers; ++l) {
    for (int32_t t = 0; t < p->T; ++t) {
      const dmt_tm_params& q = tp[t];
      if (!is_cross(q) || l >= q.num_cross_layers) continue;
      const int wt = p->tower_width[t];
      TmGroup g{};
      g.A1 = xl_of(t, l); g.lda1 = wt; g.K1 = wt;
      g.W = q.w_cross[l]; g.ldw = wt; g.bias = q.b_cross[l];
      if (q.kind == DMT_TM_CROSS_LOWRANK_LINEAR) {
        const int r = q.feat_out;
        TmGroup h{};
        h.A1 = xl_of(t, l); h.lda1 = wt; h.K1 = wt;
        h.W = q.w_cross[2 * l]; h.ldw = wt; h.bias = nullptr;
        h.C = wsp + ws[t].tl[l]; h.ldc = r;
        h.M = (int32_t)B; h.N = r; h.epi = EPI_BIAS;
        groups_t.push_back(h);
        g.A1 = wsp + ws[t].tl[l]; g.lda1 = r; g.K1 = r;
        g.W = q.w_cross[2 * l + 1]; g.ldw = r;
        g.XL = xl_of(t, l); g.ldxl = wt;
      }
      if (keptp) continue;
      // exactly the training forward's contraction: x_{l+1} from the cross epilogue, u_l on the side
      g.X0 = x_of(t); g.ldx = wt;
      g.C = wsp + ws[t].xl[l]; g.ldc = wt;
      g.U = wsp + ws[t].u[l];
      g.M = (int32_t)B; g.N = wt; g.epi = EPI_CROSS;
      groups.push_back(g);
    }
    launch_groups<DT>(p, groups_t, s, false, DMT_K_TM_BWD_GEMM);
    launch_groups<DT>(p, groups, s, false, DMT_K_TM_BWD_GEMM);
  }

  // ---- projection: operands, bias gradient, then both contractions for all towers
  std::vector<TmGroup> dgrad, dgrad2, wgrad, wgrad2;
  for (int32_t t = 0; t < p->T; ++t) {
    const dmt_tm_params& q = tp[t];
    const TowerBwdWs& w = ws[t];
    const int wt = p->tower_width[t];
    const bool dot = q.kind == DMT_TM_DOT_LINEAR;
    const bool dlrm = q.kind == DMT_TM_DLRM;
    // outputs of the projection: all of the tower's, or a DLRM tower's flat ones
    const int O = dlrm ? q.out_dim - p->tower_ntab[t] * q.feat_out : q.out_dim;
    {
      TmbItem it{};
      it.a = dy_all + (size_t)B * out_prefix[t];
      it.i2 = q.kind == DMT_TM_LINEAR_RELU;
      it.b = it.i2 ? (const void*)((const char*)tm_out + (size_t)B * out_prefix[t] * eb) : nullptr;
      it.o0 = wsp + w.dz; it.o1 = wsp + w.dzT;
      it.n0 = B; it.n1 = Bp; it.n2 = q.out_dim; it.i0 = O; it.i1 = (int32_t)w.Op;
      add_prep<DT>(batch, prep16, it);
    }
    {
      TmbItem it{};
      it.a = wsp + w.dzT; it.o0 = gr[t].db_proj; it.n0 = Bp; it.n1 = B;
      batch2.add(it, O);
    }
    // W^T [kin][Op] (a DLRM tower's goes into its combined weights below)
    if (!dlrm)
      add_transpose<DT>(batch3, dot ? (const void*)wp_of(t) : q.w_proj, O, w.kin, w.kin,
                        wsp + w.wT, w.Op);
    // z^T [kin][Bp]: the projection's input, transposed
    if (dot) {
      if (w.np_pad > 0) add_transpose<DT>(batch3, z_of(t), B, w.np_pad, w.np_pad, wsp + w.zT, Bp);
      add_transpose<DT>(batch3, x_of(t), B, wt, wt, wsp + w.zT + (size_t)w.np_pad * Bp * eb, Bp);
    } else {
      const void* z = is_cross(q) ? xl_of(t, q.num_cross_layers) : x_of(t);
      add_transpose<DT>(batch3, z, B, wt, wt, wsp + w.zT, Bp);
    }
    TmGroup g{};
    g.A1 = wsp + w.dz; g.lda1 = (int32_t)w.Op; g.K1 = (int32_t)w.Op;
    g.W = wsp + w.wT; g.ldw = (int32_t)w.Op;
    g.M = (int32_t)B; g.N = w.kin; g.epi = EPI_F32;
    if (dot) { g.C = wsp + w.dZ; g.ldc = w.kin; }
    else if (is_cross(q)) { g.C = wsp + w.dxn; g.ldc = wt; }
    else { g.C = dx_of(t); g.ldc = wt; }
    if (!dlrm) dgrad.push_back(g);
    TmGroup h{};
    h.A1 = wsp + w.dzT; h.lda1 = (int32_t)Bp; h.K1 = (int32_t)Bp;
    h.W = wsp + w.zT; h.ldw = (int32_t)Bp;
    h.M = O; h.N = w.kin; h.epi = EPI_F32;
    h.ksplit = w.ksplit; h.klen = w.klen; h.cstride = (int64_t)O * w.kin;
    h.C = (dot || w.ksplit > 1) ? (void*)(wsp + w.part) : (void*)gr[t].dw_proj;
    h.ldc = w.kin;
    wgrad.push_back(h);
    if (dlrm) {
      // the shared per-feature layer: the same steps on rows (sample, feature)
      const int nf = p->tower_ntab[t], n = p->tower_uniform_dim[t], F = q.feat_out;
      const int64_t BF = B * nf, BFp = ld_batch(BF, eb);
      {
        TmbItem it{};
        it.a = dy_all + (size_t)B * out_prefix[t] + O;
        it.o0 = wsp + w.dz2; it.o1 = wsp + w.dz2T;
        it.n0 = BF; it.n1 = BFp; it.n2 = q.out_dim; it.i0 = F; it.i1 = (int32_t)w.Fp;
        it.i3 = nf; it.i4 = F;
        add_prep<DT>(batch, prep16, it);
      }
      {
        TmbItem it{};
        it.a = wsp + w.dz2T; it.o0 = gr[t].db_cross[0]; it.n0 = BFp; it.n1 = BF;
        batch2.add(it, F);
      }
      add_transpose<DT>(batch3, x_of(t), BF, n, n, wsp + w.x2T, BFp);
      // data gradient, both layers in one contraction per feature f: the pooled block's columns
      // f n .. f n + n - 1 receive [dz1 | dz2 of feature f] . [W1^T rows f n .. | W_f^T], so
      // grad_pooled is written once; the combined weights are rows of Op + Fp columns
      const int kc = (int)(w.Op + w.Fp);
      add_transpose<DT>(batch3, q.w_proj, O, wt, wt, wsp + w.wcomb, kc, (int)w.Op);
      for (int f = 0; f < nf; ++f) {
        add_transpose<DT>(batch3, q.w_cross[0], F, n, n,
                          wsp + w.wcomb + ((size_t)f * n * kc + w.Op) * eb, kc, (int)w.Fp);
        TmGroup g2{};
        g2.A0 = wsp + w.dz; g2.lda0 = (int32_t)w.Op; g2.K0 = (int32_t)w.Op;
        g2.A1 = wsp + w.dz2 + (size_t)f * w.Fp * eb; g2.lda1 = (int32_t)(nf * w.Fp); g2.K1 = (int32_t)w.Fp;
        g2.W = wsp + w.wcomb + (size_t)f * n * kc * eb; g2.ldw = kc;
        g2.M = (int32_t)B; g2.N = n; g2.epi = EPI_F32;
        g2.C = dx_of(t) + (size_t)f * n; g2.ldc = wt;
        dgrad2.push_back(g2);
      }
      TmGroup h2{};
      h2.A1 = wsp + w.dz2T; h2.lda1 = (int32_t)BFp; h2.K1 = (int32_t)BFp;
      h2.W = wsp + w.x2T; h2.ldw = (int32_t)BFp;
      h2.M = F; h2.N = n; h2.epi = EPI_F32;
      h2.ksplit = w.ksplit2; h2.klen = w.klen2; h2.cstride = (int64_t)F * n;
      h2.C = w.ksplit2 > 1 ? (void*)(wsp + w.part2) : (void*)gr[t].dw_cross[0];
      h2.ldc = n;
      wgrad2.push_back(h2);
    }
  }
  ok &= launch_items(p, batch, tmb_prep_dy<DT>, s);
  if constexpr (DT != DMT_F32) ok &= launch_items(p, prep16, tmb_prep_dy16<DT>, s);
  ok &= launch_items(p, batch2, tmb_rowsum<DT>, s);
  ok &= launch_transposes<DT>(p, batch3, s);
  launch_groups<DT>(p, dgrad, s, false, DMT_K_TM_BWD_GEMM);
  launch_groups<DT>(p, dgrad2, s, false, DMT_K_TM_BWD_GEMM);
  launch_groups<DT>(p, wgrad, s, false, DMT_K_TM_BWD_GEMM);
  launch_groups<DT>(p, wgrad2, s, false, DMT_K_TM_BWD_GEMM);

  // ---- weight gradients: add up the slices, strip a dot tower's padding; dot towers: fold
  // the dot terms' gradients into dx
  for (int32_t t = 0; t < p->T; ++t) {
    const dmt_tm_params& q = tp[t];
    const TowerBwdWs& w = ws[t];
    const int wt = p->tower_width[t];
    const bool dot = q.kind == DMT_TM_DOT_LINEAR;
    const int O = q.kind == DMT_TM_DLRM ? q.out_dim - p->tower_ntab[t] * q.feat_out : q.out_dim;
    if (dot || w.ksplit > 1) {
      TmbItem it{};
      it.a = wsp + w.part; it.o0 = gr[t].dw_proj; it.n0 = (int64_t)O * w.kin;
      it.i0 = O; it.i1 = w.np; it.i2 = w.np_pad; it.i3 = wt; it.i4 = w.ksplit;
      batch.add(it, ((int64_t)O * (w.np + wt) + kBlock - 1) / kBlock);
    }
    if (q.kind == DMT_TM_DLRM && w.ksplit2 > 1) {
      const int n = p->tower_uniform_dim[t];
      TmbItem it{};
      it.a = wsp + w.part2; it.o0 = gr[t].dw_cross[0]; it.n0 = (int64_t)q.feat_out * n;
      it.i0 = q.feat_out; it.i1 = 0; it.i2 = 0; it.i3 = n; it.i4 = w.ksplit2;
      batch.add(it, ((int64_t)q.feat_out * n + kBlock - 1) / kBlock);
    }
    if (dot) {
      TmbItem it{};
      it.a = x_of(t); it.b = wsp + w.dZ; it.o0 = dx_of(t); it.n0 = B;
      it.i0 = p->tower_ntab[t]; it.i1 = p->tower_uniform_dim[t]; it.i2 = w.np_pad; it.i3 = w.kin;
      if (DT != DMT_F32 && it.i1 % 8 == 0) batch3.add(it, (B * (wt / 8) + kBlock - 1) / kBlock);
      else batch2.add(it, (B * wt + kBlock - 1) / kBlock);
    }
  }
  ok &= launch_items(p, batch, tmb_sum_slices, s);
  ok &= launch_items(p, batch2, tmb_dot_bwd<DT>, s);
  if constexpr (DT != DMT_F32) ok &= launch_items(p, batch3, tmb_dot_bwd8<DT>, s);

  // ---- cross towers: layers from the last to the first; dx0 accumulates in the output block,
  // where the first layer's data gradient then lands on top of it
  TmbBatch sums, sums2, prep_dt, prep_dt16, prep_t;
  for (int l = max_layers - 1; l >= 0; --l) {
    for (int32_t t = 0; t < p->T; ++t) {
      const dmt_tm_params& q = tp[t];
      if (!is_cross(q) || l >= q.num_cross_layers) continue;
      const TowerBwdWs& w = ws[t];
      const int wt = p->tower_width[t];
      {
        TmbItem it{};
        it.a = wsp + w.dxn; it.b = x_of(t); it.c = u_of(t, l); it.o0 = wsp + w.du; it.o1 = dx_of(t);
        it.i0 = l == q.num_cross_layers - 1; it.i1 = l == 0;
        if constexpr (DT == DMT_F32) {
          it.n0 = B * wt;
          it.nbx = (int32_t)ew_blocks(it.n0, V);
          batch.add(it, it.nbx);
          add_transpose<DT>(batch2, wsp + w.du, B, wt, wt, wsp + w.duT, Bp);
        } else {                                     // du and du^T from one pass
          it.o2 = wsp + w.duT; it.n0 = B; it.n1 = Bp; it.i2 = wt;
          it.nbx = (int32_t)((Bp + kVTile - 1) / kVTile);
          prep_t.add(it, (int64_t)it.nbx * ((wt + kVTile - 1) / kVTile));
        }
      }
      add_transpose<DT>(batch2, xl_of(t, l), B, wt, wt, wsp + w.zT, Bp);
      {
        TmbItem it{};
        it.a = wsp + w.duT; it.o0 = gr[t].db_cross[l]; it.n0 = Bp; it.n1 = B;
        batch3.add(it, wt);
      }
      if (q.kind == DMT_TM_CROSS_LOWRANK_LINEAR) {
        // stage 1: dt = du U_l (float32) and dU_l = du^T t_l; stage 2, once dt is rounded and
        // transposed: dx_l = dt V_l + dx_{l+1} and dV_l = dt^T x_l
        const int r = q.feat_out;
        add_transpose<DT>(batch2, wsp + w.tl[l], B, r, r, wsp + w.tT, Bp);
        add_transpose<DT>(batch2, q.w_cross[2 * l + 1], wt, r, r, wsp + w.uT, wt);     // U_l^T [r][wt]
        add_transpose<DT>(batch2, q.w_cross[2 * l], r, wt, wt, wsp + w.vT, w.rp);      // V_l^T [wt][rp]
        TmGroup g1{};
        g1.A1 = wsp + w.du; g1.lda1 = wt; g1.K1 = wt;
        g1.W = wsp + w.uT; g1.ldw = wt;
        g1.M = (int32_t)B; g1.N = r; g1.epi = EPI_F32;
        g1.C = wsp + w.dtf; g1.ldc = r;
        dgrad.push_back(g1);
        TmGroup h1{};
        h1.A1 = wsp + w.duT; h1.lda1 = (int32_t)Bp; h1.K1 = (int32_t)Bp;
        h1.W = wsp + w.tT; h1.ldw = (int32_t)Bp;
        h1.M = wt; h1.N = r; h1.epi = EPI_F32;
        h1.ksplit = w.ksplit_c; h1.klen = w.klen_c; h1.cstride = (int64_t)wt * r;
        h1.C = w.ksplit_c > 1 ? (void*)(wsp + w.part) : (void*)gr[t].dw_cross[2 * l + 1];
        h1.ldc = r;
        wgrad.push_back(h1);
        if (w.ksplit_c > 1) {
          TmbItem it{};
          it.a = wsp + w.part; it.o0 = gr[t].dw_cross[2 * l + 1]; it.n0 = (int64_t)wt * r;
          it.i0 = wt; it.i1 = 0; it.i2 = 0; it.i3 = r; it.i4 = w.ksplit_c;
          sums.add(it, ((int64_t)wt * r + kBlock - 1) / kBlock);
        }
        {
          TmbItem it{};
          it.a = wsp + w.dtf; it.o0 = wsp + w.dtq; it.o1 = wsp + w.dtT;
          it.n0 = B; it.n1 = Bp; it.n2 = r; it.i0 = r; it.i1 = w.rp;
          add_prep<DT>(prep_dt, prep_dt16, it);
        }
        TmGroup g2{};
        g2.A1 = wsp + w.dtq; g2.lda1 = w.rp; g2.K1 = w.rp;
        g2.W = wsp + w.vT; g2.ldw = w.rp;
        g2.M = (int32_t)B; g2.N = wt; g2.epi = EPI_F32_ADD;
        g2.C = l == 0 ? (void*)dx_of(t) : (void*)(wsp + w.dxn); g2.ldc = wt;
        dgrad2.push_back(g2);
        TmGroup h2{};
        h2.A1 = wsp + w.dtT; h2.lda1 = (int32_t)Bp; h2.K1 = (int32_t)Bp;
        h2.W = wsp + w.zT; h2.ldw = (int32_t)Bp;
        h2.M = r; h2.N = wt; h2.epi = EPI_F32;
        h2.ksplit = w.ksplit_c; h2.klen = w.klen_c; h2.cstride = (int64_t)r * wt;
        h2.C = w.ksplit_c > 1 ? (void*)(wsp + w.part) : (void*)gr[t].dw_cross[2 * l];
        h2.ldc = wt;
        wgrad2.push_back(h2);
        if (w.ksplit_c > 1) {
          TmbItem it{};
          it.a = wsp + w.part; it.o0 = gr[t].dw_cross[2 * l]; it.n0 = (int64_t)r * wt;
          it.i0 = r; it.i1 = 0; it.i2 = 0; it.i3 = wt; it.i4 = w.ksplit_c;
          sums2.add(it, ((int64_t)r * wt + kBlock - 1) / kBlock);
        }
        continue;
      }
      add_transpose<DT>(batch2, q.w_cross[l], wt, wt, wt, wsp + w.wlT, wt);
      TmGroup g{};
      g.A1 = wsp + w.du; g.lda1 = wt; g.K1 = wt;
      g.W = wsp + w.wlT; g.ldw = wt;
      g.M = (int32_t)B; g.N = wt; g.epi = EPI_F32_ADD;
      g.C = l == 0 ? (void*)dx_of(t) : (void*)(wsp + w.dxn); g.ldc = wt;
      dgrad.push_back(g);
      TmGroup h{};
      h.A1 = wsp + w.duT; h.lda1 = (int32_t)Bp; h.K1 = (int32_t)Bp;
      h.W = wsp + w.zT; h.ldw = (int32_t)Bp;
      h.M = wt; h.N = wt; h.epi = EPI_F32;
      h.ksplit = w.ksplit_c; h.klen = w.klen_c; h.cstride = (int64_t)wt * wt;
      h.C = w.ksplit_c > 1 ? (void*)(wsp + w.part) : (void*)gr[t].dw_cross[l];
      h.ldc = wt;
      wgrad.push_back(h);
      if (w.ksplit_c > 1) {
        TmbItem it{};
        it.a = wsp + w.part; it.o0 = gr[t].dw_cross[l]; it.n0 = (int64_t)wt * wt;
        it.i0 = wt; it.i1 = 0; it.i2 = 0; it.i3 = wt; it.i4 = w.ksplit_c;
        sums.add(it, ((int64_t)wt * wt + kBlock - 1) / kBlock);
      }
    }
    ok &= launch_items(p, batch, tmb_cross_prep<DT>, s);
    if constexpr (DT != DMT_F32) ok &= launch_items(p, prep_t, tmb_cross_prep_t<DT>, s);
    ok &= launch_transposes<DT>(p, batch2, s);
    ok &= launch_items(p, batch3, tmb_rowsum<DT>, s);
    launch_groups<DT>(p, dgrad, s, false, DMT_K_TM_BWD_GEMM);
    launch_groups<DT>(p, wgrad, s, false, DMT_K_TM_BWD_GEMM);
    ok &= launch_items(p, sums, tmb_sum_slices, s);
    // low-rank towers, stage 2 (the slices' buffer is free again after the sums above)
    ok &= launch_items(p, prep_dt, tmb_prep_dy<DT>, s);
    if constexpr (DT != DMT_F32) ok &= launch_items(p, prep_dt16, tmb_prep_dy16<DT>, s);
    launch_groups<DT>(p, dgrad2, s, false, DMT_K_TM_BWD_GEMM);
    launch_groups<DT>(p, wgrad2, s, false, DMT_K_TM_BWD_GEMM);
    ok &= launch_items(p, sums2, tmb_sum_slices, s);
  }
  if (!ok) return DMT_ENOTSUP;
  return hipGetLastError() == hipSuccess ? DMT_OK : DMT_EHIP;
}

}  // namespace

extern "C" size_t dmt_tm_bwd_workspace_bytes(const dmt_plan* plan, const dmt_tm_params* per_tower,
                                             int64_t B) {
  if (!plan || !per_tower || B <= 0) return 0;
  // enough for every dtype: the 16-bit layouts have smaller operands but may split K
  return dmt_guard_size([&]() -> size_t {
    std::vector<TowerBwdWs> ws;
    size_t b4 = 0, b2 = 0;
    if (plan_tm_bwd(plan, per_tower, B, 4, false, &ws, &b4) != DMT_OK) return 0;
    if (plan_tm_bwd(plan, per_tower, B, 2, false, &ws, &b2) != DMT_OK) b2 = 0;   // e.g. a rank no multiple of 8
    return std::max(b4, b2);
  });
}

extern "C" dmt_status dmt_tower_module_bwd(const dmt_plan* plan, const dmt_tm_params* per_tower,
                                           const void* pooled, const void* tm_out, int64_t B,
                                           const float* grad_tm_out, int32_t dtype_code,
                                           float* grad_pooled, const dmt_tm_grads* grads,
                                           const void* kept, size_t kept_bytes, void* workspace,
                                           size_t workspace_bytes, void* stream) {
  if (!plan || !per_tower || !pooled || !grad_tm_out || !grad_pooled || !grads) return DMT_EINVAL;
  if (B <= 0 || B > plan->max_batch || B >= (1LL << 31) - 128) return DMT_EINVAL;
  if (dtype_code != DMT_F32 && dtype_code != DMT_F16 && dtype_code != DMT_BF16) return DMT_EINVAL;
  const dmt_dtype dtype = (dmt_dtype)dtype_code;
  if (((uintptr_t)pooled & 15) || ((uintptr_t)tm_out & 15) || ((uintptr_t)grad_pooled & 15) ||
      ((uintptr_t)grad_tm_out & 3))
    return DMT_EINVAL;
  const int eb = dmt_elt_bytes(dtype);
  for (int32_t t = 0; t < plan->T; ++t) {
    if (plan->tower_width[t] % 8 != 0 && dtype != DMT_F32) return DMT_ENOTSUP;
    const dmt_tm_params& q = per_tower[t];
    if (q.kind == DMT_TM_LINEAR_RELU && !tm_out) return DMT_EINVAL;
    if (!grads[t].dw_proj || !grads[t].db_proj) return DMT_EINVAL;
    if (q.kind == DMT_TM_CROSS_LINEAR)
      for (int l = 0; l < q.num_cross_layers && l < DMT_MAX_CROSS_LAYERS; ++l)
        if (!grads[t].dw_cross[l] || !grads[t].db_cross[l]) return DMT_EINVAL;
    if (q.kind == DMT_TM_DLRM && (!grads[t].dw_cross[0] || !grads[t].db_cross[0])) return DMT_EINVAL;
    if (q.kind == DMT_TM_CROSS_LOWRANK_LINEAR)
      for (int l = 0; l < q.num_cross_layers && 2 * l + 1 < DMT_MAX_CROSS_LAYERS; ++l)
        if (!grads[t].dw_cross[2 * l] || !grads[t].dw_cross[2 * l + 1] || !grads[t].db_cross[l])
          return DMT_EINVAL;
  }
  return dmt_guard([&]() -> dmt_status {
  std::vector<TowerBwdWs> ws;
  size_t bytes = 0;
  const char* keptp = nullptr;
  if (kept) {
    std::vector<TmKept> k;
    const size_t need = plan_tm_kept(plan, per_tower, B, eb, &k);
    if ((uintptr_t)kept & 255) return DMT_EINVAL;
    if (kept_bytes < need) return DMT_ENOMEM;
    if (need > 0) keptp = (const char*)kept;
  }
  dmt_status st = plan_tm_bwd(plan, per_tower, B, eb, keptp != nullptr, &ws, &bytes);
  if (st != DMT_OK) return st;
  if (!workspace || ((uintptr_t)workspace & 255)) return DMT_EINVAL;
  if (workspace_bytes < bytes) return DMT_ENOMEM;
  hipStream_t s = (hipStream_t)stream;
  char* wsp = (char*)workspace;
  switch (dtype) {
    case DMT_F32:
      return run_tm_bwd<DMT_F32>(plan, per_tower, ws, pooled, tm_out, B, grad_tm_out, grad_pooled,
                                 grads, keptp, wsp, s);
    case DMT_F16:
      return run_tm_bwd<DMT_F16>(plan, per_tower, ws, pooled, tm_out, B, grad_tm_out, grad_pooled,
                                 grads, keptp, wsp, s);
    default:
      return run_tm_bwd<DMT_BF16>(plan, per_tower, ws, pooled, tm_out, B, grad_tm_out, grad_pooled,
                                  grads, keptp, wsp, s);
  }
  });
}
