// dmt_tower_module_fwd: the per-tower Tower Module (paper Sec. 3.2, Sec. 4).
//
// Every form is a chain of  C = epilogue(A . W^T + b)  contractions over the
// tower's [B][W_t] block of the pooled tensor:
//   linear(+ReLU)  one projection                                (Listing 1, c = 0)
//   dot + linear   pairwise feature dot products z_p, then a projection of
//                  [z_p | x]                                      (Sec. 3.2, Sec. 4)
//   cross + linear x_{l+1} = x0 * (W_l x_l + b_l) + x_l, then a projection
//                                                                 (Listing 2)
// 16-bit types run on MFMA (v_mfma_f32_32x32x16, float32 accumulate): block tile
// 128 x 128 x 64, four waves of 64 x 64, operands staged through padded LDS, the
// next K tile prefetched into registers while the current one is multiplied.
// All towers of one stage go into ONE launch (a grouped GEMM: block id -> tower,
// tile), because a single tower's grid cannot fill 256 CUs.  The pairwise dots
// are a Gram matrix per sample: 32 consecutive (sample, feature) rows form one
// 32 x 32 MFMA tile whose diagonal blocks hold every sample's dots, so the
// operand is read once, straight from global memory, as both A and B.
// float32 towers (a latency-bound toy size) use plain FMA kernels.
#include <algorithm>

#include "dmt_internal.h"
#include "dmt_device_utils.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kBlock = 256;
constexpr int BM = 128, BN = 128, BK = 64;
constexpr int kLdsStride = BK + 8;       // elements; 144-byte rows keep ds_read_b128 conflict-free
constexpr int kMaxGroups = 16;

enum { EPI_BIAS = 0, EPI_BIAS_RELU = 1, EPI_CROSS = 2 };

// One contraction of a grouped launch.  A is given as two K segments (the dot
// terms, then the pooled values); a plain GEMM has K0 = 0.
struct TmGroup {
  const void* A0;   // [M][lda0], first K0 columns of the operand
  const void* A1;   // [M][lda1], next K1 columns
  const void* W;    // [N][ldw], K0 + K1 columns used
  const void* bias; // [N]
  const void* X0;   // EPI_CROSS: [M][ldx] (x0); the x_l term is A1
  void* C;          // [M][ldc]
  int32_t lda0, K0, lda1, K1, ldw, ldc, ldx, M, N, epi;
  int32_t nf, fdim;       // dot terms computed in-kernel: number of features and their dim
};

struct TmLaunch {
  int32_t ngroups;
  int32_t tile_start[kMaxGroups + 1];
  TmGroup g[kMaxGroups];
};

template <int DT>
__device__ __forceinline__ floatx16 mfma32(uint4 a, uint4 b, floatx16 c) {
  if constexpr (DT == DMT_BF16)
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(halfx8, a),
                                                  __builtin_bit_cast(halfx8, b), c, 0, 0, 0);
}

template <int DT> __device__ __forceinline__ float load_elt(const void* p, int64_t i) {
  if constexpr (DT == DMT_F32) return ((const float*)p)[i];
  else if constexpr (DT == DMT_F16) return dmt::f16_bits_to_f32(((const uint16_t*)p)[i]);
  else return dmt::bf16_lo(((const uint16_t*)p)[i]);
}

template <int DT> __device__ __forceinline__ void store_elt(void* p, int64_t i, float v) {
  if constexpr (DT == DMT_F32) ((float*)p)[i] = v;
  else if constexpr (DT == DMT_F16) ((uint16_t*)p)[i] = (uint16_t)dmt::f32_to_f16_bits(v);
  else ((uint16_t*)p)[i] = (uint16_t)dmt::f32_to_bf16_bits(v);
}

// ------------------------------------------------------------- MFMA grouped GEMM

template <int DT>
__global__ __launch_bounds__(kBlock, 2) void tm_gemm_mfma(const TmLaunch L) {
  __shared__ __attribute__((aligned(16))) uint16_t As[BM * kLdsStride];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[BN * kLdsStride];
  int gi = 0;
  while (gi + 1 < L.ngroups && (int)blockIdx.x >= L.tile_start[gi + 1]) ++gi;
  const TmGroup& G = L.g[gi];
  const int tile = blockIdx.x - L.tile_start[gi];
  const int tiles_n = (G.N + BN - 1) / BN;
  const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;
  const int M = G.M, N = G.N, K0 = G.K0, K = G.K0 + G.K1;
  const uint16_t* A0 = (const uint16_t*)G.A0;
  const uint16_t* A1 = (const uint16_t*)G.A1;
  const uint16_t* W = (const uint16_t*)G.W;
  const int lda0 = G.lda0, lda1 = G.lda1, ldw = G.ldw;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  // staging: chunk c = tid + 256*i covers row c/8, 8 elements at column (c%8)*8
  const int srow = tid >> 3, scol = (tid & 7) * 8;

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  uint4 ra[4], rb[4];
  auto load_tile = [&](int kt) {
    const int k = kt * BK + scol;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = m0 + srow + i * 32;
      ra[i] = make_uint4(0, 0, 0, 0);
      if (m < M && k < K)
        ra[i] = (k < K0) ? *(const uint4*)(A0 + (int64_t)m * lda0 + k)
                         : *(const uint4*)(A1 + (int64_t)m * lda1 + (k - K0));
      const int n = n0 + srow + i * 32;
      rb[i] = make_uint4(0, 0, 0, 0);
      if (n < N && k < K) rb[i] = *(const uint4*)(W + (int64_t)n * ldw + k);
    }
  };
  auto store_tile = [&]() {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      *(uint4*)(As + (srow + i * 32) * kLdsStride + scol) = ra[i];
      *(uint4*)(Bs + (srow + i * 32) * kLdsStride + scol) = rb[i];
    }
  };

  const int nk = (K + BK - 1) / BK;
  load_tile(0);
  for (int kt = 0; kt < nk; ++kt) {
    store_tile();
    __syncthreads();
    if (kt + 1 < nk) load_tile(kt + 1);
    const uint16_t* ap = As + (wm * 64 + (lane & 31)) * kLdsStride + (lane >> 5) * 8;
    const uint16_t* bp = Bs + (wn * 64 + (lane & 31)) * kLdsStride + (lane >> 5) * 8;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      uint4 a[2], b[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        a[i] = *(const uint4*)(ap + i * 32 * kLdsStride + kk * 16);
        b[i] = *(const uint4*)(bp + i * 32 * kLdsStride + kk * 16);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = mfma32<DT>(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }

  // epilogue: lane holds column n = lane % 32 of rows (v/4)*8 + (lane/32)*4 + v%4
  const int epi = G.epi;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int n = n0 + wn * 64 + j * 32 + (lane & 31);
    if (n >= N) continue;
    const float bias = load_elt<DT>(G.bias, n);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = m0 + wm * 64 + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
        if (m >= M) continue;
        float y = acc[i][j][v] + bias;
        if (epi == EPI_BIAS_RELU) y = y > 0.f ? y : 0.f;
        if (epi == EPI_CROSS)
          y = load_elt<DT>(G.X0, (int64_t)m * G.ldx + n) * y + load_elt<DT>(G.A1, (int64_t)m * lda1 + n);
        store_elt<DT>(G.C, (int64_t)m * G.ldc + n, y);
      }
    }
  }
}

// ------------------------------------------- MFMA grouped GEMM, 256 x 256 tiles
//
// For wide outputs (N > 128).  A 128 x 128 block tile needs 1 byte from L2 per 64
// FLOP, which caps the matrix cores at a fraction of their rate; 256 x 256 halves
// that.  Eight waves (two per SIMD, so one wave's LDS waits hide behind the other's
// MFMAs) of 128 x 64 each (4 x 2 MFMA tiles, 128 accumulator registers), one block
// per CU, two LDS stages (147 KB of the CU's 160 KB): tile k+1 goes from registers
// to LDS and the global loads of tile k+2 are issued before the MFMAs of tile k, so
// a whole K step of matrix work covers the memory latency and one barrier per K
// step suffices.
constexpr int LBM = 256, LBN = 256;
constexpr int kBigThreads = 512;
constexpr int kSuper = 32;                                  // tiles an XCD keeps resident (its CUs)
constexpr int kBigTileElems = LBM * kLdsStride;            // one operand, one stage
constexpr int kBigLdsBytes = 4 * kBigTileElems * 2;         // 2 stages x (A + B)

// DOTS: the operand's first K0 columns are the tower's pairwise dot terms, which the block
// computes itself (Gram tiles, as in tm_dots_mfma) straight into the first LDS stage, so the
// pooled tensor is read once and the dot terms never exist in global memory.
template <int DT, bool DOTS>
__global__ __launch_bounds__(kBigThreads, 1) void tm_gemm_mfma_256(const TmLaunch L) {
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
  // XCD-aware rasterisation.  Consecutive block ids go to different XCDs, so block b belongs
  // to XCD b % 8 and is that XCD's (b / 8)-th block.  The launch's tiles are cut into
  // super-tiles of up to kSuper tiles (a few tile rows x all tile columns of one group) that
  // are dealt to the XCDs in turn: the 32 blocks resident on an XCD then share their A rows
  // and W columns in that XCD's L2 instead of every XCD pulling every A tile over the fabric.
  // Here L.tile_start[] counts super-tiles.
  const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
  const int gs = (idx / kSuper) * 8 + xcd, within = idx % kSuper;
  if (gs >= L.tile_start[L.ngroups]) return;
  int gi = 0;
  while (gi + 1 < L.ngroups && gs >= L.tile_start[gi + 1]) ++gi;
  const TmGroup& G = L.g[gi];
  const int tiles_n = (G.N + LBN - 1) / LBN, tiles_m = (G.M + LBM - 1) / LBM;
  const int sm = tiles_n >= kSuper ? 1 : kSuper / tiles_n;       // tile rows per super-tile
  if (within >= sm * tiles_n) return;
  const int tm = (gs - L.tile_start[gi]) * sm + within / tiles_n, tn = within % tiles_n;
  if (tm >= tiles_m) return;
  const int m0 = tm * LBM, n0 = tn * LBN;
  const int kshift = DOTS ? G.K0 : 0;              // operand columns in front of A's own
  const int M = G.M, N = G.N, K1 = G.K1, K = G.K1 + kshift;
  const uint16_t* __restrict__ A = (const uint16_t*)G.A1;
  const uint16_t* __restrict__ W = (const uint16_t*)G.W;
  const int lda = G.lda1, ldw = G.ldw;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 2, wn = wave & 3;        // 2 x 4 waves of 128 x 64
  const int srow = tid >> 3, scol = (tid & 7) * 8;

  floatx16 acc[4][2];
#pragma clang loop unroll(full)
  for (int i = 0; i < 4; ++i)
#pragma clang loop unroll(full)
    for (int j = 0; j < 2; ++j)
#pragma clang loop unroll(full)
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // element offsets of this thread's 4 + 4 chunks at k = 0 (rows past the edge are clamped
  // to the last row and zeroed on the way to LDS)
  uint32_t offa[4], offb[4];
  uint32_t oka = 0, okb = 0;
#pragma clang loop unroll(full)
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + srow + i * 64, n = n0 + srow + i * 64;
    offa[i] = (uint32_t)min(m, M - 1) * (uint32_t)lda + scol;
    offb[i] = (uint32_t)min(n, N - 1) * (uint32_t)ldw + scol;
    oka |= (m < M ? 1u : 0u) << i;
    okb |= (n < N ? 1u : 0u) << i;
  }

  uint4 ra[4], rb[4];
  // Loads are never predicated (edge rows are clamped to a valid row, a K tail to column 0),
  // so they stay in flight across the multiply; edge tiles zero what they must not use when
  // the registers are written to LDS.
  const bool interior = !DOTS && m0 + LBM <= M && n0 + LBN <= N && K % BK == 0;
  auto load_tile = [&](int kt) __attribute__((always_inline)) {
    const int kw = (kt * BK + scol < K) ? kt * BK : -scol;          // W column block
    int ka = kt * BK - kshift;                                       // A column block
    if (ka + scol < 0 || ka + scol >= K1) ka = -scol;
#pragma clang loop unroll(full)
    for (int i = 0; i < 4; ++i) {
      ra[i] = *(const uint4*)(A + offa[i] + ka);
      rb[i] = *(const uint4*)(W + offb[i] + kw);
    }
  };
  auto store_tile = [&](int stage, int kt) __attribute__((always_inline)) {
    uint16_t* As = lds + stage * 2 * kBigTileElems;
    uint16_t* Bs = As + kBigTileElems;
    const int ca = kt * BK + scol - kshift;                          // this thread's A column
    if (!interior) {
      const bool kin = kt * BK + scol < K, ain = ca >= 0 && ca < K1;
#pragma clang loop unroll(full)
      for (int i = 0; i < 4; ++i) {
        if (!(ain && ((oka >> i) & 1))) ra[i] = make_uint4(0, 0, 0, 0);
        if (!(kin && ((okb >> i) & 1))) rb[i] = make_uint4(0, 0, 0, 0);
      }
    }
#pragma clang loop unroll(full)
    for (int i = 0; i < 4; ++i) {
      *(uint4*)(As + (srow + i * 64) * kLdsStride + scol) = ra[i];
      *(uint4*)(Bs + (srow + i * 64) * kLdsStride + scol) = rb[i];
    }
  };

  const int nk = (K + BK - 1) / BK;
  load_tile(0);
  store_tile(0, 0);
  if (nk > 1) load_tile(1);
  if constexpr (DOTS) {
    // pairwise dots of this block's 256 samples, written over the zeros the first tile store
    // left in the operand's leading columns: 32 consecutive (sample, feature) rows are one
    // 32 x 32 Gram tile; eight waves share the 256 * nf / 32 row groups
    __syncthreads();
    const int nf = G.nf, fd = G.fdim;
    const int64_t nrows = (int64_t)M * nf;
    const int ngroups = LBM * nf / 32;
    for (int rg = wave; rg < ngroups; rg += kBigThreads / 64) {
      const int64_t r = (int64_t)m0 * nf + rg * 32 + (lane & 31);
      const uint16_t* xp = A + r * fd + (lane >> 5) * 8;
      floatx16 d;
#pragma clang loop unroll(full)
      for (int v = 0; v < 16; ++v) d[v] = 0.f;
      const uint16_t* xq = r < nrows ? xp : A + (lane >> 5) * 8;   // rows past the edge: row 0, zeroed
      for (int k = 0; k < fd; k += 64) {
        uint4 a[4];
#pragma clang loop unroll(full)
        for (int u = 0; u < 4; ++u) a[u] = *(const uint4*)(xq + (k + u * 16 < fd ? k + u * 16 : 0));
#pragma clang loop unroll(full)
        for (int u = 0; u < 4; ++u) {
          if (!(r < nrows && k + u * 16 < fd)) a[u] = make_uint4(0, 0, 0, 0);
          d = mfma32<DT>(a[u], a[u], d);
        }
      }
      const int c = lane & 31, sc = c / nf, j = c % nf;
      const int s_local = rg * 32 / nf + sc;
#pragma clang loop unroll(full)
      for (int v = 0; v < 16; ++v) {
        const int rr = (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
        const int i = rr % nf;
        if (rr / nf == sc && i < j)
          store_elt<DT>(lds, s_local * kLdsStride + (i * (2 * nf - i - 1) / 2 + (j - i - 1)), d[v]);
      }
    }
  }
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) store_tile(cur ^ 1, kt + 1);
    if (kt + 2 < nk) load_tile(kt + 2);
    const uint16_t* ap = lds + cur * 2 * kBigTileElems + (wm * 128 + (lane & 31)) * kLdsStride +
                         (lane >> 5) * 8;
    const uint16_t* bp = lds + cur * 2 * kBigTileElems + kBigTileElems +
                         (wn * 64 + (lane & 31)) * kLdsStride + (lane >> 5) * 8;
#pragma clang loop unroll(full)
    for (int kk = 0; kk < BK / 16; ++kk) {
      uint4 a[4], b[2];
#pragma clang loop unroll(full)
      for (int i = 0; i < 4; ++i) a[i] = *(const uint4*)(ap + i * 32 * kLdsStride + kk * 16);
#pragma clang loop unroll(full)
      for (int j = 0; j < 2; ++j) b[j] = *(const uint4*)(bp + j * 32 * kLdsStride + kk * 16);
#pragma clang loop unroll(full)
      for (int i = 0; i < 4; ++i)
#pragma clang loop unroll(full)
        for (int j = 0; j < 2; ++j) acc[i][j] = mfma32<DT>(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }

  // Epilogue through LDS, one 128-row half of the tile at a time: the waves that own the half
  // park their float32 accumulators (a lane holds one column of 16 rows: poor for global
  // memory), then all 512 threads walk the half in 8-column pieces, so bias, x0, x_l and the
  // output move as 16-byte accesses.
  const int epi = G.epi;
  float* stage = (float*)lds;
  constexpr int kStageStride = LBN + 8;            // 4*stride % 64 == 32: conflict-free parking
  const bool vec_ok =
      G.ldc % 8 == 0 && n0 + LBN <= N && (((uintptr_t)G.C | (uintptr_t)G.bias) & 15) == 0 &&
      (epi != EPI_CROSS ||
       (G.ldx % 8 == 0 && lda % 8 == 0 && (((uintptr_t)G.X0 | (uintptr_t)G.A1) & 15) == 0));
#pragma clang loop unroll(full)
  for (int h = 0; h < 2; ++h) {
    if (wm == h) {
#pragma clang loop unroll(full)
      for (int j = 0; j < 2; ++j)
#pragma clang loop unroll(full)
        for (int i = 0; i < 4; ++i)
#pragma clang loop unroll(full)
          for (int v = 0; v < 16; ++v) {
            const int r = i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
            stage[r * kStageStride + wn * 64 + j * 32 + (lane & 31)] = acc[i][j][v];
          }
    }
    __syncthreads();
    for (int c = tid; c < 128 * (LBN / 8); c += kBigThreads) {
      const int r = c / (LBN / 8), cc = (c % (LBN / 8)) * 8;
      const int m = m0 + h * 128 + r, n = n0 + cc;
      if (m >= M || n >= N) continue;
      float y[8];
      const float4 s0 = *(const float4*)(stage + r * kStageStride + cc);
      const float4 s1 = *(const float4*)(stage + r * kStageStride + cc + 4);
      y[0] = s0.x; y[1] = s0.y; y[2] = s0.z; y[3] = s0.w;
      y[4] = s1.x; y[5] = s1.y; y[6] = s1.z; y[7] = s1.w;
      if (vec_ok) {
        float bv[8], xv[8], lv[8];
        dmt::decode_chunk<DT>(bv, *(const uint4*)((const uint16_t*)G.bias + n));
#pragma clang loop unroll(full)
        for (int q = 0; q < 8; ++q) y[q] += bv[q];
        if (epi == EPI_BIAS_RELU) {
#pragma clang loop unroll(full)
          for (int q = 0; q < 8; ++q) y[q] = y[q] > 0.f ? y[q] : 0.f;
        }
        if (epi == EPI_CROSS) {
          dmt::decode_chunk<DT>(xv, *(const uint4*)((const uint16_t*)G.X0 + (int64_t)m * G.ldx + n));
          dmt::decode_chunk<DT>(lv, *(const uint4*)(A + (int64_t)m * lda + n));
#pragma clang loop unroll(full)
          for (int q = 0; q < 8; ++q) y[q] = xv[q] * y[q] + lv[q];
        }
        dmt::store_chunk<DT, 8>(G.C, (int64_t)m * G.ldc + n, y);
      } else {
        for (int q = 0; q < 8 && n + q < N; ++q) {
          float z = y[q] + load_elt<DT>(G.bias, n + q);
          if (epi == EPI_BIAS_RELU) z = z > 0.f ? z : 0.f;
          if (epi == EPI_CROSS)
            z = load_elt<DT>(G.X0, (int64_t)m * G.ldx + n + q) * z +
                load_elt<DT>(G.A1, (int64_t)m * lda + n + q);
          store_elt<DT>(G.C, (int64_t)m * G.ldc + n + q, z);
        }
      }
    }
    __syncthreads();
  }
}

// --------------------------------------------------- plain FMA GEMM (float32)

template <int DT>
__global__ __launch_bounds__(kBlock) void tm_gemm_simple(const TmLaunch L) {
  int gi = 0;
  while (gi + 1 < L.ngroups && (int)blockIdx.x >= L.tile_start[gi + 1]) ++gi;
  const TmGroup& G = L.g[gi];
  const int64_t e = (int64_t)(blockIdx.x - L.tile_start[gi]) * kBlock + threadIdx.x;
  if (e >= (int64_t)G.M * G.N) return;
  const int m = (int)(e / G.N), n = (int)(e % G.N);
  float s = 0.f;
  for (int k = 0; k < G.K0; ++k)
    s += load_elt<DT>(G.A0, (int64_t)m * G.lda0 + k) * load_elt<DT>(G.W, (int64_t)n * G.ldw + k);
  for (int k = 0; k < G.K1; ++k)
    s += load_elt<DT>(G.A1, (int64_t)m * G.lda1 + k) *
         load_elt<DT>(G.W, (int64_t)n * G.ldw + G.K0 + k);
  float y = s + load_elt<DT>(G.bias, n);
  if (G.epi == EPI_BIAS_RELU) y = y > 0.f ? y : 0.f;
  if (G.epi == EPI_CROSS)
    y = load_elt<DT>(G.X0, (int64_t)m * G.ldx + n) * y + load_elt<DT>(G.A1, (int64_t)m * G.lda1 + n);
  store_elt<DT>(G.C, (int64_t)m * G.ldc + n, y);
}

// ------------------------------------------------------------ pairwise dot terms

// Per-tower work of a grouped auxiliary launch (dot terms or weight repack).
struct TmAuxItem {
  const void* src;
  void* dst;
  int32_t nf, n, np, np_pad;   // dots: features, dim, real and padded term count
  int32_t O, wt;               // pack: output rows, tower width
};

struct TmAuxLaunch {
  int32_t ngroups;
  int32_t block_start[kMaxGroups + 1];
  int64_t B;
  TmAuxItem g[kMaxGroups];
};

__device__ __forceinline__ int aux_group(const TmAuxLaunch& L) {
  int gi = 0;
  while (gi + 1 < L.ngroups && (int)blockIdx.x >= L.block_start[gi + 1]) ++gi;
  return gi;
}

// z[s][p(i,j)] = <x[s][i][:], x[s][j][:]>, i < j, p row-major; x is [B][nf][n]
// contiguous.  One wave per 32 consecutive (sample, feature) rows; needs
// 32 % nf == 0 and n % 16 == 0.  Columns np .. np_pad-1 of z are zeroed.
template <int DT>
__global__ __launch_bounds__(kBlock) void tm_dots_mfma(const TmAuxLaunch L) {
  const int gi = aux_group(L);
  const TmAuxItem& G = L.g[gi];
  const int64_t B = L.B;
  const int nf = G.nf, n = G.n, np = G.np, np_pad = G.np_pad;
  void* __restrict__ z = G.dst;
  const int lane = threadIdx.x & 63;
  const int64_t rg = (int64_t)(blockIdx.x - L.block_start[gi]) * (kBlock / 64) + (threadIdx.x >> 6);
  const int64_t row0 = rg * 32, nrows = B * nf;
  if (row0 >= nrows) return;
  const int64_t r = row0 + (lane & 31);
  const uint16_t* xp = (const uint16_t*)G.src + r * n + (lane >> 5) * 8;
  floatx16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  for (int k = 0; k < n; k += 16) {
    uint4 a = make_uint4(0, 0, 0, 0);
    if (r < nrows) a = *(const uint4*)(xp + k);
    acc = mfma32<DT>(a, a, acc);
  }
  const int spg = 32 / nf;                       // samples per row group
  const int64_t s0 = row0 / nf;
  const int c = lane & 31, sc = c / nf, j = c % nf;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int rr = (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
    const int i = rr % nf;
    if (rr / nf == sc && i < j && s0 + sc < B)
      store_elt<DT>(z, (s0 + sc) * np_pad + (i * (2 * nf - i - 1) / 2 + (j - i - 1)), acc[v]);
  }
  const int npad = np_pad - np;
  if (lane < spg * npad) {
    const int s = lane / npad, q = lane % npad;
    if (s0 + s < B) store_elt<DT>(z, (s0 + s) * np_pad + np + q, 0.f);
  }
}

// Any nf / n, any dtype: one thread per (sample, term).
template <int DT>
__global__ __launch_bounds__(kBlock) void tm_dots_simple(const TmAuxLaunch L) {
  const int gi = aux_group(L);
  const TmAuxItem& G = L.g[gi];
  const int nf = G.nf, n = G.n, np = G.np, np_pad = G.np_pad;
  const int64_t e = (int64_t)(blockIdx.x - L.block_start[gi]) * kBlock + threadIdx.x;
  if (e >= L.B * np_pad) return;
  const int64_t s = e / np_pad;
  const int p = (int)(e % np_pad);
  float d = 0.f;
  if (p < np) {
    int i = 0, rem = p;
    while (rem >= nf - 1 - i) { rem -= nf - 1 - i; ++i; }
    const int j = i + 1 + rem;
    const int64_t bi = (s * nf + i) * n, bj = (s * nf + j) * n;
    for (int k = 0; k < n; ++k) d += load_elt<DT>(G.src, bi + k) * load_elt<DT>(G.src, bj + k);
  }
  store_elt<DT>(G.dst, e, d);
}

// Projection weights [O][np + Wt] -> [O][np_pad + Wt] with zero columns after the
// dot terms, so both K segments start 16-byte aligned.
template <int DT>
__global__ __launch_bounds__(kBlock) void tm_pack_w(const TmAuxLaunch L) {
  const int gi = aux_group(L);
  const TmAuxItem& G = L.g[gi];
  const int np = G.np, np_pad = G.np_pad, wt = G.wt;
  const int64_t e = (int64_t)(blockIdx.x - L.block_start[gi]) * kBlock + threadIdx.x;
  const int kp = np_pad + wt;
  if (e >= (int64_t)G.O * kp) return;
  const int o = (int)(e / kp), k = (int)(e % kp);
  const int64_t src = (int64_t)o * (np + wt) + (k < np ? k : np + (k - np_pad));
  if constexpr (DT == DMT_F32) {
    ((float*)G.dst)[e] = (k >= np && k < np_pad) ? 0.f : ((const float*)G.src)[src];
  } else {
    ((uint16_t*)G.dst)[e] = (k >= np && k < np_pad) ? (uint16_t)0 : ((const uint16_t*)G.src)[src];
  }
}

// ----------------------------------------------------------------- host side

struct TowerWs {
  size_t z_off = 0, wp_off = 0, x_off[2] = {0, 0};
  int np = 0, np_pad = 0;
};

// Validates the towers' parameters and lays out the scratch.  Returns total bytes
// through *bytes.
dmt_status plan_tm(const dmt_plan* p, const dmt_tm_params* tp, int64_t B, int eb,
                   std::vector<TowerWs>* ws, size_t* bytes) {
  size_t off = 0;
  auto take = [&](size_t b) { size_t o = off; off = dmt_align_up(off + b, 256); return o; };
  ws->assign(p->T, TowerWs());
  for (int32_t t = 0; t < p->T; ++t) {
    const dmt_tm_params& q = tp[t];
    const int64_t wt = p->tower_width[t];
    if (q.out_dim <= 0 || !q.w_proj || !q.b_proj) return DMT_EINVAL;
    if (((uintptr_t)q.w_proj & 15) && q.kind != DMT_TM_DOT_LINEAR) return DMT_EINVAL;
    TowerWs& w = (*ws)[t];
    switch (q.kind) {
      case DMT_TM_LINEAR:
      case DMT_TM_LINEAR_RELU:
        break;
      case DMT_TM_DOT_LINEAR: {
        const int nf = p->tower_ntab[t];
        if (p->tower_uniform_dim[t] == 0) return DMT_ENOTSUP;   // dots need one common dim
        w.np = nf * (nf - 1) / 2;
        w.np_pad = (w.np + 7) / 8 * 8;
        w.z_off = take((size_t)B * w.np_pad * eb);
        w.wp_off = take((size_t)q.out_dim * (w.np_pad + wt) * eb);
        break;
      }
      case DMT_TM_CROSS_LINEAR:
        if (q.num_cross_layers < 1 || q.num_cross_layers > DMT_MAX_CROSS_LAYERS) return DMT_EINVAL;
        for (int l = 0; l < q.num_cross_layers; ++l)
          if (!q.w_cross[l] || !q.b_cross[l] || ((uintptr_t)q.w_cross[l] & 15)) return DMT_EINVAL;
        w.x_off[0] = take((size_t)B * wt * eb);
        if (q.num_cross_layers > 1) w.x_off[1] = take((size_t)B * wt * eb);
        break;
      default:
        return DMT_EINVAL;
    }
  }
  *bytes = off;
  return DMT_OK;
}

// Whether a group can go to the 256 x 256 kernel (dots: with in-kernel dot terms).
inline bool big_ok(const TmGroup& g, bool dots) {
  return g.N > 128 && g.N <= kSuper * LBN && g.K1 >= 128 && (dots || g.K0 == 0) &&
         (int64_t)g.M * g.lda1 < (1LL << 31) && (int64_t)g.N * g.ldw < (1LL << 31);
}

template <int DT>
void launch_groups(const dmt_plan* p, std::vector<TmGroup>& groups, hipStream_t s,
                   bool dots = false) {
  for (size_t first = 0; first < groups.size(); first += kMaxGroups) {
    TmLaunch L;
    L.ngroups = (int32_t)std::min<size_t>(kMaxGroups, groups.size() - first);
    int32_t tiles = 0;
    for (int i = 0; i < L.ngroups; ++i) {
      const TmGroup& g = groups[first + i];
      L.g[i] = g;
      L.tile_start[i] = tiles;
      if constexpr (DT == DMT_F32)
        tiles += (int32_t)(((int64_t)g.M * g.N + kBlock - 1) / kBlock);
      else
        tiles += ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
    }
    L.tile_start[L.ngroups] = tiles;
    if (tiles == 0) continue;
    if constexpr (DT == DMT_F32) {
      DmtScope sc_(p, DMT_K_TM_GEMM, s);
      hipLaunchKernelGGL((tm_gemm_simple<DT>), dim3(tiles), dim3(kBlock), 0, s, L);
    } else {
      // wide outputs take the 256 x 256 kernel
      bool big = dots || dmt::env_int("DMT_TM_BIG", 1) != 0;
      for (int i = 0; i < L.ngroups; ++i) big = big && big_ok(L.g[i], dots);
      if (big) {
        static bool configured = false;
        if (!configured) {
          (void)hipFuncSetAttribute((const void*)tm_gemm_mfma_256<DT, false>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kBigLdsBytes);
          (void)hipFuncSetAttribute((const void*)tm_gemm_mfma_256<DT, true>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kBigLdsBytes);
          configured = true;
        }
        int32_t nst = 0;                                      // super-tiles of the launch
        for (int i = 0; i < L.ngroups; ++i) {
          L.tile_start[i] = nst;
          const int tn = (L.g[i].N + LBN - 1) / LBN, tm = (L.g[i].M + LBM - 1) / LBM;
          const int sm = tn >= kSuper ? 1 : kSuper / tn;
          nst += (tm + sm - 1) / sm;
        }
        L.tile_start[L.ngroups] = nst;
        const int32_t big_tiles = (nst + 7) / 8 * 8 * kSuper;
        DmtScope sc_(p, DMT_K_TM_GEMM, s);
        if (dots)
          hipLaunchKernelGGL((tm_gemm_mfma_256<DT, true>), dim3(big_tiles), dim3(kBigThreads),
                             kBigLdsBytes, s, L);
        else
          hipLaunchKernelGGL((tm_gemm_mfma_256<DT, false>), dim3(big_tiles), dim3(kBigThreads),
                             kBigLdsBytes, s, L);
      } else {
        DmtScope sc_(p, DMT_K_TM_GEMM, s);
        hipLaunchKernelGGL((tm_gemm_mfma<DT>), dim3(tiles), dim3(kBlock), 0, s, L);
      }
    }
  }
  groups.clear();
}

template <int DT>
dmt_status run_tm(const dmt_plan* p, const dmt_tm_params* tp, const std::vector<TowerWs>& ws,
                  const void* pooled, int64_t B, void* tm_out, char* wsp, hipStream_t s) {
  constexpr int eb = DT == DMT_F32 ? 4 : 2;
  const char* x_all = (const char*)pooled;
  char* y_all = (char*)tm_out;
  std::vector<int64_t> out_prefix(p->T + 1, 0);
  for (int32_t t = 0; t < p->T; ++t) out_prefix[t + 1] = out_prefix[t] + tp[t].out_dim;
  int max_layers = 0;

  // A dot-product tower whose shape fits computes its dot terms inside the projection GEMM.
  std::vector<char> fused(p->T, 0);
  if (DT != DMT_F32 && dmt::env_int("DMT_TM_FUSE", 1) != 0 && dmt::env_int("DMT_TM_BIG", 1) != 0)
    for (int32_t t = 0; t < p->T; ++t) {
      const dmt_tm_params& q = tp[t];
      if (q.kind != DMT_TM_DOT_LINEAR) continue;
      const int nf = p->tower_ntab[t], n = p->tower_uniform_dim[t], wt = p->tower_width[t];
      TmGroup g{};
      g.M = (int32_t)B; g.N = q.out_dim; g.K1 = wt; g.lda1 = wt; g.ldw = ws[t].np_pad + wt;
      fused[t] = nf >= 2 && 32 % nf == 0 && n % 16 == 0 && ws[t].np_pad <= BK && big_ok(g, true);
    }

  // stage 0: dot terms and repacked projection weights, one grouped launch per kind
  std::vector<TmAuxItem> dots_mfma, dots_simple, packs;
  std::vector<int64_t> nb_mfma, nb_simple, nb_pack;
  for (int32_t t = 0; t < p->T; ++t) {
    const dmt_tm_params& q = tp[t];
    if (q.kind == DMT_TM_CROSS_LINEAR) max_layers = std::max(max_layers, q.num_cross_layers);
    if (q.kind != DMT_TM_DOT_LINEAR) continue;
    const TowerWs& w = ws[t];
    TmAuxItem it{};
    it.nf = p->tower_ntab[t]; it.n = p->tower_uniform_dim[t]; it.np = w.np; it.np_pad = w.np_pad;
    it.O = q.out_dim; it.wt = p->tower_width[t];
    it.src = x_all + (size_t)B * p->width_prefix[t] * eb;
    it.dst = wsp + w.z_off;
    if (fused[t]) {
    } else if (DT != DMT_F32 && 32 % it.nf == 0 && it.n % 16 == 0) {
      dots_mfma.push_back(it);
      nb_mfma.push_back(((B * it.nf + 31) / 32 + 3) / 4);
    } else {
      dots_simple.push_back(it);
      nb_simple.push_back((B * w.np_pad + kBlock - 1) / kBlock);
    }
    it.src = q.w_proj;
    it.dst = wsp + w.wp_off;
    packs.push_back(it);
    nb_pack.push_back(((int64_t)q.out_dim * (w.np_pad + it.wt) + kBlock - 1) / kBlock);
  }
  auto launch_aux = [&](std::vector<TmAuxItem>& items, std::vector<int64_t>& nblocks, int which) {
    for (size_t first = 0; first < items.size(); first += kMaxGroups) {
      TmAuxLaunch L;
      L.B = B;
      L.ngroups = (int32_t)std::min<size_t>(kMaxGroups, items.size() - first);
      int32_t blocks = 0;
      for (int i = 0; i < L.ngroups; ++i) {
        L.g[i] = items[first + i];
        L.block_start[i] = blocks;
        blocks += (int32_t)nblocks[first + i];
      }
      L.block_start[L.ngroups] = blocks;
      if (blocks == 0) continue;
      if (which == 0) {
        if constexpr (DT != DMT_F32) {
          DmtScope sc_(p, DMT_K_TM_DOTS, s);
          hipLaunchKernelGGL((tm_dots_mfma<DT>), dim3(blocks), dim3(kBlock), 0, s, L);
        }
      } else if (which == 1) {
        DmtScope sc_(p, DMT_K_TM_DOTS, s);
        hipLaunchKernelGGL((tm_dots_simple<DT>), dim3(blocks), dim3(kBlock), 0, s, L);
      } else {
        DmtScope sc_(p, DMT_K_TM_PACK, s);
        hipLaunchKernelGGL((tm_pack_w<DT>), dim3(blocks), dim3(kBlock), 0, s, L);
      }
    }
  };
  launch_aux(dots_mfma, nb_mfma, 0);
  launch_aux(dots_simple, nb_simple, 1);
  launch_aux(packs, nb_pack, 2);

  // cross layers, one grouped launch per layer index
  std::vector<TmGroup> groups;
  for (int l = 0; l < max_layers; ++l) {
    for (int32_t t = 0; t < p->T; ++t) {
      const dmt_tm_params& q = tp[t];
      if (q.kind != DMT_TM_CROSS_LINEAR || l >= q.num_cross_layers) continue;
      const int wt = p->tower_width[t];
      const void* x0 = x_all + (size_t)B * p->width_prefix[t] * eb;
      TmGroup g{};
      g.A0 = nullptr; g.lda0 = 0; g.K0 = 0;
      g.A1 = l == 0 ? x0 : (const void*)(wsp + ws[t].x_off[(l - 1) & 1]);
      g.lda1 = wt; g.K1 = wt;
      g.W = q.w_cross[l]; g.ldw = wt; g.bias = q.b_cross[l];
      g.X0 = x0; g.ldx = wt;
      g.C = wsp + ws[t].x_off[l & 1]; g.ldc = wt;
      g.M = (int32_t)B; g.N = wt; g.epi = EPI_CROSS;
      groups.push_back(g);
    }
    launch_groups<DT>(p, groups, s);
  }

  // projections of every tower
  std::vector<TmGroup> groups_fused;
  for (int32_t t = 0; t < p->T; ++t) {
    const dmt_tm_params& q = tp[t];
    const int wt = p->tower_width[t];
    const void* x = x_all + (size_t)B * p->width_prefix[t] * eb;
    TmGroup g{};
    g.A0 = nullptr; g.lda0 = 0; g.K0 = 0;
    g.A1 = x; g.lda1 = wt; g.K1 = wt;
    g.W = q.w_proj; g.ldw = wt;
    if (q.kind == DMT_TM_DOT_LINEAR) {
      g.A0 = wsp + ws[t].z_off; g.lda0 = ws[t].np_pad; g.K0 = ws[t].np_pad;
      g.W = wsp + ws[t].wp_off; g.ldw = ws[t].np_pad + wt;
    } else if (q.kind == DMT_TM_CROSS_LINEAR) {
      g.A1 = wsp + ws[t].x_off[(q.num_cross_layers - 1) & 1];
    }
    g.bias = q.b_proj;
    g.X0 = nullptr; g.ldx = 0;
    g.C = y_all + (size_t)B * out_prefix[t] * eb; g.ldc = q.out_dim;
    g.M = (int32_t)B; g.N = q.out_dim;
    g.epi = q.kind == DMT_TM_LINEAR_RELU ? EPI_BIAS_RELU : EPI_BIAS;
    if (fused[t]) {
      g.A0 = nullptr; g.lda0 = 0;
      g.nf = p->tower_ntab[t]; g.fdim = p->tower_uniform_dim[t];
      groups_fused.push_back(g);
    } else {
      groups.push_back(g);
    }
  }
  launch_groups<DT>(p, groups, s);
  if constexpr (DT != DMT_F32) launch_groups<DT>(p, groups_fused, s, true);
  return hipGetLastError() == hipSuccess ? DMT_OK : DMT_EHIP;
}

}  // namespace

extern "C" size_t dmt_tm_workspace_bytes(const dmt_plan* plan, const dmt_tm_params* per_tower,
                                         int64_t B) {
  if (!plan || !per_tower || B <= 0) return 0;
  std::vector<TowerWs> ws;
  size_t bytes = 0;
  // sized for the wider element type so one figure serves every dtype
  if (plan_tm(plan, per_tower, B, 4, &ws, &bytes) != DMT_OK) return 0;
  return bytes;
}

extern "C" dmt_status dmt_tower_module_fwd(const dmt_plan* plan, const dmt_tm_params* per_tower,
                                           const void* pooled, int64_t B, void* tm_out,
                                           dmt_dtype dtype, void* workspace,
                                           size_t workspace_bytes, void* stream) {
  if (!plan || !per_tower || !pooled || !tm_out) return DMT_EINVAL;
  if (B <= 0 || B > plan->max_batch || B >= (1LL << 31)) return DMT_EINVAL;
  if (dtype != DMT_F32 && dtype != DMT_F16 && dtype != DMT_BF16) return DMT_EINVAL;
  if (((uintptr_t)pooled & 15) || ((uintptr_t)tm_out & 15)) return DMT_EINVAL;
  const int eb = dmt_elt_bytes(dtype);
  for (int32_t t = 0; t < plan->T; ++t)
    if (plan->tower_width[t] % 8 != 0 && dtype != DMT_F32) return DMT_ENOTSUP;
  std::vector<TowerWs> ws;
  size_t bytes = 0;
  dmt_status st = plan_tm(plan, per_tower, B, eb, &ws, &bytes);
  if (st != DMT_OK) return st;
  if (bytes > 0) {
    if (!workspace || ((uintptr_t)workspace & 255)) return DMT_EINVAL;
    if (workspace_bytes < bytes) return DMT_ENOMEM;
  }
  hipStream_t s = (hipStream_t)stream;
  char* wsp = (char*)workspace;
  switch (dtype) {
    case DMT_F32: return run_tm<DMT_F32>(plan, per_tower, ws, pooled, B, tm_out, wsp, s);
    case DMT_F16: return run_tm<DMT_F16>(plan, per_tower, ws, pooled, B, tm_out, wsp, s);
    default: return run_tm<DMT_BF16>(plan, per_tower, ws, pooled, B, tm_out, wsp, s);
  }
}
