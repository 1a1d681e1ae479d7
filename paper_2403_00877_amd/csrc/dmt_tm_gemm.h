// Grouped contractions of the Tower Module, shared by its forward and backward:
//   C = epilogue(A . W^T [+ b])  with both operands contiguous along the reduction
// dimension, one launch for all towers of a stage (block id -> tower, tile).
// 16-bit types run on MFMA (v_mfma_f32_32x32x16, float32 accumulate) in two tilings
// (128 x 128 x 64 with four waves, 256 x 256 x 64 with eight); float32 uses a plain
// FMA kernel.  Also the pairwise-dot (Gram tile) kernels and the projection-weight
// repack of the dot-product form.  Everything lives in an unnamed namespace: each
// translation unit that includes this header gets its own copy.
#pragma once
#include <algorithm>
#include <vector>

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

// EPI_F32 / EPI_F32_ADD: C is float32 whatever the operand type, no bias: C = acc / C += acc
// (gradients: the backward's accumulations stay in float32)
enum { EPI_BIAS = 0, EPI_BIAS_RELU = 1, EPI_CROSS = 2, EPI_F32 = 3, EPI_F32_ADD = 4 };

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
  // Split K (EPI_F32 with K0 = 0 only): ksplit > 1 cuts the K1 columns into slices of klen
  // (a multiple of 8); slice s is a contraction of its own whose result goes to
  // C + s * cstride floats, and the caller adds the slices up in a fixed order.
  int32_t ksplit, klen;
  int64_t cstride;
  // Two-level output rows (128 x 128 and plain kernels only): with rdiv > 0 row m of C starts at
  // (m / rdiv) * ldc + (m % rdiv) * ldc2, i.e. rdiv consecutive rows of the contraction share
  // one row of the output tensor.
  int32_t rdiv, ldc2;
  // EPI_CROSS: when set, u = acc + bias (before the cross product) is also stored here, laid
  // out like C (what the backward needs of a cross layer).  A group whose dot terms are computed
  // in-kernel: when set, they are also stored here as [M][K0], zeros in the padding columns.
  void* U;
  // EPI_CROSS: the x_l term, [M][ldxl]; NULL when it is the operand A1 itself (a full-rank
  // layer).  A low-rank layer contracts t = V x_l instead, and adds x_l from here.
  const void* XL;
  int32_t ldxl;
};

// bias may be NULL (no bias)
__device__ __forceinline__ const void* tm_xl(const TmGroup& g) { return g.XL ? g.XL : g.A1; }
__device__ __forceinline__ int tm_ldxl(const TmGroup& g) { return g.XL ? g.ldxl : g.lda1; }

__device__ __forceinline__ int64_t tm_crow(const TmGroup& g, int m) {
  return g.rdiv > 0 ? (int64_t)(m / g.rdiv) * g.ldc + (int64_t)(m % g.rdiv) * g.ldc2
                    : (int64_t)m * g.ldc;
}

__host__ __device__ inline int tm_slices(const TmGroup& g) { return g.ksplit > 1 ? g.ksplit : 1; }

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

// TAG (here and below) only marks the including source file in the kernel's name, so that a
// profile tells the forward's launches from the backward's.
#ifndef DMT_TM_TAG
#define DMT_TM_TAG 0
#endif

// KEEPU: the cross epilogue also stores u (TmGroup::U), in a pass of its own over the
// accumulators: a second store inside the fully unrolled epilogue cost the bf16 kernel 40
// registers and made it spill.
template <int DT, bool KEEPU = false, int TAG = DMT_TM_TAG>
__global__ __launch_bounds__(kBlock, 2) void tm_gemm_mfma(const TmLaunch L) {
  __shared__ __attribute__((aligned(16))) uint16_t As[BM * kLdsStride];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[BN * kLdsStride];
  int gi = 0;
  while (gi + 1 < L.ngroups && (int)blockIdx.x >= L.tile_start[gi + 1]) ++gi;
  const TmGroup& G = L.g[gi];
  int tile = blockIdx.x - L.tile_start[gi];
  const int tiles_n = (G.N + BN - 1) / BN;
  const int tiles_mn = ((G.M + BM - 1) / BM) * tiles_n;
  const int slice = tile / tiles_mn;                 // 0 unless K is split
  tile -= slice * tiles_mn;
  const int kofs = G.ksplit > 1 ? slice * G.klen : 0;
  const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;
  const int M = G.M, N = G.N, K0 = G.K0;
  const int K = G.K0 + (G.ksplit > 1 ? min(G.klen, G.K1 - kofs) : G.K1);
  const uint16_t* A0 = (const uint16_t*)G.A0;
  const uint16_t* A1 = (const uint16_t*)G.A1 + kofs;
  const uint16_t* W = (const uint16_t*)G.W + kofs;
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
  if constexpr (KEEPU) {
    if (epi == EPI_CROSS && G.U) {
      for (int j = 0; j < 2; ++j) {
        const int n = n0 + wn * 64 + j * 32 + (lane & 31);
        if (n >= N) continue;
        const float bias = G.bias ? load_elt<DT>(G.bias, n) : 0.f;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int m = m0 + wm * 64 + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
            if (m < M) store_elt<DT>(G.U, (int64_t)m * G.ldc + n, acc[i][j][v] + bias);
          }
        }
      }
    }
  }
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int n = n0 + wn * 64 + j * 32 + (lane & 31);
    if (n >= N) continue;
    const float bias = (epi >= EPI_F32 || !G.bias) ? 0.f : load_elt<DT>(G.bias, n);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = m0 + wm * 64 + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
        if (m >= M) continue;
        if (epi >= EPI_F32) {
          float* c = (float*)G.C + slice * G.cstride + tm_crow(G, m) + n;
          *c = epi == EPI_F32_ADD ? *c + acc[i][j][v] : acc[i][j][v];
          continue;
        }
        float y = acc[i][j][v] + bias;
        if (epi == EPI_BIAS_RELU) y = y > 0.f ? y : 0.f;
        if (epi == EPI_CROSS) {
          y = load_elt<DT>(G.X0, (int64_t)m * G.ldx + n) * y +
              load_elt<DT>(tm_xl(G), (int64_t)m * tm_ldxl(G) + n);
        }
        store_elt<DT>(G.C, tm_crow(G, m) + n, y);
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
// step suffices.  The MFMAs take the W fragment as their first operand, so the accumulators
// hold the tile transposed: a lane owns one row and four consecutive columns per register
// quad, which the epilogue parks in LDS with 16-byte stores.
constexpr int LBM = 256, LBN = 256;
constexpr int kBigThreads = 512;
constexpr int kSuper = 32;                                  // tiles an XCD keeps resident (its CUs)
constexpr int kBigTileElems = LBM * kLdsStride;            // one operand, one stage
constexpr int kBigLdsBytes = 4 * kBigTileElems * 2;         // 2 stages x (A + B)

// DOTS: the operand's first K0 columns are the tower's pairwise dot terms, which the block
// computes itself (Gram tiles, as in tm_dots_mfma) straight into the first LDS stage, so the
// pooled tensor is read once and the dot terms never exist in global memory.
//
// DIRECT (launches whose tiles are all interior: M and N multiples of 256, K of 64, no dot
// terms): the operand tiles go from global memory straight into LDS (global_load_lds_dwordx4:
// a wave's 64 lanes fill 1 KB of consecutive LDS, 16 bytes a lane), so the K loop has no
// register stage and no LDS stores.  LDS rows are then 128 bytes with no padding; each lane
// fetches the 16-byte column chunk (slot ^ (row / 2) % 8) of its row and the fragment reads
// apply the same exclusive-or.  A ds_read_b128 serves 16 lanes at a time from 64 banks; the
// 16 rows they read then fall on 16 different 16-byte bank groups (rows 2 r and 2 r + 1 lie in
// the two halves of one 256-byte bank row and share a slot, the eight pairs differ in it):
// conflict-free without padding (with slot ^ row % 8, rows r and r + 8 collide and half the
// LDS cycles are conflict cycles).  Tile kt + 2 is requested into the stage tile kt is being
// read from, behind the barrier inside step kt; every wave waits for its own requests before
// the next step's barrier.  (The requests are written as inline assembly: told about them,
// the compiler would make every LDS read of the current tile wait for the next tile's
// requests, since it cannot tell the two stages apart.)
template <int DT, bool DOTS, int TAG = DMT_TM_TAG, bool KEEPZ = false, bool DIRECT = false>
__global__ __launch_bounds__(kBigThreads, 1) void tm_gemm_mfma_256(const TmLaunch L) {
  static_assert(!(DIRECT && DOTS), "in-kernel dot terms are written into a padded first stage");
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
  // a split K multiplies the tile rows: virtual row tmv = slice * tiles_m + tm
  const int tmv = (gs - L.tile_start[gi]) * sm + within / tiles_n, tn = within % tiles_n;
  if (tmv >= tiles_m * tm_slices(G)) return;
  const int slice = tmv / tiles_m, tm = tmv - slice * tiles_m;
  const int kofs = G.ksplit > 1 ? slice * G.klen : 0;
  const int m0 = tm * LBM, n0 = tn * LBN;
  const int kshift = DOTS ? G.K0 : 0;              // operand columns in front of A's own
  const int M = G.M, N = G.N;
  const int K1 = G.ksplit > 1 ? min(G.klen, G.K1 - kofs) : G.K1, K = K1 + kshift;
  const uint16_t* __restrict__ A = (const uint16_t*)G.A1 + kofs;
  const uint16_t* __restrict__ W = (const uint16_t*)G.W + kofs;
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
  if constexpr (DIRECT) {
    constexpr int kStageEl = 2 * LBM * BK;         // one stage: A then W, 128-byte rows
    // instruction j of wave w fills LDS rows (j * 8 + w) * 8 .. + 7 of an operand; lane l holds
    // slot l % 8 of row r = (j * 8 + w) * 8 + l / 8 there and fetches column chunk
    // (l % 8) ^ ((r / 2) % 8) of that row, (r / 2) % 8 being (w % 2) * 4 + l / 16
    const uint32_t lds0 = (uint32_t)(size_t)(__attribute__((address_space(3))) uint16_t*)lds;
    const int chunk = (lane & 7) ^ (((wave & 1) << 2) | (lane >> 4));
    uint32_t va[4], vb[4];                         // byte offsets of this lane's chunks at k = 0
#pragma clang loop unroll(full)
    for (int j = 0; j < 4; ++j) {
      const int r = (j * 8 + wave) * 8 + (lane >> 3);
      va[j] = ((uint32_t)(m0 + r) * (uint32_t)lda + chunk * 8) * 2u;
      vb[j] = ((uint32_t)(n0 + r) * (uint32_t)ldw + chunk * 8) * 2u;
    }
    auto request_tile = [&](int stage, int kt) __attribute__((always_inline)) {
      const uint16_t* ak = A + kt * BK;
      const uint16_t* wk = W + kt * BK;
#pragma clang loop unroll(full)
      for (int j = 0; j < 4; ++j) {
        const uint32_t da = __builtin_amdgcn_readfirstlane(
            lds0 + (uint32_t)(stage * kStageEl * 2 + (j * 8 + wave) * 1024));
        const uint32_t db = da + LBM * BK * 2;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     :: "s"(da), "v"(va[j]), "s"(ak) : "memory");
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     :: "s"(db), "v"(vb[j]), "s"(wk) : "memory");
      }
    };
    // fragment reads: row (lane % 32) of a 32-row block, chunk 2 kk + lane / 32, in slot
    // chunk ^ ((lane % 32) / 2) % 8
    int sw[BK / 16];
#pragma clang loop unroll(full)
    for (int kk = 0; kk < BK / 16; ++kk)
      sw[kk] = (((kk * 2 + (lane >> 5)) ^ ((lane >> 1) & 7)) * 8);
    // Fragments are double-buffered in registers: the six reads of K slice kk + 1 are issued
    // before the eight MFMAs of slice kk, so LDS latency hides behind matrix work of the same
    // wave.  The barrier of a K step sits in front of its last slice's MFMAs: behind it come
    // the requests for tile kt + 2 (every wave has read the whole current stage by then) and
    // the first reads of tile kt + 1, and the last slice's MFMAs cover both.
    uint4 fa[2][4], fb[2][2];
    auto read_frag = [&](int buf, int stage, int kk) __attribute__((always_inline)) {
      const uint16_t* ap = lds + stage * kStageEl + (wm * 128 + (lane & 31)) * BK + sw[kk];
      const uint16_t* bp = lds + stage * kStageEl + LBM * BK + (wn * 64 + (lane & 31)) * BK + sw[kk];
#pragma clang loop unroll(full)
      for (int i = 0; i < 4; ++i) fa[buf][i] = *(const uint4*)(ap + i * 32 * BK);
#pragma clang loop unroll(full)
      for (int j = 0; j < 2; ++j) fb[buf][j] = *(const uint4*)(bp + j * 32 * BK);
    };
    request_tile(0, 0);
    __builtin_amdgcn_s_waitcnt(0x0f70);            // vmcnt(0): this wave's requests have landed
    __syncthreads();
    if (nk > 1) request_tile(1, 1);
    read_frag(0, 0, 0);
    for (int kt = 0; kt < nk; ++kt) {
      const int cur = kt & 1;
#pragma clang loop unroll(full)
      for (int kk = 0; kk < BK / 16; ++kk) {
        if (kk + 1 < BK / 16) {
          read_frag((kk + 1) & 1, cur, kk + 1);
        } else {
          __builtin_amdgcn_s_waitcnt(0x0f70);
          __syncthreads();
          if (kt + 2 < nk) request_tile(cur, kt + 2);
          if (kt + 1 < nk) read_frag(0, cur ^ 1, 0);
        }
#pragma clang loop unroll(full)
        for (int i = 0; i < 4; ++i)
#pragma clang loop unroll(full)
          for (int j = 0; j < 2; ++j) acc[i][j] = mfma32<DT>(fb[kk & 1][j], fa[kk & 1][i], acc[i][j]);
        // one LDS read, one MFMA, ...: left alone, the scheduler puts each read right in front
        // of the MFMA that needs it, to save registers
        if (kk + 1 < BK / 16) {
#pragma clang loop unroll(full)
          for (int q = 0; q < 6; ++q) {
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          }
          __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
        }
      }
    }
  } else {
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
        if (rr / nf == sc && i < j) {
          const int term = i * (2 * nf - i - 1) / 2 + (j - i - 1);
          store_elt<DT>(lds, s_local * kLdsStride + term, d[v]);
          if constexpr (KEEPZ)
            if (G.U && m0 + s_local < M) store_elt<DT>(G.U, (int64_t)(m0 + s_local) * G.K0 + term, d[v]);
        }
      }
      if constexpr (KEEPZ) {
        // zeros behind the terms of the row group's samples
        const int np = nf * (nf - 1) / 2, npad = G.K0 - np, spg = 32 / nf;
        if (G.U)
          for (int e = lane; e < spg * npad; e += 64) {
            const int row = m0 + rg * spg + e / npad;
            if (row < M) store_elt<DT>(G.U, (int64_t)row * G.K0 + np + e % npad, 0.f);
          }
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
        for (int j = 0; j < 2; ++j) acc[i][j] = mfma32<DT>(b[j], a[i], acc[i][j]);
    }
    __syncthreads();
  }
  }
  // Epilogue through LDS, one 128-row half of the tile at a time: the waves that own the half
  // park their float32 accumulators (a lane holds four consecutive columns of one row per
  // register quad: too narrow for global memory), then all 512 threads walk the half in
  // 8-column pieces, so bias, x0, x_l and the output move as 16-byte accesses.
  const int epi = G.epi;
  float* stage = (float*)lds;
  constexpr int kStageStride = LBN + 4;            // rows 4 banks apart: 16 lanes' float4 stores spread over all 64
  const bool vec_ok =
      G.ldc % 8 == 0 && n0 + LBN <= N &&
      (((uintptr_t)G.C | (uintptr_t)G.bias | (uintptr_t)G.U) & 15) == 0 &&
      (epi != EPI_CROSS ||
       (G.ldx % 8 == 0 && tm_ldxl(G) % 8 == 0 && (((uintptr_t)G.X0 | (uintptr_t)tm_xl(G)) & 15) == 0));
  const uint16_t* __restrict__ XLp = (const uint16_t*)tm_xl(G);
  const int ldxl = tm_ldxl(G);
  // The two epilogues that read global memory (cross: x0 and x_l; accumulate: C itself) request
  // all of a half's operands before the accumulators are parked: with one block per CU nothing
  // else hides that latency, and a thread's eight chunks one after another cost eight of them.
  constexpr int kChunks = 128 * (LBN / 8) / kBigThreads;
  // (byte offsets from the operand's base fit 32 bits: one register per address instead of two)
  const bool fast_cross = epi == EPI_CROSS && vec_ok && (int64_t)M * G.ldx < (1LL << 31) &&
                          (int64_t)M * ldxl < (1LL << 31) && (int64_t)M * G.ldc < (1LL << 31);
  const bool fast_add = epi == EPI_F32_ADD && n0 + LBN <= N && G.ldc % 4 == 0 &&
                        (int64_t)M * G.ldc < (1LL << 30) &&
                        (((uintptr_t)((float*)G.C + slice * G.cstride)) & 15) == 0;
  // bias / bias + ReLU / plain float32 tiles walk the same unrolled loop (nothing to prefetch)
  const bool fast_plain = vec_ok && epi <= EPI_BIAS_RELU && (int64_t)M * G.ldc < (1LL << 31);
  const bool fast_f32 = epi == EPI_F32 && n0 + LBN <= N && G.ldc % 4 == 0 &&
                        (int64_t)M * G.ldc < (1LL << 30) &&
                        (((uintptr_t)((float*)G.C + slice * G.cstride)) & 15) == 0;
  const bool fast = fast_cross || fast_add || fast_plain || fast_f32;
  const char* const pre_a = fast_cross ? (const char*)G.X0 : (const char*)((float*)G.C + slice * G.cstride);
  const char* const pre_b = fast_cross ? (const char*)XLp : pre_a + 16;
  const uint32_t pre_lda = fast_cross ? (uint32_t)G.ldx * 2u : (uint32_t)G.ldc * 4u;   // row pitch, bytes
  const uint32_t pre_ldb = fast_cross ? (uint32_t)ldxl * 2u : pre_lda;
  const uint32_t pre_col = fast_cross ? 2u : 4u;                                        // bytes per column
#pragma clang loop unroll(full)
  for (int h = 0; h < 2; ++h) {
    uint4 pa[kChunks], pb[kChunks];
    if (fast_cross || fast_add) {
#pragma clang loop unroll(full)
      for (int u = 0; u < kChunks; ++u) {
        const int c = tid + u * kBigThreads;
        const int r = c / (LBN / 8), cc = (c % (LBN / 8)) * 8;
        const uint32_t m = (uint32_t)min(m0 + h * 128 + r, M - 1), n = (uint32_t)(n0 + cc);
        pa[u] = *(const uint4*)(pre_a + (m * pre_lda + n * pre_col));
        pb[u] = *(const uint4*)(pre_b + (m * pre_ldb + n * pre_col));
      }
    }
    if (wm == h) {
#pragma clang loop unroll(full)
      for (int j = 0; j < 2; ++j)
#pragma clang loop unroll(full)
        for (int i = 0; i < 4; ++i)
#pragma clang loop unroll(full)
          for (int g = 0; g < 4; ++g)
            *(float4*)(stage + (i * 32 + (lane & 31)) * kStageStride + wn * 64 + j * 32 + g * 8 + (lane >> 5) * 4) =
                make_float4(acc[i][j][g * 4], acc[i][j][g * 4 + 1], acc[i][j][g * 4 + 2], acc[i][j][g * 4 + 3]);
    }
    __syncthreads();
    if (fast) {
      // chunk u of half h is row h * 128 + u * 16 + tid / 32 of the tile, the thread's own 8
      // columns: one 32-bit byte offset from C (and U), advanced by a uniform step
      const int r0 = tid / (LBN / 8), cc = (tid % (LBN / 8)) * 8;
      const uint32_t esz = epi >= EPI_F32 ? 4u : 2u;
      char* const cbase = epi >= EPI_F32 ? (char*)((float*)G.C + slice * G.cstride) : (char*)G.C;
      const uint32_t ostep = 16u * (uint32_t)G.ldc * esz;
      uint32_t off = ((uint32_t)(m0 + h * 128 + r0) * (uint32_t)G.ldc + (uint32_t)(n0 + cc)) * esz;
      // a thread's chunks all lie in one 8-column piece of the tile: one bias load serves them
      uint4 bias_raw = make_uint4(0, 0, 0, 0);
      if ((fast_cross || fast_plain) && G.bias) bias_raw = *(const uint4*)((const uint16_t*)G.bias + n0 + cc);
#pragma clang loop unroll(full)
      for (int u = 0; u < kChunks; ++u, off += ostep) {
        const int r = r0 + u * 16;
        if (m0 + h * 128 + r >= M) continue;
        float y[8];
        const float4 s0 = *(const float4*)(stage + r * kStageStride + cc);
        const float4 s1 = *(const float4*)(stage + r * kStageStride + cc + 4);
        y[0] = s0.x; y[1] = s0.y; y[2] = s0.z; y[3] = s0.w;
        y[4] = s1.x; y[5] = s1.y; y[6] = s1.z; y[7] = s1.w;
        if (fast_add) {
          const float4 p0 = __builtin_bit_cast(float4, pa[u]), p1 = __builtin_bit_cast(float4, pb[u]);
          *(float4*)(cbase + off) = make_float4(y[0] + p0.x, y[1] + p0.y, y[2] + p0.z, y[3] + p0.w);
          *(float4*)(cbase + off + 16) = make_float4(y[4] + p1.x, y[5] + p1.y, y[6] + p1.z, y[7] + p1.w);
        } else if (fast_f32) {
          *(float4*)(cbase + off) = s0;
          *(float4*)(cbase + off + 16) = s1;
        } else {
          float bv[8];
          dmt::decode_chunk<DT>(bv, bias_raw);
#pragma clang loop unroll(full)
          for (int q = 0; q < 8; ++q) y[q] += bv[q];
          if (fast_plain) {
            if (epi == EPI_BIAS_RELU) {
#pragma clang loop unroll(full)
              for (int q = 0; q < 8; ++q) y[q] = y[q] > 0.f ? y[q] : 0.f;
            }
          } else {
            float xv[8], lv[8];
            if (G.U) dmt::store_chunk<DT, 8>((char*)G.U + off, 0, y);
            dmt::decode_chunk<DT>(xv, pa[u]);
            dmt::decode_chunk<DT>(lv, pb[u]);
#pragma clang loop unroll(full)
            for (int q = 0; q < 8; ++q) y[q] = xv[q] * y[q] + lv[q];
          }
          dmt::store_chunk<DT, 8>(cbase + off, 0, y);
        }
      }
      __syncthreads();
      continue;
    }
    for (int c = tid; c < 128 * (LBN / 8); c += kBigThreads) {
      const int r = c / (LBN / 8), cc = (c % (LBN / 8)) * 8;
      const int m = m0 + h * 128 + r, n = n0 + cc;
      if (m >= M || n >= N) continue;
      float y[8];
      const float4 s0 = *(const float4*)(stage + r * kStageStride + cc);
      const float4 s1 = *(const float4*)(stage + r * kStageStride + cc + 4);
      y[0] = s0.x; y[1] = s0.y; y[2] = s0.z; y[3] = s0.w;
      y[4] = s1.x; y[5] = s1.y; y[6] = s1.z; y[7] = s1.w;
      if (epi >= EPI_F32) {
        float* c = (float*)G.C + slice * G.cstride + (int64_t)m * G.ldc + n;
        if (n + 8 <= N && ((uintptr_t)c & 15) == 0) {
          float4 lo = make_float4(y[0], y[1], y[2], y[3]), hi = make_float4(y[4], y[5], y[6], y[7]);
          if (epi == EPI_F32_ADD) {
            const float4 p0 = *(const float4*)c, p1 = *(const float4*)(c + 4);
            lo.x += p0.x; lo.y += p0.y; lo.z += p0.z; lo.w += p0.w;
            hi.x += p1.x; hi.y += p1.y; hi.z += p1.z; hi.w += p1.w;
          }
          *(float4*)c = lo;
          *(float4*)(c + 4) = hi;
          continue;
        }
        for (int q = 0; q < 8 && n + q < N; ++q) c[q] = epi == EPI_F32_ADD ? c[q] + y[q] : y[q];
        continue;
      }
      if (vec_ok) {
        float bv[8], xv[8], lv[8];
        if (G.bias) {
          dmt::decode_chunk<DT>(bv, *(const uint4*)((const uint16_t*)G.bias + n));
#pragma clang loop unroll(full)
          for (int q = 0; q < 8; ++q) y[q] += bv[q];
        }
        if (epi == EPI_BIAS_RELU) {
#pragma clang loop unroll(full)
          for (int q = 0; q < 8; ++q) y[q] = y[q] > 0.f ? y[q] : 0.f;
        }
        if (epi == EPI_CROSS) {
          if (G.U) dmt::store_chunk<DT, 8>(G.U, (int64_t)m * G.ldc + n, y);
          dmt::decode_chunk<DT>(xv, *(const uint4*)((const uint16_t*)G.X0 + (int64_t)m * G.ldx + n));
          dmt::decode_chunk<DT>(lv, *(const uint4*)(XLp + (int64_t)m * ldxl + n));
#pragma clang loop unroll(full)
          for (int q = 0; q < 8; ++q) y[q] = xv[q] * y[q] + lv[q];
        }
        dmt::store_chunk<DT, 8>(G.C, (int64_t)m * G.ldc + n, y);
      } else {
        for (int q = 0; q < 8 && n + q < N; ++q) {
          float z = y[q] + (G.bias ? load_elt<DT>(G.bias, n + q) : 0.f);
          if (epi == EPI_BIAS_RELU) z = z > 0.f ? z : 0.f;
          if (epi == EPI_CROSS) {
            if (G.U) store_elt<DT>(G.U, (int64_t)m * G.ldc + n + q, z);
            z = load_elt<DT>(G.X0, (int64_t)m * G.ldx + n + q) * z +
                load_elt<DT>(XLp, (int64_t)m * ldxl + n + q);
          }
          store_elt<DT>(G.C, (int64_t)m * G.ldc + n + q, z);
        }
      }
    }
    __syncthreads();
  }
}

// --------------------------------------------------- plain FMA GEMM (float32)

template <int DT, int TAG = DMT_TM_TAG>
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
  if (G.epi >= EPI_F32) {
    float* c = (float*)G.C + tm_crow(G, m) + n;
    *c = G.epi == EPI_F32_ADD ? *c + s : s;
    return;
  }
  float y = s + (G.bias ? load_elt<DT>(G.bias, n) : 0.f);
  if (G.epi == EPI_BIAS_RELU) y = y > 0.f ? y : 0.f;
  if (G.epi == EPI_CROSS) {
    if (G.U) store_elt<DT>(G.U, (int64_t)m * G.ldc + n, y);
    y = load_elt<DT>(G.X0, (int64_t)m * G.ldx + n) * y +
        load_elt<DT>(tm_xl(G), (int64_t)m * tm_ldxl(G) + n);
  }
  store_elt<DT>(G.C, tm_crow(G, m) + n, y);
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
  // zeros behind the terms of the row group's samples (2 features: 16 samples x 7 columns, more
  // than one per lane)
  const int npad = np_pad - np;
  for (int e = lane; e < spg * npad; e += 64) {
    const int s = e / npad, q = e % npad;
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

// What a training forward keeps for the backward: for every cross layer l of a cross tower
// (full-rank or low-rank), x_{l+1} and u_l = W_l x_l + b_l, each [B][W_t] in the compute type;
// for a dot-product tower its dot terms, [B][np_pad] (np_pad = the F (F - 1) / 2 terms rounded
// up to 8, zeros behind them), and its projection weights with zero columns inserted to match,
// [O][np_pad + W_t].  Offsets in bytes from a 256-byte-aligned base; towers of other
// kinds keep nothing (their backward needs only the pooled values).
struct TmKept {
  size_t x[DMT_MAX_CROSS_LAYERS] = {}, u[DMT_MAX_CROSS_LAYERS] = {};
  size_t z = 0, wp = 0;      // dot tower: dot terms, and the projection weights as repacked for them
  bool has_z = false;
};

inline size_t plan_tm_kept(const dmt_plan* p, const dmt_tm_params* tp, int64_t B, int eb,
                           std::vector<TmKept>* kept) {
  size_t off = 0;
  kept->assign(p->T, TmKept());
  for (int32_t t = 0; t < p->T; ++t) {
    if (tp[t].kind == DMT_TM_DOT_LINEAR) {
      const int nf = p->tower_ntab[t], np_pad = (nf * (nf - 1) / 2 + 7) / 8 * 8;
      if (np_pad > 0) {
        (*kept)[t].z = off;
        (*kept)[t].has_z = true;
        off += dmt_align_up((size_t)B * np_pad * eb, 256);
        (*kept)[t].wp = off;
        off += dmt_align_up((size_t)tp[t].out_dim * (np_pad + p->tower_width[t]) * eb, 256);
      }
      continue;
    }
    if (tp[t].kind != DMT_TM_CROSS_LINEAR && tp[t].kind != DMT_TM_CROSS_LOWRANK_LINEAR) continue;
    const size_t bytes = dmt_align_up((size_t)B * p->tower_width[t] * eb, 256);
    for (int l = 0; l < tp[t].num_cross_layers && l < DMT_MAX_CROSS_LAYERS; ++l) {
      (*kept)[t].x[l] = off; off += bytes;
      (*kept)[t].u[l] = off; off += bytes;
    }
  }
  return off;
}

// Whether a group can go to the 256 x 256 kernel (dots: with in-kernel dot terms).  At most 128
// rows or columns (a weight gradient with few outputs) would leave half of every tile empty.
inline bool big_ok(const TmGroup& g, bool dots) {
  return g.N > 128 && g.M > 128 && g.N <= kSuper * LBN && g.K1 >= 128 && (dots || g.K0 == 0) &&
         g.rdiv == 0 &&
         (int64_t)g.M * g.lda1 < (1LL << 31) && (int64_t)g.N * g.ldw < (1LL << 31);
}

template <int DT>
void launch_groups(const dmt_plan* p, std::vector<TmGroup>& groups, hipStream_t s,
                   bool dots = false, int kid = DMT_K_TM_GEMM) {
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
        tiles += ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN) * tm_slices(g);
    }
    L.tile_start[L.ngroups] = tiles;
    if (tiles == 0) continue;
    if constexpr (DT == DMT_F32) {
      DmtScope sc_(p, kid, s);
      hipLaunchKernelGGL((tm_gemm_simple<DT>), dim3(tiles), dim3(kBlock), 0, s, L);
    } else {
      // wide outputs take the 256 x 256 kernel
      bool big = dots || p->sw.tm_big != 0;
      for (int i = 0; i < L.ngroups; ++i) big = big && big_ok(L.g[i], dots);
      if (big) {
        static bool configured = false;
        if (!configured) {
          (void)hipFuncSetAttribute((const void*)tm_gemm_mfma_256<DT, false>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kBigLdsBytes);
          (void)hipFuncSetAttribute((const void*)tm_gemm_mfma_256<DT, true>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kBigLdsBytes);
          (void)hipFuncSetAttribute((const void*)tm_gemm_mfma_256<DT, true, DMT_TM_TAG, true>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kBigLdsBytes);
          (void)hipFuncSetAttribute((const void*)tm_gemm_mfma_256<DT, false, DMT_TM_TAG, false, true>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kBigLdsBytes);
          configured = true;
        }
        int32_t nst = 0;                                      // super-tiles of the launch
        for (int i = 0; i < L.ngroups; ++i) {
          L.tile_start[i] = nst;
          const int tn = (L.g[i].N + LBN - 1) / LBN;
          const int tm = (L.g[i].M + LBM - 1) / LBM * tm_slices(L.g[i]);
          const int sm = tn >= kSuper ? 1 : kSuper / tn;
          nst += (tm + sm - 1) / sm;
        }
        L.tile_start[L.ngroups] = nst;
        const int32_t big_tiles = (nst + 7) / 8 * 8 * kSuper;
        DmtScope sc_(p, kid, s);
        // every tile interior and every operand row 16-byte aligned: tiles go straight to LDS
        bool direct = !dots && p->sw.tm_direct != 0;
        for (int i = 0; i < L.ngroups; ++i) {
          const TmGroup& g = L.g[i];
          const int kk = g.ksplit > 1 ? g.klen : g.K1;
          direct = direct && g.M % LBM == 0 && g.N % LBN == 0 && kk >= BK && kk % BK == 0 && g.K1 % BK == 0 &&
                   g.lda1 % 8 == 0 && g.ldw % 8 == 0 &&
                   (((uintptr_t)g.A1 | (uintptr_t)g.W) & 15) == 0;
        }
        bool keepz = false;                   // a training forward keeps the dot terms
        for (int i = 0; i < L.ngroups; ++i) keepz = keepz || (dots && L.g[i].U != nullptr);
        if (keepz)
          hipLaunchKernelGGL((tm_gemm_mfma_256<DT, true, DMT_TM_TAG, true>), dim3(big_tiles),
                             dim3(kBigThreads), kBigLdsBytes, s, L);
        else if (dots)
          hipLaunchKernelGGL((tm_gemm_mfma_256<DT, true>), dim3(big_tiles), dim3(kBigThreads),
                             kBigLdsBytes, s, L);
        else if (direct)
          hipLaunchKernelGGL((tm_gemm_mfma_256<DT, false, DMT_TM_TAG, false, true>), dim3(big_tiles),
                             dim3(kBigThreads), kBigLdsBytes, s, L);
        else
          hipLaunchKernelGGL((tm_gemm_mfma_256<DT, false>), dim3(big_tiles), dim3(kBigThreads),
                             kBigLdsBytes, s, L);
      } else {
        bool keepu = false;
        for (int i = 0; i < L.ngroups; ++i) keepu = keepu || L.g[i].U != nullptr;
        DmtScope sc_(p, kid, s);
        if (keepu)
          hipLaunchKernelGGL((tm_gemm_mfma<DT, true>), dim3(tiles), dim3(kBlock), 0, s, L);
        else
          hipLaunchKernelGGL((tm_gemm_mfma<DT, false>), dim3(tiles), dim3(kBlock), 0, s, L);
      }
    }
  }
  groups.clear();
}
// Grouped launch of the dot-term (which = 0: Gram tiles on MFMA, 1: plain FMA) or weight-repack
// (which = 2) kernels over `items`; nblocks[i] blocks serve items[i].
template <int DT>
void launch_aux(const dmt_plan* p, int64_t B, std::vector<TmAuxItem>& items,
                std::vector<int64_t>& nblocks, int which, hipStream_t s) {
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
        DmtScope scope(p, DMT_K_TM_DOTS, s);
        hipLaunchKernelGGL((tm_dots_mfma<DT>), dim3(blocks), dim3(kBlock), 0, s, L);
      }
    } else if (which == 1) {
      DmtScope scope(p, DMT_K_TM_DOTS, s);
      hipLaunchKernelGGL((tm_dots_simple<DT>), dim3(blocks), dim3(kBlock), 0, s, L);
    } else {
      DmtScope scope(p, DMT_K_TM_PACK, s);
      hipLaunchKernelGGL((tm_pack_w<DT>), dim3(blocks), dim3(kBlock), 0, s, L);
    }
  }
}

}  // namespace
