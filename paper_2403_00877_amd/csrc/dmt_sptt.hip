// SPTT's data-shuffle steps inside one GPU's memory (paper Sec. 3.1.1): step c, the peer
// permute, and step e, the (features, peers) -> (peers, features) shuffle.  Both move whole
// blocks (the embeddings of one feature for one rank's samples) and both are transposes of a
// 2-D arrangement of blocks:
//   step c  ranks g = host * L + local, peer order position k = local * T + host:
//           [features][T hosts][L locals][block] -> [features][L][T][block]
//   step e  [features][peers][block] -> [peers][features][block]
// One kernel does either at the rate of a device-to-device copy.  With steps b and c swapped
// (Sec. 3.1.3) the permute acts on the jagged sparse inputs instead: dmt_sptt_peer_permute_ids.  (In the training step of
// this library neither is launched: dmt_tower_lookup_fwd stores its output in the final layout.
// They are the explicit form, for a deployment where step d's exchange sits between them.)
#include <algorithm>

#include "dmt_internal.h"
#include "dmt_device_utils.h"

namespace {

constexpr int kBlock = 256;
constexpr int kUnroll = 4;                   // 16-byte units per thread and workgroup pass

// out[a][q][p][:] = in[a][p][q][:] for blocks of `units` 16-byte units.  A workgroup copies one
// run of up to kBlock * kUnroll units of one destination block.
__global__ __launch_bounds__(kBlock) void sptt_transpose_blocks(const uint4* __restrict__ in,
                                                                uint4* __restrict__ out, int64_t P,
                                                                int64_t Q, int64_t units,
                                                                int64_t runs_per_block) {
  const int64_t d = blockIdx.x / runs_per_block, run = blockIdx.x % runs_per_block;
  const int64_t p = d % P, q = (d / P) % Q, a = d / (P * Q);
  const uint4* __restrict__ src = in + ((a * P + p) * Q + q) * units;
  uint4* __restrict__ dst = out + d * units;
  const int64_t u0 = run * (kBlock * kUnroll) + threadIdx.x;
  uint4 v[kUnroll];
#pragma unroll
  for (int i = 0; i < kUnroll; ++i)
    if (u0 + i * kBlock < units) v[i] = dmt::nt_load(src + u0 + i * kBlock);
#pragma unroll
  for (int i = 0; i < kUnroll; ++i)
    if (u0 + i * kBlock < units) dmt::nt_store(v[i], dst + u0 + i * kBlock);
}

dmt_status transpose_blocks(const void* in, void* out, int64_t A, int64_t P, int64_t Q,
                            int64_t block_bytes, hipStream_t s) {
  if (!in || !out || in == out || A <= 0 || P <= 0 || Q <= 0 || block_bytes <= 0) return DMT_EINVAL;
  if ((block_bytes & 15) || ((uintptr_t)in & 15) || ((uintptr_t)out & 15)) return DMT_EINVAL;
  const int64_t units = block_bytes / 16;
  const int64_t runs = (units + kBlock * kUnroll - 1) / (kBlock * kUnroll);
  // block counts and the grid stay within 31 bits
  if (A > (1 << 20) || P > (1 << 20) || Q > (1 << 20)) return DMT_ENOTSUP;
  if ((double)A * (double)P * (double)Q * (double)runs >= 2147483648.0) return DMT_ENOTSUP;
  hipLaunchKernelGGL(sptt_transpose_blocks, dim3((unsigned)(A * P * Q * runs)), dim3(kBlock), 0, s,
                     (const uint4*)in, (uint4*)out, P, Q, units, runs);
  return hipGetLastError() == hipSuccess ? DMT_OK : DMT_EHIP;
}

// ---------------------------------------------------- steps b and c swapped: the permute on ids
//
// The bags of feature f arrive as G blocks of B_l bags in rank order; the blocks go to peer
// order, position k = (g % L) * T + g / L, i.e. the block at position k comes from rank
// g = (k % T) * L + k / T.  A feature's ids stay inside the feature's own range of `indices`.

// One workgroup per feature: where each of the feature's G blocks starts in the output
// (a scan of the block lengths in peer order), then the offsets of all its bags.
__global__ __launch_bounds__(kBlock) void sptt_permute_offsets(const int64_t* __restrict__ offsets,
                                                               int64_t* __restrict__ out_offsets,
                                                               int64_t features, int32_t G, int32_t L,
                                                               int64_t Bl, int64_t nnz) {
  __shared__ int64_t start[1024 + 1];
  const int64_t f = blockIdx.x;
  const int32_t T = G / L;
  auto clamp = [&](int64_t o) { return o < 0 ? 0 : (o > nnz ? nnz : o); };
  auto rank_of = [&](int32_t k) { return (k % T) * L + k / T; };
  const int64_t base = clamp(offsets[f * G * Bl]);
  if (threadIdx.x == 0) {
    int64_t run = base;
    for (int32_t k = 0; k < G; ++k) {
      const int64_t first = (f * G + rank_of(k)) * Bl;
      const int64_t len = clamp(offsets[first + Bl]) - clamp(offsets[first]);
      start[k] = run;
      run = clamp(run + (len > 0 ? len : 0));
    }
    start[G] = run;
  }
  __syncthreads();
  for (int64_t j = threadIdx.x; j < (int64_t)G * Bl; j += kBlock) {
    const int32_t k = (int32_t)(j / Bl);
    const int64_t b = j - (int64_t)k * Bl, first = (f * G + rank_of(k)) * Bl;
    const int64_t in_block = clamp(offsets[first + b]) - clamp(offsets[first]);
    out_offsets[f * G * Bl + j] = clamp(start[k] + (in_block > 0 ? in_block : 0));
  }
  if (f == features - 1 && threadIdx.x == 0) out_offsets[features * G * Bl] = start[G];
}

// blockIdx.y = destination block (feature, position); the workgroups of a block stride over
// its ids.  Every range is clamped to [0, nnz], whatever the offsets hold.
__global__ __launch_bounds__(kBlock) void sptt_permute_ids(const int32_t* __restrict__ indices,
                                                           const int64_t* __restrict__ offsets,
                                                           const int64_t* __restrict__ out_offsets,
                                                           int32_t* __restrict__ out_indices, int32_t G,
                                                           int32_t L, int64_t Bl, int64_t nnz) {
  const int64_t d = blockIdx.y;
  const int64_t f = d / G;
  const int32_t k = (int32_t)(d - f * G), T = G / L;
  const int64_t src_first = (f * G + (k % T) * L + k / T) * Bl;
  auto clamp = [&](int64_t o) { return o < 0 ? 0 : (o > nnz ? nnz : o); };
  const int64_t s0 = clamp(offsets[src_first]), d0 = clamp(out_offsets[d * Bl]);
  int64_t len = clamp(offsets[src_first + Bl]) - s0;
  len = len < nnz - d0 ? len : nnz - d0;
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < len; i += (int64_t)gridDim.x * kBlock)
    out_indices[d0 + i] = indices[s0 + i];
}

}  // namespace

extern "C" dmt_status dmt_sptt_peer_permute_ids(const int32_t* indices, const int64_t* offsets,
                                                int64_t features, int32_t G, int32_t L, int64_t Bl,
                                                int64_t nnz, int32_t* out_indices,
                                                int64_t* out_offsets, void* stream) {
  if (!offsets || !out_offsets || (nnz > 0 && (!indices || !out_indices))) return DMT_EINVAL;
  if (features <= 0 || G <= 0 || L <= 0 || G % L != 0 || Bl <= 0 || nnz < 0) return DMT_EINVAL;
  if (indices == out_indices && nnz > 0) return DMT_EINVAL;
  if (offsets == out_offsets) return DMT_EINVAL;
  if (G > 1024 || features > (1 << 20) || features * G > 65535) return DMT_ENOTSUP;   // LDS table, grid.y
  hipStream_t s = (hipStream_t)stream;
  hipLaunchKernelGGL(sptt_permute_offsets, dim3((unsigned)features), dim3(kBlock), 0, s, offsets,
                     out_offsets, features, G, L, Bl, nnz);
  if (nnz > 0) {
    // workgroups per block of ids: enough for an average block, at most 64
    const int64_t per_block = nnz / (features * G) + 1;
    const unsigned gx = (unsigned)std::min<int64_t>(64, (per_block + kBlock * 8 - 1) / (kBlock * 8));
    hipLaunchKernelGGL(sptt_permute_ids, dim3(gx, (unsigned)(features * G)), dim3(kBlock), 0, s, indices,
                       offsets, out_offsets, out_indices, G, L, Bl, nnz);
  }
  return hipGetLastError() == hipSuccess ? DMT_OK : DMT_EHIP;
}

extern "C" dmt_status dmt_sptt_peer_order(int32_t G, int32_t L, int32_t* order) {
  if (!order || G <= 0 || L <= 0 || G % L != 0) return DMT_EINVAL;
  const int32_t T = G / L;
  // ascending (g % L, g / L): position k = (g % L) * T + g / L
  for (int32_t g = 0; g < G; ++g) order[(g % L) * T + g / L] = g;
  return DMT_OK;
}

extern "C" dmt_status dmt_sptt_peer_permute(const void* in, void* out, int64_t features, int32_t G,
                                            int32_t L, int64_t block_bytes, void* stream) {
  if (G <= 0 || L <= 0 || G % L != 0) return DMT_EINVAL;
  // source block (f, host, local) -> destination (f, local, host)
  return transpose_blocks(in, out, features, G / L, L, block_bytes, (hipStream_t)stream);
}

extern "C" dmt_status dmt_sptt_shuffle(const void* in, void* out, int64_t features, int64_t peers,
                                       int64_t block_bytes, void* stream) {
  return transpose_blocks(in, out, 1, features, peers, block_bytes, (hipStream_t)stream);
}
