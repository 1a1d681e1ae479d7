// SPTT's data-shuffle steps inside one GPU's memory (paper Sec. 3.1.1): step c, the peer
// permute, and step e, the (features, peers) -> (peers, features) shuffle.  Both move whole
// blocks (the embeddings of one feature for one rank's samples) and both are transposes of a
// 2-D arrangement of blocks:
//   step c  ranks g = host * L + local, peer order position k = local * T + host:
//           [features][T hosts][L locals][block] -> [features][L][T][block]
//   step e  [features][peers][block] -> [peers][features][block]
// One kernel does either at the rate of a device-to-device copy.  (In the training step of
// this library neither is launched: dmt_tower_lookup_fwd stores its output in the final layout.
// They are the explicit form, for a deployment where step d's exchange sits between them.)
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

}  // namespace

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
