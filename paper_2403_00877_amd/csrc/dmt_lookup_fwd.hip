// dmt_tower_lookup_fwd: tower-local sum-pooled embedding lookup with the
// tower-major permute fused into the store (paper Sec. 2.2 step b; layout of
// Sec. 3.1.1 steps c-e, i.e. `embs` of Sec. 4).
//
// HBM/L2-bound gather.  Work decomposition for wave64:
//  * a row of D elements is D*e/16 sixteen-byte chunks; LPR lanes (a power of
//    two) fetch one row with one dwordx4 load each, fully coalesced;
//  * a bag is served by a group of GL = LPR*R lanes: R rows of the bag are in
//    flight per load instruction, and every lane unrolls 4 such loads, so a
//    wave keeps up to 4*64/LPR rows in flight;  R is 1 (many bags per wave)
//    unless bags are very long;
//  * the group reads its bag's ids coalesced (one per lane) and hands them
//    round with ds_bpermute; partial sums of the R row slots are combined by a
//    fixed xor tree, so results repeat bit for bit;
//  * block -> tile mapping is XCD-aware: consecutive block ids land on
//    different XCDs, so block id b works on tile (b % 8) * tiles_per_xcd + b / 8
//    and every XCD streams through its own contiguous run of tables, keeping
//    one table's hot rows in that XCD's L2.
#include "dmt_internal.h"
#include "dmt_device_utils.h"

namespace {

// One wave per block: a block's lane groups share nothing but the staged offsets, and with
// several waves a block its wave slots are only handed on when the wave with the longest bags
// is done (measured against 256 threads: Mid and Large 2.5 - 3 % shorter, Imbalanced 3 - 4 %).
constexpr int kBlock = 64;
constexpr int kStagedBags = kBlock * 8;  // most bags of one block whose offsets are staged in LDS
#ifndef DMT_LOOKUP_UNROLL
#define DMT_LOOKUP_UNROLL 4
#endif
constexpr int kUnroll = DMT_LOOKUP_UNROLL;

template <int TD, int OD>
__global__ __launch_bounds__(kBlock) void lookup_fwd_kernel(
    const DmtTableMeta* __restrict__ meta, const int32_t* __restrict__ class_tables, int32_t D,
    const int32_t* __restrict__ indices, const int64_t* __restrict__ offsets, int64_t B,
    int64_t nnz, void* __restrict__ out, int log2_lpr, int log2_gl, int bags_per_group,
    int32_t tiles_per_table, int32_t ntiles, int32_t tiles_per_xcd, int long_thr,
    int stage_offsets, unsigned long long* __restrict__ err) {
  constexpr int EPL = dmt::ChunkElems<TD>::value;
  const int bid = blockIdx.x;
  const int tile = (bid & 7) * tiles_per_xcd + (bid >> 3);
  if (tile >= ntiles) return;
  const int k = tile / tiles_per_table;
  const int c = tile - k * tiles_per_table;
  const int f = class_tables[k];
  const char* __restrict__ tab = (const char*)meta[f].table;
  const int64_t rows = meta[f].rows, row_begin = meta[f].row_begin;
  const int64_t out_base = B * meta[f].out_prefix + meta[f].col_off;
  const int32_t tower_width = meta[f].tower_width;
  const int LPR = 1 << log2_lpr;
  const int lane = threadIdx.x & 63;
  const int chunk = threadIdx.x & (LPR - 1);
  const bool chunk_ok = chunk * EPL < D;
  const int64_t rowbytes = (int64_t)D * dmt::EltBytes<TD>::value;

  // The aligned group of 2^lg lanes this thread is in pools bag b (ids s .. s + len).
  auto pool_bag = [&](int64_t b, int64_t s, int len, int lg) {
    const int GL = 1 << lg, R = GL >> log2_lpr;
    const int gl = threadIdx.x & (GL - 1);
    const int slot = gl >> log2_lpr;
    const int group_lane0 = lane & ~(GL - 1);
    float acc[EPL];
#pragma unroll
    for (int q = 0; q < EPL; ++q) acc[q] = 0.f;
    for (int base = 0; base < len; base += GL) {
      const int n = min(GL, len - base);
      int my = 0;
      if (gl < n) {
        // a row-wise shard skips the ids of other shards silently (err is null then)
        const int64_t local = (int64_t)indices[s + base + gl] - row_begin;
        my = (int)local;
        if ((unsigned long long)local >= (unsigned long long)rows) {
          if (err) atomicMin(err, (unsigned long long)(s + base + gl));
          my = -1;
        }
      }
      for (int p0 = 0; p0 < n; p0 += R * kUnroll) {
        uint4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
          const int p = p0 + u * R + slot;
          const int r = __shfl(my, group_lane0 + (p & (GL - 1)));
          v[u] = make_uint4(0, 0, 0, 0);
          if (chunk_ok && p < n && r >= 0)
            v[u] = dmt::gload((const uint4*)(tab + (int64_t)r * rowbytes + chunk * 16));
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) dmt::accumulate_chunk<TD>(acc, v[u]);
      }
    }
    for (int o = LPR; o < GL; o <<= 1) {
#pragma unroll
      for (int q = 0; q < EPL; ++q) acc[q] += __shfl_xor(acc[q], o);
    }
    if (slot == 0 && chunk_ok)
      dmt::store_chunk<OD, EPL>(out, out_base + b * tower_width + chunk * EPL, acc);
  };

  const int GL = 1 << log2_gl;
  const int gl = threadIdx.x & (GL - 1);
  const int group = threadIdx.x >> log2_gl;
  const int ngroups = kBlock >> log2_gl;
  const int64_t b0 = (int64_t)c * ngroups * bags_per_group;
  // A block's bags are consecutive.  When every lane group pools several of them, their
  // offsets come in with one coalesced read through LDS, so that a group's next bag starts
  // at its ids; with one bag per group the direct read is the shorter path.
  __shared__ int64_t s_off[kStagedBags + 1];
  const bool staged = stage_offsets != 0;
  if (staged) {
    const int nb_blk = (int)min((int64_t)ngroups * bags_per_group, B - b0);
    for (int j = threadIdx.x; j <= nb_blk; j += kBlock) {
      const int64_t o = offsets[(int64_t)f * B + b0 + j];
      s_off[j] = o < 0 ? 0 : (o > nnz ? nnz : o);
    }
    __syncthreads();
  }
  for (int i = 0; i < bags_per_group; ++i) {
    const int64_t b = b0 + (int64_t)i * ngroups + group;
    int64_t s = 0;
    int len = 0;
    if (b < B) {
      int64_t e;
      if (staged) {
        s = s_off[b - b0];
        e = s_off[b - b0 + 1];
      } else {
        const int64_t bag = (int64_t)f * B + b;
        e = offsets[bag + 1];
        s = offsets[bag];
        s = s < 0 ? 0 : (s > nnz ? nnz : s);
        e = e > nnz ? nnz : e;
      }
      e = e < s ? s : e;
      len = (int)(e - s);
    }
    // A bag much longer than the others would hold up every other bag of its wave: the groups
    // with ordinary bags pool theirs, then the whole wave pools the long ones, one at a time,
    // 64 / LPR rows per load instruction.
    const bool is_long = long_thr > 0 && len > long_thr;
    if (b < B && !is_long) pool_bag(b, s, len, log2_gl);
    unsigned long long todo = __ballot(is_long && gl == 0);
    while (todo) {
      const int src = __builtin_ctzll(todo);
      todo &= todo - 1;
      const int64_t lb = __shfl(b, src), ls = __shfl(s, src);
      pool_bag(lb, ls, __shfl(len, src), 6);
    }
  }
}

template <int TD, int OD>
void launch(const dmt_plan* p, const DmtDimClass& c, const int32_t* indices,
            const int64_t* offsets, int64_t B, int64_t nnz, void* out, int log2_lpr, int log2_gl,
            int bpg, int long_thr, hipStream_t s) {
  const int ngroups = kBlock >> log2_gl;
  const int64_t bags_per_block = (int64_t)ngroups * bpg;
  const int32_t tiles_per_table = (int32_t)((B + bags_per_block - 1) / bags_per_block);
  const int32_t ntiles = tiles_per_table * c.num_tables;
  const int32_t tiles_per_xcd = (ntiles + 7) / 8;
  const int stage_offsets = bpg > 1 && bags_per_block <= kStagedBags;
  DmtScope scope(p, DMT_K_LOOKUP_FWD, s);
  hipLaunchKernelGGL((lookup_fwd_kernel<TD, OD>), dim3(tiles_per_xcd * 8), dim3(kBlock), 0, s,
                     p->d_meta, p->d_class_tables + c.first, c.D, indices, offsets, B, nnz, out,
                     log2_lpr, log2_gl, bpg, tiles_per_table, ntiles, tiles_per_xcd, long_thr,
                     stage_offsets, p->row_shards ? nullptr : p->d_error);
}

int ilog2_ceil(int x) {
  int l = 0;
  while ((1 << l) < x) ++l;
  return l;
}

}  // namespace

extern "C" dmt_status dmt_tower_lookup_fwd(const dmt_plan* plan, const int32_t* indices,
                                           const int64_t* offsets, int64_t B, int64_t nnz,
                                           void* pooled_out, int32_t out_dtype, void* stream) {
  if (!plan || !offsets || !pooled_out) return DMT_EINVAL;
  if (B <= 0 || B > plan->max_batch || nnz < 0 || nnz > plan->max_nnz) return DMT_EINVAL;
  if (nnz > 0 && !indices) return DMT_EINVAL;
  if (out_dtype != DMT_F32 && out_dtype != DMT_F16 && out_dtype != DMT_BF16) return DMT_EINVAL;
  if ((uintptr_t)pooled_out & 15) return DMT_EINVAL;
  if (!plan->bound) return DMT_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  const int eb = dmt_elt_bytes(plan->table_dtype);
  const double mean_len = (double)nnz / ((double)plan->F * (double)B);
  const int tuned_r = plan->sw.lookup_r, tuned_bpg = plan->sw.lookup_bpg;

  for (const DmtDimClass& c : plan->classes) {
    const int log2_lpr = ilog2_ceil(c.D * eb / 16);
    // rows of one bag in flight per load instruction.  Measured on MI355X (Mid,
    // mean length 20): one row slot per bag and more bags per wave beats a whole
    // wave per bag (0.24 ms against 0.30 ms), so slots are only added once a
    // slot's serial chain would get long.
    int r = 1;
    while (r * 2 * 16 * kUnroll <= mean_len && ((r * 2) << log2_lpr) <= 64) r *= 2;
    if (tuned_r > 0) {
      r = 1;
      while (r * 2 <= tuned_r && ((r * 2) << log2_lpr) <= 64) r *= 2;
    }
    const int log2_gl = log2_lpr + ilog2_ceil(r);
    const int ngroups = kBlock >> log2_gl;
    // bags one lane group pools in turn: short bags are batched so that a block has a few
    // dozen ids per group to work on (measured on MI355X: 8 bags at mean length 2.6, 1 at 20)
    int bpg = 1;
    while (bpg < 8 && bpg * 2 * mean_len <= 24.0) bpg *= 2;
    if (tuned_bpg > 0) bpg = tuned_bpg;
    // bags several times longer than the mean are pooled by whole waves (0: never)
    int long_thr = 4 * (int)(mean_len + 1.0);
    long_thr = (long_thr < 8 ? 8 : long_thr) * r;
    if (plan->sw.lookup_long >= 0) long_thr = plan->sw.lookup_long;
    if (log2_gl >= 6) long_thr = 0;
    const int td = (int)plan->table_dtype, od = (int)out_dtype;
#define DMT_CASE(TD, OD)                                                                      \
  if (td == TD && od == OD)                                                                   \
    launch<TD, OD>(plan, c, indices, offsets, B, nnz, pooled_out, log2_lpr, log2_gl, bpg, long_thr, s);
    DMT_CASE(DMT_F32, DMT_F32) DMT_CASE(DMT_F32, DMT_F16) DMT_CASE(DMT_F32, DMT_BF16)
    DMT_CASE(DMT_F16, DMT_F32) DMT_CASE(DMT_F16, DMT_F16) DMT_CASE(DMT_F16, DMT_BF16)
    DMT_CASE(DMT_BF16, DMT_F32) DMT_CASE(DMT_BF16, DMT_F16) DMT_CASE(DMT_BF16, DMT_BF16)
#undef DMT_CASE
  }
  return hipGetLastError() == hipSuccess ? DMT_OK : DMT_EHIP;
}
