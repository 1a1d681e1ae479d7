// dmt_tower_lookup_bwd_update: gradients to the activated rows only (paper
// Sec. 2.2), as  key build -> stable LSD radix sort by row id inside every
// table's records -> tiled segment reduce fused with the rowwise Adagrad row
// update -> fix-up of rows whose run spans several tiles.
//
// Everything is deterministic: the sort is stable (equal rows keep ascending
// bag order), every row's gradient is summed in a fixed order, and each row has
// exactly one writer.  No floating-point atomics anywhere.
//
// Data in the workspace: 64-bit records (global_row << 32 | bag), where
// global_row = (sum of rows of earlier tables) + row and bag = f*B + b.  The
// lookups arrive grouped by table (bags are table-major), so the sort never moves
// a record out of its table's range: sort blocks are aligned to the tables and
// every pass ranks only the bits of the row inside the table, which takes
// ceil(log2(largest table)) bits instead of ceil(log2(all rows)).  An id outside
// its table gets the key  kInertBit | (global id one past the table's last row):
// it sorts behind the table's rows, equals no row's key, and is never touched.
// `offsets` must tile [0, nnz) (ascending, offsets[0] = 0, last = nnz): the key build
// checks this, records the first bag that breaks it, and the reduce and fix-up kernels
// then return without touching a row (dmt_last_device_error reports DMT_EINVAL).
#include <algorithm>
#include <mutex>
#include <type_traits>

#include "dmt_internal.h"
#include "dmt_device_utils.h"

namespace {

constexpr int kBlock = 256;
#ifndef DMT_SORT_ITEMS
#define DMT_SORT_ITEMS 8
#endif
#ifndef DMT_RADIX_BITS
#define DMT_RADIX_BITS 8
#endif
constexpr int kSortItems = DMT_SORT_ITEMS;
constexpr int kMaxRadixBits = DMT_RADIX_BITS;      // digit width of one sort pass
constexpr int kMaxRadix = 1 << kMaxRadixBits;
constexpr int kDigitsPerThread = (kMaxRadix + kBlock - 1) / kBlock;
constexpr int kSortTile = kBlock * kSortItems;   // records per sort block
constexpr int kScanItems = 16;
constexpr int kScanTile = kBlock * kScanItems;   // records per head-scan block
constexpr int kReduceTile = 128;                 // sorted records per reduce tile
#ifndef DMT_RU
#define DMT_RU 4
#endif
constexpr int kReduceUnroll = DMT_RU;
constexpr uint32_t kInertBit = 0x80000000u;      // key flag of an id outside its table
constexpr int kScanThreads = 1024;               // block of the per-table offset scan
constexpr int kScanBatch = 16;                   // sort blocks whose counts it reads together

struct BwdWs {
  uint64_t* pk_a;
  uint64_t* pk_b;
  uint32_t* hist;         // [nblk_sort][kMaxRadix]
  uint32_t* seg_begin;    // [F + 1] first record of each table (seg_begin[F] = nnz)
  uint32_t* seg_blk;      // [F + 1] first sort block of each table
  uint32_t* blk_table;    // [nblk_sort] table of each sort block
  uint32_t* blk_heads;    // [nblk_scan]
  uint32_t* seg_off;      // [nnz + 1]
  uint32_t* tile_first;   // [ntiles + 1] run heads before each reduce tile
  uint32_t* num_unique;   // [1]
  float* partials;        // [2 * ntiles][Dmax]
  size_t bytes;
  int64_t nblk_sort, nblk_scan, ntiles;
};

BwdWs carve(const dmt_plan* p, int64_t nnz, void* base) {
  BwdWs w;
  const int64_t n = nnz > 0 ? nnz : 1;
  w.nblk_sort = (n + kSortTile - 1) / kSortTile + p->F;   // every table may end in a partial block
  w.nblk_scan = (n + kScanTile - 1) / kScanTile;
  w.ntiles = (n + kReduceTile - 1) / kReduceTile;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off = dmt_align_up(off + bytes, 256);
    return (char*)((uintptr_t)base + o);          // (base is null when only the size is wanted)
  };
  w.pk_a = (uint64_t*)take(sizeof(uint64_t) * n);
  w.pk_b = (uint64_t*)take(sizeof(uint64_t) * n);
  w.hist = (uint32_t*)take(sizeof(uint32_t) * kMaxRadix * w.nblk_sort);
  w.seg_begin = (uint32_t*)take(sizeof(uint32_t) * (p->F + 1));
  w.seg_blk = (uint32_t*)take(sizeof(uint32_t) * (p->F + 1));
  w.blk_table = (uint32_t*)take(sizeof(uint32_t) * w.nblk_sort);
  w.blk_heads = (uint32_t*)take(sizeof(uint32_t) * (w.nblk_scan + 1));
  w.seg_off = (uint32_t*)take(sizeof(uint32_t) * (n + 1));
  w.tile_first = (uint32_t*)take(sizeof(uint32_t) * (w.ntiles + 1));
  w.num_unique = (uint32_t*)take(sizeof(uint32_t) * 64);
  w.partials = (float*)take(sizeof(float) * 2 * w.ntiles * p->max_dim);
  w.bytes = off;
  return w;
}

// ------------------------------------------------------------------ key build

// Where each table's records start and which sort blocks cover them.  Run by one block.
// The starts come from the offsets of every table's first bag, made ascending and clamped to
// [0, nnz], so that blocks stay inside the record array whatever `offsets` holds.
__device__ void build_sort_map(const int64_t* __restrict__ offsets, uint32_t B, int F, int64_t nnz,
                               uint32_t* __restrict__ seg_begin, uint32_t* __restrict__ seg_blk,
                               uint32_t* __restrict__ blk_table) {
  __shared__ uint32_t sm[kBlock / 64];
  __shared__ uint32_t s_first[kBlock], s_nb[kBlock];
  uint32_t rec_run = 0, blk_run = 0;
  for (int f0 = 0; f0 < F; f0 += kBlock) {
    const int f = f0 + (int)threadIdx.x;
    uint32_t len = 0;
    if (f < F) {
      int64_t a = offsets[(int64_t)f * B], b = offsets[(int64_t)(f + 1) * B];
      a = a < 0 ? 0 : (a > nnz ? nnz : a);
      b = b < 0 ? 0 : (b > nnz ? nnz : b);
      len = b > a ? (uint32_t)(b - a) : 0u;
    }
    uint32_t total;
    uint32_t begin = rec_run + dmt::block_exclusive_scan<kBlock / 64>(len, sm, total);
    rec_run += total;
    begin = begin > (uint32_t)nnz ? (uint32_t)nnz : begin;
    const uint32_t end = begin + len > (uint32_t)nnz ? (uint32_t)nnz : begin + len;
    const uint32_t nb = (end - begin + kSortTile - 1) / kSortTile;
    const uint32_t first = blk_run + dmt::block_exclusive_scan<kBlock / 64>(nb, sm, total);
    blk_run += total;
    if (f < F) {
      seg_begin[f] = begin;
      seg_blk[f] = first;
    }
    // the tables' block lists are written a wave per table, a block per lane
    s_first[threadIdx.x] = first;
    s_nb[threadIdx.x] = f < F ? nb : 0u;
    __syncthreads();
    for (int q = threadIdx.x >> 6; q < kBlock && f0 + q < F; q += kBlock / 64)
      for (uint32_t j = threadIdx.x & 63; j < s_nb[q]; j += 64) blk_table[s_first[q] + j] = (uint32_t)(f0 + q);
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    seg_begin[F] = rec_run > (uint32_t)nnz ? (uint32_t)nnz : rec_run;
    seg_blk[F] = blk_run;
  }
}

// One block takes 2^log2_bpb consecutive bags and walks their lookups id by id, so the work per
// thread does not depend on how the bag lengths are spread (a lane group per bag leaves most lanes
// idle when a few bags are hundreds of ids long and most hold one or two).  The bags' offsets go
// to LDS; a thread finds the bag of its position by bisection there.
constexpr int kKeysMaxBags = 1024;
__global__ __launch_bounds__(kBlock) void bwd_build_keys(
    const DmtTableMeta* __restrict__ meta, const int32_t* __restrict__ indices,
    const int64_t* __restrict__ offsets, uint32_t B, uint32_t nbags, int64_t nnz, int F,
    uint64_t* __restrict__ pk, int log2_bpb, uint32_t* __restrict__ seg_begin,
    uint32_t* __restrict__ seg_blk, uint32_t* __restrict__ blk_table,
    unsigned long long* __restrict__ err, unsigned long long* __restrict__ err_offsets) {
  __shared__ int64_t offs[kKeysMaxBags + 1];
  if (blockIdx.x == 0) build_sort_map(offsets, B, F, nnz, seg_begin, seg_blk, blk_table);
  const uint32_t g0 = blockIdx.x << log2_bpb;
  if (g0 >= nbags) return;
  const int nb = (int)min((uint32_t)(1 << log2_bpb), nbags - g0);
  // `offsets` must tile [0, nnz): starts at 0, never descends, ends at nnz.  The first bag
  // that breaks this is recorded; the reduce and fix-up kernels then touch no row.
  for (int i = threadIdx.x; i <= nb; i += kBlock) {
    const int64_t o = offsets[g0 + i];
    const bool at_end = g0 + (uint32_t)i == nbags;
    if (o < 0 || o > nnz || (g0 + (uint32_t)i == 0 && o != 0) || (at_end && o != nnz))
      atomicMin(err_offsets, (unsigned long long)(g0 + i - (at_end ? 1 : 0)));
    offs[i] = o < 0 ? 0 : (o > nnz ? nnz : o);
  }
  __syncthreads();
  for (int i = threadIdx.x; i < nb; i += kBlock)
    if (offs[i] > offs[i + 1]) atomicMin(err_offsets, (unsigned long long)(g0 + i));
  const int64_t s = offs[0], e = offs[nb];
  for (int64_t j = s + threadIdx.x; j < e; j += kBlock) {
    int lo = 0, hi = nb;                           // offs[lo] <= j < offs[hi]
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (offs[mid] <= j) lo = mid; else hi = mid;
    }
    const uint32_t g = g0 + (uint32_t)lo;
    const uint32_t f = g / B;
    const uint64_t rows = (uint64_t)meta[f].rows;
    const uint32_t row_base = (uint32_t)meta[f].row_base;
    // a row-wise shard gives the ids of other shards the inert key silently (err is null then)
    const int64_t local = (int64_t)indices[j] - meta[f].row_begin;
    uint32_t gid = row_base + (uint32_t)local;
    if ((uint64_t)local >= rows) {
      if (err) atomicMin(err, (unsigned long long)j);
      gid = kInertBit | (row_base + (uint32_t)rows);
    }
    pk[j] = ((uint64_t)gid << 32) | g;
  }
}

// ------------------------------------------------------------------ radix sort

// A sort block's share of its table's records, and the table's first global row id.
struct SortBlock {
  uint32_t base, n, row_base, valid;
};
__device__ __forceinline__ SortBlock sort_block(const DmtTableMeta* __restrict__ meta,
                                                const uint32_t* __restrict__ seg_begin,
                                                const uint32_t* __restrict__ seg_blk,
                                                const uint32_t* __restrict__ blk_table, int F) {
  SortBlock sb{0, 0, 0, 0};
  if (blockIdx.x >= seg_blk[F]) return sb;
  const uint32_t f = blk_table[blockIdx.x];
  sb.base = seg_begin[f] + (blockIdx.x - seg_blk[f]) * (uint32_t)kSortTile;
  const uint32_t end = seg_begin[f + 1];
  sb.n = end - sb.base < (uint32_t)kSortTile ? end - sb.base : (uint32_t)kSortTile;
  sb.row_base = (uint32_t)meta[f].row_base;
  sb.valid = 1;
  return sb;
}

// The pass's digit of a record: bits [shift, shift + bits) of the row id inside the table.
__device__ __forceinline__ uint32_t sort_digit(uint64_t rec, uint32_t row_base, int shift,
                                               uint32_t mask) {
  return ((((uint32_t)(rec >> 32) & ~kInertBit) - row_base) >> shift) & mask;
}

__global__ __launch_bounds__(kBlock) void radix_hist(
    const DmtTableMeta* __restrict__ meta, const uint64_t* __restrict__ pk, int shift, int bits,
    uint32_t* __restrict__ hist, const uint32_t* __restrict__ seg_begin,
    const uint32_t* __restrict__ seg_blk, const uint32_t* __restrict__ blk_table, int F) {
  __shared__ uint32_t h[kMaxRadix];
  const SortBlock sb = sort_block(meta, seg_begin, seg_blk, blk_table, F);
  if (!sb.valid) return;
  for (int d = threadIdx.x; d < kMaxRadix; d += kBlock) h[d] = 0;
  __syncthreads();
  const uint32_t mask = (1u << bits) - 1;
#pragma unroll
  for (int i = 0; i < kSortItems; ++i) {
    const uint32_t q = i * kBlock + threadIdx.x;
    if (q < sb.n) atomicAdd(&h[sort_digit(pk[sb.base + q], sb.row_base, shift, mask)], 1u);
  }
  __syncthreads();
  for (int d = threadIdx.x; d < (1 << bits); d += kBlock)
    hist[(int64_t)blockIdx.x * kMaxRadix + d] = h[d];
}

// One block per table: turns the per-block digit counts of the table's sort blocks into the
// position of each block's first record of each digit in the sorted output (digit-major,
// block-minor inside the table's record range).  Thread (slice, digit) walks one slice of the
// table's blocks.
__global__ __launch_bounds__(kScanThreads) void radix_scan(uint32_t* __restrict__ hist, int bits,
                                                           const uint32_t* __restrict__ seg_begin,
                                                           const uint32_t* __restrict__ seg_blk) {
  __shared__ uint32_t tot[kScanThreads];
  __shared__ uint32_t dbase[kMaxRadix];
  __shared__ uint32_t sm[kScanThreads / 64];
  const int f = blockIdx.x;
  const uint32_t b0 = seg_blk[f], nb = seg_blk[f + 1] - b0;
  if (nb == 0) return;
  const int R = 1 << bits, slices = kScanThreads >> bits;
  const int sl = threadIdx.x >> bits, d = threadIdx.x & (R - 1);
  const uint32_t per = (nb + slices - 1) / slices;
  const uint32_t lo = min(nb, sl * per), hi = min(nb, lo + per);
  // (counts are read sixteen blocks at a time: one by one, every read would wait for the store
  // before it, which the compiler must assume may touch the same word)
  uint32_t run = 0;
  for (uint32_t b = lo; b < hi; b += kScanBatch) {
    uint32_t v[kScanBatch];
#pragma unroll
    for (int q = 0; q < kScanBatch; ++q)
      v[q] = b + q < hi ? hist[(int64_t)(b0 + b + q) * kMaxRadix + d] : 0u;
#pragma unroll
    for (int q = 0; q < kScanBatch; ++q) {
      if (b + q < hi) hist[(int64_t)(b0 + b + q) * kMaxRadix + d] = run;
      run += v[q];
    }
  }
  tot[threadIdx.x] = run;
  __syncthreads();
  uint32_t before = 0, all = 0;                    // this digit: earlier slices, every slice
  for (int q = 0; q < slices; ++q) {
    const uint32_t t = tot[q * R + d];
    if (q < sl) before += t;
    all += t;
  }
  uint32_t total;
  const uint32_t ex = dmt::block_exclusive_scan<kScanThreads / 64>(sl == 0 ? all : 0u, sm, total);
  if (sl == 0) dbase[d] = ex;
  __syncthreads();
  const uint32_t add = seg_begin[f] + dbase[d] + before;
  for (uint32_t b = lo; b < hi; b += kScanBatch) {
    uint32_t v[kScanBatch];
#pragma unroll
    for (int q = 0; q < kScanBatch; ++q)
      v[q] = b + q < hi ? hist[(int64_t)(b0 + b + q) * kMaxRadix + d] : 0u;
#pragma unroll
    for (int q = 0; q < kScanBatch; ++q)
      if (b + q < hi) hist[(int64_t)(b0 + b + q) * kMaxRadix + d] = v[q] + add;
  }
}

__global__ __launch_bounds__(kBlock) void radix_scatter(
    const DmtTableMeta* __restrict__ meta, const uint64_t* __restrict__ in,
    uint64_t* __restrict__ out, int shift, int bits, const uint32_t* __restrict__ hist,
    const uint32_t* __restrict__ seg_begin, const uint32_t* __restrict__ seg_blk,
    const uint32_t* __restrict__ blk_table, int F) {
  __shared__ uint64_t buf[kSortTile];
  __shared__ uint32_t cnt[kBlock / 64][kMaxRadix];
  __shared__ uint32_t tile_start[kMaxRadix];
  __shared__ uint32_t gbase[kMaxRadix];
  __shared__ uint32_t sm[8];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int radix = 1 << bits;
  const uint32_t mask = (uint32_t)radix - 1;
  const SortBlock sb = sort_block(meta, seg_begin, seg_blk, blk_table, F);
  if (!sb.valid) return;
  for (int w = 0; w < kBlock / 64; ++w)
    for (int d = tid; d < kMaxRadix; d += kBlock) cnt[w][d] = 0;
  __syncthreads();
  const uint32_t tile_base = sb.base;
  const int n_tile = (int)sb.n;
  volatile __attribute__((address_space(3))) uint32_t* my_cnt =
      (volatile __attribute__((address_space(3))) uint32_t*)cnt[wave];

  // stable rank of every record among the records of its wave with the same digit
  uint64_t rec[kSortItems];
  uint32_t rank[kSortItems];
#pragma unroll
  for (int i = 0; i < kSortItems; ++i) {
    const int q = wave * (kSortItems * 64) + i * 64 + lane;
    const bool valid = q < n_tile;
    rec[i] = valid ? in[tile_base + q] : ~0ULL;
    const uint32_t d = sort_digit(rec[i], sb.row_base, shift, mask);
    uint64_t peers = __ballot(valid);              // lanes of this wave holding the same digit
    for (int b = 0; b < bits; ++b) {
      const bool bit = (d >> b) & 1;
      const uint64_t m = __ballot(bit);
      peers &= bit ? m : ~m;
    }
    uint32_t old = 0;
    int leader = 0;
    if (valid) {
      leader = __ffsll((unsigned long long)peers) - 1;
      if (lane == leader) {
        old = my_cnt[d];
        my_cnt[d] = old + (uint32_t)__popcll(peers);
      }
    }
    old = __shfl(old, leader);
    rank[i] = old + (uint32_t)__popcll(peers & ((1ULL << lane) - 1));
    __builtin_amdgcn_wave_barrier();
  }
  __syncthreads();
  // thread t owns digits t*DPT .. t*DPT+DPT-1: totals over the waves; cnt becomes each
  // wave's offset inside the digit
  uint32_t tot[kDigitsPerThread];
  uint32_t tsum = 0;
#pragma unroll
  for (int j = 0; j < kDigitsPerThread; ++j) {
    const int d = tid * kDigitsPerThread + j;
    tot[j] = 0;
    if (d < radix) {
      uint32_t run = 0;
      for (int w = 0; w < kBlock / 64; ++w) {
        const uint32_t c = cnt[w][d];
        cnt[w][d] = run;
        run += c;
      }
      tot[j] = run;
    }
    tsum += tot[j];
  }
  uint32_t total;
  uint32_t ex = dmt::block_exclusive_scan<kBlock / 64>(tsum, sm, total);
#pragma unroll
  for (int j = 0; j < kDigitsPerThread; ++j) {
    const int d = tid * kDigitsPerThread + j;
    if (d < radix) {
      tile_start[d] = ex;
      // hist holds where this block's first record of digit d goes
      gbase[d] = hist[(int64_t)blockIdx.x * kMaxRadix + d] - ex;
    }
    ex += tot[j];
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < kSortItems; ++i) {
    const int q = wave * (kSortItems * 64) + i * 64 + lane;
    if (q < n_tile) {
      const uint32_t d = sort_digit(rec[i], sb.row_base, shift, mask);
      buf[tile_start[d] + cnt[wave][d] + rank[i]] = rec[i];
    }
  }
  __syncthreads();
  for (int q = tid; q < n_tile; q += kBlock) {
    const uint64_t r = buf[q];
    out[gbase[sort_digit(r, sb.row_base, shift, mask)] + (uint32_t)q] = r;
  }
}

// ------------------------------------------------- run heads, segment offsets

// Run-head flags of the 1024 consecutive records a wave owns inside its block's
// tile, as 16 ballots (iteration i covers records i*64 .. i*64+63, one per lane,
// so every load is one coalesced 512-byte line set).  Returns the head count.
__device__ __forceinline__ uint32_t wave_head_ballots(const uint64_t* __restrict__ pk, int64_t nnz,
                                                      int64_t wave_base,
                                                      uint64_t (&ballots)[kScanItems]) {
  const int lane = threadIdx.x & 63;
  uint32_t count = 0;
  uint32_t carry = 0;                                  // key of the record before this iteration
  if (wave_base > 0 && wave_base <= nnz) carry = (uint32_t)(pk[wave_base - 1] >> 32);
#pragma unroll
  for (int i = 0; i < kScanItems; ++i) {
    const int64_t p = wave_base + i * 64 + lane;
    const uint32_t k = p < nnz ? (uint32_t)(pk[p] >> 32) : 0;
    uint32_t prev = __shfl_up(k, 1);
    if (lane == 0) prev = carry;
    const bool head = p < nnz && (p == 0 || k != prev) && !(k & kInertBit);
    ballots[i] = __ballot(head);
    count += (uint32_t)__popcll(ballots[i]);
    carry = __shfl(k, 63);
  }
  return count;
}

__global__ __launch_bounds__(kBlock) void heads_count(const uint64_t* __restrict__ pk, int64_t nnz,
                                                      uint32_t* __restrict__ blk_heads) {
  __shared__ uint32_t sm[kBlock / 64];
  const int wave = threadIdx.x >> 6;
  uint64_t ballots[kScanItems];
  const uint32_t c = wave_head_ballots(
      pk, nnz, (int64_t)blockIdx.x * kScanTile + (int64_t)wave * (kScanItems * 64), ballots);
  if ((threadIdx.x & 63) == 0) sm[wave] = c;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t t = 0;
    for (int w = 0; w < kBlock / 64; ++w) t += sm[w];
    blk_heads[blockIdx.x] = t;
  }
}

// Single block: exclusive scan of the per-block head counts; total = number of
// distinct keys (the inert key, if present, is counted and removed by the caller
// of num_unique through `has_inert`).
__global__ __launch_bounds__(1024) void heads_scan(uint32_t* __restrict__ blk_heads, int64_t nblk,
                                                   uint32_t* __restrict__ num_unique) {
  __shared__ uint32_t sm[32];
  uint32_t running = 0;
  for (int64_t base = 0; base < nblk; base += 1024) {
    const int64_t i = base + threadIdx.x;
    const uint32_t v = i < nblk ? blk_heads[i] : 0;
    uint32_t total;
    const uint32_t ex = dmt::block_exclusive_scan<16>(v, sm, total);
    if (i < nblk) blk_heads[i] = running + ex;
    running += total;
  }
  if (threadIdx.x == 0) num_unique[0] = running;
}

__global__ __launch_bounds__(kBlock) void heads_write(
    const uint64_t* __restrict__ pk, int64_t nnz, const uint32_t* __restrict__ blk_heads,
    uint32_t* __restrict__ seg_off, uint32_t* __restrict__ tile_first) {
  __shared__ uint32_t sm[kBlock / 64];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int64_t wave_base = (int64_t)blockIdx.x * kScanTile + (int64_t)wave * (kScanItems * 64);
  uint64_t ballots[kScanItems];
  const uint32_t c = wave_head_ballots(pk, nnz, wave_base, ballots);
  if (lane == 0) sm[wave] = c;
  __syncthreads();
  uint32_t before = blk_heads[blockIdx.x];              // run heads before this wave's records
  for (int w = 0; w < wave; ++w) before += sm[w];
  const uint64_t lt = (1ULL << lane) - 1;
#pragma unroll
  for (int i = 0; i < kScanItems; ++i) {
    const int64_t p = wave_base + i * 64 + lane;
    const uint32_t mine = before + (uint32_t)__popcll(ballots[i] & lt);   // heads before p
    const bool head = (ballots[i] >> lane) & 1;
    if (p < nnz) {
      if ((p & (kReduceTile - 1)) == 0) tile_first[p / kReduceTile] = mine;
      if (head) seg_off[mine] = (uint32_t)p;
      if (p == nnz - 1) seg_off[mine + (head ? 1 : 0)] = (uint32_t)nnz;
    }
    before += (uint32_t)__popcll(ballots[i]);
  }
}

// ------------------------------------------- segment reduce + rowwise Adagrad

// One rowwise-Adagrad step on row `row` of table f with summed gradient g (the
// group's lanes hold 4 consecutive columns each; lanes past D hold zeros).
template <int TD, bool NT = false>
__device__ __forceinline__ void apply_row_update(const DmtTableMeta* __restrict__ meta, uint32_t f,
                                                 uint32_t row, float4 g, int gl, int GL, float lr,
                                                 float eps) {
  const int D = meta[f].D;
  float ss = g.x * g.x + g.y * g.y + g.z * g.z + g.w * g.w;
  for (int o = 1; o < GL; o <<= 1) ss += __shfl_xor(ss, o);
  float* state = meta[f].state;
  const float st = dmt::gload(state + row) + ss / (float)D;
  const float step = lr / (sqrtf(st) + eps);
  if (gl * 4 < D) {
    if constexpr (TD == DMT_F32) {
      float4* w = (float4*)((float*)meta[f].table + (int64_t)row * D) + gl;
      float4 v = NT ? dmt::nt_load(w) : dmt::gload(w);
      v.x -= step * g.x; v.y -= step * g.y; v.z -= step * g.z; v.w -= step * g.w;
      if (NT) dmt::nt_store(v, w); else dmt::gstore(v, w);
    } else {
      uint2* w = (uint2*)((uint16_t*)meta[f].table + (int64_t)row * D) + gl;
      const uint2 u = NT ? dmt::nt_load(w) : dmt::gload(w);
      float a, b, c, d;
      dmt::unpack2<TD>(u.x, a, b);
      dmt::unpack2<TD>(u.y, c, d);
      a -= step * g.x; b -= step * g.y; c -= step * g.z; d -= step * g.w;
      const uint2 nu = make_uint2(dmt::pack2<TD>(a, b), dmt::pack2<TD>(c, d));
      if (NT) dmt::nt_store(nu, w); else dmt::gstore(nu, w);
    }
  }
  if (gl == 0) dmt::gstore(st, state + row);
}

__device__ __forceinline__ void store_partial(float* __restrict__ partials, int64_t slot,
                                              int Dmax, int gl, float4 g) {
  if (gl * 4 < Dmax) *((float4*)(partials + slot * Dmax) + gl) = g;
}

// Sum of v over the 2^LG lanes of an aligned lane group; every lane gets the
// total.  Data-parallel-primitive moves inside a 16-lane row, a swizzle across
// rows, a permute across the two 32-lane halves.
template <int LG>
__device__ __forceinline__ float group_sum(float v) {
  auto dpp = [](float x, auto ctrl) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), decltype(ctrl)::value,
                                                      0xf, 0xf, true));
  };
  if constexpr (LG >= 1) v += dpp(v, std::integral_constant<int, 0xB1>());   // quad_perm [1,0,3,2]
  if constexpr (LG >= 2) v += dpp(v, std::integral_constant<int, 0x4E>());   // quad_perm [2,3,0,1]
  if constexpr (LG >= 3) v += dpp(v, std::integral_constant<int, 0x141>());  // row_half_mirror
  if constexpr (LG >= 4) v += dpp(v, std::integral_constant<int, 0x140>());  // row_mirror
  if constexpr (LG >= 5)
    v += __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(v), 0x401F));  // lane ^ 16
  if constexpr (LG >= 6) v += __shfl_xor(v, 32);
  return v;
}

// Orders one lane's LDS writes before other lanes' reads of them inside a wave.  The lanes of
// a wave run in lockstep, but to the compiler they are unrelated threads: without this it may
// move a lane's read in front of another lane's write.
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// A lane's four columns of a table row.
template <int TD> struct RowChunk { using type = uint2; static constexpr int bytes = 8; };
template <> struct RowChunk<DMT_F32> { using type = float4; static constexpr int bytes = 16; };

#ifndef DMT_QS
#define DMT_QS 5
#endif
constexpr int kQueueSlots = DMT_QS;
// finished runs parked before their rows are updated: per lane group, and per wave of the
// wave-per-tile kernel (whose slots are half as large)
constexpr int kQueueSlotsWave = 8;
constexpr int kWaveUnroll = 6;                   // gradient rows the wave-per-tile kernel requests at once
static_assert(kReduceUnroll <= kQueueSlots && kWaveUnroll <= kQueueSlotsWave,
              "a step of the walk parks at most as many runs as the queue holds");

// Each group of GL = 2^LG lanes walks one tile of kReduceTile sorted records,
// summing the bags' gradient slices run by run (float32, record order).  Runs
// that lie wholly inside the tile are parked in an LDS queue (their gradient
// sum, row and state address); the queue is drained four rows at a time, so the
// row / state reads of four updates are in flight together instead of one
// dependent read per run.  The piece of a run that continues from the previous
// tile goes to partial slot 2t, the piece of a run that starts here and
// continues into the next tile to slot 2t + 1.
// UD: every table has dim Dmax (no per-record width to pass round).
template <int TD, int LG, bool UD>
__global__ __launch_bounds__(kBlock) void bwd_reduce_update(
    const DmtTableMeta* __restrict__ meta, const uint64_t* __restrict__ pk, int64_t nnz, uint32_t B,
    uint32_t nbags, uint32_t total_rows, const float* __restrict__ grad,
    float* __restrict__ partials, int Dmax, int64_t ntiles, int64_t blocks_per_xcd, float lr,
    float eps, const unsigned long long* __restrict__ err_offsets) {
  if (*err_offsets != ~0ULL) return;              // malformed offsets: the records mean nothing
  constexpr int GL = 1 << LG, NG = kBlock >> LG;
  constexpr int eb = TD == DMT_F32 ? 4 : 2;
  using Chunk = typename RowChunk<TD>::type;
  __shared__ float4 q_g[kQueueSlots][kBlock];
  __shared__ unsigned long long q_rowp[NG][kQueueSlots];
  __shared__ unsigned long long q_stp[NG][kQueueSlots];
  __shared__ int q_D[NG][kQueueSlots];

  const int group = threadIdx.x >> LG;
  const int64_t tb = (int64_t)(blockIdx.x & 7) * blocks_per_xcd + (blockIdx.x >> 3);
  const int64_t t = tb * NG + group;
  const bool live = t < ntiles;                 // dead groups still take part in wave votes
  const int lane = threadIdx.x & 63;
  const int gl = threadIdx.x & (GL - 1);
  const int lane0 = lane & ~(GL - 1);
  const bool lane_on = gl * 4 < Dmax;
  const float4* __restrict__ grad4 = (const float4*)grad;

  int64_t p0 = 0;
  int n = 0;
  bool cont_prev = false, cont_next = false;
  uint32_t carry = 0;
  if (live) {
    p0 = t * kReduceTile;
    n = (int)min((int64_t)kReduceTile, nnz - p0);
    const uint32_t first_key = (uint32_t)(pk[p0] >> 32);
    if (p0 > 0) {
      carry = (uint32_t)(pk[p0 - 1] >> 32);
      cont_prev = carry == first_key;
    }
    cont_next = p0 + n < nnz && (uint32_t)(pk[p0 + n - 1] >> 32) == (uint32_t)(pk[p0 + n] >> 32);
  }
  bool has_prev = p0 > 0;
  bool run_open = cont_prev, from_left = cont_prev;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  unsigned long long cur_rowp = 0, cur_stp = 0;
  int cur_D = Dmax;
  bool cur_ok = false;
  int qn = 0;

  auto park = [&]() {                            // the open run is complete: queue its update
    if (cur_ok) {
      q_g[qn][threadIdx.x] = acc;
      q_rowp[group][qn] = cur_rowp;
      q_stp[group][qn] = cur_stp;
      if (!UD) q_D[group][qn] = cur_D;
      ++qn;
    }
  };
  auto drain = [&]() {
#pragma unroll
    for (int j0 = 0; j0 < kQueueSlots; j0 += 4) {
      if (!__any(j0 < qn)) break;
      Chunk w[4];
      float st[4];
      Chunk* wp[4];
      float* sp[4];
      int D[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (j0 + u < qn && j0 + u < kQueueSlots) {
          D[u] = UD ? Dmax : q_D[group][j0 + u];
          wp[u] = (Chunk*)(q_rowp[group][j0 + u]) + gl;
          sp[u] = (float*)(q_stp[group][j0 + u]);
          st[u] = dmt::gload(sp[u]);
          if (gl * 4 < D[u]) w[u] = dmt::gload(wp[u]);
        }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (j0 + u < qn && j0 + u < kQueueSlots) {
          const float4 g = q_g[j0 + u][threadIdx.x];
          const float ss = group_sum<LG>(g.x * g.x + g.y * g.y + g.z * g.z + g.w * g.w);
          const float sn = st[u] + ss * __builtin_amdgcn_rcpf((float)D[u]);
          const float step = lr * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(sn) + eps);
          if (gl * 4 < D[u]) {
            if constexpr (TD == DMT_F32) {
              float4 v = w[u];
              v.x -= step * g.x; v.y -= step * g.y; v.z -= step * g.z; v.w -= step * g.w;
              dmt::gstore(v, wp[u]);
            } else {
              float a, b, c, d;
              dmt::unpack2<TD>(w[u].x, a, b);
              dmt::unpack2<TD>(w[u].y, c, d);
              a -= step * g.x; b -= step * g.y; c -= step * g.z; d -= step * g.w;
              dmt::gstore(make_uint2(dmt::pack2<TD>(a, b), dmt::pack2<TD>(c, d)), wp[u]);
            }
          }
          if (gl == 0) dmt::gstore(sn, sp[u]);
        }
      }
    }
    qn = 0;
  };

  for (int sub = 0; sub < kReduceTile; sub += GL) {
    const int cnt = min(GL, n - sub);            // <= 0 once this group's tile is done
    if (!__any(cnt > 0)) break;
    // every lane prepares its own record: gradient offset, row and state address
    uint32_t key_l = total_rows, goff4_l = 0xffffffffu;
    unsigned long long rowp_l = 0, stp_l = 0;
    int D_l = 0;
    if (gl < cnt) {
      const uint64_t r = pk[p0 + sub + gl];
      const uint32_t k = (uint32_t)(r >> 32), bag = (uint32_t)r;
      if (k < total_rows && bag < nbags) {
        const uint32_t f = bag / B, b = bag - f * B;
        const DmtTableMeta& m = meta[f];
        const int64_t row = (int64_t)k - m.row_base;
        if (row >= 0 && row < m.rows) {            // key and bag agree on the table
          key_l = k;
          D_l = m.D;
          goff4_l = (uint32_t)(((int64_t)B * m.out_prefix + (int64_t)b * m.tower_width + m.col_off) >> 2);
          rowp_l = (unsigned long long)((const char*)m.table + row * D_l * eb);
          stp_l = (unsigned long long)(m.state + row);
        }
      }
    }
    // run heads of this sub-round as a bit mask, one bit per record
    uint32_t prev = __shfl_up(key_l, 1, GL);
    bool head_l = gl < cnt;
    if (gl == 0) head_l = head_l && (!has_prev || key_l != carry);
    else head_l = head_l && key_l != prev;
    const unsigned long long hm = __ballot(head_l);
    const unsigned long long gm = LG == 6 ? hm : ((hm >> lane0) & ((1ULL << (GL & 63)) - 1));
    if (cnt > 0) {
      carry = __shfl(key_l, lane0 + cnt - 1);
      has_prev = true;
    }

    for (int i0 = 0; i0 < GL; i0 += kReduceUnroll) {
      if (!__any(i0 < cnt)) break;
      float4 g[kReduceUnroll];
#pragma unroll
      for (int u = 0; u < kReduceUnroll; ++u) {
        const int src = lane0 + ((i0 + u) & (GL - 1));
        const uint32_t go = __shfl(goff4_l, src);
        // (every lane takes part in the exchange: a lane that is off would hand out nothing,
        // and the lanes past the widest row hold records like any other)
        const int D_src = UD ? Dmax : __shfl(D_l, src);
        const bool on = lane_on && i0 + u < cnt && go != 0xffffffffu && gl * 4 < D_src;
        g[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (on) g[u] = grad4[(size_t)go + gl];
      }
#pragma unroll
      for (int u = 0; u < kReduceUnroll; ++u) {
        const int i = i0 + u;
        const int src = lane0 + (i & (GL - 1));
        if (i < cnt) {
          if ((gm >> i) & 1) {                     // a run starts at this record
            if (run_open) {
              if (from_left) store_partial(partials, 2 * t, Dmax, gl, acc);
              else park();
            }
            from_left = false;
            run_open = true;
            acc = make_float4(0.f, 0.f, 0.f, 0.f);
            cur_rowp = __shfl(rowp_l, src);
            cur_stp = __shfl(stp_l, src);
            cur_ok = __shfl(key_l, src) < total_rows;
            if (!UD) cur_D = __shfl(D_l, src);
          }
          acc.x += g[u].x; acc.y += g[u].y; acc.z += g[u].z; acc.w += g[u].w;
        }
      }
      if (__any(qn > kQueueSlots - kReduceUnroll)) drain();
    }
  }
  if (run_open) {
    if (from_left) store_partial(partials, 2 * t, Dmax, gl, acc);
    else if (cont_next) { if (cur_ok) store_partial(partials, 2 * t + 1, Dmax, gl, acc); }
    else park();
  }
  drain();
}

// The same tile walk for wide rows (64 < Dmax <= 256), one WAVE per tile: the 64
// lanes hold EPL = Dmax/64 columns each, so every per-record decision (run head,
// tile end, queue state) is wave-uniform and lives in scalar registers: record
// fields are fetched with v_readlane instead of ds_bpermute, branches are
// scalar, and the two half-waves never diverge.  Same queue-and-drain scheme,
// same partial-slot protocol, same float32 summation order as bwd_reduce_update.
template <int EPL> struct LaneVec;
template <> struct LaneVec<1> { using type = float; };
template <> struct LaneVec<2> { using type = float2; };
template <> struct LaneVec<4> { using type = float4; };

template <int EPL> __device__ __forceinline__ void lv_zero(typename LaneVec<EPL>::type& a) {
  if constexpr (EPL == 1) a = 0.f;
  else if constexpr (EPL == 2) a = make_float2(0.f, 0.f);
  else a = make_float4(0.f, 0.f, 0.f, 0.f);
}
template <int EPL>
__device__ __forceinline__ void lv_add(typename LaneVec<EPL>::type& a,
                                       const typename LaneVec<EPL>::type& b) {
  if constexpr (EPL == 1) a += b;
  else if constexpr (EPL == 2) { a.x += b.x; a.y += b.y; }
  else { a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w; }
}
template <int EPL> __device__ __forceinline__ float lv_sumsq(const typename LaneVec<EPL>::type& a) {
  if constexpr (EPL == 1) return a * a;
  else if constexpr (EPL == 2) return a.x * a.x + a.y * a.y;
  else return a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
}

// row[lane*EPL .. +EPL) -= step * g, in the table's element type
template <int TD, int EPL>
__device__ __forceinline__ void lane_row_update(void* rowp, int lane,
                                                const typename LaneVec<EPL>::type& g, float step,
                                                const void* loaded) {
  if constexpr (TD == DMT_F32) {
    using V = typename LaneVec<EPL>::type;
    V v = *(const V*)loaded;
    if constexpr (EPL == 1) v -= step * g;
    else if constexpr (EPL == 2) { v.x -= step * g.x; v.y -= step * g.y; }
    else { v.x -= step * g.x; v.y -= step * g.y; v.z -= step * g.z; v.w -= step * g.w; }
    dmt::gstore(v, (V*)rowp + lane);
  } else if constexpr (EPL == 1) {
    const uint16_t u = *(const uint16_t*)loaded;
    float a = TD == DMT_F16 ? dmt::f16_bits_to_f32(u) : dmt::bf16_lo(u);
    a -= step * g;
    dmt::gstore((uint16_t)(TD == DMT_F16 ? dmt::f32_to_f16_bits(a) : dmt::f32_to_bf16_bits(a)),
                (uint16_t*)rowp + lane);
  } else if constexpr (EPL == 2) {
    float a, b;
    dmt::unpack2<TD>(*(const uint32_t*)loaded, a, b);
    a -= step * g.x; b -= step * g.y;
    dmt::gstore(dmt::pack2<TD>(a, b), (uint32_t*)rowp + lane);
  } else {
    const uint2 u = *(const uint2*)loaded;
    float a, b, c, d;
    dmt::unpack2<TD>(u.x, a, b);
    dmt::unpack2<TD>(u.y, c, d);
    a -= step * g.x; b -= step * g.y; c -= step * g.z; d -= step * g.w;
    dmt::gstore(make_uint2(dmt::pack2<TD>(a, b), dmt::pack2<TD>(c, d)), (uint2*)rowp + lane);
  }
}

template <int TD, int EPL> struct LaneChunk {            // a lane's EPL elements of a table row
  using type = typename LaneVec<EPL>::type;
};
template <int EPL> struct LaneChunk<DMT_F16, EPL> {
  using type = std::conditional_t<EPL == 1, uint16_t, std::conditional_t<EPL == 2, uint32_t, uint2>>;
};
template <int EPL> struct LaneChunk<DMT_BF16, EPL> {
  using type = typename LaneChunk<DMT_F16, EPL>::type;
};

__device__ __forceinline__ unsigned long long readlane64(unsigned long long v, int l) {
  const uint32_t lo = __builtin_amdgcn_readlane((uint32_t)v, l);
  const uint32_t hi = __builtin_amdgcn_readlane((uint32_t)(v >> 32), l);
  return ((unsigned long long)hi << 32) | lo;
}

template <int TD, int EPL, bool UD>
__global__ __launch_bounds__(kBlock) void bwd_reduce_update_wave(
    const DmtTableMeta* __restrict__ meta, const uint64_t* __restrict__ pk, int64_t nnz, uint32_t B,
    uint32_t nbags, uint32_t total_rows, const float* __restrict__ grad,
    float* __restrict__ partials, int Dmax, int64_t ntiles, int64_t blocks_per_xcd, float lr,
    float eps, const unsigned long long* __restrict__ err_offsets) {
  if (*err_offsets != ~0ULL) return;              // malformed offsets: the records mean nothing
  constexpr int NW = kBlock / 64;
  constexpr int eb = TD == DMT_F32 ? 4 : 2;
  using Vec = typename LaneVec<EPL>::type;
  using Chunk = typename LaneChunk<TD, EPL>::type;
  __shared__ Vec q_g[kQueueSlotsWave][kBlock];
  __shared__ unsigned long long q_rowp[NW][kQueueSlotsWave + 1];
  __shared__ unsigned long long q_stp[NW][kQueueSlotsWave + 1];
  __shared__ int q_D[NW][kQueueSlotsWave + 1];

  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  const int64_t tb = (int64_t)(blockIdx.x & 7) * blocks_per_xcd + (blockIdx.x >> 3);
  const int64_t t = tb * NW + wave;
  if (t >= ntiles) return;
  const bool lane_on = lane * EPL < Dmax;
  const Vec* __restrict__ gradv = (const Vec*)grad;

  const int64_t p0 = t * kReduceTile;
  const int n = (int)min((int64_t)kReduceTile, nnz - p0);
  const uint32_t first_key = __builtin_amdgcn_readfirstlane((uint32_t)(pk[p0] >> 32));
  uint32_t carry = 0;
  bool cont_prev = false;
  if (p0 > 0) {
    carry = __builtin_amdgcn_readfirstlane((uint32_t)(pk[p0 - 1] >> 32));
    cont_prev = carry == first_key;
  }
  bool cont_next = false;
  if (p0 + n < nnz)
    cont_next = __builtin_amdgcn_readfirstlane((uint32_t)(pk[p0 + n - 1] >> 32)) ==
                __builtin_amdgcn_readfirstlane((uint32_t)(pk[p0 + n] >> 32));
  bool has_prev = p0 > 0;
  bool run_open = cont_prev, from_left = cont_prev;
  Vec acc;
  lv_zero<EPL>(acc);
  bool cur_ok = false;
  int qn = 0;

  auto store_part = [&](int64_t slot) {
    if (lane_on) ((Vec*)(partials + slot * Dmax))[lane] = acc;
  };
  // the open run's row / state address sit in queue slot qn already (its head lane put
  // them there); parking adds the gradient sum and commits the slot
  auto park = [&]() {
    if (cur_ok) {
      q_g[qn][threadIdx.x] = acc;
      ++qn;
    }
  };
  auto drain = [&]() {
    const int open_slot = qn;                      // may hold the open run's addresses
    wave_lds_sync();                               // the head lanes' addresses, the parked sums
    if constexpr (EPL == 2) {
      // two parked rows per step: lanes 0-31 take one, lanes 32-63 the next (4 columns a lane)
      using Chunk2 = typename RowChunk<TD>::type;
      const int half = lane >> 5, hl = lane & 31;
#pragma unroll
      for (int j0 = 0; j0 < kQueueSlotsWave; j0 += 8) {
        if (j0 >= qn) break;
        Chunk2 w[4];
        float st[4];
        Chunk2* wp[4];
        float* sp[4];
        int D[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int j = j0 + 2 * u + half;
          if (j < qn && j < kQueueSlotsWave) {
            D[u] = UD ? Dmax : q_D[wave][j];
            wp[u] = (Chunk2*)q_rowp[wave][j] + hl;
            sp[u] = (float*)q_stp[wave][j];
            // row and state are touched once per call: keep them from evicting gradient slices
            st[u] = dmt::nt_load(sp[u]);
            if (hl * 4 < D[u]) w[u] = dmt::nt_load(wp[u]);
          }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int j = j0 + 2 * u + half;
          if (j < qn && j < kQueueSlotsWave) {
            const float4 g = ((const float4*)&q_g[j][wave * 64])[hl];
            const float ss = group_sum<5>(g.x * g.x + g.y * g.y + g.z * g.z + g.w * g.w);
            const float sn = st[u] + ss * __builtin_amdgcn_rcpf((float)D[u]);
            const float step = lr * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(sn) + eps);
            if (hl * 4 < D[u]) {
              if constexpr (TD == DMT_F32) {
                float4 v = w[u];
                v.x -= step * g.x; v.y -= step * g.y; v.z -= step * g.z; v.w -= step * g.w;
                dmt::nt_store(v, wp[u]);
              } else {
                float a, b, c, d;
                dmt::unpack2<TD>(w[u].x, a, b);
                dmt::unpack2<TD>(w[u].y, c, d);
                a -= step * g.x; b -= step * g.y; c -= step * g.z; d -= step * g.w;
                dmt::nt_store(make_uint2(dmt::pack2<TD>(a, b), dmt::pack2<TD>(c, d)), wp[u]);
              }
            }
            if (hl == 0) dmt::nt_store(sn, sp[u]);
          }
        }
      }
    } else {
#pragma unroll
      for (int j0 = 0; j0 < kQueueSlotsWave; j0 += 4) {
        if (j0 >= qn) break;
        Chunk w[4];
        float st[4];
        void* wp[4];
        float* sp[4];
        int D[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (j0 + u < qn && j0 + u < kQueueSlotsWave) {
            D[u] = UD ? Dmax : __builtin_amdgcn_readfirstlane(q_D[wave][j0 + u]);
            wp[u] = (void*)q_rowp[wave][j0 + u];
            sp[u] = (float*)q_stp[wave][j0 + u];
            st[u] = dmt::gload(sp[u]);
            if (lane * EPL < D[u]) w[u] = dmt::gload((const Chunk*)wp[u] + lane);
          }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (j0 + u < qn && j0 + u < kQueueSlotsWave) {
            const Vec g = q_g[j0 + u][threadIdx.x];
            float ss = group_sum<5>(lv_sumsq<EPL>(g));
            ss = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(ss), 0)) +
                 __int_as_float(__builtin_amdgcn_readlane(__float_as_int(ss), 32));
            const float sn = st[u] + ss * __builtin_amdgcn_rcpf((float)D[u]);
            const float step = lr * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(sn) + eps);
            if (lane * EPL < D[u]) lane_row_update<TD, EPL>(wp[u], lane, g, step, &w[u]);
            if (lane == 0) dmt::gstore(sn, sp[u]);
          }
        }
      }
    }
    wave_lds_sync();                               // every lane is done reading the slots
    // an open run keeps its addresses: move them to the slot it will be parked in now
    if (open_slot > 0 && open_slot < kQueueSlotsWave + 1 && run_open && !from_left && lane == 0) {
      q_rowp[wave][0] = q_rowp[wave][open_slot];
      q_stp[wave][0] = q_stp[wave][open_slot];
      if (!UD) q_D[wave][0] = q_D[wave][open_slot];
    }
    qn = 0;
  };

  for (int sub = 0; sub < n; sub += 64) {
    const int cnt = min(64, n - sub);
    uint32_t key_l = total_rows, goff_l = 0xffffffffu;
    unsigned long long rowp_l = 0, stp_l = 0;
    int D_l = 0;
    if (lane < cnt) {
      const uint64_t r = pk[p0 + sub + lane];
      const uint32_t k = (uint32_t)(r >> 32), bag = (uint32_t)r;
      if (k < total_rows && bag < nbags) {
        const uint32_t f = bag / B, b = bag - f * B;
        const DmtTableMeta& m = meta[f];
        const int64_t row = (int64_t)k - m.row_base;
        if (row >= 0 && row < m.rows) {            // key and bag agree on the table
          key_l = k;
          D_l = m.D;
          goff_l = (uint32_t)(((int64_t)B * m.out_prefix + (int64_t)b * m.tower_width + m.col_off) >> 2);
          rowp_l = (unsigned long long)((const char*)m.table + row * D_l * eb);
          stp_l = (unsigned long long)(m.state + row);
        }
      }
    }
    uint32_t prev = __shfl_up(key_l, 1);
    bool head_l = lane < cnt;
    if (lane == 0) head_l = head_l && (!has_prev || key_l != carry);
    else head_l = head_l && key_l != prev;
    const unsigned long long hm = __ballot(head_l);
    carry = __builtin_amdgcn_readlane(key_l, cnt - 1);
    has_prev = true;

    for (int i0 = 0; i0 < cnt; i0 += kWaveUnroll) {
      Vec g[kWaveUnroll];
#pragma unroll
      for (int u = 0; u < kWaveUnroll; ++u) {
        lv_zero<EPL>(g[u]);
        if (i0 + u < cnt) {
          const uint32_t go = __builtin_amdgcn_readlane(goff_l, i0 + u);
          bool on = lane_on && go != 0xffffffffu;
          if (!UD) on = on && lane * EPL < __builtin_amdgcn_readlane(D_l, i0 + u);
          if (on) g[u] = gradv[((size_t)go << 2) / EPL + lane];
        }
      }
#pragma unroll
      for (int u = 0; u < kWaveUnroll; ++u) {
        const int i = i0 + u;
        if (i < cnt) {
          if ((hm >> i) & 1) {                     // a run starts at this record
            if (run_open) {
              if (from_left) store_part(2 * t);
              else park();
            }
            from_left = false;
            run_open = true;
            lv_zero<EPL>(acc);
            cur_ok = __builtin_amdgcn_readlane(key_l, i) < total_rows;
            if (lane == i) {                         // the head record's lane knows the row
              q_rowp[wave][qn] = rowp_l;
              q_stp[wave][qn] = stp_l;
              if (!UD) q_D[wave][qn] = D_l;
            }
          }
          lv_add<EPL>(acc, g[u]);
        }
      }
      if (qn > kQueueSlotsWave - kWaveUnroll) drain();
    }
  }
  if (run_open) {
    if (from_left) store_part(2 * t);
    else if (cont_next) { if (cur_ok) store_part(2 * t + 1); }
    else park();
  }
  drain();
}

// The tile walk for rows of at most 128 columns, built to spend as few instructions per sorted
// record as the hardware allows and to keep a wave's row updates off its critical path.
//  * One wave per tile of kReduceTile records.  A tile is cut into chunks of up to 64
//    consecutive records of ONE table, one record per lane (two chunks, more only where the
//    tile straddles a table boundary), so everything a table decides (row width, gradient
//    base, row and state base) sits in scalar registers.
//  * Each lane reads one record and the record after it; "my key differs from the next one"
//    is one ballot, the mask of run TAILS.  Nothing else about runs is ever computed.
//  * The walk proper is, per record: one v_readlane (its gradient offset), one buffer load of
//    the slice (two columns per lane), two adds, one scalar bit test.  kLeanBatch slices are
//    requested together.
//  * At a tail the sum is parked in a ring of 8 LDS slots, and the lane number of the tail
//    record is packed into a scalar register.  Row updates come off the ring four at a time,
//    ONE instruction for four rows (16 lanes a row, 8 columns a lane), in two halves: at a
//    batch boundary the rows and states of the four oldest parked runs are REQUESTED (the
//    row's key comes from the tail record's lane by ds_bpermute, the addresses from the
//    chunk's scalars); the walk goes on, and at the next boundary the update is computed and
//    stored.  The requests are older than the next batch's slices and the memory counter
//    retires in order, so the wave waits once for both instead of once for each.
//  * Same partial-slot protocol and the same float32 summation order as the other walks.
constexpr int kLeanQueue = 8;
constexpr int kLeanGroup = 4;                    // rows updated by one instruction
constexpr int kLeanBatch = 8;                    // gradient slices requested together
static_assert(kLeanBatch <= kLeanQueue && 64 % kLeanBatch == 0,
              "every record of a batch may end a run, and all of them must fit the emptied ring");

// One wave per block: the waves of a block share nothing, and a block's slots are only handed
// on when its slowest wave is done.  Tile times spread widely (per-tile timestamps on Mid:
// 27 us at the 10th percentile, 73 at the 90th), so with four waves a block a third of the
// wave slots sat waiting for a sibling.  Filling them makes every tile slower instead (mean
// 48 -> 55 us: the gathers, not the number of waves, bound the kernel) and the launch 1 %
// faster.
constexpr int kLeanBlock = 64;
template <int TD>
__global__ __launch_bounds__(kLeanBlock) void bwd_reduce_update_lean(
    const DmtTableMeta* __restrict__ meta, const uint64_t* __restrict__ pk, int64_t nnz, uint32_t B,
    uint32_t bag_mul, uint32_t bag_shift, uint32_t F, const float* __restrict__ grad,
    float* __restrict__ partials, int Dmax, int64_t ntiles, int64_t blocks_per_xcd, float lr,
    float eps, const unsigned long long* __restrict__ err_offsets) {
  if (*err_offsets != ~0ULL) return;              // malformed offsets: the records mean nothing
  constexpr int NW = kLeanBlock / 64;
  constexpr int eb = TD == DMT_F32 ? 4 : 2;
  using Chunk = std::conditional_t<TD == DMT_F32, float4, uint4>;
  constexpr int NC = TD == DMT_F32 ? 2 : 1;
  __shared__ float q_g[NW][kLeanQueue][128];

  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  const int64_t tb = (int64_t)(blockIdx.x & 7) * blocks_per_xcd + (blockIdx.x >> 3);
  const int64_t t = tb * NW + wave;
  if (t >= ntiles) return;
  const int64_t p0 = t * kReduceTile;
  const int n = (int)min((int64_t)kReduceTile, nnz - p0);
  const int qd = lane >> 4, ql = lane & 15;        // row updates: quarter-wave qd, 8 columns from 8 ql
  float* const qbase = &q_g[wave][0][0];

  uint32_t from_left = 0;                          // the open run began in an earlier tile
  if (p0 > 0)
    from_left = __builtin_amdgcn_readfirstlane((uint32_t)(pk[p0 - 1] >> 32)) ==
                __builtin_amdgcn_readfirstlane((uint32_t)(pk[p0] >> 32));
  bool open_end = false;                           // the last record's run goes on in the next tile
  int last_D = 0;
  float2 acc = make_float2(0.f, 0.f);
  // the ring: runs parked, runs whose row and state are requested, runs updated (P >= I >= C,
  // P - C <= 8, I - C <= 4); run e lives in slot e & 7, byte e & 7 of qcodes is 4 x the lane
  // of its tail record
  uint32_t P = 0, I = 0, C = 0;
  uint64_t qcodes = 0;

  for (int pos = 0; pos < n;) {
    const int nrem = n - pos;
    const int64_t idx = p0 + pos + lane;
    uint64_t rec = ~0ULL;
    if (lane < nrem) rec = __builtin_nontemporal_load(pk + idx);
    const uint32_t key_l = (uint32_t)(rec >> 32), bag_l = (uint32_t)rec;
    // the key after each record: the next lane's, and for the last of the (up to) 64 records
    // read here the key of the record behind them, one scalar load
    const int nread = min(nrem, 64);
    const int64_t behind = p0 + pos + nread;
    uint32_t key_behind = ~key_l;                  // differs: the last record of all ends its run
    if (behind < nnz) key_behind = __builtin_amdgcn_readfirstlane((uint32_t)(pk[behind] >> 32));
    const uint32_t down = (uint32_t)__shfl_down((int)key_l, 1);
    const uint32_t next_key_l = lane == nread - 1 ? key_behind : down;
    const uint32_t f_l = B == 1 ? bag_l : (__umulhi(bag_l, bag_mul) >> bag_shift);   // bag / B
    const uint32_t f = __builtin_amdgcn_readfirstlane(f_l);
    const int cnt = __popcll(__ballot(lane < nrem && f_l == f));   // records sorted by table: a prefix
    if (f >= F) {                                  // not a record the key build wrote
      acc = make_float2(0.f, 0.f);
      from_left = 0;
      open_end = false;
      pos += cnt;
      continue;
    }
    const DmtTableMeta& m = meta[f];
    const int D = m.D;
    const uint32_t row_base = (uint32_t)m.row_base, rows = (uint32_t)m.rows;
    const char* const table = (const char*)m.table;
    float* const state = m.state;
    const uint32_t rowbytes = (uint32_t)D * eb;
    const char* const gbase = (const char*)(grad + (int64_t)B * m.out_prefix + m.col_off);
    const uint32_t tw4 = (uint32_t)m.tower_width * 4u;
    // (lanes past the chunk name sample 0's slice: every readlane below yields a valid offset)
    const uint32_t boff_l = lane < cnt ? (bag_l - f * B) * tw4 : 0u;
    const bool in_l = lane < cnt && (key_l - row_base) < rows;     // a row of this table
    const bool tail_l = in_l && next_key_l != key_l;
    const uint64_t tm = __ballot(tail_l);
    const bool last_in = (__ballot(in_l) >> (cnt - 1)) & 1;
    const bool lane_on = lane * 2 < D;
    // lanes past the row's width read the row's first columns instead (every load stays
    // unconditional and in bounds) and park zeros
    const uint32_t lane_off = lane_on ? (uint32_t)lane * 8u : 0u;
    const bool col_on = ql * 8 < D, col_hi = ql * 8 + 4 < D;
    const float inv_D = __builtin_amdgcn_rcpf((float)D);

    // rows and states requested for runs C .. I - 1, one run per quarter-wave
    Chunk pw[NC];
    float pst = 0.f;
    uint32_t prow = 0;
    // Requests the row and the state of runs I .. I + g - 1 (g <= 4).  No load is conditional:
    // a quarter-wave with no run, and lanes past the row's width, read row 0 / the row's
    // first columns.
    auto request = [&](uint32_t g) {
      const uint32_t slot = (I + qd) & 7u;
      const uint32_t code = (uint32_t)(qcodes >> (slot * 8)) & 0xffu;
      const uint32_t k = (uint32_t)__builtin_amdgcn_ds_bpermute((int)code, (int)key_l);
      prow = (uint32_t)qd < g ? k - row_base : 0u;
      const char* wp = table + (uint64_t)prow * rowbytes + (col_on ? ql * (8 * eb) : 0);
      pst = dmt::nt_load(state + prow);
      if constexpr (TD == DMT_F32) {
        pw[0] = dmt::nt_load((const float4*)wp);
        pw[1] = dmt::nt_load((const float4*)wp + (col_hi ? 1 : 0));
      } else {
        pw[0] = dmt::nt_load((const uint4*)wp);
      }
      I += g;
    };
    // Updates the rows requested last: runs C .. I - 1.
    auto update = [&]() {
      const bool on = (uint32_t)qd < I - C;
      wave_lds_sync();                             // the parked sums
      const float4* gq = (const float4*)(qbase + ((C + qd) & 7u) * 128 + ql * 8);
      const float4 g0 = gq[0], g1 = gq[1];
      float ss = g0.x * g0.x + g0.y * g0.y + g0.z * g0.z + g0.w * g0.w + g1.x * g1.x +
                 g1.y * g1.y + g1.z * g1.z + g1.w * g1.w;
      ss = group_sum<4>(ss);
      const float sn = pst + ss * inv_D;
      const float step = lr * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(sn) + eps);
      char* wp = (char*)table + (uint64_t)prow * rowbytes + (col_on ? ql * (8 * eb) : 0);
      if constexpr (TD == DMT_F32) {
        float4 v = pw[0];
        v.x -= step * g0.x; v.y -= step * g0.y; v.z -= step * g0.z; v.w -= step * g0.w;
        if (on && col_on) dmt::nt_store(v, (float4*)wp);
        v = pw[1];
        v.x -= step * g1.x; v.y -= step * g1.y; v.z -= step * g1.z; v.w -= step * g1.w;
        if (on && col_hi) dmt::nt_store(v, (float4*)wp + 1);
      } else {
        float a, b, c, d;
        uint4 o;
        dmt::unpack2<TD>(pw[0].x, a, b);
        dmt::unpack2<TD>(pw[0].y, c, d);
        a -= step * g0.x; b -= step * g0.y; c -= step * g0.z; d -= step * g0.w;
        o.x = dmt::pack2<TD>(a, b);
        o.y = dmt::pack2<TD>(c, d);
        dmt::unpack2<TD>(pw[0].z, a, b);
        dmt::unpack2<TD>(pw[0].w, c, d);
        a -= step * g1.x; b -= step * g1.y; c -= step * g1.z; d -= step * g1.w;
        o.z = dmt::pack2<TD>(a, b);
        o.w = dmt::pack2<TD>(c, d);
        if (on && col_on) dmt::nt_store(o, (uint4*)wp);
      }
      if (on && ql == 0) dmt::nt_store(sn, state + prow);
      wave_lds_sync();                             // every lane is done reading the slots
      C = I;
    };
    // the run that ends at record i of this chunk is complete
    auto close_run = [&](int i) {
      const float2 a = lane_on ? acc : make_float2(0.f, 0.f);
      if (from_left != 0) {
        if (lane * 2 < Dmax) ((float2*)(partials + 2 * t * Dmax))[lane] = a;
        from_left = 0;
      } else {
        const uint32_t sh = (P & 7u) * 8u;
        ((float2*)(qbase + (sh << 4)))[lane] = a;
        qcodes = (qcodes & ~(0xffULL << sh)) | ((uint64_t)(uint32_t)(i * 4) << sh);
        ++P;
      }
      acc = make_float2(0.f, 0.f);
    };
    // This lane's two columns of record i's gradient, as a buffer load: the table's column
    // block is the buffer, the lane's column offset the vector offset and the record's row
    // offset the scalar offset, so a record costs no address arithmetic beyond its v_readlane
    // (and a read past the block would return zeros instead of faulting).
    const __amdgpu_buffer_rsrc_t gbuf = __builtin_amdgcn_make_buffer_rsrc(
        (void*)gbase, 0, (int)((B - 1) * tw4 + (uint32_t)D * 4u), 0x00020000);
    auto slice = [&](int i) {
      const uint32_t bo = __builtin_amdgcn_readlane(boff_l, i);
      const dmt::dmt_u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(gbuf, (int)lane_off, (int)bo, 0);
      return make_float2(__uint_as_float(v.x), __uint_as_float(v.y));
    };

    // Parked runs name lanes of this chunk's key_l and live on its scalars, so the ring is
    // empty when the chunk is left.
    for (int i0 = 0;; i0 += kLeanBatch) {
      const bool more = i0 < cnt;
      const uint32_t tails = (uint32_t)(tm >> (i0 & 63)) & ((1u << kLeanBatch) - 1);
      // what was requested at the last boundary has had a batch's time to arrive
      if (I != C) update();
      // room for this batch's tails (seldom short), or everything out at the chunk's end
      while (more ? P - C + __popc(tails) > (uint32_t)kLeanQueue : P != C) {
        request(min(P - I, (uint32_t)kLeanGroup));
        update();
      }
      if (!more) break;
      if (P - I >= (uint32_t)kLeanGroup) request(kLeanGroup);
      float2 g[kLeanBatch];
      if (i0 + kLeanBatch <= cnt) {
#pragma unroll
        for (int u = 0; u < kLeanBatch; ++u) g[u] = slice(i0 + u);
#pragma unroll
        for (int u = 0; u < kLeanBatch; ++u) {
          acc.x += g[u].x;
          acc.y += g[u].y;
          if ((tails >> u) & 1) close_run(i0 + u);
        }
      } else {
#pragma unroll
        for (int u = 0; u < kLeanBatch; ++u) g[u] = slice((i0 + u) & 63);
#pragma unroll
        for (int u = 0; u < kLeanBatch; ++u) {
          if (i0 + u < cnt) {
            acc.x += g[u].x;
            acc.y += g[u].y;
            if ((tails >> u) & 1) close_run(i0 + u);
          }
        }
      }
    }
    open_end = last_in && !((tm >> (cnt - 1)) & 1);
    last_D = D;
    if (!last_in) {                                // ids outside the table end its records: nothing to carry
      acc = make_float2(0.f, 0.f);
      from_left = 0;
    }
    pos += cnt;
  }
  // (the last chunk's table decides which lanes hold columns; the others hold what they read
  // in place of them and store zeros)
  if (open_end && lane * 2 < Dmax)
    ((float2*)(partials + (2 * t + (from_left ? 0 : 1)) * Dmax))[lane] =
        lane * 2 < last_D ? acc : make_float2(0.f, 0.f);
}

// Table that owns global row id `gid` (row_base has F + 1 ascending entries).
__device__ __forceinline__ uint32_t table_of(const int64_t* __restrict__ row_base, int F,
                                             uint32_t gid) {
  int lo = 0, hi = F;                      // row_base[lo] <= gid < row_base[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if ((int64_t)gid >= row_base[mid]) lo = mid; else hi = mid;
  }
  return (uint32_t)lo;
}

// Rows whose run crosses tile boundaries: the group of the tile where the run
// starts adds the pieces in tile order and applies the update.
// one wave per block: groups are independent, and the group at the head of a long run works
// far longer than its neighbours (50.7 -> 47.4 us on Mid)
constexpr int kFixBlock = 64;
template <int TD>
__global__ __launch_bounds__(kFixBlock) void bwd_fixup_update(
    const DmtTableMeta* __restrict__ meta, uint32_t B, uint32_t nbags,
    const uint64_t* __restrict__ pk, int64_t nnz, uint32_t total_rows,
    const float* __restrict__ partials, int Dmax, int log2_gl, int64_t ntiles, float lr, float eps,
    const unsigned long long* __restrict__ err_offsets) {
  if (*err_offsets != ~0ULL) return;
  const int GL = 1 << log2_gl;
  const int64_t t0 = (int64_t)blockIdx.x * (kFixBlock >> log2_gl) + (threadIdx.x >> log2_gl);
  if (t0 >= ntiles - 1) return;
  const int gl = threadIdx.x & (GL - 1);
  const int64_t p0 = t0 * kReduceTile, p1 = p0 + kReduceTile;    // p1 < nnz here
  // (the four records the decisions below look at are requested together: their latencies
  // would otherwise follow one another in every group)
  const uint64_t r_last = pk[p1 - 1], r_next = pk[p1], r_first = pk[p0], r_before = pk[p0 > 0 ? p0 - 1 : 0];
  const uint32_t k_last = (uint32_t)(r_last >> 32);
  if (k_last != (uint32_t)(r_next >> 32) || k_last >= total_rows) return;
  // the run's table follows from the bag of any of its records (no search through the row bases)
  const uint32_t bag = (uint32_t)r_last;
  if (bag >= nbags) return;
  const uint32_t f = bag / B;
  const int64_t row = (int64_t)k_last - meta[f].row_base;
  if (row < 0 || row >= meta[f].rows) return;      // key and bag disagree: not a row to touch
  const uint32_t k_first = (uint32_t)(r_first >> 32);
  if (k_first == k_last && p0 > 0 && (uint32_t)(r_before >> 32) == k_first) return;
  // last tile the run reaches: the largest t with the run's key at the tile's first record
  // (gallop first: most runs end within a tile or two)
  int64_t t1 = t0 + 1, hi = ntiles;               // holds at t1, fails at hi
  for (int64_t step = 1; t1 + step < hi; step <<= 1) {
    if ((uint32_t)(pk[(t1 + step) * kReduceTile] >> 32) == k_last) t1 += step;
    else { hi = t1 + step; break; }
  }
  while (hi - t1 > 1) {
    const int64_t mid = (t1 + hi) >> 1;
    if ((uint32_t)(pk[mid * kReduceTile] >> 32) == k_last) t1 = mid; else hi = mid;
  }
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  const bool on = gl * 4 < Dmax;
  if (on) acc = *((const float4*)(partials + (2 * t0 + 1) * Dmax) + gl);
  for (int64_t tt = t0 + 1; tt <= t1; tt += 8) {
    float4 g[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      g[q] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (on && tt + q <= t1) g[q] = *((const float4*)(partials + 2 * (tt + q) * Dmax) + gl);
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      acc.x += g[q].x; acc.y += g[q].y; acc.z += g[q].z; acc.w += g[q].w;
    }
  }
  apply_row_update<TD, false>(meta, f, (uint32_t)row, acc, gl, GL, lr, eps);
}

// ------------------------------------------------------------- parity exports

__global__ __launch_bounds__(kBlock) void bwd_export(
    const int64_t* __restrict__ row_base, int F, const uint64_t* __restrict__ pk, int64_t nnz,
    uint32_t total_rows, const uint32_t* __restrict__ seg_off,
    const uint32_t* __restrict__ num_unique_in, int64_t* __restrict__ sorted_keys,
    int32_t* __restrict__ sorted_bag, int64_t* __restrict__ unique_keys,
    int64_t* __restrict__ seg_off_out, int64_t* __restrict__ num_unique) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  const uint32_t U = nnz > 0 ? num_unique_in[0] : 0;   // inert keys were not counted as heads
  if (i == 0 && num_unique) num_unique[0] = U;
  if (i < nnz) {
    const uint32_t gid = (uint32_t)(pk[i] >> 32);
    int64_t key = -1;
    if (gid < total_rows) {
      const uint32_t f = table_of(row_base, F, gid);
      key = ((int64_t)f << 32) | (int64_t)(gid - (uint32_t)row_base[f]);
    }
    if (sorted_keys) sorted_keys[i] = key;
    if (sorted_bag) sorted_bag[i] = (int32_t)(uint32_t)pk[i];
  }
  if (i <= U) {
    if (seg_off_out) seg_off_out[i] = nnz > 0 ? (int64_t)seg_off[i] : 0;
    if (i < U && unique_keys) {
      const uint32_t gid = (uint32_t)(pk[seg_off[i]] >> 32);
      const uint32_t f = table_of(row_base, F, gid);
      unique_keys[i] = ((int64_t)f << 32) | (int64_t)(gid - (uint32_t)row_base[f]);
    }
  }
}

int ilog2_ceil(int64_t x) {
  int l = 0;
  while ((1LL << l) < x) ++l;
  return l;
}

// One launch on `s`, bracketed by the plan's timing events when that kernel family is selected.
template <typename Kernel, typename... Args>
void timed_launch(const dmt_plan* plan, dmt_kernel_id id, hipStream_t s, Kernel kernel,
                  int64_t blocks, int threads, Args... args) {
  DmtScope scope(plan, id, s);
  hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3((unsigned)threads), 0, s, args...);
}

// What the reduce / fix-up launches share.
struct ReduceCall {
  const dmt_plan* plan;
  const BwdWs* w;
  const uint64_t* sorted;
  int64_t nnz, B;
  uint32_t nbags, total_rows;
  const float* grad;
  float lr, eps;
  hipStream_t s;
};

template <int TD, int EPL>
void launch_reduce_wave(const ReduceCall& c) {
  constexpr int kWavesPerBlock = kBlock / 64;
  const int64_t per_xcd = ((c.w->ntiles + kWavesPerBlock - 1) / kWavesPerBlock + 7) / 8;
  auto kernel = c.plan->classes.size() == 1 ? bwd_reduce_update_wave<TD, EPL, true>
                                            : bwd_reduce_update_wave<TD, EPL, false>;
  timed_launch(c.plan, DMT_K_BWD_REDUCE_UPDATE, c.s, kernel, per_xcd * 8, kBlock, c.plan->d_meta,
               c.sorted, c.nnz, (uint32_t)c.B, c.nbags, c.total_rows, c.grad, c.w->partials,
               c.plan->max_dim, c.w->ntiles, per_xcd, c.lr, c.eps, c.plan->d_error + 1);
}

// bag / B for bag < 2^31 as (bag * mul) >> (32 + shift); B = 1 is handled by the kernel.
void bag_divider(uint32_t B, uint32_t& mul, uint32_t& shift) {
  uint32_t l = 0;
  while ((1ull << l) < B) ++l;
  mul = 0;
  shift = 0;
  if (B <= 1) return;
  mul = (uint32_t)(((1ull << (31 + l)) + B - 1) / B);
  shift = l - 1;
}

template <int TD>
void launch_reduce_lean(const ReduceCall& c) {
  constexpr int kWavesPerBlock = kLeanBlock / 64;
  const int64_t per_xcd = ((c.w->ntiles + kWavesPerBlock - 1) / kWavesPerBlock + 7) / 8;
  uint32_t mul, shift;
  bag_divider((uint32_t)c.B, mul, shift);
  timed_launch(c.plan, DMT_K_BWD_REDUCE_UPDATE, c.s, bwd_reduce_update_lean<TD>, per_xcd * 8, kLeanBlock,
               c.plan->d_meta, c.sorted, c.nnz, (uint32_t)c.B, mul, shift, (uint32_t)c.plan->F, c.grad,
               c.w->partials, c.plan->max_dim, c.w->ntiles, per_xcd, c.lr, c.eps,
               c.plan->d_error + 1);
}

template <int TD, int LG>
void launch_reduce_grouped(const ReduceCall& c) {
  const int64_t blocks = (c.w->ntiles + (kBlock >> LG) - 1) / (kBlock >> LG);
  const int64_t per_xcd = (blocks + 7) / 8;
  auto kernel = c.plan->classes.size() == 1 ? bwd_reduce_update<TD, LG, true>
                                            : bwd_reduce_update<TD, LG, false>;
  timed_launch(c.plan, DMT_K_BWD_REDUCE_UPDATE, c.s, kernel, per_xcd * 8, kBlock, c.plan->d_meta,
               c.sorted, c.nnz, (uint32_t)c.B, c.nbags, c.total_rows, c.grad, c.w->partials,
               c.plan->max_dim, c.w->ntiles, per_xcd, c.lr, c.eps, c.plan->d_error + 1);
}

// Segment reduce + row update, then the rows whose run spans tiles.
template <int TD>
void launch_reduce_and_fixup(const ReduceCall& c) {
  const int max_dim = c.plan->max_dim;
  const int log2_gl = std::max(2, ilog2_ceil(max_dim / 4));       // lanes that hold one row
  const bool wave_kernel = (max_dim == 128 || max_dim == 256) && c.plan->sw.bwd_kernel != 2;
  // the lean walk addresses a gradient slice by a 32-bit byte offset inside its tower's block
  int64_t widest = 0;
  for (int32_t t = 0; t < c.plan->T; ++t) widest = std::max<int64_t>(widest, c.plan->tower_width[t]);
  const bool lean = max_dim <= 128 && c.B * widest * 4 < (1LL << 32) && c.plan->sw.bwd_kernel == 0;
  if (lean) {
    launch_reduce_lean<TD>(c);
  } else if (wave_kernel) {
    if (max_dim == 128) launch_reduce_wave<TD, 2>(c); else launch_reduce_wave<TD, 4>(c);
  } else {
    switch (log2_gl) {
      case 2: launch_reduce_grouped<TD, 2>(c); break;
      case 3: launch_reduce_grouped<TD, 3>(c); break;
      case 4: launch_reduce_grouped<TD, 4>(c); break;
      case 5: launch_reduce_grouped<TD, 5>(c); break;
      default: launch_reduce_grouped<TD, 6>(c); break;
    }
  }
  const int64_t blocks = (c.w->ntiles + (kFixBlock >> log2_gl) - 1) / (kFixBlock >> log2_gl);
  timed_launch(c.plan, DMT_K_BWD_FIXUP, c.s, bwd_fixup_update<TD>, blocks, kFixBlock, c.plan->d_meta,
               (uint32_t)c.B, c.nbags, c.sorted, c.nnz, c.total_rows, c.w->partials, max_dim,
               log2_gl, c.w->ntiles, c.lr, c.eps, c.plan->d_error + 1);
}

}  // namespace

extern "C" size_t dmt_bwd_workspace_bytes(const dmt_plan* plan, int64_t B, int64_t nnz) {
  if (!plan || B <= 0 || nnz < 0) return 0;
  return carve(plan, nnz, nullptr).bytes;
}

// Validation and launches of the update; `workspace` is any device memory of at least
// carve().bytes bytes, 256-byte aligned.  Allocates nothing.
static dmt_status bwd_update_run(const dmt_plan* plan, const int32_t* indices,
                                 const int64_t* offsets, int64_t B, int64_t nnz,
                                 const float* grad_pooled, float lr, float eps, void* workspace,
                                 size_t workspace_bytes, void* stream, const dmt_bwd_debug* dbg) {
  if (!plan || !offsets || !grad_pooled) return DMT_EINVAL;
  if (B <= 0 || B > plan->max_batch || nnz < 0 || nnz > plan->max_nnz) return DMT_EINVAL;
  if (nnz > 0 && !indices) return DMT_EINVAL;
  if (!plan->bound || !plan->has_state) return DMT_EINVAL;
  if (!(eps >= 0.f) || lr != lr) return DMT_EINVAL;
  if ((uintptr_t)grad_pooled & 15) return DMT_EINVAL;
  if (plan->max_dim > 256) return DMT_ENOTSUP;          // one float4 per lane, 64 lanes
  if (B * plan->width_prefix[plan->T] >= (1LL << 33)) return DMT_ENOTSUP;   // float4 index in 32 bits
  const BwdWs w = carve(plan, nnz, workspace);
  if (!workspace || ((uintptr_t)workspace & 255)) return DMT_EINVAL;
  if (workspace_bytes < w.bytes) return DMT_ENOMEM;
  hipStream_t s = (hipStream_t)stream;
  const uint32_t total_rows = (uint32_t)plan->total_rows;
  const uint32_t nbags = (uint32_t)((int64_t)plan->F * B);
  const uint64_t* sorted = w.pk_a;

  if (nnz > 0) {
    // keys; bags per block: about 4096 lookups' worth (a power of two, at most kKeysMaxBags)
    const double mean_len = (double)nnz / (double)nbags;
    int log2_bpb = ilog2_ceil((int64_t)(4096.0 / (mean_len > 1.0 ? mean_len : 1.0) + 0.5));
    if (plan->sw.keys_lg >= 0) log2_bpb = plan->sw.keys_lg;
    log2_bpb = log2_bpb < 4 ? 4 : (log2_bpb > 10 ? 10 : log2_bpb);
    const int64_t key_blocks = ((int64_t)nbags + (1 << log2_bpb) - 1) >> log2_bpb;
    timed_launch(plan, DMT_K_BWD_KEYS, s, bwd_build_keys, key_blocks, kBlock, plan->d_meta, indices,
                 offsets, (uint32_t)B, nbags, nnz, (int)plan->F, w.pk_a, log2_bpb, w.seg_begin,
                 w.seg_blk, w.blk_table, plan->row_shards ? nullptr : plan->d_error, plan->d_error + 1);

    // stable LSD radix sort inside every table over the bits a row id of the largest table
    // (or its one-past-the-end inert id) can set
    int64_t max_rows = 0;
    for (int32_t f = 0; f < plan->F; ++f) max_rows = std::max<int64_t>(max_rows, plan->meta[f].rows);
    const int key_bits = ilog2_ceil(max_rows + 1);
    const int passes = (key_bits + kMaxRadixBits - 1) / kMaxRadixBits;
    const int bits_per = (key_bits + passes - 1) / passes;
    uint64_t* src = w.pk_a;
    uint64_t* dst = w.pk_b;
    for (int p = 0; p < passes; ++p) {
      const int shift = p * bits_per;
      const int bits = std::min(bits_per, key_bits - shift);
      timed_launch(plan, DMT_K_BWD_SORT_HIST, s, radix_hist, w.nblk_sort, kBlock, plan->d_meta, src,
                   shift, bits, w.hist, w.seg_begin, w.seg_blk, w.blk_table, (int)plan->F);
      timed_launch(plan, DMT_K_BWD_SORT_SCAN, s, radix_scan, plan->F, kScanThreads, w.hist, bits,
                   w.seg_begin, w.seg_blk);
      timed_launch(plan, DMT_K_BWD_SORT_SCATTER, s, radix_scatter, w.nblk_sort, kBlock, plan->d_meta,
                   src, dst, shift, bits, w.hist, w.seg_begin, w.seg_blk, w.blk_table, (int)plan->F);
      std::swap(src, dst);
    }
    sorted = src;

    const ReduceCall call{plan, &w, sorted, nnz, B, nbags, total_rows, grad_pooled, lr, eps, s};
    switch (plan->table_dtype) {
      case DMT_F32: launch_reduce_and_fixup<DMT_F32>(call); break;
      case DMT_F16: launch_reduce_and_fixup<DMT_F16>(call); break;
      default: launch_reduce_and_fixup<DMT_BF16>(call); break;
    }
  }
  if (dbg && (dbg->sorted_keys || dbg->sorted_bag || dbg->unique_keys || dbg->seg_off ||
              dbg->num_unique)) {
    if (nnz > 0) {
      // run heads -> segment offsets (only the parity exports need them)
      timed_launch(plan, DMT_K_BWD_HEADS, s, heads_count, w.nblk_scan, kBlock, sorted, nnz,
                   w.blk_heads);
      timed_launch(plan, DMT_K_BWD_HEADS, s, heads_scan, 1, 1024, w.blk_heads, w.nblk_scan,
                   w.num_unique);
      timed_launch(plan, DMT_K_BWD_HEADS, s, heads_write, w.nblk_scan, kBlock, sorted, nnz,
                   w.blk_heads, w.seg_off, w.tile_first);
    }
    const int64_t n = nnz + 1;
    hipLaunchKernelGGL(bwd_export, dim3((unsigned)((n + kBlock - 1) / kBlock)), dim3(kBlock), 0, s,
                       plan->d_row_base, plan->F, sorted, nnz, total_rows, w.seg_off, w.num_unique,
                       dbg->sorted_keys, dbg->sorted_bag, dbg->unique_keys, dbg->seg_off,
                       dbg->num_unique);
  }
  return hipGetLastError() == hipSuccess ? DMT_OK : DMT_EHIP;
}

extern "C" dmt_status dmt_tower_lookup_bwd_update(const dmt_plan* plan, const int32_t* indices,
                                                  const int64_t* offsets, int64_t B, int64_t nnz,
                                                  const float* grad_pooled, float lr, float eps,
                                                  void* workspace, size_t workspace_bytes,
                                                  void* stream, const dmt_bwd_debug* dbg) {
  return bwd_update_run(plan, indices, offsets, B, nnz, grad_pooled, lr, eps, workspace,
                        workspace_bytes, stream, dbg);
}

// ------------------------------------------- the update on the library's own scratch memory

// Scratch of dmt_tower_lookup_bwd_update_noalloc: one array per GPU the library runs on, held
// until the process ends.  Host code never uses the array's name as an address: it asks the
// runtime for the array's device address once per device and passes that pointer on.
static __device__ __align__(256) unsigned char scratch[DMT_BWD_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each device, once resolved
}  // namespace

extern "C" size_t dmt_bwd_noalloc_scratch_bytes(void) { return DMT_BWD_NOALLOC_SCRATCH_BYTES; }

extern "C" dmt_status dmt_tower_lookup_bwd_update_noalloc(const dmt_plan* plan,
                                                          const int32_t* indices,
                                                          const int64_t* offsets, int64_t B,
                                                          int64_t nnz, const float* grad_pooled,
                                                          float lr, float eps, void* stream) {
  if (!plan || B <= 0 || nnz < 0) return DMT_EINVAL;
  // the size check comes first: nothing is resolved or launched for a call that cannot fit
  if (carve(plan, nnz, nullptr).bytes > (size_t)DMT_BWD_NOALLOC_SCRATCH_BYTES) return DMT_ENOMEM;
  int dev = -1;
  DMT_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return DMT_ENOTSUP;
  void* ptr = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
      void* p = nullptr;
      DMT_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
      if (!p) return DMT_EHIP;
      g_scratch_ptr[dev] = p;
    }
    ptr = g_scratch_ptr[dev];
  }
  return bwd_update_run(plan, indices, offsets, B, nnz, grad_pooled, lr, eps, ptr,
                        (size_t)DMT_BWD_NOALLOC_SCRATCH_BYTES, stream, nullptr);
}
