// Plan object: the static description of tables and towers (paper Sec. 2.1,
// Sec. 3.1), the tower-major layout arithmetic, and the device-side lookup
// tables the kernels index.
#include <stdlib.h>

#include <algorithm>
#include <new>

#include "dmt_internal.h"

extern "C" const char* dmt_status_str(int32_t status) {
  switch (status) {
    case DMT_OK: return "DMT_OK";
    case DMT_EINVAL: return "DMT_EINVAL";
    case DMT_ENOTSUP: return "DMT_ENOTSUP";
    case DMT_EBOUNDS: return "DMT_EBOUNDS";
    case DMT_ENOMEM: return "DMT_ENOMEM";
    case DMT_EHIP: return "DMT_EHIP";
  }
  return "DMT_UNKNOWN";
}

extern "C" dmt_status dmt_plan_create(dmt_plan** out, int32_t num_tables, const int64_t* rows,
                                      const int32_t* dims, int32_t table_dtype_code,
                                      int32_t num_towers, const int32_t* table_to_tower,
                                      int64_t max_batch, int64_t max_nnz) {
  if (!out) return DMT_EINVAL;
  *out = nullptr;
  if (!rows || !dims || !table_to_tower) return DMT_EINVAL;
  if (num_tables <= 0 || num_tables > DMT_MAX_TABLES) return DMT_EINVAL;
  if (num_towers <= 0 || num_towers > DMT_MAX_TOWERS || num_towers > num_tables) return DMT_EINVAL;
  if (max_batch <= 0 || max_nnz < 0) return DMT_EINVAL;
  if (table_dtype_code != DMT_F32 && table_dtype_code != DMT_F16 && table_dtype_code != DMT_BF16)
    return DMT_EINVAL;
  const dmt_dtype table_dtype = (dmt_dtype)table_dtype_code;
  // bag ids f*B + b and lookup positions are carried in 32 bits by the backward
  if ((int64_t)num_tables * max_batch >= (1LL << 31) || max_nnz >= (1LL << 31)) return DMT_ENOTSUP;
  const int eb = dmt_elt_bytes(table_dtype);
  int64_t total_rows = 0;
  for (int32_t f = 0; f < num_tables; ++f) {
    if (rows[f] <= 0 || dims[f] <= 0) return DMT_EINVAL;
    if (rows[f] >= (1LL << 31)) return DMT_ENOTSUP;
    if (table_to_tower[f] < 0 || table_to_tower[f] >= num_towers) return DMT_EINVAL;
    int64_t rb = (int64_t)dims[f] * eb;
    if (rb % 16 != 0 || rb > 1024) return DMT_ENOTSUP;
    total_rows += rows[f];
  }
  // the backward carries a global row id in 31 bits of its sort key (the top bit is a flag)
  if (total_rows >= (1LL << 31)) return DMT_ENOTSUP;

  return dmt_guard([&]() -> dmt_status {
  dmt_plan* p = new (std::nothrow) dmt_plan();
  if (!p) return DMT_ENOMEM;
  struct Drop {                                   // frees the plan unless it is handed over
    dmt_plan* p;
    ~Drop() { delete p; }
  } drop{p};
  auto env = [](const char* name, int dflt) {
    const char* v = getenv(name);
    return (v && *v) ? atoi(v) : dflt;
  };
  p->sw.tm_big = env("DMT_TM_BIG", 1);
  p->sw.tm_fuse = env("DMT_TM_FUSE", 1);
  p->sw.tm_direct = env("DMT_TM_DIRECT", 1);
  p->sw.tmb_ksplit = env("DMT_TMB_KSPLIT", 0);
  p->sw.bwd_kernel = env("DMT_BWD_KERNEL", 0);
  p->sw.keys_lg = env("DMT_KEYS_LG", -1);
  p->sw.lookup_r = env("DMT_LOOKUP_R", 0);
  p->sw.lookup_bpg = env("DMT_LOOKUP_BPG", 0);
  p->sw.lookup_long = env("DMT_LOOKUP_LONG", -1);
  p->F = num_tables;
  p->T = num_towers;
  p->table_dtype = table_dtype;
  p->max_batch = max_batch;
  p->max_nnz = max_nnz;
  p->total_rows = total_rows;
  p->meta.resize(num_tables);
  p->tower_width.assign(num_towers, 0);
  p->tower_ntab.assign(num_towers, 0);
  p->tower_first_table.assign(num_towers, -1);
  p->tower_uniform_dim.assign(num_towers, 0);
  p->width_prefix.assign(num_towers + 1, 0);
  int64_t rb = 0;
  for (int32_t f = 0; f < num_tables; ++f) {
    DmtTableMeta& m = p->meta[f];
    const int32_t t = table_to_tower[f];
    m.table = nullptr;
    m.state = nullptr;
    m.rows = rows[f];
    m.row_begin = 0;
    m.row_base = rb;
    rb += rows[f];
    m.D = dims[f];
    m.tower = t;
    m.col_off = p->tower_width[t];       // tables visited in ascending id = slot order
    p->tower_width[t] += dims[f];
    if (p->tower_ntab[t] == 0) {
      p->tower_first_table[t] = f;
      p->tower_uniform_dim[t] = dims[f];
    } else if (p->tower_uniform_dim[t] != dims[f]) {
      p->tower_uniform_dim[t] = 0;
    }
    p->tower_ntab[t]++;
    p->max_dim = std::max(p->max_dim, dims[f]);
  }
  for (int32_t t = 0; t < num_towers; ++t) {
    if (p->tower_ntab[t] == 0) return DMT_EINVAL;
    p->width_prefix[t + 1] = p->width_prefix[t] + p->tower_width[t];
  }
  for (int32_t f = 0; f < num_tables; ++f) {
    p->meta[f].tower_width = p->tower_width[p->meta[f].tower];
    p->meta[f].out_prefix = p->width_prefix[p->meta[f].tower];
  }
  // group tables by dim, classes in ascending dim, tables in ascending id
  std::vector<int32_t> ds(dims, dims + num_tables);
  std::sort(ds.begin(), ds.end());
  ds.erase(std::unique(ds.begin(), ds.end()), ds.end());
  for (int32_t d : ds) {
    DmtDimClass c;
    c.D = d;
    c.first = (int32_t)p->class_tables.size();
    for (int32_t f = 0; f < num_tables; ++f)
      if (dims[f] == d) p->class_tables.push_back(f);
    c.num_tables = (int32_t)p->class_tables.size() - c.first;
    p->classes.push_back(c);
  }
  drop.p = nullptr;
  *out = p;
  return DMT_OK;
  });
}

static void release_device(dmt_plan* p) {
  for (auto& r : p->prof.pending) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
  for (auto& e : p->prof.pool) (void)hipEventDestroy(e);
  p->prof.pending.clear();
  p->prof.pool.clear();
  if (p->d_meta) (void)hipFree(p->d_meta);
  if (p->d_class_tables) (void)hipFree(p->d_class_tables);
  if (p->d_row_base) (void)hipFree(p->d_row_base);
  if (p->d_error) (void)hipFree(p->d_error);
  p->d_meta = nullptr;
  p->d_class_tables = nullptr;
  p->d_row_base = nullptr;
  p->d_error = nullptr;
  p->bound = false;
}

extern "C" void dmt_plan_destroy(dmt_plan* plan) {
  if (!plan) return;
  release_device(plan);
  delete plan;
}

extern "C" dmt_status dmt_plan_layout(const dmt_plan* plan, int64_t B, int64_t* tower_base,
                                      int32_t* tower_width, int32_t* col_off) {
  if (!plan || B < 0) return DMT_EINVAL;
  if (tower_base)
    for (int32_t t = 0; t <= plan->T; ++t) tower_base[t] = B * plan->width_prefix[t];
  if (tower_width)
    for (int32_t t = 0; t < plan->T; ++t) tower_width[t] = plan->tower_width[t];
  if (col_off)
    for (int32_t f = 0; f < plan->F; ++f) col_off[f] = plan->meta[f].col_off;
  return DMT_OK;
}

extern "C" dmt_status dmt_plan_bind(dmt_plan* plan, const void* const* tables,
                                    float* const* adagrad_state) {
  if (!plan || !tables) return DMT_EINVAL;
  for (int32_t f = 0; f < plan->F; ++f) {
    if (!tables[f] || ((uintptr_t)tables[f] & 15)) return DMT_EINVAL;
    if (adagrad_state && (!adagrad_state[f] || ((uintptr_t)adagrad_state[f] & 3))) return DMT_EINVAL;
  }
  for (int32_t f = 0; f < plan->F; ++f) {
    plan->meta[f].table = tables[f];
    plan->meta[f].state = adagrad_state ? adagrad_state[f] : nullptr;
  }
  plan->has_state = adagrad_state != nullptr;
  if (!plan->d_meta) {
    DMT_HIP_TRY(hipMalloc((void**)&plan->d_meta, sizeof(DmtTableMeta) * plan->F));
    DMT_HIP_TRY(hipMalloc((void**)&plan->d_class_tables, sizeof(int32_t) * plan->F));
    DMT_HIP_TRY(hipMalloc((void**)&plan->d_row_base, sizeof(int64_t) * (plan->F + 1)));
    DMT_HIP_TRY(hipMalloc((void**)&plan->d_error, 2 * sizeof(unsigned long long)));
  }
  std::vector<int64_t> row_base;
  try {
    row_base.resize(plan->F + 1);
  } catch (...) {
    return DMT_ENOMEM;
  }
  for (int32_t f = 0; f < plan->F; ++f) row_base[f] = plan->meta[f].row_base;
  row_base[plan->F] = plan->total_rows;
  const unsigned long long none[2] = {~0ULL, ~0ULL};
  DMT_HIP_TRY(hipMemcpy(plan->d_meta, plan->meta.data(), sizeof(DmtTableMeta) * plan->F,
                        hipMemcpyHostToDevice));
  DMT_HIP_TRY(hipMemcpy(plan->d_class_tables, plan->class_tables.data(),
                        sizeof(int32_t) * plan->F, hipMemcpyHostToDevice));
  DMT_HIP_TRY(hipMemcpy(plan->d_row_base, row_base.data(), sizeof(int64_t) * (plan->F + 1),
                        hipMemcpyHostToDevice));
  DMT_HIP_TRY(hipMemcpy(plan->d_error, none, sizeof(none), hipMemcpyHostToDevice));
  plan->bound = true;
  return DMT_OK;
}

extern "C" dmt_status dmt_plan_set_row_shards(dmt_plan* plan, const int64_t* row_begin) {
  if (!plan || !row_begin) return DMT_EINVAL;
  // a local row is addressed as id - row_begin, which must stay within an int32 id
  for (int32_t f = 0; f < plan->F; ++f)
    if (row_begin[f] < 0 || row_begin[f] + plan->meta[f].rows > (1LL << 31)) return DMT_EINVAL;
  for (int32_t f = 0; f < plan->F; ++f) plan->meta[f].row_begin = row_begin[f];
  plan->row_shards = true;
  if (plan->bound)
    DMT_HIP_TRY(hipMemcpy(plan->d_meta, plan->meta.data(), sizeof(DmtTableMeta) * plan->F,
                          hipMemcpyHostToDevice));
  return DMT_OK;
}

extern "C" dmt_status dmt_last_device_error(const dmt_plan* plan, void* stream,
                                            int64_t* bad_position) {
  if (!plan || !bad_position) return DMT_EINVAL;
  *bad_position = -1;
  if (!plan->bound) return DMT_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  // [0] smallest position of an id outside its table, [1] first bag whose offsets are malformed
  unsigned long long v[2] = {~0ULL, ~0ULL};
  const unsigned long long none[2] = {~0ULL, ~0ULL};
  DMT_HIP_TRY(hipMemcpyAsync(v, plan->d_error, sizeof(v), hipMemcpyDeviceToHost, s));
  DMT_HIP_TRY(hipStreamSynchronize(s));
  if (v[0] == none[0] && v[1] == none[1]) return DMT_OK;
  DMT_HIP_TRY(hipMemcpyAsync(plan->d_error, none, sizeof(none), hipMemcpyHostToDevice, s));
  DMT_HIP_TRY(hipStreamSynchronize(s));
  if (v[1] != none[1]) {
    *bad_position = (int64_t)v[1];
    return DMT_EINVAL;
  }
  *bad_position = (int64_t)v[0];
  return DMT_EBOUNDS;
}

extern "C" const char* dmt_kernel_name(int32_t id) {
  static const char* names[DMT_K_COUNT] = {
      "lookup_fwd", "tm_dots", "tm_pack_w", "tm_gemm", "bwd_build_keys", "radix_hist",
      "radix_scan", "radix_scatter", "bwd_heads", "bwd_reduce_update", "bwd_fixup_update",
      "tm_bwd_gemm", "tm_bwd_aux", "tp_gram", "tp_finish"};
  return (id >= 0 && id < DMT_K_COUNT) ? names[id] : "?";
}

static void drop_pending(DmtProfile& pr) {
  for (auto& r : pr.pending) { pr.pool.push_back(r.a); pr.pool.push_back(r.b); }
  pr.pending.clear();
}

extern "C" dmt_status dmt_profile_enable(dmt_plan* plan, uint32_t kernel_mask) {
  if (!plan) return DMT_EINVAL;
  (void)hipDeviceSynchronize();
  drop_pending(plan->prof);
  plan->prof.mask = kernel_mask;
  return DMT_OK;
}

extern "C" dmt_status dmt_profile_read(dmt_plan* plan, void* stream, double* total_ms,
                                       int64_t* launches) {
  if (!plan || !total_ms || !launches) return DMT_EINVAL;
  for (int i = 0; i < DMT_K_COUNT; ++i) { total_ms[i] = 0.0; launches[i] = 0; }
  DMT_HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
  for (auto& r : plan->prof.pending) {
    float ms = 0.f;
    DMT_HIP_TRY(hipEventElapsedTime(&ms, r.a, r.b));
    total_ms[r.id] += ms;
    launches[r.id] += 1;
  }
  drop_pending(plan->prof);
  return DMT_OK;
}

__global__ __launch_bounds__(256) void dmt_copy_kernel(uint4* __restrict__ dst,
                                                       const uint4* __restrict__ src, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256)
    dst[i] = src[i];
}

// Rows of `row_bytes` bytes (16 << log2_lpr) gathered by id, 64 >> log2_lpr rows per wave
// instruction and eight instructions in flight per wave, nothing else: what random row reads
// reach on the machine at hand.  Every lane folds what it read into one word and stores it at
// the end, so that the loads cannot be dropped.
__global__ __launch_bounds__(256) void dmt_gather_kernel(const char* __restrict__ table, int64_t rows,
                                                         int log2_lpr, const int32_t* __restrict__ ids,
                                                         int64_t n, uint4* __restrict__ out) {
  constexpr int kInFlight = 8;
  const int lane = threadIdx.x & 63;
  const int rpi = 64 >> log2_lpr;                             // rows per instruction
  const int sub = lane >> log2_lpr, chunk = lane & ((1 << log2_lpr) - 1);
  const int64_t wave = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 6;
  const int64_t nwaves = ((int64_t)gridDim.x * 256) >> 6;
  const int64_t per_step = (int64_t)rpi * kInFlight;
  uint4 acc = make_uint4(0, 0, 0, 0);
  for (int64_t base = wave * per_step; base < n; base += nwaves * per_step) {
    uint4 v[kInFlight];
#pragma unroll
    for (int u = 0; u < kInFlight; ++u) {
      const int64_t i = base + (int64_t)u * rpi + sub;
      int64_t r = i < n ? (int64_t)ids[i] : 0;
      r = (uint64_t)r < (uint64_t)rows ? r : 0;               // an id outside the table reads row 0
      v[u] = make_uint4(0, 0, 0, 0);
      if (i < n) v[u] = *(const uint4*)(table + ((r << log2_lpr) + chunk) * 16);
    }
#pragma unroll
    for (int u = 0; u < kInFlight; ++u) {
      acc.x ^= v[u].x; acc.y ^= v[u].y; acc.z ^= v[u].z; acc.w ^= v[u].w;
    }
  }
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = acc;
}

extern "C" dmt_status dmt_calibration_gather(const void* table, int64_t rows, int32_t row_bytes,
                                             const int32_t* ids, int64_t n, void* out,
                                             void* stream) {
  if (!table || !ids || !out || rows <= 0 || n < 0 || ((uintptr_t)table & 15) || ((uintptr_t)out & 15))
    return DMT_EINVAL;
  int log2_lpr = 0;
  while ((16 << log2_lpr) < row_bytes) ++log2_lpr;
  if (row_bytes < 16 || row_bytes > 1024 || (16 << log2_lpr) != row_bytes) return DMT_EINVAL;
  if (n == 0) return DMT_OK;
  hipLaunchKernelGGL(dmt_gather_kernel, dim3(DMT_CALIBRATION_GATHER_BLOCKS), dim3(256), 0,
                     (hipStream_t)stream, (const char*)table, rows, log2_lpr, ids, n, (uint4*)out);
  return hipGetLastError() == hipSuccess ? DMT_OK : DMT_EHIP;
}

extern "C" dmt_status dmt_calibration_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src || (bytes & 15) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15))
    return DMT_EINVAL;
  if (bytes == 0) return DMT_OK;
  hipLaunchKernelGGL(dmt_copy_kernel, dim3(256 * 16), dim3(256), 0, (hipStream_t)stream, (uint4*)dst,
                     (const uint4*)src, bytes / 16);
  return hipGetLastError() == hipSuccess ? DMT_OK : DMT_EHIP;
}
