// Internal declarations shared by the library's translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "dmt.h"

#define DMT_HIP_TRY(expr)                     \
  do {                                        \
    hipError_t e_ = (expr);                   \
    if (e_ != hipSuccess) return DMT_EHIP;    \
  } while (0)

// No exception crosses the C boundary: an entry point whose host side allocates (std::vector)
// runs its body through one of these.
#include <new>
template <typename Body>
static inline dmt_status dmt_guard(Body body) {
  try {
    return body();
  } catch (const std::bad_alloc&) {
    return DMT_ENOMEM;
  } catch (...) {
    return DMT_EINVAL;
  }
}
template <typename Body>
static inline size_t dmt_guard_size(Body body) {
  try {
    return body();
  } catch (...) {
    return 0;
  }
}

// Per-table record the kernels read (device copy lives in the plan).
struct DmtTableMeta {
  const void* table;     // row-major [rows][D]
  float* state;          // [rows] or null
  int64_t rows;
  int64_t row_begin;     // id of the table's first local row (0 unless the table is a row-wise shard)
  int64_t row_base;      // global id of row 0 (prefix sum of rows over tables)
  int64_t out_prefix;    // sum of W_t' over towers before this table's tower; x B = tower base
  int32_t D;
  int32_t tower;
  int32_t col_off;       // first column inside the tower's rows
  int32_t tower_width;   // W_t
};

// Tables that share one embedding dim are launched together.
struct DmtDimClass {
  int32_t D;
  int32_t num_tables;
  int32_t first;         // offset into class_tables
};

// Event pairs around selected launches (dmt_profile_*).
struct DmtProfile {
  struct Rec { hipEvent_t a, b; int id; };
  uint32_t mask = 0;
  std::vector<Rec> pending;
  std::vector<hipEvent_t> pool;
};

// Kernel-choice switches, read from the environment ONCE, when the plan is created (tests reach
// both variants of a choice, sweeps need no rebuild); 0 / -1 = the library's own choice.
struct DmtSwitches {
  int tm_big = 1;        // DMT_TM_BIG=0: every contraction on the 128 x 128 kernel
  int tm_fuse = 1;       // DMT_TM_FUSE=0: dot terms by their own kernel, not inside the projection
  int tm_direct = 1;     // DMT_TM_DIRECT=0: interior launches of the 256 x 256 kernel stage through registers too
  int tmb_ksplit = 0;    // DMT_TMB_KSPLIT=n: slices of every weight gradient
  int bwd_kernel = 0;    // DMT_BWD_KERNEL=1 / 2: the wave-per-tile / lane-group segment reduce
  int keys_lg = -1;      // DMT_KEYS_LG=l: 2^l bags per key-build block
  int lookup_r = 0;      // DMT_LOOKUP_R=r: row slots per bag
  int lookup_bpg = 0;    // DMT_LOOKUP_BPG=n: bags a lane group pools in turn
  int lookup_long = -1;  // DMT_LOOKUP_LONG=n: bags longer than n ids go to whole waves (0: never)
};

struct dmt_plan {
  DmtSwitches sw;
  int32_t F = 0, T = 0;
  dmt_dtype table_dtype = DMT_F32;
  int64_t max_batch = 0, max_nnz = 0;
  std::vector<DmtTableMeta> meta;          // host copy, pointers filled by bind
  std::vector<int32_t> tower_width;        // [T]
  std::vector<int64_t> width_prefix;       // [T+1]
  std::vector<int32_t> tower_ntab;         // [T]
  std::vector<int32_t> tower_first_table;  // [T] lowest table id in the tower
  std::vector<int32_t> tower_uniform_dim;  // [T] common D of the tower's tables, or 0
  std::vector<DmtDimClass> classes;
  std::vector<int32_t> class_tables;       // table ids grouped by class
  int64_t total_rows = 0;
  int32_t max_dim = 0;
  // device side (created by dmt_plan_bind)
  bool bound = false;
  bool has_state = false;
  bool row_shards = false;                 // ids outside a table's rows belong to other shards
  DmtTableMeta* d_meta = nullptr;          // [F]
  int32_t* d_class_tables = nullptr;       // [F]
  int64_t* d_row_base = nullptr;           // [F+1]
  unsigned long long* d_error = nullptr;   // [0] smallest bad id position, [1] first bag with
                                           // malformed offsets; ~0 = none
  mutable DmtProfile prof;
};

// Times everything launched on `s` during its lifetime when family `id` is selected.
struct DmtScope {
  const dmt_plan* p;
  hipStream_t s;
  hipEvent_t b = nullptr;
  DmtScope(const dmt_plan* plan, int id, hipStream_t stream) : p(plan), s(stream) {
    DmtProfile& pr = plan->prof;
    if (!(pr.mask & (1u << id))) return;
    hipEvent_t ev[2];
    for (int i = 0; i < 2; ++i) {
      if (!pr.pool.empty()) { ev[i] = pr.pool.back(); pr.pool.pop_back(); }
      else if (hipEventCreate(&ev[i]) != hipSuccess) return;
    }
    (void)hipEventRecord(ev[0], s);
    pr.pending.push_back({ev[0], ev[1], id});
    b = ev[1];
  }
  ~DmtScope() { if (b) (void)hipEventRecord(b, s); }
};

static inline int dmt_elt_bytes(dmt_dtype t) { return t == DMT_F32 ? 4 : 2; }
static inline size_t dmt_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
