// dmt_tower_module_fwd: the per-tower Tower Module (paper Sec. 3.2, Sec. 4).
//
// Every form is a chain of  C = epilogue(A . W^T + b)  contractions over the
// tower's [B][W_t] block of the pooled tensor:
//   linear(+ReLU)  one projection                                (Listing 1, c = 0)
//   dot + linear   pairwise feature dot products z_p, then a projection of
//                  [z_p | x]                                      (Sec. 3.2, Sec. 4)
//   cross + linear x_{l+1} = x0 * (W_l x_l + b_l) + x_l, then a projection
//                                                                 (Listing 2)
//   DLRM           the flat projection next to one projection shared by every
//                  feature's embedding: a second contraction over the pooled block
//                  viewed as [B * features][dim]                  (Listing 1, c > 0)
// 16-bit types run on MFMA (v_mfma_f32_32x32x16, float32 accumulate): block tile
// 128 x 128 x 64, four waves of 64 x 64, operands staged through padded LDS, the
// next K tile prefetched into registers while the current one is multiplied.
// All towers of one stage go into ONE launch (a grouped GEMM: block id -> tower,
// tile), because a single tower's grid cannot fill 256 CUs.  The pairwise dots
// are a Gram matrix per sample: 32 consecutive (sample, feature) rows form one
// 32 x 32 MFMA tile whose diagonal blocks hold every sample's dots, so the
// operand is read once, straight from global memory, as both A and B.
// float32 towers (a latency-bound toy size) use plain FMA kernels.
#include "dmt_tm_gemm.h"

namespace {

// ----------------------------------------------------------------- host side

struct TowerWs {
  size_t z_off = 0, wp_off = 0, x_off[2] = {0, 0};
  size_t t_off = 0;            // low-rank cross layers: t = V_l x_l, [B][r]
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
      case DMT_TM_CROSS_LOWRANK_LINEAR: {
        const int L = q.num_cross_layers, r = q.feat_out;
        if (L < 1 || 2 * L > DMT_MAX_CROSS_LAYERS || r < 1) return DMT_EINVAL;
        if (eb == 2 && r % 8 != 0) return DMT_ENOTSUP;           // t is a K operand: 16-byte pieces
        for (int l = 0; l < L; ++l)
          if (!q.w_cross[2 * l] || !q.w_cross[2 * l + 1] || !q.b_cross[l] ||
              (((uintptr_t)q.w_cross[2 * l] | (uintptr_t)q.w_cross[2 * l + 1]) & 15))
            return DMT_EINVAL;
        w.x_off[0] = take((size_t)B * wt * eb);
        if (L > 1) w.x_off[1] = take((size_t)B * wt * eb);
        w.t_off = take((size_t)B * r * eb);
        break;
      }
      case DMT_TM_DLRM: {
        const int nf = p->tower_ntab[t];
        if (p->tower_uniform_dim[t] == 0) return DMT_ENOTSUP;   // one shared layer needs one dim
        if (q.feat_out < 1 || (int64_t)q.out_dim - (int64_t)nf * q.feat_out < 1) return DMT_EINVAL;
        if (!q.w_cross[0] || !q.b_cross[0] || ((uintptr_t)q.w_cross[0] & 15)) return DMT_EINVAL;
        if (B * nf >= (1LL << 31)) return DMT_ENOTSUP;
        break;
      }
      default:
        return DMT_EINVAL;
    }
  }
  *bytes = off;
  return DMT_OK;
}


template <int DT>
dmt_status run_tm(const dmt_plan* p, const dmt_tm_params* tp, const std::vector<TowerWs>& ws,
                  const void* pooled, int64_t B, void* tm_out, char* wsp, char* keptp,
                  hipStream_t s) {
  constexpr int eb = DT == DMT_F32 ? 4 : 2;
  const char* x_all = (const char*)pooled;
  char* y_all = (char*)tm_out;
  std::vector<int64_t> out_prefix(p->T + 1, 0);
  for (int32_t t = 0; t < p->T; ++t) out_prefix[t + 1] = out_prefix[t] + tp[t].out_dim;
  int max_layers = 0;
  // With `keptp` every cross layer's x_{l+1} and u_l go there instead of the two alternating
  // scratch buffers (a training forward: the backward reads them).
  std::vector<TmKept> kept;
  if (keptp) plan_tm_kept(p, tp, B, eb, &kept);
  auto x_layer = [&](int t, int l) -> char* {      // where x_{l+1} of tower t lives
    return keptp ? keptp + kept[t].x[l] : wsp + ws[t].x_off[l & 1];
  };

  // the dot terms of a dot-product tower: kept for the backward, else scratch
  auto z_of = [&](int t) -> char* {
    return keptp && kept[t].has_z ? keptp + kept[t].z : wsp + ws[t].z_off;
  };

  auto wp_of = [&](int t) -> char* {                // ... and its repacked projection weights
    return keptp && kept[t].has_z ? keptp + kept[t].wp : wsp + ws[t].wp_off;
  };

  // A dot-product tower whose shape fits computes its dot terms inside the projection GEMM.
  std::vector<char> fused(p->T, 0);
  if (DT != DMT_F32 && p->sw.tm_fuse != 0 && p->sw.tm_big != 0)
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
    if (q.kind == DMT_TM_CROSS_LINEAR || q.kind == DMT_TM_CROSS_LOWRANK_LINEAR)
      max_layers = std::max(max_layers, q.num_cross_layers);
    if (q.kind != DMT_TM_DOT_LINEAR) continue;
    const TowerWs& w = ws[t];
    TmAuxItem it{};
    it.nf = p->tower_ntab[t]; it.n = p->tower_uniform_dim[t]; it.np = w.np; it.np_pad = w.np_pad;
    it.O = q.out_dim; it.wt = p->tower_width[t];
    it.src = x_all + (size_t)B * p->width_prefix[t] * eb;
    it.dst = z_of(t);
    if (fused[t]) {
    } else if (DT != DMT_F32 && 32 % it.nf == 0 && it.n % 16 == 0) {
      dots_mfma.push_back(it);
      nb_mfma.push_back(((B * it.nf + 31) / 32 + 3) / 4);
    } else {
      dots_simple.push_back(it);
      nb_simple.push_back((B * w.np_pad + kBlock - 1) / kBlock);
    }
    it.src = q.w_proj;
    it.dst = wp_of(t);
    packs.push_back(it);
    nb_pack.push_back(((int64_t)q.out_dim * (w.np_pad + it.wt) + kBlock - 1) / kBlock);
  }
  launch_aux<DT>(p, B, dots_mfma, nb_mfma, 0, s);
  launch_aux<DT>(p, B, dots_simple, nb_simple, 1, s);
  launch_aux<DT>(p, B, packs, nb_pack, 2, s);

  // cross layers, one grouped launch per layer index (low-rank layers: t = V_l x_l first)
  std::vector<TmGroup> groups, groups_t;
  for (int l = 0; l < max_layers; ++l) {
    for (int32_t t = 0; t < p->T; ++t) {
      const dmt_tm_params& q = tp[t];
      const bool low = q.kind == DMT_TM_CROSS_LOWRANK_LINEAR;
      if ((q.kind != DMT_TM_CROSS_LINEAR && !low) || l >= q.num_cross_layers) continue;
      const int wt = p->tower_width[t];
      const void* x0 = x_all + (size_t)B * p->width_prefix[t] * eb;
      const void* xl = l == 0 ? x0 : (const void*)x_layer(t, l - 1);
      TmGroup g{};
      g.A0 = nullptr; g.lda0 = 0; g.K0 = 0;
      g.A1 = xl; g.lda1 = wt; g.K1 = wt;
      g.W = q.w_cross[l]; g.ldw = wt; g.bias = q.b_cross[l];
      if (low) {
        const int r = q.feat_out;
        TmGroup h{};
        h.A1 = xl; h.lda1 = wt; h.K1 = wt;
        h.W = q.w_cross[2 * l]; h.ldw = wt; h.bias = nullptr;
        h.C = wsp + ws[t].t_off; h.ldc = r;
        h.M = (int32_t)B; h.N = r; h.epi = EPI_BIAS;
        groups_t.push_back(h);
        g.A1 = wsp + ws[t].t_off; g.lda1 = r; g.K1 = r;
        g.W = q.w_cross[2 * l + 1]; g.ldw = r;
        g.XL = xl; g.ldxl = wt;
      }
      g.X0 = x0; g.ldx = wt;
      g.C = x_layer(t, l); g.ldc = wt;
      if (keptp) g.U = keptp + kept[t].u[l];
      g.M = (int32_t)B; g.N = wt; g.epi = EPI_CROSS;
      groups.push_back(g);
    }
    launch_groups<DT>(p, groups_t, s);
    launch_groups<DT>(p, groups, s);
  }

  // projections of every tower
  std::vector<TmGroup> groups_fused, groups_feat;
  for (int32_t t = 0; t < p->T; ++t) {
    const dmt_tm_params& q = tp[t];
    const int wt = p->tower_width[t];
    const void* x = x_all + (size_t)B * p->width_prefix[t] * eb;
    TmGroup g{};
    g.A0 = nullptr; g.lda0 = 0; g.K0 = 0;
    g.A1 = x; g.lda1 = wt; g.K1 = wt;
    g.W = q.w_proj; g.ldw = wt;
    if (q.kind == DMT_TM_DOT_LINEAR) {
      g.A0 = z_of(t); g.lda0 = ws[t].np_pad; g.K0 = ws[t].np_pad;
      g.W = wp_of(t); g.ldw = ws[t].np_pad + wt;
    } else if (q.kind == DMT_TM_CROSS_LINEAR || q.kind == DMT_TM_CROSS_LOWRANK_LINEAR) {
      g.A1 = x_layer(t, q.num_cross_layers - 1);
    }
    g.bias = q.b_proj;
    g.X0 = nullptr; g.ldx = 0;
    g.C = y_all + (size_t)B * out_prefix[t] * eb; g.ldc = q.out_dim;
    g.M = (int32_t)B; g.N = q.out_dim;
    g.epi = q.kind == DMT_TM_LINEAR_RELU ? EPI_BIAS_RELU : EPI_BIAS;
    if (q.kind == DMT_TM_DLRM) {
      // the shared per-feature layer: rows (sample, feature) of the pooled block, whose outputs
      // go behind the flat layer's in the sample's output row
      const int nf = p->tower_ntab[t], n = p->tower_uniform_dim[t];
      g.N = q.out_dim - nf * q.feat_out;
      TmGroup h{};
      h.A1 = x; h.lda1 = n; h.K1 = n;
      h.W = q.w_cross[0]; h.ldw = n; h.bias = q.b_cross[0];
      h.C = y_all + ((size_t)B * out_prefix[t] + g.N) * eb;
      h.ldc = q.out_dim; h.rdiv = nf; h.ldc2 = q.feat_out;
      h.M = (int32_t)(B * nf); h.N = q.feat_out; h.epi = EPI_BIAS;
      groups_feat.push_back(h);
    }
    if (fused[t]) {
      if (keptp && kept[t].has_z) g.U = z_of(t);
      g.A0 = nullptr; g.lda0 = 0;
      g.nf = p->tower_ntab[t]; g.fdim = p->tower_uniform_dim[t];
      groups_fused.push_back(g);
    } else {
      groups.push_back(g);
    }
  }
  launch_groups<DT>(p, groups, s);
  launch_groups<DT>(p, groups_feat, s);
  if constexpr (DT != DMT_F32) launch_groups<DT>(p, groups_fused, s, true);
  return hipGetLastError() == hipSuccess ? DMT_OK : DMT_EHIP;
}

}  // namespace

extern "C" size_t dmt_tm_workspace_bytes(const dmt_plan* plan, const dmt_tm_params* per_tower,
                                         int64_t B) {
  if (!plan || !per_tower || B <= 0) return 0;
  return dmt_guard_size([&]() -> size_t {
    std::vector<TowerWs> ws;
    size_t bytes = 0;
    // sized for the wider element type so one figure serves every dtype
    if (plan_tm(plan, per_tower, B, 4, &ws, &bytes) != DMT_OK) return 0;
    return bytes;
  });
}

namespace {

dmt_status tm_fwd_entry(const dmt_plan* plan, const dmt_tm_params* per_tower, const void* pooled,
                        int64_t B, void* tm_out, int32_t dtype_code, void* kept, size_t kept_bytes,
                        bool keep, void* workspace, size_t workspace_bytes, void* stream) {
  if (!plan || !per_tower || !pooled || !tm_out) return DMT_EINVAL;
  if (B <= 0 || B > plan->max_batch || B >= (1LL << 31)) return DMT_EINVAL;
  if (dtype_code != DMT_F32 && dtype_code != DMT_F16 && dtype_code != DMT_BF16) return DMT_EINVAL;
  const dmt_dtype dtype = (dmt_dtype)dtype_code;
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
  char* keptp = nullptr;
  if (keep) {
    std::vector<TmKept> k;
    const size_t need = plan_tm_kept(plan, per_tower, B, eb, &k);
    if (need > 0) {
      if (!kept || ((uintptr_t)kept & 255)) return DMT_EINVAL;
      if (kept_bytes < need) return DMT_ENOMEM;
      keptp = (char*)kept;
    }
  }
  hipStream_t s = (hipStream_t)stream;
  char* wsp = (char*)workspace;
  switch (dtype) {
    case DMT_F32: return run_tm<DMT_F32>(plan, per_tower, ws, pooled, B, tm_out, wsp, keptp, s);
    case DMT_F16: return run_tm<DMT_F16>(plan, per_tower, ws, pooled, B, tm_out, wsp, keptp, s);
    default: return run_tm<DMT_BF16>(plan, per_tower, ws, pooled, B, tm_out, wsp, keptp, s);
  }
}

}  // namespace

extern "C" dmt_status dmt_tower_module_fwd(const dmt_plan* plan, const dmt_tm_params* per_tower,
                                           const void* pooled, int64_t B, void* tm_out,
                                           int32_t dtype, void* workspace,
                                           size_t workspace_bytes, void* stream) {
  return dmt_guard([&] {
    return tm_fwd_entry(plan, per_tower, pooled, B, tm_out, dtype, nullptr, 0, false, workspace,
                        workspace_bytes, stream);
  });
}

extern "C" size_t dmt_tm_kept_bytes(const dmt_plan* plan, const dmt_tm_params* per_tower,
                                    int64_t B, int32_t dtype) {
  if (!plan || !per_tower || B <= 0) return 0;
  if (dtype != DMT_F32 && dtype != DMT_F16 && dtype != DMT_BF16) return 0;
  return dmt_guard_size([&]() -> size_t {
    std::vector<TmKept> k;
    return plan_tm_kept(plan, per_tower, B, dmt_elt_bytes((dmt_dtype)dtype), &k);
  });
}

extern "C" dmt_status dmt_tower_module_fwd_keep(const dmt_plan* plan,
                                                const dmt_tm_params* per_tower,
                                                const void* pooled, int64_t B, void* tm_out,
                                                int32_t dtype, void* kept, size_t kept_bytes,
                                                void* workspace, size_t workspace_bytes,
                                                void* stream) {
  return dmt_guard([&] {
    return tm_fwd_entry(plan, per_tower, pooled, B, tm_out, dtype, kept, kept_bytes, true, workspace,
                        workspace_bytes, stream);
  });
}
