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
// forward's intermediates are recomputed (dot terms, u_l = W_l x_l + b_l, x_l).
// Bias gradients are fixed-order row sums of the transposed gradient operand.
#include "dmt_tm_gemm.h"

namespace {

constexpr int kTile = 32;

template <int DT> struct EltOf { using type = uint16_t; };
template <> struct EltOf<DMT_F32> { using type = float; };

// ---------------------------------------------------------------- small kernels

// dz[b][o] = dy[b][o] (zero where ReLU was off: y[b][o] <= 0), rounded to DT, with
// zero columns O .. Op-1; dzT[o][b] the same values transposed, zero for b in
// [B, Bp).  Block = one 32 x 32 tile; grid.x over the batch, grid.y over outputs.
template <int DT>
__global__ __launch_bounds__(kBlock) void tmb_prep_dy(const float* __restrict__ dy,
                                                      const void* __restrict__ y, int relu,
                                                      int64_t B, int O, int Op, int64_t Bp,
                                                      void* __restrict__ dz,
                                                      void* __restrict__ dzT) {
  __shared__ float tile[kTile][kTile + 1];
  const int64_t b0 = (int64_t)blockIdx.x * kTile;
  const int o0 = blockIdx.y * kTile;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  for (int r = ty; r < kTile; r += kBlock / kTile) {
    const int64_t b = b0 + r;
    const int o = o0 + tx;
    float v = 0.f;
    if (b < B && o < O) {
      v = dy[b * O + o];
      if (relu && !(load_elt<DT>(y, b * O + o) > 0.f)) v = 0.f;
    }
    if (b < B && o < Op) store_elt<DT>(dz, b * Op + o, v);
    tile[r][tx] = v;
  }
  __syncthreads();
  for (int r = ty; r < kTile; r += kBlock / kTile) {
    const int o = o0 + r;
    const int64_t b = b0 + tx;
    if (o < O && b < Bp) store_elt<DT>(dzT, (int64_t)o * Bp + b, tile[tx][r]);
  }
}

// dst[c][r] = src[r][c] for r < R, 0 for R <= r < ldd; c < C.  src rows are lds
// elements apart, dst rows ldd.  grid.x over r, grid.y over c.
template <typename E>
__global__ __launch_bounds__(kBlock) void tmb_transpose(const E* __restrict__ src, int64_t R,
                                                        int C, int64_t lds, E* __restrict__ dst,
                                                        int64_t ldd) {
  __shared__ E tile[kTile][kTile + 1];
  const int64_t r0 = (int64_t)blockIdx.x * kTile;
  const int c0 = blockIdx.y * kTile;
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
    if (c < C && r < ldd) dst[(int64_t)c * ldd + r] = tile[tx][i];
  }
}

// out[r] = sum over c < ncols of src[r][c], float32, in a fixed order: thread t of
// the row's block adds columns t, t + 256, ... and the 256 partial sums are folded
// by halves.  One block per row.
template <int DT>
__global__ __launch_bounds__(kBlock) void tmb_rowsum(const void* __restrict__ src, int64_t ld,
                                                     int64_t ncols, float* __restrict__ out) {
  __shared__ float part[kBlock];
  const int64_t row = blockIdx.x;
  float s = 0.f;
  for (int64_t c = threadIdx.x; c < ncols; c += kBlock) s += load_elt<DT>(src, row * ld + c);
  part[threadIdx.x] = s;
  __syncthreads();
  for (int h = kBlock / 2; h > 0; h >>= 1) {
    if ((int)threadIdx.x < h) part[threadIdx.x] += part[threadIdx.x + h];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[row] = part[0];
}

// Dot-product tower: dx[b][i][c] = dZ[b][np_pad + i n + c]
//                                  + sum over j != i (ascending j) of dZ[b][p(i,j)] x[b][j][c]
// with p the row-major index of the pair {i, j}.  One thread per element of dx.
template <int DT>
__global__ __launch_bounds__(kBlock) void tmb_dot_bwd(const void* __restrict__ x,
                                                      const float* __restrict__ dZ, int64_t B,
                                                      int nf, int n, int np_pad, int ldz,
                                                      float* __restrict__ dx) {
  const int wt = nf * n;
  const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (e >= B * wt) return;
  const int64_t b = e / wt;
  const int r = (int)(e % wt), i = r / n, c = r % n;
  const float* z = dZ + b * ldz;
  float acc = z[np_pad + r];
  for (int j = 0; j < nf; ++j) {
    if (j == i) continue;
    const int lo = j < i ? j : i, hi = j < i ? i : j;
    acc += z[lo * (2 * nf - lo - 1) / 2 + (hi - lo - 1)] * load_elt<DT>(x, b * wt + j * n + c);
  }
  dx[e] = acc;
}

// dw[o][k] (row length np + wt) = packed[o][k'] (row length np_pad + wt): drops the
// padding columns between the dot terms and the flat part.
__global__ __launch_bounds__(kBlock) void tmb_unpack_dw(const float* __restrict__ packed, int O,
                                                        int np, int np_pad, int wt,
                                                        float* __restrict__ dw) {
  const int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  const int kin = np + wt;
  if (e >= (int64_t)O * kin) return;
  const int o = (int)(e / kin), k = (int)(e % kin);
  dw[e] = packed[(int64_t)o * (np_pad + wt) + (k < np ? k : k - np + np_pad)];
}

// Cross layer forward, elementwise part: xn = x0 * u + xl (rounded once to DT).
template <int DT>
__global__ __launch_bounds__(kBlock) void tmb_cross_next(const void* __restrict__ x0,
                                                         const void* __restrict__ u,
                                                         const void* __restrict__ xl, int64_t count,
                                                         void* __restrict__ xn) {
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  for (int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x; e < count; e += stride)
    store_elt<DT>(xn, e, load_elt<DT>(x0, e) * load_elt<DT>(u, e) + load_elt<DT>(xl, e));
}

// Cross layer backward, elementwise part: du = dxn * x0 (rounded to DT);
// dx0 = (first ? 0 : dx0) + dxn * u.
template <int DT>
__global__ __launch_bounds__(kBlock) void tmb_cross_prep(const float* __restrict__ dxn,
                                                         const void* __restrict__ x0,
                                                         const void* __restrict__ u, int first,
                                                         int64_t count, void* __restrict__ du,
                                                         float* __restrict__ dx0) {
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  for (int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x; e < count; e += stride) {
    const float g = dxn[e];
    store_elt<DT>(du, e, g * load_elt<DT>(x0, e));
    const float prev = first ? 0.f : dx0[e];
    dx0[e] = prev + g * load_elt<DT>(u, e);
  }
}

// io[e] += a[e]
__global__ __launch_bounds__(kBlock) void tmb_add(const float* __restrict__ a, int64_t count,
                                                  float* __restrict__ io) {
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  for (int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x; e < count; e += stride)
    io[e] += a[e];
}

// ----------------------------------------------------------------- host side

inline int64_t up8(int64_t v) { return (v + 7) / 8 * 8; }

struct TowerBwdWs {
  int np = 0, np_pad = 0;
  int kin = 0;                 // row length of the projection's GEMM operand (np_pad + wt for dots)
  int64_t Op = 0;
  size_t dz = 0, dzT = 0, wT = 0, zT = 0;
  size_t p = 0, wp = 0, dZ = 0, dWp = 0;                        // dot towers
  size_t xl[DMT_MAX_CROSS_LAYERS] = {}, u[DMT_MAX_CROSS_LAYERS] = {};   // cross towers
  size_t dxn = 0, du = 0, duT = 0, wlT = 0;
};

dmt_status plan_tm_bwd(const dmt_plan* p, const dmt_tm_params* tp, int64_t B, int eb,
                       std::vector<TowerBwdWs>* ws, size_t* bytes) {
  size_t off = 0;
  auto take = [&](size_t b) { size_t o = off; off = dmt_align_up(off + b, 256); return o; };
  const int64_t Bp = up8(B);
  ws->assign(p->T, TowerBwdWs());
  for (int32_t t = 0; t < p->T; ++t) {
    const dmt_tm_params& q = tp[t];
    const int64_t wt = p->tower_width[t];
    if (q.out_dim <= 0 || !q.w_proj || !q.b_proj) return DMT_EINVAL;
    if (((uintptr_t)q.w_proj & 15) && q.kind != DMT_TM_DOT_LINEAR) return DMT_EINVAL;
    TowerBwdWs& w = (*ws)[t];
    w.Op = up8(q.out_dim);
    w.kin = (int)wt;
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
        w.dWp = take((size_t)q.out_dim * w.kin * 4);
        break;
      }
      case DMT_TM_CROSS_LINEAR:
        if (q.num_cross_layers < 1 || q.num_cross_layers > DMT_MAX_CROSS_LAYERS) return DMT_EINVAL;
        for (int l = 0; l < q.num_cross_layers; ++l) {
          if (!q.w_cross[l] || !q.b_cross[l] || ((uintptr_t)q.w_cross[l] & 15)) return DMT_EINVAL;
          w.xl[l] = take((size_t)B * wt * eb);      // x_{l+1}
          w.u[l] = take((size_t)B * wt * eb);
        }
        w.dxn = take((size_t)B * wt * 4);
        w.du = take((size_t)B * wt * eb);
        w.duT = take((size_t)wt * Bp * eb);
        w.wlT = take((size_t)wt * wt * eb);
        break;
      default:
        return DMT_EINVAL;
    }
    w.dz = take((size_t)B * w.Op * eb);
    w.dzT = take((size_t)q.out_dim * Bp * eb);
    w.wT = take((size_t)w.kin * w.Op * eb);
    w.zT = take((size_t)w.kin * Bp * eb);
  }
  *bytes = off;
  return DMT_OK;
}

inline int ew_blocks(int64_t count) {
  return (int)std::min<int64_t>((count + kBlock - 1) / kBlock, 256 * 16);
}

template <int DT>
void transpose(const dmt_plan* p, const void* src, int64_t R, int C, int64_t lds, void* dst,
               int64_t ldd, hipStream_t s) {
  using E = typename EltOf<DT>::type;
  DmtScope sc_(p, DMT_K_TM_BWD_AUX, s);
  hipLaunchKernelGGL((tmb_transpose<E>), dim3((unsigned)((ldd + kTile - 1) / kTile), (C + kTile - 1) / kTile),
                     dim3(kBlock), 0, s, (const E*)src, R, C, lds, (E*)dst, ldd);
}

template <int DT>
dmt_status run_tm_bwd(const dmt_plan* p, const dmt_tm_params* tp, const std::vector<TowerBwdWs>& ws,
                      const void* pooled, const void* tm_out, int64_t B, const float* dy_all,
                      float* dx_all, const dmt_tm_grads* gr, char* wsp, hipStream_t s) {
  constexpr int eb = DT == DMT_F32 ? 4 : 2;
  const char* x_all = (const char*)pooled;
  const int64_t Bp = up8(B);
  std::vector<int64_t> out_prefix(p->T + 1, 0);
  for (int32_t t = 0; t < p->T; ++t) out_prefix[t + 1] = out_prefix[t] + tp[t].out_dim;
  auto x_of = [&](int t) { return (const void*)(x_all + (size_t)B * p->width_prefix[t] * eb); };
  auto dx_of = [&](int t) { return dx_all + (size_t)B * p->width_prefix[t]; };
  // x_l of a cross tower: l = 0 is the pooled block itself
  auto xl_of = [&](int t, int l) { return l == 0 ? x_of(t) : (const void*)(wsp + ws[t].xl[l - 1]); };
  int max_layers = 0;

  // ---- recompute what the forward did not keep: dot terms (and the repacked weights)
  std::vector<TmAuxItem> dots_mfma, dots_simple, packs;
  std::vector<int64_t> nb_mfma, nb_simple, nb_pack;
  for (int32_t t = 0; t < p->T; ++t) {
    const dmt_tm_params& q = tp[t];
    if (q.kind == DMT_TM_CROSS_LINEAR) max_layers = std::max(max_layers, q.num_cross_layers);
    if (q.kind != DMT_TM_DOT_LINEAR) continue;
    const TowerBwdWs& w = ws[t];
    TmAuxItem it{};
    it.nf = p->tower_ntab[t]; it.n = p->tower_uniform_dim[t]; it.np = w.np; it.np_pad = w.np_pad;
    it.O = q.out_dim; it.wt = p->tower_width[t];
    it.src = x_of(t);
    it.dst = wsp + w.p;
    if (w.np_pad > 0) {
      if (DT != DMT_F32 && 32 % it.nf == 0 && it.n % 16 == 0) {
        dots_mfma.push_back(it);
        nb_mfma.push_back(((B * it.nf + 31) / 32 + 3) / 4);
      } else {
        dots_simple.push_back(it);
        nb_simple.push_back((B * w.np_pad + kBlock - 1) / kBlock);
      }
    }
    it.src = q.w_proj;
    it.dst = wsp + w.wp;
    packs.push_back(it);
    nb_pack.push_back(((int64_t)q.out_dim * w.kin + kBlock - 1) / kBlock);
  }
  launch_aux<DT>(p, B, dots_mfma, nb_mfma, 0, s);
  launch_aux<DT>(p, B, dots_simple, nb_simple, 1, s);
  launch_aux<DT>(p, B, packs, nb_pack, 2, s);

  // ---- ... and the cross layers' u_l = x_l W_l^T + b_l, x_{l+1} = x0 * u_l + x_l
  std::vector<TmGroup> groups;
  for (int l = 0; l < max_layers; ++l) {
    for (int32_t t = 0; t < p->T; ++t) {
      const dmt_tm_params& q = tp[t];
      if (q.kind != DMT_TM_CROSS_LINEAR || l >= q.num_cross_layers) continue;
      const int wt = p->tower_width[t];
      TmGroup g{};
      g.A1 = xl_of(t, l); g.lda1 = wt; g.K1 = wt;
      g.W = q.w_cross[l]; g.ldw = wt; g.bias = q.b_cross[l];
      g.C = wsp + ws[t].u[l]; g.ldc = wt;
      g.M = (int32_t)B; g.N = wt; g.epi = EPI_BIAS;
      groups.push_back(g);
    }
    launch_groups<DT>(p, groups, s, false, DMT_K_TM_BWD_GEMM);
    for (int32_t t = 0; t < p->T; ++t) {
      const dmt_tm_params& q = tp[t];
      if (q.kind != DMT_TM_CROSS_LINEAR || l >= q.num_cross_layers) continue;
      const int64_t count = B * p->tower_width[t];
      DmtScope sc_(p, DMT_K_TM_BWD_AUX, s);
      hipLaunchKernelGGL((tmb_cross_next<DT>), dim3(ew_blocks(count)), dim3(kBlock), 0, s, x_of(t),
                         (const void*)(wsp + ws[t].u[l]), xl_of(t, l), count,
                         (void*)(wsp + ws[t].xl[l]));
    }
  }

  // ---- projection: operands, bias gradient, then both contractions for all towers
  std::vector<TmGroup> dgrad, wgrad;
  for (int32_t t = 0; t < p->T; ++t) {
    const dmt_tm_params& q = tp[t];
    const TowerBwdWs& w = ws[t];
    const int wt = p->tower_width[t], O = q.out_dim;
    const int relu = q.kind == DMT_TM_LINEAR_RELU;
    const float* dy = dy_all + (size_t)B * out_prefix[t];
    const void* y = relu ? (const void*)((const char*)tm_out + (size_t)B * out_prefix[t] * eb) : nullptr;
    {
      DmtScope sc_(p, DMT_K_TM_BWD_AUX, s);
      hipLaunchKernelGGL((tmb_prep_dy<DT>),
                         dim3((unsigned)((Bp + kTile - 1) / kTile), (unsigned)((w.Op + kTile - 1) / kTile)),
                         dim3(kBlock), 0, s, dy, y, relu, B, O, (int)w.Op, Bp, (void*)(wsp + w.dz),
                         (void*)(wsp + w.dzT));
    }
    {
      DmtScope sc_(p, DMT_K_TM_BWD_AUX, s);
      hipLaunchKernelGGL((tmb_rowsum<DT>), dim3(O), dim3(kBlock), 0, s, (const void*)(wsp + w.dzT),
                         Bp, B, gr[t].db_proj);
    }
    // W^T [kin][Op]
    const void* wsrc = q.kind == DMT_TM_DOT_LINEAR ? (const void*)(wsp + w.wp) : q.w_proj;
    transpose<DT>(p, wsrc, O, w.kin, w.kin, wsp + w.wT, w.Op, s);
    // z^T [kin][Bp]: the projection's input, transposed
    if (q.kind == DMT_TM_DOT_LINEAR) {
      if (w.np_pad > 0) transpose<DT>(p, wsp + w.p, B, w.np_pad, w.np_pad, wsp + w.zT, Bp, s);
      transpose<DT>(p, x_of(t), B, wt, wt, wsp + w.zT + (size_t)w.np_pad * Bp * eb, Bp, s);
    } else {
      const void* z = q.kind == DMT_TM_CROSS_LINEAR ? xl_of(t, q.num_cross_layers) : x_of(t);
      transpose<DT>(p, z, B, wt, wt, wsp + w.zT, Bp, s);
    }
    TmGroup g{};
    g.A1 = wsp + w.dz; g.lda1 = (int32_t)w.Op; g.K1 = (int32_t)w.Op;
    g.W = wsp + w.wT; g.ldw = (int32_t)w.Op;
    g.M = (int32_t)B; g.N = w.kin; g.epi = EPI_F32;
    if (q.kind == DMT_TM_DOT_LINEAR) { g.C = wsp + w.dZ; g.ldc = w.kin; }
    else if (q.kind == DMT_TM_CROSS_LINEAR) { g.C = wsp + w.dxn; g.ldc = wt; }
    else { g.C = dx_of(t); g.ldc = wt; }
    dgrad.push_back(g);
    TmGroup h{};
    h.A1 = wsp + w.dzT; h.lda1 = (int32_t)Bp; h.K1 = (int32_t)Bp;
    h.W = wsp + w.zT; h.ldw = (int32_t)Bp;
    h.M = O; h.N = w.kin; h.epi = EPI_F32;
    h.C = q.kind == DMT_TM_DOT_LINEAR ? (void*)(wsp + w.dWp) : (void*)gr[t].dw_proj;
    h.ldc = w.kin;
    wgrad.push_back(h);
  }
  launch_groups<DT>(p, dgrad, s, false, DMT_K_TM_BWD_GEMM);
  launch_groups<DT>(p, wgrad, s, false, DMT_K_TM_BWD_GEMM);

  // ---- dot towers: fold the dot terms' gradients into dx, strip dW's padding
  for (int32_t t = 0; t < p->T; ++t) {
    const dmt_tm_params& q = tp[t];
    if (q.kind != DMT_TM_DOT_LINEAR) continue;
    const TowerBwdWs& w = ws[t];
    const int wt = p->tower_width[t];
    {
      DmtScope sc_(p, DMT_K_TM_BWD_AUX, s);
      hipLaunchKernelGGL((tmb_dot_bwd<DT>), dim3((unsigned)((B * wt + kBlock - 1) / kBlock)),
                         dim3(kBlock), 0, s, x_of(t), (const float*)(wsp + w.dZ), B,
                         p->tower_ntab[t], p->tower_uniform_dim[t], w.np_pad, w.kin, dx_of(t));
    }
    {
      DmtScope sc_(p, DMT_K_TM_BWD_AUX, s);
      const int64_t count = (int64_t)q.out_dim * (w.np + wt);
      hipLaunchKernelGGL(tmb_unpack_dw, dim3((unsigned)((count + kBlock - 1) / kBlock)), dim3(kBlock),
                         0, s, (const float*)(wsp + w.dWp), q.out_dim, w.np, w.np_pad, wt,
                         gr[t].dw_proj);
    }
  }

  // ---- cross towers: layers from the last to the first; dx0 accumulates in the output block
  for (int l = max_layers - 1; l >= 0; --l) {
    for (int32_t t = 0; t < p->T; ++t) {
      const dmt_tm_params& q = tp[t];
      if (q.kind != DMT_TM_CROSS_LINEAR || l >= q.num_cross_layers) continue;
      const TowerBwdWs& w = ws[t];
      const int wt = p->tower_width[t];
      const int64_t count = B * wt;
      {
        DmtScope sc_(p, DMT_K_TM_BWD_AUX, s);
        hipLaunchKernelGGL((tmb_cross_prep<DT>), dim3(ew_blocks(count)), dim3(kBlock), 0, s,
                           (const float*)(wsp + w.dxn), x_of(t), (const void*)(wsp + w.u[l]),
                           l == q.num_cross_layers - 1 ? 1 : 0, count, (void*)(wsp + w.du), dx_of(t));
      }
      transpose<DT>(p, wsp + w.du, B, wt, wt, wsp + w.duT, Bp, s);
      {
        DmtScope sc_(p, DMT_K_TM_BWD_AUX, s);
        hipLaunchKernelGGL((tmb_rowsum<DT>), dim3(wt), dim3(kBlock), 0, s,
                           (const void*)(wsp + w.duT), Bp, B, gr[t].db_cross[l]);
      }
      transpose<DT>(p, xl_of(t, l), B, wt, wt, wsp + w.zT, Bp, s);
      transpose<DT>(p, q.w_cross[l], wt, wt, wt, wsp + w.wlT, wt, s);
      TmGroup g{};
      g.A1 = wsp + w.du; g.lda1 = wt; g.K1 = wt;
      g.W = wsp + w.wlT; g.ldw = wt;
      g.M = (int32_t)B; g.N = wt; g.epi = EPI_F32_ADD;
      g.C = wsp + w.dxn; g.ldc = wt;
      dgrad.push_back(g);
      TmGroup h{};
      h.A1 = wsp + w.duT; h.lda1 = (int32_t)Bp; h.K1 = (int32_t)Bp;
      h.W = wsp + w.zT; h.ldw = (int32_t)Bp;
      h.M = wt; h.N = wt; h.epi = EPI_F32;
      h.C = gr[t].dw_cross[l]; h.ldc = wt;
      wgrad.push_back(h);
    }
    launch_groups<DT>(p, dgrad, s, false, DMT_K_TM_BWD_GEMM);
    launch_groups<DT>(p, wgrad, s, false, DMT_K_TM_BWD_GEMM);
  }
  for (int32_t t = 0; t < p->T; ++t) {
    if (tp[t].kind != DMT_TM_CROSS_LINEAR) continue;
    const int64_t count = B * p->tower_width[t];
    DmtScope sc_(p, DMT_K_TM_BWD_AUX, s);
    hipLaunchKernelGGL(tmb_add, dim3(ew_blocks(count)), dim3(kBlock), 0, s,
                       (const float*)(wsp + ws[t].dxn), count, dx_of(t));
  }
  return hipGetLastError() == hipSuccess ? DMT_OK : DMT_EHIP;
}

}  // namespace

extern "C" size_t dmt_tm_bwd_workspace_bytes(const dmt_plan* plan, const dmt_tm_params* per_tower,
                                             int64_t B) {
  if (!plan || !per_tower || B <= 0) return 0;
  std::vector<TowerBwdWs> ws;
  size_t bytes = 0;
  if (plan_tm_bwd(plan, per_tower, B, 4, &ws, &bytes) != DMT_OK) return 0;
  return bytes;
}

extern "C" dmt_status dmt_tower_module_bwd(const dmt_plan* plan, const dmt_tm_params* per_tower,
                                           const void* pooled, const void* tm_out, int64_t B,
                                           const float* grad_tm_out, dmt_dtype dtype,
                                           float* grad_pooled, const dmt_tm_grads* grads,
                                           void* workspace, size_t workspace_bytes, void* stream) {
  if (!plan || !per_tower || !pooled || !grad_tm_out || !grad_pooled || !grads) return DMT_EINVAL;
  if (B <= 0 || B > plan->max_batch || B >= (1LL << 31) - 8) return DMT_EINVAL;
  if (dtype != DMT_F32 && dtype != DMT_F16 && dtype != DMT_BF16) return DMT_EINVAL;
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
  }
  std::vector<TowerBwdWs> ws;
  size_t bytes = 0;
  dmt_status st = plan_tm_bwd(plan, per_tower, B, eb, &ws, &bytes);
  if (st != DMT_OK) return st;
  if (!workspace || ((uintptr_t)workspace & 255)) return DMT_EINVAL;
  if (workspace_bytes < bytes) return DMT_ENOMEM;
  hipStream_t s = (hipStream_t)stream;
  char* wsp = (char*)workspace;
  switch (dtype) {
    case DMT_F32:
      return run_tm_bwd<DMT_F32>(plan, per_tower, ws, pooled, tm_out, B, grad_tm_out, grad_pooled,
                                 grads, wsp, s);
    case DMT_F16:
      return run_tm_bwd<DMT_F16>(plan, per_tower, ws, pooled, tm_out, B, grad_tm_out, grad_pooled,
                                 grads, wsp, s);
    default:
      return run_tm_bwd<DMT_BF16>(plan, per_tower, ws, pooled, tm_out, B, grad_tm_out, grad_pooled,
                                  grads, wsp, s);
  }
}
