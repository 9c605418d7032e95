// Memory-bound kernels of one pdADMM iteration: step-size selection, the p/W/b steps, the
// closed-form z, q and u updates, projection onto Delta, FISTA for z_L and the reductions behind
// the objective. All are grouped over layers through small descriptor tables in device memory;
// every reduction is two-stage with a fixed summation order (bit-reproducible, no atomics).
#pragma once
#include "common.h"

namespace pdadmm {

// ------------------------------------------------------------------------------------------
// Flat y -= s * x over float4 groups; s comes from the layer's scalars.
// ------------------------------------------------------------------------------------------
enum : int { kScaleInvTau = 0, kScaleInvTheta = 1, kScaleMinusOneIfStep = 2, kScaleFixTau = 3, kScaleFixTheta = 4 };

struct AxpySeg {
  float* y;
  const float* x;
  size_t n4;        // number of float4 groups
  int blk0, nblk;
  int layer, which;
};

constexpr int kAxpyThreads = 64;   // one wave per block, one float4 group per lane (C5, r += W d: 2.60 -> 2.49 ms against 256)
__global__ __launch_bounds__(kAxpyThreads) void axpy_kernel(const AxpySeg* __restrict__ segs, const BlockMap map,
                                                   const LayerScal* __restrict__ scal) {
  int local;
  const int si = find_group(map, blockIdx.x, &local);
  const AxpySeg S = segs[si];
  const LayerScal& sc = scal[S.layer];
  float s;
  if (S.which == kScaleInvTau) s = sc.inv_tau;
  else if (S.which == kScaleInvTheta) s = sc.inv_theta;
  else s = sc.inv_tau != 0.0f ? -1.0f : 0.0f;
  if (s == 0.0f) return;
  // one float4 group per thread, consecutive blocks own consecutive 4 KiB chunks: a pure stream
  const size_t i = (size_t)local * kAxpyThreads + threadIdx.x;
  if (i >= S.n4) return;
  f32x4* y = reinterpret_cast<f32x4*>(S.y) + i;
  const f32x4 a = stream_load(y);
  const f32x4 b = stream_load(reinterpret_cast<const f32x4*>(S.x) + i);
  stream_store(y, a - s * b);
}

// The same update as a small grid-stride kernel: the correction pass after a speculative update
// (y already holds y - s_ahead x; what is left is s = s_new - s_ahead). Almost always s = 0 and the
// blocks leave at once, which is why this pass does not get one block per 4 KiB.
__global__ __launch_bounds__(256) void axpy_fix_kernel(const AxpySeg* __restrict__ segs, const BlockMap map,
                                                       const LayerScal* __restrict__ scal) {
  int local;
  const int si = find_group(map, blockIdx.x, &local);
  const AxpySeg S = segs[si];
  const float s = scal[S.layer].fix_tau;
  if (s == 0.0f) return;
  const size_t stride = (size_t)S.nblk * 256;
  for (size_t i = (size_t)local * 256 + threadIdx.x; i < S.n4; i += stride) {
    f32x4* y = reinterpret_cast<f32x4*>(S.y) + i;
    const f32x4 a = *y;
    const f32x4 b = reinterpret_cast<const f32x4*>(S.x)[i];
    *y = a - s * b;
  }
}

// ------------------------------------------------------------------------------------------
// Step-size selection (Appendix A: tau must satisfy phi(p_new) <= U_l(p_new; tau), theta the
// analogous condition with V_l). phi is exactly quadratic in p_l and in W_l, so for the
// unprojected step the condition reads  t >= lambda  with
//   lambda_p = rho + nu ||W g||^2 / ||g||^2,   lambda_W = nu ||G p||^2 / ||G||^2.
// Schedule: start at previous/eta, multiply by eta until t >= lambda.
// One block per layer; partial sums are added in a fixed order.
// ------------------------------------------------------------------------------------------
struct SelectDesc {
  const double* part_g;   // partials of ||g||^2 (or ||G||^2, or ||d||^2)
  const double* part_t;   // partials of ||W g||^2 (or ||G p||^2, or ||W d||^2)
  int ng, nt;
  int stride_t;           // doubles per block in part_t (1 or 2)
  int layer;
};

__device__ __forceinline__ double fixed_order_sum(const double* p, int n, int stride, double* red) {
  double s = 0.0;
  for (int i = threadIdx.x; i < n; i += 256) s += p[(size_t)i * stride];
  return block_sum_256(s, red);
}

// mode 0: tau (p-update, unprojected); mode 1: theta (W-update)
__global__ __launch_bounds__(256) void select_step_kernel(const SelectDesc* __restrict__ descs, LayerScal* scal,
                                                          int mode, float rho, float nu, float eta, int max_trials,
                                                          int* err) {
  __shared__ double red[4];
  const SelectDesc D = descs[blockIdx.x];
  const double sg = fixed_order_sum(D.part_g, D.ng, 1, red);
  const double st = fixed_order_sum(D.part_t, D.nt, D.stride_t, red);
  if (threadIdx.x != 0) return;
  LayerScal& sc = scal[D.layer];
  sc.norm_g = sg;
  sc.norm_t = st;
  const float ahead = mode == 0 ? sc.spec_tau : sc.spec_theta;   // what the epilogues of this update applied
  float inv = 0.0f, next = 0.0f;
  int trials = 0;
  if (!(sg == sg) || !(st == st) || sg > 1.7e308 || st > 1.7e308) {
    atomicOr(err, kErrNonFinite);
  } else if (sg > 0.0) {
    const double lambda = (mode == 0 ? (double)rho : 0.0) + (double)nu * st / sg;
    double t = (mode == 0 ? sc.tau : sc.theta) / (double)eta;
    trials = 1;
    while (t < lambda && trials < max_trials) {
      t *= (double)eta;
      ++trials;
    }
    if (t < lambda) atomicOr(err, kErrBacktrack);
    else {
      if (mode == 0) sc.tau = t; else sc.theta = t;
      inv = (float)(1.0 / t);
      // the next update starts at t/eta: accepted at once this time, it is likely to be accepted again
      next = trials == 1 ? (float)(1.0 / (t / (double)eta)) : inv;
    }
  }
  if (mode == 0) { sc.inv_tau = inv; sc.fix_tau = inv - ahead; sc.spec_tau = next; sc.p_trials = trials; }
  else { sc.inv_theta = inv; sc.fix_theta = inv - ahead; sc.spec_theta = next; sc.w_trials = trials; }
}

// ------------------------------------------------------------------------------------------
// W-step: W <- W - G/theta, plus the transposed copy Wt[n_in][ld_out] kept for the W^T r product.
// 32x32 tiles through LDS so that both the read of W and the write of Wt are coalesced.
// ------------------------------------------------------------------------------------------
struct WStepSeg {
  float* W;         // [n_out][ld_in]
  float* Wt;        // [n_in][ld_out]
  const float* G;   // [n_out][ld_in]
  int n_out, n_in, ld_in, ld_out;
  int tiles_c;      // tiles along n_in
  int blk0, nblk;
  int layer;
};

__global__ __launch_bounds__(256) void w_step_kernel(const WStepSeg* __restrict__ segs, const BlockMap map,
                                                     const LayerScal* __restrict__ scal, int copy_only) {
  __shared__ float tile[32][33];
  int local;
  const int si = find_group(map, blockIdx.x, &local);
  const WStepSeg S = segs[si];
  const float inv = copy_only ? 0.0f : scal[S.layer].inv_theta;
  const int tr = local / S.tiles_c, tc = local % S.tiles_c;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int r = tr * 32 + ty + 8 * k, c = tc * 32 + tx;
    float w = 0.0f;
    if (r < S.n_out && c < S.n_in) {
      const size_t i = (size_t)r * S.ld_in + c;
      w = S.W[i];
      if (inv != 0.0f) {
        w -= inv * S.G[i];
        S.W[i] = w;
      }
    }
    tile[ty + 8 * k][tx] = w;
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int c = tc * 32 + ty + 8 * k, r = tr * 32 + tx;   // Wt row = c (n_in), Wt col = r (n_out)
    if (c < S.n_in && r < S.n_out) S.Wt[(size_t)c * S.ld_out + r] = tile[tx][ty + 8 * k];
  }
}

// ------------------------------------------------------------------------------------------
// Row-structured passes over [rows, ld] arrays (blocks of kRowsPerBlock rows).
// ------------------------------------------------------------------------------------------
constexpr int kRowsPerBlock = 32;

struct RowSeg {
  float* R;             // carried residual W p + b - z
  const float* T;       // G p (W-step direction image)
  float* z;
  float* q;
  float* u;
  const float* pnext;   // p_{l+1} (fp32), or null when it is kept as indices:
  const uint8_t* pnext8;  // -Q: the two index planes of p_{l+1} (p8_plane bytes each; LayerScal::cur of layer + 1 selects)
  size_t p8_plane;
  const float* m;       // column means (b-step), [ld]
  double* colpart;      // [row_blocks][ld]
  int rows, ncols, ld;
  int cw;               // float4 column groups per block row (power of two, <= 256)
  int rpb;              // rows per block of the column-sum pass
  int which;            // kScaleInvTheta: full update; kScaleFixTheta: correction after a speculative update
  int col_blocks, row_blocks;
  int blk0, nblk;       // blocks of the column-sum pass
  int layer;
};

// R <- R - T/theta and per-block column sums of the new R (b-update, Appendix A 'update b':
// the minimiser over the broadcast bias subtracts the node-mean of W p + b - z).
// A block covers kRowsPerBlock rows x (up to) 1024 columns: the 256 threads are laid out as
// cw column groups (float4) x (256 / cw) rows, cw = the power of two >= ld/4 capped at 256, so that
// one step of the block reads whole consecutive rows (a contiguous stream).
__global__ __launch_bounds__(256) void resid_colsum_kernel(const RowSeg* __restrict__ segs, const BlockMap map,
                                                           const LayerScal* __restrict__ scal) {
  __shared__ double sm[256][4];
  int local;
  const int si = find_group(map, blockIdx.x, &local);
  const RowSeg S = segs[si];
  const float inv = S.which == kScaleFixTheta ? scal[S.layer].fix_theta : scal[S.layer].inv_theta;
  // correction pass: nothing to do (and the column sums taken by the product kernel stand) if theta did not change
  if (S.which == kScaleFixTheta && inv == 0.0f) return;
  const int cb = local % S.col_blocks, rb = local / S.col_blocks;
  const int cw = S.cw, rstep = 256 / cw;
  const int cq = threadIdx.x & (cw - 1), ty = threadIdx.x / cw;
  const int col = (cb * cw + cq) * 4;
  double a0 = 0, a1 = 0, a2 = 0, a3 = 0;
  if (col < S.ld) {
    const int rend = min(S.rows, (rb + 1) * S.rpb);
    // four rows in flight per thread
    for (int r = rb * S.rpb + ty; r < rend; r += 4 * rstep) {
      f32x4 v[4], t[4];
      bool on[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        on[k] = r + k * rstep < rend;
        const size_t i = (size_t)(r + k * rstep) * S.ld + col;
        if (on[k]) {
          v[k] = stream_load(reinterpret_cast<const f32x4*>(S.R + i));
          if (inv != 0.0f) t[k] = stream_load(reinterpret_cast<const f32x4*>(S.T + i));
        }
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        if (on[k]) {
          if (inv != 0.0f) {
            v[k] -= inv * t[k];
            stream_store(reinterpret_cast<f32x4*>(S.R + (size_t)(r + k * rstep) * S.ld + col), v[k]);
          }
          a0 += (double)v[k].x; a1 += (double)v[k].y; a2 += (double)v[k].z; a3 += (double)v[k].w;
        }
      }
    }
  }
  sm[threadIdx.x][0] = a0; sm[threadIdx.x][1] = a1; sm[threadIdx.x][2] = a2; sm[threadIdx.x][3] = a3;
  __syncthreads();
  if (ty == 0 && col < S.ld) {
    double* out = S.colpart + (size_t)rb * S.ld + col;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      double t = 0.0;
      for (int j = 0; j < rstep; ++j) t += sm[j * cw + cq][k];   // fixed order
      out[k] = t;
    }
  }
}

// b <- b - mean; m <- mean. A block owns 32 columns; its 8 row groups add up a strided share of the
// per-row-block partial sums each (coalesced 256-byte reads), then the groups are combined in a
// fixed order.
struct BiasSeg {
  float* b;
  float* m;
  const double* colpart;
  int ncols, ld, row_blocks, rows;
  int blk0, nblk;
};

__global__ __launch_bounds__(256) void bias_step_kernel(const BiasSeg* __restrict__ segs, const BlockMap map) {
  __shared__ double sm[8][32];
  int local;
  const int si = find_group(map, blockIdx.x, &local);
  const BiasSeg S = segs[si];
  const int cx = threadIdx.x & 31, g = threadIdx.x >> 5;
  const int c = local * 32 + cx;
  double s = 0.0;
  if (c < S.ld)
    for (int rb = g; rb < S.row_blocks; rb += 8) s += S.colpart[(size_t)rb * S.ld + c];
  sm[g][cx] = s;
  __syncthreads();
  if (g == 0 && c < S.ld) {
    double t = 0.0;
#pragma unroll
    for (int k = 0; k < 8; ++k) t += sm[k][cx];
    const float mean = c < S.ncols ? (float)(t / (double)S.rows) : 0.0f;
    S.m[c] = mean;
    if (c < S.ncols) S.b[c] -= mean;
  }
}

// Closed-form z-update (Appendix A 'update z', l < L) on one element, for f(z) = z (z >= 0), slope*z
// (z < 0); slope = 0 is the ReLU case printed in the paper. a = W p + b (new), s = a + z_old.
// On z >= 0 the subproblem (z-a)^2 + (q-f(z))^2 + (z-z_old)^2 is 3 z^2 - 2 z (s+q) + const, on z <= 0 it
// is (2+slope^2) z^2 - 2 z (s + slope q) + const. Candidates: max((s+q)/3, 0) and
// min((s + slope q)/(2 + slope^2), 0); a candidate clamped to 0 gains nothing over z = 0, an interior
// one lowers the value by (s+q)^2/3 resp. (s + slope q)^2/(2 + slope^2): the larger gain wins, a tie
// goes to the non-positive candidate.
__device__ __forceinline__ float z_closed_form(float s, float q, float slope) {
  const float tp = s + q;
  const float tn = s + slope * q;
  const float dn = 2.0f + slope * slope;
  const float zpos = fmaxf(tp / 3.0f, 0.0f);
  const float zneg = fminf(tn / dn, 0.0f);
  const float gain_pos = tp > 0.0f ? (tp * tp) / 3.0f : 0.0f;
  const float gain_neg = tn < 0.0f ? (tn * tn) / dn : 0.0f;
  return gain_pos > gain_neg ? zpos : zneg;
}

// Fused b-shift, z-update, q-update, residual and dual update for layers l < L
// (Appendix A 'update z', 'update q', 'update u'):
//   a = R - m + z_old; z = closed form; R <- a - z;
//   q = (rho p_{l+1} + u + nu f(z)) / (rho + nu); r = p_{l+1} - q; u <- u + rho r.
// In the variant that keeps q on the grid as well (Appendix B, last paragraph) the closed-form q is
// projected onto Delta before r and u are formed.
// Blocks of ONE wave with one float4 group per lane: a block covers 1 KiB of each of its nine arrays. Measured at
// 680 MB per array (C3), threads x groups per thread: 64x1 9.21 ms, 256x1 9.63, 128x1 10.08, 512x1 10.01, 256x2 10.07,
// 256x4 10.16, 64x2 9.95, 64x4 9.76; with cached instead of nontemporal loads or stores 10.6-10.8 ms.
constexpr int kZquUnroll = 1;
constexpr int kZquThreads = 64;
__device__ __forceinline__ f32x4 zqu_load(const f32x4* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ void zqu_store(f32x4* p, f32x4 v) { __builtin_nontemporal_store(v, p); }

// pgrid: Delta when p_{l+1} is kept as 8-bit indices (-Q; levels = 0 otherwise); qgrid: Delta when q is projected too.
// IB: bytes per index of p_{l+1} (1 or 2; ignored when p_{l+1} is fp32).
template <int IB>
__global__ __launch_bounds__(kZquThreads) void zqu_kernel(const RowSeg* __restrict__ segs, const BlockMap map,
                                                  const LayerScal* __restrict__ scal, float rho, float nu,
                                                  float slope, const QuantGrid pgrid, const QuantGrid qgrid) {
  int local;
  const int si = find_group(map, blockIdx.x, &local);
  const RowSeg S = segs[si];
  const float inv_rn = 1.0f / (rho + nu);
  const uint8_t* p8 = S.pnext8 ? S.pnext8 + (size_t)scal[S.layer + 1].cur * S.p8_plane : nullptr;
  // flat over the [rows, ld] arrays: a block owns 256*kZquUnroll consecutive float4 groups
  const size_t n4 = (size_t)S.rows * (S.ld / 4);
  const int ld4 = S.ld / 4;
  const size_t base = (size_t)local * (kZquThreads * kZquUnroll) + threadIdx.x;
  f32x4 Rv[kZquUnroll], zo[kZquUnroll], qo[kZquUnroll], pn[kZquUnroll], uo[kZquUnroll], mm[kZquUnroll];
  // pad columns (ld is the width rounded up to 4) hold zeros in every input and must stay zero: the closed forms
  // map zeros to zeros, only the projection of q does not when 0 is no member of Delta
  const bool ragged = qgrid.levels > 0 && S.ncols != S.ld;
#pragma unroll
  for (int k = 0; k < kZquUnroll; ++k) {
    const size_t i = base + (size_t)k * kZquThreads;
    if (i < n4) {
      Rv[k] = zqu_load(reinterpret_cast<const f32x4*>(S.R) + i);
      zo[k] = zqu_load(reinterpret_cast<const f32x4*>(S.z) + i);
      qo[k] = zqu_load(reinterpret_cast<const f32x4*>(S.q) + i);
      if (p8) {
        pn[k] = load_members4<IB>(p8, i, pgrid);
        if (S.ncols != S.ld) {        // index 0 in a pad column stands for no value
          const int col0 = (int)(i % (size_t)ld4) * 4;
#pragma unroll
          for (int c = 0; c < 4; ++c)
            if (col0 + c >= S.ncols) pn[k][c] = 0.0f;
        }
      } else {
        pn[k] = zqu_load(reinterpret_cast<const f32x4*>(S.pnext) + i);
      }
      uo[k] = zqu_load(reinterpret_cast<const f32x4*>(S.u) + i);
      mm[k] = reinterpret_cast<const f32x4*>(S.m)[i % ld4];
    }
  }
#pragma unroll
  for (int k = 0; k < kZquUnroll; ++k) {
    const size_t i = base + (size_t)k * kZquThreads;
    if (i < n4) {
      f32x4 zn, Rn, qn, un;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const float a = Rv[k][c] - mm[k][c] + zo[k][c];
        const float z = z_closed_form(a + zo[k][c], qo[k][c], slope);
        zn[c] = z;
        Rn[c] = a - z;
        float qq = (rho * pn[k][c] + uo[k][c] + nu * act_fn(z, slope)) * inv_rn;
        if (qgrid.levels > 0) qq = quant_value(quant_index(qq, qgrid), qgrid);   // variant with q on the grid
        const float rr = pn[k][c] - qq;
        qn[c] = qq;
        un[c] = uo[k][c] + rho * rr;
      }
      if (ragged) {
        const int col0 = (int)(i % (size_t)ld4) * 4;
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (col0 + c >= S.ncols) { qn[c] = 0.0f; un[c] = 0.0f; }
      }
      zqu_store(reinterpret_cast<f32x4*>(S.z) + i, zn);
      zqu_store(reinterpret_cast<f32x4*>(S.R) + i, Rn);
      zqu_store(reinterpret_cast<f32x4*>(S.q) + i, qn);
      zqu_store(reinterpret_cast<f32x4*>(S.u) + i, un);
    }
  }
}

// ------------------------------------------------------------------------------------------
// z_L-update: FISTA with a fixed number of steps on CE(z; y) + (nu/2)||z - a||^2, per node.
// A group of G = 2^k lanes (G >= C, G <= 64) owns one node; for C > 64 each lane holds E classes.
// Step 1/(nu + 1/2) (the cross-entropy Hessian is bounded by 1/2). Unlabelled nodes take z = a.
// ------------------------------------------------------------------------------------------
template <int E>
__global__ __launch_bounds__(256) void fista_kernel(float* __restrict__ R, float* __restrict__ z,
                                                    const float* __restrict__ m, const int* __restrict__ y,
                                                    const uint8_t* __restrict__ mask, int rows, int C, int ld,
                                                    int G, float nu, int iters) {
  const int gid = (blockIdx.x * 256 + threadIdx.x) / G;
  const int gl = threadIdx.x % G;
  const bool live = gid < rows;
  const int node = live ? gid : rows - 1;
  const int label = y[node];
  const bool lab = mask ? mask[node] != 0 : true;
  float a[E], x[E], w[E];
  bool valid[E];
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const int c = gl + e * G;
    valid[e] = c < C;
    const size_t i = (size_t)node * ld + (valid[e] ? c : 0);
    const float zo = z[i];
    a[e] = R[i] - m[valid[e] ? c : 0] + zo;
    x[e] = zo;
    w[e] = zo;
  }
  const float inv_lip = 1.0f / (nu + 0.5f);
  double t = 1.0;
  if (lab) {
    for (int it = 0; it < iters; ++it) {
      float mx = -INFINITY;
#pragma unroll
      for (int e = 0; e < E; ++e) if (valid[e]) mx = fmaxf(mx, w[e]);
      for (int off = G >> 1; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, G));
      float ex[E], sum = 0.0f;
#pragma unroll
      for (int e = 0; e < E; ++e) {
        ex[e] = valid[e] ? expf(w[e] - mx) : 0.0f;
        sum += ex[e];
      }
      for (int off = G >> 1; off > 0; off >>= 1) sum += __shfl_xor(sum, off, G);
      const double tn = 0.5 * (1.0 + sqrt(1.0 + 4.0 * t * t));
      const float mom = (float)((t - 1.0) / tn);
#pragma unroll
      for (int e = 0; e < E; ++e) {
        const int c = gl + e * G;
        const float grad = ex[e] / sum - (c == label ? 1.0f : 0.0f) + nu * (w[e] - a[e]);
        const float xn = w[e] - grad * inv_lip;
        w[e] = xn + mom * (xn - x[e]);
        x[e] = xn;
      }
      t = tn;
    }
  } else {
#pragma unroll
    for (int e = 0; e < E; ++e) x[e] = a[e];
  }
  if (live) {
#pragma unroll
    for (int e = 0; e < E; ++e) {
      if (valid[e]) {
        const size_t i = (size_t)node * ld + gl + e * G;
        z[i] = x[e];
        R[i] = a[e] - x[e];
      }
    }
  }
}

// z_L-update for the least-squares risk R(z; y) = 1/2 sum_j ||z_j - e_{y_j}||^2 (Section 3.1 admits any convex
// continuous risk): the subproblem 1/2 ||z - e_y||^2 + (nu/2)||z - a||^2 of Appendix A 'update z' (l = L) has
// the closed form z = (e_y + nu a) / (1 + nu); unlabelled nodes take z = a. One thread per element.
__global__ __launch_bounds__(256) void zlast_ls_kernel(float* __restrict__ R, float* __restrict__ z,
                                                       const float* __restrict__ m, const int* __restrict__ y,
                                                       const uint8_t* __restrict__ mask, int rows, int C, int ld,
                                                       float nu) {
  const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
  const int node = (int)(e / (size_t)C), c = (int)(e % (size_t)C);
  if (node >= rows) return;
  const size_t i = (size_t)node * ld + c;
  const float a = R[i] - m[c] + z[i];
  const bool lab = mask ? mask[node] != 0 : true;
  const float zn = lab ? ((c == y[node] ? 1.0f : 0.0f) + nu * a) / (1.0f + nu) : a;
  z[i] = zn;
  R[i] = a - zn;
}

// ------------------------------------------------------------------------------------------
// pdADMM-G-Q p-update (Appendix B): p <- argmin_{delta in Delta} |delta - (p - g/tau)|.
// One backtracking trial: candidate indices, d = candidate - p, per-block ||d||^2.
// ------------------------------------------------------------------------------------------
struct QuantSeg {
  uint8_t* p8;        // the two index planes of p_l, [2][plane]: LayerScal::cur selects the one that holds p_l, the
                      // other takes the candidate of the trial in flight
  size_t p8_plane;
  const float* g;
  float* d;
  double* dpart;      // per block
  size_t n4;          // rows*ld/4
  int ncols, ld;
  int blk0, nblk;
  int layer;
};

// A block owns kQuantUnroll * 256 consecutive float4 groups (one contiguous chunk per array); all loads of a
// thread are issued before the first projection.
// 256 threads x 2 groups (C5: 3.36 ms; 256x1 3.53, 256x4 3.45, one-wave blocks 4.49 / 4.08 / 3.49 ms for 1 / 2 / 4 groups:
// the launches of a round that no layer needs any more are cheaper with fewer blocks)
constexpr int kQuantUnroll = 2;
constexpr int kQtThreads = 256;

template <int IB>
__global__ __launch_bounds__(kQtThreads) void quant_trial_kernel(const QuantSeg* __restrict__ segs, const BlockMap map,
                                                          const LayerScal* __restrict__ scal, QuantGrid grid) {
  __shared__ double red[4];
  int local;
  const int si = find_group(map, blockIdx.x, &local);
  const QuantSeg S = segs[si];
  if (!scal[S.layer].active) return;
  const float t = scal[S.layer].trial_t;
  const int cur = scal[S.layer].cur;
  const uint8_t* pin = S.p8 + (size_t)cur * S.p8_plane;
  uint8_t* pout = S.p8 + (size_t)(cur ^ 1) * S.p8_plane;
  const size_t base = (size_t)local * (kQtThreads * kQuantUnroll) + threadIdx.x;
  f32x4 pv[kQuantUnroll], gv[kQuantUnroll];
#pragma unroll
  for (int j = 0; j < kQuantUnroll; ++j) {
    const size_t i = base + (size_t)j * kQtThreads;
    if (i < S.n4) {
      pv[j] = load_members4<IB>(pin, i, grid);
      gv[j] = stream_load(reinterpret_cast<const f32x4*>(S.g) + i);
    }
  }
  double ds = 0.0;
#pragma unroll
  for (int j = 0; j < kQuantUnroll; ++j) {
    const size_t i = base + (size_t)j * kQtThreads;
    if (i >= S.n4) continue;
    const int col0 = (int)((i * 4) % (size_t)S.ld);
    f32x4 dv;
    struct { int x, y, z, w; } iv;
#define PDADMM_QT(c, k)                                                       \
  {                                                                           \
    if (col0 + k < S.ncols) {                                                 \
      const float v = sub_rn(pv[j].c, div_rn(gv[j].c, t));                    \
      const int id = quant_index(v, grid);                                    \
      iv.c = id;                                                              \
      dv.c = sub_rn(quant_value(id, grid), pv[j].c);                          \
      ds += (double)dv.c * (double)dv.c;                                      \
    } else {                                                                  \
      iv.c = 0;                                                               \
      dv.c = 0.0f;                                                            \
    }                                                                         \
  }
    PDADMM_QT(x, 0) PDADMM_QT(y, 1) PDADMM_QT(z, 2) PDADMM_QT(w, 3)
#undef PDADMM_QT
    reinterpret_cast<f32x4*>(S.d)[i] = dv;       // re-read by the product W d that follows
    store_indices4(pout, i, IB, iv.x, iv.y, iv.z, iv.w);
  }
  const double tot = kQtThreads == 64 ? wave_sum(ds) : block_sum_256(ds, red);
  if (threadIdx.x == 0) S.dpart[local] = tot;
}

// Accept/reject one -Q trial: phi(p+d) - phi(p) - <g,d> = (nu/2)||W d||^2 + (rho/2)||d||^2 exactly,
// so the condition phi(p_new) <= U_l(p_new; t) is  nu||W d||^2 + rho||d||^2 <= t ||d||^2.
// phase 0: arm the search (active = 1, trial_t = tau/eta, or tau while a rejected probe of the smaller
//          value is being waited out) for layers with g != 0.
// phase 1: judge the trial in flight.
__global__ __launch_bounds__(256) void select_quant_kernel(const SelectDesc* __restrict__ descs, LayerScal* scal,
                                                           int phase, float rho, float nu, float eta,
                                                           int max_trials, int backoff, int* err, int* flags) {
  __shared__ double red[4];
  const SelectDesc D = descs[blockIdx.x];
  LayerScal& sc = scal[D.layer];
  if (phase == 0) {
    const double sg = fixed_order_sum(D.part_g, D.ng, 1, red);
    if (threadIdx.x != 0) return;
    sc.norm_g = sg;
    sc.inv_tau = 0.0f;
    sc.p_trials = 0;
    sc.active = 0;
    if (!(sg == sg) || sg > 1.7e308) atomicOr(err, kErrNonFinite);
    else if (sg > 0.0) {
      // every trial costs a product W d: with the back-off schedule tau/eta is only probed when no rejected
      // probe is being waited out; the plain schedule starts every update at tau/eta
      const int probing = !backoff || sc.probe_skip == 0;
      if (!probing) sc.probe_skip -= 1;
      sc.probing = probing;
      sc.active = 1;
      sc.trial_t = (float)(probing ? sc.tau / (double)eta : sc.tau);
      sc.p_trials = 1;
    }
    flags[D.layer] = sc.active;
    return;
  }
  if (!sc.active) return;      // uniform per block
  const double sd = fixed_order_sum(D.part_g, D.ng, 1, red);
  const double st = fixed_order_sum(D.part_t, D.nt, D.stride_t, red);
  if (threadIdx.x != 0) return;
  sc.norm_t = st;
  sc.products += 1;
  const double t = (double)sc.trial_t;
  if (!(sd == sd) || !(st == st) || sd > 1.7e308 || st > 1.7e308) {
    atomicOr(err, kErrNonFinite);
    sc.active = 0;
    sc.p_trials = 0;
  } else if ((double)nu * st + (double)rho * sd <= t * sd) {
    sc.tau = t;
    sc.inv_tau = 1.0f;     // marks "a step was accepted"
    sc.active = 0;
    sc.cur ^= 1;           // the plane the accepted candidate was written to now holds p_l
    if (backoff && sc.probing) {   // accepted at once: probe again next time; else back off 1, 2, 4, ... iterations
      if (sc.p_trials == 1) sc.probe_wait = 0;
      else {
        sc.probe_wait = min(max(1, 2 * sc.probe_wait), kProbeCap);
        sc.probe_skip = sc.probe_wait;
      }
    }
  } else if (sc.p_trials >= max_trials) {
    atomicOr(err, kErrBacktrack);
    sc.active = 0;
    sc.p_trials = 0;
  } else {
    sc.trial_t = (float)(t * (double)eta);
    sc.p_trials += 1;
  }
  flags[D.layer] = sc.active;
}

// Values of a [rows, ld] array of indices (ncols valid columns, pad columns give 0): p_l for pdadmm_get_var.
__global__ __launch_bounds__(256) void dequantize_kernel(const uint8_t* __restrict__ idx, size_t n4, int ncols, int ld,
                                                         QuantGrid grid, float* __restrict__ val) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
    f32x4 v = load_members4(idx, i, grid);
    const int col0 = (int)((i * 4) % (size_t)ld);
#pragma unroll
    for (int c = 0; c < 4; ++c)
      if (col0 + c >= ncols) v[c] = 0.0f;
    reinterpret_cast<f32x4*>(val)[i] = v;
  }
}

// Standalone projection of a [rows, ld] array (ncols valid columns): writes indices and/or values.
__global__ __launch_bounds__(256) void quantize_kernel(const float* __restrict__ v, size_t n4, int ncols, int ld,
                                                       QuantGrid grid, uint8_t* __restrict__ idx,
                                                       float* __restrict__ val) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
    const float4 x = reinterpret_cast<const float4*>(v)[i];
    const int col0 = (int)((i * 4) % (size_t)ld);
    const int i0 = col0 + 0 < ncols ? quant_index(x.x, grid) : 0;
    const int i1 = col0 + 1 < ncols ? quant_index(x.y, grid) : 0;
    const int i2 = col0 + 2 < ncols ? quant_index(x.z, grid) : 0;
    const int i3 = col0 + 3 < ncols ? quant_index(x.w, grid) : 0;
    if (idx) store_indices4(idx, i, grid.ib, i0, i1, i2, i3);
    if (val) {
      float4 o;
      o.x = col0 + 0 < ncols ? quant_value(i0, grid) : 0.0f;
      o.y = col0 + 1 < ncols ? quant_value(i1, grid) : 0.0f;
      o.z = col0 + 2 < ncols ? quant_value(i2, grid) : 0.0f;
      o.w = col0 + 3 < ncols ? quant_value(i3, grid) : 0.0f;
      reinterpret_cast<float4*>(val)[i] = o;
    }
  }
}
// Scalar variant for arrays whose length or alignment rules out float4 access.
__global__ __launch_bounds__(256) void quantize_scalar_kernel(const float* __restrict__ v, size_t n, QuantGrid grid,
                                                              uint8_t* __restrict__ idx, float* __restrict__ val) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
    const int id = quant_index(v[i], grid);
    if (idx) {
      if (grid.ib == 2) reinterpret_cast<uint16_t*>(idx)[i] = (uint16_t)id;
      else idx[i] = (uint8_t)id;
    }
    if (val) val[i] = quant_value(id, grid);
  }
}

// ------------------------------------------------------------------------------------------
// Reductions behind the objective (Section 3.2, L_rho) and the residual (Algorithm 1).
// Per block three partials: sum (q - f(z))^2, sum u (p_next - q), sum (p_next - q)^2.
// ------------------------------------------------------------------------------------------
struct PairSeg {
  const float* z;
  const float* q;
  const float* u;
  const float* pnext;
  const uint8_t* pnext8;   // -Q: index planes of p_{l+1} in place of pnext (see RowSeg)
  size_t p8_plane;
  int next_layer, ncols, ld;
  double* part;       // 3 per block
  size_t n4;
  int blk0, nblk;
};

__global__ __launch_bounds__(256) void pair_reduce_kernel(const PairSeg* __restrict__ segs, const BlockMap map,
                                                          const LayerScal* __restrict__ scal, float slope,
                                                          const QuantGrid pgrid) {
  __shared__ double red[4];
  int local;
  const int si = find_group(map, blockIdx.x, &local);
  const PairSeg S = segs[si];
  const uint8_t* p8 = S.pnext8 ? S.pnext8 + (size_t)scal[S.next_layer].cur * S.p8_plane : nullptr;
  const size_t stride = (size_t)S.nblk * 256;
  double s_act = 0, s_dl = 0, s_dq = 0;
  for (size_t i = (size_t)local * 256 + threadIdx.x; i < S.n4; i += stride) {
    const float4 z = reinterpret_cast<const float4*>(S.z)[i];
    const float4 q = reinterpret_cast<const float4*>(S.q)[i];
    const float4 u = reinterpret_cast<const float4*>(S.u)[i];
    float4 p;
    if (p8) {
      const f32x4 v = load_members4(p8, i, pgrid);
      const int col0 = (int)((i * 4) % (size_t)S.ld);
      p.x = col0 + 0 < S.ncols ? v.x : 0.0f;
      p.y = col0 + 1 < S.ncols ? v.y : 0.0f;
      p.z = col0 + 2 < S.ncols ? v.z : 0.0f;
      p.w = col0 + 3 < S.ncols ? v.w : 0.0f;
    } else {
      p = reinterpret_cast<const float4*>(S.pnext)[i];
    }
#define PDADMM_PR(c)                                              \
  {                                                               \
    const double a = (double)q.c - (double)act_fn(z.c, slope);    \
    const double r = (double)p.c - (double)q.c;                   \
    s_act += a * a;                                               \
    s_dl += (double)u.c * r;                                      \
    s_dq += r * r;                                                \
  }
    PDADMM_PR(x) PDADMM_PR(y) PDADMM_PR(z) PDADMM_PR(w)
#undef PDADMM_PR
  }
  const double t0 = block_sum_256(s_act, red);
  const double t1 = block_sum_256(s_dl, red);
  const double t2 = block_sum_256(s_dq, red);
  if (threadIdx.x == 0) {
    double* o = S.part + (size_t)local * 3;
    o[0] = t0; o[1] = t1; o[2] = t2;
  }
}

// R(z_L; y) summed over labelled nodes: logsumexp(z) - z_y (cross-entropy, kind 0) or
// 1/2 ||z - e_y||^2 (least squares, kind 1). One thread per node.
__global__ __launch_bounds__(256) void risk_kernel(const float* __restrict__ z, const int* __restrict__ y,
                                                   const uint8_t* __restrict__ mask, int rows, int C, int ld,
                                                   int kind, double* __restrict__ part) {
  __shared__ double red[4];
  const int node = blockIdx.x * 256 + threadIdx.x;
  double v = 0.0;
  if (node < rows && (!mask || mask[node])) {
    const float* zr = z + (size_t)node * ld;
    if (kind == 0) {
      float mx = zr[0];
      for (int c = 1; c < C; ++c) mx = fmaxf(mx, zr[c]);
      double s = 0.0;
      for (int c = 0; c < C; ++c) s += exp((double)zr[c] - (double)mx);
      v = (double)mx + log(s) - (double)zr[y[node]];
    } else {
      const int label = y[node];
      for (int c = 0; c < C; ++c) {
        const double d = (double)zr[c] - (c == label ? 1.0 : 0.0);
        v += 0.5 * d * d;
      }
    }
  }
  const double t = block_sum_256(v, red);
  if (threadIdx.x == 0) part[blockIdx.x] = t;
}

// Predicted class per node = first maximum of the output layer's row; per block the number of
// counted nodes (mask != 0, or all) and of those the number whose prediction equals the label.
__global__ __launch_bounds__(256) void argmax_kernel(const float* __restrict__ z, int rows, int C, int ld,
                                                     const int* __restrict__ y, const uint8_t* __restrict__ mask,
                                                     int* __restrict__ pred, double* __restrict__ part) {
  __shared__ double red[4];
  const int node = blockIdx.x * 256 + threadIdx.x;
  double counted = 0.0, correct = 0.0;
  if (node < rows) {
    const float* zr = z + (size_t)node * ld;
    int best = 0;
    float bv = zr[0];
    for (int c = 1; c < C; ++c) {
      const float v = zr[c];
      if (v > bv) { bv = v; best = c; }
    }
    if (pred) pred[node] = best;
    if (!mask || mask[node]) {
      counted = 1.0;
      correct = best == y[node] ? 1.0 : 0.0;
    }
  }
  const double t0 = block_sum_256(counted, red);
  const double t1 = block_sum_256(correct, red);
  if (threadIdx.x == 0) {
    part[2 * blockIdx.x] = t0;
    part[2 * blockIdx.x + 1] = t1;
  }
}

}  // namespace pdadmm
