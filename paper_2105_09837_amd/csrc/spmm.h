// CSR SpMM for the multi-hop feature augmentation X_k = A~ X_{k-1} (Sections 3.1, 5.1).
// One thread owns VEC consecutive feature columns of one node and walks the node's CSR row in
// order; neighbouring threads own neighbouring column groups, so every gathered row segment is
// a coalesced read. Products and sums are rounded separately (no FMA): the result is fixed bit
// for bit by the CSR order.
#pragma once
#include "common.h"

namespace pdadmm {

// The sum over a row is sequential by definition (fp32, CSR order), but the gathers are independent:
// they are issued in batches of kSpmmBatch edges before the ordered multiply-adds consume them, so a
// hub row of a power-law graph (thousands of entries) costs a few memory round trips, not one per entry.
constexpr int kSpmmBatch = 16;

template <int VEC>
__global__ __launch_bounds__(256) void spmm_hop_kernel(int n, const int* __restrict__ rowptr,
                                                       const int* __restrict__ colidx,
                                                       const float* __restrict__ vals,
                                                       const float* __restrict__ src,  // block k-1, row stride ld
                                                       float* __restrict__ dst,        // block k,   row stride ld
                                                       int d, int ld) {
  const int groups = (d + VEC - 1) / VEC;
  const size_t item = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (item >= (size_t)n * groups) return;
  const int row = (int)(item / groups);
  const int c0 = (int)(item % groups) * VEC;
  const int beg = rowptr[row], end = rowptr[row + 1];
  if (VEC == 4) {
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    int e = beg;
    for (; e + kSpmmBatch <= end; e += kSpmmBatch) {
      float a[kSpmmBatch];
      float4 x[kSpmmBatch];
#pragma unroll
      for (int k = 0; k < kSpmmBatch; ++k) {
        a[k] = vals[e + k];
        x[k] = *reinterpret_cast<const float4*>(src + (size_t)colidx[e + k] * ld + c0);
      }
#pragma unroll
      for (int k = 0; k < kSpmmBatch; ++k) {
        acc.x = add_rn(acc.x, mul_rn(a[k], x[k].x));
        acc.y = add_rn(acc.y, mul_rn(a[k], x[k].y));
        acc.z = add_rn(acc.z, mul_rn(a[k], x[k].z));
        acc.w = add_rn(acc.w, mul_rn(a[k], x[k].w));
      }
    }
    for (; e + 4 <= end; e += 4) {
      float a[4];
      float4 x[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        a[k] = vals[e + k];
        x[k] = *reinterpret_cast<const float4*>(src + (size_t)colidx[e + k] * ld + c0);
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        acc.x = add_rn(acc.x, mul_rn(a[k], x[k].x));
        acc.y = add_rn(acc.y, mul_rn(a[k], x[k].y));
        acc.z = add_rn(acc.z, mul_rn(a[k], x[k].z));
        acc.w = add_rn(acc.w, mul_rn(a[k], x[k].w));
      }
    }
    for (; e < end; ++e) {
      const float a = vals[e];
      const float4 x = *reinterpret_cast<const float4*>(src + (size_t)colidx[e] * ld + c0);
      acc.x = add_rn(acc.x, mul_rn(a, x.x));
      acc.y = add_rn(acc.y, mul_rn(a, x.y));
      acc.z = add_rn(acc.z, mul_rn(a, x.z));
      acc.w = add_rn(acc.w, mul_rn(a, x.w));
    }
    *reinterpret_cast<float4*>(dst + (size_t)row * ld + c0) = acc;
  } else {
    float acc = 0.f;
    int e = beg;
    for (; e + 8 <= end; e += 8) {
      float a[8], x[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        a[k] = vals[e + k];
        x[k] = src[(size_t)colidx[e + k] * ld + c0];
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) acc = add_rn(acc, mul_rn(a[k], x[k]));
    }
    for (; e < end; ++e)
      acc = add_rn(acc, mul_rn(vals[e], src[(size_t)colidx[e] * ld + c0]));
    dst[(size_t)row * ld + c0] = acc;
  }
}

}  // namespace pdadmm
