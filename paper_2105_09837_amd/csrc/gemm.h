// Grouped fp32 GEMM on the CDNA4 matrix cores (v_mfma_f32_32x32x2_f32), wave64.
//
// One launch covers a list of independent problems (one per layer: the paper's layer-wise
// independence, Algorithm 1 "for different l in parallel"). Two operand layouts:
//   KCONTIG = true : C[M,N] = sum_k A[m*lda + k] * B[n*ldb + k]      ("NT": W p, W^T r, G p)
//   KCONTIG = false: C[M,N] = sum_k A[k*lda + m] * B[k*ldb + n]      ("TN": r p^T, split over k)
// Block tile 128x128x16, 4 waves in a 2x2 arrangement, each wave owns 64x64 = 2x2 MFMA blocks.
// Operands are staged in LDS as [k][m] so that the MFMA operand fetch (lane -> row lane%32,
// k = lane/32) is a conflict-free 4-byte read. Global loads of tile t+1 are issued before the
// MFMAs of tile t (register double buffering, two LDS buffers, one barrier per tile).
#pragma once
#include "common.h"

namespace pdadmm {

constexpr int BM = 128, BN = 128, BK = 16;
constexpr int LDM = BM + 4;   // LDS row stride in floats (keeps float4 rows 16-byte aligned)

typedef float floatx16 __attribute__((ext_vector_type(16)));

struct GemmProb {
  const float* A;
  const float* B;
  float* C;
  int M, N, K;
  int lda, ldb, ldc;
  int tiles_m, tiles_n, splitk, k_chunk;
  int blk0, nblk;
  int layer;          // LayerScal index consulted when the launch is predicated, else unused
  int vecA, vecB;     // 1 if 16-byte vector loads are legal for this operand
  const float* e0;    // epilogue inputs (meaning depends on the epilogue)
  const float* e1;
  const float* e2;
  float* o1;          // extra epilogue outputs
  float* o2;
  double* part;       // per-block partial sums, NS doubles per block
  float alpha, beta;
  QuantGrid grid;     // used by the forward epilogue in -Q mode (levels = 0: off)
};

// ---- epilogues: apply(P, row, col, acc, s0, s1) is called once per in-range output element
struct EpiStore {     // C = alpha * acc
  static constexpr int NS = 0;
  __device__ static __forceinline__ void apply(const GemmProb& P, float* C, int row, int col, float acc,
                                               double&, double&) {
    C[(size_t)row * P.ldc + col] = P.alpha * acc;
  }
};
struct EpiStoreNorm { // C = acc, s0 += acc^2
  static constexpr int NS = 1;
  __device__ static __forceinline__ void apply(const GemmProb& P, float* C, int row, int col, float acc,
                                               double& s0, double&) {
    C[(size_t)row * P.ldc + col] = acc;
    s0 += (double)acc * (double)acc;
  }
};
struct EpiPGrad {     // g = nu*acc + u + rho*(p - q) (gradient of phi in p_l); s0 += g^2
  static constexpr int NS = 1;
  __device__ static __forceinline__ void apply(const GemmProb& P, float* C, int row, int col, float acc,
                                               double& s0, double&) {
    const size_t i = (size_t)row * P.ldc + col;
    const float g = P.alpha * acc + P.e0[i] + P.beta * (P.e1[i] - P.e2[i]);
    C[i] = g;
    s0 += (double)g * (double)g;
  }
};
struct EpiResid {     // r = acc + b[col] - z; s0 += r^2; s1 += (r - carried)^2 when e2 != null
  static constexpr int NS = 2;
  __device__ static __forceinline__ void apply(const GemmProb& P, float* C, int row, int col, float acc,
                                               double& s0, double& s1) {
    const size_t i = (size_t)row * P.ldc + col;
    const float r = acc + P.e0[col] - P.e1[i];
    C[i] = r;
    s0 += (double)r * (double)r;
    if (P.e2) {
      const double d = (double)r - (double)P.e2[i];
      s1 += d * d;
    }
  }
};
struct EpiForward {   // z = acc + b[col]; q = relu(z); p_next = relu(z) (projected onto the grid in -Q)
  static constexpr int NS = 0;
  __device__ static __forceinline__ void apply(const GemmProb& P, float* C, int row, int col, float acc,
                                               double&, double&) {
    const size_t i = (size_t)row * P.ldc + col;
    const float z = acc + P.e0[col];
    C[i] = z;
    if (P.o1) {
      const float a = fmaxf(z, 0.0f);
      P.o1[i] = a;
      P.o2[i] = P.grid.levels > 0 ? quant_value(quant_index(a, P.grid), P.grid) : a;
    }
  }
};

template <bool KCONTIG, class Epi>
__device__ __forceinline__ void gemm_body(const GemmProb& P, const int local) {
  __shared__ __attribute__((aligned(16))) float As[2][BK][LDM];
  __shared__ __attribute__((aligned(16))) float Bs[2][BK][LDM];
  __shared__ double red[4];

  const int tiles = P.tiles_m * P.tiles_n;
  const int split = local / tiles;
  const int t2 = local - split * tiles;
  const int tm = t2 / P.tiles_n, tn = t2 - tm * P.tiles_n;
  const int m0 = tm * BM, n0 = tn * BN;
  const int kbeg = split * P.k_chunk;
  const int kend = min(P.K, kbeg + P.k_chunk);
  const int nkt = kend > kbeg ? (kend - kbeg + BK - 1) / BK : 0;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int li = lane & 31, lh = lane >> 5;

  float4 ra[2], rb[2];

  auto load_tile = [&](int kt) {
    const int kb = kbeg + kt * BK;
    if (KCONTIG) {
      const int r = tid >> 2, kq = (tid & 3) * 4;
      const int k = kb + kq;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int ma = m0 + r + 64 * h, nb = n0 + r + 64 * h;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (ma < P.M && k < kend) {
          const float* src = P.A + (size_t)ma * P.lda + k;
          if (P.vecA && k + 3 < kend) v = *reinterpret_cast<const float4*>(src);
          else {
            v.x = src[0];
            if (k + 1 < kend) v.y = src[1];
            if (k + 2 < kend) v.z = src[2];
            if (k + 3 < kend) v.w = src[3];
          }
        }
        ra[h] = v;
        v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (nb < P.N && k < kend) {
          const float* src = P.B + (size_t)nb * P.ldb + k;
          if (P.vecB && k + 3 < kend) v = *reinterpret_cast<const float4*>(src);
          else {
            v.x = src[0];
            if (k + 1 < kend) v.y = src[1];
            if (k + 2 < kend) v.z = src[2];
            if (k + 3 < kend) v.w = src[3];
          }
        }
        rb[h] = v;
      }
    } else {
      const int kr = tid >> 5, mq = (tid & 31) * 4;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int k = kb + kr + 8 * h;
        const int ma = m0 + mq, nb = n0 + mq;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (k < kend && ma < P.M) {
          const float* src = P.A + (size_t)k * P.lda + ma;
          if (P.vecA && ma + 3 < P.M) v = *reinterpret_cast<const float4*>(src);
          else {
            v.x = src[0];
            if (ma + 1 < P.M) v.y = src[1];
            if (ma + 2 < P.M) v.z = src[2];
            if (ma + 3 < P.M) v.w = src[3];
          }
        }
        ra[h] = v;
        v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (k < kend && nb < P.N) {
          const float* src = P.B + (size_t)k * P.ldb + nb;
          if (P.vecB && nb + 3 < P.N) v = *reinterpret_cast<const float4*>(src);
          else {
            v.x = src[0];
            if (nb + 1 < P.N) v.y = src[1];
            if (nb + 2 < P.N) v.z = src[2];
            if (nb + 3 < P.N) v.w = src[3];
          }
        }
        rb[h] = v;
      }
    }
  };

  auto store_tile = [&](int buf) {
    if (KCONTIG) {
      const int r = tid >> 2, kq = (tid & 3) * 4;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int c = r + 64 * h;
        As[buf][kq + 0][c] = ra[h].x;
        As[buf][kq + 1][c] = ra[h].y;
        As[buf][kq + 2][c] = ra[h].z;
        As[buf][kq + 3][c] = ra[h].w;
        Bs[buf][kq + 0][c] = rb[h].x;
        Bs[buf][kq + 1][c] = rb[h].y;
        Bs[buf][kq + 2][c] = rb[h].z;
        Bs[buf][kq + 3][c] = rb[h].w;
      }
    } else {
      const int kr = tid >> 5, mq = (tid & 31) * 4;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        *reinterpret_cast<float4*>(&As[buf][kr + 8 * h][mq]) = ra[h];
        *reinterpret_cast<float4*>(&Bs[buf][kr + 8 * h][mq]) = rb[h];
      }
    }
  };

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  if (nkt > 0) {
    load_tile(0);
    store_tile(0);
    __syncthreads();
    for (int kt = 0; kt < nkt; ++kt) {
      const int cur = kt & 1;
      if (kt + 1 < nkt) load_tile(kt + 1);
#pragma unroll
      for (int kk = 0; kk < BK; kk += 2) {
        const float a0 = As[cur][kk + lh][wm * 64 + li];
        const float a1 = As[cur][kk + lh][wm * 64 + 32 + li];
        const float b0 = Bs[cur][kk + lh][wn * 64 + li];
        const float b1 = Bs[cur][kk + lh][wn * 64 + 32 + li];
        acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
        acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
        acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
        acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
      }
      if (kt + 1 < nkt) store_tile(cur ^ 1);
      __syncthreads();
    }
  }

  // Epilogue. MFMA 32x32 output layout: register v of lane l holds
  // row 8*(v/4) + 4*(l/32) + v%4, column l%32 of the 32x32 block.
  float* Cout = P.C + (size_t)split * (size_t)P.M * (size_t)P.ldc;
  double s0 = 0.0, s1 = 0.0;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int col = n0 + wn * 64 + j * 32 + li;
      if (col < P.N) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = m0 + wm * 64 + i * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
          if (row < P.M) Epi::apply(P, Cout, row, col, acc[i][j][v], s0, s1);
        }
      }
    }
  if (Epi::NS >= 1) {
    const double t0 = block_sum_256(s0, red);
    if (tid == 0) P.part[(size_t)local * Epi::NS] = t0;
  }
  if (Epi::NS >= 2) {
    const double t1 = block_sum_256(s1, red);
    if (tid == 0) P.part[(size_t)local * Epi::NS + 1] = t1;
  }
}

// Grouped launch: block -> (problem, tile) through the table; blocks of one die are contiguous.
template <bool KCONTIG, class Epi>
__global__ __launch_bounds__(256) void gemm_kernel(const GemmProb* __restrict__ probs, int nprob, int total,
                                                   const LayerScal* __restrict__ scal, int predicated) {
  const int lb = xcd_remap(blockIdx.x, total);
  int pi = 0;
  while (pi + 1 < nprob && lb >= probs[pi + 1].blk0) ++pi;
  const GemmProb P = probs[pi];
  if (predicated && !scal[P.layer].active) return;
  gemm_body<KCONTIG, Epi>(P, lb - P.blk0);
}

// Single problem with the descriptor passed by value (no table in device memory needed).
template <bool KCONTIG, class Epi>
__global__ __launch_bounds__(256) void gemm_one_kernel(const GemmProb P) {
  gemm_body<KCONTIG, Epi>(P, xcd_remap(blockIdx.x, P.nblk));
}

// Sum the split-K partial products in a fixed order: G = alpha * sum_s part[s]; also write the
// transposed copy when Gt != null; per-block partial of ||G||_F^2.
struct ReduceProb {
  const float* part;   // [splitk][M][ld]
  float* G;            // [M][ld]
  double* norm_part;   // per block
  int M, N, ld, splitk;
  int blk0, nblk;
  float alpha;
};

__device__ __forceinline__ void splitk_reduce_body(const ReduceProb& P, const int local) {
  __shared__ double red[4];
  const size_t plane = (size_t)P.M * P.ld;
  double s = 0.0;
  for (size_t i = (size_t)local * 256 + threadIdx.x; i < plane; i += (size_t)P.nblk * 256) {
    const int col = (int)(i % P.ld);
    float sum = 0.0f;
    if (col < P.N) {
      for (int k = 0; k < P.splitk; ++k) sum += P.part[(size_t)k * plane + i];
      sum *= P.alpha;
    }
    P.G[i] = sum;
    s += (double)sum * (double)sum;
  }
  const double t = block_sum_256(s, red);
  if (threadIdx.x == 0 && P.norm_part) P.norm_part[local] = t;
}

__global__ __launch_bounds__(256) void splitk_reduce_kernel(const ReduceProb* __restrict__ probs, int nprob) {
  const int lb = blockIdx.x;
  int pi = 0;
  while (pi + 1 < nprob && lb >= probs[pi + 1].blk0) ++pi;
  const ReduceProb P = probs[pi];
  splitk_reduce_body(P, lb - P.blk0);
}
__global__ __launch_bounds__(256) void splitk_reduce_one_kernel(const ReduceProb P) {
  splitk_reduce_body(P, blockIdx.x);
}

}  // namespace pdadmm
