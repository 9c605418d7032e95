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
  double* colpart;    // per row-tile column sums of the updated residual, [tiles_m][ldc] (EpiTrialW)
  float alpha, beta;
  float slope;        // negative-side slope of the activation (epilogues that apply f)
  QuantGrid grid;     // Delta in -Q mode (levels = 0: off): forward epilogue, and wherever p_l is read as indices
  // -Q: p_l (l >= 2) exists only as 8-bit indices into Delta, in two planes of p8_plane bytes each; the plane
  // that holds p_l is LayerScal::cur of `layer` (the grouped kernel adds cur * p8_plane to p8 before use).
  // Which role p8 plays is fixed by the kernel: the k-contiguous A operand or the m-contiguous B operand in
  // place of A / B (template flag P8), or the epilogue's p input (EpiPGradQ).
  const uint8_t* p8;
  size_t p8_plane;
  uint8_t* o8;        // forward epilogue in -Q mode: indices of p_{l+1} (in place of the values in o2)
};

// ---- epilogues. For one in-range output element (flat index i = row*ldc + col): load(P, i, col) fetches
// the element's extra inputs, apply(P, C, i, col, acc, in, s0, s1) forms and stores the result. The
// tile epilogue calls load for a batch of elements before any apply, so the loads of a batch are in
// flight together (a store between two loads would order them: the compiler cannot rule out aliasing).
struct NoIn {};
struct EpiStore {     // C = alpha * acc
  static constexpr int NS = 0, kBatch = 1;
  static constexpr bool kVec = true;
  typedef NoIn In;
  typedef NoIn In4;
  static constexpr bool kExtra = false, kColsum = false;
  static constexpr int kScale = 0;
  __device__ static __forceinline__ In4 load4(const GemmProb&, size_t) { return In4{}; }
  __device__ static __forceinline__ f32x4 apply4(const GemmProb& P, f32x4 acc, const In4&, float, f32x4&) {
    return P.alpha * acc;
  }
  __device__ static __forceinline__ In load(const GemmProb&, size_t, int) { return In{}; }
  __device__ static __forceinline__ void apply(const GemmProb& P, float* C, size_t i, int, float acc,
                                               const In&, double&, double&) {
    ((float PD_GLOBAL*)C)[i] = P.alpha * acc;
  }
};
struct EpiStoreNorm { // C = acc, s0 += acc^2
  static constexpr int NS = 1, kBatch = 1;
  static constexpr bool kVec = true;
  typedef NoIn In;
  typedef NoIn In4;
  static constexpr bool kExtra = false, kColsum = false;
  static constexpr int kScale = 0;
  __device__ static __forceinline__ In4 load4(const GemmProb&, size_t) { return In4{}; }
  __device__ static __forceinline__ f32x4 apply4(const GemmProb&, f32x4 acc, const In4&, float, f32x4&) { return acc; }
  __device__ static __forceinline__ In load(const GemmProb&, size_t, int) { return In{}; }
  __device__ static __forceinline__ void apply(const GemmProb&, float* C, size_t i, int, float acc,
                                               const In&, double& s0, double&) {
    ((float PD_GLOBAL*)C)[i] = acc;
    s0 += (double)acc * (double)acc;
  }
};
// g = nu*acc + u + rho*(p - q) (gradient of phi in p_l); s0 += g^2. With UPD (pdADMM-G) the same pass
// also takes the step p -= g * s_prev with the 1/tau guessed ahead (o1 = p, in place; the old p was read
// for g), corrected later if the selection picks another tau (see EpiTrialUpd).
template <bool UPD>
struct EpiPGradT {
  static constexpr int NS = 1, kBatch = 4;   // elements whose inputs are fetched together (8 would cost the third block per compute unit)
  static constexpr bool kVec = true, kExtra = UPD, kColsum = false;
  static constexpr int kScale = UPD ? 1 : 0;
  struct In { float u, p, q; };
  struct In4 { f32x4 u, p, q; };
  __device__ static __forceinline__ In load(const GemmProb& P, size_t i, int) {
    return In{((gcf)P.e0)[i], ((gcf)P.e1)[i], ((gcf)P.e2)[i]};
  }
  __device__ static __forceinline__ void apply(const GemmProb& P, float* C, size_t i, int, float acc, const In& in,
                                               double& s0, double&) {
    const float g = P.alpha * acc + in.u + P.beta * (in.p - in.q);
    ((float PD_GLOBAL*)C)[i] = g;
    s0 += (double)g * (double)g;
  }
  __device__ static __forceinline__ In4 load4(const GemmProb& P, size_t i) {
    return In4{*reinterpret_cast<gcf4>((gcf)P.e0 + i), *reinterpret_cast<gcf4>((gcf)P.e1 + i),
               *reinterpret_cast<gcf4>((gcf)P.e2 + i)};
  }
  __device__ static __forceinline__ f32x4 apply4(const GemmProb& P, f32x4 acc, const In4& in, float s_prev, f32x4& extra) {
    const f32x4 g = P.alpha * acc + in.u + P.beta * (in.p - in.q);
    if (UPD) extra = in.p - s_prev * g;
    return g;
  }
};
typedef EpiPGradT<false> EpiPGrad;
typedef EpiPGradT<true> EpiPGradUpd;

// The same gradient in -Q mode, where p_l is read as indices into Delta (P.p8, IB bytes each) and becomes a
// value here.
template <int IB>
struct EpiPGradQT {
  static constexpr int NS = 1, kBatch = 4;
  static constexpr bool kVec = true, kExtra = false, kColsum = false;
  static constexpr int kScale = 0;
  struct In { float u, p, q; };
  typedef typename PackedIdx<IB>::type Packed;
  struct In4 { f32x4 u, q; Packed p; };
  __device__ static __forceinline__ In load(const GemmProb& P, size_t i, int) {
    const int id = IB == 2 ? (int)((const uint16_t PD_GLOBAL*)P.p8)[i] : (int)((gcu8)P.p8)[i];
    return In{((gcf)P.e0)[i], quant_value(id, P.grid), ((gcf)P.e2)[i]};
  }
  __device__ static __forceinline__ void apply(const GemmProb& P, float* C, size_t i, int, float acc, const In& in,
                                               double& s0, double&) {
    const float g = P.alpha * acc + in.u + P.beta * (in.p - in.q);
    ((float PD_GLOBAL*)C)[i] = g;
    s0 += (double)g * (double)g;
  }
  __device__ static __forceinline__ In4 load4(const GemmProb& P, size_t i) {
    return In4{*reinterpret_cast<gcf4>((gcf)P.e0 + i), *reinterpret_cast<gcf4>((gcf)P.e2 + i),
               *reinterpret_cast<const Packed PD_GLOBAL*>((gcu8)P.p8 + i * IB)};
  }
  __device__ static __forceinline__ f32x4 apply4(const GemmProb& P, f32x4 acc, const In4& in, float, f32x4&) {
    return P.alpha * acc + in.u + P.beta * (dequant4(in.p, P.grid) - in.q);
  }
};

// Step-direction products with the residual update folded in (pdADMM-G). T = acc is stored and its norm
// taken as in EpiStoreNorm; in the same pass the carried residual r = W p + b - z (o1, in place) takes the
// update r -= s_prev * T with the 1/tau or 1/theta guessed ahead by the previous selection (LayerScal::spec_*:
// the value it chose, or that value times eta while the step size is still falling), which is almost always
// what the selection that follows picks (tau and theta move on a grid of powers of eta). The difference, if
// any, a small correction pass applies afterwards (fix_tau / fix_theta). EpiTrialW also leaves the
// column sums of the updated residual (the b-update needs its node-mean) per row tile in colpart.
template <int SCALE, bool COLSUM>
struct EpiTrialUpd {
  static constexpr int NS = 1, kBatch = 1;
  static constexpr bool kVec = true, kExtra = true, kColsum = COLSUM;
  static constexpr int kScale = SCALE;      // 1: 1/tau guessed ahead, 2: 1/theta guessed ahead
  typedef NoIn In;
  struct In4 { f32x4 r; };
  __device__ static __forceinline__ In load(const GemmProb&, size_t, int) { return In{}; }
  __device__ static __forceinline__ void apply(const GemmProb&, float*, size_t, int, float, const In&, double&, double&) {}
  __device__ static __forceinline__ In4 load4(const GemmProb& P, size_t i) {
    return In4{*reinterpret_cast<gcf4>((gcf)P.o1 + i)};
  }
  __device__ static __forceinline__ f32x4 apply4(const GemmProb&, f32x4 acc, const In4& in, float s_prev, f32x4& extra) {
    extra = in.r - s_prev * acc;
    return acc;
  }
};
typedef EpiTrialUpd<1, false> EpiTrialP;   // T = g W^T; r -= T / tau_prev
typedef EpiTrialUpd<2, true> EpiTrialW;    // T = p G^T; r -= T / theta_prev; column sums of r

struct EpiResid {     // r = acc + b[col] - z; s0 += r^2; s1 += (r - carried)^2 when e2 != null
  static constexpr int NS = 2, kBatch = 4;
  static constexpr bool kVec = false;
  static constexpr int kScale = 0;
  struct In { float b, z, carried; };
  __device__ static __forceinline__ In load(const GemmProb& P, size_t i, int col) {
    return In{((gcf)P.e0)[col], ((gcf)P.e1)[i], P.e2 ? ((gcf)P.e2)[i] : 0.0f};
  }
  __device__ static __forceinline__ void apply(const GemmProb& P, float* C, size_t i, int, float acc,
                                               const In& in, double& s0, double& s1) {
    const float r = acc + in.b - in.z;
    ((float PD_GLOBAL*)C)[i] = r;
    s0 += (double)r * (double)r;
    if (P.e2) {
      const double d = (double)r - (double)in.carried;
      s1 += d * d;
    }
  }
};
struct EpiForward {   // z = acc + b[col]; q = f(z); p_next = f(z) (projected onto the grid in -Q; q too if beta != 0)
  static constexpr int NS = 0, kBatch = 1;
  static constexpr bool kVec = false;
  static constexpr int kScale = 0;
  struct In { float b; };
  __device__ static __forceinline__ In load(const GemmProb& P, size_t, int col) { return In{((gcf)P.e0)[col]}; }
  __device__ static __forceinline__ void apply(const GemmProb& P, float* C, size_t i, int, float acc,
                                               const In& in, double&, double&) {
    const float z = acc + in.b;
    ((float PD_GLOBAL*)C)[i] = z;
    if (P.o1) {
      const float a = act_fn(z, P.slope);
      const int id = P.grid.levels > 0 ? quant_index(a, P.grid) : 0;
      const float aq = P.grid.levels > 0 ? quant_value(id, P.grid) : a;
      ((float PD_GLOBAL*)P.o1)[i] = P.beta != 0.0f ? aq : a;    // beta != 0: q is kept on the grid as well
      if (P.o8) {                                               // -Q: p_{l+1} is kept as indices
        if (P.grid.ib == 2) ((uint16_t PD_GLOBAL*)P.o8)[i] = (uint16_t)id;
        else ((uint8_t PD_GLOBAL*)P.o8)[i] = (uint8_t)id;
      } else ((float PD_GLOBAL*)P.o2)[i] = aq;
    }
  }
};
struct EpiBiasAct {   // C = acc + b[col], passed through f when beta != 0 (forward pass of the model, Problem 1)
  static constexpr int NS = 0, kBatch = 1;
  static constexpr bool kVec = false;
  static constexpr int kScale = 0;
  struct In { float b; };
  __device__ static __forceinline__ In load(const GemmProb& P, size_t, int col) { return In{((gcf)P.e0)[col]}; }
  __device__ static __forceinline__ void apply(const GemmProb& P, float* C, size_t i, int, float acc,
                                               const In& in, double&, double&) {
    const float v = acc + in.b;
    ((float PD_GLOBAL*)C)[i] = P.beta != 0.0f ? act_fn(v, P.slope) : v;
  }
};

// Tile configuration: block tile BM x BN x BK, 4 waves arranged WM x WN, each wave owns
// (BM/WM) x (BN/WN) as a grid of 32x32 MFMA blocks.
// MINB: blocks per compute unit the kernel is compiled for (bounds the registers per lane).
template <int BM_, int BN_, int BK_, int WM_, int WN_, int MINB_ = 3>
struct TileCfg {
  static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_, MINB = MINB_;
  static constexpr int TM = BM / WM / 32, TN = BN / WN / 32;   // MFMA blocks per wave
  static constexpr int LDA = BM + 4, LDB = BN + 4;              // LDS row strides (floats)
  static_assert(WM * WN == 4, "256 threads = 4 waves");
  static_assert(BM % (32 * WM) == 0 && BN % (32 * WN) == 0 && BK % 4 == 0, "tile shape");
};


// Loads one operand tile (ROWS "m-like" indices x BK k indices) into registers.
//  KCONTIG: element (m, k) at base[m*ld + k]; thread owns float4 groups along k.
//  else   : element (m, k) at base[k*ld + m]; thread owns float4 groups along m.
// FAST: branch-free 16-byte loads from addresses clamped into the matrix. Whatever a clamped m
// index fetches only reaches output rows/columns that are never stored; k indices beyond the
// range are zeroed when the tile is written to LDS (store_operand). Needs ld % 4 == 0, a
// 16-byte aligned base and, for the m-contiguous layout, a width that is a multiple of 4.
// Otherwise: guarded scalar loads with zero fill.
template <bool KCONTIG, bool FAST, int ROWS, int BK, int NV>
__device__ __forceinline__ void load_operand(f32x4 (&reg)[NV], gcf base, int ld, int m0, int mlim, int kb, int kend,
                                             int tid) {
  if (KCONTIG) {
    constexpr int KQ = BK / 4;            // float4 groups per row
    constexpr int RSTEP = 256 / KQ;
    const int r = tid / KQ, k = kb + (tid % KQ) * 4;
#pragma unroll
    for (int h = 0; h < NV; ++h) {
      const int m = m0 + r + RSTEP * h;
      if (FAST) {
        const int mc = min(m, mlim - 1);
        const int kc = min(k, (kend - 1) & ~3);
        reg[h] = *reinterpret_cast<gcf4>(base + (size_t)mc * ld + kc);
      } else {
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        if (m < mlim) {
          gcf src = base + (size_t)m * ld + k;
          if (k + 0 < kend) v.x = src[0];
          if (k + 1 < kend) v.y = src[1];
          if (k + 2 < kend) v.z = src[2];
          if (k + 3 < kend) v.w = src[3];
        }
        reg[h] = v;
      }
    }
  } else {
    constexpr int MQ = ROWS / 4;          // float4 groups per k-row
    constexpr int KSTEP = 256 / MQ;
    const int kr = tid / MQ, m = m0 + (tid % MQ) * 4;
#pragma unroll
    for (int h = 0; h < NV; ++h) {
      const int k = kb + kr + KSTEP * h;
      if (FAST) {
        const int mc = min(m, mlim - 4);
        const int kc = min(k, kend - 1);
        reg[h] = *reinterpret_cast<gcf4>(base + (size_t)kc * ld + mc);
      } else {
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        if (k < kend) {
          gcf src = base + (size_t)k * ld + m;
          if (m + 0 < mlim) v.x = src[0];
          if (m + 1 < mlim) v.y = src[1];
          if (m + 2 < mlim) v.z = src[2];
          if (m + 3 < mlim) v.w = src[3];
        }
        reg[h] = v;
      }
    }
  }
}

// LDS position of element (k, c) of a staged operand tile: rows of LD floats, and rows with k & 8 set
// start 8 floats later. k-contiguous operands arrive through a transposing 4-byte store in which the
// four lanes of a quad hold k = 0, 4, 8, 12 of one tile row; with LD = 4 (mod 32) rows k and k + 8
// would meet in the same banks, the shift moves them 8 banks apart. Fragment reads (32 consecutive c of
// one k) and 16-byte row stores are unaffected. A tile buffer holds BK * LD + 8 floats.
template <int LD>
__device__ __forceinline__ constexpr int lds_pos(int k, int c) { return k * LD + (k & 8) + c; }

// Writes a register tile to LDS as [k][m]. With FAST the entries whose k lies beyond kend are zeroed here.
template <bool KCONTIG, bool FAST, int ROWS, int BK, int LD, int NV>
__device__ __forceinline__ void store_operand(float* lds, const f32x4 (&reg)[NV], int kb, int kend, int tid) {
  if (KCONTIG) {
    constexpr int KQ = BK / 4;
    constexpr int RSTEP = 256 / KQ;
    const int r = tid / KQ, kq = (tid % KQ) * 4;
    const int rem = kend - (kb + kq);     // components c < rem are inside the k range
    float* dst = lds + lds_pos<LD>(kq, r);  // kq + 0..3 share the bit kq & 8
#pragma unroll
    for (int h = 0; h < NV; ++h) {
      const int c = RSTEP * h;
      dst[0 * LD + c] = (!FAST || rem > 0) ? reg[h].x : 0.f;
      dst[1 * LD + c] = (!FAST || rem > 1) ? reg[h].y : 0.f;
      dst[2 * LD + c] = (!FAST || rem > 2) ? reg[h].z : 0.f;
      dst[3 * LD + c] = (!FAST || rem > 3) ? reg[h].w : 0.f;
    }
  } else {
    constexpr int MQ = ROWS / 4;
    constexpr int KSTEP = 256 / MQ;
    const int kr = tid / MQ, mq = (tid % MQ) * 4;
#pragma unroll
    for (int h = 0; h < NV; ++h) {
      f32x4 v = reg[h];
      if (FAST && kb + kr + KSTEP * h >= kend) v = f32x4{0.f, 0.f, 0.f, 0.f};
      *reinterpret_cast<f32x4*>(lds + lds_pos<LD>(kr + KSTEP * h, mq)) = v;
    }
  }
}

// The same two steps for an operand that is stored as indices into Delta of IB bytes each (p_l in -Q mode; rows
// of ld indices, ld a multiple of 4, base 8-byte aligned: the library's own arrays). A thread fetches the four
// indices of one group as one 32- or 64-bit word from an address clamped into the array (whatever a clamped
// index fetches only reaches output rows/columns that are never stored) and turns them into values when the
// tile is written to LDS, where entries whose k lies beyond kend become zero.
template <bool KCONTIG, int ROWS, int BK, int NV, int IB>
__device__ __forceinline__ void load_operand_u8(typename PackedIdx<IB>::type (&reg)[NV], gcu8 base, int ld, int m0,
                                                int mlim, int kb, int kend, int tid) {
  typedef typename PackedIdx<IB>::type Packed;
  if (KCONTIG) {
    constexpr int KQ = BK / 4;
    constexpr int RSTEP = 256 / KQ;
    const int r = tid / KQ, k = kb + (tid % KQ) * 4;
    const int kc = min(k, (kend - 1) & ~3);
#pragma unroll
    for (int h = 0; h < NV; ++h) {
      const int mc = min(m0 + r + RSTEP * h, mlim - 1);
      reg[h] = *reinterpret_cast<const Packed PD_GLOBAL*>(base + ((size_t)mc * ld + kc) * IB);
    }
  } else {
    constexpr int MQ = ROWS / 4;
    constexpr int KSTEP = 256 / MQ;
    const int kr = tid / MQ;
    const int mc = min(m0 + (tid % MQ) * 4, ((mlim + 3) & ~3) - 4);
#pragma unroll
    for (int h = 0; h < NV; ++h) {
      const int kc = min(kb + kr + KSTEP * h, kend - 1);
      reg[h] = *reinterpret_cast<const Packed PD_GLOBAL*>(base + ((size_t)kc * ld + mc) * IB);
    }
  }
}

template <bool KCONTIG, int ROWS, int BK, int LD, int NV, class Packed>
__device__ __forceinline__ void store_operand_u8(float* lds, const Packed (&reg)[NV], int kb, int kend, int tid,
                                                 const QuantGrid grid) {
  if (KCONTIG) {
    constexpr int KQ = BK / 4;
    constexpr int RSTEP = 256 / KQ;
    const int r = tid / KQ, kq = (tid % KQ) * 4;
    const int rem = kend - (kb + kq);
    float* dst = lds + lds_pos<LD>(kq, r);
#pragma unroll
    for (int h = 0; h < NV; ++h) {
      const int c = RSTEP * h;
      const f32x4 v = dequant4(reg[h], grid);
      dst[0 * LD + c] = rem > 0 ? v.x : 0.f;
      dst[1 * LD + c] = rem > 1 ? v.y : 0.f;
      dst[2 * LD + c] = rem > 2 ? v.z : 0.f;
      dst[3 * LD + c] = rem > 3 ? v.w : 0.f;
    }
  } else {
    constexpr int MQ = ROWS / 4;
    constexpr int KSTEP = 256 / MQ;
    const int kr = tid / MQ, mq = (tid % MQ) * 4;
#pragma unroll
    for (int h = 0; h < NV; ++h) {
      f32x4 v = dequant4(reg[h], grid);
      if (kb + kr + KSTEP * h >= kend) v = f32x4{0.f, 0.f, 0.f, 0.f};
      *reinterpret_cast<f32x4*>(lds + lds_pos<LD>(kr + KSTEP * h, mq)) = v;
    }
  }
}

constexpr int kVecBatch = 4;   // 16-byte column groups per lane whose inputs are fetched together

template <int IB> struct OperandReg { typedef typename PackedIdx<IB>::type type; };   // staging registers of an operand
template <> struct OperandReg<0> { typedef f32x4 type; };                              // (0: fp32 values)

template <bool B> struct BoolTag { static constexpr bool value = B; };

// VECC: the output and the epilogue's inputs are [*, ld] arrays with ld % 4 == 0 and 16-byte aligned
// bases (true for the library's own buffers), which allows the row-contiguous epilogue below.
// P8 = 1 or 2: the operand that carries p_l (A in the k-contiguous layout, B in the other) is P.p8, indices into
// P.grid of that many bytes each, instead of fp32 values.
template <class Cfg, bool KCONTIG, class Epi, bool VECC, int P8 = 0>
__device__ __forceinline__ void gemm_body(const GemmProb& P, const int local, const float escale) {
  constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, TM = Cfg::TM, TN = Cfg::TN;
  constexpr int LDA = Cfg::LDA, LDB = Cfg::LDB;
  constexpr int NVA = BM * BK / 4 / 256, NVB = BN * BK / 4 / 256;
  static_assert(NVA >= 1 && NVB >= 1, "tile too small for 256 loader threads");
  constexpr int BUFA = BK * LDA + 8, BUFB = BK * LDB + 8;   // one staged tile of each operand (see lds_pos)
  static_assert(BK <= 16, "lds_pos shifts the rows with k & 8 set: at most one shifted run per tile");
  __shared__ __attribute__((aligned(16))) float smem[2 * BUFA + 2 * BUFB];
  __shared__ double red[4];
  float* const As = smem;
  float* const Bs = smem + 2 * BUFA;

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
  const int wm = wave / Cfg::WN, wn = wave % Cfg::WN;
  const int li = lane & 31, lh = lane >> 5;
  const gcf A = (gcf)P.A;
  const gcf B = (gcf)P.B;
  // the branch-free loader needs 16-byte loads to be legal and, for the m-contiguous layout,
  // whole float4 groups inside the matrix
  constexpr int A8 = KCONTIG ? P8 : 0, B8 = KCONTIG ? 0 : P8;
  const bool fast = (A8 || P.vecA) && (B8 || P.vecB) &&
                    (KCONTIG || (P.M % 4 == 0 && P.M >= 4 && (B8 || (P.N % 4 == 0 && P.N >= 4))));

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  // MFMAs of one staged tile. The fragments of k-step kk+2 are fetched from LDS before the MFMAs of
  // k-step kk issue; the scheduling barriers keep that order (left alone, the compiler folds both
  // fragment sets into one register set and waits for every LDS read right before its MFMAs).
  auto compute_tile = [&](int cur, auto&& mid) {
    float a[2][TM], b[2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) a[0][i] = As[cur * BUFA + lds_pos<LDA>(0, 0) + lh * LDA + wm * (BM / Cfg::WM) + i * 32 + li];
#pragma unroll
    for (int j = 0; j < TN; ++j) b[0][j] = Bs[cur * BUFB + lds_pos<LDB>(0, 0) + lh * LDB + wn * (BN / Cfg::WN) + j * 32 + li];
#pragma unroll
    for (int kk = 0; kk < BK; kk += 2) {
      const int c = (kk >> 1) & 1, n = c ^ 1;
      if (kk + 2 < BK) {
#pragma unroll
        for (int i = 0; i < TM; ++i) a[n][i] = As[cur * BUFA + lds_pos<LDA>(kk + 2, 0) + lh * LDA + wm * (BM / Cfg::WM) + i * 32 + li];
#pragma unroll
        for (int j = 0; j < TN; ++j) b[n][j] = Bs[cur * BUFB + lds_pos<LDB>(kk + 2, 0) + lh * LDB + wn * (BN / Cfg::WN) + j * 32 + li];
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[c][i], b[c][j], acc[i][j], 0, 0, 0);
      if (kk == (BK / 2 & ~1)) mid();   // LDS store of the next tile rides in the shadow of the MFMAs
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  auto nothing = [] {};

  // Main loop with two register sets: the global loads of tile t+2 are issued before the MFMAs of
  // tile t, the LDS store of tile t+1 (loaded one tile earlier) follows them, one barrier per tile.
  // Loads and stores past the last tile are issued all the same (addresses are clamped into the
  // matrix, out-of-range k is stored as zero, the buffer written is never read): with no branch
  // around them the compiler knows exactly how many loads are in flight when a register set is
  // consumed and waits for that set only, not for the loads it has just issued.
  auto main_loop = [&](auto fast_tag) {
    constexpr bool FAST = decltype(fast_tag)::value;
    typedef typename OperandReg<A8>::type RegA;
    typedef typename OperandReg<B8>::type RegB;
    RegA ra0[NVA], ra1[NVA];
    RegB rb0[NVB], rb1[NVB];
    auto load_tile = [&](int kt, RegA (&ra)[NVA], RegB (&rb)[NVB]) {
      const int kb = kbeg + kt * BK;
      if constexpr (A8 != 0) load_operand_u8<KCONTIG, BM, BK, NVA, A8>(ra, (gcu8)P.p8, P.lda, m0, P.M, kb, kend, tid);
      else load_operand<KCONTIG, FAST, BM, BK, NVA>(ra, A, P.lda, m0, P.M, kb, kend, tid);
      if constexpr (B8 != 0) load_operand_u8<KCONTIG, BN, BK, NVB, B8>(rb, (gcu8)P.p8, P.ldb, n0, P.N, kb, kend, tid);
      else load_operand<KCONTIG, FAST, BN, BK, NVB>(rb, B, P.ldb, n0, P.N, kb, kend, tid);
    };
    auto store_tile = [&](int kt, int buf, const RegA (&ra)[NVA], const RegB (&rb)[NVB]) {
      const int kb = kbeg + kt * BK;
      if constexpr (A8 != 0) store_operand_u8<KCONTIG, BM, BK, LDA, NVA>(As + buf * BUFA, ra, kb, kend, tid, P.grid);
      else store_operand<KCONTIG, FAST, BM, BK, LDA, NVA>(As + buf * BUFA, ra, kb, kend, tid);
      if constexpr (B8 != 0) store_operand_u8<KCONTIG, BN, BK, LDB, NVB>(Bs + buf * BUFB, rb, kb, kend, tid, P.grid);
      else store_operand<KCONTIG, FAST, BN, BK, LDB, NVB>(Bs + buf * BUFB, rb, kb, kend, tid);
    };
    load_tile(0, ra0, rb0);
    load_tile(1, ra1, rb1);
    store_tile(0, 0, ra0, rb0);
    __syncthreads();
    int kt = 0;
    for (; kt + 1 < nkt; kt += 2) {
      // even tile: LDS buffer 0 is current, set 1 holds tile kt+1, set 0 is free
      load_tile(kt + 2, ra0, rb0);
      compute_tile(0, [&] { store_tile(kt + 1, 1, ra1, rb1); });
      __syncthreads();
      // odd tile: LDS buffer 1 is current, set 0 holds tile kt+2, set 1 is free
      load_tile(kt + 3, ra1, rb1);
      compute_tile(1, [&] { store_tile(kt + 2, 0, ra0, rb0); });
      __syncthreads();
    }
    if (kt < nkt) compute_tile(0, nothing);   // odd tile count: the last tile sits in buffer 0
  };
  if (nkt > 0) {
    if (fast) main_loop(BoolTag<true>{});
    else main_loop(BoolTag<false>{});
  }

  // Epilogue. MFMA 32x32 output layout: register v of lane l holds
  // row 8*(v/4) + 4*(l/32) + v%4, column l%32 of the 32x32 block.
  float* Cout = P.C + (size_t)split * (size_t)P.M * (size_t)P.ldc;
  double s0 = 0.0, s1 = 0.0;
  if constexpr (Epi::kVec && VECC) {
    // Row-contiguous epilogue: every wave passes its 64x64 sub-tile through LDS (32 rows at a time, the
    // operand buffers are free now) and then owns whole 16-byte column groups, so all global accesses
    // of the epilogue are coalesced 16-byte loads and stores, a quarter as many as element by element.
    // (a wave whose sub-tile is wider than 64 columns takes it 64 columns at a time)
    static_assert(TN % 2 == 0 && 4 * 32 * 64 <= 2 * BUFA + 2 * BUFB, "staging area");
    constexpr int CW = BN / Cfg::WN;                   // columns of one wave
    __shared__ double colred[Epi::kColsum ? 4 : 1][Epi::kColsum ? CW : 1];
    __syncthreads();                                   // all waves are done with the operand buffers
    float* stage = smem + wave * (32 * 64);
    const int rr = lane >> 4, c4 = (lane & 15) * 4;    // row (mod 4) and first column of this lane's groups
#pragma unroll
    for (int jj = 0; jj < TN; jj += 2) {
    const int col = n0 + wn * CW + jj * 32 + c4;
    const int nvalid = P.N - col;                      // columns of the group inside the matrix (>= 4: all)
    double cs0 = 0.0, cs1 = 0.0, cs2 = 0.0, cs3 = 0.0; // column sums of the second output (kColsum)
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) stage[(8 * (v >> 2) + 4 * lh + (v & 3)) * 64 + j * 32 + li] = acc[i][jj + j][v];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      // three input streams plus a second output leave registers for two groups only
      constexpr int VB = (Epi::kExtra && sizeof(typename Epi::In4) > 16) ? 2 : kVecBatch;
#pragma unroll
      for (int it = 0; it < 8; it += VB) {
        typename Epi::In4 in[VB];
        f32x4 val[VB];
        size_t idx[VB];
        bool on[VB];
#pragma unroll
        for (int b = 0; b < VB; ++b) {
          const int rl = (it + b) * 4 + rr;
          const int row = m0 + wm * (BM / Cfg::WM) + i * 32 + rl;
          on[b] = row < P.M && nvalid > 0;
          idx[b] = (size_t)row * P.ldc + col;
          val[b] = *reinterpret_cast<const f32x4*>(&stage[rl * 64 + c4]);
          if (on[b]) in[b] = Epi::load4(P, idx[b]);
        }
#pragma unroll
        for (int b = 0; b < VB; ++b) {
          if (on[b]) {
            f32x4 extra = {0.f, 0.f, 0.f, 0.f};
            f32x4 r = Epi::apply4(P, val[b], in[b], escale, extra);
            if (nvalid < 4) {                          // keep the pad columns of the row at zero
              if (nvalid < 2) { r.y = 0.f; extra.y = 0.f; }
              if (nvalid < 3) { r.z = 0.f; extra.z = 0.f; }
              r.w = 0.f;
              extra.w = 0.f;
            }
            *reinterpret_cast<f32x4 PD_GLOBAL*>((float PD_GLOBAL*)Cout + idx[b]) = r;
            if constexpr (Epi::kExtra) *reinterpret_cast<f32x4 PD_GLOBAL*>((float PD_GLOBAL*)P.o1 + idx[b]) = extra;
            if constexpr (Epi::kColsum) {
              cs0 += (double)extra.x; cs1 += (double)extra.y; cs2 += (double)extra.z; cs3 += (double)extra.w;
            }
            if (Epi::NS >= 1)
              s0 += (double)r.x * (double)r.x + (double)r.y * (double)r.y + (double)r.z * (double)r.z +
                    (double)r.w * (double)r.w;
          }
        }
      }
      __builtin_amdgcn_wave_barrier();
    }
    if constexpr (Epi::kColsum) {
      // lanes l, l+16, l+32, l+48 own the same columns (rows differ): add them up
      cs0 += __shfl_xor(cs0, 16, kWave); cs1 += __shfl_xor(cs1, 16, kWave);
      cs2 += __shfl_xor(cs2, 16, kWave); cs3 += __shfl_xor(cs3, 16, kWave);
      cs0 += __shfl_xor(cs0, 32, kWave); cs1 += __shfl_xor(cs1, 32, kWave);
      cs2 += __shfl_xor(cs2, 32, kWave); cs3 += __shfl_xor(cs3, 32, kWave);
      if (lane < 16) {
        colred[wave][jj * 32 + c4 + 0] = cs0; colred[wave][jj * 32 + c4 + 1] = cs1;
        colred[wave][jj * 32 + c4 + 2] = cs2; colred[wave][jj * 32 + c4 + 3] = cs3;
      }
    }
    }
    if constexpr (Epi::kColsum) {
      // then the waves that share the columns (wm = 0, 1) through LDS; fixed order, one value per column and
      // row tile
      static_assert(Cfg::WM == 2 && BN <= 256, "two waves per column, one thread per column");
      __syncthreads();
      if (tid < BN) {
        const int w = tid / CW, c = tid % CW;          // wn, column inside the wave's share
        const int gcol = n0 + tid;
        if (gcol < P.ldc) P.colpart[(size_t)tm * P.ldc + gcol] = colred[w][c] + colred[Cfg::WN + w][c];
      }
    }
  } else {
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = n0 + wn * (BN / Cfg::WN) + j * 32 + li;
      if (col < P.N) {
        // the 16 elements of one MFMA block in batches: all extra inputs of a batch first, then results and stores
#pragma unroll
        for (int v0 = 0; v0 < 16; v0 += Epi::kBatch) {
          typename Epi::In in[Epi::kBatch];
#pragma unroll
          for (int v = 0; v < Epi::kBatch; ++v) {
            const int row = m0 + wm * (BM / Cfg::WM) + i * 32 + 8 * ((v0 + v) >> 2) + 4 * lh + ((v0 + v) & 3);
            if (row < P.M) in[v] = Epi::load(P, (size_t)row * P.ldc + col, col);
          }
#pragma unroll
          for (int v = 0; v < Epi::kBatch; ++v) {
            const int row = m0 + wm * (BM / Cfg::WM) + i * 32 + 8 * ((v0 + v) >> 2) + 4 * lh + ((v0 + v) & 3);
            if (row < P.M) Epi::apply(P, Cout, (size_t)row * P.ldc + col, col, acc[i][j][v0 + v], in[v], s0, s1);
          }
        }
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
// The second launch bound asks for Cfg::MINB waves per SIMD (for the 128x128 tile 3 blocks per compute unit, 768 on
// the chip, which the launch plans count on): the compiler then keeps accumulators and staging registers within
// 168 in all.
template <class Cfg, bool KCONTIG, class Epi, bool VECC = false, int P8 = 0>
__global__ __launch_bounds__(256, Cfg::MINB) void gemm_kernel(const GemmProb* __restrict__ probs, const BlockMap map,
                                                   const LayerScal* __restrict__ scal, int predicated,
                                                   int panel) {
  const int lb = xcd_remap(blockIdx.x, panel);
  if (lb >= map.total) return;
  int local;
  const int pi = find_group(map, lb, &local);
  GemmProb P = probs[pi];
  if (predicated && !scal[P.layer].active) return;
  float escale = 0.0f;
  if (Epi::kScale == 1) escale = scal[P.layer].spec_tau;
  if (Epi::kScale == 2) escale = scal[P.layer].spec_theta;
  if (P.p8) P.p8 += (size_t)scal[P.layer].cur * P.p8_plane;     // the plane that holds p_l right now
  gemm_body<Cfg, KCONTIG, Epi, VECC, P8>(P, local, escale);
}

// Single problem with the descriptor passed by value (no table in device memory needed).
// (P.p8, if used, must already point at the plane that holds p_l.)
template <class Cfg, bool KCONTIG, class Epi, int P8 = 0>
__global__ __launch_bounds__(256) void gemm_one_kernel(const GemmProb P, int panel) {
  const int lb = xcd_remap(blockIdx.x, panel);
  if (lb >= P.nblk) return;
  gemm_body<Cfg, KCONTIG, Epi, false, P8>(P, lb, 0.0f);
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
  int vec;             // ld % 4 == 0 and part, G 16-byte aligned
};

// The partial sums of one element are added in the order of the chunks (fixed by the split, not by the
// launch); the loads of up to 8 chunks are issued together before their ordered additions.
__device__ __forceinline__ void splitk_reduce_body(const ReduceProb& P, const int local) {
  __shared__ double red[4];
  const size_t plane = (size_t)P.M * P.ld;
  double s = 0.0;
  if (P.vec) {   // ld % 4 == 0, 16-byte aligned bases: one float4 group per thread and step
    const size_t groups = plane / 4;
    for (size_t i = (size_t)local * 256 + threadIdx.x; i < groups; i += (size_t)P.nblk * 256) {
      const int col = (int)((i * 4) % P.ld);
      const float* src = P.part + i * 4;
      f32x4 sum = {0.f, 0.f, 0.f, 0.f};
      int k = 0;
      for (; k + 8 <= P.splitk; k += 8) {
        f32x4 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = stream_load(reinterpret_cast<const f32x4*>(src + (size_t)(k + j) * plane));
#pragma unroll
        for (int j = 0; j < 8; ++j) sum += v[j];
      }
      for (; k < P.splitk; ++k) sum += stream_load(reinterpret_cast<const f32x4*>(src + (size_t)k * plane));
      sum.x = col + 0 < P.N ? sum.x * P.alpha : 0.f;
      sum.y = col + 1 < P.N ? sum.y * P.alpha : 0.f;
      sum.z = col + 2 < P.N ? sum.z * P.alpha : 0.f;
      sum.w = col + 3 < P.N ? sum.w * P.alpha : 0.f;
      *reinterpret_cast<f32x4*>(P.G + i * 4) = sum;
      s += (double)sum.x * (double)sum.x + (double)sum.y * (double)sum.y + (double)sum.z * (double)sum.z +
           (double)sum.w * (double)sum.w;
    }
  } else {
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
  }
  const double t = block_sum_256(s, red);
  if (threadIdx.x == 0 && P.norm_part) P.norm_part[local] = t;
}

__global__ __launch_bounds__(256) void splitk_reduce_kernel(const ReduceProb* __restrict__ probs, const BlockMap map) {
  int local;
  const int pi = find_group(map, blockIdx.x, &local);
  const ReduceProb P = probs[pi];
  splitk_reduce_body(P, local);
}
__global__ __launch_bounds__(256) void splitk_reduce_one_kernel(const ReduceProb P) {
  splitk_reduce_body(P, blockIdx.x);
}

}  // namespace pdadmm
