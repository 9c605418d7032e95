// Shared device/host definitions for the pdADMM kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pdadmm {

#define PD_GLOBAL __attribute__((address_space(1)))

// Pointers that are known to address global memory (pointers read from descriptor tables are
// generic to the compiler, which would otherwise emit flat loads that also tie up the LDS counter).
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef const float PD_GLOBAL* gcf;
typedef const f32x4 PD_GLOBAL* gcf4;

// Loads/stores of data that is touched once per pass (arrays far larger than the caches): the
// nontemporal hint keeps them from displacing the operands the next product kernel re-reads.
#ifndef PDADMM_STREAM_HINT
#define PDADMM_STREAM_HINT 1
#endif
__device__ __forceinline__ f32x4 stream_load(const f32x4* p) {
#if PDADMM_STREAM_HINT
  return __builtin_nontemporal_load(p);
#else
  return *p;
#endif
}
__device__ __forceinline__ void stream_store(f32x4* p, f32x4 v) {
#if PDADMM_STREAM_HINT
  __builtin_nontemporal_store(v, p);
#else
  *p = v;
#endif
}

constexpr int kWave = 64;
constexpr int kXcd = 8;   // MI355X: 8 accelerator dies, workgroups are dealt to them round-robin

// Map the hardware block id to a logical block id. Workgroups are dealt to the 8 dies round-robin
// in block-id order, so block b runs on die b % 8 as the (b / 8)-th block of that die. Logical
// blocks are cut into panels of `panel` consecutive ids (tiles that share an operand row panel);
// a die takes whole panels, the dies take panels round-robin: neighbours in the logical order
// share a die's L2, and problems of different cost per tile are spread evenly over the dies.
// The launch is padded to a multiple of 8*panel blocks; ids >= total must exit.
__device__ __forceinline__ int xcd_remap(int bid, int panel) {
  const int x = bid % kXcd, j = bid / kXcd;
  return ((j / panel) * kXcd + x) * panel + (j % panel);
}
__host__ __device__ inline int xcd_padded(int total, int panel) {
  const int g = kXcd * panel;
  return (total + g - 1) / g * g;
}

// Block -> group lookup for the layer-grouped launches. The table of first block ids travels in the
// kernel arguments (no dependent chain of global loads at block start): lane i compares against
// entry i, a ballot gives the group index. Entries are ascending, blk0[0] = 0, n <= kMaxGroup.
constexpr int kMaxGroup = 64;
struct BlockMap {
  int n, total;
  int blk0[kMaxGroup];
};
__device__ __forceinline__ int find_group(const BlockMap& m, int lb, int* local) {
  const int lane = threadIdx.x & 63;
  const int first = lane < m.n ? m.blk0[lane] : 0x7fffffff;
  const unsigned long long hit = __ballot(lb >= first);
  const int idx = __builtin_amdgcn_readfirstlane(__popcll(hit) - 1);
  *local = lb - m.blk0[idx];
  return idx;
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

// Sum of one double per thread over a 256-thread block in a fixed order; result valid in thread 0.
__device__ __forceinline__ double block_sum_256(double v, double* smem /* >= 4 doubles */) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) smem[w] = v;
  __syncthreads();
  return smem[0] + smem[1] + smem[2] + smem[3];
}

// Device-side sticky error bits.
enum : int { kErrBacktrack = 1, kErrNonFinite = 2 };

// Per-layer scalars that live in device memory and are produced/consumed by kernels only.
struct LayerScal {
  double tau, theta;       // current backtracking parameters
  double norm_g, norm_t;   // last reduced squared norms (diagnostics)
  float inv_tau, inv_theta;  // 1/tau, 1/theta as applied by the step kernels (0 = skip the step)
  float spec_tau, spec_theta;  // 1/tau, 1/theta that the product epilogues of the NEXT update apply ahead of the
                               // selection: the value just chosen, or that value times eta if it was accepted at
                               // the first trial (a step size that is still falling usually falls again)
  float fix_tau, fix_theta;  // chosen minus applied-ahead 1/tau, 1/theta: what the correction pass still has to
                             // apply (0 when the guess was right)
  float trial_t;           // -Q: tau of the trial in flight
  int p_trials, w_trials;
  int active;              // -Q: 1 while the p-update of this layer is still searching
  int probing;             // -Q: 1 if this update started at tau/eta (a probe of the smaller value)
  int probe_wait;          // -Q: iterations to wait after a rejected probe (1, 2, 4, ... kProbeCap)
  int probe_skip;          // -Q: iterations left until the next probe
  int cur;                 // -Q: which of the layer's two index planes holds p_l (the other takes the trial candidates)
  long long products;      // -Q: trial products W d judged for this layer since init (one per backtracking trial)
};
constexpr int kProbeCap = 16;

// Activation f (Section 4: ReLU and leaky ReLU satisfy the assumption): f(z) = z for z > 0, slope*z
// otherwise; slope = 0 is ReLU.
__device__ __forceinline__ float act_fn(float z, float slope) { return z > 0.0f ? z : slope * z; }

struct QuantGrid {
  float lo, step;
  int levels;
  int ib;   // bytes per stored index: 1 for up to 256 levels, 2 for up to 65536
};

// Single fp32 operations that the compiler may not fuse with their neighbours into a fused
// multiply-add (the separate roundings are part of the specified result).
__device__ __forceinline__ float mul_rn(float a, float b) {
#pragma clang fp contract(off)
  return a * b;
}
__device__ __forceinline__ float add_rn(float a, float b) {
#pragma clang fp contract(off)
  return a + b;
}
__device__ __forceinline__ float sub_rn(float a, float b) {
#pragma clang fp contract(off)
  return a - b;
}
__device__ __forceinline__ float div_rn(float a, float b) {
#pragma clang fp contract(off)
  return a / b;
}

// Projection onto the uniform grid, every operation rounded to fp32 separately.
__device__ __forceinline__ int quant_index(float v, const QuantGrid g) {
  const float t = div_rn(sub_rn(v, g.lo), g.step);
  float r = rintf(t);
  if (!(r == r)) r = 0.0f;                      // NaN -> 0
  r = fminf(fmaxf(r, 0.0f), (float)(g.levels - 1));
  return (int)r;
}
__device__ __forceinline__ float quant_value(int idx, const QuantGrid g) {
  return add_rn(g.lo, mul_rn((float)idx, g.step));
}
// Four members of Delta from four packed 8-bit indices (byte j = index of element j). In -Q the library keeps
// p_l (l >= 2) only as such indices and forms the values where they are consumed; the value is the same
// fp32 number that quant_value gives, bit for bit.
__device__ __forceinline__ f32x4 dequant4(uint32_t packed, const QuantGrid g) {
  f32x4 v;
  v.x = quant_value((int)(packed & 0xffu), g);
  v.y = quant_value((int)((packed >> 8) & 0xffu), g);
  v.z = quant_value((int)((packed >> 16) & 0xffu), g);
  v.w = quant_value((int)(packed >> 24), g);
  return v;
}
// The same for 16-bit indices (grids of more than 256 levels): element j in bits 16 (j % 2) .. of word j / 2.
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ f32x4 dequant4(u32x2 packed, const QuantGrid g) {
  f32x4 v;
  v.x = quant_value((int)(packed.x & 0xffffu), g);
  v.y = quant_value((int)(packed.x >> 16), g);
  v.z = quant_value((int)(packed.y & 0xffffu), g);
  v.w = quant_value((int)(packed.y >> 16), g);
  return v;
}
typedef const uint8_t PD_GLOBAL* gcu8;
// Four consecutive indices as they lie in memory, by index width in bytes.
template <int IB> struct PackedIdx { typedef uint32_t type; };
template <> struct PackedIdx<2> { typedef u32x2 type; };

// Group i4 (elements 4 i4 .. 4 i4 + 3) of an index plane, as values / from indices; the width comes with the grid.
// The plane is 8-byte aligned (the library's planes start on 256-byte boundaries).
// (IB = 0: width read from the grid at run time; the streaming kernels of the iteration are compiled per width)
template <int IB = 0>
__device__ __forceinline__ f32x4 load_members4(const uint8_t* plane, size_t i4, const QuantGrid g) {
  if (IB == 2 || (IB == 0 && g.ib == 2))
    return dequant4(__builtin_nontemporal_load(reinterpret_cast<const u32x2*>(plane) + i4), g);
  return dequant4(__builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(plane) + i4), g);
}
__device__ __forceinline__ void store_indices4(uint8_t* plane, size_t i4, int ib, int i0, int i1, int i2, int i3) {
  if (ib == 2) {
    u32x2 w;
    w.x = (uint32_t)i0 | ((uint32_t)i1 << 16);
    w.y = (uint32_t)i2 | ((uint32_t)i3 << 16);
    reinterpret_cast<u32x2*>(plane)[i4] = w;
  } else {
    reinterpret_cast<uint32_t*>(plane)[i4] =
        (uint32_t)i0 | ((uint32_t)i1 << 8) | ((uint32_t)i2 << 16) | ((uint32_t)i3 << 24);
  }
}

}  // namespace pdadmm
