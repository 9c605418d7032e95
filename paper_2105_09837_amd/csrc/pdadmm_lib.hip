// C ABI of the pdADMM-G / pdADMM-G-Q iteration for MI355X (see include/pdadmm.h).
// Host side: workspace layout, descriptor tables for the layer-grouped launches, phase sequencing.
#include "../../include/pdadmm.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "common.h"
#include "elementwise.h"
#include "gemm.h"
#include "spmm.h"

using namespace pdadmm;

// Tile shape of the dense products (see gemm.h).
using Tile = TileCfg<128, 128, 16, 2, 2>;
constexpr int BM = Tile::BM, BN = Tile::BN, BK = Tile::BK;
// Product blocks resident on the chip at once: 256 compute units x 3 blocks (one wave per SIMD each,
// 164 registers per lane).
constexpr int kGemmSlots = 256 * Tile::MINB;
// Wide tile for the W-gradient products (contraction over the nodes) of a context whose p_l are fp32: a
// block's two operand panels are 128 and 256 columns of node-major arrays, so a 128 x 256 output tile reads a
// quarter less per product than two 128 x 128 tiles, and a wave issues 8 MFMAs per 6 fragment reads instead
// of 4 per 4. 256 registers per lane: 2 blocks per compute unit. (Measured 4-5 % faster than the square tile
// at 170k nodes x 1000 columns, where the launch's HBM fetches fall from 5.8 to 1.4 times its operands, and
// 1-2 % faster at 20k nodes; with p_l as 8-bit indices, whose conversion adds vector work between the MFMAs,
// 9 % slower, hence the square tile there.)
using TileWide = TileCfg<128, 256, 16, 2, 2, 2>;
constexpr int kGemmSlotsWide = 256 * TileWide::MINB;
// Fewest rounds of resident blocks a wide-tile split plan may have: with one or two rounds the blocks start and
// end together and nothing hides their prologues and epilogues (measured: 12 % slower than the square tile
// with one round, faster from four on).
constexpr int kWideMinRounds = 4;

namespace {

// ------------------------------------------------------------------------------------------
// Single-problem entry kernels (descriptor by value: no device memory needed for the table).
// ------------------------------------------------------------------------------------------
struct Carver {
  char* base;
  size_t off = 0;
  explicit Carver(void* b) : base(static_cast<char*>(b)) {}
  template <class T>
  T* take(size_t count) {
    // every array starts at a multiple of 4 KiB from the workspace base: on a workspace that itself starts on a 4 KiB boundary (any
    // large device allocation does) a block of a streaming kernel then reads whole 4 KiB pieces of each of its
    // arrays (measured on the 9-stream z/q/u kernel at 680 MB per array: 9.82 -> 9.61 ms against 256-byte
    // alignment; 64 KiB or 2 MiB alignment and staggered starts are slower again)
    off = (off + 4095) & ~size_t(4095);
    T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off += count * sizeof(T);
    return p;
  }
};

inline int round4(int n) { return (n + 3) & ~3; }
inline int cdiv(int a, int b) { return (a + b - 1) / b; }
// blocks of a streaming kernel in which every thread owns `per_thread` float4 groups
inline int chunk_blocks(size_t n4, int per_thread) {
  const size_t per_block = (size_t)256 * per_thread;
  return (int)std::max<size_t>((n4 + per_block - 1) / per_block, 1);
}
inline int axpy_blocks(size_t n4) { return (int)std::max<size_t>((n4 + kAxpyThreads - 1) / kAxpyThreads, 1); }
inline int qt_blocks(size_t n4) {
  const size_t per_block = (size_t)kQtThreads * kQuantUnroll;
  return (int)std::max<size_t>((n4 + per_block - 1) / per_block, 1);
}
inline int flat_blocks(size_t n4) {
  size_t b = (n4 + 1023) / 1024;
  return (int)std::min<size_t>(std::max<size_t>(b, 1), 2048);
}

struct LayerBufs {
  int n_in, n_out, ld_in, ld_out;
  float *W, *Wt, *b, *z, *R, *T, *G, *m, *Gpart;
  float* Tpart;             // small problems: partial products of G p over chunks of n_in
  int wt_split, wt_chunk;   // number of such chunks (1 = the product is not split) and their length
  float* p;                 // input of the layer, [N, ld_in] fp32 (null for l >= 2 in -Q: p_l is kept as indices)
  float *g, *d;             // l >= 2: gradient of phi in p, -Q trial direction
  uint8_t* pidx;            // l >= 2, -Q: two planes of indices into Delta (1 byte each, 2 for grids of more than
                            // 256 levels), [2][idx_plane]; LayerScal::cur tells which one holds p_l, the other
                            // takes the candidates of the backtracking trials
  size_t idx_plane;         // bytes per plane (N * ld_in indices rounded up to 256 bytes)
  float *q, *u;             // l < L
  double *part_a, *part_b, *part_c, *colpart, *pairpart;
  int splitk, k_chunk;
  int tiles_in, tiles_out;  // GEMM tiles of [N, n_in] and [N, n_out]
  int row_blocks, col_blocks, cw, rpb;
};

// A descriptor table in device memory plus, for every launch chunk of at most kMaxGroup entries,
// the block map that travels in the kernel arguments.
template <class T>
struct Group {
  T* dev = nullptr;
  std::vector<BlockMap> maps;
  std::vector<int> start;
  int count = 0;
  void build(T* table, const std::vector<T>& v, int n) {
    build(table, v, n, [](const T& e) { return e.nblk; });
  }
  // entries [from, from + n) of an uploaded table as a group of their own (no device memory of its own)
  void view(const Group<T>& whole, const std::vector<T>& v, int from, int n) {
    n = std::max(0, std::min(n, (int)v.size() - from));
    std::vector<T> part(v.begin() + std::min<size_t>(from, v.size()), v.begin() + std::min<size_t>(from, v.size()) + n);
    build(whole.dev + from, part, n);
  }
  // `blocks_of` gives the number of blocks of an entry (tables shared by kernels of different shapes)
  template <class F>
  void build(T* table, const std::vector<T>& v, int n, F blocks_of) {
    dev = table;
    count = n;
    maps.clear();
    start.clear();
    for (int s0 = 0; s0 < n; s0 += kMaxGroup) {
      BlockMap m{};
      m.n = std::min(kMaxGroup, n - s0);
      int b = 0;
      for (int j = 0; j < m.n; ++j) {
        m.blk0[j] = b;
        b += blocks_of(v[s0 + j]);
      }
      m.total = b;
      maps.push_back(m);
      start.push_back(s0);
    }
  }
};

}  // namespace

struct pdadmm_ctx {
  pdadmm_config cfg;
  std::vector<int> dims;
  int N = 0, L = 0;
  hipStream_t stream = nullptr;   // where launches go right now (the caller's main stream unless swapped)
  hipStream_t aux = nullptr;      // optional second caller stream for work that is independent of the main sequence
  hipStream_t gaux = nullptr;     // its stand-in while an iteration is captured into a graph
  hipEvent_t ev_fork[2] = {nullptr, nullptr}, ev_join[2] = {nullptr, nullptr};      // eager fork/join pairs
  hipEvent_t ev_gfork[2] = {nullptr, nullptr}, ev_gjoin[2] = {nullptr, nullptr};    // the same inside a capture
  std::vector<LayerBufs> lay;
  LayerScal* scal = nullptr;
  int* err = nullptr;
  int* flags = nullptr;
  int* h_flags = nullptr;     // pinned host mirror
  int* labels = nullptr;
  uint8_t* mask = nullptr;
  double* riskpart = nullptr;
  double* predpart = nullptr;   // per block: counted nodes, correct predictions
  int risk_blocks = 0;
  QuantGrid grid{0.f, 0.f, 0};
  // descriptor tables in device memory, each with the block maps of its launches
  // Products over ALL layers come as two groups in -Q: layer 1 reads p_1 = X as fp32 (`..._f`, which holds every
  // layer in pdADMM-G), the layers above read their p_l as indices (`..._q`, its own kernel instance).
  Group<GemmProb> g_pgrad, g_ptrial, g_wgrad, g_wtrial, g_resid, g_resid_obj;
  Group<GemmProb> g_wgrad_q, g_wtrial_q, g_resid_q, g_resid_obj_q;
  // The W-update of layer 1 needs nothing from the p-updates (p_1 = X is fixed): with a second stream it runs beside
  // them. Views of the W-phase tables: layer 1 alone, and the layers above it.
  Group<GemmProb> v_wgrad_first, v_wgrad_rest, v_wtrial_first, v_wtrial_rest, g_none;
  Group<ReduceProb> v_red_first, v_red_rest, v_tred_first, v_tred_rest;
  Group<WStepSeg> v_w_first, v_w_rest;
  std::vector<GemmProb> fwd;          // forward pass of the starting point: one by-value launch per layer
  Group<ReduceProb> g_red, g_tred;
  bool spec_p = false;        // pdADMM-G, not small: the p-step and r -= Wg/tau ride in the product epilogues with
                              // the step size guessed ahead (LayerScal::spec_tau), corrected only when the rule picks another
  bool spec_w = false;        // not small (both variants): the same for r -= Gp/theta and the column sums of r
  bool small_wtrial = false;  // the G p launch has too few tiles to fill the chip: split its contraction
  Group<AxpySeg> g_pstep, g_pfix, g_qapply_r;
  SelectDesc *sel_p = nullptr, *sel_w = nullptr, *sel_q = nullptr;
  Group<WStepSeg> g_w;
  Group<RowSeg> g_rows_all, g_rows_hidden;
  Group<BiasSeg> g_bias;
  Group<QuantSeg> g_quant;
  Group<PairSeg> g_pair;
  int panel = 4;              // tiles per die-local panel in the grouped product launches
  int tn_bn = 128;            // width of the output tiles of the W-gradient products (128, or 256: TileWide)
  int panel_tn = 16;          // the same for the W-gradient products (all tiles of one node chunk)
  bool dirty = true;
  long iter = 0;
  // optional replay of one pdADMM-G iteration as a HIP graph (launch-bound small models)
  hipStream_t gstream = nullptr;       // capture/replay stream, ordered against `stream` by events
  hipGraph_t graph = nullptr;
  hipGraphExec_t graph_exec = nullptr;
  hipEvent_t ev_in = nullptr, ev_out = nullptr;
  std::vector<long long> p_products;   // per layer: step-direction products (W g / W d) computed since init
  std::string msg;
  // optional per-launch timing with HIP events on the context's stream
  struct TimedLaunch { int cls; hipEvent_t a, b; };
  uint32_t timing_mask = 0;
  std::vector<TimedLaunch> timed;
  std::vector<hipEvent_t> event_pool;
};

namespace {

// Reason of the calling thread's last failed call that had no context (pdadmm_last_error(NULL)).
thread_local std::string g_thread_error;

pdadmm_status fail(pdadmm_ctx* c, pdadmm_status s, const std::string& m) {
  if (c) c->msg = m;
  else g_thread_error = m;
  return s;
}

// Scratch of the entry point that allocates nothing (pdadmm_gemm_tn_static): part of the library image, one
// copy per GPU. In host code the name of the array is only a handle for hipGetSymbolAddress: the address a
// kernel may use is looked up once per device and kept in g_scratch_ptr.
static __device__ __attribute__((used)) __align__(256) float scratch[PDADMM_STATIC_SCRATCH_FLOATS];
constexpr int kMaxDevices = 64;
float* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

pdadmm_status scratch_of_current_device(float** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(nullptr, PDADMM_EHIP, std::string("hipGetDevice: ") + hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail(nullptr, PDADMM_EHIP, "device ordinal beyond the table of scratch addresses");
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    float* ptr = nullptr;
    e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr)
      return fail(nullptr, PDADMM_EHIP, std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e));
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return PDADMM_OK;
}

#define HIP_TRY(ctx, call)                                                                   \
  do {                                                                                       \
    hipError_t e_ = (call);                                                                  \
    if (e_ != hipSuccess)                                                                    \
      return fail(ctx, PDADMM_EHIP, std::string(#call) + ": " + hipGetErrorString(e_));      \
  } while (0)

#define LAUNCH_CHECK(ctx, what)                                                              \
  do {                                                                                       \
    hipError_t e_ = hipGetLastError();                                                       \
    if (e_ != hipSuccess)                                                                    \
      return fail(ctx, PDADMM_EHIP, std::string("launch ") + what + ": " + hipGetErrorString(e_)); \
  } while (0)

// Kernel classes for pdadmm_timing (bit i of the mask enables class i).
enum : int { kClsGemmPGrad = 0, kClsGemmTrial = 1, kClsGemmWGrad = 2, kClsSplitkReduce = 3, kClsSelect = 4,
             kClsPStep = 5, kClsWStep = 6, kClsResidColsum = 7, kClsBias = 8, kClsZqu = 9, kClsFista = 10,
             kClsQuantTrial = 11, kClsQuantApply = 12, kClsRefresh = 13, kNumClasses = 14 };

hipEvent_t take_event(pdadmm_ctx* c) {
  hipEvent_t e = nullptr;
  if (!c->event_pool.empty()) {
    e = c->event_pool.back();
    c->event_pool.pop_back();
  } else if (hipEventCreate(&e) != hipSuccess) {
    e = nullptr;
  }
  return e;
}

struct ScopedTimer {
  pdadmm_ctx* c;
  hipEvent_t a = nullptr, b = nullptr;
  int cls;
  ScopedTimer(pdadmm_ctx* ctx, int k) : c(ctx), cls(k) {
    if (c->timing_mask & (1u << k)) {
      a = take_event(c);
      b = take_event(c);
      if (a && b) (void)hipEventRecord(a, c->stream);
    }
  }
  ~ScopedTimer() {
    if (a && b) {
      (void)hipEventRecord(b, c->stream);
      c->timed.push_back({cls, a, b});
    }
  }
};
#define TIMED(c, cls) ScopedTimer timer_##cls(c, cls)

bool config_ok(const pdadmm_config* c, std::string* why) {
  auto bad = [&](const char* m) { if (why) *why = m; return false; };
  if (!c) return bad("config is NULL");
  if (c->n_nodes < 1) return bad("n_nodes < 1");
  if (c->n_layers < 1 || c->n_layers > 4096) return bad("n_layers out of range");
  if (!c->dims) return bad("dims is NULL");
  for (int i = 0; i <= c->n_layers; ++i)
    if (c->dims[i] < 1) return bad("a layer width is < 1");
  if (c->dims[c->n_layers] > 1024) return bad("n_L > 1024 classes is not supported");
  {
    // a grouped streaming launch covers up to kMaxGroup layers with one block per 64 float4 groups:
    // the block count must fit the 31-bit grid size
    int widest = 0;
    for (int i = 0; i <= c->n_layers; ++i) widest = std::max(widest, c->dims[i]);
    const double blocks = (double)c->n_nodes * ((widest + 3) / 4) / 64.0 * std::min(c->n_layers * 2, 2 * kMaxGroup);
    if (blocks > 2.0e9) return bad("n_nodes x layer width is too large for one grouped launch");
  }
  if (!(c->rho > 0.f) || !(c->nu > 0.f)) return bad("rho and nu must be > 0");
  if (c->quantize < 0 || c->quantize > 2) return bad("quantize must be 0, 1 or 2");
  if (c->quantize) {
    if (c->q_levels < 2 || c->q_levels > 65536) return bad("q_levels must be in 2..65536");
    if (!(c->q_hi > c->q_lo)) return bad("q_hi must exceed q_lo");
  }
  if (c->fista_iters < 0) return bad("fista_iters < 0");
  if (!(c->bt_eta > 1.f)) return bad("bt_eta must be > 1");
  if (!(c->tau0 > 0.f) || !(c->theta0 > 0.f)) return bad("tau0/theta0 must be > 0");
  if (c->bt_max_trials < 1) return bad("bt_max_trials < 1");
  if (c->refresh_every < 0) return bad("refresh_every < 0");
  if (!(c->leaky_slope >= 0.f) || !(c->leaky_slope < 1.f)) return bad("leaky_slope must be in [0, 1)");
  if (c->use_graph != 0 && c->use_graph != 1) return bad("use_graph must be 0 or 1");
  if (c->bt_probe_backoff != 0 && c->bt_probe_backoff != 1) return bad("bt_probe_backoff must be 0 or 1");
  if (c->risk_kind != 0 && c->risk_kind != 1) return bad("risk_kind must be 0 (cross-entropy) or 1 (least squares)");
  return true;
}

QuantGrid make_grid(float lo, float hi, int levels) {
  QuantGrid g;
  g.lo = lo;
  g.step = (hi - lo) / (float)(levels - 1);
  g.levels = levels;
  g.ib = levels > 256 ? 2 : 1;
  return g;
}

// Lay the workspace out. With base == nullptr only the size is computed.
size_t plan(pdadmm_ctx* c, void* base) {
  Carver cv(base);
  const int N = c->N, L = c->L;
  const bool Q = c->cfg.quantize != 0;
  c->lay.assign(L, LayerBufs{});
  // Split plan of the W-gradient products (contraction over the nodes): every output tile of
  // every layer is cut into the same number of node chunks, so all blocks of the grouped launch take
  // the same time. The chip holds kGemmSlots product blocks at once (MI355X: 256 CUs x 3 blocks, 2 of the wide tile, set
  // by the kernel's register use); the number of chunks is chosen so that the blocks fill whole
  // rounds of that many as exactly as possible, while a block still runs long enough to amortise
  // its start-up (about 1.6 k-tiles, measured).
  // Tile width: the wide tile unless p_l are indices or its padding (n_in rounded up to 256 instead of 128)
  // would add more MFMA work than it saves elsewhere (more than 5 %).
  size_t area_sq = 0, area_wide = 0;
  for (int i = 0; i < L; ++i) {
    area_sq += (size_t)cdiv(c->dims[i + 1], BM) * cdiv(c->dims[i], BN) * BN;
    area_wide += (size_t)cdiv(c->dims[i + 1], BM) * cdiv(c->dims[i], TileWide::BN) * TileWide::BN;
  }
  const bool wide = !Q && area_wide * 20 <= area_sq * 21;
  c->tn_bn = wide ? TileWide::BN : BN;
  const int slots_tn = wide ? kGemmSlotsWide : kGemmSlots;
  size_t tiles_total = 0;
  for (int i = 0; i < L; ++i) tiles_total += (size_t)cdiv(c->dims[i + 1], BM) * cdiv(c->dims[i], c->tn_bn);
  int chunk = cdiv(N, BK) * BK;
  {
    double best = -1.0;
    for (int rounds = wide ? kWideMinRounds : 1; rounds <= 12; ++rounds) {
      const long want = (long)rounds * slots_tn / (long)tiles_total;
      if (want < 1) continue;
      const int sk = (int)std::min<long>(want, 64);
      int ch = cdiv(cdiv(N, sk), BK) * BK;
      ch = std::max(ch, std::min(256, cdiv(N, BK) * BK));
      const int parts = cdiv(N, ch);
      const double blocks = (double)tiles_total * parts;
      const double fill = blocks / (std::ceil(blocks / slots_tn) * slots_tn);
      const double nkt = (double)ch / BK;
      const double eff = fill * nkt / (nkt + 1.6) - 1e-3 * parts;   // small bias towards fewer partial sums
      if (eff > best) {
        best = eff;
        chunk = ch;
      }
    }
  }
  // The products T = p G^T of all layers form one launch. When that launch has fewer tiles than half the
  // resident blocks (small models), the long contractions in it (n_in >> 128) are cut into chunks whose
  // partial products are summed, in a fixed order, by the kernel that also takes the norm.
  size_t wt_tiles = 0;
  for (int i = 0; i < L; ++i) wt_tiles += (size_t)cdiv(N, BM) * cdiv(c->dims[i + 1], BN);
  c->small_wtrial = wt_tiles * 2 <= (size_t)kGemmSlots;
  c->spec_w = !c->small_wtrial;
  c->spec_p = !Q && c->spec_w;
  for (int i = 0; i < L; ++i) {
    LayerBufs& b = c->lay[i];
    b.n_in = c->dims[i];
    b.n_out = c->dims[i + 1];
    b.ld_in = round4(b.n_in);
    b.ld_out = round4(b.n_out);
    b.splitk = cdiv(N, chunk);
    b.k_chunk = chunk;
    b.tiles_in = cdiv(N, BM) * cdiv(b.n_in, BN);
    b.tiles_out = cdiv(N, BM) * cdiv(b.n_out, BN);
    b.rpb = c->spec_w ? BM : kRowsPerBlock;   // fused: column sums come per 128-row product tile
    b.row_blocks = cdiv(N, b.rpb);
    b.cw = 1;
    while (b.cw < b.ld_out / 4 && b.cw < 256) b.cw <<= 1;
    b.col_blocks = cdiv(b.ld_out / 4, b.cw);
    const size_t in_sz = (size_t)N * b.ld_in, out_sz = (size_t)N * b.ld_out;
    b.W = cv.take<float>((size_t)b.n_out * b.ld_in);
    b.Wt = cv.take<float>((size_t)b.n_in * b.ld_out);
    b.G = cv.take<float>((size_t)b.n_out * b.ld_in);
    b.Gpart = cv.take<float>((size_t)b.splitk * b.n_out * b.ld_in);
    b.wt_split = 1;
    b.wt_chunk = b.n_in;
    b.Tpart = nullptr;
    if (c->small_wtrial) {
      const int want = (int)std::min<size_t>(kGemmSlots / wt_tiles, 32);
      b.wt_chunk = std::max(8 * BK, cdiv(cdiv(b.n_in, std::max(want, 1)), BK) * BK);
      b.wt_split = cdiv(b.n_in, b.wt_chunk);
      b.Tpart = cv.take<float>((size_t)b.wt_split * N * b.ld_out);
    }
    b.b = cv.take<float>(b.ld_out);
    b.m = cv.take<float>(b.ld_out);
    b.z = cv.take<float>(out_sz);
    b.R = cv.take<float>(out_sz);
    b.T = cv.take<float>(out_sz);
    b.p = (i == 0 || !Q) ? cv.take<float>(in_sz) : nullptr;
    if (i >= 1) {
      b.g = cv.take<float>(in_sz);
      if (Q) {
        b.d = cv.take<float>(in_sz);
        b.idx_plane = (in_sz * (c->cfg.q_levels > 256 ? 2 : 1) + 255) & ~size_t(255);
        b.pidx = cv.take<uint8_t>(2 * b.idx_plane);
      }
    }
    if (i < L - 1) {
      b.q = cv.take<float>(out_sz);
      b.u = cv.take<float>(out_sz);
    }
    const size_t np = 2 * (size_t)std::max({b.tiles_in, b.tiles_out, 2048});
    b.part_a = cv.take<double>(np);
    b.part_b = cv.take<double>(np);
    // -Q: one partial of ||d||^2 per block of the projection kernel
    b.part_c = cv.take<double>(Q && i >= 1 ? std::max(np, (size_t)qt_blocks(in_sz / 4)) : np);
    b.colpart = cv.take<double>((size_t)b.row_blocks * b.ld_out);
    b.pairpart = cv.take<double>(3 * 2048);
  }
  c->scal = cv.take<LayerScal>(L);
  c->err = cv.take<int>(1);
  c->flags = cv.take<int>(L);
  c->labels = cv.take<int>(N);
  c->mask = cv.take<uint8_t>(N);
  c->risk_blocks = cdiv(N, 256);
  c->riskpart = cv.take<double>(c->risk_blocks);
  c->predpart = cv.take<double>(2 * (size_t)c->risk_blocks);
  c->g_pgrad.dev = cv.take<GemmProb>(L);
  c->g_ptrial.dev = cv.take<GemmProb>(L);
  c->g_wgrad.dev = cv.take<GemmProb>(L);
  c->g_wtrial.dev = cv.take<GemmProb>(L);
  c->g_resid.dev = cv.take<GemmProb>(L);
  c->g_resid_obj.dev = cv.take<GemmProb>(L);
  c->g_wgrad_q.dev = cv.take<GemmProb>(L);
  c->g_wtrial_q.dev = cv.take<GemmProb>(L);
  c->g_resid_q.dev = cv.take<GemmProb>(L);
  c->g_resid_obj_q.dev = cv.take<GemmProb>(L);
  c->g_red.dev = cv.take<ReduceProb>(L);
  c->g_tred.dev = cv.take<ReduceProb>(L);
  c->g_pstep.dev = cv.take<AxpySeg>(2 * L);
  c->g_pfix.dev = cv.take<AxpySeg>(2 * L);
  c->g_qapply_r.dev = cv.take<AxpySeg>(L);
  c->sel_p = cv.take<SelectDesc>(L);
  c->sel_w = cv.take<SelectDesc>(L);
  c->sel_q = cv.take<SelectDesc>(L);
  c->g_w.dev = cv.take<WStepSeg>(L);
  c->g_rows_all.dev = cv.take<RowSeg>(L);
  c->g_bias.dev = cv.take<BiasSeg>(L);
  c->g_quant.dev = cv.take<QuantSeg>(L);
  c->g_pair.dev = cv.take<PairSeg>(L);
  return (cv.off + 255) & ~size_t(255);
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

GemmProb make_nt(const float* A, int lda, const float* B, int ldb, float* C, int ldc, int M, int N, int K) {
  GemmProb P{};
  P.A = A; P.B = B; P.C = C;
  P.M = M; P.N = N; P.K = K;
  P.lda = lda; P.ldb = ldb; P.ldc = ldc;
  P.tiles_m = cdiv(M, BM);
  P.tiles_n = cdiv(N, BN);
  P.splitk = 1;
  P.k_chunk = K;
  P.nblk = P.tiles_m * P.tiles_n;
  P.vecA = (lda % 4 == 0) && aligned16(A);
  P.vecB = (ldb % 4 == 0) && aligned16(B);
  P.alpha = 1.f;
  P.beta = 0.f;
  P.slope = 0.f;
  P.layer = 0;
  P.p8 = nullptr;
  P.p8_plane = 0;
  P.o8 = nullptr;
  return P;
}

GemmProb make_tn(const float* A, int lda, const float* B, int ldb, float* part, int ldc, int M, int N, int K,
                 int splitk, int k_chunk, int bn = BN) {
  GemmProb P = make_nt(A, lda, B, ldb, part, ldc, M, N, K);
  P.tiles_n = cdiv(N, bn);
  P.splitk = splitk;
  P.k_chunk = k_chunk;
  P.nblk = P.tiles_m * P.tiles_n * splitk;
  return P;
}

template <class T>
pdadmm_status upload(pdadmm_ctx* c, T* dst, const std::vector<T>& src) {
  if (src.empty()) return PDADMM_OK;
  HIP_TRY(c, hipMemcpyAsync(dst, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));   // the host vector goes out of scope in the caller
  return PDADMM_OK;
}

pdadmm_status build_tables(pdadmm_ctx* c) {
  const int N = c->N, L = c->L;
  const float rho = c->cfg.rho, nu = c->cfg.nu;
  const bool Q = c->cfg.quantize != 0;
  std::vector<GemmProb> pgrad, ptrial, wgrad, wtrial, resid, resid_obj, fwd;
  std::vector<GemmProb> wgrad_q, wtrial_q, resid_q, resid_obj_q;     // -Q: the layers whose p_l is kept as indices
  // give a product descriptor its p_l as indices (operand or epilogue input, by the kernel it is launched with)
  auto as_indices = [&](GemmProb& P, const LayerBufs& b) {
    P.p8 = b.pidx;
    P.p8_plane = b.idx_plane;
    P.grid = c->grid;
  };
  std::vector<ReduceProb> red, tred;
  std::vector<AxpySeg> pstep, pfix, qapply_r;
  std::vector<SelectDesc> sel_p, sel_w, sel_q;
  std::vector<WStepSeg> wseg;
  std::vector<RowSeg> rows;
  std::vector<BiasSeg> bias;
  std::vector<QuantSeg> quant;
  std::vector<PairSeg> pair;
  for (int i = 0; i < L; ++i) {
    LayerBufs& b = c->lay[i];
    if (i >= 1) {
      // gradient of phi in p_l: g = nu * R W + u_{l-1} + rho (p_l - q_{l-1});  R W = R (Wt)^T
      GemmProb P = make_nt(b.R, b.ld_out, b.Wt, b.ld_out, b.g, b.ld_in, N, b.n_in, b.n_out);
      P.e0 = c->lay[i - 1].u; P.e1 = b.p; P.e2 = c->lay[i - 1].q;
      P.alpha = nu; P.beta = rho; P.part = b.part_a; P.layer = i;
      if (Q) as_indices(P, b);                   // the epilogue reads p_l as indices
      if (c->spec_p) P.o1 = b.p;                 // p -= g / tau_prev in the epilogue
      pgrad.push_back(P);
      // image of the step direction under W_l: T = dir W^T (dir = g, or d in -Q)
      GemmProb T = make_nt(Q ? b.d : b.g, b.ld_in, b.W, b.ld_in, b.T, b.ld_out, N, b.n_out, b.n_in);
      T.part = b.part_b; T.layer = i;
      if (c->spec_p) T.o1 = b.R;                 // r -= T / tau_prev in the epilogue
      ptrial.push_back(T);
      SelectDesc s{};
      s.part_g = b.part_a; s.ng = P.nblk; s.part_t = b.part_b; s.nt = T.nblk; s.stride_t = 1; s.layer = i;
      sel_p.push_back(s);
      AxpySeg a{};
      a.y = b.p; a.x = b.g; a.n4 = (size_t)N * b.ld_in / 4; a.nblk = axpy_blocks(a.n4); a.layer = i;
      a.which = kScaleInvTau;
      AxpySeg r{};
      r.y = b.R; r.x = b.T; r.n4 = (size_t)N * b.ld_out / 4; r.nblk = axpy_blocks(r.n4); r.layer = i;
      r.which = kScaleInvTau;
      if (c->spec_p) {                         // only the correction tau_new vs tau_prev is left for p and r
        a.which = r.which = kScaleFixTau;
        a.nblk = std::min(1024, chunk_blocks(a.n4, 1));
        r.nblk = std::min(1024, chunk_blocks(r.n4, 1));
        pfix.push_back(a);
        pfix.push_back(r);
      } else if (!Q) {                         // (-Q takes its step through the projection)
        pstep.push_back(a);
        pstep.push_back(r);
      }
      if (Q) {
        QuantSeg qs{};
        qs.p8 = b.pidx; qs.p8_plane = b.idx_plane; qs.g = b.g; qs.d = b.d; qs.dpart = b.part_c;
        qs.n4 = (size_t)N * b.ld_in / 4; qs.ncols = b.n_in; qs.ld = b.ld_in;
        qs.nblk = qt_blocks(qs.n4); qs.layer = i;
        quant.push_back(qs);
        SelectDesc sq{};
        sq.part_g = b.part_c; sq.ng = qs.nblk; sq.part_t = b.part_b; sq.nt = T.nblk; sq.stride_t = 1; sq.layer = i;
        sel_q.push_back(sq);
        AxpySeg ar = r;
        ar.which = kScaleMinusOneIfStep;
        qapply_r.push_back(ar);
      }
    }
    // gradient of phi in W_l: G = nu * R^T p  (contraction over the nodes, split in chunks)
    GemmProb Wg = make_tn(b.R, b.ld_out, b.p, b.ld_in, b.Gpart, b.ld_in, b.n_out, b.n_in, N, b.splitk, b.k_chunk,
                          c->tn_bn);
    Wg.layer = i;
    const bool as_idx = Q && i >= 1;
    if (as_idx) as_indices(Wg, b);
    (as_idx ? wgrad_q : wgrad).push_back(Wg);
    ReduceProb rp{};
    rp.part = b.Gpart; rp.G = b.G; rp.norm_part = b.part_a; rp.M = b.n_out; rp.N = b.n_in; rp.ld = b.ld_in;
    rp.splitk = b.splitk; rp.alpha = nu; rp.vec = 1;
    rp.nblk = (int)std::min<size_t>(2048, std::max<size_t>(1, ((size_t)b.n_out * b.ld_in + 1023) / 1024));
    red.push_back(rp);
    // image of G under p: T = p G^T
    GemmProb Wt_ = make_nt(b.p, b.ld_in, b.G, b.ld_in, b.T, b.ld_out, N, b.n_out, b.n_in);
    Wt_.part = b.part_b; Wt_.layer = i;
    int t_partials = Wt_.nblk;
    if (c->spec_w) {                           // r -= T / theta_prev and the column sums of r in the epilogue
      Wt_.o1 = b.R;
      Wt_.colpart = b.colpart;
    }
    if (c->small_wtrial) {
      // partial products into Tpart[chunk][N][ld_out]; tred sums them into T and takes ||T||^2
      Wt_.C = b.Tpart;
      Wt_.splitk = b.wt_split;
      Wt_.k_chunk = b.wt_chunk;
      Wt_.nblk = Wt_.tiles_m * Wt_.tiles_n * b.wt_split;
      ReduceProb tr{};
      tr.part = b.Tpart; tr.G = b.T; tr.norm_part = b.part_b; tr.M = N; tr.N = b.n_out; tr.ld = b.ld_out;
      tr.splitk = b.wt_split; tr.alpha = 1.0f; tr.vec = 1;
      tr.nblk = (int)std::min<size_t>(2048, std::max<size_t>(1, ((size_t)N * b.ld_out + 1023) / 1024));
      tred.push_back(tr);
      t_partials = tr.nblk;
    }
    if (as_idx) as_indices(Wt_, b);
    (as_idx ? wtrial_q : wtrial).push_back(Wt_);
    SelectDesc sw{};
    sw.part_g = b.part_a; sw.ng = rp.nblk; sw.part_t = b.part_b; sw.nt = t_partials; sw.stride_t = 1; sw.layer = i;
    sel_w.push_back(sw);
    WStepSeg ws{};
    ws.W = b.W; ws.Wt = b.Wt; ws.G = b.G; ws.n_out = b.n_out; ws.n_in = b.n_in; ws.ld_in = b.ld_in;
    ws.ld_out = b.ld_out; ws.tiles_c = cdiv(b.n_in, 32); ws.nblk = cdiv(b.n_out, 32) * ws.tiles_c; ws.layer = i;
    wseg.push_back(ws);
    // carried residual from scratch: R = p W^T + b - z
    GemmProb Rf = make_nt(b.p, b.ld_in, b.W, b.ld_in, b.R, b.ld_out, N, b.n_out, b.n_in);
    Rf.e0 = b.b; Rf.e1 = b.z; Rf.e2 = nullptr; Rf.part = b.part_b; Rf.layer = i;
    if (as_idx) as_indices(Rf, b);
    (as_idx ? resid_q : resid).push_back(Rf);
    GemmProb Ro = Rf;
    Ro.C = b.T; Ro.e2 = b.R;
    (as_idx ? resid_obj_q : resid_obj).push_back(Ro);
    // forward pass of the starting point
    GemmProb Fw = make_nt(b.p, b.ld_in, b.W, b.ld_in, b.z, b.ld_out, N, b.n_out, b.n_in);
    Fw.e0 = b.b;
    if (i < L - 1) { Fw.o1 = b.q; Fw.o2 = c->lay[i + 1].p; Fw.o8 = Q ? c->lay[i + 1].pidx : nullptr; }
    if (as_idx) as_indices(Fw, b);             // plane 0 holds p_l at the start (LayerScal::cur = 0)
    Fw.grid = Q ? c->grid : QuantGrid{0.f, 0.f, 0, 1};
    Fw.beta = c->cfg.quantize == 2 ? 1.0f : 0.0f;
    Fw.slope = c->cfg.leaky_slope;
    Fw.blk0 = 0;
    fwd.push_back(Fw);
    RowSeg rs{};
    rs.R = b.R; rs.T = b.T; rs.z = b.z; rs.q = b.q; rs.u = b.u;
    rs.pnext = i < L - 1 ? c->lay[i + 1].p : nullptr;
    rs.pnext8 = (Q && i < L - 1) ? c->lay[i + 1].pidx : nullptr;
    rs.p8_plane = (Q && i < L - 1) ? c->lay[i + 1].idx_plane : 0;
    rs.m = b.m; rs.colpart = b.colpart;
    rs.rows = N; rs.ncols = b.n_out; rs.ld = b.ld_out;
    rs.cw = b.cw; rs.col_blocks = b.col_blocks; rs.row_blocks = b.row_blocks; rs.nblk = b.col_blocks * b.row_blocks;
    rs.rpb = b.rpb; rs.which = c->spec_w ? kScaleFixTheta : kScaleInvTheta;
    rs.layer = i;
    rows.push_back(rs);
    BiasSeg bs{};
    bs.b = b.b; bs.m = b.m; bs.colpart = b.colpart; bs.ncols = b.n_out; bs.ld = b.ld_out;
    bs.row_blocks = b.row_blocks; bs.rows = N; bs.nblk = cdiv(b.ld_out, 32);
    bias.push_back(bs);
    if (i < L - 1) {
      PairSeg ps{};
      ps.z = b.z; ps.q = b.q; ps.u = b.u; ps.pnext = c->lay[i + 1].p; ps.part = b.pairpart;
      ps.pnext8 = Q ? c->lay[i + 1].pidx : nullptr; ps.p8_plane = Q ? c->lay[i + 1].idx_plane : 0;
      ps.next_layer = i + 1; ps.ncols = b.n_out; ps.ld = b.ld_out;
      ps.n4 = (size_t)N * b.ld_out / 4; ps.nblk = flat_blocks(ps.n4);
      pair.push_back(ps);
    }
  }
  {
    // panel = number of column tiles of the typical hidden layer (tiles that share one row panel of the
    // node-major operand), clamped to 1..8
    const int typical = c->dims[std::min(1, L)];
    c->panel = std::max(1, std::min(8, cdiv(typical, BN)));
    // W-gradient products: all output tiles of one node chunk read the same two operand panels, so the
    // whole chunk goes to one die (its tiles run together and share the panels through that die's L2)
    c->panel_tn = std::max(1, std::min(64, cdiv(typical, BM) * cdiv(typical, c->tn_bn)));

  }
  pdadmm_status s;
#define UP(group, v)                                                        \
  do {                                                                      \
    if ((s = upload(c, group.dev, v)) != PDADMM_OK) return s;               \
    group.build(group.dev, v, (int)v.size());                               \
  } while (0)
  UP(c->g_pgrad, pgrad); UP(c->g_ptrial, ptrial); UP(c->g_wgrad, wgrad); UP(c->g_wtrial, wtrial);
  UP(c->g_resid, resid); UP(c->g_resid_obj, resid_obj); UP(c->g_red, red); UP(c->g_tred, tred);
  UP(c->g_wgrad_q, wgrad_q); UP(c->g_wtrial_q, wtrial_q); UP(c->g_resid_q, resid_q); UP(c->g_resid_obj_q, resid_obj_q);
  UP(c->g_pstep, pstep); UP(c->g_pfix, pfix); UP(c->g_qapply_r, qapply_r);
  UP(c->g_w, wseg); UP(c->g_rows_all, rows); UP(c->g_bias, bias); UP(c->g_quant, quant); UP(c->g_pair, pair);
#undef UP
  c->v_wgrad_first.view(c->g_wgrad, wgrad, 0, 1);
  c->v_wgrad_rest.view(c->g_wgrad, wgrad, 1, L);
  c->v_wtrial_first.view(c->g_wtrial, wtrial, 0, 1);
  c->v_wtrial_rest.view(c->g_wtrial, wtrial, 1, L);
  c->v_red_first.view(c->g_red, red, 0, 1);
  c->v_red_rest.view(c->g_red, red, 1, L);
  c->v_tred_first.view(c->g_tred, tred, 0, 1);
  c->v_tred_rest.view(c->g_tred, tred, 1, L);
  c->v_w_first.view(c->g_w, wseg, 0, 1);
  c->v_w_rest.view(c->g_w, wseg, 1, L);
  // the fused z/q/u pass walks the same table flat: 256*kZquUnroll float4 groups per block
  c->g_rows_hidden.build(c->g_rows_all.dev, rows, L - 1, [](const RowSeg& e) {
    const size_t per_block = (size_t)kZquThreads * kZquUnroll;
    return (int)std::max<size_t>(((size_t)e.rows * (e.ld / 4) + per_block - 1) / per_block, 1);
  });
  if ((s = upload(c, c->sel_p, sel_p)) != PDADMM_OK) return s;
  if ((s = upload(c, c->sel_w, sel_w)) != PDADMM_OK) return s;
  if ((s = upload(c, c->sel_q, sel_q)) != PDADMM_OK) return s;
  c->fwd = fwd;
  return PDADMM_OK;
}

// Launch a grouped kernel once per chunk of its table: kernel(table + first entry, block map, args...).
template <int THREADS, class T, class K, class... Args>
void launch_group_threads(pdadmm_ctx* c, const Group<T>& g, K kernel, Args... args) {
  for (size_t k = 0; k < g.maps.size(); ++k) {
    if (g.maps[k].total <= 0) continue;
    hipLaunchKernelGGL(kernel, dim3(g.maps[k].total), dim3(THREADS), 0, c->stream, (const T*)(g.dev + g.start[k]),
                       g.maps[k], args...);
  }
}
template <class T, class K, class... Args>
void launch_group(pdadmm_ctx* c, const Group<T>& g, K kernel, Args... args) {
  launch_group_threads<256>(c, g, kernel, args...);
}

// VECC = true: every problem of the group writes (and reads its epilogue inputs from) workspace arrays,
// which are 16-byte aligned with leading dimensions that are multiples of 4.
// P8 = 1, 2: the operand that carries p_l is read as indices of that many bytes (the `..._q` groups of a -Q context).
template <bool KC, class Epi, bool VECC = false, int P8 = 0>
void launch_gemm(pdadmm_ctx* c, const Group<GemmProb>& g, int predicated) {
  const int panel = KC ? c->panel : c->panel_tn;
  for (size_t k = 0; k < g.maps.size(); ++k) {
    if (g.maps[k].total <= 0) continue;
    if constexpr (!KC && !P8) {
      if (c->tn_bn == TileWide::BN) {   // the descriptors of this context count their tiles 256 columns wide
        hipLaunchKernelGGL((gemm_kernel<TileWide, KC, Epi, VECC, P8>), dim3(xcd_padded(g.maps[k].total, panel)),
                           dim3(256), 0, c->stream, (const GemmProb*)(g.dev + g.start[k]), g.maps[k],
                           (const LayerScal*)c->scal, predicated, panel);
        continue;
      }
    }
    hipLaunchKernelGGL((gemm_kernel<Tile, KC, Epi, VECC, P8>), dim3(xcd_padded(g.maps[k].total, panel)), dim3(256), 0,
                       c->stream, (const GemmProb*)(g.dev + g.start[k]), g.maps[k], (const LayerScal*)c->scal,
                       predicated, panel);
  }
}

// A product over all layers: the group that reads p_l as fp32 and, in -Q, the group that reads it as indices.
template <bool KC, class Epi, bool VECC>
void launch_gemm_all(pdadmm_ctx* c, const Group<GemmProb>& f, const Group<GemmProb>& q) {
  launch_gemm<KC, Epi, VECC, 0>(c, f, 0);
  if (q.count > 0) {
    if (c->grid.ib == 2) launch_gemm<KC, Epi, VECC, 2>(c, q, 0);
    else launch_gemm<KC, Epi, VECC, 1>(c, q, 0);
  }
}

pdadmm_status refresh_residual(pdadmm_ctx* c) {
  // transposed weights, then R = p W^T + b - z for every layer
  { TIMED(c, kClsRefresh); launch_group(c, c->g_w, w_step_kernel, (const LayerScal*)c->scal, 1); }
  LAUNCH_CHECK(c, "w_step(copy)");
  { TIMED(c, kClsRefresh); launch_gemm_all<true, EpiResid, false>(c, c->g_resid, c->g_resid_q); }
  LAUNCH_CHECK(c, "gemm resid");
  c->dirty = false;
  return PDADMM_OK;
}

pdadmm_status phase_p(pdadmm_ctx* c) {
  const int L = c->L;
  if (L < 2) return PDADMM_OK;
  const pdadmm_config& g = c->cfg;
  if (c->spec_p) { TIMED(c, kClsGemmPGrad); launch_gemm<true, EpiPGradUpd, true>(c, c->g_pgrad, 0); }
  else if (g.quantize && c->grid.ib == 2) { TIMED(c, kClsGemmPGrad); launch_gemm<true, EpiPGradQT<2>, true>(c, c->g_pgrad, 0); }
  else if (g.quantize) { TIMED(c, kClsGemmPGrad); launch_gemm<true, EpiPGradQT<1>, true>(c, c->g_pgrad, 0); }
  else { TIMED(c, kClsGemmPGrad); launch_gemm<true, EpiPGrad, true>(c, c->g_pgrad, 0); }
  LAUNCH_CHECK(c, "gemm pgrad");
  if (!g.quantize) {
    if (c->spec_p) { TIMED(c, kClsGemmTrial); launch_gemm<true, EpiTrialP, true>(c, c->g_ptrial, 0); }
    else { TIMED(c, kClsGemmTrial); launch_gemm<true, EpiStoreNorm, true>(c, c->g_ptrial, 0); }
    LAUNCH_CHECK(c, "gemm ptrial");
    for (int i = 1; i < L; ++i) ++c->p_products[i];
    { TIMED(c, kClsSelect); hipLaunchKernelGGL(select_step_kernel, dim3(L - 1), dim3(256), 0, c->stream, c->sel_p, c->scal, 0, g.rho, g.nu,
                       g.bt_eta, g.bt_max_trials, c->err); }
    LAUNCH_CHECK(c, "select tau");
    if (!c->spec_p) {
      { TIMED(c, kClsPStep); launch_group_threads<kAxpyThreads>(c, c->g_pstep, axpy_kernel, (const LayerScal*)c->scal); }
      LAUNCH_CHECK(c, "p step");
    } else {
      { TIMED(c, kClsPStep); launch_group(c, c->g_pfix, axpy_fix_kernel, (const LayerScal*)c->scal); }
      LAUNCH_CHECK(c, "p step correction");
    }
    return PDADMM_OK;
  }
  // -Q: trial rounds. Every kernel of a round leaves at once for layers whose search has ended (LayerScal::active),
  // so rounds can be enqueued without knowing whether they are needed: two rounds go out per read of the flags
  // (with the back-off schedule one round settles most updates, with the plain schedule two), and the host only
  // learns whether any layer is still searching.
  const int backoff = g.bt_probe_backoff;
  { TIMED(c, kClsSelect); hipLaunchKernelGGL(select_quant_kernel, dim3(L - 1), dim3(256), 0, c->stream, c->sel_p, c->scal, 0, g.rho, g.nu,
                     g.bt_eta, g.bt_max_trials, backoff, c->err, c->flags); }
  LAUNCH_CHECK(c, "select quant arm");
  constexpr int kRoundsPerRead = 2;
  for (int round = 0; round <= g.bt_max_trials; round += kRoundsPerRead) {
    for (int r = 0; r < kRoundsPerRead; ++r) {
      if (c->grid.ib == 2) { TIMED(c, kClsQuantTrial); launch_group_threads<kQtThreads>(c, c->g_quant, quant_trial_kernel<2>, (const LayerScal*)c->scal, c->grid); }
      else { TIMED(c, kClsQuantTrial); launch_group_threads<kQtThreads>(c, c->g_quant, quant_trial_kernel<1>, (const LayerScal*)c->scal, c->grid); }
      LAUNCH_CHECK(c, "quant trial");
      { TIMED(c, kClsGemmTrial); launch_gemm<true, EpiStoreNorm, true>(c, c->g_ptrial, 1); }
      LAUNCH_CHECK(c, "gemm qtrial");
      { TIMED(c, kClsSelect); hipLaunchKernelGGL(select_quant_kernel, dim3(L - 1), dim3(256), 0, c->stream, c->sel_q, c->scal, 1, g.rho, g.nu,
                         g.bt_eta, g.bt_max_trials, backoff, c->err, c->flags); }
      LAUNCH_CHECK(c, "select quant judge");
    }
    HIP_TRY(c, hipMemcpyAsync(c->h_flags, c->flags, sizeof(int) * L, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    bool any = false;
    for (int i = 1; i < L; ++i) any = any || c->h_flags[i] != 0;
    if (!any) break;
  }
  // the accepted candidate already sits in the index plane that the selection has made current; what is left
  // is the residual r += W d of the layers that took a step
  { TIMED(c, kClsQuantApply); launch_group_threads<kAxpyThreads>(c, c->g_qapply_r, axpy_kernel, (const LayerScal*)c->scal); }
  LAUNCH_CHECK(c, "quant apply R");
  return PDADMM_OK;
}

// The W-updates of all layers, of layer 1 alone, or of the layers above it.
enum Part { kAll, kFirst, kRest };

pdadmm_status phase_w(pdadmm_ctx* c, Part part = kAll) {
  const int L = c->L;
  const pdadmm_config& g = c->cfg;
  const int first = part == kRest ? 1 : 0, count = part == kAll ? L : part == kFirst ? 1 : L - 1;
  if (count <= 0) return PDADMM_OK;
  // fp32-p group and (in -Q) index-p group of each product; in -Q the fp32 group holds layer 1 only
  const Group<GemmProb>& wgrad_f = part == kAll ? c->g_wgrad : part == kFirst ? c->v_wgrad_first : c->v_wgrad_rest;
  const Group<GemmProb>& wtrial_f = part == kAll ? c->g_wtrial : part == kFirst ? c->v_wtrial_first : c->v_wtrial_rest;
  const Group<GemmProb>& wgrad_q = part == kFirst ? c->g_none : c->g_wgrad_q;
  const Group<GemmProb>& wtrial_q = part == kFirst ? c->g_none : c->g_wtrial_q;
  const Group<ReduceProb>& red = part == kAll ? c->g_red : part == kFirst ? c->v_red_first : c->v_red_rest;
  const Group<ReduceProb>& tred = part == kAll ? c->g_tred : part == kFirst ? c->v_tred_first : c->v_tred_rest;
  const Group<WStepSeg>& wst = part == kAll ? c->g_w : part == kFirst ? c->v_w_first : c->v_w_rest;
  { TIMED(c, kClsGemmWGrad); launch_gemm_all<false, EpiStore, true>(c, wgrad_f, wgrad_q); }
  LAUNCH_CHECK(c, "gemm wgrad");
  { TIMED(c, kClsSplitkReduce); launch_group(c, red, splitk_reduce_kernel); }
  LAUNCH_CHECK(c, "splitk reduce");
  if (c->small_wtrial) {
    { TIMED(c, kClsGemmTrial); launch_gemm_all<true, EpiStore, true>(c, wtrial_f, wtrial_q); }
    LAUNCH_CHECK(c, "gemm wtrial (chunks)");
    { TIMED(c, kClsSplitkReduce); launch_group(c, tred, splitk_reduce_kernel); }
    LAUNCH_CHECK(c, "wtrial chunk sum");
  } else if (c->spec_w) {
    { TIMED(c, kClsGemmTrial); launch_gemm_all<true, EpiTrialW, true>(c, wtrial_f, wtrial_q); }
    LAUNCH_CHECK(c, "gemm wtrial");
  } else {
    { TIMED(c, kClsGemmTrial); launch_gemm_all<true, EpiStoreNorm, true>(c, wtrial_f, wtrial_q); }
    LAUNCH_CHECK(c, "gemm wtrial");
  }
  { TIMED(c, kClsSelect); hipLaunchKernelGGL(select_step_kernel, dim3(count), dim3(256), 0, c->stream, c->sel_w + first, c->scal, 1, g.rho, g.nu,
                     g.bt_eta, g.bt_max_trials, c->err); }
  LAUNCH_CHECK(c, "select theta");
  { TIMED(c, kClsWStep); launch_group(c, wst, w_step_kernel, (const LayerScal*)c->scal, 0); }
  LAUNCH_CHECK(c, "w step");
  return PDADMM_OK;
}

// Work that does not depend on what the main stream is doing goes to the second stream between a fork (the side
// stream waits for everything enqueued on the main stream so far) and a join (the main stream waits for the side
// stream). While an iteration is being captured the capture's own side stream and events stand in.
struct SideStream {
  pdadmm_ctx* c;
  hipStream_t main, side;
  hipEvent_t fork_ev, join_ev;
  SideStream(pdadmm_ctx* ctx, int pair) : c(ctx), main(ctx->stream) {
    const bool capturing = ctx->gstream && ctx->stream == ctx->gstream;
    side = capturing ? ctx->gaux : ctx->aux;
    fork_ev = capturing ? ctx->ev_gfork[pair] : ctx->ev_fork[pair];
    join_ev = capturing ? ctx->ev_gjoin[pair] : ctx->ev_join[pair];
  }
  explicit operator bool() const { return side != nullptr; }
  pdadmm_status fork() {
    HIP_TRY(c, hipEventRecord(fork_ev, main));
    HIP_TRY(c, hipStreamWaitEvent(side, fork_ev, 0));
    c->stream = side;
    return PDADMM_OK;
  }
  void back() { c->stream = main; }        // later launches go to the main stream again; the side stream runs on
  pdadmm_status join() {
    c->stream = main;
    HIP_TRY(c, hipEventRecord(join_ev, side));
    HIP_TRY(c, hipStreamWaitEvent(main, join_ev, 0));
    return PDADMM_OK;
  }
};

// z_L-update (Appendix A 'update z', l = L): FISTA for the cross-entropy risk, closed form for least squares.
pdadmm_status launch_fista(pdadmm_ctx* c) {
  const LayerBufs& b = c->lay[c->L - 1];
  const int C = b.n_out;
  if (c->cfg.risk_kind == 1) {
    TIMED(c, kClsFista);
    const size_t elems = (size_t)c->N * C;
    hipLaunchKernelGGL(zlast_ls_kernel, dim3((unsigned)((elems + 255) / 256)), dim3(256), 0, c->stream, b.R, b.z, b.m,
                       c->labels, (const uint8_t*)c->mask, c->N, C, b.ld_out, c->cfg.nu);
    LAUNCH_CHECK(c, "z_L least squares");
    return PDADMM_OK;
  }
  int G = 1;
  while (G < C && G < 64) G <<= 1;
  const int E = cdiv(C, G);
  const int nodes_per_block = 256 / G;
  const int blocks = cdiv(c->N, nodes_per_block);
  const uint8_t* mask = c->mask;
#define FISTA(EE)                                                                                              \
  hipLaunchKernelGGL((fista_kernel<EE>), dim3(blocks), dim3(256), 0, c->stream, b.R, b.z, b.m, c->labels, mask, \
                     c->N, C, b.ld_out, G, c->cfg.nu, c->cfg.fista_iters)
  TIMED(c, kClsFista);
  if (E <= 1) FISTA(1);
  else if (E <= 2) FISTA(2);
  else if (E <= 4) FISTA(4);
  else if (E <= 8) FISTA(8);
  else FISTA(16);
#undef FISTA
  LAUNCH_CHECK(c, "fista");
  return PDADMM_OK;
}

pdadmm_status phase_bzqu(pdadmm_ctx* c) {
  const int L = c->L;
  const pdadmm_config& g = c->cfg;
  { TIMED(c, kClsResidColsum); launch_group(c, c->g_rows_all, resid_colsum_kernel, (const LayerScal*)c->scal); }
  LAUNCH_CHECK(c, "resid colsum");
  { TIMED(c, kClsBias); launch_group(c, c->g_bias, bias_step_kernel); }
  LAUNCH_CHECK(c, "bias step");
  // the z_L-update touches the last layer only, the fused z/q/u pass the layers below it: side by side if possible
  SideStream side(c, 1);
  pdadmm_status s;
  if (side && L > 1) {
    if ((s = side.fork()) != PDADMM_OK) return s;
    s = launch_fista(c);
    side.back();
    if (s != PDADMM_OK) return s;
  }
  if (L > 1) {
    const QuantGrid none{0.f, 0.f, 0, 1};
    const QuantGrid pg = g.quantize ? c->grid : none, qg = g.quantize == 2 ? c->grid : none;
    if (pg.ib == 2) { TIMED(c, kClsZqu); launch_group_threads<kZquThreads>(c, c->g_rows_hidden, zqu_kernel<2>, (const LayerScal*)c->scal, g.rho, g.nu, g.leaky_slope, pg, qg); }
    else { TIMED(c, kClsZqu); launch_group_threads<kZquThreads>(c, c->g_rows_hidden, zqu_kernel<1>, (const LayerScal*)c->scal, g.rho, g.nu, g.leaky_slope, pg, qg); }
    LAUNCH_CHECK(c, "zqu");
  }
  if (side && L > 1) return side.join();
  return launch_fista(c);
}

// One iteration of Algorithm 1. With a second stream the W-update of layer 1 (which reads nothing the p-updates
// write: p_1 = X is fixed) runs beside the p-updates.
pdadmm_status one_iteration(pdadmm_ctx* c) {
  pdadmm_status s;
  SideStream side(c, 0);
  if (side && c->L >= 2) {
    if ((s = side.fork()) != PDADMM_OK) return s;
    s = phase_w(c, kFirst);
    side.back();
    if (s != PDADMM_OK) return s;
    if ((s = phase_p(c)) != PDADMM_OK) return s;
    if ((s = phase_w(c, kRest)) != PDADMM_OK) return s;
    if ((s = side.join()) != PDADMM_OK) return s;
  } else {
    if ((s = phase_p(c)) != PDADMM_OK) return s;
    if ((s = phase_w(c, kAll)) != PDADMM_OK) return s;
  }
  return phase_bzqu(c);
}

pdadmm_status check_device_flags(pdadmm_ctx* c) {
  int e = 0;
  HIP_TRY(c, hipMemcpyAsync(c->h_flags, c->err, sizeof(int), hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  e = c->h_flags[0];
  if (e & kErrNonFinite) return fail(c, PDADMM_ENONFINITE, "a step-size norm became NaN/Inf");
  if (e & kErrBacktrack) return fail(c, PDADMM_EBACKTRACK, "bt_max_trials exceeded");
  return PDADMM_OK;
}

// Which index plane of layer i (0-based, >= 1, -Q) holds p_l. Synchronises.
pdadmm_status current_plane(pdadmm_ctx* c, int i, int* cur) {
  HIP_TRY(c, hipMemcpyAsync(c->h_flags, reinterpret_cast<const char*>(c->scal + i) + offsetof(LayerScal, cur), sizeof(int),
                            hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  *cur = c->h_flags[0] & 1;
  return PDADMM_OK;
}

struct VarRef {
  void* ptr;
  int rows, cols, ld;
  size_t elem;
};

pdadmm_status locate(pdadmm_ctx* c, int kind, int layer, bool writing, VarRef* v) {
  const int L = c->L;
  if (layer < 1 || layer > L) return fail(c, PDADMM_EINVAL, "layer out of range");
  LayerBufs& b = c->lay[layer - 1];
  v->elem = sizeof(float);
  switch (kind) {
    case PDADMM_VAR_P:
      if (writing && layer == 1) return fail(c, PDADMM_EINVAL, "p_1 = X is fixed");
      // -Q, l >= 2: p_l exists as indices only; values pass through the trial-direction buffer of the layer
      *v = {b.p ? b.p : b.d, c->N, b.n_in, b.ld_in, sizeof(float)};
      return PDADMM_OK;
    case PDADMM_VAR_W: *v = {b.W, b.n_out, b.n_in, b.ld_in, sizeof(float)}; return PDADMM_OK;
    case PDADMM_VAR_B: *v = {b.b, 1, b.n_out, b.ld_out, sizeof(float)}; return PDADMM_OK;
    case PDADMM_VAR_Z: *v = {b.z, c->N, b.n_out, b.ld_out, sizeof(float)}; return PDADMM_OK;
    case PDADMM_VAR_Q:
    case PDADMM_VAR_U:
      if (layer == L) return fail(c, PDADMM_EINVAL, "q_l, u_l exist for l < L only");
      *v = {kind == PDADMM_VAR_Q ? b.q : b.u, c->N, b.n_out, b.ld_out, sizeof(float)};
      return PDADMM_OK;
    case PDADMM_VAR_PIDX:
      if (writing || !c->cfg.quantize || layer < 2) return fail(c, PDADMM_EINVAL, "PIDX: get only, -Q, l >= 2");
      *v = {b.pidx, c->N, b.n_in, b.ld_in, (size_t)c->grid.ib};      // plane 0; the caller adds the current plane
      return PDADMM_OK;
    case PDADMM_VAR_RESID:
      if (writing) return fail(c, PDADMM_EINVAL, "read-only variable");
      *v = {b.R, c->N, b.n_out, b.ld_out, sizeof(float)};
      return PDADMM_OK;
    case PDADMM_VAR_GRAD_P:
      if (writing || layer < 2) return fail(c, PDADMM_EINVAL, "GRAD_P: get only, l >= 2");
      *v = {b.g, c->N, b.n_in, b.ld_in, sizeof(float)};
      return PDADMM_OK;
    case PDADMM_VAR_GRAD_W:
      if (writing) return fail(c, PDADMM_EINVAL, "read-only variable");
      *v = {b.G, b.n_out, b.n_in, b.ld_in, sizeof(float)};
      return PDADMM_OK;
    default: return fail(c, PDADMM_EINVAL, "unknown variable kind");
  }
}

}  // namespace

// ==========================================================================================
// C ABI
// ==========================================================================================
extern "C" {

pdadmm_status pdadmm_normalize_adj(int32_t n, const int32_t* rowptr, const int32_t* colidx, int32_t* out_rowptr,
                                   int32_t* out_colidx, float* out_vals) {
  if (n < 0 || !rowptr || !out_rowptr || (!colidx && n > 0 && rowptr[n] > 0) || !out_colidx || !out_vals)
    return PDADMM_EINVAL;
  if (rowptr[0] != 0) return PDADMM_EINVAL;
  for (int i = 0; i < n; ++i) {
    if (rowptr[i + 1] < rowptr[i]) return PDADMM_EINVAL;
    for (int e = rowptr[i]; e < rowptr[i + 1]; ++e) {
      const int j = colidx[e];
      if (j < 0 || j >= n || j == i) return PDADMM_EINVAL;
      if (e > rowptr[i] && colidx[e - 1] >= j) return PDADMM_EINVAL;
    }
  }
  int64_t o = 0;
  out_rowptr[0] = 0;
  for (int i = 0; i < n; ++i) {
    const int64_t di = (int64_t)(rowptr[i + 1] - rowptr[i]) + 1;
    bool self_done = false;
    auto emit = [&](int j) {
      const int64_t dj = (int64_t)(rowptr[j + 1] - rowptr[j]) + 1;
      out_colidx[o] = j;
      out_vals[o] = (float)(1.0 / std::sqrt((double)(di * dj)));
      ++o;
    };
    for (int e = rowptr[i]; e < rowptr[i + 1]; ++e) {
      const int j = colidx[e];
      if (!self_done && j > i) {
        emit(i);
        self_done = true;
      }
      emit(j);
    }
    if (!self_done) emit(i);
    if (o > INT32_MAX) return PDADMM_EINVAL;
    out_rowptr[i + 1] = (int32_t)o;
  }
  return PDADMM_OK;
}

pdadmm_status pdadmm_augment(int32_t n, int64_t nnz, const int32_t* rowptr, const int32_t* colidx, const float* vals,
                             const float* X, int32_t d, int32_t hops, float* X_aug, void* stream) {
  if (n < 0 || nnz < 0 || d < 1 || hops < 0) return PDADMM_EINVAL;
  if (n == 0) return PDADMM_OK;
  if (!rowptr || !X || !X_aug || (nnz > 0 && (!colidx || !vals))) return PDADMM_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int ld = (hops + 1) * d;
  if (hipMemcpy2DAsync(X_aug, (size_t)ld * 4, X, (size_t)d * 4, (size_t)d * 4, n, hipMemcpyDeviceToDevice, st) !=
      hipSuccess)
    return PDADMM_EHIP;
  const bool vec = (d % 4 == 0) && aligned16(X_aug);
  for (int k = 1; k <= hops; ++k) {
    const float* src = X_aug + (size_t)(k - 1) * d;
    float* dst = X_aug + (size_t)k * d;
    if (vec) {
      const size_t items = (size_t)n * (d / 4);
      hipLaunchKernelGGL((spmm_hop_kernel<4>), dim3((unsigned)((items + 255) / 256)), dim3(256), 0, st, n, rowptr,
                         colidx, vals, src, dst, d, ld);
    } else {
      const size_t items = (size_t)n * d;
      hipLaunchKernelGGL((spmm_hop_kernel<1>), dim3((unsigned)((items + 255) / 256)), dim3(256), 0, st, n, rowptr,
                         colidx, vals, src, dst, d, ld);
    }
    if (hipGetLastError() != hipSuccess) return PDADMM_EHIP;
  }
  return PDADMM_OK;
}

pdadmm_status pdadmm_quantize(const float* v, int64_t count, float lo, float hi, int32_t levels, void* idx_out,
                              float* val, void* stream) {
  if (count < 0 || levels < 2 || levels > 65536 || !(hi > lo)) return PDADMM_EINVAL;
  if (count == 0) return PDADMM_OK;
  uint8_t* idx = static_cast<uint8_t*>(idx_out);
  if (!v || (!idx && !val)) return PDADMM_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const QuantGrid g = make_grid(lo, hi, levels);
  const bool vec = count % 4 == 0 && aligned16(v) && (!val || aligned16(val)) &&
                   (!idx || (reinterpret_cast<uintptr_t>(idx) & 7) == 0);
  if (vec) {
    const size_t n4 = (size_t)count / 4;
    // ld = a multiple of 4 large enough that no column is masked
    hipLaunchKernelGGL(quantize_kernel, dim3(flat_blocks(n4)), dim3(256), 0, st, v, n4, 4, 4, g, idx, val);
  } else {
    hipLaunchKernelGGL(quantize_scalar_kernel, dim3(flat_blocks(((size_t)count + 3) / 4)), dim3(256), 0, st, v,
                       (size_t)count, g, idx, val);
  }
  return hipGetLastError() == hipSuccess ? PDADMM_OK : PDADMM_EHIP;
}

}  // extern "C"


extern "C" {

pdadmm_status pdadmm_gemm_nt(int32_t M, int32_t N, int32_t K, const float* A, int32_t lda, const float* B,
                             int32_t ldb, float* C, int32_t ldc, void* stream) {
  if (M < 1 || N < 1 || K < 1 || !A || !B || !C || lda < K || ldb < K || ldc < N) return PDADMM_EINVAL;
  GemmProb P = make_nt(A, lda, B, ldb, C, ldc, M, N, K);
  const int panel = std::max(1, std::min(8, P.tiles_n));
  hipLaunchKernelGGL((gemm_one_kernel<Tile, true, EpiStore>), dim3(xcd_padded(P.nblk, panel)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), P, panel);
  return hipGetLastError() == hipSuccess ? PDADMM_OK : PDADMM_EHIP;
}

pdadmm_status pdadmm_gemm_tn(int32_t M, int32_t N, int32_t K, float alpha, const float* A, int32_t lda,
                             const float* B, int32_t ldb, float* C, int32_t ldc, int32_t splitk, float* part,
                             void* stream) {
  if (M < 1 || N < 1 || K < 1 || !A || !B || !C || !part || lda < M || ldb < N || ldc < N || splitk < 1 ||
      splitk > K)
    return PDADMM_EINVAL;
  const int chunk = cdiv(cdiv(K, splitk), BK) * BK;
  const int sk = cdiv(K, chunk);
  GemmProb P = make_tn(A, lda, B, ldb, part, ldc, M, N, K, sk, chunk);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int panel = std::max(1, std::min(8, P.tiles_n));
  hipLaunchKernelGGL((gemm_one_kernel<Tile, false, EpiStore>), dim3(xcd_padded(P.nblk, panel)), dim3(256), 0, st, P,
                     panel);
  if (hipGetLastError() != hipSuccess) return PDADMM_EHIP;
  ReduceProb R{};
  R.part = part; R.G = C; R.norm_part = nullptr; R.M = M; R.N = N; R.ld = ldc; R.splitk = sk; R.alpha = alpha;
  R.vec = ldc % 4 == 0 && ((reinterpret_cast<uintptr_t>(part) | reinterpret_cast<uintptr_t>(C)) & 15) == 0;
  R.nblk = (int)std::min<size_t>(2048, std::max<size_t>(1, ((size_t)M * ldc + 1023) / 1024));
  hipLaunchKernelGGL(splitk_reduce_one_kernel, dim3(R.nblk), dim3(256), 0, st, R);
  return hipGetLastError() == hipSuccess ? PDADMM_OK : PDADMM_EHIP;
}

pdadmm_status pdadmm_gemm_tn_static(int32_t M, int32_t N, int32_t K, float alpha, const float* A, int32_t lda,
                                    const float* B, int32_t ldb, float* C, int32_t ldc, int32_t splitk,
                                    void* stream) {
  if (M < 1 || N < 1 || K < 1 || !A || !B || !C || lda < M || ldb < N || ldc < N || splitk < 1 || splitk > K)
    return fail(nullptr, PDADMM_EINVAL, "pdadmm_gemm_tn_static: bad size, leading dimension or NULL pointer");
  const int chunk = cdiv(cdiv(K, splitk), BK) * BK;   // the chunking of pdadmm_gemm_tn
  const int sk = cdiv(K, chunk);
  const size_t need = (size_t)sk * (size_t)M * (size_t)ldc;
  if (need > (size_t)PDADMM_STATIC_SCRATCH_FLOATS)
    return fail(nullptr, PDADMM_EINVAL, "pdadmm_gemm_tn_static: " + std::to_string(sk) + " chunks x M x ldc = " +
                                            std::to_string(need) + " floats exceed the built-in scratch of " +
                                            std::to_string((size_t)PDADMM_STATIC_SCRATCH_FLOATS));
  float* part = nullptr;
  const pdadmm_status s = scratch_of_current_device(&part);
  if (s != PDADMM_OK) return s;
  // every element of part that the reduction adds up is written by the product kernel of this call first
  // (rows < M, columns < N of every chunk; what it reads beyond column N is masked before it is used)
  return pdadmm_gemm_tn(M, N, K, alpha, A, lda, B, ldb, C, ldc, splitk, part, stream);
}

size_t pdadmm_workspace_bytes(const pdadmm_config* cfg) {
  std::string why;
  if (!config_ok(cfg, &why)) {
    fail(nullptr, PDADMM_EINVAL, "config: " + why);
    return 0;
  }
  pdadmm_ctx tmp;
  tmp.cfg = *cfg;
  tmp.N = cfg->n_nodes;
  tmp.L = cfg->n_layers;
  tmp.dims.assign(cfg->dims, cfg->dims + cfg->n_layers + 1);
  return plan(&tmp, nullptr);
}

}  // extern "C"

namespace {

// Common part of pdadmm_init and pdadmm_grow_layers. Layer i takes W, b from layer from_layer[i] (1-based)
// of the context `from` where that entry is positive, else from the dense caller arrays W0[i], b0[i].
pdadmm_status init_common(pdadmm_ctx** out, const pdadmm_config* cfg, void* workspace, size_t workspace_bytes,
                          const float* X_aug, const int32_t* labels, const uint8_t* train_mask,
                          const float* const* W0, const float* const* b0, void* const* streams, int32_t n_streams,
                          pdadmm_ctx* from, const int32_t* from_layer) {
  if (!out) return fail(nullptr, PDADMM_EINVAL, "out is NULL");
  *out = nullptr;
  std::string why;
  if (!config_ok(cfg, &why)) return fail(nullptr, PDADMM_EINVAL, "config: " + why);
  if (!workspace || !X_aug || !labels) return fail(nullptr, PDADMM_EINVAL, "workspace, X_aug or labels is NULL");
  if (reinterpret_cast<uintptr_t>(workspace) & 255) return fail(nullptr, PDADMM_EINVAL, "workspace is not 256-byte aligned");
  if (from && !from_layer) return fail(nullptr, PDADMM_EINVAL, "from_layer is NULL");
  if (n_streams < 0 || n_streams > 2 || (n_streams > 0 && !streams))
    return fail(nullptr, PDADMM_EINVAL, "n_streams must be 0, 1 or 2 (with a streams array)");
  if (n_streams == 2 && (!streams[1] || streams[1] == streams[0]))
    return fail(nullptr, PDADMM_EINVAL, "the second stream must be a stream of its own (not NULL, not the first)");
  for (int i = 0; i < cfg->n_layers; ++i) {
    const int src = from ? from_layer[i] : 0;
    const std::string lay = "layer " + std::to_string(i + 1) + ": ";
    if (src == 0) {
      if (!W0 || !b0 || !W0[i] || !b0[i]) return fail(nullptr, PDADMM_EINVAL, lay + "no starting W, b given");
    } else {
      if (src < 0 || src > from->L) return fail(nullptr, PDADMM_EINVAL, lay + "source layer out of range");
      if (from->dims[src - 1] != cfg->dims[i] || from->dims[src] != cfg->dims[i + 1])
        return fail(nullptr, PDADMM_EINVAL, lay + "source layer has another shape");
    }
  }
  if (from) {   // its pending work writes the arrays copied below
    if (from->N != cfg->n_nodes) return fail(nullptr, PDADMM_EINVAL, "source context has another n_nodes");
    if (hipStreamSynchronize(from->stream) != hipSuccess) return fail(nullptr, PDADMM_EHIP, "synchronising the source context failed");
  }
  pdadmm_ctx* c = new pdadmm_ctx;
  c->cfg = *cfg;
  c->N = cfg->n_nodes;
  c->L = cfg->n_layers;
  c->dims.assign(cfg->dims, cfg->dims + cfg->n_layers + 1);
  c->cfg.dims = c->dims.data();
  c->p_products.assign(cfg->n_layers, 0);
  c->stream = n_streams >= 1 ? static_cast<hipStream_t>(streams[0]) : nullptr;
  c->aux = n_streams == 2 ? static_cast<hipStream_t>(streams[1]) : nullptr;
  if (cfg->quantize) c->grid = make_grid(cfg->q_lo, cfg->q_hi, cfg->q_levels);
  const size_t need = plan(c, nullptr);
  if (workspace_bytes < need) {
    delete c;
    return fail(nullptr, PDADMM_ENOMEM, "workspace holds " + std::to_string(workspace_bytes) + " bytes, " +
                                            std::to_string(need) + " are needed");
  }
  plan(c, workspace);
  *out = c;   // from here on errors are reported through the context; the caller destroys it
  const int N = c->N, L = c->L;
  HIP_TRY(c, hipHostMalloc(reinterpret_cast<void**>(&c->h_flags), sizeof(int) * std::max(L, 4), hipHostMallocDefault));
  HIP_TRY(c, hipMemsetAsync(workspace, 0, need, c->stream));
  HIP_TRY(c, hipMemcpyAsync(c->labels, labels, sizeof(int) * N, hipMemcpyDeviceToDevice, c->stream));
  if (train_mask) HIP_TRY(c, hipMemcpyAsync(c->mask, train_mask, N, hipMemcpyDeviceToDevice, c->stream));
  else c->mask = nullptr;
  {
    const LayerBufs& b = c->lay[0];
    HIP_TRY(c, hipMemcpy2DAsync(b.p, (size_t)b.ld_in * 4, X_aug, (size_t)b.n_in * 4, (size_t)b.n_in * 4, N,
                                hipMemcpyDeviceToDevice, c->stream));
  }
  std::vector<LayerScal> hs(L);
  for (int i = 0; i < L; ++i) {
    const LayerBufs& b = c->lay[i];
    const int src = from ? from_layer[i] : 0;
    const float* Wsrc = src ? from->lay[src - 1].W : W0[i];
    const float* bsrc = src ? from->lay[src - 1].b : b0[i];
    const size_t pitch = src ? (size_t)from->lay[src - 1].ld_in * 4 : (size_t)b.n_in * 4;
    HIP_TRY(c, hipMemcpy2DAsync(b.W, (size_t)b.ld_in * 4, Wsrc, pitch, (size_t)b.n_in * 4, b.n_out,
                                hipMemcpyDeviceToDevice, c->stream));
    HIP_TRY(c, hipMemcpyAsync(b.b, bsrc, sizeof(float) * b.n_out, hipMemcpyDeviceToDevice, c->stream));
    std::memset(&hs[i], 0, sizeof(LayerScal));
    hs[i].tau = cfg->tau0;
    hs[i].theta = cfg->theta0;
  }
  HIP_TRY(c, hipMemcpyAsync(c->scal, hs.data(), sizeof(LayerScal) * L, hipMemcpyHostToDevice, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  pdadmm_status s = build_tables(c);
  if (s != PDADMM_OK) return s;
  // forward-consistent start, layer after layer
  // (-Q: the epilogue of layer l writes p_{l+1} as indices, which the product of layer l+1 then reads)
  for (int i = 0; i < L; ++i) {
    const GemmProb& F = c->fwd[i];
    if (F.p8 && c->grid.ib == 2)
      hipLaunchKernelGGL((gemm_one_kernel<Tile, true, EpiForward, 2>), dim3(xcd_padded(F.nblk, c->panel)), dim3(256),
                         0, c->stream, F, c->panel);
    else if (F.p8)
      hipLaunchKernelGGL((gemm_one_kernel<Tile, true, EpiForward, 1>), dim3(xcd_padded(F.nblk, c->panel)), dim3(256),
                         0, c->stream, F, c->panel);
    else
      hipLaunchKernelGGL((gemm_one_kernel<Tile, true, EpiForward, 0>), dim3(xcd_padded(F.nblk, c->panel)), dim3(256),
                         0, c->stream, F, c->panel);
    LAUNCH_CHECK(c, "gemm forward");
  }
  c->dirty = true;
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  if (cfg->use_graph && !cfg->quantize) {
    HIP_TRY(c, hipStreamCreateWithFlags(&c->gstream, hipStreamNonBlocking));
    HIP_TRY(c, hipEventCreateWithFlags(&c->ev_in, hipEventDisableTiming));
    HIP_TRY(c, hipEventCreateWithFlags(&c->ev_out, hipEventDisableTiming));
  }
  if (c->aux) {
    for (int k = 0; k < 2; ++k) {
      HIP_TRY(c, hipEventCreateWithFlags(&c->ev_fork[k], hipEventDisableTiming));
      HIP_TRY(c, hipEventCreateWithFlags(&c->ev_join[k], hipEventDisableTiming));
    }
    if (c->gstream) {     // the captured iteration forks into a side stream of its own
      HIP_TRY(c, hipStreamCreateWithFlags(&c->gaux, hipStreamNonBlocking));
      for (int k = 0; k < 2; ++k) {
        HIP_TRY(c, hipEventCreateWithFlags(&c->ev_gfork[k], hipEventDisableTiming));
        HIP_TRY(c, hipEventCreateWithFlags(&c->ev_gjoin[k], hipEventDisableTiming));
      }
    }
  }
  return PDADMM_OK;
}

}  // namespace

extern "C" {

pdadmm_status pdadmm_init(pdadmm_ctx** out, const pdadmm_config* cfg, void* workspace, size_t workspace_bytes,
                          const float* X_aug, const int32_t* labels, const uint8_t* train_mask,
                          const float* const* W0, const float* const* b0, void* const* streams, int32_t n_streams) {
  if (!W0 || !b0) return fail(nullptr, PDADMM_EINVAL, "W0 or b0 is NULL");
  return init_common(out, cfg, workspace, workspace_bytes, X_aug, labels, train_mask, W0, b0, streams, n_streams, nullptr,
                     nullptr);
}

pdadmm_status pdadmm_grow_layers(pdadmm_ctx** out, const pdadmm_config* cfg, void* workspace, size_t workspace_bytes,
                                 const float* X_aug, const int32_t* labels, const uint8_t* train_mask,
                                 pdadmm_ctx* from, const int32_t* from_layer, const float* const* W0,
                                 const float* const* b0, void* const* streams, int32_t n_streams) {
  if (!from || !from_layer) return fail(nullptr, PDADMM_EINVAL, "from or from_layer is NULL");
  return init_common(out, cfg, workspace, workspace_bytes, X_aug, labels, train_mask, W0, b0, streams, n_streams, from,
                     from_layer);
}

pdadmm_status pdadmm_set_var(pdadmm_ctx* c, int32_t kind, int32_t layer, const void* src) {
  if (!c || !src) return PDADMM_EINVAL;
  if (kind == PDADMM_VAR_PROBE) {
    if (layer < 2 || layer > c->L) return fail(c, PDADMM_EINVAL, "layer out of range");
    const int32_t* v = static_cast<const int32_t*>(src);
    if (v[0] < 0 || v[1] < 0 || v[0] > kProbeCap || v[1] > kProbeCap) return fail(c, PDADMM_EINVAL, "probe state out of range");
    LayerScal* dst = c->scal + (layer - 1);
    HIP_TRY(c, hipMemcpyAsync(reinterpret_cast<char*>(dst) + offsetof(LayerScal, probe_wait), v, 2 * sizeof(int32_t),
                              hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return PDADMM_OK;
  }
  if (kind == PDADMM_VAR_TAU || kind == PDADMM_VAR_THETA) {
    if (layer < (kind == PDADMM_VAR_TAU ? 2 : 1) || layer > c->L) return fail(c, PDADMM_EINVAL, "layer out of range");
    const double v = *static_cast<const double*>(src);
    if (!(v > 0.0)) return fail(c, PDADMM_EINVAL, "tau/theta must be > 0");
    LayerScal* dst = c->scal + (layer - 1);
    const size_t off = kind == PDADMM_VAR_TAU ? offsetof(LayerScal, tau) : offsetof(LayerScal, theta);
    HIP_TRY(c, hipMemcpyAsync(reinterpret_cast<char*>(dst) + off, &v, sizeof(double), hipMemcpyHostToDevice,
                              c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return PDADMM_OK;
  }
  VarRef v;
  pdadmm_status s = locate(c, kind, layer, true, &v);
  if (s != PDADMM_OK) return s;
  if (v.ld == v.cols)     // rows are dense on both sides: one plain copy (much faster from pageable host memory)
    HIP_TRY(c, hipMemcpyAsync(v.ptr, src, (size_t)v.rows * v.cols * v.elem, hipMemcpyDefault, c->stream));
  else
    HIP_TRY(c, hipMemcpy2DAsync(v.ptr, (size_t)v.ld * v.elem, src, (size_t)v.cols * v.elem, (size_t)v.cols * v.elem,
                                v.rows, hipMemcpyDefault, c->stream));
  if (kind == PDADMM_VAR_Q && c->cfg.quantize == 2) {
    const LayerBufs& b = c->lay[layer - 1];
    const size_t n4 = (size_t)c->N * b.ld_out / 4;
    hipLaunchKernelGGL(quantize_kernel, dim3(flat_blocks(n4)), dim3(256), 0, c->stream, b.q, n4, b.n_out, b.ld_out,
                       c->grid, (uint8_t*)nullptr, b.q);
    LAUNCH_CHECK(c, "quantize set_var q");
  }
  if (kind == PDADMM_VAR_P && c->cfg.quantize) {     // the values sit in the layer's d buffer: keep their indices
    const LayerBufs& b = c->lay[layer - 1];
    const size_t n4 = (size_t)c->N * b.ld_in / 4;
    int cur = 0;
    if ((s = current_plane(c, layer - 1, &cur)) != PDADMM_OK) return s;
    hipLaunchKernelGGL(quantize_kernel, dim3(flat_blocks(n4)), dim3(256), 0, c->stream, (const float*)b.d, n4, b.n_in,
                       b.ld_in, c->grid, b.pidx + (size_t)cur * b.idx_plane, (float*)nullptr);
    LAUNCH_CHECK(c, "quantize set_var");
  }
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  c->dirty = true;
  return PDADMM_OK;
}

pdadmm_status pdadmm_get_var(pdadmm_ctx* c, int32_t kind, int32_t layer, void* dst) {
  if (!c || !dst) return PDADMM_EINVAL;
  if (kind == PDADMM_VAR_PROBE) {
    if (layer < 2 || layer > c->L) return fail(c, PDADMM_EINVAL, "layer out of range");
    const LayerScal* src = c->scal + (layer - 1);
    HIP_TRY(c, hipMemcpyAsync(dst, reinterpret_cast<const char*>(src) + offsetof(LayerScal, probe_wait),
                              2 * sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return PDADMM_OK;
  }
  if (kind == PDADMM_VAR_TAU || kind == PDADMM_VAR_THETA) {
    if (layer < (kind == PDADMM_VAR_TAU ? 2 : 1) || layer > c->L) return fail(c, PDADMM_EINVAL, "layer out of range");
    const LayerScal* src = c->scal + (layer - 1);
    const size_t off = kind == PDADMM_VAR_TAU ? offsetof(LayerScal, tau) : offsetof(LayerScal, theta);
    HIP_TRY(c, hipMemcpyAsync(dst, reinterpret_cast<const char*>(src) + off, sizeof(double), hipMemcpyDeviceToHost,
                              c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return PDADMM_OK;
  }
  VarRef v;
  pdadmm_status s = locate(c, kind, layer, false, &v);
  if (s != PDADMM_OK) return s;
  if (kind == PDADMM_VAR_RESID && c->dirty) {
    if ((s = refresh_residual(c)) != PDADMM_OK) return s;
  }
  if ((kind == PDADMM_VAR_P || kind == PDADMM_VAR_PIDX) && c->cfg.quantize && layer >= 2) {
    const LayerBufs& b = c->lay[layer - 1];
    int cur = 0;
    if ((s = current_plane(c, layer - 1, &cur)) != PDADMM_OK) return s;
    const uint8_t* plane = b.pidx + (size_t)cur * b.idx_plane;
    if (kind == PDADMM_VAR_PIDX) {
      v.ptr = const_cast<uint8_t*>(plane);
    } else {                                        // values into the layer's d buffer (scratch between iterations)
      const size_t n4 = (size_t)c->N * b.ld_in / 4;
      hipLaunchKernelGGL(dequantize_kernel, dim3(flat_blocks(n4)), dim3(256), 0, c->stream, plane, n4, b.n_in, b.ld_in,
                         c->grid, b.d);
      LAUNCH_CHECK(c, "dequantize get_var");
    }
  }
  if (v.ld == v.cols)
    HIP_TRY(c, hipMemcpyAsync(dst, v.ptr, (size_t)v.rows * v.cols * v.elem, hipMemcpyDefault, c->stream));
  else
    HIP_TRY(c, hipMemcpy2DAsync(dst, (size_t)v.cols * v.elem, v.ptr, (size_t)v.ld * v.elem, (size_t)v.cols * v.elem,
                                v.rows, hipMemcpyDefault, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return PDADMM_OK;
}

pdadmm_status pdadmm_step_phase(pdadmm_ctx* c, int32_t phase) {
  if (!c) return PDADMM_EINVAL;
  pdadmm_status s;
  if (c->dirty && (s = refresh_residual(c)) != PDADMM_OK) return s;
  switch (phase) {
    case PDADMM_PHASE_P: return phase_p(c);
    case PDADMM_PHASE_W: return phase_w(c, kAll);
    case PDADMM_PHASE_BZQU: return phase_bzqu(c);
    default: return fail(c, PDADMM_EINVAL, "unknown phase");
  }
}

// One pdADMM-G iteration is a fixed sequence of kernel launches with no host decision in between
// (tau and theta are chosen on the device), so it can be captured once and replayed. The graph runs on
// a stream of its own that is ordered after and before the caller's stream by events. Not used for -Q
// (the host reads the search flags), while launches are being timed, or when a refresh is due.
static pdadmm_status iterate_graph(pdadmm_ctx* c, int32_t n_iters) {
  pdadmm_status s;
  if (c->dirty && (s = refresh_residual(c)) != PDADMM_OK) return s;
  HIP_TRY(c, hipEventRecord(c->ev_in, c->stream));
  HIP_TRY(c, hipStreamWaitEvent(c->gstream, c->ev_in, 0));
  if (!c->graph_exec) {
    hipStream_t user = c->stream;
    HIP_TRY(c, hipStreamBeginCapture(c->gstream, hipStreamCaptureModeThreadLocal));
    c->stream = c->gstream;
    s = one_iteration(c);
    c->stream = user;
    const hipError_t e = hipStreamEndCapture(c->gstream, &c->graph);
    if (s != PDADMM_OK || e != hipSuccess) {     // a phase failed while recording: drop what was captured
      if (c->graph) (void)hipGraphDestroy(c->graph);
      c->graph = nullptr;
      if (s != PDADMM_OK) return s;
      return fail(c, PDADMM_EHIP, std::string("hipStreamEndCapture: ") + hipGetErrorString(e));
    }
    HIP_TRY(c, hipGraphInstantiate(&c->graph_exec, c->graph, nullptr, nullptr, 0));
    // capture recorded the launches without running them: the product counters were advanced once
    for (int i = 1; i < c->L; ++i) --c->p_products[i];
  }
  for (int it = 0; it < n_iters; ++it) {
    HIP_TRY(c, hipGraphLaunch(c->graph_exec, c->gstream));
    for (int i = 1; i < c->L; ++i) ++c->p_products[i];
    ++c->iter;
  }
  HIP_TRY(c, hipEventRecord(c->ev_out, c->gstream));
  HIP_TRY(c, hipStreamWaitEvent(c->stream, c->ev_out, 0));
  return PDADMM_OK;
}

pdadmm_status pdadmm_iterate(pdadmm_ctx* c, int32_t n_iters) {
  if (!c || n_iters < 0) return PDADMM_EINVAL;
  pdadmm_status s;
  if (c->gstream && n_iters > 0 && c->timing_mask == 0 && c->cfg.refresh_every == 0) return iterate_graph(c, n_iters);
  for (int it = 0; it < n_iters; ++it) {
    const bool periodic = c->cfg.refresh_every > 0 && c->iter > 0 && c->iter % c->cfg.refresh_every == 0;
    if ((c->dirty || periodic) && (s = refresh_residual(c)) != PDADMM_OK) return s;
    if ((s = one_iteration(c)) != PDADMM_OK) return s;
    ++c->iter;
  }
  return PDADMM_OK;
}

pdadmm_status pdadmm_sync(pdadmm_ctx* c) {
  if (!c) return PDADMM_EINVAL;
  return check_device_flags(c);
}

static pdadmm_status sum_partials(pdadmm_ctx* c, const double* dev, size_t count, std::vector<double>* host) {
  host->resize(count);
  if (count == 0) return PDADMM_OK;
  HIP_TRY(c, hipMemcpyAsync(host->data(), dev, count * sizeof(double), hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return PDADMM_OK;
}

static pdadmm_status pair_sums(pdadmm_ctx* c, std::vector<double>* act, std::vector<double>* dl,
                               std::vector<double>* dq) {
  const int L = c->L;
  act->assign(L, 0.0);
  dl->assign(L, 0.0);
  dq->assign(L, 0.0);
  if (L < 2) return PDADMM_OK;
  launch_group(c, c->g_pair, pair_reduce_kernel, (const LayerScal*)c->scal, c->cfg.leaky_slope,
               c->cfg.quantize ? c->grid : QuantGrid{0.f, 0.f, 0, 1});
  LAUNCH_CHECK(c, "pair reduce");
  std::vector<double> h;
  for (int i = 0; i < L - 1; ++i) {
    const LayerBufs& b = c->lay[i];
    const int nblk = flat_blocks((size_t)c->N * b.ld_out / 4);
    pdadmm_status s = sum_partials(c, b.pairpart, (size_t)nblk * 3, &h);
    if (s != PDADMM_OK) return s;
    for (int k = 0; k < nblk; ++k) {
      (*act)[i] += h[3 * k];
      (*dl)[i] += h[3 * k + 1];
      (*dq)[i] += h[3 * k + 2];
    }
  }
  return PDADMM_OK;
}

// fresh residuals into the T buffers; returns sum ||r||^2 and sum ||r - carried||^2
static pdadmm_status fresh_residual_sums(pdadmm_ctx* c, double* lin, double* drift) {
  pdadmm_status s;
  if (c->dirty && (s = refresh_residual(c)) != PDADMM_OK) return s;
  launch_gemm_all<true, EpiResid, false>(c, c->g_resid_obj, c->g_resid_obj_q);
  LAUNCH_CHECK(c, "gemm resid objective");
  *lin = 0.0;
  *drift = 0.0;
  std::vector<double> h;
  for (int i = 0; i < c->L; ++i) {
    const LayerBufs& b = c->lay[i];
    if ((s = sum_partials(c, b.part_b, (size_t)b.tiles_out * 2, &h)) != PDADMM_OK) return s;
    for (int k = 0; k < b.tiles_out; ++k) {
      *lin += h[2 * k];
      *drift += h[2 * k + 1];
    }
  }
  return PDADMM_OK;
}

pdadmm_status pdadmm_objective(pdadmm_ctx* c, pdadmm_objective_terms* out) {
  if (!c || !out) return PDADMM_EINVAL;
  pdadmm_status s;
  double lin = 0, drift = 0;
  if ((s = fresh_residual_sums(c, &lin, &drift)) != PDADMM_OK) return s;
  std::vector<double> act, dl, dq, h;
  if ((s = pair_sums(c, &act, &dl, &dq)) != PDADMM_OK) return s;
  const LayerBufs& bl = c->lay[c->L - 1];
  hipLaunchKernelGGL(risk_kernel, dim3(c->risk_blocks), dim3(256), 0, c->stream, bl.z, c->labels, c->mask, c->N,
                     bl.n_out, bl.ld_out, c->cfg.risk_kind, c->riskpart);
  LAUNCH_CHECK(c, "risk");
  if ((s = sum_partials(c, c->riskpart, c->risk_blocks, &h)) != PDADMM_OK) return s;
  double risk = 0;
  for (double v : h) risk += v;
  double sa = 0, sl = 0, sq = 0;
  for (int i = 0; i < c->L; ++i) { sa += act[i]; sl += dl[i]; sq += dq[i]; }
  out->risk = risk;
  out->lin_pen = 0.5 * c->cfg.nu * lin;
  out->act_pen = 0.5 * c->cfg.nu * sa;
  out->dual_lin = sl;
  out->dual_quad = 0.5 * c->cfg.rho * sq;
  out->F = out->risk + out->lin_pen + out->act_pen;
  out->L_rho = out->F + out->dual_lin + out->dual_quad;
  return check_device_flags(c);
}

pdadmm_status pdadmm_residual(pdadmm_ctx* c, double* total, double* per_layer) {
  if (!c || !total) return PDADMM_EINVAL;
  std::vector<double> act, dl, dq;
  pdadmm_status s = pair_sums(c, &act, &dl, &dq);
  if (s != PDADMM_OK) return s;
  double t = 0;
  for (int i = 0; i < c->L - 1; ++i) {
    t += dq[i];
    if (per_layer) per_layer[i] = std::sqrt(dq[i]);
  }
  *total = std::sqrt(t);
  return check_device_flags(c);
}

pdadmm_status pdadmm_stats(pdadmm_ctx* c, double* tau, double* theta, int32_t* p_trials, int32_t* w_trials,
                           double* r_drift, int64_t* p_products) {
  if (!c) return PDADMM_EINVAL;
  std::vector<LayerScal> hs(c->L);
  HIP_TRY(c, hipMemcpyAsync(hs.data(), c->scal, sizeof(LayerScal) * c->L, hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  for (int i = 0; i < c->L; ++i) {
    if (tau) tau[i] = hs[i].tau;
    if (theta) theta[i] = hs[i].theta;
    if (p_trials) p_trials[i] = hs[i].p_trials;
    if (w_trials) w_trials[i] = hs[i].w_trials;
    if (p_products) p_products[i] = c->cfg.quantize ? hs[i].products : c->p_products[i];
  }
  if (r_drift) {
    double lin = 0, drift = 0;
    pdadmm_status s = fresh_residual_sums(c, &lin, &drift);
    if (s != PDADMM_OK) return s;
    *r_drift = lin > 0 ? std::sqrt(drift / lin) : std::sqrt(drift);
  }
  return check_device_flags(c);
}

pdadmm_status pdadmm_plan_info(pdadmm_ctx* c, int32_t* fused_updates, int32_t* wgrad_split, int32_t* wtrial_split,
                               int32_t* p_bytes) {
  if (!c) return PDADMM_EINVAL;
  if (p_bytes) *p_bytes = c->cfg.quantize ? c->grid.ib : 4;
  if (fused_updates) *fused_updates = (c->spec_p ? 1 : 0) | (c->spec_w ? 2 : 0);
  if (wgrad_split)
    for (int i = 0; i < c->L; ++i) wgrad_split[i] = c->lay[i].splitk;
  if (wtrial_split) {
    int s = 1;
    for (int i = 0; i < c->L; ++i) s = std::max(s, c->lay[i].wt_split);
    *wtrial_split = s;
  }
  return PDADMM_OK;
}

pdadmm_status pdadmm_predict(pdadmm_ctx* c, int32_t* pred, float* logits, const uint8_t* mask, double* accuracy) {
  if (!c) return PDADMM_EINVAL;
  const int N = c->N, L = c->L;
  // forward pass through the current W_l, b_l; activations go through the per-layer product scratch
  const float* in = c->lay[0].p;
  int ld_in = c->lay[0].ld_in;
  for (int i = 0; i < L; ++i) {
    const LayerBufs& b = c->lay[i];
    GemmProb F = make_nt(in, ld_in, b.W, b.ld_in, b.T, b.ld_out, N, b.n_out, b.n_in);
    F.e0 = b.b;
    F.beta = i < L - 1 ? 1.0f : 0.0f;   // f on every layer but the output layer
    F.slope = c->cfg.leaky_slope;
    hipLaunchKernelGGL((gemm_one_kernel<Tile, true, EpiBiasAct>), dim3(xcd_padded(F.nblk, c->panel)), dim3(256), 0,
                       c->stream, F, c->panel);
    LAUNCH_CHECK(c, "gemm predict");
    in = b.T;
    ld_in = b.ld_out;
  }
  const LayerBufs& bl = c->lay[L - 1];
  hipLaunchKernelGGL(argmax_kernel, dim3(c->risk_blocks), dim3(256), 0, c->stream, (const float*)bl.T, N, bl.n_out,
                     bl.ld_out, (const int*)c->labels, mask, pred, c->predpart);
  LAUNCH_CHECK(c, "argmax");
  if (logits)
    HIP_TRY(c, hipMemcpy2DAsync(logits, (size_t)bl.n_out * 4, bl.T, (size_t)bl.ld_out * 4, (size_t)bl.n_out * 4, N,
                                hipMemcpyDeviceToDevice, c->stream));
  std::vector<double> h;
  pdadmm_status s = sum_partials(c, c->predpart, 2 * (size_t)c->risk_blocks, &h);
  if (s != PDADMM_OK) return s;
  double counted = 0, correct = 0;
  for (int k = 0; k < c->risk_blocks; ++k) {
    counted += h[2 * k];
    correct += h[2 * k + 1];
  }
  if (accuracy) *accuracy = counted > 0 ? correct / counted : 0.0;
  return PDADMM_OK;
}

pdadmm_status pdadmm_timing(pdadmm_ctx* c, uint32_t class_mask) {
  if (!c) return PDADMM_EINVAL;
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  for (auto& t : c->timed) {
    c->event_pool.push_back(t.a);
    c->event_pool.push_back(t.b);
  }
  c->timed.clear();
  c->timing_mask = class_mask;
  return PDADMM_OK;
}

pdadmm_status pdadmm_timing_read(pdadmm_ctx* c, double* ms, int64_t* launches, int32_t n_classes) {
  if (!c || !ms || !launches || n_classes < kNumClasses) return PDADMM_EINVAL;
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  for (int i = 0; i < n_classes; ++i) {
    ms[i] = 0.0;
    launches[i] = 0;
  }
  for (auto& t : c->timed) {
    float e = 0.f;
    HIP_TRY(c, hipEventElapsedTime(&e, t.a, t.b));
    ms[t.cls] += (double)e;
    launches[t.cls] += 1;
    c->event_pool.push_back(t.a);
    c->event_pool.push_back(t.b);
  }
  c->timed.clear();
  return PDADMM_OK;
}

const char* pdadmm_last_error(const pdadmm_ctx* c) { return c ? c->msg.c_str() : g_thread_error.c_str(); }

void pdadmm_destroy(pdadmm_ctx* c) {
  if (!c) return;
  (void)hipStreamSynchronize(c->stream);
  if (c->aux) (void)hipStreamSynchronize(c->aux);
  if (c->gstream) (void)hipStreamSynchronize(c->gstream);
  if (c->gaux) (void)hipStreamSynchronize(c->gaux);
  if (c->graph_exec) (void)hipGraphExecDestroy(c->graph_exec);
  if (c->graph) (void)hipGraphDestroy(c->graph);
  if (c->ev_in) (void)hipEventDestroy(c->ev_in);
  if (c->ev_out) (void)hipEventDestroy(c->ev_out);
  if (c->gstream) (void)hipStreamDestroy(c->gstream);
  if (c->gaux) (void)hipStreamDestroy(c->gaux);
  for (int k = 0; k < 2; ++k)
    for (hipEvent_t e : {c->ev_fork[k], c->ev_join[k], c->ev_gfork[k], c->ev_gjoin[k]})
      if (e) (void)hipEventDestroy(e);
  if (c->h_flags) (void)hipHostFree(c->h_flags);
  for (auto& t : c->timed) {
    (void)hipEventDestroy(t.a);
    (void)hipEventDestroy(t.b);
  }
  for (auto e : c->event_pool) (void)hipEventDestroy(e);
  delete c;
}

}  // extern "C"
