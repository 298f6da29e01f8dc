// Host side of libpbd.so: descriptor parsing, workspace planning, the per-block
// executors and the C ABI declared in include/pbd.h.
//
// One step (Algorithm 1 on one device, "internal relaying" of Sec. VII-A):
//   relay   : A_0 <- cast(x);  A_i <- T_i(A_{i-1}) once each, all kept in HBM
//   student : for each i: forward S_i on A_{i-1} with batch statistics, fused MSE
//             loss + gradient against A_i, backward through S_i (no gradient for
//             A_{i-1}), and the SGD-momentum update straight after (Sec. IV-B).
// Everything is enqueued on the caller's stream; the library owns no device memory.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <string>
#include <utility>
#include <vector>

#include "../../include/pbd.h"
#include "conv_kernels.h"
#include "conv_dma_kernels.h"
#include "ew_kernels.h"

using namespace pbd;

// Reduction scratch of pbd_student_step_static: partial sums of the loss, of the batch-norm statistics and of
// the weight gradients, and split-K partial tiles.  One copy per GPU, held until the process ends; every
// call on a GPU shares it.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

// Device address of `scratch` on each GPU (the array's name is only a host-side handle: each device holds
// its own copy at its own address).  Looked up once per device, with that device current.
constexpr int kMaxDevices = 64;
float* g_scratch_ptr[kMaxDevices] = {};
hipError_t static_scratch(float** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    g_scratch_ptr[dev] = static_cast<float*>(p);
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

enum { OP_CBA = 1, OP_POOL = 2, OP_ADD = 3, OP_MIX = 4 };
constexpr int32_t kMagic = 0x50424431;
constexpr int kRec = 20;
constexpr size_t kAlign = 256;

inline size_t align_up(size_t v, size_t a = kAlign) { return (v + a - 1) / a * a; }
inline int round8(int c) { return (c + 7) / 8 * 8; }
inline int out_dim(int h, int k, int s, int pad) { return (h + 2 * pad - k) / s + 1; }

struct Shape { int c, h, w; };
struct OpD { int type, nin, in[8], c_out, k, stride, pad, groups, act, pofs; };

struct OpPlan {
  OpD d;
  Shape in, out;
  int cin_p, cout_p;
  bool dw;
  size_t wn = 0;            // physical weight elements
  // teacher: byte offsets in the parameter region
  size_t t_w = 0, t_gamma = 0, t_beta = 0, t_rmean = 0, t_rvar = 0, t_a = 0, t_b = 0;
  // student: element offsets in the block's flat arena; byte offsets for statistics
  size_t e_w = 0, e_gamma = 0, e_beta = 0;
  size_t s_rmean = 0, s_rvar = 0, s_mean = 0, s_invstd = 0, s_k2 = 0, s_k3 = 0;
  long e_wt = -1;           // element offset in the block's transposed-weight arena
  // scratch byte offsets
  size_t y = 0, idx = 0;
  int mix_slot = -1;        // student mix op: which 32-float state record of the block it owns
  // 7 x 7 stride-2 stem on the 3-channel input, run as a 4 x 4 stride-1 convolution over the space-to-depth copy
  // of the input (s2d_input_kernel): byte offset (parameter region) of the repacked filter [K][4][4][16]
  bool s2d = false;
  size_t w2 = 0;
};

struct BlockPlan {
  std::vector<OpPlan> ops;
  std::vector<Shape> shapes;     // values, 0 = block input
  std::vector<size_t> val;       // scratch byte offset of each value (>=1)
  std::vector<size_t> dval;      // scratch byte offset of each value's gradient (student)
  size_t arena_elems = 0;        // student: w, gamma, beta of all ops, flat
  size_t master = 0, mom = 0, grad = 0, wc = 0, wt = 0, table = 0;  // byte offsets (param region)
  size_t wt_elems = 0;
  std::vector<TransposeEntry> ttable;
  size_t scratch_bytes = 0, red_bytes = 0;
  size_t scr_off = 0, red_off = 0;   // absolute workspace offsets of this block's scratch regions
  size_t mix = 0;                // byte offset (param region) of the mix ops' state records
  int nmix = 0;
  std::vector<char> alpha_defined;  // per mix op: alpha was loaded or trained (else p is the descriptor's)
  bool stepped = false;          // student: saved values in scratch belong to a finished step
  bool dirty = true;             // compute copies stale w.r.t. master weights
};

}  // namespace

struct pbd_ctx {
  pbd_opts o{};
  int B = 0;
  Shape in{};
  std::vector<double> pool;
  std::vector<BlockPlan> net[2];
  std::vector<Shape> act;               // A_0..A_B
  std::vector<size_t> act_off;          // byte offsets (relay region)
  size_t s2d_off = (size_t)-1;          // ... of the space-to-depth copy of A_0 (none: -1)
  size_t esz = 4;                       // bytes per tensor element
  // regions (byte offsets from the workspace base)
  size_t r_param = 0, r_relay = 0, r_relay2 = 0, r_tscr = 0, r_tred = 0, total = 0;
  bool concurrent = false;              // student blocks own disjoint scratch and may overlap
  std::vector<hipStream_t> side;        // one stream per student block (graph capture branches)
  std::vector<hipEvent_t> ev_fork, ev_join;
  char* ws = nullptr;
  int num_cu = 256;                     // compute units of the bound device (tile-count heuristics)
  hipStream_t stream = nullptr;
  bool bound = false, fold_dirty = true;
  int relayed_upto = 0;                 // A_0..A_relayed_upto hold the current input's activations
  std::string err;
  // profiling
  size_t lr_off = 0, loss_off = 0;      // device scalars: learning rate, per-block losses
  hipGraphExec_t gexec[2] = {nullptr, nullptr};   // the captured step: [0] weight round, [1] architecture round
  bool graph_tried[2] = {false, false};
  // pipelined steps (pbd_pipeline_step): the relay store exists twice; `front` is the copy the teacher
  // wrote last (the one the views and read-backs show), `pending` says that its batch still waits for
  // the students.  gpipe[q]: captured body with the teacher writing copy q and the students reading 1-q.
  int front = 0;
  bool pending = false;
  float pending_lr = 0.f;
  hipGraphExec_t gpipe[2] = {nullptr, nullptr};
  bool gpipe_tried[2] = {false, false};
  std::vector<int> pipe_order;                    // order in which the branches are captured: block indices, B = the teacher
  hipGraphExec_t gdrain[2] = {nullptr, nullptr};  // the students alone, reading copy q (pbd_pipeline_flush)
  bool gdrain_tried[2] = {false, false};
  bool prof_on = false;
  std::vector<hipEvent_t> ev;
  hipEvent_t pend_start = nullptr, pend_stop = nullptr;   // events waiting for the next launch
  std::vector<pbd_prof_entry> prof;
};

namespace {

thread_local std::string g_create_err;  // why the last pbd_create on this thread failed

int fail(pbd_ctx* c, int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (c) c->err = buf; else g_create_err = buf;
  return code;
}

#define HIP_TRY(c, expr)                                                                    \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess) return fail(c, PBD_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

// ---------------------------------------------------------------------------
// descriptor -> plan (host only)
// ---------------------------------------------------------------------------
bool parse_net(pbd_ctx* c, const int32_t* w, int nw, int& pos, int which, std::string& err) {
  Shape cur = c->in;
  for (int b = 0; b < c->B; ++b) {
    if (pos >= nw) { err = "descriptor truncated"; return false; }
    BlockPlan bp;
    const int nops = w[pos++];
    if (nops < 1) { err = "block without operations"; return false; }
    bp.shapes.push_back(cur);
    for (int j = 0; j < nops; ++j, pos += kRec) {
      if (pos + kRec > nw) { err = "descriptor truncated"; return false; }
      const int32_t* r = w + pos;
      OpPlan op{};
      OpD& o = op.d;
      o.type = r[0]; o.nin = r[1];
      for (int i = 0; i < 8; ++i) o.in[i] = r[2 + i];
      o.c_out = r[10]; o.k = r[11]; o.stride = r[12]; o.pad = r[13];
      o.groups = r[14]; o.act = r[15]; o.pofs = r[16];
      if (o.nin < 1 || o.nin > 8) { err = "bad input count"; return false; }
      for (int i = 0; i < o.nin; ++i)
        if (o.in[i] < 0 || o.in[i] > j) { err = "operation input refers forward"; return false; }
      if (o.act < 0 || o.act > 2) { err = "unknown activation"; return false; }
      const Shape s = bp.shapes[o.in[0]];
      Shape out = s;
      if (o.type == OP_CBA) {
        if (o.nin != 1 || o.k < 1 || o.k > 7 || o.stride < 1 || o.stride > 2 || o.pad != o.k / 2 ||
            o.c_out < 1) { err = "unsupported convolution geometry"; return false; }
        if (o.groups != 1 && o.k != 1 && o.k != 3 && o.k != 5 && o.k != 7) { err = "depthwise kernels are 1, 3, 5 or 7 wide"; return false; }
        if (o.groups != 1 && (o.groups != s.c || o.c_out != s.c)) { err = "groups must be 1 or C_in == C_out"; return false; }
        if (o.groups == 1 && o.c_out % 8) { err = "dense convolution needs C_out % 8 == 0"; return false; }
        out = {o.c_out, out_dim(s.h, o.k, o.stride, o.pad), out_dim(s.w, o.k, o.stride, o.pad)};
      } else if (o.type == OP_POOL) {
        if (o.nin != 1 || o.k < 1 || o.k > 15 || o.stride < 1 || o.pad < 0 || o.pad >= o.k) { err = "unsupported pooling geometry"; return false; }
        out = {s.c, out_dim(s.h, o.k, o.stride, o.pad), out_dim(s.w, o.k, o.stride, o.pad)};
      } else if (o.type == OP_ADD || o.type == OP_MIX) {
        if (o.type == OP_ADD && o.nin != 2) { err = "add takes two inputs"; return false; }
        if (o.type == OP_MIX && (o.pofs < 0 || o.pofs + o.nin > (int)c->pool.size())) { err = "mix weights outside the pool"; return false; }
        for (int i = 1; i < o.nin; ++i) {
          const Shape t = bp.shapes[o.in[i]];
          if (t.c != s.c || t.h != s.h || t.w != s.w) { err = "joined values differ in shape"; return false; }
        }
      } else { err = "unknown operation type"; return false; }
      if (out.h < 1 || out.w < 1) { err = "empty output"; return false; }
      op.in = s; op.out = out;
      op.cin_p = round8(s.c); op.cout_p = round8(out.c);
      op.dw = o.type == OP_CBA && o.groups != 1;
      if (o.type == OP_CBA) op.wn = op.dw ? (size_t)o.k * o.k * op.cout_p : (size_t)o.c_out * o.k * o.k * op.cin_p;
      bp.ops.push_back(op);
      bp.shapes.push_back(out);
    }
    cur = bp.shapes.back();
    c->net[which].push_back(std::move(bp));
  }
  return true;
}

size_t tensor_bytes(const pbd_ctx* c, Shape s) {
  return align_up((size_t)c->o.batch * s.h * s.w * round8(s.c) * c->esz);
}

// rows_per_thread: how many rows a thread should stream at least; max_blocks caps the grid
ColGrid col_grid(long M, int Cp, int rows_per_thread = 8, int max_blocks = 512) {
  ColGrid g;
  const int ncv = Cp / 8;
  // as few column slabs as 32 lanes allow, then lanes = vectors per slab: no idle lanes for channel
  // counts that are not powers of two (48, 96, 144, 576 ...), at most 256 % cvl idle threads per block
  g.slabs = (ncv + 31) / 32;
  g.cvl = (ncv + g.slabs - 1) / g.slabs;
  const int cvl = g.cvl;
  const int rl = 256 / cvl;
  long chunks = (M + (long)rl * rows_per_thread - 1) / ((long)rl * rows_per_thread);
  const long cap = std::max(1, max_blocks / g.slabs);
  // small tensors: rather fewer rows per thread than idle compute units
  const long want = std::min<long>((M + rl - 1) / rl, (256 + g.slabs - 1) / g.slabs);
  chunks = std::max(std::max(1L, want), std::min(chunks, cap));
  g.rows_per_chunk = (M + chunks - 1) / chunks;
  g.chunks = (int)((M + g.rows_per_chunk - 1) / g.rows_per_chunk);
  return g;
}

// Row chunks of the two BN reductions: up to 1024 workgroups per column slab keep enough loads in flight
// on tensors of 100 MB and more (statistics 2.0 -> 1.5 ms, backward sums 3.4 -> 2.9 ms per ResNet-50 step)
inline ColGrid bn_stats_grid(long M, int Cp) { return col_grid(M, Cp, 8, 1024); }
inline ColGrid bn_bwd_grid(long M, int Cp) { return col_grid(M, Cp, 8, 1024); }

// Partial results of a depthwise backward-weight: row chunks of the column-grid kernel, or blocks of
// tiles of the LDS-tiled kernel (bf16, stride 1, odd k <= 7, image at least 8 x 12).
inline bool dw_tiled(bool bf16, int k, int stride, int pad, int h_out, int w_out) {
  return bf16 && (k == 3 || k == 5 || k == 7) && pad == k / 2 && stride == 1 && h_out >= 8 && w_out >= 12;
}
struct DwWgradCfg { bool tiled; int chunks, tiles_h, tiles_w, ntiles, tiles_per_block; ColGrid g; };
inline DwWgradCfg dw_wgrad_cfg(bool bf16, int N, int h_out, int w_out, int Cp, int k, int stride, int pad) {
  DwWgradCfg w{};
  const long M = (long)N * h_out * w_out;
  // the tile kernel also wins on 8-wide images (half of each 8 x 16 tile empty: 11 us against 21 us for
  // 256 x 8 x 8 x 256), unlike the forward and backward-data tile kernels
  w.tiled = dw_tiled(bf16, k, stride, pad, h_out, std::max(w_out, w_out >= 8 ? 12 : 0));
  if (w.tiled) {
    w.tiles_h = (h_out + 7) / 8;
    w.tiles_w = (w_out + 15) / 16;
    w.ntiles = N * w.tiles_h * w.tiles_w;
    const int cvblocks = (Cp / 8 + 7) / 8;
    const int want = std::max(1, std::min(w.ntiles, 1024 / cvblocks));
    w.tiles_per_block = (w.ntiles + want - 1) / want;
    w.chunks = (w.ntiles + w.tiles_per_block - 1) / w.tiles_per_block;
  } else {
    w.g = col_grid(M, Cp, 16, k <= 3 ? 512 : 768 / k);
    w.chunks = w.g.chunks;
  }
  return w;
}

struct WgradCfg { int TM, TN, BKP, tiles_k, tiles_j, splits, pix_per_split; bool dma; };
// taps = R * S of the layer (J = taps * C).  Layers with a filter (taps > 1), whole 64- or 96-channel groups and a
// long pixel range take wgrad_dma_kernel: TM x 256 tiles, one workgroup per compute unit, the pixel range cut
// so that about 256 workgroups result.  Everything else (1 x 1 layers, which are bound by memory, stems) keeps
// wgrad_tr_kernel.
WgradCfg wgrad_cfg(long M, int K, int J, int taps) {
  WgradCfg w;
  w.dma = false;
  // (measured on the 3 x 3 layers of ResNet-50 x1.5 at batch 256: 192 channels 274 -> 184 us, 768 channels 265 -> 166 us,
  // 384 channels 204 -> 190 us; tiles of 128, 96 or 64 channels are no faster than wgrad_tr_kernel and stay with it)
  if (taps > 1 && M >= 8192 && J >= 512 && (K % 256 == 0 || K % 192 == 0) && (J / taps) % 8 == 0) {
    w.dma = true;
    w.TM = K % 256 == 0 ? 256 : 192;
    w.TN = kWgradTN;
    w.BKP = 32;
    w.tiles_k = K / w.TM;
    w.tiles_j = (J + w.TN - 1) / w.TN;
    const long tiles = (long)w.tiles_k * w.tiles_j;
    long splits = std::max(1L, 256 / tiles);
    splits = std::min(splits, std::max(1L, (long)(256u << 20) / ((long)K * J * 4)));
    splits = std::min(splits, (M + w.BKP - 1) / w.BKP);
    long pps = (M + splits - 1) / splits;
    pps = (pps + w.BKP - 1) / w.BKP * w.BKP;
    w.pix_per_split = (int)pps;
    w.splits = (int)((M + pps - 1) / pps);
    return w;
  }
  w.TM = K > 64 ? 128 : 64;       // a 128-wide tile that is 3/4 full still beats two 64-wide ones
  w.TN = J > 64 ? 128 : 64;
  w.BKP = 32;
  w.tiles_k = (K + w.TM - 1) / w.TM;
  w.tiles_j = (J + w.TN - 1) / w.TN;
  const long tiles = (long)w.tiles_k * w.tiles_j;
  // How many ways to cut the pixel range: q = ceil(tiles * splits / 256) workgroups share a compute unit; one alone
  // leaves the matrix cores waiting for its loads, two run 1.55 x, three or more 2 x as fast together (768 ->
  // 2048, 1 x 1, 12544 pixels, 96 tiles: 2 / 3 / 5 / 8 splits take 114 / 92 / 63 / 56 us); every split writes and
  // re-reads K x J partial sums.  Time model: q * pixels per split * 18.2 ns (a 128 x 128 tile) / speed-up + partials
  // at 3 TB/s; the smallest estimate wins, the fewest splits among equals.
  const long max_by_mem = std::max(1L, (long)(256u << 20) / ((long)K * J * 4));
  const long smax = std::max(1L, std::min(std::min(max_by_mem, (M + w.BKP - 1) / w.BKP), (2048 + tiles - 1) / tiles));
  const double c_pix = 18.2e-9 * (double)(w.TM * w.TN) / (128.0 * 128.0);
  double best = 1e30;
  long splits = 1;
  for (long sp = 1; sp <= smax; ++sp) {
    const long q = (tiles * sp + 255) / 256;
    const double eff = q >= 3 ? 2.0 : q == 2 ? 1.55 : 1.0;
    const double t = (double)q * ((double)M / sp) * c_pix / eff + (double)sp * K * J * 4.0 / 3e12;
    if (t < best * 0.999) { best = t; splits = sp; }
  }
  long pps = (M + splits - 1) / splits;
  pps = (pps + w.BKP - 1) / w.BKP * w.BKP;
  w.pix_per_split = (int)pps;
  w.splits = (int)((M + pps - 1) / pps);
  return w;
}

// Tile shape and split-K factor of an implicit-GEMM launch.  256 CUs want >= 512 workgroups: layers
// with few output tiles (late VGG / ResNet stages at small batch x image) first drop to 64-row tiles
// and then cut their reduction into slices that run side by side.
struct IgemmCfg { int BM, BN, BK, splits; };
IgemmCfg igemm_cfg(long M, int NC, int Kred, int CA) {
  IgemmCfg c;
  c.BK = CA % 64 == 0 ? 64 : 32;       // whole cache lines per row chunk where the channel count allows
  c.BN = NC >= 128 ? 128 : (NC > 32 ? 64 : 32);
  const long tn = (NC + c.BN - 1) / c.BN;
  c.BM = ((M + 127) / 128) * tn >= 512 ? 128 : 64;
  if (c.BK == 32 && c.BN == 128 && ((M + 255) / 256) * tn >= 1024) c.BM = 256;
  const long tiles = ((M + c.BM - 1) / c.BM) * tn;
  const int nk = (Kred + c.BK - 1) / c.BK, nk32 = (Kred + 31) / 32;
  c.splits = 1;
  if (tiles < 512 && nk32 >= 32)
    c.splits = (int)std::max(1L, std::min<long>(std::min<long>(std::min<long>((512 + tiles - 1) / tiles, nk32 / 16), 32L), nk));
  return c;
}
int igemm_splits(long M, int NC, int Kred, int CA) { return igemm_cfg(M, NC, Kred, CA).splits; }

// Launch shape of igemm_dma_kernel (256-row tiles, operands straight into LDS) for one dense layer, or use = false
// when the layer keeps igemm_kernel: channel counts that are no multiple of 32, fewer tiles than most of the
// compute units (there 128- and 64-row tiles and split-K fill the chip better), and reductions shorter than 256
// (one or two steps per tile: nothing to pipeline).
struct DmaCfg { bool use; int BN, BK, tiles_n, big_m, tail_m; };
// epi: what the store does (EPI_AFFINE_ACT: a folded batch norm and activation, the frozen teacher's layers)
DmaCfg dma_cfg(long M, int NC, int Kred, int CA, int num_cu, int epi) {
  DmaCfg d{};
  const bool affine = epi == EPI_AFFINE_ACT;
  if (CA % 32 != 0 || NC % 8 != 0 || NC < 64 || M < 4096) return d;
  // 1 x 1 layers from 64 channels on (measured per layer inside the ResNet-50 x1.5 step against the 128-row kernel:
  // student 96 -> 256 at 56 x 56 178 -> 162 us, 192 -> 512 at 28 x 28 126 -> 96 us; teacher 64 -> 256 with the fused
  // residual 233 -> 183 us, 128 -> 512 140 -> 105 us on the narrow tiles chosen below); filters from 256 reduction
  // elements on.
  if (Kred < (Kred == CA ? 64 : 256)) return d;
  const long tm = (M + kDmaBM - 1) / kDmaBM;
  // One workgroup per compute unit is resident: time ~ rounds x columns of the tile (a little more per column for
  // narrow tiles, whose fragments feed fewer MFMAs).  A last round that fills at most a quarter of the units is
  // run as 64-row tail tiles instead, which costs two thirds of a round (a tail tile still loads the whole
  // weight tile: measured 275.7 -> 252.6 us on 256 x 28 x 28 x 256 -> 256, 3 x 3, 784 tiles).
  // Short reductions behind a store without batch-norm sums (the teacher's, the accumulating backward-data ones)
  // run faster as two narrow workgroups per compute unit than as one wide one: one fills while the other stores
  // (1024 -> 256 at 14 x 14, affine: 91 -> 66 us; 256 -> 96 accumulating at 56 x 56: 198 -> 176 us); with the sums
  // in the store the wide tile stays ahead (192 -> 512 at 28 x 28: 97 against 103 us).  Measured per layer inside
  // the ResNet-50 x1.5 step.
  const bool narrow = (epi == EPI_AFFINE_ACT || epi == EPI_ACCUM) && (Kred <= 512 || (affine && Kred <= 1024 && NC >= 512));
  static const int kBN[5] = {256, 192, 128, 96, 64};
  static const double kCost[5] = {1.0, 1.05, 1.15, 1.25, 1.4};
  double best = 1e30;
  for (int i = 0; i < 5; ++i) {
    const int bn = kBN[i];
    if (narrow && bn > 128) continue;
    const long tn = (NC + bn - 1) / bn, T = tm * tn;
    const long slots = (bn <= 128 ? 2 : 1) * (long)num_cu;       // (narrow tiles: two resident workgroups per unit)
    const long full = T / slots, r = T % slots;
    double rounds = (double)full;
    if (r) rounds += (full >= 1 && r <= slots / 4) ? 0.66 : 1.0;
    const double t = rounds * slots * bn * kCost[i];
    if (t < best) { best = t; d.BN = bn; d.tiles_n = (int)tn; }
  }
  // K step 64 (128-byte rows) for the wide tiles; the narrow ones take 32, whose three stages fit twice in a
  // compute unit's LDS, so that two workgroups hide each other's fill, barriers and store
  // (256 x 56 x 56 x 64 -> 64, 3 x 3: 129 -> 113 us; 256 -> 96, 1 x 1: 152 -> 124 us)
  d.BK = CA % 64 == 0 && d.BN >= 192 ? 64 : 32;
  const long T = tm * d.tiles_n;
  if (T < num_cu * 7 / 10) return d;       // (use stays false)
  d.use = true;
  d.big_m = (int)tm;
  d.tail_m = 0;
  const long slots = (d.BN <= 128 ? 2 : 1) * (long)num_cu;
  const long r = T % slots;
  if (T >= slots && r && r <= slots / 4) {
    const int cut = (int)((r + d.tiles_n - 1) / d.tiles_n);     // row tiles that go to the tail
    d.big_m = (int)tm - cut;
    d.tail_m = (int)((M - (long)d.big_m * kDmaBM + kDmaTailBM - 1) / kDmaTailBM);
  }
  return d;
}

constexpr int kMseBlocks = 1024;

// the stem that is run on the space-to-depth copy of the input: first block, reads A_0, 7 x 7, stride 2, pad 3,
// at most 4 input channels, even image size, bf16 MFMA path
bool stem_s2d(const pbd_ctx* c, int block, const OpPlan& op) {
  return c->o.precision == PBD_BF16 && !c->o.force_direct && block == 0 && op.d.type == OP_CBA && !op.dw &&
         op.d.in[0] == 0 && op.d.k == 7 && op.d.stride == 2 && op.d.pad == 3 && op.in.c <= 4 && op.cin_p == 8 &&
         op.in.h % 2 == 0 && op.in.w % 2 == 0 && op.out.h == op.in.h / 2 && op.out.w == op.in.w / 2;
}
constexpr int kS2dK = 256;     // reduction length of such a stem: 4 x 4 taps x 16 lanes

int plan(pbd_ctx* c) {
  const size_t es = c->esz;
  const bool bf = c->o.precision == PBD_BF16;
  size_t p = 0;  // parameter region cursor
  auto take = [&](size_t bytes) { size_t o = p; p += align_up(bytes); return o; };
  size_t red = kMseBlocks * sizeof(float);  // reduction scratch of the block being planned
  auto need_red = [&](size_t bytes) { red = std::max(red, bytes); };

  // teacher parameters
  for (BlockPlan& bp : c->net[0])
    for (OpPlan& op : bp.ops) {
      if (op.d.type != OP_CBA) continue;
      if (!op.dw && bf) {
        const long M = (long)c->o.batch * op.out.h * op.out.w;
        need_red((size_t)igemm_splits(M, op.d.c_out, op.d.k * op.d.k * op.cin_p, op.cin_p) * M * op.d.c_out * 4);
      }
      op.t_w = take(op.wn * es);
      op.s2d = stem_s2d(c, (int)(&bp - &c->net[0][0]), op);
      if (op.s2d) {
        op.w2 = take((size_t)op.d.c_out * kS2dK * es);
        const long M = (long)c->o.batch * op.out.h * op.out.w;
        need_red((size_t)igemm_splits(M, op.d.c_out, kS2dK, 16) * M * op.d.c_out * 4);
      }
      op.t_gamma = take(op.cout_p * 4); op.t_beta = take(op.cout_p * 4);
      op.t_rmean = take(op.cout_p * 4); op.t_rvar = take(op.cout_p * 4);
      op.t_a = take(op.cout_p * 4); op.t_b = take(op.cout_p * 4);
    }
  // student parameters: one flat arena per block
  for (BlockPlan& bp : c->net[1]) {
    size_t e = 0, et = 0;
    bp.nmix = 0;
    for (OpPlan& op : bp.ops) {
      if (op.d.type == OP_MIX) op.mix_slot = bp.nmix++;
      if (op.d.type != OP_CBA) continue;
      op.e_w = e; e += op.wn;
      op.e_gamma = e; e += op.cout_p;
      op.e_beta = e; e += op.cout_p;
      for (size_t* s : {&op.s_rmean, &op.s_rvar, &op.s_mean, &op.s_invstd, &op.s_k2, &op.s_k3})
        *s = take(op.cout_p * 4);
      op.s2d = stem_s2d(c, (int)(&bp - &c->net[1][0]), op);
      if (op.s2d) op.w2 = take((size_t)op.d.c_out * kS2dK * es);
      // transposed copy for backward-data of dense convolutions that need it
      if (!op.dw && op.d.in[0] != 0 && bf) {
        op.e_wt = (long)et;
        bp.ttable.push_back({(long)op.e_w, (long)et, op.d.c_out, op.d.k * op.d.k, op.cin_p});
        et += op.wn;
      }
    }
    bp.arena_elems = e;
    bp.wt_elems = et;
    bp.master = take(e * 4); bp.mom = take(e * 4); bp.grad = take(e * 4);
    bp.wc = bf ? take(e * 2) : bp.master;
    bp.wt = take(std::max<size_t>(et, 1) * es);
    bp.table = take(std::max<size_t>(bp.ttable.size(), 1) * sizeof(TransposeEntry));
    bp.mix = take((size_t)std::max(bp.nmix, 1) * kMixState * sizeof(float));
    bp.alpha_defined.assign(bp.nmix, 0);
  }
  c->lr_off = take(256);
  c->loss_off = take((size_t)c->B * 4);
  c->r_param = 0;
  const size_t teacher_red = align_up(red);
  size_t cur = align_up(p);
  // relay store A_0..A_B
  c->r_relay = cur;
  c->act_off.clear();
  size_t r = 0;
  for (Shape s : c->act) { c->act_off.push_back(r); r += tensor_bytes(c, s); }
  c->s2d_off = (size_t)-1;
  for (int t = 0; t < 2; ++t)
    for (const OpPlan& op : c->net[t][0].ops)
      if (op.s2d && c->s2d_off == (size_t)-1) {
        c->s2d_off = r;
        r += align_up((size_t)c->o.batch * (op.in.h / 2) * (op.in.w / 2) * 16 * es);
      }
  cur += r;
  c->r_relay2 = cur;      // second copy: the teacher fills one while the students still read the other
  cur += r;
  // teacher scratch: every value of the largest block except its output (-> relay)
  size_t tmax = 0;
  for (BlockPlan& bp : c->net[0]) {
    size_t s = 0;
    bp.val.assign(bp.shapes.size(), 0);
    for (size_t v = 1; v + 1 < bp.shapes.size(); ++v) { bp.val[v] = s; s += tensor_bytes(c, bp.shapes[v]); }
    bp.scratch_bytes = s;
    tmax = std::max(tmax, s);
  }
  c->r_tscr = cur; cur += align_up(tmax);
  // student scratch per block: values, conv outputs, pool indices, value gradients
  size_t smax = 0;
  size_t ssum = 0;
  for (BlockPlan& bp : c->net[1]) {
    size_t s = 0;
    red = kMseBlocks * sizeof(float);
    bp.val.assign(bp.shapes.size(), 0);
    bp.dval.assign(bp.shapes.size(), 0);
    for (size_t v = 1; v < bp.shapes.size(); ++v) {
      bp.val[v] = s; s += tensor_bytes(c, bp.shapes[v]);
      bp.dval[v] = s; s += tensor_bytes(c, bp.shapes[v]);
      OpPlan& op = bp.ops[v - 1];
      const long M = (long)c->o.batch * op.out.h * op.out.w;
      if (op.d.type == OP_CBA) {
        op.y = s; s += tensor_bytes(c, op.out);
        const ColGrid g = bn_bwd_grid(M, op.cout_p);   // the larger of the two reductions' grids
        need_red(((size_t)g.chunks * 2 * op.cout_p + (size_t)g.slabs * g.chunks) * 4);   // (+ one loss partial a workgroup)
        if (op.dw) {
          const DwWgradCfg gw = dw_wgrad_cfg(bf && !c->o.force_direct, c->o.batch, op.out.h, op.out.w, op.cout_p, op.d.k,
                                             op.d.stride, op.d.pad);
          need_red((size_t)gw.chunks * op.d.k * op.d.k * op.cout_p * 4);
        } else if (bf && !c->o.force_direct) {
          const WgradCfg w = op.s2d ? wgrad_cfg(M, op.d.c_out, kS2dK, 16) : wgrad_cfg(M, op.d.c_out, op.d.k * op.d.k * op.cin_p, op.d.k * op.d.k);
          // (the stem on the space-to-depth input: partial sums and their sum in the repacked layout, then unpacked)
          need_red(op.s2d ? ((size_t)w.splits + 1) * op.d.c_out * kS2dK * 4 : (size_t)w.splits * op.wn * 4);
          // per-row-tile batch-norm sums from the convolution's store (64-row tiles at most), and their regrouping
          need_red(((size_t)(M + 63) / 64 + kStatGroupsMax + 1) * 2 * op.cout_p * 4);
          const long Min = (long)c->o.batch * op.in.h * op.in.w;
          need_red((size_t)igemm_splits(M, op.d.c_out, op.d.k * op.d.k * op.cin_p, op.cin_p) * M * op.d.c_out * 4);
          if (op.s2d) need_red((size_t)igemm_splits(M, op.d.c_out, kS2dK, 16) * M * op.d.c_out * 4);
          need_red((size_t)igemm_splits(Min, op.cin_p, op.d.k * op.d.k * op.d.c_out, op.d.c_out) * Min * op.cin_p * 4);
        }
      } else if (op.d.type == OP_POOL) {
        op.idx = s; s += align_up((size_t)M * op.cout_p);
      } else if (op.d.type == OP_MIX) {
        need_red((size_t)kMixDotBlocks * 8 * sizeof(float));
      }
    }
    bp.scratch_bytes = align_up(s);
    bp.red_bytes = align_up(red);
    smax = std::max(smax, bp.scratch_bytes + bp.red_bytes);
    ssum += bp.scratch_bytes + bp.red_bytes;
  }
  c->r_tred = cur; cur += teacher_red;
  // Blocks are independent (Sec. IV-B): when the sum of their scratch fits comfortably in HBM each
  // block gets its own region, so that their kernels can overlap; otherwise they share one region.
  c->concurrent = c->B > 1 && cur + ssum <= ((size_t)160 << 30);
  size_t at = cur;
  for (BlockPlan& bp : c->net[1]) {
    bp.scr_off = at;
    bp.red_off = at + bp.scratch_bytes;
    if (c->concurrent) at += bp.scratch_bytes + bp.red_bytes;
  }
  cur = c->concurrent ? at : cur + smax;
  c->total = cur;
  return PBD_OK;
}

// ---------------------------------------------------------------------------
// launch plumbing
// ---------------------------------------------------------------------------
inline int grid_for(long n, int block = 256, int cap = 256 * 32) {
  return (int)std::max(1L, std::min<long>((n + block - 1) / block, cap));
}

struct ProfScope {
  pbd_ctx* c;
  bool on;
  ProfScope(pbd_ctx* ctx, const char* name, double bytes, double flops, int net, int block, int op) : c(ctx), on(ctx->prof_on) {
    if (!on) return;
    pbd_prof_entry e{};
    snprintf(e.name, sizeof e.name, "%s", name);
    e.bytes = bytes; e.flops = flops; e.net = net; e.block = block; e.op = op;
    c->prof.push_back(e);
    const size_t need = c->prof.size() * 2;
    while (c->ev.size() < need) { hipEvent_t ev; (void)hipEventCreate(&ev); c->ev.push_back(ev); }
    c->pend_start = c->ev[need - 2]; c->pend_stop = c->ev[need - 1];   // the scope's first launch takes them
  }
  ~ProfScope() { if (on) c->pend_start = c->pend_stop = nullptr; }
};

// Launch through one place.  A profiled launch attaches its two events to the dispatch itself, so
// their distance is the kernel's own run time (what a kernel trace reports), not the gap between
// two markers in the stream.  The lambda converts every argument to the kernel's parameter type.
template <class... KA, class... A>
inline void launch(pbd_ctx* c, void (*kern)(KA...), dim3 grid, dim3 block, size_t smem, hipStream_t st, A&&... a) {
  static_assert(sizeof...(KA) == sizeof...(A), "argument count differs from the kernel's");
  [&](KA... ka) {
    void* argv[] = {(void*)&ka...};
    if (c->pend_start) {
      (void)hipExtLaunchKernel((const void*)kern, grid, block, argv, smem, st, c->pend_start, c->pend_stop, 0);
      c->pend_start = c->pend_stop = nullptr;
    } else {
      (void)hipLaunchKernel((const void*)kern, grid, block, argv, smem, st);
    }
  }(std::forward<A>(a)...);
}

// For op j of a block: the index of an add op that (a) is the only reader of j's output, (b) has two
// inputs, the other one computed before j, and (c) follows a layer without activation; else -1.
int residual_reader(const BlockPlan& bp, int j) {
  const OpD& o = bp.ops[j].d;
  if (o.type != OP_CBA || o.act != ACT_NONE) return -1;
  int reader = -1, uses = 0;
  for (int k = j + 1; k < (int)bp.ops.size(); ++k) {
    const OpD& q = bp.ops[k].d;
    const int nin = q.type == OP_ADD || q.type == OP_MIX ? q.nin : 1;
    for (int i = 0; i < nin; ++i)
      if (q.in[i] == j + 1) { ++uses; reader = k; }
  }
  if (uses != 1 || j + 2 == (int)bp.shapes.size()) return -1;      // (a block's last value is read by the loss)
  const OpD& q = bp.ops[reader].d;
  if (q.type != OP_ADD || q.nin != 2) return -1;
  const int other = q.in[0] == j + 1 ? q.in[1] : q.in[0];
  return other <= j ? reader : -1;
}
// few enough rows for the whole-column BN kernels (one block per 8-channel slab)
inline bool short_column(long M) { return M <= (long)kSmallThreads * kSmallRows; }
// For student layer j: the index of a max-pool that is the only reader of j's output (the pool then normalises what
// it reads and the normalised tensor is never written), else -1.
int pool_reader(const BlockPlan& bp, int j, int batch) {
  const OpPlan& p = bp.ops[j];
  if (p.d.type != OP_CBA || j + 2 == (int)bp.shapes.size() || short_column((long)batch * p.out.h * p.out.w)) return -1;
  int reader = -1, uses = 0;
  for (int k = j + 1; k < (int)bp.ops.size(); ++k) {
    const OpD& q = bp.ops[k].d;
    const int nin = q.type == OP_ADD || q.type == OP_MIX ? q.nin : 1;
    for (int i = 0; i < nin; ++i)
      if (q.in[i] == j + 1) { ++uses; reader = k; }
  }
  return uses == 1 && bp.ops[reader].d.type == OP_POOL ? reader : -1;
}

template <class T> struct Exec {
  pbd_ctx* c;
  hipStream_t st;
  int net = 0, blk = 0, opi = 0;
  size_t red_off;
  float* red_static = nullptr;   // reduction scratch outside the workspace (pbd_student_step_static)
  int tset, sset;      // copy of the relay store the teacher writes / the students read
  explicit Exec(pbd_ctx* ctx) : c(ctx), st(ctx->stream), red_off(ctx->r_tred), tset(ctx->front), sset(ctx->front) {}

  T* ws(size_t off) const { return reinterpret_cast<T*>(c->ws + off); }
  float* wsf(size_t off) const { return reinterpret_cast<float*>(c->ws + off); }
  T* relay_in(int i, int set) const { return ws((set ? c->r_relay2 : c->r_relay) + c->act_off[i]); }
  T* trelay(int i) const { return relay_in(i, tset); }
  T* srelay(int i) const { return relay_in(i, sset); }
  // the space-to-depth copy of A_0 that the net at hand reads
  T* s2d_input() const { return ws(((net == PBD_TEACHER ? tset : sset) ? c->r_relay2 : c->r_relay) + c->s2d_off); }
  // reduction length and gathered channels of a dense convolution as it is run
  static int kred_of(const OpPlan& op) { return op.s2d ? kS2dK : op.d.k * op.d.k * op.cin_p; }
  // (a space-to-depth stem: 64 where the direct-to-LDS kernel takes it, which gathers a filter row at a time)
  int ca_of(const OpPlan& op) const {
    if (!op.s2d) return op.cin_p;
    return dma_for((long)c->o.batch * op.out.h * op.out.w, op.d.c_out, kS2dK, 64).use ? 64 : 16;
  }
  float* red() const { return red_static ? red_static : wsf(red_off); }
  double bytes_of(Shape s) const { return (double)c->o.batch * s.h * s.w * round8(s.c) * sizeof(T); }
  bool mfma() const { return sizeof(T) == 2 && !c->o.force_direct; }
  // The batch-norm passes over a tensor of this shape use nontemporal loads and stores (bf16 tensors far larger than
  // L2: what they stream through would only push out the lines that convolutions running beside them reuse).
  // From 64 MiB on (measured 8 ... 200 MiB on the four large configurations: ResNet-50 x1.5 30.40 -> 29.74 ms per step,
  // MobileNetV2 7.53 -> 7.28, supernet 48.92 -> 48.02; smaller tensors are re-read from the caches by the next kernel).
  bool streams(Shape s) const { return sizeof(T) == 2 && bytes_of(s) >= 64.0 * 1048576.0; }

  // ---- convolution forward (dense) --------------------------------------
  // Can a two-input add that is the only reader of this convolution's output ride in its store?  Only the
  // MFMA kernel's LDS-staged store does it: no split-K, and not the 64 x 32 tile (whose idle waves skip it).
  bool fuses_residual(const OpPlan& op) const {
    if (!mfma() || op.dw) return false;
    const IgemmCfg cfg = igemm_cfg((long)c->o.batch * op.out.h * op.out.w, op.d.c_out, kred_of(op), ca_of(op));
    return cfg.splits == 1 && !(cfg.BM == 64 && cfg.BN == 32);      // (the 256-row kernel, where it is used, fuses it too)
  }
  // the 256-row, direct-to-LDS kernel takes a launch when its tile count fills the chip and no split-K is wanted
  DmaCfg dma_for(long M, int NC, int Kred, int CA, int epi = EPI_STORE) const {
    DmaCfg d = dma_cfg(M, NC, Kred, CA, c->num_cu, epi);
    if (d.use && igemm_cfg(M, NC, Kred, CA).splits != 1) d.use = false;
    return d;
  }
  // Row tiles whose staged store also delivers the batch-norm sums of the convolution's output (0: the
  // layer takes its statistics in a pass of its own).  Same conditions as fuses_residual, whole channel
  // vectors, and a column long enough for the chunked normalisation path.
  int fused_stats_tiles(const OpPlan& op) const {
    const long M = (long)c->o.batch * op.out.h * op.out.w;
    if (!fuses_residual(op) || op.d.c_out % 8 != 0 || short_column(M)) return 0;
    const DmaCfg d = dma_for(M, op.d.c_out, kred_of(op), ca_of(op));
    if (d.use) return d.big_m + d.tail_m;
    const IgemmCfg cfg = igemm_cfg(M, op.d.c_out, kred_of(op), ca_of(op));
    return (int)((M + cfg.BM - 1) / cfg.BM);
  }
  // res (optional): a residual join fused into the store, y = res_act(conv result + res); only where
  // fuses_residual(op) holds.  stats (optional): per row tile sums of y and y^2, where fused_stats_tiles(op) > 0
  void conv_fwd(const OpPlan& op, const T* x, const T* w, T* y, const float* a, const float* b, int act,
                const T* res = nullptr, int res_act = 0, float* stats = nullptr) {
    const int N = c->o.batch;
    const double flops = 2.0 * N * op.out.h * op.out.w * op.d.c_out * op.d.k * op.d.k * op.in.c;
    const double bytes = bytes_of(op.in) + bytes_of(op.out) * (res ? 2 : 1) + (double)op.wn * sizeof(T);
    if (mfma()) {
      if constexpr (sizeof(T) == 2) {
        IgemmArgs g{N, op.in.h, op.in.w, op.cin_p, op.out.h, op.out.w, op.d.c_out, op.d.k, op.d.k,
                    op.d.stride, op.d.pad, N * op.out.h * op.out.w, op.d.k * op.d.k * op.cin_p, 0,
                    (unsigned)((size_t)N * op.in.h * op.in.w * op.cin_p * 2), (unsigned)(op.wn * 2)};
        double bytes_run = bytes;
        if (op.s2d) {
          // 4 x 4, stride 1, two rows / columns of padding in front, over the space-to-depth copy of the input
          g.HA = op.in.h / 2; g.WA = op.in.w / 2; g.CA = 16; g.R = g.S = 4; g.stride = 1; g.pad = 2; g.Kred = kS2dK;
          // the four taps of a filter row are 64 contiguous elements: one tap of four pixels to the direct-to-LDS kernel
          if (dma_for(g.M, g.NC, kS2dK, 64, a ? EPI_AFFINE_ACT : EPI_STORE).use) { g.CA = 64; g.S = 1; g.pix_shift = 2; }
          g.a_bytes = (unsigned)((size_t)N * g.HA * g.WA * 16 * 2); g.b_bytes = (unsigned)(op.d.c_out * kS2dK * 2);
          x = s2d_input();
          w = reinterpret_cast<const T*>(c->ws + op.w2);
          bytes_run = (double)g.a_bytes + bytes_of(op.out) * (res ? 2 : 1) + (double)g.b_bytes;
        }
        g.res = res; g.res_act = res_act; g.stats = stats;
        launch_igemm<0>(g, (const bf16_t*)x, (const bf16_t*)w, (bf16_t*)y, a, b, act, a ? EPI_AFFINE_ACT : EPI_STORE,
                        bytes_run, flops);
      }
    } else {
      ConvGeom g{N, op.in.h, op.in.w, op.cin_p, op.out.h, op.out.w, op.d.c_out, op.d.k, op.d.k, op.d.stride, op.d.pad};
      ProfScope ps(c, "conv_fwd_direct", bytes, flops, net, blk, opi);
      launch(c, conv_direct_fwd_kernel<T, T>, grid_for((long)g.N * g.P * g.Q * g.K), 256, 0, st, x, w, y, a, b, act, g);
    }
  }

  template <int MODE>
  void launch_igemm(IgemmArgs g, const bf16_t* A, const bf16_t* Bw, bf16_t* out, const float* a,
                    const float* b, int act, int epi, double bytes, double flops) {
    DmaCfg dc = dma_for(g.M, g.NC, g.Kred, g.CA, epi);
    g.stream_out = (double)g.M * g.NC * 2.0 >= 64.0 * 1048576.0;   // (as for the batch-norm passes: see streams())
    if (MODE == 1 && g.par_classes) {
      // parity classes: par_classes x ceil(rows of a class / 256) row tiles, no tail tiles
      const long mc = (long)g.N * (g.HO / 2) * (g.WO / 2);
      const int tm = (int)((mc + kDmaBM - 1) / kDmaBM);
      // a class reduces over few taps: short tiles, for which two resident workgroups (narrow tile, K step 32)
      // beat the wide tile (256 x 28 x 28 x 384, 3 x 3: 176 us at 128 columns, 222 us at 192; 56 x 56 x 192: 266 us
      // at 96, 324 us at 192; 14 x 14 x 768: 187 us at 128, 189 us at 192)
      int bn = 0;
      for (int b : {128, 96, 64})
        if (g.NC % b == 0) { bn = b; break; }
      if (dc.use && bn && (long)tm * g.par_classes * (g.NC / bn) >= c->num_cu * 7 / 10) {
        dc.BN = bn; dc.BK = 32; dc.tiles_n = g.NC / bn;
        dc.big_m = tm * g.par_classes; dc.tail_m = 0;
      }
      else g.par_classes = 0;               // (the other kernels take the rows in pixel order)
    }
    if (dc.use && (epi == EPI_STORE || epi == EPI_AFFINE_ACT || epi == EPI_ACCUM)) {
      g.tiles_n = dc.tiles_n;
      g.tiles_m = dc.big_m + dc.tail_m;
      g.splits = 1;
      g.big_tiles = dc.big_m * dc.tiles_n;
      g.tail_m0 = dc.big_m * kDmaBM;
      const dim3 grid(g.big_tiles + dc.tail_m * dc.tiles_n);
      static const char* const kEpiName[] = {"store", "affine", "accum"};
      char name[40];
      snprintf(name, sizeof name, "igemm_%s_256x%dx%d_%s", MODE ? "dgrad" : "fwd", dc.BN, dc.BK, kEpiName[epi]);
      ProfScope ps(c, name, bytes, flops, net, blk, opi);
#define PBD_DMA(BN_, BK_, EPI_) launch(c, igemm_dma_kernel<MODE, BN_, BK_, EPI_>, grid, kDmaThreads, 0, st, A, Bw, out, a, b, act, g)
#define PBD_DMA_BK(BN_, EPI_) do { if (dc.BK == 64) PBD_DMA(BN_, 64, EPI_); else PBD_DMA(BN_, 32, EPI_); } while (0)
#define PBD_DMA_BN(EPI_) do { switch (dc.BN) { case 256: PBD_DMA_BK(256, EPI_); break; case 192: PBD_DMA_BK(192, EPI_); break; \
        case 128: PBD_DMA_BK(128, EPI_); break; case 96: PBD_DMA_BK(96, EPI_); break; default: PBD_DMA_BK(64, EPI_); } } while (0)
      // (forward launches never accumulate, backward-data launches have no folded batch norm)
      if constexpr (MODE == 0) { if (epi == EPI_AFFINE_ACT) PBD_DMA_BN(EPI_AFFINE_ACT); else PBD_DMA_BN(EPI_STORE); }
      else { if (epi == EPI_ACCUM) PBD_DMA_BN(EPI_ACCUM); else PBD_DMA_BN(EPI_STORE); }
#undef PBD_DMA_BN
#undef PBD_DMA_BK
#undef PBD_DMA
      return;
    }
    IgemmCfg cfg = igemm_cfg(g.M, g.NC, g.Kred, g.CA);
    // an accumulating 256-row tile cannot stage its fp32 results in LDS: 128 rows store whole cache lines
    if (epi == EPI_ACCUM && cfg.BM == 256) cfg.BM = 128;
    if (epi == EPI_ACCUM && cfg.BK == 32 && cfg.BM == 128 && cfg.BN == 128) cfg.BN = 64;   // (128 x 128 needs the 64-wide K step's LDS)
    const int nk = (g.Kred + cfg.BK - 1) / cfg.BK;
    g.ksteps_per_split = (nk + cfg.splits - 1) / cfg.splits;
    g.tiles_m = (g.M + cfg.BM - 1) / cfg.BM;
    g.tiles_n = (g.NC + cfg.BN - 1) / cfg.BN;
    g.splits = (nk + g.ksteps_per_split - 1) / g.ksteps_per_split;
    const dim3 grid(g.tiles_m * g.tiles_n * g.splits);
#define PBD_IG(BM_, BN_, EPI_, OUT_) do { \
      if (cfg.BK == 64) { if constexpr (BM_ != 256) launch(c, igemm_kernel<MODE, BM_, BN_, EPI_, true, 64>, grid, 256, 0, st, A, Bw, OUT_, a, b, act, g); } \
      else if (g.CA % IG_BK == 0) launch(c, igemm_kernel<MODE, BM_, BN_, EPI_, true>, grid, 256, 0, st, A, Bw, OUT_, a, b, act, g); \
      else launch(c, igemm_kernel<MODE, BM_, BN_, EPI_, false>, grid, 256, 0, st, A, Bw, OUT_, a, b, act, g); } while (0)
#define PBD_IG_BN(BM_, EPI_, OUT_) do { if (cfg.BN == 128) PBD_IG(BM_, 128, EPI_, OUT_); else if (cfg.BN == 64) PBD_IG(BM_, 64, EPI_, OUT_); else PBD_IG(BM_, 32, EPI_, OUT_); } while (0)
#define PBD_IG_BM(EPI_, OUT_) do { if (cfg.BM == 256) PBD_IG(256, 128, EPI_, OUT_); else if (cfg.BM == 128) PBD_IG_BN(128, EPI_, OUT_); else PBD_IG_BN(64, EPI_, OUT_); } while (0)
    // profile entries are named after the kernel instantiation, so that each maps to one symbol of
    // a rocprofv3 kernel trace: igemm_<fwd|dgrad>_<BM>x<BN>_<epilogue>
    static const char* const kEpi[] = {"store", "affine", "accum", "partial"};
    char name[32];
    snprintf(name, sizeof name, "igemm_%s_%dx%d_%s", MODE ? "dgrad" : "fwd", cfg.BM, cfg.BN, kEpi[g.splits > 1 ? 3 : epi]);
    if (g.splits > 1) {
      {
        ProfScope ps(c, name, bytes, flops, net, blk, opi);
        PBD_IG_BM(EPI_PARTIAL, reinterpret_cast<bf16_t*>(red()));
      }
      const long nvec = (long)g.M * g.NC / 8;
      ProfScope ps(c, "splitk_epilogue", (double)nvec * 8 * (4.0 * g.splits + 2), 0, net, blk, opi);
      launch(c, splitk_epilogue_kernel, grid_for(nvec), 256, 0, st, red(), out, a, b, act, epi, nvec, g.NC / 8, g.splits);
    } else {
      ProfScope ps(c, name, bytes, flops, net, blk, opi);
      if (epi == EPI_AFFINE_ACT) PBD_IG_BM(EPI_AFFINE_ACT, out);
      else if (epi == EPI_ACCUM) PBD_IG_BM(EPI_ACCUM, out);
      else PBD_IG_BM(EPI_STORE, out);
    }
#undef PBD_IG_BM
#undef PBD_IG_BN
#undef PBD_IG
  }

  // ---- convolution backward-data (dense) ---------------------------------
  void conv_dgrad(const OpPlan& op, const T* dy, const T* w, const T* wt, T* dx, bool accumulate) {
    const int N = c->o.batch;
    const double flops = 2.0 * N * op.out.h * op.out.w * op.d.c_out * op.d.k * op.d.k * op.in.c;
    const double bytes = bytes_of(op.in) + bytes_of(op.out) + (double)op.wn * sizeof(T);
    if (mfma()) {
      if constexpr (sizeof(T) == 2) {
        // rows = input pixels, columns = input channels, reduction over (r, s, k)
        IgemmArgs g{N, op.out.h, op.out.w, op.d.c_out, op.in.h, op.in.w, op.cin_p, op.d.k, op.d.k,
                    op.d.stride, op.d.pad, N * op.in.h * op.in.w, op.d.k * op.d.k * op.d.c_out, 0,
                    (unsigned)((size_t)N * op.out.h * op.out.w * op.d.c_out * 2), (unsigned)(op.wn * 2)};
        // stride 2: an input pixel is reached only by the taps of its own parity (1, 2, 2 and 4 of the 9 taps
        // of a 3 x 3 kernel for the four pixel classes; one class only for a 1 x 1 kernel), so the rows are
        // taken class by class, heaviest class first.  Classes no tap reaches hold zeros: an accumulating
        // launch leaves them out.
        if (op.d.stride == 2 && op.in.h % 2 == 0 && op.in.w % 2 == 0) {
          int taps[4], order[4] = {0, 1, 2, 3}, n = 0;
          for (int cl = 0; cl < 4; ++cl) {
            const int r0 = ((cl >> 1) + op.d.pad) & 1, s0 = ((cl & 1) + op.d.pad) & 1;
            taps[cl] = ((op.d.k - r0 + 1) / 2) * ((op.d.k - s0 + 1) / 2);
          }
          std::stable_sort(order, order + 4, [&](int a, int b) { return taps[a] > taps[b]; });
          for (int i = 0; i < 4; ++i)
            if (taps[order[i]] > 0 || !accumulate) { g.par_order |= order[i] << (2 * n); ++n; }
          g.par_classes = n;
        }
        launch_igemm<1>(g, (const bf16_t*)dy, (const bf16_t*)wt, (bf16_t*)dx, nullptr, nullptr, 0,
                        accumulate ? EPI_ACCUM : EPI_STORE, bytes, flops);
      }
    } else {
      ConvGeom g{N, op.in.h, op.in.w, op.cin_p, op.out.h, op.out.w, op.d.c_out, op.d.k, op.d.k, op.d.stride, op.d.pad};
      ProfScope ps(c, "conv_dgrad_direct", bytes, flops, net, blk, opi);
      launch(c, conv_direct_dgrad_kernel<T, T>, grid_for((long)g.N * g.H * g.W * g.C), 256, 0, st, dy, w, dx, accumulate, g);
    }
  }

  // ---- convolution backward-weight (dense) -------------------------------
  void conv_wgrad(const OpPlan& op, const T* dy, const T* x, float* dw) {
    const int N = c->o.batch;
    const long M = (long)N * op.out.h * op.out.w;
    const int J = op.d.k * op.d.k * op.cin_p;
    const double flops = 2.0 * M * op.d.c_out * op.d.k * op.d.k * op.in.c;
    const double bytes = bytes_of(op.in) + bytes_of(op.out) + (double)op.wn * 4;
    if (mfma()) {
      if constexpr (sizeof(T) == 2) {
        const WgradCfg w = op.s2d ? wgrad_cfg(M, op.d.c_out, kS2dK, 16) : wgrad_cfg(M, op.d.c_out, J, op.d.k * op.d.k);
        const int pq = op.out.h * op.out.w;
        WgradTrArgs g{N, op.in.h, op.in.w, op.cin_p, op.out.h, op.out.w, op.d.c_out, op.d.k, op.d.k,
                      op.d.stride, op.d.pad, (int)M, J, w.pix_per_split,
                      w.BKP / pq, (w.BKP % pq) / op.out.w, w.BKP % op.out.w,
                      (unsigned)(M * op.d.c_out * 2), (unsigned)((size_t)N * op.in.h * op.in.w * op.cin_p * 2),
                      w.tiles_k, w.tiles_j, w.splits};
        const dim3 grid(w.tiles_k * w.tiles_j * w.splits);
        float* part = w.splits == 1 ? dw : red();
        long wn_run = (long)op.wn;
        float* dw_run = dw;                        // where the summed gradient goes
        double bytes_run = bytes;
        if (op.s2d) {
          // the stem on the space-to-depth copy of the input: gradient of the repacked filter first (partial sums,
          // then their sum behind them in the scratch), unpacked into the 7 x 7 layout at the end
          g.H = op.in.h / 2; g.W = op.in.w / 2; g.C = 16; g.R = g.S = 4; g.stride = 1; g.pad = 2; g.J = kS2dK;
          g.x_bytes = (unsigned)((size_t)N * g.H * g.W * 16 * 2);
          x = s2d_input();
          wn_run = (long)op.d.c_out * kS2dK;
          dw_run = red() + (size_t)w.splits * wn_run;
          part = w.splits == 1 ? dw_run : red();
          bytes_run = (double)g.x_bytes + bytes_of(op.out) + (double)wn_run * 4;
        }
        {
          char name[32];
          snprintf(name, sizeof name, "wgrad_%dx%d", w.TM, w.TN);
          ProfScope ps(c, name, bytes_run, flops, net, blk, opi);
          if (w.dma) {
#define PBD_WGD(TM_) launch(c, wgrad_dma_kernel<TM_>, grid, kDmaThreads, 0, st, (const bf16_t*)dy, (const bf16_t*)x, part, g)
            if (w.TM == 256) PBD_WGD(256); else PBD_WGD(192);
#undef PBD_WGD
          } else {
#define PBD_WG(TM_, TN_) launch(c, wgrad_tr_kernel<TM_, TN_>, grid, 256, 0, st, (const bf16_t*)dy, (const bf16_t*)x, part, g)
            if (w.TM == 128) { if (w.TN == 128) PBD_WG(128, 128); else PBD_WG(128, 64); }
            else { if (w.TN == 128) PBD_WG(64, 128); else PBD_WG(64, 64); }
#undef PBD_WG
          }
        }
        if (w.splits > 1) {
          ProfScope ps(c, "sum_partials", (double)(w.splits + 1) * wn_run * 4, 0, net, blk, opi);
          sum_partials(part, dw_run, wn_run, w.splits);
        }
        if (op.s2d)
          launch(c, unpack_stem_grad_kernel, (op.d.c_out * 392 + 255) / 256, 256, 0, st, dw_run, dw, op.d.c_out, op.in.c);
      }
    } else {
      ConvGeom g{N, op.in.h, op.in.w, op.cin_p, op.out.h, op.out.w, op.d.c_out, op.d.k, op.d.k, op.d.stride, op.d.pad};
      ProfScope ps(c, "conv_wgrad_direct", bytes, flops, net, blk, opi);
      launch(c, conv_direct_wgrad_kernel<T>, grid_for((long)op.wn, 64), 64, 0, st, dy, x, dw, g);
    }
  }

  void sum_partials(const float* part, float* out, long n, int splits) {
    if (splits >= 64) launch(c, sum_partials_kernel<32>, grid_for(n / 4, 8), 256, 0, st, part, out, n, splits, n);
    else launch(c, sum_partials_kernel<8>, grid_for(n / 4, 32), 256, 0, st, part, out, n, splits, n);
  }

  // ---- depthwise ----------------------------------------------------------
  // sliding-window depthwise kernels: odd k in {3,5,7} with "same" padding, 4 outputs per thread
  static constexpr int kDwSlide = 4;
  static bool dw_slides(const OpPlan& op) {
    return (op.d.k == 3 || op.d.k == 5 || op.d.k == 7) && op.d.pad == op.d.k / 2 && (op.d.stride == 1 || op.d.stride == 2);
  }
  // LDS-tiled kernels: bf16, stride 1, images of at least one tile row and most of a tile's width
  static bool dw_tiles(const OpPlan& op) {
    return dw_tiled(sizeof(T) == 2, op.d.k, op.d.stride, op.d.pad, op.out.h, op.out.w);
  }
  void dw_fwd(const OpPlan& op, const T* x, const T* w, T* y, const float* a, const float* b, int act) {
    const int N = c->o.batch, ncv = op.cout_p / 8;
    const long nvec = (long)N * op.out.h * op.out.w * ncv;
    // one profile class per kernel template: tile (LDS), slide (registers), plain
    char cls[32];
    snprintf(cls, sizeof cls, "dw_fwd%s_k%d", dw_tiles(op) ? "_tile" : dw_slides(op) ? (op.d.stride == 1 ? "_slide" : "_slide_s2") : "", op.d.k);
    ProfScope ps(c, cls, bytes_of(op.in) + bytes_of(op.out), 2.0 * N * op.out.h * op.out.w * op.d.c_out * op.d.k * op.d.k,
                 net, blk, opi);
    const unsigned xe = (unsigned)((size_t)N * op.in.h * op.in.w * op.cin_p);
    if (dw_tiles(op)) {
      if constexpr (sizeof(T) == 2) {
        const int th = (op.out.h + kDwTileH - 1) / kDwTileH, tw = (op.out.w + kDwTileW - 1) / kDwTileW;
        const dim3 grid(N * th * tw, (ncv + kDwTileCv - 1) / kDwTileCv);
#define PBD_DWT(K_) launch(c, dw_tile_kernel<K_, false>, grid, 256, 0, st, (const bf16_t*)x, (const bf16_t*)w, (bf16_t*)y, a, b, act, 0, \
    N, op.in.h, op.in.w, ncv, th, tw, xe * 2u, streams(op.out) ? 1 : 0)
        if (op.d.k == 3) PBD_DWT(3); else if (op.d.k == 5) PBD_DWT(5); else PBD_DWT(7);
#undef PBD_DWT
      }
      return;
    }
    if (dw_slides(op)) {
      const long nitem = (long)N * op.out.h * ((op.out.w + kDwSlide - 1) / kDwSlide) * ncv;
#define PBD_DWS(K_, S_) launch(c, dw_slide_kernel<T, K_, S_, kDwSlide, false>, grid_for(nitem), 256, 0, st, x, w, y, a, b, act, 0, \
    N, op.in.h, op.in.w, op.out.h, op.out.w, ncv, op.d.pad, xe)
      if (op.d.stride == 1) { if (op.d.k == 3) PBD_DWS(3, 1); else if (op.d.k == 5) PBD_DWS(5, 1); else PBD_DWS(7, 1); }
      else { if (op.d.k == 3) PBD_DWS(3, 2); else if (op.d.k == 5) PBD_DWS(5, 2); else PBD_DWS(7, 2); }
#undef PBD_DWS
      return;
    }
#define PBD_DWF(KK_) launch(c, dw_fwd_kernel<T, KK_>, grid_for(nvec), 256, 0, st, x, w, y, a, b, act, N, op.in.h, op.in.w, \
    op.out.h, op.out.w, ncv, op.d.k, op.d.stride, op.d.pad, xe)
    if (op.d.k == 3) PBD_DWF(9); else if (op.d.k == 5) PBD_DWF(25); else if (op.d.k == 7) PBD_DWF(49); else PBD_DWF(1);
#undef PBD_DWF
  }
  void dw_dgrad(const OpPlan& op, const T* dy, const T* w, T* dx, bool accumulate) {
    const int N = c->o.batch, ncv = op.cout_p / 8;
    const long nvec = (long)N * op.in.h * op.in.w * ncv;
    char cls[32];
    snprintf(cls, sizeof cls, "dw_dgrad%s_k%d", dw_tiles(op) ? "_tile" : dw_slides(op) ? (op.d.stride == 1 ? "_slide" : "_s2") : "", op.d.k);
    ProfScope ps(c, cls, bytes_of(op.in) + bytes_of(op.out), 2.0 * N * op.out.h * op.out.w * op.d.c_out * op.d.k * op.d.k,
                 net, blk, opi);
    const unsigned de = (unsigned)((size_t)N * op.out.h * op.out.w * op.cout_p);
    if (dw_tiles(op)) {
      if constexpr (sizeof(T) == 2) {
        const int th = (op.in.h + kDwTileH - 1) / kDwTileH, tw = (op.in.w + kDwTileW - 1) / kDwTileW;
        const dim3 grid(N * th * tw, (ncv + kDwTileCv - 1) / kDwTileCv);
#define PBD_DWT(K_) launch(c, dw_tile_kernel<K_, true>, grid, 256, 0, st, (const bf16_t*)dy, (const bf16_t*)w, (bf16_t*)dx, (const float*)nullptr, \
    (const float*)nullptr, 0, accumulate ? 1 : 0, N, op.out.h, op.out.w, ncv, th, tw, de * 2u, streams(op.in) ? 1 : 0)
        if (op.d.k == 3) PBD_DWT(3); else if (op.d.k == 5) PBD_DWT(5); else PBD_DWT(7);
#undef PBD_DWT
      }
      return;
    }
    if (dw_slides(op) && op.d.stride == 1) {   // mirrored filter over dy: same sliding sum
      const long nitem = (long)N * op.in.h * ((op.in.w + kDwSlide - 1) / kDwSlide) * ncv;
#define PBD_DWS(K_) launch(c, dw_slide_kernel<T, K_, 1, kDwSlide, true>, grid_for(nitem), 256, 0, st, dy, w, dx, (const float*)nullptr, \
    (const float*)nullptr, 0, accumulate ? 1 : 0, N, op.out.h, op.out.w, op.in.h, op.in.w, ncv, op.d.pad, de)
      if (op.d.k == 3) PBD_DWS(3); else if (op.d.k == 5) PBD_DWS(5); else PBD_DWS(7);
#undef PBD_DWS
      return;
    }
    if (dw_slides(op) && op.d.stride == 2) {   // only the taps whose parity matches the input pixel
#define PBD_DWD2(K_) launch(c, dw_dgrad_s2_kernel<T, K_>, grid_for(nvec), 256, 0, st, dy, w, dx, N, op.in.h, op.in.w, op.out.h, \
    op.out.w, ncv, op.d.pad, accumulate ? 1 : 0, de)
      if (op.d.k == 3) PBD_DWD2(3); else if (op.d.k == 5) PBD_DWD2(5); else PBD_DWD2(7);
#undef PBD_DWD2
      return;
    }
#define PBD_DWD(KK_) launch(c, dw_dgrad_kernel<T, KK_>, grid_for(nvec), 256, 0, st, dy, w, dx, N, op.in.h, op.in.w, op.out.h, \
    op.out.w, ncv, op.d.k, op.d.stride, op.d.pad, accumulate ? 1 : 0, de)
    if (op.d.k == 3) PBD_DWD(9); else if (op.d.k == 5) PBD_DWD(25); else if (op.d.k == 7) PBD_DWD(49); else PBD_DWD(1);
#undef PBD_DWD
  }
  void dw_wgrad(const OpPlan& op, const T* dy, const T* x, float* dw) {
    const int N = c->o.batch;
    const DwWgradCfg cfg = dw_wgrad_cfg(mfma(), N, op.out.h, op.out.w, op.cout_p, op.d.k, op.d.stride, op.d.pad);
    {
      char cls[32];
      snprintf(cls, sizeof cls, "dw_wgrad%s_k%d", cfg.tiled ? "_tile" : "", op.d.k <= 3 ? 3 : cfg.tiled ? op.d.k : 7);
      ProfScope ps(c, cls, bytes_of(op.in) + bytes_of(op.out),
                   2.0 * N * op.out.h * op.out.w * op.d.c_out * op.d.k * op.d.k, net, blk, opi);
      if (cfg.tiled) {
        if constexpr (sizeof(T) == 2) {
          const int ncv = op.cout_p / 8;
          const dim3 grid(cfg.chunks, (ncv + kDwTileCv - 1) / kDwTileCv);
          const unsigned bytes = (unsigned)((size_t)N * op.out.h * op.out.w * op.cout_p * 2);
#define PBD_DWW(K_) launch(c, dw_wgrad_tile_kernel<K_>, grid, 64 * K_, 0, st, (const bf16_t*)dy, (const bf16_t*)x, red(), N, op.out.h, \
    op.out.w, ncv, cfg.tiles_h, cfg.tiles_w, cfg.ntiles, cfg.tiles_per_block, bytes)
          if (op.d.k == 3) PBD_DWW(3); else if (op.d.k == 5) PBD_DWW(5); else PBD_DWW(7);
#undef PBD_DWW
        }
      } else {
        const ColGrid g = cfg.g;
        const size_t smem = 256 * 8 * sizeof(float) * (op.d.k <= 3 ? 3 : 7);
        if (op.d.k <= 3)
          launch(c, dw_wgrad_kernel<T, 3, 3>, dim3(g.slabs, g.chunks, 1), 256, smem, st,
              dy, x, red(), N, op.in.h, op.in.w, op.out.h, op.out.w, op.cout_p, op.d.k, op.d.stride, op.d.pad, g,
              (unsigned)((size_t)N * op.in.h * op.in.w * op.cin_p));
        else
          launch(c, dw_wgrad_kernel<T, 7, 1>, dim3(g.slabs, g.chunks, op.d.k), 256, smem, st,
              dy, x, red(), N, op.in.h, op.in.w, op.out.h, op.out.w, op.cout_p, op.d.k, op.d.stride, op.d.pad, g,
              (unsigned)((size_t)N * op.in.h * op.in.w * op.cin_p));
      }
    }
    ProfScope ps(c, "sum_partials", (double)(cfg.chunks + 1) * op.wn * 4, 0, net, blk, opi);
    sum_partials(red(), dw, (long)op.wn, cfg.chunks);
  }

  // ---- joins / pool -------------------------------------------------------
  void join_fwd(const OpPlan& op, const Join& j, T* z) {
    const long nvec = (long)c->o.batch * op.out.h * op.out.w * op.cout_p / 8;
    ProfScope ps(c, "join_fwd", bytes_of(op.out) * (j.n + 1), 0, net, blk, opi);
    launch(c, join_fwd_kernel<T>, grid_for(nvec), 256, 0, st, j, z, nvec, op.d.act);
  }
  // fold (optional): x is the producing layer's convolution output, normalised and activated as it is read
  void pool_fwd(const OpPlan& op, const T* x, T* z, uint8_t* idx, NormFold fold = NormFold{}) {
    const int N = c->o.batch, ncv = op.cout_p / 8;
    const long nvec = (long)N * op.out.h * op.out.w * ncv;
    ProfScope ps(c, fold.mean ? "bn_apply_maxpool" : "maxpool_fwd", bytes_of(op.in) + bytes_of(op.out) * (idx ? 1.5 : 1.0), 0, net, blk, opi);
    if (op.d.k == 3 && op.d.stride == 2 && op.d.pad == 1)
      launch(c, maxpool_fwd_k3s2_kernel<T>, grid_for(nvec), 256, 0, st, x, z, idx, N, op.in.h, op.in.w, op.out.h, op.out.w, ncv, fold);
    else
      launch(c, maxpool_fwd_kernel<T>, grid_for(nvec), 256, 0, st, x, z, idx, N, op.in.h, op.in.w, op.out.h, op.out.w, ncv,
                                                            op.d.k, op.d.stride, op.d.pad, fold);
  }

  // =========================================================================
  // teacher block b: inference mode, output straight into the relay store
  // =========================================================================
  void teacher_block(int b) {
    BlockPlan& bp = c->net[0][b];
    net = PBD_TEACHER; blk = b;
    auto value = [&](int v) -> T* {
      if (v == 0) return trelay(b);
      if (v + 1 == (int)bp.shapes.size()) return trelay(b + 1);
      return ws(c->r_tscr + bp.val[v]);
    };
    std::vector<char> fused(bp.ops.size(), 0);      // adds that rode in their producer's store
    for (size_t j = 0; j < bp.ops.size(); ++j) {
      const OpPlan& op = bp.ops[j];
      opi = (int)j;
      if (fused[j]) continue;
      T* out = value((int)j + 1);
      const T* x = value(op.d.in[0]);
      if (op.d.type == OP_CBA) {
        const T* w = ws(op.t_w);
        const int rd = residual_reader(bp, (int)j);
        if (op.dw) dw_fwd(op, x, w, out, wsf(op.t_a), wsf(op.t_b), op.d.act);
        else if (rd >= 0 && fuses_residual(op)) {
          const OpD& q = bp.ops[rd].d;
          conv_fwd(op, x, w, value(rd + 1), wsf(op.t_a), wsf(op.t_b), op.d.act,
                   value(q.in[0] == (int)j + 1 ? q.in[1] : q.in[0]), q.act);
          fused[rd] = 1;
        } else conv_fwd(op, x, w, out, wsf(op.t_a), wsf(op.t_b), op.d.act);
      } else if (op.d.type == OP_POOL) {
        pool_fwd(op, x, out, nullptr);
      } else {
        Join jn{};
        jn.n = op.d.nin;
        for (int k = 0; k < op.d.nin; ++k) {
          jn.src[k] = value(op.d.in[k]);
          jn.p[k] = op.d.type == OP_MIX ? (float)c->pool[op.d.pofs + k] : 1.f;
        }
        join_fwd(op, jn, out);
      }
    }
  }

  void fold_teacher_bn() {
    for (BlockPlan& bp : c->net[0])
      for (OpPlan& op : bp.ops)
        if (op.d.type == OP_CBA)
          launch(c, bn_fold_kernel, (op.cout_p + 255) / 256, 256, 0, st, wsf(op.t_gamma), wsf(op.t_beta), wsf(op.t_rmean),
                                                                  wsf(op.t_rvar), wsf(op.t_a), wsf(op.t_b), op.cout_p,
                                                                  c->o.bn_eps);
    // the stems that run on the space-to-depth input: their filters in that layout
    for (OpPlan& op : c->net[0][0].ops)
      if (op.s2d)
        launch(c, pack_stem_weights_kernel<T>, (op.d.c_out * kS2dK + 255) / 256, 256, 0, st,
               reinterpret_cast<const T*>(c->ws + op.t_w), reinterpret_cast<T*>(c->ws + op.w2), op.d.c_out, op.in.c);
    c->fold_dirty = false;
  }

  void set_lr(float lr) { launch(c, set_scalar_kernel, 1, 1, 0, st, wsf(c->lr_off), lr); }

  // everything a step needs that depends on the caller's pointers or on freshly loaded parameters
  void prepare(const float* x_dev) {
    if (c->fold_dirty) fold_teacher_bn();
    for (int b = 0; b < c->B; ++b) {
      net = PBD_STUDENT; blk = b;
      if (c->net[1][b].dirty) refresh_compute_copies(c->net[1][b]);
    }
    cast_input(x_dev);
  }
  void cast_input(const float* x_dev) {
    {
      const Shape s = c->act[0];
      const long nvec = (long)c->o.batch * s.h * s.w * round8(s.c) / 8;
      net = PBD_TEACHER; blk = -1; opi = -1;
      ProfScope ps(c, "cast_input", (double)c->o.batch * s.c * s.h * s.w * 4 + bytes_of(s), 0, net, blk, opi);
      launch(c, cast_input_kernel<T>, grid_for(nvec), 256, 0, st, x_dev, trelay(0), c->o.batch, s.c, s.h * s.w, round8(s.c));
    }
    if (c->s2d_off != (size_t)-1) {
      const Shape s = c->act[0];
      const long npix = (long)c->o.batch * (s.h / 2) * (s.w / 2);
      ProfScope ps(c, "cast_input_s2d", (double)c->o.batch * s.c * s.h * s.w * 4 + (double)npix * 16 * sizeof(T), 0, net, blk, opi);
      launch(c, s2d_input_kernel<T>, grid_for(npix), 256, 0, st, x_dev, ws((tset ? c->r_relay2 : c->r_relay) + c->s2d_off),
             c->o.batch, s.c, s.h, s.w);
    }
  }
  void relay_all(const float* x_dev) { relay_prefix(x_dev, c->B); }
  // T_1..T_upto from the input: the whole relay, or what a worker of the baseline without relaying
  // runs before it can train block `upto` (Sec. III)
  void relay_prefix(const float* x_dev, int upto) {
    if (c->fold_dirty) fold_teacher_bn();
    cast_input(x_dev);
    for (int b = 0; b < upto; ++b) teacher_block(b);
    c->relayed_upto = upto;
  }
  // the pointer-independent body of a step: T_1..T_B once each, then every student block
  // With `fork` (graph capture, disjoint scratch) student block b runs on its own stream as soon as
  // T_b has produced its target, next to T_{b+1}: the one-device form of the overlap of Sec. IV-A.
  void step_body(bool fork, bool arch = false) {
    hipStream_t main = st;
    for (int b = 0; b < c->B; ++b) {
      teacher_block(b);
      if (fork) {
        (void)hipEventRecord(c->ev_fork[b], main);
        (void)hipStreamWaitEvent(c->side[b], c->ev_fork[b], 0);
        st = c->side[b];
        student_block(b, wsf(c->loss_off) + b, arch);
        (void)hipEventRecord(c->ev_join[b], st);
        st = main;
      }
    }
    for (int b = 0; b < c->B; ++b) {
      if (fork) (void)hipStreamWaitEvent(main, c->ev_join[b], 0);
      else student_block(b, wsf(c->loss_off) + b, arch);
    }
    c->relayed_upto = c->B;
  }
  // One stage of the pipeline over steps (Sec. IV-A and IV-B: with the updates decoupled, the teacher
  // goes on to the next batch while the students still train on the last one): the teacher relays the
  // new batch into copy `tset` of the store; the students train on the batch in copy `sset`.  Nothing
  // of one depends on the other, so with `fork` every student block and the teacher chain start together.
  void pipe_body(bool fork, bool teacher = true) {
    hipStream_t main = st;
    if (fork) {
      (void)hipEventRecord(c->ev_fork[0], main);
      // The branches are independent, so any order of capture gives the same results; it decides how the
      // replayed graph's branches share the hardware queues, and with that the step time (a few per cent).
      for (int i = 0; i <= c->B; ++i) {
        const int b = (int)c->pipe_order.size() == c->B + 1 ? c->pipe_order[i] : i;
        if (b == c->B) {
          st = main;
          if (teacher)
            for (int t = 0; t < c->B; ++t) teacher_block(t);
          teacher = false;
          continue;
        }
        (void)hipStreamWaitEvent(c->side[b], c->ev_fork[0], 0);
        st = c->side[b];
        student_block(b, wsf(c->loss_off) + b);
        (void)hipEventRecord(c->ev_join[b], st);
      }
      st = main;
    }
    if (teacher)
      for (int b = 0; b < c->B; ++b) teacher_block(b);
    for (int b = 0; b < c->B; ++b) {
      if (fork) (void)hipStreamWaitEvent(main, c->ev_join[b], 0);
      else student_block(b, wsf(c->loss_off) + b);
    }
  }

  // =========================================================================
  // student block b = i-1: forward, loss, backward, update
  // =========================================================================
  void refresh_compute_copies(BlockPlan& bp) {
    if constexpr (sizeof(T) == 2) {
      launch(c, cast_params_kernel, grid_for((long)bp.arena_elems / 4), 256, 0, st, wsf(bp.master), (bf16_t*)ws(bp.wc),
                                                                             (long)bp.arena_elems / 4);
    }
    transpose_weights(bp);
    bp.dirty = false;
  }
  void transpose_weights(BlockPlan& bp) {
    for (OpPlan& op : bp.ops)
      if (op.s2d)
        launch(c, pack_stem_weights_kernel<T>, (op.d.c_out * kS2dK + 255) / 256, 256, 0, st, ws(bp.wc) + op.e_w,
               reinterpret_cast<T*>(c->ws + op.w2), op.d.c_out, op.in.c);
    if (bp.ttable.empty()) return;
    ProfScope ps(c, "transpose_weights", 2.0 * bp.wt_elems * sizeof(T), 0, net, blk, -1);
    dim3 grid(64, (unsigned)bp.ttable.size());
    launch(c, transpose_weights_kernel<T>, grid, 256, 0, st, ws(bp.wc), ws(bp.wt),
                                                      reinterpret_cast<const TransposeEntry*>(c->ws + bp.table));
  }

  // arch: the architecture round (Sec. VI-A, neural architecture search) - same forward and loss;
  // the backward reaches every mix op, forms dL/dalpha there and trains alpha; weights stay frozen
  void student_block(int b, float* loss_dev, bool arch = false) {
    BlockPlan& bp = c->net[1][b];
    net = PBD_STUDENT; blk = b;
    if (bp.dirty) refresh_compute_copies(bp);
    const int N = c->o.batch;
    const size_t scr = bp.scr_off;
    red_off = bp.red_off;
    auto value = [&](int v) -> T* { return v == 0 ? srelay(b) : ws(scr + bp.val[v]); };
    auto dvalue = [&](int v) -> T* { return ws(scr + bp.dval[v]); };
    T* wc = ws(bp.wc);
    float* grad = wsf(bp.grad);
    const float* master = wsf(bp.master);
    const int nval = (int)bp.shapes.size();
    auto mix_state = [&](const OpPlan& op) -> float* { return wsf(bp.mix) + (size_t)op.mix_slot * kMixState; };

    // ---- forward ----------------------------------------------------------
    std::vector<char> fused(bp.ops.size(), 0);      // adds that rode in their producer's normalisation pass
    for (size_t j = 0; j < bp.ops.size(); ++j) {
      const OpPlan& op = bp.ops[j];
      opi = (int)j;
      if (fused[j]) continue;
      T* z = value((int)j + 1);
      const T* x = value(op.d.in[0]);
      if (op.d.type == OP_CBA) {
        T* y = ws(scr + op.y);
        const int stat_tiles = op.dw ? 0 : fused_stats_tiles(op);
        if (op.dw) dw_fwd(op, x, wc + op.e_w, y, nullptr, nullptr, 0);
        else conv_fwd(op, x, wc + op.e_w, y, nullptr, nullptr, 0, nullptr, 0, stat_tiles ? red() : nullptr);
        const long M = (long)N * op.out.h * op.out.w;
        if (short_column(M)) {
          ProfScope ps(c, "bn_small_fwd", 3 * bytes_of(op.out), 0, net, blk, opi);
          launch(c, bn_small_fwd_kernel<T>, op.cout_p / 8, kSmallThreads, 0, st, y, z, master + op.e_gamma,
                 master + op.e_beta, wsf(op.s_mean), wsf(op.s_invstd), wsf(op.s_rmean), wsf(op.s_rvar), (int)M,
                 op.cout_p, c->o.bn_eps, c->o.bn_momentum, op.d.act, (unsigned)(M * op.cout_p * sizeof(T)));
        } else {
          const float* part = red();
          const T* pivot = y;                       // the pass of its own shifts by the first row
          int chunks = stat_tiles;
          if (stat_tiles) {
            // the convolution's store left one pair of sums per row tile (no pivot); thousands of them are
            // first summed in groups so that the finalize kernel's walk stays short
            pivot = nullptr;
            if (chunks > kStatGroupsMax) {
              const int per = (chunks + kStatGroupsMax - 1) / kStatGroupsMax, n = 2 * op.cout_p;
              float* out = red() + (size_t)chunks * n;
              const int groups = (chunks + per - 1) / per;
              launch(c, regroup_partials_kernel, dim3((n + 255) / 256, groups), 256, 0, st, part, out, chunks, n, per);
              part = out; chunks = groups;
            }
          } else {
            const ColGrid g = bn_stats_grid(M, op.cout_p);
            ProfScope ps(c, streams(op.out) ? "bn_stats_nt" : "bn_stats", bytes_of(op.out), 0, net, blk, opi);
            launch(c, streams(op.out) ? bn_stats_kernel<T, true> : bn_stats_kernel<T, false>, dim3(g.slabs, g.chunks), 256,
                   256 * 16 * sizeof(float), st, y, red(), M, op.cout_p, g);
            chunks = g.chunks;
          }
          launch(c, bn_finalize_kernel<T>, op.cout_p / kFinalizeChannels, 256, 0, st, 
              part, pivot, chunks, op.cout_p, (double)M, wsf(op.s_mean), wsf(op.s_invstd), wsf(op.s_rmean),
              wsf(op.s_rvar), c->o.bn_eps, c->o.bn_momentum);
          if (pool_reader(bp, (int)j, N) < 0) {
            const ColGrid ga = col_grid(M, op.cout_p, 8, 4096);   // elementwise pass: many short workgroups
            // a residual add that only reads this layer's output rides along: the normalised tensor itself
            // is never written (the backward pass needs y and the sum, not it)
            const int rd = residual_reader(bp, (int)j);
            const T* res = nullptr;
            int res_act = 0;
            if (rd >= 0) {
              const OpD& q = bp.ops[rd].d;
              res = value(q.in[0] == (int)j + 1 ? q.in[1] : q.in[0]);
              res_act = q.act;
              z = value(rd + 1);
              fused[rd] = 1;
            }
            const bool nt = streams(op.out);    // (profile classes: one per kernel instantiation)
            ProfScope ps(c, res ? (nt ? "bn_apply_add_nt" : "bn_apply_add") : (nt ? "bn_apply_nt" : "bn_apply"), (res ? 3 : 2) * bytes_of(op.out), 0, net, blk, opi);
            launch(c, streams(op.out) ? bn_apply_kernel<T, true> : bn_apply_kernel<T, false>, dim3(ga.slabs, ga.chunks), 256, 0, st, y, z, wsf(op.s_mean), wsf(op.s_invstd),
                                                                       master + op.e_gamma, master + op.e_beta, M,
                                                                       op.cout_p, op.d.act, ga, res, res_act);
          }
        }
      } else if (op.d.type == OP_POOL) {
        const int pv = op.d.in[0];
        if (pv >= 1 && pool_reader(bp, pv - 1, N) == (int)j) {
          const OpPlan& p = bp.ops[pv - 1];
          pool_fwd(op, ws(scr + p.y), z, reinterpret_cast<uint8_t*>(c->ws + scr + op.idx),
                   NormFold{wsf(p.s_mean), wsf(p.s_invstd), master + p.e_gamma, master + p.e_beta, p.d.act});
        } else pool_fwd(op, x, z, reinterpret_cast<uint8_t*>(c->ws + scr + op.idx));
      } else {
        Join jn{};
        jn.n = op.d.nin;
        for (int k = 0; k < op.d.nin; ++k) {
          jn.src[k] = value(op.d.in[k]);
          jn.p[k] = 1.f;
        }
        if (op.d.type == OP_MIX) jn.pdev = mix_state(op) + kMixP;
        join_fwd(op, jn, z);
      }
    }

    // ---- loss and its gradient (fused) -----------------------------------
    // A block that ends in an add whose backward pass rides in a batch-norm reduction (below): that reduction also
    // forms the loss and its gradient from the block's output and the teacher's activation.
    const Shape s_out = bp.shapes.back();
    const long numel = (long)N * s_out.h * s_out.w * s_out.c;   // outputs have no padded channels
    const int last = (int)bp.ops.size() - 1;
    const bool loss_rides = !arch && last >= 1 && bp.ops[last].d.type == OP_ADD && residual_reader(bp, last - 1) == last &&
                            !short_column((long)N * s_out.h * s_out.w);
    if (!loss_rides) {
      const long nvec = (long)N * s_out.h * s_out.w * round8(s_out.c) / 8;
      const int nb = (int)std::min<long>(kMseBlocks, (nvec + 255) / 256);
      opi = -1;
      ProfScope ps(c, "mse_loss_grad", 3 * bytes_of(s_out), 0, net, blk, opi);
      launch(c, mse_kernel<T>, nb, 256, 0, st, value(nval - 1), srelay(b + 1), dvalue(nval - 1), red(), nvec, (float)(2.0 / (double)numel));
      launch(c, mse_final_kernel, 1, 256, 0, st, red(), nb, 1.0 / (double)numel, loss_dev);
    }

    // ---- backward ---------------------------------------------------------
    std::vector<char> have(nval, 0);
    have[nval - 1] = 1;
    // wanted[v]: the gradient of value v is needed.  Weight round: every value but the block's input.
    // Architecture round: only values that have a mix op at or above them.
    std::vector<char> wanted(nval, 1);
    wanted[0] = 0;
    if (arch)
      for (int j = 0; j < (int)bp.ops.size(); ++j) {
        const OpD& o = bp.ops[j].d;
        char w = o.type == OP_MIX;
        for (int k = 0; k < (o.type == OP_ADD || o.type == OP_MIX ? o.nin : 1); ++k) w |= wanted[o.in[k]];
        wanted[j + 1] = w;
      }
    // An add whose backward pass rides in the batch-norm backward of the layer right before it (the one whose
    // normalisation pass carried the add on the way forward): that layer's reduction reads the add's output
    // gradient, masks it and stores the result once, where the add's other input collects its gradient.
    struct AddBwd { const T* dz; const T* z; int act; T* dstore; bool loss; };
    std::vector<AddBwd> add_bwd(bp.ops.size(), AddBwd{nullptr, nullptr, 0, nullptr, false});
    for (int j = (int)bp.ops.size() - 1; j >= 0; --j) {
      const OpPlan& op = bp.ops[j];
      opi = j;
      if (!have[j + 1]) continue;
      T* dz = dvalue(j + 1);
      const int iv = op.d.in[0];
      if (op.d.type == OP_ADD && !arch && j >= 1 && residual_reader(bp, j - 1) == j &&
          !short_column((long)N * op.out.h * op.out.w)) {
        const int other = op.d.in[0] == j ? op.d.in[1] : op.d.in[0];
        if (!wanted[other] || !have[other]) {      // (a gradient already there would have to be added to, not replaced)
          const bool loss = loss_rides && j == last;   // (dz: the teacher's activation instead of a gradient)
          add_bwd[j - 1] = AddBwd{loss ? srelay(b + 1) : dz, op.d.act != ACT_NONE || loss ? value(j + 1) : nullptr, op.d.act,
                                  wanted[other] ? dvalue(other) : dvalue(j), loss};
          if (wanted[other]) have[other] = 1;
          have[j] = 1;
          continue;
        }
      }
      if (op.d.type == OP_CBA) {
        if (arch && !wanted[iv]) continue;   // frozen weights and nothing trainable above: nothing to do
        const T* y = ws(scr + op.y);
        const long M = (long)N * op.out.h * op.out.w;
        const AddBwd ab = add_bwd[j];
        const T* dz_in = ab.dz ? ab.dstore : dz;     // what the last stage reads (dz: in place)
        if (short_column(M)) {
          ProfScope ps(c, "bn_small_bwd", 5 * bytes_of(op.out), 0, net, blk, opi);
          launch(c, bn_small_bwd_kernel<T>, op.cout_p / 8, kSmallThreads, 0, st, dz, y, master + op.e_gamma,
                 master + op.e_beta, wsf(op.s_mean), wsf(op.s_invstd), grad + op.e_gamma, grad + op.e_beta, (int)M,
                 op.cout_p, op.d.act, (unsigned)(M * op.cout_p * sizeof(T)));
        } else {
          const ColGrid g = bn_bwd_grid(M, op.cout_p);
          if (ab.loss) {
            float* loss_part = red() + (size_t)g.chunks * 2 * op.cout_p;
            {
              ProfScope ps(c, streams(op.out) ? "bn_bwd_reduce_add_mse_nt" : "bn_bwd_reduce_add_mse", 4 * bytes_of(op.out), 0, net, blk, opi);
              launch(c, streams(op.out) ? bn_bwd_reduce_kernel<T, true, true, true> : bn_bwd_reduce_kernel<T, true, true, false>,
                  dim3(g.slabs, g.chunks), 256, 256 * 16 * sizeof(float), st,
                  ab.dz, y, master + op.e_gamma, master + op.e_beta, wsf(op.s_mean), wsf(op.s_invstd), red(), M, op.cout_p,
                  op.d.act, g, ab.z, ab.act, ab.dstore, loss_part, (float)(2.0 / (double)numel));
            }
            launch(c, mse_final_kernel, 1, 256, 0, st, loss_part, g.slabs * g.chunks, 1.0 / (double)numel, loss_dev);
          } else if (ab.dz) {
            ProfScope ps(c, streams(op.out) ? "bn_bwd_reduce_add_nt" : "bn_bwd_reduce_add", (ab.z ? 4 : 3) * bytes_of(op.out), 0, net, blk, opi);
            launch(c, streams(op.out) ? bn_bwd_reduce_kernel<T, true, false, true> : bn_bwd_reduce_kernel<T, true, false, false>,
                dim3(g.slabs, g.chunks), 256, 256 * 16 * sizeof(float), st,
                ab.dz, y, master + op.e_gamma, master + op.e_beta, wsf(op.s_mean), wsf(op.s_invstd), red(), M, op.cout_p,
                op.d.act, g, ab.z, ab.act, ab.dstore, (float*)nullptr, 0.f);
          } else {
            ProfScope ps(c, streams(op.out) ? "bn_bwd_reduce_nt" : "bn_bwd_reduce", 2 * bytes_of(op.out), 0, net, blk, opi);
            launch(c, streams(op.out) ? bn_bwd_reduce_kernel<T, false, false, true> : bn_bwd_reduce_kernel<T, false, false, false>,
                dim3(g.slabs, g.chunks), 256, 256 * 16 * sizeof(float), st,
                (const T*)dz, y, master + op.e_gamma, master + op.e_beta, wsf(op.s_mean), wsf(op.s_invstd), red(), M, op.cout_p,
                op.d.act, g, (const T*)nullptr, 0, (T*)nullptr, (float*)nullptr, 0.f);
          }
          launch(c, bn_bwd_finalize_kernel, op.cout_p / kFinalizeChannels, 256, 0, st, red(), g.chunks, op.cout_p, (double)M,
                                                                           grad + op.e_gamma, grad + op.e_beta,
                                                                           wsf(op.s_k2), wsf(op.s_k3));
          {
            const ColGrid ga = col_grid(M, op.cout_p, 8, 4096);
            ProfScope ps(c, streams(op.out) ? "bn_bwd_apply_nt" : "bn_bwd_apply", 3 * bytes_of(op.out), 0, net, blk, opi);
            launch(c, streams(op.out) ? bn_bwd_apply_kernel<T, true> : bn_bwd_apply_kernel<T, false>, dim3(ga.slabs, ga.chunks), 256, 0, st,
                dz_in, dz, y, master + op.e_gamma, master + op.e_beta, wsf(op.s_mean), wsf(op.s_invstd), wsf(op.s_k2),
                wsf(op.s_k3), M, op.cout_p, op.d.act, ga);
          }
        }
        const T* x = value(iv);
        if (!arch) {
          if (op.dw) dw_wgrad(op, dz, x, grad + op.e_w);
          else conv_wgrad(op, dz, x, grad + op.e_w);
        }
        if (wanted[iv]) {  // A_{i-1} is a constant: no backward-data for the block's first layer
          if (op.dw) dw_dgrad(op, dz, wc + op.e_w, dvalue(iv), have[iv]);
          else conv_dgrad(op, dz, wc + op.e_w, op.e_wt >= 0 ? ws(bp.wt) + op.e_wt : nullptr, dvalue(iv), have[iv]);
          have[iv] = 1;
        }
      } else if (op.d.type == OP_POOL) {
        if (wanted[iv]) {
          const int ncv = op.cout_p / 8;
          const long nvec = (long)N * op.in.h * op.in.w * ncv;
          ProfScope ps(c, "maxpool_bwd", bytes_of(op.in) + 1.5 * bytes_of(op.out), 0, net, blk, opi);
          if (op.d.k == 3 && op.d.stride == 2 && op.d.pad == 1)
            launch(c, maxpool_bwd_k3s2_kernel<T>, grid_for(nvec), 256, 0, st, (const T*)dz, reinterpret_cast<const uint8_t*>(c->ws + scr + op.idx),
                   dvalue(iv), N, op.in.h, op.in.w, op.out.h, op.out.w, ncv, have[iv] ? 1 : 0);
          else
            launch(c, maxpool_bwd_kernel<T>, grid_for(nvec), 256, 0, st, dz, reinterpret_cast<const uint8_t*>(c->ws + scr + op.idx),
                                                                  dvalue(iv), N, op.in.h, op.in.w, op.out.h, op.out.w,
                                                                  ncv, op.d.k, op.d.stride, op.d.pad, have[iv] ? 1 : 0);
          have[iv] = 1;
        }
      } else {
        Join jn{};
        jn.n = op.d.nin;
        int live = 0;
        for (int k = 0; k < op.d.nin; ++k) {
          const int v = op.d.in[k];
          jn.p[k] = 1.f;
          jn.src[k] = value(v);
          jn.dst[k] = wanted[v] ? dvalue(v) : nullptr;
          jn.accumulate[k] = wanted[v] && have[v];
          if (wanted[v]) { have[v] = 1; ++live; }
        }
        const long nvec = (long)N * op.out.h * op.out.w * op.cout_p / 8;
        if (op.d.type == OP_MIX) jn.pdev = mix_state(op) + kMixP;
        const bool train_alpha = arch && op.d.type == OP_MIX;
        const int nb = (int)std::min<long>(kMixDotBlocks, (nvec + 255) / 256);
        if (train_alpha) {
          ProfScope ps(c, "mix_dot", bytes_of(op.out) * (op.d.nin + 1 + (op.d.act ? 1 : 0)), 0, net, blk, opi);
          launch(c, mix_dot_kernel<T>, nb, 256, 0, st, jn, dz, value(j + 1), red(), nvec, op.d.act);
        }
        if (live) {
          ProfScope ps(c, "join_bwd", bytes_of(op.out) * (live + 1 + (op.d.act ? 1 : 0)), 0, net, blk, opi);
          launch(c, join_bwd_kernel<T>, grid_for(nvec), 256, 0, st, jn, dz, value(j + 1), nvec, op.d.act);
        }
        // after the last reader of this round's p: gradient, momentum step and the new softmax
        if (train_alpha)
          launch(c, mix_alpha_update_kernel, 1, 256, 0, st, red(), nb, mix_state(op), op.d.nin, wsf(c->lr_off), c->o.momentum, 1);
      }
    }

    // ---- decoupled update of this block only -----------------------------
    if (!arch) {
      opi = -1;
      const long n4 = (long)bp.arena_elems / 4;
      ProfScope ps(c, "sgd_momentum", (double)bp.arena_elems * (20 + (sizeof(T) == 2 ? 2 : 0)), 0, net, blk, opi);
      if constexpr (sizeof(T) == 2)
        launch(c, sgd_momentum_kernel<bf16_t>, grid_for(n4), 256, 0, st, wsf(bp.master), wsf(bp.mom), grad, (bf16_t*)wc, n4, wsf(c->lr_off), c->o.momentum);
      else
        launch(c, sgd_momentum_kernel<bf16_t>, grid_for(n4), 256, 0, st, wsf(bp.master), wsf(bp.mom), grad, nullptr, n4, wsf(c->lr_off), c->o.momentum);
      transpose_weights(bp);
    }
    red_off = c->r_tred;
    if (!c->concurrent)
      for (BlockPlan& other : c->net[1]) other.stepped = false;   // shared scratch was overwritten
    bp.stepped = true;
  }
};

// ---------------------------------------------------------------------------
// host <-> device tensor marshalling (textbook layouts on the host side)
// ---------------------------------------------------------------------------
inline uint16_t f2bf(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
inline float bf2f(uint16_t h) {
  const uint32_t u = (uint32_t)h << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

// textbook index of physical weight element e (or -1 for a padded channel)
long weight_host_index(const OpPlan& op, size_t e) {
  const int k = op.d.k;
  if (op.dw) {
    const int c = (int)(e % op.cout_p);
    const int rs = (int)(e / op.cout_p);
    if (c >= op.d.c_out) return -1;
    return (long)c * k * k + rs;
  }
  const int c = (int)(e % op.cin_p);
  size_t t = e / op.cin_p;
  const int rs = (int)(t % (k * k));
  const int ko = (int)(t / (k * k));
  if (c >= op.in.c) return -1;
  return ((long)ko * op.in.c + c) * k * k + rs;
}

int check_ready(pbd_ctx* c) {
  if (!c) return PBD_EINVAL;
  if (!c->bound) return fail(c, PBD_ESTATE, "no workspace bound (call pbd_bind first)");
  return PBD_OK;
}

int after_launches(pbd_ctx* c) {
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(c, PBD_EHIP, "kernel launch failed: %s", hipGetErrorString(e));
  return PBD_OK;
}

OpPlan* find_cba(pbd_ctx* c, int net, int b, int op) {
  if (net < 0 || net > 1 || b < 0 || b >= c->B) return nullptr;
  if (op < 0 || op >= (int)c->net[net][b].ops.size()) return nullptr;
  OpPlan* p = &c->net[net][b].ops[op];
  return p->d.type == OP_CBA ? p : nullptr;
}

// device address, element type (0 f32, 1 bf16) and sizes of one addressed tensor
struct TensorRef { char* ptr; bool bf; bool weight; size_t phys; size_t logical; };
int locate(pbd_ctx* c, int kind, int net, int b, int opi, int slot, TensorRef& t) {
  OpPlan* op = find_cba(c, net, b, opi);
  if (!op) return fail(c, PBD_EINVAL, "no conv+BN operation at net %d block %d op %d", net, b, opi);
  if (slot < PBD_WEIGHT || slot > PBD_RVAR) return fail(c, PBD_EINVAL, "slot %d out of range", slot);
  if (kind < PBD_PARAM || kind > PBD_MOMENTUM) return fail(c, PBD_EINVAL, "kind %d out of range", kind);
  if (kind != PBD_PARAM && (net != PBD_STUDENT || slot > PBD_BETA))
    return fail(c, PBD_EINVAL, "gradients and momentum exist for student weight/gamma/beta only");
  t.weight = slot == PBD_WEIGHT;
  t.phys = t.weight ? op->wn : (size_t)op->cout_p;
  t.logical = t.weight ? (size_t)op->d.c_out * (op->in.c / op->d.groups) * op->d.k * op->d.k : (size_t)op->d.c_out;
  t.bf = false;
  if (net == PBD_TEACHER) {
    const size_t off[5] = {op->t_w, op->t_gamma, op->t_beta, op->t_rmean, op->t_rvar};
    t.ptr = c->ws + off[slot];
    t.bf = t.weight && c->o.precision == PBD_BF16;
  } else {
    BlockPlan& bp = c->net[1][b];
    if (slot <= PBD_BETA) {
      const size_t base = kind == PBD_PARAM ? bp.master : (kind == PBD_GRAD ? bp.grad : bp.mom);
      const size_t e = slot == PBD_WEIGHT ? op->e_w : (slot == PBD_GAMMA ? op->e_gamma : op->e_beta);
      t.ptr = c->ws + base + e * 4;
    } else {
      t.ptr = c->ws + (slot == PBD_RMEAN ? op->s_rmean : op->s_rvar);
    }
  }
  return PBD_OK;
}

int upload(pbd_ctx* c, const TensorRef& t, const OpPlan& op, const float* host) {
  std::vector<float> phys(t.phys, 0.f);
  for (size_t e = 0; e < t.phys; ++e) {
    const long h = t.weight ? weight_host_index(op, e) : ((long)e < (long)t.logical ? (long)e : -1);
    if (h >= 0) phys[e] = host[h];
  }
  if (t.bf) {
    std::vector<uint16_t> h16(t.phys);
    for (size_t e = 0; e < t.phys; ++e) h16[e] = f2bf(phys[e]);
    HIP_TRY(c, hipMemcpyAsync(t.ptr, h16.data(), t.phys * 2, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
  } else {
    HIP_TRY(c, hipMemcpyAsync(t.ptr, phys.data(), t.phys * 4, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
  }
  return PBD_OK;
}

// NHWC (Cp) device tensor -> NCHW float host
int download_act(pbd_ctx* c, const char* dev, Shape s, float* host) {
  const int N = c->o.batch, cp = round8(s.c);
  const size_t n = (size_t)N * s.h * s.w * cp;
  std::vector<float> f(n);
  if (c->esz == 2) {
    std::vector<uint16_t> h16(n);
    HIP_TRY(c, hipMemcpyAsync(h16.data(), dev, n * 2, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    for (size_t i = 0; i < n; ++i) f[i] = bf2f(h16[i]);
  } else {
    HIP_TRY(c, hipMemcpyAsync(f.data(), dev, n * 4, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
  }
  const size_t hw = (size_t)s.h * s.w;
  for (int nn = 0; nn < N; ++nn)
    for (size_t p = 0; p < hw; ++p)
      for (int ch = 0; ch < s.c; ++ch)
        host[((size_t)nn * s.c + ch) * hw + p] = f[((size_t)nn * hw + p) * cp + ch];
  return PBD_OK;
}

template <class F> int dispatch(pbd_ctx* c, F&& f) {
  if (c->o.precision == PBD_BF16) { Exec<bf16_t> e(c); f(e); }
  else { Exec<float> e(c); f(e); }
  return after_launches(c);
}

// A_i in the copy of the relay store that the teacher wrote last
char* relay_ptr(pbd_ctx* c, int i) { return c->ws + (c->front ? c->r_relay2 : c->r_relay) + c->act_off[i]; }

// the calls that run one step at a time refuse to work while a pipelined batch is in flight
int check_idle(pbd_ctx* c) {
  int rc = check_ready(c);
  if (rc) return rc;
  if (c->pending) return fail(c, PBD_ESTATE, "a pipelined batch waits for its students (call pbd_pipeline_flush first)");
  return PBD_OK;
}

int check_view(pbd_ctx* c, const pbd_tensor* t, int i, const char* what) {
  if (!t) return fail(c, PBD_EINVAL, "%s is null", what);
  const Shape s = c->act[i];
  if (t->ptr != relay_ptr(c, i) || t->n != c->o.batch || t->c != s.c || t->h != s.h ||
      t->w != s.w || t->c_phys != round8(s.c) || t->dtype != c->o.precision)
    return fail(c, PBD_ESHAPE, "%s is not the relayed activation A_%d", what, i);
  return PBD_OK;
}

const OpPlan* find_mix(pbd_ctx* c, int b, int op) {
  if (b < 0 || b >= c->B) return nullptr;
  const BlockPlan& bp = c->net[1][b];
  if (op < 0 || op >= (int)bp.ops.size() || bp.ops[op].d.type != OP_MIX) return nullptr;
  return &bp.ops[op];
}
char* mix_record(pbd_ctx* c, int b, const OpPlan& op) {
  return c->ws + c->net[1][b].mix + (size_t)op.mix_slot * kMixState * sizeof(float);
}

// Before the first architecture round of block b: alpha_k = ln p_k of the descriptor's weights, which
// must then be probabilities (the round differentiates p = softmax(alpha)).
int define_alpha(pbd_ctx* c, int b) {
  BlockPlan& bp = c->net[1][b];
  for (size_t j = 0; j < bp.ops.size(); ++j) {
    const OpPlan& op = bp.ops[j];
    if (op.d.type != OP_MIX || bp.alpha_defined[op.mix_slot]) continue;
    double sum = 0.0;
    float a[8] = {};
    for (int k = 0; k < op.d.nin; ++k) {
      const double pk = c->pool[op.d.pofs + k];
      if (!(pk > 0.0)) return fail(c, PBD_ESTATE, "block %d op %zu: mix weight %d is not positive; load alpha first", b + 1, j, k);
      sum += pk;
      a[k] = (float)std::log(pk);
    }
    if (std::fabs(sum - 1.0) > 1e-6)
      return fail(c, PBD_ESTATE, "block %d op %zu: mix weights sum to %g, not 1; load alpha first", b + 1, j, sum);
    HIP_TRY(c, hipMemcpyAsync(mix_record(c, b, op) + kMixAlpha * sizeof(float), a, sizeof a, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    bp.alpha_defined[op.mix_slot] = 1;
  }
  return PBD_OK;
}

void fill_view(pbd_ctx* c, int i, pbd_tensor* t) {
  const Shape s = c->act[i];
  t->ptr = relay_ptr(c, i);
  t->n = c->o.batch; t->c = s.c; t->h = s.h; t->w = s.w;
  t->c_phys = round8(s.c);
  t->dtype = c->o.precision;
}

// One stream and two events per student block for the forked capture; false if they cannot be had.
bool side_streams(pbd_ctx* c) {
  bool ok = c->concurrent;
  if (ok && c->side.empty()) {
    for (int b = 0; b < c->B && ok; ++b) {
      hipStream_t s2; hipEvent_t e1, e2;
      ok = hipStreamCreateWithFlags(&s2, hipStreamNonBlocking) == hipSuccess &&
           hipEventCreateWithFlags(&e1, hipEventDisableTiming) == hipSuccess &&
           hipEventCreateWithFlags(&e2, hipEventDisableTiming) == hipSuccess;
      if (ok) { c->side.push_back(s2); c->ev_fork.push_back(e1); c->ev_join.push_back(e2); }
    }
  }
  return ok && (int)c->side.size() == c->B;
}

// The whole step in one of its two rounds (r = 0: weights, 1: architecture parameters).
int whole_step(pbd_ctx* c, const float* x_dev, float lr, float* losses_dev, int r) {
  int rc = check_idle(c);
  if (rc) return rc;
  if (!x_dev) return fail(c, PBD_EINVAL, "x_dev is null");
  if (!losses_dev) return fail(c, PBD_EINVAL, "losses_dev is null");
  if (!std::isfinite(lr)) return fail(c, PBD_EINVAL, "learning rate is not finite");
  if (r == 1)
    for (int b = 0; b < c->B; ++b)
      if ((rc = define_alpha(c, b))) return rc;
  // The body of the step touches only workspace addresses, so it is captured once into a HIP
  // graph and replayed: ~300 small launches per step would otherwise be bound by launch cost.
  // Capture needs a real stream and no profiling events; otherwise the kernels are launched directly.
  const bool want_graph = c->stream != nullptr && !c->prof_on && !c->o.no_graph;
  c->front = 0;        // the captured body addresses the first copy of the relay store
  rc = dispatch(c, [&](auto& e) { e.set_lr(lr); e.prepare(x_dev); });
  if (rc) return rc;
  if (want_graph && !c->gexec[r] && !c->graph_tried[r]) {
    c->graph_tried[r] = true;
    hipGraph_t graph = nullptr;
    const bool fork = side_streams(c);
    if (hipStreamBeginCapture(c->stream, hipStreamCaptureModeRelaxed) == hipSuccess) {
      dispatch(c, [&](auto& e) { e.step_body(fork, r == 1); });
      hipError_t ee = hipStreamEndCapture(c->stream, &graph);
      if (ee == hipSuccess && graph && hipGraphInstantiate(&c->gexec[r], graph, nullptr, nullptr, 0) != hipSuccess)
        c->gexec[r] = nullptr;
      if (graph) (void)hipGraphDestroy(graph);
    }
    (void)hipGetLastError();
  }
  if (want_graph && c->gexec[r]) {
    HIP_TRY(c, hipGraphLaunch(c->gexec[r], c->stream));
    c->relayed_upto = c->B;
    for (BlockPlan& bp : c->net[1]) bp.stepped = c->concurrent;
    c->net[1].back().stepped = true;
  } else {
    rc = dispatch(c, [&](auto& e) { e.step_body(false, r == 1); });
    if (rc) return rc;
  }
  HIP_TRY(c, hipMemcpyAsync(losses_dev, c->ws + c->loss_off, (size_t)c->B * 4, hipMemcpyDeviceToDevice, c->stream));
  return after_launches(c);
}

// The students' half of a pipelined step on the batch in the front copy, block after block.
int pipeline_drain(pbd_ctx* c, float* losses_dev) {
  const bool want_graph = c->stream != nullptr && !c->prof_on && !c->o.no_graph;
  const int q = c->front;
  int rc = dispatch(c, [&](auto& e) {
    e.set_lr(c->pending_lr);
    for (int b = 0; b < c->B; ++b) {
      e.net = PBD_STUDENT; e.blk = b;
      if (c->net[1][b].dirty) e.refresh_compute_copies(c->net[1][b]);
    }
  });
  if (rc) return rc;
  if (want_graph && !c->gdrain[q] && !c->gdrain_tried[q]) {
    c->gdrain_tried[q] = true;
    hipGraph_t graph = nullptr;
    const bool fork = side_streams(c);
    if (hipStreamBeginCapture(c->stream, hipStreamCaptureModeRelaxed) == hipSuccess) {
      dispatch(c, [&](auto& e) { e.pipe_body(fork, false); });
      hipError_t ee = hipStreamEndCapture(c->stream, &graph);
      if (ee == hipSuccess && graph && hipGraphInstantiate(&c->gdrain[q], graph, nullptr, nullptr, 0) != hipSuccess)
        c->gdrain[q] = nullptr;
      if (graph) (void)hipGraphDestroy(graph);
    }
    (void)hipGetLastError();
  }
  if (want_graph && c->gdrain[q]) {
    HIP_TRY(c, hipGraphLaunch(c->gdrain[q], c->stream));
  } else {
    rc = dispatch(c, [&](auto& e) { e.pipe_body(false, false); });
    if (rc) return rc;
  }
  HIP_TRY(c, hipMemcpyAsync(losses_dev, c->ws + c->loss_off, (size_t)c->B * 4, hipMemcpyDeviceToDevice, c->stream));
  c->pending = false;
  for (BlockPlan& bp : c->net[1]) bp.stepped = c->concurrent;
  c->net[1].back().stepped = true;
  return after_launches(c);
}

int pipeline_step(pbd_ctx* c, const float* x_dev, float lr, float* losses_dev) {
  int rc = check_ready(c);
  if (rc) return rc;
  if (!x_dev) return fail(c, PBD_EINVAL, "x_dev is null");
  if (!losses_dev) return fail(c, PBD_EINVAL, "losses_dev is null");
  if (!std::isfinite(lr)) return fail(c, PBD_EINVAL, "learning rate is not finite");
  const bool had = c->pending;
  const int tset = had ? 1 - c->front : c->front;
  if (!had) {
    // first batch: only the teacher has work
    rc = dispatch(c, [&](auto& e) { e.relay_all(x_dev); });
    if (rc) return rc;
  } else {
    const bool want_graph = c->stream != nullptr && !c->prof_on && !c->o.no_graph;
    rc = dispatch(c, [&](auto& e) { e.tset = tset; e.sset = 1 - tset; e.set_lr(c->pending_lr); e.prepare(x_dev); });
    if (rc) return rc;
    if (want_graph && !c->gpipe[tset] && !c->gpipe_tried[tset]) {
      c->gpipe_tried[tset] = true;
      hipGraph_t graph = nullptr;
      const bool fork = side_streams(c);
      if (hipStreamBeginCapture(c->stream, hipStreamCaptureModeRelaxed) == hipSuccess) {
        dispatch(c, [&](auto& e) { e.tset = tset; e.sset = 1 - tset; e.pipe_body(fork); });
        hipError_t ee = hipStreamEndCapture(c->stream, &graph);
        if (ee == hipSuccess && graph && hipGraphInstantiate(&c->gpipe[tset], graph, nullptr, nullptr, 0) != hipSuccess)
          c->gpipe[tset] = nullptr;
        if (graph) (void)hipGraphDestroy(graph);
      }
      (void)hipGetLastError();
    }
    if (want_graph && c->gpipe[tset]) {
      HIP_TRY(c, hipGraphLaunch(c->gpipe[tset], c->stream));
    } else {
      rc = dispatch(c, [&](auto& e) { e.tset = tset; e.sset = 1 - tset; e.pipe_body(false); });
      if (rc) return rc;
    }
    HIP_TRY(c, hipMemcpyAsync(losses_dev, c->ws + c->loss_off, (size_t)c->B * 4, hipMemcpyDeviceToDevice, c->stream));
  }
  c->front = tset;
  c->relayed_upto = c->B;
  c->pending = true;
  c->pending_lr = lr;
  for (BlockPlan& bp : c->net[1]) bp.stepped = false;    // their saved values belong to the batch before
  return after_launches(c);
}

}  // namespace

// ===========================================================================
// C ABI
// ===========================================================================
extern "C" {

int pbd_create(const int32_t* words, int32_t nwords, const double* pool, int32_t npool,
               const pbd_opts* opts, pbd_ctx** out) {
  if (!out) return fail(nullptr, PBD_EINVAL, "out is null");
  *out = nullptr;
  if (!words || !opts || (npool > 0 && !pool)) return fail(nullptr, PBD_EINVAL, "null argument");
  if (nwords < 6 || words[0] != kMagic || words[1] != 1) return fail(nullptr, PBD_ESHAPE, "bad descriptor header");
  if (opts->batch < 1 || (opts->precision != PBD_F32 && opts->precision != PBD_BF16))
    return fail(nullptr, PBD_EINVAL, "batch must be >= 1 and precision PBD_F32 or PBD_BF16");
  if (!(opts->momentum >= 0.f && opts->momentum < 1.f) || !(opts->bn_eps > 0.f) ||
      !(opts->bn_momentum >= 0.f && opts->bn_momentum <= 1.f))
    return fail(nullptr, PBD_EINVAL, "momentum, bn_eps or bn_momentum out of range");
  pbd_ctx* c = new pbd_ctx;
  c->o = *opts;
  c->esz = opts->precision == PBD_BF16 ? 2 : 4;
  c->B = words[2];
  c->in = {words[3], words[4], words[5]};
  if (c->B < 1 || c->B > 1024 || c->in.c < 1 || c->in.h < 1 || c->in.w < 1) {
    delete c;
    return fail(nullptr, PBD_ESHAPE, "block count or input shape out of range");
  }
  if (npool > 0) c->pool.assign(pool, pool + npool);
  int pos = 6;
  std::string err;
  for (int which = 0; which < 2; ++which)
    if (!parse_net(c, words, nwords, pos, which, err)) {
      delete c;
      return fail(nullptr, PBD_ESHAPE, "%s net: %s", which ? "student" : "teacher", err.c_str());
    }
  c->act.push_back(c->in);
  for (int b = 0; b < c->B; ++b) {
    const Shape t = c->net[0][b].shapes.back(), s = c->net[1][b].shapes.back();
    // Sec. II-A: the pair (T_i, S_i) produces activations of one shape
    if (t.c != s.c || t.h != s.h || t.w != s.w || t.c % 8) {
      delete c;
      return fail(nullptr, PBD_ESHAPE, "block %d: teacher and student outputs must agree in shape, channels %% 8 == 0", b + 1);
    }
    c->act.push_back(t);
  }
  // training-mode BN over a single value per channel has no variance (the unbiased running
  // variance divides by m - 1)
  for (const BlockPlan& bp : c->net[1])
    for (const OpPlan& op : bp.ops)
      if (op.d.type == OP_CBA && (long)opts->batch * op.out.h * op.out.w < 2) {
        delete c;
        return fail(nullptr, PBD_ESHAPE, "a student batch norm would see one value per channel (batch x %d x %d)", op.out.h, op.out.w);
      }
  // kernels address tensors with 32-bit byte offsets and use 0x80000000 as "outside every tensor"
  const long esize = opts->precision == PBD_BF16 ? 2 : 4;
  for (int which = 0; which < 2; ++which)
    for (const BlockPlan& bp : c->net[which])
      for (const Shape& s : bp.shapes)
        if ((long)opts->batch * s.h * s.w * round8(s.c) * esize >= (1L << 31) - 4096) {
          delete c;
          return fail(nullptr, PBD_ESHAPE, "a tensor of batch x %d x %d x %d takes 2 GiB or more", s.h, s.w, s.c);
        }
  plan(c);
  *out = c;
  return PBD_OK;
}

void pbd_destroy(pbd_ctx* c) {
  if (!c) return;
  for (hipGraphExec_t g : c->gexec) if (g) (void)hipGraphExecDestroy(g);
  for (hipGraphExec_t g : c->gpipe) if (g) (void)hipGraphExecDestroy(g);
  for (hipGraphExec_t g : c->gdrain) if (g) (void)hipGraphExecDestroy(g);
  for (hipStream_t s2 : c->side) (void)hipStreamDestroy(s2);
  for (hipEvent_t e : c->ev_fork) (void)hipEventDestroy(e);
  for (hipEvent_t e : c->ev_join) (void)hipEventDestroy(e);
  for (hipEvent_t e : c->ev) (void)hipEventDestroy(e);
  delete c;
}

const char* pbd_last_error(const pbd_ctx* c) { return c ? c->err.c_str() : g_create_err.c_str(); }
int32_t pbd_num_blocks(const pbd_ctx* c) { return c ? c->B : 0; }
size_t pbd_workspace_bytes(const pbd_ctx* c) { return c ? c->total : 0; }

int pbd_bind(pbd_ctx* c, void* dev_ws, size_t bytes, void* hip_stream) {
  if (!c) return PBD_EINVAL;
  if (!dev_ws) return fail(c, PBD_ENOMEM_WS, "workspace pointer is null");
  if (bytes < c->total) return fail(c, PBD_ENOMEM_WS, "workspace has %zu bytes, %zu needed", bytes, c->total);
  if (reinterpret_cast<uintptr_t>(dev_ws) % kAlign) return fail(c, PBD_ENOMEM_WS, "workspace must be %zu-byte aligned", kAlign);
  c->ws = static_cast<char*>(dev_ws);
  c->stream = static_cast<hipStream_t>(hip_stream);
  {
    float* sp = nullptr;      // this device's copy of the static reduction scratch (pbd_student_step_static)
    HIP_TRY(c, static_scratch(&sp));
    int dev = 0, cus = 0;
    HIP_TRY(c, hipGetDevice(&dev));
    HIP_TRY(c, hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    if (cus > 0) c->num_cu = cus;
  }
  // parameters, optimiser state and statistics start at zero; the relay store too,
  // so that padded channels never hold stale bits
  HIP_TRY(c, hipMemsetAsync(c->ws, 0, c->r_tscr, c->stream));
  for (int r = 0; r < 2; ++r) {
    if (c->gexec[r]) { (void)hipGraphExecDestroy(c->gexec[r]); c->gexec[r] = nullptr; }
    c->graph_tried[r] = false;
    if (c->gpipe[r]) { (void)hipGraphExecDestroy(c->gpipe[r]); c->gpipe[r] = nullptr; }
    c->gpipe_tried[r] = false;
    if (c->gdrain[r]) { (void)hipGraphExecDestroy(c->gdrain[r]); c->gdrain[r] = nullptr; }
    c->gdrain_tried[r] = false;
  }
  c->front = 0;
  c->pending = false;
  c->bound = true;
  c->relayed_upto = 0;
  c->fold_dirty = true;
  for (BlockPlan& bp : c->net[1]) bp.stepped = false;
  // BN identity: gamma = 1, running variance = 1
  for (int net = 0; net < 2; ++net)
    for (int b = 0; b < c->B; ++b) {
      BlockPlan& bp = c->net[net][b];
      for (size_t j = 0; j < bp.ops.size(); ++j) {
        OpPlan& op = bp.ops[j];
        if (op.d.type != OP_CBA) continue;
        std::vector<float> ones(op.d.c_out, 1.f);
        for (int slot : {PBD_GAMMA, PBD_RVAR}) {
          TensorRef t;
          int rc = locate(c, PBD_PARAM, net, b, (int)j, slot, t);
          if (rc) return rc;
          rc = upload(c, t, op, ones.data());
          if (rc) return rc;
        }
      }
      if (net == 1) {
        if (!bp.ttable.empty())
          HIP_TRY(c, hipMemcpyAsync(c->ws + bp.table, bp.ttable.data(), bp.ttable.size() * sizeof(TransposeEntry),
                                    hipMemcpyHostToDevice, c->stream));
        bp.dirty = true;
        // mix ops start from the descriptor's weights; alpha stays undefined until loaded or trained
        bp.alpha_defined.assign(bp.nmix, 0);
        for (const OpPlan& op : bp.ops) {
          if (op.d.type != OP_MIX) continue;
          float pk[8] = {};
          for (int k = 0; k < op.d.nin; ++k) pk[k] = (float)c->pool[op.d.pofs + k];
          HIP_TRY(c, hipMemcpyAsync(c->ws + bp.mix + ((size_t)op.mix_slot * kMixState + kMixP) * sizeof(float), pk,
                                    sizeof pk, hipMemcpyHostToDevice, c->stream));
          HIP_TRY(c, hipStreamSynchronize(c->stream));
        }
      }
    }
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return PBD_OK;
}

int pbd_load_param(pbd_ctx* c, int32_t net, int32_t b, int32_t op, int32_t slot, const float* host, size_t n) {
  int rc = check_ready(c);
  if (rc) return rc;
  if (!host) return fail(c, PBD_EINVAL, "host pointer is null");
  TensorRef t;
  rc = locate(c, PBD_PARAM, net, b, op, slot, t);
  if (rc) return rc;
  if (n != t.logical) return fail(c, PBD_ESHAPE, "tensor has %zu elements, %zu given", t.logical, n);
  rc = upload(c, t, *find_cba(c, net, b, op), host);
  if (rc) return rc;
  if (net == PBD_TEACHER) c->fold_dirty = true;
  else c->net[1][b].dirty = true;
  return PBD_OK;
}

int pbd_read_tensor(pbd_ctx* c, int32_t kind, int32_t net, int32_t b, int32_t opi, int32_t slot, float* host, size_t n) {
  int rc = check_ready(c);
  if (rc) return rc;
  if (!host) return fail(c, PBD_EINVAL, "host pointer is null");
  TensorRef t;
  rc = locate(c, kind, net, b, opi, slot, t);
  if (rc) return rc;
  if (n != t.logical) return fail(c, PBD_ESHAPE, "tensor has %zu elements, %zu asked", t.logical, n);
  const OpPlan& op = *find_cba(c, net, b, opi);
  std::vector<float> phys(t.phys);
  if (t.bf) {
    std::vector<uint16_t> h16(t.phys);
    HIP_TRY(c, hipMemcpyAsync(h16.data(), t.ptr, t.phys * 2, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    for (size_t e = 0; e < t.phys; ++e) phys[e] = bf2f(h16[e]);
  } else {
    HIP_TRY(c, hipMemcpyAsync(phys.data(), t.ptr, t.phys * 4, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
  }
  for (size_t e = 0; e < t.phys; ++e) {
    const long h = t.weight ? weight_host_index(op, e) : ((long)e < (long)t.logical ? (long)e : -1);
    if (h >= 0) host[h] = phys[e];
  }
  return PBD_OK;
}

int pbd_read_act(pbd_ctx* c, int32_t i, float* host, size_t n) {
  int rc = check_ready(c);
  if (rc) return rc;
  if (!host) return fail(c, PBD_EINVAL, "host pointer is null");
  if (i < 0 || i > c->B) return fail(c, PBD_EINVAL, "activation index %d outside 0..%d", i, c->B);
  if (c->relayed_upto < std::max(i, 1)) return fail(c, PBD_ESTATE, "the teacher has not produced A_%d yet", i);
  const Shape s = c->act[i];
  if (n != (size_t)c->o.batch * s.c * s.h * s.w) return fail(c, PBD_ESHAPE, "A_%d has %zu elements, %zu asked", i, (size_t)c->o.batch * s.c * s.h * s.w, n);
  return download_act(c, relay_ptr(c, i), s, host);
}

int pbd_read_value(pbd_ctx* c, int32_t b, int32_t v, float* host, size_t n) {
  int rc = check_ready(c);
  if (rc) return rc;
  if (!host) return fail(c, PBD_EINVAL, "host pointer is null");
  if (b < 0 || b >= c->B) return fail(c, PBD_EINVAL, "block %d outside 0..%d", b, c->B - 1);
  BlockPlan& bp = c->net[1][b];
  if (v < 0 || v >= (int)bp.shapes.size()) return fail(c, PBD_EINVAL, "value %d outside 0..%zu", v, bp.shapes.size() - 1);
  if (!bp.stepped) return fail(c, PBD_ESTATE, "block %d holds no saved values (not stepped, or scratch reused)", b);
  const Shape s = bp.shapes[v];
  if (n != (size_t)c->o.batch * s.c * s.h * s.w) return fail(c, PBD_ESHAPE, "value has %zu elements, %zu asked", (size_t)c->o.batch * s.c * s.h * s.w, n);
  if (v > 0 && !short_column((long)c->o.batch * s.h * s.w) && residual_reader(bp, v - 1) >= 0)
    return fail(c, PBD_ESTATE, "value %d of block %d is not kept: the residual add that reads it is fused into its normalisation", v, b);
  if (v > 0 && pool_reader(bp, v - 1, c->o.batch) >= 0)
    return fail(c, PBD_ESTATE, "value %d of block %d is not kept: the max-pool that reads it normalises the convolution output itself", v, b);
  const char* dev = v == 0 ? relay_ptr(c, b) : c->ws + bp.scr_off + bp.val[v];
  return download_act(c, dev, s, host);
}

int pbd_read_conv_out(pbd_ctx* c, int32_t b, int32_t opi, float* host, size_t n) {
  int rc = check_ready(c);
  if (rc) return rc;
  if (!host) return fail(c, PBD_EINVAL, "host pointer is null");
  const OpPlan* op = find_cba(c, PBD_STUDENT, b, opi);
  if (!op) return fail(c, PBD_EINVAL, "no conv+BN operation at student block %d op %d", b, opi);
  BlockPlan& bp = c->net[1][b];
  if (!bp.stepped) return fail(c, PBD_ESTATE, "block %d holds no saved values (not stepped, or scratch reused)", b);
  const size_t want = (size_t)c->o.batch * op->out.c * op->out.h * op->out.w;
  if (n != want) return fail(c, PBD_ESHAPE, "the convolution output has %zu elements, %zu asked", want, n);
  return download_act(c, c->ws + bp.scr_off + op->y, op->out, host);
}

int pbd_read_batch_stats(pbd_ctx* c, int32_t b, int32_t opi, float* mean_host, float* invstd_host, size_t n) {
  int rc = check_ready(c);
  if (rc) return rc;
  if (!mean_host || !invstd_host) return fail(c, PBD_EINVAL, "host pointer is null");
  const OpPlan* op = find_cba(c, PBD_STUDENT, b, opi);
  if (!op) return fail(c, PBD_EINVAL, "no conv+BN operation at student block %d op %d", b, opi);
  if (!c->net[1][b].stepped) return fail(c, PBD_ESTATE, "block %d has not been stepped", b);
  if (n != (size_t)op->d.c_out) return fail(c, PBD_ESHAPE, "the layer has %d channels, %zu asked", op->d.c_out, n);
  HIP_TRY(c, hipMemcpyAsync(mean_host, c->ws + op->s_mean, n * 4, hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipMemcpyAsync(invstd_host, c->ws + op->s_invstd, n * 4, hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return PBD_OK;
}

int pbd_read_grad_value(pbd_ctx* c, int32_t b, int32_t v, float* host, size_t n) {
  int rc = check_ready(c);
  if (rc) return rc;
  if (!host) return fail(c, PBD_EINVAL, "host pointer is null");
  if (b < 0 || b >= c->B) return fail(c, PBD_EINVAL, "block %d outside 0..%d", b, c->B - 1);
  BlockPlan& bp = c->net[1][b];
  if (v < 1 || v >= (int)bp.shapes.size()) return fail(c, PBD_EINVAL, "value %d outside 1..%zu", v, bp.shapes.size() - 1);
  if (!bp.stepped) return fail(c, PBD_ESTATE, "block %d holds no saved values (not stepped, or scratch reused)", b);
  const Shape s = bp.shapes[v];
  if (n != (size_t)c->o.batch * s.c * s.h * s.w) return fail(c, PBD_ESHAPE, "value has %zu elements, %zu asked", (size_t)c->o.batch * s.c * s.h * s.w, n);
  const int last = (int)bp.ops.size() - 1;
  if (v == last + 1 && last >= 1 && bp.ops[last].d.type == OP_ADD && residual_reader(bp, last - 1) == last &&
      !short_column((long)c->o.batch * s.h * s.w))
    return fail(c, PBD_ESTATE, "the gradient of the output of block %d is not stored: the batch-norm reduction that does the last add's "
                "backward pass forms it from the block's output and the teacher's activation", b);
  return download_act(c, c->ws + bp.scr_off + bp.dval[v], s, host);
}

int pbd_teacher_relay(pbd_ctx* c, const float* x_dev, pbd_tensor* A) {
  int rc = check_idle(c);
  if (rc) return rc;
  if (!x_dev) return fail(c, PBD_EINVAL, "x_dev is null");
  rc = dispatch(c, [&](auto& e) { e.relay_all(x_dev); });
  if (rc) return rc;
  if (A) for (int i = 0; i <= c->B; ++i) fill_view(c, i, &A[i]);
  return PBD_OK;
}

int pbd_teacher_prefix(pbd_ctx* c, const float* x_dev, int32_t upto, pbd_tensor* A) {
  int rc = check_idle(c);
  if (rc) return rc;
  if (!x_dev) return fail(c, PBD_EINVAL, "x_dev is null");
  if (upto < 1 || upto > c->B) return fail(c, PBD_EINVAL, "block index %d outside 1..%d", upto, c->B);
  rc = dispatch(c, [&](auto& e) { e.relay_prefix(x_dev, upto); });
  if (rc) return rc;
  if (A) for (int i = 0; i <= upto; ++i) fill_view(c, i, &A[i]);
  return PBD_OK;
}

int pbd_student_step(pbd_ctx* c, int32_t i, const pbd_tensor* A_prev, const pbd_tensor* A_i, float lr, float* loss_dev) {
  int rc = check_idle(c);
  if (rc) return rc;
  if (i < 1 || i > c->B) return fail(c, PBD_EINVAL, "block index %d outside 1..%d", i, c->B);
  if (!std::isfinite(lr)) return fail(c, PBD_EINVAL, "learning rate is not finite");
  if (!loss_dev) return fail(c, PBD_EINVAL, "loss_dev is null");
  if (c->relayed_upto < i) return fail(c, PBD_ESTATE, "the teacher has not produced A_%d yet", i);
  if ((rc = check_view(c, A_prev, i - 1, "A_prev"))) return rc;
  if ((rc = check_view(c, A_i, i, "A_i"))) return rc;
  return dispatch(c, [&](auto& e) { e.set_lr(lr); e.student_block(i - 1, loss_dev); });
}

int pbd_student_step_static(pbd_ctx* c, int32_t i, const pbd_tensor* A_prev, const pbd_tensor* A_i, float lr, float* loss_dev) {
  int rc = check_idle(c);
  if (rc) return rc;
  if (i < 1 || i > c->B) return fail(c, PBD_EINVAL, "block index %d outside 1..%d", i, c->B);
  if (!std::isfinite(lr)) return fail(c, PBD_EINVAL, "learning rate is not finite");
  if (!loss_dev) return fail(c, PBD_EINVAL, "loss_dev is null");
  if (c->prof_on) return fail(c, PBD_ESTATE, "profiling creates events: switch it off for the call that allocates nothing");
  if (c->relayed_upto < i) return fail(c, PBD_ESTATE, "the teacher has not produced A_%d yet", i);
  if ((rc = check_view(c, A_prev, i - 1, "A_prev"))) return rc;
  if ((rc = check_view(c, A_i, i, "A_i"))) return rc;
  const size_t need = c->net[1][i - 1].red_bytes;
  if (need > kStaticScratchBytes)
    return fail(c, PBD_ENOMEM_WS, "block %d needs %zu bytes of reduction scratch, the static buffer holds %zu: use pbd_student_step",
                i, need, kStaticScratchBytes);
  float* sp = nullptr;
  HIP_TRY(c, static_scratch(&sp));
  return dispatch(c, [&](auto& e) { e.red_static = sp; e.set_lr(lr); e.student_block(i - 1, loss_dev); });
}

int pbd_distill_step(pbd_ctx* c, const float* x_dev, float lr, float* losses_dev) {
  return whole_step(c, x_dev, lr, losses_dev, 0);
}

int pbd_distill_arch_step(pbd_ctx* c, const float* x_dev, float lr_alpha, float* losses_dev) {
  return whole_step(c, x_dev, lr_alpha, losses_dev, 1);
}

int pbd_pipeline_step(pbd_ctx* c, const float* x_dev, float lr, float* losses_dev) {
  return pipeline_step(c, x_dev, lr, losses_dev);
}

int pbd_set_pipeline_order(pbd_ctx* c, const int32_t* order, int32_t n) {
  if (!c) return PBD_EINVAL;
  if (c->pending) return fail(c, PBD_ESTATE, "a pipelined batch waits for its students (call pbd_pipeline_flush first)");
  if (!order || n != c->B + 1) return fail(c, PBD_EINVAL, "the order must name %d branches", c->B + 1);
  std::vector<char> seen(n, 0);
  for (int i = 0; i < n; ++i) {
    if (order[i] < 0 || order[i] >= n || seen[order[i]]) return fail(c, PBD_EINVAL, "the order is not a permutation of 0..%d", c->B);
    seen[order[i]] = 1;
  }
  c->pipe_order.assign(order, order + n);
  for (int q = 0; q < 2; ++q) {       // captured with the old order: capture again on the next call
    if (c->bound && c->gpipe[q]) { (void)hipStreamSynchronize(c->stream); (void)hipGraphExecDestroy(c->gpipe[q]); }
    c->gpipe[q] = nullptr;
    c->gpipe_tried[q] = false;
  }
  return PBD_OK;
}

int pbd_pipeline_flush(pbd_ctx* c, float* losses_dev) {
  int rc = check_ready(c);
  if (rc) return rc;
  if (!c->pending) return PBD_OK;
  if (!losses_dev) return fail(c, PBD_EINVAL, "losses_dev is null");
  return pipeline_drain(c, losses_dev);
}

int pbd_arch_step(pbd_ctx* c, int32_t i, const pbd_tensor* A_prev, const pbd_tensor* A_i, float lr_alpha, float* loss_dev) {
  int rc = check_idle(c);
  if (rc) return rc;
  if (i < 1 || i > c->B) return fail(c, PBD_EINVAL, "block index %d outside 1..%d", i, c->B);
  if (!std::isfinite(lr_alpha)) return fail(c, PBD_EINVAL, "learning rate is not finite");
  if (!loss_dev) return fail(c, PBD_EINVAL, "loss_dev is null");
  if (c->relayed_upto < i) return fail(c, PBD_ESTATE, "the teacher has not produced A_%d yet", i);
  if ((rc = check_view(c, A_prev, i - 1, "A_prev"))) return rc;
  if ((rc = check_view(c, A_i, i, "A_i"))) return rc;
  if ((rc = define_alpha(c, i - 1))) return rc;
  return dispatch(c, [&](auto& e) { e.set_lr(lr_alpha); e.student_block(i - 1, loss_dev, true); });
}

int pbd_load_alpha(pbd_ctx* c, int32_t b, int32_t opi, const float* host, size_t n) {
  int rc = check_ready(c);
  if (rc) return rc;
  if (!host) return fail(c, PBD_EINVAL, "host pointer is null");
  const OpPlan* op = find_mix(c, b, opi);
  if (!op) return fail(c, PBD_EINVAL, "op %d of student block %d is not a mix", opi, b);
  if (n != (size_t)op->d.nin) return fail(c, PBD_ESHAPE, "the mix has %d inputs, %zu given", op->d.nin, n);
  float rec[kMixState] = {};
  double top = -INFINITY, sum = 0.0;
  for (size_t k = 0; k < n; ++k) {
    if (!std::isfinite(host[k])) return fail(c, PBD_EINVAL, "alpha[%zu] is not finite", k);
    top = std::max(top, (double)host[k]);
  }
  for (size_t k = 0; k < n; ++k) sum += std::exp((double)host[k] - top);
  for (size_t k = 0; k < n; ++k) {
    rec[kMixAlpha + k] = host[k];
    rec[kMixP + k] = (float)(std::exp((double)host[k] - top) / sum);
  }
  char* dev = mix_record(c, b, *op);
  HIP_TRY(c, hipMemcpyAsync(dev + kMixAlpha * sizeof(float), rec + kMixAlpha, 8 * sizeof(float), hipMemcpyHostToDevice, c->stream));
  HIP_TRY(c, hipMemcpyAsync(dev + kMixP * sizeof(float), rec + kMixP, 8 * sizeof(float), hipMemcpyHostToDevice, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  c->net[1][b].alpha_defined[op->mix_slot] = 1;
  return PBD_OK;
}

int pbd_read_alpha(pbd_ctx* c, int32_t kind, int32_t b, int32_t opi, float* host, size_t n) {
  int rc = check_ready(c);
  if (rc) return rc;
  if (!host) return fail(c, PBD_EINVAL, "host pointer is null");
  const OpPlan* op = find_mix(c, b, opi);
  if (!op) return fail(c, PBD_EINVAL, "op %d of student block %d is not a mix", opi, b);
  if (n != (size_t)op->d.nin) return fail(c, PBD_ESHAPE, "the mix has %d inputs, %zu asked", op->d.nin, n);
  if (kind < PBD_PARAM || kind > PBD_PROB) return fail(c, PBD_EINVAL, "kind %d is none of PBD_PARAM, PBD_GRAD, PBD_MOMENTUM, PBD_PROB", kind);
  if (kind != PBD_PROB && !c->net[1][b].alpha_defined[op->mix_slot])
    return fail(c, PBD_ESTATE, "alpha of op %d of block %d is undefined until it is loaded or trained", opi, b);
  const int at = kind == PBD_PARAM ? kMixAlpha : kind == PBD_GRAD ? kMixGrad : kind == PBD_MOMENTUM ? kMixMom : kMixP;
  float rec[8];
  HIP_TRY(c, hipMemcpyAsync(rec, mix_record(c, b, *op) + at * sizeof(float), sizeof rec, hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  for (size_t k = 0; k < n; ++k) host[k] = rec[k];
  return PBD_OK;
}

int pbd_uses_graph(const pbd_ctx* c) { return c && (c->gexec[0] || c->gexec[1] || c->gpipe[0] || c->gpipe[1]) ? 1 : 0; }

int pbd_sync(pbd_ctx* c) {
  int rc = check_ready(c);
  if (rc) return rc;
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return after_launches(c);
}

int pbd_set_profile(pbd_ctx* c, int32_t on) {
  if (!c) return PBD_EINVAL;
  c->prof_on = on != 0;
  return PBD_OK;
}
int pbd_reset_profile(pbd_ctx* c) {
  if (!c) return PBD_EINVAL;
  if (c->bound) HIP_TRY(c, hipStreamSynchronize(c->stream));
  c->prof.clear();
  return PBD_OK;
}
int pbd_get_profile(pbd_ctx* c, pbd_prof_entry* out, int32_t max) {
  int rc = check_ready(c);
  if (rc) return rc;
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  const int n = (int)c->prof.size();
  for (int i = 0; i < n; ++i) {
    float ms = 0.f;
    HIP_TRY(c, hipEventElapsedTime(&ms, c->ev[2 * i], c->ev[2 * i + 1]));
    c->prof[i].ms = ms;
    if (out && i < max) out[i] = c->prof[i];
  }
  return n;
}

}  // extern "C"
