// Dense convolution kernels for gfx950 (CDNA4), channel-last tensors.
//
//  * igemm_kernel: forward and backward-data as an implicit GEMM on the bf16
//    matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation).  Rows of the
//    GEMM are output pixels, columns are output channels, the reduction runs over
//    (r, s, c) in 16-byte chunks of 8 channels gathered straight from the NHWC
//    tensor into LDS; weights are kept reduction-contiguous ([K][R][S][C] for
//    forward, [C][R][S][K] for backward-data) so both operands are read from LDS
//    with one 128-bit load per lane.  128 x BN x 32 tiles, 4 wavefronts of 64,
//    LDS double buffering with register prefetch.
//  * wgrad_tr_kernel: backward-weight.  The reduction runs over pixels, which is the
//    strided direction of NHWC memory; tiles go to LDS as they lie in memory and the
//    gfx950 transposing LDS read (ds_read_b64_tr_b16) hands each lane its 8
//    consecutive pixels of one channel.  The pixel range is split over workgroups;
//    partial tiles go to scratch and are summed by an ordered second stage, so the
//    result does not depend on scheduling.
//  * direct kernels: plain one-thread-per-output loops in fp32, used for the
//    float32 precision and as a cross-check of the MFMA kernels.
#pragma once
#include <type_traits>

#include "ew_kernels.h"

namespace pbd {

struct ConvGeom {
  int N, H, W, C;      // input tensor [N][H][W][C]   (C physical, multiple of 8)
  int P, Q, K;         // output tensor [N][P][Q][K]
  int R, S, stride, pad;
};

// ---------------------------------------------------------------------------
// direct kernels (fp32 accumulate)
// ---------------------------------------------------------------------------
// y[m][k] = sum_{r,s,c} x[n, p*st+r-pad, q*st+s-pad, c] * w[k][r][s][c]
template <class T, class WT>
__global__ void conv_direct_fwd_kernel(const T* __restrict__ x, const WT* __restrict__ w,
                                       T* __restrict__ y, const float* __restrict__ a,
                                       const float* __restrict__ b, int act, ConvGeom g) {
  const long total = (long)g.N * g.P * g.Q * g.K;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
    const int k = (int)(i % g.K);
    long pix = i / g.K;
    const int q = (int)(pix % g.Q); pix /= g.Q;
    const int p = (int)(pix % g.P);
    const int n = (int)(pix / g.P);
    float acc = 0.f;
    for (int r = 0; r < g.R; ++r) {
      const int h = p * g.stride + r - g.pad;
      if (h < 0 || h >= g.H) continue;
      for (int s = 0; s < g.S; ++s) {
        const int ww = q * g.stride + s - g.pad;
        if (ww < 0 || ww >= g.W) continue;
        const T* xp = x + (((long)n * g.H + h) * g.W + ww) * g.C;
        const WT* wp = w + (((long)k * g.R + r) * g.S + s) * g.C;
        for (int c = 0; c < g.C; ++c) acc = fmaf((float)xp[c], (float)wp[c], acc);
      }
    }
    if (a) acc = fmaf(acc, a[k], b[k]);
    y[i] = (T)apply_act(acc, act);
  }
}

// dx[n,h,w,c] (+)= sum_{k,r,s} dy[n,(h+pad-r)/st,(w+pad-s)/st,k] * w[k][r][s][c]
template <class T, class WT>
__global__ void conv_direct_dgrad_kernel(const T* __restrict__ dy, const WT* __restrict__ w,
                                         T* __restrict__ dx, int accumulate, ConvGeom g) {
  const long total = (long)g.N * g.H * g.W * g.C;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
    const int c = (int)(i % g.C);
    long pix = i / g.C;
    const int ww = (int)(pix % g.W); pix /= g.W;
    const int h = (int)(pix % g.H);
    const int n = (int)(pix / g.H);
    float acc = accumulate ? (float)dx[i] : 0.f;
    for (int r = 0; r < g.R; ++r) {
      const int ph = h + g.pad - r;
      if (ph < 0 || ph % g.stride) continue;
      const int p = ph / g.stride;
      if (p >= g.P) continue;
      for (int s = 0; s < g.S; ++s) {
        const int qw = ww + g.pad - s;
        if (qw < 0 || qw % g.stride) continue;
        const int q = qw / g.stride;
        if (q >= g.Q) continue;
        const T* dp = dy + (((long)n * g.P + p) * g.Q + q) * g.K;
        for (int k = 0; k < g.K; ++k)
          acc = fmaf((float)dp[k], (float)w[(((long)k * g.R + r) * g.S + s) * g.C + c], acc);
      }
    }
    dx[i] = (T)acc;
  }
}

// dw[k][r][s][c] = sum_{n,p,q} dy[n,p,q,k] * x[n, p*st+r-pad, q*st+s-pad, c]
template <class T>
__global__ void conv_direct_wgrad_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                         float* __restrict__ dw, ConvGeom g) {
  const long total = (long)g.K * g.R * g.S * g.C;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
    const int c = (int)(i % g.C);
    long t = i / g.C;
    const int s = (int)(t % g.S); t /= g.S;
    const int r = (int)(t % g.R);
    const int k = (int)(t / g.R);
    float acc = 0.f;
    for (int n = 0; n < g.N; ++n)
      for (int p = 0; p < g.P; ++p) {
        const int h = p * g.stride + r - g.pad;
        if (h < 0 || h >= g.H) continue;
        for (int q = 0; q < g.Q; ++q) {
          const int ww = q * g.stride + s - g.pad;
          if (ww < 0 || ww >= g.W) continue;
          acc = fmaf((float)dy[(((long)n * g.P + p) * g.Q + q) * g.K + k],
                     (float)x[(((long)n * g.H + h) * g.W + ww) * g.C + c], acc);
        }
      }
    dw[i] = acc;
  }
}

// ---------------------------------------------------------------------------
// MFMA implicit GEMM: forward (MODE 0) and backward-data (MODE 1)
// ---------------------------------------------------------------------------
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// Generic view: Out[m][j] = sum_kk Agather(m, kk) * Bw[j][kk]
//   rows m = (n, a, b) over an [N][HO][WO] grid, columns j < NC, kk = (r*S+s)*CA + c
//   MODE 0: source pixel (a*st + r - pad, b*st + s - pad) of A = x    [N][HA][WA][CA]
//   MODE 1: source pixel ((a+pad-r)/st, (b+pad-s)/st)     of A = dy   [N][HA][WA][CA]
struct IgemmArgs {
  int N, HA, WA, CA;
  int HO, WO, NC;
  int R, S, stride, pad;
  int M;      // N*HO*WO
  int Kred;   // R*S*CA
  int ksteps_per_split;  // reduction steps of IG_BK handled by one K slice (split-K)
  unsigned a_bytes, b_bytes;  // sizes of the A tensor and of the weight matrix
  int tiles_m, tiles_n, splits;   // the 1-D grid holds tiles_m * tiles_n * splits workgroups
  // residual join fused into the store (EPI_STORE / EPI_AFFINE_ACT through LDS): out = act(result + res),
  // the result rounded to bf16 first, exactly as a stored tensor read back by a separate add would be
  const void* res;
  int res_act;
  // batch-norm statistics of the stored result from the same pass (EPI_STORE): per row tile and channel the
  // sums of y and y^2 over the tile's rows, stats[tile_m][2][NC] (fp32; summed further in double)
  float* stats;
  // igemm_dma_kernel only: the first big_tiles workgroups take 256-row tiles (tiles_n per row tile), the others
  // 64-row tiles over the rows from tail_m0 on
  int big_tiles, tail_m0;
  // igemm_dma_kernel, backward-data with stride 2 only: the rows are taken parity class by parity class of the
  // input pixel (class id = 2 (h % 2) + w % 2; only the taps of matching parity reach such a pixel), par_classes
  // of them in the order par_order lists (2 bits per class id); 0: rows in pixel order, every tap tested
  int par_classes, par_order;
  // igemm_dma_kernel, forward only: a tap gathers a run of 1 << pix_shift neighbouring pixels of CA >> pix_shift
  // channels each (CA contiguous elements; S counts such runs).  0: a tap is one pixel of CA channels
  int pix_shift;
  // the staged stores of the output, and the loads of what they combine with (a fused residual, the gradient an
  // accumulating launch adds to), are nontemporal (tensors far larger than the caches)
  int stream_out;
};

// EPI_PARTIAL: raw fp32 partial tile of a split-K launch, summed by splitk_epilogue_kernel
enum { EPI_STORE = 0, EPI_AFFINE_ACT = 1, EPI_ACCUM = 2, EPI_PARTIAL = 3 };

// K step 32 (any channel count) or 64 (channel counts that are multiples of 64: a row's chunk is
// then a whole 128-byte cache line, 8 lanes wide, instead of half of one).  LDS row pitch 96 / 144
// bytes: conflict-free for the fragment reads (row = lane%32, 16-byte chunk = lane/32) in both
// cases; at 96 bytes the staging writes (row = lane/4, chunk = lane%4) are conflict-free too, at 144
// bytes neighbouring rows overlap on 4 of 32 banks.
constexpr int IG_BK = 32;
constexpr int ig_pitch(int bk) { return bk == 64 ? 72 : 48; }

// workgroup w runs on XCD w % 8: give XCD c the c-th contiguous run of the `total` work items
__device__ __forceinline__ int xcd_contiguous(int w, int total) {
  const int q = total >> 3, r = total & 7, c = w & 7;
  return c * q + min(c, r) + (w >> 3);
}

// UNI: the channel count of the gathered tensor is a multiple of the 32-element K step, so a step
// lies inside one filter tap and (r, s, c0) are the same for the whole workgroup: they live in
// scalar registers and a load costs a lane two adds, two compares, an add and a select.
template <int MODE, int BM, int BN, int EPI, bool UNI, int BK = IG_BK>
__global__ __launch_bounds__(256) void igemm_kernel(const bf16_t* __restrict__ A,
                                                    const bf16_t* __restrict__ Bw,
                                                    bf16_t* __restrict__ Out,
                                                    const float* __restrict__ ep_a,
                                                    const float* __restrict__ ep_b, int act,
                                                    IgemmArgs g) {
  // wave grid: 256x128 tiles 2x2 (a wave owns 128x64); 128-row tiles 2x2 (BN 128) or 4x1; 64-row
  // tiles 2x2 (BN >= 64) or 2x1 over 32 columns
  constexpr int WAVES_M = BM == 256 ? 2 : (BM == 128 ? (BN == 128 ? 2 : 4) : 2), WAVES_N = 4 / WAVES_M;
  constexpr int TM = BM / (WAVES_M * 32);
  constexpr int TN = (BN / (WAVES_N * 32)) > 0 ? BN / (WAVES_N * 32) : 1;
  constexpr bool kIdleWaves = BN / (WAVES_N * 32) == 0;      // BM 64, BN 32: waves with wn = 1 only stage tiles
  constexpr int CPR = BK / 8, RPP = 256 / CPR;   // 16-byte chunks per tile row, rows staged per pass
  constexpr int PITCH = ig_pitch(BK);
  constexpr int A_LOADS = BM / RPP;
  constexpr int B_LOADS = (BN + RPP - 1) / RPP;  // 16-byte chunks of the weight tile per thread
  static_assert(!(BK == 64) || UNI, "the 64-wide K step needs uniform taps");
  // one LDS block: the two stages of both operand tiles during the reduction, then the output tile on
  // its way to coalesced stores
  __shared__ __attribute__((aligned(16))) bf16_t smem[2 * (BM + BN) * PITCH];
  bf16_t (*As)[BM * PITCH] = reinterpret_cast<bf16_t (*)[BM * PITCH]>(smem);
  bf16_t (*Bs)[BN * PITCH] = reinterpret_cast<bf16_t (*)[BN * PITCH]>(smem + 2 * BM * PITCH);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  // Workgroups are dealt to the 8 XCDs round-robin, each with an L2 of its own.  Remapped so that
  // an XCD works through a contiguous run of tiles (column tiles of one row tile next to each other,
  // then the next row tile): the 3x3 halo rows and the rows shared by column tiles are then re-read
  // from that XCD's L2 instead of crossing the fabric once per tap.
  const int tile = xcd_contiguous(blockIdx.x, g.tiles_m * g.tiles_n * g.splits);
  const int tile_n = tile % g.tiles_n, tile_m = (tile / g.tiles_n) % g.tiles_m, kslice = tile / (g.tiles_n * g.tiles_m);
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int chunk = tid % CPR, prow = tid / CPR;
  const int sh = g.stride == 2 ? 1 : 0, smask = g.stride - 1;
  // the tile's folded batch-norm terms wait in LDS from the start, so that the store at the end does not
  // begin with a round trip to memory (columns past NC repeat the last four: they are never stored)
  __shared__ __attribute__((aligned(16))) float ep_s[EPI == EPI_AFFINE_ACT ? 2 * BN : 4];
  if (EPI == EPI_AFFINE_ACT && tid < BN / 4) {
    const int col = min(n0 + tid * 4, g.NC - 4);
    *reinterpret_cast<float4*>(ep_s + tid * 4) = *reinterpret_cast<const float4*>(ep_a + col);
    *reinterpret_cast<float4*>(ep_s + BN + tid * 4) = *reinterpret_cast<const float4*>(ep_b + col);
  }

  // The A rows this thread stages, decoded once.  All offsets are 32-bit element indices
  // (create rejects tensors of 2^31 elements or more), and the per-step work is a handful of adds.
  int rbase[A_LOADS], rh[A_LOADS], rw[A_LOADS];
  bool rvalid[A_LOADS];
#pragma unroll
  for (int i = 0; i < A_LOADS; ++i) {
    const int m = m0 + prow + RPP * i;
    rvalid[i] = m < g.M;
    const int mm = rvalid[i] ? m : 0;
    const int b_ = mm % g.WO;
    const int t = mm / g.WO;
    const int a_ = t % g.HO;
    rbase[i] = (t / g.HO) * g.HA * g.WA;                          // first pixel of image n
    rh[i] = MODE == 0 ? a_ * g.stride - g.pad : a_ + g.pad;       // row of tap (0,0) / of the output pixel
    rw[i] = MODE == 0 ? b_ * g.stride - g.pad : b_ + g.pad;
  }
  int brow[B_LOADS];
#pragma unroll
  for (int i = 0; i < B_LOADS; ++i) {
    const int row = prow + RPP * i;
    brow[i] = (row < BN && n0 + row < g.NC) ? (n0 + row) * g.Kred : -1;
  }
  // reduction position of this thread's chunk: kk = (r*S + s)*CA + c
  const int kt0 = kslice * g.ksteps_per_split;
  int kk = kt0 * BK + (UNI ? 0 : chunk * 8);
  int r, s, c;
  {
    const int rs = kk / g.CA;
    c = kk - rs * g.CA;
    r = rs / g.S;
    s = rs - r * g.S;
  }
  // UNI: byte offset = abase[i] + delta(r, s, c0), linear in the tap for either mode (for stride-2
  // backward-data the halved coordinates are exact whenever the parity test passes); rows that do
  // not exist get a coordinate that fails every range test
  unsigned abase[A_LOADS], bbase[B_LOADS];
  if (UNI) {
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) {
      if (MODE == 0) abase[i] = (unsigned)(((rbase[i] + rh[i] * g.WA + rw[i]) * g.CA + chunk * 8) * 2);
      else abase[i] = (unsigned)((rbase[i] * g.CA + ((rh[i] * g.WA + rw[i]) * g.CA >> sh) + chunk * 8) * 2);
      if (!rvalid[i]) rh[i] = -(1 << 24);
    }
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i) bbase[i] = brow[i] >= 0 ? (unsigned)(brow[i] + chunk * 8) * 2u : kOutOfRange;
  }

  // two register stages: tile kt+2 is requested while tile kt is multiplied and tile kt+1 moves to LDS
  uint4 areg[2][A_LOADS], breg[2][B_LOADS];
  const __amdgpu_buffer_rsrc_t a_rsrc = tensor_rsrc(A, g.a_bytes), b_rsrc = tensor_rsrc(Bw, g.b_bytes);
  auto load_tile = [&](auto stage) {
    constexpr int S_ = decltype(stage)::value;
    if constexpr (UNI) {
      const int tap = MODE == 0 ? r * g.WA + s : -(r * g.WA + s);
      const unsigned delta = (unsigned)(((tap * g.CA) >> (MODE == 1 ? sh : 0)) + c) * 2u;
      const unsigned hlim = MODE == 0 ? (unsigned)g.HA : (unsigned)g.HA << sh;
      const unsigned wlim = MODE == 0 ? (unsigned)g.WA : (unsigned)g.WA << sh;
#pragma unroll
      for (int i = 0; i < A_LOADS; ++i) {
        const int h = MODE == 0 ? rh[i] + r : rh[i] - r, w = MODE == 0 ? rw[i] + s : rw[i] - s;
        bool ok = (unsigned)h < hlim && (unsigned)w < wlim;
        if (MODE == 1) ok = ok && ((h | w) & smask) == 0;
        areg[S_][i] = buffer_load16(a_rsrc, ok ? abase[i] + delta : kOutOfRange);
      }
#pragma unroll
      for (int i = 0; i < B_LOADS; ++i) breg[S_][i] = buffer_load16(b_rsrc, bbase[i] + (unsigned)kk * 2u);
      kk += BK;
      c += BK;
      const bool wrap = c >= g.CA;
      c = wrap ? 0 : c;
      s += wrap ? 1 : 0;
      const bool wrap2 = s == g.S;
      s = wrap2 ? 0 : s;
      r += wrap2 ? 1 : 0;
      return;
    }
    const bool kvalid = r < g.R;
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i) {
      int h, w;
      bool ok = rvalid[i] && kvalid;
      if (MODE == 0) {
        h = rh[i] + r;
        w = rw[i] + s;
      } else {
        const int th = rh[i] - r, tw = rw[i] - s;
        ok = ok && ((th | tw) & smask) == 0;
        h = th >> sh;
        w = tw >> sh;
      }
      ok = ok && (unsigned)h < (unsigned)g.HA && (unsigned)w < (unsigned)g.WA;
      const unsigned off = (unsigned)((rbase[i] + h * g.WA + w) * g.CA + c) * 2u;
      areg[S_][i] = buffer_load16(a_rsrc, ok ? off : kOutOfRange);
    }
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i)
      breg[S_][i] = buffer_load16(b_rsrc, (brow[i] >= 0 && kvalid) ? (unsigned)(brow[i] + kk) * 2u : kOutOfRange);
    kk += BK;
    c += BK;
    if (g.CA >= BK) {             // at most one wrap per step
      const bool wrap = c >= g.CA;
      c -= wrap ? g.CA : 0;
      s += wrap ? 1 : 0;
      const bool wrap2 = s == g.S;
      s = wrap2 ? 0 : s;
      r += wrap2 ? 1 : 0;
    } else {
      while (c >= g.CA) {
        c -= g.CA;
        if (++s == g.S) { s = 0; ++r; }
      }
    }
  };
  auto store_tile = [&](auto stage, int buf) {
    constexpr int S_ = decltype(stage)::value;
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i)
      *reinterpret_cast<uint4*>(&As[buf][(prow + RPP * i) * PITCH + chunk * 8]) = areg[S_][i];
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i) {
      const int row = prow + RPP * i;
      if (row < BN) *reinterpret_cast<uint4*>(&Bs[buf][row * PITCH + chunk * 8]) = breg[S_][i];
    }
  };

  // acc[i][j]: 32 channels (rows of the MFMA result) x 32 pixels (columns): the weight fragment is
  // the first operand, so that a lane ends up with 4 consecutive channels of one pixel per register
  // group and the epilogue stores 8 bytes (bf16) or 16 bytes (fp32 partial) at a time.
  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int nk = min(g.ksteps_per_split, (g.Kred + BK - 1) / BK - kt0);
  using S0 = std::integral_constant<int, 0>;
  using S1 = std::integral_constant<int, 1>;
  load_tile(S0{});
  if (nk > 1) load_tile(S1{});
  store_tile(S0{}, 0);
  __syncthreads();
  auto iteration = [&](int kt, auto cur) {
    constexpr int C_ = decltype(cur)::value;
    using Cur = std::integral_constant<int, C_>;
    using Nxt = std::integral_constant<int, 1 - C_>;
    if (kt + 2 < nk) load_tile(Cur{});          // stage C_ went to LDS one iteration ago
    if (!(kIdleWaves && wn > 0)) {
#pragma unroll
      for (int ks = 0; ks < BK / 16; ++ks) {
        bf16x8 af[TM], bfr[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
          af[i] = *reinterpret_cast<const bf16x8*>(
              &As[C_][(wm * TM * 32 + i * 32 + (lane & 31)) * PITCH + ks * 16 + (lane >> 5) * 8]);
#pragma unroll
        for (int j = 0; j < TN; ++j)
          bfr[j] = *reinterpret_cast<const bf16x8*>(
              &Bs[C_][(wn * TN * 32 + j * 32 + (lane & 31)) * PITCH + ks * 16 + (lane >> 5) * 8]);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
      }
    }
    if (kt + 1 < nk) store_tile(Nxt{}, 1 - C_);
    __syncthreads();
  };
  for (int kt = 0; kt < nk; kt += 2) {
    iteration(kt, S0{});
    if (kt + 1 < nk) iteration(kt + 1, S1{});
  }
  // epilogue: lane holds pixel (lane%32) and channels 8*(v/4) + 4*(lane/32) + v%4 of each 32x32 tile
  const bool full = m0 + BM <= g.M && n0 + BN <= g.NC;
  if constexpr ((EPI == EPI_STORE || EPI == EPI_AFFINE_ACT) && !kIdleWaves) {
    // bf16 results go through LDS (the operand tiles are dead after the last barrier of the loop) and
    // leave as 16-byte chunks, consecutive lanes on consecutive chunks of a row: whole cache lines
    // instead of 32 rows x 16 bytes per store instruction
    constexpr int OP = BN * 2 + 16;                  // bytes per staged row; the pad spreads rows over banks
    static_assert(BM * OP <= 2 * (BM + BN) * PITCH * 2, "the output tile must fit in the operand tiles' LDS");
    unsigned char* stage = reinterpret_cast<unsigned char*>(smem);
    constexpr int CPROW = BN / 8;                    // 16-byte chunks per row
    constexpr int NCHUNK = BM * CPROW;
    static_assert(NCHUNK % 256 == 0, "chunks divide evenly over the block");
    // a fused residual is fetched now, ahead of the staging, where the registers allow (8 chunks per thread)
    constexpr bool kResEarly = NCHUNK / 256 <= 8;
    uint4 rv[kResEarly ? NCHUNK / 256 : 1];
    if (kResEarly && g.res) {
#pragma unroll
      for (int k = 0; k < NCHUNK / 256; ++k) {
        const int cidx = tid + k * 256;
        const int row = m0 + cidx / CPROW, col = n0 + (cidx % CPROW) * 8;
        rv[k] = (full || (row < g.M && col < g.NC))
                    ? *reinterpret_cast<const uint4*>(static_cast<const bf16_t*>(g.res) + (size_t)row * g.NC + col)
                    : make_uint4(0, 0, 0, 0);
      }
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int lrow = wm * TM * 32 + i * 32 + (lane & 31);
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int lcol = wn * TN * 32 + j * 32 + 8 * q + 4 * (lane >> 5);
          float o[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = acc[i][j][4 * q + e];
          if (EPI == EPI_AFFINE_ACT) {
            const float4 ea = *reinterpret_cast<const float4*>(ep_s + lcol);
            const float4 eb = *reinterpret_cast<const float4*>(ep_s + BN + lcol);
            o[0] = apply_act(fmaf(o[0], ea.x, eb.x), act); o[1] = apply_act(fmaf(o[1], ea.y, eb.y), act);
            o[2] = apply_act(fmaf(o[2], ea.z, eb.z), act); o[3] = apply_act(fmaf(o[3], ea.w, eb.w), act);
          }
          uint2 pk;
          pk.x = pack_bf2(o[0], o[1]);
          pk.y = pack_bf2(o[2], o[3]);
          *reinterpret_cast<uint2*>(stage + lrow * OP + lcol * 2) = pk;
        }
    }
    __syncthreads();
    static_assert(256 % CPROW == 0, "a thread keeps its chunk column over the rows it stores");
    float s1[8], s2[8];                              // column sums of this thread's chunks (g.stats)
#pragma unroll
    for (int e = 0; e < 8; ++e) s1[e] = s2[e] = 0.f;
#pragma unroll
    for (int k = 0; k < NCHUNK / 256; ++k) {
      const int cidx = tid + k * 256;
      const int lrow = cidx / CPROW, c16 = cidx % CPROW;
      const int row = m0 + lrow, col = n0 + c16 * 8;
      if (full || (row < g.M && col < g.NC)) {       // NC % 8 == 0: a chunk is in or out as a whole
        uint4 v = *reinterpret_cast<const uint4*>(stage + lrow * OP + c16 * 16);
        if (EPI == EPI_STORE && g.stats) {
          const float f[8] = {bf_lo(v.x), bf_hi(v.x), bf_lo(v.y), bf_hi(v.y), bf_lo(v.z), bf_hi(v.z), bf_lo(v.w), bf_hi(v.w)};
#pragma unroll
          for (int e = 0; e < 8; ++e) { s1[e] += f[e]; s2[e] = fmaf(f[e], f[e], s2[e]); }
        }
        if (g.res) {
          const uint4 r_ = kResEarly ? rv[kResEarly ? k : 0]
                                     : *reinterpret_cast<const uint4*>(static_cast<const bf16_t*>(g.res) + (size_t)row * g.NC + col);
          v.x = pack_bf2(apply_act(bf_lo(v.x) + bf_lo(r_.x), g.res_act), apply_act(bf_hi(v.x) + bf_hi(r_.x), g.res_act));
          v.y = pack_bf2(apply_act(bf_lo(v.y) + bf_lo(r_.y), g.res_act), apply_act(bf_hi(v.y) + bf_hi(r_.y), g.res_act));
          v.z = pack_bf2(apply_act(bf_lo(v.z) + bf_lo(r_.z), g.res_act), apply_act(bf_hi(v.z) + bf_hi(r_.z), g.res_act));
          v.w = pack_bf2(apply_act(bf_lo(v.w) + bf_lo(r_.w), g.res_act), apply_act(bf_hi(v.w) + bf_hi(r_.w), g.res_act));
        }
        if (g.stream_out) {                      // a tensor far larger than the caches: its lines are not kept there
          typedef unsigned int u32x4_nt __attribute__((ext_vector_type(4)));
          const u32x4_nt q = {v.x, v.y, v.z, v.w};
          __builtin_nontemporal_store(q, reinterpret_cast<u32x4_nt*>(Out + (size_t)row * g.NC + col));
        } else {
          *reinterpret_cast<uint4*>(Out + (size_t)row * g.NC + col) = v;
        }
      }
    }
    if (EPI == EPI_STORE && g.stats) {
      // threads with equal tid % CPROW hold the same 8 channels: butterfly inside the wave, then the four
      // waves in order through LDS (a fixed association)
#pragma unroll
      for (int off = CPROW; off < 64; off <<= 1)
#pragma unroll
        for (int e = 0; e < 8; ++e) { s1[e] += __shfl_xor(s1[e], off, 64); s2[e] += __shfl_xor(s2[e], off, 64); }
      __syncthreads();                               // the staged tile has been read by everyone
      float* red = reinterpret_cast<float*>(smem);   // [wave][chunk column][16]
      if (lane < CPROW) {
#pragma unroll
        for (int e = 0; e < 8; ++e) { red[(wave * CPROW + lane) * 16 + e] = s1[e]; red[(wave * CPROW + lane) * 16 + 8 + e] = s2[e]; }
      }
      __syncthreads();
      const int col = n0 + tid * 8;
      if (tid < CPROW && col < g.NC) {
        float* dst = g.stats + (size_t)tile_m * 2 * g.NC + col;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float t = (red[tid * 16 + e] + red[(CPROW + tid) * 16 + e]) + (red[(2 * CPROW + tid) * 16 + e] + red[(3 * CPROW + tid) * 16 + e]);
          dst[(e >> 3) * g.NC + (e & 7)] = t;
        }
      }
    }
    return;
  }
  // accumulating launches add in fp32 before the one rounding: the tile is staged as fp32 where the
  // operand tiles' LDS has room for it (every tile shape but 256 x 128 and the 32-wide K step's 128 x 128)
  constexpr int OPF = BN * 4 + 16;
  if constexpr (EPI == EPI_ACCUM && !kIdleWaves && BM * OPF <= 2 * (BM + BN) * PITCH * 2) {
    unsigned char* stage = reinterpret_cast<unsigned char*>(smem);
    constexpr int CPROW = BN / 8;
    constexpr int NCHUNK = BM * CPROW;
    static_assert(NCHUNK % 256 == 0, "chunks divide evenly over the block");
    static_assert(NCHUNK / 256 <= 8, "the values to add to are held in registers while the tile is staged");
    // what the tile adds to is fetched now, ahead of the staging: the stores then wait for LDS only
    uint4 old[NCHUNK / 256];
#pragma unroll
    for (int k = 0; k < NCHUNK / 256; ++k) {
      const int cidx = tid + k * 256;
      const int row = m0 + cidx / CPROW, col = n0 + (cidx % CPROW) * 8;
      old[k] = (full || (row < g.M && col < g.NC)) ? *reinterpret_cast<const uint4*>(Out + (size_t)row * g.NC + col)
                                                    : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int lrow = wm * TM * 32 + i * 32 + (lane & 31);
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int lcol = wn * TN * 32 + j * 32 + 8 * q + 4 * (lane >> 5);
          *reinterpret_cast<float4*>(stage + lrow * OPF + lcol * 4) =
              make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
        }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < NCHUNK / 256; ++k) {
      const int cidx = tid + k * 256;
      const int lrow = cidx / CPROW, c16 = cidx % CPROW;
      const int row = m0 + lrow, col = n0 + c16 * 8;
      if (full || (row < g.M && col < g.NC)) {
        bf16_t* dst = Out + (size_t)row * g.NC + col;
        const float4 lo = *reinterpret_cast<const float4*>(stage + lrow * OPF + c16 * 32);
        const float4 hi = *reinterpret_cast<const float4*>(stage + lrow * OPF + c16 * 32 + 16);
        uint4 pk;
        pk.x = pack_bf2(lo.x + bf_lo(old[k].x), lo.y + bf_hi(old[k].x));
        pk.y = pack_bf2(lo.z + bf_lo(old[k].y), lo.w + bf_hi(old[k].y));
        pk.z = pack_bf2(hi.x + bf_lo(old[k].z), hi.y + bf_hi(old[k].z));
        pk.w = pack_bf2(hi.z + bf_lo(old[k].w), hi.w + bf_hi(old[k].w));
        *reinterpret_cast<uint4*>(dst) = pk;
      }
    }
    return;
  }
  if (kIdleWaves && wn > 0) return;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int row = m0 + wm * TM * 32 + i * 32 + (lane & 31);
    if (!full && row >= g.M) continue;
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int col = n0 + wn * TN * 32 + j * 32 + 8 * q + 4 * (lane >> 5);
        if (!full && col >= g.NC) continue;   // NC % 8 == 0 and col % 4 == 0: a group is in or out as a whole
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = acc[i][j][4 * q + e];
        if (EPI == EPI_PARTIAL) {
          float* dst = reinterpret_cast<float*>(Out) + ((size_t)kslice * g.M + row) * g.NC + col;
          *reinterpret_cast<float4*>(dst) = make_float4(o[0], o[1], o[2], o[3]);
          continue;
        }
        bf16_t* dst = Out + (size_t)row * g.NC + col;
        if (EPI == EPI_AFFINE_ACT) {
          const float4 ea = *reinterpret_cast<const float4*>(ep_a + col);
          const float4 eb = *reinterpret_cast<const float4*>(ep_b + col);
          o[0] = apply_act(fmaf(o[0], ea.x, eb.x), act); o[1] = apply_act(fmaf(o[1], ea.y, eb.y), act);
          o[2] = apply_act(fmaf(o[2], ea.z, eb.z), act); o[3] = apply_act(fmaf(o[3], ea.w, eb.w), act);
        }
        if (EPI == EPI_ACCUM) {
          const uint2 old = *reinterpret_cast<const uint2*>(dst);
          o[0] += bf_lo(old.x); o[1] += bf_hi(old.x); o[2] += bf_lo(old.y); o[3] += bf_hi(old.y);
        }
        uint2 pk;
        pk.x = pack_bf2(o[0], o[1]);
        pk.y = pack_bf2(o[2], o[3]);
        *reinterpret_cast<uint2*>(dst) = pk;
      }
  }
}

// Second stage of a split-K launch: out = epilogue(sum_s part[s]) in split order.
__global__ void splitk_epilogue_kernel(const float* __restrict__ part, bf16_t* __restrict__ out,
                                       const float* __restrict__ ep_a, const float* __restrict__ ep_b,
                                       int act, int epi, long nvec, int ncv, int splits) {
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < nvec; i += (long)gridDim.x * blockDim.x) {
    const int c0 = (int)(i % ncv) * 8;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    for (int s = 0; s < splits; ++s) {
      float v[8];
      IO<float>::ld(part + ((long)s * nvec + i) * 8, v);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += v[e];
    }
    if (epi == EPI_AFFINE_ACT) {
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = apply_act(fmaf(acc[e], ep_a[c0 + e], ep_b[c0 + e]), act);
    } else if (epi == EPI_ACCUM) {
      float v[8];
      IO<bf16_t>::ld(out + i * 8, v);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += v[e];
    }
    IO<bf16_t>::st(out + i * 8, acc);
  }
}

// ---------------------------------------------------------------------------
// Weight gradient with the LDS transpose read of gfx950.
//   dW[k][j] = sum_m dy[m][k] * xcol[m][j],  j = (r*S + s)*C + c
// The reduction runs over pixels, the slow dimension of both operands, while an MFMA lane wants 8
// consecutive reduction elements of ONE channel.  ds_read_b64_tr_b16 does that exchange inside the
// LDS read: 16 lanes read a 4 (rows) x 16 (columns) block of 16-bit elements, source lane s giving
// the address of row s/4, columns 4*(s%4)..+3, and lane i receives column i of the 4 rows.  So
// tiles are staged exactly as they lie in memory (rows = pixels, channels contiguous; a plain
// 16-byte copy per thread) and no register transpose is needed.
//   LDS row pitch = tile width + 32 elements (64 bytes): the 4 rows of one read land on banks
//   16 apart and the two 16-lane groups of a half wave 8 apart: conflict-free.
// Pipeline: registers hold tile t+1 while tile t is multiplied; two LDS buffers, one barrier a step.
// ---------------------------------------------------------------------------
struct WgradTrArgs {
  int N, H, W, C;     // x  [N][H][W][C]
  int P, Q, K;        // dy [N][P][Q][K]
  int R, S, stride, pad;
  int M;              // N*P*Q
  int J;              // R*S*C
  int pix_per_split;  // multiple of 32
  int dn, dp, dq;     // 32 pixels = dn images + dp rows + dq columns (mixed radix P, Q)
  unsigned dy_bytes, x_bytes;
  int tiles_k, tiles_j, splits;   // the 1-D grid holds tiles_k * tiles_j * splits workgroups
};

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ bf16x8 lds_read_tr8(const bf16_t* p, int row_pitch) {
  typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 4 * row_pitch));
  const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

template <int TM, int TN>
__global__ __launch_bounds__(256) void wgrad_tr_kernel(const bf16_t* __restrict__ dy,
                                                       const bf16_t* __restrict__ x,
                                                       float* __restrict__ part, WgradTrArgs g) {
  constexpr int BKP = 32;
  constexpr int PA = TM + 32, PB = TN + 32;                        // LDS row pitch, elements
  constexpr int A_CPR = TM / 8, B_CPR = TN / 8;                    // 16-byte chunks per tile row
  constexpr int A_N = BKP * A_CPR / 256, B_N = BKP * B_CPR / 256;  // chunks per thread
  constexpr int A_RSTEP = 256 / A_CPR, B_RSTEP = 256 / B_CPR;      // rows between a thread's chunks
  constexpr int TWM = TM / 64, TWN = TN / 64;                      // 32x32 tiles per wave (waves 2x2)
  static_assert(A_N >= 1 && B_N >= 1, "tile too narrow for 256 threads");
  __shared__ __attribute__((aligned(16))) bf16_t As[2][BKP * PA];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[2][BKP * PB];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  // all tiles of one pixel slice read the same rows of dy and x: keep them on one XCD (one L2)
  const int tile = xcd_contiguous(blockIdx.x, g.tiles_k * g.tiles_j * g.splits);
  const int slice = tile / (g.tiles_k * g.tiles_j);
  const int k0 = ((tile / g.tiles_j) % g.tiles_k) * TM, j0 = (tile % g.tiles_j) * TN;
  const int mbeg = slice * g.pix_per_split;
  const int mend = min(g.M, mbeg + g.pix_per_split);
  const int nsteps = (mend - mbeg + BKP - 1) / BKP;
  const __amdgpu_buffer_rsrc_t rdy = tensor_rsrc(dy, g.dy_bytes), rx = tensor_rsrc(x, g.x_bytes);

  // dy chunks: row a_row + i*A_RSTEP of the step, channels k0 + a_cc*8 .. +7.  Rows past the end of
  // the tensor read as zeros (pix_per_split is a multiple of 32, so only the last split is ragged).
  const int a_cc = tid % A_CPR, a_row = tid / A_CPR;
  unsigned a_off[A_N];
#pragma unroll
  for (int i = 0; i < A_N; ++i)
    a_off[i] = k0 + a_cc * 8 < g.K ? (unsigned)((mbeg + a_row + i * A_RSTEP) * g.K + k0 + a_cc * 8) * 2u : kOutOfRange;
  const unsigned a_step = (unsigned)(BKP * g.K) * 2u;

  // x chunks: column chunk -> tap (br, bs) and first channel bc, fixed; pixel -> (n, p, q), advanced
  // by 32 pixels a step without divisions
  const int b_cc = tid % B_CPR, b_row = tid / B_CPR;
  const int jcol = j0 + b_cc * 8;
  const bool b_ok = jcol < g.J;
  int br, bs, bc;
  {
    const int rs = b_ok ? jcol / g.C : 0;
    bc = b_ok ? jcol - rs * g.C : 0;
    br = rs / g.S;
    bs = rs - br * g.S;
  }
  int bn[B_N], bp[B_N], bq[B_N], bm[B_N];
#pragma unroll
  for (int i = 0; i < B_N; ++i) {
    bm[i] = mbeg + b_row + i * B_RSTEP;
    bq[i] = bm[i] % g.Q;
    const int t = bm[i] / g.Q;
    bp[i] = t % g.P;
    bn[i] = t / g.P;
  }

  uint4 ra[A_N], rb[B_N];
  auto load_step = [&]() {
#pragma unroll
    for (int i = 0; i < A_N; ++i) {
      ra[i] = buffer_load16(rdy, a_off[i]);
      a_off[i] += a_off[i] == kOutOfRange ? 0u : a_step;
    }
#pragma unroll
    for (int i = 0; i < B_N; ++i) {
      const int h = bp[i] * g.stride + br - g.pad, w = bq[i] * g.stride + bs - g.pad;
      const bool ok = b_ok && bm[i] < mend && (unsigned)h < (unsigned)g.H && (unsigned)w < (unsigned)g.W;
      const unsigned off = (unsigned)(((bn[i] * g.H + h) * g.W + w) * g.C + bc) * 2u;
      rb[i] = buffer_load16(rx, ok ? off : kOutOfRange);
      bm[i] += BKP;
      int q = bq[i] + g.dq;
      const int c1 = q >= g.Q ? 1 : 0;
      bq[i] = q - (c1 ? g.Q : 0);
      int pp = bp[i] + g.dp + c1;
      const int c2 = pp >= g.P ? 1 : 0;
      bp[i] = pp - (c2 ? g.P : 0);
      bn[i] += g.dn + c2;
    }
  };
  auto store_step = [&](int buf) {
#pragma unroll
    for (int i = 0; i < A_N; ++i)
      *reinterpret_cast<uint4*>(&As[buf][(a_row + i * A_RSTEP) * PA + a_cc * 8]) = ra[i];
#pragma unroll
    for (int i = 0; i < B_N; ++i)
      *reinterpret_cast<uint4*>(&Bs[buf][(b_row + i * B_RSTEP) * PB + b_cc * 8]) = rb[i];
  };

  f32x16 acc[TWM][TWN];
#pragma unroll
  for (int i = 0; i < TWM; ++i)
#pragma unroll
    for (int j = 0; j < TWN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // fragment addresses: 16-lane group gl reads channels 16*(gl&1)..+15 of pixels 8*(gl>>1)..+7
  const int s16 = lane & 15, gl = lane >> 4;
  const int frag_row = 8 * (gl >> 1) + (s16 >> 2), frag_col = 16 * (gl & 1) + 4 * (s16 & 3);
  const int a_frag = frag_row * PA + wm * (TM / 2) + frag_col;
  const int b_frag = frag_row * PB + wn * (TN / 2) + frag_col;

  load_step();
  store_step(0);
  __syncthreads();
  for (int st = 0; st < nsteps; ++st) {
    const int buf = st & 1;
    if (st + 1 < nsteps) load_step();
#pragma unroll
    for (int ks = 0; ks < BKP / 16; ++ks) {
      bf16x8 af[TWM], bfr[TWN];
#pragma unroll
      for (int i = 0; i < TWM; ++i) af[i] = lds_read_tr8(&As[buf][a_frag + ks * 16 * PA + i * 32], PA);
#pragma unroll
      for (int j = 0; j < TWN; ++j) bfr[j] = lds_read_tr8(&Bs[buf][b_frag + ks * 16 * PB + j * 32], PB);
#pragma unroll
      for (int i = 0; i < TWM; ++i)
#pragma unroll
        for (int j = 0; j < TWN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (st + 1 < nsteps) store_step(buf ^ 1);
    __syncthreads();
  }

  float* out = part + (size_t)slice * g.K * g.J;
#pragma unroll
  for (int j = 0; j < TWN; ++j) {
    const int col = j0 + wn * (TN / 2) + j * 32 + (lane & 31);
    if (col >= g.J) continue;
#pragma unroll
    for (int i = 0; i < TWM; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = k0 + wm * (TM / 2) + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (row < g.K) out[(size_t)row * g.J + col] = acc[i][j][v];
      }
  }
}

}  // namespace pbd
