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
//  * wgrad_kernel: backward-weight.  The reduction runs over pixels, which is the
//    strided direction of NHWC memory, so every thread loads an 8 pixel x 8 channel
//    block, transposes it in registers and stores reduction-contiguous rows to LDS
//    (XOR-swizzled against bank conflicts).  The pixel range is split over
//    workgroups; partial tiles go to scratch and are summed by an ordered second
//    stage, so the result does not depend on scheduling.
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
  int ksteps_per_split;  // reduction steps of IG_BK handled by one blockIdx.z (split-K)
  unsigned a_bytes, b_bytes;  // sizes of the A tensor and of the weight matrix
};

// EPI_PARTIAL: raw fp32 partial tile of a split-K launch, summed by splitk_epilogue_kernel
enum { EPI_STORE = 0, EPI_AFFINE_ACT = 1, EPI_ACCUM = 2, EPI_PARTIAL = 3 };

// LDS row pitch 96 B: both the MFMA fragment reads (row = lane%32, 16-byte chunk = lane/32) and the
// staging writes (row = lane/4, chunk = lane%4) run at the full 128 B/clk with it (80 B makes the writes conflict)
constexpr int IG_BK = 32, IG_PITCH = IG_BK + 16;

template <int MODE, int BM, int BN, int EPI>
__global__ __launch_bounds__(256) void igemm_kernel(const bf16_t* __restrict__ A,
                                                    const bf16_t* __restrict__ Bw,
                                                    bf16_t* __restrict__ Out,
                                                    const float* __restrict__ ep_a,
                                                    const float* __restrict__ ep_b, int act,
                                                    IgemmArgs g) {
  // wave grid: 128-row tiles 2x2 (BN 128) or 4x1; 64-row tiles 2x2 (BN >= 64) or 2x1 over 32 columns
  constexpr int WAVES_M = BM == 128 ? (BN == 128 ? 2 : 4) : 2, WAVES_N = 4 / WAVES_M;
  constexpr int TM = BM / (WAVES_M * 32);
  constexpr int TN = (BN / (WAVES_N * 32)) > 0 ? BN / (WAVES_N * 32) : 1;
  constexpr bool kIdleWaves = BN / (WAVES_N * 32) == 0;      // BM 64, BN 32: waves with wn = 1 only stage tiles
  constexpr int A_LOADS = BM / 64;
  constexpr int B_LOADS = (BN * 4 + 255) / 256;  // 16-byte chunks of the weight tile per thread
  __shared__ __attribute__((aligned(16))) bf16_t As[2][BM * IG_PITCH];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[2][BN * IG_PITCH];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
  const int chunk = tid & 3;
  const int sh = g.stride == 2 ? 1 : 0, smask = g.stride - 1;

  // The A rows this thread stages, decoded once.  All offsets are 32-bit element indices
  // (create rejects tensors of 2^31 elements or more), and the per-step work is a handful of adds.
  int rbase[A_LOADS], rh[A_LOADS], rw[A_LOADS];
  bool rvalid[A_LOADS];
#pragma unroll
  for (int i = 0; i < A_LOADS; ++i) {
    const int m = m0 + (tid >> 2) + 64 * i;
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
    const int row = (tid >> 2) + 64 * i;
    brow[i] = (row < BN && n0 + row < g.NC) ? (n0 + row) * g.Kred : -1;
  }
  // reduction position of this thread's chunk: kk = (r*S + s)*CA + c
  const int kt0 = blockIdx.z * g.ksteps_per_split;
  int kk = kt0 * IG_BK + chunk * 8;
  int r, s, c;
  {
    const int rs = kk / g.CA;
    c = kk - rs * g.CA;
    r = rs / g.S;
    s = rs - r * g.S;
  }

  // two register stages: tile kt+2 is requested while tile kt is multiplied and tile kt+1 moves to LDS
  uint4 areg[2][A_LOADS], breg[2][B_LOADS];
  const __amdgpu_buffer_rsrc_t a_rsrc = tensor_rsrc(A, g.a_bytes), b_rsrc = tensor_rsrc(Bw, g.b_bytes);
  auto load_tile = [&](auto stage) {
    constexpr int S_ = decltype(stage)::value;
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
    kk += IG_BK;
    c += IG_BK;
    if (g.CA >= IG_BK) {          // at most one wrap per step
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
      *reinterpret_cast<uint4*>(&As[buf][((tid >> 2) + 64 * i) * IG_PITCH + chunk * 8]) = areg[S_][i];
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i) {
      const int row = (tid >> 2) + 64 * i;
      if (row < BN) *reinterpret_cast<uint4*>(&Bs[buf][row * IG_PITCH + chunk * 8]) = breg[S_][i];
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

  const int nk = min(g.ksteps_per_split, (g.Kred + IG_BK - 1) / IG_BK - kt0);
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
      for (int ks = 0; ks < IG_BK / 16; ++ks) {
        bf16x8 af[TM], bfr[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
          af[i] = *reinterpret_cast<const bf16x8*>(
              &As[C_][(wm * TM * 32 + i * 32 + (lane & 31)) * IG_PITCH + ks * 16 + (lane >> 5) * 8]);
#pragma unroll
        for (int j = 0; j < TN; ++j)
          bfr[j] = *reinterpret_cast<const bf16x8*>(
              &Bs[C_][(wn * TN * 32 + j * 32 + (lane & 31)) * IG_PITCH + ks * 16 + (lane >> 5) * 8]);
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
  if (kIdleWaves && wn > 0) return;

  // epilogue: lane holds pixel (lane%32) and channels 8*(v/4) + 4*(lane/32) + v%4 of each 32x32 tile
  const bool full = m0 + BM <= g.M && n0 + BN <= g.NC;
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
          float* dst = reinterpret_cast<float*>(Out) + ((size_t)blockIdx.z * g.M + row) * g.NC + col;
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
// MFMA backward-weight:  dW[k][j] = sum_m dy[m][k] * Xgather(m, j),  j = (r*S+s)*C + c
// Tile T x T outputs, BKP pixels per step; grid = (tiles_k, tiles_j, splits).
// ---------------------------------------------------------------------------
struct WgradArgs {
  int N, H, W, C;     // x  [N][H][W][C]
  int P, Q, K;        // dy [N][P][Q][K]
  int R, S, stride, pad;
  int M;              // N*P*Q
  int J;              // R*S*C
  int pix_per_split;  // multiple of BKP
};

__device__ __forceinline__ void transpose8x8(const uint4 (&in)[8], uint4 (&out)[8]) {
  // in[p] = 8 channels of pixel p (as 4 dwords); out[c] = 8 pixels of channel c
  const uint32_t* I = reinterpret_cast<const uint32_t*>(in);
  uint32_t* O = reinterpret_cast<uint32_t*>(out);
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t lo = I[(2 * i) * 4 + j], hi = I[(2 * i + 1) * 4 + j];
      O[(2 * j) * 4 + i] = (lo & 0xffffu) | (hi << 16);
      O[(2 * j + 1) * 4 + i] = (lo >> 16) | (hi & 0xffff0000u);
    }
}

template <int T, int BKP>
__global__ __launch_bounds__(256) void wgrad_kernel(const bf16_t* __restrict__ dy,
                                                    const bf16_t* __restrict__ x,
                                                    float* __restrict__ part, WgradArgs g) {
  static_assert((2 * T / 8) * (BKP / 8) == 256, "one 8x8 block per thread");
  constexpr int PITCH = BKP + 8;          // bf16 elements per LDS row
  constexpr int UNITS = BKP / 8;          // 16-byte units per row
  constexpr int CH = T / 8;               // channel chunks per operand
  constexpr int TW = T / 64;              // 32x32 MFMA tiles per wave per dim (waves 2x2)
  __shared__ __attribute__((aligned(16))) bf16_t As[T * PITCH];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[T * PITCH];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int k0 = blockIdx.x * T, j0 = blockIdx.y * T;
  const long mbeg = (long)blockIdx.z * g.pix_per_split;
  const long mend = min((long)g.M, mbeg + g.pix_per_split);

  const bool isA = tid < 128;
  const int blk = isA ? tid : tid - 128;
  const int cc = blk % CH, pg = blk / CH;   // channel chunk, pixel group
  // B threads: column chunk -> (r, s, c0), fixed for the whole loop
  int br = 0, bs = 0, bc = 0;
  bool colvalid;
  if (isA) {
    colvalid = (k0 + cc * 8) < g.K;
  } else {
    const int j = j0 + cc * 8;
    colvalid = j < g.J;
    const int rs = colvalid ? j / g.C : 0;
    bc = colvalid ? j - rs * g.C : 0;
    br = rs / g.S;
    bs = rs - br * g.S;
  }

  f32x16 acc[TW][TW];
#pragma unroll
  for (int i = 0; i < TW; ++i)
#pragma unroll
    for (int j = 0; j < TW; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  for (long ms = mbeg; ms < mend; ms += BKP) {
    uint4 in[8], tr[8];
    const long mfirst = ms + pg * 8;
    if (isA) {
#pragma unroll
      for (int p = 0; p < 8; ++p) {
        const long m = mfirst + p;
        in[p] = (colvalid && m < mend)
                    ? *reinterpret_cast<const uint4*>(dy + m * g.K + k0 + cc * 8)
                    : make_uint4(0, 0, 0, 0);
      }
    } else {
      long t = mfirst;
      int q = (int)(t % g.Q); t /= g.Q;
      int p_ = (int)(t % g.P);
      int n = (int)(t / g.P);
#pragma unroll
      for (int p = 0; p < 8; ++p) {
        const long m = mfirst + p;
        const int h = p_ * g.stride + br - g.pad, w = q * g.stride + bs - g.pad;
        const bool ok = colvalid && m < mend && h >= 0 && h < g.H && w >= 0 && w < g.W;
        in[p] = ok ? *reinterpret_cast<const uint4*>(x + (((long)n * g.H + h) * g.W + w) * g.C + bc)
                   : make_uint4(0, 0, 0, 0);
        if (++q == g.Q) { q = 0; if (++p_ == g.P) { p_ = 0; ++n; } }
      }
    }
    transpose8x8(in, tr);
    __syncthreads();  // previous step's MFMA reads are done
    bf16_t* dstbase = isA ? As : Bs;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = cc * 8 + i;
      const int unit = pg ^ (cc & 7);       // swizzle: rows 8 apart would share banks
      *reinterpret_cast<uint4*>(&dstbase[row * PITCH + unit * 8]) = tr[i];
    }
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < BKP / 16; ++ks) {
      bf16x8 af[TW], bfr[TW];
#pragma unroll
      for (int i = 0; i < TW; ++i) {
        const int row = wm * TW * 32 + i * 32 + (lane & 31);
        const int unit = (ks * 2 + (lane >> 5)) ^ ((row >> 3) & 7);
        af[i] = *reinterpret_cast<const bf16x8*>(&As[row * PITCH + unit * 8]);
      }
#pragma unroll
      for (int j = 0; j < TW; ++j) {
        const int row = wn * TW * 32 + j * 32 + (lane & 31);
        const int unit = (ks * 2 + (lane >> 5)) ^ ((row >> 3) & 7);
        bfr[j] = *reinterpret_cast<const bf16x8*>(&Bs[row * PITCH + unit * 8]);
      }
#pragma unroll
      for (int i = 0; i < TW; ++i)
#pragma unroll
        for (int j = 0; j < TW; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
  }
  static_assert(UNITS >= 8, "swizzle needs 8 units per row");

  float* out = part + (long)blockIdx.z * g.K * g.J;
#pragma unroll
  for (int j = 0; j < TW; ++j) {
    const int col = j0 + wn * TW * 32 + j * 32 + (lane & 31);
    if (col >= g.J) continue;
#pragma unroll
    for (int i = 0; i < TW; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = k0 + wm * TW * 32 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (row < g.K) out[(long)row * g.J + col] = acc[i][j][v];
      }
  }
}

}  // namespace pbd
