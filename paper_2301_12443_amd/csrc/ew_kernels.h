// Bandwidth-bound kernels of the blockwise-distillation step for gfx950:
// layout/cast, batch normalisation (statistics, apply, backward), activations,
// max-pool, residual add, candidate mix, depthwise convolution, fused MSE loss +
// gradient, fused SGD-momentum.  Tensors are channel-last (NHWC); a thread owns
// one vector of 8 consecutive channels, so a wavefront touches contiguous
// 1 KiB (bf16) or 2 KiB (fp32) runs and every access is a 16-byte transaction.
// All reductions are two-stage and ordered (no atomics), which keeps a step
// bit-reproducible and independent of the order in which blocks are trained
// (Sec. IV-B: blocks share no parameters).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pbd {

typedef __bf16 bf16_t;
enum { ACT_NONE = 0, ACT_RELU = 1, ACT_RELU6 = 2 };

__device__ __forceinline__ float bf_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }
// round-to-nearest-even pair conversion (v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ uint32_t pack_bf2(float a, float b) {
  typedef float f2 __attribute__((ext_vector_type(2)));
  typedef __bf16 b2 __attribute__((ext_vector_type(2)));
  f2 v = {a, b};
  b2 r = __builtin_convertvector(v, b2);
  return __builtin_bit_cast(uint32_t, r);
}

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

// Raw buffer descriptor over a whole tensor: a load whose byte offset lies outside [0, bytes) returns
// zeros in hardware, which turns padding, ragged tiles and the reduction tail into plain offsets
// (no branches, no selects).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t tensor_rsrc(const void* p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}
__device__ __forceinline__ uint4 buffer_load16(__amdgpu_buffer_rsrc_t r, unsigned byte_off) {
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, 0, 0);
  return make_uint4(v.x, v.y, v.z, v.w);
}
constexpr unsigned kOutOfRange = 0x80000000u;   // byte offset beyond any tensor (they are < 2^31 elements)

template <class T> struct IO;
// ld_raw() only starts the 16- or 32-byte load, unpack() converts later: a loop that calls ld_raw() for all its rows,
// then __builtin_amdgcn_sched_barrier(0), then unpack() has every load in flight before the first wait (left to
// itself the scheduler pairs each load with its conversion and the loads go out one at a time).
template <> struct IO<float> {
  struct Raw { float4 a, b; };
  static __device__ __forceinline__ Raw ld_raw(const float* p) {
    Raw q; q.a = reinterpret_cast<const float4*>(p)[0]; q.b = reinterpret_cast<const float4*>(p)[1]; return q;
  }
  template <bool STREAM> static __device__ __forceinline__ Raw ld_raw_t(const float* p) { return ld_raw(p); }
  template <bool STREAM> static __device__ __forceinline__ void st_t(float* p, const float v[8]) { st(p, v); }
  static __device__ __forceinline__ void unpack(const Raw& q, float v[8]) {
    v[0] = q.a.x; v[1] = q.a.y; v[2] = q.a.z; v[3] = q.a.w; v[4] = q.b.x; v[5] = q.b.y; v[6] = q.b.z; v[7] = q.b.w;
  }
  static __device__ __forceinline__ void ld(const float* p, float v[8]) {
    const float4 a = reinterpret_cast<const float4*>(p)[0], b = reinterpret_cast<const float4*>(p)[1];
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
  static __device__ __forceinline__ void st(float* p, const float v[8]) {
    reinterpret_cast<float4*>(p)[0] = make_float4(v[0], v[1], v[2], v[3]);
    reinterpret_cast<float4*>(p)[1] = make_float4(v[4], v[5], v[6], v[7]);
  }
};
template <> struct IO<bf16_t> {
  typedef uint4 Raw;
  static __device__ __forceinline__ Raw ld_raw(const bf16_t* p) { return *reinterpret_cast<const uint4*>(p); }
  // STREAM: nontemporal forms for the passes over tensors far larger than the caches: a line that is read or
  // written once per pass does not push out what the convolutions running beside the pass keep in L2
  typedef unsigned int u32x4_nt __attribute__((ext_vector_type(4)));
  template <bool STREAM> static __device__ __forceinline__ Raw ld_raw_t(const bf16_t* p) {
    if (!STREAM) return ld_raw(p);
    const u32x4_nt q = __builtin_nontemporal_load(reinterpret_cast<const u32x4_nt*>(p));
    return make_uint4(q.x, q.y, q.z, q.w);
  }
  template <bool STREAM> static __device__ __forceinline__ void st_t(bf16_t* p, const float v[8]) {
    if (!STREAM) { st(p, v); return; }
    u32x4_nt q = {pack_bf2(v[0], v[1]), pack_bf2(v[2], v[3]), pack_bf2(v[4], v[5]), pack_bf2(v[6], v[7])};
    __builtin_nontemporal_store(q, reinterpret_cast<u32x4_nt*>(p));
  }
  static __device__ __forceinline__ void unpack(const Raw& u, float v[8]) {
    v[0] = bf_lo(u.x); v[1] = bf_hi(u.x); v[2] = bf_lo(u.y); v[3] = bf_hi(u.y);
    v[4] = bf_lo(u.z); v[5] = bf_hi(u.z); v[6] = bf_lo(u.w); v[7] = bf_hi(u.w);
  }
  static __device__ __forceinline__ void ld(const bf16_t* p, float v[8]) {
    const uint4 u = *reinterpret_cast<const uint4*>(p);
    v[0] = bf_lo(u.x); v[1] = bf_hi(u.x); v[2] = bf_lo(u.y); v[3] = bf_hi(u.y);
    v[4] = bf_lo(u.z); v[5] = bf_hi(u.z); v[6] = bf_lo(u.w); v[7] = bf_hi(u.w);
  }
  static __device__ __forceinline__ void st(bf16_t* p, const float v[8]) {
    uint4 u;
    u.x = pack_bf2(v[0], v[1]); u.y = pack_bf2(v[2], v[3]);
    u.z = pack_bf2(v[4], v[5]); u.w = pack_bf2(v[6], v[7]);
    *reinterpret_cast<uint4*>(p) = u;
  }
};

// Gathered 8-channel loads through a buffer descriptor: issue() only starts the load (an invalid
// position becomes an out-of-range offset and reads as zeros), unpack() converts later, so that a
// whole stencil of loads is in flight before the first use.
template <class T> struct BufIO;
template <> struct BufIO<bf16_t> {
  typedef uint4 Raw;
  static __device__ __forceinline__ Raw issue(__amdgpu_buffer_rsrc_t r, unsigned elem, bool ok) {
    return buffer_load16(r, ok ? elem * 2u : kOutOfRange);
  }
  static __device__ __forceinline__ void unpack(const Raw& u, float v[8]) {
    v[0] = bf_lo(u.x); v[1] = bf_hi(u.x); v[2] = bf_lo(u.y); v[3] = bf_hi(u.y);
    v[4] = bf_lo(u.z); v[5] = bf_hi(u.z); v[6] = bf_lo(u.w); v[7] = bf_hi(u.w);
  }
};
template <> struct BufIO<float> {
  struct Raw { uint4 a, b; };
  static __device__ __forceinline__ Raw issue(__amdgpu_buffer_rsrc_t r, unsigned elem, bool ok) {
    Raw q;
    q.a = buffer_load16(r, ok ? elem * 4u : kOutOfRange);
    q.b = buffer_load16(r, ok ? elem * 4u + 16u : kOutOfRange);
    return q;
  }
  static __device__ __forceinline__ void unpack(const Raw& u, float v[8]) {
    v[0] = __uint_as_float(u.a.x); v[1] = __uint_as_float(u.a.y); v[2] = __uint_as_float(u.a.z);
    v[3] = __uint_as_float(u.a.w); v[4] = __uint_as_float(u.b.x); v[5] = __uint_as_float(u.b.y);
    v[6] = __uint_as_float(u.b.z); v[7] = __uint_as_float(u.b.w);
  }
};

// Written as selects on two values derived from `act` (a clamp bound that no value reaches unless the layer is a
// ReLU6, and "no rectifier at all"), not as a branch per case: `act` is a launch argument, the kernels call this
// per element inside their loops, and the compiler keeps a branch chain per element otherwise.  Same value as the
// case-by-case definition for every input, NaN and infinities included:
//   ReLU: v > 0 ? v : 0;  ReLU6: v > 0 ? min(v, 6) : 0;  none: v
__device__ __forceinline__ float apply_act(float v, int act) {
  const bool all = act != ACT_RELU && act != ACT_RELU6;
  const float hi = act == ACT_RELU6 ? 6.f : __builtin_nanf("");     // (v >= NaN never holds)
  const float t = v >= hi ? hi : v;
  return (all || v > 0.f) ? t : 0.f;
}
// slope of the activation at pre-activation v (1 where it passes the gradient):
//   ReLU: v > 0;  ReLU6: 0 < v < 6;  none: always
__device__ __forceinline__ bool act_pass(float v, int act) {
  const bool all = act != ACT_RELU && act != ACT_RELU6;
  const float hi = act == ACT_RELU6 ? 6.f : __builtin_nanf("");
  return all || (v > 0.f && !(v >= hi));
}
// ---------------------------------------------------------------------------
// layout / cast:  x float32 NCHW  ->  A_0  T NHWC with Cp channels (pads = 0)
// ---------------------------------------------------------------------------
template <class T>
__global__ void cast_input_kernel(const float* __restrict__ x, T* __restrict__ out, int N, int C,
                                  int HW, int Cp) {
  const long nvec = (long)N * HW * (Cp / 8);
  const int ncv = Cp / 8;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < nvec; i += (long)gridDim.x * blockDim.x) {
    const int cv = (int)(i % ncv);
    const long pix = i / ncv;
    const int n = (int)(pix / HW), hw = (int)(pix % HW);
    float v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int c = cv * 8 + k;
      v[k] = c < C ? x[((long)n * C + c) * HW + hw] : 0.f;
    }
    IO<T>::st(out + i * 8, v);
  }
}

// ---------------------------------------------------------------------------
// Space-to-depth form of a 3-channel input for a 7 x 7 stride-2 stem (pad 3):
//   x float32 NCHW  ->  x2 T [N][H/2][W/2][16],  x2[n][i][j][(dy*2 + dx)*3 + c] = x[n][c][2i + dy][2j + dx], lanes 12..15 = 0.
// With the filter repacked the same way (pack_stem_weights_kernel) the stem is a 4 x 4 stride-1 convolution
// over 16 channels with two rows / columns of padding in front:
//   out[a][b] = sum_{r,s,c} W[r][s][c] x[2a-3+r][2b-3+s][c],  row 2a-3+r = 2 (a-2+br) + dy  <=>  r = 2 br + dy - 1,
// a reduction of 4*4*16 = 256 elements (147 of them real) instead of 7*7*8 = 392 with the channels padded to 8.
// ---------------------------------------------------------------------------
template <class T>
__global__ void s2d_input_kernel(const float* __restrict__ x, T* __restrict__ out, int N, int C, int H, int W) {
  const int H2 = H / 2, W2 = W / 2;
  const long npix = (long)N * H2 * W2;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < npix; i += (long)gridDim.x * blockDim.x) {
    const int j = (int)(i % W2);
    const long t = i / W2;
    const int ii = (int)(t % H2), n = (int)(t / H2);
    float v[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = 0.f;
#pragma unroll
    for (int dy = 0; dy < 2; ++dy)
      for (int c = 0; c < C; ++c) {                  // (C <= 4)
        const float2 p = *reinterpret_cast<const float2*>(x + (((long)n * C + c) * H + 2 * ii + dy) * W + 2 * j);
        v[(dy * 2 + 0) * C + c] = p.x;
        v[(dy * 2 + 1) * C + c] = p.y;
      }
    IO<T>::st(out + i * 16, v);
    IO<T>::st(out + i * 16 + 8, v + 8);
  }
}
// w [K][7][7][8] (channel lanes >= C are zero) -> w2 [K][4][4][16] as above; one thread per element of w2
template <class T>
__global__ void pack_stem_weights_kernel(const T* __restrict__ w, T* __restrict__ w2, int K, int C) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= K * 256) return;
  const int lane = i & 15, bs = (i >> 4) & 3, br = (i >> 6) & 3, k = i >> 8;
  const int q = lane / C, c = lane % C;              // q = dy*2 + dx
  const int r = 2 * br + (q >> 1) - 1, s_ = 2 * bs + (q & 1) - 1;
  T v = T(0);
  if (lane < 4 * C && r >= 0 && s_ >= 0) v = w[((k * 7 + r) * 7 + s_) * 8 + c];
  w2[i] = v;
}
// the inverse on the weight gradient: dw2 float32 [K][4][4][16] -> dw float32 [K][7][7][8] (lanes >= C zero)
__global__ void unpack_stem_grad_kernel(const float* __restrict__ dw2, float* __restrict__ dw, int K, int C) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= K * 392) return;
  const int c = i & 7, t = i >> 3, s_ = t % 7, r = (t / 7) % 7, k = t / 49;
  float v = 0.f;
  if (c < C) {
    const int br = (r + 1) >> 1, dy = (r + 1) & 1, bs = (s_ + 1) >> 1, dx = (s_ + 1) & 1;
    v = dw2[((k * 4 + br) * 4 + bs) * 16 + (dy * 2 + dx) * C + c];
  }
  dw[i] = v;
}

// ---------------------------------------------------------------------------
// inference-mode BN folded to  y = a*x + b  (teacher; Sec. II-A: the teacher is
// pretrained and only evaluated)
// ---------------------------------------------------------------------------
__global__ void bn_fold_kernel(const float* gamma, const float* beta, const float* rmean,
                               const float* rvar, float* a, float* b, int C, float eps) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= C) return;
  const float s = gamma[c] / sqrtf(rvar[c] + eps);
  a[c] = s;
  b[c] = beta[c] - rmean[c] * s;
}

// ---------------------------------------------------------------------------
// per-channel column reductions over the M = N*H*W rows of an NHWC matrix.
// Block = 256 threads = cvl channel-vector lanes x (256/cvl) row lanes; grid =
// (column slabs, row chunks).  Each block writes one ordered partial.
// ---------------------------------------------------------------------------
struct ColGrid {
  int cvl;        // channel-vector lanes per block (<= 32); 256 / cvl row lanes, the rest of the block idles
  int slabs;      // ceil(ncv / cvl)
  int chunks;     // row chunks (gridDim.y)
  long rows_per_chunk;
};

// in-block reduction of NV floats per thread over the row lanes.  Threads are numbered
// row_lane * cvl + cv_lane (row lanes 0 .. 256/cvl - 1 take part).  The association is fixed in both
// forms, so the result never depends on scheduling.  smem: at least 256 * NV floats.
//  * cvl a power of two: the lanes of a wave that share a channel vector are cvl apart, so a butterfly
//    (lane ^ cvl, ^ 2 cvl, ... ^ 32) adds them without leaving the registers; the four waves' sums then
//    meet in LDS and are added as (w0 + w1) + (w2 + w3).
//  * any other cvl (channel counts such as 48, 96, 144): every thread leaves its sums in LDS as
//    [row_lane][cv_lane][NV]; thread o adds column o over the row lanes in order.
template <int NV>
__device__ __forceinline__ void block_col_reduce(float (&acc)[NV], float* smem, int cvl, int cv_lane,
                                                 int row_lane, float* out /*[NV]*/, bool& owner) {
  owner = row_lane == 0;
  if ((cvl & (cvl - 1)) == 0) {
    for (int off = cvl; off < 64; off <<= 1) {
#pragma unroll
      for (int k = 0; k < NV; ++k) acc[k] += __shfl_xor(acc[k], off, 64);
    }
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (lane < cvl) {
      float* mine = smem + (wave * cvl + lane) * NV;
#pragma unroll
      for (int k = 0; k < NV; ++k) mine[k] = acc[k];
    }
    __syncthreads();
    if (owner) {   // wave 0, lane == cv_lane
      const float* w0 = smem + cv_lane * NV;
      const int ws = cvl * NV;
#pragma unroll
      for (int k = 0; k < NV; ++k) out[k] = (w0[k] + w0[ws + k]) + (w0[2 * ws + k] + w0[3 * ws + k]);
    }
    __syncthreads();
    return;
  }
  const int rl = 256 / cvl, nout = cvl * NV;
  if (row_lane < rl) {
    float* mine = smem + (row_lane * cvl + cv_lane) * NV;
#pragma unroll
    for (int k = 0; k < NV; ++k) mine[k] = acc[k];
  }
  __syncthreads();
  for (int o = threadIdx.x; o < nout; o += 256) {
    float sum = smem[o];
    for (int r = 1; r < rl; ++r) sum += smem[r * nout + o];
    smem[o] = sum;       // column o of row 0 is read by this thread only
  }
  __syncthreads();
  if (owner) {
#pragma unroll
    for (int k = 0; k < NV; ++k) out[k] = smem[cv_lane * NV + k];
  }
  __syncthreads();
}

// training-mode BN + activation:  z = act((y - mean) * (gamma*invstd) + beta).
// Column-grid launch: a thread keeps its 8 channels' coefficients in registers and streams rows.
// what a value reads back as after it was stored in T
template <class T> __device__ __forceinline__ float as_stored(float v);
template <> __device__ __forceinline__ float as_stored<float>(float v) { return v; }
template <> __device__ __forceinline__ float as_stored<bf16_t>(float v) { return bf_lo(pack_bf2(v, 0.f)); }

// res (optional): a residual add fused into the pass, z = res_act(stored(act(bn(y))) + res): the same
// numbers as storing the normalised tensor and adding in a second kernel, without that tensor
template <class T, bool STREAM = false>
__global__ __launch_bounds__(256) void bn_apply_kernel(const T* __restrict__ y, T* __restrict__ z,
                                                       const float* __restrict__ mean,
                                                       const float* __restrict__ invstd,
                                                       const float* __restrict__ gamma,
                                                       const float* __restrict__ beta, long M, int Cp,
                                                       int act, ColGrid g, const T* __restrict__ res, int res_act) {
  const int ncv = Cp / 8;
  const int cv_lane = threadIdx.x % g.cvl, row_lane = threadIdx.x / g.cvl, rl = 256 / g.cvl;
  const int cv = blockIdx.x * g.cvl + cv_lane;
  if (cv >= ncv || row_lane >= rl) return;
  const long r0 = blockIdx.y * g.rows_per_chunk;
  const long r1 = min(M, r0 + g.rows_per_chunk);
  float mu[8], a[8], b[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const int c = cv * 8 + k;
    mu[k] = mean[c]; a[k] = gamma[c] * invstd[c]; b[k] = beta[c];
  }
  long r = r0 + row_lane;
  for (; r + 3 * rl < r1; r += 4 * rl) {             // four rows (with a residual: eight loads) in flight
    typename IO<T>::Raw yr[4], sr[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) yr[u] = IO<T>::template ld_raw_t<STREAM>(y + ((r + u * rl) * ncv + cv) * 8);
    if (res) {
#pragma unroll
      for (int u = 0; u < 4; ++u) sr[u] = IO<T>::template ld_raw_t<STREAM>(res + ((r + u * rl) * ncv + cv) * 8);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      float v[8];
      IO<T>::unpack(yr[u], v);
#pragma unroll
      for (int k = 0; k < 8; ++k) v[k] = apply_act(fmaf(v[k] - mu[k], a[k], b[k]), act);
      if (res) {
        float s[8];
        IO<T>::unpack(sr[u], s);
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = apply_act(as_stored<T>(v[k]) + s[k], res_act);
      }
      IO<T>::template st_t<STREAM>(z + ((r + u * rl) * ncv + cv) * 8, v);
    }
  }
  for (; r < r1; r += rl) {
    float v[8];
    IO<T>::ld(y + (r * ncv + cv) * 8, v);
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = apply_act(fmaf(v[k] - mu[k], a[k], b[k]), act);
    if (res) {
      float s[8];
      IO<T>::ld(res + (r * ncv + cv) * 8, s);
#pragma unroll
      for (int k = 0; k < 8; ++k) v[k] = apply_act(as_stored<T>(v[k]) + s[k], res_act);
    }
    IO<T>::template st_t<STREAM>(z + (r * ncv + cv) * 8, v);
  }
}

// part[chunk][0][c] = sum (y - piv), part[chunk][1][c] = sum (y - piv)^2 with the pivot
// piv[c] = y[row 0][c]: shifting by a sample of the channel keeps the variance free of the
// cancellation that  E[y^2] - mean^2  suffers when |mean| >> std
template <class T, bool STREAM = false>
__global__ __launch_bounds__(256) void bn_stats_kernel(const T* __restrict__ y, float* __restrict__ part,
                                                       long M, int Cp, ColGrid g) {
  extern __shared__ float smem[];
  const int ncv = Cp / 8;
  const int cv_lane = threadIdx.x % g.cvl, row_lane = threadIdx.x / g.cvl, rl = 256 / g.cvl;
  const int cv = blockIdx.x * g.cvl + cv_lane;
  const long r0 = blockIdx.y * g.rows_per_chunk;
  const long r1 = min(M, r0 + g.rows_per_chunk);
  float acc[16];
#pragma unroll
  for (int k = 0; k < 16; ++k) acc[k] = 0.f;
  if (cv < ncv && row_lane < rl) {
    float piv[8];
    IO<T>::ld(y + (long)cv * 8, piv);
    long r = r0 + row_lane;
    for (; r + 3 * rl < r1; r += 4 * rl) {           // four rows in flight
      typename IO<T>::Raw yr[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) yr[u] = IO<T>::template ld_raw_t<STREAM>(y + ((r + u * rl) * ncv + cv) * 8);
      __builtin_amdgcn_sched_barrier(0);
      float v[4][8];
#pragma unroll
      for (int u = 0; u < 4; ++u) IO<T>::unpack(yr[u], v[u]);
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const float d = v[u][k] - piv[k];
          acc[k] += d;
          acc[8 + k] = fmaf(d, d, acc[8 + k]);
        }
    }
    for (; r < r1; r += rl) {
      float v[8];
      IO<T>::ld(y + (r * ncv + cv) * 8, v);
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const float d = v[k] - piv[k];
        acc[k] += d;
        acc[8 + k] = fmaf(d, d, acc[8 + k]);
      }
    }
  }
  float out[16];
  bool owner;
  block_col_reduce<16>(acc, smem, g.cvl, cv_lane, row_lane, out, owner);
  if (owner && cv < ncv) {
    float* p = part + (long)blockIdx.y * 2 * Cp + cv * 8;
#pragma unroll
    for (int k = 0; k < 8; ++k) { p[k] = out[k]; p[Cp + k] = out[8 + k]; }
  }
}

// Finalize kernels run 8 channels x 32 lanes per block (thread = lane * 8 + channel): lane l adds
// chunks l, l+32, ... in order, the 8 lanes of a channel inside one wave are added by a butterfly and
// the 4 waves in a fixed order (fixed association, independent of scheduling).  Few chunks per lane
// keep the chain of dependent loads short: these kernels sit between two passes over the tensor.
constexpr int kFinalizeChannels = 8;
__device__ __forceinline__ void finalize_sums(const float* __restrict__ part, int chunks, int Cp, int c,
                                              int lane, double& s1, double& s2) {
  __shared__ double red1[4][kFinalizeChannels], red2[4][kFinalizeChannels];
  const int cl = threadIdx.x & (kFinalizeChannels - 1);
  double a = 0.0, b = 0.0;
  if (c < Cp) {
#pragma unroll 4
    for (int k = lane; k < chunks; k += 32) {
      a += (double)part[(long)k * 2 * Cp + c];
      b += (double)part[(long)k * 2 * Cp + Cp + c];
    }
  }
#pragma unroll
  for (int off = kFinalizeChannels; off < 64; off <<= 1) {
    a += __shfl_xor(a, off, 64);
    b += __shfl_xor(b, off, 64);
  }
  if ((threadIdx.x & 63) < kFinalizeChannels) {
    red1[threadIdx.x >> 6][cl] = a;
    red2[threadIdx.x >> 6][cl] = b;
  }
  __syncthreads();
  s1 = (red1[0][cl] + red1[1][cl]) + (red1[2][cl] + red1[3][cl]);
  s2 = (red2[0][cl] + red2[1][cl]) + (red2[2][cl] + red2[3][cl]);
}

// mean, biased variance -> inv std; running statistics
//   rm <- (1-rho) rm + rho mean,  rv <- (1-rho) rv + rho var m/(m-1)
template <class T>
__global__ void bn_finalize_kernel(const float* __restrict__ part, const T* __restrict__ y, int chunks,
                                   int Cp, double m, float* mean, float* invstd, float* rmean,
                                   float* rvar, float eps, float rho) {
  const int c = blockIdx.x * kFinalizeChannels + (threadIdx.x & (kFinalizeChannels - 1)), lane = threadIdx.x >> 3;
  double s1, s2;
  finalize_sums(part, chunks, Cp, c, lane, s1, s2);
  if (c >= Cp || lane != 0) return;
  const double shift = s1 / m;
  const double mu = (y ? (double)(float)y[c] : 0.0) + shift;     // y: the pivot row the sums were shifted by, if any
  double var = s2 / m - shift * shift;
  if (var < 0.0) var = 0.0;
  mean[c] = (float)mu;
  invstd[c] = (float)(1.0 / sqrt(var + (double)eps));
  rmean[c] = (1.f - rho) * rmean[c] + rho * (float)mu;
  rvar[c] = (1.f - rho) * rvar[c] + rho * (float)(var * m / (m - 1.0));
}

// out[g][i] = sum of part[k][i] over the `per` chunks of group g, in order: shortens the list of partial
// sums that a finalize kernel walks through when a convolution's row tiles delivered thousands of them
constexpr int kStatGroupsMax = 1024;   // partial sums a batch-norm finalize walks through at most
__global__ void regroup_partials_kernel(const float* __restrict__ part, float* __restrict__ out, int chunks, int n, int per) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int k0 = blockIdx.y * per, k1 = min(chunks, k0 + per);
  float s = 0.f;
  for (int k = k0; k < k1; ++k) s += part[(long)k * n + i];
  out[(long)blockIdx.y * n + i] = s;
}

// BN backward, stage 1: with xhat = (y - mean)*invstd, pre = gamma*xhat + beta and
// dpre = [act passes at pre] * dz:  part[chunk][0][c] = sum dpre, part[chunk][1][c] = sum dpre*xhat
// RES: the layer's output went straight into a two-input add (fused into its normalisation pass on the way
// forward).  dz is then the gradient of the add's output and zres that output: the gradient passes where the
// add's activation res_act does (zres == nullptr: no activation), is stored to dstore (the gradient of both
// inputs of the add: the backward pass of the add itself, done here) and enters the sums.
// LOSS (with RES and zres): the add's output is the block's output S.  dz is then the teacher's activation A,
// the gradient of the add's output is 2 (S - A) / M rounded as it would be stored (Sec. II-A, the loss of the
// block's output), and loss_part[workgroup] = sum (S - A)^2 over the workgroup's elements.
template <class T, bool RES = false, bool LOSS = false, bool STREAM = false>
__global__ __launch_bounds__(256) void bn_bwd_reduce_kernel(
    const T* __restrict__ dz, const T* __restrict__ y, const float* __restrict__ gamma,
    const float* __restrict__ beta, const float* __restrict__ mean, const float* __restrict__ invstd,
    float* __restrict__ part, long M, int Cp, int act, ColGrid g, const T* __restrict__ zres = nullptr,
    int res_act = 0, T* __restrict__ dstore = nullptr, float* __restrict__ loss_part = nullptr,
    float two_over_m = 0.f) {
  static_assert(RES || !LOSS, "the loss rides only where the add does");
  float lacc = 0.f;
  extern __shared__ float smem[];
  const int ncv = Cp / 8;
  const int cv_lane = threadIdx.x % g.cvl, row_lane = threadIdx.x / g.cvl, rl = 256 / g.cvl;
  const int cv = blockIdx.x * g.cvl + cv_lane;
  const long r0 = blockIdx.y * g.rows_per_chunk;
  const long r1 = min(M, r0 + g.rows_per_chunk);
  float acc[16];
#pragma unroll
  for (int k = 0; k < 16; ++k) acc[k] = 0.f;
  if (cv < ncv && row_lane < rl) {
    float av[8], bv[8], mv[8], iv[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      av[k] = gamma[cv * 8 + k]; bv[k] = beta[cv * 8 + k]; mv[k] = mean[cv * 8 + k]; iv[k] = invstd[cv * 8 + k];
    }
    float sc[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) sc[k] = av[k] * iv[k];
    long r = r0 + row_lane;
    for (; r + 3 * rl < r1; r += 4 * rl) {           // four rows (eight loads, twelve with an add's output) in flight
      typename IO<T>::Raw dr[4], yr[4], zr[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        dr[u] = IO<T>::template ld_raw_t<STREAM>(dz + ((r + u * rl) * ncv + cv) * 8);
        yr[u] = IO<T>::template ld_raw_t<STREAM>(y + ((r + u * rl) * ncv + cv) * 8);
      }
      if (RES && zres) {
#pragma unroll
        for (int u = 0; u < 4; ++u) zr[u] = IO<T>::template ld_raw_t<STREAM>(zres + ((r + u * rl) * ncv + cv) * 8);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        float d[8], v[8];
        IO<T>::unpack(dr[u], d);
        IO<T>::unpack(yr[u], v);
        if (RES) {
          if (zres) {
            float z[8];
            IO<T>::unpack(zr[u], z);
            if (LOSS) {
#pragma unroll
              for (int k = 0; k < 8; ++k) {
                const float e = z[k] - d[k];
                lacc = fmaf(e, e, lacc);
                d[k] = as_stored<T>(e * two_over_m);
              }
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) d[k] = act_pass(z[k], res_act) ? d[k] : 0.f;
          }
          IO<T>::template st_t<STREAM>(dstore + ((r + u * rl) * ncv + cv) * 8, d);
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const float yc = v[k] - mv[k];
          const float dp = act_pass(fmaf(yc, sc[k], bv[k]), act) ? d[k] : 0.f;
          acc[k] += dp;
          acc[8 + k] = fmaf(dp, yc * iv[k], acc[8 + k]);
        }
      }
    }
    for (; r < r1; r += rl) {
      float d[8], v[8];
      IO<T>::ld(dz + (r * ncv + cv) * 8, d);
      IO<T>::ld(y + (r * ncv + cv) * 8, v);
      if (RES) {
        if (zres) {
          float z[8];
          IO<T>::ld(zres + (r * ncv + cv) * 8, z);
          if (LOSS) {
#pragma unroll
            for (int k = 0; k < 8; ++k) {
              const float e = z[k] - d[k];
              lacc = fmaf(e, e, lacc);
              d[k] = as_stored<T>(e * two_over_m);
            }
          }
#pragma unroll
          for (int k = 0; k < 8; ++k) d[k] = act_pass(z[k], res_act) ? d[k] : 0.f;
        }
        IO<T>::template st_t<STREAM>(dstore + (r * ncv + cv) * 8, d);
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const float yc = v[k] - mv[k];
        const float dp = act_pass(fmaf(yc, sc[k], bv[k]), act) ? d[k] : 0.f;
        acc[k] += dp;
        acc[8 + k] = fmaf(dp, yc * iv[k], acc[8 + k]);
      }
    }
  }
  float out[16];
  bool owner;
  block_col_reduce<16>(acc, smem, g.cvl, cv_lane, row_lane, out, owner);
  if (owner && cv < ncv) {
    float* p = part + (long)blockIdx.y * 2 * Cp + cv * 8;
#pragma unroll
    for (int k = 0; k < 8; ++k) { p[k] = out[k]; p[Cp + k] = out[8 + k]; }
  }
  if (LOSS) {                                        // the workgroup's share of sum (S - A)^2, added in a fixed order
    __syncthreads();
    smem[threadIdx.x] = lacc;
    __syncthreads();
    for (int h = 128; h > 0; h >>= 1) {
      if ((int)threadIdx.x < h) smem[threadIdx.x] += smem[threadIdx.x + h];
      __syncthreads();
    }
    if (threadIdx.x == 0) loss_part[blockIdx.y * gridDim.x + blockIdx.x] = smem[0];
  }
}

// stage 2: dbeta, dgamma (the parameter gradients) and the per-channel terms
// k2 = dbeta/m, k3 = dgamma/m of  dy = gamma*invstd*(dpre - k2 - xhat*k3)
__global__ void bn_bwd_finalize_kernel(const float* __restrict__ part, int chunks, int Cp, double m,
                                       float* g_gamma, float* g_beta, float* k2, float* k3) {
  const int c = blockIdx.x * kFinalizeChannels + (threadIdx.x & (kFinalizeChannels - 1)), lane = threadIdx.x >> 3;
  double sb, sg;
  finalize_sums(part, chunks, Cp, c, lane, sb, sg);
  if (c >= Cp || lane != 0) return;
  g_beta[c] = (float)sb;
  g_gamma[c] = (float)sg;
  k2[c] = (float)(sb / m);
  k3[c] = (float)(sg / m);
}

// stage 3: gradient w.r.t. the convolution output, written to dy (dy == dz: in place; column-grid launch, each
// thread reads its elements before it writes them)
template <class T, bool STREAM = false>
__global__ __launch_bounds__(256) void bn_bwd_apply_kernel(
    const T* dz, T* dy, const T* __restrict__ y, const float* __restrict__ gamma,
    const float* __restrict__ beta, const float* __restrict__ mean, const float* __restrict__ invstd,
    const float* __restrict__ k2, const float* __restrict__ k3, long M, int Cp, int act, ColGrid g) {
  const int ncv = Cp / 8;
  const int cv_lane = threadIdx.x % g.cvl, row_lane = threadIdx.x / g.cvl, rl = 256 / g.cvl;
  const int cv = blockIdx.x * g.cvl + cv_lane;
  if (cv >= ncv || row_lane >= rl) return;
  const long r0 = blockIdx.y * g.rows_per_chunk;
  const long r1 = min(M, r0 + g.rows_per_chunk);
  float mu[8], a[8], b[8], is[8], c2[8], c3[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const int c = cv * 8 + k;
    mu[k] = mean[c]; is[k] = invstd[c]; a[k] = gamma[c] * is[k]; b[k] = beta[c];
    c2[k] = k2[c]; c3[k] = k3[c];
  }
  long r = r0 + row_lane;
  for (; r + 3 * rl < r1; r += 4 * rl) {             // four rows (eight loads) in flight
    typename IO<T>::Raw dr[4], yr[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      dr[u] = IO<T>::template ld_raw_t<STREAM>(dz + ((r + u * rl) * ncv + cv) * 8);
      yr[u] = IO<T>::template ld_raw_t<STREAM>(y + ((r + u * rl) * ncv + cv) * 8);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      float d[8], v[8];
      IO<T>::unpack(dr[u], d);
      IO<T>::unpack(yr[u], v);
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const float yc = v[k] - mu[k];
        const float dp = act_pass(fmaf(yc, a[k], b[k]), act) ? d[k] : 0.f;
        d[k] = a[k] * (dp - c2[k] - yc * is[k] * c3[k]);
      }
      IO<T>::template st_t<STREAM>(dy + ((r + u * rl) * ncv + cv) * 8, d);
    }
  }
  for (; r < r1; r += rl) {
    float d[8], v[8];
    IO<T>::ld(dz + (r * ncv + cv) * 8, d);
    IO<T>::ld(y + (r * ncv + cv) * 8, v);
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const float yc = v[k] - mu[k];
      const float dp = act_pass(fmaf(yc, a[k], b[k]), act) ? d[k] : 0.f;
      d[k] = a[k] * (dp - c2[k] - yc * is[k] * c3[k]);
    }
    IO<T>::template st_t<STREAM>(dy + (r * ncv + cv) * 8, d);
  }
}

// ---------------------------------------------------------------------------
// Whole-column kernels for short matrices (M <= 4096 rows).  One block of 512 threads owns an
// 8-channel slab over ALL rows and keeps its (at most 8) rows per thread in registers, so
// statistics, their finalisation and the elementwise pass are one launch and one read instead of
// three launches and two reads: at these sizes the launches, not the bytes, are the cost.
// ---------------------------------------------------------------------------
constexpr int kSmallThreads = 512;                   // 8 waves: up to 256 registers per thread
constexpr int kSmallRows = 8;                        // rows per thread

// consecutive slabs go to the same XCD (blocks are dealt round-robin over 8 XCDs), so each cache
// line of a row is pulled into one L2 only
__device__ __forceinline__ int xcd_slab(int b, int nslab) {
  return (nslab & 7) == 0 ? (b & 7) * (nslab >> 3) + (b >> 3) : b;
}

// Sum of 16 per-thread values over the block, result in every thread.  In the wave: a
// reduce-scatter butterfly (exchange half of the values with lane^32, a quarter with lane^16, ...:
// 17 cross-lane moves instead of 96), float.  Across the waves: added in order, in double (BN
// backward subtracts these means from the gradient and what is left feeds weight gradients whose
// own sum cancels, so the totals want more than float).  A fixed association throughout.
__device__ __forceinline__ void block_sum16(const float (&v)[16], double (&out)[16], float (*red)[16], double* tot) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float w8[8], w4[4], w2[2], w1;
  const bool h32 = lane & 32, h16 = lane & 16, h8 = lane & 8, h4 = lane & 4;
#pragma unroll
  for (int i = 0; i < 8; ++i) w8[i] = (h32 ? v[8 + i] : v[i]) + __shfl_xor(h32 ? v[i] : v[8 + i], 32, 64);
#pragma unroll
  for (int i = 0; i < 4; ++i) w4[i] = (h16 ? w8[4 + i] : w8[i]) + __shfl_xor(h16 ? w8[i] : w8[4 + i], 16, 64);
#pragma unroll
  for (int i = 0; i < 2; ++i) w2[i] = (h8 ? w4[2 + i] : w4[i]) + __shfl_xor(h8 ? w4[i] : w4[2 + i], 8, 64);
  w1 = (h4 ? w2[1] : w2[0]) + __shfl_xor(h4 ? w2[0] : w2[1], 4, 64);
  w1 += __shfl_xor(w1, 2, 64);
  w1 += __shfl_xor(w1, 1, 64);
  if ((lane & 3) == 0) red[wave][(h32 ? 8 : 0) + (h16 ? 4 : 0) + (h8 ? 2 : 0) + (h4 ? 1 : 0)] = w1;
  __syncthreads();
  if (threadIdx.x < 16) {
    double t = (double)red[0][threadIdx.x];
#pragma unroll 1
    for (int w = 1; w < kSmallThreads / 64; ++w) t += (double)red[w][threadIdx.x];
    tot[threadIdx.x] = t;
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 16; ++k) out[k] = tot[k];
}

// y -> batch statistics (pivot-shifted sums as in bn_stats_kernel), running statistics, then
// z = act((y - mean) * (gamma*invstd) + beta)
template <class T>
__global__ __launch_bounds__(kSmallThreads) void bn_small_fwd_kernel(
    const T* __restrict__ y, T* __restrict__ z, const float* __restrict__ gamma, const float* __restrict__ beta,
    float* __restrict__ mean, float* __restrict__ invstd, float* __restrict__ rmean, float* __restrict__ rvar,
    int M, int Cp, float eps, float rho, int act, unsigned bytes) {
  __shared__ float red[kSmallThreads / 64][16];
  __shared__ double tot[16];
  const int ncv = Cp / 8, cv = xcd_slab(blockIdx.x, ncv), tid = threadIdx.x;
  const __amdgpu_buffer_rsrc_t ry = tensor_rsrc(y, bytes);
  typename BufIO<T>::Raw raw[kSmallRows];
#pragma unroll
  for (int u = 0; u < kSmallRows; ++u) {
    const int r = u * kSmallThreads + tid;
    raw[u] = BufIO<T>::issue(ry, (unsigned)(r * ncv + cv) * 8u, r < M);
  }
  float piv[8];
  IO<T>::ld(y + (long)cv * 8, piv);
  float acc[16];
#pragma unroll
  for (int k = 0; k < 16; ++k) acc[k] = 0.f;
#pragma unroll
  for (int u = 0; u < kSmallRows; ++u) {
    if (u * kSmallThreads + (tid & ~63) >= M) continue;     // no lane of this wave owns the row
    const bool ok = u * kSmallThreads + tid < M;
    float v[8];
    BufIO<T>::unpack(raw[u], v);
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const float d = ok ? v[k] - piv[k] : 0.f;
      acc[k] += d;
      acc[8 + k] = fmaf(d, d, acc[8 + k]);
    }
  }
  double sum[16];
  block_sum16(acc, sum, red, tot);
  // thread k < 8 finalises channel k in double (once, not in every thread) and hands the float
  // coefficients to the block through LDS
  __shared__ float coef[3][8];
  if (tid < 8) {
    const int c = cv * 8 + tid;
    const double m = (double)M;
    double s1 = 0.0, s2 = 0.0;
    float pv = 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k)
      if (k == tid) { s1 = sum[k]; s2 = sum[8 + k]; pv = piv[k]; }
    const double shift = s1 / m;
    const double mean_d = (double)pv + shift;
    double var = s2 / m - shift * shift;
    if (var < 0.0) var = 0.0;
    const float is = (float)(1.0 / sqrt(var + (double)eps));
    const float muf = (float)mean_d;
    mean[c] = muf;
    invstd[c] = is;
    rmean[c] = (1.f - rho) * rmean[c] + rho * muf;
    rvar[c] = (1.f - rho) * rvar[c] + rho * (float)(var * m / (m - 1.0));
    coef[0][tid] = muf; coef[1][tid] = gamma[c] * is; coef[2][tid] = beta[c];
  }
  __syncthreads();
  float mu[8], a[8], b[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) { mu[k] = coef[0][k]; a[k] = coef[1][k]; b[k] = coef[2][k]; }
#pragma unroll
  for (int u = 0; u < kSmallRows; ++u) {
    const int r = u * kSmallThreads + tid;
    if (r >= M) continue;
    float v[8];
    BufIO<T>::unpack(raw[u], v);
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = apply_act(fmaf(v[k] - mu[k], a[k], b[k]), act);
    IO<T>::st(z + ((long)r * ncv + cv) * 8, v);
  }
}

// BN backward in one launch: sums of dpre and dpre*xhat, the parameter gradients, then
// dy = gamma*invstd*(dpre - dbeta/m - xhat*dgamma/m) over dz in place
template <class T>
__global__ __launch_bounds__(kSmallThreads) void bn_small_bwd_kernel(
    T* dz, const T* __restrict__ y, const float* __restrict__ gamma, const float* __restrict__ beta,
    const float* __restrict__ mean, const float* __restrict__ invstd, float* __restrict__ g_gamma,
    float* __restrict__ g_beta, int M, int Cp, int act, unsigned bytes) {
  __shared__ float red[kSmallThreads / 64][16];
  __shared__ double tot[16];
  const int ncv = Cp / 8, cv = xcd_slab(blockIdx.x, ncv), tid = threadIdx.x;
  const __amdgpu_buffer_rsrc_t ry = tensor_rsrc(y, bytes), rd = tensor_rsrc(dz, bytes);
  typename BufIO<T>::Raw rawd[kSmallRows], rawy[kSmallRows];
#pragma unroll
  for (int u = 0; u < kSmallRows; ++u) {
    const int r = u * kSmallThreads + tid;
    rawd[u] = BufIO<T>::issue(rd, (unsigned)(r * ncv + cv) * 8u, r < M);
    rawy[u] = BufIO<T>::issue(ry, (unsigned)(r * ncv + cv) * 8u, r < M);
  }
  float mu[8], a[8], b[8], is[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const int c = cv * 8 + k;
    mu[k] = mean[c]; is[k] = invstd[c]; a[k] = gamma[c] * is[k]; b[k] = beta[c];
  }
  float acc[16];
#pragma unroll
  for (int k = 0; k < 16; ++k) acc[k] = 0.f;
#pragma unroll
  for (int u = 0; u < kSmallRows; ++u) {
    if (u * kSmallThreads + (tid & ~63) >= M) continue;     // no lane of this wave owns the row
    float d[8], v[8];                                // rows past M read as dz = 0: they add nothing
    BufIO<T>::unpack(rawd[u], d);
    BufIO<T>::unpack(rawy[u], v);
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const float yc = v[k] - mu[k];
      const float dp = act_pass(fmaf(yc, a[k], b[k]), act) ? d[k] : 0.f;
      acc[k] += dp;
      acc[8 + k] = fmaf(dp, yc * is[k], acc[8 + k]);
    }
  }
  double sum[16];
  block_sum16(acc, sum, red, tot);
  __shared__ float coef[2][8];
  if (tid < 8) {
    double sb = 0.0, sg = 0.0;
#pragma unroll
    for (int k = 0; k < 8; ++k)
      if (k == tid) { sb = sum[k]; sg = sum[8 + k]; }
    const double m = (double)M;
    g_beta[cv * 8 + tid] = (float)sb;
    g_gamma[cv * 8 + tid] = (float)sg;
    coef[0][tid] = (float)(sb / m);
    coef[1][tid] = (float)(sg / m);
  }
  __syncthreads();
  float c2[8], c3[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) { c2[k] = coef[0][k]; c3[k] = coef[1][k]; }
#pragma unroll
  for (int u = 0; u < kSmallRows; ++u) {
    const int r = u * kSmallThreads + tid;
    if (r >= M) continue;
    float d[8], v[8];
    BufIO<T>::unpack(rawd[u], d);
    BufIO<T>::unpack(rawy[u], v);
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const float yc = v[k] - mu[k];
      const float dp = act_pass(fmaf(yc, a[k], b[k]), act) ? d[k] : 0.f;
      d[k] = a[k] * (dp - c2[k] - yc * is[k] * c3[k]);
    }
    IO<T>::st(dz + ((long)r * ncv + cv) * 8, d);
  }
}

// ---------------------------------------------------------------------------
// max-pool; idx keeps the window position r*k+t of the first maximum
// ---------------------------------------------------------------------------
// The producing layer's normalisation and activation applied to every element a pool reads (mean == nullptr: x is
// read as it is): x is then that layer's convolution output, each element becomes what bn_apply_kernel would have
// stored (same arithmetic, same rounding), and the normalised tensor, which only the pool reads, is never written.
struct NormFold { const float* mean; const float* invstd; const float* gamma; const float* beta; int act; };

template <class T>
__global__ void maxpool_fwd_kernel(const T* __restrict__ x, T* __restrict__ z, uint8_t* __restrict__ idx,
                                   int N, int H, int W, int P, int Q, int ncv, int k, int stride, int pad,
                                   NormFold fold) {
  const long nvec = (long)N * P * Q * ncv;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < nvec; i += (long)gridDim.x * blockDim.x) {
    const int cv = (int)(i % ncv);
    long pix = i / ncv;
    const int q = (int)(pix % Q); pix /= Q;
    const int p = (int)(pix % P);
    const int n = (int)(pix / P);
    float best[8];
    int bi[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { best[e] = 0.f; bi[e] = -1; }
    float mu[8], fa[8], fb[8];
    if (fold.mean) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int ch = cv * 8 + e;
        mu[e] = fold.mean[ch]; fa[e] = fold.gamma[ch] * fold.invstd[ch]; fb[e] = fold.beta[ch];
      }
    }
    for (int r = 0; r < k; ++r) {
      const int h = p * stride + r - pad;
      if (h < 0 || h >= H) continue;
      for (int t = 0; t < k; ++t) {
        const int w = q * stride + t - pad;
        if (w < 0 || w >= W) continue;
        float v[8];
        IO<T>::ld(x + ((((long)n * H + h) * W + w) * ncv + cv) * 8, v);
        if (fold.mean) {
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] = as_stored<T>(apply_act(fmaf(v[e] - mu[e], fa[e], fb[e]), fold.act));
        }
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (bi[e] < 0 || v[e] > best[e]) { best[e] = v[e]; bi[e] = r * k + t; }
      }
    }
    IO<T>::st(z + i * 8, best);
    if (idx) {
      uint2 pk;
      pk.x = (uint32_t)bi[0] | ((uint32_t)bi[1] << 8) | ((uint32_t)bi[2] << 16) | ((uint32_t)bi[3] << 24);
      pk.y = (uint32_t)bi[4] | ((uint32_t)bi[5] << 8) | ((uint32_t)bi[6] << 16) | ((uint32_t)bi[7] << 24);
      *reinterpret_cast<uint2*>(idx + i * 8) = pk;
    }
  }
}

// The 3 x 3, stride-2, pad-1 pool (the ResNet stem's) with all nine taps of a window loaded before the first is looked at
// (out-of-range taps read a clamped position and are skipped): one memory latency per window instead of one per
// tap.  Same values and window positions as maxpool_fwd_kernel.
template <class T>
__global__ void maxpool_fwd_k3s2_kernel(const T* __restrict__ x, T* __restrict__ z, uint8_t* __restrict__ idx,
                                        int N, int H, int W, int P, int Q, int ncv, NormFold fold) {
  const long nvec = (long)N * P * Q * ncv;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < nvec; i += (long)gridDim.x * blockDim.x) {
    const int cv = (int)(i % ncv);
    long pix = i / ncv;
    const int q = (int)(pix % Q); pix /= Q;
    const int p = (int)(pix % P);
    const int n = (int)(pix / P);
    float mu[8], fa[8], fb[8];
    if (fold.mean) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int ch = cv * 8 + e;
        mu[e] = fold.mean[ch]; fa[e] = fold.gamma[ch] * fold.invstd[ch]; fb[e] = fold.beta[ch];
      }
    }
    typename IO<T>::Raw raw[9];
    unsigned ok = 0;
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) {
      const int h = 2 * p - 1 + tap / 3, w = 2 * q - 1 + tap % 3;
      if (h >= 0 && h < H && w >= 0 && w < W) ok |= 1u << tap;
      const int hc = min(max(h, 0), H - 1), wc = min(max(w, 0), W - 1);
      raw[tap] = IO<T>::ld_raw(x + ((((long)n * H + hc) * W + wc) * ncv + cv) * 8);
    }
    __builtin_amdgcn_sched_barrier(0);
    float best[8];
    int bi[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { best[e] = 0.f; bi[e] = -1; }
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) {
      if (!(ok >> tap & 1)) continue;
      float v[8];
      IO<T>::unpack(raw[tap], v);
      if (fold.mean) {
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = as_stored<T>(apply_act(fmaf(v[e] - mu[e], fa[e], fb[e]), fold.act));
      }
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (bi[e] < 0 || v[e] > best[e]) { best[e] = v[e]; bi[e] = tap; }
    }
    IO<T>::st(z + i * 8, best);
    if (idx) {
      uint2 pk;
      pk.x = (uint32_t)bi[0] | ((uint32_t)bi[1] << 8) | ((uint32_t)bi[2] << 16) | ((uint32_t)bi[3] << 24);
      pk.y = (uint32_t)bi[4] | ((uint32_t)bi[5] << 8) | ((uint32_t)bi[6] << 16) | ((uint32_t)bi[7] << 24);
      *reinterpret_cast<uint2*>(idx + i * 8) = pk;
    }
  }
}

// Its backward pass: an input pixel lies in one window per direction when its coordinate is even (tap 1) and in two when
// it is odd (taps 0 and 2), so at most four windows, whose positions and gradients are all loaded before the first
// comparison; contributions are added in the tap order of maxpool_bwd_kernel.
template <class T>
__global__ void maxpool_bwd_k3s2_kernel(const T* __restrict__ dz, const uint8_t* __restrict__ idx,
                                        T* __restrict__ dx, int N, int H, int W, int P, int Q, int ncv, int accumulate) {
  const long nvec = (long)N * H * W * ncv;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < nvec; i += (long)gridDim.x * blockDim.x) {
    const int cv = (int)(i % ncv);
    long pix = i / ncv;
    const int w = (int)(pix % W); pix /= W;
    const int h = (int)(pix % H);
    const int n = (int)(pix / H);
    // candidate windows per direction, in tap order: odd coordinate: tap 0 of window (c + 1) / 2, tap 2 of (c - 1) / 2;
    // even: tap 1 of window c / 2
    int pr[2], rr[2], qc[2], tc[2];
    bool pv[2], qv[2];
    if (h & 1) { rr[0] = 0; pr[0] = (h + 1) >> 1; pv[0] = pr[0] < P; rr[1] = 2; pr[1] = (h - 1) >> 1; pv[1] = pr[1] < P; }
    else { rr[0] = 1; pr[0] = h >> 1; pv[0] = pr[0] < P; rr[1] = 0; pr[1] = 0; pv[1] = false; }
    if (w & 1) { tc[0] = 0; qc[0] = (w + 1) >> 1; qv[0] = qc[0] < Q; tc[1] = 2; qc[1] = (w - 1) >> 1; qv[1] = qc[1] < Q; }
    else { tc[0] = 1; qc[0] = w >> 1; qv[0] = qc[0] < Q; tc[1] = 0; qc[1] = 0; qv[1] = false; }
    uint2 pk[4];
    typename IO<T>::Raw raw[4];
    bool valid[4];
    uint32_t me[4];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        const int k = a * 2 + b;
        valid[k] = pv[a] && qv[b];
        const int pp = min(pr[a], P - 1), qq = min(qc[b], Q - 1);
        const long o = ((((long)n * P + pp) * Q + qq) * ncv + cv) * 8;
        pk[k] = *reinterpret_cast<const uint2*>(idx + o);
        raw[k] = IO<T>::ld_raw(dz + o);
        me[k] = (uint32_t)(rr[a] * 3 + tc[b]);
      }
    float acc[8];
    if (accumulate) IO<T>::ld(dx + i * 8, acc);
    else {
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      float d[8];
      IO<T>::unpack(raw[k], d);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint32_t word = e < 4 ? pk[k].x : pk[k].y;
        if (valid[k] && ((word >> (8 * (e & 3))) & 0xffu) == me[k]) acc[e] += d[e];
      }
    }
    IO<T>::st(dx + i * 8, acc);
  }
}

// gather form: every input pixel collects from the windows that chose it
template <class T>
__global__ void maxpool_bwd_kernel(const T* __restrict__ dz, const uint8_t* __restrict__ idx,
                                   T* __restrict__ dx, int N, int H, int W, int P, int Q, int ncv,
                                   int k, int stride, int pad, int accumulate) {
  const long nvec = (long)N * H * W * ncv;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < nvec; i += (long)gridDim.x * blockDim.x) {
    const int cv = (int)(i % ncv);
    long pix = i / ncv;
    const int w = (int)(pix % W); pix /= W;
    const int h = (int)(pix % H);
    const int n = (int)(pix / H);
    float acc[8];
    if (accumulate) IO<T>::ld(dx + i * 8, acc);
    else {
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    }
    for (int r = 0; r < k; ++r) {
      const int ph = h + pad - r;
      if (ph < 0 || ph % stride) continue;
      const int p = ph / stride;
      if (p >= P) continue;
      for (int t = 0; t < k; ++t) {
        const int qw = w + pad - t;
        if (qw < 0 || qw % stride) continue;
        const int q = qw / stride;
        if (q >= Q) continue;
        const long o = ((((long)n * P + p) * Q + q) * ncv + cv) * 8;
        const uint2 pk = *reinterpret_cast<const uint2*>(idx + o);
        float d[8];
        IO<T>::ld(dz + o, d);
        const uint32_t me = (uint32_t)(r * k + t);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const uint32_t word = e < 4 ? pk.x : pk.y;
          if (((word >> (8 * (e & 3))) & 0xffu) == me) acc[e] += d[e];
        }
      }
    }
    IO<T>::st(dx + i * 8, acc);
  }
}

// ---------------------------------------------------------------------------
// joins: z = act(sum_k p_k v_k) forward; backward fans  s_k*[act passes at z]*dz
// out to up to 8 destinations, each either written or accumulated
// ---------------------------------------------------------------------------
struct Join {
  const void* src[8];
  void* dst[8];
  float p[8];
  const float* pdev;     // when set, the weights are read from device memory instead (trainable mix)
  int accumulate[8];
  int n;
};

__device__ __forceinline__ void join_weights(const Join& j, float (&p)[8]) {
#pragma unroll
  for (int k = 0; k < 8; ++k) p[k] = k < j.n ? (j.pdev ? j.pdev[k] : j.p[k]) : 0.f;
}

template <class T>
__global__ void join_fwd_kernel(Join j, T* __restrict__ z, long nvec, int act) {
  float p[8];
  join_weights(j, p);
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < nvec; i += (long)gridDim.x * blockDim.x) {
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      if (k >= j.n) break;
      float v[8];
      IO<T>::ld(static_cast<const T*>(j.src[k]) + i * 8, v);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = fmaf(p[k], v[e], acc[e]);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = apply_act(acc[e], act);
    IO<T>::st(z + i * 8, acc);
  }
}

// z is the post-activation output: for ReLU the gradient passes where z > 0
template <class T>
__global__ void join_bwd_kernel(Join j, const T* __restrict__ dz, const T* __restrict__ z, long nvec, int act) {
  float p[8];
  join_weights(j, p);
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < nvec; i += (long)gridDim.x * blockDim.x) {
    float d[8];
    IO<T>::ld(dz + i * 8, d);
    if (act != ACT_NONE) {
      float v[8];
      IO<T>::ld(z + i * 8, v);
#pragma unroll
      for (int e = 0; e < 8; ++e) d[e] = act_pass(v[e], act) ? d[e] : 0.f;
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      if (k >= j.n) break;
      T* dst = static_cast<T*>(j.dst[k]);
      if (!dst) continue;
      float o[8];
      if (j.accumulate[k]) {
        IO<T>::ld(dst + i * 8, o);
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = fmaf(p[k], d[e], o[e]);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = p[k] * d[e];
      }
      IO<T>::st(dst + i * 8, o);
    }
  }
}

// ---------------------------------------------------------------------------
// architecture round of a supernet (Sec. VI-A, neural architecture search): a mix op computes
// z = act(sum_k p_k y_k) with p = softmax(alpha).  With d = dL/dz masked by the activation,
//   g_k = <d, y_k>,   dL/dalpha_j = p_j (g_j - sum_k p_k g_k).
// mix_dot_kernel leaves one partial g per workgroup; mix_alpha_update_kernel sums them in a fixed
// order, forms the gradient, applies  v <- mu v + g ; alpha <- alpha - lr v  and writes the new p.
// One mix op owns 32 floats of state: alpha[8], momentum[8], gradient[8], p[8].
// ---------------------------------------------------------------------------
constexpr int kMixState = 32, kMixAlpha = 0, kMixMom = 8, kMixGrad = 16, kMixP = 24;
constexpr int kMixDotBlocks = 512;

template <class T>
__global__ __launch_bounds__(256) void mix_dot_kernel(Join j, const T* __restrict__ dz, const T* __restrict__ z,
                                                      float* __restrict__ part, long nvec, int act) {
  __shared__ float red[4][8];
  float acc[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) acc[k] = 0.f;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < nvec; i += (long)gridDim.x * blockDim.x) {
    float d[8];
    IO<T>::ld(dz + i * 8, d);
    if (act != ACT_NONE) {
      float v[8];
      IO<T>::ld(z + i * 8, v);
#pragma unroll
      for (int e = 0; e < 8; ++e) d[e] = act_pass(v[e], act) ? d[e] : 0.f;
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      if (k >= j.n) break;
      float v[8];
      IO<T>::ld(static_cast<const T*>(j.src[k]) + i * 8, v);
      float s = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) s = fmaf(d[e], v[e], s);
      acc[k] += s;
    }
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    float v = acc[k];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    if (lane == 0) red[wave][k] = v;
  }
  __syncthreads();
  if (threadIdx.x < 8) part[blockIdx.x * 8 + threadIdx.x] = (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
}

// one workgroup of 256 threads; state = the mix op's 32 floats; update == 0 leaves alpha, momentum and p
__global__ __launch_bounds__(256) void mix_alpha_update_kernel(const float* __restrict__ part, int nblocks,
                                                               float* __restrict__ state, int n,
                                                               const float* __restrict__ lr_ptr, float mu, int update) {
  __shared__ double red[32][8];
  __shared__ double g[8];
  __shared__ float alpha[8];
  const int k = threadIdx.x & 7, row = threadIdx.x >> 3;
  double s = 0.0;
  for (int b = row; b < nblocks; b += 32) s += (double)part[b * 8 + k];
  red[row][k] = s;
  __syncthreads();
  for (int h = 16; h > 0; h >>= 1) {
    if (row < h) red[row][k] += red[row + h][k];
    __syncthreads();
  }
  if (threadIdx.x < 8) g[threadIdx.x] = red[0][threadIdx.x];
  __syncthreads();
  if ((int)threadIdx.x < n) {
    double mean = 0.0;
    for (int q = 0; q < n; ++q) mean += (double)state[kMixP + q] * g[q];
    const float grad = (float)((double)state[kMixP + threadIdx.x] * (g[threadIdx.x] - mean));
    state[kMixGrad + threadIdx.x] = grad;
    float a = state[kMixAlpha + threadIdx.x];
    if (update) {
      const float v = fmaf(mu, state[kMixMom + threadIdx.x], grad);
      a -= *lr_ptr * v;
      state[kMixMom + threadIdx.x] = v;
      state[kMixAlpha + threadIdx.x] = a;
    }
    alpha[threadIdx.x] = a;
  }
  __syncthreads();   // every read of the old p is done; alpha[] is complete
  if (update && (int)threadIdx.x < n) {
    float top = alpha[0];
    for (int q = 1; q < n; ++q) top = fmaxf(top, alpha[q]);
    float sum = 0.f;
    for (int q = 0; q < n; ++q) sum += expf(alpha[q] - top);
    state[kMixP + threadIdx.x] = expf(alpha[threadIdx.x] - top) / sum;
  }
}

// ---------------------------------------------------------------------------
// fused MSE loss + gradient (Sec. II-A, L(delta output)):
//   part[block] = sum (s-t)^2 ;  ds = 2 (s-t) / M ;  loss = sum(part) / M
// ---------------------------------------------------------------------------
template <class T>
__global__ __launch_bounds__(256) void mse_kernel(const T* __restrict__ s, const T* __restrict__ t,
                                                  T* __restrict__ ds, float* __restrict__ part,
                                                  long nvec, float two_over_m) {
  __shared__ float red[256];
  float acc = 0.f;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < nvec; i += (long)gridDim.x * blockDim.x) {
    float a[8], b[8];
    IO<T>::ld(s + i * 8, a);
    IO<T>::ld(t + i * 8, b);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float d = a[e] - b[e];
      acc = fmaf(d, d, acc);
      a[e] = d * two_over_m;
    }
    IO<T>::st(ds + i * 8, a);
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int s2 = 128; s2 > 0; s2 >>= 1) {
    if ((int)threadIdx.x < s2) red[threadIdx.x] += red[threadIdx.x + s2];
    __syncthreads();
  }
  if (threadIdx.x == 0) part[blockIdx.x] = red[0];
}

__global__ __launch_bounds__(256) void mse_final_kernel(const float* __restrict__ part, int n, double inv_m,
                                                        float* loss) {
  __shared__ double red[256];
  double s = 0.0;
  for (int i = threadIdx.x; i < n; i += 256) s += (double)part[i];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int h = 128; h > 0; h >>= 1) {
    if ((int)threadIdx.x < h) red[threadIdx.x] += red[threadIdx.x + h];
    __syncthreads();
  }
  if (threadIdx.x == 0) *loss = (float)(red[0] * inv_m);
}

// ---------------------------------------------------------------------------
// fused SGD-momentum over one block's flat parameter arena (Algorithm 1,
// update_weight; Sec. IV-B):  v <- mu v + g ; w <- w - lr v ; compute copy <- rne(w)
// ---------------------------------------------------------------------------
template <class T>
__global__ void sgd_momentum_kernel(float* __restrict__ w, float* __restrict__ v,
                                    const float* __restrict__ g, T* __restrict__ wc, long n4,
                                    const float* __restrict__ lr_ptr, float mu) {
  const float lr = *lr_ptr;  // device scalar: a captured graph stays valid when the rate changes
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < n4; i += (long)gridDim.x * blockDim.x) {
    float4 wv = reinterpret_cast<float4*>(w)[i], vv = reinterpret_cast<float4*>(v)[i];
    const float4 gv = reinterpret_cast<const float4*>(g)[i];
    vv.x = fmaf(mu, vv.x, gv.x); vv.y = fmaf(mu, vv.y, gv.y);
    vv.z = fmaf(mu, vv.z, gv.z); vv.w = fmaf(mu, vv.w, gv.w);
    wv.x -= lr * vv.x; wv.y -= lr * vv.y; wv.z -= lr * vv.z; wv.w -= lr * vv.w;
    reinterpret_cast<float4*>(v)[i] = vv;
    reinterpret_cast<float4*>(w)[i] = wv;
    if (wc) {
      uint2 pk;
      pk.x = pack_bf2(wv.x, wv.y);
      pk.y = pack_bf2(wv.z, wv.w);
      reinterpret_cast<uint2*>(wc)[i] = pk;
    }
  }
}

__global__ void set_scalar_kernel(float* p, float v) { *p = v; }

// compute copy <- rne(master) without an update (after parameters were loaded)
__global__ void cast_params_kernel(const float* __restrict__ w, bf16_t* __restrict__ wc, long n4) {
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < n4; i += (long)gridDim.x * blockDim.x) {
    const float4 wv = reinterpret_cast<const float4*>(w)[i];
    uint2 pk;
    pk.x = pack_bf2(wv.x, wv.y);
    pk.y = pack_bf2(wv.z, wv.w);
    reinterpret_cast<uint2*>(wc)[i] = pk;
  }
}

// Transposed weight copies for backward-data: src [K][RS][C] -> dst [C][RS][K].
struct TransposeEntry { long src, dst; int K, RS, C; };
template <class T>
__global__ __launch_bounds__(256) void transpose_weights_kernel(const T* __restrict__ wc, T* __restrict__ wt,
                                                                const TransposeEntry* __restrict__ table) {
  // 64 x 64 tiles of one filter tap through LDS: rows of 64 consecutive c are read, rows of 64 consecutive k
  // written, both whole cache lines per wave
  __shared__ T tile[64][65];
  const TransposeEntry e = table[blockIdx.y];
  const int tk = (e.K + 63) / 64, tc = (e.C + 63) / 64;
  const long ntiles = (long)tk * tc * e.RS;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (long t = blockIdx.x; t < ntiles; t += gridDim.x) {
    const int k0 = (int)(t % tk) * 64;
    const long r = t / tk;
    const int c0 = (int)(r % tc) * 64, rs = (int)(r / tc);
    T v[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) {                  // all sixteen loads in flight
      const int k = k0 + ty + 4 * j, c = c0 + tx;
      v[j] = (k < e.K && c < e.C) ? wc[e.src + ((long)k * e.RS + rs) * e.C + c] : T(0);
    }
#pragma unroll
    for (int j = 0; j < 16; ++j) tile[ty + 4 * j][tx] = v[j];
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const int c = c0 + ty + 4 * j, k = k0 + tx;
      if (k < e.K && c < e.C) wt[e.dst + ((long)c * e.RS + rs) * e.K + k] = tile[tx][ty + 4 * j];
    }
    __syncthreads();
  }
}

// out[j] = sum_s part[s*stride + j]   (ordered second stage of split reductions); n % 4 == 0.
// Block = (256/SL) float4 outputs x SL split lanes: lane l adds splits l, l+SL, ... in order (four
// loads in flight), then the SL lane sums are added in order, so the result does not depend on
// scheduling.  SL = 8 for a few partials of a large tensor, 32 for many partials of a small one.
template <int SL>
__global__ __launch_bounds__(256) void sum_partials_kernel(const float* __restrict__ part,
                                                           float* __restrict__ out, long n, int splits,
                                                           long stride) {
  constexpr int NO = 256 / SL;
  __shared__ float4 red[SL][NO];
  const int o = threadIdx.x % NO, l = threadIdx.x / NO;
  const long n4 = n / 4;
  for (long base = (long)blockIdx.x * NO; base < n4; base += (long)gridDim.x * NO) {
    const long i = base + o;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < n4) {
      int k = l;
      for (; k + 3 * SL < splits; k += 4 * SL) {
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = *reinterpret_cast<const float4*>(part + (long)(k + u * SL) * stride + i * 4);
#pragma unroll
        for (int u = 0; u < 4; ++u) { s.x += v[u].x; s.y += v[u].y; s.z += v[u].z; s.w += v[u].w; }
      }
      for (; k < splits; k += SL) {
        const float4 v = *reinterpret_cast<const float4*>(part + (long)k * stride + i * 4);
        s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
      }
    }
    red[l][o] = s;
    __syncthreads();
    if (l == 0 && i < n4) {
      float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
      for (int k = 0; k < SL; ++k) { t.x += red[k][o].x; t.y += red[k][o].y; t.z += red[k][o].z; t.w += red[k][o].w; }
      *reinterpret_cast<float4*>(out + i * 4) = t;
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------
// depthwise convolution, weights [k*k][Cp] (channel-last)
// ---------------------------------------------------------------------------
// Forward: one thread = 8 channels of one output pixel; all k*k taps are requested before the
// first multiply.  KK = k*k.
template <class T, int KK>
__global__ __launch_bounds__(256) void dw_fwd_kernel(const T* __restrict__ x, const T* __restrict__ w,
                                                     T* __restrict__ y, const float* __restrict__ a,
                                                     const float* __restrict__ b, int act, int N, int H, int W,
                                                     int P, int Q, int ncv, int k, int stride, int pad,
                                                     unsigned x_elems) {
  const long nvec = (long)N * P * Q * ncv;
  const __amdgpu_buffer_rsrc_t xr = tensor_rsrc(x, x_elems * (unsigned)sizeof(T));
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < nvec; i += (long)gridDim.x * blockDim.x) {
    const int cv = (int)(i % ncv);
    long pix = i / ncv;
    const int q = (int)(pix % Q); pix /= Q;
    const int p = (int)(pix % P);
    const int n = (int)(pix / P);
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    constexpr int G = KK < 25 ? KK : 25;     // taps in flight at once (bounds the register footprint)
#pragma unroll
    for (int t0 = 0; t0 < KK; t0 += G) {
      typename BufIO<T>::Raw raw[G];
#pragma unroll
      for (int u = 0; u < G; ++u) {
        const int t = t0 + u;
        const int r = t / k, s = t - r * k;    // k is uniform: scalar arithmetic after unrolling
        const int h = p * stride + r - pad, ww = q * stride + s - pad;
        const bool ok = t < KK && (unsigned)h < (unsigned)H && (unsigned)ww < (unsigned)W;
        raw[u] = BufIO<T>::issue(xr, (unsigned)(((n * H + h) * W + ww) * ncv + cv) * 8u, ok);
      }
#pragma unroll
      for (int u = 0; u < G; ++u) {
        if (t0 + u >= KK) continue;
        float v[8], f[8];
        BufIO<T>::unpack(raw[u], v);
        IO<T>::ld(w + ((long)(t0 + u) * ncv + cv) * 8, f);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = fmaf(v[e], f[e], acc[e]);
      }
    }
    if (a) {  // folded inference-mode BN + activation (teacher)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = apply_act(fmaf(acc[e], a[cv * 8 + e], b[cv * 8 + e]), act);
    }
    IO<T>::st(y + i * 8, acc);
  }
}

// Sliding-window forward / stride-1 backward-data: one thread = 8 channels of WS consecutive output
// pixels of one row.  Per filter row it loads the (WS-1)*STRIDE + K input pixels once and uses each
// for up to K outputs, so the loads per output drop from K*K to K*((WS-1)*STRIDE+K)/WS: the vector
// memory pipeline, not HBM, is what a one-pixel-per-thread depthwise kernel saturates.
// FLIP: read the filter mirrored (backward-data of a stride-1 convolution is the same sliding
// sum with taps (K-1-r, K-1-s)); `accumulate` then adds to what dst holds.
template <class T, int K, int STRIDE, int WS, bool FLIP>
__global__ __launch_bounds__(256) void dw_slide_kernel(const T* __restrict__ x, const T* __restrict__ w,
                                                       T* dst, const float* __restrict__ a,
                                                       const float* __restrict__ b, int act, int accumulate,
                                                       int N, int H, int W, int P, int Q, int ncv, int pad,
                                                       unsigned x_elems) {
  constexpr int NIN = (WS - 1) * STRIDE + K;
  const int QS = (Q + WS - 1) / WS;
  const long nitem = (long)N * P * QS * ncv;
  const __amdgpu_buffer_rsrc_t xr = tensor_rsrc(x, x_elems * (unsigned)sizeof(T));
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < nitem; i += (long)gridDim.x * blockDim.x) {
    const int cv = (int)(i % ncv);
    long seg = i / ncv;
    const int qs = (int)(seg % QS); seg /= QS;
    const int p = (int)(seg % P);
    const int n = (int)(seg / P);
    const int q0 = qs * WS, w0 = q0 * STRIDE - pad;
    float ea[8], eb[8];                // folded BN terms, fetched ahead of the taps they follow
    if (a) {
#pragma unroll
      for (int e = 0; e < 8; ++e) { ea[e] = a[cv * 8 + e]; eb[e] = b[cv * 8 + e]; }
    }
    float acc[WS][8];
#pragma unroll
    for (int o = 0; o < WS; ++o)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[o][e] = 0.f;
#pragma unroll(K == 3 ? 3 : 1)
    for (int r = 0; r < K; ++r) {      // 5x5 and 7x7: one filter row at a time bounds the registers
      const int h = p * STRIDE + r - pad;
      const bool row_ok = (unsigned)h < (unsigned)H;
      const unsigned rowoff = (unsigned)((n * H + h) * W + w0) * (unsigned)ncv + (unsigned)cv;
      typename BufIO<T>::Raw raw[NIN];
#pragma unroll
      for (int j = 0; j < NIN; ++j)
        raw[j] = BufIO<T>::issue(xr, (rowoff + (unsigned)(j * ncv)) * 8u, row_ok && (unsigned)(w0 + j) < (unsigned)W);
      float f[K][8];
#pragma unroll
      for (int t = 0; t < K; ++t) {
        const int tap = FLIP ? (K - 1 - r) * K + (K - 1 - t) : r * K + t;
        IO<T>::ld(w + ((long)tap * ncv + cv) * 8, f[t]);
      }
#pragma unroll
      for (int j = 0; j < NIN; ++j) {
        float v[8];
        BufIO<T>::unpack(raw[j], v);
#pragma unroll
        for (int o = 0; o < WS; ++o) {
          const int t = j - o * STRIDE;       // compile-time after unrolling
          if (t < 0 || t >= K) continue;
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[o][e] = fmaf(v[e], f[t][e], acc[o][e]);
        }
      }
    }
#pragma unroll
    for (int o = 0; o < WS; ++o) {
      if (q0 + o >= Q) continue;
      T* out = dst + ((((long)n * P + p) * Q + q0 + o) * ncv + cv) * 8;
      if (a) {  // folded inference-mode BN + activation (teacher)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[o][e] = apply_act(fmaf(acc[o][e], ea[e], eb[e]), act);
      }
      if (accumulate) {
        float old[8];
        IO<T>::ld(out, old);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[o][e] += old[e];
      }
      IO<T>::st(out, acc[o]);
    }
  }
}

// LDS-tiled stride-1 depthwise convolution (bf16): a block stages the (8+K-1) x (16+K-1) input
// pixels x 64 channels behind an 8 x 16 output tile in LDS with ONE round of global loads (all in
// flight together), then every thread slides over 4 outputs reading LDS.  Each input element is
// fetched once per tile instead of ~K*K/2 times, which takes the kernel off the vector-memory
// pipeline and onto HBM.  LDS pixel pitch 160 B: the two 4-pixel segments of a 16-lane group land
// 128 B apart modulo the 256 B bank span.  FLIP / accumulate as in dw_slide_kernel.
constexpr int kDwTileH = 8, kDwTileW = 16, kDwTileCv = 8, kDwTilePitch = kDwTileCv * 16 + 32;

template <int K, bool FLIP>
__global__ __launch_bounds__(256) void dw_tile_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ w,
                                                      bf16_t* dst, const float* __restrict__ a,
                                                      const float* __restrict__ b, int act, int accumulate,
                                                      int N, int H, int W, int ncv, int tiles_h, int tiles_w,
                                                      unsigned x_bytes, int stream) {
  constexpr int TH = kDwTileH, TW = kDwTileW, WS = 4, CVB = kDwTileCv, PIXB = kDwTilePitch;
  constexpr int IH = TH + K - 1, IW = TW + K - 1, NIN = WS + K - 1, pad = K / 2;
  constexpr int TOTAL = IH * IW * CVB, NLOAD = (TOTAL + 255) / 256;
  __shared__ __attribute__((aligned(16))) unsigned char tile[IH * IW * PIXB];
  __shared__ __attribute__((aligned(16))) float wl[K * K * CVB * 8];   // the block's filters, unpacked once
  const int tid = threadIdx.x;
  int t = blockIdx.x;
  const int tw = t % tiles_w; t /= tiles_w;
  const int th_ = t % tiles_h;
  const int n = t / tiles_h;
  const int h0 = th_ * TH, w0 = tw * TW, cv0 = blockIdx.y * CVB;
  const __amdgpu_buffer_rsrc_t xr = tensor_rsrc(x, x_bytes);

  uint4 raw[NLOAD];
#pragma unroll
  for (int i = 0; i < NLOAD; ++i) {
    const int c = tid + i * 256;
    const int pix = c / CVB, cvl = c % CVB;
    const int ih = pix / IW, iw = pix % IW;
    const int h = h0 - pad + ih, ww = w0 - pad + iw;
    const bool ok = c < TOTAL && (unsigned)h < (unsigned)H && (unsigned)ww < (unsigned)W && cv0 + cvl < ncv;
    raw[i] = buffer_load16(xr, ok ? (unsigned)(((n * H + h) * W + ww) * ncv + cv0 + cvl) * 16u : kOutOfRange);
  }
  constexpr int NW = (K * K * CVB + 255) / 256;
#pragma unroll
  for (int i = 0; i < NW; ++i) {
    const int c = tid + i * 256;
    if (c < K * K * CVB) {
      const int tap = c / CVB, wcv = cv0 + c % CVB;
      float f[8];
      if (wcv < ncv) IO<bf16_t>::ld(w + ((long)tap * ncv + wcv) * 8, f);
      else {
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] = 0.f;
      }
      float* dstw = &wl[((FLIP ? K * K - 1 - tap : tap) * CVB + c % CVB) * 8];
      *reinterpret_cast<float4*>(dstw) = make_float4(f[0], f[1], f[2], f[3]);
      *reinterpret_cast<float4*>(dstw + 4) = make_float4(f[4], f[5], f[6], f[7]);
    }
  }
#pragma unroll
  for (int i = 0; i < NLOAD; ++i) {
    const int c = tid + i * 256;
    if (c < TOTAL) *reinterpret_cast<uint4*>(&tile[(c / CVB) * PIXB + (c % CVB) * 16]) = raw[i];
  }
  __syncthreads();

  const int cvl = tid % CVB, seg = (tid / CVB) % (TW / WS), th = tid / (CVB * (TW / WS));
  const int cv = cv0 + cvl;
  if (cv >= ncv) return;
  float ea[8], eb[8];                  // folded BN terms, fetched ahead of the taps they follow
  if (a) {
#pragma unroll
    for (int e = 0; e < 8; ++e) { ea[e] = a[cv * 8 + e]; eb[e] = b[cv * 8 + e]; }
  }
  float acc[WS][8];
#pragma unroll
  for (int o = 0; o < WS; ++o)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[o][e] = 0.f;
#pragma unroll 1
  for (int r = 0; r < K; ++r) {
    const unsigned char* rowp = &tile[((th + r) * IW + seg * WS) * PIXB + cvl * 16];
    uint4 in[NIN];
#pragma unroll
    for (int j = 0; j < NIN; ++j) in[j] = *reinterpret_cast<const uint4*>(rowp + j * PIXB);
    float f[K][8];
#pragma unroll
    for (int tt = 0; tt < K; ++tt) {
      const float* wr = &wl[((r * K + tt) * CVB + cvl) * 8];
      const float4 lo = *reinterpret_cast<const float4*>(wr), hi = *reinterpret_cast<const float4*>(wr + 4);
      f[tt][0] = lo.x; f[tt][1] = lo.y; f[tt][2] = lo.z; f[tt][3] = lo.w;
      f[tt][4] = hi.x; f[tt][5] = hi.y; f[tt][6] = hi.z; f[tt][7] = hi.w;
    }
#pragma unroll
    for (int j = 0; j < NIN; ++j) {
      float v[8];
      BufIO<bf16_t>::unpack(in[j], v);
#pragma unroll
      for (int o = 0; o < WS; ++o) {
        const int tt = j - o;
        if (tt < 0 || tt >= K) continue;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[o][e] = fmaf(v[e], f[tt][e], acc[o][e]);
      }
    }
  }
  const int h = h0 + th;
  if (h >= H) return;
#pragma unroll
  for (int o = 0; o < WS; ++o) {
    const int ww = w0 + seg * WS + o;
    if (ww >= W) continue;
    bf16_t* out = dst + ((((long)n * H + h) * W + ww) * ncv + cv) * 8;
    if (a) {
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[o][e] = apply_act(fmaf(acc[o][e], ea[e], eb[e]), act);
    }
    if (accumulate) {
      float old[8];
      IO<bf16_t>::ld(out, old);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[o][e] += old[e];
    }
    if (stream) IO<bf16_t>::st_t<true>(out, acc[o]);   // (outputs far larger than the caches)
    else IO<bf16_t>::st(out, acc[o]);
  }
}

// Backward-data in gather form: dx[h,w] (+)= sum_taps dy[(h+pad-r)/st, (w+pad-s)/st] * w[r][s]
template <class T, int KK>
__global__ __launch_bounds__(256) void dw_dgrad_kernel(const T* __restrict__ dy, const T* __restrict__ w,
                                                       T* __restrict__ dx, int N, int H, int W, int P, int Q,
                                                       int ncv, int k, int stride, int pad, int accumulate,
                                                       unsigned dy_elems) {
  const long nvec = (long)N * H * W * ncv;
  const __amdgpu_buffer_rsrc_t dr = tensor_rsrc(dy, dy_elems * (unsigned)sizeof(T));
  const int sh = stride == 2 ? 1 : 0, smask = stride - 1;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < nvec; i += (long)gridDim.x * blockDim.x) {
    const int cv = (int)(i % ncv);
    long pix = i / ncv;
    const int ww = (int)(pix % W); pix /= W;
    const int h = (int)(pix % H);
    const int n = (int)(pix / H);
    float acc[8];
    if (accumulate) IO<T>::ld(dx + i * 8, acc);
    else {
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    }
    constexpr int G = KK < 25 ? KK : 25;
#pragma unroll
    for (int t0 = 0; t0 < KK; t0 += G) {
      typename BufIO<T>::Raw raw[G];
#pragma unroll
      for (int u = 0; u < G; ++u) {
        const int t = t0 + u;
        const int r = t / k, s = t - r * k;
        const int ph = h + pad - r, qw = ww + pad - s;
        const int p = ph >> sh, q = qw >> sh;
        const bool ok = t < KK && ((ph | qw) & smask) == 0 && (unsigned)p < (unsigned)P && (unsigned)q < (unsigned)Q;
        raw[u] = BufIO<T>::issue(dr, (unsigned)(((n * P + p) * Q + q) * ncv + cv) * 8u, ok);
      }
#pragma unroll
      for (int u = 0; u < G; ++u) {
        if (t0 + u >= KK) continue;
        float d[8], f[8];
        BufIO<T>::unpack(raw[u], d);
        IO<T>::ld(w + ((long)(t0 + u) * ncv + cv) * 8, f);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = fmaf(d[e], f[e], acc[e]);
      }
    }
    IO<T>::st(dx + i * 8, acc);
  }
}

// Backward-data of a stride-2 depthwise convolution: an input pixel only meets the taps whose
// parity matches its own, (K+1)/2 per dimension, so only those are visited (K*K/4 instead of K*K
// masked loads).
template <class T, int K>
__global__ __launch_bounds__(256) void dw_dgrad_s2_kernel(const T* __restrict__ dy, const T* __restrict__ w,
                                                          T* __restrict__ dx, int N, int H, int W, int P, int Q,
                                                          int ncv, int pad, int accumulate, unsigned dy_elems) {
  constexpr int HK = (K + 1) / 2;
  const long nvec = (long)N * H * W * ncv;
  const __amdgpu_buffer_rsrc_t dr = tensor_rsrc(dy, dy_elems * (unsigned)sizeof(T));
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < nvec; i += (long)gridDim.x * blockDim.x) {
    const int cv = (int)(i % ncv);
    long pix = i / ncv;
    const int ww = (int)(pix % W); pix /= W;
    const int h = (int)(pix % H);
    const int n = (int)(pix / H);
    const int ph = h + pad, qw = ww + pad, r0 = ph & 1, s0 = qw & 1;
    float acc[8];
    if (accumulate) IO<T>::ld(dx + i * 8, acc);
    else {
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    }
    typename BufIO<T>::Raw raw[HK * HK];
#pragma unroll
    for (int a = 0; a < HK; ++a)
#pragma unroll
      for (int b = 0; b < HK; ++b) {
        const int r = r0 + 2 * a, s = s0 + 2 * b;
        const int p = (ph - r) >> 1, q = (qw - s) >> 1;
        const bool ok = r < K && s < K && (unsigned)p < (unsigned)P && (unsigned)q < (unsigned)Q;
        raw[a * HK + b] = BufIO<T>::issue(dr, (unsigned)(((n * P + p) * Q + q) * ncv + cv) * 8u, ok);
      }
#pragma unroll
    for (int a = 0; a < HK; ++a)
#pragma unroll
      for (int b = 0; b < HK; ++b) {
        const int r = min(r0 + 2 * a, K - 1), s = min(s0 + 2 * b, K - 1);   // clamped taps carry zeros
        float d[8], f[8];
        BufIO<T>::unpack(raw[a * HK + b], d);
        IO<T>::ld(w + ((long)(r * K + s) * ncv + cv) * 8, f);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = fmaf(d[e], f[e], acc[e]);
      }
    IO<T>::st(dx + i * 8, acc);
  }
}

// dW[r][t][c] = sum over output pixels dY * X(shifted).  ROWS tap rows per block: 3x3 filters keep all
// 9 x 8 accumulators in registers and read dY / X once; larger filters take one tap row per
// blockIdx.z (grid = (slabs, chunks, k / ROWS)).  All taps of a pixel are requested before use.
template <class T, int KMAX, int ROWS>
__global__ __launch_bounds__(256) void dw_wgrad_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                       float* __restrict__ part, int N, int H, int W,
                                                       int P, int Q, int Cp, int k, int stride, int pad,
                                                       ColGrid g, unsigned x_elems) {
  extern __shared__ float smem[];
  const int ncv = Cp / 8;
  const int cv_lane = threadIdx.x % g.cvl, row_lane = threadIdx.x / g.cvl, rl = 256 / g.cvl;
  const int cv = blockIdx.x * g.cvl + cv_lane;
  const int rbase = blockIdx.z * ROWS;
  const long M = (long)N * P * Q;
  const long r0 = blockIdx.y * g.rows_per_chunk;
  const long r1 = min(M, r0 + g.rows_per_chunk);
  const __amdgpu_buffer_rsrc_t xr = tensor_rsrc(x, x_elems * (unsigned)sizeof(T));
  float acc[ROWS][KMAX * 8];
#pragma unroll
  for (int a = 0; a < ROWS; ++a)
#pragma unroll
    for (int t = 0; t < KMAX * 8; ++t) acc[a][t] = 0.f;
  if (cv < ncv && row_lane < rl && r0 + row_lane < r1) {
    // (n, p, q) of this thread's first row, then advanced by rl rows per step without divisions
    long pix = r0 + row_lane;
    int q = (int)(pix % Q); pix /= Q;
    int p = (int)(pix % P);
    int n = (int)(pix / P);
    const int dq = rl % Q, dp = (rl / Q) % P, dn = rl / (Q * P);
    for (long m = r0 + row_lane; m < r1; m += rl) {
      typename BufIO<T>::Raw raw[ROWS][KMAX];
#pragma unroll
      for (int a = 0; a < ROWS; ++a)
#pragma unroll
        for (int t = 0; t < KMAX; ++t) {
          const int h = p * stride + rbase + a - pad, ww = q * stride + t - pad;
          const bool ok = rbase + a < k && t < k && (unsigned)h < (unsigned)H && (unsigned)ww < (unsigned)W;
          raw[a][t] = BufIO<T>::issue(xr, (unsigned)(((n * H + h) * W + ww) * ncv + cv) * 8u, ok);
        }
      float d[8];
      IO<T>::ld(dy + (m * ncv + cv) * 8, d);
#pragma unroll
      for (int a = 0; a < ROWS; ++a)
#pragma unroll
        for (int t = 0; t < KMAX; ++t) {
          float v[8];
          BufIO<T>::unpack(raw[a][t], v);
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[a][t * 8 + e] = fmaf(d[e], v[e], acc[a][t * 8 + e]);
        }
      q += dq;
      if (q >= Q) { q -= Q; ++p; }
      p += dp;
      if (p >= P) { p -= P; ++n; }
      n += dn;
    }
  }
  // tree reduction over the row lanes, one tap row (KMAX x 8 values) at a time
#pragma unroll
  for (int a = 0; a < ROWS; ++a) {
    if (rbase + a >= k) continue;   // uniform over the block
    float out[KMAX * 8];
    bool owner;
    block_col_reduce<KMAX * 8>(acc[a], smem, g.cvl, cv_lane, row_lane, out, owner);
    if (owner && cv < ncv) {
#pragma unroll
      for (int t = 0; t < KMAX; ++t) {
        if (t >= k) continue;
        float* pp = part + ((long)blockIdx.y * k * k + (rbase + a) * k + t) * Cp + cv * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) pp[e] = out[t * 8 + e];
      }
    }
  }
}


// LDS-tiled depthwise backward-weight (bf16, stride 1).  Wavefront r of the block owns filter row r:
// it walks the 256 (output row, 4-pixel segment, channel vector) items of each 8 x 16 tile and
// accumulates dW[r][t][c] += dy[o] * x[o + t] for the K taps of its row, x and dy read from LDS
// tiles staged as in dw_tile_kernel.  A block runs over `tiles_per_block` tiles, so x and dy are
// fetched once (not once per filter row) and the K x 8 accumulators are reduced over the lanes
// that share a channel vector only once, at the end (xor tree: a fixed association).
template <int K>
__global__ __launch_bounds__(64 * K) void dw_wgrad_tile_kernel(const bf16_t* __restrict__ dy,
                                                               const bf16_t* __restrict__ x,
                                                               float* __restrict__ part, int N, int H, int W,
                                                               int ncv, int tiles_h, int tiles_w, int ntiles,
                                                               int tiles_per_block, unsigned bytes) {
  constexpr int TH = kDwTileH, TW = kDwTileW, WS = 4, CVB = kDwTileCv, PIXB = kDwTilePitch, NT = 64 * K;
  constexpr int IH = TH + K - 1, IW = TW + K - 1, NIN = WS + K - 1, pad = K / 2;
  constexpr int TOTX = IH * IW * CVB, NLX = (TOTX + NT - 1) / NT;
  constexpr int TOTD = TH * TW * CVB, NLD = (TOTD + NT - 1) / NT;
  __shared__ __attribute__((aligned(16))) unsigned char xt[IH * IW * PIXB];
  __shared__ __attribute__((aligned(16))) unsigned char dt[TH * TW * PIXB];
  const int tid = threadIdx.x, lane = tid & 63, r = tid >> 6;
  const int cv0 = blockIdx.y * CVB;
  const __amdgpu_buffer_rsrc_t xr = tensor_rsrc(x, bytes), dr = tensor_rsrc(dy, bytes);
  float acc[K][8];
#pragma unroll
  for (int t = 0; t < K; ++t)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[t][e] = 0.f;

  const int tile_end = min(ntiles, ((int)blockIdx.x + 1) * tiles_per_block);
  for (int tile = blockIdx.x * tiles_per_block; tile < tile_end; ++tile) {
    int t_ = tile;
    const int tw = t_ % tiles_w; t_ /= tiles_w;
    const int th_ = t_ % tiles_h;
    const int n = t_ / tiles_h;
    const int h0 = th_ * TH, w0 = tw * TW;
    uint4 rx[NLX], rd[NLD];
#pragma unroll
    for (int i = 0; i < NLX; ++i) {
      const int c = tid + i * NT;
      const int pix = c / CVB, cvl = c % CVB;
      const int h = h0 - pad + pix / IW, ww = w0 - pad + pix % IW;
      const bool ok = c < TOTX && (unsigned)h < (unsigned)H && (unsigned)ww < (unsigned)W && cv0 + cvl < ncv;
      rx[i] = buffer_load16(xr, ok ? (unsigned)(((n * H + h) * W + ww) * ncv + cv0 + cvl) * 16u : kOutOfRange);
    }
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int c = tid + i * NT;
      const int pix = c / CVB, cvl = c % CVB;
      const int h = h0 + pix / TW, ww = w0 + pix % TW;
      const bool ok = c < TOTD && h < H && ww < W && cv0 + cvl < ncv;
      rd[i] = buffer_load16(dr, ok ? (unsigned)(((n * H + h) * W + ww) * ncv + cv0 + cvl) * 16u : kOutOfRange);
    }
    __syncthreads();                                 // the previous tile has been consumed
#pragma unroll
    for (int i = 0; i < NLX; ++i) {
      const int c = tid + i * NT;
      if (c < TOTX) *reinterpret_cast<uint4*>(&xt[(c / CVB) * PIXB + (c % CVB) * 16]) = rx[i];
    }
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int c = tid + i * NT;
      if (c < TOTD) *reinterpret_cast<uint4*>(&dt[(c / CVB) * PIXB + (c % CVB) * 16]) = rd[i];
    }
    __syncthreads();
#pragma unroll 1
    for (int it = 0; it < TOTD / (64 * WS); ++it) {
      const int item = lane + 64 * it;
      const int cvl = item % CVB, seg = (item / CVB) % (TW / WS), th = item / (CVB * (TW / WS));
      const unsigned char* dp = &dt[(th * TW + seg * WS) * PIXB + cvl * 16];
      const unsigned char* xp = &xt[((th + r) * IW + seg * WS) * PIXB + cvl * 16];
      uint4 din[WS], xin[NIN];
#pragma unroll
      for (int o = 0; o < WS; ++o) din[o] = *reinterpret_cast<const uint4*>(dp + o * PIXB);
#pragma unroll
      for (int j = 0; j < NIN; ++j) xin[j] = *reinterpret_cast<const uint4*>(xp + j * PIXB);
      float d[WS][8];
#pragma unroll
      for (int o = 0; o < WS; ++o) BufIO<bf16_t>::unpack(din[o], d[o]);
#pragma unroll
      for (int j = 0; j < NIN; ++j) {
        float v[8];
        BufIO<bf16_t>::unpack(xin[j], v);
#pragma unroll
        for (int o = 0; o < WS; ++o) {
          const int t = j - o;
          if (t < 0 || t >= K) continue;
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[t][e] = fmaf(d[o][e], v[e], acc[t][e]);
        }
      }
    }
  }
  // lanes with equal lane % 8 hold the same channel vector
#pragma unroll
  for (int t = 0; t < K; ++t)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
#pragma unroll
      for (int m = 8; m < 64; m <<= 1) acc[t][e] += __shfl_xor(acc[t][e], m, 64);
    }
  if (lane < CVB && cv0 + lane < ncv) {
#pragma unroll
    for (int t = 0; t < K; ++t) {
      float* pp = part + ((long)blockIdx.x * K * K + r * K + t) * (ncv * 8) + (cv0 + lane) * 8;
#pragma unroll
      for (int e = 0; e < 8; ++e) pp[e] = acc[t][e];
    }
  }
}

}  // namespace pbd
