// Implicit-GEMM convolution (forward and backward-data) for the large layers: 256-row tiles, eight
// wavefronts, operands moved from global memory straight into LDS.
//
// Same mathematics and argument block as igemm_kernel (conv_kernels.h):
//   Out[m][j] = sum_kk Agather(m, kk) * Bw[j][kk],  m = (n, a, b),  kk = (r*S + s)*CA + c
// What differs is how the tile loop is fed:
//  * Tile 256 x BN x BK, 512 threads, BN one of 256 / 192 / 128 / 96 / 64 (the channel counts of the
//    workloads are 64 2^k and 96 2^k), BK 64 or 32.  The eight wavefronts form a WAVES_M x WAVES_N grid and each owns
//    TM x TN blocks of 32 x 32 (128 x 64 for BN 256 down to 32 x 64 for BN 64), so every fragment read from LDS feeds
//    up to four v_mfma_f32_32x32x16_bf16: half the L2 -> LDS and LDS -> register bytes per multiply-add of a
//    128 x 128 tile.
//  * Global -> LDS without a register round trip: buffer_load_dwordx4 ... lds writes the 64 lanes' 16-byte
//    chunks to 1 KiB of consecutive LDS (lane l at +16 l).  Rows are therefore unpadded (BK * 2 bytes); bank
//    conflicts of the fragment reads are avoided by a swizzle instead: lane l of a load fetches the global
//    chunk (l % CPR) ^ swz(row) of its row, so chunk kc of row r sits in slot kc ^ swz(r), with
//    swz(r) = (r >> 1) & 7 for 128-byte rows and (r >> 2) & 3 for 64-byte rows: the 16 lanes that one
//    ds_read_b128 cycle serves (16 consecutive rows, one chunk index) then hit 16 different 16-byte bank groups.
//    An out-of-range lane (padding, ragged tile) gets the descriptor's zeros written.
//  * A ring of NS stages with ONE barrier per reduction step: at step kt a wave waits for its own loads of
//    stage kt (s_waitcnt vmcnt), passes the barrier (now every wave's part of stage kt is in LDS, and every
//    wave has finished reading stage kt-1), issues the loads of stage kt+NS-1 into the buffer of stage kt-1,
//    and multiplies stage kt.
//  * Fragment reads are ds_read_b128 in inline assembly with their own s_waitcnt lgkmcnt: the compiler
//    would otherwise order every LDS read behind ALL outstanding direct-to-LDS loads (it cannot tell the
//    stages apart) and the prefetch would be lost.  Fragments of sub-step ks+1 are requested before the
//    MFMAs of sub-step ks.
//  * Tail tiles.  One workgroup per compute unit is resident (the ring takes most of the LDS), so a launch whose
//    tile count is a little over a multiple of the number of compute units would end with a nearly empty round as
//    long as a full one.  The host may therefore cut the last row tiles into 64-row tiles (blockIdx >= the number
//    of big tiles): same code with BM = 64, a quarter of the time each, spread over four times as many units.
//  * Backward-data of a stride-2 layer takes the input pixels parity class by parity class (see dma_tile): only the
//    taps that reach a class are reduced over.
//  * Forward only: a tap may span a run of neighbouring pixels (IgemmArgs::pix_shift), which is how the 7 x 7 stem is
//    run on the space-to-depth copy of its 3-channel input: a filter row of four 16-channel pixels is one
//    64-element tap, and each 16-byte chunk is range-tested against the pixel it belongs to.
// Needs CA % BK == 0 (a reduction step lies inside one filter tap: taps are uniform over the block).
#pragma once
#include "conv_kernels.h"


namespace pbd {

typedef __attribute__((address_space(3))) void* lds_void_ptr;

__device__ __forceinline__ void dma_load16(__amdgpu_buffer_rsrc_t r, unsigned char* lds_wave_base, unsigned byte_off) {
  // lane l's 16 bytes land at lds_wave_base + 16 l (the base must be uniform over the wavefront)
  __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_void_ptr)lds_wave_base, 16, (int)byte_off, 0, 0, 0);
}

// Wait until at most N of this wave's vector-memory operations are outstanding.  The "memory" clobbers keep
// the compiler from moving the direct-to-LDS loads (memory operations to it) across the wait or the barrier.
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ void block_barrier() { asm volatile("s_barrier" ::: "memory"); }
template <int N> __device__ __forceinline__ void wait_lgkmcnt() {
  static_assert(N >= 0 && N < 16, "lgkmcnt is a 4-bit counter");
  asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ bf16x8 lds_read16_async(unsigned addr) {
  // the result arrives later: only use it behind wait_lgkmcnt + pin()
  bf16x8 v;
  asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr) : "memory");
  return v;
}
__device__ __forceinline__ void pin(bf16x8& v) { asm volatile("" : "+v"(v)); }

// wait until at most n (0..16) vector-memory operations of this wave are outstanding; n is uniform
__device__ __forceinline__ void wait_vmcnt_dyn(int n) {
  switch (n) {
    case 0: wait_vmcnt<0>(); break;
    case 1: wait_vmcnt<1>(); break;
    case 2: wait_vmcnt<2>(); break;
    case 3: wait_vmcnt<3>(); break;
    case 4: wait_vmcnt<4>(); break;
    case 5: wait_vmcnt<5>(); break;
    case 6: wait_vmcnt<6>(); break;
    case 7: wait_vmcnt<7>(); break;
    case 8: wait_vmcnt<8>(); break;
    case 9: wait_vmcnt<9>(); break;
    case 10: wait_vmcnt<10>(); break;
    case 11: wait_vmcnt<11>(); break;
    case 12: wait_vmcnt<12>(); break;
    case 13: wait_vmcnt<13>(); break;
    case 14: wait_vmcnt<14>(); break;
    case 15: wait_vmcnt<15>(); break;
    default: wait_vmcnt<16>(); break;
  }
}

constexpr int kDmaThreads = 512;
constexpr int kDmaBM = 256;      // rows of a big tile
constexpr int kDmaTailBM = 64;   // rows of a tail tile
// waves along the rows of a big tile
constexpr int dma_waves_m(int BN) { return BN == 256 ? 2 : (BN == 192 || BN == 128) ? 4 : 8; }
// ring depth: what 160 KB of LDS hold
constexpr int dma_stages(int BN, int BK) { return BK == 64 && BN >= 192 ? 2 : 3; }
constexpr int dma_lds_bytes(int BN, int BK, bool accum) {
  const int ring = dma_stages(BN, BK) * (kDmaBM + BN) * BK * 2;
  const int out = 128 * (BN * (accum ? 4 : 2) + 16);   // 128 staged output rows
  const int red = kDmaThreads * 16 * 4;                 // batch-norm sums on their way to the column threads
  return ring > out ? (ring > red ? ring : red) : (out > red ? out : red);
}

// One tile of BM rows starting at row m0, columns n0 .. n0 + BN.  stat_row: which row of g.stats it fills.
// cls >= 0 (backward-data, stride 2): the rows are the input pixels (2a + cls / 2, 2b + cls % 2) in (n, a, b) order
// and the reduction runs over the taps whose parity reaches them: a quarter of the pixels with 1, 2, 2 and 4 of
// the 9 taps of a 3 x 3 kernel instead of all pixels with 9 taps of which three quarters load zeros.
template <int MODE, int BM, int BN, int BK, int WAVES_M, int EPI>
__device__ __forceinline__ void dma_tile(unsigned char* smem, float* ep_s, const bf16_t* __restrict__ A,
                                         const bf16_t* __restrict__ Bw, bf16_t* __restrict__ Out,
                                         const float* __restrict__ ep_a, const float* __restrict__ ep_b, int act,
                                         const IgemmArgs& g, int m0, int n0, int stat_row, int cls = -1) {
  // waves that multiply: WAVES_M x WAVES_N of the 8 (a 64-row tail tile of few columns leaves some idle; they still load)
  constexpr int TM = BM / (WAVES_M * 32);
  constexpr int WAVES_N_MAX = 8 / WAVES_M;
  constexpr int TN = BN / 32 >= WAVES_N_MAX ? BN / (WAVES_N_MAX * 32) : 1;
  constexpr int WAVES_N = BN / (TN * 32);
  static_assert(TM >= 1 && TM * WAVES_M * 32 == BM && TN * WAVES_N * 32 == BN && WAVES_N <= WAVES_N_MAX, "wave grid");
  constexpr int CPR = BK / 8;                    // 16-byte chunks per tile row
  constexpr int ROWB = BK * 2;                   // bytes per tile row in LDS (no padding)
  constexpr int NS = dma_stages(BN, BK);
  constexpr int A_BYTES = kDmaBM * ROWB, STAGE = (kDmaBM + BN) * ROWB;   // (a tail tile uses the top of the A region)
  constexpr int A_CHUNKS = BM * CPR, B_CHUNKS = BN * CPR;
  constexpr int A_INSTR = (A_CHUNKS + kDmaThreads - 1) / kDmaThreads, B_INSTR = (B_CHUNKS + kDmaThreads - 1) / kDmaThreads;
  constexpr int KS = BK / 16;                    // MFMA sub-steps per stage
  constexpr int RPI = 64 / CPR;                  // rows one wave instruction covers

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // uniform, and known to the compiler as such
  const int wm = wave / WAVES_N_MAX, wn = wave % WAVES_N_MAX;
  const bool active = wn < WAVES_N;
  const int sh = g.stride == 2 ? 1 : 0, smask = g.stride - 1;
  const bool par = MODE == 1 && cls >= 0;
  const int ph = par ? cls >> 1 : 0, pw = par ? cls & 1 : 0;
  const int HOr = par ? g.HO >> 1 : g.HO, WOr = par ? g.WO >> 1 : g.WO;      // the row grid
  const int Mrows = par ? g.N * HOr * WOr : g.M;
  // first tap and tap step in each direction, reduction steps
  const int r0 = par ? (ph + g.pad) & 1 : 0, s0 = par ? (pw + g.pad) & 1 : 0, tstep = par ? 2 : 1;
  const int nk = par ? ((g.R - r0 + 1) >> 1) * ((g.S - s0 + 1) >> 1) * (g.CA / BK) : g.Kred / BK;

  if (EPI == EPI_AFFINE_ACT && tid < BN / 4) {
    const int col = min(n0 + tid * 4, g.NC - 4);
    *reinterpret_cast<float4*>(ep_s + tid * 4) = *reinterpret_cast<const float4*>(ep_a + col);
    *reinterpret_cast<float4*>(ep_s + BN + tid * 4) = *reinterpret_cast<const float4*>(ep_b + col);
  }

  // ---- what this thread loads: chunk (i*8 + wave)*64 + lane of the A tile and of the B tile, where it exists ----
  // slot = lane % CPR is where the chunk lands in its row; the global chunk it fetches is slot ^ swz(row)
  const int lrow = lane / CPR, slot = lane % CPR;
  auto swz = [](int row) { return BK == 64 ? (row >> 1) & 7 : (row >> 2) & 3; };
  unsigned abase[A_INSTR];
  int rh[A_INSTR], rw[A_INSTR], kc8[A_INSTR];
  // elements between neighbouring pixels of A: the channel count, except for a tap that spans several pixels
  // (g.pix_shift > 0: CA = a run of CA >> pix_shift-wide pixels, each range-tested on its own)
  const int pitch = MODE == 0 && g.pix_shift ? g.CA >> g.pix_shift : g.CA;
  const int pshift = MODE == 0 && g.pix_shift ? 31 - __builtin_clz(pitch) : 31;     // (x >> 31 = 0: one pixel per tap)
  int a_cnt = 0, b_cnt = 0;                      // loads this WAVE issues per stage (uniform)
#pragma unroll
  for (int i = 0; i < A_INSTR; ++i) {
    if ((i * 8 + wave) * 64 < A_CHUNKS) ++a_cnt;
    const int row = (i * 8 + wave) * RPI + lrow;
    const int m = m0 + row;
    const bool valid = row < BM && m < Mrows;
    const int mm = valid ? m : 0;
    const int b_ = mm % WOr;
    const int t = mm / WOr;
    const int a_ = t % HOr;
    const int nbase = (t / HOr) * g.HA * g.WA;
    const int h0 = MODE == 0 ? a_ * g.stride - g.pad : (par ? 2 * a_ + ph : a_) + g.pad;
    const int w0 = MODE == 0 ? b_ * g.stride - g.pad : (par ? 2 * b_ + pw : b_) + g.pad;
    const int kc = slot ^ swz(row);
    kc8[i] = kc * 8;
    if (MODE == 0) abase[i] = (unsigned)(((nbase + h0 * g.WA + w0) * pitch + kc * 8) * 2);
    else abase[i] = (unsigned)((nbase * g.CA + ((h0 * g.WA + w0) * g.CA >> sh) + kc * 8) * 2);
    rh[i] = valid ? h0 : -(1 << 24);             // rows past the end fail every range test
    rw[i] = w0;
  }
  unsigned bbase[B_INSTR];
#pragma unroll
  for (int i = 0; i < B_INSTR; ++i) {
    if ((i * 8 + wave) * 64 < B_CHUNKS) ++b_cnt;
    const int row = (i * 8 + wave) * RPI + lrow;
    const int kc = slot ^ swz(row);
    bbase[i] = row < BN && n0 + row < g.NC ? (unsigned)((n0 + row) * g.Kred + kc * 8) * 2u : kOutOfRange;
  }
  const int lps = a_cnt + b_cnt;
  constexpr int LPS_MAX = A_INSTR + B_INSTR;
  const __amdgpu_buffer_rsrc_t a_rsrc = tensor_rsrc(A, g.a_bytes), b_rsrc = tensor_rsrc(Bw, g.b_bytes);

  // reduction position of the next stage to be loaded: kk = (r*S + s)*CA + c, uniform over the block
  int r = r0, s = s0, c = 0;
  auto issue_stage = [&](int stage) {
    unsigned char* sa = smem + stage * STAGE + wave * 1024;
    const int tap = MODE == 0 ? r * g.WA + s : -(r * g.WA + s);
    const unsigned delta = (unsigned)(((tap * (MODE == 0 ? pitch : g.CA)) >> (MODE == 1 ? sh : 0)) + c) * 2u;
    const unsigned hlim = MODE == 0 ? (unsigned)g.HA : (unsigned)g.HA << sh;
    const unsigned wlim = MODE == 0 ? (unsigned)g.WA : (unsigned)g.WA << sh;
    const unsigned kk = (unsigned)((r * g.S + s) * g.CA + c);
#pragma unroll
    for (int i = 0; i < A_INSTR; ++i) {
      if ((i * 8 + wave) * 64 >= A_CHUNKS) continue;        // (uniform over the wave)
      const int h = MODE == 0 ? rh[i] + r : rh[i] - r, w = MODE == 0 ? rw[i] + s : rw[i] - s;
      bool ok = (unsigned)h < hlim && (unsigned)(w + ((c + kc8[i]) >> pshift)) < wlim;
      if (MODE == 1) ok = ok && ((h | w) & smask) == 0;
      dma_load16(a_rsrc, sa + i * 8 * 1024, ok ? abase[i] + delta : kOutOfRange);
    }
#pragma unroll
    for (int i = 0; i < B_INSTR; ++i) {
      if ((i * 8 + wave) * 64 >= B_CHUNKS) continue;
      dma_load16(b_rsrc, sa + A_BYTES + i * 8 * 1024, bbase[i] == kOutOfRange ? kOutOfRange : bbase[i] + kk * 2u);
    }
    c += BK;
    const bool wrap = c >= g.CA;
    c = wrap ? 0 : c;
    s += wrap ? tstep : 0;
    const bool wrap2 = s >= g.S;
    s = wrap2 ? s0 : s;
    r += wrap2 ? tstep : 0;
  };
  // wait until this wave's loads of stage kt have landed: up to NS - 2 younger stages may stay in flight
  auto wait_stage = [&](int younger) { wait_vmcnt_dyn(min(NS - 2, younger) * lps); };

  // ---- fragment addresses: row = lane % 32 (+ 32 i), chunk = 2 ks + lane / 32, slot = chunk ^ swz(row) ----
  const int frow = lane & 31, fhi = lane >> 5;
  unsigned fa[KS], fb[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    const unsigned so = (unsigned)(((ks * 2 + fhi) ^ swz(frow)) * 16);   // (blocks start at multiples of 32 rows: same swizzle)
    fa[ks] = (unsigned)((wm * TM * 32 + frow) * ROWB) + so;
    fb[ks] = (unsigned)(A_BYTES + (wn * TN * 32 + frow) * ROWB) + so;
  }

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  struct Frag { bf16x8 a[TM], b[TN]; };
  auto read_frag = [&](Frag& f, unsigned addr_a, unsigned addr_b) {
#pragma unroll
    for (int i = 0; i < TM; ++i) f.a[i] = lds_read16_async(addr_a + i * 32 * ROWB);
#pragma unroll
    for (int j = 0; j < TN; ++j) f.b[j] = lds_read16_async(addr_b + j * 32 * ROWB);
  };
  auto pin_frag = [&](Frag& f) {
#pragma unroll
    for (int i = 0; i < TM; ++i) pin(f.a[i]);
#pragma unroll
    for (int j = 0; j < TN; ++j) pin(f.b[j]);
  };

  // ---- the ring ----
#pragma unroll
  for (int st = 0; st < NS - 1; ++st)
    if (st < nk) issue_stage(st);
  int stage = 0, next = NS - 1;                 // buffer of step kt, buffer the next loads go to
  for (int kt = 0; kt < nk; ++kt) {
    wait_stage(nk - 1 - kt);
    block_barrier();
    // every wave is past step kt-1: its buffer takes the loads of step kt+NS-1
    if (kt + NS - 1 < nk) issue_stage(next);
    if (active) {
      const unsigned sbase = (unsigned)(stage * STAGE);
      Frag f[2];
      read_frag(f[0], fa[0] + sbase, fb[0] + sbase);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        if (ks + 1 < KS) read_frag(f[(ks + 1) & 1], fa[ks + 1] + sbase, fb[ks + 1] + sbase);
        Frag& cur = f[ks & 1];
        // LDS reads return in order: the older group is complete once at most the newer group's reads are pending
        if (ks + 1 < KS) wait_lgkmcnt<TM + TN>(); else wait_lgkmcnt<0>();
        pin_frag(cur);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur.b[j], cur.a[i], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);      // keep the next group's reads behind these MFMAs' issue, not ahead of the wait
      }
    }
    stage = stage + 1 == NS ? 0 : stage + 1;
    next = next + 1 == NS ? 0 : next + 1;
  }
  wait_vmcnt<0>();
  __syncthreads();                              // the ring is dead: LDS now stages the output tile

  // ---- epilogue: up to 128 staged rows at a time, then coalesced 16-byte stores ----------------------
  // lane holds pixel (lane % 32) and channels 8 (v / 4) + 4 (lane / 32) + v % 4 of each 32 x 32 block
  const bool full = m0 + BM <= Mrows && n0 + BN <= g.NC;
  // where row m of the tile's row grid lies in the output tensor
  auto out_row = [&](int m) -> size_t {
    if (!par) return (size_t)m;
    const int b_ = m % WOr, t = m / WOr;
    return (size_t)((t / HOr) * g.HO + 2 * (t % HOr) + ph) * g.WO + 2 * b_ + pw;
  };
  constexpr int ESZ = EPI == EPI_ACCUM ? 4 : 2;
  constexpr int OP = BN * ESZ + 16;              // bytes per staged row
  constexpr int CPROW = BN / 8;                  // 8-channel chunks per row
  constexpr int ST = (CPROW & (CPROW - 1)) == 0 ? kDmaThreads : 384;   // storing threads: a multiple of CPROW (12 and 24 divide 384)
  constexpr int PR = BM < 128 ? BM : 128;        // rows per pass
  constexpr int NCHUNK = PR * CPROW;
  constexpr int CPT = NCHUNK / ST;               // chunks per storing thread and pass
  static_assert(ST % CPROW == 0 && NCHUNK % ST == 0, "a storing thread keeps its chunk column over the rows it stores");
  float s1[8], s2[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) s1[e] = s2[e] = 0.f;
#pragma unroll
  for (int pass = 0; pass < BM / PR; ++pass) {
    const int rbase = pass * PR;
    // values the stores of this pass combine with (a fused residual, or what an accumulating launch adds to)
    uint4 extra[CPT];
    const bf16_t* esrc = EPI == EPI_ACCUM ? Out : static_cast<const bf16_t*>(g.res);
    if (esrc && tid < ST) {
#pragma unroll
      for (int k = 0; k < CPT; ++k) {
        const int cidx = tid + k * ST;
        const int row = m0 + rbase + cidx / CPROW, col = n0 + (cidx % CPROW) * 8;
        const bool in = full || (row < Mrows && col < g.NC);
        if (g.stream_out) {                      // (read once, like the output is written once: not kept in the caches)
          typedef unsigned int u32x4_nt __attribute__((ext_vector_type(4)));
          u32x4_nt q = {0u, 0u, 0u, 0u};
          if (in) q = __builtin_nontemporal_load(reinterpret_cast<const u32x4_nt*>(esrc + out_row(row) * g.NC + col));
          extra[k] = make_uint4(q.x, q.y, q.z, q.w);
        } else {
          extra[k] = in ? *reinterpret_cast<const uint4*>(esrc + out_row(row) * g.NC + col) : make_uint4(0, 0, 0, 0);
        }
      }
    }
    if (pass) __syncthreads();                   // the previous pass has been read out
    if (active && (wm * TM * 32) / PR == pass) {
      // column block outermost: the affine pair of a column is fetched once and is live for TM rows only
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int lcol = wn * TN * 32 + j * 32 + 8 * q + 4 * (lane >> 5);
          float4 ea = make_float4(1.f, 1.f, 1.f, 1.f), eb = make_float4(0.f, 0.f, 0.f, 0.f);
          if (EPI == EPI_AFFINE_ACT) {
            ea = *reinterpret_cast<const float4*>(ep_s + lcol);
            eb = *reinterpret_cast<const float4*>(ep_s + BN + lcol);
          }
#pragma unroll
          for (int i = 0; i < TM; ++i) {
            const int lr = (wm * TM * 32) % PR + i * 32 + (lane & 31);
            float o[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = acc[i][j][4 * q + e];
            if (EPI == EPI_ACCUM) {
              *reinterpret_cast<float4*>(smem + lr * OP + lcol * 4) = make_float4(o[0], o[1], o[2], o[3]);
            } else {
              if (EPI == EPI_AFFINE_ACT) {
                o[0] = apply_act(fmaf(o[0], ea.x, eb.x), act); o[1] = apply_act(fmaf(o[1], ea.y, eb.y), act);
                o[2] = apply_act(fmaf(o[2], ea.z, eb.z), act); o[3] = apply_act(fmaf(o[3], ea.w, eb.w), act);
              }
              uint2 pk;
              pk.x = pack_bf2(o[0], o[1]);
              pk.y = pack_bf2(o[2], o[3]);
              *reinterpret_cast<uint2*>(smem + lr * OP + lcol * 2) = pk;
            }
          }
        }
    }
    __syncthreads();
    if (tid < ST) {
#pragma unroll
      for (int k = 0; k < CPT; ++k) {
        const int cidx = tid + k * ST;
        const int lr = cidx / CPROW, c16 = cidx % CPROW;
        const int row = m0 + rbase + lr, col = n0 + c16 * 8;
        if (full || (row < Mrows && col < g.NC)) {   // NC % 8 == 0: a chunk is in or out as a whole
          uint4 v;
          if (EPI == EPI_ACCUM) {
            const float4 lo = *reinterpret_cast<const float4*>(smem + lr * OP + c16 * 32);
            const float4 hi = *reinterpret_cast<const float4*>(smem + lr * OP + c16 * 32 + 16);
            v.x = pack_bf2(lo.x + bf_lo(extra[k].x), lo.y + bf_hi(extra[k].x));
            v.y = pack_bf2(lo.z + bf_lo(extra[k].y), lo.w + bf_hi(extra[k].y));
            v.z = pack_bf2(hi.x + bf_lo(extra[k].z), hi.y + bf_hi(extra[k].z));
            v.w = pack_bf2(hi.z + bf_lo(extra[k].w), hi.w + bf_hi(extra[k].w));
          } else {
            v = *reinterpret_cast<const uint4*>(smem + lr * OP + c16 * 16);
            if (EPI == EPI_STORE && g.stats) {
              const float f[8] = {bf_lo(v.x), bf_hi(v.x), bf_lo(v.y), bf_hi(v.y), bf_lo(v.z), bf_hi(v.z), bf_lo(v.w), bf_hi(v.w)};
#pragma unroll
              for (int e = 0; e < 8; ++e) { s1[e] += f[e]; s2[e] = fmaf(f[e], f[e], s2[e]); }
            }
            if (g.res) {
              const uint4 r_ = extra[k];
              v.x = pack_bf2(apply_act(bf_lo(v.x) + bf_lo(r_.x), g.res_act), apply_act(bf_hi(v.x) + bf_hi(r_.x), g.res_act));
              v.y = pack_bf2(apply_act(bf_lo(v.y) + bf_lo(r_.y), g.res_act), apply_act(bf_hi(v.y) + bf_hi(r_.y), g.res_act));
              v.z = pack_bf2(apply_act(bf_lo(v.z) + bf_lo(r_.z), g.res_act), apply_act(bf_hi(v.z) + bf_hi(r_.z), g.res_act));
              v.w = pack_bf2(apply_act(bf_lo(v.w) + bf_lo(r_.w), g.res_act), apply_act(bf_hi(v.w) + bf_hi(r_.w), g.res_act));
            }
          }
          if (g.stream_out) {                    // a tensor far larger than the caches: its lines are not kept there
            typedef unsigned int u32x4_nt __attribute__((ext_vector_type(4)));
            const u32x4_nt q = {v.x, v.y, v.z, v.w};
            __builtin_nontemporal_store(q, reinterpret_cast<u32x4_nt*>(Out + out_row(row) * g.NC + col));
          } else {
            *reinterpret_cast<uint4*>(Out + out_row(row) * g.NC + col) = v;
          }
        }
      }
    }
  }
  if (EPI == EPI_STORE && g.stats) {
    // storing threads with equal tid % CPROW hold the same 8 channels: their sums meet in LDS and the column's
    // first thread adds them in thread order (a fixed association)
    __syncthreads();                             // the staged rows have been read by everyone
    float* red = reinterpret_cast<float*>(smem); // [storing thread][16]
    if (tid < ST) {
      *reinterpret_cast<float4*>(red + tid * 16) = make_float4(s1[0], s1[1], s1[2], s1[3]);
      *reinterpret_cast<float4*>(red + tid * 16 + 4) = make_float4(s1[4], s1[5], s1[6], s1[7]);
      *reinterpret_cast<float4*>(red + tid * 16 + 8) = make_float4(s2[0], s2[1], s2[2], s2[3]);
      *reinterpret_cast<float4*>(red + tid * 16 + 12) = make_float4(s2[4], s2[5], s2[6], s2[7]);
    }
    __syncthreads();
    // thread t: column t / 16, value t % 16 (8 sums, 8 sums of squares)
    const int cc = tid >> 4, e = tid & 15, col = n0 + cc * 8;
    if (cc < CPROW && col < g.NC) {
      float t = 0.f;
      for (int w = 0; w < ST / CPROW; ++w) t += red[(w * CPROW + cc) * 16 + e];
      g.stats[(size_t)stat_row * 2 * g.NC + (e >> 3) * g.NC + col + (e & 7)] = t;
    }
  }
}

// blockIdx.x < g.big_tiles: big tile number xcd_contiguous(blockIdx.x, big_tiles) (column tiles of a row tile
// next to each other, each XCD a contiguous run).  Above that: 64-row tail tiles over the rows from
// g.tail_m0 on, in order.  With parity classes (g.par_classes > 0) the big tiles are ordered column tile
// fastest, then class, then row tile: the classes of one row range read the same rows of A, and every XCD
// gets the same mix of heavy and light classes.
template <int MODE, int BN, int BK, int EPI>
__global__ __launch_bounds__(kDmaThreads) void igemm_dma_kernel(const bf16_t* __restrict__ A,
                                                                const bf16_t* __restrict__ Bw,
                                                                bf16_t* __restrict__ Out,
                                                                const float* __restrict__ ep_a,
                                                                const float* __restrict__ ep_b, int act,
                                                                IgemmArgs g) {
  __shared__ __attribute__((aligned(1024))) unsigned char smem[dma_lds_bytes(BN, BK, EPI == EPI_ACCUM)];
  __shared__ __attribute__((aligned(16))) float ep_s[EPI == EPI_AFFINE_ACT ? 2 * BN : 4];
  if ((int)blockIdx.x < g.big_tiles) {
    const int tile = xcd_contiguous(blockIdx.x, g.big_tiles);
    const int tile_n = tile % g.tiles_n;
    int tile_m = tile / g.tiles_n, cls = -1;
    if (MODE == 1 && g.par_classes) {
      cls = (g.par_order >> (2 * (tile_m % g.par_classes))) & 3;
      tile_m /= g.par_classes;
    }
    dma_tile<MODE, kDmaBM, BN, BK, dma_waves_m(BN), EPI>(smem, ep_s, A, Bw, Out, ep_a, ep_b, act, g, tile_m * kDmaBM, tile_n * BN, tile_m, cls);
  } else {
    const int tile = blockIdx.x - g.big_tiles;
    const int tile_n = tile % g.tiles_n, tile_m = tile / g.tiles_n;
    dma_tile<MODE, kDmaTailBM, BN, BK, 1, EPI>(smem, ep_s, A, Bw, Out, ep_a, ep_b, act, g, g.tail_m0 + tile_m * kDmaTailBM,
                                               tile_n * BN, g.big_tiles / g.tiles_n + tile_m);
  }
}

// ---------------------------------------------------------------------------
// Weight gradient for the 3 x 3 layers: 256-column tiles, eight wavefronts, direct-to-LDS loads.
//   dW[k][j] = sum_m dy[m][k] * xcol[m][j],  j = (r*S + s)*C + c          (same as wgrad_tr_kernel)
// Tile TM (output channels k: 256 / 192 / 128 / 96 / 64) x 256 (columns j), reduction over pixels in steps of
// 32, ring of four stages, one barrier a step.  Tiles lie in LDS as they lie in memory (rows = pixels) and the
// MFMA fragments come out of the transposing read ds_read_b64_tr_b16, as in wgrad_tr_kernel; what changes is
// that a stage is written by buffer_load ... lds (no register round trip), so rows are unpadded and bank
// conflicts of the transposing reads are avoided by a swizzle: one read cycle serves 32 lanes = 4 pixel rows x
// 64 contiguous bytes, so the 64-byte blocks of a row are permuted by the row number such that four consecutive
// rows land in four different 16-bank groups (which permutation depends on the row pitch modulo 256 bytes).
// Reads are inline assembly with their own waits, for the reason given at igemm_dma_kernel.
// ---------------------------------------------------------------------------
// XOR mask on the 16-byte chunk index of a row of `elems` bf16 elements
__device__ __forceinline__ constexpr int tr_swizzle(int elems, int row) {
  return elems == 96 ? 0 : (elems == 192 || elems == 64) ? ((row >> 1) & 1) << 2 : (row & 3) << 2;
}

typedef short s16x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ s16x4_t lds_read_tr4_async(unsigned addr) {
  s16x4_t v;
  asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(v) : "v"(addr) : "memory");
  return v;
}
__device__ __forceinline__ void pin4(s16x4_t& v) { asm volatile("" : "+v"(v)); }

constexpr int kWgradTN = 256;
constexpr int kWgradStages = 4;
constexpr int wgrad_dma_lds_bytes(int TM) { return kWgradStages * 32 * (TM + kWgradTN) * 2; }

template <int TM>
__global__ __launch_bounds__(kDmaThreads) void wgrad_dma_kernel(const bf16_t* __restrict__ dy,
                                                                const bf16_t* __restrict__ x,
                                                                float* __restrict__ part, WgradTrArgs g) {
  constexpr int TN = kWgradTN, BKP = 32, NS = kWgradStages;
  constexpr int WK = TM >= 128 ? 2 : 1, WJ = 8 / WK;              // wave grid: channels x columns
  constexpr int WTM = TM / WK, WTN = TN / WJ;                      // a wave's part of the tile
  constexpr int TWM = WTM / 32, TWN = WTN / 32;
  static_assert(TWM * 32 * WK == TM && TWN * 32 * WJ == TN, "wave grid");
  constexpr int CPA = TM / 8, CPB = TN / 8;                        // 16-byte chunks per tile row
  constexpr int PA = TM * 2, PB = TN * 2;                          // row pitch, bytes
  constexpr int A_BYTES = BKP * PA, STAGE = BKP * (PA + PB);
  constexpr int A_INSTR_ALL = BKP * CPA / 64, B_INSTR_ALL = BKP * CPB / 64;   // wave instructions per stage
  constexpr int A_INSTR = (A_INSTR_ALL + 7) / 8, B_INSTR = B_INSTR_ALL / 8;   // ... per wave (A: at most)
  static_assert(B_INSTR_ALL % 8 == 0 && (BKP * CPA) % 64 == 0, "whole wave instructions");
  __shared__ __attribute__((aligned(1024))) unsigned char smem[wgrad_dma_lds_bytes(TM)];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // uniform, and known to the compiler as such
  const int wm = wave / WJ, wn = wave % WJ;
  // all tiles of one pixel slice read the same rows of dy and x: keep them on one XCD (one L2)
  const int tile = xcd_contiguous(blockIdx.x, g.tiles_k * g.tiles_j * g.splits);
  const int slice = tile / (g.tiles_k * g.tiles_j);
  const int k0 = ((tile / g.tiles_j) % g.tiles_k) * TM, j0 = (tile % g.tiles_j) * TN;
  const int mbeg = slice * g.pix_per_split;
  const int mend = min(g.M, mbeg + g.pix_per_split);
  const int nsteps = (mend - mbeg + BKP - 1) / BKP;
  const __amdgpu_buffer_rsrc_t rdy = tensor_rsrc(dy, g.dy_bytes), rx = tensor_rsrc(x, g.x_bytes);

  // ---- dy chunks of this thread: flat chunk (i*8 + wave)*64 + lane of the 32 x TM tile -----------
  unsigned a_off[A_INSTR];
  int a_cnt = 0;
#pragma unroll
  for (int i = 0; i < A_INSTR; ++i) {
    const int u = i * 8 + wave;
    if (u < A_INSTR_ALL) ++a_cnt;
    const int ci = u * 64 + lane, row = ci / CPA, slot = ci % CPA;
    const int kc = k0 + (slot ^ tr_swizzle(TM, row)) * 8;
    // rows past the end of the tensor read as zeros (pix_per_split is a multiple of 32: only the last slice is ragged)
    a_off[i] = u < A_INSTR_ALL && kc < g.K ? (unsigned)((mbeg + row) * g.K + kc) * 2u : kOutOfRange;
  }
  const unsigned a_step = (unsigned)(BKP * g.K) * 2u;
  // ---- x chunks: the column chunk fixes the tap (br, bs) and first channel bc; the pixel advances by 32 a step ----
  const int b_slot = lane % CPB;                                   // (CPB = 32: the same slot for both instructions)
  int bn[B_INSTR], bp[B_INSTR], bq[B_INSTR], bm[B_INSTR], br[B_INSTR], bs[B_INSTR], bc[B_INSTR];
  bool b_ok[B_INSTR];
#pragma unroll
  for (int i = 0; i < B_INSTR; ++i) {
    const int ci = (i * 8 + wave) * 64 + lane, row = ci / CPB;
    const int jcol = j0 + ((b_slot ^ tr_swizzle(TN, row)) * 8);
    b_ok[i] = jcol < g.J;
    const int rs = b_ok[i] ? jcol / g.C : 0;
    bc[i] = b_ok[i] ? jcol - rs * g.C : 0;
    br[i] = rs / g.S;
    bs[i] = rs - br[i] * g.S;
    bm[i] = mbeg + row;
    bq[i] = bm[i] % g.Q;
    const int t = bm[i] / g.Q;
    bp[i] = t % g.P;
    bn[i] = t / g.P;
  }
  const int lps = a_cnt + B_INSTR;

  auto issue_stage = [&](int stage) {
    unsigned char* sa = smem + stage * STAGE + wave * 1024;
#pragma unroll
    for (int i = 0; i < A_INSTR; ++i) {
      if (i * 8 + wave >= A_INSTR_ALL) continue;                  // (uniform over the wave)
      dma_load16(rdy, sa + i * 8 * 1024, a_off[i]);
      a_off[i] += a_off[i] == kOutOfRange ? 0u : a_step;
    }
#pragma unroll
    for (int i = 0; i < B_INSTR; ++i) {
      const int h = bp[i] * g.stride + br[i] - g.pad, w = bq[i] * g.stride + bs[i] - g.pad;
      const bool ok = b_ok[i] && bm[i] < mend && (unsigned)h < (unsigned)g.H && (unsigned)w < (unsigned)g.W;
      dma_load16(rx, sa + A_BYTES + i * 8 * 1024, ok ? (unsigned)(((bn[i] * g.H + h) * g.W + w) * g.C + bc[i]) * 2u : kOutOfRange);
      bm[i] += BKP;
      const int q = bq[i] + g.dq;
      const int c1 = q >= g.Q ? 1 : 0;
      bq[i] = q - (c1 ? g.Q : 0);
      const int pp = bp[i] + g.dp + c1;
      const int c2 = pp >= g.P ? 1 : 0;
      bp[i] = pp - (c2 ? g.P : 0);
      bn[i] += g.dn + c2;
    }
  };

  // ---- fragment addresses: 16-lane group gl reads channels 16 (gl & 1) .. +15 of pixels 8 (gl >> 1) .. +3 (and +4) ----
  const int s16 = lane & 15, gl = lane >> 4;
  const int frow = 8 * (gl >> 1) + (s16 >> 2), fcol = 16 * (gl & 1) + 4 * (s16 & 3);
  unsigned fa[TWM], fb[TWN];
#pragma unroll
  for (int i = 0; i < TWM; ++i) {
    const int col = wm * WTM + i * 32 + fcol;
    fa[i] = (unsigned)(frow * PA + (((col >> 3) ^ tr_swizzle(TM, frow)) << 4) + (col & 7) * 2);
  }
#pragma unroll
  for (int j = 0; j < TWN; ++j) {
    const int col = wn * WTN + j * 32 + fcol;
    fb[j] = (unsigned)(A_BYTES + frow * PB + (((col >> 3) ^ tr_swizzle(TN, frow)) << 4) + (col & 7) * 2);
  }

  f32x16 acc[TWM][TWN];
#pragma unroll
  for (int i = 0; i < TWM; ++i)
#pragma unroll
    for (int j = 0; j < TWN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  struct Frag { s16x4_t a[TWM][2], b[TWN][2]; };
  auto read_frag = [&](Frag& f, unsigned base, int ks) {
    // rows 16 ks + frow (+4): offsets are multiples of 4 rows, so a lane's swizzle mask is the same for all of them
#pragma unroll
    for (int i = 0; i < TWM; ++i) {
      f.a[i][0] = lds_read_tr4_async(base + fa[i] + ks * 16 * PA);
      f.a[i][1] = lds_read_tr4_async(base + fa[i] + ks * 16 * PA + 4 * PA);
    }
#pragma unroll
    for (int j = 0; j < TWN; ++j) {
      f.b[j][0] = lds_read_tr4_async(base + fb[j] + ks * 16 * PB);
      f.b[j][1] = lds_read_tr4_async(base + fb[j] + ks * 16 * PB + 4 * PB);
    }
  };
  auto mfma_frag = [&](Frag& f) {
    bf16x8 af[TWM], bfr[TWN];
#pragma unroll
    for (int i = 0; i < TWM; ++i) {
      pin4(f.a[i][0]); pin4(f.a[i][1]);
      af[i] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(f.a[i][0], f.a[i][1], 0, 1, 2, 3, 4, 5, 6, 7));
    }
#pragma unroll
    for (int j = 0; j < TWN; ++j) {
      pin4(f.b[j][0]); pin4(f.b[j][1]);
      bfr[j] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(f.b[j][0], f.b[j][1], 0, 1, 2, 3, 4, 5, 6, 7));
    }
#pragma unroll
    for (int i = 0; i < TWM; ++i)
#pragma unroll
      for (int j = 0; j < TWN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
  };

#pragma unroll
  for (int st = 0; st < NS - 1; ++st)
    if (st < nsteps) issue_stage(st);
  int stage = 0, next = NS - 1;
  for (int st = 0; st < nsteps; ++st) {
    // younger stages whose loads may stay in flight: up to NS - 2
    wait_vmcnt_dyn(min(NS - 2, nsteps - 1 - st) * lps);
    block_barrier();
    if (st + NS - 1 < nsteps) issue_stage(next);
    const unsigned sbase = (unsigned)(stage * STAGE);
    Frag f0, f1;
    read_frag(f0, sbase, 0);
    read_frag(f1, sbase, 1);
    wait_lgkmcnt<2 * (TWM + TWN)>();            // LDS reads return in order: the first group is complete
    mfma_frag(f0);
    __builtin_amdgcn_sched_barrier(0);
    wait_lgkmcnt<0>();
    mfma_frag(f1);
    __builtin_amdgcn_sched_barrier(0);
    stage = stage + 1 == NS ? 0 : stage + 1;
    next = next + 1 == NS ? 0 : next + 1;
  }
  wait_vmcnt<0>();

  float* out = part + (size_t)slice * g.K * g.J;
#pragma unroll
  for (int j = 0; j < TWN; ++j) {
    const int col = j0 + wn * WTN + j * 32 + (lane & 31);
    if (col >= g.J) continue;
#pragma unroll
    for (int i = 0; i < TWM; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = k0 + wm * WTM + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (row < g.K) out[(size_t)row * g.J + col] = acc[i][j][v];
      }
  }
}

}  // namespace pbd
