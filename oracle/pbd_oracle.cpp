// CPU oracle for one blockwise-distillation step.  TEST INFRASTRUCTURE ONLY:
// it exists to check the HIP library and to be timed beside it; nothing on the
// product path may call it.  It shares no code with the HIP path.
//
// What it computes (Sec. II-A; Algorithm 1, the load / T.forward / S.forward /
// S.backward(L) / update_weight lines; Sec. IV-B for the per-block update):
//   A_0 = x,  A_i = T_i(A_{i-1})         teacher, frozen, BN in inference mode
//   S^_i = S_i(A_{i-1})                   student, BN with batch statistics
//   loss_i = mean((S^_i - A_i)^2)         L(delta output), read as MSE
//   backprop through S_i only, then  v <- mu v + g,  w <- w - lr v.
// The method only reschedules work (Abstract; Sec. VII-D), so the oracle is the
// plain definition: direct nested loops over NCHW tensors, no blocking, no
// BLAS.  `relay` keeps every A_i; `redundant` re-runs T_1..T_{i-1} from A_0 for
// each block the way the data-parallel baseline does (Sec. II-B, Sec. III).
// Scalar type R is double (reference of record) or float (noise-floor / timing).
//
// Readings where the paper is silent: MSE averaged over all elements; PyTorch
// form of SGD momentum, no weight decay; teacher BN frozen, student BN in
// training mode with running statistics updated (eps 1e-5, rate 0.1, unbiased
// running variance); convolutions are cross-correlations without bias and
// with zero padding; max-pool gradients go to the first maximum in row-major
// window order.
//
// Architecture round of a NAS supernet (Sec. VI-A, the neural architecture search workload): a mix
// op's weights are p = softmax(alpha) over its candidates, alpha being the trainable architecture
// parameters; a step has a second forward/backward round that trains alpha with the weights frozen,
// and that round is an ordinary training step of the block.  Here: same forward (student BN in
// training mode, running statistics updated), same loss, backward through the block to every mix,
//   g_k = <dL/dz, y_k>,   dL/dalpha_j = p_j (g_j - sum_k p_k g_k)      (chain rule through softmax)
// then the SGD-momentum rule on alpha only.  Readings where the paper is silent: the same optimiser
// rule for alpha as for weights with a learning rate of its own; every candidate evaluated and
// mixed (no sampling of paths); alpha starts at ln p_k of the descriptor's weights, and a mix keeps
// the descriptor's p_k untouched until alpha is set or trained.
//
// Optional storage rounding (storage = 1): the bf16 path of the method keeps tensors
// (activations, compute copies of weights, activation gradients) in bfloat16 and
// everything else in wider precision.  ReLU masks, max-pool winners and the bf16
// codes themselves are decisions taken by floating point, and a gradient summed over
// a kinked network is discontinuous in them; so that both sides take those decisions
// in the same precision, this mode rounds to bfloat16 (nearest even) exactly where the
// path stores a tensor and keeps every other operation in R.  storage = 0 is the
// plain definition and stays the reference for losses and activations.
//
// Pins (tests/test_oracle_*.py): brute-force convolution, 1x1 conv == matrix
// product, adjoint identities for dgrad/wgrad, BN closed forms, central finite
// differences of loss_i over every parameter, PyTorch-CPU fp64 autograd on the
// same blocks, SGD closed form, relay == redundant bitwise, block-order
// independence; for the architecture round central finite differences of loss_i over alpha,
// PyTorch autograd with alpha as a leaf, sum_j dL/dalpha_j = 0, identical candidates.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <memory>
#include <string>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

enum { OP_CBA = 1, OP_POOL = 2, OP_ADD = 3, OP_MIX = 4 };
enum { ACT_NONE = 0, ACT_RELU = 1, ACT_RELU6 = 2 };
constexpr int32_t kMagic = 0x50424431;
constexpr int kRec = 20;

// ---------------------------------------------------------------------------
// primitives (NCHW, direct loops)
// ---------------------------------------------------------------------------

inline int out_dim(int h, int k, int s, int pad) { return (h + 2 * pad - k) / s + 1; }

// Y[n,k,p,q] = sum_{c,r,t} X[n, g*Cg + c, p*s + r - pad, q*s + t - pad] * W[k,c,r,t]
template <class R>
void conv_fwd(const R* x, const R* w, R* y, int N, int C, int H, int W, int K, int k,
              int stride, int pad, int groups) {
  const int P = out_dim(H, k, stride, pad), Q = out_dim(W, k, stride, pad);
  const int Cg = C / groups, Kg = K / groups;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int ko = 0; ko < K; ++ko) {
      const int g = ko / Kg;
      for (int p = 0; p < P; ++p)
        for (int q = 0; q < Q; ++q) {
          R acc = 0;
          for (int c = 0; c < Cg; ++c)
            for (int r = 0; r < k; ++r) {
              const int h = p * stride + r - pad;
              if (h < 0 || h >= H) continue;
              for (int t = 0; t < k; ++t) {
                const int ww = q * stride + t - pad;
                if (ww < 0 || ww >= W) continue;
                acc += x[((size_t)(n * C + g * Cg + c) * H + h) * W + ww] *
                       w[((size_t)(ko * Cg + c) * k + r) * k + t];
              }
            }
          y[((size_t)(n * K + ko) * P + p) * Q + q] = acc;
        }
    }
}

// dX = adjoint of conv_fwd in X: every output position scatters dY*W back.
template <class R>
void conv_dgrad(const R* dy, const R* w, R* dx, int N, int C, int H, int W, int K, int k,
                int stride, int pad, int groups) {
  const int P = out_dim(H, k, stride, pad), Q = out_dim(W, k, stride, pad);
  const int Cg = C / groups, Kg = K / groups;
#pragma omp parallel for schedule(static)
  for (int n = 0; n < N; ++n) {
    std::fill(dx + (size_t)n * C * H * W, dx + (size_t)(n + 1) * C * H * W, R(0));
    for (int ko = 0; ko < K; ++ko) {
      const int g = ko / Kg;
      for (int p = 0; p < P; ++p)
        for (int q = 0; q < Q; ++q) {
          const R d = dy[((size_t)(n * K + ko) * P + p) * Q + q];
          for (int c = 0; c < Cg; ++c)
            for (int r = 0; r < k; ++r) {
              const int h = p * stride + r - pad;
              if (h < 0 || h >= H) continue;
              for (int t = 0; t < k; ++t) {
                const int ww = q * stride + t - pad;
                if (ww < 0 || ww >= W) continue;
                dx[((size_t)(n * C + g * Cg + c) * H + h) * W + ww] +=
                    d * w[((size_t)(ko * Cg + c) * k + r) * k + t];
              }
            }
        }
    }
  }
}

// dW[k,c,r,t] = sum_{n,p,q} dY[n,k,p,q] * X[n, g*Cg + c, p*s + r - pad, q*s + t - pad]
template <class R>
void conv_wgrad(const R* dy, const R* x, R* dw, int N, int C, int H, int W, int K, int k,
                int stride, int pad, int groups) {
  const int P = out_dim(H, k, stride, pad), Q = out_dim(W, k, stride, pad);
  const int Cg = C / groups, Kg = K / groups;
#pragma omp parallel for collapse(2) schedule(static)
  for (int ko = 0; ko < K; ++ko)
    for (int c = 0; c < Cg; ++c) {
      const int g = ko / Kg;
      for (int r = 0; r < k; ++r)
        for (int t = 0; t < k; ++t) {
          R acc = 0;
          for (int n = 0; n < N; ++n)
            for (int p = 0; p < P; ++p) {
              const int h = p * stride + r - pad;
              if (h < 0 || h >= H) continue;
              for (int q = 0; q < Q; ++q) {
                const int ww = q * stride + t - pad;
                if (ww < 0 || ww >= W) continue;
                acc += dy[((size_t)(n * K + ko) * P + p) * Q + q] *
                       x[((size_t)(n * C + g * Cg + c) * H + h) * W + ww];
              }
            }
          dw[((size_t)(ko * Cg + c) * k + r) * k + t] = acc;
        }
    }
}

// Batch normalisation with batch statistics: per channel over m = N*HW,
// mu = mean, var = biased variance, xhat = (x-mu)/sqrt(var+eps), y = gamma*xhat+beta.
template <class R>
void bn_train_fwd(const R* x, const R* gamma, const R* beta, R* y, R* mean, R* var, int N,
                  int C, int HW, R eps) {
  const R m = (R)N * (R)HW;
#pragma omp parallel for schedule(static)
  for (int c = 0; c < C; ++c) {
    R s = 0;
    for (int n = 0; n < N; ++n)
      for (int i = 0; i < HW; ++i) s += x[((size_t)n * C + c) * HW + i];
    const R mu = s / m;
    R v = 0;
    for (int n = 0; n < N; ++n)
      for (int i = 0; i < HW; ++i) {
        const R d = x[((size_t)n * C + c) * HW + i] - mu;
        v += d * d;
      }
    v /= m;
    mean[c] = mu;
    var[c] = v;
    const R inv = R(1) / std::sqrt(v + eps);
    for (int n = 0; n < N; ++n)
      for (int i = 0; i < HW; ++i) {
        const size_t o = ((size_t)n * C + c) * HW + i;
        y[o] = gamma[c] * ((x[o] - mu) * inv) + beta[c];
      }
  }
}

// dbeta = sum dy, dgamma = sum dy*xhat,
// dx = gamma/sqrt(var+eps) * (dy - dbeta/m - xhat*dgamma/m)
template <class R>
void bn_train_bwd(const R* dy, const R* x, const R* gamma, const R* mean, const R* var, R* dx,
                  R* dgamma, R* dbeta, int N, int C, int HW, R eps) {
  const R m = (R)N * (R)HW;
#pragma omp parallel for schedule(static)
  for (int c = 0; c < C; ++c) {
    const R inv = R(1) / std::sqrt(var[c] + eps);
    R sb = 0, sg = 0;
    for (int n = 0; n < N; ++n)
      for (int i = 0; i < HW; ++i) {
        const size_t o = ((size_t)n * C + c) * HW + i;
        sb += dy[o];
        sg += dy[o] * ((x[o] - mean[c]) * inv);
      }
    dbeta[c] = sb;
    dgamma[c] = sg;
    for (int n = 0; n < N; ++n)
      for (int i = 0; i < HW; ++i) {
        const size_t o = ((size_t)n * C + c) * HW + i;
        const R xh = (x[o] - mean[c]) * inv;
        dx[o] = gamma[c] * inv * (dy[o] - sb / m - xh * sg / m);
      }
  }
}

// Inference-mode BN: y = gamma*(x - rmean)/sqrt(rvar+eps) + beta.
template <class R>
void bn_eval(const R* x, const R* gamma, const R* beta, const R* rmean, const R* rvar, R* y,
             int N, int C, int HW, R eps) {
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int c = 0; c < C; ++c) {
      const R inv = R(1) / std::sqrt(rvar[c] + eps);
      for (int i = 0; i < HW; ++i) {
        const size_t o = ((size_t)n * C + c) * HW + i;
        y[o] = gamma[c] * ((x[o] - rmean[c]) * inv) + beta[c];
      }
    }
}

template <class R>
void act_fwd(const R* x, R* y, size_t n, int act) {
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < n; ++i) {
    R v = x[i];
    if (act == ACT_RELU) v = v > 0 ? v : R(0);
    if (act == ACT_RELU6) v = v > 0 ? (v < 6 ? v : R(6)) : R(0);
    y[i] = v;
  }
}

// x is the pre-activation; gradient passes where the activation has slope 1.
template <class R>
void act_bwd(const R* dy, const R* x, R* dx, size_t n, int act) {
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < n; ++i) {
    bool pass = true;
    if (act == ACT_RELU) pass = x[i] > 0;
    if (act == ACT_RELU6) pass = x[i] > 0 && x[i] < 6;
    dx[i] = pass ? dy[i] : R(0);
  }
}

// Window max over a (-inf)-padded input; idx keeps the flat h*W+w of the first
// maximum met in row-major window order.
template <class R>
void maxpool_fwd(const R* x, R* y, int32_t* idx, int N, int C, int H, int W, int k, int stride,
                 int pad) {
  const int P = out_dim(H, k, stride, pad), Q = out_dim(W, k, stride, pad);
#pragma omp parallel for schedule(static)
  for (int nc = 0; nc < N * C; ++nc)
    for (int p = 0; p < P; ++p)
      for (int q = 0; q < Q; ++q) {
        R best = -std::numeric_limits<R>::infinity();
        int bi = -1;
        for (int r = 0; r < k; ++r) {
          const int h = p * stride + r - pad;
          if (h < 0 || h >= H) continue;
          for (int t = 0; t < k; ++t) {
            const int ww = q * stride + t - pad;
            if (ww < 0 || ww >= W) continue;
            const R v = x[((size_t)nc * H + h) * W + ww];
            if (bi < 0 || v > best) { best = v; bi = h * W + ww; }
          }
        }
        y[((size_t)nc * P + p) * Q + q] = best;
        idx[((size_t)nc * P + p) * Q + q] = bi;
      }
}

template <class R>
void maxpool_bwd(const R* dy, const int32_t* idx, R* dx, int N, int C, int H, int W, int P, int Q) {
#pragma omp parallel for schedule(static)
  for (int nc = 0; nc < N * C; ++nc) {
    R* d = dx + (size_t)nc * H * W;
    std::fill(d, d + (size_t)H * W, R(0));
    for (int o = 0; o < P * Q; ++o) d[idx[(size_t)nc * P * Q + o]] += dy[(size_t)nc * P * Q + o];
  }
}

// loss = (1/M) sum (s-t)^2 ; ds = 2 (s-t) / M
template <class R>
R mse(const R* s, const R* t, R* ds, size_t M) {
  R acc = 0;
  for (size_t i = 0; i < M; ++i) {
    const R d = s[i] - t[i];
    acc += d * d;
    if (ds) ds[i] = R(2) * d / (R)M;
  }
  return acc / (R)M;
}

// v <- mu v + g ; w <- w - lr v
template <class R>
void sgd(R* w, R* v, const R* g, size_t n, R lr, R mu) {
  for (size_t i = 0; i < n; ++i) {
    v[i] = mu * v[i] + g[i];
    w[i] = w[i] - lr * v[i];
  }
}

// Gradient of the loss with respect to the architecture parameters of one weighted sum
// z = sum_k p_k y_k, p = softmax(alpha) (Sec. VI-A, the architecture round), given dL/dz:
//   g_k = <dL/dz, y_k>,   dL/dalpha_j = p_j (g_j - sum_k p_k g_k)      (dp_k/dalpha_j = p_k ([k == j] - p_j))
template <class R>
void mix_alpha_grad(const R* dz, const R* const* y, const R* p, int n, size_t numel, R* dalpha) {
  std::vector<R> g(n, R(0));
  R mean = 0;
  for (int k = 0; k < n; ++k) {
    for (size_t i = 0; i < numel; ++i) g[k] += dz[i] * y[k][i];
    mean += p[k] * g[k];
  }
  for (int k = 0; k < n; ++k) dalpha[k] = p[k] * (g[k] - mean);
}

// nearest-even rounding to bfloat16 (8 significand bits), the storage type of the bf16 path
inline double round_bf16(double v) {
  float f = (float)v;
  uint32_t u;
  std::memcpy(&u, &f, 4);
  if ((u & 0x7f800000u) == 0x7f800000u) return (double)f;  // inf / nan unchanged
  u += 0x7fffu + ((u >> 16) & 1u);
  u &= 0xffff0000u;
  std::memcpy(&f, &u, 4);
  return (double)f;
}

// ---------------------------------------------------------------------------
// descriptor
// ---------------------------------------------------------------------------

struct OpD {
  int type, nin, in[8], c_out, k, stride, pad, groups, act, pofs;
};
struct Shape {
  int c, h, w;
  size_t numel() const { return (size_t)c * h * w; }
};
struct BlockD {
  std::vector<OpD> ops;
  std::vector<Shape> shapes;  // value 0 = block input
};

struct Desc {
  int B = 0;
  Shape in{};
  std::vector<BlockD> net[2];
  std::vector<double> pool;
  std::vector<Shape> act;  // A_0..A_B

  bool parse(const int32_t* w, int nw, const double* p, int np, std::string& err) {
    if (nw < 6 || w[0] != kMagic || w[1] != 1) { err = "bad header"; return false; }
    B = w[2];
    in = {w[3], w[4], w[5]};
    pool.assign(p, p + np);
    int pos = 6;
    for (int which = 0; which < 2; ++which) {
      Shape cur = in;
      for (int b = 0; b < B; ++b) {
        if (pos >= nw) { err = "truncated"; return false; }
        BlockD blk;
        const int nops = w[pos++];
        blk.shapes.push_back(cur);
        for (int j = 0; j < nops; ++j, pos += kRec) {
          if (pos + kRec > nw) { err = "truncated"; return false; }
          const int32_t* r = w + pos;
          OpD o{};
          o.type = r[0]; o.nin = r[1];
          for (int i = 0; i < 8; ++i) o.in[i] = r[2 + i];
          o.c_out = r[10]; o.k = r[11]; o.stride = r[12]; o.pad = r[13];
          o.groups = r[14]; o.act = r[15]; o.pofs = r[16];
          for (int i = 0; i < o.nin; ++i)
            if (o.in[i] < 0 || o.in[i] > j) { err = "input refers forward"; return false; }
          const Shape s = blk.shapes[o.in[0]];
          Shape out = s;
          if (o.type == OP_CBA) {
            if (o.groups != 1 && (o.groups != s.c || o.c_out != s.c)) { err = "groups"; return false; }
            out = {o.c_out, out_dim(s.h, o.k, o.stride, o.pad), out_dim(s.w, o.k, o.stride, o.pad)};
          } else if (o.type == OP_POOL) {
            out = {s.c, out_dim(s.h, o.k, o.stride, o.pad), out_dim(s.w, o.k, o.stride, o.pad)};
          } else if (o.type == OP_ADD || o.type == OP_MIX) {
            for (int i = 1; i < o.nin; ++i) {
              const Shape t = blk.shapes[o.in[i]];
              if (t.c != s.c || t.h != s.h || t.w != s.w) { err = "join shapes"; return false; }
            }
          } else { err = "op type"; return false; }
          blk.ops.push_back(o);
          blk.shapes.push_back(out);
        }
        cur = blk.shapes.back();
        net[which].push_back(std::move(blk));
      }
    }
    act.clear();
    act.push_back(in);
    for (int b = 0; b < B; ++b) {
      const Shape t = net[0][b].shapes.back(), s = net[1][b].shapes.back();
      if (t.c != s.c || t.h != s.h || t.w != s.w) { err = "teacher/student block shapes differ"; return false; }
      act.push_back(t);
    }
    return true;
  }
};

// ---------------------------------------------------------------------------
// networks
// ---------------------------------------------------------------------------

struct NetBase {
  virtual ~NetBase() = default;
  virtual int set_tensor(int kind, int net, int b, int j, int slot, const double* d, long n) = 0;
  virtual int get_tensor(int kind, int net, int b, int j, int slot, double* d, long n) = 0;
  virtual void teacher_relay(const double* x) = 0;
  virtual void teacher_upto(const double* x, int i, double* out) = 0;
  virtual long act_numel(int i) = 0;
  virtual void get_act(int i, double* out) = 0;
  virtual double student_step(int i, const double* a_prev, const double* a_i, double lr, int mode) = 0;
  virtual void relay_step(const double* x, double lr, double* losses) = 0;
  virtual void redundant_step(const double* x, double lr, double* losses) = 0;
  virtual long value_numel(int b, int v) = 0;
  virtual double kink_margin(int b) = 0;
  virtual void get_value(int b, int v, double* out) = 0;
  virtual long saved_numel(int b, int j, int which) = 0;
  virtual void get_saved(int b, int j, int which, double* out) = 0;
  virtual int set_alpha(int b, int j, const double* a, int n) = 0;
  virtual int get_alpha(int kind, int b, int j, double* out, int n) = 0;
  virtual void relay_arch_step(const double* x, double lr, double* losses) = 0;
};

template <class R>
struct Cba {
  std::vector<R> p[5];  // weight, gamma, beta, running mean, running var
  std::vector<R> g[3];  // gradients of weight, gamma, beta
  std::vector<R> v[3];  // momentum
};

template <class R>
struct Net final : NetBase {
  Desc d;
  int N;
  R mu, eps, rho;
  std::vector<std::vector<Cba<R>>> par[2];  // [net][block][op]
  std::vector<std::vector<R>> A;            // relay store A_0..A_B
  // student forward state of the block last run
  struct Saved {
    std::vector<R> conv, mean, var, pre;  // CBA: conv output, batch stats, BN output
    std::vector<int32_t> idx;             // POOL
  };
  std::vector<std::vector<std::vector<R>>> val;  // [block][value]
  std::vector<std::vector<Saved>> saved;         // [block][op]

  // architecture parameters of the student's mix ops [block][op]: value, gradient, momentum;
  // empty until set or trained (the mix then uses the descriptor's weights)
  std::vector<std::vector<std::vector<R>>> alpha, alpha_g, alpha_v;

  int storage = 0;  // 1: round stored tensors to bfloat16

  void rnd(std::vector<R>& v) const {
    if (!storage) return;
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < v.size(); ++i) v[i] = (R)round_bf16((double)v[i]);
  }
  // the compute copy of a weight tensor
  std::vector<R> stored(const std::vector<R>& w) const {
    std::vector<R> c = w;
    rnd(c);
    return c;
  }

  Net(const Desc& desc, int batch, double momentum, double e, double r, int st)
      : d(desc), N(batch), mu((R)momentum), eps((R)e), rho((R)r), storage(st) {
    for (int which = 0; which < 2; ++which) {
      par[which].resize(d.B);
      for (int b = 0; b < d.B; ++b) {
        const BlockD& blk = d.net[which][b];
        par[which][b].resize(blk.ops.size());
        for (size_t j = 0; j < blk.ops.size(); ++j) {
          const OpD& o = blk.ops[j];
          if (o.type != OP_CBA) continue;
          const int cin = blk.shapes[o.in[0]].c;
          Cba<R>& c = par[which][b][j];
          c.p[0].assign((size_t)o.c_out * (cin / o.groups) * o.k * o.k, R(0));
          c.p[1].assign(o.c_out, R(1));
          c.p[2].assign(o.c_out, R(0));
          c.p[3].assign(o.c_out, R(0));
          c.p[4].assign(o.c_out, R(1));
          for (int s = 0; s < 3; ++s) {
            c.g[s].assign(c.p[s].size(), R(0));
            c.v[s].assign(c.p[s].size(), R(0));
          }
        }
      }
    }
    A.resize(d.B + 1);
    val.resize(d.B);
    saved.resize(d.B);
    alpha.resize(d.B);
    alpha_g.resize(d.B);
    alpha_v.resize(d.B);
    for (int b = 0; b < d.B; ++b) {
      alpha[b].resize(d.net[1][b].ops.size());
      alpha_g[b].resize(d.net[1][b].ops.size());
      alpha_v[b].resize(d.net[1][b].ops.size());
    }
  }

  // mixing weights of student mix op j of block b: softmax(alpha) once alpha exists
  std::vector<R> probs(int b, int j) const {
    const OpD& o = d.net[1][b].ops[j];
    std::vector<R> p(o.nin);
    const std::vector<R>& a = alpha[b][j];
    if (a.empty()) {
      for (int k = 0; k < o.nin; ++k) p[k] = (R)d.pool[o.pofs + k];
      return p;
    }
    const R top = *std::max_element(a.begin(), a.end());
    R sum = 0;
    for (int k = 0; k < o.nin; ++k) { p[k] = std::exp(a[k] - top); sum += p[k]; }
    for (int k = 0; k < o.nin; ++k) p[k] /= sum;
    return p;
  }
  void define_alpha(int b) {
    const BlockD& blk = d.net[1][b];
    for (size_t j = 0; j < blk.ops.size(); ++j) {
      const OpD& o = blk.ops[j];
      if (o.type != OP_MIX) continue;
      if (alpha[b][j].empty()) {
        alpha[b][j].resize(o.nin);
        for (int k = 0; k < o.nin; ++k) alpha[b][j][k] = (R)std::log(d.pool[o.pofs + k]);
      }
      if (alpha_g[b][j].empty()) alpha_g[b][j].assign(o.nin, R(0));
      if (alpha_v[b][j].empty()) alpha_v[b][j].assign(o.nin, R(0));
    }
  }
  int set_alpha(int b, int j, const double* a, int n) override {
    if (b < 0 || b >= d.B || j < 0 || j >= (int)d.net[1][b].ops.size()) return -1;
    const OpD& o = d.net[1][b].ops[j];
    if (o.type != OP_MIX || n != o.nin) return -1;
    alpha[b][j].resize(n);
    for (int k = 0; k < n; ++k) alpha[b][j][k] = (R)a[k];
    return 0;
  }
  // kind 0: alpha, 1: its gradient, 2: its momentum, 3: the mixing weights in use
  int get_alpha(int kind, int b, int j, double* out, int n) override {
    if (b < 0 || b >= d.B || j < 0 || j >= (int)d.net[1][b].ops.size()) return -1;
    const OpD& o = d.net[1][b].ops[j];
    if (o.type != OP_MIX || n != o.nin) return -1;
    if (kind == 3) {
      const std::vector<R> p = probs(b, j);
      for (int k = 0; k < n; ++k) out[k] = (double)p[k];
      return 0;
    }
    const std::vector<R>& src = kind == 0 ? alpha[b][j] : kind == 1 ? alpha_g[b][j] : alpha_v[b][j];
    if (kind < 0 || kind > 2 || (int)src.size() != n) return -1;
    for (int k = 0; k < n; ++k) out[k] = (double)src[k];
    return 0;
  }

  std::vector<R>* find(int kind, int net, int b, int j, int slot) {
    if (net < 0 || net > 1 || b < 0 || b >= d.B) return nullptr;
    if (j < 0 || j >= (int)d.net[net][b].ops.size()) return nullptr;
    if (d.net[net][b].ops[j].type != OP_CBA) return nullptr;
    Cba<R>& c = par[net][b][j];
    if (kind == 0 && slot >= 0 && slot < 5) return &c.p[slot];
    if (kind == 1 && slot >= 0 && slot < 3) return &c.g[slot];
    if (kind == 2 && slot >= 0 && slot < 3) return &c.v[slot];
    return nullptr;
  }
  int set_tensor(int kind, int net, int b, int j, int slot, const double* src, long n) override {
    auto* t = find(kind, net, b, j, slot);
    if (!t || (long)t->size() != n) return -1;
    for (long i = 0; i < n; ++i) (*t)[i] = (R)src[i];
    return 0;
  }
  int get_tensor(int kind, int net, int b, int j, int slot, double* dst, long n) override {
    auto* t = find(kind, net, b, j, slot);
    if (!t || (long)t->size() != n) return -1;
    for (long i = 0; i < n; ++i) dst[i] = (double)(*t)[i];
    return 0;
  }

  // ---- teacher: every op in inference mode --------------------------------
  std::vector<R> teacher_block(int b, const std::vector<R>& x) {
    const BlockD& blk = d.net[0][b];
    std::vector<std::vector<R>> v(blk.ops.size() + 1);
    v[0] = x;
    for (size_t j = 0; j < blk.ops.size(); ++j) {
      const OpD& o = blk.ops[j];
      const Shape si = blk.shapes[o.in[0]], so = blk.shapes[j + 1];
      std::vector<R>& out = v[j + 1];
      out.assign((size_t)N * so.numel(), R(0));
      if (o.type == OP_CBA) {
        const Cba<R>& c = par[0][b][j];
        std::vector<R> y(out.size());
        const std::vector<R> w = stored(c.p[0]);
        conv_fwd(v[o.in[0]].data(), w.data(), y.data(), N, si.c, si.h, si.w, so.c, o.k,
                 o.stride, o.pad, o.groups);
        bn_eval(y.data(), c.p[1].data(), c.p[2].data(), c.p[3].data(), c.p[4].data(), y.data(), N,
                so.c, so.h * so.w, eps);
        act_fwd(y.data(), out.data(), out.size(), o.act);
        rnd(out);
      } else if (o.type == OP_POOL) {
        std::vector<int32_t> idx(out.size());
        maxpool_fwd(v[o.in[0]].data(), out.data(), idx.data(), N, si.c, si.h, si.w, o.k, o.stride,
                    o.pad);
      } else if (o.type == OP_ADD) {
        for (size_t i = 0; i < out.size(); ++i) out[i] = v[o.in[0]][i] + v[o.in[1]][i];
        act_fwd(out.data(), out.data(), out.size(), o.act);
        rnd(out);
      } else {  // OP_MIX
        for (int k = 0; k < o.nin; ++k) {
          const R p = (R)d.pool[o.pofs + k];
          for (size_t i = 0; i < out.size(); ++i) out[i] += p * v[o.in[k]][i];
        }
        rnd(out);
      }
    }
    return v.back();
  }

  void teacher_relay(const double* x) override {
    A[0].resize((size_t)N * d.in.numel());
    for (size_t i = 0; i < A[0].size(); ++i) A[0][i] = (R)x[i];
    rnd(A[0]);
    for (int b = 0; b < d.B; ++b) A[b + 1] = teacher_block(b, A[b]);  // each T_i once
  }
  // A_i recomputed from the raw input, T_1..T_i (the baseline's redundant work)
  std::vector<R> teacher_from_start(const double* x, int i) {
    std::vector<R> cur((size_t)N * d.in.numel());
    for (size_t k = 0; k < cur.size(); ++k) cur[k] = (R)x[k];
    rnd(cur);
    for (int b = 0; b < i; ++b) cur = teacher_block(b, cur);
    return cur;
  }
  void teacher_upto(const double* x, int i, double* out) override {
    std::vector<R> a = teacher_from_start(x, i);
    for (size_t k = 0; k < a.size(); ++k) out[k] = (double)a[k];
  }
  long act_numel(int i) override { return (long)N * (long)d.act[i].numel(); }
  void get_act(int i, double* out) override {
    for (size_t k = 0; k < A[i].size(); ++k) out[k] = (double)A[i][k];
  }

  // ---- student -------------------------------------------------------------
  void student_forward(int b, const std::vector<R>& x) {
    const BlockD& blk = d.net[1][b];
    auto& v = val[b];
    auto& sv = saved[b];
    v.assign(blk.ops.size() + 1, {});
    sv.assign(blk.ops.size(), {});
    v[0] = x;
    for (size_t j = 0; j < blk.ops.size(); ++j) {
      const OpD& o = blk.ops[j];
      const Shape si = blk.shapes[o.in[0]], so = blk.shapes[j + 1];
      std::vector<R>& out = v[j + 1];
      out.assign((size_t)N * so.numel(), R(0));
      if (o.type == OP_CBA) {
        const Cba<R>& c = par[1][b][j];
        Saved& s = sv[j];
        s.conv.resize(out.size());
        s.pre.resize(out.size());
        s.mean.resize(so.c);
        s.var.resize(so.c);
        const std::vector<R> w = stored(c.p[0]);
        conv_fwd(v[o.in[0]].data(), w.data(), s.conv.data(), N, si.c, si.h, si.w, so.c, o.k,
                 o.stride, o.pad, o.groups);
        rnd(s.conv);
        bn_train_fwd(s.conv.data(), c.p[1].data(), c.p[2].data(), s.pre.data(), s.mean.data(),
                     s.var.data(), N, so.c, so.h * so.w, eps);
        act_fwd(s.pre.data(), out.data(), out.size(), o.act);
        rnd(out);
      } else if (o.type == OP_POOL) {
        sv[j].idx.resize(out.size());
        maxpool_fwd(v[o.in[0]].data(), out.data(), sv[j].idx.data(), N, si.c, si.h, si.w, o.k,
                    o.stride, o.pad);
      } else if (o.type == OP_ADD) {
        sv[j].pre.resize(out.size());
        for (size_t i = 0; i < out.size(); ++i) sv[j].pre[i] = v[o.in[0]][i] + v[o.in[1]][i];
        act_fwd(sv[j].pre.data(), out.data(), out.size(), o.act);
        rnd(out);
      } else {
        const std::vector<R> p = probs(b, (int)j);
        for (int k = 0; k < o.nin; ++k)
          for (size_t i = 0; i < out.size(); ++i) out[i] += p[k] * v[o.in[k]][i];
        rnd(out);
      }
    }
  }

  // Diagnostic, not part of the step: how close the last forward of block b came to a point
  // where its gradient is discontinuous - the smallest |pre| (and |pre - 6| for ReLU6) over
  // rectified elements, and the smallest winner-to-runner-up gap over max-pool windows whose
  // winner is positive.  A comparison at finite precision is meaningless below this margin.
  double kink_margin(int b) override {
    const BlockD& blk = d.net[1][b];
    double m = std::numeric_limits<double>::infinity();
    for (size_t j = 0; j < blk.ops.size(); ++j) {
      const OpD& o = blk.ops[j];
      if ((o.type == OP_CBA || o.type == OP_ADD) && o.act != ACT_NONE) {
        const Saved& sv = saved[b][j];
        // a residual sum is not normalised: measure its distance from the kink in units of its rms
        double unit = 1.0;
        if (o.type == OP_ADD) {
          double ss = 0.0;
          for (R p : sv.pre) ss += (double)p * (double)p;
          unit = std::max(1.0, std::sqrt(ss / (double)sv.pre.size()));
        }
        for (size_t i = 0; i < sv.pre.size(); ++i) {
          // a channel fed by an all-zero input is zero in any arithmetic: not a coincidence
          if (o.type == OP_CBA && sv.conv[i] == R(0) && sv.pre[i] == R(0)) continue;
          const double p = (double)sv.pre[i];
          m = std::min(m, std::fabs(p) / unit);
          if (o.act == ACT_RELU6) m = std::min(m, std::fabs(p - 6.0) / unit);
        }
      } else if (o.type == OP_POOL) {
        const Shape si = blk.shapes[o.in[0]], so = blk.shapes[j + 1];
        const std::vector<R>& x = val[b][o.in[0]];
        for (int nc = 0; nc < N * si.c; ++nc)
          for (int p = 0; p < so.h; ++p)
            for (int q = 0; q < so.w; ++q) {
              double best = -std::numeric_limits<double>::infinity(), second = best;
              for (int r = 0; r < o.k; ++r)
                for (int t = 0; t < o.k; ++t) {
                  const int h = p * o.stride + r - o.pad, w = q * o.stride + t - o.pad;
                  if (h < 0 || h >= si.h || w < 0 || w >= si.w) continue;
                  const double v = (double)x[((size_t)nc * si.h + h) * si.w + w];
                  if (v > best) { second = best; best = v; } else if (v > second) second = v;
                }
              if (best > 0 && std::isfinite(second)) m = std::min(m, best - second);
            }
      }
    }
    return m;
  }

  void update_running_stats(int b) {
    const BlockD& blk = d.net[1][b];
    for (size_t j = 0; j < blk.ops.size(); ++j) {
      if (blk.ops[j].type != OP_CBA) continue;
      const Shape so = blk.shapes[j + 1];
      const R m = (R)N * (R)(so.h * so.w);
      Cba<R>& c = par[1][b][j];
      for (int k = 0; k < so.c; ++k) {
        c.p[3][k] = (R(1) - rho) * c.p[3][k] + rho * saved[b][j].mean[k];
        c.p[4][k] = (R(1) - rho) * c.p[4][k] + rho * saved[b][j].var[k] * m / (m - R(1));
      }
    }
  }

  // gradient of loss_i w.r.t. every parameter of S_i; dval[0] (w.r.t. A_{i-1}) is never formed.
  // arch: the architecture round - gradients of alpha instead of those of the frozen weights
  void student_backward(int b, std::vector<R>& dout, bool arch = false) {
    const BlockD& blk = d.net[1][b];
    auto& v = val[b];
    std::vector<std::vector<R>> dv(blk.ops.size() + 1);
    dv.back() = std::move(dout);
    auto accumulate = [&](int id, const std::vector<R>& gsrc) {
      if (id == 0) return;  // the teacher activation is a constant
      if (dv[id].empty()) dv[id] = gsrc;
      else for (size_t i = 0; i < gsrc.size(); ++i) dv[id][i] += gsrc[i];
      rnd(dv[id]);  // a stored activation gradient
    };
    for (int j = (int)blk.ops.size() - 1; j >= 0; --j) {
      const OpD& o = blk.ops[j];
      const Shape si = blk.shapes[o.in[0]], so = blk.shapes[j + 1];
      std::vector<R>& dy = dv[j + 1];
      if (dy.empty()) continue;  // value feeds nothing on the way to the loss
      if (o.type == OP_CBA) {
        Cba<R>& c = par[1][b][j];
        Saved& s = saved[b][j];
        std::vector<R> dpre(dy.size()), dconv(dy.size());
        act_bwd(dy.data(), s.pre.data(), dpre.data(), dy.size(), o.act);
        bn_train_bwd(dpre.data(), s.conv.data(), c.p[1].data(), s.mean.data(), s.var.data(),
                     dconv.data(), c.g[1].data(), c.g[2].data(), N, so.c, so.h * so.w, eps);
        rnd(dconv);
        if (!arch)
          conv_wgrad(dconv.data(), v[o.in[0]].data(), c.g[0].data(), N, si.c, si.h, si.w, so.c, o.k,
                     o.stride, o.pad, o.groups);
        if (o.in[0] != 0) {
          std::vector<R> dx((size_t)N * si.numel());
          const std::vector<R> w = stored(c.p[0]);
          conv_dgrad(dconv.data(), w.data(), dx.data(), N, si.c, si.h, si.w, so.c, o.k,
                     o.stride, o.pad, o.groups);
          accumulate(o.in[0], dx);
        }
      } else if (o.type == OP_POOL) {
        if (o.in[0] != 0) {
          std::vector<R> dx((size_t)N * si.numel());
          maxpool_bwd(dy.data(), saved[b][j].idx.data(), dx.data(), N, si.c, si.h, si.w, so.h, so.w);
          accumulate(o.in[0], dx);
        }
      } else if (o.type == OP_ADD) {
        std::vector<R> dpre(dy.size());
        act_bwd(dy.data(), saved[b][j].pre.data(), dpre.data(), dy.size(), o.act);
        accumulate(o.in[0], dpre);
        accumulate(o.in[1], dpre);
      } else {
        const std::vector<R> p = probs(b, j);
        if (arch) {
          std::vector<const R*> ys(o.nin);
          for (int k = 0; k < o.nin; ++k) ys[k] = v[o.in[k]].data();
          mix_alpha_grad(dy.data(), ys.data(), p.data(), o.nin, dy.size(), alpha_g[b][j].data());
        }
        for (int k = 0; k < o.nin; ++k) {
          std::vector<R> g(dy.size());
          for (size_t i = 0; i < dy.size(); ++i) g[i] = p[k] * dy[i];
          accumulate(o.in[k], g);
        }
      }
      std::vector<R>().swap(dy);
    }
  }

  // mode 0: loss only (no state change); 1: loss + gradients; 2: full step;
  // 3: architecture round, loss + gradients of alpha; 4: architecture round, full step
  R student_step_r(int i, const std::vector<R>& a_prev, const std::vector<R>& a_i, R lr, int mode) {
    const int b = i - 1;
    const bool arch = mode >= 3;
    if (arch) define_alpha(b);
    student_forward(b, a_prev);
    const std::vector<R>& s = val[b].back();
    std::vector<R> ds(mode ? s.size() : 0);
    const R loss = mse(s.data(), a_i.data(), mode ? ds.data() : nullptr, s.size());
    if (mode == 0) return loss;
    rnd(ds);
    student_backward(b, ds, arch);
    if (mode == 4) {
      update_running_stats(b);
      for (size_t j = 0; j < alpha[b].size(); ++j)
        if (!alpha[b][j].empty())
          sgd(alpha[b][j].data(), alpha_v[b][j].data(), alpha_g[b][j].data(), alpha[b][j].size(), lr, mu);
    }
    if (mode == 2) {
      update_running_stats(b);
      for (Cba<R>& c : par[1][b])
        for (int t = 0; t < 3; ++t)
          if (!c.p[t].empty()) sgd(c.p[t].data(), c.v[t].data(), c.g[t].data(), c.p[t].size(), lr, mu);
    }
    return loss;
  }
  double student_step(int i, const double* a_prev, const double* a_i, double lr, int mode) override {
    std::vector<R> ap((size_t)N * d.act[i - 1].numel()), ai((size_t)N * d.act[i].numel());
    for (size_t k = 0; k < ap.size(); ++k) ap[k] = (R)a_prev[k];
    for (size_t k = 0; k < ai.size(); ++k) ai[k] = (R)a_i[k];
    return (double)student_step_r(i, ap, ai, (R)lr, mode);
  }

  // teacher once, activations kept; every student block trained on (A_{i-1}, A_i)
  void relay_step(const double* x, double lr, double* losses) override {
    teacher_relay(x);
    for (int i = 1; i <= d.B; ++i) losses[i - 1] = (double)student_step_r(i, A[i - 1], A[i], (R)lr, 2);
  }
  // the architecture round of every block on relayed activations
  void relay_arch_step(const double* x, double lr, double* losses) override {
    teacher_relay(x);
    for (int i = 1; i <= d.B; ++i) losses[i - 1] = (double)student_step_r(i, A[i - 1], A[i], (R)lr, 4);
  }
  // block by block, teacher re-run from the input each time (Sec. II-B baseline)
  void redundant_step(const double* x, double lr, double* losses) override {
    for (int i = 1; i <= d.B; ++i) {
      std::vector<R> a_prev = teacher_from_start(x, i - 1);
      std::vector<R> a_i = teacher_block(i - 1, a_prev);
      losses[i - 1] = (double)student_step_r(i, a_prev, a_i, (R)lr, 2);
    }
  }
  long value_numel(int b, int v) override {
    if (b < 0 || b >= d.B || v < 0 || v >= (int)val[b].size()) return -1;
    return (long)val[b][v].size();
  }
  void get_value(int b, int v, double* out) override {
    for (size_t k = 0; k < val[b][v].size(); ++k) out[k] = (double)val[b][v][k];
  }
  // read-only view of what the last forward of student block b kept for op j.  which 0: the
  // convolution's output, 1: the normalised tensor before the activation (the sum, for an add),
  // 2: batch mean, 3: biased batch variance
  const std::vector<R>* saved_ref(int b, int j, int which) {
    if (b < 0 || b >= d.B || j < 0 || j >= (int)saved[b].size()) return nullptr;
    const Saved& s = saved[b][j];
    return which == 0 ? &s.conv : which == 1 ? &s.pre : which == 2 ? &s.mean : which == 3 ? &s.var : nullptr;
  }
  long saved_numel(int b, int j, int which) override {
    const std::vector<R>* t = saved_ref(b, j, which);
    return t ? (long)t->size() : -1;
  }
  void get_saved(int b, int j, int which, double* out) override {
    const std::vector<R>* t = saved_ref(b, j, which);
    if (t) for (size_t k = 0; k < t->size(); ++k) out[k] = (double)(*t)[k];
  }
};

}  // namespace

// ---------------------------------------------------------------------------
// C interface for the ctypes wrapper (doubles at the boundary in both precisions)
// ---------------------------------------------------------------------------
extern "C" {

void* orc_create(const int32_t* words, int nwords, const double* pool, int npool, int batch,
                 int precision, double momentum, double eps, double rho, int storage) {
  Desc d;
  std::string err;
  if (!d.parse(words, nwords, pool, npool, err)) return nullptr;
  if (precision == 64) return new Net<double>(d, batch, momentum, eps, rho, storage);
  if (precision == 32) return new Net<float>(d, batch, momentum, eps, rho, storage);
  return nullptr;
}
void orc_destroy(void* h) { delete static_cast<NetBase*>(h); }
int orc_set_tensor(void* h, int kind, int net, int b, int j, int slot, const double* d, long n) {
  return static_cast<NetBase*>(h)->set_tensor(kind, net, b, j, slot, d, n);
}
int orc_get_tensor(void* h, int kind, int net, int b, int j, int slot, double* d, long n) {
  return static_cast<NetBase*>(h)->get_tensor(kind, net, b, j, slot, d, n);
}
void orc_teacher_relay(void* h, const double* x) { static_cast<NetBase*>(h)->teacher_relay(x); }
void orc_teacher_upto(void* h, const double* x, int i, double* out) {
  static_cast<NetBase*>(h)->teacher_upto(x, i, out);
}
long orc_act_numel(void* h, int i) { return static_cast<NetBase*>(h)->act_numel(i); }
void orc_get_act(void* h, int i, double* out) { static_cast<NetBase*>(h)->get_act(i, out); }
double orc_student_step(void* h, int i, const double* a_prev, const double* a_i, double lr, int mode) {
  return static_cast<NetBase*>(h)->student_step(i, a_prev, a_i, lr, mode);
}
void orc_relay_step(void* h, const double* x, double lr, double* losses) {
  static_cast<NetBase*>(h)->relay_step(x, lr, losses);
}
void orc_redundant_step(void* h, const double* x, double lr, double* losses) {
  static_cast<NetBase*>(h)->redundant_step(x, lr, losses);
}
void orc_relay_arch_step(void* h, const double* x, double lr, double* losses) {
  static_cast<NetBase*>(h)->relay_arch_step(x, lr, losses);
}
int orc_set_alpha(void* h, int b, int j, const double* a, int n) { return static_cast<NetBase*>(h)->set_alpha(b, j, a, n); }
int orc_get_alpha(void* h, int kind, int b, int j, double* out, int n) {
  return static_cast<NetBase*>(h)->get_alpha(kind, b, j, out, n);
}
double orc_kink_margin(void* h, int b) { return static_cast<NetBase*>(h)->kink_margin(b); }
long orc_value_numel(void* h, int b, int v) { return static_cast<NetBase*>(h)->value_numel(b, v); }
void orc_get_value(void* h, int b, int v, double* out) { static_cast<NetBase*>(h)->get_value(b, v, out); }
long orc_saved_numel(void* h, int b, int j, int which) { return static_cast<NetBase*>(h)->saved_numel(b, j, which); }
void orc_get_saved(void* h, int b, int j, int which, double* out) { static_cast<NetBase*>(h)->get_saved(b, j, which, out); }
// the storage rounding of the bf16 mode on its own, so that it can be pinned against a library conversion
void orc_round_bf16(const double* in, double* out, long n) {
  for (long i = 0; i < n; ++i) out[i] = round_bf16(in[i]);
}
int orc_num_threads() {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

// fp64 primitives, exported one by one so that each can be pinned on its own
void orc_conv_fwd(const double* x, const double* w, double* y, int N, int C, int H, int W, int K,
                  int k, int stride, int pad, int groups) {
  conv_fwd(x, w, y, N, C, H, W, K, k, stride, pad, groups);
}
void orc_conv_dgrad(const double* dy, const double* w, double* dx, int N, int C, int H, int W,
                    int K, int k, int stride, int pad, int groups) {
  conv_dgrad(dy, w, dx, N, C, H, W, K, k, stride, pad, groups);
}
void orc_conv_wgrad(const double* dy, const double* x, double* dw, int N, int C, int H, int W,
                    int K, int k, int stride, int pad, int groups) {
  conv_wgrad(dy, x, dw, N, C, H, W, K, k, stride, pad, groups);
}
void orc_bn_train_fwd(const double* x, const double* gamma, const double* beta, double* y,
                      double* mean, double* var, int N, int C, int HW, double eps) {
  bn_train_fwd(x, gamma, beta, y, mean, var, N, C, HW, eps);
}
void orc_bn_train_bwd(const double* dy, const double* x, const double* gamma, const double* mean,
                      const double* var, double* dx, double* dgamma, double* dbeta, int N, int C,
                      int HW, double eps) {
  bn_train_bwd(dy, x, gamma, mean, var, dx, dgamma, dbeta, N, C, HW, eps);
}
void orc_bn_eval(const double* x, const double* gamma, const double* beta, const double* rmean,
                 const double* rvar, double* y, int N, int C, int HW, double eps) {
  bn_eval(x, gamma, beta, rmean, rvar, y, N, C, HW, eps);
}
void orc_act_fwd(const double* x, double* y, long n, int act) { act_fwd(x, y, (size_t)n, act); }
void orc_act_bwd(const double* dy, const double* x, double* dx, long n, int act) {
  act_bwd(dy, x, dx, (size_t)n, act);
}
void orc_maxpool_fwd(const double* x, double* y, int32_t* idx, int N, int C, int H, int W, int k,
                     int stride, int pad) {
  maxpool_fwd(x, y, idx, N, C, H, W, k, stride, pad);
}
void orc_maxpool_bwd(const double* dy, const int32_t* idx, double* dx, int N, int C, int H, int W,
                     int P, int Q) {
  maxpool_bwd(dy, idx, dx, N, C, H, W, P, Q);
}
void orc_mix_alpha_grad(const double* dz, const double* ys, const double* p, int n, long numel, double* dalpha) {
  std::vector<const double*> y(n);
  for (int k = 0; k < n; ++k) y[k] = ys + (size_t)k * (size_t)numel;
  mix_alpha_grad(dz, y.data(), p, n, (size_t)numel, dalpha);
}
double orc_mse(const double* s, const double* t, double* ds, long M) { return mse(s, t, ds, (size_t)M); }
void orc_sgd(double* w, double* v, const double* g, long n, double lr, double mu) {
  sgd(w, v, g, (size_t)n, lr, mu);
}

}  // extern "C"
