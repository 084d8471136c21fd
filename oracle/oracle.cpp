// CPU ORACLE -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
//
// A plain, slow, direct-loop implementation of what one model partition computes in
// HyPar-Flow-style model-parallel training: the forward pass of the partition's layers on
// activations received from the previous partition, the back-propagation from the partial
// error received from the next partition (producing weight gradients and the partial error
// with respect to the partition's own input -- the paper's "grad layer" result, Section
// "Implementing Distributed Back-Propagation", Eq. 5-7), accumulation of weight gradients over
// the micro-batches of one batch ("Exploiting Pipeline Stages within Each Minibatch"; one
// synchronous update per batch, Section "Background", Data-Parallelism) and the optimizer
// step (apply_gradients, same section as Eq. 5-7).
//
// The method reaches exactly the result of ordinary back-propagation, so every function here is
// the textbook definition written out: no blocking, no im2col, no BLAS, no fusion.  Storage type
// T is float (the fp32 reference) or double (for finite-difference checks); every reduction
// accumulates in double, so the reference is not the noisy side of a comparison.
//
// Storage reading for the GPU's bf16 mode (the paper never states a precision): with storage = 1 every
// tensor that the bf16 mode keeps in memory as bfloat16 -- convolution operands (activations after
// BN+ReLU, weight copies, im2col columns of the stem), convolution outputs including the residual sum,
// and the gradient tensors flowing backward -- is rounded to the nearest-even bfloat16 at the point it
// is produced; statistics, parameters, weight gradients, the loss and all arithmetic in between stay
// in double.  This puts the ReLU decisions z > 0 on the same stored values on both sides of a parity
// test (a floating-point value deciding a boolean must be decided in the same precision).  With
// storage = 0 nothing is rounded: that is the plain reference.
//
// Only tests, the smoke check and the benchmark's cpu_baseline leg may call this library.  It
// shares no code with the HIP path.
//
// Pins (tests/test_oracle_*.py): finite differences for every gradient, 1x1 conv == matmul,
// delta-filter identity, stride-2 == subsampled stride-1, adjoint identities for dgrad/wgrad,
// BN moment identities, softmax-CE closed forms, the two-linear-layer closed form of Eq. 1-7,
// partition equivalence, micro-batch equivalence with frozen BN, accumulation and SGD closed
// forms.  Parity unpinned: anything tied to trained accuracy (needs the paper's dataset).
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <memory>
#include <string>
#include <vector>

namespace {

// Nearest-even rounding of a value to bfloat16 (8 exponent bits, 7 stored mantissa bits), returned
// in the storage type.  st == 0: identity.
template <class T>
inline T rnd(T v, int st) {
  if (!st) return v;
  float f = (float)v;
  uint32_t u;
  std::memcpy(&u, &f, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return v;   // NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  u &= 0xffff0000u;
  std::memcpy(&f, &u, 4);
  return (T)f;
}

template <class T>
std::vector<T> rounded_copy(const T* w, size_t n, int st) {
  std::vector<T> r(w, w + n);
  if (st) for (auto& v : r) v = rnd(v, st);
  return r;
}

// ------------------------------------------------------------------------------------------
// Convolution, NHWC activations, [R][S][Cin][Cout] weights, zero padding (R-1)/2, no bias.
// y[n,p,q,k] = sum_{r,s,c} x[n, p*st + r - pad, q*st + s - pad, c] * w[r,s,c,k]  (+ add[n,p,q,k])
// `add` (may be null, may alias y) is the shortcut of a residual block: the sum is formed before the
// result is stored.  bf: storage reading (weights are used, and y is stored, as bfloat16).
// ------------------------------------------------------------------------------------------
template <class T>
void conv_fwd(const T* x, const T* w_in, T* y, int n, int h, int wd, int cin, int cout, int R, int st,
              const T* add = nullptr, int bf = 0) {
  const std::vector<T> wq = rounded_copy(w_in, (size_t)R * R * cin * cout, bf);
  const T* w = wq.data();
  const int pad = (R - 1) / 2;
  const int ho = (h + 2 * pad - R) / st + 1, wo = (wd + 2 * pad - R) / st + 1;
#pragma omp parallel for collapse(2) schedule(static)
  for (int in = 0; in < n; ++in)
    for (int p = 0; p < ho; ++p) {
      std::vector<double> acc(cout);
      for (int q = 0; q < wo; ++q) {
        std::fill(acc.begin(), acc.end(), 0.0);
        for (int r = 0; r < R; ++r) {
          const int hi = p * st + r - pad;
          if (hi < 0 || hi >= h) continue;
          for (int s = 0; s < R; ++s) {
            const int wi = q * st + s - pad;
            if (wi < 0 || wi >= wd) continue;
            const T* xp = x + ((size_t)(in * h + hi) * wd + wi) * cin;
            const T* wp = w + (size_t)(r * R + s) * cin * cout;
            for (int c = 0; c < cin; ++c) {
              const double xv = xp[c];
              const T* wr = wp + (size_t)c * cout;
              for (int k = 0; k < cout; ++k) acc[k] += xv * (double)wr[k];
            }
          }
        }
        const size_t o = ((size_t)(in * ho + p) * wo + q) * cout;
        for (int k = 0; k < cout; ++k) y[o + k] = rnd((T)(acc[k] + (add ? (double)add[o + k] : 0.0)), bf);
      }
    }
}

// dx[n,h,w,c] = sum over (p,q,r,s,k) with p*st + r - pad == h and q*st + s - pad == w of
//               dy[n,p,q,k] * w[r,s,c,k]          (the adjoint of conv_fwd in x)
template <class T>
void conv_dgrad(const T* dy, const T* w_in, T* dx, int n, int h, int wd, int cin, int cout, int R, int st,
                const T* add = nullptr, int bf = 0) {
  const std::vector<T> wq = rounded_copy(w_in, (size_t)R * R * cin * cout, bf);
  const T* w = wq.data();
  const int pad = (R - 1) / 2;
  const int ho = (h + 2 * pad - R) / st + 1, wo = (wd + 2 * pad - R) / st + 1;
#pragma omp parallel for collapse(2) schedule(static)
  for (int in = 0; in < n; ++in)
    for (int hi = 0; hi < h; ++hi) {
      std::vector<double> acc(cin);
      for (int wi = 0; wi < wd; ++wi) {
        std::fill(acc.begin(), acc.end(), 0.0);
        for (int r = 0; r < R; ++r) {
          const int t = hi + pad - r;
          if (t < 0 || t % st != 0 || t / st >= ho) continue;
          const int p = t / st;
          for (int s = 0; s < R; ++s) {
            const int u = wi + pad - s;
            if (u < 0 || u % st != 0 || u / st >= wo) continue;
            const int q = u / st;
            const T* dyp = dy + ((size_t)(in * ho + p) * wo + q) * cout;
            const T* wp = w + (size_t)(r * R + s) * cin * cout;
            for (int c = 0; c < cin; ++c) {
              const T* wr = wp + (size_t)c * cout;
              double a = 0.0;
              for (int k = 0; k < cout; ++k) a += (double)dyp[k] * (double)wr[k];
              acc[c] += a;
            }
          }
        }
        const size_t o = ((size_t)(in * h + hi) * wd + wi) * cin;
        for (int c = 0; c < cin; ++c) dx[o + c] = rnd((T)(acc[c] + (add ? (double)add[o + c] : 0.0)), bf);
      }
    }
}

// dw[r,s,c,k] += sum_{n,p,q} x[n, p*st + r - pad, q*st + s - pad, c] * dy[n,p,q,k]
template <class T>
void conv_wgrad(const T* x, const T* dy, double* dw, int n, int h, int wd, int cin, int cout, int R, int st) {
  const int pad = (R - 1) / 2;
  const int ho = (h + 2 * pad - R) / st + 1, wo = (wd + 2 * pad - R) / st + 1;
#pragma omp parallel for collapse(2) schedule(static)
  for (int rs = 0; rs < R * R; ++rs)
    for (int c = 0; c < cin; ++c) {
      const int r = rs / R, s = rs % R;
      std::vector<double> acc(cout, 0.0);
      for (int in = 0; in < n; ++in)
        for (int p = 0; p < ho; ++p) {
          const int hi = p * st + r - pad;
          if (hi < 0 || hi >= h) continue;
          for (int q = 0; q < wo; ++q) {
            const int wi = q * st + s - pad;
            if (wi < 0 || wi >= wd) continue;
            const double xv = x[((size_t)(in * h + hi) * wd + wi) * cin + c];
            const T* dyp = dy + ((size_t)(in * ho + p) * wo + q) * cout;
            for (int k = 0; k < cout; ++k) acc[k] += xv * (double)dyp[k];
          }
        }
      double* o = dw + ((size_t)rs * cin + c) * cout;
      for (int k = 0; k < cout; ++k) o[k] += acc[k];
    }
}

// ------------------------------------------------------------------------------------------
// BatchNorm + ReLU over the M = b*H*W rows of one micro-batch, per channel.
// mode 0: mean = mean(x), var = mean((x-mean)^2) (biased); mode 1: frozen mean 0, var 1.
// xhat = (x-mean)/sqrt(var+eps); z = gamma*xhat + beta; a = max(z, 0).
// ------------------------------------------------------------------------------------------
// given_mean / given_var (both or neither): use these statistics instead (inference with running statistics).
template <class T>
void bn_relu_fwd(const T* x, const T* gamma, const T* beta, T* a, double* mean, double* invstd,
                 size_t M, int C, double eps, int mode, int bf = 0, const double* given_mean = nullptr,
                 const double* given_var = nullptr) {
#pragma omp parallel for schedule(static)
  for (int c = 0; c < C; ++c) {
    double mu = 0.0, var = 1.0;
    if (given_mean) {
      mu = given_mean[c]; var = given_var[c];
    } else if (mode == 0) {
      double s = 0.0;
      for (size_t m = 0; m < M; ++m) s += (double)x[m * C + c];
      mu = s / (double)M;
      double v = 0.0;
      for (size_t m = 0; m < M; ++m) { const double d = (double)x[m * C + c] - mu; v += d * d; }
      var = v / (double)M;
    }
    const double is = 1.0 / std::sqrt(var + eps);
    mean[c] = mu; invstd[c] = is;
    for (size_t m = 0; m < M; ++m) {
      const double z = (double)gamma[c] * (((double)x[m * C + c] - mu) * is) + (double)beta[c];
      a[m * C + c] = rnd((T)(z > 0.0 ? z : 0.0), bf);
    }
  }
}

// dz = da * [z > 0]; dbeta = sum dz; dgamma = sum dz*xhat;
// mode 0: dx = gamma*invstd * (dz - dbeta/M - xhat*dgamma/M); mode 1: dx = gamma*invstd*dz.
// `skip` (may be null) is the gradient arriving over an identity shortcut, added before storing.
// dgamma/dbeta are added into the accumulators.  The ReLU mask is recomputed from z as the
// forward pass computed it (same precision, same expression).
template <class T>
void bn_relu_bwd(const T* x, const T* da, const T* gamma, const T* beta, const double* mean,
                 const double* invstd, T* dx, double* dgamma, double* dbeta, size_t M, int C, int mode,
                 const T* skip = nullptr, int bf = 0) {
#pragma omp parallel for schedule(static)
  for (int c = 0; c < C; ++c) {
    const double mu = mean[c], is = invstd[c], g = gamma[c], bt = beta[c];
    double sb = 0.0, sg = 0.0;
    for (size_t m = 0; m < M; ++m) {
      const double xh = ((double)x[m * C + c] - mu) * is;
      const double z = g * xh + bt;
      const double dz = z > 0.0 ? (double)da[m * C + c] : 0.0;
      sb += dz; sg += dz * xh;
    }
    dbeta[c] += sb; dgamma[c] += sg;
    for (size_t m = 0; m < M; ++m) {
      const double xh = ((double)x[m * C + c] - mu) * is;
      const double z = g * xh + bt;
      const double dz = z > 0.0 ? (double)da[m * C + c] : 0.0;
      const double v = mode == 0 ? (dz - sb / (double)M - xh * sg / (double)M) : dz;
      dx[m * C + c] = rnd((T)(g * is * v + (skip ? (double)skip[m * C + c] : 0.0)), bf);
    }
  }
}

// ------------------------------------------------------------------------------------------
// Head after its BN+ReLU: global average pool, FC with bias, softmax cross-entropy.
// g[n,c] = mean_{h,w} a[n,h,w,c]; logits = g*Wfc + bfc; loss_n = -log softmax(logits_n)[y_n];
// returns sum_n loss_n / divisor and dlogits = (softmax - onehot)/divisor.
// ------------------------------------------------------------------------------------------
template <class T>
double head_fwd(const T* a, const T* wfc, const T* bfc, const int32_t* labels, T* g, T* dlogits,
                int n, int hw, int C, int classes, double divisor) {
  double loss = 0.0;
  for (int in = 0; in < n; ++in) {
    for (int c = 0; c < C; ++c) {
      double s = 0.0;
      for (int i = 0; i < hw; ++i) s += (double)a[((size_t)in * hw + i) * C + c];
      g[(size_t)in * C + c] = (T)(s / (double)hw);
    }
    std::vector<double> lg(classes);
    double mx = -1e300;
    for (int j = 0; j < classes; ++j) {
      double s = (double)bfc[j];
      for (int c = 0; c < C; ++c) s += (double)g[(size_t)in * C + c] * (double)wfc[(size_t)c * classes + j];
      lg[j] = s; if (s > mx) mx = s;
    }
    double den = 0.0;
    for (int j = 0; j < classes; ++j) den += std::exp(lg[j] - mx);
    const int y = labels[in];
    loss += -(lg[y] - mx - std::log(den)) / divisor;
    for (int j = 0; j < classes; ++j)
      dlogits[(size_t)in * classes + j] = (T)((std::exp(lg[j] - mx) / den - (j == y ? 1.0 : 0.0)) / divisor);
  }
  return loss;
}

// dWfc += g^T dlogits; dbfc += sum_n dlogits; dg = dlogits * Wfc^T; da[n,h,w,c] = dg[n,c]/(H*W).
template <class T>
void head_bwd(const T* g, const T* dlogits, const T* wfc, double* dwfc, double* dbfc, T* da,
              int n, int hw, int C, int classes, int bf = 0) {
  for (int in = 0; in < n; ++in) {
    for (int j = 0; j < classes; ++j) dbfc[j] += (double)dlogits[(size_t)in * classes + j];
    for (int c = 0; c < C; ++c) {
      double dg = 0.0;
      for (int j = 0; j < classes; ++j) {
        const double d = dlogits[(size_t)in * classes + j];
        dwfc[(size_t)c * classes + j] += (double)g[(size_t)in * C + c] * d;
        dg += d * (double)wfc[(size_t)c * classes + j];
      }
      for (int i = 0; i < hw; ++i) da[((size_t)in * hw + i) * C + c] = rnd((T)(dg / (double)hw), bf);
    }
  }
}

// ------------------------------------------------------------------------------------------
// The layers of the paper's two other models (Section "Model-Parallelism on a Single Node": VGG-16 and the
// post-activation ResNet-110-v1), each the textbook definition.
// ------------------------------------------------------------------------------------------
// y = x + bias[c], followed by max(., 0) when relu.
template <class T>
void bias_act_fwd(const T* x, const T* bias, T* y, size_t M, int C, int relu, int bf = 0) {
#pragma omp parallel for schedule(static)
  for (size_t m = 0; m < M; ++m)
    for (int c = 0; c < C; ++c) {
      const double v = (double)x[m * C + c] + (double)bias[c];
      y[m * C + c] = rnd((T)(relu && !(v > 0.0) ? 0.0 : v), bf);
    }
}
// dz = dy * [y > 0] (relu) or dy; dbias += sum_m dz; dx = dz.
template <class T>
void bias_act_bwd(const T* y, const T* dy, T* dx, double* dbias, size_t M, int C, int relu, int bf = 0) {
#pragma omp parallel for schedule(static)
  for (int c = 0; c < C; ++c) {
    double s = 0.0;
    for (size_t m = 0; m < M; ++m) {
      const double dz = (!relu || (double)y[m * C + c] > 0.0) ? (double)dy[m * C + c] : 0.0;
      s += dz;
      dx[m * C + c] = rnd((T)dz, bf);
    }
    dbias[c] += s;
  }
}
// 2x2 max-pool, stride 2 (h, w even): y[n,p,q,c] = max over the window.
template <class T>
void maxpool2_fwd(const T* x, T* y, int n, int h, int w, int C) {
  const int ho = h / 2, wo = w / 2;
#pragma omp parallel for collapse(2) schedule(static)
  for (int in = 0; in < n; ++in)
    for (int p = 0; p < ho; ++p)
      for (int q = 0; q < wo; ++q)
        for (int c = 0; c < C; ++c) {
          T best = x[((size_t)(in * h + 2 * p) * w + 2 * q) * C + c];
          for (int r = 0; r < 2; ++r)
            for (int s = 0; s < 2; ++s) {
              const T v = x[((size_t)(in * h + 2 * p + r) * w + 2 * q + s) * C + c];
              if (v > best) best = v;
            }
          y[((size_t)(in * ho + p) * wo + q) * C + c] = best;
        }
}
// The gradient of a window goes to its maximum; among equal maxima to the first in row-major order.
template <class T>
void maxpool2_bwd(const T* x, const T* dy, T* dx, int n, int h, int w, int C) {
  const int ho = h / 2, wo = w / 2;
#pragma omp parallel for collapse(2) schedule(static)
  for (int in = 0; in < n; ++in)
    for (int p = 0; p < ho; ++p)
      for (int q = 0; q < wo; ++q)
        for (int c = 0; c < C; ++c) {
          int br = 0, bs = 0;
          T best = x[((size_t)(in * h + 2 * p) * w + 2 * q) * C + c];
          for (int r = 0; r < 2; ++r)
            for (int s = 0; s < 2; ++s) {
              const T v = x[((size_t)(in * h + 2 * p + r) * w + 2 * q + s) * C + c];
              if (v > best) { best = v; br = r; bs = s; }
            }
          for (int r = 0; r < 2; ++r)
            for (int s = 0; s < 2; ++s)
              dx[((size_t)(in * h + 2 * p + r) * w + 2 * q + s) * C + c] =
                  (r == br && s == bs) ? dy[((size_t)(in * ho + p) * wo + q) * C + c] : (T)0;
        }
}
// Post-activation residual join: y = max(gamma*xhat + beta + add, 0), statistics as in bn_relu_fwd.
template <class T>
void bn_add_relu_fwd(const T* x, const T* gamma, const T* beta, const T* add, T* y, double* mean, double* invstd,
                     size_t M, int C, double eps, int mode, int bf = 0, const double* given_mean = nullptr,
                     const double* given_var = nullptr) {
#pragma omp parallel for schedule(static)
  for (int c = 0; c < C; ++c) {
    double mu = 0.0, var = 1.0;
    if (given_mean) {
      mu = given_mean[c]; var = given_var[c];
    } else if (mode == 0) {
      double s = 0.0;
      for (size_t m = 0; m < M; ++m) s += (double)x[m * C + c];
      mu = s / (double)M;
      double v = 0.0;
      for (size_t m = 0; m < M; ++m) { const double d = (double)x[m * C + c] - mu; v += d * d; }
      var = v / (double)M;
    }
    const double is = 1.0 / std::sqrt(var + eps);
    mean[c] = mu; invstd[c] = is;
    for (size_t m = 0; m < M; ++m) {
      const double z = (double)gamma[c] * (((double)x[m * C + c] - mu) * is) + (double)beta[c] + (double)add[m * C + c];
      y[m * C + c] = rnd((T)(z > 0.0 ? z : 0.0), bf);
    }
  }
}
// dz = dy * [y > 0]; dadd = dz; dbeta += sum dz; dgamma += sum dz*xhat;
// mode 0: dx = gamma*invstd*(dz - dbeta/M - xhat*dgamma/M); mode 1: dx = gamma*invstd*dz.
template <class T>
void bn_add_relu_bwd(const T* x, const T* y, const T* dy, const T* gamma, const double* mean, const double* invstd,
                     T* dx, T* dadd, double* dgamma, double* dbeta, size_t M, int C, int mode, int bf = 0) {
#pragma omp parallel for schedule(static)
  for (int c = 0; c < C; ++c) {
    const double mu = mean[c], is = invstd[c], g = gamma[c];
    double sb = 0.0, sg = 0.0;
    for (size_t m = 0; m < M; ++m) {
      const double dz = (double)y[m * C + c] > 0.0 ? (double)dy[m * C + c] : 0.0;
      sb += dz; sg += dz * (((double)x[m * C + c] - mu) * is);
    }
    dbeta[c] += sb; dgamma[c] += sg;
    for (size_t m = 0; m < M; ++m) {
      const double dz = (double)y[m * C + c] > 0.0 ? (double)dy[m * C + c] : 0.0;
      const double xh = ((double)x[m * C + c] - mu) * is;
      const double v = mode == 0 ? (dz - sb / (double)M - xh * sg / (double)M) : dz;
      dx[m * C + c] = rnd((T)(g * is * v), bf);
      dadd[m * C + c] = rnd((T)dz, bf);
    }
  }
}

// ------------------------------------------------------------------------------------------
// The partition: stem? + residual blocks + head?, canonical flat parameter order
//   stem W; per block bn1.g, bn1.b, W1, bn2.g, bn2.b, W2, [bn3.g, bn3.b, W3], [Wproj];
//   head bn.g, bn.b, Wfc, bfc.
// ------------------------------------------------------------------------------------------
struct BlockDesc { int kind, c_in, c_mid, c_out, stride; };

struct Desc {
  int in_h, in_w, in_c, has_stem, stem_c_out, n_blocks, has_head, num_classes;
  int microbatch, num_microbatches, loss_divisor, bn_mode;
  int storage = 0;   // 0: nothing rounded; 1: stored tensors and conv weight operands are bfloat16
  // Cuts at layer granularity (Section "Special Handling for Non-consecutive Models"): the partition holds
  // convolutions [first_from, nconv) of its first block and [0, last_to) of its last block (0 = the whole block;
  // a BatchNorm+ReLU goes with the convolution it feeds, the projection with convolution 0, the residual add
  // with the last convolution).  A block cut this way sends its shortcut value (x, or the projection of
  // relu(bn1(x))) straight from the partition that holds its start to the one that holds its end.
  int first_from = 0, last_to = 0;
  int head_bn = 1;   // the head starts with BatchNorm + relu; 0: global average pool - FC only (ResNet-v1, VGG)
  double bn_eps;
  std::vector<BlockDesc> blocks;
};
// Unit kinds: 0 / 1 pre-activation basic / bottleneck block; 2 post-activation basic block (ResNet-v1);
// 3 conv3x3 + bias + relu (+ 2x2 max-pool iff stride == 2); 4 flatten - dense + bias (+ relu iff c_mid != 0);
// 5 BatchNorm + relu; 6 bias + relu.
enum { K_BASIC = 0, K_BOTTLENECK = 1, K_POSTACT = 2, K_CONV_RELU = 3, K_DENSE = 4, K_BN_RELU = 5, K_BIAS_RELU = 6 };

struct ConvP { size_t w; int cin, cout, R, st; };
struct BnP { size_t g, b; int c; size_t run = 0; /* running mean at run, running variance at run + c */ };
struct BlockP {
  BlockDesc d; int h_in, w_in, h_out, w_out; bool proj;
  BnP bn[3]; ConvP cv[3]; ConvP pj; int nconv;
  int j0, j1;   // convolutions [j0, j1) of the block belong to this partition
  size_t bias = 0;   // kinds 3, 4, 6
};

template <class T>
struct BnSave { std::vector<T> x; std::vector<double> mean, invstd; };

template <class T>
struct BlockStash {
  BnSave<T> bn[3]; std::vector<T> a[3];
  std::vector<T> x, y, y0;   // kinds 2 ... 6: unit input, output (after the relu), output before the pool
};

template <class T>
struct MbStash {
  std::vector<T> stem_in;
  std::vector<T> skip_in;   // shortcut value received for a first block that starts after its convolution 0
  std::vector<BlockStash<T>> blk;
  BnSave<T> head_bn; std::vector<T> head_a, g, dlogits;
  bool fwd_done = false, bwd_done = false;
};

enum { OK = 0, E_INVAL = 1, E_STATE = 2 };

template <class T>
struct Partition {
  Desc d;
  std::vector<T> params, momentum;
  std::vector<double> grad;
  std::vector<BlockP> bp;
  size_t stem_w = 0; BnP head_bn{}; size_t wfc = 0, bfc = 0;
  int out_h, out_w, out_c, c0;
  std::vector<MbStash<T>> st;
  int n_bwd_done = 0;
  // Running statistics of every BatchNorm held here, in model order: mean[c] then variance[c]; start at 0 / 1.
  // A training forward with momentum < 1 moves them towards the statistics of its micro-batch (biased variance):
  // r <- bn_momentum*r + (1-bn_momentum)*batch.  The paper trains Keras models; it says nothing about these buffers
  // beyond using the framework's layers, so this is the framework's moving-average rule.
  std::vector<double> running;
  double bn_momentum = 1.0;   // 1: never updated

  size_t n_running = 0;
  size_t plan() {
    size_t off = 0;
    int h = d.in_h, w = d.in_w, c = d.in_c;
    if (d.has_stem) { stem_w = off; off += (size_t)9 * d.in_c * d.stem_c_out; c = d.stem_c_out; }
    c0 = c;
    for (size_t bi = 0; bi < d.blocks.size(); ++bi) {
      const BlockDesc& b = d.blocks[bi];
      BlockP p{}; p.d = b;
      if (b.kind >= K_POSTACT) {   // the other models' units: no cuts inside them
        auto bn2 = [&](int ch) { BnP r{off, off + (size_t)ch, ch, n_running}; off += 2 * (size_t)ch; n_running += 2 * (size_t)ch; return r; };
        auto cv2 = [&](int ci, int co, int R, int s) { ConvP r{off, ci, co, R, s}; off += (size_t)R * R * ci * co; return r; };
        p.h_in = h; p.w_in = w; p.j0 = 0;
        if (b.kind == K_POSTACT) {
          p.nconv = 2; p.h_out = h / b.stride; p.w_out = w / b.stride;
          p.proj = (b.stride != 1 || b.c_in != b.c_out);
          p.cv[0] = cv2(b.c_in, b.c_mid, 3, b.stride); p.bn[0] = bn2(b.c_mid);
          p.cv[1] = cv2(b.c_mid, b.c_out, 3, 1);       p.bn[1] = bn2(b.c_out);
          if (p.proj) p.pj = cv2(b.c_in, b.c_out, 1, b.stride);
        } else if (b.kind == K_CONV_RELU) {
          p.nconv = 1; p.h_out = h / b.stride; p.w_out = w / b.stride;
          p.cv[0] = cv2(b.c_in, b.c_out, 3, 1); p.bias = off; off += b.c_out;
        } else if (b.kind == K_DENSE) {
          p.nconv = 1; p.h_out = 1; p.w_out = 1;
          p.cv[0] = cv2(h * w * b.c_in, b.c_out, 1, 1); p.bias = off; off += b.c_out;
        } else if (b.kind == K_BN_RELU) {
          p.nconv = 0; p.h_out = h; p.w_out = w; p.bn[0] = bn2(b.c_in);
        } else {
          p.nconv = 0; p.h_out = h; p.w_out = w; p.bias = off; off += b.c_in;
        }
        p.j1 = p.nconv;
        bp.push_back(p);
        h = p.h_out; w = p.w_out; c = b.c_out;
        continue;
      }
      p.nconv = b.kind == 0 ? 2 : 3;
      p.j0 = (bi == 0) ? d.first_from : 0;
      p.j1 = (bi + 1 == d.blocks.size() && d.last_to > 0) ? d.last_to : p.nconv;
      if (p.j0 == 0) { p.h_in = h; p.w_in = w; p.h_out = h / b.stride; p.w_out = w / b.stride; }
      else { p.h_in = h * b.stride; p.w_in = w * b.stride; p.h_out = h; p.w_out = w; }   // the input is already at the block's output size
      p.proj = (b.stride != 1 || b.c_in != b.c_out);
      auto bn = [&](int ch) { BnP r{off, off + (size_t)ch, ch, n_running}; off += 2 * (size_t)ch; n_running += 2 * (size_t)ch; return r; };
      auto cv = [&](int ci, int co, int R, int s) { ConvP r{off, ci, co, R, s}; off += (size_t)R * R * ci * co; return r; };
      const int cin[3] = {b.c_in, b.c_mid, b.c_mid};
      const int cout[3] = {b.c_mid, b.kind == 0 ? b.c_out : b.c_mid, b.c_out};
      const int R[3] = {b.kind == 0 ? 3 : 1, 3, 1};
      for (int j = 0; j < p.nconv; ++j) {
        const ConvP shape{0, cin[j], cout[j], R[j], j == 0 ? b.stride : 1};
        p.cv[j] = shape; p.bn[j] = BnP{0, 0, cin[j]};
        if (j >= p.j0 && j < p.j1) {     // parameters only of the layers held here, in canonical order
          p.bn[j] = bn(cin[j]);
          p.cv[j] = cv(cin[j], cout[j], R[j], shape.st);
        }
      }
      if (p.proj) { p.pj = ConvP{0, b.c_in, b.c_out, 1, b.stride}; if (p.j0 == 0) p.pj = cv(b.c_in, b.c_out, 1, b.stride); }
      bp.push_back(p);
      h = p.h_out; w = p.w_out; c = p.j1 == p.nconv ? b.c_out : cout[p.j1 - 1];
    }
    out_h = h; out_w = w; out_c = c;
    if (d.has_head) {
      if (d.head_bn) { head_bn = BnP{off, off + (size_t)c, c, n_running}; off += 2 * (size_t)c; n_running += 2 * (size_t)c; }
      wfc = off; off += (size_t)c * d.num_classes;
      bfc = off; off += d.num_classes;
    }
    return off;
  }

  Partition(const Desc& dd, const T* host_params) : d(dd) {
    const size_t P = plan();
    params.assign(host_params, host_params + P);
    momentum.assign(P, (T)0);
    grad.assign(P, 0.0);
    st.resize(d.num_microbatches);
    running.assign(n_running, 0.0);
    auto init = [&](const BnP& b) { for (int c = 0; c < b.c; ++c) running[b.run + b.c + c] = 1.0; };
    for (auto& p : bp) {
      if (p.d.kind == K_BN_RELU) init(p.bn[0]);
      else if (p.d.kind <= K_POSTACT) for (int j = p.j0; j < p.j1; ++j) init(p.bn[j]);
    }
    if (d.has_head && d.head_bn) init(head_bn);
  }

  void update_running(const BnP& b, const double* mean, const double* invstd) {
    if (!(bn_momentum < 1.0) || d.bn_mode != 0) return;
    for (int c = 0; c < b.c; ++c) {
      const double var = 1.0 / (invstd[c] * invstd[c]) - d.bn_eps;
      running[b.run + c] = bn_momentum * running[b.run + c] + (1.0 - bn_momentum) * mean[c];
      running[b.run + b.c + c] = bn_momentum * running[b.run + b.c + c] + (1.0 - bn_momentum) * var;
    }
  }

  // skip_in / skip_out: shortcut value of a first block that starts, or a last block that ends, inside the block
  int forward(int mb, const T* act_in, const T* skip_in, const int32_t* labels, T* act_out, T* skip_out, double* loss_accum) {
    if (mb < 0 || mb >= d.num_microbatches) return E_INVAL;
    MbStash<T>& S = st[mb];
    if (S.fwd_done) return E_STATE;
    const int rc = forward_impl(S, false, act_in, skip_in, labels, act_out, skip_out, loss_accum);
    if (rc == OK) S.fwd_done = true;
    return rc;
  }

  // Inference: the same layers with every BatchNorm normalising by its running statistics; nothing is kept for
  // a backward pass.  `out`: logits [microbatch, classes] if the partition holds the head, else act_out.
  int infer(const T* act_in, const T* skip_in, T* out, T* skip_out) {
    MbStash<T> S;
    return forward_impl(S, true, act_in, skip_in, nullptr, out, skip_out, nullptr);
  }

  int forward_impl(MbStash<T>& S, bool inference, const T* act_in, const T* skip_in, const int32_t* labels, T* act_out,
                   T* skip_out, double* loss_accum) {
    const int b = d.microbatch, bf = d.storage;
    const T* P = params.data();
    std::vector<T> x;
    int h = d.in_h, w = d.in_w;
    if (d.has_stem) {
      S.stem_in.assign(act_in, act_in + (size_t)b * h * w * d.in_c);
      for (auto& v : S.stem_in) v = rnd(v, bf);          // the stem's operand tensor is stored
      x.resize((size_t)b * h * w * d.stem_c_out);
      conv_fwd(S.stem_in.data(), P + stem_w, x.data(), b, h, w, d.in_c, d.stem_c_out, 3, 1, (const T*)nullptr, bf);
    } else {
      x.assign(act_in, act_in + (size_t)b * h * w * d.in_c);
    }
    S.blk.assign(bp.size(), BlockStash<T>());
    for (size_t i = 0; i < bp.size(); ++i) {
      const BlockP& p = bp[i]; BlockStash<T>& B = S.blk[i];
      const size_t M_out = (size_t)b * p.h_out * p.w_out;
      auto bnrelu = [&](int j, std::vector<T>& in) {
        B.bn[j].x = in; B.bn[j].mean.resize(p.bn[j].c); B.bn[j].invstd.resize(p.bn[j].c);
        B.a[j].resize(in.size());
        const double* rm = inference ? running.data() + p.bn[j].run : nullptr;
        bn_relu_fwd(in.data(), P + p.bn[j].g, P + p.bn[j].b, B.a[j].data(), B.bn[j].mean.data(),
                    B.bn[j].invstd.data(), in.size() / p.bn[j].c, p.bn[j].c, d.bn_eps, d.bn_mode, bf, rm,
                    rm ? rm + p.bn[j].c : nullptr);
        if (!inference) update_running(p.bn[j], B.bn[j].mean.data(), B.bn[j].invstd.data());
      };
      if (p.d.kind >= K_POSTACT) {
        const size_t M_in = (size_t)b * p.h_in * p.w_in;
        const double* none_d = nullptr;
        auto run_of = [&](const BnP& q) { return inference ? running.data() + q.run : none_d; };
        B.x = x;
        if (p.d.kind == K_POSTACT) {
          // c1 = conv1(x); a1 = relu(bn1(c1)); c2 = conv2(a1); y = relu(bn2(c2) + shortcut)
          std::vector<T> c1(M_out * p.d.c_mid), c2(M_out * p.d.c_out), sc2, y(M_out * p.d.c_out);
          conv_fwd(x.data(), P + p.cv[0].w, c1.data(), b, p.h_in, p.w_in, p.cv[0].cin, p.cv[0].cout, 3, p.cv[0].st, (const T*)nullptr, bf);
          bnrelu(0, c1);
          conv_fwd(B.a[0].data(), P + p.cv[1].w, c2.data(), b, p.h_out, p.w_out, p.cv[1].cin, p.cv[1].cout, 3, 1, (const T*)nullptr, bf);
          if (p.proj) {
            sc2.resize(M_out * p.d.c_out);
            conv_fwd(x.data(), P + p.pj.w, sc2.data(), b, p.h_in, p.w_in, p.pj.cin, p.pj.cout, 1, p.pj.st, (const T*)nullptr, bf);
          } else {
            sc2 = x;
          }
          B.bn[1].x = c2; B.bn[1].mean.resize(p.bn[1].c); B.bn[1].invstd.resize(p.bn[1].c);
          const double* rm = run_of(p.bn[1]);
          bn_add_relu_fwd(c2.data(), P + p.bn[1].g, P + p.bn[1].b, sc2.data(), y.data(), B.bn[1].mean.data(), B.bn[1].invstd.data(),
                          M_out, p.bn[1].c, d.bn_eps, d.bn_mode, bf, rm, rm ? rm + p.bn[1].c : nullptr);
          if (!inference) update_running(p.bn[1], B.bn[1].mean.data(), B.bn[1].invstd.data());
          B.y = y;
          x.swap(y);
        } else if (p.d.kind == K_CONV_RELU) {
          std::vector<T> cc(M_in * p.d.c_out);
          conv_fwd(x.data(), P + p.cv[0].w, cc.data(), b, p.h_in, p.w_in, p.cv[0].cin, p.cv[0].cout, 3, 1, (const T*)nullptr, bf);
          B.y0.resize(cc.size());
          bias_act_fwd(cc.data(), P + p.bias, B.y0.data(), M_in, p.d.c_out, 1, bf);
          if (p.d.stride == 2) {
            std::vector<T> y(M_out * p.d.c_out);
            maxpool2_fwd(B.y0.data(), y.data(), b, p.h_in, p.w_in, p.d.c_out);
            x.swap(y);
          } else {
            x = B.y0;
          }
        } else if (p.d.kind == K_DENSE) {
          std::vector<T> cc((size_t)b * p.d.c_out);
          conv_fwd(x.data(), P + p.cv[0].w, cc.data(), b, 1, 1, p.cv[0].cin, p.cv[0].cout, 1, 1, (const T*)nullptr, bf);
          B.y0.resize(cc.size());
          bias_act_fwd(cc.data(), P + p.bias, B.y0.data(), (size_t)b, p.d.c_out, p.d.c_mid != 0, bf);
          x = B.y0;
        } else if (p.d.kind == K_BN_RELU) {
          bnrelu(0, x);
          x = B.a[0];
        } else {
          B.y0.resize(x.size());
          bias_act_fwd(x.data(), P + p.bias, B.y0.data(), M_in, p.d.c_in, 1, bf);
          x = B.y0;
        }
        continue;
      }
      std::vector<T> sc;                                   // shortcut: x, or the 1x1 projection of a
      std::vector<T> r;
      if (p.j0 == 0) {
        bnrelu(0, x);                                      // a = relu(bn1(x))
        if (p.proj) {
          sc.resize(M_out * p.d.c_out);
          conv_fwd(B.a[0].data(), P + p.pj.w, sc.data(), b, p.h_in, p.w_in, p.pj.cin, p.pj.cout, 1, p.pj.st,
                   (const T*)nullptr, bf);
        } else {
          sc = x;
        }
      } else {                                             // x is the output of convolution j0-1
        r = x;
        if (p.j1 == p.nconv) {
          if (!skip_in) return E_INVAL;
          S.skip_in.assign(skip_in, skip_in + M_out * p.d.c_out);
          for (auto& v : S.skip_in) v = rnd(v, bf);
          sc = S.skip_in;
        }
      }
      for (int j = p.j0; j < p.j1; ++j) {
        const bool last = (j == p.nconv - 1);
        if (j > 0) bnrelu(j, r);
        std::vector<T> r2(M_out * p.cv[j].cout);
        conv_fwd(B.a[j].data(), P + p.cv[j].w, r2.data(), b, j == 0 ? p.h_in : p.h_out, j == 0 ? p.w_in : p.w_out,
                 p.cv[j].cin, p.cv[j].cout, p.cv[j].R, p.cv[j].st, last ? sc.data() : (const T*)nullptr, bf);
        r.swap(r2);                                        // after the last conv: y = shortcut + branch
      }
      if (p.j1 < p.nconv && p.j0 == 0) {                   // the block ends elsewhere: its shortcut value leaves too
        if (!skip_out) return E_INVAL;
        std::memcpy(skip_out, sc.data(), sc.size() * sizeof(T));
      }
      x.swap(r);
    }
    if (d.has_head) {
      const int C = out_c, hw = out_h * out_w;
      if (d.head_bn) {
        S.head_bn.x = x; S.head_bn.mean.resize(C); S.head_bn.invstd.resize(C);
        S.head_a.resize(x.size());
        const double* rm = inference ? running.data() + head_bn.run : nullptr;
        bn_relu_fwd(x.data(), P + head_bn.g, P + head_bn.b, S.head_a.data(), S.head_bn.mean.data(),
                    S.head_bn.invstd.data(), (size_t)b * hw, C, d.bn_eps, d.bn_mode, bf, rm, rm ? rm + C : nullptr);
        if (!inference) update_running(head_bn, S.head_bn.mean.data(), S.head_bn.invstd.data());
      } else {
        S.head_a = x;   // pool - FC directly on the last unit's output
      }
      S.g.resize((size_t)b * C); S.dlogits.resize((size_t)b * d.num_classes);
      if (inference) {   // logits = mean_{h,w}(a) * Wfc + bfc
        if (!act_out) return E_INVAL;
        for (int n = 0; n < b; ++n)
          for (int j = 0; j < d.num_classes; ++j) {
            double sum = (double)P[bfc + j];
            for (int c = 0; c < C; ++c) {
              double g = 0.0;
              for (int i = 0; i < hw; ++i) g += (double)S.head_a[((size_t)n * hw + i) * C + c];
              sum += (double)(T)(g / (double)hw) * (double)P[wfc + (size_t)c * d.num_classes + j];
            }
            act_out[(size_t)n * d.num_classes + j] = (T)sum;
          }
        return OK;
      }
      if (!labels) return E_INVAL;
      const double l = head_fwd(S.head_a.data(), P + wfc, P + bfc, labels, S.g.data(), S.dlogits.data(),
                                b, hw, C, d.num_classes, (double)d.loss_divisor);
      if (loss_accum) *loss_accum += l;
    } else {
      if (!act_out) return E_INVAL;
      std::memcpy(act_out, x.data(), x.size() * sizeof(T));
    }
    return OK;
  }

  // skip_err_in: gradient w.r.t. skip_out; skip_err_out: gradient w.r.t. skip_in
  int backward(int mb, const T* err_in, const T* skip_err_in, T* err_out, T* skip_err_out) {
    if (mb < 0 || mb >= d.num_microbatches) return E_INVAL;
    MbStash<T>& S = st[mb];
    if (!S.fwd_done || S.bwd_done) return E_STATE;
    const int b = d.microbatch, bf = d.storage;
    const T* P = params.data();
    double* G = grad.data();
    const T* none = nullptr;
    std::vector<T> dy;   // gradient w.r.t. the current unit's output
    if (d.has_head) {
      const int C = out_c, hw = out_h * out_w;
      std::vector<T> da((size_t)b * hw * C);
      head_bwd(S.g.data(), S.dlogits.data(), P + wfc, G + wfc, G + bfc, da.data(), b, hw, C, d.num_classes, bf);
      if (d.head_bn) {
        dy.resize(da.size());
        bn_relu_bwd(S.head_bn.x.data(), da.data(), P + head_bn.g, P + head_bn.b, S.head_bn.mean.data(),
                    S.head_bn.invstd.data(), dy.data(), G + head_bn.g, G + head_bn.b, (size_t)b * hw, C, d.bn_mode, none, bf);
      } else {
        dy.swap(da);
      }
    } else {
      if (!err_in) return E_INVAL;
      dy.assign(err_in, err_in + (size_t)b * out_h * out_w * out_c);
    }
    for (size_t ii = bp.size(); ii-- > 0;) {
      const BlockP& p = bp[ii]; BlockStash<T>& B = S.blk[ii];
      const size_t M_in = (size_t)b * p.h_in * p.w_in, M_out = (size_t)b * p.h_out * p.w_out;
      if (p.d.kind >= K_POSTACT) {
        std::vector<T> dx(B.x.size());
        if (p.d.kind == K_POSTACT) {
          // through the join: dz = dy*[y>0] goes to the shortcut as it is and through bn2 to c2
          std::vector<T> dc2(dy.size()), dz(dy.size());
          bn_add_relu_bwd(B.bn[1].x.data(), B.y.data(), dy.data(), P + p.bn[1].g, B.bn[1].mean.data(), B.bn[1].invstd.data(),
                          dc2.data(), dz.data(), G + p.bn[1].g, G + p.bn[1].b, M_out, p.bn[1].c, d.bn_mode, bf);
          conv_wgrad(B.a[0].data(), dc2.data(), G + p.cv[1].w, b, p.h_out, p.w_out, p.cv[1].cin, p.cv[1].cout, 3, 1);
          std::vector<T> da1(M_out * p.d.c_mid), dc1(M_out * p.d.c_mid);
          conv_dgrad(dc2.data(), P + p.cv[1].w, da1.data(), b, p.h_out, p.w_out, p.cv[1].cin, p.cv[1].cout, 3, 1, none, bf);
          bn_relu_bwd(B.bn[0].x.data(), da1.data(), P + p.bn[0].g, P + p.bn[0].b, B.bn[0].mean.data(), B.bn[0].invstd.data(),
                      dc1.data(), G + p.bn[0].g, G + p.bn[0].b, M_out, p.bn[0].c, d.bn_mode, none, bf);
          conv_wgrad(B.x.data(), dc1.data(), G + p.cv[0].w, b, p.h_in, p.w_in, p.cv[0].cin, p.cv[0].cout, 3, p.cv[0].st);
          if (p.proj) {
            conv_wgrad(B.x.data(), dz.data(), G + p.pj.w, b, p.h_in, p.w_in, p.pj.cin, p.pj.cout, 1, p.pj.st);
            std::vector<T> dsx(dx.size());
            conv_dgrad(dz.data(), P + p.pj.w, dsx.data(), b, p.h_in, p.w_in, p.pj.cin, p.pj.cout, 1, p.pj.st, none, bf);
            conv_dgrad(dc1.data(), P + p.cv[0].w, dx.data(), b, p.h_in, p.w_in, p.cv[0].cin, p.cv[0].cout, 3, p.cv[0].st, dsx.data(), bf);
          } else {
            conv_dgrad(dc1.data(), P + p.cv[0].w, dx.data(), b, p.h_in, p.w_in, p.cv[0].cin, p.cv[0].cout, 3, p.cv[0].st, dz.data(), bf);
          }
        } else if (p.d.kind == K_CONV_RELU) {
          std::vector<T> d0(B.y0.size()), dz(B.y0.size());
          if (p.d.stride == 2) maxpool2_bwd(B.y0.data(), dy.data(), d0.data(), b, p.h_in, p.w_in, p.d.c_out);
          else d0 = dy;
          bias_act_bwd(B.y0.data(), d0.data(), dz.data(), G + p.bias, M_in, p.d.c_out, 1, bf);
          conv_wgrad(B.x.data(), dz.data(), G + p.cv[0].w, b, p.h_in, p.w_in, p.cv[0].cin, p.cv[0].cout, 3, 1);
          conv_dgrad(dz.data(), P + p.cv[0].w, dx.data(), b, p.h_in, p.w_in, p.cv[0].cin, p.cv[0].cout, 3, 1, none, bf);
        } else if (p.d.kind == K_DENSE) {
          std::vector<T> dz(B.y0.size());
          bias_act_bwd(B.y0.data(), dy.data(), dz.data(), G + p.bias, (size_t)b, p.d.c_out, p.d.c_mid != 0, bf);
          conv_wgrad(B.x.data(), dz.data(), G + p.cv[0].w, b, 1, 1, p.cv[0].cin, p.cv[0].cout, 1, 1);
          conv_dgrad(dz.data(), P + p.cv[0].w, dx.data(), b, 1, 1, p.cv[0].cin, p.cv[0].cout, 1, 1, none, bf);
        } else if (p.d.kind == K_BN_RELU) {
          bn_relu_bwd(B.bn[0].x.data(), dy.data(), P + p.bn[0].g, P + p.bn[0].b, B.bn[0].mean.data(), B.bn[0].invstd.data(),
                      dx.data(), G + p.bn[0].g, G + p.bn[0].b, M_in, p.bn[0].c, d.bn_mode, none, bf);
        } else {
          bias_act_bwd(B.y0.data(), dy.data(), dx.data(), G + p.bias, M_in, p.d.c_in, 1, bf);
        }
        dy.swap(dx);
        continue;
      }
      // residual branch, last conv held here to first; dsc: gradient w.r.t. the shortcut value
      std::vector<T> dr = dy;
      std::vector<T> dsc;
      if (p.j1 == p.nconv) {
        dsc = dy;                                          // y = shortcut + branch
      } else if (p.j0 == 0) {
        if (!skip_err_in) return E_INVAL;
        dsc.assign(skip_err_in, skip_err_in + M_out * p.d.c_out);
        for (auto& v : dsc) v = rnd(v, bf);
      }
      for (int j = p.j1 - 1; j >= std::max(p.j0, 1); --j) {
        conv_wgrad(B.a[j].data(), dr.data(), G + p.cv[j].w, b, p.h_out, p.w_out, p.cv[j].cin, p.cv[j].cout, p.cv[j].R, 1);
        std::vector<T> da(M_out * p.cv[j].cin);
        conv_dgrad(dr.data(), P + p.cv[j].w, da.data(), b, p.h_out, p.w_out, p.cv[j].cin, p.cv[j].cout, p.cv[j].R, 1, none, bf);
        std::vector<T> dx(da.size());
        bn_relu_bwd(B.bn[j].x.data(), da.data(), P + p.bn[j].g, P + p.bn[j].b, B.bn[j].mean.data(),
                    B.bn[j].invstd.data(), dx.data(), G + p.bn[j].g, G + p.bn[j].b, M_out, p.bn[j].c, d.bn_mode, none, bf);
        dr.swap(dx);
      }
      if (p.j0 > 0) {                                      // dr is the gradient w.r.t. the partition's input
        if (p.j1 == p.nconv) {
          if (!skip_err_out) return E_INVAL;
          std::memcpy(skip_err_out, dsc.data(), dsc.size() * sizeof(T));
        }
        dy.swap(dr);
        continue;
      }
      conv_wgrad(B.a[0].data(), dr.data(), G + p.cv[0].w, b, p.h_in, p.w_in, p.cv[0].cin, p.cv[0].cout, p.cv[0].R, p.cv[0].st);
      std::vector<T> da(M_in * p.d.c_in);
      conv_dgrad(dr.data(), P + p.cv[0].w, da.data(), b, p.h_in, p.w_in, p.cv[0].cin, p.cv[0].cout, p.cv[0].R, p.cv[0].st, none, bf);
      if (p.proj) {   // a = relu(bn1(x)) feeds both the branch and the projection: their gradients add
        conv_wgrad(B.a[0].data(), dsc.data(), G + p.pj.w, b, p.h_in, p.w_in, p.pj.cin, p.pj.cout, 1, p.pj.st);
        conv_dgrad(dsc.data(), P + p.pj.w, da.data(), b, p.h_in, p.w_in, p.pj.cin, p.pj.cout, 1, p.pj.st, da.data(), bf);
      }
      std::vector<T> dx(da.size());  // identity shortcut: x also feeds the output directly, so dsc is added
      bn_relu_bwd(B.bn[0].x.data(), da.data(), P + p.bn[0].g, P + p.bn[0].b, B.bn[0].mean.data(),
                  B.bn[0].invstd.data(), dx.data(), G + p.bn[0].g, G + p.bn[0].b, M_in, p.bn[0].c, d.bn_mode,
                  p.proj ? none : dsc.data(), bf);
      dy.swap(dx);
    }
    if (d.has_stem) {
      conv_wgrad(S.stem_in.data(), dy.data(), G + stem_w, b, d.in_h, d.in_w, d.in_c, d.stem_c_out, 3, 1);
      if (err_out) conv_dgrad(dy.data(), P + stem_w, err_out, b, d.in_h, d.in_w, d.in_c, d.stem_c_out, 3, 1, none, bf);
    } else if (err_out) {
      std::memcpy(err_out, dy.data(), dy.size() * sizeof(T));
    }
    S.bwd_done = true; ++n_bwd_done;
    S.blk.clear(); S.blk.shrink_to_fit();
    return OK;
  }

  int grad_read(T* dst, size_t n) {
    if (n != grad.size()) return E_INVAL;
    for (size_t i = 0; i < n; ++i) dst[i] = (T)grad[i];
    return OK;
  }

  void new_step() {
    for (auto& s : st) { s.fwd_done = s.bwd_done = false; }
    n_bwd_done = 0;
  }

  // v <- mu*v + G; w <- w - lr*v; then the gradient buffer is cleared and a new step begins.
  int sgd_step(double lr, double mu) {
    if (n_bwd_done != d.num_microbatches) return E_STATE;
    for (size_t i = 0; i < params.size(); ++i) {
      const double v = mu * (double)momentum[i] + grad[i];
      momentum[i] = (T)v;
      params[i] = (T)((double)params[i] - lr * v);
      grad[i] = 0.0;
    }
    new_step();
    return OK;
  }
};

struct Handle {
  bool f64;
  std::unique_ptr<Partition<float>> pf;
  std::unique_ptr<Partition<double>> pd;
};

bool valid(const Desc& d) {
  if (d.in_h <= 0 || d.in_w <= 0 || d.in_c <= 0 || d.microbatch <= 0 || d.num_microbatches <= 0) return false;
  if (d.loss_divisor <= 0 || d.n_blocks < 0) return false;
  if (!d.has_stem && !d.has_head && d.n_blocks == 0) return false;
  int h = d.in_h, w = d.in_w, c = d.has_stem ? d.stem_c_out : d.in_c;
  if (d.has_stem && d.stem_c_out <= 0) return false;
  const int nb = (int)d.blocks.size();
  if (d.first_from < 0 || d.last_to < 0) return false;
  if (d.first_from > 0 && (nb == 0 || d.has_stem)) return false;
  if (d.last_to > 0 && (nb == 0 || d.has_head)) return false;
  for (int i = 0; i < nb; ++i) {
    const BlockDesc& b = d.blocks[i];
    if (b.kind >= K_POSTACT && b.kind <= K_BIAS_RELU) {
      if ((i == 0 && d.first_from > 0) || (i == nb - 1 && d.last_to > 0)) return false;   // no cuts inside these units
      if (b.c_in != c || b.c_out <= 0) return false;
      if (b.kind == K_POSTACT && (b.c_mid != b.c_out || (b.stride != 1 && b.stride != 2))) return false;
      if (b.kind == K_CONV_RELU && (b.stride != 1 && b.stride != 2)) return false;
      if ((b.kind == K_DENSE || b.kind == K_BN_RELU || b.kind == K_BIAS_RELU) && b.stride != 1) return false;
      if ((b.kind == K_BN_RELU || b.kind == K_BIAS_RELU) && b.c_in != b.c_out) return false;
      if (b.kind == K_DENSE) { h = 1; w = 1; }
      else { if (h % b.stride || w % b.stride) return false; h /= b.stride; w /= b.stride; }
      c = b.c_out;
      continue;
    }
    if (b.kind != 0 && b.kind != 1) return false;
    const int nconv = b.kind == 0 ? 2 : 3;
    const int j0 = i == 0 ? d.first_from : 0, j1 = (i == nb - 1 && d.last_to > 0) ? d.last_to : nconv;
    if (j0 >= j1 || j1 > nconv || (i == nb - 1 && d.last_to >= nconv)) return false;
    if (b.c_mid <= 0 || b.c_out <= 0) return false;
    if (b.c_in != c && j0 == 0) return false;
    if (j0 > 0 && c != b.c_mid) return false;      // the input is the output of convolution j0-1
    if (b.kind == 0 && b.c_mid != b.c_out) return false;
    if (b.stride != 1 && b.stride != 2) return false;
    if (j0 == 0) {
      if (h % b.stride || w % b.stride) return false;
      h /= b.stride; w /= b.stride;
    }
    c = j1 == nconv ? b.c_out : b.c_mid;
  }
  if (d.has_head && d.num_classes <= 0) return false;
  if (d.storage != 0 && d.storage != 1) return false;
  return true;
}

}  // namespace

extern "C" {

// desc_i: in_h,in_w,in_c,has_stem,stem_c_out,n_blocks,has_head,num_classes,microbatch,
//         num_microbatches,loss_divisor,bn_mode,storage,first_from,last_to,head_bn ; blocks: n_blocks x (kind,c_in,c_mid,c_out,stride)
void* oracle_partition_create(const int32_t* desc_i, double bn_eps, const int32_t* blocks,
                              const void* host_params, int is_f64) {
  Desc d;
  d.in_h = desc_i[0]; d.in_w = desc_i[1]; d.in_c = desc_i[2]; d.has_stem = desc_i[3];
  d.stem_c_out = desc_i[4]; d.n_blocks = desc_i[5]; d.has_head = desc_i[6]; d.num_classes = desc_i[7];
  d.microbatch = desc_i[8]; d.num_microbatches = desc_i[9]; d.loss_divisor = desc_i[10]; d.bn_mode = desc_i[11];
  d.storage = desc_i[12]; d.first_from = desc_i[13]; d.last_to = desc_i[14]; d.head_bn = desc_i[15];
  d.bn_eps = bn_eps;
  for (int i = 0; i < d.n_blocks; ++i)
    d.blocks.push_back(BlockDesc{blocks[5 * i], blocks[5 * i + 1], blocks[5 * i + 2], blocks[5 * i + 3], blocks[5 * i + 4]});
  if (!valid(d)) return nullptr;
  Handle* h = new Handle();
  h->f64 = is_f64 != 0;
  if (h->f64) h->pd.reset(new Partition<double>(d, (const double*)host_params));
  else h->pf.reset(new Partition<float>(d, (const float*)host_params));
  return h;
}

void oracle_partition_destroy(void* hp) { delete (Handle*)hp; }

size_t oracle_n_params(void* hp) {
  Handle* h = (Handle*)hp;
  return h->f64 ? h->pd->params.size() : h->pf->params.size();
}

int oracle_forward_microbatch_cut(void* hp, int mb, const void* act_in, const void* skip_in, const int32_t* labels,
                                  void* act_out, void* skip_out, double* loss_accum) {
  Handle* h = (Handle*)hp;
  return h->f64 ? h->pd->forward(mb, (const double*)act_in, (const double*)skip_in, labels, (double*)act_out, (double*)skip_out, loss_accum)
                : h->pf->forward(mb, (const float*)act_in, (const float*)skip_in, labels, (float*)act_out, (float*)skip_out, loss_accum);
}

int oracle_forward_microbatch(void* hp, int mb, const void* act_in, const int32_t* labels, void* act_out,
                              double* loss_accum) {
  return oracle_forward_microbatch_cut(hp, mb, act_in, nullptr, labels, act_out, nullptr, loss_accum);
}

int oracle_backward_microbatch_cut(void* hp, int mb, const void* err_in, const void* skip_err_in, void* err_out,
                                   void* skip_err_out) {
  Handle* h = (Handle*)hp;
  return h->f64 ? h->pd->backward(mb, (const double*)err_in, (const double*)skip_err_in, (double*)err_out, (double*)skip_err_out)
                : h->pf->backward(mb, (const float*)err_in, (const float*)skip_err_in, (float*)err_out, (float*)skip_err_out);
}

int oracle_backward_microbatch(void* hp, int mb, const void* err_in, void* err_out) {
  return oracle_backward_microbatch_cut(hp, mb, err_in, nullptr, err_out, nullptr);
}

// out: logits [microbatch, classes] with a head, else act_out; BatchNorm uses the running statistics
int oracle_forward_inference(void* hp, const void* act_in, const void* skip_in, void* out, void* skip_out) {
  Handle* h = (Handle*)hp;
  return h->f64 ? h->pd->infer((const double*)act_in, (const double*)skip_in, (double*)out, (double*)skip_out)
                : h->pf->infer((const float*)act_in, (const float*)skip_in, (float*)out, (float*)skip_out);
}

void oracle_set_bn_momentum(void* hp, double momentum) {
  Handle* h = (Handle*)hp;
  if (h->f64) h->pd->bn_momentum = momentum; else h->pf->bn_momentum = momentum;
}

size_t oracle_n_bn_running(void* hp) {
  Handle* h = (Handle*)hp;
  return h->f64 ? h->pd->running.size() : h->pf->running.size();
}

// running statistics as doubles: per BatchNorm in model order mean[c] then variance[c]
int oracle_bn_running_read(void* hp, double* dst, size_t n) {
  Handle* h = (Handle*)hp;
  const std::vector<double>& r = h->f64 ? h->pd->running : h->pf->running;
  if (n != r.size()) return E_INVAL;
  std::memcpy(dst, r.data(), n * sizeof(double));
  return OK;
}

int oracle_bn_running_write(void* hp, const double* src, size_t n) {
  Handle* h = (Handle*)hp;
  std::vector<double>& r = h->f64 ? h->pd->running : h->pf->running;
  if (n != r.size()) return E_INVAL;
  std::memcpy(r.data(), src, n * sizeof(double));
  return OK;
}

int oracle_grad_accum_read(void* hp, void* dst, size_t n) {
  Handle* h = (Handle*)hp;
  return h->f64 ? h->pd->grad_read((double*)dst, n) : h->pf->grad_read((float*)dst, n);
}

int oracle_sgd_step(void* hp, double lr, double mu) {
  Handle* h = (Handle*)hp;
  return h->f64 ? h->pd->sgd_step(lr, mu) : h->pf->sgd_step(lr, mu);
}

// Clears the accumulated gradients and begins a new batch (all micro-batches may run again).
int oracle_grad_accum_zero(void* hp) {
  Handle* h = (Handle*)hp;
  if (h->f64) { std::fill(h->pd->grad.begin(), h->pd->grad.end(), 0.0); h->pd->new_step(); }
  else { std::fill(h->pf->grad.begin(), h->pf->grad.end(), 0.0); h->pf->new_step(); }
  return OK;
}

int oracle_params_read(void* hp, void* dst, size_t n) {
  Handle* h = (Handle*)hp;
  if (n != oracle_n_params(hp)) return E_INVAL;
  if (h->f64) std::memcpy(dst, h->pd->params.data(), n * sizeof(double));
  else std::memcpy(dst, h->pf->params.data(), n * sizeof(float));
  return OK;
}

int oracle_params_write(void* hp, const void* src, size_t n) {
  Handle* h = (Handle*)hp;
  if (n != oracle_n_params(hp)) return E_INVAL;
  if (h->f64) std::memcpy(h->pd->params.data(), src, n * sizeof(double));
  else std::memcpy(h->pf->params.data(), src, n * sizeof(float));
  return OK;
}

#define ORACLE_OPS(SUF, T)                                                                              \
  void oracle_conv_fwd_##SUF(const T* x, const T* w, T* y, int n, int h, int wd, int cin, int cout,     \
                             int R, int st, const T* add, int bf) {                                     \
    conv_fwd<T>(x, w, y, n, h, wd, cin, cout, R, st, add, bf); }                                        \
  void oracle_conv_dgrad_##SUF(const T* dy, const T* w, T* dx, int n, int h, int wd, int cin, int cout, \
                               int R, int st, const T* add, int bf) {                                   \
    conv_dgrad<T>(dy, w, dx, n, h, wd, cin, cout, R, st, add, bf); }                                    \
  void oracle_conv_wgrad_##SUF(const T* x, const T* dy, double* dw, int n, int h, int wd, int cin,      \
                               int cout, int R, int st) {                                               \
    conv_wgrad<T>(x, dy, dw, n, h, wd, cin, cout, R, st); }                                             \
  void oracle_bn_relu_fwd_##SUF(const T* x, const T* g, const T* b, T* a, double* mean, double* invstd, \
                                size_t M, int C, double eps, int mode, int bf) {                        \
    bn_relu_fwd<T>(x, g, b, a, mean, invstd, M, C, eps, mode, bf); }                                    \
  void oracle_bn_relu_bwd_##SUF(const T* x, const T* da, const T* g, const T* b, const double* mean,    \
                                const double* invstd, T* dx, double* dg, double* db, size_t M, int C,   \
                                int mode, const T* skip, int bf) {                                      \
    bn_relu_bwd<T>(x, da, g, b, mean, invstd, dx, dg, db, M, C, mode, skip, bf); }                      \
  double oracle_head_fwd_##SUF(const T* a, const T* wfc, const T* bfc, const int32_t* labels, T* g,     \
                               T* dlogits, int n, int hw, int C, int classes, double divisor) {         \
    return head_fwd<T>(a, wfc, bfc, labels, g, dlogits, n, hw, C, classes, divisor); }                  \
  void oracle_head_bwd_##SUF(const T* g, const T* dl, const T* wfc, double* dwfc, double* dbfc, T* da,  \
                             int n, int hw, int C, int classes) {                                       \
    head_bwd<T>(g, dl, wfc, dwfc, dbfc, da, n, hw, C, classes); }                                       \
  void oracle_bias_act_fwd_##SUF(const T* x, const T* bias, T* y, size_t M, int C, int relu) {          \
    bias_act_fwd<T>(x, bias, y, M, C, relu); }                                                          \
  void oracle_bias_act_bwd_##SUF(const T* y, const T* dy, T* dx, double* db, size_t M, int C, int relu) { \
    bias_act_bwd<T>(y, dy, dx, db, M, C, relu); }                                                       \
  void oracle_maxpool2_fwd_##SUF(const T* x, T* y, int n, int h, int w, int C) {                        \
    maxpool2_fwd<T>(x, y, n, h, w, C); }                                                                \
  void oracle_maxpool2_bwd_##SUF(const T* x, const T* dy, T* dx, int n, int h, int w, int C) {          \
    maxpool2_bwd<T>(x, dy, dx, n, h, w, C); }                                                           \
  void oracle_bn_add_relu_fwd_##SUF(const T* x, const T* g, const T* b, const T* add, T* y, double* mean, \
                                    double* invstd, size_t M, int C, double eps, int mode) {            \
    bn_add_relu_fwd<T>(x, g, b, add, y, mean, invstd, M, C, eps, mode); }                               \
  void oracle_bn_add_relu_bwd_##SUF(const T* x, const T* y, const T* dy, const T* g, const double* mean, \
                                    const double* invstd, T* dx, T* dadd, double* dg, double* db,       \
                                    size_t M, int C, int mode) {                                        \
    bn_add_relu_bwd<T>(x, y, dy, g, mean, invstd, dx, dadd, dg, db, M, C, mode); }

float oracle_round_bf16(float v) { return rnd<float>(v, 1); }

ORACLE_OPS(f32, float)
ORACLE_OPS(f64, double)

}  // extern "C"
