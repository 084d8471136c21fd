// fp32 check-mode convolutions: direct, one output element per thread, fp32 tensors, accumulation
// in double (so a stored output is the correctly rounded sum, as in a double-accumulating
// reference, and downstream ReLU decisions see the same values).  They exist so that the whole
// runtime (scheduling, stash, indexing, BN, accumulation) can be compared with the CPU reference
// at fp32 accuracy; speed is not their purpose.
#include "hpf_device.h"

namespace hpf {
namespace {

// out[m, n] = sum_{tap, c} src[row(m,tap), c] * W(tap, c, n)  (+ add[m, n])
//   CONV_FWD  : W(tap,c,n) = w[tap][c][n]   (Cs = Cin,  N = Cout)
//   CONV_DGRAD: W(tap,c,n) = w[tap][n][c]   (Cs = Cout, N = Cin)
template <int MODE>
__global__ __launch_bounds__(256) void k_conv_f32(PtrTab srcs, const float* __restrict__ w, PtrTab outs, PtrTab adds,
                                                  ConvGeom g) {
  const float* __restrict__ src = (const float*)pick(srcs, blockIdx.z);
  float* out = (float*)pick(outs, blockIdx.z);
  const float* add = (const float*)pick(adds, blockIdx.z);
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (size_t)g.M * g.N) return;
  const int n = (int)(idx % g.N);
  const int m = (int)(idx / g.N);
  const int img = m / (g.Ho * g.Wo);
  const int rem = m - img * g.Ho * g.Wo;
  const int p = rem / g.Wo, q = rem - p * g.Wo;
  double acc = 0.0;
  for (int r = 0; r < g.R; ++r) {
    int hs;
    if (MODE == CONV_FWD) {
      hs = p * g.stride + r - g.pad;
    } else {
      const int t = p + g.pad - r;
      if (t < 0 || (t % g.stride) != 0) continue;
      hs = t / g.stride;
    }
    if (hs < 0 || hs >= g.Hs) continue;
    for (int s = 0; s < g.R; ++s) {
      int ws;
      if (MODE == CONV_FWD) {
        ws = q * g.stride + s - g.pad;
      } else {
        const int t = q + g.pad - s;
        if (t < 0 || (t % g.stride) != 0) continue;
        ws = t / g.stride;
      }
      if (ws < 0 || ws >= g.Ws) continue;
      const float* sp = src + ((size_t)(img * g.Hs + hs) * g.Ws + ws) * g.Cs;
      const int tap = r * g.R + s;
      if (MODE == CONV_FWD) {
        const float* wp = w + (size_t)tap * g.Cs * g.N + n;
        for (int c = 0; c < g.Cs; ++c) acc += (double)sp[c] * (double)wp[(size_t)c * g.N];
      } else {
        const float* wp = w + ((size_t)tap * g.N + n) * g.Cs;
        for (int c = 0; c < g.Cs; ++c) acc += (double)sp[c] * (double)wp[c];
      }
    }
  }
  if (add) acc += (double)add[idx];
  out[idx] = (float)acc;
}

// dw[tap][c][n] += sum over this block's row slice of a[row(m,tap), c] * dy[m, n]
__global__ __launch_bounds__(256) void k_wgrad_f32(PtrTab as, PtrTab dys, float* dw, WgradGeom g, int rows_per_slice) {
  const float* __restrict__ a = (const float*)pick(as, blockIdx.z);
  const float* __restrict__ dy = (const float*)pick(dys, blockIdx.z);
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t total = (size_t)g.R * g.R * g.c_valid * g.N;
  if (idx >= total) return;
  const int n = (int)(idx % g.N);
  const int c = (int)((idx / g.N) % g.c_valid);
  const int tap = (int)(idx / ((size_t)g.N * g.c_valid));
  const int r = tap / g.R, s = tap - r * g.R;
  const int m0 = blockIdx.y * rows_per_slice;
  const int m1 = min(g.M, m0 + rows_per_slice);
  double acc = 0.0;
  for (int m = m0; m < m1; ++m) {
    const int img = m / (g.Ho * g.Wo);
    const int rem = m - img * g.Ho * g.Wo;
    const int p = rem / g.Wo, q = rem - p * g.Wo;
    const int hi = p * g.stride + r - g.pad, wi = q * g.stride + s - g.pad;
    if ((unsigned)hi >= (unsigned)g.H || (unsigned)wi >= (unsigned)g.W) continue;
    acc += (double)a[((size_t)(img * g.H + hi) * g.W + wi) * g.Cin + c] * (double)dy[(size_t)m * g.N + n];
  }
  atomicAdd(&dw[idx], (float)acc);
}

}  // namespace

hipError_t launch_conv_f32(int mode, int ng, const PtrTab& src, const float* w_hwio, const PtrTab& out, const PtrTab& add,
                           const ConvGeom& g, hipStream_t stream) {
  const size_t total = (size_t)g.M * g.N;
  const dim3 grid((unsigned)((total + 255) / 256), 1, (unsigned)ng);
  if (mode == CONV_FWD)
    k_conv_f32<CONV_FWD><<<grid, 256, 0, stream>>>(src, w_hwio, out, add, g);
  else
    k_conv_f32<CONV_DGRAD><<<grid, 256, 0, stream>>>(src, w_hwio, out, add, g);
  return hipGetLastError();
}

hipError_t launch_wgrad_f32(int ng, const PtrTab& a, const PtrTab& dy, float* dw, const WgradGeom& g, hipStream_t stream) {
  const size_t total = (size_t)g.R * g.R * g.c_valid * g.N;
  const unsigned gx = (unsigned)((total + 255) / 256);
  int slices = (int)(1024 / (gx ? gx : 1));
  if (slices < 1) slices = 1;
  const int max_slices = (g.M + 63) / 64;
  if (slices > max_slices) slices = max_slices;
  const int rows = (g.M + slices - 1) / slices;
  slices = (g.M + rows - 1) / rows;
  k_wgrad_f32<<<dim3(gx, (unsigned)slices, (unsigned)ng), 256, 0, stream>>>(a, dy, dw, g, rows);
  return hipGetLastError();
}

}  // namespace hpf
