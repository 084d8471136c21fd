// Fused BatchNorm + ReLU, forward and backward, over the M = b*H*W rows of one micro-batch.
//
// These are the bandwidth-bound kernels of the partition's forward / backward pass (every
// convolution of a pre-activation residual block is preceded by one).  Tensors are [M, C] with the
// channel contiguous (NHWC), so a group of <= 32 threads reads one row's <= 256 channels as 16-byte
// vectors and consecutive thread groups read consecutive rows: every load is fully coalesced.
//
// forward : statistics pass (per-channel mean and 1/sqrt(var+eps), biased variance) then
//           a = max(gamma*xhat + beta, 0).
// backward: reduction pass (dbeta = sum dz, dgamma = sum dz*xhat with dz = da*[z>0]) then
//           dx = gamma*invstd*(dz - dbeta/M - xhat*dgamma/M) (+ the skip gradient of an identity
//           shortcut).
// Reductions: per-thread fp32 partial sums -> LDS across the row groups of a block -> one partial
// per block in global memory -> the last block to finish (atomic ticket) adds the partials in block
// order, so the result does not depend on scheduling.  The variance uses sums shifted by the first
// row's value, which removes the cancellation of the sum-of-squares form.
#include "hpf_device.h"

namespace hpf {
namespace {

constexpr int BN_THREADS = 256;
constexpr int BN_MAX_ROW_BLOCKS = 128;

struct BnMap {
  int rl, rpp, c0;
  bool active;
};

__device__ __forceinline__ BnMap bn_map(int C) {
  const int CG = C >> 3;
  const int CGB = CG < 32 ? CG : 32;
  BnMap m;
  m.rpp = BN_THREADS / CGB;
  m.rl = threadIdx.x / CGB;
  const int cg = blockIdx.y * CGB + threadIdx.x % CGB;
  m.active = (m.rl < m.rpp) && (cg < CG);
  m.c0 = cg * 8;
  return m;
}

// Sums the 16 per-thread values over the row groups of the block; result valid in threads rl == 0.
__device__ __forceinline__ void block_reduce16(float (&s)[16], const BnMap& m, int C, float (*sh)[BN_THREADS]) {
  const int CG = C >> 3;
  const int CGB = CG < 32 ? CG : 32;
#pragma unroll
  for (int j = 0; j < 16; ++j) sh[j][threadIdx.x] = s[j];
  __syncthreads();
  if (m.rl == 0) {
    for (int r = 1; r < m.rpp; ++r) {
#pragma unroll
      for (int j = 0; j < 16; ++j) s[j] += sh[j][threadIdx.x + r * CGB];
    }
  }
}

// Returns true in every thread of the block that finished last among the blocks with this blockIdx.y.
__device__ __forceinline__ bool last_block_of_slice(unsigned* tickets) {
  __shared__ int is_last;
  __threadfence();
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned t = atomicAdd(&tickets[blockIdx.y], 1u);
    is_last = (t == gridDim.x - 1);
  }
  __syncthreads();
  if (is_last) __threadfence();
  return is_last != 0;
}

template <class T>
__global__ __launch_bounds__(BN_THREADS) void k_bn_stats(const T* __restrict__ x, int M, int C, int rows_per_block,
                                                         float eps, float* __restrict__ stats,
                                                         float* partials, unsigned* tickets) {
  __shared__ float sh[16][BN_THREADS];
  const BnMap m = bn_map(C);
  float s[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) s[j] = 0.f;
  if (m.active) {
    float k[8], v[8];
    load8(x + m.c0, k);  // shift: first row
    const int r0 = blockIdx.x * rows_per_block;
    const int r1 = min(M, r0 + rows_per_block);
    for (int r = r0 + m.rl; r < r1; r += m.rpp) {
      load8(x + (size_t)r * C + m.c0, v);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float d = v[j] - k[j];
        s[j] += d;
        s[8 + j] = fmaf(d, d, s[8 + j]);
      }
    }
  }
  block_reduce16(s, m, C, sh);
  if (m.active && m.rl == 0) {
    float* p = partials + ((size_t)blockIdx.x * C + m.c0) * 2;
#pragma unroll
    for (int j = 0; j < 8; ++j) { p[2 * j] = s[j]; p[2 * j + 1] = s[8 + j]; }
  }
  if (!last_block_of_slice(tickets)) return;
  const int c = blockIdx.y * 256 + threadIdx.x;
  if (c < C) {
    const volatile float* vp = partials;
    float s1 = 0.f, s2 = 0.f;
    for (unsigned bx = 0; bx < gridDim.x; ++bx) {
      s1 += vp[((size_t)bx * C + c) * 2];
      s2 += vp[((size_t)bx * C + c) * 2 + 1];
    }
    const float inv_m = 1.0f / (float)M;
    const float d = s1 * inv_m;
    float var = fmaf(-d, d, s2 * inv_m);
    var = var > 0.f ? var : 0.f;
    stats[c] = to_f32(x[c]) + d;
    stats[C + c] = 1.0f / sqrtf(var + eps);
  }
  if (threadIdx.x == 0) tickets[blockIdx.y] = 0;
}

template <class T>
__global__ __launch_bounds__(BN_THREADS) void k_bn_apply_relu(const T* __restrict__ x, T* __restrict__ a,
                                                              const float* __restrict__ gamma,
                                                              const float* __restrict__ beta,
                                                              const float* __restrict__ stats, int M, int C) {
  const BnMap m = bn_map(C);
  if (!m.active) return;
  float mu[8], is[8], g[8], bt[8], v[8];
  load8(stats + m.c0, mu); load8(stats + C + m.c0, is); load8(gamma + m.c0, g); load8(beta + m.c0, bt);
  for (int r = blockIdx.x * m.rpp + m.rl; r < M; r += gridDim.x * m.rpp) {
    load8(x + (size_t)r * C + m.c0, v);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float z = fmaf((v[j] - mu[j]) * is[j], g[j], bt[j]);
      v[j] = z > 0.f ? z : 0.f;
    }
    store8(a + (size_t)r * C + m.c0, v);
  }
}

template <class T>
__global__ __launch_bounds__(BN_THREADS) void k_bn_bwd_reduce(const T* __restrict__ x, const T* __restrict__ da,
                                                              const float* __restrict__ gamma,
                                                              const float* __restrict__ beta,
                                                              const float* __restrict__ stats, int M, int C,
                                                              int rows_per_block, float* __restrict__ sums,
                                                              float* g_gamma, float* g_beta, float* partials,
                                                              unsigned* tickets) {
  __shared__ float sh[16][BN_THREADS];
  const BnMap m = bn_map(C);
  float s[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) s[j] = 0.f;
  if (m.active) {
    float mu[8], is[8], g[8], bt[8], v[8], d[8];
    load8(stats + m.c0, mu); load8(stats + C + m.c0, is); load8(gamma + m.c0, g); load8(beta + m.c0, bt);
    const int r0 = blockIdx.x * rows_per_block;
    const int r1 = min(M, r0 + rows_per_block);
    for (int r = r0 + m.rl; r < r1; r += m.rpp) {
      load8(x + (size_t)r * C + m.c0, v);
      load8(da + (size_t)r * C + m.c0, d);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float xh = (v[j] - mu[j]) * is[j];
        const float z = fmaf(xh, g[j], bt[j]);
        const float dz = z > 0.f ? d[j] : 0.f;
        s[j] += dz;
        s[8 + j] = fmaf(dz, xh, s[8 + j]);
      }
    }
  }
  block_reduce16(s, m, C, sh);
  if (m.active && m.rl == 0) {
    float* p = partials + ((size_t)blockIdx.x * C + m.c0) * 2;
#pragma unroll
    for (int j = 0; j < 8; ++j) { p[2 * j] = s[j]; p[2 * j + 1] = s[8 + j]; }
  }
  if (!last_block_of_slice(tickets)) return;
  const int c = blockIdx.y * 256 + threadIdx.x;
  if (c < C) {
    const volatile float* vp = partials;
    float s1 = 0.f, s2 = 0.f;
    for (unsigned bx = 0; bx < gridDim.x; ++bx) {
      s1 += vp[((size_t)bx * C + c) * 2];
      s2 += vp[((size_t)bx * C + c) * 2 + 1];
    }
    sums[c] = s1;
    sums[C + c] = s2;
    atomicAdd(&g_beta[c], s1);
    atomicAdd(&g_gamma[c], s2);
  }
  if (threadIdx.x == 0) tickets[blockIdx.y] = 0;
}

template <class T>
__global__ __launch_bounds__(BN_THREADS) void k_bn_bwd_apply(const T* __restrict__ x, const T* __restrict__ da,
                                                             const float* __restrict__ gamma,
                                                             const float* __restrict__ beta,
                                                             const float* __restrict__ stats,
                                                             const float* __restrict__ sums, const T* skip,
                                                             T* dx, int M, int C, int frozen) {
  const BnMap m = bn_map(C);
  if (!m.active) return;
  float mu[8], is[8], g[8], bt[8], sb[8], sg[8], v[8], d[8], k[8];
  load8(stats + m.c0, mu); load8(stats + C + m.c0, is); load8(gamma + m.c0, g); load8(beta + m.c0, bt);
  load8(sums + m.c0, sb); load8(sums + C + m.c0, sg);
  const float inv_m = frozen ? 0.f : 1.0f / (float)M;
#pragma unroll
  for (int j = 0; j < 8; ++j) { sb[j] *= inv_m; sg[j] *= inv_m; }
  for (int r = blockIdx.x * m.rpp + m.rl; r < M; r += gridDim.x * m.rpp) {
    const size_t o = (size_t)r * C + m.c0;
    load8(x + o, v);
    load8(da + o, d);
    if (skip) load8(skip + o, k);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float xh = (v[j] - mu[j]) * is[j];
      const float z = fmaf(xh, g[j], bt[j]);
      const float dz = z > 0.f ? d[j] : 0.f;
      float o_ = g[j] * is[j] * (dz - sb[j] - xh * sg[j]);
      if (skip) o_ += k[j];
      v[j] = o_;
    }
    store8(dx + o, v);
  }
}

__global__ void k_bn_frozen_stats(float* stats, int C, float eps) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c < C) { stats[c] = 0.f; stats[C + c] = 1.0f / sqrtf(1.0f + eps); }
}

struct BnGrid { dim3 grid; int rows_per_block; };

BnGrid reduce_grid(int M, int C) {
  const int CG = C / 8, CGB = CG < 32 ? CG : 32, rpp = BN_THREADS / CGB;
  int gx = (M + rpp - 1) / rpp;
  if (gx > BN_MAX_ROW_BLOCKS) gx = BN_MAX_ROW_BLOCKS;
  int rpb = (M + gx - 1) / gx;
  rpb = (rpb + rpp - 1) / rpp * rpp;
  gx = (M + rpb - 1) / rpb;
  return BnGrid{dim3((unsigned)gx, (unsigned)((CG + CGB - 1) / CGB)), rpb};
}

dim3 apply_grid(int M, int C) {
  const int CG = C / 8, CGB = CG < 32 ? CG : 32, rpp = BN_THREADS / CGB;
  int gx = (M + rpp - 1) / rpp;
  if (gx > 2048) gx = 2048;
  return dim3((unsigned)gx, (unsigned)((CG + CGB - 1) / CGB));
}

}  // namespace

size_t bn_partials_floats(int C) { return (size_t)BN_MAX_ROW_BLOCKS * C * 2; }

hipError_t launch_bn_stats(int dt, const void* x, int M, int C, float eps, float* stats, float* partials,
                           unsigned* tickets, hipStream_t stream) {
  const BnGrid g = reduce_grid(M, C);
  if (dt == DT_BF16)
    k_bn_stats<bf16_t><<<g.grid, BN_THREADS, 0, stream>>>((const bf16_t*)x, M, C, g.rows_per_block, eps, stats, partials, tickets);
  else
    k_bn_stats<float><<<g.grid, BN_THREADS, 0, stream>>>((const float*)x, M, C, g.rows_per_block, eps, stats, partials, tickets);
  return hipGetLastError();
}

hipError_t launch_bn_apply_relu(int dt, const void* x, void* a, const float* gamma, const float* beta,
                                const float* stats, int M, int C, hipStream_t stream) {
  const dim3 grid = apply_grid(M, C);
  if (dt == DT_BF16)
    k_bn_apply_relu<bf16_t><<<grid, BN_THREADS, 0, stream>>>((const bf16_t*)x, (bf16_t*)a, gamma, beta, stats, M, C);
  else
    k_bn_apply_relu<float><<<grid, BN_THREADS, 0, stream>>>((const float*)x, (float*)a, gamma, beta, stats, M, C);
  return hipGetLastError();
}

hipError_t launch_bn_bwd_reduce(int dt, const void* x, const void* da, const float* gamma, const float* beta,
                                const float* stats, int M, int C, float* sums, float* g_gamma, float* g_beta,
                                float* partials, unsigned* tickets, hipStream_t stream) {
  const BnGrid g = reduce_grid(M, C);
  if (dt == DT_BF16)
    k_bn_bwd_reduce<bf16_t><<<g.grid, BN_THREADS, 0, stream>>>((const bf16_t*)x, (const bf16_t*)da, gamma, beta, stats, M, C,
                                                               g.rows_per_block, sums, g_gamma, g_beta, partials, tickets);
  else
    k_bn_bwd_reduce<float><<<g.grid, BN_THREADS, 0, stream>>>((const float*)x, (const float*)da, gamma, beta, stats, M, C,
                                                              g.rows_per_block, sums, g_gamma, g_beta, partials, tickets);
  return hipGetLastError();
}

hipError_t launch_bn_bwd_apply(int dt, const void* x, const void* da, const float* gamma, const float* beta,
                               const float* stats, const float* sums, const void* skip, void* dx, int M, int C,
                               int frozen, hipStream_t stream) {
  const dim3 grid = apply_grid(M, C);
  if (dt == DT_BF16)
    k_bn_bwd_apply<bf16_t><<<grid, BN_THREADS, 0, stream>>>((const bf16_t*)x, (const bf16_t*)da, gamma, beta, stats, sums,
                                                            (const bf16_t*)skip, (bf16_t*)dx, M, C, frozen);
  else
    k_bn_bwd_apply<float><<<grid, BN_THREADS, 0, stream>>>((const float*)x, (const float*)da, gamma, beta, stats, sums,
                                                           (const float*)skip, (float*)dx, M, C, frozen);
  return hipGetLastError();
}

hipError_t launch_bn_frozen_stats(float* stats, int C, float eps, hipStream_t stream) {
  k_bn_frozen_stats<<<(C + 255) / 256, 256, 0, stream>>>(stats, C, eps);
  return hipGetLastError();
}

}  // namespace hpf
