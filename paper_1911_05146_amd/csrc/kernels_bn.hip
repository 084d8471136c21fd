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
// Reductions: per-thread partial sums -> cross-lane shuffles and LDS across the row groups of a
// block -> one partial per block in global memory; a second, one-block-per-256-channels kernel adds
// the partials in a fixed order, so the result does not depend on scheduling (a grid-wide
// "last block finishes" scheme was measured slower here: its device-scope fence and atomic round
// trips cost more than a kernel boundary).  The variance uses sums shifted by the first row's
// value, which removes the cancellation of the sum-of-squares form.
//
// Arithmetic type A: float in bf16 mode; double in the fp32 check mode, where tensors are fp32 but
// every reduction, statistic and the pre-activation z are computed in double, so that the ReLU
// decision z > 0 is taken on (practically) the same value as a double-accumulating reference.
// Statistics, per-micro-batch sums and partials are arrays of A.
#include "hpf_device.h"

namespace hpf {
namespace {

constexpr int BN_THREADS = 256;
constexpr int BN_MAX_ROW_BLOCKS = 128;

template <class A>
__device__ __forceinline__ void load8a(const A* p, A (&v)[8]) {
#pragma unroll
  for (int j = 0; j < 8; ++j) v[j] = p[j];
}
template <class T, class A>
__device__ __forceinline__ void load8t(const T* p, A (&v)[8]) {
  float f[8];
  load8(p, f);
#pragma unroll
  for (int j = 0; j < 8; ++j) v[j] = (A)f[j];
}
template <class T, class A>
__device__ __forceinline__ void store8t(T* p, const A (&v)[8]) {
  float f[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) f[j] = (float)v[j];
  store8(p, f);
}
__device__ __forceinline__ float rsqrt_exact(float v) { return 1.0f / sqrtf(v); }
__device__ __forceinline__ double rsqrt_exact(double v) { return 1.0 / sqrt(v); }

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

__device__ __forceinline__ float shfl_xor_a(float v, int o) { return __shfl_xor(v, o); }
__device__ __forceinline__ double shfl_xor_a(double v, int o) { return __shfl_xor(v, o); }

// Sums the 16 per-thread values over the row groups of the block; result valid in threads rl == 0.
// When the channel-group count per block is a power of two (every ResNet width here) the rows held
// by one wavefront are added with cross-lane shuffles and only 4 values per column go through LDS;
// otherwise the first row group adds the others serially.
template <class A>
__device__ __forceinline__ void block_reduce16(A (&s)[16], const BnMap& m, int C, A (*sh)[BN_THREADS]) {
  const int CG = C >> 3;
  const int CGB = CG < 32 ? CG : 32;
  if ((CGB & (CGB - 1)) == 0) {
    for (int o = CGB; o < 64; o <<= 1) {
#pragma unroll
      for (int j = 0; j < 16; ++j) s[j] += shfl_xor_a(s[j], o);
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane < CGB) {
#pragma unroll
      for (int j = 0; j < 16; ++j) sh[j][wave * 32 + lane] = s[j];
    }
    __syncthreads();
    if (m.rl == 0) {   // threads 0 .. CGB-1 of wave 0
#pragma unroll
      for (int j = 0; j < 16; ++j) s[j] = ((sh[j][lane] + sh[j][32 + lane]) + sh[j][64 + lane]) + sh[j][96 + lane];
    }
    return;
  }
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

// Statistics partial of one block of rows (or one convolution output tile), per channel:
// {K, S1 = sum(v - K), S2 = sum((v - K)^2), n} with the shift K = the block's first row.  The
// shifted sums avoid the cancellation of the plain sum-of-squares form; blocks with different
// shifts are merged exactly (pairwise update of count / mean / sum of squared deviations).
template <class T, class A>
__global__ __launch_bounds__(BN_THREADS) void k_bn_stats(PtrTab xs, int M, int C, int rows_per_block, PtrTab parts) {
  const T* __restrict__ x = (const T*)pick(xs, blockIdx.z);
  A* __restrict__ partials = (A*)pick(parts, blockIdx.z);
  __shared__ A sh[16][BN_THREADS];
  const BnMap m = bn_map(C);
  A s[16], k[8];
#pragma unroll
  for (int j = 0; j < 16; ++j) s[j] = 0;
  const int r0 = blockIdx.x * rows_per_block;
  const int r1 = min(M, r0 + rows_per_block);
  if (m.active) {
    A v[8];
    load8t(x + (size_t)r0 * C + m.c0, k);  // shift: first row of this block
    for (int r = r0 + m.rl; r < r1; r += m.rpp) {
      load8t(x + (size_t)r * C + m.c0, v);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const A d = v[j] - k[j];
        s[j] += d;
        s[8 + j] += d * d;
      }
    }
  }
  block_reduce16(s, m, C, sh);
  if (m.active && m.rl == 0) {
    A* p = partials + ((size_t)blockIdx.x * C + m.c0) * 4;
#pragma unroll
    for (int j = 0; j < 8; ++j) { p[4 * j] = k[j]; p[4 * j + 1] = s[j]; p[4 * j + 2] = s[8 + j]; p[4 * j + 3] = (A)(r1 - r0); }
  }
}

// Finalize: block = 32 channels x 8 row-groups, grid (ceil(C/32), 1, g).  Two passes over the records
// (the second hits the cache): first the mean from the tile sums, then the sum of squared deviations
// about that mean, M2 = sum_t [S2_t - S1_t^2/n_t + n_t (mean_t - mean)^2].  All additions are
// independent (no serial merge chain) and their order is fixed: strided partial sums per row-group,
// then the 8 row-groups in order through LDS.
constexpr int FIN_CH = 32, FIN_RG = BN_THREADS / FIN_CH;

template <class A>
__device__ __forceinline__ A fin_sum(A v, A (*sh)[FIN_CH], int cl, int j) {
  __syncthreads();
  sh[j][cl] = v;
  __syncthreads();
  A t = sh[0][cl];
#pragma unroll
  for (int r = 1; r < FIN_RG; ++r) t += sh[r][cl];
  return t;
}

template <class A>
__global__ __launch_bounds__(BN_THREADS) void k_bn_stats_finalize(int M, int C, unsigned nblocks, float eps, PtrTab parts,
                                                                  PtrTab statss) {
  const A* __restrict__ partials = (const A*)pick(parts, blockIdx.z);
  A* __restrict__ stats = (A*)pick(statss, blockIdx.z);
  __shared__ A sh[FIN_RG][FIN_CH];
  const int cl = threadIdx.x % FIN_CH, j = threadIdx.x / FIN_CH;
  const int c = blockIdx.x * FIN_CH + cl;
  const bool cv = c < C;
  const A* p = partials + (size_t)(cv ? c : 0) * 4;
  A tot = 0;
  if (cv) {
#pragma unroll 4
    for (unsigned bx = j; bx < nblocks; bx += FIN_RG) {
      const A* q = p + (size_t)bx * C * 4;
      tot += q[3] * q[0] + q[1];                 // n*K + S1 = sum of the tile's values
    }
  }
  const A mean = fin_sum(tot, sh, cl, j) / (A)M;
  A m2 = 0;
  if (cv) {
#pragma unroll 4
    for (unsigned bx = j; bx < nblocks; bx += FIN_RG) {
      const A* q = p + (size_t)bx * C * 4;
      const A n = q[3];
      if (n > 0) {
        const A s1n = q[1] / n, d = q[0] + s1n - mean;
        m2 += q[2] - q[1] * s1n + n * d * d;
      }
    }
  }
  m2 = fin_sum(m2, sh, cl, j);
  if (cv && j == 0) {
    A var = m2 / (A)M;
    var = var > 0 ? var : 0;
    stats[c] = mean;
    stats[C + c] = rsqrt_exact(var + (A)eps);
  }
}

// The float (bf16 mode) finalize kernels: the same two-pass arithmetic with 16 channels x 16 row-groups per block and
// the first FIN_CACHE records of every thread held in registers -- all their loads are in flight at once and the
// second pass does not go back to memory (up to 128 tile rows: one memory round trip instead of a chain of them;
// these launches sit between every convolution and its consumer, so their latency is on the critical path).
constexpr int FINW_CH = 16, FINW_RG = BN_THREADS / FINW_CH, FIN_CACHE = 8;

__device__ __forceinline__ float finw_sum(float v, float (*sh)[FINW_CH + 1], int cl, int j) {
  __syncthreads();
  sh[j][cl] = v;
  __syncthreads();
  float t = sh[0][cl];
#pragma unroll
  for (int r = 1; r < FINW_RG; ++r) t += sh[r][cl];
  return t;
}

__global__ __launch_bounds__(BN_THREADS) void k_bn_stats_finalize_wide(int M, int C, unsigned nblocks, float eps, PtrTab parts,
                                                                       PtrTab statss) {
  const float4* __restrict__ partials = (const float4*)pick(parts, blockIdx.z);
  float* __restrict__ stats = (float*)pick(statss, blockIdx.z);
  __shared__ float sh[FINW_RG][FINW_CH + 1];
  const int cl = threadIdx.x % FINW_CH, j = threadIdx.x / FINW_CH;
  const int c = blockIdx.x * FINW_CH + cl;
  const bool cv = c < C;
  const float4* p = partials + (cv ? c : 0);
  float4 rec[FIN_CACHE];   // {K, S1, S2, n}
#pragma unroll
  for (int i = 0; i < FIN_CACHE; ++i) {
    const unsigned bx = (unsigned)j + (unsigned)i * FINW_RG;
    rec[i] = (cv && bx < nblocks) ? p[(size_t)bx * C] : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  float tot = 0.f;
#pragma unroll
  for (int i = 0; i < FIN_CACHE; ++i) tot += rec[i].w * rec[i].x + rec[i].y;   // n*K + S1 = sum of the tile's values
  if (cv)
    for (unsigned bx = (unsigned)j + FIN_CACHE * FINW_RG; bx < nblocks; bx += FINW_RG) {
      const float4 q = p[(size_t)bx * C];
      tot += q.w * q.x + q.y;
    }
  const float mean = finw_sum(tot, sh, cl, j) / (float)M;
  auto dev2 = [&](const float4& q) {   // sum of squared deviations of the tile about the overall mean
    if (!(q.w > 0.f)) return 0.f;
    const float s1n = q.y / q.w, d = q.x + s1n - mean;
    return q.z - q.y * s1n + q.w * d * d;
  };
  float m2 = 0.f;
#pragma unroll
  for (int i = 0; i < FIN_CACHE; ++i) m2 += dev2(rec[i]);
  if (cv)
    for (unsigned bx = (unsigned)j + FIN_CACHE * FINW_RG; bx < nblocks; bx += FINW_RG) m2 += dev2(p[(size_t)bx * C]);
  m2 = finw_sum(m2, sh, cl, j);
  if (cv && j == 0) {
    float var = m2 / (float)M;
    var = var > 0.f ? var : 0.f;
    stats[c] = mean;
    stats[C + c] = rsqrt_exact(var + eps);
  }
}

__global__ __launch_bounds__(BN_THREADS) void k_bn_bwd_finalize_wide(int C, unsigned nblocks, PtrTab parts, PtrTab sumss, float* g_gamma,
                                                                     float* g_beta) {
  const float2* __restrict__ partials = (const float2*)pick(parts, blockIdx.z);
  float* __restrict__ sums = (float*)pick(sumss, blockIdx.z);
  __shared__ float sh[FINW_RG][FINW_CH + 1];
  const int cl = threadIdx.x % FINW_CH, j = threadIdx.x / FINW_CH;
  const int c = blockIdx.x * FINW_CH + cl;
  const bool cv = c < C;
  const float2* p = partials + (cv ? c : 0);
  float2 rec[FIN_CACHE];
#pragma unroll
  for (int i = 0; i < FIN_CACHE; ++i) {
    const unsigned bx = (unsigned)j + (unsigned)i * FINW_RG;
    rec[i] = (cv && bx < nblocks) ? p[(size_t)bx * C] : make_float2(0.f, 0.f);
  }
  float a1 = 0.f, a2 = 0.f;
#pragma unroll
  for (int i = 0; i < FIN_CACHE; ++i) { a1 += rec[i].x; a2 += rec[i].y; }
  if (cv)
    for (unsigned bx = (unsigned)j + FIN_CACHE * FINW_RG; bx < nblocks; bx += FINW_RG) {
      const float2 q = p[(size_t)bx * C];
      a1 += q.x; a2 += q.y;
    }
  a1 = finw_sum(a1, sh, cl, j);
  a2 = finw_sum(a2, sh, cl, j);
  if (cv && j == 0) {
    sums[c] = a1;
    sums[C + c] = a2;
    atomicAdd(&g_beta[c], a1);
    if (g_gamma) atomicAdd(&g_gamma[c], a2);
  }
}

template <class T, class A>
__global__ __launch_bounds__(BN_THREADS) void k_bn_apply_relu(PtrTab xs, PtrTab as, const float* __restrict__ gamma,
                                                              const float* __restrict__ beta, PtrTab statss, int M,
                                                              int C) {
  const T* __restrict__ x = (const T*)pick(xs, blockIdx.z);
  T* __restrict__ a = (T*)pick(as, blockIdx.z);
  const A* __restrict__ stats = (const A*)pick(statss, blockIdx.z);
  const BnMap m = bn_map(C);
  if (!m.active) return;
  A mu[8], is[8], g[8], bt[8], v[8];
  load8a(stats + m.c0, mu); load8a(stats + C + m.c0, is); load8t(gamma + m.c0, g); load8t(beta + m.c0, bt);
  for (int r = blockIdx.x * m.rpp + m.rl; r < M; r += gridDim.x * m.rpp) {
    load8t(x + (size_t)r * C + m.c0, v);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const A z = g[j] * ((v[j] - mu[j]) * is[j]) + bt[j];
      v[j] = z > 0 ? z : (A)0;
    }
    store8t(a + (size_t)r * C + m.c0, v);
  }
}

template <class T, class A>
__global__ __launch_bounds__(BN_THREADS) void k_bn_bwd_reduce(PtrTab xs, PtrTab das, const float* __restrict__ gamma,
                                                              const float* __restrict__ beta, PtrTab statss, int M,
                                                              int C, int rows_per_block, PtrTab parts) {
  const T* __restrict__ x = (const T*)pick(xs, blockIdx.z);
  const T* __restrict__ da = (const T*)pick(das, blockIdx.z);
  const A* __restrict__ stats = (const A*)pick(statss, blockIdx.z);
  A* __restrict__ partials = (A*)pick(parts, blockIdx.z);
  __shared__ A sh[16][BN_THREADS];
  const BnMap m = bn_map(C);
  A s[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) s[j] = 0;
  if (m.active) {
    A mu[8], is[8], g[8], bt[8], v[8], d[8];
    load8a(stats + m.c0, mu); load8a(stats + C + m.c0, is); load8t(gamma + m.c0, g); load8t(beta + m.c0, bt);
    const int r0 = blockIdx.x * rows_per_block;
    const int r1 = min(M, r0 + rows_per_block);
    for (int r = r0 + m.rl; r < r1; r += m.rpp) {
      load8t(x + (size_t)r * C + m.c0, v);
      load8t(da + (size_t)r * C + m.c0, d);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const A xh = (v[j] - mu[j]) * is[j];
        const A z = g[j] * xh + bt[j];
        const A dz = z > 0 ? d[j] : (A)0;
        s[j] += dz;
        s[8 + j] += dz * xh;
      }
    }
  }
  block_reduce16(s, m, C, sh);
  if (m.active && m.rl == 0) {
    A* p = partials + ((size_t)blockIdx.x * C + m.c0) * 2;
#pragma unroll
    for (int j = 0; j < 8; ++j) { p[2 * j] = s[j]; p[2 * j + 1] = s[8 + j]; }
  }
}

// grid (ceil(C/32), 1, g): dbeta / dgamma of each micro-batch from the partials; also added into the
// gradient buffer shared by all micro-batches.
template <class A>
__global__ __launch_bounds__(BN_THREADS) void k_bn_bwd_finalize(int C, unsigned nblocks, PtrTab parts, PtrTab sumss,
                                                                float* g_gamma, float* g_beta) {
  const A* __restrict__ partials = (const A*)pick(parts, blockIdx.z);
  A* __restrict__ sums = (A*)pick(sumss, blockIdx.z);
  __shared__ A sh[FIN_RG][FIN_CH];
  const int cl = threadIdx.x % FIN_CH, j = threadIdx.x / FIN_CH;
  const int c = blockIdx.x * FIN_CH + cl;
  const bool cv = c < C;
  const A* p = partials + (size_t)(cv ? c : 0) * 2;
  A a1 = 0, a2 = 0;
  if (cv) {
#pragma unroll 8
    for (unsigned bx = j; bx < nblocks; bx += FIN_RG) {
      a1 += p[(size_t)bx * C * 2];
      a2 += p[(size_t)bx * C * 2 + 1];
    }
  }
  a1 = fin_sum(a1, sh, cl, j);
  a2 = fin_sum(a2, sh, cl, j);
  if (cv && j == 0) {
    sums[c] = a1;
    sums[C + c] = a2;
    atomicAdd(&g_beta[c], (float)a1);
    if (g_gamma) atomicAdd(&g_gamma[c], (float)a2);
  }
}

template <class T, class A>
__global__ __launch_bounds__(BN_THREADS) void k_bn_bwd_apply(PtrTab xs, PtrTab das, const float* __restrict__ gamma,
                                                             const float* __restrict__ beta, PtrTab statss, PtrTab sumss,
                                                             PtrTab skips, PtrTab dxs, int M, int C, int frozen) {
  const T* __restrict__ x = (const T*)pick(xs, blockIdx.z);
  const T* __restrict__ da = (const T*)pick(das, blockIdx.z);
  const A* __restrict__ stats = (const A*)pick(statss, blockIdx.z);
  const A* __restrict__ sums = (const A*)pick(sumss, blockIdx.z);
  const T* skip = (const T*)pick(skips, blockIdx.z);
  T* dx = (T*)pick(dxs, blockIdx.z);
  const BnMap m = bn_map(C);
  if (!m.active) return;
  A mu[8], is[8], g[8], bt[8], sb[8], sg[8], v[8], d[8], k[8];
  load8a(stats + m.c0, mu); load8a(stats + C + m.c0, is); load8t(gamma + m.c0, g); load8t(beta + m.c0, bt);
  load8a(sums + m.c0, sb); load8a(sums + C + m.c0, sg);
  const A inv_m = frozen ? (A)0 : (A)1 / (A)M;
#pragma unroll
  for (int j = 0; j < 8; ++j) { sb[j] *= inv_m; sg[j] *= inv_m; }
  for (int r = blockIdx.x * m.rpp + m.rl; r < M; r += gridDim.x * m.rpp) {
    const size_t o = (size_t)r * C + m.c0;
    load8t(x + o, v);
    load8t(da + o, d);
    if (skip) load8t(skip + o, k);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const A xh = (v[j] - mu[j]) * is[j];
      const A z = g[j] * xh + bt[j];
      const A dz = z > 0 ? d[j] : (A)0;
      A o_ = g[j] * is[j] * (dz - sb[j] - xh * sg[j]);
      if (skip) o_ += k[j];
      v[j] = o_;
    }
    store8t(dx + o, v);
  }
}

template <class A>
__global__ void k_bn_frozen_stats(PtrTab statss, int C, float eps) {
  A* stats = (A*)pick(statss, blockIdx.z);
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c < C) { stats[c] = 0; stats[C + c] = rsqrt_exact((A)1 + (A)eps); }
}

// One block per BatchNorm; a thread walks its channels and, per channel, the group's members in order.
template <class A>
__global__ __launch_bounds__(256) void k_bn_running_update(PtrTab bases, const BnRunDesc* __restrict__ table, float* running, int ng,
                                                           float momentum, float eps) {
  const BnRunDesc d = table[blockIdx.x];
  float* rm = running + d.run_off;
  float* rv = rm + d.C;
  for (int c = threadIdx.x; c < d.C; c += blockDim.x) {
    A m = (A)rm[c], v = (A)rv[c];
    for (int i = 0; i < ng; ++i) {
      const A* st = (const A*)((const char*)pick(bases, i) + d.stats_off);
      const A is = st[d.C + c];
      const A var = (A)1 / (is * is) - (A)eps;
      m = (A)momentum * m + ((A)1 - (A)momentum) * st[c];
      v = (A)momentum * v + ((A)1 - (A)momentum) * var;
    }
    rm[c] = (float)m; rv[c] = (float)v;
  }
}

template <class A>
__global__ void k_bn_running_stats(PtrTab statss, const float* __restrict__ running, int C, float eps) {
  A* stats = (A*)pick(statss, blockIdx.z);
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c < C) { stats[c] = (A)running[c]; stats[C + c] = rsqrt_exact((A)running[C + c] + (A)eps); }
}


// ------------------------------------------------------------------------------------------------------------
// Layers of the paper's two other models (Section "Model-Parallelism on a Single Node": VGG-16, ResNet-110-v1),
// built on the same row / channel mapping and the same two-step reductions.
// ------------------------------------------------------------------------------------------------------------
// y = x + bias[c], then max(., 0) when relu.
template <class T, class A>
__global__ __launch_bounds__(BN_THREADS) void k_bias_act_fwd(PtrTab xs, PtrTab ys, const float* __restrict__ bias, int M, int C,
                                                             int relu) {
  const T* x = (const T*)pick(xs, blockIdx.z);   // may be y (in place)
  T* y = (T*)pick(ys, blockIdx.z);
  const BnMap m = bn_map(C);
  if (!m.active) return;
  A bs[8], v[8];
  load8t(bias + m.c0, bs);
  for (int r = blockIdx.x * m.rpp + m.rl; r < M; r += gridDim.x * m.rpp) {
    load8t(x + (size_t)r * C + m.c0, v);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const A z = v[j] + bs[j];
      v[j] = (relu && !(z > 0)) ? (A)0 : z;
    }
    store8t(y + (size_t)r * C + m.c0, v);
  }
}
// dx = dz = dy * [y > 0] (relu) or dy; partial sums of dz per block of rows (record layout of the BatchNorm backward).
template <class T, class A>
__global__ __launch_bounds__(BN_THREADS) void k_bias_act_bwd(PtrTab ys, PtrTab dys, PtrTab dxs, int M, int C, int relu,
                                                             int rows_per_block, PtrTab parts) {
  const T* __restrict__ y = (const T*)pick(ys, blockIdx.z);
  const T* __restrict__ dy = (const T*)pick(dys, blockIdx.z);
  T* __restrict__ dx = (T*)pick(dxs, blockIdx.z);
  A* __restrict__ partials = (A*)pick(parts, blockIdx.z);
  __shared__ A sh[16][BN_THREADS];
  const BnMap m = bn_map(C);
  A s[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) s[j] = 0;
  if (m.active) {
    A v[8], d[8];
    const int r0 = blockIdx.x * rows_per_block;
    const int r1 = min(M, r0 + rows_per_block);
    for (int r = r0 + m.rl; r < r1; r += m.rpp) {
      const size_t o = (size_t)r * C + m.c0;
      load8t(y + o, v);
      load8t(dy + o, d);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const A dz = (!relu || v[j] > 0) ? d[j] : (A)0;
        s[j] += dz;
        d[j] = dz;
      }
      store8t(dx + o, d);
    }
  }
  block_reduce16(s, m, C, sh);
  if (m.active && m.rl == 0) {
    A* p = partials + ((size_t)blockIdx.x * C + m.c0) * 2;
#pragma unroll
    for (int j = 0; j < 8; ++j) { p[2 * j] = s[j]; p[2 * j + 1] = 0; }
  }
}

// 2x2 max-pool of stride 2.  One thread per output pixel and 8 channels.
template <class T>
__global__ __launch_bounds__(256) void k_maxpool2_fwd(PtrTab xs, PtrTab ys, int b, int h, int w, int C) {
  const T* __restrict__ x = (const T*)pick(xs, blockIdx.z);
  T* __restrict__ y = (T*)pick(ys, blockIdx.z);
  const int ho = h / 2, wo = w / 2, CG = C / 8;
  const size_t total = (size_t)b * ho * wo * CG;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const int cg = (int)(i % CG);
    const size_t px = i / CG;
    const int q = (int)(px % wo), p = (int)((px / wo) % ho), n = (int)(px / ((size_t)wo * ho));
    float best[8], v[8];
    load8(x + (((size_t)n * h + 2 * p) * w + 2 * q) * C + cg * 8, best);
#pragma unroll
    for (int t = 1; t < 4; ++t) {
      load8(x + (((size_t)n * h + 2 * p + (t >> 1)) * w + 2 * q + (t & 1)) * C + cg * 8, v);
#pragma unroll
      for (int j = 0; j < 8; ++j) best[j] = v[j] > best[j] ? v[j] : best[j];
    }
    store8(y + px * C + cg * 8, best);
  }
}
// The gradient of a window goes to its maximum; among equal maxima to the first in row-major order.
template <class T>
__global__ __launch_bounds__(256) void k_maxpool2_bwd(PtrTab xs, PtrTab dys, PtrTab dxs, int b, int h, int w, int C) {
  const T* __restrict__ x = (const T*)pick(xs, blockIdx.z);
  const T* __restrict__ dy = (const T*)pick(dys, blockIdx.z);
  T* __restrict__ dx = (T*)pick(dxs, blockIdx.z);
  const int ho = h / 2, wo = w / 2, CG = C / 8;
  const size_t total = (size_t)b * ho * wo * CG;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const int cg = (int)(i % CG);
    const size_t px = i / CG;
    const int q = (int)(px % wo), p = (int)((px / wo) % ho), n = (int)(px / ((size_t)wo * ho));
    float v[4][8], d[8], o[8];
    int arg[8];
#pragma unroll
    for (int t = 0; t < 4; ++t) load8(x + (((size_t)n * h + 2 * p + (t >> 1)) * w + 2 * q + (t & 1)) * C + cg * 8, v[t]);
    load8(dy + px * C + cg * 8, d);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float best = v[0][j];
      arg[j] = 0;
#pragma unroll
      for (int t = 1; t < 4; ++t)
        if (v[t][j] > best) { best = v[t][j]; arg[j] = t; }
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
#pragma unroll
      for (int j = 0; j < 8; ++j) o[j] = arg[j] == t ? d[j] : 0.f;
      store8(dx + (((size_t)n * h + 2 * p + (t >> 1)) * w + 2 * q + (t & 1)) * C + cg * 8, o);
    }
  }
}

// Residual join of a post-activation block: y = max(gamma*xhat + beta + add, 0).
template <class T, class A>
__global__ __launch_bounds__(BN_THREADS) void k_bn_add_relu_apply(PtrTab xs, PtrTab adds, PtrTab ys, const float* __restrict__ gamma,
                                                                  const float* __restrict__ beta, PtrTab statss, int M, int C) {
  const T* __restrict__ x = (const T*)pick(xs, blockIdx.z);
  const T* __restrict__ add = (const T*)pick(adds, blockIdx.z);
  T* __restrict__ y = (T*)pick(ys, blockIdx.z);
  const A* __restrict__ stats = (const A*)pick(statss, blockIdx.z);
  const BnMap m = bn_map(C);
  if (!m.active) return;
  A mu[8], is[8], g[8], bt[8], v[8], k[8];
  load8a(stats + m.c0, mu); load8a(stats + C + m.c0, is); load8t(gamma + m.c0, g); load8t(beta + m.c0, bt);
  for (int r = blockIdx.x * m.rpp + m.rl; r < M; r += gridDim.x * m.rpp) {
    const size_t o = (size_t)r * C + m.c0;
    load8t(x + o, v);
    load8t(add + o, k);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const A z = g[j] * ((v[j] - mu[j]) * is[j]) + bt[j] + k[j];
      v[j] = z > 0 ? z : (A)0;
    }
    store8t(y + o, v);
  }
}
// Its backward pass: dz = dy * [y > 0]; partial sums {sum dz, sum dz*xhat}.
template <class T, class A>
__global__ __launch_bounds__(BN_THREADS) void k_join_bwd_reduce(PtrTab xs, PtrTab ys, PtrTab dys, PtrTab statss, int M, int C,
                                                                int rows_per_block, PtrTab parts) {
  const T* __restrict__ x = (const T*)pick(xs, blockIdx.z);
  const T* __restrict__ y = (const T*)pick(ys, blockIdx.z);
  const T* __restrict__ dy = (const T*)pick(dys, blockIdx.z);
  const A* __restrict__ stats = (const A*)pick(statss, blockIdx.z);
  A* __restrict__ partials = (A*)pick(parts, blockIdx.z);
  __shared__ A sh[16][BN_THREADS];
  const BnMap m = bn_map(C);
  A s[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) s[j] = 0;
  if (m.active) {
    A mu[8], is[8], v[8], d[8], yy[8];
    load8a(stats + m.c0, mu); load8a(stats + C + m.c0, is);
    const int r0 = blockIdx.x * rows_per_block;
    const int r1 = min(M, r0 + rows_per_block);
    for (int r = r0 + m.rl; r < r1; r += m.rpp) {
      const size_t o = (size_t)r * C + m.c0;
      load8t(x + o, v);
      load8t(dy + o, d);
      load8t(y + o, yy);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const A dz = yy[j] > 0 ? d[j] : (A)0;
        s[j] += dz;
        s[8 + j] += dz * ((v[j] - mu[j]) * is[j]);
      }
    }
  }
  block_reduce16(s, m, C, sh);
  if (m.active && m.rl == 0) {
    A* p = partials + ((size_t)blockIdx.x * C + m.c0) * 2;
#pragma unroll
    for (int j = 0; j < 8; ++j) { p[2 * j] = s[j]; p[2 * j + 1] = s[8 + j]; }
  }
}
// dx = gamma*invstd*(dz - dbeta/M - xhat*dgamma/M) (frozen: gamma*invstd*dz) and dadd = dz for the shortcut.
template <class T, class A>
__global__ __launch_bounds__(BN_THREADS) void k_join_bwd_apply(PtrTab xs, PtrTab ys, PtrTab dys, const float* __restrict__ gamma,
                                                               PtrTab statss, PtrTab sumss, PtrTab dxs, PtrTab dadds, int M, int C,
                                                               int frozen) {
  const T* __restrict__ x = (const T*)pick(xs, blockIdx.z);
  const T* __restrict__ y = (const T*)pick(ys, blockIdx.z);
  const T* __restrict__ dy = (const T*)pick(dys, blockIdx.z);
  const A* __restrict__ stats = (const A*)pick(statss, blockIdx.z);
  const A* __restrict__ sums = (const A*)pick(sumss, blockIdx.z);
  T* __restrict__ dx = (T*)pick(dxs, blockIdx.z);
  T* __restrict__ dadd = (T*)pick(dadds, blockIdx.z);
  const BnMap m = bn_map(C);
  if (!m.active) return;
  A mu[8], is[8], g[8], sb[8], sg[8], v[8], d[8], yy[8];
  load8a(stats + m.c0, mu); load8a(stats + C + m.c0, is); load8t(gamma + m.c0, g);
  load8a(sums + m.c0, sb); load8a(sums + C + m.c0, sg);
  const A inv_m = frozen ? (A)0 : (A)1 / (A)M;
#pragma unroll
  for (int j = 0; j < 8; ++j) { sb[j] *= inv_m; sg[j] *= inv_m; }
  for (int r = blockIdx.x * m.rpp + m.rl; r < M; r += gridDim.x * m.rpp) {
    const size_t o = (size_t)r * C + m.c0;
    load8t(x + o, v);
    load8t(dy + o, d);
    load8t(y + o, yy);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const A xh = (v[j] - mu[j]) * is[j];
      const A dz = yy[j] > 0 ? d[j] : (A)0;
      v[j] = g[j] * is[j] * (dz - sb[j] - xh * sg[j]);
      d[j] = dz;
    }
    store8t(dx + o, v);
    store8t(dadd + o, d);
  }
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

size_t bn_partials_floats(int C) { return (size_t)BN_MAX_ROW_BLOCKS * C * 4 * 2; }  // 4 values, sized for double

static dim3 finw(int C, int ng) { return dim3((unsigned)((C + FINW_CH - 1) / FINW_CH), 1u, (unsigned)ng); }

hipError_t launch_bn_stats(int dt, int ng, const PtrTab& x, int M, int C, float eps, const PtrTab& stats,
                           const PtrTab& partials, hipStream_t stream) {
  const BnGrid g = reduce_grid(M, C);
  const dim3 grid(g.grid.x, g.grid.y, (unsigned)ng), fin((unsigned)((C + FIN_CH - 1) / FIN_CH), 1, (unsigned)ng);
  if (dt == DT_BF16) {
    k_bn_stats<bf16_t, float><<<grid, BN_THREADS, 0, stream>>>(x, M, C, g.rows_per_block, partials);
    k_bn_stats_finalize_wide<<<finw(C, ng), BN_THREADS, 0, stream>>>(M, C, g.grid.x, eps, partials, stats);
  } else {
    k_bn_stats<float, double><<<grid, BN_THREADS, 0, stream>>>(x, M, C, g.rows_per_block, partials);
    k_bn_stats_finalize<double><<<fin, BN_THREADS, 0, stream>>>(M, C, g.grid.x, eps, partials, stats);
  }
  return hipGetLastError();
}

// Finalize only: the partial records were written by a convolution epilogue (one record row per
// pixel-row tile).  float arithmetic (bf16 mode).
hipError_t launch_bn_stats_finalize(int ng, int M, int C, int nrows, float eps, const PtrTab& partials, const PtrTab& stats,
                                    hipStream_t stream) {
  k_bn_stats_finalize_wide<<<finw(C, ng), BN_THREADS, 0, stream>>>(M, C, (unsigned)nrows, eps, partials, stats);
  return hipGetLastError();
}

hipError_t launch_bn_bwd_finalize(int ng, int C, int nrows, const PtrTab& partials, const PtrTab& sums, float* g_gamma,
                                  float* g_beta, hipStream_t stream) {
  k_bn_bwd_finalize_wide<<<finw(C, ng), BN_THREADS, 0, stream>>>(C, (unsigned)nrows, partials, sums, g_gamma, g_beta);
  return hipGetLastError();
}

hipError_t launch_bn_apply_relu(int dt, int ng, const PtrTab& x, const PtrTab& a, const float* gamma, const float* beta,
                                const PtrTab& stats, int M, int C, hipStream_t stream) {
  dim3 grid = apply_grid(M, C);
  grid.z = (unsigned)ng;
  if (dt == DT_BF16)
    k_bn_apply_relu<bf16_t, float><<<grid, BN_THREADS, 0, stream>>>(x, a, gamma, beta, stats, M, C);
  else
    k_bn_apply_relu<float, double><<<grid, BN_THREADS, 0, stream>>>(x, a, gamma, beta, stats, M, C);
  return hipGetLastError();
}

hipError_t launch_bn_bwd_reduce(int dt, int ng, const PtrTab& x, const PtrTab& da, const float* gamma, const float* beta,
                                const PtrTab& stats, int M, int C, const PtrTab& sums, float* g_gamma, float* g_beta,
                                const PtrTab& partials, hipStream_t stream) {
  const BnGrid g = reduce_grid(M, C);
  const dim3 grid(g.grid.x, g.grid.y, (unsigned)ng), fin((unsigned)((C + FIN_CH - 1) / FIN_CH), 1, (unsigned)ng);
  if (dt == DT_BF16) {
    k_bn_bwd_reduce<bf16_t, float><<<grid, BN_THREADS, 0, stream>>>(x, da, gamma, beta, stats, M, C, g.rows_per_block, partials);
    k_bn_bwd_finalize_wide<<<finw(C, ng), BN_THREADS, 0, stream>>>(C, g.grid.x, partials, sums, g_gamma, g_beta);
  } else {
    k_bn_bwd_reduce<float, double><<<grid, BN_THREADS, 0, stream>>>(x, da, gamma, beta, stats, M, C, g.rows_per_block, partials);
    k_bn_bwd_finalize<double><<<fin, BN_THREADS, 0, stream>>>(C, g.grid.x, partials, sums, g_gamma, g_beta);
  }
  return hipGetLastError();
}

hipError_t launch_bn_bwd_apply(int dt, int ng, const PtrTab& x, const PtrTab& da, const float* gamma, const float* beta,
                               const PtrTab& stats, const PtrTab& sums, const PtrTab& skip, const PtrTab& dx, int M,
                               int C, int frozen, hipStream_t stream) {
  dim3 grid = apply_grid(M, C);
  grid.z = (unsigned)ng;
  if (dt == DT_BF16)
    k_bn_bwd_apply<bf16_t, float><<<grid, BN_THREADS, 0, stream>>>(x, da, gamma, beta, stats, sums, skip, dx, M, C, frozen);
  else
    k_bn_bwd_apply<float, double><<<grid, BN_THREADS, 0, stream>>>(x, da, gamma, beta, stats, sums, skip, dx, M, C, frozen);
  return hipGetLastError();
}

hipError_t launch_bn_frozen_stats(int dt, int ng, const PtrTab& stats, int C, float eps, hipStream_t stream) {
  const dim3 grid((unsigned)((C + 255) / 256), 1, (unsigned)ng);
  if (dt == DT_BF16) k_bn_frozen_stats<float><<<grid, 256, 0, stream>>>(stats, C, eps);
  else k_bn_frozen_stats<double><<<grid, 256, 0, stream>>>(stats, C, eps);
  return hipGetLastError();
}

hipError_t launch_bn_running_update(int dt, int ng, const PtrTab& bases, const BnRunDesc* table_dev, int n_bn, float* running,
                                    float momentum, float eps, hipStream_t stream) {
  if (n_bn <= 0) return hipSuccess;
  if (dt == DT_BF16) k_bn_running_update<float><<<n_bn, 256, 0, stream>>>(bases, table_dev, running, ng, momentum, eps);
  else k_bn_running_update<double><<<n_bn, 256, 0, stream>>>(bases, table_dev, running, ng, momentum, eps);
  return hipGetLastError();
}

hipError_t launch_bn_running_stats(int dt, int ng, const PtrTab& stats, const float* running_mean_var, int C, float eps,
                                   hipStream_t stream) {
  const dim3 grid((unsigned)((C + 255) / 256), 1, (unsigned)ng);
  if (dt == DT_BF16) k_bn_running_stats<float><<<grid, 256, 0, stream>>>(stats, running_mean_var, C, eps);
  else k_bn_running_stats<double><<<grid, 256, 0, stream>>>(stats, running_mean_var, C, eps);
  return hipGetLastError();
}

hipError_t launch_bias_act_fwd(int dt, int ng, const PtrTab& x, const PtrTab& y, const float* bias, int M, int C, int relu,
                               hipStream_t stream) {
  dim3 grid = apply_grid(M, C);
  grid.z = (unsigned)ng;
  if (dt == DT_BF16) k_bias_act_fwd<bf16_t, float><<<grid, BN_THREADS, 0, stream>>>(x, y, bias, M, C, relu);
  else k_bias_act_fwd<float, double><<<grid, BN_THREADS, 0, stream>>>(x, y, bias, M, C, relu);
  return hipGetLastError();
}

hipError_t launch_bias_act_bwd(int dt, int ng, const PtrTab& y, const PtrTab& dy, const PtrTab& dx, float* g_bias, int M, int C,
                               int relu, const PtrTab& sums, const PtrTab& partials, hipStream_t stream) {
  const BnGrid g = reduce_grid(M, C);
  const dim3 grid(g.grid.x, g.grid.y, (unsigned)ng), fin((unsigned)((C + FIN_CH - 1) / FIN_CH), 1, (unsigned)ng);
  if (dt == DT_BF16) {
    k_bias_act_bwd<bf16_t, float><<<grid, BN_THREADS, 0, stream>>>(y, dy, dx, M, C, relu, g.rows_per_block, partials);
    k_bn_bwd_finalize_wide<<<finw(C, ng), BN_THREADS, 0, stream>>>(C, g.grid.x, partials, sums, nullptr, g_bias);
  } else {
    k_bias_act_bwd<float, double><<<grid, BN_THREADS, 0, stream>>>(y, dy, dx, M, C, relu, g.rows_per_block, partials);
    k_bn_bwd_finalize<double><<<fin, BN_THREADS, 0, stream>>>(C, g.grid.x, partials, sums, nullptr, g_bias);
  }
  return hipGetLastError();
}

hipError_t launch_maxpool2_fwd(int dt, int ng, const PtrTab& x, const PtrTab& y, int b, int h, int w, int C, hipStream_t stream) {
  const size_t total = (size_t)b * (h / 2) * (w / 2) * (C / 8);
  const dim3 grid((unsigned)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096), 1, (unsigned)ng);
  if (dt == DT_BF16) k_maxpool2_fwd<bf16_t><<<grid, 256, 0, stream>>>(x, y, b, h, w, C);
  else k_maxpool2_fwd<float><<<grid, 256, 0, stream>>>(x, y, b, h, w, C);
  return hipGetLastError();
}

hipError_t launch_maxpool2_bwd(int dt, int ng, const PtrTab& x, const PtrTab& dy, const PtrTab& dx, int b, int h, int w, int C,
                               hipStream_t stream) {
  const size_t total = (size_t)b * (h / 2) * (w / 2) * (C / 8);
  const dim3 grid((unsigned)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096), 1, (unsigned)ng);
  if (dt == DT_BF16) k_maxpool2_bwd<bf16_t><<<grid, 256, 0, stream>>>(x, dy, dx, b, h, w, C);
  else k_maxpool2_bwd<float><<<grid, 256, 0, stream>>>(x, dy, dx, b, h, w, C);
  return hipGetLastError();
}

hipError_t launch_bn_add_relu_apply(int dt, int ng, const PtrTab& x, const PtrTab& add, const PtrTab& y, const float* gamma,
                                    const float* beta, const PtrTab& stats, int M, int C, hipStream_t stream) {
  dim3 grid = apply_grid(M, C);
  grid.z = (unsigned)ng;
  if (dt == DT_BF16) k_bn_add_relu_apply<bf16_t, float><<<grid, BN_THREADS, 0, stream>>>(x, add, y, gamma, beta, stats, M, C);
  else k_bn_add_relu_apply<float, double><<<grid, BN_THREADS, 0, stream>>>(x, add, y, gamma, beta, stats, M, C);
  return hipGetLastError();
}

hipError_t launch_join_bwd(int dt, int ng, const PtrTab& x, const PtrTab& y, const PtrTab& dy, const float* gamma, const PtrTab& stats,
                           int M, int C, const PtrTab& sums, float* g_gamma, float* g_beta, const PtrTab& partials, const PtrTab& dx,
                           const PtrTab& dadd, int frozen, hipStream_t stream) {
  const BnGrid g = reduce_grid(M, C);
  const dim3 grid(g.grid.x, g.grid.y, (unsigned)ng), fin((unsigned)((C + FIN_CH - 1) / FIN_CH), 1, (unsigned)ng);
  dim3 ag = apply_grid(M, C);
  ag.z = (unsigned)ng;
  if (dt == DT_BF16) {
    k_join_bwd_reduce<bf16_t, float><<<grid, BN_THREADS, 0, stream>>>(x, y, dy, stats, M, C, g.rows_per_block, partials);
    k_bn_bwd_finalize_wide<<<finw(C, ng), BN_THREADS, 0, stream>>>(C, g.grid.x, partials, sums, g_gamma, g_beta);
    k_join_bwd_apply<bf16_t, float><<<ag, BN_THREADS, 0, stream>>>(x, y, dy, gamma, stats, sums, dx, dadd, M, C, frozen);
  } else {
    k_join_bwd_reduce<float, double><<<grid, BN_THREADS, 0, stream>>>(x, y, dy, stats, M, C, g.rows_per_block, partials);
    k_bn_bwd_finalize<double><<<fin, BN_THREADS, 0, stream>>>(C, g.grid.x, partials, sums, g_gamma, g_beta);
    k_join_bwd_apply<float, double><<<ag, BN_THREADS, 0, stream>>>(x, y, dy, gamma, stats, sums, dx, dadd, M, C, frozen);
  }
  return hipGetLastError();
}

}  // namespace hpf
