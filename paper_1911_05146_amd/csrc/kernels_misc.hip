// Small kernels around the convolutions: stem im2col, classification head (global average pool,
// FC, softmax cross-entropy -- the loss of the last partition, paper Eq. 1-2), SGD with momentum
// (apply_gradients), weight packing for the MFMA operands, fills and copies.
#include "hpf_device.h"

namespace hpf {
namespace {

// col[m, k] for k = (r*3+s)*Cin + c, zero for taps outside the image and for k >= 9*Cin.
__global__ __launch_bounds__(256) void k_im2col3x3(PtrTab imgs, PtrTab cols, int b, int H, int W, int Cin, int Kc) {
  const float* __restrict__ img = (const float*)pick(imgs, blockIdx.z);
  bf16_t* __restrict__ col = (bf16_t*)pick(cols, blockIdx.z);
  const size_t total = (size_t)b * H * W * Kc;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const int k = (int)(i % Kc);
    const size_t m = i / Kc;
    const int q = (int)(m % W);
    const int p = (int)((m / W) % H);
    const int n = (int)(m / ((size_t)W * H));
    float v = 0.f;
    if (k < 9 * Cin) {
      const int tap = k / Cin, c = k - tap * Cin;
      const int hi = p + tap / 3 - 1, wi = q + tap % 3 - 1;
      if ((unsigned)hi < (unsigned)H && (unsigned)wi < (unsigned)W) v = img[(((size_t)n * H + hi) * W + wi) * Cin + c];
    }
    col[i] = f32_to_bf16(v);
  }
}

__device__ __forceinline__ float block_reduce_max(float v, float* sh) {
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = sh[0];
  for (int w = 1; w < (int)(blockDim.x >> 6); ++w) r = fmaxf(r, sh[w]);
  __syncthreads();
  return r;
}

__device__ __forceinline__ float block_reduce_sum(float v, float* sh) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = sh[0];
  for (int w = 1; w < (int)(blockDim.x >> 6); ++w) r += sh[w];
  __syncthreads();
  return r;
}

// logits[j] = bias[j] + sum_c gs[c] * W[c][j] for one sample, all 256 threads at work whatever the class count: the
// threads form CS slices over the channels x JT class lanes (JT = the power of two that covers min(classes, 256)),
// every thread sums its channel slice for its classes and the slices are added in a fixed order through LDS.
// part: 256 floats of LDS.  Ends with a barrier; lg[0 .. classes) is then complete.
__device__ __forceinline__ void fc_logits(const float* gs, const float* __restrict__ wfc, const float* __restrict__ bfc, float* lg, float* part,
                                          int C, int classes) {
  if (classes <= 16) {
    // few classes (the benchmark heads have 10): every thread takes channels tid, tid + 256, ... for all classes -- its
    // loads are independent of each other (consecutive threads read consecutive weight rows) and in flight together,
    // where a thread per (class, channel slice) walked C/16 dependent steps; sums by wave shuffles, then over the 4 waves
    float acc[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[j] = 0.f;
    for (int c = threadIdx.x; c < C; c += 256) {
      const float gv = gs[c];
      const float* wr = wfc + (size_t)c * classes;
#pragma unroll
      for (int j = 0; j < 16; ++j)
        if (j < classes) acc[j] = fmaf(gv, wr[j], acc[j]);
    }
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      float v = acc[j];
      for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
      if ((threadIdx.x & 63) == 0) part[(threadIdx.x >> 6) * 16 + j] = v;
    }
    __syncthreads();
    if ((int)threadIdx.x < classes) lg[threadIdx.x] = bfc[threadIdx.x] + ((part[threadIdx.x] + part[16 + threadIdx.x]) + (part[32 + threadIdx.x] + part[48 + threadIdx.x]));
    __syncthreads();
    return;
  }
  int jt = 1;
  while (jt < classes && jt < 256) jt <<= 1;
  const int cs_n = 256 / jt, jl = threadIdx.x % jt, cs = threadIdx.x / jt;
  for (int j0 = 0; j0 < classes; j0 += jt) {
    const int j = j0 + jl;
    float s = 0.f;
    if (j < classes)
      for (int c = cs; c < C; c += cs_n) s = fmaf(gs[c], wfc[(size_t)c * classes + j], s);
    part[cs * jt + jl] = s;
    __syncthreads();
    if (cs == 0 && j < classes) {
      float t = bfc[j];
      for (int k = 0; k < cs_n; ++k) t += part[k * jt + jl];
      lg[j] = t;
    }
    __syncthreads();
  }
}

// One block per sample.  Dynamic LDS: C + classes floats.
template <class T>
__global__ __launch_bounds__(256) void k_head_fwd(PtrTab as, const float* __restrict__ wfc, const float* __restrict__ bfc,
                                                  PtrTab labelss, PtrTab gs_, PtrTab dls, float* loss_accum, int hw, int C,
                                                  int classes, float inv_div) {
  const T* __restrict__ a = (const T*)pick(as, blockIdx.z);
  const int32_t* __restrict__ labels = (const int32_t*)pick(labelss, blockIdx.z);
  float* __restrict__ g = (float*)pick(gs_, blockIdx.z);
  float* __restrict__ dlogits = (float*)pick(dls, blockIdx.z);
  extern __shared__ float dyn[];
  __shared__ float red[8];
  __shared__ float part[256];
  float* gs = dyn;
  float* lg = dyn + C;
  const int n = blockIdx.x;
  const T* an = a + (size_t)n * hw * C;
  const float inv_hw = 1.0f / (float)hw;
  for (int c = threadIdx.x; c < C; c += blockDim.x) {
    float s = 0.f;
    for (int i = 0; i < hw; ++i) s += to_f32(an[(size_t)i * C + c]);
    s *= inv_hw;
    gs[c] = s;
    g[(size_t)n * C + c] = s;
  }
  __syncthreads();
  fc_logits(gs, wfc, bfc, lg, part, C, classes);
  float mx = -3.0e38f;
  for (int j = threadIdx.x; j < classes; j += blockDim.x) mx = fmaxf(mx, lg[j]);
  mx = block_reduce_max(mx, red);
  float den = 0.f;
  for (int j = threadIdx.x; j < classes; j += blockDim.x) den += expf(lg[j] - mx);
  den = block_reduce_sum(den, red);
  const int y = labels[n];
  for (int j = threadIdx.x; j < classes; j += blockDim.x)
    dlogits[(size_t)n * classes + j] = (expf(lg[j] - mx) / den - (j == y ? 1.f : 0.f)) * inv_div;
  if (threadIdx.x == 0) atomicAdd(loss_accum, -(lg[y] - mx - logf(den)) * inv_div);
}

// Inference head, one block per sample: logits = mean_{h,w}(a) * Wfc + bfc.  Dynamic LDS: C + classes floats.
template <class T>
__global__ __launch_bounds__(256) void k_head_logits(PtrTab as, const float* __restrict__ wfc, const float* __restrict__ bfc,
                                                     PtrTab outs, int hw, int C, int classes) {
  const T* __restrict__ a = (const T*)pick(as, blockIdx.z);
  float* __restrict__ out = (float*)pick(outs, blockIdx.z);
  extern __shared__ float dyn[];
  __shared__ float part[256];
  float* gs = dyn;
  float* lg = dyn + C;
  const int n = blockIdx.x;
  const T* an = a + (size_t)n * hw * C;
  const float inv_hw = 1.0f / (float)hw;
  for (int c = threadIdx.x; c < C; c += blockDim.x) {
    float s = 0.f;
    for (int i = 0; i < hw; ++i) s += to_f32(an[(size_t)i * C + c]);
    gs[c] = s * inv_hw;
  }
  __syncthreads();
  fc_logits(gs, wfc, bfc, lg, part, C, classes);
  for (int j = threadIdx.x; j < classes; j += blockDim.x) out[(size_t)n * classes + j] = lg[j];
}

// dWfc[c][j] += sum over the samples of all members of g[n][c] * dlogits[n][j]: a thread per output element walks the
// samples (one atomic per element and launch; a block per sample adding its outer product cost b*g atomics per element).
// Dynamic LDS: ng * b * classes floats (the dlogits of the launch).
__global__ __launch_bounds__(256) void k_head_wgrad(PtrTab gs_, PtrTab dls, float* g_wfc, int ng, int b, int C, int classes) {
  extern __shared__ float sdl[];
  for (int z = 0; z < ng; ++z) {
    const float* __restrict__ dl = (const float*)pick(dls, z);
    for (int i = threadIdx.x; i < b * classes; i += 256) sdl[z * b * classes + i] = dl[i];
  }
  __syncthreads();
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= C * classes) return;
  const int c = i / classes, j = i - c * classes;
  float s = 0.f;
  for (int z = 0; z < ng; ++z) {
    const float* __restrict__ g = (const float*)pick(gs_, z);
    for (int n = 0; n < b; ++n) s = fmaf(g[(size_t)n * C + c], sdl[(z * b + n) * classes + j], s);
  }
  atomicAdd(&g_wfc[i], s);
}

// One block per sample: dbfc += dlogits, da[n,i,c] = (dlogits[n] . Wfc[c]) / hw (dWfc: k_head_wgrad).
template <class T>
__global__ __launch_bounds__(256) void k_head_bwd(PtrTab gs_, PtrTab dls, const float* __restrict__ wfc, float* g_wfc,
                                                  float* g_bfc, PtrTab das, int hw, int C, int classes) {
  (void)gs_; (void)g_wfc;
  const float* __restrict__ dlogits = (const float*)pick(dls, blockIdx.z);
  T* __restrict__ da = (T*)pick(das, blockIdx.z);
  extern __shared__ float dyn[];
  float* dl = dyn;          // classes
  float* dg = dyn + classes;  // C
  const int n = blockIdx.x;
  for (int j = threadIdx.x; j < classes; j += blockDim.x) {
    const float d = dlogits[(size_t)n * classes + j];
    dl[j] = d;
    atomicAdd(&g_bfc[j], d);
  }
  __syncthreads();
  const float inv_hw = 1.0f / (float)hw;
  for (int c = threadIdx.x; c < C; c += blockDim.x) {
    float s = 0.f;
    for (int j = 0; j < classes; ++j) s = fmaf(dl[j], wfc[(size_t)c * classes + j], s);
    dg[c] = s * inv_hw;
  }
  __syncthreads();
  T* dan = da + (size_t)n * hw * C;
  for (int i = threadIdx.x; i < hw * C; i += blockDim.x) from_f32(&dan[i], dg[i % C]);
}

// invalid (may be null): set when the batch's gradients are not to be trusted (an image-resident launch gave up
// waiting for its partners); the step then leaves parameters, momentum and gradients alone.
__global__ __launch_bounds__(256) void k_sgd(float* __restrict__ w, float* __restrict__ v, float* __restrict__ g,
                                             size_t n, float lr, float mu, const int* __restrict__ invalid) {
  if (invalid && *invalid) return;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
    const float vel = fmaf(mu, v[i], g[i]);
    v[i] = vel;
    w[i] = fmaf(-lr, vel, w[i]);
    g[i] = 0.f;
  }
}

__global__ __launch_bounds__(256) void k_zero_f32(float* __restrict__ p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0.f;
}

// Every work-group copies contiguous 16 KiB chunks (four 16-byte units per lane in flight) with streaming
// loads and stores: measured 5.6-5.9 TB/s on 1 GiB, against 4.2-4.6 TB/s for a grid-stride loop over the
// whole buffer and 4.8 TB/s for the runtime's device-to-device copy.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr size_t COPY_CHUNK = 1024;   // 16-byte units per work-group and step
__global__ __launch_bounds__(256) void k_copy16(u32x4* __restrict__ dst, const u32x4* __restrict__ src, size_t n16,
                                                unsigned char* dtail, const unsigned char* stail, int ntail) {
  for (size_t c0 = (size_t)blockIdx.x * COPY_CHUNK; c0 < n16; c0 += (size_t)gridDim.x * COPY_CHUNK) {
    const size_t i = c0 + threadIdx.x;
    if (c0 + COPY_CHUNK <= n16) {
      u32x4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(src + i + u * 256);
#pragma unroll
      for (int u = 0; u < 4; ++u) __builtin_nontemporal_store(v[u], dst + i + u * 256);
    } else {
      for (size_t j = i; j < n16; j += 256) dst[j] = src[j];
    }
  }
  if (blockIdx.x == 0 && (int)threadIdx.x < ntail) dtail[threadIdx.x] = stail[threadIdx.x];
}

// grid (n_convs, Y): the Y blocks of conv i share its work round-robin.  The forward copy is a transpose of the
// fp32 master ([k][n] -> [n][k]), done in 64 x 64 tiles through LDS so that both the reads and the writes are
// contiguous; the data-gradient copy keeps n contiguous and is a flat loop.
__global__ __launch_bounds__(256) void k_pack_weights(const float* __restrict__ params, bf16_t* __restrict__ packed,
                                                      const PackDesc* __restrict__ table) {
  __shared__ float tile[64][65];
  const PackDesc d = table[blockIdx.x];
  const float* w = params + d.w_off;
  {
    bf16_t* wf = packed + d.wf_off;  // [Cout][Kf], k = tap*Cin + c
    const int ktot = d.T * d.Cin;
    const int tk = (d.Kf + 63) / 64, tn = (d.Cout + 63) / 64;
    const int lx = threadIdx.x & 63, ly = threadIdx.x >> 6;
    const bool wide = d.Cout % 4 == 0 && d.Kf % 8 == 0 && d.w_off % 4 == 0 && d.wf_off % 8 == 0;   // 16-byte loads along n and 16-byte stores along k
    for (int t = blockIdx.y; t < tk * tn; t += gridDim.y) {
      const int k0 = (t / tn) * 64, n0 = (t % tn) * 64;
      __syncthreads();
      if (wide) {
        // load: a thread takes 4 consecutive n of one k row (16 lanes per row, 16 rows per pass)
        const int c4 = (threadIdx.x & 15) * 4, r0 = threadIdx.x >> 4;
#pragma unroll
        for (int r = r0; r < 64; r += 16) {
          const int k = k0 + r, n = n0 + c4;
          float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
          if (k < ktot && n < d.Cout) v = *reinterpret_cast<const float4*>(w + (size_t)k * d.Cout + n);
          tile[r][c4] = v.x; tile[r][c4 + 1] = v.y; tile[r][c4 + 2] = v.z; tile[r][c4 + 3] = v.w;
        }
        __syncthreads();
        // store: a thread takes 8 consecutive k of one n row (8 lanes per row, 32 rows per pass)
        const int k8 = (threadIdx.x & 7) * 8, nr0 = threadIdx.x >> 3;
#pragma unroll
        for (int r = nr0; r < 64; r += 32) {
          const int n = n0 + r, k = k0 + k8;
          if (n < d.Cout && k < d.Kf) {
            uint4 st;
            st.x = pack_bf16x2(tile[k8][r], tile[k8 + 1][r]); st.y = pack_bf16x2(tile[k8 + 2][r], tile[k8 + 3][r]);
            st.z = pack_bf16x2(tile[k8 + 4][r], tile[k8 + 5][r]); st.w = pack_bf16x2(tile[k8 + 6][r], tile[k8 + 7][r]);
            *reinterpret_cast<uint4*>(wf + (size_t)n * d.Kf + k) = st;
          }
        }
        continue;
      }
#pragma unroll 4
      for (int r = ly; r < 64; r += 4) {
        const int k = k0 + r, n = n0 + lx;
        tile[r][lx] = (k < ktot && n < d.Cout) ? w[(size_t)k * d.Cout + n] : 0.f;
      }
      __syncthreads();
#pragma unroll 4
      for (int r = ly; r < 64; r += 4) {
        const int n = n0 + r, k = k0 + lx;
        if (n < d.Cout && k < d.Kf) wf[(size_t)n * d.Kf + k] = f32_to_bf16(tile[lx][r]);
      }
    }
  }
  if (d.wd_off != ~0ull) {
    bf16_t* wd = packed + d.wd_off;  // [Cin][Kd], k = tap*Cout + n
    const int ktot = d.T * d.Cout;
    if (d.Cout % 2 == 0 && d.Kd % 2 == 0 && d.w_off % 2 == 0 && d.wd_off % 2 == 0) {   // pairs of n: 8-byte loads, 4-byte stores, no divisions
      uint32_t* wd2 = reinterpret_cast<uint32_t*>(wd);
      const int half = d.Cout >> 1, kd2 = d.Kd >> 1;
      for (int c = blockIdx.y; c < d.Cin; c += gridDim.y) {
        for (int tap = 0; tap < d.T; ++tap) {
          const float* src = w + ((size_t)tap * d.Cin + c) * d.Cout;
          for (int n2 = threadIdx.x; n2 < half; n2 += 256) {
            const float2 v = *reinterpret_cast<const float2*>(src + 2 * n2);
            wd2[(size_t)c * kd2 + tap * half + n2] = pack_bf16x2(v.x, v.y);
          }
        }
        for (int k2 = (ktot >> 1) + threadIdx.x; k2 < kd2; k2 += 256) wd2[(size_t)c * kd2 + k2] = 0u;   // padding
      }
    } else {
      const int total = d.Cin * d.Kd;
      for (int i = blockIdx.y * 256 + threadIdx.x; i < total; i += gridDim.y * 256) {
        const int c = i / d.Kd, k = i - c * d.Kd;
        float v = 0.f;
        if (k < ktot) {
          const int tap = k / d.Cout, n = k - tap * d.Cout;
          v = w[((size_t)tap * d.Cin + c) * d.Cout + n];
        }
        wd[i] = f32_to_bf16(v);
      }
    }
  }
}

unsigned grid_for(size_t n, unsigned cap = 2048) {
  size_t g = (n + 255) / 256;
  if (g < 1) g = 1;
  return (unsigned)(g > cap ? cap : g);
}

}  // namespace

hipError_t launch_im2col3x3(int ng, const PtrTab& img, const PtrTab& col, int b, int H, int W, int Cin, int Kc,
                            hipStream_t stream) {
  k_im2col3x3<<<dim3(grid_for((size_t)b * H * W * Kc), 1, (unsigned)ng), 256, 0, stream>>>(img, col, b, H, W, Cin, Kc);
  return hipGetLastError();
}

hipError_t launch_head_fwd(int dt, int ng, const PtrTab& a, const float* wfc, const float* bfc, const PtrTab& labels,
                           const PtrTab& gp, const PtrTab& dlogits, float* loss_accum, int b, int hw, int C,
                           int classes, float divisor, hipStream_t stream) {
  const size_t lds = (size_t)(C + classes) * sizeof(float);
  const dim3 grid((unsigned)b, 1, (unsigned)ng);
  if (dt == DT_BF16)
    k_head_fwd<bf16_t><<<grid, 256, lds, stream>>>(a, wfc, bfc, labels, gp, dlogits, loss_accum, hw, C, classes, 1.0f / divisor);
  else
    k_head_fwd<float><<<grid, 256, lds, stream>>>(a, wfc, bfc, labels, gp, dlogits, loss_accum, hw, C, classes, 1.0f / divisor);
  return hipGetLastError();
}

hipError_t launch_head_logits(int dt, int ng, const PtrTab& a, const float* wfc, const float* bfc, const PtrTab& logits, int b,
                              int hw, int C, int classes, hipStream_t stream) {
  const size_t lds = (size_t)(C + classes) * sizeof(float);
  const dim3 grid((unsigned)b, 1, (unsigned)ng);
  if (dt == DT_BF16) k_head_logits<bf16_t><<<grid, 256, lds, stream>>>(a, wfc, bfc, logits, hw, C, classes);
  else k_head_logits<float><<<grid, 256, lds, stream>>>(a, wfc, bfc, logits, hw, C, classes);
  return hipGetLastError();
}

hipError_t launch_head_bwd(int dt, int ng, const PtrTab& gp, const PtrTab& dlogits, const float* wfc, float* g_wfc,
                           float* g_bfc, const PtrTab& da, int b, int hw, int C, int classes, hipStream_t stream) {
  const size_t lds = (size_t)(C + classes) * sizeof(float);
  const dim3 grid((unsigned)b, 1, (unsigned)ng);
  if (dt == DT_BF16)
    k_head_bwd<bf16_t><<<grid, 256, lds, stream>>>(gp, dlogits, wfc, g_wfc, g_bfc, da, hw, C, classes);
  else
    k_head_bwd<float><<<grid, 256, lds, stream>>>(gp, dlogits, wfc, g_wfc, g_bfc, da, hw, C, classes);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const size_t wl = (size_t)ng * b * classes * sizeof(float);
  if (wl > 48 * 1024) return hipErrorInvalidValue;
  k_head_wgrad<<<dim3((unsigned)(((size_t)C * classes + 255) / 256)), 256, wl, stream>>>(gp, dlogits, g_wfc, ng, b, C, classes);
  return hipGetLastError();
}

hipError_t launch_sgd(float* w, float* v, float* g, size_t n, float lr, float mu, const int* invalid, hipStream_t stream) {
  k_sgd<<<grid_for(n, 4096), 256, 0, stream>>>(w, v, g, n, lr, mu, invalid);
  return hipGetLastError();
}

hipError_t launch_zero_f32(float* p, size_t n, hipStream_t stream) {
  k_zero_f32<<<grid_for(n, 4096), 256, 0, stream>>>(p, n);
  return hipGetLastError();
}

hipError_t launch_pack_weights(const float* params, bf16_t* packed, const PackDesc* table_dev, int n_convs, size_t max_elems,
                               hipStream_t stream) {
  if (n_convs <= 0) return hipSuccess;
  // blocks per convolution: one per 8192 elements of the largest one (blocks with nothing to do leave at once)
  size_t y = (max_elems + 8191) / 8192;
  y = y < 8 ? 8 : (y > 1024 ? 1024 : y);
  k_pack_weights<<<dim3((unsigned)n_convs, (unsigned)y), 256, 0, stream>>>(params, packed, table_dev);
  return hipGetLastError();
}

// Register-only MFMA loops: independent accumulator tiles per wave, `iters` rounds of one MFMA on each.  No
// memory traffic inside the loop; the sums are written once so that the loop cannot be dropped.  The MFMA is
// written as an in-place accumulate (the builtin in this loop shape made the compiler rotate the accumulators
// through ~70 register moves per round, which measured the moves, not the matrix unit).
// WIDE = false: 8 tiles of v_mfma_f32_16x16x32_bf16; WIDE = true: 4 tiles of v_mfma_f32_32x32x16_bf16 (twice the
// flop per instruction): 131 072 flop per round and wave either way.
template <bool WIDE>
__global__ __launch_bounds__(256) void k_probe_mfma_bf16(float* __restrict__ sink, int iters) {
  typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
  typedef float floatx4 __attribute__((ext_vector_type(4)));
  typedef float floatx16 __attribute__((ext_vector_type(16)));
  const uint32_t seed = 0x3f803f80u + ((threadIdx.x & 7u) << 16);   // bf16 pairs near 1.0
  const bf16x8 a = __builtin_bit_cast(bf16x8, make_uint4(seed, seed ^ 0x00010000u, seed, seed ^ 0x00000001u));
  const bf16x8 b = __builtin_bit_cast(bf16x8, make_uint4(seed ^ 0x80000000u, seed, seed ^ 0x00008000u, seed));
  float t = 0.f;
  if (WIDE) {
    floatx16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 4; ++i) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[i]) : "v"(a), "v"(b));
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) t += acc[i][e];
  } else {
    floatx4 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 8; ++i) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc[i]) : "v"(a), "v"(b));
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) t += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
  }
  sink[(size_t)blockIdx.x * 256 + threadIdx.x] = t;
}

hipError_t launch_probe_mfma_bf16(float* sink, int workgroups, int iters, bool wide, hipStream_t stream) {
  if (wide) k_probe_mfma_bf16<true><<<workgroups, 256, 0, stream>>>(sink, iters);
  else k_probe_mfma_bf16<false><<<workgroups, 256, 0, stream>>>(sink, iters);
  return hipGetLastError();
}

hipError_t launch_copy_bytes(void* dst, const void* src, size_t bytes, hipStream_t stream) {
  const size_t n16 = bytes / 16;
  const int ntail = (int)(bytes - n16 * 16);
  const size_t chunks = (n16 + COPY_CHUNK - 1) / COPY_CHUNK;
  const unsigned grid = (unsigned)(chunks < 1 ? 1 : chunks > (1u << 20) ? (1u << 20) : chunks);
  k_copy16<<<grid, 256, 0, stream>>>((u32x4*)dst, (const u32x4*)src, n16, (unsigned char*)dst + n16 * 16,
                                                    (const unsigned char*)src + n16 * 16, ntail);
  return hipGetLastError();
}

}  // namespace hpf
