// Implicit-GEMM convolution forward and data-gradient on bf16 MFMA (v_mfma_f32_16x16x32_bf16),
// fp32 accumulation, NHWC tiles staged through LDS.
//
// Both passes are the same gather-GEMM
//     out[m, n] = sum_k W[n, k] * src[row(m, tap(k)), c(k)],      k = tap*Cs + c,
// with the reduction index k running over (filter tap, source channel).  The packed weights are
// [N][Kpad] (k contiguous), the source tensor is NHWC, so for a fixed pixel row 8 consecutive k are
// 16 contiguous bytes of one source pixel (Cs is a multiple of 8): the im2col matrix is never
// materialised, each LDS-staging thread decodes (tap, c) for its 16-byte unit and either loads the
// source pixel or writes zeros (padding, stride holes of the data-gradient, K padding).
//
// MFMA orientation: the weight tile is the first operand (rows = output channels) and the pixel
// tile the second (columns = pixels), so each lane ends up with 4 consecutive output channels of
// one pixel: the epilogue stores (and reads the optional residual) 8 bytes per lane, and the 4
// lane groups of a wave cover 16 consecutive channels = 32 contiguous bytes per pixel.
//
// Work-group: 256 threads = 4 waves arranged WR x WC over a BM (pixels) x BN (channels) tile;
// K advances 32 per step (one MFMA), double-buffered in LDS with one barrier per step and the
// next step's global loads in flight during the MFMAs.
#include <mutex>

#include "hpf_device.h"

namespace hpf {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int KC = 32;          // reduction elements per step
constexpr size_t BIG_MAX_LDS = 128 * 1024;   // dynamic LDS limit set for the 128 x 128 x 64 kernels (stages + coefficients)
constexpr int LSTR = KC + 8;    // LDS row stride in bf16 (80 bytes: conflict-free 16-byte reads)

// relu(bn(x)) of the 8 bf16 values in q, channels c..c+7 (c a multiple of 8); coef holds per channel
// {scale = gamma*invstd, shift = beta - mean*scale}, so the operand is max(x*scale + shift, 0).
__device__ __forceinline__ uint4 bn_relu_unit(const uint4& q, const float2* coef, int c) {
  const uint32_t w[4] = {q.x, q.y, q.z, q.w};
  const float4* cf = reinterpret_cast<const float4*>(coef + c);   // two channels per 16-byte read
  uint32_t r[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float4 k = cf[i];
    const float x0 = __uint_as_float(w[i] << 16), x1 = __uint_as_float(w[i] & 0xffff0000u);
    r[i] = pack_bf16x2(fmaxf(fmaf(x0, k.x, k.y), 0.f), fmaxf(fmaf(x1, k.z, k.w), 0.f));
  }
  return make_uint4(r[0], r[1], r[2], r[3]);
}

// Epilogue of a BM x BN tile whose accumulators are spread over WR x WC waves (wave (wr, wc) holds pixel rows
// wr*PT*16.. and channels wc*CT*16..): residual add, bf16 store, and the optional per-channel sums (statistics of
// the stored values, or BatchNorm-backward sums) written as one partial record per tile row and channel.
// `scratch` is LDS that no wave reads as operand storage any more: BN + WR*BN*2 floats; tile_row is the index of
// the tile's partial record.
template <int BM, int BN, int WR, int WC, int PT, int CT, int EPI>
__device__ __forceinline__ void conv_epilogue(floatx4 (&acc)[CT][PT], int wr, int wc, int tile_row, int row0, int ch0, float* scratch,
                                              const ConvGeom& g, const ConvEpi& epi, const bf16_t* add, bf16_t* out) {
  constexpr int WPX = PT * 16, WCH = CT * 16;
  static_assert(WR * WPX == BM && WC * WCH == BN, "wave grid covers the tile");
  const int tid = threadIdx.x, lane = tid & 63;
  // acc[i][j][v]: channel = ch0 + wc*WCH + i*16 + (lane>>4)*4 + v, pixel row = row0 + wr*WPX + j*16 + (lane&15)
  // Epilogue scratch in the (now idle) staging LDS: shift per channel and per-wave-row sums.
  float* sK = scratch;                                     // [BN]
  float* sS = sK + BN;                                     // [WR][BN][2]
  float s1[CT][4], s2[CT][4];
#pragma unroll
  for (int i = 0; i < CT; ++i)
#pragma unroll
    for (int v = 0; v < 4; ++v) { s1[i][v] = 0.f; s2[i][v] = 0.f; }

  // per-channel BN constants of this lane's channels (EPI_BNBWD), loaded once
  float mu_[CT][4], is_[CT][4], ga_[CT][4], be_[CT][4];
  if (EPI == EPI_BNBWD) {
    const float* stt = (const float*)pick(epi.stats, blockIdx.z);
#pragma unroll
    for (int i = 0; i < CT; ++i) {
      const int ch = ch0 + wc * WCH + i * 16 + (lane >> 4) * 4;
      const float4 mu = *reinterpret_cast<const float4*>(stt + ch);
      const float4 is = *reinterpret_cast<const float4*>(stt + g.N + ch);
      const float4 ga = *reinterpret_cast<const float4*>(epi.gamma + ch);
      const float4 be = *reinterpret_cast<const float4*>(epi.beta + ch);
      mu_[i][0] = mu.x; mu_[i][1] = mu.y; mu_[i][2] = mu.z; mu_[i][3] = mu.w;
      is_[i][0] = is.x; is_[i][1] = is.y; is_[i][2] = is.z; is_[i][3] = is.w;
      ga_[i][0] = ga.x; ga_[i][1] = ga.y; ga_[i][2] = ga.z; ga_[i][3] = ga.w;
      be_[i][0] = be.x; be_[i][1] = be.y; be_[i][2] = be.z; be_[i][3] = be.w;
    }
  }

#pragma unroll
  for (int j = 0; j < PT; ++j) {
    const int m = row0 + wr * WPX + j * 16 + (lane & 15);
    const bool mv = m < g.M;
#pragma unroll
    for (int i = 0; i < CT; ++i) {
      const int chl = wc * WCH + i * 16 + (lane >> 4) * 4;
      const int ch = ch0 + chl;
      const size_t o = (size_t)(mv ? m : 0) * g.N + ch;
      float vv[4] = {acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]};
      if (add && mv) {
        const uint2 t = *reinterpret_cast<const uint2*>(add + o);
        vv[0] += __uint_as_float(t.x << 16); vv[1] += __uint_as_float(t.x & 0xffff0000u);
        vv[2] += __uint_as_float(t.y << 16); vv[3] += __uint_as_float(t.y & 0xffff0000u);
      }
      uint2 st;
      st.x = pack_bf16x2(vv[0], vv[1]);
      st.y = pack_bf16x2(vv[2], vv[3]);
      if (EPI != EPI_NONE) {   // continue with the values as stored
        vv[0] = __uint_as_float(st.x << 16); vv[1] = __uint_as_float(st.x & 0xffff0000u);
        vv[2] = __uint_as_float(st.y << 16); vv[3] = __uint_as_float(st.y & 0xffff0000u);
      }
      if (EPI == EPI_BNBWD) {
        if (mv) {
          const bf16_t* xt = (const bf16_t*)pick(epi.x, blockIdx.z);
          const uint2 xr = *reinterpret_cast<const uint2*>(xt + o);
          const float xv[4] = {__uint_as_float(xr.x << 16), __uint_as_float(xr.x & 0xffff0000u),
                               __uint_as_float(xr.y << 16), __uint_as_float(xr.y & 0xffff0000u)};
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const float xh = (xv[v] - mu_[i][v]) * is_[i][v];
            const float z = ga_[i][v] * xh + be_[i][v];
            const float dz = z > 0.f ? vv[v] : 0.f;
            vv[v] = dz;
            s1[i][v] += dz;
            s2[i][v] += dz * xh;
          }
          st.x = pack_bf16x2(vv[0], vv[1]);   // exact: dz is a stored value or 0
          st.y = pack_bf16x2(vv[2], vv[3]);
        }
      }
      if (EPI == EPI_STATS) {
        if (j == 0 && wr == 0 && (lane & 15) == 0) {   // the tile's first row gives the shift
#pragma unroll
          for (int v = 0; v < 4; ++v) sK[chl + v] = vv[v];
        }
        // keep the stored values for the second pass over the registers
        acc[i][j][0] = vv[0]; acc[i][j][1] = vv[1]; acc[i][j][2] = vv[2]; acc[i][j][3] = vv[3];
      }
      if (mv) *reinterpret_cast<uint2*>(out + o) = st;
    }
  }
  if (EPI == EPI_NONE) return;

  if (EPI == EPI_STATS) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < CT; ++i) {
      const int chl = wc * WCH + i * 16 + (lane >> 4) * 4;
      const float4 k4 = *reinterpret_cast<const float4*>(sK + chl);
      const float k_[4] = {k4.x, k4.y, k4.z, k4.w};
#pragma unroll
      for (int j = 0; j < PT; ++j) {
        const int m = row0 + wr * WPX + j * 16 + (lane & 15);
        if (m < g.M) {
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const float d = acc[i][j][v] - k_[v];
            s1[i][v] += d;
            s2[i][v] += d * d;
          }
        }
      }
    }
  }
  // sum over the 16 pixel lanes of each lane group, then over the wave rows through LDS (fixed order)
#pragma unroll
  for (int i = 0; i < CT; ++i)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) {
        s1[i][v] += __shfl_xor(s1[i][v], o);
        s2[i][v] += __shfl_xor(s2[i][v], o);
      }
    }
  if ((lane & 15) == 0) {
#pragma unroll
    for (int i = 0; i < CT; ++i) {
      const int chl = wc * WCH + i * 16 + (lane >> 4) * 4;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        sS[(wr * BN + chl + v) * 2] = s1[i][v];
        sS[(wr * BN + chl + v) * 2 + 1] = s2[i][v];
      }
    }
  }
  __syncthreads();
  if (tid < BN) {
    float a1 = 0.f, a2 = 0.f;
#pragma unroll
    for (int w = 0; w < WR; ++w) { a1 += sS[(w * BN + tid) * 2]; a2 += sS[(w * BN + tid) * 2 + 1]; }
    float* part = (float*)pick(epi.partials, blockIdx.z);
    if (EPI == EPI_STATS) {
      const int nrows = min(BM, g.M - row0);
      *reinterpret_cast<float4*>(part + ((size_t)tile_row * g.N + ch0 + tid) * 4) = make_float4(sK[tid], a1, a2, (float)nrows);
    } else {
      *reinterpret_cast<float2*>(part + ((size_t)tile_row * g.N + ch0 + tid) * 2) = make_float2(a1, a2);
    }
  }
}

template <int BM, int BN, int WR, int WC, int MODE, int EPI, int PRO>
__global__ __launch_bounds__(256) void k_conv_mfma(PtrTab srcs, const bf16_t* __restrict__ wpk, PtrTab outs, PtrTab adds,
                                                   ConvGeom g, ConvEpi epi, ConvPro pro) {
  extern __shared__ float2 coef[];   // PRO: per source channel {scale, shift}
  const bf16_t* __restrict__ src = (const bf16_t*)pick(srcs, blockIdx.z);
  bf16_t* out = (bf16_t*)pick(outs, blockIdx.z);
  const bf16_t* add = (const bf16_t*)pick(adds, blockIdx.z);
  static_assert(WR * WC == 4, "4 waves");
  constexpr int WPX = BM / WR, WCH = BN / WC, PT = WPX / 16, CT = WCH / 16;
  static_assert(PT >= 1 && CT >= 1, "tile too small");
  constexpr int A_UNITS = (BM * 4) / 256;
  static_assert(A_UNITS >= 1, "BM >= 64");
  constexpr int W_UNITS = (BN * 4 + 255) / 256;

  __shared__ __attribute__((aligned(16))) bf16_t sA[2][BM * LSTR];
  __shared__ __attribute__((aligned(16))) bf16_t sW[2][BN * LSTR];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave / WC, wc = wave % WC;
  const int row0 = blockIdx.x * BM, ch0 = blockIdx.y * BN;
  const int grp = tid & 3;
  const int HoWo = g.Ho * g.Wo;
  const int sshift = g.stride - 1;  // stride is 1 or 2

  int a_img[A_UNITS], a_h[A_UNITS], a_w[A_UNITS];
  bool a_ok[A_UNITS];
#pragma unroll
  for (int u = 0; u < A_UNITS; ++u) {
    const int m = row0 + (tid >> 2) + u * 64;
    a_ok[u] = m < g.M;
    const int mm = a_ok[u] ? m : 0;
    const int img = mm / HoWo;
    const int rem = mm - img * HoWo;
    const int p = rem / g.Wo, q = rem - p * g.Wo;
    a_img[u] = img * g.Hs * g.Ws;
    if (MODE == CONV_FWD) { a_h[u] = p * g.stride - g.pad; a_w[u] = q * g.stride - g.pad; }
    else { a_h[u] = p + g.pad; a_w[u] = q + g.pad; }
  }

  // NPRE chunks are kept in flight in registers: at these sizes a work-group lives for a handful of
  // K steps only, so what matters is how many global loads are outstanding, not the MFMA rate.
  constexpr int NPRE = 4;
  struct Slot { uint4 a[A_UNITS]; uint4 w[W_UNITS]; int c; bool av[A_UNITS]; };
  Slot sl0, sl1, sl2, sl3;   // named, not an array: they must stay in registers
  if (PRO) {
    const float* stt = (const float*)pick(pro.stats, blockIdx.z);
    for (int c = tid; c < g.Cs; c += 256) {
      const float sc = pro.gamma[c] * stt[g.Cs + c];
      coef[c] = make_float2(sc, pro.beta[c] - stt[c] * sc);
    }
    __syncthreads();
  }

  // (filter tap row, tap column, channel) of this thread's 16-byte unit in the chunk that is loaded
  // next; chunks are loaded in order, so the position advances by KC channels per load (no divisions)
  int lk = grp * 8, lr, ls, lc;
  {
    const int tap = lk / g.Cs;
    lc = lk - tap * g.Cs;
    lr = tap / g.R;
    ls = tap - lr * g.R;
  }
  auto load_chunk = [&](int kc, Slot& q) {
    uint4 (&qa)[A_UNITS] = q.a;
    uint4 (&qw)[W_UNITS] = q.w;
    const int c = lc, r = lr, s = ls;
    const bool kvalid = lk < g.Ktot;
    lk += KC; lc += KC;
    while (lc >= g.Cs) { lc -= g.Cs; if (++ls == g.R) { ls = 0; ++lr; } }
    q.c = c;
#pragma unroll
    for (int u = 0; u < A_UNITS; ++u) {
      int hs, ws;
      bool v = a_ok[u] && kvalid;
      if (MODE == CONV_FWD) {
        hs = a_h[u] + r; ws = a_w[u] + s;
      } else {
        const int th = a_h[u] - r, tw = a_w[u] - s;
        v = v && th >= 0 && tw >= 0 && (((th | tw) & sshift) == 0);
        hs = th >> sshift; ws = tw >> sshift;
      }
      v = v && (unsigned)hs < (unsigned)g.Hs && (unsigned)ws < (unsigned)g.Ws;
      q.av[u] = v;
      qa[u] = v ? *reinterpret_cast<const uint4*>(src + (size_t)(a_img[u] + hs * g.Ws + ws) * g.Cs + c)
                : make_uint4(0u, 0u, 0u, 0u);
    }
#pragma unroll
    for (int u = 0; u < W_UNITS; ++u) {
      const int unit = tid + u * 256;
      if (unit < BN * 4)
        qw[u] = *reinterpret_cast<const uint4*>(wpk + (size_t)(ch0 + (unit >> 2)) * g.Kpad + kc * KC + (unit & 3) * 8);
    }
  };
  auto store_chunk = [&](int buf, const Slot& q) {
    const uint4 (&qa)[A_UNITS] = q.a;
    const uint4 (&qw)[W_UNITS] = q.w;
#pragma unroll
    for (int u = 0; u < A_UNITS; ++u) {
      uint4 val = qa[u];
      if (PRO) { if (q.av[u]) val = bn_relu_unit(val, coef, q.c); }
      *reinterpret_cast<uint4*>(&sA[buf][((tid >> 2) + u * 64) * LSTR + grp * 8]) = val;
    }
#pragma unroll
    for (int u = 0; u < W_UNITS; ++u) {
      const int unit = tid + u * 256;
      if (unit < BN * 4) *reinterpret_cast<uint4*>(&sW[buf][(unit >> 2) * LSTR + (unit & 3) * 8]) = qw[u];
    }
  };

  floatx4 acc[CT][PT];
#pragma unroll
  for (int i = 0; i < CT; ++i)
#pragma unroll
    for (int j = 0; j < PT; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};

  const int nk = g.Kpad / KC;
  load_chunk(0, sl0);
  if (1 < nk) load_chunk(1, sl1);
  if (2 < nk) load_chunk(2, sl2);
  if (3 < nk) load_chunk(3, sl3);
  store_chunk(0, sl0);
  __syncthreads();
  const int frag_row = lane & 15, frag_k = (lane >> 4) * 8;
  // one K step: chunk kc is in LDS buffer kc&1 and its register slot `cur` is free again
  auto step = [&](int kc, Slot& cur, const Slot& nxt) {
    if (kc >= nk) return;
    const int buf = kc & 1;
    if (kc + NPRE < nk) load_chunk(kc + NPRE, cur);
    bf16x8 fa[PT], fw[CT];
#pragma unroll
    for (int j = 0; j < PT; ++j)
      fa[j] = *reinterpret_cast<const bf16x8*>(&sA[buf][(wr * WPX + j * 16 + frag_row) * LSTR + frag_k]);
#pragma unroll
    for (int i = 0; i < CT; ++i)
      fw[i] = *reinterpret_cast<const bf16x8*>(&sW[buf][(wc * WCH + i * 16 + frag_row) * LSTR + frag_k]);
#pragma unroll
    for (int i = 0; i < CT; ++i)
#pragma unroll
      for (int j = 0; j < PT; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fw[i], fa[j], acc[i][j], 0, 0, 0);
    if (kc + 1 < nk) store_chunk(buf ^ 1, nxt);
    __syncthreads();
  };
  for (int kc0 = 0; kc0 < nk; kc0 += NPRE) {
    step(kc0, sl0, sl1);
    step(kc0 + 1, sl1, sl2);
    step(kc0 + 2, sl2, sl3);
    step(kc0 + 3, sl3, sl0);
  }

  static_assert((BN + WR * BN * 2) * 4 <= (int)sizeof(sA), "epilogue scratch fits the staging buffer");
  conv_epilogue<BM, BN, WR, WC, PT, CT, EPI>(acc, wr, wc, blockIdx.x, row0, ch0, reinterpret_cast<float*>(&sA[0][0]), g, epi, add, out);
}

// ---- long reductions on wide tensors ---------------------------------------------------------------------
// 128 x 128 tile, 8 waves, 64 reduction elements per step, three LDS stages.  The waves form two groups of 2 x 2: both groups take
// the same 64 x 64 quadrants, group 0 over the first and group 1 over the second 32 reduction elements of every
// step, so each SIMD holds two waves (one hides the other's LDS and barrier waits) while every operand fragment
// is still read from LDS once.  At the end the groups exchange half of their sums through LDS: group 0 ends
// up with pixel rows 0..31 of each quadrant, group 1 with rows 32..63, and the epilogue sees a 4 x 2 wave grid.
// Needs Cs % 64 == 0 (a step stays within one filter tap, so tap and padding are decided per pixel row, not per
// 16-byte unit) and Kpad % 64 == 0.
constexpr int BIG_T = 128, BIG_K = 64, BIG_LS = BIG_K + 8;   // LDS rows of 144 bytes: 16-byte reads of 16 rows hit 16 bank groups
constexpr int BIG_STAGE = 2 * BIG_T * BIG_LS;                // bf16 elements per stage (pixel tile, then weight tile)
constexpr int BIG_OPERAND_BYTES = 3 * BIG_STAGE * 2;         // three stages

// SPLIT: grid y = number of work-groups that share a reduction; each takes a contiguous range of the steps and
// stores its fp32 partial tile into its slab of the member's buffer epi.splitk_ws (k_splitk_finish adds the slabs up): for long reductions
// into few output tiles (VGG-16's 512 -> 512 convolutions on 4x4 and 2x2 pixels: 32-64 tiles, 72 steps).
template <int MODE, int EPI, int PRO, bool SPLIT = false>
__global__ __launch_bounds__(512) void k_conv_big(PtrTab srcs, const bf16_t* __restrict__ wpk, PtrTab outs, PtrTab adds, ConvGeom g,
                                                  ConvEpi epi, ConvPro pro) {
  static_assert(!SPLIT || (EPI == EPI_NONE && PRO == 0), "partial sums leave the kernel as they are");
  extern __shared__ __attribute__((aligned(16))) unsigned char big_smem[];
  bf16_t* stage = reinterpret_cast<bf16_t*>(big_smem);
  float2* coef = reinterpret_cast<float2*>(big_smem + BIG_OPERAND_BYTES);   // PRO: per source channel {scale, shift}
  const bf16_t* __restrict__ src = (const bf16_t*)pick(srcs, blockIdx.z);
  bf16_t* out = (bf16_t*)pick(outs, blockIdx.z);
  const bf16_t* add = (const bf16_t*)pick(adds, blockIdx.z);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kh = wave >> 2, wr = (wave >> 1) & 1, wc = wave & 1;
  // Work-groups go to the 8 XCDs (each with its own L2) round-robin by index.  Tiles are numbered with the channel
  // tile fastest and every XCD takes a contiguous range of them: the work-groups that share a pixel tile run on one
  // XCD at the same time, and each XCD reads only its share of the source tensor.
  const int n_nt = g.N / BIG_T, tiles = ((g.M + BIG_T - 1) / BIG_T) * n_nt, per_xcd = (tiles + 7) >> 3;
  const int q = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (q >= tiles) return;              // the whole work-group, before any barrier
  const int mt = q / n_nt;
  const int row0 = mt * BIG_T, ch0 = (q - mt * n_nt) * BIG_T;
  const int grp = tid & 7;             // 16-byte unit within the 128-byte row of a step
  const int HoWo = g.Ho * g.Wo;
  const int sshift = g.stride - 1;     // stride is 1 or 2

  // staging: rows (tid >> 3) and (tid >> 3) + 64 of both tiles
  int a_img[2], a_h[2], a_w[2];
  bool a_ok[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int m = row0 + (tid >> 3) + u * 64;
    a_ok[u] = m < g.M;
    const int mm = a_ok[u] ? m : 0;
    const int img = mm / HoWo;
    const int rem = mm - img * HoWo;
    const int p = rem / g.Wo, q = rem - p * g.Wo;
    a_img[u] = img * g.Hs * g.Ws;
    if (MODE == CONV_FWD) { a_h[u] = p * g.stride - g.pad; a_w[u] = q * g.stride - g.pad; }
    else { a_h[u] = p + g.pad; a_w[u] = q + g.pad; }
  }
  if (PRO) {
    const float* stt = (const float*)pick(pro.stats, blockIdx.z);
    for (int c = tid; c < g.Cs; c += 512) {
      const float sc = pro.gamma[c] * stt[g.Cs + c];
      coef[c] = make_float2(sc, pro.beta[c] - stt[c] * sc);
    }
    __syncthreads();
  }

  // Two or three steps of global loads stay in flight, in registers.  Every step issues the same four loads
  // unconditionally (rows outside the image or the tensor read a clamped address and are zeroed when they are
  // stored to LDS; past the last step the last one is loaded again), so the counter of outstanding loads is known
  // at every wait and a wait for the oldest step never drains the younger ones.
  struct Slot { uint4 a[2]; uint4 w[2]; int c; bool av[2]; };
  Slot sl0, sl1, sl2;
  const int nk_all = g.Kpad / BIG_K;
  const int k_begin = SPLIT ? (int)((long)blockIdx.y * nk_all / gridDim.y) : 0;
  const int nk = SPLIT ? (int)((long)(blockIdx.y + 1) * nk_all / gridDim.y) - k_begin : nk_all;   // this work-group's steps
  int lk = 0, lc = 0, lr = 0, ls = 0;  // index, channel base and filter tap of the step that is loaded next (uniform)
  if (SPLIT) {
    const int tap = (k_begin * BIG_K) / g.Cs;
    lc = k_begin * BIG_K - tap * g.Cs; lr = tap / g.R; ls = tap - lr * g.R;
  }
  const bf16_t* wrow = wpk + (size_t)(ch0 + (tid >> 3)) * g.Kpad + grp * 8 + (size_t)k_begin * BIG_K;   // second unit: 64 rows further (uniform offset)
  auto load_chunk = [&](Slot& q) {
    const int cb = lc, c = cb + grp * 8, r = lr, s = ls, kc = lk;
    if (lk + 1 < nk) {                 // state only: no loads under this branch
      ++lk; lc += BIG_K;
      if (lc >= g.Cs) { lc = 0; if (++ls == g.R) { ls = 0; ++lr; } }
    }
    q.c = cb;                          // uniform: the lane's channels are q.c + grp*8
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      int hs, ws;
      bool v = a_ok[u];
      if (MODE == CONV_FWD) {
        hs = a_h[u] + r; ws = a_w[u] + s;
      } else {
        const int th = a_h[u] - r, tw = a_w[u] - s;
        v = v && th >= 0 && tw >= 0 && (((th | tw) & sshift) == 0);
        hs = th >> sshift; ws = tw >> sshift;
      }
      v = v && (unsigned)hs < (unsigned)g.Hs && (unsigned)ws < (unsigned)g.Ws;
      q.av[u] = v;
      const size_t off = v ? (size_t)(a_img[u] + hs * g.Ws + ws) * g.Cs + c : (size_t)c;
      q.a[u] = *reinterpret_cast<const uint4*>(src + off);
      q.w[u] = *reinterpret_cast<const uint4*>(wrow + (size_t)u * 64 * g.Kpad + kc * BIG_K);
    }
  };
  auto store_chunk = [&](int st, const Slot& q) {
    bf16_t* sA = stage + st * BIG_STAGE;
    bf16_t* sW = sA + BIG_T * BIG_LS;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      uint4 val = q.a[u];
      if (PRO) val = bn_relu_unit(val, coef, q.c + grp * 8);
      if (!q.av[u]) val = make_uint4(0u, 0u, 0u, 0u);
      *reinterpret_cast<uint4*>(&sA[((tid >> 3) + u * 64) * BIG_LS + grp * 8]) = val;
      *reinterpret_cast<uint4*>(&sW[((tid >> 3) + u * 64) * BIG_LS + grp * 8]) = q.w[u];
    }
  };

  floatx4 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};

  // Three LDS stages.  During step kc the waves multiply the fragments of chunk kc (in registers since the step
  // before), read the fragments of chunk kc+1 (complete in LDS since the last barrier) into the second register
  // set, and write chunk kc+2 from its register slot to the third stage; the slot then takes the loads of a later
  // chunk.  LDS reads, LDS writes, global loads and MFMAs of a step are independent of each other, so they overlap
  // within a wave, and one barrier per step orders the stages.
  struct Frags { bf16x8 a[4], w[4]; };
  const int frag_off_a = (wr * 64 + (lane & 15)) * BIG_LS + kh * 32 + (lane >> 4) * 8;
  const int frag_off_w = BIG_T * BIG_LS + (wc * 64 + (lane & 15)) * BIG_LS + kh * 32 + (lane >> 4) * 8;
  auto read_frags = [&](int st, Frags& f) {
    const bf16_t* base = stage + st * BIG_STAGE;
#pragma unroll
    for (int j = 0; j < 4; ++j) f.a[j] = *reinterpret_cast<const bf16x8*>(&base[frag_off_a + j * 16 * BIG_LS]);
#pragma unroll
    for (int i = 0; i < 4; ++i) f.w[i] = *reinterpret_cast<const bf16x8*>(&base[frag_off_w + i * 16 * BIG_LS]);
  };
  constexpr int NS = PRO ? 2 : 3;      // register slots: with the BatchNorm prologue registers are short
  load_chunk(sl0);
  load_chunk(sl1);
  if (NS == 3) load_chunk(sl2);
  store_chunk(0, sl0);
  load_chunk(sl0);                     // chunk 3 (chunk 2 with two slots)
  store_chunk(1, sl1);
  load_chunk(sl1);                     // chunk 4 (chunk 3)
  __syncthreads();
  Frags f0, f1;
  read_frags(0, f0);
  // st = kc % 3 (stage of chunk kc); `slot` holds chunk kc+2 and then takes the loads of chunk kc+2+NS
  auto step = [&](int st, Slot& slot, const Frags& cur, Frags& nxt) {
    const int st1 = st == 2 ? 0 : st + 1, st2 = st == 0 ? 2 : st - 1;
    read_frags(st1, nxt);
    store_chunk(st2, slot);            // past the last chunk: a copy of the last one, in a stage that nobody reads
    load_chunk(slot);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cur.w[i], cur.a[j], acc[i][j], 0, 0, 0);
    __syncthreads();
  };
  int kc0 = 0;
  if (NS == 3) {
    for (; kc0 + 6 <= nk; kc0 += 6) {
      step(0, sl2, f0, f1);
      step(1, sl0, f1, f0);
      step(2, sl1, f0, f1);
      step(0, sl2, f1, f0);
      step(1, sl0, f0, f1);
      step(2, sl1, f1, f0);
    }
    if (kc0 + 0 < nk) step(0, sl2, f0, f1);
    if (kc0 + 1 < nk) step(1, sl0, f1, f0);
    if (kc0 + 2 < nk) step(2, sl1, f0, f1);
    if (kc0 + 3 < nk) step(0, sl2, f1, f0);
    if (kc0 + 4 < nk) step(1, sl0, f0, f1);
  } else {
    for (; kc0 + 6 <= nk; kc0 += 6) {
      step(0, sl0, f0, f1);
      step(1, sl1, f1, f0);
      step(2, sl0, f0, f1);
      step(0, sl1, f1, f0);
      step(1, sl0, f0, f1);
      step(2, sl1, f1, f0);
    }
    if (kc0 + 0 < nk) step(0, sl0, f0, f1);
    if (kc0 + 1 < nk) step(1, sl1, f1, f0);
    if (kc0 + 2 < nk) step(2, sl0, f0, f1);
    if (kc0 + 3 < nk) step(0, sl1, f1, f0);
    if (kc0 + 4 < nk) step(1, sl0, f0, f1);
  }

  // Epilogue through LDS (all operand reads are behind the last barrier, so the stages are free): group 1 writes
  // its sums into an fp32 tile [128 pixels][128 channels], group 0 adds its own, and then every thread takes
  // (pixel row, 8 consecutive channels) units, so that 16 lanes cover the 256 contiguous bytes of a row in the
  // residual read, the BatchNorm-input read and the store.
  constexpr int TS = BIG_T + 4;        // fp32 row stride: rows shift by 4 banks
  float* tile = reinterpret_cast<float*>(big_smem);
  float* sK = tile + BIG_T * TS;       // [128] shift per channel (EPI_STATS)
  float* sS = sK + BIG_T;              // [32 row groups][128 channels][2]
  static_assert((BIG_T * TS + BIG_T + 32 * BIG_T * 2) * 4 <= BIG_OPERAND_BYTES, "epilogue tile and sums fit the stages");
  {
    float* t0 = tile + (wr * 64 + (lane & 15)) * TS + wc * 64 + (lane >> 4) * 4;
    if (kh == 1) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) *reinterpret_cast<floatx4*>(t0 + j * 16 * TS + i * 16) = acc[i][j];
    }
    __syncthreads();
    if (kh == 0) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          floatx4* t = reinterpret_cast<floatx4*>(t0 + j * 16 * TS + i * 16);
          *t = *t + acc[i][j];
        }
    }
    __syncthreads();
  }
  const int cg = tid & 15, rg = tid >> 4;      // channels ch0 + cg*8 .. +8, rows rg + 32*u
  const int ch = ch0 + cg * 8;
  float vals[4][8];
  float s1[8], s2[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { s1[e] = 0.f; s2[e] = 0.f; }
  float mu_[8], is_[8], ga_[8], be_[8];
  if (EPI == EPI_BNBWD) {
    const float* stt = (const float*)pick(epi.stats, blockIdx.z);
    load8(stt + ch, mu_); load8(stt + g.N + ch, is_); load8(epi.gamma + ch, ga_); load8(epi.beta + ch, be_);
  }
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int rl = rg + 32 * u, m = row0 + rl;
    const bool mv = m < g.M;
    const size_t o = (size_t)(mv ? m : 0) * g.N + ch;
    float (&vv)[8] = vals[u];
    load8(tile + rl * TS + cg * 8, vv);
    if (SPLIT) {
      if (mv) {
        float* o4 = (float*)pick(epi.splitk_ws, blockIdx.z) + ((size_t)blockIdx.y * g.M + m) * g.N + ch;
        *reinterpret_cast<float4*>(o4) = make_float4(vv[0], vv[1], vv[2], vv[3]);
        *reinterpret_cast<float4*>(o4 + 4) = make_float4(vv[4], vv[5], vv[6], vv[7]);
      }
      continue;
    }
    if (add) {
      float rv[8];
      load8(add + o, rv);
#pragma unroll
      for (int e = 0; e < 8; ++e) vv[e] += rv[e];
    }
    uint4 st;
    st.x = pack_bf16x2(vv[0], vv[1]); st.y = pack_bf16x2(vv[2], vv[3]);
    st.z = pack_bf16x2(vv[4], vv[5]); st.w = pack_bf16x2(vv[6], vv[7]);
    if (EPI != EPI_NONE) {             // continue with the values as stored
      const uint32_t w[4] = {st.x, st.y, st.z, st.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) { vv[2 * e] = __uint_as_float(w[e] << 16); vv[2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u); }
    }
    if (EPI == EPI_BNBWD) {
      float xv[8];
      load8((const bf16_t*)pick(epi.x, blockIdx.z) + o, xv);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float xh = (xv[e] - mu_[e]) * is_[e];
        const float z = ga_[e] * xh + be_[e];
        const float dz = (mv && z > 0.f) ? vv[e] : 0.f;
        vv[e] = dz;
        s1[e] += dz;
        s2[e] += dz * xh;
      }
      st.x = pack_bf16x2(vv[0], vv[1]); st.y = pack_bf16x2(vv[2], vv[3]);   // exact: dz is a stored value or 0
      st.z = pack_bf16x2(vv[4], vv[5]); st.w = pack_bf16x2(vv[6], vv[7]);
    }
    if (EPI == EPI_STATS && rl == 0) {   // the tile's first row gives the shift
#pragma unroll
      for (int e = 0; e < 8; ++e) sK[cg * 8 + e] = vv[e];
    }
    if (mv) *reinterpret_cast<uint4*>(out + o) = st;
  }
  if (EPI == EPI_NONE) return;
  if (EPI == EPI_STATS) {
    __syncthreads();
    float k_[8];
    load8(sK + cg * 8, k_);
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (row0 + rg + 32 * u < g.M) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float d = vals[u][e] - k_[e];
          s1[e] += d;
          s2[e] += d * d;
        }
      }
  }
  // sums over the 32 row groups through LDS, in a fixed order
#pragma unroll
  for (int e = 0; e < 8; ++e) *reinterpret_cast<float2*>(&sS[(rg * BIG_T + cg * 8 + e) * 2]) = make_float2(s1[e], s2[e]);
  __syncthreads();
  if (tid < BIG_T) {
    float a1 = 0.f, a2 = 0.f;
#pragma unroll 8
    for (int r = 0; r < 32; ++r) {
      const float2 t = *reinterpret_cast<const float2*>(&sS[(r * BIG_T + tid) * 2]);
      a1 += t.x; a2 += t.y;
    }
    float* part = (float*)pick(epi.partials, blockIdx.z);
    if (EPI == EPI_STATS) {
      const int nrows = min(BIG_T, g.M - row0);
      *reinterpret_cast<float4*>(part + ((size_t)mt * g.N + ch0 + tid) * 4) = make_float4(sK[tid], a1, a2, (float)nrows);
    } else {
      *reinterpret_cast<float2*>(part + ((size_t)mt * g.N + ch0 + tid) * 2) = make_float2(a1, a2);
    }
  }
}

// out[z][m][n] = bf16(sum over the slabs of the fp32 partial sums); 8 elements per thread
__global__ __launch_bounds__(256) void k_splitk_finish(PtrTab wss, PtrTab outs, int splits, size_t mn) {
  const size_t u = (size_t)blockIdx.x * 256 + threadIdx.x;   // unit of 8 elements within a member
  const int z = blockIdx.y;
  if (u * 8 >= mn) return;
  const float* __restrict__ ws = (const float*)pick(wss, z);
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < splits; ++s) {
    const float4* q = reinterpret_cast<const float4*>(ws + (size_t)s * mn + u * 8);
    const float4 a = q[0], b = q[1];
    acc[0] += a.x; acc[1] += a.y; acc[2] += a.z; acc[3] += a.w;
    acc[4] += b.x; acc[5] += b.y; acc[6] += b.z; acc[7] += b.w;
  }
  uint4 st;
  st.x = pack_bf16x2(acc[0], acc[1]); st.y = pack_bf16x2(acc[2], acc[3]);
  st.z = pack_bf16x2(acc[4], acc[5]); st.w = pack_bf16x2(acc[6], acc[7]);
  *reinterpret_cast<uint4*>((bf16_t*)pick(outs, z) + u * 8) = st;
}

bool big_tile_fits(const ConvGeom& g) { return g.N % BIG_T == 0 && g.Cs % BIG_K == 0 && g.Kpad % BIG_K == 0 && g.Kpad == g.Ktot; }

// Reductions of at least 16 steps into so few tiles that half of the CUs would idle are split over up to four
// work-groups (each keeps at least 8 steps).
int big_splits(int ng, const ConvGeom& g) {
  const long wgs = (long)((g.M + BIG_T - 1) / BIG_T) * (g.N / BIG_T) * ng;
  const int nk = g.Kpad / BIG_K;
  if (nk < 16 || wgs > 128) return 1;
  int s = (int)(256 / wgs);
  if (s > 4) s = 4;
  if (s > nk / 8) s = nk / 8;
  return s < 2 ? 1 : s;
}

hipError_t launch_big(int mode, int ng, const PtrTab& src, const bf16_t* wpk, const PtrTab& out, const PtrTab& add, const ConvGeom& g,
                      hipStream_t stream, const ConvEpi& epi, const ConvPro& pro) {
  const int tiles = ((g.M + BIG_T - 1) / BIG_T) * (g.N / BIG_T);
  const size_t dyn = BIG_OPERAND_BYTES + (pro.on ? (size_t)g.Cs * sizeof(float2) : 0);
  if (dyn > BIG_MAX_LDS) return hipErrorInvalidValue;
  const int splits = (epi.kind == EPI_NONE && !pro.on && add.p[0] == nullptr && epi.splitk_floats) ? big_splits(ng, g) : 1;
  if (splits > 1 && (size_t)splits * g.M * g.N <= epi.splitk_floats) {
    const dim3 sgrid((unsigned)(8 * ((tiles + 7) / 8)), (unsigned)splits, (unsigned)ng);
    if (mode == CONV_FWD) k_conv_big<CONV_FWD, EPI_NONE, 0, true><<<sgrid, 512, dyn, stream>>>(src, wpk, out, add, g, epi, pro);
    else k_conv_big<CONV_DGRAD, EPI_NONE, 0, true><<<sgrid, 512, dyn, stream>>>(src, wpk, out, add, g, epi, pro);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t mn = (size_t)g.M * g.N;   // a multiple of 128
    k_splitk_finish<<<dim3((unsigned)((mn / 8 + 255) / 256), (unsigned)ng), 256, 0, stream>>>(epi.splitk_ws, out, splits, mn);
    return hipGetLastError();
  }
  const dim3 grid((unsigned)(8 * ((tiles + 7) / 8)), 1u, (unsigned)ng);
#define HPF_CONV(MODE_, EPI_, PRO_) k_conv_big<MODE_, EPI_, PRO_><<<grid, 512, dyn, stream>>>(src, wpk, out, add, g, epi, pro)
  if (mode == CONV_FWD) {
    if (epi.kind == EPI_STATS) { if (pro.on) HPF_CONV(CONV_FWD, EPI_STATS, 1); else HPF_CONV(CONV_FWD, EPI_STATS, 0); }
    else if (epi.kind == EPI_NONE) { if (pro.on) HPF_CONV(CONV_FWD, EPI_NONE, 1); else HPF_CONV(CONV_FWD, EPI_NONE, 0); }
    else return hipErrorInvalidValue;
  } else {
    if (pro.on) return hipErrorInvalidValue;
    if (epi.kind == EPI_BNBWD) HPF_CONV(CONV_DGRAD, EPI_BNBWD, 0);
    else if (epi.kind == EPI_NONE) HPF_CONV(CONV_DGRAD, EPI_NONE, 0);
    else return hipErrorInvalidValue;
  }
#undef HPF_CONV
  return hipGetLastError();
}

template <int BM, int BN, int WR, int WC>
hipError_t launch_tile(int mode, int ng, const PtrTab& src, const bf16_t* wpk, const PtrTab& out, const PtrTab& add,
                       const ConvGeom& g, hipStream_t stream, const ConvEpi& epi, const ConvPro& pro) {
  const dim3 grid((unsigned)((g.M + BM - 1) / BM), (unsigned)(g.N / BN), (unsigned)ng);
  const size_t dyn = pro.on ? (size_t)g.Cs * sizeof(float2) : 0;
#define HPF_CONV(MODE_, EPI_, PRO_) \
  k_conv_mfma<BM, BN, WR, WC, MODE_, EPI_, PRO_><<<grid, 256, dyn, stream>>>(src, wpk, out, add, g, epi, pro)
  if (mode == CONV_FWD) {
    if (epi.kind == EPI_STATS) { if (pro.on) HPF_CONV(CONV_FWD, EPI_STATS, 1); else HPF_CONV(CONV_FWD, EPI_STATS, 0); }
    else if (epi.kind == EPI_NONE) { if (pro.on) HPF_CONV(CONV_FWD, EPI_NONE, 1); else HPF_CONV(CONV_FWD, EPI_NONE, 0); }
    else return hipErrorInvalidValue;
  } else {
    if (pro.on) return hipErrorInvalidValue;
    if (epi.kind == EPI_BNBWD) HPF_CONV(CONV_DGRAD, EPI_BNBWD, 0);
    else if (epi.kind == EPI_NONE) HPF_CONV(CONV_DGRAD, EPI_NONE, 0);
    else return hipErrorInvalidValue;
  }
#undef HPF_CONV
  return hipGetLastError();
}

// 0: 128x128, 1: 64x64, 2: 64x32, 3: 64x16, 4: 128x128 with 64-element steps on 8 waves
constexpr int BIG_MIN_K = 256;        // reductions from here on count as wide for the choice of what is written to memory
// The 8-wave tile pays a fixed 8 us per work-group (pipeline fill, epilogue through LDS) and runs one work-group
// per CU: with four reduction steps (K = 256) the 64x64 tiles, five work-groups per CU, are faster (1x1 256 -> 1024
// on 12 544 rows: 22.8 us against 27.8 us); from eight steps on the wide tile wins (K = 512: 11.6 against 14.7 us).
constexpr int BIG_MIN_K_TILE = 512;
int pick_tile(int ng, const ConvGeom& g) {
  if (big_tile_fits(g) && g.Kpad >= BIG_MIN_K_TILE) return 4;
  // the 128x128 tile pays off through operand reuse over a long reduction; short reductions are
  // latency bound and want many small work-groups
  if (g.N % 128 == 0 && g.Kpad >= 512) {
    const long wgs = (long)((g.M + 127) / 128) * (g.N / 128) * ng;
    if (wgs >= 512) return 0;   // at least two work-groups per CU, else the smaller tile hides latency better
  }
  if (g.N % 64 == 0) return 1;
  if (g.N % 32 == 0) return 2;
  return 3;
}

}  // namespace

int conv_mfma_tile_rows(int ng, const ConvGeom& g) {
  const int t = pick_tile(ng, g);
  return t == 0 || t == 4 ? 128 : 64;
}

int conv_splitk(int ng, const ConvGeom& g) {
  if (g.N % 16 != 0 || g.Cs % 8 != 0 || g.Kpad % KC != 0) return 1;
  return pick_tile(ng, g) == 4 ? big_splits(ng, g) : 1;
}

int conv_operand_reuse(int cin, int cout, int R) {
  if (cout % BIG_T != 0 || cin % BIG_K != 0 || R * R * cin < BIG_MIN_K) return 0;
  return R * R * (cout / BIG_T);
}

// The 8-wave kernels take their LDS as dynamic shared memory above the default limit: state it once per device
// before the first launch (not a stream operation, so it stays out of captured graphs).
hipError_t conv_prepare() {
  static std::mutex mu;
  static bool done[64] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  std::lock_guard<std::mutex> lock(mu);
  if (dev >= 0 && dev < 64 && done[dev]) return hipSuccess;
  auto set = [&](const void* f) {
    if (e == hipSuccess) e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)BIG_MAX_LDS);
  };
  set(reinterpret_cast<const void*>(k_conv_big<CONV_FWD, EPI_STATS, 1>));
  set(reinterpret_cast<const void*>(k_conv_big<CONV_FWD, EPI_STATS, 0>));
  set(reinterpret_cast<const void*>(k_conv_big<CONV_FWD, EPI_NONE, 1>));
  set(reinterpret_cast<const void*>(k_conv_big<CONV_FWD, EPI_NONE, 0>));
  set(reinterpret_cast<const void*>(k_conv_big<CONV_DGRAD, EPI_BNBWD, 0>));
  set(reinterpret_cast<const void*>(k_conv_big<CONV_DGRAD, EPI_NONE, 0>));
  set(reinterpret_cast<const void*>(k_conv_big<CONV_FWD, EPI_NONE, 0, true>));
  set(reinterpret_cast<const void*>(k_conv_big<CONV_DGRAD, EPI_NONE, 0, true>));
  if (e == hipSuccess && dev >= 0 && dev < 64) done[dev] = true;
  return e;
}

// Tile choice: the widest channel tile that divides N, then the pixel tile that still gives the
// chip (256 CUs) enough work-groups.
hipError_t launch_conv_mfma(int mode, int ng, const PtrTab& src, const bf16_t* wpk, const PtrTab& out, const PtrTab& add,
                            const ConvGeom& g, hipStream_t stream, const ConvEpi& epi, const ConvPro& pro) {
  if (ng < 1 || ng > MAX_GROUP) return hipErrorInvalidValue;
  if (g.N % 16 != 0 || g.Cs % 8 != 0 || g.Kpad % KC != 0 || (g.stride != 1 && g.stride != 2)) return hipErrorInvalidValue;
  switch (pick_tile(ng, g)) {
    case 4: return launch_big(mode, ng, src, wpk, out, add, g, stream, epi, pro);
    case 0: return launch_tile<128, 128, 2, 2>(mode, ng, src, wpk, out, add, g, stream, epi, pro);
    case 1: return launch_tile<64, 64, 2, 2>(mode, ng, src, wpk, out, add, g, stream, epi, pro);
    case 2: return launch_tile<64, 32, 4, 1>(mode, ng, src, wpk, out, add, g, stream, epi, pro);
    default: return launch_tile<64, 16, 4, 1>(mode, ng, src, wpk, out, add, g, stream, epi, pro);
  }
}

}  // namespace hpf
