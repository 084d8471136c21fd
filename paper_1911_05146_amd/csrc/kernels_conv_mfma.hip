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
#include "hpf_device.h"

namespace hpf {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int KC = 32;          // reduction elements per step
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

  // acc[i][j][v]: channel = ch0 + wc*WCH + i*16 + (lane>>4)*4 + v, pixel row = row0 + wr*WPX + j*16 + (lane&15)
  // Epilogue scratch in the (now idle) staging LDS: shift per channel and per-wave-row sums.
  float* sK = reinterpret_cast<float*>(&sA[0][0]);        // [BN]
  float* sS = sK + BN;                                     // [WR][BN][2]
  static_assert((BN + WR * BN * 2) * 4 <= (int)sizeof(sA), "epilogue scratch fits the staging buffer");
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
      *reinterpret_cast<float4*>(part + ((size_t)blockIdx.x * g.N + ch0 + tid) * 4) = make_float4(sK[tid], a1, a2, (float)nrows);
    } else {
      *reinterpret_cast<float2*>(part + ((size_t)blockIdx.x * g.N + ch0 + tid) * 2) = make_float2(a1, a2);
    }
  }
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

// 0: 128x128, 1: 64x64, 2: 64x32, 3: 64x16
int pick_tile(int ng, const ConvGeom& g) {
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

int conv_mfma_tile_rows(int ng, const ConvGeom& g) { return pick_tile(ng, g) == 0 ? 128 : 64; }

// Tile choice: the widest channel tile that divides N, then the pixel tile that still gives the
// chip (256 CUs) enough work-groups.
hipError_t launch_conv_mfma(int mode, int ng, const PtrTab& src, const bf16_t* wpk, const PtrTab& out, const PtrTab& add,
                            const ConvGeom& g, hipStream_t stream, const ConvEpi& epi, const ConvPro& pro) {
  if (ng < 1 || ng > MAX_GROUP) return hipErrorInvalidValue;
  if (g.N % 16 != 0 || g.Cs % 8 != 0 || g.Kpad % KC != 0 || (g.stride != 1 && g.stride != 2)) return hipErrorInvalidValue;
  switch (pick_tile(ng, g)) {
    case 0: return launch_tile<128, 128, 2, 2>(mode, ng, src, wpk, out, add, g, stream, epi, pro);
    case 1: return launch_tile<64, 64, 2, 2>(mode, ng, src, wpk, out, add, g, stream, epi, pro);
    case 2: return launch_tile<64, 32, 4, 1>(mode, ng, src, wpk, out, add, g, stream, epi, pro);
    default: return launch_tile<64, 16, 4, 1>(mode, ng, src, wpk, out, add, g, stream, epi, pro);
  }
}

}  // namespace hpf
