// Convolution weight-gradient on bf16 MFMA with fp32 accumulation, added in place into the fp32
// gradient buffer that collects all micro-batches of a batch (the buffer the per-partition
// allreduce of the hybrid-parallel design would consume).
//
//   dw[tap][c][n] += sum_m a[row(m, tap), c] * dy[m, n]
//
// The reduction runs over the pixel rows m (hundreds to thousands), the output is tiny, so the rows
// are split over work-groups (grid.x) and every work-group owns one (tap, BC x BN) output tile
// (grid.y).  Inside a work-group the four waves take consecutive 32-row slices of each 128-row
// step, accumulate the same output tile, and are summed through LDS at the end; one atomic add per
// output element and work-group then goes to the gradient buffer.
//
// Both MFMA operands need 8 consecutive reduction indices (pixel rows) per lane while memory has
// the channel contiguous, so the staging threads transpose: each loads 16 bytes (8 channels) of two
// adjacent rows and writes 8 dwords {row 2j, row 2j+1} into the channel-major LDS tile.
#include "hpf_device.h"

namespace hpf {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int MC = 128;         // pixel rows per step (32 per wave); the 128 x 128 class takes 64-row steps

// A staging unit is (pixel pair of the 128-row step, group of 8 channels).  With at least 4 channel groups,
// four neighbouring lanes take four consecutive groups of one pair (64 contiguous bytes of a pixel) and the
// 16 lane quads of a wave 16 consecutive pairs: global loads touch 16 cache lines per instruction instead of
// 64, and the transposing LDS stores stay within a 2-way bank conflict.  Narrow tiles keep one pair per lane.
template <int G>
__device__ __forceinline__ void unit_map(int unit, int& pr, int& grp) {
  if (G >= 4) {
    const int lane = unit & 63, q = unit >> 6;
    grp = (q % (G / 4)) * 4 + (lane & 3);
    pr = (q / (G / 4)) * 16 + (lane >> 2);
  } else {
    pr = unit & 63;
    grp = unit >> 6;
  }
}

template <int BC, int BN, int ROWS = MC>
struct WgradTile {
  static constexpr int CTL = BC / 16, NTL = BN / 16;
  static constexpr int PAIRS = ROWS / 2;            // pixel pairs per step
  static constexpr int LSTR = ROWS + 8;             // LDS row stride in bf16 (272 or 144 bytes: 16 rows hit 16 bank groups)
  static constexpr int A_UNITS = (PAIRS * (BC / 8) + 255) / 256;
  static constexpr int D_UNITS = (PAIRS * (BN / 8) + 255) / 256;
  static constexpr int LDS_A = BC * LSTR, LDS_D = BN * LSTR;
  static constexpr int RED_BYTES = BC * BN * 4;
  static constexpr int OP_BYTES = (LDS_A + LDS_D) * 2;
  static constexpr int QUAD_BYTES = OP_BYTES + BC * 8;   // + {scale, shift} per tile channel
  static constexpr int SMEM_BYTES = OP_BYTES > RED_BYTES ? OP_BYTES : RED_BYTES;
};

// Adds sum over rows [m_begin, m_end) of a[row(m,tap), c0..c0+BC) (x) dy[m, n0..n0+BN) into acc
// (each of the 4 waves holds the sum over its 32-row slices).
// bn_stats != nullptr: `a` is the input of a BatchNorm and the operand is relu(bn(a)), recomputed while
// staging from {mean, invstd} = bn_stats[0..Cin), [Cin..2Cin) and gamma / beta (the normalised
// activation is not kept in memory); rows outside the image stay zero.
// QUAD = false: the four waves take 32-row slices of each step and all accumulate the whole BC x BN tile
// (acc is [BC/16][BN/16], summed over the waves afterwards).  QUAD = true (large tiles): every wave takes all
// rows of the step and owns one quadrant of the tile (acc is [BC/32][BN/32]): half the operand traffic per flop.
template <int BC, int BN, bool QUAD = false>
__device__ __forceinline__ void wgrad_accumulate(const bf16_t* __restrict__ a, const bf16_t* __restrict__ dy, const WgradGeom& g,
                                                 int tap, int c0, int n0, int m_begin, int m_end, bf16_t* sA, bf16_t* sD,
                                                 floatx4 (&acc)[BC / (QUAD ? 32 : 16)][BN / (QUAD ? 32 : 16)],
                                                 const float* bn_stats = nullptr, const float* gamma = nullptr,
                                                 const float* beta = nullptr) {
  constexpr int ROWS = QUAD ? 64 : MC;
  typedef WgradTile<BC, BN, ROWS> TT;
  constexpr int CTL = BC / (QUAD ? 32 : 16), NTL = BN / (QUAD ? 32 : 16), A_UNITS = TT::A_UNITS, D_UNITS = TT::D_UNITS;
  constexpr int LSTR = TT::LSTR, A_N = TT::PAIRS * (BC / 8), D_N = TT::PAIRS * (BN / 8);   // staging units per step
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = tap / g.R, s = tap - r * g.R;
  const int HoWo = g.Ho * g.Wo;

  uint4 ra[A_UNITS][2], rd[D_UNITS][2];
  bool rv[A_UNITS][2];
  // {scale, shift} of the BatchNorm: held per thread for its 8 channels (fixed over the steps), or -- for the
  // large tiles, where registers are short -- per tile channel in LDS behind the operand tiles
  float2 cf[QUAD ? 1 : A_UNITS][8];
  float2* sCf = reinterpret_cast<float2*>(sD + TT::LDS_D);
  if (bn_stats) {
    if (QUAD) {
      if (tid < BC) {
        const int c = c0 + tid;
        const float sc = gamma[c] * bn_stats[g.Cin + c];
        sCf[tid] = make_float2(sc, beta[c] - bn_stats[c] * sc);   // read after the first barrier of the step loop
      }
    } else {
#pragma unroll
      for (int u = 0; u < A_UNITS; ++u) {
        const int unit = tid + u * 256;
        if (unit < A_N) {
          int pr_, cg_;
          unit_map<BC / 8>(unit, pr_, cg_);
          const int c = c0 + cg_ * 8;
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const float sc = gamma[c + i] * bn_stats[g.Cin + c + i];
            cf[QUAD ? 0 : u][i] = make_float2(sc, beta[c + i] - bn_stats[c + i] * sc);
          }
        }
      }
    }
  }
  auto bn_relu8 = [&](const uint4& q, const float2 (&k)[8]) {
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
    uint32_t r_[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float x0 = __uint_as_float(w[i] << 16), x1 = __uint_as_float(w[i] & 0xffff0000u);
      r_[i] = pack_bf16x2(fmaxf(fmaf(x0, k[2 * i].x, k[2 * i].y), 0.f), fmaxf(fmaf(x1, k[2 * i + 1].x, k[2 * i + 1].y), 0.f));
    }
    return make_uint4(r_[0], r_[1], r_[2], r_[3]);
  };

  // (image, output row, output column) of every pixel row this thread stages: decoded once with divisions for
  // the first step, then advanced by ROWS rows per step with carries (ROWS = dimg*HoWo + dp*Wo + dq)
  const int dimg = ROWS / HoWo, drem = ROWS - dimg * HoWo, dp = drem / g.Wo, dq = drem - dp * g.Wo;
  int pi[A_UNITS], pp[A_UNITS], pq[A_UNITS];   // of the even row of each pair; the odd row follows it
#pragma unroll
  for (int u = 0; u < A_UNITS; ++u) {
    const int unit = tid + u * 256;
    int pr, cg;
    unit_map<BC / 8>(unit < A_N ? unit : 0, pr, cg);
    const int m = m_begin + 2 * pr;
    pi[u] = m / HoWo;
    const int rem = m - pi[u] * HoWo;
    pp[u] = rem / g.Wo;
    pq[u] = rem - pp[u] * g.Wo;
  }
  // All loads are issued unconditionally (rows past the end or outside the image read a clamped address and are
  // zeroed when they are stored to LDS), so the count of outstanding loads is known at every wait.
  bool dv[D_UNITS][2];
  auto load_step = [&](int m0) {
#pragma unroll
    for (int u = 0; u < A_UNITS; ++u) {
      const int unit = tid + u * 256;
      int pr, cg;
      unit_map<BC / 8>(unit < A_N ? unit : 0, pr, cg);
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const int m = m0 + 2 * pr + e;
        int im = pi[u], p = pp[u], q = pq[u] + e;
        if (q >= g.Wo) { q = 0; if (++p >= g.Ho) { p = 0; ++im; } }
        const int hi = p * g.stride + r - g.pad, wi = q * g.stride + s - g.pad;
        const bool v = (unit < A_N) && m < m_end && (unsigned)hi < (unsigned)g.H && (unsigned)wi < (unsigned)g.W;
        const size_t off = v ? ((size_t)(im * g.H + hi) * g.W + wi) * g.Cin + c0 + cg * 8 : (size_t)0;
        rv[u][e] = v;
        ra[u][e] = *reinterpret_cast<const uint4*>(a + off);
      }
      // next step's rows
      pq[u] += dq;
      if (pq[u] >= g.Wo) { pq[u] -= g.Wo; ++pp[u]; }
      pp[u] += dp;
      if (pp[u] >= g.Ho) { pp[u] -= g.Ho; ++pi[u]; }
      pi[u] += dimg;
    }
#pragma unroll
    for (int u = 0; u < D_UNITS; ++u) {
      const int unit = tid + u * 256;
      int pr, ng;
      unit_map<BN / 8>(unit < D_N ? unit : 0, pr, ng);
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const int m = m0 + 2 * pr + e;
        const bool v = (unit < D_N) && m < m_end;
        dv[u][e] = v;
        rd[u][e] = *reinterpret_cast<const uint4*>(dy + (v ? (size_t)m * g.N + n0 + ng * 8 : (size_t)0));
      }
    }
  };
  // {lo half of x = element 2i, hi half = element 2i+1}: interleave two rows into {row0, row1} dwords
  auto store_pairs = [&](bf16_t* tile_base, int pr, int grp, const uint4& v0, const uint4& v1) {
    uint32_t* dst = reinterpret_cast<uint32_t*>(tile_base + (grp * 8) * LSTR + 2 * pr);
    constexpr int RS = LSTR / 2;  // dwords per LDS row
    const uint32_t e0[4] = {v0.x, v0.y, v0.z, v0.w}, e1[4] = {v1.x, v1.y, v1.z, v1.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      dst[(2 * i) * RS] = (e0[i] & 0xffffu) | (e1[i] << 16);
      dst[(2 * i + 1) * RS] = (e0[i] >> 16) | (e1[i] & 0xffff0000u);
    }
  };
  auto store_step = [&]() {
#pragma unroll
    for (int u = 0; u < A_UNITS; ++u) {
      const int unit = tid + u * 256;
      if (unit < A_N) {
        int pr, cg;
        unit_map<BC / 8>(unit, pr, cg);
        if (bn_stats) {
          if (QUAD) {
            const float4* k4 = reinterpret_cast<const float4*>(sCf + cg * 8);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const float4 k = k4[i];
              cf[0][2 * i] = make_float2(k.x, k.y);
              cf[0][2 * i + 1] = make_float2(k.z, k.w);
            }
          }
          ra[u][0] = bn_relu8(ra[u][0], cf[QUAD ? 0 : u]);
          ra[u][1] = bn_relu8(ra[u][1], cf[QUAD ? 0 : u]);
        }
        const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
        store_pairs(sA, pr, cg, rv[u][0] ? ra[u][0] : zero, rv[u][1] ? ra[u][1] : zero);
      }
    }
#pragma unroll
    for (int u = 0; u < D_UNITS; ++u) {
      const int unit = tid + u * 256;
      if (unit < D_N) {
        int pr, ng;
        unit_map<BN / 8>(unit, pr, ng);
        const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
        store_pairs(sD, pr, ng, dv[u][0] ? rd[u][0] : zero, dv[u][1] ? rd[u][1] : zero);
      }
    }
  };

  const int frag_row = lane & 15, frag_m = wave * 32 + (lane >> 4) * 8;
  if (m_begin < m_end) load_step(m_begin);
  for (int m0 = m_begin; m0 < m_end; m0 += ROWS) {
    __syncthreads();  // previous step's LDS reads are done
    store_step();
    __syncthreads();
    if (m0 + ROWS < m_end) load_step(m0 + ROWS);
    if (QUAD) {
      const int qc = (wave >> 1) * (BC / 2), qn = (wave & 1) * (BN / 2);
#pragma unroll
      for (int ks = 0; ks < ROWS / 32; ++ks) {
        const int fm = ks * 32 + (lane >> 4) * 8;
        bf16x8 fa[CTL], fd[NTL];
#pragma unroll
        for (int i = 0; i < CTL; ++i) fa[i] = *reinterpret_cast<const bf16x8*>(&sA[(qc + i * 16 + frag_row) * LSTR + fm]);
#pragma unroll
        for (int j = 0; j < NTL; ++j) fd[j] = *reinterpret_cast<const bf16x8*>(&sD[(qn + j * 16 + frag_row) * LSTR + fm]);
#pragma unroll
        for (int i = 0; i < CTL; ++i)
#pragma unroll
          for (int j = 0; j < NTL; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[i], fd[j], acc[i][j], 0, 0, 0);
      }
    } else {
      bf16x8 fa[CTL], fd[NTL];
#pragma unroll
      for (int i = 0; i < CTL; ++i) fa[i] = *reinterpret_cast<const bf16x8*>(&sA[(i * 16 + frag_row) * LSTR + frag_m]);
#pragma unroll
      for (int j = 0; j < NTL; ++j) fd[j] = *reinterpret_cast<const bf16x8*>(&sD[(j * 16 + frag_row) * LSTR + frag_m]);
#pragma unroll
      for (int i = 0; i < CTL; ++i)
#pragma unroll
        for (int j = 0; j < NTL; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[i], fd[j], acc[i][j], 0, 0, 0);
    }
  }
}

// Sums the four waves' accumulators through LDS and adds the tile into dw with one atomic per element.
template <int BC, int BN>
__device__ __forceinline__ void wgrad_flush(floatx4 (&acc)[BC / 16][BN / 16], float* red, float* dw, const WgradGeom& g, int tap,
                                            int c0, int n0) {
  constexpr int CTL = BC / 16, NTL = BN / 16;
  const int tid = threadIdx.x, lane = tid & 63;
  __syncthreads();
  for (int i = tid; i < BC * BN; i += 256) red[i] = 0.f;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < CTL; ++i)
#pragma unroll
    for (int j = 0; j < NTL; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int c = i * 16 + (lane >> 4) * 4 + v, n = j * 16 + (lane & 15);
        atomicAdd(&red[c * BN + n], acc[i][j][v]);
      }
  __syncthreads();
  for (int i = tid; i < BC * BN; i += 256) {
    const int c = c0 + i / BN, n = n0 + i % BN;
    if (c < g.c_valid) atomicAdd(&dw[((size_t)tap * g.c_valid + c) * g.N + n], red[i]);
  }
}

template <int BC, int BN>
__global__ __launch_bounds__(256) void k_wgrad_mfma(PtrTab as, PtrTab dys, float* dw, WgradGeom g, int rows_per_split) {
  typedef WgradTile<BC, BN> TT;
  __shared__ __attribute__((aligned(16))) unsigned char smem[TT::SMEM_BYTES];
  bf16_t* sA = reinterpret_cast<bf16_t*>(smem);
  bf16_t* sD = sA + TT::LDS_A;
  const int n_ct = g.Cin / BC, n_nt = g.N / BN;
  int tile = blockIdx.y;
  const int nt = tile % n_nt; tile /= n_nt;
  const int ct = tile % n_ct; tile /= n_ct;
  const int tap = tile;
  const int m_begin = blockIdx.x * rows_per_split;
  const int m_end = min(g.M, m_begin + rows_per_split);
  floatx4 acc[TT::CTL][TT::NTL];
#pragma unroll
  for (int i = 0; i < TT::CTL; ++i)
#pragma unroll
    for (int j = 0; j < TT::NTL; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
  wgrad_accumulate<BC, BN>((const bf16_t*)pick(as, blockIdx.z), (const bf16_t*)pick(dys, blockIdx.z), g, tap, ct * BC, nt * BN, m_begin,
                           m_end, sA, sD, acc);
  wgrad_flush<BC, BN>(acc, reinterpret_cast<float*>(smem), dw, g, tap, ct * BC, nt * BN);
}

// One work-group per item; the micro-batches of the group are accumulated in registers.
template <int BC, int BN>
__global__ __launch_bounds__(256) void k_wgrad_grouped(const WgradItem* __restrict__ items, int ng, PtrTab bases, PtrTab caller_dy,
                                                       PtrTab caller_a, const float* __restrict__ params, float* grads) {
  typedef WgradTile<BC, BN> TT;
  __shared__ __attribute__((aligned(16))) unsigned char smem[TT::SMEM_BYTES];
  bf16_t* sA = reinterpret_cast<bf16_t*>(smem);
  bf16_t* sD = sA + TT::LDS_A;
  const WgradItem it = items[blockIdx.x];
  floatx4 acc[TT::CTL][TT::NTL];
#pragma unroll
  for (int i = 0; i < TT::CTL; ++i)
#pragma unroll
    for (int j = 0; j < TT::NTL; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
  for (int z = 0; z < ng; ++z) {
    const char* base = (const char*)pick(bases, z);
    const bf16_t* a = it.a_off == WGRAD_DY_CALLER ? (const bf16_t*)pick(caller_a, z) : (const bf16_t*)(base + it.a_off);
    const bf16_t* dy = it.dy_off == WGRAD_DY_CALLER ? (const bf16_t*)pick(caller_dy, z) : (const bf16_t*)(base + it.dy_off);
    if (it.stats_off != WGRAD_NO_BN)
      wgrad_accumulate<BC, BN>(a, dy, it.g, it.tap, it.c0, it.n0, it.m_begin, it.m_end, sA, sD, acc,
                               (const float*)(base + it.stats_off), params + it.gamma_off, params + it.beta_off);
    else
      wgrad_accumulate<BC, BN>(a, dy, it.g, it.tap, it.c0, it.n0, it.m_begin, it.m_end, sA, sD, acc);
  }
  wgrad_flush<BC, BN>(acc, reinterpret_cast<float*>(smem), grads + it.dw_off, it.g, it.tap, it.c0, it.n0);
}

// The 128 x 128 class: every wave owns a 64 x 64 quadrant over the whole reduction, so the sums go straight
// from the accumulators to the gradient buffer (one atomic per output element and work-group).
__global__ __launch_bounds__(256, 2) void k_wgrad_grouped_quad(const WgradItem* __restrict__ items, int ng, PtrTab bases, PtrTab caller_dy,
                                                            PtrTab caller_a, const float* __restrict__ params, float* grads) {
  constexpr int BC = 128, BN = 128;
  typedef WgradTile<BC, BN, 64> TT;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_q[];
  bf16_t* sA = reinterpret_cast<bf16_t*>(smem_q);
  bf16_t* sD = sA + TT::LDS_A;
  const WgradItem it = items[blockIdx.x];
  floatx4 acc[BC / 32][BN / 32];
#pragma unroll
  for (int i = 0; i < BC / 32; ++i)
#pragma unroll
    for (int j = 0; j < BN / 32; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
  for (int z = 0; z < ng; ++z) {
    const char* base = (const char*)pick(bases, z);
    const bf16_t* a = it.a_off == WGRAD_DY_CALLER ? (const bf16_t*)pick(caller_a, z) : (const bf16_t*)(base + it.a_off);
    const bf16_t* dy = it.dy_off == WGRAD_DY_CALLER ? (const bf16_t*)pick(caller_dy, z) : (const bf16_t*)(base + it.dy_off);
    if (it.stats_off != WGRAD_NO_BN)
      wgrad_accumulate<BC, BN, true>(a, dy, it.g, it.tap, it.c0, it.n0, it.m_begin, it.m_end, sA, sD, acc,
                                     (const float*)(base + it.stats_off), params + it.gamma_off, params + it.beta_off);
    else
      wgrad_accumulate<BC, BN, true>(a, dy, it.g, it.tap, it.c0, it.n0, it.m_begin, it.m_end, sA, sD, acc);
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int qc = it.c0 + (wave >> 1) * (BC / 2), qn = it.n0 + (wave & 1) * (BN / 2);
  float* dw = grads + it.dw_off;
#pragma unroll
  for (int i = 0; i < BC / 32; ++i)
#pragma unroll
    for (int j = 0; j < BN / 32; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int c = qc + i * 16 + (lane >> 4) * 4 + v, n = qn + j * 16 + (lane & 15);
        if (c < it.g.c_valid) atomicAdd(&dw[((size_t)it.tap * it.g.c_valid + c) * it.g.N + n], acc[i][j][v]);
      }
}

// ---- whole 3x3 convolutions between 16 and 16 channels --------------------------------------------------------
// With 16 channels on both sides a per-tap item moves 64 bytes per pixel for one MFMA per 32 pixels, nine times
// per convolution.  Here one work-group takes whole images: both operands of an image go to LDS once, channel-major
// (the input with a zero row above and below), and every 32-pixel step feeds nine MFMAs: the three filter rows are
// three fragment reads of the input at row offsets, the three filter columns three variants of the one gradient
// fragment, shifted by a pixel in registers (the pixel that crosses into the next 8-pixel chunk comes from the lane
// that holds that chunk; at the image border it is zero).  Needs stride 1, H*W = 1024 and W in {8, 16, 32}.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int T9_P = 1024, T9_NU = T9_P / 256;   // pixels per image; staging units (pixel pair x 8 channels) per thread and operand
__host__ __device__ constexpr int t9_sa(int H, int W) { return (H + 2) * W + 8; }   // channel stride of the padded input tile (bf16):
__host__ __device__ constexpr int t9_sd(int H, int W) { return H * W + 8; }         // = 8 mod 16, so 16 channels hit 16 bank groups
__host__ __device__ constexpr int t9_lds_bytes(int H, int W) { return 16 * (t9_sa(H, W) + t9_sd(H, W)) * 2 + MAX_GROUP * 16 * 8; }   // tiles + {scale, shift} per member and channel
constexpr int T9_MAX_LDS = t9_lds_bytes(32, 32);   // the widest rows pad the most

__global__ __launch_bounds__(256) void k_wgrad_grouped_t9(const WgradItem* __restrict__ items, int ng, PtrTab bases, PtrTab caller_dy,
                                                          PtrTab caller_a, const float* __restrict__ params, float* grads) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_t9[];
  const WgradItem it = items[blockIdx.x];
  const int H = it.g.H, W = it.g.W;
  const int SA = t9_sa(H, W), SD = t9_sd(H, W);
  bf16_t* sA = reinterpret_cast<bf16_t*>(smem_t9);
  bf16_t* sD = sA + 16 * SA;
  uint32_t* sA32 = reinterpret_cast<uint32_t*>(sA);
  uint32_t* sD32 = reinterpret_cast<uint32_t*>(sD);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int hf = tid & 1;                       // the thread's channels: 8*hf .. 8*hf+7 (256 is even: the same for all its units)
  // the zero rows of the input tile (the staging below never writes them)
  for (int i = tid; i < 16 * W; i += 256) {
    const int c = i / W, j = i - c * W;
    const int row = j >= (W >> 1) ? H + 1 : 0, col2 = j >= (W >> 1) ? j - (W >> 1) : j;
    sA32[((c * SA + row * W) >> 1) + col2] = 0u;
  }

  const int nimg = (it.m_end - it.m_begin) / T9_P, img0 = it.m_begin / T9_P;
  const int total = ng * nimg;
  // Loads: 16-byte unit u of an image (pixel u/2, channel half u%2) goes to thread u % 256, so a wave reads 1 KB of
  // contiguous memory per instruction.  Lanes t and t^2 then hold the two pixels of a pair (same channel half): they
  // swap half of their channels (DPP within the quad), so that each ends up with 4 channels of both pixels and writes
  // them as 4 dwords {pixel 2pp, pixel 2pp+1} into the channel-major tiles.
  constexpr int T9_LD = 2 * T9_NU;               // loads per thread, operand and image
  struct Regs { uint4 a[T9_LD], d[T9_LD]; };
  Regs set0, set1;                               // two images on their way: a set is refilled as soon as it has been staged
  const int odd = (tid >> 1) & 1;                // this thread's pixels are the odd ones of their pairs
  auto load_image = [&](int i, Regs& rg) {
    const int z = i / nimg, img = img0 + (i - z * nimg);
    const char* base = (const char*)pick(bases, z);
    const bf16_t* a = it.a_off == WGRAD_DY_CALLER ? (const bf16_t*)pick(caller_a, z) : (const bf16_t*)(base + it.a_off);
    const bf16_t* dy = it.dy_off == WGRAD_DY_CALLER ? (const bf16_t*)pick(caller_dy, z) : (const bf16_t*)(base + it.dy_off);
    a += (size_t)img * T9_P * 16 + tid * 8;
    dy += (size_t)img * T9_P * 16 + tid * 8;
#pragma unroll
    for (int k = 0; k < T9_LD; ++k) {
      rg.a[k] = *reinterpret_cast<const uint4*>(a + (size_t)k * 256 * 8);
      rg.d[k] = *reinterpret_cast<const uint4*>(dy + (size_t)k * 256 * 8);
    }
  };
  // {scale, shift} of the BatchNorm recomputed on the input, for every member of the launch: in LDS once, so that the
  // images do not wait for a round trip to memory each
  float2* sCf = reinterpret_cast<float2*>(sD + 16 * SD);
  const bool bn = it.stats_off != WGRAD_NO_BN;
  if (bn && tid < ng * 16) {
    const int z = tid >> 4, c = tid & 15;
    const float* stt = (const float*)((const char*)pick(bases, z) + it.stats_off);
    const float sc = params[it.gamma_off + c] * stt[16 + c];
    sCf[tid] = make_float2(sc, params[it.beta_off + c] - stt[c] * sc);
  }
  __syncthreads();
  float2 cf[8];
  auto bn_relu8 = [&](const uint4& q) {
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
    uint32_t r_[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float x0 = __uint_as_float(w[i] << 16), x1 = __uint_as_float(w[i] & 0xffff0000u);
      r_[i] = pack_bf16x2(fmaxf(fmaf(x0, cf[2 * i].x, cf[2 * i].y), 0.f), fmaxf(fmaf(x1, cf[2 * i + 1].x, cf[2 * i + 1].y), 0.f));
    }
    return make_uint4(r_[0], r_[1], r_[2], r_[3]);
  };
  // transposing store of one unit: the even-pixel lane keeps its channels 0..3 and takes the partner's, the odd-pixel
  // lane its channels 4..7; dst points at channel row 8*hf + 4*odd, pixel pair pp
  auto store_unit = [&](uint32_t* dst, int cstride2, const uint4& q) {
    const uint32_t send0 = odd ? q.x : q.z, send1 = odd ? q.y : q.w;
    const uint32_t recv0 = (uint32_t)__builtin_amdgcn_mov_dpp((int)send0, 0x4E, 0xF, 0xF, true);   // quad_perm [2,3,0,1]: lane ^ 2
    const uint32_t recv1 = (uint32_t)__builtin_amdgcn_mov_dpp((int)send1, 0x4E, 0xF, 0xF, true);
    const uint32_t f0 = odd ? recv0 : q.x, f1 = odd ? recv1 : q.y;   // the pair's first (even) pixel
    const uint32_t s0 = odd ? q.z : recv0, s1 = odd ? q.w : recv1;   // its second pixel
    dst[0] = (f0 & 0xffffu) | (s0 << 16);
    dst[cstride2] = (f0 >> 16) | (s0 & 0xffff0000u);
    dst[2 * cstride2] = (f1 & 0xffffu) | (s1 << 16);
    dst[3 * cstride2] = (f1 >> 16) | (s1 & 0xffff0000u);
  };

  floatx4 acc[9];
#pragma unroll
  for (int i = 0; i < 9; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
  const int r = lane & 15, g = lane >> 4;
  if (total > 0) load_image(0, set0);
  if (total > 1) load_image(1, set1);
  auto image = [&](int i, Regs& rg) {
    if (bn && i % nimg == 0) {                  // a new member: its coefficients
#pragma unroll
      for (int e = 0; e < 8; ++e) cf[e] = sCf[(i / nimg) * 16 + hf * 8 + e];
    }
#pragma unroll
    for (int k = 0; k < T9_LD; ++k) {
      const int pp = (tid >> 2) + 64 * k;       // pixel pair of unit tid + 256*k
      uint4 q = rg.a[k];
      if (bn) q = bn_relu8(q);
      store_unit(sA32 + (((hf * 8 + odd * 4) * SA + W) >> 1) + pp, SA >> 1, q);
      store_unit(sD32 + (((hf * 8 + odd * 4) * SD) >> 1) + pp, SD >> 1, rg.d[k]);
    }
    if (i + 2 < total) load_image(i + 2, rg);
    __syncthreads();
#pragma unroll 4
    for (int st = 0; st < T9_P / 128; ++st) {
      const int px = (wave * (T9_P / 128) + st) * 32 + g * 8;   // first pixel of the lane's chunk
      const int col = px & (W - 1);
      const u32x4 d = *reinterpret_cast<const u32x4*>(&sD[r * SD + px]);
      uint32_t left = (uint32_t)__builtin_amdgcn_ds_bpermute((lane - 16) * 4, (int)d.w);
      uint32_t right = (uint32_t)__builtin_amdgcn_ds_bpermute((lane + 16) * 4, (int)d.x);
      if (col == 0) left = 0u;
      if (col + 8 >= W) right = 0u;
      // filter column 0 multiplies input pixel w-1 with gradient pixel w: per input pixel w' the gradient of w'+1; column 2: of w'-1
      u32x4 dm, dp;
      dm.x = __builtin_amdgcn_alignbit(d.y, d.x, 16); dm.y = __builtin_amdgcn_alignbit(d.z, d.y, 16);
      dm.z = __builtin_amdgcn_alignbit(d.w, d.z, 16); dm.w = __builtin_amdgcn_alignbit(right, d.w, 16);
      dp.x = __builtin_amdgcn_alignbit(d.x, left, 16); dp.y = __builtin_amdgcn_alignbit(d.y, d.x, 16);
      dp.z = __builtin_amdgcn_alignbit(d.z, d.y, 16); dp.w = __builtin_amdgcn_alignbit(d.w, d.z, 16);
      const bf16x8 f0 = __builtin_bit_cast(bf16x8, dm), f1 = __builtin_bit_cast(bf16x8, d), f2 = __builtin_bit_cast(bf16x8, dp);
#pragma unroll
      for (int fr = 0; fr < 3; ++fr) {          // filter row fr reads the input one row up, in place, one row down
        const bf16x8 fa = *reinterpret_cast<const bf16x8*>(&sA[r * SA + fr * W + px]);
        acc[fr * 3 + 0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, f0, acc[fr * 3 + 0], 0, 0, 0);
        acc[fr * 3 + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, f1, acc[fr * 3 + 1], 0, 0, 0);
        acc[fr * 3 + 2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, f2, acc[fr * 3 + 2], 0, 0, 0);
      }
    }
    __syncthreads();
  };
  for (int i = 0; i < total; i += 2) {
    image(i, set0);
    if (i + 1 < total) image(i + 1, set1);
  }
  // the four waves' sums through LDS, then one atomic per output element and work-group
  float* red = reinterpret_cast<float*>(smem_t9);
  for (int i = tid; i < 9 * 256; i += 256) red[i] = 0.f;
  __syncthreads();
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int v = 0; v < 4; ++v) atomicAdd(&red[t * 256 + (g * 4 + v) * 16 + r], acc[t][v]);
  __syncthreads();
  float* dw = grads + it.dw_off;
  for (int i = tid; i < 9 * 256; i += 256) atomicAdd(&dw[i], red[i]);
}

template <int BC, int BN>
hipError_t launch_tile(int ng, const PtrTab& a, const PtrTab& dy, float* dw, const WgradGeom& g, hipStream_t stream) {
  const int tiles = g.R * g.R * (g.Cin / BC) * (g.N / BN);
  const int max_splits = (g.M + MC - 1) / MC;
  int splits = (512 + tiles * ng - 1) / (tiles * ng);
  if (splits > max_splits) splits = max_splits;
  if (splits < 1) splits = 1;
  int rows = (g.M + splits - 1) / splits;
  rows = (rows + MC - 1) / MC * MC;
  splits = (g.M + rows - 1) / rows;
  k_wgrad_mfma<BC, BN><<<dim3((unsigned)splits, (unsigned)tiles, (unsigned)ng), 256, 0, stream>>>(a, dy, dw, g, rows);
  return hipGetLastError();
}

template <int BC>
hipError_t pick_bn(int ng, const PtrTab& a, const PtrTab& dy, float* dw, const WgradGeom& g, hipStream_t stream) {
  if (g.N % 64 == 0) return launch_tile<BC, 64>(ng, a, dy, dw, g, stream);
  if (g.N % 32 == 0) return launch_tile<BC, 32>(ng, a, dy, dw, g, stream);
  return launch_tile<BC, 16>(ng, a, dy, dw, g, stream);
}

}  // namespace

hipError_t launch_wgrad_mfma(int ng, const PtrTab& a, const PtrTab& dy, float* dw, const WgradGeom& g, hipStream_t stream) {
  if (ng < 1 || ng > MAX_GROUP || g.Cin % 16 != 0 || g.N % 16 != 0) return hipErrorInvalidValue;
  if (g.Cin % 64 == 0) return pick_bn<64>(ng, a, dy, dw, g, stream);
  if (g.Cin % 32 == 0) return pick_bn<32>(ng, a, dy, dw, g, stream);
  return pick_bn<16>(ng, a, dy, dw, g, stream);
}

namespace {
int tile_index(int c) { return c % 64 == 0 ? 2 : (c % 32 == 0 ? 1 : 0); }
}  // namespace

int wgrad_t9_lds_bytes(int H, int W) { return t9_lds_bytes(H, W); }

int wgrad_tile_class(int cin, int cout) {
  if (cin % 128 == 0 && cout % 128 == 0) return 9;
  return tile_index(cin) * 3 + tile_index(cout);
}

int wgrad_item_class(const WgradGeom& g) {
  if (g.Cin == 16 && g.N == 16 && g.c_valid == 16 && g.R == 3 && g.stride == 1 && g.H * g.W == T9_P &&
      (g.W == 8 || g.W == 16 || g.W == 32))
    return WGRAD_CLASS_T9;
  return wgrad_tile_class(g.Cin, g.N);
}

void wgrad_tile_dims(int tile_class, int* bc, int* bn) {
  static const int sz[3] = {16, 32, 64};
  if (tile_class == WGRAD_CLASS_T9) { *bc = 16; *bn = 16; return; }
  if (tile_class == 9) { *bc = 128; *bn = 128; return; }
  *bc = sz[tile_class / 3];
  *bn = sz[tile_class % 3];
}

// The 128 x 128 class takes its LDS (two operand tiles and the BatchNorm coefficients) as dynamic shared memory:
// state the size once per device before the first launch (not a stream operation, so it stays out of captured graphs).
hipError_t wgrad_prepare() {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_wgrad_grouped_quad), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     WgradTile<128, 128, 64>::QUAD_BYTES);
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(k_wgrad_grouped_t9), hipFuncAttributeMaxDynamicSharedMemorySize,
                             T9_MAX_LDS);
}

hipError_t launch_wgrad_grouped(int tile_class, int ng, const WgradItem* items_dev, int n_items, const PtrTab& region_base,
                                const PtrTab& caller_dy, const PtrTab& caller_a, const float* params, float* grads,
                                hipStream_t stream, int lds_bytes) {
  if (n_items <= 0) return hipSuccess;
  if (ng < 1 || ng > MAX_GROUP) return hipErrorInvalidValue;
  const dim3 grid((unsigned)n_items);
#define HPF_WG(BC, BN) \
  k_wgrad_grouped<BC, BN><<<grid, 256, 0, stream>>>(items_dev, ng, region_base, caller_dy, caller_a, params, grads)
  switch (tile_class) {
    case 0: HPF_WG(16, 16); break;
    case 1: HPF_WG(16, 32); break;
    case 2: HPF_WG(16, 64); break;
    case 3: HPF_WG(32, 16); break;
    case 4: HPF_WG(32, 32); break;
    case 5: HPF_WG(32, 64); break;
    case 6: HPF_WG(64, 16); break;
    case 7: HPF_WG(64, 32); break;
    case 8: HPF_WG(64, 64); break;
    case 9:
      k_wgrad_grouped_quad<<<grid, 256, WgradTile<128, 128, 64>::QUAD_BYTES, stream>>>(items_dev, ng, region_base, caller_dy, caller_a, params,
                                                                                 grads);
      break;
    case WGRAD_CLASS_T9: {
      // all items of the class have one image shape (checked by the planner): the LDS size comes with the call
      if (lds_bytes < 9 * 256 * 4 || lds_bytes > T9_MAX_LDS) return hipErrorInvalidValue;
      k_wgrad_grouped_t9<<<grid, 256, (size_t)lds_bytes, stream>>>(items_dev, ng, region_base, caller_dy, caller_a, params, grads);
      break;
    }
    default: return hipErrorInvalidValue;
  }
#undef HPF_WG
  return hipGetLastError();
}

}  // namespace hpf
