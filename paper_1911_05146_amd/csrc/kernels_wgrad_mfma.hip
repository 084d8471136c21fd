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

constexpr int MC = 128;         // pixel rows per step (32 per wave)
constexpr int LSTR = MC + 8;    // LDS row stride in bf16 (272 bytes)

template <int BC, int BN>
__global__ __launch_bounds__(256) void k_wgrad_mfma(PtrTab as, PtrTab dys, float* dw, WgradGeom g, int rows_per_split) {
  const bf16_t* __restrict__ a = (const bf16_t*)as.p[blockIdx.z];
  const bf16_t* __restrict__ dy = (const bf16_t*)dys.p[blockIdx.z];
  constexpr int CTL = BC / 16, NTL = BN / 16;
  constexpr int A_UNITS = (64 * (BC / 8) + 255) / 256;
  constexpr int D_UNITS = (64 * (BN / 8) + 255) / 256;
  constexpr int LDS_A = BC * LSTR, LDS_D = BN * LSTR;
  constexpr int RED_BYTES = BC * BN * 4;
  constexpr int OP_BYTES = (LDS_A + LDS_D) * 2;
  __shared__ __attribute__((aligned(16))) unsigned char smem[OP_BYTES > RED_BYTES ? OP_BYTES : RED_BYTES];
  bf16_t* sA = reinterpret_cast<bf16_t*>(smem);
  bf16_t* sD = sA + LDS_A;
  float* red = reinterpret_cast<float*>(smem);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n_ct = g.Cin / BC, n_nt = g.N / BN;
  int tile = blockIdx.y;
  const int nt = tile % n_nt; tile /= n_nt;
  const int ct = tile % n_ct; tile /= n_ct;
  const int tap = tile;
  const int r = tap / g.R, s = tap - r * g.R;
  const int c0 = ct * BC, n0 = nt * BN;
  const int m_begin = blockIdx.x * rows_per_split;
  const int m_end = min(g.M, m_begin + rows_per_split);
  const int HoWo = g.Ho * g.Wo;

  floatx4 acc[CTL][NTL];
#pragma unroll
  for (int i = 0; i < CTL; ++i)
#pragma unroll
    for (int j = 0; j < NTL; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};

  uint4 ra[A_UNITS][2], rd[D_UNITS][2];

  auto load_step = [&](int m0) {
#pragma unroll
    for (int u = 0; u < A_UNITS; ++u) {
      const int unit = tid + u * 256;
      const int pr = unit & 63, cg = unit >> 6;
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const int m = m0 + 2 * pr + e;
        bool v = (unit < 64 * (BC / 8)) && m < m_end;
        size_t off = 0;
        if (v) {
          const int img = m / HoWo;
          const int rem = m - img * HoWo;
          const int p = rem / g.Wo, q = rem - p * g.Wo;
          const int hi = p * g.stride + r - g.pad, wi = q * g.stride + s - g.pad;
          v = (unsigned)hi < (unsigned)g.H && (unsigned)wi < (unsigned)g.W;
          off = ((size_t)(img * g.H + hi) * g.W + wi) * g.Cin + c0 + cg * 8;
        }
        ra[u][e] = v ? *reinterpret_cast<const uint4*>(a + off) : make_uint4(0u, 0u, 0u, 0u);
      }
    }
#pragma unroll
    for (int u = 0; u < D_UNITS; ++u) {
      const int unit = tid + u * 256;
      const int pr = unit & 63, ng = unit >> 6;
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const int m = m0 + 2 * pr + e;
        const bool v = (unit < 64 * (BN / 8)) && m < m_end;
        rd[u][e] = v ? *reinterpret_cast<const uint4*>(dy + (size_t)m * g.N + n0 + ng * 8) : make_uint4(0u, 0u, 0u, 0u);
      }
    }
  };
  // {lo half of x = element 2i, hi half = element 2i+1}: interleave two rows into {row0, row1} dwords
  auto store_pairs = [&](bf16_t* tile_base, int unit, const uint4& v0, const uint4& v1) {
    const int pr = unit & 63, grp = unit >> 6;
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
      if (unit < 64 * (BC / 8)) store_pairs(sA, unit, ra[u][0], ra[u][1]);
    }
#pragma unroll
    for (int u = 0; u < D_UNITS; ++u) {
      const int unit = tid + u * 256;
      if (unit < 64 * (BN / 8)) store_pairs(sD, unit, rd[u][0], rd[u][1]);
    }
  };

  const int frag_row = lane & 15, frag_m = wave * 32 + (lane >> 4) * 8;
  if (m_begin < m_end) load_step(m_begin);
  for (int m0 = m_begin; m0 < m_end; m0 += MC) {
    __syncthreads();  // previous step's LDS reads are done
    store_step();
    __syncthreads();
    if (m0 + MC < m_end) load_step(m0 + MC);
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

  // sum the four waves through LDS, then one atomic per output element
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

}  // namespace hpf
