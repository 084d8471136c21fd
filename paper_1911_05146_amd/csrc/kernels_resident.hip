// Image-resident forward and backward kernels for runs of identity bottleneck blocks (bf16 mode).
//
// A partition of a deep pre-activation ResNet (paper Section "Model Generator" / Table of models:
// ResNet-110 ... ResNet-1001) is mostly a long run of identical blocks at one resolution.  At CIFAR
// resolutions a whole image of the residual stream fits in one CU's LDS (16x16x128 bf16 = 64 KiB), so
// one work-group keeps "its" image resident for the whole run: per block it only reads the weights and
// writes what back-propagation needs later (the BatchNorm inputs c1, c2, y).  The backward kernel walks
// the run in reverse with the gradient of the residual stream resident instead.
//
// BatchNorm uses the statistics of the micro-batch, so the work-groups of one micro-batch exchange small
// per-image records three times per block and direction.  The exchange is an all-gather through device
// memory in which every float travels in one 8-byte word together with the tag of its phase: the words
// are written and polled with single-copy-atomic device-scope accesses, so a reader that sees the tag
// has the value, and no cache write-back or invalidate is needed.  Merges run in a fixed order in every
// work-group, so all of them derive bit-identical statistics.
//
// All work-groups of a micro-batch must be on the chip together; the launchers check the grid against
// the number of CUs, and a bounded spin turns a missing partner into an error flag instead of a hang.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "hpf_device.h"

namespace hpf {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned long long u64;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int RES_NT = 512;            // threads per work-group (8 waves)
constexpr int RES_NWV = RES_NT / 64;
constexpr unsigned RES_SPIN_LIMIT = 1u << 19;

// The wave's index within the work-group as a scalar: conditions on it become scalar branches instead of
// compare / exec-mask sequences.
__device__ __forceinline__ int wave_index() { return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)); }

__device__ __forceinline__ float bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// {scale, shift} of a BatchNorm channel: bn(x) = x*scale + shift
__device__ __forceinline__ float2 bn_scale_shift(float mean, float invstd, float gamma, float beta) {
  const float sc = gamma * invstd;
  return make_float2(sc, fmaf(-mean, sc, beta));
}

// Sums within a row of 16 lanes by DPP row rotations (one VALU instruction per step, no LDS round trip).
// row_sum<N>(v): every lane gets the sum over the lanes of its row that are congruent to it modulo N.
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
template <int N>
__device__ __forceinline__ float row_sum(float v) {
  static_assert(N == 1 || N == 2 || N == 4 || N == 8 || N == 16, "N divides 16");
  if (N <= 8) v += dpp_mov<0x128>(v);   // row_ror:8
  if (N <= 4) v += dpp_mov<0x124>(v);   // row_ror:4
  if (N <= 2) v += dpp_mov<0x122>(v);   // row_ror:2
  if (N <= 1) v += dpp_mov<0x121>(v);   // row_ror:1
  return v;
}
__device__ __forceinline__ float sum16(float v) { return row_sum<1>(v); }   // over the 16 pixels of a tile

// ---- tiles: a [P][Cc] bf16 image in LDS has row stride Cc + 8 (16-byte reads of 16 consecutive rows hit distinct banks)
template <int Cc>
__device__ __forceinline__ void tile_load(bf16_t* s, const bf16_t* g, int P) {
  constexpr int U = Cc / 8;
  for (int u = threadIdx.x; u < P * U; u += RES_NT) {
    const int row = u / U, col = u - row * U;
    *reinterpret_cast<uint4*>(s + row * (Cc + 8) + col * 8) = *reinterpret_cast<const uint4*>(g + (size_t)u * 8);
  }
}
template <int Cc>
__device__ __forceinline__ void tile_store(bf16_t* g, const bf16_t* s, int P) {
  constexpr int U = Cc / 8;
  for (int u = threadIdx.x; u < P * U; u += RES_NT) {
    const int row = u / U, col = u - row * U;
    // streaming store: the tensor is read again only by the backward pass, long after it has left the caches
    __builtin_nontemporal_store(*reinterpret_cast<const u32x4*>(s + row * (Cc + 8) + col * 8), reinterpret_cast<u32x4*>(g + (size_t)u * 8));
  }
}
// All `nmem` work-groups of a micro-batch publish `nw` floats each and collect everybody's in
// gath[m*nw + w] (LDS).  The two halves are separate so that independent work can fill the flight time.
__device__ __forceinline__ void publish_word(u64* slot, int me, int nw, int w, float v, unsigned tag) {
  __hip_atomic_store(slot + (size_t)me * nw + w, ((u64)tag << 32) | (u64)__float_as_uint(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Returns false, uniformly over the work-group, when a partner did not show up.  Ends with a barrier.
// INFL: words in flight per thread and polling round (a micro-batch of 32 images exchanges 4 words per thread
// for the narrow tensors, 16 for the wide ones: one round each).
// MASKED: a word that has arrived is not asked for again, so the later rounds of a wide exchange move a few words
// instead of all (measured: 1 % on the backward launch, where the polls share the memory pipeline with the loads
// of the stashed tensors; the forward launch is 1 % faster re-reading everything with straight-line code).
template <int INFL, bool MASKED = false>
__device__ __forceinline__ bool collect(const u64* slot, int nmem, int nw, unsigned tag, float* gath, int* abort_flag) {
  const int total = nmem * nw;
  int timed_out = 0;
  for (int i0 = threadIdx.x; i0 < total; i0 += RES_NT * INFL) {
    u64 v[INFL];
    unsigned spins = 0;
    if (MASKED) {
      unsigned missing = 0;
#pragma unroll
      for (int i = 0; i < INFL; ++i)
        if (i0 + i * RES_NT < total) missing |= 1u << i;
      for (;;) {
#pragma unroll
        for (int i = 0; i < INFL; ++i)
          if (missing >> i & 1u) v[i] = __hip_atomic_load(slot + i0 + i * RES_NT, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int i = 0; i < INFL; ++i)
          if ((missing >> i & 1u) && (unsigned)(v[i] >> 32) == tag) missing &= ~(1u << i);
        if (!missing) break;
        if (++spins > RES_SPIN_LIMIT) { timed_out = 1; break; }
      }
    } else {
      for (;;) {
        bool all = true;
#pragma unroll
        for (int i = 0; i < INFL; ++i)
          if (i0 + i * RES_NT < total) v[i] = __hip_atomic_load(slot + i0 + i * RES_NT, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int i = 0; i < INFL; ++i)
          if (i0 + i * RES_NT < total) all = all && (unsigned)(v[i] >> 32) == tag;
        if (all) break;
        if (++spins > RES_SPIN_LIMIT) { timed_out = 1; break; }
      }
    }
#pragma unroll
    for (int i = 0; i < INFL; ++i)
      if (i0 + i * RES_NT < total) gath[i0 + i * RES_NT] = __uint_as_float((unsigned)v[i]);
  }
  const int any = __syncthreads_or(timed_out);
  if (any && threadIdx.x == 0) atomicExch(abort_flag, 1);
  return any == 0;
}
// Gathered per-image {mean, M2} (equal pixel counts) -> micro-batch mean / invstd -> coef[c] = {scale, shift}.
// The 32 rows of 16 lanes of the work-group take Cc/32 channels each, the lanes of a row split the members
// and combine by row rotations: the same arithmetic in the same order in every work-group.  stats_out
// (member 0 only) receives {mean(Cc), invstd(Cc)} for the backward pass and the weight gradients.
// Ends with a barrier.
template <int Cc>
__device__ __forceinline__ void merge_coef(const float* gath, int nmem, int P, float eps, const float* gamma, const float* beta,
                                           float2* coef, float* stats_out) {
  constexpr int CR = Cc >= 32 ? Cc / 32 : 1;   // channels per row (below 32 channels only the first Cc rows work)
  constexpr int MP = 16 / CR;        // member subsets per row
  const int l16 = threadIdx.x & 15, row = threadIdx.x >> 4;
  const bool act = row * CR < Cc;
  const int c = act ? row * CR + l16 % CR : 0, part = l16 / CR;
  const float g = gamma[c], b = beta[c];
  float s = 0.f;
  for (int m = part; m < nmem; m += MP) s += gath[m * 2 * Cc + c];
  s = row_sum<CR>(s);
  const float inv_n = 1.f / (float)nmem;
  const float mean = s * inv_n;
  float s2 = 0.f;
  for (int m = part; m < nmem; m += MP) {
    const float d = gath[m * 2 * Cc + c] - mean;
    s2 += gath[m * 2 * Cc + Cc + c] + (float)P * d * d;
  }
  s2 = row_sum<CR>(s2);
  if (act && part == 0) {
    const float var = s2 * inv_n / (float)P;
    const float is = 1.0f / sqrtf(var + eps);
    coef[c] = bn_scale_shift(mean, is, g, b);
    if (stats_out) { stats_out[c] = mean; stats_out[Cc + c] = is; }
  }
  __syncthreads();
}

__device__ __forceinline__ bf16x8 frag_bn_relu(const uint4& q, const float2 (&cf)[8]) {
  const uint32_t w[4] = {q.x, q.y, q.z, q.w};
  uint32_t r[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    r[i] = pack_bf16x2(fmaxf(fmaf(bf_lo(w[i]), cf[2 * i].x, cf[2 * i].y), 0.f),
                       fmaxf(fmaf(bf_hi(w[i]), cf[2 * i + 1].x, cf[2 * i + 1].y), 0.f));
  return __builtin_bit_cast(bf16x8, make_uint4(r[0], r[1], r[2], r[3]));
}
__device__ __forceinline__ bf16x8 frag_zero() { return __builtin_bit_cast(bf16x8, make_uint4(0u, 0u, 0u, 0u)); }
__device__ __forceinline__ uint2 pack4(const floatx4& v) { return make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])); }
__device__ __forceinline__ float elem4(const uint2& q, int e) {
  return e == 0 ? bf_lo(q.x) : e == 1 ? bf_hi(q.x) : e == 2 ? bf_lo(q.y) : bf_hi(q.y);
}
struct ResCtx {
  char* base; void* act_in; void* act_out; void* err_in; void* err_out;
  __device__ __forceinline__ bf16_t* tensor(unsigned long long off) const {
    void* p = base + off;
    p = off == RES_ACT_IN ? act_in : p;
    p = off == RES_ACT_OUT ? act_out : p;
    p = off == RES_ERR_IN ? err_in : p;
    p = off == RES_ERR_OUT ? err_out : p;
    return (bf16_t*)p;
  }
};

// Weight fragments of one GEMM as the first MFMA operand: fragment (kt, nt) holds rows nt*16..+15 and
// k = kt*32..+31 of a row-major [rows][ld] bf16 matrix.  PRE = true keeps all fragments in registers, loaded
// where load() is called (ahead of an exchange, so the memory latency hides behind the wait); PRE = false
// fetches each fragment where it is used.
template <int KT, int NT, bool PRE>
struct WFrags;
template <int KT, int NT>
struct WFrags<KT, NT, true> {
  static constexpr bool pre = true, staged = false;
  bf16x8 r[KT][NT];
  __device__ __forceinline__ void load(const bf16_t* w, int ld, int fr, int fk) {
#pragma unroll
    for (int kt = 0; kt < KT; ++kt)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) r[kt][nt] = *reinterpret_cast<const bf16x8*>(w + (size_t)(nt * 16 + fr) * ld + kt * 32 + fk);
  }
  __device__ __forceinline__ bf16x8 get(int kt, int nt) const { return r[kt][nt]; }
};
template <int KT, int NT>
struct WFrags<KT, NT, false> {
  static constexpr bool pre = false, staged = false;
  const bf16_t* w; int ld, fr, fk;
  __device__ __forceinline__ void load(const bf16_t* w_, int ld_, int fr_, int fk_) { w = w_; ld = ld_; fr = fr_; fk = fk_; }
  __device__ __forceinline__ bf16x8 get(int kt, int nt) const {
    return *reinterpret_cast<const bf16x8*>(w + (size_t)(nt * 16 + fr) * ld + kt * 32 + fk);
  }
};

// Third form: the fragments come from an LDS copy of the matrix that the whole work-group stages once.  load()
// only asks for this thread's 16-byte units (into registers, ahead of an exchange); commit() stores them to the
// LDS area behind the wait, when every wave has finished with the matrix staged before (the caller puts a barrier
// between the last get() of the old matrix and commit(), and one between commit() and the first get()).  With
// weights fetched where they are used every reduction step is an L2 round trip that nothing hides when a wave has
// one pixel tile to work on; from LDS a step costs an LDS read.  Rows are KT*32 long (the packed matrix is exactly
// that wide) and padded by 8 elements in LDS: 16 consecutive rows start in 16 different bank groups.
template <int KT, int NT>
struct WFragsL {
  static constexpr bool pre = true;    // get() takes constants only (the same loop shapes as the register form)
  static constexpr bool staged = true;
  static constexpr int ROWS = NT * 16, LEN = KT * 32, STRIDE = LEN + 8, UNITS = ROWS * LEN / 8, NU = (UNITS + RES_NT - 1) / RES_NT;
  const bf16_t* s;
  int fr, fk;
  // st: the thread's staging registers, shared by the matrices of a block (one is in flight at a time)
  template <int N>
  __device__ __forceinline__ void issue(u32x4 (&st)[N], const bf16_t* w, int fr_, int fk_) {
    static_assert(NU <= N, "staging registers");
    fr = fr_; fk = fk_;
#pragma unroll
    for (int i = 0; i < NU; ++i) {
      const int u = threadIdx.x + i * RES_NT;
      st[i] = *reinterpret_cast<const u32x4*>(w + (size_t)(u < UNITS ? u : 0) * 8);   // the packed matrix is contiguous
    }
  }
  template <int N>
  __device__ __forceinline__ void commit(const u32x4 (&st)[N], bf16_t* sw) {
    s = sw;
#pragma unroll
    for (int i = 0; i < NU; ++i) {
      const int u = threadIdx.x + i * RES_NT;
      if (u < UNITS) {
        const int row = u / (LEN / 8), col = u - row * (LEN / 8);
        *reinterpret_cast<u32x4*>(sw + row * STRIDE + col * 8) = st[i];
      }
    }
  }
  // a column block of a wider matrix (rows ld apart), into / from the staging registers st[OFF .. OFF+NU)
  template <int OFF, int N>
  __device__ __forceinline__ void issue_cols(u32x4 (&st)[N], const bf16_t* w, int ld, int fr_, int fk_) {
    static_assert(OFF + NU <= N, "staging registers");
    fr = fr_; fk = fk_;
#pragma unroll
    for (int i = 0; i < NU; ++i) {
      const int u = threadIdx.x + i * RES_NT, uu = u < UNITS ? u : 0;
      const int row = uu / (LEN / 8), col = uu - row * (LEN / 8);
      st[OFF + i] = *reinterpret_cast<const u32x4*>(w + (size_t)row * ld + col * 8);
    }
  }
  template <int OFF, int N>
  __device__ __forceinline__ void commit_from(const u32x4 (&st)[N], bf16_t* sw) {
    s = sw;
#pragma unroll
    for (int i = 0; i < NU; ++i) {
      const int u = threadIdx.x + i * RES_NT;
      if (u < UNITS) {
        const int row = u / (LEN / 8), col = u - row * (LEN / 8);
        *reinterpret_cast<u32x4*>(sw + row * STRIDE + col * 8) = st[OFF + i];
      }
    }
  }
  __device__ __forceinline__ bf16x8 get(int kt, int nt) const {
    return *reinterpret_cast<const bf16x8*>(s + (nt * 16 + fr) * STRIDE + kt * 32 + fk);
  }
};
// issue / commit for any form: the register and fetch-where-used forms load at once and have nothing to commit
template <class WF, int N>
__device__ __forceinline__ void w_issue(WF& w, u32x4 (&st)[N], const bf16_t* p, int ld, int fr, int fk) {
  if constexpr (WF::staged) w.issue(st, p, fr, fk);
  else w.load(p, ld, fr, fk);
}
template <class WF, int N>
__device__ __forceinline__ void w_commit(WF& w, const u32x4 (&st)[N], bf16_t* sw) {
  if constexpr (WF::staged) w.commit(st, sw);
}

// 3x3 convolution (stride 1, zero padding) of a [P][MID] tile in LDS, both directions:
//   forward : out(p,q) += src(p+r-1, q+s-1) * W[r][s]       weights [MID][9*MID], k = tap*MID + c
//   backward: out(p,q) += src(p+1-r, q+1-s) * W[r][s]^T     weights [MID][9*MID], k = tap*MID + n
// TAP0, NTAPS: the filter taps this call adds (wfr then holds the columns of these taps only, from k = 0).
template <int MID, int PTW, bool BACKWARD, int TAP0 = 0, int NTAPS = 9, class WF>
__device__ __forceinline__ void conv3x3_tile(const bf16_t* src, const WF& wfr, int H, int W, int npt, int wave, int fr, int fk,
                                             floatx4 (&acc)[PTW][MID / 16]) {
  constexpr int MS = MID + 8;
  int py[PTW], px[PTW];
#pragma unroll
  for (int j = 0; j < PTW; ++j) {
    const int p = (wave + j * RES_NWV) * 16 + fr;
    py[j] = p / W;
    px[j] = p - py[j] * W;
  }
  if constexpr (MID == 16) {
    // 16 channels per tap fill half an MFMA step: a step covers two taps, lane groups 0-1 the first and 2-3 the second
    // (the packed weights [16][160] have k = tap*16 + channel contiguous and are zero beyond k = 144)
    const int fq = fk >> 3, c8 = (fq & 1) * 8;
    auto step = [&](int st) {
      const int tap = 2 * st + (fq >> 1);
      const int r = tap / 3, s = tap - r * 3;
      const int dh = BACKWARD ? 1 - r : r - 1, dw = BACKWARD ? 1 - s : s - 1;
      const bf16x8 wf = wfr.get(st, 0);
#pragma unroll
      for (int j = 0; j < PTW; ++j) {
        if (wave + j * RES_NWV < npt) {
          const int hs = py[j] + dh, ws = px[j] + dw;
          const bool ok = tap < 9 && (unsigned)hs < (unsigned)H && (unsigned)ws < (unsigned)W;
          const int row = ok ? hs * W + ws : 0;
          bf16x8 bfrag = *reinterpret_cast<const bf16x8*>(src + row * MS + c8);
          if (!ok) bfrag = frag_zero();
          acc[j][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, bfrag, acc[j][0], 0, 0, 0);
        }
      }
    };
    if constexpr (WF::pre && !WF::staged) {   // fragments in registers: the step index must be a constant
#pragma unroll
      for (int st = 0; st < 5; ++st) step(st);
    } else {                   // fetched where used or read from LDS: a rolled loop keeps the addresses of 40 operand reads out of the registers
#pragma unroll 1
      for (int st = 0; st < 5; ++st) step(st);
    }
    return;
  }
#pragma unroll
  for (int tap = TAP0; tap < TAP0 + NTAPS; ++tap) {
    const int r = tap / 3, s = tap % 3;
    const int dh = BACKWARD ? 1 - r : r - 1, dw = BACKWARD ? 1 - s : s - 1;
#pragma unroll
    for (int ks = 0; ks < MID / 32; ++ks) {
      bf16x8 wf[MID / 16];
#pragma unroll
      for (int nt = 0; nt < MID / 16; ++nt) wf[nt] = wfr.get((tap - TAP0) * (MID / 32) + ks, nt);
#pragma unroll
      for (int j = 0; j < PTW; ++j) {
        if (wave + j * RES_NWV < npt) {
          const int hs = py[j] + dh, ws = px[j] + dw;
          const bool ok = (unsigned)hs < (unsigned)H && (unsigned)ws < (unsigned)W;
          const int row = ok ? hs * W + ws : 0;
          bf16x8 bfrag = *reinterpret_cast<const bf16x8*>(src + row * MS + ks * 32 + fk);
          if (!ok) bfrag = frag_zero();
#pragma unroll
          for (int nt = 0; nt < MID / 16; ++nt) acc[j][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[nt], bfrag, acc[j][nt], 0, 0, 0);
        }
      }
    }
  }
}

// Per-channel {mean, M2} of this image's [P][Cc] tile, published as the work-group's record (words c and
// Cc + c).  Sums are taken about the first pixel's value, so a large common offset does not cancel.
// A row of 16 lanes reads one 16-byte unit (8 channels) of 16 consecutive pixels at a time and sums by row
// rotations; the 32 rows of the work-group cover the U units of a pixel times 32/U pixel groups.
template <int Cc>
__device__ __forceinline__ void stats_publish(const bf16_t* s, int P, float* red, u64* slot, int me, unsigned tag) {
  constexpr int U = Cc / 8;          // 16-byte units per pixel
  constexpr int NG = 32 / U;         // pixel groups (of 16 pixels per step)
  static_assert(U <= 32 && 32 % U == 0, "unit count");
  const int l16 = threadIdx.x & 15, row = threadIdx.x >> 4;
  const int unit = row % U, grp = row / U;
  float K[8], s1[8], s2[8];
  load8(s + unit * 8, K);
#pragma unroll
  for (int i = 0; i < 8; ++i) { s1[i] = 0.f; s2[i] = 0.f; }
  for (int p = grp * 16 + l16; p < P; p += NG * 16) {
    float v[8];
    load8(s + p * (Cc + 8) + unit * 8, v);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float d = v[i] - K[i];
      s1[i] += d;
      s2[i] = fmaf(d, d, s2[i]);
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) { s1[i] = row_sum<1>(s1[i]); s2[i] = row_sum<1>(s2[i]); }
  if (l16 == 0) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      red[grp * 2 * Cc + unit * 8 + i] = s1[i];
      red[grp * 2 * Cc + Cc + unit * 8 + i] = s2[i];
    }
  }
  __syncthreads();
  if (threadIdx.x < Cc) {
    const int c = threadIdx.x;
    float S1 = 0.f, S2 = 0.f;
#pragma unroll
    for (int i = 0; i < NG; ++i) { S1 += red[i * 2 * Cc + c]; S2 += red[i * 2 * Cc + Cc + c]; }
    const float inv = 1.f / (float)P;
    publish_word(slot, me, 2 * Cc, c, bf16_to_f32(s[c]) + S1 * inv, tag);
    publish_word(slot, me, 2 * Cc, Cc + c, fmaxf(S2 - S1 * S1 * inv, 0.f), tag);
  }
}

// in place: s = relu(s*scale + shift)
template <int Cc>
__device__ __forceinline__ void tile_bn_relu(bf16_t* s, const float2* coef, int P) {
  constexpr int U = Cc / 8;
  for (int u = threadIdx.x; u < P * U; u += RES_NT) {
    const int row = u / U, col = u - row * U;
    uint4* q = reinterpret_cast<uint4*>(s + row * (Cc + 8) + col * 8);
    const uint4 v = *q;
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    const float4* cf = reinterpret_cast<const float4*>(coef + col * 8);
    uint32_t r[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float4 k = cf[i];
      r[i] = pack_bf16x2(fmaxf(fmaf(bf_lo(w[i]), k.x, k.y), 0.f), fmaxf(fmaf(bf_hi(w[i]), k.z, k.w), 0.f));
    }
    *q = make_uint4(r[0], r[1], r[2], r[3]);
  }
}

// Inference: a BatchNorm is the fixed map of its running statistics run = {mean(Cc), variance(Cc)}: no
// statistics are taken and nothing is exchanged.  Ends with a barrier.
template <int Cc>
__device__ __forceinline__ void running_coef(float2* coef, const float* run, const float* gamma, const float* beta, float eps) {
  for (int c = threadIdx.x; c < Cc; c += RES_NT) coef[c] = bn_scale_shift(run[c], 1.0f / sqrtf(run[Cc + c] + eps), gamma[c], beta[c]);
  __syncthreads();
}

// ------------------------------------------------------------------------------------------ forward
// PTW: pixel tiles (16 pixels) per wave, i.e. images of up to 16*PTW*RES_NWV pixels.
// PRE: weight fragments are preloaded into registers ahead of the exchanges (needs the register room).
// INFER: inference forward (BatchNorm by running statistics): the images are independent, nothing is stashed and
// only the output of the last block is written.
// HW: 0 = image height and width from the arguments; 16 = 16 x 16 pixels as compile-time constants in the 3x3 convolution
// (the shape of the benchmark partition: pixel-row decodes and tap addresses become shifts).
// WL: the weights go through LDS (WFragsL).  1: into an area of their own, for shapes with LDS to spare (256-64 at 8x8).
// 2: into the MID-wide tile that is idle at the time (128-64 at 16x16, whose tiles fill the LDS: eight waves fetching
// the same 106 KB of weights per block from L2 were what bound that shape): conv1's matrix goes to the c2 tile (dead
// since the conv3 before), conv3's to the c1 tile (dead since conv2), conv2's in three rounds of three filter taps to
// the c2 tile, which the convolution only writes when all rounds are done.
template <int C, int MID, int PTW, bool PRE, bool INFER = false, int HW = 0, int WL = 0>
__global__ void __launch_bounds__(RES_NT) k_res_forward(const ResArgs a, const int gath_own) {
  static_assert(!(WL && (PRE || INFER)), "the LDS form replaces the fetch-where-used form of the training kernels");
  constexpr bool WT = WL == 2;   // staged in the tiles that are idle at the time
  constexpr int XS = C + 8, MS = MID + 8;
  const int tid = threadIdx.x, lane = tid & 63, wave = wave_index();
  const int fr = lane & 15, fq = lane >> 4, fk = fq * 8;
  const int H = HW ? HW : a.H, W = HW ? HW : a.W;   // constants in the pixel-row arithmetic of the 3x3 convolution only:
  const int P = a.H * a.W, npt = P >> 4;           // with constant trip counts the tile loops unroll into register spills
  // work-groups are dealt to the XCDs round-robin by linear id: with g == 8 micro-batch z lives on XCD z
  const int z = blockIdx.x % a.ngroup, me = blockIdx.x / a.ngroup;
  ResCtx cx{(char*)pick(a.base, z), pick(a.act_in, z), pick(a.act_out, z), pick(a.err_in, z), pick(a.err_out, z)};
  u64* xchg = reinterpret_cast<u64*>(cx.base + a.xchg_off);
  unsigned* tagp = reinterpret_cast<unsigned*>(cx.base + a.tag_off);
  const unsigned tag0 = *tagp;
  unsigned phase = 0;

  extern __shared__ __align__(16) unsigned char smem[];
  bf16_t* sx = reinterpret_cast<bf16_t*>(smem);           // residual stream of the image, [P][XS]
  bf16_t* smA = sx + (size_t)P * XS;                      // c1, then relu(bn2(c1))
  bf16_t* smB = smA + (size_t)P * MS;                     // c2, then relu(bn3(c2))
  float2* coefC = reinterpret_cast<float2*>(smB + (size_t)P * MS);
  float2* coefM = coefC + C;
  float* red = reinterpret_cast<float*>(coefM + MID);     // RES_NWV * 2*C floats
  float* own = red + RES_NWV * 2 * C;                     // gather area of its own when the tiles are too small
  float* gathA = gath_own ? own : reinterpret_cast<float*>(smA);
  float* gathB = gath_own ? own : reinterpret_cast<float*>(smB);
  auto slot = [&]() { return xchg + (size_t)(phase & 1u) * a.nmem * (2 * C); };

  std::conditional_t<WL != 0, WFragsL<C / 32, MID / 16>, WFrags<C / 32, MID / 16, PRE>> w1;            // conv1 [MID][C]
  std::conditional_t<WL == 1, WFragsL<9 * MID / 32, MID / 16>,
                     std::conditional_t<WT, WFragsL<3 * MID / 32, MID / 16>, WFrags<9 * MID / 32, MID / 16, PRE>>> w2;  // conv2 [MID][9*MID] (WT: three taps of it)
  std::conditional_t<WL != 0, WFragsL<MID / 32, C / 16>, WFrags<MID / 32, C / 16, PRE>> w3;            // conv3 [C][MID]
  bf16_t* sW = reinterpret_cast<bf16_t*>(own + (gath_own ? (size_t)a.nmem * 2 * C : 0));   // WL == 1: the staged matrix
  bf16_t* const sW1 = WT ? smB : sW;
  bf16_t* const sW3 = WT ? smA : sW;
  // the C-wide records of a large micro-batch (more than 36 images at 128 channels) reach from the c1 tile into the c2
  // tile: conv1's matrix then goes there only when they have been merged (one more barrier per block)
  const bool w1_late = WT && !gath_own && (size_t)a.nmem * 2 * C * sizeof(float) > (size_t)P * MS * sizeof(bf16_t);
  constexpr int W2NU = (3 * MID * MID / 8 + RES_NT - 1) / RES_NT;                            // WT: units per thread and round
  u32x4 wst[WL == 1 ? (9 * MID / 32 * (MID / 16) + 7) / 8 : WT ? 3 * W2NU : 1];             // the units on their way
  static_assert(!WT || (MID * (C + 8) <= 256 * (MID + 8) && C * (MID + 8) <= 256 * (MID + 8) && MID * (3 * MID + 8) <= 256 * (MID + 8)),
                "the matrices fit a MID-wide tile of 256 pixels");

  {
    const ResBlock B0 = a.blocks[0];
    tile_load<C>(sx, cx.tensor(B0.x_off) + (size_t)me * P * C, P);
    w_issue(w1, wst, a.packed + B0.wf_off[0], C, fr, fk);
    __syncthreads();
    if (INFER) {
      running_coef<C>(coefC, a.running + B0.run_off[0], a.params + B0.gamma_off[0], a.params + B0.beta_off[0], a.eps);
    } else {
      stats_publish<C>(sx, P, red, slot(), me, tag0 + 1u + phase);
      if (!collect<16>(slot(), a.nmem, 2 * C, tag0 + 1u + phase, gathA, a.abort_flag)) return;
      ++phase;
      if (!w1_late) w_commit(w1, wst, sW1);   // the barrier at the end of the merge lies between this and conv1
      merge_coef<C>(gathA, a.nmem, P, a.eps, a.params + B0.gamma_off[0], a.params + B0.beta_off[0], coefC,
                    me == 0 ? reinterpret_cast<float*>(cx.base + B0.stats_off[0]) : nullptr);
      if (w1_late) {
        w_commit(w1, wst, sW1);
        __syncthreads();
      }
    }
  }

  for (int bi = 0; bi < a.nblk; ++bi) {
    const ResBlock B = a.blocks[bi];
    // ---- conv1 (1x1, C -> MID) on relu(bn1(x)), normalised while the operand is read from LDS
    {
      floatx4 acc[PTW][MID / 16];
#pragma unroll
      for (int j = 0; j < PTW; ++j)
#pragma unroll
        for (int nt = 0; nt < MID / 16; ++nt) acc[j][nt] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < C / 32; ++ks) {
        float2 cf[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) cf[i] = coefC[ks * 32 + fk + i];
        bf16x8 wf[MID / 16];
#pragma unroll
        for (int nt = 0; nt < MID / 16; ++nt) wf[nt] = w1.get(ks, nt);
#pragma unroll
        for (int j = 0; j < PTW; ++j) {
          const int pt = wave + j * RES_NWV;
          if (pt < npt) {
            const uint4 xv = *reinterpret_cast<const uint4*>(sx + (pt * 16 + fr) * XS + ks * 32 + fk);
            const bf16x8 bfrag = frag_bn_relu(xv, cf);
#pragma unroll
            for (int nt = 0; nt < MID / 16; ++nt) acc[j][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[nt], bfrag, acc[j][nt], 0, 0, 0);
          }
        }
      }
#pragma unroll
      for (int j = 0; j < PTW; ++j) {
        const int pt = wave + j * RES_NWV;
        if (pt < npt)
#pragma unroll
          for (int nt = 0; nt < MID / 16; ++nt)
            *reinterpret_cast<uint2*>(smA + (pt * 16 + fr) * MS + nt * 16 + fq * 4) = pack4(acc[j][nt]);
      }
    }
    if constexpr (WT) {   // all three rounds are asked for now: the exchange below hides the latency
      w2.template issue_cols<0>(wst, a.packed + B.wf_off[1], 9 * MID, fr, fk);
      w2.template issue_cols<W2NU>(wst, a.packed + B.wf_off[1] + 3 * MID, 9 * MID, fr, fk);
      w2.template issue_cols<2 * W2NU>(wst, a.packed + B.wf_off[1] + 6 * MID, 9 * MID, fr, fk);
    } else {
      w_issue(w2, wst, a.packed + B.wf_off[1], 9 * MID, fr, fk);
    }
    __syncthreads();
    if (INFER) {
      running_coef<MID>(coefM, a.running + B.run_off[1], a.params + B.gamma_off[1], a.params + B.beta_off[1], a.eps);
    } else {
      stats_publish<MID>(smA, P, red, slot(), me, tag0 + 1u + phase);
      if (!collect<4>(slot(), a.nmem, 2 * MID, tag0 + 1u + phase, gathB, a.abort_flag)) return;
      tile_store<MID>(cx.tensor(B.c1_off) + (size_t)me * P * MID, smA, P);   // after the polls (measured: 2 % faster than before them)
      ++phase;
      if constexpr (!WT) w_commit(w2, wst, sW);   // conv1 is behind the barrier above the statistics; conv2 behind the ones below
      merge_coef<MID>(gathB, a.nmem, P, a.eps, a.params + B.gamma_off[1], a.params + B.beta_off[1], coefM,
                      me == 0 ? reinterpret_cast<float*>(cx.base + B.stats_off[1]) : nullptr);
      if constexpr (WT) w2.template commit_from<0>(wst, smB);   // the gathered records in that tile are behind the merge's barrier
    }
    tile_bn_relu<MID>(smA, coefM, P);   // once, not per filter tap
    __syncthreads();
    // ---- conv2 (3x3, MID -> MID)
    {
      floatx4 acc[PTW][MID / 16];
#pragma unroll
      for (int j = 0; j < PTW; ++j)
#pragma unroll
        for (int nt = 0; nt < MID / 16; ++nt) acc[j][nt] = floatx4{0.f, 0.f, 0.f, 0.f};
      if constexpr (WT) {   // a barrier on either side of every re-staging; the last one frees the tile for the output
        conv3x3_tile<MID, PTW, false, 0, 3>(smA, w2, H, W, npt, wave, fr, fk, acc);
        __syncthreads();
        w2.template commit_from<W2NU>(wst, smB);
        __syncthreads();
        conv3x3_tile<MID, PTW, false, 3, 3>(smA, w2, H, W, npt, wave, fr, fk, acc);
        __syncthreads();
        w2.template commit_from<2 * W2NU>(wst, smB);
        __syncthreads();
        conv3x3_tile<MID, PTW, false, 6, 3>(smA, w2, H, W, npt, wave, fr, fk, acc);
        __syncthreads();
      } else {
        conv3x3_tile<MID, PTW, false>(smA, w2, H, W, npt, wave, fr, fk, acc);
      }
#pragma unroll
      for (int j = 0; j < PTW; ++j) {
        const int pt = wave + j * RES_NWV;
        if (pt < npt)
#pragma unroll
          for (int nt = 0; nt < MID / 16; ++nt)
            *reinterpret_cast<uint2*>(smB + (pt * 16 + fr) * MS + nt * 16 + fq * 4) = pack4(acc[j][nt]);
      }
    }
    w_issue(w3, wst, a.packed + B.wf_off[2], MID, fr, fk);
    __syncthreads();
    if (INFER) {
      running_coef<MID>(coefM, a.running + B.run_off[2], a.params + B.gamma_off[2], a.params + B.beta_off[2], a.eps);
    } else {
      stats_publish<MID>(smB, P, red, slot(), me, tag0 + 1u + phase);
      if (!collect<4>(slot(), a.nmem, 2 * MID, tag0 + 1u + phase, gathA, a.abort_flag)) return;
      tile_store<MID>(cx.tensor(B.c2_off) + (size_t)me * P * MID, smB, P);
      ++phase;
      if constexpr (!WT) w_commit(w3, wst, sW);
      merge_coef<MID>(gathA, a.nmem, P, a.eps, a.params + B.gamma_off[2], a.params + B.beta_off[2], coefM,
                      me == 0 ? reinterpret_cast<float*>(cx.base + B.stats_off[2]) : nullptr);
      if constexpr (WT) {   // into the tile the records were gathered in: behind the merge's barrier, and one before conv3
        w_commit(w3, wst, sW3);
        __syncthreads();
      }
    }
    // ---- conv3 (1x1, MID -> C) on relu(bn3(c2)) + residual: y = x + branch, written over x in LDS
    {
      bf16x8 bfrag[PTW][MID / 32];
#pragma unroll
      for (int ks = 0; ks < MID / 32; ++ks) {
        float2 cf[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) cf[i] = coefM[ks * 32 + fk + i];
#pragma unroll
        for (int j = 0; j < PTW; ++j) {
          const int pt = wave + j * RES_NWV;
          bfrag[j][ks] = pt < npt ? frag_bn_relu(*reinterpret_cast<const uint4*>(smB + (pt * 16 + fr) * MS + ks * 32 + fk), cf) : frag_zero();
        }
      }
#pragma unroll
      for (int nt = 0; nt < C / 16; ++nt) {
#pragma unroll
        for (int j = 0; j < PTW; ++j) {
          const int pt = wave + j * RES_NWV;
          if (pt < npt) {
            floatx4 acc = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < MID / 32; ++ks) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w3.get(ks, nt), bfrag[j][ks], acc, 0, 0, 0);
            uint2* q = reinterpret_cast<uint2*>(sx + (pt * 16 + fr) * XS + nt * 16 + fq * 4);
            const uint2 xr = *q;
            acc[0] += bf_lo(xr.x); acc[1] += bf_hi(xr.x); acc[2] += bf_lo(xr.y); acc[3] += bf_hi(xr.y);
            *q = pack4(acc);
          }
        }
      }
    }
    const bool more = bi + 1 < a.nblk;
    const ResBlock Bn = a.blocks[more ? bi + 1 : bi];
    if (more) w_issue(w1, wst, a.packed + Bn.wf_off[0], C, fr, fk);
    __syncthreads();
    if (INFER) {
      if (more) running_coef<C>(coefC, a.running + Bn.run_off[0], a.params + Bn.gamma_off[0], a.params + Bn.beta_off[0], a.eps);
      else tile_store<C>(cx.tensor(B.y_off) + (size_t)me * P * C, sx, P);
      continue;
    }
    if (more) stats_publish<C>(sx, P, red, slot(), me, tag0 + 1u + phase);
    tile_store<C>(cx.tensor(B.y_off) + (size_t)me * P * C, sx, P);   // while the records travel (measured: better before the polls)
    if (more) {
      if (!collect<16>(slot(), a.nmem, 2 * C, tag0 + 1u + phase, gathA, a.abort_flag)) return;
      ++phase;
      if (!w1_late) w_commit(w1, wst, sW1);
      merge_coef<C>(gathA, a.nmem, P, a.eps, a.params + Bn.gamma_off[0], a.params + Bn.beta_off[0], coefC,
                    me == 0 ? reinterpret_cast<float*>(cx.base + Bn.stats_off[0]) : nullptr);
      if (w1_late) {
        w_commit(w1, wst, sW1);
        __syncthreads();
      }
    }
  }
  // every member has read the counter before it took part in the first exchange, which member 0 has left
  if (!INFER && me == 0 && tid == 0) *tagp = tag0 + phase;
}

// ------------------------------------------------------------------------------------------ backward
// BatchNorm + ReLU backward on a gradient tile held in accumulator layout (lane: 4 channels of one pixel).
//   dz = da * [z > 0];  sums over the micro-batch {sum dz, sum dz*xhat} (all-gather);
//   out = scale * (dz - sum_dz/M - xhat * sum_dzxhat/M)  =  a1*dz + a2*x + a3  with per-channel a1..a3
// cf[c] = {scale, shift, invstd, -mean*invstd}; xin = the BatchNorm input at the same positions; tab = Cc
// float4 of LDS for {a1, a2, a3}.  fin(j, nt, out) receives the result tile by tile.  dgb (member 0 only,
// else null) receives the micro-batch sums {sum dz (Cc), sum dz*xhat (Cc)}: the gradients of beta and gamma, which
// the weight-gradient launch adds into the gradient buffer (as atomics here they cost member 0, and with it every
// exchange of its micro-batch, 13 us per launch of 21 blocks).
template <int Cc, int PTW, class Fin>
__device__ __forceinline__ bool bn_relu_bwd_acc(floatx4 (&dz)[PTW][Cc / 16], const uint2 (&xin)[PTW][Cc / 16], const float4* cf_,
                                                int npt, int wave, int fr, int fq, float* red, float4* tab_, float* gath,
                                                u64* slot, int me, int nmem, int P, unsigned tag, float* dgb,
                                                int* abort_flag, Fin&& fin, float* g_beta = nullptr, float* g_gamma = nullptr) {
  // g_beta / g_gamma (member 0 of runs without a weight-gradient launch of their own, else null): the sums are added
  // into the gradients of beta and gamma right here
  constexpr int NTL = Cc / 16;
  const float4* cf = reinterpret_cast<const float4*>(__builtin_assume_aligned(cf_, 16));
  float4* tab = reinterpret_cast<float4*>(__builtin_assume_aligned(tab_, 16));
#pragma unroll
  for (int nt = 0; nt < NTL; ++nt) {
    float4 k[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) k[e] = cf[nt * 16 + fq * 4 + e];
    float sb[4] = {0.f, 0.f, 0.f, 0.f}, sg[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < PTW; ++j) {
      if (wave + j * RES_NWV < npt) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float v = elem4(xin[j][nt], e);
          const float d = fmaf(v, k[e].x, k[e].y) > 0.f ? dz[j][nt][e] : 0.f;
          dz[j][nt][e] = d;
          sb[e] += d;
          sg[e] = fmaf(d, fmaf(v, k[e].z, k[e].w), sg[e]);
        }
      }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) { sb[e] = sum16(sb[e]); sg[e] = sum16(sg[e]); }
    if (fr == 0) {
      *reinterpret_cast<float4*>(red + wave * 2 * Cc + nt * 16 + fq * 4) = make_float4(sb[0], sb[1], sb[2], sb[3]);
      *reinterpret_cast<float4*>(red + wave * 2 * Cc + Cc + nt * 16 + fq * 4) = make_float4(sg[0], sg[1], sg[2], sg[3]);
    }
  }
  __syncthreads();
  for (int w = threadIdx.x; w < 2 * Cc; w += RES_NT) {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < RES_NWV; ++i) s += red[i * 2 * Cc + w];
    publish_word(slot, me, 2 * Cc, w, s, tag);
  }
  if (!collect<(Cc >= 128 ? 16 : 4), true>(slot, nmem, 2 * Cc, tag, gath, abort_flag)) return false;
  const float invM = 1.f / ((float)nmem * (float)P);
  {   // the 32 rows of 16 lanes take Cc/32 channels each (one each, on the first 16 rows, for 16 channels); the lanes of a row split the members (fixed order)
    constexpr int CR = Cc >= 32 ? Cc / 32 : 1, MP = 16 / CR;
    const int l16 = threadIdx.x & 15, row = threadIdx.x >> 4;
    const bool act = row * CR < Cc;
    const int c = act ? row * CR + l16 % CR : 0, part = l16 / CR;
    float sb = 0.f, sg = 0.f;
    for (int m = part; m < nmem; m += MP) { sb += gath[m * 2 * Cc + c]; sg += gath[m * 2 * Cc + Cc + c]; }
    sb = row_sum<CR>(sb);
    sg = row_sum<CR>(sg);
    if (act && part == 0) {
      if (dgb) { dgb[c] = sb; dgb[Cc + c] = sg; }
      if (g_beta) { atomicAdd(g_beta + c, sb); atomicAdd(g_gamma + c, sg); }
      const float4 k = cf[c];
      // scale*(dz - sb/M - (x*is + nm)*sg/M)
      tab[c] = make_float4(k.x, -k.x * sg * invM * k.z, -k.x * invM * (sb + k.w * sg), 0.f);
    }
  }
  __syncthreads();
#pragma unroll
  for (int nt = 0; nt < NTL; ++nt) {
    float4 t[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) t[e] = tab[nt * 16 + fq * 4 + e];
#pragma unroll
    for (int j = 0; j < PTW; ++j) {
      if (wave + j * RES_NWV < npt) {
        floatx4 out;
#pragma unroll
        for (int e = 0; e < 4; ++e) out[e] = fmaf(t[e].x, dz[j][nt][e], fmaf(t[e].y, elem4(xin[j][nt], e), t[e].z));
        fin(j, nt, out);
      }
    }
  }
  return true;
}

// What the backward pass of one block reads from memory besides the weights, fetched into registers ahead
// of use: c1 / c2 and the BatchNorm tables.  c1 / c2 are only needed at the accumulator positions of the
// BatchNorm backward, so they are read there straight from memory (8 bytes per lane) instead of being staged
// as whole tiles: two MID-wide tiles in LDS instead of four (128-64 blocks at 256 pixels would not fit
// otherwise), no tile stores, and 4 % less time per launch on 128-32 blocks.
template <int C, int MID, int PTW>
struct BwdLoads {
  uint2 x1[PTW][MID / 16], x2[PTW][MID / 16];   // c1 / c2 at this lane's accumulator positions
  float4 t1, t2, t3;
  __device__ __forceinline__ void issue(const ResBlock& B, const ResCtx& cx, const float* params, int me, int P, int npt, int wave,
                                        int fr, int fq) {
    const bf16_t* g1 = cx.tensor(B.c1_off) + (size_t)me * P * MID;
    const bf16_t* g2 = cx.tensor(B.c2_off) + (size_t)me * P * MID;
#pragma unroll
    for (int j = 0; j < PTW; ++j) {
      const int pt = wave + j * RES_NWV;
      const size_t row = (size_t)((pt < npt ? pt : 0) * 16 + fr) * MID + fq * 4;   // always a valid address
#pragma unroll
      for (int nt = 0; nt < MID / 16; ++nt) {
        x1[j][nt] = *reinterpret_cast<const uint2*>(g1 + row + nt * 16);
        x2[j][nt] = *reinterpret_cast<const uint2*>(g2 + row + nt * 16);
      }
    }
    const int c = threadIdx.x;
    t1 = table(reinterpret_cast<const float*>(cx.base + B.stats_off[0]), params + B.gamma_off[0], params + B.beta_off[0], c < C ? c : 0, C);
    t2 = table(reinterpret_cast<const float*>(cx.base + B.stats_off[1]), params + B.gamma_off[1], params + B.beta_off[1], c < MID ? c : 0, MID);
    t3 = table(reinterpret_cast<const float*>(cx.base + B.stats_off[2]), params + B.gamma_off[2], params + B.beta_off[2], c < MID ? c : 0, MID);
  }
  static __device__ __forceinline__ float4 table(const float* stats, const float* gamma, const float* beta, int c, int Cc) {
    const float mean = stats[c], is = stats[Cc + c];
    const float2 ss = bn_scale_shift(mean, is, gamma[c], beta[c]);
    return make_float4(ss.x, ss.y, is, -mean * is);
  }
  __device__ __forceinline__ void commit_tables(float4* cf1, float4* cf2, float4* cf3) const {
    const int c = threadIdx.x;
    if (c < C) cf1[c] = t1;
    if (c < MID) { cf2[c] = t2; cf3[c] = t3; }
  }
};

template <int C, int MID, int PTW, bool PRE, int HW = 0, int WL = 0>
__global__ void __launch_bounds__(RES_NT) k_res_backward(const ResArgs a, const int gath_own) {
  static_assert(!(WL && PRE), "the LDS form replaces the fetch-where-used form");
  // WL == 2: the matrices go to the idle MID-wide tile: conv3's and conv1's to the dc2 tile (idle between the conv2
  // contraction and the BN3 backward of the next block), conv2's in three rounds of three taps to the dc1 tile
  constexpr bool WT = WL == 2;
  constexpr int XS = C + 8, MS = MID + 8;
  const int tid = threadIdx.x, lane = tid & 63, wave = wave_index();
  const int fr = lane & 15, fq = lane >> 4, fk = fq * 8;
  const int H = HW ? HW : a.H, W = HW ? HW : a.W;   // constants in the pixel-row arithmetic of the 3x3 convolution only:
  const int P = a.H * a.W, npt = P >> 4;           // with constant trip counts the tile loops unroll into register spills
  // work-groups are dealt to the XCDs round-robin by linear id: with g == 8 micro-batch z lives on XCD z
  const int z = blockIdx.x % a.ngroup, me = blockIdx.x / a.ngroup;
  ResCtx cx{(char*)pick(a.base, z), pick(a.act_in, z), pick(a.act_out, z), pick(a.err_in, z), pick(a.err_out, z)};
  u64* xchg = reinterpret_cast<u64*>(cx.base + a.xchg_off);
  unsigned* tagp = reinterpret_cast<unsigned*>(cx.base + a.tag_off);
  const unsigned tag0 = *tagp;
  unsigned phase = 0;

  extern __shared__ __align__(16) unsigned char smem[];
  bf16_t* sdy = reinterpret_cast<bf16_t*>(smem);          // gradient of the residual stream, [P][XS]
  bf16_t* sm2 = sdy + (size_t)P * XS;                     // dc1
  bf16_t* sdc = sm2 + (size_t)P * MS;                     // dc2
  float4* cf1 = reinterpret_cast<float4*>(sdc + (size_t)P * MS);
  float4* cf2 = cf1 + C;
  float4* cf3 = cf2 + MID;
  float* red = reinterpret_cast<float*>(cf3 + MID);       // RES_NWV * 2*C floats
  float4* tab = reinterpret_cast<float4*>(red + RES_NWV * 2 * C);   // C float4: per-channel coefficients of a BN backward
  float* own = reinterpret_cast<float*>(tab + C);
  auto slot = [&]() { return xchg + (size_t)(phase & 1u) * a.nmem * (2 * C); };

  std::conditional_t<WL != 0, WFragsL<C / 32, MID / 16>, WFrags<C / 32, MID / 16, PRE>> w3;            // conv3 data gradient [MID][C]
  std::conditional_t<WL == 1, WFragsL<9 * MID / 32, MID / 16>,
                     std::conditional_t<WT, WFragsL<3 * MID / 32, MID / 16>, WFrags<9 * MID / 32, MID / 16, PRE>>> w2;  // conv2 data gradient [MID][9*MID] (WT: three taps of it)
  std::conditional_t<WL != 0, WFragsL<MID / 32, C / 16>, WFrags<MID / 32, C / 16, PRE>> w1;            // conv1 data gradient [C][MID]
  bf16_t* sW = reinterpret_cast<bf16_t*>(own + (gath_own ? (size_t)a.nmem * 2 * C : 0));   // WL == 1: the staged matrix
  bf16_t* const sW13 = WT ? sdc : sW;
  constexpr int W2NU = (3 * MID * MID / 8 + RES_NT - 1) / RES_NT;                            // WT: units per thread and round
  u32x4 wst[WL == 1 ? (9 * MID / 32 * (MID / 16) + 7) / 8 : WT ? 3 * W2NU : 1];             // the units on their way
  static_assert(!WT || (MID * (C + 8) <= 256 * (MID + 8) && C * (MID + 8) <= 256 * (MID + 8) && MID * (3 * MID + 8) <= 256 * (MID + 8)),
                "the matrices fit a MID-wide tile of 256 pixels");
  {
    const ResBlock BL = a.blocks[a.nblk - 1];
    tile_load<C>(sdy, cx.tensor(BL.gy_off) + (size_t)me * P * C, P);
    if constexpr (WL != 0) {   // the first block's conv3 matrix; later ones are staged behind the exchange before
      w_issue(w3, wst, a.packed + BL.wd_off[2], C, fr, fk);
      w_commit(w3, wst, sW13);
    }
  }
  __syncthreads();   // the first contraction reads the tile right away
  for (int bi = a.nblk - 1; bi >= 0; --bi) {
    const ResBlock B = a.blocks[bi];
    uint2 xc1[PTW][MID / 16], xc2[PTW][MID / 16];   // c1 / c2 at this lane's accumulator positions
    // ---- conv3 data gradient: da3[p][c] = sum_n dy[p][n] * W3[c][n]; then BN3 + ReLU backward -> dc2
    // One round trip to memory for everything the block reads up front; the weights are asked for first and the
    // contraction, which needs nothing else, runs while the stashed tensors and the tables are on their way.
    floatx4 acc3[PTW][MID / 16];
    {
      BwdLoads<C, MID, PTW> ld;
      if constexpr (WL == 0) w3.load(a.packed + B.wd_off[2], C, fr, fk);
      ld.issue(B, cx, a.params, me, P, npt, wave, fr, fq);
#pragma unroll
      for (int j = 0; j < PTW; ++j)
#pragma unroll
        for (int nt = 0; nt < MID / 16; ++nt) acc3[j][nt] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < C / 32; ++ks) {
#pragma unroll
        for (int j = 0; j < PTW; ++j) {
          const int pt = wave + j * RES_NWV;
          if (pt < npt) {
            const bf16x8 bfrag = *reinterpret_cast<const bf16x8*>(sdy + (pt * 16 + fr) * XS + ks * 32 + fk);
#pragma unroll
            for (int nt = 0; nt < MID / 16; ++nt) acc3[j][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w3.get(ks, nt), bfrag, acc3[j][nt], 0, 0, 0);
          }
        }
      }
      ld.commit_tables(cf1, cf2, cf3);
#pragma unroll
      for (int j = 0; j < PTW; ++j)
#pragma unroll
        for (int nt = 0; nt < MID / 16; ++nt) { xc1[j][nt] = ld.x1[j][nt]; xc2[j][nt] = ld.x2[j][nt]; }
    }
    __syncthreads();
    {
      floatx4 (&acc)[PTW][MID / 16] = acc3;
      uint2 xin[PTW][MID / 16];
#pragma unroll
      for (int j = 0; j < PTW; ++j) {
        const int pt = wave + j * RES_NWV;
#pragma unroll
        for (int nt = 0; nt < MID / 16; ++nt) {
          xin[j][nt] = pt < npt ? xc2[j][nt] : make_uint2(0u, 0u);
        }
      }
      if constexpr (WT) {   // all three rounds are asked for now: the exchange below hides the latency
        w2.template issue_cols<0>(wst, a.packed + B.wd_off[1], 9 * MID, fr, fk);
        w2.template issue_cols<W2NU>(wst, a.packed + B.wd_off[1] + 3 * MID, 9 * MID, fr, fk);
        w2.template issue_cols<2 * W2NU>(wst, a.packed + B.wd_off[1] + 6 * MID, 9 * MID, fr, fk);
      } else {
        w_issue(w2, wst, a.packed + B.wd_off[1], 9 * MID, fr, fk);
      }
      float* gath = gath_own ? own : reinterpret_cast<float*>(sdc);
      if (!bn_relu_bwd_acc<MID, PTW>(acc, xin, cf3, npt, wave, fr, fq, red, tab, gath, slot(), me, a.nmem, P, tag0 + 1u + phase,
                                     me == 0 ? reinterpret_cast<float*>(cx.base + B.dgb_off[2]) : nullptr, a.abort_flag,
                                     [&](int j, int nt, const floatx4& out) {
                                       *reinterpret_cast<uint2*>(sdc + ((wave + j * RES_NWV) * 16 + fr) * MS + nt * 16 + fq * 4) = pack4(out);
                                     }))
        return;
      ++phase;
      if constexpr (WT) w2.template commit_from<0>(wst, sm2);   // that tile was last read as the gather area of the block before
      else w_commit(w2, wst, sW);   // conv3's matrix was last read above the barrier that follows the tables
    }
    __syncthreads();
    tile_store<MID>(cx.tensor(B.dc2_off) + (size_t)me * P * MID, sdc, P);
    // ---- conv2 data gradient, BN2 + ReLU backward -> dc1 (into the tile that held c2)
    uint2 x1[PTW][C / 16];   // the block input at this lane's accumulator positions, for the BN1 backward below
    {
      floatx4 acc[PTW][MID / 16];
      uint2 xin[PTW][MID / 16];
#pragma unroll
      for (int j = 0; j < PTW; ++j)
#pragma unroll
        for (int nt = 0; nt < MID / 16; ++nt) acc[j][nt] = floatx4{0.f, 0.f, 0.f, 0.f};
      {   // issued ahead of the contraction: the latency passes behind it and the first BN pass
        const bf16_t* xg = cx.tensor(B.x_off) + (size_t)me * P * C;
#pragma unroll
        for (int j = 0; j < PTW; ++j) {
          const int pt = wave + j * RES_NWV;
#pragma unroll
          for (int nt = 0; nt < C / 16; ++nt)
            x1[j][nt] = *reinterpret_cast<const uint2*>(xg + (size_t)((pt < npt ? pt : 0) * 16 + fr) * C + nt * 16 + fq * 4);
        }
      }
      if constexpr (WT) {   // a barrier on either side of every re-staging (the BN backward below starts with one)
        conv3x3_tile<MID, PTW, true, 0, 3>(sdc, w2, H, W, npt, wave, fr, fk, acc);
        __syncthreads();
        w2.template commit_from<W2NU>(wst, sm2);
        __syncthreads();
        conv3x3_tile<MID, PTW, true, 3, 3>(sdc, w2, H, W, npt, wave, fr, fk, acc);
        __syncthreads();
        w2.template commit_from<2 * W2NU>(wst, sm2);
        __syncthreads();
        conv3x3_tile<MID, PTW, true, 6, 3>(sdc, w2, H, W, npt, wave, fr, fk, acc);
      } else {
        conv3x3_tile<MID, PTW, true>(sdc, w2, H, W, npt, wave, fr, fk, acc);
      }
#pragma unroll
      for (int j = 0; j < PTW; ++j) {
        const int pt = wave + j * RES_NWV;
#pragma unroll
        for (int nt = 0; nt < MID / 16; ++nt) {
          xin[j][nt] = pt < npt ? xc1[j][nt] : make_uint2(0u, 0u);
        }
      }
      w_issue(w1, wst, a.packed + B.wd_off[0], MID, fr, fk);
      float* gath = gath_own ? own : reinterpret_cast<float*>(sm2);
      if (!bn_relu_bwd_acc<MID, PTW>(acc, xin, cf2, npt, wave, fr, fq, red, tab, gath, slot(), me, a.nmem, P, tag0 + 1u + phase,
                                     me == 0 ? reinterpret_cast<float*>(cx.base + B.dgb_off[1]) : nullptr, a.abort_flag,
                                     [&](int j, int nt, const floatx4& out) {
                                       *reinterpret_cast<uint2*>(sm2 + ((wave + j * RES_NWV) * 16 + fr) * MS + nt * 16 + fq * 4) = pack4(out);
                                     }))
        return;
      ++phase;
      w_commit(w1, wst, sW13);   // WT: dc2 in that tile was last read by the contraction above the exchange
    }
    __syncthreads();
    tile_store<MID>(cx.tensor(B.dc1_off) + (size_t)me * P * MID, sm2, P);
    // ---- conv1 data gradient, BN1 + ReLU backward, plus the shortcut: dx = bn1_bwd(...) + dy, written over dy
    {
      floatx4 acc[PTW][C / 16];
      bf16x8 bfrag[PTW][MID / 32];
#pragma unroll
      for (int j = 0; j < PTW; ++j) {
        const int pt = wave + j * RES_NWV;
#pragma unroll
        for (int ks = 0; ks < MID / 32; ++ks)
          bfrag[j][ks] = pt < npt ? *reinterpret_cast<const bf16x8*>(sm2 + (pt * 16 + fr) * MS + ks * 32 + fk) : frag_zero();
      }
#pragma unroll
      for (int nt = 0; nt < C / 16; ++nt) {
#pragma unroll
        for (int j = 0; j < PTW; ++j) {
          acc[j][nt] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int ks = 0; ks < MID / 32; ++ks) acc[j][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w1.get(ks, nt), bfrag[j][ks], acc[j][nt], 0, 0, 0);
        }
      }
      __syncthreads();   // all waves are done with the small tiles: they become the gather area
      if constexpr (WL != 0)
        if (bi > 0) w_issue(w3, wst, a.packed + a.blocks[bi - 1].wd_off[2], C, fr, fk);   // the next block's conv3 matrix
      float* gath = gath_own ? own : reinterpret_cast<float*>(sm2);   // dc1 left the tile above
      if (!bn_relu_bwd_acc<C, PTW>(acc, x1, cf1, npt, wave, fr, fq, red, tab, gath, slot(), me, a.nmem, P, tag0 + 1u + phase,
                                   me == 0 ? reinterpret_cast<float*>(cx.base + B.dgb_off[0]) : nullptr, a.abort_flag,
                                   [&](int j, int nt, const floatx4& out) {
                                     uint2* q = reinterpret_cast<uint2*>(sdy + ((wave + j * RES_NWV) * 16 + fr) * XS + nt * 16 + fq * 4);
                                     const uint2 d = *q;
                                     floatx4 v = out;
                                     v[0] += bf_lo(d.x); v[1] += bf_hi(d.x); v[2] += bf_lo(d.y); v[3] += bf_hi(d.y);
                                     *q = pack4(v);
                                   }))
        return;
      ++phase;
      if constexpr (WL != 0)
        if (bi > 0) w_commit(w3, wst, sW13);   // WT: conv1's matrix in that tile was last read above the barrier before the exchange
    }
    __syncthreads();   // dx is complete; the BN tables and the small tiles of this block are no longer read
    tile_store<C>(cx.tensor(B.gx_off) + (size_t)me * P * C, sdy, P);
  }
  if (me == 0 && tid == 0) *tagp = tag0 + phase;
}

// ------------------------------------------------------------------------------------------ weight gradients
// Weight gradients of the blocks of a run, one launch for all of them.  A work-group takes one (block,
// convolution [, 64-channel chunk]) and a group of images of one micro-batch; per image it stages the two
// operands ONCE, transposed (channel-major, so that every MFMA lane finds its 8 consecutive pixels with one
// 16-byte LDS read), runs every filter tap and output tile from LDS, and keeps the sums in registers over its
// images; one fp32 atomic add per output element and work-group then goes to the gradient buffer.
//   dw[tap][c][n] += sum_p a[p + shift(tap)][c] * dy[p][n],   a = relu(bn(x)) recomputed while staging.
// The 3x3 convolution keeps three copies of `a`, shifted by -1 / 0 / +1 pixel along the image row with the
// wrapped column zeroed, on a canvas with one zero image row above and below: every tap is then an aligned
// read at offset r*W.
// Threads per work-group: 4 waves for the 32-wide tensors; 8 for the 64-wide ones, whose 3x3 item fills the LDS
// of a CU on its own (one work-group per CU) and whose sums would otherwise take 200 registers per lane.
constexpr int rw_threads(int mid) { return mid >= 64 ? 512 : 256; }
// Register sets of image loads in flight per lane (measured on 128-32 blocks: 242 us per launch with 2, 247 with 3).
constexpr int rw_sets(int) { return 2; }

// Pixel pairs of an image tile in registers: channels [c0, c0+CH) of an image [P][CT].  A unit is (pixel pair,
// group of 8 channels); four neighbouring lanes take four consecutive channel groups of one pair (64
// contiguous bytes), the 16 lane quads of a wave 16 consecutive pairs: global loads touch 16 lines per
// instruction and the transposing LDS stores stay within a 2-way bank conflict.
template <int CH, int NTH>
struct PairRegs {
  static constexpr int G = CH / 8;                       // channel groups (4 or 8)
  static constexpr int NU = 128 * G / NTH;
  static_assert(G % 4 == 0 && (128 * G) % NTH == 0, "tile shape");
  uint4 v[NU][2];
  static __device__ __forceinline__ void unit(int u, int& pr, int& cg) {
    const int lane = threadIdx.x & 63, q = u * (NTH / 64) + (threadIdx.x >> 6);
    cg = (q % (G / 4)) * 4 + (lane & 3);
    pr = (q / (G / 4)) * 16 + (lane >> 2);
  }
  __device__ __forceinline__ void load(const bf16_t* img, int CT, int c0, int P) {
#pragma unroll
    for (int u = 0; u < NU; ++u) {
      int pr, cg;
      unit(u, pr, cg);
      const bf16_t* q = img + (size_t)(2 * pr < P ? 2 * pr : 0) * CT + c0 + cg * 8;   // always a valid address
      v[u][0] = *reinterpret_cast<const uint4*>(q);
      v[u][1] = *reinterpret_cast<const uint4*>(q + CT);
    }
  }
};
// two pixels' 8 channels -> 8 dwords {pixel at pos, pixel at pos+1} in the channel-major tile (pos even)
__device__ __forceinline__ void store_pair(bf16_t* T, int PS, int ch0, int pos, const uint4& e0, const uint4& e1) {
  uint32_t* dst = reinterpret_cast<uint32_t*>(T + (size_t)ch0 * PS + pos);
  const int RS = PS >> 1;
  const uint32_t a[4] = {e0.x, e0.y, e0.z, e0.w}, b[4] = {e1.x, e1.y, e1.z, e1.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    dst[(2 * i) * RS] = (a[i] & 0xffffu) | (b[i] << 16);
    dst[(2 * i + 1) * RS] = (a[i] >> 16) | (b[i] & 0xffff0000u);
  }
}
__device__ __forceinline__ uint4 bn_relu8(const uint4& q, const float2* coef) {
  const uint32_t w[4] = {q.x, q.y, q.z, q.w};
  const float4* cf = reinterpret_cast<const float4*>(__builtin_assume_aligned(coef, 16));
  uint32_t r[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float4 k = cf[i];
    r[i] = pack_bf16x2(fmaxf(fmaf(bf_lo(w[i]), k.x, k.y), 0.f), fmaxf(fmaf(bf_hi(w[i]), k.z, k.w), 0.f));
  }
  return make_uint4(r[0], r[1], r[2], r[3]);
}
// value of the lane four below / above (same channel group, previous / next pixel pair)
__device__ __forceinline__ uint4 lanes_up4(const uint4& v) {
  return make_uint4(__shfl_up(v.x, 4), __shfl_up(v.y, 4), __shfl_up(v.z, 4), __shfl_up(v.w, 4));
}
__device__ __forceinline__ uint4 lanes_down4(const uint4& v) {
  return make_uint4(__shfl_down(v.x, 4), __shfl_down(v.y, 4), __shfl_down(v.z, 4), __shfl_down(v.w, 4));
}

struct ResWgArgs {
  const ResBlock* blocks;
  int nmem, ipw, H, W;       // images per micro-batch, images per work-group (divides nmem), image shape
  int ngroup;                // micro-batches in the launch
  PtrTab base, act_in, err_in;
  const float* params;
  float* grads;
};

struct WgImage {   // where the work-group's image i lives
  const ResWgArgs& a; int img0;
  __device__ __forceinline__ ResCtx ctx(int i, int& me) const {
    const int img = img0 + i, z = img / a.nmem;
    me = img - z * a.nmem;
    return ResCtx{(char*)pick(a.base, z), pick(a.act_in, z), nullptr, pick(a.err_in, z), nullptr};
  }
};

// BN table of the `a` operand's channels [c0, c0+CA) -> LDS coef (the group's images share one micro-batch)
template <int CA, int NTH>
__device__ __forceinline__ void wg_coef(float2* coef, const float* stats, const float* gamma, const float* beta, int c0, int CT) {
  for (int c = threadIdx.x; c < CA; c += NTH)
    coef[c] = bn_scale_shift(stats[c0 + c], stats[CT + c0 + c], gamma[c0 + c], beta[c0 + c]);
}

// 1x1 convolution: a channels [ca0, ca0+CA) of CTA, dy channels [nd0, nd0+ND) of CTD; dw is [CTA][CTD].
template <int CA, int ND, int NTH>
__device__ __forceinline__ void res_wgrad_1x1(const ResWgArgs& a, int img0, unsigned long long a_off, int CTA, int ca0,
                                              unsigned long long st_off, const float* gamma, const float* beta,
                                              unsigned long long dy_off, int CTD, int nd0, float* dw, unsigned char* smem) {
  const int P = a.H * a.W, PS = P + 8;
  const int tid = threadIdx.x, lane = tid & 63, wave = wave_index(), fr = lane & 15, fq = lane >> 4, fk = fq * 8;
  bf16_t* Ta = reinterpret_cast<bf16_t*>(smem);
  bf16_t* Td = Ta + (size_t)CA * PS;
  float2* coef = reinterpret_cast<float2*>(Td + (size_t)ND * PS);
  constexpr int NTD = ND / 16, TPW = (CA / 16) * NTD / (NTH / 64);
  static_assert((CA / 16) * NTD % (NTH / 64) == 0, "output tiles per wave");
  floatx4 acc[TPW];
#pragma unroll
  for (int t = 0; t < TPW; ++t) acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
  const WgImage wi{a, img0};
  auto load_img = [&](int i, PairRegs<CA, NTH>& A, PairRegs<ND, NTH>& D) {
    int me;
    const ResCtx cx = wi.ctx(i, me);
    A.load(cx.tensor(a_off) + (size_t)me * P * CTA, CTA, ca0, P);
    D.load(cx.tensor(dy_off) + (size_t)me * P * CTD, CTD, nd0, P);
  };
  auto stage = [&](const PairRegs<CA, NTH>& A, const PairRegs<ND, NTH>& D) {
#pragma unroll
    for (int u = 0; u < PairRegs<CA, NTH>::NU; ++u) {
      int pr, cg;
      PairRegs<CA, NTH>::unit(u, pr, cg);
      if (2 * pr < P) store_pair(Ta, PS, cg * 8, 2 * pr, bn_relu8(A.v[u][0], coef + cg * 8), bn_relu8(A.v[u][1], coef + cg * 8));
    }
#pragma unroll
    for (int u = 0; u < PairRegs<ND, NTH>::NU; ++u) {
      int pr, cg;
      PairRegs<ND, NTH>::unit(u, pr, cg);
      if (2 * pr < P) store_pair(Td, PS, cg * 8, 2 * pr, D.v[u][0], D.v[u][1]);
    }
  };
  auto mma = [&]() {
    for (int ks = 0; ks < P / 32; ++ks) {
#pragma unroll
      for (int t = 0; t < TPW; ++t) {
        const int tile = wave * TPW + t, ct = tile / NTD, nt = tile % NTD;
        const bf16x8 fa = *reinterpret_cast<const bf16x8*>(Ta + (size_t)(ct * 16 + fr) * PS + ks * 32 + fk);
        const bf16x8 fd = *reinterpret_cast<const bf16x8*>(Td + (size_t)(nt * 16 + fr) * PS + ks * 32 + fk);
        acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fd, acc[t], 0, 0, 0);
      }
    }
  };
  // NS register sets in rotation: an image's loads are issued NS - 1 images before they are staged
  constexpr int NS = rw_sets(NTH);
  PairRegs<CA, NTH> as[NS];
  PairRegs<ND, NTH> ds[NS];
  {
    int me;
    const ResCtx cx = wi.ctx(0, me);
    wg_coef<CA, NTH>(coef, reinterpret_cast<const float*>(cx.base + st_off), gamma, beta, ca0, CTA);
  }
  // a register set is refilled as soon as it has been staged: its loads then have the contraction of this image
  // and the whole turns of the other sets to arrive
#pragma unroll
  for (int k = 0; k < NS; ++k)
    if (k < a.ipw) load_img(k, as[k], ds[k]);
  for (int i = 0; i < a.ipw; i += NS) {
#pragma unroll
    for (int k = 0; k < NS; ++k) {
      if (i + k < a.ipw) {
        __syncthreads();   // the previous image's fragments are read (and coef is written, first time)
        stage(as[k], ds[k]);
        if (i + k + NS < a.ipw) load_img(i + k + NS, as[k], ds[k]);
        __syncthreads();
        mma();
      }
    }
  }
#pragma unroll
  for (int t = 0; t < TPW; ++t) {
    const int tile = wave * TPW + t, ct = tile / NTD, nt = tile % NTD;
#pragma unroll
    for (int v = 0; v < 4; ++v)
      atomicAdd(dw + (size_t)(ca0 + ct * 16 + fq * 4 + v) * CTD + nd0 + nt * 16 + fr, acc[t][v]);
  }
}

// 3x3 convolution, MID -> MID channels, stride 1, zero padding; dw is [9][MID][MID].
template <int MID, int NTH>
__device__ __forceinline__ void res_wgrad_3x3(const ResWgArgs& a, int img0, unsigned long long a_off, unsigned long long st_off,
                                              const float* gamma, const float* beta, unsigned long long dy_off, float* dw,
                                              unsigned char* smem) {
  const int P = a.H * a.W, W = a.W, PS = P + 8, PSH = P + 2 * W + 8;
  const bool plain = gamma == nullptr;   // the operand is the stored tensor as it is (no BatchNorm + ReLU in front of the convolution)
  const int tid = threadIdx.x, lane = tid & 63, wave = wave_index(), fr = lane & 15, fq = lane >> 4, fk = fq * 8;
  bf16_t* Tsh = reinterpret_cast<bf16_t*>(smem);          // [3][MID][PSH]: a shifted by s-1 pixels along the row
  bf16_t* Td = Tsh + (size_t)3 * MID * PSH;               // [MID][PS]
  float2* coef = reinterpret_cast<float2*>(Td + (size_t)MID * PS);
  constexpr int NT = MID / 16, PPW = NT * NT / (NTH / 64);
  static_assert(NT * NT % (NTH / 64) == 0, "tile pairs per wave");         // (input tile, output tile) pairs per wave
  floatx4 acc[PPW][9];
#pragma unroll
  for (int t = 0; t < PPW; ++t)
#pragma unroll
    for (int k = 0; k < 9; ++k) acc[t][k] = floatx4{0.f, 0.f, 0.f, 0.f};
  // the zero image rows above and below
  for (int i = tid; i < 3 * MID * 2 * W; i += NTH) {
    const int ch = i / (2 * W), j = i - ch * 2 * W;
    Tsh[(size_t)ch * PSH + (j < W ? j : P + j)] = 0;
  }
  const WgImage wi{a, img0};
  const int half_w = W >> 1;
  auto load_img = [&](int i, PairRegs<MID, NTH>& A, PairRegs<MID, NTH>& D) {
    int me;
    const ResCtx cx = wi.ctx(i, me);
    A.load(cx.tensor(a_off) + (size_t)me * P * MID, MID, 0, P);
    D.load(cx.tensor(dy_off) + (size_t)me * P * MID, MID, 0, P);
  };
  auto stage = [&](const PairRegs<MID, NTH>& A, const PairRegs<MID, NTH>& D) {
#pragma unroll
    for (int u = 0; u < PairRegs<MID, NTH>::NU; ++u) {
      int pr, cg;
      PairRegs<MID, NTH>::unit(u, pr, cg);
      const bool ok = 2 * pr < P;
      const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
      const uint4 e0 = plain ? A.v[u][0] : bn_relu8(A.v[u][0], coef + cg * 8), e1 = plain ? A.v[u][1] : bn_relu8(A.v[u][1], coef + cg * 8);
      // the neighbouring pairs of the image row sit four lanes away (the 16 pairs of a wave hold whole rows)
      uint4 left = lanes_up4(e1), right = lanes_down4(e0);
      const int pc = pr % half_w;
      if (pc == 0) left = zero;
      if (pc == half_w - 1) right = zero;
      if (ok) {
        const int pos = 2 * pr + W;
        store_pair(Tsh, PSH, cg * 8, pos, left, e0);                       // a[col-1]
        store_pair(Tsh + (size_t)MID * PSH, PSH, cg * 8, pos, e0, e1);     // a[col]
        store_pair(Tsh + (size_t)2 * MID * PSH, PSH, cg * 8, pos, e1, right);   // a[col+1]
        store_pair(Td, PS, cg * 8, 2 * pr, D.v[u][0], D.v[u][1]);
      }
    }
  };
  auto mma = [&]() {
    for (int ks = 0; ks < P / 32; ++ks) {
#pragma unroll
      for (int t = 0; t < PPW; ++t) {
        const int pair = wave * PPW + t, ct = pair / NT, nt = pair % NT;
        const bf16x8 fd = *reinterpret_cast<const bf16x8*>(Td + (size_t)(nt * 16 + fr) * PS + ks * 32 + fk);
#pragma unroll
        for (int tap = 0; tap < 9; ++tap) {
          const int r = tap / 3, s = tap % 3;
          const bf16x8 fa = *reinterpret_cast<const bf16x8*>(Tsh + ((size_t)s * MID + ct * 16 + fr) * PSH + ks * 32 + fk + r * W);
          acc[t][tap] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fd, acc[t][tap], 0, 0, 0);
        }
      }
    }
  };
  constexpr int NS = rw_sets(NTH);
  PairRegs<MID, NTH> as[NS], ds[NS];
  {
    int me;
    const ResCtx cx = wi.ctx(0, me);
    if (!plain) wg_coef<MID, NTH>(coef, reinterpret_cast<const float*>(cx.base + st_off), gamma, beta, 0, MID);
  }
#pragma unroll
  for (int k = 0; k < NS; ++k)
    if (k < a.ipw) load_img(k, as[k], ds[k]);
  for (int i = 0; i < a.ipw; i += NS) {
#pragma unroll
    for (int k = 0; k < NS; ++k) {
      if (i + k < a.ipw) {
        __syncthreads();
        stage(as[k], ds[k]);
        if (i + k + NS < a.ipw) load_img(i + k + NS, as[k], ds[k]);   // refilled as soon as staged (see the 1x1 case)
        __syncthreads();
        mma();
      }
    }
  }
#pragma unroll
  for (int t = 0; t < PPW; ++t) {
    const int pair = wave * PPW + t, ct = pair / NT, nt = pair % NT;
#pragma unroll
    for (int tap = 0; tap < 9; ++tap)
#pragma unroll
      for (int v = 0; v < 4; ++v)
        atomicAdd(dw + ((size_t)tap * MID + ct * 16 + fq * 4 + v) * MID + nt * 16 + fr, acc[t][tap][v]);
  }
}

// Gradients of beta and gamma of one BatchNorm (Cc channels) of a block: the backward launch left {sum dz,
// sum dz*xhat} per micro-batch at dgb_off; one work-group per block adds them up over the micro-batches of the
// launch.  The loads of a lane are issued before the first use: one trip to memory.
template <int NTH>
__device__ __forceinline__ void add_bn_param_grads(const ResWgArgs& a, unsigned long long dgb_off, float* g_beta, float* g_gamma, int Cc) {
  for (int c = threadIdx.x; c < 2 * Cc; c += NTH) {
    float v[MAX_GROUP];
#pragma unroll
    for (int z = 0; z < MAX_GROUP; ++z)
      v[z] = z < a.ngroup ? reinterpret_cast<const float*>((const char*)pick(a.base, z) + dgb_off)[c] : 0.f;
    float s = 0.f;
#pragma unroll
    for (int z = 0; z < MAX_GROUP; ++z) s += v[z];
    atomicAdd(c < Cc ? g_beta + c : g_gamma + (c - Cc), s);
  }
}

// grid: (image groups, 2*C/64 + 1 items, blocks of the run).  Items: conv1 in chunks of 64 input channels,
// conv2, conv3 in chunks of 64 output channels.
template <int C, int MID>
__global__ void __launch_bounds__(rw_threads(MID)) k_res_wgrad(const ResWgArgs a) {
  constexpr int NTH = rw_threads(MID);
  extern __shared__ __align__(16) unsigned char smem[];
  const ResBlock B = a.blocks[blockIdx.z];
  const int img0 = blockIdx.x * a.ipw;
  constexpr int NCH = C / 64;
  const int item = blockIdx.y;
  if (item < NCH)
    res_wgrad_1x1<64, MID, NTH>(a, img0, B.x_off, C, item * 64, B.stats_off[0], a.params + B.gamma_off[0], a.params + B.beta_off[0],
                           B.dc1_off, MID, 0, a.grads + B.w_off[0], smem);
  else if (item == NCH) {
    res_wgrad_3x3<MID, NTH>(a, img0, B.c1_off, B.stats_off[1], a.params + B.gamma_off[1], a.params + B.beta_off[1], B.dc2_off,
                       a.grads + B.w_off[1], smem);
    if (blockIdx.x == 0) {
      add_bn_param_grads<NTH>(a, B.dgb_off[0], a.grads + B.beta_off[0], a.grads + B.gamma_off[0], C);
      add_bn_param_grads<NTH>(a, B.dgb_off[1], a.grads + B.beta_off[1], a.grads + B.gamma_off[1], MID);
      add_bn_param_grads<NTH>(a, B.dgb_off[2], a.grads + B.beta_off[2], a.grads + B.gamma_off[2], MID);
    }
  } else
    res_wgrad_1x1<MID, 64, NTH>(a, img0, B.c2_off, MID, 0, B.stats_off[2], a.params + B.gamma_off[2], a.params + B.beta_off[2],
                           B.gy_off, C, (item - NCH - 1) * 64, a.grads + B.w_off[2], smem);
}

// ------------------------------------------------------------------------------------------ basic blocks
// The same ownership for runs of basic blocks (two 3x3 convolutions of C channels, identity shortcut: the
// ResNet-20 / ResNet-110 family):  a1 = relu(bn1(x)); c1 = conv1(a1); a2 = relu(bn2(c1)); y = x + conv2(a2).
// Two exchanges per block and direction.  ResBlock fields used: x, c1, y, gy, dc1, gx and entries 0 / 1 of the
// per-BatchNorm / per-convolution arrays.
// dst = relu(src*scale + shift), tile to tile
template <int Cc>
__device__ __forceinline__ void tile_bn_relu_to(bf16_t* dst, const bf16_t* src, const float2* coef, int P) {
  constexpr int U = Cc / 8;
  for (int u = threadIdx.x; u < P * U; u += RES_NT) {
    const int row = u / U, col = u - row * U;
    const uint4 v = *reinterpret_cast<const uint4*>(src + row * (Cc + 8) + col * 8);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    const float4* cf = reinterpret_cast<const float4*>(coef + col * 8);
    uint32_t r[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float4 k = cf[i];
      r[i] = pack_bf16x2(fmaxf(fmaf(bf_lo(w[i]), k.x, k.y), 0.f), fmaxf(fmaf(bf_hi(w[i]), k.z, k.w), 0.f));
    }
    *reinterpret_cast<uint4*>(dst + row * (Cc + 8) + col * 8) = make_uint4(r[0], r[1], r[2], r[3]);
  }
}

// floats of the reduction area: 8 waves x 2*C sums (backward), and 32/(C/8) pixel groups x 2*C (statistics) = 512
constexpr int V1_RED(int C) { return RES_NWV * 2 * C > 512 ? RES_NWV * 2 * C : 512; }

template <int C, int PTW, bool PRE, bool INFER = false, bool WL = false>
__global__ void __launch_bounds__(RES_NT) k_bb_forward(const ResArgs a, const int gath_own) {
  static_assert(!(WL && (PRE || INFER)), "the LDS form replaces the fetch-where-used form of the training kernels");
  constexpr int XS = C + 8;
  const int tid = threadIdx.x, lane = tid & 63, wave = wave_index();
  const int fr = lane & 15, fq = lane >> 4, fk = fq * 8;
  // the 16-channel shape is 32 x 32 pixels only: constants instead of kernel arguments (fewer address temporaries)
  const int H = C == 16 ? 32 : a.H, W = C == 16 ? 32 : a.W;
  const int P = H * W, npt = P >> 4;
  const int z = blockIdx.x % a.ngroup, me = blockIdx.x / a.ngroup;
  ResCtx cx{(char*)pick(a.base, z), pick(a.act_in, z), pick(a.act_out, z), pick(a.err_in, z), pick(a.err_out, z)};
  u64* xchg = reinterpret_cast<u64*>(cx.base + a.xchg_off);
  unsigned* tagp = reinterpret_cast<unsigned*>(cx.base + a.tag_off);
  const unsigned tag0 = *tagp;
  unsigned phase = 0;

  extern __shared__ __align__(16) unsigned char smem[];
  bf16_t* sx = reinterpret_cast<bf16_t*>(smem);           // residual stream of the image, [P][XS]
  bf16_t* sA = sx + (size_t)P * XS;                       // relu(bn1(x))
  bf16_t* sB = sA + (size_t)P * XS;                       // c1, then relu(bn2(c1))
  float2* coef = reinterpret_cast<float2*>(sB + (size_t)P * XS);
  float* red = reinterpret_cast<float*>(coef + C);        // V1_RED(C) floats
  float* own = red + V1_RED(C);
  float* gath = gath_own ? own : reinterpret_cast<float*>(sA);
  auto slot = [&]() { return xchg + (size_t)(phase & 1u) * a.nmem * (2 * C); };
  constexpr int KT = (9 * C + 31) / 32, LD = KT * 32;     // reduction steps and row length of the packed weights
  std::conditional_t<WL, WFragsL<KT, C / 16>, WFrags<KT, C / 16, PRE>> w1, w2;
  bf16_t* sW = reinterpret_cast<bf16_t*>(own + (gath_own ? (size_t)a.nmem * 2 * C : 0));   // WL: the staged matrix
  u32x4 wst[WL ? (KT * (C / 16) + 7) / 8 : 1];                                      // WL: its units on their way

  auto store_acc = [&](bf16_t* dst, floatx4 (&acc)[PTW][C / 16]) {
#pragma unroll
    for (int j = 0; j < PTW; ++j) {
      const int pt = wave + j * RES_NWV;
      if (pt < npt)
#pragma unroll
        for (int nt = 0; nt < C / 16; ++nt)
          *reinterpret_cast<uint2*>(dst + (pt * 16 + fr) * XS + nt * 16 + fq * 4) = pack4(acc[j][nt]);
    }
  };
  {
    const ResBlock B0 = a.blocks[0];
    tile_load<C>(sx, cx.tensor(B0.x_off) + (size_t)me * P * C, P);
    w_issue(w1, wst, a.packed + B0.wf_off[0], LD, fr, fk);
    __syncthreads();
    if (INFER) {
      running_coef<C>(coef, a.running + B0.run_off[0], a.params + B0.gamma_off[0], a.params + B0.beta_off[0], a.eps);
    } else {
      stats_publish<C>(sx, P, red, slot(), me, tag0 + 1u + phase);
      if (!collect<4>(slot(), a.nmem, 2 * C, tag0 + 1u + phase, gath, a.abort_flag)) return;
      ++phase;
      w_commit(w1, wst, sW);
      merge_coef<C>(gath, a.nmem, P, a.eps, a.params + B0.gamma_off[0], a.params + B0.beta_off[0], coef,
                    me == 0 ? reinterpret_cast<float*>(cx.base + B0.stats_off[0]) : nullptr);
    }
  }
  for (int bi = 0; bi < a.nblk; ++bi) {
    const ResBlock B = a.blocks[bi];
    tile_bn_relu_to<C>(sA, sx, coef, P);
    __syncthreads();
    {   // ---- conv1 (3x3) on relu(bn1(x))
      floatx4 acc[PTW][C / 16];
#pragma unroll
      for (int j = 0; j < PTW; ++j)
#pragma unroll
        for (int nt = 0; nt < C / 16; ++nt) acc[j][nt] = floatx4{0.f, 0.f, 0.f, 0.f};
      conv3x3_tile<C, PTW, false>(sA, w1, H, W, npt, wave, fr, fk, acc);
      store_acc(sB, acc);
    }
    w_issue(w2, wst, a.packed + B.wf_off[1], LD, fr, fk);
    __syncthreads();
    if (INFER) {
      running_coef<C>(coef, a.running + B.run_off[1], a.params + B.gamma_off[1], a.params + B.beta_off[1], a.eps);
    } else {
      stats_publish<C>(sB, P, red, slot(), me, tag0 + 1u + phase);
      tile_store<C>(cx.tensor(B.c1_off) + (size_t)me * P * C, sB, P);
      if (!collect<4>(slot(), a.nmem, 2 * C, tag0 + 1u + phase, gath, a.abort_flag)) return;   // sA is free: conv1 is done
      ++phase;
      w_commit(w2, wst, sW);   // conv1 read its matrix above the barrier before the statistics
      merge_coef<C>(gath, a.nmem, P, a.eps, a.params + B.gamma_off[1], a.params + B.beta_off[1], coef,
                    me == 0 ? reinterpret_cast<float*>(cx.base + B.stats_off[1]) : nullptr);
    }
    tile_bn_relu<C>(sB, coef, P);
    __syncthreads();
    {   // ---- conv2 (3x3) on relu(bn2(c1)) + shortcut, written over x
      floatx4 acc[PTW][C / 16];
#pragma unroll
      for (int j = 0; j < PTW; ++j)
#pragma unroll
        for (int nt = 0; nt < C / 16; ++nt) acc[j][nt] = floatx4{0.f, 0.f, 0.f, 0.f};
      conv3x3_tile<C, PTW, false>(sB, w2, H, W, npt, wave, fr, fk, acc);
#pragma unroll
      for (int j = 0; j < PTW; ++j) {
        const int pt = wave + j * RES_NWV;
        if (pt < npt)
#pragma unroll
          for (int nt = 0; nt < C / 16; ++nt) {
            uint2* q = reinterpret_cast<uint2*>(sx + (pt * 16 + fr) * XS + nt * 16 + fq * 4);
            const uint2 xr = *q;
            floatx4 v = acc[j][nt];
            v[0] += bf_lo(xr.x); v[1] += bf_hi(xr.x); v[2] += bf_lo(xr.y); v[3] += bf_hi(xr.y);
            *q = pack4(v);
          }
      }
    }
    const bool more = bi + 1 < a.nblk;
    const ResBlock Bn = a.blocks[more ? bi + 1 : bi];
    if (more) w_issue(w1, wst, a.packed + Bn.wf_off[0], LD, fr, fk);
    __syncthreads();
    if (INFER) {
      if (more) running_coef<C>(coef, a.running + Bn.run_off[0], a.params + Bn.gamma_off[0], a.params + Bn.beta_off[0], a.eps);
      else tile_store<C>(cx.tensor(B.y_off) + (size_t)me * P * C, sx, P);
      continue;
    }
    if (more) stats_publish<C>(sx, P, red, slot(), me, tag0 + 1u + phase);
    tile_store<C>(cx.tensor(B.y_off) + (size_t)me * P * C, sx, P);
    if (more) {
      if (!collect<4>(slot(), a.nmem, 2 * C, tag0 + 1u + phase, gath, a.abort_flag)) return;
      ++phase;
      w_commit(w1, wst, sW);
      merge_coef<C>(gath, a.nmem, P, a.eps, a.params + Bn.gamma_off[0], a.params + Bn.beta_off[0], coef,
                    me == 0 ? reinterpret_cast<float*>(cx.base + Bn.stats_off[0]) : nullptr);
    }
  }
  if (!INFER && me == 0 && tid == 0) *tagp = tag0 + phase;
}

template <int C, int PTW, bool PRE, bool WL = false>
__global__ void __launch_bounds__(RES_NT) k_bb_backward(const ResArgs a, const int gath_own) {
  static_assert(!(WL && PRE), "the LDS form replaces the fetch-where-used form");
  constexpr int XS = C + 8;
  const int tid = threadIdx.x, lane = tid & 63, wave = wave_index();
  const int fr = lane & 15, fq = lane >> 4, fk = fq * 8;
  const int H = C == 16 ? 32 : a.H, W = C == 16 ? 32 : a.W;   // as in the forward kernel
  const int P = H * W, npt = P >> 4;
  const int z = blockIdx.x % a.ngroup, me = blockIdx.x / a.ngroup;
  ResCtx cx{(char*)pick(a.base, z), pick(a.act_in, z), pick(a.act_out, z), pick(a.err_in, z), pick(a.err_out, z)};
  u64* xchg = reinterpret_cast<u64*>(cx.base + a.xchg_off);
  unsigned* tagp = reinterpret_cast<unsigned*>(cx.base + a.tag_off);
  const unsigned tag0 = *tagp;
  unsigned phase = 0;
  // 16 channels: the weight gradients go through the grouped launch, which knows nothing of the stored BatchNorm sums:
  // member 0 adds them into the gradients of beta and gamma itself
  constexpr bool DIRECT = C == 16;

  extern __shared__ __align__(16) unsigned char smem[];
  bf16_t* sdy = reinterpret_cast<bf16_t*>(smem);          // gradient of the residual stream
  bf16_t* sdc = sdy + (size_t)P * XS;                     // dc1
  float4* cf1 = reinterpret_cast<float4*>(sdc + (size_t)P * XS);
  float4* cf2 = cf1 + C;
  float* red = reinterpret_cast<float*>(cf2 + C);         // V1_RED(C) floats
  float4* tab = reinterpret_cast<float4*>(red + V1_RED(C));
  float* own = reinterpret_cast<float*>(tab + C);
  auto slot = [&]() { return xchg + (size_t)(phase & 1u) * a.nmem * (2 * C); };
  constexpr int KT = (9 * C + 31) / 32, LD = KT * 32;
  std::conditional_t<WL, WFragsL<KT, C / 16>, WFrags<KT, C / 16, PRE>> w2, w1;   // data-gradient operands [C][LD]
  bf16_t* sW = reinterpret_cast<bf16_t*>(own + (gath_own ? (size_t)a.nmem * 2 * C : 0));   // WL: the staged matrix
  u32x4 wst[WL ? (KT * (C / 16) + 7) / 8 : 1];

  // x / c1 (the BatchNorm inputs) are needed only at this lane's accumulator positions: read there from memory
  auto at_acc = [&](const bf16_t* g, uint2 (&xin)[PTW][C / 16]) {
#pragma unroll
    for (int j = 0; j < PTW; ++j) {
      const int pt = wave + j * RES_NWV;
      const size_t row = (size_t)((pt < npt ? pt : 0) * 16 + fr) * C + fq * 4;   // always a valid address
#pragma unroll
      for (int nt = 0; nt < C / 16; ++nt) xin[j][nt] = *reinterpret_cast<const uint2*>(g + row + nt * 16);
    }
  };
  {
    const ResBlock BL = a.blocks[a.nblk - 1];
    tile_load<C>(sdy, cx.tensor(BL.gy_off) + (size_t)me * P * C, P);
    if constexpr (WL) {   // the first block's conv2 matrix (the barrier below the tables precedes its use); later ones are
      w_issue(w2, wst, a.packed + BL.wd_off[1], LD, fr, fk);   // staged behind the last exchange of the block before
      w_commit(w2, wst, sW);
    }
  }
  for (int bi = a.nblk - 1; bi >= 0; --bi) {
    const ResBlock B = a.blocks[bi];
    uint2 xc0[PTW][C / 16], xc1[PTW][C / 16];
    {   // one round trip to memory for everything the block reads up front
      at_acc(cx.tensor(B.c1_off) + (size_t)me * P * C, xc1);
      at_acc(cx.tensor(B.x_off) + (size_t)me * P * C, xc0);
      const int c = tid < C ? tid : 0;
      const float4 t1 = BwdLoads<C, C, 1>::table(reinterpret_cast<const float*>(cx.base + B.stats_off[0]), a.params + B.gamma_off[0],
                                              a.params + B.beta_off[0], c, C);
      const float4 t2 = BwdLoads<C, C, 1>::table(reinterpret_cast<const float*>(cx.base + B.stats_off[1]), a.params + B.gamma_off[1],
                                              a.params + B.beta_off[1], c, C);
      if constexpr (!WL) w2.load(a.packed + B.wd_off[1], LD, fr, fk);
      if (tid < C) { cf1[tid] = t1; cf2[tid] = t2; }
    }
    __syncthreads();
    {   // ---- conv2 data gradient, BN2 + ReLU backward -> dc1
      floatx4 acc[PTW][C / 16];
      uint2 xin[PTW][C / 16];
#pragma unroll
      for (int j = 0; j < PTW; ++j)
#pragma unroll
        for (int nt = 0; nt < C / 16; ++nt) acc[j][nt] = floatx4{0.f, 0.f, 0.f, 0.f};
      conv3x3_tile<C, PTW, true>(sdy, w2, H, W, npt, wave, fr, fk, acc);
#pragma unroll
      for (int j = 0; j < PTW; ++j)
#pragma unroll
        for (int nt = 0; nt < C / 16; ++nt) xin[j][nt] = wave + j * RES_NWV < npt ? xc1[j][nt] : make_uint2(0u, 0u);
      w_issue(w1, wst, a.packed + B.wd_off[0], LD, fr, fk);
      float* gath = gath_own ? own : reinterpret_cast<float*>(sdc);
      if (!bn_relu_bwd_acc<C, PTW>(acc, xin, cf2, npt, wave, fr, fq, red, tab, gath, slot(), me, a.nmem, P, tag0 + 1u + phase,
                                   me == 0 && !DIRECT ? reinterpret_cast<float*>(cx.base + B.dgb_off[1]) : nullptr, a.abort_flag,
                                   [&](int j, int nt, const floatx4& out) {
                                     *reinterpret_cast<uint2*>(sdc + ((wave + j * RES_NWV) * 16 + fr) * XS + nt * 16 + fq * 4) = pack4(out);
                                   },
                                   me == 0 && DIRECT ? a.grads + B.beta_off[1] : nullptr, me == 0 && DIRECT ? a.grads + B.gamma_off[1] : nullptr))
        return;
      ++phase;
      w_commit(w1, wst, sW);
    }
    __syncthreads();
    tile_store<C>(cx.tensor(B.dc1_off) + (size_t)me * P * C, sdc, P);
    {   // ---- conv1 data gradient, BN1 + ReLU backward, plus the shortcut: dx = bn1_bwd(...) + dy over dy
      floatx4 acc[PTW][C / 16];
      uint2 xin[PTW][C / 16];
#pragma unroll
      for (int j = 0; j < PTW; ++j)
#pragma unroll
        for (int nt = 0; nt < C / 16; ++nt) acc[j][nt] = floatx4{0.f, 0.f, 0.f, 0.f};
      conv3x3_tile<C, PTW, true>(sdc, w1, H, W, npt, wave, fr, fk, acc);
      if constexpr (WL)
        if (bi > 0) w_issue(w2, wst, a.packed + a.blocks[bi - 1].wd_off[1], LD, fr, fk);   // the next block's conv2 matrix
#pragma unroll
      for (int j = 0; j < PTW; ++j)
#pragma unroll
        for (int nt = 0; nt < C / 16; ++nt) xin[j][nt] = wave + j * RES_NWV < npt ? xc0[j][nt] : make_uint2(0u, 0u);
      // dc1 is read for the last time by the contraction above; the barrier inside the BatchNorm backward lies
      // between that and the first write of the gathered words
      float* gath = gath_own ? own : reinterpret_cast<float*>(sdc);
      if (!bn_relu_bwd_acc<C, PTW>(acc, xin, cf1, npt, wave, fr, fq, red, tab, gath, slot(), me, a.nmem, P, tag0 + 1u + phase,
                                   me == 0 && !DIRECT ? reinterpret_cast<float*>(cx.base + B.dgb_off[0]) : nullptr, a.abort_flag,
                                   [&](int j, int nt, const floatx4& out) {
                                     uint2* q = reinterpret_cast<uint2*>(sdy + ((wave + j * RES_NWV) * 16 + fr) * XS + nt * 16 + fq * 4);
                                     const uint2 d = *q;
                                     floatx4 v = out;
                                     v[0] += bf_lo(d.x); v[1] += bf_hi(d.x); v[2] += bf_lo(d.y); v[3] += bf_hi(d.y);
                                     *q = pack4(v);
                                   },
                                   me == 0 && DIRECT ? a.grads + B.beta_off[0] : nullptr, me == 0 && DIRECT ? a.grads + B.gamma_off[0] : nullptr))
        return;
      ++phase;
      if constexpr (WL)
        if (bi > 0) w_commit(w2, wst, sW);   // every wave is past conv1's data gradient: the barriers of the BatchNorm backward
    }
    __syncthreads();
    tile_store<C>(cx.tensor(B.gx_off) + (size_t)me * P * C, sdy, P);
  }
  if (me == 0 && tid == 0) *tagp = tag0 + phase;
}

// weight gradients of a run of basic blocks: grid (image groups, 2 convolutions, blocks)
template <int C>
__global__ void __launch_bounds__(rw_threads(C)) k_bb_wgrad(const ResWgArgs a) {
  constexpr int NTH = rw_threads(C);
  extern __shared__ __align__(16) unsigned char smem[];
  const ResBlock B = a.blocks[blockIdx.z];
  const int img0 = blockIdx.x * a.ipw;
  if (blockIdx.y == 0) {
    res_wgrad_3x3<C, NTH>(a, img0, B.x_off, B.stats_off[0], a.params + B.gamma_off[0], a.params + B.beta_off[0], B.dc1_off,
                     a.grads + B.w_off[0], smem);
    if (blockIdx.x == 0) {
      add_bn_param_grads<NTH>(a, B.dgb_off[0], a.grads + B.beta_off[0], a.grads + B.gamma_off[0], C);
      add_bn_param_grads<NTH>(a, B.dgb_off[1], a.grads + B.beta_off[1], a.grads + B.gamma_off[1], C);
    }
  } else
    res_wgrad_3x3<C, NTH>(a, img0, B.c1_off, B.stats_off[1], a.params + B.gamma_off[1], a.params + B.beta_off[1], B.gy_off,
                     a.grads + B.w_off[1], smem);
}

// ------------------------------------------------------------------------------------------ post-activation blocks
// The same ownership for runs of post-activation basic blocks with identity shortcut (ResNet-v1, paper Section
// "Model-Parallelism on a Single Node": ResNet-110-v1):
//   c1 = conv1(x); a1 = relu(bn1(c1)); c2 = conv2(a1); y = relu(bn2(c2) + x).
// x is the stored output of the block before, so conv1 reads it as it is and nothing is exchanged ahead of the first
// block; two exchanges per block and direction (statistics of c1 and c2; sums of the two BatchNorm backward passes).
// Backward: dz = dy*[y > 0] is the gradient of the shortcut and, through BN2's backward (no ReLU of its own), of c2.
// ResBlock fields used: x, c1, c2, y, gy, dc1, dc2, gx and entries 0 / 1 of the per-BatchNorm / per-convolution arrays.
// The weight gradients of the 32- and 64-channel runs have a launch of their own (k_v1_wgrad, further down), those of
// the 16-channel runs go through the grouped per-layer launch; inference goes through the per-layer kernels.

// y = relu(c2*scale + shift + x), tile to tile (written over x)
template <int Cc>
__device__ __forceinline__ void tile_join_relu(bf16_t* sx, const bf16_t* sc2, const float2* coef, int P) {
  constexpr int U = Cc / 8;
  for (int u = threadIdx.x; u < P * U; u += RES_NT) {
    const int row = u / U, col = u - row * U;
    uint4* q = reinterpret_cast<uint4*>(sx + row * (Cc + 8) + col * 8);
    const uint4 xv = *q, cv = *reinterpret_cast<const uint4*>(sc2 + row * (Cc + 8) + col * 8);
    const uint32_t xw[4] = {xv.x, xv.y, xv.z, xv.w}, cw[4] = {cv.x, cv.y, cv.z, cv.w};
    const float4* cf = reinterpret_cast<const float4*>(coef + col * 8);
    uint32_t r[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float4 k = cf[i];
      r[i] = pack_bf16x2(fmaxf(fmaf(bf_lo(cw[i]), k.x, k.y) + bf_lo(xw[i]), 0.f), fmaxf(fmaf(bf_hi(cw[i]), k.z, k.w) + bf_hi(xw[i]), 0.f));
    }
    *q = make_uint4(r[0], r[1], r[2], r[3]);
  }
}

template <int C, int PTW, bool PRE, bool WL = false>
__global__ void __launch_bounds__(RES_NT) k_v1_forward(const ResArgs a, const int gath_own) {
  static_assert(!(WL && PRE), "the LDS form replaces the fetch-where-used form");
  constexpr int XS = C + 8;
  const int tid = threadIdx.x, lane = tid & 63, wave = wave_index();
  const int fr = lane & 15, fq = lane >> 4, fk = fq * 8;
  // the 16-channel shape is 32 x 32 pixels only: constants instead of kernel arguments (fewer address temporaries)
  const int H = C == 16 ? 32 : a.H, W = C == 16 ? 32 : a.W;
  const int P = H * W, npt = P >> 4;
  const int z = blockIdx.x % a.ngroup, me = blockIdx.x / a.ngroup;
  ResCtx cx{(char*)pick(a.base, z), pick(a.act_in, z), pick(a.act_out, z), pick(a.err_in, z), pick(a.err_out, z)};
  u64* xchg = reinterpret_cast<u64*>(cx.base + a.xchg_off);
  unsigned* tagp = reinterpret_cast<unsigned*>(cx.base + a.tag_off);
  const unsigned tag0 = *tagp;
  unsigned phase = 0;

  extern __shared__ __align__(16) unsigned char smem[];
  bf16_t* sx = reinterpret_cast<bf16_t*>(smem);           // block input, then block output, [P][XS]
  bf16_t* sB = sx + (size_t)P * XS;                       // c1, then relu(bn1(c1))
  bf16_t* sC = sB + (size_t)P * XS;                       // c2
  float2* coef = reinterpret_cast<float2*>(sC + (size_t)P * XS);
  float* red = reinterpret_cast<float*>(coef + C);        // V1_RED(C) floats
  float* own = red + V1_RED(C);
  auto slot = [&]() { return xchg + (size_t)(phase & 1u) * a.nmem * (2 * C); };
  constexpr int KT = (9 * C + 31) / 32, LD = KT * 32;     // reduction steps and row length of the packed weights
  std::conditional_t<WL, WFragsL<KT, C / 16>, WFrags<KT, C / 16, PRE>> w1, w2;
  bf16_t* sW = reinterpret_cast<bf16_t*>(own + (gath_own ? (size_t)a.nmem * 2 * C : 0));   // WL: the staged matrix
  u32x4 wst[WL ? (KT * (C / 16) + 7) / 8 : 1];                                              // WL: its units on their way

  auto store_acc = [&](bf16_t* dst, floatx4 (&acc)[PTW][C / 16]) {
#pragma unroll
    for (int j = 0; j < PTW; ++j) {
      const int pt = wave + j * RES_NWV;
      if (pt < npt)
#pragma unroll
        for (int nt = 0; nt < C / 16; ++nt)
          *reinterpret_cast<uint2*>(dst + (pt * 16 + fr) * XS + nt * 16 + fq * 4) = pack4(acc[j][nt]);
    }
  };
  {
    const ResBlock B0 = a.blocks[0];
    tile_load<C>(sx, cx.tensor(B0.x_off) + (size_t)me * P * C, P);
    w_issue(w1, wst, a.packed + B0.wf_off[0], LD, fr, fk);
    w_commit(w1, wst, sW);
    __syncthreads();
  }
  for (int bi = 0; bi < a.nblk; ++bi) {
    const ResBlock B = a.blocks[bi];
    {   // ---- conv1 (3x3) on x
      floatx4 acc[PTW][C / 16];
#pragma unroll
      for (int j = 0; j < PTW; ++j)
#pragma unroll
        for (int nt = 0; nt < C / 16; ++nt) acc[j][nt] = floatx4{0.f, 0.f, 0.f, 0.f};
      conv3x3_tile<C, PTW, false>(sx, w1, H, W, npt, wave, fr, fk, acc);
      store_acc(sB, acc);
    }
    w_issue(w2, wst, a.packed + B.wf_off[1], LD, fr, fk);
    __syncthreads();
    {
      float* gath = gath_own ? own : reinterpret_cast<float*>(sC);   // c2 of the block before has been consumed
      stats_publish<C>(sB, P, red, slot(), me, tag0 + 1u + phase);
      tile_store<C>(cx.tensor(B.c1_off) + (size_t)me * P * C, sB, P);
      if (!collect<4>(slot(), a.nmem, 2 * C, tag0 + 1u + phase, gath, a.abort_flag)) return;
      ++phase;
      w_commit(w2, wst, sW);   // conv1 read its matrix above the barrier before the statistics
      merge_coef<C>(gath, a.nmem, P, a.eps, a.params + B.gamma_off[0], a.params + B.beta_off[0], coef,
                    me == 0 ? reinterpret_cast<float*>(cx.base + B.stats_off[0]) : nullptr);
    }
    tile_bn_relu<C>(sB, coef, P);
    __syncthreads();
    {   // ---- conv2 (3x3) on relu(bn1(c1))
      floatx4 acc[PTW][C / 16];
#pragma unroll
      for (int j = 0; j < PTW; ++j)
#pragma unroll
        for (int nt = 0; nt < C / 16; ++nt) acc[j][nt] = floatx4{0.f, 0.f, 0.f, 0.f};
      conv3x3_tile<C, PTW, false>(sB, w2, H, W, npt, wave, fr, fk, acc);
      store_acc(sC, acc);
    }
    if (bi + 1 < a.nblk) w_issue(w1, wst, a.packed + a.blocks[bi + 1].wf_off[0], LD, fr, fk);
    __syncthreads();
    {
      float* gath = gath_own ? own : reinterpret_cast<float*>(sB);   // conv2 has read relu(bn1(c1)): barrier above
      stats_publish<C>(sC, P, red, slot(), me, tag0 + 1u + phase);
      tile_store<C>(cx.tensor(B.c2_off) + (size_t)me * P * C, sC, P);
      if (!collect<4>(slot(), a.nmem, 2 * C, tag0 + 1u + phase, gath, a.abort_flag)) return;
      ++phase;
      if (bi + 1 < a.nblk) w_commit(w1, wst, sW);
      merge_coef<C>(gath, a.nmem, P, a.eps, a.params + B.gamma_off[1], a.params + B.beta_off[1], coef,
                    me == 0 ? reinterpret_cast<float*>(cx.base + B.stats_off[1]) : nullptr);
    }
    tile_join_relu<C>(sx, sC, coef, P);
    __syncthreads();
    tile_store<C>(cx.tensor(B.y_off) + (size_t)me * P * C, sx, P);
  }
  if (me == 0 && tid == 0) *tagp = tag0 + phase;
}

// BatchNorm backward on a gradient tile in accumulator layout (cf. bn_relu_bwd_acc), for the two BatchNorms of a
// post-activation block.  JOIN = false: BN + ReLU backward, the mask recomputed from the BatchNorm input xin.
// JOIN = true: the ReLU sits behind the shortcut add, so the mask is [y > 0] with y = ysrc the stored block output;
// dz is left masked in place (it is also the gradient of the shortcut) and the BatchNorm itself has no ReLU.
// g_beta / g_gamma (member 0 only, else null): the micro-batch sums are added to the parameter gradients.
template <int Cc, int PTW, bool JOIN, class Fin>
__device__ __forceinline__ bool v1_bn_bwd_acc(floatx4 (&dz)[PTW][Cc / 16], const uint2 (&xin)[PTW][Cc / 16], const uint2 (&ysrc)[PTW][Cc / 16],
                                              const float4* cf_, int npt, int wave, int fr, int fq, float* red, float4* tab_, float* gath,
                                              u64* slot, int me, int nmem, int P, unsigned tag, float* g_beta, float* g_gamma,
                                              int* abort_flag, Fin&& fin) {
  constexpr int NTL = Cc / 16;
  const float4* cf = reinterpret_cast<const float4*>(__builtin_assume_aligned(cf_, 16));
  float4* tab = reinterpret_cast<float4*>(__builtin_assume_aligned(tab_, 16));
#pragma unroll
  for (int nt = 0; nt < NTL; ++nt) {
    float4 k[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) k[e] = cf[nt * 16 + fq * 4 + e];
    float sb[4] = {0.f, 0.f, 0.f, 0.f}, sg[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < PTW; ++j) {
      if (wave + j * RES_NWV < npt) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float v = elem4(xin[j][nt], e);
          const bool on = JOIN ? elem4(ysrc[j][nt], e) > 0.f : fmaf(v, k[e].x, k[e].y) > 0.f;
          const float d = on ? dz[j][nt][e] : 0.f;
          dz[j][nt][e] = d;
          sb[e] += d;
          sg[e] = fmaf(d, fmaf(v, k[e].z, k[e].w), sg[e]);
        }
      }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) { sb[e] = sum16(sb[e]); sg[e] = sum16(sg[e]); }
    if (fr == 0) {
      *reinterpret_cast<float4*>(red + wave * 2 * Cc + nt * 16 + fq * 4) = make_float4(sb[0], sb[1], sb[2], sb[3]);
      *reinterpret_cast<float4*>(red + wave * 2 * Cc + Cc + nt * 16 + fq * 4) = make_float4(sg[0], sg[1], sg[2], sg[3]);
    }
  }
  __syncthreads();
  for (int w = threadIdx.x; w < 2 * Cc; w += RES_NT) {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < RES_NWV; ++i) s += red[i * 2 * Cc + w];
    publish_word(slot, me, 2 * Cc, w, s, tag);
  }
  if (!collect<4, true>(slot, nmem, 2 * Cc, tag, gath, abort_flag)) return false;
  const float invM = 1.f / ((float)nmem * (float)P);
  {
    constexpr int CR = Cc >= 32 ? Cc / 32 : 1, MP = 16 / CR;
    const int l16 = threadIdx.x & 15, row = threadIdx.x >> 4;
    const bool act = row * CR < Cc;
    const int c = act ? row * CR + l16 % CR : 0, part = l16 / CR;
    float sb = 0.f, sg = 0.f;
    for (int m = part; m < nmem; m += MP) { sb += gath[m * 2 * Cc + c]; sg += gath[m * 2 * Cc + Cc + c]; }
    sb = row_sum<CR>(sb);
    sg = row_sum<CR>(sg);
    if (act && part == 0) {
      if (g_beta) { atomicAdd(g_beta + c, sb); atomicAdd(g_gamma + c, sg); }
      const float4 k = cf[c];
      tab[c] = make_float4(k.x, -k.x * sg * invM * k.z, -k.x * invM * (sb + k.w * sg), 0.f);
    }
  }
  __syncthreads();
#pragma unroll
  for (int nt = 0; nt < NTL; ++nt) {
    float4 t[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) t[e] = tab[nt * 16 + fq * 4 + e];
#pragma unroll
    for (int j = 0; j < PTW; ++j) {
      if (wave + j * RES_NWV < npt) {
        floatx4 out;
#pragma unroll
        for (int e = 0; e < 4; ++e) out[e] = fmaf(t[e].x, dz[j][nt][e], fmaf(t[e].y, elem4(xin[j][nt], e), t[e].z));
        fin(j, nt, out);
      }
    }
  }
  return true;
}

template <int C, int PTW, bool PRE, bool WL = false>
__global__ void __launch_bounds__(RES_NT) k_v1_backward(const ResArgs a, const int gath_own) {
  static_assert(!(WL && PRE), "the LDS form replaces the fetch-where-used form");
  constexpr int XS = C + 8;
  const int tid = threadIdx.x, lane = tid & 63, wave = wave_index();
  const int fr = lane & 15, fq = lane >> 4, fk = fq * 8;
  // the 16-channel shape is 32 x 32 pixels only: constants instead of kernel arguments (fewer address temporaries)
  const int H = C == 16 ? 32 : a.H, W = C == 16 ? 32 : a.W;
  const int P = H * W, npt = P >> 4;
  const int z = blockIdx.x % a.ngroup, me = blockIdx.x / a.ngroup;
  ResCtx cx{(char*)pick(a.base, z), pick(a.act_in, z), pick(a.act_out, z), pick(a.err_in, z), pick(a.err_out, z)};
  u64* xchg = reinterpret_cast<u64*>(cx.base + a.xchg_off);
  unsigned* tagp = reinterpret_cast<unsigned*>(cx.base + a.tag_off);
  const unsigned tag0 = *tagp;
  unsigned phase = 0;

  extern __shared__ __align__(16) unsigned char smem[];
  bf16_t* sdy = reinterpret_cast<bf16_t*>(smem);          // gradient w.r.t. the block output, then w.r.t. its input
  bf16_t* sdc = sdy + (size_t)P * XS;                     // dc2, then dc1
  float4* cf1 = reinterpret_cast<float4*>(sdc + (size_t)P * XS);
  float4* cf2 = cf1 + C;
  float* red = reinterpret_cast<float*>(cf2 + C);         // V1_RED(C) floats
  float4* tab = reinterpret_cast<float4*>(red + V1_RED(C));
  float* own = reinterpret_cast<float*>(tab + C);
  auto slot = [&]() { return xchg + (size_t)(phase & 1u) * a.nmem * (2 * C); };
  constexpr int KT = (9 * C + 31) / 32, LD = KT * 32;
  std::conditional_t<WL, WFragsL<KT, C / 16>, WFrags<KT, C / 16, PRE>> w2, w1;   // data-gradient operands [C][LD]
  bf16_t* sW = reinterpret_cast<bf16_t*>(own + (gath_own ? (size_t)a.nmem * 2 * C : 0));   // WL: the staged matrix
  u32x4 wst[WL ? (KT * (C / 16) + 7) / 8 : 1];

  auto at_acc = [&](const bf16_t* g, uint2 (&xin)[PTW][C / 16]) {
#pragma unroll
    for (int j = 0; j < PTW; ++j) {
      const int pt = wave + j * RES_NWV;
      const size_t row = (size_t)((pt < npt ? pt : 0) * 16 + fr) * C + fq * 4;   // always a valid address
#pragma unroll
      for (int nt = 0; nt < C / 16; ++nt) xin[j][nt] = *reinterpret_cast<const uint2*>(g + row + nt * 16);
    }
  };
  {
    const ResBlock BL = a.blocks[a.nblk - 1];
    tile_load<C>(sdy, cx.tensor(BL.gy_off) + (size_t)me * P * C, P);
  }
  for (int bi = a.nblk - 1; bi >= 0; --bi) {
    const ResBlock B = a.blocks[bi];
    float* const gb1 = me == 0 ? a.grads + B.beta_off[0] : nullptr;
    float* const gb2 = me == 0 ? a.grads + B.beta_off[1] : nullptr;
    uint2 xc1[PTW][C / 16], xc2[PTW][C / 16], yv[PTW][C / 16];
    floatx4 dzs[PTW][C / 16];   // dy*[y > 0]: the gradient of the shortcut, added to the input gradient at the end
    {   // one round trip to memory for everything the block reads up front
      at_acc(cx.tensor(B.y_off) + (size_t)me * P * C, yv);
      at_acc(cx.tensor(B.c2_off) + (size_t)me * P * C, xc2);
      at_acc(cx.tensor(B.c1_off) + (size_t)me * P * C, xc1);
      const int c = tid < C ? tid : 0;
      const float4 t1 = BwdLoads<C, C, 1>::table(reinterpret_cast<const float*>(cx.base + B.stats_off[0]), a.params + B.gamma_off[0],
                                              a.params + B.beta_off[0], c, C);
      const float4 t2 = BwdLoads<C, C, 1>::table(reinterpret_cast<const float*>(cx.base + B.stats_off[1]), a.params + B.gamma_off[1],
                                              a.params + B.beta_off[1], c, C);
      w_issue(w2, wst, a.packed + B.wd_off[1], LD, fr, fk);
      if (tid < C) { cf1[tid] = t1; cf2[tid] = t2; }
    }
    __syncthreads();   // the tables; and (first block) the gradient tile
    {   // ---- through the join and BN2: dz = dy*[y > 0] -> dc2
#pragma unroll
      for (int j = 0; j < PTW; ++j) {
        const int pt = wave + j * RES_NWV;
#pragma unroll
        for (int nt = 0; nt < C / 16; ++nt) {
          const uint2 d = pt < npt ? *reinterpret_cast<const uint2*>(sdy + (pt * 16 + fr) * XS + nt * 16 + fq * 4) : make_uint2(0u, 0u);
          dzs[j][nt] = floatx4{bf_lo(d.x), bf_hi(d.x), bf_lo(d.y), bf_hi(d.y)};
        }
      }
      float* gath = gath_own ? own : reinterpret_cast<float*>(sdc);
      if (!v1_bn_bwd_acc<C, PTW, true>(dzs, xc2, yv, cf2, npt, wave, fr, fq, red, tab, gath, slot(), me, a.nmem, P, tag0 + 1u + phase, gb2,
                                       a.grads + B.gamma_off[1], a.abort_flag, [&](int j, int nt, const floatx4& out) {
                                         *reinterpret_cast<uint2*>(sdc + ((wave + j * RES_NWV) * 16 + fr) * XS + nt * 16 + fq * 4) = pack4(out);
                                       }))
        return;
      ++phase;
      w_commit(w2, wst, sW);   // the matrix staged before was last read above the barrier that ends the block before
    }
    __syncthreads();
    tile_store<C>(cx.tensor(B.dc2_off) + (size_t)me * P * C, sdc, P);
    {   // ---- conv2 data gradient, BN1 + ReLU backward -> dc1 (over dc2)
      floatx4 acc[PTW][C / 16];
      uint2 xin[PTW][C / 16];
#pragma unroll
      for (int j = 0; j < PTW; ++j)
#pragma unroll
        for (int nt = 0; nt < C / 16; ++nt) acc[j][nt] = floatx4{0.f, 0.f, 0.f, 0.f};
      conv3x3_tile<C, PTW, true>(sdc, w2, H, W, npt, wave, fr, fk, acc);
#pragma unroll
      for (int j = 0; j < PTW; ++j)
#pragma unroll
        for (int nt = 0; nt < C / 16; ++nt) xin[j][nt] = wave + j * RES_NWV < npt ? xc1[j][nt] : make_uint2(0u, 0u);
      w_issue(w1, wst, a.packed + B.wd_off[0], LD, fr, fk);
      // every wave is past its reads of dc2 at the first barrier inside; the results are written behind the last one
      float* gath = gath_own ? own : reinterpret_cast<float*>(sdc);
      if (!v1_bn_bwd_acc<C, PTW, false>(acc, xin, xin, cf1, npt, wave, fr, fq, red, tab, gath, slot(), me, a.nmem, P, tag0 + 1u + phase, gb1,
                                        a.grads + B.gamma_off[0], a.abort_flag, [&](int j, int nt, const floatx4& out) {
                                          *reinterpret_cast<uint2*>(sdc + ((wave + j * RES_NWV) * 16 + fr) * XS + nt * 16 + fq * 4) = pack4(out);
                                        }))
        return;
      ++phase;
      w_commit(w1, wst, sW);
    }
    __syncthreads();
    tile_store<C>(cx.tensor(B.dc1_off) + (size_t)me * P * C, sdc, P);
    {   // ---- conv1 data gradient plus the shortcut: dx = conv1^T(dc1) + dz, written over dy
      floatx4 acc[PTW][C / 16];
#pragma unroll
      for (int j = 0; j < PTW; ++j)
#pragma unroll
        for (int nt = 0; nt < C / 16; ++nt) acc[j][nt] = dzs[j][nt];
      conv3x3_tile<C, PTW, true>(sdc, w1, H, W, npt, wave, fr, fk, acc);
#pragma unroll
      for (int j = 0; j < PTW; ++j) {
        const int pt = wave + j * RES_NWV;
        if (pt < npt)
#pragma unroll
          for (int nt = 0; nt < C / 16; ++nt)
            *reinterpret_cast<uint2*>(sdy + (pt * 16 + fr) * XS + nt * 16 + fq * 4) = pack4(acc[j][nt]);
      }
    }
    __syncthreads();
    tile_store<C>(cx.tensor(B.gx_off) + (size_t)me * P * C, sdy, P);
  }
  if (me == 0 && tid == 0) *tagp = tag0 + phase;
}

// weight gradients of a run of post-activation blocks: grid (image groups, 2 convolutions, blocks).  conv1 takes the
// stored block input as it is, conv2 relu(bn1(c1)) recomputed while staging; the BatchNorm parameter gradients were
// added by the backward launch.
template <int C>
__global__ void __launch_bounds__(rw_threads(C)) k_v1_wgrad(const ResWgArgs a) {
  constexpr int NTH = rw_threads(C);
  extern __shared__ __align__(16) unsigned char smem[];
  const ResBlock B = a.blocks[blockIdx.z];
  const int img0 = blockIdx.x * a.ipw;
  if (blockIdx.y == 0)
    res_wgrad_3x3<C, NTH>(a, img0, B.x_off, 0, nullptr, nullptr, B.dc1_off, a.grads + B.w_off[0], smem);
  else
    res_wgrad_3x3<C, NTH>(a, img0, B.c1_off, B.stats_off[0], a.params + B.gamma_off[0], a.params + B.beta_off[0], B.dc2_off,
                     a.grads + B.w_off[1], smem);
}

// ------------------------------------------------------------------------------------------ row bands
// Runs of identity bottleneck blocks whose image does not fit one CU's LDS (ResNet-1001's first stage: 64-16-16-64
// channels at 32x32, 128 KiB of residual stream per image): the image is cut into bands of BAND_ROWS image rows and
// one work-group owns one band.  In NHWC a band is a contiguous range of 256 pixels, so every tensor of the band
// sits at member_index * 256 * channels, exactly like an image of the kernels above; what is new is the 3x3
// convolution, which needs the image rows just above and below the band.  Those two rows of c1 (bf16, as stored)
// travel with the BatchNorm records of the exchange that separates conv1 from conv2 anyway -- each work-group
// publishes its first and last row next to its {mean, M2} record and collects the facing rows of its two
// neighbours -- so a block still has three exchanges.  The members of an exchange are the bands of all images of the
// micro-batch (statistics are over the micro-batch); neighbours are the members me - 1 / me + 1 of the same image.
// A reduction of 16 channels per filter tap fills half an MFMA step, so a step of the 3x3 convolution covers two
// taps (lane groups 0-1 the first, 2-3 the second; the packed weights have k = tap*16 + c contiguous, which is the
// same thing), and the 1x1 convolution out of 16 channels runs a half-empty step against zero-padded weights.
constexpr int BAND_ROWS = 8, BAND_W = 32, BAND_P = BAND_ROWS * BAND_W;   // 256 pixels = 16 pixel tiles, two per wave
constexpr int BAND_PTW = BAND_P / 16 / RES_NWV;
constexpr int BAND_HALO_F = BAND_W * 16 / 2;     // words of one row of 16 bf16 channels (two values per word)
constexpr int BAND_HALO_B = BAND_W * 16;         // words of one row of 16 fp32 channels (backward)
constexpr int BAND_RW = 2 * 16 + 2 * BAND_HALO_B;   // record width in words: the widest record (sums + two rows of dz, backward), >= 2*64
static_assert(BAND_RW >= 2 * 64 && BAND_PTW == 2, "record width / tiles per wave");

// Collects, from the records of all nwg members, the first ns words each into gath[m*ns + w], and nh words from
// offset off_up of member `up` / off_dn of member `dn` (a negative member: none, nothing is read) into halo[0..nh) /
// halo[nh..2nh) as raw 32-bit payloads.  Returns false, uniformly, when a word did not arrive.  Ends with a barrier.
__device__ __forceinline__ bool band_collect(const u64* slot, int nwg, int ns, unsigned tag, float* gath, int up, int dn, int off_up,
                                             int off_dn, int nh, uint32_t* halo, int* abort_flag) {
  constexpr int INFL = 8;   // words in flight per thread and polling round
  const int n_stats = nwg * ns, total = n_stats + 2 * nh;
  int timed_out = 0;
  for (int i0 = threadIdx.x; i0 < total; i0 += RES_NT * INFL) {
    const u64* src[INFL];
    bool want[INFL];
    u64 v[INFL];
#pragma unroll
    for (int k = 0; k < INFL; ++k) {
      const int i = i0 + k * RES_NT;
      want[k] = i < total;
      src[k] = slot;
      v[k] = 0;
      if (i < n_stats) {
        const int m = i / ns;
        src[k] = slot + (size_t)m * BAND_RW + (i - m * ns);
      } else if (i < total) {
        const int j = i - n_stats, second = j >= nh ? 1 : 0, w = j - second * nh;
        const int mem = second ? dn : up;
        want[k] = mem >= 0;
        src[k] = slot + (size_t)(mem >= 0 ? mem : 0) * BAND_RW + (second ? off_dn : off_up) + w;
      }
    }
    unsigned spins = 0;
    for (;;) {
#pragma unroll
      for (int k = 0; k < INFL; ++k)
        if (want[k]) v[k] = __hip_atomic_load(src[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      bool all = true;
#pragma unroll
      for (int k = 0; k < INFL; ++k) all = all && (!want[k] || (unsigned)(v[k] >> 32) == tag);
      if (all) break;
      if (++spins > RES_SPIN_LIMIT) { timed_out = 1; break; }
    }
#pragma unroll
    for (int k = 0; k < INFL; ++k) {
      const int i = i0 + k * RES_NT;
      if (i < n_stats) gath[i] = __uint_as_float((unsigned)v[k]);
      else if (i < total) halo[i - n_stats] = want[k] ? (uint32_t)v[k] : 0u;
    }
  }
  const int any = __syncthreads_or(timed_out);
  if (any && threadIdx.x == 0) atomicExch(abort_flag, 1);
  return any == 0;
}

// stats_publish for a record of width BAND_RW: words c and Cc + c of `rec`.
template <int Cc>
__device__ __forceinline__ void band_stats_publish(const bf16_t* s, float* red, u64* rec, unsigned tag) {
  constexpr int U = Cc / 8, NG = 32 / U, P = BAND_P;
  static_assert(U <= 32 && 32 % U == 0, "unit count");
  const int l16 = threadIdx.x & 15, row = threadIdx.x >> 4;
  const int unit = row % U, grp = row / U;
  float K[8], s1[8], s2[8];
  load8(s + unit * 8, K);
#pragma unroll
  for (int i = 0; i < 8; ++i) { s1[i] = 0.f; s2[i] = 0.f; }
  for (int p = grp * 16 + l16; p < P; p += NG * 16) {
    float v[8];
    load8(s + p * (Cc + 8) + unit * 8, v);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float d = v[i] - K[i];
      s1[i] += d;
      s2[i] = fmaf(d, d, s2[i]);
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) { s1[i] = row_sum<1>(s1[i]); s2[i] = row_sum<1>(s2[i]); }
  if (l16 == 0) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      red[grp * 2 * Cc + unit * 8 + i] = s1[i];
      red[grp * 2 * Cc + Cc + unit * 8 + i] = s2[i];
    }
  }
  __syncthreads();
  if (threadIdx.x < Cc) {
    const int c = threadIdx.x;
    float S1 = 0.f, S2 = 0.f;
#pragma unroll
    for (int i = 0; i < NG; ++i) { S1 += red[i * 2 * Cc + c]; S2 += red[i * 2 * Cc + Cc + c]; }
    const float inv = 1.f / (float)P;
    __hip_atomic_store(rec + c, ((u64)tag << 32) | (u64)__float_as_uint(bf16_to_f32(s[c]) + S1 * inv), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(rec + Cc + c, ((u64)tag << 32) | (u64)__float_as_uint(fmaxf(S2 - S1 * S1 * inv, 0.f)), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

// merge_coef for 16 <= Cc: channels are dealt to the rows of 16 lanes CR at a time (CR = 1 below 32 channels, where
// only the first Cc rows work), the lanes of a row split the members.  Ends with a barrier.
template <int Cc>
__device__ __forceinline__ void band_merge_coef(const float* gath, int nwg, float eps, const float* gamma, const float* beta, float2* coef,
                                                float* stats_out) {
  constexpr int CR = Cc >= 32 ? Cc / 32 : 1, MP = 16 / CR, ROWS = Cc / CR;
  const int l16 = threadIdx.x & 15, row = threadIdx.x >> 4;
  const bool act = row < ROWS;
  const int c = act ? row * CR + l16 % CR : 0, part = l16 / CR;
  const float g = gamma[c], b = beta[c];
  float s = 0.f;
  for (int m = part; m < nwg; m += MP) s += gath[m * 2 * Cc + c];
  s = row_sum<CR>(s);
  const float inv_n = 1.f / (float)nwg;
  const float mean = s * inv_n;
  float s2 = 0.f;
  for (int m = part; m < nwg; m += MP) {
    const float d = gath[m * 2 * Cc + c] - mean;
    s2 += gath[m * 2 * Cc + Cc + c] + (float)BAND_P * d * d;
  }
  s2 = row_sum<CR>(s2);
  if (act && part == 0) {
    const float var = s2 * inv_n / (float)BAND_P;
    const float is = 1.0f / sqrtf(var + eps);
    coef[c] = bn_scale_shift(mean, is, g, b);
    if (stats_out) { stats_out[c] = mean; stats_out[Cc + c] = is; }
  }
  __syncthreads();
}

// 3x3 convolution of 16 -> 16 channels over a band tile with one halo row above and below: src is [10 rows][32][MS],
// output pixel (r, q) of the band reads tile rows r .. r+2; two filter taps per MFMA step (see above).  Weights
// [16][160] bf16, k = tap*16 + c (forward) or tap*16 + n (backward), zero beyond k = 144.
template <bool BACKWARD, class WF>
__device__ __forceinline__ void band_conv3x3(const bf16_t* src, const WF& wfr, int wave, int fr, int fq, floatx4 (&acc)[BAND_PTW][1]) {
  constexpr int MS = 16 + 8;
  int py[BAND_PTW], px[BAND_PTW];
#pragma unroll
  for (int j = 0; j < BAND_PTW; ++j) {
    const int p = (wave + j * RES_NWV) * 16 + fr;
    py[j] = p / BAND_W;
    px[j] = p - py[j] * BAND_W;
  }
  const int c8 = (fq & 1) * 8;
#pragma unroll
  for (int st = 0; st < 5; ++st) {
    const int tap = 2 * st + (fq >> 1);
    const int r = tap / 3, s = tap - r * 3;
    const int dh = BACKWARD ? 1 - r : r - 1, dw = BACKWARD ? 1 - s : s - 1;
    const bf16x8 wf = wfr.get(st, 0);
#pragma unroll
    for (int j = 0; j < BAND_PTW; ++j) {
      const int ws = px[j] + dw;
      const bool ok = tap < 9 && (unsigned)ws < (unsigned)BAND_W;
      const int row = ok ? (py[j] + 1 + dh) * BAND_W + ws : 0;
      bf16x8 bfrag = *reinterpret_cast<const bf16x8*>(src + row * MS + c8);
      if (!ok) bfrag = frag_zero();
      acc[j][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, bfrag, acc[j][0], 0, 0, 0);
    }
  }
}

template <int C, int MID>
__global__ void __launch_bounds__(RES_NT) k_band_forward(const ResArgs a) {
  static_assert(C == 64 && MID == 16, "the shape of ResNet-1001's first stage");
  constexpr int XS = C + 8, MS = MID + 8, P = BAND_P, PTW = BAND_PTW;
  const int tid = threadIdx.x, lane = tid & 63, wave = wave_index();
  const int fr = lane & 15, fq = lane >> 4, fk = fq * 8;
  const int nb = a.H / BAND_ROWS, nwg = a.nmem * nb;      // bands per image, members of an exchange
  const int z = blockIdx.x % a.ngroup, me = blockIdx.x / a.ngroup;
  const int band = me % nb;
  const int up = band > 0 ? me - 1 : -1, dn = band + 1 < nb ? me + 1 : -1;
  ResCtx cx{(char*)pick(a.base, z), pick(a.act_in, z), pick(a.act_out, z), pick(a.err_in, z), pick(a.err_out, z)};
  u64* xchg = reinterpret_cast<u64*>(cx.base + a.xchg_off);
  unsigned* tagp = reinterpret_cast<unsigned*>(cx.base + a.tag_off);
  const unsigned tag0 = *tagp;
  unsigned phase = 0;

  extern __shared__ __align__(16) unsigned char smem[];
  bf16_t* sx = reinterpret_cast<bf16_t*>(smem);               // residual stream of the band, [P][XS]
  bf16_t* smA = sx + (size_t)P * XS;                          // c1 with its halo rows, then relu(bn2(.)): [10*32][MS]
  bf16_t* smB = smA + (size_t)(P + 2 * BAND_W) * MS;          // c2, [P][MS]
  float2* coefC = reinterpret_cast<float2*>(smB + (size_t)P * MS);
  float2* coefM = coefC + C;
  float* red = reinterpret_cast<float*>(coefM + MID);         // RES_NWV * 2*C floats
  float* gath = red + RES_NWV * 2 * C;                        // nwg * 2*C floats
  uint32_t* halo = reinterpret_cast<uint32_t*>(gath + (size_t)nwg * 2 * C);   // 2 * BAND_HALO_F words
  bf16_t* bandA = smA + BAND_W * MS;                          // the band's own rows of the c1 tile
  auto slot = [&]() { return xchg + (size_t)(phase & 1u) * nwg * BAND_RW; };

  WFrags<C / 32, 1, true> w1;     // conv1 [MID][C]
  WFrags<5, 1, true> w2;          // conv2 [MID][160]
  WFrags<1, C / 16, true> w3;     // conv3 [C][32], k >= MID zero

  {
    const ResBlock B0 = a.blocks[0];
    tile_load<C>(sx, cx.tensor(B0.x_off) + (size_t)me * P * C, P);
    w1.load(a.packed + B0.wf_off[0], C, fr, fk);
    __syncthreads();
    band_stats_publish<C>(sx, red, slot() + (size_t)me * BAND_RW, tag0 + 1u + phase);
    if (!band_collect(slot(), nwg, 2 * C, tag0 + 1u + phase, gath, -1, -1, 0, 0, 0, halo, a.abort_flag)) return;
    ++phase;
    band_merge_coef<C>(gath, nwg, a.eps, a.params + B0.gamma_off[0], a.params + B0.beta_off[0], coefC,
                       me == 0 ? reinterpret_cast<float*>(cx.base + B0.stats_off[0]) : nullptr);
  }

  for (int bi = 0; bi < a.nblk; ++bi) {
    const ResBlock B = a.blocks[bi];
    // ---- conv1 (1x1, C -> MID) on relu(bn1(x))
    {
      floatx4 acc[PTW];
#pragma unroll
      for (int j = 0; j < PTW; ++j) acc[j] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < C / 32; ++ks) {
        float2 cf[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) cf[i] = coefC[ks * 32 + fk + i];
        const bf16x8 wf = w1.get(ks, 0);
#pragma unroll
        for (int j = 0; j < PTW; ++j) {
          const int pt = wave + j * RES_NWV;
          const uint4 xv = *reinterpret_cast<const uint4*>(sx + (pt * 16 + fr) * XS + ks * 32 + fk);
          acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, frag_bn_relu(xv, cf), acc[j], 0, 0, 0);
        }
      }
#pragma unroll
      for (int j = 0; j < PTW; ++j)
        *reinterpret_cast<uint2*>(bandA + ((wave + j * RES_NWV) * 16 + fr) * MS + fq * 4) = pack4(acc[j]);
    }
    w2.load(a.packed + B.wf_off[1], 160, fr, fk);
    __syncthreads();
    {
      u64* rec = slot() + (size_t)me * BAND_RW;
      const unsigned tag = tag0 + 1u + phase;
      band_stats_publish<MID>(bandA, red, rec, tag);
      // the band's first and last row of c1 (as stored) for the neighbours: word w = pixel w/8, channels 2*(w%8), +1
      {
        const int w = tid & (BAND_HALO_F - 1), last = tid >> 8;     // RES_NT == 2 * BAND_HALO_F
        const int px = w >> 3, ch = (w & 7) * 2;
        const uint32_t v = *reinterpret_cast<const uint32_t*>(bandA + ((last ? BAND_ROWS - 1 : 0) * BAND_W + px) * MS + ch);
        __hip_atomic_store(rec + 2 * MID + last * BAND_HALO_F + w, ((u64)tag << 32) | (u64)v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      // the row above the band is the last row of the member before, the row below the first row of the member after
      if (!band_collect(slot(), nwg, 2 * MID, tag, gath, up, dn, 2 * MID + BAND_HALO_F, 2 * MID, BAND_HALO_F, halo, a.abort_flag)) return;
      tile_store<MID>(cx.tensor(B.c1_off) + (size_t)me * P * MID, bandA, P);
      ++phase;
      band_merge_coef<MID>(gath, nwg, a.eps, a.params + B.gamma_off[1], a.params + B.beta_off[1], coefM,
                           me == 0 ? reinterpret_cast<float*>(cx.base + B.stats_off[1]) : nullptr);
    }
    // relu(bn2(.)) in place over the band and the two halo rows; a row outside the image is zero AFTER the activation
    {
      const int w = tid & (BAND_HALO_F - 1), below = tid >> 8;
      const int px = w >> 3, ch = (w & 7) * 2;
      *reinterpret_cast<uint32_t*>(smA + ((below ? BAND_ROWS + 1 : 0) * BAND_W + px) * MS + ch) = halo[below * BAND_HALO_F + w];
    }
    __syncthreads();
    for (int u = tid; u < (P + 2 * BAND_W) * 2; u += RES_NT) {
      const int row = u >> 1, col = u & 1;
      const int trow = row / BAND_W;
      uint4* q = reinterpret_cast<uint4*>(smA + row * MS + col * 8);
      const bool outside = (trow == 0 && up < 0) || (trow == BAND_ROWS + 1 && dn < 0);
      const uint4 v = *q;
      const uint32_t wv[4] = {v.x, v.y, v.z, v.w};
      const float4* cf = reinterpret_cast<const float4*>(coefM + col * 8);
      uint32_t r[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float4 k = cf[i];
        r[i] = pack_bf16x2(fmaxf(fmaf(bf_lo(wv[i]), k.x, k.y), 0.f), fmaxf(fmaf(bf_hi(wv[i]), k.z, k.w), 0.f));
      }
      *q = outside ? make_uint4(0u, 0u, 0u, 0u) : make_uint4(r[0], r[1], r[2], r[3]);
    }
    __syncthreads();
    // ---- conv2 (3x3, MID -> MID)
    {
      floatx4 acc[PTW][1];
#pragma unroll
      for (int j = 0; j < PTW; ++j) acc[j][0] = floatx4{0.f, 0.f, 0.f, 0.f};
      band_conv3x3<false>(smA, w2, wave, fr, fq, acc);
#pragma unroll
      for (int j = 0; j < PTW; ++j)
        *reinterpret_cast<uint2*>(smB + ((wave + j * RES_NWV) * 16 + fr) * MS + fq * 4) = pack4(acc[j][0]);
    }
    w3.load(a.packed + B.wf_off[2], 32, fr, fk);
    __syncthreads();
    {
      const unsigned tag = tag0 + 1u + phase;
      band_stats_publish<MID>(smB, red, slot() + (size_t)me * BAND_RW, tag);
      if (!band_collect(slot(), nwg, 2 * MID, tag, gath, -1, -1, 0, 0, 0, halo, a.abort_flag)) return;
      tile_store<MID>(cx.tensor(B.c2_off) + (size_t)me * P * MID, smB, P);
      ++phase;
      band_merge_coef<MID>(gath, nwg, a.eps, a.params + B.gamma_off[2], a.params + B.beta_off[2], coefM,
                           me == 0 ? reinterpret_cast<float*>(cx.base + B.stats_off[2]) : nullptr);
    }
    // ---- conv3 (1x1, MID -> C) on relu(bn3(c2)) + residual, written over x; lane groups 2-3 hold the empty half of the step
    {
      bf16x8 bfrag[PTW];
      float2 cf[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) cf[i] = coefM[(fk + i) & (MID - 1)];
#pragma unroll
      for (int j = 0; j < PTW; ++j) {
        const uint4 cv = *reinterpret_cast<const uint4*>(smB + ((wave + j * RES_NWV) * 16 + fr) * MS + (fk & (MID - 1)));
        bfrag[j] = fq < 2 ? frag_bn_relu(cv, cf) : frag_zero();
      }
#pragma unroll
      for (int nt = 0; nt < C / 16; ++nt) {
#pragma unroll
        for (int j = 0; j < PTW; ++j) {
          floatx4 acc = floatx4{0.f, 0.f, 0.f, 0.f};
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w3.get(0, nt), bfrag[j], acc, 0, 0, 0);
          uint2* q = reinterpret_cast<uint2*>(sx + ((wave + j * RES_NWV) * 16 + fr) * XS + nt * 16 + fq * 4);
          const uint2 xr = *q;
          acc[0] += bf_lo(xr.x); acc[1] += bf_hi(xr.x); acc[2] += bf_lo(xr.y); acc[3] += bf_hi(xr.y);
          *q = pack4(acc);
        }
      }
    }
    const bool more = bi + 1 < a.nblk;
    const ResBlock Bn = a.blocks[more ? bi + 1 : bi];
    if (more) w1.load(a.packed + Bn.wf_off[0], C, fr, fk);
    __syncthreads();
    if (more) band_stats_publish<C>(sx, red, slot() + (size_t)me * BAND_RW, tag0 + 1u + phase);
    tile_store<C>(cx.tensor(B.y_off) + (size_t)me * P * C, sx, P);
    if (more) {
      if (!band_collect(slot(), nwg, 2 * C, tag0 + 1u + phase, gath, -1, -1, 0, 0, 0, halo, a.abort_flag)) return;
      ++phase;
      band_merge_coef<C>(gath, nwg, a.eps, a.params + Bn.gamma_off[0], a.params + Bn.beta_off[0], coefC,
                         me == 0 ? reinterpret_cast<float*>(cx.base + Bn.stats_off[0]) : nullptr);
    }
  }
  if (me == 0 && tid == 0) *tagp = tag0 + phase;
}

// BatchNorm + ReLU backward on a gradient tile in accumulator layout, for a band (cf. bn_relu_bwd_acc): records of
// width BAND_RW, nwg members of BAND_P pixels each, any channel count from 16.  HALO: the band's first and last row
// of dz (fp32, one word per value) travel with the sums, and halo[0 .. BAND_HALO_B) / halo[BAND_HALO_B ..) return
// the last row of the member above / the first row of the member below (zeros where there is none).
// g_beta / g_gamma (member 0 only, else null): the micro-batch sums are added to the parameter gradients.
template <int Cc, bool HALO, class Fin>
__device__ __forceinline__ bool band_bn_relu_bwd_acc(floatx4 (&dz)[BAND_PTW][Cc / 16], const uint2 (&xin)[BAND_PTW][Cc / 16], const float4* cf_,
                                                     int wave, int fr, int fq, float* red, float4* tab_, float* gath, u64* slot, int me,
                                                     int nwg, int up, int dn, uint32_t* halo, unsigned tag, float* g_beta, float* g_gamma,
                                                     int* abort_flag, Fin&& fin) {
  constexpr int NTL = Cc / 16, PTW = BAND_PTW;
  static_assert(!HALO || Cc == 16, "halo rows are 16 channels wide");
  const float4* cf = reinterpret_cast<const float4*>(__builtin_assume_aligned(cf_, 16));
  float4* tab = reinterpret_cast<float4*>(__builtin_assume_aligned(tab_, 16));
  u64* rec = slot + (size_t)me * BAND_RW;
#pragma unroll
  for (int nt = 0; nt < NTL; ++nt) {
    float4 k[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) k[e] = cf[nt * 16 + fq * 4 + e];
    float sb[4] = {0.f, 0.f, 0.f, 0.f}, sg[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < PTW; ++j) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float v = elem4(xin[j][nt], e);
        const float d = fmaf(v, k[e].x, k[e].y) > 0.f ? dz[j][nt][e] : 0.f;
        dz[j][nt][e] = d;
        sb[e] += d;
        sg[e] = fmaf(d, fmaf(v, k[e].z, k[e].w), sg[e]);
      }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) { sb[e] = sum16(sb[e]); sg[e] = sum16(sg[e]); }
    if (fr == 0) {
      *reinterpret_cast<float4*>(red + wave * 2 * Cc + nt * 16 + fq * 4) = make_float4(sb[0], sb[1], sb[2], sb[3]);
      *reinterpret_cast<float4*>(red + wave * 2 * Cc + Cc + nt * 16 + fq * 4) = make_float4(sg[0], sg[1], sg[2], sg[3]);
    }
  }
  if (HALO) {   // pixel tiles 0, 1 are the band's first row, tiles 14, 15 its last: word = pixel*16 + channel
#pragma unroll
    for (int j = 0; j < PTW; ++j) {
      const int pt = wave + j * RES_NWV;
      const bool first = pt < 2, last = pt >= BAND_P / 16 - 2;
      if (first || last) {
        const int px = (first ? pt : pt - (BAND_P / 16 - 2)) * 16 + fr;
        u64* dst = rec + 2 * Cc + (last ? BAND_HALO_B : 0) + px * 16 + fq * 4;
#pragma unroll
        for (int e = 0; e < 4; ++e)
          __hip_atomic_store(dst + e, ((u64)tag << 32) | (u64)__float_as_uint(dz[j][0][e]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
  __syncthreads();
  for (int w = threadIdx.x; w < 2 * Cc; w += RES_NT) {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < RES_NWV; ++i) s += red[i * 2 * Cc + w];
    __hip_atomic_store(rec + w, ((u64)tag << 32) | (u64)__float_as_uint(s), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  if (!band_collect(slot, nwg, 2 * Cc, tag, gath, HALO ? up : -1, HALO ? dn : -1, 2 * Cc + BAND_HALO_B, 2 * Cc, HALO ? BAND_HALO_B : 0, halo,
                    abort_flag))
    return false;
  const float invM = 1.f / ((float)nwg * (float)BAND_P);
  {
    constexpr int CR = Cc >= 32 ? Cc / 32 : 1, MP = 16 / CR, ROWS = Cc / CR;
    const int l16 = threadIdx.x & 15, row = threadIdx.x >> 4;
    const bool act = row < ROWS;
    const int c = act ? row * CR + l16 % CR : 0, part = l16 / CR;
    float sb = 0.f, sg = 0.f;
    for (int m = part; m < nwg; m += MP) { sb += gath[m * 2 * Cc + c]; sg += gath[m * 2 * Cc + Cc + c]; }
    sb = row_sum<CR>(sb);
    sg = row_sum<CR>(sg);
    if (act && part == 0) {
      if (g_beta) { atomicAdd(g_beta + c, sb); atomicAdd(g_gamma + c, sg); }
      const float4 k = cf[c];
      tab[c] = make_float4(k.x, -k.x * sg * invM * k.z, -k.x * invM * (sb + k.w * sg), 0.f);
    }
  }
  __syncthreads();
#pragma unroll
  for (int nt = 0; nt < NTL; ++nt) {
    float4 t[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) t[e] = tab[nt * 16 + fq * 4 + e];
#pragma unroll
    for (int j = 0; j < PTW; ++j) {
      floatx4 out;
#pragma unroll
      for (int e = 0; e < 4; ++e) out[e] = fmaf(t[e].x, dz[j][nt][e], fmaf(t[e].y, elem4(xin[j][nt], e), t[e].z));
      fin(j, nt, out);
    }
  }
  return true;
}

template <int C, int MID>
__global__ void __launch_bounds__(RES_NT) k_band_backward(const ResArgs a) {
  static_assert(C == 64 && MID == 16, "the shape of ResNet-1001's first stage");
  constexpr int XS = C + 8, MS = MID + 8, P = BAND_P, PTW = BAND_PTW;
  const int tid = threadIdx.x, lane = tid & 63, wave = wave_index();
  const int fr = lane & 15, fq = lane >> 4, fk = fq * 8;
  const int nb = a.H / BAND_ROWS, nwg = a.nmem * nb;
  const int z = blockIdx.x % a.ngroup, me = blockIdx.x / a.ngroup;
  const int band = me % nb;
  const int up = band > 0 ? me - 1 : -1, dn = band + 1 < nb ? me + 1 : -1;
  ResCtx cx{(char*)pick(a.base, z), pick(a.act_in, z), pick(a.act_out, z), pick(a.err_in, z), pick(a.err_out, z)};
  u64* xchg = reinterpret_cast<u64*>(cx.base + a.xchg_off);
  unsigned* tagp = reinterpret_cast<unsigned*>(cx.base + a.tag_off);
  const unsigned tag0 = *tagp;
  unsigned phase = 0;

  extern __shared__ __align__(16) unsigned char smem[];
  bf16_t* sdy = reinterpret_cast<bf16_t*>(smem);              // gradient of the residual stream of the band, [P][XS]
  bf16_t* sm2 = sdy + (size_t)P * XS;                         // dc1, [P][MS]
  bf16_t* sdc = sm2 + (size_t)P * MS;                         // dc2 with one halo row above and below, [10*32][MS]
  float4* cf1 = reinterpret_cast<float4*>(sdc + (size_t)(P + 2 * BAND_W) * MS);
  float4* cf2 = cf1 + C;
  float4* cf3 = cf2 + MID;
  float* red = reinterpret_cast<float*>(cf3 + MID);           // RES_NWV * 2*C floats
  float4* tab = reinterpret_cast<float4*>(red + RES_NWV * 2 * C);   // C float4
  float* gath = reinterpret_cast<float*>(tab + C);            // nwg * 2*C floats
  uint32_t* halo = reinterpret_cast<uint32_t*>(gath + (size_t)nwg * 2 * C);   // 2 * BAND_HALO_B words
  bf16_t* bandD = sdc + BAND_W * MS;                          // the band's own rows of the dc2 tile
  auto slot = [&]() { return xchg + (size_t)(phase & 1u) * nwg * BAND_RW; };

  WFrags<C / 32, 1, true> w3;     // conv3 data gradient [MID][C]
  WFrags<5, 1, true> w2;          // conv2 data gradient [MID][160]
  WFrags<1, C / 16, true> w1;     // conv1 data gradient [C][32], k >= MID zero
  {
    const ResBlock BL = a.blocks[a.nblk - 1];
    tile_load<C>(sdy, cx.tensor(BL.gy_off) + (size_t)me * P * C, P);
  }
  __syncthreads();
  for (int bi = a.nblk - 1; bi >= 0; --bi) {
    const ResBlock B = a.blocks[bi];
    float* const g_b[3] = {me == 0 ? a.grads + B.beta_off[0] : nullptr, me == 0 ? a.grads + B.beta_off[1] : nullptr,
                           me == 0 ? a.grads + B.beta_off[2] : nullptr};
    float* const g_g[3] = {a.grads + B.gamma_off[0], a.grads + B.gamma_off[1], a.grads + B.gamma_off[2]};
    uint2 xc1[PTW][1], xc2[PTW][1];   // c1 / c2 at this lane's accumulator positions
    // ---- conv3 data gradient, then BN3 + ReLU backward -> dc2 (with the neighbours' rows next to the band)
    floatx4 acc3[PTW][1];
    // c2 at the halo positions (two values per thread: word w = row*512 + pixel*16 + channel), asked for up front
    bf16_t hx[2];
    {
      BwdLoads<C, MID, PTW> ld;
      w3.load(a.packed + B.wd_off[2], C, fr, fk);
      ld.issue(B, cx, a.params, me, P, P >> 4, wave, fr, fq);
      const bf16_t* g2 = cx.tensor(B.c2_off) + (size_t)me * P * MID;
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const int w = tid + q * RES_NT, below = w >> 9, px = (w >> 4) & (BAND_W - 1), ch = w & 15;
        const bool have = below ? dn >= 0 : up >= 0;
        const long off = have ? ((long)(below ? P : -BAND_W) + px) * MID + ch : 0;   // the neighbour's row sits right next to the band
        hx[q] = g2[off];
      }
#pragma unroll
      for (int j = 0; j < PTW; ++j) acc3[j][0] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < C / 32; ++ks) {
#pragma unroll
        for (int j = 0; j < PTW; ++j) {
          const bf16x8 bfrag = *reinterpret_cast<const bf16x8*>(sdy + ((wave + j * RES_NWV) * 16 + fr) * XS + ks * 32 + fk);
          acc3[j][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w3.get(ks, 0), bfrag, acc3[j][0], 0, 0, 0);
        }
      }
      ld.commit_tables(cf1, cf2, cf3);
#pragma unroll
      for (int j = 0; j < PTW; ++j) { xc1[j][0] = ld.x1[j][0]; xc2[j][0] = ld.x2[j][0]; }
    }
    __syncthreads();
    w2.load(a.packed + B.wd_off[1], 160, fr, fk);
    if (!band_bn_relu_bwd_acc<MID, true>(acc3, xc2, cf3, wave, fr, fq, red, tab, gath, slot(), me, nwg, up, dn, halo, tag0 + 1u + phase,
                                         g_b[2], g_g[2], a.abort_flag, [&](int j, int, const floatx4& out) {
                                           *reinterpret_cast<uint2*>(bandD + ((wave + j * RES_NWV) * 16 + fr) * MS + fq * 4) = pack4(out);
                                         }))
      return;
    ++phase;
    // the neighbours' rows of dc2: the same map applied to their dz and their c2 (tab is complete: barrier inside)
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const int w = tid + q * RES_NT, below = w >> 9, px = (w >> 4) & (BAND_W - 1), ch = w & 15;
      const bool have = below ? dn >= 0 : up >= 0;
      const float4 t = tab[ch];
      const float v = fmaf(t.x, __uint_as_float(halo[w]), fmaf(t.y, bf16_to_f32(hx[q]), t.z));
      sdc[((below ? BAND_ROWS + 1 : 0) * BAND_W + px) * MS + ch] = have ? f32_to_bf16(v) : (bf16_t)0;
    }
    __syncthreads();
    tile_store<MID>(cx.tensor(B.dc2_off) + (size_t)me * P * MID, bandD, P);
    // ---- conv2 data gradient, BN2 + ReLU backward -> dc1
    uint2 x1[PTW][C / 16];   // the block input at this lane's accumulator positions, for the BN1 backward below
    {
      floatx4 acc[PTW][1];
#pragma unroll
      for (int j = 0; j < PTW; ++j) acc[j][0] = floatx4{0.f, 0.f, 0.f, 0.f};
      {
        const bf16_t* xg = cx.tensor(B.x_off) + (size_t)me * P * C;
#pragma unroll
        for (int j = 0; j < PTW; ++j)
#pragma unroll
          for (int nt = 0; nt < C / 16; ++nt)
            x1[j][nt] = *reinterpret_cast<const uint2*>(xg + (size_t)((wave + j * RES_NWV) * 16 + fr) * C + nt * 16 + fq * 4);
      }
      band_conv3x3<true>(sdc, w2, wave, fr, fq, acc);
      w1.load(a.packed + B.wd_off[0], 32, fr, fk);
      if (!band_bn_relu_bwd_acc<MID, false>(acc, xc1, cf2, wave, fr, fq, red, tab, gath, slot(), me, nwg, -1, -1, halo, tag0 + 1u + phase,
                                            g_b[1], g_g[1], a.abort_flag, [&](int j, int, const floatx4& out) {
                                              *reinterpret_cast<uint2*>(sm2 + ((wave + j * RES_NWV) * 16 + fr) * MS + fq * 4) = pack4(out);
                                            }))
        return;
      ++phase;
    }
    __syncthreads();
    tile_store<MID>(cx.tensor(B.dc1_off) + (size_t)me * P * MID, sm2, P);
    // ---- conv1 data gradient (half-empty step), BN1 + ReLU backward, plus the shortcut: dx = bn1_bwd(...) + dy over dy
    {
      floatx4 acc[PTW][C / 16];
      bf16x8 bfrag[PTW];
#pragma unroll
      for (int j = 0; j < PTW; ++j) {
        const bf16x8 v = *reinterpret_cast<const bf16x8*>(sm2 + ((wave + j * RES_NWV) * 16 + fr) * MS + (fk & (MID - 1)));
        bfrag[j] = fq < 2 ? v : frag_zero();
      }
#pragma unroll
      for (int nt = 0; nt < C / 16; ++nt)
#pragma unroll
        for (int j = 0; j < PTW; ++j)
          acc[j][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w1.get(0, nt), bfrag[j], floatx4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
      if (!band_bn_relu_bwd_acc<C, false>(acc, x1, cf1, wave, fr, fq, red, tab, gath, slot(), me, nwg, -1, -1, halo, tag0 + 1u + phase, g_b[0],
                                          g_g[0], a.abort_flag, [&](int j, int nt, const floatx4& out) {
                                            uint2* q = reinterpret_cast<uint2*>(sdy + ((wave + j * RES_NWV) * 16 + fr) * XS + nt * 16 + fq * 4);
                                            const uint2 d = *q;
                                            floatx4 v = out;
                                            v[0] += bf_lo(d.x); v[1] += bf_hi(d.x); v[2] += bf_lo(d.y); v[3] += bf_hi(d.y);
                                            *q = pack4(v);
                                          }))
        return;
      ++phase;
    }
    __syncthreads();
    tile_store<C>(cx.tensor(B.gx_off) + (size_t)me * P * C, sdy, P);
  }
  if (me == 0 && tid == 0) *tagp = tag0 + phase;
}

size_t bb_lds(int C, int P, int nmem, bool backward, int* own) {
  const size_t tile = (size_t)P * (C + 8) * 2;
  const size_t fixed = backward ? (size_t)2 * C * 16 + (size_t)V1_RED(C) * 4 + (size_t)C * 16
                                : (size_t)C * 8 + (size_t)V1_RED(C) * 4;
  *own = (size_t)nmem * 2 * C * 4 > tile ? 1 : 0;
  return (backward ? 2 : 3) * tile + fixed + (*own ? (size_t)nmem * 2 * C * 4 : 0);
}
size_t v1_lds(int C, int P, int nmem, bool backward, int* own) {
  const size_t tile = (size_t)P * (C + 8) * 2;
  const size_t fixed = backward ? (size_t)2 * C * 16 + (size_t)V1_RED(C) * 4 + (size_t)C * 16 : (size_t)C * 8 + (size_t)V1_RED(C) * 4;
  *own = (size_t)nmem * 2 * C * 4 > tile ? 1 : 0;
  return (backward ? 2 : 3) * tile + fixed + (*own ? (size_t)nmem * 2 * C * 4 : 0);
}
size_t bb_wgrad_lds(int C, int P, int W) {
  return (size_t)3 * C * (P + 2 * W + 8) * 2 + (size_t)C * (P + 8) * 2 + (size_t)C * 8;
}

size_t wgrad_lds(int C, int MID, int P, int W) {
  const size_t one = (size_t)(64 + MID) * (P + 8) * 2 + 64 * 8;
  const size_t three = (size_t)3 * MID * (P + 2 * W + 8) * 2 + (size_t)MID * (P + 8) * 2 + (size_t)MID * 8;
  (void)C;
  return one > three ? one : three;
}

// LDS bytes of the two kernels; *own = 1 when the gather area cannot overlay the small tiles
size_t fwd_lds(int C, int MID, int P, int nmem, int* own) {
  const size_t tiles = (size_t)P * (C + 8) * 2 + 2 * (size_t)P * (MID + 8) * 2;
  const size_t fixed = (size_t)(C + MID) * 8 + (size_t)RES_NWV * 2 * C * 4;
  const size_t one_tile = (size_t)P * (MID + 8) * 2;
  *own = ((size_t)nmem * 2 * C * 4 > 2 * one_tile || (size_t)nmem * 2 * MID * 4 > one_tile) ? 1 : 0;
  return tiles + fixed + (*own ? (size_t)nmem * 2 * C * 4 : 0);
}
// LDS copy of the largest weight matrix of a block (rows padded by 8 elements), for the kernels that stage their weights
size_t wl_bytes(int C, int MID) {
  const size_t m1 = (size_t)MID * (C + 8) * 2, m2 = (size_t)MID * (9 * MID + 8) * 2, m3 = (size_t)C * (MID + 8) * 2;
  return m1 > m2 ? (m1 > m3 ? m1 : m3) : (m2 > m3 ? m2 : m3);
}
size_t bwd_lds(int C, int MID, int P, int nmem, int* own) {
  const size_t tiles = (size_t)P * (C + 8) * 2 + 2 * (size_t)P * (MID + 8) * 2;
  const size_t fixed = (size_t)(C + 2 * MID) * 16 + (size_t)RES_NWV * 2 * C * 4 + 4 * (size_t)C * 4;
  const size_t one_tile = (size_t)P * (MID + 8) * 2;
  *own = ((size_t)nmem * 2 * C * 4 > 2 * one_tile || (size_t)nmem * 2 * MID * 4 > one_tile) ? 1 : 0;
  return tiles + fixed + (*own ? (size_t)nmem * 2 * C * 4 : 0);
}

constexpr size_t RES_LDS_BYTES = 160 * 1024 - 1024;   // LDS of a gfx950 CU, less room for the kernels' static allocations

// row-band kernels (64-16 blocks at 32x32): tiles, coefficient tables, reduction and gather areas, halo words
size_t band_bwd_lds(int nwg) {
  const int C = 64, MID = 16;
  return (size_t)BAND_P * (C + 8) * 2 + (size_t)(2 * BAND_P + 2 * BAND_W) * (MID + 8) * 2 + (size_t)(C + 2 * MID) * 16 +
         (size_t)RES_NWV * 2 * C * 4 + (size_t)C * 16 + (size_t)nwg * 2 * C * 4 + (size_t)2 * BAND_HALO_B * 4;
}
size_t band_fwd_lds(int nwg) {
  const int C = 64, MID = 16;
  return (size_t)BAND_P * (C + 8) * 2 + (size_t)(2 * BAND_P + 2 * BAND_W) * (MID + 8) * 2 + (size_t)(C + MID) * 8 +
         (size_t)RES_NWV * 2 * C * 4 + (size_t)nwg * 2 * C * 4 + (size_t)2 * BAND_HALO_F * 4;
}

template <class K>
hipError_t launch_res(K kernel, size_t lds, int own, int g, const ResArgs& a, hipStream_t stream) {
  ResArgs b = a;
  b.ngroup = g;
  kernel<<<dim3((unsigned)(a.nmem * g)), RES_NT, lds, stream>>>(b, own);
  return hipGetLastError();
}

}  // namespace

int resident_bands(int kind, int C, int MID, int H, int W) {
  return (kind == 1 && C == 64 && MID == 16 && H == 32 && W == BAND_W && H % BAND_ROWS == 0) ? H / BAND_ROWS : 1;
}

size_t resident_xchg_bytes(int C, int nmem, int bands) {
  if (bands > 1) return 2 * (size_t)nmem * bands * BAND_RW * sizeof(u64);
  return 2 * (size_t)nmem * 2 * C * sizeof(u64);
}

bool resident_shape_ok(int kind, int C, int MID, int H, int W, int nmem) {
  const int P = H * W;
  // whole 32-pixel reduction steps in the weight gradients; image rows that keep 16-byte alignment under a row shift
  // and whose pixel pairs fit the 16-lane rows used for neighbour exchange
  if (H <= 0 || (W != 8 && W != 16 && W != 32) || P % 32) return false;
  if (nmem < 1 || nmem > 1024) return false;
  int own = 0;
  if (const int nb = resident_bands(kind, C, MID, H, W); nb > 1)
    return band_fwd_lds(nmem * nb) <= RES_LDS_BYTES && band_bwd_lds(nmem * nb) <= RES_LDS_BYTES;
  if (kind == 2) {   // post-activation basic blocks: three / two tiles, no weight-gradient launch
    if (!((C == 16 && P == 1024 && W == 32) || (C == 32 && P <= 256) || (C == 64 && P <= 128)) || MID != C) return false;
    return v1_lds(C, P, nmem, false, &own) <= RES_LDS_BYTES && v1_lds(C, P, nmem, true, &own) <= RES_LDS_BYTES &&
           (C == 16 || bb_wgrad_lds(C, P, W) <= RES_LDS_BYTES);
  }
  if (kind == 0) {   // basic blocks: C -> C -> C
    if (!((C == 16 && P == 1024 && W == 32) || (C == 32 && P <= 256) || (C == 64 && P <= 128)) || MID != C) return false;
    return bb_lds(C, P, nmem, false, &own) <= RES_LDS_BYTES && bb_lds(C, P, nmem, true, &own) <= RES_LDS_BYTES &&
           (C == 16 || bb_wgrad_lds(C, P, W) <= RES_LDS_BYTES);
  }
  if (!((C == 128 && (MID == 32 || MID == 64) && P <= 256) || (C == 256 && MID == 64 && P <= 128))) return false;
  return fwd_lds(C, MID, P, nmem, &own) <= RES_LDS_BYTES && bwd_lds(C, MID, P, nmem, &own) <= RES_LDS_BYTES;
}

int resident_max_group(int nmem) {
  int dev = 0, cus = 0;
  if (nmem < 1 || hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
    return 0;
  const int g = cus / nmem;
  return g > MAX_GROUP ? MAX_GROUP : g;
}

hipError_t resident_prepare() {
  const int lds = (int)RES_LDS_BYTES;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_res_forward<128, 32, 2, true>), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_res_forward<256, 64, 1, false>), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_res_backward<128, 32, 2, true>), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_res_backward<256, 64, 1, false>), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  const void* bb[] = {reinterpret_cast<const void*>(k_bb_forward<32, 2, true>),  reinterpret_cast<const void*>(k_bb_forward<64, 1, false>),
                      reinterpret_cast<const void*>(k_bb_backward<32, 2, true>), reinterpret_cast<const void*>(k_bb_backward<64, 1, false>),
                      reinterpret_cast<const void*>(k_bb_forward<32, 2, false, false, true>), reinterpret_cast<const void*>(k_bb_backward<32, 2, false, true>),
                      reinterpret_cast<const void*>(k_bb_forward<16, 8, false, false, true>), reinterpret_cast<const void*>(k_bb_backward<16, 8, false, true>),
                      reinterpret_cast<const void*>(k_bb_wgrad<32>),             reinterpret_cast<const void*>(k_bb_wgrad<64>)};
  for (const void* f : bb)
    if (e == hipSuccess) e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_res_wgrad<128, 32>), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_res_wgrad<256, 64>), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  const void* wide[] = {reinterpret_cast<const void*>(k_res_forward<128, 64, 2, false>), reinterpret_cast<const void*>(k_res_backward<128, 64, 2, false>),
                        reinterpret_cast<const void*>(k_res_wgrad<128, 64>)};
  for (const void* f : wide)
    if (e == hipSuccess) e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  const void* sq[] = {reinterpret_cast<const void*>(k_res_forward<128, 32, 2, true, false, 16>), reinterpret_cast<const void*>(k_res_forward<128, 64, 2, false, false, 16, 2>),
                      reinterpret_cast<const void*>(k_res_backward<128, 32, 2, true, 16>),       reinterpret_cast<const void*>(k_res_backward<128, 64, 2, false, 16, 2>)};
  for (const void* f : sq)
    if (e == hipSuccess) e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_res_forward<128, 32, 2, false, false, 16, 1>), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_res_backward<128, 32, 2, false, 16, 1>), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_res_forward<256, 64, 1, false, false, 0, 1>), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_res_backward<256, 64, 1, false, 0, 1>), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_v1_wgrad<32>), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_v1_wgrad<64>), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  const void* v1[] = {reinterpret_cast<const void*>(k_v1_forward<32, 2, true>),  reinterpret_cast<const void*>(k_v1_forward<64, 1, false>),
                      reinterpret_cast<const void*>(k_v1_backward<32, 2, true>), reinterpret_cast<const void*>(k_v1_backward<64, 1, false>),
                      reinterpret_cast<const void*>(k_v1_forward<16, 8, false>),  reinterpret_cast<const void*>(k_v1_backward<16, 8, false>),
                      reinterpret_cast<const void*>(k_v1_forward<16, 8, false, true>),  reinterpret_cast<const void*>(k_v1_backward<16, 8, false, true>),
                      reinterpret_cast<const void*>(k_v1_forward<32, 2, false, true>),  reinterpret_cast<const void*>(k_v1_backward<32, 2, false, true>),
                      reinterpret_cast<const void*>(k_v1_forward<64, 1, false, true>), reinterpret_cast<const void*>(k_v1_backward<64, 1, false, true>),
                      reinterpret_cast<const void*>(k_bb_forward<64, 1, false, false, true>), reinterpret_cast<const void*>(k_bb_backward<64, 1, false, true>)};
  for (const void* f : v1)
    if (e == hipSuccess) e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_band_forward<64, 16>), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_band_backward<64, 16>), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  const void* infer[] = {reinterpret_cast<const void*>(k_res_forward<128, 32, 2, true, true>), reinterpret_cast<const void*>(k_res_forward<128, 64, 2, false, true>),
                         reinterpret_cast<const void*>(k_res_forward<256, 64, 1, false, true>), reinterpret_cast<const void*>(k_bb_forward<32, 2, true, true>),
                         reinterpret_cast<const void*>(k_bb_forward<16, 8, false, true>),
                         reinterpret_cast<const void*>(k_bb_forward<64, 1, false, true>)};
  for (const void* f : infer)
    if (e == hipSuccess) e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  return e;
}

hipError_t launch_resident_forward(int kind, int g, int C, int MID, const ResArgs& a, hipStream_t stream) {
  if (const int nb = resident_bands(kind, C, MID, a.H, a.W); nb > 1) {   // one work-group per band of 8 image rows
    const int nwg = a.nmem * nb;
    if (!resident_shape_ok(kind, C, MID, a.H, a.W, a.nmem) || a.nblk < 1 || g < 1 || g > resident_max_group(nwg)) return hipErrorInvalidValue;
    ResArgs b = a;
    b.ngroup = g;
    k_band_forward<64, 16><<<dim3((unsigned)(nwg * g)), RES_NT, band_fwd_lds(nwg), stream>>>(b);
    return hipGetLastError();
  }
  if (!resident_shape_ok(kind, C, MID, a.H, a.W, a.nmem) || a.nblk < 1 || g < 1 || g > resident_max_group(a.nmem)) return hipErrorInvalidValue;
  int own = 0;
  if (kind == 2) {
    const size_t lds = v1_lds(C, a.H * a.W, a.nmem, false, &own);
    const size_t wl16 = (size_t)16 * (160 + 8) * 2;   // the [16][160] matrices through LDS: five L2 round trips per convolution less
    if (C == 16) return lds + wl16 <= RES_LDS_BYTES ? launch_res(k_v1_forward<16, 8, false, true>, lds + wl16, own, g, a, stream)
                                                    : launch_res(k_v1_forward<16, 8, false>, lds, own, g, a, stream);
    if (C == 32) {
      const size_t wl32 = (size_t)32 * (288 + 8) * 2;
      return lds + wl32 <= RES_LDS_BYTES ? launch_res(k_v1_forward<32, 2, false, true>, lds + wl32, own, g, a, stream)
                                         : launch_res(k_v1_forward<32, 2, true>, lds, own, g, a, stream);
    }
    const size_t wl = (size_t)C * (9 * C + 8) * 2;   // one pixel tile per wave: the 3x3 matrices through LDS where they fit
    if (lds + wl <= RES_LDS_BYTES) return launch_res(k_v1_forward<64, 1, false, true>, lds + wl, own, g, a, stream);
    return launch_res(k_v1_forward<64, 1, false>, lds, own, g, a, stream);
  }
  if (kind == 0) {
    const size_t lds = bb_lds(C, a.H * a.W, a.nmem, false, &own);
    if (C == 16) {   // 32x32 images; the [16][160] matrices through LDS
      const size_t wl16 = (size_t)16 * (160 + 8) * 2;
      if (lds + wl16 > RES_LDS_BYTES) return hipErrorInvalidValue;
      return launch_res(k_bb_forward<16, 8, false, false, true>, lds + wl16, own, g, a, stream);
    }
    if (C == 32) {
      const size_t wl32 = (size_t)32 * (288 + 8) * 2;
      return lds + wl32 <= RES_LDS_BYTES ? launch_res(k_bb_forward<32, 2, false, false, true>, lds + wl32, own, g, a, stream)
                                         : launch_res(k_bb_forward<32, 2, true>, lds, own, g, a, stream);
    }
    const size_t wl = (size_t)C * (9 * C + 8) * 2;
    if (lds + wl <= RES_LDS_BYTES) return launch_res(k_bb_forward<64, 1, false, false, true>, lds + wl, own, g, a, stream);
    return launch_res(k_bb_forward<64, 1, false>, lds, own, g, a, stream);
  }
  const size_t lds = fwd_lds(C, MID, a.H * a.W, a.nmem, &own);
  const bool sq16 = a.H == 16 && a.W == 16;
  if (C == 128 && MID == 64)
    return sq16 ? launch_res(k_res_forward<128, 64, 2, false, false, 16, 2>, lds, own, g, a, stream)   // weights through the idle tiles
                : launch_res(k_res_forward<128, 64, 2, false>, lds, own, g, a, stream);
  if (C == 128)
    return sq16 ? (lds + wl_bytes(C, MID) <= RES_LDS_BYTES
                       ? launch_res(k_res_forward<128, 32, 2, false, false, 16, 1>, lds + wl_bytes(C, MID), own, g, a, stream)
                       : launch_res(k_res_forward<128, 32, 2, true, false, 16>, lds, own, g, a, stream))
                : launch_res(k_res_forward<128, 32, 2, true>, lds, own, g, a, stream);
  // one pixel tile per wave: the weights through LDS where the tiles leave room for them (8x8 images)
  if (lds + wl_bytes(C, MID) <= RES_LDS_BYTES)
    return launch_res(k_res_forward<256, 64, 1, false, false, 0, 1>, lds + wl_bytes(C, MID), own, g, a, stream);
  return launch_res(k_res_forward<256, 64, 1, false>, lds, own, g, a, stream);
}

// Inference forward of a run: the images are independent (no exchange), so any number of work-groups may queue.
hipError_t launch_resident_inference(int kind, int g, int C, int MID, const ResArgs& a, hipStream_t stream) {
  if (resident_bands(kind, C, MID, a.H, a.W) > 1) return hipErrorInvalidValue;   // bands: forward and backward launches only
  if (kind == 2) return hipErrorInvalidValue;   // post-activation runs: forward and backward launches only
  if (!resident_shape_ok(kind, C, MID, a.H, a.W, a.nmem) || a.nblk < 1 || g < 1 || g > MAX_GROUP || !a.running) return hipErrorInvalidValue;
  int own = 0;
  if (kind == 0) {
    const size_t lds = bb_lds(C, a.H * a.W, a.nmem, false, &own);
    if (C == 16) return launch_res(k_bb_forward<16, 8, false, true>, lds, 0, g, a, stream);
    if (C == 32) return launch_res(k_bb_forward<32, 2, true, true>, lds, 0, g, a, stream);
    return launch_res(k_bb_forward<64, 1, false, true>, lds, 0, g, a, stream);
  }
  const size_t lds = fwd_lds(C, MID, a.H * a.W, a.nmem, &own);
  if (C == 128 && MID == 64) return launch_res(k_res_forward<128, 64, 2, false, true>, lds, 0, g, a, stream);
  if (C == 128) return launch_res(k_res_forward<128, 32, 2, true, true>, lds, 0, g, a, stream);
  return launch_res(k_res_forward<256, 64, 1, false, true>, lds, 0, g, a, stream);
}

hipError_t launch_resident_wgrad(int kind, int g, int C, int MID, const ResArgs& a, hipStream_t stream) {
  if (resident_bands(kind, C, MID, a.H, a.W) > 1) return hipErrorInvalidValue;   // bands: forward and backward launches only
  if (!resident_has_wgrad_launch(kind, C, 1)) return hipErrorInvalidValue;
  if (!resident_shape_ok(kind, C, MID, a.H, a.W, a.nmem) || a.nblk < 1 || g < 1 || g > MAX_GROUP) return hipErrorInvalidValue;
  ResWgArgs w{};
  w.blocks = a.blocks; w.nmem = a.nmem; w.H = a.H; w.W = a.W;
  w.ipw = 1;
  for (int k = 8; k >= 1; k >>= 1)
    if (a.nmem % k == 0) { w.ipw = k; break; }
  w.base = a.base; w.act_in = a.act_in; w.err_in = a.err_in; w.params = a.params; w.grads = a.grads;
  w.ngroup = g;
  const unsigned groups = (unsigned)(g * a.nmem / w.ipw);
  if (kind == 0 || kind == 2) {
    const size_t lds = bb_wgrad_lds(C, a.H * a.W, a.W);
    const dim3 grid(groups, 2u, (unsigned)a.nblk);
    if (kind == 2) {
      if (C == 32) k_v1_wgrad<32><<<grid, rw_threads(32), lds, stream>>>(w);
      else k_v1_wgrad<64><<<grid, rw_threads(64), lds, stream>>>(w);
    } else if (C == 32) k_bb_wgrad<32><<<grid, rw_threads(32), lds, stream>>>(w);
    else k_bb_wgrad<64><<<grid, rw_threads(64), lds, stream>>>(w);
    return hipGetLastError();
  }
  const size_t lds = wgrad_lds(C, MID, a.H * a.W, a.W);
  const dim3 grid(groups, (unsigned)(2 * (C / 64) + 1), (unsigned)a.nblk);
  if (C == 128 && MID == 64) k_res_wgrad<128, 64><<<grid, rw_threads(64), lds, stream>>>(w);
  else if (C == 128) k_res_wgrad<128, 32><<<grid, rw_threads(32), lds, stream>>>(w);
  else k_res_wgrad<256, 64><<<grid, rw_threads(64), lds, stream>>>(w);
  return hipGetLastError();
}

hipError_t launch_resident_backward(int kind, int g, int C, int MID, const ResArgs& a, hipStream_t stream) {
  if (const int nb = resident_bands(kind, C, MID, a.H, a.W); nb > 1) {
    const int nwg = a.nmem * nb;
    if (!resident_shape_ok(kind, C, MID, a.H, a.W, a.nmem) || a.nblk < 1 || g < 1 || g > resident_max_group(nwg)) return hipErrorInvalidValue;
    ResArgs b = a;
    b.ngroup = g;
    k_band_backward<64, 16><<<dim3((unsigned)(nwg * g)), RES_NT, band_bwd_lds(nwg), stream>>>(b);
    return hipGetLastError();
  }
  if (!resident_shape_ok(kind, C, MID, a.H, a.W, a.nmem) || a.nblk < 1 || g < 1 || g > resident_max_group(a.nmem)) return hipErrorInvalidValue;
  int own = 0;
  if (kind == 2) {
    const size_t lds = v1_lds(C, a.H * a.W, a.nmem, true, &own);
    const size_t wl16 = (size_t)16 * (160 + 8) * 2;
    if (C == 16) return lds + wl16 <= RES_LDS_BYTES ? launch_res(k_v1_backward<16, 8, false, true>, lds + wl16, own, g, a, stream)
                                                    : launch_res(k_v1_backward<16, 8, false>, lds, own, g, a, stream);
    if (C == 32) {
      const size_t wl32 = (size_t)32 * (288 + 8) * 2;
      return lds + wl32 <= RES_LDS_BYTES ? launch_res(k_v1_backward<32, 2, false, true>, lds + wl32, own, g, a, stream)
                                         : launch_res(k_v1_backward<32, 2, true>, lds, own, g, a, stream);
    }
    const size_t wl = (size_t)C * (9 * C + 8) * 2;
    if (lds + wl <= RES_LDS_BYTES) return launch_res(k_v1_backward<64, 1, false, true>, lds + wl, own, g, a, stream);
    return launch_res(k_v1_backward<64, 1, false>, lds, own, g, a, stream);
  }
  if (kind == 0) {
    const size_t lds = bb_lds(C, a.H * a.W, a.nmem, true, &own);
    if (C == 16) {
      const size_t wl16 = (size_t)16 * (160 + 8) * 2;
      if (lds + wl16 > RES_LDS_BYTES) return hipErrorInvalidValue;
      return launch_res(k_bb_backward<16, 8, false, true>, lds + wl16, own, g, a, stream);
    }
    if (C == 32) {
      const size_t wl32 = (size_t)32 * (288 + 8) * 2;
      return lds + wl32 <= RES_LDS_BYTES ? launch_res(k_bb_backward<32, 2, false, true>, lds + wl32, own, g, a, stream)
                                         : launch_res(k_bb_backward<32, 2, true>, lds, own, g, a, stream);
    }
    const size_t wl = (size_t)C * (9 * C + 8) * 2;
    if (lds + wl <= RES_LDS_BYTES) return launch_res(k_bb_backward<64, 1, false, true>, lds + wl, own, g, a, stream);
    return launch_res(k_bb_backward<64, 1, false>, lds, own, g, a, stream);
  }
  const size_t lds = bwd_lds(C, MID, a.H * a.W, a.nmem, &own);
  const bool sq16 = a.H == 16 && a.W == 16;
  if (C == 128 && MID == 64)
    return sq16 ? launch_res(k_res_backward<128, 64, 2, false, 16, 2>, lds, own, g, a, stream)
                : launch_res(k_res_backward<128, 64, 2, false>, lds, own, g, a, stream);
  if (C == 128)
    return sq16 ? (lds + wl_bytes(C, MID) <= RES_LDS_BYTES
                       ? launch_res(k_res_backward<128, 32, 2, false, 16, 1>, lds + wl_bytes(C, MID), own, g, a, stream)
                       : launch_res(k_res_backward<128, 32, 2, true, 16>, lds, own, g, a, stream))
                : launch_res(k_res_backward<128, 32, 2, true>, lds, own, g, a, stream);
  if (lds + wl_bytes(C, MID) <= RES_LDS_BYTES)
    return launch_res(k_res_backward<256, 64, 1, false, 0, 1>, lds + wl_bytes(C, MID), own, g, a, stream);
  return launch_res(k_res_backward<256, 64, 1, false>, lds, own, g, a, stream);
}

}  // namespace hpf
