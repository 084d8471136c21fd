// Internal interface between the host runtime and the HIP kernels of the partition engine.
// Every launcher only enqueues work on `stream` and returns hipGetLastError().
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace hpf {

typedef uint16_t bf16_t;  // raw bfloat16 bits

enum : int { DT_F32 = 0, DT_BF16 = 1 };

// Micro-batches of one batch are independent until the gradient accumulation, and at CIFAR shapes a
// single micro-batch cannot fill 256 CUs nor amortise a kernel dispatch.  Every kernel of the
// forward / backward schedule therefore takes a group of up to MAX_GROUP micro-batches in one launch:
// blockIdx.z selects the member, PtrTab carries one pointer per member for every per-micro-batch
// tensor (stash, statistics, scratch, caller buffers).  Statistics stay per micro-batch.
constexpr int MAX_GROUP = 8;
struct PtrTab {
  void* p[MAX_GROUP];
};
inline PtrTab one_ptr(const void* q) {
  PtrTab t{};
  t.p[0] = const_cast<void*>(q);
  return t;
}
enum : int { CONV_FWD = 0, CONV_DGRAD = 1 };

// Geometry of one gather-GEMM:  out[m, n] = sum_{tap, c} src[row(m, tap), c] * W(tap, c, n).
// The output row space is b x Ho x Wo; the source tensor is b x Hs x Ws x Cs.
//   CONV_FWD  : out = conv output,      src = conv input,   row(m,tap) = (p*stride + r - pad, q*stride + s - pad)
//   CONV_DGRAD: out = input gradient,   src = output grad,  row(m,tap) = ((p + pad - r)/stride, (q + pad - s)/stride)
//               where both quotients must be exact.
struct ConvGeom {
  int b, Ho, Wo, Hs, Ws, Cs, N, R, stride, pad;
  int M;     // b*Ho*Wo
  int Ktot;  // R*R*Cs
  int Kpad;  // Ktot rounded up to 32 (packed bf16 weights are [N][Kpad], zero padded)
};

// Weight gradient of one convolution: dw[tap][c][n] += sum_m a[row(m,tap), c] * dy[m, n],
// a is b x H x W x Cin, dy is b x Ho x Wo x N, row(m,tap) as in CONV_FWD.  Only rows c < c_valid
// are written and dw has c_valid rows per tap (the stem runs on im2col columns padded to Cin).
struct WgradGeom {
  int b, H, W, Cin, Ho, Wo, N, R, stride, pad, M, c_valid;
};

// One convolution's fp32 master and its packed bf16 copies (offsets in elements).
struct PackDesc {
  unsigned long long w_off;   // fp32 master [T][Cin][Cout] in the parameter vector
  unsigned long long wf_off;  // bf16 [Cout][Kf]  k = tap*Cin + c     (forward operand)
  unsigned long long wd_off;  // bf16 [Cin][Kd]   k = tap*Cout + n    (data-gradient operand); ~0 = none
  int T, Cin, Cout, Kf, Kd;
};

// Optional reduction fused into the convolution epilogue (the output tile is still in registers):
//   EPI_STATS : statistics partial records {K, S1, S2, n} of the stored output, one record row per
//               pixel-row tile and channel, for the BatchNorm that consumes this output;
//   EPI_BNBWD : the output is the gradient da w.r.t. a BN+ReLU output: it is masked with the ReLU
//               decision recomputed from the BN input x (dz = da*[z>0], stored instead of da) and the
//               partial sums {sum dz, sum dz*xhat} are written, one row per pixel-row tile.
enum : int { EPI_NONE = 0, EPI_STATS = 1, EPI_BNBWD = 2 };
struct ConvEpi {
  int kind = EPI_NONE;
  PtrTab partials{};        // EPI_STATS: 4 floats, EPI_BNBWD: 2 floats per (tile row, channel)
  PtrTab x{};               // EPI_BNBWD: BN input [M, N] bf16
  PtrTab stats{};           // EPI_BNBWD: {mean(N), invstd(N)} float
  const float* gamma = nullptr;
  const float* beta = nullptr;
  // EPI_NONE without residual operand: room for a reduction split over several work-groups (long reductions
  // into few output tiles): per member a buffer of splitk_floats floats, slab s holds fp32 partial sums [M][N] at s*M*N;
  // 0 floats = none.  Per member, because calls for different micro-batches may overlap on different streams.
  PtrTab splitk_ws{};
  size_t splitk_floats = 0;
};
// Work-groups a bf16 convolution launch of g members splits every reduction over (1 = no split), and the fp32
// workspace that takes per member (conv_splitk * M * N floats).
int conv_splitk(int g, const ConvGeom& geom);
// Optional BatchNorm + ReLU applied to the source tensor while it is staged (forward convolutions):
// the source is the BatchNorm input x and the operand becomes bf16(max(gamma*((x-mean)*invstd)+beta, 0)),
// so the normalised activation is never written to memory.  Padding stays zero.
struct ConvPro {
  int on = 0;
  PtrTab stats{};            // {mean(Cs), invstd(Cs)} float, per member
  const float* gamma = nullptr;
  const float* beta = nullptr;
};
int conv_mfma_tile_rows(int g, const ConvGeom& geom);   // pixel rows per tile the launcher will use
hipError_t conv_prepare();                               // once per device before the first convolution launch
// How often the bf16 convolution kernels stage each element of the source tensor (filter taps x channel tiles);
// 0 for shapes that run on the narrow tiles.
int conv_operand_reuse(int cin, int cout, int R);

// g = number of group members (grid z); tables hold g valid pointers.  `add` tables may be all-null.
hipError_t launch_conv_mfma(int mode, int g, const PtrTab& src, const bf16_t* wpk, const PtrTab& out, const PtrTab& add,
                            const ConvGeom& geom, hipStream_t stream, const ConvEpi& epi = ConvEpi(),
                            const ConvPro& pro = ConvPro());
hipError_t launch_wgrad_mfma(int g, const PtrTab& a, const PtrTab& dy, float* dw, const WgradGeom& geom, hipStream_t stream);

// All weight gradients of a backward pass in one launch per tile class.  An item is one (convolution,
// filter tap, BC x BN output tile, slice of pixel rows); the work-group that takes it loops over the
// group's micro-batches, so one atomic add per output element and item reaches the gradient buffer.
// a / dy live at byte offsets in each member's arena region (dy_off == WGRAD_DY_CALLER: the caller's
// err_in buffer of that member).
constexpr unsigned long long WGRAD_DY_CALLER = ~0ull;
constexpr unsigned long long WGRAD_NO_BN = ~0ull;
struct WgradItem {
  unsigned long long a_off, dy_off, dw_off;   // bytes, bytes, floats; a_off == WGRAD_DY_CALLER: the caller's act_in
  unsigned long long stats_off;               // bytes; != WGRAD_NO_BN: `a` is a BatchNorm input and the operand is
  unsigned long long gamma_off, beta_off;     //   relu(bn(a)) recomputed while staging (floats into the parameters)
  WgradGeom g;
  int tap, c0, n0, m_begin, m_end;
};
// tile_class: 0..8 = (BC index)*3 + (BN index) with sizes {16, 32, 64}; 9 = 128 x 128 (both channel counts
// multiples of 128: each wave owns a 64 x 64 quadrant of the tile over the whole reduction)
// 10 = whole 3x3 convolutions between 16 and 16 channels on 1024-pixel images: an item is a range of whole images
// (m_begin, m_end multiples of 1024; tap, c0, n0 unused) and its work-group forms all nine taps from one staging
constexpr int WGRAD_CLASSES = 11;
constexpr int WGRAD_CLASS_T9 = 10;
int wgrad_tile_class(int cin, int cout);
int wgrad_item_class(const WgradGeom& g);      // WGRAD_CLASS_T9 where it applies, else wgrad_tile_class
int wgrad_t9_lds_bytes(int H, int W);          // dynamic LDS of a class-10 launch for that image shape
void wgrad_tile_dims(int tile_class, int* bc, int* bn);
hipError_t wgrad_prepare();   // once per device before the first grouped launch
hipError_t launch_wgrad_grouped(int tile_class, int g, const WgradItem* items_dev, int n_items, const PtrTab& region_base,
                                const PtrTab& caller_dy, const PtrTab& caller_a, const float* params, float* grads,
                                hipStream_t stream, int lds_bytes = 0);

// ---- image-resident runs of identity blocks (bf16 mode, BatchNorm on micro-batch statistics)
// A run is a sequence of consecutive blocks of one kind and shape (bottleneck or basic) with stride 1 and identity
// shortcut.  One
// work-group owns one image for the whole run: the residual stream of the image stays in LDS from block
// to block, all three convolutions of a block run from LDS, and only what the backward pass and the
// weight gradients read later goes to memory.  The one cross-image dependency, the BatchNorm reductions
// over the micro-batch, is an all-gather of small per-image records between the work-groups of a
// micro-batch, so all of them must be resident on the chip together (checked by the launchers).
// tensor locations outside the micro-batch region: the caller's buffers of the member
constexpr unsigned long long RES_ACT_IN = ~0ull, RES_ACT_OUT = ~1ull, RES_ERR_IN = ~2ull, RES_ERR_OUT = ~3ull;
struct ResBlock {
  // byte offsets into a micro-batch region (or RES_*): block input, conv1 / conv2 outputs, block output
  // (basic blocks have two convolutions: c2 / dc2 and entry 2 of the arrays are unused)
  unsigned long long x_off, c1_off, c2_off, y_off;
  // gradients w.r.t. the block output, c1, c2, and where the gradient w.r.t. the block input goes
  unsigned long long gy_off, dc1_off, dc2_off, gx_off;
  unsigned long long stats_off[3];           // {mean, invstd} floats of the three BatchNorms (bytes)
  unsigned long long wf_off[3], wd_off[3];   // packed bf16 weights (elements)
  unsigned long long w_off[3];               // fp32 masters / gradients [tap][Cin][Cout] (floats)
  unsigned long long gamma_off[3], beta_off[3];   // floats into the parameter / gradient vectors
  // {sum dz (C floats), sum dz*xhat (C floats)} of the three BatchNorms over the micro-batch (bytes into its region):
  // written by the backward launch, added into the gradients of beta and gamma by the weight-gradient launch
  unsigned long long dgb_off[3];
  unsigned long long run_off[3];             // running {mean(C), variance(C)} of the three BatchNorms (floats)
};
struct ResArgs {
  const ResBlock* blocks;   // device table of the run
  int nblk;
  int nmem;                 // images per micro-batch = work-groups per exchange group
  int ngroup;               // micro-batches in the launch (set by the launchers)
  int H, W;
  float eps;
  PtrTab base;              // micro-batch regions of the group members (grid z)
  PtrTab act_in, act_out, err_in, err_out;   // caller buffers per member (null where the pass does not use them)
  const float* params;
  const float* running;     // running BatchNorm statistics (inference launches)
  const bf16_t* packed;
  float* grads;
  unsigned long long xchg_off;   // bytes into the region: exchange words, resident_xchg_bytes()
  unsigned long long tag_off;    // bytes into the region: phase tag counter (one unsigned, starts at 0)
  int* abort_flag;          // set when an exchange timed out (the pass is then invalid)
};
// Shapes this path covers (a property of the shapes alone).
bool resident_shape_ok(int kind, int C, int MID, int H, int W, int nmem);   // kind: 0 basic (MID == C), 1 bottleneck, 2 post-activation basic
// Runs cut into bands and 16-channel runs (kinds 0 and 2) have forward and backward launches only (weight gradients:
// the grouped per-layer launch); banded runs and all runs of kind 2 go through the per-layer kernels at inference.
inline bool resident_has_wgrad_launch(int kind, int C, int bands) { (void)kind; return bands == 1 && C != 16; }
inline bool resident_has_inference_launch(int kind, int bands) { return bands == 1 && kind != 2; }
// Largest number of micro-batches of nmem images one launch may hold on the current device (0: none):
// every work-group takes a CU of its own and all of them must be resident together.
int resident_max_group(int nmem);   // nmem: work-groups per micro-batch (images x bands)
// Runs whose image does not fit one CU's LDS are cut into row bands, one work-group each (64-16-16-64 bottlenecks at
// 32x32: 4 bands of 8 rows): bands per image of the shape, 1 = whole images.  Such runs have a forward and a backward launch;
// their weight gradients go through the grouped per-layer launch and inference through the per-layer kernels.
int resident_bands(int kind, int C, int MID, int H, int W);
size_t resident_xchg_bytes(int C, int nmem, int bands);
hipError_t resident_prepare();   // once per process, outside stream capture: raises the kernels' LDS limits
hipError_t launch_resident_forward(int kind, int g, int C, int MID, const ResArgs& a, hipStream_t stream);
hipError_t launch_resident_backward(int kind, int g, int C, int MID, const ResArgs& a, hipStream_t stream);
// Weight gradients of all blocks of the run (after the backward launch): reads the stash and the gradient
// tensors the backward launch wrote, adds into a.grads.
hipError_t launch_resident_wgrad(int kind, int g, int C, int MID, const ResArgs& a, hipStream_t stream);
// Inference forward of a run (BatchNorm by the running statistics in a.running): only the output of the last block
// is written; no exchange, so there is no limit on the work-groups of a launch (g <= MAX_GROUP micro-batches).
hipError_t launch_resident_inference(int kind, int g, int C, int MID, const ResArgs& a, hipStream_t stream);

hipError_t launch_conv_f32(int mode, int g, const PtrTab& src, const float* w_hwio, const PtrTab& out, const PtrTab& add,
                           const ConvGeom& geom, hipStream_t stream);
hipError_t launch_wgrad_f32(int g, const PtrTab& a, const PtrTab& dy, float* dw, const WgradGeom& geom, hipStream_t stream);

// BatchNorm + ReLU.  All tensors are [M, C] of dtype dt.  stats = [mean(C), invstd(C)], sums =
// [dbeta(C), dgamma(C)] and partials are arrays of the arithmetic type: float for DT_BF16, double for
// DT_F32 (the check mode reduces and takes the ReLU decision in double).  partials holds
// bn_partials_floats(C) floats per member.
size_t bn_partials_floats(int C);
hipError_t launch_bn_stats(int dt, int g, const PtrTab& x, int M, int C, float eps, const PtrTab& stats,
                           const PtrTab& partials, hipStream_t stream);
// Finalize steps alone, for partial records written by a convolution epilogue (nrows record rows).
hipError_t launch_bn_stats_finalize(int g, int M, int C, int nrows, float eps, const PtrTab& partials, const PtrTab& stats,
                                    hipStream_t stream);
hipError_t launch_bn_bwd_finalize(int g, int C, int nrows, const PtrTab& partials, const PtrTab& sums, float* g_gamma,
                                  float* g_beta, hipStream_t stream);
hipError_t launch_bn_apply_relu(int dt, int g, const PtrTab& x, const PtrTab& a, const float* gamma, const float* beta,
                                const PtrTab& stats, int M, int C, hipStream_t stream);
// sums of each micro-batch; also atomically added into g_gamma / g_beta (fp32 gradient buffer).
hipError_t launch_bn_bwd_reduce(int dt, int g, const PtrTab& x, const PtrTab& da, const float* gamma, const float* beta,
                                const PtrTab& stats, int M, int C, const PtrTab& sums, float* g_gamma, float* g_beta,
                                const PtrTab& partials, hipStream_t stream);
// dx = gamma*invstd*(dz - dbeta/M - xhat*dgamma/M) [+ skip]; frozen: dx = gamma*invstd*dz [+ skip].
hipError_t launch_bn_bwd_apply(int dt, int g, const PtrTab& x, const PtrTab& da, const float* gamma, const float* beta,
                               const PtrTab& stats, const PtrTab& sums, const PtrTab& skip, const PtrTab& dx, int M,
                               int C, int frozen, hipStream_t stream);
hipError_t launch_bn_frozen_stats(int dt, int g, const PtrTab& stats, int C, float eps, hipStream_t stream);

// Layers of VGG-16 and of the post-activation ResNet-v1 block; tensors [M, C] (or b x h x w x C) of dtype dt, C % 8 == 0.
// y = x + bias[c], then max(., 0) when relu.
hipError_t launch_bias_act_fwd(int dt, int g, const PtrTab& x, const PtrTab& y, const float* bias, int M, int C, int relu,
                               hipStream_t stream);
// dx = dy * [y > 0] (relu) or dy; g_bias[c] += sum of dx over the rows.  sums / partials: scratch as for the BatchNorm backward.
hipError_t launch_bias_act_bwd(int dt, int g, const PtrTab& y, const PtrTab& dy, const PtrTab& dx, float* g_bias, int M, int C,
                               int relu, const PtrTab& sums, const PtrTab& partials, hipStream_t stream);
// 2x2 max-pool of stride 2 (h, w even) and its backward pass (gradient to the first maximum in row-major order).
hipError_t launch_maxpool2_fwd(int dt, int g, const PtrTab& x, const PtrTab& y, int b, int h, int w, int C, hipStream_t stream);
hipError_t launch_maxpool2_bwd(int dt, int g, const PtrTab& x, const PtrTab& dy, const PtrTab& dx, int b, int h, int w, int C,
                               hipStream_t stream);
// Residual join of a post-activation block, y = max(bn(x) + add, 0) (statistics given), and its backward pass:
// dz = dy * [y > 0]; dadd = dz; dx through the BatchNorm; dgamma / dbeta added into g_gamma / g_beta.
hipError_t launch_bn_add_relu_apply(int dt, int g, const PtrTab& x, const PtrTab& add, const PtrTab& y, const float* gamma,
                                    const float* beta, const PtrTab& stats, int M, int C, hipStream_t stream);
hipError_t launch_join_bwd(int dt, int g, const PtrTab& x, const PtrTab& y, const PtrTab& dy, const float* gamma, const PtrTab& stats,
                           int M, int C, const PtrTab& sums, float* g_gamma, float* g_beta, const PtrTab& partials, const PtrTab& dx,
                           const PtrTab& dadd, int frozen, hipStream_t stream);
// Running statistics (fp32): per BatchNorm mean[C] then variance[C] at run_off floats into `running`.
struct BnRunDesc { unsigned long long stats_off; int C; int run_off; };   // stats_off: bytes into a member's region
// After a training forward: for the group's members in order, r <- momentum*r + (1-momentum)*{mean, 1/invstd^2 - eps}.
hipError_t launch_bn_running_update(int dt, int g, const PtrTab& bases, const BnRunDesc* table_dev, int n_bn, float* running,
                                    float momentum, float eps, hipStream_t stream);
// Inference: stats = {running mean, 1/sqrt(running variance + eps)}.
hipError_t launch_bn_running_stats(int dt, int g, const PtrTab& stats, const float* running_mean_var, int C, float eps,
                                   hipStream_t stream);

// Stem: fp32 image [b,H,W,Cin] -> bf16 im2col columns [b*H*W, Kc], k = (r*3+s)*Cin + c, zero padded.
hipError_t launch_im2col3x3(int g, const PtrTab& img, const PtrTab& col, int b, int H, int W, int Cin, int Kc,
                            hipStream_t stream);

// Head: a [b,hw,C] (dtype dt) -> g [b,C] fp32, dlogits [b,classes] fp32, loss_accum += sum CE / divisor.
// Inference head: logits[b, classes] (fp32) = mean_{h,w}(a) * Wfc + bfc.
hipError_t launch_head_logits(int dt, int g, const PtrTab& a, const float* wfc, const float* bfc, const PtrTab& logits, int b,
                              int hw, int C, int classes, hipStream_t stream);
hipError_t launch_head_fwd(int dt, int g, const PtrTab& a, const float* wfc, const float* bfc, const PtrTab& labels,
                           const PtrTab& gp, const PtrTab& dlogits, float* loss_accum, int b, int hw, int C,
                           int classes, float divisor, hipStream_t stream);
hipError_t launch_head_bwd(int dt, int g, const PtrTab& gp, const PtrTab& dlogits, const float* wfc, float* g_wfc,
                           float* g_bfc, const PtrTab& da, int b, int hw, int C, int classes, hipStream_t stream);

// invalid (device, may be null): when it reads non-zero the step changes nothing
hipError_t launch_sgd(float* w, float* v, float* g, size_t n, float lr, float mu, const int* invalid, hipStream_t stream);
hipError_t launch_zero_f32(float* p, size_t n, hipStream_t stream);
// max_elems: elements of the largest convolution's forward copy (sizes the grid)
hipError_t launch_pack_weights(const float* params, bf16_t* packed, const PackDesc* table_dev, int n_convs, size_t max_elems,
                               hipStream_t stream);
hipError_t launch_copy_bytes(void* dst, const void* src, size_t bytes, hipStream_t stream);
// iters rounds of 131 072 flop of bf16 MFMA per wave (8 x 16x16x32, or 4 x 32x32x16 when wide), 4 waves per
// work-group; sink: workgroups*256 floats
hipError_t launch_probe_mfma_bf16(float* sink, int workgroups, int iters, bool wide, hipStream_t stream);

}  // namespace hpf
