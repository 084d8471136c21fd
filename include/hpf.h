/*
 * hpf.h -- C ABI of the MI355X partition engine.
 *
 * One handle = one contiguous model partition of a pre-activation ResNet in HyPar-Flow-style
 * model/hybrid-parallel training, at one GPU's share of the work.  Per batch the caller runs, for
 * every micro-batch ("pipeline stage", paper Section "Exploiting Pipeline Stages within Each
 * Minibatch"), one forward call that consumes the activations the previous partition would send
 * and produces those for the next partition (paper Section "Realizing Inter-Partition/-Replica
 * Comm.", basic design: send/recv of partial predictions), and one backward call that consumes
 * the partial error the next partition would send and produces the partial error for the previous
 * partition (the "grad layer" result of Section "Implementing Distributed Back-Propagation",
 * Eq. 5-7).  Weight gradients of all micro-batches are summed into one fp32 buffer -- the buffer
 * the per-partition allreduce of the hybrid design would consume -- and applied once per batch
 * (synchronous update, Section "Background"; optimizer.apply_gradients, Eq. 5-7 section).
 *
 * Conventions
 *  - All pointers marked (dev) are raw device addresses on the current HIP device; (host) are
 *    host addresses.  Streams are hipStream_t passed as void* (NULL = the default stream).
 *  - The caller owns every device buffer, including the arena from which the library carves its
 *    parameters, gradients, momentum, stashed activations and scratch.  The library calls no
 *    hipMalloc.  The library owns only the host-side handle.
 *  - Activations are NHWC.  Convolution weights are [R][S][Cin][Cout] fp32 in the flat parameter
 *    vector.  Canonical flat parameter / gradient order: stem W; per block bn1.gamma, bn1.beta,
 *    W1, bn2.gamma, bn2.beta, W2, [bn3.gamma, bn3.beta, W3], [Wproj]; head bn.gamma, bn.beta,
 *    Wfc [C][classes], bfc.
 *  - forward / backward / grad_accum_zero / sgd_step only enqueue work and return; ordering
 *    between calls issued on different streams (micro-batches may each use their own stream) is
 *    handled inside the library with events (two calls on one and the same stream rely on the
 *    stream's own order).  A stream handed to a call must stay alive until the work of the batch
 *    it took part in has completed.  grad_accum_read to host memory blocks until done.
 *  - Every call returns a status; nothing throws or aborts.  A call that returns HPF_EINVAL,
 *    HPF_ESTATE or HPF_EUNSUPPORTED has had no effect.  hpf_last_error() gives a message.
 *  - Call order per batch (else HPF_ESTATE): forward(mb) once, then backward(mb) once, for every
 *    mb in [0, num_microbatches) in any interleaving; then grad_accum_read any number of times;
 *    then sgd_step (applies and clears the gradients) or grad_accum_zero (clears them) starts the
 *    next batch.
 *  - A handle is not thread-safe; use one host thread per handle.
 */
#ifndef HPF_H
#define HPF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HPF_ABI_VERSION 2u

typedef struct hpf_partition hpf_partition; /* opaque, owned by the library */

typedef enum {
  HPF_OK = 0,
  HPF_EINVAL = 1,       /* bad argument or descriptor */
  HPF_ESTATE = 2,       /* call order violated */
  HPF_ENOMEM = 3,       /* arena too small */
  HPF_EDEVICE = 4,      /* a HIP call failed */
  HPF_EUNSUPPORTED = 5  /* valid description this build has no kernels for */
} hpf_status;

typedef enum {
  HPF_F32 = 0, /* check mode: fp32 tensors; sums, statistics and ReLU decisions in double */
  HPF_BF16 = 1 /* bf16 tensors and MFMA operands, fp32 accumulation, fp32 statistics/gradients */
} hpf_dtype;

/* One unit of the partition.
 * Pre-activation residual blocks (the ResNets of the benchmark configurations):
 *   kind 0 (basic):      bn-relu-conv3x3(stride) -> bn-relu-conv3x3;            c_mid must equal c_out
 *   kind 1 (bottleneck): bn-relu-conv1x1(stride) -> bn-relu-conv3x3 -> bn-relu-conv1x1
 *   Shortcut: identity if stride == 1 and c_in == c_out, else a 1x1 convolution (same stride) of the
 *   block's first bn-relu output.  3x3 convolutions use symmetric zero padding 1; no conv bias.
 * Units of the paper's two other models (Section "Model-Parallelism on a Single Node": ResNet-110-v1, VGG-16);
 * they cannot be cut inside and, except inside the runs of hpf_partition_set_fusion level 2, run as per-layer
 * launches that keep every intermediate:
 *   kind 2 (post-activation basic block): y = relu(bn2(conv3x3(relu(bn1(conv3x3_stride(x))))) + shortcut), c_mid == c_out;
 *           shortcut = x, or a 1x1 convolution (same stride, no BatchNorm) of x iff stride != 1 or c_in != c_out.
 *           Parameters: W1, bn1.gamma, bn1.beta, W2, bn2.gamma, bn2.beta, [Wproj].
 *   kind 3 (conv unit):  relu(conv3x3(x) + bias), padding 1, stride 1; a 2x2 max-pool of stride 2 follows iff
 *           `stride` == 2 (its gradient goes to the first maximum of a window in row-major order).  Parameters: W, bias.
 *   kind 4 (dense unit): flatten(x) [h*w*c_in, in h, w, c order] * W + bias, relu iff c_mid != 0; the output is
 *           1 x 1 x c_out.  Parameters: W [h*w*c_in][c_out], bias.  stride must be 1.
 *   kind 5 (bn-relu):    relu(bn(x)), c_in == c_out (the stem of ResNet-v1 is has_stem followed by this unit).
 *           Parameters: gamma, beta.
 *   kind 6 (bias-relu):  relu(x + bias), c_in == c_out (VGG's first convolution is has_stem followed by this unit).
 *           Parameters: bias. */
typedef struct {
  int32_t kind;
  int32_t c_in, c_mid, c_out;
  int32_t stride; /* 1 or 2 */
} hpf_block_desc;

typedef struct {
  uint32_t abi_version;           /* HPF_ABI_VERSION */
  int32_t in_h, in_w, in_c;       /* shape of act_in per image */
  int32_t has_stem, stem_c_out;   /* first partition: 3x3 stride-1 conv in_c -> stem_c_out */
  int32_t n_blocks;
  const hpf_block_desc* blocks;   /* (host) n_blocks entries, copied */
  int32_t has_head, num_classes;  /* last partition: 1 = bn-relu, global average pool, FC+bias, softmax-CE;
                                     2 = the same without the bn-relu (ResNet-v1, VGG: parameters Wfc, bfc only) */
  int32_t microbatch;             /* images per micro-batch */
  int32_t num_microbatches;       /* micro-batches per batch */
  int32_t loss_divisor;           /* full batch size B: loss = sum over samples of CE / B */
  hpf_dtype compute_dtype;        /* dtype of interior boundary tensors, stash and conv operands */
  float bn_eps;
  int32_t bn_mode;                /* 0: statistics of the micro-batch; 1: frozen mean 0, variance 1 */
  /* Cuts at layer granularity (paper Section "Special Handling for Non-consecutive Models": a partition is a
   * range of layers, and a skip connection whose ends fall into different partitions is exchanged between those
   * two directly).  The partition holds convolutions [first_block_from_conv, n) of its first block and
   * [0, last_block_to_conv) of its last block; 0 means the whole block.  A BatchNorm+ReLU goes with the
   * convolution it feeds, the projection shortcut with convolution 0, the residual add with the last convolution.
   * first_block_from_conv = j > 0: act_in is the output of convolution j-1 (block-output size, c_mid channels;
   * in_h, in_w, in_c describe it), needs no stem; if the block also ends here, its shortcut value arrives as
   * skip_in.  last_block_to_conv = j > 0 (j < n): act_out is the output of convolution j-1, needs no head; if
   * the block also starts here, its shortcut value (the block input, or its projection) leaves as skip_out.
   * Parameters: those of the layers held, in canonical order. */
  int32_t first_block_from_conv;
  int32_t last_block_to_conv;
} hpf_partition_desc;

typedef struct {
  size_t n_params;       /* floats in the flat parameter / gradient vector */
  size_t arena_bytes;    /* device bytes hpf_partition_create needs (256-byte aligned base) */
  size_t stash_bytes;    /* part of arena_bytes: stashed activations of all micro-batches */
  size_t act_in_elems;   /* elements per micro-batch of act_in / err_out */
  size_t act_out_elems;  /* elements per micro-batch of act_out / err_in (0 if has_head) */
  size_t skip_in_elems;  /* elements per micro-batch of skip_in / skip_err_out (0: none) */
  size_t skip_out_elems; /* elements per micro-batch of skip_out / skip_err_in (0: none) */
  size_t n_bn_running;   /* floats of BatchNorm running statistics (hpf_bn_running_read / _write) */
} hpf_sizes;

/* Validates the description and reports sizes.  No device work. */
hpf_status hpf_partition_sizes(const hpf_partition_desc* desc, hpf_sizes* out);

/* Builds a partition inside `device_arena` (dev, >= arena_bytes, 256-byte aligned).  host_params
 * (host): n_params fp32 values in canonical order, copied.  Gradients and momentum start at zero.
 * Synchronous.  The arena must outlive the handle. */
hpf_status hpf_partition_create(const hpf_partition_desc* desc, void* device_arena, size_t arena_bytes,
                                const float* host_params, hpf_partition** out);

/* Forward of micro-batch mb.
 *  act_in  (dev) [microbatch, in_h, in_w, in_c]; fp32 if has_stem, else compute_dtype.  It is read
 *          again by backward(mb) and must stay valid and unchanged until that call's work is done.
 *  labels  (dev) [microbatch] int32 in [0, num_classes); required iff has_head.
 *  act_out (dev) [microbatch, out_h, out_w, out_c] compute_dtype; required iff !has_head.
 *  loss_accum (dev) one float, atomically incremented by this micro-batch's share of the loss;
 *          required iff has_head. */
hpf_status hpf_forward_microbatch(hpf_partition* p, int32_t mb, const void* act_in, const int32_t* labels,
                                  void* act_out, float* loss_accum, void* hip_stream);

/* Backward of micro-batch mb (after its forward).
 *  err_in  (dev) gradient of the loss w.r.t. act_out, same shape/dtype; required iff !has_head.
 *  err_out (dev) gradient w.r.t. act_in, compute_dtype, shape of act_in; required iff !has_stem,
 *          must be NULL if has_stem (images have no upstream partition).
 * Adds this micro-batch's weight gradients into the fp32 gradient buffer. */
hpf_status hpf_backward_microbatch(hpf_partition* p, int32_t mb, const void* err_in, void* err_out,
                                   void* hip_stream);

/* The same two calls for partitions cut at layer granularity (paper Section "Special Handling for
 * Non-consecutive Models"); they also accept partitions without cuts (all skip arguments NULL).
 *  skip_in      (dev) [microbatch, out_h0, out_w0, c_out0] compute_dtype: shortcut value of the first block,
 *               sent by the partition that holds the block's start; required iff skip_in_elems > 0.
 *  skip_out     (dev) shortcut value of the last block, for the partition that holds the block's end;
 *               required iff skip_out_elems > 0.
 *  skip_err_in  (dev) gradient w.r.t. skip_out, returned by that partition; required iff skip_out_elems > 0.
 *  skip_err_out (dev) gradient w.r.t. skip_in, for the partition that sent it; required iff skip_in_elems > 0.
 * hpf_forward_microbatch / hpf_backward_microbatch and the group calls return HPF_EINVAL for a partition
 * that needs one of these tensors. */
hpf_status hpf_forward_microbatch_cut(hpf_partition* p, int32_t mb, const void* act_in, const void* skip_in,
                                      const int32_t* labels, void* act_out, void* skip_out, float* loss_accum,
                                      void* hip_stream);
hpf_status hpf_backward_microbatch_cut(hpf_partition* p, int32_t mb, const void* err_in, const void* skip_err_in,
                                       void* err_out, void* skip_err_out, void* hip_stream);

/* Several consecutive micro-batches [mb_first, mb_first + count) in one call: the same work as `count`
 * single calls, but every layer is launched once for the whole group (the micro-batch is a grid
 * dimension; BatchNorm statistics stay per micro-batch).  At small spatial sizes one micro-batch neither
 * fills the GPU nor amortises a kernel dispatch, so this is how the micro-batches of a batch that are in
 * flight at the same time should be issued on one GPU; the group size plays the role the paper's
 * number of pipeline stages plays for its granularity/overlap trade-off.  Arrays are (host) arrays of
 * `count` (dev) pointers with the meaning of the single-call arguments (labels / act_out / err_in /
 * err_out arrays may be NULL exactly when the single-call argument would be NULL).  Groups larger than
 * 8 are processed 8 at a time.  Outputs of all members are complete (in stream order) when the call's
 * work is. */
hpf_status hpf_forward_microbatches(hpf_partition* p, int32_t mb_first, int32_t count, const void* const* act_in,
                                   const int32_t* const* labels, void* const* act_out, float* loss_accum,
                                   void* hip_stream);
hpf_status hpf_backward_microbatches(hpf_partition* p, int32_t mb_first, int32_t count, const void* const* err_in,
                                    void* const* err_out, void* hip_stream);

/* Copies the accumulated gradient (n_params floats) to dst after all backward work issued so far.
 * dst_is_device != 0: dst is (dev) and the copy is enqueued on hip_stream; else dst is (host) and
 * the call blocks until the copy is complete.  Needs all micro-batches' backward calls. */
hpf_status hpf_grad_accum_read(hpf_partition* p, float* dst, size_t n_floats, int32_t dst_is_device,
                               void* hip_stream);

/* Clears the gradient buffer and starts the next batch without updating the weights. */
hpf_status hpf_grad_accum_zero(hpf_partition* p, void* hip_stream);

/* v <- momentum*v + G; w <- w - lr*v on the fp32 masters (all parameters, BN and bias included);
 * refreshes the bf16 weight copies; clears G; starts the next batch.  Needs all backward calls. */
hpf_status hpf_sgd_step(hpf_partition* p, float lr, float momentum, void* hip_stream);

/* Forward and backward kernel sequences of a micro-batch are captured into HIP graphs on first use
 * and replayed while the caller passes the same buffers (a call with other pointers re-captures).
 * enable == 0 switches to plain launches; default is enabled.  The default (NULL) stream, a
 * stream that is itself being captured by the caller, and sequences of fewer than 8 launches
 * (cheaper to launch than a graph) always get plain launches. */
hpf_status hpf_partition_set_graphs(hpf_partition* p, int32_t enable);

/* How far bf16 mode fuses the kernel schedule; the arithmetic is the same at every level, summation
 * orders and the points where intermediate gradients are rounded to bf16 differ.
 *   0  every step a kernel of its own (convolution, BatchNorm statistics, normalise + ReLU, ...);
 *   1  BatchNorm reductions (forward statistics, backward dbeta/dgamma sums) in the epilogue of the
 *      convolution that produces the tensor, normalise + ReLU while the consuming convolution and
 *      weight gradient stage their operand;
 *   2  (default) additionally, runs of consecutive blocks of one shape with stride 1 and identity
 *      shortcut -- bottleneck 128->32->32->128 or 128->64->64->128 channels at up to 256 pixels or 256->64->64->256 at
 *      up to 128; basic (two 3x3 convolutions) with 32 channels at up to 256 pixels, 64 at up to
 *      128 or 16 at 32 x 32; post-activation basic (kind 2) of the same three shapes; image width 8, 16 or 32,
 *      pixel count a multiple of 32 -- run
 *      in one launch per direction that keeps each image in the LDS of one CU: one work-group per
 *      image, all of them on the chip together.  Bottleneck 64->16->16->64 at 32 x 32 pixels, whose image
 *      does not fit, runs the same way with each image cut into four bands of eight rows, one work-group
 *      per band (the image rows next to a band travel with the BatchNorm records).  Needs
 *      microbatch (x 4 for banded runs) <= number of CUs; a group call
 *      then processes floor(CUs / that) micro-batches (at most 8) per launch, and launches
 *      of this kind from all streams and partitions of the process are serialised through events
 *      recorded at call time.  A stream that the CALLER is capturing into a graph cannot take part
 *      in that: forward / backward calls on such a stream return HPF_EUNSUPPORTED at level 2 when the
 *      partition has such runs -- set level 1 for partitions whose calls are captured.  If a launch
 *      ever waits in vain for its partner work-groups it gives up after about a second and sets a
 *      flag in the arena that marks the handle's results invalid.  The flag is sticky (it stays set
 *      until the handle is destroyed) and is reported as HPF_EDEVICE by every call that already
 *      blocks -- hpf_grad_accum_read to host memory, hpf_params_read, hpf_bn_running_read,
 *      hpf_partition_profile_read, hpf_stash_read -- and by hpf_partition_check; hpf_sgd_step tests it
 *      on the device and then leaves parameters, momentum and gradients untouched; the calls that
 *      only enqueue work (hpf_grad_accum_read to device memory among them) cannot report it.
 * Not allowed while a micro-batch is between forward and backward (HPF_ESTATE). */
hpf_status hpf_partition_set_fusion(hpf_partition* p, int32_t level);

/* BatchNorm running statistics and inference.  The paper trains the framework's layers and reports test
 * accuracy (Section "Verifying the Correctness of HyPar-Flow"); evaluating a trained partition needs the
 * inference form of BatchNorm, i.e. moving averages of the micro-batch statistics.  Every BatchNorm of the
 * partition keeps a running mean (start 0) and a running variance (start 1) in the arena.
 *
 * hpf_partition_set_bn_momentum: with momentum m < 1 every training forward moves them,
 *   r <- m*r + (1-m)*(mean | biased variance of the micro-batch), once per micro-batch, in micro-batch order
 *   within a group call and in call order between calls (with m < 1 the library chains forward calls issued on
 *   different streams through an event, so they no longer overlap each other; a caller that captures the calls
 *   into a graph of its own must keep them on one stream).
 *   m = 1 (the default) never touches them; bn_mode 1 neither.  [0, 1] else HPF_EINVAL; HPF_ESTATE while a
 *   micro-batch is between forward and backward.
 * hpf_bn_running_read / _write: (host) n_bn_running floats: per BatchNorm in model order mean[C], variance[C].
 *   Synchronise the device.  Variances must be >= 0.
 * hpf_forward_inference: the partition's layers on one micro-batch with every BatchNorm normalising by its
 *   running statistics; nothing is kept for a backward pass, no state of the batch in progress changes.
 *   act_in / skip_in / skip_out as in hpf_forward_microbatch_cut; out (dev): act_out, or with has_head the
 *   logits [microbatch, num_classes] fp32.  Works in the region of micro-batch 0: HPF_ESTATE while any
 *   micro-batch is between forward and backward.
 * hpf_forward_inference_group: the same for `count` micro-batches (1 .. min(num_microbatches, 8)) in one call,
 *   every layer launched once for all of them; arguments are (host) arrays of `count` (dev) pointers, the skip
 *   arrays NULL exactly when the single-call arguments would be.
 *   At fusion level 2 the runs of pre-activation blocks with whole images per work-group go through inference
 *   variants of the same kernels (nothing is exchanged, so these launches are not serialised); banded runs and
 *   runs of kind-2 blocks use the per-layer kernels. */
hpf_status hpf_partition_set_bn_momentum(hpf_partition* p, float momentum);
hpf_status hpf_bn_running_read(hpf_partition* p, float* host_dst, size_t n_floats);
hpf_status hpf_bn_running_write(hpf_partition* p, const float* host_src, size_t n_floats);
hpf_status hpf_forward_inference(hpf_partition* p, const void* act_in, const void* skip_in, void* out, void* skip_out,
                                 void* hip_stream);
hpf_status hpf_forward_inference_group(hpf_partition* p, int32_t count, const void* const* act_in,
                                       const void* const* skip_in, void* const* out, void* const* skip_out,
                                       void* hip_stream);

/* Per-kernel-class timing, measured with HIP events on the stream the kernels are launched on.
 * While enabled the passes run as plain launches (no graph replay) with an event pair around every
 * segment of consecutive launches of one class; the classes are
 *   "resident_forward" / "resident_backward" / "resident_wgrad"
 *                                             one launch each per run of bottleneck blocks and group,
 *   "wgrad_grouped"                           the other deferred weight-gradient launches (one per tile class),
 *   "conv_forward" / "conv_dgrad"             the bf16 MFMA convolution launches outside image-resident runs,
 *   "other_forward" / "other_backward"        every other kernel of the pass.
 * hpf_partition_profile_read waits for the device, adds the finished segments to the totals kept
 * since profiling was enabled, and writes up to `capacity` entries (classes with no launch are
 * skipped); *count receives the number written.  bytes / flops are the algorithmic figures of the
 * class per launch (each stashed tensor read or written once per pass, 2*M*K*N per contraction;
 * 0 where the library keeps no figure). */
typedef struct hpf_profile_entry {
  char name[32];
  int64_t launches;
  double total_ms;
  double bytes_per_launch;
  double flops_per_launch;
} hpf_profile_entry;
hpf_status hpf_partition_set_profiling(hpf_partition* p, int32_t enable);
hpf_status hpf_partition_profile_read(hpf_partition* p, hpf_profile_entry* entries, int32_t capacity, int32_t* count);

/* fp32 master parameters to host_dst (host), canonical order.  Blocks. */
hpf_status hpf_params_read(hpf_partition* p, float* host_dst, size_t n_floats);

/* Waits for all work of the device and reports what only a blocking call can: HPF_EDEVICE if a HIP error is
 * pending or if an image-resident launch of this handle ever gave up waiting (see hpf_partition_set_fusion).  For
 * callers that read the gradients into device memory and never through a blocking call. */
hpf_status hpf_partition_check(hpf_partition* p);

/* Test aid: writes the handle's "results invalid" flag from the host (a plain copy into the arena after a device
 * synchronisation; no kernel runs), so that the error path of the calls above can be tested without making a
 * launch time out.  HPF_EUNSUPPORTED for a partition without image-resident runs (it has no such flag). */
hpf_status hpf_debug_set_invalid(hpf_partition* p, int32_t value);

/* Test and debugging aid: reads one of the tensors that back-propagation keeps per micro-batch (paper Section
 * "Implementing Distributed Back-Propagation": the layer inputs of the forward pass and the partial errors of
 * Eq. 5-7 that the weight gradients are formed from), so that every layer of a deep partition can be checked on
 * its own.  Valid after backward(mb) and before the next batch's forward(mb) overwrites the region.
 *  unit    -1: the stem; 0 .. n_blocks-1: a residual block; n_blocks: the head.
 *  tensor  one of hpf_tensor_id; tensors of compute_dtype are copied as stored (bf16 bits or fp32), HPF_T_STATS*
 *          as 2*C values {mean[C], invstd[C]} of the BatchNorm in front of convolution 0 / 1 / 2 (of the head's
 *          BatchNorm: HPF_T_STATS0), float in bf16 mode and double in the fp32 check mode.
 *          stem: HPF_T_Y (its output), HPF_T_GY (gradient w.r.t. it); head: HPF_T_X (its input), HPF_T_GX
 *          (gradient w.r.t. its input), HPF_T_STATS0.
 *  host_dst / bytes  (host) destination and its exact size (else HPF_EINVAL).  host_dst == NULL asks only for
 *          the size and the place: *bytes_needed (if non-NULL) and *where are set, nothing is copied.
 *  where   receives 0 when the tensor was copied; when the tensor lives in a caller buffer of that micro-batch
 *          nothing is copied and it receives 1: act_in, 2: act_out, 3: err_in, 4: err_out, 5: skip_in,
 *          6: skip_out, 7: skip_err_in, 8: skip_err_out.
 * HPF_EINVAL for a tensor the partition does not keep (a layer it does not hold, an activation that the
 * convolutions recompute instead of storing).  Synchronises the device. */
typedef enum {
  HPF_T_X = 0,    /* block input (BatchNorm-1 input) */
  HPF_T_C1 = 1,   /* output of convolution 0 */
  HPF_T_C2 = 2,   /* output of convolution 1 (bottleneck) */
  HPF_T_Y = 3,    /* block output */
  HPF_T_GY = 4,   /* gradient w.r.t. the block output */
  HPF_T_DC1 = 5,  /* gradient w.r.t. c1 */
  HPF_T_DC2 = 6,  /* gradient w.r.t. c2 */
  HPF_T_GX = 7,   /* gradient w.r.t. the block input */
  HPF_T_STATS0 = 8, HPF_T_STATS1 = 9, HPF_T_STATS2 = 10,
  HPF_T_A0 = 11, HPF_T_A1 = 12, HPF_T_A2 = 13,  /* relu(bn_j(.)) where the partition stores it */
  /* units of kinds 2 ... 6: HPF_T_X, HPF_T_Y, HPF_T_GY, HPF_T_GX for all of them; kind 2 also HPF_T_C1 (first
   * convolution's output), HPF_T_A0 (relu(bn1(c1))), HPF_T_C2, HPF_T_SC (the shortcut value added before the last
   * relu), HPF_T_STATS0 / 1; kind 5 HPF_T_STATS0; kind 3 with a max-pool HPF_T_Y0 (the output before the pool) */
  HPF_T_Y0 = 14, HPF_T_SC = 15
} hpf_tensor_id;
hpf_status hpf_stash_read(hpf_partition* p, int32_t mb, int32_t unit, int32_t tensor, void* host_dst, size_t bytes,
                          size_t* bytes_needed, int32_t* where);

/* Frees the host-side handle (after synchronising the device).  The arena is the caller's. */
void hpf_partition_destroy(hpf_partition* p);

/* ---- Single-kernel entry points ------------------------------------------------------------
 * The kernels the partition schedule is made of, callable one at a time on caller tensors, for
 * kernel-level parity tests and roofline measurements.  All pointers (dev); tensors NHWC of `dtype`
 * (fp32 or bf16 bits); weights and weight gradients fp32 [R][R][Cin][Cout]; statistics fp32.
 * `workspace` (dev, 256-byte aligned) holds packed bf16 weights / reduction partials; its size
 * comes from hpf_op_workspace_bytes.  Work is enqueued on hip_stream.  The bf16 convolutions read
 * packed weight copies kept in the workspace: repack != 0 rebuilds them from w first (this
 * synchronises the stream once); repack == 0 reuses the copies of the previous call with the same w,
 * shape and workspace, and launches the convolution kernel only.  Convolution layers and their
 * gradients: paper Section "Background" (DNN training) and Eq. 5-7. */
size_t hpf_op_workspace_bytes(int32_t cin, int32_t cout, int32_t R);

/* y[b,h/stride,w/stride,cout] = conv(x[b,h,w,cin], w) (+ add, same shape as y, may alias y). */
hpf_status hpf_op_conv_forward(hpf_dtype dtype, const void* x, const float* w, void* y, const void* add,
                               int32_t b, int32_t h, int32_t wd, int32_t cin, int32_t cout, int32_t R,
                               int32_t stride, void* workspace, size_t workspace_bytes, int32_t repack,
                               void* hip_stream);
/* dx[b,h,w,cin] = adjoint of the convolution applied to dy[b,h/stride,w/stride,cout] (+ add). */
hpf_status hpf_op_conv_dgrad(hpf_dtype dtype, const void* dy, const float* w, void* dx, const void* add,
                             int32_t b, int32_t h, int32_t wd, int32_t cin, int32_t cout, int32_t R,
                             int32_t stride, void* workspace, size_t workspace_bytes, int32_t repack,
                             void* hip_stream);
/* dw[R][R][cin][cout] (fp32) += sum over pixels of x (x) dy. */
hpf_status hpf_op_conv_wgrad(hpf_dtype dtype, const void* x, const void* dy, float* dw, int32_t b, int32_t h,
                             int32_t wd, int32_t cin, int32_t cout, int32_t R, int32_t stride, void* hip_stream);
/* stats[2C] = {mean, 1/sqrt(var+eps)} of x[M,C]; a = max(gamma*xhat + beta, 0).  stats holds float
 * values in bf16 mode and double values in the fp32 check mode (which reduces in double). */
hpf_status hpf_op_bn_relu_forward(hpf_dtype dtype, const void* x, const float* gamma, const float* beta,
                                  float eps, void* a, void* stats, int32_t M, int32_t C, void* workspace,
                                  size_t workspace_bytes, void* hip_stream);
/* dgamma[C], dbeta[C] += reductions; dx = BN+ReLU backward of da (+ skip if non-NULL). */
hpf_status hpf_op_bn_relu_backward(hpf_dtype dtype, const void* x, const void* da, const float* gamma,
                                   const float* beta, const void* stats, const void* skip, void* dx,
                                   float* dgamma, float* dbeta, int32_t M, int32_t C, void* workspace,
                                   size_t workspace_bytes, void* hip_stream);

/* hpf_op_bn_relu_forward for callers that cannot allocate device memory or carry a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same results; the reduction
 * partials go to an array built into the library (4 MiB per GPU the library runs on, held until the process
 * ends) instead of a caller workspace, so the call allocates nothing.  Limit: C <= 1024 (else HPF_EUNSUPPORTED).
 * All calls on one GPU share that array: calls that overlap in time on one GPU (different streams or threads)
 * race; calls on one stream, or otherwise ordered, are safe.  Nothing in the array needs clearing between calls. */
hpf_status hpf_op_bn_relu_forward_noalloc(hpf_dtype dtype, const void* x, const float* gamma, const float* beta,
                                          float eps, void* a, void* stats, int32_t M, int32_t C, void* hip_stream);

/* ---- Measurement aids ------------------------------------------------------------------------
 * Not steps of the method: two plain kernels that say what this chip achieves, so that kernel rates can be
 * quoted against a measured ceiling next to the data-sheet one.
 * hpf_probe_copy: dst[0..bytes) = src[0..bytes) (dev, dev; no overlap) with the library's 16-byte grid-stride
 * copy kernel: 2*bytes of HBM traffic per call.
 * hpf_probe_mfma_bf16: `workgroups` work-groups of 4 waves each run `iters` rounds of independent MFMA on
 * registers: 8 x v_mfma_f32_16x16x32_bf16 per round (wide == 0) or 4 x v_mfma_f32_32x32x16_bf16 (wide != 0):
 * flops = workgroups * 4 * iters * 131072 either way.  sink (dev) receives workgroups*256 floats (each
 * lane's sum of its accumulators).  1 <= workgroups <= 65536, 1 <= iters <= 2^20.  Both enqueue on hip_stream. */
hpf_status hpf_probe_copy(void* dst, const void* src, size_t bytes, void* hip_stream);
hpf_status hpf_probe_mfma_bf16(float* sink, int32_t workgroups, int32_t iters, int32_t wide, void* hip_stream);

/* Message for the last non-OK status on this thread (static storage, never NULL). */
const char* hpf_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* HPF_H */
