// Host runtime of the partition engine: description validation, arena layout, the per-micro-batch
// kernel schedule of one partition's forward and backward pass, the call-order state machine and
// the C ABI of include/hpf.h.
//
// What runs per micro-batch (paper Sections "Implementing Distributed Back-Propagation" and
// "Exploiting Pipeline Stages within Each Minibatch"): forward over the partition's units on the
// received activations, stashing what the backward pass needs; backward from the received partial
// error, adding weight gradients into the shared fp32 buffer and emitting the partial error for
// the previous partition.  Units: [stem conv] + pre-activation residual blocks + [head].
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/hpf.h"
#include "hpf_kernels.h"

using namespace hpf;

namespace {

thread_local char g_err[512] = "";

hpf_status fail(hpf_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}

constexpr size_t ALIGN = 256;
size_t align_up(size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }
int round_up32(int v) { return (v + 31) / 32 * 32; }

// Where a tensor lives: inside this micro-batch's arena region, or in a caller buffer.
enum LocKind { IN_MB = 0, CALLER_ACT_IN, CALLER_ACT_OUT, CALLER_ERR_IN, CALLER_ERR_OUT,
               CALLER_SKIP_IN, CALLER_SKIP_OUT, CALLER_SKIP_ERR_IN, CALLER_SKIP_ERR_OUT, NOWHERE };
struct Loc { LocKind kind = NOWHERE; size_t off = 0; };

struct ConvPlan {
  int cin = 0, cout = 0, R = 1, stride = 1, h_in = 0, w_in = 0, h_out = 0, w_out = 0;
  size_t w_off = 0;                 // fp32 master / gradient offset (floats)
  size_t wf_off = 0, wd_off = 0;    // packed bf16 offsets (elements)
  int Kf = 0, Kd = 0;
};

// implicit-GEMM geometry of a convolution of the plan, per micro-batch of b images
ConvGeom conv_geom_fwd(const ConvPlan& cv, int b) {
  ConvGeom q{};
  q.b = b; q.Ho = cv.h_out; q.Wo = cv.w_out; q.Hs = cv.h_in; q.Ws = cv.w_in; q.Cs = cv.cin; q.N = cv.cout;
  q.R = cv.R; q.stride = cv.stride; q.pad = (cv.R - 1) / 2; q.M = q.b * q.Ho * q.Wo; q.Ktot = cv.R * cv.R * cv.cin; q.Kpad = cv.Kf;
  return q;
}
ConvGeom conv_geom_dgrad(const ConvPlan& cv, int b) {
  ConvGeom q{};
  q.b = b; q.Ho = cv.h_in; q.Wo = cv.w_in; q.Hs = cv.h_out; q.Ws = cv.w_out; q.Cs = cv.cout; q.N = cv.cin;
  q.R = cv.R; q.stride = cv.stride; q.pad = (cv.R - 1) / 2; q.M = q.b * q.Ho * q.Wo; q.Ktot = cv.R * cv.R * cv.cout; q.Kpad = cv.Kd;
  return q;
}
struct BnPlan { int C = 0; size_t g_off = 0, b_off = 0; size_t stats_off = 0; /* bytes in mb region */ size_t run_off = 0; /* floats: running mean, then variance */ };
struct BlockPlan {
  hpf_block_desc d{};
  int h_in = 0, w_in = 0, h_out = 0, w_out = 0, nconv = 0;
  bool proj = false;
  int j0 = 0, j1 = 0;   // the partition holds convolutions [j0, j1) of the block (cuts at layer granularity)
  bool whole() const { return j0 == 0 && j1 == nconv; }
  BnPlan bn[3]; ConvPlan cv[3]; ConvPlan pj;
  Loc x_in, a[3], c[2], y;
  bool mat[3] = {false, false, false};   // bf16 mode: a[j] = relu(bn_j(.)) is written to memory (else applied while staging)
  Loc gy;      // gradient w.r.t. the block output (kept until the deferred weight-gradient pass)
  Loc dc[3];   // gradient w.r.t. c[j], the output of conv j (j < nconv-1); units of the other models (bf16 mode): the
               // gradient operand of the unit's convolution j (2: the projection), kept for the deferred weight gradients
  // units of the other models (kinds HPF_POSTACT ... HPF_BIAS_RELU)
  size_t bias_off = 0;   // floats: the unit's bias vector
  Loc y0;                // conv + bias + relu output before the max-pool (== y without a pool)
  Loc sc;                // post-activation block: the projected shortcut (== x_in for an identity shortcut)
  bool copy_out = false; // the unit is the partition's last and its backward pass reads y: y stays in the arena and a
                         // copy goes to the caller's act_out (a backward call is not handed the forward's act_out)
  bool residual() const { return d.kind == 0 || d.kind == 1; }
};
enum : int { K_POSTACT = 2, K_CONV_RELU = 3, K_DENSE = 4, K_BN_RELU = 5, K_BIAS_RELU = 6 };

struct Plan {
  hpf_partition_desc d{};
  std::vector<hpf_block_desc> blocks;
  int dt = DT_BF16; size_t esz = 2;
  size_t n_params = 0;
  // stem
  ConvPlan stem; int stem_kc = 0; Loc stem_col, stem_out;
  std::vector<BlockPlan> bp;
  // head
  BnPlan head_bn; size_t wfc_off = 0, bfc_off = 0; Loc head_x, head_a, head_g, head_dl;
  int out_h = 0, out_w = 0, out_c = 0;
  // per-micro-batch region
  size_t mb_bytes = 0, stash_bytes_per_mb = 0;
  size_t sums_off = 0, partials_off = 0, tickets_off = 0;
  size_t scratch_off[4] = {0, 0, 0, 0};
  size_t max_elems = 0; int max_c = 0;
  // global regions (bytes from arena base)
  size_t params_off = 0, grads_off = 0, mom_off = 0, packed_off = 0, table_off = 0, mb_off = 0;
  size_t packed_elems = 0; int n_convs = 0;
  Loc g_stem;                          // gradient w.r.t. the stem output
  int t9_h = 0, t9_w = 0;                          // image shape of the whole-convolution weight-gradient items (class 10)
  std::vector<WgradItem> items[WGRAD_CLASSES];     // deferred weight-gradient work, per tile class (bf16 mode)
  std::vector<WgradItem> items_nr[WGRAD_CLASSES];  // the same without the blocks of image-resident runs (those have a launch of their own)
  size_t items_nr_off[WGRAD_CLASSES] = {};
  double wg_nr_bytes[WGRAD_CLASSES] = {}, wg_nr_flops[WGRAD_CLASSES] = {};
  size_t items_off[WGRAD_CLASSES] = {};
  double wg_bytes[WGRAD_CLASSES] = {}, wg_flops[WGRAD_CLASSES] = {};   // per micro-batch
  size_t arena_bytes = 0;
  size_t act_in_elems = 0, act_out_elems = 0;
  size_t skip_in_elems = 0, skip_out_elems = 0;   // shortcut value of a first / last block that is cut (0: none)
  size_t n_running = 0, running_off = 0, bn_table_off = 0;   // BatchNorm running statistics (fp32) and their table
  std::vector<BnRunDesc> bn_table;
  std::vector<PackDesc> table;
  size_t pack_max_elems() const {
    size_t m = 0;
    for (const PackDesc& d : table) m = std::max(m, (size_t)d.Cout * d.Kf);
    return m;
  }
  // image-resident runs of identity bottleneck blocks (bf16 mode, micro-batch statistics)
  struct ResRun { int first = 0, count = 0, kind = 1, C = 0, MID = 0, bands = 1; size_t table_off = 0; /* bytes from the arena base */ };
  std::vector<ResRun> runs;
  std::vector<int> run_at;             // per block: index of the run that starts (forward) at this block, else -1
  std::vector<int> run_end_at;         // per block: index of the run that ends at this block, else -1
  std::vector<ResBlock> res_blocks;
  size_t res_off = 0, abort_off = 0;   // global regions
  size_t splitk_off = 0, splitk_floats = 0;   // per micro-batch: fp32 partial sums of convolutions whose reduction is split over work-groups (bf16 mode)
  size_t xchg_off = 0, tag_off = 0;    // per-micro-batch region
};

hpf_status build_plan(const hpf_partition_desc* desc, Plan& P) {
  if (!desc) return fail(HPF_EINVAL, "null description");
  if (desc->abi_version != HPF_ABI_VERSION) return fail(HPF_EINVAL, "abi_version %u, expected %u", desc->abi_version, HPF_ABI_VERSION);
  P.d = *desc;
  const hpf_partition_desc& d = P.d;
  if (d.in_h <= 0 || d.in_w <= 0 || d.in_c <= 0) return fail(HPF_EINVAL, "input shape must be positive");
  if (d.microbatch <= 0 || d.num_microbatches <= 0 || d.loss_divisor <= 0) return fail(HPF_EINVAL, "microbatch, num_microbatches and loss_divisor must be positive");
  if (d.n_blocks < 0 || (d.n_blocks > 0 && !d.blocks)) return fail(HPF_EINVAL, "bad block list");
  if (!d.has_stem && !d.has_head && d.n_blocks == 0) return fail(HPF_EINVAL, "a partition needs at least one unit");
  if (d.compute_dtype != HPF_F32 && d.compute_dtype != HPF_BF16) return fail(HPF_EINVAL, "unknown compute_dtype");
  if (d.bn_mode != 0 && d.bn_mode != 1) return fail(HPF_EINVAL, "bn_mode must be 0 or 1");
  if (!(d.bn_eps > 0.f)) return fail(HPF_EINVAL, "bn_eps must be positive");
  if (d.has_stem && d.stem_c_out <= 0) return fail(HPF_EINVAL, "stem_c_out must be positive");
  if (d.has_head && d.num_classes <= 0) return fail(HPF_EINVAL, "num_classes must be positive");
  if (d.has_head < 0 || d.has_head > 2) return fail(HPF_EINVAL, "has_head must be 0, 1 or 2");
  P.blocks.assign(d.blocks, d.blocks + d.n_blocks);
  P.d.blocks = nullptr;
  P.dt = d.compute_dtype == HPF_BF16 ? DT_BF16 : DT_F32;
  P.esz = P.dt == DT_BF16 ? 2 : 4;
  const int cmul = P.dt == DT_BF16 ? 16 : 8;

  // ---- shape chain + validation
  int h = d.in_h, w = d.in_w, c = d.has_stem ? d.stem_c_out : d.in_c;
  if (c % cmul) return fail(HPF_EUNSUPPORTED, "channel count %d is not a multiple of %d", c, cmul);
  const int cmax = 1024;   // bf16 mode keeps a per-channel table of the source tensor in LDS
  if (d.first_block_from_conv < 0 || d.last_block_to_conv < 0) return fail(HPF_EINVAL, "negative layer cut");
  if (d.first_block_from_conv > 0 && (d.n_blocks == 0 || d.has_stem)) return fail(HPF_EINVAL, "first_block_from_conv needs a first block and no stem");
  if (d.last_block_to_conv > 0 && (d.n_blocks == 0 || d.has_head)) return fail(HPF_EINVAL, "last_block_to_conv needs a last block and no head");
  for (int i = 0; i < d.n_blocks; ++i) {
    const hpf_block_desc& b = P.blocks[i];
    if (b.kind >= K_POSTACT && b.kind <= K_BIAS_RELU) {   // units of VGG-16 / ResNet-v1: no cuts inside them
      if ((i == 0 && d.first_block_from_conv > 0) || (i == d.n_blocks - 1 && d.last_block_to_conv > 0))
        return fail(HPF_EINVAL, "block %d: layer cuts exist only inside pre-activation residual blocks", i);
      if (b.c_out <= 0 || b.c_in != c) return fail(HPF_EINVAL, "block %d: c_in %d does not continue the chain (%d)", i, b.c_in, c);
      if (b.kind == K_POSTACT && b.c_mid != b.c_out) return fail(HPF_EINVAL, "block %d: a post-activation block needs c_mid == c_out", i);
      if ((b.kind == K_BN_RELU || b.kind == K_BIAS_RELU) && b.c_in != b.c_out) return fail(HPF_EINVAL, "block %d: c_in must equal c_out", i);
      const bool strided = b.kind == K_POSTACT || b.kind == K_CONV_RELU;
      if (b.stride != 1 && !(strided && b.stride == 2)) return fail(HPF_EINVAL, "block %d: stride %d", i, b.stride);
      if (h % b.stride || w % b.stride) return fail(HPF_EINVAL, "block %d: %dx%d not divisible by stride", i, h, w);
      const long flat = (long)h * w * b.c_in;
      if (b.kind == K_DENSE && flat > (1 << 20)) return fail(HPF_EUNSUPPORTED, "block %d: dense input of %ld values", i, flat);
      if (b.c_in % cmul || b.c_out % cmul) return fail(HPF_EUNSUPPORTED, "block %d: channel counts must be multiples of %d", i, cmul);
      if (b.kind == K_DENSE) { h = 1; w = 1; } else { h /= b.stride; w /= b.stride; }
      c = b.c_out;
      continue;
    }
    if (b.kind != 0 && b.kind != 1) return fail(HPF_EINVAL, "block %d: kind %d", i, b.kind);
    const int nconv = b.kind == 0 ? 2 : 3;
    const int j0 = i == 0 ? d.first_block_from_conv : 0;
    const int j1 = (i == d.n_blocks - 1 && d.last_block_to_conv > 0) ? d.last_block_to_conv : nconv;
    if (j0 >= j1 || j1 > nconv || (i == d.n_blocks - 1 && d.last_block_to_conv >= nconv))
      return fail(HPF_EINVAL, "block %d: convolutions [%d, %d) of %d", i, j0, j1, nconv);
    if (b.c_mid <= 0 || b.c_out <= 0) return fail(HPF_EINVAL, "block %d: channel counts must be positive", i);
    if (j0 == 0 && b.c_in != c) return fail(HPF_EINVAL, "block %d: c_in %d does not continue the chain (%d)", i, b.c_in, c);
    if (j0 > 0 && b.c_mid != c) return fail(HPF_EINVAL, "block %d: c_mid %d does not continue the chain (%d)", i, b.c_mid, c);
    if (b.kind == 0 && b.c_mid != b.c_out) return fail(HPF_EINVAL, "block %d: a basic block needs c_mid == c_out", i);
    if (b.stride != 1 && b.stride != 2) return fail(HPF_EINVAL, "block %d: stride %d", i, b.stride);
    if (j0 == 0 && (h % b.stride || w % b.stride)) return fail(HPF_EINVAL, "block %d: %dx%d not divisible by stride", i, h, w);
    if (b.c_in % cmul || b.c_mid % cmul || b.c_out % cmul) return fail(HPF_EUNSUPPORTED, "block %d: channel counts must be multiples of %d", i, cmul);
    if (P.dt == DT_BF16 && (b.c_in > cmax || b.c_mid > cmax || b.c_out > cmax)) return fail(HPF_EUNSUPPORTED, "block %d: more than %d channels", i, cmax);
    if (j0 == 0) { h /= b.stride; w /= b.stride; }   // else the input already has the block's output size
    c = j1 == nconv ? b.c_out : b.c_mid;
  }
  P.out_h = h; P.out_w = w; P.out_c = c;
  if ((size_t)d.microbatch * d.in_h * d.in_w >= (1u << 30)) return fail(HPF_EUNSUPPORTED, "micro-batch too large");

  // ---- parameters (canonical order) and packed weights
  size_t off = 0, pk = 0;
  auto add_pack = [&](ConvPlan& cv, int pack_cin, bool want_dgrad) {
    if (P.dt != DT_BF16) return;
    const int T = cv.R * cv.R;
    cv.Kf = round_up32(T * pack_cin);
    cv.wf_off = pk; pk += (size_t)cv.cout * cv.Kf; pk = (pk + 7) / 8 * 8;
    PackDesc pd{};
    pd.w_off = cv.w_off; pd.wf_off = cv.wf_off; pd.wd_off = ~0ull;
    pd.T = T; pd.Cin = pack_cin; pd.Cout = cv.cout; pd.Kf = cv.Kf; pd.Kd = 0;
    if (want_dgrad) {
      cv.Kd = round_up32(T * cv.cout);
      cv.wd_off = pk; pk += (size_t)cv.cin * cv.Kd; pk = (pk + 7) / 8 * 8;
      pd.wd_off = cv.wd_off; pd.Kd = cv.Kd;
    }
    P.table.push_back(pd);
  };
  auto mk_conv = [&](int ci, int co, int R, int st, int hi, int wi) {
    ConvPlan cv; cv.cin = ci; cv.cout = co; cv.R = R; cv.stride = st; cv.h_in = hi; cv.w_in = wi;
    cv.h_out = hi / st; cv.w_out = wi / st; cv.w_off = off; off += (size_t)R * R * ci * co;
    return cv;
  };
  auto mk_bn = [&](int ch) {
    BnPlan b; b.C = ch; b.g_off = off; b.b_off = off + ch; off += 2 * (size_t)ch;
    b.run_off = P.n_running; P.n_running += 2 * (size_t)ch;
    return b;
  };

  h = d.in_h; w = d.in_w;
  if (d.has_stem) {
    P.stem = mk_conv(d.in_c, d.stem_c_out, 3, 1, h, w);
    P.stem_kc = round_up32(9 * d.in_c);
    if (P.dt == DT_BF16) {
      // runs as a 1x1 convolution over im2col columns: k = tap*in_c + c, a single "tap" of 9*in_c channels
      ConvPlan as1x1 = P.stem; as1x1.R = 1;
      add_pack(as1x1, 9 * d.in_c, false);
      P.stem.Kf = as1x1.Kf; P.stem.wf_off = as1x1.wf_off;
    }
  }
  P.bp.resize(d.n_blocks);
  for (int i = 0; i < d.n_blocks; ++i) {
    BlockPlan& p = P.bp[i];
    const hpf_block_desc& b = P.blocks[i];
    p.d = b;
    if (!p.residual()) {
      p.h_in = h; p.w_in = w;
      p.h_out = b.kind == K_DENSE ? 1 : h / b.stride; p.w_out = b.kind == K_DENSE ? 1 : w / b.stride;
      p.j0 = 0;
      if (b.kind == K_POSTACT) {
        p.nconv = 2;
        p.proj = (b.stride != 1 || b.c_in != b.c_out);
        p.cv[0] = mk_conv(b.c_in, b.c_mid, 3, b.stride, h, w); p.bn[0] = mk_bn(b.c_mid);
        p.cv[1] = mk_conv(b.c_mid, b.c_out, 3, 1, p.h_out, p.w_out); p.bn[1] = mk_bn(b.c_out);
        if (p.proj) p.pj = mk_conv(b.c_in, b.c_out, 1, b.stride, h, w);
        add_pack(p.cv[0], p.cv[0].cin, true); add_pack(p.cv[1], p.cv[1].cin, true);
        if (p.proj) add_pack(p.pj, p.pj.cin, true);
      } else if (b.kind == K_CONV_RELU) {
        p.nconv = 1;
        p.cv[0] = mk_conv(b.c_in, b.c_out, 3, 1, h, w); p.bias_off = off; off += b.c_out;
        add_pack(p.cv[0], p.cv[0].cin, true);
      } else if (b.kind == K_DENSE) {
        p.nconv = 1;
        p.cv[0] = mk_conv(h * w * b.c_in, b.c_out, 1, 1, 1, 1); p.bias_off = off; off += b.c_out;
        add_pack(p.cv[0], p.cv[0].cin, true);
      } else if (b.kind == K_BN_RELU) {
        p.nconv = 0; p.bn[0] = mk_bn(b.c_in);
      } else {
        p.nconv = 0; p.bias_off = off; off += b.c_in;
      }
      p.j1 = p.nconv;
      h = p.h_out; w = p.w_out;
      continue;
    }
    p.nconv = b.kind == 0 ? 2 : 3;
    p.j0 = i == 0 ? d.first_block_from_conv : 0;
    p.j1 = (i == d.n_blocks - 1 && d.last_block_to_conv > 0) ? d.last_block_to_conv : p.nconv;
    if (p.j0 == 0) { p.h_in = h; p.w_in = w; p.h_out = h / b.stride; p.w_out = w / b.stride; }
    else { p.h_in = h * b.stride; p.w_in = w * b.stride; p.h_out = h; p.w_out = w; }
    p.proj = (b.stride != 1 || b.c_in != b.c_out);
    const int cin[3] = {b.c_in, b.c_mid, b.c_mid};
    const int cout[3] = {b.c_mid, b.kind == 0 ? b.c_out : b.c_mid, b.c_out};
    const int R[3] = {b.kind == 0 ? 3 : 1, 3, 1};
    for (int j = p.j0; j < p.j1; ++j) {   // parameters only of the layers held here, in canonical order
      p.bn[j] = mk_bn(cin[j]);
      p.cv[j] = j == 0 ? mk_conv(cin[0], cout[0], R[0], b.stride, p.h_in, p.w_in) : mk_conv(cin[j], cout[j], R[j], 1, p.h_out, p.w_out);
    }
    if (p.proj && p.j0 == 0) p.pj = mk_conv(b.c_in, b.c_out, 1, b.stride, p.h_in, p.w_in);
    else p.proj = p.proj && p.j0 == 0;    // the projection lives with convolution 0
    for (int j = p.j0; j < p.j1; ++j) add_pack(p.cv[j], p.cv[j].cin, true);
    if (p.proj) add_pack(p.pj, p.pj.cin, true);
    h = p.h_out; w = p.w_out;
  }
  if (d.has_head) {
    if (d.has_head == 1) P.head_bn = mk_bn(P.out_c);
    P.wfc_off = off; off += (size_t)P.out_c * d.num_classes;
    P.bfc_off = off; off += d.num_classes;
  }
  P.n_params = off;
  P.packed_elems = pk;
  P.n_convs = (int)P.table.size();

  // ---- per-micro-batch region
  size_t mo = 0;
  size_t max_elems = 0; int max_c = 0;
  const size_t b_ = (size_t)d.microbatch;
  auto alloc = [&](size_t bytes) { Loc l; l.kind = IN_MB; l.off = mo; mo += align_up(bytes); return l; };
  auto tensor = [&](size_t elems) { if (elems > max_elems) max_elems = elems; return alloc(elems * P.esz); };
  size_t max_tile_part = 0;   // floats: partial records written by convolution epilogues (64-row tiles)
  auto stats = [&](BnPlan& bn, size_t M) {
    bn.stats_off = alloc(2 * (size_t)bn.C * sizeof(double)).off;
    P.bn_table.push_back(BnRunDesc{bn.stats_off, bn.C, (int)bn.run_off});
    if (bn.C > max_c) max_c = bn.C;
    const size_t need = ((M + 63) / 64) * (size_t)bn.C * 4;
    if (need > max_tile_part) max_tile_part = need;
  };

  P.act_in_elems = b_ * d.in_h * d.in_w * d.in_c;
  P.act_out_elems = d.has_head ? 0 : b_ * P.out_h * P.out_w * P.out_c;   // out_c: c_mid if the last block is cut
  Loc cur; cur.kind = CALLER_ACT_IN;
  if (d.has_stem) {
    const size_t Mst = b_ * d.in_h * d.in_w;
    if (P.dt == DT_BF16) P.stem_col = alloc(Mst * P.stem_kc * 2);
    const bool direct_out = (d.n_blocks == 0 && !d.has_head);
    if (direct_out) { P.stem_out.kind = CALLER_ACT_OUT; } else P.stem_out = tensor(Mst * d.stem_c_out);
    if (Mst * d.stem_c_out > max_elems) max_elems = Mst * d.stem_c_out;
    cur = P.stem_out;
  } else if (P.act_in_elems > max_elems) {
    max_elems = P.act_in_elems;
  }
  for (int i = 0; i < d.n_blocks; ++i) {
    BlockPlan& p = P.bp[i];
    const size_t M_in = b_ * p.h_in * p.w_in, M_out = b_ * p.h_out * p.w_out;
    if (!p.residual()) {   // every intermediate tensor of these units is kept; nothing is recomputed
      const bool to_caller = (i == d.n_blocks - 1) && !d.has_head;
      // needs_y: the unit's backward pass reads its output (the ReLU decision is taken on y)
      auto out_tensor = [&](size_t elems, bool needs_y) {
        if (to_caller && !needs_y) { Loc l; l.kind = CALLER_ACT_OUT; if (elems > max_elems) max_elems = elems; return l; }
        if (to_caller) p.copy_out = true;
        return tensor(elems);
      };
      p.x_in = cur;
      if (p.d.kind == K_POSTACT) {
        stats(p.bn[0], M_out); stats(p.bn[1], M_out);
        p.c[0] = tensor(M_out * p.d.c_mid); p.a[0] = tensor(M_out * p.d.c_mid); p.c[1] = tensor(M_out * p.d.c_out);
        p.sc = p.proj ? tensor(M_out * p.d.c_out) : p.x_in;
        p.y = out_tensor(M_out * p.d.c_out, true);
      } else if (p.d.kind == K_CONV_RELU) {
        if (p.d.stride == 2) { p.y0 = tensor(M_in * p.d.c_out); p.y = out_tensor(M_out * p.d.c_out, false); }
        else { p.y = out_tensor(M_out * p.d.c_out, true); p.y0 = p.y; }
      } else if (p.d.kind == K_DENSE) {
        p.y = out_tensor(b_ * p.d.c_out, true); p.y0 = p.y;
      } else if (p.d.kind == K_BN_RELU) {
        stats(p.bn[0], M_in);
        p.y = out_tensor(M_in * p.d.c_in, false); p.a[0] = p.y;   // the mask is recomputed from x
      } else {
        p.y = out_tensor(M_in * p.d.c_in, true); p.y0 = p.y;
      }
      if (M_in * p.d.c_in > max_elems) max_elems = M_in * p.d.c_in;
      if (M_in * p.d.c_out > max_elems) max_elems = M_in * p.d.c_out;
      if (p.d.c_out > max_c) max_c = p.d.c_out;   // the bias-gradient sums use the BatchNorm scratch
      cur = p.y;
      continue;
    }
    if (p.j0 == 0) p.x_in = cur; else p.c[p.j0 - 1] = cur;   // a block cut after its start takes convolution j0-1's output
    // bf16 mode: the convolutions apply a = relu(bn(x)) while staging x, so a is not written to memory -- except
    // where the staged operand is re-read so often (filter taps x channel tiles) that one pass writing a is cheaper
    const bool keep_a = (P.dt != DT_BF16);
    if (P.dt == DT_BF16) {
      for (int j = p.j0; j < p.j1; ++j) p.mat[j] = conv_operand_reuse(p.cv[j].cin, p.cv[j].cout, p.cv[j].R) >= 4;
      if (p.proj && conv_operand_reuse(p.pj.cin, p.pj.cout, p.pj.R) >= 4) p.mat[0] = true;
    }
    for (int j = p.j0; j < p.j1; ++j) {
      const size_t Mj = j == 0 ? M_in : M_out;
      stats(p.bn[j], Mj);
      if (keep_a || p.mat[j]) p.a[j] = tensor(Mj * p.cv[j].cin);
      if (j + 1 < p.j1) p.c[j] = tensor(M_out * p.cv[j].cout);
    }
    const bool last = (i == d.n_blocks - 1);
    if (p.j1 == p.nconv) {
      if (last && !d.has_head) { p.y.kind = CALLER_ACT_OUT; if (M_out * p.d.c_out > max_elems) max_elems = M_out * p.d.c_out; }
      else p.y = tensor(M_out * p.d.c_out);
      cur = p.y;
      if (p.j0 > 0) P.skip_in_elems = M_out * p.d.c_out;
    } else {   // the block ends in a later partition: convolution j1-1's output and the shortcut value leave
      p.c[p.j1 - 1].kind = CALLER_ACT_OUT;
      if (M_out * p.cv[p.j1 - 1].cout > max_elems) max_elems = M_out * p.cv[p.j1 - 1].cout;
      if (p.j0 == 0) { P.skip_out_elems = M_out * p.d.c_out; if (P.skip_out_elems > max_elems) max_elems = P.skip_out_elems; }
      cur = p.c[p.j1 - 1];
    }
  }
  if (d.has_head) {
    P.head_x = cur;
    if (d.has_head == 1) {
      stats(P.head_bn, b_ * P.out_h * P.out_w);
      P.head_a = tensor(b_ * P.out_h * P.out_w * P.out_c);
    } else {
      P.head_a = cur;   // global average pool - FC on the last unit's output as it is
    }
    P.head_g = alloc(b_ * P.out_c * sizeof(float));
    P.head_dl = alloc(b_ * d.num_classes * sizeof(float));
  }
  // gradient tensors: every gradient that a weight-gradient consumes keeps its own buffer, so that all
  // weight gradients of the pass can run as one grouped launch after the data-gradient chain
  if (d.has_stem) {
    if (d.n_blocks > 0 || d.has_head) P.g_stem = tensor(b_ * d.in_h * d.in_w * d.stem_c_out);
    else P.g_stem.kind = CALLER_ERR_IN;
  }
  for (int i = 0; i < d.n_blocks; ++i) {
    BlockPlan& p = P.bp[i];
    const size_t M_out = b_ * p.h_out * p.w_out;
    const bool last = (i == d.n_blocks - 1);
    if (!p.residual()) {
      if (last && !d.has_head) p.gy.kind = CALLER_ERR_IN; else p.gy = tensor(M_out * p.d.c_out);
      if (P.dt == DT_BF16) {   // what the deferred weight gradients read
        const size_t M_in = b_ * p.h_in * p.w_in;
        if (p.d.kind == K_POSTACT) {
          p.dc[0] = tensor(M_out * p.d.c_mid); p.dc[1] = tensor(M_out * p.d.c_out);
          if (p.proj) p.dc[2] = tensor(M_out * p.d.c_out);
        } else if (p.d.kind == K_CONV_RELU) {
          p.dc[0] = tensor(M_in * p.d.c_out);
        } else if (p.d.kind == K_DENSE) {
          p.dc[0] = tensor(b_ * p.d.c_out);
        }
      }
      continue;
    }
    if (p.j1 == p.nconv) {
      if (last && !d.has_head) p.gy.kind = CALLER_ERR_IN; else p.gy = tensor(M_out * p.d.c_out);
    } else {
      p.dc[p.j1 - 1].kind = CALLER_ERR_IN;                 // gradient w.r.t. the output that left
      if (p.j0 == 0) p.gy = tensor(M_out * p.d.c_out);     // the gradient w.r.t. the shortcut value is copied here
    }
    for (int j = p.j0 > 0 ? p.j0 - 1 : 0; j + 1 < p.j1; ++j) {
      if (j == p.j0 - 1) p.dc[j].kind = CALLER_ERR_OUT;    // gradient w.r.t. the partition's input
      else p.dc[j] = tensor(M_out * p.cv[j].cout);
    }
  }
  P.stash_bytes_per_mb = mo;
  P.max_elems = max_elems; P.max_c = max_c;
  if (max_c > 0) {
    P.sums_off = alloc(2 * (size_t)max_c * sizeof(double)).off;
    const size_t pf = bn_partials_floats(max_c) > max_tile_part ? bn_partials_floats(max_c) : max_tile_part;
    P.partials_off = alloc(pf * sizeof(float)).off;
  }
  P.tickets_off = alloc(64 * sizeof(unsigned)).off;
  for (int i = 0; i < 4; ++i) P.scratch_off[i] = alloc(max_elems * P.esz).off;

  // ---- image-resident runs: maximal sequences of identity bottleneck blocks of one shape
  P.run_at.assign(d.n_blocks, -1);
  P.run_end_at.assign(d.n_blocks, -1);
  if (P.dt == DT_BF16 && d.bn_mode == 0) {
    auto eligible = [&](int i) {
      const BlockPlan& p = P.bp[i];
      if (p.d.kind == K_POSTACT)   // post-activation basic block with identity shortcut
        return p.d.stride == 1 && !p.proj && p.d.c_in == p.d.c_mid && resident_shape_ok(2, p.d.c_in, p.d.c_mid, p.h_in, p.w_in, d.microbatch);
      return p.residual() && p.whole() && p.d.stride == 1 && !p.proj && resident_shape_ok(p.d.kind, p.d.c_in, p.d.c_mid, p.h_in, p.w_in, d.microbatch);
    };
    int cmax_run = 0;
    size_t xchg_bytes = 0;
    for (int i = 0; i < d.n_blocks;) {
      if (!eligible(i)) { ++i; continue; }
      int j = i + 1;
      while (j < d.n_blocks && eligible(j) && P.bp[j].d.kind == P.bp[i].d.kind && P.bp[j].d.c_in == P.bp[i].d.c_in &&
             P.bp[j].d.c_mid == P.bp[i].d.c_mid)
        ++j;
      Plan::ResRun r;
      r.first = i; r.count = j - i; r.kind = P.bp[i].d.kind; r.C = P.bp[i].d.c_in; r.MID = P.bp[i].d.c_mid;
      r.bands = resident_bands(r.kind, r.C, r.MID, P.bp[i].h_in, P.bp[i].w_in);
      r.table_off = P.res_blocks.size() * sizeof(ResBlock);   // made absolute below
      auto res_loc = [](const Loc& l) -> unsigned long long {
        switch (l.kind) {
          case IN_MB: return l.off;
          case CALLER_ACT_IN: return RES_ACT_IN;
          case CALLER_ACT_OUT: return RES_ACT_OUT;
          case CALLER_ERR_IN: return RES_ERR_IN;
          default: return RES_ERR_OUT;
        }
      };
      for (int k = i; k < j; ++k) {
        const BlockPlan& p = P.bp[k];
        ResBlock rb{};
        rb.x_off = res_loc(p.x_in); rb.c1_off = res_loc(p.c[0]); rb.y_off = res_loc(p.y);
        rb.gy_off = res_loc(p.gy); rb.dc1_off = res_loc(p.dc[0]);
        if (p.nconv == 3 || p.d.kind == K_POSTACT) { rb.c2_off = res_loc(p.c[1]); rb.dc2_off = res_loc(p.dc[1]); }
        Loc gx; gx.kind = CALLER_ERR_OUT;
        if (k > 0) gx = P.bp[k - 1].gy; else if (d.has_stem) gx = P.g_stem;
        rb.gx_off = res_loc(gx);
        for (int q = 0; q < p.nconv; ++q) {
          rb.stats_off[q] = p.bn[q].stats_off;
          rb.wf_off[q] = p.cv[q].wf_off; rb.wd_off[q] = p.cv[q].wd_off; rb.w_off[q] = p.cv[q].w_off;
          rb.gamma_off[q] = p.bn[q].g_off; rb.beta_off[q] = p.bn[q].b_off;
          rb.dgb_off[q] = alloc(2 * (size_t)p.bn[q].C * sizeof(float)).off;
          rb.run_off[q] = p.bn[q].run_off;
        }
        P.res_blocks.push_back(rb);
      }
      P.run_at[i] = (int)P.runs.size();
      P.run_end_at[j - 1] = (int)P.runs.size();
      P.runs.push_back(r);
      if (r.C > cmax_run) cmax_run = r.C;
      xchg_bytes = std::max(xchg_bytes, resident_xchg_bytes(r.C, d.microbatch, r.bands));
      i = j;
    }
    if (!P.runs.empty()) {
      P.xchg_off = alloc(std::max(xchg_bytes, resident_xchg_bytes(cmax_run, d.microbatch, 1))).off;
      P.tag_off = alloc(sizeof(unsigned)).off;
    }
  }
  if (P.dt == DT_BF16) {   // fp32 partial sums of the largest split convolution of the plan, either direction, any group size (capped: beyond, no split)
    const size_t cap = (size_t)8 << 20;   // floats per micro-batch
    auto need = [&](const ConvGeom& q) {
      for (int gm = 1; gm <= MAX_GROUP && gm <= d.num_microbatches; ++gm) {
        const int sp = conv_splitk(gm, q);
        const size_t n = (size_t)sp * q.M * q.N;
        if (sp > 1 && n <= cap && n > P.splitk_floats) P.splitk_floats = n;
      }
    };
    for (int i = 0; i < d.n_blocks; ++i) {
      const BlockPlan& p = P.bp[i];
      for (int j = 0; j < p.nconv; ++j) { need(conv_geom_fwd(p.cv[j], d.microbatch)); need(conv_geom_dgrad(p.cv[j], d.microbatch)); }
      if (p.proj) { need(conv_geom_fwd(p.pj, d.microbatch)); need(conv_geom_dgrad(p.pj, d.microbatch)); }
    }
    if (P.splitk_floats) P.splitk_off = alloc(P.splitk_floats * sizeof(float)).off;
  }
  P.mb_bytes = mo;

  // ---- deferred weight-gradient items (bf16 mode)
  if (P.dt == DT_BF16) {
    // the operand of a block convolution is relu(bn(x)) recomputed from the BatchNorm input x
    struct WConv { const ConvPlan* cv; int cin_run, c_valid, R; Loc a, dy; const BnPlan* bn; bool in_run; };
    std::vector<WConv> wc;
    ConvPlan stem1x1 = P.stem;
    if (d.has_stem) wc.push_back(WConv{&stem1x1, P.stem_kc, 9 * d.in_c, 1, P.stem_col, P.g_stem, nullptr, false});
    for (int i = 0; i < d.n_blocks; ++i) {
      const BlockPlan& p = P.bp[i];
      bool in_run = false;
      for (const Plan::ResRun& r : P.runs)   // runs without a weight-gradient launch of their own stay in the grouped launch
        in_run = in_run || (resident_has_wgrad_launch(r.kind, r.C, r.bands) && i >= r.first && i < r.first + r.count);
      if (!p.residual()) {   // the operands are stored activations (no BatchNorm to recompute)
        if (p.d.kind == K_POSTACT) {
          wc.push_back(WConv{&p.cv[0], p.cv[0].cin, p.cv[0].cin, p.cv[0].R, p.x_in, p.dc[0], nullptr, in_run});
          wc.push_back(WConv{&p.cv[1], p.cv[1].cin, p.cv[1].cin, p.cv[1].R, p.c[0], p.dc[1], &p.bn[0], in_run});   // relu(bn1(c1)) recomputed: a resident run does not write it
          if (p.proj) wc.push_back(WConv{&p.pj, p.pj.cin, p.pj.cin, 1, p.x_in, p.dc[2], nullptr, false});
        } else if (p.d.kind == K_CONV_RELU || p.d.kind == K_DENSE) {
          wc.push_back(WConv{&p.cv[0], p.cv[0].cin, p.cv[0].cin, p.cv[0].R, p.x_in, p.dc[0], nullptr, false});
        }
        continue;
      }
      for (int j = p.j0; j < p.j1; ++j)
        wc.push_back(WConv{&p.cv[j], p.cv[j].cin, p.cv[j].cin, p.cv[j].R, p.mat[j] ? p.a[j] : (j == 0 ? p.x_in : p.c[j - 1]),
                           j == p.nconv - 1 ? p.gy : p.dc[j], p.mat[j] ? nullptr : &p.bn[j], in_run});
      if (p.proj) wc.push_back(WConv{&p.pj, p.pj.cin, p.pj.cin, 1, p.mat[0] ? p.a[0] : p.x_in, p.gy, p.mat[0] ? nullptr : &p.bn[0], false});
    }
    // output tiles per class: the pixel rows are split so that every class launches roughly 1500 work-groups
    // (5-6 per CU: enough to hide the staging latency) while atomics per output element stay few
    auto geom_of = [&](const WConv& w) {
      const ConvPlan& cv = *w.cv;
      WgradGeom q{};
      q.b = d.microbatch; q.H = cv.h_in; q.W = cv.w_in; q.Cin = w.cin_run; q.Ho = cv.h_out; q.Wo = cv.w_out; q.N = cv.cout;
      q.R = w.R; q.stride = cv.stride; q.pad = (w.R - 1) / 2; q.M = q.b * q.Ho * q.Wo; q.c_valid = w.c_valid;
      return q;
    };
    // whole-convolution items (3x3 between 16 and 16 channels) share one launch, so one image shape: the first one's
    auto class_of = [&](const WgradGeom& q) {
      int cls = wgrad_item_class(q);
      if (cls == WGRAD_CLASS_T9) {
        if (P.t9_h == 0) { P.t9_h = q.H; P.t9_w = q.W; }
        if (q.H != P.t9_h || q.W != P.t9_w) cls = wgrad_tile_class(q.Cin, q.N);
      }
      return cls;
    };
    for (int pass = 0; pass < 2; ++pass) {   // pass 1: without the convolutions of image-resident runs
    if (pass == 1 && P.runs.empty()) break;
    long tiles_in_class[WGRAD_CLASSES] = {}, steps_in_class[WGRAD_CLASSES] = {};   // steps: 128 pixel rows of one output tile
    for (const WConv& w : wc) {
      if (pass == 1 && w.in_run) continue;
      const int cls = class_of(geom_of(w));
      int bc, bn;
      wgrad_tile_dims(cls, &bc, &bn);
      const long tiles = cls == WGRAD_CLASS_T9 ? 1 : (long)w.R * w.R * (w.cin_run / bc) * (w.cv->cout / bn);
      tiles_in_class[cls] += tiles;
      steps_in_class[cls] += tiles * ((d.microbatch * w.cv->h_out * w.cv->w_out + 127) / 128);
    }
    for (const WConv& w : wc) {
      if (pass == 1 && w.in_run) continue;
      const ConvPlan& cv = *w.cv;
      const WgradGeom q = geom_of(w);
      const int cls = class_of(q);
      int bc, bn;
      wgrad_tile_dims(cls, &bc, &bn);
      (pass ? P.wg_nr_bytes : P.wg_bytes)[cls] += 2.0 * ((double)q.b * q.H * q.W * q.Cin + (double)q.M * q.N);
      (pass ? P.wg_nr_flops : P.wg_flops)[cls] += 2.0 * q.M * (double)(w.R * w.R * q.Cin) * q.N;
      auto item = [&](int tap, int c0, int n0, int m_begin, int m_end) {
        WgradItem it{};
        it.a_off = w.a.kind == IN_MB ? w.a.off : WGRAD_DY_CALLER;
        it.dy_off = w.dy.kind == IN_MB ? w.dy.off : WGRAD_DY_CALLER;
        it.dw_off = cv.w_off;
        it.stats_off = w.bn ? w.bn->stats_off : WGRAD_NO_BN;
        it.gamma_off = w.bn ? w.bn->g_off : 0;
        it.beta_off = w.bn ? w.bn->b_off : 0;
        it.g = q; it.tap = tap; it.c0 = c0; it.n0 = n0;
        it.m_begin = m_begin; it.m_end = m_end;
        (pass ? P.items_nr : P.items)[cls].push_back(it);
      };
      if (cls == WGRAD_CLASS_T9) {   // whole images per item; about 1000 work-groups (two per CU at 67 KiB of LDS, twice over)
        int parts = (int)((1024 + tiles_in_class[cls] - 1) / tiles_in_class[cls]);
        if (parts > q.b) parts = q.b;
        const int imgs = (q.b + parts - 1) / parts, px = q.H * q.W;
        for (int i0 = 0; i0 < q.b; i0 += imgs) item(0, 0, 0, i0 * px, (i0 + imgs < q.b ? i0 + imgs : q.b) * px);
        continue;
      }
      // Items of equal length: a class may mix convolutions with few tiles over many pixel rows and ones with many
      // tiles over few rows (VGG-16: 128 -> 128 channels at 16x16 next to 4096 x 4096 over 16 rows); with one split
      // count for all, the former made a handful of work-groups run 64 times longer than the rest of the launch.
      const long want = 1536;
      const long per_item = (steps_in_class[cls] + want - 1) / want;   // steps of 128 rows an item should take
      const int max_splits = (q.M + 127) / 128;
      int splits = (int)((max_splits + per_item - 1) / per_item);
      if (splits > max_splits) splits = max_splits;
      if (splits < 1) splits = 1;
      const int rows = ((q.M + splits - 1) / splits + 127) / 128 * 128;
      splits = (q.M + rows - 1) / rows;
      for (int tap = 0; tap < w.R * w.R; ++tap)
        for (int c0 = 0; c0 < w.cin_run; c0 += bc)
          for (int n0 = 0; n0 < cv.cout; n0 += bn)
            for (int sp = 0; sp < splits; ++sp) item(tap, c0, n0, sp * rows, (sp + 1) * rows < q.M ? (sp + 1) * rows : q.M);
    }
    }
  }

  // ---- global regions
  size_t g = 0;
  P.params_off = g; g += align_up(P.n_params * sizeof(float));
  P.grads_off = g;  g += align_up(P.n_params * sizeof(float));
  P.mom_off = g;    g += align_up(P.n_params * sizeof(float));
  P.packed_off = g; g += align_up(P.packed_elems * 2);
  P.table_off = g;  g += align_up(P.table.size() * sizeof(PackDesc));
  for (int k = 0; k < WGRAD_CLASSES; ++k) { P.items_off[k] = g; g += align_up(P.items[k].size() * sizeof(WgradItem)); }
  for (int k = 0; k < WGRAD_CLASSES; ++k) { P.items_nr_off[k] = g; g += align_up(P.items_nr[k].size() * sizeof(WgradItem)); }
  P.res_off = g;    g += align_up(P.res_blocks.size() * sizeof(ResBlock));
  for (Plan::ResRun& r : P.runs) r.table_off += P.res_off;
  P.abort_off = g;  g += align_up(sizeof(int));
  P.running_off = g; g += align_up(P.n_running * sizeof(float));
  P.bn_table_off = g; g += align_up(P.bn_table.size() * sizeof(BnRunDesc));
  P.mb_off = g;     g += P.mb_bytes * (size_t)d.num_microbatches;
  P.arena_bytes = g;
  return HPF_OK;
}

}  // namespace

enum ProfCat { PROF_NONE = -1, PROF_RES_FWD = 0, PROF_RES_BWD, PROF_RES_WGRAD, PROF_WGRAD, PROF_CONV_FWD, PROF_CONV_DGRAD, PROF_OTHER_FWD,
               PROF_OTHER_BWD, PROF_N };
const char* const kProfNames[PROF_N] = {"resident_forward", "resident_backward", "resident_wgrad", "wgrad_grouped", "conv_forward",
                                        "conv_dgrad",       "other_forward",     "other_backward"};

// One captured HIP graph of a micro-batch's forward or backward kernel sequence, valid for the caller
// pointers it was captured with.
struct GraphSlot {
  hipGraphExec_t exec = nullptr;
  std::vector<const void*> key;
  bool direct = false;   // the sequence is so short that plain launches are cheaper than a graph launch
};
constexpr int kMinGraphLaunches = 8;

struct hpf_partition {
  Plan P;
  bool use_graphs = true;
  // bf16 mode: 0 = every BatchNorm step a kernel of its own, 1 = BN reductions in the convolution epilogues and
  // normalisation in the consuming convolutions, 2 = additionally image-resident kernels for runs of identity
  // bottleneck blocks
  int fuse = 2;
  int res_group = 0;   // micro-batches one image-resident launch may hold on this device (0: path unavailable)
  float bn_momentum = 1.f;   // running statistics: r <- m*r + (1-m)*batch after every training forward; 1: never
  // per-kernel-class timing
  bool profiling = false;
  struct ProfSeg { int cat; hipEvent_t e0, e1; int launches; double bytes, flops; };
  std::vector<ProfSeg> prof_pending;
  std::vector<hipEvent_t> ev_pool;
  double prof_ms[PROF_N] = {}, prof_bytes[PROF_N] = {}, prof_flops[PROF_N] = {};
  long long prof_launches[PROF_N] = {};
  hipEvent_t prof_event() {
    hipEvent_t e = nullptr;
    if (!ev_pool.empty()) { e = ev_pool.back(); ev_pool.pop_back(); return e; }
    return hipEventCreate(&e) == hipSuccess ? e : nullptr;
  }
  std::vector<GraphSlot> g_fwd, g_bwd;
  GraphSlot g_inf[8];   // inference forward: graphs of the last 8 distinct argument sets
  int g_inf_next = 0;
  char* arena = nullptr;
  std::vector<unsigned char> fwd_done, bwd_done;
  std::vector<const void*> act_in;
  int n_bwd = 0;
  std::vector<hipEvent_t> ev_fwd, ev_bwd;
  // the members of one launch share its first member's event: fwd_ev[mb] / bwd_ev[mb] say whose event covers mb
  std::vector<int> fwd_ev, bwd_ev;
  std::vector<hipStream_t> fwd_stream, bwd_stream;   // the stream each leader's event was last recorded on
  hipEvent_t ev_step = nullptr;
  bool step_recorded = false;
  hipStream_t step_stream = nullptr, run_stream = nullptr;
  hipEvent_t ev_run = nullptr;   // last forward that moved the BatchNorm running statistics
  bool run_recorded = false;

  float* params() const { return (float*)(arena + P.params_off); }
  float* grads() const { return (float*)(arena + P.grads_off); }
  float* mom() const { return (float*)(arena + P.mom_off); }
  bf16_t* packed() const { return (bf16_t*)(arena + P.packed_off); }
  char* mb_base(int mb) const { return arena + P.mb_off + (size_t)mb * P.mb_bytes; }
  int* abort_flag() const { return (int*)(arena + P.abort_off); }
  float* running() const { return (float*)(arena + P.running_off); }
  bool resident() const { return fuse >= 2 && res_group >= 1 && !P.runs.empty(); }
  int group_limit() const { return resident() ? res_group : MAX_GROUP; }
};

namespace {

// Everything one call needs: the handle, the group of consecutive micro-batches [mb0, mb0+g), the stream
// and the caller buffers of every member.
struct Ctx {
  hpf_partition* h; int mb0; int g; hipStream_t s;
  const void* act_in[MAX_GROUP]; void* act_out[MAX_GROUP]; const void* err_in[MAX_GROUP]; void* err_out[MAX_GROUP];
  // shortcut value of a cut block: received / sent in forward, its gradient sent back / received in backward
  const void* skip_in[MAX_GROUP] = {}; void* skip_out[MAX_GROUP] = {}; const void* skip_err_in[MAX_GROUP] = {}; void* skip_err_out[MAX_GROUP] = {};
  bool inference = false;   // BatchNorm by running statistics, nothing kept for a backward pass, logits instead of the loss
  hipError_t err = hipSuccess;
  const char* where = "";
  hpf_partition::ProfSeg cur{PROF_NONE, nullptr, nullptr, 0, 0, 0};

  // Profiling: launches from here on belong to class `cat` (a new segment starts even if the class repeats)
  void seg(int cat, double bytes = 0, double flops = 0) {
    if (!h->profiling) return;
    seg_end();
    cur = hpf_partition::ProfSeg{cat, h->prof_event(), h->prof_event(), 0, bytes, flops};
    if (cur.e0) (void)hipEventRecord(cur.e0, s);
  }
  void seg_same(int cat) { if (h->profiling && cur.cat != cat) seg(cat); }
  void seg_end() {
    if (cur.cat == PROF_NONE) return;
    if (cur.e1) (void)hipEventRecord(cur.e1, s);
    if (cur.e0 && cur.e1 && cur.launches > 0) h->prof_pending.push_back(cur);
    else { if (cur.e0) h->ev_pool.push_back(cur.e0); if (cur.e1) h->ev_pool.push_back(cur.e1); }
    cur.cat = PROF_NONE;
  }

  PtrTab tab(const Loc& l) const {
    PtrTab t{};
    for (int i = 0; i < g; ++i) {
      switch (l.kind) {
        case IN_MB: t.p[i] = h->mb_base(mb0 + i) + l.off; break;
        case CALLER_ACT_IN: t.p[i] = const_cast<void*>(act_in[i]); break;
        case CALLER_ACT_OUT: t.p[i] = act_out[i]; break;
        case CALLER_ERR_IN: t.p[i] = const_cast<void*>(err_in[i]); break;
        case CALLER_ERR_OUT: t.p[i] = err_out[i]; break;
        case CALLER_SKIP_IN: t.p[i] = const_cast<void*>(skip_in[i]); break;
        case CALLER_SKIP_OUT: t.p[i] = skip_out[i]; break;
        case CALLER_SKIP_ERR_IN: t.p[i] = const_cast<void*>(skip_err_in[i]); break;
        case CALLER_SKIP_ERR_OUT: t.p[i] = skip_err_out[i]; break;
        default: t.p[i] = nullptr;
      }
    }
    return t;
  }
  PtrTab mbp(size_t off) const { Loc l; l.kind = IN_MB; l.off = off; return tab(l); }
  PtrTab scratch(int i) const { return mbp(h->P.scratch_off[i]); }
  static PtrTab none() { return PtrTab{}; }
  int n_launches = 0;
  void chk(hipError_t e, const char* w) {
    if (err == hipSuccess && e != hipSuccess) { err = e; where = w; }
    if (cur.cat != PROF_NONE) ++cur.launches;
    ++n_launches;
  }

  bool fused() const { return h->fuse >= 1 && h->P.dt == DT_BF16 && h->P.d.bn_mode == 0; }
  void copy(const PtrTab& dst, const PtrTab& src, size_t bytes) {
    for (int i = 0; i < g; ++i) chk(launch_copy_bytes(dst.p[i], src.p[i], bytes, s), "copy");
  }

  // part_rows > 0: the producing convolution already wrote that many statistics partial rows.
  // apply == false: only the statistics (the consuming convolutions normalise while staging)
  void bn_fwd(const BnPlan& bn, const PtrTab& x, const PtrTab& a, size_t M, int part_rows = 0, bool apply = true) {
    const Plan& P = h->P;
    const PtrTab st = mbp(bn.stats_off);
    if (inference)
      chk(launch_bn_running_stats(P.dt, g, st, h->running() + bn.run_off, bn.C, P.d.bn_eps, s), "bn_running_stats");
    else if (P.d.bn_mode != 0)
      chk(launch_bn_frozen_stats(P.dt, g, st, bn.C, P.d.bn_eps, s), "bn_frozen_stats");
    else if (part_rows > 0)
      chk(launch_bn_stats_finalize(g, (int)M, bn.C, part_rows, P.d.bn_eps, mbp(P.partials_off), st, s), "bn_stats_finalize");
    else
      chk(launch_bn_stats(P.dt, g, x, (int)M, bn.C, P.d.bn_eps, st, mbp(P.partials_off), s), "bn_stats");
    if (apply)
      chk(launch_bn_apply_relu(P.dt, g, x, a, h->params() + bn.g_off, h->params() + bn.b_off, st, (int)M, bn.C, s), "bn_apply_relu");
  }
  // part_rows > 0: `da` already holds dz and the producing data-gradient wrote that many partial rows.
  void bn_bwd(const BnPlan& bn, const PtrTab& x, const PtrTab& da, const PtrTab& skip, const PtrTab& dx, size_t M,
              int part_rows = 0) {
    const Plan& P = h->P;
    const PtrTab st = mbp(bn.stats_off);
    if (part_rows > 0)
      chk(launch_bn_bwd_finalize(g, bn.C, part_rows, mbp(P.partials_off), mbp(P.sums_off), h->grads() + bn.g_off,
                                 h->grads() + bn.b_off, s),
          "bn_bwd_finalize");
    else
      chk(launch_bn_bwd_reduce(P.dt, g, x, da, h->params() + bn.g_off, h->params() + bn.b_off, st, (int)M, bn.C, mbp(P.sums_off),
                               h->grads() + bn.g_off, h->grads() + bn.b_off, mbp(P.partials_off), s),
          "bn_bwd_reduce");
    chk(launch_bn_bwd_apply(P.dt, g, x, da, h->params() + bn.g_off, h->params() + bn.b_off, st, mbp(P.sums_off), skip, dx, (int)M,
                            bn.C, P.d.bn_mode, s),
        "bn_bwd_apply");
  }
  // Profiling: a bf16 convolution launch is a segment of its own with its algorithmic figures (2*M*K*N flop; source,
  // weights, output [, residual operand] once).  Returns the class to go back to afterwards (PROF_NONE: not profiling).
  int conv_seg(int cat, const ConvGeom& q, bool has_add) {
    if (!h->profiling) return PROF_NONE;
    const int back = cur.cat == PROF_NONE ? (cat == PROF_CONV_FWD ? PROF_OTHER_FWD : PROF_OTHER_BWD) : cur.cat;
    const double m_src = (double)q.b * q.Hs * q.Ws;
    seg(cat, (double)g * 2.0 * (m_src * q.Cs + (double)q.Ktot * q.N + (double)q.M * q.N * (has_add ? 2.0 : 1.0)),
        (double)g * 2.0 * q.M * (double)q.Ktot * q.N);
    return back;
  }
  ConvGeom geom_fwd(const ConvPlan& cv) const { return conv_geom_fwd(cv, h->P.d.microbatch); }
  ConvGeom geom_dgrad(const ConvPlan& cv) const { return conv_geom_dgrad(cv, h->P.d.microbatch); }
  // want_stats: the output feeds a BatchNorm; returns the number of partial rows written (0 = none).
  // pro_bn (bf16 mode): x is the input of that BatchNorm and the convolution normalises it while staging.
  int conv_fwd(const ConvPlan& cv, const PtrTab& x, const PtrTab& y, const PtrTab& add, bool want_stats = false,
               const BnPlan* pro_bn = nullptr) {
    const ConvGeom q = geom_fwd(cv);
    if (h->P.dt == DT_BF16) {
      ConvEpi epi;
      ConvPro pro;
      if (pro_bn) {
        pro.on = 1; pro.stats = mbp(pro_bn->stats_off);
        pro.gamma = h->params() + pro_bn->g_off; pro.beta = h->params() + pro_bn->b_off;
      }
      int rows = 0;
      if (want_stats && fused() && !inference) {
        epi.kind = EPI_STATS; epi.partials = mbp(h->P.partials_off);
        const int bm = conv_mfma_tile_rows(g, q);
        rows = (q.M + bm - 1) / bm;
      }
      if (h->P.splitk_floats) { epi.splitk_ws = mbp(h->P.splitk_off); epi.splitk_floats = h->P.splitk_floats; }
      const int back = conv_seg(PROF_CONV_FWD, q, add.p[0] != nullptr);
      chk(launch_conv_mfma(CONV_FWD, g, x, h->packed() + cv.wf_off, y, add, q, s, epi, pro), "conv_fwd");
      if (back != PROF_NONE) seg(back);
      return rows;
    }
    chk(launch_conv_f32(CONV_FWD, g, x, h->params() + cv.w_off, y, add, q, s), "conv_fwd_f32");
    return 0;
  }
  // bn / bn_x: the BatchNorm (and its stashed input) whose backward consumes dx; returns partial rows.
  int conv_dgrad(const ConvPlan& cv, const PtrTab& dy, const PtrTab& dx, const PtrTab& add, const BnPlan* bn = nullptr,
                 const PtrTab* bn_x = nullptr) {
    const ConvGeom q = geom_dgrad(cv);
    if (h->P.dt == DT_BF16) {
      ConvEpi epi;
      int rows = 0;
      if (bn && fused()) {
        epi.kind = EPI_BNBWD; epi.partials = mbp(h->P.partials_off); epi.x = *bn_x; epi.stats = mbp(bn->stats_off);
        epi.gamma = h->params() + bn->g_off; epi.beta = h->params() + bn->b_off;
        const int bm = conv_mfma_tile_rows(g, q);
        rows = (q.M + bm - 1) / bm;
      }
      if (h->P.splitk_floats) { epi.splitk_ws = mbp(h->P.splitk_off); epi.splitk_floats = h->P.splitk_floats; }
      const int back = conv_seg(PROF_CONV_DGRAD, q, add.p[0] != nullptr);
      chk(launch_conv_mfma(CONV_DGRAD, g, dy, h->packed() + cv.wd_off, dx, add, q, s, epi), "conv_dgrad");
      if (back != PROF_NONE) seg(back);
      return rows;
    }
    chk(launch_conv_f32(CONV_DGRAD, g, dy, h->params() + cv.w_off, dx, add, q, s), "conv_dgrad_f32");
    return 0;
  }
  ResArgs res_args(const Plan::ResRun& r) const {
    const Plan& P = h->P;
    const BlockPlan& p0 = P.bp[r.first];
    ResArgs a{};
    a.blocks = (const ResBlock*)(h->arena + r.table_off);
    a.nblk = r.count; a.nmem = P.d.microbatch; a.H = p0.h_in; a.W = p0.w_in; a.eps = P.d.bn_eps;
    for (int i = 0; i < g; ++i) {
      a.base.p[i] = h->mb_base(mb0 + i);
      a.act_in.p[i] = const_cast<void*>(act_in[i]); a.act_out.p[i] = act_out[i];
      a.err_in.p[i] = const_cast<void*>(err_in[i]); a.err_out.p[i] = err_out[i];
    }
    a.params = h->params(); a.running = h->running(); a.packed = h->packed(); a.grads = h->grads();
    a.xchg_off = P.xchg_off; a.tag_off = P.tag_off; a.abort_flag = h->abort_flag();
    return a;
  }
  // algorithmic figures of a run per image: every stashed tensor once (elements), contraction flop of one direction
  static void res_figures(const Plan::ResRun& r, double px, double* stash_elems, double* flops) {
    if (r.kind == 2) { *stash_elems = px * 3.0 * r.C; *flops = 2.0 * px * 2.0 * 9.0 * r.C * r.C; }
    else if (r.kind == 0) { *stash_elems = px * 2.0 * r.C; *flops = 2.0 * px * 2.0 * 9.0 * r.C * r.C; }
    else { *stash_elems = px * (2.0 * r.MID + r.C); *flops = 2.0 * px * (2.0 * r.C * r.MID + 9.0 * r.MID * r.MID); }
  }
  void res_forward(const Plan::ResRun& r) {
    const BlockPlan& p0 = h->P.bp[r.first];
    const double img = (double)g * h->P.d.microbatch, px = (double)p0.h_in * p0.w_in;
    double st, fl;
    res_figures(r, px, &st, &fl);
    seg(PROF_RES_FWD, img * 2.0 * (px * r.C + r.count * st), img * r.count * fl);
    chk(launch_resident_forward(r.kind, g, r.C, r.MID, res_args(r), s), "resident_forward");
    seg_end();
  }
  void res_inference(const Plan::ResRun& r) {
    const BlockPlan& p0 = h->P.bp[r.first];
    const double img = (double)g * h->P.d.microbatch, px = (double)p0.h_in * p0.w_in;
    double st, fl;
    res_figures(r, px, &st, &fl);
    seg(PROF_RES_FWD, img * 2.0 * 2.0 * px * r.C, img * r.count * fl);   // run input read, run output written
    chk(launch_resident_inference(r.kind, g, r.C, r.MID, res_args(r), s), "resident_inference");
    seg_end();
  }
  void res_backward(const Plan::ResRun& r) {
    const BlockPlan& p0 = h->P.bp[r.first];
    const double img = (double)g * h->P.d.microbatch, px = (double)p0.h_in * p0.w_in;
    double st, fl;
    res_figures(r, px, &st, &fl);
    seg(PROF_RES_BWD, img * 2.0 * (px * r.C + r.count * 2.0 * st), img * r.count * fl);
    chk(launch_resident_backward(r.kind, g, r.C, r.MID, res_args(r), s), "resident_backward");
    seg_end();
  }
  void res_wgrad(const Plan::ResRun& r) {
    const BlockPlan& p0 = h->P.bp[r.first];
    const double img = (double)g * h->P.d.microbatch, px = (double)p0.h_in * p0.w_in;
    double st, fl;
    res_figures(r, px, &st, &fl);
    seg(PROF_RES_WGRAD, img * r.count * 2.0 * 2.0 * st, img * r.count * fl);
    chk(launch_resident_wgrad(r.kind, g, r.C, r.MID, res_args(r), s), "resident_wgrad");
    seg_end();
  }
  void conv_wgrad(const ConvPlan& cv, const PtrTab& a, const PtrTab& dy) {
    WgradGeom q{};
    q.b = h->P.d.microbatch; q.H = cv.h_in; q.W = cv.w_in; q.Cin = cv.cin; q.Ho = cv.h_out; q.Wo = cv.w_out; q.N = cv.cout;
    q.R = cv.R; q.stride = cv.stride; q.pad = (cv.R - 1) / 2; q.M = q.b * q.Ho * q.Wo; q.c_valid = cv.cin;
    if (h->P.dt == DT_BF16)
      chk(launch_wgrad_mfma(g, a, dy, h->grads() + cv.w_off, q, s), "conv_wgrad");
    else
      chk(launch_wgrad_f32(g, a, dy, h->grads() + cv.w_off, q, s), "conv_wgrad_f32");
  }
};

// The unit starts with a BatchNorm on its input, so the convolution in front of it may take the statistics in its epilogue.
bool takes_stats(const BlockPlan& p) { return p.residual() || p.d.kind == K_BN_RELU; }

void run_forward(Ctx& c, const PtrTab& labels, float* loss_accum) {
  const Plan& P = c.h->P;
  const size_t b = (size_t)P.d.microbatch;
  int part_rows = 0;   // statistics partial rows pending for the next BatchNorm (written by the last conv)
  const bool resident = c.h->resident();
  c.seg_same(PROF_OTHER_FWD);
  if (P.d.has_stem) {
    Loc in; in.kind = CALLER_ACT_IN;
    const bool feeds_bn = (!P.bp.empty() && !(resident && P.run_at[0] >= 0) && takes_stats(P.bp[0])) || (P.bp.empty() && P.d.has_head == 1);
    if (P.dt == DT_BF16) {
      const PtrTab col = c.tab(P.stem_col);
      c.chk(launch_im2col3x3(c.g, c.tab(in), col, (int)b, P.d.in_h, P.d.in_w, P.d.in_c, P.stem_kc, c.s), "im2col");
      ConvPlan cv = P.stem; cv.R = 1; cv.cin = P.stem_kc;   // 1x1 convolution over the im2col columns
      part_rows = c.conv_fwd(cv, col, c.tab(P.stem_out), Ctx::none(), feeds_bn);
    } else {
      c.conv_fwd(P.stem, c.tab(in), c.tab(P.stem_out), Ctx::none());
    }
  }
  for (size_t bi = 0; bi < P.bp.size(); ++bi) {
    if (resident && P.run_at[bi] >= 0 &&
        !(c.inference && !resident_has_inference_launch(P.runs[P.run_at[bi]].kind, P.runs[P.run_at[bi]].bands))) {   // the whole run in one launch; it takes its own statistics
      const Plan::ResRun& r = P.runs[P.run_at[bi]];
      if (c.inference) c.res_inference(r);
      else c.res_forward(r);
      bi += r.count - 1;
      if (const BlockPlan& pl = P.bp[bi]; pl.copy_out) {   // the partition's last unit keeps its output for the backward pass
        Loc lo; lo.kind = CALLER_ACT_OUT;
        c.copy(c.tab(lo), c.tab(pl.y), b * pl.h_out * pl.w_out * pl.d.c_out * P.esz);
      }
      part_rows = 0;
      continue;
    }
    c.seg_same(PROF_OTHER_FWD);
    const BlockPlan& p = P.bp[bi];
    const size_t M_in = b * p.h_in * p.w_in, M_out = b * p.h_out * p.w_out;
    const bool bf = (P.dt == DT_BF16);
    if (!p.residual()) {   // a unit of VGG-16 / ResNet-v1: plain launches, every intermediate tensor kept
      const PtrTab x = c.tab(p.x_in), y = c.tab(p.y);
      const float* bias = c.h->params() + p.bias_off;
      if (p.d.kind == K_POSTACT) {
        // c1 = conv1(x); a1 = relu(bn1(c1)); c2 = conv2(a1); y = relu(bn2(c2) + shortcut)
        const PtrTab c1 = c.tab(p.c[0]), a1 = c.tab(p.a[0]), c2 = c.tab(p.c[1]);
        // the BatchNorm sums come out of the producing convolution's epilogue (fusion levels 1 and 2)
        const int rows1 = c.conv_fwd(p.cv[0], x, c1, Ctx::none(), true);
        c.bn_fwd(p.bn[0], c1, a1, M_out, rows1);
        if (p.proj) c.conv_fwd(p.pj, x, c.tab(p.sc), Ctx::none());
        const int rows2 = c.conv_fwd(p.cv[1], a1, c2, Ctx::none(), true);
        c.bn_fwd(p.bn[1], c2, Ctx::none(), M_out, rows2, false);   // statistics only
        c.chk(launch_bn_add_relu_apply(P.dt, c.g, c2, c.tab(p.sc), y, c.h->params() + p.bn[1].g_off, c.h->params() + p.bn[1].b_off,
                                       c.mbp(p.bn[1].stats_off), (int)M_out, p.bn[1].C, c.s),
              "bn_add_relu");
      } else if (p.d.kind == K_CONV_RELU || p.d.kind == K_DENSE) {
        const PtrTab y0 = c.tab(p.y0);
        c.conv_fwd(p.cv[0], x, y0, Ctx::none());
        const int rows = p.d.kind == K_DENSE ? (int)b : (int)M_in;
        c.chk(launch_bias_act_fwd(P.dt, c.g, y0, y0, bias, rows, p.d.c_out, p.d.kind == K_DENSE ? (p.d.c_mid != 0) : 1, c.s), "bias_act");
        if (p.d.kind == K_CONV_RELU && p.d.stride == 2)
          c.chk(launch_maxpool2_fwd(P.dt, c.g, y0, y, (int)b, p.h_in, p.w_in, p.d.c_out, c.s), "maxpool");
      } else if (p.d.kind == K_BN_RELU) {
        c.bn_fwd(p.bn[0], x, y, M_in, part_rows);
      } else {
        c.chk(launch_bias_act_fwd(P.dt, c.g, x, y, bias, (int)M_in, p.d.c_in, 1, c.s), "bias_act");
      }
      if (p.copy_out) {
        Loc lo; lo.kind = CALLER_ACT_OUT;
        c.copy(c.tab(lo), y, b * p.h_out * p.w_out * p.d.c_out * P.esz);
      }
      part_rows = 0;
      continue;
    }
    // bf16: BN + ReLU applied inside the consuming convolutions unless the plan writes the activation out
    PtrTab shortcut{}, src{};
    bool pro = false;
    Loc lskip_in; lskip_in.kind = CALLER_SKIP_IN;
    Loc lskip_out; lskip_out.kind = CALLER_SKIP_OUT;
    if (p.j0 == 0) {
      const PtrTab x = c.tab(p.x_in);
      pro = bf && !p.mat[0];
      c.bn_fwd(p.bn[0], x, c.tab(p.a[0]), M_in, part_rows, !pro);
      // the shortcut value: x, or the projection of relu(bn1(x)); it leaves the partition if the block ends elsewhere
      const PtrTab sc_dst = p.j1 == p.nconv ? c.tab(p.y) : c.tab(lskip_out);
      if (p.proj) c.conv_fwd(p.pj, pro ? x : c.tab(p.a[0]), sc_dst, Ctx::none(), false, pro ? &p.bn[0] : nullptr);
      else if (p.j1 < p.nconv) c.copy(sc_dst, x, M_out * p.d.c_out * P.esz);
      shortcut = p.proj ? sc_dst : x;
      src = pro ? x : c.tab(p.a[0]);
    } else {
      const PtrTab in = c.tab(p.c[p.j0 - 1]);
      pro = bf && !p.mat[p.j0];
      c.bn_fwd(p.bn[p.j0], in, c.tab(p.a[p.j0]), M_out, 0, !pro);
      shortcut = c.tab(lskip_in);
      src = pro ? in : c.tab(p.a[p.j0]);
    }
    for (int j = p.j0; j < p.j1; ++j) {
      const bool last = (j == p.nconv - 1);
      const PtrTab out = last ? c.tab(p.y) : c.tab(p.c[j]);
      const bool next_resident = resident && bi + 1 < P.bp.size() && P.run_at[bi + 1] >= 0;
      const bool feeds_bn = (!last && j + 1 < p.j1) ||
                            (last && ((bi + 1 < P.bp.size() && !next_resident && takes_stats(P.bp[bi + 1])) || (bi + 1 == P.bp.size() && P.d.has_head == 1)));
      part_rows = c.conv_fwd(p.cv[j], src, out, last ? shortcut : Ctx::none(), feeds_bn, pro ? &p.bn[j] : nullptr);
      if (j + 1 < p.j1) {
        pro = bf && !p.mat[j + 1];
        c.bn_fwd(p.bn[j + 1], out, c.tab(p.a[j + 1]), M_out, part_rows, !pro);
        src = pro ? out : c.tab(p.a[j + 1]);
      }
    }
  }
  if (P.d.has_head) {
    const size_t M = b * P.out_h * P.out_w;
    c.seg_same(PROF_OTHER_FWD);
    if (P.d.has_head == 1) c.bn_fwd(P.head_bn, c.tab(P.head_x), c.tab(P.head_a), M, part_rows);
    if (c.inference) {
      Loc lo; lo.kind = CALLER_ACT_OUT;   // logits
      c.chk(launch_head_logits(P.dt, c.g, c.tab(P.head_a), c.h->params() + P.wfc_off, c.h->params() + P.bfc_off, c.tab(lo), (int)b,
                               P.out_h * P.out_w, P.out_c, P.d.num_classes, c.s),
            "head_logits");
    } else {
      c.chk(launch_head_fwd(P.dt, c.g, c.tab(P.head_a), c.h->params() + P.wfc_off, c.h->params() + P.bfc_off, labels,
                            c.tab(P.head_g), c.tab(P.head_dl), loss_accum, (int)b, P.out_h * P.out_w, P.out_c, P.d.num_classes,
                            (float)P.d.loss_divisor, c.s),
            "head_fwd");
    }
  }
  if (!c.inference && c.h->bn_momentum < 1.f && P.d.bn_mode == 0 && !P.bn_table.empty()) {
    PtrTab bases{};
    for (int i = 0; i < c.g; ++i) bases.p[i] = c.h->mb_base(c.mb0 + i);
    c.chk(launch_bn_running_update(P.dt, c.g, bases, (const BnRunDesc*)(c.h->arena + P.bn_table_off), (int)P.bn_table.size(),
                                   c.h->running(), c.h->bn_momentum, P.d.bn_eps, c.s),
          "bn_running_update");
  }
  c.seg_end();
}

void run_backward(Ctx& c) {
  const Plan& P = c.h->P;
  const size_t b = (size_t)P.d.microbatch;
  const bool deferred = (P.dt == DT_BF16);   // weight gradients after the data-gradient chain, one grouped launch
  const PtrTab tA = c.scratch(2);
  Loc lout; lout.kind = CALLER_ERR_OUT;
  // where the gradient w.r.t. the input of block `i` (= output of block i-1 / the stem) goes
  auto grad_in_loc = [&](size_t i) -> Loc {
    if (i > 0) return P.bp[i - 1].gy;
    return P.d.has_stem ? P.g_stem : lout;
  };
  c.seg_same(PROF_OTHER_BWD);
  if (P.d.has_head) {
    const size_t M = b * P.out_h * P.out_w;
    const PtrTab dst = P.d.has_head == 1 ? tA : c.tab(grad_in_loc(P.bp.size()));   // without a BatchNorm: straight to the last unit
    c.chk(launch_head_bwd(P.dt, c.g, c.tab(P.head_g), c.tab(P.head_dl), c.h->params() + P.wfc_off, c.h->grads() + P.wfc_off,
                          c.h->grads() + P.bfc_off, dst, (int)b, P.out_h * P.out_w, P.out_c, P.d.num_classes, c.s),
          "head_bwd");
    if (P.d.has_head == 1) c.bn_bwd(P.head_bn, c.tab(P.head_x), tA, Ctx::none(), c.tab(grad_in_loc(P.bp.size())), M);
  }
  for (size_t ii = P.bp.size(); ii-- > 0;) {
    if (c.h->resident() && P.run_end_at[ii] >= 0) {
      const Plan::ResRun& r = P.runs[P.run_end_at[ii]];
      c.res_backward(r);
      ii = (size_t)r.first;
      continue;
    }
    c.seg_same(PROF_OTHER_BWD);
    const BlockPlan& p = P.bp[ii];
    const size_t M_in = b * p.h_in * p.w_in, M_out = b * p.h_out * p.w_out;
    if (!p.residual()) {   // a unit of VGG-16 / ResNet-v1; the gradient operands of its convolutions keep buffers of their
                           // own when the weight gradients are deferred (fp32 mode forms them at once, from scratch tensors)
      const PtrTab x = c.tab(p.x_in), dy = c.tab(p.gy), gx = c.tab(grad_in_loc(ii));
      const PtrTab t2 = c.scratch(2);
      const PtrTab t0 = deferred && p.d.kind == K_POSTACT ? c.tab(p.dc[1]) : c.scratch(0);
      const PtrTab t1 = deferred && (p.d.kind == K_CONV_RELU || p.d.kind == K_DENSE) ? c.tab(p.dc[0])
                        : deferred && p.d.kind == K_POSTACT && p.proj ? c.tab(p.dc[2]) : c.scratch(1);
      const PtrTab t3 = deferred && p.d.kind == K_POSTACT ? c.tab(p.dc[0]) : c.scratch(3);
      const PtrTab sums = c.mbp(P.sums_off), parts = c.mbp(P.partials_off);
      float* g_bias = c.h->grads() + p.bias_off;
      if (p.d.kind == K_POSTACT) {
        const PtrTab c1 = c.tab(p.c[0]), a1 = c.tab(p.a[0]), c2 = c.tab(p.c[1]);
        // through the join: dz = dy*[y>0] (t1) feeds the shortcut, dc2 (t0) the branch
        c.chk(launch_join_bwd(P.dt, c.g, c2, c.tab(p.y), dy, c.h->params() + p.bn[1].g_off, c.mbp(p.bn[1].stats_off), (int)M_out,
                              p.bn[1].C, sums, c.h->grads() + p.bn[1].g_off, c.h->grads() + p.bn[1].b_off, parts, t0, t1,
                              P.d.bn_mode, c.s),
              "join_bwd");
        if (!deferred) c.conv_wgrad(p.cv[1], a1, t0);
        const int rows = c.conv_dgrad(p.cv[1], t0, t2, Ctx::none(), &p.bn[0], &c1);
        c.bn_bwd(p.bn[0], c1, t2, Ctx::none(), t3, M_out, rows);        // dc1
        if (!deferred) c.conv_wgrad(p.cv[0], x, t3);
        if (p.proj) {
          if (!deferred) c.conv_wgrad(p.pj, x, t1);
          c.conv_dgrad(p.pj, t1, t2, Ctx::none());                      // t2 is free again
          c.conv_dgrad(p.cv[0], t3, gx, t2);
        } else {
          c.conv_dgrad(p.cv[0], t3, gx, t1);
        }
      } else if (p.d.kind == K_CONV_RELU || p.d.kind == K_DENSE) {
        const PtrTab y0 = c.tab(p.y0);
        PtrTab d0 = dy;
        if (p.d.kind == K_CONV_RELU && p.d.stride == 2) {
          c.chk(launch_maxpool2_bwd(P.dt, c.g, y0, dy, t0, (int)b, p.h_in, p.w_in, p.d.c_out, c.s), "maxpool_bwd");
          d0 = t0;
        }
        const int rows = p.d.kind == K_DENSE ? (int)b : (int)M_in;
        c.chk(launch_bias_act_bwd(P.dt, c.g, y0, d0, t1, g_bias, rows, p.d.c_out, p.d.kind == K_DENSE ? (p.d.c_mid != 0) : 1, sums, parts, c.s),
              "bias_act_bwd");
        if (!deferred) c.conv_wgrad(p.cv[0], x, t1);
        c.conv_dgrad(p.cv[0], t1, gx, Ctx::none());
      } else if (p.d.kind == K_BN_RELU) {
        c.bn_bwd(p.bn[0], x, dy, Ctx::none(), gx, M_in);
      } else {
        c.chk(launch_bias_act_bwd(P.dt, c.g, c.tab(p.y0), dy, gx, g_bias, (int)M_in, p.d.c_in, 1, sums, parts, c.s), "bias_act_bwd");
      }
      continue;
    }
    Loc lskip_err_in; lskip_err_in.kind = CALLER_SKIP_ERR_IN;
    Loc lskip_err_out; lskip_err_out.kind = CALLER_SKIP_ERR_OUT;
    // dy: gradient w.r.t. the block output, which is also the gradient w.r.t. the shortcut value.  A block that
    // ends in a later partition receives the latter from there (copied into the arena: the deferred weight
    // gradient of the projection reads it) and starts from the gradient w.r.t. the output that left.
    const PtrTab dy = c.tab(p.gy);
    if (p.j1 < p.nconv && p.j0 == 0) c.copy(dy, c.tab(lskip_err_in), M_out * p.d.c_out * P.esz);
    PtrTab dr = p.j1 == p.nconv ? dy : c.tab(p.dc[p.j1 - 1]);
    for (int j = p.j1 - 1; j >= (p.j0 > 1 ? p.j0 : 1); --j) {
      const PtrTab xj = c.tab(p.c[j - 1]);
      if (!deferred) c.conv_wgrad(p.cv[j], c.tab(p.a[j]), dr);
      const int rows = c.conv_dgrad(p.cv[j], dr, tA, Ctx::none(), &p.bn[j], &xj);
      const PtrTab dcj = c.tab(p.dc[j - 1]);
      c.bn_bwd(p.bn[j], xj, tA, Ctx::none(), dcj, M_out, rows);
      dr = dcj;
    }
    if (p.j0 > 0) {   // the block started in an earlier partition: the gradient w.r.t. its shortcut value goes back there
      if (p.j1 == p.nconv) c.copy(c.tab(lskip_err_out), dy, M_out * p.d.c_out * P.esz);
      continue;
    }
    const PtrTab x0 = c.tab(p.x_in);
    if (!deferred) c.conv_wgrad(p.cv[0], c.tab(p.a[0]), dr);
    if (p.proj) {   // a = relu(bn1(x)) feeds the branch and the projection: the two data-gradients add
      if (!deferred) c.conv_wgrad(p.pj, c.tab(p.a[0]), dy);
      c.conv_dgrad(p.pj, dy, tA, Ctx::none());
    }
    const int rows0 = c.conv_dgrad(p.cv[0], dr, tA, p.proj ? tA : Ctx::none(), &p.bn[0], &x0);
    c.bn_bwd(p.bn[0], x0, tA, p.proj ? Ctx::none() : dy, c.tab(grad_in_loc(ii)), M_in, rows0);
  }
  c.seg_same(PROF_OTHER_BWD);
  if (P.d.has_stem && !deferred) {
    Loc in; in.kind = CALLER_ACT_IN;
    c.conv_wgrad(P.stem, c.tab(in), c.tab(P.g_stem));
  }
  if (deferred) {
    PtrTab bases{}, caller_dy{}, caller_a{};
    for (int i = 0; i < c.g; ++i) {
      bases.p[i] = c.h->mb_base(c.mb0 + i);
      caller_dy.p[i] = const_cast<void*>(c.err_in[i]);
      caller_a.p[i] = const_cast<void*>(c.act_in[i]);
    }
    const bool res = c.h->resident();
    if (res)
      for (const Plan::ResRun& r : P.runs)
        if (resident_has_wgrad_launch(r.kind, r.C, r.bands)) c.res_wgrad(r);
    for (int k = 0; k < WGRAD_CLASSES; ++k) {
      const std::vector<WgradItem>& items = res ? P.items_nr[k] : P.items[k];
      if (items.empty()) continue;
      c.seg(PROF_WGRAD, c.g * (res ? P.wg_nr_bytes : P.wg_bytes)[k], c.g * (res ? P.wg_nr_flops : P.wg_flops)[k]);
      c.chk(launch_wgrad_grouped(k, c.g, (const WgradItem*)(c.h->arena + (res ? P.items_nr_off : P.items_off)[k]), (int)items.size(),
                                 bases, caller_dy, caller_a, c.h->params(), c.h->grads(), c.s,
                                 k == WGRAD_CLASS_T9 ? wgrad_t9_lds_bytes(P.t9_h, P.t9_w) : 0),
            "wgrad_grouped");
    }
  }
  c.seg_end();
}

bool all_backward_done(const hpf_partition* p) { return p->n_bwd == p->P.d.num_microbatches; }

bool stream_is_capturing(hipStream_t s) {
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  return s != nullptr && hipStreamIsCapturing(s, &cs) == hipSuccess && cs != hipStreamCaptureStatusNone;
}
// Work queued on one stream runs in the order of the calls, so only a wait across streams needs a marker in
// the queue (each costs a few microseconds of stream time).  A stream under capture always gets the wait.
hpf_status wait_for(hipStream_t s, hipEvent_t ev, hipStream_t recorded_on) {
  if (recorded_on == s && !stream_is_capturing(s)) return HPF_OK;
  if (hipStreamWaitEvent(s, ev, 0) != hipSuccess) return fail(HPF_EDEVICE, "hipStreamWaitEvent failed");
  return HPF_OK;
}

hpf_status wait_all_backward(hpf_partition* p, hipStream_t s) {
  for (int i = 0; i < p->P.d.num_microbatches; ++i)
    if (p->bwd_done[i] && p->bwd_ev[i] == i) {
      const hpf_status st = wait_for(s, p->ev_bwd[i], p->bwd_stream[i]);
      if (st != HPF_OK) return st;
    }
  return HPF_OK;
}

// Runs `body` (kernel launches on stream s only) through a HIP graph: replayed if one captured with the
// same caller pointers exists, captured and instantiated first otherwise.  The sequences contain kernel
// nodes only.  Falls back to direct launches when graphs are off or the stream is already capturing.
template <class Body>
hpf_status run_graphed(hpf_partition* p, GraphSlot& slot, const std::vector<const void*>& key, hipStream_t s, Ctx& c, Body body) {
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  // the default (NULL) stream cannot be captured
  if (!p->use_graphs || p->profiling || s == nullptr || hipStreamIsCapturing(s, &cs) != hipSuccess || cs != hipStreamCaptureStatusNone) {
    body();
    return c.err == hipSuccess ? HPF_OK : fail(HPF_EDEVICE, "%s: %s", c.where, hipGetErrorString(c.err));
  }
  if (slot.direct && slot.key == key) {
    body();
    return c.err == hipSuccess ? HPF_OK : fail(HPF_EDEVICE, "%s: %s", c.where, hipGetErrorString(c.err));
  }
  const bool hit = slot.exec && slot.key == key;
  if (!hit) {
    slot.direct = false;
    if (slot.exec) { (void)hipGraphExecDestroy(slot.exec); slot.exec = nullptr; }
    hipGraph_t graph = nullptr;
    if (hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal) != hipSuccess) return fail(HPF_EDEVICE, "hipStreamBeginCapture failed");
    body();
    const hipError_t e = hipStreamEndCapture(s, &graph);
    if (c.err != hipSuccess || e != hipSuccess || !graph) {
      if (graph) (void)hipGraphDestroy(graph);
      return fail(HPF_EDEVICE, "graph capture failed: %s: %s", c.where, hipGetErrorString(c.err != hipSuccess ? c.err : e));
    }
    slot.key = key;
    if (c.n_launches < kMinGraphLaunches) {   // capture recorded the launches without running them: run them now
      (void)hipGraphDestroy(graph);
      slot.direct = true;
      c.n_launches = 0;
      body();
      return c.err == hipSuccess ? HPF_OK : fail(HPF_EDEVICE, "%s: %s", c.where, hipGetErrorString(c.err));
    }
    const hipError_t ei = hipGraphInstantiate(&slot.exec, graph, nullptr, nullptr, 0);
    (void)hipGraphDestroy(graph);
    if (ei != hipSuccess) { slot.exec = nullptr; return fail(HPF_EDEVICE, "hipGraphInstantiate: %s", hipGetErrorString(ei)); }
  }
  if (hipGraphLaunch(slot.exec, s) != hipSuccess) return fail(HPF_EDEVICE, "hipGraphLaunch failed");
  return HPF_OK;
}

// Image-resident kernels need every work-group of a launch on the chip at once and take a CU each, so two
// of them must never share the device: launches of this process are chained through one event.
// The link of the chain is the completion event the last such call recorded anyway (its owner re-records it
// only after a later launch of its own, so waiting on it never waits for too little).
std::mutex g_res_mu;
struct ResidentLink { hipEvent_t ev = nullptr; hipStream_t stream = nullptr; const hpf_partition* owner = nullptr; } g_res;

// Launches of this kind are ordered against each other through events recorded at call time, which a stream under
// capture by the caller cannot take part in: two captured partitions replayed side by side would each wait for CUs
// the other holds.  Such calls are refused instead.
const char* const kNoCaptureMsg =
    "image-resident launches (fusion level 2) cannot be recorded into a caller's graph capture: call "
    "hpf_partition_set_fusion(p, 1) for partitions whose calls are captured";

hpf_status resident_enter(hpf_partition* p, hipStream_t s) {
  if (!p->resident()) return HPF_OK;
  std::lock_guard<std::mutex> lk(g_res_mu);
  return g_res.owner ? wait_for(s, g_res.ev, g_res.stream) : HPF_OK;
}
// done: the event recorded on s after the call's last launch
void resident_leave(hpf_partition* p, hipStream_t s, hipEvent_t done) {
  if (!p->resident()) return;
  std::lock_guard<std::mutex> lk(g_res_mu);
  g_res.ev = done; g_res.stream = s; g_res.owner = p;
}
void resident_forget(const hpf_partition* p) {   // the partition's events are about to be destroyed (device idle)
  std::lock_guard<std::mutex> lk(g_res_mu);
  if (g_res.owner == p) g_res = ResidentLink{};
}
// An exchange between the work-groups of an image-resident launch timed out: the batch is invalid.
hpf_status check_abort_flag(hpf_partition* p) {
  if (p->P.runs.empty()) return HPF_OK;
  int flag = 0;
  if (hipMemcpy(&flag, p->abort_flag(), sizeof(int), hipMemcpyDeviceToHost) != hipSuccess) return fail(HPF_EDEVICE, "device-to-host copy failed");
  if (flag) return fail(HPF_EDEVICE, "an image-resident launch timed out waiting for its partner work-groups");
  return HPF_OK;
}

void begin_next_batch(hpf_partition* p, hipStream_t s) {
  std::fill(p->fwd_done.begin(), p->fwd_done.end(), 0);
  std::fill(p->bwd_done.begin(), p->bwd_done.end(), 0);
  p->n_bwd = 0;
  (void)hipEventRecord(p->ev_step, s);
  p->step_recorded = true;
  p->step_stream = s;
}

}  // namespace

extern "C" {

const char* hpf_last_error(void) { return g_err; }

hpf_status hpf_partition_sizes(const hpf_partition_desc* desc, hpf_sizes* out) {
  if (!out) return fail(HPF_EINVAL, "null output");
  Plan P;
  const hpf_status st = build_plan(desc, P);
  if (st != HPF_OK) return st;
  out->n_params = P.n_params;
  out->arena_bytes = P.arena_bytes;
  out->stash_bytes = P.stash_bytes_per_mb * (size_t)P.d.num_microbatches;
  out->act_in_elems = P.act_in_elems;
  out->act_out_elems = P.act_out_elems;
  out->skip_in_elems = P.skip_in_elems;
  out->skip_out_elems = P.skip_out_elems;
  out->n_bn_running = P.n_running;
  return HPF_OK;
}

hpf_status hpf_partition_create(const hpf_partition_desc* desc, void* device_arena, size_t arena_bytes,
                                const float* host_params, hpf_partition** out) {
  if (!out) return fail(HPF_EINVAL, "null output");
  *out = nullptr;
  if (!device_arena || !host_params) return fail(HPF_EINVAL, "null arena or parameters");
  if ((uintptr_t)device_arena % ALIGN) return fail(HPF_EINVAL, "arena must be %zu-byte aligned", ALIGN);
  hpf_partition* p = new (std::nothrow) hpf_partition();
  if (!p) return fail(HPF_ENOMEM, "host allocation failed");
  hpf_status st = build_plan(desc, p->P);
  if (st != HPF_OK) { delete p; return st; }
  if (arena_bytes < p->P.arena_bytes) {
    const size_t need = p->P.arena_bytes;
    delete p;
    return fail(HPF_ENOMEM, "arena has %zu bytes, %zu needed", arena_bytes, need);
  }
  p->arena = (char*)device_arena;
  const Plan& P = p->P;
  const int m = P.d.num_microbatches;
  p->fwd_done.assign(m, 0); p->bwd_done.assign(m, 0); p->act_in.assign(m, nullptr);
  p->g_fwd.resize(m); p->g_bwd.resize(m);
  hipError_t e = hipSuccess;
  auto ok = [&](hipError_t r) { if (e == hipSuccess) e = r; };
  ok(hipMemcpy(p->params(), host_params, P.n_params * sizeof(float), hipMemcpyHostToDevice));
  ok(hipMemset(p->grads(), 0, P.n_params * sizeof(float)));
  ok(hipMemset(p->mom(), 0, P.n_params * sizeof(float)));
  for (int i = 0; i < m; ++i) ok(hipMemset(p->mb_base(i) + P.tickets_off, 0, 64 * sizeof(unsigned)));
  if (!P.table.empty()) {
    ok(hipMemcpy(p->arena + P.table_off, P.table.data(), P.table.size() * sizeof(PackDesc), hipMemcpyHostToDevice));
    ok(launch_pack_weights(p->params(), p->packed(), (const PackDesc*)(p->arena + P.table_off), P.n_convs, P.pack_max_elems(), nullptr));
  }
  for (int k = 0; k < WGRAD_CLASSES; ++k)
    if (!P.items[k].empty())
      ok(hipMemcpy(p->arena + P.items_off[k], P.items[k].data(), P.items[k].size() * sizeof(WgradItem), hipMemcpyHostToDevice));
  for (int k = 0; k < WGRAD_CLASSES; ++k)
    if (!P.items_nr[k].empty())
      ok(hipMemcpy(p->arena + P.items_nr_off[k], P.items_nr[k].data(), P.items_nr[k].size() * sizeof(WgradItem), hipMemcpyHostToDevice));
  ok(conv_prepare());
  if (P.n_running) {
    std::vector<float> r0(P.n_running, 0.f);
    for (const BnRunDesc& d : P.bn_table) for (int c = 0; c < d.C; ++c) r0[(size_t)d.run_off + d.C + c] = 1.f;
    ok(hipMemcpy(p->running(), r0.data(), P.n_running * sizeof(float), hipMemcpyHostToDevice));
    ok(hipMemcpy(p->arena + P.bn_table_off, P.bn_table.data(), P.bn_table.size() * sizeof(BnRunDesc), hipMemcpyHostToDevice));
  }
  if (!P.items[9].empty() || !P.items[WGRAD_CLASS_T9].empty()) ok(wgrad_prepare());
  if (!P.runs.empty()) {
    ok(hipMemcpy(p->arena + P.res_off, P.res_blocks.data(), P.res_blocks.size() * sizeof(ResBlock), hipMemcpyHostToDevice));
    ok(hipMemset(p->abort_flag(), 0, sizeof(int)));
    for (int i = 0; i < m; ++i) {
      ok(hipMemset(p->mb_base(i) + P.xchg_off, 0, P.tag_off - P.xchg_off));
      ok(hipMemset(p->mb_base(i) + P.tag_off, 0, sizeof(unsigned)));
    }
    int max_bands = 1;
    for (const Plan::ResRun& r : P.runs) max_bands = std::max(max_bands, r.bands);
    p->res_group = resident_max_group(P.d.microbatch * max_bands);
    if (p->res_group >= 1) ok(resident_prepare());
  }
  p->ev_fwd.resize(m); p->ev_bwd.resize(m);
  p->fwd_ev.assign(m, 0); p->bwd_ev.assign(m, 0);
  p->fwd_stream.assign(m, nullptr); p->bwd_stream.assign(m, nullptr);
  for (int i = 0; i < m; ++i) { p->fwd_ev[i] = i; p->bwd_ev[i] = i; }
  for (int i = 0; i < m; ++i) {
    ok(hipEventCreateWithFlags(&p->ev_fwd[i], hipEventDisableTiming));
    ok(hipEventCreateWithFlags(&p->ev_bwd[i], hipEventDisableTiming));
  }
  ok(hipEventCreateWithFlags(&p->ev_step, hipEventDisableTiming));
  ok(hipEventCreateWithFlags(&p->ev_run, hipEventDisableTiming));
  ok(hipDeviceSynchronize());
  if (e != hipSuccess) {
    st = fail(HPF_EDEVICE, "create: %s", hipGetErrorString(e));
    hpf_partition_destroy(p);
    return st;
  }
  *out = p;
  return HPF_OK;
}

void hpf_partition_destroy(hpf_partition* p) {
  if (!p) return;
  (void)hipDeviceSynchronize();
  resident_forget(p);
  for (hipEvent_t ev : p->ev_fwd) if (ev) (void)hipEventDestroy(ev);
  for (hipEvent_t ev : p->ev_bwd) if (ev) (void)hipEventDestroy(ev);
  if (p->ev_step) (void)hipEventDestroy(p->ev_step);
  if (p->ev_run) (void)hipEventDestroy(p->ev_run);
  for (auto& sg : p->prof_pending) { (void)hipEventDestroy(sg.e0); (void)hipEventDestroy(sg.e1); }
  for (hipEvent_t ev : p->ev_pool) (void)hipEventDestroy(ev);
  for (GraphSlot& g : p->g_fwd) if (g.exec) (void)hipGraphExecDestroy(g.exec);
  for (GraphSlot& g : p->g_bwd) if (g.exec) (void)hipGraphExecDestroy(g.exec);
  for (GraphSlot& g : p->g_inf) if (g.exec) (void)hipGraphExecDestroy(g.exec);
  delete p;
}

}  // extern "C"

namespace {

// skip_in / skip_out: arrays like act_in / act_out for the shortcut value of a cut block, or NULL
hpf_status forward_group(hpf_partition* p, int32_t mb_first, int32_t count, const void* const* act_in, const void* const* skip_in,
                         const int32_t* const* labels, void* const* act_out, void* const* skip_out, float* loss_accum,
                         void* hip_stream) {
  if (!p) return fail(HPF_EINVAL, "null handle");
  const Plan& P = p->P;
  if (P.skip_in_elems && !skip_in) return fail(HPF_EINVAL, "the first block starts after its first convolution: skip_in is required (hpf_forward_microbatch_cut)");
  if (P.skip_out_elems && !skip_out) return fail(HPF_EINVAL, "the last block ends in a later partition: skip_out is required (hpf_forward_microbatch_cut)");
  for (int i = 0; i < count && count >= 1; ++i) {
    if (P.skip_in_elems && !skip_in[i]) return fail(HPF_EINVAL, "skip_in[%d] is null", i);
    if (P.skip_out_elems && !skip_out[i]) return fail(HPF_EINVAL, "skip_out[%d] is null", i);
  }
  if (count < 1 || mb_first < 0 || mb_first + count > P.d.num_microbatches)
    return fail(HPF_EINVAL, "micro-batches [%d, %d) out of range", mb_first, mb_first + count);
  if (!act_in) return fail(HPF_EINVAL, "act_in is required");
  if (P.d.has_head && (!labels || !loss_accum)) return fail(HPF_EINVAL, "labels and loss_accum are required with a head");
  if (!P.d.has_head && !act_out) return fail(HPF_EINVAL, "act_out is required without a head");
  for (int i = 0; i < count; ++i) {
    if (!act_in[i]) return fail(HPF_EINVAL, "act_in[%d] is null", i);
    if (P.d.has_head && !labels[i]) return fail(HPF_EINVAL, "labels[%d] is null", i);
    if (!P.d.has_head && !act_out[i]) return fail(HPF_EINVAL, "act_out[%d] is null", i);
    if (p->fwd_done[mb_first + i]) return fail(HPF_ESTATE, "forward(%d) already ran in this batch", mb_first + i);
  }
  hipStream_t s = (hipStream_t)hip_stream;
  if (p->resident() && stream_is_capturing(s)) return fail(HPF_EUNSUPPORTED, kNoCaptureMsg);
  if (p->step_recorded) {
    const hpf_status st = wait_for(s, p->ev_step, p->step_stream);
    if (st != HPF_OK) return st;
  }
  const int gmax = p->group_limit();
  {
    const hpf_status st = resident_enter(p, s);
    if (st != HPF_OK) return st;
  }
  for (int c0 = 0; c0 < count; c0 += gmax) {
    const int g = count - c0 < gmax ? count - c0 : gmax;
    Ctx c{p, mb_first + c0, g, s};
    PtrTab lab{};
    std::vector<const void*> key;
    key.push_back((const void*)(intptr_t)g);
    key.push_back(loss_accum);
    for (int i = 0; i < g; ++i) {
      c.act_in[i] = act_in[c0 + i];
      c.act_out[i] = P.d.has_head ? nullptr : act_out[c0 + i];
      c.err_in[i] = nullptr; c.err_out[i] = nullptr;
      lab.p[i] = P.d.has_head ? const_cast<int32_t*>(labels[c0 + i]) : nullptr;
      c.skip_in[i] = P.skip_in_elems ? skip_in[c0 + i] : nullptr;
      c.skip_out[i] = P.skip_out_elems ? skip_out[c0 + i] : nullptr;
      key.push_back(c.act_in[i]); key.push_back(c.act_out[i]); key.push_back(lab.p[i]);
      key.push_back(c.skip_in[i]); key.push_back(c.skip_out[i]);
    }
    // forwards that move the running statistics read and write the same buffers: chain them in call order
    const bool moves_running = p->bn_momentum < 1.f && P.d.bn_mode == 0 && P.n_running > 0 && !stream_is_capturing(s);
    if (moves_running && p->run_recorded) {
      const hpf_status st = wait_for(s, p->ev_run, p->run_stream);
      if (st != HPF_OK) return st;
    }
    const hpf_status st = run_graphed(p, p->g_fwd[mb_first + c0], key, s, c, [&] { run_forward(c, lab, loss_accum); });
    if (st != HPF_OK) return st;
    if (moves_running) {
      if (hipEventRecord(p->ev_run, s) != hipSuccess) return fail(HPF_EDEVICE, "hipEventRecord failed");
      p->run_recorded = true;
      p->run_stream = s;
    }
    if (hipEventRecord(p->ev_fwd[mb_first + c0], s) != hipSuccess) return fail(HPF_EDEVICE, "hipEventRecord failed");
    for (int i = 0; i < g; ++i) {
      const int mb = mb_first + c0 + i;
      p->fwd_ev[mb] = mb_first + c0;
      p->act_in[mb] = c.act_in[i];
      p->fwd_done[mb] = 1;
    }
    p->fwd_stream[mb_first + c0] = s;
    resident_leave(p, s, p->ev_fwd[mb_first + c0]);
  }
  return HPF_OK;
}

// skip_err_in: gradient w.r.t. skip_out (from the partition that took it); skip_err_out: gradient w.r.t. skip_in
hpf_status backward_group(hpf_partition* p, int32_t mb_first, int32_t count, const void* const* err_in, const void* const* skip_err_in,
                          void* const* err_out, void* const* skip_err_out, void* hip_stream) {
  if (!p) return fail(HPF_EINVAL, "null handle");
  const Plan& P = p->P;
  if (P.skip_out_elems && !skip_err_in) return fail(HPF_EINVAL, "the last block ends in a later partition: skip_err_in is required (hpf_backward_microbatch_cut)");
  if (P.skip_in_elems && !skip_err_out) return fail(HPF_EINVAL, "the first block starts after its first convolution: skip_err_out is required (hpf_backward_microbatch_cut)");
  for (int i = 0; i < count && count >= 1; ++i) {
    if (P.skip_out_elems && !skip_err_in[i]) return fail(HPF_EINVAL, "skip_err_in[%d] is null", i);
    if (P.skip_in_elems && !skip_err_out[i]) return fail(HPF_EINVAL, "skip_err_out[%d] is null", i);
  }
  if (count < 1 || mb_first < 0 || mb_first + count > P.d.num_microbatches)
    return fail(HPF_EINVAL, "micro-batches [%d, %d) out of range", mb_first, mb_first + count);
  if (!P.d.has_head && !err_in) return fail(HPF_EINVAL, "err_in is required without a head");
  if (!P.d.has_stem && !err_out) return fail(HPF_EINVAL, "err_out is required");
  for (int i = 0; i < count; ++i) {
    const int mb = mb_first + i;
    if (!P.d.has_head && !err_in[i]) return fail(HPF_EINVAL, "err_in[%d] is null", i);
    if (P.d.has_stem && err_out && err_out[i]) return fail(HPF_EINVAL, "err_out must be NULL for the partition that holds the stem");
    if (!P.d.has_stem && !err_out[i]) return fail(HPF_EINVAL, "err_out[%d] is null", i);
    if (!p->fwd_done[mb]) return fail(HPF_ESTATE, "backward(%d) before forward(%d)", mb, mb);
    if (p->bwd_done[mb]) return fail(HPF_ESTATE, "backward(%d) already ran in this batch", mb);
  }
  hipStream_t s = (hipStream_t)hip_stream;
  if (p->resident() && stream_is_capturing(s)) return fail(HPF_EUNSUPPORTED, kNoCaptureMsg);
  for (int i = 0; i < count; ++i)
    if (i == 0 || p->fwd_ev[mb_first + i] != p->fwd_ev[mb_first + i - 1]) {
      const int lead = p->fwd_ev[mb_first + i];
      const hpf_status st = wait_for(s, p->ev_fwd[lead], p->fwd_stream[lead]);
      if (st != HPF_OK) return st;
    }
  const int gmax = p->group_limit();
  {
    const hpf_status st = resident_enter(p, s);
    if (st != HPF_OK) return st;
  }
  for (int c0 = 0; c0 < count; c0 += gmax) {
    const int g = count - c0 < gmax ? count - c0 : gmax;
    Ctx c{p, mb_first + c0, g, s};
    std::vector<const void*> key;
    key.push_back((const void*)(intptr_t)g);
    for (int i = 0; i < g; ++i) {
      c.act_in[i] = p->act_in[mb_first + c0 + i];
      c.act_out[i] = nullptr;
      c.err_in[i] = P.d.has_head ? nullptr : err_in[c0 + i];
      c.err_out[i] = P.d.has_stem ? nullptr : err_out[c0 + i];
      c.skip_err_in[i] = P.skip_out_elems ? skip_err_in[c0 + i] : nullptr;
      c.skip_err_out[i] = P.skip_in_elems ? skip_err_out[c0 + i] : nullptr;
      key.push_back(c.act_in[i]); key.push_back(c.err_in[i]); key.push_back(c.err_out[i]);
      key.push_back(c.skip_err_in[i]); key.push_back(c.skip_err_out[i]);
    }
    const hpf_status st = run_graphed(p, p->g_bwd[mb_first + c0], key, s, c, [&] { run_backward(c); });
    if (st != HPF_OK) return st;
    if (hipEventRecord(p->ev_bwd[mb_first + c0], s) != hipSuccess) return fail(HPF_EDEVICE, "hipEventRecord failed");
    for (int i = 0; i < g; ++i) {
      const int mb = mb_first + c0 + i;
      p->bwd_ev[mb] = mb_first + c0;
      p->bwd_done[mb] = 1;
      ++p->n_bwd;
    }
    p->bwd_stream[mb_first + c0] = s;
    resident_leave(p, s, p->ev_bwd[mb_first + c0]);
  }
  return HPF_OK;
}

}  // namespace

extern "C" {

hpf_status hpf_forward_microbatches(hpf_partition* p, int32_t mb_first, int32_t count, const void* const* act_in,
                                   const int32_t* const* labels, void* const* act_out, float* loss_accum, void* hip_stream) {
  return forward_group(p, mb_first, count, act_in, nullptr, labels, act_out, nullptr, loss_accum, hip_stream);
}

hpf_status hpf_backward_microbatches(hpf_partition* p, int32_t mb_first, int32_t count, const void* const* err_in,
                                    void* const* err_out, void* hip_stream) {
  return backward_group(p, mb_first, count, err_in, nullptr, err_out, nullptr, hip_stream);
}

hpf_status hpf_forward_microbatch_cut(hpf_partition* p, int32_t mb, const void* act_in, const void* skip_in, const int32_t* labels,
                                      void* act_out, void* skip_out, float* loss_accum, void* hip_stream) {
  if (p && p->P.d.has_head && !labels) return fail(HPF_EINVAL, "labels and loss_accum are required with a head");
  if (p && !p->P.d.has_head && !act_out) return fail(HPF_EINVAL, "act_out is required without a head");
  if (!act_in) return fail(HPF_EINVAL, "act_in is required");
  if (p && !p->P.skip_in_elems && skip_in) return fail(HPF_EINVAL, "skip_in given, but the first block starts at its first convolution");
  if (p && !p->P.skip_out_elems && skip_out) return fail(HPF_EINVAL, "skip_out given, but the last block ends here");
  return forward_group(p, mb, 1, &act_in, &skip_in, &labels, &act_out, &skip_out, loss_accum, hip_stream);
}

hpf_status hpf_backward_microbatch_cut(hpf_partition* p, int32_t mb, const void* err_in, const void* skip_err_in, void* err_out,
                                       void* skip_err_out, void* hip_stream) {
  if (p && !p->P.d.has_head && !err_in) return fail(HPF_EINVAL, "err_in is required without a head");
  if (p && !p->P.d.has_stem && !err_out) return fail(HPF_EINVAL, "err_out is required");
  if (p && p->P.d.has_stem && err_out) return fail(HPF_EINVAL, "err_out must be NULL for the partition that holds the stem");
  if (p && !p->P.skip_out_elems && skip_err_in) return fail(HPF_EINVAL, "skip_err_in given, but the last block ends here");
  if (p && !p->P.skip_in_elems && skip_err_out) return fail(HPF_EINVAL, "skip_err_out given, but the first block starts at its first convolution");
  return backward_group(p, mb, 1, &err_in, &skip_err_in, &err_out, &skip_err_out, hip_stream);
}

hpf_status hpf_forward_microbatch(hpf_partition* p, int32_t mb, const void* act_in, const int32_t* labels, void* act_out,
                                  float* loss_accum, void* hip_stream) {
  if (p && p->P.d.has_head && !labels) return fail(HPF_EINVAL, "labels and loss_accum are required with a head");
  if (p && !p->P.d.has_head && !act_out) return fail(HPF_EINVAL, "act_out is required without a head");
  if (!act_in) return fail(HPF_EINVAL, "act_in is required");
  return hpf_forward_microbatches(p, mb, 1, &act_in, &labels, &act_out, loss_accum, hip_stream);
}

hpf_status hpf_backward_microbatch(hpf_partition* p, int32_t mb, const void* err_in, void* err_out, void* hip_stream) {
  if (p && !p->P.d.has_head && !err_in) return fail(HPF_EINVAL, "err_in is required without a head");
  if (p && !p->P.d.has_stem && !err_out) return fail(HPF_EINVAL, "err_out is required");
  if (p && p->P.d.has_stem && err_out) return fail(HPF_EINVAL, "err_out must be NULL for the partition that holds the stem");
  return hpf_backward_microbatches(p, mb, 1, &err_in, &err_out, hip_stream);
}

hpf_status hpf_grad_accum_read(hpf_partition* p, float* dst, size_t n_floats, int32_t dst_is_device, void* hip_stream) {
  if (!p || !dst) return fail(HPF_EINVAL, "null argument");
  if (n_floats != p->P.n_params) return fail(HPF_EINVAL, "n_floats %zu, expected %zu", n_floats, p->P.n_params);
  if (!all_backward_done(p)) return fail(HPF_ESTATE, "gradients read before all micro-batches ran backward");
  hipStream_t s = (hipStream_t)hip_stream;
  const hpf_status st = wait_all_backward(p, s);
  if (st != HPF_OK) return st;
  if (dst_is_device) {
    if (launch_copy_bytes(dst, p->grads(), n_floats * sizeof(float), s) != hipSuccess) return fail(HPF_EDEVICE, "copy failed");
    return HPF_OK;
  }
  if (hipMemcpyAsync(dst, p->grads(), n_floats * sizeof(float), hipMemcpyDeviceToHost, s) != hipSuccess ||
      hipStreamSynchronize(s) != hipSuccess)
    return fail(HPF_EDEVICE, "device-to-host copy failed: %s", hipGetErrorString(hipGetLastError()));
  return check_abort_flag(p);
}

hpf_status hpf_grad_accum_zero(hpf_partition* p, void* hip_stream) {
  if (!p) return fail(HPF_EINVAL, "null handle");
  for (int i = 0; i < p->P.d.num_microbatches; ++i)
    if (p->fwd_done[i] && !p->bwd_done[i]) return fail(HPF_ESTATE, "micro-batch %d is between forward and backward", i);
  hipStream_t s = (hipStream_t)hip_stream;
  const hpf_status st = wait_all_backward(p, s);
  if (st != HPF_OK) return st;
  if (launch_zero_f32(p->grads(), p->P.n_params, s) != hipSuccess) return fail(HPF_EDEVICE, "zero failed");
  begin_next_batch(p, s);
  return HPF_OK;
}

hpf_status hpf_sgd_step(hpf_partition* p, float lr, float momentum, void* hip_stream) {
  if (!p) return fail(HPF_EINVAL, "null handle");
  if (!all_backward_done(p)) return fail(HPF_ESTATE, "sgd_step before all micro-batches ran backward");
  hipStream_t s = (hipStream_t)hip_stream;
  const hpf_status st = wait_all_backward(p, s);
  if (st != HPF_OK) return st;
  const Plan& P = p->P;
  // a batch whose image-resident launches timed out has no valid gradients: the kernel then leaves everything alone
  if (launch_sgd(p->params(), p->mom(), p->grads(), P.n_params, lr, momentum, P.runs.empty() ? nullptr : p->abort_flag(), s) != hipSuccess)
    return fail(HPF_EDEVICE, "sgd failed");
  if (launch_pack_weights(p->params(), p->packed(), (const PackDesc*)(p->arena + P.table_off), P.n_convs, P.pack_max_elems(), s) != hipSuccess)
    return fail(HPF_EDEVICE, "pack failed");
  begin_next_batch(p, s);
  return HPF_OK;
}

hpf_status hpf_partition_set_graphs(hpf_partition* p, int32_t enable) {
  if (!p) return fail(HPF_EINVAL, "null handle");
  p->use_graphs = enable != 0;
  return HPF_OK;
}

hpf_status hpf_partition_set_fusion(hpf_partition* p, int32_t enable) {
  if (!p) return fail(HPF_EINVAL, "null handle");
  if (enable < 0 || enable > 2) return fail(HPF_EINVAL, "fusion level %d (0, 1 or 2)", enable);
  for (int i = 0; i < p->P.d.num_microbatches; ++i)
    if (p->fwd_done[i] && !p->bwd_done[i]) return fail(HPF_ESTATE, "micro-batch %d is between forward and backward", i);
  if (p->fuse != enable) {   // cached graphs hold the other kernel sequence
    for (GraphSlot& g : p->g_fwd) { if (g.exec) (void)hipGraphExecDestroy(g.exec); g.exec = nullptr; g.direct = false; g.key.clear(); }
    for (GraphSlot& g : p->g_bwd) { if (g.exec) (void)hipGraphExecDestroy(g.exec); g.exec = nullptr; g.direct = false; g.key.clear(); }
    for (GraphSlot& g : p->g_inf) { if (g.exec) (void)hipGraphExecDestroy(g.exec); g.exec = nullptr; g.direct = false; g.key.clear(); }
  }
  p->fuse = enable;
  return HPF_OK;
}

hpf_status hpf_partition_set_bn_momentum(hpf_partition* p, float momentum) {
  if (!p) return fail(HPF_EINVAL, "null handle");
  if (!(momentum >= 0.f && momentum <= 1.f)) return fail(HPF_EINVAL, "momentum %g outside [0, 1]", (double)momentum);
  for (int i = 0; i < p->P.d.num_microbatches; ++i)
    if (p->fwd_done[i] && !p->bwd_done[i]) return fail(HPF_ESTATE, "micro-batch %d is between forward and backward", i);
  if (p->bn_momentum != momentum) {   // cached graphs hold the other kernel sequence / the old factor
    for (GraphSlot& g : p->g_fwd) { if (g.exec) (void)hipGraphExecDestroy(g.exec); g.exec = nullptr; g.direct = false; g.key.clear(); }
  }
  p->bn_momentum = momentum;
  return HPF_OK;
}

hpf_status hpf_bn_running_read(hpf_partition* p, float* host_dst, size_t n_floats) {
  if (!p || (!host_dst && n_floats)) return fail(HPF_EINVAL, "null argument");
  if (n_floats != p->P.n_running) return fail(HPF_EINVAL, "n_floats %zu, expected %zu", n_floats, p->P.n_running);
  if (hipDeviceSynchronize() != hipSuccess) return fail(HPF_EDEVICE, "synchronize failed");
  if (n_floats && hipMemcpy(host_dst, p->running(), n_floats * sizeof(float), hipMemcpyDeviceToHost) != hipSuccess)
    return fail(HPF_EDEVICE, "device-to-host copy failed");
  return check_abort_flag(p);
}

hpf_status hpf_bn_running_write(hpf_partition* p, const float* host_src, size_t n_floats) {
  if (!p || (!host_src && n_floats)) return fail(HPF_EINVAL, "null argument");
  if (n_floats != p->P.n_running) return fail(HPF_EINVAL, "n_floats %zu, expected %zu", n_floats, p->P.n_running);
  for (const BnRunDesc& d : p->P.bn_table)
    for (int c = 0; c < d.C; ++c)
      if (!(host_src[(size_t)d.run_off + d.C + c] >= 0.f)) return fail(HPF_EINVAL, "negative running variance");
  if (hipDeviceSynchronize() != hipSuccess) return fail(HPF_EDEVICE, "synchronize failed");
  if (n_floats && hipMemcpy(p->running(), host_src, n_floats * sizeof(float), hipMemcpyHostToDevice) != hipSuccess)
    return fail(HPF_EDEVICE, "host-to-device copy failed");
  return HPF_OK;
}

hpf_status hpf_forward_inference_group(hpf_partition* p, int32_t count, const void* const* act_in, const void* const* skip_in,
                                       void* const* out, void* const* skip_out, void* hip_stream) {
  if (!p) return fail(HPF_EINVAL, "null handle");
  const Plan& P = p->P;
  const int cmax = P.d.num_microbatches < MAX_GROUP ? P.d.num_microbatches : MAX_GROUP;
  if (count < 1 || count > cmax) return fail(HPF_EINVAL, "count %d outside [1, %d]", count, cmax);
  if (!act_in || !out) return fail(HPF_EINVAL, "act_in and out are required");
  if ((P.skip_in_elems != 0) != (skip_in != nullptr)) return fail(HPF_EINVAL, "skip_in is required exactly when the first block starts after its first convolution");
  if ((P.skip_out_elems != 0) != (skip_out != nullptr)) return fail(HPF_EINVAL, "skip_out is required exactly when the last block ends in a later partition");
  for (int i = 0; i < count; ++i)
    if (!act_in[i] || !out[i] || (skip_in && !skip_in[i]) || (skip_out && !skip_out[i])) return fail(HPF_EINVAL, "null tensor for member %d", i);
  for (int i = 0; i < P.d.num_microbatches; ++i)   // the pass works in the regions of micro-batches 0 .. count-1
    if (p->fwd_done[i] && !p->bwd_done[i]) return fail(HPF_ESTATE, "micro-batch %d is between forward and backward", i);
  hipStream_t s = (hipStream_t)hip_stream;
  if (p->step_recorded) {
    const hpf_status st = wait_for(s, p->ev_step, p->step_stream);
    if (st != HPF_OK) return st;
  }
  hpf_status st = wait_all_backward(p, s);
  if (st != HPF_OK) return st;
  Ctx c{p, 0, count, s};
  c.inference = true;
  std::vector<const void*> key;
  key.push_back((const void*)(intptr_t)count);
  for (int i = 0; i < count; ++i) {
    c.act_in[i] = act_in[i]; c.act_out[i] = out[i]; c.err_in[i] = nullptr; c.err_out[i] = nullptr;
    c.skip_in[i] = skip_in ? skip_in[i] : nullptr; c.skip_out[i] = skip_out ? skip_out[i] : nullptr;
    key.push_back(c.act_in[i]); key.push_back(c.act_out[i]); key.push_back(c.skip_in[i]); key.push_back(c.skip_out[i]);
  }
  GraphSlot* slot = nullptr;
  for (GraphSlot& g : p->g_inf) if (g.key == key) slot = &g;
  if (!slot) { slot = &p->g_inf[p->g_inf_next]; p->g_inf_next = (p->g_inf_next + 1) % 8; }
  st = run_graphed(p, *slot, key, s, c, [&] { run_forward(c, PtrTab{}, nullptr); });
  if (st != HPF_OK) return st;
  if (hipEventRecord(p->ev_step, s) != hipSuccess) return fail(HPF_EDEVICE, "hipEventRecord failed");   // later forwards reuse the regions
  p->step_recorded = true;
  p->step_stream = s;
  return HPF_OK;
}

hpf_status hpf_forward_inference(hpf_partition* p, const void* act_in, const void* skip_in, void* out, void* skip_out,
                                 void* hip_stream) {
  if (p && (p->P.skip_in_elems != 0) != (skip_in != nullptr)) return fail(HPF_EINVAL, "skip_in is required exactly when the first block starts after its first convolution");
  if (p && (p->P.skip_out_elems != 0) != (skip_out != nullptr)) return fail(HPF_EINVAL, "skip_out is required exactly when the last block ends in a later partition");
  return hpf_forward_inference_group(p, 1, &act_in, skip_in ? &skip_in : nullptr, &out, skip_out ? &skip_out : nullptr, hip_stream);
}

hpf_status hpf_partition_set_profiling(hpf_partition* p, int32_t enable) {
  if (!p) return fail(HPF_EINVAL, "null handle");
  if (enable && !p->profiling) {
    for (int i = 0; i < PROF_N; ++i) { p->prof_ms[i] = 0; p->prof_bytes[i] = 0; p->prof_flops[i] = 0; p->prof_launches[i] = 0; }
  }
  p->profiling = enable != 0;
  return HPF_OK;
}

hpf_status hpf_partition_profile_read(hpf_partition* p, hpf_profile_entry* entries, int32_t capacity, int32_t* count) {
  if (!p || !entries || !count || capacity < 0) return fail(HPF_EINVAL, "bad argument");
  if (hipDeviceSynchronize() != hipSuccess) return fail(HPF_EDEVICE, "synchronize failed");
  for (auto& sg : p->prof_pending) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, sg.e0, sg.e1) == hipSuccess) {
      p->prof_ms[sg.cat] += ms; p->prof_launches[sg.cat] += sg.launches;
      p->prof_bytes[sg.cat] += sg.bytes; p->prof_flops[sg.cat] += sg.flops;
    }
    p->ev_pool.push_back(sg.e0); p->ev_pool.push_back(sg.e1);
  }
  p->prof_pending.clear();
  int n = 0;
  for (int i = 0; i < PROF_N && n < capacity; ++i) {
    if (p->prof_launches[i] == 0) continue;
    hpf_profile_entry& e = entries[n++];
    std::memset(&e, 0, sizeof(e));
    std::strncpy(e.name, kProfNames[i], sizeof(e.name) - 1);
    e.launches = p->prof_launches[i];
    e.total_ms = p->prof_ms[i];
    e.bytes_per_launch = p->prof_bytes[i] / (double)p->prof_launches[i];
    e.flops_per_launch = p->prof_flops[i] / (double)p->prof_launches[i];
  }
  *count = n;
  return check_abort_flag(p);
}

hpf_status hpf_partition_check(hpf_partition* p) {
  if (!p) return fail(HPF_EINVAL, "null handle");
  if (hipDeviceSynchronize() != hipSuccess) return fail(HPF_EDEVICE, "synchronize failed: %s", hipGetErrorString(hipGetLastError()));
  return check_abort_flag(p);
}

hpf_status hpf_debug_set_invalid(hpf_partition* p, int32_t value) {
  if (!p) return fail(HPF_EINVAL, "null handle");
  if (p->P.runs.empty()) return fail(HPF_EUNSUPPORTED, "the partition has no image-resident runs and therefore no such flag");
  const int v = value != 0;
  if (hipDeviceSynchronize() != hipSuccess || hipMemcpy(p->abort_flag(), &v, sizeof(int), hipMemcpyHostToDevice) != hipSuccess)
    return fail(HPF_EDEVICE, "host-to-device copy failed");
  return HPF_OK;
}

hpf_status hpf_stash_read(hpf_partition* p, int32_t mb, int32_t unit, int32_t tensor, void* host_dst, size_t bytes,
                          size_t* bytes_needed, int32_t* where) {
  if (!p || !where) return fail(HPF_EINVAL, "null argument");
  const Plan& P = p->P;
  const int nb = (int)P.bp.size();
  if (mb < 0 || mb >= P.d.num_microbatches) return fail(HPF_EINVAL, "micro-batch %d out of range", mb);
  if (unit < -1 || unit > nb) return fail(HPF_EINVAL, "unit %d out of range", unit);
  const size_t b = (size_t)P.d.microbatch;
  const size_t asz = P.dt == DT_BF16 ? sizeof(float) : sizeof(double);
  Loc loc;          // NOWHERE until resolved
  size_t need = 0;
  Loc lout; lout.kind = CALLER_ERR_OUT;
  auto grad_in = [&](int i) -> Loc { return i > 0 ? P.bp[i - 1].gy : (P.d.has_stem ? P.g_stem : lout); };
  auto stats_of = [&](const BnPlan& bn) { loc.kind = IN_MB; loc.off = bn.stats_off; need = 2 * (size_t)bn.C * asz; };
  if (unit == -1) {
    if (!P.d.has_stem) return fail(HPF_EINVAL, "the partition has no stem");
    const size_t n = b * P.d.in_h * P.d.in_w * P.d.stem_c_out * P.esz;
    if (tensor == HPF_T_Y) { loc = P.stem_out; need = n; }
    else if (tensor == HPF_T_GY) { loc = P.g_stem; need = n; }
  } else if (unit == nb) {
    if (!P.d.has_head) return fail(HPF_EINVAL, "the partition has no head");
    const size_t n = b * P.out_h * P.out_w * P.out_c * P.esz;
    if (tensor == HPF_T_X) { loc = P.head_x; need = n; }
    else if (tensor == HPF_T_A0) { loc = P.head_a; need = n; }
    else if (tensor == HPF_T_GX) { loc = grad_in(nb); need = n; }
    else if (tensor == HPF_T_STATS0) stats_of(P.head_bn);
  } else {
    const BlockPlan& q = P.bp[unit];
    const size_t M_in = b * q.h_in * q.w_in, M_out = b * q.h_out * q.w_out;
    auto held = [&](int j) { return j >= q.j0 && j < q.j1; };
    auto in_run = [&](int i) {
      for (const Plan::ResRun& r : P.runs)
        if (i >= r.first && i < r.first + r.count) return true;
      return false;
    };
    if (!q.residual()) {   // units of VGG-16 / ResNet-v1: input, output, the tensors in between, the boundary gradients
      const size_t n_in = M_in * q.d.c_in, n_out = (q.d.kind == K_DENSE ? b : M_out) * q.d.c_out;
      switch (tensor) {
        case HPF_T_X: loc = q.x_in; need = n_in * P.esz; break;
        case HPF_T_Y: loc = q.y; need = n_out * P.esz; break;
        case HPF_T_Y0: if (q.d.kind == K_CONV_RELU) { loc = q.y0; need = M_in * q.d.c_out * P.esz; } break;
        case HPF_T_GY: loc = q.gy; need = n_out * P.esz; break;
        case HPF_T_GX: loc = grad_in(unit); need = n_in * P.esz; break;
        case HPF_T_C1: if (q.d.kind == K_POSTACT) { loc = q.c[0]; need = M_out * q.d.c_mid * P.esz; } break;
        case HPF_T_A0:   // inside an image-resident run relu(bn1(c1)) never reaches memory
          if (q.d.kind == K_POSTACT && !(p->resident() && (P.run_at[unit] >= 0 || in_run(unit)))) { loc = q.a[0]; need = M_out * q.d.c_mid * P.esz; }
          break;
        case HPF_T_C2: if (q.d.kind == K_POSTACT) { loc = q.c[1]; need = M_out * q.d.c_out * P.esz; } break;
        case HPF_T_SC: if (q.d.kind == K_POSTACT) { loc = q.sc; need = M_out * q.d.c_out * P.esz; } break;
        case HPF_T_STATS0: if (q.d.kind == K_POSTACT || q.d.kind == K_BN_RELU) stats_of(q.bn[0]); break;
        case HPF_T_STATS1: if (q.d.kind == K_POSTACT) stats_of(q.bn[1]); break;
        default: break;
      }
    } else
    switch (tensor) {
      case HPF_T_X: if (q.j0 == 0) { loc = q.x_in; need = M_in * q.d.c_in * P.esz; } break;
      case HPF_T_C1: if (held(0) || q.j0 == 1) { loc = q.c[0]; need = M_out * q.d.c_mid * P.esz; } break;
      case HPF_T_C2: if (q.nconv == 3 && (held(1) || q.j0 == 2)) { loc = q.c[1]; need = M_out * q.d.c_mid * P.esz; } break;
      case HPF_T_Y: if (q.j1 == q.nconv) { loc = q.y; need = M_out * q.d.c_out * P.esz; } break;
      case HPF_T_GY: if (q.j1 == q.nconv || q.j0 == 0) { loc = q.gy; need = M_out * q.d.c_out * P.esz; } break;
      case HPF_T_DC1: if (held(0) || q.j0 == 1) { loc = q.dc[0]; need = M_out * q.d.c_mid * P.esz; } break;
      case HPF_T_DC2: if (q.nconv == 3 && (held(1) || q.j0 == 2)) { loc = q.dc[1]; need = M_out * q.d.c_mid * P.esz; } break;
      case HPF_T_GX: if (q.j0 == 0) { loc = grad_in(unit); need = M_in * q.d.c_in * P.esz; } break;
      case HPF_T_STATS0: case HPF_T_STATS1: case HPF_T_STATS2:
        if (tensor - HPF_T_STATS0 < q.nconv && held(tensor - HPF_T_STATS0)) stats_of(q.bn[tensor - HPF_T_STATS0]);
        break;
      case HPF_T_A0: case HPF_T_A1: case HPF_T_A2: {
        const int j = tensor - HPF_T_A0;
        if (j < q.nconv && held(j) && q.a[j].kind != NOWHERE) { loc = q.a[j]; need = (j == 0 ? M_in : M_out) * q.cv[j].cin * P.esz; }
        break;
      }
      default: break;
    }
  }
  if (loc.kind == NOWHERE || need == 0) return fail(HPF_EINVAL, "unit %d does not keep tensor %d", unit, tensor);
  if (bytes_needed) *bytes_needed = need;
  if (loc.kind != IN_MB) { *where = (int32_t)loc.kind; return HPF_OK; }   // CALLER_ACT_IN = 1 ... CALLER_SKIP_ERR_OUT = 8
  *where = 0;
  if (!host_dst) return HPF_OK;   // a query for the size and the place
  if (bytes != need) return fail(HPF_EINVAL, "destination has %zu bytes, the tensor %zu", bytes, need);
  if (hipDeviceSynchronize() != hipSuccess ||
      hipMemcpy(host_dst, p->mb_base(mb) + loc.off, need, hipMemcpyDeviceToHost) != hipSuccess)
    return fail(HPF_EDEVICE, "device-to-host copy failed");
  return check_abort_flag(p);
}

hpf_status hpf_params_read(hpf_partition* p, float* host_dst, size_t n_floats) {
  if (!p || !host_dst) return fail(HPF_EINVAL, "null argument");
  if (n_floats != p->P.n_params) return fail(HPF_EINVAL, "n_floats %zu, expected %zu", n_floats, p->P.n_params);
  if (hipDeviceSynchronize() != hipSuccess ||
      hipMemcpy(host_dst, p->params(), n_floats * sizeof(float), hipMemcpyDeviceToHost) != hipSuccess)
    return fail(HPF_EDEVICE, "device-to-host copy failed");
  return check_abort_flag(p);
}

// ---------------------------------------------------------------------------------------------
// single-kernel entry points
// ---------------------------------------------------------------------------------------------
static bool op_conv_args_ok(int b, int h, int wd, int cin, int cout, int R, int stride, bool bf16) {
  if (b <= 0 || h <= 0 || wd <= 0 || cin <= 0 || cout <= 0) return false;
  if ((R != 1 && R != 3) || (stride != 1 && stride != 2)) return false;
  if (h % stride || wd % stride) return false;
  if (bf16 && (cin % 16 || cout % 16)) return false;
  return true;
}

// workspace layout: [0, 64*4) tickets | sums 2*Cmax floats | partials | packed bf16 weights (both copies)
static size_t op_ws_tickets() { return 256; }
static size_t op_ws_sums_bytes(int cmax) { return align_up(2 * (size_t)cmax * sizeof(double)); }
static size_t op_ws_packed_off(int cmax) { return op_ws_tickets() + op_ws_sums_bytes(cmax) + align_up(bn_partials_floats(cmax) * 4); }

size_t hpf_op_workspace_bytes(int32_t cin, int32_t cout, int32_t R) {
  const int cmax = cin > cout ? cin : cout;
  const size_t T = (size_t)R * R;
  return op_ws_packed_off(cmax) + align_up(((size_t)cout * round_up32((int)(T * cin)) + (size_t)cin * round_up32((int)(T * cout))) * 2 + 64) +
         align_up(sizeof(PackDesc));
}

static hpf_status op_conv(int mode, hpf_dtype dtype, const void* src, const float* w, void* out, const void* add, int b, int h,
                          int wd, int cin, int cout, int R, int stride, void* ws, size_t ws_bytes, int repack, hipStream_t s) {
  if (!src || !w || !out) return fail(HPF_EINVAL, "null tensor");
  const bool bf = dtype == HPF_BF16;
  if (!op_conv_args_ok(b, h, wd, cin, cout, R, stride, bf)) return fail(HPF_EUNSUPPORTED, "unsupported convolution shape");
  ConvGeom g{};
  g.b = b; g.R = R; g.stride = stride; g.pad = (R - 1) / 2;
  if (mode == CONV_FWD) { g.Ho = h / stride; g.Wo = wd / stride; g.Hs = h; g.Ws = wd; g.Cs = cin; g.N = cout; }
  else { g.Ho = h; g.Wo = wd; g.Hs = h / stride; g.Ws = wd / stride; g.Cs = cout; g.N = cin; }
  g.M = b * g.Ho * g.Wo; g.Ktot = R * R * g.Cs; g.Kpad = round_up32(g.Ktot);
  if (!bf) {
    if (launch_conv_f32(mode, 1, one_ptr(src), w, one_ptr(out), one_ptr(add), g, s) != hipSuccess) return fail(HPF_EDEVICE, "launch failed");
    return HPF_OK;
  }
  if (!ws || ws_bytes < hpf_op_workspace_bytes(cin, cout, R)) return fail(HPF_ENOMEM, "workspace too small");
  const int cmax = cin > cout ? cin : cout;
  char* base = (char*)ws + op_ws_packed_off(cmax);
  PackDesc pd{};
  pd.w_off = 0; pd.T = R * R; pd.Cin = cin; pd.Cout = cout;
  pd.Kf = round_up32(pd.T * cin); pd.Kd = round_up32(pd.T * cout);
  pd.wf_off = 0; pd.wd_off = ((size_t)cout * pd.Kf + 7) / 8 * 8;
  const size_t table_off = align_up((pd.wd_off + (size_t)cin * pd.Kd) * 2);
  if (repack) {
    if (hipMemcpyAsync(base + table_off, &pd, sizeof(pd), hipMemcpyHostToDevice, s) != hipSuccess) return fail(HPF_EDEVICE, "table copy failed");
    if (hipStreamSynchronize(s) != hipSuccess) return fail(HPF_EDEVICE, "sync failed");   // pd is a stack object
    if (launch_pack_weights(w, (bf16_t*)base, (const PackDesc*)(base + table_off), 1, (size_t)cout * pd.Kf, s) != hipSuccess) return fail(HPF_EDEVICE, "pack failed");
  }
  const bf16_t* wp = (const bf16_t*)base + (mode == CONV_FWD ? pd.wf_off : pd.wd_off);
  if (conv_prepare() != hipSuccess) return fail(HPF_EDEVICE, "kernel set-up failed");
  if (launch_conv_mfma(mode, 1, one_ptr(src), wp, one_ptr(out), one_ptr(add), g, s) != hipSuccess) return fail(HPF_EDEVICE, "launch failed");
  return HPF_OK;
}

hpf_status hpf_op_conv_forward(hpf_dtype dtype, const void* x, const float* w, void* y, const void* add, int32_t b, int32_t h,
                               int32_t wd, int32_t cin, int32_t cout, int32_t R, int32_t stride, void* workspace,
                               size_t workspace_bytes, int32_t repack, void* hip_stream) {
  return op_conv(CONV_FWD, dtype, x, w, y, add, b, h, wd, cin, cout, R, stride, workspace, workspace_bytes, repack, (hipStream_t)hip_stream);
}

hpf_status hpf_op_conv_dgrad(hpf_dtype dtype, const void* dy, const float* w, void* dx, const void* add, int32_t b, int32_t h,
                             int32_t wd, int32_t cin, int32_t cout, int32_t R, int32_t stride, void* workspace,
                             size_t workspace_bytes, int32_t repack, void* hip_stream) {
  return op_conv(CONV_DGRAD, dtype, dy, w, dx, add, b, h, wd, cin, cout, R, stride, workspace, workspace_bytes, repack, (hipStream_t)hip_stream);
}

hpf_status hpf_op_conv_wgrad(hpf_dtype dtype, const void* x, const void* dy, float* dw, int32_t b, int32_t h, int32_t wd,
                             int32_t cin, int32_t cout, int32_t R, int32_t stride, void* hip_stream) {
  if (!x || !dy || !dw) return fail(HPF_EINVAL, "null tensor");
  const bool bf = dtype == HPF_BF16;
  if (!op_conv_args_ok(b, h, wd, cin, cout, R, stride, bf)) return fail(HPF_EUNSUPPORTED, "unsupported convolution shape");
  WgradGeom g{};
  g.b = b; g.H = h; g.W = wd; g.Cin = cin; g.Ho = h / stride; g.Wo = wd / stride; g.N = cout; g.R = R; g.stride = stride;
  g.pad = (R - 1) / 2; g.M = b * g.Ho * g.Wo; g.c_valid = cin;
  const hipError_t e = bf ? launch_wgrad_mfma(1, one_ptr(x), one_ptr(dy), dw, g, (hipStream_t)hip_stream)
                          : launch_wgrad_f32(1, one_ptr(x), one_ptr(dy), dw, g, (hipStream_t)hip_stream);
  return e == hipSuccess ? HPF_OK : fail(HPF_EDEVICE, "launch failed");
}

hpf_status hpf_op_bn_relu_forward(hpf_dtype dtype, const void* x, const float* gamma, const float* beta, float eps, void* a,
                                  void* stats, int32_t M, int32_t C, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!x || !gamma || !beta || !a || !stats || !workspace) return fail(HPF_EINVAL, "null tensor");
  if (M <= 0 || C <= 0 || C % 8) return fail(HPF_EUNSUPPORTED, "C must be a positive multiple of 8");
  if (workspace_bytes < op_ws_packed_off(C)) return fail(HPF_ENOMEM, "workspace too small");
  hipStream_t s = (hipStream_t)hip_stream;
  const int dt = dtype == HPF_BF16 ? DT_BF16 : DT_F32;
  char* ws = (char*)workspace;
  void* partials = ws + op_ws_tickets() + op_ws_sums_bytes(C);
  if (launch_bn_stats(dt, 1, one_ptr(x), M, C, eps, one_ptr(stats), one_ptr(partials), s) != hipSuccess) return fail(HPF_EDEVICE, "launch failed");
  if (launch_bn_apply_relu(dt, 1, one_ptr(x), one_ptr(a), gamma, beta, one_ptr(stats), M, C, s) != hipSuccess) return fail(HPF_EDEVICE, "launch failed");
  return HPF_OK;
}

hpf_status hpf_op_bn_relu_backward(hpf_dtype dtype, const void* x, const void* da, const float* gamma, const float* beta,
                                   const void* stats, const void* skip, void* dx, float* dgamma, float* dbeta, int32_t M,
                                   int32_t C, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!x || !da || !gamma || !beta || !stats || !dx || !dgamma || !dbeta || !workspace) return fail(HPF_EINVAL, "null tensor");
  if (M <= 0 || C <= 0 || C % 8) return fail(HPF_EUNSUPPORTED, "C must be a positive multiple of 8");
  if (workspace_bytes < op_ws_packed_off(C)) return fail(HPF_ENOMEM, "workspace too small");
  hipStream_t s = (hipStream_t)hip_stream;
  const int dt = dtype == HPF_BF16 ? DT_BF16 : DT_F32;
  char* ws = (char*)workspace;
  void* sums = ws + op_ws_tickets();
  void* partials = ws + op_ws_tickets() + op_ws_sums_bytes(C);
  if (launch_bn_bwd_reduce(dt, 1, one_ptr(x), one_ptr(da), gamma, beta, one_ptr(stats), M, C, one_ptr(sums), dgamma, dbeta, one_ptr(partials), s) != hipSuccess)
    return fail(HPF_EDEVICE, "launch failed");
  if (launch_bn_bwd_apply(dt, 1, one_ptr(x), one_ptr(da), gamma, beta, one_ptr(stats), one_ptr(sums), one_ptr(skip), one_ptr(dx), M, C, 0, s) != hipSuccess)
    return fail(HPF_EDEVICE, "launch failed");
  return HPF_OK;
}

// ---------------------------------------------------------------------------------------------
// hpf_op_bn_relu_forward for callers that cannot allocate: the reduction partials live in a file-scope device
// array instead of a caller workspace.  Every GPU holds its own copy of the array at its own address, looked up
// once per device; all calls on one GPU share it.
// ---------------------------------------------------------------------------------------------
constexpr int kStaticBnMaxC = 1024;
constexpr size_t kStaticBnFloats = (size_t)128 * kStaticBnMaxC * 4 * 2;   // = bn_partials_floats(kStaticBnMaxC): 4 MiB
static __device__ __align__(256) float scratch[kStaticBnFloats];
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mu;
static void* g_scratch_ptr[kMaxDevices] = {};

static hpf_status static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return fail(HPF_EDEVICE, "no current device");
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) return fail(HPF_EDEVICE, "hipGetSymbolAddress: %s", hipGetErrorString(e));
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return HPF_OK;
}

hpf_status hpf_op_bn_relu_forward_noalloc(hpf_dtype dtype, const void* x, const float* gamma, const float* beta, float eps,
                                          void* a, void* stats, int32_t M, int32_t C, void* hip_stream) {
  if (!x || !gamma || !beta || !a || !stats) return fail(HPF_EINVAL, "null tensor");
  if (dtype != HPF_BF16 && dtype != HPF_F32) return fail(HPF_EINVAL, "unknown dtype");
  if (M <= 0 || C <= 0 || C % 8) return fail(HPF_EUNSUPPORTED, "C must be a positive multiple of 8");
  if (C > kStaticBnMaxC) return fail(HPF_EUNSUPPORTED, "C = %d exceeds the %d channels the built-in scratch array is sized for", C, kStaticBnMaxC);
  if (bn_partials_floats(C) > kStaticBnFloats) return fail(HPF_EUNSUPPORTED, "reduction partials do not fit the built-in scratch array");
  void* partials = nullptr;
  const hpf_status st = static_scratch(&partials);
  if (st != HPF_OK) return st;
  hipStream_t s = (hipStream_t)hip_stream;
  const int dt = dtype == HPF_BF16 ? DT_BF16 : DT_F32;
  // every partial record the finalize step reads is written by the statistics kernel of the same call: nothing in
  // the array has to start at zero
  if (launch_bn_stats(dt, 1, one_ptr(x), M, C, eps, one_ptr(stats), one_ptr(partials), s) != hipSuccess) return fail(HPF_EDEVICE, "launch failed");
  if (launch_bn_apply_relu(dt, 1, one_ptr(x), one_ptr(a), gamma, beta, one_ptr(stats), M, C, s) != hipSuccess) return fail(HPF_EDEVICE, "launch failed");
  return HPF_OK;
}

hpf_status hpf_probe_copy(void* dst, const void* src, size_t bytes, void* hip_stream) {
  if (!dst || !src) return fail(HPF_EINVAL, "null pointer");
  const char* d = (const char*)dst; const char* s0 = (const char*)src;
  if (d < s0 + bytes && s0 < d + bytes) return fail(HPF_EINVAL, "source and destination overlap");
  if (bytes && launch_copy_bytes(dst, src, bytes, (hipStream_t)hip_stream) != hipSuccess) return fail(HPF_EDEVICE, "copy launch failed");
  return HPF_OK;
}

hpf_status hpf_probe_mfma_bf16(float* sink, int32_t workgroups, int32_t iters, int32_t wide, void* hip_stream) {
  if (!sink) return fail(HPF_EINVAL, "null sink");
  if (workgroups < 1 || workgroups > 65536 || iters < 1 || iters > (1 << 20)) return fail(HPF_EINVAL, "workgroups in [1, 65536], iters in [1, 2^20]");
  if (launch_probe_mfma_bf16(sink, workgroups, iters, wide != 0, (hipStream_t)hip_stream) != hipSuccess) return fail(HPF_EDEVICE, "probe launch failed");
  return HPF_OK;
}

}  // extern "C"
