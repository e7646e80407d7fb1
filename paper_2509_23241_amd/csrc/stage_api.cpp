// C ABI of the stage library: host-side bookkeeping of weight versions, the stash ring and
// the in-flight mini-batches, and the order in which the kernels of a stage are enqueued.
//
// The weight rules follow Sections "V-TiMePReSt" and "I-TiMePReSt" (Eq. 1-2), the retention
// rule follows Section "Memory Overhead", the nF1B order follows Section "Methodology".
#include "../../include/timeprest_stage.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "conv.h"
#include "transformer.h"
#include "batchnorm.h"
#include "kernels.h"

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

inline uint64_t round_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

struct LayerPlan {
  tp_layer_desc d;
  uint64_t in_elems, out_elems;  // values per sample in / out
  uint64_t w_elems;              // elements of the weight tensor (0: no parameters)
  uint64_t w_off, b_off;  // elements inside one weight version
  uint64_t x_off, z_off;  // bytes inside one activation slot; z_off: saved act'(z) (UINT64_MAX: none)
  uint64_t xpad_off = UINT64_MAX;  // first image layer in bf16: the input again, padded to 8 channels per pixel
  uint64_t stat_off = UINT64_MAX;  // layer norm: mean and 1/std per token; attention: log-sum-exp per (head, query)
  uint64_t stat_elems = 0;         // floats per sample behind stat_off
  uint64_t stat_bytes = 0;         // batch norm: bytes behind stat_off (per micro-batch, not per sample)
  int tokens = 1;                  // positions per sample (rows of the layer's matrices per sample)
  int skip_layer = -1;             // residual add: index of the layer that remembered the skip activation
  bool relu_out = false;           // ReLU whose derivative is read off its saved OUTPUT (the next layer's input): no act' tensor
};

struct Slot {
  bool occupied = false;
  uint64_t version = 0;
  uint32_t refcnt = 0;
};

struct InFlight {
  uint64_t mb_id;
  uint64_t v_f;           // version of the first micro-batch forward (pinned under stashing)
  uint32_t forwards;      // micro-batch forwards seen
  int act_slot;
  bool pinned;
};

struct Plan {
  std::vector<LayerPlan> layers;
  tp_sizes sizes;
  uint64_t act_slot_bytes = 0;
  uint64_t dz_bytes = 0;       // one backward temporary
  uint64_t partial_floats = 0; // reduction partials
  uint64_t deferred_floats = 0; // behind them: partials of the backward pass's sums, which one launch forms at its end
  uint64_t fwd2_floats = 0;     // behind those: scratch of the normalisation forward kernels on a second forward stream
  uint64_t attn_scratch_bytes = 0;  // transient score matrices of the matrix-core attention
  size_t elt_size = 4;
};

// output pixels per image of a convolution layer (geom: H, W, kernel, stride, pad)
inline uint64_t conv_out_px(const tp_layer_desc& L) { return (uint64_t)(L.geom[0] / L.geom[3]) * (L.geom[1] / L.geom[3]); }

int check_desc(const tp_stage_desc* d) {
  if (!d) return fail(TP_EINVAL, "null stage description");
  if (d->num_layers < 1 || d->num_layers > TP_MAX_LAYERS)
    return fail(TP_EINVAL, "num_layers %d outside 1..%d", d->num_layers, TP_MAX_LAYERS);
  if (d->dtype != TP_F32 && d->dtype != TP_BF16) return fail(TP_EINVAL, "unknown dtype %d", d->dtype);
  if (d->mb < 1 || d->n < 1) return fail(TP_EINVAL, "mb and n must be positive");
  if ((int64_t)d->mb * d->n > (1 << 24)) return fail(TP_EINVAL, "mini-batch too large");
  if (d->num_stages < 1 || d->stage_index < 0 || d->stage_index >= d->num_stages)
    return fail(TP_EINVAL, "stage_index %d outside 0..%d", d->stage_index, d->num_stages - 1);
  if (d->ring_capacity < 1 || d->ring_capacity > TP_MAX_SLOTS)
    return fail(TP_EINVAL, "ring_capacity %d outside 1..%d", d->ring_capacity, TP_MAX_SLOTS);
  if (d->max_in_flight < 1 || d->max_in_flight > TP_MAX_IN_FLIGHT)
    return fail(TP_EINVAL, "max_in_flight %d outside 1..%d", d->max_in_flight, TP_MAX_IN_FLIGHT);
  if (d->policy < TP_LATEST || d->policy > TP_TIMEPREST) return fail(TP_EINVAL, "unknown policy %d", d->policy);
  if (!(d->lambda > 0.0) || !std::isfinite(d->lambda)) return fail(TP_EINVAL, "lambda must be > 0");
  if (!std::isfinite(d->lr) || !std::isfinite(d->momentum)) return fail(TP_EINVAL, "lr/momentum not finite");
  uint64_t prev_out = 0;
  int open_skip = -1;  // layer of a residual begin that has not met its add yet
  int open_swap = -1;  // layer of the swap between that begin and its add, if there is one
  for (int l = 0; l < d->num_layers; ++l) {
    const tp_layer_desc& L = d->layers[l];
    if (L.act < TP_ACT_NONE || L.act > TP_ACT_GELU) return fail(TP_EINVAL, "layer %d: unknown activation", l);
    if (L.in_features < 1 || L.out_features < 1) return fail(TP_EINVAL, "layer %d: empty shape", l);
    uint64_t in_e, out_e;
    if (L.type == TP_LAYER_DENSE) {
      for (int r = 1; r < 5; ++r)
        if (L.geom[r] != 0) return fail(TP_EINVAL, "layer %d: geometry fields 1..4 must be zero for a dense layer", l);
      if (L.geom[0] < 0) return fail(TP_EINVAL, "layer %d: negative token count", l);
      const uint64_t T = L.geom[0] > 1 ? L.geom[0] : 1;
      in_e = T * L.in_features;
      out_e = T * L.out_features;
    } else if (L.type == TP_LAYER_BATCHNORM) {
      if (L.geom[0] < 1 || L.in_features != L.out_features || L.geom[1] || L.geom[2] || L.geom[3] || L.geom[4])
        return fail(TP_EINVAL, "layer %d: malformed batch normalisation layer", l);
      in_e = out_e = (uint64_t)L.geom[0] * L.in_features;
    } else if (L.type == TP_LAYER_RESIDUAL && L.geom[1] == 2) {
      // swap: the main branch's result is set aside and the tensor remembered at the begin comes back,
      // so that the layers up to the add form a second branch (a projection shortcut)
      if (open_skip < 0 || open_swap >= 0) return fail(TP_EINVAL, "layer %d: residual swap needs an open begin and no earlier swap", l);
      const tp_layer_desc& B = d->layers[open_skip];
      if (L.geom[0] < 1 || L.geom[2] < 1 || L.act != TP_ACT_NONE || L.geom[3] || L.geom[4])
        return fail(TP_EINVAL, "layer %d: malformed residual swap", l);
      if (L.out_features != B.in_features || L.geom[2] != B.geom[0])
        return fail(TP_EINVAL, "layer %d: residual swap does not give back the shape remembered at layer %d", l, open_skip);
      open_swap = l;
      in_e = (uint64_t)L.geom[0] * L.in_features;
      out_e = (uint64_t)L.geom[2] * L.out_features;
    } else if (L.type == TP_LAYER_LAYERNORM || L.type == TP_LAYER_RESIDUAL) {
      const bool act_ok = L.act == TP_ACT_NONE || (L.type == TP_LAYER_RESIDUAL && L.geom[1] == 1);
      if (L.geom[0] < 1 || L.in_features != L.out_features || !act_ok || L.geom[2] || L.geom[3] || L.geom[4])
        return fail(TP_EINVAL, "layer %d: malformed %s layer", l, L.type == TP_LAYER_LAYERNORM ? "normalisation" : "residual");
      if (L.type == TP_LAYER_LAYERNORM && (L.geom[1] != 0 || L.in_features > 20480))
        return fail(TP_EINVAL, "layer %d: malformed normalisation layer", l);
      if (L.type == TP_LAYER_RESIDUAL) {
        if (L.geom[1] != 0 && L.geom[1] != 1) return fail(TP_EINVAL, "layer %d: residual mark must be 0, 1 or 2", l);
        if (L.geom[1] != (open_skip >= 0 ? 1 : 0))
          return fail(TP_EINVAL, "layer %d: residual marks must alternate begin, add", l);
        if (L.geom[1] == 0) {
          open_skip = l;
        } else {
          const int kept = open_swap >= 0 ? open_swap : open_skip;
          const tp_layer_desc& B = d->layers[kept];
          if (B.in_features != L.in_features || B.geom[0] != L.geom[0])
            return fail(TP_EINVAL, "layer %d: residual add does not match the shape remembered at layer %d", l, kept);
          open_skip = open_swap = -1;
        }
      }
      in_e = out_e = (uint64_t)L.geom[0] * L.in_features;
    } else if (L.type == TP_LAYER_ATTENTION) {
      if (L.geom[0] < 1 || L.geom[1] < 1 || L.act != TP_ACT_NONE || L.geom[2] || L.geom[3] || L.geom[4] ||
          L.in_features != 3 * L.out_features || L.out_features % L.geom[1] != 0)
        return fail(TP_EINVAL, "layer %d: malformed attention layer", l);
      if (!tp::attention_supported(L.geom[0], L.geom[1], L.out_features / L.geom[1]))
        return fail(TP_EINVAL, "layer %d: head width %d is outside what the attention kernels take", l,
                    L.out_features / L.geom[1]);
      if (l == d->num_layers - 1) return fail(TP_EINVAL, "layer %d: attention must not be the last layer of a stage", l);
      in_e = (uint64_t)L.geom[0] * L.in_features;
      out_e = (uint64_t)L.geom[0] * L.out_features;
    } else if (L.type == TP_LAYER_CONV2D) {
      if (L.geom[0] < 1 || L.geom[1] < 1) return fail(TP_EINVAL, "layer %d: empty image", l);
      if (!tp::conv_geometry_supported(L.geom[2], L.geom[3], L.geom[4]))
        return fail(TP_EINVAL, "layer %d: convolutions are built for kernels 1, 3, 5, 7 with stride 1 or 2 and pad (kernel-1)/2", l);
      if (L.geom[3] == 2 && ((L.geom[0] & 1) || (L.geom[1] & 1)))
        return fail(TP_EINVAL, "layer %d: a stride-2 convolution needs even height and width", l);
      in_e = (uint64_t)L.geom[0] * L.geom[1] * L.in_features;
      out_e = (uint64_t)(L.geom[0] / L.geom[3]) * (L.geom[1] / L.geom[3]) * L.out_features;
    } else if (L.type == TP_LAYER_MAXPOOL2) {
      if (L.geom[0] < 2 || L.geom[1] < 2 || (L.geom[0] & 1) || (L.geom[1] & 1))
        return fail(TP_EINVAL, "layer %d: pooling needs even height and width", l);
      if (L.in_features != L.out_features || L.act != TP_ACT_NONE || L.geom[2] || L.geom[3] || L.geom[4])
        return fail(TP_EINVAL, "layer %d: malformed pooling layer", l);
      in_e = (uint64_t)L.geom[0] * L.geom[1] * L.in_features;
      out_e = in_e / 4;
    } else if (L.type == TP_LAYER_AVGPOOL) {
      if (L.geom[0] < 1 || L.in_features != L.out_features || L.act != TP_ACT_NONE || L.geom[1] || L.geom[2] || L.geom[3] ||
          L.geom[4])
        return fail(TP_EINVAL, "layer %d: malformed average pooling layer", l);
      in_e = (uint64_t)L.geom[0] * L.in_features;
      out_e = L.out_features;
    } else if (L.type == TP_LAYER_SUBSAMPLE2) {
      if (L.geom[0] < 2 || L.geom[1] < 2 || (L.geom[0] & 1) || (L.geom[1] & 1))
        return fail(TP_EINVAL, "layer %d: subsampling needs even height and width", l);
      if (L.in_features != L.out_features || L.act != TP_ACT_NONE || L.geom[2] || L.geom[3] || L.geom[4])
        return fail(TP_EINVAL, "layer %d: malformed subsampling layer", l);
      if ((L.in_features * (d->dtype == TP_BF16 ? 2 : 4)) % 16)
        return fail(TP_EINVAL, "layer %d: subsampling needs pixels of whole 16-byte units", l);
      in_e = (uint64_t)L.geom[0] * L.geom[1] * L.in_features;
      out_e = in_e / 4;
    } else {
      return fail(TP_EINVAL, "layer %d: unknown type %d", l, L.type);
    }
    if (in_e > (1u << 30) || out_e > (1u << 30)) return fail(TP_EINVAL, "layer %d: sample too large", l);
    if (l > 0 && prev_out != in_e)
      return fail(TP_EINVAL, "layer %d: input of %llu values does not match previous output of %llu", l,
                  (unsigned long long)in_e, (unsigned long long)prev_out);
    prev_out = out_e;
    for (int r = 0; r < 7; ++r)
      if (L.reserved[r] != 0) return fail(TP_EINVAL, "layer %d: reserved fields must be zero", l);
  }
  if (open_skip >= 0) return fail(TP_EINVAL, "layer %d: residual begin without an add", open_skip);
  return TP_OK;
}

// Floats of partial sums one layer's backward pass keeps until the sums are formed (each rounded up to 64).
struct DeferredNeed {
  uint64_t bias = 0, weight = 0, norm = 0;
  uint64_t total() const { return bias + weight + norm; }
};
constexpr uint64_t kMaxDeferredFloats = 1ull << 28;  // 1 GiB

DeferredNeed deferred_need(const tp_stage_desc& d, const LayerPlan& lp) {
  DeferredNeed need;
  if (!lp.w_elems) return need;
  const uint64_t rows = (uint64_t)d.mb * d.n;
  const tp_layer_desc& L = lp.d;
  if (L.type == TP_LAYER_LAYERNORM) {
    need.norm = round_up(tp::layernorm_scratch_floats(rows * lp.tokens, L.in_features), 64);
  } else if (L.type == TP_LAYER_BATCHNORM) {
    need.norm = round_up((uint64_t)d.n * 3 * L.in_features, 64);  // per micro-batch: two column sums + those of dx
  } else if (L.type == TP_LAYER_CONV2D) {
    const uint64_t px = rows * conv_out_px(L);
    need.bias = round_up(tp::colsum_scratch_floats((int)px, L.out_features), 64);
    need.weight = round_up(tp::conv_wgrad_scratch_floats((int)px, L.in_features, L.out_features, L.geom[2]), 64);
  } else if (L.type == TP_LAYER_DENSE) {
    const uint64_t r = rows * lp.tokens;
    need.bias = round_up(tp::colsum_scratch_floats((int)r, L.out_features), 64);
    need.weight = round_up(tp::wgrad_scratch_floats(d.dtype, (int)r, L.out_features, L.in_features), 64);
  }
  return need;
}

int make_plan(const tp_stage_desc* d, Plan* p) {
  int rc = check_desc(d);
  if (rc) return rc;
  p->elt_size = d->dtype == TP_BF16 ? 2 : 4;
  const uint64_t rows = (uint64_t)d->mb * d->n;
  std::memset(&p->sizes, 0, sizeof(p->sizes));
  uint64_t off = 0, act = 0, max_feat = 0;
  uint64_t conv_scratch = 0, norm_scratch = 0;
  int open_skip = -1, open_swap = -1;
  int alias_of = -1;  // >= 0: this layer reads the tensor layer `alias_of` saved (it follows a residual begin or swap)
  for (int l = 0; l < d->num_layers; ++l) {
    LayerPlan lp;
    lp.d = d->layers[l];
    const tp_layer_desc& L = lp.d;
    if (L.type == TP_LAYER_DENSE) {
      lp.tokens = L.geom[0] > 1 ? L.geom[0] : 1;
      lp.in_elems = (uint64_t)lp.tokens * L.in_features;
      lp.out_elems = (uint64_t)lp.tokens * L.out_features;
      lp.w_elems = (uint64_t)L.in_features * L.out_features;
    } else if (L.type == TP_LAYER_LAYERNORM) {
      lp.tokens = L.geom[0];
      lp.in_elems = lp.out_elems = (uint64_t)lp.tokens * L.in_features;
      lp.w_elems = L.in_features;                      // gamma; beta sits where a dense layer keeps its bias
      lp.stat_elems = 2 * (uint64_t)lp.tokens;
      norm_scratch = std::max<uint64_t>(norm_scratch, tp::layernorm_scratch_floats(rows * lp.tokens, L.in_features));
    } else if (L.type == TP_LAYER_BATCHNORM) {
      lp.tokens = L.geom[0];
      lp.in_elems = lp.out_elems = (uint64_t)lp.tokens * L.in_features;
      lp.w_elems = L.in_features;
      lp.stat_bytes = (uint64_t)d->n * 2 * L.in_features * 4;   // (mean, 1/std) per channel and micro-batch
      norm_scratch = std::max<uint64_t>(norm_scratch, tp::batchnorm_scratch_floats((size_t)d->mb * lp.tokens, L.in_features, d->n) +
                                                          (uint64_t)d->n * 2 * L.in_features);
      p->fwd2_floats = std::max<uint64_t>(p->fwd2_floats,
                                          round_up(tp::batchnorm_scratch_floats((size_t)d->mb * lp.tokens, L.in_features, 1), 64));
    } else if (L.type == TP_LAYER_ATTENTION) {
      lp.tokens = L.geom[0];
      lp.in_elems = (uint64_t)lp.tokens * L.in_features;
      lp.out_elems = (uint64_t)lp.tokens * L.out_features;
      lp.w_elems = 0;
      lp.stat_elems = (uint64_t)lp.tokens * L.geom[1];
      p->attn_scratch_bytes = std::max<uint64_t>(
          p->attn_scratch_bytes,
          tp::attention_scratch_bytes(d->dtype, (int)rows, lp.tokens, L.geom[1], L.out_features / L.geom[1]));
    } else if (L.type == TP_LAYER_RESIDUAL) {
      lp.tokens = L.geom[0];
      lp.in_elems = lp.out_elems = (uint64_t)lp.tokens * L.in_features;
      lp.w_elems = 0;
      if (L.geom[1] == 0) {
        open_skip = l;
      } else if (L.geom[1] == 2) {
        lp.out_elems = (uint64_t)L.geom[2] * L.out_features;
        lp.skip_layer = open_skip;   // whose saved input the next layer reads
        open_swap = l;
      } else {
        lp.skip_layer = open_swap >= 0 ? open_swap : open_skip;  // the tensor that is added: saved input of that layer
        open_skip = open_swap = -1;
      }
    } else if (L.type == TP_LAYER_CONV2D) {
      lp.in_elems = (uint64_t)L.geom[0] * L.geom[1] * L.in_features;
      lp.out_elems = conv_out_px(L) * L.out_features;
      lp.w_elems = (uint64_t)L.out_features * L.geom[2] * L.geom[2] * L.in_features;
      conv_scratch = std::max<uint64_t>(conv_scratch, tp::conv_wgrad_scratch_floats((int)(rows * conv_out_px(L)),
                                                                                    L.in_features, L.out_features, L.geom[2]));
    } else if (L.type == TP_LAYER_AVGPOOL) {
      lp.tokens = L.geom[0];
      lp.in_elems = (uint64_t)lp.tokens * L.in_features;
      lp.out_elems = L.out_features;
      lp.w_elems = 0;
    } else {
      lp.in_elems = (uint64_t)L.geom[0] * L.geom[1] * L.in_features;
      lp.out_elems = lp.in_elems / 4;
      lp.w_elems = 0;
    }
    lp.w_off = off;
    lp.b_off = off;
    if (lp.w_elems) {
      off += round_up(lp.w_elems, 64);
      lp.b_off = off;
      off += round_up((uint64_t)L.out_features, 64);
    }
    if (alias_of >= 0) {
      lp.x_off = p->layers[alias_of].x_off;
    } else {
      lp.x_off = act;
      act += round_up(rows * lp.in_elems * p->elt_size, 256);
    }
    alias_of = L.type != TP_LAYER_RESIDUAL ? -1 : L.geom[1] == 0 ? l : L.geom[1] == 2 ? lp.skip_layer : -1;
    if (lp.stat_elems || lp.stat_bytes) {
      lp.stat_off = act;
      act += round_up(lp.stat_bytes ? lp.stat_bytes : rows * lp.stat_elems * 4, 256);
    }
    // act'(z) is kept for the backward pass -- except for a ReLU whose output the stage keeps anyway as the next
    // layer's input: relu'(z) = (output > 0).  Not for the last layer (its output goes to the caller) and not in
    // front of a residual add (the add may be formed in this layer's kernel, the bare output then never exists).
    const bool next_is_add = l + 1 < d->num_layers && d->layers[l + 1].type == TP_LAYER_RESIDUAL && d->layers[l + 1].geom[1] == 1;
    lp.relu_out = L.act == TP_ACT_RELU && l + 1 < d->num_layers && !next_is_add;
    if (L.act != TP_ACT_NONE && !lp.relu_out) {
      lp.z_off = act;
      act += round_up(rows * lp.out_elems * p->elt_size, 256);
    } else {
      lp.z_off = UINT64_MAX;
    }
    const bool c8_3x3 = L.geom[2] == 3 && L.geom[3] == 1 &&
                        tp::conv_c8_supported((int)rows, L.geom[0], L.geom[1], L.in_features, L.out_features) &&
                        tp::conv_c8_supported(d->mb, L.geom[0], L.geom[1], L.in_features, L.out_features);
    const bool c8_stem = L.geom[2] == 7 && L.geom[3] == 2 &&
                         tp::conv_stem_supported((int)rows, L.geom[0], L.geom[1], L.in_features, L.out_features) &&
                         tp::conv_stem_supported(d->mb, L.geom[0], L.geom[1], L.in_features, L.out_features);
    if (l == 0 && L.type == TP_LAYER_CONV2D && d->dtype == TP_BF16 && (c8_3x3 || c8_stem)) {
      lp.xpad_off = act;
      act += round_up(rows * L.geom[0] * L.geom[1] * 8 * p->elt_size, 256);
    }
    max_feat = std::max<uint64_t>(max_feat, std::max(lp.in_elems, lp.out_elems));
    p->sizes.w_offset[l] = lp.w_off;
    p->sizes.b_offset[l] = lp.b_off;
    p->layers.push_back(lp);
  }
  const uint64_t P = off;
  p->act_slot_bytes = act;
  p->dz_bytes = round_up(rows * max_feat * p->elt_size, 256);
  uint64_t wg = 0;
  for (const LayerPlan& lp : p->layers) {
    if (!lp.w_elems) continue;
    // bias gradients: column sums over rows (dense) or over all pixels (conv)
    if (lp.d.type == TP_LAYER_LAYERNORM || lp.d.type == TP_LAYER_BATCHNORM) continue;
    const uint64_t r = lp.d.type == TP_LAYER_CONV2D ? rows * conv_out_px(lp.d) : rows * lp.tokens;
    wg = std::max<uint64_t>(wg, tp::colsum_scratch_floats((int)r, lp.d.out_features));
    if (lp.d.type == TP_LAYER_DENSE)
      wg = std::max<uint64_t>(wg, tp::wgrad_scratch_floats(d->dtype, (int)r, lp.d.out_features, lp.d.in_features));
  }
  p->partial_floats = round_up(std::max<uint64_t>({wg, tp::update_scratch_floats(), rows, conv_scratch, norm_scratch}), 64);
  // Every sum of partials the backward pass needs (bias and split weight gradients, scale and shift gradients of the
  // normalisations) is put off to one launch at its end: each keeps partials of its own until then.
  uint64_t deferred = 0;
  for (const LayerPlan& lp : p->layers) deferred += deferred_need(*d, lp).total();
  p->deferred_floats = deferred <= kMaxDeferredFloats ? deferred : 0;  // beyond that: sums right away, shared partials
  tp_sizes& s = p->sizes;
  s.param_count = P;
  s.ring_bytes = (uint64_t)d->ring_capacity * P * 4;
  s.momentum_bytes = P * 4;
  s.grad_bytes = P * 4;
  s.wfwd_bytes = d->dtype == TP_BF16 ? P * 2 : 0;
  s.wbwd_bytes = d->policy == TP_LATEST ? 0 : P * p->elt_size;  // V-TiMePReSt never builds intermediate weights
  s.act_bytes = (uint64_t)d->max_in_flight * act;
  s.scratch_bytes = 3 * p->dz_bytes + (p->partial_floats + p->deferred_floats + TP_MAX_FORWARD_STREAMS * p->fwd2_floats) * 4 + 512 + p->attn_scratch_bytes;  // + an aligned block of 256 zero bytes (conv padding)
  s.diag_bytes = TP_DIAG_COUNT * sizeof(double);
  return TP_OK;
}

// policies under which a mini-batch's forward version is stashed for its backward pass
bool stashing(int policy) { return policy == TP_INTERMEDIATE_EQ1 || policy == TP_INTERMEDIATE_CONVEX || policy == TP_STASHED; }

}  // namespace

struct ProfEntry {
  int cls;
  hipEvent_t start, stop;
};

struct tp_stage {
  tp_stage_desc desc;
  // profiling: event pairs recorded around each launch while switched on
  bool prof_on = false;
  std::vector<ProfEntry> prof_pool;
  size_t prof_used = 0;
  uint64_t prof_dropped = 0;
  Plan plan;
  tp_buffers bufs;
  hipStream_t stream;
  bool dry;                     // no device buffers given: bookkeeping only, nothing is launched
  uint64_t latest = 0;
  Slot slots[TP_MAX_SLOTS];
  std::vector<InFlight> inflight;
  bool act_used[TP_MAX_IN_FLIGHT] = {};
  bool grad_pending = false;
  uint64_t grad_mb = 0;
  // W_b prepared ahead by the fused update
  bool wb_valid = false;
  uint64_t wb_mb = TP_NONE, wb_vf = 0, wb_vnow = 0;
  // TP_TIMEPREST in bf16 mode: the version whose compute copy wbwd_dev holds (passes on a version that is no
  // longer the latest read their weights from there)
  bool copy_valid = false;
  uint64_t copy_version = 0;
  // Optional second stream of the caller's: the forward passes of odd micro-batches run there, beside the even ones.
  int fwd_streams = 0;                                    // how many the caller gave
  hipStream_t fwd_stream[TP_MAX_FORWARD_STREAMS] = {};
  hipEvent_t ev_main = nullptr;                           // "the stage's stream is ready for forwards"
  hipEvent_t ev_fwd[TP_MAX_FORWARD_STREAMS] = {};         // "this forward stream is done"
  bool main_dirty = true;                                 // the stage's stream got work other than forwards since ev_main was recorded
  bool fwd_pending[TP_MAX_FORWARD_STREAMS] = {};          // the stream holds forwards the stage's stream has not waited for yet
  // per activation slot (= mini-batch in flight) and forward stream: the last forward of that mini-batch there, which
  // its backward pass waits for -- and for no other, so that forwards of later mini-batches run beside it
  hipEvent_t ev_slot[TP_MAX_IN_FLIGHT][TP_MAX_FORWARD_STREAMS] = {};
  bool slot_fwd[TP_MAX_IN_FLIGHT][TP_MAX_FORWARD_STREAMS] = {};
  bool slot_event_lost = false;  // such an event could not be recorded: the next backward pass waits for every forward stream

  int find_slot(uint64_t v) const {
    const Slot& s = slots[v % desc.ring_capacity];
    return (s.occupied && s.version == v) ? (int)(v % desc.ring_capacity) : -1;
  }
  InFlight* find_mb(uint64_t mb) {
    for (InFlight& f : inflight)
      if (f.mb_id == mb) return &f;
    return nullptr;
  }
  float* ring(int slot) const { return (float*)bufs.ring_dev + (uint64_t)slot * plan.sizes.param_count; }
  char* act_slot(int q) const { return (char*)bufs.act_dev + (uint64_t)q * plan.act_slot_bytes; }
  char* dz_buf(int i) const { return (char*)bufs.scratch_dev + (uint64_t)i * plan.dz_bytes; }
  float* partials() const { return (float*)((char*)bufs.scratch_dev + 3 * plan.dz_bytes); }
  float* deferred_partials() const { return partials() + plan.partial_floats; }
  float* fwd2_scratch(int k) const { return deferred_partials() + plan.deferred_floats + (uint64_t)k * plan.fwd2_floats; }
  std::vector<tp::SumJob> sum_jobs;  // the backward pass under way: sums still to be formed
  const void* zeros() const {  // 256-byte aligned, behind the partial sums
    const uintptr_t p = (uintptr_t)bufs.scratch_dev + 3 * plan.dz_bytes + (plan.partial_floats + plan.deferred_floats + TP_MAX_FORWARD_STREAMS * plan.fwd2_floats) * 4;
    return (const void*)((p + 255) & ~(uintptr_t)255);
  }
  void* attn_scratch() const { return plan.attn_scratch_bytes ? (char*)zeros() + 256 : nullptr; }
  // drop a version that nobody needs any more
  void evict_if_unused(uint64_t v) {
    int s = find_slot(v);
    if (s >= 0 && v != latest && slots[s].refcnt == 0) slots[s].occupied = false;
  }
};

// Brackets the launches made during its lifetime with an event pair when profiling is on.
struct ProfScope {
  tp_stage* st;
  ProfEntry* e = nullptr;
  ProfScope(tp_stage* s, int cls) : st(s) {
    if (!st->prof_on) return;
    if (st->prof_used >= st->prof_pool.size()) { st->prof_dropped++; return; }
    e = &st->prof_pool[st->prof_used++];
    e->cls = cls;
    (void)hipEventRecord(e->start, st->stream);
  }
  ~ProfScope() {
    if (e) (void)hipEventRecord(e->stop, st->stream);
  }
};

#define HIP_TRY(expr)                                                                     \
  do {                                                                                    \
    hipError_t e_ = (expr);                                                               \
    if (e_ != hipSuccess) return fail(TP_EHIP, "%s: %s", #expr, hipGetErrorString(e_));   \
  } while (0)

// Every entry point that enqueues work other than a forward pass, or hands out results, starts here: the stage's
// stream waits for the forwards the second stream still holds, and the next forward knows it has to order itself
// behind what this call enqueues.
int join_forwards(tp_stage* st) {
  st->main_dirty = true;
  for (int k = 0; k < TP_MAX_FORWARD_STREAMS; ++k) {
    if (!st->fwd_pending[k]) continue;
    HIP_TRY(hipEventRecord(st->ev_fwd[k], st->fwd_stream[k]));
    HIP_TRY(hipStreamWaitEvent(st->stream, st->ev_fwd[k], 0));
    st->fwd_pending[k] = false;
    for (int q = 0; q < TP_MAX_IN_FLIGHT; ++q) st->slot_fwd[q][k] = false;  // ordered with everything else on the stream
  }
  return TP_OK;
}

extern "C" {

const char* tp_last_error(void) { return g_err; }

int tp_blend_coefficients(int32_t policy, uint32_t delta, double lambda, double* alpha, double* beta) {
  if (!alpha || !beta) return fail(TP_EINVAL, "null output");
  if (!(lambda > 0.0)) return fail(TP_EINVAL, "lambda must be > 0");
  // Eq. 2: significance of weights that are `delta` updates old.
  const double f = std::exp(-lambda * (double)delta);
  switch (policy) {
    case TP_LATEST: *alpha = 0.0; *beta = 1.0; break;
    case TP_STASHED: *alpha = 1.0; *beta = 0.0; break;
    case TP_TIMEPREST: *alpha = 1.0; *beta = 0.0; break;   // the version the pass started on, as it is
    case TP_INTERMEDIATE_EQ1: *alpha = 2.0 - 1.0 / f; *beta = 0.0; break;          // Eq. 1
    case TP_INTERMEDIATE_CONVEX: *alpha = f; *beta = 1.0 - f; break;               // Appendix A.2
    default: return fail(TP_EINVAL, "unknown policy %d", policy);
  }
  return TP_OK;
}

int tp_schedule_events(int32_t K, uint64_t num_mb, tp_event* out, uint64_t capacity, uint64_t* count) {
  if (K < 1 || K > 1024 || !count) return fail(TP_EINVAL, "bad schedule arguments");
  // Per-stage programme: K-s forwards, then backward/forward alternating.  The clock
  // advances one operation per stage per tick; an operation runs once its producer has
  // finished on an earlier tick.  Within a tick: backwards from the last stage down, then
  // forwards from the first stage up.
  struct Cursor { uint64_t next_f = 0, next_b = 0; };
  std::vector<Cursor> cur(K);
  std::vector<std::vector<int64_t>> f_done(K), b_done(K);
  for (int s = 0; s < K; ++s) { f_done[s].assign(num_mb, -1); b_done[s].assign(num_mb, -1); }
  uint64_t emitted = 0;
  const uint64_t total = 2ull * K * num_mb;
  for (int64_t t = 0; emitted < total; ++t) {
    if (t > (int64_t)(4 * total + 16)) return fail(TP_ESTATE, "schedule did not terminate");
    std::vector<int> run_b, run_f;
    for (int s = 0; s < K; ++s) {
      Cursor& c = cur[s];
      if (c.next_b >= num_mb) continue;
      const uint64_t warm = std::min<uint64_t>(K - s, num_mb);
      // the stage's next operation: forward while warming up or right after a backward
      const bool want_f = c.next_f < num_mb && (c.next_f < warm || c.next_f < c.next_b + warm);
      if (want_f) {
        const uint64_t j = c.next_f;
        if (s == 0 || (f_done[s - 1][j] >= 0 && f_done[s - 1][j] < t)) run_f.push_back(s);
      } else {
        const uint64_t j = c.next_b;
        const int64_t dep = (s == K - 1) ? f_done[s][j] : b_done[s + 1][j];
        if (dep >= 0 && dep < t) run_b.push_back(s);
      }
    }
    for (auto it = run_b.rbegin(); it != run_b.rend(); ++it) {
      const int s = *it;
      const uint64_t j = cur[s].next_b++;
      b_done[s][j] = t;
      if (out && emitted < capacity) out[emitted] = tp_event{(int32_t)t, 1, s, 0, j};
      ++emitted;
    }
    for (int s : run_f) {
      const uint64_t j = cur[s].next_f++;
      f_done[s][j] = t;
      if (out && emitted < capacity) out[emitted] = tp_event{(int32_t)t, 0, s, 0, j};
      ++emitted;
    }
  }
  *count = emitted;
  return TP_OK;
}

int tp_schedule_microbatch_events(int32_t K, uint64_t num_mb, int32_t n, int32_t mid_pass_updates, tp_event* out,
                                  uint64_t capacity, uint64_t* count) {
  if (K < 1 || K > 1024 || n < 1 || n > 65536 || !count) return fail(TP_EINVAL, "bad schedule arguments");
  // One box per stage and tick: the forward pass of one micro-batch or the backward pass (and update) of one
  // mini-batch.  A stage holds at most K-s mini-batches between first forward and backward; a backward pass that
  // is ready goes first -- between two micro-batches of one mini-batch only if mid_pass_updates is set.
  struct StageCursor { uint64_t f_mb = 0; int32_t f_ub = 0; uint64_t b_mb = 0; };
  std::vector<StageCursor> cur(K);
  // tick at which (stage, mini-batch, micro-batch) was forwarded / (stage, mini-batch) went backward; -1: not yet
  std::vector<std::vector<int64_t>> f_at(K, std::vector<int64_t>(num_mb * (uint64_t)n, -1));
  std::vector<std::vector<int64_t>> b_at(K, std::vector<int64_t>(num_mb, -1));
  struct Box { int kind, s, ub; uint64_t j; };
  uint64_t emitted = 0;
  const uint64_t total = (uint64_t)K * num_mb * ((uint64_t)n + 1);
  for (int64_t t = 0; emitted < total; ++t) {
    if (t > (int64_t)(4 * total + 16)) return fail(TP_ESTATE, "schedule did not terminate");
    std::vector<Box> bwd, fwd;
    for (int s = 0; s < K; ++s) {
      const StageCursor& c = cur[s];
      if (c.b_mb >= num_mb) continue;
      const int64_t b_dep = s == K - 1 ? f_at[s][c.b_mb * n + (n - 1)] : b_at[s + 1][c.b_mb];
      const bool b_ready = b_dep >= 0 && b_dep < t;
      bool f_ready = c.f_mb < num_mb;
      if (f_ready && s > 0) {
        const int64_t dep = f_at[s - 1][c.f_mb * n + c.f_ub];
        f_ready = dep >= 0 && dep < t;
      }
      if (f_ready && c.f_ub == 0) f_ready = c.f_mb - c.b_mb < (uint64_t)(K - s);   // a new mini-batch: in-flight limit
      const bool mid_pass = c.f_ub > 0;
      if (b_ready && (mid_pass_updates || !mid_pass || !f_ready)) bwd.push_back(Box{1, s, 0, c.b_mb});
      else if (f_ready) fwd.push_back(Box{0, s, c.f_ub, c.f_mb});
    }
    if (bwd.empty() && fwd.empty()) return fail(TP_ESTATE, "schedule deadlock");
    for (auto it = bwd.rbegin(); it != bwd.rend(); ++it) {
      b_at[it->s][it->j] = t;
      cur[it->s].b_mb++;
      if (out && emitted < capacity) out[emitted] = tp_event{(int32_t)t, 1, it->s, 0, it->j};
      ++emitted;
    }
    for (const Box& b : fwd) {
      f_at[b.s][b.j * n + b.ub] = t;
      StageCursor& c = cur[b.s];
      if (++c.f_ub == n) { c.f_ub = 0; c.f_mb++; }
      if (out && emitted < capacity) out[emitted] = tp_event{(int32_t)t, 0, b.s, b.ub, b.j};
      ++emitted;
    }
  }
  *count = emitted;
  return TP_OK;
}

int stage_workspace_query(const tp_stage_desc* desc, tp_sizes* out) {
  if (!out) return fail(TP_EINVAL, "null output");
  Plan p;
  int rc = make_plan(desc, &p);
  if (rc) return rc;
  *out = p.sizes;
  return TP_OK;
}

int stage_init(const tp_stage_desc* desc, const tp_buffers* bufs, void* hip_stream, tp_stage** out) {
  if (!out) return fail(TP_EINVAL, "null output");
  *out = nullptr;
  tp_stage* st = new (std::nothrow) tp_stage();
  if (!st) return fail(TP_EINVAL, "out of host memory");
  int rc = make_plan(desc, &st->plan);
  if (rc) { delete st; return rc; }
  st->desc = *desc;
  st->stream = (hipStream_t)hip_stream;
  // bufs == NULL: bookkeeping only (host tests of versions, slots and reference counts);
  // no kernel is ever launched on such a stage.
  st->dry = bufs == nullptr;
  if (bufs) {
    st->bufs = *bufs;
    const bool bf = desc->dtype == TP_BF16;
    if (!bufs->ring_dev || !bufs->momentum_dev || !bufs->grad_dev || !bufs->act_dev || !bufs->scratch_dev ||
        !bufs->diag_dev || (bf && !bufs->wfwd_dev) || (desc->policy != TP_LATEST && !bufs->wbwd_dev)) {
      delete st;
      return fail(TP_EINVAL, "null device buffer");
    }
    {  // the block of zeros that convolution padding reads
      hipError_t e = hipMemsetAsync((void*)st->zeros(), 0, 256, st->stream);
      if (e != hipSuccess) { delete st; return fail(TP_EHIP, "memset: %s", hipGetErrorString(e)); }
    }
    if (bf) {
      hipError_t e = tp::launch_convert(st->stream, tp::ELT_BF16, st->plan.sizes.param_count, st->ring(0),
                                        bufs->wfwd_dev);
      if (e != hipSuccess) { delete st; return fail(TP_EHIP, "convert: %s", hipGetErrorString(e)); }
    }
  } else {
    std::memset(&st->bufs, 0, sizeof(st->bufs));
  }
  st->slots[0].occupied = true;
  st->slots[0].version = 0;
  st->slots[0].refcnt = 0;
  *out = st;
  return TP_OK;
}

int stage_destroy(tp_stage* st) {
  if (!st) return fail(TP_EINVAL, "null stage");
  for (int k = 0; k < TP_MAX_FORWARD_STREAMS; ++k) {
    if (st->fwd_stream[k]) (void)hipStreamSynchronize(st->fwd_stream[k]);  // nothing of this stage is left on the caller's streams
    if (st->ev_fwd[k]) (void)hipEventDestroy(st->ev_fwd[k]);
    for (int q = 0; q < TP_MAX_IN_FLIGHT; ++q)
      if (st->ev_slot[q][k]) (void)hipEventDestroy(st->ev_slot[q][k]);
  }
  if (st->ev_main) (void)hipEventDestroy(st->ev_main);
  for (ProfEntry& e : st->prof_pool) {
    (void)hipEventDestroy(e.start);
    (void)hipEventDestroy(e.stop);
  }
  delete st;
  return TP_OK;
}

int stage_set_forward_streams(tp_stage* st, void* const* hip_streams, int32_t count) {
  if (!st) return fail(TP_EINVAL, "null stage");
  if (st->dry) return fail(TP_ESTATE, "a stage without device buffers launches nothing");
  if (count < 0 || count > TP_MAX_FORWARD_STREAMS) return fail(TP_EINVAL, "0 .. %d forward streams", TP_MAX_FORWARD_STREAMS);
  if (count > 0 && !hip_streams) return fail(TP_EINVAL, "null stream list");
  for (int k = 0; k < count; ++k) {
    if (!hip_streams[k] || (hipStream_t)hip_streams[k] == st->stream)
      return fail(TP_EINVAL, "a forward stream must be a stream of its own, not null and not the stage's");
    for (int q = 0; q < k; ++q)
      if (hip_streams[q] == hip_streams[k]) return fail(TP_EINVAL, "forward streams %d and %d are the same", q, k);
  }
  if (count > 0) {
    if (st->desc.policy == TP_TIMEPREST)
      return fail(TP_EINVAL, "forward passes on versions other than the latest share one compute copy: one stream only");
    for (const LayerPlan& lp : st->plan.layers)
      if (lp.d.type == TP_LAYER_ATTENTION)
        return fail(TP_EINVAL, "the forward kernels of attention layers share their scratch memory: one stream only");
  }
  if (int rc = join_forwards(st)) return rc;  // streams given earlier are drained into the stage's first
  if (count > 0 && !st->ev_main) HIP_TRY(hipEventCreateWithFlags(&st->ev_main, hipEventDisableTiming));
  for (int k = 0; k < count; ++k) {
    if (!st->ev_fwd[k]) HIP_TRY(hipEventCreateWithFlags(&st->ev_fwd[k], hipEventDisableTiming));
    for (int q = 0; q < st->desc.max_in_flight; ++q)
      if (!st->ev_slot[q][k]) HIP_TRY(hipEventCreateWithFlags(&st->ev_slot[q][k], hipEventDisableTiming));
  }
  for (int k = 0; k < TP_MAX_FORWARD_STREAMS; ++k) st->fwd_stream[k] = k < count ? (hipStream_t)hip_streams[k] : nullptr;
  st->fwd_streams = count;
  st->main_dirty = true;
  return TP_OK;
}

int stage_forward_join(tp_stage* st) {
  if (!st) return fail(TP_EINVAL, "null stage");
  if (st->dry) return TP_OK;
  return join_forwards(st);
}

int stash_push(tp_stage* st, uint64_t version, uint32_t* slot) {
  if (!st) return fail(TP_EINVAL, "null stage");
  int s = st->find_slot(version);
  if (s < 0) return fail(TP_ENOVERSION, "version %llu is not in the ring", (unsigned long long)version);
  st->slots[s].refcnt++;
  if (slot) *slot = (uint32_t)s;
  return TP_OK;
}

int stash_evict(tp_stage* st, uint64_t version) {
  if (!st) return fail(TP_EINVAL, "null stage");
  int s = st->find_slot(version);
  if (s < 0) return fail(TP_ENOVERSION, "version %llu is not in the ring", (unsigned long long)version);
  Slot& sl = st->slots[s];
  // Users the stage itself holds: mini-batches between their forward and their backward (Section "Memory
  // Overhead": their stale version stays until their intermediate weights are built).  Only pins taken
  // with stash_push can be dropped from outside.
  uint32_t own = 0;
  for (const InFlight& f : st->inflight)
    if (f.pinned && f.v_f == version) ++own;
  if (sl.refcnt > own) sl.refcnt--;
  else if (own > 0)
    return fail(TP_EBUSY, "version %llu is held by %u mini-batches in flight", (unsigned long long)version, own);
  if (sl.refcnt > 0) return fail(TP_EBUSY, "version %llu still has %u users", (unsigned long long)version, sl.refcnt);
  if (version == st->latest) return fail(TP_EBUSY, "version %llu is the latest", (unsigned long long)version);
  sl.occupied = false;
  return TP_OK;
}

int stage_input_ptr(tp_stage* st, uint64_t mb_id, uint32_t ub_idx, void** x_dev) {
  if (!st || !x_dev) return fail(TP_EINVAL, "null argument");
  if (ub_idx >= (uint32_t)st->desc.n) return fail(TP_EINVAL, "micro-batch index %u out of range", ub_idx);
  InFlight* f = st->find_mb(mb_id);
  int q;
  if (f) {
    q = f->act_slot;
  } else {
    // the slot the mini-batch will get when its first forward arrives
    q = -1;
    for (int i = 0; i < st->desc.max_in_flight; ++i)
      if (!st->act_used[i]) { q = i; break; }
    if (q < 0) return fail(TP_ESTATE, "more than %d mini-batches in flight", st->desc.max_in_flight);
  }
  const LayerPlan& l0 = st->plan.layers[0];
  *x_dev = st->dry ? nullptr
                   : st->act_slot(q) + l0.x_off + (uint64_t)ub_idx * st->desc.mb * l0.in_elems * st->plan.elt_size;
  return TP_OK;
}

int stage_saved_input_ptr(tp_stage* st, uint64_t mb_id, uint32_t ub_idx, int32_t layer, void** x_dev, uint64_t* bytes) {
  if (!st || !x_dev) return fail(TP_EINVAL, "null argument");
  if (layer < 0 || layer >= st->desc.num_layers) return fail(TP_EINVAL, "layer %d out of range", layer);
  InFlight* f = st->find_mb(mb_id);
  if (!f || ub_idx >= f->forwards)
    return fail(TP_ESTATE, "micro-batch %u of mini-batch %llu has not been forwarded (or its backward is done)", ub_idx,
                (unsigned long long)mb_id);
  const LayerPlan& lp = st->plan.layers[layer];
  const uint64_t nbytes = (uint64_t)st->desc.mb * lp.in_elems * st->plan.elt_size;
  if (bytes) *bytes = nbytes;
  *x_dev = st->dry ? nullptr : st->act_slot(f->act_slot) + lp.x_off + (uint64_t)ub_idx * nbytes;
  if (!st->dry)
    if (int rc = join_forwards(st)) return rc;  // whoever reads it on the stage's stream sees every forward enqueued so far
  return TP_OK;
}

}  // extern "C"

namespace {
// bf16 compute copy of a version that is not the latest (TP_TIMEPREST): converted into wbwd_dev on demand
int old_version_copy(tp_stage* st, uint64_t v, int slot, const char** out) {
  if (!(st->copy_valid && st->copy_version == v)) {
    ProfScope ps(st, TP_K_COPY);
    HIP_TRY(tp::launch_convert(st->stream, tp::ELT_BF16, st->plan.sizes.param_count, st->ring(slot), st->bufs.wbwd_dev));
    st->copy_valid = true;
    st->copy_version = v;
    st->wb_valid = false;
  }
  *out = (const char*)st->bufs.wbwd_dev;
  return TP_OK;
}

// `version`: TP_NONE = the latest version at the stage (every policy); a retained version under TP_TIMEPREST
int forward_impl(tp_stage* st, uint64_t mb_id, uint32_t ub_idx, const void* x_dev, void* y_dev, uint64_t version,
                 uint64_t* version_used) {
  if (!st->dry && (!x_dev || !y_dev)) return fail(TP_EINVAL, "null activation pointer");
  if (mb_id == TP_NONE) return fail(TP_EINVAL, "reserved mini-batch id");
  const tp_stage_desc& d = st->desc;
  if (version != TP_NONE && d.policy != TP_TIMEPREST)
    return fail(TP_EINVAL, "only TP_TIMEPREST names the version a pass reads");
  const uint64_t v_read = version == TP_NONE ? st->latest : version;
  if (st->find_slot(v_read) < 0)
    return fail(TP_ENOVERSION, "version %llu is not in the ring", (unsigned long long)v_read);
  InFlight* f = st->find_mb(mb_id);
  if (!f) {
    if (ub_idx != 0) return fail(TP_ESTATE, "mini-batch %llu: first forward must be micro-batch 0", (unsigned long long)mb_id);
    int q = -1;
    for (int i = 0; i < d.max_in_flight; ++i)
      if (!st->act_used[i]) { q = i; break; }
    if (q < 0) return fail(TP_ESTATE, "more than %d mini-batches in flight", d.max_in_flight);
    InFlight nf{mb_id, v_read, 0, q, false};
    if (stashing(d.policy)) {
      int rc = stash_push(st, st->latest, nullptr);   // the forward version stays until blended
      if (rc) return rc;
      nf.pinned = true;
    }
    st->act_used[q] = true;
    for (int k = 0; k < TP_MAX_FORWARD_STREAMS; ++k) st->slot_fwd[q][k] = false;
    st->inflight.push_back(nf);
    f = &st->inflight.back();
  }
  if (ub_idx != f->forwards || ub_idx >= (uint32_t)d.n)
    return fail(TP_ESTATE, "mini-batch %llu: expected micro-batch %u, got %u", (unsigned long long)mb_id, f->forwards, ub_idx);
  if (stashing(d.policy) && f->v_f != st->latest)
    return fail(TP_ESTATE, "an update landed between micro-batches of mini-batch %llu", (unsigned long long)mb_id);
  const uint64_t v = v_read;                           // the latest weights at the stage, unless the pass names its version
  if (version_used) *version_used = v;
  f->forwards++;
  if (st->dry) return TP_OK;

  const int slot = st->find_slot(v);
  const size_t es = st->plan.elt_size;
  const float* master = st->ring(slot);
  const char* wcopy = (const char*)master;
  if (d.dtype == TP_BF16) {
    wcopy = (const char*)st->bufs.wfwd_dev;
    if (v != st->latest)
      if (int rc = old_version_copy(st, v, slot, &wcopy)) return rc;
  }
  char* aslot = st->act_slot(f->act_slot);
  // With S forward streams of the caller's, micro-batch ub runs on forward stream ub % S and the stage's own stream
  // runs no forward, so that the backward pass of an earlier mini-batch can go on there meanwhile (not while kernels
  // are timed one by one).  A stage that holds one mini-batch at a time has no such backward pass: there the stage's
  // own stream takes a turn too (ub % (S + 1) == 0).  Every stream's forwards start behind everything the stage's
  // stream held before this run of forwards.
  hipStream_t fs = st->stream;
  int fsk = -1;  // index of the forward stream in use
  const int act_q = f->act_slot;
  if (st->fwd_streams > 0 && !st->prof_on) {
    if (st->main_dirty) {
      HIP_TRY(hipEventRecord(st->ev_main, st->stream));
      st->main_dirty = false;
    }
    fsk = d.max_in_flight == 1 ? (int)(ub_idx % (uint32_t)(st->fwd_streams + 1)) - 1 : (int)(ub_idx % (uint32_t)st->fwd_streams);
    if (fsk >= 0) {
      HIP_TRY(hipStreamWaitEvent(st->fwd_stream[fsk], st->ev_main, 0));
      fs = st->fwd_stream[fsk];
      st->fwd_pending[fsk] = true;
    }
  }
  // however the call ends, what it enqueued on a forward stream is what the mini-batch's backward pass waits for
  struct MarkForward {
    tp_stage* st; int q, k; hipStream_t s;
    ~MarkForward() {
      if (k < 0) return;
      if (hipEventRecord(st->ev_slot[q][k], s) == hipSuccess) st->slot_fwd[q][k] = true;
      else st->slot_event_lost = true;
    }
  } mark_forward{st, act_q, fsk, fs};
  const uint64_t row0 = (uint64_t)ub_idx * d.mb;
  const int L = d.num_layers;
  for (int l = 0; l < L; ++l) {
    const LayerPlan& lp = st->plan.layers[l];
    char* x_saved = aslot + lp.x_off + row0 * lp.in_elems * es;
    // a micro-batch that did not arrive in its workspace slot is copied there by its first GEMM
    const bool need_copy = l == 0 && x_dev != (const void*)x_saved;
    const void* x_in = need_copy ? x_dev : (const void*)x_saved;
    void* z_out = lp.z_off == UINT64_MAX ? nullptr : aslot + lp.z_off + row0 * lp.out_elems * es;
    void* a_out = (l == L - 1) ? y_dev : (void*)(aslot + st->plan.layers[l + 1].x_off + row0 * lp.out_elems * es);
    if (lp.d.type == TP_LAYER_DENSE) {
      ProfScope ps(st, TP_K_FPROP);
      // a dense layer followed by a plain residual add: the epilogue of the GEMM adds the kept tensor
      if (l + 1 < L && st->plan.layers[l + 1].d.type == TP_LAYER_RESIDUAL && st->plan.layers[l + 1].d.geom[1] == 1 &&
          st->plan.layers[l + 1].d.act == TP_ACT_NONE &&
          tp::fprop_add_supported(d.dtype, d.mb * lp.tokens, lp.d.out_features, lp.d.in_features)) {
        const LayerPlan& add = st->plan.layers[l + 1];
        const char* skip = aslot + st->plan.layers[add.skip_layer].x_off + row0 * add.in_elems * es;
        void* add_a = (l + 1 == L - 1) ? y_dev : (void*)(aslot + st->plan.layers[l + 2].x_off + row0 * add.out_elems * es);
        if ((((uintptr_t)skip | (uintptr_t)add_a) & 15) == 0) {
          HIP_TRY(tp::launch_fprop(fs, d.dtype, d.mb * lp.tokens, lp.d.out_features, lp.d.in_features, x_in,
                                   wcopy + lp.w_off * es, master + lp.b_off, lp.d.act, z_out, add_a,
                                   need_copy ? x_saved : nullptr, skip));
          ++l;  // the add is done
          continue;
        }
      }
      HIP_TRY(tp::launch_fprop(fs, d.dtype, d.mb * lp.tokens, lp.d.out_features, lp.d.in_features, x_in,
                               wcopy + lp.w_off * es, master + lp.b_off, lp.d.act, z_out, a_out,
                               need_copy ? x_saved : nullptr));
      continue;
    }
    if (lp.xpad_off != UINT64_MAX) {
      // few-channel first layer: what is kept for the backward pass is the 8-channel padded input
      const size_t px = (size_t)lp.d.geom[0] * lp.d.geom[1];
      uint16_t* x8 = (uint16_t*)(aslot + lp.xpad_off) + row0 * px * 8;
      {
        ProfScope ps(st, TP_K_COPY);
        HIP_TRY(tp::conv_c8_pad(fs, d.mb * px, lp.d.in_features, (const uint16_t*)x_in, x8));
      }
      ProfScope ps(st, TP_K_FPROP);
      if (lp.d.geom[2] == 7)
        HIP_TRY(tp::conv_stem_fprop(fs, d.mb, lp.d.geom[0], lp.d.geom[1], lp.d.in_features, lp.d.out_features, x8,
                                    (const uint16_t*)(wcopy + lp.w_off * es), master + lp.b_off, lp.d.act, (uint16_t*)z_out,
                                    (uint16_t*)a_out, (const uint16_t*)st->zeros()));
      else
        HIP_TRY(tp::conv_c8_fprop(fs, d.mb, lp.d.geom[0], lp.d.geom[1], lp.d.in_features, lp.d.out_features, x8,
                                  (const uint16_t*)(wcopy + lp.w_off * es), master + lp.b_off, lp.d.act, (uint16_t*)z_out,
                                  (uint16_t*)a_out, (const uint16_t*)st->zeros()));
      continue;
    }
    if (need_copy) {
      ProfScope ps(st, TP_K_COPY);
      HIP_TRY(tp::launch_copy(fs, x_dev, x_saved, (size_t)d.mb * lp.in_elems * es));
    }
    if (lp.d.type == TP_LAYER_LAYERNORM) {
      ProfScope ps(st, TP_K_NORM);
      float* stats = (float*)(aslot + lp.stat_off) + row0 * lp.stat_elems;
      HIP_TRY(tp::launch_layernorm_fwd(fs, d.dtype, (size_t)d.mb * lp.tokens, lp.d.in_features, x_saved,
                                       master + lp.w_off, master + lp.b_off, a_out, stats));
      continue;
    }
    if (lp.d.type == TP_LAYER_ATTENTION) {
      ProfScope ps(st, TP_K_ATTN);
      float* lse = (float*)(aslot + lp.stat_off) + row0 * lp.stat_elems;
      const int heads = lp.d.geom[1];
      HIP_TRY(tp::launch_attention_fwd(fs, d.dtype, d.mb, lp.tokens, heads, lp.d.out_features / heads, x_saved, a_out,
                                       lse, st->attn_scratch(), st->plan.attn_scratch_bytes));
      continue;
    }
    if (lp.d.type == TP_LAYER_RESIDUAL) {
      if (lp.skip_layer < 0) continue;  // begin: the next layer reads this layer's input in place
      if (lp.d.geom[1] == 2) continue;  // swap: this layer's input stays saved for the add, the next layer reads the begin's
      ProfScope ps(st, TP_K_ADD);
      const char* skip = aslot + st->plan.layers[lp.skip_layer].x_off + row0 * lp.in_elems * es;
      if (lp.d.act == TP_ACT_NONE)
        HIP_TRY(tp::launch_add(fs, d.dtype, (size_t)d.mb * lp.in_elems, x_saved, skip, a_out));
      else
        HIP_TRY(tp::launch_add_act(fs, d.dtype, (size_t)d.mb * lp.in_elems, x_saved, skip, lp.d.act, a_out, z_out));
      continue;
    }
    if (lp.d.type == TP_LAYER_BATCHNORM) {
      ProfScope ps(st, TP_K_NORM);
      const int C = lp.d.in_features;
      float* stats = (float*)(aslot + lp.stat_off) + (size_t)ub_idx * 2 * C;
      // a normalisation without activation followed by a residual add: one kernel forms act(bn(x) + kept tensor)
      // and act' of it, written where the add would have written them
      if (l + 1 < L && lp.d.act == TP_ACT_NONE && st->plan.layers[l + 1].d.type == TP_LAYER_RESIDUAL &&
          st->plan.layers[l + 1].d.geom[1] == 1 && tp::batchnorm_fwd_add_supported(d.dtype, (size_t)d.mb * lp.tokens, C)) {
        const LayerPlan& add = st->plan.layers[l + 1];
        const char* skip = aslot + st->plan.layers[add.skip_layer].x_off + row0 * add.in_elems * es;
        void* add_z = add.z_off == UINT64_MAX ? nullptr : aslot + add.z_off + row0 * add.out_elems * es;
        void* add_a = (l + 1 == L - 1) ? y_dev : (void*)(aslot + st->plan.layers[l + 2].x_off + row0 * add.out_elems * es);
        if ((((uintptr_t)x_saved | (uintptr_t)skip | (uintptr_t)add_a | (uintptr_t)add_z) & 15) == 0) {
          HIP_TRY(tp::launch_batchnorm_fwd(fs, d.dtype, (size_t)d.mb * lp.tokens, C, x_saved, master + lp.w_off,
                                           master + lp.b_off, add.d.act, add_a, add_z, stats, fsk < 0 ? st->partials() : st->fwd2_scratch(fsk), skip));
          ++l;  // the add is done
          continue;
        }
      }
      HIP_TRY(tp::launch_batchnorm_fwd(fs, d.dtype, (size_t)d.mb * lp.tokens, C, x_saved, master + lp.w_off,
                                       master + lp.b_off, lp.d.act, a_out, z_out, stats, fsk < 0 ? st->partials() : st->fwd2_scratch(fsk)));
      continue;
    }
    if (lp.d.type == TP_LAYER_CONV2D) {
      ProfScope ps(st, TP_K_FPROP);
      HIP_TRY(tp::launch_conv_fprop(fs, d.dtype, d.mb, lp.d.geom[0], lp.d.geom[1], lp.d.geom[2], lp.d.geom[3],
                                    lp.d.in_features, lp.d.out_features, x_saved, wcopy + lp.w_off * es, master + lp.b_off,
                                    lp.d.act, z_out, a_out, st->zeros()));
    } else if (lp.d.type == TP_LAYER_AVGPOOL) {
      ProfScope ps(st, TP_K_POOL);
      HIP_TRY(tp::launch_avgpool_fwd(fs, d.dtype, d.mb, lp.tokens, lp.d.in_features, x_saved, a_out));
    } else if (lp.d.type == TP_LAYER_SUBSAMPLE2) {
      ProfScope ps(st, TP_K_POOL);
      HIP_TRY(tp::launch_subsample_fwd(fs, d.dtype, d.mb, lp.d.geom[0], lp.d.geom[1], lp.d.in_features, x_saved,
                                       a_out));
    } else {
      ProfScope ps(st, TP_K_POOL);
      HIP_TRY(tp::launch_maxpool_fwd(fs, d.dtype, d.mb, lp.d.geom[0], lp.d.geom[1], lp.d.in_features, x_saved,
                                     a_out));
    }
  }
  return TP_OK;
}
}  // namespace

extern "C" {

int stage_forward(tp_stage* st, uint64_t mb_id, uint32_t ub_idx, const void* x_dev, void* y_dev,
                  uint64_t* version_used) {
  if (!st) return fail(TP_EINVAL, "null stage");
  return forward_impl(st, mb_id, ub_idx, x_dev, y_dev, TP_NONE, version_used);
}

int stage_forward_on(tp_stage* st, uint64_t mb_id, uint32_t ub_idx, uint64_t version, const void* x_dev, void* y_dev) {
  if (!st) return fail(TP_EINVAL, "null stage");
  if (version == TP_NONE) return fail(TP_EINVAL, "stage_forward_on needs a version");
  return forward_impl(st, mb_id, ub_idx, x_dev, y_dev, version, nullptr);
}

int stage_loss_softmax_ce(tp_stage* st, uint64_t mb_id, const void* logits_dev, const int32_t* labels_dev,
                          void* dlogits_dev, float* loss_dev) {
  if (!st) return fail(TP_EINVAL, "null stage");
  InFlight* f = st->find_mb(mb_id);
  if (!f || f->forwards != (uint32_t)st->desc.n)
    return fail(TP_ESTATE, "loss of mini-batch %llu needs all %d forwards", (unsigned long long)mb_id, st->desc.n);
  if (st->dry) return TP_OK;
  if (!logits_dev || !labels_dev || !dlogits_dev || !loss_dev) return fail(TP_EINVAL, "null pointer");
  if (int rc = join_forwards(st)) return rc;
  const int rows = st->desc.mb * st->desc.n;
  if (st->plan.layers.back().d.type != TP_LAYER_DENSE) return fail(TP_EINVAL, "the loss needs a dense last layer");
  const int classes = st->plan.layers.back().d.out_features;
  ProfScope ps(st, TP_K_LOSS);
  HIP_TRY(tp::launch_softmax_ce(st->stream, st->desc.dtype, rows, classes, logits_dev, labels_dev, dlogits_dev,
                                st->partials(), loss_dev));
  return TP_OK;
}

}  // extern "C"

namespace {
int backward_impl(tp_stage* st, uint64_t mb_id, const void* dy_dev, void* dx_dev, uint64_t version, uint32_t* delta_used) {
  const tp_stage_desc& d = st->desc;
  if (version != TP_NONE && d.policy != TP_TIMEPREST)
    return fail(TP_EINVAL, "only TP_TIMEPREST names the version a pass reads");
  InFlight* f = st->find_mb(mb_id);
  if (!f) return fail(TP_ESTATE, "mini-batch %llu is not in flight", (unsigned long long)mb_id);
  if (f->forwards != (uint32_t)d.n)
    return fail(TP_ESTATE, "mini-batch %llu: %u of %d forwards seen", (unsigned long long)mb_id, f->forwards, d.n);
  if (st->grad_pending) return fail(TP_ESTATE, "gradient of mini-batch %llu has not been applied yet", (unsigned long long)st->grad_mb);
  if (!st->dry && (!dy_dev || (d.needs_dx && !dx_dev))) return fail(TP_EINVAL, "null gradient pointer");

  // Which weights: V reads the latest; I blends the stashed forward version towards it; TiMePReSt reads the
  // version its backward pass started on, as it is.
  const uint64_t v_now = version == TP_NONE ? st->latest : version;
  const uint64_t v_f = stashing(d.policy) ? f->v_f : v_now;
  const uint32_t delta = (uint32_t)(v_now - v_f);
  const int slot_now = st->find_slot(v_now);
  const int slot_f = st->find_slot(v_f);
  if (slot_now < 0) return fail(TP_ENOVERSION, "version %llu is not in the ring", (unsigned long long)v_now);
  if (slot_f < 0) return fail(TP_ENOVERSION, "forward version %llu of mini-batch %llu is no longer stashed", (unsigned long long)v_f, (unsigned long long)mb_id);
  if (delta_used) *delta_used = delta;

  if (!st->dry) {
    // The stage's stream waits for the forwards of THIS mini-batch only: forwards of later mini-batches may still be
    // running on the forward streams and go on beside this pass (they share no buffer with it).
    st->main_dirty = true;
    if (st->slot_event_lost) {
      if (int rc = join_forwards(st)) return rc;
      st->slot_event_lost = false;
    }
    for (int k = 0; k < TP_MAX_FORWARD_STREAMS; ++k)
      if (st->slot_fwd[f->act_slot][k]) {
        HIP_TRY(hipStreamWaitEvent(st->stream, st->ev_slot[f->act_slot][k], 0));
        st->slot_fwd[f->act_slot][k] = false;
      }
    const size_t es = st->plan.elt_size;
    const uint64_t P = st->plan.sizes.param_count;
    const char* wb;
    if (delta == 0) {
      // no staleness: intermediate = stale = latest (bit for bit)
      wb = d.dtype == TP_BF16 ? (const char*)st->bufs.wfwd_dev : (const char*)st->ring(slot_now);
      if (d.dtype == TP_BF16 && v_now != st->latest)
        if (int rc = old_version_copy(st, v_now, slot_now, &wb)) return rc;
    } else if (st->wb_valid && st->wb_mb == mb_id && st->wb_vf == v_f && st->wb_vnow == v_now) {
      wb = (const char*)st->bufs.wbwd_dev;            // built by the fused update
    } else {
      double a, b;
      int rc = tp_blend_coefficients(d.policy, delta, d.lambda, &a, &b);
      if (rc) return rc;
      ProfScope ps(st, TP_K_BLEND);
      HIP_TRY(tp::launch_blend(st->stream, d.dtype, P, st->ring(slot_f), st->ring(slot_now), (float)a, (float)b, st->bufs.wbwd_dev));
      st->copy_valid = false;
      wb = (const char*)st->bufs.wbwd_dev;
    }

    const int rows = d.mb * d.n;
    const int L = d.num_layers;
    char* aslot = st->act_slot(f->act_slot);
    float* g = (float*)st->bufs.grad_dev;
    const void* dz = nullptr;  // gradient w.r.t. the pre-activation output of layer l (or pooled output)
    // Three temporaries: the gradient in hand, the one being formed, and the one a residual add has
    // set aside for the matching begin.
    const void* pinned = nullptr;
    bool begin_added = false;  // the layer behind a residual begin has already added the gradient that was set aside
    auto scratch_for = [&](const void* cur) -> void* {
      for (int i = 0; i < 3; ++i)
        if (st->dz_buf(i) != cur && st->dz_buf(i) != pinned) return st->dz_buf(i);
      return nullptr;
    };
    // scale of a layer normalisation in the backward pass: the intermediate weight, formed in fp32
    double ca = 1.0, cb = 0.0;
    if (delta != 0) {
      int rc = tp_blend_coefficients(d.policy, delta, d.lambda, &ca, &cb);
      if (rc) return rc;
    }
    // Sums of partials are put off to one launch behind the loop (when the plan has room for every layer's partials
    // side by side): `hold(need)` hands out the next `need` floats, SumsDeferred makes the launchers record their sums.
    const bool defer = st->plan.deferred_floats > 0;
    st->sum_jobs.clear();
    uint64_t held = 0;
    bool held_overflow = false;
    auto hold = [&](uint64_t need) -> float* {
      if (!defer) return st->partials();
      if (held + need > st->plan.deferred_floats) { held_overflow = true; return st->partials(); }
      float* at = st->deferred_partials() + held;
      held += need;
      return at;
    };
    struct SumsDeferred {
      explicit SumsDeferred(std::vector<tp::SumJob>* jobs) { tp::set_sum_sink(jobs); }
      ~SumsDeferred() { tp::set_sum_sink(nullptr); }
    };
    std::vector<tp::SumJob>* sink = defer ? &st->sum_jobs : nullptr;
    bool bias_summed = false;  // the bias gradient of the layer coming up has already been formed (or recorded)
    {
      const LayerPlan& last = st->plan.layers[L - 1];
      if (last.d.act == TP_ACT_NONE) {
        dz = dy_dev;
      } else {
        ProfScope ps(st, TP_K_ACT_BWD);
        void* buf = scratch_for(nullptr);
        const void* dlast = aslot + last.z_off;
        // a dense or convolution layer: the pass that forms dz = dy (.) act'(z) also takes its column sums
        const bool with_bias = (last.d.type == TP_LAYER_DENSE || last.d.type == TP_LAYER_CONV2D) &&
                               tp::act_backward_colsum_supported(d.dtype, last.d.out_features) &&
                               ((((uintptr_t)dy_dev | (uintptr_t)dlast | (uintptr_t)buf) & 15) == 0);
        if (with_bias) {
          const int grad_rows = last.d.type == TP_LAYER_CONV2D ? rows * (int)conv_out_px(last.d) : rows * last.tokens;
          SumsDeferred later(sink);
          HIP_TRY(tp::launch_act_backward_colsum(st->stream, d.dtype, grad_rows, last.d.out_features, dy_dev, dlast, buf, 0,
                                                 g + last.b_off, hold(deferred_need(d, last).bias)));
          bias_summed = true;
        } else {
          HIP_TRY(tp::launch_act_backward(st->stream, d.dtype, (size_t)rows * last.out_elems, dy_dev, dlast, buf));
        }
        dz = buf;
      }
    }
    for (int l = L - 1; l >= 0; --l) {
      const LayerPlan& lp = st->plan.layers[l];
      const DeferredNeed need = deferred_need(d, lp);
      if (held_overflow) return fail(TP_ESTATE, "partial sums of the backward pass outgrew their plan");
      // where the gradient w.r.t. this layer's input goes, and what it is multiplied with on the way
      const bool to_caller = l == 0;
      const bool no_dx = to_caller && !d.needs_dx;
      if (no_dx && (lp.d.type == TP_LAYER_MAXPOOL2 || lp.d.type == TP_LAYER_SUBSAMPLE2 || lp.d.type == TP_LAYER_ATTENTION ||
                    lp.d.type == TP_LAYER_AVGPOOL))
        break;
      // what the gradient w.r.t. this layer's input is multiplied with: the saved act'(z) of the previous layer, or
      // (dmask = 1) that layer's saved ReLU output, which is this layer's own saved input
      const void* dprev = nullptr;
      int dmask = 0;
      if (l > 0) {
        const LayerPlan& prev = st->plan.layers[l - 1];
        if (prev.z_off != UINT64_MAX) {
          dprev = aslot + prev.z_off;
        } else if (prev.relu_out) {
          dprev = aslot + lp.x_off;
          dmask = 1;
        }
      }
      void* dst = to_caller && !no_dx ? dx_dev : scratch_for(dz);
      auto through_activation = [&](void* grad) -> int {  // dz_prev = dx (.) act'(z_prev), in place
        if (!dprev) return TP_OK;
        ProfScope ps(st, TP_K_ACT_BWD);
        HIP_TRY(tp::launch_act_backward(st->stream, d.dtype, (size_t)rows * lp.in_elems, grad, dprev, grad, dmask));
        return TP_OK;
      };
      if (lp.d.type == TP_LAYER_MAXPOOL2) {
        // the activation in front of the pooling is passed by the same kernel where it takes 16-byte units
        const bool fused = dprev && tp::maxpool_bwd_fuses_activation(d.dtype, lp.d.in_features) &&
                           ((((uintptr_t)dz | (uintptr_t)dst | (uintptr_t)dprev) & 15) == 0);
        {
          ProfScope ps(st, TP_K_POOL);
          HIP_TRY(tp::launch_maxpool_bwd(st->stream, d.dtype, rows, lp.d.geom[0], lp.d.geom[1], lp.d.in_features,
                                         aslot + lp.x_off, dz, dst, fused ? dprev : nullptr, dmask));
        }
        if (!fused)
          if (int rc = through_activation(dst)) return rc;
        dz = dst;
        continue;
      }
      if (lp.d.type == TP_LAYER_AVGPOOL) {
        {
          ProfScope ps(st, TP_K_POOL);
          HIP_TRY(tp::launch_avgpool_bwd(st->stream, d.dtype, rows, lp.tokens, lp.d.in_features, dz, dst));
        }
        if (int rc = through_activation(dst)) return rc;
        dz = dst;
        continue;
      }
      if (lp.d.type == TP_LAYER_SUBSAMPLE2) {
        {
          ProfScope ps(st, TP_K_POOL);
          HIP_TRY(tp::launch_subsample_bwd(st->stream, d.dtype, rows, lp.d.geom[0], lp.d.geom[1], lp.d.in_features, dz, dst));
        }
        if (int rc = through_activation(dst)) return rc;
        dz = dst;
        continue;
      }
      if (lp.d.type == TP_LAYER_RESIDUAL && lp.d.geom[1] == 2) {
        // swap: what came down the second branch is the gradient w.r.t. the tensor remembered at the begin and
        // waits for it; the gradient set aside at the add goes on into the main branch.
        const void* main_grad = pinned;
        pinned = dz;
        if (dprev) {
          void* buf = scratch_for(main_grad);  // not the one just set aside, not the one read
          ProfScope ps(st, TP_K_ACT_BWD);
          HIP_TRY(tp::launch_act_backward(st->stream, d.dtype, (size_t)rows * lp.in_elems, main_grad, dprev, buf, dmask));
          main_grad = buf;
        }
        dz = main_grad;
        continue;
      }
      if (lp.d.type == TP_LAYER_RESIDUAL) {
        if (lp.skip_layer >= 0) {  // add: the gradient goes on unchanged and is set aside for the begin
          pinned = dz;
          if (dprev) {
            ProfScope ps(st, TP_K_ACT_BWD);
            HIP_TRY(tp::launch_act_backward(st->stream, d.dtype, (size_t)rows * lp.in_elems, dz, dprev, dst, dmask));
            dz = dst;
          }
          continue;
        }
        if (no_dx) break;
        if (begin_added) {  // dz already holds the sum (it lies in one of the temporaries)
          begin_added = false;
          pinned = nullptr;
          if (int rc = through_activation(const_cast<void*>(dz))) return rc;
          continue;
        }
        if (dprev && ((((uintptr_t)dz | (uintptr_t)pinned | (uintptr_t)dst | (uintptr_t)dprev) & 15) == 0)) {
          // the two gradients meet and pass the activation in front of the begin in one kernel
          ProfScope ps(st, TP_K_ACT_BWD);
          HIP_TRY(tp::launch_act_backward(st->stream, d.dtype, (size_t)rows * lp.in_elems, dz, dprev, dst, dmask, pinned));
          pinned = nullptr;
        } else {
          {
            ProfScope ps(st, TP_K_ADD);
            HIP_TRY(tp::launch_add(st->stream, d.dtype, (size_t)rows * lp.in_elems, dz, pinned, dst));
          }
          pinned = nullptr;
          if (int rc = through_activation(dst)) return rc;
        }
        dz = dst;
        continue;
      }
      if (lp.d.type == TP_LAYER_LAYERNORM) {
        const float* gl = st->ring(slot_now) + lp.w_off;
        const float* gs = delta != 0 ? st->ring(slot_f) + lp.w_off : gl;
        {
          // a residual begin right in front (not the stage's first layer): the gradient set aside at the add is
          // added by this kernel, where the begin would have needed a launch of its own
          const bool fuse = l >= 2 && pinned && st->plan.layers[l - 1].d.type == TP_LAYER_RESIDUAL &&
                            st->plan.layers[l - 1].d.geom[1] == 0 && tp::layernorm_bwd_add_supported(d.dtype, lp.d.in_features) &&
                            ((((uintptr_t)dz | (uintptr_t)pinned | (uintptr_t)dst) & 15) == 0);
          ProfScope ps(st, TP_K_NORM);
          SumsDeferred later(sink);
          HIP_TRY(tp::launch_layernorm_bwd(st->stream, d.dtype, (size_t)rows * lp.tokens, lp.d.in_features, dz, aslot + lp.x_off,
                                           (const float*)(aslot + lp.stat_off), gs, gl, (float)ca, (float)cb, dst,
                                           g + lp.w_off, g + lp.b_off, hold(need.norm), fuse ? pinned : nullptr));
          begin_added = fuse;
        }
        if (no_dx) break;
        if (int rc = through_activation(dst)) return rc;
        dz = dst;
        continue;
      }
      if (lp.d.type == TP_LAYER_BATCHNORM) {
        const int C = lp.d.in_features;
        const float* gl = st->ring(slot_now) + lp.w_off;
        const float* gs = delta != 0 ? st->ring(slot_f) + lp.w_off : gl;
        const size_t seg_rows = (size_t)d.mb * lp.tokens;        // the statistics belong to one micro-batch
        const size_t bn_scratch = tp::batchnorm_scratch_floats(seg_rows, C, d.n);
        // [n][2*C], then [n][C]: with the sums put off they wait in this layer's own block, else behind the scratch
        // of the streaming kernels
        float* sums = defer ? hold(need.norm) : st->partials() + bn_scratch;
        float* dx_sums = nullptr;
        {
          ProfScope ps(st, TP_K_NORM);
          if (tp::batchnorm_fused_bwd_supported(d.dtype, seg_rows, C)) {
            // a dense or convolution layer without activation right in front: its bias gradient is the column sum
            // of the dx formed here, which this kernel holds in registers anyway
            if (defer && l > 0 && !dprev && !no_dx) {
              const tp_layer_desc& pl = st->plan.layers[l - 1].d;
              if ((pl.type == TP_LAYER_DENSE || pl.type == TP_LAYER_CONV2D) && pl.out_features == C)
                dx_sums = sums + (size_t)d.n * 2 * C;
            }
            HIP_TRY(tp::launch_batchnorm_bwd_fused(st->stream, d.dtype, seg_rows, C, d.n, dz, aslot + lp.x_off,
                                                   (const float*)(aslot + lp.stat_off), gs, gl, (float)ca, (float)cb, dst, sums,
                                                   dx_sums));
          } else {
            HIP_TRY(tp::launch_batchnorm_bwd(st->stream, d.dtype, seg_rows, C, d.n, dz, aslot + lp.x_off,
                                             (const float*)(aslot + lp.stat_off), gs, gl, (float)ca, (float)cb, dst, sums,
                                             st->partials()));
          }
          SumsDeferred later(sink);
          if (lp.b_off == lp.w_off + (uint64_t)C) {  // scale and shift gradients lie side by side: one launch sums both
            HIP_TRY(tp::launch_sum_partials_strided(st->stream, 2 * (size_t)C, d.n, sums, 2 * (size_t)C, g + lp.w_off));
          } else {
            HIP_TRY(tp::launch_sum_partials_strided(st->stream, (size_t)C, d.n, sums, 2 * (size_t)C, g + lp.w_off));
            HIP_TRY(tp::launch_sum_partials_strided(st->stream, (size_t)C, d.n, sums + C, 2 * (size_t)C, g + lp.b_off));
          }
          if (dx_sums) {
            HIP_TRY(tp::launch_sum_partials_strided(st->stream, (size_t)C, d.n, dx_sums, (size_t)C,
                                                    g + st->plan.layers[l - 1].b_off));
            bias_summed = true;
          }
        }
        if (no_dx) break;
        if (int rc = through_activation(dst)) return rc;
        dz = dst;
        continue;
      }
      if (lp.d.type == TP_LAYER_ATTENTION) {
        const int heads = lp.d.geom[1];
        {
          ProfScope ps(st, TP_K_ATTN);
          HIP_TRY(tp::launch_attention_bwd(st->stream, d.dtype, rows, lp.tokens, heads, lp.d.out_features / heads,
                                           aslot + lp.x_off, aslot + st->plan.layers[l + 1].x_off, dz,
                                           (const float*)(aslot + lp.stat_off), dst, st->attn_scratch(),
                                           st->plan.attn_scratch_bytes));
        }
        if (int rc = through_activation(dst)) return rc;
        dz = dst;
        continue;
      }
      const int grad_rows = lp.d.type == TP_LAYER_CONV2D ? rows * (int)conv_out_px(lp.d) : rows * lp.tokens;
      if (bias_summed) {
        bias_summed = false;
      } else {
        ProfScope ps(st, TP_K_COLSUM);
        SumsDeferred later(sink);
        HIP_TRY(tp::launch_colsum(st->stream, d.dtype, grad_rows, lp.d.out_features, dz, g + lp.b_off, hold(need.bias)));
      }
      {
        ProfScope ps(st, TP_K_WGRAD);
        SumsDeferred later(sink);
        float* part = hold(need.weight);
        if (lp.d.type == TP_LAYER_DENSE)
          HIP_TRY(tp::launch_wgrad(st->stream, d.dtype, grad_rows, lp.d.out_features, lp.d.in_features, dz, aslot + lp.x_off,
                                   g + lp.w_off, part));
        else if (lp.xpad_off != UINT64_MAX && lp.d.geom[2] == 7)
          HIP_TRY(tp::conv_stem_wgrad(st->stream, rows, lp.d.geom[0], lp.d.geom[1], lp.d.in_features, lp.d.out_features,
                                      (const uint16_t*)dz, (const uint16_t*)(aslot + lp.xpad_off), g + lp.w_off, part,
                                      (const uint16_t*)st->zeros()));
        else if (lp.xpad_off != UINT64_MAX)
          HIP_TRY(tp::conv_c8_wgrad(st->stream, rows, lp.d.geom[0], lp.d.geom[1], lp.d.in_features, lp.d.out_features,
                                    (const uint16_t*)dz, (const uint16_t*)(aslot + lp.xpad_off), g + lp.w_off, part,
                                    (const uint16_t*)st->zeros()));
        else
          HIP_TRY(tp::launch_conv_wgrad(st->stream, d.dtype, rows, lp.d.geom[0], lp.d.geom[1], lp.d.geom[2], lp.d.geom[3],
                                        lp.d.in_features, lp.d.out_features, dz, aslot + lp.x_off, g + lp.w_off, part,
                                        st->zeros()));
      }
      if (no_dx) break;
      {
        ProfScope ps(st, TP_K_DGRAD);
        if (lp.d.type == TP_LAYER_DENSE)
          HIP_TRY(tp::launch_dgrad(st->stream, d.dtype, grad_rows, lp.d.out_features, lp.d.in_features, dz, wb + lp.w_off * es,
                                   dprev, dst, dmask));
        else
          HIP_TRY(tp::launch_conv_dgrad(st->stream, d.dtype, rows, lp.d.geom[0], lp.d.geom[1], lp.d.geom[2], lp.d.geom[3],
                                        lp.d.in_features, lp.d.out_features, dz, wb + lp.w_off * es, dprev, dst, st->zeros(),
                                        dmask));
      }
      dz = dst;
    }
    if (held_overflow) return fail(TP_ESTATE, "partial sums of the backward pass outgrew their plan");
    if (!st->sum_jobs.empty()) {
      ProfScope ps(st, TP_K_SUMS);
      HIP_TRY(tp::launch_sum_jobs(st->stream, st->sum_jobs.data(), st->sum_jobs.size()));
      st->sum_jobs.clear();
    }
  }

  st->wb_valid = false;
  // The intermediate weights are built: the mini-batch no longer needs its stashed version.
  if (f->pinned) {
    Slot& sl = st->slots[slot_f];
    if (sl.refcnt > 0) sl.refcnt--;
    st->evict_if_unused(v_f);
  }
  st->act_used[f->act_slot] = false;
  st->inflight.erase(st->inflight.begin() + (f - st->inflight.data()));
  st->grad_pending = true;
  st->grad_mb = mb_id;
  return TP_OK;
}
}  // namespace

extern "C" {

int stage_backward(tp_stage* st, uint64_t mb_id, const void* dy_dev, void* dx_dev, uint32_t* delta_used) {
  if (!st) return fail(TP_EINVAL, "null stage");
  return backward_impl(st, mb_id, dy_dev, dx_dev, TP_NONE, delta_used);
}

int stage_backward_on(tp_stage* st, uint64_t mb_id, uint64_t version, const void* dy_dev, void* dx_dev) {
  if (!st) return fail(TP_EINVAL, "null stage");
  if (version == TP_NONE) return fail(TP_EINVAL, "stage_backward_on needs a version");
  return backward_impl(st, mb_id, dy_dev, dx_dev, version, nullptr);
}

}  // extern "C"

namespace {
// The update (Section "Pipeline Parallelism": after every mini-batch) with the look-ahead blend (Eq. 1-2);
// `partials`: where the update kernel leaves the block partials of its diagnostics.
int blend_update_impl(tp_stage* st, uint64_t mb_id_done, uint64_t mb_id_next_bwd, uint64_t* new_version, float* partials) {
  const tp_stage_desc& d = st->desc;
  if (!st->grad_pending || st->grad_mb != mb_id_done)
    return fail(TP_ESTATE, "no gradient of mini-batch %llu is pending", (unsigned long long)mb_id_done);
  const uint64_t v = st->latest;
  const int C = d.ring_capacity;
  const int slot_old = (int)(v % C), slot_new = (int)((v + 1) % C);
  if (slot_new == slot_old) {
    if (st->slots[slot_old].refcnt != 0)
      return fail(TP_EFULL, "ring of capacity %d cannot keep version %llu for its %u users", C, (unsigned long long)v, st->slots[slot_old].refcnt);
  } else if (st->slots[slot_new].occupied) {
    return fail(TP_EFULL, "ring slot %d still holds version %llu", slot_new, (unsigned long long)st->slots[slot_new].version);
  }
  // Optional look-ahead: W_b of the next backward, with W[v+1] as the latest weights.
  bool blend = false;
  uint64_t vf_next = 0;
  double a = 0.0, b = 1.0;
  int slot_stale = -1;
  if (mb_id_next_bwd != TP_NONE && stashing(d.policy)) {
    InFlight* nx = st->find_mb(mb_id_next_bwd);
    if (!nx) return fail(TP_ESTATE, "mini-batch %llu is not in flight", (unsigned long long)mb_id_next_bwd);
    vf_next = nx->v_f;
    slot_stale = st->find_slot(vf_next);
    if (slot_stale < 0) return fail(TP_ENOVERSION, "version %llu is not in the ring", (unsigned long long)vf_next);
    const uint32_t delta = (uint32_t)(v + 1 - vf_next);
    int rc = tp_blend_coefficients(d.policy, delta, d.lambda, &a, &b);
    if (rc) return rc;
    blend = slot_stale != slot_new;                    // never read the slot being overwritten
  }
  if (!st->dry) {
    if (int rc = join_forwards(st)) return rc;  // forwards on the second stream still read the weights being replaced
    tp::UpdateArgs u;
    u.count = st->plan.sizes.param_count;
    u.g = (const float*)st->bufs.grad_dev;
    u.m = (float*)st->bufs.momentum_dev;
    u.w_old = st->ring(slot_old);
    u.w_new = st->ring(slot_new);
    u.w_stale = blend ? st->ring(slot_stale) : nullptr;
    u.wfwd = d.dtype == TP_BF16 ? st->bufs.wfwd_dev : nullptr;
    u.wb = blend ? st->bufs.wbwd_dev : nullptr;
    u.lr = (float)d.lr;
    u.mu = (float)d.momentum;
    u.alpha = (float)a;
    u.beta = (float)b;
    u.partials = partials;
    u.diag = (double*)st->bufs.diag_dev;
    ProfScope ps(st, TP_K_UPDATE);
    HIP_TRY(tp::launch_update(st->stream, d.dtype, u));
  }
  st->wb_valid = blend;
  if (blend) st->copy_valid = false;
  st->wb_mb = blend ? mb_id_next_bwd : TP_NONE;
  st->wb_vf = vf_next;
  st->wb_vnow = v + 1;
  // bookkeeping: the new version takes its slot; the old one goes unless still stashed
  st->slots[slot_new].occupied = true;
  st->slots[slot_new].version = v + 1;
  st->slots[slot_new].refcnt = 0;
  st->latest = v + 1;
  if (slot_new != slot_old) st->evict_if_unused(v);
  st->grad_pending = false;
  if (new_version) *new_version = v + 1;
  return TP_OK;
}
}  // namespace

extern "C" {

int stage_blend_update(tp_stage* st, uint64_t mb_id_done, uint64_t mb_id_next_bwd, uint64_t* new_version) {
  if (!st) return fail(TP_EINVAL, "null stage");
  return blend_update_impl(st, mb_id_done, mb_id_next_bwd, new_version, st->dry ? nullptr : st->partials());
}

int stage_blend_update_noalloc(tp_stage* st, uint64_t mb_id_done, uint64_t mb_id_next_bwd, uint64_t* new_version) {
  if (!st) return fail(TP_EINVAL, "null stage");
  if (st->plan.sizes.param_count > TP_NOALLOC_MAX_PARAMS)
    return fail(TP_EINVAL, "stage_blend_update_noalloc takes at most %llu parameters per version, this stage has %llu",
                (unsigned long long)TP_NOALLOC_MAX_PARAMS, (unsigned long long)st->plan.sizes.param_count);
  float* partials = nullptr;
  if (!st->dry) {
    size_t floats = 0;
    hipError_t e = tp::update_static_scratch(&partials, &floats);
    if (e != hipSuccess) return fail(TP_EHIP, "address of the library's scratch array: %s", hipGetErrorString(e));
    if (floats < tp::update_scratch_floats()) return fail(TP_EINVAL, "the library's scratch array is too small");
  }
  return blend_update_impl(st, mb_id_done, mb_id_next_bwd, new_version, partials);
}

int stage_query(const tp_stage* st, tp_state* out) {
  if (!st || !out) return fail(TP_EINVAL, "null argument");
  std::memset(out, 0, sizeof(*out));
  out->latest_version = st->latest;
  out->ring_capacity = st->desc.ring_capacity;
  for (int i = 0; i < st->desc.ring_capacity; ++i) {
    out->slot_occupied[i] = st->slots[i].occupied ? 1 : 0;
    out->slot_version[i] = st->slots[i].version;
    out->slot_refcnt[i] = st->slots[i].refcnt;
  }
  out->num_in_flight = (int32_t)st->inflight.size();
  for (size_t i = 0; i < st->inflight.size() && i < TP_MAX_IN_FLIGHT; ++i) {
    out->in_flight_mb[i] = st->inflight[i].mb_id;
    out->in_flight_vf[i] = st->inflight[i].v_f;
    out->in_flight_forwards[i] = st->inflight[i].forwards;
  }
  out->wb_ready_mb = st->wb_valid ? st->wb_mb : TP_NONE;
  return TP_OK;
}

int stage_export_params(tp_stage* st, uint64_t version, void* dst_dev) {
  if (!st) return fail(TP_EINVAL, "null stage");
  int s = st->find_slot(version);
  if (s < 0) return fail(TP_ENOVERSION, "version %llu is not in the ring", (unsigned long long)version);
  if (st->dry) return TP_OK;
  if (!dst_dev) return fail(TP_EINVAL, "null destination");
  if (int rc = join_forwards(st)) return rc;
  HIP_TRY(hipMemcpyAsync(dst_dev, st->ring(s), st->plan.sizes.param_count * 4, hipMemcpyDeviceToDevice, st->stream));
  return TP_OK;
}

int stage_profile_begin(tp_stage* st, uint32_t max_launches) {
  if (!st) return fail(TP_EINVAL, "null stage");
  if (st->dry) return fail(TP_ESTATE, "a stage without device buffers launches nothing");
  if (st->prof_on) return fail(TP_ESTATE, "profiling is already on");
  if (int rc = join_forwards(st)) return rc;
  while (st->prof_pool.size() < max_launches) {
    ProfEntry e{};
    HIP_TRY(hipEventCreate(&e.start));
    hipError_t err = hipEventCreate(&e.stop);
    if (err != hipSuccess) { (void)hipEventDestroy(e.start); return fail(TP_EHIP, "hipEventCreate: %s", hipGetErrorString(err)); }
    st->prof_pool.push_back(e);
  }
  st->prof_used = 0;
  st->prof_dropped = 0;
  st->prof_on = true;
  return TP_OK;
}

int stage_profile_end(tp_stage* st, tp_profile* out) {
  if (!st || !out) return fail(TP_EINVAL, "null argument");
  if (!st->prof_on) return fail(TP_ESTATE, "profiling is not on");
  st->prof_on = false;
  std::memset(out, 0, sizeof(*out));
  HIP_TRY(hipStreamSynchronize(st->stream));
  for (size_t i = 0; i < st->prof_used; ++i) {
    const ProfEntry& e = st->prof_pool[i];
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, e.start, e.stop));
    out->launches[e.cls]++;
    out->ms[e.cls] += (double)ms;
  }
  out->dropped = st->prof_dropped;
  return TP_OK;
}

}  // extern "C"
