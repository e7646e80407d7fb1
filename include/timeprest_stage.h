/*
 * timeprest_stage.h -- C ABI of the MI355X stage library for V-TiMePReSt / I-TiMePReSt.
 *
 * One `tp_stage` is one pipeline stage (a run of consecutive layers, Section
 * "Pipeline Parallelism") living on one GPU.  The calls follow the paper's own
 * statement of the method:
 *   - every mini-batch is split into n micro-batches; the n forward passes run one
 *     after the other and ONE backward pass serves the whole mini-batch (nF1B,
 *     Section "Methodology");
 *   - the weights are updated after every mini-batch (Section "Pipeline Parallelism");
 *     a weight version is named by the number of updates applied so far;
 *   - V-TiMePReSt: forward and backward always read the latest version, nothing is
 *     stashed (Section "V-TiMePReSt");
 *   - I-TiMePReSt: the forward version is stashed; the backward pass runs on an
 *     intermediate weight built from the stashed version and the degree of staleness
 *     delta through the significance f(delta) = exp(-lambda*delta) (Section
 *     "I-TiMePReSt", Eq. 1-2, Appendix A.1-A.2); a stashed version is kept until the
 *     last mini-batch that used it in forward has built its intermediate weights
 *     (Section "Memory Overhead").
 *
 * Conventions
 *   - Every function returns 0 (TP_OK) or a negative tp_status; none throws, aborts or
 *     synchronises the device.  tp_last_error() gives the text of the last failure on
 *     the calling thread.
 *   - Pointers named *_dev are DEVICE pointers; everything else is HOST memory.
 *   - The caller owns every device buffer (ring arena, momentum, gradient, compute
 *     copies, activation workspace, scratch) and passes them in tp_buffers; sizes come
 *     from stage_workspace_query.  The library allocates no device memory, creates no
 *     stream, and enqueues work only on the stream given to stage_init (and on the one given
 *     to stage_set_forward_streams, if any).  Buffers must
 *     stay alive, and must not be written by the caller, until stage_destroy -- except
 *     ring slot 0, which the caller fills with the initial weights (version 0), and the
 *     momentum buffer, which the caller zeroes, both before stage_init.
 *   - Version ids, slot indices, reference counts and delta are integers computed on
 *     the host inside the call; they are returned through out-parameters.
 *   - Matrices are row-major.  Activations are [rows x features]; a mini-batch is the
 *     n micro-batches stacked in order, [n*mb x features].  In TP_BF16 mode activations,
 *     incoming/outgoing gradients and the compute copies of the weights are bfloat16,
 *     while ring, momentum and gradient stay fp32; in TP_F32 mode everything is fp32.
 *   - Parameter arena: per layer that has parameters the weight tensor (dense W[out x in],
 *     conv W[Cout][k][k][Cin]) followed by the bias b[out]; each tensor starts at a multiple of
 *     64 elements (offsets are reported by stage_workspace_query; padding elements are zero
 *     and stay zero).  Activations of conv/pool layers are NHWC; a row of a mini-batch is one
 *     sample with all its values.
 */
#ifndef TIMEPREST_STAGE_H
#define TIMEPREST_STAGE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum tp_status {
  TP_OK = 0,
  TP_EINVAL = -1,     /* null pointer, bad shape, unknown enum value                      */
  TP_ESTATE = -2,     /* call out of order (backward before n forwards, twice, ...)       */
  TP_ENOVERSION = -3, /* a version that is not (or no longer) held in the ring            */
  TP_EFULL = -4,      /* the ring slot the new version needs is still occupied            */
  TP_EBUSY = -5,      /* evict: version still has users or is the latest -- not freed     */
  TP_EHIP = -6        /* a HIP call or kernel launch failed                               */
};

/* Which weights the backward pass runs on: W_b = alpha * W[v_f] + beta * W[latest]. */
enum tp_policy {
  TP_LATEST = 0,              /* V-TiMePReSt: alpha=0, beta=1; nothing stashed                */
  TP_INTERMEDIATE_EQ1 = 1,    /* I-TiMePReSt as printed in Eq. 1: alpha = 2 - 1/f, beta = 0   */
  TP_INTERMEDIATE_CONVEX = 2, /* I-TiMePReSt read as a blend (Appendix A.2: the stale weight
                                 scaled by f, the rest 1-f to the latest): alpha=f, beta=1-f */
  TP_STASHED = 3,             /* backward on the forward's own version: alpha=1, beta=0      */
  TP_TIMEPREST = 4            /* the parent method (Sections "Methodology", "V-TiMePReSt" Challenge 1): no
                                 horizontal stashing, but a pass cannot pick up updates that happen while it is
                                 under way -- every stage of a pass reads the version that was the latest THERE
                                 when the pass started.  The caller, who drives all stages, knows that version:
                                 it pins it with stash_push when the pass starts, names it in stage_forward_on /
                                 stage_backward_on, and drops it with stash_evict when the pass has left the
                                 stage.  stage_forward / stage_backward read the latest version as under
                                 TP_LATEST; nothing is pinned by the stage itself and no blend is built.  In
                                 TP_BF16 mode wbwd_dev holds the compute copy of the one older version in use. */
};

enum tp_dtype { TP_F32 = 0, TP_BF16 = 1 };
enum tp_act { TP_ACT_NONE = 0, TP_ACT_RELU = 1, TP_ACT_GELU = 2 /* exact erf form */ };
enum tp_layer_type {
  TP_LAYER_DENSE = 0,    /* z = x W^T + b, a = act(z);  W[out x in].  geom[0] = token positions per sample
                            (0 or 1: one): the layer is applied to every position of a [tokens x in] sample */
  TP_LAYER_CONV2D = 1,   /* k x k convolution with k = 1, 3, 5 or 7, stride s = 1 or 2, zero padding (k-1)/2, + bias +
                            act, on NHWC activations: in_features = Cin, out_features = Cout,
                            geom = {H, W, k, s, (k-1)/2} (H, W of the input, even for s = 2); W[Cout][k][k][Cin],
                            b[Cout]; a sample is H*W*Cin values in, (H/s)*(W/s)*Cout out: output pixel (i, j) is
                            centred on input pixel (s*i, s*j).  The matrix-core kernels take k = 3; other kernel
                            sizes run on the generic kernels in both precisions */
  TP_LAYER_MAXPOOL2 = 2, /* 2x2 max pooling, stride 2, no parameters: in_features = out_features = C,
                            geom = {H, W} of the input (both even); first maximum wins ties             */
  /* Layers of a transformer-shaped stage; samples are [tokens x features].  The paper prescribes no layer
     formulas; these are the standard ones. */
  TP_LAYER_LAYERNORM = 3, /* y = gamma (x - mean)/sqrt(var + 1e-5) + beta over the features of each token;
                             in_features = out_features = D, geom = {tokens}; parameters gamma[D] (stored where a
                             dense layer keeps W) and beta[D] (where it keeps b), both fp32 in every mode   */
  TP_LAYER_ATTENTION = 4, /* causal multi-head self-attention, no parameters: in_features = 3*D (queries | keys |
                             values, head h in columns h*D/heads ..), out_features = D, geom = {tokens, heads};
                             must not be the last layer of a stage (its output is kept for the backward pass) */
  TP_LAYER_RESIDUAL = 5,  /* skip connection, no parameters: in_features = out_features = D, geom = {tokens, mark};
                             mark 0 remembers the activation at this point, mark 1 adds the remembered one to
                             the activation at this point and applies `act`; marks alternate 0, 1, 0, 1, ...
                             Between a 0 and its 1 there may be one mark 2 (projection shortcut): it sets the
                             activation at this point aside as the remembered one and hands the tensor remembered
                             at mark 0 to the next layer, so the layers up to mark 1 form the second branch;
                             in_features, geom[0] = features, tokens coming in; out_features, geom[2] = those of
                             the tensor remembered at mark 0 */
  TP_LAYER_BATCHNORM = 6, /* batch normalisation in training mode + act (bottleneck-shaped stages): statistics per
                             channel over all samples and positions of the micro-batch a forward call sees, biased
                             variance, eps 1e-5; in_features = out_features = C, geom = {positions per sample};
                             parameters gamma[C], beta[C] (fp32 in every mode); no running statistics are kept */
  TP_LAYER_SUBSAMPLE2 = 7, /* every second pixel of every second row (the pixels a stride-2 1x1 convolution reads), no
                             parameters: in_features = out_features = C, geom = {H, W} of the input (both even),
                             C * element size a multiple of 16 bytes */
  TP_LAYER_AVGPOOL = 8    /* global average pooling, no parameters: a sample of [positions x C] values becomes the C
                             means over its positions; in_features = out_features = C, geom = {positions} */
};

#define TP_MAX_LAYERS 64
#define TP_NONE UINT64_MAX /* "no mini-batch" for stage_blend_update */

typedef struct tp_layer_desc {
  int32_t type;         /* tp_layer_type */
  int32_t act;          /* tp_act */
  int32_t in_features;  /* dense: columns of the layer input;  conv/pool: input channels;  others: see the type */
  int32_t out_features; /* dense: columns of the layer output; conv/pool: output channels; others: see the type */
  int32_t geom[5];      /* conv: {H, W, kernel, stride, pad}; pool: {H, W, 0, 0, 0}; dense, layer norm: {tokens};
                           attention: {tokens, heads}; residual: {tokens, mark[, tokens out]}; batch norm: {positions};
                           subsampling: {H, W}; average pooling: {positions}; unused entries zero */
  int32_t reserved[7];  /* must be zero */
} tp_layer_desc;

typedef struct tp_stage_desc {
  int32_t num_layers;
  int32_t dtype;         /* tp_dtype */
  int32_t mb;            /* samples per micro-batch */
  int32_t n;             /* micro-batches per mini-batch */
  int32_t stage_index;   /* s, 0-based */
  int32_t num_stages;    /* K */
  int32_t ring_capacity; /* C: weight versions the ring can hold (K - s covers the nF1B
                            schedule under the stashing policies; 1 suffices for TP_LATEST) */
  int32_t max_in_flight; /* mini-batches between forward and backward whose activations are
                            saved at once (K - s for the nF1B schedule) */
  int32_t policy;        /* tp_policy */
  int32_t needs_dx;      /* 0: the stage has no predecessor, no input gradient is formed */
  double lambda;         /* constant of the significance function, > 0 */
  double lr;             /* learning rate */
  double momentum;       /* mu of m <- mu*m + g; W <- W - lr*m */
  tp_layer_desc layers[TP_MAX_LAYERS];
} tp_stage_desc;

typedef struct tp_sizes {
  uint64_t param_count;  /* P: elements of one weight version, padding included */
  uint64_t ring_bytes;   /* ring_capacity * P * 4 */
  uint64_t momentum_bytes;
  uint64_t grad_bytes;
  uint64_t wfwd_bytes;   /* bf16 copy of the latest version (0 in TP_F32 mode) */
  uint64_t wbwd_bytes;   /* W_b compute copy, P elements of the activation type (0 under TP_LATEST, which
                            never builds intermediate weights: wbwd_dev may then be NULL) */
  uint64_t act_bytes;    /* saved activations of max_in_flight mini-batches */
  uint64_t scratch_bytes;/* backward temporaries and reduction partials */
  uint64_t diag_bytes;   /* TP_DIAG_COUNT doubles written by stage_blend_update */
  uint64_t w_offset[TP_MAX_LAYERS]; /* element offset of W of layer l inside a version */
  uint64_t b_offset[TP_MAX_LAYERS]; /* element offset of b of layer l */
} tp_sizes;

/* Diagnostics the update kernel reduces on the fly (doubles in tp_buffers.diag_dev). */
enum {
  TP_DIAG_GRAD_SQ = 0,   /* sum g^2                                   */
  TP_DIAG_WEIGHT_SQ = 1, /* sum W[v+1]^2                              */
  TP_DIAG_DRIFT_SQ = 2,  /* sum (W[v+1] - W[v_f])^2, 0 when no blend  */
  TP_DIAG_WB_SQ = 3,     /* sum W_b^2, 0 when no blend                */
  TP_DIAG_COUNT = 4
};

typedef struct tp_buffers {
  void* ring_dev;
  void* momentum_dev;
  void* grad_dev;
  void* wfwd_dev;
  void* wbwd_dev;
  void* act_dev;
  void* scratch_dev;
  void* diag_dev;
} tp_buffers;

#define TP_MAX_SLOTS 16
#define TP_MAX_IN_FLIGHT 16

typedef struct tp_state {
  uint64_t latest_version;
  int32_t ring_capacity;
  int32_t slot_occupied[TP_MAX_SLOTS];
  uint64_t slot_version[TP_MAX_SLOTS];
  uint32_t slot_refcnt[TP_MAX_SLOTS];
  int32_t num_in_flight;
  uint64_t in_flight_mb[TP_MAX_IN_FLIGHT];
  uint64_t in_flight_vf[TP_MAX_IN_FLIGHT];
  uint32_t in_flight_forwards[TP_MAX_IN_FLIGHT]; /* micro-batch forwards seen so far */
  uint64_t wb_ready_mb; /* mini-batch whose W_b is already built by the fused update, or TP_NONE */
} tp_state;

typedef struct tp_stage tp_stage; /* opaque; host memory owned by the library */

/* Sizes and arena offsets for a stage description.  Host only, no GPU needed. */
int stage_workspace_query(const tp_stage_desc* desc, tp_sizes* out);

/* Create a stage.  `bufs` holds device pointers of at least the queried sizes;
 * `hip_stream` is a hipStream_t (NULL = the default stream).  Ring slot 0 must hold the
 * initial weights and momentum_dev must be zero.  In TP_BF16 mode the call enqueues the
 * conversion of version 0 into wfwd_dev. */
int stage_init(const tp_stage_desc* desc, const tp_buffers* bufs, void* hip_stream, tp_stage** out);
int stage_destroy(tp_stage* st);

/* Forward of micro-batch `ub_idx` (0..n-1, in order) of mini-batch `mb_id` on the latest
 * weights at the stage at the time of the call (Sections "V-TiMePReSt", "I-TiMePReSt").
 * x_dev: [mb x in] input; y_dev: [mb x out] output.  The stage keeps what the backward
 * needs in its activation workspace; x_dev may be the pointer returned by
 * stage_input_ptr (then no copy is made).  On the first micro-batch of a mini-batch the
 * version is recorded and, under the stashing policies, pinned in the ring.
 * version_used (optional) receives the version read.
 * TP_ESTATE: ub_idx out of order, more than max_in_flight mini-batches in flight, or (stashing
 * policies) an update landed between two micro-batches of the same mini-batch. */
int stage_forward(tp_stage* st, uint64_t mb_id, uint32_t ub_idx, const void* x_dev, void* y_dev,
                  uint64_t* version_used);

/* TP_TIMEPREST only: stage_forward on `version` (which must be in the ring: pin it with stash_push when the
 * pass starts) instead of the latest one.  TP_EINVAL under any other policy, TP_ENOVERSION if the ring does
 * not hold the version. */
int stage_forward_on(tp_stage* st, uint64_t mb_id, uint32_t ub_idx, uint64_t version, const void* x_dev,
                     void* y_dev);

/* Optional: up to TP_MAX_FORWARD_STREAMS streams of the caller's for the forward passes (hipStream_t of default
 * priority, none of them NULL or the stage's own, none synchronising with it implicitly; count = 0 takes them away
 * again).  The micro-batch forward passes of a mini-batch do not depend on one another (Section "Methodology": they
 * run one after another through the pipeline on the same weights), and the forward passes of a later mini-batch do
 * not depend on the backward pass of an earlier one, only on the update before it (Sections "V-TiMePReSt",
 * "I-TiMePReSt": a forward reads the latest version).  With S such streams stage_forward and stage_forward_on enqueue
 * micro-batch ub on hip_streams[ub % S] and nothing of a forward on the stage's own stream (a stage with
 * max_in_flight = 1, whose backward pass always needs the forwards just enqueued, lets its own stream take a turn:
 * ub % (S + 1) == 0 runs there, the others on hip_streams[ub % (S + 1) - 1]); the kernels and their results are the
 * same bits.  Ordering, kept with events of the library's own:
 *   - a forward pass starts behind everything the stage's stream held when the most recent call other than a forward
 *     returned (the update that made its weights, the backward pass that freed its activation slot).  x_dev must be
 *     complete, or ordered before that point, when the call is made;
 *   - stage_backward / stage_backward_on make the stage's stream wait for the forward passes of THEIR mini-batch
 *     and for no others: forwards of later mini-batches enqueued before the call keep running beside the backward
 *     pass;
 *   - every other call that enqueues work or hands out results (stage_blend_update[_noalloc], stage_loss_softmax_ce,
 *     stage_saved_input_ptr, stage_export_params, stage_profile_begin, stage_forward_join) first makes the stage's
 *     stream wait for all forward streams.  Read y_dev on the stage's stream only after one of them.
 * Refused (TP_EINVAL) for stages with attention layers, whose forward kernels share their scratch memory, and under
 * TP_TIMEPREST.  Not used while profiling is on.  The streams must outlive the stage or be taken away first;
 * stage_destroy waits for them. */
#define TP_MAX_FORWARD_STREAMS 3
int stage_set_forward_streams(tp_stage* st, void* const* hip_streams, int32_t count);
int stage_forward_join(tp_stage* st);

/* Where the stage wants the input of (mb_id, ub_idx) to be written so that
 * stage_forward needs no copy.  Valid for the mini-batch's first micro-batch onwards. */
int stage_input_ptr(tp_stage* st, uint64_t mb_id, uint32_t ub_idx, void** x_dev);

/* Where the stage keeps the input of layer `layer` (0-based) for micro-batch `ub_idx` of the in-flight
 * mini-batch `mb_id`: the tensor saved for the single backward pass of the mini-batch (Section "Methodology");
 * for layer > 0 it is the stored output of layer - 1, [mb x values per sample] in the activation type.  For
 * inspection (parity tests read every stored activation, not only the stage's output); the memory belongs to the
 * stage and must not be written.  Valid from that micro-batch's stage_forward until the mini-batch's
 * stage_backward.  Not every layer's input is materialised: the input of a residual add whose producer formed
 * the sum in its own kernel, and of a few-channel first convolution (kept padded to 8 channels elsewhere), are
 * never written -- the contents behind their pointers are unspecified.  bytes (optional) receives the size.
 * TP_ESTATE: that micro-batch is not in flight. */
int stage_saved_input_ptr(tp_stage* st, uint64_t mb_id, uint32_t ub_idx, int32_t layer, void** x_dev,
                          uint64_t* bytes);

/* Softmax cross-entropy of a whole mini-batch at the last stage (Section "Methodology":
 * the loss is taken at the last node and starts the backward pass), mean over the n*mb
 * rows.  logits_dev: [n*mb x classes] in the activation type, labels_dev: int32[n*mb],
 * dlogits_dev: [n*mb x classes] = (softmax - onehot)/(n*mb), loss_dev: one float.
 * classes = out_features of the stage's last layer. */
int stage_loss_softmax_ce(tp_stage* st, uint64_t mb_id, const void* logits_dev,
                          const int32_t* labels_dev, void* dlogits_dev, float* loss_dev);

/* The one backward pass of mini-batch `mb_id` over all its n micro-batches (Section
 * "Methodology"), on W_b = alpha(delta) W[v_f] + beta(delta) W[latest] with
 * delta = latest - v_f (Eq. 1-2).  dy_dev: [n*mb x out]; dx_dev: [n*mb x in] or NULL when
 * needs_dx = 0.  Writes the gradient of every parameter into grad_dev (overwriting it).
 * If the fused update already built W_b for this mini-batch it is used, otherwise the
 * blend is enqueued first.  Afterwards the mini-batch's stashed version loses one user and
 * is evicted when unused (Section "Memory Overhead").  delta_used (optional) receives delta.
 * TP_ESTATE: unknown mini-batch or not all n forwards seen; TP_ENOVERSION: its forward
 * version is no longer in the ring. */
int stage_backward(tp_stage* st, uint64_t mb_id, const void* dy_dev, void* dx_dev,
                   uint32_t* delta_used);

/* TP_TIMEPREST only: stage_backward with every use of a parameter in the backward pass reading `version` as
 * it is (the version the backward pass started on; no blend, delta plays no part).  Errors as stage_forward_on. */
int stage_backward_on(tp_stage* st, uint64_t mb_id, uint64_t version, const void* dy_dev, void* dx_dev);

/* Update after mini-batch `mb_id_done` (its backward must be the last one run):
 * m <- mu*m + g, W[v+1] = W[v] - lr*m written into ring slot (v+1) mod C, plus the bf16
 * compute copy in TP_BF16 mode.  If mb_id_next_bwd is not TP_NONE, the same pass over the
 * parameters also builds W_b for that mini-batch's coming backward, with W[v+1] as the
 * latest weights (valid as long as no other update happens before that backward; the
 * backward re-checks).  new_version (optional) receives v+1.
 * TP_EFULL: slot (v+1) mod C still holds a live version; TP_ESTATE: no gradient pending. */
int stage_blend_update(tp_stage* st, uint64_t mb_id_done, uint64_t mb_id_next_bwd,
                       uint64_t* new_version);

/* stage_blend_update for callers that cannot allocate device memory and bring no workspace for it: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results,
 * bookkeeping and errors as stage_blend_update; the block partials of the diagnostics live in a 32 KiB device
 * array the library itself holds on every GPU it runs on (for the life of the process) instead of in
 * tp_buffers.scratch_dev, so the call touches no memory but the stage's ring, momentum, gradient, compute
 * copies and diag_dev, calls no allocating routine, and enqueues two kernels on the stage's stream.
 * Stages of more than TP_NOALLOC_MAX_PARAMS parameters per version are refused with TP_EINVAL.  All stages on
 * one GPU share that array: two such calls whose kernels may overlap on one GPU (different streams) race on
 * the diagnostics; calls on one stream, or ordered by events, do not.  Nothing in the array has to be
 * cleared between calls (every partial that is read has been written by the same call). */
#define TP_NOALLOC_MAX_PARAMS (1ull << 31)
int stage_blend_update_noalloc(tp_stage* st, uint64_t mb_id_done, uint64_t mb_id_next_bwd,
                               uint64_t* new_version);

/* Pin `version` for one more forward user (refcount + 1); slot (optional) receives its
 * ring slot.  TP_ENOVERSION if the ring does not hold it. */
int stash_push(tp_stage* st, uint64_t version, uint32_t* slot);

/* Drop one user of `version` that was added with stash_push; the slot is freed when no user is left and
 * the version is not the latest, else TP_EBUSY is returned (an outside user has still been dropped if there
 * was one).  The users the stage holds itself -- mini-batches between their forward and their backward
 * (Section "Memory Overhead") -- cannot be dropped from outside: with only those left the call changes
 * nothing and returns TP_EBUSY.  TP_ENOVERSION if the ring does not hold the version. */
int stash_evict(tp_stage* st, uint64_t version);

/* Snapshot of the host bookkeeping. */
int stage_query(const tp_stage* st, tp_state* out);

/* Copy the fp32 master of `version` (P floats) to dst_dev on the stage's stream. */
int stage_export_params(tp_stage* st, uint64_t version, void* dst_dev);

/* (alpha, beta) for a policy and degree of staleness, in double (Eq. 1-2). Host only. */
int tp_blend_coefficients(int32_t policy, uint32_t delta, double lambda, double* alpha,
                          double* beta);

/* nF1B event order of a K-stage pipeline at mini-batch granularity (Section
 * "Methodology"): stage s takes in K-s mini-batches, then alternates backward+update and
 * forward.  Writes up to `capacity` events, returns the total number in *count.
 * kind: 0 = forward of all n micro-batches, 1 = backward followed by update. Host only. */
typedef struct tp_event {
  int32_t t;
  int32_t kind;
  int32_t stage;
  int32_t ub;      /* micro-batch index of a forward event of tp_schedule_microbatch_events; else 0 */
  uint64_t mb_id;
} tp_event;
int tp_schedule_events(int32_t num_stages, uint64_t num_minibatches, tp_event* out,
                       uint64_t capacity, uint64_t* count);

/* The same pipeline at micro-batch granularity, one box per stage and tick as the paper's timing figures are
 * described (Section "Methodology", last paragraph): kind 0 = forward pass of ONE micro-batch (`ub`), 1 =
 * backward pass of the mini-batch followed by its update.  A stage takes a micro-batch as soon as the stage
 * before it has produced it, holds at most K-s mini-batches between first forward and backward, and lets a
 * backward pass that is ready go first -- with mid_pass_updates != 0 also between two micro-batches of one
 * mini-batch, so that the update lands in the middle of that mini-batch's forward pass and its remaining
 * micro-batches read the newer weights (V-TiMePReSt "checks for the newer versions of weights even during the
 * execution of a pass", Section "V-TiMePReSt"; the stashing policies need mid_pass_updates = 0).  With
 * mid_pass_updates = 0 the version every mini-batch reads is the one tp_schedule_events gives.  Host only. */
int tp_schedule_microbatch_events(int32_t num_stages, uint64_t num_minibatches, int32_t n,
                                  int32_t mid_pass_updates, tp_event* out, uint64_t capacity, uint64_t* count);

/* Measurement hooks (not part of the method): while profiling is on, every kernel the stage
 * enqueues is bracketed by a pair of HIP events on the stage's stream.  stage_profile_end waits
 * for the stream (the only call of this library that synchronises), adds up the elapsed time
 * per kernel class and switches profiling off.  max_launches bounds the number of event pairs;
 * launches beyond it are counted in `dropped` and not timed. */
enum tp_kernel_class {
  TP_K_FPROP = 0,    /* z = x W^T + b, a = act(z)                    */
  TP_K_DGRAD = 1,    /* dx = dz W_b (.) act'                         */
  TP_K_WGRAD = 2,    /* dW = dz^T x                                  */
  TP_K_COLSUM = 3,   /* db = column sums of dz                       */
  TP_K_ACT_BWD = 4,  /* dz = dy (.) act'(z)                          */
  TP_K_UPDATE = 5,   /* fused momentum + update + copies + blend     */
  TP_K_BLEND = 6,    /* intermediate weights on their own            */
  TP_K_LOSS = 7,     /* softmax cross-entropy                        */
  TP_K_COPY = 8,     /* device-to-device copies and conversions      */
  TP_K_POOL = 9,     /* max pooling forward / backward               */
  TP_K_NORM = 10,    /* layer normalisation forward / backward       */
  TP_K_ATTN = 11,    /* attention forward / backward                 */
  TP_K_ADD = 12,     /* residual additions                           */
  TP_K_SUMS = 13,    /* a backward pass's sums of partials, one launch */
  TP_K_CLASSES = 14
};
typedef struct tp_profile {
  uint64_t launches[TP_K_CLASSES];
  double ms[TP_K_CLASSES];
  uint64_t dropped;
} tp_profile;
int stage_profile_begin(tp_stage* st, uint32_t max_launches);
int stage_profile_end(tp_stage* st, tp_profile* out);

const char* tp_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* TIMEPREST_STAGE_H */
