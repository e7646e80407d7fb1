"""ctypes binding of libtimeprest_stage.so: same names as the C ABI, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os

from .build import lib_path

TP_OK, TP_EINVAL, TP_ESTATE, TP_ENOVERSION, TP_EFULL, TP_EBUSY, TP_EHIP = 0, -1, -2, -3, -4, -5, -6
TP_LATEST, TP_INTERMEDIATE_EQ1, TP_INTERMEDIATE_CONVEX, TP_STASHED, TP_TIMEPREST = 0, 1, 2, 3, 4
TP_F32, TP_BF16 = 0, 1
TP_ACT_NONE, TP_ACT_RELU, TP_ACT_GELU = 0, 1, 2
TP_LAYER_DENSE, TP_LAYER_CONV2D, TP_LAYER_MAXPOOL2, TP_LAYER_LAYERNORM, TP_LAYER_ATTENTION, TP_LAYER_RESIDUAL, TP_LAYER_BATCHNORM = 0, 1, 2, 3, 4, 5, 6
TP_LAYER_SUBSAMPLE2 = 7
TP_LAYER_AVGPOOL = 8
TP_MAX_LAYERS, TP_MAX_SLOTS, TP_MAX_IN_FLIGHT = 64, 16, 16
TP_NONE = (1 << 64) - 1
TP_DIAG_GRAD_SQ, TP_DIAG_WEIGHT_SQ, TP_DIAG_DRIFT_SQ, TP_DIAG_WB_SQ, TP_DIAG_COUNT = 0, 1, 2, 3, 4

POLICY = {"latest": TP_LATEST, "eq1": TP_INTERMEDIATE_EQ1, "convex": TP_INTERMEDIATE_CONVEX, "stashed": TP_STASHED,
          "timeprest": TP_TIMEPREST}
ACT = {"none": TP_ACT_NONE, "relu": TP_ACT_RELU, "gelu": TP_ACT_GELU}
DTYPE = {"f32": TP_F32, "bf16": TP_BF16}

EXPORTS = ["stage_workspace_query", "stage_init", "stage_destroy", "stage_set_forward_streams", "stage_forward_join", "stage_forward", "stage_forward_on", "stage_backward_on", "stage_input_ptr", "stage_saved_input_ptr",
           "stage_loss_softmax_ce", "stage_backward", "stage_blend_update", "stage_blend_update_noalloc", "stash_push", "stash_evict",
           "stage_query", "stage_export_params", "tp_blend_coefficients", "tp_schedule_events", "tp_schedule_microbatch_events",
           "stage_profile_begin", "stage_profile_end", "tp_last_error"]


class tp_layer_desc(C.Structure):
    _fields_ = [("type", C.c_int32), ("act", C.c_int32), ("in_features", C.c_int32), ("out_features", C.c_int32),
                ("geom", C.c_int32 * 5), ("reserved", C.c_int32 * 7)]


class tp_stage_desc(C.Structure):
    _fields_ = [("num_layers", C.c_int32), ("dtype", C.c_int32), ("mb", C.c_int32), ("n", C.c_int32),
                ("stage_index", C.c_int32), ("num_stages", C.c_int32), ("ring_capacity", C.c_int32),
                ("max_in_flight", C.c_int32), ("policy", C.c_int32), ("needs_dx", C.c_int32),
                ("lambda_", C.c_double), ("lr", C.c_double), ("momentum", C.c_double),
                ("layers", tp_layer_desc * TP_MAX_LAYERS)]


class tp_sizes(C.Structure):
    _fields_ = [("param_count", C.c_uint64), ("ring_bytes", C.c_uint64), ("momentum_bytes", C.c_uint64),
                ("grad_bytes", C.c_uint64), ("wfwd_bytes", C.c_uint64), ("wbwd_bytes", C.c_uint64),
                ("act_bytes", C.c_uint64), ("scratch_bytes", C.c_uint64), ("diag_bytes", C.c_uint64),
                ("w_offset", C.c_uint64 * TP_MAX_LAYERS), ("b_offset", C.c_uint64 * TP_MAX_LAYERS)]


class tp_buffers(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in ("ring_dev", "momentum_dev", "grad_dev", "wfwd_dev", "wbwd_dev", "act_dev",
                                          "scratch_dev", "diag_dev")]


class tp_state(C.Structure):
    _fields_ = [("latest_version", C.c_uint64), ("ring_capacity", C.c_int32),
                ("slot_occupied", C.c_int32 * TP_MAX_SLOTS), ("slot_version", C.c_uint64 * TP_MAX_SLOTS),
                ("slot_refcnt", C.c_uint32 * TP_MAX_SLOTS), ("num_in_flight", C.c_int32),
                ("in_flight_mb", C.c_uint64 * TP_MAX_IN_FLIGHT), ("in_flight_vf", C.c_uint64 * TP_MAX_IN_FLIGHT),
                ("in_flight_forwards", C.c_uint32 * TP_MAX_IN_FLIGHT), ("wb_ready_mb", C.c_uint64)]


class tp_event(C.Structure):
    _fields_ = [("t", C.c_int32), ("kind", C.c_int32), ("stage", C.c_int32), ("ub", C.c_int32),
                ("mb_id", C.c_uint64)]


KERNEL_CLASSES = ["fprop", "dgrad", "wgrad", "colsum", "act_bwd", "update", "blend", "loss", "copy", "pool", "norm", "attn",
                  "add", "sums"]


class tp_profile(C.Structure):
    _fields_ = [("launches", C.c_uint64 * len(KERNEL_CLASSES)), ("ms", C.c_double * len(KERNEL_CLASSES)),
                ("dropped", C.c_uint64)]


class StageLibError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"timeprest_stage error {code}: {text}")
        self.code = code


def _load():
    # The library must share the HIP runtime of the process that owns the device memory and the
    # streams it is handed.  torch ships its own libamdhip64 (same soname); importing torch first
    # makes the dynamic loader resolve the library's dependency to that already-loaded runtime.
    import torch  # noqa: F401
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it first (python -m paper_2509_23241_amd.build); "
                          "there is no fallback path")
    return C.CDLL(path)


lib = _load()
_vp, _u64, _u32, _i32 = C.c_void_p, C.c_uint64, C.c_uint32, C.c_int32
lib.stage_workspace_query.argtypes = [C.POINTER(tp_stage_desc), C.POINTER(tp_sizes)]
lib.stage_init.argtypes = [C.POINTER(tp_stage_desc), C.POINTER(tp_buffers), _vp, C.POINTER(_vp)]
lib.stage_destroy.argtypes = [_vp]
lib.stage_forward.argtypes = [_vp, _u64, _u32, _vp, _vp, C.POINTER(_u64)]
lib.stage_forward_on.argtypes = [_vp, _u64, _u32, _u64, _vp, _vp]
lib.stage_backward_on.argtypes = [_vp, _u64, _u64, _vp, _vp]
lib.stage_input_ptr.argtypes = [_vp, _u64, _u32, C.POINTER(_vp)]
lib.stage_set_forward_streams.argtypes = [_vp, C.POINTER(_vp), _i32]
lib.stage_forward_join.argtypes = [_vp]
lib.stage_saved_input_ptr.argtypes = [_vp, _u64, _u32, _i32, C.POINTER(_vp), C.POINTER(_u64)]
lib.stage_loss_softmax_ce.argtypes = [_vp, _u64, _vp, _vp, _vp, _vp]
lib.stage_backward.argtypes = [_vp, _u64, _vp, _vp, C.POINTER(_u32)]
lib.stage_blend_update.argtypes = [_vp, _u64, _u64, C.POINTER(_u64)]
lib.stage_blend_update_noalloc.argtypes = [_vp, _u64, _u64, C.POINTER(_u64)]
lib.stash_push.argtypes = [_vp, _u64, C.POINTER(_u32)]
lib.stash_evict.argtypes = [_vp, _u64]
lib.stage_query.argtypes = [_vp, C.POINTER(tp_state)]
lib.stage_export_params.argtypes = [_vp, _u64, _vp]
lib.tp_blend_coefficients.argtypes = [_i32, _u32, C.c_double, C.POINTER(C.c_double), C.POINTER(C.c_double)]
lib.tp_schedule_events.argtypes = [_i32, _u64, C.POINTER(tp_event), _u64, C.POINTER(_u64)]
lib.tp_schedule_microbatch_events.argtypes = [_i32, _u64, _i32, _i32, C.POINTER(tp_event), _u64, C.POINTER(_u64)]
lib.stage_profile_begin.argtypes = [_vp, _u32]
lib.stage_profile_end.argtypes = [_vp, C.POINTER(tp_profile)]
lib.tp_last_error.restype = C.c_char_p
for _name in EXPORTS[:-1]:
    getattr(lib, _name).restype = C.c_int


def tp_last_error() -> str:
    return lib.tp_last_error().decode()


def _check(rc, soft=()):
    if rc != TP_OK and rc not in soft:
        raise StageLibError(rc, tp_last_error())
    return rc


def make_desc(layers, *, dtype, mb, n, stage_index, num_stages, ring_capacity, max_in_flight, policy, needs_dx,
              lam, lr, momentum) -> tp_stage_desc:
    """layers: sequence of (in_features, out_features, act-name[, tokens]) for dense layers,
    ("conv", cin, cout, H, W, act-name[, stride[, kernel]]) for kernel x kernel convolutions (default 3) with pad
    (kernel-1)/2, ("pool", C, H, W) for 2x2 pooling, ("sub", C, H, W) for 2x subsampling, ("avg", C, positions) for
    global average pooling, ("ln", D, tokens), ("attn", D, heads, tokens),
    ("res", D, tokens, "begin" | "add"[, act-name]), ("swap", D_in, tokens_in, D_out, tokens_out) for the residual
    mark that starts a projection shortcut, ("bn", C, positions, act-name)."""
    if len(layers) > TP_MAX_LAYERS:
        raise ValueError(f"{len(layers)} layers: a stage takes at most {TP_MAX_LAYERS}")
    d = tp_stage_desc()
    d.num_layers = len(layers)
    d.dtype = DTYPE[dtype] if isinstance(dtype, str) else dtype
    d.mb, d.n = mb, n
    d.stage_index, d.num_stages = stage_index, num_stages
    d.ring_capacity, d.max_in_flight = ring_capacity, max_in_flight
    d.policy = POLICY[policy] if isinstance(policy, str) else policy
    d.needs_dx = int(bool(needs_dx))
    d.lambda_, d.lr, d.momentum = lam, lr, momentum
    for i, spec in enumerate(layers[:TP_MAX_LAYERS]):
        L = d.layers[i]
        if spec[0] == "conv":
            _, cin, cout, H, W, act = spec[:6]
            L.type, L.in_features, L.out_features = TP_LAYER_CONV2D, cin, cout
            k = spec[7] if len(spec) > 7 else 3
            L.geom[0], L.geom[1], L.geom[2], L.geom[3], L.geom[4] = H, W, k, (spec[6] if len(spec) > 6 else 1), (k - 1) // 2
        elif spec[0] == "pool":
            _, c, H, W = spec
            act = "none"
            L.type, L.in_features, L.out_features = TP_LAYER_MAXPOOL2, c, c
            L.geom[0], L.geom[1] = H, W
        elif spec[0] == "sub":
            _, c, H, W = spec
            act = "none"
            L.type, L.in_features, L.out_features = TP_LAYER_SUBSAMPLE2, c, c
            L.geom[0], L.geom[1] = H, W
        elif spec[0] == "avg":
            _, c, positions = spec
            act = "none"
            L.type, L.in_features, L.out_features = TP_LAYER_AVGPOOL, c, c
            L.geom[0] = positions
        elif spec[0] == "swap":
            _, din, tin, dout, tout = spec
            act = "none"
            L.type, L.in_features, L.out_features = TP_LAYER_RESIDUAL, din, dout
            L.geom[0], L.geom[1], L.geom[2] = tin, 2, tout
        elif spec[0] == "ln":
            _, dm, tokens = spec
            act = "none"
            L.type, L.in_features, L.out_features = TP_LAYER_LAYERNORM, dm, dm
            L.geom[0] = tokens
        elif spec[0] == "attn":
            _, dm, heads, tokens = spec
            act = "none"
            L.type, L.in_features, L.out_features = TP_LAYER_ATTENTION, 3 * dm, dm
            L.geom[0], L.geom[1] = tokens, heads
        elif spec[0] == "res":
            _, dm, tokens, mark = spec[:4]
            act = spec[4] if len(spec) > 4 else "none"
            L.type, L.in_features, L.out_features = TP_LAYER_RESIDUAL, dm, dm
            L.geom[0], L.geom[1] = tokens, {"begin": 0, "add": 1}[mark]
        elif spec[0] == "bn":
            _, ch, tokens, act = spec
            L.type, L.in_features, L.out_features = TP_LAYER_BATCHNORM, ch, ch
            L.geom[0] = tokens
        else:
            fin, fout, act = spec[:3]
            L.type, L.in_features, L.out_features = TP_LAYER_DENSE, fin, fout
            L.geom[0] = spec[3] if len(spec) > 3 and spec[3] > 1 else 0
        L.act = ACT[act] if isinstance(act, str) else act
    return d


def layer_in_elems(spec) -> int:
    """Values per sample a layer takes in / gives out (same tuple format as make_desc)."""
    if spec[0] == "conv":
        return spec[3] * spec[4] * spec[1]
    if spec[0] in ("pool", "sub"):
        return spec[2] * spec[3] * spec[1]
    if spec[0] in ("ln", "bn", "swap", "avg"):
        return spec[1] * spec[2]
    if spec[0] == "attn":
        return 3 * spec[1] * spec[3]
    if spec[0] == "res":
        return spec[1] * spec[2]
    return spec[0] * (spec[3] if len(spec) > 3 else 1)


def layer_out_elems(spec) -> int:
    if spec[0] == "conv":
        st = spec[6] if len(spec) > 6 else 1
        return (spec[3] // st) * (spec[4] // st) * spec[2]
    if spec[0] in ("pool", "sub"):
        return (spec[2] // 2) * (spec[3] // 2) * spec[1]
    if spec[0] == "swap":
        return spec[3] * spec[4]
    if spec[0] == "avg":
        return spec[1]
    if spec[0] in ("ln", "bn"):
        return spec[1] * spec[2]
    if spec[0] == "attn":
        return spec[1] * spec[3]
    if spec[0] == "res":
        return spec[1] * spec[2]
    return spec[1] * (spec[3] if len(spec) > 3 else 1)


def layer_param_shapes(spec):
    if spec[0] == "conv":
        k = spec[7] if len(spec) > 7 else 3
        return [(spec[2], k, k, spec[1]), (spec[2],)]
    if spec[0] in ("pool", "attn", "res", "sub", "swap", "avg"):
        return []
    if spec[0] in ("ln", "bn"):
        return [(spec[1],), (spec[1],)]
    return [(spec[1], spec[0]), (spec[1],)]


def stage_workspace_query(desc: tp_stage_desc) -> tp_sizes:
    out = tp_sizes()
    _check(lib.stage_workspace_query(C.byref(desc), C.byref(out)))
    return out


def stage_init(desc: tp_stage_desc, bufs, hip_stream: int):
    """bufs: tp_buffers or None (bookkeeping-only stage that launches nothing)."""
    handle = _vp()
    _check(lib.stage_init(C.byref(desc), C.byref(bufs) if bufs is not None else None, _vp(hip_stream), C.byref(handle)))
    return handle


def stage_destroy(st):
    _check(lib.stage_destroy(st))


def stage_forward(st, mb_id: int, ub_idx: int, x_dev: int, y_dev: int) -> int:
    v = _u64()
    _check(lib.stage_forward(st, mb_id, ub_idx, _vp(x_dev), _vp(y_dev), C.byref(v)))
    return v.value


def stage_forward_on(st, mb_id: int, ub_idx: int, version: int, x_dev: int, y_dev: int):
    _check(lib.stage_forward_on(st, mb_id, ub_idx, version, _vp(x_dev), _vp(y_dev)))


def stage_backward_on(st, mb_id: int, version: int, dy_dev: int, dx_dev: int):
    _check(lib.stage_backward_on(st, mb_id, version, _vp(dy_dev), _vp(dx_dev)))


TP_MAX_FORWARD_STREAMS = 3


def stage_set_forward_streams(st, hip_streams):
    """hip_streams: sequence of stream handles (integers); empty takes the forward streams away."""
    arr = (_vp * max(len(hip_streams), 1))(*[_vp(h) for h in hip_streams])
    _check(lib.stage_set_forward_streams(st, arr, len(hip_streams)))


def stage_forward_join(st):
    _check(lib.stage_forward_join(st))


def stage_input_ptr(st, mb_id: int, ub_idx: int) -> int:
    p = _vp()
    _check(lib.stage_input_ptr(st, mb_id, ub_idx, C.byref(p)))
    return p.value or 0


def stage_saved_input_ptr(st, mb_id: int, ub_idx: int, layer: int):
    """(device pointer, bytes) of the saved input of `layer` for micro-batch ub_idx of mini-batch mb_id."""
    p, nb = _vp(), _u64()
    _check(lib.stage_saved_input_ptr(st, mb_id, ub_idx, layer, C.byref(p), C.byref(nb)))
    return (p.value or 0), nb.value


def stage_loss_softmax_ce(st, mb_id: int, logits_dev: int, labels_dev: int, dlogits_dev: int, loss_dev: int):
    _check(lib.stage_loss_softmax_ce(st, mb_id, _vp(logits_dev), _vp(labels_dev), _vp(dlogits_dev), _vp(loss_dev)))


def stage_backward(st, mb_id: int, dy_dev: int, dx_dev: int) -> int:
    d = _u32()
    _check(lib.stage_backward(st, mb_id, _vp(dy_dev), _vp(dx_dev), C.byref(d)))
    return d.value


def stage_blend_update(st, mb_id_done: int, mb_id_next_bwd: int = TP_NONE) -> int:
    v = _u64()
    _check(lib.stage_blend_update(st, mb_id_done, mb_id_next_bwd, C.byref(v)))
    return v.value


def stage_blend_update_noalloc(st, mb_id_done: int, mb_id_next_bwd: int = TP_NONE) -> int:
    v = _u64()
    _check(lib.stage_blend_update_noalloc(st, mb_id_done, mb_id_next_bwd, C.byref(v)))
    return v.value


def stash_push(st, version: int) -> int:
    s = _u32()
    _check(lib.stash_push(st, version, C.byref(s)))
    return s.value


def stash_evict(st, version: int) -> int:
    """Returns TP_OK when the slot was freed, TP_EBUSY when the version stays."""
    return _check(lib.stash_evict(st, version), soft=(TP_EBUSY,))


def stage_query(st) -> tp_state:
    out = tp_state()
    _check(lib.stage_query(st, C.byref(out)))
    return out


def stage_export_params(st, version: int, dst_dev: int):
    _check(lib.stage_export_params(st, version, _vp(dst_dev)))


def tp_blend_coefficients(policy, delta: int, lam: float):
    a, b = C.c_double(), C.c_double()
    _check(lib.tp_blend_coefficients(POLICY[policy] if isinstance(policy, str) else policy, delta, lam,
                                     C.byref(a), C.byref(b)))
    return a.value, b.value


def tp_schedule_events(num_stages: int, num_minibatches: int):
    """List of (t, kind, stage, mb_id); kind 'F' or 'B'."""
    cap = 2 * num_stages * num_minibatches
    arr = (tp_event * max(cap, 1))()
    cnt = _u64()
    _check(lib.tp_schedule_events(num_stages, num_minibatches, arr, cap, C.byref(cnt)))
    return [(arr[i].t, "FB"[arr[i].kind], arr[i].stage, arr[i].mb_id) for i in range(cnt.value)]


def tp_schedule_microbatch_events(num_stages: int, num_minibatches: int, n: int, mid_pass_updates: bool):
    """List of (t, kind, stage, mb_id, ub); kind 'F' (one micro-batch) or 'B' (backward + update, ub 0)."""
    cap = num_stages * num_minibatches * (n + 1)
    arr = (tp_event * max(cap, 1))()
    cnt = _u64()
    _check(lib.tp_schedule_microbatch_events(num_stages, num_minibatches, n, 1 if mid_pass_updates else 0, arr, cap,
                                             C.byref(cnt)))
    return [(arr[i].t, "FB"[arr[i].kind], arr[i].stage, arr[i].mb_id, arr[i].ub) for i in range(cnt.value)]


def stage_profile_begin(st, max_launches: int):
    _check(lib.stage_profile_begin(st, max_launches))


def stage_profile_end(st) -> dict:
    """Waits for the stage's stream; returns {class: (launches, total_ms)} plus 'dropped'."""
    p = tp_profile()
    _check(lib.stage_profile_end(st, C.byref(p)))
    out = {name: (p.launches[i], p.ms[i]) for i, name in enumerate(KERNEL_CLASSES)}
    out["dropped"] = p.dropped
    return out
