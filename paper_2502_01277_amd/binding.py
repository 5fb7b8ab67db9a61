"""ctypes binding over libocto.so (see include/octo.h).

Argument marshalling only: every step of the path runs inside the library's HIP
kernels.  PyTorch appears here solely as the owner of device memory and streams.
The binding fails loudly when the shared library is missing; there is no CPU
fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from . import zoo
from .synth import to_storage

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libocto.so")

MAX_LEVELS, MAX_ANCHORS, MAX_EDGES, MAX_CHILD_LABELS, MAX_LAYER_INPUTS = 3, 3, 4, 2, 4
OK, EINVAL, ENOMEM, ECAP, ESTATE, EHIP, ENOTREADY = 0, -1, -2, -3, -4, -5, -6
DTYPES = {"f32": 0, "f16": 1, "bf16": 2, "f8": 3}       # f8 (E4M3): octo_op_conv only
OPS = {"conv": 0, "maxpool": 1, "upsample2x": 2, "concat": 3, "add": 4, "gap": 5, "fc": 6}
KINDS = {"detector": 0, "classifier": 1}

CAND_DTYPE = np.dtype([("x1", "<f4"), ("y1", "<f4"), ("x2", "<f4"), ("y2", "<f4"), ("score", "<f4"),
                       ("cls", "<i4"), ("idx", "<i4"), ("pad_", "<i4")])
ROI_DTYPE = np.dtype([("frame", "<i4"), ("rank", "<i4"), ("cls", "<i4"), ("pad_", "<i4"),
                      ("x1", "<f4"), ("y1", "<f4"), ("x2", "<f4"), ("y2", "<f4")])
BOX_DTYPE = np.dtype([("x1", "<f4"), ("y1", "<f4"), ("x2", "<f4"), ("y2", "<f4"), ("score", "<f4"),
                      ("cls", "<i4"), ("child_label", "<i4", (MAX_CHILD_LABELS,))])
FRAME_DTYPE = np.dtype([("frame_id", "<i8"), ("n_boxes", "<i4"), ("latency_ms", "<f4"), ("slo_met", "<i4"),
                        ("flags", "<i4"), ("box_offset", "<i4"), ("pad_", "<i4")])


class OctoLayer(C.Structure):
    _fields_ = [("op", C.c_int32), ("n_in", C.c_int32), ("in_", C.c_int32 * MAX_LAYER_INPUTS),
                ("cout", C.c_int32), ("kh", C.c_int32), ("kw", C.c_int32), ("stride", C.c_int32), ("pad", C.c_int32),
                ("act", C.c_int32), ("res_mode", C.c_int32), ("weight", C.c_void_p), ("bias", C.c_void_p)]


class OctoModelDesc(C.Structure):
    _fields_ = [("name", C.c_char_p), ("dtype", C.c_int32), ("kind", C.c_int32),
                ("in_h", C.c_int32), ("in_w", C.c_int32), ("in_c", C.c_int32),
                ("layers", C.POINTER(OctoLayer)), ("n_layers", C.c_int32),
                ("outputs", C.c_int32 * MAX_LEVELS), ("n_outputs", C.c_int32),
                ("n_classes", C.c_int32), ("n_anchors", C.c_int32), ("stride", C.c_int32 * MAX_LEVELS),
                ("anchors", C.c_float * (MAX_LEVELS * MAX_ANCHORS * 2)),
                ("score_thr", C.c_float), ("iou_thr", C.c_float), ("topk", C.c_int32), ("max_det", C.c_int32),
                ("norm_scale", C.c_float * 3), ("norm_bias", C.c_float * 3), ("pad_value", C.c_int32),
                ("batch_size", C.c_int32)]


class OctoEdge(C.Structure):
    _fields_ = [("parent", C.c_int32), ("child", C.c_int32), ("class_mask", C.c_uint64 * 2)]


class OctoPipelineDesc(C.Structure):
    _fields_ = [("models", C.POINTER(OctoModelDesc)), ("n_models", C.c_int32),
                ("edges", C.POINTER(OctoEdge)), ("n_edges", C.c_int32), ("slo_ms", C.c_float),
                ("src_h", C.c_int32), ("src_w", C.c_int32), ("max_frames", C.c_int32),
                ("max_rois_per_frame", C.c_int32), ("max_queue", C.c_int32), ("keep_all_tensors", C.c_int32)]


class OctoSchedModel(C.Structure):
    _fields_ = [("parent", C.c_int32), ("n_profile", C.c_int32), ("profile_bz", C.c_int32 * 8),
                ("profile_ms", C.c_float * 8), ("rate", C.c_float), ("burstiness", C.c_float), ("util", C.c_float),
                ("weight_mem", C.c_float), ("inter_mem", C.c_float), ("bz", C.c_int32)]


class OctoSchedPipeline(C.Structure):
    _fields_ = [("models", C.POINTER(OctoSchedModel)), ("n_models", C.c_int32), ("slo_ms", C.c_float)]


class OctoPlacement(C.Structure):
    _fields_ = [("pipeline", C.c_int32), ("model", C.c_int32), ("stream", C.c_int32),
                ("start_ms", C.c_float), ("end_ms", C.c_float), ("duty_cycle_ms", C.c_float)]


class OctoPlanModel(C.Structure):
    _fields_ = [("parent", C.c_int32), ("rate", C.c_float), ("burstiness", C.c_float), ("weight_mem", C.c_float), ("inter_mem", C.c_float),
                ("width", C.c_int32), ("n_profile", C.c_int32), ("profile_bz", C.c_int32 * 8), ("profile_ms", (C.c_float * 8) * 4)]


class OctoPlaceModel(C.Structure):
    _fields_ = [("parent", C.c_int32), ("rate", C.c_float), ("burstiness", C.c_float), ("n_profile", C.c_int32), ("profile_bz", C.c_int32 * 8),
                ("server_ms", C.c_float * 8), ("edge_ms", C.c_float * 8), ("in_bytes", C.c_double), ("result_bytes", C.c_double),
                ("bz", C.c_int32), ("on_edge", C.c_int32)]


class OctoExecQueue(C.Structure):
    _fields_ = [("bz", C.c_int32), ("batches_per_cycle", C.c_int32), ("slo_ms", C.c_float),
                ("head_pool", C.POINTER(C.c_void_p)), ("head_item_bytes", C.POINTER(C.c_size_t)), ("n_levels", C.c_int32),
                ("scaler_window", C.c_int32), ("scaler_up", C.c_float), ("scaler_down", C.c_float)]


class OctoExecInstance(C.Structure):
    _fields_ = [("pipe", C.c_void_p), ("queue", C.c_int32), ("standby", C.c_int32), ("streams", C.POINTER(C.c_void_p)),
                ("n_models", C.c_int32), ("slot_ms", C.c_float), ("head_buffers", C.POINTER(C.c_void_p)),
                ("max_frames", C.c_int32), ("max_batch", C.c_int32), ("max_det", C.c_int32)]


class OctoExecCamera(C.Structure):
    _fields_ = [("queue", C.c_int32), ("arrivals_s", C.POINTER(C.c_double)), ("n_arrivals", C.c_int32),
                ("d_frames", C.POINTER(C.c_void_p)), ("pitch_bytes", C.POINTER(C.c_size_t)), ("n_frames", C.c_int32),
                ("pool_offset", C.c_int32)]


class OctoExecDesc(C.Structure):
    _fields_ = [("queues", C.POINTER(OctoExecQueue)), ("n_queues", C.c_int32),
                ("instances", C.POINTER(OctoExecInstance)), ("n_instances", C.c_int32),
                ("cameras", C.POINTER(OctoExecCamera)), ("n_cameras", C.c_int32),
                ("duty_ms", C.c_float), ("slotted", C.c_int32), ("drop_late", C.c_int32), ("keep_results", C.c_int32),
                ("sched", C.POINTER(OctoSchedPipeline)), ("gpu_mem", C.c_double), ("n_streams", C.c_int32),
                ("stream_index", C.POINTER(C.c_int32)), ("stream_handle", C.POINTER(C.c_void_p)),
                ("stream_first_cu", C.POINTER(C.c_int32)), ("stream_n_cu", C.POINTER(C.c_int32)), ("n_sched_streams", C.c_int32),
                ("masked", C.c_int32), ("plain_stream", C.c_void_p)]


class OctoExecStats(C.Structure):
    _fields_ = [("submitted", C.c_int64), ("served", C.c_int64), ("slo_met", C.c_int64), ("boxes", C.c_int64), ("dropped", C.c_int64),
                ("latency_ms_p50", C.c_float), ("latency_ms_p99", C.c_float), ("latency_ms_max", C.c_float)]


class OctoScaleEvent(C.Structure):
    _fields_ = [("t_s", C.c_float), ("queue", C.c_int32), ("change", C.c_int32)]


class OctoConvOp(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("n", C.c_int32), ("h", C.c_int32), ("w", C.c_int32), ("cin", C.c_int32), ("x_ld", C.c_int32),
                ("cout", C.c_int32), ("kh", C.c_int32), ("kw", C.c_int32), ("stride", C.c_int32), ("pad", C.c_int32),
                ("act", C.c_int32), ("res_mode", C.c_int32), ("out_f32", C.c_int32), ("y_ld", C.c_int32), ("res_ld", C.c_int32),
                ("d_x", C.c_void_p), ("d_w", C.c_void_p), ("d_bias", C.c_void_p), ("d_scale", C.c_void_p), ("d_res", C.c_void_p),
                ("d_y", C.c_void_p), ("res_scale", C.c_float), ("y_inv_scale", C.c_float)]


# Every symbol include/octo.h declares.
EXPORTS = [
    "octo_pipeline_workspace_size", "octo_pipeline_create", "octo_pipeline_destroy", "octo_submit_frames", "octo_run",
    "octo_collect", "octo_set_batch_size", "octo_set_detector_batch", "octo_last_error", "octo_now_ms", "octo_stream_create_masked", "octo_stream_create_range",
    "octo_stream_destroy", "octo_device_cu_count", "octo_cwd_search", "octo_coral_schedule", "octo_est_latency_ms",
    "octo_est_throughput", "octo_burstiness", "octo_batches_per_cycle", "octo_width_to_cus", "octo_choose_width", "octo_late_prefix",
    "octo_plan_pipeline", "octo_to_edge", "octo_scaler_create", "octo_scaler_observe", "octo_scaler_destroy", "octo_run_model",
    "octo_executor_create", "octo_executor_serve", "octo_executor_stats", "octo_executor_scale_events", "octo_executor_streams",
    "octo_executor_results", "octo_executor_last_error", "octo_executor_destroy", "octo_profile_layers", "octo_set_layer_timing", "octo_get_layer_info", "octo_set_stage_timing", "octo_get_stage_ms",
    "octo_debug_get_tensor", "octo_debug_tensor_shape", "octo_debug_set_head", "octo_debug_run_model",
    "octo_debug_get_detections", "octo_debug_get_rois", "octo_debug_get_labels", "octo_letterbox_geometry", "octo_op_letterbox",
    "octo_op_crop_resize", "octo_op_decode", "octo_op_topk", "octo_op_nms", "octo_op_nms_scratch_bytes", "octo_op_nms_static", "octo_op_compact", "octo_probe_copy", "octo_probe_mfma",
    "octo_op_conv", "octo_op_conv_packed_bytes", "octo_op_conv_padded_cout", "octo_op_conv_pack", "octo_quantize_e4m3", "octo_dequantize_e4m3",
]

_lib = None


def lib() -> C.CDLL:
    """Load libocto.so (built by paper_2502_01277_amd.build); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libocto.so not found at %s - build it with `python -m paper_2502_01277_amd.build`" % LIB_PATH)
        L = C.CDLL(LIB_PATH)
        L.octo_last_error.restype = C.c_char_p
        L.octo_last_error.argtypes = [C.c_void_p]
        L.octo_now_ms.restype = C.c_double
        L.octo_op_nms_scratch_bytes.restype = C.c_size_t
        L.octo_est_latency_ms.restype = C.c_float
        L.octo_est_throughput.restype = C.c_float
        vp, i32, f32 = C.c_void_p, C.c_int32, C.c_float
        L.octo_pipeline_workspace_size.argtypes = [vp, vp]
        L.octo_pipeline_create.argtypes = [vp, vp, C.c_size_t, vp]
        L.octo_pipeline_destroy.argtypes = [vp]
        L.octo_submit_frames.argtypes = [vp, vp, vp, vp, vp, i32]
        L.octo_run.argtypes = [vp, vp, vp]
        L.octo_run_model.argtypes = [vp, i32, vp, vp]
        L.octo_collect.argtypes = [vp, vp, i32, vp, i32, vp, vp, i32]
        L.octo_set_batch_size.argtypes = [vp, i32, i32]
        L.octo_set_detector_batch.argtypes = [vp, i32]
        L.octo_stream_create_masked.argtypes = [vp, i32, vp]
        L.octo_stream_create_range.argtypes = [i32, i32, vp]
        L.octo_stream_destroy.argtypes = [vp]
        L.octo_device_cu_count.argtypes = [vp]
        L.octo_cwd_search.argtypes = [vp]
        L.octo_coral_schedule.argtypes = [vp, i32, C.c_double, C.c_double, i32, vp]
        L.octo_est_latency_ms.argtypes = [vp]
        L.octo_est_throughput.argtypes = [vp]
        f64 = C.c_double
        L.octo_burstiness.argtypes = [vp, i32, vp]
        L.octo_batches_per_cycle.argtypes = [f64, f64, i32, vp]
        L.octo_width_to_cus.argtypes = [f64, i32, i32, vp]
        L.octo_choose_width.argtypes = [vp, vp, i32, i32, f64, vp]
        L.octo_late_prefix.argtypes = [vp, i32, f64, f64, vp]
        L.octo_to_edge.argtypes = [vp, i32, f32, f64, f64, vp, vp]
        L.octo_plan_pipeline.argtypes = [vp, i32, f32, f64, f64, vp, i32, i32, vp, vp, vp, vp, vp]
        L.octo_scaler_create.argtypes = [f64, i32, f64, f64, i32, vp]
        L.octo_scaler_observe.argtypes = [vp, C.c_int64, C.c_int64, i32, vp]
        L.octo_scaler_destroy.argtypes = [vp]
        L.octo_executor_create.argtypes = [vp, vp]
        L.octo_executor_serve.argtypes = [vp, f64, f64, vp]
        L.octo_executor_stats.argtypes = [vp, i32, vp]
        L.octo_executor_scale_events.argtypes = [vp, vp, i32, vp]
        L.octo_executor_streams.argtypes = [vp, vp, vp, vp, i32, vp]
        L.octo_executor_results.argtypes = [vp, i32, vp, vp, vp, vp, i32, vp, i32, vp, vp]
        L.octo_executor_last_error.argtypes = [vp]
        L.octo_executor_last_error.restype = C.c_char_p
        L.octo_executor_destroy.argtypes = [vp]
        L.octo_profile_layers.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, i32]
        L.octo_set_stage_timing.argtypes = [vp, i32]
        L.octo_set_layer_timing.argtypes = [vp, i32]
        L.octo_get_layer_info.argtypes = [vp, i32, vp, vp, vp, vp, vp, i32, vp]
        L.octo_get_stage_ms.argtypes = [vp, vp, i32, vp]
        L.octo_debug_get_tensor.argtypes = [vp, i32, i32, i32, i32, vp, C.c_size_t]
        L.octo_debug_tensor_shape.argtypes = [vp, i32, i32, vp, vp, vp]
        L.octo_debug_set_head.argtypes = [vp, i32, i32, vp]
        L.octo_debug_run_model.argtypes = [vp, i32, vp, i32, vp]
        L.octo_debug_get_detections.argtypes = [vp, i32, i32, vp, vp, i32, vp, vp, i32, vp]
        L.octo_debug_get_rois.argtypes = [vp, i32, vp, i32, vp]
        L.octo_debug_get_labels.argtypes = [vp, i32, vp, i32, vp]
        L.octo_letterbox_geometry.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp]
        L.octo_op_letterbox.argtypes = [vp, vp, i32, i32, i32, vp, i32, i32, i32, vp, vp, i32, vp]
        L.octo_op_crop_resize.argtypes = [vp, vp, i32, i32, i32, vp, vp, i32, vp, i32, i32, i32, vp, vp, vp]
        L.octo_op_decode.argtypes = [vp, vp, i32, vp, vp, i32, vp]
        L.octo_op_topk.argtypes = [vp, vp, i32, i32, i32, vp, vp, i32, vp]
        L.octo_op_nms.argtypes = [vp, vp, i32, i32, f32, i32, vp, vp, vp, vp]
        L.octo_op_nms_scratch_bytes.argtypes = [i32, i32]
        L.octo_probe_copy.argtypes = [vp, vp, C.c_size_t, i32, vp, vp]
        L.octo_probe_mfma.argtypes = [i32, vp, C.c_size_t, i32, i32, vp, vp]
        L.octo_op_nms_static.argtypes = [vp, vp, i32, i32, f32, i32, vp, vp, vp]
        L.octo_op_compact.argtypes = [vp, i32, vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, vp, i32, vp, vp, vp, vp, vp]
        L.octo_op_conv.argtypes = [vp, vp, vp]
        L.octo_op_conv_packed_bytes.restype = C.c_size_t
        L.octo_op_conv_packed_bytes.argtypes = [i32, i32, i32, i32, i32]
        L.octo_op_conv_padded_cout.argtypes = [i32]
        L.octo_op_conv_pack.argtypes = [i32, vp, i32, i32, i32, i32, vp]
        L.octo_quantize_e4m3.argtypes = [vp, C.c_size_t, f32, vp]
        L.octo_dequantize_e4m3.argtypes = [vp, C.c_size_t, f32, vp]
        _lib = L
    return _lib


class OctoError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__("octo status %d: %s" % (status, msg))
        self.status = status


def _torch():
    import torch
    return torch


def torch_dtype(dtype: str):
    t = _torch()
    return {"f32": t.float32, "f16": t.float16, "bf16": t.bfloat16}[dtype]


def to_device(x_f32: np.ndarray, dtype: str, device="cuda"):
    """fp32 numpy values (representable in `dtype`) -> device tensor of that type."""
    t = _torch()
    raw = to_storage(x_f32, dtype)
    if dtype == "bf16":
        return t.from_numpy(raw.view(np.int16)).to(device).view(t.bfloat16)
    return t.from_numpy(raw).to(device)


def _stream_ptr(stream) -> int:
    if stream is None:
        return int(_torch().cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return stream
    return int(stream.cuda_stream)


def model_desc(m: zoo.ModelSpec, keep: list) -> OctoModelDesc:
    """Marshal a ModelSpec; host arrays the struct points to are appended to `keep`."""
    layers = (OctoLayer * len(m.layers))()
    for i, L in enumerate(m.layers):
        o = layers[i]
        o.op = OPS[L.op]; o.n_in = len(L.inputs)
        for k, t in enumerate(L.inputs):
            o.in_[k] = t
        o.cout, o.kh, o.kw, o.stride, o.pad, o.act, o.res_mode = L.cout, L.kh, L.kw, L.stride, L.pad, L.act, L.res_mode
        if L.weight is not None:
            w = np.ascontiguousarray(to_storage(L.weight, m.dtype))
            b = np.ascontiguousarray(L.bias, dtype=np.float32)
            keep += [w, b]
            o.weight = w.ctypes.data; o.bias = b.ctypes.data
    keep.append(layers)
    d = OctoModelDesc()
    name = m.name.encode(); keep.append(name)
    d.name = name; d.dtype = DTYPES[m.dtype]; d.kind = KINDS[m.kind]
    d.in_h, d.in_w, d.in_c = m.in_h, m.in_w, m.in_c
    d.layers = layers; d.n_layers = len(m.layers)
    for k, t in enumerate(m.outputs):
        d.outputs[k] = t
    d.n_outputs = len(m.outputs)
    d.n_classes, d.n_anchors = m.n_classes, m.n_anchors
    for k, s in enumerate(m.strides):
        d.stride[k] = s
    if m.anchors is not None:
        for l in range(m.anchors.shape[0]):
            for a in range(m.anchors.shape[1]):
                for j in range(2):
                    d.anchors[(l * MAX_ANCHORS + a) * 2 + j] = float(m.anchors[l, a, j])
    d.score_thr, d.iou_thr, d.topk, d.max_det = m.score_thr, m.iou_thr, m.topk, m.max_det
    for c in range(3):
        d.norm_scale[c] = m.norm_scale[c]; d.norm_bias[c] = m.norm_bias[c]
    d.pad_value = m.pad_value; d.batch_size = m.batch_size
    return d


def pipeline_desc(p: zoo.PipelineSpec, keep: list, keep_all_tensors=False) -> OctoPipelineDesc:
    models = (OctoModelDesc * len(p.models))(*[model_desc(m, keep) for m in p.models])
    edges = (OctoEdge * max(1, len(p.edges)))()
    for i, e in enumerate(p.edges):
        edges[i].parent, edges[i].child = e.parent, e.child
        edges[i].class_mask[0] = e.class_mask & ((1 << 64) - 1)
        edges[i].class_mask[1] = (e.class_mask >> 64) & ((1 << 64) - 1)
    keep += [models, edges]
    d = OctoPipelineDesc()
    d.models = models; d.n_models = len(p.models); d.edges = edges; d.n_edges = len(p.edges)
    d.slo_ms = p.slo_ms; d.src_h, d.src_w = p.src_h, p.src_w
    d.max_frames, d.max_rois_per_frame = p.max_frames, p.max_rois_per_frame
    d.max_queue = 0; d.keep_all_tensors = int(keep_all_tensors)
    return d


class Pipeline:
    """Owner of one octo_pipeline handle and of the device workspace behind it."""

    def __init__(self, spec: zoo.PipelineSpec, keep_all_tensors=False, device="cuda"):
        t = _torch()
        self.L = lib()
        self.spec = spec
        self._keep: list = []
        self.desc = pipeline_desc(spec, self._keep, keep_all_tensors)
        nbytes = C.c_size_t(0)
        st = self.L.octo_pipeline_workspace_size(C.byref(self.desc), C.byref(nbytes))
        if st != OK:
            raise OctoError(st, self.L.octo_last_error(None).decode())
        self.workspace_bytes = nbytes.value
        self.workspace = t.empty(nbytes.value + 256, dtype=t.uint8, device=device)
        base = (self.workspace.data_ptr() + 255) & ~255
        self.h = C.c_void_p()
        st = self.L.octo_pipeline_create(C.byref(self.desc), base, nbytes.value, C.byref(self.h))
        if st != OK:
            raise OctoError(st, self.L.octo_last_error(None).decode())
        self._frames_alive: list = []

    def _check(self, st, ok=(OK,)):
        if st not in ok:
            raise OctoError(st, self.L.octo_last_error(self.h).decode())
        return st

    def close(self):
        if self.h:
            self.L.octo_pipeline_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- serving calls ----
    def submit(self, frames: Sequence, arrival_ms: Optional[Sequence[float]] = None, frame_ids: Optional[Sequence[int]] = None):
        """frames: device uint8 tensors [H][W][3] (rows may be strided)."""
        n = len(frames)
        ptrs = (C.c_void_p * n)(*[int(f.data_ptr()) for f in frames])
        pitches = (C.c_size_t * n)(*[int(f.stride(0)) for f in frames])
        arr = (C.c_double * n)(*arrival_ms) if arrival_ms is not None else None
        ids = (C.c_int64 * n)(*frame_ids) if frame_ids is not None else None
        self._frames_alive.append(list(frames))
        if len(self._frames_alive) > 16:
            self._frames_alive.pop(0)
        return self._check(self.L.octo_submit_frames(self.h, ptrs, pitches, arr, ids, n))

    def run(self, stream=None) -> int:
        n = C.c_int32(0)
        self._check(self.L.octo_run(self.h, _stream_ptr(stream), C.byref(n)))
        return n.value

    def run_model(self, model: int, stream=None) -> int:
        n = C.c_int32(0)
        self._check(self.L.octo_run_model(self.h, model, _stream_ptr(stream), C.byref(n)))
        return n.value

    def collect(self, blocking=True, frame_cap=None, box_cap=None):
        frame_cap = frame_cap or 4 * self.spec.max_frames
        box_cap = box_cap or frame_cap * self.spec.models[0].max_det
        frames = np.zeros(frame_cap, FRAME_DTYPE)
        boxes = np.zeros(box_cap, BOX_DTYPE)
        nf, nb = C.c_int32(0), C.c_int32(0)
        st = self._check(self.L.octo_collect(self.h, frames.ctypes.data, frame_cap, boxes.ctypes.data, box_cap,
                                             C.byref(nf), C.byref(nb), 1 if blocking else 0), ok=(OK, ECAP, ENOTREADY))
        return frames[:nf.value], boxes[:nb.value], st

    def set_batch_size(self, model: int, bz: int):
        self._check(self.L.octo_set_batch_size(self.h, model, bz))

    def set_detector_batch(self, frames_per_execution: int):
        self._check(self.L.octo_set_detector_batch(self.h, frames_per_execution))

    # ---- hooks ----
    def tensor_shape(self, model: int, tid: int):
        h, w, c = C.c_int32(), C.c_int32(), C.c_int32()
        self._check(self.L.octo_debug_tensor_shape(self.h, model, tid, C.byref(h), C.byref(w), C.byref(c)))
        return h.value, w.value, c.value

    def get_tensor(self, model: int, tid: int, n: int, first: int = 0) -> np.ndarray:
        """Items [first, first + n) of a tensor of the last run as fp32 numpy [n][h][w][c]."""
        from .synth import from_storage
        h, w, c = self.tensor_shape(model, tid)
        m = self.spec.models[model]
        is_fc = tid > 0 and m.layers[tid - 1].op == "fc"
        dt = "f32" if is_fc else m.dtype
        raw = np.empty((n, h, w, c), {"f32": np.float32, "f16": np.float16, "bf16": np.uint16}[dt])
        self._check(self.L.octo_debug_get_tensor(self.h, model, tid, first, n, raw.ctypes.data, raw.nbytes))
        return from_storage(raw, dt)

    def set_head(self, model: int, level: int, tensor):
        self._check(self.L.octo_debug_set_head(self.h, model, level, None if tensor is None else int(tensor.data_ptr())))

    def run_model_on(self, model: int, x, stream=None):
        self._check(self.L.octo_debug_run_model(self.h, model, int(x.data_ptr()), int(x.shape[0]), _stream_ptr(stream)))

    def get_detections(self, model: int, item: int):
        m = self.spec.models[model]
        kc = (min(m.topk, m.n_cand()) + 63) // 64 * 64
        top = np.zeros(kc, CAND_DTYPE)
        keep = np.zeros(m.max_det, np.int32)
        cc, nt, nk = C.c_int32(), C.c_int32(), C.c_int32()
        self._check(self.L.octo_debug_get_detections(self.h, model, item, C.byref(cc), top.ctypes.data, kc, C.byref(nt),
                                                     keep.ctypes.data, m.max_det, C.byref(nk)))
        return cc.value, top[:nt.value], keep[:nk.value]

    def get_rois(self, edge: int):
        cap = self.spec.max_frames * self.spec.max_rois_per_frame
        rois = np.zeros(cap, ROI_DTYPE)
        n = C.c_int32()
        self._check(self.L.octo_debug_get_rois(self.h, edge, rois.ctypes.data, cap, C.byref(n)))
        return rois[:min(n.value, cap)]

    def get_labels(self, edge: int):
        cap = self.spec.max_frames * self.spec.max_rois_per_frame
        lab = np.zeros(cap, np.int32)
        n = C.c_int32()
        self._check(self.L.octo_debug_get_labels(self.h, edge, lab.ctypes.data, cap, C.byref(n)))
        return lab[:min(n.value, cap)]

    def profile_layers(self, model: int, n: int, iters: int = 10, stream=None):
        nl = len(self.spec.models[model].layers)
        ms = np.zeros(nl, np.float32); fl = np.zeros(nl, np.float64); by = np.zeros(nl, np.float64)
        self._check(self.L.octo_profile_layers(self.h, model, n, iters, _stream_ptr(stream), ms.ctypes.data,
                                               fl.ctypes.data, by.ctypes.data, nl))
        return ms, fl, by

    def set_layer_timing(self, on: bool):
        self._check(self.L.octo_set_layer_timing(self.h, 1 if on else 0))

    def layer_info(self, model: int):
        """(ms, kernel_id, flops per item, bytes per item) per layer for the most recently collected batch."""
        nl = len(self.spec.models[model].layers)
        ms = np.zeros(nl, np.float32); kid = np.zeros(nl, np.int32); fl = np.zeros(nl, np.float64); by = np.zeros(nl, np.float64)
        wb = np.zeros(nl, np.float64)
        n = C.c_int32()
        self._check(self.L.octo_get_layer_info(self.h, model, ms.ctypes.data, kid.ctypes.data, fl.ctypes.data, by.ctypes.data,
                                               wb.ctypes.data, nl, C.byref(n)))
        return ms, kid, fl, by, wb

    def set_stage_timing(self, on: bool):
        self._check(self.L.octo_set_stage_timing(self.h, 1 if on else 0))

    def stage_ms(self) -> np.ndarray:
        ms = np.zeros(32, np.float32); n = C.c_int32()
        self._check(self.L.octo_get_stage_ms(self.h, ms.ctypes.data, 32, C.byref(n)))
        return ms[:n.value]


# ---- stage-level calls -------------------------------------------------------
def _st(st):
    if st != OK:
        raise OctoError(st, "stage call failed")


def frame_tables(frames: Sequence):
    """Device tables (pointers, pitches) for a list of device uint8 frames."""
    t = _torch()
    ptrs = t.tensor([int(f.data_ptr()) for f in frames], dtype=t.int64, device=frames[0].device)
    pitches = t.tensor([int(f.stride(0)) for f in frames], dtype=t.int64, device=frames[0].device)
    return ptrs, pitches


def letterbox_geometry(src_h: int, src_w: int, dst_h: int, dst_w: int):
    """(nw, nh, left, top) of the resized frame inside the model input, from the library (host only)."""
    v = [C.c_int32() for _ in range(4)]
    _st(lib().octo_letterbox_geometry(src_h, src_w, dst_h, dst_w, *[C.byref(x) for x in v]))
    return tuple(int(x.value) for x in v)


def op_letterbox(frames: Sequence, dst_h, dst_w, dtype: str, scale=(1 / 255.0,) * 3, bias=(0.0,) * 3, pad_value=114, stream=None):
    t = _torch()
    ptrs, pitches = frame_tables(frames)
    n, (sh, sw) = len(frames), frames[0].shape[:2]
    out = t.empty((n, dst_h, dst_w, 3), dtype=torch_dtype(dtype), device=frames[0].device)
    sc = (C.c_float * 3)(*scale); bi = (C.c_float * 3)(*bias)
    _st(lib().octo_op_letterbox(ptrs.data_ptr(), pitches.data_ptr(), n, sh, sw, out.data_ptr(), dst_h, dst_w, DTYPES[dtype],
                                sc, bi, pad_value, _stream_ptr(stream)))
    return out


def op_crop_resize(frames: Sequence, rois: np.ndarray, out_h, out_w, dtype: str, cap=None, scale=(1 / 255.0,) * 3,
                   bias=(0.0,) * 3, stream=None):
    t = _torch()
    ptrs, pitches = frame_tables(frames)
    sh, sw = frames[0].shape[:2]
    cap = cap or max(1, len(rois))
    d_rois = t.from_numpy(np.ascontiguousarray(rois).view(np.uint8).reshape(-1)).to(frames[0].device)
    if len(rois) == 0:
        d_rois = t.zeros(32, dtype=t.uint8, device=frames[0].device)
    d_n = t.tensor([len(rois)], dtype=t.int32, device=frames[0].device)
    out = t.zeros((cap, out_h, out_w, 3), dtype=torch_dtype(dtype), device=frames[0].device)
    sc = (C.c_float * 3)(*scale); bi = (C.c_float * 3)(*bias)
    _st(lib().octo_op_crop_resize(ptrs.data_ptr(), pitches.data_ptr(), len(frames), sh, sw, d_rois.data_ptr(), d_n.data_ptr(), cap,
                                  out.data_ptr(), out_h, out_w, DTYPES[dtype], sc, bi, _stream_ptr(stream)))
    return out


def op_decode(m: zoo.ModelSpec, heads: Sequence, cap=None, stream=None):
    """heads: device tensors [n][G][G][A*(5+C)] of the model's type.  Returns (cand tensor uint8 view, counts)."""
    t = _torch()
    keep: list = []
    hdr = zoo.ModelSpec(name=m.name, dtype=m.dtype, in_h=m.in_h, in_w=m.in_w, kind=m.kind)   # geometry and thresholds only
    hdr.outputs = list(range(1, len(m.outputs) + 1))
    hdr.n_classes, hdr.n_anchors, hdr.grids, hdr.strides, hdr.anchors = m.n_classes, m.n_anchors, m.grids, m.strides, m.anchors
    hdr.score_thr, hdr.iou_thr, hdr.topk, hdr.max_det = m.score_thr, m.iou_thr, m.topk, m.max_det
    d = model_desc(hdr, keep)
    n = int(heads[0].shape[0])
    cap = cap or m.n_cand()
    cand = t.zeros((n, cap, 32), dtype=t.uint8, device=heads[0].device)
    count = t.zeros(n, dtype=t.int32, device=heads[0].device)
    hp = (C.c_void_p * len(heads))(*[int(h.data_ptr()) for h in heads])
    _st(lib().octo_op_decode(C.byref(d), hp, n, cand.data_ptr(), count.data_ptr(), cap, _stream_ptr(stream)))
    return cand, count


def cands_to_device(lists: List[np.ndarray], cap: int, device="cuda"):
    """Pack per-item candidate arrays (CAND_DTYPE) into a device table [n][cap] plus counts."""
    t = _torch()
    n = len(lists)
    host = np.zeros((n, cap), CAND_DTYPE)
    for i, l in enumerate(lists):
        host[i, :len(l)] = l
    cand = t.from_numpy(host.view(np.uint8).reshape(n, cap, 32)).to(device)
    count = t.tensor([len(l) for l in lists], dtype=t.int32, device=device)
    return cand, count


def cands_from_device(cand, count) -> List[np.ndarray]:
    c = cand.cpu().numpy().reshape(cand.shape[0], cand.shape[1] * 32).view(CAND_DTYPE)
    k = count.cpu().numpy()
    return [c[i, :min(int(k[i]), c.shape[1])].copy() for i in range(c.shape[0])]


def op_topk(cand, count, k: int, stream=None):
    t = _torch()
    n, in_cap = int(cand.shape[0]), int(cand.shape[1])
    k_cap = (k + 63) // 64 * 64
    out = t.zeros((n, k_cap, 32), dtype=t.uint8, device=cand.device)
    oc = t.zeros(n, dtype=t.int32, device=cand.device)
    _st(lib().octo_op_topk(cand.data_ptr(), count.data_ptr(), in_cap, n, k, out.data_ptr(), oc.data_ptr(), k_cap, _stream_ptr(stream)))
    return out, oc


def op_nms(top, top_count, iou_thr: float, max_det: int, stream=None):
    t = _torch()
    n, k_cap = int(top.shape[0]), int(top.shape[1])
    scratch = t.empty(max(8, lib().octo_op_nms_scratch_bytes(n, k_cap)), dtype=t.uint8, device=top.device)
    keep = t.zeros((n, max_det), dtype=t.int32, device=top.device)
    nk = t.zeros(n, dtype=t.int32, device=top.device)
    _st(lib().octo_op_nms(top.data_ptr(), top_count.data_ptr(), k_cap, n, iou_thr, max_det, scratch.data_ptr(),
                          keep.data_ptr(), nk.data_ptr(), _stream_ptr(stream)))
    return keep, nk


NMS_STATIC_BYTES = 8 << 20


def op_nms_static(top, top_count, iou_thr: float, max_det: int, keep, n_keep, stream=None) -> int:
    """octo_op_nms_static on caller-made output tensors (the call itself allocates nothing); returns the status."""
    n, k_cap = int(top.shape[0]), int(top.shape[1])
    return int(lib().octo_op_nms_static(top.data_ptr(), top_count.data_ptr(), k_cap, n, iou_thr, max_det,
                                        keep.data_ptr(), n_keep.data_ptr(), _stream_ptr(stream)))


def op_compact(top, keep, n_keep, src_hw, in_hw, class_mask: int, cap: int, stream=None):
    t = _torch()
    n, k_cap, max_det = int(top.shape[0]), int(top.shape[1]), int(keep.shape[1])
    dev = top.device
    rois = t.zeros((max(cap, 1), 32), dtype=t.uint8, device=dev)
    n_roi = t.zeros(1, dtype=t.int32, device=dev)
    roi_of = t.full((n, max_det), -1, dtype=t.int32, device=dev)
    boxes = t.zeros((n, max_det, 32), dtype=t.uint8, device=dev)
    flags = t.zeros(n, dtype=t.int32, device=dev)
    item_counts = t.zeros(n, dtype=t.int32, device=dev)
    cm = (C.c_uint64 * 2)(class_mask & ((1 << 64) - 1), (class_mask >> 64) & ((1 << 64) - 1))
    _st(lib().octo_op_compact(top.data_ptr(), k_cap, keep.data_ptr(), n_keep.data_ptr(), max_det, n, src_hw[0], src_hw[1],
                              in_hw[0], in_hw[1], cm, rois.data_ptr(), n_roi.data_ptr(), cap, roi_of.data_ptr(),
                              item_counts.data_ptr(), boxes.data_ptr(), flags.data_ptr(), _stream_ptr(stream)))
    nr = int(n_roi.cpu()[0])
    r = rois.cpu().numpy().reshape(-1).view(ROI_DTYPE)[:nr].copy()
    b = boxes.cpu().numpy().reshape(n, max_det * 32).view(BOX_DTYPE)
    return r, roi_of.cpu().numpy(), b, flags.cpu().numpy()


# ---- one convolution layer ------------------------------------------------------
def quantize_e4m3(x: np.ndarray, inv_scale: float = 1.0) -> np.ndarray:
    """fp32 values -> E4M3 codes of x * inv_scale (host, the library's own rounding)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, np.uint8)
    _st(lib().octo_quantize_e4m3(x.ctypes.data, x.size, inv_scale, out.ctypes.data))
    return out


def dequantize_e4m3(codes: np.ndarray, scale: float = 1.0) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    out = np.empty(codes.shape, np.float32)
    _st(lib().octo_dequantize_e4m3(codes.ctypes.data, codes.size, scale, out.ctypes.data))
    return out


def conv_pack(w_raw: np.ndarray, dtype: str) -> np.ndarray:
    """w_raw [cout][kh][kw][cin] in storage form (to_storage(...), or uint8 codes for f8) -> the packed bytes the kernels read."""
    cout, kh, kw, cin = w_raw.shape
    w_raw = np.ascontiguousarray(w_raw)
    nbytes = lib().octo_op_conv_packed_bytes(DTYPES[dtype], cout, kh, kw, cin)
    if not nbytes:
        raise OctoError(-1, "bad weight shape or type")
    out = np.empty(nbytes, np.uint8)
    _st(lib().octo_op_conv_pack(DTYPES[dtype], w_raw.ctypes.data, cout, kh, kw, cin, out.ctypes.data))
    return out


class ConvOp:
    """Device-side state of one convolution layer for op_conv: packed weights, padded bias and (f8) scale vector."""

    def __init__(self, w_raw: np.ndarray, bias: np.ndarray, dtype: str, stride=1, pad=0, act=0, scale: np.ndarray = None):
        t = _torch()
        self.dtype, self.stride, self.pad, self.act = dtype, stride, pad, act
        self.cout, self.kh, self.kw, self.cin = w_raw.shape
        rows = lib().octo_op_conv_padded_cout(self.cout)
        self.w = t.from_numpy(conv_pack(w_raw, dtype)).cuda()
        b = np.zeros(rows, np.float32); b[:self.cout] = bias
        self.bias = t.from_numpy(b).cuda()
        self.scale = None
        if dtype == "f8":
            sc = np.zeros(rows, np.float32); sc[:self.cout] = scale
            self.scale = t.from_numpy(sc).cuda()

    def out_hw(self, h, w):
        return (h + 2 * self.pad - self.kh) // self.stride + 1, (w + 2 * self.pad - self.kw) // self.stride + 1


def op_conv(layer: ConvOp, x, y, res=None, res_mode=0, out_f32=False, res_scale=0.0, y_inv_scale=1.0, stream=None) -> int:
    """y = conv(x) on device tensors [n][h][w][c] (channels contiguous; a wider last stride is passed on as the pitch).
    Tensors of type f8 are uint8 tensors of E4M3 codes.  Returns the id of the kernel that ran."""
    n, h, w, cin = x.shape
    op = OctoConvOp()
    op.dtype = DTYPES[layer.dtype]
    op.n, op.h, op.w, op.cin, op.x_ld = n, h, w, cin, x.stride(2)
    op.cout, op.kh, op.kw, op.stride, op.pad = layer.cout, layer.kh, layer.kw, layer.stride, layer.pad
    op.act, op.res_mode, op.out_f32 = layer.act, res_mode, 1 if out_f32 else 0
    op.y_ld = y.stride(2)
    op.d_x, op.d_w, op.d_bias, op.d_y = x.data_ptr(), layer.w.data_ptr(), layer.bias.data_ptr(), y.data_ptr()
    op.d_scale = layer.scale.data_ptr() if layer.scale is not None else None
    if res is not None:
        op.d_res, op.res_ld = res.data_ptr(), res.stride(2)
    op.res_scale, op.y_inv_scale = res_scale, y_inv_scale
    kid = C.c_int32(0)
    _st(lib().octo_op_conv(C.byref(op), _stream_ptr(stream), C.byref(kid)))
    return int(kid.value)


# ---- CU-masked streams --------------------------------------------------------
def probe_copy(mib: int = 512, reps: int = 5, stream=None) -> float:
    """GB/s (read + write) of a plain device copy of `mib` MiB, measured by the library's own copy kernel."""
    t = _torch()
    src = t.full((mib << 18,), 1.0, dtype=t.float32, device="cuda")
    dst = t.empty_like(src)
    out = C.c_double()
    _st(lib().octo_probe_copy(src.data_ptr(), dst.data_ptr(), src.numel() * 4, reps, _stream_ptr(stream), C.byref(out)))
    return float(out.value)


def probe_mfma(dtype: str = "bf16", iters: int = 20000, reps: int = 3, stream=None) -> float:
    """TFLOP/s of a register-only MFMA loop with random operand values (what the matrix cores sustain at their real clock)."""
    t = _torch()
    scratch = t.empty(1 << 20, dtype=t.float32, device="cuda")
    out = C.c_double()
    _st(lib().octo_probe_mfma(DTYPES[dtype], scratch.data_ptr(), scratch.numel() * 4, iters, reps, _stream_ptr(stream), C.byref(out)))
    return float(out.value)


def device_cu_count() -> int:
    n = C.c_int32(0)
    _st(lib().octo_device_cu_count(C.byref(n)))
    return n.value


def stream_create_range(first_cu: int, n_cu: int) -> int:
    """Raw HIP stream restricted to compute units [first_cu, first_cu + n_cu); release with stream_destroy."""
    h = C.c_void_p()
    _st(lib().octo_stream_create_range(first_cu, n_cu, C.byref(h)))
    return int(h.value)


def stream_destroy(stream: int):
    _st(lib().octo_stream_destroy(C.c_void_p(stream)))


# ---- scheduling ---------------------------------------------------------------
# ---- run-time rules of the serving loop (host only) ----
def burstiness(times) -> float:
    a = np.ascontiguousarray(times, np.float64)
    out = C.c_double()
    _st(lib().octo_burstiness(a.ctypes.data if a.size else None, int(a.size), C.byref(out)))
    return float(out.value)


def batches_per_cycle(rate_per_s: float, duty_ms: float, bz: int) -> int:
    out = C.c_int32()
    _st(lib().octo_batches_per_cycle(float(rate_per_s), float(duty_ms), int(bz), C.byref(out)))
    return int(out.value)


def width_to_cus(util: float, total_cus: int, grain: int = 8) -> int:
    out = C.c_int32()
    _st(lib().octo_width_to_cus(float(util), int(total_cus), int(grain), C.byref(out)))
    return int(out.value)


def choose_width(latency_by_width: dict, rule: str = "efficient", tol: float = 0.10) -> int:
    ws = np.asarray(list(latency_by_width), np.int32)
    lat = np.asarray([latency_by_width[int(w)] for w in ws], np.float64)
    out = C.c_int32()
    _st(lib().octo_choose_width(ws.ctypes.data, lat.ctypes.data, int(ws.size), 0 if rule == "latency" else 1, float(tol), C.byref(out)))
    return int(out.value)


def late_prefix(arrival_ms, now_ms: float, slo_ms: float) -> int:
    a = np.ascontiguousarray(arrival_ms, np.float64)
    out = C.c_int32()
    _st(lib().octo_late_prefix(a.ctypes.data if a.size else None, int(a.size), float(now_ms), float(slo_ms), C.byref(out)))
    return int(out.value)


class Scaler:
    """octo_scaler: the horizontal-scaling decision of one pipeline."""

    def __init__(self, capacity: float, window: int = 5, up: float = 1.0, down: float = 0.75, max_instances: int = 2):
        self.h = C.c_void_p()
        _st(lib().octo_scaler_create(float(capacity), int(window), float(up), float(down), int(max_instances), C.byref(self.h)))

    def observe(self, arrived: int, backlog: int, n_active: int) -> int:
        out = C.c_int32()
        _st(lib().octo_scaler_observe(self.h, int(arrived), int(backlog), int(n_active), C.byref(out)))
        return int(out.value)

    def close(self):
        if self.h:
            lib().octo_scaler_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def plan_pipeline(models: Sequence[dict], slo_ms: float, duty_ms: float, cycle_share: float, widths: Sequence[int], total_cus: int,
                  fixed_bz: Optional[Sequence[int]] = None):
    """octo_plan_pipeline.  models: dicts with parent, rate, burstiness, weight_mem, inter_mem, width and by_width {compute
    units: {batch size: ms}}.  Returns (model dicts as sched_pipeline takes them, batches per cycle, est. latency, est. throughput)."""
    ws = list(widths)
    arr = (OctoPlanModel * len(models))()
    for i, m in enumerate(models):
        a = arr[i]
        a.parent, a.rate, a.burstiness, a.weight_mem, a.inter_mem, a.width = m["parent"], m["rate"], m["burstiness"], m["weight_mem"], m["inter_mem"], m["width"]
        bzs = sorted(m["by_width"][ws[0]])
        a.n_profile = len(bzs)
        for k, b in enumerate(bzs):
            a.profile_bz[k] = b
            for j, w in enumerate(ws):
                a.profile_ms[j][k] = m["by_width"][w][b]
    out = (OctoSchedModel * len(models))()
    ks = (C.c_int32 * len(models))()
    lat, thr = C.c_float(), C.c_float()
    wa = (C.c_int32 * len(ws))(*ws)
    fb = (C.c_int32 * len(models))(*fixed_bz) if fixed_bz is not None else None
    _st(lib().octo_plan_pipeline(arr, len(models), slo_ms, duty_ms, cycle_share, wa, len(ws), total_cus, fb, out, ks, C.byref(lat), C.byref(thr)))
    res = [dict(parent=o.parent, profile={o.profile_bz[k]: o.profile_ms[k] for k in range(o.n_profile)}, rate=o.rate, burstiness=o.burstiness,
                util=o.util, weight_mem=o.weight_mem, inter_mem=o.inter_mem, bz=o.bz) for o in out]
    return res, [int(k) for k in ks], float(lat.value), float(thr.value)


def to_edge(models: Sequence[dict], slo_ms: float, bandwidth_bytes_per_s: float, alpha: float = 1.0):
    """octo_to_edge.  models: dicts with parent, rate, burstiness, server_ms {bz: ms}, edge_ms {bz: ms}, in_bytes, result_bytes, bz.
    Returns ([(on_edge, bz)] per model, estimated latency ms, estimated throughput per second)."""
    arr = (OctoPlaceModel * len(models))()
    for i, m in enumerate(models):
        a = arr[i]
        a.parent, a.rate, a.burstiness, a.in_bytes, a.result_bytes, a.bz = m["parent"], m["rate"], m["burstiness"], m["in_bytes"], m.get("result_bytes", 0.0), m["bz"]
        bzs = sorted(m["server_ms"])
        a.n_profile = len(bzs)
        for k, b in enumerate(bzs):
            a.profile_bz[k], a.server_ms[k], a.edge_ms[k] = b, m["server_ms"][b], m["edge_ms"][b]
    lat, thr = C.c_float(), C.c_float()
    _st(lib().octo_to_edge(arr, len(models), slo_ms, bandwidth_bytes_per_s, alpha, C.byref(lat), C.byref(thr)))
    return [(bool(a.on_edge), int(a.bz)) for a in arr], float(lat.value), float(thr.value)


def sched_pipeline(models: Sequence[dict], slo_ms: float, keep: list) -> OctoSchedPipeline:
    """models: dicts with parent, profile {bz: ms}, rate, burstiness, util, weight_mem, inter_mem, bz."""
    arr = (OctoSchedModel * len(models))()
    for i, m in enumerate(models):
        a = arr[i]
        a.parent = m["parent"]
        bzs = sorted(m["profile"])
        a.n_profile = len(bzs)
        for k, b in enumerate(bzs):
            a.profile_bz[k] = b; a.profile_ms[k] = m["profile"][b]
        a.rate = m.get("rate", 15.0); a.burstiness = m.get("burstiness", 0.0); a.util = m.get("util", 0.25)
        a.weight_mem = m.get("weight_mem", 0.0); a.inter_mem = m.get("inter_mem", 0.0); a.bz = m.get("bz", 1)
    keep.append(arr)
    p = OctoSchedPipeline()
    p.models = arr; p.n_models = len(models); p.slo_ms = slo_ms
    return p


def cwd_search(models: Sequence[dict], slo_ms: float) -> List[int]:
    keep: list = []
    p = sched_pipeline(models, slo_ms, keep)
    _st(lib().octo_cwd_search(C.byref(p)))
    return [p.models[i].bz for i in range(len(models))]


def coral_schedule(pipelines: Sequence[tuple], mem: float, util_max: float, n_streams: int):
    """pipelines: (models, slo_ms) tuples with bz already chosen.  Returns placement tuples."""
    keep: list = []
    ps = (OctoSchedPipeline * len(pipelines))(*[sched_pipeline(m, slo, keep) for m, slo in pipelines])
    total = sum(len(m) for m, _ in pipelines)
    out = (OctoPlacement * total)()
    _st(lib().octo_coral_schedule(ps, len(pipelines), mem, util_max, n_streams, out))
    return [(o.pipeline, o.model, o.stream, o.start_ms, o.end_ms, o.duty_cycle_ms) for o in out]


# ---- slot executor (octo_executor_*) -----------------------------------------
@dataclass
class PipelineStats:
    submitted: int = 0
    served: int = 0
    slo_met: int = 0
    boxes: int = 0
    dropped: int = 0                    # requests dropped at batch formation because they were already late
    latency_ms: Tuple[float, float, float] = (0.0, 0.0, 0.0)       # p50, p99, max
    results: Dict[int, Tuple[int, np.ndarray]] = field(default_factory=dict)   # frame id -> (pool index, boxes)


class SlotExecutor:
    """The library's slot executor (octo_executor_*; Sec. III-C 'Inference Stream', Sec. III-D, Sec. IV-A) fed from a
    Schedule: this class creates the schedule's streams, installs the planted-head buffers, marshals the description and
    reads the statistics back.  The serving loop, batch formation, lazy dropping and scaling all run in the library.

    spares: one stand-by copy per pipeline (or None) for the run-time scaler; scaler: dict(window, up, down)."""

    def __init__(self, pipes: List["Pipeline"], schedule, cameras: List,
                 head_pools: Optional[List[Optional[List]]] = None, slotted: bool = True, masked: bool = True,
                 keep_results: bool = False, drop_late: bool = False,
                 spares: Optional[List[Optional[Pipeline]]] = None, scaler: Optional[dict] = None):
        import torch
        L = lib()
        self.pipes, self.sch, self.keep_results = pipes, schedule, keep_results
        self._keep: list = [cameras, head_pools]
        self._owned: List[int] = []
        self._plain = torch.cuda.Stream()
        plain = int(self._plain.cuda_stream)
        streams = {}
        for st, (first, n) in schedule.stream_cus.items():
            streams[st] = plain
            if masked:
                streams[st] = stream_create_range(first, n)
                self._owned.append(streams[st])
        head_pools = head_pools or [None] * len(pipes)

        def stream_of(i, m):
            """A model Algorithm 2 could not place follows its parent's stream (a root: the first stream)."""
            st = schedule.placement(i, m)[2]
            if st >= 0:
                return streams[st]
            parent = {e.child: e.parent for e in pipes[i].spec.edges}.get(m, -1)
            return stream_of(i, parent) if parent >= 0 else (streams[min(streams)] if streams else plain)

        def vp_array(vals):
            arr = (C.c_void_p * max(1, len(vals)))(*vals)
            self._keep.append(arr)
            return arr

        queues = (OctoExecQueue * len(pipes))()
        for i, P in enumerate(pipes):
            q, hp = queues[i], head_pools[i]
            q.bz, q.batches_per_cycle, q.slo_ms = schedule.bz[i][0], schedule.batches_per_cycle[i][0], P.spec.slo_ms
            if hp is not None:
                q.n_levels = len(hp)
                q.head_pool = vp_array([int(h.data_ptr()) for h in hp])
                sizes = (C.c_size_t * len(hp))(*[int(h[0].numel() * h.element_size()) for h in hp])
                self._keep.append(sizes)
                q.head_item_bytes = sizes
            sc = scaler or {}
            q.scaler_window, q.scaler_up, q.scaler_down = sc.get("window", 0), sc.get("up", 0.0), sc.get("down", 0.0)
        copies = [(i, P) for i, P in enumerate(spares or []) if P is not None and slotted]
        self._override = []
        inst = (OctoExecInstance * (len(pipes) + len(copies)))()
        for k, (i, P, standby) in enumerate([(i, P, 0) for i, P in enumerate(pipes)] + [(i, P, 1) for i, P in copies]):
            I, nm = inst[k], len(P.spec.models)
            I.pipe, I.queue, I.standby, I.n_models = P.h.value, i, standby, nm
            I.streams = vp_array([stream_of(i, m) for m in range(nm)])
            I.slot_ms = schedule.placement(i, 0)[3]
            I.max_frames, I.max_batch, I.max_det = P.spec.max_frames, P.spec.models[0].batch_size, P.spec.models[0].max_det
            if head_pools[i] is not None:
                bufs = [torch.empty((P.spec.max_frames,) + tuple(h.shape[1:]), dtype=h.dtype, device=h.device) for h in head_pools[i]]
                for l, b in enumerate(bufs):
                    P.set_head(0, l, b)
                self._override.append((P, bufs))
                I.head_buffers = vp_array([int(b.data_ptr()) for b in bufs])
        cams = (OctoExecCamera * max(1, len(cameras)))()
        for k, c in enumerate(cameras):
            arr = np.ascontiguousarray(c.arrivals_s, np.float64)
            pit = (C.c_size_t * len(c.pool))(*[int(f.stride(0)) for f in c.pool])
            self._keep += [arr, pit]
            cams[k].queue, cams[k].n_arrivals, cams[k].n_frames, cams[k].pool_offset = c.pipeline, arr.size, len(c.pool), c.pool_offset
            cams[k].arrivals_s = arr.ctypes.data_as(C.POINTER(C.c_double))
            cams[k].d_frames = vp_array([int(f.data_ptr()) for f in c.pool])
            cams[k].pitch_bytes = pit
        d = OctoExecDesc()
        d.queues, d.n_queues, d.instances, d.n_instances, d.cameras, d.n_cameras = queues, len(pipes), inst, len(inst), cams, len(cameras)
        d.duty_ms, d.slotted, d.drop_late, d.keep_results = schedule.duty_ms, int(slotted), int(drop_late), int(keep_results)
        d.masked, d.plain_stream = int(masked), plain
        if copies:
            ps = (OctoSchedPipeline * len(pipes))(*[sched_pipeline(m, slo, self._keep) for m, slo in schedule.coral_inputs])
            d.sched, d.gpu_mem, d.n_streams = ps, schedule.gpu_mem_mb, schedule.n_streams
        idx = sorted(streams)
        d.n_sched_streams = len(idx)
        i32s = lambda v: (C.c_int32 * max(1, len(v)))(*v)
        d.stream_index, d.stream_handle = i32s(idx), vp_array([streams[s] for s in idx])
        d.stream_first_cu, d.stream_n_cu = i32s([schedule.stream_cus[s][0] for s in idx]), i32s([schedule.stream_cus[s][1] for s in idx])
        self._keep += [queues, inst, cams, d]
        self.h = C.c_void_p()
        _st(L.octo_executor_create(C.byref(d), C.byref(self.h)))
        self.stats = [PipelineStats() for _ in pipes]
        self.stream_cus: Dict[int, Tuple[int, int]] = dict(schedule.stream_cus)
        self.scale_events: List[Tuple[float, int, int]] = []

    def close(self):
        if self.h:
            lib().octo_executor_destroy(self.h)
            self.h = C.c_void_p()
        for h in self._owned:
            stream_destroy(h)
        self._owned = []
        for P, bufs in self._override:
            for l in range(len(bufs)):
                P.set_head(0, l, None)
        self._override = []

    def serve(self, duration_s: float, drain_s: float = 2.0) -> dict:
        L = lib()
        wall = C.c_double()
        st = L.octo_executor_serve(self.h, float(duration_s), float(drain_s), C.byref(wall))
        if st != OK:
            raise OctoError(st, L.octo_executor_last_error(self.h).decode())
        per = []
        for i, S in enumerate(self.stats):
            r = OctoExecStats()
            _st(L.octo_executor_stats(self.h, i, C.byref(r)))
            S.submitted, S.served, S.slo_met, S.boxes, S.dropped = r.submitted, r.served, r.slo_met, r.boxes, r.dropped
            S.latency_ms = (r.latency_ms_p50, r.latency_ms_p99, r.latency_ms_max)
            per.append(dict(pipeline=self.pipes[i].spec.name, submitted=S.submitted, served=S.served, slo_met=S.slo_met,
                            dropped=S.dropped, objects=S.boxes, latency_ms_p50=r.latency_ms_p50,
                            latency_ms_p99=r.latency_ms_p99, latency_ms_max=r.latency_ms_max))
            if self.keep_results:
                nf, nb = C.c_int32(), C.c_int32()
                L.octo_executor_results(self.h, i, None, None, None, None, 0, None, 0, C.byref(nf), C.byref(nb))      # sizes
                ids, pool = np.zeros(max(1, nf.value), np.int64), np.zeros(max(1, nf.value), np.int32)
                off, cnt = np.zeros(max(1, nf.value), np.int32), np.zeros(max(1, nf.value), np.int32)
                bx = np.zeros(max(1, nb.value), BOX_DTYPE)
                _st(L.octo_executor_results(self.h, i, ids.ctypes.data, pool.ctypes.data, off.ctypes.data, cnt.ctypes.data, ids.size,
                                                    bx.ctypes.data, bx.size, C.byref(nf), C.byref(nb)))
                S.results = {int(ids[k]): (int(pool[k]), bx[off[k]: off[k] + cnt[k]].copy()) for k in range(nf.value)}
        n = C.c_int32()
        ev = (OctoScaleEvent * 256)()
        L.octo_executor_scale_events(self.h, ev, 256, C.byref(n))
        self.scale_events = [(round(ev[k].t_s, 3), ev[k].queue, ev[k].change) for k in range(min(256, n.value))]
        si, sf, sn = (C.c_int32 * 64)(), (C.c_int32 * 64)(), (C.c_int32 * 64)()
        L.octo_executor_streams(self.h, si, sf, sn, 64, C.byref(n))
        self.stream_cus = {si[k]: (sf[k], sn[k]) for k in range(min(64, n.value))}
        span = max(duration_s, 1e-9)
        return dict(duration_s=duration_s, wall_s=wall.value, per_pipeline=per,
                    effective_frames_per_s=sum(S.slo_met for S in self.stats) / span,
                    total_frames_per_s=sum(S.served for S in self.stats) / span,
                    objects_per_s=sum(S.boxes for S in self.stats) / span,
                    slo_attainment=sum(S.slo_met for S in self.stats) / max(1, sum(S.submitted for S in self.stats)),
                    dropped=sum(S.dropped for S in self.stats), scale_events=self.scale_events)
