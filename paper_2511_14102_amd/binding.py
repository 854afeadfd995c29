"""ctypes binding of libmoespeq.so.  Same names as the C ABI; torch tensors are used only as
device-memory handles (data_ptr) and streams.  There is no fallback: if the library is not
built, or a call fails, an exception is raised."""
import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("MOESPEQ_LIB") or os.path.join(_HERE, "libmoespeq.so")
_lib = None

MOE_VERIFY_ACCUMULATE = 1
MOE_VERIFY_ONLY_LISTED = 2
MOE_VERIFY_STRICT = 4
MOE_DRAFT_OK, MOE_DRAFT_TIMED_OUT = 0, 1
MOE_MAX_TOKENS, MOE_MAX_DRAFT_TOKENS, MOE_MAX_PREFILL_TOKENS = 16, 8, 4096
MOE_OK, MOE_ERR_INVALID_ARG, MOE_ERR_WORKSPACE, MOE_ERR_HIP, MOE_ERR_MISSING_EXPERT = 0, -1, -2, -3, -4

EXPORTS = [
    "moe_create", "moe_destroy", "moe_status_string", "moe_last_hip_error", "moe_validate_desc",
    "moe_draft_call_fits",
    "moe_bf16_expert_bytes", "moe_int4_expert_q_bytes", "moe_int4_expert_sz_bytes",
    "moe_int4_expert_scale_bytes", "moe_workspace_bytes", "moe_workspace_init",
    "moe_workspace_idle_bytes", "moe_set_draft_spin_limit", "moe_draft_status", "moe_route_topk",
    "moe_draft_layer_int4", "moe_noalloc_scratch_bytes", "moe_draft_layer_int4_noalloc",
    "moe_prefill_workspace_bytes", "moe_draft_prefill_int4", "moe_expert_union",
    "moe_verify_layer_bf16", "moe_expert_copy_async",
    "moe_profile_enable", "moe_profile_read", "moe_kernel_name", "moe_stream_read_probe",
]
# include/moespeq_sched.h (host-side control plane)
SCHED_EXPORTS = [
    "moe_governor_create", "moe_governor_destroy", "moe_governor_observe", "moe_governor_probabilities",
    "moe_governor_k_accept", "moe_governor_cycle_time", "moe_governor_evaluate", "moe_governor_choose_k",
    "moe_elb_create", "moe_elb_destroy", "moe_elb_reset", "moe_elb_put_step", "moe_elb_steps", "moe_elb_entry",
    "moe_cache_create", "moe_cache_destroy", "moe_cache_place", "moe_cache_slot_table", "moe_cache_use",
    "moe_cache_stats", "moe_cache_end_window", "moe_sched_plan", "moe_sched_on_demand",
]
KERNEL_COUNT = 12


class MoeError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__("%s: status %d (%s)" % (what, status, status_string(status)))
        self.status = status


class LayerDesc(ctypes.Structure):
    _fields_ = [("hidden", ctypes.c_int32), ("n_experts", ctypes.c_int32), ("inter", ctypes.c_int32),
                ("top_k", ctypes.c_int32), ("n_shared", ctypes.c_int32),
                ("group_size", ctypes.c_int32), ("renormalize", ctypes.c_int32)]

    @classmethod
    def from_config(cls, cfg):
        return cls(cfg.hidden, cfg.n_experts, cfg.inter, cfg.top_k, cfg.n_shared, cfg.group_size,
                   cfg.renormalize)


class Int4Experts(ctypes.Structure):
    _fields_ = [("q", ctypes.c_void_p), ("sz", ctypes.c_void_p),
                ("expert_stride_q", ctypes.c_size_t), ("expert_stride_sz", ctypes.c_size_t),
                ("symmetric", ctypes.c_int32)]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads the built library; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError("libmoespeq.so is not built: run `python -m paper_2511_14102_amd.build` "
                               "(or __graft_entry__.build())")
        L = ctypes.CDLL(_LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        dp = ctypes.POINTER(LayerDesc)
        L.moe_create.argtypes = [ctypes.POINTER(vp), i32]
        L.moe_destroy.argtypes = [vp]
        L.moe_status_string.argtypes = [i32]; L.moe_status_string.restype = ctypes.c_char_p
        L.moe_last_hip_error.argtypes = [vp]; L.moe_last_hip_error.restype = ctypes.c_char_p
        L.moe_validate_desc.argtypes = [dp]
        L.moe_draft_call_fits.argtypes = [dp, i32]
        for n in ("moe_bf16_expert_bytes", "moe_int4_expert_q_bytes", "moe_int4_expert_sz_bytes",
                  "moe_int4_expert_scale_bytes"):
            getattr(L, n).argtypes = [dp]; getattr(L, n).restype = sz
        L.moe_workspace_bytes.argtypes = [dp, i32, ctypes.POINTER(sz)]
        L.moe_workspace_init.argtypes = [vp, vp, sz, vp]
        L.moe_workspace_idle_bytes.argtypes = [dp, ctypes.POINTER(sz)]
        L.moe_set_draft_spin_limit.argtypes = [vp, ctypes.c_uint32]
        L.moe_draft_status.argtypes = [vp, vp, sz, ctypes.POINTER(ctypes.c_int32), vp]
        L.moe_route_topk.argtypes = [vp, dp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp]
        L.moe_draft_layer_int4.argtypes = [vp, dp, vp, vp, vp, ctypes.POINTER(Int4Experts), vp, i32,
                                           vp, vp, vp, vp, sz, vp]
        L.moe_noalloc_scratch_bytes.argtypes = []; L.moe_noalloc_scratch_bytes.restype = sz
        L.moe_draft_layer_int4_noalloc.argtypes = [vp, dp, vp, vp, vp, ctypes.POINTER(Int4Experts), vp, i32,
                                                   vp, vp, vp, vp]
        L.moe_prefill_workspace_bytes.argtypes = [dp, i32, ctypes.POINTER(sz)]
        L.moe_draft_prefill_int4.argtypes = [vp, dp, vp, vp, vp, ctypes.POINTER(Int4Experts), vp, i32,
                                             vp, vp, vp, vp, sz, vp]
        L.moe_expert_union.argtypes = [vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, vp]
        L.moe_verify_layer_bf16.argtypes = [vp, dp, vp, vp, vp, vp, sz, vp, vp, i32, i32,
                                            vp, vp, vp, vp, vp, sz, vp]
        L.moe_expert_copy_async.argtypes = [vp, vp, vp, sz, vp, vp]
        L.moe_profile_enable.argtypes = [vp, i32]
        L.moe_profile_read.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_double),
                                       ctypes.POINTER(ctypes.c_int64)]
        L.moe_kernel_name.argtypes = [i32]; L.moe_kernel_name.restype = ctypes.c_char_p
        L.moe_stream_read_probe.argtypes = [vp, vp, ctypes.c_size_t, i32, vp, vp]
        for n in EXPORTS:
            if n not in ("moe_status_string", "moe_last_hip_error", "moe_bf16_expert_bytes",
                         "moe_int4_expert_q_bytes", "moe_int4_expert_sz_bytes",
                         "moe_int4_expert_scale_bytes", "moe_kernel_name", "moe_noalloc_scratch_bytes"):
                getattr(L, n).restype = i32
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return load_library().moe_status_string(status).decode()


def validate_desc(desc: LayerDesc) -> int:
    return load_library().moe_validate_desc(ctypes.byref(desc))


def draft_call_fits(desc: LayerDesc, T: int) -> int:
    return load_library().moe_draft_call_fits(ctypes.byref(desc), T)


def bf16_expert_bytes(desc: LayerDesc) -> int:
    return load_library().moe_bf16_expert_bytes(ctypes.byref(desc))


def int4_expert_q_bytes(desc: LayerDesc) -> int:
    return load_library().moe_int4_expert_q_bytes(ctypes.byref(desc))


def int4_expert_sz_bytes(desc: LayerDesc) -> int:
    return load_library().moe_int4_expert_sz_bytes(ctypes.byref(desc))


def int4_expert_scale_bytes(desc: LayerDesc) -> int:
    return load_library().moe_int4_expert_scale_bytes(ctypes.byref(desc))


def workspace_bytes(desc: LayerDesc, max_tokens: int) -> int:
    out = ctypes.c_size_t(0)
    rc = load_library().moe_workspace_bytes(ctypes.byref(desc), max_tokens, ctypes.byref(out))
    if rc != MOE_OK:
        raise MoeError(rc, "moe_workspace_bytes")
    return out.value


def workspace_idle_bytes(desc: LayerDesc) -> int:
    out = ctypes.c_size_t(0)
    rc = load_library().moe_workspace_idle_bytes(ctypes.byref(desc), ctypes.byref(out))
    if rc != MOE_OK:
        raise MoeError(rc, "moe_workspace_idle_bytes")
    return out.value


def noalloc_scratch_bytes() -> int:
    return load_library().moe_noalloc_scratch_bytes()


def prefill_workspace_bytes(desc: LayerDesc, T: int) -> int:
    out = ctypes.c_size_t(0)
    rc = load_library().moe_prefill_workspace_bytes(ctypes.byref(desc), T, ctypes.byref(out))
    if rc != MOE_OK:
        raise MoeError(rc, "moe_prefill_workspace_bytes")
    return out.value


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


class Context:
    """moe_create / moe_destroy plus one method per entry point."""

    def __init__(self, device: int = 0):
        self._lib = load_library()
        h = ctypes.c_void_p()
        rc = self._lib.moe_create(ctypes.byref(h), device)
        if rc != MOE_OK:
            raise MoeError(rc, "moe_create")
        self._h = h
        self.device = device

    def close(self):
        if getattr(self, "_h", None):
            self._lib.moe_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int, what: str):
        if rc != MOE_OK:
            extra = ""
            if rc == MOE_ERR_HIP:
                extra = " [" + self._lib.moe_last_hip_error(self._h).decode() + "]"
            raise MoeError(rc, what + extra)

    def workspace_init(self, workspace, stream=None):
        self._check(self._lib.moe_workspace_init(self._h, _ptr(workspace),
                                                 workspace.numel() * workspace.element_size(),
                                                 _stream(stream)), "moe_workspace_init")

    def set_draft_spin_limit(self, polls: int):
        self._check(self._lib.moe_set_draft_spin_limit(self._h, polls), "moe_set_draft_spin_limit")

    def draft_status(self, workspace, stream=None) -> int:
        out = ctypes.c_int32(-1)
        self._check(self._lib.moe_draft_status(self._h, _ptr(workspace), workspace.numel() * workspace.element_size(),
                                               ctypes.byref(out), _stream(stream)), "moe_draft_status")
        return out.value

    def route_topk(self, desc, x, w_router, router_bias, T, topk_ids, topk_w, topk_conf=None,
                   counts=None, offsets=None, perm=None, stream=None):
        self._check(self._lib.moe_route_topk(self._h, ctypes.byref(desc), _ptr(x), _ptr(w_router),
                                             _ptr(router_bias), T, _ptr(topk_ids), _ptr(topk_w),
                                             _ptr(topk_conf), _ptr(counts), _ptr(offsets), _ptr(perm),
                                             _stream(stream)), "moe_route_topk")

    def draft_layer_int4(self, desc, x, w_router, router_bias, q_blob, sz_blob, stride_q, stride_sz,
                         shared_bf16, T, y_f32, ids_out, conf_out, workspace, stream=None,
                         symmetric=False):
        ex = Int4Experts(q_blob.data_ptr(), sz_blob.data_ptr(), stride_q, stride_sz, int(bool(symmetric)))
        self._check(self._lib.moe_draft_layer_int4(
            self._h, ctypes.byref(desc), _ptr(x), _ptr(w_router), _ptr(router_bias), ctypes.byref(ex),
            _ptr(shared_bf16), T, _ptr(y_f32), _ptr(ids_out), _ptr(conf_out), _ptr(workspace),
            workspace.numel() * workspace.element_size(), _stream(stream)), "moe_draft_layer_int4")

    def draft_layer_int4_noalloc(self, desc, x, w_router, router_bias, q_blob, sz_blob, stride_q, stride_sz,
                                 shared_bf16, T, y_f32, ids_out, conf_out, stream=None, symmetric=False):
        ex = Int4Experts(q_blob.data_ptr(), sz_blob.data_ptr(), stride_q, stride_sz, int(bool(symmetric)))
        self._check(self._lib.moe_draft_layer_int4_noalloc(
            self._h, ctypes.byref(desc), _ptr(x), _ptr(w_router), _ptr(router_bias), ctypes.byref(ex),
            _ptr(shared_bf16), T, _ptr(y_f32), _ptr(ids_out), _ptr(conf_out), _stream(stream)),
            "moe_draft_layer_int4_noalloc")

    def draft_prefill_int4(self, desc, x, w_router, router_bias, q_blob, sz_blob, stride_q, stride_sz,
                           shared_bf16, T, y_f32, ids_out, conf_out, workspace, stream=None, symmetric=False):
        ex = Int4Experts(q_blob.data_ptr(), sz_blob.data_ptr(), stride_q, stride_sz, int(bool(symmetric)))
        self._check(self._lib.moe_draft_prefill_int4(
            self._h, ctypes.byref(desc), _ptr(x), _ptr(w_router), _ptr(router_bias), ctypes.byref(ex),
            _ptr(shared_bf16), T, _ptr(y_f32), _ptr(ids_out), _ptr(conf_out), _ptr(workspace),
            workspace.numel() * workspace.element_size(), _stream(stream)), "moe_draft_prefill_int4")

    def expert_union(self, ids, n_ids, n_experts, slot_of_expert, mask, lst, n_list, missing,
                     n_missing, stream=None):
        self._check(self._lib.moe_expert_union(self._h, _ptr(ids), n_ids, n_experts,
                                               _ptr(slot_of_expert), _ptr(mask), _ptr(lst),
                                               _ptr(n_list), _ptr(missing), _ptr(n_missing),
                                               _stream(stream)), "moe_expert_union")

    def verify_layer_bf16(self, desc, x, w_router, router_bias, slot_pool, slot_stride,
                          slot_of_expert, shared_bf16, T, flags, y_bf16, ids_out, missing, n_missing,
                          workspace, stream=None):
        self._check(self._lib.moe_verify_layer_bf16(
            self._h, ctypes.byref(desc), _ptr(x), _ptr(w_router), _ptr(router_bias), _ptr(slot_pool),
            slot_stride, _ptr(slot_of_expert), _ptr(shared_bf16), T, flags, _ptr(y_bf16),
            _ptr(ids_out), _ptr(missing), _ptr(n_missing), _ptr(workspace),
            workspace.numel() * workspace.element_size(), _stream(stream)), "moe_verify_layer_bf16")

    def expert_copy_async(self, dst_slot, src_pinned, nbytes, copy_stream, done_event=None):
        ev = None
        if done_event is not None:
            ev = ctypes.c_void_p(done_event.cuda_event)
        self._check(self._lib.moe_expert_copy_async(self._h, _ptr(dst_slot), _ptr(src_pinned), nbytes,
                                                    _stream(copy_stream), ev), "moe_expert_copy_async")

    def stream_read_probe(self, src, nbytes, workgroups, sink, stream=None):
        self._check(self._lib.moe_stream_read_probe(self._h, _ptr(src), nbytes, workgroups, _ptr(sink),
                                                    _stream(stream)), "moe_stream_read_probe")

    def profile_enable(self, enable: bool):
        self._check(self._lib.moe_profile_enable(self._h, int(bool(enable))), "moe_profile_enable")

    def profile_read(self):
        """{kernel name: (total ms, launches)} since the last read."""
        out = {}
        for kid in range(KERNEL_COUNT):
            ms, n = ctypes.c_double(0), ctypes.c_int64(0)
            self._check(self._lib.moe_profile_read(self._h, kid, ctypes.byref(ms), ctypes.byref(n)),
                        "moe_profile_read")
            out[self._lib.moe_kernel_name(kid).decode()] = (ms.value, n.value)
        return out
