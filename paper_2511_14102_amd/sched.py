"""ctypes binding of include/moespeq_sched.h (host-side control plane): argument marshalling only."""
import ctypes
from typing import Optional, Sequence

from . import binding as B

MAX_K = 64


class GovernorConfig(ctypes.Structure):
    _fields_ = [("t_draft_base", ctypes.c_double), ("t_draft_token", ctypes.c_double),
                ("t_pcie_init", ctypes.c_double), ("t_pcie_overhead", ctypes.c_double),
                ("b_pcie", ctypes.c_double), ("s_expert", ctypes.c_double),
                ("n_verify", ctypes.c_int32),
                ("verify_tokens", ctypes.POINTER(ctypes.c_int32)),
                ("verify_seconds", ctypes.POINTER(ctypes.c_double)),
                ("ema_alpha", ctypes.c_double), ("p_init", ctypes.c_double),
                ("k_min", ctypes.c_int32), ("k_max", ctypes.c_int32)]


_ready = False


def _lib():
    global _ready
    L = B.load_library()
    if not _ready:
        vp, i32, dp = ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(ctypes.c_double)
        L.moe_governor_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(GovernorConfig)]
        L.moe_governor_destroy.argtypes = [vp]
        L.moe_governor_observe.argtypes = [vp, i32, i32]
        L.moe_governor_probabilities.argtypes = [vp, dp]
        L.moe_governor_k_accept.argtypes = [vp, i32, dp]
        L.moe_governor_cycle_time.argtypes = [vp, i32, i32, dp]
        L.moe_governor_evaluate.argtypes = [vp, i32, i32, dp, dp]
        L.moe_governor_choose_k.argtypes = [vp, ctypes.POINTER(i32), i32, ctypes.POINTER(i32), dp]
        for n in B.SCHED_EXPORTS:
            getattr(L, n).restype = i32
        _ready = True
    return L


def _check(rc: int, what: str):
    if rc != B.MOE_OK:
        raise B.MoeError(rc, what)


class Governor:
    """moe_governor_* with Python numbers in and out.  cfg: dict with the fields of
    moe_governor_config (verify_tokens / verify_seconds as sequences)."""

    def __init__(self, cfg: dict):
        self._L = _lib()
        vt = (ctypes.c_int32 * len(cfg["verify_tokens"]))(*cfg["verify_tokens"])
        vs = (ctypes.c_double * len(cfg["verify_seconds"]))(*cfg["verify_seconds"])
        c = GovernorConfig(cfg["t_draft_base"], cfg["t_draft_token"], cfg["t_pcie_init"],
                           cfg["t_pcie_overhead"], cfg["b_pcie"], cfg["s_expert"], len(vt), vt, vs,
                           cfg["ema_alpha"], cfg["p_init"], cfg["k_min"], cfg["k_max"])
        h = ctypes.c_void_p()
        _check(self._L.moe_governor_create(ctypes.byref(h), ctypes.byref(c)), "moe_governor_create")
        self._h, self.k_max = h, cfg["k_max"]

    def close(self):
        if getattr(self, "_h", None):
            self._L.moe_governor_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def observe(self, drafted: int, accepted: int):
        _check(self._L.moe_governor_observe(self._h, drafted, accepted), "moe_governor_observe")

    def probabilities(self):
        p = (ctypes.c_double * self.k_max)()
        _check(self._L.moe_governor_probabilities(self._h, p), "moe_governor_probabilities")
        return list(p)

    def k_accept(self, k: int) -> float:
        out = ctypes.c_double()
        _check(self._L.moe_governor_k_accept(self._h, k, ctypes.byref(out)), "moe_governor_k_accept")
        return out.value

    def cycle_time(self, k: int, n_new: int) -> float:
        out = ctypes.c_double()
        _check(self._L.moe_governor_cycle_time(self._h, k, n_new, ctypes.byref(out)), "moe_governor_cycle_time")
        return out.value

    def evaluate(self, k: int, n_new: int):
        th, it = ctypes.c_double(), ctypes.c_double()
        _check(self._L.moe_governor_evaluate(self._h, k, n_new, ctypes.byref(th), ctypes.byref(it)),
               "moe_governor_evaluate")
        return th.value, it.value

    def choose_k(self, n_new_by_k: Sequence[int], k_slo: int = 0):
        arr = (ctypes.c_int32 * len(n_new_by_k))(*n_new_by_k)
        k, th = ctypes.c_int32(), ctypes.c_double()
        _check(self._L.moe_governor_choose_k(self._h, arr, k_slo, ctypes.byref(k), ctypes.byref(th)),
               "moe_governor_choose_k")
        return k.value, th.value
