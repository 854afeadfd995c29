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


# ---- Expert Lookahead Buffer and expert cache --------------------------------------------------
PHASE_PRIME, PHASE_GUIDED, PHASE_SATURATE = 1, 2, 3


class Fetch(ctypes.Structure):
    _fields_ = [("layer", ctypes.c_int32), ("expert", ctypes.c_int32), ("slot", ctypes.c_int32),
                ("evicted", ctypes.c_int32)]

    def astuple(self):
        return (self.layer, self.expert, self.slot, self.evicted)


_ready2 = False


def _lib2():
    global _ready2
    L = _lib()
    if not _ready2:
        vp, i32 = ctypes.c_void_p, ctypes.c_int32
        ip, fp = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_float)
        L.moe_elb_create.argtypes = [ctypes.POINTER(vp), i32, i32, i32]
        L.moe_elb_destroy.argtypes = [vp]
        L.moe_elb_reset.argtypes = [vp]
        L.moe_elb_put_step.argtypes = [vp, i32, ip, fp]
        L.moe_elb_steps.argtypes = [vp, ip]
        L.moe_elb_entry.argtypes = [vp, i32, i32, ip, fp]
        L.moe_cache_create.argtypes = [ctypes.POINTER(vp), i32, i32, i32]
        L.moe_cache_destroy.argtypes = [vp]
        L.moe_cache_place.argtypes = [vp, i32, i32, i32]
        L.moe_cache_slot_table.argtypes = [vp, i32, ip]
        L.moe_cache_use.argtypes = [vp, i32, ip, i32, ip, ip]
        L.moe_cache_stats.argtypes = [vp, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64)]
        L.moe_cache_end_window.argtypes = [vp]
        L.moe_sched_plan.argtypes = [vp, vp, i32, i32, ctypes.c_float, ctypes.POINTER(Fetch), i32, ip]
        L.moe_sched_on_demand.argtypes = [vp, i32, ip, i32, ctypes.POINTER(Fetch)]
        for n in B.SCHED_EXPORTS:
            getattr(L, n).restype = i32
        _ready2 = True
    return L


def _ints(seq):
    seq = [int(v) for v in seq]
    return (ctypes.c_int32 * max(len(seq), 1))(*seq), len(seq)


class Elb:
    def __init__(self, n_layers: int, k_max: int, top_k: int):
        self._L = _lib2()
        h = ctypes.c_void_p()
        _check(self._L.moe_elb_create(ctypes.byref(h), n_layers, k_max, top_k), "moe_elb_create")
        self._h, self.n_layers, self.top_k = h, n_layers, top_k

    def close(self):
        if getattr(self, "_h", None):
            self._L.moe_elb_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def reset(self):
        _check(self._L.moe_elb_reset(self._h), "moe_elb_reset")

    def put_step(self, step: int, ids, conf=None):
        """ids / conf: [n_layers][top_k] nested sequences (or flat)."""
        flat = [int(v) for row in ids for v in (row if hasattr(row, "__len__") else [row])]
        arr, _ = _ints(flat)
        cf = None
        if conf is not None:
            cflat = [float(v) for row in conf for v in (row if hasattr(row, "__len__") else [row])]
            cf = (ctypes.c_float * len(cflat))(*cflat)
        _check(self._L.moe_elb_put_step(self._h, step, arr, cf), "moe_elb_put_step")

    def steps(self) -> int:
        n = ctypes.c_int32()
        _check(self._L.moe_elb_steps(self._h, ctypes.byref(n)), "moe_elb_steps")
        return n.value

    def entry(self, step: int, layer: int):
        ids = (ctypes.c_int32 * self.top_k)()
        cf = (ctypes.c_float * self.top_k)()
        _check(self._L.moe_elb_entry(self._h, step, layer, ids, cf), "moe_elb_entry")
        return list(ids), list(cf)


class Cache:
    def __init__(self, n_layers: int, n_experts: int, n_slots: int):
        self._L = _lib2()
        h = ctypes.c_void_p()
        _check(self._L.moe_cache_create(ctypes.byref(h), n_layers, n_experts, n_slots), "moe_cache_create")
        self._h, self.n_layers, self.n_experts, self.n_slots = h, n_layers, n_experts, n_slots

    def close(self):
        if getattr(self, "_h", None):
            self._L.moe_cache_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def place(self, layer: int, expert: int, slot: int):
        _check(self._L.moe_cache_place(self._h, layer, expert, slot), "moe_cache_place")

    def slot_table(self, layer: int):
        t = (ctypes.c_int32 * self.n_experts)()
        _check(self._L.moe_cache_slot_table(self._h, layer, t), "moe_cache_slot_table")
        return list(t)

    def use(self, layer: int, ids):
        arr, n = _ints(ids)
        h, m = ctypes.c_int32(), ctypes.c_int32()
        _check(self._L.moe_cache_use(self._h, layer, arr, n, ctypes.byref(h), ctypes.byref(m)), "moe_cache_use")
        return h.value, m.value

    def stats(self):
        h, m = ctypes.c_int64(), ctypes.c_int64()
        _check(self._L.moe_cache_stats(self._h, ctypes.byref(h), ctypes.byref(m)), "moe_cache_stats")
        return h.value, m.value

    def end_window(self):
        _check(self._L.moe_cache_end_window(self._h), "moe_cache_end_window")

    def plan(self, elb: Elb, phase: int, max_fetch: int = 0, min_conf: float = 0.0, max_out: Optional[int] = None):
        max_out = self.n_layers * self.n_slots if max_out is None else max_out
        out = (Fetch * max(max_out, 1))()
        n = ctypes.c_int32()
        _check(self._L.moe_sched_plan(self._h, elb._h, phase, max_fetch, min_conf, out, max_out, ctypes.byref(n)),
               "moe_sched_plan")
        return [out[i].astuple() for i in range(n.value)]

    def on_demand(self, layer: int, missing):
        arr, n = _ints(missing)
        out = (Fetch * max(n, 1))()
        _check(self._L.moe_sched_on_demand(self._h, layer, arr, n, out), "moe_sched_on_demand")
        return [out[i].astuple() for i in range(n)]
