"""ctypes front end of the fp64 CPU oracle (moe_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by the
cpu_baseline leg of bench.py.  Nothing here imports the GPU package, and the GPU package
never imports this.

Arrays are numpy: 16-bit formats travel as uint16 bit patterns, int4 codes as one uint8 per
code, everything else int32 / float32 / float64.  `bits()` turns a torch bf16 / fp16 tensor
into that uint16 view without changing a bit.
"""
import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_LIB = os.path.join(_HERE, "libmoe_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile moe_oracle.c with gcc (fp contraction off so that a*b+c is two roundings, as
    written)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared", "-std=c11",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.check_call(cmd)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.orc_num_threads.restype = ctypes.c_int
        L.orc_bf16_to_f64.restype = ctypes.c_double
        L.orc_bf16_to_f64.argtypes = [ctypes.c_uint16]
        L.orc_fp16_to_f64.restype = ctypes.c_double
        L.orc_fp16_to_f64.argtypes = [ctypes.c_uint16]
        _lib = L
    return _lib


def bits(t) -> np.ndarray:
    """uint16 bit patterns of a torch bf16/fp16 tensor (or of a numpy float16 array)."""
    if isinstance(t, np.ndarray):
        if t.dtype == np.uint16:
            return np.ascontiguousarray(t)
        assert t.dtype == np.float16
        return np.ascontiguousarray(t).view(np.uint16)
    import torch
    assert t.dtype in (torch.bfloat16, torch.float16), t.dtype
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a)
    assert a.dtype == dtype, (a.dtype, dtype)
    return a


def num_threads() -> int:
    return int(lib().orc_num_threads())


def set_num_threads(n: int) -> None:
    lib().orc_set_num_threads(ctypes.c_int(n))


def bf16_to_f64(b: int) -> float:
    return float(lib().orc_bf16_to_f64(int(b)))


def fp16_to_f64(h: int) -> float:
    return float(lib().orc_fp16_to_f64(int(h)))


def route(x_bits, wr_bits, bias, k: int, renormalize: bool = True):
    """-> ids [T,k] int32, w [T,k] f64, conf [T,k] f64, logits [T,E] f64"""
    x = _c(x_bits, np.uint16); wr = _c(wr_bits, np.uint16)
    T, H = x.shape
    E, H2 = wr.shape
    assert H == H2 and 1 <= k <= E
    b = None if bias is None else _c(np.asarray(bias, dtype=np.float32), np.float32)
    ids = np.empty((T, k), np.int32)
    w = np.empty((T, k), np.float64)
    conf = np.empty((T, k), np.float64)
    logits = np.empty((T, E), np.float64)
    lib().orc_route(_p(x), _p(wr), _p(b), T, H, E, k, int(bool(renormalize)),
                    _p(ids), _p(w), _p(conf), _p(logits))
    return ids, w, conf, logits


def perm(ids, n_experts: int):
    """-> count [E], off [E+1], perm [n]"""
    a = _c(np.asarray(ids, dtype=np.int32).reshape(-1), np.int32)
    assert a.size == 0 or (a.min() >= 0 and a.max() < n_experts)
    count = np.empty(n_experts, np.int32)
    off = np.empty(n_experts + 1, np.int32)
    pm = np.empty(a.size, np.int32)
    lib().orc_perm(_p(a), a.size, n_experts, _p(count), _p(off), _p(pm))
    return count, off, pm


def union(ids, n_experts: int, slot_of_expert=None):
    """-> mask [ceil(E/64)] uint64, list (ascending unique ids), missing (listed, slot -1)"""
    a = _c(np.asarray(ids, dtype=np.int32).reshape(-1), np.int32)
    assert a.size == 0 or (a.min() >= 0 and a.max() < n_experts)
    slot = None if slot_of_expert is None else _c(np.asarray(slot_of_expert, np.int32), np.int32)
    mask = np.empty((n_experts + 63) // 64, np.uint64)
    lst = np.empty(n_experts, np.int32)
    miss = np.empty(n_experts, np.int32)
    nl = ctypes.c_int32(0)
    nm = ctypes.c_int32(0)
    lib().orc_union(_p(a), a.size, n_experts, _p(slot), _p(mask), _p(lst), ctypes.byref(nl),
                    _p(miss), ctypes.byref(nm))
    return mask, lst[:nl.value].copy(), miss[:nm.value].copy()


def dequant(q, s_bits, z_bits, g: int) -> np.ndarray:
    q = _c(q, np.uint8); s = _c(s_bits, np.uint16); z = _c(z_bits, np.uint16)
    R, C = q.shape
    assert s.shape == (R, C // g) and z.shape == s.shape and C % g == 0
    out = np.empty((R, C), np.float64)
    lib().orc_dequant(_p(q), _p(s), _p(z), R, C, g, _p(out))
    return out


def ffn_bf16(wg_bits, wu_bits, wd_bits, x_f64) -> np.ndarray:
    wg = _c(wg_bits, np.uint16); wu = _c(wu_bits, np.uint16); wd = _c(wd_bits, np.uint16)
    I, H = wg.shape
    assert wu.shape == (I, H) and wd.shape == (H, I)
    x = _c(np.asarray(x_f64, np.float64), np.float64)
    assert x.shape == (H,)
    out = np.empty(H, np.float64)
    lib().orc_ffn_bf16(_p(wg), _p(wu), _p(wd), H, I, _p(x), _p(out))
    return out


def ffn_int4(qg, sg, zg, qu, su, zu, qd, sd, zd, g: int, x_f64) -> np.ndarray:
    qg = _c(qg, np.uint8); qu = _c(qu, np.uint8); qd = _c(qd, np.uint8)
    I, H = qg.shape
    assert qu.shape == (I, H) and qd.shape == (H, I)
    arrs = [_c(a, np.uint16) for a in (sg, zg, su, zu, sd, zd)]
    assert arrs[0].shape == (I, H // g) and arrs[4].shape == (H, I // g)
    x = _c(np.asarray(x_f64, np.float64), np.float64)
    out = np.empty(H, np.float64)
    lib().orc_ffn_int4(_p(qg), _p(arrs[0]), _p(arrs[1]), _p(qu), _p(arrs[2]), _p(arrs[3]),
                       _p(qd), _p(arrs[4]), _p(arrs[5]), H, I, g, _p(x), _p(out))
    return out


def layer_bf16(x_bits, wg_bits, wu_bits, wd_bits, n_experts: int, ids, w, present=None):
    """Verify-pass layer.  wg/wu [E+S,I,H], wd [E+S,H,I] uint16.  -> y [T,H] f64"""
    x = _c(x_bits, np.uint16)
    wg = _c(wg_bits, np.uint16); wu = _c(wu_bits, np.uint16); wd = _c(wd_bits, np.uint16)
    T, H = x.shape
    Etot, I, H2 = wg.shape
    assert H2 == H and wu.shape == wg.shape and wd.shape == (Etot, H, I)
    S = Etot - n_experts
    ids = _c(np.asarray(ids, np.int32), np.int32)
    w = _c(np.asarray(w, np.float64), np.float64)
    k = ids.shape[1]
    assert ids.shape == (T, k) and w.shape == (T, k)
    pr = None if present is None else _c(np.asarray(present, np.uint8), np.uint8)
    y = np.empty((T, H), np.float64)
    lib().orc_layer_bf16(_p(x), _p(wg), _p(wu), _p(wd), T, H, I, n_experts, S, k,
                         _p(ids), _p(w), _p(pr), _p(y))
    return y


def layer_int4(x_bits, q, s_bits, z_bits, g: int, ids, w, shared=None):
    """Draft-pass layer.  q, s_bits, z_bits: dicts with keys gate/up/down ([E,rows,cols] uint8,
    [E,rows,cols/g] uint16).  shared: None or (wg [S,I,H], wu, wd [S,H,I]) uint16."""
    x = _c(x_bits, np.uint16)
    T, H = x.shape
    qg = _c(q["gate"], np.uint8); qu = _c(q["up"], np.uint8); qd = _c(q["down"], np.uint8)
    E, I, H2 = qg.shape
    assert H2 == H and qd.shape == (E, H, I)
    sz = {}
    for n in ("gate", "up", "down"):
        sz["s" + n] = _c(s_bits[n], np.uint16)
        sz["z" + n] = _c(z_bits[n], np.uint16)
    assert sz["sgate"].shape == (E, I, H // g) and sz["zdown"].shape == (E, H, I // g)
    ids = _c(np.asarray(ids, np.int32), np.int32)
    w = _c(np.asarray(w, np.float64), np.float64)
    k = ids.shape[1]
    if shared is None:
        S, swg, swu, swd = 0, None, None, None
    else:
        swg, swu, swd = (_c(a, np.uint16) for a in shared)
        S = swg.shape[0]
        assert swg.shape == (S, I, H) and swd.shape == (S, H, I)
    y = np.empty((T, H), np.float64)
    lib().orc_layer_int4(_p(x), _p(qg), _p(sz["sgate"]), _p(sz["zgate"]),
                         _p(qu), _p(sz["sup"]), _p(sz["zup"]),
                         _p(qd), _p(sz["sdown"]), _p(sz["zdown"]),
                         _p(swg), _p(swu), _p(swd), T, H, I, E, S, k, g,
                         _p(ids), _p(w), _p(y))
    return y
