"""Host-side checks that need no GPU: the packers against the layout formulas documented in
include/moespeq.h (read back element by element from the byte image), the exported symbols,
and the host-only entry points."""
import ctypes
import os
import re

import numpy as np
import pytest
import torch

import synth
from paper_2511_14102_amd import binding as B
from paper_2511_14102_amd import pack

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared(header):
    hdr = open(os.path.join(ROOT, "include", header)).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    return set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", hdr))


def test_library_exports_every_declared_symbol():
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["moespeq.h", "moespeq_sched.h"]
    names = _declared("moespeq.h")
    assert {"moe_route_topk", "moe_draft_layer_int4", "moe_expert_union",
            "moe_verify_layer_bf16", "moe_expert_copy_async"} <= names
    sched = _declared("moespeq_sched.h")
    lib = ctypes.CDLL(B.library_path())
    for n in sorted(names | sched):
        assert hasattr(lib, n), n
    assert names == set(B.EXPORTS)
    assert sched == set(B.SCHED_EXPORTS)


def test_bf16_tile16x32_layout_matches_the_header_formula():
    rng = np.random.default_rng(0)
    R, C = 48, 96
    w = torch.from_numpy(rng.standard_normal((R, C), dtype=np.float32)).to(torch.bfloat16)
    img = pack.pack_bf16_matrix(w).numpy()
    assert img.size == R * C * 2
    bits = w.view(torch.int16).numpy().view(np.uint16)
    for r in range(R):
        for c in range(C):
            tile = (r // 16) * (C // 32) + c // 32
            lane = ((c % 32) // 8) * 16 + r % 16
            o = (tile * 64 + lane) * 16 + (c % 8) * 2
            assert int(img[o]) | (int(img[o + 1]) << 8) == int(bits[r, c])


def _code_at(words, tile, chunk, r, d, n):
    """Code n (0..7) of the word that lane chunk * 16 + r of `tile` holds for row block d."""
    p = n // 2 if n % 2 == 0 else 4 + n // 2
    return (int(words[(tile * 64 + chunk * 16 + r) * 4 + d]) >> (4 * p)) & 15


def test_int4_slice_layout_matches_the_header_formula():
    rng = np.random.default_rng(1)
    H, I, g = 128, 96, 32
    q = {n: torch.from_numpy(rng.integers(0, 16, shp).astype(np.uint8))
         for n, shp in (("gate", (I, H)), ("up", (I, H)), ("down", (H, I)))}
    s = {n: torch.from_numpy(rng.random((q[n].shape[0], q[n].shape[1] // g)).astype(np.float16)) for n in q}
    z = {n: torch.from_numpy(rng.integers(0, 16, s[n].shape).astype(np.float16)) for n in q}
    qb, sb = pack.pack_int4_expert(q, s, z)
    assert qb.numel() == 3 * H * I // 2 and sb.numel() == 3 * H * I // g * 4
    words = qb.numpy().view("<u4")
    n_gu_tiles = (I // 32) * (H // 32)
    for row in range(I):
        for col in range(H):
            sl, u = row // 32, col // 32
            tile = sl * (H // 32) + u
            d, r = (row % 32) // 16, row % 16
            chunk, n = (col % 32) // 8, col % 8
            assert _code_at(words, tile, chunk, r, d, n) == int(q["gate"][row, col])
            assert _code_at(words, tile, chunk, r, d + 2, n) == int(q["up"][row, col])
    for row in range(H):
        for col in range(I):
            tile = n_gu_tiles + (col // 32) * (H // 64) + row // 64
            d, r = (row % 64) // 16, row % 16
            assert _code_at(words, tile, (col % 32) // 8, r, d, col % 8) == int(q["down"][row, col])
    ent = sb.numpy().view("<u2").reshape(-1, 2)
    G = H // g
    bits = lambda t: t.numpy().view(np.uint16)
    for row in range(I):
        for gi in range(G):
            d, r = (row % 32) // 16, row % 16
            i = (((row // 32) * G + gi) * 16 + r) * 4 + d
            assert ent[i, 0] == bits(s["gate"])[row, gi] and ent[i, 1] == bits(z["gate"])[row, gi]
            assert ent[i + 2, 0] == bits(s["up"])[row, gi] and ent[i + 2, 1] == bits(z["up"])[row, gi]
    base = (I // 32) * G * 64
    for row in range(H):
        for gi in range(I // g):
            d, r = (row % 64) // 16, row % 16
            i = base + ((gi * (H // 64) + row // 64) * 16 + r) * 4 + d
            assert ent[i, 0] == bits(s["down"])[row, gi] and ent[i, 1] == bits(z["down"])[row, gi]


def test_symmetric_scale_layout_matches_the_header_formula():
    rng = np.random.default_rng(2)
    H, I, g = 256, 96, 32
    q = {n: torch.from_numpy(rng.integers(0, 16, shp).astype(np.uint8))
         for n, shp in (("gate", (I, H)), ("up", (I, H)), ("down", (H, I)))}
    s = {n: torch.from_numpy(rng.random((q[n].shape[0], q[n].shape[1] // g)).astype(np.float16)) for n in q}
    qb, sb = pack.pack_int4_expert_symmetric(q, s)
    z8 = {n: torch.full_like(s[n], 8.0) for n in s}
    assert torch.equal(qb, pack.pack_int4_expert(q, s, z8)[0])       # the codes do not change
    assert sb.numel() == 3 * H * I // g * 2
    ent = sb.numpy().view("<u2")
    G = H // g
    bits = lambda t: t.numpy().view(np.uint16)
    for row in range(I):
        for gi in range(G):
            d, r = (row % 32) // 16, row % 16
            i = ((((row // 32) * (G // 2) + gi // 2) * 16 + r) * 2 + gi % 2) * 4 + d
            assert ent[i] == bits(s["gate"])[row, gi] and ent[i + 2] == bits(s["up"])[row, gi]
    base = (I // 32) * G * 64
    for row in range(H):
        for gi in range(I // g):
            rt, d, r = row // 64, (row % 64) // 16, row % 16
            i = base + (((gi * (H // 128) + rt // 2) * 16 + r) * 2 + rt % 2) * 4 + d
            assert ent[i] == bits(s["down"])[row, gi]
    d = B.LayerDesc(H, 4, 128, 2, 0, g, 1)
    assert B.int4_expert_scale_bytes(d) == 3 * H * 128 // g * 2 == B.int4_expert_sz_bytes(d) // 2
    # shapes the format cannot hold: an odd number of groups per row, or of 64-row tiles
    assert B.int4_expert_scale_bytes(B.LayerDesc(384, 4, 128, 2, 0, 128, 1)) == 0
    assert B.int4_expert_scale_bytes(B.LayerDesc(192, 4, 64, 2, 0, 32, 1)) == 0
    assert B.int4_expert_sz_bytes(B.LayerDesc(192, 4, 64, 2, 0, 32, 1)) > 0


def test_code_pairs_unpack_with_one_mask():
    # the property the kernel relies on: ((word >> 4j) & 0x000F000F) holds codes (2j, 2j+1)
    q = torch.zeros((64, 32), dtype=torch.uint8)
    q[5, 8:16] = torch.tensor([3, 14, 1, 7, 9, 0, 15, 6], dtype=torch.uint8)
    words = pack.pack_int4_down_codes(q).numpy().view("<u4").reshape(64, 4)   # [lane, d]
    w = int(words[1 * 16 + 5, 0])                                             # chunk 1, r 5, row block 0
    got = []
    for j in range(4):
        m = (w >> (4 * j)) & 0x000F000F
        got += [m & 0xF, (m >> 16) & 0xF]
    assert got == [3, 14, 1, 7, 9, 0, 15, 6]


def test_expert_blob_sizes_and_order():
    cfg = synth.config_by_name("tiny")
    d = B.LayerDesc.from_config(cfg)
    w = synth.make_experts_bf16(cfg, experts=[0])
    blob = pack.pack_bf16_expert(w["gate"][0], w["up"][0], w["down"][0])
    assert blob.numel() == B.bf16_expert_bytes(d) == cfg.bf16_expert_bytes
    n = cfg.hidden * cfg.inter * 2
    assert torch.equal(blob[n:2 * n], pack.pack_bf16_matrix(w["up"][0]))
    assert torch.equal(blob[2 * n:], pack.pack_bf16_matrix(w["down"][0]))
    q, s, z = {}, {}, {}
    for name in ("gate", "up", "down"):
        q[name], s[name], z[name] = synth.quantize_rtn_int4(w[name][0], cfg.group_size)
    qb, sb = pack.pack_int4_expert(q, s, z)
    assert qb.numel() == B.int4_expert_q_bytes(d) and sb.numel() == B.int4_expert_sz_bytes(d)
    assert qb.numel() + sb.numel() == cfg.int4_expert_bytes


def test_host_only_entry_points():
    for cfg in synth.CONFIGS:
        d = B.LayerDesc.from_config(cfg)
        assert B.validate_desc(d) == 0
        assert B.workspace_bytes(d, max(cfg.verify_tokens)) > 0
    bad = [dict(hidden=100), dict(inter=96), dict(n_experts=0), dict(n_experts=257), dict(top_k=0),
           dict(top_k=17), dict(group_size=48), dict(n_shared=5), dict(hidden=64, group_size=128)]
    base = synth.config_by_name("tiny")
    for change in bad:
        d = B.LayerDesc.from_config(base)
        for kk, v in change.items():
            setattr(d, kk, v)
        assert B.validate_desc(d) == B.MOE_ERR_INVALID_ARG, change
        assert B.bf16_expert_bytes(d) == 0
    d = B.LayerDesc.from_config(base)
    with pytest.raises(B.MoeError):
        B.workspace_bytes(d, 17)
    d.top_k = 8
    with pytest.raises(B.MoeError):
        B.workspace_bytes(d, 17)
    assert B.status_string(0) == "ok" and "resident" in B.status_string(-4)
    # what a draft call keeps in LDS must fit in 140 KiB (the formula of the header, evaluated here).  One
    # token: its copy 2 H + 16 + 4 H / g, plus 12 E of routing scratch when E > 32.  More tokens (T rounded
    # up to 2, 4, 8): the copy T (2 H + 16 + 4 H / g), 12 T E of routing scratch, and per wave (8) two copies
    # of the scale / zero entries of its share of one work item in whole KiB.
    def lds_need(H, g, E, cap, sym=False):
        if cap == 1:
            return 2 * H + 16 + 4 * H // g + (12 * E + 8 if E > 32 else 0)
        need = (cap * (2 * H + 16 + 4 * H // g) + 7) // 8 * 8 + 12 * cap * E
        need = (need + 15) // 16 * 16
        epl = 2 if sym else 1
        nw = 8                                             # waves of the workgroup
        blocks = lambda n: ((n // epl + nw - 1) // nw + 3) // 4
        return need + 2 * nw * (blocks(H // g) + blocks(H // 64)) * 1024
    for H, g in ((4096, 128), (8192, 32), (8192, 128), (12288, 128), (16384, 128), (32768, 128), (65536, 128)):
        dd = B.LayerDesc(H, 4, 128, 1, 0, g, 1)
        assert B.validate_desc(dd) == 0
        for T in range(1, 9):
            cap = 1 if T <= 1 else 2 if T <= 2 else 4 if T <= 4 else 8
            fits = lds_need(H, g, 4, cap) <= 140 * 1024
            assert (B.draft_call_fits(dd, T) == 0) == fits, (H, g, T)
    assert B.draft_call_fits(B.LayerDesc(4096, 4, 128, 1, 0, 128, 1), 9) == B.MOE_ERR_INVALID_ARG
    seen = set()
    for H in (4096, 6144, 8192):                       # many experts: the routing scratch counts
        many = B.LayerDesc(H, 256, 128, 8, 0, 128, 1)
        for T in (1, 2, 4, 8):
            fits = lds_need(H, 128, 256, T) <= 140 * 1024
            assert (B.draft_call_fits(many, T) == 0) == fits, (H, T)
            seen.add(fits)
    assert seen == {True, False}
    # prefill: any number of tokens up to the limit
    d = B.LayerDesc.from_config(base)
    assert B.prefill_workspace_bytes(d, 1) > 0
    assert B.prefill_workspace_bytes(d, 4096) >= 2 * 4096 * d.top_k * 4
    for bad_T in (0, 4097):
        with pytest.raises(B.MoeError):
            B.prefill_workspace_bytes(d, bad_T)
    ds = B.LayerDesc.from_config(synth.config_by_name("dsv2lite"))     # shared experts: room for one chunk
    assert B.prefill_workspace_bytes(ds, 16) > B.workspace_bytes(ds, 16)
    lib = B.load_library()
    # a null context is rejected before any device work
    assert lib.moe_route_topk(None, ctypes.byref(d), None, None, None, 1, None, None, None, None,
                              None, None, None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_expert_copy_async(None, None, None, 0, None, None) == B.MOE_ERR_INVALID_ARG
    if not torch.cuda.is_available():
        with pytest.raises(B.MoeError) as ei:
            B.Context(0)
        assert ei.value.status == B.MOE_ERR_HIP
