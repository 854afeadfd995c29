"""Packers from row-major logical arrays to the kernel-native weight layouts documented in
include/moespeq.h ("tile16x32" for bf16, slice tiles for the int4 codes and scale/zero, or scales alone in the
symmetric format).

Off the hot path: run once when weights are loaded.  Works on CPU or GPU torch tensors and
returns flat uint8 tensors (byte images of the blobs)."""
import torch


def pack_bf16_matrix(w: torch.Tensor) -> torch.Tensor:
    """[R, C] bf16 -> bytes of the tile16x32 layout (R % 16 == 0, C % 32 == 0)."""
    assert w.dtype == torch.bfloat16 and w.dim() == 2
    R, C = w.shape
    assert R % 16 == 0 and C % 32 == 0
    # [R/16, 16 r, C/32, 4 chunk, 8 elem] -> [R/16, C/32, chunk, r, elem]; lane = chunk*16 + r
    t = w.reshape(R // 16, 16, C // 32, 4, 8).permute(0, 2, 3, 1, 4).contiguous()
    return t.view(torch.uint8).reshape(-1)


def pack_bf16_expert(gate: torch.Tensor, up: torch.Tensor, down: torch.Tensor) -> torch.Tensor:
    """One expert blob: gate [I,H] | up [I,H] | down [H,I]."""
    return torch.cat([pack_bf16_matrix(gate), pack_bf16_matrix(up), pack_bf16_matrix(down)])


# code number n (0..7) of a 32-bit word -> nibble position: even codes fill the low half-word
# nibbles, odd codes the high half-word nibbles, so that (word & 0x000F000F) is the pair (0, 1)
_NIBBLE_OF_CODE = [0, 4, 1, 5, 2, 6, 3, 7]


def _units(q: torch.Tensor) -> torch.Tensor:
    """[R, C] uint8 codes -> [R, C/32, 16] uint8: the 16-byte unit of every 32 codes of a row."""
    assert q.dtype == torch.uint8 and q.dim() == 2 and q.shape[1] % 32 == 0
    R, C = q.shape
    t = q.reshape(R, C // 32, 4, 8).to(torch.int64)                 # [row, unit, word, code]
    word = torch.zeros(t.shape[:-1], dtype=torch.int64, device=q.device)
    for n in range(8):
        word |= t[..., n] << (4 * _NIBBLE_OF_CODE[n])
    b = torch.stack([(word >> (8 * i)) & 0xFF for i in range(4)], dim=-1).to(torch.uint8)
    return b.reshape(R, C // 32, 16)


def _dwords(q: torch.Tensor) -> torch.Tensor:
    """[R, C] codes -> [R, C/32, 4, 4] uint8: row, 32-code unit, 8-code chunk c, the chunk's 4 bytes."""
    R, C = q.shape
    return _units(q).reshape(R, C // 32, 4, 4)


def pack_int4_gateup_codes(qg: torch.Tensor, qu: torch.Tensor) -> torch.Tensor:
    """gate, up codes [I, H] -> tiles (slice, unit): lane = chunk * 16 + r, word d = row block
    (gate rows 0-15, gate rows 16-31, up rows 0-15, up rows 16-31 of the slice)."""
    I, H = qg.shape
    assert qu.shape == (I, H) and I % 32 == 0
    dg = _dwords(qg).reshape(I // 32, 2, 16, H // 32, 4, 4)          # [slice, half, r, unit, chunk, 4B]
    du = _dwords(qu).reshape(I // 32, 2, 16, H // 32, 4, 4)
    t = torch.cat([dg, du], dim=1)                                    # [slice, d, r, unit, chunk, 4B]
    return t.permute(0, 3, 4, 2, 1, 5).contiguous().reshape(-1)      # [slice, unit, chunk, r, d, 4B]


def pack_int4_down_codes(qd: torch.Tensor) -> torch.Tensor:
    """down codes [H, I] -> tiles (slice of 32 input columns, row tile of 64 outputs): lane =
    chunk * 16 + r, word d = rows 16 d + r of the row tile."""
    H, I = qd.shape
    assert H % 64 == 0 and I % 32 == 0
    t = _dwords(qd).reshape(H // 64, 4, 16, I // 32, 4, 4)           # [rt, d, r, slice, chunk, 4B]
    return t.permute(3, 0, 4, 2, 1, 5).contiguous().reshape(-1)      # [slice, rt, chunk, r, d, 4B]


def _sz_pairs(s: torch.Tensor, z: torch.Tensor) -> torch.Tensor:
    assert s.dtype == torch.float16 and z.dtype == torch.float16 and s.shape == z.shape
    return torch.stack([s, z], dim=-1)                               # [..., 2] fp16


def pack_int4_gateup_sz(sg, zg, su, zu) -> torch.Tensor:
    """scale / zero [I, H/g] of gate and up -> entries (slice, group, r, d), d as for the codes."""
    I, G = sg.shape
    pg = _sz_pairs(sg, zg).reshape(I // 32, 2, 16, G, 2)
    pu = _sz_pairs(su, zu).reshape(I // 32, 2, 16, G, 2)
    t = torch.cat([pg, pu], dim=1)                                   # [slice, d, r, group, 2]
    return t.permute(0, 3, 2, 1, 4).contiguous().view(torch.uint8).reshape(-1)


def pack_int4_down_sz(sd, zd) -> torch.Tensor:
    """scale / zero [H, I/g] of down -> entries (group, rt, r, d)."""
    H, G = sd.shape
    t = _sz_pairs(sd, zd).reshape(H // 64, 4, 16, G, 2)              # [rt, d, r, group, 2]
    return t.permute(3, 0, 2, 1, 4).contiguous().view(torch.uint8).reshape(-1)


def pack_int4_gateup_scales(sg, su) -> torch.Tensor:
    """Symmetric format: scales [I, H/g] of gate and up -> fp16 entries (slice, group pair, r,
    group parity, d), d as for the codes."""
    I, G = sg.shape
    assert sg.dtype == torch.float16 and su.dtype == torch.float16 and G % 2 == 0
    t = torch.cat([sg.reshape(I // 32, 2, 16, G // 2, 2), su.reshape(I // 32, 2, 16, G // 2, 2)], dim=1)
    return t.permute(0, 3, 2, 4, 1).contiguous().view(torch.uint8).reshape(-1)   # [slice, pair, r, parity, d]


def pack_int4_down_scales(sd) -> torch.Tensor:
    """Symmetric format: scales [H, I/g] of down -> fp16 entries (group, row-tile pair, r, row-tile
    parity, d)."""
    H, G = sd.shape
    assert sd.dtype == torch.float16 and H % 128 == 0
    t = sd.reshape(H // 128, 2, 4, 16, G)                             # [rt pair, parity, d, r, group]
    return t.permute(4, 0, 3, 1, 2).contiguous().view(torch.uint8).reshape(-1)


def pack_int4_expert_symmetric(q, s):
    """q, s: dicts gate/up/down of one expert whose zero points are all 8 -> (codes blob,
    scale blob)."""
    qb = torch.cat([pack_int4_gateup_codes(q["gate"], q["up"]), pack_int4_down_codes(q["down"])])
    sb = torch.cat([pack_int4_gateup_scales(s["gate"], s["up"]), pack_int4_down_scales(s["down"])])
    return qb, sb


def pack_int4_expert(q, s, z):
    """q, s, z: dicts gate/up/down of one expert -> (codes blob, scale-zero blob)."""
    qb = torch.cat([pack_int4_gateup_codes(q["gate"], q["up"]), pack_int4_down_codes(q["down"])])
    sb = torch.cat([pack_int4_gateup_sz(s["gate"], z["gate"], s["up"], z["up"]),
                    pack_int4_down_sz(s["down"], z["down"])])
    return qb, sb
