"""Packers from row-major logical arrays to the kernel-native weight layouts documented in
include/moespeq.h ("tile16x32" for bf16, "tile64x32" for int4 codes and scale/zero).

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


def pack_int4_codes(q: torch.Tensor) -> torch.Tensor:
    """[R, C] uint8 codes 0..15 -> bytes of the tile64x32 layout (R % 64 == 0, C % 32 == 0)."""
    assert q.dtype == torch.uint8 and q.dim() == 2
    R, C = q.shape
    assert R % 64 == 0 and C % 32 == 0
    t = q.reshape(R // 64, 64, C // 32, 4, 8).to(torch.int64)      # [rt, lane, ku, word, code]
    word = torch.zeros(t.shape[:-1], dtype=torch.int64, device=q.device)
    for n in range(8):
        word |= t[..., n] << (4 * _NIBBLE_OF_CODE[n])
    word = word.permute(0, 2, 1, 3).contiguous()                   # [rt, ku, lane, word]
    b = torch.stack([(word >> (8 * i)) & 0xFF for i in range(4)], dim=-1).to(torch.uint8)
    return b.reshape(-1)


def pack_int4_sz(s: torch.Tensor, z: torch.Tensor) -> torch.Tensor:
    """scale, zero [R, C/g] fp16 -> bytes: [R/64, C/g, 64 lanes, (s, z)]."""
    assert s.dtype == torch.float16 and z.dtype == torch.float16 and s.shape == z.shape
    R, G = s.shape
    assert R % 64 == 0
    t = torch.stack([s, z], dim=-1).reshape(R // 64, 64, G, 2).permute(0, 2, 1, 3).contiguous()
    return t.view(torch.uint8).reshape(-1)


def pack_int4_expert(q, s, z):
    """q, s, z: dicts gate/up/down of one expert -> (codes blob, scale-zero blob)."""
    qb = torch.cat([pack_int4_codes(q[n]) for n in ("gate", "up", "down")])
    sb = torch.cat([pack_int4_sz(s[n], z[n]) for n in ("gate", "up", "down")])
    return qb, sb
