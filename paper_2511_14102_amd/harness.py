"""Device-side bookkeeping around the C ABI for tests, smoke and benchmark: packs one layer's
weights into the kernel-native blobs, owns the expert-slot pool / slot table / workspace
tensors, and wraps the entry points so that a call takes and returns torch tensors.
No arithmetic of the layer happens here."""
from typing import Dict, Optional, Sequence

import torch

from . import binding as B
from . import pack


class DeviceLayer:
    """One MoE layer resident on the GPU.

    L: a layer in the logical layouts (see synth.gen): 'router', 'router_bias', 'gate', 'up',
    'down' (bf16, E+S experts) and, when the draft path is wanted, 'q_*', 's_*', 'z_*'.
    resident: expert ids that get a slot (default: all E, expert e in slot e); others are absent
    until load_expert() is called.  n_slots: size of the slot pool (default len(resident)).
    symmetric: the int4 experts go to the device in the symmetric format (scale blobs); every
    zero point of L must then be 8."""

    def __init__(self, ctx: B.Context, cfg, L: Dict, max_tokens: int,
                 resident: Optional[Sequence[int]] = None, n_slots: Optional[int] = None,
                 draft: bool = True, verify: bool = True, device: str = "cuda:0",
                 symmetric: bool = False):
        self.ctx, self.cfg, self.dev = ctx, cfg, torch.device(device)
        self.desc = B.LayerDesc.from_config(cfg)
        assert B.validate_desc(self.desc) == 0, "unsupported layer shape"
        E, S = cfg.n_experts, cfg.n_shared
        dev = self.dev
        self.router = L["router"].to(dev).contiguous()
        self.bias = None if L.get("router_bias") is None else L["router_bias"].to(dev).contiguous()
        self.bf16_bytes = B.bf16_expert_bytes(self.desc)
        self.q_bytes = B.int4_expert_q_bytes(self.desc)
        self.symmetric = bool(symmetric)
        self.sz_bytes = B.int4_expert_scale_bytes(self.desc) if symmetric else B.int4_expert_sz_bytes(self.desc)
        assert self.sz_bytes > 0, "shape not supported by the symmetric format"
        self.workspace = torch.empty(B.workspace_bytes(self.desc, max_tokens), dtype=torch.uint8, device=dev)
        ctx.workspace_init(self.workspace)
        self.max_tokens = max_tokens

        self.shared = None
        if S:
            self.shared = torch.empty(S * self.bf16_bytes, dtype=torch.uint8, device=dev)
            for s in range(S):
                self.shared[s * self.bf16_bytes:(s + 1) * self.bf16_bytes] = self._pack_bf16(L, E + s)
        self.q_blob = self.sz_blob = None
        if draft:
            self.q_blob = torch.empty(E * self.q_bytes, dtype=torch.uint8, device=dev)
            self.sz_blob = torch.empty(E * self.sz_bytes, dtype=torch.uint8, device=dev)
            for e in range(E):
                q, s, z = ({n: L[p + n][e].to(dev) for n in ("gate", "up", "down")} for p in ("q_", "s_", "z_"))
                if symmetric:
                    assert all(bool((v == 8).all()) for v in z.values()), "symmetric format needs z = 8"
                    qb, sb = pack.pack_int4_expert_symmetric(q, s)
                else:
                    qb, sb = pack.pack_int4_expert(q, s, z)
                self.q_blob[e * self.q_bytes:(e + 1) * self.q_bytes] = qb
                self.sz_blob[e * self.sz_bytes:(e + 1) * self.sz_bytes] = sb
        self.slot_pool = self.slot_of_expert = None
        if verify:
            resident = list(range(E)) if resident is None else list(resident)
            self.n_slots = len(resident) if n_slots is None else n_slots
            assert self.n_slots >= len(resident)
            self.slot_pool = torch.empty(max(self.n_slots, 1) * self.bf16_bytes, dtype=torch.uint8, device=dev)
            table = torch.full((E,), -1, dtype=torch.int32)
            for slot, e in enumerate(resident):
                self.slot_view(slot).copy_(self._pack_bf16(L, e))
                table[e] = slot
            self.slot_host = table.clone()
            self.slot_of_expert = table.to(dev)
        self.missing = torch.zeros(E, dtype=torch.int32, device=dev)
        self.n_missing = torch.zeros(1, dtype=torch.int32, device=dev)

    def _pack_bf16(self, L, e):
        dev = self.dev
        return pack.pack_bf16_expert(L["gate"][e].to(dev), L["up"][e].to(dev), L["down"][e].to(dev))

    def slot_view(self, slot: int) -> torch.Tensor:
        return self.slot_pool[slot * self.bf16_bytes:(slot + 1) * self.bf16_bytes]

    def set_slot(self, expert: int, slot: int):
        """Marks `expert` resident in `slot` (the blob must already be, or be about to be, there)."""
        self.slot_host[expert] = slot
        self.slot_of_expert[expert] = slot

    # ---- entry points -------------------------------------------------------------------
    def route(self, x: torch.Tensor, with_perm: bool = True, stream=None):
        T, k, E = x.shape[0], self.cfg.top_k, self.cfg.n_experts
        dev = self.dev
        ids = torch.empty((T, k), dtype=torch.int32, device=dev)
        w = torch.empty((T, k), dtype=torch.float32, device=dev)
        conf = torch.empty((T, k), dtype=torch.float32, device=dev)
        cnt = off = pm = None
        if with_perm:
            cnt = torch.empty(E, dtype=torch.int32, device=dev)
            off = torch.empty(E + 1, dtype=torch.int32, device=dev)
            pm = torch.empty(T * k, dtype=torch.int32, device=dev)
        self.ctx.route_topk(self.desc, x, self.router, self.bias, T, ids, w, conf, cnt, off, pm, stream)
        return dict(ids=ids, w=w, conf=conf, count=cnt, off=off, perm=pm)

    def draft(self, x: torch.Tensor, y=None, ids=None, conf=None, stream=None):
        T, k = x.shape[0], self.cfg.top_k
        dev = self.dev
        y = torch.empty((T, self.cfg.hidden), dtype=torch.float32, device=dev) if y is None else y
        ids = torch.empty((T, k), dtype=torch.int32, device=dev) if ids is None else ids
        conf = torch.empty((T, k), dtype=torch.float32, device=dev) if conf is None else conf
        self.ctx.draft_layer_int4(self.desc, x, self.router, self.bias, self.q_blob, self.sz_blob,
                                  self.q_bytes, self.sz_bytes, self.shared, T, y, ids, conf,
                                  self.workspace, stream, symmetric=self.symmetric)
        return dict(y=y, ids=ids, conf=conf)

    def prefill(self, x: torch.Tensor, y=None, ids=None, conf=None, stream=None):
        """The draft layer over a long run of tokens (moe_draft_prefill_int4)."""
        T, k = x.shape[0], self.cfg.top_k
        dev = self.dev
        y = torch.empty((T, self.cfg.hidden), dtype=torch.float32, device=dev) if y is None else y
        ids = torch.empty((T, k), dtype=torch.int32, device=dev) if ids is None else ids
        conf = torch.empty((T, k), dtype=torch.float32, device=dev) if conf is None else conf
        need = B.prefill_workspace_bytes(self.desc, T)
        if getattr(self, "_prefill_ws", None) is None or self._prefill_ws.numel() < need:
            self._prefill_ws = torch.empty(need, dtype=torch.uint8, device=dev)
        self.ctx.draft_prefill_int4(self.desc, x, self.router, self.bias, self.q_blob, self.sz_blob,
                                    self.q_bytes, self.sz_bytes, self.shared, T, y, ids, conf, self._prefill_ws,
                                    stream, symmetric=self.symmetric)
        return dict(y=y, ids=ids, conf=conf)

    def verify(self, x: torch.Tensor, flags: int = 0, y=None, ids=None, stream=None):
        T, k = x.shape[0], self.cfg.top_k
        dev = self.dev
        y = torch.empty((T, self.cfg.hidden), dtype=torch.bfloat16, device=dev) if y is None else y
        ids = torch.empty((T, k), dtype=torch.int32, device=dev) if ids is None else ids
        self.ctx.verify_layer_bf16(self.desc, x, self.router, self.bias, self.slot_pool,
                                   self.bf16_bytes, self.slot_of_expert, self.shared, T, flags, y, ids,
                                   self.missing, self.n_missing, self.workspace, stream)
        return dict(y=y, ids=ids, missing=self.missing, n_missing=self.n_missing)

    def union(self, ids: torch.Tensor, use_slots: bool = True, stream=None):
        E = self.cfg.n_experts
        dev = self.dev
        mask = torch.empty((E + 63) // 64, dtype=torch.int64, device=dev)
        lst = torch.empty(E, dtype=torch.int32, device=dev)
        miss = torch.empty(E, dtype=torch.int32, device=dev)
        nl = torch.empty(1, dtype=torch.int32, device=dev)
        nm = torch.empty(1, dtype=torch.int32, device=dev)
        flat = ids.reshape(-1).contiguous()
        self.ctx.expert_union(flat, flat.numel(), E, self.slot_of_expert if use_slots else None,
                              mask, lst, nl, miss, nm, stream)
        return dict(mask=mask, list=lst, n_list=nl, missing=miss, n_missing=nm)
