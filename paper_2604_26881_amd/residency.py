"""On-demand residency of expert-block weights (FaaSMoE Sec. 3: expert blocks are instantiated on
demand and released when idle, so only the blocks a workload activates hold memory; Sec. 4.3.1:
memory follows expert demand instead of model size).

The GPU form: the weights of all E experts stay in pinned host memory; the device holds a pool of
``slots`` block buffers (g experts each).  A block invocation first makes its block resident - a hit
costs nothing, a miss evicts the least recently used block and copies g experts (three tensors)
host -> device on a copy stream - and then runs the ordinary block call on the pool slot.  The
compute kernels are the library's: a slot is handed over as "the full weight tensor" whose base
pointer is moved back by ``lo`` experts, so that expert id e in [lo, lo+g) lands inside the slot; ids
outside the block are never dereferenced by a block call.

Orchestration only (which block, which slot, which stream waits for which event); the arithmetic of
a block call is the same as with fully resident weights, bit for bit.
"""
from __future__ import annotations

from collections import OrderedDict
from typing import Dict, List, Optional, Tuple

import torch

from .binding import MoeError, _check, _ptr, _stream, load


class ExpertResidency:
    def __init__(self, Wg_host: torch.Tensor, Wu_host: torch.Tensor, Wd_host: torch.Tensor, g: int, slots: int,
                 device="cuda"):
        """Wg_host, Wu_host [E,I,H], Wd_host [E,H,I]: bf16 CPU tensors (pinned here if they are not).
        g: experts per block (E need not be a multiple; the last block is shorter).
        slots: blocks the device pool can hold at once."""
        E, I, H = Wg_host.shape
        if Wu_host.shape != (E, I, H) or Wd_host.shape != (E, H, I):
            raise MoeError("ExpertResidency: weight shapes do not match")
        if g < 1 or slots < 1:
            raise MoeError("ExpertResidency: g and slots must be positive")
        self.E, self.I, self.H, self.g = E, I, H, g
        self.blocks: List[Tuple[int, int]] = [(lo, min(lo + g, E)) for lo in range(0, E, g)]
        self.slots = min(slots, len(self.blocks))
        pin = lambda t: t if t.is_pinned() else t.contiguous().pin_memory()
        self.host = (pin(Wg_host), pin(Wu_host), pin(Wd_host))
        bf = dict(dtype=torch.bfloat16, device=device)
        self.pool = (torch.empty((self.slots, g, I, H), **bf), torch.empty((self.slots, g, I, H), **bf),
                     torch.empty((self.slots, g, H, I), **bf))
        self.copy_stream = torch.cuda.Stream()
        self.slot_of: "OrderedDict[int, int]" = OrderedDict()    # resident block -> slot, least recently used first
        self.free: List[int] = list(range(self.slots))
        self.ready: Dict[int, torch.cuda.Event] = {}             # slot -> its copy has landed
        self.last_use: Dict[int, torch.cuda.Event] = {}          # slot -> the last kernels reading it are done
        self.hits = self.misses = 0
        self.bytes_copied = 0

    # ---------------------------------------------------------------- residency
    def resident_bytes(self) -> int:
        return sum(p.numel() * p.element_size() for p in self.pool)

    def block_of(self, e: int) -> int:
        return e // self.g

    def ensure(self, b: int) -> int:
        """Make block b resident; returns its slot.  The caller's stream must wait for self.ready[slot]."""
        if b in self.slot_of:
            self.hits += 1
            self.slot_of.move_to_end(b)
            return self.slot_of[b]
        self.misses += 1
        if self.free:
            slot = self.free.pop()
        else:
            _victim, slot = self.slot_of.popitem(last=False)       # least recently used
        lo, hi = self.blocks[b]
        n = hi - lo
        with torch.cuda.stream(self.copy_stream):
            if slot in self.last_use:                              # kernels still reading the evicted block
                self.copy_stream.wait_event(self.last_use[slot])
            for pool, host in zip(self.pool, self.host):
                pool[slot, :n].copy_(host[lo:hi], non_blocking=True)
                self.bytes_copied += host[lo:hi].numel() * 2
            ev = torch.cuda.Event()
            ev.record(self.copy_stream)
        self.ready[slot] = ev
        self.slot_of[b] = slot
        return slot

    # ---------------------------------------------------------------- block invocation
    def block_forward(self, b: int, tokens: torch.Tensor, src_of_row: Optional[torch.Tensor], K: int,
                      expert_offsets: torch.Tensor, Yp: torch.Tensor, workspace: torch.Tensor, policy: int = 0):
        """moe_expert_group_forward for block b on the current stream, loading the block first if needed.
        tokens is Xp when src_of_row is None, else x (rows read through src_of_row)."""
        slot = self.ensure(b)
        cur = torch.cuda.current_stream()
        cur.wait_event(self.ready[slot])
        lo, hi = self.blocks[b]
        elem = self.I * self.H * 2
        # the slot as "the full tensor": base moved back by lo experts, so that id e maps into the slot
        pg, pu, pd = (int(p[slot].data_ptr()) - lo * elem for p in self.pool)
        P = Yp.shape[0]
        lib = load()
        ws_bytes = workspace.numel() * workspace.element_size()
        if src_of_row is None:
            rc = lib.moe_expert_group_forward_ex(lo, hi, _ptr(tokens, torch.bfloat16, "Xp"),
                                                 _ptr(expert_offsets, torch.int32, "expert_offsets"), pg, pu, pd, P,
                                                 self.H, self.E, self.I, _ptr(Yp, torch.bfloat16, "Yp"),
                                                 _ptr(workspace, None, "workspace"), ws_bytes, int(policy), _stream())
        else:
            rc = lib.moe_expert_group_forward_gather(lo, hi, _ptr(tokens, torch.bfloat16, "x"),
                                                     _ptr(src_of_row, torch.int32, "src_of_row"), int(K),
                                                     _ptr(expert_offsets, torch.int32, "expert_offsets"), pg, pu, pd,
                                                     P, self.H, self.E, self.I, _ptr(Yp, torch.bfloat16, "Yp"),
                                                     _ptr(workspace, None, "workspace"), ws_bytes, int(policy),
                                                     _stream())
        _check(rc, "ExpertResidency.block_forward")
        ev = torch.cuda.Event()
        ev.record(cur)
        self.last_use[slot] = ev
        return Yp

    def forward_active_blocks(self, rows_per_expert, tokens, src_of_row, K, expert_offsets, Yp, workspace,
                              policy: int = 0) -> int:
        """Invoke every block that has rows (rows_per_expert: host-side counts, the orchestrator's
        knowledge of which blocks a batch activates).  Returns the number of blocks invoked."""
        n = 0
        for b, (lo, hi) in enumerate(self.blocks):
            if any(rows_per_expert[e] > 0 for e in range(lo, hi)):
                self.block_forward(b, tokens, src_of_row, K, expert_offsets, Yp, workspace, policy)
                n += 1
        return n
