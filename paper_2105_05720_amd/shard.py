"""Device memory of one GPU's parameter shard, laid out for the library: plumbing only, no arithmetic.

Every array kind (w, m, v fp32; w16 fp16; R gradient slices fp16) is one arena in HBM; tensor k of the list
starts at the same aligned element offset in each arena, so the tensors are scattered buffers with their own
base pointers, as a framework allocates them.  State arenas exist twice ("ping" and "pong"): a step reads one
copy and writes the other, and the caller adopts the written copy only when the overflow flag is 0.  That is
how a whole step is skipped in one pass without an undo.
"""
from __future__ import annotations

from typing import Callable, List, Optional, Sequence

import torch

from . import binding as cc
from .workloads import aligned_offsets


class Shard:
    def __init__(self, numels: Sequence[int], weight_decays: Sequence[float], R: int, device="cuda",
                 chunk_elems: int = 0, in_place: bool = False, align_elems: int = 4096, skew_elems: int = 0,
                 grad_dtype: torch.dtype = torch.float16, schedule: int = cc.CC_SCHEDULE_AUTO, workgroups: int = 0,
                 cache_policy: int = cc.CC_CACHE_AUTO, unfused: Optional[bool] = None):
        """align_elems: tensor starts are multiples of this many elements (>= 8 keeps them 16-byte aligned
        in the fp16 arenas).  The default places every tensor on a chunk boundary (4096 elements = 16 KiB of
        fp32), which measures ~5 % faster than 256-byte alignment: a chunk then covers whole DRAM interleave
        units instead of straddling them.  skew_elems shifts the whole arena start (multiple of 8).
        schedule / workgroups: passed to cc_plan_set_schedule for both plans (AUTO leaves the library's choice).
        cache_policy: passed to cc_plan_set_cache_policy.  unfused: also reserve the unfused pipelines' intermediate
        buffer (4 bytes per element and plan), which cc_unfused_* need; None reserves it for shards below 32 Mi elements."""
        assert align_elems % 8 == 0 and skew_elems % 8 == 0
        self.numels = list(numels)
        self.wds = list(weight_decays)
        self.R = R
        self.device = torch.device(device)
        self.in_place = in_place
        self.offsets, total = aligned_offsets(self.numels, align_elems)
        self.total = total
        self.skew = skew_elems
        copies = 1 if in_place else 2
        n = total + skew_elems
        f32 = lambda: torch.zeros(n, dtype=torch.float32, device=self.device)
        self.w = [f32() for _ in range(copies)]
        self.m = [f32() for _ in range(copies)]
        self.v = [f32() for _ in range(copies)]
        self.w16 = [torch.zeros(n, dtype=torch.float16, device=self.device) for _ in range(copies)]
        assert grad_dtype in (torch.float16, torch.float32)
        self.grad_dtype = grad_dtype
        gsize = 2 if grad_dtype == torch.float16 else 4
        self.grads = [torch.zeros(n, dtype=grad_dtype, device=self.device) for _ in range(R)]
        self.flag = torch.zeros(1, dtype=torch.int32, device=self.device)
        self.cur = 0
        self.plans: List[cc.Plan] = []
        for src in range(copies):
            dst = src if in_place else 1 - src
            tens = [cc.Tensor(numel=nk,
                              w_in=self._addr(self.w[src], k, 4), m_in=self._addr(self.m[src], k, 4),
                              v_in=self._addr(self.v[src], k, 4),
                              w_out=self._addr(self.w[dst], k, 4), m_out=self._addr(self.m[dst], k, 4),
                              v_out=self._addr(self.v[dst], k, 4),
                              w16_out=self._addr(self.w16[dst], k, 2),
                              grad=[self._addr(g, k, gsize) for g in self.grads],
                              weight_decay=self.wds[k])
                    for k, nk in enumerate(self.numels)]
            self.plans.append(cc.cc_plan_create_ex(tens, R, chunk_elems,
                                                   cc.CC_GRAD_F16 if grad_dtype == torch.float16 else cc.CC_GRAD_F32))
            if schedule != cc.CC_SCHEDULE_AUTO or workgroups:
                cc.cc_plan_set_schedule(self.plans[-1], schedule, workgroups)
            if cache_policy != cc.CC_CACHE_AUTO:
                cc.cc_plan_set_cache_policy(self.plans[-1], cache_policy)
        if unfused or (unfused is None and total < (32 << 20)):
            self.reserve_unfused()

    def reserve_unfused(self) -> None:
        for p in self.plans:
            cc.cc_plan_reserve_unfused(p)

    def _addr(self, arena: torch.Tensor, k: int, itemsize: int) -> int:
        return arena.data_ptr() + (self.skew + self.offsets[k]) * itemsize

    def view(self, arena: torch.Tensor, k: int) -> torch.Tensor:
        a = self.skew + self.offsets[k]
        return arena[a:a + self.numels[k]]

    # committed state (what the next step reads)
    def w_of(self, k): return self.view(self.w[self.cur], k)
    def m_of(self, k): return self.view(self.m[self.cur], k)
    def v_of(self, k): return self.view(self.v[self.cur], k)
    def w16_of(self, k): return self.view(self.w16[self.cur], k)
    def grad_of(self, r, k): return self.view(self.grads[r], k)

    @property
    def out_index(self) -> int:
        return self.cur if self.in_place else 1 - self.cur

    def run(self, step_fn: Callable, hp, stream=None) -> None:
        """Enqueue one step from the committed copy into the other one.  Does not synchronise or commit."""
        step_fn(self.plans[self.cur], hp, self.flag, stream)

    def commit(self) -> None:
        """Adopt the copy the last step wrote (call only after reading a zero flag)."""
        if not self.in_place:
            self.cur = 1 - self.cur

    def step(self, step_fn: Callable, hp, stream=None) -> int:
        """run + read the flag + commit if it is 0.  Returns the flag."""
        self.run(step_fn, hp, stream)
        flag = int(self.flag.item())
        if flag == 0 or hp.skip_mode == 1:
            self.commit()
        return flag

    def destroy(self):
        for p in self.plans:
            p.destroy()
        self.plans = []
