"""Device-side harness around the binding: uploads a synthetic workload, owns the
torch-allocated input / output / workspace buffers and issues the calls of one
reshard step.  Plumbing only -- every step of the path runs in the HIP library.
"""
from __future__ import annotations

from typing import Dict, List, Optional

import numpy as np
import torch

from . import binding as B
from .workloads import Workload

_NP2TORCH = {1: torch.uint8, 2: torch.int16, 4: torch.int32}


def _as_torch_bits(a: np.ndarray) -> torch.Tensor:
    """Host tensor with the same bytes (payloads are opaque bit patterns)."""
    a = np.ascontiguousarray(a)
    return torch.from_numpy(a.view({1: np.uint8, 2: np.int16, 4: np.int32}[a.itemsize]))


class DeviceBatch:
    """One workload resident in HBM plus every buffer a reshard step writes."""

    def __init__(self, w: Workload, device: str = "cuda:0", align_tokens: Optional[int] = None,
                 cap: int = 0, poison: bool = False):
        self.w = w
        self.dev = torch.device(device)
        self._side = None
        dev = self.dev
        N, P = w.n_seq, w.n_shards
        self.align = w.align_tokens if align_tokens is None else align_tokens
        self.prm = B.make_params(N, P, w.token_budget, float(w.eps), w.ddof, cap, self.align)
        self.capacity = w.total_tokens + P * (self.align - 1)

        self.seq_len = torch.from_numpy(w.seq_len).to(dev)
        self.reward = torch.from_numpy(w.reward).to(dev)
        self.group_off = torch.from_numpy(w.group_off).to(dev)
        self.src_tok_off = torch.from_numpy(w.src_tok_off).to(dev)
        self.source = B.Source(w.src_shard_seq_off, w.src_shard_tokens, self.src_tok_off)

        # rollout-layout payload, one tensor per field and rollout shard
        self.src_fields: Dict[str, List[torch.Tensor]] = {
            f.name: [_as_torch_bits(a).to(dev) for a in f.shards] for f in w.fields}
        self.elem_bytes: Dict[str, int] = {f.name: f.elem_bytes for f in w.fields}
        self.adv_tok_src = [torch.zeros(int(t), dtype=torch.float32, device=dev) for t in w.src_shard_tokens]
        self.elem_bytes["adv_tok"] = 4

        # outputs
        self.status = torch.zeros(1, dtype=torch.int32, device=dev)
        self.perm = torch.zeros(N, dtype=torch.int32, device=dev)
        self.shard_seq_off = torch.zeros(P + 1, dtype=torch.int32, device=dev)
        self.shard_of_seq = torch.zeros(N, dtype=torch.int32, device=dev)
        self.shard_load = torch.zeros(P, dtype=torch.int64, device=dev)
        self.adv_seq = torch.zeros(N, dtype=torch.float32, device=dev)
        self.dst_tok_off = torch.zeros(N + 1, dtype=torch.int64, device=dev)
        self.shard_tok_off = torch.zeros(P + 1, dtype=torch.int64, device=dev)
        self.shard_mb_off = torch.zeros(P + 1, dtype=torch.int32, device=dev)
        self.mb_seq_off = torch.zeros(N + 1, dtype=torch.int32, device=dev)
        self.cu_seqlens = torch.zeros(2 * N + 1, dtype=torch.int32, device=dev)
        self.n_mb = torch.zeros(1, dtype=torch.int32, device=dev)
        self.ws_bytes = B.dc_workspace_bytes(self.prm, self.capacity)
        self.ws = torch.zeros(self.ws_bytes, dtype=torch.uint8, device=dev)
        # more sequences than dc_balance takes: dc_balance_ws and its workspace
        self.large = N > B.DC_MAX_SEQ
        self.bal_ws_bytes = B.dc_balance_workspace_bytes(self.prm)
        self.bal_ws = torch.zeros(self.bal_ws_bytes, dtype=torch.uint8, device=dev) if self.bal_ws_bytes else None

        self.dst_fields: Dict[str, torch.Tensor] = {}
        for name, eb in self.elem_bytes.items():
            t = torch.zeros(self.capacity, dtype=_NP2TORCH[eb], device=dev)
            if poison:
                t.fill_({1: 0x5A, 2: 0x5A5A, 4: 0x5A5A5A5A}[eb])
            self.dst_fields[name] = t
        names = list(self.elem_bytes.keys())
        self.field_names = names
        self.fields = B.Fields([
            (self.adv_tok_src if n == "adv_tok" else self.src_fields[n], self.dst_fields[n], self.elem_bytes[n])
            for n in names])
        self.payload_bytes_per_token = sum(self.elem_bytes.values())
        # the same without adv_tok: dc_gather_advantage makes that arena from the mask and adv_seq
        self.moved_names = [n for n in names if n != "adv_tok"]
        self.moved_fields = B.Fields([(self.src_fields[n], self.dst_fields[n], self.elem_bytes[n])
                                      for n in self.moved_names])

    # ---- the calls of one step ----
    def group_advantage(self, per_token: bool = True, stream=None) -> None:
        B.dc_group_advantage(self.prm, self.source, self.seq_len, self.reward, self.group_off, self.w.n_groups,
                             self.src_fields["mask"] if per_token else None, self.adv_seq,
                             self.adv_tok_src if per_token else None, self.status, stream)

    def balance(self) -> None:
        if self.large:
            B.dc_balance_ws(self.prm, self.seq_len, self.perm, self.shard_seq_off, self.shard_of_seq,
                            self.shard_load, self.bal_ws, self.bal_ws_bytes, self.status)
            return
        B.dc_balance(self.prm, self.seq_len, self.perm, self.shard_seq_off, self.shard_of_seq,
                     self.shard_load, self.status)

    def plan(self) -> None:
        B.dc_plan(self.prm, self.source, self.seq_len, self.perm, self.shard_seq_off, self.capacity,
                  self.dst_tok_off, self.shard_tok_off, self.shard_mb_off, self.mb_seq_off, self.cu_seqlens,
                  self.n_mb, self.ws, self.ws_bytes, self.status)

    def gather(self, dispatch_events=None) -> None:
        """dispatch_events: optional (begins, ends) torch events, each recorded once before, that the gather kernel's
        dispatch updates with its own start and end times (dc_gather_timed)."""
        if dispatch_events is not None:
            B.dc_gather_timed(self.prm, self.source, self.fields, self.capacity, self.dst_tok_off, self.ws,
                              self.ws_bytes, self.status, dispatch_events[0], dispatch_events[1])
            return
        B.dc_gather(self.prm, self.source, self.fields, self.capacity, self.dst_tok_off, self.ws,
                    self.ws_bytes, self.status)

    def gather_advantage(self) -> None:
        """dc_gather of every field but adv_tok; the adv_tok arena is made from the mask and adv_seq."""
        B.dc_gather_advantage(self.prm, self.source, self.moved_fields, self.moved_names.index("mask"), self.perm,
                              self.adv_seq, self.dst_fields["adv_tok"].view(torch.float32), self.capacity,
                              self.dst_tok_off, self.ws, self.ws_bytes, self.status)

    def repack(self) -> None:
        B.dc_repack(self.prm, self.source, self.seq_len, self.perm, self.shard_seq_off, self.fields,
                    self.capacity, self.dst_tok_off, self.shard_tok_off, self.shard_mb_off, self.mb_seq_off,
                    self.cu_seqlens, self.n_mb, self.ws, self.ws_bytes, self.status)

    def repack_noalloc(self) -> None:
        """dc_repack planning in the library's own device array (no workspace argument)."""
        B.dc_repack_noalloc(self.prm, self.source, self.seq_len, self.perm, self.shard_seq_off, self.fields,
                            self.capacity, self.dst_tok_off, self.shard_tok_off, self.shard_mb_off, self.mb_seq_off,
                            self.cu_seqlens, self.n_mb, self.status)

    def step(self) -> None:
        """One pass of the whole path: advantage, balance, plan, gather."""
        self.group_advantage()
        self.balance()
        self.plan()
        self.gather()

    def balance_group_advantage(self, per_token: bool = True) -> None:
        if self.large:                                   # the one-launch form keeps dc_balance's size limit
            self.group_advantage(per_token)
            self.balance()
            return
        B.dc_balance_group_advantage(self.prm, self.source, self.seq_len, self.perm, self.shard_seq_off,
                                     self.shard_of_seq, self.shard_load, self.reward, self.group_off, self.w.n_groups,
                                     self.src_fields["mask"] if per_token else None, self.adv_seq,
                                     self.adv_tok_src if per_token else None, self.status)

    def balance_plan_group_advantage(self, per_token: bool = True) -> None:
        if self.large:                                   # the call keeps dc_balance's size limit
            self.group_advantage(per_token)
            self.balance()
            self.plan()
            return
        B.dc_balance_plan_group_advantage(self.prm, self.source, self.seq_len, self.perm, self.shard_seq_off,
                                          self.shard_of_seq, self.shard_load, self.reward, self.group_off,
                                          self.w.n_groups, self.src_fields["mask"] if per_token else None, self.adv_seq,
                                          self.adv_tok_src if per_token else None, self.capacity, self.dst_tok_off,
                                          self.shard_tok_off, self.shard_mb_off, self.mb_seq_off, self.cu_seqlens,
                                          self.n_mb, self.ws, self.ws_bytes, self.status)

    def step_two_calls(self, gather_events=None, per_token: bool = True, dispatch_events=None) -> None:
        """The whole pass as two calls: dc_balance_plan_group_advantage (balance, advantage stage and plan: two
        launches where the shape allows it), then the gather.  gather_events: optional (start, end) torch events
        recorded around the gather launch; dispatch_events: optional (begins, ends) events carried by the gather
        kernel's dispatch itself (see gather)."""
        self.balance_plan_group_advantage(per_token)
        if gather_events is not None:
            gather_events[0].record()
        if per_token:
            self.gather(dispatch_events)
        else:
            self.gather_advantage()
        if gather_events is not None:
            gather_events[1].record()

    def step_fused(self, gather_events=None) -> None:
        """The same pass on ONE stream: balance and the advantage stage share a launch (the advantage
        workgroups stream the tokens while the balance workgroup runs), then plan, then gather.
        gather_events: optional (start, end) torch events recorded around the gather launch."""
        self.balance_group_advantage()
        self.plan()
        if gather_events is not None:
            gather_events[0].record()
        self.gather()
        if gather_events is not None:
            gather_events[1].record()

    def step_no_rollout_adv(self, gather_events=None) -> None:
        """The pass without the rollout-layout copy of the per-token advantages: the fused launch
        computes the per-sequence advantages only, the gather makes the per-token field."""
        self.balance_group_advantage(per_token=False)
        self.plan()
        if gather_events is not None:
            gather_events[0].record()
        self.gather_advantage()
        if gather_events is not None:
            gather_events[1].record()

    def step_overlapped(self, gather_events=None) -> None:
        """The same pass with the two independent halves on two HIP streams: the advantage
        kernel (bandwidth-bound, whole chip) runs beside balance + plan (latency-bound, one
        workgroup each); the gather waits for both.  Streams have the default priority.
        gather_events: optional (start, end) torch events recorded around the gather launch."""
        main = torch.cuda.current_stream(self.dev)
        if self._side is None:
            self._side = torch.cuda.Stream(device=self.dev)
            self._ev_in = torch.cuda.Event()
            self._ev_adv = torch.cuda.Event()
        self._ev_in.record(main)                           # inputs (and the previous step) are ordered before both halves
        self._side.wait_event(self._ev_in)
        self.group_advantage(stream=self._side)
        self._ev_adv.record(self._side)
        self.balance()
        self.plan()
        main.wait_event(self._ev_adv)
        if gather_events is not None:
            gather_events[0].record(main)
        self.gather()
        if gather_events is not None:
            gather_events[1].record(main)

    def prepare_scatter(self, names: Optional[List[str]] = None, fill: int = 0x5A) -> None:
        """Rollout-layout buffers to scatter the named training-layout fields back into."""
        names = self.field_names if names is None else names
        self.back_names = names
        self.back_fields: Dict[str, List[torch.Tensor]] = {}
        for n in names:
            eb = self.elem_bytes[n]
            pat = {1: fill, 2: fill * 0x0101, 4: fill * 0x01010101}[eb]
            self.back_fields[n] = [torch.full((int(t),), pat, dtype=_NP2TORCH[eb], device=self.dev)
                                   for t in self.w.src_shard_tokens]
        self.back = B.Fields([(self.back_fields[n], self.dst_fields[n], self.elem_bytes[n]) for n in names])
        self.sws_bytes = B.dc_scatter_workspace_bytes(self.prm, self.source)
        self.sws = torch.zeros(self.sws_bytes, dtype=torch.uint8, device=self.dev)

    def release_scatter(self) -> None:
        """Drop the buffers prepare_scatter made."""
        self.back_fields = {}
        self.back = None
        self.sws = None

    def scatter(self) -> None:
        """Reverse path: training arenas -> rollout buffers (after plan / gather of the same step)."""
        B.dc_scatter(self.prm, self.source, self.seq_len, self.perm, self.back, self.capacity, self.dst_tok_off,
                     self.sws, self.sws_bytes, self.status)

    def prepare_gae(self) -> None:
        """Rollout-layout outputs of the PPO advantage stage (needs float32 value and, with the KL
        penalty, old_logprob / ref_logprob fields)."""
        self.gae_adv = [torch.full((int(t),), float("nan"), dtype=torch.float32, device=self.dev)
                        for t in self.w.src_shard_tokens]
        self.gae_ret = [torch.full((int(t),), float("nan"), dtype=torch.float32, device=self.dev)
                        for t in self.w.src_shard_tokens]

    def gae(self, gamma: float = 1.0, lam: float = 0.95, kl_coef: float = 0.0, stream=None) -> None:
        as_f32 = lambda ts: [t.view(torch.float32) for t in ts]
        B.dc_gae(self.prm, self.source, self.seq_len, self.reward, as_f32(self.src_fields["value"]),
                 self.src_fields["mask"],
                 as_f32(self.src_fields["old_logprob"]) if kl_coef != 0.0 else None,
                 as_f32(self.src_fields["ref_logprob"]) if kl_coef != 0.0 else None,
                 gamma, lam, kl_coef, self.gae_adv, self.gae_ret, self.status, stream)

    def read_status(self) -> int:
        return int(self.status.item())
