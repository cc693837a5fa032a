"""A seeded workload resident in HBM: inputs, per-slot packed weights, preallocated outputs.

This module is the GPU side of `synth` (the generators in `gen.py` and `configs.py` serve the CPU
oracle's tests as well and never import it).  Plumbing around the binding for the tests, the smoke check and the benchmark: it draws the
synthetic workload on the device, packs the weights into the library's layouts, owns every
buffer the four data-path calls write, and can record those calls into one graph.  All compute
happens inside the library calls.
"""
from __future__ import annotations

from typing import Dict, Iterable, List, Optional

import numpy as np
import torch

import synth
from paper_2602_21140_amd.binding import ReviveLayer, pack_expert, pack_router


class ResidentLayer:
    def __init__(self, cfg: synth.LayerConfig, device="cuda:0", with_weights=True, failed: Optional[Iterable[int]] = None,
                 replica_copies=True):
        self.cfg = cfg
        self.device = device
        self.layer = ReviveLayer(cfg, device=device)
        self.p2l = synth.make_placement(cfg)
        self.layer.set_placement(self.p2l)
        self.failed = synth.failed_mask(cfg, failed)
        self.expert_failed = None
        self.stats = self.layer.update_map(self.failed)
        self.x = synth.draw_x(cfg, device)
        self.w_router = synth.draw_router(cfg, device)        # [H, E]
        self.w_router_packed = pack_router(self.w_router)     # [E, H]
        self.sh_gate_up = self.sh_down = None
        self.gu: List[Optional[torch.Tensor]] = [None] * cfg.P
        self.dn: List[Optional[torch.Tensor]] = [None] * cfg.P
        if with_weights:
            for e in range(cfg.E):
                slots = np.nonzero(self.p2l == e)[0]
                if slots.size == 0:
                    continue
                w = synth.draw_expert(cfg, e, device)
                g, d = pack_expert(w["gate"], w["up"], w["down"])
                del w
                for i, p in enumerate(slots):   # each replica owns its own copy of the bits
                    self.gu[p] = g if (i == 0 or not replica_copies) else g.clone()
                    self.dn[p] = d if (i == 0 or not replica_copies) else d.clone()
            self.layer.set_expert_weights(self.gu, self.dn)
            sh = synth.draw_shared(cfg, device)
            if sh is not None:
                self.sh_gate_up, self.sh_down = pack_expert(sh["gate"], sh["up"], sh["down"])
        T, k, H, E, P = cfg.T, cfg.k, cfg.H, cfg.E, cfg.P
        L = self.layer
        i32, f32 = torch.int32, torch.float32
        self.buf: Dict[str, Optional[torch.Tensor]] = dict(
            logits=L.empty(T, E, dtype=f32), topk_logical=L.empty(T, k, dtype=i32),
            topk_weight=L.empty(T, k, dtype=f32), topk_phys=L.empty(T, k, dtype=i32),
            x_perm=L.empty(T * k, H), slot_offsets=L.empty(P + 1, dtype=i32), dst_row=L.empty(T * k, dtype=i32),
            src_of=L.empty(T * k, dtype=i32), y_perm=L.empty(T * k, H),
            y_shared=L.empty(T, H) if self.sh_gate_up is not None else None, out=L.empty(T, H))
        self.graph = None
        self._side = torch.cuda.Stream(device=device)
        self._ev_fork = torch.cuda.Event()
        self._ev_join = torch.cuda.Event()

    def set_failed(self, failed: Iterable[int], stream=None, expert_failed=None) -> Dict[str, int]:
        self.failed = synth.failed_mask(self.cfg, failed)
        self.expert_failed = expert_failed
        self.stats = self.layer.update_map(self.failed, stream=stream, expert_failed=expert_failed)
        return self.stats

    def forward(self, logits: Optional[torch.Tensor] = None, shared=True, stream=None,
                overlap_shared=True, stage_marks: Optional[list] = None) -> Dict[str, Optional[torch.Tensor]]:
        """route -> dispatch -> expert_ffn -> combine into the preallocated buffers (returned).

        With overlap_shared the shared expert runs on a side stream next to route/dispatch/routed
        FFN (fork and join through events, which a stream capture records as graph edges).
        stage_marks, if given, receives five timing events recorded on the main stream: before
        route, and after route, dispatch, expert_ffn and combine."""
        c, L, b = self.cfg, self.layer, self.buf
        T = c.T
        main = torch.cuda.current_stream() if stream is None else stream
        use_shared = shared and self.sh_gate_up is not None
        fork = use_shared and overlap_shared
        if fork:
            self._ev_fork.record(main)
            self._side.wait_event(self._ev_fork)
            L.shared_ffn(self.x, self.sh_gate_up, self.sh_down, T, out=b["y_shared"], stream=self._side)
            self._ev_join.record(self._side)
        def mark():
            if stage_marks is not None:
                ev = torch.cuda.Event(enable_timing=True)
                ev.record(main)
                stage_marks.append(ev)

        out3 = (b["topk_logical"], b["topk_weight"], b["topk_phys"])
        mark()
        if logits is None:
            L.route(self.x, self.w_router_packed, T, logits=b["logits"], out=out3, stream=main)
        else:
            with torch.cuda.stream(main):      # ordered before the gate on the stream the gate runs on (and recorded by a capture of it)
                b["logits"].copy_(logits)
            L.route(None, None, T, logits=b["logits"], logits_given=True, out=out3, stream=main)
        mark()
        L.dispatch(self.x, b["topk_phys"], T, out=(b["x_perm"], b["slot_offsets"], b["dst_row"], b["src_of"]), stream=main)
        mark()
        inline_shared = use_shared and not fork
        L.expert_ffn(b["x_perm"], b["slot_offsets"], T, x=self.x, w_sh_gate_up=self.sh_gate_up, w_sh_down=self.sh_down,
                     out=(b["y_perm"], b["y_shared"] if inline_shared else None), shared=inline_shared, stream=main)
        if fork:
            main.wait_event(self._ev_join)
        mark()
        L.combine(b["y_perm"], b["dst_row"], b["topk_weight"], b["y_shared"] if use_shared else None, T, out=b["out"],
                  stream=main)
        mark()
        return b

    def capture(self, stream: torch.cuda.Stream, overlap_shared=True):
        """Record one forward on `stream` into a graph (instantiated once)."""
        self.layer.graph_begin(stream)
        try:
            self.forward(stream=stream, overlap_shared=overlap_shared)
        finally:
            self.graph = self.layer.graph_end(stream)
        return self.graph

    def replay(self, stream: torch.cuda.Stream):
        self.layer.graph_launch(self.graph, stream)

    def close(self):
        self.layer.close()


class MicrobatchPipeline:
    """The layer over n microbatches of the same batch, each on its own stream (Sec. 2.2: the
    batch is divided into microbatches so that the stages of different microbatches run
    concurrently; here the route/dispatch/combine kernels of one microbatch run beside the
    expert GEMMs of the other).

    Every microbatch has its own context (map tables and workspace are per context) and its own
    intermediate buffers; weights, inputs and the output tensor are those of `base` (microbatch m
    reads rows [m*T/n, (m+1)*T/n) of x and writes the same rows of out).  Every context is told
    where its rows start in the whole batch, so a token picks the replica the undivided batch would
    pick and topk_phys of the microbatches is the single batch's, row for row."""

    def __init__(self, base: ResidentLayer, n_micro: int = 2):
        cfg = base.cfg
        if n_micro < 1 or cfg.T % n_micro:
            raise ValueError("T must be a multiple of the number of microbatches")
        self.base, self.n, self.Tm = base, n_micro, cfg.T // n_micro
        Tm, k, H, E, P = self.Tm, cfg.k, cfg.H, cfg.E, cfg.P
        i32, f32 = torch.int32, torch.float32
        self.parts = []
        for m in range(n_micro):
            L = ReviveLayer(cfg, device=base.device, T_max=Tm)
            L.set_placement(base.p2l)
            L.update_map(base.failed, expert_failed=base.expert_failed)
            L.set_expert_weights(base.gu, base.dn)
            L.set_token_offset(m * Tm)          # replicas are chosen by the token's index in the whole batch
            rows = slice(m * Tm, (m + 1) * Tm)
            buf = dict(
                x=base.x[rows], out=base.buf["out"][rows],
                logits=L.empty(Tm, E, dtype=f32), topk_logical=L.empty(Tm, k, dtype=i32),
                topk_weight=L.empty(Tm, k, dtype=f32), topk_phys=L.empty(Tm, k, dtype=i32),
                x_perm=L.empty(Tm * k, H), slot_offsets=L.empty(P + 1, dtype=i32), dst_row=L.empty(Tm * k, dtype=i32),
                src_of=L.empty(Tm * k, dtype=i32), y_perm=L.empty(Tm * k, H),
                y_shared=L.empty(Tm, H) if base.sh_gate_up is not None else None)
            self.parts.append((L, buf, torch.cuda.Stream(device=base.device), torch.cuda.Event()))
        self._fork = torch.cuda.Event()
        self.graph = None

    def set_failed(self, failed: Iterable[int], stream=None, expert_failed=None) -> Dict[str, int]:
        """The same map update for every microbatch's context (and the base layer's)."""
        stats = self.base.set_failed(failed, stream=stream, expert_failed=expert_failed)
        for L, _buf, _s, _e in self.parts:
            L.update_map(self.base.failed, stream=stream, expert_failed=expert_failed)
        return stats

    def forward(self, stream: Optional[torch.cuda.Stream] = None):
        """Fork from `stream`, run every microbatch's four calls on its own stream, join."""
        base, Tm = self.base, self.Tm
        main = torch.cuda.current_stream() if stream is None else stream
        self._fork.record(main)
        for L, b, s, done in self.parts:
            s.wait_event(self._fork)
            L.route(b["x"], base.w_router_packed, Tm, logits=b["logits"],
                    out=(b["topk_logical"], b["topk_weight"], b["topk_phys"]), stream=s)
            L.dispatch(b["x"], b["topk_phys"], Tm, out=(b["x_perm"], b["slot_offsets"], b["dst_row"], b["src_of"]), stream=s)
            shared = base.sh_gate_up is not None
            L.expert_ffn(b["x_perm"], b["slot_offsets"], Tm, x=b["x"], w_sh_gate_up=base.sh_gate_up, w_sh_down=base.sh_down,
                         out=(b["y_perm"], b["y_shared"]), shared=shared, stream=s)
            L.combine(b["y_perm"], b["dst_row"], b["topk_weight"], b["y_shared"], Tm, out=b["out"], stream=s)
            done.record(s)
        for _L, _b, _s, done in self.parts:
            main.wait_event(done)
        return base.buf["out"]

    def capture(self, stream: torch.cuda.Stream):
        """Record one forward (all microbatches, fork and join included) into one graph."""
        L0 = self.parts[0][0]
        L0.graph_begin(stream)
        try:
            self.forward(stream)
        finally:
            self.graph = L0.graph_end(stream)
        return self.graph

    def replay(self, stream: torch.cuda.Stream):
        self.parts[0][0].graph_launch(self.graph, stream)

    def close(self):
        for L, _b, _s, _e in self.parts:
            L.close()
