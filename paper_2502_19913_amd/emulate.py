"""Several pipeline nodes hosted on one GPU, one HIP stream each (the way the paper's throughput runs host
several homogeneous nodes inside a single GPU, section "Throughput").

A node holds one stage (nodes of stage 0 also hold the embedding and the output head: the pipeline is a
closed loop, section "Allocating Nodes to Stages").  Every microbatch follows its path of nodes forward, has
its loss taken on its start node, and walks the path back; what a node has to do is enqueued on that node's
stream in the order of the scheduler's timeline, a backward pass before a forward pass where the two would
start together (1F1B, footnote of "Throughput Constraints"), and waits for the microbatch's previous step
through an event.  Two microbatches that meet on one node therefore queue up on its stream: a collision
costs what it costs in the paper.  Transfers between nodes are not emulated (one GPU: the residual stream
stays where it is).

Every node accumulates the gradients of its own replica; ``run`` returns their sum scaled to the mean over
microbatches, i.e. what ``sp_run_paths`` returns for the same stage paths.  All arithmetic runs in the
library's kernels; this module only orders the calls.
"""
from __future__ import annotations

from typing import Dict, List

import numpy as np

from . import binding as sp


class NodeEmulator:
    def __init__(self, cfg: dict, node_stage, n_mb: int):
        import torch
        self.torch = torch
        self.cfg = dict(cfg)
        assert cfg["has_embed"] and cfg["has_head"], "the emulated model is a whole model"
        self.node_stage = [int(s) for s in node_stage]
        self.n_mb = n_mb
        self.Nmb = cfg["seqs_per_mb"] * cfg["seq_len"]
        self.dt = sp.torch_dtype(cfg)
        full = dict(cfg, local_stage_begin=0, local_stage_count=cfg["n_stages"])
        self.n_params = sp.param_count(full)
        # where each stage's parameters start in the flat layout
        self.stage_off, self.stage_len = {}, {}
        for name, stage, layer, off, rows, cols in sp.param_layout(full):
            if stage >= 0:
                self.stage_off[stage] = min(self.stage_off.get(stage, off), off)
                self.stage_len[stage] = max(self.stage_len.get(stage, 0), off + rows * cols)
        for st in self.stage_off:
            self.stage_len[st] -= self.stage_off[st]
        self.streams, self.ctx, self.grads = [], [], []
        for st in self.node_stage:
            stream = torch.cuda.Stream()
            if st == 0:
                c = sp.Context(full, n_mb, n_mb, stream=stream)          # embedding, stage 0, head
            else:
                c = sp.Context(dict(cfg, has_embed=0, has_head=0, local_stage_begin=st, local_stage_count=1), n_mb, n_mb,
                               stream=stream)
            self.streams.append(stream); self.ctx.append(c)
            self.grads.append(torch.zeros(self.n_params, dtype=torch.float32, device="cuda"))

    def close(self):
        for c in self.ctx:
            c.close()

    def _views(self, node, params):
        st = self.node_stage[node]
        if st == 0:
            return params, self.grads[node]
        o, n = self.stage_off[st], self.stage_len[st]
        return params[o:o + n], self.grads[node][o:o + n]

    def run(self, params, tokens, targets, path_nodes: np.ndarray, lens: np.ndarray, fwd_start: np.ndarray,
            compute_fwd, compute_bwd, comm) -> Dict:
        """One iteration.  path_nodes/lens/fwd_start: the scheduler's output (fwd_start = its `arrive`).
        Returns loss, loss_mb, grads (flat float tensor), wall_ms, and per node busy_ms and n_ops."""
        torch = self.torch
        n_mb, Nmb, d = self.n_mb, self.Nmb, self.cfg["dim"]
        act = torch.empty(n_mb * Nmb * d, dtype=self.dt, device="cuda")
        dact = torch.empty_like(act)
        loss_mb = torch.zeros(n_mb, dtype=torch.float32, device="cuda")
        for g in self.grads:
            g.zero_()
        # ---- every step of every microbatch with its planned start: (start, backward?, mb, node, kind)
        ops: List[tuple] = []
        for mb in range(n_mb):
            nodes = [int(x) for x in path_nodes[mb, :lens[mb]]]
            for j, nd in enumerate(nodes):
                ops.append((float(fwd_start[mb, j]), 1, mb, nd, "embed+fwd" if j == 0 else "fwd"))
            t = float(fwd_start[mb, len(nodes) - 1]) + float(compute_fwd[nodes[-1]])
            if len(nodes) > 1:
                t += float(comm[nodes[-1], nodes[0]])
            ops.append((t, 0, mb, nodes[0], "head"))
            if len(nodes) > 1:
                t += float(comm[nodes[0], nodes[-1]])
            for j in range(len(nodes) - 1, -1, -1):
                ops.append((t, 0, mb, nodes[j], "bwd+embed" if j == 0 else "bwd"))
                t += float(compute_bwd[nodes[j]]) + (float(comm[nodes[j], nodes[j - 1]]) if j else 0.0)
        # per microbatch the planned starts increase along its chain, so this order enqueues every step after
        # the one it depends on; on a node, a backward step goes before a forward step planned for the same time
        order = sorted(range(len(ops)), key=lambda i: (ops[i][0], ops[i][1], ops[i][2]))
        chain_pos = {}
        for i in sorted(range(len(ops)), key=lambda i: (ops[i][2], i)):
            chain_pos.setdefault(ops[i][2], []).append(i)
        assert all(order.index(c[k]) < order.index(c[k + 1]) for c in chain_pos.values() for k in range(len(c) - 1))
        last_event = {}
        spans = []
        t0 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0.record()
        for s in self.streams:
            s.wait_event(t0)
        for i in order:
            _, _, mb, nd, kind = ops[i]
            stream, ctx, st = self.streams[nd], self.ctx[nd], self.node_stage[nd]
            p, g = self._views(nd, params)
            if mb in last_event:
                stream.wait_event(last_event[mb])
            with torch.cuda.stream(stream):
                e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                sl = slice(mb * Nmb * d, (mb + 1) * Nmb * d)
                if kind == "embed+fwd":
                    ctx.embed_fwd(p, tokens[mb * Nmb:(mb + 1) * Nmb], 1, act[sl])
                if kind in ("embed+fwd", "fwd"):
                    ctx.stage_fwd(st, p, act, [mb])
                elif kind == "head":
                    ctx.head_fwd_bwd(p, act[sl], targets[mb * Nmb:(mb + 1) * Nmb], 1, loss_mb[mb:mb + 1], dact[sl], g)
                else:
                    ctx.stage_bwd(st, p, dact, [mb], g)
                    if kind == "bwd+embed":
                        ctx.embed_bwd(tokens[mb * Nmb:(mb + 1) * Nmb], dact[sl], 1, g)
                e1.record(stream)
            last_event[mb] = e1
            spans.append((nd, e0, e1))
        t1 = torch.cuda.Event(enable_timing=True)
        for s in self.streams:
            torch.cuda.current_stream().wait_stream(s)
        t1.record()
        torch.cuda.synchronize()
        # every head call took its microbatch's loss alone; the iteration's loss is their mean
        total = torch.empty_like(self.grads[0])
        sp.grad_reduce(self.grads, total, 1.0 / n_mb)
        torch.cuda.synchronize()
        busy = [0.0] * len(self.node_stage); n_ops = [0] * len(self.node_stage)
        for nd, e0, e1 in spans:
            busy[nd] += e0.elapsed_time(e1); n_ops[nd] += 1
        lm = loss_mb.cpu().numpy()
        return dict(loss=float(lm.astype(np.float64).mean()), loss_mb=lm, grads=total, wall_ms=t0.elapsed_time(t1),
                    busy_ms=busy, n_ops=n_ops)
