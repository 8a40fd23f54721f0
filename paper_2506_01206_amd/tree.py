"""Batch-wise state caches and a graph cache for tree-structured drafting (Sec. 4.1 of the paper).

For a tree configuration T = (N_1..N_gamma) the batch size at draft position i is
B_i = N_1 * ... * N_i.  ``TreeDraftCache`` asks the library for the cache layout
(``mamba_tree_plan``), allocates ONE device slab holding a conv/SSM state cache per distinct batch
size plus the parent-index arrays, and keeps one captured HIP graph per draft position (every
call there has the fixed shape (B_i, 1), which is what makes the capture possible).  It only
arranges buffers and launches: every computation is a call into the C-ABI kernels.

The per-layer work of a draft position is what the selective-SSM core does there: the conv and SSM
state rows are taken from the parent, the layer runs its conv step on the new token's features and
its selective state update, all in one launch per layer (``mamba_conv_state_step``).  What lies
between those two in a full model (the projections that produce dt, B, C) is not part of this
library, so the caller provides the per-layer token tensors in the static input buffers
``inputs[i][l]`` before a position is run.
"""
from __future__ import annotations

import torch

from . import binding as m


class TreeDraftCache:
    def __init__(self, tree, n_layers, D, N, K, io_dtype=torch.bfloat16, device="cuda:0"):
        self.tree = tuple(int(n) for n in tree)
        self.n_layers, self.D, self.N, self.K, self.io_dtype = n_layers, D, N, K, io_dtype
        self.plan = m.mamba_tree_plan(self.tree, n_layers, D, N, K, io_dtype)
        self.gamma = self.plan.gamma
        self.batch = [int(self.plan.batch[i]) for i in range(self.gamma + 1)]
        self.slab = torch.empty(max(int(self.plan.total_bytes), 16), dtype=torch.uint8, device=device)
        e = torch.empty((), dtype=io_dtype).element_size()
        self.conv, self.ssm = [], []
        for c in range(self.plan.n_caches):
            b = int(self.plan.cache_batch[c])
            co, so = int(self.plan.conv_offset[c]), int(self.plan.ssm_offset[c])
            self.conv.append(self.slab[co:co + n_layers * b * D * (K - 1) * e].view(io_dtype)
                             .view(n_layers, b, D, K - 1))
            self.ssm.append(self.slab[so:so + n_layers * b * D * N * 4].view(torch.float32)
                            .view(n_layers, b, D, N))
        self.parent = [None]
        for i in range(1, self.gamma + 1):
            po = int(self.plan.parent_offset[i])
            self.parent.append(None if po < 0 else
                               self.slab[po:po + self.batch[i] * 4].view(torch.int32))
        m.mamba_tree_parents(self.slab, self.plan, self.tree)
        # static per-position token inputs and outputs (fixed shape (B_i, 1) per layer)
        mk = lambda b, w: torch.zeros((n_layers, b, w), dtype=io_dtype, device=device)
        self.inputs = [None] + [dict(x=mk(b, D), dt=mk(b, D), z=mk(b, D), Bm=mk(b, N), Cm=mk(b, N))
                                for b in self.batch[1:]]
        self.out = [None] + [mk(b, D) for b in self.batch[1:]]
        self._xc = [None] + [torch.empty((b, 1, D), dtype=io_dtype, device=device) for b in self.batch[1:]]
        self._graphs = {}

    def cache_index(self, i):
        return int(self.plan.cache_of_depth[i])

    def set_root(self, conv_state, ssm_state):
        """States after the prefill: conv (n_layers,1,D,K-1), ssm (n_layers,1,D,N)."""
        self.conv[0].copy_(conv_state)
        self.ssm[0].copy_(ssm_state)

    def run_position(self, i, params, staged=False):
        """Eager launches for draft position i (1-based). ``params[l]`` holds A, Dskip, dt_bias,
        conv_w, conv_bias of layer l.  One launch per layer (fork of both states, conv step and state
        update); ``staged`` runs the same as conv-state fork, conv step and state step instead."""
        src, dst = self.cache_index(i - 1), self.cache_index(i)
        par = self.parent[i]
        inp = self.inputs[i]
        if not staged:
            for l in range(self.n_layers):
                p = params[l]
                m.mamba_conv_state_step(self.ssm[src][l], self.conv[src][l], inp["x"][l], p["conv_w"], p["conv_bias"],
                                        inp["dt"][l], p["A"], inp["Bm"][l], inp["Cm"][l], p["Dskip"], inp["z"][l],
                                        p["dt_bias"], parent_idx=par, h_out=self.ssm[dst][l],
                                        conv_state_out=self.conv[dst][l], out=self.out[i][l])
            return
        if par is not None:
            m.mamba_state_fork(self.conv[src], None, par, conv_dst=self.conv[dst])
        for l in range(self.n_layers):
            p = params[l]
            m.mamba_conv1d_fwd(inp["x"][l].unsqueeze(1), p["conv_w"], p["conv_bias"],
                               conv_state_in=self.conv[dst][l], y=self._xc[i],
                               conv_state_out=self.conv[dst][l])
            m.mamba_state_step(self.ssm[src][l], self._xc[i].squeeze(1), inp["dt"][l], p["A"], inp["Bm"][l],
                               inp["Cm"][l], p["Dskip"], inp["z"][l], p["dt_bias"], parent_idx=par,
                               h_out=self.ssm[dst][l], out=self.out[i][l])

    def capture(self, i, params):
        """Capture position i once; later calls replay it (graph cache)."""
        if i in self._graphs:
            return self._graphs[i]
        # a position that steps in place is not idempotent, so nothing is launched outside the capture
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                self.run_position(i, params)
        torch.cuda.current_stream().wait_stream(side)
        self._graphs[i] = g
        return g

    def draft(self, params, use_graphs=True):
        """Run positions 1..gamma on whatever the input buffers hold."""
        for i in range(1, self.gamma + 1):
            if use_graphs:
                self.capture(i, params).replay()
            else:
                self.run_position(i, params)
        return self.out[self.gamma]
