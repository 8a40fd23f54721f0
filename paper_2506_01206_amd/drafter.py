"""A whole Mamba drafter with tree-structured drafting, assembled from the C-ABI kernels.

The paper's drafter is a Mamba language model (Mamba-130M, Sec. 3.1): embedding, a stack of Mamba
blocks, a final RMSNorm and the LM head.  It encodes the prefix once and then drafts a tree
(N_1..N_gamma) as batch generation (Sec. 4.1): at position i every live branch proposes N_i children,
the children copy their parent's states and all B_i = N_1 * ... * N_i branches advance together.
Here the N_i children of a node are its N_i most probable next tokens (greedy candidates instead of
samples, so that runs are reproducible).  States live in one cache per distinct batch size
(``mamba_tree_plan``); every draft position has fixed shapes, allocates nothing and never touches
the host, so a whole draft round is captured once per tree in a HIP graph and replayed.

This module only arranges buffers and launches; every computation is a call into the library.
"""
from __future__ import annotations

import torch

from . import binding as m


class MambaDrafter:
    def __init__(self, embedding, blocks, norm_f, lm_head=None, eps=1e-5):
        """embedding (V, d_model) bf16; blocks: list of binding.Block; norm_f (d_model) f32;
        lm_head (V, d_model) bf16 (the embedding matrix when None: tied weights)."""
        self.embedding, self.blocks, self.norm_f, self.eps = embedding, list(blocks), norm_f, eps
        self.lm_head = embedding if lm_head is None else lm_head
        self.V, self.dm = embedding.shape
        b = self.blocks[0]
        self.D, self.N, self.K, self.nl = b.d_inner, b.d_state, b.d_conv, len(self.blocks)
        self.dev = embedding.device
        # the root of every draft tree: states and next-token logits after the prefix.  Allocated once, so
        # that captured draft rounds keep reading the right memory after a new prefix is encoded.
        self.root_conv = torch.empty((self.nl, 1, self.D, self.K - 1), dtype=torch.bfloat16, device=self.dev)
        self.root_ssm = torch.empty((self.nl, 1, self.D, self.N), dtype=torch.float32, device=self.dev)
        self.root_logits = torch.empty((1, self.V), dtype=torch.bfloat16, device=self.dev)
        self._trees = {}

    # ------------------------------------------------------------------ prefix encoding
    def prefill(self, tokens):
        """Encode a prefix (int32[L]); returns the logits of the next token (1, V) and keeps the
        per-layer states of the prefix as the root of later draft trees."""
        L = tokens.shape[0]
        hid = m.mamba_embedding_fwd(tokens, self.embedding).view(1, L, self.dm)
        ws = torch.empty(max(m.mamba_block_workspace_bytes(self.blocks[0], 1, L), 16), dtype=torch.uint8, device=self.dev)
        for l, blk in enumerate(self.blocks):
            m.mamba_block_fwd(blk, hid, hidden_out=hid, conv_state_out=self.root_conv[l], h_final=self.root_ssm[l],
                              workspace=ws)
        last = m.mamba_rmsnorm_fwd(hid[0, L - 1:L].contiguous(), self.norm_f, self.eps)
        m.mamba_linear_fwd(last, self.lm_head, outs=[self.root_logits])
        return self.root_logits

    # ------------------------------------------------------------------ tree drafting
    def _buffers(self, tree):
        tree = tuple(int(n) for n in tree)
        if tree in self._trees:
            return self._trees[tree]
        from .tree import TreeDraftCache
        c = TreeDraftCache(tree, self.nl, self.D, self.N, self.K, torch.bfloat16, self.dev)
        bufs = dict(cache=c, tree=tree, graph=None, pos=[None])
        for i in range(1, c.gamma + 1):
            b_i, b_prev, n_i = c.batch[i], c.batch[i - 1], tree[i - 1]
            mk = lambda shape, dt: torch.empty(shape, dtype=dt, device=self.dev)
            bufs["pos"].append(dict(
                cand=mk((b_prev, n_i), torch.int32), cand_val=mk((b_prev, n_i), torch.float32),
                hid=mk((b_i, self.dm), torch.bfloat16), normed=mk((b_i, self.dm), torch.bfloat16),
                logits=mk((b_i, self.V), torch.bfloat16),
                ws=mk((max(m.mamba_block_workspace_bytes(self.blocks[0], b_i, 1), 16),), torch.uint8)))
        self._trees[tree] = bufs
        return bufs

    def _round(self, bufs):
        c, tree = bufs["cache"], bufs["tree"]
        logits = self.root_logits
        for i in range(1, c.gamma + 1):
            p, n_i = bufs["pos"][i], tree[i - 1]
            # the N_i most probable tokens of every branch become its children: child j of branch b sits
            # in row b * N_i + j, which is the order parent[row] = row // N_i assumes
            m.mamba_topk_fwd(logits, n_i, idx=p["cand"], val=p["cand_val"])
            m.mamba_embedding_fwd(p["cand"].view(-1), self.embedding, out=p["hid"])
            src, dst = c.cache_index(i - 1), c.cache_index(i)
            for l, blk in enumerate(self.blocks):
                m.mamba_block_step(blk, p["hid"], c.conv[src][l], c.ssm[src][l], parent_idx=c.parent[i],
                                   conv_dst=c.conv[dst][l], ssm_dst=c.ssm[dst][l], hidden_out=p["hid"],
                                   workspace=p["ws"])
            m.mamba_rmsnorm_fwd(p["hid"], self.norm_f, self.eps, y=p["normed"])
            m.mamba_linear_fwd(p["normed"], self.lm_head, outs=[p["logits"]])
            logits = p["logits"]

    def draft(self, tree, use_graph=True):
        """Draft one tree from the current root.  Returns, per position, the draft tokens int32[B_i]
        (device tensors; parents are j // N_i) and the logits after the last position."""
        bufs = self._buffers(tree)
        c = bufs["cache"]
        c.set_root(self.root_conv, self.root_ssm)
        if not use_graph:
            self._round(bufs)
        else:
            if bufs["graph"] is None:
                self._round(bufs)                        # loads every kernel before the capture
                c.set_root(self.root_conv, self.root_ssm)
                g = torch.cuda.CUDAGraph()
                side = torch.cuda.Stream()
                side.wait_stream(torch.cuda.current_stream())
                with torch.cuda.stream(side):
                    with torch.cuda.graph(g, stream=side):
                        self._round(bufs)
                torch.cuda.current_stream().wait_stream(side)
                bufs["graph"] = g
            bufs["graph"].replay()
        tokens = [bufs["pos"][i]["cand"].view(-1) for i in range(1, c.gamma + 1)]
        return tokens, bufs["pos"][c.gamma]["logits"]
