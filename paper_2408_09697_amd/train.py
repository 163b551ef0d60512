"""One mini-batch training step with every stage on the device, as a sequence of library calls.

Algorithm 1 of the paper, one worker's share for one iteration: sample the k-hop neighbourhood of
the mini-batch (Section 2.2), run the relation-aggregation-first layers forward over the sampled
blocks (Eq. 1 per layer, ReLU between layers), take the loss gradient on the seeds from the caller,
run the local backward through every layer, and update the parameters: the per-relation weights
and - only on the rows the mini-batch touched - the learnable feature vectors of featureless
node types with their Adam moments (Sections 2.2 and 6).  This module allocates buffers and
orders calls; all arithmetic is in libheta.
"""
from __future__ import annotations

from typing import Callable, Dict, List, Optional, Sequence

import torch

from . import binding as hb
from . import sampler as hs
from .layer import RafLayer


class MiniBatchTrainer:
    """A k-layer R-GCN-style model over a device-resident heterogeneous graph.

    base      : the whole graph (binding.Graph); its node types say which tables are learnable
    tables[t] : device [N_t, d_t] feature / embedding tables (fp32 or bf16), updated in place when learnable
    W[l][r]   : device [d_in(l, r), d_hidden] weights of layer l (0 = outermost), updated in place
    fanouts   : outermost hop first, e.g. [25, 20]
    """

    def __init__(self, base: hb.Graph, tables: Sequence[torch.Tensor], W: Sequence[Sequence[torch.Tensor]],
                 fanouts: Sequence[int], d_hidden: int, op: int, seed_type: int, lr: float = 1e-3,
                 beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8, seed: int = 0):
        if len(W) != len(fanouts):
            raise ValueError("one weight list per layer")
        self.base, self.tables, self.W = base, list(tables), [list(w) for w in W]
        self.fanouts, self.d_hidden, self.op, self.seed_type = list(fanouts), d_hidden, op, seed_type
        self.lr, self.beta1, self.beta2, self.eps, self.seed = lr, beta1, beta2, eps, seed
        self.T = len(base.ntypes)
        f32 = torch.float32
        self.learnable = [t for t in range(self.T) if base.ntypes[t][2]]
        # Adam moments: one pair per weight matrix, one pair per learnable table (fp32, the table's shape)
        self.mW = [[torch.zeros(w.shape, dtype=f32, device=w.device) for w in ws] for ws in self.W]
        self.vW = [[torch.zeros(w.shape, dtype=f32, device=w.device) for w in ws] for ws in self.W]
        self.mT = {t: torch.zeros(self.tables[t].shape, dtype=f32, device=self.tables[t].device) for t in self.learnable}
        self.vT = {t: torch.zeros(self.tables[t].shape, dtype=f32, device=self.tables[t].device) for t in self.learnable}
        self.t = 0
        self.last_blocks: Optional[List[hs.DeviceBlock]] = None
        self.last_layers: Optional[List[RafLayer]] = None

    def _layers(self, blocks: List[hs.DeviceBlock]) -> List[RafLayer]:
        T = self.T
        layers: List[RafLayer] = []
        prev: Optional[Dict[int, torch.Tensor]] = None
        for l, b in enumerate(blocks):
            rels = [i for i in range(len(b.graph.rels)) if b.graph.n_dst(i) > 0]
            if l == 0:
                tabs: List[Optional[torch.Tensor]] = list(self.tables) + [None] * T
                gid: Optional[List[Optional[torch.Tensor]]] = list(b.src_ids) + [None] * T
            else:
                tabs = [prev.get(T + k) for k in range(T)] + [None] * T
                gid = None
            for i in rels:  # a source type nobody sampled still needs a (dummy) table of the right width
                s = b.graph.rels[i][0]
                if tabs[s] is None:
                    tabs[s] = torch.zeros((1, self.W[l][i].shape[0]), dtype=torch.float32, device=self.W[l][i].device)
            layer = RafLayer(b.graph, self.op, tabs, self.W[l], self.d_hidden, src_gid=gid,
                             relu=(l < len(blocks) - 1), rels=rels)
            prev = layer.forward()  # on torch's current stream, like every buffer the layer allocated
            layers.append(layer)
        return layers

    def step(self, seeds: torch.Tensor, loss_grad: Callable[[torch.Tensor], torch.Tensor], stream=None,
             keep_blocks: bool = False) -> torch.Tensor:
        """One iteration on the mini-batch `seeds` (device int64, distinct).  `loss_grad(H)` returns dL/dH
        for the seeds' embeddings H [n_seeds, d_hidden] (fp32).  Returns H.

        The whole iteration - sampling, the buffers torch allocates for it, forward, backward, updates and
        `loss_grad` - runs on ONE stream: torch's current stream, or `stream` (a torch stream or a raw
        hipStream_t), which is made the current stream for the duration of the call.  The caller orders that
        stream against whatever produced `seeds` and the tables."""
        if stream is not None:
            ts = stream if isinstance(stream, torch.cuda.Stream) else torch.cuda.ExternalStream(int(stream))
            with torch.cuda.stream(ts):
                return self._step(seeds, loss_grad, keep_blocks)
        return self._step(seeds, loss_grad, keep_blocks)

    def _step(self, seeds: torch.Tensor, loss_grad: Callable[[torch.Tensor], torch.Tensor], keep_blocks: bool) -> torch.Tensor:
        stream = None  # every library call below takes torch's current stream
        self.t += 1
        T = self.T
        blocks = hs.sample_blocks(self.base, self.seed_type, seeds, self.fanouts, self.seed + self.t, stream=stream)
        layers = self._layers(blocks)
        H = layers[-1].H[T + self.seed_type]
        G: Dict[int, torch.Tensor] = {T + self.seed_type: loss_grad(H)}
        for l in reversed(range(len(layers))):
            _, dH0, _ = layers[l].backward(G, stream=stream)
            if l > 0:
                G = {T + s: g for s, g in dH0.items() if (T + s) in layers[l - 1].H}
                for t, h in layers[l - 1].H.items():  # destination types of the layer below that got no gradient
                    if t not in G:
                        G[t] = torch.zeros_like(h)
        # parameter update: dense Adam on the weights, sparse Adam on the touched rows of learnable tables
        # (every update of the iteration in one call: up to 16 tables share a launch)
        updates = [(self.W[l][r], self.mW[l][r], self.vW[l][r], layer.dW[r], None) for l, layer in enumerate(layers) for r in layer.rels]
        first = layers[0]
        for t in self.learnable:
            if t in first.dH0 and blocks[0].src_ids[t].numel() > 0:
                updates.append((self.tables[t], self.mT[t], self.vT[t], first.dH0[t], blocks[0].src_ids[t]))
        hb.heta_sparse_adam_multi(updates, lr=self.lr, beta1=self.beta1, beta2=self.beta2, eps=self.eps, step=self.t, stream=stream)
        if keep_blocks:
            self.last_blocks, self.last_layers = blocks, layers
        else:
            for b in blocks:
                b.graph.destroy()
        return H
