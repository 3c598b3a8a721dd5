"""Training schedules built on ff_train_step: host loops only, every arithmetic step runs in the library.

* look-ahead schedule (Section IV-C, Algorithm 1; Section V-A): all layers are updated in every
  iteration from one forward pass, the look-ahead weight lambda starts at `lam0` and grows by `dlam`
  after every epoch (the paper uses 0 and 0.001).
* greedy schedule (Section III, the vanilla Forward-Forward procedure): layer 1 is trained for its
  epochs, then frozen; layer 2 is trained on layer 1's outputs; and so on.  Expressed with
  ff_net_desc.train_layer on the prefix stack [0..i], lambda = 0.

A "batch" is a pair of device tensors (x_pos, x_neg), fp32, [batch, features] (conv: NHWC flattened).
The step counter that keys the stochastic-rounding streams increases by one per iteration over the
whole run, so that a schedule is reproducible from (seed, step0).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import torch

from . import binding as ff


@dataclass
class TrainState:
    """Device tensors of a layer stack: fp32 master weights and their int8 working copies."""
    layers: Sequence
    batch: int
    w_master: List[torch.Tensor]
    w_q: List[torch.Tensor]
    s_w: List[torch.Tensor]

    @staticmethod
    def from_weights(layers: Sequence, batch: int, weights) -> "TrainState":
        w_master = [torch.as_tensor(w).reshape(w.shape[0], -1).to(device="cuda", dtype=torch.float32).contiguous()
                    for w in weights]
        w_q = [torch.zeros((l.N, ff.ff_pitch(l.K)), dtype=torch.int8, device="cuda") for l in layers]
        s_w = [torch.zeros(1, device="cuda") for _ in layers]
        ws = torch.empty(ff.WS_MIN_BYTES, dtype=torch.uint8, device="cuda")
        for i, l in enumerate(layers):
            ff.ff_quantize(w_master[i], l.N, l.K, ff.ROUND_NEAREST, 0, 0, w_q[i], None, s_w[i], ws)
        return TrainState(layers, batch, w_master, w_q, s_w)

    def net(self, n_layers: Optional[int] = None, train_layer: Optional[Sequence[int]] = None,
            lookahead: str = "coeff") -> ff.Net:
        k = len(self.layers) if n_layers is None else n_layers
        return ff.Net(self.layers[:k], self.batch, self.w_master[:k], self.w_q[:k], self.s_w[:k], train_layer, lookahead)


@dataclass
class History:
    """One record per logged iteration: (step, lambda, loss [k][2], mean goodness [k][2])."""
    step: List[int] = field(default_factory=list)
    lam: List[float] = field(default_factory=list)
    loss: List[List[List[float]]] = field(default_factory=list)
    goodness_mean: List[List[List[float]]] = field(default_factory=list)

    def separation(self, layer: int) -> List[float]:
        """mean goodness of the positive set minus that of the negative set, per logged iteration"""
        return [g[layer][0] - g[layer][1] for g in self.goodness_mean if layer < len(g)]


def _run(net: ff.Net, batches, n_iter_epochs: int, theta: float, lr: float, seed: int, step: int,
         lam0: float, dlam: float, hist: History, log_every: int, use_graph: bool = False) -> int:
    k, B = net.k, net.batch
    ws = torch.empty(net.workspace_bytes(), dtype=torch.uint8, device="cuda")
    loss = torch.empty((k, 2), device="cuda")
    good = torch.empty((k, 2, B), device="cuda")
    lam = lam0
    if use_graph and batches:
        # One captured step per epoch (lambda is a launch argument), replayed for every batch of the epoch: the batch is
        # copied into fixed input buffers and the step number lives in device memory (ff_train_step_at), so that
        # launch latency, which dominates small networks, is paid once per epoch.
        x_pos_s = torch.empty_like(batches[0][0])
        x_neg_s = torch.empty_like(batches[0][1])
        step_dev = torch.tensor([step], dtype=torch.int64, device="cuda")
    for _ in range(n_iter_epochs):
        graph = None
        if use_graph and batches:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                with torch.cuda.graph(graph, stream=side):
                    ff.ff_train_step_at(net, x_pos_s, x_neg_s, theta, lam, lr, seed, step_dev, 1, loss, good, ws)
            torch.cuda.current_stream().wait_stream(side)
        for (x_pos, x_neg) in batches:
            if graph is not None:
                x_pos_s.copy_(x_pos)
                x_neg_s.copy_(x_neg)
                graph.replay()
            else:
                ff.ff_train_step(net, x_pos, x_neg, theta, lam, lr, seed, step, loss, good, ws)
            if log_every and step % log_every == 0:
                hist.step.append(step)
                hist.lam.append(lam)
                hist.loss.append(loss.cpu().tolist())
                hist.goodness_mean.append(good.mean(dim=2).cpu().tolist())
            step += 1
        lam += dlam
    return step


def train_lookahead(state: TrainState, batches: Sequence[Tuple[torch.Tensor, torch.Tensor]], epochs: int,
                    theta: float, lr: float, seed: int, lam0: float = 0.0, dlam: float = 0.001, step0: int = 0,
                    log_every: int = 1, lookahead: str = "coeff", use_graph: bool = False) -> History:
    """Algorithm 1 for `epochs` passes over `batches`; lambda = lam0 + epoch * dlam (Section V-A).
    lookahead = "chain": Eq. (4) as an exact derivative through the later layers (dense stacks only).
    use_graph: replay one captured HIP graph per epoch instead of launching every step eagerly (same results)."""
    hist = History()
    _run(state.net(lookahead=lookahead), batches, epochs, theta, lr, seed, step0, lam0, dlam, hist, log_every, use_graph)
    return hist


def train_greedy(state: TrainState, batches: Sequence[Tuple[torch.Tensor, torch.Tensor]], epochs_per_layer: int,
                 theta: float, lr: float, seed: int, step0: int = 0, log_every: int = 1) -> History:
    """Section III: train layer i for `epochs_per_layer` epochs with layers < i frozen, for i = 0, 1, ..."""
    hist = History()
    step = step0
    for i in range(len(state.layers)):
        net = state.net(i + 1, [0] * i + [1])
        step = _run(net, batches, epochs_per_layer, theta, lr, seed, step, 0.0, 0.0, hist, log_every)
    return hist
