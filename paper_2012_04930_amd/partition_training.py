"""The training scheme of Section 3.2 on one GPU: the graph is cut into M partitions, every partition is extended by
Algorithm 1 (Section 3.1) with a given overlap and the cut edges that the sampling did not bring in are dropped
(Section 4); each of M workers holds a full copy of the network and trains it for one full-batch epoch on its own
extended partition; at the end of every epoch the workers' parameters are replaced by their average.

Here the M workers are M models on M streams of one GPU (across GPUs the averaging is one all-reduce of the flat weight
buffer and nothing else changes).  Every step runs in the library's kernels: gcn_augment_partition, gcn_gather_rows,
gcn_graph_create, gcn_forward / gcn_loss_acc / gcn_backward / gcn_sgd_step or gcn_adam_step, gcn_average_weights.
This module only strings the calls together and keeps the books.

Run as a script for the accuracy-per-epoch comparison of two overlaps on a planted-community graph:
    python -m paper_2012_04930_amd.partition_training --parts 5 --overlaps 0 0.1 --epochs 30
"""
from __future__ import annotations

import argparse
import json

import numpy as np
import torch

from . import binding as B


class Workers:
    """M extended partitions of one graph, a model on each, a stream for each."""

    def __init__(self, rowptr, col, x, labels, train_mask, part, n_parts: int, overlap: float, dims, weights,
                 seed: int = 0, sampled_vertices_train: bool = True, dropout_p: float = 0.0):
        """rowptr, col, x, labels, train_mask, part: device tensors of the full graph (int64, int32, float32 [n x f],
        int32, uint8, int32).  sampled_vertices_train: whether the vertices that Algorithm 1 adds to a partition take
        part in that worker's loss when they are in the train mask (the extended partition is simply the worker's
        training graph) or only lend their features to their neighbours."""
        self.n_parts = n_parts
        self.graphs, self.models, self.streams, self.sizes = [], [], [], []
        for p in range(n_parts):
            v, n_local, rp, cl = B.gcn_augment_partition(rowptr, col, part, n_parts, p, overlap, seed)
            mask = train_mask[v.long()].contiguous()      # one byte per vertex: plain indexing, not a kernel of the path
            if not sampled_vertices_train:
                mask[n_local:] = 0
            g = B.gcn_graph_create(rp, cl, B.gcn_gather_rows(x, v), B.gcn_gather_rows(labels, v), mask, dims[-1])
            m = B.gcn_model_create(g, dims, dropout_p=dropout_p, seed=seed)
            B.gcn_set_weights(m, weights)
            self.graphs.append(g)
            self.models.append(m)
            self.streams.append(torch.cuda.Stream())                     # default priority
            self.sizes.append((int(v.numel()), int(n_local), int(cl.numel())))
        torch.cuda.synchronize()

    def epoch(self, lr: float, optimizer: str = "sgd", read_back: bool = True):
        """One epoch of every worker, each on its own stream, then the parameter average on the current stream.
        -> per-worker (loss, accuracy) of the epoch (before the update), or None when read_back is False."""
        main = torch.cuda.current_stream()
        for s in self.streams:
            s.wait_stream(main)
        for m, s in zip(self.models, self.streams):
            with torch.cuda.stream(s):
                B.gcn_forward(m, True)
                B.gcn_loss_acc(m, sync=False)
                B.gcn_backward(m)
        out = None
        if read_back:      # everything above is enqueued on all streams before the first wait
            out = []
            for m, s in zip(self.models, self.streams):
                with torch.cuda.stream(s):
                    out.append(B.gcn_loss_acc(m))      # waits for this worker's stream; same numbers as above
        for m, s in zip(self.models, self.streams):
            with torch.cuda.stream(s):
                if optimizer == "adam":
                    B.gcn_adam_step(m, lr)
                else:
                    B.gcn_sgd_step(m, lr)
        for s in self.streams:
            main.wait_stream(s)
        B.gcn_average_weights(self.models)
        return out

    def weights(self):
        """The (averaged) weights of worker 0, one device tensor per layer."""
        m = self.models[0]
        return [B.gcn_get_tensor(m, B.GCN_T_W, l) for l in range(1, len(m.dims))]


class Evaluator:
    """The whole graph with a mask of its own: accuracy of a set of weights on the vertices of that mask."""

    def __init__(self, rowptr, col, x, labels, mask, dims):
        self.g = B.gcn_graph_create(rowptr, col, x, labels, mask, dims[-1])
        self.m = B.gcn_model_create(self.g, dims)

    def __call__(self, weights):
        B.gcn_set_weights(self.m, torch.cat([w.reshape(-1) for w in weights]))
        B.gcn_forward(self.m, False)
        return B.gcn_loss_acc(self.m)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--n", type=int, default=20_000)
    ap.add_argument("--communities", type=int, default=40)
    ap.add_argument("--parts", type=int, default=5)
    ap.add_argument("--overlaps", type=float, nargs="+", default=[0.0, 0.1])
    ap.add_argument("--epochs", type=int, default=30)
    ap.add_argument("--optimizer", default="adam", choices=["sgd", "adam"])
    ap.add_argument("--lr", type=float, default=0.02)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--features-only", action="store_true",
                    help="sampled vertices lend their features but stay outside their worker's loss")
    args = ap.parse_args()
    from synth import workloads
    wl = workloads.planted_classes(seed=args.seed, n=args.n, n_comm=args.communities)
    dev = lambda a, t: torch.from_numpy(np.ascontiguousarray(a, dtype=t)).cuda()
    rowptr, col, x = dev(wl.rowptr, np.int64), dev(wl.col, np.int32), dev(wl.x, np.float32)
    labels, train, held = dev(wl.labels, np.int32), dev(wl.mask, np.uint8), dev(wl.extra["heldout"], np.uint8)
    # partitions = runs of whole communities, as an edge-cut partitioner returns them for such a graph
    per = -(-args.communities // args.parts) * (args.n // args.communities)
    part = dev(np.minimum(np.arange(wl.n) // per, args.parts - 1), np.int32)
    ev_held = Evaluator(rowptr, col, x, labels, held, wl.dims)
    ev_train = Evaluator(rowptr, col, x, labels, train, wl.dims)
    for overlap in args.overlaps:
        w = Workers(rowptr, col, x, labels, train, part, args.parts, overlap, wl.dims, wl.weights, seed=args.seed,
                    sampled_vertices_train=not args.features_only)
        rows = []
        for e in range(args.epochs):
            stats = w.epoch(args.lr, args.optimizer)
            agg = w.weights()
            h_loss, h_acc = ev_held(agg)
            t_loss, t_acc = ev_train(agg)
            rows.append({"epoch": e + 1, "workers_mean_loss": round(float(np.mean([s[0] for s in stats])), 4),
                         "workers_mean_acc": round(float(np.mean([s[1] for s in stats])), 4),
                         "full_graph_train_acc": round(t_acc, 4), "full_graph_heldout_acc": round(h_acc, 4),
                         "full_graph_heldout_loss": round(h_loss, 4)})
        print(json.dumps({"scheme": "Section 3.2: %d workers, parameter averaging every epoch" % args.parts,
                          "graph": wl.name, "n": wl.n, "overlap": overlap, "optimizer": args.optimizer, "lr": args.lr,
                          "sampled_vertices_train": not args.features_only,
                          "partition_sizes_vertices_local_entries": w.sizes, "epochs": rows}))
        del w
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
