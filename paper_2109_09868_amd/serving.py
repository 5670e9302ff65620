"""The serving loop of ApproxIFER (Section 2, "System Architecture") around the library's calls.

    queries -> groups of K -> encode -> N workers run the hosted model f -> wait for the fastest N - S
            -> (locate and drop A Byzantine workers) -> decode -> top-1

Every coding step is one call of the C ABI on buffers this object allocates once; nothing is allocated per
step.  What is NOT the library's belongs to the caller and comes in as arguments: the hosted model (a callable
on a [rows, D] device tensor), the workers' response times, and whatever the Byzantine workers do to their
answers.  There is no CPU path here: the binding raises if the HIP library is missing.
"""
from __future__ import annotations

import numpy as np

from . import binding


class ServingLoop:
    """Buffers and call sequence for streams of up to `max_queries` queries of D floats, C classes.

    K queries per group, N workers, the decoder waits for the fastest N - S of them and, with A > 0, drops the A
    workers Algorithm 2 locates (eq. (3) then needs N - S >= 2 (K + A)).  sign_mode as in approxifer_decode().
    """

    def __init__(self, K, N, S, A, D, C, max_queries, device, sign_mode=binding.SIGN_SURVIVOR_RANK):
        import torch
        if A > 0 and N - S < 2 * (K + A):
            raise ValueError("the Byzantine decoder needs N - S >= 2 (K + A) workers to wait for")
        if A == 0 and N - S < 1:
            raise ValueError("nobody to wait for")
        self.K, self.N, self.S, self.A, self.D, self.C = K, N, S, A, D, C
        self.sign_mode = sign_mode
        self.alpha, self.beta = binding.approxifer_chebyshev_nodes(K, N)
        G = binding.approxifer_group_count(max_queries, K)
        self.max_groups = G
        f32, dev = torch.float32, device
        self.queries = torch.zeros((G * K, D), dtype=f32, device=dev)      # the stream lands here, row by row
        self.coded = torch.empty((G, N, D), dtype=f32, device=dev)
        self.preds = torch.empty((G, N, C), dtype=f32, device=dev)
        self.mask = torch.empty((G, N), dtype=torch.uint8, device=dev)
        self.count = torch.empty((G,), dtype=torch.int32, device=dev)
        self.out = torch.empty((G, K, C), dtype=f32, device=dev)
        self.top1 = torch.empty((G, K), dtype=torch.int32, device=dev)
        self.status = torch.empty((G,), dtype=torch.int32, device=dev)
        self.adv = torch.empty((G, max(A, 1)), dtype=torch.int32, device=dev)[:, :A]
        need = binding.approxifer_workspace_bytes(G, K, N, S, A, C) if A > 0 else 0
        self.workspace = torch.empty((need,), dtype=torch.uint8, device=dev) if need else binding.NO_WORKSPACE

    def load(self, stream):
        """Copies a [Q, D] float32 stream (host or device tensor) into the query buffer; returns Q."""
        Q = int(stream.shape[0])
        if Q > self.max_groups * self.K or Q < 1:
            raise ValueError("between 1 and %d queries" % (self.max_groups * self.K))
        self.queries[:Q].copy_(stream)
        return Q

    def step(self, Q, model, arrival, tamper=None, want_values=True):
        """One pass over the Q queries in the buffer.

        model(coded [G N, D]) -> [G N, C] float32 predictions of the hosted model on every coded query;
        arrival [G, N] float32 device tensor, the workers' response times (not finite: never answers);
        tamper(preds [G, N, C]) edits the answers in place: what Byzantine workers send.
        Returns a dict of views: values [Q, C] (None unless want_values or A > 0), top1 [Q], mask [G, N],
        adv [G, A], status [G] (0: decoded), groups G.
        """
        K, N, S, A, D, C = self.K, self.N, self.S, self.A, self.D, self.C
        G = binding.approxifer_group_count(Q, K)
        groups = binding.approxifer_pad_last_group(self.queries, Q, K)            # [G, K, D] view, last group completed
        coded = binding.approxifer_encode(groups, self.alpha, self.beta, coded=self.coded[:G])
        preds = self.preds[:G]
        preds.view(G * N, C).copy_(model(coded.view(G * N, D)))
        if tamper is not None:
            tamper(preds)
        mask, count = binding.approxifer_wait_mask(arrival[:G], N - S, mask=self.mask[:G], count=self.count[:G])
        out, top1, status = self.out[:G], self.top1[:G], self.status[:G]
        adv = self.adv[:G]
        values = None
        if A > 0:
            binding.approxifer_decode_byzantine(preds, mask, self.alpha, self.beta, S, A, self.sign_mode, out=out, adv=adv,
                                                status=status, workspace=self.workspace)
            binding.approxifer_top1(out, top1=top1, want_score=False)
            values = out
        elif want_values:
            binding.approxifer_decode(preds, mask, self.alpha, self.beta, S, self.sign_mode, out=out, status=status)
            binding.approxifer_top1(out, top1=top1, want_score=False)
            values = out
        else:
            binding.approxifer_decode_top1(preds, mask, self.alpha, self.beta, S, self.sign_mode, top1=top1, status=status,
                                           want_score=False)
        return {"values": None if values is None else values.view(G * K, C)[:Q], "top1": top1.view(G * K)[:Q],
                "mask": mask, "adv": adv, "status": status, "groups": G, "coded": coded, "preds": preds}


def exponential_arrivals(G, N, seed, device, slow_fraction=0.0):
    """Response times for the loop above: unit-mean exponential draws per (group, worker), with a fraction of the
    workers never answering.  Seeded with numpy on the host so that a CPU check can draw the same times."""
    import torch
    rng = np.random.default_rng(seed)
    t = rng.exponential(1.0, (G, N)).astype(np.float32)
    if slow_fraction > 0.0:
        t[rng.random((G, N)) < slow_fraction] = np.inf
    return t, torch.from_numpy(t).to(device)
