"""Run one library call on one synthetic workload shape a few times (for profilers).

    python3 -m paper_2109_09868_amd.run_workload --workload text_k32 --op encode --reps 5
    rocprofv3 --kernel-trace --stats -- python3 -m paper_2109_09868_amd.run_workload --workload byzantine --op decode_byzantine
    python3 -m paper_2109_09868_amd.run_workload --shape 2048,16,24,6,0,4096,4096 --op decode      # G,K,N,S,A,D,C

Inputs are drawn on the device with torch (values do not matter to a profile; shapes, masks and
launch configuration are those of the named workload).
"""
from __future__ import annotations

import argparse

import numpy as np


def main():
    import torch

    from . import binding, synthetic as syn

    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="imagenet", choices=sorted(syn.WORKLOADS))
    ap.add_argument("--op", default="encode", choices=["encode", "decode", "decode_top1", "decode_byzantine",
                                                         "decode_byzantine_homogeneous", "decode_rational"])
    ap.add_argument("--shape", default=None,
                    help="G,K,N,S,A,D,C: these sizes instead of the named workload's (its seeds and mask recipe stay)")
    ap.add_argument("--no-workspace", action="store_true", help="Byzantine ops: pass no workspace")
    ap.add_argument("--linear-model", action="store_true",
                    help="Byzantine ops: predictions = a linear map of the coded queries plus noise on A workers "
                         "(exactly rational data, the case the locators are built for) instead of plain noise")
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--sign-mode", type=int, default=0)
    args = ap.parse_args()

    w = syn.WORKLOADS[args.workload]
    if args.shape:
        G, K, N, S, A, D, C = (int(x) for x in args.shape.split(","))
        w = syn.scaled(w, name="%s[%s]" % (w.name, args.shape), G=G, K=K, W=N, S=S, A=A, query_shape=(D,), C=C)
    dev = torch.device("cuda:0")
    alpha, beta = binding.approxifer_chebyshev_nodes(w.K, w.W)
    gen = torch.Generator(device=dev).manual_seed(syn.BASE_SEED + w.index)
    if args.op == "encode":
        q = torch.rand((w.G, w.K, w.D), dtype=torch.float32, device=dev, generator=gen)
        coded = torch.empty((w.G, w.W, w.D), dtype=torch.float32, device=dev)
        fn = lambda: binding.approxifer_encode(q, alpha, beta, coded=coded)
    else:
        mask_h = syn.masks(w)
        mask = torch.from_numpy(mask_h).to(dev)
        preds = torch.randn((w.G, w.W, w.C), dtype=torch.float32, device=dev, generator=gen)
        out = torch.empty((w.G, w.K, w.C), dtype=torch.float32, device=dev)
        st = torch.empty((w.G,), dtype=torch.int32, device=dev)
        if args.op == "decode":
            fn = lambda: binding.approxifer_decode(preds, mask, alpha, beta, w.S, args.sign_mode, out=out, status=st)
        elif args.op == "decode_top1":
            top1 = torch.empty((w.G, w.K), dtype=torch.int32, device=dev)
            fn = lambda: binding.approxifer_decode_top1(preds, mask, alpha, beta, w.S, args.sign_mode, top1=top1,
                                                        status=st, want_score=False)
        else:
            if w.A < 1:
                raise SystemExit("workload %s has no adversaries" % w.name)
            if args.linear_model:
                q = torch.rand((w.G, w.K, w.D), dtype=torch.float32, device=dev, generator=gen)
                lin = torch.randn((w.D, w.C), dtype=torch.float32, device=dev, generator=gen) / w.D ** 0.5
                preds = (binding.approxifer_encode(q, alpha, beta).reshape(-1, w.D) @ lin).reshape(w.G, w.W, w.C)
                bad = torch.from_numpy(syn.adversaries(w, mask_h)).to(dev).long()           # [G, A]
                noise = 10 * preds.std() * torch.randn((w.G, w.A, w.C), dtype=torch.float32, device=dev, generator=gen)
                preds = preds.scatter_add(1, bad[:, :, None].expand(-1, -1, w.C), noise).contiguous()
            adv = torch.empty((w.G, w.A), dtype=torch.int32, device=dev)
            if args.op == "decode_rational":
                fn = lambda: binding.approxifer_decode_rational(preds, mask, alpha, beta, w.S, w.A, out=out, status=st)
            else:
                need = 0 if args.no_workspace else binding.approxifer_workspace_bytes(w.G, w.K, w.W, w.S, w.A, w.C)
                ws = torch.empty((need,), dtype=torch.uint8, device=dev) if need else binding.NO_WORKSPACE
                entry = (binding.approxifer_decode_byzantine if args.op == "decode_byzantine"
                         else binding.approxifer_decode_byzantine_homogeneous)
                fn = lambda: entry(preds, mask, alpha, beta, w.S, w.A, args.sign_mode, out=out, adv=adv, status=st,
                                   workspace=ws)
    for _ in range(args.reps):
        fn()
    torch.cuda.synchronize()
    print("%s %s x%d done" % (w.name, args.op, args.reps))


if __name__ == "__main__":
    main()
