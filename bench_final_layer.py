#!/usr/bin/env python3
"""Final-layer step of a SASRec-shaped model: cce_neg_loss against a cross-entropy with negative sampling that
materialises its logits in plain PyTorch, on the same GPU (time per forward + backward and peak extra memory).

    python bench_final_layer.py [--reps 10]

The paper compares CE- (logits [positions x (1 + ns)] materialised by PyTorch) with CCE- (its fused kernels) by memory
and time per epoch of whole training runs (Sec. 5.2, the CE / CE- against CCE / CCE- table).  The datasets and the
model are not reproduced here; what is measured is the part the two differ in: the loss over the final-layer output
H [bs * sl, d] and the item table E [V, d] with ns shared uniform negatives, at (bs, sl, ns, V) combinations of the
size class of that table's rows, d = 256, bf16, random values.  One JSON line per shape.
"""
from __future__ import annotations

import argparse
import json
import sys
import os

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

SHAPES = [   # name, batch, sequence length, negatives, catalogue size
    ("bs256_sl512_ns1511_V15k", 256, 512, 1511, 15_000),
    ("bs1024_sl32_ns511_V12k", 1024, 32, 511, 12_000),
    ("bs1024_sl320_ns511_V310k", 1024, 320, 511, 310_000),
    ("bs128_sl200_ns4095_V1M", 128, 200, 4095, 1_000_000),
]


def materialised_ce_minus(H, E, tgt, neg, mask):
    """Reference formulation in plain PyTorch: logits of the correct item and of the shared negatives are written out,
    collisions with the position's own target are masked, log-softmax picks column 0, mean over valid positions."""
    import torch

    pos = (H * E[tgt.long()]).sum(-1, dtype=torch.float32)
    logits = (H @ E[neg.long()].T).float()                                # [N, ns]
    logits = logits.masked_fill(neg[None, :] == tgt[:, None], float("-inf"))
    full = torch.cat([pos[:, None], logits], 1)                            # [N, 1 + ns]
    per_pos = torch.logsumexp(full, 1) - pos
    m = mask.to(torch.float32)
    return (per_pos * m).sum() / m.sum().clamp_min(1.0)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--reps", type=int, default=10)
    ap.add_argument("--d", type=int, default=256)
    args = ap.parse_args()
    import torch

    if not torch.cuda.is_available():
        print("bench_final_layer.py needs a GPU", file=sys.stderr)
        return 2
    import paper_2509_09682_amd as P

    for name, bs, sl, ns, V in SHAPES:
        N, d = bs * sl, args.d
        g = torch.Generator(device="cuda").manual_seed(7)
        Hd = torch.randn(N, d, device="cuda", generator=g).to(torch.bfloat16)
        Ed = (0.02 * torch.randn(V, d, device="cuda", generator=g)).to(torch.bfloat16)
        tgt = torch.randint(0, V, (N,), device="cuda", generator=g, dtype=torch.int32)
        neg = torch.randint(0, V, (ns,), device="cuda", generator=g, dtype=torch.int32)
        lengths = torch.randint(sl // 2, sl + 1, (bs,), device="cuda", generator=g)
        mask = (torch.arange(sl, device="cuda")[None, :] < lengths[:, None]).reshape(-1).to(torch.uint8)
        grad_buf = torch.zeros(V, d, device="cuda", dtype=torch.float32)

        def run(kind):
            H = Hd.clone().requires_grad_(True)
            E = Ed.clone().requires_grad_(kind != "cce_buffer")
            torch.cuda.synchronize()
            base = torch.cuda.memory_allocated()
            torch.cuda.reset_peak_memory_stats()
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            times, value = [], None
            for rep in range(args.reps + 2):
                H.grad = None
                E.grad = None
                ev[0].record()
                if kind == "materialised":
                    loss = materialised_ce_minus(H, E, tgt, neg, mask)
                else:
                    loss = P.cce_neg_loss(H, E, tgt, neg, mask, reduction="mean",
                                          grad_E_out=grad_buf if kind == "cce_buffer" else None)
                loss.backward()
                ev[1].record()
                torch.cuda.synchronize()
                if rep >= 2:
                    times.append(ev[0].elapsed_time(ev[1]))
                value = float(loss.detach())
            return dict(ms=sorted(times)[len(times) // 2], peak_extra_mb=(torch.cuda.max_memory_allocated() - base) / 1e6,
                        loss=value, dH=H.grad.float().clone())

        res = {k: run(k) for k in ("materialised", "cce_dense_grad", "cce_buffer")}
        ref = res["materialised"]
        out = {"shape": name, "positions": N, "d": d, "ns": ns, "V": V, "logits_fp32_mb": N * (ns + 1) * 4 / 1e6}
        for k, r in res.items():
            out[k] = {"ms_per_step": round(r["ms"], 4), "peak_extra_mb": round(r["peak_extra_mb"], 1), "loss": r["loss"],
                      "dH_vs_materialised": float((r["dH"] - ref["dH"]).abs().max() / ref["dH"].abs().max())}
        out["speedup_buffer"] = ref["ms"] / res["cce_buffer"]["ms"]
        out["memory_ratio_buffer"] = res["cce_buffer"]["peak_extra_mb"] / max(ref["peak_extra_mb"], 1e-9)
        print(json.dumps(out), flush=True)
        del Hd, Ed, grad_buf
        P.clear_workspaces()
        torch.cuda.empty_cache()
    return 0


if __name__ == "__main__":
    sys.exit(main())
