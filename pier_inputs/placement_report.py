"""Placement diagnostic: how fast the two optimizer kernels stream at one workload's size under
different placements of its buffers in HBM.

    python -m pier_inputs.placement_report [--workload gpt2_xl] [--policies plain two_class pairs spread]

"plain" allocates every buffer separately, kind by kind; the others carve them out of an arena
classified by pier_hbm_probe (see PlacedState for the policies).  Each policy runs in
the same process on freshly allocated state; prints one line per policy with the AdamW rate of
every replica and the outer-step rates.  No optimizer arithmetic here: it only times launches.

    python -m pier_inputs.placement_report --outer-layouts

times the outer step alone with its G + 2 buffers at explicit offsets of one large allocation
(meaningful in a fresh process, where the allocation maps linearly onto the address classes:
0-96, 96-192, 192-288 GiB on a 288 GiB MI355X).
"""
import argparse
import gc
import json
import time

import torch

import paper_2511_17849_amd as pier
from pier_inputs import device as dev
from pier_inputs import shapes


def measure(w, policy, iters):
    N, G = w.N, w.G
    st = torch.cuda.current_stream()
    hp = dict(lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, weight_decay=w.weight_decay)
    gdt = torch.bfloat16 if w.grad_bf16 else torch.float32
    info = {"policy": policy}
    arena = None
    if policy != "plain":
        free, _ = torch.cuda.mem_get_info()
        t0 = time.time()
        arena = pier.HbmArena(free - (8 << 30))
        info["probe_s"] = round(time.time() - t0, 2)
        info["classes"] = "".join(str(c) for c in arena.classes)
    S = dev.PlacedState(w.numels, G, grad_dtype=gdt, arena=arena, policy=policy if arena else "two_class")
    for g in range(G):
        dev.fill_normal(S.P[g].flat, seed=w.seed, stream=shapes.PARAM_STREAM, step=0, std=w.param_std)
        dev.fill_normal(S.Gd[g].flat, seed=w.seed, stream=g, step=1, std=w.grad_std)
    S.A.flat.copy_(S.P[0].flat)
    ctx = pier.pier_ctx_create(w.numels, G)
    for g in range(G):
        pier.pier_bind_replica(ctx, g, S.P[g].tensors, S.M1[g].tensors, S.V[g].tensors, S.Gd[g].tensors,
                               w.grad_bf16)
    pier.pier_bind_outer(ctx, pier.PIER_LOC_DEVICE, S.A.tensors, S.Mo.tensors)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        for _ in range(iters):
            fn()
        e1.record(st)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    step = [0]
    gbytes = 26 if w.grad_bf16 else 28
    rates = []
    for g in range(G):
        def f(g=g):
            step[0] += 1
            pier.pier_inner_adamw(ctx, g, step=step[0], stream=st, **hp)
        rates.append(gbytes * N / timed(f) / 1e6)
    info["adamw_GBps_per_replica"] = [round(r) for r in rates]
    info["adamw_GBps_mean"] = round(sum(rates) / len(rates))
    for name, phase, bpe in (("outer_pier_GBps", pier.PIER_PHASE_PIER, 8 * G + 16),
                             ("outer_lazy_start_GBps", pier.PIER_PHASE_WARMUP, 4 * G + 16)):
        ms = timed(lambda: pier.pier_outer_step(ctx, outer_lr=1.1, mu=0.9, phase=phase, stream=st))
        info[name] = round(bpe * N / ms / 1e6)
    if arena is not None:
        info["placement"] = {"theta": [p.cls for p in S.P], "m": [p.cls for p in S.M1], "v": [p.cls for p in S.V],
                             "grad": [p.cls for p in S.Gd], "anchor": S.A.cls, "M": S.Mo.cls}
    pier.pier_ctx_destroy(ctx)
    return info


def outer_layouts(w, iters):
    """The outer step with theta_0 .. theta_{G-1}, anchor, M at explicit GiB offsets."""
    N, G = w.N, w.G
    GiB = 1 << 30
    st = torch.cuda.current_stream()
    free, _ = torch.cuda.mem_get_info()
    arena = torch.empty(((free - (8 << 30)) // GiB) * GiB, dtype=torch.uint8, device="cuda")
    arena.zero_()
    size = arena.numel() // GiB
    need = -(-4 * N // GiB)
    starts, off = [], 0
    for n in w.numels:
        starts.append(off)
        off += n

    def tensors_at(gib):
        flat = arena[int(gib * GiB):int(gib * GiB) + 4 * N].view(torch.float32)
        return [flat[s:s + n] for s, n in zip(starts, w.numels)]

    half = (G + 2 + 1) // 2
    sp = max(need + 1, 16 if need <= 8 else 2 * need)
    layouts = [
        ("all in class 0, packed", [need * k for k in range(G + 2)]),
        ("classes 0 and 1, half each, in blocks", [sp * k for k in range(half)] + [96 + sp * k for k in range(G + 2 - half)]),
        ("classes 0 and 1, half each, interleaved", [(96 if k % 2 else 0) + sp * (k // 2) for k in range(G + 2)]),
        ("classes 0 and 2, half each, in blocks", [sp * k for k in range(half)] + [192 + sp * k for k in range(G + 2 - half)]),
        ("three classes, a third each", [96 * (k % 3) + sp * (k // 3) for k in range(G + 2)]),
        ("classes 0 and 1, all but two in class 0", [need * k for k in range(G)] + [96, 96 + sp]),
    ]
    for name, pos in layouts:
        srt = sorted(pos)
        if srt[-1] + need > size or any(b - a < need for a, b in zip(srt, srt[1:])):
            print(json.dumps({"layout": name, "skipped": "does not fit"}), flush=True)
            continue
        lists = [tensors_at(p) for p in pos]
        ctx = pier.pier_ctx_create(w.numels, G)
        for g in range(G):          # only the outer step runs: m, v, grad are never touched
            pier.pier_bind_replica(ctx, g, lists[g], lists[g], lists[g], lists[g])
        pier.pier_bind_outer(ctx, pier.PIER_LOC_DEVICE, lists[G], lists[G + 1])
        info = {"layout": name, "offsets_GiB": pos}
        for key, phase, bpe in (("outer_pier_GBps", pier.PIER_PHASE_PIER, 8 * G + 16),
                                ("outer_lazy_start_GBps", pier.PIER_PHASE_WARMUP, 4 * G + 16)):
            fn = lambda: pier.pier_outer_step(ctx, outer_lr=1.1, mu=0.9, phase=phase, stream=st)
            fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(st)
            for _ in range(iters):
                fn()
            e1.record(st)
            torch.cuda.synchronize()
            info[key] = round(bpe * N / (e0.elapsed_time(e1) / iters) / 1e6)
        pier.pier_ctx_destroy(ctx)
        print(json.dumps(info), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="gpt2_xl")
    ap.add_argument("--policies", nargs="+", default=["plain", "two_class", "pairs", "spread"])
    ap.add_argument("--iters", type=int, default=5)
    ap.add_argument("--outer-layouts", action="store_true")
    args = ap.parse_args()
    w = shapes.workloads()[args.workload]
    torch.cuda.set_device(0)
    if args.outer_layouts:
        outer_layouts(w, args.iters)
        return
    for policy in args.policies:
        print(json.dumps(measure(w, policy, args.iters)), flush=True)
        gc.collect()
        torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
