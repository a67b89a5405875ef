#!/usr/bin/env python3
"""Measurement studies on one MI355X, printed as Markdown tables.

  python -m paper_2602_22575_amd.studies abcd         overhead decomposition (paper App. A,
      "Why Online Permutation Adds Negligible Overhead", kernels A-D): the same dense amount
      of work, adding one mechanism at a time --
        A  contiguous causal attention (S = L: one segment, no maps)
        B  + indexed gather with identity maps          (stop_mode 2)
        C  + ranked maps from s2o_plan                  (stop_mode 2)
        D  + the early-stop vote, never stopping        (stop_mode 0, tau = -1)
      followed by the same four in the non-causal setting (params.non_causal: every query
      walks all L keys; A is the walk without a key map).
  python -m paper_2602_22575_amd.studies topk         fixed budget on the ranked order (the top-k
      selection of the appendix's matched-sparsity comparison): non-causal walk without a
      stop rule visiting the first k tiles of every ranked row, k = a fraction of L/64;
      time and speed-up over the full walk against the ideal 1/fraction.
  python -m paper_2602_22575_amd.studies plan-table   ranking time over (L, S) (the paper's
      retrieval-latency table in "Additional details on end-to-end operator performance"),
      with time * S / L^2 to check the L^2 / S law.

  python -m paper_2602_22575_amd.studies mixed        the mixed workload (half the KV groups
      unstructured, half with a strong heavy-key boost) at 64x64 and 128x64 tiles: times and
      the spread of the per-head density.

  python -m paper_2602_22575_amd.studies qperm        with and without the query permutation
      (paper's component ablation and "Single-pass Variant"): time, density and MSE against
      the dense output, for the two-launch form, the fused launch, and original query order.

  python -m paper_2602_22575_amd.studies power        is the prefix walk limited by its instruction
      schedule or by the chip's power budget?  The same dense walk (tau = 0: every tile folded
      in, identical instruction stream) on the workload's Gaussian data, with V zeroed, and with
      Q, K and V all zero, with the shader clock the driver reports sampled meanwhile: equal
      time x clock products with very different clocks mean the cycle count is fixed and the
      clock is what the data's switching activity leaves of the power budget.  Followed by the
      own-segment pass on the workload's data and on zeros.

Inputs are the seeded synthetic workloads of inputs.py; every figure is the mean of a few
launches timed with events on the launch stream.
"""
from __future__ import annotations

import sys

import numpy as np


def _timed(fn, iters=3):
    import torch
    fn()
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(iters + 1)]
    ev[0].record()
    for i in range(iters):
        fn()
        ev[i + 1].record()
    torch.cuda.synchronize()
    return float(np.mean([ev[i].elapsed_time(ev[i + 1]) for i in range(iters)]))


def _dev(bits):
    import torch
    return torch.from_numpy(bits.view(np.int16)).to("cuda:0").view(torch.bfloat16)


def abcd():
    import torch
    from . import binding as s2o, inputs
    print("| L | S | A contiguous ms (TFLOP/s) | B identity gather ms | C ranked gather ms | D + stop vote ms | B/A | C/B | D/C |")
    print("|---|---|---|---|---|---|---|---|---|")
    for name in ("llama8k", "llama32k", "llama128k"):
        w = inputs.workload(name)
        Qd, Kd, Vd = (_dev(x) for x in inputs.make_qkv(w))
        T = w.L // 64
        flops = 4.0 * 64 * 64 * w.D * T * (T + 1) / 2 * w.Z * w.H
        pa = s2o.make_params(w.Z, w.H, w.Hkv, w.L, w.D, w.L, w.BM, w.BN, use_q_perm=0)
        state = torch.empty(s2o.s2o_attention_sizes(pa)["scratch"], dtype=torch.uint8, device="cuda:0")
        O = torch.empty_like(Qd)
        cnt = torch.empty((w.Z, w.H, w.L // w.BM), dtype=torch.int32, device="cuda:0")
        cnt2 = torch.empty_like(cnt)
        kw = dict(O=O, computed=cnt, skipped=cnt2, scratch=state)
        p2 = s2o.make_params(w.Z, w.H, w.Hkv, w.L, w.D, w.S, w.BM, w.BN, stop_mode=2)
        p0 = s2o.make_params(w.Z, w.H, w.Hkv, w.L, w.D, w.S, w.BM, w.BN, stop_mode=0)
        plan = s2o.s2o_plan(Qd, Kd, p2, want_scores=False)
        N = w.L // w.S
        qi = torch.arange(w.S, dtype=torch.int32, device="cuda:0").expand(w.Z, w.H, N, w.S).contiguous()
        row = torch.cat([torch.arange(n * w.S, dtype=torch.int32, device="cuda:0") for n in range(1, N)])
        ki = row.expand(w.Z, w.H, row.numel()).contiguous()
        variants = [lambda: s2o.s2o_attention(Qd, Kd, Vd, pa, None, None, -1.0, **kw),
                    lambda: s2o.s2o_attention(Qd, Kd, Vd, p2, qi, ki, -1.0, **kw),
                    lambda: s2o.s2o_attention(Qd, Kd, Vd, p2, plan.q_perm, plan.kv_perm, -1.0, **kw),
                    lambda: s2o.s2o_attention(Qd, Kd, Vd, p0, plan.q_perm, plan.kv_perm, -1.0, **kw)]
        # the clock sags as the chip warms up: interleave the variants and take medians
        times = [[] for _ in variants]
        for rep in range(5):
            for i, fn in enumerate(variants):
                times[i].append(_timed(fn, 1))
        a, b, c, d = (float(np.median(t)) for t in times)
        print(f"| {w.L} | {w.S} | {a:.2f} ({flops / a / 1e9:.0f}) | {b:.2f} | {c:.2f} | {d:.2f} | "
              f"{b / a:.3f} | {c / b:.3f} | {d / c:.3f} |", flush=True)
        del Qd, Kd, Vd, O, state, plan, qi, ki
        torch.cuda.empty_cache()
    print()
    print("| L | S | non-causal: A no map ms (TFLOP/s) | B identity gather ms | C ranked gather ms | D + stop vote ms | B/A | C/B | D/C |")
    print("|---|---|---|---|---|---|---|---|---|")
    for name in ("llama8k", "llama32k", "llama128k"):
        w = inputs.workload(name)
        Qd, Kd, Vd = (_dev(x) for x in inputs.make_qkv(w))
        T = w.L // 64
        flops = 4.0 * 64 * 64 * w.D * T * T * w.Z * w.H
        O = torch.empty_like(Qd)
        cnt = torch.empty((w.Z, w.H, w.L // w.BM), dtype=torch.int32, device="cuda:0")
        cnt2 = torch.empty_like(cnt)
        kw = dict(O=O, computed=cnt, skipped=cnt2)
        p2 = s2o.make_params(w.Z, w.H, w.Hkv, w.L, w.D, w.S, w.BM, w.BN, stop_mode=2, non_causal=1)
        p0 = s2o.make_params(w.Z, w.H, w.Hkv, w.L, w.D, w.S, w.BM, w.BN, stop_mode=0, non_causal=1)
        plan = s2o.s2o_plan(Qd, Kd, p2, want_scores=False)
        N = w.L // w.S
        qi = torch.arange(w.S, dtype=torch.int32, device="cuda:0").expand(w.Z, w.H, N, w.S).contiguous()
        ki = torch.arange(w.L, dtype=torch.int32, device="cuda:0").repeat(N).expand(w.Z, w.H, N * w.L).contiguous()
        pa = s2o.make_params(w.Z, w.H, w.Hkv, w.L, w.D, w.S, w.BM, w.BN, stop_mode=2, non_causal=1, use_q_perm=0)
        variants = [lambda: s2o.s2o_attention(Qd, Kd, Vd, pa, None, None, -1.0, **kw),
                    lambda: s2o.s2o_attention(Qd, Kd, Vd, p2, qi, ki, -1.0, **kw),
                    lambda: s2o.s2o_attention(Qd, Kd, Vd, p2, plan.q_perm, plan.kv_perm, -1.0, **kw),
                    lambda: s2o.s2o_attention(Qd, Kd, Vd, p0, plan.q_perm, plan.kv_perm, -1.0, **kw)]
        times = [[] for _ in variants]
        for rep in range(3):
            for i, fn in enumerate(variants):
                times[i].append(_timed(fn, 1))
        a_, b_, c, d = (float(np.median(t)) for t in times)
        print(f"| {w.L} | {w.S} | {a_:.2f} ({flops / a_ / 1e9:.0f}) | {b_:.2f} | {c:.2f} | {d:.2f} | "
              f"{b_ / a_:.3f} | {c / b_:.3f} | {d / c:.3f} |", flush=True)
        del Qd, Kd, Vd, O, plan, qi, ki
        torch.cuda.empty_cache()


def topk():
    import torch
    from . import binding as s2o, inputs
    print("| L | kept fraction of key tiles | attention ms | speed-up over the full walk | ideal |")
    print("|---|---|---|---|---|")
    for name in ("llama32k", "llama128k"):
        w = inputs.workload(name)
        Qd, Kd, Vd = (_dev(x) for x in inputs.make_qkv(w))
        O = torch.empty_like(Qd)
        cnt = torch.empty((w.Z, w.H, w.L // w.BM), dtype=torch.int32, device="cuda:0")
        cnt2 = torch.empty_like(cnt)
        pp = s2o.make_params(w.Z, w.H, w.Hkv, w.L, w.D, w.S, w.BM, w.BN, stop_mode=2, non_causal=1)
        plan = s2o.s2o_plan(Qd, Kd, pp, want_scores=False)
        nK = w.L // w.BN
        full = None
        for frac in (1.0, 0.5, 0.25, 0.125, 0.0625, 0.03125):
            k = max(1, int(round(frac * nK)))
            p = s2o.make_params(w.Z, w.H, w.Hkv, w.L, w.D, w.S, w.BM, w.BN, stop_mode=2, non_causal=1,
                                max_prefix_tiles=k)
            ms = _timed(lambda: s2o.s2o_attention(Qd, Kd, Vd, p, plan.q_perm, plan.kv_perm, -1.0, O=O,
                                                  computed=cnt, skipped=cnt2), 3)
            full = ms if full is None else full
            print(f"| {w.L} | {k / nK:.4f} | {ms:.2f} | {full / ms:.2f} | {nK / k:.2f} |", flush=True)
        del Qd, Kd, Vd, O, plan
        torch.cuda.empty_cache()


def plan_table():
    import torch
    from . import binding as s2o, inputs
    Ss = (512, 1024, 2048, 4096)
    print("| L | " + " | ".join(f"S={S} ms (ms*S/L^2 *1e9)" for S in Ss) + " |")
    print("|---|" + "---|" * len(Ss))
    for L in (4096, 8192, 16384, 32768, 65536, 131072):
        w = inputs.workload("llama128k", L=L, S=min(2048, L // 2))
        Qb, Kb, _ = inputs.make_qkv(w)
        Qd, Kd = _dev(Qb), _dev(Kb)
        cells = []
        for S in Ss:
            if L // S < 2:
                cells.append("-")
                continue
            p = s2o.make_params(w.Z, w.H, w.Hkv, L, w.D, S)
            scratch = torch.empty(s2o.s2o_plan_sizes(p)["scratch"], dtype=torch.uint8, device="cuda:0")
            N = L // S
            P = S * N * (N - 1) // 2
            maps = (torch.empty((w.Z, w.H, N, S), dtype=torch.int32, device="cuda:0"),
                    torch.empty((w.Z, w.H, max(P, 4)), dtype=torch.int32, device="cuda:0"))
            ms = _timed(lambda: s2o.s2o_plan(Qd, Kd, p, want_scores=False, scratch=scratch, maps=maps), 5)
            cells.append(f"{ms:.3f} ({ms * S / L / L * 1e9:.1f})")
            del scratch, maps
        print(f"| {L} | " + " | ".join(cells) + " |", flush=True)
        del Qd, Kd
        torch.cuda.empty_cache()


def qperm():
    import torch
    from . import binding as s2o, inputs
    w = inputs.workload("llama128k")
    Qd, Kd, Vd = (_dev(x) for x in inputs.make_qkv(w))
    p1 = s2o.make_params(w.Z, w.H, w.Hkv, w.L, w.D, w.S, w.BM, w.BN, use_q_perm=1)
    p0 = s2o.make_params(w.Z, w.H, w.Hkv, w.L, w.D, w.S, w.BM, w.BN, use_q_perm=0)
    plan = s2o.s2o_plan(Qd, Kd, p1, want_scores=False)
    state = torch.empty(s2o.s2o_attention_sizes(p1)["scratch"], dtype=torch.uint8, device="cuda:0")
    dense = torch.empty_like(Qd)
    s2o.s2o_attention(Qd, Kd, Vd, p1, plan.q_perm, plan.kv_perm, 0.0, O=dense, scratch=state)
    ref = dense.float()
    den2 = float((ref ** 2).sum())
    N, TJ, per = w.L // w.S, w.S // w.BM, w.S // w.BN
    nk = torch.from_numpy(np.repeat(np.arange(N) * per, TJ)).to("cuda:0")
    T = w.L // w.BM
    causal = T * (T + 1) // 2
    local = N * TJ * (TJ + 1) // 2
    O = torch.empty_like(Qd)
    c = torch.empty((w.Z, w.H, w.L // w.BM), dtype=torch.int32, device="cuda:0")
    sk = torch.empty_like(c)
    print(f"workload {w.name}: L={w.L} S={w.S}, 64x64 tiles")
    print("| tau | variant | attention ms | density | MSE vs dense | relative MSE |")
    print("|---|---|---|---|---|---|")
    for tau in (1e-3, 5e-3, 2e-2):
        variants = [("Q_perm, two launches (Alg. 2 + Alg. 3)", p1, plan.q_perm, True),
                    ("Q_perm, one fused launch", p1, plan.q_perm, False),
                    ("original query order, one fused launch (Alg. 4)", p0, None, False),
                    ("original query order, two launches", p0, None, True)]
        for name, p, qp, two in variants:
            fn = lambda: s2o.s2o_attention(Qd, Kd, Vd, p, qp, plan.kv_perm, tau, O=O, computed=c, skipped=sk,
                                           scratch=state if two else None, two_pass=two)
            ms = _timed(fn, 3)
            dens = float((local * w.H + (nk[None, None] - sk).sum()) / (causal * w.H))
            d = O.float() - ref
            mse = float((d ** 2).mean(dim=(0, 2, 3)).mean())
            print(f"| {tau} | {name} | {ms:.2f} | {dens:.4f} | {mse:.3e} | {float((d ** 2).sum()) / den2:.3e} |", flush=True)
            del d


def mixed():
    import torch
    from . import binding as s2o, inputs
    w0 = inputs.workload("mixed128k")
    Qd, Kd, Vd = (_dev(x) for x in inputs.make_qkv(w0))
    tau = 5e-3
    print(f"workload {w0.name}: L={w0.L} S={w0.S} tau={tau}; heads 0-{w0.H // 2 - 1} unstructured, the rest boosted")
    print("| tiles | local ms | prefix ms | density all heads | unstructured heads min/median/max | boosted heads min/median/max |")
    print("|---|---|---|---|---|---|")
    for BM in (64, 128):
        p = s2o.make_params(w0.Z, w0.H, w0.Hkv, w0.L, w0.D, w0.S, BM, w0.BN)
        plan = s2o.s2o_plan(Qd, Kd, p, want_scores=False)
        state = torch.empty(s2o.s2o_attention_sizes(p)["scratch"], dtype=torch.uint8, device="cuda:0")
        O = torch.empty_like(Qd)
        c = torch.empty((w0.Z, w0.H, w0.L // BM), dtype=torch.int32, device="cuda:0")
        sk = torch.empty_like(c)
        tl = _timed(lambda: s2o.s2o_attention_local(Qd, Kd, Vd, p, scratch=state), 5)
        tp = _timed(lambda: s2o.s2o_attention_prefix(Qd, Kd, Vd, p, plan.q_perm, plan.kv_perm, tau, state, O=O,
                                                     computed=c, skipped=sk), 5)
        skn = sk.cpu().numpy()[0]                                   # [H, L/BM]
        N, TJ, per = w0.L // w0.S, w0.S // BM, w0.S // w0.BN
        nk = np.repeat(np.arange(N) * per, TJ)
        local = N * sum(-(-((b + 1) * BM) // w0.BN) for b in range(TJ))
        causal = sum(-(-((b + 1) * BM) // w0.BN) for b in range(w0.L // BM))
        dens = (local + (nk[None] - skn).sum(axis=1)) / causal      # per head
        half = w0.H // 2
        fmt = lambda d: f"{d.min():.4f} / {np.median(d):.4f} / {d.max():.4f}"
        print(f"| {BM}x{w0.BN} | {tl:.2f} | {tp:.2f} | {dens.mean():.4f} | {fmt(dens[:half])} | {fmt(dens[half:])} |",
              flush=True)
        del plan, state, O, c, sk
        torch.cuda.empty_cache()


def power():
    import glob
    import threading
    import time
    import torch
    from . import binding as s2o, inputs
    w = inputs.workload("llama128k")
    Qd, Kd, Vd = (_dev(x) for x in inputs.make_qkv(w))
    p = s2o.make_params(w.Z, w.H, w.Hkv, w.L, w.D, w.S, w.BM, w.BN)
    plan = s2o.s2o_plan(Qd, Kd, p, want_scores=False)
    state = torch.empty(s2o.s2o_attention_sizes(p)["scratch"], dtype=torch.uint8, device="cuda:0")
    O = torch.empty_like(Qd)
    files = sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))

    def sclk():
        try:
            for line in open(files[0]):
                if line.rstrip().endswith("*"):
                    return float(line.split(":")[1].strip().split("Mhz")[0])
        except Exception:
            return None
        return None

    dense_flops = 4.0 * w.BM * w.BN * w.D * sum(n * (w.S // w.BN) * (w.S // w.BM) for n in range(w.N)) * w.Z * w.H
    print(f"workload {w.name}: dense prefix walk (tau = 0, ranked maps of the real data in every case), 64x64 tiles")
    print("| data | ms | TFLOP/s | shader clock MHz (median of samples) | ms x GHz |")
    print("|---|---|---|---|---|")
    zero = lambda t: torch.zeros_like(t)
    for name, (q_, k_, v_) in (("Gaussian Q, K, V (the workload)", (Qd, Kd, Vd)),
                               ("Gaussian Q, K; V = 0", (Qd, Kd, zero(Vd))),
                               ("Q = K = V = 0", (zero(Qd), zero(Kd), zero(Vd))),
                               ("Gaussian Q, K, V again", (Qd, Kd, Vd))):
        s2o.s2o_attention_local(q_, k_, v_, p, scratch=state)
        torch.cuda.synchronize()
        samples, stop = [], [False]

        def loop():
            while not stop[0]:
                v = sclk() if files else None
                if v:
                    samples.append(v)
                time.sleep(0.002)
        th = threading.Thread(target=loop)
        th.start()
        ms = _timed(lambda: s2o.s2o_attention_prefix(q_, k_, v_, p, plan.q_perm, plan.kv_perm, 0.0, state, O=O), 3)
        stop[0] = True
        th.join()
        mhz = float(np.median(samples)) if samples else float("nan")
        print(f"| {name} | {ms:.2f} | {dense_flops / (ms * 1e-3) / 1e12:.0f} | {mhz:.0f} | {ms * mhz / 1e3:.1f} |", flush=True)

    # the own-segment pass the same way: 120 launches back to back per row (a single launch of
    # 2.5 ms is too short for the clock to settle, or to be sampled)
    tq = w.S // w.BN
    local_flops = 4.0 * w.BN * w.BN * w.D * (tq * (tq + 1) // 2) * w.N * w.Z * w.H   # 64x64 tiles on or below the diagonal
    print()
    print(f"workload {w.name}: own-segment pass, 120 launches back to back")
    print("| data | ms per launch | TFLOP/s (64x64 tiles on or below the diagonal, counted whole) | shader clock MHz | ms x GHz |")
    print("|---|---|---|---|---|")

    def burst(q_, k_, v_, n=120):
        for _ in range(5):
            s2o.s2o_attention_local(q_, k_, v_, p, scratch=state)
        torch.cuda.synchronize()
        samples, stop = [], [False]

        def loop():
            while not stop[0]:
                v = sclk() if files else None
                if v:
                    samples.append(v)
                time.sleep(0.002)
        th = threading.Thread(target=loop)
        th.start()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(n):
            s2o.s2o_attention_local(q_, k_, v_, p, scratch=state)
        b.record()
        torch.cuda.synchronize()
        stop[0] = True
        th.join()
        return a.elapsed_time(b) / n, (float(np.median(samples)) if samples else float("nan"))
    for name, (q_, k_, v_) in (("Gaussian Q, K, V (the workload)", (Qd, Kd, Vd)),
                               ("Q = K = V = 0", (zero(Qd), zero(Kd), zero(Vd))),
                               ("Gaussian Q, K, V again", (Qd, Kd, Vd))):
        ms, mhz = burst(q_, k_, v_)
        print(f"| {name} | {ms:.3f} | {local_flops / (ms * 1e-3) / 1e12:.0f} | {mhz:.0f} | {ms * mhz / 1e3:.2f} |", flush=True)


if __name__ == "__main__":
    what = sys.argv[1] if len(sys.argv) > 1 else ""
    if what == "abcd":
        abcd()
    elif what == "topk":
        topk()
    elif what == "plan-table":
        plan_table()
    elif what == "mixed":
        mixed()
    elif what == "qperm":
        qperm()
    elif what == "power":
        power()
    else:
        print(__doc__)
        sys.exit(2)
