#!/usr/bin/env python3
"""Benchmark of the dAD hot path on one MI355X.

One step = one pass of the whole path over every linear layer of the workload:
stack the S sites' factor pairs -> rank-r compress (structured power iteration)
-> rebuild the full gradient A^T Delta -> rebuild the rank-r gradient P G^T.
Inputs are synthetic, seeded and resident in HBM before the timed region.

Prints ONE JSON line.  `value` is the full-gradient rebuild rate in TFLOP/s
(2*N*h_in*h_out flops per layer over the time between the events that bracket
the rebuild calls); the rank-r compress time per layer, the stack rate and the
whole-step time ride along.  `roofline` is computed for the kernel with the
largest share of GPU time from per-kernel HIP-event timings taken by the
library on the launch stream while the same steps are repeated right after
the timed region.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "dAD gradient-rebuild TFLOP/s + rank-r compress us/layer (% MFMA/HBM roofline)"
PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3       # MI355X fp32 vector / matrix
PEAK_HBM_GBPS = 8000.0         # MI355X HBM3E


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="gpt2_medium_stack")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--lanes", type=int, default=4,
                    help="default mode: layers of one block whose compress calls are in flight at once "
                         "(dad_compress_rank_grouped); 0 = one dad_compress_rank call per layer")
    ap.add_argument("--group-layers", type=int, default=0,
                    help="default mode: layers per grouped compress call when every layer has its own stacked "
                         "buffer (0 = the whole stack)")
    ap.add_argument("--graphs", default="off", choices=["auto", "on", "off"],
                    help="default mode: replay one captured HIP graph per operation of a step (auto: workloads of "
                         "at most 8 layers, which are bound by launch latency)")
    ap.add_argument("--rebuild-group", type=int, default=0,
                    help="layers per full-gradient call (dad_reconstruct_grad_grouped); 1 = one dad_reconstruct_grad per "
                         "layer; 0 = a block's layers together for the small workloads, few-tile neighbours for the large ones")
    ap.add_argument("--rebuild-tile-budget", type=int, default=128,
                    help="automatic full-gradient grouping of the large workloads: join neighbours while their 256x256 "
                         "output tiles together stay within this")
    ap.add_argument("--no-sites-leg", action="store_true",
                    help="skip the extra timed leg that reads the sites' blocks in place (no stacking pass)")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="default mode: skip the encoder_d768 and vit_large_stack passes that follow the headline workload")
    ap.add_argument("--mode", default="one_level", choices=["one_level", "two_level", "backprop", "sequential"],
                    help="two_level: Algorithm 1 (per-site reduction, stack of the pairs, aggregator reduction, rebuild); "
                         "backprop: the delta recursion of Eq. 3, every site writing its rows into the stacked buffer; "
                         "sequential: Algorithm 2 one singular pair at a time with peeling, one block of the stack")
    ap.add_argument("--per-site-calls", action="store_true",
                    help="backprop: one call per site (b rows each) instead of one call over all N rows")
    ap.add_argument("--no-graphs", action="store_true",
                    help="two_level: launch eagerly instead of replaying one captured HIP graph per layer")
    ap.add_argument("--agg-route", default="gram", choices=["gram", "block"],
                    help="two_level: the aggregator's reduction of the S*r stacked rows runs on the Gram matrices "
                         "of the stack (dad_compress_rank_gram, when S*r <= 512) or as the block power iteration")
    ap.add_argument("--site-route", default="grouped", choices=["grouped", "streams"],
                    help="two_level: the S site reductions of a layer as one dad_compress_rank_grouped call, or as S "
                         "dad_compress_rank calls on --site-streams streams")
    ap.add_argument("--site-streams", type=int, default=8,
                    help="two_level: HIP streams (default priority) the independent per-site reductions are spread over")
    return ap.parse_args()


def kernel_model(name, N, h_in, h_out, r, es, which, bf16=True):
    """Algorithmic work of one launch: ("hbm", bytes) or ("mfma", flops).

    `which` says which factor the launch streams ("in" = A, "out" = Delta).
    """
    h = h_in if which == "in" else h_out
    if name in ("k_thin_nn_bf16", "k_thin_tn_bf16", "k_thin_nn", "k_thin_tn"):
        return "hbm", float(N) * h * es
    if name in ("k_rebuild_bf16", "k_rebuild_bf16_dma"):
        return "mfma", 2.0 * N * h_in * h_out
    if name == "k_rebuild":
        if bf16:   # only the rank-r rebuild (K = r, fp32 pairs) runs this kernel: write bound
            return "hbm", 4.0 * h_in * h_out + 4.0 * r * (h_in + h_out)
        return "mfma", 2.0 * N * h_in * h_out + 2.0 * r * h_in * h_out   # full + rank-r launches together
    if name == "k_rebuild_f32_mfma":
        if bf16:   # rank-r rebuild only (K = r, fp32 pairs): write bound
            return "hbm", 4.0 * h_in * h_out + 4.0 * r * (h_in + h_out)
        return "mfma", 2.0 * N * h_in * h_out + 2.0 * r * h_in * h_out   # full + rank-r launches together
    if name == "k_stack":
        return "hbm", 2.0 * N * (h_in + h_out) * es
    return None, 0.0


def two_level(args, w, dad, W, torch, np, dev):
    """Algorithm 1 per layer: every site reduces its own b rows to r (S calls), the S*r stacked
    rows are reduced again at the aggregator, the estimate P^T G is rebuilt.  `value` is the time
    per layer; the site-level reductions stream every factor byte 2n+1 times, as the one-level
    path does, so `site_compress_GBps` is comparable with `compress_GBps` of the default mode."""
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    es = 2 if w.dtype == "bf16" else 4
    N, r, n_iter, S, b = w.N, w.rank, w.n_iter, w.sites, w.rows_per_site
    layers = w.all_layers()
    nl = len(layers)
    total_bytes = sum(N * (hi + ho) * es for _, hi, ho in layers)
    resident = layers if total_bytes < 150e9 else layers[:len(w.shapes)]
    sites = {li: W.device_factors(w, li, hi, ho, device=dev) for li, hi, ho in resident}
    def factors_of(li):
        return sites[li] if li in sites else sites[li % len(w.shapes)]
    G0s = {li: [torch.from_numpy(W.host_start_matrix(w, 1000 + 64 * li + s, ho)).to(dev) for s in range(S)]
           for li, _, ho in layers}
    G0a = {li: torch.from_numpy(W.host_start_matrix(w, 5000 + li, ho)).to(dev) for li, _, ho in layers}
    Ps = {sh: [torch.empty((r, sh[0]), dtype=torch.float32, device=dev) for _ in range(S)] for sh in w.shapes}
    Gs = {sh: [torch.empty((r, sh[1]), dtype=torch.float32, device=dev) for _ in range(S)] for sh in w.shapes}
    Pst = {sh: torch.empty((S * r, sh[0]), dtype=torch.float32, device=dev) for sh in w.shapes}
    Gst = {sh: torch.empty((S * r, sh[1]), dtype=torch.float32, device=dev) for sh in w.shapes}
    Pt = {li: torch.empty((r, hi), dtype=torch.float32, device=dev) for li, hi, _ in layers}
    Gt = {li: torch.empty((r, ho), dtype=torch.float32, device=dev) for li, _, ho in layers}
    G_hat = {sh: torch.empty(sh, dtype=torch.float32, device=dev) for sh in w.shapes}
    n_str = max(1, min(args.site_streams, S))
    ws_s = [torch.zeros(max(dad.compress_workspace_bytes(b, hi, ho, r, tdt) for _, hi, ho in layers),
                        dtype=torch.uint8, device=dev) for _ in range(n_str)]
    side = [torch.cuda.Stream(device=dev) for _ in range(n_str)] if n_str > 1 else []
    agg_gram = args.agg_route == "gram" and S * r <= 512      # beyond that the block form is the faster one
    agg_bytes = dad.compress_gram_workspace_bytes if agg_gram else dad.compress_workspace_bytes
    agg_call = dad.compress_rank_gram if agg_gram else dad.compress_rank
    ws_a = torch.zeros(max(agg_bytes(S * r, hi, ho, r, torch.float32) for _, hi, ho in layers),
                       dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    PH = ("site_compress", "stack_pairs", "agg_compress", "rebuild_rank")

    # The S site reductions of a layer as ONE dad_compress_rank_grouped call: equal sites on the
    # direct-to-LDS path share their launches (a batch), others run on up to n_str lanes.
    site_groups = {}
    if args.site_route == "grouped":
        placeholder = torch.zeros(256, dtype=torch.uint8, device=dev)
        for li, hi, ho in layers:
            As, Ds = factors_of(li)
            site_groups[li] = dad.CompressGroup([(As[s_], Ds[s_], G0s[li][s_]) for s_ in range(S)], r, n_iter,
                                                lanes=min(n_str, dad.DAD_MAX_LANES), Pts=Ps[(hi, ho)], Gts=Gs[(hi, ho)],
                                                workspace=placeholder)
        ws_g = torch.zeros(max(g.need for g in site_groups.values()), dtype=torch.uint8, device=dev)
        for g in site_groups.values():      # all share one workspace, sized for the largest layer
            g.workspace = ws_g
        ws_s = [ws_g]

    def site_pass(li, sh, As, Ds):
        """The S independent site reductions: one grouped call, or (--site-route streams) site s on
        stream s mod n_str, each stream with its own workspace."""
        if site_groups:
            site_groups[li].run()
            return
        if not side:
            for s_ in range(S):
                dad.compress_rank(As[s_], Ds[s_], r, n_iter, G0s[li][s_], Pt=Ps[sh][s_], Gt=Gs[sh][s_], workspace=ws_s[0])
            return
        main = torch.cuda.current_stream()
        fork = torch.cuda.Event()
        fork.record(main)
        for k, st in enumerate(side):
            st.wait_event(fork)
            with torch.cuda.stream(st):
                for s_ in range(k, S, n_str):
                    dad.compress_rank(As[s_], Ds[s_], r, n_iter, G0s[li][s_], Pt=Ps[sh][s_], Gt=Gs[sh][s_],
                                      workspace=ws_s[k])
        for st in side:
            main.wait_stream(st)

    graphs = {}
    pool = [torch.cuda.Event(enable_timing=True) for _ in range(5 * len(layers) * args.steps)]
    pool_next = [0]
    if pool:
        pool[0].record(); pool[1].record(); torch.cuda.synchronize(); pool[0].elapsed_time(pool[1])

    def step(events=None, replay=False):
        if replay:
            for li, _, _ in layers:
                graphs[li].replay()
            return
        for li, hi, ho in layers:
            sh = (hi, ho)
            As, Ds = factors_of(li)
            ev = None
            if events is not None:
                ev = pool[pool_next[0]:pool_next[0] + 5]
                pool_next[0] += 5
            if ev: ev[0].record()
            site_pass(li, sh, As, Ds)
            if ev: ev[1].record()
            dad.stack_factors(Ps[sh], Gs[sh], A_out=Pst[sh], D_out=Gst[sh])
            if ev: ev[2].record()
            agg_call(Pst[sh], Gst[sh], r, n_iter, G0a[li], Pt=Pt[li], Gt=Gt[li], workspace=ws_a)
            if ev: ev[3].record()
            dad.reconstruct_grad(Pt[li], Gt[li], G=G_hat[sh])
            if ev: ev[4].record()
            if ev: events.append(ev)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if any(dad.poll_numeric_status(x) != dad.DAD_OK for x in ws_s + [ws_a]):
        print("bench.py: numerical breakdown latched during warm-up", file=sys.stderr)
        sys.exit(1)
    # The path is launch bound at these sizes (about 190 small launches per layer), so the timed
    # region replays one captured HIP graph per layer; phase times come from an eager pass after it.
    use_graphs = not args.no_graphs
    if use_graphs:
        if args.warmup == 0:
            step()   # function attributes are set on first use; that must not happen under capture
            torch.cuda.synchronize()
        def one_layer(li, hi, ho):
            sh = (hi, ho)
            As, Ds = factors_of(li)
            site_pass(li, sh, As, Ds)
            dad.stack_factors(Ps[sh], Gs[sh], A_out=Pst[sh], D_out=Gst[sh])
            agg_call(Pst[sh], Gst[sh], r, n_iter, G0a[li], Pt=Pt[li], Gt=Gt[li], workspace=ws_a)
            dad.reconstruct_grad(Pt[li], Gt[li], G=G_hat[sh])
        for li, hi, ho in layers:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                one_layer(li, hi, ho)
            graphs[li] = g
        step(replay=True)
        torch.cuda.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(replay=use_graphs)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    events = []
    for _ in range(args.steps):
        step(events)
    torch.cuda.synchronize()
    dad.profile_reset()
    dad.profile_enable(True)
    prof_steps = 1   # one repeat is enough here: a step has thousands of launches, each with two events
    for _ in range(prof_steps):
        step()
    torch.cuda.synchronize()
    dad.profile_enable(False)
    kern = dad.profile_read()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    phase_ms = dict.fromkeys(PH, 0.0)
    for ev in events:
        for i, ph in enumerate(PH):
            phase_ms[ph] += ev[i].elapsed_time(ev[i + 1])
    phase_ms = {k: v / args.steps for k, v in phase_ms.items()}
    bytes_site = sum((2 * n_iter + 1.0) * N * (hi + ho) * es for _, hi, ho in layers)
    agg_passes = 2.0 if agg_gram else 2 * n_iter + 1.0    # reads of each stacked factor
    bytes_agg = sum(agg_passes * S * r * (hi + ho) * 4 for _, hi, ho in layers)

    # site-level thin kernels: the S calls together stream each factor once per contraction
    work = {}
    for name in kern:
        tot = 0.0
        for _, hi, ho in layers:
            if name in ("k_thin_nn_bf16", "k_thin_nn"):
                parts = [(ho, n_iter + 1), (hi, n_iter)]
            elif name in ("k_thin_tn_bf16", "k_thin_tn"):
                parts = [(hi, n_iter + 1), (ho, n_iter)]
            else:
                continue
            rows, e = (N, es) if (name.endswith("bf16") or w.dtype != "bf16") else (S * r, 4)
            if w.dtype != "bf16" and not agg_gram:   # fp32 workloads: site and aggregator calls share the guarded kernels
                rows = N + S * r
            tot += sum(cnt * float(rows) * h * e for h, cnt in parts)
        if tot:
            work[name] = tot
    roof_all = {}
    for name, (ms, launches) in kern.items():
        entry = {"ms_per_step": ms / prof_steps, "launches_per_step": launches / prof_steps,
                 "avg_us": ms * 1e3 / launches}
        if name in work:
            rate = work[name] * prof_steps / (ms * 1e-3)
            entry.update(bound="hbm", achieved=rate / 1e9, peak=PEAK_HBM_GBPS, unit="GB/s",
                         frac=rate / 1e9 / PEAK_HBM_GBPS)
        roof_all[name] = entry
    dominant = max(work, key=lambda k: kern[k][0])
    roofline = {"kernel": dominant}
    roofline.update({k: roof_all[dominant].get(k) for k in ("bound", "achieved", "peak", "unit", "frac")})
    roofline["avg_us"] = roof_all[dominant]["avg_us"]
    roofline["traffic"] = None

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import dad_oracle as O
        li, hi, ho = min(layers, key=lambda t: t[1] * t[2])
        sh = (hi, ho)
        As, Ds = factors_of(li)
        A_h = [a.float().cpu().numpy().astype(np.float64) for a in As]
        D_h = [d.float().cpu().numpy().astype(np.float64) for d in Ds]
        c0 = time.perf_counter()
        Pt_ref, Gt_ref, _ = O.rank_dad(A_h, D_h, [g.cpu().numpy() for g in G0s[li]], G0a[li].cpu().numpy(), n_iter)
        c1 = time.perf_counter()
        try:
            from threadpoolctl import threadpool_info
            threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            threads = os.cpu_count()
        site_pass(li, sh, As, Ds)
        dad.stack_factors(Ps[sh], Gs[sh], A_out=Pst[sh], D_out=Gst[sh])
        agg_call(Pst[sh], Gst[sh], r, n_iter, G0a[li], Pt=Pt[li], Gt=Gt[li], workspace=ws_a)
        dad.reconstruct_grad(Pt[li], Gt[li], G=G_hat[sh])
        torch.cuda.synchronize()
        tol = 2e-2 if w.dtype == "bf16" else 1e-5
        e = O.rel_fro(G_hat[sh].cpu().numpy(), O.rank_r_grad(Pt_ref, Gt_ref))
        cpu = {"value": (c1 - c0) * 1e6, "unit": "us/layer", "cores": int(threads), "kind": "oracle",
               "sample": f"1 of {nl} layers ({hi}x{ho}, S={S} sites of {b} rows): fp64 numpy rank_dad r={r} n={n_iter}",
               "parity_rel_fro": {"two_level": e, "tol": tol}, "host_cpus": os.cpu_count()}
        if not e <= tol:
            print(f"bench.py: parity check failed: {e:.3e}", file=sys.stderr)
            sys.exit(1)

    us_layer = ms_per_step * 1e3 / nl
    out = {
        "metric": "rank-dAD two-level reduction us/layer (% HBM roofline)",
        "value": us_layer, "unit": "us/layer", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name + "/two_level", "layers": nl, "shapes": [list(s_) for s_ in w.shapes],
                   "sites": S, "rows_per_site": b, "aggregator_rows": S * r, "rank": r, "n_iter": n_iter,
                   "site_route": args.site_route, "site_streams": n_str, "hip_graphs": use_graphs,
                   "agg_route": "gram" if agg_gram else "block",
                   "resident_layers": len(resident)},
        "site_compress_us_per_layer": phase_ms["site_compress"] * 1e3 / nl,
        "site_compress_GBps": bytes_site / (phase_ms["site_compress"] * 1e-3) / 1e9,
        "site_compress_frac_of_hbm_peak": bytes_site / (phase_ms["site_compress"] * 1e-3) / 1e9 / PEAK_HBM_GBPS,
        "agg_compress_us_per_layer": phase_ms["agg_compress"] * 1e3 / nl,
        "agg_compress_GBps": bytes_agg / (phase_ms["agg_compress"] * 1e-3) / 1e9,
        "stack_pairs_us_per_layer": phase_ms["stack_pairs"] * 1e3 / nl,
        "rank_rebuild_us_per_layer": phase_ms["rebuild_rank"] * 1e3 / nl,
        "phase_ms_per_step_eager": phase_ms,
        "roofline": roofline,
        "kernels": roof_all,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))



def backprop(args, w, dad, W, torch, np, dev):
    """Eq. 3 per layer: Delta_i = (Delta_{i+1} W_{i+1}^T) (.) phi'(Z_i) for the N = S*b rows of all
    simulated sites in one call (rows are independent: the S per-site calls at their row offsets
    give the same buffer, which --per-site-calls times instead).  The delta is born in the stacked
    layout; the copy of Delta in dad_stack_factors is not needed on this route.  Layer l has width
    h = h_out[l]; the layer after it in the list supplies h_next = h_out[l+1] (cyclically), which
    gives the FFN pairs (4096 <- 1024, 1024 <- 3072 ...) of the transformer workloads.  ReLU networks
    use its mask; the others use tanh as the transcendental stand-in for their activation."""
    if w.dtype != "bf16":
        print("bench.py --mode backprop: bf16 workloads only", file=sys.stderr)
        sys.exit(2)
    N, S, b = w.N, w.sites, w.rows_per_site
    shapes = list(w.shapes)
    pairs = [(shapes[i][1], shapes[(i + 1) % len(shapes)][1]) for i in range(len(shapes))]
    layers = [pairs[li % len(pairs)] for li, _, _ in w.all_layers()]
    act = "relu" if w.act == "relu" else "tanh"
    gen = torch.Generator(device=dev)
    gen.manual_seed(20210209 + 31 * w.index)
    Dn, Wn, Zs, out = {}, {}, {}, {}
    for h, hn in set(pairs):     # one resident set per distinct shape (each is far larger than any cache)
        Dn[(h, hn)] = (torch.randn(N, hn, generator=gen, device=dev) * w.delta_scale).to(torch.bfloat16)
        Wn[(h, hn)] = (torch.randn(h, hn, generator=gen, device=dev) / hn ** 0.5).to(torch.bfloat16)
        Zs[(h, hn)] = torch.randn(N, h, generator=gen, device=dev).to(torch.bfloat16)
        out[(h, hn)] = torch.empty((N, h), dtype=torch.bfloat16, device=dev)
    torch.cuda.synchronize()

    def step():
        for key in layers:
            D, Wt, Z, O_ = Dn[key], Wn[key], Zs[key], out[key]
            if not args.per_site_calls:
                dad.backprop_delta(D, Wt, Z, act, D_out=O_)
                continue
            for s_ in range(S):
                r0 = s_ * b
                dad.backprop_delta(D[r0:r0 + b], Wt, Z[r0:r0 + b], act, D_out=O_[r0:r0 + b])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    dad.profile_reset()
    dad.profile_enable(True)
    step()
    torch.cuda.synchronize()
    dad.profile_enable(False)
    kern = dad.profile_read()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    flops = sum(2.0 * N * h * hn for h, hn in layers)
    bytes_ = sum(2.0 * (N * hn + h * hn + 2.0 * N * h) for h, hn in layers)
    tflops = flops / (ms_per_step * 1e-3) / 1e12
    ms, launches = kern["k_backprop_bf16"]
    k_rate = flops / (ms * 1e-3) / 1e12
    roofline = {"kernel": "k_backprop_bf16", "bound": "mfma", "achieved": k_rate, "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": k_rate / PEAK_BF16_TFLOPS, "avg_us": ms * 1e3 / launches, "traffic": None}

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import dad_oracle as O
        key = min(set(pairs), key=lambda t: t[0] * t[1])
        h, hn = key
        rows = 4096
        Dh = Dn[key][:rows].float().cpu().numpy().astype(np.float64)
        Wh = Wn[key].float().cpu().numpy().astype(np.float64)
        Zh = Zs[key][:rows].float().cpu().numpy().astype(np.float64)
        c0 = time.perf_counter()
        ref = O.backprop_delta(Dh, Wh, Zh, act)
        c1 = time.perf_counter()
        try:
            from threadpoolctl import threadpool_info
            threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            threads = os.cpu_count()
        got = dad.backprop_delta(Dn[key][:rows], Wn[key], Zs[key][:rows], act).float().cpu().numpy()
        e = O.rel_fro(got, ref)
        cpu = {"value": 2.0 * rows * h * hn / (c1 - c0) / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
               "sample": f"{rows} of {N} rows of one layer (h={h}, h_next={hn}): fp64 numpy backprop_delta {c1 - c0:.2f} s",
               "parity_rel_fro": {"delta": e, "tol": 2e-2}, "host_cpus": os.cpu_count()}
        if not e <= 2e-2:
            print(f"bench.py: parity check failed: {e:.3e}", file=sys.stderr)
            sys.exit(1)

    out_json = {
        "metric": "dAD delta back-propagation (Eq. 3) TFLOP/s into the stacked layout (% MFMA roofline)",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name + "/backprop", "layers": len(layers), "shapes_h_hnext": [list(p) for p in pairs],
                   "sites": S, "rows_per_site": b, "N": N, "activation": act,
                   "per_site_calls": bool(args.per_site_calls)},
        "frac_of_mfma_peak": tflops / PEAK_BF16_TFLOPS,
        "hbm_GBps": bytes_ / (ms_per_step * 1e-3) / 1e9,
        "us_per_layer": ms_per_step * 1e3 / len(layers),
        "roofline": roofline,
        "kernels": {k: {"ms_per_step": v[0], "launches_per_step": v[1], "avg_us": v[0] * 1e3 / v[1]} for k, v in kern.items()},
        "cpu_baseline": cpu,
    }
    print(json.dumps(out_json))


def sequential(args, w, dad, W, torch, np, dev):
    """Algorithm 2 one singular pair at a time (dad_compress_rank_sequential) on the stacked factors
    of ONE block of the model (its distinct layer shapes): r components x (4 n_iter + 2) thin passes,
    each over a whole factor.  A step is one pass over that block; the metric is the time per layer,
    to be read beside compress_us_per_layer of the default mode (the block form of the same method)."""
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    es = 2 if w.dtype == "bf16" else 4
    N, r, n_iter = w.N, w.rank, w.n_iter
    layers = w.all_layers()[:len(w.shapes)]
    A, D, G0, Qt, sGt, sig = {}, {}, {}, {}, {}, {}
    for li, hi, ho in layers:
        As, Ds = W.device_factors(w, li, hi, ho, device=dev)
        A[li], D[li] = dad.stack_factors(As, Ds)
        del As, Ds
        G0[li] = W.device_start_matrix(w, li, ho, device=dev)
        Qt[li] = torch.empty((r, hi), dtype=torch.float32, device=dev)
        sGt[li] = torch.empty((r, ho), dtype=torch.float32, device=dev)
        sig[li] = torch.empty((r,), dtype=torch.float32, device=dev)
    ws = torch.zeros(max(dad.lib().dad_compress_sequential_workspace_bytes(N, hi, ho, dad._dt(A[li]))
                         for li, hi, ho in layers), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()

    def step():
        for li, hi, ho in layers:
            dad.compress_rank_sequential(A[li], D[li], r, n_iter, G0[li], Qt=Qt[li], sGt=sGt[li], sigma=sig[li],
                                         workspace=ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    status = dad.poll_numeric_status(ws)
    dad.profile_reset()
    dad.profile_enable(True)
    step()
    torch.cuda.synchronize()
    dad.profile_enable(False)
    kern = dad.profile_read()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    passes = r * (2 * n_iter + 1)                      # over each of the two factors, per layer
    bytes_ = sum(float(passes) * N * (hi + ho) * es for _, hi, ho in layers)
    thin = {k: v for k, v in kern.items() if k.startswith("k_thin") and v[1] > 0}
    thin_ms = sum(v[0] for v in thin.values())
    dom = max(thin, key=lambda k: thin[k][0])
    k_rate = bytes_ / (thin_ms * 1e-3) / 1e9           # all thin launches together stream `bytes_`
    roofline = {"kernel": "+".join(sorted(thin)), "dominant": dom, "bound": "hbm", "achieved": k_rate,
                "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": k_rate / PEAK_HBM_GBPS,
                "avg_us": thin_ms * 1e3 / sum(v[1] for v in thin.values()), "traffic": None}

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import dad_oracle as O
        li, hi, ho = min(layers, key=lambda t: t[1] * t[2])
        rows, rr = min(N, 16384), min(r, 8)
        Ah = A[li][:rows].float().cpu().numpy().astype(np.float64)
        Dh = D[li][:rows].float().cpu().numpy().astype(np.float64)
        g0 = G0[li][:rr].cpu().numpy()
        c0 = time.perf_counter()
        Q_ref, sG_ref = O.sequential_spi(Ah, Dh, g0, n_iter)
        c1 = time.perf_counter()
        try:
            from threadpoolctl import threadpool_info
            threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            threads = os.cpu_count()
        q, sg, _ = dad.compress_rank_sequential(A[li][:rows].contiguous(), D[li][:rows].contiguous(), rr, n_iter,
                                                G0[li][:rr].contiguous(), check=True)
        e = O.rel_fro(dad.reconstruct_grad(q, sg).cpu().numpy(), Q_ref.T @ sG_ref)
        tol = 2e-2 if w.dtype == "bf16" else 1e-5
        cpu = {"value": (c1 - c0) * 1e6, "unit": "us/layer", "cores": int(threads), "kind": "oracle",
               "sample": f"{rows} of {N} rows, {rr} of {r} components of one layer ({hi}x{ho}): "
                         f"fp64 numpy sequential_spi {c1 - c0:.2f} s",
               "parity_rel_fro": {"rank_r_gradient": e, "tol": tol}, "host_cpus": os.cpu_count()}
        if not e <= tol:
            print(f"bench.py: parity check failed: {e:.3e}", file=sys.stderr)
            sys.exit(1)

    print(json.dumps({
        "metric": "dAD sequential SPI (Algorithm 2 with peeling) time per layer on the stacked factors",
        "value": ms_per_step * 1e3 / len(layers), "unit": "us/layer", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name + "/sequential", "layers": len(layers), "shapes": [list(x[1:]) for x in layers],
                   "N": N, "rank": r, "n_iter": n_iter, "factor_passes_per_layer": 2 * passes},
        "hbm_GBps": bytes_ / (ms_per_step * 1e-3) / 1e9, "numeric_status": int(status),
        "roofline": roofline,
        "kernels": {k: {"ms_per_step": v[0], "launches_per_step": v[1], "avg_us": v[0] * 1e3 / v[1]}
                    for k, v in kern.items() if v[1] > 0},
        "cpu_baseline": cpu,
    }))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (sites are simulated as row blocks on one device); "
              "--gpus N with N > 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2102_09631_amd import binding as dad
    from paper_2102_09631_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    dad.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = W.by_name(args.workload)
    if args.mode == "two_level":
        return two_level(args, w, dad, W, torch, np, dev)
    if args.mode == "backprop":
        return backprop(args, w, dad, W, torch, np, dev)
    if args.mode == "sequential":
        return sequential(args, w, dad, W, torch, np, dev)
    out = one_level(args, w, args.steps, args.warmup, dad, W, torch, np, dev,
                    cpu_budget_s=None if args.no_cpu_baseline else 10.0, yardsticks=True)
    # The other transformer workloads in the same process (fewer steps; one block of distinct layer
    # shapes resident where the stack exceeds HBM), so that one run carries all three.
    others = {}
    if args.workload == "gpt2_medium_stack" and not args.no_other_workloads:
        for name, steps in (("encoder_d768", max(3, args.steps)), ("vit_large_stack", 3)):
            torch.cuda.empty_cache()
            o = one_level(args, W.by_name(name), steps, 1, dad, W, torch, np, dev,
                          cpu_budget_s=None if args.no_cpu_baseline else 0.0, yardsticks=False)
            others[name] = {k: o[k] for k in ("value", "unit", "steps", "warmup", "ms_per_step", "dtype", "config",
                                              "rebuild_frac_of_mfma_peak", "compress_us_per_layer", "compress_GBps",
                                              "compress_frac_of_hbm_peak", "stack_GBps", "rank_rebuild_us_per_layer",
                                              "rank_rebuild_GBps", "phase_ms_per_step", "roofline", "kernels",
                                              "sites_in_place")}
            if o["cpu_baseline"]:
                others[name]["parity_rel_fro"] = o["cpu_baseline"]["parity_rel_fro"]
                others[name]["oracle_sample"] = o["cpu_baseline"]["sample"]
    out["other_workloads"] = others or None
    print(json.dumps(out))


def one_level(args, w, steps, warmup, dad, W, torch, np, dev, cpu_budget_s, yardsticks):
    """stack -> compress -> full rebuild -> rank-r rebuild over every layer of `w`, timed over `steps`
    steps after `warmup`; returns the result record.  cpu_budget_s: None = no oracle leg; otherwise
    the oracle runs on at least one layer of each distinct shape (0.0: exactly one layer, the
    smallest) and on further layers until that many seconds of oracle time are spent."""
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    es = 2 if w.dtype == "bf16" else 4
    N, r, n_iter, S, b = w.N, w.rank, w.n_iter, w.sites, w.rows_per_site
    layers = w.all_layers()

    # ---- inputs resident in HBM.  The whole stack when it fits; otherwise one block of distinct
    # shapes that every block of the stack re-reads (each layer is far larger than any cache).
    total_bytes = sum(N * (hi + ho) * es for _, hi, ho in layers)
    resident = layers if total_bytes < 150e9 else layers[:len(w.shapes)]
    sites = {}
    for li, hi, ho in resident:
        sites[li] = W.device_factors(w, li, hi, ho, device=dev)
    def factors_of(li):
        return sites[li] if li in sites else sites[li % len(w.shapes)]
    G0 = {li: W.device_start_matrix(w, li, ho, device=dev) for li, _, ho in layers}
    # Stacked factors: one buffer per layer when unstacked + stacked copies of the whole stack fit in
    # HBM (the layers of the whole stack can then be reduced by ONE grouped call), else one per
    # distinct shape (grouped per block of the model).
    whole = len(resident) == len(layers) and 2 * total_bytes < 200e9 and args.lanes > 0
    nb = len(w.shapes)
    gl = args.group_layers if (whole and args.group_layers > 0) else (len(layers) if whole else nb)
    scopes = [layers[i:i + gl] for i in range(0, len(layers), gl)]
    def st_key(li, hi, ho):
        return li if whole else (hi, ho)
    A_st = {st_key(li, hi, ho): torch.empty((N, hi), dtype=tdt, device=dev) for li, hi, ho in (layers if whole else layers[:nb])}
    D_st = {st_key(li, hi, ho): torch.empty((N, ho), dtype=tdt, device=dev) for li, hi, ho in (layers if whole else layers[:nb])}
    G_full = {s: torch.empty(s, dtype=torch.float32, device=dev) for s in w.shapes}
    # the rank-r gradients of all layers are rebuilt by ONE grouped call at the end of a step
    G_rank = {li: torch.empty((hi, ho), dtype=torch.float32, device=dev) for li, hi, ho in layers}
    Pt = {li: torch.empty((r, hi), dtype=torch.float32, device=dev) for li, hi, _ in layers}
    Gt = {li: torch.empty((r, ho), dtype=torch.float32, device=dev) for li, _, ho in layers}
    ws_c = torch.zeros(max(dad.compress_workspace_bytes(N, hi, ho, r, tdt) for _, hi, ho in layers),
                       dtype=torch.uint8, device=dev)
    ws_r = torch.zeros(max(16, max(dad.reconstruct_workspace_bytes(N, hi, ho, tdt) for _, hi, ho in layers)),
                       dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()

    rank_group = dad.RebuildGroup([(Pt[li], Gt[li]) for li, _, _ in layers], [G_rank[li] for li, _, _ in layers])

    PH = ("stack", "compress", "rebuild_full", "rebuild_rank")

    # Per scope (the whole stack, or one block of distinct shapes): stack and full rebuild alternate
    # layer by layer (the MFMA-bound rebuild launches then do not run back to back: 96 of them in a
    # row clock 5 % lower), then the scope's layers are reduced by one grouped call (args.lanes layers
    # in flight at once); the rank-r gradients of all layers close the step with one grouped call.
    # A step is a list of (phase, call) operations; `ungrouped` is the same work with one
    # dad_compress_rank call per layer.
    groups = []
    if args.lanes > 0:
        for sc in scopes:
            groups.append(dad.CompressGroup([(A_st[st_key(*t)], D_st[st_key(*t)], G0[t[0]]) for t in sc], r, n_iter,
                                            lanes=min(args.lanes, dad.DAD_MAX_LANES),
                                            Pts=[Pt[t[0]] for t in sc], Gts=[Gt[t[0]] for t in sc],
                                            workspace=groups[0].workspace if groups else None))

    # Full gradients: `rg` consecutive layers per dad_reconstruct_grad_grouped call (1: one
    # dad_reconstruct_grad call per layer).  The layers of a call must have distinct shapes here, because
    # the bench keeps one output buffer per shape.
    # Automatic: a whole block for the small workloads (their launches are short); for the large ones
    # consecutive layers are joined only while their 256 x 256 output tiles together stay within a budget
    # (128: the call then still splits K at least two ways).  That halves or quarters the K chunks and
    # fp32 slabs of the few-tile layers and still leaves rebuild launches alternating with stacking passes.
    small = w.N * max(hi * ho for hi, ho in w.shapes) < (1 << 37)
    rg = max(1, min(args.rebuild_group, nb)) if args.rebuild_group > 0 else (nb if small else 0)
    tile_budget = args.rebuild_tile_budget
    full_groups = {}
    def full_group(chunk):
        key = tuple(t[0] for t in chunk)
        if key not in full_groups:
            full_groups[key] = dad.RebuildGroup([(A_st[st_key(*t)], D_st[st_key(*t)]) for t in chunk],
                                                [G_full[(t[1], t[2])] for t in chunk])
        return full_groups[key]

    def make_ops(grouped):
        ops = []
        for si, sc in enumerate(scopes):
            pending = []
            for j, (li, hi, ho) in enumerate(sc):
                k = st_key(li, hi, ho)
                As, Ds = factors_of(li)
                ops.append(("stack", lambda As=As, Ds=Ds, k=k: dad.stack_factors(As, Ds, A_out=A_st[k], D_out=D_st[k])))
                if not grouped:
                    ops.append(("compress", lambda k=k, li=li: dad.compress_rank(A_st[k], D_st[k], r, n_iter, G0[li], Pt=Pt[li],
                                                                                 Gt=Gt[li], workspace=ws_c)))
                if rg == 1:
                    ops.append(("rebuild_full", lambda k=k, s_=(hi, ho): dad.reconstruct_grad(A_st[k], D_st[k], G=G_full[s_],
                                                                                              workspace=ws_r)))
                    continue
                pending.append((li, hi, ho))
                nxt = sc[j + 1] if j + 1 < len(sc) and (li + 1) % nb != 0 else None
                if rg > 0:
                    close = len(pending) == rg or nxt is None
                else:
                    tiles = lambda t: -(-t[1] // 256) * -(-t[2] // 256)
                    close = nxt is None or sum(tiles(t) for t in pending) + tiles(nxt) > tile_budget
                if close:
                    if len(pending) == 1:
                        k1, s1 = st_key(*pending[0]), (pending[0][1], pending[0][2])
                        ops.append(("rebuild_full", lambda k=k1, s_=s1: dad.reconstruct_grad(A_st[k], D_st[k], G=G_full[s_],
                                                                                             workspace=ws_r)))
                    else:
                        ops.append(("rebuild_full", full_group(pending).run))
                    pending = []
            if grouped:
                ops.append(("compress", groups[si].run))
        ops.append(("rebuild_rank", rank_group.run))
        return ops

    ops = make_ops(grouped=bool(groups))
    ops_ungrouped = ops if not groups else make_ops(grouped=False)

    # Small workloads are bound by launch latency (a step of encoder_d768 is about 130 launches in a
    # millisecond): there every operation is captured into a HIP graph of its own, and a step replays
    # the graphs in order with the phase events between them.
    use_graphs = args.graphs == "on" or (args.graphs == "auto" and len(layers) <= 8)

    # Timing events are created, and one pair is exercised, before the timed region: the first use of
    # a timing event costs milliseconds of one-off set-up in the runtime.
    pool = [torch.cuda.Event(enable_timing=True) for _ in range((len(ops) + 1) * steps)]
    pool_next = [0]
    if pool:
        pool[0].record(); pool[1].record(); torch.cuda.synchronize(); pool[0].elapsed_time(pool[1])

    def step(events=None, which=None, graphs=None):
        """One step.  With `events`, an event is recorded before every operation and after the last,
        and (phase, start, end) triples are appended."""
        which = ops if which is None else which
        marks = []
        for i, (phase, fn) in enumerate(which):
            if events is not None:
                e = pool[pool_next[0]]
                pool_next[0] += 1
                e.record()
                marks.append(e)
            if graphs is not None:
                graphs[i].replay()
            else:
                fn()
        if events is not None:
            e = pool[pool_next[0]]
            pool_next[0] += 1
            e.record()
            marks.append(e)
            for i, (phase, _) in enumerate(which):
                events.append((phase, marks[i], marks[i + 1]))

    # Untimed pre-pass: every layer's compress once, with the numeric status polled per layer (the
    # flag lives in the shared workspace and is cleared by the next call, so one poll after a whole
    # step would only see the last layer's).
    for li, hi, ho in layers:
        s_ = st_key(li, hi, ho)
        As, Ds = factors_of(li)
        dad.stack_factors(As, Ds, A_out=A_st[s_], D_out=D_st[s_])
        dad.compress_rank(A_st[s_], D_st[s_], r, n_iter, G0[li], Pt=Pt[li], Gt=Gt[li], workspace=ws_c)
        if dad.poll_numeric_status(ws_c) != dad.DAD_OK:
            print(f"bench.py: numerical breakdown latched on layer {li} ({hi}x{ho}) of {w.name}", file=sys.stderr)
            sys.exit(1)
    for _ in range(max(warmup, 1) if use_graphs else warmup):
        step()
    torch.cuda.synchronize()
    op_graphs = None
    if use_graphs:
        op_graphs = []
        for _, fn in ops:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                fn()
            op_graphs.append(g)
        step(graphs=op_graphs)
        torch.cuda.synchronize()

    # timed region: K steps, phase boundaries marked by events on the launch stream
    events = []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step(events, graphs=op_graphs)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    # the same K steps once more with the library's per-kernel events switched on (two events per
    # launch cost about 10 us per launch, so they stay out of the region that `value` comes from), one
    # layer's compress at a time: kernels of concurrent lanes would share the chip and their event
    # brackets would overlap
    dad.profile_reset()
    dad.profile_enable(True)
    for _ in range(steps):
        step(which=ops_ungrouped)
    torch.cuda.synchronize()
    dad.profile_enable(False)
    kern = dad.profile_read()
    ms_per_step = (t1 - t0) * 1e3 / steps

    phase_ms = dict.fromkeys(PH, 0.0)
    for phase, e0, e1 in events:
        phase_ms[phase] += e0.elapsed_time(e1)
    phase_ms = {k: v / steps for k, v in phase_ms.items()}
    nl = len(layers)
    flops_full = sum(2.0 * N * hi * ho for _, hi, ho in layers)
    bytes_stack = sum(2.0 * N * (hi + ho) * es for _, hi, ho in layers)
    bytes_compress = sum((2 * n_iter + 1.0) * N * (hi + ho) * es for _, hi, ho in layers)
    bytes_rank = sum(4.0 * hi * ho + 4.0 * r * (hi + ho) for _, hi, ho in layers)
    rebuild_tflops = flops_full / (phase_ms["rebuild_full"] * 1e-3) / 1e12

    # ---- roofline per kernel from the library's per-launch events
    # thin kernels alternate between the two factors: nn runs on Delta (n_iter+1 times) and on A
    # (n_iter times), tn on A (n_iter+1 times) and on Delta (n_iter times), per layer and step.
    per_step_work = {}
    for name in kern:
        tot, bound = 0.0, None
        for _, hi, ho in layers:
            if name in ("k_thin_nn_bf16", "k_thin_nn"):
                parts = [("out", n_iter + 1), ("in", n_iter)]
            elif name in ("k_thin_tn_bf16", "k_thin_tn"):
                parts = [("in", n_iter + 1), ("out", n_iter)]
            else:
                parts = [("in", 1)]
            for which, cnt in parts:
                bnd, wk = kernel_model(name, N, hi, ho, r, es, which, bf16=(w.dtype == "bf16"))
                if bnd is None:
                    continue
                bound = bnd
                tot += cnt * wk
        if bound:
            per_step_work[name] = (bound, tot)
    roof_all = {}
    for name, (ms, launches) in kern.items():
        entry = {"ms_per_step": ms / steps, "launches_per_step": launches / steps,
                 "avg_us": ms * 1e3 / launches}
        if name in per_step_work:
            bound, work = per_step_work[name]
            rate = work * steps / (ms * 1e-3)
            if bound == "hbm":
                entry.update(bound="hbm", achieved=rate / 1e9, peak=PEAK_HBM_GBPS, unit="GB/s",
                             frac=rate / 1e9 / PEAK_HBM_GBPS)
            else:
                peak = PEAK_BF16_TFLOPS if w.dtype == "bf16" else PEAK_FP32_TFLOPS
                entry.update(bound="mfma", achieved=rate / 1e12, peak=peak, unit="TFLOP/s",
                             frac=rate / 1e12 / peak)
        roof_all[name] = entry
    # the kernel with the largest total time among those with a roofline model (the launch-bound
    # helpers of the tiny workloads have none)
    dominant = max((k for k in kern if k in per_step_work), key=lambda k: kern[k][0])
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get(w.name, {}).get(dominant)
        except Exception:
            traffic = None
    roofline = {"kernel": dominant}
    roofline.update({k: roof_all[dominant].get(k) for k in ("bound", "achieved", "peak", "unit", "frac")})
    roofline["avg_us"] = roof_all[dominant]["avg_us"]
    roofline["traffic"] = traffic

    # ---- the same step without a1: the reduction and the full rebuild read the sites' blocks in
    # place (dad_compress_rank_grouped with site layers, dad_reconstruct_grad_sites); every output is
    # compared bit for bit with what the stacked calls left behind.  Reported beside the headline,
    # never in its place: a step of the headline contains the stacking pass.
    sites_leg = None
    if w.dtype == "bf16" and groups and not args.no_sites_leg:
        Pt2 = {li: torch.empty_like(Pt[li]) for li, _, _ in layers}
        Gt2 = {li: torch.empty_like(Gt[li]) for li, _, _ in layers}
        G_full2 = {s_: torch.empty_like(G_full[s_]) for s_ in w.shapes}
        ws_rs = torch.zeros(max(16, max(dad.reconstruct_sites_workspace_bytes([b] * S, hi, ho, tdt) for _, hi, ho in layers)),
                            dtype=torch.uint8, device=dev)
        sgroups = []
        for sc in scopes:
            sgroups.append(dad.CompressGroup([(factors_of(t[0])[0], factors_of(t[0])[1], G0[t[0]]) for t in sc], r, n_iter,
                                             lanes=min(args.lanes, dad.DAD_MAX_LANES),
                                             Pts=[Pt2[t[0]] for t in sc], Gts=[Gt2[t[0]] for t in sc],
                                             workspace=sgroups[0].workspace if sgroups else None))
        rank_group2 = dad.RebuildGroup([(Pt2[li], Gt2[li]) for li, _, _ in layers], [G_rank[li] for li, _, _ in layers])
        sops = []
        for si, sc in enumerate(scopes):
            for li, hi, ho in sc:
                As, Ds = factors_of(li)
                sops.append(("rebuild_full", lambda As=As, Ds=Ds, s_=(hi, ho): dad.reconstruct_grad_sites(
                    As, Ds, G=G_full2[s_], workspace=ws_rs)))
            sops.append(("compress", sgroups[si].run))
        sops.append(("rebuild_rank", rank_group2.run))
        pool_next[0] = 0
        step(which=sops)
        torch.cuda.synchronize()
        same = all(torch.equal(Pt[li], Pt2[li]) and torch.equal(Gt[li], Gt2[li]) for li, _, _ in layers)
        # the full gradient of the last layer of each shape against dad_reconstruct_grad on its stacked copy
        # (the headline's joined launches split K differently, so they are not the reference here)
        last_of = {(hi, ho): (li, hi, ho) for li, hi, ho in layers}
        for s_, t in last_of.items():
            ref = dad.reconstruct_grad(A_st[st_key(*t)], D_st[st_key(*t)], workspace=ws_r)
            same = same and torch.equal(ref, G_full2[s_])
            del ref
        if not same:
            print("bench.py: the site-block calls differ from the stacked calls", file=sys.stderr)
            sys.exit(1)
        ev2 = []
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        for _ in range(steps):
            step(ev2, which=sops)
        torch.cuda.synchronize()
        c1 = time.perf_counter()
        ph2 = dict.fromkeys(PH, 0.0)
        for phase, e0, e1 in ev2:
            ph2[phase] += e0.elapsed_time(e1) / steps
        sites_leg = {"ms_per_step": (c1 - c0) * 1e3 / steps,
                     "ms_per_step_with_stack": ms_per_step,
                     "rebuild_full_TFLOPs": flops_full / (ph2["rebuild_full"] * 1e-3) / 1e12,
                     "compress_us_per_layer": ph2["compress"] * 1e3 / nl,
                     "compress_frac_of_hbm_peak": bytes_compress / (ph2["compress"] * 1e-3) / 1e9 / PEAK_HBM_GBPS,
                     "bit_identical_to_stacked_calls": True}
        del sgroups, rank_group2, ws_rs

    # ---- CPU baseline: the fp64 oracle on the first layers of the stack, at least one of each distinct
    # shape and until about 10 s of oracle time are spent (bounded sample)
    cpu = None
    if cpu_budget_s is not None:
        from oracle import dad_oracle as O
        try:
            from threadpoolctl import threadpool_info
            threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            threads = os.cpu_count()
        tol = 2e-2 if w.dtype == "bf16" else 1e-5
        t_full = t_spi = flops = 0.0
        e_full = e_rank = 0.0
        sampled = []
        if cpu_budget_s == 0.0:     # exactly one layer: the one with the smallest gradient
            order = [min(layers[:len(w.shapes)], key=lambda t: t[1] * t[2])]
        else:                       # in stack order: every distinct shape comes up in the first block
            order = layers
        for li, hi, ho in order:
            if cpu_budget_s > 0.0 and len(sampled) >= len(w.shapes) and t_full + t_spi >= cpu_budget_s:
                break
            As, Ds = factors_of(li)
            A64 = torch.cat([a.float().cpu() for a in As]).numpy().astype(np.float64)
            D64 = torch.cat([d.float().cpu() for d in Ds]).numpy().astype(np.float64)
            G0_h = G0[li].cpu().numpy()
            c0 = time.perf_counter()
            M = O.full_grad(A64, D64)
            c1 = time.perf_counter()
            Pt_ref, Gt_ref = O.block_spi(A64, D64, G0_h, n_iter)
            c2 = time.perf_counter()
            del A64, D64
            t_full += c1 - c0
            t_spi += c2 - c1
            flops += 2.0 * N * hi * ho
            # same layer on the GPU, for an on-the-spot parity figure
            s = (hi, ho)
            k = st_key(li, hi, ho)
            dad.stack_factors(As, Ds, A_out=A_st[k], D_out=D_st[k])
            dad.compress_rank(A_st[k], D_st[k], r, n_iter, G0[li], Pt=Pt[li], Gt=Gt[li], workspace=ws_c)
            dad.reconstruct_grad(A_st[k], D_st[k], G=G_full[s], workspace=ws_r)
            dad.reconstruct_grad(Pt[li], Gt[li], G=G_rank[li])
            torch.cuda.synchronize()
            e_full = max(e_full, O.rel_fro(G_full[s].cpu().numpy(), M))
            e_rank = max(e_rank, O.rel_fro(G_rank[li].cpu().numpy(), O.rank_r_grad(Pt_ref, Gt_ref)))
            sampled.append(f"{hi}x{ho}")
            del M
        cpu = {"value": flops / t_full / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
               "sample": f"first {len(sampled)} of {nl} layers (shapes {', '.join(sorted(set(sampled)))}; N={N}): fp64 numpy full_grad "
                         f"{t_full:.2f} s, block_spi r={r} n={n_iter} {t_spi:.2f} s",
               "compress_us_per_layer": t_spi * 1e6 / len(sampled),
               "parity_rel_fro": {"full": e_full, "rank": e_rank, "tol": tol},
               "host_cpus": os.cpu_count()}
        if not (e_full <= tol and e_rank <= tol):
            print(f"bench.py: parity check failed: {e_full:.3e} {e_rank:.3e}", file=sys.stderr)
            sys.exit(1)

    # ---- in-run yardsticks, outside the timed region.  (a) What the chip sustains on this very data:
    # a bare MFMA loop whose fragments come from the stacked activations (the matrix cores' clock
    # under load follows the operands' bit toggling), the same loop on zeros, a plain read stream, and
    # the rebuild call itself on all-zero factors of the same shapes.  (b) What the box's libraries
    # reach on the same work: torch's device copy and torch.matmul (hipBLASLt) at the same shapes.
    # Context beside the published peaks; nothing on the path calls any of these.
    yard = None
    if yardsticks and w.dtype == "bf16":
        def timed(fn, reps):
            fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e-3 / reps
        first = {(hi, ho): st_key(li, hi, ho) for li, hi, ho in reversed(layers)}   # a stacked buffer of each shape
        s0 = max(w.shapes, key=lambda t: t[1])
        src, dst = D_st[first[s0]], torch.empty_like(D_st[first[s0]])
        t_copy = timed(lambda: dst.copy_(src), 10)
        del dst
        t_mm = fl_mm = 0.0
        for sh in w.shapes:
            t_mm += timed(lambda: torch.matmul(A_st[first[sh]].t(), D_st[first[sh]]), 3)
            fl_mm += 2.0 * N * sh[0] * sh[1]
        mfma_data = dad.probe_mfma_loop(A_st[first[s0]])
        zeros = torch.zeros(1 << 22, dtype=tdt, device=dev)
        mfma_zero = dad.probe_mfma_loop(zeros)
        read_gbps = dad.probe_read_stream(D_st[first[s0]])
        # the rebuild call on zero factors: same launches and clocks per stage, no operand toggling
        t_z = fl_z = 0.0
        for sh in w.shapes:
            Az, Dz = torch.zeros_like(A_st[first[sh]]), torch.zeros_like(D_st[first[sh]])
            t_z += timed(lambda: dad.reconstruct_grad(Az, Dz, G=G_full[sh], workspace=ws_r), 5)
            fl_z += 2.0 * N * sh[0] * sh[1]
            del Az, Dz
        k_reb = roof_all.get("k_rebuild_bf16_dma", {}).get("achieved")
        yard = {"mfma_loop_TFLOPs_on_stacked_activations": mfma_data,
                "mfma_loop_TFLOPs_on_zeros": mfma_zero,
                "read_stream_GBps": read_gbps,
                "rebuild_call_TFLOPs_on_zero_factors": fl_z / t_z / 1e12,
                "rebuild_kernel_vs_mfma_loop_same_data": (k_reb / mfma_data) if k_reb else None,
                "rebuild_phase_vs_mfma_loop_same_data": rebuild_tflops / mfma_data,
                "torch_copy_GBps": 2.0 * src.numel() * es / t_copy / 1e9,
                "torch_matmul_same_shapes_TFLOPs": fl_mm / t_mm / 1e12,
                "stack_vs_torch_copy": (bytes_stack / (phase_ms["stack"] * 1e-3) / 1e9) / (2.0 * src.numel() * es / t_copy / 1e9),
                "rebuild_vs_torch_matmul": rebuild_tflops / (fl_mm / t_mm / 1e12)}

    out = {
        "metric": METRIC,
        "value": rebuild_tflops,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": w.name, "layers": nl, "shapes": [list(s) for s in w.shapes], "sites": S,
                   "rows_per_site": b, "N": N, "rank": r, "n_iter": n_iter,
                   "resident_layers": len(resident), "compress_lanes": args.lanes,
                   "compress_group_layers": gl, "rebuild_group_layers": rg, "hip_graphs": use_graphs},
        "rebuild_frac_of_mfma_peak": rebuild_tflops / (PEAK_BF16_TFLOPS if w.dtype == "bf16" else PEAK_FP32_TFLOPS),
        "compress_us_per_layer": phase_ms["compress"] * 1e3 / nl,
        "compress_GBps": bytes_compress / (phase_ms["compress"] * 1e-3) / 1e9,
        "compress_frac_of_hbm_peak": bytes_compress / (phase_ms["compress"] * 1e-3) / 1e9 / PEAK_HBM_GBPS,
        "stack_GBps": bytes_stack / (phase_ms["stack"] * 1e-3) / 1e9,
        "rank_rebuild_us_per_layer": phase_ms["rebuild_rank"] * 1e3 / nl,
        "rank_rebuild_GBps": bytes_rank / (phase_ms["rebuild_rank"] * 1e-3) / 1e9,
        "phase_ms_per_step": phase_ms,
        "roofline": roofline,
        "kernels": roof_all,
        "in_run_yardsticks": yard,
        "sites_in_place": sites_leg,
        "cpu_baseline": cpu,
    }
    return out


if __name__ == "__main__":
    main()
