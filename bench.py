#!/usr/bin/env python3
"""Benchmark of the SpecPV verification path on one MI355X.

Metric (the benchmark spec): partial-verify attention microseconds per verify step at
128K context, LLaMA-3.1-8B attention shape, plus achieved HBM GB/s.

One step = the partial-verification attention of a 60-node draft tree over the
4096-token partial KV cache (1 sink + 55 retrieval + 8 local blocks of 64 tokens),
for all 32 layers one after another, each layer with its own seeded K/V, queries
and kept-block list.  The block lists come from an untimed full-verify refresh
(summaries -> scores -> top-k), as in the paper's schedule where selection happens
only on refresh steps.  Inputs are synthetic and resident in HBM before timing.

Prints ONE JSON line.  Extra keys: "roofline", "cpu_baseline", "extras".
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# RECORDED, not live: HBM bytes per specpv_partial_verify_attn call from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# (KiB per dispatch, FETCH scaled by 2.0 as a plain device copy calibrates it), and the per-kernel durations of a
# rocprofv3 --kernel-trace --stats run, as committed under profiles/.  They describe the launch plan named here
# (kernels and split count); the line carries them only while the library still plans the call that way.
RECORDED = {"llama8b_128k": {
    "plan": {"kernels": ["attn_ctx_mfma_kernel", "combine_kernel"], "splits": 8},
    "traffic_bytes": (8663 + 2419) * 2 * 1024 + (3960 + 480) * 1024,
    "traffic_source": "profiles/pmc_traffic_llama8b_128k.md",
    "kernels": [{"name": "attn_ctx_mfma_kernel", "us": 12.5}, {"name": "combine_kernel", "us": 4.8}],
    "kernels_source": "profiles/kernel_durations_llama8b_128k.md"}}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="llama8b_128k")
    ap.add_argument("--layers", type=int, default=None, help="override the number of layers (default: the workload's)")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true")
    ap.add_argument("--no-offload", action="store_true", help="skip the host-offload leg of the extras (2 GiB of pinned memory)")
    ap.add_argument("--no-batch", action="store_true", help="skip the 16-sequence leg of the extras (4 GiB of K / V)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--settle", type=float, default=0.3,
                    help="seconds of untimed replays during set-up, before the W warm-up steps, to bring the box to its working clocks")
    ap.add_argument("--route", type=int, default=0,
                    help="specpv_debug_set_route value for the partial-verify attention (0: the library's choice; 2: one kernel)")
    ap.add_argument("--copy-calib", action="store_true",
                    help="also run 4 plain device copies of 256 MiB (read 256 MiB + write 256 MiB each) so that "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings can be scaled by a kernel of known traffic")
    return ap.parse_args()


def algorithmic_bytes_per_layer(case):
    """Bytes one layer's partial-verify attention must move: the kept K and V blocks,
    the draft tokens' K/V, the queries and the outputs (bf16 = 2 bytes)."""
    sz = 2 if case["dtype"] == "bf16" else 4
    kv = 0
    for b in range(case["batch"]):
        nb = (int(case["ctx_len"][b]) + case["B"] - 1) // case["B"]
        kv += min(case["n_sel"], nb) * case["B"] * case["Hkv"] * case["D"] * 2 * sz
    M, Hq, Hkv, D, batch = case["M"], case["Hq"], case["Hkv"], case["D"], case["batch"]
    draft = batch * M * Hkv * D * 2 * sz
    qo = batch * M * Hq * D * 2 * sz
    return kv + draft + qo, kv


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import workloads
    import paper_2512_02337_amd as specpv
    specpv.load()   # raises if the HIP library is missing: there is no fallback
    specpv.specpv_debug_set_route(args.route)
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = workloads.CONFIGS[args.workload]
    n_layers = args.layers or cfg["layers"]

    # ---- build every layer's inputs on the device, then the untimed refresh ----------
    layers = []
    t0 = time.time()
    for layer in range(n_layers):
        case = workloads.make_case(args.workload, seed=args.seed, layer=layer, device=dev)
        kv = specpv.KV(case["k"], case["v"], case["ctx_len"], case["B"], case["max_blocks"])
        tree = specpv.Tree(case["q"], case["kd"], case["vd"], case["parent"])
        scfg = specpv.SelectCfg(case["ns"], case["nr"], case["k_blocks"], "mean")
        shp = kv.summary_shape()
        st = dict(case=case, kv=kv, tree=tree, cfg=scfg,
                  kmax=torch.empty(shp, dtype=case["q"].dtype, device=dev),
                  kmin=torch.empty(shp, dtype=case["q"].dtype, device=dev),
                  sel_idx=torch.empty((case["batch"], case["Hkv"], scfg.n_sel), dtype=torch.int32, device=dev),
                  sel_count=torch.empty((case["batch"], case["Hkv"]), dtype=torch.int32, device=dev),
                  out=torch.empty_like(case["q"]),
                  out_full=torch.empty_like(case["q"]))
        layers.append(st)
    ws_bytes = max(specpv.specpv_workspace_bytes(l["kv"], l["tree"], l["cfg"]) for l in layers)
    ws = torch.zeros((ws_bytes,), dtype=torch.uint8, device=dev)   # zero-filled once: the arrival words
    for l in layers:   # untimed: the refresh that produces the kept-block lists
        specpv.specpv_full_verify_refresh(l["kv"], l["tree"], l["kmax"], l["kmin"], 0, l["cfg"], l["out_full"], None,
                                          l["sel_idx"], l["sel_count"], None, ws)
    torch.cuda.synchronize()
    setup_s = time.time() - t0

    def partial_step():
        for l in layers:
            specpv.specpv_partial_verify_attn(l["kv"], l["tree"], l["sel_idx"], l["sel_count"], l["out"], None, ws)

    def select_attend_step():
        for l in layers:
            specpv.specpv_select_blocks(l["kv"], l["tree"], l["kmax"], l["kmin"], l["cfg"], l["sel_idx"],
                                        l["sel_count"], None, ws)
            specpv.specpv_partial_verify_attn(l["kv"], l["tree"], l["sel_idx"], l["sel_count"], l["out"], None, ws)

    def refresh_step():
        for l in layers:
            specpv.specpv_full_verify_refresh(l["kv"], l["tree"], l["kmax"], l["kmin"], -1, l["cfg"], l["out_full"],
                                              None, l["sel_idx"], l["sel_count"], None, ws)

    def timed(fn, steps, warmup, graph, per_step=None, settle_s=0.0):
        """ms per step over `steps` steps, after `warmup` untimed ones, with HIP events on
        the stream the library launches on."""
        stream = torch.cuda.Stream()
        stream.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(stream):
            run = fn
            if graph:
                fn()
                stream.synchronize()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=stream):
                    fn()
                run = g.replay
            if settle_s > 0:
                # part of the set-up, not of the W warm-up steps: a fresh box needs a few hundred milliseconds of
                # load before its clocks and the graph's first replays have settled (20 steps right after 5
                # warm-up steps otherwise read about 4 % slower than every later step)
                t_end = time.time() + settle_s
                while time.time() < t_end:
                    for _ in range(20):
                        run()
                    stream.synchronize()
            for _ in range(warmup):
                run()
            stream.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record(stream)
            for _ in range(steps):
                run()
            e1.record(stream)
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / steps
            if per_step is not None:
                # a second pass with an event between the steps: median and minimum of single steps
                ev = [torch.cuda.Event(enable_timing=True) for _ in range(per_step + 1)]
                ev[0].record(stream)
                for i in range(per_step):
                    run()
                    ev[i + 1].record(stream)
                torch.cuda.synchronize()
                each = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(per_step))
                timed.last_per_step = {"n": per_step, "median_us": round(each[len(each) // 2] * 1e3, 2),
                                       "min_us": round(each[0] * 1e3, 2), "max_us": round(each[-1] * 1e3, 2)}
            return ms

    if args.copy_calib:
        src = torch.empty((256 << 20,), dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    use_graph = not args.no_graph
    ms = timed(partial_step, args.steps, args.warmup, use_graph, per_step=max(100, args.steps), settle_s=args.settle)
    per_step_stats = timed.last_per_step
    us_step = ms * 1e3
    bytes_layer, kv_bytes_layer = algorithmic_bytes_per_layer(layers[0]["case"])
    us_layer = us_step / n_layers
    achieved = bytes_layer / (us_layer * 1e-6) / 1e9

    extras = {}
    if not args.no_extras:
        k2 = max(3, args.steps // 10)
        extras["partial_eager_us_per_step"] = round(timed(partial_step, k2, 3, False) * 1e3, 2)
        extras["select_plus_attend_us_per_step"] = round(timed(select_attend_step, k2, 3, use_graph) * 1e3, 2)
        rf = timed(refresh_step, max(2, k2 // 4), 1, use_graph) * 1e3
        extras["full_verify_refresh_us_per_step"] = round(rf, 2)
        c0 = layers[0]["case"]
        full_bytes = sum(int(x) for x in c0["ctx_len"]) * c0["Hkv"] * c0["D"] * 2 * 2
        extras["full_verify_refresh_kv_GBs"] = round(full_bytes * n_layers / (rf * 1e-6) / 1e9, 1)
        # buffer commit after a partial step (Section 3.2: accepted candidates stay pending, the rest
        # is dropped): 4 accepted tokens per layer into a 28-token buffer
        c0 = layers[0]["case"]
        P, Mt = 28, c0["M"]
        cb = {"k": torch.zeros((c0["batch"], P + Mt, c0["Hkv"], c0["D"]), dtype=c0["q"].dtype, device=dev),
              "n_pending": torch.zeros((c0["batch"],), dtype=torch.int32, device=dev),
              "accepted": torch.tensor([[0, 1, 2, 3]] * c0["batch"], dtype=torch.int32, device=dev),
              "n_accepted": torch.full((c0["batch"],), 4, dtype=torch.int32, device=dev)}
        cb["v"] = torch.zeros_like(cb["k"])

        def commit_step():
            for l in layers:
                specpv.specpv_commit_accepted(l["kv"], cb["k"], cb["v"], P, Mt, cb["n_pending"], cb["accepted"],
                                              cb["n_accepted"], specpv.MODE_PARTIAL, None, None, ws)
        extras["commit_partial_us_per_step"] = round(timed(commit_step, k2, 3, use_graph) * 1e3, 2)
        # ... and the same through the call that commits every layer of the model at once (one buffer
        # per layer, the counters shared)
        bufs_k = [torch.zeros_like(cb["k"]) for _ in layers]
        bufs_v = [torch.zeros_like(cb["k"]) for _ in layers]
        shared_kvs = [specpv.KV(l["kv"].k, l["kv"].v, layers[0]["kv"].ctx_len, c0["B"], c0["max_blocks"]) for l in layers]

        def commit_all_step():
            specpv.specpv_commit_accepted_layers(shared_kvs, bufs_k, bufs_v, P, Mt, cb["n_pending"], cb["accepted"],
                                                 cb["n_accepted"], specpv.MODE_PARTIAL, None, None, ws)
        extras["commit_partial_all_layers_us_per_step"] = round(timed(commit_all_step, k2, 3, use_graph) * 1e3, 2)
        # the paper's physically gathered partial cache (Section 3.2) against reading the blocks in
        # place: one gather per layer, and the partial step over the gathered segments
        g = []
        for l in layers:
            c = l["case"]
            gk = torch.empty((c["batch"], c["Hkv"], c["n_sel"] * c["B"], c["D"]), dtype=c["q"].dtype, device=dev)
            gv = torch.empty_like(gk)
            glen = torch.zeros((c["batch"],), dtype=torch.int32, device=dev)
            specpv.specpv_gather_blocks(l["kv"], l["sel_idx"], l["sel_count"], gk, gv, glen)
            g.append({"k": gk, "v": gv, "len": glen, "kv": specpv.KV(gk, gv, glen, c["B"], c["n_sel"])})

        def gather_step():
            for l, x in zip(layers, g):
                specpv.specpv_gather_blocks(l["kv"], l["sel_idx"], l["sel_count"], x["k"], x["v"], x["len"])

        def gathered_partial_step():
            for l, x in zip(layers, g):
                specpv.specpv_partial_verify_attn(x["kv"], l["tree"], None, None, l["out"], None, ws)
        extras["gather_us_per_step"] = round(timed(gather_step, k2, 3, use_graph) * 1e3, 2)
        extras["partial_on_gathered_us_per_step"] = round(timed(gathered_partial_step, k2, 3, use_graph) * 1e3, 2)
        # Section 3.3's offload: the full cache of 4 layers in pinned host memory, two device slots,
        # the next layer copied in while the current one runs its full verification + refresh + gather
        # of the new partial cache (PCIe-bound: reported per layer, with the host-to-device rate)
        if n_layers >= 4 and not args.no_offload:
            from paper_2512_02337_amd.offload import LayerPrefetcher
            sub = layers[:4]
            hk = [l["kv"].k.cpu().pin_memory() for l in sub]
            hv = [l["kv"].v.cpu().pin_memory() for l in sub]
            pf = LayerPrefetcher(hk, hv, slots=2)
            staged = []
            for i in range(2):
                c = sub[i]["case"]
                staged.append(specpv.KV(pf.dev_k[i], pf.dev_v[i], c["ctx_len"], c["B"], c["max_blocks"]))

            def offload_pass():
                pf.prefetch(0)
                for i, (l, x) in enumerate(zip(sub, g)):
                    if i + 1 < len(sub):
                        pf.prefetch(i + 1)
                    pf.acquire(i)
                    kv = staged[i % 2]
                    specpv.specpv_full_verify_refresh(kv, l["tree"], l["kmax"], l["kmin"], -1, l["cfg"], l["out_full"],
                                                      None, l["sel_idx"], l["sel_count"], None, ws)
                    specpv.specpv_gather_blocks(kv, l["sel_idx"], l["sel_count"], x["k"], x["v"], x["len"])
                    pf.release(i)
            offload_pass()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(2):
                offload_pass()
            e1.record()
            torch.cuda.synchronize()
            per_layer_ms = e0.elapsed_time(e1) / (2 * len(sub))
            extras["offload_full_refresh_us_per_layer"] = round(per_layer_ms * 1e3, 1)
            extras["offload_h2d_GBs"] = round((hk[0].numel() + hv[0].numel()) * hk[0].element_size() / (per_layer_ms * 1e-3) / 1e9, 1)
            del pf, hk, hv, staged
        # the same partial step as a throughput problem: 16 sequences of this shape with 32K of context
        # each in ONE call per layer (two layers' inputs in turn: 4 GiB of K / V, kept blocks scattered)
        if args.workload == "llama8b_128k" and not args.no_batch:
            bcfg = dict(cfg)
            bcfg.update(ctx=[32768] * 16, rho=[0.05] * 16, layers=1, name="llama8b_batch16_32k")
            bsets = []
            for layer in range(2):
                bc = workloads.make_case(bcfg, seed=args.seed, layer=layer, device=dev)
                bkv = specpv.KV(bc["k"], bc["v"], bc["ctx_len"], bc["B"], bc["max_blocks"])
                btree = specpv.Tree(bc["q"], bc["kd"], bc["vd"], bc["parent"])
                bscfg = specpv.SelectCfg(bc["ns"], bc["nr"], bc["k_blocks"], "mean")
                bkmax = torch.empty(bkv.summary_shape(), dtype=bc["q"].dtype, device=dev)
                bkmin = torch.empty_like(bkmax)
                bsel = torch.empty((bc["batch"], bc["Hkv"], bscfg.n_sel), dtype=torch.int32, device=dev)
                bcnt = torch.empty((bc["batch"], bc["Hkv"]), dtype=torch.int32, device=dev)
                bws = torch.zeros((specpv.specpv_workspace_bytes(bkv, btree, bscfg),), dtype=torch.uint8, device=dev)
                specpv.specpv_block_summarize(bkv, 0, -1, bkmax, bkmin)
                specpv.specpv_select_blocks(bkv, btree, bkmax, bkmin, bscfg, bsel, bcnt, None, bws)
                bsets.append((bc, bkv, btree, bsel, bcnt, torch.empty_like(bc["q"]), bws))

            def batched_partial_step():
                for (_, bkv, btree, bsel, bcnt, bout, bws) in bsets:
                    specpv.specpv_partial_verify_attn(bkv, btree, bsel, bcnt, bout, None, bws)
            bus = timed(batched_partial_step, k2, 3, use_graph) * 1e3 / len(bsets)
            bbytes, _ = algorithmic_bytes_per_layer(bsets[0][0])
            extras["batch16_32k_partial_us_per_call"] = round(bus, 2)
            extras["batch16_32k_partial_GBs"] = round(bbytes / (bus * 1e-6) / 1e9, 1)
            del bsets
        # Section 3.2's buffer on a partial step: 16 partially verified tokens wait in front of the 60
        # candidates.  They are keys only (no query rows), so the step costs what it costs without them
        # plus 16 more draft K / V rows in the tree segment.
        if args.workload == "llama8b_128k":
            import numpy as np
            n_pend = 16
            pl = []
            for l in layers:
                c = l["case"]
                g = torch.Generator(device=dev).manual_seed(1234)
                pk = torch.randn((c["batch"], n_pend, c["Hkv"], c["D"]), generator=g, device=dev).to(c["q"].dtype)
                pv = torch.randn((c["batch"], n_pend, c["Hkv"], c["D"]), generator=g, device=dev).to(c["q"].dtype)
                par = specpv.specpv_extend_parents(c["parent"][0].tolist(), n_pend)
                ptree = specpv.Tree(c["q"], torch.cat([pk, c["kd"]], 1).contiguous(), torch.cat([pv, c["vd"]], 1).contiguous(),
                                    torch.tensor([par] * c["batch"], dtype=torch.int32, device=dev))
                pl.append(ptree)

            pout = torch.empty_like(layers[0]["out"])

            def pending_step():
                for l, ptree in zip(layers, pl):
                    specpv.specpv_partial_verify_attn(l["kv"], ptree, l["sel_idx"], l["sel_count"], pout, None, ws)
            extras["partial_16_pending_us_per_step"] = round(timed(pending_step, k2, 3, use_graph) * 1e3, 2)
            del pl
        # the Qwen3-14B-shaped ragged batch (40 / 8 heads, G = 5, contexts 32K + 64K + 96K + 128K): one layer's
        # partial step and one layer's full verification + refresh, per call
        if args.workload == "llama8b_128k" and not args.no_batch:
            rc = workloads.make_case("qwen14b_batch4", seed=args.seed, device=dev)
            rkv = specpv.KV(rc["k"], rc["v"], rc["ctx_len"], rc["B"], rc["max_blocks"])
            rtree = specpv.Tree(rc["q"], rc["kd"], rc["vd"], rc["parent"])
            rcfg = specpv.SelectCfg(rc["ns"], rc["nr"], rc["k_blocks"], "mean")
            rkmax = torch.empty(rkv.summary_shape(), dtype=rc["q"].dtype, device=dev)
            rkmin = torch.empty_like(rkmax)
            rsel = torch.empty((rc["batch"], rc["Hkv"], rcfg.n_sel), dtype=torch.int32, device=dev)
            rcnt = torch.empty((rc["batch"], rc["Hkv"]), dtype=torch.int32, device=dev)
            rout = torch.empty_like(rc["q"])
            rws = torch.zeros((specpv.specpv_workspace_bytes(rkv, rtree, rcfg),), dtype=torch.uint8, device=dev)
            specpv.specpv_full_verify_refresh(rkv, rtree, rkmax, rkmin, 0, rcfg, rout, None, rsel, rcnt, None, rws)
            rp = timed(lambda: specpv.specpv_partial_verify_attn(rkv, rtree, rsel, rcnt, rout, None, rws), k2, 3, use_graph) * 1e3
            rf2 = timed(lambda: specpv.specpv_full_verify_refresh(rkv, rtree, rkmax, rkmin, -1, rcfg, rout, None, rsel, rcnt,
                                                                   None, rws), max(3, k2 // 4), 1, use_graph) * 1e3
            rs = timed(lambda: specpv.specpv_select_blocks(rkv, rtree, rkmax, rkmin, rcfg, rsel, rcnt, None, rws), k2, 3, use_graph) * 1e3
            rbytes, _ = algorithmic_bytes_per_layer(rc)
            rfull = sum(int(x) for x in rc["ctx_len"]) * rc["Hkv"] * rc["D"] * 2 * 2
            extras["qwen14b_batch4_partial_us_per_call"] = round(rp, 2)
            extras["qwen14b_batch4_partial_GBs"] = round(rbytes / (rp * 1e-6) / 1e9, 1)
            extras["qwen14b_batch4_full_refresh_us_per_call"] = round(rf2, 2)
            extras["qwen14b_batch4_full_refresh_kv_GBs"] = round(rfull / (rf2 * 1e-6) / 1e9, 1)
            extras["qwen14b_batch4_select_us_per_call"] = round(rs, 2)
            del rc, rkv, rtree, rkmax, rkmin, rws
        # what this machine's HBM delivers to plain streaming kernels, next to the published peak: a device
        # copy of 1 GiB (read + write bytes), and the library's own read-only stream (eq. 1 over one
        # layer's K, rotating over the layers so that the 256 MB last-level cache cannot serve it)
        src = torch.empty((1 << 30,), dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        cp = timed(lambda: dst.copy_(src), 10, 2, False)
        extras["hbm_copy_ceiling_GBs"] = round(2 * src.numel() / (cp * 1e-3) / 1e9, 1)
        del src, dst

        def summarize_all():
            for l in layers:
                specpv.specpv_block_summarize(l["kv"], 0, -1, l["kmax"], l["kmin"])
        sm = timed(summarize_all, 5, 1, False)
        k_bytes = sum(int(x) for x in c0["ctx_len"]) * c0["Hkv"] * c0["D"] * 2
        extras["hbm_read_stream_GBs"] = round(k_bytes * n_layers / (sm * 1e-3) / 1e9, 1)
        extras["setup_s"] = round(setup_s, 1)

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(layers)

    # the recorded counter / trace figures only describe the launch plan they were taken with: 8 context splits
    # (read off the workspace size: 64 KiB of arrival words + (splits + 1) x (partial O + (m, l) pairs) + scores)
    rec = RECORDED.get(args.workload) if n_layers == cfg["layers"] else None
    if rec is not None:
        c0 = layers[0]["case"]
        up = lambda x: (x + 255) & ~255
        rows = c0["batch"] * c0["Hq"] * c0["M"]
        part_only = specpv.specpv_workspace_bytes(specpv.KV(c0["k"][:, :, :c0["n_sel"] * c0["B"]], c0["v"][:, :, :c0["n_sel"] * c0["B"]],
                                                            c0["ctx_len"], c0["B"], c0["n_sel"]), layers[0]["tree"])
        if part_only != 65536 + up(rows * (rec["plan"]["splits"] + 1) * c0["D"] * 4) + up(rows * (rec["plan"]["splits"] + 1) * 8) + \
                up(c0["batch"] * c0["Hkv"] * c0["n_sel"] * 4):
            rec = None   # the planner has moved on: the recorded figures no longer describe this build

    line = {
        "metric": "partial_verify_attention_us_per_step",
        "value": round(us_step, 2),
        "unit": "us/step",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms, 5),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": layers[0]["case"]["dtype"],
        "data": "synthetic",
        "config": {"workload": args.workload, "layers": n_layers, "context": [int(x) for x in layers[0]["case"]["ctx_len"]],
                   "block": layers[0]["case"]["B"], "kept_blocks": layers[0]["case"]["n_sel"], "tree_nodes": layers[0]["case"]["M"],
                   "q_heads": layers[0]["case"]["Hq"], "kv_heads": layers[0]["case"]["Hkv"], "head_dim": layers[0]["case"]["D"],
                   "launch": "hip_graph" if use_graph else "eager", "settle_s_before_warmup": args.settle, "route": args.route},
        "achieved_hbm_GBs": round(achieved, 1),
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": rec["traffic_bytes"] if rec else None,
                     "traffic_is": "recorded (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, %s), not measured by this run" % rec["traffic_source"] if rec else None,
                     "kernel": "context attention (attn_ctx_mfma_kernel at the default workload; the planner picks by shape) + combine_kernel = one specpv_partial_verify_attn call (one layer)",
                     "kernels": [dict(k, frac=round(bytes_layer / (k["us"] * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                                      source="recorded: " + rec["kernels_source"]) for k in rec["kernels"]] if rec else None,
                     "algorithmic_bytes_per_launch": bytes_layer, "us_per_launch": round(us_layer, 3),
                     "us_per_step_single_replays": per_step_stats,
                     "box_copy_GBs": extras.get("hbm_copy_ceiling_GBs"), "box_read_stream_GBs": extras.get("hbm_read_stream_GBs")},
        "cpu_baseline": cpu,
        "extras": extras,
    }
    print(json.dumps(line))


def cpu_baseline(layers):
    """The fp64 oracle, as it stands (built -O3 -march=native for this leg, same source, no fast-math), on the
    host's cores: the attention-only partial step over every layer of the same workload (one whole step,
    about ten seconds of CPU work), then the full verification of ONE layer at the full context (a bounded
    sample: the whole step would be 32 times that), and the CPU's full / partial ratio per layer -- the
    paper's premise that verification cost follows the attended tokens (Section 3.2, Figure 1)."""
    import numpy as np
    import torch
    import oracle
    oracle.use_native_build()
    total, err0 = 0.0, None
    for li, layer in enumerate(layers):
        case = layer["case"]
        B, Hkv = case["B"], case["Hkv"]
        idx = layer["sel_idx"][0].cpu().numpy()
        cnt = layer["sel_count"][0].cpu().numpy()
        n = int(cnt.max())
        # hand the oracle only the kept blocks (per KV head, renumbered 0..n-1): attention
        # does not depend on where a block sits, so this is the same computation
        blocks = torch.from_numpy(idx[:, :n].astype(np.int64)).to(case["k"].device)          # [Hkv, n]
        tok = (blocks[:, :, None] * B + torch.arange(B, device=blocks.device)[None, None]).reshape(Hkv, n * B)
        K = torch.gather(case["k"][0], 1, tok[:, :, None].expand(-1, -1, case["D"])).permute(1, 0, 2).contiguous().cpu()
        V = torch.gather(case["v"][0], 1, tok[:, :, None].expand(-1, -1, case["D"])).permute(1, 0, 2).contiguous().cpu()
        Q, Kd, Vd = case["q"][0].cpu(), case["kd"][0].cpu(), case["vd"][0].cpu()
        parent = case["parent"][0].cpu().numpy()
        t0 = time.time()
        O, _, _ = oracle.tree_attention(Q, K, V, Kd, Vd, parent, B)
        total += time.time() - t0
        if li == 0:
            err0 = float(np.abs(layer["out"][0].float().cpu().numpy() - O).max())
    # full verification of layer 0 over the whole context
    case = layers[0]["case"]
    L = int(case["ctx_len"][0])
    K = case["k"][0, :, :L].permute(1, 0, 2).contiguous().cpu()
    V = case["v"][0, :, :L].permute(1, 0, 2).contiguous().cpu()
    t0 = time.time()
    Of, _, _ = oracle.tree_attention(case["q"][0].cpu(), K, V, case["kd"][0].cpu(), case["vd"][0].cpu(),
                                     case["parent"][0].cpu().numpy(), case["B"])
    full_s = time.time() - t0
    errf = float(np.abs(layers[0]["out_full"][0].float().cpu().numpy() - Of).max())
    partial_layer_s = total / len(layers)
    return {"value": round(total * 1e6, 1), "unit": "us/step", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "one whole step: partial-verify attention of all %d layers, fp64, %.2f s; full verification: one "
                      "layer at %d tokens, %.2f s" % (len(layers), total, L, full_s),
            "build": "gcc -O3 -march=native -fopenmp (the parity tests use -O2 generic; same source)",
            "full_verification_us_per_layer": round(full_s * 1e6, 1),
            "partial_verification_us_per_layer": round(partial_layer_s * 1e6, 1),
            "full_over_partial": round(full_s / partial_layer_s, 2),
            "attended_tokens_full_over_partial": round((L + case["M"]) / (case["n_sel"] * case["B"] + case["M"]), 2),
            "gpu_vs_oracle_max_abs_err_layer0": round(err0, 6),
            "gpu_vs_oracle_max_abs_err_full_layer0": round(errf, 6)}


if __name__ == "__main__":
    main()
