"""Where the time of one partial-verify attention kernel goes: in-kernel time stamps.

    python -m paper_2512_02337_amd.build --timeline          # on the build machine: libspecpv_timeline.so
    python -m paper_2512_02337_amd.timeline [--route N]       # on the GPU

The instrumented library is the product's source compiled with -DSPECPV_TIMELINE: thread 0 of every
workgroup of the attention kernel stores the 100 MHz real-time counter at the points named below.  The
script runs the 32-layer partial-verify step of the headline workload (the launch configuration that
bench.py times, eager launches) and prints, per point, the median over workgroups and repetitions of
the time since the kernel's first workgroup entered.  Only the later layers of a step are read, where
kernels follow each other back to back.  It also prints the core clock that the workgroups saw.

    python -m paper_2512_02337_amd.timeline --full

measures the attention kernel of the full verification instead: core clock, lifetime and core cycles per
32-token chunk of its workgroups.
"""
import argparse
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
os.environ.setdefault("SPECPV_LIB", os.path.join(HERE, "libspecpv_timeline.so"))   # before the binding is imported; another instrumented build can be named
sys.path.insert(0, os.path.dirname(HERE))

import numpy as np   # noqa: E402
import torch   # noqa: E402

import paper_2512_02337_amd as sp   # noqa: E402
import workloads   # noqa: E402

POINTS = ["entry", "arguments, lengths, list ids, query rows in", "first chunks requested (one kernel: draft rows done)",
          "chunk 0 landed", "chunk 1 landed", "chunk 2 landed", "chunk 3 landed", "chunk loop done",
          "partials stored (issued)", "two kernels: lengths and list length in (scalar reads) | one kernel: stores acknowledged", "one kernel: arrival known",
          "one kernel: merged and stored (last workgroup of a tile)",
          "wavefront 0 starts to wait for chunk 0", "... for chunk 1 (done with chunk 0)", "... for chunk 2", "... for chunk 3"]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--route", type=int, default=0, help="specpv_debug_set_route value (0/1 two kernels, 2/3 one kernel)")
    ap.add_argument("--workload", default="llama8b_128k")
    ap.add_argument("--layers", type=int, default=8)
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--pending", type=int, default=0, help="partially verified tokens in front of the tree (keys only)")
    ap.add_argument("--full", action="store_true",
                    help="measure the full verification (attention over the whole cache) instead: per workgroup of its attention "
                         "kernel the core clock (s_memtime against the 100 MHz counter), the time and the cycles per 32-token chunk")
    a = ap.parse_args()
    if not os.path.exists(os.environ["SPECPV_LIB"]):
        raise SystemExit("build the instrumented library first: python -m paper_2512_02337_amd.build --timeline")
    sp.specpv_debug_set_route(a.route)
    dev = torch.device("cuda")
    layers = []
    for layer in range(a.layers):
        case = workloads.make_case(a.workload, seed=0, layer=layer, device=dev)
        kv = sp.KV(case["k"], case["v"], case["ctx_len"], case["B"], case["max_blocks"])
        tree = sp.Tree(case["q"], case["kd"], case["vd"], case["parent"])
        ptree = tree
        if a.pending > 0:   # the partial step then attends a chain of `pending` key-only nodes as well
            g = torch.Generator(device=dev).manual_seed(1234)
            shp = (case["k"].shape[0], a.pending, case["k"].shape[1], case["q"].shape[-1])
            pk = torch.randn(shp, generator=g, device=dev).to(case["q"].dtype)
            pv = torch.randn(shp, generator=g, device=dev).to(case["q"].dtype)
            par = [sp.specpv_extend_parents(case["parent"][b].tolist(), a.pending) for b in range(case["k"].shape[0])]
            ptree = sp.Tree(case["q"], torch.cat([pk, case["kd"]], 1).contiguous(), torch.cat([pv, case["vd"]], 1).contiguous(),
                            torch.tensor(par, dtype=torch.int32, device=dev))
        cfg = sp.SelectCfg(case["ns"], case["nr"], case["k_blocks"], "mean")
        batch, hkv = case["k"].shape[0], case["k"].shape[1]
        st = dict(kv=kv, tree=tree, ptree=ptree, cfg=cfg, kmax=torch.empty(kv.summary_shape(), dtype=case["q"].dtype, device=dev),
                  sel_idx=torch.empty((batch, hkv, cfg.n_sel), dtype=torch.int32, device=dev),
                  sel_count=torch.empty((batch, hkv), dtype=torch.int32, device=dev), out=torch.empty_like(case["q"]))
        st["kmin"] = torch.empty_like(st["kmax"])
        layers.append(st)
    ws = torch.zeros((max(sp.specpv_workspace_bytes(l["kv"], l["tree"], l["cfg"]) for l in layers),), dtype=torch.uint8, device=dev)
    for l in layers:   # builds the kept lists
        sp.specpv_full_verify_refresh(l["kv"], l["tree"], l["kmax"], l["kmin"], 0, l["cfg"], l["out"], None, l["sel_idx"], l["sel_count"], None, ws)
    torch.cuda.synchronize()
    max_wg = 4096
    tl = torch.zeros((len(layers), max_wg, 16), dtype=torch.int64, device=dev)

    def clock_lines(rows, what):
        """rows [n, >= 3]: core cycles, 10 ns ticks, chunks of one workgroup each"""
        rows = rows[rows[:, 1] > 0]
        if rows.shape[0] == 0:
            return
        mhz = rows[:, 0] / rows[:, 1] * 100.0
        print("%s: %d workgroups; core clock %.0f MHz (median; %.0f .. %.0f); a workgroup lives %.1f us (median)"
              % (what, rows.shape[0], np.median(mhz), mhz.min(), mhz.max(), np.median(rows[:, 1]) / 100.0))
        return rows

    if a.full:
        print("full verification, workload %s, %d layers per step" % (a.workload, len(layers)))
        for rep in range(a.reps):
            tl.zero_()
            for i, l in enumerate(layers):
                sp.specpv_debug_set_timeline(tl[i] if rep >= 2 else None)
                sp.specpv_full_verify_refresh(l["kv"], l["tree"], l["kmax"], l["kmin"], -1, l["cfg"], l["out"], None, l["sel_idx"], l["sel_count"], None, ws)
            torch.cuda.synchronize()
            if rep >= 2:
                x = tl[:, :2048].reshape(-1, 16).cpu().numpy().astype(np.float64)
                rows = clock_lines(x, "step %d, attention kernel" % rep)
                if rows is not None:
                    print("    %d chunks per workgroup, %.0f core cycles per chunk (median)" % (rows[0, 2], np.median(rows[:, 0] / rows[:, 2])))
        sp.specpv_debug_set_timeline(None)
        return

    def step(record):
        for i, l in enumerate(layers):
            sp.specpv_debug_set_timeline(tl[i] if record else None)
            sp.specpv_partial_verify_attn(l["kv"], l["ptree"], l["sel_idx"], l["sel_count"], l["out"], None, ws)

    for _ in range(5):
        step(False)
    res, cres = [], []
    for _ in range(a.reps):
        tl.zero_()
        step(True)
        torch.cuda.synchronize()
        for x in tl[len(layers) // 2:].cpu().numpy().astype(np.float64):
            xa, xc = x[:2048], x[2048:3072]   # attention kernel's workgroups, combine kernel's (rows from 3072: clock readings)
            xa = xa[xa[:, 0] > 0]   # workgroups that ran
            t0 = xa[:, 0].min()
            res.append(np.where(xa > 0, (xa - t0) / 100.0, np.nan))   # microseconds
            xc = xc[xc[:, 0] > 0]
            if xc.shape[0]:
                cres.append(np.where(xc > 0, (xc - t0) / 100.0, np.nan))
    clock_lines(tl[len(layers) // 2:, 3072:].reshape(-1, 16).cpu().numpy().astype(np.float64), "attention kernel, last repetition")
    sp.specpv_debug_set_timeline(None)
    n_wg = res[0].shape[0]
    res = np.stack([r for r in res if r.shape[0] == n_wg])
    print("workload %s, route %d, %d pending tokens, %d workgroups per launch, %d launches read" % (a.workload, a.route, a.pending, n_wg, res.shape[0]))
    print("microseconds since the first workgroup's entry: median over workgroups and launches, 10th / 90th percentile")
    for i, name in enumerate(POINTS):
        col = res[:, :, i]
        if np.all(np.isnan(col)):
            continue
        print("%2d %-58s %6.2f   %6.2f  %6.2f" % (i, name, np.nanmedian(col), np.nanpercentile(col, 10), np.nanpercentile(col, 90)))
    print("last stamp of a launch, median over launches: %.2f" % np.median(np.nanmax(res, axis=(1, 2))))
    if cres:
        cr = np.stack([r for r in cres if r.shape[0] == cres[0].shape[0]])
        print("combine kernel, %d workgroups per launch: microseconds since the ATTENTION kernel's first workgroup entered" % cr.shape[1])
        for i, name in enumerate(["entry", "parents in, root path walked", "context partials in and merged",
                                  "draft K / V rows in, tree segment done", "stored (issued)"]):
            col = cr[:, :, i]
            if np.all(np.isnan(col)):
                continue
            print("%2d %-58s %6.2f   %6.2f  %6.2f" % (i, name, np.nanmedian(col), np.nanpercentile(col, 10), np.nanpercentile(col, 90)))
        print("last stamp of the combine, median over launches: %.2f" % np.median(np.nanmax(cr, axis=(1, 2))))


if __name__ == "__main__":
    main()
