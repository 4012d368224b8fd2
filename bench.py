#!/usr/bin/env python3
"""Benchmark of the embed-and-aggregate path on one MI355X.

A step is one pass of the whole path over one synthetic workload whose inputs
already sit in HBM: CSR construction from the raw pair list, plan creation,
then every round (dense transform + neighbourhood aggregation) and the final
classifier transform.  The headline value is the edge*feature arithmetic of
all aggregations in the pass (2 flop per CSR entry and feature column) divided
by the wall time of the whole step.

Prints one JSON line.  Extra objects:
  roofline      the dominant kernel (the widest aggregation) against the 8 TB/s HBM peak
  cpu_baseline  the CPU oracle timed on a bounded sample of the same workload
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM bytes per launch of the dominant aggregation measured with rocprofv3 --pmc
# (FETCH_SIZE and WRITE_SIZE runs, scaled by a copy kernel of known size); see profiles/.
MEASURED_TRAFFIC_BYTES = {
    "sage_large_powerlaw": 108037992371,     # profiles/bench_sage_large_powerlaw.md
    "gat_products_powerlaw": 133628371786,   # profiles/bench_gat_products_powerlaw.md
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=3, help="workload index (0-4; 3 = Reddit-shaped, 4 = ogbn-products-shaped)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--cpu-rows", type=int, default=0, help="rows in the oracle sample (0 = per-workload default)")
    ap.add_argument("--option", action="append", default=[], metavar="NAME=VALUE",
                    help="set a tuning knob of the library (retexo_set_option) before running, for experiments")
    ap.add_argument("--probe", action="store_true",
                    help="for rocprofv3 --pmc runs: one pass, then one 1 GiB device copy (the known-size "
                         "reference for the byte counters) and one launch of the dominant aggregation; no JSON")
    return ap.parse_args()


def algorithmic_bytes(n, nnz, F, concat, gat_heads=0):
    """Bytes one aggregation must move in the gather model: one F-float row per
    CSR entry, the index arrays, the output, and the self copy if concatenated."""
    b = 4 * nnz * F + 4 * nnz + 8 * (n + 1) + 4 * n * F
    if concat:
        b += 2 * 4 * n * F           # read z_v, write it into the self half
    if gat_heads:
        b += 4 * nnz * gat_heads + 8 * n * gat_heads
    return b


def cpu_baseline(w, src, dst, feats, params, n_rows):
    """Oracle cost per unit on a bounded sample, scaled to one whole pass."""
    import oracle
    from paper_2302_13053_amd import workloads as wl
    n = w.n_nodes
    t0 = time.perf_counter()
    m = min(src.size, 4_000_000)
    oracle.csr_from_coo(src[:m], dst[:m], n, w.self_loops)
    t_csr = (time.perf_counter() - t0) * (src.size / max(m, 1))
    rp, ci = oracle.csr_from_coo(src, dst, n, w.self_loops)     # needed to run the sample; not timed
    rng = np.random.Generator(np.random.Philox(key=12345))
    rows = np.sort(rng.choice(n, size=min(n_rows, n), replace=False)).astype(np.int64)
    nnz = int(rp[-1])
    sample_edges = int((rp[rows + 1] - rp[rows]).sum())
    total = t_csr
    spent = 0.0
    for i, st in enumerate(w.stages):
        p = params[i]
        if i == 0:
            H = feats
        else:
            H = wl.random_matrix(n, st.d_in, 100 + i, ld=wl.pad_ld(st.d_in))
        if st.w:
            t0 = time.perf_counter()
            oracle.transform(H, st.d_in, p.W, p.b, st.relu, rows=rows)
            dt = time.perf_counter() - t0
            spent += dt
            total += dt * n / rows.size
        if st.kind == "round":
            Z = H if not st.w else wl.random_matrix(n, st.d_out, 200 + i, ld=wl.pad_ld(st.d_out))
            t0 = time.perf_counter()
            oracle.aggregate(st.mode, rp, ci, Z, st.d_out, heads=st.heads, a_src=p.a_src, a_dst=p.a_dst,
                             self_concat=st.concat, rows=rows)
            dt = time.perf_counter() - t0
            spent += dt
            total += dt * nnz / max(sample_edges, 1)
    flops = sum(2.0 * nnz * st.d_out for st in w.stages if st.kind == "round")
    return {
        "value": flops / total / 1e9,
        "unit": "GFLOP/s (edge*feature, whole pass)",
        "cores": oracle.threads(),
        "kind": "oracle",
        "sample": "%d random rows of every stage (%d CSR entries) plus CSR build of the first %d pairs, "
                  "%.1f s of oracle time, scaled per row / per entry / per pair to one whole pass"
                  % (rows.size, sample_edges, m, spent),
        "estimated_pass_seconds": total,
    }


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2302_13053_amd import binding as B
    from paper_2302_13053_amd import harness as Hn
    from paper_2302_13053_amd import workloads as wl

    B.load()
    for item in args.option:
        name, _, value = item.partition("=")
        B.check(B.retexo_set_option(name, int(value)), "retexo_set_option(%s)" % item)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)

    w = wl.workload(args.config)
    t0 = time.perf_counter()
    src, dst = wl.make_graph(w)
    feats = wl.make_features(w, ld=wl.pad_ld(w.feat_dim))
    params = wl.make_params(w)
    t_gen = time.perf_counter() - t0

    pipe = Hn.Pipeline(w, src, dst, feats, params)
    if args.probe:
        pipe.run()
        torch.cuda.synchronize()
        ref_src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        ref_dst = torch.empty_like(ref_src)
        torch.cuda.synchronize()
        ref_dst.copy_(ref_src)                       # 1 GiB read + 1 GiB written
        torch.cuda.synchronize()
        di = max((i for i, st in enumerate(w.stages) if st.kind == "round"),
                 key=lambda i: w.stages[i].d_out)
        st = w.stages[di]
        Zin = pipe.H0 if not st.w else torch.empty((w.n_nodes, wl.pad_ld(st.d_out)), dtype=torch.float32,
                                                   device="cuda").normal_()
        _, _, a_s, a_d = pipe.params[di]
        Hn.aggregate(pipe.graph, st.mode, Zin, st.d_out, heads=st.heads, a_src=a_s, a_dst=a_d, concat=st.concat)
        torch.cuda.synchronize()
        print("probe done: copy of %d bytes each way, then stage %d aggregation (F=%d)"
              % (ref_src.numel() * 4, di, st.d_out))
        pipe.close()
        return
    for _ in range(args.warmup):
        pipe.run()
    torch.cuda.synchronize()

    events = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        pipe.run(events=events)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps

    n, nnz = w.n_nodes, pipe.graph.nnz
    # per-step-kind mean over the timed steps, from events on the launch stream
    per = {}
    for label, a, b in events:
        per.setdefault(label, []).append(a.elapsed_time(b))
    stages = []
    flops = 0.0
    dominant = None
    for i, st in enumerate(w.stages):
        label = "%s%d" % (st.kind, i)
        ms = float(np.mean(per[label]))
        rec = {"stage": label, "ms": ms, "d_in": st.d_in, "d_out": st.d_out}
        if st.kind == "round":
            ef = float(nnz) * st.d_out
            flops += 2.0 * ef
            rec["mode"] = st.mode
            rec["edge_features"] = ef
            rec["identity_transform"] = not st.w
            if not st.w:
                gb = algorithmic_bytes(n, nnz, st.d_out, st.concat, st.heads if st.mode == "gat_softmax" else 0)
                rec["agg_effective_GBs"] = gb / ms / 1e6
            if dominant is None or ef > dominant[1]:
                dominant = (i, ef)
        if st.w:
            rec["transform_gflop"] = 2.0 * n * st.d_in * st.d_out / 1e9
        stages.append(rec)

    # roofline of the dominant aggregation: time it alone (aggregate call only) on the launch stream
    di = dominant[0]
    dst_stage = w.stages[di]
    gat = dst_stage.mode == "gat_softmax"
    F = dst_stage.d_out
    if dst_stage.w:
        # the aggregation's input is the transform's output; a resident random matrix of that shape stands in
        Zin = torch.empty((n, wl.pad_ld(F)), dtype=torch.float32, device="cuda").normal_()
    else:
        Zin = pipe.H0 if di == 0 else pipe.outs[di - 1]
    W_, b_, a_s, a_d = pipe.params[di]
    agg_out = torch.empty((n, wl.pad_ld(dst_stage.out_width)), dtype=torch.float32, device="cuda")
    ws = Hn.ws_tensor(B.retexo_workspace_bytes(pipe.graph.plan, F, B.MODES[dst_stage.mode], dst_stage.heads,
                                               B.F_SELF_CONCAT if dst_stage.concat else 0))
    reps = max(3, args.steps)
    Hn.aggregate(pipe.graph, dst_stage.mode, Zin, F, heads=dst_stage.heads, a_src=a_s, a_dst=a_d,
                 concat=dst_stage.concat, out=agg_out, workspace=ws)
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        Hn.aggregate(pipe.graph, dst_stage.mode, Zin, F, heads=dst_stage.heads, a_src=a_s, a_dst=a_d,
                     concat=dst_stage.concat, out=agg_out, workspace=ws)
    e1.record()
    torch.cuda.synchronize()
    agg_ms = e0.elapsed_time(e1) / reps
    gbytes = algorithmic_bytes(n, nnz, F, dst_stage.concat, dst_stage.heads if gat else 0)
    achieved = gbytes / agg_ms / 1e6
    roofline = {
        "bound": "hbm",
        "kernel": ("agg_gat_flash_kernel (wave per row, eight waves per long row; scores formed from the gathered "
                   "rows; other head widths: gat_scores_kernel + agg_gat_fast_kernel with a score table)"
                   if gat else
                   "aggregation call = agg_rowgroup_kernel + agg_grouped_kernel per source range (narrow slabs) "
                   "or agg_linear_kernel (whole rows), chosen by the plan"),
        "stage": "round%d aggregation, F=%d" % (di, F),
        "achieved": achieved,
        "peak": HBM_PEAK_GBS,
        "unit": "GB/s",
        "frac": achieved / HBM_PEAK_GBS,
        "traffic": MEASURED_TRAFFIC_BYTES.get(w.name),
        "algorithmic_bytes": gbytes,
        "ms_per_launch": agg_ms,
        "edge_features_per_s": float(nnz) * F / (agg_ms * 1e-3),
    }

    out = {
        "metric": "aggregated edge*feature GFLOP/s per lazy-MP pass (whole path: CSR build, plan, all rounds)",
        "value": flops / (ms_per_step * 1e-3) / 1e9,
        "unit": "GFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic (seeded %s graph, %s)" % (w.graph, w.stands_in_for),
        "config": {"workload": w.name, "config_index": w.index, "family": w.family, "nodes": n,
                   "raw_pairs": int(src.size), "csr_entries": int(nnz),
                   "max_degree": B.retexo_plan_max_degree(pipe.graph.plan), "feat_dim": w.feat_dim,
                   "stages": [st.kind + ":" + (st.mode if st.kind == "round" else "dense") +
                              ":%d->%d" % (st.d_in, st.d_out) for st in w.stages]},
        "csr_plan_ms": float(np.mean(per["csr+plan"])),
        "stages": stages,
        "input_generation_s": t_gen,
        "roofline": roofline,
    }
    # the row after the hot path: one local training step (loss + gradients + SGD update) of the first
    # trained layer with its temporary classifier, on the aggregated features that are already resident
    hidden = next((i for i, st in enumerate(w.stages) if st.kind == "round" and st.w and st.mode != "gat_softmax"),
                  None)
    if hidden is not None:
        st = w.stages[hidden]
        n_cls = w.stages[-1].d_out
        X = pipe.outs[hidden - 1] if hidden > 0 else pipe.H0
        g = torch.Generator(device="cuda").manual_seed(1234)
        labels = torch.randint(0, n_cls, (n,), generator=g, device="cuda", dtype=torch.int32)
        labels[torch.rand(n, generator=g, device="cuda") > 0.66] = -1       # two thirds are training nodes
        W1, b1 = pipe.params[hidden][0].clone(), pipe.params[hidden][1].clone()
        Wc = torch.empty((st.d_out, n_cls), dtype=torch.float32, device="cuda").uniform_(-0.1, 0.1, generator=g)
        bc = torch.zeros(n_cls, dtype=torch.float32, device="cuda")
        tws = Hn.ws_tensor(B.retexo_train_workspace_bytes(n, st.d_in, st.d_out, n_cls))

        def train_once():
            loss, *grads = Hn.layer_grad(X, st.d_in, labels, W1, b1, Wc, bc, workspace=tws)
            for p_, g_ in zip((W1, b1, Wc, bc), grads):
                B.check(B.retexo_sgd_update(p_.numel(), p_.data_ptr(), g_.data_ptr(), 0.01, Hn._stream_ptr()),
                        "retexo_sgd_update")
            return loss
        l0 = float(train_once().cpu()[0])
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            last = train_once()
        e1.record()
        torch.cuda.synchronize()
        tms = e0.elapsed_time(e1) / reps
        tfl = (4.0 * n * st.d_in * st.d_out + 6.0 * n * st.d_out * n_cls) / tms / 1e9
        out["train_step"] = {"layer": "%d->%d (ReLU) + classifier %d->%d" % (st.d_in, st.d_out, st.d_out, n_cls),
                             "ms": tms, "TFLOP/s": tfl, "frac_fp32_mfma": tfl / 157.3,
                             "loss_first": l0, "loss_last": float(last.cpu()[0]), "sgd_steps": reps + 1}
        # the same step with dropout 0.5 on the hidden units (a fresh mask per step)
        draw = [0]

        def train_dropout_once():
            draw[0] += 1
            loss, *grads = Hn.layer_grad(X, st.d_in, labels, W1, b1, Wc, bc, workspace=tws,
                                         dropout=(0.5, 20230213, draw[0]))
            for p_, g_ in zip((W1, b1, Wc, bc), grads):
                B.check(B.retexo_sgd_update(p_.numel(), p_.data_ptr(), g_.data_ptr(), 0.01, Hn._stream_ptr()),
                        "retexo_sgd_update")
        train_dropout_once()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            train_dropout_once()
        e1.record()
        torch.cuda.synchronize()
        out["train_step"]["ms_with_dropout"] = e0.elapsed_time(e1) / reps
    # a layer whose aggregation has trainable parameters (edge softmax) trains with the aggregation in the
    # loop: time its backward (dL/dZ and the attention-vector gradients) on the first such round's shape
    att = next((i for i, st in enumerate(w.stages) if st.kind == "round" and st.mode == "gat_softmax"
                and st.d_out <= 1024), None)
    if att is not None:
        st = w.stages[att]
        Fz, width = st.d_out, pipe.outs[att].shape[1]
        Zb = pipe.outs[att]                               # stands in for the round's transformed features
        Gb = torch.empty_like(Zb).normal_(generator=torch.Generator(device="cuda").manual_seed(4321))
        a_s, a_d = pipe.params[att][2], pipe.params[att][3]
        dZb = torch.empty_like(Zb)
        bws = Hn.ws_tensor(B.retexo_aggregate_backward_workspace_bytes(pipe.graph.plan, B.MODES[st.mode], Fz, st.heads))

        def backward_once():
            return Hn.aggregate_backward(pipe.graph, st.mode, Fz, Gb, Z=Zb, heads=st.heads, a_src=a_s, a_dst=a_d,
                                         dZ=dZb, workspace=bws)
        backward_once()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            backward_once()
        e1.record()
        torch.cuda.synchronize()
        bms = e0.elapsed_time(e1) / reps
        gbs = 2.0 * nnz * Fz * 4 / bms / 1e6              # two gather passes, one row of F floats per entry each
        out["aggregate_backward"] = {"shape": "%s F=%d heads=%d ld=%d" % (st.mode, Fz, st.heads, width), "ms": bms,
                                     "GB/s_algorithmic": gbs, "frac_hbm": gbs / 8000.0}
        # in a training loop: the forward in save mode, then the backward that reuses what it kept (one gather pass)
        try:
            sws = Hn.ws_tensor(B.retexo_workspace_bytes(pipe.graph.plan, Fz, B.MODES[st.mode], st.heads, B.F_SAVE))
            fout = torch.empty_like(Zb)

            def forward_save():
                Hn.aggregate(pipe.graph, st.mode, Zb, Fz, heads=st.heads, a_src=a_s, a_dst=a_d, out=fout,
                             workspace=sws, save=True)

            def backward_saved():
                Hn.aggregate_backward(pipe.graph, st.mode, Fz, Gb, Z=Zb, heads=st.heads, a_src=a_s, a_dst=a_d,
                                      dZ=dZb, workspace=bws, saved=sws)
            times = []
            for fn in (forward_save, backward_saved):
                fn()
                torch.cuda.synchronize()
                e0.record()
                for _ in range(reps):
                    fn()
                e1.record()
                torch.cuda.synchronize()
                times.append(e0.elapsed_time(e1) / reps)
            out["aggregate_backward"].update({"forward_save_mode_ms": times[0], "backward_after_save_ms": times[1],
                                              "GB/s_algorithmic_after_save": nnz * Fz * 4 / times[1] / 1e6})
        except B.RetexoError:
            pass                                           # layout without save mode: the plain backward stands
    # variant: the dominant aggregation over a table in 16-bit storage (half the gathered bytes; the stored value
    # is the float32 value rounded to nearest even, sums stay in float32)
    try:
        Z16 = Hn.store_rows(Zin, F, "bf16")               # the table the roofline figure above was measured on
        kw16 = dict(heads=dst_stage.heads, a_src=pipe.params[di][2], a_dst=pipe.params[di][3]) if gat else {}
        run16 = lambda: Hn.aggregate_stored(pipe.graph, dst_stage.mode, Z16, F, "bf16", concat=dst_stage.concat,
                                            out=agg_out, workspace=ws, **kw16)
        run16()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            run16()
        e1.record()
        torch.cuda.synchronize()
        ms16 = e0.elapsed_time(e1) / reps
        out["stored_aggregation"] = {"storage": "bf16", "stage": roofline["stage"], "ms": ms16,
                                     "fp32_ms": roofline["ms_per_launch"],
                                     "GB/s_algorithmic": nnz * F * 2 / ms16 / 1e6}
        del Z16
    except B.RetexoError:
        pass
    # the partition-shaped run: one worker's share of this graph (seeded random ownership over 4 workers for
    # the dense graph, 2 for the large sparse one, as the paper distributes them) and the pack / unpack of all
    # its boundary rows at the first round's width
    if w.index in (3, 4):
        n_workers = 4 if w.index == 3 else 2
        owner = torch.from_numpy(np.random.Generator(np.random.Philox(key=70 + w.index))
                                 .integers(0, n_workers, n).astype(np.int32)).cuda()
        share = Hn.partition_share(pipe.graph, owner, n_workers, 0)             # size query + real call
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            share = Hn.partition_share(pipe.graph, owner, n_workers, 0)
        torch.cuda.synchronize()
        share_ms = (time.perf_counter() - t0) / reps * 1e3
        Fp = w.stages[0].d_out
        table = pipe.outs[0][:share.n_inner + share.n_halo]                      # any resident table of that width
        buf = Hn.halo_pack(share.recv_ids, table, Fp)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            Hn.halo_pack(share.recv_ids, table, Fp, buf=buf)
            Hn.halo_unpack(share.recv_ids, buf, table, Fp)
        e1.record()
        torch.cuda.synchronize()
        pu_ms = e0.elapsed_time(e1) / reps
        out["partition"] = {"workers": n_workers, "inner": share.n_inner, "boundary": share.n_halo,
                            "local_entries": share.graph.nnz, "share_ms_incl_size_query_and_allocation": share_ms,
                            "pack_plus_unpack_ms": pu_ms, "rows": share.n_halo, "width": Fp,
                            "GB/s_read_plus_write": 4.0 * share.n_halo * Fp * 4 / pu_ms / 1e6}
    pipe.close()
    if not args.no_cpu:
        default_rows = w.n_nodes      # the oracle is fast enough to run every row of every stage in 10-30 s
        out["cpu_baseline"] = cpu_baseline(w, src, dst, feats, params, args.cpu_rows or default_rows)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
