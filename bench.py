#!/usr/bin/env python3
"""Stage throughput of one zero-bubble pipeline stage on one MI355X.

A step is one whole iteration of the hot path: gradient zeroing, all 3m passes of the workload's
ZB-H1 / ZB-H2 order (zb_run_schedule) and, for workloads that have one, the post-validated AdamW
step.  Inputs (parameters, all m seeded activations and upstream gradients) are resident in HBM
before the timed region.  value = Table-1 model FLOPs (L*m*sbh(72h+12s), no causal discount) per
second.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
PEAK_FP32_TFLOPS = 157.3    # fp32 vector
PEAK_HBM_GBS = 8000.0


def cpu_baseline(w):
    """The oracle, as it stands, timed on the host cores on a bounded sample of the same workload:
    ONE microbatch's F + B + W through all layers of the stage (1/m of the step's passes, no optimizer)."""
    import zb_inputs
    from oracle.stage import StageOracle
    from oracle.schedule import F, B, W
    orc = StageOracle(layers=w.layers, hidden=w.hidden, heads=w.heads, ffn=w.ffn, seq=w.seq, mb_size=w.mb_size,
                      dtype=w.dtype, params=zb_inputs.stage_params(w))
    orc.begin_iteration(1)
    orc.set_input(0, zb_inputs.stage_input(w, 0, 0))
    orc.set_upstream_grad(0, zb_inputs.upstream_grad(w, 0, 0))
    t0 = time.perf_counter()
    orc.run([(F, 0), (B, 0), (W, 0)])
    dt = time.perf_counter() - t0
    s, b, h = w.seq, w.mb_size, w.hidden
    flops = w.layers * s * b * h * (72 * h + 12 * s)
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count() or 1
    for var in ("OPENBLAS_NUM_THREADS", "OMP_NUM_THREADS"):
        if os.environ.get(var, "").isdigit():
            cores = min(cores, int(os.environ[var]))
            break
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "seconds": round(dt, 3),
            "sample": f"numpy fp64 oracle, 1 of the {w.m} microbatches: F+B+W through the {w.layers} layers of "
                      f"{w.name} ({flops / 1e12:.2f} TFLOP of the step's {w.m * flops / 1e12:.0f})"}


def measured_traffic(workload):
    """HBM bytes per GEMM launch from the rocprofv3 counter runs summarised under profiles/ (FETCH_SIZE and
    WRITE_SIZE, each scaled by its reading for a plain copy of known size); None if no summary is there."""
    path = os.path.join(ROOT, "profiles", f"gemm_hbm_traffic_{workload}.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch"):
                return float(line.split("=")[1])
    except OSError:
        pass
    return None


XGMI_LINK_GBS = 153.0   # one xGMI link, the path of a stage-to-stage activation (design figure, not measured here)


def auto_schedule_report(zb, st, w, m, class_ms):
    """Sec. 3.1's automatic scheduler fed with this stage's measured pass times: T_F, T_B, T_W are the
    event-timed kernel classes of one step divided by m, T_comm is one [tokens, h] activation over one xGMI
    link, the memory model is the stage's real stash.  Bubble rates are those of a p-stage pipeline made of
    p copies of this stage (Sec. 5.3's definition), for the handcrafted orders and for the search under the
    memory of 1F1B (p M_B) and twice that."""
    t_f = (class_ms.get("gemm_fwd", 0) + class_ms.get("attention_fwd", 0) + class_ms.get("layernorm_fwd", 0)) / m
    t_b = (class_ms.get("gemm_dgrad", 0) + class_ms.get("attention_bwd", 0) + class_ms.get("layernorm_bwd", 0)) / m
    t_w = (class_ms.get("gemm_wgrad", 0) + class_ms.get("bias_grad_colsum", 0)) / m
    elem = 2 if w.dtype == "bf16" else 4
    t_comm = w.seq * w.mb_size * w.hidden * elem / (XGMI_LINK_GBS * 1e9) * 1e3
    m_b, m_w = st.stash_bytes()
    p = w.p
    rates = {}
    for kind in ("1F1B", "H1", "H2"):
        orders = [zb.schedule_order(p, i, m, kind) for i in range(p)]
        rates["1F1B" if kind == "1F1B" else "ZB-" + kind] = round(
            zb.simulate_pipeline(orders, t_f, t_b, t_w, t_comm, fused_backward=(kind == "1F1B"))[1], 4)
    # W passes of the steady state `grp` at a time (zb_order_group_w, bench --w-group), every stage regrouped the
    # same way, at the SAME pass times: the price in bubbles alone (at most one t_comm per group); what it
    # buys - grouped W run faster - is in `w_grouped` below.
    for grp in (2, 4):
        orders = [zb.order_group_w(zb.schedule_order(p, i, m, w.kind), grp) for i in range(p)]
        rates[f"ZB-{w.kind}, W in groups of {grp}"] = round(zb.simulate_pipeline(orders, t_f, t_b, t_w, t_comm)[1], 4)
    # ZB-V: every stage as two chunks, each chunk's pass taking half the stage's time
    rates["ZB-V"] = round(zb.simulate_pipeline_v(zb.schedule_order_v(p, m), m, t_f / 2, t_b / 2, t_w / 2, t_comm)[1], 4)
    t0 = time.perf_counter()
    found = {}
    for name, mult in (("auto, limit p*M_B", 1), ("auto, limit 2p*M_B", 2)):
        orders, cost, rate, flags = zb.auto_schedule_search(p, m, t_f, t_b, t_w, t_comm, mult * p * m_b, m_b, m_w)
        rates[name] = round(rate, 4)
        found[name] = {"extra_warmup_f": flags[0], "skip_f": flags[1],
                       "stage_peak_bytes": zb.order_memory_peak(orders[w.stage], m_b, m_w)}
    search_ms = (time.perf_counter() - t0) * 1e3
    return {"p": p, "m": m, "t_f_ms": round(t_f, 4), "t_b_ms": round(t_b, 4), "t_w_ms": round(t_w, 4),
            "t_comm_ms": round(t_comm, 4), "t_comm_source": f"{XGMI_LINK_GBS} GB/s link figure, not measured",
            "m_b_bytes": m_b, "m_w_bytes": m_w, "bubble_rate": rates, "search": found,
            "search_host_ms": round(search_ms, 2)}


def grouped_w_report(zb, st, w, m, kind, group, flops, auto, class_ms):
    """The same iteration with the W passes of the order's steady state run `group` at a time
    (zb_order_group_w; Sec. 2: a W may run anywhere after its B, Appendix A): not the order `value` is
    measured on, reported beside it.  W in one launch read and write every gradient once, so the W class gets
    faster on one GPU; the p-stage timing model, fed with the measured time of a W that opens a run of W
    (t_w_first) and of one that follows another (t_w_next), says what that does to a whole pipeline of such
    stages, every stage regrouped the same way."""
    import torch
    import zb_inputs
    base_ops = zb.schedule_order(w.p, w.stage, m, kind)
    ops = zb.order_group_w(base_ops, group)

    def step(it):
        st.begin_iteration(it, m)
        st.run_order(ops)
        if w.optimizer:
            st.optimizer_step_validated(0.0, zb_inputs.rest_state(w, it), want_report=False)

    step(100)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    n = 3
    for i in range(n):
        step(101 + i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / n * 1e3
    st.profile_enable(True)
    step(110)
    pstats = {r["name"]: r for r in st.profile_read()}
    st.profile_enable(False)
    wg = pstats["gemm_wgrad"]

    def runs_of_w(o):
        return sum(1 for i, (c, _) in enumerate(o) if c == 2 and (i == 0 or o[i - 1][0] != 2))

    r0, r1 = runs_of_w(base_ops), runs_of_w(ops)
    T0, T1 = class_ms["gemm_wgrad"] + class_ms.get("bias_grad_colsum", 0), wg["total_ms"]
    rep = {"group": group, "value": round(flops / (ms * 1e-3) / 1e12, 2), "unit": "TFLOP/s",
           "ms_per_step": round(ms, 3), "steps": n,
           "gemm_wgrad": {"launches": wg["launches"], "total_ms": round(wg["total_ms"], 3),
                          "tflops": round(wg["flops"] / wg["total_ms"] / 1e9, 1)},
           "w_stash_slots": zb.order_stash_need(ops)[1], "w_stash_slots_plain_order": zb.order_stash_need(base_ops)[1]}
    # T = runs * t_first + (m - runs) * t_next for the two orders of this stage
    det = r0 * (m - r1) - r1 * (m - r0)
    if det != 0:
        t_first = (T0 * (m - r1) - T1 * (m - r0)) / det
        t_next = (r0 * T1 - r1 * T0) / det
        t_f, t_b, t_comm = auto["t_f_ms"], auto["t_b_ms"], auto["t_comm_ms"]
        if t_first > 0 and t_next >= 0:
            base_all = [zb.schedule_order(w.p, i, m, kind) for i in range(w.p)]
            grp_all = [zb.order_group_w(o, group) for o in base_all]
            c0 = zb.simulate_pipeline_w_runs(base_all, t_f, t_b, t_first, t_comm, t_next)[0]
            c1 = zb.simulate_pipeline_w_runs(grp_all, t_f, t_b, t_first, t_comm, t_next)[0]
            rep["pipeline_model"] = {"t_w_first_ms": round(t_first, 4), "t_w_next_ms": round(t_next, 4),
                                     "iteration_ms": round(c0, 3), "iteration_ms_w_grouped": round(c1, 3),
                                     "speedup": round(c0 / c1, 4)}
    return rep


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="c4")
    ap.add_argument("--m", type=int, default=0, help="override the number of microbatches (debug)")
    ap.add_argument("--order", default="workload", choices=["workload", "1F1B", "1F1B-fused", "ZB-V"],
                    help="per-stage order: the workload's ZB-H1 / ZB-H2 (default), 1F1B with B and W as separate "
                         "passes, 1F1B with the traditional single backward (B and W fused layer by layer), or ZB-V "
                         "(Sec. 6: the stage's layers as two chunks, 2m virtual microbatches; needs an even "
                         "number of layers)")
    ap.add_argument("--w-group", type=int, default=1,
                    help="run the order with the W passes of its steady state this many at a time "
                         "(zb_order_group_w: same results bit for bit, group-1 more microbatches of W stash); 1 = the "
                         "order as the paper gives it (default; the default workload then also measures groups of 2 "
                         "and 4, untimed for `value`, and reports them as `w_grouped`)")
    ap.add_argument("--role", default="middle", choices=["middle", "first", "last"],
                    help="first / last stage of the pipeline (Sec. 5.1): one transformer layer fewer than the "
                         "workload's middle stage, plus the embedding lookup (first) or the final LayerNorm, head "
                         "and cross-entropy loss (last), vocabulary 50432; order of stage 0 / stage p-1")
    ap.add_argument("--no-w-grouped", action="store_true",
                    help="leave out the extra steps in the order with grouped W (so that a kernel trace of the run "
                         "holds the paper's order only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy kernel (calibrates FETCH_SIZE / WRITE_SIZE "
                         "in a rocprofv3 --pmc run of this command)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build covers one pipeline stage on ONE GPU; --gpus above 1 is not supported "
              "(no collectives, no second device are part of it).", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import zb_inputs
    import paper_2401_10241_amd as zb

    w = zb_inputs.workload(args.workload)
    if args.m:
        w = w.scaled(m=args.m)
    vocab = 0
    if args.role != "middle":
        if w.layers < 2 or args.order == "ZB-V":
            print("bench.py: --role first/last needs a workload with at least two layers and one chunk", file=sys.stderr)
            sys.exit(2)
        vocab = 50432   # a GPT-3-like vocabulary (50257 entries) padded to a multiple of 256
        w = w.scaled(layers=w.layers - 1, stage=0 if args.role == "first" else w.p - 1)
    m = w.m
    torch.cuda.set_device(0)
    kind = w.kind if args.order == "workload" else "1F1B"
    zbv = args.order == "ZB-V"
    if zbv:
        if w.layers % 2:
            print(f"bench.py: ZB-V splits the stage's layers into two chunks; {w.name} has {w.layers}", file=sys.stderr)
            sys.exit(2)
        v_ops = zb.schedule_order_v(w.p, m)[w.stage]
        pb, pw, fl = zb.order_stash_need(v_ops)
    elif args.w_group > 1:
        v_ops = zb.order_group_w(zb.schedule_order(w.p, w.stage, m, kind), args.w_group)
        pb, pw, fl = zb.order_stash_need(v_ops)
    else:
        pb, pw, fl = zb.schedule_stash_need(w.p, w.stage, m, kind)
    explicit = zbv or args.w_group > 1
    # the default run also measures the order with grouped W afterwards, on the same stage: give the pools its slots
    also_grouped = (2, 4) if (not explicit and args.order == "workload" and args.role == "middle"
                              and not args.no_profile and not args.m and not args.no_w_grouped) else ()
    for g in also_grouped:
        pb2, pw2, fl2 = zb.order_stash_need(zb.order_group_w(zb.schedule_order(w.p, w.stage, m, kind), g))
        pb, pw, fl = max(pb, pb2), max(pw, pw2), max(fl, fl2)
    m_run = 2 * m if zbv else m          # virtual microbatches (chunk * m + microbatch) under ZB-V
    st = zb.Stage(role=args.role, vocab=vocab, fuse_bw=(args.order == "1F1B-fused"), chunks=(2 if zbv else 1), layers=w.layers, hidden=w.hidden, heads=w.heads, ffn=w.ffn, seq=w.seq, mb_size=w.mb_size,
                  dtype=w.dtype, max_microbatches=m_run, max_pending_b=pb, max_pending_w=pw, max_inflight=fl,
                  lr=w.lr, beta1=w.beta1, beta2=w.beta2, adam_eps=w.adam_eps, weight_decay=w.weight_decay,
                  clip=w.clip, ln_eps=w.ln_eps)
    t0 = time.perf_counter()
    st.set_params(zb_inputs.stage_params(w))
    if args.role != "middle":
        st.set_stage_params(zb_inputs.end_stage_params(w, args.role, vocab))
    for k in range(m_run):
        if args.role == "first":
            st.set_ids(zb.T_INPUT_IDS, k, zb_inputs.token_ids(w, 0, k, vocab))
        else:
            st.set_tensor(zb.T_INPUT_X, 0, k, zb_inputs.stage_input(w, 0, k))
        if args.role == "last":
            st.set_ids(zb.T_TARGET_IDS, k, zb_inputs.target_ids(w, 0, k, vocab))
        else:
            st.set_tensor(zb.T_INPUT_DY, 0, k, zb_inputs.upstream_grad(w, 0, k))
    setup_s = time.perf_counter() - t0

    it_counter = [0]

    def step():
        it = it_counter[0]
        it_counter[0] += 1
        st.begin_iteration(it, m_run)
        if explicit:
            st.run_order(v_ops)
        else:
            st.run_schedule(w.p, w.stage, m, kind)
        if w.optimizer:
            st.optimizer_step_validated(0.0, zb_inputs.rest_state(w, it), want_report=False)

    if args.copy_probe:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)      # one elementwise copy kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    flops = st.model_flops(m_run)
    value = flops / (ms_per_step * 1e-3) / 1e12

    out = {
        "metric": "stage TFLOP/s (F+B+W over m microbatches) + % bf16 MFMA peak, 1xMI355X",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == "bf16" else "f32", "data": "synthetic",
        "pct_of_bf16_mfma_peak": round(100.0 * value / PEAK_BF16_TFLOPS, 2),
        "config": {"workload": f"{w.name}: " + (f"{args.role} " if args.role != "middle" else "") + f"stage {w.stage} of p={w.p}, "
                               + (f"ZB-{w.kind}" if args.order == "workload" else args.order)
                               + (f" order with steady-state W passes {args.w_group} at a time" if args.w_group > 1
                                  else " order") + f", m={m}, {w.layers} GPT "
                               f"decoder layers h={w.hidden} a={w.heads} ffn={w.ffn} seq={w.seq} b={w.mb_size}"
                               + (", validated AdamW step" if w.optimizer else ""),
                   "model_flops_per_step": flops, "setup_seconds": round(setup_s, 1)},
    }

    if not args.no_profile:
        # one more step with every kernel launch bracketed by HIP events on the stage's stream
        st.profile_enable(True)
        step()
        stats = st.profile_read()
        st.profile_enable(False)
        kern = {}
        for r in stats:
            ms = r["total_ms"]
            # the optimistic step, the rollback and the repeated step are launched every iteration and predicated on device state:
            # in an iteration that commits they return at once, so a bandwidth figure would be meaningless
            idle = r["name"] in ("adamw_step", "adamw_rollback", "adamw_restep") and r["bytes"] / ms / 1e6 > PEAK_HBM_GBS
            kern[r["name"]] = {"launches": r["launches"], "avg_us": round(1e3 * ms / r["launches"], 2),
                               "total_ms": round(ms, 3),
                               "tflops": round(r["flops"] / ms / 1e9, 1) if r["flops"] else None,
                               "gbs": None if idle else round(r["bytes"] / ms / 1e6, 1)}
            if idle:
                kern[r["name"]]["note"] = "predicated off on the device in this iteration"
            if r["flops"] and r["bytes"] and r["name"].startswith("gemm_"):
                # the lower of the matrix peak and what the algorithmic bytes allow at the HBM peak (the wgrad
                # GEMMs with their fp32 read-modify-write sit near that ridge)
                ceil_tf = min(PEAK_BF16_TFLOPS if w.dtype == "bf16" else PEAK_FP32_TFLOPS,
                              r["flops"] / r["bytes"] * PEAK_HBM_GBS / 1e3)
                kern[r["name"]]["ceiling_tflops"] = round(ceil_tf, 1)
                kern[r["name"]]["frac_of_ceiling"] = round(r["flops"] / ms / 1e9 / ceil_tf, 4)
        gemm = [r for r in stats if r["name"].startswith("gemm_")]
        g_ms = sum(r["total_ms"] for r in gemm)
        g_fl = sum(r["flops"] for r in gemm)
        g_n = sum(r["launches"] for r in gemm)
        g_by = sum(r["bytes"] for r in gemm)
        peak = PEAK_BF16_TFLOPS if w.dtype == "bf16" else PEAK_FP32_TFLOPS
        all_ms = sum(r["total_ms"] for r in stats)
        # the dominant kernel: the class with the largest share of the step's kernel time (at the bf16 workloads
        # the wgrad kernel, one launch per W pass: the accumulate GEMMs of all its layers)
        top = max(gemm, key=lambda r: r["total_ms"])
        ach = top["flops"] / top["total_ms"] / 1e9
        out["roofline"] = {"kernel": top["name"],
                           "bound": "mfma" if w.dtype == "bf16" else "alu", "achieved": round(ach, 1),
                           "peak": peak, "unit": "TFLOP/s", "frac": round(ach / peak, 4),
                           "traffic": measured_traffic(w.name) if not (args.m or args.w_group > 1 or args.role != "middle") else None,
                           "algorithmic_bytes_per_launch": top["bytes"] / top["launches"],
                           "hbm_limited_ceiling_tflops": round(min(peak, top["flops"] / top["bytes"] * PEAK_HBM_GBS / 1e3), 1),
                           "launches": top["launches"], "avg_launch_us": round(1e3 * top["total_ms"] / top["launches"], 2),
                           "flops_per_launch": top["flops"] / top["launches"],
                           "share_of_step_kernel_time": round(top["total_ms"] / all_ms, 3)}
        out["gemm_all"] = {"achieved": round(g_fl / g_ms / 1e9, 1), "frac": round(g_fl / g_ms / 1e9 / peak, 4),
                           "launches": g_n, "avg_launch_us": round(1e3 * g_ms / g_n, 2),
                           "share_of_step_kernel_time": round(g_ms / all_ms, 3)}
        if w.optimizer:
            # One more optimizer call on the gradients still in place, untimed: forced to take the optimistic step
            # although the norm is above the threshold, so that validation rolls it back and redoes it clipped -
            # the step with its journal, the rollback and the redo all move their bytes and get a bandwidth figure.
            st.profile_enable(True)
            rep = st.optimizer_step_validated(0.0, zb_inputs.rest_state(w, 0) + 4.0, force_optimistic=True)
            forced = {r["name"]: r for r in st.profile_read()}
            st.profile_enable(False)
            fr = {"outcome": rep.outcome_name, "alg1_mismatch_elems": rep.alg1_mismatch_elems,
                  "journal_bytes_per_param": 12}
            for name in ("adamw_step", "adamw_rollback", "adamw_restep"):
                if name in forced:
                    r = forced[name]
                    fr[name] = {"ms": round(r["total_ms"], 3), "gbs": round(r["bytes"] / r["total_ms"] / 1e6, 1)}
                    if name == "adamw_rollback" and kern.get(name, {}).get("gbs") is None:
                        kern[name]["gbs_when_it_runs"] = fr[name]["gbs"]
            out["optimizer_forced_rollback"] = fr
        out["kernels"] = kern
        out["auto_schedule"] = auto_schedule_report(zb, st, w, m, {r["name"]: r["total_ms"] for r in stats})
        if also_grouped:
            out["w_grouped"] = [grouped_w_report(zb, st, w, m, kind, g, flops, out["auto_schedule"],
                                                 {r["name"]: r["total_ms"] for r in stats}) for g in also_grouped]
    st.close()
    del st
    torch.cuda.empty_cache()

    if not args.no_cpu_baseline and args.role == "middle":
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
